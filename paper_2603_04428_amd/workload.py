"""Device-side set-up of a benchmark workload: fill paged Q4 pools on the GPU from the seeded generator,
through the library's own q4kv_append entry point.  Used by the benchmark, the smoke check and the GPU tests."""
import numpy as np
import torch

from . import binding as b


def build_device_cache(w, device="cuda", poison=True, extra_blocks=1, tokens=None, param_format=b.PARAMS_F16):
    """Returns (spec, kpool, vpool, table (host int32 [A][max_blocks], -1 = unused), table on the device).
    Every agent's tokens 0..len-1 are generated on the device layer by layer and appended into freshly
    allocated blocks whose physical ids are shuffled over the pool."""
    spec = b.make_spec(w.num_layers, w.num_q_heads, w.num_kv_heads, w.k_dim, w.v_dim, w.v_aliases_k,
                       param_format=param_format)
    table, nb = w.block_table()
    nb += extra_blocks
    kpool = b.Pool(spec, w.k_dim, nb, device, poison)
    vpool = None if w.v_aliases_k else b.Pool(spec, w.v_dim, nb, device, poison)
    # unused table entries point at a spare (poisoned) block, or at block 0 when there is no spare
    table_d = torch.from_numpy(np.where(table < 0, nb - 1 if extra_blocks else 0, table).astype(np.int32)).to(device)
    zero = torch.zeros(1, dtype=torch.int32, device=device)
    lens = w.final_lens() if tokens is None else tokens
    for l in range(w.num_layers):
        for a, n in enumerate(lens):
            if n == 0:
                continue
            k_new = w.k_rows(l, a, 0, n, device)[None, None].contiguous()
            v_new = None if w.v_aliases_k else w.v_rows(l, a, 0, n, device)[None, None].contiguous()
            b.q4kv_append(spec, kpool, vpool, k_new, v_new, table_d[a:a + 1].contiguous(), zero, l, l + 1)
    return spec, kpool, vpool, table, table_d
