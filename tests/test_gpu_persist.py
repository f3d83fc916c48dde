"""GPU parity of the block image entry points (save / restore of an agent's cache): the exported bytes are the
oracle-side cache's bytes, tensor by tensor through a file read back with the safetensors library; a cache restored
into other physical blocks attends bit-identically."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import binding as b
from paper_2603_04428_amd import persist, synth
from tests.gpu_util import DEV, bits, gpu_cache, host_cache

pytestmark = pytest.mark.gpu


def attend(w, spec, kpool, vpool, table_d):
    sl = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    out = b.q4kv_batched_attention(spec, kpool, vpool, w.q_all(DEV), table_d, sl, max(w.seq_lens), w.sm_scale)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("shape", [(2, 4, 2, 128, 128, False), (1, 16, 16, 192, 128, False), (2, 16, 1, 576, 512, True)])
def test_export_file_import_round_trip(tmp_path, shape):
    from safetensors.numpy import load_file
    L, Hq, Hkv, dk, dv, alias = shape
    w = synth.small(61, L, Hq, Hkv, dk, dv, alias, (700, 130))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    before = attend(w, spec, kpool, vpool, table_d)
    agent, nb = 0, 3                                                  # 700 tokens: three blocks
    ids = table_d[agent, :nb].contiguous()
    image = b.q4kv_export_blocks(spec, kpool, vpool, ids)
    assert image.numel() == persist.image_bytes(spec, nb) == b.q4kv_block_image_bytes(spec, nb)
    path = os.path.join(tmp_path, "agent0.safetensors")
    persist.save_agent(path, spec, image.cpu(), nb, 700)
    # every tensor of the file is the oracle-side cache's array of that (layer, block)
    tensors = load_file(path)
    for l in range(L):
        for i in range(nb):
            blk = otable[agent, i]
            for tag, pool in (("K", okp),) + ((() if alias else (("V", ovp),))):
                assert np.array_equal(tensors[f"L{l}_B{i}_{tag}_weights"], pool.codes[l, blk])
                assert np.array_equal(tensors[f"L{l}_B{i}_{tag}_scales"].view(np.uint16), pool.scale[l, blk])
                assert np.array_equal(tensors[f"L{l}_B{i}_{tag}_biases"].view(np.uint16), pool.bias[l, blk])
    # restore into a fresh, poisoned pool at other physical blocks, through pinned host memory
    meta, img = persist.open_agent(path)
    assert meta["seq_len"] == 700 and meta["num_blocks"] == nb
    pinned = torch.empty(img.size, dtype=torch.uint8, pin_memory=True)
    persist.load_agent_into(path, pinned)
    nb_pool = kpool.num_blocks
    k2 = b.Pool(spec, dk, nb_pool + 2, DEV, True)
    v2 = None if alias else b.Pool(spec, dv, nb_pool + 2, DEV, True)
    new_ids = torch.tensor([nb_pool + 1, 0, nb_pool], dtype=torch.int32, device=DEV)
    b.q4kv_import_blocks(spec, k2, v2, new_ids, pinned)               # the kernel reads the host image directly
    torch.cuda.synchronize()
    for name in ("codes", "scale", "bias"):
        for src, dst in ((kpool, k2),) + (() if alias else ((vpool, v2),)):
            assert torch.equal(getattr(dst, name)[:, new_ids.long()], getattr(src, name)[:, ids.long()])
    # the second agent keeps its blocks: copy them over by hand, then both pools must attend identically
    other = table_d[1, :1].long()
    for name in ("codes", "scale", "bias"):
        for src, dst in ((kpool, k2),) + (() if alias else ((vpool, v2),)):
            getattr(dst, name)[:, other] = getattr(src, name)[:, other]
    table2 = table_d.clone()
    table2[agent, :nb] = new_ids
    after = attend(w, spec, k2, v2, table2)
    assert np.array_equal(before.view(np.uint16), after.view(np.uint16))


def test_export_into_pinned_host_memory_and_skipped_ids():
    w = synth.small(62, 2, 4, 2, 64, 64, False, (300,))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ids = table_d[0, :2].contiguous()
    dev_image = b.q4kv_export_blocks(spec, kpool, vpool, ids)
    pinned = torch.zeros(dev_image.numel(), dtype=torch.uint8, pin_memory=True)
    b.q4kv_export_blocks(spec, kpool, vpool, ids, pinned)
    torch.cuda.synchronize()
    assert torch.equal(pinned, dev_image.cpu())
    # an id outside the pool: its records keep whatever the image held
    bad = ids.clone()
    bad[1] = 10_000
    marked = torch.full_like(dev_image, 0xA5)
    b.q4kv_export_blocks(spec, kpool, vpool, bad, marked)
    torch.cuda.synchronize()
    rec = persist.image_bytes(spec, 1) // spec.num_layers
    got, want = marked.cpu().view(spec.num_layers, 2, rec), dev_image.cpu().view(spec.num_layers, 2, rec)
    assert torch.equal(got[:, 0], want[:, 0]) and bool((got[:, 1] == 0xA5).all())
    before = [getattr(p, n).clone() for p in (kpool, vpool) for n in ("codes", "scale", "bias")]
    b.q4kv_import_blocks(spec, kpool, vpool, torch.tensor([-1, 99], dtype=torch.int32, device=DEV), dev_image)
    torch.cuda.synchronize()
    after = [getattr(p, n) for p in (kpool, vpool) for n in ("codes", "scale", "bias")]
    assert all(torch.equal(x, y) for x, y in zip(before, after))
    with pytest.raises(b.Q4KVError):
        b.q4kv_export_blocks(spec, kpool, vpool, ids, dev_image[:-16])          # image too small
    assert b.q4kv_export_blocks(spec, kpool, vpool, ids[:0]).numel() == 0         # nothing to do


def test_agents_paged_through_a_small_pool(tmp_path):
    """Sec. 3.1 / Sec. 1 (caches paged between memory and disk): five agents take turns on a device pool that holds
    three of them.  The block pool names the least recently used agent, its blocks leave through a file and come back
    into whatever blocks are free; every agent's decode output keeps the bits it had when all of its cache was first
    resident."""
    L, Hq, Hkv, D = 2, 4, 2, 64
    lens = (600, 300, 520, 257, 700)                       # 3, 2, 3, 2, 3 blocks
    w = synth.small(63, L, Hq, Hkv, D, D, False, lens)
    NB, MB = 8, 3
    spec = b.make_spec(L, Hq, Hkv, D)
    kpool, vpool = b.Pool(spec, D, NB, DEV, True), b.Pool(spec, D, NB, DEV, True)
    book = b.BlockPool(NB)
    on_disk = {}

    def make_room(agent, tokens):
        while True:
            try:
                return book.reserve(agent, tokens)
            except b.Q4KVError as e:
                assert e.code == b.BlockPool.ENOSPACE
            victim = book.lru_victim()
            assert victim >= 0 and victim != agent
            ids = torch.tensor(book.blocks(victim), dtype=torch.int32, device=DEV)
            image = b.q4kv_export_blocks(spec, kpool, vpool, ids)
            torch.cuda.synchronize()
            path = os.path.join(tmp_path, f"agent{victim}.safetensors")
            persist.save_agent(path, spec, image.cpu(), ids.numel(), lens[victim])
            on_disk[victim] = path
            # what the victim leaves behind must not matter to anyone: poison it
            for pool in (kpool, vpool):
                pool.codes[:, ids.long()] = -1
                pool.scale[:, ids.long()] = 0x7E00
                pool.bias[:, ids.long()] = 0x7E00
            book.release(victim)

    def decode(agent):
        row = torch.tensor([book.table_row(agent, MB, fill=0)], dtype=torch.int32, device=DEV)
        sl = torch.tensor([lens[agent]], dtype=torch.int32, device=DEV)
        q = w.q_all(DEV)[:, agent:agent + 1].contiguous()
        out = b.q4kv_batched_attention(spec, kpool, vpool, q, row, sl, lens[agent], w.sm_scale)
        torch.cuda.synchronize()
        return out.cpu().numpy().view(np.uint16)

    first = {}
    order = [0, 1, 2, 3, 0, 4, 1, 2, 0, 3, 4]
    evictions = 0
    for agent in order:
        if agent in first and agent not in on_disk:
            book.touch(agent)                                # still resident
        elif agent in on_disk:                               # restore into whatever blocks are free now
            meta, img = persist.open_agent(on_disk.pop(agent))
            make_room(agent, meta["seq_len"])
            evictions += 1
            pinned = torch.empty(img.size, dtype=torch.uint8, pin_memory=True)
            persist.load_agent_into(os.path.join(tmp_path, f"agent{agent}.safetensors"), pinned)
            ids = torch.tensor(book.blocks(agent), dtype=torch.int32, device=DEV)
            b.q4kv_import_blocks(spec, kpool, vpool, ids, pinned)
        else:                                                # first arrival: prefill its cache through q4kv_append
            make_room(agent, lens[agent])
            row = torch.tensor([book.table_row(agent, MB, fill=0)], dtype=torch.int32, device=DEV)
            zero = torch.zeros(1, dtype=torch.int32, device=DEV)
            for l in range(L):
                b.q4kv_append(spec, kpool, vpool, w.k_rows(l, agent, 0, lens[agent], DEV)[None, None].contiguous(),
                              w.v_rows(l, agent, 0, lens[agent], DEV)[None, None].contiguous(), row, zero, l, l + 1)
        got = decode(agent)
        if agent in first:
            assert np.array_equal(got, first[agent]), f"agent {agent} changed after paging"
        else:
            first[agent] = got
        # isolation: every block has at most one owner and the resident agents' lists are disjoint
        owners = [book.owner(i) for i in range(NB)]
        for a in set(o for o in owners if o >= 0):
            assert sorted(i for i, o in enumerate(owners) if o == a) == sorted(book.blocks(a))
    assert evictions >= 3 and len(first) == 5
    # and the first results are the oracle's
    ospec, okp, ovp, otable = host_cache(w)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
    for agent in range(5):
        ok = np.abs(first[agent].view(np.float16).astype(np.float64)[:, 0] - want[:, agent].astype(np.float64)) <= \
            2e-3 + 2e-3 * np.abs(want[:, agent].astype(np.float64))
        assert ok.all()


def test_bfloat16_cache_file_round_trip(tmp_path):
    """A pool with bfloat16 scale / bias (appendix "safetensors Q4 Format") saved and read back with the format's own
    torch reader: the scale and bias tensors are bfloat16 tensors holding the oracle-side cache's bits."""
    from safetensors.torch import load_file
    BF = b.PARAMS_BF16
    w = synth.small(64, 2, 4, 2, 128, 128, False, (520, 90))
    spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=BF)
    ospec, okp, ovp, otable = host_cache(w, param_format=BF)
    agent, nb = 0, 3
    ids = table_d[agent, :nb].contiguous()
    image = b.q4kv_export_blocks(spec, kpool, vpool, ids)
    path = os.path.join(tmp_path, "agent0_bf16.safetensors")
    persist.save_agent(path, spec, image.cpu(), nb, 520)
    tensors = load_file(path)
    for l in range(2):
        for i in range(nb):
            blk = otable[agent, i]
            for tag, pool in (("K", okp), ("V", ovp)):
                assert np.array_equal(tensors[f"L{l}_B{i}_{tag}_weights"].numpy().view(np.uint32), pool.codes[l, blk])
                for kind, arr in (("scales", pool.scale), ("biases", pool.bias)):
                    t = tensors[f"L{l}_B{i}_{tag}_{kind}"]
                    assert t.dtype == torch.bfloat16
                    assert np.array_equal(t.view(torch.int16).numpy().view(np.uint16), arr[l, blk])
    meta, img = persist.open_agent(path)
    assert meta["spec"]["param_format"] == BF
    # back into other blocks of a fresh pool: attention over the restored agent is bit-identical
    k2, v2 = b.Pool(spec, 128, 6, DEV, True), b.Pool(spec, 128, 6, DEV, True)
    new_ids = torch.tensor([5, 0, 3], dtype=torch.int32, device=DEV)
    b.q4kv_import_blocks(spec, k2, v2, new_ids, torch.from_numpy(np.asarray(img).copy()).to(DEV))
    sl = torch.tensor([520], dtype=torch.int32, device=DEV)
    q = w.q_all(DEV)[:, :1].contiguous()
    row_old = table_d[:1, :3].contiguous()
    row_new = new_ids[None].contiguous()
    a = b.q4kv_batched_attention(spec, kpool, vpool, q, row_old, sl, 520, w.sm_scale)
    c = b.q4kv_batched_attention(spec, k2, v2, q, row_new, sl, 520, w.sm_scale)
    torch.cuda.synchronize()
    assert torch.equal(a, c)
