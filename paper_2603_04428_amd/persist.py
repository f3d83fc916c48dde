"""Agent cache files: a block image behind a safetensors header.

The paper keeps every agent's cache on disk in the Q4 form it has in memory, one tensor per (layer, block, array),
so that a restore is a copy and no prefill (Sec. 3.1, Sec. 3.2 "Q4 at rest", appendix "safetensors Q4 Format").
The image produced by q4kv_export_blocks already is the data section of such a file: this module only writes and
parses the header around it.  No arithmetic happens here.

File = 8-byte little-endian header length, a JSON header padded with spaces to a multiple of 8 bytes, the image.
Tensor names follow the appendix: L{l}_B{b}_K_weights / _K_scales / _K_biases / _V_weights / _V_scales / _V_biases,
b counting the agent's blocks in token order.  Shapes are the device layout's, token-major: weights uint32
(kv_heads, 256, dim/8), scales and biases float16 or, when the cache shape says param_format 1, bfloat16
(kv_heads, 256, dim/64): the appendix names bfloat16 for one model family and float16 for another.  (The shapes printed in the appendix
disagree with each other about the grouped axis and are not reproduced.)  The header's __metadata__ carries the
cache shape, the block count and the token count as strings.
"""
import json
import struct

import numpy as np

FORMAT = "q4kv-block-image-1"
SPEC_FIELDS = ("num_layers", "num_q_heads", "num_kv_heads", "k_dim", "v_dim", "v_aliases_k", "block_tokens", "group_size",
               "param_format")
PARAM_DTYPES = {0: "F16", 1: "BF16"}   # safetensors dtype of scales and biases by q4kv_param_format


def spec_dict(spec):
    d = {f: int(getattr(spec, f, 0)) for f in SPEC_FIELDS}
    if d["param_format"] not in PARAM_DTYPES:
        raise ValueError(f"unknown param_format {d['param_format']}")
    return d


def tensor_table(spec, num_blocks):
    """[(name, dtype, shape, begin, end)] in image order; begin / end are byte offsets into the image."""
    sd = spec if isinstance(spec, dict) else spec_dict(spec)
    H, T = sd["num_kv_heads"], sd["block_tokens"]
    arrays = [("K", sd["k_dim"])] + ([] if sd["v_aliases_k"] else [("V", sd["v_dim"])])
    pdt = PARAM_DTYPES[sd.get("param_format", 0)]
    out, off = [], 0
    for l in range(sd["num_layers"]):
        for b in range(num_blocks):
            for tag, dim in arrays:
                for kind, dtype, last, width in (("weights", "U32", dim // 8, 4), ("scales", pdt, dim // 64, 2),
                                                 ("biases", pdt, dim // 64, 2)):
                    n = H * T * last * width
                    out.append((f"L{l}_B{b}_{tag}_{kind}", dtype, [H, T, last], off, off + n))
                    off += n
    return out


def image_bytes(spec, num_blocks):
    t = tensor_table(spec, num_blocks)
    return t[-1][4] if t else 0


def _header(spec, num_blocks, seq_len, extra):
    sd = spec_dict(spec)
    meta = {"format": FORMAT, "num_blocks": str(num_blocks), "seq_len": str(int(seq_len))}
    meta.update({k: str(v) for k, v in sd.items()})
    for k, v in (extra or {}).items():
        meta[str(k)] = str(v)
    hdr = {"__metadata__": meta}
    for name, dtype, shape, b, e in tensor_table(sd, num_blocks):
        hdr[name] = {"dtype": dtype, "shape": shape, "data_offsets": [b, e]}
    raw = json.dumps(hdr, separators=(",", ":")).encode("utf-8")
    raw += b" " * (-len(raw) % 8)
    return raw


def save_agent(path, spec, image, num_blocks, seq_len, extra=None):
    """image: the block image as a host array (numpy uint8, or a CPU torch tensor), image_bytes(spec, num_blocks) long."""
    buf = image.numpy() if hasattr(image, "numpy") else np.asarray(image)
    buf = buf.reshape(-1).view(np.uint8)
    need = image_bytes(spec, num_blocks)
    if buf.size != need:
        raise ValueError(f"image has {buf.size} bytes, the cache shape needs {need}")
    if not 0 <= int(seq_len) <= num_blocks * int(spec.block_tokens):
        raise ValueError("seq_len does not fit the blocks")
    raw = _header(spec, num_blocks, seq_len, extra)
    with open(path, "wb") as f:
        f.write(struct.pack("<Q", len(raw)))
        f.write(raw)
        f.write(memoryview(buf))


def open_agent(path):
    """-> (metadata dict, image as a read-only numpy memmap).  Checks that the header describes exactly the image
    this cache shape has and that the file is complete."""
    with open(path, "rb") as f:
        head = f.read(8)
        if len(head) != 8:
            raise ValueError("not an agent cache file: too short")
        (n,) = struct.unpack("<Q", head)
        if n <= 0 or n > (1 << 31):
            raise ValueError("not an agent cache file: bad header length")
        raw = f.read(n)
        if len(raw) != n:
            raise ValueError("truncated header")
        f.seek(0, 2)
        size = f.tell()
    hdr = json.loads(raw.decode("utf-8"))
    meta = hdr.get("__metadata__") or {}
    if meta.get("format") != FORMAT:
        raise ValueError("not a q4kv agent cache file")
    sd = {k: int(meta.get(k, 0)) for k in SPEC_FIELDS}      # files written before param_format existed hold binary16
    if sd["param_format"] not in PARAM_DTYPES:
        raise ValueError("unknown param_format in the header")
    num_blocks = int(meta["num_blocks"])
    table = tensor_table(sd, num_blocks)
    if len(hdr) - 1 != len(table):
        raise ValueError("header lists a different set of tensors than the cache shape has")
    for name, dtype, shape, b, e in table:
        ent = hdr.get(name)
        if ent is None or ent["dtype"] != dtype or ent["shape"] != shape or ent["data_offsets"] != [b, e]:
            raise ValueError(f"tensor {name} does not match the cache shape")
    need = table[-1][4] if table else 0
    if size != 8 + n + need:
        raise ValueError(f"file has {size - 8 - n} bytes of data, the header describes {need}")
    image = np.memmap(path, dtype=np.uint8, mode="r", offset=8 + n, shape=(need,))
    out = dict(meta)
    out["spec"] = sd
    out["num_blocks"] = num_blocks
    out["seq_len"] = int(meta["seq_len"])
    return out, image


def load_agent_into(path, pinned):
    """Read the image of a file into `pinned` (a uint8 torch tensor in pinned host memory, large enough); -> metadata."""
    meta, image = open_agent(path)
    if pinned.numel() < image.size:
        raise ValueError("destination too small")
    pinned.numpy()[:image.size] = image
    return meta
