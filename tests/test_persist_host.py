"""Agent cache files (host side, no GPU): the header written around a block image is a valid safetensors file --
checked by loading it with the safetensors library itself --, names follow the paper's appendix, sizes follow the
paper's byte count, and damaged files are refused."""
import json
import os
import struct

import numpy as np
import pytest

import oracle
from paper_2603_04428_amd import persist


class _Spec:
    def __init__(self, L, Hq, Hkv, dk, dv, alias=0, param_format=0):
        self.num_layers, self.num_q_heads, self.num_kv_heads = L, Hq, Hkv
        self.k_dim, self.v_dim, self.v_aliases_k, self.block_tokens, self.group_size = dk, dv, alias, 256, 64
        self.param_format = param_format


def _random_image(spec, nb, seed=0):
    n = persist.image_bytes(spec, nb)
    return np.random.default_rng(seed).integers(0, 256, n, dtype=np.uint8)


@pytest.mark.parametrize("shape", [(2, 4, 2, 128, 128, 0), (1, 16, 16, 192, 128, 0), (3, 16, 1, 576, 512, 1)])
def test_file_is_a_safetensors_file_with_the_appendix_names(tmp_path, shape):
    from safetensors.numpy import load_file                     # the format's own reader: an external check
    spec = _Spec(*shape)
    nb = 3
    img = _random_image(spec, nb)
    path = os.path.join(tmp_path, "agent.safetensors")
    persist.save_agent(path, spec, img, nb, 600, {"agent_id": "a7"})
    tensors = load_file(path)
    kinds = ["K"] + ([] if spec.v_aliases_k else ["V"])
    assert set(tensors) == {f"L{l}_B{b}_{t}_{k}" for l in range(spec.num_layers) for b in range(nb) for t in kinds
                            for k in ("weights", "scales", "biases")}
    for name, dtype, shp, b, e in persist.tensor_table(spec, nb):
        t = tensors[name]
        assert list(t.shape) == shp and t.dtype == {"U32": np.uint32, "F16": np.float16}[dtype]
        assert np.array_equal(t.reshape(-1).view(np.uint8), img[b:e]), name
    H = spec.num_kv_heads
    assert tensors["L0_B0_K_weights"].shape == (H, 256, spec.k_dim // 8)
    assert tensors["L0_B0_K_scales"].shape == (H, 256, spec.k_dim // 64)
    meta, image = persist.open_agent(path)
    assert meta["seq_len"] == 600 and meta["num_blocks"] == nb and meta["agent_id"] == "a7"
    assert meta["spec"] == persist.spec_dict(spec)
    assert np.array_equal(np.asarray(image), img)


def test_bfloat16_parameters_are_declared_as_such(tmp_path):
    """Appendix "safetensors Q4 Format": scales and biases of one model family are bfloat16 tensors.  The format's own
    torch reader must hand them back as bfloat16 with the image's bits."""
    import torch
    from safetensors.torch import load_file
    spec = _Spec(2, 4, 2, 128, 64, 0, param_format=1)
    nb = 2
    img = _random_image(spec, nb, seed=3)
    path = os.path.join(tmp_path, "agent_bf16.safetensors")
    persist.save_agent(path, spec, img, nb, 300)
    tensors = load_file(path)
    for name, dtype, shp, b, e in persist.tensor_table(spec, nb):
        t = tensors[name]
        assert list(t.shape) == shp
        if name.endswith("weights"):
            assert dtype == "U32"
            continue
        assert dtype == "BF16" and t.dtype == torch.bfloat16
        assert np.array_equal(t.view(torch.int16).numpy().reshape(-1).view(np.uint8), img[b:e]), name
    meta, image = persist.open_agent(path)
    assert meta["spec"]["param_format"] == 1 and np.array_equal(np.asarray(image), img)
    # same sizes as the binary16 form
    assert persist.image_bytes(spec, nb) == persist.image_bytes(_Spec(2, 4, 2, 128, 64), nb)
    with pytest.raises(ValueError):
        persist.image_bytes(_Spec(2, 4, 2, 128, 64, 0, param_format=3), nb)


def test_image_size_is_the_papers_byte_count():
    """Sec. 3.2: a Q4 layer of n tokens takes h d n (1 + 8/g) / 2 ... bytes for K and V together; an image of B blocks
    holds 256 B tokens of every layer (the oracle's closed form, itself pinned to the paper's printed numbers)."""
    for L, Hkv, dk, dv in ((48, 8, 256, 256), (27, 16, 192, 128), (32, 8, 128, 128)):
        spec = _Spec(L, 2 * Hkv, Hkv, dk, dv)
        for nb in (1, 16, 128):
            assert persist.image_bytes(spec, nb) == L * oracle.q4_layer_bytes(Hkv, dk, dv, 256 * nb)
    # Gemma-3-12B-shaped agent at 4K tokens: 432 MiB, the appendix' figure
    assert persist.image_bytes(_Spec(48, 16, 8, 256, 256), 16) == 432 * 1024 * 1024


def test_damaged_or_foreign_files_are_refused(tmp_path):
    spec = _Spec(1, 2, 2, 64, 64)
    img = _random_image(spec, 2)
    good = os.path.join(tmp_path, "good.safetensors")
    persist.save_agent(good, spec, img, 2, 300)
    raw = open(good, "rb").read()
    (n,) = struct.unpack("<Q", raw[:8])

    def write(name, data):
        p = os.path.join(tmp_path, name)
        open(p, "wb").write(data)
        return p

    with pytest.raises(ValueError):
        persist.open_agent(write("short", raw[:5]))
    with pytest.raises(ValueError):
        persist.open_agent(write("cut", raw[:-100]))                      # data section incomplete
    with pytest.raises(ValueError):
        persist.open_agent(write("long", raw + b"\0" * 16))                # trailing bytes
    hdr = json.loads(raw[8:8 + n])
    hdr["__metadata__"]["format"] = "something else"
    other = json.dumps(hdr).encode()
    with pytest.raises(ValueError):
        persist.open_agent(write("foreign", struct.pack("<Q", len(other)) + other + raw[8 + n:]))
    hdr = json.loads(raw[8:8 + n])
    hdr["L0_B0_K_scales"]["shape"] = [2, 64, 4]                            # a header that disagrees with the cache shape
    other = json.dumps(hdr).encode()
    with pytest.raises(ValueError):
        persist.open_agent(write("reshaped", struct.pack("<Q", len(other)) + other + raw[8 + n:]))
    with pytest.raises(ValueError):
        persist.save_agent(os.path.join(tmp_path, "bad"), spec, img[:-1], 2, 300)      # image of the wrong size
    with pytest.raises(ValueError):
        persist.save_agent(os.path.join(tmp_path, "bad"), spec, img, 2, 513)           # more tokens than the blocks hold
