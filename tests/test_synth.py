"""The synthetic input generator: determinism, slice consistency, distribution, layout of block tables."""
import numpy as np
import torch

from paper_2603_04428_amd import synth


def test_slices_regenerate_the_same_values():
    w = synth.config(2)
    full = w.k_rows(3, 1, 0, 50)
    part = w.k_rows(3, 1, 20, 30, h0=2, h1=5)
    assert torch.equal(full[20:30, 2:5], part)
    assert not torch.equal(w.k_rows(3, 1, 0, 5), w.k_rows(4, 1, 0, 5))
    assert not torch.equal(w.k_rows(3, 1, 0, 5), w.k_rows(3, 2, 0, 5))
    assert not torch.equal(w.k_rows(3, 1, 0, 5), w.v_rows(3, 1, 0, 5))


def test_values_look_standard_normal_with_k_outliers():
    w = synth.config(0)
    v = w.v_rows(0, 0, 0, 1024).float().numpy()
    assert abs(v.mean()) < 0.01 and abs(v.std() - 1.0) < 0.01
    assert abs(np.mean(v ** 4) - 3.0) < 0.1
    k = w.k_rows(0, 0, 0, 1024).float().numpy()
    std = k.std(axis=0)                                  # [heads][dim]
    for h in range(8):
        hot = np.sort(np.argsort(std[h])[-4:])
        assert np.array_equal(hot, w.outliers[0, h])
        assert np.all(std[h, hot] > 7.0) and np.all(np.delete(std[h], hot) < 1.2)
    # successive counters are uncorrelated
    flat = v.reshape(-1)
    assert abs(np.corrcoef(flat[:-1], flat[1:])[0, 1]) < 0.01


def test_integer_hash_matches_python_reference():
    # the tensor path (wrapping int64) against arbitrary-precision Python integers
    key = synth.stream_key(5, synth.TENSOR_K, 2, 3)
    t = synth.draw(5, synth.TENSOR_K, 2, 3, 7, 8, 4, 64)[0]
    table = synth.normal_table()
    for h in range(4):
        for d in (0, 13, 63):
            counter = (7 * 4 + h) * 64 + d
            bits = synth._mix64_int(counter * synth.GAMMA + key)
            assert t[h, d] == table[bits >> 48].to(torch.float16)


def test_configs_have_the_stated_shapes():
    c1, c2, c3, c4 = (synth.config(i) for i in (1, 2, 3, 4))
    assert (c1.num_layers, c1.num_q_heads, c1.num_kv_heads, c1.k_dim, c1.seq_lens) == (32, 32, 8, 128, [4096] * 5)
    assert c2.num_agents == 10 and all(1024 <= n <= 8192 for n in c2.seq_lens) and len(set(c2.seq_lens)) > 1
    assert c2.q4_bytes_per_token_layer() == 2304 and c1.q4_bytes_per_token_layer() == 1152
    assert (c3.k_dim, c3.v_dim, c3.v_aliases_k, c3.num_kv_heads) == (576, 512, True, 1)
    assert c3.q4_bytes_per_token_layer() == 324
    assert c4.q_len == 512 and all(4096 <= n <= 32768 for n in c4.seq_lens)
    assert c4.final_lens() == [n + 512 for n in c4.seq_lens]


def test_block_table_is_a_permutation_without_sharing():
    w = synth.config(2)
    table, nb = w.block_table()
    used = table[table >= 0]
    assert len(used) == nb == len(set(used.tolist())) and used.min() == 0 and used.max() == nb - 1
    for a, n in enumerate(w.seq_lens):
        need = (n + 255) // 256
        assert (table[a, :need] >= 0).all() and (table[a, need:] == -1).all()
