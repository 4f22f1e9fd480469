"""The seeded input generator: host C, host Python and device torch evaluations agree bit for bit."""
import numpy as np
import pytest

import synth


def test_c_hash_matches_python_reference():
    k1, k2 = synth.keys(42, 7 * 64 + 3)
    tab = synth.normal_table(0.0, 0.02)
    bits = synth.tensor_bits(42, 7 * 64 + 3, 500, 0.0, 0.02, i0=123456)
    ref = np.array([tab[synth.hash_py(k1, k2, 123456 + i) & 0xFFFF] for i in range(500)], dtype=np.uint16)
    np.testing.assert_array_equal(bits, ref)
    np.testing.assert_array_equal(synth.tensor_f32(42, 7 * 64 + 3, 500, 0.0, 0.02, i0=123456),
                                  synth.bf16_bits_to_f32(ref))


def test_distribution_and_independence():
    a = synth.tensor_f32(1, 100, 1 << 20, 0.0, 1.0)
    b = synth.tensor_f32(1, 101, 1 << 20, 0.0, 1.0)
    c = synth.tensor_f32(2, 100, 1 << 20, 0.0, 1.0)
    for t in (a, b, c):
        assert abs(t.mean()) < 5e-3 and abs(t.std() - 1.0) < 5e-3
    assert abs(np.corrcoef(a, b)[0, 1]) < 5e-3 and abs(np.corrcoef(a, c)[0, 1]) < 5e-3
    assert abs(np.corrcoef(a[:-1], a[1:])[0, 1]) < 5e-3
    g = synth.tensor_f32(1, 5, 1 << 16, 1.0, 0.02)
    assert abs(g.mean() - 1.0) < 1e-3 and abs(g.std() - 0.02) < 1e-3


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38], np.float32)   # 1+2^-8 (tie->even), 1+3*2^-8 (tie->even)
    back = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    np.testing.assert_array_equal(back[:4], np.array([1.0, 1.0, 1.015625, -2.5], np.float32))


def test_step_draw_page_tables_are_disjoint_and_sized():
    rng = np.random.default_rng(0)
    s = synth.LLAMA3_8B
    st = synth.draw_step(rng, s, [1, 4, 16, 64], 128, 4096, synth.pool_pages_for(s, 64, 4096))
    assert st.batch in (1, 4, 16, 64)
    assert len(set(st.page_ids.tolist())) == len(st.page_ids)
    for b in range(st.batch):
        assert st.page_indptr[b + 1] - st.page_indptr[b] == (st.kv_len[b] + 1 + 15) // 16


@pytest.mark.gpu
def test_device_generator_matches_host_bits():
    import torch
    from synth import gpu
    n = (1 << 20) + 17
    t = gpu.tensor_gpu(9, 3 * 64 + 6, n, 0.0, 0.02, i0=5)
    host = synth.tensor_bits(9, 3 * 64 + 6, n, 0.0, 0.02, i0=5)
    np.testing.assert_array_equal(t.view(torch.int16).cpu().numpy().view(np.uint16), host)
