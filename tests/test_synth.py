"""The seeded input generator: determinism, shapes and the stated structure."""
import numpy as np

from paper_2506_15050_amd import synth


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], np.float32)   # 1+2^-8 ties to even (down), 1+3*2^-8 ties up
    bits = synth.f32_to_bf16_bits(x)
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]
    assert np.array_equal(synth.bf16_bits_to_f32(bits), np.array([1.0, 1.0, 1.015625, -2.5, 0.0], np.float32))


def test_tiny_shape_and_determinism():
    a, b = synth.make_batch("tiny"), synth.make_batch("tiny")
    for k, v in a.items():
        if isinstance(v, np.ndarray):
            assert np.array_equal(v, b[k]), k
    assert a["B"] == 4 and a["done"].tolist() == [1, 0, 1, 0]
    assert a["win_len"][1] == 64 and a["win_len"][3] == 64
    assert a["hidden"].dtype == np.float32 and a["hidden"].shape == (a["n_tok"], 64)
    assert a["w_head"].shape == (1000, 64)
    fin_last = a["resp_off"][1:][a["done"] != 0] - 1
    assert np.all(np.abs(a["rewards"][fin_last]) == 1.0)
    assert np.count_nonzero(a["rewards"]) == 2
    assert a["input_ids"].min() >= 0 and a["input_ids"].max() < 1000


def test_longcot_structure():
    b = synth.make_batch("longcot")
    assert b["B"] == 512 and 256 <= b["win_len"].min() and b["win_len"].max() <= 20480
    assert 0.2 < b["done"].mean() < 0.4
    assert np.abs(b["values"]).max() <= 1.0
    assert np.count_nonzero(b["rewards"]) == int(b["done"].sum())


def test_small_is_bf16_and_threads_do_not_matter():
    b = synth.make_batch("small", B=3, H=64, V=300)
    assert b["hidden"].dtype == np.uint16 and b["w_head"].shape == (300, 64)
    w = synth.bf16_bits_to_f32(b["w_head"])
    assert 0.015 < w.std() < 0.025
    m1 = synth._normal_matrix(5, "w", 10000, 8, 1.0, "f32", block_rows=1024)
    m2 = synth._normal_matrix(5, "w", 10000, 8, 1.0, "f32", block_rows=1024)
    assert np.array_equal(m1, m2)


def test_drop_fraction_solver():
    b = synth.make_batch("head7b", with_head=False)
    trunc = b["win_len"][b["done"] == 0]
    dropped = np.minimum(trunc, b["tail_drop"]).sum()
    assert abs(dropped / b["n_resp"] - 0.25) < 0.01


def test_sampling_ids_cpu_small():
    b = synth.make_batch("head32b", B=2, H=32, V=97, ctx=4, window=16,
                         len_dist=("uniform", 4, 16))
    before = b["input_ids"].copy()
    synth.sample_ids_from_policy(b, device="cpu", row_block=7)
    ids = b["input_ids"]
    assert ids.min() >= 0 and ids.max() < 97
    cu, ctx = b["cu_seqlens"], b["ctx_len"]
    for i in range(2):     # context tokens untouched
        assert np.array_equal(ids[cu[i]:cu[i] + ctx[i]], before[cu[i]:cu[i] + ctx[i]])
