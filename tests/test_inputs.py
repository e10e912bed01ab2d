"""The seeded input generator: determinism, storage formats, structure of the five workloads."""
import numpy as np
import torch

import covspec_inputs as I


def test_bf16_rounding_matches_torch_and_roundtrips():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 3.0e38], dtype=np.float32)])
    bits = I.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    back = I.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(I.f32_to_bf16_bits(back), bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


def test_generation_is_deterministic_and_seeded_per_image():
    w = I.small_workload(cid=7, n_tokens=40, d_model=32, n_query=3, factor_rank=8, dtype=I.BF16)
    a, b = I.make_image(w, 0), I.make_image(w, 0)
    c = I.make_image(w, 1)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    assert not np.array_equal(a["X"], c["X"])
    assert a["X"].dtype == np.uint16 and a["hidden"].shape == (w.n_act_layers + 1, 40, 32)
    np.testing.assert_array_equal(a["hidden"][0], a["X"])
    wt = I.make_weights(w)
    assert wt["Wq"].shape == (32, 32) and not np.array_equal(wt["Wq"], wt["Wk"])


def test_workload_table_matches_the_benchmark_configs():
    shapes = {c: (w.batch, w.n_tokens, w.d_model, w.n_query, w.n_heads, w.keep_k) for c, w in I.WORKLOADS.items()}
    assert shapes == {1: (1, 576, 1024, 16, 8, 64), 2: (1, 576, 4096, 32, 32, 144), 3: (8, 2304, 3584, 64, 28, 576),
                      4: (4, 8192, 1536, 64, 12, 819), 5: (64, 2880, 4096, 128, 32, 320)}
    assert I.WORKLOADS[1].dtype == I.FP32 and all(I.WORKLOADS[c].dtype == I.BF16 for c in (2, 3, 4, 5))
    for w in I.WORKLOADS.values():
        assert w.d_model // w.n_heads == 128 and w.preselect_m == 2 * w.keep_k


def test_structure_unit_rms_duplicates_and_outliers():
    w = I.WORKLOADS[2]
    im = I.make_image(w, 0)
    X = I.as_f64(im["X"], w.dtype)
    norms = np.sqrt((X * X).mean(axis=1))
    assert (norms > 10).sum() == 8                                   # the 20x outliers
    assert 0.7 < np.median(norms) < 1.4                              # unit-RMS signal
    _, inv, counts = np.unique(im["X"], axis=0, return_inverse=True, return_counts=True)
    assert (counts == 2).sum() == 29                                 # 5% exact duplicates
    dup_rows = np.where(counts[inv] == 2)[0]
    for l in range(w.n_act_layers + 1):                              # duplicated in every hidden slice
        assert np.unique(im["hidden"][l][dup_rows], axis=0).shape[0] == 29
