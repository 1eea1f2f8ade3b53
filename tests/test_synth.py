"""The input generator: addressable by (seed, stream, index), right distributions, right formats."""
import numpy as np

import synth


def test_counter_addressing_and_determinism():
    a = synth.normal_f64(7, "t", 1000)
    b = synth.normal_f64(7, "t", 1000)
    assert np.array_equal(a, b)
    # a slice regenerated on its own equals the slice of the whole (even offsets keep pairs aligned)
    c = synth.normal_f64(7, "t", 100, first=400)
    assert np.array_equal(a[400:500], c)
    assert not np.array_equal(a, synth.normal_f64(8, "t", 1000))
    assert not np.array_equal(a, synth.normal_f64(7, "u", 1000))


def test_normal_moments_and_bf16_rounding():
    a = synth.normal_f64(0, "m", 400000)
    assert abs(a.mean()) < 0.01 and abs(a.std() - 1.0) < 0.01
    assert abs(np.mean(a ** 3)) < 0.03 and abs(np.mean(a ** 4) - 3.0) < 0.1
    f = synth.normal_f32(0, "w", 50000, 0.0, 0.02)
    b = synth.normal_bf16(0, "w", 50000, 0.0, 0.02)
    back = synth.bf16_bits_to_f32(b)
    assert np.all(np.abs(back - f) <= np.abs(f) * 2.0 ** -8)          # within half a bf16 ulp
    assert np.array_equal(b, synth.f32_to_bf16_bits(f))               # one rounding, nearest-even
    assert abs(back.std() - 0.02) < 4e-4


def test_integer_draws():
    d = synth.uniform_i32(3, "d", 200000, 0, 256)
    assert d.min() == 0 and d.max() == 255
    cnt = np.bincount(d, minlength=256)
    assert cnt.min() > 600 and cnt.max() < 960
    wl = synth.WORKLOADS["C2"]
    off = synth.make_offsets_geometric(synth.Workload("x", synth.TINY, 0, 8, 100, batch=4000, K=7), 0.5)
    assert abs(np.mean(off == 0) - 0.5) < 0.02                       # P(delta = 0) = p
    assert abs(np.mean(np.abs(off) == 1) - 0.25) < 0.02
    assert abs(np.mean(off[off != 0] > 0) - 0.5) < 0.03
    sk = synth.make_skip_mask(synth.Workload("x", synth.TINY, 0, 8, 100, batch=20000, K=7, skip_p=0.3))
    assert abs(sk.mean() - 0.3) < 0.015
    assert wl.prefix_len == 276 and wl.shape.bin_base == 31744


def test_workload_table_matches_configs():
    w = synth.WORKLOADS
    assert (w["C0"].shape.n_layers, w["C0"].shape.d_model, w["C0"].shape.d_ffn, w["C0"].prefix_len) == (2, 256, 688, 64)
    assert w["C1"].shape.weight_bytes() == 32 * 404750336            # 12.952 GB of layer weights
    assert (w["C3"].prefix_len, w["C3"].batch, w["C3"].K) == (532, 16, 14)
    assert (w["C4"].batch * w["C4"].K) == 448
    ws = synth.make_weights(synth.ModelShape(1, 16, 2, 8, 24, 300), seed=1)
    assert ws["wq"][0].shape == (16, 16) and ws["w_down"][0].shape == (16, 24) and ws["lm_head"].dtype == np.uint16
    assert np.all(ws["final_norm"] == 1.0)
