"""The seeded input generator: bf16 rounding, determinism, distributions, planted columns.  CPU only."""
import numpy as np

from paper_2605_10453_amd import synth


def test_bf16_round_to_nearest_even():
    f = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 0.0, 3.0e38], dtype=np.float32)
    b = synth.f32_to_bf16_bits(f)
    back = synth.bf16_bits_to_f32(b)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa (1.0)
    # 1.005859375 = 1 + 1.5*2^-8 rounds up to 1.0078125
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1.0078125 and 1.015625 -> even (1.015625)
    assert back.tolist()[:5] == [1.0, 1.0, 1.0078125, 1.015625, -2.5]
    assert b[5] == 0
    assert np.array_equal(synth.f32_to_bf16_bits(back), b)          # idempotent
    assert synth.bf16_bits_to_f64(b).dtype == np.float64


def test_seeded_and_distinct():
    cfg = synth.small_config(rows=20, d=128, r=16, V=2048, k=4, peaked_every=10)
    a, b, c = synth.make_inputs(cfg, 3), synth.make_inputs(cfg, 3), synth.make_inputs(cfg, 4)
    assert np.array_equal(a.h, b.h) and np.array_equal(a.B, b.B) and np.array_equal(a.A, b.A)
    assert not np.array_equal(a.B, c.B)
    assert a.W is None and synth.make_inputs(cfg, 3, with_full_head=True).W.shape == (128, 2048)
    # adding the full head afterwards does not change h, A, B (draw order h, A, B, W)
    assert np.array_equal(synth.make_inputs(cfg, 3, with_full_head=True).B, a.B)


def test_scales_and_peaked_rows():
    cfg = synth.small_config(rows=30, d=1024, r=128, V=4096, k=4, peaked_every=10)
    x = synth.make_inputs(cfg, 0, with_full_head=True)
    h, A, B, W = (synth.bf16_bits_to_f64(m) for m in (x.h, x.A, x.B, x.W))
    assert abs(A.std() * cfg.d ** 0.5 - 1) < 0.02        # variance 1/d
    assert abs(B.std() * cfg.r ** 0.5 - 1) < 0.02        # variance 1/r
    assert abs(W.std() * cfg.d ** 0.5 - 1) < 0.02
    rms = np.sqrt((h ** 2).mean(axis=1))
    peaked = np.arange(cfg.rows) % 10 == 0
    assert np.all(np.abs(rms[peaked] - 4) < 0.4) and np.all(np.abs(rms[~peaked] - 1) < 0.1)
    z = (h @ A) @ B
    assert abs(z[~peaked].std() - 1) < 0.1               # unit-variance logits


def test_plant_identical_columns():
    cfg = synth.small_config(rows=1, d=8, r=4, V=32, k=2)
    x = synth.make_inputs(cfg, 0)
    synth.plant_identical_columns(x.B, np.array([0.1, -2.0, 3.3, 0.0]), [0, 16, 31])
    assert np.array_equal(x.B[:, 0], x.B[:, 16]) and np.array_equal(x.B[:, 0], x.B[:, 31])
    assert synth.bf16_bits_to_f32(x.B[:, 0])[1] == -2.0


def test_named_configs_have_the_stated_shapes():
    c = synth.CONFIGS
    assert (c["C1"].rows, c["C1"].d, c["C1"].r, c["C1"].V, c["C1"].k) == (1, 256, 32, 8192, 8)
    assert (c["C2"].rows, c["C2"].d, c["C2"].r, c["C2"].V, c["C2"].k) == (1, 4096, 512, 128256, 10)
    assert (c["C3"].rows, c["C3"].d, c["C3"].r, c["C3"].V, c["C3"].k) == (1, 5120, 640, 151936, 10)
    assert (c["C4"].rows, c["C4"].d, c["C4"].r, c["C4"].V, c["C4"].k) == (512, 4096, 512, 128256, 10)
    assert (c["C5"].rows, c["C5"].d, c["C5"].r, c["C5"].V, c["C5"].k) == (256, 8192, 1024, 128256, 16)
    assert c["C4_r256"].r == 256 and c["C4_r1024"].r == 1024
