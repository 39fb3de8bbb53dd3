"""Pins of the checker's functions for the heads around the low-rank head (truncated vocabulary, position-specific
down-projections, router-then-exact) and for Gumbel-max sampling: closed forms, reductions to the already pinned
heads, the Gumbel-max theorem's frequencies.  CPU only."""
import math

import numpy as np
import pytest

from paper_2605_10453_amd import synth


@pytest.fixture(scope="module")
def inputs():
    cfg = synth.small_config(rows=5, d=48, r=16, V=200, k=7)
    return synth.make_inputs(cfg, seed=11, with_full_head=True)


# ------------------------------------------------------------------ truncated-vocabulary head

def test_truncated_identity_map_is_the_full_head(oracle_mod, inputs):
    x = inputs
    V = x.cfg.V
    a = oracle_mod.truncated_head_topk(x.h, x.W, np.arange(V), 7)
    b = oracle_mod.full_head_topk(x.h, x.W, 7)
    assert np.array_equal(a.ids, b.ids) and np.array_equal(a.logprobs, b.logprobs) and np.array_equal(a.lse, b.lse)


def test_truncated_permuted_columns_map_back(oracle_mod, inputs):
    """W_tr = W[:, perm] with id_map = perm is the same head (random weights: no ties)."""
    x = inputs
    perm = np.random.default_rng(3).permutation(x.cfg.V).astype(np.int32)
    a = oracle_mod.truncated_head_topk(x.h, np.ascontiguousarray(x.W[:, perm]), perm, 7)
    b = oracle_mod.full_head_topk(x.h, x.W, 7)
    assert np.array_equal(a.ids, b.ids)
    assert np.allclose(a.logprobs, b.logprobs, atol=1e-6) and np.allclose(a.lse, b.lse, atol=1e-12)


def test_truncated_subset_renormalises_the_full_distribution(oracle_mod, inputs):
    """Masked softmax (section 4.2): over a kept subset S, log p~(v) = log p(v) - log sum_{u in S} p(u)."""
    x = inputs
    V = x.cfg.V
    keep = np.sort(np.random.default_rng(5).choice(V, 60, replace=False)).astype(np.int32)
    full = oracle_mod.full_head_topk(x.h, x.W, V)                      # k = V: the whole sorted distribution
    lp_full = np.empty((x.cfg.rows, V))
    for i in range(x.cfg.rows):
        lp_full[i, full.ids[i]] = full.logprobs[i]
    tr = oracle_mod.truncated_head_topk(x.h, np.ascontiguousarray(x.W[:, keep]), keep, 9)
    for i in range(x.cfg.rows):
        mass = np.log(np.exp(lp_full[i, keep]).sum())
        assert np.allclose(tr.logprobs[i], lp_full[i, tr.ids[i]] - mass, atol=2e-6)
        best = keep[np.argsort(-lp_full[i, keep], kind="stable")[:9]]
        assert np.array_equal(tr.ids[i], best)


def test_truncated_ties_break_by_column_not_by_mapped_id(oracle_mod):
    h = synth.f32_to_bf16_bits(np.ones((1, 8), np.float32))
    W = synth.f32_to_bf16_bits(np.ones((8, 4), np.float32))              # four identical columns
    r = oracle_mod.truncated_head_topk(h, W, np.array([9, 3, 7, 1], np.int32), 3)
    assert r.ids[0].tolist() == [9, 3, 7]


# ------------------------------------------------------------------ position-specific down-projections

def test_positions_one_position_is_the_plain_head(oracle_mod, inputs):
    x = inputs
    a = oracle_mod.slimspec_head_topk_positions(x.h, x.A[None], [0, x.cfg.rows], x.B, 7)
    b = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, 7)
    assert np.array_equal(a.ids, b.ids) and np.array_equal(a.logprobs, b.logprobs)


def test_positions_rows_use_their_own_projection(oracle_mod, inputs):
    """Rows of position p must give what the plain head gives with A_stack[p] alone; an empty position is allowed."""
    x = inputs
    rng = np.random.default_rng(8)
    A2 = synth.f32_to_bf16_bits((rng.standard_normal(x.A.shape) * x.cfg.d ** -0.5).astype(np.float32))
    A3 = synth.f32_to_bf16_bits((rng.standard_normal(x.A.shape) * x.cfg.d ** -0.5).astype(np.float32))
    stack = np.stack([x.A, A2, A3])
    off = [0, 2, 2, 5]
    got = oracle_mod.slimspec_head_topk_positions(x.h, stack, off, x.B, 7, return_logits=True)
    for p, Ap in enumerate(stack):
        r0, r1 = off[p], off[p + 1]
        if r1 == r0:
            continue
        ref = oracle_mod.slimspec_head_topk(x.h[r0:r1], Ap, x.B, 7, return_logits=True)
        assert np.array_equal(got.ids[r0:r1], ref.ids) and np.array_equal(got.z[r0:r1], ref.z)
    # and the rows of position 2 differ from what position 0's projection would give
    other = oracle_mod.slimspec_head_topk(x.h[2:5], x.A, x.B, 7, return_logits=True)
    assert not np.allclose(other.z, got.z[2:5])


# ------------------------------------------------------------------ Gumbel-max sampling

def test_gumbel_noise_has_the_standard_gumbel_moments(oracle_mod):
    g = np.concatenate([oracle_mod.gumbel_noise(seed, row, np.arange(20000)) for seed, row in ((1, 0), (2, 5), (2 ** 40 + 3, 1))])
    n = g.size
    assert abs(g.mean() - 0.5772156649) < 5 * math.sqrt(math.pi ** 2 / 6 / n)
    assert abs(g.var() - math.pi ** 2 / 6) < 0.03
    # P(g <= x) = exp(-exp(-x)) at a few points
    for xq in (-1.0, 0.0, 1.0, 3.0):
        p = math.exp(-math.exp(-xq))
        assert abs((g <= xq).mean() - p) < 5 * math.sqrt(p * (1 - p) / n)


def test_gumbel_noise_depends_on_seed_row_and_id(oracle_mod):
    ids = np.arange(64)
    a = oracle_mod.gumbel_noise(7, 0, ids)
    assert not np.array_equal(a, oracle_mod.gumbel_noise(8, 0, ids))
    assert not np.array_equal(a, oracle_mod.gumbel_noise(7 + 2 ** 32, 0, ids))         # the high half of the seed counts
    assert not np.array_equal(a, oracle_mod.gumbel_noise(7, 1, ids))
    assert np.array_equal(a, oracle_mod.gumbel_noise(7, 0, ids))
    assert len(set(np.round(a, 12))) == 64
    # draws of neighbouring ids / rows / seeds are uncorrelated
    big = oracle_mod.gumbel_noise(7, 0, np.arange(40001))
    assert abs(np.corrcoef(big[:-1], big[1:])[0, 1]) < 0.02
    assert abs(np.corrcoef(oracle_mod.gumbel_noise(7, 0, np.arange(20000)), oracle_mod.gumbel_noise(7, 1, np.arange(20000)))[0, 1]) < 0.03
    assert abs(np.corrcoef(oracle_mod.gumbel_noise(7, 0, np.arange(20000)), oracle_mod.gumbel_noise(8, 0, np.arange(20000)))[0, 1]) < 0.03


def test_sample_with_one_dominant_logit_is_the_argmax(oracle_mod):
    z = np.zeros(300)
    z[123] = 100.0
    for seed in range(50):
        assert oracle_mod.sample_row(z, seed, 0)[0] == 123


def test_sample_frequencies_follow_the_softmax(oracle_mod):
    """Gumbel-max theorem: over many seeds the sampled id has the softmax's frequencies (binomial bound, 5 sigma)."""
    z = np.log(np.array([0.5, 0.25, 0.125, 0.0625, 0.03125, 0.03125]))
    p = np.exp(z) / np.exp(z).sum()
    n = 20000
    counts = np.zeros(6)
    for seed in range(n):
        counts[oracle_mod.sample_row(z, seed, 3)[0]] += 1
    for v in range(6):
        assert abs(counts[v] / n - p[v]) < 5 * math.sqrt(p[v] * (1 - p[v]) / n), (v, counts / n, p)
    # shift invariance: adding a constant to every logit draws the same token
    for seed in range(100):
        assert oracle_mod.sample_row(z, seed, 0)[0] == oracle_mod.sample_row(z + 7.25, seed, 0)[0]


def test_head_sample_is_the_head_plus_a_row_sample(oracle_mod, inputs):
    x = inputs
    s = oracle_mod.head_sample(x.h, x.A, x.B, 7, seed=99, return_logits=True)
    ref = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, 7, return_logits=True)
    assert np.array_equal(s.ids, ref.ids) and np.array_equal(s.logprobs, ref.logprobs) and np.array_equal(s.lse, ref.lse)
    for i in range(x.cfg.rows):
        sid, _ = oracle_mod.sample_row(ref.z[i], 99, i)
        assert s.sample_ids[i] == sid
        assert abs(s.sample_logprobs[i] - (ref.z[i, sid] - ref.lse[i])) < 1e-6
        g = oracle_mod.gumbel_noise(99, i, np.arange(x.cfg.V))
        assert sid == int(np.argmax(ref.z[i] + g))
    f = oracle_mod.head_sample(x.h, None, x.W, 7, seed=99)
    assert np.array_equal(f.ids, oracle_mod.full_head_topk(x.h, x.W, 7).ids)


# ------------------------------------------------------------------ router-then-exact head

def test_routed_head_with_every_token_routed_is_the_full_head(oracle_mod, inputs):
    x = inputs
    ids, lp, lse, route = oracle_mod.routed_head_topk(x.h, x.A, x.B, x.W, x.cfg.V, 7)
    full = oracle_mod.full_head_topk(x.h, x.W, 7)
    assert np.array_equal(ids, full.ids) and np.allclose(lp, full.logprobs, atol=1e-6) and np.allclose(lse, full.lse, atol=1e-10)
    assert np.array_equal(route, oracle_mod.slimspec_head_topk(x.h, x.A, x.B, x.cfg.V).ids)


def test_routed_head_renormalises_over_the_routed_subset(oracle_mod, inputs):
    """The k_route router winners, exact logits on them, softmax over that subset only."""
    x = inputs
    kr = 20
    ids, lp, lse, route = oracle_mod.routed_head_topk(x.h, x.A, x.B, x.W, kr, 5)
    router = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, kr)
    assert np.array_equal(route, router.ids)
    zW = synth.bf16_bits_to_f64(x.h) @ synth.bf16_bits_to_f64(x.W)
    for i in range(x.cfg.rows):
        y = zW[i, route[i]]
        ref_lse = np.log(np.exp(y - y.max()).sum()) + y.max()
        order = np.lexsort((route[i], -y))[:5]
        assert np.array_equal(ids[i], route[i][order])
        assert np.allclose(lp[i], y[order] - ref_lse, atol=1e-6) and abs(lse[i] - ref_lse) < 1e-10
