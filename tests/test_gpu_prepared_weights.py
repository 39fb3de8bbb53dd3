"""GPU parity of slimspec_head_topk_prepared (the low-rank head with the caller's column-major copy of B) against the
CPU fp64 checker, to the same bar as slimspec_head_topk: the special cases of test_gpu_parity.py run again with the
head call replaced, plus the copy itself and a seeded sweep of random shapes."""
import numpy as np
import pytest

import test_gpu_parity as base
from paper_2605_10453_amd import synth
from parity_util import to_dev_bf16
from test_gpu_parity import gpu  # noqa: F401  (the module's fixture)

pytestmark = pytest.mark.gpu


def run_low_rank_prepared(gpu, x, k):
    torch, b = gpu
    B = to_dev_bf16(x.B)
    Bt = b.slimspec_transpose_weights(B)
    ids, lp = b.slimspec_head_topk_prepared(to_dev_bf16(x.h), to_dev_bf16(x.A), B, Bt, k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), lp.cpu().numpy()


@pytest.fixture
def prepared(monkeypatch):
    """check_low_rank and the tests of test_gpu_parity.py call the prepared entry point."""
    monkeypatch.setattr(base, "run_low_rank", run_low_rank_prepared)


@pytest.mark.parametrize("K,V", [(8, 8), (40, 520), (64, 64), (72, 8200), (512, 4104), (1024, 1032)])
def test_column_major_copy(gpu, K, V):
    torch, b = gpu
    rng = np.random.default_rng(K * 131 + V)
    M = rng.integers(0, 1 << 16, size=(K, V), dtype=np.uint16)
    Mt = b.slimspec_transpose_weights(to_dev_bf16(M))
    torch.cuda.synchronize()
    assert np.array_equal(Mt.view(torch.int16).cpu().numpy().view(np.uint16), np.ascontiguousarray(M.T))


SPECIAL = {
    "not_gaussian_scaled_columns_k10": (base.test_matrix_core_path_weights_not_gaussian, dict(kind="scaled_columns", k=10)),
    "not_gaussian_scaled_columns_k16": (base.test_matrix_core_path_weights_not_gaussian, dict(kind="scaled_columns", k=16)),
    "not_gaussian_heavy_tailed_k10": (base.test_matrix_core_path_weights_not_gaussian, dict(kind="heavy_tailed", k=10)),
    "not_gaussian_heavy_tailed_k16": (base.test_matrix_core_path_weights_not_gaussian, dict(kind="heavy_tailed", k=16)),
    "not_gaussian_small_rows_k10": (base.test_matrix_core_path_weights_not_gaussian, dict(kind="small_every_8th_row", k=10)),
    "not_gaussian_large_rows_k16": (base.test_matrix_core_path_weights_not_gaussian, dict(kind="large_every_8th_row_offset_3", k=16)),
    "wide_rounding_bound": (base.test_wide_rounding_bound_with_few_winners, {}),
    "two_probable_tokens_in_one_group": (base.test_two_probable_tokens_in_one_group_of_sixteen, {}),
    "logit_far_above_the_running_maximum": (base.test_logit_far_above_the_running_maximum, {}),
    "rising_logits_k16": (base.test_rising_logits_through_the_exhaustive_pass, dict(k=16)),
    "rising_logits_k10": (base.test_rising_logits_through_the_exhaustive_pass, dict(k=10)),
    "zero_hidden_state": (base.test_zero_hidden_state_all_tied, {}),
    "planted_exact_ties_six_rows": (base.test_planted_exact_ties, dict(rows=6)),
    "zero_rows_inside_a_batch": (base.test_zero_rows_inside_a_many_row_batch, {}),
    "more_rows_than_one_launch": (base.test_more_rows_than_one_launch, {}),
    "few_rows_do_not_read_the_copy": (base.test_low_rank_small, dict(zip(("rows", "d", "r", "V", "k"), base.SMALL[6]))),
    "large_k_does_not_read_the_copy": (base.test_many_rows_large_k, dict(rows=20, k=17)),
    "four_best_in_one_lane_stream_4_records": (base.test_four_best_logits_in_one_lane_stream, dict(rows=300, V=40960)),
    "four_best_in_one_lane_stream_2_records": (base.test_four_best_logits_in_one_lane_stream, dict(rows=200, V=70000)),
    "four_best_in_one_lane_stream_1_record": (base.test_four_best_logits_in_one_lane_stream, dict(rows=20, V=70000)),
    "C4": (base.test_config4_low_rank, dict(name="C4")),
    "C4_r256": (base.test_config4_low_rank, dict(name="C4_r256")),
    "C4_r1024": (base.test_config4_low_rank, dict(name="C4_r1024")),
    "C5_planted_ties": (base.test_config5_with_planted_ties, {}),
}


@pytest.mark.parametrize("case", list(SPECIAL))
def test_special_cases_with_prepared_weights(gpu, oracle_mod, prepared, case):
    fn, kwargs = SPECIAL[case]
    fn(gpu, oracle_mod, **kwargs)


@pytest.mark.parametrize("rows,d,r,V,k", [c for c in base.SMALL if c[0] >= 5 and c[4] <= 16])
def test_small_shapes_with_prepared_weights(gpu, oracle_mod, prepared, rows, d, r, V, k):
    base.test_low_rank_small(gpu, oracle_mod, rows, d, r, V, k)


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        rows = int(rng.choice([5, 6, 9, 17, 33, 70, 129, 200, 513]))
        d = 8 * int(rng.integers(1, 65))
        r = 8 * int(rng.integers(1, 130))                   # contraction lengths on both sides of one 512-element step
        V = 8 * int(rng.integers(1, 1500))
        k = int(min(V, rng.choice([1, 2, 5, 10, 13, 16])))
        out.append((rows, d, r, V, k, int(rng.choice([0, 3, 10])), bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("rows,d,r,V,k,peaked_every,scaled", _random_cases(40, 20261128))
def test_random_shapes_with_prepared_weights(gpu, oracle_mod, prepared, rows, d, r, V, k, peaked_every, scaled):
    """Seeded shapes nobody picked by hand on the matrix-core path; in half of them some columns of B are 8 and 32
    times larger than the rest (wide rounding bounds: more exact re-evaluations, unlisted members)."""
    cfg = synth.small_config(rows=rows, d=d, r=r, V=V, k=k, peaked_every=peaked_every)
    x = synth.make_inputs(cfg, 31000 + rows + V)
    if scaled:
        rng = np.random.default_rng(V)
        B = synth.bf16_bits_to_f32(x.B)
        cols = rng.choice(V, min(V, 24), replace=False)
        B[:, cols[:16]] *= np.float32(8.0)
        B[:, cols[16:]] *= np.float32(32.0)
        x.B = synth.f32_to_bf16_bits(B)
    base.check_low_rank(gpu, oracle_mod, x, k)


def test_prepared_call_is_deterministic_and_matches_the_plain_call(gpu):
    """Same ids as slimspec_head_topk and log-probabilities within the last bits (the exact logits are summed in another
    order); two prepared calls agree bit for bit."""
    torch, b = gpu
    cfg = synth.small_config(rows=300, d=256, r=520, V=20008, k=10, peaked_every=4)
    x = synth.make_inputs(cfg, 8)
    h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
    Bt = b.slimspec_transpose_weights(B)
    ids0, lp0 = b.slimspec_head_topk(h, A, B, cfg.k)
    ids1, lp1 = b.slimspec_head_topk_prepared(h, A, B, Bt, cfg.k)
    ids2, lp2 = b.slimspec_head_topk_prepared(h, A, B, Bt, cfg.k)
    torch.cuda.synchronize()
    assert torch.equal(ids1, ids2) and torch.equal(lp1.view(torch.int32), lp2.view(torch.int32))
    assert torch.equal(ids0, ids1)
    assert float((lp0 - lp1).abs().max()) < 1e-4
