"""GPU parity of the heads around the low-rank head (truncated vocabulary, position-specific down-projections,
router-then-exact) and of the stochastic-decoding outputs, against the CPU fp64 checker.  Same bar as the main
parity tests: ids identical except where the checker's logits are within 1e-3, log-probabilities within 2e-2."""
import numpy as np
import pytest

from paper_2605_10453_amd import synth
from parity_util import compare_with_oracle, to_dev_bf16, to_dev_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2605_10453_amd import binding
    assert torch.cuda.is_available(), "these tests need the GPU"
    binding.load_library()
    return torch, binding


# ------------------------------------------------------------------ truncated-vocabulary head

@pytest.mark.parametrize("rows,d,V_full,V_tr,k,w_f32", [
    (1, 256, 20000, 8200, 10, False),       # streaming path
    (3, 128, 9000, 3080, 7, True),          # fp32 weights
    (9, 96, 9000, 2056, 6, False),          # matrix-core path, natural-unit mode
    (70, 128, 12000, 5000, 16, False),
    (12, 2048, 9000, 4104, 8, False),       # long contraction: parked rows
])
def test_truncated_head(gpu, oracle_mod, rows, d, V_full, V_tr, k, w_f32):
    torch, b = gpu
    print(f"truncated head rows={rows} d={d} V={V_full} V_tr={V_tr} k={k} f32={w_f32}", flush=True)
    x = synth.make_inputs(synth.small_config(rows, d, 8, V_full, k, peaked_every=4), seed=40 + rows, with_full_head=True)
    keep = np.sort(np.random.default_rng(rows).choice(V_full, V_tr, replace=False)).astype(np.int32)
    id_map = keep[np.random.default_rng(rows + 1).permutation(V_tr)]                # kept columns in an arbitrary order
    W_tr = np.ascontiguousarray(x.W[:, id_map])
    if w_f32:
        W_tr = synth.bf16_bits_to_f32(W_tr)
    Wd = to_dev_f32(W_tr) if w_f32 else to_dev_bf16(W_tr)
    ids, lp = b.truncated_head_topk(to_dev_bf16(x.h), Wd, torch.from_numpy(id_map).cuda(), k)
    torch.cuda.synchronize()
    ids, lp = ids.cpu().numpy(), lp.cpu().numpy()
    ora = oracle_mod.truncated_head_topk(x.h, W_tr, id_map, k)
    # back to columns of W_tr, where the comparator and the checker's logits live
    col_of = np.full(V_full, -1, np.int64)
    col_of[id_map] = np.arange(V_tr)
    assert (col_of[ids] >= 0).all(), "an id outside the kept subset"
    z_at = lambda ri, ci: oracle_mod.full_logits_at(x.h, W_tr, ri, ci)
    compare_with_oracle(col_of[ids].astype(np.int32), lp, col_of[ora.ids].astype(np.int32), ora.lse, z_at, V_tr)


def test_truncated_head_tied_columns_break_by_column(gpu, oracle_mod):
    """Identical kept columns: the smaller column wins whatever vocabulary id it maps to."""
    torch, b = gpu
    for rows in (2, 12):
        x = synth.make_inputs(synth.small_config(rows, 64, 8, 1032, 4), seed=3, with_full_head=True)
        W = x.W.copy()
        h0 = synth.bf16_bits_to_f64(x.h[0])
        synth.plant_identical_columns(W, 0.5 * h0 / 8.0, [5, 500, 1000])
        id_map = np.arange(1032, dtype=np.int32)[::-1].copy()                       # column c is vocabulary id 1031 - c
        ids, _ = b.truncated_head_topk(to_dev_bf16(x.h), to_dev_bf16(W), torch.from_numpy(id_map).cuda(), 4)
        torch.cuda.synchronize()
        ora = oracle_mod.truncated_head_topk(x.h, W, id_map, 4)
        assert ids.cpu().numpy()[0, :3].tolist() == [1026, 531, 31] == ora.ids[0, :3].tolist()


# ------------------------------------------------------------------ position-specific down-projections

@pytest.mark.parametrize("sizes,d,r,V,k", [
    ((1, 1, 1), 256, 32, 8200, 8),                  # streaming path, every row its own matrix
    ((2, 0, 2), 128, 16, 5000, 5),                  # ... an empty position
    ((4,), 128, 16, 5000, 5),                       # one position: the plain head
    ((3, 1, 0, 5), 96, 24, 2056, 7),                # matrix-core path, groups smaller than a tile
    ((70, 1, 0, 129), 128, 40, 3080, 10),           # groups that end inside a row tile
    ((64, 64, 64), 256, 64, 4104, 16),              # groups that fill their tiles; f16 operands
    ((300, 250, 50), 64, 32, 1032, 5),              # two launches: a group crosses the 512-row boundary
    ((9, 11), 128, 32, 3080, 20),                   # k beyond the matrix-core path: streaming in row groups of 8
    ((100, 60, 40), 64, 64, 70000, 5),              # many column blocks: two records per block and row
    ((7, 13), 64, 64, 70000, 5),                    # ... one record
])
@pytest.mark.parametrize("prepared", [False, True])
def test_position_specific_down_projections(gpu, oracle_mod, sizes, d, r, V, k, prepared):
    torch, b = gpu
    rows, n_pos = sum(sizes), len(sizes)
    print(f"positions case sizes={sizes} d={d} r={r} V={V} k={k}", flush=True)
    x = synth.make_inputs(synth.small_config(rows, d, r, V, k, peaked_every=5), seed=70 + rows)
    rng = np.random.default_rng(rows)
    stack = np.stack([x.A] + [synth.f32_to_bf16_bits((rng.standard_normal((d, r)) * d ** -0.5).astype(np.float32))
                              for _ in range(n_pos - 1)])
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    stack_dev, B = to_dev_bf16(stack.reshape(n_pos * d, r)).view(n_pos, d, r), to_dev_bf16(x.B)
    if prepared:      # with the column-major copy of B as well
        ids, lp = b.slimspec_head_topk_positions_prepared(to_dev_bf16(x.h), stack_dev, off.tolist(), B, b.slimspec_transpose_weights(B), k)
    else:
        ids, lp = b.slimspec_head_topk_positions(to_dev_bf16(x.h), stack_dev, off.tolist(), B, k)
    torch.cuda.synchronize()
    ora = oracle_mod.slimspec_head_topk_positions(x.h, stack, off, x.B, k, return_logits=True)
    z_at = lambda ri, ci: ora.z[ri, ci]
    compare_with_oracle(ids.cpu().numpy(), lp.cpu().numpy(), ora.ids, ora.lse, z_at, V)


def test_positions_with_one_matrix_equal_the_plain_head(gpu):
    torch, b = gpu
    for rows in (2, 40):
        x = synth.make_inputs(synth.small_config(rows, 128, 32, 4104, 6), seed=5)
        h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
        a_ids, a_lp = b.slimspec_head_topk(h, A, B, 6)
        p_ids, p_lp = b.slimspec_head_topk_positions(h, A.view(1, 128, 32), [0, rows], B, 6)
        torch.cuda.synchronize()
        assert torch.equal(a_ids, p_ids) and torch.equal(a_lp.view(torch.int32), p_lp.view(torch.int32))


# ------------------------------------------------------------------ stochastic-decoding outputs

def check_sample_outputs(torch, out, ora, seed, V, z_rows, oracle_mod):
    """out: the library's five outputs; ora: the checker's SampleResult with z.  The drawn id must be the checker's,
    or one whose z + g (checker's arithmetic) is within the tie tolerance of the checker's largest."""
    ids, lp, lse, sid, slp = [t.cpu().numpy() for t in out]
    rows = ids.shape[0]
    z_at = lambda ri, ci: z_rows[ri, ci]
    compare_with_oracle(ids, lp, ora.ids, ora.lse, z_at, V)
    assert np.abs(lse - ora.lse).max() <= 2e-2, np.abs(lse - ora.lse).max()
    n_other = 0
    for i in range(rows):
        assert 0 <= sid[i] < V
        if sid[i] != ora.sample_ids[i]:
            g = oracle_mod.gumbel_noise(seed, i, [sid[i], ora.sample_ids[i]])
            w_gpu, w_ora = z_rows[i, sid[i]] + g[0], z_rows[i, ora.sample_ids[i]] + g[1]
            assert w_ora - w_gpu <= 1e-3, (i, sid[i], ora.sample_ids[i], w_gpu, w_ora)
            n_other += 1
        assert abs(slp[i] - (z_rows[i, sid[i]] - ora.lse[i])) <= 2e-2
    return n_other


@pytest.mark.parametrize("rows,d,r,V,k,seed", [
    (1, 256, 32, 8200, 8, 1), (1, 64, 16, 140000, 5, 2 ** 40 + 17), (3, 128, 16, 5000, 6, 3), (4, 512, 64, 10248, 10, 4),
    (9, 96, 24, 2056, 7, 5), (40, 256, 32, 4104, 12, 6), (130, 64, 40, 2056, 5, 7), (20, 128, 32, 3080, 20, 8),
    (12, 64, 24, 2056, 16, 9),
    (200, 64, 64, 70000, 5, 10), (20, 64, 64, 70000, 5, 11),       # many column blocks: two records, one record per block and row
])
@pytest.mark.parametrize("prepared", [False, True])
def test_low_rank_head_sample(gpu, oracle_mod, rows, d, r, V, k, seed, prepared):
    torch, b = gpu
    print(f"sample case rows={rows} d={d} r={r} V={V} k={k} seed={seed} prepared={prepared}", flush=True)
    x = synth.make_inputs(synth.small_config(rows, d, r, V, k, peaked_every=4), seed=200 + rows)
    if prepared:      # with the column-major copy of B as well
        B = to_dev_bf16(x.B)
        out = b.slimspec_head_sample_prepared(to_dev_bf16(x.h), to_dev_bf16(x.A), B, b.slimspec_transpose_weights(B), k, seed)
    else:
        out = b.slimspec_head_sample(to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B), k, seed)
    torch.cuda.synchronize()
    ora = oracle_mod.head_sample(x.h, x.A, x.B, k, seed, return_logits=True)
    check_sample_outputs(torch, out, ora, seed, V, ora.z, oracle_mod)
    # the top-k of a sampling call is the top-k of the plain call
    ids, lp = b.slimspec_head_topk(to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B), k)
    torch.cuda.synchronize()
    assert torch.equal(ids, out[0])


@pytest.mark.parametrize("rows,w_f32", [(2, False), (3, True), (33, False)])
def test_full_head_sample(gpu, oracle_mod, rows, w_f32):
    torch, b = gpu
    x = synth.make_inputs(synth.small_config(rows, 128, 8, 6152, 9, peaked_every=3), seed=300 + rows, with_full_head=True)
    W = synth.bf16_bits_to_f32(x.W) if w_f32 else x.W
    out = b.full_head_sample(to_dev_bf16(x.h), to_dev_f32(W) if w_f32 else to_dev_bf16(W), 9, 77)
    torch.cuda.synchronize()
    ora = oracle_mod.head_sample(x.h, None, W, 9, 77, return_logits=True)
    check_sample_outputs(torch, out, ora, 77, 6152, ora.z, oracle_mod)


def test_sample_frequencies_on_the_gpu(gpu, oracle_mod):
    """Many seeds on one row: the drawn ids follow the checker's softmax (binomial bound on the most likely tokens)."""
    torch, b = gpu
    x = synth.make_inputs(synth.small_config(1, 64, 8, 520, 5), seed=12)
    hf = synth.bf16_bits_to_f32(x.h) * np.float32(2.0)                 # a sharper row: a few tokens carry most of the mass
    x.h = synth.f32_to_bf16_bits(hf)
    h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
    ora = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, 5, return_logits=True)
    p = np.exp(ora.z[0] - ora.lse[0])
    n = 3000
    counts = np.zeros(520)
    for seed in range(n):
        counts[int(b.slimspec_head_sample(h, A, B, 5, seed)[3][0])] += 1
    for v in np.argsort(-p)[:4]:
        assert abs(counts[v] / n - p[v]) < 5 * np.sqrt(p[v] * (1 - p[v]) / n), (v, counts[v] / n, p[v])


def test_config2_sample(gpu, oracle_mod):
    """The single-row latency workload with the outputs of stochastic decoding, three seeds."""
    torch, b = gpu
    cfg = synth.CONFIGS["C2"]
    x = synth.make_inputs(cfg, 0)
    h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
    for seed in (0, 1, 2 ** 33 + 5):
        out = b.slimspec_head_sample(h, A, B, cfg.k, seed)
        torch.cuda.synchronize()
        ora = oracle_mod.head_sample(x.h, x.A, x.B, cfg.k, seed, return_logits=True)
        check_sample_outputs(torch, out, ora, seed, cfg.V, ora.z, oracle_mod)


@pytest.mark.parametrize("prepared", [False, True])
def test_config4_sample(gpu, oracle_mod, prepared):
    """The 512-row throughput workload (matrix-core path, peaked rows) with the outputs of stochastic decoding."""
    torch, b = gpu
    cfg = synth.CONFIGS["C4"]
    x = synth.make_inputs(cfg, 0)
    if prepared:
        B = to_dev_bf16(x.B)
        out = b.slimspec_head_sample_prepared(to_dev_bf16(x.h), to_dev_bf16(x.A), B, b.slimspec_transpose_weights(B), cfg.k, 12345)
    else:
        out = b.slimspec_head_sample(to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B), cfg.k, 12345)
    torch.cuda.synchronize()
    ora = oracle_mod.head_sample(x.h, x.A, x.B, cfg.k, 12345, return_logits=True)
    n_other = check_sample_outputs(torch, out, ora, 12345, cfg.V, ora.z, oracle_mod)
    print(f"C4 sampling: {n_other} of {cfg.rows} rows drew another id within the tolerance", flush=True)
    assert n_other <= 2


# ------------------------------------------------------------------ router-then-exact head

@pytest.mark.parametrize("rows,d,r,V,k_route,k,w_f32", [
    (1, 256, 32, 8200, 32, 8, False), (1, 4096, 512, 20000, 64, 10, False), (3, 128, 16, 5000, 16, 16, True),
    (9, 96, 24, 2056, 12, 5, False), (20, 136, 32, 3080, 40, 7, False),
    (70, 264, 64, 8200, 16, 8, False), (130, 1032, 520, 4104, 13, 13, True),        # the router on the matrix-core path
])
@pytest.mark.parametrize("layout", ["W_d_by_V", "token_major_Wt", "token_major_Wt_and_Bt"])
def test_routed_head(gpu, oracle_mod, rows, d, r, V, k_route, k, w_f32, layout):
    torch, b = gpu
    print(f"routed head rows={rows} d={d} r={r} V={V} k_route={k_route} k={k} f32={w_f32} {layout}", flush=True)
    x = synth.make_inputs(synth.small_config(rows, d, r, V, k, peaked_every=4), seed=400 + rows, with_full_head=True)
    # a full head that agrees with the router on the whole but not in detail (as a trained router would)
    zr = synth.bf16_bits_to_f64(x.A) @ synth.bf16_bits_to_f64(x.B)
    W = synth.f32_to_bf16_bits((zr + 0.3 * synth.bf16_bits_to_f64(x.W)).astype(np.float32))
    Wh = synth.bf16_bits_to_f32(W) if w_f32 else W
    if layout == "W_d_by_V":
        ids, lp = b.routed_head_topk(to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B),
                                     to_dev_f32(Wh) if w_f32 else to_dev_bf16(Wh), k_route, k)
    else:
        Wt = np.ascontiguousarray(Wh.T)                     # transposed on the host: the layout a framework stores
        B = to_dev_bf16(x.B)
        Bt = b.slimspec_transpose_weights(B) if layout.endswith("Bt") else None
        ids, lp = b.routed_head_topk_prepared(to_dev_bf16(x.h), to_dev_bf16(x.A), B,
                                              to_dev_f32(Wt) if w_f32 else to_dev_bf16(Wt), k_route, k, Bt=Bt)
    torch.cuda.synchronize()
    ids, lp = ids.cpu().numpy(), lp.cpu().numpy()
    o_ids, o_lp, o_lse, o_route = oracle_mod.routed_head_topk(x.h, x.A, x.B, Wh, k_route, k)
    # The routed subset itself is a top-k of the router and may differ from the checker's at near-ties of the router's
    # k_route-th place; the comparison below therefore runs over the checker's exact logits of whatever was returned.
    y_at = lambda ri, ci: oracle_mod.full_logits_at(x.h, Wh, ri, ci)
    router = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, k_route, return_logits=True)
    for i in range(rows):
        kth = router.z[i, router.ids[i, -1]]
        assert np.all(router.z[i, ids[i]] >= kth - 1e-3), "an id the router would not have kept"
    compare_with_oracle(ids, lp, o_ids, o_lse, y_at, V)


# ------------------------------------------------------------------ the same heads at the sizes bench.py times

def test_truncated_and_routed_heads_at_the_single_row_workload(gpu, oracle_mod):
    """d = 4096, V = 128256, one row (the latency workload's shape): the truncated head on 65536 and 16384 kept
    columns in an arbitrary order, and the routed head with 64 routed ids, both against the checker."""
    torch, b = gpu
    cfg = synth.CONFIGS["C2"]
    x = synth.make_inputs(cfg, seed=3, with_full_head=True)
    h = to_dev_bf16(x.h)
    for v_tr in (65536, 16384):
        print(f"truncated head at d={cfg.d} V_tr={v_tr}", flush=True)
        id_map = np.random.default_rng(v_tr).permutation(cfg.V)[:v_tr].astype(np.int32)
        W_tr = np.ascontiguousarray(x.W[:, id_map])
        ids, lp = b.truncated_head_topk(h, to_dev_bf16(W_tr), torch.from_numpy(id_map).cuda(), cfg.k)
        torch.cuda.synchronize()
        ora = oracle_mod.truncated_head_topk(x.h, W_tr, id_map, cfg.k)
        col_of = np.full(cfg.V, -1, np.int64)
        col_of[id_map] = np.arange(v_tr)
        ids = ids.cpu().numpy()
        assert (col_of[ids] >= 0).all(), "an id outside the kept subset"
        z_at = lambda ri, ci: oracle_mod.full_logits_at(x.h, W_tr, ri, ci)
        compare_with_oracle(col_of[ids].astype(np.int32), lp.cpu().numpy(), col_of[ora.ids].astype(np.int32), ora.lse, z_at, v_tr)
        del W_tr
    print("routed head at the same shape, k_route = 64", flush=True)
    k_route = 64
    ids, lp = b.routed_head_topk(h, to_dev_bf16(x.A), to_dev_bf16(x.B), to_dev_bf16(x.W), k_route, cfg.k)
    torch.cuda.synchronize()
    ids, lp = ids.cpu().numpy(), lp.cpu().numpy()
    o_ids, o_lp, o_lse, o_route = oracle_mod.routed_head_topk(x.h, x.A, x.B, x.W, k_route, cfg.k)
    router = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, k_route, return_logits=True)
    kth = router.z[0, router.ids[0, -1]]
    assert np.all(router.z[0, ids[0]] >= kth - 1e-3), "an id the router would not have kept"
    y_at = lambda ri, ci: oracle_mod.full_logits_at(x.h, x.W, ri, ci)
    compare_with_oracle(ids, lp, o_ids, o_lse, y_at, cfg.V)
    print("... and from the token-major full head", flush=True)
    ids_t, lp_t = b.routed_head_topk_prepared(h, to_dev_bf16(x.A), to_dev_bf16(x.B), to_dev_bf16(np.ascontiguousarray(x.W.T)), k_route, cfg.k)
    torch.cuda.synchronize()
    compare_with_oracle(ids_t.cpu().numpy(), lp_t.cpu().numpy(), o_ids, o_lse, y_at, cfg.V)
    assert np.array_equal(ids_t.cpu().numpy(), ids)


def test_positions_at_the_512_row_workload(gpu, oracle_mod):
    """512 rows, d = 4096, r = 512, V = 128256 (the throughput workload's shape) as six drafted positions with a
    down-projection each: the checker runs on the first and last row of every position and on every 8th row."""
    torch, b = gpu
    cfg = synth.CONFIGS["C4"]
    x = synth.make_inputs(cfg, seed=2)
    sizes = (86, 86, 85, 85, 85, 85)
    n_pos = len(sizes)
    rng = np.random.default_rng(6)
    stack = np.stack([x.A] + [synth.f32_to_bf16_bits((rng.standard_normal((cfg.d, cfg.r)) * cfg.d ** -0.5).astype(np.float32))
                              for _ in range(n_pos - 1)])
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    print(f"positions at rows={cfg.rows} d={cfg.d} r={cfg.r} V={cfg.V}, sizes {sizes}", flush=True)
    ids, lp = b.slimspec_head_topk_positions(to_dev_bf16(x.h), to_dev_bf16(stack.reshape(n_pos * cfg.d, cfg.r)).view(n_pos, cfg.d, cfg.r),
                                             off.tolist(), to_dev_bf16(x.B), cfg.k)
    torch.cuda.synchronize()
    ids, lp = ids.cpu().numpy(), lp.cpu().numpy()
    for p in range(n_pos):
        sub = sorted(set([int(off[p]), int(off[p + 1]) - 1]) | set(range(int(off[p]) + (-int(off[p])) % 8, int(off[p + 1]), 8)))
        ora = oracle_mod.slimspec_head_topk(np.ascontiguousarray(x.h[sub]), stack[p], x.B, cfg.k, return_logits=True)
        z_at = lambda ri, ci: ora.z[ri, ci]
        compare_with_oracle(ids[sub], lp[sub], ora.ids, ora.lse, z_at, cfg.V)
