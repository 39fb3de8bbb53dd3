"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 checker on the
same seeded inputs.  Bar: ids identical except where the checker's logits are within 1e-3;
log-probabilities within 2e-2 absolute."""
import math

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


def run_low_rank(gpu, x, k):
    torch, b = gpu
    ids, lp = b.slimspec_head_topk(to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B), k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), lp.cpu().numpy()


def run_full(gpu, h_bits, W, k):
    torch, b = gpu
    Wd = to_dev_f32(W) if W.dtype == np.float32 else to_dev_bf16(W)
    ids, lp = b.full_head_topk(to_dev_bf16(h_bits), Wd, k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), lp.cpu().numpy()


def check_low_rank(gpu, oracle_mod, x, k, exact_rows=()):
    print(f"low-rank case rows={x.cfg.rows} d={x.cfg.d} r={x.cfg.r} V={x.cfg.V} k={k} seed={x.seed}", flush=True)
    g_ids, g_lp = run_low_rank(gpu, x, k)
    ora = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, k)
    z_at = lambda ri, ci: oracle_mod.slimspec_logits_at(x.h, x.A, x.B, ri, ci)
    n_exempt, err = compare_with_oracle(g_ids, g_lp, ora.ids, ora.lse, z_at, x.cfg.V)
    for i in exact_rows:
        assert np.array_equal(g_ids[i], ora.ids[i]), (i, g_ids[i], ora.ids[i])
    return g_ids, g_lp, ora, n_exempt


def check_full(gpu, oracle_mod, h, W, k, rows_subset=None):
    print(f"full-head case rows={h.shape[0]} d={h.shape[1]} V={W.shape[1]} k={k} W={W.dtype}", flush=True)
    g_ids, g_lp = run_full(gpu, h, W, k)
    if rows_subset is not None:
        hs = np.ascontiguousarray(h[rows_subset])
        g_ids, g_lp = g_ids[rows_subset], g_lp[rows_subset]
    else:
        hs = h
    ora = oracle_mod.full_head_topk(hs, W, k)
    z_at = lambda ri, ci: oracle_mod.full_logits_at(hs, W, ri, ci)
    compare_with_oracle(g_ids, g_lp, ora.ids, ora.lse, z_at, W.shape[1])
    return g_ids, g_lp, ora


# ------------------------------------------------------------------ seeded sweep of small random shapes

def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        rows = int(rng.choice([1, 2, 3, 4, 5, 6, 9, 17, 33, 70, 129, 200]))
        d = 8 * int(rng.integers(1, 65))
        r = 8 * int(rng.integers(1, 17))
        V = 8 * int(rng.integers(1, 1200))
        k = int(min(V, rng.choice([1, 2, 5, 10, 16, 17, 40, 64])))
        out.append((rows, d, r, V, k))
    return out


@pytest.mark.parametrize("rows,d,r,V,k", _random_shapes(24, 2024))
def test_random_small_shapes_both_heads(gpu, oracle_mod, rows, d, r, V, k):
    """Every dispatch branch on shapes nobody picked by hand: few / many rows, k on both sides of the matrix-core
    limit, contraction lengths and vocabularies that are not multiples of any tile."""
    cfg = synth.small_config(rows=rows, d=d, r=r, V=V, k=k, peaked_every=3)
    x = synth.make_inputs(cfg, 1000 + rows + V, with_full_head=True)
    check_low_rank(gpu, oracle_mod, x, k)
    check_full(gpu, oracle_mod, x.h, x.W, k)


# ------------------------------------------------------------------ small shapes, several tiles + ragged tails

SMALL = [
    # rows, d,   r,   V,     k
    (1, 256, 32, 8192, 8),          # config 1
    (1, 40, 24, 520, 5),            # one full chunk + 8 columns; d, r not multiples of 32
    (1, 64, 8, 8, 8),               # k == V, a single lane of a single chunk
    (1, 64, 16, 72, 64),            # k = KMAX with fewer valid columns per lane group than k
    (2, 128, 16, 5000, 1),          # k = 1 is the argmax
    (3, 200, 40, 3072, 16),
    (4, 512, 64, 10248, 10),
    (7, 264, 72, 1544, 33),
    (8, 1024, 128, 20000, 10),
    (9, 96, 24, 2056, 7),           # one row more than a row group
    (17, 128, 32, 4104, 12),        # three row groups
    (40, 256, 32, 1032, 3),
    (130, 64, 40, 2056, 5),         # two 128-row halves of a 256-row block, contraction tail, column tail
    (300, 128, 64, 5000, 10),       # two 256-row blocks, the second mostly padding
    (20, 64, 8, 1032, 4),           # a single, partial stage of the contraction
    (12, 64, 24, 2056, 16),         # the largest k of the matrix-core path
    (5, 128, 32, 4104, 10),         # the smallest row count of the matrix-core path
    (1, 64, 16, 140000, 10),        # one row, more than 256 chunks: narrower chunks, 8-wavefront blocks
    (1, 64, 16, 300000, 10),        # ... more than 512: 4-wavefront blocks
    (1, 64, 8, 600008, 5),          # ... more than 1024: full-width chunks in several rounds
    (2, 64, 16, 140000, 10),        # two rows keep 512-column chunks
]


def test_more_rows_than_one_launch(gpu, oracle_mod):
    """More rows than one launch of the matrix-core kernels takes (512): the call loops over launches; the last has 4 rows."""
    x = synth.make_inputs(synth.small_config(4100, 64, 32, 1032, 5, peaked_every=7), seed=4100)
    check_low_rank(gpu, oracle_mod, x, 5)



@pytest.mark.parametrize("rows,d,r,V,k", SMALL)
def test_low_rank_small(gpu, oracle_mod, rows, d, r, V, k):
    x = synth.make_inputs(synth.small_config(rows, d, r, V, k, peaked_every=5), seed=rows * 1000 + k)
    check_low_rank(gpu, oracle_mod, x, k)


@pytest.mark.parametrize("rows,d,r,V,k", SMALL[:8] + SMALL[-4:-2])
@pytest.mark.parametrize("w_f32", [False, True])
def test_full_head_small(gpu, oracle_mod, rows, d, r, V, k, w_f32):
    x = synth.make_inputs(synth.small_config(rows, d, r, V, k), seed=77 + rows, with_full_head=True)
    W = synth.bf16_bits_to_f32(x.W) if w_f32 else x.W
    check_full(gpu, oracle_mod, x.h, W, k)


@pytest.mark.parametrize("rows,d,r,V,k", SMALL[9:13])
def test_full_head_small_many_rows(gpu, oracle_mod, rows, d, r, V, k):
    """More than 8 rows and bf16 weights: the full head runs on the matrix cores."""
    x = synth.make_inputs(synth.small_config(rows, d, r, V, k, peaked_every=4), seed=177 + rows, with_full_head=True)
    check_full(gpu, oracle_mod, x.h, x.W, k)


@pytest.mark.parametrize("n_tied", [2, 40, 600, 2400])
def test_full_head_long_contraction_exact_reevaluation(gpu, oracle_mod, n_tied):
    """Full head with d >= 2048 and many rows: rows that need exact re-evaluations are parked by the merge and
    finished by two more launches.  Exactly tied top columns force the re-evaluation for row 0 (2 and 40 tied
    columns and the about 400 that 600 leave outside the duplicated block fit a parked row's list; 2400 leave
    about 1600, more than a parked row holds, and are evaluated in place); a duplicated block of columns makes
    every other row tie at some ranks too."""
    cfg = synth.small_config(rows=12, d=2048, r=8, V=4104, k=8)
    x = synth.make_inputs(cfg, 5, with_full_head=True)
    V = cfg.V
    x.W[:, 2048:2048 + 1024] = x.W[:, :1024]                    # every row: its best column below 1024 has a twin
    h0 = synth.bf16_bits_to_f64(x.h[0])
    cols = sorted(set(int(c) for c in np.linspace(1030, V - 1, n_tied).astype(np.int64)) - set(range(2048, 3072)))
    synth.plant_identical_columns(x.W, 0.35 * h0 / math.sqrt(cfg.d), cols)
    g_ids, g_lp, ora = check_full(gpu, oracle_mod, x.h, x.W, cfg.k)
    n_top = min(len(cols), cfg.k)
    assert g_ids[0, :n_top].tolist() == cols[:n_top]
    assert np.array_equal(g_ids, ora.ids)                       # exact values, ties by id: nothing left to the tolerance


@pytest.mark.parametrize("rows,k", [(20, 17), (140, 40)])
def test_many_rows_large_k(gpu, oracle_mod, rows, k):
    """k above the matrix-core path's limit: the call takes the streaming path in row groups."""
    x = synth.make_inputs(synth.small_config(rows, 128, 32, 3080, k, peaked_every=3), seed=900 + rows)
    check_low_rank(gpu, oracle_mod, x, k)


def test_zero_rows_inside_a_many_row_batch(gpu, oracle_mod):
    """Padded batch slots (all-zero hidden states) among ordinary rows on the matrix-core path."""
    x = synth.make_inputs(synth.small_config(33, 128, 32, 3080, 6), seed=4242)
    x.h[5] = 0
    x.h[32] = 0
    check_low_rank(gpu, oracle_mod, x, 6)


def test_config1_both_heads_agree(gpu, oracle_mod):
    """Config 1: the full-head comparator uses W = A B materialised in fp32."""
    cfg = synth.CONFIGS["C1"]
    x = synth.make_inputs(cfg, 0)
    g_ids, g_lp, ora, _ = check_low_rank(gpu, oracle_mod, x, cfg.k)
    W = (synth.bf16_bits_to_f64(x.A) @ synth.bf16_bits_to_f64(x.B)).astype(np.float32)
    f_ids, f_lp, _ = check_full(gpu, oracle_mod, x.h, W, cfg.k)
    assert np.array_equal(f_ids, g_ids)
    assert np.allclose(f_lp, g_lp, atol=1e-3)


# ------------------------------------------------------------------ degenerate cases

def test_zero_hidden_state_all_tied(gpu, oracle_mod):
    """h = 0: every logit is exactly 0, so ids must be 0..k-1 and every logprob -ln V."""
    cfg = synth.small_config(rows=3, d=64, r=16, V=4104, k=9)
    x = synth.make_inputs(cfg, 1)
    x.h[:] = 0
    g_ids, g_lp = run_low_rank(gpu, x, cfg.k)
    assert g_ids.tolist() == [list(range(cfg.k))] * 3
    assert np.allclose(g_lp, -math.log(cfg.V), atol=1e-4)


@pytest.mark.parametrize("rows", [1, 6])
def test_planted_exact_ties(gpu, oracle_mod, rows):
    cfg = synth.small_config(rows=rows, d=256, r=64, V=6152, k=5)
    x = synth.make_inputs(cfg, 21)
    V = cfg.V
    t = oracle_mod.down_projection(x.h, x.A)
    synth.plant_identical_columns(x.B, 0.35 * t[0] / math.sqrt(cfg.r) * 2, [0, V // 2, V - 1])
    g_ids, g_lp, ora, _ = check_low_rank(gpu, oracle_mod, x, cfg.k, exact_rows=[0])
    assert g_ids[0, :3].tolist() == [0, V // 2, V - 1]
    assert g_lp[0, 0] == g_lp[0, 1] == g_lp[0, 2]
    for k in (1, 2, 3):
        ids, _ = run_low_rank(gpu, x, k)
        assert ids[0].tolist() == [0, V // 2, V - 1][:k]


@pytest.mark.parametrize("k", [16, 10])
def test_rising_logits_through_the_exhaustive_pass(gpu, oracle_mod, k):
    """Logits that rise strictly with the column id over the whole vocabulary.  With k = 16 the matrix cores take an
    f16 contraction input, which overflows for rows 0-2 here, so the merge answers with its exhaustive exact pass;
    there every scanned column beats the running k-th key, which fills the pass's key buffer to its bound."""
    rows, d, r, V = 6, 8, 8, 16384
    one = synth.f32_to_bf16_bits(np.float32(1.0))
    h = np.zeros((rows, d), np.float32)
    h[:, 0] = [65536.0, -65536.0, 98304.0, 0.0, 1.0, 65536.0]
    A = np.zeros((d, r), np.float32)
    A[0, 0], A[0, 1] = 1.0, 2.0 ** -8
    v = np.arange(V)
    B = np.zeros((r, V), np.float32)
    B[0] = 1.0 + (v >> 7) / 128.0
    B[1] = 1.0 + (v & 127) / 128.0
    x = synth.HeadInputs(cfg=synth.small_config(rows, d, r, V, k), seed=0, h=synth.f32_to_bf16_bits(h),
                         A=synth.f32_to_bf16_bits(A), B=synth.f32_to_bf16_bits(B))
    assert one == 0x3F80 and np.array_equal(synth.bf16_bits_to_f32(x.B), B)         # every value is exact in bf16
    g_ids, _, ora, _ = check_low_rank(gpu, oracle_mod, x, k)
    assert np.array_equal(g_ids, ora.ids)
    assert g_ids[0].tolist() == list(range(V - 1, V - 1 - k, -1))
    assert g_ids[1].tolist() == list(range(k))


@pytest.mark.parametrize("rows,d,r,V,k", [(1, 512, 64, 20000, 10), (3, 256, 32, 9000, 7), (5, 512, 64, 20000, 10),
                                          (512, 256, 64, 20000, 10), (40, 128, 32, 6000, 16)])
def test_run_to_run_determinism(gpu, rows, d, r, V, k):
    """Same inputs, same bits out: the streaming path, the matrix-core path with both operand modes and two row blocks."""
    cfg = synth.small_config(rows=rows, d=d, r=r, V=V, k=k, peaked_every=7)
    x = synth.make_inputs(cfg, 3)
    a = run_low_rank(gpu, x, cfg.k)
    for _ in range(2):
        b = run_low_rank(gpu, x, cfg.k)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


def test_run_to_run_determinism_full_head_parked_rows(gpu):
    """Full head with a long contraction: rows that need exact re-evaluations are parked and finished by later launches."""
    cfg = synth.small_config(rows=12, d=2048, r=8, V=4104, k=8)
    x = synth.make_inputs(cfg, 5, with_full_head=True)
    x.W[:, 2048:2048 + 1024] = x.W[:, :1024]
    a = run_full(gpu, x.h, x.W, cfg.k)
    for _ in range(2):
        b = run_full(gpu, x.h, x.W, cfg.k)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


def test_side_stream_and_caller_buffers(gpu, oracle_mod):
    torch, b = gpu
    cfg = synth.small_config(rows=2, d=256, r=32, V=9000, k=6)
    x = synth.make_inputs(cfg, 4)
    h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
    need = b.slimspec_workspace_bytes(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k)
    ws = torch.full((need,), 0xAB, dtype=torch.uint8, device="cuda")      # poisoned scratch
    ids = torch.full((cfg.rows, cfg.k), -7, dtype=torch.int32, device="cuda")
    lp = torch.full((cfg.rows, cfg.k), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    b.slimspec_head_topk(h, A, B, cfg.k, out_ids=ids, out_logprobs=lp, workspace=ws, stream=s)
    s.synchronize()
    ora = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, cfg.k)
    z_at = lambda ri, ci: oracle_mod.slimspec_logits_at(x.h, x.A, x.B, ri, ci)
    compare_with_oracle(ids.cpu().numpy(), lp.cpu().numpy(), ora.ids, ora.lse, z_at, cfg.V)
    # too small a workspace is refused and nothing is written
    ids.fill_(-7)
    with pytest.raises(b.SlimspecError) as e:
        b.slimspec_head_topk(h, A, B, cfg.k, out_ids=ids, out_logprobs=lp, workspace=ws[:1024])
    assert e.value.status == b.STATUS_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert int((ids == -7).sum()) == ids.numel()


def test_two_host_threads_on_two_streams(gpu):
    """Calls from two host threads, each on a stream and a workspace of its own, overlap freely (the library keeps no
    state but per thread); every result equals the one the same call gives alone."""
    import threading
    torch, b = gpu
    jobs = []
    for rows, seed in ((1, 11), (40, 12)):                      # the streaming path and the matrix-core path
        cfg = synth.small_config(rows=rows, d=512, r=64, V=30000, k=10, peaked_every=7)
        x = synth.make_inputs(cfg, seed)
        h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
        ref_ids, ref_lp = b.slimspec_head_topk(h, A, B, cfg.k)
        torch.cuda.synchronize()
        jobs.append((cfg, h, A, B, ref_ids.clone(), ref_lp.clone()))
    errors = []

    def worker(job):
        cfg, h, A, B, ref_ids, ref_lp = job
        try:
            s = torch.cuda.Stream()
            ws = torch.empty(b.slimspec_workspace_bytes(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k), dtype=torch.uint8, device="cuda")
            ids = torch.empty((cfg.rows, cfg.k), dtype=torch.int32, device="cuda")
            lp = torch.empty((cfg.rows, cfg.k), dtype=torch.float32, device="cuda")
            for it in range(60):
                ids.fill_(-1)
                b.slimspec_head_topk(h, A, B, cfg.k, out_ids=ids, out_logprobs=lp, workspace=ws, stream=s)
                s.synchronize()
                if not (torch.equal(ids, ref_ids) and torch.equal(lp.view(torch.int32), ref_lp.view(torch.int32))):
                    errors.append((cfg.rows, it))
                    return
        except Exception as exc:                                # reported by the main thread
            errors.append((cfg.rows, repr(exc)))

    threads = [threading.Thread(target=worker, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_graph_replays_of_the_matrix_core_path(gpu):
    """Two calls of the many-row path captured in one HIP graph (no allocation, no synchronisation, no memset inside
    the library): every replay, with other work of the process between them, gives the eager results."""
    torch, b = gpu
    cfg = synth.small_config(rows=48, d=512, r=128, V=30000, k=10, peaked_every=5)
    xs = [synth.make_inputs(cfg, seed) for seed in (21, 22)]
    dev = [(to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)) for x in xs]
    outs = [(torch.empty((cfg.rows, cfg.k), dtype=torch.int32, device="cuda"),
             torch.empty((cfg.rows, cfg.k), dtype=torch.float32, device="cuda")) for _ in xs]
    ws = torch.empty(b.slimspec_workspace_bytes(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k), dtype=torch.uint8, device="cuda")
    eager = []
    for (h, A, B), (ids, lp) in zip(dev, outs):
        b.slimspec_head_topk(h, A, B, cfg.k, out_ids=ids, out_logprobs=lp, workspace=ws)
        torch.cuda.synchronize()
        eager.append((ids.clone(), lp.clone()))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for (h, A, B), (ids, lp) in zip(dev, outs):
                b.slimspec_head_topk(h, A, B, cfg.k, out_ids=ids, out_logprobs=lp, workspace=ws)
    for rep in range(4):
        for ids, lp in outs:
            ids.fill_(-1)
            lp.fill_(0.0)
        junk = torch.randn(1 << 20, device="cuda").sum()           # the process's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (ids, lp), (e_ids, e_lp) in zip(outs, eager):
            assert torch.equal(ids, e_ids), rep
            assert torch.equal(lp.view(torch.int32), e_lp.view(torch.int32)), rep
        del junk


# ------------------------------------------------------------------ weights that are not i.i.d. Gaussian

def _non_gaussian_B(kind, cfg, seed):
    """B for the matrix-core path's error model (the rounding of t to 16 bits is bounded per vocabulary tile from a
    sample of B): a few columns much larger than the rest, heavy tails, and a periodic pattern over the rows."""
    x = synth.make_inputs(cfg, seed)
    rng = np.random.default_rng(seed + 99)
    B = synth.bf16_bits_to_f32(x.B)
    if kind == "scaled_columns":
        cols = rng.choice(cfg.V, 40, replace=False)
        B[:, cols[:30]] *= np.float32(8.0)                      # exact in bf16
        B[:, cols[30:]] *= np.float32(32.0)
    elif kind == "heavy_tailed":
        B = (rng.standard_t(3, size=B.shape) * (cfg.r ** -0.5) / math.sqrt(3.0)).astype(np.float32)
    elif kind == "small_every_8th_row":
        B[::8] *= np.float32(2.0 ** -4)
    elif kind == "large_every_8th_row_offset_3":
        B[3::8] *= np.float32(16.0)
    else:
        raise ValueError(kind)
    x.B = synth.f32_to_bf16_bits(B)
    return x


@pytest.mark.parametrize("k", [10, 16])
@pytest.mark.parametrize("kind", ["scaled_columns", "heavy_tailed", "small_every_8th_row", "large_every_8th_row_offset_3"])
def test_matrix_core_path_weights_not_gaussian(gpu, oracle_mod, kind, k):
    cfg = synth.small_config(rows=96, d=256, r=512, V=20008, k=k, peaked_every=6)
    x = _non_gaussian_B(kind, cfg, seed=500 + k)
    _, _, _, n_exempt = check_low_rank(gpu, oracle_mod, x, k)
    print(f"{kind} k={k}: {n_exempt} positions used the tie exemption", flush=True)


def test_wide_rounding_bound_with_few_winners(gpu, oracle_mod):
    """Peaked rows (hidden states x 4) over a B whose every 8th row is 6 times larger, k = 2: the rounding errors of
    the few coordinates that carry the logits then share a sign by chance in some rows, the computed logits of the
    row's probable tokens are all off the same way, and the log-sum-exp follows them unless those tokens, winners or
    not, are re-evaluated too (row 33 of this draw: 3.7e-2 before any correction, 2.2e-2 with the two winners exact)."""
    cfg = synth.small_config(rows=64, d=648, r=192, V=6968, k=2, peaked_every=3)
    x = synth.make_inputs(cfg, seed=406289933)
    B = synth.bf16_bits_to_f32(x.B)
    B[1::8] *= np.float32(6.0)
    x.B = synth.f32_to_bf16_bits(B)
    check_low_rank(gpu, oracle_mod, x, cfg.k)


def test_two_probable_tokens_in_one_group_of_sixteen(gpu, oracle_mod):
    """The row's two most probable tokens sit in the same group of 16 logits of one lane (columns b + 1 and b + 18 of a
    32-column tile), so only the larger one is listed with its computed value; the other one carries 40 % of the
    probability and, by construction, a large rounding error (a component orthogonal to t).  The merge has to replace
    its term of the sum of exponentials too, for which it recomputes the logit the head kernel saw."""
    cfg = synth.small_config(rows=24, d=256, r=96, V=2048, k=4, peaked_every=0)
    x = synth.make_inputs(cfg, seed=91)
    x.h = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(x.h) * np.float32(16.0))
    t = synth.bf16_bits_to_f64(x.h) @ synth.bf16_bits_to_f64(x.A)
    B = synth.bf16_bits_to_f32(x.B)
    rng = np.random.default_rng(5)
    for i in range(cfg.rows):
        ti = t[i]
        base = 64 * i
        u = rng.standard_normal(cfg.r)
        u -= (u @ ti) / (ti @ ti) * ti
        u *= 2.0 / np.linalg.norm(u)
        B[:, base + 1] = (90.0 * ti / (ti @ ti)).astype(np.float32)
        B[:, base + 18] = (89.6 * ti / (ti @ ti) + u).astype(np.float32)
    x.B = synth.f32_to_bf16_bits(B)
    check_low_rank(gpu, oracle_mod, x, cfg.k)


def test_logit_far_above_the_running_maximum(gpu, oracle_mod):
    """One column per row, late in the vocabulary (in a tile that is not the first one its block works on), whose logit is 126 to 130 binary orders above everything the row has
    seen until then (natural logits 88 ... 92 over a background of 2 ... 5): the running sum of exponentials has to be
    rescaled by a factor at the very bottom of the float range, or, just beyond it, the row has to be redone exactly."""
    cfg = synth.small_config(rows=512, d=256, r=144, V=36784, k=5, peaked_every=0)
    x = synth.make_inputs(cfg, seed=77)
    t = synth.bf16_bits_to_f64(x.h) @ synth.bf16_bits_to_f64(x.A)
    B = synth.bf16_bits_to_f32(x.B)
    for i in range(0, 512, 16):
        alpha = 88.0 + 0.125 * (i // 16)
        B[:, 32768 + 7 * i] = (alpha * t[i] / (t[i] @ t[i])).astype(np.float32)
    # ... and, in other rows, 170 to 440 binary orders above: the exponential overflows, the stream's sum becomes
    # infinite and then, rescaled by zero, not a number; such a row must end in the exact pass, not lose the stream
    for i in range(8, 512, 16):
        alpha = 120.0 + 6.0 * (i // 16)
        B[:, 32768 + 7 * i] = (alpha * t[i] / (t[i] @ t[i])).astype(np.float32)
    x.B = synth.f32_to_bf16_bits(B)
    check_low_rank(gpu, oracle_mod, x, cfg.k)


@pytest.mark.parametrize("rows,V", [(300, 40960), (200, 70000), (20, 70000)])
def test_four_best_logits_in_one_lane_stream(gpu, oracle_mod, rows, V):
    """The matrix-core kernel lists three groups of 16 logits per lane stream (a row's share of four of a vocabulary
    tile's eight 32-column MFMA tiles in one half-wavefront, over the tiles of a column block).  Here a row's four
    largest logits sit in four different groups of one lane stream (columns 256 vt + 32 j + 4, j = 4 ... 7), so one of
    them is dropped from the list and the merge has to rescan every column of the record that stream went into.  The
    three shapes leave four, two and one record per row and column block (few, more, many column blocks)."""
    cfg = synth.small_config(rows=rows, d=64, r=64, V=V, k=5, peaked_every=0)
    x = synth.make_inputs(cfg, seed=rows + V)
    t = synth.bf16_bits_to_f64(x.h) @ synth.bf16_bits_to_f64(x.A)
    B = synth.bf16_bits_to_f32(x.B)
    planted = {}
    for n, i in enumerate((0, 7, rows - 1)):
        vt = 1 + 2 * n
        cols = [256 * vt + 32 * j + 4 for j in (4, 5, 6, 7)]
        for c, alpha in zip(cols, (12.0, 11.5, 11.0, 10.5)):
            B[:, c] = (alpha * t[i] / (t[i] @ t[i])).astype(np.float32)
        planted[i] = cols
    x.B = synth.f32_to_bf16_bits(B)
    g_ids, _, ora, _ = check_low_rank(gpu, oracle_mod, x, cfg.k, exact_rows=list(planted))
    for i, cols in planted.items():
        assert g_ids[i, :4].tolist() == cols, (i, g_ids[i], cols)


# ------------------------------------------------------------------ the five workloads at full size

@pytest.mark.parametrize("seed", list(range(10)))
def test_config2_low_rank(gpu, oracle_mod, seed):
    cfg = synth.CONFIGS["C2"]
    check_low_rank(gpu, oracle_mod, synth.make_inputs(cfg, seed), cfg.k)


def test_config2_full_head(gpu, oracle_mod):
    cfg = synth.CONFIGS["C2"]
    x = synth.make_inputs(cfg, 0, with_full_head=True)
    check_full(gpu, oracle_mod, x.h, x.W, cfg.k)


def test_config3_both_heads(gpu, oracle_mod):
    cfg = synth.CONFIGS["C3"]
    x = synth.make_inputs(cfg, 0, with_full_head=True)
    check_low_rank(gpu, oracle_mod, x, cfg.k)
    check_full(gpu, oracle_mod, x.h, x.W, cfg.k)


@pytest.mark.parametrize("name", ["C4", "C4_r256", "C4_r1024"])
def test_config4_low_rank(gpu, oracle_mod, name):
    cfg = synth.CONFIGS[name]
    _, _, _, n_exempt = check_low_rank(gpu, oracle_mod, synth.make_inputs(cfg, 0), cfg.k)
    print(f"{name}: {n_exempt} positions used the tie exemption", flush=True)


def test_config4_full_head_row_subset(gpu, oracle_mod):
    """The full-head checker costs 0.5 G fp64 MACs per row: all 512 rows run on the GPU,
    a fixed subset (first 16 rows and every peaked row) is checked."""
    cfg = synth.CONFIGS["C4"]
    x = synth.make_inputs(cfg, 0, with_full_head=True)
    subset = sorted(set(range(16)) | set(range(0, cfg.rows, cfg.peaked_every)))
    check_full(gpu, oracle_mod, x.h, x.W, cfg.k, rows_subset=np.array(subset))


def test_config5_with_planted_ties(gpu, oracle_mod):
    cfg = synth.CONFIGS["C5"]
    x = synth.make_inputs(cfg, 0, with_full_head=True)
    V = cfg.V
    t = oracle_mod.down_projection(x.h[:1], x.A)
    synth.plant_identical_columns(x.B, 0.35 * t[0] / math.sqrt(cfg.r), [0, V // 2, V - 1])
    g_ids, g_lp, ora, _ = check_low_rank(gpu, oracle_mod, x, cfg.k, exact_rows=[0])
    assert g_ids[0, :3].tolist() == [0, V // 2, V - 1]
    assert g_lp[0, 0] == g_lp[0, 1] == g_lp[0, 2]
    # full head of the same workload, ties planted through h[0] itself
    h0 = synth.bf16_bits_to_f64(x.h[0])
    synth.plant_identical_columns(x.W, 0.35 * h0 / math.sqrt(cfg.d), [0, V // 2, V - 1])
    subset = np.arange(0, cfg.rows, 8)
    f_ids, f_lp, _ = check_full(gpu, oracle_mod, x.h, x.W, cfg.k, rows_subset=subset)
    assert f_ids[0, :3].tolist() == [0, V // 2, V - 1]
