"""The allocation-free entry point (scratch built into the library) against the entry point that takes a caller's
workspace: same kernels, so the outputs must be the same bits; two calls in a row, the second on a smaller input,
share the one scratch array."""
import numpy as np
import pytest

from paper_2605_10453_amd import synth
from parity_util import compare_with_oracle, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("first,second", [((300, 256, 64, 20000, 10), (9, 128, 32, 4104, 10)),     # matrix cores, two row blocks -> one
                                          ((3, 512, 64, 40000, 8), (1, 256, 32, 8192, 8)),          # streaming path
                                          ((64, 256, 128, 9000, 16), (2, 64, 16, 1032, 5))])        # f16 operands -> streaming
def test_static_scratch_entry_matches_workspace_entry(oracle_mod, first, second):
    import torch
    from paper_2605_10453_amd import binding as b
    assert torch.cuda.is_available()
    b.load_library()
    for n, (rows, d, r, V, k) in enumerate((first, second)):
        print(f"static-scratch case call {n}: rows={rows} d={d} r={r} V={V} k={k}", flush=True)
        x = synth.make_inputs(synth.small_config(rows, d, r, V, k, peaked_every=5), seed=31 + n)
        h, A, B = to_dev_bf16(x.h), to_dev_bf16(x.A), to_dev_bf16(x.B)
        ref_ids, ref_lp = b.slimspec_head_topk(h, A, B, k)
        ids = torch.full((rows, k), -7, dtype=torch.int32, device="cuda")
        lp = torch.full((rows, k), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        b.slimspec_head_topk_static(h, A, B, k, out_ids=ids, out_logprobs=lp)
        torch.cuda.synchronize()
        assert torch.equal(ids, ref_ids)
        assert torch.equal(lp.view(torch.int32), ref_lp.view(torch.int32))
        ora = oracle_mod.slimspec_head_topk(x.h, x.A, x.B, k)
        z_at = lambda ri, ci: oracle_mod.slimspec_logits_at(x.h, x.A, x.B, ri, ci)
        compare_with_oracle(ids.cpu().numpy(), lp.cpu().numpy(), ora.ids, ora.lse, z_at, V)


def test_static_scratch_entry_refuses_what_does_not_fit():
    import torch
    from paper_2605_10453_amd import binding as b
    rows, d, r, V, k = 4096, 8192, 4096, 65536, 10
    assert b.slimspec_workspace_bytes(rows, d, r, V, k) > b.STATIC_SCRATCH_BYTES
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    shape = b.SlimspecShape(rows, d, r, V)
    import ctypes
    p = dummy.data_ptr()
    st = b.load_library().slimspec_head_topk_static(p, p, p, ctypes.byref(shape), k, p, p, None)
    assert st == b.STATUS_SCRATCH_LIMIT                 # refused on the host: nothing was enqueued
    assert "scratch" in b.status_string(st)
