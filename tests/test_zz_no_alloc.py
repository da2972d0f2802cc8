"""The entry point for callers that cannot allocate or pass a workspace
(specpv_partial_verify_attn_static: split-KV partial results in the library's own static device
array) against specpv_partial_verify_attn on the same inputs: two calls in a row through the C
ABI, the second with a smaller input, both bit-identical to the workspace call (same kernels),
which the parity tests hold to the oracle; and against the oracle directly."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import ATOL, GpuRun, say

pytestmark = pytest.mark.gpu


def _both(sp, name, seed, M=None):
    case = workloads.to_device(workloads.make_case(name, seed=seed, M=M), "cuda")
    run = GpuRun(sp, case)
    run.summarize(); run.select(); run.attend()
    torch.cuda.synchronize()
    ref_out, ref_lse = run.out.clone(), run.lse.clone()
    out, lse = torch.zeros_like(run.out), torch.zeros_like(run.lse)
    say("static-scratch call:", name, "M =", case["M"])
    sp.specpv_partial_verify_attn_static(run.kv, run.tree, run.sel_idx, run.sel_count, out, lse)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), name
    o = workloads.oracle_views(case, 0)
    O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"],
                                      run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0])
    err = np.abs(out[0].float().cpu().numpy() - O).max()
    say("   max-abs err vs oracle %.3g" % err)
    assert err <= ATOL[case["dtype"]]
    return run


def test_static_scratch_entry_point_matches_the_workspace_call(gpu_lib):
    sp = gpu_lib
    _both(sp, "llama8b_16k", 3)            # bf16, matrix-core kernels, several splits
    _both(sp, "llama8b_16k", 3, M=24)      # a smaller input right after: stale partials of the first call stay unused
    run = _both(sp, "tiny_f32", 2)         # fp32 path
    # every block (sel_idx == NULL)
    ref = torch.zeros_like(run.out)
    sp.specpv_partial_verify_attn(run.kv, run.tree, None, None, ref, None, run.ws)
    out = torch.zeros_like(run.out)
    sp.specpv_partial_verify_attn_static(run.kv, run.tree, None, None, out, None)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_static_scratch_rejects_what_does_not_fit(gpu_lib):
    sp = gpu_lib
    dev = torch.device("cuda")
    # 16 sequences x 40 query heads x 128 nodes: far more partial results than the array holds;
    # rejected on the host before any launch (the tensors are never read)
    batch, Hkv, Hq, D, T, M = 16, 8, 40, 128, 4096, 128
    k = torch.zeros((batch, Hkv, T, D), dtype=torch.bfloat16, device=dev)
    kv = sp.KV(k, k, torch.full((batch,), T, dtype=torch.int32, device=dev), 64)
    q = torch.zeros((batch, M, Hq, D), dtype=torch.bfloat16, device=dev)
    kd = torch.zeros((batch, M, Hkv, D), dtype=torch.bfloat16, device=dev)
    tree = sp.Tree(q, kd, kd, torch.zeros((batch, M), dtype=torch.int32, device=dev))
    assert sp.specpv_workspace_bytes(kv, tree) > sp.STATIC_SCRATCH_BYTES
    with pytest.raises(sp.SpecPVError) as ei:
        sp.specpv_partial_verify_attn_static(kv, tree, None, None, torch.zeros_like(q))
    assert ei.value.status == -3 and "static scratch" in str(ei.value)
