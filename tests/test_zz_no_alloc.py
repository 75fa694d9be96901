"""hpct_plan_launch_noalloc, the entry point for callers that cannot allocate: called through the C ABI and
compared with hpct_plan_launch (caller's workspace) and with the CPU checker, on two calls in a row, the second
with a smaller input.  Collected last (file name), so a failure here hides no other test."""
import ctypes as C

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import compare, ref  # noqa: E402
from paper_2506_10401_amd import datagen, hpct  # noqa: E402


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def raw_launch(entry, plan, ins, outs, workspace=None):
    """one call of `entry` (a ctypes function of the library) with plain pointer arrays"""
    vp = C.c_void_p
    a = (vp * len(ins))(*[t.data_ptr() for t in ins])
    o = (vp * len(outs))(*[t.data_ptr() for t in outs])
    s = vp(torch.cuda.current_stream().cuda_stream)
    if workspace is None:
        st = entry(plan._h, a, o, s)
    else:
        st = entry(plan._h, a, o, vp(workspace.data_ptr()), workspace.numel() * 4, s)
    assert st == hpct.HPCT_OK, hpct.hpct_last_error()


def test_noalloc_refuses_a_workspace_beyond_the_scratch():
    # host-side decision, taken before any HIP call: a split-K GEMM whose partial products need 16 MB
    lib = hpct.load()
    d = hpct.op_desc(hpct.HPCT_ANCHOR_GEMM, [], hpct.HPCT_RED_NONE, 0, [(1024, 4096), (4096, 1024)], [(1024, 1024)])
    p = hpct.Plan(d)
    assert p.workspace_bytes > hpct.NOALLOC_SCRATCH_BYTES
    vp = C.c_void_p
    one = (vp * 1)(vp(16))
    two = (vp * 2)(vp(16), vp(32))
    st = lib.hpct_plan_launch_noalloc(p._h, two, one, None)
    assert st == hpct.HPCT_ERR_WORKSPACE and "scratch" in hpct.hpct_last_error()
    assert lib.hpct_plan_launch_noalloc(None, two, one, None) == hpct.HPCT_ERR_NULL


@pytest.mark.gpu
def test_noalloc_matches_the_workspace_launch_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    lib = hpct.load()
    # first call: the dropout chain (GEMM + dropout + row means + softmax over the means) with 64 KB of partial row
    # sums; second call: a smaller one (9.6 KB), which finds the first call's contents in the shared array
    for M, K, N in ((1024, 96, 2048), (300, 40, 1000)):
        print("noalloc chain6 M=%d K=%d N=%d" % (M, K, N), flush=True)
        t = datagen.make(6, M=M, K=K, N=N)
        X, W, b = dev(t["X"]), dev(t["W"]), dev(t["bias"])
        want_out = torch.full((M,), float("nan"), device="cuda")
        got_out = torch.full((M,), float("nan"), device="cuda")
        plan, ins = hpct.matmul_dropout_mean_softmax_plan(X, W, b, want_out, datagen.CHAIN6_P, datagen.CHAIN6_SEED)
        assert 0 < plan.workspace_bytes <= hpct.NOALLOC_SCRATCH_BYTES
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
        raw_launch(lib.hpct_plan_launch, plan, ins, [want_out], ws)
        raw_launch(lib.hpct_plan_launch_noalloc, plan, ins, [got_out])
        want, got = host(want_out), host(got_out)
        assert np.array_equal(want, got)                       # same kernels, same order: bit for bit
        Z = ref.gemm_bias(t["X"], t["W"], t["bias"])
        mu = ref.mean_rows(ref.dropout_hash(Z, datagen.CHAIN6_P, datagen.CHAIN6_SEED))
        assert compare.pointwise(got, ref.softmax_rows(mu.reshape(1, -1)).reshape(-1))
    # split-K GEMMs (partial products of the K slices in the scratch) after the calls above: one that needs the
    # whole array, then a smaller one
    for M, K, N in ((256, 4096, 512), (256, 2048, 256)):
        print("noalloc split-K gemm M=%d K=%d N=%d" % (M, K, N), flush=True)
        t = datagen.make(1, M=M, K=K, N=N)
        X, W, b = dev(t["X"]), dev(t["W"]), dev(t["bias"])
        want_out = torch.full((M, N), float("nan"), device="cuda")
        got_out = torch.full((M, N), float("nan"), device="cuda")
        plan, ins = hpct.gemm_bias_relu_softmax_plan(X, W, b, want_out, relu=True, softmax=False)
        print("kernel", plan.kernel_name, "workspace", plan.workspace_bytes, flush=True)
        assert 0 < plan.workspace_bytes <= hpct.NOALLOC_SCRATCH_BYTES
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
        raw_launch(lib.hpct_plan_launch, plan, ins, [want_out], ws)
        raw_launch(lib.hpct_plan_launch_noalloc, plan, ins, [got_out])
        want, got = host(want_out), host(got_out)
        assert np.array_equal(want, got)
        Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
        assert compare.contraction(got, ref.relu(Z), Dn)
    # a plan without a workspace goes through unchanged
    t = datagen.make(3, M=8, N=4096)
    out = torch.full((8, 4096), float("nan"), device="cuda")
    Xd, g, be = dev(t["X"]), dev(t["gamma"]), dev(t["beta"])
    plan, ins = hpct.layernorm_gelu_plan(Xd, g, be, out)
    assert plan.workspace_bytes == 0
    raw_launch(lib.hpct_plan_launch_noalloc, plan, ins, [out])
    assert compare.pointwise(host(out), ref.chain3(t["X"], t["gamma"], t["beta"]))
