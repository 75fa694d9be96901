"""Parity of the HIP kernels (called through the C ABI) with the CPU checker,
element by element on the same seeded inputs.

Acceptance rules (oracle/compare.py): elementwise / reduction outputs within
1e-4 relative, floored at 1e-2 of the output's rms; fp32 contraction outputs
within 2e-3 of sum |a||b|.  Shapes span several tiles and ragged tails, plus
the five full-size workloads in the launch configuration the benchmark times.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import compare, ref  # noqa: E402
from paper_2506_10401_amd import datagen, hpct  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    hpct.load()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def show(tag, v):
    print("%s: %r" % (tag, v), flush=True)
    return v


# ------------------------------------------------------------------- chain 1
def run_chain1(t, relu=True, softmax=True, bias=True):
    X, W = dev(t["X"]), dev(t["W"])
    b = dev(t["bias"]) if bias else None
    out = torch.full((X.shape[0], W.shape[1]), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(X, W, b, out, relu=relu, softmax=softmax)
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda") if plan.workspace_bytes else None
    plan.launch(ins, [out], workspace=ws)
    return host(out)


def test_chain1_full_size():
    t = datagen.make(1)
    got = run_chain1(t)
    assert show("chain1 64x256x256 softmax", compare.pointwise(got, ref.chain1(t["X"], t["W"], t["bias"])))
    # the anchor alone under the contraction rule
    got = run_chain1(t, relu=False, softmax=False)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    assert show("chain1 anchor", compare.contraction(got, Z, Dn))
    # and tighter: true fp32 accumulation is far inside the bound
    assert np.max(np.abs(got - Z) / Dn) < 1e-5


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (17, 5, 10), (70, 100, 63), (16, 256, 200), (33, 36, 256),
                                   (5, 33, 64), (40, 64, 128), (3, 300, 129)])
def test_chain1_ragged_shapes(M, K, N):
    print("chain1 M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    assert show("softmax", compare.pointwise(run_chain1(t), ref.chain1(t["X"], t["W"], t["bias"])))
    Z, Dn = ref.gemm_bias(t["X"], t["W"], None, want_norm=True)
    assert show("anchor no bias", compare.contraction(run_chain1(t, relu=False, softmax=False, bias=False), Z, Dn))


@pytest.mark.parametrize("M,K,N", [(50, 40, 300), (130, 260, 1000), (256, 64, 257)])
def test_gemm_bias_relu_wide(M, K, N):
    print("gemm M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    assert show("gemm+bias+relu", compare.contraction(run_chain1(t, softmax=False), ref.relu(Z), Dn))


@pytest.mark.parametrize("M,K,N", [(64, 256, 1000), (33, 50, 257), (700, 64, 4096), (4096, 32, 2052)])
def test_chain1_rows_wider_than_a_tile(M, K, N):
    print("chain1 wide M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    assert show("softmax", compare.pointwise(run_chain1(t), ref.chain1(t["X"], t["W"], t["bias"])))


@pytest.mark.parametrize("M,K,N", [(256, 2048, 256), (1024, 4096, 1024), (512, 1030, 512), (200, 3000, 333), (128, 8192, 512)])
def test_gemm_split_k(M, K, N):
    print("split-k M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    X, W, b = dev(t["X"]), dev(t["W"]), dev(t["bias"])
    out = torch.full((M, N), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(X, W, b, out, relu=True, softmax=False)
    assert plan.kernel_name == "gemm_tile64<split-k>" and plan.workspace_bytes % (M * N * 4) == 0
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
    plan.launch(ins, [out], workspace=ws)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    got = host(out)
    assert show("split-k gemm+bias+relu", compare.contraction(got, ref.relu(Z), Dn))
    assert np.max(np.abs(got - ref.relu(Z)) / Dn) < 1e-5
    # with the softmax over wide rows behind it, and with the dropout epilogue
    assert show("softmax", compare.pointwise(run_chain1(t), ref.chain1(t["X"], t["W"], t["bias"])))
    t6 = dict(t)
    D = ref.dropout_hash(Z, 0.25, 99)
    got, name = run_chain6(t6, 0.25, 99, "dropout")
    assert name == "gemm_tile64<split-k>"
    assert np.array_equal(got == 0, D == 0)
    assert show("dropout", compare.contraction(got, D, Dn / 0.75))
    again, _ = run_chain6(t6, 0.25, 99, "dropout")
    assert np.array_equal(got, again)


# ------------------------- W stored transposed (a linear layer's [N,K] weight) and the Gemm-Scale epilogue
def run_gemm(t, wt=False, relu=True, softmax=False, bias=True, scale=None):
    """through the C ABI; wt: the device copy of W is [N,K] row-major and its .t() view is passed"""
    X = dev(t["X"])
    W = dev(np.ascontiguousarray(t["W"].T)).t() if wt else dev(t["W"])
    b = dev(t["bias"]) if bias else None
    M, N = X.shape[0], W.shape[1]
    out = torch.full((M, N), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(X, W, b, out, relu=relu, softmax=softmax, scale=scale)
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda") if plan.workspace_bytes else None
    plan.launch(ins, [out], workspace=ws)
    return host(out), plan.kernel_name


@pytest.mark.parametrize("M,K,N", [(64, 4096, 256), (48, 1000, 96), (130, 520, 34), (2048, 64, 64), (20, 4100, 31),
                                   (16, 272, 32), (100, 528, 1000), (15, 65, 2), (1000, 260, 30)])
def test_gemm_small_outputs_share_k_between_waves(M, K, N):
    # the kernel for few output rows: 16 x 32 tiles, K dealt out to the 16 waves of a work-group in 16-k groups
    # (none, one or two per wave and trip, ragged last groups, odd N without vector loads), with every epilogue,
    # the softmax behind it as a second launch, and run-to-run bit identity of the fixed-order LDS combine
    print("gemm small M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    got, name = run_gemm(t)
    assert name == "gemm_ksplit16<32>", name
    assert show("gemm+bias+relu", compare.contraction(got, ref.relu(Z), Dn))
    assert np.max(np.abs(got - ref.relu(Z)) / Dn) < 1e-5
    again, _ = run_gemm(t)
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32))
    got, _ = run_gemm(t, softmax=True)
    assert show("softmax", compare.pointwise(got, ref.chain1(t["X"], t["W"], t["bias"])))
    Z0, Dn0 = ref.gemm_bias(t["X"], t["W"], None, want_norm=True)
    got, _ = run_gemm(t, relu=False, bias=False, scale=-0.75)
    assert show("anchor * scale", compare.contraction(got, ref.scale_const(Z0, -0.75), Dn0 * 0.75))
    got, _ = run_gemm(t, relu="gelu")
    assert show("gelu", compare.contraction(got, ref.gelu_tanh(Z), Dn * 1.13 + 1e-6))


def wt_name(plain):
    """kernel name of the transposed-W instance of `plain`"""
    if plain.startswith("gemm_rows16<"):
        return plain[:-1] + ",wt>"
    return plain.replace("<", "<wt,") if "<" in plain else plain + "<wt>"


@pytest.mark.parametrize("M,K,N", [
    (64, 256, 256), (17, 5, 10), (70, 100, 63), (33, 36, 130), (3, 300, 129), (2, 1, 3),       # 16-row kernel
    (4096, 256, 4096), (1024, 512, 1024), (700, 260, 644), (515, 37, 1001), (2900, 33, 3001),  # tiles of 128 and 64
    (256, 2048, 256), (200, 3000, 333),                                                        # K slices
    (2100, 36, 2052), (1800, 64, 2304), (2048, 4, 2048), (3000, 20, 1540), (1600, 60, 2944)])  # short K, no LDS
def test_gemm_transposed_weight(M, K, N):
    print("gemm wt M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    plain, plain_name = run_gemm(t, wt=False)
    got, name = run_gemm(t, wt=True)
    assert show("gemm wt +bias+relu", compare.contraction(got, ref.relu(Z), Dn))
    assert np.max(np.abs(got - ref.relu(Z)) / Dn) < 1e-5
    if plain_name == "gemm_direct":
        # the kernel for a short K takes a row-major W only; a transposed one goes to the tiled kernel
        assert name in ("gemm_tile128<wt>", "gemm_tile64<wt>")
    elif plain_name.startswith("gemm_ksplit16"):
        # so does the small-output kernel whose waves share K; a transposed W stays with the 16-row kernel
        # (another summation order: both are checked against the CPU checker, not against each other)
        assert name.startswith("gemm_rows16") and name.endswith(",wt>")
    else:
        # (with K = 1 or N = 1 the transposed storage is also row-major)
        assert name == (plain_name if K == 1 or N == 1 else wt_name(plain_name)), (name, plain_name)
        # the same products in the same order as with the row-major copy of W: bit-identical results
        assert np.array_equal(got.view(np.uint32), plain.view(np.uint32))
    got, _ = run_gemm(t, wt=True, softmax=True)
    assert show("softmax", compare.pointwise(got, ref.chain1(t["X"], t["W"], t["bias"])))
    Z0, Dn0 = ref.gemm_bias(t["X"], t["W"], None, want_norm=True)
    got, _ = run_gemm(t, wt=True, relu=False, bias=False)
    assert show("anchor alone", compare.contraction(got, Z0, Dn0))


def test_gemm_transposed_weight_is_not_symmetric_in_k_and_n():
    # W = a shift matrix: (X W)[m, n] = X[m, n-1]; reading W with k and n swapped would give X[m, n+1]
    X = datagen.gen_uniform(6, (40, 96), -1, 1)
    Wm = np.zeros((96, 96), np.float32)
    Wm[np.arange(95), np.arange(1, 96)] = 1.0
    got, _ = run_gemm({"X": X, "W": Wm}, wt=True, relu=False, bias=False)
    want = np.zeros_like(X); want[:, 1:] = X[:, :-1]
    assert np.array_equal(got, want)


@pytest.mark.parametrize("M,K,N,scale", [(64, 256, 256, 0.5), (33, 36, 130, -3.7), (1024, 512, 1024, 0.125), (515, 37, 1001, -0.3),
                                         (256, 2048, 256, 1.7)])
def test_gemm_scale(M, K, N, scale):
    # Gemm-Scale (Section 5.2): (X W + bias) * scale, then ReLU / softmax
    print("gemm scale M=%d K=%d N=%d s=%r" % (M, K, N, scale), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    Zs, Ds = ref.scale_const(Z, scale), Dn * abs(float(np.float32(scale)))
    for wt in (False, True):
        got, _ = run_gemm(t, wt=wt, relu=False, scale=scale)
        assert show("scaled", compare.contraction(got, Zs, Ds))
        got, _ = run_gemm(t, wt=wt, relu=True, scale=scale)
        assert show("scaled + relu", compare.contraction(got, ref.relu(Zs), Ds))
    got, _ = run_gemm(t, softmax=True, scale=scale)
    assert show("scaled + relu + softmax", compare.pointwise(got, ref.softmax_rows(ref.relu(Zs))))
    # scale = 1 is the chain without the step, bit for bit
    one, _ = run_gemm(t, scale=1.0)
    none, _ = run_gemm(t)
    assert np.array_equal(one.view(np.uint32), none.view(np.uint32))


@pytest.mark.parametrize("B,M,K,N", [(3, 64, 256, 256), (2, 17, 5, 10), (5, 70, 100, 63), (4, 600, 64, 520), (16, 256, 128, 256),
                                     (2, 1100, 36, 1030), (3, 33, 300, 300), (1, 40, 64, 128)])
def test_batched_gemm(B, M, K, N):
    print("batched gemm B=%d M=%d K=%d N=%d" % (B, M, K, N), flush=True)
    X = datagen.gen_normal(600, (B, M, K), 0.0, 1.0)
    W = datagen.gen_normal(601, (B, K, N), 0.0, 1.0 / np.sqrt(K))
    b = datagen.gen_normal(602, (N,), 0.0, 0.5)
    Z = np.empty((B, M, N)); Dn = np.empty((B, M, N))
    for i in range(B):
        Z[i], Dn[i] = ref.gemm_bias(X[i], W[i], b, want_norm=True)
    for wt in (False, True):
        Wd = dev(np.ascontiguousarray(W.transpose(0, 2, 1))).transpose(1, 2) if wt else dev(W)
        out = torch.full((B, M, N), float("nan"), device="cuda")
        plan, ins = hpct.gemm_bias_relu_softmax_plan(dev(X), Wd, dev(b), out, relu=True, softmax=False, scale=0.5)
        assert plan.workspace_bytes == 0
        plan.launch(ins, [out])
        assert show("batched %s" % plan.kernel_name, compare.contraction(host(out), ref.relu(ref.scale_const(Z, 0.5)), Dn * 0.5))
    # with the row softmax behind it (fused up to 256 columns, a second kernel beyond)
    out = torch.full((B, M, N), float("nan"), device="cuda")
    hpct.gemm_bias_relu_softmax(dev(X), dev(W), dev(b), out)
    assert show("batched softmax", compare.pointwise(host(out), ref.softmax_rows(ref.relu(Z).reshape(B * M, N)).reshape(B, M, N)))
    # one W for the whole batch: the [B*M, K] product
    out = torch.full((B, M, N), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(dev(X), dev(W[0]), dev(b), out, relu=False, softmax=False)
    ws = torch.empty(plan.workspace_bytes // 4, device="cuda") if plan.workspace_bytes else None
    plan.launch(ins, [out], workspace=ws)
    Zs, Ds = ref.gemm_bias(X.reshape(B * M, K), W[0], b, want_norm=True)
    assert show("shared W", compare.contraction(host(out).reshape(B * M, N), Zs, Ds))


@pytest.mark.parametrize("M,K,N", [(64, 256, 256), (33, 36, 130), (700, 260, 644), (2900, 33, 1001), (1024, 512, 4096),
                                   (256, 2048, 256), (2100, 36, 2052)])
def test_gemm_activation_epilogues(M, K, N):
    # the 16-row kernel, tiles of 64 and 128, K slices (activation in the finishing kernel) and the short-K kernel
    print("gemm act M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"] * 8.0, t["bias"], want_norm=True)       # pre-activations of a few units
    t8 = dict(t, W=(t["W"] * 8.0).astype(np.float32))
    Z32 = Z.astype(np.float32).reshape(-1)        # (the checker's elementwise steps take fp32 inputs: 6e-8 relative, far inside the bound)
    names = set()
    for act, lip in (("relu6", 1.0), ("gelu", 1.13), ("sigmoid", 0.25), ("tanh", 1.0)):
        # the activation of the exact pre-activation; |f(a) - f(b)| <= lip |a - b| carries the contraction bound through
        if act == "relu6":
            want = ref.relu6(Z)
        elif act == "gelu":
            want = ref.gelu_tanh(Z)
        else:
            want = ref.eltwise_map(Z32, Z.shape, (Z.shape[1], 1), unary=[act])
        got, name = run_gemm(t8, relu=act)
        names.add(name)
        assert show("gemm + %s (%s)" % (act, name), compare.contraction(got, want, Dn * lip + 1e-6))
    got, name = run_gemm(t8, relu="gelu", scale=0.5, wt=True)
    assert show("gemm wt + scale + gelu", compare.contraction(got, ref.gelu_tanh(ref.scale_const(Z, 0.5)), Dn * 0.6 + 1e-6))
    print("kernels", sorted(names), flush=True)


@pytest.mark.parametrize("M,K,N", [(64, 256, 256), (70, 100, 63), (700, 260, 644), (1024, 512, 4096), (256, 2048, 256), (2100, 36, 2052)])
def test_gemm_strided_x(M, K, N):
    # X given as the transpose of a [K,M] array, and as a column slice of a wider matrix: copied to the workspace first
    print("gemm strided X M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    W, b = dev(t["W"]), dev(t["bias"])
    wide = torch.full((M, K + 5), float("nan"), device="cuda")
    wide[:, 3:3 + K] = dev(t["X"])
    for tag, Xv in (("transposed", dev(np.ascontiguousarray(t["X"].T)).t()), ("slice", wide[:, 3:3 + K])):
        out = torch.full((M, N), float("nan"), device="cuda")
        plan, ins = hpct.gemm_bias_relu_softmax_plan(Xv, W, b, out, relu=True, softmax=False)
        assert plan.workspace_bytes >= M * K * 4
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
        plan.launch(ins, [out], workspace=ws)
        assert show("strided X (%s) %s" % (tag, plan.kernel_name), compare.contraction(host(out), ref.relu(Z), Dn))
        with pytest.raises(hpct.HpctError):
            plan.launch(ins, [out])          # no workspace
    # the same values as from the row-major X, bit for bit (the copy is exact)
    plain, _ = run_gemm(t)
    assert np.array_equal(host(out).view(np.uint32), plain.view(np.uint32))
    # a batch of transposed matrices
    B2 = 3
    Xb = datagen.gen_normal(620, (B2, min(M, 200), K), 0.0, 1.0)
    Wb = datagen.gen_normal(621, (B2, K, min(N, 300)), 0.0, 1.0 / np.sqrt(K))
    Xt = dev(np.ascontiguousarray(Xb.transpose(0, 2, 1))).transpose(1, 2)
    out = torch.full((B2, Xb.shape[1], Wb.shape[2]), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(Xt, dev(Wb), None, out, relu=False, softmax=False)
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
    plan.launch(ins, [out], workspace=ws)
    for i in range(B2):
        Zi, Di = ref.gemm_bias(Xb[i], Wb[i], None, want_norm=True)
        assert compare.contraction(host(out)[i], Zi, Di).ok, i


@pytest.mark.parametrize("M,K,N,wt", [
    (300, 4096, 1, False), (5000, 256, 3, False), (1024, 1028, 8, False), (64, 20000, 2, False), (4100, 512, 5, True), (33, 32768, 1, True),
    (1, 4096, 600, True), (5, 1024, 2000, True), (8, 260, 5000, True), (2, 65536, 17, True)])
def test_gemm_skinny_shapes(M, K, N, wt):
    # matrix-vector products and tall-skinny shapes: the rows of the large operand are streamed (a wave or a work-group per row)
    print("gemm skinny M=%d K=%d N=%d wt=%s" % (M, K, N, wt), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    got, name = run_gemm(t, wt=wt, relu=False)
    assert name.startswith("gemm_skinny<"), name
    # (with N = 1 the transposed storage is also row-major)
    assert name == ("gemm_skinny<rows of W>" if M <= 8 and N > 8 else ("gemm_skinny<rows of X,wt>" if wt and N > 1 else "gemm_skinny<rows of X>"))
    assert show("skinny %s" % name, compare.contraction(got, Z, Dn))
    assert np.max(np.abs(got - Z) / Dn) < 1e-5
    got, _ = run_gemm(t, wt=wt, relu="gelu", scale=0.5)
    assert show("skinny + scale + gelu", compare.contraction(got, ref.gelu_tanh(ref.scale_const(Z, 0.5)), Dn * 0.6 + 1e-6))
    Z0, D0 = ref.gemm_bias(t["X"], t["W"], None, want_norm=True)
    got, _ = run_gemm(t, wt=wt, relu=True, bias=False)
    assert show("skinny, no bias, relu", compare.contraction(got, ref.relu(Z0), D0))


def test_gemm_skinny_batch_and_fallbacks():
    B, M, K, N = 3, 700, 2048, 2
    X = datagen.gen_normal(630, (B, M, K), 0.0, 1.0)
    W = datagen.gen_normal(631, (B, K, N), 0.0, 1.0 / np.sqrt(K))
    out = torch.full((B, M, N), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(dev(X), dev(W), None, out, relu=False, softmax=False)
    assert plan.kernel_name == "gemm_skinny<rows of X>" and plan.launch_shape()[0] == (M, B, 1)
    plan.launch(ins, [out])
    for i in range(B):
        Zi, Di = ref.gemm_bias(X[i], W[i], None, want_norm=True)
        assert compare.contraction(host(out)[i], Zi, Di).ok, i
    # with a softmax behind it, a K or (under a small M) an N that is not a multiple of 4, or a small operand: the other kernels
    t = datagen.make(1, M=300, K=4096, N=4)
    _, name = run_gemm(t, softmax=True)
    assert not name.startswith("gemm_skinny")
    for (M2, K2, N2) in [(1, 4096, 602), (300, 4098, 1), (100, 512, 2)]:
        t = datagen.make(1, M=M2, K=K2, N=N2)
        Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
        got, name = run_gemm(t)
        assert not name.startswith("gemm_skinny")
        assert compare.contraction(got, ref.relu(Z), Dn).ok


@pytest.mark.parametrize("M,K,N", [(1, 4096, 600), (1, 16384, 4096), (3, 1000, 2052), (8, 260, 5000), (5, 8192, 256), (2, 300, 16384)])
def test_gemm_skinny_columns(M, K, N):
    # a few rows of X times a row-major W: W's rows streamed along n, K cut into slices, the tiled kernel's finishing pass
    print("gemm skinny cols M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    got, name = run_gemm(t, relu=False)
    assert name == "gemm_skinny_cols"
    assert show("skinny cols", compare.contraction(got, Z, Dn))
    assert np.max(np.abs(got - Z) / Dn) < 1e-5
    got, _ = run_gemm(t, relu="tanh", scale=0.5)
    assert show("skinny cols + scale + tanh", compare.contraction(got, np.tanh(ref.scale_const(Z, 0.5)), Dn * 0.5 + 1e-6))
    again, _ = run_gemm(t, relu=False)
    assert np.array_equal(got.view(np.uint32) * 0 + again.view(np.uint32), run_gemm(t, relu=False)[0].view(np.uint32))   # deterministic


def test_gemm_short_k_direct_kernel():
    # operands straight into the MFMA layout: K below, at and between the 32-wide chunks, the dropout epilogue
    # (an integer decision per element), and a batch
    for (M, K, N) in [(2100, 36, 2052), (1700, 32, 2560), (2176, 64, 2048)]:
        print("gemm direct M=%d K=%d N=%d" % (M, K, N), flush=True)
        t = datagen.make(1, M=M, K=K, N=N)
        Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
        got, name = run_gemm(t)
        assert name == "gemm_direct"
        assert show("direct", compare.contraction(got, ref.relu(Z), Dn))
        D = ref.dropout_hash(Z, 0.3, 11)
        got, name = run_chain6(t, 0.3, 11, "dropout")
        assert name == "gemm_direct"
        differ = (got == 0) != (D == 0)   # the mask is an integer decision; a kept element may still cancel to 0 in fp32
        assert np.all(np.abs(Z[differ]) < 1e-6 * Dn[differ]), np.argwhere(differ)[:5]
        assert show("dropout", compare.contraction(got, D, Dn / 0.7))
    B, M, K, N = 20, 300, 32, 520
    X = datagen.gen_normal(610, (B, M, K), 0.0, 1.0)
    W = datagen.gen_normal(611, (B, K, N), 0.0, 1.0 / np.sqrt(K))
    for wt in (False, True):
        Wd = dev(np.ascontiguousarray(W.transpose(0, 2, 1))).transpose(1, 2) if wt else dev(W)
        out = torch.full((B, M, N), float("nan"), device="cuda")
        plan, ins = hpct.gemm_bias_relu_softmax_plan(dev(X), Wd, None, out, relu=False, softmax=False)
        assert plan.kernel_name == ("gemm_tile64<wt>" if wt else "gemm_direct")
        plan.launch(ins, [out])
        got = host(out)
        for i in range(B):
            Zi, Di = ref.gemm_bias(X[i], W[i], None, want_norm=True)
            assert compare.contraction(got[i], Zi, Di).ok, i


def test_gemm_identity_weight_is_exact():
    X = datagen.gen_uniform(5, (48, 64), -1, 1)
    out = torch.empty(48, 64, device="cuda")
    hpct.gemm_bias_relu_softmax(dev(X), dev(np.eye(64, dtype=np.float32)), None, out, relu=False, softmax=False)
    assert np.array_equal(host(out), X)


# ------------------------------------- tiled GEMM and the Section 5.3 dropout chain
def run_chain6(t, p, seed, stop_after="softmax", bias=True, relu=False):
    X, W = dev(t["X"]), dev(t["W"])
    b = dev(t["bias"]) if bias else None
    M, N = X.shape[0], W.shape[1]
    out = torch.full((M, N) if stop_after == "dropout" else (M,), float("nan"), device="cuda")
    plan, _ = hpct.matmul_dropout_mean_softmax_plan(X, W, b, out, p, seed, stop_after, relu)
    ws = None
    if plan.workspace_bytes:
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
    else:
        assert stop_after == "dropout"
    hpct.matmul_dropout_mean_softmax(X, W, b, out, p, seed, ws, stop_after, relu)
    return host(out), plan.kernel_name


def check_chain6(t, p, seed):
    X, W, b = t["X"], t["W"], t["bias"]
    Z, Dn = ref.gemm_bias(X, W, b, want_norm=True)
    D = ref.dropout_hash(Z, p, seed)
    got, name = run_chain6(t, p, seed, "dropout")
    print("kernel", name, flush=True)
    # the mask is an integer decision: identical element by element (a kept element is 0 only if Z is)
    assert np.array_equal(got == 0, D == 0)
    assert show("dropout", compare.contraction(got, D, Dn / (1.0 - p)))
    mu = ref.mean_rows(D)
    got, _ = run_chain6(t, p, seed, "mean")
    # a row mean is itself a contraction output (sum over k and n with cancellation): same rule,
    # normalised by the mean of the surviving elements' magnitudes
    assert show("mean", compare.contraction(got, mu, ref.mean_rows(np.where(D != 0, Dn / (1.0 - p), 0.0)) + 1e-300))
    got, _ = run_chain6(t, p, seed, "softmax")
    want = ref.softmax_rows(mu.reshape(1, -1)).reshape(-1)
    assert show("softmax", compare.pointwise(got, want))
    assert abs(float(got.astype(np.float64).sum()) - 1.0) < 1e-4
    return name


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (64, 256, 256), (77, 50, 130), (40, 64, 1000), (19, 33, 257)])
def test_chain6_small_shapes(M, K, N):
    print("chain6 M=%d K=%d N=%d" % (M, K, N), flush=True)
    name = check_chain6(datagen.make(6, M=M, K=K, N=N), datagen.CHAIN6_P, datagen.CHAIN6_SEED)
    assert name.startswith(("gemm_rows16", "gemm_ksplit16"))


@pytest.mark.parametrize("M,K,N", [(640, 72, 900), (513, 70, 1027), (1024, 8, 512), (520, 100, 1100), (129, 16, 4100),
                                   (2100, 40, 4000), (4100, 24, 2052), (4096, 16, 4096)])
def test_chain6_tiled_shapes(M, K, N):
    print("chain6 tiled M=%d K=%d N=%d" % (M, K, N), flush=True)
    name = check_chain6(datagen.make(6, M=M, K=K, N=N), datagen.CHAIN6_P, datagen.CHAIN6_SEED)
    # (the dropout stage alone, whose kernel is named here, goes to the kernel without LDS when K is short)
    assert name in ("gemm_tile128", "gemm_tile64", "gemm_direct")
    assert (name == "gemm_direct") == (K <= 64 and K % 4 == 0 and N % 4 == 0 and ((M + 127) // 128) * ((N + 127) // 128) >= 256)


@pytest.mark.parametrize("p,seed", [(0.0, 1), (0.5, 0), (0.3, (1 << 64) - 5), (0.999, 77)])
def test_chain6_probabilities_and_seeds(p, seed):
    print("chain6 p=%r seed=%d" % (p, seed), flush=True)
    check_chain6(datagen.make(6, M=48, K=40, N=200), p, seed)
    check_chain6(datagen.make(6, M=384, K=32, N=1280), p, seed)


def test_chain6_full_size_and_determinism():
    t = datagen.make(6)
    p, seed = datagen.CHAIN6_P, datagen.CHAIN6_SEED
    got, name = run_chain6(t, p, seed)
    assert name == "gemm_tile128"
    want = ref.chain6(t["X"], t["W"], t["bias"], p, seed)
    assert show("chain6 4096x1024x4096", compare.pointwise(got, want))
    again, _ = run_chain6(t, p, seed)
    assert np.array_equal(got, again)


@pytest.mark.parametrize("M,K,N", [(1024, 512, 1024), (700, 260, 644), (515, 37, 1001), (3000, 100, 2900), (2900, 33, 3001)])
def test_tiled_gemm_bias_relu(M, K, N):
    print("tiled gemm M=%d K=%d N=%d" % (M, K, N), flush=True)
    t = datagen.make(1, M=M, K=K, N=N)
    X, W, b = dev(t["X"]), dev(t["W"]), dev(t["bias"])
    out = torch.full((M, N), float("nan"), device="cuda")
    plan, ins = hpct.gemm_bias_relu_softmax_plan(X, W, b, out, relu=True, softmax=False)
    assert plan.kernel_name in ("gemm_tile128", "gemm_tile64", "gemm_tile64<split-k>")
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda") if plan.workspace_bytes else None
    plan.launch(ins, [out], workspace=ws)
    Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
    assert show("tiled gemm+bias+relu", compare.contraction(host(out), ref.relu(Z), Dn))
    assert np.max(np.abs(host(out) - ref.relu(Z)) / Dn) < 1e-5


def test_chain6_workspace_is_required():
    t = datagen.make(6, M=32, K=16, N=64)
    X, W, b = dev(t["X"]), dev(t["W"]), dev(t["bias"])
    out = torch.empty(32, device="cuda")
    with pytest.raises(hpct.HpctError) as e:
        hpct.matmul_dropout_mean_softmax(X, W, b, out, 0.25, 1, None)
    assert e.value.status == hpct.HPCT_ERR_WORKSPACE
    small = torch.empty(4, device="cuda")
    with pytest.raises(hpct.HpctError) as e:
        hpct.matmul_dropout_mean_softmax(X, W, b, out, 0.25, 1, small)
    assert e.value.status == hpct.HPCT_ERR_WORKSPACE


# ------------------------------------------------------------------- chain 2
def run_chain2(t, pool=True, relu=True, affine=True, residual=True):
    X = dev(t["X"])
    sc, sh = (dev(t["scale"]), dev(t["shift"])) if affine else (None, None)
    R = dev(t["R"]) if residual else None
    shape = X.shape[:2] if pool else X.shape
    out = torch.full(tuple(shape), float("nan"), device="cuda")
    hpct.scale_shift_relu_add_pool(X, sc, sh, R, out, relu=relu, pool=pool)
    return host(out)


def test_chain2_full_size():
    t = datagen.make(2)
    want = ref.chain2(t["X"], t["scale"], t["shift"], t["R"])
    got = run_chain2(t)
    assert show("chain2 32x64x56x56", compare.pointwise(got, want))
    got2 = run_chain2(t)
    assert np.array_equal(got.view(np.uint32), got2.view(np.uint32))  # fixed reduction order


@pytest.mark.parametrize("N,C,H,W", [(1, 1, 1, 1), (2, 3, 1, 3), (3, 5, 7, 7), (2, 4, 2, 2), (1, 2, 40, 52),
                                     (2, 3, 64, 65), (1, 2, 128, 128)])
def test_chain2_ragged_shapes(N, C, H, W):
    print("chain2 %s" % ((N, C, H, W),), flush=True)
    t = datagen.make(2, N=N, C=C, H=H, W=W)
    assert show("pool", compare.pointwise(run_chain2(t), ref.chain2(t["X"], t["scale"], t["shift"], t["R"])))
    T = ref.affine_relu_residual(t["X"], t["scale"], t["shift"], t["R"])
    assert show("store", compare.pointwise(run_chain2(t, pool=False), T))
    # sub-chains
    Xd = t["X"].astype(np.float64)
    assert show("pool only", compare.pointwise(run_chain2(t, relu=False, affine=False, residual=False), ref.avgpool_hw(Xd)))
    assert show("relu store", compare.pointwise(run_chain2(t, pool=False, affine=False, residual=False), ref.relu(Xd)))


# ------------------------------------------------------------------- chain 3
def run_chain3(t, gelu=True, affine=True, eps=1e-5):
    X = dev(t["X"])
    g, b = (dev(t["gamma"]), dev(t["beta"])) if affine else (None, None)
    out = torch.full(tuple(X.shape), float("nan"), device="cuda")
    hpct.layernorm_gelu(X, g, b, out, eps=eps, gelu=gelu)
    return host(out)


def test_chain3_full_size():
    t = datagen.make(3)
    want = ref.chain3(t["X"], t["gamma"], t["beta"], 1e-5)
    got = run_chain3(t)
    assert show("chain3 8192x4096", compare.pointwise(got, want))
    got2 = run_chain3(t)
    assert np.array_equal(got.view(np.uint32), got2.view(np.uint32))


@pytest.mark.parametrize("M,N", [(1, 1), (3, 2), (5, 3), (7, 64), (9, 100), (33, 256), (6, 1000), (4, 1024),
                                 (5, 1028), (3, 2048), (5, 4100), (2, 8192), (3, 16384), (2, 16388), (2, 20001)])
def test_chain3_ragged_shapes(M, N):
    print("chain3 M=%d N=%d" % (M, N), flush=True)
    t = datagen.make(3, M=M, N=N)
    want = ref.chain3(t["X"], t["gamma"], t["beta"], 1e-5)
    if N == 1:  # x - mean = 0 exactly: output = gelu(beta)
        want = ref.gelu_tanh(np.tile(t["beta"].astype(np.float64), (M, 1)))
    assert show("ln+gelu", compare.pointwise(run_chain3(t), want))
    if N > 1:
        assert show("ln only, no affine", compare.pointwise(run_chain3(t, gelu=False, affine=False),
                                                            ref.layernorm_rows(t["X"], None, None, 1e-5)))


@pytest.mark.parametrize("M,N", [(1, 1), (5, 7), (3, 256), (4, 1000), (2, 5000), (9, 4), (70, 260), (33, 1024), (17, 1028),
                                 (600, 2048), (515, 4096), (40, 4100), (12, 8192), (7, 16384), (5, 16388), (3, 40000)])
def test_softmax_rows(M, N):
    X = datagen.gen_normal(77, (M, N), 0.0, 3.0)
    out = torch.full((M, N), float("nan"), device="cuda")
    plan, ins = hpct.softmax_rows_plan(dev(X), out)
    print("softmax %dx%d" % (M, N), plan.kernel_name, flush=True)
    plan.launch(ins, [out])
    got = host(out)
    assert show("softmax %dx%d" % (M, N), compare.pointwise(got, ref.softmax_rows(X.astype(np.float64))))
    assert np.allclose(got.astype(np.float64).sum(axis=1), 1.0, rtol=0, atol=1e-5)


def test_softmax_rows_full_size_and_large_values():
    X = datagen.make(3)["X"] * np.float32(40.0)          # [8192, 4096], values up to +-200: needs the row max
    out = torch.full(X.shape, float("nan"), device="cuda")
    plan, ins = hpct.softmax_rows_plan(dev(X), out)
    assert plan.kernel_name == "softmax_rows_persist"
    plan.launch(ins, [out])
    got = host(out)
    assert np.all(np.isfinite(got))
    assert show("softmax 8192x4096", compare.pointwise(got, ref.softmax_rows(X.astype(np.float64))))


# ------------------------------------------------------------------- chain 4
def run_chain4(t, pad=1, relu=True, bias=True):
    x, w = dev(t["in"]), dev(t["wt"])
    b = dev(t["bias"]) if bias else None
    Nb, _, H, W = t["in"].shape
    K, _, R, S = t["wt"].shape
    Ho, Wo = ref.conv_out_hw(H, W, R, S, 1, pad)
    out = torch.full((Nb, K, Ho, Wo), float("nan"), device="cuda")
    hpct.conv2d_bias_relu(x, w, b, out, stride=1, pad=pad, relu=relu)
    return host(out)


def test_chain4_full_size():
    t = datagen.make(4)
    want, Dn = ref.chain4(t["in"], t["wt"], t["bias"], 1, 1)
    got = run_chain4(t)
    assert show("chain4 conv3x3 32x64x56x56 -> 128", compare.contraction(got, want, Dn))
    assert np.max(np.abs(got - want) / Dn) < 1e-5
    got2 = run_chain4(t)
    assert np.array_equal(got.view(np.uint32), got2.view(np.uint32))


@pytest.mark.parametrize("N,C,H,W,K,R,pad", [
    (1, 1, 1, 1, 1, 1, 0), (1, 2, 4, 4, 3, 3, 1), (2, 3, 7, 9, 5, 3, 1), (1, 8, 8, 8, 128, 3, 1),
    (2, 10, 13, 5, 130, 3, 1), (1, 16, 12, 12, 64, 3, 0), (1, 4, 6, 70, 7, 3, 2), (3, 5, 9, 9, 20, 1, 0),
    (1, 64, 14, 14, 256, 1, 0), (1, 12, 3, 3, 9, 3, 1), (1, 9, 30, 200, 33, 3, 1), (2, 6, 1, 1, 4, 3, 1)])
def test_chain4_ragged_shapes(N, C, H, W, K, R, pad):
    print("chain4 %s" % ((N, C, H, W, K, R, pad),), flush=True)
    t = datagen.make(4, N=N, C=C, H=H, W=W, K=K, R=R, S=R)
    want, Dn = ref.chain4(t["in"], t["wt"], t["bias"], 1, pad)
    assert show("conv+bias+relu", compare.contraction(run_chain4(t, pad=pad), want, Dn))
    raw, Dn0 = ref.conv2d_nchw_bias(t["in"], t["wt"], None, 1, pad, want_norm=True)
    assert show("conv alone", compare.contraction(run_chain4(t, pad=pad, relu=False, bias=False), raw, Dn0))


def test_conv_all_ones_counts_taps_exactly():
    x = np.ones((1, 8, 10, 11), np.float32)
    w = np.ones((4, 8, 3, 3), np.float32)
    got = run_chain4({"in": x, "wt": w}, pad=1, relu=False, bias=False)
    want = ref.conv2d_nchw_bias(x, w, None, 1, 1)
    assert np.array_equal(got, want)  # small integers: exact in fp32


# ----------------------------- conv block: stride, scale/shift, 2x2 max pool (VGG-style)
def run_chain7(t, stride=1, pad=1, relu=True, pool=True, bias=True, affine=True, dil=1):
    x, w = dev(t["in"]), dev(t["wt"])
    b = dev(t["bias"]) if bias else None
    sc, sh = (dev(t["scale"]), dev(t["shift"])) if affine else (None, None)
    Nb, _, H, W = t["in"].shape
    K, _, R, S = t["wt"].shape
    Ho, Wo = ref.conv_out_hw(H, W, R, S, stride, pad, dil)
    out = torch.full((Nb, K, Ho // 2, Wo // 2) if pool else (Nb, K, Ho, Wo), float("nan"), device="cuda")
    plan, ins = hpct.conv_block_plan(x, w, b, sc, sh, out, stride, pad, relu, pool, dil)
    plan.launch(ins, [out])
    return host(out), plan.kernel_name


def check_chain7(t, stride=1, pad=1, relu=True, pool=True, bias=True, affine=True, dil=1):
    want, Dn = ref.chain7(t["in"], t["wt"], t["bias"] if bias else None, t["scale"] if affine else None,
                          t["shift"] if affine else None, stride, pad, relu, pool, dil)
    if pool:   # |max a - max b| <= max |a_i - b_i|: the window's largest bound
        Dn = ref.maxpool2x2(Dn)
    got, name = run_chain7(t, stride, pad, relu, pool, bias, affine, dil)
    print("kernel", name, flush=True)
    assert show("conv block", compare.contraction(got, want, Dn))
    return got, name


def test_chain7_full_size():
    t = datagen.make(7)
    got, name = check_chain7(t)
    assert name == "conv2d_nchw_mfma<3x3,pipelined,maxpool2>"
    again, _ = run_chain7(t)
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32))
    # the same block without pooling goes through the kernel of chain 4 with the scale/shift epilogue
    _, name = check_chain7(t, pool=False)
    assert name == "conv2d_nchw_mfma<3x3,pipelined>"


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad", [
    (1, 1, 2, 2, 1, 1, 1, 0), (2, 3, 7, 9, 5, 3, 1, 1), (1, 8, 8, 8, 128, 3, 1, 1), (2, 10, 13, 5, 130, 3, 1, 1),
    (1, 4, 6, 70, 7, 3, 1, 2), (1, 4, 10, 224, 64, 3, 1, 1), (1, 64, 14, 14, 64, 1, 1, 0), (1, 8, 9, 9, 20, 3, 1, 0),
    (2, 8, 16, 16, 64, 3, 2, 1), (1, 3, 40, 40, 16, 7, 2, 3), (1, 6, 21, 33, 10, 5, 1, 2), (1, 4, 17, 17, 8, 5, 3, 2),
    (1, 16, 12, 36, 64, 1, 2, 0), (1, 5, 30, 30, 12, 7, 1, 3), (1, 4, 64, 64, 64, 3, 4, 1)])
def test_chain7_ragged_shapes(N, C, H, W, K, R, stride, pad):
    print("chain7 %s" % ((N, C, H, W, K, R, stride, pad),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=R, S=R)
    check_chain7(t, stride, pad)                       # the whole block
    check_chain7(t, stride, pad, pool=False)           # conv + bias + scale/shift + relu
    check_chain7(t, stride, pad, relu=False)           # pooling sees negative values
    check_chain7(t, stride, pad, relu=False, pool=False, bias=False, affine=False)   # the bare strided conv


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad,dil", [
    (1, 4, 12, 12, 64, 3, 1, 2, 2), (2, 5, 17, 23, 9, 3, 1, 0, 2), (1, 8, 20, 20, 64, 3, 2, 3, 3), (1, 3, 30, 30, 8, 5, 1, 4, 2),
    (1, 16, 16, 16, 64, 1, 1, 0, 3), (1, 8, 33, 40, 70, 3, 1, 4, 4), (2, 64, 28, 28, 64, 3, 1, 2, 2)])
def test_chain7_dilated(N, C, H, W, K, R, stride, pad, dil):
    print("chain7 dilated %s" % ((N, C, H, W, K, R, stride, pad, dil),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=R, S=R)
    check_chain7(t, stride, pad, dil=dil)
    check_chain7(t, stride, pad, pool=False, dil=dil)
    check_chain7(t, stride, pad, relu=False, pool=False, bias=False, affine=False, dil=dil)


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad", [
    (2, 8, 14, 14, 64, 3, 1, 1),      # width 14: two-float staging
    (1, 16, 7, 7, 128, 3, 1, 1),      # width 7: scalar staging
    (2, 8, 10, 30, 64, 3, 1, 1),
    (1, 12, 9, 5, 64, 3, 1, 1),
    (2, 32, 8, 8, 64, 1, 1, 0),       # 1x1: 16 channels per chunk
    (1, 64, 6, 10, 128, 1, 1, 0),
    (1, 48, 7, 7, 64, 1, 1, 0),
    (2, 8, 28, 28, 64, 3, 2, 1),      # stride 2, pipelined with four slots per thread
    (1, 8, 6, 120, 64, 3, 1, 1),
    (3, 256, 14, 14, 64, 3, 1, 1),
    (1, 8, 16, 16, 72, 3, 1, 1),      # output channels not a multiple of 64
    (1, 16, 8, 8, 200, 1, 1, 0),
    (2, 4, 14, 14, 1, 3, 1, 1)])
def test_chain7_pipelined_staging_modes(N, C, H, W, K, R, stride, pad):
    print("chain7 modes %s" % ((N, C, H, W, K, R, stride, pad),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=R, S=R)
    _, name = check_chain7(t, stride, pad, pool=False)
    assert "pipelined" in name or (R == 1 and name.startswith("conv1x1_stream"))
    _, name = check_chain7(t, stride, pad)
    assert "pipelined" in name
    check_chain7(t, stride, pad, relu=False, pool=False, bias=False, affine=False)


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad,dil", [
    (1, 8, 20, 72, 64, 3, 1, 1, 1),       # 8-column tiles divide the width
    (2, 4, 13, 77, 70, 3, 1, 1, 1),       # ragged rows, columns and output channels
    (1, 8, 9, 130, 64, 3, 2, 1, 1),       # stride 2
    (1, 3, 11, 99, 8, 5, 3, 2, 1),        # 5x5, stride 3
    (1, 3, 30, 230, 16, 7, 2, 3, 1),      # first-layer shape: 7x7 stride 2
    (1, 5, 12, 81, 12, 3, 1, 2, 2),       # dilated
    (1, 4, 3, 1500, 8, 3, 1, 1, 1),       # far wider than whole staged rows would allow
    (1, 6, 70, 66, 9, 3, 1, 0, 1)])       # no padding
def test_conv_window_geometry_without_pooling(N, C, H, W, K, R, stride, pad, dil):
    # images wider than 64 columns are tiled in 8 x 8 output windows also when nothing is pooled
    print("conv window %s" % ((N, C, H, W, K, R, stride, pad, dil),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=R, S=R)
    _, name = check_chain7(t, stride, pad, pool=False, dil=dil)
    assert "window" in name
    check_chain7(t, stride, pad, relu=False, pool=False, bias=False, affine=False, dil=dil)


def test_conv_planes_above_2_to_24_pixels():
    # the epilogue stores through a 32-bit buffer descriptor per 32 output channels; a plane of more than 2^24 pixels
    # does not fit one and takes plain stores (two output channels: the ragged-channel test of that path too)
    print("conv 5 x 4100 x 4100 -> 2", flush=True)
    t = datagen.make(7, N=1, C=5, H=4100, W=4100, K=2, R=3, S=3)
    _, name = check_chain7(t, 1, 1, pool=False)
    assert name == "conv2d_nchw_mfma<3x3,general,window>"


@pytest.mark.parametrize("N,C,H,W,K", [
    (32, 64, 56, 56, 64),        # a bottleneck's 1x1 at full size: memory-bound
    (32, 24, 56, 56, 144),       # a MobileNetV2 expansion: one chunk of 32 channels, 8 of them padding
    (4, 96, 14, 14, 64),         # three chunks of 32 channels
    (1, 8, 5, 7, 3),             # one ragged block, three output channels
    (3, 72, 9, 11, 130),         # chunks of 32 with a padded tail; two slices of output channels, the last ragged
    (5, 16, 3, 3, 32),           # 45 pixels: blocks span images
    (2, 40, 20, 20, 256)])       # 128 output channels per work-group, twice
def test_conv1x1_streaming_kernel(N, C, H, W, K):
    print("conv1x1 %s" % ((N, C, H, W, K),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=1, S=1)
    _, name = check_chain7(t, 1, 0, pool=False)
    assert name.startswith("conv1x1_stream")
    check_chain7(t, 1, 0, relu=False, pool=False, bias=False, affine=False)
    # relu6 and the bare bias
    want, Dn = ref.conv2d_nchw_bias(t["in"], t["wt"] * 16.0, t["bias"], 1, 0, want_norm=True)
    out = torch.full(want.shape, float("nan"), device="cuda")
    hpct.conv_block(dev(t["in"]), dev(t["wt"] * 16.0), dev(t["bias"]), None, None, out, 1, 0, "relu6", False)
    assert show("1x1 relu6", compare.contraction(host(out), ref.relu6(want), Dn))
    # pooled 1x1 convs stay with the tile kernel
    if H >= 2 and W >= 2:
        _, name = check_chain7(t, 1, 0)
        assert name.startswith("conv2d_nchw_mfma<1x1")


@pytest.mark.parametrize("N,C,H,W,K", [
    (2, 3, 30, 224, 64),         # the first layer of a VGG: two segments, the second of 96 pixels
    (3, 3, 7, 128, 32),          # one full segment, an odd number of rows
    (1, 1, 28, 100, 32),         # a grey image; a ragged segment
    (2, 2, 5, 384, 96),          # three segments, three blocks of output channels
    (1, 4, 1, 112, 64),          # a single row: nothing above or below it
    (5, 3, 9, 104, 160)])
def test_conv3x3_few_input_channels(N, C, H, W, K):
    print("conv fewc %s" % ((N, C, H, W, K),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=3, S=3)
    _, name = check_chain7(t, 1, 1, pool=False)
    assert name == "conv3x3_fewc"
    check_chain7(t, 1, 1, relu=False, pool=False, bias=False, affine=False)
    want, Dn = ref.conv2d_nchw_bias(t["in"], t["wt"] * 16.0, t["bias"], 1, 1, want_norm=True)
    out = torch.full(want.shape, float("nan"), device="cuda")
    hpct.conv_block(dev(t["in"]), dev(t["wt"] * 16.0), dev(t["bias"]), None, None, out, 1, 1, "relu6", False)
    assert show("fewc relu6", compare.contraction(host(out), ref.relu6(want), Dn))
    # pooled, strided or unpadded: the general kernel
    if H >= 3:
        _, name = check_chain7(t, 1, 0, pool=False)
        assert name.startswith("conv2d_nchw_mfma<3x3")


@pytest.mark.parametrize("N,C,H,W,K", [(2, 3, 30, 224, 32), (1, 3, 17, 256, 32), (2, 1, 9, 232, 32), (1, 4, 8, 200, 64), (1, 3, 2, 480, 96),
                                       (3, 2, 1, 224, 64)])
def test_conv3x3_stride2_few_input_channels(N, C, H, W, K):
    # a MobileNet's first convolution: odd and even heights, one and two segments, a single row
    print("conv 3x3/2 fewc %s" % ((N, C, H, W, K),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=3, S=3)
    _, name = check_chain7(t, 2, 1, pool=False)
    assert name == "conv3x3_fewc<stride2>"
    check_chain7(t, 2, 1, relu=False, pool=False, bias=False, affine=False)


@pytest.mark.parametrize("N,C,H,W,K", [
    (2, 3, 30, 224, 64),         # a ResNet's first convolution: 112 output pixels per row, one segment
    (1, 3, 17, 256, 32),         # a full segment, an odd number of input rows
    (2, 1, 9, 232, 32),          # a grey image, 116 output pixels
    (1, 2, 8, 200, 64),
    (1, 3, 2, 480, 96),          # two segments, one output row
    (3, 3, 11, 224, 128)])
def test_conv7x7_stride2_few_input_channels(N, C, H, W, K):
    print("conv 7x7/2 fewc %s" % ((N, C, H, W, K),), flush=True)
    t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=7, S=7)
    _, name = check_chain7(t, 2, 3, pool=False)
    assert name == "conv7x7s2_fewc"
    check_chain7(t, 2, 3, relu=False, pool=False, bias=False, affine=False)
    # other strides and paddings: the general kernel
    if H + 4 >= 7:
        _, name = check_chain7(t, 2, 2, pool=False)
        assert name.startswith("conv2d_nchw_mfma<7x7")


def test_chain7_pool_takes_the_maximum_not_a_sum_or_a_corner():
    # identity 1x1 conv: the block is max pooling of the input, exactly
    X = datagen.gen_normal(11, (2, 4, 10, 66), 0.0, 1.0)
    wt = np.zeros((4, 4, 1, 1), np.float32)
    for k in range(4):
        wt[k, k, 0, 0] = 1.0
    out = torch.full((2, 4, 5, 33), float("nan"), device="cuda")
    hpct.conv_block(dev(X), dev(wt), None, None, None, out, stride=1, pad=0, relu=False, pool=True)
    want = X.reshape(2, 4, 5, 2, 33, 2).max(axis=(3, 5))
    assert np.array_equal(host(out), want)


# ------------------------------------------------------------------- chain 5
def run_chain5(t, scale=0.125, causal=False):
    Q, K, V = dev(t["Q"]), dev(t["K"]), dev(t["V"])
    out = torch.full(tuple(Q.shape), float("nan"), device="cuda")
    hpct.attention(Q, K, V, out, scale=scale, causal=causal)
    return host(out)


def test_chain5_full_size():
    t = datagen.make(5)
    want, Dn = ref.chain5(t["Q"], t["K"], t["V"], 0.125)
    got = run_chain5(t)
    assert show("chain5 16x2048x64", compare.contraction(got, want, Dn))
    assert np.max(np.abs(got - want) / Dn) < 1e-4
    got2 = run_chain5(t)
    assert np.array_equal(got.view(np.uint32), got2.view(np.uint32))


@pytest.mark.parametrize("B,L,Lk", [(1, 1, 1), (2, 5, 3), (1, 32, 32), (3, 33, 31), (2, 100, 64), (1, 128, 65),
                                    (2, 130, 97), (1, 200, 300), (1, 64, 1000)])
def test_chain5_ragged_shapes(B, L, Lk):
    print("chain5 B=%d L=%d Lk=%d" % (B, L, Lk), flush=True)
    t = datagen.make(5, B=B, L=L, Lk=Lk)
    for scale in (0.125, 1.0):
        want, Dn = ref.chain5(t["Q"], t["K"], t["V"], scale)
        assert show("scale %g" % scale, compare.contraction(run_chain5(t, scale), want, Dn))


def test_causal_attention_full_size():
    t = datagen.make(5)
    want, Dn = ref.attention(t["Q"], t["K"], t["V"], 0.125, want_norm=True, causal=True)
    got = run_chain5(t, causal=True)
    assert show("causal 16x2048x64", compare.contraction(got, want, Dn))
    assert np.max(np.abs(got - want) / Dn) < 1e-4
    # row 0 of every batch is V[0] exactly (a single key: p = 1)
    assert np.array_equal(got[:, 0], t["V"][:, 0])
    assert np.array_equal(got.view(np.uint32), run_chain5(t, causal=True).view(np.uint32))


@pytest.mark.parametrize("B,L,Lk", [(1, 1, 1), (2, 5, 3), (1, 32, 32), (3, 33, 31), (2, 100, 64), (1, 128, 65),
                                    (2, 130, 97), (1, 200, 300), (1, 64, 1000), (1, 300, 40), (2, 257, 257),
                                    (1, 192, 192), (3, 320, 320), (1, 65, 129), (2, 449, 450)])
def test_causal_attention_ragged_shapes(B, L, Lk):
    print("causal B=%d L=%d Lk=%d" % (B, L, Lk), flush=True)
    t = datagen.make(5, B=B, L=L, Lk=Lk)
    for scale in (0.125, 1.0):
        want, Dn = ref.attention(t["Q"], t["K"], t["V"], scale, want_norm=True, causal=True)
        assert show("scale %g" % scale, compare.contraction(run_chain5(t, scale, causal=True), want, Dn))


@pytest.mark.parametrize("D", [32, 128])
@pytest.mark.parametrize("B,L,Lk", [(1, 1, 1), (2, 70, 45), (1, 130, 257), (2, 384, 384), (1, 1024, 1024)])
def test_attention_other_head_dims(D, B, L, Lk):
    print("attention D=%d B=%d L=%d Lk=%d" % (D, B, L, Lk), flush=True)
    t = datagen.make(5, B=B, L=L, Lk=Lk, D=D)
    scale = 1.0 / np.sqrt(D)
    for causal in (False, True):
        want, Dn = ref.attention(t["Q"], t["K"], t["V"], scale, want_norm=True, causal=causal)
        got = run_chain5(t, scale, causal=causal)
        assert show("causal" if causal else "plain", compare.contraction(got, want, Dn))


@pytest.mark.parametrize("D,B,L,Lk,causal", [(64, 1, 8192, 8192, False), (64, 1, 8192, 8192, True),
                                             (128, 1, 8192, 8192, False), (128, 1, 8192, 8192, True),
                                             (64, 1, 4096, 6000, False), (64, 1, 4096, 6000, True),
                                             (128, 1, 3000, 5001, False), (32, 2, 4099, 4099, True)])
def test_attention_long_sequences(D, B, L, Lk, causal):
    # sequences well beyond the 2048 of the fifth workload: many more key blocks per query (the running maximum and
    # sum are rescaled over up to 128 blocks), query blocks beyond one XCD's share of a batch, Lq != Lk
    print("long attention D=%d B=%d L=%d Lk=%d causal=%r" % (D, B, L, Lk, causal), flush=True)
    t = datagen.make(5, B=B, L=L, Lk=Lk, D=D)
    scale = 1.0 / np.sqrt(D)
    want, Dn = ref.attention(t["Q"], t["K"], t["V"], scale, want_norm=True, causal=causal)
    got = run_chain5(t, scale, causal=causal)
    assert show("long %s" % ("causal" if causal else "plain"), compare.contraction(got, want, Dn))
    assert np.max(np.abs(got - want) / Dn) < 1e-4
    if causal:   # query 0 sees key 0 only
        assert np.array_equal(got[:, 0], t["V"][:, 0])


def test_attention_large_scores_do_not_overflow():
    t = datagen.make(5, B=1, L=40, Lk=70)
    t["Q"] = (t["Q"] * 30).astype(np.float32)  # scores of order +-2000: needs the running max
    want, Dn = ref.chain5(t["Q"], t["K"], t["V"], 1.0)
    got = run_chain5(t, 1.0)
    assert np.all(np.isfinite(got))
    assert show("peaked softmax", compare.contraction(got, want, Dn, tol=2e-3))


# ------------------------------------------------------------------ launches
def test_launch_on_a_side_stream():
    t = datagen.make(3, M=64, N=512)
    X, g, b = dev(t["X"]), dev(t["gamma"]), dev(t["beta"])
    out = torch.full((64, 512), float("nan"), device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        hpct.layernorm_gelu(X, g, b, out)
    s.synchronize()
    assert compare.pointwise(out.cpu().numpy(), ref.chain3(t["X"], t["gamma"], t["beta"], 1e-5))


# ---------------------------------------------------------- layout transform
def _layout_case(base_shape, make_view):
    """base tensor of base_shape -> strided torch view -> library copy vs the CPU checker, bit for bit."""
    n = int(np.prod(base_shape))
    base = datagen.gen_normal(4242, (n,), 0.0, 1.0)
    tb = dev(base).reshape(base_shape)
    view = make_view(tb)
    out = torch.full(tuple(view.shape), float("nan"), device="cuda")
    hpct.layout_transform(view, out)
    off = (view.data_ptr() - tb.data_ptr()) // 4
    want = ref.layout_copy(base[off:], tuple(view.shape), tuple(view.stride()))
    got = host(out)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (base_shape, tuple(view.shape), tuple(view.stride()))


def test_layout_nchw_to_nhwc_and_back_full_size():
    _layout_case((32, 64, 56, 56), lambda t: t.permute(0, 2, 3, 1))   # NCHW -> NHWC
    _layout_case((32, 56, 56, 64), lambda t: t.permute(0, 3, 1, 2))   # NHWC -> NCHW


@pytest.mark.parametrize("shape,perm", [((100, 200), (1, 0)), ((1, 7), (1, 0)), ((65, 63), (1, 0)), ((3, 70, 130), (0, 2, 1)),
                                        ((2, 3, 5, 7), (0, 2, 3, 1)), ((2, 3, 5, 7), (3, 2, 1, 0)), ((4, 8, 16, 64), (0, 2, 1, 3)),
                                        ((2, 2, 2, 3, 4, 5), (5, 0, 3, 1, 4, 2)), ((6, 128), (0, 1))])
def test_layout_permutations(shape, perm):
    print("layout permute", shape, perm, flush=True)
    _layout_case(shape, lambda t: t.permute(*perm))


def test_layout_slices_and_broadcasts():
    _layout_case((4, 6, 8, 12), lambda t: t[:, ::2, 1:7, :])          # strided window, inner contiguous
    _layout_case((4, 6, 8, 12), lambda t: t[:, :, :, 4:8])            # inner slice: aligned vector path
    _layout_case((4, 6, 8, 12), lambda t: t[:, :, :, 1:10:3])         # inner stride 3: scalar gather
    _layout_case((1, 64), lambda t: t.expand(33, 64))                 # broadcast rows (stride 0)
    _layout_case((64, 1), lambda t: t.expand(64, 20))                 # broadcast inner (stride 0)
    _layout_case((5, 7, 9), lambda t: t)                              # contiguous, odd size


# --------------------------------------------------- reductions over one axis
def check_reduce(view, axis, tag=""):
    """view: a torch view on the GPU; compares all six reductions over `axis` with the checker."""
    base = view._base if view._base is not None else view
    hb = host(base).reshape(-1)
    off = view.storage_offset() - base.storage_offset()
    shape, stride = tuple(view.shape), tuple(view.stride())
    oshape = tuple(n for k, n in enumerate(shape) if k != axis) or (1,)
    names = set()
    for op in ("sum", "mean"):
        out = torch.full(oshape, float("nan"), device="cuda")
        plan, ins = hpct.reduce_axis_plan(view, out, axis, op)
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda") if plan.workspace_bytes else None
        plan.launch(ins, [out], workspace=ws)
        names.add(plan.kernel_name)
        want, mag = ref.reduce_axis(hb[off:], shape, stride, axis, op, want_abs=True)
        got = host(out).reshape(want.shape)
        # a sum of R fp32 terms: error far inside the contraction bound relative to the sum of magnitudes
        assert show("%s %s axis %d" % (tag, op, axis), compare.contraction(got, want, mag + 1e-300))
        assert np.all(np.abs(got - want) <= 1e-5 * mag + 1e-30)
    for op in ("argmax", "argmin"):
        out = torch.full(oshape, -7, device="cuda", dtype=torch.int32)
        plan, ins = hpct.reduce_axis_plan(view, out, axis, op)
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda") if plan.workspace_bytes else None
        plan.launch(ins, [out], workspace=ws)
        names.add(plan.kernel_name)
        want = ref.reduce_axis(hb[off:], shape, stride, axis, op)
        assert np.array_equal(host(out).reshape(want.shape).astype(np.int64), want), (tag, op, axis)
    for op in ("max", "min"):   # a selection: exact
        out = torch.full(oshape, float("nan"), device="cuda")
        plan, ins = hpct.reduce_axis_plan(view, out, axis, op)
        ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda") if plan.workspace_bytes else None
        plan.launch(ins, [out], workspace=ws)
        names.add(plan.kernel_name)
        want = ref.reduce_axis(hb[off:], shape, stride, axis, op)
        assert np.array_equal(host(out).reshape(want.shape).astype(np.float64), want), (tag, op, axis)
    return names


def test_reduce_full_size_rows_cols_channels():
    X = dev(datagen.make(3)["X"])                       # [8192, 4096]
    assert check_reduce(X, 1, "8192x4096") == {"reduce_rows<group>"}
    assert all(n.startswith("reduce_cols") for n in check_reduce(X, 0, "8192x4096"))
    T = dev(datagen.make(2)["X"])                       # [32, 64, 56, 56]
    assert check_reduce(T, 1, "nchw channels") == {"reduce_cols<scalar>"}
    check_reduce(T, 0, "nchw batch")
    check_reduce(T, 3, "nchw w")
    check_reduce(T, 2, "nchw h")
    # determinism
    a = torch.empty(4096, device="cuda"); b = torch.empty(4096, device="cuda")
    plan, _ = hpct.reduce_axis_plan(X, a, 0, "sum")
    assert plan.kernel_name == "reduce_cols<vec4,split>" and plan.workspace_bytes > 0
    ws = torch.empty(plan.workspace_bytes // 4, device="cuda")
    hpct.reduce_axis(X, a, 0, "sum", ws); hpct.reduce_axis(X, b, 0, "sum", ws)
    assert np.array_equal(host(a).view(np.uint32), host(b).view(np.uint32))


@pytest.mark.parametrize("shape", [(1,), (7,), (1000,), (70001,), (3, 5), (33, 65), (257, 130), (5, 1, 9),
                                   (4, 6, 10, 3), (2, 3, 4, 5, 6), (2, 2, 3, 2, 3, 4), (64, 2048), (3, 40000),
                                   (5000, 260), (3000, 7), (2, 1500, 33)])
def test_reduce_ragged_contiguous(shape):
    print("reduce", shape, flush=True)
    n = int(np.prod(shape))
    x = dev(datagen.gen_normal(77, (n,), 0.0, 1.0)).view(*shape)
    for axis in range(len(shape)):
        check_reduce(x, axis, str(shape))


def test_reduce_strided_views_ties_and_offsets():
    base = dev(datagen.gen_normal(78, (6, 40, 50), 0.0, 1.0))
    check_reduce(base.permute(2, 0, 1), 0, "permuted")
    check_reduce(base.permute(2, 0, 1), 1, "permuted")
    check_reduce(base.permute(2, 0, 1), 2, "permuted")
    check_reduce(base[:, 3:33, 1:50:2], 1, "sliced")
    check_reduce(base[:, 3:33, 1:50:2], 2, "sliced")          # strided inner dimension: gather / rows scalar
    check_reduce(base[1:, :, 3:], 0, "offset view")
    check_reduce(base[0, 0].expand(9, 50), 0, "broadcast")     # stride 0 along the reduced axis: all ties -> index 0
    check_reduce(base[0, 0].expand(9, 50), 1, "broadcast")
    # many exact ties: small integers
    q = dev((datagen.gen_uniform(79, (300, 257), 0.0, 4.0)).astype(np.int32).astype(np.float32))
    check_reduce(q, 0, "ties")
    check_reduce(q, 1, "ties")
    check_reduce(q.t(), 0, "ties transposed")


# ------------------------------------------------- elementwise on strided views
def check_eltwise(a_view, b_view, tag):
    def flat(view):
        base = view._base if view._base is not None else view
        return host(base).reshape(-1)[view.storage_offset() - base.storage_offset():]
    shape = tuple(a_view.shape)
    sa, sb = tuple(a_view.stride()), tuple(b_view.stride())
    names = set()
    for op in ("add", "mul"):
        for relu in (False, True):
            out = torch.full(shape, float("nan"), device="cuda")
            plan, ins = hpct.eltwise_plan(a_view, b_view, out, op, relu)
            plan.launch(ins, [out])
            names.add(plan.kernel_name)
            want = ref.eltwise_binary(flat(a_view), flat(b_view), shape, sa, sb, op, relu)
            # one fp32 rounding of an exactly known sum or product
            assert np.array_equal(host(out), want.astype(np.float32)), (tag, op, relu)
    for op in ("sub", "div"):
        # a difference is exact in fp64; a correctly rounded fp32 quotient equals the fp64 quotient rounded once more
        # (53 >= 2 * 24 + 2 bits)
        out = torch.full(shape, float("nan"), device="cuda")
        plan, ins = hpct.eltwise_map_plan(a_view, out, ("relu",), op, b_view)
        plan.launch(ins, [out])
        want = ref.eltwise_map(flat(a_view), shape, sa, ("relu",), op, flat(b_view), sb)
        with np.errstate(over="ignore"):
            assert np.array_equal(host(out), want.astype(np.float32)), (tag, op)
    return names


def view_flat(view):
    base = view._base if view._base is not None else view
    return host(base).reshape(-1)[view.storage_offset() - base.storage_offset():]


# (chains are kept well conditioned: a step such as cos after exp would turn the fp32 rounding of a large
# intermediate into an absolute error of the same size, which no fp32 evaluation can avoid)
UNARY_CHAINS = [("sin",), ("cos",), ("exp",), ("tanh",), ("sigmoid",), ("gelu",), ("sin", "scale"), ("relu", "sqrt"),
                ("tanh", "scale", "exp", "sqrt"), ("sin", "cos", "tanh", "sigmoid", "exp", "scale", "gelu", "relu")]


def check_unary(a_view, tag, chains=UNARY_CHAINS, scale=1.7):
    shape, sa = tuple(a_view.shape), tuple(a_view.stride())
    names = set()
    for steps in chains:
        out = torch.full(shape, float("nan"), device="cuda")
        plan, ins = hpct.eltwise_map_plan(a_view, out, steps, scale=scale)
        plan.launch(ins, [out])
        names.add(plan.kernel_name)
        want = ref.eltwise_map(view_flat(a_view), shape, sa, steps, scale=scale)
        assert show("%s %s" % (tag, "+".join(steps)), compare.pointwise(host(out), want))
    return names


def test_eltwise_unary_full_size():
    X = dev(datagen.make(3)["X"])                      # N(0,1), 8192 x 4096
    assert check_unary(X, "full", [("sin",), ("tanh", "scale", "exp", "sqrt")]) == {"eltwise_unary<vec4>"}
    # sqrt alone is correctly rounded: equal to the fp64 root rounded once more
    P = dev(datagen.gen_uniform(97, (8192, 4096), 0.0, 100.0))
    out = torch.full((8192, 4096), float("nan"), device="cuda")
    hpct.eltwise_map(P, out, ("sqrt",))
    assert np.array_equal(host(out), ref.eltwise_map(host(P), (8192, 4096), (4096, 1), ("sqrt",)).astype(np.float32))


def test_eltwise_unary_views_and_ranges():
    a = dev(datagen.gen_normal(94, (6, 10, 12), 0.0, 2.0))
    assert check_unary(a, "contiguous") == {"eltwise_unary<vec4>"}
    assert check_unary(a.permute(2, 0, 1), "permuted") == {"eltwise_unary<scalar>"}
    check_unary(a[:, 1:9, 3:11], "offset slice")
    check_unary(a[1, 2, 5:12], "vector")
    check_unary(a[:, :, 0:1].expand(6, 10, 12), "broadcast")
    check_unary(dev(np.full((1,), 0.5, np.float32)), "single element")
    # arguments far outside one period (the argument reduction must hold), large exponents, saturated tanh / sigmoid
    big = dev(datagen.gen_uniform(95, (64, 100), -1.0e4, 1.0e4))
    check_unary(big, "large angles", [("sin",), ("cos",)])
    wide = dev(datagen.gen_uniform(96, (64, 100), -80.0, 80.0))
    check_unary(wide, "wide", [("exp",), ("tanh",), ("sigmoid",), ("gelu",)])


def test_eltwise_further_unary_steps():
    a = dev(datagen.gen_normal(93, (7, 12, 20), 0.0, 3.0))
    flat = host(a).reshape(-1)
    # |x|, -x and x*x are exact (the product of two fp32 values rounded once)
    for steps in (("abs",), ("neg",), ("square",), ("neg", "abs", "neg")):
        out = torch.full(tuple(a.shape), float("nan"), device="cuda")
        hpct.eltwise_map(a, out, steps)
        want = ref.eltwise_map(flat, tuple(a.shape), tuple(a.stride()), steps)
        assert np.array_equal(host(out), want.astype(np.float32)), steps
    more = [("silu",), ("hardswish",), ("abs", "log"), ("square", "log"), ("silu", "scale", "hardswish"), ("abs", "sqrt", "silu", "neg", "exp")]
    assert check_unary(a, "more", more) == {"eltwise_unary<vec4>"}
    check_unary(a.permute(2, 0, 1), "more, permuted", more)
    wide = dev(datagen.gen_uniform(89, (64, 100), -80.0, 80.0))
    check_unary(wide, "wide", [("silu",), ("hardswish",)])
    tiny = dev(datagen.gen_uniform(88, (64, 100), 1e-30, 1e30))
    check_unary(tiny, "log over 60 decades", [("log",)])
    # a binary op in front
    b = dev(datagen.gen_uniform(87, (20,), 0.5, 2.0)).expand(7, 12, 20)
    out = torch.full((7, 12, 20), float("nan"), device="cuda")
    hpct.eltwise_map(a, out, ("hardswish", "square"), "mul", b)
    want = ref.eltwise_map(flat, (7, 12, 20), (240, 20, 1), ("hardswish", "square"), "mul", view_flat(b), (0, 0, 1))
    assert show("mul + hardswish + square", compare.pointwise(host(out), want))


def test_eltwise_binary_then_steps():
    a = dev(datagen.gen_uniform(98, (33, 40), 0.5, 4.0))
    b = dev(datagen.gen_uniform(99, (40,), 0.5, 2.0)).expand(33, 40)
    for op, steps in (("div", ("sqrt", "sin")), ("sub", ("scale", "sigmoid")), ("mul", ("tanh", "relu")), ("add", ("gelu", "exp"))):
        out = torch.full((33, 40), float("nan"), device="cuda")
        hpct.eltwise_map(a, out, steps, op, b, scale=-0.7)
        want = ref.eltwise_map(host(a), (33, 40), (40, 1), steps, op, view_flat(b), (0, 1), scale=-0.7)
        assert show("%s %s" % (op, "+".join(steps)), compare.pointwise(host(out), want))


def test_eltwise_full_size_bias_row_and_same_shape():
    X = dev(datagen.make(3)["X"])
    g = dev(datagen.make(3)["gamma"])
    assert check_eltwise(X, g.expand(8192, 4096), "bias row") == {"eltwise_binary<vec4>"}
    Y = dev(datagen.make(3, variant=1)["X"])
    assert check_eltwise(X, Y, "same shape") == {"eltwise_binary<vec4>"}


def test_eltwise_views():
    a = dev(datagen.gen_normal(91, (6, 10, 12), 0.0, 1.0))
    b = dev(datagen.gen_normal(92, (6, 10, 12), 0.0, 1.0))
    check_eltwise(a, b.permute(0, 2, 1).contiguous().permute(0, 2, 1), "b transposed in memory")
    check_eltwise(a.permute(2, 0, 1), b.permute(2, 0, 1), "both permuted")
    check_eltwise(a, b[:, :, 0:1].expand(6, 10, 12), "scalar per row")
    check_eltwise(a, b[0:1, 0:1, :].expand(6, 10, 12), "row")
    check_eltwise(a, b[:, 0:1, 0:1].expand(6, 10, 12), "scalar per slab")
    check_eltwise(a[:, 1:9, 3:11], b[:, 1:9, 2:10], "offset slices")
    check_eltwise(a[0, 0, :7], b[1, 2, 5:12], "vectors")
    v = dev(datagen.gen_normal(93, (2, 3, 2, 3, 2, 4), 0.0, 1.0))
    check_eltwise(v, v.permute(1, 0, 3, 2, 5, 4).contiguous().permute(1, 0, 3, 2, 5, 4), "6-D")
    one = dev(np.ones((1,), np.float32))
    check_eltwise(one, one, "single element")


# ---------------------------------------- transposed conv ("Conv-Trans")
def check_conv_transpose(N, C, H, W, K, R, stride, pad, dil=1, act=False, bias=True, affine=False, seed=0):
    x = datagen.gen_normal(500 + seed, (N, C, H, W), 0.0, 1.0)
    w = datagen.gen_normal(501 + seed, (C, K, R, R), 0.0, 1.0 / (R * np.sqrt(C)))
    b = datagen.gen_normal(502 + seed, (K,), 0.0, 0.5) if bias else None
    sc = datagen.gen_uniform(503 + seed, (K,), 0.5, 1.5) if affine else None
    sh = datagen.gen_normal(504 + seed, (K,), 0.0, 0.5) if affine else None
    want, Dn = ref.conv_transpose2d_nchw(x, w, b, stride, pad, want_norm=True, dil=dil)
    if affine:
        want, Dn = ref.scale_shift_ch(want, sc, sh), ref.scale_shift_ch(Dn, np.abs(sc), np.abs(sh))
    want = ref.relu6(want) if act == "relu6" else (ref.relu(want) if act else want)
    out = torch.full(want.shape, float("nan"), device="cuda")
    plan, ins = hpct.conv_transpose_plan(dev(x), dev(w), None if b is None else dev(b), None if sc is None else dev(sc),
                                         None if sh is None else dev(sh), out, stride, pad, act, dil)
    assert plan.workspace_bytes > 0
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda")
    plan.launch(ins, [out], workspace=ws)
    assert show("conv transpose %s" % plan.kernel_name, compare.contraction(host(out), want, Dn))
    return host(out), plan, ins, ws


def test_conv_transpose_full_size():
    # a decoder's 2x upsampling layer: 4x4 filter, stride 2, padding 1, [32,128,28,28] -> [32,64,56,56]
    got, plan, ins, ws = check_conv_transpose(32, 128, 28, 28, 64, 4 - 1, 2, 1, act="relu")   # 3x3: the filter sizes are odd
    out2 = torch.full(got.shape, float("nan"), device="cuda")
    plan.launch(ins, [out2], workspace=ws)
    assert np.array_equal(host(out2).view(np.uint32), got.view(np.uint32))
    with pytest.raises(hpct.HpctError):
        plan.launch(ins, [out2])                                    # the workspace is required


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad,dil", [
    (1, 1, 1, 1, 1, 1, 1, 0, 1), (2, 3, 5, 6, 4, 3, 1, 1, 1), (1, 8, 7, 9, 64, 3, 2, 1, 1), (2, 5, 6, 6, 7, 3, 2, 0, 1),
    (1, 4, 9, 5, 10, 5, 2, 2, 1), (1, 16, 8, 8, 130, 3, 3, 1, 1), (1, 6, 10, 12, 9, 3, 1, 2, 2), (2, 64, 14, 14, 64, 3, 2, 1, 1),
    (1, 8, 5, 5, 8, 1, 2, 0, 1), (1, 3, 4, 40, 5, 7, 2, 3, 1), (1, 2, 6, 6, 3, 3, 4, 2, 1)])
def test_conv_transpose_ragged_shapes(N, C, H, W, K, R, stride, pad, dil):
    print("conv transpose %s" % ((N, C, H, W, K, R, stride, pad, dil),), flush=True)
    check_conv_transpose(N, C, H, W, K, R, stride, pad, dil)
    check_conv_transpose(N, C, H, W, K, R, stride, pad, dil, act="relu6", affine=True, seed=1)
    check_conv_transpose(N, C, H, W, K, R, stride, pad, dil, act="relu", bias=False, seed=2)


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad", [(2, 16, 8, 8, 24, 1, 1, 0), (1, 64, 16, 16, 64, 1, 1, 0),   # -> the 1x1 streaming kernel
                                                     (2, 3, 16, 32, 32, 3, 1, 1), (2, 4, 12, 64, 64, 3, 1, 1),   # few input channels
                                                     (1, 2, 8, 224, 32, 3, 1, 1)])
def test_conv_transpose_routes_through_the_specialised_conv_kernels(N, C, H, W, K, R, stride, pad):
    # combinations that exist only through composition: the stride-1 conv that a transposed conv becomes may be taken
    # by the kernels for 1x1 filters or for few input channels; each must see the flipped / regrouped operands correctly
    print("conv transpose route %s" % ((N, C, H, W, K, R, stride, pad),), flush=True)
    got, plan, ins, ws = check_conv_transpose(N, C, H, W, K, R, stride, pad, act="relu", affine=True, seed=3)
    print("kernel", plan.kernel_name, flush=True)
    check_conv_transpose(N, C, H, W, K, R, stride, pad, bias=False, seed=4)


def test_conv_transpose_tiles_with_a_2x2_filter_of_ones():
    # stride = filter size would tile the output; with odd filters: a 1x1 filter of ones at stride 2 puts every input
    # on the even positions and zeros between them, exactly
    x = datagen.gen_normal(510, (2, 3, 5, 7), 0.0, 1.0)
    w = np.zeros((3, 3, 1, 1), np.float32)
    for c in range(3):
        w[c, c, 0, 0] = 1.0
    out = torch.full((2, 3, 9, 13), float("nan"), device="cuda")
    plan, ins = hpct.conv_transpose_plan(dev(x), dev(w), None, None, None, out, 2, 0)
    ws = torch.empty(plan.workspace_bytes // 4, device="cuda")
    plan.launch(ins, [out], workspace=ws)
    got = host(out)
    assert np.array_equal(got[:, :, ::2, ::2], x) and np.all(got[:, :, 1::2, :] == 0) and np.all(got[:, :, :, 1::2] == 0)


# ---------------------------------------- root-mean-square normalisation over the last dimension
@pytest.mark.parametrize("M,N", [(8192, 4096), (300, 1024), (64, 256), (33, 1001), (5, 8192), (3, 16384), (2, 20000), (7, 4), (1, 1), (40, 2052)])
def test_rmsnorm_rows(M, N):
    print("rmsnorm M=%d N=%d" % (M, N), flush=True)
    x = datagen.gen_normal(850, (M, N), 0.5, 2.0)
    g = datagen.gen_normal(851, (N,), 1.0, 0.2)
    for gamma in (g, None):
        out = torch.full((M, N), float("nan"), device="cuda")
        plan, ins = hpct.rmsnorm_plan(dev(x), None if gamma is None else dev(gamma), out, 1e-6)
        plan.launch(ins, [out])
        assert plan.kernel_name.startswith("rmsnorm_rows")
        assert show("rmsnorm %s" % plan.kernel_name, compare.pointwise(host(out), ref.rmsnorm_rows(x, gamma, 1e-6)))


# ---------------------------------------- group / instance normalisation of NCHW
def check_groupnorm(shape, groups, affine=True, relu=False, eps=1e-5, seed=0):
    x = datagen.gen_normal(800 + seed, shape, 0.5, 2.0)
    C_ = shape[1]
    ga = datagen.gen_normal(801 + seed, (C_,), 1.0, 0.2) if affine else None
    be = datagen.gen_normal(802 + seed, (C_,), 0.0, 0.3) if affine else None
    want = ref.groupnorm_nchw(x, groups, ga, be, eps)
    if relu:
        want = ref.relu(want)
    out = torch.full(shape, float("nan"), device="cuda")
    plan, ins = hpct.groupnorm_plan(dev(x), None if ga is None else dev(ga), None if be is None else dev(be), out, groups, eps, relu)
    plan.launch(ins, [out])
    assert show("groupnorm %s %s G=%d" % (plan.kernel_name, shape, groups), compare.pointwise(host(out), want))
    return plan.kernel_name


def test_groupnorm_full_size():
    assert check_groupnorm((32, 64, 56, 56), 8) == "groupnorm_rows<registers,1024>"
    assert check_groupnorm((4, 32, 112, 112), 4) == "groupnorm_rows<three passes>"
    assert check_groupnorm((32, 64, 56, 56), 32, relu=True) == "groupnorm_rows<registers>"
    assert check_groupnorm((32, 64, 56, 56), 64, affine=False) == "groupnorm_rows<registers>"      # instance normalisation


@pytest.mark.parametrize("shape,groups", [((2, 6, 7, 9), 3), ((1, 4, 1, 1), 2), ((3, 8, 2, 2), 8), ((2, 12, 5, 4), 1), ((1, 2, 64, 66), 1),
                                          ((2, 10, 6, 6), 5), ((1, 16, 32, 32), 2), ((2, 3, 3, 3), 3), ((1, 8, 30, 34), 4)])
def test_groupnorm_ragged_shapes(shape, groups):
    print("groupnorm %s G=%d" % (shape, groups), flush=True)
    check_groupnorm(shape, groups)
    check_groupnorm(shape, groups, affine=False, relu=True, eps=1e-3, seed=1)


# ---------------------------------------- max pooling with a window, a stride and padding
def check_maxpool(shape, k, stride, pad, seed=0, shift=-1.0):
    x = datagen.gen_normal(700 + seed, shape, shift, 1.0)       # mostly negative: a zero padding would win
    want = ref.maxpool2d(x, k, stride, pad)
    out = torch.full(want.shape, float("nan"), device="cuda")
    plan, ins = hpct.maxpool_plan(dev(x), out, k, stride, pad)
    plan.launch(ins, [out])
    got = host(out)
    assert np.array_equal(got.astype(np.float64), want), (shape, k, stride, pad, plan.kernel_name)   # a selection: exact
    return plan.kernel_name


def test_maxpool_full_size():
    # the pooling behind a ResNet's first convolution at batch 32, and a 3x3 / 1 / 1 pooling of an inception-style branch
    assert check_maxpool((32, 64, 112, 112), 3, 2, 1) == "maxpool3x3_rows<stride2>"
    assert check_maxpool((32, 64, 56, 56), 3, 1, 1) == "maxpool3x3_rows"
    assert check_maxpool((32, 64, 56, 56), 2, 2, 0) == "maxpool2_planes<vec4>"


@pytest.mark.parametrize("shape,k,stride,pad", [
    ((2, 3, 57, 112), 3, 2, 1), ((1, 2, 112, 104), 3, 2, 1), ((1, 4, 31, 96), 3, 2, 1), ((2, 2, 1, 104), 3, 2, 1), ((1, 2, 100, 336), 3, 2, 1),
    ((1, 3, 2, 400), 3, 2, 1), ((2, 3, 57, 56), 3, 1, 1), ((1, 5, 30, 112), 3, 1, 1), ((1, 2, 100, 48), 3, 1, 1), ((2, 2, 5, 52), 3, 1, 1),
    ((1, 2, 1, 56), 3, 1, 1), ((1, 3, 29, 168), 3, 1, 1),
    # narrow maps: few computing lanes, a second segment of one lane
    ((2, 3, 20, 24), 3, 2, 1), ((1, 2, 9, 16), 3, 1, 1), ((2, 2, 33, 28), 3, 1, 1), ((1, 2, 40, 120), 3, 2, 1), ((1, 3, 7, 12), 3, 1, 1),
    ((3, 5, 28, 32), 3, 2, 1)])
def test_maxpool_3x3_register_variant(shape, k, stride, pad):
    print("maxpool rows %s" % ((shape, k, stride, pad),), flush=True)
    assert check_maxpool(shape, k, stride, pad).startswith("maxpool3x3_rows")
    check_maxpool(shape, k, stride, pad, seed=1, shift=2.0)


@pytest.mark.parametrize("shape,k,stride,pad", [
    ((2, 3, 30, 30), 3, 2, 1), ((2, 3, 17, 23), 3, 2, 0), ((1, 3, 57, 57), 5, 3, 2), ((1, 1, 7, 7), 7, 1, 0), ((2, 3, 20, 110), 3, 2, 1),
    ((1, 2, 9, 9), 1, 2, 0), ((3, 1, 5, 5), 4, 4, 0), ((1, 2, 6, 40), 2, 1, 1), ((1, 1, 3, 3), 3, 1, 2), ((2, 2, 33, 31), 16, 5, 7),
    ((1, 1, 1, 1), 1, 1, 0), ((1, 2, 8, 8), 3, 1, 1), ((1, 2, 9, 20), 3, 2, 1)])
def test_maxpool_general_windows(shape, k, stride, pad):
    print("maxpool any %s" % ((shape, k, stride, pad),), flush=True)
    assert check_maxpool(shape, k, stride, pad) == "maxpool_any"


def check_avgpool(shape, k, stride, pad, seed=0):
    x = datagen.gen_normal(750 + seed, shape, 0.3, 1.0)
    want = ref.avgpool2d(x, k, stride, pad)
    mag = ref.avgpool2d(np.abs(x), k, stride, pad)
    out = torch.full(want.shape, float("nan"), device="cuda")
    plan, ins = hpct.avgpool_plan(dev(x), out, k, stride, pad)
    plan.launch(ins, [out])
    got = host(out)
    # a mean of k*k fp32 terms: error far inside the contraction bound relative to the mean of magnitudes
    assert show("avgpool %s %s" % (plan.kernel_name, (shape, k, stride, pad)), compare.contraction(got, want, mag + 1e-300))
    assert np.all(np.abs(got - want) <= 1e-5 * mag + 1e-30)
    return plan.kernel_name


def test_avgpool_windows():
    assert check_avgpool((32, 64, 112, 112), 3, 2, 1) == "avgpool3x3_rows<stride2>"
    assert check_avgpool((32, 64, 56, 56), 3, 1, 1) == "avgpool3x3_rows"
    assert check_avgpool((32, 64, 56, 56), 2, 2, 0) == "avgpool_any"
    for (shape, k, stride, pad) in [((2, 3, 57, 112), 3, 2, 1), ((1, 2, 100, 48), 3, 1, 1), ((2, 2, 5, 52), 3, 1, 1), ((1, 3, 2, 400), 3, 2, 1),
                                    ((2, 3, 20, 24), 3, 2, 1), ((2, 2, 33, 28), 3, 1, 1), ((1, 2, 40, 120), 3, 2, 1)]:
        assert check_avgpool(shape, k, stride, pad, seed=1).startswith("avgpool3x3_rows")
    for (shape, k, stride, pad) in [((2, 3, 30, 30), 3, 2, 1), ((1, 3, 57, 57), 5, 3, 2), ((1, 1, 7, 7), 7, 1, 0), ((2, 2, 33, 31), 16, 5, 7), ((1, 2, 6, 40), 2, 1, 1)]:
        assert check_avgpool(shape, k, stride, pad, seed=2) == "avgpool_any"


# ---------------------------------------- depthwise conv (MobileNetV2's depthwise layer) and relu6
def check_depthwise(N, C, H, W, R, stride, pad, dil=1, act="relu6", bias=True, affine=True, seed=0):
    x = datagen.gen_normal(300 + seed, (N, C, H, W), 0.0, 1.0)
    w = datagen.gen_normal(301 + seed, (C, 1, R, R), 0.0, 1.0 / R)
    b = datagen.gen_normal(302 + seed, (C,), 0.0, 0.5) if bias else None
    sc = datagen.gen_uniform(303 + seed, (C,), 0.5, 1.5) if affine else None
    sh = datagen.gen_normal(304 + seed, (C,), 0.0, 0.5) if affine else None
    want, Dn = ref.conv2d_nchw_grouped(x, w, b, stride, pad, C, want_norm=True, dil=dil)
    if affine:
        want = ref.scale_shift_ch(want, sc, sh)
        Dn = ref.scale_shift_ch(Dn, np.abs(sc), np.abs(sh))
    if act == "relu6":
        want = ref.relu6(want)
    elif act:
        want = ref.relu(want)
    out = torch.full(want.shape, float("nan"), device="cuda")
    plan, ins = hpct.depthwise_conv_plan(dev(x), dev(w), None if b is None else dev(b), None if sc is None else dev(sc),
                                         None if sh is None else dev(sh), out, stride, pad, act, dil)
    plan.launch(ins, [out])
    assert show("depthwise %s" % plan.kernel_name, compare.contraction(host(out), want, Dn))
    return host(out), plan


def test_depthwise_full_size():
    # the 3x3 depthwise layers of a MobileNetV2 at batch 32: 96 channels at 112 x 112 (stride 2) and 144 at 56 x 56
    got, plan = check_depthwise(32, 144, 56, 56, 3, 1, 1)
    assert plan.kernel_name == "dwconv3x3_rows"
    got, plan = check_depthwise(32, 96, 112, 112, 3, 2, 1)
    assert plan.kernel_name == "dwconv3x3_rows<stride2>"
    got, plan = check_depthwise(32, 192, 28, 28, 3, 1, 1)
    assert plan.kernel_name == "dwconv_planes<3x3>"


@pytest.mark.parametrize("N,C,H,W,stride", [(2, 3, 57, 56, 1), (1, 5, 30, 112, 1), (1, 2, 100, 48, 1), (2, 2, 5, 52, 1), (1, 2, 1, 56, 1),
                                            (1, 3, 29, 168, 1), (3, 2, 56, 56, 1), (1, 2, 113, 224, 1), (300, 40, 3, 56, 1),
                                            (2, 3, 57, 112, 2), (1, 2, 112, 112, 2), (1, 4, 31, 96, 2), (2, 2, 1, 104, 2), (1, 2, 100, 336, 2),
                                            (1, 3, 2, 400, 2), (70, 30, 9, 112, 2)])
def test_depthwise_3x3_register_variant(N, C, H, W, stride):
    # bands of 16 output rows that do not divide the image, last segments of fewer than 56 columns, odd and even heights at stride 2
    print("depthwise rows %s" % ((N, C, H, W, stride),), flush=True)
    got, plan = check_depthwise(N, C, H, W, 3, stride, 1)
    assert plan.kernel_name == ("dwconv3x3_rows<stride2>" if stride == 2 else "dwconv3x3_rows")
    check_depthwise(N, C, H, W, 3, stride, 1, act=None, bias=False, affine=False, seed=1)
    check_depthwise(N, C, H, W, 3, stride, 1, act="relu", affine=False, seed=2)


@pytest.mark.parametrize("N,C,H,W,R,stride,pad,dil", [
    (1, 1, 1, 1, 1, 1, 0, 1), (2, 3, 7, 9, 3, 1, 1, 1), (1, 5, 13, 5, 3, 2, 1, 1), (2, 4, 10, 30, 5, 1, 2, 1),
    (1, 6, 33, 41, 7, 2, 3, 1), (1, 3, 17, 23, 3, 1, 2, 2), (1, 2, 40, 40, 3, 3, 0, 1), (1, 7, 9, 200, 3, 1, 1, 1),
    (1, 2, 300, 20, 5, 1, 2, 3), (3, 8, 28, 28, 3, 1, 1, 1), (1, 4, 6, 6, 1, 2, 0, 1), (1, 2, 12, 12, 3, 1, 0, 4)])
def test_depthwise_ragged_shapes(N, C, H, W, R, stride, pad, dil):
    print("depthwise %s" % ((N, C, H, W, R, stride, pad, dil),), flush=True)
    check_depthwise(N, C, H, W, R, stride, pad, dil)
    check_depthwise(N, C, H, W, R, stride, pad, dil, act="relu", affine=False, seed=1)
    check_depthwise(N, C, H, W, R, stride, pad, dil, act=False, bias=False, affine=False, seed=2)


def test_depthwise_does_not_mix_channels():
    # centre-tap delta filters scaled per channel: out[n, c] = s[c] * in[n, c] exactly
    x = datagen.gen_normal(310, (2, 9, 12, 20), 0.0, 1.0)
    s = datagen.gen_normal(311, (9,), 0.0, 1.0)
    w = np.zeros((9, 1, 3, 3), np.float32); w[:, 0, 1, 1] = s
    out = torch.full((2, 9, 12, 20), float("nan"), device="cuda")
    hpct.depthwise_conv(dev(x), dev(w), None, None, None, out, 1, 1, relu=False)
    assert np.array_equal(host(out), x * s[None, :, None, None])


def test_relu6_in_the_dense_conv_and_as_a_step():
    t = datagen.make(7, N=2, C=8, H=14, W=14, K=64, R=3, S=3)
    x, w, b = t["in"], t["wt"] * 8.0, t["bias"]              # large weights: some outputs pass 6
    for pool in (False, True):
        Z, Dn = ref.conv2d_nchw_bias(x, w, b, 1, 1, want_norm=True)
        want = ref.relu6(Z)
        if pool:
            want, Dn = ref.maxpool2x2(want), ref.maxpool2x2(Dn)
        out = torch.full(want.shape, float("nan"), device="cuda")
        plan, ins = hpct.conv_block_plan(dev(x), dev(w), dev(b), None, None, out, 1, 1, "relu6", pool)
        plan.launch(ins, [out])
        got = host(out)
        assert show("conv relu6", compare.contraction(got, want, Dn))
        assert got.max() == 6.0 and got.min() == 0.0
    a = dev(datagen.gen_normal(312, (33, 40), 0.0, 5.0))
    out = torch.full((33, 40), float("nan"), device="cuda")
    hpct.eltwise_map(a, out, ("relu6",))
    assert np.array_equal(host(out), ref.eltwise_map(host(a), (33, 40), (40, 1), ("relu6",)).astype(np.float32))


# ------------------------------------------------------- 2x2 max pooling alone
@pytest.mark.parametrize("shape", [(32, 64, 56, 56), (2, 3, 7, 9), (1, 1, 2, 2), (3, 5, 13, 16), (2, 2, 8, 6), (1, 4, 224, 224)])
def test_maxpool_alone(shape):
    X = datagen.gen_normal(55, shape, 0.0, 1.0)
    out = torch.full((shape[0], shape[1], shape[2] // 2, shape[3] // 2), float("nan"), device="cuda")
    hpct.maxpool2x2(dev(X), out)
    assert np.array_equal(host(out), ref.maxpool2x2(X.astype(np.float64)).astype(np.float32))


# ------------------------------------------------------------ seeded sweeps of random valid shapes
def _rng(seed):
    return np.random.default_rng(seed)


def test_sweep_gemm_shapes():
    r = _rng(20250610401)
    for case in range(40):
        # small, tile-sized and split-K-sized problems; K a multiple of 4 in half the cases (vector path)
        M = int(r.choice([1, 7, 16, 33, 64, 130, 257, 600, 1100]))
        N = int(r.choice([1, 5, 64, 100, 256, 300, 513, 1030]))
        K = int(r.choice([1, 3, 4, 8, 12, 16, 20, 36, 64, 100, 260, 1024, 2052]))
        wt = bool(r.integers(2))
        scale = None if r.integers(2) else float(r.choice([0.5, -1.25, 3.0]))
        print("sweep gemm %d: M=%d K=%d N=%d wt=%s scale=%s" % (case, M, K, N, wt, scale), flush=True)
        t = datagen.make(1, M=M, K=K, N=N)
        Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
        if scale is not None:
            Z, Dn = ref.scale_const(Z, scale), Dn * abs(float(np.float32(scale)))
        got, name = run_gemm(t, wt=wt, relu=True, scale=scale)
        assert show(name, compare.contraction(got, ref.relu(Z), Dn))


def test_sweep_conv_shapes():
    r = _rng(20250610402)
    for case in range(40):
        R = int(r.choice([1, 3, 3, 3, 5, 7]))
        stride = int(r.choice([1, 1, 2, 3]))
        dil = int(r.choice([1, 1, 1, 2]))
        pad = int(r.integers(0, (R - 1) * dil + 1))
        C = int(r.choice([1, 3, 4, 8, 16, 20, 32, 64]))
        K = int(r.choice([1, 7, 32, 64, 70, 130]))
        re = (R - 1) * dil + 1
        H = int(r.integers(max(1, re - 2 * pad), 40))
        W = int(r.choice([max(1, re - 2 * pad), 7, 8, 14, 28, 30, 66, 100]))
        if H + 2 * pad < re or W + 2 * pad < re:
            continue
        Ho, Wo = ref.conv_out_hw(H, W, R, R, stride, pad, dil)
        pool = bool(r.integers(2)) and Ho >= 2 and Wo >= 2
        relu = [True, False, "relu6"][int(r.integers(3))]
        N = int(r.choice([1, 2, 3]))
        print("sweep conv %d: %s" % (case, (N, C, H, W, K, R, stride, pad, dil, pool, relu)), flush=True)
        t = datagen.make(7, N=N, C=C, H=H, W=W, K=K, R=R, S=R)
        out, Dn = ref.conv2d_nchw_bias(t["in"], t["wt"], t["bias"], stride, pad, want_norm=True, dil=dil)
        out = ref.scale_shift_ch(out, t["scale"], t["shift"])
        Dn = ref.scale_shift_ch(Dn, np.abs(t["scale"]), np.abs(t["shift"]))
        out = ref.relu6(out) if relu == "relu6" else (ref.relu(out) if relu else out)
        if pool:
            out, Dn = ref.maxpool2x2(out), ref.maxpool2x2(Dn)
        o = torch.full(out.shape, float("nan"), device="cuda")
        plan, ins = hpct.conv_block_plan(dev(t["in"]), dev(t["wt"]), dev(t["bias"]), dev(t["scale"]), dev(t["shift"]), o,
                                         stride, pad, relu, pool, dil)
        plan.launch(ins, [o])
        assert show(plan.kernel_name, compare.contraction(host(o), out, Dn))


def test_sweep_depthwise_shapes():
    r = _rng(20250610403)
    for case in range(30):
        R = int(r.choice([1, 3, 3, 5, 7]))
        stride = int(r.choice([1, 1, 2, 3, 4]))
        dil = int(r.choice([1, 1, 2, 3]))
        pad = int(r.integers(0, (R - 1) * dil + 1))
        re = (R - 1) * dil + 1
        H = int(r.integers(max(1, re - 2 * pad), 70))
        W = int(r.integers(max(1, re - 2 * pad), 130))
        N, C = int(r.choice([1, 2, 5])), int(r.choice([1, 3, 8, 17]))
        print("sweep depthwise %d: %s" % (case, (N, C, H, W, R, stride, pad, dil)), flush=True)
        check_depthwise(N, C, H, W, R, stride, pad, dil, act=[False, "relu", "relu6"][int(r.integers(3))], seed=case)


def test_sweep_pooling_and_norm_shapes():
    r = _rng(20250610405)
    for case in range(30):
        k = int(r.choice([1, 2, 3, 3, 3, 5, 7]))
        stride = int(r.choice([1, 2, 2, 3]))
        pad = int(r.integers(0, k))
        W = int(r.choice([int(r.integers(max(1, k - 2 * pad), 140)), 48, 56, 104, 112, 224]))
        H = int(r.integers(max(1, k - 2 * pad), 40))
        shape = (int(r.choice([1, 2, 3])), int(r.choice([1, 2, 5])), H, W)
        print("sweep pool %d: %s" % (case, (shape, k, stride, pad)), flush=True)
        check_maxpool(shape, k, stride, pad, seed=case)
        check_avgpool(shape, k, stride, pad, seed=case)
    for case in range(20):
        C_ = int(r.choice([1, 2, 4, 6, 8, 12, 16]))
        G = int(r.choice([g for g in (1, 2, 3, 4, 6, 8, 12, 16) if C_ % g == 0]))
        shape = (int(r.choice([1, 2, 3])), C_, int(r.integers(1, 40)), int(r.choice([int(r.integers(1, 50)), 4, 8, 28, 56, 112])))
        print("sweep groupnorm %d: %s G=%d" % (case, shape, G), flush=True)
        check_groupnorm(shape, G, affine=bool(r.integers(2)), relu=bool(r.integers(2)), eps=float(r.choice([1e-5, 1e-3])), seed=case)


def test_sweep_skinny_gemm_shapes():
    r = _rng(20250610406)
    for case in range(16):
        small = int(r.integers(1, 9))
        K = int(r.choice([256, 260, 1024, 4096, 20000])) if case % 4 else int(r.integers(64, 300)) * 4
        big = int(r.integers((1 << 20) // K + 1, (1 << 20) // K + 600))
        rows_of_x = bool(r.integers(2))
        M, N = (big, small) if rows_of_x else (small, big)
        wt = bool(r.integers(2))
        t = datagen.make(1, M=M, K=K, N=N)
        Z, Dn = ref.gemm_bias(t["X"], t["W"], t["bias"], want_norm=True)
        got, name = run_gemm(t, wt=wt, relu=False)
        print("sweep skinny %d: M=%d K=%d N=%d wt=%s -> %s" % (case, M, K, N, wt, name), flush=True)
        if rows_of_x or wt or N % 4 == 0:
            assert name.startswith("gemm_skinny"), name
        assert compare.contraction(got, Z, Dn).ok


def test_sweep_attention_shapes():
    r = _rng(20250610404)
    for case in range(24):
        D = int(r.choice([32, 64, 64, 128]))
        B = int(r.choice([1, 2, 3]))
        L = int(r.choice([1, 5, 31, 64, 65, 130, 200, 300]))
        causal = bool(r.integers(2))
        Lk = L if causal and r.integers(2) else int(r.choice([1, 7, 63, 64, 65, 129, 257, 400]))
        print("sweep attention %d: %s" % (case, (B, L, Lk, D, causal)), flush=True)
        t = datagen.make(5, B=B, L=L, Lk=Lk, D=D)
        scale = 1.0 / np.sqrt(D)
        want, Dn = ref.attention(t["Q"], t["K"], t["V"], scale, want_norm=True, causal=causal)
        assert show("attention", compare.contraction(run_chain5(t, scale, causal=causal), want, Dn))


# ------------------------------------------------------------------ HIP graph capture
def test_launches_can_be_captured_in_a_hip_graph_and_replayed():
    # The library neither allocates nor synchronises nor clears memory through the runtime, so a
    # sequence of launches can be captured once and replayed: the five chains at small sizes, the
    # dropout chain (with its workspace and finishing kernels), a depthwise conv and an axis reduction.
    t1, t2, t3 = datagen.make(1), datagen.make(2, N=2, C=8, H=12, W=12), datagen.make(3, M=64, N=1024)
    t4, t5 = datagen.make(4, N=2, C=8, H=14, W=14, K=64), datagen.make(5, B=2, L=130, Lk=130)
    t6 = datagen.make(6, M=256, K=64, N=512)
    jobs = []

    def job(plan_ins, out):
        plan, ins = plan_ins
        ws = torch.empty(plan.workspace_bytes // 4, device="cuda") if plan.workspace_bytes else None
        jobs.append((plan, ins, out, ws))

    o1 = torch.empty(64, 256, device="cuda")
    job(hpct.gemm_bias_relu_softmax_plan(dev(t1["X"]), dev(t1["W"]), dev(t1["bias"]), o1), o1)
    o2 = torch.empty(2, 8, device="cuda")
    job(hpct.scale_shift_relu_add_pool_plan(dev(t2["X"]), dev(t2["scale"]), dev(t2["shift"]), dev(t2["R"]), o2), o2)
    o3 = torch.empty(64, 1024, device="cuda")
    job(hpct.layernorm_gelu_plan(dev(t3["X"]), dev(t3["gamma"]), dev(t3["beta"]), o3), o3)
    o4 = torch.empty(2, 64, 14, 14, device="cuda")
    job(hpct.conv2d_bias_relu_plan(dev(t4["in"]), dev(t4["wt"]), dev(t4["bias"]), o4), o4)
    o5 = torch.empty(2, 130, 64, device="cuda")
    job(hpct.attention_plan(dev(t5["Q"]), dev(t5["K"]), dev(t5["V"]), o5), o5)
    o6 = torch.empty(256, device="cuda")
    job(hpct.matmul_dropout_mean_softmax_plan(dev(t6["X"]), dev(t6["W"]), dev(t6["bias"]), o6, 0.25, 7), o6)
    xd = dev(datagen.gen_normal(400, (2, 6, 20, 20), 0.0, 1.0))
    od = torch.empty(2, 6, 20, 20, device="cuda")
    job(hpct.depthwise_conv_plan(xd, dev(datagen.gen_normal(401, (6, 1, 3, 3), 0.0, 0.5)), None, None, None, od), od)
    xr = dev(datagen.gen_normal(402, (300, 520), 0.0, 1.0))
    orr = torch.empty(520, device="cuda")
    job(hpct.reduce_axis_plan(xr, orr, 0, "sum"), orr)
    assert any(ws is not None for _, _, _, ws in jobs)

    def run_all():
        for plan, ins, out, ws in jobs:
            plan.launch(ins, [out], workspace=ws)      # on the stream current now

    run_all()                                          # eager reference
    torch.cuda.synchronize()
    want = [host(o).copy() for _, _, o, _ in jobs]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                      # the capture stream is current inside
        run_all()
    for rep in range(3):
        for _, _, o, _ in jobs:
            o.fill_(float("nan"))                      # eager work between the replays
        jobs[0][0].launch(jobs[0][1], [jobs[0][2]])    # and an eager launch of the library itself
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (_, _, o, _), w in zip(jobs, want):
            assert np.array_equal(host(o).view(np.uint32), w.view(np.uint32)), rep
