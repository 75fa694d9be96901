"""The C-ABI library: loads, exports every symbol the header declares, and its
host-side logic (descriptor validation, chain recognition, launch shapes,
launch-time pointer checks) behaves as the header states.  No kernel is
launched here, so this runs without a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2506_10401_amd import hpct as H

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hpct.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hpct_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = H.load()
    names = declared_functions()
    assert {"hpct_plan_create", "hpct_plan_workspace_bytes", "hpct_plan_launch", "hpct_plan_destroy",
            "hpct_last_error", "hpct_version"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None
    assert "gfx950" in H.hpct_version()


def test_struct_sizes_match_the_c_layout():
    # int32 + pad + 6*int64 + 6*int64 + enum + pad
    assert C.sizeof(H.TensorDesc) == 112
    assert C.sizeof(H.OpDesc) == 4 + 4 + 8 * 4 + 4 + 4 + 4 + 4 + 8 * 112 + 4 + 4 + 2 * 112 + 8 + 8 + 4 + 4 + 4 + 4 + 8 + 4 + 8 + 4 + 8
    # and the library reports the same sizes for the structs it was compiled with
    lib = H.load()
    assert lib.hpct_sizeof_tensor_desc() == C.sizeof(H.TensorDesc)
    assert lib.hpct_sizeof_op_desc() == C.sizeof(H.OpDesc)


def cfg_desc(i):
    if i == 1:
        return H.op_desc(H.HPCT_ANCHOR_GEMM, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_SOFTMAX_LAST, 0,
                         [(64, 256), (256, 256), (256,)], [(64, 256)])
    if i == 2:
        return H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SCALE_SHIFT_CH, H.HPCT_EPI_RELU, H.HPCT_EPI_ADD_RESIDUAL],
                         H.HPCT_RED_AVGPOOL_HW, 0, [(32, 64, 56, 56), (64,), (64,), (32, 64, 56, 56)], [(32, 64)])
    if i == 3:
        return H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_GELU_TANH], H.HPCT_RED_LAYERNORM_LAST, 1,
                         [(8192, 4096), (4096,), (4096,)], [(8192, 4096)], eps=1e-5)
    if i == 4:
        return H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0,
                         [(32, 64, 56, 56), (128, 64, 3, 3), (128,)], [(32, 128, 56, 56)], pad_hw=(1, 1))
    return H.op_desc(H.HPCT_ANCHOR_BGEMM_SOFTMAX_BGEMM, [H.HPCT_EPI_SCALE_CONST], H.HPCT_RED_NONE, 0,
                     [(16, 2048, 64)] * 3, [(16, 2048, 64)], scale=0.125)


def test_the_five_workloads_plan_and_launch_shapes():
    want = {
        1: ("gemm_ksplit16<32>", (8, 4, 1), (1024, 1, 1)),
        2: ("affine_planes_vec<pool>", (2048, 1, 1), (256, 1, 1)),
        3: ("layernorm_rows_persist", (768, 1, 1), (256, 1, 1)),
        4: ("conv2d_nchw_mfma<3x3,pipelined>", (3136, 1, 1), (256, 1, 1)),
        5: ("attn_fwd_d64<ks2>", (256, 1, 1), (512, 1, 1)),
    }
    for i in range(1, 6):
        p = H.Plan(cfg_desc(i))
        grid, block, lds = p.launch_shape()
        assert (p.kernel_name, grid, block) == want[i]
        assert lds <= 160 * 1024
        assert p.workspace_bytes == 0
    # shape/index logic that must be exact: tiles cover the outputs
    g, b, _ = H.Plan(cfg_desc(4)).launch_shape()
    assert g[0] == 32 * ((56 * 56 + 63) // 64) * (128 // 64) and g[1] == 1  # pixel tiles x channel blocks
    g, b, _ = H.Plan(cfg_desc(5)).launch_shape()
    assert g[0] == 16 * (2048 // 128) and g[1] == 1  # batches x query blocks


def expect(status, desc):
    with pytest.raises(H.HpctError) as e:
        H.Plan(desc)
    assert e.value.status == status, e.value
    assert e.value.message  # an error text is always set
    return e.value


def test_null_arguments():
    lib = H.load()
    h = C.c_void_p()
    assert lib.hpct_plan_create(None, C.byref(h)) == H.HPCT_ERR_NULL
    assert lib.hpct_plan_create(C.byref(cfg_desc(1)), None) == H.HPCT_ERR_NULL
    assert b"NULL" in lib.hpct_last_error()
    assert lib.hpct_plan_workspace_bytes(None) == 0
    assert lib.hpct_plan_kernel_name(None) == b""
    assert lib.hpct_plan_launch_shape(None, None, None, None) == H.HPCT_ERR_NULL
    lib.hpct_plan_destroy(None)
    assert lib.hpct_plan_launch(None, None, None, None, 0, None) == H.HPCT_ERR_NULL


def test_bad_descriptors():
    d = cfg_desc(1); d.in_[0].ndim = 0
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.in_[0].ndim = 7
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.in_[1].shape[0] = 0
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.in_[1].shape[1] = -4
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.in_[0].stride[0] = -1
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.n_in = 0
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.n_in = 9
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.n_out = 3
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.n_epi = 9
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.anchor = 17
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.reduce = -1
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.epi[0] = 99
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.n_in = 2  # bias listed in the epilogues but not supplied
    expect(H.HPCT_ERR_BAD_DESC, d)
    # overflow of the element count / the largest offset
    big = 1 << 62
    d = cfg_desc(3); d.in_[0] = H.tensor_desc((big, 4), (4, 1))
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(3); d.in_[0] = H.tensor_desc((8192, 4096), (big, 1))
    expect(H.HPCT_ERR_BAD_DESC, d)
    # overlapping output elements
    d = cfg_desc(3); d.out[0] = H.tensor_desc((8192, 4096), (0, 1))
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(3); d.eps = -1.0
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(4); d.stride_hw[0] = 0
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(4); d.pad_hw[1] = -1
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(5); d.scale = float("inf")
    expect(H.HPCT_ERR_BAD_DESC, d)


def test_shape_mismatches():
    d = cfg_desc(1); d.in_[1] = H.tensor_desc((255, 256))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(1); d.in_[2] = H.tensor_desc((255,))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(1); d.out[0] = H.tensor_desc((256, 64))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(1); d.in_[0] = H.tensor_desc((64, 16, 16))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(2); d.in_[1] = H.tensor_desc((63,))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(2); d.in_[3] = H.tensor_desc((32, 64, 56, 55))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(2); d.out[0] = H.tensor_desc((64, 32))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(3); d.in_[1] = H.tensor_desc((8192,))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(4); d.in_[1] = H.tensor_desc((128, 63, 3, 3))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(4); d.out[0] = H.tensor_desc((32, 128, 54, 54))  # that would be pad 0
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(4); d.in_[0] = H.tensor_desc((1, 64, 2, 2)); d.pad_hw[0] = d.pad_hw[1] = 0
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)  # filter larger than the input
    d = cfg_desc(5); d.in_[2] = H.tensor_desc((16, 2047, 64))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = cfg_desc(5); d.in_[1] = H.tensor_desc((15, 2048, 64)); d.in_[2] = H.tensor_desc((15, 2048, 64))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)


def test_unsupported_but_well_formed():
    d = cfg_desc(1); d.in_[0].dtype = 1
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(1); d.epi[0], d.epi[1] = H.HPCT_EPI_RELU, H.HPCT_EPI_BIAS_COL  # order not offered
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(1); d.reduce = H.HPCT_RED_AVGPOOL_HW
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    # (a softmax row wider than one work-group tile is supported: GEMM, then an in-place row softmax)
    d = H.op_desc(H.HPCT_ANCHOR_GEMM, [], H.HPCT_RED_SOFTMAX_LAST, 0, [(64, 256), (256, 512)], [(64, 512)])
    assert H.Plan(d).kernel_name == "gemm_ksplit16<32>" and H.Plan(d).launch_shape()[0] == (16, 4, 1)
    # (a short K keeps the 16-row kernel, whose work-group holds whole rows of up to 256 columns)
    d = H.op_desc(H.HPCT_ANCHOR_GEMM, [], H.HPCT_RED_SOFTMAX_LAST, 0, [(64, 32), (32, 512)], [(64, 512)])
    assert H.Plan(d).kernel_name == "gemm_rows16<256>" and H.Plan(d).launch_shape()[0] == (4, 2, 1)
    # non-contiguous layouts
    d = cfg_desc(1); d.in_[1] = H.tensor_desc((256, 256), (1, 256))  # transposed W: an instance of its own
    assert H.Plan(d).kernel_name == "gemm_rows16<256,wt>"
    d = cfg_desc(1); d.in_[1] = H.tensor_desc((256, 256), (512, 2))  # any other stride pattern is refused
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(3); d.in_[0] = H.tensor_desc((8192, 4096), (8192, 1))  # row pitch
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(3); d.reduce_before_epi = 0
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(4); d.stride_hw[0], d.stride_hw[1] = 2, 1           # anisotropic stride
    d.out[0] = H.tensor_desc((32, 128, 28, 56))
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(4); d.stride_hw[0] = d.stride_hw[1] = 5
    d.out[0] = H.tensor_desc((32, 128, 12, 12))
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(4); d.in_[1] = H.tensor_desc((128, 64, 4, 4)); d.out[0] = H.tensor_desc((32, 128, 55, 55))   # even filter
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(4); d.in_[1] = H.tensor_desc((128, 64, 3, 5)); d.out[0] = H.tensor_desc((32, 128, 56, 54))   # not square
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(5); d.in_[0] = d.in_[1] = d.in_[2] = H.tensor_desc((16, 2048, 48)); d.out[0] = H.tensor_desc((16, 2048, 48))
    expect(H.HPCT_ERR_UNSUPPORTED, d)            # head dims 32, 64, 128 only
    d = cfg_desc(5); d.epi[0] = H.HPCT_EPI_RELU
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    # index range of the kernels
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_LAYERNORM_LAST, 0, [(4, 1 << 32)], [(4, 1 << 32)])
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def test_variants_of_the_chains_are_recognised():
    ok = [
        H.op_desc(H.HPCT_ANCHOR_GEMM, [], H.HPCT_RED_NONE, 0, [(5, 7), (7, 1000)], [(5, 1000)]),
        H.op_desc(H.HPCT_ANCHOR_GEMM, [H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0, [(5, 7), (7, 9)], [(5, 9)]),
        H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_SOFTMAX_LAST, 0, [(5, 7)], [(5, 7)]),
        H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_LAYERNORM_LAST, 0, [(5, 7)], [(5, 7)], eps=1e-5),
        H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_RELU], H.HPCT_RED_AVGPOOL_HW, 0, [(2, 3, 3, 5)], [(2, 3)]),
        H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SCALE_SHIFT_CH, H.HPCT_EPI_ADD_RESIDUAL], H.HPCT_RED_NONE, 0,
                  [(2, 3, 4, 5), (3,), (3,), (2, 3, 4, 5)], [(2, 3, 4, 5)]),
        H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [], H.HPCT_RED_NONE, 0, [(1, 3, 8, 8), (5, 3, 1, 1)], [(1, 5, 8, 8)]),
        H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0, [(1, 3, 8, 8), (5, 3, 3, 3)],
                  [(1, 5, 6, 6)]),
        H.op_desc(H.HPCT_ANCHOR_BGEMM_SOFTMAX_BGEMM, [], H.HPCT_RED_NONE, 0, [(2, 5, 64), (2, 9, 64), (2, 9, 64)],
                  [(2, 5, 64)]),
    ]
    for d in ok:
        p = H.Plan(d)
        assert p.kernel_name
    # odd sizes pick the unvectorised variants
    assert "any" in H.Plan(ok[3]).kernel_name
    assert "any" in H.Plan(ok[4]).kernel_name


def test_launch_time_pointer_checks_return_before_any_launch():
    p = H.Plan(cfg_desc(3))
    nbytes = 8192 * 4096 * 4
    base = 0x7F0000000000  # fake device addresses: every case below is rejected on the host
    x, g, b, y = base, base + nbytes, base + nbytes + 16384, base + 2 * nbytes
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, 0, b], [y])
    assert e.value.status == H.HPCT_ERR_NULL
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, g, b], [0])
    assert e.value.status == H.HPCT_ERR_NULL
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x + 4, g, b], [y])
    assert e.value.status == H.HPCT_ERR_ALIGNMENT
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, g, b], [y + 8])
    assert e.value.status == H.HPCT_ERR_ALIGNMENT
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, g, b], [x])  # in place
    assert e.value.status == H.HPCT_ERR_BAD_DESC
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, g, b], [x + nbytes - 16])  # output starts inside X's last row
    assert e.value.status == H.HPCT_ERR_BAD_DESC
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, g, b], [g - nbytes + 16])  # output's tail reaches gamma
    assert e.value.status == H.HPCT_ERR_BAD_DESC


def test_layout_transform_plans():
    def plan(shape, stride):
        return H.Plan(H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_NONE, 0, [H.tensor_desc(shape, stride)], [shape]))
    # NCHW -> NHWC collapses to [N, HW, C] and is a tiled transpose of C against HW
    p = plan((32, 56, 56, 64), (64 * 3136, 56, 1, 3136))
    assert p.kernel_name == "layout_transpose<32x32>"
    assert p.launch_shape()[0] == (32 * 98 * 2, 1, 1)  # 32 images x ceil(3136/32) x ceil(64/32) tiles
    assert plan((32, 64, 64, 64), (64 * 4096, 64, 1, 4096)).kernel_name == "layout_transpose<64x128>"
    assert plan((100, 200), (1, 100)).kernel_name == "layout_transpose<32x32>"
    assert plan((4096, 8192), (1, 4096)).kernel_name == "layout_transpose<128x128>"
    assert plan((8, 16, 32, 64), (16 * 32 * 64, 64, 16 * 64, 1)).kernel_name == "layout_rows<vec4>"
    assert plan((5, 7), (0, 1)).kernel_name == "layout_rows<scalar>"
    # the tiled transpose works with 32-bit tile coordinates: an extent beyond them falls back to the gather
    assert plan((2, 3 * 10**9), (1, 2)).kernel_name == "layout_rows<scalar>"
    assert plan((2, 2 * 10**9), (1, 2)).kernel_name == "layout_transpose<32x32>"
    assert plan((4, 6, 8, 4), (6 * 8 * 12, 8 * 12, 12, 3)).kernel_name == "layout_rows<scalar>"  # no unit stride anywhere
    # the output must be contiguous and of the view's shape
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_NONE, 0, [H.tensor_desc((4, 6), (1, 4))], [H.tensor_desc((4, 6), (1, 4))])
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_NONE, 0, [H.tensor_desc((4, 6), (1, 4))], [(6, 4)])
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    # overlap of the view's extent with the output is caught at launch, before any kernel
    p = plan((100, 200), (1, 100))
    base = 0x7F0000000000
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([base], [base + 16])
    assert e.value.status == H.HPCT_ERR_BAD_DESC


def chain6_desc(M=4096, K=1024, N=4096, stop="softmax", p=0.25, seed=0x250610401, anchor=None):
    red = H.HPCT_RED_NONE if stop == "dropout" else H.HPCT_RED_MEAN_LAST
    red2 = H.HPCT_RED_SOFTMAX_LAST if stop == "softmax" else H.HPCT_RED_NONE
    return H.op_desc(H.HPCT_ANCHOR_GEMM if anchor is None else anchor, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_DROPOUT_HASH], red, 0,
                     [(M, K), (K, N), (N,)], [(M, N) if stop == "dropout" else (M,)], dropout_p=p, dropout_seed=seed,
                     reduce2=red2)


def test_matmul_dropout_mean_softmax_plans():
    p = H.Plan(chain6_desc())
    assert p.kernel_name == "gemm_tile128"
    assert p.launch_shape() == ((32 * 32, 1, 1), (256, 1, 1), (2 * 128 * 20 + 2 * 16 * 136 + 2 * 128) * 4)
    assert p.workspace_bytes == 32 * 4096 * 4          # one float per (column tile, row)
    assert H.Plan(chain6_desc(stop="dropout")).workspace_bytes == 0
    assert H.Plan(chain6_desc(stop="mean")).workspace_bytes == 32 * 4096 * 4
    small = H.Plan(chain6_desc(64, 256, 256))
    assert small.kernel_name == "gemm_rows16<256>" and small.workspace_bytes == 64 * 4
    wide = H.Plan(chain6_desc(64, 256, 1000))
    assert wide.kernel_name == "gemm_rows16<256>" and wide.workspace_bytes == 4 * 64 * 4
    # a large GEMM without the dropout chain also takes the tiled kernel; the fused row softmax keeps the 16-row one
    g = H.op_desc(H.HPCT_ANCHOR_GEMM, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0,
                  [(2048, 512), (512, 2048), (2048,)], [(2048, 2048)])
    pg = H.Plan(g)
    assert pg.kernel_name == "gemm_tile64" and pg.launch_shape()[0] == (32 * 32, 1, 1)   # 256 128-tiles would be one per CU
    g = H.op_desc(H.HPCT_ANCHOR_GEMM, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0,
                  [(4096, 512), (512, 2048), (2048,)], [(4096, 2048)])
    assert H.Plan(g).kernel_name == "gemm_tile128"
    g = H.op_desc(H.HPCT_ANCHOR_GEMM, [], H.HPCT_RED_SOFTMAX_LAST, 0, [(8192, 64), (64, 256)], [(8192, 256)])
    assert H.Plan(g).kernel_name == "gemm_rows16<256>"


def test_matmul_dropout_mean_softmax_errors():
    expect(H.HPCT_ERR_BAD_DESC, chain6_desc(p=1.0))
    expect(H.HPCT_ERR_BAD_DESC, chain6_desc(p=-0.1))
    expect(H.HPCT_ERR_BAD_DESC, chain6_desc(p=float("nan")))
    d = chain6_desc(); d.out[0] = H.tensor_desc((4096, 4096))      # MEAN_LAST drops the last dim
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = chain6_desc(stop="mean"); d.reduce2 = H.HPCT_RED_LAYERNORM_LAST
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = chain6_desc(stop="dropout"); d.reduce2 = H.HPCT_RED_SOFTMAX_LAST   # second reduction without the first
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = chain6_desc(); d.reduce2 = 99
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = chain6_desc(); d.epi[0], d.epi[1] = H.HPCT_EPI_DROPOUT_HASH, H.HPCT_EPI_BIAS_COL   # order matters
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    # MEAN_LAST / DROPOUT_HASH outside a GEMM chain
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_MEAN_LAST, 0, [(8, 8)], [(8,)])
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(4); d.epi[1] = H.HPCT_EPI_DROPOUT_HASH
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(3); d.reduce2 = H.HPCT_RED_SOFTMAX_LAST
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def test_workspace_checks_return_before_any_launch():
    p = H.Plan(chain6_desc(256, 64, 512))
    need = p.workspace_bytes
    assert need == 2 * 256 * 4
    base = 0x7F0000000000  # fake device addresses: every case below is rejected on the host
    x, w, b, y, ws = base, base + (1 << 20), base + (2 << 20), base + (3 << 20), base + (4 << 20)
    for args in [dict(), dict(workspace=ws, workspace_bytes=need - 4), dict(workspace=0, workspace_bytes=need)]:
        with pytest.raises(H.HpctError) as e:
            p.launch_ptrs([x, w, b], [y], **args)
        assert e.value.status == H.HPCT_ERR_WORKSPACE
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, w, b], [y], workspace=ws + 4, workspace_bytes=need)
    assert e.value.status == H.HPCT_ERR_ALIGNMENT
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, w, b], [y], workspace=y, workspace_bytes=need)          # workspace on the output
    assert e.value.status == H.HPCT_ERR_BAD_DESC
    with pytest.raises(H.HpctError) as e:
        p.launch_ptrs([x, w, b], [y], workspace=w + 64, workspace_bytes=need)     # workspace inside W
    assert e.value.status == H.HPCT_ERR_BAD_DESC


def conv_block_desc(pool=True, stride=1, R=3, pad=1, shape=(32, 64, 56, 56), K=128, dil=1):
    Nb, Cc, Hh, Ww = shape
    Re = (R - 1) * dil + 1
    Ho, Wo = (Hh + 2 * pad - Re) // stride + 1, (Ww + 2 * pad - Re) // stride + 1
    return H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_SCALE_SHIFT_CH, H.HPCT_EPI_RELU],
                     H.HPCT_RED_MAXPOOL2_HW if pool else H.HPCT_RED_NONE, 0,
                     [shape, (K, Cc, R, R), (K,), (K,), (K,)], [(Nb, K, Ho // 2, Wo // 2) if pool else (Nb, K, Ho, Wo)],
                     stride_hw=(stride, stride), pad_hw=(pad, pad), dilation_hw=(dil, dil))


def test_conv_block_plans():
    p = H.Plan(conv_block_desc())
    assert p.kernel_name == "conv2d_nchw_mfma<3x3,pipelined,maxpool2>"
    # 7 x 7 tiles of 8 x 8 output pixels x 32 images x 2 channel blocks
    assert p.launch_shape()[0] == (7 * 7 * 32 * 2, 1, 1) and p.launch_shape()[1] == (256, 1, 1)
    assert p.workspace_bytes == 0
    assert H.Plan(conv_block_desc(pool=False)).kernel_name == "conv2d_nchw_mfma<3x3,pipelined>"
    assert H.Plan(conv_block_desc(stride=2)).kernel_name == "conv2d_nchw_mfma<3x3,pipelined,maxpool2>"
    assert H.Plan(conv_block_desc(pool=False, stride=2, R=7, pad=3, shape=(4, 3, 64, 64), K=64)).kernel_name == \
        "conv2d_nchw_mfma<7x7,general>"
    assert H.Plan(conv_block_desc(R=5, pad=2, shape=(2, 8, 30, 30), K=16)).kernel_name == "conv2d_nchw_mfma<5x5,general,maxpool2>"
    # images wider than 64 columns: 8 x 8 output windows also without pooling (28 x 28 of them x 2 x 1)
    p = H.Plan(conv_block_desc(pool=False, shape=(2, 8, 224, 224), K=64))
    assert p.kernel_name == "conv2d_nchw_mfma<3x3,pipelined,window>" and p.launch_shape()[0] == (28 * 28 * 2, 1, 1)
    assert H.Plan(conv_block_desc(pool=False, R=1, pad=0, stride=2, shape=(2, 16, 20, 100), K=64)).kernel_name == \
        "conv2d_nchw_mfma<1x1,general>"                                       # 1x1 filters keep whole rows
    assert H.Plan(conv_block_desc(R=1, pad=0)).kernel_name == "conv2d_nchw_mfma<1x1,pipelined,maxpool2>"
    # dilation: the filter spans (R-1)*dil + 1 rows; 0 in the descriptor means 1
    assert H.Plan(conv_block_desc(pool=False, dil=2, pad=2)).kernel_name == "conv2d_nchw_mfma<3x3,general>"
    d = conv_block_desc(); d.dilation_hw[0] = d.dilation_hw[1] = 0
    assert H.Plan(d).kernel_name == "conv2d_nchw_mfma<3x3,pipelined,maxpool2>"
    d = conv_block_desc(pool=False, dil=2, pad=2); d.dilation_hw[1] = 1
    d.out[0] = H.tensor_desc((32, 128, 56, 58))
    expect(H.HPCT_ERR_UNSUPPORTED, d)                                         # anisotropic dilation
    expect(H.HPCT_ERR_UNSUPPORTED, conv_block_desc(pool=False, dil=5, pad=5))
    d = conv_block_desc(); d.dilation_hw[0] = -1
    expect(H.HPCT_ERR_BAD_DESC, d)
    # errors
    d = conv_block_desc(); d.out[0] = H.tensor_desc((32, 128, 56, 56))        # pooled output is half the size
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = conv_block_desc(); d.in_[3] = H.tensor_desc((64,))                    # scale is per OUTPUT channel
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = conv_block_desc(shape=(1, 4, 1, 8), pad=1)                            # conv output 1 x 8: nothing to pool
    d.out[0] = H.tensor_desc((1, 128, 1, 4))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = conv_block_desc(); d.epi[1], d.epi[2] = H.HPCT_EPI_RELU, H.HPCT_EPI_SCALE_SHIFT_CH   # order not offered
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = conv_block_desc(); d.reduce = H.HPCT_RED_AVGPOOL_HW
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(2); d.reduce = H.HPCT_RED_MAXPOOL2_HW                        # pooling without a conv anchor
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def reduce_desc(shape, stride, axis, red, out_shape=None, out_dtype=None):
    if out_shape is None:
        out_shape = tuple(n for k, n in enumerate(shape) if k != axis) or (1,)
    arg = red in (H.HPCT_RED_ARGMAX_AXIS, H.HPCT_RED_ARGMIN_AXIS)
    if out_dtype is None:
        out_dtype = H.HPCT_I32 if arg else H.HPCT_F32
    return H.op_desc(H.HPCT_ANCHOR_NONE, [], red, 0, [H.tensor_desc(shape, stride)],
                     [H.tensor_desc(out_shape, None, out_dtype)], axis=axis)


def test_axis_reduction_plans():
    # rows of a matrix: the reduced axis is contiguous, a wave per output; a work-group per output from 4096 columns
    p = H.Plan(reduce_desc((8192, 2048), (2048, 1), 1, H.HPCT_RED_SUM_AXIS))
    assert p.kernel_name == "reduce_rows<wave>" and p.launch_shape()[0] == (2048, 1, 1)
    p = H.Plan(reduce_desc((8192, 4096), (4096, 1), 1, H.HPCT_RED_SUM_AXIS))
    assert p.kernel_name == "reduce_rows<group>" and p.launch_shape()[0] == (8192, 1, 1)
    # few long rows: a work-group per output
    p = H.Plan(reduce_desc((16, 1 << 20), (1 << 20, 1), 1, H.HPCT_RED_MEAN_AXIS))
    assert p.kernel_name == "reduce_rows<group>" and p.launch_shape()[0] == (16, 1, 1)
    # columns of a matrix, channels of NCHW: threads along the contiguous kept dimension
    p = H.Plan(reduce_desc((8192, 4096), (4096, 1), 0, H.HPCT_RED_SUM_AXIS))
    assert p.kernel_name == "reduce_cols<vec4,split>"      # 4096 outputs cannot fill the chip: the axis is split
    split = p.workspace_bytes // (4096 * 4)
    assert 2 <= split <= 64 and p.workspace_bytes == split * 4096 * 4
    g = p.launch_shape()[0][0]
    assert g >= 256 and g % split == 0 and 4096 % (g // split) == 0   # column strips x pieces
    pa = H.Plan(reduce_desc((8192, 4096), (4096, 1), 0, H.HPCT_RED_ARGMIN_AXIS))
    assert pa.workspace_bytes == 2 * p.workspace_bytes      # value and index per piece
    p = H.Plan(reduce_desc((32, 64, 56, 56), (200704, 3136, 56, 1), 1, H.HPCT_RED_ARGMAX_AXIS))
    assert p.kernel_name == "reduce_cols<scalar>"    # H and W collapse into one contiguous dimension of 3136
    assert p.launch_shape()[0] == (49 * 32, 1, 1) and p.workspace_bytes == 0
    # nothing contiguous: gather
    p = H.Plan(reduce_desc((10, 20, 30), (1200, 60, 2), 1, H.HPCT_RED_ARGMIN_AXIS))
    assert p.kernel_name == "reduce_gather"
    # a vector reduces to shape [1]
    assert H.Plan(reduce_desc((1000,), (1,), 0, H.HPCT_RED_SUM_AXIS)).kernel_name.startswith("reduce_rows")
    # the extreme values themselves: the arg kernels, fp32 out
    pm = H.Plan(reduce_desc((8192, 4096), (4096, 1), 0, H.HPCT_RED_MAX_AXIS))
    assert pm.kernel_name == "reduce_cols<vec4,split>" and pm.workspace_bytes == pa.workspace_bytes
    assert H.Plan(reduce_desc((8192, 4096), (4096, 1), 1, H.HPCT_RED_MIN_AXIS)).kernel_name == "reduce_rows<group>"
    assert p.workspace_bytes == 0


def test_axis_reduction_errors():
    expect(H.HPCT_ERR_BAD_DESC, reduce_desc((4, 5), (5, 1), 2, H.HPCT_RED_SUM_AXIS, out_shape=(4,)))
    expect(H.HPCT_ERR_BAD_DESC, reduce_desc((4, 5), (5, 1), -1, H.HPCT_RED_SUM_AXIS, out_shape=(4,)))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_SUM_AXIS, out_shape=(5,)))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_SUM_AXIS, out_shape=(4, 1)))
    # dtypes: indices are int32, sums fp32
    expect(H.HPCT_ERR_UNSUPPORTED, reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_ARGMAX_AXIS, out_dtype=H.HPCT_F32))
    expect(H.HPCT_ERR_UNSUPPORTED, reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_SUM_AXIS, out_dtype=H.HPCT_I32))
    expect(H.HPCT_ERR_UNSUPPORTED, reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_MAX_AXIS, out_dtype=H.HPCT_I32))
    expect(H.HPCT_ERR_BAD_DESC, reduce_desc((4, 5), (5, 1), 1, 16))      # one past the last reduction
    d = cfg_desc(3); d.out[0].dtype = H.HPCT_I32          # int32 anywhere else
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_SUM_AXIS); d.n_epi = 1; d.epi[0] = H.HPCT_EPI_RELU
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_SUM_AXIS); d.anchor = H.HPCT_ANCHOR_GEMM
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = reduce_desc((4, 5), (5, 1), 1, H.HPCT_RED_SUM_AXIS); d.out[0] = H.tensor_desc((4,), (2,))   # strided output
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def test_causal_attention_plan():
    d = cfg_desc(5); d.n_epi = 2; d.epi[1] = H.HPCT_EPI_CAUSAL_MASK
    p = H.Plan(d)
    # 32 query blocks of 64 per batch, handled in pairs (i, 31 - i): 16 work-groups per batch
    assert p.kernel_name == "attn_fwd_d64<ks4,causal,paired>" and p.launch_shape()[:2] == ((256, 1, 1), (512, 1, 1))
    d = cfg_desc(5); d.n_epi = 1; d.epi[0] = H.HPCT_EPI_CAUSAL_MASK       # mask without a scale: scale 1
    assert H.Plan(d).kernel_name == "attn_fwd_d64<ks4,causal,paired>"
    d = cfg_desc(5); d.n_epi = 2; d.epi[0], d.epi[1] = H.HPCT_EPI_CAUSAL_MASK, H.HPCT_EPI_SCALE_CONST
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = cfg_desc(1); d.epi[1] = H.HPCT_EPI_CAUSAL_MASK                   # only on attention scores
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def test_attention_head_dims():
    for D, plain, causal in [(32, "attn_fwd_d32<ks2>", "attn_fwd_d32<ks4,causal,paired>"),
                             (128, "attn_fwd_d128<ks2>", "attn_fwd_d128<ks2,causal,paired>")]:
        d = cfg_desc(5); d.in_[0] = d.in_[1] = d.in_[2] = H.tensor_desc((16, 2048, D)); d.out[0] = H.tensor_desc((16, 2048, D))
        p = H.Plan(d)
        assert p.kernel_name == plain and p.launch_shape()[0] == (256, 1, 1)
        assert p.launch_shape()[2] == 2 * 64 * (2 * D + 12) * 4      # two stages of 64 keys, K and V rows padded by 4 and 8
        d.n_epi = 2; d.epi[1] = H.HPCT_EPI_CAUSAL_MASK
        assert H.Plan(d).kernel_name == causal


def test_gemm_split_k_plans():
    g = H.op_desc(H.HPCT_ANCHOR_GEMM, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0,
                  [(1024, 4096), (4096, 1024), (1024,)], [(1024, 1024)])
    p = H.Plan(g)
    assert p.kernel_name == "gemm_tile64<split-k>"
    assert p.workspace_bytes == 2 * 1024 * 1024 * 4 and p.launch_shape()[0] == (16 * 16 * 2, 1, 1)
    # a short K is not split, and neither is the chain with fused row sums
    g = H.op_desc(H.HPCT_ANCHOR_GEMM, [], H.HPCT_RED_NONE, 0, [(1024, 256), (256, 1024)], [(1024, 1024)])
    assert H.Plan(g).kernel_name == "gemm_tile64" and H.Plan(g).workspace_bytes == 0
    assert H.Plan(chain6_desc(1024, 4096, 1024)).kernel_name == "gemm_tile64"


def test_gemm_transposed_weight_and_scale_plans():
    def g(M, K, N, wstride, epi=(H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU), red=H.HPCT_RED_NONE, scale=1.0):
        ins = [(M, K), H.tensor_desc((K, N), wstride)] + ([(N,)] if H.HPCT_EPI_BIAS_COL in epi else [])
        return H.op_desc(H.HPCT_ANCHOR_GEMM, list(epi), red, 0, ins, [(M, N)], scale=scale)
    # W as the transposed view of an [N,K] row-major array: strides (1, K)
    assert H.Plan(g(64, 256, 256, (1, 256), red=H.HPCT_RED_SOFTMAX_LAST)).kernel_name == "gemm_rows16<256,wt>"
    assert H.Plan(g(4096, 1024, 4096, (1, 1024))).kernel_name == "gemm_tile128<wt>"
    p = H.Plan(g(256, 2048, 256, (1, 2048)))
    assert p.kernel_name == "gemm_tile64<wt,split-k>" and p.workspace_bytes == H.Plan(g(256, 2048, 256, (256, 1))).workspace_bytes
    assert H.Plan(g(64, 256, 256, (256, 1))).kernel_name == "gemm_ksplit16<32>"
    assert H.Plan(g(64, 48, 256, (256, 1))).kernel_name == "gemm_rows16<256>"
    assert H.Plan(g(2064, 256, 256, (256, 1), red=H.HPCT_RED_SOFTMAX_LAST)).kernel_name == "gemm_rows16<256>"   # more than 128 row blocks
    # any other W layout is refused; the bias and the output stay contiguous (a strided X is copied: its own test)
    expect(H.HPCT_ERR_UNSUPPORTED, g(64, 256, 256, (1, 512)))
    expect(H.HPCT_ERR_UNSUPPORTED, g(64, 256, 256, (512, 1)))
    expect(H.HPCT_ERR_UNSUPPORTED, g(64, 256, 256, (2, 512)))
    d = g(64, 256, 256, (256, 1)); d.out[0] = H.tensor_desc((64, 256), (1, 64))
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = g(64, 256, 256, (256, 1)); d.in_[2] = H.tensor_desc((256,), (2,))
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    # Gemm-Scale: SCALE_CONST sits between the bias and the ReLU
    e = (H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_SCALE_CONST, H.HPCT_EPI_RELU)
    assert H.Plan(g(64, 256, 256, (256, 1), e, scale=0.5)).kernel_name == "gemm_ksplit16<32>"
    assert H.Plan(g(64, 256, 256, (256, 1), (H.HPCT_EPI_SCALE_CONST,), scale=0.5)).kernel_name == "gemm_ksplit16<32>"
    assert H.Plan(g(64, 32, 256, (256, 1), e, scale=0.5)).kernel_name == "gemm_rows16<256>"
    assert H.Plan(g(4096, 1024, 4096, (1, 1024), e + (H.HPCT_EPI_DROPOUT_HASH,), scale=2.0)).kernel_name == "gemm_tile128<wt>"
    expect(H.HPCT_ERR_UNSUPPORTED, g(64, 256, 256, (256, 1), (H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU, H.HPCT_EPI_SCALE_CONST)))
    expect(H.HPCT_ERR_UNSUPPORTED, g(64, 256, 256, (256, 1), (H.HPCT_EPI_SCALE_CONST, H.HPCT_EPI_BIAS_COL)))


def test_eltwise_further_steps_plans():
    for e in (H.HPCT_EPI_ABS, H.HPCT_EPI_NEG, H.HPCT_EPI_SQUARE, H.HPCT_EPI_LOG, H.HPCT_EPI_SILU, H.HPCT_EPI_HARDSWISH):
        p = H.Plan(H.op_desc(H.HPCT_ANCHOR_NONE, [e, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0, [(64, 128)], [(64, 128)]))
        assert p.kernel_name == "eltwise_unary<vec4>"
        # unary steps of elementwise chains only: no contraction chain takes them
        expect(H.HPCT_ERR_UNSUPPORTED, H.op_desc(H.HPCT_ANCHOR_GEMM, [e], H.HPCT_RED_NONE, 0, [(64, 32), (32, 64)], [(64, 64)]))
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SIN], H.HPCT_RED_NONE, 0, [(7, 9)], [(7, 9)]); d.epi[0] = 25
    expect(H.HPCT_ERR_BAD_DESC, d)


def test_gemm_skinny_plans():
    def g(M, K, N, wstride=None, red=H.HPCT_RED_NONE, epi=(H.HPCT_EPI_BIAS_COL,)):
        return H.op_desc(H.HPCT_ANCHOR_GEMM, list(epi), red, 0, [(M, K), H.tensor_desc((K, N), wstride), (N,)], [(M, N)])
    # a matrix times a vector: a wave per row of X, four rows per group; few long rows: a group per row
    p = H.Plan(g(8192, 4096, 1))
    assert p.kernel_name == "gemm_skinny<rows of X>" and p.launch_shape()[0] == (2048, 1, 1) and p.workspace_bytes == 0
    p = H.Plan(g(256, 131072, 1))
    assert p.kernel_name == "gemm_skinny<rows of X>" and p.launch_shape()[0] == (256, 1, 1)
    assert H.Plan(g(8192, 4096, 8, wstride=(1, 4096))).kernel_name == "gemm_skinny<rows of X,wt>"
    # a vector times a linear layer's transposed weight: the rows of W are streamed
    p = H.Plan(g(1, 4096, 8192, wstride=(1, 4096)))
    assert p.kernel_name == "gemm_skinny<rows of W>" and p.launch_shape()[0] == (2048, 1, 1)
    # a vector times a row-major W: its rows streamed along n, K in slices with a finishing pass (one float per slice and output)
    p = H.Plan(g(1, 4096, 8192))
    assert p.kernel_name == "gemm_skinny_cols" and p.launch_shape()[0] == (32, 32, 1) and p.workspace_bytes == 32 * 1 * 8192 * 4
    # not: 9 columns, a softmax or dropout behind it, K % 4, small operands, N % 4 under a small M and a row-major W
    for d in (g(8192, 4096, 9), g(1, 4096, 8190), g(8192, 4096, 4, red=H.HPCT_RED_SOFTMAX_LAST),
              g(8192, 4096, 4, epi=(H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_DROPOUT_HASH)), g(8192, 4098, 1), g(512, 512, 1)):
        assert not H.Plan(d).kernel_name.startswith("gemm_skinny")


def test_gemm_strided_x_plans():
    def g(xstride, M=512, K=256, N=512):
        return H.op_desc(H.HPCT_ANCHOR_GEMM, [H.HPCT_EPI_BIAS_COL], H.HPCT_RED_NONE, 0,
                         [H.tensor_desc((M, K), xstride), (K, N), (N,)], [(M, N)])
    assert H.Plan(g(None)).workspace_bytes == 0
    # the transpose of a [K,M] array, a slice of a wider matrix: a row-major copy of X in the workspace
    assert H.Plan(g((1, 512))).workspace_bytes == 512 * 256 * 4
    assert H.Plan(g((300, 1))).workspace_bytes == 512 * 256 * 4
    # behind the K slices' partial products, on a 256-byte boundary
    p = H.Plan(g((1, 256), M=256, K=2048, N=256))
    q = H.Plan(g(None, M=256, K=2048, N=256))
    assert q.workspace_bytes > 0 and p.workspace_bytes == (q.workspace_bytes + 255) // 256 * 256 + 256 * 2048 * 4
    assert p.kernel_name == q.kernel_name


def test_gemm_activation_plans():
    def g(epi):
        return H.op_desc(H.HPCT_ANCHOR_GEMM, list(epi), H.HPCT_RED_NONE, 0, [(512, 256), (256, 512), (512,)], [(512, 512)])
    for act in (H.HPCT_EPI_RELU, H.HPCT_EPI_RELU6, H.HPCT_EPI_GELU_TANH, H.HPCT_EPI_SIGMOID, H.HPCT_EPI_TANH):
        H.Plan(g([H.HPCT_EPI_BIAS_COL, act]))
        H.Plan(g([H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_SCALE_CONST, act, H.HPCT_EPI_DROPOUT_HASH]))
        expect(H.HPCT_ERR_UNSUPPORTED, g([act, H.HPCT_EPI_BIAS_COL]))                       # the activation comes after the bias
    expect(H.HPCT_ERR_UNSUPPORTED, g([H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU, H.HPCT_EPI_TANH]))   # one activation only
    expect(H.HPCT_ERR_UNSUPPORTED, g([H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_SIN]))
    # the conv chains keep RELU and RELU6 only
    def c(epi):
        return H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, list(epi), H.HPCT_RED_NONE, 0, [(2, 8, 12, 12), (16, 8, 3, 3), (16,)], [(2, 16, 12, 12)],
                         stride_hw=(1, 1), pad_hw=(1, 1))
    H.Plan(c([H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU6]))
    expect(H.HPCT_ERR_UNSUPPORTED, c([H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_GELU_TANH]))
    expect(H.HPCT_ERR_UNSUPPORTED, c([H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU, H.HPCT_EPI_RELU6]))


def test_batched_gemm_plans():
    def g(xs, ws, os_, epi=(H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU), red=H.HPCT_RED_NONE, wstride=None):
        return H.op_desc(H.HPCT_ANCHOR_GEMM, list(epi), red, 0, [xs, H.tensor_desc(ws, wstride), (ws[-1],)], [os_])
    # 16 products of 256 x 128 x 256: tiles of all the matrices fill one grid
    p = H.Plan(g((16, 256, 128), (16, 128, 256), (16, 256, 256)))
    assert p.kernel_name == "gemm_tile64" and p.launch_shape()[0] == (16 * 4 * 4, 1, 1) and p.workspace_bytes == 0
    # small matrices: the batch in grid.z of the kernel whose waves share K, or (short K) of the 16-row kernel
    p = H.Plan(g((3, 64, 256), (3, 256, 256), (3, 64, 256), red=H.HPCT_RED_SOFTMAX_LAST))
    assert p.kernel_name == "gemm_ksplit16<32>" and p.launch_shape()[0] == (8, 4, 3)
    p = H.Plan(g((3, 64, 32), (3, 32, 256), (3, 64, 256), red=H.HPCT_RED_SOFTMAX_LAST))
    assert p.kernel_name == "gemm_rows16<256>" and p.launch_shape()[0] == (4, 1, 3)
    # a short K: no LDS staging
    p = H.Plan(g((64, 512, 64), (64, 64, 512), (64, 512, 512)))
    assert p.kernel_name == "gemm_direct" and p.launch_shape() == ((64 * 4 * 4, 1, 1), (256, 1, 1), 0) and p.workspace_bytes == 0
    assert H.Plan(g((16384, 32), (32, 16384), (16384, 16384))).kernel_name == "gemm_direct"
    assert H.Plan(g((16384, 32), (32, 16384), (16384, 16384), wstride=(1, 32))).kernel_name == "gemm_tile128<wt>"   # row-major W only
    assert H.Plan(g((256, 64, 64), (256, 64, 64), (256, 64, 64))).kernel_name == "gemm_tile64"   # matrices smaller than its tile
    assert H.Plan(g((16384, 34), (34, 16384), (16384, 16384))).kernel_name == "gemm_tile128"     # K % 4
    assert H.Plan(g((16384, 68), (68, 16384), (16384, 16384))).kernel_name == "gemm_tile128"     # K > 64
    assert H.Plan(g((1024, 32), (32, 1024), (1024, 1024))).kernel_name == "gemm_tile64"          # 64 tiles of 128 x 128
    # per-batch transposed W
    p = H.Plan(g((16, 256, 128), (16, 128, 256), (16, 256, 256), wstride=(128 * 256, 1, 128)))
    assert p.kernel_name == "gemm_tile64<wt>"
    # one W for all: a single tall product
    p = H.Plan(g((16, 256, 128), (128, 256), (16, 256, 256)))
    assert p.kernel_name == "gemm_tile64" and p.launch_shape()[0] == (64 * 4, 1, 1)
    expect(H.HPCT_ERR_SHAPE_MISMATCH, g((16, 256, 128), (15, 128, 256), (16, 256, 256)))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, g((16, 256, 128), (16, 128, 256), (16 * 256, 256)))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, g((256, 128), (16, 128, 256), (16, 256, 256)))
    expect(H.HPCT_ERR_UNSUPPORTED, g((16, 256, 128), (16, 128, 256), (16, 256), red=H.HPCT_RED_MEAN_LAST))
    expect(H.HPCT_ERR_UNSUPPORTED, g((16, 256, 128), (16, 128, 256), (16, 256, 256),
                                     epi=(H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_DROPOUT_HASH)))


def eltwise_desc(shape, sa, sb, add=True, relu=False, out_shape=None):
    epi = [H.HPCT_EPI_ADD_TENSOR if add else H.HPCT_EPI_MUL_TENSOR] + ([H.HPCT_EPI_RELU] if relu else [])
    return H.op_desc(H.HPCT_ANCHOR_NONE, epi, H.HPCT_RED_NONE, 0, [H.tensor_desc(shape, sa), H.tensor_desc(shape, sb)],
                     [out_shape or shape])


def test_eltwise_plans_and_errors():
    # matrix + bias row broadcast over the rows: the last dim is contiguous in A and B -> 128-bit access
    p = H.Plan(eltwise_desc((8192, 4096), (4096, 1), (0, 1), relu=True))
    assert p.kernel_name == "eltwise_binary<vec4>" and p.workspace_bytes == 0
    # per-row scalar broadcast along the last dim is vectorised too; a transposed operand is not
    assert H.Plan(eltwise_desc((8192, 4096), (4096, 1), (1, 0), add=False)).kernel_name == "eltwise_binary<vec4>"
    assert H.Plan(eltwise_desc((64, 64), (64, 1), (1, 64))).kernel_name == "eltwise_binary<scalar>"
    assert H.Plan(eltwise_desc((5, 7), (7, 1), (7, 1))).kernel_name == "eltwise_binary<scalar>"
    expect(H.HPCT_ERR_SHAPE_MISMATCH, eltwise_desc((4, 8), (8, 1), (8, 1), out_shape=(8, 4)))
    d = eltwise_desc((4, 8), (8, 1), (8, 1)); d.in_[1] = H.tensor_desc((4, 4), (4, 1))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = eltwise_desc((4, 8), (8, 1), (8, 1)); d.n_epi = 2; d.epi[1] = H.HPCT_EPI_GELU_TANH   # any unary step may follow
    assert H.Plan(d).kernel_name == "eltwise_binary<vec4>"
    d = eltwise_desc((4, 8), (8, 1), (8, 1)); d.n_epi = 2; d.epi[1] = H.HPCT_EPI_BIAS_COL    # ... nothing else
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = eltwise_desc((4, 8), (8, 1), (8, 1)); d.n_epi = 2; d.epi[1] = H.HPCT_EPI_SUB_TENSOR  # one tensor operand only
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = eltwise_desc((4, 8), (8, 1), (8, 1)); d.reduce = H.HPCT_RED_SOFTMAX_LAST
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = eltwise_desc((4, 8), (8, 1), (8, 1)); d.n_in = 1
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.epi[0] = H.HPCT_EPI_ADD_TENSOR          # not after an anchor
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def test_eltwise_chain_plans():
    un = [H.HPCT_EPI_SCALE_CONST, H.HPCT_EPI_SIN, H.HPCT_EPI_COS, H.HPCT_EPI_EXP, H.HPCT_EPI_TANH, H.HPCT_EPI_SIGMOID,
          H.HPCT_EPI_SQRT, H.HPCT_EPI_RELU]
    # one operand, eight steps; a strided slice runs through the scalar variant
    d = H.op_desc(H.HPCT_ANCHOR_NONE, un, H.HPCT_RED_NONE, 0, [(8192, 4096)], [(8192, 4096)], scale=0.5)
    p = H.Plan(d)
    assert p.kernel_name == "eltwise_unary<vec4>" and p.workspace_bytes == 0
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SQRT], H.HPCT_RED_NONE, 0, [H.tensor_desc((3, 5), (10, 2))], [(3, 5)])
    assert H.Plan(d).kernel_name == "eltwise_unary<scalar>"
    for b in (H.HPCT_EPI_SUB_TENSOR, H.HPCT_EPI_DIV_TENSOR):
        d = H.op_desc(H.HPCT_ANCHOR_NONE, [b, H.HPCT_EPI_SQRT], H.HPCT_RED_NONE, 0, [(16, 8), H.tensor_desc((16, 8), (0, 1))], [(16, 8)])
        assert H.Plan(d).kernel_name == "eltwise_binary<vec4>"
    # RELU alone on a contiguous NCHW tensor stays with the per-channel chain; on any other view it is a step
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0, [(2, 3, 4, 4)], [(2, 3, 4, 4)])
    assert H.Plan(d).kernel_name.startswith("affine_planes")
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0, [(7, 9)], [(7, 9)])
    assert H.Plan(d).kernel_name == "eltwise_unary<scalar>"
    # a unary chain takes one input; the steps are not epilogues of an anchor; the tensor op must come first
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SIN], H.HPCT_RED_NONE, 0, [(7, 9), (7, 9)], [(7, 9)])
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = cfg_desc(1); d.epi[1] = H.HPCT_EPI_SIN
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SIN, H.HPCT_EPI_ADD_TENSOR], H.HPCT_RED_NONE, 0, [(7, 9), (7, 9)], [(7, 9)])
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_SIN], H.HPCT_RED_NONE, 0, [(7, 9)], [(7, 9)]); d.epi[0] = 99
    expect(H.HPCT_ERR_BAD_DESC, d)


def dw_desc(shape=(32, 96, 56, 56), R=3, stride=1, pad=1, dil=1, act=None, groups=None, K=None, wt_c=1, pool=False):
    Nb, Cc, Hh, Ww = shape
    K = Cc if K is None else K
    Ho = (Hh + 2 * pad - (R - 1) * dil - 1) // stride + 1
    Wo = (Ww + 2 * pad - (R - 1) * dil - 1) // stride + 1
    epi = [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_SCALE_SHIFT_CH] + ([act] if act is not None else [])
    return H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, epi, H.HPCT_RED_MAXPOOL2_HW if pool else H.HPCT_RED_NONE, 0,
                     [shape, (K, wt_c, R, R), (K,), (K,), (K,)], [(Nb, K, Ho // 2, Wo // 2) if pool else (Nb, K, Ho, Wo)],
                     stride_hw=(stride, stride), pad_hw=(pad, pad), dilation_hw=(dil, dil),
                     groups=Cc if groups is None else groups)


def test_conv_few_input_channels_plans():
    def cd(shape, K, stride=1, pad=1, pool=False):
        Nb, Cc, Hh, Ww = shape
        Ho = (Hh + 2 * pad - 3) // stride + 1
        Wo = (Ww + 2 * pad - 3) // stride + 1
        return H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU],
                         H.HPCT_RED_MAXPOOL2_HW if pool else H.HPCT_RED_NONE, 0, [shape, (K, Cc, 3, 3), (K,)],
                         [(Nb, K, Ho // 2, Wo // 2) if pool else (Nb, K, Ho, Wo)], stride_hw=(stride, stride), pad_hw=(pad, pad))
    # a network's first layer: a wave per 32 channels x 128 pixels x 4 rows, no LDS
    p = H.Plan(cd((32, 3, 224, 224), 64))
    assert p.kernel_name == "conv3x3_fewc" and p.launch_shape() == ((32 * 56 * 2 * 2 // 4, 1, 1), (256, 1, 1), 0)
    assert H.Plan(cd((2, 1, 28, 100), 32)).kernel_name == "conv3x3_fewc"
    # a ResNet's: 7x7 / 2 / pad 3, a wave per 32 channels x 128 output pixels x 2 rows
    d7 = H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0,
                   [(32, 3, 224, 224), (64, 3, 7, 7), (64,)], [(32, 64, 112, 112)], stride_hw=(2, 2), pad_hw=(3, 3))
    p = H.Plan(d7)
    assert p.kernel_name == "conv7x7s2_fewc" and p.launch_shape() == ((32 * 112 * 1 * 2 // 4, 1, 1), (256, 1, 1), 0)
    # a MobileNet's: 3x3 / 2 / pad 1
    p = H.Plan(cd((32, 3, 224, 224), 32, stride=2))
    assert p.kernel_name == "conv3x3_fewc<stride2>" and p.launch_shape()[0] == (32 * 112 * 1 * 1 // 4, 1, 1)   # a row per wave: few waves otherwise
    for d in (cd((32, 3, 224, 224), 48), cd((32, 3, 224, 224), 64, stride=3), cd((32, 3, 224, 224), 64, pad=0), cd((32, 3, 224, 220), 64, stride=2),
              cd((32, 3, 224, 224), 64, pool=True), cd((32, 3, 224, 222), 64), cd((32, 5, 224, 224), 64), cd((2, 3, 32, 32), 64)):
        assert H.Plan(d).kernel_name.startswith("conv2d_nchw_mfma<3x3")


def test_conv_refuses_planes_beyond_its_32_bit_store_offsets():
    # the conv epilogue addresses a lane's element inside a group of 8 output channels with a 32-bit byte offset:
    # more than 2^27 output pixels per channel are refused when the plan is made (8 input channels: the MFMA kernel)
    def cd(Hh, Ww):
        return H.op_desc(H.HPCT_ANCHOR_CONV2D_NCHW, [H.HPCT_EPI_BIAS_COL, H.HPCT_EPI_RELU], H.HPCT_RED_NONE, 0,
                         [(1, 8, Hh, Ww), (2, 8, 3, 3), (2,)], [(1, 2, Hh, Ww)], stride_hw=(1, 1), pad_hw=(1, 1))
    assert H.Plan(cd(11000, 12000)).kernel_name.startswith("conv2d_nchw_mfma<3x3")   # 1.32e8 <= 2^27 = 1.34e8
    e = expect(H.HPCT_ERR_UNSUPPORTED, cd(11500, 12000))
    assert "2^27" in e.message


def gn_desc(shape=(32, 64, 56, 56), groups=8, affine=True, relu=False, rbe=1, eps=1e-5):
    Cc = shape[1]
    ins = [shape] + ([(Cc,), (Cc,)] if affine else [])
    return H.op_desc(H.HPCT_ANCHOR_NONE, [H.HPCT_EPI_RELU] if relu else [], H.HPCT_RED_GROUPNORM_NCHW, rbe, ins, [shape],
                     eps=eps, groups=groups)


def test_rmsnorm_plans_and_errors():
    def r(M, N, gamma=True, epi=(), eps=1e-6):
        return H.op_desc(H.HPCT_ANCHOR_NONE, list(epi), H.HPCT_RED_RMSNORM_LAST, 0, [(M, N)] + ([(N,)] if gamma else []), [(M, N)], eps=eps)
    assert H.Plan(r(8192, 4096)).kernel_name == "rmsnorm_rows_persist"
    assert H.Plan(r(8192, 1024, gamma=False)).kernel_name == "rmsnorm_rows_vec<wave-per-row>"
    assert H.Plan(r(100, 1001)).kernel_name == "rmsnorm_rows_any"
    expect(H.HPCT_ERR_UNSUPPORTED, r(64, 64, epi=(H.HPCT_EPI_RELU,)))
    expect(H.HPCT_ERR_BAD_DESC, r(64, 64, eps=-1.0))
    d = r(64, 64); d.in_[1].shape[0] = 63
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = r(64, 64); d.n_in = 3
    expect(H.HPCT_ERR_BAD_DESC, d)


def test_groupnorm_plans_and_errors():
    # a work-group per (image, group); rows of up to 8192 elements stay in registers
    p = H.Plan(gn_desc())
    assert p.kernel_name == "groupnorm_rows<registers,1024>" and p.launch_shape()[:2] == ((32 * 8, 1, 1), (1024, 1, 1)) and p.workspace_bytes == 0
    assert H.Plan(gn_desc(shape=(2, 64, 112, 112), groups=8)).kernel_name == "groupnorm_rows<three passes>"
    assert H.Plan(gn_desc(groups=32, relu=True)).kernel_name == "groupnorm_rows<registers>"
    p = H.Plan(gn_desc(groups=64, affine=False))                       # instance normalisation
    assert p.kernel_name == "groupnorm_rows<registers>" and p.launch_shape()[0] == (32 * 64, 1, 1)
    assert H.Plan(gn_desc(shape=(2, 6, 7, 9), groups=3)).kernel_name == "groupnorm_rows_any"
    expect(H.HPCT_ERR_BAD_DESC, gn_desc(groups=0))
    expect(H.HPCT_ERR_BAD_DESC, gn_desc(groups=5))                     # does not divide 64
    expect(H.HPCT_ERR_BAD_DESC, gn_desc(eps=-1.0))
    expect(H.HPCT_ERR_UNSUPPORTED, gn_desc(relu=True, rbe=0))
    d = gn_desc(); d.epi[0] = H.HPCT_EPI_GELU_TANH; d.n_epi = 1
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = gn_desc(); d.in_[1].shape[0] = 63
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = gn_desc(); d.n_in = 2
    expect(H.HPCT_ERR_BAD_DESC, d)
    d = gn_desc(); d.out[0].shape[3] = 55
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)


def pool_desc(shape, k, stride, pad, out_shape=None, epi=()):
    Nb, Cc, Hh, Ww = shape
    if out_shape is None:
        out_shape = (Nb, Cc, (Hh + 2 * pad - k) // stride + 1, (Ww + 2 * pad - k) // stride + 1)
    return H.op_desc(H.HPCT_ANCHOR_NONE, list(epi), H.HPCT_RED_MAXPOOL_HW, 0, [shape], [out_shape], stride_hw=(stride, stride),
                     pad_hw=(pad, pad), window_hw=(k, k))


def test_maxpool_plans_and_errors():
    # a ResNet's pooling: 3x3 / 2 / pad 1 on 112 x 112: a wave per 56 output columns x 8 output rows
    p = H.Plan(pool_desc((32, 64, 112, 112), 3, 2, 1))
    assert p.kernel_name == "maxpool3x3_rows<stride2>" and p.launch_shape() == ((32 * 64 * 7 // 4, 1, 1), (256, 1, 1), 0)
    assert H.Plan(pool_desc((8, 16, 56, 56), 3, 1, 1)).kernel_name == "maxpool3x3_rows"
    # narrow maps keep the register kernel down to three computing lanes (12 output columns)
    assert H.Plan(pool_desc((8, 16, 28, 28), 3, 1, 1)).kernel_name == "maxpool3x3_rows"
    assert H.Plan(pool_desc((8, 16, 24, 24), 3, 2, 1)).kernel_name == "maxpool3x3_rows<stride2>"
    assert H.Plan(pool_desc((8, 16, 8, 8), 3, 1, 1)).kernel_name == "maxpool_any"
    # 2x2 / 2 / 0 is the VGG pooling's kernel
    assert H.Plan(pool_desc((32, 64, 56, 56), 2, 2, 0)).kernel_name == "maxpool2_planes<vec4>"
    # anything else: an output per thread
    for (shape, k, s, pad) in [((2, 3, 30, 30), 3, 2, 1), ((2, 3, 112, 112), 3, 2, 0), ((2, 3, 57, 57), 5, 3, 2), ((1, 1, 7, 7), 7, 1, 0),
                               ((2, 3, 112, 110), 3, 2, 1)]:
        assert H.Plan(pool_desc(shape, k, s, pad)).kernel_name == "maxpool_any"
    # average pooling: the same kernels' AVG instances; 2x2 has no kernel of its own
    def avg(shape, k, s_, pad):
        d = pool_desc(shape, k, s_, pad); d.reduce = H.HPCT_RED_AVGPOOL_WIN_HW
        return H.Plan(d).kernel_name
    assert avg((32, 64, 112, 112), 3, 2, 1) == "avgpool3x3_rows<stride2>" and avg((8, 16, 56, 56), 3, 1, 1) == "avgpool3x3_rows"
    assert avg((32, 64, 56, 56), 2, 2, 0) == "avgpool_any" and avg((2, 3, 57, 57), 5, 3, 2) == "avgpool_any"
    expect(H.HPCT_ERR_BAD_DESC, pool_desc((2, 3, 8, 8), 3, 2, 3))                    # padding as large as the window
    expect(H.HPCT_ERR_BAD_DESC, pool_desc((2, 3, 8, 8), 0, 1, 0, out_shape=(2, 3, 8, 8)))
    expect(H.HPCT_ERR_BAD_DESC, pool_desc((2, 3, 8, 8), 3, 0, 1, out_shape=(2, 3, 8, 8)))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, pool_desc((2, 3, 8, 8), 3, 2, 1, out_shape=(2, 3, 5, 4)))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, pool_desc((2, 3, 2, 2), 5, 1, 0, out_shape=(2, 3, 1, 1)))
    expect(H.HPCT_ERR_UNSUPPORTED, pool_desc((2, 3, 8, 8), 3, 2, 1, epi=(H.HPCT_EPI_RELU,)))
    d = pool_desc((2, 3, 8, 8), 3, 2, 1); d.window_hw[1] = 2
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = pool_desc((2, 3, 8, 8), 3, 2, 1); d.anchor = H.HPCT_ANCHOR_GEMM
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def test_depthwise_conv_plans():
    # 3x3, stride 1, pad 1, rows of 56: the register variant, a wave per 16 rows of a plane, four waves per group
    p = H.Plan(dw_desc(act=H.HPCT_EPI_RELU6))
    assert p.kernel_name == "dwconv3x3_rows" and p.workspace_bytes == 0
    assert p.launch_shape() == ((32 * 96 * 4 // 4, 1, 1), (256, 1, 1), 0)
    # wide rows: segments of 56 columns
    assert H.Plan(dw_desc(shape=(8, 32, 112, 112))).launch_shape()[0] == (8 * 32 * 7 * 2 // 4, 1, 1)
    # rows that would leave most lanes idle, other strides, pads and filters: through LDS
    p = H.Plan(dw_desc(shape=(32, 96, 28, 28), act=H.HPCT_EPI_RELU6))
    assert p.kernel_name == "dwconv_planes<3x3>" and p.launch_shape()[0] == (32 * 96, 1, 1) and p.launch_shape()[1] == (256, 1, 1)
    assert H.Plan(dw_desc(pad=0)).kernel_name == "dwconv_planes<3x3>"
    assert H.Plan(dw_desc(shape=(2, 4, 56, 54))).kernel_name == "dwconv_planes<3x3>"
    # larger planes are cut into bands of rows
    # the same at stride 2, when the output rows fill the lanes: 56 output columns from 112
    p = H.Plan(dw_desc(shape=(32, 96, 112, 112), stride=2))
    assert p.kernel_name == "dwconv3x3_rows<stride2>" and p.launch_shape() == ((32 * 96 * 4 // 4, 1, 1), (256, 1, 1), 0)
    assert H.Plan(dw_desc(stride=2)).kernel_name == "dwconv_planes<3x3>"           # 28 output columns
    p = H.Plan(dw_desc(shape=(32, 32, 112, 112), R=5, pad=2, act=H.HPCT_EPI_RELU))
    assert p.launch_shape()[0][0] % (32 * 32) == 0 and p.launch_shape()[0][0] > 32 * 32 and p.launch_shape()[2] <= 16 * 1024
    assert H.Plan(dw_desc(R=5, pad=2, stride=2)).kernel_name == "dwconv_planes<5x5>"
    assert H.Plan(dw_desc(R=7, pad=3, shape=(2, 8, 30, 30))).kernel_name == "dwconv_planes<7x7>"
    assert H.Plan(dw_desc(R=1, pad=0)).kernel_name == "dwconv_planes<1x1>"
    # groups = 0 / 1 is the dense conv: wt must then be [K, C, R, R]
    expect(H.HPCT_ERR_SHAPE_MISMATCH, dw_desc(groups=1))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, dw_desc(groups=0))
    expect(H.HPCT_ERR_SHAPE_MISMATCH, dw_desc(wt_c=2))                       # depthwise filters have one input channel
    expect(H.HPCT_ERR_UNSUPPORTED, dw_desc(groups=48, wt_c=2))                # grouped, not depthwise
    expect(H.HPCT_ERR_UNSUPPORTED, dw_desc(K=192))                            # channel multiplier 2
    expect(H.HPCT_ERR_UNSUPPORTED, dw_desc(pool=True))
    expect(H.HPCT_ERR_UNSUPPORTED, dw_desc(R=3, pad=3))
    expect(H.HPCT_ERR_BAD_DESC, dw_desc(groups=-1))
    # RELU6 takes the place of RELU in the dense conv chain too, not beside it
    d = conv_block_desc(); d.epi[2] = H.HPCT_EPI_RELU6
    assert H.Plan(d).kernel_name == "conv2d_nchw_mfma<3x3,pipelined,maxpool2>"
    d = conv_block_desc(); d.n_epi = 4; d.epi[3] = H.HPCT_EPI_RELU6
    expect(H.HPCT_ERR_UNSUPPORTED, d)


def convt_desc(shape=(32, 128, 28, 28), K=64, R=3, stride=2, pad=1, dil=1, act=None, wt_c=None, out=None):
    Nb, Cc, Hh, Ww = shape
    Ho = (Hh - 1) * stride - 2 * pad + (R - 1) * dil + 1
    Wo = (Ww - 1) * stride - 2 * pad + (R - 1) * dil + 1
    epi = [H.HPCT_EPI_BIAS_COL] + ([act] if act is not None else [])
    return H.op_desc(H.HPCT_ANCHOR_CONVT2D_NCHW, epi, H.HPCT_RED_NONE, 0,
                     [shape, (Cc if wt_c is None else wt_c, K, R, R), (K,)], [out or (Nb, K, Ho, Wo)],
                     stride_hw=(stride, stride), pad_hw=(pad, pad), dilation_hw=(dil, dil))


def test_conv_transpose_plans():
    p = H.Plan(convt_desc(act=H.HPCT_EPI_RELU))
    # workspace: the flipped filter (rounded to 256 bytes) and the zero-dilated input [32,128,55,55]
    assert p.workspace_bytes == 64 * 128 * 9 * 4 + 32 * 128 * 55 * 55 * 4
    assert p.kernel_name.startswith("conv2d_nchw_mfma<3x3")
    # stride 1 needs only the filter
    p = H.Plan(convt_desc(shape=(2, 8, 10, 10), K=5, stride=1))
    assert p.workspace_bytes == (5 * 8 * 9 * 4 + 255) // 256 * 256
    assert H.Plan(convt_desc(R=5, pad=2)).workspace_bytes > 0
    expect(H.HPCT_ERR_SHAPE_MISMATCH, convt_desc(wt_c=64))                         # wt is [C,K,R,S]: input channels first
    expect(H.HPCT_ERR_SHAPE_MISMATCH, convt_desc(out=(32, 64, 56, 56)))            # (28-1)*2 - 2 + 3 = 55
    expect(H.HPCT_ERR_UNSUPPORTED, convt_desc(R=3, pad=3))
    d = convt_desc(); d.reduce = H.HPCT_RED_MAXPOOL2_HW
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = convt_desc(); d.groups = 2
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = convt_desc(); d.stride_hw[1] = 1
    expect(H.HPCT_ERR_UNSUPPORTED, d)
    d = convt_desc(); d.anchor = 5
    expect(H.HPCT_ERR_BAD_DESC, d)


def test_maxpool_alone_plans():
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_MAXPOOL2_HW, 0, [(32, 64, 56, 56)], [(32, 64, 28, 28)])
    assert H.Plan(d).kernel_name == "maxpool2_planes<vec4>"
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_MAXPOOL2_HW, 0, [(2, 3, 7, 9)], [(2, 3, 3, 4)])
    assert H.Plan(d).kernel_name == "maxpool2_planes<scalar>"
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_MAXPOOL2_HW, 0, [(2, 3, 7, 9)], [(2, 3, 4, 5)])
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_MAXPOOL2_HW, 0, [(2, 3, 1, 9)], [(2, 3, 1, 4)])
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
    d = H.op_desc(H.HPCT_ANCHOR_NONE, [], H.HPCT_RED_MAXPOOL2_HW, 0, [(8, 8)], [(4, 4)])
    expect(H.HPCT_ERR_SHAPE_MISMATCH, d)
