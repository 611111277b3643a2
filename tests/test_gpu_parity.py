"""GPU parity tests: the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs.

Small and medium geometries are compared element by element over whole tensors (sizes span
several tiles of the matrix-core kernels plus ragged tails); the full-size Jasper-shaped
workloads are compared on sampled output elements the oracle evaluates one by one.  Gate:
max |g-o|/(|o|+rms(o)) <= 1e-2 for bf16 storage (float32 accumulation), <= 1e-5 for float32
storage; bf16 results must also have a relative RMS error <= 3e-3.

Backward checks take the saved forward output from the input recipe (or from the oracle's own
forward, rounded to the storage type on the host), never from the GPU.
"""
import numpy as np
import pytest

import _util as U
from oracle import conv1d_oracle as orc
from paper_1909_09577_amd import binding as nm
from paper_1909_09577_amd import inputs as syn
from paper_1909_09577_amd.inputs import LayerCfg

pytestmark = pytest.mark.gpu


def run_fwd(cfg, inp, dtype, force_direct):
    y = nm.nm_conv1d_block_fwd(
        U.to_dev(inp, "x", dtype), U.to_dev(inp, "w", dtype),
        U.to_dev(inp, "scale", dtype) if cfg.affine else None,
        U.to_dev(inp, "shift", dtype) if cfg.affine else None,
        U.to_dev(inp, "residual", dtype) if cfg.residual else None,
        relu=cfg.relu, force_direct=force_direct, **U.geom_kw(cfg))
    return y


def run_bwd(cfg, inp, dtype, force_direct, y_saved_dev):
    scale = U.to_dev(inp, "scale", dtype) if cfg.affine else None
    dy, w, x = U.to_dev(inp, "dy", dtype), U.to_dev(inp, "w", dtype), U.to_dev(inp, "x", dtype)
    ysv = y_saved_dev if cfg.relu else None
    dx, dres = nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=ysv, scale=scale, relu=cfg.relu, want_dres=True,
                                     force_direct=force_direct, **U.geom_kw(cfg))
    dw = nm.nm_conv1d_bwd_weight(x, dy, cfg.K, y=ysv, scale=scale, relu=cfg.relu, force_direct=force_direct,
                                 **U.geom_kw(cfg))
    return dx, dw, dres


def L(name, B, Cin, Cout, T, K, stride=1, dilation=1, pad=0, affine=True, relu=True, residual=False, seed=11):
    return LayerCfg(name, B, Cin, Cout, T, K, stride, dilation, pad, affine, relu, residual, seed,
                    T_out=orc.out_len(T, K, stride, dilation, pad))


# Odd shapes: ragged channel counts and lengths, strides, dilations, pad 0 / larger than needed,
# K = 1 and even K, every epilogue combination.
SMALL = [
    L("s_basic", 2, 8, 8, 40, 3, pad=1, residual=True),
    L("s_noepi", 1, 5, 7, 33, 5, pad=2, affine=False, relu=False),
    L("s_k1", 3, 16, 29, 50, 1),
    L("s_k2_even", 2, 6, 10, 37, 2, pad=1),
    L("s_stride2", 2, 12, 20, 101, 11, stride=2, pad=5),
    L("s_stride3_d2", 1, 7, 9, 64, 4, stride=3, dilation=2, pad=3, residual=True),
    L("s_dil3_pad0", 2, 9, 5, 70, 5, dilation=3, pad=0),
    L("s_bigpad", 1, 4, 6, 20, 3, pad=7, relu=False, residual=True),
    L("s_t1", 2, 3, 4, 1, 1),
    L("s_affine_only", 2, 10, 12, 45, 7, pad=3, relu=False),
]

# Medium: several 64x160 tiles with ragged tails in every dimension (oracle: a few seconds each).
MEDIUM = [
    L("m_ragged", 3, 72, 100, 336, 11, pad=5, residual=True),
    L("m_odd_len", 2, 40, 48, 333, 7, pad=3, residual=True),      # T % 8 != 0: plain kernels
    L("m_two_tiles", 2, 128, 192, 320, 17, pad=8, residual=True),
    L("m_dil2", 2, 96, 80, 248, 9, dilation=2, pad=8),
    L("m_pad_not_same", 2, 64, 64, 176, 5, pad=6),               # T_out = T + 8
    L("m_k29_d2", 1, 48, 72, 240, 29, dilation=2, pad=28),
    L("m_k1_wide", 2, 200, 29, 400, 1, affine=False, relu=False),
    L("m_stride2_prolog", 2, 64, 96, 400, 11, stride=2, pad=5),
    L("m_cin_small", 2, 16, 64, 480, 5, pad=2),
    # the remaining Jasper filter widths, with 3, 5 and 2 reduction chunks (uneven over the four wavefronts)
    L("m_k13", 2, 96, 64, 320, 13, pad=6, residual=True),
    L("m_k21", 1, 160, 72, 328, 21, pad=10),
    L("m_k25", 1, 64, 128, 336, 25, pad=12, residual=True),
    # pointwise layers on the K=1 GEMM kernels: ragged channel tiles, a length that is no multiple of the 80-step unit,
    # with and without the mask pass
    L("m_k1_ragged", 3, 136, 200, 336, 1, residual=True),
    L("m_k1_proj", 5, 320, 264, 88, 1, relu=False),
    L("m_k1_tiles", 2, 384, 520, 400, 1),
    # the 512-channel x 128-step tile of the K=1 kernel: forward (1000 rows) resp. input gradient (1000 rows), ragged
    # in rows, time (200 = 128 + 72) and reduction length (136 = 2 stages of 64 + 8)
    L("m_k1_bigtile", 2, 136, 1000, 200, 1, residual=True),
    L("m_k1_bigtile_t", 2, 1000, 136, 200, 1),
    # pointwise layers with at most 32 output channels: the forward pass streams x once (decoder-style kernel)
    L("m_k1_skinny", 3, 96, 29, 328, 1, residual=True),
    L("m_k1_skinny32", 2, 160, 32, 136, 1, relu=False),
    L("m_k1_skinny5", 2, 64, 5, 264, 1),
]


FULL = [syn.JASPER_B1, syn.JASPER_B3, syn.EPILOG_A, syn.EPILOG_B, syn.EPILOG_C]


def takes_matrix_core_path(cfg):
    """The forward matrix-core kernel needs scratch for packed weights, the plain one none."""
    return nm.nm_conv1d_workspace_bytes(nm.NM_OP_FWD, *cfg.dims(), nm.NM_BF16, 0) > 0


def test_matrix_core_path_is_selected_for_the_jasper_shapes():
    for cfg in FULL + [syn.TINY] + [c for c in MEDIUM if c.name != "m_odd_len"]:
        assert takes_matrix_core_path(cfg), cfg.name
        assert nm.nm_conv1d_workspace_bytes(nm.NM_OP_FWD, *cfg.dims(), nm.NM_BF16, nm.NM_FORCE_DIRECT) == 0


def check_layer(cfg, dtype, force_direct):
    inp = syn.make_inputs(cfg, dtype)
    y = run_fwd(cfg, inp, dtype, force_direct)
    y_ref = U.oracle_fwd(cfg, inp)
    U.assert_close(U.to_host_f64(y), y_ref, dtype, f"{cfg.name} y")
    # backward: saved output = the oracle's forward rounded to storage on the host
    y_saved = U.round_to_storage(y_ref, dtype)
    dx, dw, dres = run_bwd(cfg, inp, dtype, force_direct, U.arr_to_dev(y_saved, dtype))
    dx_ref, dw_ref, dres_ref = U.oracle_bwd(cfg, inp, y_saved.astype(np.float64))
    U.assert_close(U.to_host_f64(dx), dx_ref, dtype, f"{cfg.name} dx")
    U.assert_close(U.to_host_f64(dw), dw_ref, dtype, f"{cfg.name} dw", rms_bound=U.RMS_DW_BF16)
    # dres = dy*[y>0] is exact in any precision
    np.testing.assert_array_equal(U.to_host_f64(dres), dres_ref)


@pytest.mark.parametrize("force_direct", [False, True], ids=["auto", "direct"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_small_shapes_full_tensor(cfg, dtype, force_direct):
    if dtype == "f32" and not force_direct:
        pytest.skip("float32 storage always takes the plain kernels")
    check_layer(cfg, dtype, force_direct)


@pytest.mark.parametrize("force_direct", [False, True], ids=["auto", "direct"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cfg", MEDIUM + [syn.TINY], ids=lambda c: c.name)
def test_medium_shapes_full_tensor(cfg, dtype, force_direct):
    if dtype == "f32" and not force_direct:
        pytest.skip("float32 storage always takes the plain kernels")
    check_layer(cfg, dtype, force_direct)


# 1280 output tiles of 64 channels x 160 steps on 256 CUs: every wavefront computes one tile on its
# own and every workgroup one more with its reduction split four ways -- both epilogues of the
# unrolled kernel, compared on the whole tensor (forward for 128->512, input gradient for 512->128).
PRIVATE_TILES = [
    L("p_fwd_1280_tiles", 20, 128, 512, 1280, 11, pad=5, residual=True),
    L("p_dgrad_1280_tiles", 20, 512, 128, 1280, 11, pad=5, residual=True),
]


@pytest.mark.parametrize("cfg", PRIVATE_TILES, ids=lambda c: c.name)
def test_private_and_shared_tiles_full_tensor(cfg):
    check_layer(cfg, "bf16", False)


# Shapes on which the weight gradient takes the kernel that splits the taps over the wavefronts
# (its planner wants the workgroups to fill 256 CUs in whole rounds: 8 x 32 = 256 output tiles here),
# one per tap-group size it is built for; K=25 runs as two groups (13 + 12), K=29 with dilation 2 as 15 + 14.
SHARED_WGRAD = [
    L("w_k11", 2, 1024, 512, 160, 11, pad=5, affine=False, relu=False),
    L("w_k13", 1, 1024, 512, 240, 13, pad=6, affine=False, relu=False),
    L("w_k17", 2, 1024, 512, 160, 17, pad=8, affine=False, relu=False),
    L("w_k21", 1, 1000, 500, 320, 21, pad=10, affine=False, relu=False),          # ragged channel tiles
    L("w_k25", 1, 1024, 512, 160, 25, pad=12, affine=False, relu=False),
    L("w_k29_d2", 1, 1024, 512, 160, 29, dilation=2, pad=28, affine=False, relu=False),
]
# the same geometries with the whole epilogue on (affine + ReLU + residual): the mask and the scale
# factor of dz then pass through the weight-gradient kernel's operand path
SHARED_WGRAD += [
    L(c.name + "_epi", c.B, c.Cin, c.Cout, c.T, c.K, dilation=c.dilation, pad=c.pad, affine=True, relu=True, residual=True,
      seed=12)
    for c in list(SHARED_WGRAD)
]


@pytest.mark.parametrize("cfg", SHARED_WGRAD, ids=lambda c: c.name)
def test_weight_gradient_with_taps_split_over_wavefronts(cfg):
    check_layer(cfg, "bf16", False)


def sample_indices(n_total, n, rng, extra=()):
    idx = rng.choice(n_total, size=min(n, n_total), replace=False)
    return np.unique(np.concatenate([idx, np.asarray(list(extra), dtype=np.int64)])).astype(np.int64)


def edge_indices(shape):
    """Flat indices of corners and tile-boundary positions of a 3-d tensor."""
    d0, d1, d2 = shape
    picks = []
    for a in {0, d0 - 1}:
        for b in {0, min(63, d1 - 1), min(64, d1 - 1), d1 - 1}:
            for c in {0, 1, min(159, d2 - 1), min(160, d2 - 1), d2 - 2 if d2 > 1 else 0, d2 - 1}:
                picks.append((a * d1 + b) * d2 + c)
    return picks


def check_sampled(cfg, n_act=4096, n_w=2048, seed=99):
    """One bf16 layer in the launch configuration of its full size; the oracle evaluates sampled
    elements (plus corners and tile edges) of each output tensor, dres is compared everywhere."""
    dtype = "bf16"
    rng = np.random.default_rng(seed)
    inp = syn.make_inputs(cfg, dtype)
    x64, w64 = inp["x"].astype(np.float64), inp["w"].astype(np.float64)
    scale = inp["scale"] if cfg.affine else None
    shift = inp["shift"] if cfg.affine else None
    res = inp["residual"] if cfg.residual else None
    kw = U.geom_kw(cfg)
    To = cfg.T_out

    y = U.to_host_f64(run_fwd(cfg, inp, dtype, False)).reshape(-1)
    idx = sample_indices(y.size, n_act, rng, edge_indices((cfg.B, cfg.Cout, To)))
    y_ref = orc.block_fwd_at(x64, w64, idx, scale, shift, res, cfg.relu, **kw)
    # rms of the whole output is estimated from the sample (the sample is uniform)
    U.assert_close(y[idx], y_ref, dtype, f"{cfg.name} y (sampled)")
    if cfg.relu:
        assert np.mean(y == 0) > 0.05 and np.mean(y > 0) > 0.05

    ysv = U.to_dev(inp, "y_saved", dtype)
    dx, dw, dres = run_bwd(cfg, inp, dtype, False, ysv)
    dz, dres_ref = orc.epilogue_bwd(inp["dy"], inp["y_saved"] if cfg.relu else None, scale, cfg.relu)
    np.testing.assert_array_equal(U.to_host_f64(dres), dres_ref)
    dx = U.to_host_f64(dx).reshape(-1)
    idx = sample_indices(dx.size, n_act, rng, edge_indices((cfg.B, cfg.Cin, cfg.T)))
    U.assert_close(dx[idx], orc.bwd_data_at(dz, w64, cfg.T, idx, **kw), dtype, f"{cfg.name} dx (sampled)")
    dw = U.to_host_f64(dw).reshape(-1)
    idx = sample_indices(dw.size, n_w, rng, [0, dw.size - 1, cfg.K - 1, cfg.Cin * cfg.K - 1])
    U.assert_close(dw[idx], orc.bwd_weight_at(x64, dz, cfg.K, idx, **kw), dtype, f"{cfg.name} dw (sampled)",
                   rms_bound=U.RMS_DW_BF16)


@pytest.mark.parametrize("cfg", FULL, ids=lambda c: c.name)
def test_full_size_workloads_full_tensor(cfg):
    """The named full-size bf16 workloads (B=32, T=800) in the launch configuration the benchmark times:
    every element of y, dx, dres and dw against the oracle (tens of seconds of oracle time each)."""
    check_layer(cfg, "bf16", False)


@pytest.mark.parametrize("cfg", FULL, ids=lambda c: c.name)
def test_full_size_workloads_sampled(cfg):
    """The same workloads with the saved output taken from the input recipe (not from the oracle's
    forward), on sampled elements plus corners and tile edges."""
    check_sampled(cfg)


def distinct_stack_layers():
    """One layer per distinct shape of the 64-layer 10x5 encoder stack (B=32, T=1600 -> 800), each
    with its own seed from the layer list; shapes already in FULL are left out."""
    seen = {(c.Cin, c.Cout, c.K, c.stride, c.dilation, c.residual, c.affine, c.relu) for c in FULL}
    out = []
    for entry in syn.jasper_10x5_layers():
        c = entry["cfg"]
        key = (c.Cin, c.Cout, c.K, c.stride, c.dilation, c.residual, c.affine, c.relu)
        if key not in seen:
            seen.add(key)
            out.append(c)
    return out


@pytest.mark.parametrize("cfg", distinct_stack_layers(), ids=lambda c: f"{c.name}_{c.Cin}to{c.Cout}_k{c.K}")
def test_stack_layer_shapes_sampled(cfg):
    """Every distinct layer shape of the full encoder stack at its full size, layer-local: seeded
    synthetic inputs per layer (no tensor travels from one layer's GPU result into the oracle)."""
    check_sampled(cfg, n_act=1024, n_w=512, seed=cfg.seed)


def test_full_size_f32_mode_sampled():
    """float32 storage at the B1 shape (smaller batch keeps the plain kernels quick)."""
    cfg = syn.shrink(syn.JASPER_B1, B=4)
    dtype = "f32"
    rng = np.random.default_rng(5)
    inp = syn.make_inputs(cfg, dtype)
    x64, w64 = inp["x"].astype(np.float64), inp["w"].astype(np.float64)
    kw = U.geom_kw(cfg)
    y = U.to_host_f64(run_fwd(cfg, inp, dtype, True)).reshape(-1)
    idx = sample_indices(y.size, 4096, rng)
    U.assert_close(y[idx], orc.block_fwd_at(x64, w64, idx, inp["scale"], inp["shift"], inp["residual"], True, **kw),
                   dtype, "f32 y")
    dx, dw, dres = run_bwd(cfg, inp, dtype, True, U.to_dev(inp, "y_saved", dtype))
    dz, dres_ref = orc.epilogue_bwd(inp["dy"], inp["y_saved"], inp["scale"], True)
    dx = U.to_host_f64(dx).reshape(-1)
    idx = sample_indices(dx.size, 4096, rng)
    U.assert_close(dx[idx], orc.bwd_data_at(dz, w64, cfg.T, idx, **kw), dtype, "f32 dx")
    dw = U.to_host_f64(dw).reshape(-1)
    idx = sample_indices(dw.size, 2048, rng)
    U.assert_close(dw[idx], orc.bwd_weight_at(x64, dz, cfg.K, idx, **kw), dtype, "f32 dw")


def check_f32_sampled(cfg, n_act, n_w, seed):
    """float32 storage (plain kernels), sampled outputs against the oracle at the 1e-5 gate."""
    dtype = "f32"
    rng = np.random.default_rng(seed)
    inp = syn.make_inputs(cfg, dtype)
    x64, w64 = inp["x"].astype(np.float64), inp["w"].astype(np.float64)
    scale = inp["scale"] if cfg.affine else None
    shift = inp["shift"] if cfg.affine else None
    res = inp["residual"] if cfg.residual else None
    kw = U.geom_kw(cfg)
    y = U.to_host_f64(run_fwd(cfg, inp, dtype, True)).reshape(-1)
    idx = sample_indices(y.size, n_act, rng, edge_indices((cfg.B, cfg.Cout, cfg.T_out)))
    U.assert_close(y[idx], orc.block_fwd_at(x64, w64, idx, scale, shift, res, cfg.relu, **kw), dtype, f"{cfg.name} f32 y")
    dx, dw, dres = run_bwd(cfg, inp, dtype, True, U.to_dev(inp, "y_saved", dtype))
    dz, dres_ref = orc.epilogue_bwd(inp["dy"], inp["y_saved"] if cfg.relu else None, scale, cfg.relu)
    np.testing.assert_array_equal(U.to_host_f64(dres), dres_ref)
    dx = U.to_host_f64(dx).reshape(-1)
    idx = sample_indices(dx.size, n_act, rng, edge_indices((cfg.B, cfg.Cin, cfg.T)))
    U.assert_close(dx[idx], orc.bwd_data_at(dz, w64, cfg.T, idx, **kw), dtype, f"{cfg.name} f32 dx")
    dw = U.to_host_f64(dw).reshape(-1)
    idx = sample_indices(dw.size, n_w, rng, [0, dw.size - 1, cfg.K - 1, cfg.Cin * cfg.K - 1])
    U.assert_close(dw[idx], orc.bwd_weight_at(x64, dz, cfg.K, idx, **kw), dtype, f"{cfg.name} f32 dw")


@pytest.mark.parametrize("cfg", [syn.JASPER_B3, syn.EPILOG_A], ids=lambda c: c.name)
def test_f32_mode_at_the_long_reduction_lengths(cfg):
    """float32 mode where its 1e-5 gate is hardest: 8 704-term (512 channels x 17 taps) and 22 272-term
    (768 x 29) forward / input-gradient sums, 25 600-term weight-gradient sums (full batch, B=32, T=800)."""
    check_f32_sampled(cfg, n_act=2048, n_w=1024, seed=7)


def test_pure_gradients_without_epilogue_and_accumulate():
    """y=NULL, scale=NULL: the backward entry points are plain convolution gradients;
    NM_ACCUM_DW adds into dw."""
    import torch
    cfg = L("pure", 2, 24, 40, 170, 7, pad=3, affine=False, relu=False)
    for dtype, fd in (("bf16", False), ("bf16", True), ("f32", True)):
        inp = syn.make_inputs(cfg, dtype)
        dx, dw, dres = run_bwd(cfg, inp, dtype, fd, None)
        dx_ref, dw_ref, dres_ref = U.oracle_bwd(cfg, inp, None)
        U.assert_close(U.to_host_f64(dx), dx_ref, dtype, "pure dx")
        U.assert_close(U.to_host_f64(dw), dw_ref, dtype, "pure dw")
        np.testing.assert_array_equal(U.to_host_f64(dres), inp["dy"].astype(np.float64))
        base = torch.full_like(dw, 0.5)
        acc = nm.nm_conv1d_bwd_weight(U.to_dev(inp, "x", dtype), U.to_dev(inp, "dy", dtype), cfg.K, dw=base.clone(),
                                      accumulate=True, force_direct=fd, **U.geom_kw(cfg))
        U.assert_close(U.to_host_f64(acc), dw_ref + 0.5, dtype, "accumulated dw")


@pytest.mark.parametrize("cfg", [
    L("acc_k1_proj", 2, 256, 384, 320, 1, relu=False),                   # a residual projection: the K=1 kernel
    L("acc_k1_few_outputs", 2, 200, 29, 328, 1, affine=False, relu=False),  # the store-bound kernel does not accumulate: the GEMM kernel takes it
    L("acc_k11", 2, 72, 100, 336, 11, pad=5, residual=True),             # unrolled engine, ragged channel tiles
    L("acc_k5", 2, 64, 64, 176, 5, pad=2),                               # tap-pair engine
    L("acc_odd_len", 2, 40, 48, 333, 7, pad=3),                          # plain kernels
    L("acc_stride2", 2, 64, 96, 400, 11, stride=2, pad=5),               # stride 2: accumulation on the plain kernel
], ids=lambda c: c.name)
def test_input_gradient_accumulation(cfg):
    """NM_ACCUM_DX: dx = round(dx_old + gradient), through nm_conv1d_bwd_data and nm_conv1d_bwd."""
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    kw = U.geom_kw(cfg)
    scale = U.to_dev(inp, "scale", dtype) if cfg.affine else None
    x, dy, w = U.to_dev(inp, "x", dtype), U.to_dev(inp, "dy", dtype), U.to_dev(inp, "w", dtype)
    ysv = U.to_dev(inp, "y_saved", dtype) if cfg.relu else None
    old = U.to_dev(inp, "x", dtype)  # any bf16 tensor of dx's shape serves as the old value
    dz, _ = orc.epilogue_bwd(inp["dy"], inp["y_saved"] if cfg.relu else None, inp["scale"] if cfg.affine else None, cfg.relu)
    ref = inp["x"].astype(np.float64) + orc.bwd_data(dz, inp["w"], cfg.T, **kw)
    dx1, _ = nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=ysv, scale=scale, dx=old.clone(), relu=cfg.relu, accumulate_dx=True, **kw)
    U.assert_close(U.to_host_f64(dx1), ref, dtype, f"{cfg.name} accumulated dx")
    dx2, _, _ = nm.nm_conv1d_bwd(x, dy, w, y=ysv, scale=scale, dx=old.clone(), relu=cfg.relu, accumulate_dx=True, **kw)
    assert np.array_equal(U.to_host_f64(dx1), U.to_host_f64(dx2)), "fused call differs from nm_conv1d_bwd_data"
    dx3, _ = nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=ysv, scale=scale, dx=old.clone(), relu=cfg.relu, accumulate_dx=True,
                                   force_direct=True, **kw)
    U.assert_close(U.to_host_f64(dx3), ref, dtype, f"{cfg.name} accumulated dx (plain kernel)")


def test_impulse_recovers_weights_on_gpu():
    """Completeness of the index set on the GPU path itself: a unit impulse must return every
    weight exactly (bf16 weights are exact in float32, no other term contributes)."""
    import torch
    cfg = L("impulse", 2, 70, 90, 200, 17, pad=8, affine=False, relu=False)
    inp = syn.make_inputs(cfg, "bf16")
    for ci0, t0 in ((0, 0), (33, 97), (69, 199), (64, 160), (31, 159)):
        x = np.zeros((cfg.B, cfg.Cin, cfg.T), dtype=np.float32)
        x[1, ci0, t0] = 1.0
        y = nm.nm_conv1d_block_fwd(U.arr_to_dev(x, "bf16"), U.to_dev(inp, "w", "bf16"), pad=cfg.pad)
        y = U.to_host_f64(y)
        expect = np.zeros_like(y)
        for t in range(cfg.T_out):
            k = t0 - (t - cfg.pad)
            if 0 <= k < cfg.K:
                expect[1, :, t] = inp["w"][:, ci0, k]
        np.testing.assert_array_equal(y, expect)


def test_determinism_and_guard_bands():
    """Two runs give identical bits; nothing is written outside the output tensors; inputs
    are left untouched."""
    import torch
    cfg = L("guard", 2, 72, 100, 333, 11, pad=5, residual=True)
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    To = cfg.T_out
    guard = 4096

    def guarded(n, tdtype):
        buf = torch.full((n + 2 * guard,), 7.0, dtype=tdtype, device="cuda")
        return buf, buf[guard:guard + n]

    x, w = U.to_dev(inp, "x", dtype), U.to_dev(inp, "w", dtype)
    x0, w0 = x.clone(), w.clone()
    scale, shift, res = U.to_dev(inp, "scale", dtype), U.to_dev(inp, "shift", dtype), U.to_dev(inp, "residual", dtype)
    dy, ysv = U.to_dev(inp, "dy", dtype), U.to_dev(inp, "y_saved", dtype)
    outs = []
    for _ in range(2):
        ybuf, yv = guarded(cfg.B * cfg.Cout * To, torch.bfloat16)
        dxbuf, dxv = guarded(cfg.B * cfg.Cin * cfg.T, torch.bfloat16)
        drbuf, drv = guarded(cfg.B * cfg.Cout * To, torch.bfloat16)
        dwbuf, dwv = guarded(cfg.Cout * cfg.Cin * cfg.K, torch.float32)
        kw = U.geom_kw(cfg)
        nm.nm_conv1d_block_fwd(x, w, scale, shift, res, y=yv.view(cfg.B, cfg.Cout, To), relu=True, **kw)
        nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=ysv, scale=scale, dx=dxv.view(cfg.B, cfg.Cin, cfg.T),
                              dres=drv.view(cfg.B, cfg.Cout, To), relu=True, **kw)
        nm.nm_conv1d_bwd_weight(x, dy, cfg.K, y=ysv, scale=scale, dw=dwv.view(cfg.Cout, cfg.Cin, cfg.K), relu=True, **kw)
        torch.cuda.synchronize()
        for buf in (ybuf, dxbuf, drbuf, dwbuf):
            assert (buf[:guard] == 7.0).all() and (buf[-guard:] == 7.0).all(), "write outside the output"
        outs.append([t.clone() for t in (yv, dxv, drv, dwv)])
    for a, b in zip(*outs):
        assert torch.equal(a, b), "results differ between two identical calls"
    assert torch.equal(x, x0) and torch.equal(w, w0)


# ---- both gradients in one call ------------------------------------------------------------------
FUSED = [
    L("f_ragged", 3, 72, 100, 336, 11, pad=5, residual=True),        # fused path, ragged channel tiles
    L("f_two_tiles", 2, 128, 192, 320, 17, pad=8, residual=True),
    L("f_dil2", 2, 96, 80, 248, 9, dilation=2, pad=8),
    L("f_no_epilogue", 2, 64, 64, 176, 5, pad=6, affine=False, relu=False),  # dz = dy: two calls inside
    L("f_odd_len", 2, 40, 48, 333, 7, pad=3, residual=True),         # plain kernels: two calls inside
    L("f_stride2", 2, 64, 96, 400, 11, stride=2, pad=5),
    L("f_k1", 3, 136, 200, 336, 1, residual=True),                   # K=1: the input gradient's g feeds the weight-gradient GEMM
    L("f_k1_no_relu", 2, 320, 264, 88, 1, relu=False),               # K=1 without a mask pass: g is dy
]


@pytest.mark.parametrize("cfg", FUSED, ids=lambda c: c.name)
def test_fused_backward_equals_the_two_calls_and_the_oracle(cfg):
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    scale = U.to_dev(inp, "scale", dtype) if cfg.affine else None
    x, dy, w = U.to_dev(inp, "x", dtype), U.to_dev(inp, "dy", dtype), U.to_dev(inp, "w", dtype)
    ysv = U.to_dev(inp, "y_saved", dtype) if cfg.relu else None
    kw = U.geom_kw(cfg)
    dx2, dres2 = nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=ysv, scale=scale, relu=cfg.relu, want_dres=True, **kw)
    dw2 = nm.nm_conv1d_bwd_weight(x, dy, cfg.K, y=ysv, scale=scale, relu=cfg.relu, **kw)
    dx1, dres1, dw1 = nm.nm_conv1d_bwd(x, dy, w, y=ysv, scale=scale, relu=cfg.relu, want_dres=True, **kw)
    for a, b, what in ((dx1, dx2, "dx"), (dres1, dres2, "dres"), (dw1, dw2, "dw")):
        assert np.array_equal(U.to_host_f64(a), U.to_host_f64(b)), f"{cfg.name}: fused {what} differs from the separate call"
    # and against the oracle (saved output from the input recipe)
    dx_ref, dw_ref, dres_ref = U.oracle_bwd(cfg, inp, inp["y_saved"].astype(np.float64))
    U.assert_close(U.to_host_f64(dx1), dx_ref, dtype, f"{cfg.name} fused dx")
    U.assert_close(U.to_host_f64(dw1), dw_ref, dtype, f"{cfg.name} fused dw", rms_bound=U.RMS_DW_BF16)
    np.testing.assert_array_equal(U.to_host_f64(dres1), dres_ref)
    # accumulation and a call without dres
    dw_acc = dw2.clone()
    dx3, none, dw3 = nm.nm_conv1d_bwd(x, dy, w, y=ysv, scale=scale, dw=dw_acc, relu=cfg.relu, accumulate=True, **kw)
    assert none is None and np.array_equal(U.to_host_f64(dx3), U.to_host_f64(dx2))
    np.testing.assert_allclose(U.to_host_f64(dw3), 2.0 * U.to_host_f64(dw2), rtol=1e-6, atol=0)


def test_fused_backward_full_size_headline_matches_the_two_calls():
    cfg = syn.HEADLINE
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    scale = U.to_dev(inp, "scale", dtype)
    x, dy, w, ysv = (U.to_dev(inp, n, dtype) for n in ("x", "dy", "w", "y_saved"))
    kw = U.geom_kw(cfg)
    dx2, dres2 = nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=ysv, scale=scale, relu=True, want_dres=True, **kw)
    dw2 = nm.nm_conv1d_bwd_weight(x, dy, cfg.K, y=ysv, scale=scale, relu=True, **kw)
    dx1, dres1, dw1 = nm.nm_conv1d_bwd(x, dy, w, y=ysv, scale=scale, relu=True, want_dres=True, **kw)
    import torch
    assert torch.equal(dx1, dx2) and torch.equal(dres1, dres2) and torch.equal(dw1, dw2)


# ---- seeded random geometries ---------------------------------------------------------------------
def random_layers(n, seed):
    """Random small layers whose time lengths keep them on the matrix-core kernels (multiples of 16),
    drawn so that every kernel family is hit: unrolled and tap-pair engines, private and shared tiles,
    the K=1 GEMM, stride-2 forward and input gradient, dilations 1-3, ragged channel counts."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        K = int(rng.choice([1, 2, 3, 5, 7, 11, 13, 17, 21, 25, 29]))
        stride = int(rng.choice([1, 1, 1, 2]))
        dil = int(rng.choice([1, 1, 2, 3])) if K > 1 else 1
        T = 16 * int(rng.integers(2, 30))
        pad_same = dil * (K - 1) // 2
        pad = int(rng.choice([pad_same, pad_same, 0, pad_same + 3]))
        if T + 2 * pad - dil * (K - 1) - 1 < 0:
            pad = pad_same
        Cin = int(rng.choice([8, 24, 32, 64, 96, 128, 136, 256]))
        Cout = int(rng.choice([5, 29, 64, 72, 128, 160, 256]))
        B = int(rng.integers(1, 4))
        out.append(L(f"r{i}_b{B}_{Cin}to{Cout}_t{T}_k{K}_s{stride}_d{dil}_p{pad}", B, Cin, Cout, T, K, stride=stride,
                     dilation=dil, pad=pad, affine=bool(rng.integers(0, 2)), relu=bool(rng.integers(0, 2)),
                     residual=bool(rng.integers(0, 2)), seed=1000 + i))
    return out


@pytest.mark.parametrize("cfg", random_layers(36, 2024), ids=lambda c: c.name)
def test_random_geometries_full_tensor(cfg):
    check_layer(cfg, "bf16", False)
