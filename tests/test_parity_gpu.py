"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle."""
import numpy as np
import pytest

from mbconv_inputs import (BlockShape, CONFIG0, CONFIG1, CONFIG2, CONFIG3, MBV2_BLOCK, b0_chain,
                           make_block_inputs)
from oracle import oracle as orc
from parity_util import compare_block, rel_err, run_gpu_block, TOL

pytestmark = pytest.mark.gpu


def _shape(**kw):
    base = dict(N=2, Cin=8, H=9, W=11, Cexp=24, Cse=2, Cout=8, k=3, stride=1, residual=True)
    base.update(kw)
    return BlockShape(**base)


# small blocks: ragged planes, channel counts that are not multiples of the GEMM tiles,
# every (k, stride), with and without expansion / residual, planes of each thread-group size
SMALL = {
    "k3s1_ragged": _shape(),
    "k5s1": _shape(k=5, H=14, W=14, Cin=16, Cexp=40, Cout=16),
    "k3s2": _shape(stride=2, residual=False, Cout=12, H=16, W=16),
    # expansion-conv backward in one pass (narrow input <= 32 channels, HW % 4 == 0): full tiles on
    # both sides with eight wavefronts and 32-pixel chunks that straddle images; and a ragged case
    # (5 and 100 channels: a wavefront without weight-gradient work, a last chunk of 12 pixels)
    "fused_bwd_full": _shape(N=3, Cin=32, Cexp=256, Cse=8, Cout=32, H=6, W=6),
    "fused_bwd_ragged": _shape(N=5, Cin=5, Cexp=100, Cse=4, Cout=5, H=6, W=10),
    "k5s2_odd": _shape(k=5, stride=2, residual=False, Cout=20, H=15, W=13),
    "noexpand": _shape(Cin=24, Cexp=24, Cout=16, has_expand=False, residual=False, H=20, W=20),
    "noexpand_res": _shape(Cin=16, Cexp=16, Cout=16, has_expand=False, residual=True, k=5),
    # both sides of the projection conv within one 32-channel tile: its backward runs with a
    # wavefront per pixel chunk (full tiles, ragged channel counts, a ragged last chunk, bf16)
    "noexpand_32_16": _shape(N=3, Cin=32, Cexp=32, Cse=8, Cout=16, has_expand=False, residual=False,
                             H=12, W=20),
    "noexpand_ragged_nn": _shape(N=5, Cin=21, Cexp=21, Cse=5, Cout=10, has_expand=False,
                                 residual=False, H=6, W=6, k=5),
    "bf16_noexpand": _shape(dtype="bf16", N=32, Cin=32, Cexp=32, Cse=8, Cout=16, has_expand=False,
                            residual=False, H=12, W=12),
    "wide": _shape(N=3, Cin=72, Cexp=200, Cse=18, Cout=72, H=7, W=7, k=5),
    "plane_1024_threads": _shape(N=1, Cin=8, Cexp=16, Cout=8, H=70, W=66),
    "plane_256_threads": _shape(N=2, Cin=8, Cexp=16, Cout=8, H=28, W=28, k=5),
    "n1_tiny": _shape(N=1, Cin=1, Cexp=1, Cse=1, Cout=1, H=3, W=3, has_expand=False),
    # the largest plane the library accepts (128x128), on each depthwise kernel family
    "max_plane_k5": _shape(N=1, Cin=8, Cexp=8, Cout=8, H=128, W=128, k=5),
    "max_plane_s2": _shape(N=1, Cin=8, Cexp=8, Cout=8, H=128, W=128, k=5, stride=2, residual=False),
    "max_plane_ragged": _shape(N=1, Cin=8, Cexp=8, Cout=8, H=127, W=125, k=5),
    "one_pixel": _shape(N=3, Cin=4, Cexp=8, Cse=2, Cout=4, H=1, W=1),
    # 64 <-> 192 channels on 14x14: the wide fp32 conv kernels without a split contraction
    "mid_14x14": _shape(N=4, Cin=64, Cexp=192, Cse=16, Cout=64, H=14, W=14),
    # depthwise forward with two images of a channel per workgroup (planes of 1025..4096 elements,
    # at least 2048 such workgroups): an odd batch (the last workgroup of a channel has one image),
    # 5x5 and 3x3, with and without the expansion conv, fp32 and bf16
    "dw_two_images_k5": _shape(N=5, Cin=24, Cexp=684, Cse=6, Cout=24, H=36, W=36, k=5),
    "dw_two_images_noexpand": _shape(N=5, Cin=684, Cexp=684, Cse=6, Cout=24, H=36, W=36,
                                     has_expand=False, residual=False),
    "dw_two_images_bf16": _shape(dtype="bf16", N=5, Cin=24, Cexp=684, Cse=6, Cout=24, H=36, W=36),
    # fp32 wide blocks on the bf16 matrix cores (three-plane operand splits): plane tiles whose size
    # leaves a partial pixel run of two, three and one pixels (6x7, 3x5, 7x7), the last two with a
    # split contraction (few tiles, long K) and a residual in the epilogue of the data gradient;
    # ragged row and k tiles (40, 56, 72 channels; K = 40, 72: a last chunk of 8 of 32);
    # weight gradients with a narrow operand on either side (64-row tile, swapped operands)
    "x3_plane_6x7": _shape(N=3, Cin=40, Cexp=96, Cse=10, Cout=48, H=6, W=7, residual=False),
    "x3_plane_3x5_split": _shape(N=5, Cin=64, Cexp=512, Cse=16, Cout=64, H=3, W=5, k=5),
    "x3_plane_7x7_split": _shape(N=9, Cin=40, Cexp=320, Cse=10, Cout=40, H=7, W=7, k=5),
    "x3_narrow_wgrad": _shape(N=2, Cin=48, Cexp=288, Cse=12, Cout=56, H=8, W=8, residual=False),
    "x3_split_res": _shape(N=2, Cin=72, Cexp=432, Cse=18, Cout=72, H=4, W=4),
    "x3_ragged_pixels": _shape(N=3, Cin=72, Cexp=136, Cse=18, Cout=72, H=6, W=10),
    # expansion-conv backward of at most 16 -> 96 channels (a multiple of eight) on planes of an
    # even number of pixels: a wavefront per 32-pixel chunk on the bf16 matrix cores, with six,
    # four and two 16-channel tiles; full tiles with the residual; a ragged narrow side, 40 wide
    # channels (the last 16-channel tile half empty) and a last chunk of 18 pixels that starts in
    # one image and ends in the next; 24 channels on 8x8
    "x3_bwd1x1_96": _shape(N=3, Cin=16, Cexp=96, Cse=4, Cout=16, H=8, W=12),
    "x3_bwd1x1_ragged": _shape(N=3, Cin=5, Cexp=40, Cse=3, Cout=7, H=6, W=5, residual=False),
    "x3_bwd1x1_two_tiles": _shape(N=2, Cin=8, Cexp=24, Cse=2, Cout=8, H=8, W=8),
    # 1x1 convolutions with a short contraction and many rows (expansion conv, projection data
    # gradient): weights resident in LDS, a wavefront per 32-pixel chunk.  An odd plane (single
    # pixels per lane instead of pairs, a last chunk of 19 pixels, 40 = one full and one quarter
    # step of the contraction, 168 rows = two slabs and 40 rows); the longest contraction (192)
    # with the statistics epilogue; other shapes above take the same kernels (mid_14x14, wide, ...)
    "xw_odd_plane": _shape(N=3, Cin=40, Cexp=168, Cse=10, Cout=40, H=7, W=7, k=5),
    "xw_k192": _shape(N=2, Cin=192, Cexp=320, Cse=8, Cout=96, H=4, W=6, residual=False),
    "bf16_small": _shape(dtype="bf16", H=14, W=14, k=5, Cin=16, Cexp=64, Cout=16, N=4),
    "bf16_s2": _shape(dtype="bf16", H=16, W=16, k=3, stride=2, Cin=16, Cexp=32, Cout=24, N=4,
                      residual=False),
    # bf16 on planes whose width or size is not a multiple of four: the two- and one-element
    # lane groups of the small-plane depthwise kernels, the scalar paths of the plane reductions
    # and of the final elementwise pass, the generic depthwise kernels on ragged planes, and the
    # fp32-MFMA fallback of the wide 1x1 kernels (their bf16 form needs HW % 4 == 0):
    # EfficientNet-B0's 7x7 stage, a ragged stride-2 plane, a ragged stride-1 plane
    "bf16_7x7_wide": _shape(dtype="bf16", N=8, Cin=96, Cexp=288, Cse=24, Cout=96, H=7, W=7, k=5),
    # (batch 32: with a few hundred samples per channel the bf16 storage noise alone, measured
    # with the CPU rounding model, exceeds 2e-2 on two-element tensors)
    "bf16_k5s2_odd": _shape(dtype="bf16", N=32, k=5, stride=2, residual=False, Cin=16, Cexp=48,
                            Cse=4, Cout=20, H=15, W=13),
    "bf16_ragged": _shape(dtype="bf16", N=32, Cin=16, Cexp=48, Cse=4, Cout=16, H=9, W=11),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_block_matches_oracle(name):
    s = SMALL[name]
    t = make_block_inputs(s, seed=7)
    print(f"[parity] {name} {s}", flush=True)
    res, blk = run_gpu_block(s, t)
    f, b = orc.mbconv_step(s, t)
    compare_block(s, t, res, f, b, blk)


@pytest.mark.parametrize("name", ["k3s1_ragged", "k5s2_odd", "bf16_small", "bf16_ragged",
                                  "noexpand_32_16"])
def test_store_policy_matches_oracle(name):
    s = SMALL[name]
    # (bf16_ragged: a seed for which the storage-rounding noise of BN1's gamma gradient, measured
    # with the CPU rounding model, is 1e-2 rather than the 1.7e-2 of seed 11)
    t = make_block_inputs(s, seed=15 if name == "bf16_ragged" else 11)
    print(f"[parity/store] {name}", flush=True)
    res, blk = run_gpu_block(s, t, policy=1)
    f, b = orc.mbconv_step(s, t)
    compare_block(s, t, res, f, b, blk)
    from parity_util import metric_for
    tol = TOL[s.dtype]["fwd"]
    if s.has_expand:  # (without an expansion conv the depthwise input is x itself: nothing is kept)
        assert metric_for(s)(blk.saved_tensor("a1"), f.tape["a1"]) <= tol
    assert metric_for(s)(blk.saved_tensor("sc"), f.tape["sc"]) <= tol


def test_bn_finalised_by_consumer_with_many_partials():
    """BN3's statistics are finalised inside the final elementwise pass for planes of 1024
    elements or more.  With the STORE policy the projection conv leaves one partial sum per
    128 pixels: 48*56*56/128 = 1176 per channel, more than the 4*256 a thread group of that
    kernel takes in its first round, so the loop over further rounds runs too; BN1 goes through
    the separate finalise launch here (STORE), BN3's running statistics through the fused one."""
    s = _shape(N=48, Cin=8, Cexp=16, Cse=4, Cout=8, H=56, W=56)
    t = make_block_inputs(s, seed=21)
    print(f"[parity/bn-consumer] {s}", flush=True)
    res, blk = run_gpu_block(s, t, policy=1)
    f, b = orc.mbconv_step(s, t)
    compare_block(s, t, res, f, b, blk)


def _random_shapes(count, seed):
    """Seeded random block shapes, drawn so that every kernel family is reached: ragged and
    4-divisible planes, the plane sizes of the depthwise variants (56, 28, 14, 7 and a few
    pixels), narrow and wide channel counts on either side of the 1x1 kernels' switch points,
    both activations, with and without expansion / SE / residual, both policies.  At least two
    input channels: with one, the expansion weight gradient is a difference that cancels to
    O(eps) and no relative bound holds for it."""
    import random
    rng = random.Random(seed)
    out = []
    for _ in range(count):
        k, stride = rng.choice([3, 5]), rng.choice([1, 1, 2])
        fam = rng.choice(["ragged", "mult4", "p56", "p28", "p14", "p7", "tiny", "wide"])
        if fam == "ragged":
            H, W = rng.randint(3, 24), rng.randint(3, 24)
        elif fam == "mult4":
            H, W = 4 * rng.randint(1, 10), 4 * rng.randint(1, 10)
        elif fam == "tiny":
            H, W = rng.randint(1, 4), rng.randint(1, 4)
        elif fam == "wide":
            H, W = rng.choice([(7, 7), (14, 14), (8, 8), (6, 10)])
        else:
            H = W = int(fam[1:])
        if fam == "wide":
            Cin = rng.choice([40, 48, 64, 72, 80, 112])
            ratio = rng.choice([3, 6])
            Cout = rng.choice([Cin, 40, 96, 112, 192])
        else:
            Cin = rng.choice([2, 3, 5, 8, 16, 17, 24, 32, 33, 40])
            ratio = rng.choice([1, 1, 3, 4, 6])
            Cout = rng.choice([Cin, 1, 7, 16, 24, 32, 33, 40, 48])
        N = rng.randint(1, 6)
        Cexp = Cin * ratio
        N = max(1, min(N, 3_000_000 // (H * W * Cexp)))
        # at least eight samples per channel behind BN2 and BN3: batch normalisation over a
        # handful of samples amplifies rounding noise without bound (over one sample the
        # gradient is exactly zero and no relative error is defined)
        pad = (k - 1) // 2
        HoWo = ((H + 2 * pad - k) // stride + 1) * ((W + 2 * pad - k) // stride + 1)
        N = max(N, -(-8 // HoWo))
        out.append((BlockShape(N=N, Cin=Cin, H=H, W=W, Cexp=Cexp, Cse=max(1, Cin // 4), Cout=Cout, k=k,
                               stride=stride, has_expand=(ratio != 1 or rng.random() < 0.3),
                               residual=(stride == 1 and Cin == Cout and rng.random() < 0.7),
                               activation=rng.choice(["swish", "swish", "relu6"]),
                               has_se=rng.random() < 0.8),
                    rng.choice([0, 0, 1])))
    return out


@pytest.mark.parametrize("index", range(48))
def test_random_shape_matches_oracle(index):
    """Training step and evaluation-mode forward on a seeded random shape (fp32)."""
    import torch
    from paper_2110_10802_amd.harness import DeviceBlock, to_numpy
    from parity_util import metric_for

    s, policy = _random_shapes(48, seed=20211020)[index]
    t = make_block_inputs(s, seed=300 + index)
    print(f"[parity/random {index}] policy={policy} {s}", flush=True)
    res, blk = run_gpu_block(s, t, policy=policy)
    f, b = orc.mbconv_step(s, t)
    compare_block(s, t, res, f, b, blk)
    te = _with_running(s, t, seed=400 + index)
    ref = orc.mbconv_forward_eval(s, te)
    blk2 = DeviceBlock(s, te)
    out = to_numpy(blk2.forward_eval(blk2.to_device(te["x"])))
    torch.cuda.synchronize()
    assert metric_for(s)(out, ref) <= TOL[s.dtype]["fwd"]


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_benchmark_config_matches_oracle(cfg):
    s = [CONFIG0, CONFIG1, CONFIG2, CONFIG3][cfg]
    t = make_block_inputs(s, seed=0)
    print(f"[parity] config {cfg} {s}", flush=True)
    res, blk = run_gpu_block(s, t)
    print("[parity] gpu done, running oracle", flush=True)
    f, b = orc.mbconv_step(s, t)
    errs = compare_block(s, t, res, f, b, blk)
    print({k: f"{v[0]:.2e}" for k, v in errs.items()}, flush=True)


@pytest.mark.parametrize("name", ["k5s1", "fused_bwd_full", "wide", "k3s2", "noexpand_32_16"])
def test_backward_is_bitwise_repeatable(name):
    """No floating-point atomics anywhere and every reduction in a fixed order: ten runs of the
    same step give the same bits (each run in freshly allocated buffers)."""
    s = SMALL[name]
    t = make_block_inputs(s, seed=3)
    r1, _ = run_gpu_block(s, t)
    for _ in range(9):
        r2, _ = run_gpu_block(s, t)
        assert np.array_equal(r1["out"], r2["out"]) and np.array_equal(r1["dx"], r2["dx"])
        for n in r1["grads"]:
            assert np.array_equal(r1["grads"][n], r2["grads"][n]), n
        for n in r1["running"]:
            assert np.array_equal(r1["running"][n], r2["running"][n]), n


# Batch statistics far from zero mean: x ~ N(mu, 1), so that the expansion output e and the
# depthwise output d have |mean| of several (mu = 3) to several tens (mu = 30) of standard
# deviations in most channels.  The oracle's statistics are two-pass; a one-pass E[x^2]-E[x]^2
# in single precision would lose (mean/std)^2 * 2^-24 of the variance.  One shape per depthwise
# kernel family (stride-1 vectorised, small-plane, stride-2) and one block without expansion,
# where the depthwise kernel sees the offset input directly.
OFFSET_SHAPES = {
    "dw4": _shape(N=4, Cin=24, Cexp=48, Cse=6, Cout=24, H=56, W=56),
    "dwr": _shape(N=16, Cin=40, Cexp=120, Cse=10, Cout=40, H=14, W=14, k=5),
    "dw2": _shape(N=4, Cin=24, Cexp=48, Cse=6, Cout=40, H=56, W=56, k=5, stride=2, residual=False),
    "noexpand": _shape(N=4, Cin=32, Cexp=32, Cse=8, Cout=16, H=28, W=28, has_expand=False,
                       residual=False),
}


@pytest.mark.parametrize("mu", [3.0, 30.0])
@pytest.mark.parametrize("name", list(OFFSET_SHAPES))
def test_offset_inputs_match_oracle(name, mu):
    s = OFFSET_SHAPES[name]
    t = make_block_inputs(s, seed=31)
    t["x"] = (t["x"] + np.float32(mu)).astype(np.float32)
    print(f"[parity/offset] {name} mu={mu} {s}", flush=True)
    res, blk = run_gpu_block(s, t)
    f, b = orc.mbconv_step(s, t)
    ratios = []
    for nm in ("e", "d"):
        v = f.tape[nm]
        if v.size > 1:
            r = np.abs(v.mean(axis=(0, 2, 3))) / np.maximum(v.std(axis=(0, 2, 3)), 1e-30)
            ratios.append(f"{nm}: median |mean|/std {np.median(r):.1f}, max {r.max():.1f}")
    print("[parity/offset] " + "; ".join(ratios), flush=True)
    errs = compare_block(s, t, res, f, b, blk)
    print({k: f"{v[0]:.2e}" for k, v in errs.items()}, flush=True)


# Two families of degenerate shapes are outside the relative bounds of the random sweep (see
# _random_shapes): one input channel with an expansion conv, and fewer than eight samples per
# channel behind BN2/BN3.  The library must still return finite results whose ABSOLUTE error is
# small against the size of the terms that cancel.
DEGENERATE = {
    "one_input_channel": _shape(N=3, Cin=1, Cexp=6, Cse=1, Cout=1, H=8, W=8),
    "two_samples": _shape(N=2, Cin=4, Cexp=8, Cse=1, Cout=4, H=1, W=1),
    "one_sample": _shape(N=1, Cin=4, Cexp=8, Cse=1, Cout=4, H=1, W=1),
    "four_samples_s2": _shape(N=1, Cin=4, Cexp=8, Cse=1, Cout=6, H=4, W=4, stride=2, residual=False),
}


@pytest.mark.parametrize("name", list(DEGENERATE))
def test_degenerate_shapes_are_finite_and_absolutely_bounded(name):
    s = DEGENERATE[name]
    t = make_block_inputs(s, seed=41)
    print(f"[parity/degenerate] {name} {s}", flush=True)
    res, _ = run_gpu_block(s, t)
    f, b = orc.mbconv_step(s, t)
    assert np.all(np.isfinite(res["out"])) and np.all(np.isfinite(res["dx"]))
    # forward: normalised values are O(1); absolute error against that scale
    assert np.max(np.abs(res["out"] - f.out)) <= 1e-3 * (1.0 + np.max(np.abs(f.out)))
    # gradients: every term of the cancelling sums is bounded by |dout| * |activations| summed over
    # the samples; the absolute error is held to 1e-3 of the largest gradient magnitude in the
    # block (not of the tensor's own, which may be a fully cancelled zero)
    scale = max(float(np.max(np.abs(v))) for v in list(b.grads.values()) + [b.dx])
    assert np.max(np.abs(res["dx"] - b.dx)) <= 1e-3 * scale
    for n, g in res["grads"].items():
        assert np.all(np.isfinite(g)), n
        assert np.max(np.abs(g - b.grads[n])) <= 1e-3 * scale, (n, float(np.max(np.abs(g - b.grads[n]))), scale)


def _rounding_model(s, t, mfma_bf16=False):
    """The oracle's steps with bf16 rounding at the HIP path's storage points (and, with
    `mfma_bf16`, at the operands of the bf16 matrix-core kernels): tests/rounding_model.py."""
    from rounding_model import rounding_model
    return rounding_model(s, t, storage=True, mfma_bf16=mfma_bf16)


@pytest.mark.parametrize("name", ["bf16_small", "bf16_7x7_wide", "bf16_k5s2_odd", "bf16_ragged",
                                  "config3_n16", "config3"])
def test_bf16_matches_rounding_model(name):
    """bf16 storage: element-wise agreement with the oracle steps once the same storage
    rounding is applied.  A value within fp32 noise of a bf16 rounding boundary may round the
    other way (one bf16 ulp = 2^-7 of the value) and a flipped input can flip the tensor stored
    after it, so the bound is two bf16 ulps, 2^-6, under the element-wise metric that the
    unrounded oracle cannot be held to.  Every bound used here is fixed by a CPU test that
    involves no HIP code (tests/test_bf16_bounds.py): noise of fp32 size ahead of the roundings
    of the fp64 model itself moves `out` by up to 2^-6 + 1.5e-3 (a flip of p is scaled by BN3
    before out is rounded again) and BN1's gamma gradient, the small residual of a heavily
    cancelling sum, by more than 2^-6 at batch 16 but never by 2^-5; everything else stays within
    2^-6.  "config3" is the benchmark configuration at its stated batch of 128; for it the
    distance of the HIP path and of the model from the UNROUNDED oracle is reported under both
    metrics (element-wise rms-floored / relative to the largest magnitude)."""
    s = {"config3_n16": CONFIG3.with_batch(16), "config3": CONFIG3}.get(name) or SMALL[name]
    t = make_block_inputs(s, seed=5)
    print(f"[parity/bf16-model] {name}", flush=True)
    res, blk = run_gpu_block(s, t)
    # config 3's channel counts route every 1x1 convolution and weight gradient through the bf16
    # matrix-core kernels; the small shape stays on the register-direct fp32-MFMA kernels
    # (nor do planes that are not a multiple of four elements: the bf16 matrix-core kernels need
    # 8-byte aligned rows, so the 7x7 stage falls back to the fp32-MFMA kernels)
    on_bf16_cores = name in ("config3_n16", "config3")
    m = _rounding_model(s, t, mfma_bf16=on_bf16_cores)
    got = {"out": res["out"], "dx": res["dx"], **{n: blk.saved_tensor(n) for n in ("e", "d", "p")}}
    errs = {n: rel_err(got[n], m[n]) for n in got}
    gerrs = {n: rel_err(res["grads"][n], m["grads"][n]) for n in res["grads"]}
    print(errs, gerrs, flush=True)
    two = 2.0 ** -6
    sbounds = {"out": two + 1.5e-3, "e": two, "d": two, "p": two, "dx": two}
    bad = {n: (v, sbounds[n]) for n, v in errs.items() if v > sbounds[n]}
    assert not bad, bad
    bounds = {n: two for n in gerrs}
    if on_bf16_cores:
        bounds["bn1_gamma"] = 2.0 ** -5
    bad = {n: (v, bounds[n]) for n, v in gerrs.items() if v > bounds[n]}
    assert not bad, bad
    if name == "config3":
        from parity_util import linf_err
        f, b = orc.mbconv_step(s, t)
        ref = {"out": f.out, "e": f.tape["e"], "d": f.tape["d"], "p": f.tape["p"], "dx": b.dx}
        table = {}
        for n, r in list(ref.items()) + list(b.grads.items()):
            g_ = got[n] if n in got else res["grads"][n]
            m_ = m[n] if n in m else m["grads"][n]
            table[n] = {"hip_elementwise": rel_err(g_, r), "hip_linf": linf_err(g_, r),
                        "model_elementwise": rel_err(m_, r), "model_linf": linf_err(m_, r)}
        print("[parity/bf16-model] config 3 at batch 128 against the unrounded oracle "
              "(HIP element-wise / linf; rounding model element-wise / linf):", flush=True)
        for n, v in table.items():
            print(f"  {n:10s} {v['hip_elementwise']:.4f} / {v['hip_linf']:.4f}    "
                  f"{v['model_elementwise']:.4f} / {v['model_linf']:.4f}", flush=True)
        import json
        import os
        d = os.environ.get("MBCONV_PARITY_REPORT_DIR", "")
        if d and os.path.isdir(d):
            with open(os.path.join(d, "config3_bf16_both_metrics.json"), "w") as fh:
                json.dump(table, fh, indent=1)
        # relative to the largest magnitude the HIP path is inside the benchmark's 2e-2
        assert all(v["hip_linf"] <= TOL["bf16"]["grad"] for v in table.values()), table


def _oracle_chain(blocks, seed0=100):
    """Oracle forward through the whole chain, then backward; returns per-block inputs/results."""
    recs = []
    x = None
    for i, s in enumerate(blocks):
        t = make_block_inputs(s, seed=seed0 + i, with_x=(i == 0), with_dout=(i == len(blocks) - 1))
        if i > 0:
            t["x"] = x
        f = orc.mbconv_forward(s, t)
        recs.append({"shape": s, "t": t, "f": f})
        x = f.out
    dout = recs[-1]["t"]["dout"].astype(np.float64)
    for r in reversed(recs):
        r["dout"] = dout
        r["b"] = orc.mbconv_backward(r["shape"], r["t"], r["f"].tape, dout)
        dout = r["b"].dx
    return recs


@pytest.mark.parametrize("batch", [4, 64])
def test_b0_chain_matches_oracle(batch):
    """The 16 MBConv blocks of EfficientNet-B0 (benchmark config 4), at batch 4 and at the
    stated batch of 64 (kernel selection, tile shapes and split counts depend on the batch):
    every block is run on the GPU from the oracle's input and upstream gradient (isolated,
    standard tolerances), and the chain is also run end to end on the GPU (block i fed by GPU
    block i-1) with ONE scratch workspace shared by all blocks, sized to the largest request:
    the arrangement bench.py times."""
    import torch
    from paper_2110_10802_amd import binding as B
    from paper_2110_10802_amd.harness import DeviceBlock, to_numpy

    blocks = b0_chain(N=batch)
    recs = _oracle_chain(blocks)
    print(f"[parity/chain] oracle chain at batch {batch} done", flush=True)
    # isolated
    failures = []
    for i, r in enumerate(recs):
        s = r["shape"]
        t = dict(r["t"])
        t["x"] = np.asarray(t["x"], dtype=np.float32)
        t["dout"] = np.asarray(r["dout"], dtype=np.float32)
        print(f"[parity/chain] N={batch} block {i + 1} {s.Cin}->{s.Cexp}->{s.Cout} {s.H}x{s.W} "
              f"k{s.k}s{s.stride}", flush=True)
        res, blk = run_gpu_block(s, t)
        # the oracle saw float64 x/dout; the GPU their float32 roundings (1e-7, far below tolerance)
        try:
            compare_block(s, t, res, r["f"], r["b"], blk)
        except AssertionError as exc:  # keep going: report every failing block at once
            failures.append(f"block {i + 1}: {str(exc).splitlines()[0]}")
        del blk, res
        # only the block's output, input gradient and parameter gradients are needed below
        r["f"].tape = None
    torch.cuda.empty_cache()
    assert not failures, "\n".join(failures)
    # end to end, one shared scratch workspace
    scratch_bytes = max(B.mbconv_workspace_size(B.make_desc(r["shape"]))[1] for r in recs)
    scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device="cuda")
    dev = []
    x = None
    for i, r in enumerate(recs):
        blk = DeviceBlock(r["shape"], r["t"], scratch=scratch)
        assert blk.scratch.data_ptr() == scratch.data_ptr()
        xin = blk.to_device(r["t"]["x"]) if i == 0 else x
        blk.forward(xin)
        dev.append((blk, xin))
        x = blk.out
    torch.cuda.synchronize()
    e2e = {"out": rel_err(to_numpy(dev[-1][0].out), recs[-1]["f"].out)}
    dout = dev[-1][0].to_device(recs[-1]["t"]["dout"])
    for blk, xin in reversed(dev):
        blk.backward(xin, dout)
        dout = blk.dx
    torch.cuda.synchronize()
    e2e["dx"] = rel_err(to_numpy(dev[0][0].dx), recs[0]["b"].dx)
    worst = ("", 0.0)
    for i, ((blk, _), r) in enumerate(zip(dev, recs)):
        # d(beta3) of an inner block is zero by invariance (see compare_block): absolute floor
        d = np.asarray(r["dout"], dtype=np.float64)
        beta_floor = float(np.sqrt(np.mean(d * d)) * np.sqrt(d.size / d.shape[1]))
        for n, g in blk.grads.items():
            floor = beta_floor if n == "bn3_beta" else 0.0
            err = rel_err(to_numpy(g), r["b"].grads[n], floor)
            if err > worst[1]:
                worst = (f"block{i + 1}.{n}", err)
    e2e["worst_grad"] = worst
    print(f"[parity/chain] N={batch} end to end (shared scratch): {e2e}", flush=True)
    # End to end the GPU blocks see each other's outputs, so rounding differences could compound
    # over 16 blocks forward and 16 back; each block's BN renormalises and they do not: the chain
    # is held to the single-block bounds (measured: out 2.5e-5, dx 1.1e-4, worst gradient 6.5e-5).
    assert e2e["out"] <= TOL["f32"]["fwd"], e2e
    assert e2e["dx"] <= TOL["f32"]["grad"], e2e
    assert worst[1] <= TOL["f32"]["grad"], e2e


@pytest.mark.parametrize("index", [0, 1, 4, 6])
def test_b0_chain_blocks_full_batch(index):
    """Blocks of config 4 at the full batch of 64, where the launch shapes differ from the
    batch-4 chain: blocks 1 and 2 (112x112 planes, the largest thread-group shape, no expansion /
    stride 2) and blocks 5 and 7 (the wide-GEMM kernels pick their 128-column tiles only when
    the batch is large)."""
    s = b0_chain(N=64)[index]
    t = make_block_inputs(s, seed=0)
    print(f"[parity/chain-full] block {index + 1} {s}", flush=True)
    res, blk = run_gpu_block(s, t)
    f, b = orc.mbconv_step(s, t)
    compare_block(s, t, res, f, b, blk)


# ------------------------------------------------------------ evaluation mode ------

def _with_running(s, t, seed):
    """The block's inputs with running statistics that are neither (0, 1) nor the batch's."""
    rng = np.random.default_rng(seed)
    t = dict(t)
    for i, C_ in ((1, s.Cexp), (2, s.Cexp), (3, s.Cout)):
        if i == 1 and not s.has_expand:
            continue
        t[f"bn{i}_mean"] = (0.3 * rng.standard_normal(C_)).astype(np.float32)
        t[f"bn{i}_var"] = (0.5 + rng.random(C_)).astype(np.float32)
    return t


@pytest.mark.parametrize("name", ["k3s1_ragged", "k5s1", "k5s2_odd", "noexpand_res", "wide",
                                  "mid_14x14", "plane_1024_threads", "max_plane_ragged", "one_pixel",
                                  "n1_tiny", "bf16_small", "bf16_s2", "config1", "config3"])
def test_eval_forward_matches_oracle(name):
    import torch
    from paper_2110_10802_amd.harness import DeviceBlock, to_numpy
    from parity_util import metric_for

    s = {"config1": CONFIG1, "config3": CONFIG3}.get(name) or SMALL[name]
    t = _with_running(s, make_block_inputs(s, seed=5), seed=17)
    print(f"[parity/eval] {name} {s}", flush=True)
    ref = orc.mbconv_forward_eval(s, t)
    blk = DeviceBlock(s, t)
    x = blk.to_device(t["x"])
    out = to_numpy(blk.forward_eval(x))
    torch.cuda.synchronize()
    err = metric_for(s)(out, ref)
    print(f"[parity/eval] {name} err {err:.2e}", flush=True)
    assert err <= TOL[s.dtype]["fwd"], err
    # the running statistics are inputs here: unchanged, bit for bit
    for n, r in blk.running.items():
        assert np.array_equal(to_numpy(r), np.asarray(t[n], dtype=np.float32)), n
    # a training step in between (it owns other workspaces) does not disturb a second call
    blk.forward(x)
    for n, r in blk.running.items():  # restore what the training call updated
        r.copy_(torch.from_numpy(np.asarray(t[n], dtype=np.float32)))
    out2 = to_numpy(blk.forward_eval(x))
    torch.cuda.synchronize()
    assert np.array_equal(out, out2)


# ------------------------------------- MobileNet-V2 block: ReLU6, no squeeze-and-excitation ------

MBV2 = {
    "mbv2_s1": _shape(activation="relu6", has_se=False, Cse=1, Cexp=48, H=14, W=14),
    "mbv2_s2_ragged": _shape(activation="relu6", has_se=False, Cse=1, Cexp=48, stride=2,
                             residual=False, Cout=12, H=15, W=13),
    "mbv2_t1": _shape(activation="relu6", has_se=False, Cse=1, Cin=16, Cexp=16, Cout=8,
                      has_expand=False, residual=False, H=28, W=28, N=2),
    "mbv2_wide_7x7": _shape(activation="relu6", has_se=False, Cse=1, N=4, Cin=96, Cexp=576,
                            Cout=96, H=7, W=7),
    # the two switches are independent
    "relu6_with_se": _shape(activation="relu6", Cexp=48, H=14, W=14, k=5),
    "swish_without_se": _shape(has_se=False, Cse=1, Cexp=48, H=14, W=14),
    "mbv2_block": MBV2_BLOCK,
}


@pytest.mark.parametrize("name", list(MBV2))
def test_mobilenet_v2_block_matches_oracle(name):
    s = MBV2[name]
    t = make_block_inputs(s, seed=21)
    print(f"[parity/mbv2] {name} {s}", flush=True)
    res, blk = run_gpu_block(s, t)
    f, b = orc.mbconv_step(s, t)
    errs = compare_block(s, t, res, f, b, blk)
    print({k: f"{v[0]:.2e}" for k, v in errs.items()}, flush=True)


@pytest.mark.parametrize("name", ["mbv2_s1", "mbv2_s2_ragged", "mbv2_wide_7x7", "mbv2_block"])
def test_mobilenet_v2_eval_forward_matches_oracle(name):
    import torch
    from paper_2110_10802_amd.harness import DeviceBlock, to_numpy
    from parity_util import metric_for

    s = MBV2[name]
    t = _with_running(s, make_block_inputs(s, seed=5), seed=17)
    ref = orc.mbconv_forward_eval(s, t)
    blk = DeviceBlock(s, t)
    out = to_numpy(blk.forward_eval(blk.to_device(t["x"])))
    torch.cuda.synchronize()
    err = metric_for(s)(out, ref)
    print(f"[parity/mbv2 eval] {name} err {err:.2e}", flush=True)
    assert err <= TOL[s.dtype]["fwd"], err


def test_mobilenet_v2_bf16_matches_rounding_model():
    """ReLU6 with bf16 storage.  The derivative of ReLU6 is discontinuous, and a stored
    pre-normalisation tensor rounded to bf16 moves about one pre-activation in a hundred across
    a kink, so against the unrounded oracle the gradients differ by O(1) at those elements
    whatever the implementation; the comparison that can be made element by element is against
    the oracle's steps with the same storage and matrix-core operand roundings (MobileNet-V2's
    14x14 stage: 96 -> 576 -> 96 channels, every 1x1 conv and weight gradient on the bf16 matrix
    cores)."""
    s = _shape(activation="relu6", has_se=False, Cse=1, dtype="bf16", N=8, Cin=96, Cexp=576,
               Cout=96, H=14, W=14)
    t = make_block_inputs(s, seed=23)
    print(f"[parity/mbv2 bf16-model] {s}", flush=True)
    res, blk = run_gpu_block(s, t)
    m = _rounding_model(s, t, mfma_bf16=True)
    errs = {"out": rel_err(res["out"], m["out"])}
    for n in ("e", "d", "p"):
        errs[n] = rel_err(blk.saved_tensor(n), m[n])
    gerrs = {n: rel_err(res["grads"][n], m["grads"][n]) for n in res["grads"]}
    # dx: a bf16 boundary flip of a stored tensor next to a kink flips a mask; counted, bounded
    # and excluded from the element-wise figure (see _relu6_kink_tolerant for the fp32 case)
    ref = m["dx"]
    rms = float(np.sqrt(np.mean(ref * ref)))
    rel = np.abs(res["dx"] - ref) / np.maximum(np.abs(ref), rms)
    outliers = int(np.count_nonzero(rel > 2.0 ** -6))
    errs["dx_rms"] = float(np.sqrt(np.mean((res["dx"] - ref) ** 2))) / rms
    print(errs, gerrs, f"dx outliers {outliers} of {ref.size}", flush=True)
    assert max(errs.values()) <= 2.0 ** -6, errs
    assert outliers <= ref.size // 1000, outliers
    bounds = {n: 2.0 ** -6 for n in gerrs}
    bounds["bn1_gamma"] = 2.0 ** -5
    bad = {n: (v, bounds[n]) for n, v in gerrs.items() if v > bounds[n]}
    assert not bad, bad
