"""GPU parity: the HIP path (through the C ABI, via the ctypes binding) against
the fp64 CPU oracle on the same seeded inputs.

Bars (from the benchmark spec): integer codes -- at most 1e-3 of them may
differ and none by more than one level (in practice both sides compute in fp64
and the tests below see zero differences); scales / zeros within 1e-5
relative; layer loss within 1e-3 relative.  Intermediate fp64 quantities (H,
Hinv, S, W_work, Hinv_work) are compared at tolerances that follow from fp64
rounding and the conditioning of the damped Hessian.
"""
import sys

import numpy as np
import pytest

import oracle
import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def fobq():
    import paper_2509_05576_amd as f
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (no CPU fallback exists)")
    f.load_library()
    return f


@pytest.fixture()
def ctx(fobq):
    c = fobq.Ctx(0)
    yield c
    c.close()


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def _problem(r, d, n, seed, w_std=None):
    rng = np.random.default_rng(seed)
    std = w_std if w_std is not None else np.sqrt(2.0 / d)
    W = (rng.standard_normal((r, d)) * std).astype(np.float32)
    X = np.maximum(rng.standard_normal((d, n)), 0).astype(np.float32)
    return W, X


def _oracle_with_gpu_perm(W, H, gpu_perm, ref, **kw):
    """Several processing orders are correct when two column scores tie to within
    rounding.  If the GPU's order differs from the oracle's only at such ties the
    oracle is re-run with the GPU's order; any other difference is a failure."""
    if np.array_equal(gpu_perm, ref.perm):
        return ref
    assert sorted(gpu_perm.tolist()) == list(range(len(gpu_perm))), "GPU perm is not a permutation"
    bad = np.nonzero(gpu_perm != ref.perm)[0]
    for t in bad:
        a, b = ref.S[ref.perm[t]], ref.S[gpu_perm[t]]
        assert abs(a - b) <= 1e-9 * max(abs(a), abs(b)), f"order differs at step {t} beyond a rounding tie"
    return oracle.quantize_layer(W, H=H, order_mode=oracle.ORDER_CUSTOM, perm=gpu_perm, **kw)


def _compare_layer(out, ref, W, bits, exact=True):
    codes = out.codes.cpu().numpy().astype(np.int64)
    diff = codes != ref.codes
    frac = diff.mean()
    maxlev = np.abs(codes - ref.codes).max()
    assert frac <= 1e-3, f"{frac:.2e} of codes differ"
    assert maxlev <= 1, f"a code differs by {maxlev} levels"
    if exact:
        assert frac == 0.0, f"{diff.sum()} codes differ (fp64 on both sides: expected none)"
    s = out.scales.cpu().numpy().astype(np.float64)
    z = out.zeros.cpu().numpy().astype(np.float64)
    assert np.allclose(s, ref.scales, rtol=1e-5, atol=0)
    assert np.allclose(z, ref.zeros, rtol=1e-5, atol=0)
    loss = float(out.loss.cpu()[0])
    # absolute floor: when every weight sits on its grid (e.g. one column per row) the loss is
    # rounding dust of order eps^2 |W|^2 and has no meaningful relative error
    floor = 1e-24 * float(np.sum(W.astype(np.float64) ** 2))
    assert abs(loss - ref.loss) <= 1e-3 * abs(ref.loss) + floor
    Q = out.Q.cpu().numpy().astype(np.float64)
    if frac == 0.0:
        assert np.allclose(Q, ref.Q, rtol=1e-6, atol=1e-12)
        assert abs(loss - ref.loss) <= 1e-9 * abs(ref.loss) + floor
    return frac


# --------------------------------------------------------------------------- stages
@pytest.mark.parametrize("d,n,ld_pad,chunk", [(128, 512, 0, None), (200, 1000, 0, 256), (300, 777, 3, 100),
                                              (64, 40, 0, None), (17, 5, 1, None),
                                              # 128-wide tiles (triangular diagonal tiles, ranges of equal cost):
                                              (384, 96, 0, None),      # three tile rows, three chunks
                                              (512, 1500, 1, 400),     # unaligned rows, calls of different length
                                              (1000, 2049, 0, 1000),   # eight tile rows, ragged last tile, a one-column call
                                              (640, 700, 0, 33)])      # many short calls (two chunks each)
def test_hessian_matches_oracle(fobq, ctx, d, n, ld_pad, chunk):
    _say(f"hessian d={d} n={n} ld_pad={ld_pad} chunk={chunk}")
    _, X = _problem(1, d, n, 100 + d)
    ref = oracle.hessian(X)
    Xd = torch.zeros((d, n + ld_pad), dtype=torch.float32, device="cuda")
    Xd[:, :n] = _dev(X)
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.hessian(Xd[:, :n], chunk=chunk, H_out=H)
    torch.cuda.synchronize()
    Hh = H.cpu().numpy()
    assert np.allclose(Hh, ref, rtol=1e-12, atol=1e-14)
    assert np.array_equal(Hh, Hh.T)


@pytest.mark.parametrize("n,h,w,c,k,stride,pad,per_call", [
    (3, 9, 7, 5, 3, 1, 1, None),        # ragged everything, one tile
    (2, 8, 8, 16, 1, 1, 0, None),       # 1 x 1 convolution: X is the maps themselves
    (4, 11, 10, 7, 3, 2, 1, 3),         # stride 2, images split over two calls
    (2, 13, 13, 3, 6, 2, 2, None),      # the 6 x 6 stride-2 stem shape
    (3, 10, 10, 130, 3, 1, 1, 2),       # d = 1170: 10 tile rows, ragged last tile, taps change inside a tile
    (1, 5, 5, 4, 5, 1, 0, None),        # kernel covers the whole map: one output pixel per image
    (5, 12, 9, 8, 3, 2, 1, 2),          # channels % 4 == 0 (16-byte loads), stride 2, three calls
    (2, 9, 9, 132, 3, 1, 1, None),      # channels % 4 == 0, d = 1188: several tiles, ragged last tile
])
def test_hessian_from_feature_maps_matches_oracle(fobq, ctx, n, h, w, c, k, stride, pad, per_call):
    # the Hessian of a k x k convolution accumulated straight from NHWC maps equals the
    # Hessian of the unfolded input (the definition, written out on the CPU)
    _say(f"hessian_conv n={n} h={h} w={w} c={c} k={k} stride={stride} pad={pad}")
    rng = np.random.default_rng(n * 1000 + h * 100 + c)
    maps = np.maximum(rng.standard_normal((n, h, w, c)), 0).astype(np.float32)
    X = workloads.im2col(maps, k, stride, pad)
    ref = oracle.hessian(X)
    d = c * k * k
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.hessian_conv(_dev(maps), k, stride, pad, images_per_call=per_call, H_out=H)
    torch.cuda.synchronize()
    Hh = H.cpu().numpy()
    assert np.allclose(Hh, ref, rtol=1e-12, atol=1e-14)
    assert np.array_equal(Hh, Hh.T)


# X X^T by exact int8 slices (FOBQ_HESSIAN_INT8_SLICES): the 19 kept slice products are exact, what is dropped is
# bounded by the weight of the first dropped antidiagonal, 256^-6 relative to the leading products; measured on
# the fp64 emulation of the same slicing the error is 3e-13 of the largest entry.  The bar here: 1e-12 of
# sqrt(H_ii H_jj) for every entry (a relative bound that also holds rows of very different magnitude to account).
def _check_int8_hessian(Hg, H):
    scale = np.sqrt(np.outer(np.diag(H), np.diag(H)))
    scale[scale == 0] = 1.0
    err = np.abs(Hg - H) / scale
    assert err.max() <= 1e-12, f"int8-slice Hessian off by {err.max():.2e} of sqrt(H_ii H_jj)"
    assert np.array_equal(Hg, Hg.T)


@pytest.mark.parametrize("d,n,ld_pad,chunk,kind", [
    (384, 2048, 0, None, "relu"),          # the smallest call the mode applies to: 6 tiles, 64 k-steps
    (500, 5000, 0, None, "relu"),          # ragged rows and columns
    (500, 5000, 3, None, "scaled"),        # unaligned rows; signed values, row magnitudes over 12 decades
    (1000, 20001, 0, 7000, "relu"),        # three calls (the last one 6001 columns), own row exponents per call
    (640, 9000, 0, 4000, "const"),         # constant rows: every slice product adds coherently; last call below
                                           # the mode's minimum length, so it runs the fp64 kernel into the same slabs
])
def test_hessian_int8_slices_matches_oracle(fobq, ctx, d, n, ld_pad, chunk, kind):
    _say(f"int8-slice hessian d={d} n={n} ld_pad={ld_pad} chunk={chunk} {kind}")
    rng = np.random.default_rng(700 + d + n)
    if kind == "relu":
        X = np.maximum(rng.standard_normal((d, n)), 0).astype(np.float32)
    elif kind == "scaled":
        X = (rng.standard_normal((d, n)) * 10.0 ** rng.uniform(-6, 6, size=(d, 1))).astype(np.float32)
    else:
        X = np.repeat(rng.uniform(-3, 3, size=(d, 1)), n, axis=1).astype(np.float32)
    ref = oracle.hessian(X)
    Xd = torch.zeros((d, n + ld_pad), dtype=torch.float32, device="cuda")
    Xd[:, :n] = _dev(X)
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    ctx.hessian(Xd[:, :n], chunk=chunk, H_out=H)
    torch.cuda.synchronize()
    _check_int8_hessian(H.cpu().numpy(), ref)
    # twice the same bits
    H2 = torch.empty_like(H)
    ctx.hessian(Xd[:, :n], chunk=chunk, H_out=H2)
    torch.cuda.synchronize()
    assert torch.equal(H, H2)


@pytest.mark.parametrize("n,h,w,c,k,stride,pad,per_call", [
    (6, 20, 20, 64, 3, 1, 1, None),      # d = 576: channels fill two row blocks exactly
    (12, 47, 41, 44, 3, 2, 1, 5),        # d = 396: row blocks straddle taps; stride 2; calls of 5, 5, 2 images, the
                                         # last one short enough to run the fp64 kernel into the same slabs
    (3, 30, 30, 16, 5, 1, 2, None),      # d = 400, 5 x 5 kernel
    (8, 33, 33, 512, 1, 2, 0, None),     # 1 x 1, stride 2 (projection shortcut)
])
def test_hessian_int8_slices_from_feature_maps_matches_oracle(fobq, ctx, n, h, w, c, k, stride, pad, per_call):
    _say(f"int8-slice hessian_conv n={n} h={h} w={w} c={c} k={k} stride={stride} pad={pad} per_call={per_call}")
    rng = np.random.default_rng(800 + c + k)
    maps = (np.maximum(rng.standard_normal((n, h, w, c)), 0) * 10.0 ** rng.uniform(-3, 3, size=c)).astype(np.float32)
    X = workloads.im2col(maps, k, stride, pad)
    assert X.shape[1] // n * (per_call or n) >= 2048       # else every call falls back to the fp64 kernel
    ref = oracle.hessian(X)
    d = c * k * k
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    ctx.hessian_conv(_dev(maps), k, stride, pad, images_per_call=per_call, H_out=H)
    torch.cuda.synchronize()
    _check_int8_hessian(H.cpu().numpy(), ref)


# Stride 1 with a multiple of 64 channels: the Hessian by tap offsets (two block rows from the digit-product kernel, every
# other block by corrections over single rows and columns of the padded maps).  Same bar as the other int8 cases.
@pytest.mark.parametrize("n,h,w,c,k,pad,per_call", [
    (16, 14, 14, 128, 3, 1, None),       # the usual 3 x 3, pad 1
    (9, 11, 17, 256, 3, 1, 4),           # not square; calls of 4, 4 and 1 image (the last one short)
    (10, 13, 12, 128, 3, 0, None),       # no padding: no strip vanishes
    (6, 12, 15, 128, 3, 2, 3),           # padding wider than the kernel needs
    (12, 16, 9, 128, 2, 1, None),        # 2 x 2 kernel, padding on both sides
    (5, 5, 40, 256, 3, 1, None),         # maps barely taller than the kernel
    (8, 20, 21, 64, 3, 1, 3),            # 64 channels: a base tap is half a 128-row tile
    (6, 10, 12, 192, 3, 1, None),        # 192 channels: the base taps' rows end inside a tile
])
def test_hessian_by_tap_offsets_matches_oracle(fobq, ctx, n, h, w, c, k, pad, per_call):
    _say(f"hessian by tap offsets n={n} h={h} w={w} c={c} k={k} pad={pad} per_call={per_call}")
    rng = np.random.default_rng(900 + c + k + pad + h)
    maps = (np.maximum(rng.standard_normal((n, h, w, c)), 0) * 10.0 ** rng.uniform(-3, 3, size=c)).astype(np.float32)
    X = workloads.im2col(maps, k, 1, pad)
    assert X.shape[1] // n * (per_call or n) >= 512        # the first call decides: it has to take the int8 form
    ref = oracle.hessian(X)
    d = c * k * k
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    ctx.hessian_conv(_dev(maps), k, 1, pad, images_per_call=per_call, H_out=H)
    torch.cuda.synchronize()
    Hh = H.cpu().numpy()
    _check_int8_hessian(Hh, ref)
    assert np.array_equal(Hh, Hh.T)
    # a second accumulation on the same context (slabs and corrections start from zero again)
    ctx.hessian_conv(_dev(maps), k, 1, pad, images_per_call=per_call, H_out=H)
    torch.cuda.synchronize()
    assert np.array_equal(H.cpu().numpy(), Hh)


def test_hessian_by_tap_offsets_rejects_a_strided_later_call(fobq, ctx):
    maps = torch.relu(torch.randn((8, 12, 12, 128), device="cuda"))
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    fobq.fobq_hessian_begin(ctx.handle, 128 * 9)
    fobq.fobq_hessian_accumulate_conv(ctx.handle, maps, 3, 1, 1)
    with pytest.raises(fobq.FobqError) as e:
        fobq.fobq_hessian_accumulate_conv(ctx.handle, maps, 3, 2, 1)
    assert e.value.code == fobq.ESTATE
    fobq.fobq_hessian_finalize(ctx.handle, None)


# At least one 128 x 128 tile per workgroup (256 tiles: d > 2816) and more digits than the memory-side cache holds:
# the workgroups take the tiles in step -- whole rounds, then the tiles left over in several parts, one slab each.
@pytest.mark.parametrize("d,n,chunk", [
    (2900, 18700, None),       # 276 tiles: one round and 20 tiles left over, in 8 parts; ragged d and n
    (3001, 36000, 20000),      # 300 tiles, 44 left over; the second call (16000 columns) is short enough for the
                               # ranges of the smaller layers, into the same slabs
])
def test_hessian_int8_slices_tiles_in_step_matches_oracle(fobq, ctx, d, n, chunk):
    _say(f"int8-slice hessian, tiles in step d={d} n={n} chunk={chunk}")
    X = workloads.relu_normal_f32((d, n), 6, d)
    ref = oracle.hessian(X)
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    ctx.hessian(_dev(X), chunk=chunk, H_out=H)
    torch.cuda.synchronize()
    _check_int8_hessian(H.cpu().numpy(), ref)
    H2 = torch.empty_like(H)                 # a second accumulation on the context, with the slabs already grown
    ctx.hessian(_dev(X), chunk=chunk, H_out=H2)
    torch.cuda.synchronize()
    assert torch.equal(H, H2)


def test_hessian_int8_slices_tiles_in_step_from_feature_maps(fobq, ctx):
    # stride 2 (so not by tap offsets), d = 2880 = 23 tile rows, 20000 output pixels
    n, h, w, c, k, stride, pad = 8, 100, 100, 320, 3, 2, 1
    _say(f"int8-slice hessian_conv, tiles in step n={n} h={h} w={w} c={c} k={k} stride={stride}")
    rng = np.random.default_rng(811)
    maps = np.maximum(rng.standard_normal((n, h, w, c)), 0).astype(np.float32)
    X = workloads.im2col(maps, k, stride, pad)
    assert X.shape == (2880, 20000)
    ref = oracle.hessian(X)
    H = torch.empty((2880, 2880), dtype=torch.float64, device="cuda")
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    ctx.hessian_conv(_dev(maps), k, stride, pad, H_out=H)
    torch.cuda.synchronize()
    _check_int8_hessian(H.cpu().numpy(), ref)
    # the next accumulation on the context is a small one again (ranges, its own count of slabs)
    Xs = np.maximum(rng.standard_normal((500, 3000)), 0).astype(np.float32)
    Hs = torch.empty((500, 500), dtype=torch.float64, device="cuda")
    ctx.hessian(_dev(Xs), H_out=Hs)
    torch.cuda.synchronize()
    _check_int8_hessian(Hs.cpu().numpy(), oracle.hessian(Xs))


@pytest.mark.slow
def test_hessian_int8_slices_long_pieces_fold_in_between(fobq, ctx):
    # 384 rows x 0.72 M columns: 6 tiles x 22528 k-steps over 256 workgroups = 528 k-steps per piece, more than
    # the 512 after which the int32 sums are folded into fp64
    d, n = 384, 720896
    _say(f"int8-slice hessian, long pieces d={d} n={n}")
    X = workloads.relu_normal_f32((d, n), 5, 77)
    ref = oracle.hessian(X)
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    ctx.hessian(_dev(X), H_out=H)
    torch.cuda.synchronize()
    _check_int8_hessian(H.cpu().numpy(), ref)


def test_hessian_int8_slices_mode_errors_and_non_finite_input(fobq, ctx):
    with pytest.raises(fobq.FobqError) as e:
        ctx.set_hessian_mode(7)
    assert e.value.code == fobq.EINVAL
    X = torch.relu(torch.randn((384, 4096), device="cuda"))
    fobq.fobq_hessian_begin(ctx.handle, 384)
    fobq.fobq_hessian_accumulate(ctx.handle, X)
    with pytest.raises(fobq.FobqError) as e:
        ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)      # not in the middle of an accumulation
    assert e.value.code == fobq.ESTATE
    fobq.fobq_hessian_finalize(ctx.handle)
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES)
    # an Inf among the inputs: H is NaN throughout, the layer fails as not positive definite, and the context
    # works again afterwards
    Xb = X.clone()
    Xb[17, 1234] = float("inf")
    H = torch.empty((384, 384), dtype=torch.float64, device="cuda")
    ctx.hessian(Xb, H_out=H)
    torch.cuda.synchronize()
    assert bool(torch.isnan(H).all())
    W = torch.randn((8, 384), device="cuda")
    with pytest.raises(fobq.FobqError) as e:
        ctx.quantize_layer(W)
    assert e.value.code == fobq.ENOTPD
    ctx.hessian(X, H_out=H)
    ctx.quantize_layer(W)
    assert bool(torch.isfinite(H).all())


def test_hessian_conv_argument_and_state_errors(fobq, ctx):
    maps = _dev(np.ones((2, 6, 6, 4), dtype=np.float32))
    X = _dev(np.ones((36, 10), dtype=np.float32))
    fobq.fobq_hessian_begin(ctx.handle, 36)
    for kw in ({"k": 2}, {"k": 3, "stride": 0}, {"k": 3, "pad": -1}):
        with pytest.raises(fobq.FobqError) as e:
            fobq.fobq_hessian_accumulate_conv(ctx.handle, maps, **kw)
        assert e.value.code == fobq.EINVAL
    with pytest.raises(fobq.FobqError) as e:      # 7 x 7 kernel does not fit a 6 x 6 map
        fobq.fobq_hessian_begin(ctx.handle, 4 * 49)
        fobq.fobq_hessian_accumulate_conv(ctx.handle, maps, 7)
    assert e.value.code == fobq.EINVAL
    fobq.fobq_hessian_begin(ctx.handle, 36)
    fobq.fobq_hessian_accumulate_conv(ctx.handle, maps, 3, 1, 1)
    with pytest.raises(fobq.FobqError) as e:      # plain and convolution calls do not mix
        fobq.fobq_hessian_accumulate(ctx.handle, X)
    assert e.value.code == fobq.ESTATE
    fobq.fobq_hessian_begin(ctx.handle, 36)
    fobq.fobq_hessian_accumulate(ctx.handle, X)
    with pytest.raises(fobq.FobqError) as e:
        fobq.fobq_hessian_accumulate_conv(ctx.handle, maps, 3, 1, 1)
    assert e.value.code == fobq.ESTATE
    fobq.fobq_hessian_finalize(ctx.handle)


@pytest.mark.parametrize("d", [1, 7, 64, 65, 100, 128, 129, 192, 257, 300, 1000])
def test_spd_inverse_matches_oracle(fobq, ctx, d):
    _say(f"spd_inverse d={d}")
    _, X = _problem(1, d, max(2 * d, 8), 200 + d)
    Hd, _ = oracle.damp(oracle.hessian(X), 0.01)
    ref = oracle.spd_inverse(Hd)
    got = fobq.fobq_spd_inverse(ctx.handle, _dev(Hd)).cpu().numpy()
    scale = np.abs(ref).max()
    assert np.max(np.abs(got - ref)) <= 1e-9 * scale
    assert np.allclose(got @ Hd, np.eye(d), atol=1e-8)
    assert np.array_equal(got, got.T)


def test_spd_inverse_reports_non_pd(fobq, ctx):
    _, X = _problem(1, 96, 32, 3)            # N < d: singular
    H = oracle.hessian(X)
    with pytest.raises(fobq.FobqError) as e:
        fobq.fobq_spd_inverse(ctx.handle, _dev(H))
    assert e.value.code == fobq.ENOTPD
    # the context stays usable
    Hd, _ = oracle.damp(H, 0.01)
    got = fobq.fobq_spd_inverse(ctx.handle, _dev(Hd)).cpu().numpy()
    assert np.allclose(got @ Hd, np.eye(96), atol=1e-8)


@pytest.mark.parametrize("r,d,bits,group", [(64, 128, 4, 0), (33, 96, 3, 32), (130, 70, 8, 0), (5, 600, 2, 200)])
def test_sensitivity_and_order_match_oracle(fobq, ctx, r, d, bits, group):
    _say(f"sensitivity r={r} d={d} bits={bits} group={group}")
    W, X = _problem(r, d, 3 * d, 300 + d)
    Hd, _ = oracle.damp(oracle.hessian(X), 0.01)
    Hinv = oracle.spd_inverse(Hd)
    s, z = oracle.grid(W, bits, group)
    S_ref = oracle.sensitivity(W, np.ascontiguousarray(np.diag(Hinv)), bits, group, s, z)
    S, perm = fobq.fobq_sensitivity(ctx.handle, _dev(W), _dev(Hinv), bits=bits, group=group)
    S = S.cpu().numpy()
    assert np.allclose(S, S_ref, rtol=1e-12, atol=0)
    # order: exactly the stable descending order of the GPU's own scores, and equal to the
    # oracle's order wherever the scores are separated by more than rounding
    p = perm.cpu().numpy()
    assert np.array_equal(p, np.argsort(-S, kind="stable").astype(np.int32))
    p_ref = oracle.order(S_ref)
    if not np.array_equal(p, p_ref):
        for t in np.nonzero(p != p_ref)[0]:
            assert abs(S_ref[p_ref[t]] - S_ref[p[t]]) <= 1e-9 * abs(S_ref[p_ref[t]])


# --------------------------------------------------------------------------- whole path, small
SMALL = [
    # r, d, n, bits, group, order, block
    (64, 128, 512, 4, 0, 1, 0),
    (64, 128, 512, 4, 0, 1, 1),
    (70, 200, 450, 3, 0, 1, 0),       # ragged rows, ragged last block
    (70, 200, 450, 3, 0, 1, 1),
    (70, 200, 450, 3, 0, 1, 16),
    (33, 192, 100, 4, 64, 1, 0),      # groups, N < d (rank deficient without damping)
    (33, 192, 100, 4, 64, 0, 1),      # natural order, unblocked
    (300, 320, 900, 8, 0, 1, 0),
    (1, 64, 200, 2, 0, 1, 0),         # single row
    (16, 1, 10, 4, 0, 1, 0),          # single column
    (9, 63, 200, 5, 0, 0, 7),         # odd block width
]


@pytest.mark.parametrize("r,d,n,bits,group,order,block", SMALL)
def test_quantize_layer_matches_oracle(fobq, ctx, r, d, n, bits, group, order, block):
    _say(f"layer r={r} d={d} n={n} bits={bits} group={group} order={order} block={block}")
    W, X = _problem(r, d, n, 400 + r + d + bits, w_std=0.05)
    Xd = _dev(X)
    ctx.hessian(Xd)
    out = ctx.quantize_layer(_dev(W), bits=bits, group=group, order=order, block=block, damp=0.01)
    ref = oracle.quantize_layer(W, X=X, bits=bits, group=group, order_mode=order)
    ref = _oracle_with_gpu_perm(W, ref.H, out.perm.cpu().numpy(), ref, bits=bits, group=group)
    _compare_layer(out, ref, W, bits)


# Layers whose first panels have 800 or more trailing tiles: the panel is stored by a launch of its own and the
# trailing tiles take one product each.  3001 columns: the elimination's launches are of that kind, the Cholesky's
# carry the inverse and are not; 4200 columns (beyond 4096: separate inverse): both.  Ragged last blocks.
@pytest.mark.parametrize("r,d,n,int8", [(16, 3001, 3300, False), (12, 4200, 4500, True)])
def test_stored_panel_layers_match_oracle(fobq, ctx, r, d, n, int8):
    _say(f"stored-panel layer r={r} d={d} n={n} int8={int8}")
    W, X = _problem(r, d, n, 7000 + d, w_std=0.02)
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES if int8 else fobq.HESSIAN_FP64)
    ctx.hessian(_dev(X))
    out = ctx.quantize_layer(_dev(W), bits=4, group=0, damp=0.01)
    _say("stored-panel layer: oracle")
    ref = oracle.quantize_layer(W, X=X, bits=4, group=0)
    ref = _oracle_with_gpu_perm(W, ref.H, out.perm.cpu().numpy(), ref, bits=4, group=0)
    _compare_layer(out, ref, W, 4)


def test_random_small_layers_match_oracle(fobq, ctx):
    # seeded draw of shapes and options: block counts from 1 to 10 with ragged tails, every bit width,
    # groups, the blocked, narrow-block and unblocked column loops
    rng = np.random.default_rng(20250905)
    for case in range(24):
        d = int(rng.integers(1, 640))
        r = int(rng.integers(1, 260))
        n = int(rng.integers(max(4, d // 2), 3 * d + 8))
        bits = int(rng.integers(2, 9))
        divisors = [g for g in (8, 16, 32, 64, 128) if d % g == 0]
        group = int(rng.choice(divisors)) if divisors and rng.random() < 0.4 else 0
        order = int(rng.choice([0, 1, 1, 5]))
        block = int(rng.choice([0, 0, 0, 64, 32, 1]))
        _say(f"random layer {case}: r={r} d={d} n={n} bits={bits} group={group} order={order} block={block}")
        W, X = _problem(r, d, n, 9000 + case, w_std=0.05)
        ctx.hessian(_dev(X))
        out = ctx.quantize_layer(_dev(W), bits=bits, group=group, order=order, block=block, damp=0.01)
        ref = oracle.quantize_layer(W, X=X, bits=bits, group=group, order_mode=order)
        ref = _oracle_with_gpu_perm(W, ref.H, out.perm.cpu().numpy(), ref, bits=bits, group=group)
        _compare_layer(out, ref, W, bits)


@pytest.mark.parametrize("order", [3, 4, 5, 6, 7])
def test_ablation_orders_match_oracle(fobq, ctx, order):
    # the sort keys and directions of the ordering ablation (Section 4.1, Table 3)
    _say(f"order {order}")
    W, X = _problem(48, 170, 500, 30 + order, w_std=0.05)
    H = oracle.hessian(X)
    out = ctx.quantize_layer(_dev(W), _dev(H), bits=4, order=order)
    ref = oracle.quantize_layer(W, H=H, bits=4, order_mode=order)
    ref = _oracle_with_gpu_perm(W, H, out.perm.cpu().numpy(), ref, bits=4)
    _compare_layer(out, ref, W, 4)
    kind, asc = oracle._ORDER_KEYS[order]
    key = oracle.column_key(W, np.diag(ref.Hinv).copy(), 4, 0, ref.scales, ref.zeros, kind)
    S, perm = fobq.fobq_sensitivity(ctx.handle, _dev(W), _dev(ref.Hinv), bits=4, order=order)
    assert np.allclose(S.cpu().numpy(), key, rtol=1e-12)
    assert np.array_equal(perm.cpu().numpy(), out.perm.cpu().numpy())


@pytest.mark.parametrize("r,d,n,bits,group,stop", [(48, 170, 500, 4, 0, -1), (33, 96, 300, 3, 32, -1),
                                                   (20, 130, 400, 4, 0, 57), (70, 1100, 2500, 4, 0, -1)])
def test_dynamic_order_matches_oracle(fobq, ctx, r, d, n, bits, group, stop):
    # Section 5 read literally: the scores are recomputed and the order decided before every column
    _say(f"dynamic order r={r} d={d} bits={bits} group={group} stop_after={stop}")
    W, X = _problem(r, d, n, 600 + r + d, w_std=0.05)
    H = oracle.hessian(X)
    out = ctx.quantize_layer(_dev(W), _dev(H), bits=bits, group=group, order=fobq.ORDER_SENSI_DYNAMIC,
                             stop_after=stop)
    steps = d if stop < 0 else stop
    ref = oracle.quantize_layer(W, H=H, bits=bits, group=group, order_mode=oracle.ORDER_SENSI_DYNAMIC, steps=steps)
    perm = out.perm.cpu().numpy()
    assert sorted(perm.tolist()) == list(range(d))
    assert np.array_equal(perm[:steps], ref.perm[:steps])
    _compare_layer(out, ref, W, bits)
    # the static order is a different one on these inputs (otherwise this test shows nothing)
    assert not np.array_equal(ref.perm, oracle.quantize_layer(W, H=H, bits=bits, group=group).perm)
    with pytest.raises(fobq.FobqError) as e:
        fobq.fobq_sensitivity(ctx.handle, _dev(W), _dev(ref.Hinv), bits=bits, group=group,
                              order=fobq.ORDER_SENSI_DYNAMIC)
    assert e.value.code == fobq.EINVAL


def test_custom_order_and_explicit_h(fobq, ctx):
    W, X = _problem(40, 150, 400, 5, w_std=0.05)
    H = oracle.hessian(X)
    perm = np.random.default_rng(6).permutation(150).astype(np.int32)
    out = ctx.quantize_layer(_dev(W), _dev(H), bits=4, order=fobq.ORDER_CUSTOM, perm_in=_dev(perm))
    ref = oracle.quantize_layer(W, H=H, bits=4, order_mode=oracle.ORDER_CUSTOM, perm=perm)
    assert np.array_equal(out.perm.cpu().numpy(), perm)
    _compare_layer(out, ref, W, 4)


def test_bad_custom_order_is_rejected(fobq, ctx):
    W, X = _problem(8, 32, 100, 7)
    H = _dev(oracle.hessian(X))
    for bad in ([0] * 32, list(range(31)) + [40], list(range(31)) + [-1]):
        with pytest.raises(fobq.FobqError) as e:
            ctx.quantize_layer(_dev(W), H, order=fobq.ORDER_CUSTOM, perm_in=_dev(np.array(bad, dtype=np.int32)))
        assert e.value.code == fobq.EINVAL


def test_argument_errors(fobq, ctx):
    W, X = _problem(8, 32, 100, 8)
    Wd, H = _dev(W), _dev(oracle.hessian(X))
    for kw in ({"bits": 1}, {"bits": 9}, {"group": 5}, {"block": 65}, {"stop_after": 33}, {"damp": -1.0},
               {"order": 9}, {"order": -1}, {"order": fobq.ORDER_CUSTOM}):
        with pytest.raises(fobq.FobqError) as e:
            ctx.quantize_layer(Wd, H, **kw)
        assert e.value.code == fobq.EINVAL, kw
    with pytest.raises(fobq.FobqError) as e:       # no Hessian in the context
        ctx.quantize_layer(Wd)
    assert e.value.code == fobq.ESTATE
    with pytest.raises(fobq.FobqError) as e:       # accumulate before begin
        fobq.fobq_hessian_accumulate(ctx.handle, _dev(X))
    assert e.value.code == fobq.ESTATE
    ctx.hessian(_dev(X))
    with pytest.raises(fobq.FobqError) as e:       # d_col mismatch with the accumulated Hessian
        ctx.quantize_layer(_dev(W[:, :16].copy()))
    assert e.value.code == fobq.EINVAL
    ctx.quantize_layer(Wd)                          # and the context still works


@pytest.mark.parametrize("block", [0, 1])
def test_rank_deficient_without_damping_is_enotpd(fobq, ctx, block):
    W, X = _problem(8, 96, 32, 9)
    ctx.hessian(_dev(X))
    with pytest.raises(fobq.FobqError) as e:
        ctx.quantize_layer(_dev(W), damp=0.0, block=block)
    assert e.value.code == fobq.ENOTPD
    ctx.quantize_layer(_dev(W), damp=0.01, block=block)


@pytest.mark.parametrize("block", [0, 1])
def test_failure_with_work_in_flight_leaves_the_context_usable(fobq, ctx, block):
    # the n-th internal status check reports a failure (host-side test hook; every kernel that was
    # launched still runs to its end): the call must wait for what it enqueued, and a good layer on
    # the same context must then match the oracle
    r, d, n = 40, 200, 500
    W, X = _problem(r, d, n, 77, w_std=0.05)
    Wd, Xd = _dev(W), _dev(X)
    ref = oracle.quantize_layer(W, X=X, bits=4)
    ctx.hessian(Xd)
    ctx.quantize_layer(Wd, bits=4, block=block)          # workspace exists: later checks are launches
    for nth in (1, 5, 12, 20, 26, 33):
        _say(f"injected failure at check {nth}, block={block}")
        fobq.fobq_debug_fail_after(ctx.handle, nth)
        with pytest.raises(fobq.FobqError) as e:
            ctx.quantize_layer(Wd, bits=4, block=block)
        assert e.value.code == fobq.EHIP and "injected" in str(e.value)
        out = ctx.quantize_layer(Wd, bits=4, block=block)
        _compare_layer(out, ref, W, 4)
    # enqueue / finish: a failed enqueue leaves nothing pending
    fobq.fobq_debug_fail_after(ctx.handle, 15)
    with pytest.raises(fobq.FobqError):
        ctx.quantize_layer(Wd, bits=4, block=block, wait=False)
    ctx.finish()
    out = ctx.quantize_layer(Wd, bits=4, block=block, wait=False)
    ctx.finish()
    _compare_layer(out, ref, W, 4)


@pytest.mark.parametrize("block", [0, 1, 16])
def test_stop_after_snapshots(fobq, ctx, block):
    r, d, n = 37, 150, 400
    W, X = _problem(r, d, n, 10, w_std=0.05)
    H = oracle.hessian(X)
    Hd_, Wd_ = _dev(H), _dev(W)
    for t in [0, 1, 16, 64, 77, 149, 150]:
        _say(f"snapshot block={block} t={t}")
        out = ctx.quantize_layer(Wd_, Hd_, bits=4, block=block, stop_after=t, debug=True)
        ref = oracle.quantize_layer(W, H=H, bits=4, steps=t)
        p = out.perm.cpu().numpy()
        ref = _oracle_with_gpu_perm(W, H, p, ref, bits=4, steps=t)
        # running weights, processing order -> original order
        Ww = np.empty((r, d))
        Ww[:, p] = out.W_work.cpu().numpy()
        assert np.allclose(Ww, ref.W_work, rtol=1e-9, atol=1e-12)
        Hw = np.empty((d, d))
        Hw[np.ix_(p, p)] = out.Hinv_work.cpu().numpy()
        assert np.max(np.abs(Hw - ref.Hinv_work)) <= 1e-9 * np.abs(ref.Hinv).max()
        codes = out.codes.cpu().numpy().astype(np.int64)
        assert np.array_equal(codes, ref.codes)
        assert abs(float(out.loss.cpu()[0]) - ref.loss) <= 1e-9 * abs(ref.loss) + 1e-300


def test_stop_after_snapshots_of_a_tall_layer(fobq, ctx):
    # many more rows than columns: the deferred compensation is most of the column loop's work.  Stops after an even and
    # an odd number of blocks, inside a block, and at the end; the running weights must be the oracle's at each.
    r, d, n = 1100, 330, 700
    W, X = _problem(r, d, n, 14, w_std=0.05)
    H = oracle.hessian(X)
    Hd_, Wd_ = _dev(H), _dev(W)
    full = ctx.quantize_layer(Wd_, Hd_, bits=4, block=0)
    for t in [64, 128, 150, 192, 256, 300, 330]:
        _say(f"tall snapshot t={t}")
        out = ctx.quantize_layer(Wd_, Hd_, bits=4, block=0, stop_after=t, debug=True)
        ref = oracle.quantize_layer(W, H=H, bits=4, steps=t)
        p = out.perm.cpu().numpy()
        ref = _oracle_with_gpu_perm(W, H, p, ref, bits=4, steps=t)
        Ww = np.empty((r, d))
        Ww[:, p] = out.W_work.cpu().numpy()
        assert np.allclose(Ww, ref.W_work, rtol=1e-9, atol=1e-12)
        assert np.array_equal(out.codes.cpu().numpy().astype(np.int64), ref.codes)
        assert abs(float(out.loss.cpu()[0]) - ref.loss) <= 1e-9 * abs(ref.loss) + 1e-300
    # the same layer with the unblocked path (one pass per column): same codes
    one = ctx.quantize_layer(Wd_, Hd_, bits=4, block=1)
    assert torch.equal(full.codes, one.codes)


def test_blocked_and_unblocked_agree_and_runs_are_deterministic(fobq, ctx):
    W, X = _problem(100, 260, 700, 11, w_std=0.05)
    Wd_ = _dev(W)
    ctx.hessian(_dev(X))
    a = ctx.quantize_layer(Wd_, bits=4, block=0)
    b = ctx.quantize_layer(Wd_, bits=4, block=1)
    c = ctx.quantize_layer(Wd_, bits=4, block=0)
    assert torch.equal(a.codes, b.codes)
    assert torch.equal(a.codes, c.codes) and torch.equal(a.Q, c.Q) and torch.equal(a.loss, c.loss)
    assert abs(float(a.loss[0]) - float(b.loss[0])) <= 1e-10 * float(a.loss[0])


def test_loss_equals_layer_output_error_plus_damping_term(fobq, ctx):
    # property that holds at any size: loss = (1/N)|(W-Q)X|^2 + lambda/2 |W-Q|^2, from X directly
    W, X = _problem(50, 180, 500, 12, w_std=0.05)
    ctx.hessian(_dev(X))
    out = ctx.quantize_layer(_dev(W), bits=4)
    Q = out.Q.cpu().numpy().astype(np.float64)
    lam = 0.01 * np.mean(np.diag(oracle.hessian(X)))
    dW = W.astype(np.float64) - Q
    expect = oracle.output_error(W, Q, X) + 0.5 * lam * np.sum(dW ** 2)
    assert abs(float(out.loss.cpu()[0]) - expect) <= 1e-6 * expect


def test_stage_timing_of_chosen_stages(fobq, ctx):
    # FOBQ_PROFILE_STAGE masks: only the chosen stages record events; True times every stage
    W, X = _problem(24, 200, 300, 77, w_std=0.05)
    Wd_, Xd = _dev(W), _dev(X)
    chol, xxt = fobq.STAGES.index("cholesky"), fobq.STAGES.index("xxt")
    fobq.fobq_profile_enable(ctx.handle, fobq.FOBQ_PROFILE_STAGE(xxt))
    fobq.fobq_profile_reset(ctx.handle)
    ctx.hessian(Xd)
    ctx.quantize_layer(Wd_, bits=4)
    st = ctx.stage_ms()
    assert st["xxt"][1] == 1 and st["xxt"][0] > 0.0
    assert all(st[name][1] == 0 for name in fobq.STAGES if name != "xxt")
    fobq.fobq_profile_enable(ctx.handle, fobq.FOBQ_PROFILE_STAGE(xxt) + fobq.FOBQ_PROFILE_STAGE(chol))
    fobq.fobq_profile_reset(ctx.handle)
    ctx.hessian(Xd)
    ctx.quantize_layer(Wd_, bits=4)
    st = ctx.stage_ms()
    assert st["xxt"][1] == 1 and st["cholesky"][1] == 1 and st["columns"][1] == 0
    fobq.fobq_profile_enable(ctx.handle, True)
    fobq.fobq_profile_reset(ctx.handle)
    ctx.hessian(Xd)
    ctx.quantize_layer(Wd_, bits=4)
    st = ctx.stage_ms()
    assert all(st[name][1] >= 1 for name in ("xxt", "finalize", "cholesky", "order", "permute", "columns", "emit"))
    fobq.fobq_profile_enable(ctx.handle, False)
    fobq.fobq_profile_reset(ctx.handle)
    ctx.hessian(Xd)
    ctx.quantize_layer(Wd_, bits=4)
    assert all(v[1] == 0 for v in ctx.stage_ms().values())


def test_enqueue_and_finish_on_several_contexts(fobq, ctx):
    # independent layers in flight on three contexts / streams at once give the results of the blocking call
    probs = [_problem(40 + 10 * i, 150 + 40 * i, 500, 40 + i, w_std=0.05) for i in range(3)]
    streams = [torch.cuda.Stream() for _ in probs]
    ctxs = [fobq.Ctx(0, stream=s.cuda_stream) for s in streams]
    torch.cuda.synchronize()
    keep, outs = [], []
    for c, (W, X) in zip(ctxs, probs):
        Wd_, Xd = _dev(W), _dev(X)
        keep.append((Wd_, Xd))
        torch.cuda.synchronize()                     # inputs were produced on torch's stream
        c.hessian(Xd)
        outs.append(c.quantize_layer(Wd_, bits=4, wait=False))
    with pytest.raises(fobq.FobqError) as e:        # one layer per context until fobq_finish
        ctxs[0].quantize_layer(keep[0][0], bits=4, wait=False)
    assert e.value.code == fobq.ESTATE
    for c in ctxs:
        c.finish()
    for (W, X), out in zip(probs, outs):
        ref = oracle.quantize_layer(W, X=X, bits=4)
        ref = _oracle_with_gpu_perm(W, ref.H, out.perm.cpu().numpy(), ref, bits=4)
        _compare_layer(out, ref, W, 4)
    # a failure detected on the device is reported by fobq_finish
    _, Xs = _problem(1, 96, 32, 3)
    ctxs[0].hessian(_dev(Xs))
    Ws = _dev(np.ones((4, 96), dtype=np.float32))
    ctxs[0].quantize_layer(Ws, bits=4, damp=0.0, wait=False)
    with pytest.raises(fobq.FobqError) as e:
        ctxs[0].finish()
    assert e.value.code == fobq.ENOTPD
    ctxs[0].finish()                                 # nothing pending: synchronises, no error
    for c in ctxs:
        c.close()


# Batched small layers: every stage is one launch for all layers of the batch.  Shapes mix everything the
# sweeps' small layers have: one to four panels, ragged d_col and d_row, a single row, a single column, groups.
BATCH_SHAPES = [(64, 64, 300), (256, 64, 200), (32, 32, 100), (255, 128, 500), (64, 256, 700), (1024, 256, 400),
                (33, 147, 400), (128, 108, 300), (1, 200, 400), (17, 1, 9), (40, 65, 100), (300, 192, 90)]


@pytest.mark.parametrize("bits,group,order", [(4, 0, 1), (3, 0, 0), (8, 0, 6), (4, 32, 1)])
def test_batched_small_layers_match_oracle(fobq, ctx, bits, group, order):
    _say(f"batched small layers bits={bits} group={group} order={order}")
    Ws, Xs, Wd, Hd = [], [], [], []
    for i, (r, d, n) in enumerate(BATCH_SHAPES):
        if group and d % group:
            continue                    # the group width must divide every d_col of the batch
        W, X = _problem(r, d, n, 5000 + i, w_std=0.05)
        Ws.append(W)
        Xs.append(X)
        Wd.append(_dev(W))
        H = torch.empty((d, d), dtype=torch.float64, device="cuda")
        ctx.hessian(_dev(X), H_out=H)
        Hd.append(H)
    outs = ctx.quantize_layers_batched(Wd, Hd, bits=bits, group=group, order=order, damp=0.01)
    torch.cuda.synchronize()
    for W, X, H, out in zip(Ws, Xs, Hd, outs):
        Hh = H.cpu().numpy()
        ref = oracle.quantize_layer(W, H=Hh, bits=bits, group=group, order_mode=order)
        ref = _oracle_with_gpu_perm(W, Hh, out.perm.cpu().numpy(), ref, bits=bits, group=group)
        _compare_layer(out, ref, W, bits)
    # the same layers one at a time through fobq_quantize_layer: same codes, same order
    for Wt, H, out in zip(Wd, Hd, outs):
        single = ctx.quantize_layer(Wt, H, bits=bits, group=group, order=order, damp=0.01)
        assert torch.equal(single.codes, out.codes) and torch.equal(single.perm, out.perm)
        assert torch.allclose(single.loss, out.loss, rtol=1e-9)


def test_batched_small_layers_errors(fobq, ctx):
    W = torch.randn((8, 300), device="cuda")
    H = torch.eye(300, dtype=torch.float64, device="cuda")
    with pytest.raises(fobq.FobqError) as e:
        ctx.quantize_layers_batched([W], [H])                  # more than 256 columns
    assert e.value.code == fobq.EINVAL and "layer 0" in str(e.value)
    W = torch.randn((8, 64), device="cuda")
    H = torch.eye(64, dtype=torch.float64, device="cuda")
    with pytest.raises(fobq.FobqError) as e:
        ctx.quantize_layers_batched([W], [H], order=fobq.ORDER_SENSI_DYNAMIC)
    assert e.value.code == fobq.EINVAL
    assert ctx.quantize_layers_batched([], []) == []
    # a layer whose Hessian is not positive definite is named; the others are complete
    Hbad = -torch.eye(64, dtype=torch.float64, device="cuda")
    outs = [None, None]
    with pytest.raises(fobq.FobqError) as e:
        ctx.quantize_layers_batched([W, W], [H, Hbad], damp=0.0)
    assert e.value.code == fobq.ENOTPD and "layer 1" in str(e.value)
    out = ctx.quantize_layers_batched([W, W], [H, H])
    assert torch.equal(out[0].codes, out[1].codes)


def test_non_finite_inputs_do_not_break_the_context(fobq, ctx):
    # NaN / Inf in the inputs are not rejected on the host; they must neither fault nor poison later calls
    W, X = _problem(20, 130, 400, 14, w_std=0.05)
    H = oracle.hessian(X)
    Xbad = X.copy()
    Xbad[5, 7] = np.nan
    ctx.hessian(_dev(Xbad))
    with pytest.raises(fobq.FobqError) as e:          # H has a NaN row: no positive pivot
        ctx.quantize_layer(_dev(W), bits=4)
    assert e.value.code == fobq.ENOTPD
    Wbad = W.copy()
    Wbad[3, 10] = np.nan
    Wbad[4, 11] = np.inf
    out = ctx.quantize_layer(_dev(Wbad), _dev(H), bits=4)        # returns; the order is still a permutation
    assert sorted(out.perm.cpu().numpy().tolist()) == list(range(130))
    good = [i for i in range(20) if i not in (3, 4)]
    assert torch.isfinite(out.Q[good]).all()
    # and the context still gives the right answer afterwards
    out = ctx.quantize_layer(_dev(W), _dev(H), bits=4)
    ref = oracle.quantize_layer(W, H=H, bits=4)
    ref = _oracle_with_gpu_perm(W, H, out.perm.cpu().numpy(), ref, bits=4)
    _compare_layer(out, ref, W, 4)


def test_maximum_d_row(fobq, ctx):
    # the largest d_row the library accepts, checked against the oracle in full
    r, d = 65535, 96
    _say(f"maximum d_row: {r} x {d}")
    W, X = _problem(r, d, 400, 13, w_std=0.05)
    H = oracle.hessian(X)
    out = ctx.quantize_layer(_dev(W), _dev(H), bits=4, group=32)
    ref = oracle.quantize_layer(W, H=H, bits=4, group=32)
    ref = _oracle_with_gpu_perm(W, H, out.perm.cpu().numpy(), ref, bits=4, group=32)
    _compare_layer(out, ref, W, 4)
    with pytest.raises(fobq.FobqError) as e:
        ctx.quantize_layer(torch.zeros((65536, 8), dtype=torch.float32, device="cuda"),
                           torch.eye(8, dtype=torch.float64, device="cuda"))
    assert e.value.code == fobq.EINVAL


@pytest.mark.slow
@pytest.mark.parametrize("d", [16384, 32768])
def test_large_d_col_properties(fobq, ctx, d):
    """d_col far beyond what the oracle can follow (32768 is the largest the library accepts): the
    properties that hold at any size.  The order is a permutation, the codes are on the grid, and the
    loss accumulated step by step equals 1/2 tr(dW H_d dW^T) evaluated from the Hessian -- which only
    holds if the inverse, the elimination and every compensation step are right."""
    r, n = 8, 2048
    _say(f"large d_col: {r} x {d}, N = {n}")
    rng = np.random.default_rng(d)
    X = torch.from_numpy(np.maximum(rng.standard_normal((d, n)), 0).astype(np.float32)).cuda()
    W = torch.from_numpy((rng.standard_normal((r, d)) * 0.02).astype(np.float32)).cuda()
    H = torch.empty((d, d), dtype=torch.float64, device="cuda")
    ctx.hessian(X, H_out=H)
    _say("large d_col: quantize")
    out = ctx.quantize_layer(W, bits=4, damp=0.01)
    _say("large d_col: checks")
    perm = out.perm.cpu().numpy()
    assert np.array_equal(np.sort(perm), np.arange(d))
    assert int(out.codes.max()) <= 15
    lam = 0.01 * float(torch.diagonal(H).mean())
    dW = W.double() - out.Q.double()
    expect = 0.5 * float(((dW @ H) * dW).sum()) + 0.5 * lam * float((dW * dW).sum())
    loss = float(out.loss.cpu()[0])
    assert abs(loss - expect) <= 1e-6 * expect, (loss, expect)
    # Q is what the codes say
    G = out.scales.shape[1]
    q = out.scales.double() * (out.codes.double().reshape(r, G, -1).permute(2, 0, 1) - out.zeros.double())
    assert torch.allclose(q.permute(1, 2, 0).reshape(r, d), out.Q.double(), rtol=1e-6, atol=1e-12)
    with pytest.raises(fobq.FobqError) as e:
        fobq.fobq_hessian_begin(ctx.handle, 32769)
    assert e.value.code == fobq.EINVAL


# --------------------------------------------------------------------------- the benchmark configurations
def _run_config(fobq, ctx, name, rows=None, block=0, chunk=None, spec=None, int8=False):
    spec = spec if spec is not None else workloads.configs()[name]
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES if int8 else fobq.HESSIAN_FP64)
    _say(f"config {name}: generating inputs")
    W = spec.make_w()
    from_maps = spec.conv is not None and name != "c2_resnet50_3x3"
    if from_maps:
        # a sweep layer that is a k x k or strided convolution: the GPU path gets the input maps
        # (`chunk` = images per call), the oracle their unfolding
        maps = spec.make_maps()
        _images, _side, _ch, k, pad = spec.conv
        Md = _dev(maps)
        _say(f"config {name}: GPU path from the feature maps (k={k} stride={spec.stride} pad={pad})")
        if chunk is not None:
            ctx.hessian_conv(Md, k, spec.stride, pad, images_per_call=chunk)
            Hc = torch.empty((spec.d_col, spec.d_col), dtype=torch.float64, device="cuda")
            fobq.fobq_hessian_finalize(ctx.handle, Hc)
            torch.cuda.synchronize()
            Hc = Hc.cpu().numpy()
        ctx.hessian_conv(Md, k, spec.stride, pad)
        out = ctx.quantize_layer(_dev(W), bits=spec.bits, group=spec.group, damp=spec.damp, block=block)
        del Md
        _say(f"config {name}: unfolding the maps for the oracle")
        X = workloads.im2col(maps, k, spec.stride, pad)
        del maps
        assert X.shape == (spec.d_col, spec.n)
    else:
        X = spec.make_x()
        Xd = _dev(X)
        _say(f"config {name}: GPU path")
        if chunk is not None:
            # accumulation over several calls gives the same Hessian as one call (up to summation order)
            ctx.hessian(Xd, chunk=chunk)
            Hc = torch.empty((spec.d_col, spec.d_col), dtype=torch.float64, device="cuda")
            fobq.fobq_hessian_finalize(ctx.handle, Hc)
            torch.cuda.synchronize()
            Hc = Hc.cpu().numpy()
        ctx.hessian(Xd)          # one launch over all calibration columns: the configuration bench.py times
        out = ctx.quantize_layer(_dev(W), bits=spec.bits, group=spec.group, damp=spec.damp, block=block)
        del Xd
    _say(f"config {name}: oracle")
    H = oracle.hessian(X)
    del X
    Hg = torch.empty((spec.d_col, spec.d_col), dtype=torch.float64, device="cuda")
    fobq.fobq_hessian_finalize(ctx.handle, Hg)
    torch.cuda.synchronize()
    if int8:
        _check_int8_hessian(Hg.cpu().numpy(), H)
        if chunk is not None:
            _check_int8_hessian(Hc, H)
    else:
        assert np.allclose(Hg.cpu().numpy(), H, rtol=1e-11, atol=1e-13)
        if chunk is not None:
            assert np.allclose(Hc, H, rtol=1e-11, atol=1e-13)
    if rows is None:
        ref = oracle.quantize_layer(W, H=H, bits=spec.bits, group=spec.group, damp_rel=spec.damp)
        ref = _oracle_with_gpu_perm(W, H, out.perm.cpu().numpy(), ref, bits=spec.bits, group=spec.group,
                                    damp_rel=spec.damp)
        # with the int8-slice Hessian the two sides differ by 3e-13 in H, not only by summation order: the bar
        # of the benchmark spec applies (at most 1e-3 of the codes, none by more than one level; loss 1e-3), and the
        # count of differing codes is printed
        frac = _compare_layer(out, ref, W, spec.bits, exact=not int8)
    else:
        # rows of W never interact once the order is fixed: the oracle quantizes a sample of rows
        # under the order computed from ALL rows
        Hd, _lam = oracle.damp(H, spec.damp)
        Hinv = oracle.spd_inverse(Hd)
        s, z = oracle.grid(W, spec.bits, spec.group)
        S = oracle.sensitivity(W, np.ascontiguousarray(np.diag(Hinv)), spec.bits, spec.group, s, z)
        p_ref = oracle.order(S)
        p = out.perm.cpu().numpy()
        if not np.array_equal(p, p_ref):
            assert sorted(p.tolist()) == list(range(spec.d_col))
            for t in np.nonzero(p != p_ref)[0]:
                a, b = S[p_ref[t]], S[p[t]]
                assert abs(a - b) <= 1e-9 * max(abs(a), abs(b))
        sel = np.unique(np.linspace(0, spec.d_row - 1, rows).astype(int))
        _say(f"config {name}: oracle column loop on {len(sel)} sampled rows")
        ref = oracle.column_loop(np.ascontiguousarray(W[sel]), Hinv, p, spec.bits, spec.group,
                                 np.ascontiguousarray(s[sel]), np.ascontiguousarray(z[sel]))
        codes = out.codes.cpu().numpy().astype(np.int64)[sel]
        diff = codes != ref.codes
        frac = diff.mean()
        assert frac <= 1e-3 and np.abs(codes - ref.codes).max() <= 1
        assert frac == 0.0
        assert np.allclose(out.scales.cpu().numpy(), s, rtol=1e-5)
        assert np.allclose(out.zeros.cpu().numpy(), z, rtol=1e-5)
        assert np.allclose(out.Q.cpu().numpy()[sel], ref.Q, rtol=1e-6, atol=1e-12)
        # the loss over all rows, from the definition, with the GPU's Q
        Q = out.Q.cpu().numpy().astype(np.float64)
        expect = oracle.loss_eval(W, Q, Hd)
        assert abs(float(out.loss.cpu()[0]) - expect) <= 1e-3 * expect
    _say(f"config {name}: {frac:.2e} of codes differ")


def test_config_c1_tiny(fobq, ctx):
    _run_config(fobq, ctx, "c1_tiny")
    _run_config(fobq, ctx, "c1_tiny", block=1)


def test_config_c2_resnet50_3x3(fobq, ctx):
    _run_config(fobq, ctx, "c2_resnet50_3x3", chunk=6272)


@pytest.mark.parametrize("name,chunk", [("c2_resnet50_3x3", None), ("c3a_expand_w4", 8000), ("c3a_expand_w8", None)])
def test_config_with_int8_slice_hessian(fobq, ctx, name, chunk):
    _run_config(fobq, ctx, name, chunk=chunk, int8=True)


@pytest.mark.slow
def test_config_c5_large_d_with_int8_slice_hessian(fobq, ctx):
    _run_config(fobq, ctx, "c5_large_d", int8=True)


@pytest.mark.slow
@pytest.mark.parametrize("model,layer,chunk", [
    ("resnet50", "resnet50_64x576_n401408_0", None),       # 3 x 3 from maps, 925 MB of unfolded input in one call
    ("resnet50", "resnet50_128x1152_n100352_0", 50),       # 3 x 3 stride 2, calls of 50, 50, 28 images
    ("resnet50", "resnet50_512x4608_n6272_0", None),       # N barely above d_col
    ("yolov5s", "yolov5s_128x576_n819200_0", None),        # 1.9 GB of unfolded input: two launches of the matrix kernel
])
def test_config_c4_sweep_layers_with_int8_slice_hessian(fobq, ctx, model, layer, chunk):
    spec = next(l for l in workloads.sweep_layers(model) if l.name == layer)
    _run_config(fobq, ctx, layer, chunk=chunk, spec=spec, int8=True)


def test_config_c2_hessian_from_feature_maps(fobq, ctx):
    # config 2 with the Hessian accumulated from the 128 x 14 x 14 x 256 maps instead of the
    # unfolded 2304 x 25088 matrix: same H, same codes
    spec = workloads.configs()["c2_resnet50_3x3"]
    _images, _side, _ch, k, pad = spec.conv
    _say("config c2 from feature maps")
    maps = spec.make_maps()
    W = spec.make_w()
    X = workloads.im2col(maps, k, 1, pad)
    H = oracle.hessian(X)
    Hg = torch.empty((spec.d_col, spec.d_col), dtype=torch.float64, device="cuda")
    ctx.hessian_conv(_dev(maps), k, 1, pad, H_out=Hg)
    out = ctx.quantize_layer(_dev(W), bits=spec.bits, group=spec.group, damp=spec.damp)
    assert np.allclose(Hg.cpu().numpy(), H, rtol=1e-11, atol=1e-13)
    ref = oracle.quantize_layer(W, H=H, bits=spec.bits, group=spec.group, damp_rel=spec.damp)
    ref = _oracle_with_gpu_perm(W, H, out.perm.cpu().numpy(), ref, bits=spec.bits, group=spec.group,
                                damp_rel=spec.damp)
    _compare_layer(out, ref, W, spec.bits)


@pytest.mark.parametrize("name", ["c3a_expand_w8", "c3a_expand_w4"])
def test_config_c3a(fobq, ctx, name):
    _run_config(fobq, ctx, name)


@pytest.mark.parametrize("name", ["c3b_fc_w8", "c3b_fc_w4"])
def test_config_c3b(fobq, ctx, name):
    _run_config(fobq, ctx, name)


@pytest.mark.parametrize("name", ["c1_tiny", pytest.param("c3a_expand_w4", marks=pytest.mark.slow)])
def test_config_with_dynamic_order(fobq, ctx, name):
    spec = workloads.configs()[name]
    _say(f"config {name}, dynamic order")
    W, X = spec.make_w(), spec.make_x()
    ctx.hessian(_dev(X))
    out = ctx.quantize_layer(_dev(W), bits=spec.bits, group=spec.group, damp=spec.damp,
                             order=fobq.ORDER_SENSI_DYNAMIC)
    ref = oracle.quantize_layer(W, X=X, bits=spec.bits, group=spec.group, damp_rel=spec.damp,
                                order_mode=oracle.ORDER_SENSI_DYNAMIC)
    assert np.array_equal(out.perm.cpu().numpy(), ref.perm)
    _compare_layer(out, ref, W, spec.bits)


@pytest.mark.slow
def test_config_c5_large_d(fobq, ctx):
    # every one of the 2048 rows against the oracle
    _run_config(fobq, ctx, "c5_large_d")


# config 4 (whole-model sweep): parity on layers of the sweep, fed as the sweep feeds them (k x k and
# strided convolutions from their seeded input maps, the rest from X), one per kernel path that the other
# configs do not reach: ragged d_col (147, 108) and d_row (255), very long calibration sets accumulated
# over several calls, the 64-wide tiles of X X^T (d_col = 64, 288, 576), strided 3 x 3 and 1 x 1
# convolutions, d_col = 1152 and 1024, d_col = 4608 with N barely above d_col, and N << d_col.
# (model, layer, images or columns per call of the chunked accumulation)
SWEEP_CASES = [
    ("resnet50", "resnet50_64x147_n1605632_0", 48),        # 7 x 7 stride 2 stem
    ("resnet50", "resnet50_64x576_n401408_0", None),       # 3 x 3, 64-wide tiles
    ("resnet50", "resnet50_128x1152_n100352_0", 50),       # 3 x 3 stride 2
    ("resnet50", "resnet50_512x256_n100352_0", None),      # 1 x 1 stride 2 (projection shortcut)
    ("resnet50", "resnet50_512x1024_n25088_0", 10000),     # 1 x 1, d_row 512
    ("resnet50", "resnet50_512x4608_n6272_0", None),       # 3 x 3 stride 2, N barely above d_col
    ("resnet50", "resnet50_1000x2048_n128_0", None),       # classifier, N << d_col
    ("yolov5s", "yolov5s_32x108_n13107200_0", 40),         # 6 x 6 stride 2 stem, 13.1 M columns
    ("yolov5s", "yolov5s_64x288_n3276800_0", None),        # 3 x 3 stride 2, 64-wide tiles
    ("yolov5s", "yolov5s_32x64_n3276800_0", 1 << 20),      # 1 x 1, one 64-wide tile
    ("yolov5s", "yolov5s_255x128_n819200_0", 200000),      # detection head, ragged d_row
]


@pytest.mark.slow
@pytest.mark.parametrize("model,layer,chunk", SWEEP_CASES)
def test_config_c4_sweep_layers(fobq, ctx, model, layer, chunk):
    spec = next(l for l in workloads.sweep_layers(model) if l.name == layer)
    _run_config(fobq, ctx, layer, chunk=chunk, spec=spec)


def test_int8_matrix_rate_probe(fobq, ctx):
    """The measurement aid returns a rate between zero and the published int8 peak for every operand kind,
    the loop on equal bytes is not slower than on random ones, and an unknown kind is an error."""
    _say("int8 matrix rate probe")
    rates = [ctx.probe_int8_matrix_rate(k) for k in (fobq.PROBE_EQUAL_BYTES, fobq.PROBE_RANDOM_BYTES, fobq.PROBE_RELU_DIGITS)]
    assert all(100.0 < r < 5200.0 for r in rates), rates
    assert rates[0] >= 0.95 * rates[1], rates
    with pytest.raises(fobq.FobqError):
        ctx.probe_int8_matrix_rate(7)


# --------------------------------------------------------------------------- the per-row baseline (OBQ)
OBQ_CASES = [
    # r, d, n, bits, group, rows
    (64, 128, 512, 4, 0, None),        # config 1's shape, the inverse in LDS
    (33, 96, 300, 3, 32, (5, 29)),     # groups, a row range
    (20, 200, 450, 4, 0, (0, 20)),     # beyond 128 columns: the rows' inverses in device scratch
    (6, 333, 700, 2, 111, (1, 6)),     # ragged everything
    (3, 1, 10, 4, 0, None),            # single column
]


@pytest.mark.parametrize("r,d,n,bits,group,rows", OBQ_CASES)
def test_obq_rows_match_oracle(fobq, ctx, r, d, n, bits, group, rows):
    """fobq_obq_rows against the oracle's per-row baseline on the same Hinv: both take every step's decisions
    (greedy choice, grid code) in fp64 with the same operations, so order and codes are compared exactly;
    a row whose orders differ must differ at a tie of the loss terms (relative gap below 1e-9)."""
    _say(f"obq rows r={r} d={d} bits={bits} group={group} rows={rows}")
    W, X = _problem(r, d, n, 900 + r + d, w_std=0.05)
    Hd, _ = oracle.damp(oracle.hessian(X), 0.01)
    Hinv = oracle.spd_inverse(Hd)
    s, z = oracle.grid(W, bits, group)
    ref = oracle.obq_rows(W, Hinv, bits, group, s, z, rows)
    codes, Q, order, lossrow = ctx.obq_rows(_dev(W), _dev(Hinv), bits=bits, group=group, rows=rows)
    lo, hi = (0, r) if rows is None else rows
    codes, Q, order, lossrow = (t.cpu().numpy() for t in (codes, Q, order, lossrow))
    same_order = np.all(order[lo:hi] == ref.order[lo:hi], axis=1)
    assert same_order.mean() >= 0.9, f"{(~same_order).sum()} of {hi - lo} rows took another order"
    rows_same = np.arange(lo, hi)[same_order]
    assert np.array_equal(codes[rows_same].astype(np.int64), ref.codes[rows_same])
    assert np.allclose(Q[rows_same], ref.Q[rows_same], rtol=1e-6, atol=0)
    assert np.allclose(lossrow[rows_same], ref.lossrow[rows_same], rtol=1e-9, atol=0)
    # a row with another order: valid permutation, loss within the layer tolerance
    for i in np.arange(lo, hi)[~same_order]:
        assert sorted(order[i].tolist()) == list(range(d))
        assert abs(lossrow[i] - ref.lossrow[i]) <= 1e-3 * ref.lossrow[i]
    # rows outside the range are untouched
    assert not codes[:lo].any() and not codes[hi:].any()


def test_obq_rows_errors(fobq, ctx):
    W = torch.zeros((4, 4160), dtype=torch.float32, device="cuda")
    Hinv = torch.eye(4160, dtype=torch.float64, device="cuda")
    with pytest.raises(fobq.FobqError, match="small layers"):
        ctx.obq_rows(W, Hinv)
    W = torch.ones((4, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(fobq.FobqError, match="rows"):
        ctx.obq_rows(W, torch.eye(8, dtype=torch.float64, device="cuda"), rows=(2, 9))
    with pytest.raises(fobq.FobqError) as e:
        ctx.obq_rows(W, -torch.eye(8, dtype=torch.float64, device="cuda"))
    assert e.value.code == fobq.ENOTPD
