"""GPU parity: the HIP kernels, called through the C ABI, against the CPU oracle on identical
seeded inputs, element by element: at sizes the oracle finishes in seconds (several workgroup
passes and a ragged tail) and at the benchmark's full sizes, where every token of y and dx is
compared (the oracle walks the tensor in chunks) next to the full dalpha/dbeta reductions."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_08343_amd as wht
from paper_2603_08343_amd import binding, synth
from parity import assert_grad_close, assert_io_close, nan_filled, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def _announce(msg):
    print(f"[parity] {msg}", flush=True)


def _method(d):
    return "matrix" if d <= 512 else "fast"


TWELVE_D = [768, 1536, 3072, 6144, 12288]      # d = 12 * 2^m: H = P12 (x) Sylvester, bfloat16 only


def run_forward(inp):
    x = to_gpu(inp.x, inp.dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y = wht.wht_affine_forward(x, a, b)
    torch.cuda.synchronize()
    return y


def run_backward(inp):
    x, dy = to_gpu(inp.x, inp.dtype), to_gpu(inp.dy, inp.dtype)
    a = torch.from_numpy(inp.alpha).cuda()
    out = wht.wht_affine_backward(dy, x, a)
    torch.cuda.synchronize()
    return out


def check_forward_full(inp, what):
    y = run_forward(inp)
    ref = oracle.forward(inp.x, inp.alpha, inp.beta, _method(inp.d))
    assert_io_close(y, ref.reshape(inp.N, inp.d), inp.dtype, f"{what} y")


def check_backward_full(inp, what):
    dx, da, db = run_backward(inp)
    rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, _method(inp.d))
    assert_io_close(dx, rdx.reshape(inp.N, inp.d), inp.dtype, f"{what} dx")
    assert_grad_close(da, rda, f"{what} dalpha")
    assert_grad_close(db, rdb, f"{what} dbeta")


CHUNK = 4096      # tokens per oracle call at full size (bounds the float64 working set)


def _assert_all_tokens(got_t, ref_of_chunk, N, dtype, what):
    """Every token of a full-size output against the oracle, CHUNK tokens at a time."""
    for lo in range(0, N, CHUNK):
        hi = min(N, lo + CHUNK)
        assert_io_close(got_t[lo:hi], ref_of_chunk(lo, hi), dtype, f"{what} tokens {lo}..{hi - 1}")


ALL_D = [32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", ALL_D)
def test_forward_every_d(d, dtype):
    # N chosen so that the last workgroup pass is ragged for every tokens-per-workgroup value
    if dtype == "f32" and d > 8192:
        pytest.skip("float32 tensors are limited to WHT_MAX_D_F32 = 8192")
    N = 67 if d <= 2048 else 9
    _announce(f"forward d={d} {dtype} N={N}")
    check_forward_full(synth.make_inputs(N, d, dtype, seed=d, backward=False), f"fwd d={d} {dtype}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", ALL_D)
def test_backward_every_d(d, dtype):
    if dtype == "f32" and d > 8192:
        pytest.skip("float32 tensors are limited to WHT_MAX_D_F32 = 8192")
    N = 67 if d <= 2048 else 9
    _announce(f"backward d={d} {dtype} N={N}")
    check_backward_full(synth.make_inputs(N, d, dtype, seed=d + 1), f"bwd d={d} {dtype}")


@pytest.mark.parametrize("d", TWELVE_D)
def test_forward_twelve_widths(d):
    # 67 / 9 tokens: ragged last pass for every tokens-per-workgroup value (4 at d = 768, else 1)
    N = 67 if d <= 1536 else 9
    _announce(f"forward d={d} (12 * 2^m) bf16 N={N}")
    inp = synth.make_inputs(N, d, "bf16", seed=d, backward=False)
    y = run_forward(inp)
    # the first tokens against the O(d^2) definition, everything against the fast method
    ref_def = oracle.forward(inp.x[:3], inp.alpha, inp.beta, "matrix")
    assert_io_close(y[:3], ref_def, "bf16", f"fwd d={d} y vs definition")
    assert_io_close(y, oracle.forward(inp.x, inp.alpha, inp.beta, "fast"), "bf16", f"fwd d={d} y")


@pytest.mark.parametrize("d", TWELVE_D)
def test_backward_twelve_widths(d):
    N = 67 if d <= 1536 else 9
    _announce(f"backward d={d} (12 * 2^m) bf16 N={N}")
    check_backward_full(synth.make_inputs(N, d, "bf16", seed=d + 1), f"bwd d={d}")


@pytest.mark.parametrize("d", [768, 6144])
def test_twelve_widths_unit_vectors_and_blocks(d):
    # one-hot inputs make every sign of a column of H visible in y (alpha = 1, beta = 0): any wrong
    # entry of the order-12 factor, block order or slot mapping shows up as a sign flip
    m = d // 12
    ks = [0, 1, 8, m - 1, m, 3 * m + 5, 7 * m + 16, 11 * m, d - 1]
    x = np.zeros((len(ks), d), dtype=np.float32)
    for row, k in enumerate(ks):
        x[row, k] = 1.0
    _announce(f"one-hot columns d={d}")
    xb = synth.f32_to_bf16_bits(x)
    y = wht.wht_affine_forward(to_gpu(xb, "bf16"), torch.ones(d, device="cuda"), torch.zeros(d, device="cuda"))
    torch.cuda.synchronize()
    ref = oracle.forward(xb, np.ones(d), np.zeros(d), "matrix")
    got = to_f64(y)
    assert np.array_equal(np.sign(got), np.sign(ref))
    assert_io_close(y, ref, "bf16", f"one-hot d={d}")


@pytest.mark.parametrize("d,N", [(768, 263), (1536, 67), (6144, 35), (12288, 5)])
def test_forward_residual_twelve_widths(d, N):
    _announce(f"forward+residual d={d} (12 * 2^m) N={N}")
    inp = synth.make_inputs(N, d, "bf16", seed=d + 7)
    x, resid = to_gpu(inp.x, "bf16"), to_gpu(inp.dy, "bf16")
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y = wht.wht_affine_forward_residual(x, a, b, resid)
    torch.cuda.synchronize()
    ref = oracle.forward_residual(inp.x, inp.alpha, inp.beta, inp.dy, "fast")
    assert_io_close(y, ref, "bf16", f"fwd+resid d={d}")


@pytest.mark.parametrize("N", [1, 2, 3, 5, 127, 129, 1031])
def test_twelve_widths_reduction_over_odd_token_counts(N):
    _announce(f"reduction N={N} d=768")
    check_backward_full(synth.make_inputs(N, 768, "bf16", seed=N), f"bwd N={N} d=768")


@pytest.mark.parametrize("d", [1536, 6144])
def test_twelve_width_full_size(d):
    # the paper's Base width, and the widest 12 * 2^m row of the benchmark, at a training-sized
    # batch: every token of y and dx, full reductions
    N = 32768
    _announce(f"full size N={N} d={d}: generating inputs")
    inp = synth.make_inputs(N, d, "bf16", seed=0)
    x, dy = to_gpu(inp.x, "bf16"), to_gpu(inp.dy, "bf16")
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y = wht.wht_affine_forward(x, a, b, y=nan_filled(N, d, "bf16"))
    dx, da, db = wht.wht_affine_backward(dy, x, a, dx=nan_filled(N, d, "bf16"))
    torch.cuda.synchronize()
    _announce(f"d={d}: every token against the oracle")
    _assert_all_tokens(y, lambda lo, hi: oracle.forward(inp.x[lo:hi], inp.alpha, inp.beta, "fast"), N, "bf16", f"d={d} y")
    _assert_all_tokens(dx, lambda lo, hi: oracle.backward(inp.dy[lo:hi], inp.x[lo:hi], inp.alpha, "fast",
                                                          want_param_grads=False)[0], N, "bf16", f"d={d} dx")
    _, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, "fast", want_dx=False)
    assert_grad_close(da, rda, f"d={d} dalpha")
    assert_grad_close(db, rdb, f"d={d} dbeta")


@pytest.mark.parametrize("N", [1, 2, 3, 127, 128, 129, 1031])
@pytest.mark.parametrize("d,dtype", [(256, "f32"), (1024, "bf16"), (8192, "bf16")])
def test_reduction_over_odd_token_counts(N, d, dtype):
    if d == 8192 and N > 129:
        N = 257
    _announce(f"reduction N={N} d={d} {dtype}")
    check_backward_full(synth.make_inputs(N, d, dtype, seed=N), f"bwd N={N} d={d}")


@pytest.mark.parametrize("N", [2048, 2085, 4099])
def test_forward_clustered_deal_with_ragged_regions(N):
    # d = 8192 with at least 4 x 512 token groups: the forward kernels deal the groups to clusters of
    # workgroups, each with its own contiguous region (four regions, two with the residual); token
    # counts that do not divide evenly leave the last region short.  Every element is checked.
    _announce(f"clustered forward d=8192 N={N}")
    inp = synth.make_inputs(N, 8192, "bf16", seed=N)
    x, resid = to_gpu(inp.x, "bf16"), to_gpu(inp.dy, "bf16")
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y = wht.wht_affine_forward(x, a, b)
    yr = wht.wht_affine_forward_residual(x, a, b, resid)
    torch.cuda.synchronize()
    assert_io_close(y, oracle.forward(inp.x, inp.alpha, inp.beta, "fast"), "bf16", f"clustered y N={N}")
    assert_io_close(yr, oracle.forward_residual(inp.x, inp.alpha, inp.beta, inp.dy, "fast"), "bf16",
                    f"clustered y+resid N={N}")


def test_many_passes_per_workgroup():
    # more token groups than the grid cap: every workgroup loops several times, last pass ragged
    inp = synth.make_inputs(70005, 256, "bf16", seed=3)
    _announce("grid-stride d=256 N=70005 (tokens per workgroup 32, 2188 groups)")
    check_forward_full(inp, "fwd strided")
    inp2 = synth.make_inputs(140001, 64, "f32", seed=4)
    _announce("grid-stride d=64 N=140001")
    check_forward_full(inp2, "fwd strided d=64")
    check_backward_full(inp2, "bwd strided d=64")


# ------------------------------------------------------------------ few tokens per call (decoding)
#
# Calls of up to 2^22 elements (2^24 for bfloat16 rows of 1024 and 2048 elements, 2^21 for d = 12 * 2^m)
# run on a kernel of their own:
# one token group per workgroup, no token loop.  The small cases above pass through it; the cases
# here pin the decode shapes of the paper's Table 2 widths, the hand-over to the persistent kernel
# and that kernel just above the limit, where it has the fewest passes per workgroup.

def _few_token_limit(d, dtype="bf16"):
    """Largest N that runs the one-pass kernel (the library's rule, restated)."""
    if d % 3 == 0:
        elems = 1 << 21
    elif dtype == "bf16" and d in (1024, 2048):
        elems = 1 << 24
    else:
        elems = 1 << 22
    return elems // d


@pytest.mark.parametrize("N", [1, 16, 64, 256])
@pytest.mark.parametrize("d,dtype", [(768, "bf16"), (1024, "bf16"), (1536, "bf16"), (2048, "bf16"), (4096, "bf16"),
                                     (8192, "bf16"), (16384, "bf16"), (12288, "bf16"), (512, "bf16"),
                                     (256, "f32"), (4096, "f32")])
def test_forward_few_tokens(d, dtype, N):
    _announce(f"few tokens: forward and forward+residual d={d} {dtype} N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=3 * d + N)      # dy doubles as the residual stream
    x, resid = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    # one row more than the call may touch: it must keep its NaN fill
    buf, bufr = nan_filled(N + 1, d, dtype), nan_filled(N + 1, d, dtype)
    y = wht.wht_affine_forward(x, a, b, y=buf[:N])
    yr = wht.wht_affine_forward_residual(x, a, b, resid, y=bufr[:N])
    ys, sumsq = wht.wht_affine_forward_residual_stats(x, a, b, resid)
    torch.cuda.synchronize()
    assert_io_close(y, oracle.forward(inp.x, inp.alpha, inp.beta, _method(d)), dtype, f"few d={d} N={N} y")
    assert_io_close(yr, oracle.forward_residual(inp.x, inp.alpha, inp.beta, inp.dy, _method(d)), dtype,
                    f"few d={d} N={N} y+resid")
    assert bool(torch.isnan(buf[N].float()).all()) and bool(torch.isnan(bufr[N].float()).all())
    # with the norm statistic: the same y, and the statistic of the unrounded values
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(ys.view(bits), yr.view(bits))
    _, ref_sq = oracle.forward_residual_stats(inp.x, inp.alpha, inp.beta, inp.dy, _method(d))
    np.testing.assert_allclose(to_f64(sumsq), ref_sq, rtol=1e-5)


@pytest.mark.parametrize("d,dtype", [(d, "bf16") for d in ALL_D + TWELVE_D] + [(d, "f32") for d in ALL_D[:-1]])
def test_forward_on_both_sides_of_the_few_token_limit(d, dtype):
    # N = limit runs the one-pass kernel, N = limit + 37 the persistent one (ragged last group): both
    # against the oracle, and bit for bit against each other on the rows they share.
    lim = _few_token_limit(d, dtype)
    N = lim + 37
    _announce(f"few-token limit d={d} {dtype}: N={lim} and N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=d + 11, backward=False)
    x = to_gpu(inp.x, dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y_few = wht.wht_affine_forward(x[:lim], a, b, y=nan_filled(lim, d, dtype))
    y_all = wht.wht_affine_forward(x, a, b, y=nan_filled(N, d, dtype))
    torch.cuda.synchronize()
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(y_few.view(bits), y_all[:lim].view(bits))
    _assert_all_tokens(y_all, lambda lo, hi: oracle.forward(inp.x[lo:hi], inp.alpha, inp.beta, "fast"),
                       N, dtype, f"limit d={d} y")


@pytest.mark.parametrize("d,dtype", [(256, "f32"), (512, "bf16"), (1024, "bf16"), (2048, "bf16"), (4096, "bf16"),
                                     (768, "bf16"), (6144, "bf16"), (16384, "bf16"), (4096, "f32")])
def test_forward_residual_stats_above_the_few_token_limit(d, dtype):
    # the persistent kernel's residual + statistic variant, ragged last group, every width class
    N = _few_token_limit(d, dtype) + 37
    _announce(f"forward+residual+stats above the few-token limit d={d} {dtype} N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=d + 13)
    x, resid = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y, ss = wht.wht_affine_forward_residual_stats(x, a, b, resid, y=nan_filled(N, d, dtype))
    torch.cuda.synchronize()
    got = to_f64(ss)
    for lo in range(0, N, CHUNK):
        hi = min(N, lo + CHUNK)
        ref_y, ref_ss = oracle.forward_residual_stats(inp.x[lo:hi], inp.alpha, inp.beta, inp.dy[lo:hi], "fast")
        assert_io_close(y[lo:hi], ref_y, dtype, f"stats above limit d={d} y tokens {lo}..{hi - 1}")
        assert np.max(np.abs(got[lo:hi] - ref_ss) / ref_ss) <= 1e-5


# ------------------------------------------------------------------ residual add fused into the epilogue

@pytest.mark.parametrize("d,dtype,N", [(64, "f32", 70), (256, "f32", 64), (512, "bf16", 131), (1024, "bf16", 263),
                                       (2048, "bf16", 67), (4096, "bf16", 35), (8192, "bf16", 1031),
                                       (16384, "bf16", 5), (8192, "f32", 9)])
def test_forward_residual(d, dtype, N):
    _announce(f"forward+residual d={d} {dtype} N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=d + 7)          # dy doubles as the residual stream
    x, resid = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y = wht.wht_affine_forward_residual(x, a, b, resid)
    torch.cuda.synchronize()
    ref = oracle.forward_residual(inp.x, inp.alpha, inp.beta, inp.dy, _method(d))
    assert_io_close(y, ref, dtype, f"fwd+resid d={d} {dtype}")
    # in place on the residual stream, as a framework would call it
    wht.wht_affine_forward_residual(x, a, b, resid, y=resid)
    torch.cuda.synchronize()
    assert torch.equal(resid.view(torch.int16 if dtype == "bf16" else torch.int32),
                       y.view(torch.int16 if dtype == "bf16" else torch.int32))


@pytest.mark.parametrize("d,dtype,N", [(32, "f32", 70), (64, "bf16", 300), (256, "f32", 64), (512, "bf16", 131),
                                       (1024, "bf16", 263), (2048, "bf16", 67), (4096, "bf16", 35),
                                       (8192, "bf16", 2085), (16384, "bf16", 5), (8192, "f32", 9),
                                       (768, "bf16", 263), (1536, "bf16", 67), (6144, "bf16", 35), (12288, "bf16", 5)])
def test_forward_residual_stats(d, dtype, N):
    """The fused residual forward that also returns sum_j y^2 per token: y must be bit-identical to
    the call without the statistic; the statistic is checked against the oracle's (1e-5 relative: it
    is a float32 sum of d squares of float32 values that themselves carry ~1e-6) and against the sum
    of squares of the kernel's own stored y (which differs by the rounding of y to its dtype)."""
    _announce(f"forward+residual+stats d={d} {dtype} N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=d + 11)
    x, resid = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y_plain = wht.wht_affine_forward_residual(x, a, b, resid)
    y, ss = wht.wht_affine_forward_residual_stats(x, a, b, resid)
    torch.cuda.synchronize()
    view = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(y.view(view), y_plain.view(view))
    ref_y, ref_ss = oracle.forward_residual_stats(inp.x, inp.alpha, inp.beta, inp.dy, _method(d))
    got = ss.cpu().numpy().astype(np.float64)
    assert got.shape == (N,) and np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref_ss) / ref_ss) <= 1e-5
    stored = np.sum(to_f64(y) ** 2, axis=1)
    assert np.max(np.abs(got - stored) / stored) <= (2e-2 if dtype == "bf16" else 1e-5)
    # second call with the same inputs: the reduction order is fixed
    y2, ss2 = wht.wht_affine_forward_residual_stats(x, a, b, resid)
    torch.cuda.synchronize()
    assert torch.equal(ss2, ss)


def test_forward_residual_full_size_C5():
    w = synth.WORKLOADS["C5_large"]
    _announce("forward+residual at C5 size, every token")
    inp = synth.make_workload("C5_large")
    x, resid = to_gpu(inp.x, "bf16"), to_gpu(inp.dy, "bf16")
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y = wht.wht_affine_forward_residual(x, a, b, resid, y=nan_filled(w.N, w.d, "bf16"))
    torch.cuda.synchronize()
    _assert_all_tokens(y, lambda lo, hi: oracle.forward_residual(inp.x[lo:hi], inp.alpha, inp.beta, inp.dy[lo:hi], "fast"),
                       w.N, "bf16", "C5 fwd+resid")


# ------------------------------------------------------------------ the benchmark configurations

def test_config_C1_tiny():
    inp = synth.make_workload("C1_tiny")
    _announce("C1 tiny N=64 d=256 f32")
    check_forward_full(inp, "C1")
    # the definition itself, not only the butterfly oracle
    y = run_forward(inp)
    assert_io_close(y, oracle.forward(inp.x, inp.alpha, inp.beta, "matrix"), "f32", "C1 vs matrix")


@pytest.mark.parametrize("N", [1, 16, 64, 256])
def test_config_C4_decode(N):
    inp = synth.make_workload(f"C4_decode_n{N}")
    _announce(f"C4 decode N={N} d=4096 bf16")
    check_forward_full(inp, f"C4 N={N}")


def _full_size(name, check_bwd):
    w = synth.WORKLOADS[name]
    _announce(f"{name} full size N={w.N} d={w.d} {w.dtype}: generating inputs")
    inp = synth.make_workload(name)
    x = to_gpu(inp.x, inp.dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    _announce(f"{name}: forward on GPU, then every token against the oracle")
    y = wht.wht_affine_forward(x, a, b, y=nan_filled(w.N, w.d, inp.dtype))
    torch.cuda.synchronize()
    _assert_all_tokens(y, lambda lo, hi: oracle.forward(inp.x[lo:hi], inp.alpha, inp.beta, "fast"),
                       w.N, inp.dtype, f"{name} y")
    # a few tokens against the O(d^2) definition as well
    few = np.array([0, 1, w.N // 2, w.N - 2, w.N - 1])
    assert_io_close(y[torch.from_numpy(few).cuda()], oracle.forward(inp.x[few], inp.alpha, inp.beta, "matrix"),
                    inp.dtype, f"{name} y (definition)")
    del y
    if not check_bwd:
        return
    _announce(f"{name}: backward on GPU")
    dy = to_gpu(inp.dy, inp.dtype)
    dx, da, db = wht.wht_affine_backward(dy, x, a, dx=nan_filled(w.N, w.d, inp.dtype))
    torch.cuda.synchronize()
    _announce(f"{name}: oracle dalpha/dbeta over all {w.N} tokens")
    _, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, "fast", want_dx=False)
    assert_grad_close(da, rda, f"{name} dalpha")
    assert_grad_close(db, rdb, f"{name} dbeta")
    _announce(f"{name}: dx, every token against the oracle")
    _assert_all_tokens(dx, lambda lo, hi: oracle.backward(inp.dy[lo:hi], inp.x[lo:hi], inp.alpha, "fast",
                                                          want_param_grads=False)[0],
                       w.N, inp.dtype, f"{name} dx")


def test_config_C2_training_full_size():
    _full_size("C2_train", True)


def test_config_C3_prefill_full_size_with_outliers():
    _full_size("C3_prefill", False)


def test_config_C4b_roofline_shape_full_size():
    _full_size("C4b_roofline", True)


def test_config_C5_large_full_size():
    _full_size("C5_large", True)


# ------------------------------------------------------------------ edge cases and the boundary

def test_special_inputs():
    d, N = 1024, 5
    ones, zeros = torch.ones(d, device="cuda"), torch.zeros(d, device="cuda")
    inp = synth.make_inputs(N, d, "f32", seed=9, backward=False)
    x = to_gpu(inp.x, "f32")
    # alpha = 1, beta = 0: y = Hx, and applying the layer twice returns x (H is an involution)
    z = wht.wht_affine_forward(x, ones, zeros)
    back = wht.wht_affine_forward(z, ones, zeros)
    torch.cuda.synchronize()
    assert float((back - x).abs().max()) <= 1e-5 * float(x.abs().max())
    # x = 0: y = beta exactly
    b = torch.from_numpy(inp.beta).cuda()
    y0 = wht.wht_affine_forward(torch.zeros(N, d, device="cuda"), torch.from_numpy(inp.alpha).cuda(), b)
    assert torch.equal(y0, b.expand(N, d))
    # unit vector: y = alpha * column k of H + beta
    k = 37
    e = torch.zeros(1, d, device="cuda")
    e[0, k] = 1.0
    ye = wht.wht_affine_forward(e, torch.from_numpy(inp.alpha).cuda(), b)
    ref = oracle.forward(e.cpu().numpy(), inp.alpha, inp.beta, "matrix")
    assert_io_close(ye, ref, "f32", "unit vector")


def test_in_place_and_preallocated_outputs():
    inp = synth.make_inputs(33, 2048, "bf16", seed=11)
    x, dy = to_gpu(inp.x, "bf16"), to_gpu(inp.dy, "bf16")
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    y_ref = wht.wht_affine_forward(x, a, b)
    x2 = x.clone()
    wht.wht_affine_forward(x2, a, b, y=x2)                       # y aliases x exactly
    dx_ref, da_ref, db_ref = wht.wht_affine_backward(dy, x, a)
    dy2 = dy.clone()
    dx2, da2, db2 = wht.wht_affine_backward(dy2, x, a, dx=dy2)   # dx aliases dy exactly
    torch.cuda.synchronize()
    assert torch.equal(x2.view(torch.int16), y_ref.view(torch.int16))
    assert torch.equal(dx2.view(torch.int16), dx_ref.view(torch.int16))
    assert torch.equal(da2, da_ref) and torch.equal(db2, db_ref)


@pytest.mark.parametrize("d,dtype,N", [(4096, "bf16", 523), (8192, "bf16", 261), (6144, "bf16", 70), (2048, "bf16", 300),
                                       (1024, "f32", 67)])
@pytest.mark.parametrize("alias", ["x", "dy"])
def test_backward_dx_aliases_an_input(d, dtype, N, alias):
    # the header allows dx to alias x or dy exactly: several token groups per workgroup, so that
    # stores of one group and prefetches of the next are in flight together
    _announce(f"backward in place dx={alias} d={d} {dtype} N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=d + N)
    x, dy = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a = torch.from_numpy(inp.alpha).cuda()
    target = x if alias == "x" else dy
    dx, da, db = wht.wht_affine_backward(dy, x, a, dx=target)
    torch.cuda.synchronize()
    assert dx.data_ptr() == target.data_ptr()
    rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, _method(d))
    assert_io_close(dx, rdx, dtype, f"in place dx={alias} d={d}")
    assert_grad_close(da, rda, f"in place dx={alias} d={d} dalpha")
    assert_grad_close(db, rdb, f"in place dx={alias} d={d} dbeta")


@pytest.mark.parametrize("N", [4099])
def test_float32_many_tokens_at_the_widest_row(N):
    # float32 I/O at d = 8192 with more token groups than workgroups and a ragged tail
    _announce(f"float32 d=8192 N={N}")
    inp = synth.make_inputs(N, 8192, "f32", seed=3)
    check_forward_full(inp, "f32 d=8192 fwd")
    check_backward_full(inp, "f32 d=8192 bwd")


@pytest.mark.parametrize("d,N", [(4096, 1), (4096, 2), (4096, 3), (4096, 511), (4096, 513), (4096, 1031), (8192, 255),
                                 (8192, 256), (8192, 257), (8192, 600), (3072, 515), (6144, 259)])
def test_backward_teams_kernel_token_counts(d, N):
    # the three-team backward kernel (one LDS exchange per transform: d = 4096, 8192, 3072, 6144): fewer
    # token groups than workgroups, exactly as many, one more, ragged last groups
    _announce(f"backward (teams) d={d} N={N}")
    check_backward_full(synth.make_inputs(N, d, "bf16", seed=7 * d + N), f"teams bwd d={d} N={N}")


@pytest.mark.parametrize("d,N", [(4096, 16), (8192, 70), (1536, 33), (256, 40)])
def test_hip_graph_replays_match_eager(d, N):
    """Forward, fused-residual forward and backward captured once into a HIP graph and replayed with
    new inputs each time (the buffers are rewritten in place between replays, with the program's own
    eager work and synchronisations in between): every replay must equal the eager result bit for
    bit, and the first replay's result must equal the oracle's."""
    _announce(f"graph replay d={d} N={N}")
    a = torch.from_numpy(synth.make_inputs(1, d, "bf16", seed=1).alpha).cuda()
    b = torch.from_numpy(synth.make_inputs(1, d, "bf16", seed=1).beta).cuda()
    x = torch.empty(N, d, device="cuda", dtype=torch.bfloat16)
    dy, resid = torch.empty_like(x), torch.empty_like(x)
    y, yr, dx = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    yr2, ss = torch.empty_like(x), torch.empty(N, device="cuda")
    da, db = torch.empty(d, device="cuda"), torch.empty(d, device="cuda")
    ws = torch.empty(max(16, wht.wht_affine_backward_workspace_bytes(N, d, wht.DTYPE_BF16)),
                     dtype=torch.uint8, device="cuda")

    def step():
        wht.wht_affine_forward(x, a, b, y=y)
        wht.wht_affine_forward_residual(x, a, b, resid, y=yr)
        wht.wht_affine_forward_residual_stats(x, a, b, resid, y=yr2, sumsq=ss)
        wht.wht_affine_backward(dy, x, a, dx=dx, dalpha=da, dbeta=db, workspace=ws)

    def load(seed):
        inp = synth.make_inputs(N, d, "bf16", seed=seed)
        x.copy_(to_gpu(inp.x, "bf16"))
        dy.copy_(to_gpu(inp.dy, "bf16"))
        resid.copy_(to_gpu(synth.make_inputs(N, d, "bf16", seed=seed + 100).x, "bf16"))
        return inp

    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                        # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay, seed in enumerate((21, 22, 23, 24)):
        inp = load(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, yr, dx, da, db, yr2, ss)]
        for t in (y, yr, dx, da, db, yr2, ss):
            t.zero_()
        step()                                        # eager, same buffers
        torch.cuda.synchronize()
        for name, g, e in zip(("y", "y+resid", "dx", "dalpha", "dbeta", "y+resid (stats call)", "sumsq"), got,
                              (y, yr, dx, da, db, yr2, ss)):
            view = torch.int16 if g.dtype == torch.bfloat16 else torch.int32
            assert torch.equal(g.view(view), e.view(view)), f"replay {replay}: {name} differs from eager"
        if replay == 0:
            assert_io_close(got[0], oracle.forward(inp.x, inp.alpha * 0 + a.cpu().numpy(), b.cpu().numpy(), "fast"),
                            "bf16", "graph y")
            rdx, rda, rdb = oracle.backward(inp.dy, inp.x, a.cpu().numpy(), "fast")
            assert_io_close(got[2], rdx, "bf16", "graph dx")
            assert_grad_close(got[3], rda, "graph dalpha")
            assert_grad_close(got[4], rdb, "graph dbeta")


@pytest.mark.parametrize("d,dtype", [(1024, "bf16"), (768, "bf16"), (256, "f32")])
def test_autograd_module_matches_oracle(d, dtype):
    """The autograd wrapper only routes tensors: a [B, S, d] activation through the Module, a loss
    whose gradient with respect to y is a given dy, and .backward() must reproduce the oracle's
    y, dx, dalpha, dbeta (and pass dy through to the residual stream)."""
    from paper_2603_08343_amd.autograd import WhtAffine
    B, S = 3, 11
    inp = synth.make_inputs(B * S, d, dtype, seed=31)
    _announce(f"autograd d={d} {dtype}")
    layer = WhtAffine(d, device="cuda")
    with torch.no_grad():
        layer.alpha.copy_(torch.from_numpy(inp.alpha))
        layer.beta.copy_(torch.from_numpy(inp.beta))
    x = to_gpu(inp.x, dtype).view(B, S, d).requires_grad_(True)
    resid = to_gpu(synth.make_inputs(B * S, d, dtype, seed=32).x, dtype).view(B, S, d).requires_grad_(True)
    dy = to_gpu(inp.dy, dtype).view(B, S, d)
    y = layer(x, resid)
    assert y.shape == (B, S, d) and y.dtype == x.dtype
    y.backward(dy)
    torch.cuda.synchronize()
    rin = synth.make_inputs(B * S, d, dtype, seed=32).x
    assert_io_close(y.detach().view(B * S, d), oracle.forward_residual(inp.x, inp.alpha, inp.beta, rin, _method(d)),
                    dtype, "module y")
    rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, _method(d))
    assert_io_close(x.grad.view(B * S, d), rdx, dtype, "module dx")
    assert_grad_close(layer.alpha.grad, rda, "module dalpha")
    assert_grad_close(layer.beta.grad, rdb, "module dbeta")
    view = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(resid.grad.view(view), dy.view(view))
    # without the residual stream
    x2 = to_gpu(inp.x, dtype).view(B, S, d)
    assert_io_close(layer(x2).detach().view(B * S, d), oracle.forward(inp.x, inp.alpha, inp.beta, _method(d)),
                    dtype, "module y (no residual)")


@pytest.mark.parametrize("d,dtype,N", [(64, "f32", 70), (512, "bf16", 131), (1024, "bf16", 263), (4096, "bf16", 35),
                                       (8192, "bf16", 129), (768, "bf16", 67), (6144, "bf16", 9), (8192, "f32", 9)])
def test_backward_with_outputs_left_out(d, dtype, N):
    """dx alone (frozen parameters) and the parameter gradients alone: the values must be those of
    the full call, bit for bit, and hence the oracle's."""
    _announce(f"backward, optional outputs d={d} {dtype} N={N}")
    inp = synth.make_inputs(N, d, dtype, seed=d + 3)
    x, dy = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a = torch.from_numpy(inp.alpha).cuda()
    dx, da, db = wht.wht_affine_backward(dy, x, a)
    dx_only, none_a, none_b = wht.wht_affine_backward(dy, None, a, want_param_grads=False)
    none_x, da_only, db_only = wht.wht_affine_backward(dy, x, a, want_dx=False)
    torch.cuda.synchronize()
    assert none_a is None and none_b is None and none_x is None
    view = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(dx_only.view(view), dx.view(view))
    assert torch.equal(da_only, da) and torch.equal(db_only, db)
    rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, _method(d))
    assert_io_close(dx_only, rdx, dtype, "dx alone")
    assert_grad_close(da_only, rda, "dalpha alone")
    assert_grad_close(db_only, rdb, "dbeta alone")
    with pytest.raises(ValueError):
        wht.wht_affine_backward(dy, x, a, want_dx=False, want_param_grads=False)


def test_autograd_frozen_parameters_take_the_dx_only_path():
    from paper_2603_08343_amd.autograd import WhtAffine
    d, N = 2048, 40
    inp = synth.make_inputs(N, d, "bf16", seed=41)
    layer = WhtAffine(d, device="cuda")
    with torch.no_grad():
        layer.alpha.copy_(torch.from_numpy(inp.alpha))
    layer.alpha.requires_grad_(False)
    layer.beta.requires_grad_(False)
    x = to_gpu(inp.x, "bf16").requires_grad_(True)
    layer(x).backward(to_gpu(inp.dy, "bf16"))
    torch.cuda.synchronize()
    assert layer.alpha.grad is None and layer.beta.grad is None
    rdx, _, _ = oracle.backward(inp.dy, inp.x, inp.alpha, "fast", want_param_grads=False)
    assert_io_close(x.grad, rdx, "bf16", "frozen-parameter dx")


def test_backward_is_bit_reproducible():
    inp = synth.make_inputs(4099, 1024, "bf16", seed=13)
    first = run_backward(inp)
    second = run_backward(inp)
    assert torch.equal(first[1], second[1]) and torch.equal(first[2], second[2])
    assert torch.equal(first[0].view(torch.int16), second[0].view(torch.int16))


def test_zero_tokens():
    d = 512
    a = torch.ones(d, device="cuda")
    x = torch.empty(0, d, device="cuda", dtype=torch.bfloat16)
    y = wht.wht_affine_forward(x, a, a)
    assert y.shape == (0, d)
    da = torch.full((d,), 7.0, device="cuda")
    db = torch.full((d,), 7.0, device="cuda")
    wht.wht_affine_backward(x, x, a, dalpha=da, dbeta=db)
    torch.cuda.synchronize()
    assert float(da.abs().max()) == 0.0 and float(db.abs().max()) == 0.0


def test_non_default_stream():
    inp = synth.make_inputs(300, 4096, "bf16", seed=17, backward=False)
    x = to_gpu(inp.x, "bf16")
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        y = wht.wht_affine_forward(x, a, b)
    s.synchronize()
    ref = oracle.forward(inp.x, inp.alpha, inp.beta, "fast")
    assert_io_close(y, ref, "bf16", "side stream")


def test_boundary_errors_on_gpu():
    d, N = 256, 4
    x = torch.zeros(N, d, device="cuda")
    a = torch.ones(d, device="cuda")
    ws = torch.empty(64, dtype=torch.uint8, device="cuda")
    before_da = torch.full((d,), 3.0, device="cuda")
    rc = binding.wht_affine_backward_raw(x.data_ptr(), x.data_ptr(), a.data_ptr(), x.data_ptr(),
                                         before_da.data_ptr(), before_da.data_ptr(), N, d, 0,
                                         ws.data_ptr(), 64)
    assert rc == 5                                                # WHT_ERR_WORKSPACE, nothing enqueued
    torch.cuda.synchronize()
    assert float(before_da.min()) == 3.0
    assert binding.wht_affine_forward_raw(x.data_ptr() + 4, a.data_ptr(), a.data_ptr(), x.data_ptr(), N, d, 0) == 4
    with pytest.raises(wht.WhtAffineError):
        wht.wht_affine_forward(torch.zeros(2, 96, device="cuda"), torch.ones(96, device="cuda"),
                               torch.ones(96, device="cuda"))


def test_bench_copy_kernel_copies():
    # the bench-only copy kernel (not part of the layer's ABI): the ceiling the benchmark quotes and
    # the profiler's byte-counter reference must at least be a correct copy
    import bench
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, ((1 << 20) + 4,), dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    bench.bench_copy(torch, src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_bench_stream_events_time_a_known_interval():
    # the benchmark's events (bench-only library, no system-scope fence) against torch's on the same
    # stream, around the same 64 MiB copy: the two clocks must agree to a few microseconds
    import bench
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (16 << 20,), dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    for _ in range(3):
        bench.bench_copy(torch, src, dst)
    a, b = bench.StreamEvent(torch), bench.StreamEvent(torch)
    ta, tb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ta.record()
    a.record()
    for _ in range(10):
        bench.bench_copy(torch, src, dst)
    b.record()
    tb.record()
    torch.cuda.synchronize()
    ours, theirs = a.elapsed_time(b), ta.elapsed_time(tb)
    assert 0.0 < ours <= theirs + 0.002
    assert theirs - ours < 0.05
