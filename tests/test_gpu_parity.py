"""GPU parity: the HIP path (through the C ABI) against the CPU checker, element
by element, on the same seeded inputs.

Bars.  Integer work (predictor codes, masks, lists, counts): bit-exact.
Floating point: relative L2 error of y <= 1e-2 for bf16 storage (fp32
accumulation) and <= 1e-4 for fp32 storage; the folded matrix and the fitted
lines have their own bounds stated at each test.
"""
import numpy as np
import pytest
import torch

from oracle import tardis_oracle as O
from paper_2501_10054_amd import synth
from paper_2501_10054_amd import tardis as T

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
Y_TOL = {"f32": 1e-4, "bf16": 1e-2}


def dev(x, dtype):
    """numpy float32 array (values representable in `dtype`) -> device tensor."""
    if x is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).to(DEV).contiguous()


def host(t):
    return t.detach().to("cpu").to(torch.float32).numpy().astype(np.float64)


def rel_l2(got, want):
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def assert_y_close(got, want, F, X, flags, dtype="bf16"):
    """y against the checker: relative L2 over all tokens, per token, and ELEMENT BY ELEMENT.

    Element bound for bf16 storage (fp32 accumulation); bf16 keeps 8 significant bits, so rounding
    to it moves a value by at most 2^-8 of itself (half a unit in the last place at the bottom of a
    binade).  (1) The library's W' is the checker's rounded once to bf16, |eps_ik| <= 2^-8 |W'_ik|
    and, as a rounding error, uniform within its half unit: the folded product of token x is off by
    a sum of independent terms of standard deviation at most 2^-8/sqrt(3) * r_i,
    r_i = sqrt(sum_k (W'_ik x_k)^2).  (2) The paths that carry the repair factors delta_j as bf16
    (passes of 17-64 tokens, prompts) add the same kind of sum over the token's flagged neurons,
    q_i = sqrt(sum_j (delta_j W2_ij)^2).  Six standard deviations of (1) + (2) are allowed.
    (3) The bf16 output adds at most 2^-8 |y_i| (1.5 x 2^-8 of the checker's value allowed).
    Everything else (fp32 sums, erf) is orders below.  One wrong element - off by its own size -
    fails this, where a norm over the token would let it pass.
    fp32 storage: 1e-4 of |y_i| + r_i + q_i (sums of d and h fp32 terms)."""
    got = np.atleast_2d(np.asarray(got, np.float64))
    want = np.atleast_2d(np.asarray(want, np.float64))
    X = np.atleast_2d(np.asarray(X, np.float64))
    flags = np.atleast_2d(np.asarray(flags, bool))
    assert got.shape == want.shape and X.shape[0] == want.shape[0] == flags.shape[0]
    assert np.isfinite(got).all()
    err = rel_l2(got, want)
    assert err <= Y_TOL[dtype], err
    per_tok = np.linalg.norm(got - want, axis=1) / np.maximum(np.linalg.norm(want, axis=1), 1e-30)
    assert per_tok.max() <= 3 * Y_TOL[dtype], per_tok.max()
    r2 = (X * X) @ (F.Wp ** 2).T
    for t in range(X.shape[0]):
        idx, delta = O.fix_terms(F, X[t], flags[t])
        r2[t] += (F.W2[:, idx] ** 2) @ (delta ** 2)
    r = np.sqrt(r2)
    floor = 1e-6 * np.abs(want).max()
    if dtype == "bf16":
        tol = 1.5 * 2.0 ** -8 * np.abs(want) + 6.0 * (2.0 ** -8 / np.sqrt(3.0)) * r + floor
    else:
        tol = 1e-4 * (np.abs(want) + r) + floor
    bad = np.abs(got - want) > tol
    assert not bad.any(), (int(bad.sum()), float((np.abs(got - want) / tol).max()))
    return err


def make_ffn(layer, act="gelu_erf"):
    return T.FFN(dev(layer.W1, layer.dtype), dev(layer.W2, layer.dtype), dev(layer.b1, layer.dtype),
                 dev(layer.b2, layer.dtype), act)


def unpack_mask(mask_t, h):
    w = mask_t.cpu().numpy().view(np.uint32)
    bits = (w[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1
    return bits.reshape(w.shape[0], -1)[:, :h].astype(bool)


def custom_layer(d, h, dtype, seed, w1_std, bias):
    return synth.make_layer(d, h, dtype, seed, w1_std=w1_std, w2_std=0.05, heavy_frac=0.02, with_bias=bias)


def run_case(layer, X_cal, X_test, coverage, act="gelu_erf", batched=False, check_calibrate=True, sketch_bits=8,
             max_batch=None):
    """Full pipeline on the GPU and in the checker; returns a dict of diagnostics."""
    dt = layer.dtype
    ffn = make_ffn(layer, act)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, dt), coverage)
    torch.cuda.synchronize()
    lo_h, hi_h, a_h, c_h = (t.cpu().numpy() for t in (lo, hi, a, c))

    if check_calibrate:
        olo, ohi, oa, oc = O.calibrate(layer.W1, layer.b1, X_cal, coverage, act)
        scale = max(1e-6, float(np.abs(np.concatenate([olo, ohi])).max()))
        assert np.abs(lo_h - olo).max() <= 2e-5 * scale
        assert np.abs(hi_h - ohi).max() <= 2e-5 * scale
        # a sample sitting within rounding distance of a range end may be in on one side and out
        # on the other; that moves the fit by O(1/n)
        n_cal = X_cal.shape[0]
        assert np.abs(a_h - oa).max() <= 5.0 / n_cal + 1e-4
        assert np.abs(c_h - oc).max() <= (5.0 / n_cal + 1e-4) * max(1.0, scale)

    # from here on both sides use the SAME (lo, hi, a, c): the library's
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=max_batch or max(1, X_test.shape[0]), sketch_bits=sketch_bits)
    F = O.build(layer.W1, layer.b1, layer.W2, layer.b2, lo_h, hi_h, a_h, c_h, act, sketch_bits=sketch_bits)

    Wp, bp = T.tardis_get_folded(L)
    Q, tlo, thi = T.tardis_get_predictor_state(L)
    torch.cuda.synchronize()
    wp_err = rel_l2(host(Wp), F.Wp)
    assert wp_err <= (3e-3 if dt == "bf16" else 1e-5), wp_err     # bf16: one rounding of W' (2^-9)
    assert rel_l2(host(bp), F.bp) <= 1e-5 or np.abs(host(bp) - F.bp).max() <= 1e-6
    np.testing.assert_array_equal(Q.cpu().numpy(), F.sk.Q)
    np.testing.assert_array_equal(tlo.cpu().numpy(), F.sk.tlo)
    np.testing.assert_array_equal(thi.cpu().numpy(), F.sk.thi)
    if sketch_bits == 4:
        np.testing.assert_array_equal(T.tardis_get_sketch_groups(L).cpu().numpy(), F.sk.m)

    n = X_test.shape[0]
    Xd = dev(X_test, dt)
    Yo, FLo = O.forward(F, X_test)
    if batched:
        Y = T.tardis_ffn_forward_batched(L, Xd)
        mask, counts, lst = T.tardis_get_last_outliers(L, n)
        ucnt, umask = T.tardis_get_last_union(L, n, want_mask=True)
        torch.cuda.synchronize()
        # the union of the call's flag sets, computed on the device: what the batch must fetch
        assert int(ucnt.item()) == int(FLo.any(axis=0).sum())
        np.testing.assert_array_equal(umask.cpu().numpy().view(np.uint32), O.pack_mask(FLo.any(axis=0)[None])[0])
        Yg = host(Y)
        FLg = unpack_mask(mask, layer.h)
        counts = counts.cpu().numpy()
        lst = lst.cpu().numpy()
        lists = [lst[t, :counts[t]] for t in range(n)]
    else:
        Yg = np.empty((n, layer.d))
        FLg = np.empty((n, layer.h), bool)
        counts = np.empty(n, np.int64)
        lists = []
        for t in range(n):
            y = T.tardis_ffn_forward(L, Xd[t])
            mask, cnt, lst = T.tardis_get_last_outliers(L, 1)
            torch.cuda.synchronize()
            Yg[t] = host(y)
            FLg[t] = unpack_mask(mask, layer.h)[0]
            counts[t] = int(cnt.item())
            lists.append(lst.cpu().numpy()[0, :counts[t]])

    np.testing.assert_array_equal(FLg, FLo)                         # mask: bit-exact
    for t in range(n):
        assert counts[t] == FLo[t].sum()
        np.testing.assert_array_equal(np.sort(lists[t]), np.flatnonzero(FLo[t]))   # list: same set
    err = assert_y_close(Yg, Yo, F, X_test, FLo, dt)               # norms and element by element

    # dense baseline against the checker's dense FFN
    Yd = host(T.tardis_dense_forward(L, Xd))
    derr = rel_l2(Yd, O.dense(layer.W1, layer.b1, layer.W2, layer.b2, X_test, act))
    assert derr <= Y_TOL[dt], derr
    L.close()
    return dict(y_err=err, wp_err=wp_err, dense_err=derr, rate=float(FLo.mean()))


# ------------------------------------------------------------------ config 0
def test_tiny_fp32_batch1():
    w = synth.tiny()
    r = run_case(w.layer, w.X_cal, w.X_test, w.coverage)
    assert 0.03 < r["rate"] < 0.2


def test_tiny_hard_fp32_with_bias():
    w = synth.tiny(hard=True, with_bias=True)
    r = run_case(w.layer, w.X_cal, w.X_test, w.coverage)
    assert 0.03 < r["rate"] < 0.2


@pytest.mark.parametrize("act", ["gelu_tanh", "relu", "identity"])
def test_tiny_other_activations(act):
    w = synth.tiny(hard=True, with_bias=True)
    run_case(w.layer, w.X_cal, w.X_test[:8], 0.8, act=act)


def test_tiny_batched_call():
    w = synth.tiny(hard=True)
    run_case(w.layer, w.X_cal, w.X_test, 0.85, batched=True)


# ------------------------------------------------- ragged and several-tile shapes
@pytest.mark.parametrize("d,h,dtype", [(72, 200, "f32"), (50, 77, "f32"), (200, 1000, "bf16"),
                                       (136, 330, "bf16"), (70, 99, "bf16")])
def test_ragged_shapes(d, h, dtype):
    seed = synth.workload_seed(9, d)
    layer = custom_layer(d, h, dtype, seed, w1_std=0.15, bias=True)
    X_cal = synth.make_tokens(300, d, dtype, seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(6, d, dtype, seed, synth.STREAM_TEST)
    run_case(layer, X_cal, X_test, 0.9)


def test_mid_bf16_heavy_tail():
    w = synth.decode(d=512, h=2048, n_cal=1024, n_test=16, coverage=0.95)
    r = run_case(w.layer, w.X_cal, w.X_test, w.coverage)
    assert 0.02 < r["rate"] < 0.12


def test_mid_bf16_batched_high_fallback():
    w = synth.decode(d=512, h=2048, n_cal=512, n_test=12, coverage=0.85)
    r = run_case(w.layer, w.X_cal, w.X_test, w.coverage, batched=True)
    assert 0.08 < r["rate"] < 0.25


@pytest.mark.parametrize("n,coverage", [(2, 0.95), (3, 0.95), (4, 0.9), (7, 0.85), (5, 0.9), (6, 0.95), (8, 0.95), (9, 0.95), (11, 0.9), (15, 0.95), (16, 0.9), (17, 0.9),
                                        (20, 0.95), (48, 0.85), (64, 0.95), (70, 0.99), (150, 0.95)])
def test_batched_passes_of_64_tokens(n, coverage):
    """Up to 16 tokens: groups of 16, 8, 4 (two kernels: records, then the column-sliced down
    projection; 3, 5-7 and 9-15 tokens run as partly empty groups), 2 and 1 tokens (one kernel).
    17 to 64: one weight stream per pass, every tile count (1, 2, 4 token tiles), the masked-dense
    scatter.  70 and 150: the prompt path at a fraction of one tile row."""
    w = synth.decode(d=1024, h=4096, n_cal=512, n_test=n, coverage=coverage, config=2)
    run_case(w.layer, w.X_cal, w.X_test, coverage, batched=True, check_calibrate=False)


def test_batched_with_bias_and_relu():
    seed = synth.workload_seed(2, 7)
    layer = synth.make_layer(512, 2048, "bf16", seed, w1_std=0.05, w2_std=0.05, heavy_frac=0.01, with_bias=True)
    X_cal = synth.make_tokens(400, 512, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(33, 512, "bf16", seed, synth.STREAM_TEST)
    run_case(layer, X_cal, X_test, 0.9, act="relu", batched=True, check_calibrate=False)


# ------------------------------------------------------------- prompt path (dense matrix products)
@pytest.mark.parametrize("d,h,n,bits", [(1024, 4096, 256, 8), (1024, 4096, 333, 8), (512, 2048, 300, 4),
                                        (1024, 4096, 700, 4), (384, 1152, 200, 8), (384, 1160, 66, 8),
                                        (640, 1992, 129, 8)])
def test_prompt_path_many_tokens(d, h, n, bits):
    """65 tokens and more: integer predictor sums, pre-activations, folded product and the masked
    delta's down projection as four matrix products (ragged token counts span a partial tile);
    masks bit-exact, lists and counts as for every other path.  d = 384 and 640: odd numbers of K
    slices (3 and 5 of int8, 9 per range of the down projection); h = 1160, 1992: a ragged last
    tile column and a K of the down projection that is no multiple of the slice."""
    w = synth.decode(d=d, h=h, n_cal=512, n_test=n, coverage=0.9, config=3)
    run_case(w.layer, w.X_cal, w.X_test, 0.9, batched=True, check_calibrate=False, sketch_bits=bits)


def test_prompt_path_with_bias_and_relu():
    seed = synth.workload_seed(3, 11)
    layer = synth.make_layer(512, 2048, "bf16", seed, w1_std=0.05, w2_std=0.05, heavy_frac=0.01, with_bias=True)
    X_cal = synth.make_tokens(400, 512, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(257, 512, "bf16", seed, synth.STREAM_TEST)
    run_case(layer, X_cal, X_test, 0.9, act="relu", batched=True, check_calibrate=False)


def test_prompt_path_in_chunks(monkeypatch):
    """A prompt longer than the scratch is sized for runs in chunks (here 3 of 256 tokens, the last
    one ragged); masks and outputs land at their tokens' rows."""
    monkeypatch.setenv("TARDIS_PREFILL_CHUNK", "256")
    w = synth.decode(d=1024, h=4096, n_cal=512, n_test=700, coverage=0.9, config=3)
    run_case(w.layer, w.X_cal, w.X_test, 0.9, batched=True, check_calibrate=False)


def test_prompt_threshold_off_takes_token_passes(monkeypatch):
    """With the prompt path's threshold out of reach the same 300 tokens run as passes of 64 (four
    full passes and a ragged last one)."""
    monkeypatch.setenv("TARDIS_PREFILL_MIN", "1000000")
    w = synth.decode(d=1024, h=4096, n_cal=512, n_test=300, coverage=0.9, config=3)
    run_case(w.layer, w.X_cal, w.X_test, 0.9, batched=True, check_calibrate=False)


# ------------------------------------------------------------- greedy range search
TIE_REL = 1e-3      # two candidates' errors closer than this (relative) ...
TIE_GAP = 2e-5      # ... or a sample this close (x the largest range end) to an end a step compares with


def assert_search_differences_are_near_ties(Z, tj, step, act, differing, scale):
    """Every neuron whose searched range differs from the checker's had a growth step that the
    rounding of the pre-activations (fp32 dot products here, fp64 there) can decide either way:
    two candidate errors within TIE_REL of each other, or a sample within TIE_GAP x scale of one
    of the range ends that step compares samples with."""
    for j in differing:
        tr = []
        O.range_search(Z[:, j], float(tj[j]), step, act, trace=tr)
        rel = [abs(el - er) / max(el, er, 1e-300) for _, el, er, _ in tr if el is not None]
        gap = [g for *_, g in tr]
        assert min(rel, default=1.0) <= TIE_REL or min(gap, default=1.0) <= TIE_GAP * scale, \
            (j, min(rel, default=None), min(gap, default=None))


@pytest.mark.parametrize("dtype,d,h,n_cal,t,step,act,per_neuron",
                         [("f32", 64, 96, 400, 0.9, 0.05, "gelu_erf", False),
                          ("bf16", 256, 64, 1000, 0.85, 0.1, "gelu_erf", False),
                          ("f32", 64, 48, 300, 0.8, 0.08, "relu", True),
                          ("bf16", 128, 72, 600, 0.8, 0.06, "gelu_erf", True),
                          ("f32", 48, 40, 257, 1.0, 0.25, "gelu_tanh", False)])
def test_calibrate_search_against_checker(dtype, d, h, n_cal, t, step, act, per_neuron):
    """The two sides see pre-activations that differ in the last bits (fp32 against fp64 dot
    products), and every growth step is a comparison of two error sums and of samples with range
    ends: a step decided by less than that noise may go the other way.  So: almost all neurons
    equal to rounding; every neuron that is not is SHOWN to have had such a step (the checker
    reports each step's margins), lies a whole number of steps away, and satisfies the search's
    invariants.  With per_neuron, every neuron has its own target portion (coverage_per_neuron)."""
    t, step = float(np.float32(t)), float(np.float32(step))
    seed = synth.workload_seed(9, 21)
    layer = synth.make_layer(d, h, dtype, seed, w1_std=0.2 if d < 128 else 0.1, w2_std=0.05, heavy_frac=0.02,
                             with_bias=True)
    X_cal = synth.make_tokens(n_cal, d, dtype, seed, synth.STREAM_CAL)
    ffn = make_ffn(layer, act)
    if per_neuron:      # 0.7, 0.8, 0.9 of t's neighbourhood in turn (all exactly representable steps apart in fp32)
        tj32 = (np.float32(t) + np.float32(0.1) * (np.arange(h) % 3 - 1).astype(np.float32)).astype(np.float32)
        tj = tj32.astype(np.float64)
        got = T.tardis_calibrate_search(ffn, dev(X_cal, dtype), t, step,
                                        coverage_per_neuron=torch.from_numpy(tj32).to(DEV))
    else:
        tj = np.full(h, t)
        got = T.tardis_calibrate_search(ffn, dev(X_cal, dtype), t, step)
    lo, hi, a, c = (v.cpu().numpy() for v in got)
    olo, ohi, oa, oc = O.calibrate_search(layer.W1, layer.b1, X_cal, tj, step, act)
    scale = float(np.abs(np.concatenate([olo, ohi])).max())
    same = (np.abs(lo - olo) <= 1e-4 * scale) & (np.abs(hi - ohi) <= 1e-4 * scale)
    assert same.mean() >= 0.95, same.mean()
    assert np.abs(a - oa)[same].max() <= 5.0 / n_cal + 1e-4
    assert np.abs(c - oc)[same].max() <= (5.0 / n_cal + 1e-4) * max(1.0, scale)
    Z = O.preact(layer.W1, layer.b1, X_cal)
    assert_search_differences_are_near_ties(Z, tj, step, act, np.flatnonzero(~same), scale)
    for j in range(h):
        inside = (Z[:, j] >= np.float64(lo[j])) & (Z[:, j] < np.float64(hi[j]))
        assert inside.mean() >= tj[j] - 2.0 / n_cal               # reached the target (up to samples on the edge)
        # the range is the centroid grown by whole steps on either side
        cen = O.kde_centroid(np.sort(Z[:, j]))
        kl, kr = (cen - lo[j]) / step, (hi[j] - cen) / step
        if inside.mean() < 1.0:
            assert abs(kl - round(kl)) < 2e-2 and abs(kr - round(kr)) < 2e-2
        if not same[j]:                                           # a different but valid sequence of steps
            assert abs((lo[j] - olo[j]) / step - round((lo[j] - olo[j]) / step)) < 2e-2
        # and its line is the least-squares line of its own samples
        aj, cj = O.fit_line(Z[inside, j], O.act(Z[inside, j], act), float(lo[j]), act)
        assert abs(a[j] - aj) <= 5.0 / n_cal + 1e-4 and abs(c[j] - cj) <= (5.0 / n_cal + 1e-4) * max(1.0, scale)
    if per_neuron:      # the three groups of neurons really got three different portions
        cov = np.array([((Z[:, j] >= np.float64(lo[j])) & (Z[:, j] < np.float64(hi[j]))).mean() for j in range(h)])
        assert cov[0::3].mean() < cov[1::3].mean() < cov[2::3].mean()


def test_calibrate_search_refuses_a_step_that_needs_too_many_steps():
    """Algorithm 1 has no limit on the number of growth steps; the kernel guards one block's run time
    with 4096 and fails the whole call rather than substitute a range."""
    w = synth.tiny(hard=True)
    ffn = make_ffn(w.layer)
    with pytest.raises(T.TardisError) as e:
        T.tardis_calibrate_search(ffn, dev(w.X_cal, "f32"), 0.99, 1e-5)
    assert e.value.status == T.ERR_INVALID_ARG
    lo, hi, a, c = T.tardis_calibrate_search(ffn, dev(w.X_cal, "f32"), 0.9, 0.05)       # and works afterwards
    assert torch.isfinite(lo).all() and (hi > lo).all()


@pytest.mark.parametrize("dtype,d,h,n_cal,act", [("f32", 64, 96, 400, "gelu_erf"), ("bf16", 256, 200, 700, "gelu_tanh"),
                                                 ("bf16", 1024, 512, 512, "relu")])
def test_estimate_errors_against_checker(dtype, d, h, n_cal, act):
    """E_n = sum over the calibration inputs of the section's error metric.  The two sides' pre-
    activations differ in the last bits, so a sample within rounding distance of a range end may be
    inside on one side and outside on the other: the library's value has to lie between the checker's
    sums without and with such samples."""
    seed = synth.workload_seed(9, 31)
    layer = synth.make_layer(d, h, dtype, seed, w1_std=0.2 if d < 128 else 0.06, w2_std=0.05, heavy_frac=0.02, with_bias=True)
    X_cal = synth.make_tokens(n_cal, d, dtype, seed, synth.STREAM_CAL)
    ffn = make_ffn(layer, act)
    Xd = dev(X_cal, dtype)
    lo, hi, a, c = T.tardis_calibrate(ffn, Xd, 0.9)
    err, tot = T.tardis_estimate_errors(ffn, Xd, lo, hi, a, c)
    torch.cuda.synchronize()
    lo_h, hi_h, a_h, c_h = (v.cpu().numpy() for v in (lo, hi, a, c))
    E = O.neuron_errors(layer.W1, layer.b1, layer.W2, X_cal, lo_h, hi_h, a_h, c_h, act)
    Z = O.preact(layer.W1, layer.b1, X_cal)
    scale = float(np.abs(np.concatenate([lo_h, hi_h])).max())
    eps = 2e-5 * scale
    lo64, hi64 = lo_h.astype(np.float64), hi_h.astype(np.float64)
    resid = np.abs(O.act(Z, act) - (Z * a_h.astype(np.float64) + c_h.astype(np.float64)))
    cn = np.sqrt((layer.W2.astype(np.float64) ** 2).sum(axis=0))
    sure = (Z >= lo64 + eps) & (Z < hi64 - eps)
    maybe = (Z >= lo64 - eps) & (Z < hi64 + eps)
    E_lo, E_hi = (resid * sure).sum(0) * cn, (resid * maybe).sum(0) * cn
    got = err.cpu().numpy().astype(np.float64)
    slack = 1e-4 * E + 1e-7 * E.max()
    assert (got >= E_lo - slack).all() and (got <= E_hi + slack).all()
    assert (E_lo <= E).all() and (E <= E_hi).all() and np.median((E_hi - E_lo) / np.maximum(E, 1e-30)) < 1e-3
    assert float(tot.item()) == pytest.approx(got.sum(), rel=1e-5)            # the layer's error: the sum over its neurons
    assert (got > 0).mean() > 0.9 or act == "relu"


@pytest.mark.parametrize("n,t,t_min,t_max", [(1, 0.9, 0.8, 1.0), (5, 0.8, 0.6, 0.9), (257, 0.85, 0.7, 0.95),
                                             (16384, 0.95, 0.9, 1.0), (1000, 0.6, 0.0, 1.0), (64, 0.9, 0.9, 0.9),
                                             (300, 0.9, 0.5, 0.9), (300, 0.5, 0.5, 0.9)])
def test_assign_thresholds_against_checker(n, t, t_min, t_max):
    """The threshold programme on the device against the checker on the same errors: the same
    floats out, ties (a quarter of the items share their error with another) resolved by index."""
    rng = np.random.default_rng(n)
    E = rng.uniform(0.0, 3.0, n).astype(np.float32)
    E[rng.integers(0, n, n // 4)] = E[rng.integers(0, n, n // 4)]           # repeated values
    t, t_min, t_max = (float(np.float32(v)) for v in (t, t_min, t_max))
    got = T.tardis_assign_thresholds(torch.from_numpy(E).to(DEV), t, t_min, t_max).cpu().numpy()
    want = O.error_aware_threshold(E, t, t_min, t_max)
    np.testing.assert_array_equal(got, want)
    assert got.astype(np.float64).sum() == pytest.approx(t * n, rel=1e-5, abs=1e-4)
    assert got.min() >= np.float32(t_min) and got.max() <= np.float32(t_max)


def test_adaptive_thresholds_feed_the_range_search():
    """Algorithm 1's outer loop for one layer, as its listing orders it: ranges at the layer's
    threshold, the neurons' errors on them, the error-aware thresholds, the search again with a
    threshold per neuron - then fold and run.  Neurons that err more get the smaller portion, the
    portions average to the layer's, and the programme's objective does not exceed the uniform one."""
    w = synth.decode(d=1024, h=768, n_cal=768, n_test=6, coverage=0.85)
    lay = w.layer
    ffn = make_ffn(lay)
    Xd = dev(w.X_cal, "bf16")
    t, step = float(np.float32(0.85)), float(np.float32(0.1))
    lo, hi, a, c = T.tardis_calibrate_search(ffn, Xd, t, step)
    err, tot0 = T.tardis_estimate_errors(ffn, Xd, lo, hi, a, c)
    tn = T.tardis_assign_thresholds(err, t, 0.7, 1.0)
    np.testing.assert_array_equal(tn.cpu().numpy(), O.error_aware_threshold(err.cpu().numpy(), t, float(np.float32(0.7)), 1.0))
    lo2, hi2, a2, c2 = T.tardis_calibrate_search(ffn, Xd, t, step, coverage_per_neuron=tn)
    _, tot1 = T.tardis_estimate_errors(ffn, Xd, lo2, hi2, a2, c2)
    torch.cuda.synchronize()
    e, tnh = err.cpu().numpy(), tn.cpu().numpy()
    assert tnh.astype(np.float64).mean() == pytest.approx(t, abs=1e-4)
    assert e[tnh == tnh.min()].min() >= e[tnh == tnh.max()].max()              # the worst neurons got the least
    Z = O.preact(lay.W1, None, w.X_cal)
    cov = ((Z >= lo2.cpu().numpy().astype(np.float64)) & (Z < hi2.cpu().numpy().astype(np.float64))).mean(0)
    assert (cov >= tnh - 2.0 / w.X_cal.shape[0]).all()                         # every neuron reached its own portion
    # the programme's objective is no worse than giving every neuron the layer's threshold
    assert float(e.astype(np.float64) @ tnh.astype(np.float64)) <= float(e.astype(np.float64).sum()) * t * (1 + 1e-6)
    assert np.isfinite(float(tot0.item())) and np.isfinite(float(tot1.item())) and float(tot1.item()) > 0
    L = T.tardis_fold(ffn, lo2, hi2, a2, c2, max_batch=6)
    F = O.build(lay.W1, None, lay.W2, None, *(v.cpu().numpy() for v in (lo2, hi2, a2, c2)))
    Yo, FLo = O.forward(F, w.X_test)
    Y = T.tardis_ffn_forward_batched(L, dev(w.X_test, "bf16"))
    mask, _, _ = T.tardis_get_last_outliers(L, 6, want_list=False)
    np.testing.assert_array_equal(unpack_mask(mask, lay.h), FLo)
    assert_y_close(host(Y), Yo, F, w.X_test, FLo)
    L.close()


def test_calibrate_search_feeds_the_online_path():
    # ranges from the search go through fold and forward like any others
    w = synth.decode(d=1024, h=512, n_cal=512, n_test=4, coverage=0.9)
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate_search(ffn, dev(w.X_cal, "bf16"), 0.9, 0.1)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=4)
    F = O.build(w.layer.W1, None, w.layer.W2, None, *(v.cpu().numpy() for v in (lo, hi, a, c)))
    Yo, FLo = O.forward(F, w.X_test)
    Y = T.tardis_ffn_forward_batched(L, dev(w.X_test, "bf16"))
    mask, _, _ = T.tardis_get_last_outliers(L, 4, want_list=False)
    np.testing.assert_array_equal(unpack_mask(mask, 512), FLo)
    assert_y_close(host(Y), Yo, F, w.X_test, FLo)
    assert 0.05 < FLo.mean() < 0.2
    L.close()


# ------------------------------------------------------------- 4-bit grouped sketch
def test_sketch4_tiny_fp32_and_ragged_groups():
    w = synth.tiny(hard=True, with_bias=True)                    # d = 64: two whole groups
    run_case(w.layer, w.X_cal, w.X_test, w.coverage, sketch_bits=4)
    seed = synth.workload_seed(9, 11)
    layer = synth.make_layer(50, 77, "f32", seed, w1_std=0.2, w2_std=0.05, heavy_frac=0.05)   # last group: 18 columns
    run_case(layer, synth.make_tokens(300, 50, "f32", seed, synth.STREAM_CAL),
             synth.make_tokens(6, 50, "f32", seed, synth.STREAM_TEST), 0.9, sketch_bits=4, batched=True)


@pytest.mark.parametrize("bits,margin", [(3, 0.0), (2, 0.0), (4, 0.1), (2, 0.2), (8, 0.15)])
def test_narrow_sketches_and_predictor_margin(bits, margin):
    """Codes of 3 and 2 bits (largest code 3 and 1) and the margin that narrows the range the
    predictor tests against: codes, multipliers, bounds and masks bit for bit, y to the bar, on a
    bf16 layer through the single-launch kernel, a group, a pass of tokens and the prompt path."""
    w = synth.decode(d=2048, h=1536, n_cal=512, n_test=70, coverage=0.9)
    lay = w.layer
    ffn = make_ffn(lay)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=70, sketch_bits=bits, margin=margin)
    F = O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)), sketch_bits=bits, margin=margin)
    Q, tlo, thi = T.tardis_get_predictor_state(L)
    np.testing.assert_array_equal(Q.cpu().numpy(), F.sk.Q)
    np.testing.assert_array_equal(tlo.cpu().numpy(), F.sk.tlo)
    np.testing.assert_array_equal(thi.cpu().numpy(), F.sk.thi)
    if bits < 8:
        np.testing.assert_array_equal(T.tardis_get_sketch_groups(L).cpu().numpy(), F.sk.m)
        assert int(np.abs(F.sk.q4).max()) == 2 ** (bits - 1) - 1
    Yo, FLo = O.forward(F, w.X_test)
    Xd = dev(w.X_test, "bf16")
    for n in (1, 6, 40, 70):
        Y = T.tardis_ffn_forward_batched(L, Xd[:n].contiguous())
        mask, _, _ = T.tardis_get_last_outliers(L, n, want_list=False)
        np.testing.assert_array_equal(unpack_mask(mask, lay.h), FLo[:n])
        assert_y_close(host(Y), Yo[:n], F, w.X_test[:n], FLo[:n])
    if margin > 0:      # the narrowed test flags a superset of what the plain one flags
        F0 = O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)), sketch_bits=bits)
        _, FL0 = O.forward(F0, w.X_test[:8])
        assert (FLo[:8] | FL0).sum() == FLo[:8].sum() and FLo[:8].sum() > FL0.sum()
    L.close()


@pytest.mark.parametrize("d,h", [(2048, 4096), (4096, 2048), (1024, 1000)])
def test_fp8_storage_of_the_folded_matrix(d, h):
    """folded_dtype = e4m3: the stored matrix is the checker's 8-bit rounding of W' (row scales
    powers of two, values on the format's grid, all but a sliver of the elements identical - the
    two sides' fp32 / fp64 sums differ in the last bits, which moves an element sitting on a rounding
    boundary by one step); with THAT matrix the online results meet the usual bars on every path;
    against the exact folded matrix y is a few percent off - the budget the header quotes."""
    w = synth.decode(d=d, h=h, n_cal=512, n_test=40, coverage=0.9)
    lay = w.layer
    ffn = make_ffn(lay)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    cal = tuple(t.cpu().numpy() for t in (lo, hi, a, c))
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=40, folded_fp8=True)
    Wp, bp = T.tardis_get_folded(L)
    got = host(Wp)
    F = O.build(lay.W1, None, lay.W2, None, *cal)
    vals, codes, e = O.fp8_rows(F.Wp)
    assert (got == vals).mean() > 0.99 and rel_l2(got, vals) < 1e-2
    # on the grid: each row is e4m3 numbers times one power of two
    mx = np.abs(got).max(axis=1)
    sc = 2.0 ** np.ceil(np.log2(np.maximum(mx, 1e-300) / 448.0))
    np.testing.assert_array_equal(O.round_e4m3(got / sc[:, None])[1] * sc[:, None], got)
    # the online paths with the library's own stored matrix
    F8 = O.build(lay.W1, None, lay.W2, None, *cal, wp_round=lambda W: got)
    Yo, FLo = O.forward(F8, w.X_test)
    Ye, _ = O.forward(F, w.X_test)
    Xd = dev(w.X_test, "bf16")
    for n in (1, 2, 5, 16, 40):
        Y = T.tardis_ffn_forward_batched(L, Xd[:n].contiguous())
        mask, _, _ = T.tardis_get_last_outliers(L, n, want_list=False)
        np.testing.assert_array_equal(unpack_mask(mask, lay.h), FLo[:n])
        assert_y_close(host(Y), Yo[:n], F8, w.X_test[:n], FLo[:n])
        assert rel_l2(host(Y), Yo[:n]) < 3e-3                    # same matrix on both sides: accumulation and output rounding only
    y1 = host(T.tardis_ffn_forward(L, Xd[0]))
    y5 = host(T.tardis_ffn_forward_batched(L, Xd[:5].contiguous()))[0]
    assert rel_l2(y1, y5) < 3e-3                                 # the 8-bit rows and the bf16 copy hold the same numbers
    budget = rel_l2(host(T.tardis_ffn_forward_batched(L, Xd)), Ye)
    assert 5e-3 < budget < 8e-2, budget                          # three mantissa bits: a few percent against the exact fold
    L.close()


@pytest.mark.parametrize("n", [1, 2, 6])
def test_stack_of_layers_with_fp8_folded_matrices(n):
    """Chained layers whose folded matrices are stored in 8 bits (the one- and two-token kernels apply
    the norm glue while streaming the 8-bit rows): each layer on the GPU's own hand-over against the
    checker holding the library's stored matrix."""
    d, h, nl = 2048, 2048, 3
    layers, oracles = [], []
    for li in range(nl):
        seed = synth.workload_seed(16, li)
        lay = synth.make_layer(d, h, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01)
        ffn = make_ffn(lay)
        X_cal = synth.make_tokens(384, d, "bf16", seed, synth.STREAM_CAL)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, "bf16"), 0.9)
        L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=n, folded_fp8=True)
        stored = host(T.tardis_get_folded(L)[0])
        layers.append(L)
        oracles.append(O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)),
                               wp_round=lambda W, stored=stored: stored))
    x0 = synth.make_tokens(n, d, "bf16", synth.workload_seed(16, 99), synth.STREAM_TEST)
    y = T.tardis_stack_forward(layers, dev(x0, "bf16"))
    torch.cuda.synchronize()
    x_in = x0.astype(np.float64)
    for li in range(nl):
        Yo, FLo = O.forward(oracles[li], x_in)
        mask, _, _ = T.tardis_get_last_outliers(layers[li], n, want_list=False)
        np.testing.assert_array_equal(unpack_mask(mask, h), FLo)
        if li < nl - 1:
            xn = host(T.tardis_get_handover(layers[li], n))
            assert rel_l2(xn, O.to_bf16(O.rmsnorm(Yo))) <= Y_TOL["bf16"]
            x_in = xn
        else:
            assert_y_close(host(y), Yo, oracles[li], x_in, FLo, "bf16")
    for L in layers:
        L.close()


def test_sketch4_zero_rows_and_zero_groups():
    seed = synth.workload_seed(9, 12)
    layer = custom_layer(96, 64, "f32", seed, w1_std=0.3, bias=True)
    layer.W1[5] = 0.0                                            # zero row, bias inside or outside its range
    layer.W1[6] = 0.0
    layer.b1[6] = 100.0
    layer.W1[7, 32:64] = 0.0                                     # a zero group in a live row
    layer.W1[8, :] = 0.0
    layer.W1[8, 70] = 0.25                                       # one non-zero weight in the whole row
    run_case(layer, synth.make_tokens(200, 96, "f32", seed, synth.STREAM_CAL),
             synth.make_tokens(5, 96, "f32", seed, synth.STREAM_TEST), 0.9, sketch_bits=4)


@pytest.mark.parametrize("d,h,n,batched", [(1024, 2048, 3, False), (2048, 1000, 3, False), (2048, 1000, 7, True),
                                           (2048, 4096, 20, True), (4096, 2048, 5, True)])
def test_sketch4_bf16_paths(d, h, n, batched):
    """d = 1024: the single-launch kernel on one-byte effective codes.  d = 2048, 4096: the packed
    4-bit rows (1, 2 and 4 tokens per launch); 20 tokens: the 64-token-pass path on effective codes."""
    seed = synth.workload_seed(9, 13)
    layer = synth.make_layer(d, h, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01, with_bias=True)
    X_cal = synth.make_tokens(256, d, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(n, d, "bf16", seed, synth.STREAM_TEST)
    run_case(layer, X_cal, X_test, 0.9, check_calibrate=False, batched=batched, sketch_bits=4)


@pytest.mark.parametrize("n", [3, 4, 8, 13, 16])
def test_sketch4_groups_on_one_byte_codes(n):
    """A 4-bit layer that also keeps one-byte effective codes (folded for more tokens than one
    decode call takes): groups of 4, 8 and 16 tokens read those (8 and 16 through the matrix-core
    predictor instead of running as two groups of half the size); same integers, same masks."""
    seed = synth.workload_seed(9, 21)
    d, h = 2048, 8192
    layer = synth.make_layer(d, h, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01, with_bias=True)
    X_cal = synth.make_tokens(256, d, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(n, d, "bf16", seed, synth.STREAM_TEST)
    run_case(layer, X_cal, X_test, 0.9, check_calibrate=False, batched=True, sketch_bits=4, max_batch=32)


# ----------------------------------------------------------------- edge cases
def test_degenerate_tokens_and_neurons():
    d, h = 64, 96
    seed = synth.workload_seed(9, 1)
    layer = custom_layer(d, h, "f32", seed, w1_std=0.3, bias=True)
    layer.W1[5] = 0.0                       # all-zero neuron: z = b1 for every token
    layer.W1[6] = 0.0
    layer.b1[6] = 100.0
    X_cal = synth.make_tokens(200, d, "f32", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(6, d, "f32", seed, synth.STREAM_TEST)
    X_test[0] = 0.0                         # zero token
    X_test[1] *= 1e-30                      # tiny token
    X_test[2] *= 1e20                       # huge token: everything out of range
    X_test[3, 1:] = 0.0                     # one-hot-like
    run_case(layer, X_cal, X_test, 0.9)


@pytest.mark.parametrize("n", [8, 40, 130])
def test_degenerate_tokens_on_the_bf16_paths(n):
    """Zero, tiny, huge and one-hot tokens and all-zero neurons through the fused decode kernels
    (8 tokens), a 64-token pass (40) and the prompt path (130)."""
    d, h = 1024, 2048
    seed = synth.workload_seed(9, 17)
    layer = synth.make_layer(d, h, "bf16", seed, w1_std=0.04, w2_std=0.03, heavy_frac=0.01, with_bias=True)
    layer.W1[5] = 0.0                       # all-zero neurons: z = b1 for every token
    layer.W1[700] = 0.0
    layer.b1[700] = 100.0
    X_cal = synth.make_tokens(300, d, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(n, d, "bf16", seed, synth.STREAM_TEST)
    X_test[0] = 0.0                         # zero token
    X_test[1] = (X_test[1].astype(np.float64) * 2.0 ** -100).astype(X_test.dtype)    # tiny token
    X_test[2] = (X_test[2].astype(np.float64) * 2.0 ** 40).astype(X_test.dtype)      # huge token: everything out of range
    X_test[3, 1:] = 0.0                     # one-hot-like
    X_test[n - 1] = 0.0
    run_case(layer, X_cal, X_test, 0.9, batched=True, check_calibrate=False)


def test_all_flagged_equals_dense_and_none_flagged_equals_folded():
    w = synth.tiny(hard=True)
    layer = w.layer
    ffn = make_ffn(layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "f32"), 0.9)
    Xd = dev(w.X_test[:4], "f32")
    # empty ranges: every neuron is flagged, the result is the exact FFN
    L = T.tardis_fold(ffn, hi.clone(), hi.clone(), a, c, max_batch=4)
    Y = host(T.tardis_ffn_forward_batched(L, Xd))
    _, counts, _ = T.tardis_get_last_outliers(L, 4)
    assert (counts.cpu().numpy() == layer.h).all()
    ref = O.dense(layer.W1, None, layer.W2, None, w.X_test[:4])
    assert rel_l2(Y, ref) <= 1e-4
    L.close()
    # infinite ranges: nothing is flagged, the result is W'x + b'
    inf = torch.full_like(lo, float("inf"))
    L = T.tardis_fold(ffn, -inf, inf, a, c, max_batch=4)
    Y = host(T.tardis_ffn_forward_batched(L, Xd))
    _, counts, _ = T.tardis_get_last_outliers(L, 4)
    assert (counts.cpu().numpy() == 0).all()
    Wp, bp = O.fold(layer.W1, None, layer.W2, None, a.cpu().numpy(), c.cpu().numpy())
    assert rel_l2(Y, w.X_test[:4].astype(np.float64) @ Wp.T + bp) <= 1e-4
    L.close()


def test_per_neuron_coverage_and_single_calibration_token():
    w = synth.tiny(hard=True)
    ffn = make_ffn(w.layer)
    t = np.linspace(0.5, 0.99, w.layer.h).astype(np.float32)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "f32"), 0.0, torch.from_numpy(t).to(DEV))
    olo, ohi, oa, oc = O.calibrate(w.layer.W1, None, w.X_cal, t)
    assert np.abs(lo.cpu().numpy() - olo).max() < 1e-5 and np.abs(hi.cpu().numpy() - ohi).max() < 1e-5
    assert np.abs(a.cpu().numpy() - oa).max() < 2e-2
    # n_cal = 1: lo = hi = z, no sample inside [lo, hi): slope 0, intercept sigma(lo)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal[:1], "f32"), 0.9)
    olo, ohi, oa, oc = O.calibrate(w.layer.W1, None, w.X_cal[:1], 0.9)
    np.testing.assert_allclose(lo.cpu().numpy(), olo, rtol=2e-6, atol=2e-6)     # fp32 vs fp64 dot products
    np.testing.assert_allclose(hi.cpu().numpy(), ohi, rtol=2e-6, atol=2e-6)
    np.testing.assert_array_equal(a.cpu().numpy(), 0.0)
    np.testing.assert_allclose(c.cpu().numpy(), oc, rtol=1e-5, atol=1e-5)


def test_calibrate_many_samples_uses_large_lds():
    # 20000 calibration tokens: the per-neuron sort needs 128 KiB of LDS (padded to 32768 samples)
    seed = synth.workload_seed(9, 3)
    layer = synth.make_layer(64, 128, "f32", seed, w1_std=0.2, w2_std=0.05)
    X_cal = synth.make_tokens(20000, 64, "f32", seed, synth.STREAM_CAL)
    ffn = make_ffn(layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, "f32"), 0.95)
    olo, ohi, oa, oc = O.calibrate(layer.W1, None, X_cal, 0.95)
    assert np.abs(lo.cpu().numpy() - olo).max() < 2e-5 and np.abs(hi.cpu().numpy() - ohi).max() < 2e-5
    assert np.abs(a.cpu().numpy() - oa).max() < 1e-3 and np.abs(c.cpu().numpy() - oc).max() < 1e-3


def test_fused_kernel_with_ragged_hidden_width_and_bias():
    # d = 2048 takes the single-launch kernel; h = 1000 is neither a multiple of 32 nor of the
    # per-block neuron count, and the layer has biases
    seed = synth.workload_seed(9, 4)
    layer = synth.make_layer(2048, 1000, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01, with_bias=True)
    X_cal = synth.make_tokens(256, 2048, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(7, 2048, "bf16", seed, synth.STREAM_TEST)
    run_case(layer, X_cal, X_test[:5], 0.9, check_calibrate=False)
    run_case(layer, X_cal, X_test, 0.9, check_calibrate=False, batched=True)     # groups of 4 + 2 + 1 tokens


def test_fused_kernel_many_flagged_per_block():
    # 40 % fallback: every block repairs far more neurons than one pass holds
    w = synth.decode(d=1024, h=4096, n_cal=256, n_test=4, coverage=0.6, config=9)
    r = run_case(w.layer, w.X_cal, w.X_test, 0.6, check_calibrate=False)
    assert r["rate"] > 0.3
    r = run_case(w.layer, w.X_cal, w.X_test, 0.6, check_calibrate=False, batched=True)   # four tokens per launch
    assert r["rate"] > 0.3


def test_two_kernel_groups_with_many_records_per_block():
    # h = 20000 gives 96 neurons per block: more record slots than a wavefront holds at once, and no
    # matrix-core tiling (eight tokens run as two groups of four); 80 % fallback fills most slots
    seed = synth.workload_seed(9, 31)
    layer = synth.make_layer(1024, 20000, "bf16", seed, w1_std=0.03, w2_std=0.01, heavy_frac=0.01)
    X_cal = synth.make_tokens(256, 1024, "bf16", seed, synth.STREAM_CAL)
    X_test = synth.make_tokens(8, 1024, "bf16", seed, synth.STREAM_TEST)
    r = run_case(layer, X_cal, X_test, 0.2, check_calibrate=False, batched=True)
    assert r["rate"] > 0.7


def test_graph_capture_and_replay_of_forward():
    # the online call allocates nothing and records no memset: it can be captured and replayed
    # (one-, two-, four- and eight-token groups: the last two run as two kernels each)
    w = synth.decode(d=1024, h=4096, n_cal=256, n_test=15, coverage=0.9, config=9)
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=16)
    X = dev(w.X_test, "bf16")
    y_eager = torch.stack([T.tardis_ffn_forward(L, X[t]).clone() for t in range(3)])
    yb_eager = T.tardis_ffn_forward_batched(L, X).clone()
    torch.cuda.synchronize()
    y_g = torch.zeros_like(y_eager)
    yb_g = torch.zeros_like(yb_eager)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for t in range(3):
            T.tardis_ffn_forward(L, X[t], y_g[t])
        T.tardis_ffn_forward_batched(L, X, yb_g)
    for rep in range(3):
        y_g.zero_()
        yb_g.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert rel_l2(host(y_g), host(y_eager)) < 2e-3, rep       # atomic ordering only
        assert rel_l2(host(yb_g), host(yb_eager)) < 2e-3, rep
        T.tardis_ffn_forward(L, X[5])                              # eager work between replays
        torch.cuda.synchronize()
    L.close()


@pytest.mark.parametrize("n", [40, 100, 300])
def test_graph_capture_of_pass_and_prompt_paths(n):
    """40 tokens (one 64-token pass), 100 (short-tile products that add atomically into results the
    library zeroes itself) and 300 (square tiles, K in ranges): captured once, replayed three
    times with eager work in between; every replay reproduces the eager call, masks bit for bit."""
    w = synth.decode(d=1024, h=4096, n_cal=256, n_test=n, coverage=0.9, config=9)
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=n)
    X = dev(w.X_test, "bf16")
    y_eager = T.tardis_ffn_forward_batched(L, X).clone()
    mask_eager = T.tardis_get_last_outliers(L, n, want_list=False)[0].clone()
    torch.cuda.synchronize()
    y_g = torch.zeros_like(y_eager)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        T.tardis_ffn_forward_batched(L, X, y_g)
    for rep in range(3):
        y_g.zero_()
        T.tardis_ffn_forward_batched(L, torch.roll(X, 1, 0).contiguous())   # eager work on other tokens in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert rel_l2(host(y_g), host(y_eager)) < 2e-3, rep       # atomic ordering only
        mask = T.tardis_get_last_outliers(L, n, want_list=False)[0]   # the replay's masks
        assert torch.equal(mask, mask_eager), rep
    L.close()


def test_result_does_not_depend_on_how_many_tokens_share_a_call():
    """The same tokens through every dispatch path - single launches, groups of 2-16, a 64-token
    pass, short and square tiles of the prompt path: the masks of a token are the same bits whatever
    call it is part of, its output agrees to rounding (strictly per-token semantics)."""
    w = synth.decode(d=1024, h=4096, n_cal=512, n_test=300, coverage=0.9, config=3)
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=300)
    X = dev(w.X_test, "bf16")
    ref_y, ref_m = [], []
    for t in range(300):
        ref_y.append(T.tardis_ffn_forward(L, X[t]).clone())
        ref_m.append(T.tardis_get_last_outliers(L, 1, want_list=False)[0][0].clone())
    ref_y, ref_m = torch.stack(ref_y), torch.stack(ref_m)
    torch.cuda.synchronize()
    for n in (2, 3, 5, 8, 13, 16, 17, 31, 64, 65, 100, 128, 129, 200, 256, 257, 300):
        y = T.tardis_ffn_forward_batched(L, X[:n].contiguous())
        m = T.tardis_get_last_outliers(L, n, want_list=False)[0]
        torch.cuda.synchronize()
        assert torch.equal(m, ref_m[:n]), n
        err = np.linalg.norm(host(y) - host(ref_y[:n]), axis=1) / np.linalg.norm(host(ref_y[:n]), axis=1)
        assert err.max() < 8e-3, (n, err.max())                  # two bf16 roundings of y apart at most
    L.close()


def test_next_layer_hint_changes_nothing_but_time():
    """Two layers that name each other as next: one- and two-token calls request the other layer's
    first predictor rows at the end of their kernel; masks and outputs are those of the unhinted
    calls.  A hint to a destroyed layer is ignored, a hint to a layer of another shape too."""
    ws = [synth.decode(d=1024, h=4096, n_cal=256, n_test=4, coverage=0.9, config=9, layer=li) for li in range(2)]
    Ls = []
    for w in ws:
        ffn = make_ffn(w.layer)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
        Ls.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=4))
    X = dev(ws[0].X_test, "bf16")

    def run_all():
        out = []
        for L in Ls:
            for n in (1, 2):
                y = T.tardis_ffn_forward_batched(L, X[:n].contiguous()).clone()
                m = T.tardis_get_last_outliers(L, n, want_list=False)[0].clone()
                out.append((y, m))
        torch.cuda.synchronize()
        return out

    ref = run_all()
    T.tardis_set_next_layer(Ls[0], Ls[1])
    T.tardis_set_next_layer(Ls[1], Ls[0])
    for (y, m), (yr, mr) in zip(run_all(), ref):
        assert torch.equal(m, mr)
        assert rel_l2(host(y), host(yr)) < 2e-3                  # atomic ordering only
    T.tardis_set_next_layer(Ls[0], Ls[0])                       # the same layer again: allowed
    y = T.tardis_ffn_forward(Ls[0], X[0])
    assert rel_l2(host(y), host(ref[0][0][0])) < 2e-3
    # another shape: accepted, ignored at launch
    w3 = synth.decode(d=1024, h=2048, n_cal=256, n_test=2, coverage=0.9, config=9, layer=5)
    ffn3 = make_ffn(w3.layer)
    L3 = T.tardis_fold(ffn3, *T.tardis_calibrate(ffn3, dev(w3.X_cal, "bf16"), 0.9), max_batch=2)
    T.tardis_set_next_layer(Ls[0], L3)
    y = T.tardis_ffn_forward(Ls[0], X[0])
    assert rel_l2(host(y), host(ref[0][0][0])) < 2e-3
    # destroyed: the stale hint is ignored
    T.tardis_set_next_layer(Ls[0], Ls[1])
    Ls[1].close()
    y = T.tardis_ffn_forward(Ls[0], X[0])
    torch.cuda.synchronize()
    assert rel_l2(host(y), host(ref[0][0][0])) < 2e-3
    T.tardis_set_next_layer(Ls[0], None)
    Ls[0].close()
    L3.close()


def test_destroy_returns_the_layer_s_memory():
    """Folding and destroying a layer many times (with every scratch area: records, 64-token
    passes, prompt path) leaves the device's free memory where it was."""
    w = synth.decode(d=1024, h=4096, n_cal=256, n_test=128, coverage=0.9, config=9)
    ffn = make_ffn(w.layer)
    cal = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    X = dev(w.X_test, "bf16")
    Y = torch.empty_like(X)

    def cycle():
        L = T.tardis_fold(ffn, *cal, max_batch=128)
        T.tardis_ffn_forward_batched(L, X, Y)
        T.tardis_ffn_forward_batched(L, X[:40].contiguous(), Y[:40])
        T.tardis_ffn_forward(L, X[0], Y[0])
        torch.cuda.synchronize()
        L.close()

    cycle()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(20):
        cycle()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert abs(free1 - free0) <= 8 << 20, (free0, free1)      # nothing of a layer's ~100 MB stays behind


def test_runtime_argument_errors():
    w = synth.tiny()
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "f32"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=2)
    X = dev(w.X_test[:4], "f32")
    with pytest.raises(T.TardisError) as e:
        T.tardis_ffn_forward_batched(L, X)                       # n > max_batch
    assert e.value.status == T.ERR_SHAPE
    with pytest.raises(T.TardisError) as e:
        T.tardis_ffn_forward(L, X[0], X[0])                      # aliasing
    assert e.value.status == T.ERR_INVALID_ARG
    T.tardis_ffn_forward_batched(L, X[:2])
    with pytest.raises(T.TardisError) as e:
        T.tardis_get_last_outliers(L, 1)                         # last call had 2 tokens
    assert e.value.status == T.ERR_STATE
    L.close()


def test_repeated_calls_are_stable():
    # the same token twice gives the same mask and (up to atomic ordering) the same y
    w = synth.tiny(hard=True)
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "f32"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c)
    x = dev(w.X_test[3], "f32")
    y1 = host(T.tardis_ffn_forward(L, x))
    m1, c1, _ = T.tardis_get_last_outliers(L, 1)
    m1 = m1.clone()
    for _ in range(5):
        y2 = host(T.tardis_ffn_forward(L, x))
    m2, c2, _ = T.tardis_get_last_outliers(L, 1)
    assert torch.equal(m1, m2) and int(c1.item()) == int(c2.item())
    assert rel_l2(y2, y1) < 1e-6
    L.close()


# ------------------------------------------------------------- stacked layers
@pytest.mark.parametrize("d,h", [(1024, 4096), (4096, 2048), (2048, 1000)])
def test_deterministic_layer_is_bit_identical_from_run_to_run(d, h):
    """opts.deterministic = 1: the repair is accumulated in counted fixed-point words (integer adds
    commute) and flagged lists are walked in ascending order, so twenty repeats of a call give the
    same bits; against the checker the results are held to the same bars as any layer."""
    w = synth.decode(d=d, h=h, n_cal=512, n_test=40, coverage=0.9)
    lay = w.layer
    ffn = make_ffn(lay)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.9)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=40, deterministic=True)
    Lf = T.tardis_fold(ffn, lo, hi, a, c, max_batch=40)
    F = O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)))
    X = dev(w.X_test, "bf16")
    for n in (1, 2, 3, 4, 7, 8, 13, 16, 40):
        xb = X[:n].contiguous()
        first = T.tardis_ffn_forward_batched(L, xb).clone()
        mask, counts, lst = T.tardis_get_last_outliers(L, n)
        mask, counts, lst = mask.clone(), counts.clone(), lst.clone()
        for rep in range(20):
            y = T.tardis_ffn_forward_batched(L, xb)
            assert torch.equal(y, first), (n, rep)
        Yo, FLo = O.forward(F, w.X_test[:n])
        np.testing.assert_array_equal(unpack_mask(mask, h), FLo)
        assert_y_close(host(first), Yo, F, w.X_test[:n], FLo)
        cn, ls = counts.cpu().numpy(), lst.cpu().numpy()
        for t in range(n):
            np.testing.assert_array_equal(ls[t, :cn[t]], np.flatnonzero(FLo[t]))       # ascending
        # and the same numbers, to rounding, as the layer folded without the option
        yf = T.tardis_ffn_forward_batched(Lf, xb)
        assert rel_l2(host(first), host(yf)) < 2e-3
    L.close()
    Lf.close()


def test_deterministic_stack_and_refusals():
    d, h, nl = 1024, 2048, 3
    layers, oracles = [], []
    for li in range(nl):
        seed = synth.workload_seed(4, 50 + li)
        lay = synth.make_layer(d, h, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01)
        ffn = make_ffn(lay)
        X_cal = synth.make_tokens(512, d, "bf16", seed, synth.STREAM_CAL)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, "bf16"), 0.9)
        layers.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=8, deterministic=True))
        oracles.append(O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c))))
    x0 = synth.make_tokens(8, d, "bf16", synth.workload_seed(4, 60), synth.STREAM_TEST)
    for n in (1, 2, 5, 8):
        xb = dev(x0[:n], "bf16")
        first = T.tardis_stack_forward(layers, xb).clone()
        hand = [T.tardis_get_handover(layers[li], n).clone() for li in range(nl - 1)]
        for rep in range(10):
            assert torch.equal(T.tardis_stack_forward(layers, xb), first), (n, rep)
        x_in = x0[:n].astype(np.float64)
        for li in range(nl):      # teacher-forced against the checker, as for any stack
            Yo, FLo = O.forward(oracles[li], x_in)
            mask, _, _ = T.tardis_get_last_outliers(layers[li], n, want_list=False)
            np.testing.assert_array_equal(unpack_mask(mask, h), FLo)
            if li < nl - 1:
                assert rel_l2(host(hand[li]), O.to_bf16(O.rmsnorm(Yo))) <= 1e-2
                x_in = host(hand[li])
            else:
                assert_y_close(host(first), Yo, oracles[li], x_in, FLo)
    for L in layers:
        L.close()
    # an fp32 layer has no ordered path: refused when folded, not silently run unordered
    wt = synth.tiny()
    ffn = make_ffn(wt.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(wt.X_cal, "f32"), 0.9)
    with pytest.raises(T.TardisError) as e:
        T.tardis_fold(ffn, lo, hi, a, c, deterministic=True)
    assert e.value.status == T.ERR_SHAPE


def test_fixed_point_accumulators_by_knob(monkeypatch):
    """TARDIS_FIXED_POINT=1 puts the counted fixed-point accumulators under the ordinary dispatch
    (token passes and prompts unchanged): the decode groups against the checker, single token,
    groups, a partly filled group, graph replay."""
    monkeypatch.setenv("TARDIS_FIXED_POINT", "1")
    w = synth.decode(d=2048, h=4096, n_cal=512, n_test=16, coverage=0.9)
    r = run_case(w.layer, w.X_cal, w.X_test[:11], 0.9, batched=True, check_calibrate=False, max_batch=16)
    assert r["y_err"] < 1e-2
    r = run_case(w.layer, w.X_cal, w.X_test[:3], 0.9, batched=False, check_calibrate=False)
    assert r["y_err"] < 1e-2
    lay = custom_layer(1024, 777, "bf16", synth.workload_seed(5, 3), 0.05, True)     # ragged h, biases
    Xc = synth.make_tokens(400, 1024, "bf16", 77, synth.STREAM_CAL)
    Xt = synth.make_tokens(9, 1024, "bf16", 77, synth.STREAM_TEST)
    run_case(lay, Xc, Xt, 0.8, act="gelu_tanh", batched=True, max_batch=9)


@pytest.mark.parametrize("d,h,dtype,n", [(1024, 4096, "bf16", 1), (1024, 4096, "bf16", 3), (64, 256, "f32", 2),
                                         (1024, 4096, "bf16", 12), (2048, 2048, "bf16", 8), (2048, 2048, "bf16", 16),
                                         (2048, 2048, "bf16", 6), (1024, 4096, "bf16", 40), (1024, 2048, "bf16", 90)])
def test_stack_teacher_forced(d, h, dtype, n):
    """Every layer is checked on the input the GPU itself handed to it: mask bit-exact, the
    normalised hand-over and the final output within the y tolerance.  (40 tokens: a 64-token pass
    per layer; 90: the prompt path, whose last kernel applies the norm.)"""
    nl = 3
    layers, oracles = [], []
    x0 = synth.make_tokens(n, d, dtype, synth.workload_seed(4, 99), synth.STREAM_TEST)
    for li in range(nl):
        seed = synth.workload_seed(4, li)
        lay = synth.make_layer(d, h, dtype, seed, w1_std=0.03 if dtype == "bf16" else 0.2, w2_std=0.03,
                               heavy_frac=0.01)
        ffn = make_ffn(lay)
        X_cal = synth.make_tokens(512, d, dtype, seed, synth.STREAM_CAL)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, dtype), 0.9)
        layers.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=n))
        oracles.append(O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c))))
    y = T.tardis_stack_forward(layers, dev(x0, dtype))
    torch.cuda.synchronize()
    x_in = x0.astype(np.float64)
    for li in range(nl):
        Yo, FLo = O.forward(oracles[li], x_in)
        mask, counts, _ = T.tardis_get_last_outliers(layers[li], n, want_list=False)
        np.testing.assert_array_equal(unpack_mask(mask, h), FLo)
        assert (counts.cpu().numpy() == FLo.sum(1)).all()
        if li < nl - 1:
            xn = host(T.tardis_get_handover(layers[li], n))
            want = O.rmsnorm(Yo)
            if dtype == "bf16":
                want = O.to_bf16(want)
            assert rel_l2(xn, want) <= Y_TOL[dtype]
            x_in = xn                                   # teacher forcing: the GPU's own hand-over
        else:
            assert_y_close(host(y), Yo, oracles[li], x_in, FLo, dtype)
    # one call per layer with host-side glue gives the same final result
    for L in layers:
        L.close()


@pytest.mark.parametrize("d,h,nl", [(2048, 4096, 6), (1024, 3000, 5), (4096, 4096, 4)])
def test_single_token_stack_in_one_launch(d, h, nl, monkeypatch):
    """One token through a stack runs as ONE resident launch (blocks wait for each layer's published
    output).  Several tokens one after the other - the counters and accumulators must come back
    re-armed - each checked layer by layer on the GPU's own hand-over; the per-layer launches
    (TARDIS_STACK_FUSED=0 at fold time) serve as a second opinion on the final output."""
    calib, lays, oracles = [], [], []
    for li in range(nl):
        seed = synth.workload_seed(14, li)
        lay = synth.make_layer(d, h, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01)
        ffn = make_ffn(lay)
        X_cal = synth.make_tokens(384, d, "bf16", seed, synth.STREAM_CAL)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, "bf16"), 0.9)
        calib.append((ffn, lo, hi, a, c))
        lays.append(lay)
        oracles.append(O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c))))
    monkeypatch.setenv("TARDIS_STACK_FUSED", "2")      # refuse instead of falling back to a launch per layer
    fused = [T.tardis_fold(*cal, max_batch=1) for cal in calib]
    monkeypatch.setenv("TARDIS_STACK_FUSED", "0")
    layerwise = [T.tardis_fold(*cal, max_batch=1) for cal in calib]
    monkeypatch.delenv("TARDIS_STACK_FUSED")
    X = synth.make_tokens(3, d, "bf16", synth.workload_seed(14, 99), synth.STREAM_TEST)
    for t in (0, 1, 2, 0):
        x0 = X[t:t + 1]
        y = T.tardis_stack_forward(fused, dev(x0, "bf16"))
        y2 = T.tardis_stack_forward(layerwise, dev(x0, "bf16"))
        torch.cuda.synchronize()
        x_in = x0.astype(np.float64)
        for li in range(nl):
            Yo, FLo = O.forward(oracles[li], x_in)
            mask, counts, _ = T.tardis_get_last_outliers(fused[li], 1, want_list=False)
            np.testing.assert_array_equal(unpack_mask(mask, h), FLo, err_msg=f"token {t} layer {li}")
            assert (counts.cpu().numpy() == FLo.sum(1)).all()
            if li < nl - 1:
                xn = host(T.tardis_get_handover(fused[li], 1))
                assert rel_l2(xn, O.to_bf16(O.rmsnorm(Yo))) <= Y_TOL["bf16"], (t, li)
                if li == 0:     # same input, same mask: the two paths differ by summation order only
                    m2, _, _ = T.tardis_get_last_outliers(layerwise[0], 1, want_list=False)
                    assert torch.equal(mask, m2)
                    assert rel_l2(host(T.tardis_get_handover(layerwise[0], 1)), xn) <= 1e-2
                x_in = xn
            else:
                assert_y_close(host(y), Yo, oracles[li], x_in, FLo, "bf16")
        assert torch.isfinite(y2.float()).all()
    for L in fused + layerwise:
        L.close()


def test_single_launch_stack_gives_up_loudly_and_recovers(monkeypatch):
    """The resident launch waits for every layer's counter with a bounded number of polls.  With the
    bound forced down to one poll from the host (every kernel still runs to its end) the blocks give
    up: the call's output is all NaN rather than a plausible wrong vector, and the kernel behind the
    launch has re-armed every layer - the same handles then serve a two-token call (a launch per
    layer) correctly."""
    d, h, nl = 1024, 2048, 4
    monkeypatch.setenv("TARDIS_STACK_FUSED", "1")
    monkeypatch.setenv("TARDIS_STACK_SPIN_LIMIT", "1")
    layers, oracles = [], []
    for li in range(nl):
        seed = synth.workload_seed(15, li)
        lay = synth.make_layer(d, h, "bf16", seed, w1_std=0.03, w2_std=0.03, heavy_frac=0.01)
        ffn = make_ffn(lay)
        X_cal = synth.make_tokens(256, d, "bf16", seed, synth.STREAM_CAL)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(X_cal, "bf16"), 0.9)
        layers.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=2))
        oracles.append(O.build(lay.W1, None, lay.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c))))
    X = synth.make_tokens(2, d, "bf16", synth.workload_seed(15, 99), synth.STREAM_TEST)
    for rep in range(2):
        y = T.tardis_stack_forward(layers, dev(X[:1], "bf16"))
        torch.cuda.synchronize()
        assert torch.isnan(y.float()).all(), rep
    y2 = T.tardis_stack_forward(layers, dev(X, "bf16"))
    torch.cuda.synchronize()
    x_in = X.astype(np.float64)
    for li in range(nl):
        Yo, FLo = O.forward(oracles[li], x_in)
        mask, _, _ = T.tardis_get_last_outliers(layers[li], 2, want_list=False)
        np.testing.assert_array_equal(unpack_mask(mask, h), FLo)
        if li < nl - 1:
            x_in = host(T.tardis_get_handover(layers[li], 2))
        else:
            assert_y_close(host(y2), Yo, oracles[li], x_in, FLo, "bf16")
    for L in layers:
        L.close()


# ------------------------------------------------ config 1 at full size (d=4096, h=16384, bf16)
@pytest.fixture(scope="module")
def decode_full():
    w = synth.decode(n_cal=4096, n_test=2048, coverage=0.95)
    ffn = make_ffn(w.layer)
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), w.coverage)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=2048)
    torch.cuda.synchronize()
    box = {}

    def oracle():
        if "F" not in box:      # built once: the fp64 fold of the full layer takes several seconds
            box["F"] = O.build(w.layer.W1, None, w.layer.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)))
        return box["F"]

    yield w, ffn, (lo, hi, a, c), L, oracle
    L.close()


def test_full_size_calibrate_on_sampled_neurons(decode_full):
    w, ffn, (lo, hi, a, c), L, _ = decode_full
    rng = np.random.default_rng(0)
    sub = np.sort(rng.choice(w.layer.h, 192, replace=False))
    sub[:4] = w.layer.heavy_neurons[:4]
    olo, ohi, oa, oc = O.calibrate(w.layer.W1[sub], None, w.X_cal, w.coverage)
    glo, ghi, ga, gc = (t.cpu().numpy()[sub] for t in (lo, hi, a, c))
    scale = float(np.abs(np.concatenate([olo, ohi])).max())
    assert np.abs(glo - olo).max() <= 2e-5 * scale and np.abs(ghi - ohi).max() <= 2e-5 * scale
    assert np.abs(ga - oa).max() <= 2e-3 and np.abs(gc - oc).max() <= 2e-3 * max(1.0, scale)
    # the range really holds the requested portion of the calibration inputs
    Z = O.preact(w.layer.W1[sub], None, w.X_cal)
    frac = ((Z >= glo[None, :].astype(np.float64)) & (Z < ghi[None, :].astype(np.float64))).mean(0)
    assert np.abs(frac - w.coverage).max() <= 3.0 / w.X_cal.shape[0]


def test_full_size_calibrate_search_on_sampled_neurons(decode_full):
    w, ffn, _, _, _ = decode_full
    t, step = float(np.float32(0.95)), float(np.float32(0.05))
    lo, hi, a, c = (v.cpu().numpy() for v in T.tardis_calibrate_search(ffn, dev(w.X_cal, "bf16"), t, step))
    rng = np.random.default_rng(1)
    sub = np.sort(rng.choice(w.layer.h, 48, replace=False))
    sub[:3] = w.layer.heavy_neurons[:3]
    olo, ohi, oa, oc = O.calibrate_search(w.layer.W1[sub], None, w.X_cal, t, step)
    scale = float(np.abs(np.concatenate([olo, ohi])).max())
    same = (np.abs(lo[sub] - olo) <= 1e-4 * scale) & (np.abs(hi[sub] - ohi) <= 1e-4 * scale)
    assert same.mean() >= 0.9, same.mean()
    Zs = O.preact(w.layer.W1[sub], None, w.X_cal)
    assert_search_differences_are_near_ties(Zs, np.full(len(sub), t), step, "gelu_erf", np.flatnonzero(~same), scale)
    assert np.abs(a[sub] - oa)[same].max() <= 2e-3 and np.abs(c[sub] - oc)[same].max() <= 2e-3 * max(1.0, scale)
    Z = O.preact(w.layer.W1[sub], None, w.X_cal)
    frac = ((Z >= lo[sub][None, :].astype(np.float64)) & (Z < hi[sub][None, :].astype(np.float64))).mean(0)
    assert (frac >= t - 2.0 / w.X_cal.shape[0]).all() and (frac < t + 0.05).all()
    assert np.isfinite(lo).all() and np.isfinite(hi).all() and (hi > lo).all()


def test_full_size_decode_batch1(decode_full):
    w, ffn, (lo, hi, a, c), L, oracle = decode_full
    layer = w.layer
    F = oracle()
    Wp, bp = T.tardis_get_folded(L)
    Q, tlo, thi = T.tardis_get_predictor_state(L)
    assert rel_l2(host(Wp), F.Wp) <= 3e-3
    assert rel_l2(host(bp), F.bp) <= 1e-5
    assert torch.equal(Q.cpu(), torch.from_numpy(F.sk.Q))
    np.testing.assert_array_equal(tlo.cpu().numpy(), F.sk.tlo)
    np.testing.assert_array_equal(thi.cpu().numpy(), F.sk.thi)
    n = 16
    Xd = dev(w.X_test[:n], "bf16")
    Yo, FLo = O.forward(F, w.X_test[:n])
    Yg = np.empty_like(Yo)
    rates = []
    for t in range(n):
        y = T.tardis_ffn_forward(L, Xd[t])
        mask, cnt, lst = T.tardis_get_last_outliers(L, 1)
        torch.cuda.synchronize()
        Yg[t] = host(y)
        np.testing.assert_array_equal(unpack_mask(mask, layer.h)[0], FLo[t])
        k = int(cnt.item())
        assert k == FLo[t].sum()
        np.testing.assert_array_equal(np.sort(lst.cpu().numpy()[0, :k]), np.flatnonzero(FLo[t]))
        rates.append(k / layer.h)
    assert_y_close(Yg, Yo, F, w.X_test[:n], FLo)
    assert abs(np.mean(rates) - 0.05) < 0.01                      # test-time fallback rate ~ 1 - t
    # the fix matters: without it the folded product alone is far from the checker's result
    Y0, _ = O.forward(F, w.X_test[:n], np.zeros_like(FLo))
    assert rel_l2(Y0, Yo) > 5 * rel_l2(Yg, Yo)
    Yd = host(T.tardis_dense_forward(L, Xd[:8]))
    assert rel_l2(Yd, O.dense(layer.W1, None, layer.W2, None, w.X_test[:8])) <= 1e-2


def test_full_size_batched_matches_per_token(decode_full):
    w, ffn, _, L, _ = decode_full
    Xd = dev(w.X_test[16:24], "bf16")
    Yb = T.tardis_ffn_forward_batched(L, Xd)
    mb, cb, _ = T.tardis_get_last_outliers(L, 8, want_list=False)
    mb, cb = mb.clone(), cb.clone()
    for t in range(8):
        y = T.tardis_ffn_forward(L, Xd[t])
        m1, c1, _ = T.tardis_get_last_outliers(L, 1, want_list=False)
        assert torch.equal(m1[0], mb[t]) and int(c1.item()) == int(cb[t].item())
        assert rel_l2(host(y), host(Yb[t])) <= 2e-3            # bf16 output, atomic ordering


@pytest.mark.parametrize("B", [2, 3, 4, 7, 8, 13, 16, 64])
def test_full_size_batched_decode_sampled_tokens(decode_full, B):
    """Batched decode at the full layer size, in the configuration the sweep times: the checker
    recomputes a sample of the batch's tokens one by one."""
    w, ffn, _, L, oracle = decode_full
    F = oracle()
    X = w.X_test[100:100 + B]
    Y = T.tardis_ffn_forward_batched(L, dev(X, "bf16"))
    mask, counts, _ = T.tardis_get_last_outliers(L, B, want_list=False)
    torch.cuda.synchronize()
    FLg = unpack_mask(mask, w.layer.h)
    for t in sorted({0, 1, B // 2, B - 1}):
        yo, flo = O.forward_token(F, X[t])
        np.testing.assert_array_equal(FLg[t], flo)
        assert int(counts[t].item()) == flo.sum()
        assert_y_close(host(Y[t]), yo, F, X[t], flo)
    ucnt, _ = T.tardis_get_last_union(L, B)
    assert int(ucnt.item()) == FLg.any(axis=0).sum() >= FLg[0].sum()


@pytest.fixture(scope="module", params=[0.99, 0.85])
def decode_full_other_rates(request, decode_full):
    """The decode layer calibrated for the other two fallback rates of the batched sweep (about 1 %
    and 15 %), folded for 64 tokens per call as the sweep does."""
    w, ffn, _, _, _ = decode_full
    cov = request.param
    lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), cov)
    L = T.tardis_fold(ffn, lo, hi, a, c, max_batch=64)
    torch.cuda.synchronize()
    F = O.build(w.layer.W1, None, w.layer.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)))
    yield w, L, F, cov
    L.close()


@pytest.mark.parametrize("B", [4, 16, 64])
def test_full_size_batched_decode_other_fallback_rates(decode_full_other_rates, B):
    """Batched decode sweep at full size, the 1 % and 15 % legs: masks bit for bit on every token,
    sampled tokens against the checker element by element, the measured rate near 1 - t."""
    w, L, F, cov = decode_full_other_rates
    X = w.X_test[200:200 + B]
    Y = T.tardis_ffn_forward_batched(L, dev(X, "bf16"))
    mask, counts, _ = T.tardis_get_last_outliers(L, B, want_list=False)
    torch.cuda.synchronize()
    FLg = unpack_mask(mask, w.layer.h)
    for t in sorted({0, B // 3, B - 1}):
        yo, flo = O.forward_token(F, X[t])
        np.testing.assert_array_equal(FLg[t], flo)
        assert int(counts[t].item()) == flo.sum()
        assert_y_close(host(Y[t]), yo, F, X[t], flo)
    # every token's mask against the checker's predictor alone (cheap: no repair)
    for t in range(B):
        np.testing.assert_array_equal(FLg[t], O.predict(F.sk, X[t]))
    rate = FLg.mean()
    assert abs(rate - (1.0 - cov)) < 0.35 * (1.0 - cov) + 0.002, rate


def test_full_size_prefill_sampled_tokens(decode_full):
    """2048 tokens x d=4096 through the layer (the prompt path): sampled tokens against the checker,
    and every token's flag count against the expected fallback rate."""
    w, ffn, _, L, oracle = decode_full
    F = oracle()
    n = 2048
    Y = T.tardis_ffn_forward_batched(L, dev(w.X_test, "bf16"))
    mask, counts, _ = T.tardis_get_last_outliers(L, n, want_list=False)
    torch.cuda.synchronize()
    FLg = unpack_mask(mask, w.layer.h)
    for t in (0, 63, 64, 1000, 2047):
        yo, flo = O.forward_token(F, w.X_test[t])
        np.testing.assert_array_equal(FLg[t], flo)
        assert_y_close(host(Y[t]), yo, F, w.X_test[t], flo)
    cnt = counts.cpu().numpy()
    assert (cnt == FLg.sum(1)).all()
    assert abs(cnt.mean() / w.layer.h - 0.05) < 0.005
    assert torch.isfinite(Y.float()).all()


def test_full_size_prompt_256_tokens(decode_full):
    """256 tokens at full size: one row of output tiles, so every product of the prompt path cuts K
    into ranges that add atomically (the int8 sums stay exact: integer adds)."""
    w, ffn, _, L, oracle = decode_full
    F = oracle()
    n = 256
    Y = T.tardis_ffn_forward_batched(L, dev(w.X_test[:n], "bf16"))
    mask, counts, _ = T.tardis_get_last_outliers(L, n, want_list=False)
    torch.cuda.synchronize()
    FLg = unpack_mask(mask, w.layer.h)
    for t in (0, 100, 255):
        yo, flo = O.forward_token(F, w.X_test[t])
        np.testing.assert_array_equal(FLg[t], flo)
        assert_y_close(host(Y[t]), yo, F, w.X_test[t], flo)
    assert (counts.cpu().numpy() == FLg.sum(1)).all()
    assert torch.isfinite(Y.float()).all()


def test_full_size_sketch4_decode(decode_full):
    """The full layer folded with the 4-bit sketch: codes and multipliers bit-exact, masks bit-exact
    and y within the bar for single tokens and a group of four; the flag rate rises a little
    because the coarser predictor errs on both sides."""
    w, ffn, (lo, hi, a, c), _, _ = decode_full
    L4 = T.tardis_fold(ffn, lo, hi, a, c, max_batch=8, sketch_bits=4)
    sk = O.sketch(w.layer.W1, None, lo.cpu().numpy(), hi.cpu().numpy(), bits=4)
    Q, tlo, thi = T.tardis_get_predictor_state(L4)
    assert torch.equal(Q.cpu(), torch.from_numpy(sk.Q))
    np.testing.assert_array_equal(T.tardis_get_sketch_groups(L4).cpu().numpy(), sk.m)
    np.testing.assert_array_equal(tlo.cpu().numpy(), sk.tlo)
    np.testing.assert_array_equal(thi.cpu().numpy(), sk.thi)
    F = O.build(w.layer.W1, None, w.layer.W2, None, *(t.cpu().numpy() for t in (lo, hi, a, c)), sketch_bits=4)
    X = w.X_test[300:306]
    Yo, FLo = O.forward(F, X)
    Xd = dev(X, "bf16")
    for t in range(2):
        y = T.tardis_ffn_forward(L4, Xd[t])
        mask, cnt, _ = T.tardis_get_last_outliers(L4, 1, want_list=False)
        np.testing.assert_array_equal(unpack_mask(mask, w.layer.h)[0], FLo[t])
        assert_y_close(host(y), Yo[t], F, X[t], FLo[t])
    Y = T.tardis_ffn_forward_batched(L4, Xd)                     # 4 + 2 tokens per launch
    mask, counts, _ = T.tardis_get_last_outliers(L4, 6, want_list=False)
    np.testing.assert_array_equal(unpack_mask(mask, w.layer.h), FLo)
    assert_y_close(host(Y), Yo, F, X, FLo)
    assert 0.04 < FLo.mean() < 0.09
    L4.close()


def test_full_size_stack_of_three_layers():
    """Three independent full-size layers chained with the RMS-norm glue at batch 1 and 32; every
    layer is checked on the input the GPU handed to it (sampled tokens for the batch)."""
    d, h, nl = 4096, 16384, 3
    layers, lays, cals = [], [], []
    for li in range(nl):
        w = synth.decode(layer=li, n_cal=1024, n_test=32, coverage=0.95, config=4)
        ffn = make_ffn(w.layer)
        lo, hi, a, c = T.tardis_calibrate(ffn, dev(w.X_cal, "bf16"), 0.95)
        layers.append(T.tardis_fold(ffn, lo, hi, a, c, max_batch=32))
        lays.append(w.layer)
        cals.append(tuple(t.cpu().numpy() for t in (lo, hi, a, c)))
        if li == 0:
            X0 = w.X_test
    for B, sample in ((1, [0]), (32, [0, 31])):
        x0 = X0[:B]
        y = T.tardis_stack_forward(layers, dev(x0, "bf16"))
        torch.cuda.synchronize()
        x_in = x0.astype(np.float64)
        for li in range(nl):
            F = O.build(lays[li].W1, None, lays[li].W2, None, *cals[li])
            mask, counts, _ = T.tardis_get_last_outliers(layers[li], B, want_list=False)
            FLg = unpack_mask(mask, h)
            xn = host(T.tardis_get_handover(layers[li], B)) if li < nl - 1 else None
            for t in sample:
                yo, flo = O.forward_token(F, x_in[t])
                np.testing.assert_array_equal(FLg[t], flo)
                if li < nl - 1:
                    assert rel_l2(xn[t], O.to_bf16(O.rmsnorm(yo[None])[0])) <= 1e-2
                else:
                    assert_y_close(host(y)[t], yo, F, x_in[t], flo)
            del F
            x_in = xn
    for L in layers:
        L.close()
