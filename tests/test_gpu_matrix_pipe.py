"""The accumulation error of the bf16 matrix pipe against the figure the default BMU search's rounding bound counts.

The search (Section 3.3.1, b(x)) forms its scores with v_mfma_f32_32x32x16_bf16 and re-decides by float32 direct
differences every sample whose best two scores are closer than a worst-case error bound.  That bound charges each
MFMA  16 * 2^-24 * (|C| + sum_k |a_k b_k|):  what seventeen float32 terms can lose when they are added in ANY order
with one round-to-nearest per addition (the products themselves are exact in float32).  How the pipe really adds is
not documented, so this file measures it, on operands built to be as bad as possible for an adder that aligns,
truncates or adds sequentially (random operands almost never are), and fails at the first result outside the figure.

The exact sums are taken in x87 extended precision (64-bit significand), which holds every term of every case here
without rounding: the cases keep all terms inside a window of 2^42 (16 product bits and 5 carry bits on top stay below 64).
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

UNITS_CHARGED = 16.0          # per MFMA, in units of 2^-24 (|C| + sum |products|): the figure in som_bmu.hip
U = 2.0 ** -24


@pytest.fixture(scope="module")
def som():
    from paper_2604_26555_amd import Som
    s = Som(0)
    yield s
    s.close()


def to_bf16(x):
    """Round float32 values to the nearest bf16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return u.view(np.float32)


def run_case(som, name, A, Bt, C, report):
    """A, Bt: (n, 32, 16) float32 holding bf16 values; C: (n, 32, 32) float32.  Returns the largest error in units."""
    assert np.array_equal(to_bf16(A), A) and np.array_equal(to_bf16(Bt), Bt)
    D = som.som_matrix_pipe_probe(torch.from_numpy(A).to(torch.bfloat16).cuda(), torch.from_numpy(Bt).to(torch.bfloat16).cuda(),
                                  torch.from_numpy(C).cuda())
    som.som_sync()
    D = D.cpu().numpy()
    L = np.longdouble
    assert np.finfo(L).nmant >= 63, "needs x87 extended precision for the exact sums"
    prod = A.astype(L)[:, :, None, :] * Bt.astype(L)[:, None, :, :]          # (n, 32, 32, 16), exact
    exact = C.astype(L) + prod.sum(axis=3)
    mag = np.abs(C.astype(L)) + np.abs(prod).sum(axis=3)
    # the window claim: every non-zero term is at least 2^-42 of the total magnitude in its sum
    small = np.where(prod != 0, np.abs(prod), np.inf).min(axis=3)
    assert (small[np.isfinite(small)] >= (mag * L(2.0) ** -42)[np.isfinite(small)]).all(), name
    err = np.abs(D.astype(L) - exact)
    units = np.where(mag > 0, err / np.where(mag > 0, mag * L(U), 1), 0).astype(np.float64)
    units_of_max = np.where(mag > 0, err / (np.maximum(np.abs(C.astype(L)), np.abs(prod).sum(axis=3)) * L(U) + L(1e-300)), 0)
    rounded = exact.astype(np.float32)
    frac_correct = float((D == rounded).mean())
    worst = float(units.max())
    report.append((name, worst, float(units_of_max.max()), frac_correct, D.size))
    print(f"{name:34s} worst {worst:6.3f} units of 2^-24 (|C| + sum|p|)   {float(units_of_max.max()):6.3f} of 2^-24 max(|C|, sum|p|)"
          f"   correctly rounded {frac_correct:.4f} of {D.size}", flush=True)
    assert worst <= UNITS_CHARGED, f"{name}: {worst} units exceed the {UNITS_CHARGED} the search's bound charges per MFMA"
    return worst


def shuffle_k(rng, A, Bt):
    """The same sums with the sixteen products in another k order per problem (the adder's tree is unknown)."""
    for t in range(A.shape[0]):
        p = rng.permutation(16)
        A[t] = A[t][:, p]
        Bt[t] = Bt[t][:, p]
    return A, Bt


def mant(rng, shape, ones=False):
    """bf16 significands in [1, 2): all ones (1.9921875) or random."""
    if ones:
        return np.full(shape, 1.9921875, dtype=np.float32)
    return (1.0 + rng.integers(0, 128, size=shape) / 128.0).astype(np.float32)


def test_bf16_mfma_accumulation_error_on_structured_worst_cases(som):
    rng = np.random.default_rng(2604)
    n = 96
    report = []

    # 1. half-ulp flood: C of order one, sixteen same-sign products each just below (or at, or above) half a unit in
    #    the last place of C.  A sequential round-to-nearest adder loses every one of them.
    for sign_rule in ("same", "opposite", "mixed"):
        for ones in (True, False):
            A = mant(rng, (n, 32, 16), ones) * 0.5
            shift = -(24.0 + np.arange(32) % 8 - 3.0)                            # column j: products near 2^-21 .. 2^-28
            Bt = np.broadcast_to((2.0 ** shift)[None, :, None], (n, 32, 16)).astype(np.float32) * mant(rng, (n, 32, 16), ones)
            Bt = to_bf16(Bt)
            C = (1.0 + rng.integers(0, 2 ** 23, size=(n, 32, 32)) / 2.0 ** 23).astype(np.float32)
            if sign_rule == "opposite":
                C = -C
            if sign_rule == "mixed":
                A *= rng.choice([-1.0, 1.0], size=A.shape).astype(np.float32)
            A, Bt = shuffle_k(rng, A.copy(), Bt.copy())
            run_case(som, f"flood {sign_rule} ones={ones}", A, Bt, C, report)

    # 2. products with descending exponents, same sign, all-ones significands: an adder that aligns to the largest
    #    term and truncates loses a piece of every smaller one.
    for step in (1, 2, 3):
        for cexp in (None, -30, 0, 6):
            A = mant(rng, (n, 32, 16), True) * (2.0 ** (-step * np.arange(16)))[None, None, :].astype(np.float32)
            A = to_bf16(A)
            Bt = mant(rng, (n, 32, 16), False)
            C = np.zeros((n, 32, 32), dtype=np.float32) if cexp is None else \
                ((1.0 + rng.integers(0, 2 ** 23, size=(n, 32, 32)) / 2.0 ** 23) * 2.0 ** cexp).astype(np.float32)
            if cexp == -30:
                C = np.maximum(C, np.float32(2.0 ** -30))
            A, Bt = shuffle_k(rng, A.copy(), Bt.copy())
            # the window: smallest product 2^(-15 step) against a sum of order 2^max(2, cexp)
            if 15 * step + max(2, cexp or 0) <= 40:
                run_case(som, f"descending 2^-{step}k, C~2^{cexp}", A, Bt, C, report)

    # 3. cancellation: eight positive and eight negative products of nearly equal size, C close to minus their sum
    for spread in (0, 6):
        A = mant(rng, (n, 32, 16), False) * (2.0 ** rng.integers(-spread, 1, size=(n, 32, 16))).astype(np.float32)
        A[:, :, 8:] *= -1.0
        Bt = mant(rng, (n, 32, 16), False)
        s = np.einsum("tik,tjk->tij", A.astype(np.float64), Bt.astype(np.float64))
        C = (-s * (1.0 + rng.normal(size=s.shape) * 1e-3)).astype(np.float32)
        A, Bt = shuffle_k(rng, A.copy(), Bt.copy())
        run_case(som, f"cancellation spread 2^{spread}", A, Bt, C, report)

    # 4. one dominant product, fifteen small ones of mixed sign at column-dependent depth, C anywhere
    for cexp in (-20, -8, 0, 8):
        A = mant(rng, (n, 32, 16), False) * rng.choice([-1.0, 1.0], size=(n, 32, 16)).astype(np.float32)
        depth = 8.0 + (np.arange(32) % 16) * 1.25
        Bt = mant(rng, (n, 32, 16), True) * (2.0 ** -np.floor(depth))[None, :, None].astype(np.float32)
        Bt[:, :, 0] = mant(rng, (n, 32), True)
        Bt = to_bf16(Bt)
        C = ((1.0 + rng.integers(0, 2 ** 23, size=(n, 32, 32)) / 2.0 ** 23) * 2.0 ** cexp
             * rng.choice([-1.0, 1.0], size=(n, 32, 32))).astype(np.float32)
        A, Bt = shuffle_k(rng, A.copy(), Bt.copy())
        run_case(som, f"one dominant, C~2^{cexp}", A, Bt, C, report)

    # 5. the search's own regime: random operands, exponents spread over 2^spread, C of the order of the sum or larger
    for spread in (0, 4, 8, 12):
        for cexp in (-8, 0, 8):
            A = to_bf16((rng.uniform(-1, 1, size=(n, 32, 16)) * 2.0 ** rng.integers(-spread, 1, size=(n, 32, 16))).astype(np.float32))
            Bt = to_bf16((rng.uniform(-1, 1, size=(n, 32, 16)) * 2.0 ** rng.integers(-spread, 1, size=(n, 32, 16))).astype(np.float32))
            A = np.where(np.abs(A) < 2.0 ** -(spread + 4), np.float32(2.0 ** -(spread + 4)), A).astype(np.float32)
            Bt = np.where(np.abs(Bt) < 2.0 ** -(spread + 4), np.float32(2.0 ** -(spread + 4)), Bt).astype(np.float32)
            C = (rng.uniform(-1, 1, size=(n, 32, 32)) * 2.0 ** cexp).astype(np.float32)
            run_case(som, f"random spread 2^{spread}, C~2^{cexp}", A, Bt, C, report)

    worst = max(r[1] for r in report)
    print(f"largest error over {sum(r[4] for r in report)} outputs: {worst:.3f} units; charged {UNITS_CHARGED}", flush=True)
    assert worst <= UNITS_CHARGED


def test_measurement_probes_run(som):
    """The two rate probes (sustained MFMA loop, plain streaming read) run and give plausible figures."""
    t = torch.ones(1 << 24, dtype=torch.float32, device="cuda")
    for fn in (lambda: som.som_read_probe(t), lambda: som.som_mfma_rate_probe(2, 2, 2000), lambda: som.som_mfma_rate_probe(0, 1, 2000)):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        assert 0.0 < a.elapsed_time(b) < 50.0
    from paper_2604_26555_amd import SomError
    with pytest.raises(SomError):
        som.som_mfma_rate_probe(3, 2, 10)
