"""Comparison rules between the HIP path and the CPU oracle.

Logits: elementwise, |err| <= 2e-2 for bf16 storage, <= 1e-4 * max(1, |z|) for float32.
Index sets and draft tokens are integer results decided by floating-point scores that the two
sides accumulate in different orders, so they are compared exactly wherever the oracle's
score gap exceeds the tolerance and for validity inside the tolerance band.
"""
import numpy as np

TOL_BF16 = 2e-2
RTOL_F32 = 1e-4
# The tight band for selections on bf16 storage: the two sides' float32 scores differ by ~1e-6, except where
# their float32 h' values straddle a bf16 rounding boundary (one element of h' then moves by one bf16 ulp and
# every score by |W_vocab[v, j]| * ulp, ~1e-4 at the configurations' magnitudes).  Set differences must stay
# inside this band in number; the benchmark spec's tolerance above bounds them in value.
TOL_S_BF16 = 1e-3


def logits_tol(dtype: str, ref: np.ndarray) -> np.ndarray:
    if dtype == "bf16":
        return np.full_like(ref, TOL_BF16, dtype=np.float64)
    return RTOL_F32 * np.maximum(1.0, np.abs(ref))


def assert_logits_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = "logits"):
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    err = np.abs(got - ref)
    tol = logits_tol(dtype, ref)
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond tolerance, max err {err.max():.3e}"
    return float(err.max())


def score_tol(dtype: str, tau: float) -> float:
    return TOL_BF16 if dtype == "bf16" else RTOL_F32 * max(1.0, abs(tau))


def check_selected_set(got_idx: np.ndarray, s_ref: np.ndarray, ref_idx: np.ndarray, k: int, dtype: str,
                       tight: bool = False):
    """One row.  got_idx: the HIP result; s_ref: the oracle's full score vector; ref_idx: the
    oracle's set.  Returns (band population, number of ids that differ from the oracle's set); with
    tight=True (bf16 storage at the configurations' magnitudes) also asserts that no more ids differ than
    scores lie within TOL_S_BF16 of the k-th one, and returns (band, diff, tight band population, ids that
    differ and lie outside the tight band)."""
    V = s_ref.shape[0]
    got_idx = np.asarray(got_idx)
    assert got_idx.shape == (k,)
    assert got_idx.min() >= 0 and got_idx.max() < V
    assert np.all(np.diff(got_idx) > 0), "ids must be unique and ascending"
    tau = np.sort(s_ref)[V - k]
    tol = score_tol(dtype, tau)
    member = np.zeros(V, dtype=bool)
    member[got_idx] = True
    must = s_ref > tau + tol
    never = s_ref < tau - tol
    assert member[must].all(), "a token clearly above the k-th score is missing"
    assert not member[never].any(), "a token clearly below the k-th score was selected"
    band = int(((s_ref >= tau - tol) & (s_ref <= tau + tol)).sum())
    diff = int(np.setdiff1d(got_idx, ref_idx).size)
    if band == 1:
        assert diff == 0, "no other score near the k-th one: the set must equal the oracle's"
    if not tight:
        return band, diff
    tol_s = TOL_S_BF16 if dtype == "bf16" else tol
    in_tight = (s_ref >= tau - tol_s) & (s_ref <= tau + tol_s)
    band_s = int(in_tight.sum())
    assert diff <= band_s, f"{diff} ids differ from the oracle's set, only {band_s} scores lie within {tol_s} of the k-th"
    ref_member = np.zeros(V, dtype=bool)
    ref_member[ref_idx] = True
    outside = int(((member != ref_member) & ~in_tight).sum())
    return band, diff, band_s, outside


def check_draft_tokens(got_tok, got_prob, z_ref_row, idx_row, ref_tok, ref_prob, dtype: str):
    """One row of the end-to-end draft top-kd, where each side ranks ITS OWN logits.  z_ref_row: the
    oracle's subset logits.  If the two sides' logits differ by at most tol element by element, the t-th
    largest values of the two vectors differ by at most tol as well, so the ORACLE logit of the token the
    HIP side puts at position t lies within 2 tol of the oracle's t-th logit; it must be the very token
    wherever the neighbouring oracle gaps exceed 2 tol.  Probabilities: p = exp(z - lse), both z and lse
    move by at most tol, so p agrees to a factor exp(2 tol)."""
    kd = len(ref_tok)
    pos = {int(t): j for j, t in enumerate(idx_row)}
    order = np.sort(z_ref_row)[::-1]
    assert len(set(int(t) for t in got_tok)) == kd, "draft tokens must be distinct"
    for t in range(kd):
        assert int(got_tok[t]) in pos, "draft token outside the subset"
        zt = z_ref_row[pos[int(got_tok[t])]]
        tol = TOL_BF16 if dtype == "bf16" else RTOL_F32 * max(1.0, abs(order[t]))
        assert abs(zt - order[t]) <= 2 * tol, (t, zt, order[t])
        gap_up = order[t - 1] - order[t] if t > 0 else np.inf
        gap_dn = order[t] - order[t + 1] if t + 1 < len(order) else np.inf
        if gap_up > 2 * tol and gap_dn > 2 * tol:
            assert int(got_tok[t]) == int(ref_tok[t]), (t, got_tok, ref_tok)
            assert abs(got_prob[t] - ref_prob[t]) <= 1e-5 + np.expm1(2 * tol) * ref_prob[t]
