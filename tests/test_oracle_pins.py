"""Pins for the CPU oracle: every check here compares the oracle with something that is not
the oracle -- a hand-worked example, a closed form, a library routine (numpy float64
matmul / argsort, torch's bf16 cast), brute-force enumeration, or an identity that the
paper's definitions imply (Section 3.1, Section 3.3, Table 4).  CPU only.
"""
import math
import os

import numpy as np
import pytest

import oracle
from workloads import bf16_bits_to_f32, f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers
def _as(dtype, x):
    x = np.asarray(x, dtype=np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def _f64(a):
    """Exact float64 view of a stored matrix."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def _rand(rng, shape, std, dtype):
    return _as(dtype, rng.standard_normal(shape).astype(np.float32) * np.float32(std))


def _parse_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":", 1)
            rows = [[float(t) for t in part.split()] for part in val.split("|")]
            out[key.strip()] = np.array(rows if len(rows) > 1 else rows[0], dtype=np.float64)
    return out


def _brute_topk(s, k):
    """Rank counting, no sort: v is kept iff fewer than k tokens beat it
    (larger score, or equal score and smaller id)."""
    V = len(s)
    keep = []
    for v in range(V):
        beat = sum(1 for u in range(V) if s[u] > s[v] or (s[u] == s[v] and u < v))
        if beat < k:
            keep.append(v)
    return np.array(keep, dtype=np.int32)


# ------------------------------------------------------------------ P10 hand example
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("acc", ["f32", "f64"])
def test_hand_example(dtype, acc):
    g = _parse_golden(os.path.join(GOLDEN, "hand_example.txt"))
    h, U = _as(dtype, g["h"]), _as(dtype, g["U"])
    Wd, Wv = _as(dtype, g["W_down"]), _as(dtype, g["W_vocab"])
    k, kd = int(g["k"][0]), int(g["kd"][0])
    idx, sc, s_full, hp = oracle.select(h, Wd, Wv, k, acc=acc, full=True)
    assert np.array_equal(hp[0], g["expect_hprime"])
    assert np.array_equal(s_full[0], g["expect_s"])
    assert np.array_equal(idx[0], g["expect_idx"].astype(np.int32))
    assert np.array_equal(sc[0], g["expect_s"][idx[0]])
    assert np.array_equal(oracle.dense_logits(h, U, acc=acc)[0], g["expect_z"])
    zsub = oracle.subset_logits(h, U, idx, acc=acc)
    assert np.array_equal(zsub[0], g["expect_zsub"])
    tok, prob = oracle.softmax_topk(zsub, idx, kd)
    assert np.array_equal(tok[0], g["expect_tok"].astype(np.int32))
    assert np.allclose(prob[0], g["expect_prob"], rtol=0, atol=float(g["expect_prob_tol"][0]))


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_hot_rows_closed_form(dtype):
    """U[v, i] = (v % 7 + 1) if i == v % d else 0  =>  z[r, v] = (v % 7 + 1) * h[r, v % d].
    A wrong row/column index, a transposed operand or a wrong stride breaks it."""
    d, V, rows = 24, 101, 3
    U = np.zeros((V, d), dtype=np.float32)
    for v in range(V):
        U[v, v % d] = v % 7 + 1
    h = (np.arange(rows * d, dtype=np.float32).reshape(rows, d) % 11) - 5.0
    expect = np.array([[(v % 7 + 1) * h[r, v % d] for v in range(V)] for r in range(rows)])
    for acc in ("f32", "f64"):
        assert np.array_equal(oracle.dense_logits(_as(dtype, h), _as(dtype, U), acc=acc), expect)
        idx = np.array([[100, 3, 50, 24], [0, 1, 2, 99], [77, 76, 5, 23]], dtype=np.int32)
        got = oracle.subset_logits(_as(dtype, h), _as(dtype, U), idx, acc=acc)
        assert np.array_equal(got, np.take_along_axis(expect, idx.astype(np.int64), axis=1))
        shared = np.array([9, 100, 42], dtype=np.int32)
        got = oracle.subset_logits(_as(dtype, h), _as(dtype, U), shared, acc=acc)
        assert np.array_equal(got, expect[:, shared])


def test_softmax_geometric_series_closed_form():
    """z_j = j ln 2  =>  q_j = 2^j / (2^k - 1) (geometric series); top-kd are the last kd."""
    k, kd = 12, 5
    z = (np.arange(k) * math.log(2.0)).astype(np.float32)
    idx = np.arange(100, 100 + k, dtype=np.int32)
    tok, prob, q = oracle.softmax_topk(z, idx, kd, full=True)
    expect = np.array([2.0 ** j / (2.0 ** k - 1) for j in range(k)])
    assert np.allclose(q[0], expect, rtol=2e-6, atol=0)  # z is ln2*j rounded to float32
    assert abs(q.sum() - 1.0) < 1e-12
    assert list(tok[0]) == [100 + k - 1 - t for t in range(kd)]
    assert np.allclose(prob[0], expect[::-1][:kd], rtol=2e-6)


def test_softmax_uniform_and_shift_invariance():
    k = 37
    idx = np.arange(k, dtype=np.int32)[::-1].copy()
    _, _, q = oracle.softmax_topk(np.full(k, 3.25, np.float32), idx, 1, full=True)
    assert np.allclose(q, 1.0 / k, rtol=1e-15)
    rng = np.random.default_rng(5)
    z = rng.standard_normal(k).astype(np.float32)
    z = np.round(z * 64) / 64  # so that z + 8 is exact in float32
    _, _, q0 = oracle.softmax_topk(z, idx, 1, full=True)
    _, _, q1 = oracle.softmax_topk(z + np.float32(8.0), idx, 1, full=True)
    assert np.allclose(q0, q1, rtol=1e-13)
    # a row whose logits are all negative is an ordinary row, not an empty one
    _, _, qn = oracle.softmax_topk(z - np.float32(8.0), idx, 1, full=True)
    assert np.allclose(q0, qn, rtol=1e-13) and abs(qn.sum() - 1.0) < 1e-12
    # huge logits must not overflow (max is subtracted)
    _, p = oracle.softmax_topk(np.array([1e4, 1e4 - 1.0], np.float32), np.array([3, 9], np.int32), 2)
    assert np.allclose(p[0], [1 / (1 + math.exp(-1)), math.exp(-1) / (1 + math.exp(-1))], rtol=1e-12)


# ------------------------------------------------------------------ P7 library routines
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_against_numpy_float64(dtype):
    """The indexed LM head as a library computes it: U[idx] @ h in float64 (Figure 3a)."""
    rng = np.random.default_rng(11)
    rows, d, V, k, dp = 3, 80, 257, 33, 12
    U = _rand(rng, (V, d), 0.05, dtype)
    h = _rand(rng, (rows, d), 1.0, dtype)
    Wd = _rand(rng, (dp, d), 0.1, dtype)
    Wv = _rand(rng, (V, dp), 0.1, dtype)
    U64, h64, Wd64, Wv64 = _f64(U), _f64(h), _f64(Wd), _f64(Wv)

    z64 = h64 @ U64.T
    assert np.allclose(oracle.dense_logits(h, U, acc="f64"), z64, rtol=1e-12, atol=1e-14)
    assert np.allclose(oracle.dense_logits(h, U, acc="f32"), z64, rtol=0, atol=2e-5)

    idx = np.stack([rng.permutation(V)[:k] for _ in range(rows)]).astype(np.int32)
    zs64 = np.stack([U64[idx[r]] @ h64[r] for r in range(rows)])
    assert np.allclose(oracle.subset_logits(h, U, idx, acc="f64"), zs64, rtol=1e-12, atol=1e-14)
    assert np.allclose(oracle.subset_logits(h, U, idx, acc="f32"), zs64, rtol=0, atol=2e-5)
    assert np.allclose(oracle.subset_logits(h, U, idx[0], acc="f64"), h64 @ U64[idx[0]].T,
                       rtol=1e-12, atol=1e-14)

    # selector, no intermediate rounding: s = W_vocab (W_down h)
    sel_idx, sel_sc, s_full, hp = oracle.select(h, Wd, Wv, k, hprime_round=False, acc="f64", full=True)
    hp64 = h64 @ Wd64.T
    s64 = hp64 @ Wv64.T
    assert np.allclose(hp, hp64, rtol=1e-12, atol=1e-14)
    assert np.allclose(s_full, s64, rtol=1e-11, atol=1e-14)
    for r in range(rows):
        top = np.sort(np.argsort(-s64[r], kind="stable")[:k])
        assert np.array_equal(sel_idx[r], top)
        assert np.allclose(sel_sc[r], s64[r, top], rtol=1e-11, atol=1e-14)

    # softmax / top-kd against numpy on the same float32 logits
    z32 = zs64.astype(np.float32)
    tok, prob, q = oracle.softmax_topk(z32, idx, 7, full=True)
    e = np.exp(z32.astype(np.float64) - z32.astype(np.float64).max(axis=1, keepdims=True))
    qn = e / e.sum(axis=1, keepdims=True)
    assert np.allclose(q, qn, rtol=1e-13)
    for r in range(rows):
        order = np.argsort(-z32[r], kind="stable")[:7]
        assert np.array_equal(tok[r], idx[r, order])
        assert np.allclose(prob[r], qn[r, order], rtol=1e-13)


def test_hprime_rounding_matches_torch_bf16_cast():
    """With bf16 storage the intermediate h' is rounded to bf16 (round-to-nearest-even) before
    the second projection; torch's cast is the library reference for that rounding."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    rows, d, dp, V = 2, 64, 16, 50
    h = _rand(rng, (rows, d), 1.0, "bf16")
    Wd = _rand(rng, (dp, d), 0.3, "bf16")
    Wv = _rand(rng, (V, dp), 0.3, "bf16")
    _, _, s_r, hp_r = oracle.select(h, Wd, Wv, 5, hprime_round=True, acc="f32", full=True)
    _, _, s_k, hp_k = oracle.select(h, Wd, Wv, 5, hprime_round=False, acc="f32", full=True)
    expect = torch.from_numpy(hp_k.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(hp_r, expect)
    assert not np.array_equal(hp_r, hp_k)  # the rounding is not a no-op on this input
    assert np.allclose(s_r, expect @ _f64(Wv).T, rtol=0, atol=1e-5)
    # default: round for bf16 storage, keep for float32 storage
    _, _, _, hp_def = oracle.select(h, Wd, Wv, 5, full=True)
    assert np.array_equal(hp_def, hp_r)
    hf, Wdf, Wvf = (bf16_bits_to_f32(a) for a in (h, Wd, Wv))
    _, _, _, hp_f = oracle.select(hf, Wdf, Wvf, 5, full=True)
    assert np.array_equal(hp_f, hp_k)


def test_hprime_rounding_ties_go_to_even():
    """h' = [1 + 2^-8, 1 + 3*2^-8] sit exactly half-way between bf16 neighbours: round-to-nearest-
    even gives 1.0 (not 1 + 2^-7) and 1 + 2^-6."""
    h = np.array([[1.0, 2.0 ** -8]], np.float32)
    Wd = np.array([[1.0, 1.0], [1.0, 3.0]], np.float32)
    Wv = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]], np.float32)
    _, _, s, hp = oracle.select(h, Wd, Wv, 1, hprime_round=True, full=True)
    assert list(hp[0]) == [1.0, 1.0 + 2.0 ** -6]
    assert list(s[0]) == [1.0, 1.0 + 2.0 ** -6, 2.0 + 2.0 ** -6]


def test_leading_dimensions():
    """Rows taken out of wider matrices (row stride > d) must give the same logits."""
    rng = np.random.default_rng(47)
    rows, d, V, pad = 3, 20, 31, 12
    Uw = _rand(rng, (V, d + pad), 0.1, "bf16")
    hw = _rand(rng, (rows, d + 4), 1.0, "bf16")
    U, h = Uw[:, :d], hw[:, :d]
    assert not U.flags.c_contiguous
    z = oracle.dense_logits(h, U, acc="f64")
    assert np.allclose(z, _f64(np.ascontiguousarray(h)) @ _f64(np.ascontiguousarray(U)).T, rtol=1e-12)
    idx = np.array([[30, 0, 7]] * rows, dtype=np.int32)
    assert np.array_equal(oracle.subset_logits(h, U, idx, acc="f64"), z[:, [30, 0, 7]])
    Wd = _rand(rng, (4, d), 0.1, "bf16")
    Wv = _rand(rng, (V, 4), 0.1, "bf16")
    a = oracle.select(h, Wd, Wv, 5, full=True)
    b = oracle.select(np.ascontiguousarray(h), Wd, Wv, 5, full=True)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


# ------------------------------------------------------------------ brute force on tiny inputs
def test_select_brute_force_with_ties():
    rng = np.random.default_rng(17)
    for trial in range(20):
        d, dp, V = 4, 3, int(rng.integers(2, 24))
        k = int(rng.integers(1, V + 1))
        # small integers: exact arithmetic and many tied scores
        h = rng.integers(-2, 3, size=(1, d)).astype(np.float32)
        Wd = rng.integers(-1, 2, size=(dp, d)).astype(np.float32)
        Wv = rng.integers(-1, 2, size=(V, dp)).astype(np.float32)
        s = (Wv.astype(np.int64) @ (Wd.astype(np.int64) @ h[0].astype(np.int64)))
        idx, sc = oracle.select(h, Wd, Wv, k)
        assert np.array_equal(idx[0], _brute_topk(list(s), k)), (trial, s, k)
        assert np.array_equal(sc[0], s[idx[0]])


def test_draft_topk_brute_force_with_ties():
    rng = np.random.default_rng(19)
    for trial in range(20):
        k = int(rng.integers(1, 20))
        kd = int(rng.integers(1, k + 1))
        z = rng.integers(-2, 3, size=k).astype(np.float32)
        idx = rng.permutation(50)[:k].astype(np.int32)
        tok, prob = oracle.softmax_topk(z, idx, kd)
        # enumerate: position t holds the token beaten by exactly t others
        expect = [None] * k
        for a in range(k):
            beat = sum(1 for b in range(k) if z[b] > z[a] or (z[b] == z[a] and idx[b] < idx[a]))
            expect[beat] = (idx[a], z[a])
        assert [t for t, _ in expect[:kd]] == list(tok[0])
        den = sum(math.exp(float(v) - float(z.max())) for v in z)
        assert np.allclose(prob[0], [math.exp(float(v) - float(z.max())) / den for _, v in expect[:kd]],
                           rtol=1e-13)


def test_tie_break_prefers_smaller_token_id():
    """Duplicated rows of W_vocab / U give bit-identical scores; the smaller id must win."""
    rng = np.random.default_rng(23)
    d, dp, V = 16, 4, 12
    h = _rand(rng, (1, d), 1.0, "bf16")
    Wd = _rand(rng, (dp, d), 0.2, "bf16")
    Wv = _rand(rng, (V, dp), 0.2, "bf16")
    Wv[:] = Wv[0]                       # all scores identical
    for k in (1, 5, V):
        idx, _ = oracle.select(h, Wd, Wv, k)
        assert list(idx[0]) == list(range(k))
    z = np.full(6, 1.5, np.float32)
    tok, _ = oracle.softmax_topk(z, np.array([40, 7, 19, 3, 88, 5], np.int32), 4)
    assert list(tok[0]) == [3, 5, 7, 19]


# ------------------------------------------------------------------ identities from the definitions
@pytest.fixture(scope="module")
def tiny():
    """Config-1-shaped case (d=256, V=8192, float32, k=512) kept small enough for the CPU suite."""
    from workloads import CONFIGS, make_rng, zipf_subset
    c = CONFIGS[1]
    U = c.weights()
    h = c.hidden(2).reshape(2, c.d)
    rng = make_rng(1, 2)
    idx = np.stack([zipf_subset(rng, c.V, c.k) for _ in range(2)])
    return c, U, h, idx


def test_p1_subset_is_slice_of_dense(tiny):
    c, U, h, idx = tiny
    for acc in ("f32", "f64"):
        z = oracle.dense_logits(h, U, acc=acc)
        zs = oracle.subset_logits(h, U, idx, acc=acc)
        assert np.array_equal(zs, np.take_along_axis(z, idx.astype(np.int64), axis=1))
    z32, z64 = oracle.dense_logits(h, U, acc="f32"), oracle.dense_logits(h, U, acc="f64")
    assert np.abs(z32 - z64).max() < 1e-5          # float32 accumulation error at this scale
    assert np.allclose(z64, h.astype(np.float64) @ U.astype(np.float64).T, rtol=1e-12, atol=1e-14)


def test_p2_subset_all_v_is_dense(tiny):
    c, U, h, _ = tiny
    allv = np.arange(c.V, dtype=np.int32)
    z = oracle.dense_logits(h, U)
    assert np.array_equal(oracle.subset_logits(h, U, allv), z)
    tok, prob, q = oracle.softmax_topk(z, allv, c.kd, full=True)
    z32 = z.astype(np.float32).astype(np.float64)
    e = np.exp(z32 - z32.max(axis=1, keepdims=True))
    qn = e / e.sum(axis=1, keepdims=True)
    assert np.allclose(q, qn, rtol=1e-12)
    for r in range(h.shape[0]):
        assert np.array_equal(tok[r], np.argsort(-z32[r], kind="stable")[:c.kd])


def test_p3_permutation_equivariance(tiny):
    c, U, h, idx = tiny
    rng = np.random.default_rng(29)
    perm = rng.permutation(c.k)
    z0 = oracle.subset_logits(h, U, idx)
    z1 = oracle.subset_logits(h, U, idx[:, perm])
    assert np.array_equal(z1, z0[:, perm])
    t0, p0 = oracle.softmax_topk(z0, idx, c.kd)
    t1, p1 = oracle.softmax_topk(z1, idx[:, perm], c.kd)
    assert np.array_equal(t0, t1)
    assert np.allclose(p0, p1, rtol=1e-12)


def test_p4_renormalisation(tiny):
    """q_K(x) = q(x) / sum_{y in K} q(y): the subset softmax is the full softmax renormalised."""
    c, U, h, idx = tiny
    z = oracle.dense_logits(h, U)
    _, _, q_full = oracle.softmax_topk(z, np.arange(c.V, dtype=np.int32), 1, full=True)
    zs = oracle.subset_logits(h, U, idx)
    _, _, q_sub = oracle.softmax_topk(zs, idx, 1, full=True)
    for r in range(h.shape[0]):
        qk = q_full[r, idx[r]]
        assert np.allclose(q_sub[r], qk / qk.sum(), rtol=1e-10)
        assert abs(q_sub[r].sum() - 1.0) < 1e-12


def test_p5_coverage_gives_full_vocab_draft(tiny):
    c, U, h, idx = tiny
    z = oracle.dense_logits(h, U)
    full_tok, _ = oracle.softmax_topk(z, np.arange(c.V, dtype=np.int32), c.kd)
    for r in range(h.shape[0]):
        K = np.union1d(idx[r], full_tok[r]).astype(np.int32)      # K covers the true top-kd
        zs = oracle.subset_logits(h[r:r + 1], U, K[None, :])
        tok, _ = oracle.softmax_topk(zs, K[None, :], c.kd)
        assert np.array_equal(tok[0], full_tok[r])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p6_exact_selector_reduces_to_lm_head(dtype):
    """d' = d, W_down = I, W_vocab = U  =>  s = z and select is the exact top-k of the logits."""
    rng = np.random.default_rng(31)
    d, V, k, kd = 32, 300, 40, 6
    U = _rand(rng, (V, d), 0.1, dtype)
    h = _rand(rng, (2, d), 1.0, dtype)
    eye = _as(dtype, np.eye(d, dtype=np.float32))
    idx, sc, s_full, hp = oracle.select(h, eye, U, k, full=True)
    z = oracle.dense_logits(h, U)
    assert np.array_equal(hp, _f64(h))              # identity projection, and bf16 rounding is a no-op
    assert np.array_equal(s_full, z)
    for r in range(2):
        assert np.array_equal(idx[r], np.sort(np.argsort(-z[r], kind="stable")[:k]))
    tok_sub, _ = oracle.softmax_topk(oracle.subset_logits(h, U, idx), idx, kd)
    tok_full, _ = oracle.softmax_topk(z, np.arange(V, dtype=np.int32), kd)
    assert np.array_equal(tok_sub, tok_full)


def test_p8_operation_counts():
    """Table 4: full vocabulary V*d; SpecVocab V*d' + k*d (plus d*d' for the down-projection,
    which the table leaves out) multiply-accumulates per row."""
    rng = np.random.default_rng(37)
    rows, d, dp, V, k = 3, 48, 6, 200, 17
    U = _rand(rng, (V, d), 0.1, "bf16")
    h = _rand(rng, (rows, d), 1.0, "bf16")
    Wd = _rand(rng, (dp, d), 0.1, "bf16")
    Wv = _rand(rng, (V, dp), 0.1, "bf16")
    oracle.reset_mac_count()
    oracle.dense_logits(h, U)
    assert oracle.mac_count() == rows * V * d
    oracle.dense_logits(h, U, acc="f64")                   # the float64 cross-check counts alike
    assert oracle.mac_count() == 2 * rows * V * d
    oracle.reset_mac_count()
    idx, _ = oracle.select(h, Wd, Wv, k)
    assert oracle.mac_count() == rows * (V * dp + d * dp)
    oracle.subset_logits(h, U, idx)
    assert oracle.mac_count() == rows * (V * dp + d * dp + k * d)
    # the paper's break-even: V*d'/d + k < |V'|
    assert V * dp / d + k < V


def test_p9_degenerate_k():
    rng = np.random.default_rng(41)
    d, dp, V = 20, 5, 64
    h = _rand(rng, (2, d), 1.0, "f32")
    Wd = _rand(rng, (dp, d), 0.3, "f32")
    Wv = _rand(rng, (V, dp), 0.3, "f32")
    _, _, s, _ = oracle.select(h, Wd, Wv, 1, full=True)
    i1, _ = oracle.select(h, Wd, Wv, 1)
    assert np.array_equal(i1[:, 0], s.argmax(axis=1))
    iv, _ = oracle.select(h, Wd, Wv, V)
    assert np.array_equal(iv, np.tile(np.arange(V, dtype=np.int32), (2, 1)))
    z = rng.standard_normal((1, 9)).astype(np.float32)
    idx = rng.permutation(30)[:9].astype(np.int32)
    tok, prob = oracle.softmax_topk(z, idx[None], 9)           # kd = k: a full sort
    assert np.array_equal(tok[0], idx[np.argsort(-z[0], kind="stable")])
    assert abs(prob.sum() - 1.0) < 1e-12
    assert np.all(np.diff(prob[0]) <= 0)


def test_uses_original_hidden_state_in_step3():
    """Step 3 uses h_t, not h': the subset logits must not depend on the selector at all."""
    rng = np.random.default_rng(43)
    d, V = 24, 90
    U = _rand(rng, (V, d), 0.1, "bf16")
    h = _rand(rng, (1, d), 1.0, "bf16")
    idx = np.array([[3, 50, 89]], dtype=np.int32)
    z = oracle.subset_logits(h, U, idx)
    assert np.allclose(z[0], _f64(U)[idx[0]] @ _f64(h)[0], atol=1e-5)


def test_error_paths():
    h = np.zeros((1, 4), np.float32)
    U = np.zeros((6, 4), np.float32)
    with pytest.raises(RuntimeError):
        oracle.subset_logits(h, U, np.array([[0, 6]], np.int32))
    with pytest.raises(RuntimeError):
        oracle.subset_logits(h, U, np.array([[-2]], np.int32))      # -1 alone is the padding slot
    with pytest.raises(RuntimeError):
        oracle.select(h, np.zeros((2, 4), np.float32), np.zeros((6, 2), np.float32), 7)
    with pytest.raises(TypeError):
        oracle.dense_logits(h, U.astype(np.float64))
    with pytest.raises(TypeError):
        oracle.dense_logits(h, np.zeros((6, 4), np.uint16))


# --------------------------------------------------------------------------
# Section 3.4: q_aux = softmax(s) over the entire vocabulary, as log-probabilities
# --------------------------------------------------------------------------
def test_log_softmax_closed_form():
    """s = (0, ln 2, ln 3)  =>  q_aux = (1/6, 2/6, 3/6)."""
    out = oracle.log_softmax(np.array([[0.0, math.log(2.0), math.log(3.0)]]))
    want = np.log(np.array([[1.0, 2.0, 3.0]]) / 6.0)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-15)
    # equal scores: the uniform distribution, also where exp(s) itself would overflow
    out = oracle.log_softmax(np.full((2, 5), 1000.0))
    np.testing.assert_allclose(out, np.full((2, 5), -math.log(5.0)), rtol=0, atol=1e-12)


def test_log_softmax_against_scipy_and_invariants():
    from scipy.special import log_softmax as scipy_log_softmax, logsumexp
    rng = np.random.default_rng(34)
    s = rng.normal(0.0, 3.0, size=(4, 1000))
    out = oracle.log_softmax(s)
    np.testing.assert_allclose(out, scipy_log_softmax(s, axis=1), rtol=0, atol=1e-12)
    np.testing.assert_allclose(logsumexp(out, axis=1), 0.0, atol=1e-12)          # probabilities sum to one
    np.testing.assert_allclose(oracle.log_softmax(s + 7.25), out, atol=1e-12)     # shift invariance
    assert np.array_equal(out.argmax(axis=1), s.argmax(axis=1))
    # differences of log-probabilities are differences of scores
    np.testing.assert_allclose(out[:, 1:] - out[:, :-1], s[:, 1:] - s[:, :-1], atol=1e-12)


def test_q_aux_restricted_to_a_subset_is_the_subset_softmax():
    """Renormalising q_aux over a subset K gives softmax(s[K]) -- the same function the subset softmax of
    Section 3.3 computes on logits."""
    rng = np.random.default_rng(35)
    s = rng.normal(0.0, 2.0, size=(2, 300)).astype(np.float32)
    K = np.sort(rng.permutation(300)[:40]).astype(np.int32)
    logq = oracle.log_softmax(s.astype(np.float64))
    q_sub = np.exp(logq[:, K])
    q_sub /= q_sub.sum(axis=1, keepdims=True)
    _, _, q_K = oracle.softmax_topk(s[:, K], K, 5, full=True)
    np.testing.assert_allclose(q_sub, q_K, rtol=1e-12, atol=0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_aux_log_softmax_composes_the_selector_scores(dtype):
    """log q_aux = log softmax(W_vocab (W_down h)): against numpy float64 on the widened inputs, with h'
    rounded through bf16 exactly where select rounds it."""
    rng = np.random.default_rng(36)
    d, dp, V = 64, 16, 200
    def draw(shape, scale):
        a = rng.normal(0.0, scale, size=shape).astype(np.float32)
        return f32_to_bf16_bits(a) if dtype == "bf16" else a
    def wide(a):
        return bf16_bits_to_f32(a).astype(np.float64) if dtype == "bf16" else a.astype(np.float64)
    h, Wd, Wv = draw((3, d), 1.0), draw((dp, d), 0.2), draw((V, dp), 0.2)
    hp = wide(h) @ wide(Wd).T
    if dtype == "bf16":
        hp = bf16_bits_to_f32(f32_to_bf16_bits(hp.astype(np.float32))).astype(np.float64)
    s = hp @ wide(Wv).T
    want = s - s.max(axis=1, keepdims=True)
    want = want - np.log(np.exp(want).sum(axis=1, keepdims=True))
    got = oracle.aux_log_softmax(h, Wd, Wv, acc="f64")
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-9)
    # the float32-accumulated variant stays within accumulation noise of it
    np.testing.assert_allclose(oracle.aux_log_softmax(h, Wd, Wv), want, rtol=0, atol=2e-5 if dtype == "f32" else 2e-2)


# --------------------------------------------------------------------------
# Variable subset sizes inside fixed-size lists: padding slots (-1) and a score threshold.
# Section 3.3 Step 2 only says that k may vary; the encoding is this implementation's, so the pins
# are its defining properties: padding changes nothing for the real entries, and a padded list
# behaves as the compacted list of its real entries.
# --------------------------------------------------------------------------
def test_padding_slots_in_subset_logits_and_softmax():
    rng = np.random.default_rng(41)
    d, V, k, kd = 32, 200, 30, 6
    h = rng.normal(size=(2, d)).astype(np.float32)
    U = rng.normal(scale=0.3, size=(V, d)).astype(np.float32)
    idx = np.stack([rng.permutation(V)[:k] for _ in range(2)]).astype(np.int32)
    pad = idx.copy()
    holes = [np.array([0, 7, 8, 29]), np.array([3, 4, 5, 6, 20])]
    for r in range(2):
        pad[r, holes[r]] = -1
    z, zp = oracle.subset_logits(h, U, idx), oracle.subset_logits(h, U, pad)
    for r in range(2):
        real = np.setdiff1d(np.arange(k), holes[r])
        assert np.array_equal(zp[r, real], z[r, real])                  # real entries untouched
        assert np.all(np.isneginf(zp[r, holes[r]]))                     # padding: logit -inf
        # the padded list behaves as the compacted list of its real entries
        tok_p, prob_p, q_p = oracle.softmax_topk(zp[r:r + 1], pad[r:r + 1], kd, full=True)
        tok_c, prob_c, q_c = oracle.softmax_topk(z[r:r + 1, real], idx[r:r + 1, real], kd, full=True)
        assert np.array_equal(tok_p, tok_c)
        np.testing.assert_allclose(prob_p, prob_c, rtol=1e-14)
        np.testing.assert_allclose(q_p[0, real], q_c[0], rtol=1e-14)
        assert np.all(q_p[0, holes[r]] == 0.0)


def test_fewer_real_entries_than_draft_tokens_and_empty_rows():
    z = np.array([[1.0, -np.inf, 0.0, -np.inf], [-np.inf] * 4], dtype=np.float32)
    idx = np.array([[5, -1, 9, -1], [-1, -1, -1, -1]], dtype=np.int32)
    tok, prob, q = oracle.softmax_topk(z, idx, 3, full=True)
    e = math.exp(-1.0)
    assert tok[0].tolist() == [5, 9, -1]
    np.testing.assert_allclose(prob[0], [1 / (1 + e), e / (1 + e), 0.0], rtol=1e-15)
    assert tok[1].tolist() == [-1, -1, -1] and np.all(prob[1] == 0.0) and np.all(q[1] == 0.0)


def test_score_threshold_pads_the_selected_list_in_place():
    rng = np.random.default_rng(42)
    d, dp, V, k = 24, 8, 300, 40
    h = rng.normal(size=(3, d)).astype(np.float32)
    Wd = rng.normal(scale=0.3, size=(dp, d)).astype(np.float32)
    Wv = rng.normal(scale=0.3, size=(V, dp)).astype(np.float32)
    idx, sc = oracle.select(h, Wd, Wv, k)
    tau = float(np.median(sc))                                          # keeps about half of each list
    idx_t, sc_t = oracle.select(h, Wd, Wv, k, tau=tau)
    keep = sc >= tau
    assert np.array_equal(idx_t, np.where(keep, idx, -1))
    assert np.array_equal(sc_t, np.where(keep, sc, -np.inf))
    assert 0 < keep.sum() < keep.size
    # the threshold is inclusive: a token scoring exactly tau stays
    tau_eq = float(sc[1, 7])
    idx_e, sc_e = oracle.select(h, Wd, Wv, k, tau=tau_eq)
    assert idx_e[1, 7] == idx[1, 7] and sc_e[1, 7] == tau_eq
    assert np.array_equal(idx_e, np.where(sc >= tau_eq, idx, -1))
    # tau = -inf is the plain selection; tau above every score empties the lists
    assert np.array_equal(oracle.select(h, Wd, Wv, k, tau=-np.inf)[0], idx)
    assert np.all(oracle.select(h, Wd, Wv, k, tau=1e30)[0] == -1)

