"""GPU parity: the HIP library (through its C ABI binding) against the CPU oracle on the same
seeded inputs.  Small shapes cover several tiles, ragged tails and the degenerate cases; the
full-size cases run in the launch configuration the benchmark times."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_13836_amd as sv
from compare import (assert_logits_close, check_draft_tokens, check_selected_set)
from workloads import CONFIGS, f32_to_bf16_bits, make_rng, tree_subsets, zipf_subset

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def rand(rng, shape, std, dtype):
    x = rng.standard_normal(shape).astype(np.float32) * np.float32(std)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------- subset / dense logits
LOGIT_SHAPES = [
    # dtype, rows, d,    V,    k,    mode
    ("f32", 1, 256, 8192, 512, "per_row"),       # config 1
    ("bf16", 1, 256, 8192, 512, "per_row"),
    ("bf16", 3, 264, 1000, 77, "per_row"),       # 33 16-byte units: ragged last load
    ("bf16", 2, 3840, 3000, 333, "per_step"),    # Gemma-style d, 7.5 KiB rows
    ("bf16", 5, 4096, 2048, 1, "per_row"),       # k = 1
    ("bf16", 2, 520, 301, 301, "per_step"),      # k = V
    ("bf16", 1, 8192, 600, 129, "per_row"),      # 16 loads per lane
    ("bf16", 2, 8200, 300, 50, "per_row"),       # longer than 16 KiB: the kernel that walks a row in pieces
    ("f32", 2, 260, 500, 64, "per_row"),
    ("f32", 1, 4096, 700, 100, "per_step"),      # 16 loads per lane, float32
    ("f32", 2, 4100, 300, 33, "per_row"),        # long-row path, float32
    ("f32", 70, 260, 500, 64, "per_row"),        # float32 has no matrix-core path: one launch row by row
    ("bf16", 7, 1024, 5000, 1000, "per_row"),
    # one row per wavefront, hidden row in LDS: rows of 3 to 16 KiB, whole and ragged numbers of 1 KiB pieces
    ("bf16", 1, 3840, 3000, 333, "per_row"),     # 480 units: 8 loads per lane, the last one half empty
    ("bf16", 3, 1544, 900, 200, "per_row"),      # 193 units: 4 loads per lane, the last one a single unit
    ("f32", 1, 2052, 700, 100, "per_row"),       # 513 units: 9 loads per lane
    ("bf16", 1, 8184, 500, 129, "per_row"),      # 1023 units: 16 loads per lane, one unit short
    ("bf16", 2, 5120, 800, 300, "per_row"),      # 640 units: 10 whole loads per lane
    ("bf16", 1, 3584, 600, 100, "per_row"),      # 448 units: 7 whole loads per lane
    ("f32", 1, 1536, 601, 601, "per_step"),      # 384 units: 6 whole loads per lane, k = V, odd item count
    ("bf16", 4, 8192, 30000, 13000, "per_row"),  # few rows, enough gathered bytes for the union-of-sets path
    ("bf16", 16, 1024, 6000, 1100, "per_row"),   # 16 rows: union-of-sets path
    ("bf16", 60, 520, 3000, 600, "per_row"),     # a tree's worth of rows, ragged reduction slice
    ("bf16", 70, 256, 4000, 300, "per_row"),     # more than 64 hidden rows, sets that cover the vocabulary (128-item tiles)
    ("bf16", 33, 3840, 2500, 2500, "per_row"),   # every row asks for the whole vocabulary
    ("bf16", 64, 1024, 9000, 77, "per_step"),    # 64 rows, one shared set
    ("bf16", 17, 4096, 1500, 1500, "per_step"),
    ("bf16", 60, 2048, 20000, 9000, "per_step"), # 60 rows, few items, long rows: reduction split, two row groups
    ("bf16", 40, 2048, 40000, 20000, "per_step"),# mid-size shared set: widest skinny workgroups
    ("bf16", 65, 1024, 3000, 700, "per_step"),   # more than 64 rows: LDS-tiled matrix-core kernel, ragged tiles
    ("bf16", 130, 200, 1111, 1111, "per_step"),  # three row tiles (last one 2 rows), 25 units: ragged last slice
    ("bf16", 200, 4096, 2000, 129, "per_step"),  # one item tile plus one item
    ("bf16", 150, 512, 5000, 900, "per_row"),    # 150 unsorted sets that cover the vocabulary: grouped by tile, pick epilogue
    ("bf16", 150, 512, 50000, 300, "per_row"),   # 150 sets that do not: union of the sets on the tiled kernel
    ("bf16", 300, 256, 70000, 900, "per_row"),   # 256 x 256 tiles with the pick epilogue, lists in any order, ragged last tile
    ("bf16", 70, 8, 300, 300, "per_step"),       # one 16-byte unit per row: a single, ragged reduction slice
    ("bf16", 300, 64, 100, 1, "per_step"),       # one item, three row tiles
    ("bf16", 256, 1024, 1500, 1500, "per_step"), # 256 x 256 tiles, hand-ordered main loop
    ("bf16", 300, 264, 700, 300, "per_step"),    # 128-row tiles with the hand-ordered loop, ragged last slice
    ("bf16", 500, 1000, 2100, 2100, "per_step"), # two 256-row tiles (last one 244 rows), odd slice count
    ("bf16", 256, 1088, 1200, 1200, "per_step"), # 256 x 256 tiles, 17 whole slices: the loop of alternating wavefronts, rotated walk
    ("bf16", 512, 448, 900, 700, "per_step"),    # the same loop on 7 slices (no rotation), two row tiles, a gathered list
    ("bf16", 1, 3840, 9000, 4000, "per_row"),    # one row, a few thousand items: eight-wavefront workgroups, clamped loads
    ("f32", 1, 1536, 6000, 3001, "per_row"),     # the same in float32, odd item count
    ("bf16", 16, 64, 600000, 300, "per_row"),    # a vocabulary beyond the ordered union: ranges reserved by atomics
    ("bf16", 24, 520, 9000, 8500, "per_step"),   # 17 to 32 rows, mid-size list: 32 x 64 tiles, ragged last tile and slice
    ("bf16", 50, 264, 6000, 5500, "per_step"),   # 33 to 64 rows, up to 64 x CUs items: 64 x 64 tiles
    ("bf16", 20, 64, 100000, 95000, "per_step"), # 17 to 32 rows, a long list: back on the kernel without LDS tiles
    ("bf16", 60, 136, 45001, 44000, "per_step"), # 64-row tiles whose width follows the list's length (192 of 256 items), ragged last tile
    ("bf16", 40, 2368, 9000, 6000, "per_step"),  # 37 slices: the other stride between the workgroups' starts in the rotated walk
    ("bf16", 40, 264, 12000, 900, "per_row"),    # union of 40 sets, at most 12000 rows: 64 x 64 tiles with the count on the device
    ("bf16", 48, 136, 30000, 1500, "per_row"),   # ... at most 30000 rows: 64 x 128 tiles
]


@pytest.mark.parametrize("dtype,rows,d,V,k,mode", LOGIT_SHAPES)
def test_subset_and_dense_logits(dtype, rows, d, V, k, mode):
    say(f"subset/dense logits {dtype} rows={rows} d={d} V={V} k={k} {mode}")
    rng = np.random.default_rng(hash((rows, d, V, k)) % (2 ** 31))
    U = rand(rng, (V, d), 0.02, dtype)
    h = rand(rng, (rows, d), 1.0, dtype)
    if mode == "per_step":
        idx = rng.permutation(V)[:k].astype(np.int32)
    else:
        idx = np.stack([rng.permutation(V)[:k] for _ in range(rows)]).astype(np.int32)
    tU, th, tidx = to_dev(U), to_dev(h), torch.from_numpy(idx).to(DEV)
    z = sv.subset_logits(th, tU, tidx).cpu().numpy()
    zd = sv.dense_logits(th, tU).cpu().numpy()
    z_ref = oracle.subset_logits(h, U, idx)
    zd_ref = oracle.dense_logits(h, U)
    assert_logits_close(z, z_ref, dtype, "subset logits")
    assert_logits_close(zd, zd_ref, dtype, "dense logits")
    # also against the float64-accumulated oracle (bounds the oracle's own rounding)
    assert_logits_close(z, oracle.subset_logits(h, U, idx, acc="f64"), dtype, "subset logits vs f64")


@pytest.mark.parametrize("rows,d,V,k,pool", [
    # (the gates are for reductions of 2048 elements and more, which the reduction-split form takes)
    (40, 2048, 50000, 900, 3000),     # bound 36000, union <= 3000: the launch gated for the reduction-split form serves it
    (40, 2048, 50000, 900, 9000),     # union ~8900: the launch gated for small tiles
    (40, 2048, 50000, 900, 50000),    # union ~26000: the same launch, near the upper end of its gate
    (40, 2048, 100000, 2000, 100000), # union ~55000: the launch picked by the bound, both others leave
    (60, 2048, 90000, 4096, 4600),    # sets longer than three quarters of the first crossover: that gate is not launched
    (24, 2048, 50000, 900, 2500),     # up to 32 rows: one gate
    (24, 2048, 50000, 900, 50000),
    (8, 4096, 40000, 8192, 9000),     # few rows, 512 MB of pairs: union path with the gates of 8 rows
    (40, 264, 50000, 900, 3000),      # a short reduction: no gates, the kernel that the bound picks
])
def test_union_size_known_on_device_only(rows, d, V, k, pool):
    """One set per row whose union is much smaller than rows x k (or not): whichever gated launch serves it,
    the logits are those of the oracle."""
    say(f"union on device rows={rows} d={d} V={V} k={k} pool={pool}")
    rng = np.random.default_rng(rows * 1000 + pool)
    U = rand(rng, (V, d), 0.02, "bf16")
    h = rand(rng, (rows, d), 1.0, "bf16")
    members = rng.permutation(V)[:pool]
    idx = np.stack([rng.permutation(members)[:k] for _ in range(rows)]).astype(np.int32)
    z = sv.subset_logits(to_dev(h), to_dev(U), torch.from_numpy(idx).to(DEV)).cpu().numpy()
    assert_logits_close(z, oracle.subset_logits(h, U, idx), "bf16", "subset logits")


@pytest.mark.parametrize("rows,d,V,k", [
    (3, 512, 700, 200),          # row kernel
    (1, 4096, 600, 200),         # one row per wavefront, whole 8 KiB rows inside a wider matrix
    (2, 3840, 500, 100),         # ... ragged rows
    (24, 2048, 3000, 800),       # skinny matrix-core kernels (shared set: reduction split; dense: streamed)
    (90, 512, 1500, 400),        # tiled matrix-core kernel
])
def test_strided_rows(rows, d, V, k):
    """h and U taken as column slices of wider matrices (row stride > d)."""
    say(f"strided rows rows={rows}")
    rng = np.random.default_rng(5)
    Uw = rand(rng, (V, d + 64), 0.02, "bf16")
    hw = rand(rng, (rows, d + 8), 1.0, "bf16")
    idx = np.stack([rng.permutation(V)[:k] for _ in range(rows)]).astype(np.int32)
    tU, th = to_dev(Uw)[:, :d], to_dev(hw)[:, :d]
    z = sv.subset_logits(th, tU, torch.from_numpy(idx).to(DEV)).cpu().numpy()
    zd = sv.dense_logits(th, tU).cpu().numpy()
    assert_logits_close(z, oracle.subset_logits(hw[:, :d], Uw[:, :d], idx), "bf16")
    assert_logits_close(zd, oracle.dense_logits(hw[:, :d], Uw[:, :d]), "bf16")
    zs = sv.subset_logits(th, tU, torch.from_numpy(idx[0]).to(DEV)).cpu().numpy()      # one shared set
    assert_logits_close(zs, oracle.subset_logits(hw[:, :d], Uw[:, :d], idx[0]), "bf16")


@pytest.mark.parametrize("rows,d,V,k,kind", [
    (70, 512, 3000, 900, "sorted"),          # 128-row tiles, compiler-ordered loop
    (150, 512, 5000, 900, "sorted"),         # two 128-row tiles, hand-ordered loop, ragged last item tile
    (300, 264, 3000, 3000, "sorted"),        # k = V, ragged reduction slice
    (512, 256, 9000, 4000, "sorted"),        # 256 x 256 tiles
    (512, 64, 2000, 10, "sorted"),           # sparse lists: most item tiles ask for nothing from a row
    (200, 256, 4000, 1500, "repeats"),       # sorted with repeated ids
    (256, 128, 1000, 1000, "clustered"),     # every id of a row inside one item tile
    (100, 256, 30000, 100, "sorted"),        # too few pairs for the vocabulary: the declaration changes nothing
    (70, 64, 50000, 45000, "sorted"),        # lists too long to be grouped and put back in order inside LDS
])
def test_subset_logits_many_rows_sorted_lists(rows, d, V, k, kind):
    """More than 64 hidden rows with their own lists, declared SORTED, that together cover the vocabulary: the
    product over all of U whose epilogue stores only the asked entries.  Element by element against the oracle
    and bit for bit against the same call without the declaration and against the same sets with every list
    shuffled (lists in any order are grouped by item tile on the device and take the same product)."""
    say(f"many rows, own sorted lists ({kind}) rows={rows} d={d} V={V} k={k}")
    rng = np.random.default_rng(rows + V + k)
    U, h = rand(rng, (V, d), 0.02, "bf16"), rand(rng, (rows, d), 1.0, "bf16")
    if kind == "repeats":
        idx = np.sort(rng.integers(0, V, (rows, k)), axis=1).astype(np.int32)
    elif kind == "clustered":
        base = rng.integers(0, V - 100, (rows, 1))
        idx = np.sort(base + rng.integers(0, 100, (rows, k)), axis=1).astype(np.int32)
    else:
        idx = np.stack([np.sort(rng.permutation(V)[:k]) for _ in range(rows)]).astype(np.int32)
    tU, th, tidx = to_dev(U), to_dev(h), torch.from_numpy(idx).to(DEV)
    z = sv.subset_logits(th, tU, tidx, sorted_lists=True)
    if rows * k >= 16384:                                   # both paths then multiply on the same matrix-core kernel
        assert torch.equal(z, sv.subset_logits(th, tU, tidx))
    # the same sets with every list in an order of its own: grouped by item tile on the device, same product
    order = np.stack([rng.permutation(k) for _ in range(rows)])
    shuffled = np.take_along_axis(idx, order, axis=1)
    z_shuffled = sv.subset_logits(th, tU, torch.from_numpy(shuffled).to(DEV)).cpu().numpy()
    z = z.cpu().numpy()
    if rows * k >= 16384:
        assert np.array_equal(z_shuffled, np.take_along_axis(z, order, axis=1))
    assert_logits_close(z_shuffled, oracle.subset_logits(h, U, shuffled), "bf16")
    assert_logits_close(z, oracle.subset_logits(h, U, idx), "bf16")
    z2, tok, prob, _ = sv.draft_step(th, tU, tidx, min(10, k), sorted_lists=True)
    assert np.array_equal(z2.cpu().numpy(), z)
    if kind != "repeats":                                   # draft tokens need unique ids within a row
        tok_ref, _ = oracle.softmax_topk(z, idx, min(10, k))
        assert np.array_equal(tok.cpu().numpy(), tok_ref)


def test_debug_mode_checks_a_declared_order(monkeypatch):
    """SPECVOCAB_VALIDATE=1: a list declared sorted that descends is reported, nothing is launched."""
    say("debug mode: declared order")
    rng = np.random.default_rng(81)
    rows, d, V, k = 70, 256, 2000, 500
    U, h = to_dev(rand(rng, (V, d), 0.02, "bf16")), to_dev(rand(rng, (rows, d), 1.0, "bf16"))
    idx = np.stack([np.sort(rng.permutation(V)[:k]) for _ in range(rows)]).astype(np.int32)
    good = torch.from_numpy(idx).to(DEV)
    idx[33, [5, 6]] = idx[33, [6, 5]]
    bad = torch.from_numpy(idx).to(DEV)
    monkeypatch.setenv("SPECVOCAB_VALIDATE", "1")
    out = torch.full((rows, k), 7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(sv.SpecVocabError) as e:
        sv.subset_logits(h, U, bad, out=out, sorted_lists=True)
    assert e.value.status == 7
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    z = sv.subset_logits(h, U, bad)                         # without the declaration any order is fine
    assert torch.equal(sv.subset_logits(h, U, good, sorted_lists=True), sv.subset_logits(h, U, good))
    monkeypatch.delenv("SPECVOCAB_VALIDATE")
    assert z.shape == (rows, k)


def test_duplicate_and_unsorted_indices_are_just_gathered():
    say("duplicate indices")
    rng = np.random.default_rng(6)
    d, V = 1024, 100
    U, h = rand(rng, (V, d), 0.02, "bf16"), rand(rng, (1, d), 1.0, "bf16")
    idx = np.array([[99, 0, 0, 50, 99, 1, 0]], dtype=np.int32)
    z = sv.subset_logits(to_dev(h), to_dev(U), torch.from_numpy(idx).to(DEV)).cpu().numpy()
    assert_logits_close(z, oracle.subset_logits(h, U, idx), "bf16")
    assert z[0, 1] == z[0, 2] == z[0, 6] and z[0, 0] == z[0, 4]


@pytest.mark.parametrize("dtype,rows,d,V,k,mode", [
    ("bf16", 1, 2048, 9000, 512, "per_row"), ("bf16", 1, 2560, 7000, 2048, "per_row"),
    ("bf16", 3, 4096, 5000, 700, "per_row"), ("bf16", 2, 1024, 3000, 333, "per_step"), ("f32", 1, 256, 8192, 512, "per_row"),
])
def test_naive_indexed_head_comparator(dtype, rows, d, V, k, mode):
    """The materialise-then-multiply comparator must give the logits of the fused gather."""
    say(f"naive indexed head {dtype} rows={rows} d={d} V={V} k={k} {mode}")
    rng = np.random.default_rng(d + V + k)
    U = rand(rng, (V, d), 0.02, dtype)
    h = rand(rng, (rows, d), 1.0, dtype)
    if mode == "per_step":
        idx = np.sort(rng.permutation(V)[:k]).astype(np.int32)
    else:
        idx = np.stack([np.sort(rng.permutation(V)[:k]) for _ in range(rows)]).astype(np.int32)
    tU, th, tidx = to_dev(U), to_dev(h), torch.from_numpy(idx).to(DEV)
    zn = sv.indexed_head_naive(th, tU, tidx).cpu().numpy()
    assert_logits_close(zn, oracle.subset_logits(h, U, idx), dtype)
    assert_logits_close(zn, sv.subset_logits(th, tU, tidx).cpu().numpy().astype(np.float64), dtype, "naive vs fused")


@pytest.mark.parametrize("dtype,d,V,k", [("bf16", 1024, 5000, 1300), ("f32", 264, 900, 77), ("bf16", 8200, 300, 300)])
def test_static_vocabulary_mode(dtype, d, V, k):
    """pack_rows once, then dense logits over the packed matrix + top-kd with the static ids: the same
    tokens and probabilities as the gathered path over the same set."""
    say(f"static vocabulary {dtype} d={d} V={V} k={k}")
    rng = np.random.default_rng(d + k)
    U, h = rand(rng, (V, d), 0.02, dtype), rand(rng, (3, d), 1.0, dtype)
    idx = np.sort(rng.permutation(V)[:k]).astype(np.int32)
    tU, th, tidx = to_dev(U), to_dev(h), torch.from_numpy(idx).to(DEV)
    Up = sv.pack_rows(tU, tidx)
    assert torch.equal(Up, tU[tidx.long()])                  # a byte-exact copy of the chosen rows
    z = sv.dense_logits(th, Up)
    assert_logits_close(z.cpu().numpy(), oracle.subset_logits(h, U, idx), dtype, "logits over the packed matrix")
    tok, prob, _ = sv.draft_topk(z, tidx, 10)
    tok_ref, prob_ref = oracle.softmax_topk(z.cpu().numpy(), idx, 10)
    assert np.array_equal(tok.cpu().numpy(), tok_ref)
    np.testing.assert_allclose(prob.cpu().numpy(), prob_ref, rtol=2e-5, atol=1e-9)


def test_debug_mode_rejects_out_of_range_indices(monkeypatch):
    """SPECVOCAB_VALIDATE=1: a bad index list is reported on the host and nothing is launched."""
    say("debug-mode index validation")
    rng = np.random.default_rng(8)
    d, V, k = 256, 500, 40
    U, h = to_dev(rand(rng, (V, d), 0.02, "bf16")), to_dev(rand(rng, (2, d), 1.0, "bf16"))
    good = torch.from_numpy(np.stack([rng.permutation(V)[:k] for _ in range(2)]).astype(np.int32)).to(DEV)
    bad = good.clone()
    bad[1, 7] = V                                        # one past the end
    neg = good.clone()
    neg[0, 0] = -1
    monkeypatch.setenv("SPECVOCAB_VALIDATE", "1")
    out = torch.full((2, k), 7.0, dtype=torch.float32, device=DEV)
    for broken in (bad, neg):
        with pytest.raises(sv.SpecVocabError) as e:
            sv.subset_logits(h, U, broken, out=out)
        assert e.value.status == 7
        with pytest.raises(sv.SpecVocabError):
            sv.draft_step(h, U, broken, 5)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                      # untouched: the operation was never enqueued
    z = sv.subset_logits(h, U, good)                     # a valid list still goes through in debug mode
    # -1 is legal exactly when the list is declared padded; anything below never is
    with pytest.raises(sv.SpecVocabError):
        sv.subset_logits(h, U, neg)
    zp = sv.subset_logits(h, U, neg, padded=True)
    assert bool(torch.isneginf(zp[0, 0])) and torch.equal(zp[1], z[1])
    neg2 = good.clone()
    neg2[1, 3] = -2
    with pytest.raises(sv.SpecVocabError) as e:
        sv.subset_logits(h, U, neg2, padded=True)
    assert e.value.status == 7
    monkeypatch.delenv("SPECVOCAB_VALIDATE")
    assert torch.equal(z, sv.subset_logits(h, U, good))


# ---------------------------------------------------------------- softmax + draft top-kd
TOPK_SHAPES = [
    # rows, k, kd, mode
    (1, 1, 1, "per_row"), (3, 7, 7, "per_row"), (2, 64, 64, "per_step"), (4, 300, 10, "per_row"),
    (2, 2048, 10, "per_row"), (2, 2049, 10, "per_row"), (1, 8192, 10, "per_row"),
    (3, 8192, 64, "per_step"), (2, 20000, 10, "per_row"), (2, 32768, 8, "per_row"),
    (1, 40000, 10, "per_row"), (60, 4096, 10, "per_row"),
    (2, 12000, 10, "per_row"), (1, 12001, 10, "per_row"), (1, 16384, 64, "per_step"),   # tokens fetched late
    (2, 30001, 5, "per_row"),
]


@pytest.mark.parametrize("rows,k,kd,mode", TOPK_SHAPES)
@pytest.mark.parametrize("ties", [False, True, "negative"])
def test_draft_topk_matches_oracle_on_identical_logits(rows, k, kd, mode, ties):
    """Both sides get the same float32 logits, so tokens must match bit-exactly, ties included."""
    say(f"draft_topk rows={rows} k={k} kd={kd} {mode} ties={ties}")
    rng = np.random.default_rng(1000 * k + kd + rows)
    z = (rng.standard_normal((rows, k)) * 3.0).astype(np.float32)
    if ties == "negative":
        z = -np.abs(z) - np.float32(40.0)     # every logit far below zero: still an ordinary row
    elif ties:
        z = np.round(z * 2.0) / 2.0           # a handful of distinct values: ties everywhere
        z[z == 0.0] = -0.0                    # -0.0 must order like +0.0
    V = max(4 * k, 1000)
    if mode == "per_step":
        idx = rng.permutation(V)[:k].astype(np.int32)
    else:
        idx = np.stack([rng.permutation(V)[:k] for _ in range(rows)]).astype(np.int32)
    tok, prob, q = sv.draft_topk(torch.from_numpy(z).to(DEV), torch.from_numpy(idx).to(DEV), kd,
                                 want_probs=True)
    tok, prob, q = tok.cpu().numpy(), prob.cpu().numpy(), q.cpu().numpy()
    tok_ref, prob_ref, q_ref = oracle.softmax_topk(z, idx, kd, full=True)
    assert np.array_equal(tok, tok_ref)
    assert np.allclose(prob, prob_ref, rtol=1e-3, atol=1e-5)
    assert np.allclose(q, q_ref, rtol=1e-3, atol=1e-5)
    assert np.allclose(q.sum(axis=1), 1.0, atol=1e-4)


# ---------------------------------------------------------------- draft step in one call
def test_signed_zeros_tie():
    """-0.0 and +0.0 are equal logits: the tie goes to the smaller token id, as in the oracle."""
    say("draft top-kd with signed zeros")
    rng = np.random.default_rng(5)
    k, kd = 3000, 12
    z = np.where(rng.random((2, k)) < 0.5, -0.0, 0.0).astype(np.float32)
    z[0, 100:110] = -1.0                                     # and something smaller in the way
    idx = np.stack([rng.permutation(50000)[:k] for _ in range(2)]).astype(np.int32)
    tok, prob, _ = sv.draft_topk(torch.from_numpy(z).to(DEV), torch.from_numpy(idx).to(DEV), kd)
    tok_ref, prob_ref = oracle.softmax_topk(z, idx, kd)
    assert np.array_equal(tok.cpu().numpy(), tok_ref)
    np.testing.assert_allclose(prob.cpu().numpy(), prob_ref, rtol=2e-5)


STEP_SHAPES = [
    # dtype, rows, d,   V,    k,    kd, mode
    ("f32", 1, 256, 8192, 512, 8, "per_row"),         # config 1
    ("bf16", 3, 1024, 5000, 1000, 10, "per_row"),
    ("bf16", 2, 3840, 9000, 4096, 10, "per_step"),
    ("bf16", 1, 4096, 20000, 8192, 64, "per_row"),
    ("bf16", 2, 512, 3000, 1001, 5, "per_row"),
    ("bf16", 65, 256, 2000, 64, 3, "per_step"),
    # one set per row, union path: the top-k kernel picks the logits from the union's product itself
    ("bf16", 20, 520, 30000, 4096, 10, "per_row"),    # four entries per thread
    ("bf16", 16, 264, 9000, 2052, 7, "per_row"),      # groups of four, half of the threads without entries
    ("bf16", 16, 264, 9000, 1201, 7, "per_row"),      # two entries per thread, odd length
    ("bf16", 24, 264, 9000, 700, 64, "per_row"),      # one entry per thread, kd = 64
    ("bf16", 18, 136, 40000, 8192, 64, "per_row"),    # eight entries per thread
    ("bf16", 16, 264, 9000, 4098, 7, "per_row"),      # k no multiple of four: the pick stays a launch of its own
]


@pytest.mark.parametrize("dtype,rows,d,V,k,kd,mode", STEP_SHAPES)
def test_draft_step_equals_the_two_calls(dtype, rows, d, V, k, kd, mode):
    say(f"draft_step {dtype} rows={rows} d={d} V={V} k={k} kd={kd} {mode}")
    rng = np.random.default_rng(d + V + k)
    U = rand(rng, (V, d), 0.02, dtype)
    h = rand(rng, (rows, d), 1.0, dtype)
    if mode == "per_step":
        idx = np.sort(rng.permutation(V)[:k]).astype(np.int32)
    else:
        idx = np.stack([np.sort(rng.permutation(V)[:k]) for _ in range(rows)]).astype(np.int32)
    tU, th, tidx = to_dev(U), to_dev(h), torch.from_numpy(idx).to(DEV)
    for rep in range(2):
        z, tok, prob, q = sv.draft_step(th, tU, tidx, kd, want_probs=True)
        z2 = sv.subset_logits(th, tU, tidx)
        tok2, prob2, q2 = sv.draft_topk(z2, tidx, kd, want_probs=True)
        assert torch.equal(z, z2) and torch.equal(tok, tok2)
        # the softmax denominator may be summed in another order (different elements per thread)
        assert torch.allclose(prob, prob2, rtol=1e-5, atol=1e-9) and torch.allclose(q, q2, rtol=1e-5, atol=1e-9)
    z_ref = oracle.subset_logits(h, U, idx)
    assert_logits_close(z.cpu().numpy(), z_ref, dtype)
    tok_same, prob_same = oracle.softmax_topk(z.cpu().numpy(), idx, kd)
    assert np.array_equal(tok.cpu().numpy(), tok_same)
    assert np.allclose(prob.cpu().numpy(), prob_same, rtol=1e-3, atol=1e-6)


def test_draft_step_sees_fresh_logits_in_a_reused_buffer():
    """The top-kd stage reads logits written just before it on the same stream; with one output
    buffer reused over many different inputs a stale read would show."""
    say("draft_step with reused output buffers")
    rng = np.random.default_rng(99)
    d, V, k, kd = 2048, 30000, 8192, 10
    U = to_dev(rand(rng, (V, d), 0.02, "bf16"))
    z = torch.empty((1, k), dtype=torch.float32, device=DEV)
    tok = torch.empty((1, kd), dtype=torch.int32, device=DEV)
    prob = torch.empty((1, kd), dtype=torch.float32, device=DEV)
    hs = to_dev(rand(rng, (40, d), 1.0, "bf16"))
    idxs = torch.from_numpy(np.stack([np.sort(rng.permutation(V)[:k]) for _ in range(40)]).astype(np.int32)).to(DEV)
    for t in range(40):
        sv.draft_step(hs[t:t + 1], U, idxs[t:t + 1], kd, logits_out=z, tok_out=tok, prob_out=prob)
        z2 = sv.subset_logits(hs[t:t + 1], U, idxs[t:t + 1])
        tok2, prob2, _ = sv.draft_topk(z2, idxs[t:t + 1], kd)
        assert torch.equal(z, z2) and torch.equal(tok, tok2), t
        assert torch.allclose(prob, prob2, rtol=1e-5, atol=1e-9), t


@pytest.mark.parametrize("rows,d,dp,V,k", [
    (2, 1024, 64, 30000, 4096),      # the latency-shaped kernels of a chain step
    (72, 2048, 64, 9000, 600),       # a batch: matrix-core down-projection and scores, many-row tail, union path
])
def test_whole_step_replays_from_a_graph(rows, d, dp, V, k):
    """select -> draft_step captured once into a HIP graph and replayed with eager work and
    synchronisations in between: every replay must reproduce the eager results."""
    say(f"graph capture and replay of select + draft_step, rows={rows}")
    rng = np.random.default_rng(2024)
    kd = 10
    U = to_dev(rand(rng, (V, d), 0.02, "bf16"))
    Wd = to_dev(rand(rng, (dp, d), 0.05, "bf16"))
    Wv = to_dev(rand(rng, (V, dp), 0.05, "bf16"))
    hs = [to_dev(rand(rng, (rows, d), 1.0, "bf16")) for _ in range(3)]
    h = hs[0].clone()
    ws_sel = torch.empty(sv.workspace_bytes(sv.SV_OP_SELECT, rows, d, V, k, dp, 0, sv.SV_BF16), dtype=torch.uint8,
                         device=DEV)
    ws_step = torch.empty(max(1, sv.workspace_bytes(sv.SV_OP_DRAFT_STEP, rows, d, V, k, 0, kd, sv.SV_BF16)),
                          dtype=torch.uint8, device=DEV)
    sel = torch.empty((rows, k), dtype=torch.int32, device=DEV)
    z = torch.empty((rows, k), dtype=torch.float32, device=DEV)
    tok = torch.empty((rows, kd), dtype=torch.int32, device=DEV)
    prob = torch.empty((rows, kd), dtype=torch.float32, device=DEV)

    def run():
        sv.select(h, Wd, Wv, k, idx_out=sel, ws=ws_sel)
        sv.draft_step(h, U, sel, kd, logits_out=z, tok_out=tok, prob_out=prob, ws=ws_step)

    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()                               # the inputs were made on the default stream
    with torch.cuda.stream(stream):
        run()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=stream):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        h.copy_(hs[rep])                                   # eager work between the replays
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            g.replay()
        torch.cuda.synchronize()
        got = (sel.clone(), z.clone(), tok.clone(), prob.clone())
        sel.zero_(); z.zero_(); tok.zero_(); prob.zero_()
        torch.cuda.synchronize()
        run()                                              # eager reference on the default stream
        torch.cuda.synchronize()
        assert torch.equal(got[0], sel) and torch.equal(got[1], z) and torch.equal(got[2], tok), rep
        assert torch.allclose(got[3], prob, rtol=1e-6, atol=0), rep


# ---------------------------------------------------------------- select
SELECT_SHAPES = [
    # dtype, rows, d,   d',  V,     k
    ("f32", 1, 256, 32, 8192, 512),           # config 1 with a selector
    ("bf16", 2, 512, 64, 5000, 1000),         # two vocabulary blocks, ragged
    ("bf16", 1, 256, 8, 4096, 1),             # k = 1, one 16-byte unit per selector row
    ("bf16", 3, 256, 24, 4097, 4097),         # k = V, one entry spills into a second block
    ("bf16", 2, 1024, 240, 9000, 300),        # 30 units: two idle lanes per row group
    ("bf16", 1, 1024, 256, 20000, 2048),
    ("bf16", 2, 1024, 512, 6000, 100),        # a full wave per selector row
    ("bf16", 1, 1024, 520, 3000, 64),         # longer than a wave-wide load: generic row kernel
    ("f32", 2, 264, 12, 700, 33),
    ("bf16", 100, 512, 64, 3000, 500),        # a batch of rows: scores on the tiled matrix-core kernel
    ("bf16", 5, 256, 32, 4099, 4099),         # five rows on the few-row tail: k = V, rows of s not 16-byte aligned
    ("bf16", 11, 256, 32, 4099, 4099),        # many-row tail kernels: the same
    ("bf16", 9, 256, 64, 10007, 777),         # three vocabulary blocks per row, ragged, odd V
    ("f32", 6, 264, 12, 5001, 100),
    ("f32", 10, 264, 12, 5001, 100),          # float32 scores through the many-row tail
    ("bf16", 8, 512, 64, 9000, 2000),         # the last row count of the few-row tail
    ("bf16", 40, 2048, 48, 3000, 300),        # batch down-projection on the matrix cores (two row groups)
]


@pytest.mark.parametrize("dtype,rows,d,dp,V,k", SELECT_SHAPES)
def test_select(dtype, rows, d, dp, V, k):
    say(f"select {dtype} rows={rows} d={d} d'={dp} V={V} k={k}")
    rng = np.random.default_rng(V + k + dp)
    h = rand(rng, (rows, d), 1.0, dtype)
    Wd = rand(rng, (dp, d), 0.05, dtype)
    Wv = rand(rng, (V, dp), 0.05, dtype)
    idx, sc = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k, want_scores=True)
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy()
    ref_idx, _, s_ref, _ = oracle.select(h, Wd, Wv, k, full=True)
    for r in range(rows):
        band, diff = check_selected_set(idx[r], s_ref[r], ref_idx[r], k, dtype)
        say(f"  row {r}: {band} scores within tolerance of the k-th, {diff} ids differ from the oracle")
        assert_logits_close(sc[r], s_ref[r, idx[r]], dtype, "scores at the selected ids")


@pytest.mark.parametrize("rows", [2, 6, 12])      # 12 rows: the many-row forms of the tail kernels
def test_select_ties_go_to_smaller_ids(rows):
    """Rows of W_vocab repeated: repeated rows score bit-identically on the GPU as well, so the
    set is decided by the tie rule alone wherever the distinct scores are far apart."""
    say(f"select ties rows={rows}")
    rng = np.random.default_rng(77)
    d, dp, V = 256, 16, 10000
    h = rand(rng, (rows, d), 1.0, "bf16")
    Wd = rand(rng, (dp, d), 0.05, "bf16")
    base = rand(rng, (5, dp), 0.5, "bf16")                # 5 distinct rows, well separated scores
    Wv = base[rng.integers(0, 5, size=V)]
    for k in (1, 1999, 2000, 5000, V):
        idx, _ = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k)
        ref_idx, _, s_ref, _ = oracle.select(h, Wd, Wv, k, full=True)
        clear = []                                            # rows that meet the premise of an exact comparison
        for r in range(rows):
            vals = np.unique(s_ref[r])
            assert len(vals) == 5
            if np.diff(vals).min() > 0.01:                    # >> any rounding difference
                clear.append(r)
        assert 2 * len(clear) > rows
        assert np.array_equal(idx.cpu().numpy()[clear], ref_idx[clear]), k
    Wv[:] = Wv[0]
    idx, _ = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), 4321)
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(4321, dtype=np.int32), (rows, 1)))


@pytest.mark.parametrize("rows", [1, 5, 9])
def test_select_at_the_largest_vocabulary(rows):
    """V = 4194304, the most specvocab_select accepts: 1024 vocabulary blocks per row, both forms of the
    tail kernels."""
    say(f"select V=4194304 rows={rows}")
    rng = np.random.default_rng(80 + rows)
    d, dp, V, k = 16, 8, 4194304, 1000
    h, Wd, Wv = rand(rng, (rows, d), 1.0, "bf16"), rand(rng, (dp, d), 0.3, "bf16"), rand(rng, (V, dp), 0.3, "bf16")
    idx, sc = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k, want_scores=True)
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy()
    ref_idx, _, s_ref, _ = oracle.select(h, Wd, Wv, k, full=True)
    for r in range(rows):
        check_selected_set(idx[r], s_ref[r], ref_idx[r], k, "bf16")
        assert_logits_close(sc[r], s_ref[r, idx[r]], "bf16", "scores at the selected ids")


AUX_SHAPES = [
    # dtype, rows, d,   d',  V
    ("f32", 1, 256, 32, 8192),
    ("bf16", 1, 1024, 256, 20000),       # one hidden row: row kernel over 512-byte selector rows
    ("bf16", 3, 512, 64, 4099),          # rows of the output not 16-byte aligned, two vocabulary blocks
    ("bf16", 20, 2048, 128, 9000),       # matrix-core projections
    ("bf16", 80, 512, 64, 5000),         # tiled matrix-core scores
    ("bf16", 2, 256, 8, 1),              # V = 1: log q = 0
    ("bf16", 1, 16, 8, 5000000),         # past the selection's vocabulary limit: larger vocabulary blocks
]


@pytest.mark.parametrize("dtype,rows,d,dp,V", AUX_SHAPES)
def test_aux_log_softmax(dtype, rows, d, dp, V):
    """log q_aux over the whole vocabulary (Section 3.4) against the oracle: the scores carry the logit
    tolerance, the normaliser is common to a row."""
    say(f"aux log-softmax {dtype} rows={rows} d={d} d'={dp} V={V}")
    rng = np.random.default_rng(V + dp + rows)
    h, Wd, Wv = rand(rng, (rows, d), 1.0, dtype), rand(rng, (dp, d), 0.05, dtype), rand(rng, (V, dp), 0.05, dtype)
    got = sv.aux_log_softmax(to_dev(h), to_dev(Wd), to_dev(Wv)).cpu().numpy()
    ref = oracle.aux_log_softmax(h, Wd, Wv)
    assert_logits_close(got, ref, dtype, "log q_aux")
    # each row is a normalised distribution, to float32 accuracy
    lse = np.log(np.exp(got.astype(np.float64)).sum(axis=1))
    assert np.abs(lse).max() < 5e-5, lse


PADDED_SHAPES = [
    # dtype, rows, d, V, k, mode          (which kernel family the clean copy goes through)
    ("bf16", 1, 1024, 9000, 2048, "per_row"),     # row gather: the kernels read the padding slots themselves
    ("bf16", 1, 4096, 3000, 1000, "per_step"),    # ... one row per wavefront
    ("bf16", 3, 8200, 300, 120, "per_row"),       # ... rows longer than 16 KiB
    ("f32", 2, 264, 900, 100, "per_row"),
    ("bf16", 6, 1024, 5000, 700, "per_step"),     # matrix cores, one shared padded list
    ("bf16", 20, 512, 6000, 1100, "per_row"),     # union of sets
    ("bf16", 70, 256, 3000, 300, "per_step"),     # tiled matrix-core kernel
    ("bf16", 80, 256, 2000, 300, "per_row"),      # many rows whose sets cover the vocabulary: grouped by tile, pick epilogue
]


@pytest.mark.parametrize("dtype,rows,d,V,k,mode", PADDED_SHAPES)
def test_padded_index_lists(dtype, rows, d, V, k, mode):
    """SV_IDX_PADDED: padding slots (-1) give -inf logits and probability 0; the real entries and the
    draft tokens are those of the oracle on the same padded list."""
    say(f"padded lists {dtype} rows={rows} d={d} V={V} k={k} {mode}")
    rng = np.random.default_rng(rows * 31 + k)
    U, h = rand(rng, (V, d), 0.02, dtype), rand(rng, (rows, d), 1.0, dtype)
    shape = (k,) if mode == "per_step" else (rows, k)
    idx = (rng.permutation(V)[:k] if mode == "per_step"
           else np.stack([rng.permutation(V)[:k] for _ in range(rows)])).astype(np.int32)
    idx = np.where(rng.random(shape) < 0.3, -1, idx).astype(np.int32)       # 30 % padding
    if mode == "per_row":
        idx[0, :] = -1
        idx[0, k // 2] = 17                                                   # a row with a single real entry
    tU, th, tidx = to_dev(U), to_dev(h), torch.from_numpy(idx).to(DEV)
    z = sv.subset_logits(th, tU, tidx, padded=True).cpu().numpy()
    z_ref = oracle.subset_logits(h, U, idx)
    pad = np.broadcast_to(idx < 0, z.shape)
    assert np.all(np.isneginf(z[pad])) and np.all(np.isneginf(z_ref[pad]))
    assert_logits_close(z[~pad], z_ref[~pad], dtype, "logits of the real entries")
    kd = 5
    zz, tok, prob, q = sv.draft_step(th, tU, tidx, kd, want_probs=True, padded=True)
    assert np.array_equal(np.isneginf(zz.cpu().numpy()), pad)
    tok_ref, prob_ref, q_ref = oracle.softmax_topk(zz.cpu().numpy(), idx, kd, full=True)
    assert np.array_equal(tok.cpu().numpy(), tok_ref)
    np.testing.assert_allclose(prob.cpu().numpy(), prob_ref, rtol=2e-5, atol=1e-9)
    np.testing.assert_allclose(q.cpu().numpy(), q_ref, rtol=2e-5, atol=1e-9)
    if mode == "per_row":                                                     # one real entry, kd = 5
        assert tok_ref[0].tolist() == [17, -1, -1, -1, -1] and prob_ref[0, 0] == 1.0


def test_empty_rows_and_draft_topk_on_padding():
    """A row of padding only: all probabilities 0, tokens -1 (through the slow exact path as well)."""
    say("draft top-kd on rows of padding")
    k, kd = 3000, 8
    z = np.full((3, k), -np.inf, dtype=np.float32)
    idx = np.full((3, k), -1, dtype=np.int32)
    z[1, 5], idx[1, 5] = 2.0, 40                    # one real entry among 2999 padding slots
    z[2, :4], idx[2, :4] = [0.5, 0.25, 0.5, -1.0], [9, 8, 7, 6]
    tok, prob, q = sv.draft_topk(torch.from_numpy(z).to(DEV), torch.from_numpy(idx).to(DEV), kd, want_probs=True)
    tok_ref, prob_ref, q_ref = oracle.softmax_topk(z, idx, kd, full=True)
    assert np.array_equal(tok.cpu().numpy(), tok_ref)
    np.testing.assert_allclose(prob.cpu().numpy(), prob_ref, rtol=2e-5, atol=0)
    np.testing.assert_allclose(q.cpu().numpy(), q_ref, rtol=2e-5, atol=0)
    assert tok_ref[0].tolist() == [-1] * kd and tok_ref[2].tolist()[:4] == [7, 9, 8, 6]


@pytest.mark.parametrize("rows", [1, 7, 10])
def test_select_threshold_pads_in_place(rows):
    """specvocab_select_threshold: the plain selection with the entries scoring below tau turned into
    padding slots, then usable as a padded list."""
    say(f"select with a score threshold rows={rows}")
    rng = np.random.default_rng(90 + rows)
    d, dp, V, k = 512, 64, 7000, 900
    h, Wd, Wv = rand(rng, (rows, d), 1.0, "bf16"), rand(rng, (dp, d), 0.05, "bf16"), rand(rng, (V, dp), 0.05, "bf16")
    U = rand(rng, (V, d), 0.02, "bf16")
    th, tWd, tWv = to_dev(h), to_dev(Wd), to_dev(Wv)
    idx, sc = sv.select(th, tWd, tWv, k, want_scores=True)
    tau = float(np.median(sc.cpu().numpy()))
    idx_t, sc_t = sv.select(th, tWd, tWv, k, want_scores=True, tau=tau)
    keep = sc >= tau
    assert torch.equal(idx_t, torch.where(keep, idx, torch.full_like(idx, -1)))
    assert torch.equal(sc_t, torch.where(keep, sc, torch.full_like(sc, -float("inf"))))
    assert 0 < int(keep.sum()) < keep.numel()
    tau_eq = float(sc[0, 5])                                 # inclusive: a token scoring exactly tau stays
    idx_e, _ = sv.select(th, tWd, tWv, k, tau=tau_eq)
    assert int(idx_e[0, 5]) == int(idx[0, 5]) and torch.equal(idx_e, torch.where(sc >= tau_eq, idx, torch.full_like(idx, -1)))
    # and the oracle agrees on what stays (scores within tolerance of tau may fall on either side)
    ref_idx, ref_sc = oracle.select(h, Wd, Wv, k, tau=tau)
    got, want = idx_t.cpu().numpy(), ref_idx
    differ = (got != want)
    s_ref = oracle.select(h, Wd, Wv, k, full=True)[2]
    for r, j in zip(*np.nonzero(differ)):
        v = got[r, j] if got[r, j] >= 0 else want[r, j]
        assert v >= 0 and abs(s_ref[r, v] - tau) < 2e-2, (r, j, got[r, j], want[r, j])
    z = sv.subset_logits(th, to_dev(U), idx_t, padded=True)
    assert torch.equal(torch.isneginf(z), idx_t < 0)


def _int_valued(rng, shape, span, dtype):
    x = rng.integers(-span, span + 1, shape).astype(np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def test_select_is_exact_on_integer_valued_inputs():
    """Small integers make every product and sum exact on both sides whatever the order of accumulation,
    and leave thousands of exactly tied scores: ids and scores must equal the oracle's one by one (the k-th
    score falls inside a tie almost always, so this is the tie rule at every size the tail kernels branch on)."""
    rng = np.random.default_rng(12345)
    for case in range(60):
        rows = int(rng.choice([1, 1, 2, 3, 4, 5, 6, 9, 17]))
        if case % 10 == 9:
            rows = (17, 70, 300)[(case // 10) % 3]            # batches: the matrix-core forms of the selection
        V = int(rng.choice([1, 2, 3, 5, 63, 64, 100, 1000, 4095, 4096, 4097, 9000, 20000, 70001]))
        k = min(V, int(rng.choice([1, 2, max(1, V // 16), max(1, V // 2), max(1, V - 1), V])))
        dp = int(rng.choice([8, 16, 24, 64]))
        d = dp + int(rng.choice([0, 8, 40]))
        span = int(rng.choice([1, 2, 3]))
        dtype = str(rng.choice(["bf16", "f32"]))
        tau = float(rng.integers(-3, 6)) if rng.random() < 0.3 else None
        say(f"integer select {case}: {dtype} rows={rows} V={V} k={k} d'={dp} d={d} span={span} tau={tau}")
        h = _int_valued(rng, (rows, d), span, dtype)
        Wd = np.zeros((dp, d), np.float32)
        Wd[np.arange(dp), np.arange(dp)] = 1.0              # h' = the first d' entries of h
        Wd = Wd if dtype == "f32" else f32_to_bf16_bits(Wd)
        Wv = _int_valued(rng, (V, dp), span, dtype)
        idx, sc = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k, want_scores=True, tau=tau)
        ref_idx, ref_sc = oracle.select(h, Wd, Wv, k, tau=tau)[:2]
        assert np.array_equal(idx.cpu().numpy(), ref_idx), (case, dtype, rows, V, k)
        assert np.array_equal(sc.cpu().numpy(), ref_sc.astype(np.float32)), (case, dtype, rows, V, k)


@pytest.mark.parametrize("rows", [1, 12, 70])
def test_select_is_exact_at_the_full_vocabulary(rows):
    """The same exactness at the size of the Qwen3-8B-shaped configuration (V = 151936, d' = 256, k = 8192):
    integer-valued inputs, thousands of exactly tied scores around the k-th, every id equal to the oracle's."""
    say(f"integer select at V=151936 d'=256 rows={rows}")
    rng = np.random.default_rng(151936 + rows)
    V, dp, d, k = 151936, 256, 264, 8192
    h = _int_valued(rng, (rows, d), 2, "bf16")
    Wd = np.zeros((dp, d), np.float32)
    Wd[np.arange(dp), np.arange(dp)] = 1.0
    Wd = f32_to_bf16_bits(Wd)
    Wv = _int_valued(rng, (V, dp), 2, "bf16")
    idx, sc = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k, want_scores=True)
    ref_idx, ref_sc = oracle.select(h, Wd, Wv, k)[:2]
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert np.array_equal(sc.cpu().numpy(), ref_sc.astype(np.float32))
    idx2, _ = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k)          # without the scores output
    assert torch.equal(idx2, idx)


def test_draft_step_is_exact_on_integer_valued_inputs():
    """The same for subset logits + top-kd: exact logits, exact ties, so tokens equal the oracle's."""
    rng = np.random.default_rng(54321)
    for case in range(40):
        rows = int(rng.choice([1, 1, 2, 3, 5, 18, 70]))
        d = int(rng.choice([8, 64, 264, 1024, 4096]))
        V = int(rng.choice([10, 300, 5000, 20000]))
        k = min(V, int(rng.choice([1, 7, 64, 1000, 1025, 4096, 8192, 9001])))
        kd = min(k, int(rng.choice([1, 4, 10, 64])))
        per_row = bool(rng.random() < 0.5)
        say(f"integer draft step {case}: rows={rows} d={d} V={V} k={k} kd={kd} per_row={per_row}")
        U = _int_valued(rng, (V, d), 1, "bf16")
        h = _int_valued(rng, (rows, d), 1, "bf16")
        if per_row:
            idx = np.stack([rng.permutation(V)[:k] for _ in range(rows)]).astype(np.int32)
        else:
            idx = rng.permutation(V)[:k].astype(np.int32)
        z, tok, prob, _ = sv.draft_step(to_dev(h), to_dev(U), torch.from_numpy(idx).to(DEV), kd)
        z_ref = oracle.subset_logits(h, U, idx)
        assert np.array_equal(z.cpu().numpy(), z_ref.astype(np.float32)), case
        ref_tok, ref_prob = oracle.softmax_topk(z_ref, idx, kd)
        assert np.array_equal(tok.cpu().numpy(), ref_tok), case
        np.testing.assert_allclose(prob.cpu().numpy(), ref_prob, rtol=2e-5, atol=1e-30)


def test_k_varies_from_step_to_step():
    """Section 3.3 Step 2 allows k to change per decoding step: k is a call argument, and buffers and
    workspace sized once for the largest k serve every step."""
    say("k varies per step")
    rng = np.random.default_rng(79)
    d, dp, V, kmax = 512, 64, 6000, 2048
    U, Wd, Wv = rand(rng, (V, d), 0.02, "bf16"), rand(rng, (dp, d), 0.05, "bf16"), rand(rng, (V, dp), 0.05, "bf16")
    tU, tWd, tWv = to_dev(U), to_dev(Wd), to_dev(Wv)
    ws = torch.empty(sv.workspace_bytes(sv.SV_OP_SELECT, 1, d, V, kmax, dp, 0, sv.SV_BF16), dtype=torch.uint8,
                     device=DEV)
    sel_buf = torch.empty(kmax, dtype=torch.int32, device=DEV)
    z_buf = torch.empty(kmax, dtype=torch.float32, device=DEV)
    for step, k in enumerate((2048, 300, 1, 1024, 17)):
        h = rand(rng, (1, d), 1.0, "bf16")
        th = to_dev(h)
        sel, z = sel_buf[:k].view(1, k), z_buf[:k].view(1, k)
        sv.select(th, tWd, tWv, k, idx_out=sel, ws=ws)
        _, tok, prob, _ = sv.draft_step(th, tU, sel, min(10, k), logits_out=z)
        ref_idx, _, s_ref, _ = oracle.select(h, Wd, Wv, k, full=True)
        check_selected_set(sel.cpu().numpy()[0], s_ref[0], ref_idx[0], k, "bf16")
        z_ref = oracle.subset_logits(h, U, sel.cpu().numpy())
        assert_logits_close(z.cpu().numpy(), z_ref, "bf16", f"step {step} k={k}")
        tok_ref, prob_ref = oracle.softmax_topk(z.cpu().numpy(), sel.cpu().numpy(), min(10, k))
        assert np.array_equal(tok.cpu().numpy(), tok_ref)
        np.testing.assert_allclose(prob.cpu().numpy(), prob_ref, rtol=2e-5, atol=1e-9)


def test_exact_selector_reduces_to_dense_topk():
    """d' = d, W_down = I, W_vocab = U: select must return the top-k of the true logits."""
    say("select with the exact selector")
    rng = np.random.default_rng(78)
    d, V, k = 256, 3000, 200
    U, h = rand(rng, (V, d), 0.05, "bf16"), rand(rng, (2, d), 1.0, "bf16")
    eye = f32_to_bf16_bits(np.eye(d, dtype=np.float32))
    idx, _ = sv.select(to_dev(h), to_dev(eye), to_dev(U), k)
    z_ref = oracle.dense_logits(h, U)
    for r in range(2):
        ref = np.sort(np.argsort(-z_ref[r], kind="stable")[:k]).astype(np.int32)
        check_selected_set(idx[r].cpu().numpy(), z_ref[r], ref, k, "bf16")


# ---------------------------------------------------------------- selection for a batch without the score matrix
BATCH_SELECT_SHAPES = [
    # rows, d,  d',  V,     k        (bf16, 65 rows or more, V >= 32768, no scores output: the bracketed selection)
    (65, 256, 32, 32768, 100),       # 128-row tiles, one of them half empty; the smallest vocabulary of the path
    (70, 256, 32, 33000, 500),
    (100, 1024, 256, 50001, 4096),   # ragged last item tile
    (128, 256, 40, 40007, 1),        # k = 1
    (130, 256, 64, 36000, 18000),    # two 128-row tiles with the hand-ordered loop, half the vocabulary selected
    (300, 256, 64, 50001, 5000),     # three 128-row tiles
    (512, 512, 256, 40000, 2048),    # 256 x 256 tiles
    (257, 256, 128, 70001, 70001),   # k = V: everything is selected
    (90, 256, 24, 45000, 44999),     # k = V - 1
    (66, 256, 32, 140000, 8192),     # more item tiles than the resolve step holds in registers
    (12, 512, 64, 40000, 3000),      # below 65 rows: the path that materialises the scores (a control)
]


@pytest.mark.parametrize("rows,d,dp,V,k", BATCH_SELECT_SHAPES)
def test_select_batch_without_score_matrix(rows, d, dp, V, k):
    """65 or more bf16 rows and no scores output: the selection that never writes s.  Checked against the
    oracle (band rule) and bit for bit against the path that materialises s (asking for the scores selects it;
    both compute s with the same matrix-core kernel)."""
    say(f"batch select rows={rows} d={d} d'={dp} V={V} k={k}")
    rng = np.random.default_rng(rows * 7 + V + k)
    h = rand(rng, (rows, d), 1.0, "bf16")
    Wd = rand(rng, (dp, d), 0.05, "bf16")
    Wv = rand(rng, (V, dp), 0.05, "bf16")
    th, tWd, tWv = to_dev(h), to_dev(Wd), to_dev(Wv)
    idx, _ = sv.select(th, tWd, tWv, k)
    idx_s, sc = sv.select(th, tWd, tWv, k, want_scores=True)      # asks for scores: the materialising path
    assert torch.equal(idx, idx_s)
    idx = idx.cpu().numpy()
    check_rows = range(rows) if rows <= 70 else range(0, rows, 7)
    for r in check_rows:
        ref_idx, _, s_ref, _ = oracle.select(h[r:r + 1], Wd, Wv, k, full=True)
        check_selected_set(idx[r], s_ref[0], ref_idx[0], k, "bf16")
    assert np.all(np.diff(idx, axis=1) > 0) and idx.min() >= 0 and idx.max() < V


def _adversarial_selector(rng, V, dp, sign):
    """W_vocab whose sampled rows (ids floor(j V / SELECT_SAMPLE)) are all zero while every other row scores
    sign * (positive integer) against an all-ones h': the sample says nothing about the rest."""
    Wv = (sign * rng.integers(1, 4, (V, dp))).astype(np.float32)
    sampled = (np.arange(sv.SELECT_SAMPLE, dtype=np.int64) * V) // sv.SELECT_SAMPLE
    Wv[sampled] = 0.0
    return f32_to_bf16_bits(Wv), sampled


@pytest.mark.parametrize("rows,V,k", [(65, 40000, 2000), (70, 65536, 8192), (130, 33001, 33001)])
def test_select_batch_redoes_rows_whose_bracket_missed(rows, V, k):
    """Inputs built to defeat the sample: every sampled token scores 0, every other token scores high, so far
    more than k scores lie above the bracket and every row is redone by the exact one-workgroup path.
    Integer-valued, hence exact: ids must equal the oracle's."""
    say(f"batch select with a useless sample rows={rows} V={V} k={k}")
    rng = np.random.default_rng(V + rows)
    dp, d = 16, 24
    Wv, _ = _adversarial_selector(rng, V, dp, +1)
    h = np.zeros((rows, d), np.float32)
    h[:, :dp] = rng.integers(1, 3, (rows, dp))
    h = f32_to_bf16_bits(h)
    Wd = np.zeros((dp, d), np.float32)
    Wd[np.arange(dp), np.arange(dp)] = 1.0
    Wd = f32_to_bf16_bits(Wd)
    idx, _ = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k)
    ref_idx = oracle.select(h, Wd, Wv, k)[0]
    assert np.array_equal(idx.cpu().numpy(), ref_idx)


def test_select_batch_when_the_sample_holds_all_the_best():
    """The mirror case: every token outside the sample scores below it, so the k best are sampled tokens with
    exactly tied scores (all 0): the bracket holds, the tie rule decides among thousands of candidates."""
    say("batch select, the best tokens are exactly the sampled ones")
    rng = np.random.default_rng(4242)
    rows, V, k, dp, d = 67, 50000, 3000, 16, 16
    Wv, sampled = _adversarial_selector(rng, V, dp, -1)
    h = f32_to_bf16_bits(rng.integers(1, 3, (rows, d)).astype(np.float32))
    Wd = f32_to_bf16_bits(np.eye(dp, d, dtype=np.float32))
    idx, _ = sv.select(to_dev(h), to_dev(Wd), to_dev(Wv), k)
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.sort(sampled)[:k].astype(np.int32), (rows, 1)))
    assert np.array_equal(idx.cpu().numpy(), oracle.select(h, Wd, Wv, k)[0])



# ---------------------------------------------------------------- whole draft step, config 1
def test_config1_all_steps():
    c = CONFIGS[1]
    say("config 1: every step, float32")
    U, hs, idxs = c.weights(), c.hidden(), c.indices()
    Wd, Wv = c.selector()
    tU = to_dev(U)
    allv = torch.arange(c.V, dtype=torch.int32, device=DEV)
    for t in range(c.steps):
        h, idx = hs[t], idxs[t]
        th, tidx = to_dev(h), torch.from_numpy(idx).to(DEV)
        z = sv.subset_logits(th, tU, tidx)
        z_ref = oracle.subset_logits(h, U, idx)
        assert_logits_close(z.cpu().numpy(), z_ref, "f32")
        tok, prob, _ = sv.draft_topk(z, tidx, c.kd)
        tok_ref, prob_ref = oracle.softmax_topk(z_ref, idx, c.kd)
        for r in range(c.rows):
            check_draft_tokens(tok[r].cpu().numpy(), prob[r].cpu().numpy(), z_ref[r], idx[r], tok_ref[r],
                               prob_ref[r], "f32")
        # the full-vocabulary check: subset = all V reproduces the dense projection
        zd = sv.dense_logits(th, tU)
        za = sv.subset_logits(th, tU, allv)
        assert torch.equal(zd, za) or np.allclose(zd.cpu().numpy(), za.cpu().numpy(), rtol=1e-5, atol=1e-6)
        assert_logits_close(zd.cpu().numpy(), oracle.dense_logits(h, U), "f32")
        assert_logits_close(z.cpu().numpy(), zd.cpu().numpy()[np.arange(c.rows)[:, None], idx].astype(np.float64),
                            "f32", "subset vs slice of dense")
        tokf, _, _ = sv.draft_topk(zd, allv, c.kd)
        tokf_ref, _ = oracle.softmax_topk(zd.cpu().numpy(), np.arange(c.V, dtype=np.int32), c.kd)
        assert np.array_equal(tokf.cpu().numpy(), tokf_ref)
        sel, _ = sv.select(th, to_dev(Wd), to_dev(Wv), c.k)
        ref_sel, _, s_ref, _ = oracle.select(h, Wd, Wv, c.k, full=True)
        check_selected_set(sel[0].cpu().numpy(), s_ref[0], ref_sel[0], c.k, "f32")


# ---------------------------------------------------------------- full-size configurations
@pytest.fixture(scope="module")
def llama_head():
    say("drawing the Llama-3-8B-shaped output embedding (128256 x 4096 bf16)")
    U = CONFIGS[2].weights()
    return U, to_dev(U)


def test_config2_chain_full_size(llama_head):
    """d=4096, V=128256, k=8192, one row per step: the configuration the benchmark times."""
    c = CONFIGS[2]
    U, tU = llama_head
    steps = 3
    hs, idxs = c.hidden(steps), c.indices(steps)
    Wd, Wv = c.selector()
    tWd, tWv = to_dev(Wd), to_dev(Wv)
    for t in range(steps):
        say(f"config 2 step {t}")
        h, idx = hs[t], idxs[t]
        th, tidx = to_dev(h), torch.from_numpy(idx).to(DEV)
        z = sv.subset_logits(th, tU, tidx)
        z_ref = oracle.subset_logits(h, U, idx)
        err = assert_logits_close(z.cpu().numpy(), z_ref, "bf16")
        say(f"  subset logits max |err| = {err:.3e}")
        tok, prob, _ = sv.draft_topk(z, tidx, c.kd)
        tok_ref, prob_ref = oracle.softmax_topk(z_ref, idx, c.kd)
        check_draft_tokens(tok[0].cpu().numpy(), prob[0].cpu().numpy(), z_ref[0], idx[0], tok_ref[0],
                           prob_ref[0], "bf16")
        tok_same, prob_same = oracle.softmax_topk(z.cpu().numpy(), idx, c.kd)
        assert np.array_equal(tok.cpu().numpy(), tok_same)
        assert np.allclose(prob.cpu().numpy(), prob_same, rtol=1e-3, atol=1e-6)
        zf, tokf, probf, _ = sv.draft_step(th, tU, tidx, c.kd)        # the launch the benchmark times
        assert torch.equal(zf, z) and torch.equal(tokf, tok) and torch.allclose(probf, prob, rtol=1e-5, atol=1e-9)
    say("config 2 dense baseline, all 128256 logits")
    zd = sv.dense_logits(to_dev(hs[0]), tU).cpu().numpy()
    assert_logits_close(zd, oracle.dense_logits(hs[0], U), "bf16", "dense logits")
    assert_logits_close(sv.subset_logits(to_dev(hs[0]), tU, torch.from_numpy(idxs[0]).to(DEV)).cpu().numpy(),
                        zd[:, idxs[0][0]].astype(np.float64), "bf16", "subset vs slice of dense")
    say("config 2 shape with the selector (d'=256)")
    sel, sc = sv.select(to_dev(hs[0]), tWd, tWv, c.k, want_scores=True)
    ref_sel, _, s_ref, _ = oracle.select(hs[0], Wd, Wv, c.k, full=True)
    band, diff, band_s, outside = check_selected_set(sel[0].cpu().numpy(), s_ref[0], ref_sel[0], c.k, "bf16", tight=True)
    say(f"  config 2 select: {band} scores within 2e-2 of the k-th, {band_s} within 1e-3, {diff} ids differ from "
        f"the oracle's set, {outside} of them outside the 1e-3 band")
    assert_logits_close(sc[0].cpu().numpy(), s_ref[0, sel[0].cpu().numpy()], "bf16")


def test_config3_tree_full_size(llama_head):
    """60 tree rows, own k=4096 subset each (half shared step-wide), top-10 per row."""
    c = CONFIGS[3]
    U, tU = llama_head
    say("config 3: 60 rows x 4096")
    h = c.hidden(1)[0]
    idx = c.indices(1)[0]
    th, tidx = to_dev(h), torch.from_numpy(idx).to(DEV)
    z = sv.subset_logits(th, tU, tidx)
    tok, prob, _ = sv.draft_topk(z, tidx, c.kd)
    zn, tokn, probn = z.cpu().numpy(), tok.cpu().numpy(), prob.cpu().numpy()
    z_ref = oracle.subset_logits(h, U, idx)                  # all 60 rows x 4096 entries
    err = assert_logits_close(zn, z_ref, "bf16")
    say(f"  config 3: all {c.rows} x {c.k} logits against the oracle, max |err| = {err:.3e}")
    tok_ref, prob_ref = oracle.softmax_topk(z_ref, idx, c.kd)
    for r in range(c.rows):
        check_draft_tokens(tokn[r], probn[r], z_ref[r], idx[r], tok_ref[r], prob_ref[r], "bf16")
    tok_same, _ = oracle.softmax_topk(zn, idx, c.kd)
    assert np.array_equal(tokn, tok_same)
    # property that holds for every row: shared tokens get the logit <U[tok], h_r> whichever row asks
    zd = sv.dense_logits(th, tU).cpu().numpy()
    assert np.abs(np.take_along_axis(zd, idx.astype(np.int64), axis=1) - zn).max() <= 2e-2


def test_config4_gemma_head_full_size():
    """d=3840, V=262144, 8 rows, k in {2048, 8192, 32768}, one set per step and one per row."""
    c = CONFIGS[4]
    say("drawing the 262144 x 3840 output embedding")
    U = c.weights()
    tU = to_dev(U)
    h = c.hidden(1)[0]
    th = to_dev(h)
    rng = make_rng(4, 2)
    for k in c.k_sweep:
        say(f"config 4 k={k}")
        shared = zipf_subset(rng, c.V, k)
        z = sv.subset_logits(th, tU, torch.from_numpy(shared).to(DEV)).cpu().numpy()
        err = assert_logits_close(z, oracle.subset_logits(h, U, shared), "bf16")     # every entry, all 8 rows
        say(f"  shared set: all {c.rows} x {k} logits against the oracle, max |err| = {err:.3e}")
        per_row = np.stack([zipf_subset(rng, c.V, k) for _ in range(c.rows)])
        z = sv.subset_logits(th, tU, torch.from_numpy(per_row).to(DEV))
        z_ref = oracle.subset_logits(h, U, per_row)
        err = assert_logits_close(z.cpu().numpy(), z_ref, "bf16")
        say(f"  one set per row: all {c.rows} x {k} logits against the oracle, max |err| = {err:.3e}")
        tok, _, _ = sv.draft_topk(z, torch.from_numpy(per_row).to(DEV), c.kd)
        tok_same, _ = oracle.softmax_topk(z.cpu().numpy(), per_row, c.kd)
        assert np.array_equal(tok.cpu().numpy(), tok_same)
        tok_ref, prob_ref = oracle.softmax_topk(z_ref, per_row, c.kd)
        probn = sv.draft_topk(z, torch.from_numpy(per_row).to(DEV), c.kd)[1].cpu().numpy()
        for r in range(c.rows):
            check_draft_tokens(tok[r].cpu().numpy(), probn[r], z_ref[r], per_row[r], tok_ref[r], prob_ref[r], "bf16")
    say("config 4 dense baseline on sampled vocabulary entries")
    zd = sv.dense_logits(th, tU).cpu().numpy()
    sample = rng.permutation(c.V)[:2048].astype(np.int32)
    assert_logits_close(zd[:, sample], oracle.subset_logits(h, U, sample), "bf16")
    del tU
    torch.cuda.empty_cache()


def test_config5_full_step_with_selection():
    """d=4096, V=151936, 512 rows, selector d'=256, k=8192, top-10: select -> logits -> top-kd."""
    c = CONFIGS[5]
    say("drawing the Qwen3-8B-shaped head and selector")
    U = c.weights()
    Wd, Wv = c.selector()
    h = c.hidden(1)[0]
    tU, tWd, tWv, th = to_dev(U), to_dev(Wd), to_dev(Wv), to_dev(h)
    say("config 5 select")
    sel, _ = sv.select(th, tWd, tWv, c.k)
    say("config 5 subset logits")
    z = sv.subset_logits(th, tU, sel, sorted_lists=True)       # the selection emits ascending ids
    say("config 5 subset logits, the same sets with every list in an order of its own and nothing declared")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(55)
    order = torch.stack([torch.randperm(c.k, generator=gen, device=DEV) for _ in range(c.rows)])
    z_any = sv.subset_logits(th, tU, torch.gather(sel, 1, order).contiguous())
    assert torch.equal(z_any, torch.gather(z, 1, order))        # the same product, entry for entry
    del z_any, order
    say("config 5 draft top-kd")
    tok, prob, _ = sv.draft_topk(z, sel, c.kd)
    torch.cuda.synchronize()
    seln, zn, tokn, probn = sel.cpu().numpy(), z.cpu().numpy(), tok.cpu().numpy(), prob.cpu().numpy()
    # every row: a valid, ascending, unique id set
    assert seln.min() >= 0 and seln.max() < c.V and np.all(np.diff(seln, axis=1) > 0)
    tok_same, prob_same = oracle.softmax_topk(zn, seln, c.kd)
    assert np.array_equal(tokn, tok_same)
    assert np.allclose(probn, prob_same, rtol=1e-3, atol=1e-6)
    rows_checked = list(range(0, c.rows, 8))      # 64 of the 512 rows against the oracle, select and logits
    bands, diffs, bands_s, outs, worst = [], [], [], [], 0.0
    for r in rows_checked:
        ref_sel, _, s_ref, _ = oracle.select(h[r:r + 1], Wd, Wv, c.k, full=True)
        band, diff, band_s, outside = check_selected_set(seln[r], s_ref[0], ref_sel[0], c.k, "bf16", tight=True)
        bands.append(band); diffs.append(diff); bands_s.append(band_s); outs.append(outside)
        z_ref = oracle.subset_logits(h[r:r + 1], U, seln[r:r + 1])
        worst = max(worst, assert_logits_close(zn[r:r + 1], z_ref, "bf16"))
        tok_ref, prob_ref = oracle.softmax_topk(z_ref, seln[r:r + 1], c.kd)
        check_draft_tokens(tokn[r], probn[r], z_ref[0], seln[r], tok_ref[0], prob_ref[0], "bf16")
    say(f"  config 5 select over {len(rows_checked)} rows: scores within 2e-2 of the k-th per row {min(bands)}..{max(bands)}, "
        f"within 1e-3 {min(bands_s)}..{max(bands_s)}; ids differing from the oracle's set per row "
        f"{min(diffs)}..{max(diffs)} (total {sum(diffs)}), of them outside the 1e-3 band {sum(outs)}; "
        f"subset logits max |err| = {worst:.3e}")


# ---------------------------------------------------------------- first call inside a stream capture
_CAPTURE_FIRST = r"""
import sys
import numpy as np, torch
sys.path.insert(0, {root!r})
import paper_2602_13836_amd as sv
dev = "cuda:0"
gen = torch.Generator(device=dev); gen.manual_seed(5)
rows, d, V = 512, 256, 3000
U = (torch.randn((V, d), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
h = torch.randn((rows, d), generator=gen, device=dev).to(torch.bfloat16)
out = torch.zeros((rows, V), dtype=torch.float32, device=dev)
sv.init()                                   # device set-up outside the capture; no kernel has run yet
stream = torch.cuda.Stream()
g = torch.cuda.CUDAGraph()
torch.cuda.synchronize()
with torch.cuda.stream(stream):
    with torch.cuda.graph(g, stream=stream):
        sv.dense_logits(h, U, out=out)      # 256 x 256 tiles: 144 KiB of LDS, opted in by init()
torch.cuda.synchronize()
for rep in range(2):
    out.zero_()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        g.replay()
    torch.cuda.synchronize()
    got = out.clone()
    ref = sv.dense_logits(h, U)
    torch.cuda.synchronize()
    assert torch.equal(got, ref), rep
ref64 = h.double() @ U.double().T
assert float((got.double() - ref64).abs().max()) <= 2e-2
print("captured-first-call ok")
"""


def test_first_call_may_be_captured_after_init():
    """A fresh process whose FIRST library call happens inside a stream capture: specvocab_init has done the
    per-device set-up (the LDS opt-in of the 256 x 256 tile kernel among it) beforehand, so nothing but the
    kernel launch falls into the capture."""
    import os
    import subprocess
    import sys
    say("first call inside a capture, fresh process")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", _CAPTURE_FIRST.format(root=root)], capture_output=True, text=True,
                         timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "captured-first-call ok" in res.stdout
