"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before enqueueing anything."""
import ctypes
import os
import re

import pytest

import paper_2602_13836_amd as sv
from paper_2602_13836_amd import build as sv_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "specvocab.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sv.LIB_PATH):
        sv_build.build_library()
    return sv.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specvocab_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree_on_exports(lib):
    names = _declared_functions()
    assert names == sorted(sv.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert sv.version() == 100
    assert sv.status_string(0) == "ok"
    seen = {sv.status_string(s) for s in (1, 2, 3, 4, 5, 6, 7, 8)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert sv.status_string(77) == "unknown status"


def test_workspace_bytes(lib):
    assert sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 1, 4096, 128256, 8192) == 0
    assert sv.workspace_bytes(sv.SV_OP_DENSE_LOGITS, 1, 4096, 128256) == 0
    assert sv.workspace_bytes(sv.SV_OP_DRAFT_TOPK, 1, 0, 0, 8192, 0, 10) == 0
    n = sv.workspace_bytes(sv.SV_OP_SELECT, 2, 4096, 128256, 8192, 256)
    assert n >= 2 * 128256 * 4 + 2 * 256 * 2           # the score matrix and h'
    assert n % 256 == 0
    with pytest.raises(sv.SpecVocabError) as e:
        sv.workspace_bytes(sv.SV_OP_SELECT, 1, 4096, 100, 101, 256)     # k > V
    assert e.value.status == 2
    with pytest.raises(sv.SpecVocabError) as e:
        sv.workspace_bytes(99)
    assert e.value.status == 3
    assert lib.specvocab_workspace_bytes(0, 1, 8, 8, 1, 8, 0, 1, 0, None) == 1


# fake, never dereferenced device addresses: every call below must fail validation on the host
A = ctypes.c_void_p(0x10000)          # 16-byte aligned
MIS = ctypes.c_void_p(0x10008)        # misaligned


def test_subset_logits_rejects_bad_arguments(lib):
    f = lib.specvocab_subset_logits
    ok = dict(h=A, rows=1, d=256, ldh=256, U=A, V=1000, ldu=256, dt=1, idx=A, k=10, mode=0, out=A)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["h"], a["rows"], a["d"], a["ldh"], a["U"], a["V"], a["ldu"], a["dt"], a["idx"], a["k"],
                 a["mode"], a["out"], None, 0, None)

    assert call(h=None) == 1 and call(U=None) == 1 and call(idx=None) == 1 and call(out=None) == 1
    assert call(rows=0) == 2 and call(k=0) == 2 and call(V=0) == 2
    assert call(ldh=128) == 2 and call(ldu=255) == 2
    assert call(dt=7) == 3 and call(mode=2) == 3 and call(mode=3) == 3 and call(mode=16) == 3   # flags: 4 padded, 8 sorted
    assert call(d=252, ldh=252, ldu=252) == 6             # row not a whole number of 16-byte units
    assert call(ldu=260) == 4                              # stride not 16-byte aligned
    assert call(h=MIS) == 4 and call(U=MIS) == 4
    assert call(rows=70000) == 2


def test_dense_select_topk_reject_bad_arguments(lib):
    d = lib.specvocab_dense_logits
    assert d(None, 1, 256, 256, A, 10, 256, 1, A, None, 0, None) == 1
    assert d(A, 1, 256, 256, A, 10, 256, 9, A, None, 0, None) == 3
    assert d(A, 1, 256, 100, A, 10, 256, 1, A, None, 0, None) == 2
    assert d(A, 1, 256, 256, MIS, 10, 256, 1, A, None, 0, None) == 4

    s = lib.specvocab_select
    assert s(A, 1, 256, 256, A, 32, A, 1000, 1, 10, None, None, A, 1 << 30, None) == 1
    assert s(A, 1, 256, 256, A, 32, A, 1000, 1, 1001, A, None, A, 1 << 30, None) == 2      # k > V
    assert s(A, 1, 256, 256, A, 32, A, 1000, 1, 10, A, None, None, 0, None) == 5            # no workspace
    assert s(A, 1, 256, 256, A, 32, A, 1000, 1, 10, A, None, A, 16, None) == 5              # too small
    assert s(A, 1, 256, 256, A, 30, A, 1000, 1, 10, A, None, A, 1 << 30, None) == 6         # d' % 8
    assert s(A, 1, 256, 256, A, 32, A, 1000, 4, 10, A, None, A, 1 << 30, None) == 3
    assert s(A, 1, 256, 256, A, 32, A, 4194305, 1, 10, A, None, A, 1 << 40, None) == 6      # V above the limit

    n = lib.specvocab_indexed_head_naive
    assert n(A, 1, 256, 256, A, 1000, 256, 1, A, 100, 0, A, None, 0, None) == 5          # needs its workspace
    assert n(A, 1, 256, 256, A, 1000, 256, 1, None, 100, 0, A, A, 1 << 30, None) == 1
    assert sv.workspace_bytes(sv.SV_OP_INDEXED_HEAD_NAIVE, 2, 4096, 128256, 8192) == 2 * 8192 * 4096 * 2

    st = lib.specvocab_select_threshold
    assert st(A, 1, 256, 256, A, 32, A, 1000, 1, 10, float("nan"), A, None, A, 1 << 30, None) == 2
    assert st(A, 1, 256, 256, A, 32, A, 1000, 1, 10, 0.5, None, None, A, 1 << 30, None) == 1
    # a padded list needs room for its clean copy where the matrix cores multiply (several hidden rows, one
    # shared list), none where the row-gather kernel reads the list itself; the comparator takes plain lists only
    assert sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 1, 4096, 128256, 8192, idx_mode=sv.SV_IDX_PADDED) == 0
    plain = sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 8, 4096, 128256, 8192, idx_mode=sv.SV_IDX_PER_STEP)
    assert sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 8, 4096, 128256, 8192,
                              idx_mode=sv.SV_IDX_PER_STEP | sv.SV_IDX_PADDED) == plain + 8192 * 4
    assert lib.specvocab_subset_logits(A, 8, 256, 256, A, 1000, 256, 1, A, 100, 5, A, None, 0, None) == 5
    assert lib.specvocab_indexed_head_naive(A, 1, 256, 256, A, 1000, 256, 1, A, 100, 4, A, A, 1 << 30, None) == 6
    assert lib.specvocab_subset_logits(A, 1, 256, 256, A, 1000, 256, 1, A, 100, 2, A, None, 0, None) == 3

    # several hidden rows with their own padded lists: the clean copy AND the union of the sets must fit, and
    # that is decided before anything is enqueued (a workspace that holds the clean copy only is refused)
    both = sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 20, 256, 5000, 1000, idx_mode=sv.SV_IDX_PER_ROW | sv.SV_IDX_PADDED)
    pad_only = 20 * 1000 * 4
    assert both > pad_only + 5000 * 8
    assert lib.specvocab_subset_logits(A, 20, 256, 256, A, 5000, 256, 1, A, 1000, 4, A, A, 80128, None) == 5
    assert lib.specvocab_subset_logits(A, 20, 256, 256, A, 5000, 256, 1, A, 1000, 4, A, A, both - 1, None) == 5
    assert lib.specvocab_subset_logits(A, 20, 256, 256, A, 5000, 256, 1, A, 1000, 4, A, MIS, both, None) == 4
    assert lib.specvocab_draft_step(A, 20, 256, 256, A, 5000, 256, 1, A, 1000, 4, 10, A, A, A, None, A, 80128,
                                    None) == 5

    # many rows whose sets cover the vocabulary: the table of slices per (row, item tile) -- and, unless the lists
    # are declared sorted, their positions grouped by tile -- instead of the union scratch
    tab = sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 512, 4096, 151936, 8192, idx_mode=sv.SV_IDX_PER_ROW | sv.SV_IDX_SORTED)
    grp = sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 512, 4096, 151936, 8192, idx_mode=sv.SV_IDX_PER_ROW)
    assert 512 * 594 * 4 <= tab <= 512 * 600 * 4 and grp == tab + 3 * 512 * 8192 * 4
    assert lib.specvocab_subset_logits(A, 512, 256, 256, A, 151936, 256, 1, A, 8192, 8, A, A, tab - 1, None) == 5
    assert lib.specvocab_subset_logits(A, 512, 256, 256, A, 151936, 256, 1, A, 8192, 0, A, A, grp - 1, None) == 5
    # sets that cannot cover the vocabulary keep the union of the sets
    assert sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 100, 4096, 151936, 2048, idx_mode=sv.SV_IDX_PER_ROW) > 100 * 151936 * 4
    # the declaration changes nothing where the general path is the better one anyway
    assert sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 60, 4096, 128256, 4096, idx_mode=sv.SV_IDX_SORTED) == \
        sv.workspace_bytes(sv.SV_OP_SUBSET_LOGITS, 60, 4096, 128256, 4096)

    q = lib.specvocab_aux_log_softmax
    assert q(A, 1, 256, 256, A, 32, A, 1000, 1, None, A, 1 << 30, None) == 1
    assert q(A, 1, 256, 256, A, 32, A, 1000, 1, A, None, 0, None) == 5
    assert q(A, 1, 256, 256, A, 30, A, 1000, 1, A, A, 1 << 30, None) == 6
    assert q(A, 0, 256, 256, A, 32, A, 1000, 1, A, A, 1 << 30, None) == 2
    assert sv.workspace_bytes(sv.SV_OP_AUX_LOG_SOFTMAX, 2, 4096, 128256, 0, 256) > 2 * 256 * 2

    pk = lib.specvocab_pack_rows
    assert pk(A, 1000, 256, 256, 1, None, 10, A, None) == 1
    assert pk(A, 1000, 256, 256, 1, A, 0, A, None) == 2
    assert pk(A, 1000, 256, 256, 7, A, 10, A, None) == 3
    assert pk(A, 1000, 252, 256, 1, A, 10, A, None) == 6                                   # d % 8
    assert pk(A, 1000, 256, 256, 1, A, 10, MIS, None) == 4

    f = lib.specvocab_draft_step
    assert f(A, 1, 256, 256, A, 1000, 256, 1, A, 100, 0, 10, None, A, A, None, None, 0, None) == 1   # no logits_out
    assert f(A, 1, 256, 256, A, 1000, 256, 1, A, 100, 0, 101, A, A, A, None, None, 0, None) == 2     # kd > k
    assert f(A, 1, 256, 256, A, 1000, 256, 1, A, 100, 0, 65, A, A, A, None, None, 0, None) == 6
    assert f(A, 1, 256, 256, MIS, 1000, 256, 1, A, 100, 0, 10, A, A, A, None, None, 0, None) == 4

    t = lib.specvocab_draft_topk
    assert t(None, A, 0, 1, 100, 10, A, A, None, None, 0, None) == 1
    assert t(A, A, 0, 1, 100, 101, A, A, None, None, 0, None) == 2                          # kd > k
    assert t(A, A, 0, 1, 100, 0, A, A, None, None, 0, None) == 2
    assert t(A, A, 0, 1, 1000, 65, A, A, None, None, 0, None) == 6                          # kd > 64
    assert t(A, A, 3, 1, 100, 10, A, A, None, None, 0, None) == 3


def test_select_static_rejects_before_touching_the_device(lib):
    """The entry point without a workspace argument: the usual validation, and shapes whose scratch need
    exceeds the static array are refused with the workspace status."""
    f = lib.specvocab_select_static
    assert f(None, 1, 256, 256, A, 32, A, 1000, 1, 10, A, None, None) == 1
    assert f(A, 1, 256, 256, A, 32, A, 1000, 1, 10, None, None, None) == 1
    assert f(A, 1, 256, 256, A, 32, A, 1000, 1, 1001, A, None, None) == 2                    # k > V
    assert f(A, 1, 256, 256, A, 30, A, 1000, 1, 10, A, None, None) == 6                      # d' % 8
    assert f(A, 1, 256, 256, A, 32, A, 1000, 9, 10, A, None, None) == 3
    # config 2's shape fits the 8 MiB array, 16 rows of it do not
    assert sv.workspace_bytes(sv.SV_OP_SELECT, 1, 4096, 128256, 8192, 256) <= sv.STATIC_SCRATCH_BYTES
    assert sv.workspace_bytes(sv.SV_OP_SELECT, 16, 4096, 128256, 8192, 256) > sv.STATIC_SCRATCH_BYTES
    assert f(A, 16, 4096, 4096, A, 256, A, 128256, 1, 8192, A, None, None) == 5
    assert f(A, 1, 4096, 4096, A, 256, A, 4194304, 1, 8192, A, None, None) == 5


def test_binding_refuses_cpu_tensors(lib):
    import torch
    h = torch.zeros(1, 256, dtype=torch.bfloat16)
    U = torch.zeros(10, 256, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        sv.dense_logits(h, U)
    with pytest.raises(ValueError):
        sv.subset_logits(h, U, torch.zeros(4, dtype=torch.int32))


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        sv.load_library(str(tmp_path / "libspecvocab.so"))
