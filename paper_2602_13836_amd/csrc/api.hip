// C ABI of the SpecVocab draft-step library: host-side argument validation, workspace carving
// and launch planning.  Nothing here touches device memory on the host, allocates, or
// synchronises; every check happens before the first kernel is enqueued.
#include "../../include/specvocab.h"

#include "sv_device.h"
#include "sv_launch.h"

#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>

// Device scratch of the entry point that takes no workspace (specvocab_select_static): one array per GPU the
// library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and host calls use the per-device address kept in DeviceState.
static __device__ __align__(256) unsigned char scratch[SPECVOCAB_STATIC_SCRATCH_BYTES];

namespace sv {

namespace {

// Per-device set-up, done once under a lock and published with release/acquire: device attributes, the
// opt-in of the kernels that use more than 64 KiB of LDS, and this device's address of the scratch array.
struct DeviceState {
    std::atomic<int> ready{0};
    int cus = 0;
    void* scratch_ptr = nullptr;
};
constexpr int kMaxDevices = 64;
DeviceState g_dev[kMaxDevices];
std::mutex g_dev_mutex;

hipError_t device_state(const DeviceState** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    DeviceState& st = g_dev[dev];
    if (!st.ready.load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(g_dev_mutex);
        if (!st.ready.load(std::memory_order_relaxed)) {
            int cus = 0;
            e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
            if (e != hipSuccess) return e;
            st.cus = cus > 0 ? cus : 256;
            e = configure_skinny_mfma_lds();
            if (e != hipSuccess) return e;
            e = configure_tile_mfma_lds();
            if (e != hipSuccess) return e;
            e = configure_select_lds();
            if (e != hipSuccess) return e;
            e = configure_union_lds();
            if (e != hipSuccess) return e;
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            st.scratch_ptr = p;
            st.ready.store(1, std::memory_order_release);
        }
    }
    *out = &st;
    return hipSuccess;
}

}  // namespace

hipError_t device_info(DeviceInfo* out) {
    const DeviceState* st = nullptr;
    hipError_t e = device_state(&st);
    if (e != hipSuccess) return e;
    out->cus = st->cus;
    out->valid = 1;
    return hipSuccess;
}

}  // namespace sv

namespace {

constexpr int64_t kMaxRows = 65535;            // rows ride on gridDim.y
constexpr int64_t kMaxVocab = 2147483647LL;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t n) { return (n + 255u) & ~static_cast<size_t>(255u); }
inline int esize_of(int dt) { return dt == SV_BF16 ? 2 : 4; }
inline bool dtype_ok(int dt) { return dt == SV_F32 || dt == SV_BF16; }
constexpr int kModeFlags = SV_IDX_PADDED | SV_IDX_SORTED;
inline bool mode_ok(int m) { return (m & ~kModeFlags) == SV_IDX_PER_ROW || (m & ~kModeFlags) == SV_IDX_PER_STEP; }
inline bool is_padded(int m) { return (m & SV_IDX_PADDED) != 0; }
inline bool is_sorted(int m) { return (m & SV_IDX_SORTED) != 0 && !is_padded(m); }   // a padded list is not sorted once cleaned
inline int base_mode(int m) { return m & ~kModeFlags; }

// a row of `n` elements must be a whole number of 16-byte units, and so must its stride
inline int check_row(int64_t n, int64_t ld, int dt) {
    if (n < 1 || ld < n) return SV_ERR_SHAPE;
    const int per16 = 16 / esize_of(dt);
    if (n % per16 != 0) return SV_ERR_UNSUPPORTED;
    if (ld % per16 != 0) return SV_ERR_ALIGN;
    return SV_OK;
}

// the library's per-device set-up, if this is the first call on the current device
inline int ensure_device() {
    sv::DeviceInfo di;
    return sv::device_info(&di) == hipSuccess ? SV_OK : SV_ERR_HIP;
}

struct SelectWs {
    size_t hp_off, s_off, radix_off, total;
    size_t bracket_off;      // scratch of the bracketed selection (it aliases the score matrix: one or the other)
};
SelectWs select_ws(int64_t rows, int64_t V, int64_t d_prime, int64_t k, int dt) {
    SelectWs w;
    w.hp_off = 0;
    w.s_off = round256((size_t)rows * (size_t)d_prime * (size_t)esize_of(dt));
    w.radix_off = w.s_off + round256((size_t)rows * (size_t)V * sizeof(float));
    w.total = w.radix_off + round256(sv::select_scratch_words(rows, V) * sizeof(uint32_t));
    w.bracket_off = w.s_off;
    if (sv::bracket_select_supported(dt, rows, V, k)) {
        const size_t t = w.bracket_off + round256(sv::bracket_scratch_words(rows, V) * sizeof(uint32_t));
        if (t > w.total) w.total = t;
    }
    return w;
}

// Debug mode (environment variable SPECVOCAB_VALIDATE=1): range-check an index list before using it.
int validate_indices(const int32_t* idx, int64_t n, int64_t V, hipStream_t s, bool padded = false,
                     int64_t sorted_row_len = 0) {
    const char* v = getenv("SPECVOCAB_VALIDATE");
    if (!v || strcmp(v, "1") != 0) return SV_OK;
    unsigned bad = 0;
    if (sv::count_bad_indices(idx, n, V, padded, sorted_row_len, s, &bad) != hipSuccess) return SV_ERR_HIP;
    return bad ? SV_ERR_INDEX : SV_OK;
}

// Picks the kernel family for out[r, j] = <M[row(r, j)], x[r]>:
//   several hidden rows sharing one set of rows of M  -> matrix cores, M read once
//   several hidden rows with their own sets           -> union of the sets, then matrix cores
//   otherwise (one hidden row, float32, small cases)  -> row-gather kernel
// defer != nullptr: the caller can do the union path's pick itself (see sv::DeferredPick; untouched on other paths)
int launch_rows_product(int dt, const sv::GemvArgs& g, int64_t V, void* ws, size_t ws_bytes, hipStream_t s,
                        sv::DeferredPick* defer = nullptr) {
    if (sv::skinny_mfma_supported(dt, g)) return sv::launch_skinny_mfma(g, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
    if (sv::union_path_wanted(dt, g)) {
        if (!ws || ws_bytes < sv::union_ws_bytes(g.rows, V, g.n_items)) return SV_ERR_WORKSPACE;
        if (!aligned16(ws)) return SV_ERR_ALIGN;
        return sv::launch_union_logits(g, V, ws, s, defer) == hipSuccess ? SV_OK : SV_ERR_HIP;
    }
    return sv::launch_gemv(dt, g, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
}

// the gather arguments shared by specvocab_subset_logits and specvocab_draft_step
sv::GemvArgs gather_args(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* U, int64_t V, int64_t ldu, int dt,
                         const int32_t* idx, int64_t k, int idx_mode, float* logits_out) {
    const int es = esize_of(dt);
    sv::GemvArgs g{};
    g.x = static_cast<const char*>(h);
    g.x_row_bytes = ldh * es;
    g.M = static_cast<const char*>(U);
    g.m_row_bytes = ldu * es;
    g.idx = idx;
    g.idx_row_stride = base_mode(idx_mode) == SV_IDX_PER_ROW ? k : 0;
    g.n_items = k;
    g.chunks = (int)(d * es / 16);
    g.rows = (int)rows;
    g.out_f32 = logits_out;
    g.out_row_stride = k;
    g.m_rows = V;
    return g;
}

// the row-gather kernels take padding slots as they are; the matrix-core and union paths need a clean copy
bool padded_needs_copy(int dt, const sv::GemvArgs& g) {
    return sv::skinny_mfma_supported(dt, g) || sv::union_path_wanted(dt, g);
}

// bytes of the clean copy of a padded index list (0 if the list is not padded or no copy is needed)
size_t pad_ws_bytes(int64_t rows, int64_t k, int idx_mode, int dt, const sv::GemvArgs& g) {
    if (!is_padded(idx_mode) || !padded_needs_copy(dt, g)) return 0;
    const int64_t sets = base_mode(idx_mode) == SV_IDX_PER_ROW ? rows : 1;
    return round256((size_t)sets * (size_t)k * sizeof(int32_t));
}

// what the product itself needs from the workspace: the slice table of the sorted-lists path, or the union
size_t product_ws_bytes(int dt, const sv::GemvArgs& g, int64_t rows, int64_t V, int64_t k, int idx_mode) {
    if (sv::pick_path_wanted(dt, g, V, is_sorted(idx_mode))) return sv::pick_ws_bytes(rows, V, k, is_sorted(idx_mode));
    return sv::union_path_wanted(dt, g) ? sv::union_ws_bytes(rows, V, k) : 0;
}

size_t gather_ws_bytes(int64_t rows, int64_t d, int64_t V, int64_t k, int dt, int idx_mode) {
    sv::GemvArgs g = gather_args(nullptr, rows, d, d, nullptr, V, d, dt, reinterpret_cast<const int32_t*>(16), k,
                                 idx_mode, nullptr);
    return pad_ws_bytes(rows, k, idx_mode, dt, g) + product_ws_bytes(dt, g, rows, V, k, idx_mode);
}

// Gathered logits for an index list that may carry padding slots (SV_IDX_PADDED).  The row-gather
// kernels read a padding slot as "row 0, result -inf" themselves.  The matrix-core and union paths run
// on a clean copy of the list (padding -> token 0) and the padding slots get -inf afterwards, so those
// paths stay exactly as they are for plain lists.
int launch_gather(int dt, const void* h, int64_t rows, int64_t d, int64_t ldh, const void* U, int64_t V,
                  int64_t ldu, const int32_t* idx, int64_t k, int idx_mode, float* logits_out, void* ws,
                  size_t ws_bytes, hipStream_t s, sv::DeferredPick* defer = nullptr) {
    const bool padded = is_padded(idx_mode);
    const int64_t sets = base_mode(idx_mode) == SV_IDX_PER_ROW ? rows : 1;
    const sv::GemvArgs g0 = gather_args(h, rows, d, ldh, U, V, ldu, dt, idx, k, idx_mode, logits_out);
    // everything the call will need from the workspace (clean copy of a padded list, union of the sets) is
    // checked here, before the first launch
    const bool copy = padded && padded_needs_copy(dt, g0);
    const size_t pb = copy ? pad_ws_bytes(rows, k, idx_mode, dt, g0) : 0;
    const size_t need = pb + product_ws_bytes(dt, g0, rows, V, k, idx_mode);
    if (need) {
        if (!ws || ws_bytes < need) return SV_ERR_WORKSPACE;
        if (!aligned16(ws)) return SV_ERR_ALIGN;
    }
    sv::DeviceInfo di;
    if (sv::device_info(&di) != hipSuccess) return SV_ERR_HIP;       // device set-up, if this is the first call
    int st = validate_indices(idx, sets * k, V, s, padded, is_sorted(idx_mode) ? k : 0);
    if (st != SV_OK) return st;
    if (padded && !copy) return sv::launch_gemv(dt, g0, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
    const int32_t* use = idx;
    char* rest = static_cast<char*>(ws);
    size_t rest_bytes = ws_bytes;
    if (copy) {
        if (sv::launch_pad_clean(idx, sets * k, reinterpret_cast<int32_t*>(ws), s) != hipSuccess) return SV_ERR_HIP;
        use = reinterpret_cast<const int32_t*>(ws);
        rest += pb;
        rest_bytes -= pb;
    }
    const sv::GemvArgs g = gather_args(h, rows, d, ldh, U, V, ldu, dt, use, k, idx_mode, logits_out);
    if (sv::pick_path_wanted(dt, g, V, is_sorted(idx_mode)))
        st = sv::launch_pick_logits(g, V, is_sorted(idx_mode), rest, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
    else
        st = launch_rows_product(dt, g, V, rest_bytes ? rest : nullptr, rest_bytes, s, copy ? nullptr : defer);
    if (st != SV_OK) return st;
    if (copy && sv::launch_pad_mask(idx, g.idx_row_stride, (int)rows, k, logits_out, s) != hipSuccess)
        return SV_ERR_HIP;
    return SV_OK;
}

// h'[r, :] = W_down h[r, :] into hp ([rows x d_prime] in the storage dtype; bf16: round to nearest even);
// optionally clears zero_words words at zero_ptr in the same launch
int launch_down_projection(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* W_down,
                           int64_t d_prime, int dt, char* hp, uint32_t* zero_ptr, size_t zero_words,
                           hipStream_t s, int32_t* spread_ptr = nullptr, int64_t spread_n = 0, int64_t spread_V = 0) {
    const int es = esize_of(dt);
    sv::GemvArgs g{};
    g.x = static_cast<const char*>(h);
    g.x_row_bytes = ldh * es;
    g.M = static_cast<const char*>(W_down);
    g.m_row_bytes = d * es;
    g.idx = nullptr;
    g.idx_row_stride = 0;
    g.n_items = d_prime;
    g.chunks = (int)(d * es / 16);
    g.rows = (int)rows;
    g.out_f32 = dt == SV_BF16 ? nullptr : reinterpret_cast<float*>(hp);
    g.out_bf16 = dt == SV_BF16 ? reinterpret_cast<uint16_t*>(hp) : nullptr;
    g.out_row_stride = d_prime;
    g.zero_ptr = zero_ptr;
    g.zero_words = zero_words;
    g.spread_ptr = spread_ptr;
    g.spread_n = spread_n;
    g.spread_V = spread_V;
    if (sv::ksplit_rows_supported(dt, g))              // a batch of rows: W_down read once per 32 of them
        return sv::launch_ksplit_rows(g, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
    return sv::launch_gemv(dt, g, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
}

int check_select_shape(int64_t rows, int64_t d, int64_t V, int64_t k, int64_t d_prime, int dt) {
    if (!dtype_ok(dt)) return SV_ERR_DTYPE;
    if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab || k < 1 || k > V) return SV_ERR_SHAPE;
    int st = check_row(d, d, dt);
    if (st != SV_OK) return st;
    st = check_row(d_prime, d_prime, dt);
    if (st != SV_OK) return st;
    if (d > (1 << 24) || d_prime > (1 << 24) || V > sv::select_max_vocab()) return SV_ERR_UNSUPPORTED;
    return SV_OK;
}

int check_aux_shape(int64_t rows, int64_t d, int64_t V, int64_t d_prime, int dt) {
    if (!dtype_ok(dt)) return SV_ERR_DTYPE;
    if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab) return SV_ERR_SHAPE;
    int st = check_row(d, d, dt);
    if (st != SV_OK) return st;
    st = check_row(d_prime, d_prime, dt);
    if (st != SV_OK) return st;
    if (d > (1 << 24) || d_prime > (1 << 24)) return SV_ERR_UNSUPPORTED;
    return SV_OK;
}

struct AuxWs {
    size_t hp_off, partial_off, total;
};
AuxWs aux_ws(int64_t rows, int64_t V, int64_t d_prime, int dt) {
    AuxWs w;
    w.hp_off = 0;
    w.partial_off = round256((size_t)rows * (size_t)d_prime * (size_t)esize_of(dt));
    w.total = w.partial_off + round256(sv::log_softmax_ws_floats(rows, V) * sizeof(float));
    return w;
}

}  // namespace

extern "C" {

int specvocab_version(void) { return SPECVOCAB_VERSION; }

const char* specvocab_status_string(int status) {
    switch (status) {
        case SV_OK: return "ok";
        case SV_ERR_NULL: return "a required pointer is NULL";
        case SV_ERR_SHAPE: return "a size is out of range or sizes disagree";
        case SV_ERR_DTYPE: return "unknown dtype, index mode or operation";
        case SV_ERR_ALIGN: return "pointer or row stride is not 16-byte aligned";
        case SV_ERR_WORKSPACE: return "workspace missing or too small";
        case SV_ERR_UNSUPPORTED: return "shape not supported by this build";
        case SV_ERR_INDEX: return "an index lies outside [0, V) (debug mode)";
        case SV_ERR_HIP: return "a HIP runtime call failed";
        default: return "unknown status";
    }
}

int specvocab_workspace_bytes(int op, int64_t rows, int64_t d, int64_t V, int64_t k, int64_t d_prime,
                              int64_t kd, int dt, int idx_mode, size_t* bytes_out) {
    (void)kd;
    if (!bytes_out) return SV_ERR_NULL;
    *bytes_out = 0;
    switch (op) {
        case SV_OP_SELECT: {
            const int st = check_select_shape(rows, d, V, k, d_prime, dt);
            if (st != SV_OK) return st;
            *bytes_out = select_ws(rows, V, d_prime, k, dt).total;
            return SV_OK;
        }
        case SV_OP_SUBSET_LOGITS:
        case SV_OP_DRAFT_STEP:
            if (!dtype_ok(dt) || !mode_ok(idx_mode)) return SV_ERR_DTYPE;
            if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab || k < 1 || d < 1) return SV_ERR_SHAPE;
            *bytes_out = gather_ws_bytes(rows, d, V, k, dt, idx_mode);
            return SV_OK;
        case SV_OP_INDEXED_HEAD_NAIVE: {
            if (!dtype_ok(dt) || !mode_ok(idx_mode)) return SV_ERR_DTYPE;
            if (rows < 1 || rows > kMaxRows || k < 1 || d < 1) return SV_ERR_SHAPE;
            if (is_padded(idx_mode)) return SV_ERR_UNSUPPORTED;
            const int64_t sets = base_mode(idx_mode) == SV_IDX_PER_ROW ? rows : 1;
            *bytes_out = round256((size_t)sets * (size_t)k * (size_t)d * (size_t)esize_of(dt));
            return SV_OK;
        }
        case SV_OP_AUX_LOG_SOFTMAX: {
            const int st = check_aux_shape(rows, d, V, d_prime, dt);
            if (st != SV_OK) return st;
            *bytes_out = aux_ws(rows, V, d_prime, dt).total;
            return SV_OK;
        }
        case SV_OP_DRAFT_TOPK:
        case SV_OP_DENSE_LOGITS:
            return SV_OK;
        default:
            return SV_ERR_DTYPE;
    }
}

static int select_impl(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* W_down, int64_t d_prime,
                       const void* W_vocab, int64_t V, int dt, int64_t k, float tau, int32_t* idx_out,
                       float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    if (!h || !W_down || !W_vocab || !idx_out) return SV_ERR_NULL;
    int st = check_select_shape(rows, d, V, k, d_prime, dt);
    if (st != SV_OK) return st;
    st = check_row(d, ldh, dt);
    if (st != SV_OK) return st;
    if (!aligned16(h) || !aligned16(W_down) || !aligned16(W_vocab) || !aligned16(ws)) return SV_ERR_ALIGN;
    const SelectWs w = select_ws(rows, V, d_prime, k, dt);
    if (!ws || ws_bytes < w.total) return SV_ERR_WORKSPACE;
    if (ensure_device() != SV_OK) return SV_ERR_HIP;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int es = esize_of(dt);
    char* base = static_cast<char*>(ws);
    char* hp = base + w.hp_off;
    float* scores = reinterpret_cast<float*>(base + w.s_off);
    uint32_t* radix = reinterpret_cast<uint32_t*>(base + w.radix_off);

    // A batch of hidden rows whose scores nobody asked for: the selection that never writes the score matrix
    // (a sample of the vocabulary brackets every row's k-th score; the full product is classified in the
    // epilogue of the matrix-core kernel).  The down-projection launch also writes the sample's ids.
    if (!scores_out && tau == -INFINITY && sv::bracket_select_supported(dt, rows, V, k)) {
        uint32_t* bscratch = reinterpret_cast<uint32_t*>(base + w.bracket_off);
        int32_t* ids = nullptr;
        int64_t m = 0;
        float* samp = nullptr;
        sv::bracket_sample(rows, V, bscratch, &ids, &m, &samp);
        if (launch_down_projection(h, rows, d, ldh, W_down, d_prime, dt, hp, nullptr, 0, s, ids, m, V) != SV_OK)
            return SV_ERR_HIP;
        sv::GemvArgs gs{};
        gs.x = hp;
        gs.x_row_bytes = d_prime * es;
        gs.M = static_cast<const char*>(W_vocab);
        gs.m_row_bytes = d_prime * es;
        gs.idx = ids;
        gs.n_items = m;
        gs.chunks = (int)(d_prime * es / 16);
        gs.rows = (int)rows;
        gs.out_f32 = samp;
        gs.out_row_stride = m;
        const hipError_t e = rows > 64 ? sv::launch_tile_mfma(gs, s, true) : sv::launch_skinny_mfma(gs, s);
        if (e != hipSuccess) return SV_ERR_HIP;
        sv::BracketArgs ba{};
        ba.hp = hp;
        ba.Wv = static_cast<const char*>(W_vocab);
        ba.chunks = gs.chunks;
        ba.V = V;
        ba.rows = (int)rows;
        ba.k = k;
        ba.idx_out = idx_out;
        ba.scratch = bscratch;
        return sv::launch_bracket_select(ba, s) == hipSuccess ? SV_OK : SV_ERR_HIP;
    }

    // Step 1a: h' = W_down h, stored in the storage dtype (bf16: rounded to nearest even); the same launch
    // clears the selection's counters and histogram
    size_t zero_words = 0;
    sv::select_zero_range(rows, V, &zero_words);
    if (launch_down_projection(h, rows, d, ldh, W_down, d_prime, dt, hp, radix, zero_words, s) != SV_OK)
        return SV_ERR_HIP;

    // Step 1b: s = W_vocab h'.  One hidden row: a bandwidth-bound stream over W_vocab fused with the
    // first histogram pass of the selection.  Several rows: a real matrix product -> matrix cores.
    const int vchunks = (int)(d_prime * es / 16);
    sv::GemvArgs g2{};
    g2.x = hp;
    g2.x_row_bytes = d_prime * es;
    g2.M = static_cast<const char*>(W_vocab);
    g2.m_row_bytes = d_prime * es;
    g2.n_items = V;
    g2.chunks = vchunks;
    g2.rows = (int)rows;
    g2.out_f32 = scores;
    g2.out_row_stride = V;
    if (sv::skinny_mfma_supported(dt, g2)) {
        if (sv::launch_skinny_mfma(g2, s) != hipSuccess) return SV_ERR_HIP;
        if (sv::launch_hist(scores, V, k, (int)rows, radix, s) != hipSuccess) return SV_ERR_HIP;
    } else if (sv::scores_supported(vchunks)) {
        sv::ScoresArgs sa{};
        sa.hp = hp;
        sa.Wv = static_cast<const char*>(W_vocab);
        sa.V = V;
        sa.k = k;
        sa.chunks = vchunks;
        sa.rows = (int)rows;
        sa.s = scores;
        if (sv::launch_scores_hist(dt, sa, radix, s) != hipSuccess) return SV_ERR_HIP;
    } else {
        if (sv::launch_gemv(dt, g2, s) != hipSuccess) return SV_ERR_HIP;
        if (sv::launch_hist(scores, V, k, (int)rows, radix, s) != hipSuccess) return SV_ERR_HIP;
    }

    // Step 2: exact top-k, ascending ids
    sv::RadixArgs ra{};
    ra.s = scores;
    ra.V = V;
    ra.rows = (int)rows;
    ra.k = k;
    ra.idx_out = idx_out;
    ra.scores_out = scores_out;
    ra.tau = tau;
    ra.scratch = radix;
    if (sv::launch_topk_of_scores(ra, s) != hipSuccess) return SV_ERR_HIP;
    return SV_OK;
}

int specvocab_select(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* W_down,
                     int64_t d_prime, const void* W_vocab, int64_t V, int dt, int64_t k,
                     int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    return select_impl(h, rows, d, ldh, W_down, d_prime, W_vocab, V, dt, k, -INFINITY, idx_out, scores_out, ws,
                       ws_bytes, stream);
}

int specvocab_init(void) { return ensure_device(); }

int specvocab_select_static(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* W_down,
                            int64_t d_prime, const void* W_vocab, int64_t V, int dt, int64_t k,
                            int32_t* idx_out, float* scores_out, void* stream) {
    // the same validation as specvocab_select, first the part that says whether the shape has a workspace size
    if (!h || !W_down || !W_vocab || !idx_out) return SV_ERR_NULL;
    const int st = check_select_shape(rows, d, V, k, d_prime, dt);
    if (st != SV_OK) return st;
    if (select_ws(rows, V, d_prime, k, dt).total > (size_t)SPECVOCAB_STATIC_SCRATCH_BYTES) return SV_ERR_WORKSPACE;
    const sv::DeviceState* dev = nullptr;
    if (sv::device_state(&dev) != hipSuccess) return SV_ERR_HIP;
    return select_impl(h, rows, d, ldh, W_down, d_prime, W_vocab, V, dt, k, -INFINITY, idx_out, scores_out,
                       dev->scratch_ptr, (size_t)SPECVOCAB_STATIC_SCRATCH_BYTES, stream);
}

int specvocab_select_threshold(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* W_down,
                               int64_t d_prime, const void* W_vocab, int64_t V, int dt, int64_t k, float tau,
                               int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    if (tau != tau) return SV_ERR_SHAPE;                        // NaN orders nothing
    return select_impl(h, rows, d, ldh, W_down, d_prime, W_vocab, V, dt, k, tau, idx_out, scores_out, ws,
                       ws_bytes, stream);
}

int specvocab_aux_log_softmax(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* W_down,
                              int64_t d_prime, const void* W_vocab, int64_t V, int dt, float* logq_out, void* ws,
                              size_t ws_bytes, void* stream) {
    if (!h || !W_down || !W_vocab || !logq_out) return SV_ERR_NULL;
    int st = check_aux_shape(rows, d, V, d_prime, dt);
    if (st != SV_OK) return st;
    st = check_row(d, ldh, dt);
    if (st != SV_OK) return st;
    if (!aligned16(h) || !aligned16(W_down) || !aligned16(W_vocab) || !aligned16(ws)) return SV_ERR_ALIGN;
    const AuxWs w = aux_ws(rows, V, d_prime, dt);
    if (!ws || ws_bytes < w.total) return SV_ERR_WORKSPACE;
    if (ensure_device() != SV_OK) return SV_ERR_HIP;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int es = esize_of(dt);
    char* hp = static_cast<char*>(ws) + w.hp_off;
    float* partial = reinterpret_cast<float*>(static_cast<char*>(ws) + w.partial_off);
    st = launch_down_projection(h, rows, d, ldh, W_down, d_prime, dt, hp, nullptr, 0, s);
    if (st != SV_OK) return st;
    // s = W_vocab h' straight into the output, then normalised in place
    sv::GemvArgs g{};
    g.x = hp;
    g.x_row_bytes = d_prime * es;
    g.M = static_cast<const char*>(W_vocab);
    g.m_row_bytes = d_prime * es;
    g.n_items = V;
    g.chunks = (int)(d_prime * es / 16);
    g.rows = (int)rows;
    g.out_f32 = logq_out;
    g.out_row_stride = V;
    st = launch_rows_product(dt, g, V, nullptr, 0, s);
    if (st != SV_OK) return st;
    if (sv::launch_log_softmax_rows(logq_out, V, (int)rows, partial, s) != hipSuccess) return SV_ERR_HIP;
    return SV_OK;
}

int specvocab_subset_logits(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* U, int64_t V,
                            int64_t ldu, int dt, const int32_t* idx, int64_t k, int idx_mode,
                            float* logits_out, void* ws, size_t ws_bytes, void* stream) {
    if (!h || !U || !idx || !logits_out) return SV_ERR_NULL;
    if (!dtype_ok(dt) || !mode_ok(idx_mode)) return SV_ERR_DTYPE;
    if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab || k < 1) return SV_ERR_SHAPE;
    int st = check_row(d, ldh, dt);
    if (st != SV_OK) return st;
    st = check_row(d, ldu, dt);
    if (st != SV_OK) return st;
    if (!aligned16(h) || !aligned16(U)) return SV_ERR_ALIGN;
    return launch_gather(dt, h, rows, d, ldh, U, V, ldu, idx, k, idx_mode, logits_out, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

int specvocab_indexed_head_naive(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* U, int64_t V,
                                 int64_t ldu, int dt, const int32_t* idx, int64_t k, int idx_mode,
                                 float* logits_out, void* ws, size_t ws_bytes, void* stream) {
    if (!h || !U || !idx || !logits_out) return SV_ERR_NULL;
    if (!dtype_ok(dt) || !mode_ok(idx_mode)) return SV_ERR_DTYPE;
    if (is_padded(idx_mode)) return SV_ERR_UNSUPPORTED;        // the comparator takes plain lists only
    if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab || k < 1) return SV_ERR_SHAPE;
    int st = check_row(d, ldh, dt);
    if (st != SV_OK) return st;
    st = check_row(d, ldu, dt);
    if (st != SV_OK) return st;
    if (!aligned16(h) || !aligned16(U) || !aligned16(ws)) return SV_ERR_ALIGN;
    const int es = esize_of(dt);
    const int64_t sets = base_mode(idx_mode) == SV_IDX_PER_ROW ? rows : 1;
    const size_t need = (size_t)sets * (size_t)k * (size_t)d * (size_t)es;
    if (!ws || ws_bytes < need) return SV_ERR_WORKSPACE;
    if (ensure_device() != SV_OK) return SV_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = validate_indices(idx, sets * k, V, s);
    if (st != SV_OK) return st;
    const int chunks = (int)(d * es / 16);
    // 1. U' = U[idx, :] written out (Figure 3a: read k rows, write k rows)
    if (sv::launch_materialize_rows(static_cast<const char*>(U), ldu * es, idx, sets * k, chunks,
                                    static_cast<char*>(ws), s) != hipSuccess)
        return SV_ERR_HIP;
    // 2. logits = U' h over the copy (read k rows again): the dense row kernel, one hidden row at a time
    for (int64_t r = 0; r < rows; ++r) {
        sv::GemvArgs g{};
        g.x = static_cast<const char*>(h) + r * ldh * es;
        g.x_row_bytes = ldh * es;
        g.M = static_cast<const char*>(ws) + (base_mode(idx_mode) == SV_IDX_PER_ROW ? (size_t)r * k * d * es : 0);
        g.m_row_bytes = d * es;
        g.idx = nullptr;
        g.n_items = k;
        g.chunks = chunks;
        g.rows = 1;
        g.out_f32 = logits_out + r * k;
        g.out_row_stride = k;
        if (sv::launch_gemv(dt, g, s) != hipSuccess) return SV_ERR_HIP;
    }
    return SV_OK;
}

int specvocab_pack_rows(const void* U, int64_t V, int64_t d, int64_t ldu, int dt, const int32_t* idx, int64_t k,
                        void* U_packed, void* stream) {
    if (!U || !idx || !U_packed) return SV_ERR_NULL;
    if (!dtype_ok(dt)) return SV_ERR_DTYPE;
    if (V < 1 || V > kMaxVocab || k < 1 || k > kMaxVocab) return SV_ERR_SHAPE;
    int st = check_row(d, ldu, dt);
    if (st != SV_OK) return st;
    if (!aligned16(U) || !aligned16(U_packed)) return SV_ERR_ALIGN;
    if (ensure_device() != SV_OK) return SV_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = validate_indices(idx, k, V, s);
    if (st != SV_OK) return st;
    const int es = esize_of(dt);
    if (sv::launch_materialize_rows(static_cast<const char*>(U), ldu * es, idx, k, (int)(d * es / 16),
                                    static_cast<char*>(U_packed), s) != hipSuccess)
        return SV_ERR_HIP;
    return SV_OK;
}

int specvocab_draft_topk(const float* logits, const int32_t* idx, int idx_mode, int64_t rows, int64_t k,
                         int64_t kd, int32_t* tok_out, float* prob_out, float* probs_full_out, void* ws,
                         size_t ws_bytes, void* stream) {
    (void)ws;
    (void)ws_bytes;
    if (!logits || !idx || !tok_out || !prob_out) return SV_ERR_NULL;
    if (!mode_ok(idx_mode)) return SV_ERR_DTYPE;
    if (rows < 1 || k < 1 || k > kMaxVocab || kd < 1 || kd > k) return SV_ERR_SHAPE;
    if (kd > SPECVOCAB_MAX_KD) return SV_ERR_UNSUPPORTED;
    if (rows > kMaxVocab) return SV_ERR_SHAPE;
    if (ensure_device() != SV_OK) return SV_ERR_HIP;

    sv::TopkArgs t{};
    t.logits = logits;
    t.idx = idx;
    t.idx_row_stride = base_mode(idx_mode) == SV_IDX_PER_ROW ? k : 0;
    t.rows = (int)rows;
    t.k = k;
    t.kd = (int)kd;
    t.tok_out = tok_out;
    t.prob_out = prob_out;
    t.probs_full_out = probs_full_out;
    if (sv::launch_softmax_topk(t, static_cast<hipStream_t>(stream)) != hipSuccess) return SV_ERR_HIP;
    return SV_OK;
}

int specvocab_draft_step(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* U, int64_t V,
                         int64_t ldu, int dt, const int32_t* idx, int64_t k, int idx_mode, int64_t kd,
                         float* logits_out, int32_t* tok_out, float* prob_out, float* probs_full_out, void* ws,
                         size_t ws_bytes, void* stream) {
    if (!h || !U || !idx || !logits_out || !tok_out || !prob_out) return SV_ERR_NULL;
    if (!dtype_ok(dt) || !mode_ok(idx_mode)) return SV_ERR_DTYPE;
    if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab || k < 1 || k > kMaxVocab || kd < 1 || kd > k)
        return SV_ERR_SHAPE;
    if (kd > SPECVOCAB_MAX_KD) return SV_ERR_UNSUPPORTED;
    int st = check_row(d, ldh, dt);
    if (st != SV_OK) return st;
    st = check_row(d, ldu, dt);
    if (st != SV_OK) return st;
    if (!aligned16(h) || !aligned16(U)) return SV_ERR_ALIGN;

    sv::TopkArgs t{};
    t.logits = logits_out;
    t.idx = idx;
    t.idx_row_stride = base_mode(idx_mode) == SV_IDX_PER_ROW ? k : 0;
    t.rows = (int)rows;
    t.k = k;
    t.kd = (int)kd;
    t.tok_out = tok_out;
    t.prob_out = prob_out;
    t.probs_full_out = probs_full_out;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // on the union path (one set per row) the top-k kernel picks each row's logits from the union's product
    // itself and writes logits_out on the way: one launch and one pass over the logits less
    sv::DeferredPick pick{};
    const bool can_pick = !is_padded(idx_mode) && sv::softmax_topk_can_pick(t);
    st = launch_gather(dt, h, rows, d, ldh, U, V, ldu, idx, k, idx_mode, logits_out, ws, ws_bytes, s,
                       can_pick ? &pick : nullptr);
    if (st != SV_OK) return st;
    if (pick.pos) {
        t.pick_pos = pick.pos;
        t.pick_zu = pick.zu;
        t.pick_zu_stride = pick.zu_stride;
        t.pick_logits_out = logits_out;
    }
    if (sv::launch_softmax_topk(t, s) != hipSuccess) return SV_ERR_HIP;
    return SV_OK;
}

int specvocab_stream_read_probe(const void* buf, size_t bytes, void* ws, size_t ws_bytes, void* stream) {
    if (!buf || !ws) return SV_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return SV_ERR_SHAPE;
    if (!aligned16(buf) || !aligned16(ws)) return SV_ERR_ALIGN;
    sv::DeviceInfo di;
    if (sv::device_info(&di) != hipSuccess) return SV_ERR_HIP;
    if (ws_bytes < (size_t)sv::stream_read_blocks(di.cus) * sizeof(uint32_t)) return SV_ERR_WORKSPACE;
    return sv::launch_stream_read(buf, bytes, static_cast<uint32_t*>(ws), static_cast<hipStream_t>(stream)) == hipSuccess
               ? SV_OK
               : SV_ERR_HIP;
}

int specvocab_dense_logits(const void* h, int64_t rows, int64_t d, int64_t ldh, const void* U, int64_t V,
                           int64_t ldu, int dt, float* logits_out, void* ws, size_t ws_bytes, void* stream) {
    if (!h || !U || !logits_out) return SV_ERR_NULL;
    if (!dtype_ok(dt)) return SV_ERR_DTYPE;
    if (rows < 1 || rows > kMaxRows || V < 1 || V > kMaxVocab) return SV_ERR_SHAPE;
    int st = check_row(d, ldh, dt);
    if (st != SV_OK) return st;
    st = check_row(d, ldu, dt);
    if (st != SV_OK) return st;
    if (!aligned16(h) || !aligned16(U)) return SV_ERR_ALIGN;
    if (ensure_device() != SV_OK) return SV_ERR_HIP;

    const int es = esize_of(dt);
    sv::GemvArgs g{};
    g.x = static_cast<const char*>(h);
    g.x_row_bytes = ldh * es;
    g.M = static_cast<const char*>(U);
    g.m_row_bytes = ldu * es;
    g.idx = nullptr;
    g.n_items = V;
    g.chunks = (int)(d * es / 16);
    g.rows = (int)rows;
    g.out_f32 = logits_out;
    g.out_row_stride = V;
    return launch_rows_product(dt, g, V, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

}  // extern "C"
