// Host-side launch interface between the C ABI (api.hip) and the kernel files.
// Every launcher only enqueues kernels on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sv {

struct DeviceInfo {
    int cus;         // compute units of the current device
    int valid;
};
// Cached per device; the first call on a device runs the library's device set-up (attributes, LDS opt-in of
// the large matrix-core kernels, address of the static scratch array) under a lock.  That first call must
// not happen while the calling thread's stream is being captured: specvocab_init() exists for that.
hipError_t device_info(DeviceInfo* out);
// opt-in of the kernel instances that need more than 64 KiB of LDS, on the current device
hipError_t configure_skinny_mfma_lds();
hipError_t configure_tile_mfma_lds();
hipError_t configure_select_lds();
hipError_t configure_union_lds();

// out[r, j] = < M[row(r, j), :], x[r, :] >  for j in [0, n_items)
//   row(r, j) = j                       if idx == nullptr   (dense)
//             = idx[r * idx_row_stride + j]                 (gathered; stride 0 = one set per step)
// M: rows of `chunks` 16-byte units, row stride m_row_bytes.  x: [rows x d], row stride x_row_bytes.
// out_f32 [rows x out_row_stride] or, if out_bf16 != nullptr, bf16 (RNE) to out_bf16 instead.
struct GemvArgs {
    const char* x;
    int64_t x_row_bytes;
    const char* M;
    int64_t m_row_bytes;
    const int32_t* idx;
    int64_t idx_row_stride;
    int64_t n_items;
    int chunks;
    int rows;
    float* out_f32;
    uint16_t* out_bf16;
    int64_t out_row_stride;
    uint32_t* zero_ptr;      // optional: words cleared by the same launch (scratch of a later kernel)
    size_t zero_words;
    int32_t* spread_ptr;     // optional: spread_n evenly spaced ids of [0, spread_V) written by the same launch,
    int64_t spread_n;        // spread_ptr[j] = floor(j * spread_V / spread_n)  (the sample of the bracketed selection)
    int64_t spread_V;
    const uint32_t* n_items_dev;   // optional (matrix-core kernel only): the item count lives on the
                                   // device; n_items is then an upper bound that sizes the grid
    int plain_order;               // matrix-core kernels: every workgroup walks the reduction from offset 0 (set when
                                   // the place of an item in the list may differ from run to run)
    int64_t m_rows;                // number of rows of M that idx may name, 0 if the caller does not say (a kernel that
                                   // keeps row offsets in 32 bits is then not used with an index list)
    int64_t n_items_min;           // with a count on the device: what the count is expected to reach at least (a hint that
                                   // saves launches, 0 if the caller has none; a smaller count is still served correctly)
    int balance_cus;               // LDS-tiled kernel, product stored: if > 0, the width of an item tile shrinks (in steps
                                   // of 32 items) so that the list's tiles fill whole rounds of this many workgroups
    int64_t gate_lo, gate_hi;      // matrix-core kernels with a count on the device, if gate_hi != 0: the launch does its
                                   // work only if gate_lo < count <= gate_hi and leaves at once otherwise (two launches
                                   // with complementary gates let the device pick the kernel that fits the count)
};
// true if this launch is the one that serves a list of n_items items
__device__ __forceinline__ bool gate_open(const GemvArgs& a, int64_t n_items) {
    return a.gate_hi == 0 || (n_items > a.gate_lo && n_items <= a.gate_hi);
}
// what a launch does for later kernels besides its product: every thread of the grid calls this once
__device__ __forceinline__ void prepare_scratch(const GemvArgs& a) {
    if (a.zero_words == 0 && a.spread_n == 0) return;
    const size_t nthr = (size_t)gridDim.x * gridDim.y * blockDim.x;
    const size_t me = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
    for (size_t i = me; i < a.zero_words; i += nthr) a.zero_ptr[i] = 0u;
    for (size_t j = me; j < (size_t)a.spread_n; j += nthr)
        a.spread_ptr[j] = (int32_t)((uint64_t)j * (uint64_t)a.spread_V / (uint64_t)a.spread_n);   // j * V < 2^63
}

// (the row-gather kernels behind launch_gemv accept idx entries of -1 = no token: such a slot reads
// row 0 and gets -inf in a float32 output; the matrix-core and union paths need lists without them)
hipError_t launch_gemv(int dt, const GemvArgs& a, hipStream_t stream);

// debug aid: number of entries of idx[0..n) outside [0, V) (padded: -1 is allowed) plus, if sorted_row_len > 0,
// the number of descents inside the lists of that length; synchronises the stream
hipError_t count_bad_indices(const int32_t* idx, int64_t n, int64_t V, bool padded, int64_t sorted_row_len,
                             hipStream_t stream, unsigned* bad_out);

// copies rows M[idx[j], :] (j < n_sets * k) into a dense [n_sets * k x chunks * 16 B] matrix
hipError_t launch_materialize_rows(const char* M, int64_t m_row_bytes, const int32_t* idx, int64_t n_rows,
                                   int chunks, char* dst, hipStream_t stream);

// the same product on the matrix cores, for several rows of x sharing one set of rows of M
bool skinny_mfma_supported(int dt, const GemvArgs& a);
hipError_t launch_skinny_mfma(const GemvArgs& a, hipStream_t stream);
// a batch of rows of x against few rows of M: reduction split over the wavefronts of a workgroup;
// also supports out_bf16 and zero_ptr
bool ksplit_rows_supported(int dt, const GemvArgs& a);
hipError_t launch_ksplit_rows(const GemvArgs& a, hipStream_t stream);
// more than 64 rows of x: LDS-tiled product (launch_skinny_mfma forwards to it); small_tiles: 128 x 128 tiles
// whatever the row count (few items: more workgroups matter more than operand reuse)
hipError_t launch_tile_mfma(const GemvArgs& a, hipStream_t stream, bool small_tiles = false);

// The tiled product with the epilogue of the bracketed selection instead of a store: nothing of the product
// is written; per hidden row r and item j the score f = out[r, j] is compared with the row's bracket
// (thr[r] = {hi, lo}):  f > hi -> bit j of the row's bit mask;  lo <= f <= hi -> (key, id) appended to the
// candidate region of (r, item tile), whose entry count goes to cnt.  Every word of bits and every cnt entry
// is written.  Any row count >= 1.
// Candidates of a (row, item tile): the first kCandFirst in a compact array (a row's are contiguous: the
// resolve pass streams them), any further ones (tied scores) in the tile-sized region of the pair.
constexpr int kCandFirst = 16;
struct BracketEpi {
    const float* thr;        // [rows][2]
    uint32_t* bits;          // [rows][words_per_row], words_per_row = item_tiles * tile_items / 32
    int64_t words_per_row;
    uint64_t* cand_first;    // [rows][item_tiles][kCandFirst]   ((ordered key << 32) | ~id)
    uint64_t* cand;          // [rows][item_tiles][tile_items]   slots kCandFirst .. of the same list
    uint32_t* cnt;           // [rows][item_tiles]
    int64_t item_tiles;
};
int bracket_tile_items(int rows);      // items per tile of the instance launch_tile_mfma_bracket picks
hipError_t launch_tile_mfma_bracket(const GemvArgs& a, const BracketEpi& ep, hipStream_t stream);

// The tiled product over ALL rows of M (a.idx == nullptr, a.n_items = V) with the pick epilogue: only
//     out[r, j] = < M[idx[r, j], :], x[r, :] >
// is stored.  Every row's list must be sorted (non-decreasing); off[r, t] = first j with idx[r, j] >= t * tile
// items (off[r, tiles] = k) says which slice of the list falls into item tile t.
struct PickEpi {
    const uint32_t* off;     // [rows][off_stride]
    int64_t off_stride;      // item tiles + 1
    const int32_t* idx;      // [rows][k]: lists in which the entries of an item tile are contiguous
    int64_t k;
    float* out;              // [rows][k], in the order of idx
};
int pick_tile_items(int rows);
hipError_t launch_tile_mfma_pick(const GemvArgs& a, const PickEpi& pk, hipStream_t stream);

// in place: s[r, :] <- log softmax(s[r, :]) for rows of V float32 scores; partial: log_softmax_ws_floats floats
size_t log_softmax_ws_floats(int64_t rows, int64_t V);
hipError_t launch_log_softmax_rows(float* s, int64_t V, int rows, float* partial, hipStream_t stream);

// Index lists with padding slots (-1): clean[p] = max(idx[p], 0), and afterwards
// logits[r, j] = -inf wherever idx(r, j) < 0 (idx_row_stride 0: one list for every row)
hipError_t launch_pad_clean(const int32_t* idx, int64_t n, int32_t* clean, hipStream_t stream);
hipError_t launch_pad_mask(const int32_t* idx, int64_t idx_row_stride, int rows, int64_t k, float* logits,
                           hipStream_t stream);

// Per-row index sets for several hidden rows (a draft tree): the union of the sets is formed on the
// device, every row of M in the union is read once and multiplied with all hidden rows on the matrix
// cores, and each (row, j) picks its logit out of that product.
// Many hidden rows with their own lists that together are likely to cover the vocabulary: the product over all
// rows of M with the pick epilogue (sorted: the caller declared the lists ascending); ws: pick_ws_bytes
bool pick_path_wanted(int dt, const GemvArgs& a, int64_t V, bool sorted);
size_t pick_ws_bytes(int64_t rows, int64_t V, int64_t k, bool sorted);
hipError_t launch_pick_logits(const GemvArgs& a, int64_t V, bool sorted, void* ws, hipStream_t stream);
bool union_path_wanted(int dt, const GemvArgs& a);
size_t union_ws_bytes(int64_t rows, int64_t V, int64_t k);
// the last step of the union path when the caller leaves it to a later kernel (the top-k kernel of a draft step):
// logit[r, j] = zu[r * zu_stride + pos[idx[r, j]]]
struct DeferredPick {
    const uint32_t* pos;
    const float* zu;
    int64_t zu_stride;
};
// defer != nullptr: everything but the pick is launched, *defer says what is left to do (a.out_f32 stays unwritten)
hipError_t launch_union_logits(const GemvArgs& a, int64_t V, void* ws, hipStream_t stream, DeferredPick* defer = nullptr);

// s[r, v] = < W_vocab[v, :], hp[r, :] > for short rows (d_prime * esize <= 1024 bytes), fused with the
// first histogram pass of the top-k selection
struct ScoresArgs {
    const char* hp;        // [rows x d_prime] in dt
    const char* Wv;        // [V x d_prime] in dt, dense rows
    int64_t V;
    int64_t k;
    int chunks;            // d_prime * esize / 16
    int rows;
    float* s;              // [rows x V]
};
bool scores_supported(int chunks);
hipError_t launch_scores_hist(int dt, const ScoresArgs& a, uint32_t* scratch, hipStream_t stream);
// the histogram pass alone, for scores produced by another kernel
hipError_t launch_hist(const float* s, int64_t V, int64_t k, int rows, uint32_t* scratch, hipStream_t stream);

// exact top-k of every row of s (after the histogram pass), ids ascending
struct RadixArgs {
    const float* s;        // [rows x V]
    int64_t V;
    int rows;
    int64_t k;
    int32_t* idx_out;      // [rows x k]
    float* scores_out;     // [rows x k] or nullptr
    float tau;             // selected entries scoring below tau are emitted as padding (-1, -inf); -inf: none
    uint32_t* scratch;     // select_scratch_words(rows, V) uint32 words; the first
                           // select_zero_range() words must be zero before the histogram pass
};
int64_t select_max_vocab();
size_t select_scratch_words(int64_t rows, int64_t V);
void select_zero_range(int64_t rows, int64_t V, size_t* words);
hipError_t launch_topk_of_scores(const RadixArgs& a, hipStream_t stream);

// Exact top-k of every row for a batch of hidden rows WITHOUT the score matrix in memory (bf16): the scores of a
// sample of the vocabulary bracket each row's k-th score, the full product is classified against the bracket
// in the epilogue of the matrix-core kernel, and the few scores inside the bracket are resolved exactly.
// Order of use: bracket_sample() says where the sample's ids and scores live in the scratch (the caller has
// the ids written -- GemvArgs::spread_* -- and the sample scores computed), then launch_bracket_select().
struct BracketArgs {
    const char* hp;        // [rows x d'] bf16
    const char* Wv;        // [V x d'] bf16, dense rows
    int chunks;            // d' * 2 / 16
    int64_t V;
    int rows;
    int64_t k;
    int32_t* idx_out;      // [rows x k]
    uint32_t* scratch;     // bracket_scratch_words(rows, V) words; nothing needs clearing
};
bool bracket_select_supported(int dt, int64_t rows, int64_t V, int64_t k);
size_t bracket_scratch_words(int64_t rows, int64_t V);
void bracket_sample(int64_t rows, int64_t V, uint32_t* scratch, int32_t** ids, int64_t* m, float** samp);
hipError_t launch_bracket_select(const BracketArgs& a, hipStream_t stream);

// measurement aid: a plain coalesced read of `bytes` (a multiple of 16) from buf; sink: stream_read_blocks() words
inline int stream_read_blocks(int cus) { return cus * 64; }
hipError_t launch_stream_read(const void* buf, size_t bytes, uint32_t* sink, hipStream_t stream);

// subset softmax + top-kd
struct TopkArgs {
    const float* logits;   // [rows x k]
    const int32_t* idx;
    int64_t idx_row_stride;  // k (per row) or 0 (per step)
    int rows;
    int64_t k;
    int kd;
    int32_t* tok_out;
    float* prob_out;
    float* probs_full_out;
    // optional: the logits are not there yet but picked by this launch from the product over the union of the rows'
    // sets, logit[r, j] = pick_zu[r * pick_zu_stride + pick_pos[idx[r, j]]], and written to pick_logits_out (the
    // same [rows x k] array that `logits` names)
    const uint32_t* pick_pos;
    const float* pick_zu;
    int64_t pick_zu_stride;
    float* pick_logits_out;
};
hipError_t launch_softmax_topk(const TopkArgs& a, hipStream_t stream);
// true if launch_softmax_topk can do the pick itself for these arguments (pick_* not looked at)
bool softmax_topk_can_pick(const TopkArgs& a);

}  // namespace sv
