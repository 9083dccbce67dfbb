/*
 * specvocab.h -- C ABI of the SpecVocab draft-step library for AMD MI355X (gfx950).
 *
 * The library computes the draft model's output distribution over a per-step speculative
 * vocabulary (arxiv 2602.13836, Section 3): it scores the whole vocabulary with a low-rank
 * selector and keeps the k best tokens (Section 3.3, Steps 1-2), computes the exact logits of
 * those k tokens only by reading their rows of the output embedding once (Section 3.3, Step 3,
 * and "Custom kernel" in Section 3.5), and turns them into the subset softmax and the top-kd
 * draft tokens.  A full-vocabulary projection (Section 3.1) is exported as the baseline.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Memory.   Every pointer named "device" is GPU memory of the current HIP device, owned by the
 *           caller for the whole call and until the stream has finished the enqueued work.  The
 *           library allocates nothing, frees nothing and keeps no pointer after returning.
 * Layout.   Matrices are row-major.  ld* arguments are row strides in ELEMENTS.  h, U, W_down and
 *           W_vocab of one call share one storage type `dt`: SV_F32 (IEEE float32) or SV_BF16
 *           (bfloat16).  Logits, scores and probabilities are float32; token ids are int32.
 * Alignment.Base pointers of h, U, W_down, W_vocab and the workspace are 16-byte aligned; a row
 *           of h / U / W_down / W_vocab is a whole number of 16-byte units (d, d_prime multiples
 *           of 8 for bf16, of 4 for float32) and so are the row strides.
 * Stream.   `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *           enqueue work: they do not synchronise, do not read device memory on the host, and can
 *           be captured into a HIP graph.  Outputs are valid once the stream reaches that point.
 *           The first call on a device also runs a one-time device set-up (see specvocab_init); a
 *           caller whose first call would fall inside a stream capture calls specvocab_init before.
 * Workspace.`ws` is device scratch of at least specvocab_workspace_bytes(...) bytes for the same
 *           shape (may be NULL when that is 0).  Its contents need not be initialised and are
 *           undefined afterwards.  Calls that share a workspace must be ordered on one stream.
 * Errors.   Every entry point returns an sv_status.  Arguments are validated on the host before
 *           anything is enqueued; on any status other than SV_OK nothing has been launched.
 *           Index CONTENTS (range, uniqueness) are the caller's contract and are not checked --
 *           except in the debug mode switched on by the environment variable SPECVOCAB_VALIDATE=1:
 *           every call that takes an index list then first runs a range check over it, waits for
 *           the stream (so the call is no longer asynchronous nor capturable), and returns
 *           SV_ERR_INDEX without launching the operation if an entry lies outside [0, V) (a padding
 *           slot, -1, is accepted in lists passed with SV_IDX_PADDED) or if a list declared with
 *           SV_IDX_SORTED descends.
 * Precision.Products of the stored values are accumulated in float32 (order unspecified).
 *           With SV_BF16 storage the intermediate h' of the selector is rounded to bfloat16
 *           (round-to-nearest-even) before the second projection; with SV_F32 it stays float32.
 * Ties.     Wherever "largest" decides, equal values are ordered by smaller token id first.
 * Threads.  Entry points may be called from several host threads; the library keeps no per-call
 *           state on the host (only the per-device set-up, done once under a lock and read-only
 *           afterwards).  specvocab_select_static is the exception: see there.
 */
#ifndef SPECVOCAB_H
#define SPECVOCAB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPECVOCAB_VERSION 100 /* major*10000 + minor*100 + patch */

typedef enum {
    SV_OK = 0,
    SV_ERR_NULL = 1,        /* a required pointer is NULL */
    SV_ERR_SHAPE = 2,       /* a size is out of range or sizes disagree (k > V, kd > k, ld < d ...) */
    SV_ERR_DTYPE = 3,       /* unknown sv_dtype / sv_idx_mode / sv_op value */
    SV_ERR_ALIGN = 4,       /* pointer or stride not 16-byte aligned */
    SV_ERR_WORKSPACE = 5,   /* workspace missing or too small */
    SV_ERR_UNSUPPORTED = 6, /* legal in principle, not handled by this build (see each function) */
    SV_ERR_INDEX = 7,       /* debug mode only: an index lies outside [0, V) */
    SV_ERR_HIP = 8          /* a HIP runtime call (kernel launch, device query) failed */
} sv_status;

typedef enum { SV_F32 = 0, SV_BF16 = 1 } sv_dtype;

/* SV_IDX_PER_ROW: idx is [rows x k], row r of h uses idx[r, :].
 * SV_IDX_PER_STEP: idx is [k], one set shared by every row of the step. */
typedef enum { SV_IDX_PER_ROW = 0, SV_IDX_PER_STEP = 1 } sv_idx_mode;

/* Subset sizes that differ from row to row inside fixed-size lists (Section 3.3 Step 2 lets k vary).
 * OR this flag into idx_mode to say that the index list may hold PADDING SLOTS: entries equal to -1
 * name no token.  A padding slot reads no row of U, its logit is -inf and its probability 0; the real
 * entries of the row are computed exactly as without padding, and the draft top-kd behaves as on the
 * compacted list of real entries (if a row has fewer than kd of them, the remaining tok_out entries
 * are -1 with probability 0; a row of padding only gets all probabilities 0).  With one hidden
 * row (and wherever the row-gather kernel serves the call) a padded list costs nothing extra; where
 * the matrix cores multiply (several bf16 hidden rows) the gathering calls need extra workspace
 * (specvocab_workspace_bytes with the flagged idx_mode) and two small extra launches.  Lists
 * without the flag must not contain -1. */
#define SV_IDX_PADDED 4

/* OR this flag into idx_mode to DECLARE that every list is sorted by ascending id (repeats allowed), which is how
 * specvocab_select emits its lists.  A declaration, not a request: the library does not sort, and a list that is
 * not sorted then gives wrong logits (never an access out of bounds; the debug mode reports SV_ERR_INDEX).  It
 * matters for a large batch: with more than 64 bf16 hidden rows, one list per row and rows * k >= 2 V -- sets that
 * together cover the vocabulary -- the gathering calls read all of U once, tile by tile, and store only the
 * entries each row asks for.  Lists in any order take the same route between a pass that groups every list by
 * tile and one that puts the logits back into the caller's order (two more small launches, 3 rows * k more words
 * of workspace, about a tenth more time at 512 rows); the declaration saves both.  Ignored together with
 * SV_IDX_PADDED and wherever it makes no difference. */
#define SV_IDX_SORTED 8

typedef enum {
    SV_OP_SELECT = 0,
    SV_OP_SUBSET_LOGITS = 1,
    SV_OP_DRAFT_TOPK = 2,
    SV_OP_DENSE_LOGITS = 3,
    SV_OP_DRAFT_STEP = 4,
    SV_OP_INDEXED_HEAD_NAIVE = 5,
    SV_OP_AUX_LOG_SOFTMAX = 6
} sv_op;

/* Largest kd the draft top-kd accepts. */
#define SPECVOCAB_MAX_KD 64

/* SPECVOCAB_VERSION of the loaded library. */
int specvocab_version(void);

/* One-time set-up of the current HIP device: device attributes, the opt-in of the kernels that use more
 * than 64 KiB of LDS, and the device address of the static scratch array of specvocab_select_static.
 * Every entry point does this by itself on its first call on a device; call specvocab_init explicitly,
 * once per device and outside any stream capture, when that first call would otherwise happen while a
 * stream is being captured.  Idempotent and thread-safe.  Returns SV_OK or SV_ERR_HIP. */
int specvocab_init(void);

/* Static, NUL-terminated description of an sv_status value. */
const char* specvocab_status_string(int status);

/* Bytes of device workspace the given operation needs for the given shape, written to
 * *bytes_out (host pointer).  Arguments an operation does not have are ignored (pass 0).
 * 0 is a valid answer.  Returns SV_ERR_SHAPE / SV_ERR_DTYPE on sizes the operation rejects. */
int specvocab_workspace_bytes(int op, int64_t rows, int64_t d, int64_t V, int64_t k,
                              int64_t d_prime, int64_t kd, int dt, int idx_mode,
                              size_t* bytes_out);

/* Section 3.3, Steps 1 and 2: the candidate vocabulary of every row.
 *     h'[r, :] = W_down h[r, :]          W_down  device [d_prime x d], row stride d
 *     s[r, :]  = W_vocab h'[r, :]        W_vocab device [V x d_prime], row stride d_prime
 *     idx_out[r, :] = token ids of the k largest s[r, :], in ascending id order
 * h: device [rows x d], row stride ldh.  idx_out: device [rows x k] int32.
 * scores_out: device [rows x k] float32 receiving s[r, idx_out[r, j]], or NULL.
 * Requires 1 <= k <= V, 1 <= d_prime, rows >= 1; V above 4194304 is SV_ERR_UNSUPPORTED.
 * Cost.  With 65 or more bf16 hidden rows, 32768 <= V <= 393216 and scores_out == NULL the scores are never
 * written to memory: the scores of 8192 evenly spaced tokens (ids floor(j V / 8192)) bracket every row's k-th
 * score, the full product is classified against the bracket on the fly and only the few per cent of scores
 * inside it are kept and resolved exactly.  The result is the same exact top-k; a row whose bracket misses
 * (probability ~1e-9 per row on scores that do not depend on the token id modulo the sampling stride; certain
 * for inputs built so that the sampled tokens score unlike all others) is recomputed by a slow exact path,
 * about a millisecond per such row.  Every other shape, and every call with scores_out, materialises s in the
 * workspace. */
int specvocab_select(const void* h, int64_t rows, int64_t d, int64_t ldh,
                     const void* W_down, int64_t d_prime,
                     const void* W_vocab, int64_t V,
                     int dt, int64_t k,
                     int32_t* idx_out, float* scores_out,
                     void* ws, size_t ws_bytes, void* stream);

/* specvocab_select for callers that cannot allocate device memory or pass a workspace: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as specvocab_select, but the scratch memory is a static device array inside the library
 * (SPECVOCAB_STATIC_SCRATCH_BYTES per GPU the library runs on, held until the process ends) instead of a
 * workspace argument; the call allocates nothing and frees nothing.  Shapes whose
 * specvocab_workspace_bytes(SV_OP_SELECT, ...) exceeds SPECVOCAB_STATIC_SCRATCH_BYTES return
 * SV_ERR_WORKSPACE (8 MiB holds one hidden row at V up to about 600000, or four rows at V = 128256).
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents (the kernels
 * clear what must start at zero): calls that overlap on one GPU -- different streams or host threads
 * without ordering between them -- race; order them on one stream. */
#define SPECVOCAB_STATIC_SCRATCH_BYTES (8u << 20)
int specvocab_select_static(const void* h, int64_t rows, int64_t d, int64_t ldh,
                            const void* W_down, int64_t d_prime,
                            const void* W_vocab, int64_t V,
                            int dt, int64_t k,
                            int32_t* idx_out, float* scores_out, void* stream);

/* specvocab_select with a score threshold: of the k best tokens of a row only those with
 * s[r, v] >= tau stay; the others become padding slots in place (idx_out = -1, scores_out = -inf),
 * so that the list keeps its length k and its ascending id order and can be passed on with
 * SV_IDX_PADDED.  tau = -INFINITY is specvocab_select; NaN is SV_ERR_SHAPE.  Workspace as for
 * SV_OP_SELECT. */
int specvocab_select_threshold(const void* h, int64_t rows, int64_t d, int64_t ldh,
                               const void* W_down, int64_t d_prime,
                               const void* W_vocab, int64_t V,
                               int dt, int64_t k, float tau,
                               int32_t* idx_out, float* scores_out,
                               void* ws, size_t ws_bytes, void* stream);

/* Section 3.3, Step 3 (the fused indexed LM head of Section 3.5, "Custom kernel"):
 *     logits_out[r, j] = < U[idx(r, j), :], h[r, :] >
 * without materialising U[idx, :]; each needed row of U is read from memory once per use.
 * h: device [rows x d] stride ldh.  U: device [V x d] stride ldu.
 * idx: device int32, [rows x k] (SV_IDX_PER_ROW) or [k] (SV_IDX_PER_STEP), any order; every
 * entry must lie in [0, V) (caller's contract, unchecked) or, with SV_IDX_PADDED, be -1.
 * Duplicates just repeat the value.
 * logits_out: device [rows x k] float32.
 * With several hidden rows and one set per row (a draft tree) the union of the sets is formed in
 * the workspace and each needed row of U is read once per step rather than once per asking row;
 * specvocab_workspace_bytes(SV_OP_SUBSET_LOGITS, ...) says how much that needs (0 otherwise). */
int specvocab_subset_logits(const void* h, int64_t rows, int64_t d, int64_t ldh,
                            const void* U, int64_t V, int64_t ldu, int dt,
                            const int32_t* idx, int64_t k, int idx_mode,
                            float* logits_out,
                            void* ws, size_t ws_bytes, void* stream);

/* Subset softmax (Section 3.3, q_K = softmax(z')) and the top-kd draft tokens of every row
 * (inference hyper-parameter "Top-k", 10 in the paper's appendix):
 *     q[r, j]      = exp(logits[r, j] - max_j) / sum_l exp(logits[r, l] - max_j)
 *     tok_out[r,t] = idx(r, j_t), prob_out[r, t] = q[r, j_t], where j_0, j_1, ... order the row by
 *                    descending logit, equal logits by ascending token id
 * logits: device [rows x k] float32 (finite).  idx: as in specvocab_subset_logits; token ids of
 * one row must be unique.  tok_out: device [rows x kd] int32.  prob_out: device [rows x kd]
 * float32.  probs_full_out: device [rows x k] float32 receiving q, or NULL.
 * Requires 1 <= kd <= min(k, SPECVOCAB_MAX_KD), else SV_ERR_SHAPE / SV_ERR_UNSUPPORTED. */
int specvocab_draft_topk(const float* logits, const int32_t* idx, int idx_mode,
                         int64_t rows, int64_t k, int64_t kd,
                         int32_t* tok_out, float* prob_out, float* probs_full_out,
                         void* ws, size_t ws_bytes, void* stream);

/* The whole draft step after selection: specvocab_subset_logits followed by specvocab_draft_topk on
 * the logits it produced (Section 3.3 Step 3 and q_K = softmax(z'), then the top-kd tokens), with the
 * same arguments, results and tie rule as those two calls, enqueued back to back on `stream`.
 * (Two kernels on purpose: on this multi-die GPU a kernel boundary is the cheapest device-wide
 * synchronisation; a single-launch version with an in-kernel hand-over measured slower.)
 * logits_out: device [rows x k] float32, required (the top-kd stage reads it). */
int specvocab_draft_step(const void* h, int64_t rows, int64_t d, int64_t ldh,
                         const void* U, int64_t V, int64_t ldu, int dt,
                         const int32_t* idx, int64_t k, int idx_mode, int64_t kd,
                         float* logits_out, int32_t* tok_out, float* prob_out, float* probs_full_out,
                         void* ws, size_t ws_bytes, void* stream);

/* Comparator, not part of the method: the indexed LM head done the naive way the paper's kernel
 * replaces (Section 3.5 "Custom kernel", Figure 3a): U' = U[idx, :] is first materialised in the
 * workspace (k rows read and written), then logits_out = U' h is computed over the copy (k rows read
 * again).  Same arguments and results as specvocab_subset_logits; exists so that the benchmark can
 * put the fused gather next to the three-times-the-traffic path on the same GPU.
 * One index set per hidden row or per step; the workspace holds rows x k x d (or k x d) elements. */
int specvocab_indexed_head_naive(const void* h, int64_t rows, int64_t d, int64_t ldh,
                                 const void* U, int64_t V, int64_t ldu, int dt,
                                 const int32_t* idx, int64_t k, int idx_mode,
                                 float* logits_out,
                                 void* ws, size_t ws_bytes, void* stream);

/* Static-vocabulary mode (the fixed sub-vocabularies the paper compares against: Section 2 "Static
 * sub-vocabularies", the 32K-token baselines of Section 4): packs U' = U[idx, :] into a dense matrix
 * once, when the static vocabulary is chosen,
 *     U_packed[j, :] = U[idx[j], :]            j < k
 * after which every draft step is specvocab_dense_logits over U_packed (V = k) followed by
 * specvocab_draft_topk with the same idx as the token ids (SV_IDX_PER_STEP).
 * idx: device [k] int32, entries in [0, V) (caller's contract).  U_packed: device [k x d] in `dt`, row
 * stride d, 16-byte aligned, written completely; it must not overlap U. */
int specvocab_pack_rows(const void* U, int64_t V, int64_t d, int64_t ldu, int dt,
                        const int32_t* idx, int64_t k, void* U_packed, void* stream);

/* Section 3.4 (training side, forward only): the vocabulary speculator's own output distribution over
 * the ENTIRE vocabulary, q_aux = softmax(s) with s = W_vocab (W_down h) as in specvocab_select, returned
 * as natural-log probabilities (what a cross-entropy style distillation loss consumes):
 *     logq_out[r, v] = s[r, v] - log sum_u exp(s[r, u])
 * Arguments as in specvocab_select; logq_out: device [rows x V] float32.  No limit on V beyond int32. */
int specvocab_aux_log_softmax(const void* h, int64_t rows, int64_t d, int64_t ldh,
                              const void* W_down, int64_t d_prime,
                              const void* W_vocab, int64_t V, int dt,
                              float* logq_out,
                              void* ws, size_t ws_bytes, void* stream);

/* Measurement aid, not part of the method: one plain streaming read of buf (device, 16-byte aligned, `bytes` a
 * multiple of 16): every lane loads 16 bytes per instruction, consecutive lanes consecutive addresses, nothing
 * is written.  Timed over a buffer much larger than the caches it gives the read bandwidth a kernel can reach on
 * the machine, which the benchmark quotes beside the published HBM peak.  ws: 262144 bytes of device scratch. */
int specvocab_stream_read_probe(const void* buf, size_t bytes, void* ws, size_t ws_bytes, void* stream);

/* Section 3.1, the full-vocabulary baseline:  logits_out[r, v] = < U[v, :], h[r, :] >.
 * logits_out: device [rows x V] float32. */
int specvocab_dense_logits(const void* h, int64_t rows, int64_t d, int64_t ldh,
                           const void* U, int64_t V, int64_t ldu, int dt,
                           float* logits_out,
                           void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECVOCAB_H */
