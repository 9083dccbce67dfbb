// Gathered logits for several hidden rows with one index set per row (Section 3.3 Step 3 on the
// batches of hidden states of a draft tree, Section 3.5).
//
// Gathering per (row, j) pair would read a row of U once for every hidden row that wants it; the
// sets of one step overlap heavily (a tree's rows share most of their likely tokens), so the bytes
// that have to move are the UNIQUE rows of U.  Per step:
//   mark     flag[v] = 1 (a byte) for every token any row asks for              (plain stores)
//   compact  the flagged tokens become the union list, in token order, and pos[v] the token's position
//            in it: a workgroup counts the flags in front of its 4096 tokens itself (4 KB of flag bytes per
//            earlier workgroup) and prefix-sums its own, so the list is the same in every run -- with ranges
//            reserved by atomics the order of the workgroups' ranges, and with it the tile and the order of
//            the float32 additions of a token in the product, changed from run to run.  Very large
//            vocabularies (more than kOrderedMaxBlocks workgroups) keep the atomics and the product then
//            keeps its plain reduction order
//   product  every row of U in the union x all hidden rows, on the matrix cores (mfma_kernels.hip),
//            reading each needed row of U exactly once
//   pick     logits[r, j] = product[r, pos[idx[r, j]]]
// The product computes entries nobody asked for; on this part those flops are free next to the HBM
// stream, and the kernel stays a dense, coalesced read of whole rows.
//
// Many hidden rows whose sets together cover the vocabulary (a large batch, Section 3.5 "Inference"): the
// union is (nearly) everything, so there is nothing to compact, and a [rows x |union|] scratch plus a pick
// pass would move more bytes than U.  When the caller declares every row's list sorted -- what the selection
// emits -- the slice of a list that falls into an item tile is contiguous:
//   slices   off[r, t] = first j with idx[r, j] >= t * tile items;
//   product  over ALL rows of U, tile by tile, whose epilogue stores only the asked entries, straight
//            into logits_out (tile_mfma_kernels.hip).
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

constexpr int kUThreads = 1024;
constexpr int kUWaves = kUThreads / 64;
constexpr int kUEpt = 4;

constexpr int64_t kOrderedMaxBlocks = 128;          // vocabularies up to 524288 tokens: union list in token order
struct UnionWs {
    uint32_t* counter;   // [4]  number of tokens in the union (word 0)
    uint8_t* flag;       // [V]  1 = some row asks for the token
    uint32_t* pos;       // [V]  position in the union list
    int32_t* ulist;      // [V]  union list
    float* zu;           // [rows][zu_stride] product
    int64_t zu_stride;
};
__host__ __device__ inline size_t flag_words(int64_t V) { return (((size_t)V + 15) / 16) * 4; }   // 16-byte multiple
__host__ __device__ inline int64_t union_cap(int64_t rows, int64_t V, int64_t k) {
    const int64_t pairs = rows * k;
    const int64_t cap = pairs < V ? pairs : V;
    return (cap + 3) & ~(int64_t)3;
}
inline UnionWs carve(void* ws, int64_t rows, int64_t V, int64_t k) {
    UnionWs w;
    uint32_t* base = static_cast<uint32_t*>(ws);
    const size_t vpad = ((size_t)V + 3) & ~(size_t)3;
    w.counter = base;
    w.flag = reinterpret_cast<uint8_t*>(base + 4);
    w.pos = base + 4 + flag_words(V);
    w.ulist = reinterpret_cast<int32_t*>(base + 4 + flag_words(V) + vpad);
    w.zu = reinterpret_cast<float*>(base + 4 + flag_words(V) + 2 * vpad);
    w.zu_stride = union_cap(rows, V, k);
    return w;
}

__global__ __launch_bounds__(256) void clear_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

__global__ __launch_bounds__(256) void mark_kernel(const int32_t* idx, int64_t pairs, uint8_t* flag) {
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < pairs; p += (int64_t)gridDim.x * blockDim.x)
        flag[idx[p]] = 1;
}

// ORDERED: the workgroup's first slot is the number of flags in front of its tokens, counted here (the flag
// bytes are 0 or 1, so a word's population count is its number of flags); the last workgroup leaves the size
// of the union in counter[0].  Otherwise: a range reserved with one atomic per workgroup, in any order.
template <bool ORDERED>
__global__ __launch_bounds__(kUThreads) void compact_kernel(const uint8_t* flag, uint32_t* pos, int64_t V,
                                                            int32_t* ulist, uint32_t* counter) {
    __shared__ uint32_t s_w[kUWaves];
    __shared__ uint32_t s_w2[kUWaves];
    __shared__ uint32_t s_base;
    const int tid = threadIdx.x;
    const int64_t v0 = ((int64_t)blockIdx.x * kUThreads + tid) * kUEpt;
    static_assert(kUEpt == 4, "a thread's four flags are one 32-bit word");
    const uint32_t* flag_w = reinterpret_cast<const uint32_t*>(flag);         // the array is a multiple of 16 bytes long
    const uint32_t own = v0 < V ? flag_w[v0 / 4] : 0u;                        // (bytes past V are never set)
    uint32_t before_me = 0u;
    if constexpr (ORDERED) {
        // words of the earlier workgroups: kUThreads per workgroup, this thread takes one of each, eight at a time
        const int nb = (int)blockIdx.x;
        for (int b0 = 0; b0 < nb; b0 += 8) {
            uint32_t w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = flag_w[(int64_t)(b0 + u < nb ? b0 + u : nb - 1) * kUThreads + tid];
#pragma unroll
            for (int u = 0; u < 8; ++u) before_me += b0 + u < nb ? (uint32_t)__popc(w[u]) : 0u;
        }
    }
    uint32_t f[kUEpt];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < kUEpt; ++i) {
        f[i] = (v0 + i < V) ? (own >> (8 * i)) & 1u : 0u;
        mine += f[i];
    }
    const uint32_t before = block_prefix_exclusive<kUWaves>(mine, s_w);
    if constexpr (ORDERED) {
        before_me = wave_sum_u32(before_me);
        if ((tid & 63) == 0) s_w2[tid >> 6] = before_me;
    }
    if (tid == kUThreads - 1) {
        const uint32_t total = before + mine;
        if constexpr (!ORDERED) s_base = total ? atomicAdd(counter, total) : 0u;
        else s_base = total;                                   // (the last thread's inclusive sum: the workgroup's count)
    }
    __syncthreads();
    uint32_t slot;
    if constexpr (ORDERED) {
        uint32_t base = 0u;
#pragma unroll
        for (int w = 0; w < kUWaves; ++w) base += s_w2[w];
        if (blockIdx.x == gridDim.x - 1 && tid == 0) counter[0] = base + s_base;
        slot = base + before;
    } else {
        slot = s_base + before;
    }
#pragma unroll
    for (int i = 0; i < kUEpt; ++i) {
        if (f[i]) {
            ulist[slot] = (int32_t)(v0 + i);
            pos[v0 + i] = slot;
            ++slot;
        }
    }
}

// (hidden rows ride on gridDim.y: a division of the pair number by k per entry costs more than the entry's loads)
__global__ __launch_bounds__(256) void pick_kernel(const int32_t* idx, int64_t k, const uint32_t* pos, const float* zu,
                                                   int64_t zu_stride, float* out) {
    const int64_t r = blockIdx.y;
    const int32_t* list = idx + r * k;
    const float* z = zu + r * zu_stride;
    float* o = out + r * k;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < k; j += (int64_t)gridDim.x * blockDim.x)
        o[j] = z[pos[list[j]]];
}

// off[r, t] for t = 0 .. tiles (see the overview), one thread per list entry: the entry at j fills the table
// for every tile that starts after its predecessor and not after itself; the last entry also closes the row.
// A list that is not sorted (the caller's contract) leaves entries of the table unwritten or inconsistent; the
// product's epilogue clamps what it reads from it, so the result is then wrong but every access stays in bounds.
// (tile_items is a power of two, 1 << tile_shift: tile numbers by 32-bit shifts -- 64-bit divisions per entry
// made this kernel several times slower than reading the lists takes)
__global__ __launch_bounds__(256) void slice_table_kernel(const int32_t* idx, int64_t k, int tile_shift, int64_t tiles,
                                                          uint32_t* off) {
    const int64_t r = blockIdx.y;
    const int32_t* list = idx + r * k;
    uint32_t* o = off + r * (tiles + 1);
    const int last_tile = (int)tiles - 1;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < k; j += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = list[j];
        const int32_t prev = j > 0 ? list[j - 1] : 0;
        if (prev < 0) continue;                               // (negative ids: outside the contract)
        const int t_first = j > 0 ? (prev >> tile_shift) + 1 : 0;             // tiles that start after the predecessor
        int t_last = v >= 0 ? v >> tile_shift : -1;
        if (t_last > last_tile) t_last = last_tile;           // (an id past the vocabulary: the caller's contract)
        for (int t = t_first; t <= t_last; ++t) o[t] = (uint32_t)j;
        if (j == k - 1)
            for (int64_t t = (t_last < 0 ? 0 : t_last + 1); t <= tiles; ++t) o[t] = (uint32_t)k;
    }
}

// The same table for lists in ANY order, plus grouped[r, :] and perm[r, :]: the ids of row r's list grouped by
// item tile (off[r, t] .. off[r, t + 1] are the places of the entries that fall into tile t) and the positions in
// the caller's list they came from.  One workgroup per
// hidden row: count per tile in LDS, scan, scatter.  The order inside a tile's group depends on the run; every
// position appears exactly once, which is all the epilogue needs.  Ids outside [0, V) (the caller's contract)
// are counted into the first or last tile, where the epilogue finds no column for them and stores nothing.
constexpr int kBucketThreads = 1024;
constexpr int kBucketMaxTiles = 8192;                        // two LDS arrays of that many words
constexpr size_t kStageLdsBytes = 156 * 1024;                // dynamic LDS these kernels may ask for (opted in at set-up)
// STAGE: the two grouped arrays of the row are put together in LDS and stored as contiguous runs (scattered
// 4-byte stores to memory are several times slower than the whole rest of the kernel); rows too long for that
// scatter their stores.
template <bool STAGE>
__global__ __launch_bounds__(kBucketThreads) void bucket_kernel(const int32_t* idx, int64_t k, int tile_shift, int tiles,
                                                               uint32_t* off, uint32_t* perm, int32_t* grouped) {
    extern __shared__ uint32_t s_tiles[];                    // [tiles] counts, [tiles] cursors, STAGE: [k] places, [k] ids
    __shared__ uint32_t s_w[kBucketThreads / 64];
    uint32_t* s_cnt = s_tiles;
    uint32_t* s_cur = s_tiles + tiles;
    uint32_t* s_perm = s_tiles + 2 * tiles;
    int32_t* s_gid = reinterpret_cast<int32_t*>(s_perm + (STAGE ? k : 0));
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    const int32_t* list = idx + r * k;
    uint32_t* o = off + r * ((int64_t)tiles + 1);
    uint32_t* p = perm + r * k;
    int32_t* gid = grouped + r * k;
    for (int t = tid; t < tiles; t += kBucketThreads) s_cnt[t] = 0u;
    __syncthreads();
    auto tile_of = [&](int32_t v) {
        const int t = v >= 0 ? v >> tile_shift : 0;
        return t < tiles ? t : tiles - 1;
    };
    for (int64_t j = tid; j < k; j += kBucketThreads) atomicAdd(&s_cnt[tile_of(list[j])], 1u);
    __syncthreads();
    const int per = (tiles + kBucketThreads - 1) / kBucketThreads;           // consecutive tiles per thread
    uint32_t sum = 0u;
    for (int c = 0; c < per; ++c) {
        const int t = tid * per + c;
        if (t < tiles) sum += s_cnt[t];
    }
    uint32_t base = block_prefix_exclusive<kBucketThreads / 64>(sum, s_w);
    for (int c = 0; c < per; ++c) {
        const int t = tid * per + c;
        if (t < tiles) {
            const uint32_t n = s_cnt[t];
            s_cur[t] = base;
            o[t] = base;
            base += n;
        }
    }
    if (tid == 0) o[tiles] = (uint32_t)k;
    __syncthreads();
    for (int64_t j = tid; j < k; j += kBucketThreads) {
        const int32_t v = list[j];
        const uint32_t q = atomicAdd(&s_cur[tile_of(v)], 1u);
        (STAGE ? s_perm : p)[q] = (uint32_t)j;
        (STAGE ? s_gid : gid)[q] = v;
    }
    if constexpr (STAGE) {
        __syncthreads();
        for (int64_t q = tid; q < k; q += kBucketThreads) {
            p[q] = s_perm[q];
            gid[q] = s_gid[q];
        }
    }
}

// out[r, perm[r, q]] = grouped_out[r, q]: the logits back into the order of the caller's list, one workgroup per
// hidden row.  (Stored straight from the product's epilogue these scattered 4-byte stores come from all dies
// over the whole launch and reach memory as partial lines: +50 to +100 us at 512 rows x 8192.)  STAGE: the row is
// put together in LDS and stored as one contiguous run.
template <bool STAGE>
__global__ __launch_bounds__(1024) void unpermute_kernel(const float* grouped_out, const uint32_t* perm, int64_t k, float* out) {
    extern __shared__ float s_row[];                         // STAGE: [k]
    const int64_t r = blockIdx.x;
    const float* z = grouped_out + r * k;
    const uint32_t* p = perm + r * k;
    float* o = out + r * k;
    for (int64_t q = threadIdx.x; q < k; q += blockDim.x) (STAGE ? s_row : o)[p[q]] = z[q];
    if constexpr (STAGE) {
        __syncthreads();
        for (int64_t j = threadIdx.x; j < k; j += blockDim.x) o[j] = s_row[j];
    }
}

}  // namespace

// bf16, one index set per row, at least two rows, and enough gathered bytes that reading only the
// unique rows can pay for the four extra small launches (a few microseconds each).  How much the sets
// overlap is not known here.  Measured at 8 to 12 hidden rows of 8 KiB embeddings: sets that share half
// their tokens gain from about 300 MB of per-pair bytes on (537 MB: 60 us against 84), independent
// Zipf-distributed sets still lose at 500 MB (87 us against 79) because the caches absorb their overlap.
bool union_path_wanted(int dt, const GemvArgs& a) {
    if (!(dt == DT_BF16 && a.rows >= 2 && a.idx != nullptr && a.idx_row_stride != 0 && a.out_bf16 == nullptr))
        return false;
    const int64_t pairs = (int64_t)a.rows * a.n_items;
    const int64_t naive_bytes = pairs * (int64_t)a.chunks * 16;
    return pairs >= 16384 && (a.rows >= 16 || naive_bytes >= ((int64_t)512 << 20));
}

// more than 64 KiB of dynamic LDS needs an explicit opt-in per kernel and device (called once per device, outside
// any stream capture, by the library's device set-up)
hipError_t configure_union_lds() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bucket_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStageLdsBytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&unpermute_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStageLdsBytes);
    return e;
}

// Many rows whose sets are likely to cover most of the vocabulary (rows k >= 2 V), where reading all of U costs
// no more than reading the union: the product over all of U whose epilogue stores only the asked entries.  Lists
// declared ascending need only the table of slices; lists in any order are grouped by tile first, which needs
// the tile counters of a row in LDS.
static int64_t pick_tiles(int rows, int64_t V) { return (V + pick_tile_items(rows) - 1) / pick_tile_items(rows); }
bool pick_path_wanted(int dt, const GemvArgs& a, int64_t V, bool sorted) {
    return dt == DT_BF16 && a.rows > 64 && a.idx != nullptr && a.idx_row_stride != 0 && a.out_bf16 == nullptr &&
           (int64_t)a.rows * a.n_items >= 2 * V && (sorted || pick_tiles(a.rows, V) <= kBucketMaxTiles);
}
static size_t pick_table_words(int64_t rows, int64_t V) {
    return ((size_t)rows * (size_t)(pick_tiles((int)rows, V) + 1) + 3) & ~(size_t)3;
}
size_t pick_ws_bytes(int64_t rows, int64_t V, int64_t k, bool sorted) {
    return (pick_table_words(rows, V) + (sorted ? 0 : 3 * (size_t)rows * (size_t)k)) * sizeof(uint32_t);
}

hipError_t launch_pick_logits(const GemvArgs& a, int64_t V, bool sorted, void* ws, hipStream_t stream) {
    const int64_t k = a.n_items;
    const int tn = pick_tile_items(a.rows);
    const int64_t tiles = pick_tiles(a.rows, V);
    uint32_t* table = static_cast<uint32_t*>(ws);
    uint32_t* perm = sorted ? nullptr : table + pick_table_words(a.rows, V);
    int32_t* grouped = sorted ? nullptr : reinterpret_cast<int32_t*>(perm + (size_t)a.rows * (size_t)k);
    float* grouped_out = sorted ? nullptr : reinterpret_cast<float*>(grouped + (size_t)a.rows * (size_t)k);
    int tile_shift = 0;
    while ((1 << tile_shift) < tn) ++tile_shift;
    if ((1 << tile_shift) != tn) return hipErrorInvalidValue;      // tiles are 128 or 256 items
    if (sorted) {
        const unsigned sb = (unsigned)((k + 1023) / 1024);
        hipLaunchKernelGGL(slice_table_kernel, dim3(sb, (unsigned)a.rows), dim3(256), 0, stream, a.idx, k, tile_shift,
                           tiles, table);
    } else {
        if (tiles > kBucketMaxTiles) return hipErrorInvalidValue;
        const size_t plain = (size_t)2 * tiles * sizeof(uint32_t), staged = plain + (size_t)2 * k * sizeof(uint32_t);
        if (staged <= kStageLdsBytes)
            hipLaunchKernelGGL(bucket_kernel<true>, dim3((unsigned)a.rows), dim3(kBucketThreads), staged, stream, a.idx, k,
                               tile_shift, (int)tiles, table, perm, grouped);
        else
            hipLaunchKernelGGL(bucket_kernel<false>, dim3((unsigned)a.rows), dim3(kBucketThreads), plain, stream, a.idx, k,
                               tile_shift, (int)tiles, table, perm, grouped);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    GemvArgs dense = a;
    dense.idx = nullptr;
    dense.idx_row_stride = 0;
    dense.n_items = V;
    dense.out_f32 = nullptr;
    PickEpi pk{};
    pk.off = table;
    pk.off_stride = tiles + 1;
    pk.idx = sorted ? a.idx : grouped;
    pk.k = k;
    pk.out = sorted ? a.out_f32 : grouped_out;
    e = launch_tile_mfma_pick(dense, pk, stream);
    if (e != hipSuccess || sorted) return e;
    if ((size_t)k * sizeof(float) <= kStageLdsBytes)
        hipLaunchKernelGGL(unpermute_kernel<true>, dim3((unsigned)a.rows), dim3(1024), (size_t)k * sizeof(float), stream,
                           grouped_out, perm, k, a.out_f32);
    else
        hipLaunchKernelGGL(unpermute_kernel<false>, dim3((unsigned)a.rows), dim3(1024), 0, stream, grouped_out, perm, k,
                           a.out_f32);
    return hipGetLastError();
}

size_t union_ws_bytes(int64_t rows, int64_t V, int64_t k) {
    const size_t vpad = ((size_t)V + 3) & ~(size_t)3;
    return (4 + flag_words(V) + 2 * vpad + (size_t)rows * (size_t)union_cap(rows, V, k)) * sizeof(uint32_t);
}

hipError_t launch_union_logits(const GemvArgs& a, int64_t V, void* ws, hipStream_t stream, DeferredPick* defer) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    const int64_t k = a.n_items;
    const int64_t pairs = (int64_t)a.rows * k;
    const UnionWs w = carve(ws, a.rows, V, k);

    const size_t nclear = 4 + flag_words(V);              // counter + flag bytes (contiguous)
    unsigned cb = (unsigned)((nclear + 1023) / 1024);
    if (cb > (unsigned)di.cus * 4) cb = (unsigned)di.cus * 4;
    hipLaunchKernelGGL(clear_kernel, dim3(cb), dim3(256), 0, stream, w.counter, nclear);
    unsigned mb = (unsigned)((pairs + 1023) / 1024);
    if (mb > (unsigned)di.cus * 8) mb = (unsigned)di.cus * 8;
    hipLaunchKernelGGL(mark_kernel, dim3(mb), dim3(256), 0, stream, a.idx, pairs, w.flag);
    const int64_t vb = (V + kUThreads * kUEpt - 1) / (kUThreads * kUEpt);
    const bool ordered = vb <= kOrderedMaxBlocks;
    if (ordered)
        hipLaunchKernelGGL(compact_kernel<true>, dim3((unsigned)vb), dim3(kUThreads), 0, stream, w.flag, w.pos, V, w.ulist,
                           w.counter);
    else
        hipLaunchKernelGGL(compact_kernel<false>, dim3((unsigned)vb), dim3(kUThreads), 0, stream, w.flag, w.pos, V, w.ulist,
                           w.counter);

    GemvArgs u = a;                                       // product over the union list, all hidden rows
    u.idx = w.ulist;
    u.idx_row_stride = 0;
    u.n_items = w.zu_stride;                              // upper bound: sizes the grid
    u.n_items_dev = w.counter;
    u.n_items_min = k;                                    // every row's k items are in the union
    u.plain_order = ordered ? 0 : 1;                      // a list in run-dependent order: no rotated reduction
    u.out_f32 = w.zu;
    u.out_row_stride = w.zu_stride;
    e = launch_skinny_mfma(u, stream);
    if (e != hipSuccess) return e;
    if (defer) {
        defer->pos = w.pos;
        defer->zu = w.zu;
        defer->zu_stride = w.zu_stride;
        return hipSuccess;
    }

    unsigned pb = (unsigned)((k + 1023) / 1024);              // four entries per thread
    if ((int64_t)pb * a.rows > (int64_t)di.cus * 16) pb = (unsigned)(((int64_t)di.cus * 16 + a.rows - 1) / a.rows);
    hipLaunchKernelGGL(pick_kernel, dim3(pb, (unsigned)a.rows), dim3(256), 0, stream, a.idx, k, w.pos, w.zu, w.zu_stride,
                       a.out_f32);
    return hipGetLastError();
}

}  // namespace sv
