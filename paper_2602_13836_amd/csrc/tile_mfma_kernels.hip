// Tiled matrix product on the matrix cores for MANY hidden-state rows (more than 32):
//     out[r, j] = < M[row(j), :], x[r, :] >      r < rows, j < n_items
// with row(j) = j (the full-vocabulary projection of Section 3.1, or the selector's score matrix of
// Section 3.3 Step 1 for a whole batch) or row(j) = idx[j] (Section 3.3 Step 3 over one set of rows
// shared by every hidden row).  bf16 storage only.
//
// With hundreds of hidden rows the product is a real contraction (Section 3.4 counts V d
// multiply-adds per hidden row): reading M once per 64 hidden rows, as the skinny kernel does, turns
// into many passes over M.  Here a workgroup owns a TM x TN tile of the output (TM hidden rows, TN
// rows of M) and walks the reduction in slices of 64 elements: both operand slices go
// global -> registers -> LDS (double buffered, one barrier per slice) and every wavefront multiplies
// its part of the tile with v_mfma_f32_32x32x16_bf16 from LDS.  LDS rows are padded to 144 bytes so
// that the 16-byte operand reads of consecutive lanes fall into distinct banks (measured: full LDS
// read rate, no bank conflicts).  Workgroups that share rows of M (the different hidden-row tiles of
// one TN block) are given consecutive slots on the same XCD, so that M comes from HBM once and from
// that die's L2 afterwards (measured: HBM traffic 1.27 x the size of M at 512 hidden rows).
//
// Three forms of the main loop.  The plain one leaves the order of loads, LDS traffic and MFMAs to the
// compiler and relies on two workgroups per CU to overlap them: best while the kernel is bound by
// the one pass over M (up to 128 hidden rows).  The other two are for tiles whose SIMDs hold one or two
// wavefronts and nothing else to hide their waits.  In the interleaved one every wavefront reads its operand
// fragments one 16-element step ahead and spreads the LDS copy of the next slice over the four steps of the
// current one (LDS writes run at a third of the read rate; a burst of them stalls the fragment
// reads), with scheduling-group fences pinning that order against the compiler's own scheduler.  In the
// alternating one (256 x 256 tiles, rows of whole slices) the two wavefronts of a SIMD take turns between
// multiplying and memory work, a barrier per turn: 5 % faster than the interleaved loop at 512 hidden rows.
#include "sv_device.h"
#include "sv_launch.h"

#include <type_traits>

namespace sv {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kTK = 64;                  // reduction elements per slice (128 bytes of a row)
constexpr int kRowB = kTK * 2 + 16;      // padded LDS row (144 B = 36 words)
constexpr int kXcds = 8;

// Wanted instruction order of one 16-element step: M MFMAs with R LDS reads, W LDS writes and W global
// loads spread evenly between them (the sizes of a scheduling group must be compile-time constants).
template <int M, int R, int W, int I>
__device__ __forceinline__ void sched_pattern() {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
    constexpr int r = (I + 1) * R / M - I * R / M;
    if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);  // LDS reads
    constexpr int w = (I + 1) * W / M - I * W / M;
    if constexpr (w > 0) {
        __builtin_amdgcn_sched_group_barrier(0x200, w, 0);                   // LDS writes
        __builtin_amdgcn_sched_group_barrier(0x020, w, 0);                   // global loads
    }
    if constexpr (I + 1 < M) sched_pattern<M, R, W, I + 1>();
}

// loops whose index must be a compile-time constant inside the body (an instruction's immediate operand)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// dst with lanes LO and HI replaced by the two halves of the wavefront-uniform mask m (two v_writelane_b32).
// The mask comes straight from a vector comparison: on this architecture a vector instruction that reads a
// scalar register written by the vector instruction just before it needs two wait states in between; the
// compiler inserts them for its own instructions, not for the operands of an asm block, hence the s_nop.
template <int LO, int HI>
__device__ __forceinline__ uint32_t write_lanes(uint32_t dst, uint64_t m) {
    static_assert(LO >= 0 && LO < 64 && HI >= 0 && HI < 64, "lanes of a 64-wide wavefront");
    asm("s_nop 1\n\tv_writelane_b32 %0, %1, %3\n\tv_writelane_b32 %0, %2, %4"
        : "+v"(dst)
        : "s"((uint32_t)m), "s"((uint32_t)(m >> 32)), "n"(LO), "n"(HI));
    return dst;
}

// 2 x + (this lane's bit of the wavefront-wide mask m): one add-with-carry whose carry-in is the mask.  The mask
// must come from a scalar instruction (see write_lanes for why not straight from a vector comparison).
__device__ __forceinline__ uint32_t shift_in_lane_bit(uint32_t x, uint64_t m) {
    uint64_t carry_out;
    asm volatile("v_addc_co_u32_e64 %0, %1, %0, %0, %2" : "+v"(x), "=s"(carry_out) : "s"(m));
    return x;
}

// LDS the bracket epilogue needs (it reuses the operand buffers after the main loop): per tile row the
// bracket and a candidate counter (16 bytes reserved), per wavefront the scores of one 32-row band
template <int GM, int GN, int WM, int WN>
constexpr size_t bracket_lds_bytes() {
    return (size_t)32 * GM * WM * 16 + (size_t)GM * GN * (16 * WN * 64) * 4;
}

// GM x GN wavefronts; each owns WM x WN MFMA tiles of 32 x 32: TM = 32 GM WM hidden rows, TN = 32 GN WN items.
// PIPE: 0 the plain main loop, 1 the interleaved, 2 the alternating one.  EPI: what happens to the product --
//   EPI_STORE    it is stored;
//   EPI_BRACKET  the epilogue of the bracketed selection (Section 3.3 Step 2 for a batch of hidden rows)
//                classifies it, nothing is stored;
//   EPI_PICK     Section 3.3 Step 3 for a batch of hidden rows with one index list each: only the entries
//                a row asks for are stored, straight to their place in logits_out.
enum { EPI_STORE = 0, EPI_BRACKET = 1, EPI_PICK = 2 };
template <int GM, int GN, int WM, int WN, int PIPE, int EPI>
__global__ __launch_bounds__(64 * GM * GN) void tile_mfma_kernel(const GemvArgs a, const BracketEpi ep, const PickEpi pk) {
    constexpr int kThreads = 64 * GM * GN;
    constexpr int kRowsPerPass = kThreads / 8;           // loader: 8 threads per 128-byte row slice
    constexpr int TM = 32 * GM * WM, TN = 32 * GN * WN;
    constexpr int QA = TM / kRowsPerPass, QB = TN / kRowsPerPass;   // 16-byte loads per thread and slice
    static_assert(TM % kRowsPerPass == 0 && TN % kRowsPerPass == 0, "tile rows must fill whole loader passes");
    constexpr int kStage = (TM + TN) * kRowB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][TM + TN][kRowB]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave / GN, wc = wave % GN;
    const int C = a.chunks;
    const int nk = (C + 7) / 8;
    const int64_t n_items = a.n_items_dev ? (int64_t)*a.n_items_dev : a.n_items;
    const int RT = (a.rows + TM - 1) / TM;
    // Width of an item tile: TN, or (a.balance_cus workgroups at a time, product stored) the smallest multiple of
    // 32 with which the list still takes as many rounds of workgroups as with TN -- 50223 items on 256 CUs: 225
    // tiles of 224 items instead of 197 of 256.  The wavefronts past that width multiply copies of the tile's last
    // row and store nothing.
    int64_t tn = TN;
    if (EPI == EPI_STORE && a.balance_cus > 0 && n_items > 0) {
        const int64_t per_round = (int64_t)TN * a.balance_cus;
        const int64_t rounds = (n_items + per_round - 1) / per_round;
        const int64_t lanes32 = (int64_t)32 * a.balance_cus * rounds;
        tn = 32 * ((n_items + lanes32 - 1) / lanes32);
    }
    const int64_t IT = (n_items + tn - 1) / tn;
    // block id -> (XCD, slot on that XCD); consecutive slots of one XCD: the RT hidden-row tiles of one item tile
    const int64_t slot = blockIdx.x / kXcds;
    const int rt = (int)(slot % RT);
    const int64_t it = (slot / RT) * kXcds + (blockIdx.x % kXcds);
    if (it >= IT || !gate_open(a, n_items)) return;
    const int64_t tile0 = it * tn;
    const int64_t tile_end = tile0 + tn < n_items ? tile0 + tn : n_items;

    // loader role: 8 threads cover the 128-byte slice of one row, 32 rows per pass
    const int piece = tid & 7, r0 = tid >> 3;
    const u32x4* pa[QA];
    const u32x4* pb[QB];
#pragma unroll
    for (int q = 0; q < QA; ++q) {
        int row = rt * TM + r0 + kRowsPerPass * q;
        if (row > a.rows - 1) row = a.rows - 1;                       // padding rows: computed, never stored
        pa[q] = reinterpret_cast<const u32x4*>(a.x + (int64_t)row * a.x_row_bytes);
    }
#pragma unroll
    for (int q = 0; q < QB; ++q) {
        int64_t item = tile0 + r0 + kRowsPerPass * q;
        if (item > tile_end - 1) item = tile_end - 1;
        const int64_t mrow = a.idx ? (int64_t)a.idx[item] : item;
        pb[q] = reinterpret_cast<const u32x4*>(a.M + mrow * a.m_row_bytes);
    }
    // Loads and stores of the pipeline are unconditional (slice and unit indices are clamped; the
    // units of a ragged last slice that lie past the row are zeroed on their way into LDS, when the
    // data has arrived anyway): without branches between them the compiler can count the loads in
    // flight and wait for exactly the oldest slice.
    // Workgroups walk the reduction in rotated order (slice ks of the walk is slice eff(ks) of the rows): rows a
    // power of two apart put the same offset of every row on the same memory channels, and workgroups that all
    // start at offset 0 keep hitting the same channels together.  With one tile of hidden rows (up to 128)
    // consecutive workgroups of one XCD start 37 slices apart (modulo the number of slices): the starts of even a
    // few dozen workgroups -- a launch of one workgroup per CU has 32 slots per XCD -- then spread over the whole
    // row.  With starts one slice apart such a
    // launch kept all its workgroups within the same 4 KB of their rows at any time: 60 rows x 50200 gathered
    // rows of 8 KB 97 us against 88, x 65536 117 against 105, all 128256 rows 201 against 192-194 (rows padded
    // to 8320 bytes had shown the same gain, which is how the channels were found out).
    // (Short reductions have nothing to spread.  a.plain_order: the place of an item in the list may vary from
    // run to run, and the order of a token's float32 additions must not.)
    // (Several tiles of hidden rows keep starts one slice apart: measured equal or better there, 512 rows 663
    // against 693 us -- the hidden-row tiles of one item tile share the rows of M through their XCD's L2, and
    // neighbouring item tiles that walk almost in step seem to help that.  One tile of 65 to 128 rows gains like
    // the smaller ones: 100 rows x 50200 items 120 -> 112 us, 128 rows x 65536 135 -> 128.)
    const int64_t rot_step = RT == 1 ? (nk % 37 ? 37 : 41) : 1;
    const int rot = nk >= 16 && !a.plain_order ? (int)((slot * rot_step) % nk) : 0;
    auto eff = [&](int ks) { const int e = min(ks, nk - 1) + rot; return e >= nk ? e - nk : e; };
    auto load = [&](int ks, u32x4 (&ga)[QA], u32x4 (&gb)[QB]) {
        const int u = min(eff(ks) * 8 + piece, C - 1);
#pragma unroll
        for (int q = 0; q < QB; ++q) gb[q] = pb[q][u];
#pragma unroll
        for (int q = 0; q < QA; ++q) ga[q] = pa[q][u];
    };
    auto store = [&](int ks, const u32x4 (&ga)[QA], const u32x4 (&gb)[QB]) {      // slice ks -> buffer ks % 2
        unsigned char* base = smem + (size_t)(ks & 1) * kStage + (size_t)r0 * kRowB + piece * 16;
        const bool past = ks >= nk || eff(ks) * 8 + piece >= C;
#pragma unroll
        for (int q = 0; q < QA; ++q)
            *reinterpret_cast<u32x4*>(base + (size_t)(kRowsPerPass * q) * kRowB) = past ? zero16() : ga[q];
#pragma unroll
        for (int q = 0; q < QB; ++q)
            *reinterpret_cast<u32x4*>(base + (size_t)(TM + kRowsPerPass * q) * kRowB) = past ? zero16() : gb[q];
    };

    f32x16_t acc[WM][WN];
#pragma unroll
    for (int m = 0; m < WM; ++m)
#pragma unroll
        for (int n = 0; n < WN; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;

    // operand role: lane = (row within the 32 x 32 tile = lane % 32, k-group = lane / 32)
    const size_t a_off = (size_t)(wr * 32 * WM + (lane & 31)) * kRowB + (lane >> 5) * 16;
    const size_t b_off = (size_t)(TM + wc * 32 * WN + (lane & 31)) * kRowB + (lane >> 5) * 16;
    auto multiply = [&](int buf) {
        const unsigned char* sa = smem + (size_t)buf * kStage + a_off;
        const unsigned char* sb = smem + (size_t)buf * kStage + b_off;
#pragma unroll
        for (int kk = 0; kk < kTK / 16; ++kk) {
            bf16x8_t af[WM], bf[WN];
#pragma unroll
            for (int m = 0; m < WM; ++m)
                af[m] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sa + (size_t)(32 * m) * kRowB + kk * 32));
#pragma unroll
            for (int n = 0; n < WN; ++n)
                bf[n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sb + (size_t)(32 * n) * kRowB + kk * 32));
#pragma unroll
            for (int m = 0; m < WM; ++m)
#pragma unroll
                for (int n = 0; n < WN; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[m], bf[n], acc[m][n], 0, 0, 0);
        }
    };
    if constexpr (PIPE == 2) {
        // Two wavefronts share a SIMD and take turns, a barrier ending every turn: while one multiplies a
        // 16-element step (nothing but its MFMAs), the other issues its memory work -- the LDS reads of its NEXT
        // step's fragments, a part of its share of the copy of the next slice into LDS, and the global loads that
        // refill the registers just copied -- and waits for none of it: whatever a wavefront issues in a memory
        // turn is known complete at the end of its following multiply turn (one s_waitcnt there, long satisfied).
        // So the multiplying wavefront never queues behind a memory instruction.
        //
        // Both groups run the same program, the second (wavefronts 4..7) one turn behind the first.  Turns are
        // numbered globally: slice s starts at turn b = 8 s, the first group has its memory turns at b + 2 m, the
        // second at b + 2 m + 1 (m = 0..3).  In memory turn m of slice s a wavefront
        //   reads the fragments of step m + 1 (m = 3: of step 0 of slice s + 1), and in m = 2 -- a slice's last
        //     reads -- waits for them at once, so that slice s is read between turns b - 2 and b + 5;
        //   copies part 1, 2 of slice s + 1 (m = 0, 1) or part 0 of slice s + 2 (m = 3): slice s is written in
        //     turns b - 10 .. b - 5 and complete at the end of b - 4 -- after the last read of slice s - 2 in the
        //     same buffer (b - 11), before its own first read (b - 2).
        static_assert(GM * GN == 8, "eight wavefronts: two per SIMD");
        constexpr int NOPS = QA + QB;                        // 16-byte units per thread and slice: first M, then x
        constexpr int PER = (NOPS + 2) / 3;                  // ... copied in three parts
        u32x4 g[NOPS];
        bf16x8_t fa[2][WM], fb[2][WN];
        // Rows are whole slices here (the launcher sends other lengths to the other loop), so no unit is ever past
        // a row's end.  A unit's address is a wavefront-uniform base (matrix + the slice's offset, kept in scalar
        // registers) plus a per-thread offset in 16-byte units that never changes: one register per unit.
        uint32_t off16[NOPS];
#pragma unroll
        for (int o = 0; o < NOPS; ++o)
            off16[o] = (uint32_t)(((o < QB ? reinterpret_cast<const char*>(pb[o]) - a.M : reinterpret_cast<const char*>(pa[o - QB]) - a.x) >> 4) + piece);
        // wavefronts w and w + 4 of a workgroup run on the same SIMD (the dispatcher deals them round robin; a
        // machine that dealt them otherwise would make the turns collide, which costs time and nothing else)
        const bool second = __builtin_amdgcn_readfirstlane(wave) >= 4;
        auto turn_ends = [&]() { asm volatile("s_barrier" ::: "memory"); };
        auto read_frags = [&](int buf, int kk, bf16x8_t (&A)[WM], bf16x8_t (&B)[WN]) {
            const unsigned char* sa = smem + (size_t)buf * kStage + a_off + kk * 32;
            const unsigned char* sb = smem + (size_t)buf * kStage + b_off + kk * 32;
#pragma unroll
            for (int m = 0; m < WM; ++m)
                A[m] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sa + (size_t)(32 * m) * kRowB));
#pragma unroll
            for (int n = 0; n < WN; ++n)
                B[n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sb + (size_t)(32 * n) * kRowB));
        };
        auto request = [&](auto oc, int ks) {               // unit o of slice ks (slices past the end: the last one again)
            constexpr int o = decltype(oc)::value;
            const char* base = (o < QB ? a.M : a.x) + (size_t)eff(ks) * (kTK * 2);
            uint32_t t = off16[o];
            asm volatile("" : "+v"(t));      // the 64-bit form of the offset is made here, not kept in registers
            g[o] = *reinterpret_cast<const u32x4*>(base + ((size_t)t << 4));
        };
        // part P of slice ks: registers -> LDS buffer ks % 2 (store_part), then the same registers <- slice ks + 1
        // (refill_part)
        auto store_part = [&](auto pc, int ks) {
            constexpr int P = decltype(pc)::value;
            constexpr int lo = P * PER, hi = (P + 1) * PER < NOPS ? (P + 1) * PER : NOPS;
            unsigned char* base = smem + (size_t)(ks & 1) * kStage + (size_t)r0 * kRowB + piece * 16;
            static_for<lo, hi>([&](auto oc) {
                constexpr int o = decltype(oc)::value;
                constexpr int row = o < QB ? TM + kRowsPerPass * o : kRowsPerPass * (o - QB);
                *reinterpret_cast<u32x4*>(base + (size_t)row * kRowB) = g[o];
            });
        };
        auto refill_part = [&](auto pc, int ks) {
            constexpr int P = decltype(pc)::value;
            constexpr int lo = P * PER, hi = (P + 1) * PER < NOPS ? (P + 1) * PER : NOPS;
            static_for<lo, hi>([&](auto oc) { request(oc, ks + 1); });
        };
        auto copy_part = [&](auto pc, int ks) { store_part(pc, ks); refill_part(pc, ks); };
        auto memory_turn = [&](auto mc, int ks) {
            constexpr int m = decltype(mc)::value;
            if constexpr (m < 3) read_frags(ks & 1, m + 1, fa[(m + 1) & 1], fb[(m + 1) & 1]);
            else read_frags((ks + 1) & 1, 0, fa[0], fb[0]);
            if constexpr (m == 3) store_part(std::integral_constant<int, 0>{}, ks + 2);
            else if constexpr (m < 2) store_part(std::integral_constant<int, m + 1>{}, ks + 1);
            else __builtin_amdgcn_s_waitcnt(0xC07F);         // the slice's last reads: done before this turn ends
            turn_ends();
        };
        // The refill of the registers a memory turn has copied is requested in the multiply turn after it, behind
        // the MFMAs: a wavefront issues in order, the address unit takes a 1 KB load per ~22 cycles and the LDS a
        // request per ~30, and in one turn the loads queued behind the LDS work -- the two units then worked one
        // after the other; now one group's loads run while the other group's LDS work does.
        auto multiply_turn = [&](auto mc, int ks) {
            constexpr int m = decltype(mc)::value;
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int n = 0; n < WN; ++n)
                    acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m & 1][i], fb[m & 1][n], acc[i][n], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (m == 3) refill_part(std::integral_constant<int, 0>{}, ks + 2);
            else if constexpr (m < 2) refill_part(std::integral_constant<int, m + 1>{}, ks + 1);
            __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): what the last memory turn issued is done
            turn_ends();
        };
        // slice 0 -> buffer 0, slice 1 -> registers; then memory turn 3 of "slice -1"
        static_for<0, NOPS>([&](auto oc) { request(oc, 0); });
        copy_part(std::integral_constant<int, 0>{}, 0);
        copy_part(std::integral_constant<int, 1>{}, 0);
        copy_part(std::integral_constant<int, 2>{}, 0);
        copy_part(std::integral_constant<int, 0>{}, 1);
        __syncthreads();
        read_frags(0, 0, fa[0], fb[0]);
        __builtin_amdgcn_s_waitcnt(0xC07F);
        if (second) turn_ends();               // the second group starts one turn later ...
        for (int ks = 0; ks < nk; ++ks) {
            static_for<0, 4>([&](auto mc) {
                memory_turn(mc, ks);
                multiply_turn(mc, ks);
            });
        }
        if (!second) turn_ends();              // ... and the first ends one turn earlier: the same count for all
    } else if constexpr (PIPE == 1) {
        // the slice is walked in four 16-element steps with the operand fragments of the next step
        // already on their way from LDS while the current step multiplies
        u32x4 ga[QA], gb[QB];
        bf16x8_t fa[2][WM], fb[2][WN];
        auto read_frags = [&](int buf, int kk, bf16x8_t (&A)[WM], bf16x8_t (&B)[WN]) {
            const unsigned char* sa = smem + (size_t)buf * kStage + a_off + kk * 32;
            const unsigned char* sb = smem + (size_t)buf * kStage + b_off + kk * 32;
#pragma unroll
            for (int m = 0; m < WM; ++m)
                A[m] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sa + (size_t)(32 * m) * kRowB));
#pragma unroll
            for (int n = 0; n < WN; ++n)
                B[n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sb + (size_t)(32 * n) * kRowB));
        };
        auto mfmas = [&](const bf16x8_t (&A)[WM], const bf16x8_t (&B)[WN]) {
#pragma unroll
            for (int m = 0; m < WM; ++m)
#pragma unroll
                for (int n = 0; n < WN; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[m], B[n], acc[m][n], 0, 0, 0);
        };
        // The copy of the next slice into LDS is cut into four parts, one per step; each part's
        // registers are reloaded with the slice after next at once.  Part 0 goes right after the
        // barrier (the buffer just read is free then), parts 1..3 in the first three steps.
        static_assert(QA % 4 == 0 && QB % 4 == 0, "the staged slice is copied in four parts");
        constexpr int PA = QA / 4, PB = QB / 4;
        auto load_part = [&](int j, int ks) {
            const int u = min(eff(ks) * 8 + piece, C - 1);
#pragma unroll
            for (int q = 0; q < PB; ++q) gb[j * PB + q] = pb[j * PB + q][u];
#pragma unroll
            for (int q = 0; q < PA; ++q) ga[j * PA + q] = pa[j * PA + q][u];
        };
        auto store_part = [&](int j, int ks) {
            unsigned char* base = smem + (size_t)(ks & 1) * kStage + (size_t)r0 * kRowB + piece * 16;
            const bool past = ks >= nk || eff(ks) * 8 + piece >= C;
#pragma unroll
            for (int q = 0; q < PA; ++q)
                *reinterpret_cast<u32x4*>(base + (size_t)(kRowsPerPass * (j * PA + q)) * kRowB) = past ? zero16() : ga[j * PA + q];
#pragma unroll
            for (int q = 0; q < PB; ++q)
                *reinterpret_cast<u32x4*>(base + (size_t)(TM + kRowsPerPass * (j * PB + q)) * kRowB) = past ? zero16() : gb[j * PB + q];
        };
        // one step: fragment reads of the next step, a quarter of the slice copy, and this step's MFMAs,
        // interleaved so that every memory instruction issues in the shadow of a running MFMA
        auto interleave = [&]() {
            sched_pattern<WM * WN, WM + WN, PA + PB, 0>();
            __builtin_amdgcn_sched_barrier(0);
        };
        load(0, ga, gb);
        store(0, ga, gb);
        load(1, ga, gb);
        __syncthreads();
        store_part(0, 1);
        load_part(0, 2);
        read_frags(0, 0, fa[0], fb[0]);
        for (int ks = 0; ks < nk; ++ks) {
            const int buf = ks & 1;
            read_frags(buf, 1, fa[1], fb[1]);
            store_part(1, ks + 1);
            load_part(1, ks + 2);
            mfmas(fa[0], fb[0]);
            interleave();
            read_frags(buf, 2, fa[0], fb[0]);
            store_part(2, ks + 1);
            load_part(2, ks + 2);
            mfmas(fa[1], fb[1]);
            interleave();
            read_frags(buf, 3, fa[1], fb[1]);
            store_part(3, ks + 1);
            load_part(3, ks + 2);
            mfmas(fa[0], fb[0]);
            interleave();
            __syncthreads();     // slice ks + 1 is complete in the other buffer; this one is free again
            read_frags(buf ^ 1, 0, fa[0], fb[0]);
            store_part(0, ks + 2);
            load_part(0, ks + 3);
            mfmas(fa[1], fb[1]);
            interleave();
        }
    } else {
        // Two register sets keep two slices in flight from global memory while a third is multiplied
        // out of LDS: on entry to step(ks, set) the set holds slice ks + 1 (the other set slice ks + 2).
        u32x4 ga0[QA], gb0[QB], ga1[QA], gb1[QB];
        auto step = [&](int ks, u32x4 (&ga)[QA], u32x4 (&gb)[QB]) {
            multiply(ks & 1);
            store(ks + 1, ga, gb);            // the other buffer: nobody reads it during this slice
            __syncthreads();                  // everyone is done with this buffer; the other is complete
            load(ks + 3, ga, gb);
        };
        load(0, ga0, gb0);
        store(0, ga0, gb0);
        load(1, ga0, gb0);
        load(2, ga1, gb1);
        __syncthreads();
        for (int ks = 0; ks < nk; ks += 2) {  // an odd slice count runs one more step, on a slice of zeros
            step(ks, ga0, gb0);
            step(ks + 1, ga1, gb1);
        }
    }

    // D[i][j]: j = lane % 32 (item), i = 8 (e / 4) + 4 (lane / 32) + e % 4 (hidden row) for element e
    const int64_t item0 = tile0 + wc * 32 * WN + (lane & 31);
    const int row0 = rt * TM + wr * 32 * WM + 4 * (lane >> 5);
    if constexpr (EPI == EPI_PICK) {
        // Band by band (the 32 GM rows that the wavefronts hold in the same accumulator group) the product goes
        // to LDS as a [32 GM x TN] tile; then 8 (4) threads per row walk the entries of the row's index list that
        // fall into this item tile -- places pk.off[r, it] .. pk.off[r, it + 1] of the list (ascending, or a copy
        // grouped by tile: all that matters here is that a tile's entries are contiguous) -- and store the asked
        // entries at the same places of the output.
        constexpr int kBandRows = 32 * GM;
        constexpr int kPerRow = kThreads / kBandRows;
        static_assert((size_t)kBandRows * TN * 4 <= (size_t)2 * kStage, "the band tile reuses the operand buffers");
        float* s_band = reinterpret_cast<float*>(smem);
        const int br = tid / kPerRow, sub = tid % kPerRow;                // this thread's row of the band
        const int tile_row0 = (br / 32) * 32 * WM + (br % 32);            // + 32 m: its row of the tile
#pragma unroll
        for (int m = 0; m < WM; ++m) {
            const int r = rt * TM + tile_row0 + 32 * m;
            // the slice bounds are requested before the barrier: their latency overlaps the copy to LDS
            uint32_t ja = 0u, jb = 0u;
            if (r < a.rows) {
                ja = pk.off[(int64_t)r * pk.off_stride + it];
                jb = pk.off[(int64_t)r * pk.off_stride + it + 1];
                if (jb > (uint32_t)pk.k) jb = (uint32_t)pk.k;             // (a table built from an unsorted list: stay in bounds)
            }
            __syncthreads();                               // the band tile (or, first, the operand buffers) is free
#pragma unroll
            for (int n = 0; n < WN; ++n)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    s_band[(wr * 32 + 8 * (e >> 2) + (e & 3) + 4 * (lane >> 5)) * TN + wc * 32 * WN + 32 * n + (lane & 31)] =
                        acc[m][n][e];
            __syncthreads();
            const int32_t* list = pk.idx + (int64_t)r * pk.k;
            float* o = pk.out + (int64_t)r * pk.k;
            for (uint32_t j = ja + sub; j < jb; j += kPerRow) {
                const uint32_t col = (uint32_t)(list[j] - (int32_t)(it * TN));
                if (col < (uint32_t)TN) o[j] = s_band[br * TN + col];     // always true for a consistent table
            }
        }
        return;
    }
    if constexpr (EPI == EPI_BRACKET) {
        // Nothing of the product is stored.  Per accumulator register (64 scores: 32 items of two hidden rows)
        // two comparisons with the rows' brackets give two lane masks:
        //   above hi  -> 2 x 32 bits of the rows' bit masks, gathered lane = row so that one store per wavefront
        //                and 64 rows writes them;
        //   in band   -> the (rare) lanes append (score, position) to a wavefront-private LDS list, which is
        //                emptied after every 32-row band by a dense loop that turns each entry into
        //                (key, id) in the candidate region of its (row, item tile).
        static_assert(WM % 2 == 0, "a lane collects the words of rows lane, lane + 64, ...");
        static_assert(16 * WN == 32, "the registers of a 32-row band map to the 32 bits of one word per lane");
        static_assert(bracket_lds_bytes<GM, GN, WM, WN>() <= (size_t)2 * kStage, "the epilogue reuses the operand buffers");
        float2* s_thr = reinterpret_cast<float2*>(smem);                          // [TM] {hi, lo}
        uint32_t* s_cnt = reinterpret_cast<uint32_t*>(smem + (size_t)TM * 8);     // [TM] candidates of the row in this tile
        // per wavefront: the scores of one 32-row band, [16 WN / 4 register quads][64 lanes][4 floats]
        f32x4_t* s_dump = reinterpret_cast<f32x4_t*>(smem + (size_t)TM * 16) + (size_t)wave * (4 * WN * 64);
        __syncthreads();                                   // every wavefront is out of the operand buffers
        for (int t = tid; t < TM; t += kThreads) {
            const int row = rt * TM + t;
            // rows past the end: nothing is above +inf, nothing reaches +inf
            s_thr[t] = row < a.rows ? reinterpret_cast<const float2*>(ep.thr)[row] : float2{INFINITY, INFINITY};
            s_cnt[t] = 0u;
        }
        if (it == IT - 1) {                                // items past the end compare false with everything
#pragma unroll
            for (int n = 0; n < WN; ++n)
                if (item0 + 32 * n >= n_items) {
#pragma unroll
                    for (int m = 0; m < WM; ++m)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[m][n][e] = __builtin_nanf("");
                }
        }
        __syncthreads();
        uint32_t words[WM / 2][WN];
#pragma unroll
        for (int j = 0; j < WM / 2; ++j)
#pragma unroll
            for (int n = 0; n < WN; ++n) words[j][n] = 0u;
        // candidate regions of this tile's rows: region of tile row t at cand_tile + t * row_stride (32-bit
        // arithmetic below: 64-bit multiplications per candidate cost more than everything else there)
        uint64_t* cand_tile = ep.cand + ((int64_t)rt * TM * ep.item_tiles + it) * TN;
        const uint32_t row_stride = (uint32_t)(ep.item_tiles * TN);          // < 2^24 (the vocabulary, padded)
        uint64_t* first_tile = ep.cand_first + ((int64_t)rt * TM * ep.item_tiles + it) * kCandFirst;
        const uint32_t first_stride = (uint32_t)(ep.item_tiles * kCandFirst);
        static_for<0, WM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int kHalfRows = 4;                   // lanes 32..63 hold the row four below
            float2 th[16];                                 // the brackets of this band's rows: one batch of LDS reads
#pragma unroll
            for (int e = 0; e < 16; ++e)
                th[e] = s_thr[wr * 32 * WM + 32 * m + 8 * (e >> 2) + (e & 3) + kHalfRows * (lane >> 5)];
            // the band's scores go to LDS as they are (the few lanes inside a bracket fetch theirs from there below)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                for (int n = 0; n < WN; ++n)
                    s_dump[(q4 * WN + n) * 64 + lane] = f32x4_t{acc[m][n][4 * q4], acc[m][n][4 * q4 + 1], acc[m][n][4 * q4 + 2], acc[m][n][4 * q4 + 3]};
            uint32_t inside = 0u;                          // per lane: bit 31 - (e WN + n) <=> score inside its row's bracket
            static_for<0, 16>([&](auto ec) {
                constexpr int e = decltype(ec)::value;
                constexpr int rlo = 32 * m + 8 * (e >> 2) + (e & 3);      // row within the wavefront's rows, lanes 0..31
                static_for<0, WN>([&](auto nc) {
                    constexpr int n = decltype(nc)::value;
                    const float f = acc[m][n][e];
                    const uint64_t ma = __builtin_amdgcn_ballot_w64(f > th[e].x);
                    const uint64_t mi = __builtin_amdgcn_ballot_w64(f >= th[e].y);
                    static_assert(rlo / 64 == (rlo + kHalfRows) / 64, "both rows of a register belong to the same lane group");
                    words[rlo / 64][n] = write_lanes<rlo % 64, (rlo + kHalfRows) % 64>(words[rlo / 64][n], ma);
                    // inside = 2 inside + (this lane's bit of the mask): one add-with-carry whose carry-in is the mask
                    inside = shift_in_lane_bit(inside, mi & ~ma);
                });
            });
            // The lanes with scores inside their bracket (about one per lane and band) take them out, up to four
            // per round with the four LDS reads, the four slot reservations and the four stores each issued
            // together: one round is the common case, and its latencies are paid once instead of per score.
            while (__builtin_amdgcn_ballot_w64(inside != 0u)) {
                constexpr int kPer = 4;
                int q[kPer];
                bool has[kPer];
#pragma unroll
                for (int u = 0; u < kPer; ++u) {
                    has[u] = inside != 0u;
                    q[u] = has[u] ? __clz((int)inside) : 0;               // e WN + n of the highest set bit
                    inside &= ~(0x80000000u >> q[u]);                     // (clears bit 31 of a word that is already 0)
                }
                float f[kPer];
                int row_t[kPer];
#pragma unroll
                for (int u = 0; u < kPer; ++u) {
                    const int e = q[u] / WN, n = q[u] % WN;
                    f[u] = reinterpret_cast<const float*>(s_dump)[(((e >> 2) * WN + n) * 64 + lane) * 4 + (e & 3)];
                    row_t[u] = wr * 32 * WM + 32 * m + 8 * (e >> 2) + (e & 3) + 4 * (lane >> 5);
                }
                uint32_t slot[kPer];
#pragma unroll
                for (int u = 0; u < kPer; ++u) slot[u] = has[u] ? atomicAdd(&s_cnt[row_t[u]], 1u) : 0u;   // < TN
#pragma unroll
                for (int u = 0; u < kPer; ++u) {
                    if (has[u]) {
                        const uint32_t item = (uint32_t)item0 + 32u * (uint32_t)(q[u] % WN);
                        uint64_t* dst = slot[u] < (uint32_t)kCandFirst
                                            ? first_tile + (__umul24((uint32_t)row_t[u], first_stride) + slot[u])
                                            : cand_tile + (__umul24((uint32_t)row_t[u], row_stride) + slot[u]);
                        *dst = ((uint64_t)f32_to_ord(f[u]) << 32) | (uint32_t)(~item);
                    }
                }
            }
        });
        // lane l stores the words of the wavefront's rows l, l + 64, ...
#pragma unroll
        for (int j = 0; j < WM / 2; ++j) {
            const int row = rt * TM + wr * 32 * WM + 64 * j + lane;
            if (row < a.rows) {
                uint32_t* o = ep.bits + (int64_t)row * ep.words_per_row + it * (TN / 32) + wc * WN;
#pragma unroll
                for (int n = 0; n < WN; ++n) o[n] = words[j][n];
            }
        }
        __syncthreads();                                   // all candidates of the tile are counted
        for (int t = tid; t < TM; t += kThreads) {
            const int row = rt * TM + t;
            if (row < a.rows) ep.cnt[(int64_t)row * ep.item_tiles + it] = s_cnt[t];
        }
        return;
    }
#pragma unroll
    for (int m = 0; m < WM; ++m)
#pragma unroll
        for (int n = 0; n < WN; ++n) {
            const int64_t item = item0 + 32 * n;
            if (item >= tile_end) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = row0 + 32 * m + 8 * (e >> 2) + (e & 3);
                if (r < a.rows) a.out_f32[(int64_t)r * a.out_row_stride + item] = acc[m][n][e];
            }
        }
}

template <int GM, int GN, int WM, int WN>
constexpr size_t tile_lds_bytes() { return (size_t)2 * (32 * GM * WM + 32 * GN * WN) * kRowB; }

// more than 64 KiB of dynamic LDS needs an explicit opt-in per kernel instance and device
template <int GM, int GN, int WM, int WN, int PIPE, int EPI>
hipError_t opt_in_lds() {
    if (tile_lds_bytes<GM, GN, WM, WN>() <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&tile_mfma_kernel<GM, GN, WM, WN, PIPE, EPI>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)tile_lds_bytes<GM, GN, WM, WN>());
}

template <int GM, int GN, int WM, int WN, int PIPE, int EPI = EPI_STORE>
hipError_t launch_tile(const GemvArgs& a, hipStream_t stream, const BracketEpi& ep = BracketEpi{},
                       const PickEpi& pk = PickEpi{}) {
    constexpr int TM = 32 * GM * WM, TN = 32 * GN * WN;
    const int64_t RT = (a.rows + TM - 1) / TM;
    int64_t IT = (a.n_items + TN - 1) / TN;
    if (EPI == EPI_STORE && a.balance_cus > 0)                  // narrower tiles: whole rounds of balance_cus workgroups
        IT = (IT + a.balance_cus - 1) / a.balance_cus * a.balance_cus;
    const int64_t groups = (IT + kXcds - 1) / kXcds;            // item tiles per XCD, rounded up
    const int64_t bx = groups * RT * kXcds;
    if (bx > 0x7fffffffLL) return hipErrorInvalidValue;         // more tiles than a grid dimension holds
    const size_t lds = tile_lds_bytes<GM, GN, WM, WN>();     // above 64 KiB: opted in by configure_tile_mfma_lds()
    hipLaunchKernelGGL((tile_mfma_kernel<GM, GN, WM, WN, PIPE, EPI>), dim3((unsigned)bx), dim3(64 * GM * GN), lds, stream,
                       a, ep, pk);
    return hipGetLastError();
}

}  // namespace

// every instance launch_tile_mfma can pick, on the current device (called once per device, outside any
// stream capture, by the library's device set-up)
hipError_t configure_tile_mfma_lds() {
    hipError_t e = hipSuccess;
    auto all_epilogues = [&](auto fn) {
        if (e == hipSuccess) e = fn(std::integral_constant<int, EPI_STORE>{});
        if (e == hipSuccess) e = fn(std::integral_constant<int, EPI_BRACKET>{});
        if (e == hipSuccess) e = fn(std::integral_constant<int, EPI_PICK>{});
    };
    if (e == hipSuccess) e = opt_in_lds<1, 8, 2, 1, 0, EPI_STORE>();
    if (e == hipSuccess) e = opt_in_lds<2, 4, 2, 2, 0, EPI_STORE>();
    all_epilogues([](auto ec) { return opt_in_lds<2, 2, 2, 2, 0, decltype(ec)::value>(); });
    all_epilogues([](auto ec) { return opt_in_lds<2, 2, 2, 2, 1, decltype(ec)::value>(); });
    all_epilogues([](auto ec) { return opt_in_lds<2, 4, 4, 2, 1, decltype(ec)::value>(); });
    all_epilogues([](auto ec) { return opt_in_lds<2, 4, 4, 2, 2, decltype(ec)::value>(); });
    return e;
}

// The loop in which two wavefronts of a SIMD take turns handles rows that are whole 64-element slices (a short
// reduction such as the selector's 256 elements runs equally fast in either loop).  Both loops add a token's
// products in the same order, so the choice never changes a result.
static bool turns_fit(const GemvArgs& a) {
    // ... and keeps every row's offset from its matrix in 32 bits of 16-byte units
    const int64_t m_rows = a.idx ? a.m_rows : a.n_items;
    constexpr int64_t kSpan = (int64_t)1 << 36;
    return a.chunks % 8 == 0 && m_rows > 0 && m_rows <= kSpan / a.m_row_bytes && a.rows <= kSpan / a.x_row_bytes;
}

// the same choice of instance as launch_tile_mfma, so that both compute bit-identical products
static int tile_instance(int rows) {
    if (rows <= 128) return 0;                                 // 128 x 128, compiler-ordered loop
    const int pad256 = (rows + 255) / 256 * 256, pad128 = (rows + 127) / 128 * 128;
    return pad256 == pad128 ? 2 : 1;                           // 256 x 256 / 128 x 128, hand-ordered loop
}

int bracket_tile_items(int rows) { return tile_instance(rows) == 2 ? 256 : 128; }

hipError_t launch_tile_mfma_bracket(const GemvArgs& a, const BracketEpi& ep, hipStream_t stream) {
    if (a.n_items <= 0 || a.rows <= 0) return hipSuccess;
    switch (tile_instance(a.rows)) {
        case 0: return launch_tile<2, 2, 2, 2, 0, EPI_BRACKET>(a, stream, ep);
        case 1: return launch_tile<2, 2, 2, 2, 1, EPI_BRACKET>(a, stream, ep);
        default:
            return turns_fit(a) ? launch_tile<2, 4, 4, 2, 2, EPI_BRACKET>(a, stream, ep)
                                : launch_tile<2, 4, 4, 2, 1, EPI_BRACKET>(a, stream, ep);
    }
}

int pick_tile_items(int rows) { return bracket_tile_items(rows); }

hipError_t launch_tile_mfma_pick(const GemvArgs& a, const PickEpi& pk, hipStream_t stream) {
    if (a.n_items <= 0 || a.rows <= 0) return hipSuccess;
    switch (tile_instance(a.rows)) {
        case 0: return launch_tile<2, 2, 2, 2, 0, EPI_PICK>(a, stream, BracketEpi{}, pk);
        case 1: return launch_tile<2, 2, 2, 2, 1, EPI_PICK>(a, stream, BracketEpi{}, pk);
        default:
            return turns_fit(a) ? launch_tile<2, 4, 4, 2, 2, EPI_PICK>(a, stream, BracketEpi{}, pk)
                                : launch_tile<2, 4, 4, 2, 1, EPI_PICK>(a, stream, BracketEpi{}, pk);
    }
}

hipError_t launch_tile_mfma(const GemvArgs& a, hipStream_t stream, bool small_tiles) {
    if (a.n_items <= 0 || a.rows <= 0) return hipSuccess;
    // Up to 64 hidden rows (the caller decides when this beats the kernel without LDS tiles) the product is one
    // pass over M at the rate of the memory system, and what matters is how evenly the list's items spread over
    // the chip.  17 to 32 rows: 32 x 64 tiles (two wavefronts, five workgroups per CU).  33 to 64 rows: 64 x 256
    // tiles (eight wavefronts, one workgroup per CU) stream best when the list fills its last round of 256 x CUs
    // items, or more than half of it (a tree step of 60 rows over 50223 rows of U: 110 against 113 us with the
    // tiles below; all 128256 rows: 197 against 200) -- and for a count on the device, which such a tree step has;
    // otherwise small tiles with several workgroups per CU: 64 x 64 (four per CU) up to 64 x CUs items, 64 x 128
    // (four wavefronts, two per CU) beyond.  60 rows, 64 x 64 / 64 x 128 / 64 x 256: 16384 items 37 / 44 / 61 us,
    // 32768 59 / 60 / 76, 81920 150 / 144 / 161, 98304 186 / 160 / 170.
    if (a.rows <= 32) return launch_tile<1, 2, 1, 1, 0>(a, stream);
    if (a.rows <= 64) {
        DeviceInfo di;
        const hipError_t e = device_info(&di);
        if (e != hipSuccess) return e;
        const int64_t round_items = (int64_t)256 * di.cus, last = a.n_items % round_items;
        // (with a count on the device a.n_items is its upper bound: at most half a round, and the list is short for sure)
        const bool unknown = a.n_items_dev != nullptr && 2 * a.n_items > round_items;
        if (unknown || last == 0 || 2 * last > round_items) {
            // ... of a width that fills whole rounds of workgroups (40960 items: 80 against 87 us; unions of 30940 and
            // 44831 rows: a tree step in 82 and 104 us against 88 and 109)
            GemvArgs b = a;
            b.balance_cus = di.cus;
            return launch_tile<1, 8, 2, 1, 0>(b, stream);
        }
        return a.n_items <= (int64_t)64 * di.cus ? launch_tile<1, 2, 2, 1, 0>(a, stream) : launch_tile<1, 4, 2, 1, 0>(a, stream);
    }
    if (small_tiles) return a.rows <= 128 ? launch_tile<2, 2, 2, 2, 0>(a, stream) : launch_tile<2, 2, 2, 2, 1>(a, stream);
    // Up to 128 hidden rows the work is bound by streaming M once: small tiles, two workgroups per
    // CU.  Beyond that the 256 x 256 tile halves the operand traffic per multiply-add -- unless rounding
    // the row count up to 256s would add a whole idle half-tile that 128-row tiles avoid.
    switch (tile_instance(a.rows)) {
        case 0: {
            // 65 to 128 hidden rows: 128 x 256 tiles with eight wavefronts and one workgroup per CU stream 3-8 %
            // faster than two workgroups of 128 x 128 (128 rows x 128256: 244 against 261 us) -- when the list fills
            // its last round of 256 x CUs items more than half, like the 64-row tiles; else they lose up to a third
            // (100 rows x 16384 items: 82 against 61 us).  A count on the device: the smaller tiles.
            DeviceInfo di;
            const hipError_t e = device_info(&di);
            if (e != hipSuccess) return e;
            const int64_t round_items = (int64_t)256 * di.cus, last = a.n_items % round_items;
            if (a.n_items_dev == nullptr && (last == 0 || 2 * last > round_items)) return launch_tile<2, 4, 2, 2, 0>(a, stream);
            return launch_tile<2, 2, 2, 2, 0>(a, stream);
        }
        case 1: return launch_tile<2, 2, 2, 2, 1>(a, stream);
        default: return turns_fit(a) ? launch_tile<2, 4, 4, 2, 2>(a, stream) : launch_tile<2, 4, 4, 2, 1>(a, stream);
    }
}

}  // namespace sv
