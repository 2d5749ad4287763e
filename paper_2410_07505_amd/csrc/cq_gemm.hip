// W8A8 linear layer Y = X . W on integer codes (Background section): INT8 MFMA GEMM with int32
// accumulation and the scale epilogue  Y_ik = fl16(fl32(fl32(float(acc_ik) * a_i) * s_k)).
//
// Both operands are stored with the contraction axis contiguous (qx [T][I], qw [O][I]), which is
// the layout the INT8 matrix instructions want: every lane supplies 16 consecutive bytes of one row.
//
// Two kernels, same results (integer accumulation is exact, so tiling and order cannot matter):
//   - gemm_i8_ring_kernel, the fast path: 16-byte aligned operands, K a multiple of 128, any T (edge tiles
//     read clamped rows and drop the surplus outputs).  512 threads = 8 waves in a 2 x 4 arrangement, each
//     wave owning 128 x 64 = 8 x 4 MFMA tiles of 16 x 16 (128 accumulator registers); operands go from
//     global memory straight into a five-slot LDS ring (described at the kernel); one block per CU walks over
//     several tiles, requesting the next tile's first operands before it scales and stores the current one, and
//     the results leave straight from the accumulator registers (8 bytes per lane, whole 128-byte lines per
//     16 lanes); a last round of tiles that is at most half full runs as 256 x 128 half tiles;
//   - gemm_i8_kernel<true>, any shape and alignment: 256 threads = 4 waves in a 2 x 2 arrangement
//     (128 x 128 per wave), two LDS stages of (256 + 256) rows x 128 B = 128 KiB; the next K step
//     is fetched into registers (bounds-checked) while the current one is multiplied, then stored
//     to the other stage: one barrier per K step.
// Common to both:
//   - block tile 256 x 256, K step 128 bytes;
//   - LDS rows are 128 B = 8 chunks of 16 B, stored at chunk ^ ((row >> 1) & 7) so that the 16
//     rows a quarter-wave reads (and the row pairs it writes) fall in 16 distinct bank groups of the
//     64-bank LDS (the ring kernel's weight tile differs in one detail, see its loader);
//   - block -> tile mapping: consecutive block ids land on different XCDs, so ids are first
//     de-interleaved by XCD (each XCD gets a contiguous range of tiles, hence its own L2 sees a
//     compact patch), then walked in groups of 4 tile-rows so that concurrently resident tiles
//     share A rows and B columns.
#include <algorithm>
#include <type_traits>

#include "cq_gemm_common.h"

namespace cq {
namespace {

constexpr int BK = 128;
constexpr int kThreads = 256;
constexpr int kStageBytes = (BM + BN) * BK;       // 64 KiB
constexpr int kLdsBytes = 2 * kStageBytes;         // 128 KiB

__device__ __forceinline__ int swz(int row, int chunk) { return (chunk ^ ((row >> 1) & 7)) * 16; }

// one 16-byte chunk of row `row`, bytes [kb, kb+16) of an int8 matrix with `ld` = I bytes per row
template <bool GENERIC>
__device__ __forceinline__ v4i load_chunk(const int8_t* __restrict__ base, int row, int nrows, int kb, int I,
                                          bool vec) {
    v4i v = {0, 0, 0, 0};
    if (!GENERIC) {
        v = *reinterpret_cast<const v4i*>(base + (int64_t)row * I + kb);
    } else if (row < nrows && kb < I) {
        const int8_t* p = base + (int64_t)row * I + kb;
        if (vec && kb + 16 <= I) {
            v = *reinterpret_cast<const v4i*>(p);
        } else {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            for (int e = 0; e < 16; ++e)
                if (kb + e < I) w[e >> 2] |= (uint32_t)(uint8_t)p[e] << (8 * (e & 3));
            v = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        }
    }
    return v;
}

template <bool GENERIC>
__global__ void __launch_bounds__(kThreads)
gemm_i8_kernel(const int8_t* __restrict__ qx, const float* __restrict__ row_scale, const int8_t* __restrict__ qw,
               const float* __restrict__ w_scale, int T, int I, int O, uint16_t* __restrict__ Y, int64_t ldy,
               int32_t* __restrict__ acc_debug, int tiles_m, int tiles_n, bool vec) {
    extern __shared__ __align__(16) int8_t lds[];

    // ---- block id -> tile
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const int L = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (L >= total) return;                        // whole block leaves before any barrier
    const int group_sz = kGroupM * tiles_n;
    const int g = L / group_sz;
    const int gm = min(kGroupM, tiles_m - g * kGroupM);
    const int in_g = L - g * group_sz;
    const int tile_m = g * kGroupM + in_g % gm;
    const int tile_n = in_g / gm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global -> LDS staging: thread handles chunk (tid & 7) of rows (tid >> 3) + 32 * i
    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;
    const int nk = (I + BK - 1) / BK;

    v4i ga[8], gb[8];
    auto fetch = [&](int kt) {
        const int kb = kt * BK + ld_chunk * 16;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = ld_row + 32 * i;
            ga[i] = load_chunk<GENERIC>(qx, m0 + r, T, kb, I, vec);
            gb[i] = load_chunk<GENERIC>(qw, n0 + r, O, kb, I, vec);
        }
    };
    auto stash = [&](int stage) {
        int8_t* As = lds + stage * kStageBytes;
        int8_t* Bs = As + BM * BK;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = ld_row + 32 * i;
            *reinterpret_cast<v4i*>(As + r * BK + swz(r, ld_chunk)) = ga[i];
            *reinterpret_cast<v4i*>(Bs + r * BK + swz(r, ld_chunk)) = gb[i];
        }
    };

    v16i acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0;

    fetch(0);
    stash(0);
    __syncthreads();

    const int frag_row = lane & 31;     // row of the 32-row MFMA tile this lane supplies
    const int frag_half = lane >> 5;    // which 16-byte half of the 32-byte K slab

    for (int kt = 0; kt < nk; ++kt) {
        const bool more = (kt + 1 < nk);
        if (more) fetch(kt + 1);
        const int8_t* As = lds + (kt & 1) * kStageBytes;
        const int8_t* Bs = As + BM * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            v4i af[4], bf[4];
            const int chunk = ks * 2 + frag_half;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) {
                const int r = wm * 128 + mi * 32 + frag_row;
                af[mi] = *reinterpret_cast<const v4i*>(As + r * BK + swz(r, chunk));
            }
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const int r = wn * 128 + ni * 32 + frag_row;
                bf[ni] = *reinterpret_cast<const v4i*>(Bs + r * BK + swz(r, chunk));
            }
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[mi], bf[ni], acc[mi][ni], 0, 0, 0);
        }
        if (more) stash((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 128 + mi * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
            if (GENERIC && row >= T) continue;
            const float a = row_scale[row];
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const int col = n0 + wn * 128 + ni * 32 + frag_row;
                if (GENERIC && col >= O) continue;
                const int v = acc[mi][ni][r];
                float y = (float)v * a;
                y = rounded_f32(y * w_scale[col]);
                Y[(int64_t)row * ldy + col] = (uint16_t)f2h(y);
                if (acc_debug) acc_debug[(int64_t)row * O + col] = v;
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Fast path (full tiles, 16-byte aligned operands): global -> LDS loads that bypass registers.
// global_load_lds_dwordx4 writes the 64 lanes' 16-byte pieces to LDS at base + lane * 16, i.e. one
// instruction fills 8 consecutive 128-byte LDS rows.  The XOR swizzle is therefore applied on
// the global side: the lane that will land in physical chunk p of row R fetches logical chunk
// p ^ ((R >> 1) & 7) of that row (still the same 128 contiguous bytes per 8 lanes).
// Software pipeline per K step (2 slabs of 64 bytes, each worked on as activation tiles 0-3 then 4-7; two sets of
// 4 activation fragments and two sets of weight fragments alternate):
//   read s0 hi | mfma s0 lo ; read s1 lo + weights s1 | mfma s0 hi ; read s1 hi | mfma s1 lo ;
//   wait for the next tile, barrier ; read s0 lo + weights s0 of the next tile | mfma s1 hi.
// ---------------------------------------------------------------------------------------------

// Fragments of the 16 x 16 x 64 instruction: a lane supplies 16 consecutive bytes of row (lane & 15), K chunk
// lane >> 4 of the 64-byte slab (which K positions those are inside the instruction does not matter for an integer
// dot product, as long as both operands are read the same way).  A K step of 128 bytes is two slabs; a slab is
// worked on in two phases of 4 activation tiles each, so that only 4 + G fragments have to be held ahead.
// a_off / b_off: byte offset of this lane's row and swizzled chunk for slab 0; slab 1 flips bit 2 of the chunk,
// i.e. XORs the byte offset with 64.  Activation tile mi is 16 LDS rows further on.  Weight tile ni of a wave holds
// the channels G fr + ni (fr = lane & 15), so that a lane ends up with G consecutive output channels; in LDS those
// rows sit at G fr + (ni ^ (fr & 1)) (see the loader): b_off is tile 0's offset, b_flip the step to tile 1, and
// tiles 2, 3 are two rows further on.
__device__ __forceinline__ void load_a4(v4i (&af)[4], const int8_t* As, int a_off, int half, int slab) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
        af[mi] = *reinterpret_cast<const v4i*>(As + (4 * half + mi) * 16 * BK + (a_off ^ (slab * 64)));
}
template <int G>
__device__ __forceinline__ void load_b(v4i (&bf)[G], const int8_t* Bs, int b_off, int b_flip, int slab) {
#pragma unroll
    for (int ni = 0; ni < G; ++ni)
        bf[ni] = *reinterpret_cast<const v4i*>(Bs + (ni >> 1) * 2 * BK + (ni & 1) * b_flip + (b_off ^ (slab * 64)));
}

// The activation fragment is the first MFMA operand.  With the weight fragment first the accumulator tile comes
// out transposed, but the kernel runs 4.6 % slower on the 70B-shaped layer (720 -> 687 us, 4 % on the 7B-shaped one,
// 1 % on the heavy-tailed 13B-shaped one): which operand the smaller codes travel on changes what the matrix
// instruction draws, and this kernel is limited by power.  For the same reason the instruction is the 16 x 16 x 64
// one: it reads and writes half as many accumulator registers per multiply-add as 32 x 32 x 32, and a loop fed
// from LDS at this kernel's ratio sustains 9 % more with it on code-like operands (3.13-3.22 against 2.87-2.95 POP/s).
template <int G>
__device__ __forceinline__ void mfma_phase(v4i (&acc)[8][G], int half, const v4i (&af)[4], const v4i (&bf)[G]) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < G; ++ni)
            acc[4 * half + mi][ni] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[mi], bf[ni], acc[4 * half + mi][ni], 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// Ring variant of the fast path (8 waves): the loads of the two wave groups are taken apart in
// time so that one wave of every SIMD multiplies while the other is held up issuing loads.
//
// Measured on this chip: every vector-memory instruction holds its wave for ~96 cycles, so the 8
// loads a wave owes per K step cost it ~770 cycles -- three quarters of its 1024 cycles of
// MFMA work.  With all waves loading right after the barrier (the only place a 2-stage pipeline
// allows) both waves of a SIMD stall together and the matrix pipe idles.  Here LDS is a ring of
// five 32 KiB slots holding half tiles in load order A0 B0 A1 B1 A2 ... (half tile n lives in
// slot n % 5).  The spare slot lets A(kt+2) be requested a whole step early, so:
//   waves 0-3 (one per SIMD): multiply first, then request A(kt+2) (all 32 instructions of it)
//                             just before the step's barrier;
//   waves 4-7 (their SIMD mates): request B(kt+2) right after the barrier, then multiply.
// Slot reuse: A(kt+2) takes the slot of B(kt-1), free since barrier kt-1; B(kt+2) takes the slot
// of A(kt), free after barrier kt (all of tile kt's fragments are in registers by then).
// ---------------------------------------------------------------------------------------------
constexpr int kSlotBytes = BM * BK;               // 32 KiB: one operand's 256 x 128 tile
constexpr int kRingSlots = 5;
constexpr int kRingLds = kRingSlots * kSlotBytes; // 160 KiB: the whole LDS of a gfx950 CU

// One output tile of 256 tokens x (128 NI) channels starting at (m0, n0).  NI = 2 is the full 256 x 256 tile;
// NI = 1 the half tile of the last, partly filled round (see launch_w8a8_linear): the same schedule with
// 128 x 32 wave tiles, half the weight requests and half the matrix instructions per step.
// A block calls this for one tile after the other.  `prefetched`: the block's previous tile has already requested
// this tile's first two half tiles; (next_m0, next_n0): the tile this one does that for (next_m0 < 0: none).
// DEBUG: the raw accumulators are stored too (no prefetch then); STREAM: Y is written through to memory.
template <int NI, bool DEBUG, bool STREAM>
__device__ __forceinline__ void ring_tile(const int8_t* __restrict__ qx, const float* __restrict__ row_scale,
                                          const int8_t* __restrict__ qw, const float* __restrict__ w_scale, int T, int I,
                                          int O, uint16_t* __restrict__ Y, int64_t ldy,
                                          int32_t* __restrict__ acc_debug, int m0, int n0, int8_t* lds,
                                          bool prefetched, int next_m0, int next_n0, int next_ni) {
    constexpr int WN = 4, WTN = 32 * NI;
    constexpr int G = 2 * NI, LOG2G = NI;         // weight tiles of 16 channels per wave (4 or 2)
    constexpr int NLB = 4 * NI;                   // requests a weight-loading wave makes per half tile (8 or 4)

    // (the thread id goes through an empty asm: the lane-dependent offsets below are then worked out again for every
    // tile of the block's walk instead of being kept, and spilled, across the whole loop over tiles)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int nk = I / BK;
    const bool b_loader = wave >= 4;              // waves 4-7 load B, waves 0-3 load A

    // ---- loader: loader wave lw = wave & 3 fills rows [64 lw, 64 lw + 64) of its operand's half
    // tile with 8 instructions; instruction ii covers rows 64 lw + 8 ii + (lane >> 3), physical
    // chunk lane & 7 (the swizzle is applied to the global column).
    const int lw = wave & 3;
    // Tiles on the bottom / right edge of a ragged problem read a clamped (valid) row instead of
    // the rows past the end; what lands in those LDS rows only feeds outputs the epilogue drops.
    // (a weight-loading wave of a half tile fills 32 rows with 4 requests)
    // The loader is written for a tile of either kind (ni_c: 2 = full tile, 1 = half tile): besides this tile's own
    // operands a block requests the first operands of its next tile, which may be of the other kind.
    const int8_t* gsrc[8];
    auto set_sources = [&](auto ni_c, int tile_m0, int tile_n0) {
        constexpr int NIx = decltype(ni_c)::value;
        constexpr int LOG2Gx = NIx, NLBx = 4 * NIx;
        const int rows_per_loader = b_loader ? 8 * NLBx : 64;
        // (worked out from scratch at each of the two calls rather than kept in registers in between)
        int l = lane;
        asm volatile("" : "+v"(l));
        const int ld_r = l >> 3, ld_p = l & 7;
        const int8_t* base = b_loader ? qw : qx;
        const int first = b_loader ? tile_n0 : tile_m0, last = (b_loader ? O : T) - 1;
        // LDS row R of an operand tile holds, for activations, tile row R with chunk c at c ^ ((R >> 1) & 7): a
        // fragment's 16 lanes per LDS cycle read 16 consecutive rows, whose parity picks the half of the 64 banks
        // and whose (R >> 1) & 7 picks the 16-byte group.  Weight tile ni takes the tile rows G fr + ni (see
        // b_off), which for one ni all have the same parity; so LDS row R holds tile row R ^ ((R / G) & 1) (the
        // rows of a pair change places in every other group of G) and the swizzle term comes from R / (2 G): a lane
        // then reads LDS row G fr + (ni ^ (fr & 1)), parity and group exactly as for the activation fragment.
        const int sw_shift = b_loader ? LOG2Gx + 1 : 1;
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            const int R = rows_per_loader * lw + 8 * ii + ld_r;
            const int c = ld_p ^ ((R >> sw_shift) & 7);
            const int tile_row = b_loader ? (R ^ ((R >> LOG2Gx) & 1)) : R;
            gsrc[ii] = base + (int64_t)min(first + tile_row, last) * I + c * 16;
        }
    };
    using this_kind = std::integral_constant<int, NI>;
    set_sources(this_kind{}, m0, n0);
    auto issue_half = [&](auto ni_c, int kt, int slot) {
        constexpr int NLBx = 4 * decltype(ni_c)::value;
        const int rows_per_loader = b_loader ? 8 * NLBx : 64;
        int8_t* dst = lds + slot * kSlotBytes + lw * (rows_per_loader * BK);
        const int64_t koff = (int64_t)kt * BK;
#pragma unroll
        // cache policy sc0: the data goes straight to LDS and is never looked up in the vector L1 again, so the
        // requests bypass it (no measurable difference on the 70B-shaped layer; non-temporal requests are 6 % slower)
        for (int ii = 0; ii < 8; ++ii)
            if (ii < NLBx || !b_loader)
                __builtin_amdgcn_global_load_lds((gptr_t)(gsrc[ii] + koff), (lptr_t)(dst + ii * 1024), 16, 0, 1);
    };
    // "all but the requests of the last half tile have landed", for this wave's kind of half tile
    auto wait_for_previous_half = [&]() {
        if (NLB == 8 || !b_loader) __builtin_amdgcn_s_waitcnt(waitcnt_imm(8, 15));
        else __builtin_amdgcn_s_waitcnt(waitcnt_imm(NLB, 15));
    };

    const int frag_row = lane & 15, frag_chunk = lane >> 4;
    const int sw = (frag_row >> 1) & 7;
    const int a_off = (wm * 128 + frag_row) * BK + ((frag_chunk ^ sw) * 16);
    // weight tile ni: channel wn * WTN + G * frag_row + ni, which sits in LDS row
    // wn * WTN + G * frag_row + (ni ^ (frag_row & 1)); b_off is tile 0's offset, b_flip the step to tile 1
    const int b_par = frag_row & 1;
    const int b_off = (wn * WTN + G * frag_row + b_par) * BK + ((frag_chunk ^ sw) * 16);
    const int b_flip = b_par ? -BK : BK;

    v4i acc[8][G];
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < G; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mi][ni][r] = 0;

    // prologue: A0 A1 (waves 0-3) / B0 B1 (waves 4-7); half tile n -> slot n % 5.  The block's previous tile may
    // have requested them already (see the end of this function): then its 32 stores are the newest requests of
    // this wave, after A1 / B1, and "A0 / B0 has landed" is "at most 8 + 32 requests in flight" (the counter is
    // decremented in the order of issue).
    if (!prefetched) {
        issue_half(this_kind{}, 0, b_loader ? 1 : 0);
        if (nk > 1) issue_half(this_kind{}, 1, b_loader ? 3 : 2);
        if (nk > 1) wait_for_previous_half();
        else __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));
    } else if (NLB == 8 || !b_loader) {
        if (nk > 1) __builtin_amdgcn_s_waitcnt(waitcnt_imm(8 + kEpilogue16Stores, 15));
        else __builtin_amdgcn_s_waitcnt(waitcnt_imm(kEpilogue16Stores, 15));
    } else {
        if (nk > 1) __builtin_amdgcn_s_waitcnt(waitcnt_imm(NLB + kEpilogue16Stores, 15));
        else __builtin_amdgcn_s_waitcnt(waitcnt_imm(kEpilogue16Stores, 15));
    }
    // (a bare barrier, as in the loop below: the second half tile's requests stay in flight across it)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);

    // slots of the current tile (sa, sb) and of the next one (na, nb), advanced by 2 mod 5 per step
    int sa = 0, sb = 1;
    auto adv = [](int v) { v += 2; return v >= kRingSlots ? v - kRingSlots : v; };

    // fragment registers: two sets of 4 activation tiles (the two halves of a slab alternate), two sets of G weight tiles
    v4i a_lo[4], a_hi[4], b0[G], b1[G];
    load_a4(a_lo, lds + sa * kSlotBytes, a_off, 0, 0);
    load_b<G>(b0, lds + sb * kSlotBytes, b_off, b_flip, 0);

    constexpr int NMF = 4 * G;                     // matrix instructions of a phase
    auto interleave_reads = [&](auto n_reads) {
        constexpr int NRD = decltype(n_reads)::value;
#pragma unroll
        for (int i = 0; i < NRD; ++i) {
            // an MFMA first (its operands were read a phase ago), then one read for the next phase:
            // the reads are all out before the phase's last MFMAs, which cover their latency
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMF - NRD, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    using rd_a = std::integral_constant<int, 4>;
    using rd_ab = std::integral_constant<int, 4 + G>;
    using rd_none = std::integral_constant<int, 0>;
    auto k_step = [&](int kt, auto issue_c, auto prefetch_c) {
        constexpr bool ISSUE = decltype(issue_c)::value;        // kt + 2 < nk
        constexpr bool PREFETCH = decltype(prefetch_c)::value;  // kt + 1 < nk
        const int8_t* As = lds + sa * kSlotBytes;
        const int8_t* Bs = lds + sb * kSlotBytes;
        const int na = adv(sa), nb = adv(sb);                   // slots of tile kt+1
        // slab 0: activation tiles 0-3, then 4-7
        load_a4(a_hi, As, a_off, 1, 0);
        mfma_phase<G>(acc, 0, a_lo, b0);
        interleave_reads(rd_a{});
        load_a4(a_lo, As, a_off, 0, 1);
        load_b<G>(b1, Bs, b_off, b_flip, 1);
        mfma_phase<G>(acc, 1, a_hi, b0);
        interleave_reads(rd_ab{});
        // slab 1
        load_a4(a_hi, As, a_off, 1, 1);
        mfma_phase<G>(acc, 0, a_lo, b1);
        interleave_reads(rd_a{});
        // A loaders: A(kt+2) = half tile 2kt+4 -> slot (2kt+4) % 5 = adv(na); its previous tenant
        // B(kt-1) was released at the previous barrier.  Then tile kt+1's A (requested a step ago)
        // must have landed: at most the 8 requests just made may still be in flight.
        if (!b_loader) {
            if (ISSUE) {
                issue_half(this_kind{}, kt + 2, adv(na));
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(8, 0));
            } else {
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
            }
        } else {
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));      // B(kt+1), requested after the last barrier
        }
        // a bare barrier: __syncthreads() would add a release fence, i.e. a wait for *all* of this
        // wave's outstanding loads, including the ones requested a moment ago for two steps ahead.
        // LDS needs no fence: this wave's reads are complete (lgkmcnt(0) above) and the loads the
        // next tile depends on are complete in the waves that issued them (their vmcnt wait above).
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // B loaders: B(kt+2) = half tile 2kt+5 -> slot (2kt+5) % 5 = sa, tile kt's A slot, which
        // nobody reads any more (the last phase's fragments are in registers)
        if (b_loader && ISSUE) issue_half(this_kind{}, kt + 2, sa);
        __builtin_amdgcn_sched_barrier(0);
        if (PREFETCH) {
            load_a4(a_lo, lds + na * kSlotBytes, a_off, 0, 0);
            load_b<G>(b0, lds + nb * kSlotBytes, b_off, b_flip, 0);
        }
        mfma_phase<G>(acc, 1, a_hi, b1);
        if (PREFETCH) interleave_reads(rd_ab{});
        else interleave_reads(rd_none{});
        sa = na;
        sb = nb;
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int kt = 0;
    for (; kt + 2 < nk; ++kt) k_step(kt, yes{}, yes{});
    if (kt + 1 < nk) {
        k_step(kt, no{}, yes{});
        ++kt;
    }
    EpilogueScales16<G> scales;
    epilogue16_load_scales<G>(scales, row_scale, w_scale, T, O, m0 + wm * 128, n0 + wn * WTN, lane);
    __builtin_amdgcn_sched_barrier(0);              // requested now, in flight during the last step
    k_step(kt, no{}, no{});

    // Every wave is past the last step's barrier: nothing in the ring is read any more.  The first two half tiles
    // of the block's next tile are requested now, into their slots 0-3, and travel while this tile's results are
    // scaled and stored; the epilogue keeps its row factors in slot 4, which the next tile's loop does not write
    // before its first barrier.  The next tile may be of the other kind (next_ni).  (Not with DEBUG: the number of
    // stores in flight is not fixed then.)
    if (!DEBUG && next_m0 >= 0) {
        auto request_next = [&](auto ni_c) {
            set_sources(ni_c, next_m0, next_n0);
            issue_half(ni_c, 0, b_loader ? 1 : 0);
            if (nk > 1) issue_half(ni_c, 1, b_loader ? 3 : 2);
        };
        if (next_ni == 2) request_next(std::integral_constant<int, 2>{});
        else request_next(std::integral_constant<int, 1>{});
    }
    float* a_lds = reinterpret_cast<float*>(lds + 4 * kSlotBytes + wave * 512);
    epilogue16_store<WTN, G, DEBUG, STREAM>(acc, a_lds, scales, Y, ldy, acc_debug, T, O, m0 + wm * 128, n0 + wn * WTN, lane);
    __builtin_amdgcn_sched_barrier(0);
}

// Work of a block.  The grid is one block per CU (a block fills a CU's LDS) and every block walks over several
// tiles: block b belongs to XCD b % 8 (block ids are dealt round-robin) and takes positions i, i + per, i + 2 per, ...
// of that XCD's contiguous range of the tile walk, i = b / 8, per = gridDim.x / 8, so that the blocks running
// together in one XCD work on neighbouring tiles as in tile_of_block.  Staying in the kernel between tiles means
// that the stores of one tile drain while the next tile's first operands are on their way, and no wave has to be
// launched in between.  The first n_main tiles of the walk are taken whole; the remaining ones as half tiles of
// 128 channels (half tile h = column half h & 1 of tile n_main + h / 2), dealt the same way so that the two
// halves of a tile, which share their activation rows, sit in one L2.  n_main equals the tile count when no tile
// is split.
template <bool DEBUG, bool STREAM>
__global__ void __launch_bounds__(512)
gemm_i8_ring_kernel(const int8_t* __restrict__ qx, const float* __restrict__ row_scale,
                    const int8_t* __restrict__ qw, const float* __restrict__ w_scale, int T, int I, int O,
                    uint16_t* __restrict__ Y, int64_t ldy, int32_t* __restrict__ acc_debug, int tiles_m,
                    int tiles_n, int n_main) {
    extern __shared__ __align__(16) int8_t lds[];
    const int xcd = blockIdx.x % kXcds, first = blockIdx.x / kXcds, per = gridDim.x / kXcds;
    int tile_m, tile_n;
    const int main_per_xcd = (n_main + kXcds - 1) / kXcds;
    const int n_half = 2 * (tiles_m * tiles_n - n_main);
    const int half_per_xcd = (n_half + kXcds - 1) / kXcds;
    // position i of this XCD's half tiles -> its origin; false if there is none (past the end, or the empty second
    // half of a tile on the ragged edge)
    auto half_tile_at = [&](int i, int& m0, int& n0) {
        if (i >= half_per_xcd) return false;
        const int h = xcd * half_per_xcd + i;
        if (h >= n_half) return false;
        int tm, tn;
        tile_of_index(n_main + h / 2, tiles_m, tiles_n, tm, tn);
        m0 = tm * BM;
        n0 = tn * BN + (h & 1) * (BN / 2);
        return n0 < O;
    };
    bool prefetched = false;
    for (int i = first; i < main_per_xcd; i += per) {
        const int L = xcd * main_per_xcd + i;
        if (L >= n_main) break;
        tile_of_index(L, tiles_m, tiles_n, tile_m, tile_n);
        // the tile after this one, whose first operands this one requests before its epilogue: the next whole tile
        // of the walk or, after the last one, the block's first half tile
        int next_m0 = -1, next_n0 = -1, next_ni = 2;
        if (i + per < main_per_xcd && L + per < n_main) {
            int next_m, next_n;
            tile_of_index(L + per, tiles_m, tiles_n, next_m, next_n);
            next_m0 = next_m * BM;
            next_n0 = next_n * BN;
        } else if (half_tile_at(first, next_m0, next_n0)) {
            next_ni = 1;
        } else {
            next_m0 = -1;
        }
        ring_tile<2, DEBUG, STREAM>(qx, row_scale, qw, w_scale, T, I, O, Y, ldy, acc_debug, tile_m * BM, tile_n * BN, lds,
                                    prefetched, next_m0, next_n0, next_ni);
        prefetched = next_m0 >= 0 && !DEBUG;
    }
    // (a half tile that does not exist -- the empty second half of a tile on the ragged edge -- is neither run nor
    // requested for by the tile before it)
    for (int i = first; i < half_per_xcd; i += per) {
        int m0, n0;
        if (!half_tile_at(i, m0, n0)) {
            prefetched = false;
            continue;
        }
        int next_m0 = -1, next_n0 = -1;
        if (!half_tile_at(i + per, next_m0, next_n0)) next_m0 = -1;
        ring_tile<1, DEBUG, STREAM>(qx, row_scale, qw, w_scale, T, I, O, Y, ldy, acc_debug, m0, n0, lds, prefetched, next_m0,
                                    next_n0, 1);
        prefetched = next_m0 >= 0 && !DEBUG;
    }
}

}  // namespace

hipError_t launch_w8a8_linear(const int8_t* qx, const float* row_scale, const int8_t* qw, const float* w_scale,
                              int T, int I, int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug,
                              hipStream_t stream) {
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (O + BN - 1) / BN;
    if (!grid_fits((int64_t)tiles_m * tiles_n + kXcds, 512)) return hipErrorInvalidValue;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)(per_xcd * kXcds)), block(kThreads);
    const bool vec = (reinterpret_cast<uintptr_t>(qx) % 16 == 0) && (reinterpret_cast<uintptr_t>(qw) % 16 == 0) &&
                     (I % 16 == 0);
    auto al16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
    // fast path: K a multiple of the K step and everything the vector loads/stores touch aligned to 16
    // bytes (any T; O a multiple of 8)
    // (the fast path's epilogue addresses a wave's 128 output rows with 32-bit byte offsets)
    const bool full = vec && (I % BK == 0) && (O % 8 == 0) && al16(Y) && (ldy % 8 == 0) && al16(w_scale) &&
                      al16(acc_debug) && ldy < ((int64_t)1 << 22);
    hipError_t e;
    if (full) {
        // four instances: with or without the raw accumulators, Y streamed to memory or left in the caches
        using kernel_t = void (*)(const int8_t*, const float*, const int8_t*, const float*, int, int, int, uint16_t*,
                                  int64_t, int32_t*, int, int, int);
        static const kernel_t kernels[4] = {&gemm_i8_ring_kernel<false, false>, &gemm_i8_ring_kernel<false, true>,
                                            &gemm_i8_ring_kernel<true, false>, &gemm_i8_ring_kernel<true, true>};
        static std::atomic<uint64_t> lds_allowed[4];
        const int which = (acc_debug ? 2 : 0) + (y_stays_cached(T, O) ? 0 : 1);
        const kernel_t kernel = kernels[which];
        e = allow_dynamic_lds(reinterpret_cast<const void*>(kernel), kRingLds, lds_allowed[which]);
        if (e != hipSuccess) return e;
        // One block fills a CU, so the tiles run in rounds of n_cu.  A last round that is at most half full is
        // run as half tiles (256 x 128) instead, which spreads it over twice as many CUs: 2048 x 4096 x 11008
        // has 344 tiles = 1.34 rounds of 256 and took 2 tile times; the 88 tiles of its last round now take
        // 176 CUs for about 0.6 of a tile time.
        int n_cu = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
            n_cu = 256;
        const int rem = total % n_cu;
        const int n_main = (rem > 0 && 2 * rem <= n_cu) ? total - rem : total;
        const int main_blocks = ((n_main + kXcds - 1) / kXcds) * kXcds;
        const int half_blocks = ((2 * (total - n_main) + kXcds - 1) / kXcds) * kXcds;
        // one block per CU (a multiple of the XCD count), fewer when there are fewer tiles than that
        const int cu_blocks = n_cu >= kXcds ? n_cu / kXcds * kXcds : kXcds;
        const int blocks = std::min(cu_blocks, std::max(main_blocks, half_blocks));
        kernel<<<dim3((unsigned)blocks), dim3(512), kRingLds, stream>>>(qx, row_scale, qw, w_scale, T, I, O, Y, ldy,
                                                                        acc_debug, tiles_m, tiles_n, n_main);
    } else {
        static std::atomic<uint64_t> lds_allowed{0};
        e = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_i8_kernel<true>), kLdsBytes, lds_allowed);
        if (e != hipSuccess) return e;
        gemm_i8_kernel<true><<<grid, block, kLdsBytes, stream>>>(qx, row_scale, qw, w_scale, T, I, O, Y, ldy,
                                                                 acc_debug, tiles_m, tiles_n, vec);
    }
    return hipGetLastError();
}

}  // namespace cq
