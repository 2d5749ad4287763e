// A4W4 linear layer on the FP6 matrix instruction (the W4A4 rows of the paper's accuracy tables).
//
// gfx950 has no INT4 matrix instruction, but the f8f6f4 matrix instructions multiply 6-bit floats at
// twice the INT8 rate, and every INT4 code q in [-7, 7] is exactly representable in FP6 E2M3
// (1 sign, 2 exponent, 3 mantissa bits, bias 1: 0, 1, 2, 3, 4, 5, 6, 7 are 0b000000, 0b001000,
// 0b010000, 0b010100, 0b011000, 0b011010, 0b011100, 0b011110).  Products are integers of at most
// 49 and the accumulator is binary32, so a dot product over I <= 2^18 channels stays below 2^24
// and is exact: the result equals the integer GEMM bit for bit, and the scale epilogue is the
// same sequence of binary32 operations as in the INT8 path.
//
// Operand format ("FP6 fragments"), produced by pack_fp6_kernel.  A fragment holds 32 rows x 64 K elements: lane
// slot s (0..63) is the 32 consecutive K elements [32 (s >> 5), +32) of row (s & 31) as one 192-bit little-endian
// stream (element j in bits [6j, 6j + 6)).  A matrix of R rows and K columns is stored as [ceil(R/32)][K/64]
// fragments of 1536 bytes, each fragment as a 1024-byte plane (64 slots x 16 bytes: bits [0, 128) of every
// slot's stream) followed by a 512-byte plane (64 slots x 8 bytes: bits [128, 192)); rows past R are zero.
// The weight operand uses the same fragments with its rows in a different order (pack_fp6_kernel<.., true>):
// inside every group of 64 output channels, stored row 16 n + f holds channel 4 f + n, so that the 16 rows of
// the kernel's weight tile n are the channels 4 f + n and a lane ends up with four adjacent channels.
//
// The matrix instruction is v_mfma_f32_16x16x128_f8f6f4: lane l supplies row (l & 15) and the 32 consecutive K
// elements of chunk l >> 4 of a 128-element K step, i.e. slot 16 p + (l & 15) + 32 (c & 1) of fragment c >> 1
// of the two fragments along K, for the rows [16 p, 16 p + 16) of a 32-row block: one 16-byte and one 8-byte
// LDS read per lane and tile.  (Which K positions a lane's elements take inside the instruction does not matter
// for a dot product, as long as both operands are read the same way.)  The 16-byte reads of 16 lanes are
// consecutive; for the 8-byte reads, of which the LDS serves 32 lanes per cycle, the two halves of a fragment's
// second plane would fall on the same banks, so in LDS the two 128-byte pieces of that plane's second half
// change places (done by the global -> LDS requests, which pick their 16 source bytes per lane).
// The 16 x 16 x 128 instruction instead of 32 x 32 x 64: half the accumulator register traffic per multiply-add
// (a loop fed from LDS sustains about 5 % more with it), and the accumulator layout the direct epilogue wants.
//
// The kernel follows the INT8 ring kernel's schedule with 6-bit operands: 256 x 256 block tile,
// 8 waves of 128 x 64 (8 x 4 tiles of 16 x 16), K step 128 elements (two fragments along K, 24 KiB per operand).
// The smaller operands leave room for a ring of six LDS slots, i.e. three tiles in flight: requests
// run two to three steps ahead (described at the kernel).  Per K step a wave issues 32 matrix
// instructions (half the cycles of the INT8 kernel for the same K) against 18 KiB of LDS reads,
// so this kernel is bound by operand movement rather than by the matrix pipe.
#include <algorithm>
#include <type_traits>

#include "cq_gemm_common.h"

namespace cq {
namespace {

constexpr int kFragBytes = 1536;                     // 32 rows x 64 elements x 6 bits
constexpr int kFragLo = 1024;                        // first plane: 64 lanes x 16 bytes
constexpr int kF6Slot = 8 * 2 * kFragBytes;          // 24 KiB: 256 rows x 128 elements
constexpr int kF6Slots = 6;
constexpr int kF6Ring = kF6Slots * kF6Slot;         // 144 KiB
constexpr int kF6Lds = kF6Ring + 8 * 512;           // ... and the epilogue's row factors behind it
static_assert(kF6Lds <= 160 * 1024, "LDS budget of a gfx950 CU");

// ---- packing ---------------------------------------------------------------------------------
// One thread builds one lane's 24 bytes of one fragment.  SRC 8: int8 codes [R][K]; SRC 4: packed
// two's-complement nibbles [R][K/2], even column in the low nibble.  Codes are clamped to +-7.
// WEIGHTS: stored row 64 g + 16 n + f holds row 64 g + 4 f + n of the source (see the head of this file).
template <int SRC, bool WEIGHTS>
__global__ void pack_fp6_kernel(const uint8_t* __restrict__ src, int R, int K, uint8_t* __restrict__ dst,
                                int64_t n_slots) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_slots) return;
    const int lane = (int)(idx & 63);
    const int64_t frag = idx >> 6;
    const int KB = K / 64;
    const int kb = (int)(frag % KB), rb = (int)(frag / KB);
    const int stored = rb * 32 + (lane & 31);
    const int row = WEIGHTS ? (stored & ~63) + 4 * (stored & 15) + ((stored >> 4) & 3) : stored;
    const int k0 = kb * 64 + 32 * (lane >> 5);
    uint32_t w[6] = {0u, 0u, 0u, 0u, 0u, 0u};
    if (row < R) {
        int8_t q[32];
        if (SRC == 8) {
            const uint4* p = reinterpret_cast<const uint4*>(src + (int64_t)row * K + k0);
            const uint4 v0 = p[0], v1 = p[1];
            const uint32_t u[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int j = 0; j < 32; ++j) q[j] = (int8_t)((u[j >> 2] >> (8 * (j & 3))) & 0xFFu);
        } else {
            const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)row * (K / 2) + k0 / 2);
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int nib = (int)((u[j >> 3] >> (4 * (j & 7))) & 0xFu);
                q[j] = (int8_t)((nib ^ 8) - 8);                     // sign-extend 4 bits
            }
        }
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int v = q[j];
            const int mag = min(v < 0 ? -v : v, 7);
            // E2M3 patterns of 0..7, one per byte
            const uint32_t e = (uint32_t)((0x1E1C1A1814100800ull >> (8 * mag)) & 0xFFu) | (v < 0 ? 32u : 0u);
            const int bit = 6 * j;
            w[bit >> 5] |= e << (bit & 31);
            if ((bit & 31) > 26) w[(bit >> 5) + 1] |= e >> (32 - (bit & 31));
        }
    }
    uint8_t* f = dst + frag * kFragBytes;
    *reinterpret_cast<uint4*>(f + lane * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    *reinterpret_cast<uint2*>(f + kFragLo + lane * 8) = make_uint2(w[4], w[5]);
}

// ---- global -> LDS ------------------------------------------------------------------------------
// One request: every lane's 16 bytes at `src` go to LDS at dst + 16 * lane (1 KiB per wave), without
// passing through registers; completion is counted by vmcnt.  Written as inline assembly rather
// than with the compiler's builtin: for the builtin the compiler makes every later LDS read wait
// until all such requests have landed (it cannot tell that the ring's slots differ), which would
// serialise the requests made two and three steps ahead with the reads of the current step.  The
// kernel orders reads and in-flight writes itself (slot discipline, explicit vmcnt waits, barriers).
__device__ __forceinline__ void dma_1k(const uint8_t* src, const int8_t* dst) {
    const uint32_t lds_off = (uint32_t)(uintptr_t)((lptr_t)dst);     // wave-uniform
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off sc0"
                 :
                 : "v"(src), "s"(lds_off)
                 : "m0");
}

// s_waitcnt vmcnt(n), lgkmcnt(0) for a wave-uniform n in [0, 12] (the instruction takes an immediate)
__device__ __forceinline__ void wait_vmcnt_upto(int n) {
    switch (n) {
        case 0: __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0)); break;
        case 1: __builtin_amdgcn_s_waitcnt(waitcnt_imm(1, 0)); break;
        case 2: __builtin_amdgcn_s_waitcnt(waitcnt_imm(2, 0)); break;
        case 3: __builtin_amdgcn_s_waitcnt(waitcnt_imm(3, 0)); break;
        case 4: __builtin_amdgcn_s_waitcnt(waitcnt_imm(4, 0)); break;
        case 5: __builtin_amdgcn_s_waitcnt(waitcnt_imm(5, 0)); break;
        case 6: __builtin_amdgcn_s_waitcnt(waitcnt_imm(6, 0)); break;
        case 7: __builtin_amdgcn_s_waitcnt(waitcnt_imm(7, 0)); break;
        case 8: __builtin_amdgcn_s_waitcnt(waitcnt_imm(8, 0)); break;
        case 9: __builtin_amdgcn_s_waitcnt(waitcnt_imm(9, 0)); break;
        case 10: __builtin_amdgcn_s_waitcnt(waitcnt_imm(10, 0)); break;
        case 11: __builtin_amdgcn_s_waitcnt(waitcnt_imm(11, 0)); break;
        default: __builtin_amdgcn_s_waitcnt(waitcnt_imm(12, 0)); break;
    }
}

// ---- fragments: LDS -> registers ---------------------------------------------------------------
struct frag6 {
    uint4 lo;
    uint2 hi;
};

__device__ __forceinline__ v8i as_operand(const frag6& f) {
    v8i v;
    v[0] = (int)f.lo.x; v[1] = (int)f.lo.y; v[2] = (int)f.lo.z; v[3] = (int)f.lo.w;
    v[4] = (int)f.hi.x; v[5] = (int)f.hi.y;
    v[6] = 0; v[7] = 0;
    return v;
}

// Where a piece of a fragment sits in LDS: the two 128-byte pieces of the second plane's second half change places
// (fragment-local byte offsets [1280, 1408) and [1408, 1536)); everything else is where the operand format has it.
__device__ __forceinline__ int lds_place(int frag_offset) {
    return frag_offset >= 1280 ? frag_offset ^ 128 : frag_offset;      // 1280 = 10 * 128: the xor swaps the two pieces
}

// Per-lane read offsets inside a slot, for the 16 x 16 tile made of the rows [16 p, 16 p + 16) of a 32-row block:
// lane l = row (l & 15), K chunk c = l >> 4 -> fragment c >> 1 along K, slot 16 p + (l & 15) + 32 (c & 1).
struct FragLane {
    int lo[2];             // 16-byte piece, p = 0 / 1
    int hi[2][2];          // 8-byte piece, [p][row block even / odd]
};
__device__ __forceinline__ FragLane frag_lane(int lane) {
    const int r = lane & 15, c = lane >> 4;
    FragLane f;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int slot = 16 * p + r + 32 * (c & 1);
        f.lo[p] = (c >> 1) * kFragBytes + slot * 16;
        f.hi[p][0] = (c >> 1) * kFragBytes + lds_place(kFragLo + slot * 8);
        // The odd row block's offset goes through an empty asm so that the compiler cannot see that it is the even
        // one's plus a constant: it would otherwise pair the 8-byte reads of two row blocks into one instruction
        // and then has to move the halves of its result next to each tile's 16-byte piece, waiting for the read first.
        f.hi[p][1] = f.hi[p][0] + 2 * kFragBytes;
        asm volatile("" : "+v"(f.hi[p][1]));
    }
    return f;
}
// tile `tile` (16 rows) of the operand rows that start at row block rb0 (even) of the slot
__device__ __forceinline__ frag6 read_tile(const int8_t* slot, int rb0, int tile, const FragLane& fl) {
    const int8_t* f_even = slot + (rb0 + ((tile >> 1) & ~1)) * (2 * kFragBytes);
    frag6 r;
    r.lo = *reinterpret_cast<const uint4*>(f_even + ((tile >> 1) & 1) * (2 * kFragBytes) + fl.lo[tile & 1]);
    r.hi = *reinterpret_cast<const uint2*>(f_even + fl.hi[tile & 1][(tile >> 1) & 1]);
    return r;
}

// Activation fragment first, as in the INT8 kernel (weights first runs 3 to 4 % slower): the accumulator tile has the
// instruction's natural orientation (lane l: channel l & 15 of the weight tile, tokens 4 (l >> 4) + register).
// Format 2 = FP6 E2M3 for both operands; scale operands 0 select the unscaled instruction.
__device__ __forceinline__ v4f mfma6(const frag6& a, const frag6& b, v4f acc) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(a), as_operand(b), acc, 2, 2, 0, 0, 0, 0);
}

// s_waitcnt vmcnt(n + 32), lgkmcnt(0) for a wave-uniform n in [0, 12]: the same with the 32 stores of the block's
// previous tile still allowed in flight
__device__ __forceinline__ void wait_vmcnt_upto_after_stores(int n) {
    static_assert(kEpilogue16Stores == 32, "the store count of the shared epilogue");
    switch (n) {
        case 0: __builtin_amdgcn_s_waitcnt(waitcnt_imm(32, 0)); break;
        case 1: __builtin_amdgcn_s_waitcnt(waitcnt_imm(33, 0)); break;
        case 2: __builtin_amdgcn_s_waitcnt(waitcnt_imm(34, 0)); break;
        case 3: __builtin_amdgcn_s_waitcnt(waitcnt_imm(35, 0)); break;
        case 4: __builtin_amdgcn_s_waitcnt(waitcnt_imm(36, 0)); break;
        case 5: __builtin_amdgcn_s_waitcnt(waitcnt_imm(37, 0)); break;
        case 6: __builtin_amdgcn_s_waitcnt(waitcnt_imm(38, 0)); break;
        case 7: __builtin_amdgcn_s_waitcnt(waitcnt_imm(39, 0)); break;
        case 8: __builtin_amdgcn_s_waitcnt(waitcnt_imm(40, 0)); break;
        case 9: __builtin_amdgcn_s_waitcnt(waitcnt_imm(41, 0)); break;
        case 10: __builtin_amdgcn_s_waitcnt(waitcnt_imm(42, 0)); break;
        case 11: __builtin_amdgcn_s_waitcnt(waitcnt_imm(43, 0)); break;
        default: __builtin_amdgcn_s_waitcnt(waitcnt_imm(44, 0)); break;
    }
}

// One output tile of 256 tokens x 256 channels starting at (m0, n0).  `prefetched`: the block's previous tile has
// requested this tile's first half tiles already; (next_m0, next_n0): the tile this one does that for (next_m0 < 0:
// none).
template <bool DEBUG, bool STREAM>
__device__ __forceinline__ void f6_tile(const uint8_t* __restrict__ qx6, const float* __restrict__ row_scale,
                                        const uint8_t* __restrict__ qw6, const float* __restrict__ w_scale, int T, int I,
                                        int O, uint16_t* __restrict__ Y, int64_t ldy, int32_t* __restrict__ acc_debug,
                                        int m0, int n0, int8_t* lds, bool prefetched, int next_m0, int next_n0) {
    constexpr int WN = 4, WTN = 64, G = 4;

    // (the thread id goes through an empty asm: the lane-dependent offsets below are then worked out again for every
    // tile of the block's walk instead of being kept, and spilled, across the whole loop over tiles)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int KB = I / 64;                        // fragments along K
    const int nk = I / 128;                       // K steps
    // Six LDS slots hold three tiles: half tile h (A(kt) = 2 kt, B(kt) = 2 kt + 1) lives in slot
    // h % 6, so requests run two to three steps ahead of their use (the loads' latency from the
    // memory-side cache is longer than one step).
    //   waves 0-3 ("early"): request B(kt+2) before the barrier of step kt; its slot was B(kt-1)'s,
    //                        released at barrier kt-1;
    //   waves 4-7 ("late"):  request A(kt+3) after the barrier of step kt (the early waves take a
    //                        share of it, see the loader below); its slot was A(kt)'s, which nobody
    //                        reads after that barrier.
    // One wave of every SIMD multiplies while its mate is held in load issue, as in the INT8 kernel.
    const bool late = wave >= 4;

    // ---- loader: a slot (half tile) is 24 instructions of 1 KiB.  Instruction n fills bytes
    // [1024 (n % 3), +1024) of the two consecutive fragments (3072 bytes) of row block n / 3 in LDS; a lane's
    // 16 bytes come from where lds_place puts them.  Row blocks past the end of a ragged operand are replaced
    // by the last valid one: what lands there only feeds outputs the epilogue drops.
    //   B(kt+2), before the barrier: early wave lw issues instructions 6 lw .. 6 lw + 5;
    //   A(kt+3), after the barrier:  late wave lw issues kLateA of them, early wave lw the other
    //                                kEarlyA = 6 - kLateA (the late waves are the critical path of a
    //                                step, the early ones would otherwise idle at the barrier).
    const int lw = wave & 3;
    constexpr int kEarlyA = 2, kLateA = 6 - kEarlyA;   // 0 / 6 measured ~4 % slower, 1..3 alike
    auto src_of = [&](const uint8_t* base, int first_rb, int last_rb, int n, int ln) {
        const int rb = min(first_rb + n / 3, last_rb);
        const int pair_offset = (n % 3) * 1024 + ln * 16;                    // where the 16 bytes land, in the pair
        const int frag = pair_offset >= kFragBytes ? 1 : 0;
        // (lds_place is its own inverse)
        return base + (int64_t)rb * KB * kFragBytes + frag * kFragBytes + lds_place(pair_offset - frag * kFragBytes);
    };
    const uint8_t* src_b[6];                      // early waves only
    const uint8_t* src_a[kLateA > kEarlyA ? kLateA : kEarlyA];
    const int n_a = late ? kLateA : kEarlyA;      // this wave's share of an A half tile ...
    const int a_first = late ? kLateA * lw : 4 * kLateA + kEarlyA * lw;   // ... starting at this instruction
    auto set_sources = [&](int tile_m0, int tile_n0) {
        // (worked out from scratch at each of the two calls rather than kept in registers in between)
        int ln = lane;
        asm volatile("" : "+v"(ln));
        // (the weight operand always has whole groups of 64 channels, i.e. an even number of row blocks)
#pragma unroll
        for (int ii = 0; ii < 6; ++ii) src_b[ii] = src_of(qw6, tile_n0 / 32, 2 * ((O + 63) / 64) - 1, 6 * lw + ii, ln);
#pragma unroll
        for (int ii = 0; ii < (kLateA > kEarlyA ? kLateA : kEarlyA); ++ii)
            src_a[ii] = src_of(qx6, tile_m0 / 32, (T + 31) / 32 - 1, a_first + min(ii, n_a > 0 ? n_a - 1 : 0), ln);
    };
    set_sources(m0, n0);
    auto issue_b = [&](int kt, int slot) {        // early waves
        int8_t* dst = lds + slot * kF6Slot + lw * (6 * 1024);
        const int64_t koff = (int64_t)kt * (2 * kFragBytes);
#pragma unroll
        for (int ii = 0; ii < 6; ++ii) dma_1k(src_b[ii] + koff, dst + ii * 1024);
    };
    auto issue_a = [&](int kt, int slot) {        // all waves, n_a instructions each
        int8_t* dst = lds + slot * kF6Slot + a_first * 1024;
        const int64_t koff = (int64_t)kt * (2 * kFragBytes);
        if (late) {
#pragma unroll
            for (int ii = 0; ii < kLateA; ++ii) dma_1k(src_a[ii] + koff, dst + ii * 1024);
        } else {
#pragma unroll
            for (int ii = 0; ii < kEarlyA; ++ii) dma_1k(src_a[ii] + koff, dst + ii * 1024);
        }
    };
    // requests of this wave that may still be in flight when tile kt+1 has to be complete: its share
    // of A(kt+2) and, for the early waves, B(kt+2)
    const int pend_a = n_a;

    const int a_rb = wm * 4, b_rb = wn * 2;       // first row block of this wave inside the A / B slot
    const FragLane fl = frag_lane(lane);

    v4f acc[8][G];
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < G; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mi][ni][r] = 0.0f;

    // prologue, oldest first: B0 A0 B1 A1 A2 (B by the early waves only); tile 0 must have landed,
    // the rest may still be in flight -- and, when the block's previous tile made these requests before its
    // epilogue, so may that tile's 32 stores, which are this wave's newest requests (the counter is decremented in
    // the order of issue)
    auto issue_prologue = [&]() {
        if (!late) issue_b(0, 1);
        issue_a(0, 0);
        if (nk > 1) {
            if (!late) issue_b(1, 3);
            issue_a(1, 2);
        }
        if (nk > 2) issue_a(2, 4);
    };
    {
        const int later = (nk > 1 ? (late ? 0 : 6) + pend_a : 0) + (nk > 2 ? pend_a : 0);
        if (!prefetched) {
            issue_prologue();
            wait_vmcnt_upto(later);
        } else {
            wait_vmcnt_upto_after_stores(later);
        }
    }
    __builtin_amdgcn_s_barrier();

    int sa = 0, sb = 1;
    auto adv = [](int v) { v += 2; return v >= kF6Slots ? v - kF6Slots : v; };

    // Fragment registers: the activation tiles 0-3 and 4-7 of a step alternate (a_lo, a_hi), the four weight tiles
    // are replaced one by one as the step's second half finishes with them.  A step is two phases of 16 matrix
    // instructions, walked weight tile by weight tile:
    //   phase 1: tokens 0-63   (a_lo x bf) while a_hi of this step is read;
    //   [requests, waits and the step's barrier]
    //   phase 2: tokens 64-127 (a_hi x bf) while a_lo and then bf of the next step are read, each weight tile
    //            after the four instructions that used its predecessor.
    frag6 a_lo[4], a_hi[4], bf[G];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) a_lo[mi] = read_tile(lds + sa * kF6Slot, a_rb, mi, fl);
#pragma unroll
    for (int ni = 0; ni < G; ++ni) bf[ni] = read_tile(lds + sb * kF6Slot, b_rb, ni, fl);

    // The arguments that only the epilogue uses are brought into registers here.  Left to the compiler their scalar
    // loads stay pending into the loop, and while one is pending every wait for an LDS read at the head of the loop has
    // to be a wait for all of them (scalar loads return out of order, on the same counter): the first matrix
    // instruction of a step then waits for the last read of the step before.
    asm volatile("" ::"s"(row_scale), "s"(w_scale), "s"(Y), "s"(ldy), "s"(acc_debug), "s"(T), "s"(O));
    auto k_step = [&](int kt, auto ahead2_c, auto ahead3_c, auto prefetch_c) {
        constexpr bool AHEAD2 = decltype(ahead2_c)::value;      // kt + 2 < nk
        constexpr bool AHEAD3 = decltype(ahead3_c)::value;      // kt + 3 < nk
        constexpr bool PREFETCH = decltype(prefetch_c)::value;  // kt + 1 < nk
        const int8_t* As = lds + sa * kF6Slot;
        const int na = adv(sa), nb = adv(sb);                   // slots of tile kt+1
        // phase 1
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) a_hi[mi] = read_tile(As, a_rb, 4 + mi, fl);
#pragma unroll
        for (int ni = 0; ni < G; ++ni)
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) acc[mi][ni] = mfma6(a_lo[mi], bf[ni], acc[mi][ni]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {                           // 8 reads, one after each of the first 8 instructions
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        __builtin_amdgcn_sched_barrier(0);
        // Before the barrier every wave makes sure its share of tile kt+1 has landed; requests are
        // served in order, so it is enough that at most the newest ones (its share of A(kt+2) and
        // B(kt+2)) are still in flight.  lgkmcnt(0): this wave's reads of tile kt are done (its slots
        // are handed over at the barrier).
        if (!late && AHEAD2) issue_b(kt + 2, adv(nb));          // B(kt+2) -> slot of B(kt-1)
        if (AHEAD2) {
            // (in a prefetched tile's first step the previous tile's stores are still younger than tile 1's requests)
            if (prefetched && kt == 0) wait_vmcnt_upto_after_stores(pend_a + (late ? 0 : 6));
            else wait_vmcnt_upto(pend_a + (late ? 0 : 6));
        } else {
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
        }
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (AHEAD3) issue_a(kt + 3, sa);                        // A(kt+3) -> slot of A(kt)
        __builtin_amdgcn_sched_barrier(0);
        // phase 2
        if (PREFETCH) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) a_lo[mi] = read_tile(lds + na * kF6Slot, a_rb, mi, fl);
        }
#pragma unroll
        for (int ni = 0; ni < G; ++ni) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) acc[4 + mi][ni] = mfma6(a_hi[mi], bf[ni], acc[4 + mi][ni]);
            if (PREFETCH) bf[ni] = read_tile(lds + nb * kF6Slot, b_rb, ni, fl);
        }
        if (PREFETCH) {
            // reads 1-8 (a_lo) behind instructions 1-8, the weight tiles' behind 9-14, the last tile's after 16
#pragma unroll
            for (int i = 0; i < 14; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        sa = na;
        sb = nb;
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int kt = 0;
    for (; kt + 3 < nk; ++kt) k_step(kt, yes{}, yes{}, yes{});
    if (kt + 2 < nk) {
        k_step(kt, yes{}, no{}, yes{});
        ++kt;
    }
    if (kt + 1 < nk) {
        k_step(kt, no{}, no{}, yes{});
        ++kt;
    }
    EpilogueScales16<G> scales;
    epilogue16_load_scales<G>(scales, row_scale, w_scale, T, O, m0 + wm * 128, n0 + wn * WTN, lane);
    __builtin_amdgcn_sched_barrier(0);              // requested now, in flight during the last step
    k_step(kt, no{}, no{}, no{});

    // Every wave is past the last step's barrier and all requests have landed: the ring is free.  The prologue of the
    // block's next tile is requested now and travels while this tile's results are scaled and stored; the row
    // factors of the epilogue sit behind the ring.  (Not with DEBUG: the number of stores in flight is not fixed then.)
    if (!DEBUG && next_m0 >= 0) {
        set_sources(next_m0, next_n0);
        issue_prologue();
    }
    float* a_lds = reinterpret_cast<float*>(lds + kF6Ring + wave * 512);
    epilogue16_store<WTN, G, DEBUG, STREAM>(acc, a_lds, scales, Y, ldy, acc_debug, T, O, m0 + wm * 128, n0 + wn * WTN, lane);
    __builtin_amdgcn_sched_barrier(0);
}

// One block per CU (a block fills a CU's LDS) walks over several tiles, as in the INT8 kernel: block b belongs to XCD
// b % 8 and takes positions i, i + per, ... of that XCD's contiguous range of the tile walk, i = b / 8, per =
// gridDim.x / 8.
template <bool DEBUG, bool STREAM>
__global__ void __launch_bounds__(512)
gemm_f6_ring_kernel(const uint8_t* __restrict__ qx6, const float* __restrict__ row_scale,
                    const uint8_t* __restrict__ qw6, const float* __restrict__ w_scale, int T, int I, int O,
                    uint16_t* __restrict__ Y, int64_t ldy, int32_t* __restrict__ acc_debug, int tiles_m,
                    int tiles_n) {
    extern __shared__ __align__(16) int8_t lds[];
    const int xcd = blockIdx.x % kXcds, first = blockIdx.x / kXcds, per = gridDim.x / kXcds;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    bool prefetched = false;
    for (int i = first; i < per_xcd; i += per) {
        const int L = xcd * per_xcd + i;
        if (L >= total) break;
        int tile_m, tile_n, next_m = -1, next_n = -1;
        tile_of_index(L, tiles_m, tiles_n, tile_m, tile_n);
        const bool has_next = i + per < per_xcd && L + per < total;
        if (has_next) tile_of_index(L + per, tiles_m, tiles_n, next_m, next_n);
        f6_tile<DEBUG, STREAM>(qx6, row_scale, qw6, w_scale, T, I, O, Y, ldy, acc_debug, tile_m * BM, tile_n * BN, lds,
                               prefetched, has_next ? next_m * BM : -1, next_n * BN);
        prefetched = has_next && !DEBUG;
    }
}

}  // namespace

int64_t fp6_packed_bytes(int64_t R, int64_t K) { return ((R + 31) / 32) * (K / 64) * (int64_t)kFragBytes; }
int64_t fp6_packed_weight_bytes(int64_t O, int64_t K) { return fp6_packed_bytes(((O + 63) / 64) * 64, K); }

hipError_t launch_pack_fp6(const void* codes, int src_format, bool weights, int R, int K, void* packed,
                           hipStream_t stream) {
    const int64_t row_blocks = weights ? 2 * (((int64_t)R + 63) / 64) : ((int64_t)R + 31) / 32;
    const int64_t n_slots = row_blocks * (K / 64) * 64;
    if (!grid_fits((n_slots + 255) / 256, 256)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((n_slots + 255) / 256)), block(256);
    const uint8_t* src = static_cast<const uint8_t*>(codes);
    uint8_t* dst = static_cast<uint8_t*>(packed);
    if (src_format == 8) {
        if (weights) pack_fp6_kernel<8, true><<<grid, block, 0, stream>>>(src, R, K, dst, n_slots);
        else pack_fp6_kernel<8, false><<<grid, block, 0, stream>>>(src, R, K, dst, n_slots);
    } else {
        if (weights) pack_fp6_kernel<4, true><<<grid, block, 0, stream>>>(src, R, K, dst, n_slots);
        else pack_fp6_kernel<4, false><<<grid, block, 0, stream>>>(src, R, K, dst, n_slots);
    }
    return hipGetLastError();
}

hipError_t launch_w4a4_linear(const void* qx6, const float* row_scale, const void* qw6, const float* w_scale, int T,
                              int I, int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug, hipStream_t stream) {
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (O + BN - 1) / BN;
    if (!grid_fits((int64_t)tiles_m * tiles_n + kXcds, 512)) return hipErrorInvalidValue;
    if (ldy >= ((int64_t)1 << 22)) return hipErrorInvalidValue;      // the epilogue's 32-bit byte offsets
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    // four instances: with or without the raw accumulators, Y streamed to memory or left in the caches
    using kernel_t = void (*)(const uint8_t*, const float*, const uint8_t*, const float*, int, int, int, uint16_t*, int64_t,
                              int32_t*, int, int);
    static const kernel_t kernels[4] = {&gemm_f6_ring_kernel<false, false>, &gemm_f6_ring_kernel<false, true>,
                                        &gemm_f6_ring_kernel<true, false>, &gemm_f6_ring_kernel<true, true>};
    static std::atomic<uint64_t> lds_allowed[4];
    const int which = (acc_debug ? 2 : 0) + (y_stays_cached(T, O) ? 0 : 1);
    const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kernels[which]), kF6Lds, lds_allowed[which]);
    if (e != hipSuccess) return e;
    // one block per CU (a multiple of the XCD count), fewer when there are fewer tiles than that
    int n_cu = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
        n_cu = 256;
    const int cu_blocks = n_cu >= kXcds ? n_cu / kXcds * kXcds : kXcds;
    const int blocks = std::min(cu_blocks, per_xcd * kXcds);
    kernels[which]<<<dim3((unsigned)blocks), dim3(512), kF6Lds, stream>>>(
        static_cast<const uint8_t*>(qx6), row_scale, static_cast<const uint8_t*>(qw6), w_scale, T, I, O, Y, ldy,
        acc_debug, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace cq
