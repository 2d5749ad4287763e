// A4W4 linear layer on the FP6 matrix instruction (the W4A4 rows of the paper's accuracy tables).
//
// gfx950 has no INT4 matrix instruction, but v_mfma_f32_32x32x64_f8f6f4 multiplies 6-bit floats at
// twice the INT8 rate, and every INT4 code q in [-7, 7] is exactly representable in FP6 E2M3
// (1 sign, 2 exponent, 3 mantissa bits, bias 1: 0, 1, 2, 3, 4, 5, 6, 7 are 0b000000, 0b001000,
// 0b010000, 0b010100, 0b011000, 0b011010, 0b011100, 0b011110).  Products are integers of at most
// 49 and the accumulator is binary32, so a dot product over I <= 2^18 channels stays below 2^24
// and is exact: the result equals the integer GEMM bit for bit, and the scale epilogue is the
// same sequence of binary32 operations as in the INT8 path.
//
// Operand format ("FP6 fragments"), produced by pack_fp6_kernel.  The instruction wants, in lane
// l, the 32 consecutive K elements [32 (l >> 5), +32) of row (l & 31) as one 192-bit little-endian
// stream (element j in bits [6j, 6j + 6)).  A matrix of R rows and K columns is therefore stored
// as [ceil(R/32)][K/64] fragments of 1536 bytes, each fragment as a 1024-byte plane (64 lanes x
// 16 bytes: bits [0, 128) of every lane's stream) followed by a 512-byte plane (64 lanes x 8 bytes:
// bits [128, 192)); rows past R are zero.  A fragment is copied to LDS verbatim and a wave picks
// its operand up with one 16-byte and one 8-byte read per lane, each a contiguous run across the
// wave: no bank conflicts, no swizzle, no register shuffling.
//
// The kernel follows the INT8 ring kernel's schedule with 6-bit operands: 256 x 256 block tile,
// 8 waves of 128 x 64, K step 128 elements (two fragments along K, 24 KiB per operand).  The
// smaller operands leave room for a ring of six LDS slots, i.e. three tiles in flight: requests
// run two to three steps ahead (described at the kernel).  Per K step a wave issues 16 matrix
// instructions (half the cycles of the INT8 kernel for the same K) against 18 KiB of LDS reads,
// so this kernel is bound by operand movement rather than by the matrix pipe.
#include <type_traits>

#include "cq_gemm_common.h"

namespace cq {
namespace {

constexpr int kFragBytes = 1536;                     // 32 rows x 64 elements x 6 bits
constexpr int kFragLo = 1024;                        // first plane: 64 lanes x 16 bytes
constexpr int kF6Slot = 8 * 2 * kFragBytes;          // 24 KiB: 256 rows x 128 elements
constexpr int kF6Slots = 6;
// the ring takes 144 KiB
constexpr int kF6Ring = kF6Slots * kF6Slot;
// ... or a little more: the epilogue's staging areas and row factors (148 KiB) reuse the ring's LDS
constexpr int kF6Lds = kF6Ring > epilogue_rows_lds(8, 64) ? kF6Ring : epilogue_rows_lds(8, 64);
static_assert(kF6Lds <= 160 * 1024, "LDS budget of a gfx950 CU");

// ---- packing ---------------------------------------------------------------------------------
// One thread builds one lane's 24 bytes of one fragment.  SRC 8: int8 codes [R][K]; SRC 4: packed
// two's-complement nibbles [R][K/2], even column in the low nibble.  Codes are clamped to +-7.
template <int SRC>
__global__ void pack_fp6_kernel(const uint8_t* __restrict__ src, int R, int K, uint8_t* __restrict__ dst,
                                int64_t n_slots) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_slots) return;
    const int lane = (int)(idx & 63);
    const int64_t frag = idx >> 6;
    const int KB = K / 64;
    const int kb = (int)(frag % KB), rb = (int)(frag / KB);
    const int row = rb * 32 + (lane & 31);
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

// slot: one operand's 256 rows x 128 elements as [row block 8][k fragment 2] fragments
__device__ __forceinline__ frag6 read_frag(const int8_t* slot, int row_block, int kf, int lane) {
    const int8_t* f = slot + (row_block * 2 + kf) * kFragBytes;
    frag6 r;
    r.lo = *reinterpret_cast<const uint4*>(f + lane * 16);
    r.hi = *reinterpret_cast<const uint2*>(f + kFragLo + lane * 8);
    return r;
}

template <int NI>
__device__ __forceinline__ void load_frags6(frag6 (&af)[4], frag6 (&bf)[NI], const int8_t* As, const int8_t* Bs,
                                            int a_rb, int b_rb, int kf, int lane) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) af[mi] = read_frag(As, a_rb + mi, kf, lane);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bf[ni] = read_frag(Bs, b_rb + ni, kf, lane);
}

// Activation fragment first, as in the INT8 kernel (weights first runs 3 to 4 % slower): the accumulator tile has the
// instruction's natural orientation, a lane holds channels l & 31 and 32 + (l & 31) of its wave's 64 (the operand
// format keeps 32 consecutive rows in a fragment), and the shared row-oriented epilogue takes them apart again.
// Format 2 = FP6 E2M3 for both operands; scale operands 0 select the unscaled instruction.
template <int NI>
__device__ __forceinline__ void mfma_slab6(v16f (&acc)[4][NI], const frag6 (&af)[4], const frag6 (&bf)[NI]) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(af[mi]), as_operand(bf[ni]),
                                                                          acc[mi][ni], 2, 2, 0, 0, 0, 0);
}

__global__ void __launch_bounds__(512)
gemm_f6_ring_kernel(const uint8_t* __restrict__ qx6, const float* __restrict__ row_scale,
                    const uint8_t* __restrict__ qw6, const float* __restrict__ w_scale, int T, int I, int O,
                    uint16_t* __restrict__ Y, int64_t ldy, int32_t* __restrict__ acc_debug, int tiles_m,
                    int tiles_n, int y_cached) {
    constexpr int WN = 4, WTN = 64, NI = 2;
    extern __shared__ __align__(16) int8_t lds[];

    int tile_m, tile_n;
    if (!tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
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

    // ---- loader: a slot (half tile) is 24 instructions of 1 KiB.  Instruction n copies bytes
    // [1024 (n % 3), +1024) of the two consecutive fragments (3072 bytes) of row block n / 3.  Row
    // blocks past the end of a ragged operand are replaced by the last valid one: what lands there
    // only feeds outputs the epilogue drops.
    //   B(kt+2), before the barrier: early wave lw issues instructions 6 lw .. 6 lw + 5;
    //   A(kt+3), after the barrier:  late wave lw issues kLateA of them, early wave lw the other
    //                                kEarlyA = 6 - kLateA (the late waves are the critical path of a
    //                                step, the early ones would otherwise idle at the barrier).
    const int lw = wave & 3;
    constexpr int kEarlyA = 2, kLateA = 6 - kEarlyA;   // 0 / 6 measured ~4 % slower, 1..3 alike
    auto src_of = [&](const uint8_t* base, int first_rb, int last_rb, int n) {
        const int rb = min(first_rb + n / 3, last_rb);
        return base + (int64_t)rb * KB * kFragBytes + (n % 3) * 1024 + lane * 16;
    };
    const uint8_t* src_b[6];                      // early waves only
    const uint8_t* src_a[kLateA > kEarlyA ? kLateA : kEarlyA];
    const int n_a = late ? kLateA : kEarlyA;      // this wave's share of an A half tile ...
    const int a_first = late ? kLateA * lw : 4 * kLateA + kEarlyA * lw;   // ... starting at this instruction
#pragma unroll
    for (int ii = 0; ii < 6; ++ii) src_b[ii] = src_of(qw6, n0 / 32, (O + 31) / 32 - 1, 6 * lw + ii);
#pragma unroll
    for (int ii = 0; ii < (kLateA > kEarlyA ? kLateA : kEarlyA); ++ii)
        src_a[ii] = src_of(qx6, m0 / 32, (T + 31) / 32 - 1, a_first + min(ii, n_a > 0 ? n_a - 1 : 0));
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

    v16f acc[4][NI];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.0f;

    // prologue, oldest first: B0 A0 B1 A1 A2 (B by the early waves only); tile 0 must have landed,
    // the rest may still be in flight
    if (!late) issue_b(0, 1);
    issue_a(0, 0);
    if (nk > 1) {
        if (!late) issue_b(1, 3);
        issue_a(1, 2);
    }
    if (nk > 2) issue_a(2, 4);
    {
        const int later = (nk > 1 ? (late ? 0 : 6) + pend_a : 0) + (nk > 2 ? pend_a : 0);
        wait_vmcnt_upto(later);
    }
    __builtin_amdgcn_s_barrier();

    int sa = 0, sb = 1;
    auto adv = [](int v) { v += 2; return v >= kF6Slots ? v - kF6Slots : v; };

    frag6 af0[4], bf0[NI], af1[4], bf1[NI];
    load_frags6<NI>(af0, bf0, lds + sa * kF6Slot, lds + sb * kF6Slot, a_rb, b_rb, 0, lane);

    constexpr int NMF = 4 * NI;                   // matrix instructions per slab
    constexpr int NRD = 2 * (4 + NI);             // LDS reads per slab (one 16-byte, one 8-byte per fragment)
    auto interleave_reads = [&]() {
#pragma unroll
        for (int i = 0; i < NMF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (NRD + NMF - 1) / NMF, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    auto k_step = [&](int kt, auto ahead2_c, auto ahead3_c, auto prefetch_c) {
        constexpr bool AHEAD2 = decltype(ahead2_c)::value;      // kt + 2 < nk
        constexpr bool AHEAD3 = decltype(ahead3_c)::value;      // kt + 3 < nk
        constexpr bool PREFETCH = decltype(prefetch_c)::value;  // kt + 1 < nk
        const int8_t* As = lds + sa * kF6Slot;
        const int8_t* Bs = lds + sb * kF6Slot;
        const int na = adv(sa), nb = adv(sb);                   // slots of tile kt+1
        load_frags6<NI>(af1, bf1, As, Bs, a_rb, b_rb, 1, lane);
        mfma_slab6<NI>(acc, af0, bf0);
        interleave_reads();
        // Before the barrier every wave makes sure its share of tile kt+1 has landed; requests are
        // served in order, so it is enough that at most the newest ones (its share of A(kt+2) and
        // B(kt+2)) are still in flight.  lgkmcnt(0): this wave's reads of tile kt are done (its slots
        // are handed over at the barrier).
        if (!late && AHEAD2) issue_b(kt + 2, adv(nb));          // B(kt+2) -> slot of B(kt-1)
        if (AHEAD2) wait_vmcnt_upto(pend_a + (late ? 0 : 6));
        else __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (AHEAD3) issue_a(kt + 3, sa);                        // A(kt+3) -> slot of A(kt)
        __builtin_amdgcn_sched_barrier(0);
        if (PREFETCH) load_frags6<NI>(af0, bf0, lds + na * kF6Slot, lds + nb * kF6Slot, a_rb, b_rb, 0, lane);
        mfma_slab6<NI>(acc, af1, bf1);
        if (PREFETCH) {
            interleave_reads();
        } else {
            __builtin_amdgcn_sched_barrier(0);
        }
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
    EpilogueScalesRows<NI> scales;
    epilogue_rows_load_scales<NI, true>(scales, row_scale, w_scale, T, O, m0 + wm * 128, n0 + wn * WTN, lane);
    __builtin_amdgcn_sched_barrier(0);              // requested now, in flight during the last step
    k_step(kt, no{}, no{}, no{});

    // every wave's fragments are in registers and all loads have landed: the ring can be reused
    __syncthreads();
    epilogue_rows_store<v16f, WTN, NI, 8, true>(acc, lds, scales, Y, ldy, acc_debug, T, O, m0 + wm * 128, n0 + wn * WTN,
                                                lane, wave, y_cached != 0);
}

}  // namespace

int64_t fp6_packed_bytes(int64_t R, int64_t K) { return ((R + 31) / 32) * (K / 64) * (int64_t)kFragBytes; }

hipError_t launch_pack_fp6(const void* codes, int src_format, int R, int K, void* packed, hipStream_t stream) {
    const int64_t n_slots = ((int64_t)(R + 31) / 32) * (K / 64) * 64;
    if (!grid_fits((n_slots + 255) / 256, 256)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((n_slots + 255) / 256)), block(256);
    if (src_format == 8)
        pack_fp6_kernel<8><<<grid, block, 0, stream>>>(static_cast<const uint8_t*>(codes), R, K,
                                                       static_cast<uint8_t*>(packed), n_slots);
    else
        pack_fp6_kernel<4><<<grid, block, 0, stream>>>(static_cast<const uint8_t*>(codes), R, K,
                                                       static_cast<uint8_t*>(packed), n_slots);
    return hipGetLastError();
}

hipError_t launch_w4a4_linear(const void* qx6, const float* row_scale, const void* qw6, const float* w_scale, int T,
                              int I, int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug, hipStream_t stream) {
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (O + BN - 1) / BN;
    if (!grid_fits((int64_t)tiles_m * tiles_n + kXcds, 512)) return hipErrorInvalidValue;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    static std::atomic<uint64_t> lds_allowed{0};
    const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_f6_ring_kernel), kF6Lds, lds_allowed);
    if (e != hipSuccess) return e;
    gemm_f6_ring_kernel<<<dim3((unsigned)(per_xcd * kXcds)), dim3(512), kF6Lds, stream>>>(
        static_cast<const uint8_t*>(qx6), row_scale, static_cast<const uint8_t*>(qw6), w_scale, T, I, O, Y, ldy,
        acc_debug, tiles_m, tiles_n, y_stays_cached(T, O) ? 1 : 0);
    return hipGetLastError();
}

}  // namespace cq
