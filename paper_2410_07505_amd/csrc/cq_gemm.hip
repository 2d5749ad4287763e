// W8A8 linear layer Y = X . W on integer codes (Background section): INT8 MFMA GEMM with int32
// accumulation and the scale epilogue  Y_ik = fl16(fl32(fl32(float(acc_ik) * a_i) * s_k)).
//
// Both operands are stored with the contraction axis contiguous (qx [T][I], qw [O][I]), which is
// the layout v_mfma_i32_32x32x32_i8 wants: every lane supplies 16 consecutive bytes of one row.
//
// Tiling for gfx950 (256 CUs, 160 KiB LDS per CU, 64-wide waves):
//   - block tile 256 x 256, K step 128 bytes, 256 threads = 4 waves in a 2 x 2 arrangement,
//     each wave owning 128 x 128 = 4 x 4 MFMA tiles of 32 x 32 (256 accumulator registers);
//   - two LDS stages of (256 + 256) rows x 128 B = 128 KiB; the next K step is fetched from
//     global memory into registers while the current one is multiplied, then stored to the
//     other stage: one barrier per K step;
//   - LDS rows are 128 B = 8 chunks of 16 B, stored at chunk ^ ((row >> 1) & 7) so that the 16
//     rows a quarter-wave reads (and the row pairs it writes) fall in 16 distinct bank groups;
//   - block -> tile mapping: consecutive block ids land on different XCDs, so ids are first
//     de-interleaved by XCD (each XCD gets a contiguous range of tiles, hence its own L2 sees a
//     compact patch), then walked in groups of 4 tile-rows so that concurrently resident tiles
//     share A rows and B columns.
// Integer accumulation is exact, so tiling and order cannot change a result.
#include "cq_kernels.h"

namespace cq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kThreads = 256;
constexpr int kStageBytes = (BM + BN) * BK;       // 64 KiB
constexpr int kLdsBytes = 2 * kStageBytes;         // 128 KiB
constexpr int kXcds = 8;
constexpr int kGroupM = 4;

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

}  // namespace

hipError_t launch_w8a8_linear(const int8_t* qx, const float* row_scale, const int8_t* qw, const float* w_scale,
                              int T, int I, int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug,
                              hipStream_t stream) {
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (O + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)(per_xcd * kXcds)), block(kThreads);
    const bool vec = (reinterpret_cast<uintptr_t>(qx) % 16 == 0) && (reinterpret_cast<uintptr_t>(qw) % 16 == 0) &&
                     (I % 16 == 0);
    const bool full = vec && (T % BM == 0) && (O % BN == 0) && (I % BK == 0);
    hipError_t e;
    if (full) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_i8_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        gemm_i8_kernel<false><<<grid, block, kLdsBytes, stream>>>(qx, row_scale, qw, w_scale, T, I, O, Y, ldy,
                                                                  acc_debug, tiles_m, tiles_n, vec);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_i8_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        gemm_i8_kernel<true><<<grid, block, kLdsBytes, stream>>>(qx, row_scale, qw, w_scale, T, I, O, Y, ldy,
                                                                 acc_debug, tiles_m, tiles_n, vec);
    }
    return hipGetLastError();
}

}  // namespace cq
