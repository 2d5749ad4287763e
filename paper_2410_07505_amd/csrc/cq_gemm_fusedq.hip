// Linear layer with the CrossQuant step inside the GEMM's activation load: X (binary16) goes in, the codes
// never exist in memory.  Same arithmetic as crossquant_quantize followed by crossquant_w8a8_linear
// (the CrossQuant equation for the codes; Y = X . W of the Background section on them), bit for bit.
//
// What it is for: the codes round trip (1 byte written + 1 byte read per element) disappears, but every
// activation element is quantized once per column tile that uses it, i.e. ceil(O / 256) times, at about a
// dozen vector instructions each, inside a kernel whose matrix instructions leave little vector issue room.
// It exists to measure that trade on real shapes (the benchmark reports it next to the two-call path); it is
// slower than the two calls on every layer shape tried, by the factor the count above predicts.
//
// Structure: the register-staged GEMM (256 threads = 4 waves in 2 x 2, 128 x 128 per wave, two LDS stages,
// one barrier per K step).  A thread that used to fetch 8 chunks of 16 int8 codes per K step now fetches the
// same 8 x 16 elements as binary16 (two 16-byte loads per chunk), the 16 column factors of its chunk, and
// quantizes them with the quantize kernel's own routine (fast quotient, exact division near a tie) before it
// stores the bytes to LDS.  The row factors of a thread's 8 rows stay in registers for the whole contraction.
#include "cq_device.h"
#include "cq_gemm_common.h"

namespace cq {
namespace {

constexpr int BK = 128;
constexpr int kThreads = 256;
constexpr int kStageBytes = (BM + BN) * BK;       // 64 KiB
constexpr int kLdsBytes = 2 * kStageBytes;         // 128 KiB

__device__ __forceinline__ int swz(int row, int chunk) { return (chunk ^ ((row >> 1) & 7)) * 16; }

// Requires: X 16-byte aligned, ldx % 8 == 0, I % 128 == 0, qw 16-byte aligned; any T, O.
__global__ void __launch_bounds__(kThreads)
gemm_xq_kernel(const uint16_t* __restrict__ X, int64_t ldx, const float* __restrict__ a_vec,
               const float* __restrict__ b_vec, float qmax, const int8_t* __restrict__ qw,
               const float* __restrict__ w_scale, int T, int I, int O, uint16_t* __restrict__ Y, int64_t ldy,
               int32_t* __restrict__ acc_debug, int tiles_m, int tiles_n) {
    extern __shared__ __align__(16) int8_t lds[];
    int tile_m, tile_n;
    if (!tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int ld_chunk = tid & 7;          // 16 columns of the K step
    const int ld_row = tid >> 3;           // rows ld_row + 32 i
    const int nk = I / BK;

    // row factors of this thread's 8 activation rows (rows past the end are read from the last row and only
    // feed outputs that are never stored)
    float a_r[8], ra_r[8];
    bool a_tiny = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a_r[i] = a_vec[min(m0 + ld_row + 32 * i, T - 1)];
        ra_r[i] = safe_rcp(a_r[i]);
        a_tiny |= tiny_factor(a_r[i]);
    }

    uint4 gx[8][2];      // 16 binary16 values per chunk
    v4i gb[8];
    float bcol[16];
    auto fetch = [&](int kt) {
        const int kcol = kt * BK + ld_chunk * 16;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = ld_row + 32 * i;
            const uint16_t* px = X + (int64_t)min(m0 + r, T - 1) * ldx + kcol;
            gx[i][0] = *reinterpret_cast<const uint4*>(px);
            gx[i][1] = *reinterpret_cast<const uint4*>(px + 8);
            gb[i] = *reinterpret_cast<const v4i*>(qw + (int64_t)min(n0 + r, O - 1) * I + kcol);
        }
#pragma unroll
        for (int e = 0; e < 16; e += 4) {
            const float4 f = *reinterpret_cast<const float4*>(b_vec + kcol + e);
            bcol[e] = f.x; bcol[e + 1] = f.y; bcol[e + 2] = f.z; bcol[e + 3] = f.w;
        }
    };
    auto stash = [&](int stage) {
        int8_t* As = lds + stage * kStageBytes;
        int8_t* Bs = As + BM * BK;
        float b_lo[8], b_hi[8], rb_lo[8], rb_hi[8];
        bool tiny = a_tiny;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            b_lo[e] = bcol[e];
            b_hi[e] = bcol[8 + e];
            rb_lo[e] = safe_rcp(b_lo[e]);
            rb_hi[e] = safe_rcp(b_hi[e]);
            tiny |= tiny_factor(b_lo[e]) || tiny_factor(b_hi[e]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = ld_row + 32 * i;
            float m[8], q[8];
            quantize8(gx[i][0], a_r[i], ra_r[i], b_lo, rb_lo, qmax, m, q, tiny);
            const u32x2 lo = pack_codes_i8(m);
            quantize8(gx[i][1], a_r[i], ra_r[i], b_hi, rb_hi, qmax, m, q, tiny);
            const u32x2 hi = pack_codes_i8(m);
            *reinterpret_cast<v4i*>(As + r * BK + swz(r, ld_chunk)) = v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
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

    // epilogue: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 128 + mi * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
            if (row >= T) continue;
            const float a = a_vec[row];
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const int col = n0 + wn * 128 + ni * 32 + frag_row;
                if (col >= O) continue;
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

// a, b: outputs (the scale factors, formed first by the scale-finalize kernel)
hipError_t launch_quantize_linear(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c,
                                  float alpha, int bits, float* a, float* b, const int8_t* qw, const float* w_scale,
                                  int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug, hipStream_t stream) {
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (O + BN - 1) / BN;
    if (!grid_fits((int64_t)tiles_m * tiles_n + kXcds, kThreads)) return hipErrorInvalidValue;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    static std::atomic<uint64_t> lds_allowed{0};
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_xq_kernel), kLdsBytes, lds_allowed);
    if (e != hipSuccess) return e;
    const int qmax = (1 << (bits - 1)) - 1;
    e = launch_scale_finalize(t, c, T, I, alpha, qmax, a, b, nullptr, 0, stream);
    if (e != hipSuccess) return e;
    gemm_xq_kernel<<<dim3((unsigned)(per_xcd * kXcds)), dim3(kThreads), kLdsBytes, stream>>>(
        X, ldx, a, b, (float)qmax, qw, w_scale, T, I, O, Y, ldy, acc_debug, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace cq
