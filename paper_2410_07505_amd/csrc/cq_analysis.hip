// Quantization-kernel analysis (Definition 1; Table 1; the "Remove Kernel" experiment of the
// zero-shot accuracy figures): one pass over X that writes X with its kernel elements zeroed and
// counts the kernel size and the two indicators of the kernel-size analysis,
//   case II:  c_j >= t_i          and          B~_ij < B_ij  (zero bound of CrossQuant below per-token's).
// Only "is the code zero" is needed, and q = rne(fl32(x / fl32(a b))) is 0 exactly when the quotient
// is at most 1/2, so the sign of one fma, |x| (1/b) - a/2, decides; a wave in which any lane has
// the two sides within 2^-20 of each other (the approximation is within 2^-22) takes the correctly
// rounded division for its row piece instead.  The three counts are kept per lane (one compare and
// one add-with-carry each) and summed once per wave at the end: as population counts of compare masks
// they cost three scalar instructions per wave-wide compare, 72 per row piece (4096 x 8192: the call
// took 41 us that way, 38.5 us now).  With the division everywhere the kernel was bound by the vector
// unit (35 instructions per element).
#include "cq_device.h"

namespace cq {
namespace {

constexpr int kWaves = 8;
constexpr int kU = 4;

__global__ void zero_counters_kernel(unsigned long long* __restrict__ counters) {
    if (threadIdx.x < 3) counters[threadIdx.x] = 0ull;
}

// Block: 8 waves share 512 columns; each wave takes nb batches of 4 consecutive rows.
// OWN_FACTORS: a_vec / b_vec are not given; the block forms the factors of its rows and columns itself
// (as the quantize kernel does) and keeps them in LDS.
template <bool VEC, bool OWN_FACTORS>
__global__ void __launch_bounds__(kWaves * kLanes)
analysis_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, const float* __restrict__ t_vec,
                const float* __restrict__ c_vec, const float* __restrict__ a_vec, const float* __restrict__ b_vec,
                double alpha, int qmax_i, uint16_t* __restrict__ xrk, unsigned long long* __restrict__ counters,
                int n_col_chunks, int nb, bool out_vec) {
    __shared__ uint32_t lds_cnt[kWaves][3];
    __shared__ float lds_a[OWN_FACTORS ? kWaves * kLanes : 1];
    __shared__ float lds_b[OWN_FACTORS ? kColsPerWave : 1];
    const float qmax = (float)qmax_i;
    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    const int col_chunk = blockIdx.x % n_col_chunks;
    const int row_chunk = blockIdx.x / n_col_chunks;
    const int j0 = col_chunk * kColsPerWave + lane * 8;
    const int rows_per_wave = nb * kU;
    const int row0 = row_chunk * (kWaves * rows_per_wave) + wave * rows_per_wave;
    if (OWN_FACTORS) {
        block_scale_factors(t_vec, c_vec, alpha, qmax_i, T, I, col_chunk * kColsPerWave,
                            row_chunk * (kWaves * rows_per_wave), kWaves * rows_per_wave, lds_a, lds_b, nullptr, nullptr);
        __syncthreads();
    }

    // Columns past the end: x reads as 0 there, so the code is 0 (not counted as non-zero); c = -1 is never
    // >= t_i, and a step of +infinity (NaN for a_i = 0) is never below the per-token step.
    float b[8], rb[8], c[8], b_cmp[8];
    bool odd = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool exists = j0 + e < I;
        b[e] = exists ? (OWN_FACTORS ? lds_b[lane * 8 + e] : b_vec[j0 + e]) : 0.0f;
        c[e] = exists ? c_vec[j0 + e] : -1.0f;
        b_cmp[e] = exists ? b[e] : __builtin_inff();
        rb[e] = safe_rcp(b[e]);
        odd |= tiny_factor(b[e]);
    }
    int nvalid = I - j0;
    nvalid = nvalid < 0 ? 0 : (nvalid > 8 ? 8 : nvalid);
    // per row: a_i, t_i and the per-token step fl32(t_i / q_max), one row per lane
    const bool has_row = lane < rows_per_wave && row0 + lane < T;
    const float a_lane = has_row ? (OWN_FACTORS ? lds_a[wave * rows_per_wave + lane] : a_vec[row0 + lane]) : 0.0f;
    const float t_lane = has_row ? t_vec[row0 + lane] : 0.0f;
    const float pt_lane = (float)((double)t_lane / (double)qmax);

    uint32_t nz_lane = 0, ge_lane = 0, sm_lane = 0;         // this lane's counts: codes != 0, c_j >= t_i, B~ < B
    int rows_done = 0;
    for (int bi = 0; bi < nb; ++bi) {
        const int rbase = row0 + bi * kU;
        if (rbase >= T) break;                              // wave-uniform
        uint4 v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u)
            v[u] = (rbase + u < T) ? load8<VEC>(X + (int64_t)(rbase + u) * ldx, j0, I) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int r = rbase + u;
            if (r >= T) break;                              // wave-uniform
            ++rows_done;
            const int ri = bi * kU + u;
            const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a_lane), ri));
            const float ti = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t_lane), ri));
            const float pt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pt_lane), ri));
            const float ha = 0.5f * a, tol = ha * kTieTol;
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            _Float16 h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = __builtin_bit_cast(_Float16, (unsigned short)(w[e >> 1] >> (16 * (e & 1))));
            bool nonzero[8];                                // element e has a non-zero code
            float nearest = __builtin_inff();               // min over the 8 elements of | |x|/b - a/2 |
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = __builtin_fmaf(__builtin_fabsf((float)h[e]), rb[e], -ha);
                nonzero[e] = d > 0.0f;
                nearest = __builtin_fminf(nearest, __builtin_fabsf(d));
            }
            // a == 0: D = 0 and every code of the row is 0 by definition (left to the exact path)
            if (__any(nearest <= tol || odd || tiny_factor(a) || a == 0.0f)) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float D = a * b[e];
                    float q = (D == 0.0f) ? 0.0f : __builtin_rintf((float)h[e] / D);
                    q = __builtin_amdgcn_fmed3f(q, -qmax, qmax);
                    nonzero[e] = q != 0.0f;
                }
            }
            uint32_t out[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t keep = (nonzero[2 * p] ? 0x0000FFFFu : 0u) | (nonzero[2 * p + 1] ? 0xFFFF0000u : 0u);
                out[p] = w[p] & keep;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                nz_lane += nonzero[e] ? 1u : 0u;
                ge_lane += (c[e] >= ti) ? 1u : 0u;
                sm_lane += (a * b_cmp[e] < pt) ? 1u : 0u;                // 0.5 * D < 0.5 * pt, exactly
            }
            if (xrk) {
                uint16_t* dst = xrk + (int64_t)r * I + j0;
                if (out_vec && nvalid == 8) {
                    __builtin_nontemporal_store(u32x4{out[0], out[1], out[2], out[3]}, reinterpret_cast<u32x4*>(dst));
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e < nvalid) dst[e] = (uint16_t)((e & 1) ? (out[e >> 1] >> 16) : (out[e >> 1] & 0xFFFFu));
                }
            }
        }
    }

    // wave totals
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        nz_lane += (uint32_t)__shfl_xor((int)nz_lane, off, kLanes);
        ge_lane += (uint32_t)__shfl_xor((int)ge_lane, off, kLanes);
        sm_lane += (uint32_t)__shfl_xor((int)sm_lane, off, kLanes);
    }
    if (lane == 0) {
        int wave_cols = I - col_chunk * kColsPerWave;        // columns of this wave that exist
        wave_cols = wave_cols > kColsPerWave ? kColsPerWave : wave_cols;
        lds_cnt[wave][0] = (uint32_t)(rows_done * wave_cols) - nz_lane;
        lds_cnt[wave][1] = ge_lane;
        lds_cnt[wave][2] = sm_lane;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        uint32_t s = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += lds_cnt[w][threadIdx.x];
        if (s) atomicAdd(&counters[threadIdx.x], (unsigned long long)s);
    }
}

}  // namespace

// a, b null: the kernel forms the factors itself (counters cleared by a kernel of their own first);
// otherwise a, b are work vectors that a scale-finalize kernel fills first (it also clears the counters).
hipError_t launch_kernel_analysis(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c,
                                  float* a, float* b, float alpha, int qmax, uint16_t* xrk,
                                  unsigned long long* counters, hipStream_t stream) {
    const int ncc = (I + 511) / 512;
    const int nb = quantize_batches_per_wave(ncc, T);                      // rows per block = 32 * nb
    const int nrc = (T + 32 * nb - 1) / (32 * nb);
    if (!grid_fits((int64_t)ncc * nrc, kWaves * kLanes)) return hipErrorInvalidValue;     // before anything is enqueued
    const dim3 grid((unsigned)(ncc * nrc)), block(kWaves * kLanes);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0);
    const bool out_vec = (I % 8 == 0) && (reinterpret_cast<uintptr_t>(xrk) % 16 == 0);
    const double al = (double)alpha;
    if (a && b) {
        const hipError_t e = launch_scale_finalize(t, c, T, I, alpha, qmax, a, b, counters, 3, stream);
        if (e != hipSuccess) return e;
        if (vec)
            analysis_kernel<true, false><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, a, b, al, qmax, xrk, counters,
                                                                    ncc, nb, out_vec);
        else
            analysis_kernel<false, false><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, a, b, al, qmax, xrk, counters,
                                                                     ncc, nb, out_vec);
    } else {
        zero_counters_kernel<<<dim3(1), dim3(64), 0, stream>>>(counters);
        if (vec)
            analysis_kernel<true, true><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, nullptr, nullptr, al, qmax, xrk,
                                                                   counters, ncc, nb, out_vec);
        else
            analysis_kernel<false, true><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, nullptr, nullptr, al, qmax, xrk,
                                                                    counters, ncc, nb, out_vec);
    }
    return hipGetLastError();
}

}  // namespace cq
