// Quantization-kernel analysis (Definition 1; Table 1; the "Remove Kernel" experiment of the
// zero-shot accuracy figures): one pass over X that writes X with its kernel elements zeroed and
// counts the kernel size and the two indicators of the kernel-size analysis,
//   case II:  c_j >= t_i          and          B~_ij < B_ij  (zero bound of CrossQuant below per-token's).
// Only "is the code zero" is needed, and q = rne(fl32(x / fl32(a b))) is 0 exactly when the quotient
// is at most 1/2, so the sign of one fma, |x| (1/b) - a/2, decides; a wave in which any lane has
// the two sides within 2^-20 of each other (the approximation is within 2^-22) takes the correctly
// rounded division for its row piece instead.  The three counts are population counts of compare
// masks.  About 9 vector instructions per element; with the division everywhere it was 35 and the
// kernel was bound by them, not by the 4 bytes per element it moves.
#include "cq_device.h"

namespace cq {
namespace {

constexpr int kWaves = 8;
constexpr int kU = 4;

// Block: 8 waves share 512 columns; each wave takes nb batches of 4 consecutive rows.
template <bool VEC>
__global__ void __launch_bounds__(kWaves * kLanes)
analysis_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, const float* __restrict__ t_vec,
                const float* __restrict__ c_vec, const float* __restrict__ a_vec, const float* __restrict__ b_vec,
                float qmax, uint16_t* __restrict__ xrk, unsigned long long* __restrict__ counters,
                int n_col_chunks, int nb, bool out_vec) {
    __shared__ uint32_t lds_cnt[kWaves][3];
    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    const int col_chunk = blockIdx.x % n_col_chunks;
    const int row_chunk = blockIdx.x / n_col_chunks;
    const int j0 = col_chunk * kColsPerWave + lane * 8;
    const int rows_per_wave = nb * kU;
    const int row0 = row_chunk * (kWaves * rows_per_wave) + wave * rows_per_wave;

    float b[8], rb[8], c[8];
    unsigned long long valid[8];                            // lanes whose column e exists
    bool odd = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        b[e] = (j0 + e < I) ? b_vec[j0 + e] : 0.0f;
        c[e] = (j0 + e < I) ? c_vec[j0 + e] : 0.0f;
        rb[e] = safe_rcp(b[e]);
        odd |= tiny_factor(b[e]);
        valid[e] = __ballot(j0 + e < I);
    }
    int nvalid = I - j0;
    nvalid = nvalid < 0 ? 0 : (nvalid > 8 ? 8 : nvalid);
    // per row: a_i, t_i and the per-token step fl32(t_i / q_max), one row per lane
    const bool has_row = lane < rows_per_wave && row0 + lane < T;
    const float a_lane = has_row ? a_vec[row0 + lane] : 0.0f;
    const float t_lane = has_row ? t_vec[row0 + lane] : 0.0f;
    const float pt_lane = (float)((double)t_lane / (double)qmax);

    uint32_t zeros = 0, col_ge = 0, smaller = 0;            // wave totals (uniform)
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
            bool close = false;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = __builtin_fmaf(__builtin_fabsf((float)h[e]), rb[e], -ha);
                nonzero[e] = d > 0.0f;
                close |= __builtin_fabsf(d) <= tol;
            }
            // a == 0: D = 0 and every code of the row is 0 by definition (left to the exact path)
            if (__any(close || odd || tiny_factor(a) || a == 0.0f)) {
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
                const float D = a * b[e];
                zeros += (uint32_t)__builtin_popcountll(valid[e] & ~__ballot(nonzero[e]));
                col_ge += (uint32_t)__builtin_popcountll(valid[e] & __ballot(c[e] >= ti));
                smaller += (uint32_t)__builtin_popcountll(valid[e] & __ballot(D < pt));      // 0.5 * D < 0.5 * pt, exactly
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

    if (lane == 0) {
        lds_cnt[wave][0] = zeros;
        lds_cnt[wave][1] = col_ge;
        lds_cnt[wave][2] = smaller;
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

hipError_t launch_kernel_analysis(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c,
                                  const float* a, const float* b, int qmax, uint16_t* xrk,
                                  unsigned long long* counters, hipStream_t stream) {
    const int ncc = (I + 511) / 512;
    // rows per block = 32 * nb: the smallest nb >= 2 with at most 512 blocks, as for the quantize kernel
    auto n_blocks_for = [&](int n) { return (int64_t)ncc * ((T + 32 * n - 1) / (32 * n)); };
    const int nb_max = T >= 512 ? 16 : (T + 31) / 32;
    int nb = nb_max < 2 ? nb_max : 2;
    while (nb < nb_max && n_blocks_for(nb) > 512) ++nb;
    if (nb == 2 && n_blocks_for(2) < 200) nb = 1;
    const int nrc = (T + 32 * nb - 1) / (32 * nb);
    if (!grid_fits((int64_t)ncc * nrc, kWaves * kLanes)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(ncc * nrc)), block(kWaves * kLanes);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0);
    const bool out_vec = (I % 8 == 0) && (reinterpret_cast<uintptr_t>(xrk) % 16 == 0);
    if (vec)
        analysis_kernel<true><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, a, b, (float)qmax, xrk, counters, ncc,
                                                         nb, out_vec);
    else
        analysis_kernel<false><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, a, b, (float)qmax, xrk, counters, ncc,
                                                          nb, out_vec);
    return hipGetLastError();
}

}  // namespace cq
