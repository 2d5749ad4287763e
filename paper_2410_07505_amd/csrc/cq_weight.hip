// Per-output-channel weight quantization (Eq. 2) with an optional per-input-channel fold
// factor, written transposed ([O][I], contraction axis contiguous) for the integer GEMM.
// Weight preparation: done once per weight (or once per calibrated column scale), so these
// kernels are kept straightforward -- coalesced reads, an LDS transpose, exact division.
//   W'_jk = fl32(f_j * W_jk);  s_k = fl32(max_j |W'_jk| / q_max);  qw_kj = clamp(rne(fl32(W'_jk / s_k)))
#include "cq_kernels.h"

namespace cq {
namespace {

constexpr int kLanes = 64;

__global__ void zero_u32_kernel(uint32_t* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
    return h2f(h);
}

// max_j |f_j * W_jk| accumulated into smax_bits[k] (binary32 bit pattern of a value >= 0).
// Block: 256 threads = 4 waves sharing 512 columns; each wave takes RPW consecutive rows.
template <int RPW>
__global__ void __launch_bounds__(256)
weight_colmax_kernel(const uint16_t* __restrict__ W, int I, int O, const float* __restrict__ fold,
                     uint32_t* __restrict__ smax_bits, int n_col_chunks, bool vec) {
    __shared__ uint32_t lds[4][8][kLanes];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col_chunk = blockIdx.x % n_col_chunks, row_chunk = blockIdx.x / n_col_chunks;
    const int k0 = col_chunk * 512 + lane * 8;
    const int j_begin = row_chunk * (4 * RPW) + wave * RPW;
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = 0.0f;
    // batches of 8 rows: all eight loads are issued before the first value is used
    for (int jb = 0; jb < RPW; jb += 8) {
        const int j8 = j_begin + jb;
        if (j8 >= I) break;                              // wave-uniform
        uint4 v[8];
        float f[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int j = j8 + r;
            v[r] = make_uint4(0u, 0u, 0u, 0u);
            f[r] = 1.0f;
            if (j < I) {
                const uint16_t* row = W + (int64_t)j * O;
                if (fold) f[r] = fold[j];
                if (vec && k0 + 8 <= O) {
                    v[r] = *reinterpret_cast<const uint4*>(row + k0);
                } else {
                    uint32_t h[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) h[e] = (k0 + e < O) ? row[k0 + e] : 0u;
                    v[r] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t w32[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float w = half_bits_to_float((w32[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
                if (fold) w = f[r] * w;
                m[e] = __builtin_fmaxf(m[e], __builtin_fabsf(w));
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) lds[wave][e][lane] = __float_as_uint(m[e]);
    __syncthreads();
    for (int idx = threadIdx.x; idx < 8 * kLanes; idx += 256) {
        const int e = idx / kLanes, ln = idx % kLanes;
        uint32_t v = max(max(lds[0][e][ln], lds[1][e][ln]), max(lds[2][e][ln], lds[3][e][ln]));
        const int k = col_chunk * 512 + ln * 8 + e;
        if (k < O && v) atomicMax(&smax_bits[k], v);
    }
}

__global__ void weight_scale_kernel(float* __restrict__ s, int O, float qmax) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < O) s[k] = s[k] / qmax;      // in place: max -> step
}

// 128 (input channels j) x 64 (output channels k) tile: read along k, write along j in whole
// 128-byte row pieces.
__global__ void __launch_bounds__(256)
weight_quant_kernel(const uint16_t* __restrict__ W, int I, int O, const float* __restrict__ fold,
                    const float* __restrict__ s, float qmax, int8_t* __restrict__ qw, int n_k_tiles,
                    bool in_vec, bool out_vec) {
    __shared__ __align__(16) int8_t tile[64][128 + 16];    // [k][j], padded
    const int kt = blockIdx.x % n_k_tiles, jt = blockIdx.x / n_k_tiles;
    const int k_base = kt * 64, j_base = jt * 128;
    const int c8 = threadIdx.x & 7;          // which group of 8 output channels
    const int k0 = k_base + c8 * 8;
    // The correctly rounded division is taken only where it can matter (as in the activation
    // quantizer): w * (1/s) is rounded to an integer by one fma against 1.5 * 2^23 (the sum's ulp is
    // 1), a second fma gives the distance from it, and a wave in which any lane is within the
    // approximation's error of a rounding tie (or has a step so small that its reciprocal leaves the
    // normal range) redoes its eight elements with the division.
    constexpr float kRound = 12582912.0f;             // 1.5 * 2^23
    constexpr float kTol = 1.9073486328125e-06f;      // 2^-19; the approximation is within 2^-22
    float sk[8], rs[8];
    bool odd_step = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        sk[e] = (k0 + e < O) ? s[k0 + e] : 0.0f;
        rs[e] = (sk[e] == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(sk[e]);
        odd_step |= sk[e] != 0.0f && !(sk[e] >= 7.888609052210118e-31f);     // 2^-100, also catches NaN
    }
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int jl = pass * 32 + (threadIdx.x >> 3);
        const int j = j_base + jl;
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = 0u;
        float f = 1.0f;
        if (j < I) {
            const uint16_t* row = W + (int64_t)j * O;
            if (fold) f = fold[j];
            if (in_vec && k0 + 8 <= O) {
                const uint4 v = *reinterpret_cast<const uint4*>(row + k0);
                h[0] = v.x & 0xFFFFu; h[1] = v.x >> 16; h[2] = v.y & 0xFFFFu; h[3] = v.y >> 16;
                h[4] = v.z & 0xFFFFu; h[5] = v.z >> 16; h[6] = v.w & 0xFFFFu; h[7] = v.w >> 16;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) h[e] = (k0 + e < O) ? row[k0 + e] : 0u;
            }
        }
        float w[8], m[8];
        float score = 0.0f, big = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            w[e] = half_bits_to_float(h[e]);
            if (fold) w[e] = f * w[e];
            m[e] = __builtin_fmaf(w[e], rs[e], kRound);
            const float q = m[e] - kRound;
            const float d = __builtin_fmaf(w[e], rs[e], -q);
            score = __builtin_fmaxf(score, __builtin_fmaf(__builtin_fabsf(q), kTol, __builtin_fabsf(d)));
            big = __builtin_fmaxf(big, __builtin_fabsf(q));
        }
        if (__any(score >= 0.5f - kTol || !(big <= qmax) || odd_step)) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float r = (sk[e] == 0.0f) ? 0.0f : w[e] / sk[e];
                r = __builtin_rintf(r);
                r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
                m[e] = r + kRound;
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[c8 * 8 + e][jl] = (int8_t)(__float_as_uint(m[e]) & 0xFFu);   // low byte = code
    }
    __syncthreads();
    // 64 rows (k) of 128 bytes (j): thread -> (k local, 32-byte piece) = two 16-byte stores
    const int kl = threadIdx.x >> 2, piece = threadIdx.x & 3;
    const int k = k_base + kl;
    if (k < O) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int jo = piece * 32 + half * 16;
            const int j = j_base + jo;
            int8_t* dst = qw + (int64_t)k * I + j;
            if (out_vec && j + 16 <= I) {
                *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(&tile[kl][jo]);
            } else {
                for (int e = 0; e < 16; ++e)
                    if (j + e < I) dst[e] = tile[kl][jo + e];
            }
        }
    }
}

// Group-wise variant: every output channel is cut into groups of g consecutive input channels,
// each with its own step (Background section's group-wise quantization).  One block handles one
// group of one 64-channel tile: pass 1 finds the 64 group maxima, pass 2 quantizes, transposes
// through LDS 32 input channels at a time, and optionally writes the dequantized weights.
__global__ void __launch_bounds__(256)
weight_group_kernel(const uint16_t* __restrict__ W, int I, int O, const float* __restrict__ fold, int g,
                    float qmax, int8_t* __restrict__ qw, float* __restrict__ s, uint16_t* __restrict__ wdq,
                    int n_k_tiles, bool in_vec, bool out_vec) {
    __shared__ float lmax[32][64 + 1];
    __shared__ float lstep[64];
    __shared__ __align__(16) int8_t tile[64][128 + 16];        // [k][j within the 128-row chunk]
    const int kt = blockIdx.x % n_k_tiles, G = blockIdx.x / n_k_tiles;
    const int ng = I / g;
    const int c8 = threadIdx.x & 7, jr = threadIdx.x >> 3;
    const int k0 = kt * 64 + c8 * 8;
    const int j_begin = G * g, j_end = j_begin + g;

    auto load_row = [&](int j, float (&w)[8]) {
        uint32_t h[8];
        const uint16_t* row = W + (int64_t)j * O;
        if (in_vec && k0 + 8 <= O) {
            const uint4 v = *reinterpret_cast<const uint4*>(row + k0);
            h[0] = v.x & 0xFFFFu; h[1] = v.x >> 16; h[2] = v.y & 0xFFFFu; h[3] = v.y >> 16;
            h[4] = v.z & 0xFFFFu; h[5] = v.z >> 16; h[6] = v.w & 0xFFFFu; h[7] = v.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = (k0 + e < O) ? row[k0 + e] : 0u;
        }
        const float f = fold ? fold[j] : 1.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            w[e] = h2f(h[e]);
            if (fold) w[e] = f * w[e];
        }
    };

    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = 0.0f;
    for (int j = j_begin + jr; j < j_end; j += 32) {
        float w[8];
        load_row(j, w);
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] = __builtin_fmaxf(m[e], __builtin_fabsf(w[e]));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) lmax[jr][c8 * 8 + e] = m[e];
    __syncthreads();
    if (threadIdx.x < 64) {
        float mm = 0.0f;
        for (int r = 0; r < 32; ++r) mm = __builtin_fmaxf(mm, lmax[r][threadIdx.x]);
        const float step = mm / qmax;
        lstep[threadIdx.x] = step;
        const int k = kt * 64 + threadIdx.x;
        if (k < O) s[(int64_t)k * ng + G] = step;
    }
    __syncthreads();
    // the division is taken only near a rounding tie, as in weight_quant_kernel
    constexpr float kRound = 12582912.0f;             // 1.5 * 2^23
    constexpr float kTol = 1.9073486328125e-06f;      // 2^-19
    float sk[8], rs[8];
    bool odd_step = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        sk[e] = lstep[c8 * 8 + e];
        rs[e] = (sk[e] == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(sk[e]);
        odd_step |= sk[e] != 0.0f && !(sk[e] >= 7.888609052210118e-31f);     // 2^-100, also catches NaN
    }

    // up to 128 input channels of the group at a time (4 passes of 32 rows), so that the codes leave
    // in whole 128-byte row pieces where the group is that long
    for (int jc = j_begin; jc < j_end; jc += 128) {
        const int jc_end = min(jc + 128, j_end);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
            const int j = jc + sub * 32 + jr;
            const bool live = j < jc_end;
            float w[8], q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = 0.0f;
            if (live) load_row(j, w);
            float score = 0.0f, big = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float mm = __builtin_fmaf(w[e], rs[e], kRound);
                q[e] = mm - kRound;
                const float d = __builtin_fmaf(w[e], rs[e], -q[e]);
                score = __builtin_fmaxf(score, __builtin_fmaf(__builtin_fabsf(q[e]), kTol, __builtin_fabsf(d)));
                big = __builtin_fmaxf(big, __builtin_fabsf(q[e]));
            }
            if (__any(score >= 0.5f - kTol || !(big <= qmax) || odd_step)) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float r = (sk[e] == 0.0f) ? 0.0f : w[e] / sk[e];
                    r = __builtin_rintf(r);
                    q[e] = __builtin_amdgcn_fmed3f(r, -qmax, qmax) + 0.0f;      // -0 (from rounding e.g. -0.3) -> +0
                }
            }
            if (live) {
                uint32_t hq[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    tile[c8 * 8 + e][sub * 32 + jr] = (int8_t)(int)q[e];
                    hq[e] = f2h(rounded_f32(q[e] * sk[e]));
                }
                if (wdq) {
                    uint16_t* dst = wdq + (int64_t)j * O + k0;
                    if (in_vec && k0 + 8 <= O && (reinterpret_cast<uintptr_t>(wdq) % 16 == 0)) {
                        *reinterpret_cast<uint4*>(dst) = make_uint4(hq[0] | (hq[1] << 16), hq[2] | (hq[3] << 16),
                                                                    hq[4] | (hq[5] << 16), hq[6] | (hq[7] << 16));
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (k0 + e < O) dst[e] = (uint16_t)hq[e];
                    }
                }
            }
        }
        __syncthreads();
        {   // 64 rows (k) of up to 128 bytes (j): thread -> (k local, 32-byte piece) = two 16-byte stores
            const int kl = threadIdx.x >> 2, piece = threadIdx.x & 3;
            const int k = kt * 64 + kl;
            if (k < O) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int jl = piece * 32 + half * 16;
                    const int jo = jc + jl;
                    int8_t* dst = qw + (int64_t)k * I + jo;
                    if (out_vec && jo + 16 <= jc_end) {
                        *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(&tile[kl][jl]);
                    } else {
                        for (int e = 0; e < 16; ++e)
                            if (jo + e < jc_end) dst[e] = tile[kl][jl + e];
                    }
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_weight_quantize(const uint16_t* W, int I, int O, const float* fold, int qmax, int8_t* qw,
                                  float* w_scale, hipStream_t stream) {
    constexpr int RPW = 32;
    if (!grid_fits((int64_t)((O + 63) / 64) * ((I + 127) / 128), 256)) return hipErrorInvalidValue;   // the larger of the two grids
    zero_u32_kernel<<<dim3((O + 255) / 256), dim3(256), 0, stream>>>(reinterpret_cast<uint32_t*>(w_scale), O);
    const bool in_vec = (reinterpret_cast<uintptr_t>(W) % 16 == 0) && (O % 8 == 0);
    {
        const int ncc = (O + 511) / 512, nrc = (I + 4 * RPW - 1) / (4 * RPW);
        weight_colmax_kernel<RPW><<<dim3((unsigned)(ncc * nrc)), dim3(256), 0, stream>>>(
            W, I, O, fold, reinterpret_cast<uint32_t*>(w_scale), ncc, in_vec);
    }
    weight_scale_kernel<<<dim3((O + 255) / 256), dim3(256), 0, stream>>>(w_scale, O, (float)qmax);
    {
        const int nkt = (O + 63) / 64, njt = (I + 127) / 128;
        const bool out_vec = (reinterpret_cast<uintptr_t>(qw) % 16 == 0) && (I % 16 == 0);
        weight_quant_kernel<<<dim3((unsigned)(nkt * njt)), dim3(256), 0, stream>>>(
            W, I, O, fold, w_scale, (float)qmax, qw, nkt, in_vec, out_vec);
    }
    return hipGetLastError();
}

hipError_t launch_weight_quantize_grouped(const uint16_t* W, int I, int O, const float* fold, int group, int qmax,
                                          int8_t* qw, float* w_scale, uint16_t* wdq, hipStream_t stream) {
    const int nkt = (O + 63) / 64, ng = I / group;
    const bool in_vec = (reinterpret_cast<uintptr_t>(W) % 16 == 0) && (O % 8 == 0);
    const bool out_vec = (reinterpret_cast<uintptr_t>(qw) % 16 == 0) && (I % 16 == 0) && (group % 16 == 0);
    if (!grid_fits((int64_t)nkt * ng, 256)) return hipErrorInvalidValue;
    weight_group_kernel<<<dim3((unsigned)(nkt * ng)), dim3(256), 0, stream>>>(W, I, O, fold, group, (float)qmax, qw,
                                                                             w_scale, wdq, nkt, in_vec, out_vec);
    return hipGetLastError();
}

}  // namespace cq
