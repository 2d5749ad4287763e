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
    for (int jj = 0; jj < RPW; ++jj) {
        const int j = j_begin + jj;
        if (j >= I) break;
        const float f = fold ? fold[j] : 1.0f;
        const uint16_t* row = W + (int64_t)j * O;
        uint32_t h[8];
        if (vec && k0 + 8 <= O) {
            const uint4 v = *reinterpret_cast<const uint4*>(row + k0);
            h[0] = v.x & 0xFFFFu; h[1] = v.x >> 16; h[2] = v.y & 0xFFFFu; h[3] = v.y >> 16;
            h[4] = v.z & 0xFFFFu; h[5] = v.z >> 16; h[6] = v.w & 0xFFFFu; h[7] = v.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = (k0 + e < O) ? row[k0 + e] : 0u;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float w = half_bits_to_float(h[e]);
            if (fold) w = f * w;
            m[e] = __builtin_fmaxf(m[e], __builtin_fabsf(w));
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

// 64 (input channels j) x 64 (output channels k) tile: read along k, write along j.
__global__ void __launch_bounds__(256)
weight_quant_kernel(const uint16_t* __restrict__ W, int I, int O, const float* __restrict__ fold,
                    const float* __restrict__ s, float qmax, int8_t* __restrict__ qw, int n_k_tiles,
                    bool in_vec, bool out_vec) {
    __shared__ __align__(16) int8_t tile[64][64 + 16];     // [k][j], padded
    const int kt = blockIdx.x % n_k_tiles, jt = blockIdx.x / n_k_tiles;
    const int k_base = kt * 64, j_base = jt * 64;
    const int c8 = threadIdx.x & 7;          // which group of 8 output channels
    const int k0 = k_base + c8 * 8;
    float sk[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sk[e] = (k0 + e < O) ? s[k0 + e] : 0.0f;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
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
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float w = half_bits_to_float(h[e]);
            if (fold) w = f * w;
            float r = (sk[e] == 0.0f) ? 0.0f : w / sk[e];
            r = __builtin_rintf(r);
            r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
            tile[c8 * 8 + e][jl] = (int8_t)(int)r;
        }
    }
    __syncthreads();
    // 64 rows (k) of 64 bytes (j): thread -> (k local, 16-byte piece)
    const int kl = threadIdx.x >> 2, piece = threadIdx.x & 3;
    const int k = k_base + kl;
    if (k < O) {
        const int j = j_base + piece * 16;
        int8_t* dst = qw + (int64_t)k * I + j;
        if (out_vec && j + 16 <= I) {
            *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(&tile[kl][piece * 16]);
        } else {
            for (int e = 0; e < 16; ++e)
                if (j + e < I) dst[e] = tile[kl][piece * 16 + e];
        }
    }
}

}  // namespace

hipError_t launch_weight_quantize(const uint16_t* W, int I, int O, const float* fold, int qmax, int8_t* qw,
                                  float* w_scale, hipStream_t stream) {
    constexpr int RPW = 32;
    zero_u32_kernel<<<dim3((O + 255) / 256), dim3(256), 0, stream>>>(reinterpret_cast<uint32_t*>(w_scale), O);
    const bool in_vec = (reinterpret_cast<uintptr_t>(W) % 16 == 0) && (O % 8 == 0);
    {
        const int ncc = (O + 511) / 512, nrc = (I + 4 * RPW - 1) / (4 * RPW);
        weight_colmax_kernel<RPW><<<dim3((unsigned)(ncc * nrc)), dim3(256), 0, stream>>>(
            W, I, O, fold, reinterpret_cast<uint32_t*>(w_scale), ncc, in_vec);
    }
    weight_scale_kernel<<<dim3((O + 255) / 256), dim3(256), 0, stream>>>(w_scale, O, (float)qmax);
    {
        const int nkt = (O + 63) / 64, njt = (I + 63) / 64;
        const bool out_vec = (reinterpret_cast<uintptr_t>(qw) % 16 == 0) && (I % 16 == 0);
        weight_quant_kernel<<<dim3((unsigned)(nkt * njt)), dim3(256), 0, stream>>>(
            W, I, O, fold, w_scale, (float)qmax, qw, nkt, in_vec, out_vec);
    }
    return hipGetLastError();
}

}  // namespace cq
