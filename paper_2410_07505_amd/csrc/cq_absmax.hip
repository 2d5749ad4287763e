// Row and column absolute maxima of a binary16 matrix in one pass (Eq. 1: t_i; the CrossQuant
// equation: c_j).  HBM-bound: 2 bytes per element are read once; everything else is T+I floats.
//
// Work decomposition for 64-wide wavefronts: a wave owns 512 consecutive columns (one 16-byte
// load of 8 halfs per lane = 1 KiB contiguous per row) and RPW consecutive rows.  The W waves of
// a block share the column range and stack their rows, so a block covers (W*RPW) x 512.
//   - column maxima stay in 4 packed-u16 registers per lane across the row loop (|x| as an
//     integer: for non-negative binary16 the bit pattern is monotonic), are combined across the
//     block's waves through LDS, then leave as one atomic max per column per block;
//   - row maxima are reduced across the 64 lanes with shuffles and leave as one atomic max per
//     row per wave.
// The atomics act on the binary32 bit pattern as an unsigned integer (values are >= 0), so the
// result is exact and independent of the order in which blocks finish.
#include "cq_kernels.h"

namespace cq {
namespace {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

constexpr int kLanes = 64;
constexpr int kColsPerWave = kLanes * 8;  // 512

__device__ __forceinline__ uint32_t pkmax(uint32_t a, uint32_t b) {
    us2 r = __builtin_elementwise_max(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b));
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ uint32_t half_bits_to_float_bits(uint32_t h) {
    return __float_as_uint(h2f(h));
}

// 8 halfs starting at column j of a row; columns >= I read as zero (neutral for a maximum).
template <bool VEC>
__device__ __forceinline__ uint4 load8(const uint16_t* __restrict__ row, int j, int I) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (VEC && j + 8 <= I) {
        v = *reinterpret_cast<const uint4*>(row + j);
    } else if (j < I) {
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = (j + e < I) ? row[j + e] : 0u;
        v.x = h[0] | (h[1] << 16);
        v.y = h[2] | (h[3] << 16);
        v.z = h[4] | (h[5] << 16);
        v.w = h[6] | (h[7] << 16);
    }
    return v;
}

__global__ void zero_fill_kernel(uint32_t* __restrict__ p0, int n0, uint32_t* __restrict__ p1, int n1) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n0) p0[i] = 0u;
    else if (i - n0 < n1) p1[i - n0] = 0u;
}

template <int WAVES, int RPW, bool VEC>
__global__ void __launch_bounds__(WAVES * kLanes)
absmax_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx,
              uint32_t* __restrict__ t_bits, uint32_t* __restrict__ c_bits, int n_col_chunks) {
    __shared__ uint32_t lds_col[WAVES][4][kLanes];  // [wave][packed reg][lane]

    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    // flat grid, column chunk fastest: neighbouring blocks read neighbouring 1 KiB pieces of a row
    const int col_chunk = blockIdx.x % n_col_chunks;
    const int row_chunk = blockIdx.x / n_col_chunks;
    const int j0 = col_chunk * kColsPerWave + lane * 8;
    const int row0 = row_chunk * (WAVES * RPW) + wave * RPW;

    uint4 v[RPW];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
        const int r = row0 + k;
        v[k] = (r < T) ? load8<VEC>(X + (int64_t)r * ldx, j0, I) : make_uint4(0u, 0u, 0u, 0u);
    }

    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
    uint32_t rowmax[RPW];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
        const uint32_t x0 = v[k].x & 0x7FFF7FFFu, x1 = v[k].y & 0x7FFF7FFFu;
        const uint32_t x2 = v[k].z & 0x7FFF7FFFu, x3 = v[k].w & 0x7FFF7FFFu;
        c0 = pkmax(c0, x0);
        c1 = pkmax(c1, x1);
        c2 = pkmax(c2, x2);
        c3 = pkmax(c3, x3);
        uint32_t m = pkmax(pkmax(x0, x1), pkmax(x2, x3));
        m = max(m & 0xFFFFu, m >> 16);
        rowmax[k] = m;
    }

    // rows: pack two rows per register, butterfly over the 64 lanes
#pragma unroll
    for (int k = 0; k < RPW; k += 2) {
        uint32_t m = rowmax[k] | ((k + 1 < RPW ? rowmax[k + 1] : 0u) << 16);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = pkmax(m, (uint32_t)__shfl_xor((int)m, off, kLanes));
        if (lane == 0) {
            const int r = row0 + k;
            if (r < T) atomicMax(&t_bits[r], half_bits_to_float_bits(m & 0xFFFFu));
            if (k + 1 < RPW && r + 1 < T) atomicMax(&t_bits[r + 1], half_bits_to_float_bits(m >> 16));
        }
    }

    // columns: combine the block's waves through LDS, then one atomic per column
    lds_col[wave][0][lane] = c0;
    lds_col[wave][1][lane] = c1;
    lds_col[wave][2][lane] = c2;
    lds_col[wave][3][lane] = c3;
    __syncthreads();
    for (int idx = threadIdx.x; idx < 4 * kLanes; idx += WAVES * kLanes) {
        const int reg = idx / kLanes, ln = idx % kLanes;
        uint32_t m = lds_col[0][reg][ln];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) m = pkmax(m, lds_col[w][reg][ln]);
        const int j = col_chunk * kColsPerWave + ln * 8 + reg * 2;
        if (j < I && (m & 0xFFFFu)) atomicMax(&c_bits[j], half_bits_to_float_bits(m & 0xFFFFu));
        if (j + 1 < I && (m >> 16)) atomicMax(&c_bits[j + 1], half_bits_to_float_bits(m >> 16));
    }
}

}  // namespace

hipError_t launch_absmax(const uint16_t* X, int T, int I, int64_t ldx, float* t, float* c,
                         hipStream_t stream) {
    constexpr int WAVES = 8, RPW = 16;
    {
        const int n = T + I;
        zero_fill_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(
            reinterpret_cast<uint32_t*>(t), T, reinterpret_cast<uint32_t*>(c), I);
    }
    const int ncc = (I + kColsPerWave - 1) / kColsPerWave;
    const int nrc = (T + WAVES * RPW - 1) / (WAVES * RPW);
    const dim3 grid((unsigned)(ncc * nrc));
    const dim3 block(WAVES * kLanes);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0);
    if (vec)
        absmax_kernel<WAVES, RPW, true><<<grid, block, 0, stream>>>(
            X, T, I, ldx, reinterpret_cast<uint32_t*>(t), reinterpret_cast<uint32_t*>(c), ncc);
    else
        absmax_kernel<WAVES, RPW, false><<<grid, block, 0, stream>>>(
            X, T, I, ldx, reinterpret_cast<uint32_t*>(t), reinterpret_cast<uint32_t*>(c), ncc);
    return hipGetLastError();
}

}  // namespace cq
