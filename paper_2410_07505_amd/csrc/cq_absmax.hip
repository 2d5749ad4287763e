// Row and column absolute maxima of a binary16 matrix in one pass (Eq. 1: t_i; the CrossQuant
// equation: c_j).  HBM-bound: 2 bytes per element are read once; everything else is T+I floats.
//
// Work decomposition for 64-wide wavefronts: a wave owns 512 consecutive columns (one 16-byte
// load of 8 halfs per lane = 1 KiB contiguous per row) and streams over its rows in batches of
// 8 loads.  The 4 waves of a block share the column range and stack their rows.
//   - column maxima stay in 4 packed-u16 registers per lane for the whole stream (|x| as an
//     integer: for non-negative binary16 the bit pattern is monotonic), are combined across the
//     block's waves through LDS, then leave as one atomic max per column per block;
//   - row maxima of a batch of 8 rows are reduced across the 64 lanes by a transposed butterfly
//     (each exchange step halves the number of rows a lane still carries: 7 shuffles for 8 rows
//     instead of 48), ending with row g in lane 8*g.
// Device-wide atomics are resolved at the memory side and are far slower per cache line than
// loads, so both kinds are issued densely: consecutive lanes hit consecutive words (8 rows = one
// 32-byte request; 64 columns = 256 bytes per instruction).
// The atomics act on the binary32 bit pattern as an unsigned integer (values are >= 0), so the
// result is exact and independent of the order in which blocks finish.
#include "cq_kernels.h"

namespace cq {
namespace {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

constexpr int kLanes = 64;
constexpr int kColsPerWave = kLanes * 8;  // 512
constexpr int kWaves = 4;
constexpr int kBatch = 8;                 // rows per wave per batch

__device__ __forceinline__ uint32_t pkmax(uint32_t a, uint32_t b) {
    us2 r = __builtin_elementwise_max(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b));
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ uint32_t half_bits_to_float_bits(uint32_t h) { return __float_as_uint(h2f(h)); }

__device__ __forceinline__ uint32_t shx(uint32_t v, int off) { return (uint32_t)__shfl_xor((int)v, off, kLanes); }

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

// rm[g] = this lane's maximum over its 8 columns of row g (a 16-bit pattern).  Returns, in lane
// l with (l & 7) == 0, the maximum over all 64 lanes of row (l >> 3).
__device__ __forceinline__ uint32_t rows8_reduce(const uint32_t* rm, int lane) {
    const uint32_t p0 = rm[0] | (rm[1] << 16), p1 = rm[2] | (rm[3] << 16);
    const uint32_t p2 = rm[4] | (rm[5] << 16), p3 = rm[6] | (rm[7] << 16);
    const bool b5 = lane & 32, b4 = lane & 16, b3 = lane & 8;
    // lanes with bit 5 clear keep rows 0-3 and hand rows 4-7 to their partner, and vice versa
    const uint32_t q0 = pkmax(b5 ? p2 : p0, shx(b5 ? p0 : p2, 32));
    const uint32_t q1 = pkmax(b5 ? p3 : p1, shx(b5 ? p1 : p3, 32));
    const uint32_t r = pkmax(b4 ? q1 : q0, shx(b4 ? q0 : q1, 16));
    const uint32_t keep = b3 ? (r >> 16) : (r & 0xFFFFu);
    const uint32_t send = b3 ? (r & 0xFFFFu) : (r >> 16);
    uint32_t m = max(keep, shx(send, 8));
    m = max(m, shx(m, 4));
    m = max(m, shx(m, 2));
    m = max(m, shx(m, 1));
    return m;
}

__global__ void zero_fill_kernel(uint32_t* __restrict__ p0, int n0, uint32_t* __restrict__ p1, int n1) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n0) p0[i] = 0u;
    else if (i - n0 < n1) p1[i - n0] = 0u;
}

// Block: 4 waves x (nb batches of 8 rows) x 512 columns.
template <bool VEC>
__global__ void __launch_bounds__(kWaves * kLanes)
absmax_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, uint32_t* __restrict__ t_bits,
              uint32_t* __restrict__ c_bits, int n_col_chunks, int nb) {
    __shared__ uint32_t lds_col[kWaves][4][kLanes];  // [wave][packed reg][lane]

    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    // flat grid, column chunk fastest: neighbouring blocks read neighbouring 1 KiB pieces of a row
    const int col_chunk = blockIdx.x % n_col_chunks;
    const int row_chunk = blockIdx.x / n_col_chunks;
    const int j0 = col_chunk * kColsPerWave + lane * 8;
    const int rows_per_wave = nb * kBatch;
    const int row0 = row_chunk * (kWaves * rows_per_wave) + wave * rows_per_wave;

    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
    for (int b = 0; b < nb; ++b) {
        const int rb = row0 + b * kBatch;
        if (rb >= T) break;                               // wave-uniform
        uint4 v[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k)
            v[k] = (rb + k < T) ? load8<VEC>(X + (int64_t)(rb + k) * ldx, j0, I) : make_uint4(0u, 0u, 0u, 0u);
        uint32_t rm[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const uint32_t x0 = v[k].x & 0x7FFF7FFFu, x1 = v[k].y & 0x7FFF7FFFu;
            const uint32_t x2 = v[k].z & 0x7FFF7FFFu, x3 = v[k].w & 0x7FFF7FFFu;
            c0 = pkmax(c0, x0);
            c1 = pkmax(c1, x1);
            c2 = pkmax(c2, x2);
            c3 = pkmax(c3, x3);
            const uint32_t m = pkmax(pkmax(x0, x1), pkmax(x2, x3));
            rm[k] = max(m & 0xFFFFu, m >> 16);
        }
        const uint32_t m = rows8_reduce(rm, lane);
        const int r = rb + (lane >> 3);
        if ((lane & 7) == 0 && r < T && m) atomicMax(&t_bits[r], half_bits_to_float_bits(m));
    }

    // columns: combine the block's waves through LDS, then one atomic per column.  Thread idx
    // takes columns 2*idx and 2*idx+1 of the chunk = packed register (idx & 3) of lane (idx >> 2).
    lds_col[wave][0][lane] = c0;
    lds_col[wave][1][lane] = c1;
    lds_col[wave][2][lane] = c2;
    lds_col[wave][3][lane] = c3;
    __syncthreads();
    {
        const int idx = threadIdx.x;
        const int reg = idx & 3, ln = idx >> 2;
        const uint32_t m = pkmax(pkmax(lds_col[0][reg][ln], lds_col[1][reg][ln]),
                                 pkmax(lds_col[2][reg][ln], lds_col[3][reg][ln]));
        const int j = col_chunk * kColsPerWave + idx * 2;
        if (j < I && (m & 0xFFFFu)) atomicMax(&c_bits[j], half_bits_to_float_bits(m & 0xFFFFu));
        if (j + 1 < I && (m >> 16)) atomicMax(&c_bits[j + 1], half_bits_to_float_bits(m >> 16));
    }
}

}  // namespace

hipError_t launch_absmax(const uint16_t* X, int T, int I, int64_t ldx, float* t, float* c,
                         hipStream_t stream) {
    {
        const int n = T + I;
        zero_fill_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(
            reinterpret_cast<uint32_t*>(t), T, reinterpret_cast<uint32_t*>(c), I);
    }
    const int ncc = (I + kColsPerWave - 1) / kColsPerWave;
    // rows per block = 32 * nb: as many as keep at least 512 blocks in flight (fewer, larger
    // blocks mean fewer atomics; too few blocks leave CUs idle)
    int nb = 8;
    while (nb > 1 && (int64_t)ncc * ((T + 32 * nb - 1) / (32 * nb)) < 512) nb >>= 1;
    const int nrc = (T + 32 * nb - 1) / (32 * nb);
    const dim3 grid((unsigned)(ncc * nrc)), block(kWaves * kLanes);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0);
    if (vec)
        absmax_kernel<true><<<grid, block, 0, stream>>>(X, T, I, ldx, reinterpret_cast<uint32_t*>(t),
                                                        reinterpret_cast<uint32_t*>(c), ncc, nb);
    else
        absmax_kernel<false><<<grid, block, 0, stream>>>(X, T, I, ldx, reinterpret_cast<uint32_t*>(t),
                                                         reinterpret_cast<uint32_t*>(c), ncc, nb);
    return hipGetLastError();
}

}  // namespace cq
