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
//
// A batch of B matrices (sequences of a [B][S][I] activation tensor, each with its own column
// maxima) is one launch: the flat grid is B copies of the one-matrix grid, and a block first
// steps its pointers to its own matrix.
#include "cq_device.h"

namespace cq {
namespace {

constexpr int kWaves = 4;
constexpr int kBatch = 8;                 // rows per wave per batch

__global__ void zero_fill_kernel(uint32_t* __restrict__ p0, int n0, uint32_t* __restrict__ p1, int n1) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n0) p0[i] = 0u;
    else if (i - n0 < n1) p1[i - n0] = 0u;
}

// Block: 4 waves x (nb batches of 8 rows) x 512 columns.
template <bool VEC>
__global__ void __launch_bounds__(kWaves * kLanes)
absmax_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, uint32_t* __restrict__ t_bits,
              uint32_t* __restrict__ c_bits, int n_col_chunks, int nb, int blocks_per_matrix, int64_t matrix_stride) {
    __shared__ uint32_t lds_col[kWaves][4][kLanes];  // [wave][packed reg][lane]

    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    const int matrix = blockIdx.x / blocks_per_matrix;
    const int blk = blockIdx.x - matrix * blocks_per_matrix;
    X += (int64_t)matrix * matrix_stride;
    t_bits += (int64_t)matrix * T;
    c_bits += (int64_t)matrix * I;
    // flat grid, column chunk fastest: neighbouring blocks read neighbouring 1 KiB pieces of a row
    const int col_chunk = blk % n_col_chunks;
    const int row_chunk = blk / n_col_chunks;
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
        for (int k = 0; k < kBatch; ++k) rm[k] = absmax8(v[k], c0, c1, c2, c3);
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

hipError_t launch_absmax(const uint16_t* X, int B, int T, int I, int64_t ldx, int64_t matrix_stride, float* t,
                         float* c, hipStream_t stream) {
    const int ncc = (I + kColsPerWave - 1) / kColsPerWave;
    // rows per block = 32 * nb (4 waves x nb batches of 8 rows).  Small blocks are best for this read-only kernel
    // (a block's cost besides its reads is one atomic per column), and the quantize kernel that normally follows
    // walks each wave's rows from the last to the first: it finds them in the caches when a wave's rows here end
    // where a wave's rows there end, i.e. when 8 nb is a multiple of the 4 nbq rows of a quantize wave -- equal
    // to it if nbq is even.  Measured in a step, K1 + K3 stages: 4096 x 8192 (nbq 4) 50.4 us with nb 2, 52.2 with
    // nb 3, 53.2 with nb 4; 4096 x 5120 (nbq 3) 37.1 us with nb 3, 39.5 with nb 2 or 4.  Large odd nbq would make
    // blocks too big for this kernel's own good: nb 3 then.  Huge inputs take more rows per block, to bound the
    // number of column atomics.
    auto n_blocks_for = [&](int n) { return (int64_t)B * ncc * ((T + 32 * n - 1) / (32 * n)); };
    const int nbq = quantize_batches_per_wave((int64_t)B * ncc, T);
    int nb = nbq % 2 == 0 ? nbq / 2 : (nbq <= 3 ? nbq : 3);
    while (nb < 16 && n_blocks_for(nb) > 4096) ++nb;
    const int nrc = (T + 32 * nb - 1) / (32 * nb);
    if (!grid_fits((int64_t)B * ncc * nrc, kWaves * kLanes)) return hipErrorInvalidValue;
    {
        const int n = B * (T + I);                        // t is [B*T], c is [B*I]
        zero_fill_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(
            reinterpret_cast<uint32_t*>(t), B * T, reinterpret_cast<uint32_t*>(c), B * I);
    }
    const dim3 grid((unsigned)(B * ncc * nrc)), block(kWaves * kLanes);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0) && (B == 1 || matrix_stride % 8 == 0);
    if (vec)
        absmax_kernel<true><<<grid, block, 0, stream>>>(X, T, I, ldx, reinterpret_cast<uint32_t*>(t),
                                                        reinterpret_cast<uint32_t*>(c), ncc, nb, ncc * nrc, matrix_stride);
    else
        absmax_kernel<false><<<grid, block, 0, stream>>>(X, T, I, ldx, reinterpret_cast<uint32_t*>(t),
                                                         reinterpret_cast<uint32_t*>(c), ncc, nb, ncc * nrc, matrix_stride);
    return hipGetLastError();
}

}  // namespace cq
