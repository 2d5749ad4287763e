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
#include <mutex>

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

// The same pass for the layout every real activation has (X 16-byte aligned, ldx % 8 == 0, I % 8 == 0), with three
// differences:
//   - rows are read as raw buffers (base and length in scalar registers, range-checked by the hardware: columns
//     past the end read as 0 with no per-lane branch);
//   - the row maxima wait in LDS until the block has read all its rows, so every atomic of the block is issued at
//     its very end;
//   - CLEAR: the launch clears t and c itself.  The first n_clear blocks do nothing but store zeros (at device
//     scope), wait until the stores have been performed and then add 1 to a counter in library-owned device
//     memory; it counts the clearing blocks that have finished over all launches on this stream slot so far.
//     Every other block reads the counter when it is about to issue its atomics, more than ten microseconds
//     later in a full-size launch, and waits (bounded) until it has reached `target`, the value it has when this
//     launch's clearing blocks are done.  Blocks are dispatched in index order, so the clearing blocks are
//     running or finished before any other block exists.  This saves the separate clearing kernel and the gap
//     between the two launches.
template <bool CLEAR>
__global__ void __launch_bounds__(kWaves * kLanes)
absmax_stream_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, uint32_t* __restrict__ t_bits,
                     uint32_t* __restrict__ c_bits, int n_col_chunks, int nb, int blocks_per_matrix,
                     int64_t matrix_stride, int n_clear, int n_t_words, int n_c_words, unsigned int* cleared,
                     unsigned int target, unsigned int spin_limit) {
    __shared__ uint32_t lds_col[kWaves][4][kLanes];  // [wave][packed reg][lane]
    __shared__ uint32_t lds_row[kWaves * 16 * kBatch];   // row maxima of the block's rows (16-bit patterns)
    __shared__ int lds_go;

    int block = blockIdx.x;
    if (CLEAR) {
        if (block < n_clear) {
            // clearing block: an equal share of the words of t followed by those of c
            const int total = n_t_words + n_c_words;
            const int share = (total + n_clear - 1) / n_clear;
            const int end = min(total, (block + 1) * share);
            for (int w = block * share + (int)threadIdx.x; w < end; w += kWaves * kLanes) {
                uint32_t* dst = w < n_t_words ? t_bits + w : c_bits + (w - n_t_words);
                __hip_atomic_store(dst, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this thread's stores have been performed
            __syncthreads();
            if (threadIdx.x == 0) __hip_atomic_fetch_add(cleared, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        block -= n_clear;
    }
    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
    const int matrix = block / blocks_per_matrix;
    const int blk = block - matrix * blocks_per_matrix;
    X += (int64_t)matrix * matrix_stride;
    t_bits += (int64_t)matrix * T;
    c_bits += (int64_t)matrix * I;
    const int col_chunk = blk % n_col_chunks;
    const int row_chunk = blk / n_col_chunks;
    const int col0 = col_chunk * kColsPerWave;
    const int cols_here = min(kColsPerWave, I - col0);           // a multiple of 8
    const int rows_per_wave = nb * kBatch;
    const int rows_per_block = kWaves * rows_per_wave;
    const int block_row0 = row_chunk * rows_per_block;
    const int row0 = block_row0 + wave * rows_per_wave;

    // rows past the last one are read from the last row (a duplicate changes no maximum)
    auto load_batch = [&](uint4 (&dst)[kBatch], int b) {
        if (b >= nb) return;                                     // scalar condition
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int r = min(row0 + b * kBatch + k, T - 1);
            dst[k] = buffer_load16(row_buffer(X + (int64_t)r * ldx + col0, cols_here * 2), lane * 16);
        }
    };
    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
    auto reduce_batch = [&](const uint4 (&v)[kBatch], int b) {
        uint32_t rm[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) rm[k] = absmax8(v[k], c0, c1, c2, c3);
        const uint32_t m = rows8_reduce(rm, lane);
        if ((lane & 7) == 0) lds_row[wave * rows_per_wave + b * kBatch + (lane >> 3)] = m;
    };
    // One set of 8 rows at a time: with a second set in flight while the first is reduced, this kernel got 0.6 us
    // slower and the quantize kernel that follows it 1 us slower (4096 x 8192, in a step).
    uint4 v[kBatch];
    for (int b = 0; b < nb; ++b) {
        load_batch(v, b);
        reduce_batch(v, b);
    }
    lds_col[wave][0][lane] = c0;
    lds_col[wave][1][lane] = c1;
    lds_col[wave][2][lane] = c2;
    lds_col[wave][3][lane] = c3;
    if (CLEAR && threadIdx.x == 0) {
        int go = 0;
        for (unsigned spin = 0; spin < spin_limit; ++spin) {
            // the counter only grows (mod 2^32): reached when the difference is not negative
            if ((int)(__hip_atomic_load(cleared, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0) {
                go = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
        lds_go = go;       // 0 only if the clearing blocks have not finished after seconds: the maxima are then unreliable
    }
    __syncthreads();
    {
        // rows: thread k takes row k of the block (consecutive lanes hit consecutive words)
        const int k = (int)threadIdx.x;
        for (int rr = k; rr < rows_per_block; rr += kWaves * kLanes) {
            const int r = block_row0 + rr;
            const uint32_t m = lds_row[rr];
            if (r < T && m) atomicMax(&t_bits[r], half_bits_to_float_bits(m));
        }
        // columns: thread idx takes columns 2*idx and 2*idx+1 of the chunk = packed register (idx & 3) of lane (idx >> 2)
        const int reg = k & 3, ln = k >> 2;
        const uint32_t m = pkmax(pkmax(lds_col[0][reg][ln], lds_col[1][reg][ln]),
                                 pkmax(lds_col[2][reg][ln], lds_col[3][reg][ln]));
        const int j = col0 + k * 2;
        if (j < I && (m & 0xFFFFu)) atomicMax(&c_bits[j], half_bits_to_float_bits(m & 0xFFFFu));
        if (j + 1 < I && (m >> 16)) atomicMax(&c_bits[j + 1], half_bits_to_float_bits(m >> 16));
    }
    (void)lds_go;
}

// Clearing blocks that have finished, over all launches of a stream slot (see absmax_stream_kernel).
__device__ unsigned int g_cleared[kStateSlots];

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
    // blocks too big for this kernel's own good: nb 3 then.  A wave wants at least two batches to have loads in
    // flight while it reduces (4096 x 4096, nbq 2: this kernel 12.6 us with nb 1, 10.8 with nb 2).  Four waves
    // per block is the optimum as well: 4096 x 8192 takes 23.6, 17.3, 15.8, 18.3 and 18.5 us as a stage with 1, 2,
    // 4, 8 and 16 waves (more blocks mean more column atomics, larger blocks turn over too slowly).  Huge inputs take more rows per block, to bound the
    // number of column atomics.
    auto n_blocks_for = [&](int n) { return (int64_t)B * ncc * ((T + 32 * n - 1) / (32 * n)); };
    const int nbq = quantize_batches_per_wave((int64_t)B * ncc, T);
    int nb = nbq % 2 == 0 ? (nbq >= 4 ? nbq / 2 : 2) : (nbq <= 3 ? nbq : 3);
    while (nb < 16 && n_blocks_for(nb) > 4096) ++nb;
    const int nrc = (T + 32 * nb - 1) / (32 * nb);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0) && (B == 1 || matrix_stride % 8 == 0);
    const int64_t n_work = (int64_t)B * ncc * nrc;
    const int n_words = B * (T + I);                          // t is [B*T], c is [B*I]
    // clearing blocks of the self-clearing launch: a multiple of 8, so that a working block keeps the L2 (block
    // index mod 8) it has without them, the one that holds its columns when the quantize kernel comes for them
    int n_clear = 8 * ((n_words + 8 * 2048 - 1) / (8 * 2048));
    if (n_clear > 64) n_clear = 64;
    if (!grid_fits(n_work + n_clear, kWaves * kLanes)) return hipErrorInvalidValue;
    uint32_t* tb = reinterpret_cast<uint32_t*>(t);
    uint32_t* cb = reinterpret_cast<uint32_t*>(c);
    const dim3 block(kWaves * kLanes);
    if (vec && I % 8 == 0) {
        // One launch that clears for itself needs a counter of its own (a stream slot) and a target value that
        // differs from launch to launch, which a captured graph cannot have (its arguments are frozen): captured
        // calls and streams without a slot clear with a kernel of their own first.
        const int slot = stream_slot(stream);
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        const bool plain_stream = slot >= 0 && hipStreamIsCapturing(stream, &cap) == hipSuccess &&
                                  cap == hipStreamCaptureStatusNone;
        if (plain_stream) {
            static std::mutex mu;
            static unsigned int reached[64][kStateSlots];      // what a device's g_cleared[slot] reaches once all launches so far have cleared
            static unsigned int* counters[64];                 // device address of g_cleared on each device, once known
            int dev = 0;
            hipError_t e = hipGetDevice(&dev);
            if (e != hipSuccess) return e;
            if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
            std::lock_guard<std::mutex> lock(mu);              // launches and targets stay in the same order
            if (!counters[dev]) {
                e = hipGetSymbolAddress(reinterpret_cast<void**>(&counters[dev]), HIP_SYMBOL(g_cleared));
                if (e != hipSuccess) return e;
            }
            unsigned int* counter = counters[dev];
            const unsigned int target = reached[dev][slot] + (unsigned)n_clear;
            absmax_stream_kernel<true><<<dim3((unsigned)(n_work + n_clear)), block, 0, stream>>>(
                X, T, I, ldx, tb, cb, ncc, nb, ncc * nrc, matrix_stride, n_clear, B * T, B * I, counter + slot, target,
                1u << 22);
            e = hipGetLastError();
            if (e == hipSuccess) reached[dev][slot] = target;
            return e;
        }
        zero_fill_kernel<<<dim3((n_words + 255) / 256), dim3(256), 0, stream>>>(tb, B * T, cb, B * I);
        absmax_stream_kernel<false><<<dim3((unsigned)n_work), block, 0, stream>>>(X, T, I, ldx, tb, cb, ncc, nb, ncc * nrc,
                                                                                  matrix_stride, 0, 0, 0, nullptr, 0u, 0u);
        return hipGetLastError();
    }
    zero_fill_kernel<<<dim3((n_words + 255) / 256), dim3(256), 0, stream>>>(tb, B * T, cb, B * I);
    const dim3 grid((unsigned)n_work);
    if (vec)
        absmax_kernel<true><<<grid, block, 0, stream>>>(X, T, I, ldx, tb, cb, ncc, nb, ncc * nrc, matrix_stride);
    else
        absmax_kernel<false><<<grid, block, 0, stream>>>(X, T, I, ldx, tb, cb, ncc, nb, ncc * nrc, matrix_stride);
    return hipGetLastError();
}

}  // namespace cq
