// CrossQuant scale factors and the fused quantize / dequantize / kernel-count pass
// (the CrossQuant equation, Definition 1, and the dequantization of the appendix listing).
//
// The element-wise step is D_ij = fl32(a_i * b_j) with a_i = t_i^alpha / q_max and
// b_j = c_j^(1-alpha); the code is q_ij = clamp(rne(fl32(x_ij / D_ij)), +-q_max).
//
// Two kernels: quantize_stream_kernel for the layout every real activation has (aligned, I % 8 == 0), and
// quantize_kernel, its older form with per-lane bounds handling, for everything else.
//
// The kernel moves 2 B read + 1 or 0.5 B codes + optionally 2 B dequantized per element, and on this
// part it is the vector-instruction count per element that decides whether it keeps up with that
// (packed binary32 arithmetic is not used), so the per-element work is kept small.  A correctly
// rounded binary32 division costs more than the rest of the element's work together, so it is taken
// only where it can matter: the quotient is approximated as x * (1/a_i) * (1/b_j) (reciprocals
// formed once per row / per lane, each within 1 ulp), which lies within 2^-21 relative of the
// correctly rounded quotient; the product is rounded straight to an integer by one fma against
// 1.5 * 2^23 (the sum's low mantissa bits are the two's-complement code), a second fma gives its
// distance from that integer, and the integer can differ from the one the exact quotient gives only
// if that distance is within the bound of 1/2.  Lanes test for that with a 3x to 4x margin, and a
// wave in which any lane trips recomputes its eight elements with the exact division (quantize8 in
// cq_device.h).  The result is therefore identical, bit for bit, to dividing every element.
#include "cq_device.h"

namespace cq {
namespace {

__global__ void scale_finalize_kernel(const float* __restrict__ t, const float* __restrict__ c, int T,
                                      int I, float alpha, int qmax, float* __restrict__ a,
                                      float* __restrict__ b, unsigned long long* __restrict__ counters,
                                      int n_counters) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const double al = (double)alpha;
    if (idx < n_counters && counters) counters[idx] = 0ull;
    if (idx < T) a[idx] = row_factor(t[idx], al, qmax);
    else if (idx - T < I) b[idx - T] = col_factor(c[idx - T], al);
}

constexpr int kWaves = 8;   // waves per block
constexpr int kU = 4;       // rows a wave has in flight (8 and 16 measured slower, also for the count-only form)

// Zero-count accumulators of the quantize kernel: library-owned (one array per device, one word
// per stream slot), zero between launches.  Bits 0..40 hold the running count (at most 2^40
// elements), bits 41..63 the number of blocks that have added theirs (a launch of 512-thread blocks
// has fewer than 2^23 of them).  The block whose add
// brings the second field to the grid size knows the total, stores it to the caller's counter
// and clears the accumulator again, so no kernel has to run beforehand to clear anything.
constexpr int kTicketShift = 41;
__device__ unsigned long long g_zero_state[kStateSlots];

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0ull; }

// MODE 0: count only; 1: INT8 codes; 2: packed INT4 codes; 3: INT4 codes as FP6 fragments (one matrix,
// I % 64 == 0).
// Block: 8 waves sharing 512 columns; each wave streams over nb batches of 4 consecutive rows.
// The block first forms the scale factors of its own columns and rows from t and c (binary64
// pow: thread k takes column k, then row k if the block has that many rows; the first batch of X
// rows is requested before, so the memory system is busy meanwhile) and shares them through LDS;
// the blocks of column chunk 0 / row chunk 0 also write them to a_out / b_out for the caller.  Every block that needs a factor
// computes the same bits from the same inputs, so no kernel has to run beforehand.
// Codes and the dequantized matrix are written through to memory (store_through).
// A batch of B matrices (each with its own column factors) is one launch: B copies of the
// one-matrix grid; a block first steps its pointers to its own matrix.
template <int MODE, bool XHAT, bool VEC>
__global__ void __launch_bounds__(kWaves * kLanes)
quantize_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, const float* __restrict__ t_vec,
                const float* __restrict__ c_vec, double alpha, int qmax_i, float* __restrict__ a_out,
                float* __restrict__ b_out, uint8_t* __restrict__ codes, uint16_t* __restrict__ xhat,
                unsigned long long* __restrict__ zero_count, int slot,
                int n_col_chunks, int nb, bool out_vec, int blocks_per_matrix, int64_t matrix_stride) {
    __shared__ uint32_t lds_cnt[kWaves];
    __shared__ float lds_b[kColsPerWave];
    __shared__ float lds_a[kWaves * kLanes];                // row factors of the block's (at most 512) rows
    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    const int matrix = blockIdx.x / blocks_per_matrix;
    const int blk = blockIdx.x - matrix * blocks_per_matrix;
    X += (int64_t)matrix * matrix_stride;
    t_vec += (int64_t)matrix * T;
    c_vec += (int64_t)matrix * I;
    if (a_out) a_out += (int64_t)matrix * T;           // null: the caller does not want the factors (count only)
    if (b_out) b_out += (int64_t)matrix * I;
    if (MODE == 1) codes += (int64_t)matrix * T * I;
    if (MODE == 2) codes += (int64_t)matrix * T * (I / 2);
    if (XHAT) xhat += (int64_t)matrix * T * I;
    const int col_chunk = blk % n_col_chunks;
    const int row_chunk = blk / n_col_chunks;
    const int j0 = col_chunk * kColsPerWave + lane * 8;
    const int rows_per_wave = nb * kU;                      // <= 64
    const int rows_per_block = kWaves * rows_per_wave;      // <= 512 = the block's thread count
    const int row0 = row_chunk * rows_per_block + wave * rows_per_wave;
    const float qmax = (float)qmax_i;

    // A wave walks its batches from the last to the first: the absmax kernel, which normally ran just before,
    // walks them first to last, so the rows it touched last are still in the caches when they are read here
    // first (measured in a step on 4096 x 8192: this kernel 32.4 -> 30.2 us, the same in five processes).
    // (The count-only form walks first to last: it normally follows the quantize call, whose last rows are
    // its first: 20.8 -> 19.3 us on 4096 x 8192.)
    auto batch_at = [&](int bi) { return MODE == 0 ? bi : nb - 1 - bi; };
    auto batch_row = [&](int bi) { return row0 + batch_at(bi) * kU; };
    // first two batches of rows: in flight while the scale factors are formed
    uint4 v[kU], w[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u)
        v[u] = (batch_row(0) + u < T) ? load8<VEC>(X + (int64_t)(batch_row(0) + u) * ldx, j0, I)
                                      : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int u = 0; u < kU; ++u)
        w[u] = (nb > 1 && batch_row(1) + u < T) ? load8<VEC>(X + (int64_t)(batch_row(1) + u) * ldx, j0, I)
                                                : make_uint4(0u, 0u, 0u, 0u);

    block_scale_factors(t_vec, c_vec, alpha, qmax_i, T, I, col_chunk * kColsPerWave, row_chunk * rows_per_block,
                        rows_per_block, lds_a, lds_b, col_chunk == 0 ? a_out : nullptr, row_chunk == 0 ? b_out : nullptr);
    __syncthreads();
    // the wave's row factors, one per lane, handed out with readlane as the rows come up
    const float a_lane = lds_a[wave * rows_per_wave + (lane < rows_per_wave ? lane : 0)];

    float b[8], rb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        b[e] = lds_b[lane * 8 + e];                         // 0 for columns past the end
        rb[e] = safe_rcp(b[e]);
    }
    bool b_tiny = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) b_tiny |= tiny_factor(b[e]);
    int nvalid = I - j0;                                    // columns of this lane that exist
    nvalid = nvalid < 0 ? 0 : (nvalid > 8 ? 8 : nvalid);

    uint32_t nonzero = 0u;    // codes != 0 seen by this wave (uniform)
    int rows_done = 0;
    for (int bi = 0; bi < nb; ++bi) {
        const int rbase = batch_row(bi);
        if (bi == 1) {
#pragma unroll
            for (int u = 0; u < kU; ++u) v[u] = w[u];
        } else if (bi > 1) {
#pragma unroll
            for (int u = 0; u < kU; ++u)
                v[u] = (rbase + u < T) ? load8<VEC>(X + (int64_t)(rbase + u) * ldx, j0, I) : make_uint4(0u, 0u, 0u, 0u);
        }
        if (rbase >= T) continue;                           // wave-uniform: a batch past the last row
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int r = rbase + u;
            if (r >= T) break;                              // wave-uniform
            ++rows_done;
            const float a = __builtin_bit_cast(
                float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a_lane), batch_at(bi) * kU + u));
            if (MODE == 0) {
                // a == 0 means D = 0 and every code of the row is 0 by definition: left to the exact path
                nonzero += count_row8_wave(v[u], a, 0.5f * a, 0.5f * a * kTieTol, b, rb, qmax,
                                           b_tiny || tiny_factor(a) || a == 0.0f);
                continue;
            }
            float m[8], q[8];
            quantize8(v[u], a, safe_rcp(a), b, rb, qmax, m, q, b_tiny || tiny_factor(a));
            nonzero += count_nonzero8_wave(m);
            if (MODE == 1) store_codes_i8(m, codes + (int64_t)r * I + j0, out_vec, nvalid);
            if (MODE == 2) store_codes_i4(m, codes + (int64_t)r * (I / 2) + j0 / 2, out_vec, nvalid);
            if (MODE == 3) store_codes_fp6(m, codes, r, col_chunk * kColsPerWave, lane, I / 64, j0 < I);
            if (XHAT) store_xhat(q, a, b, xhat + (int64_t)r * I + j0, out_vec, nvalid);
        }
    }

    if (zero_count) {
        // padded columns hold x = 0 and add nothing to `nonzero`
        int wave_cols = I - col_chunk * kColsPerWave;       // columns of this wave that exist
        wave_cols = wave_cols > kColsPerWave ? kColsPerWave : wave_cols;
        const uint32_t zeros = (uint32_t)(rows_done * wave_cols) - nonzero;
        if (lane == 0) lds_cnt[wave] = zeros;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t s = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += lds_cnt[w];
            // one atomic per block: same-address atomics serialise, so the grid is kept small
            if (slot >= 0) {
                unsigned long long* zero_state = &g_zero_state[slot];
                const unsigned long long add = (1ull << kTicketShift) | (unsigned long long)s;
                const unsigned long long old =
                    __hip_atomic_fetch_add(zero_state, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((unsigned)(old >> kTicketShift) == gridDim.x - 1u) {        // every other block has added
                    *zero_count = (old + add) & ((1ull << kTicketShift) - 1ull);
                    __hip_atomic_store(zero_state, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            } else if (s) {
                atomicAdd(zero_count, (unsigned long long)s);                    // caller's counter, cleared before
            }
        }
    }
}

// The same kernel for the layout every real activation has: X 16-byte aligned with ldx % 8 == 0, I % 8 == 0 and
// aligned outputs, so that a lane's 8 columns exist or not as a whole.  What differs from quantize_kernel:
//   - rows are addressed as raw buffers (base and length in scalar registers, range-checked by the hardware), so
//     the loop body has no per-lane branches and no 64-bit vector address arithmetic;
//   - the stores are buffer stores with the write-through policy the compiler knows about, so its vmcnt waits for
//     the next rows' loads do not also wait for this row's stores to be acknowledged by memory;
//   - the loop is software-pipelined by hand: two register sets of kU rows alternate, the loads of batch bi + 1
//     are requested before batch bi is worked on.  (The loop is kept a loop: unrolled completely for a known
//     number of batches, where the compiler's count of outstanding memory operations becomes exact, it ran 4 us
//     slower on the 4096 x 8192 layer than with the loop's conservative waits.  Two sets is the optimum also for
//     the count-only form, which has registers to spare: 4096 x 8192 in a layer step takes 17.7 us with two sets,
//     18.6 with one, 19.6 with three and 23.3 with four, i.e. with all of X requested at once.)
template <int MODE, bool XHAT>
__global__ void __launch_bounds__(kWaves * kLanes)
quantize_stream_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, const float* __restrict__ t_vec,
                       const float* __restrict__ c_vec, double alpha, int qmax_i, float* __restrict__ a_out,
                       float* __restrict__ b_out, uint8_t* __restrict__ codes, uint16_t* __restrict__ xhat,
                       unsigned long long* __restrict__ zero_count, int slot, int n_col_chunks, int nb,
                       int blocks_per_matrix, int64_t matrix_stride) {
    __shared__ uint32_t lds_cnt[kWaves];
    __shared__ float lds_b[kColsPerWave];
    __shared__ float lds_a[kWaves * kLanes];
    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);     // row indices are scalar values
    const int matrix = blockIdx.x / blocks_per_matrix;
    const int blk = blockIdx.x - matrix * blocks_per_matrix;
    X += (int64_t)matrix * matrix_stride;
    t_vec += (int64_t)matrix * T;
    c_vec += (int64_t)matrix * I;
    if (a_out) a_out += (int64_t)matrix * T;
    if (b_out) b_out += (int64_t)matrix * I;
    if (MODE == 1) codes += (int64_t)matrix * T * I;
    if (MODE == 2) codes += (int64_t)matrix * T * (I / 2);
    if (XHAT) xhat += (int64_t)matrix * T * I;
    const int col_chunk = blk % n_col_chunks;
    const int row_chunk = blk / n_col_chunks;
    const int col0 = col_chunk * kColsPerWave;
    const int cols_here = min(kColsPerWave, I - col0);      // columns of this chunk that exist: a multiple of 8
    const int rows_per_wave = nb * kU;                      // <= 64
    const int rows_per_block = kWaves * rows_per_wave;      // <= 512 = the block's thread count
    const int row0 = row_chunk * rows_per_block + wave * rows_per_wave;
    const float qmax = (float)qmax_i;

    // walk order as in quantize_kernel: last batch first, except for the count-only form
    auto batch_at = [&](int bi) { return MODE == 0 ? bi : nb - 1 - bi; };
    // Rows past the last one are read from the last row instead (and never worked on): a register that is
    // written by nothing but loads lets the compiler count outstanding loads instead of waiting for all of them.
    auto load_batch = [&](uint4 (&dst)[kU], int bi) {
        if (bi >= nb) return;                                // scalar condition
        const int rbase = row0 + batch_at(bi) * kU;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int r = min(rbase + u, T - 1);
            dst[u] = buffer_load16(row_buffer(X + (int64_t)r * ldx + col0, cols_here * 2), lane * 16);
        }
    };
    // The maxima this thread turns into scale factors (column col0 + k, row k of the block) are requested before
    // the rows of X: memory operations return in order, so behind the first batches they would arrive only with
    // the wave's share of the launch's first 32 MiB, and the pow calls would start that much later (4096 x 8192 in
    // a layer step: quantize 30.2 -> 29.5 us, count only 18.2 -> 17.7 us).  The compiler moves plain loads down to
    // their use, behind the row requests, and before it lets the value of an atomic load be used it waits for
    // nearly everything in flight, so the two requests and their wait are written out by hand.  The contract:
    // between the requests and the wait exactly 2 kU = 8 further vector-memory requests are issued (both are
    // assembly statements that the compiler does not move memory operations across), and s_waitcnt vmcnt(8) lets
    // exactly those stay in flight.  The registers of c_in and t_in must not be read before the wait; every parity
    // test of the quantizer would show it (the scale factors would be stale).
    const int k_thread = (int)threadIdx.x;
    float c_in, t_in;
    {
        const float* cp = c_vec + min(col0 + k_thread, I - 1);
        const float* tp = t_vec + min(row_chunk * rows_per_block + k_thread, T - 1);
        asm volatile("global_load_dword %0, %2, off sc1\n\tglobal_load_dword %1, %3, off sc1"
                     : "=&v"(c_in), "=&v"(t_in)
                     : "v"(cp), "v"(tp)
                     : "memory");
    }
    uint4 va[kU], vb[kU];
    load_batch(va, 0);
    if (nb >= 2) load_batch(vb, 1);
    else load_batch(vb, 0);                                 // a wave with one batch requests it twice: always 2 kU requests
    static_assert(kU == 4, "the wait below counts the row requests of two batches");
    asm volatile("s_waitcnt vmcnt(8)" : "+v"(c_in), "+v"(t_in)::"memory");

    {
        // thread k: factor of column col0 + k (0 past the last column) and, if the block has that many rows, of its
        // row k (0 past the last row); the blocks of column chunk 0 / row chunk 0 also write them out for the caller
        const int j = col0 + k_thread;
        float bj = 0.0f;
        if (j < I) {
            bj = col_factor(c_in, alpha);
            if (row_chunk == 0 && b_out) b_out[j] = bj;
        }
        lds_b[k_thread] = bj;
        const int r = row_chunk * rows_per_block + k_thread;
        float ar = 0.0f;
        if (k_thread < rows_per_block && r < T) {
            ar = row_factor(t_in, alpha, qmax_i);
            if (col_chunk == 0 && a_out) a_out[r] = ar;
        }
        lds_a[k_thread] = ar;
    }
    __syncthreads();
    // the wave's row factors and their reciprocals, one row per lane, handed out with readlane as the rows come up
    const float a_lane = lds_a[wave * rows_per_wave + (lane < rows_per_wave ? lane : 0)];
    const float ra_lane = safe_rcp(a_lane);

    float b[8], rb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        b[e] = lds_b[lane * 8 + e];                         // 0 for columns past the end
        rb[e] = safe_rcp(b[e]);
    }
    bool b_tiny = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) b_tiny |= tiny_factor(b[e]);

    uint32_t nonzero_lane = 0u;   // codes != 0 seen by this lane
    int rows_done = 0;
    // No branch depends on whether a row exists: rows past the last one are worked on like the others (their data
    // is the last row's, their factor is 0), but their stores go to an empty buffer, which drops them, and their
    // counts are not added.  The only branch left is the rare exact-division path inside quantize8.
    auto work = [&](const uint4 (&v)[kU], int bi) {
        const int rbase = row0 + batch_at(bi) * kU;
        Fp6Batch f6;                                        // MODE 3: the batch's four rows leave together
        if (MODE == 3) {
#pragma unroll
            for (int k = 0; k < 4; ++k) f6.lo[k] = f6.hi[k] = 0u;
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int r = rbase + u;
            const bool row_ok = r < T;                      // scalar
            const int rr = row_ok ? r : 0;
            rows_done += row_ok ? 1 : 0;
            const int ri = batch_at(bi) * kU + u;
            const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a_lane), ri));
            const float ra = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, ra_lane), ri));
            if (MODE == 0) {
                // a == 0 means D = 0 and every code of the row is 0 by definition: left to the exact path
                const uint32_t nz = count_row8_lane(v[u], a, 0.5f * a, 0.5f * a * kTieTol, b, rb, qmax,
                                                    b_tiny || tiny_factor(a) || a == 0.0f);
                nonzero_lane += row_ok ? nz : 0u;
                continue;
            }
            const int live = row_ok ? cols_here : 0;         // columns of this row that may be stored
            // count, pack and store one row piece; returns the lane's number of non-zero codes in it
            auto emit = [&](const float (&m)[8], const float (&q)[8]) -> uint32_t {
                const uint32_t nz = count_nonzero8_lane(m);
                if (MODE == 1)
                    __builtin_amdgcn_raw_buffer_store_b64(pack_codes_i8(m), row_buffer(codes + (int64_t)rr * I + col0, live),
                                                          lane * 8, 0, kWriteThrough);
                if (MODE == 2)
                    __builtin_amdgcn_raw_buffer_store_b32(pack_codes_i4(m),
                                                          row_buffer(codes + (int64_t)rr * (I / 2) + col0 / 2, live / 2),
                                                          lane * 4, 0, kWriteThrough);
                if (MODE == 3) fp6_batch_row(f6, m, u);
                if (XHAT)
                    __builtin_amdgcn_raw_buffer_store_b128(pack_xhat(q, a, b), row_buffer(xhat + (int64_t)rr * I + col0, live * 2),
                                                           lane * 16, 0, kWriteThrough);
                return nz;
            };
            // The exact path packs and stores for itself instead of handing m and q back: values that come out of
            // either path would need register copies where the paths join, and the compiler puts those copies
            // (3 per element) on the common path.
            float m[8], q[8];
            uint32_t nz;
            if (__builtin_expect(quantize8_fast(v[u], ra, rb, qmax, m, q, b_tiny || tiny_factor(a)), 0)) {
                float mx[8], qx[8];
                quantize8_exact(v[u], a, b, qmax, mx, qx);
                nz = emit(mx, qx);
            } else {
                nz = emit(m, q);
            }
            nonzero_lane += row_ok ? nz : 0u;
            __builtin_amdgcn_sched_barrier(0);               // rows one after the other: keeps scalar register pressure down
        }
        if (MODE == 3) {
            static_assert(kU == 4, "a batch is the four rows a quad of lanes shares out");
            const int left = T - rbase;                      // rows of the batch that exist
            const uint32_t rows_ok = left >= 4 ? 0xFu : (left > 0 ? (1u << left) - 1u : 0u);
            fp6_batch_store(f6, codes, rbase, col0, lane, I / 64, rows_ok, lane * 8 < cols_here);
        }
    };
    for (int bi = 0; bi < nb; bi += 2) {
        work(va, bi);
        load_batch(va, bi + 2);
        if (bi + 1 < nb) {
            work(vb, bi + 1);
            load_batch(vb, bi + 3);
        }
    }

    if (zero_count) {
        uint32_t nonzero = nonzero_lane;                    // ... and by the wave
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) nonzero += shx(nonzero, off);
        // columns past the end read as x = 0 and add nothing to `nonzero`
        const uint32_t zeros = (uint32_t)(rows_done * cols_here) - nonzero;
        if (lane == 0) lds_cnt[wave] = zeros;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t s = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += lds_cnt[w];
            // one atomic per block: same-address atomics serialise, so the grid is kept small
            if (slot >= 0) {
                unsigned long long* zero_state = &g_zero_state[slot];
                const unsigned long long add = (1ull << kTicketShift) | (unsigned long long)s;
                const unsigned long long old =
                    __hip_atomic_fetch_add(zero_state, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((unsigned)(old >> kTicketShift) == gridDim.x - 1u) {        // every other block has added
                    *zero_count = (old + add) & ((1ull << kTicketShift) - 1ull);
                    __hip_atomic_store(zero_state, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            } else if (s) {
                atomicAdd(zero_count, (unsigned long long)s);                    // caller's counter, cleared before
            }
        }
    }
}

template <int MODE, bool XHAT>
hipError_t launch_mode(const uint16_t* X, int B, int T, int I, int64_t ldx, int64_t matrix_stride, const float* t,
                       const float* c, double alpha, int qmax, float* a, float* b, uint8_t* codes, uint16_t* xhat,
                       unsigned long long* zc, hipStream_t stream) {
    const int ncc = (I + kColsPerWave - 1) / kColsPerWave;
    const int nb = quantize_batches_per_wave((int64_t)B * ncc, T);        // rows per block = 32 * nb
    const int nrc = (T + 32 * nb - 1) / (32 * nb);
    if (!grid_fits((int64_t)B * ncc * nrc, kWaves * kLanes)) return hipErrorInvalidValue;    // hence < 2^23 blocks
    const unsigned n_blocks = (unsigned)(B * ncc * nrc);
    const dim3 grid(n_blocks), block(kWaves * kLanes);
    const bool vec = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 8 == 0) && (B == 1 || matrix_stride % 8 == 0);
    // vector stores need every lane's piece aligned: I % 8 == 0 and aligned bases
    const bool out_vec = (I % 8 == 0) && (reinterpret_cast<uintptr_t>(codes) % 8 == 0) &&
                         (reinterpret_cast<uintptr_t>(xhat) % 16 == 0);
    // no slot: clear the caller's counter and add to it directly
    const int state = zc ? stream_slot(stream) : -1;
    if (zc && state < 0) zero_u64_kernel<<<dim3(1), dim3(1), 0, stream>>>(zc);
    // the layout every real activation has: the streaming kernel (no partial pieces, no misaligned pointers)
    const bool stream_ok = vec && (I % 8 == 0) && (reinterpret_cast<uintptr_t>(codes) % 8 == 0) &&
                           (reinterpret_cast<uintptr_t>(xhat) % 16 == 0);
    if (stream_ok)
        quantize_stream_kernel<MODE, XHAT><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, alpha, qmax, a, b, codes, xhat,
                                                                      zc, state, ncc, nb, ncc * nrc, matrix_stride);
    else if (vec)
        quantize_kernel<MODE, XHAT, true><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, alpha, qmax, a, b, codes, xhat,
                                                                     zc, state, ncc, nb, out_vec, ncc * nrc,
                                                                     matrix_stride);
    else
        quantize_kernel<MODE, XHAT, false><<<grid, block, 0, stream>>>(X, T, I, ldx, t, c, alpha, qmax, a, b, codes,
                                                                      xhat, zc, state, ncc, nb, out_vec, ncc * nrc,
                                                                      matrix_stride);
    return hipGetLastError();
}

// Packed two's-complement nibbles -> int8 codes (even column in the low nibble), so that INT4
// activations can feed the INT8 MFMA GEMM (gfx950 has no INT4 matrix instruction).
// One thread expands 8 packed bytes to 16 codes.
__global__ void unpack_int4_kernel(const uint8_t* __restrict__ packed, int64_t n_bytes, int8_t* __restrict__ codes,
                                   bool vec) {
    const int64_t i8 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
    if (i8 >= n_bytes) return;
    uint32_t lo = 0u, hi = 0u;
    const bool full = vec && i8 + 8 <= n_bytes;
    if (full) {
        const uint2 v = *reinterpret_cast<const uint2*>(packed + i8);
        lo = v.x;
        hi = v.y;
    } else {
        for (int e = 0; e < 8 && i8 + e < n_bytes; ++e) {
            const uint32_t b = packed[i8 + e];
            if (e < 4) lo |= b << (8 * e); else hi |= b << (8 * (e - 4));
        }
    }
    uint32_t out[4];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const uint32_t src = w ? hi : lo;
#pragma unroll
        for (int h = 0; h < 2; ++h) {                // two output words per input word
            uint32_t o = 0u;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint32_t byte = (src >> (16 * h + 8 * e)) & 0xFFu;
                const int n0 = (int)(byte & 0xFu), n1 = (int)(byte >> 4);
                const int c0 = (n0 ^ 8) - 8, c1 = (n1 ^ 8) - 8;      // sign-extend 4 bits
                o |= ((uint32_t)(c0 & 0xFF) << (16 * e)) | ((uint32_t)(c1 & 0xFF) << (16 * e + 8));
            }
            out[2 * w + h] = o;
        }
    }
    int8_t* dst = codes + 2 * i8;
    if (full) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
    } else {
        for (int e = 0; e < 16 && i8 + e / 2 < n_bytes; ++e) dst[e] = (int8_t)((out[e >> 2] >> (8 * (e & 3))) & 0xFFu);
    }
}

}  // namespace

hipError_t launch_unpack_int4(const uint8_t* packed, int64_t n_bytes, int8_t* codes, hipStream_t stream) {
    const bool vec = (reinterpret_cast<uintptr_t>(packed) % 8 == 0) && (reinterpret_cast<uintptr_t>(codes) % 16 == 0);
    const int64_t n_threads = (n_bytes + 7) / 8;
    if (!grid_fits((n_threads + 255) / 256, 256)) return hipErrorInvalidValue;
    unpack_int4_kernel<<<dim3((unsigned)((n_threads + 255) / 256)), dim3(256), 0, stream>>>(packed, n_bytes, codes, vec);
    return hipGetLastError();
}

hipError_t launch_scale_finalize(const float* t, const float* c, int T, int I, float alpha, int qmax,
                                 float* a, float* b, unsigned long long* counters, int n_counters,
                                 hipStream_t stream) {
    const int n = T + I;
    scale_finalize_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(t, c, T, I, alpha, qmax, a, b,
                                                                           counters, n_counters);
    return hipGetLastError();
}

hipError_t launch_quantize(const uint16_t* X, int B, int T, int I, int64_t ldx, int64_t matrix_stride, const float* t,
                           const float* c, float alpha, int bits, float* a, float* b, void* codes, uint16_t* xhat,
                           unsigned long long* zero_count, hipStream_t stream) {
    const int qmax = (1 << (bits - 1)) - 1;
    const double al = (double)alpha;
    uint8_t* cp = static_cast<uint8_t*>(codes);
    if (!cp)
        return launch_mode<0, false>(X, B, T, I, ldx, matrix_stride, t, c, al, qmax, a, b, nullptr, nullptr, zero_count,
                                     stream);
    if (bits == 8)
        return xhat ? launch_mode<1, true>(X, B, T, I, ldx, matrix_stride, t, c, al, qmax, a, b, cp, xhat, zero_count, stream)
                    : launch_mode<1, false>(X, B, T, I, ldx, matrix_stride, t, c, al, qmax, a, b, cp, nullptr, zero_count,
                                            stream);
    return xhat ? launch_mode<2, true>(X, B, T, I, ldx, matrix_stride, t, c, al, qmax, a, b, cp, xhat, zero_count, stream)
                : launch_mode<2, false>(X, B, T, I, ldx, matrix_stride, t, c, al, qmax, a, b, cp, nullptr, zero_count,
                                        stream);
}

// INT4 codes written straight into the FP6 operand format (I % 64 == 0, packed 16-byte aligned)
hipError_t launch_quantize_fp6(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c, float alpha,
                               float* a, float* b, void* packed, uint16_t* xhat, unsigned long long* zero_count,
                               hipStream_t stream) {
    uint8_t* cp = static_cast<uint8_t*>(packed);
    const double al = (double)alpha;
    return xhat ? launch_mode<3, true>(X, 1, T, I, ldx, 0, t, c, al, 7, a, b, cp, xhat, zero_count, stream)
                : launch_mode<3, false>(X, 1, T, I, ldx, 0, t, c, al, 7, a, b, cp, nullptr, zero_count, stream);
}


// crossquant_absmax_quantize: the two kernels one after the other on the stream.  Two one-launch forms were built
// and measured on the 4096 x 8192 layer, and both lost to this: keeping the tile in registers and LDS across a grid
// barrier (X read once: 79 us in a step against 56 us), and re-reading the tile from the caches after a grid barrier
// (70 us against 39 us back to back; 41 us with the barrier's waits compiled out, i.e. no gain even from a free
// barrier).  A barrier through memory costs two to three round trips to the device's coherence point plus the
// slowest block's lag; the boundary between two kernels costs about 3 us.
hipError_t launch_absmax_quantize(const uint16_t* X, int T, int I, int64_t ldx, float alpha, int bits, float* t,
                                  float* c, float* a, float* b, void* codes, uint16_t* xhat,
                                  unsigned long long* zero_count, hipStream_t stream) {
    // both grids are checked before the first kernel is enqueued
    const int ncc = (I + kColsPerWave - 1) / kColsPerWave;
    const int nb = quantize_batches_per_wave(ncc, T);
    if (!grid_fits((int64_t)ncc * ((T + 32 * nb - 1) / (32 * nb)), kWaves * kLanes)) return hipErrorInvalidValue;
    const hipError_t e = launch_absmax(X, 1, T, I, ldx, 0, t, c, stream);
    if (e != hipSuccess) return e;
    return launch_quantize(X, 1, T, I, ldx, 0, t, c, alpha, bits, a, b, codes, xhat, zero_count, stream);
}

}  // namespace cq
