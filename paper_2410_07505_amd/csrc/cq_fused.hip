// Single-read CrossQuant: row/column maxima, scale factors and quantize / dequantize / count in
// ONE kernel that reads X from HBM once and keeps it in registers across a grid-wide barrier.
//
// The two-call path reads X twice (maxima, then quantize) because every element's step depends
// on the maxima of its whole row and column.  An MI355X has 256 CUs x 512 KiB of vector
// registers, so a 64 MiB activation matrix (4096 x 8192 binary16) fits on chip: each of the
// 256 blocks (one per CU, 512 threads) owns a 256-row x 512-column tile, 512 bytes of it per
// thread (32 rows x 16 bytes).  Phase 1 loads the tile and accumulates the maxima with the same
// dense atomics as the absmax kernel; a grid-wide barrier makes t and c complete;
// phase 2 has every block compute the 256 + 512 scale factors it needs (binary64 pow, the same
// device routine as the two-call path, so the factors are bit-identical); phase 3 quantizes out
// of the registers.  HBM traffic drops from 7 to 5 bytes per element (with the dequantized
// output; 5 to 3 without).
//
// Measured on 4096 x 8192: the call is slower than the absmax and quantize kernels it replaces (about 47 us
// against 40 us back to back, more inside a layer step): the barrier splits the kernel into a phase that only
// reads and a phase that only writes, so the memory system never sees both directions at once, and the barrier
// itself costs more than the boundary between two kernels.  It is kept as an entry point of its own for the
// traffic figure and for callers whose input is cheaper to read once; crossquant_absmax_quantize does not use it.
//
// The grid barrier is a counter in device memory that every block increments once and then polls
// (a cooperative launch plus the runtime's grid sync costs ~35 us per call on this stack, more
// than either phase; this barrier costs a few).  It needs every block resident at the same time:
// a block fills a CU (128 KiB of LDS, ~250 registers x 512 threads), so the host side refuses
// grids with more blocks than the device has CUs (CQ_ERR_UNSUPPORTED: the caller uses
// crossquant_absmax_quantize).  Blocks of other kernels still running on the device only delay the barrier.
// The wait is bounded: a block that does not see the barrier open within the poll limit (seconds;
// only possible if part of the device is unavailable to this process) stops waiting, skips the
// quantize phase and writes NaN scale factors for its tile, so the kernel always terminates.

#include "cq_device.h"


namespace cq {
namespace {

// 8 waves per block = 2 per SIMD, so every thread may use 256 registers.  A thread's 32 rows x
// 16 bytes of the tile would take 128 of them; together with the quantize phase's temporaries the
// compiler then spills part of the tile to scratch, i.e. to HBM.  So kFLdsRows of a thread's rows
// wait in LDS instead (16 bytes x 512 threads per row: every lane reads back its own slot, no
// bank conflicts) and only kFRegRows stay in registers.
constexpr int kFWaves = 8;           // waves per block
constexpr int kFRows = 32;           // rows per wave
constexpr int kFRegRows = 16;                         // ... of which held in registers (24: spills)
constexpr int kFLdsRows = kFRows - kFRegRows;         // ... and in LDS
constexpr int kFBlockRows = kFWaves * kFRows;   // 256
constexpr int kFThreads = kFWaves * kLanes;
constexpr int kFLdsBytes = kFLdsRows * kFThreads * 16;
constexpr unsigned kFSpinLimit = 1u << 22;        // default poll limit; a poll takes a microsecond or two

// Grid barrier state: blocks that have arrived at the barrier and blocks that have left it.  One pair per
// stream slot (calls on different streams may overlap; calls on one stream are ordered), zero between
// launches: every block arrives once and leaves once, and the block that leaves last clears the pair.
struct FusedBarrier {
    unsigned int arrivals, departures;
};
__device__ FusedBarrier g_fused_barrier[kStateSlots];

__global__ void fused_zero_kernel(uint32_t* __restrict__ t, int T, uint32_t* __restrict__ c, int I,
                                  unsigned long long* __restrict__ zc) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && zc) *zc = 0ull;
    if (i < T) t[i] = 0u;
    else if (i - T < I) c[i - T] = 0u;
}

// MODE 1: INT8 codes; 2: packed INT4 codes.  Requires I % 8 == 0 and 16-byte aligned rows.
template <int MODE, bool XHAT>
__global__ void __launch_bounds__(kFThreads)
fused_kernel(const uint16_t* __restrict__ X, int T, int I, int64_t ldx, float alpha, int qmax_i,
             uint32_t* t_bits, uint32_t* c_bits, float* __restrict__ a_out, float* __restrict__ b_out,
             uint8_t* __restrict__ codes, uint16_t* __restrict__ xhat, unsigned long long* __restrict__ zero_count,
             int n_col_chunks, unsigned spin_limit, int slot) {
    __shared__ uint32_t lds_col[kFWaves][4][kLanes];
    __shared__ float lds_a[kFBlockRows];
    __shared__ __align__(16) float lds_b[kColsPerWave];
    __shared__ uint32_t lds_cnt[kFWaves];

    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes;
    const int col_chunk = blockIdx.x % n_col_chunks;
    const int row_chunk = blockIdx.x / n_col_chunks;
    const int j0 = col_chunk * kColsPerWave + lane * 8;
    const int row0 = row_chunk * kFBlockRows + wave * kFRows;
    const bool col_ok = j0 < I;                       // I % 8 == 0: a lane's 8 columns exist or not together

    // ---- phase 1: load the tile, maxima.  Rows [0, kFRegRows) of the wave stay in v[], rows
    // [kFRegRows, 32) go to LDS.  Out-of-range rows/columns are read from a clamped (valid)
    // address and zeroed, so the loads carry no branches.
    extern __shared__ __align__(16) uint4 lds_tile[];   // [kFLdsRows][kFThreads]
    uint4 v[kFRegRows];
    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
    const int jc = col_ok ? j0 : 0;
    auto load_row = [&](int k) -> uint4 {
        const int r = min(row0 + k, T - 1);
        uint4 w = *reinterpret_cast<const uint4*>(X + (int64_t)r * ldx + jc);
        if (!(col_ok && row0 + k < T)) w = make_uint4(0u, 0u, 0u, 0u);
        return w;
    };
    // the register rows' loads go out first and stay in flight while the LDS rows pass through
#pragma unroll
    for (int k = 0; k < kFRegRows; ++k) v[k] = load_row(k);
#pragma unroll
    for (int g = 0; g < kFLdsRows / 8; ++g) {
        uint4 w[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = load_row(kFRegRows + 8 * g + k);
        uint32_t rm[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            rm[k] = absmax8(w[k], c0, c1, c2, c3);
            lds_tile[(8 * g + k) * kFThreads + threadIdx.x] = w[k];
        }
        const uint32_t m = rows8_reduce(rm, lane);
        const int r = row0 + kFRegRows + 8 * g + (lane >> 3);
        if ((lane & 7) == 0 && r < T && m) atomicMax(&t_bits[r], half_bits_to_float_bits(m));
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int g = 0; g < kFRegRows / 8; ++g) {
        uint32_t rm[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) rm[k] = absmax8(v[8 * g + k], c0, c1, c2, c3);
        const uint32_t m = rows8_reduce(rm, lane);
        const int r = row0 + 8 * g + (lane >> 3);
        if ((lane & 7) == 0 && r < T && m) atomicMax(&t_bits[r], half_bits_to_float_bits(m));
        __builtin_amdgcn_sched_barrier(0);             // keep the groups apart: short live ranges
    }
    lds_col[wave][0][lane] = c0;
    lds_col[wave][1][lane] = c1;
    lds_col[wave][2][lane] = c2;
    lds_col[wave][3][lane] = c3;
    __syncthreads();
    if (threadIdx.x < 256) {                          // 256 threads x 2 columns = the chunk's 512 columns
        const int idx = threadIdx.x;
        const int reg = idx & 3, ln = idx >> 2;
        uint32_t m = lds_col[0][reg][ln];
#pragma unroll
        for (int w = 1; w < kFWaves; ++w) m = pkmax(m, lds_col[w][reg][ln]);
        const int j = col_chunk * kColsPerWave + idx * 2;
        if (j < I && (m & 0xFFFFu)) atomicMax(&c_bits[j], half_bits_to_float_bits(m & 0xFFFFu));
        if (j + 1 < I && (m >> 16)) atomicMax(&c_bits[j + 1], half_bits_to_float_bits(m >> 16));
    }

    // ---- grid barrier: t and c are final once every block has arrived.  The only data that
    // crosses blocks travels in device-scope atomics (performed at the device's coherence point,
    // and read back below with device-scope atomic loads), so no cache write-back or invalidate
    // is needed: each thread just waits until its own atomics have been acknowledged (vmcnt
    // counts them down as the acknowledgements return), then the block arrives.
    __shared__ int lds_open;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        FusedBarrier* bar = &g_fused_barrier[slot];
        __hip_atomic_fetch_add(&bar->arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int open = 0;
        for (unsigned spin = 0; spin < spin_limit; ++spin) {
            if (__hip_atomic_load(&bar->arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= gridDim.x) {
                open = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        lds_open = open;
        // leave (also after giving up): whoever leaves last has seen every block arrive, and nobody polls any more
        const unsigned left = __hip_atomic_fetch_add(&bar->departures, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left == gridDim.x - 1u) {
            __hip_atomic_store(&bar->arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&bar->departures, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    const bool barrier_open = lds_open != 0;          // block-uniform

    // ---- phase 2: the scale factors this block needs (read at device scope: the values were
    // produced by other CUs' atomics)
    const double al = (double)alpha;
    for (int idx = threadIdx.x; idx < kFBlockRows + kColsPerWave; idx += kFThreads) {
        if (idx < kFBlockRows) {
            const int r = row_chunk * kFBlockRows + idx;
            float a = 0.0f;
            if (r < T) {
                const float tv = __uint_as_float(__hip_atomic_load(&t_bits[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                a = barrier_open ? row_factor(tv, al, qmax_i) : __builtin_nanf("");
                if (col_chunk == 0 || !barrier_open) a_out[r] = a;
            }
            lds_a[idx] = a;
        } else {
            const int jl = idx - kFBlockRows;
            const int j = col_chunk * kColsPerWave + jl;
            float b = 0.0f;
            if (j < I) {
                const float cv = __uint_as_float(__hip_atomic_load(&c_bits[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                b = barrier_open ? col_factor(cv, al) : __builtin_nanf("");
                if (row_chunk == 0 || !barrier_open) b_out[j] = b;
            }
            lds_b[jl] = b;
        }
    }
    __syncthreads();
    if (!barrier_open) return;                        // block-uniform: maxima incomplete, nothing to quantize

    // ---- phase 3: quantize out of the registers
    const float qmax = (float)qmax_i;
    float b[8], rb[8];
    {
        const float4 b0 = *reinterpret_cast<const float4*>(&lds_b[lane * 8]);
        const float4 b1 = *reinterpret_cast<const float4*>(&lds_b[lane * 8 + 4]);
        b[0] = b0.x; b[1] = b0.y; b[2] = b0.z; b[3] = b0.w;
        b[4] = b1.x; b[5] = b1.y; b[6] = b1.z; b[7] = b1.w;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) rb[e] = safe_rcp(b[e]);
    // (the maxima are the data's own here, so no factor can be tiny: see quantize8)
    // the wave's 32 row factors, one per lane, handed out with readlane (scalar registers)
    const float a_lane = lds_a[wave * kFRows + (lane & (kFRows - 1))];
    float nonzero = 0.0f;
    int rows_done = 0;
    // output pointers advance row by row (computing all 32 rows' addresses up front would take
    // more registers than the tile leaves free)
    uint8_t* cp = codes + (MODE == 1 ? (int64_t)row0 * I + j0 : (int64_t)row0 * (I / 2) + j0 / 2);
    uint16_t* hp = xhat + (int64_t)row0 * I + j0;
    const int c_step = (MODE == 1) ? I : I / 2;
#pragma unroll
    for (int k = 0; k < kFRows; ++k) {
        if (row0 + k < T) {                            // wave-uniform
            ++rows_done;
            const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a_lane), k));
            float m[8], q[8];
            const uint4 xv = (k < kFRegRows) ? v[k < kFRegRows ? k : 0] : lds_tile[(k - kFRegRows) * kFThreads + threadIdx.x];
            quantize8(xv, a, safe_rcp(a), b, rb, qmax, m, q, false);
            nonzero += count_nonzero8(m);
            if (col_ok) {
                if (MODE == 1) store_codes_i8(m, cp, true, 8);
                if (MODE == 2) store_codes_i4(m, cp, true, 8);
                if (XHAT) store_xhat(q, a, b, hp, true, 8);
            }
        }
        cp += c_step;
        if (XHAT) hp += I;
        __builtin_amdgcn_sched_barrier(0);             // one row at a time: the tile fills half the registers
    }
    if (zero_count) {
        uint32_t zeros = (col_ok ? (uint32_t)(rows_done * 8) : 0u) - (uint32_t)nonzero;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) zeros += (uint32_t)__shfl_xor((int)zeros, off, kLanes);
        if (lane == 0) lds_cnt[wave] = zeros;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t s = 0;
#pragma unroll
            for (int w = 0; w < kFWaves; ++w) s += lds_cnt[w];
            if (s) atomicAdd(zero_count, (unsigned long long)s);
        }
    }
}

// Host-side poll limit handed to every launch (see set_fused_barrier_polls).
unsigned g_spin_limit = kFSpinLimit;

template <int MODE, bool XHAT>
hipError_t launch_fused_mode(const uint16_t* X, int T, int I, int64_t ldx, float alpha, int qmax, float* t, float* c,
                             float* a, float* b, uint8_t* codes, uint16_t* xhat, unsigned long long* zc, int ncc,
                             int nblocks, int slot, hipStream_t stream) {
    // everything that can fail is checked before the first kernel of the call is enqueued
    static std::atomic<uint64_t> lds_allowed{0};
    const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&fused_kernel<MODE, XHAT>), kFLdsBytes, lds_allowed);
    if (e != hipSuccess) return e;
    {
        const int n = T + I;
        fused_zero_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(reinterpret_cast<uint32_t*>(t), T,
                                                                           reinterpret_cast<uint32_t*>(c), I, zc);
    }
    fused_kernel<MODE, XHAT><<<dim3((unsigned)nblocks), dim3(kFThreads), kFLdsBytes, stream>>>(
        X, T, I, ldx, alpha, qmax, reinterpret_cast<uint32_t*>(t), reinterpret_cast<uint32_t*>(c), a, b, codes, xhat, zc,
        ncc, g_spin_limit, slot);
    return hipGetLastError();
}

}  // namespace

// Test hook: polls a block makes at the grid barrier before it gives up.  0 makes every block give
// up at once, which exercises the failure path without ever making a GPU wait.
void set_fused_barrier_polls(unsigned polls) { g_spin_limit = polls; }

// returns hipErrorNotSupported (without launching) when the matrix does not fit on chip
hipError_t launch_absmax_quantize_single_read(const uint16_t* X, int T, int I, int64_t ldx, float alpha, int bits, float* t,
                                  float* c, float* a, float* b, void* codes, uint16_t* xhat,
                                  unsigned long long* zero_count, hipStream_t stream) {
    const int ncc = (I + kColsPerWave - 1) / kColsPerWave;
    const int nrc = (T + kFBlockRows - 1) / kFBlockRows;
    const int64_t nblocks = (int64_t)ncc * nrc;
    int dev = 0, n_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    // a block fills a CU, and the grid barrier needs all blocks resident together: one block per CU
    if (nblocks > n_cu) return hipErrorNotSupported;
    // the barrier's counters belong to a stream slot: a stream without one takes the two calls
    const int slot = stream_slot(stream);
    if (slot < 0) return hipErrorNotSupported;
    const int qmax = (1 << (bits - 1)) - 1;
    uint8_t* cp = static_cast<uint8_t*>(codes);
    if (bits == 8)
        return xhat ? launch_fused_mode<1, true>(X, T, I, ldx, alpha, qmax, t, c, a, b, cp, xhat, zero_count, ncc,
                                                 (int)nblocks, slot, stream)
                    : launch_fused_mode<1, false>(X, T, I, ldx, alpha, qmax, t, c, a, b, cp, nullptr, zero_count, ncc,
                                                  (int)nblocks, slot, stream);
    return xhat ? launch_fused_mode<2, true>(X, T, I, ldx, alpha, qmax, t, c, a, b, cp, xhat, zero_count, ncc,
                                             (int)nblocks, slot, stream)
                : launch_fused_mode<2, false>(X, T, I, ldx, alpha, qmax, t, c, a, b, cp, nullptr, zero_count, ncc,
                                              (int)nblocks, slot, stream);
}

}  // namespace cq
