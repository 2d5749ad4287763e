// Calibration kernels for the rooflines: what this device reaches on a plain streaming read, a
// plain copy and a loop of nothing but INT8 matrix instructions.  They are not part of the method;
// the benchmark times them next to the real kernels so that every rate can be read against both
// the published peak and the rate the part actually sustains.
#include "cq_kernels.h"

namespace cq {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kCalibThreads = 256;

// 16 bytes per lane per load, four loads in flight, grid-stride.  The xor of everything read
// is kept so the loads cannot be dropped; it is stored only if it equals a value it cannot have
// been steered to.
__global__ void __launch_bounds__(kCalibThreads)
calib_read_kernel(const u32x4* __restrict__ src, int64_t n16, unsigned long long* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * kCalibThreads;
    int64_t i = (int64_t)blockIdx.x * kCalibThreads + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        acc ^= v0 ^ v1 ^ v2 ^ v3;
    }
    for (; i < n16; i += stride) acc ^= src[i];
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u && sink) atomicAdd(sink, 1ull);
}

__global__ void __launch_bounds__(kCalibThreads)
calib_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * kCalibThreads;
    int64_t i = (int64_t)blockIdx.x * kCalibThreads + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        dst[i] = v0;
        dst[i + stride] = v1;
        dst[i + 2 * stride] = v2;
        dst[i + 3 * stride] = v3;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

__device__ __forceinline__ uint32_t calib_hash(uint32_t s) {
    s ^= s >> 13; s *= 0x5bd1e995u; s ^= s >> 15; s *= 2654435761u; s ^= s >> 16;
    return s;
}

// One wave per SIMD, 16 independent 32x32 accumulators, operands fixed in registers: the matrix
// pipe never waits for data.  data_mode 0: all-zero operands; 1: bell-shaped int8 codes (sum of
// four 6-bit uniforms, |q| up to ~42), about what quantized activations and weights look like.
// The sustained rate depends on the operands' switching activity, so both are reported.
__global__ void __launch_bounds__(256)
calib_mfma_kernel(int iters, int data_mode, int* __restrict__ sink) {
    v4i a[4], b[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t wa = 0, wb = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t ra = calib_hash(threadIdx.x * 977u + k * 131u + e * 17u + c + blockIdx.x * 7919u);
                const uint32_t rb = calib_hash(threadIdx.x * 613u + k * 37u + e * 11u + c + 99991u + blockIdx.x * 104729u);
                const int qa = (int)((ra & 63) + ((ra >> 6) & 63) + ((ra >> 12) & 63) + ((ra >> 18) & 63)) - 126;
                const int qb = (int)((rb & 63) + ((rb >> 6) & 63) + ((rb >> 12) & 63) + ((rb >> 18) & 63)) - 126;
                wa |= (uint32_t)(uint8_t)(int8_t)(data_mode ? qa / 3 : 0) << (8 * c);
                wb |= (uint32_t)(uint8_t)(int8_t)(data_mode ? qb / 3 : 0) << (8 * c);
            }
            a[k][e] = (int)wa;
            b[k][e] = (int)wb;
        }
    v16i acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 0x7fffffff && sink) sink[0] = s;
}

// The same loop on the 16 x 16 x 64 instruction, the one the linear kernel uses (half the accumulator registers read
// and written per multiply-add): 32 independent 16 x 16 accumulators, operands fixed in registers, code-like data.
// Two waves per SIMD: one wave alone cannot keep the pipe full with an instruction this short.
__global__ void __launch_bounds__(512)
calib_mfma16_kernel(int iters, int* __restrict__ sink) {
    v4i a[8], b[4];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t wa = 0, wb = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t ra = calib_hash(threadIdx.x * 977u + k * 131u + e * 17u + c + blockIdx.x * 7919u);
                const uint32_t rb = calib_hash(threadIdx.x * 613u + k * 37u + e * 11u + c + 99991u + blockIdx.x * 104729u);
                const int qa = (int)((ra & 63) + ((ra >> 6) & 63) + ((ra >> 12) & 63) + ((ra >> 18) & 63)) - 126;
                const int qb = (int)((rb & 63) + ((rb >> 6) & 63) + ((rb >> 12) & 63) + ((rb >> 18) & 63)) - 126;
                wa |= (uint32_t)(uint8_t)(int8_t)(qa / 3) << (8 * c);
                wb |= (uint32_t)(uint8_t)(int8_t)(qb / 3) << (8 * c);
            }
            a[k][e] = (int)wa;
            if (k < 4) b[k][e] = (int)wb;
        }
    v4i acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[i][j][r];
    if (s == 0x7fffffff && sink) sink[0] = s;
}

// Fed the way the linear kernel's inner loop is: 8 waves per CU (two per SIMD), every step reads 8 + 4 operand
// fragments (1 KiB each per wave) from LDS and issues the 32 matrix instructions (16 x 16 x 64) of a 128 x 64 wave
// tile over 64 bytes of the contraction, i.e. 0.75 KiB of LDS reads per 32 x 32 x 32 worth of multiply-adds; no
// global loads, no barriers, no epilogue.  LDS holds the bell-shaped codes of data_mode 1.  What this loop sustains
// is the ceiling of any kernel with that wave tile and instruction on such data.
__global__ void __launch_bounds__(512)
calib_mfma_lds_kernel(int iters, int* __restrict__ sink) {
    __shared__ __align__(16) int8_t lds[32768];
    for (int i = threadIdx.x; i < 32768 / 4; i += 512) {
        uint32_t w = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t r = calib_hash((uint32_t)i * 4u + c + blockIdx.x * 7919u);
            const int q = (int)((r & 63) + ((r >> 6) & 63) + ((r >> 12) & 63) + ((r >> 18) & 63)) - 126;
            w |= (uint32_t)(uint8_t)(int8_t)(q / 3) << (8 * c);
        }
        reinterpret_cast<uint32_t*>(lds)[i] = w;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // a fragment = 64 lanes x 16 consecutive bytes (conflict-free); the twelve fragments of a step are 1 KiB apart
    const int8_t* p = lds + lane * 16;
    v4i acc[8][4];
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mi][ni][r] = 0;
    for (int it = 0; it < iters; ++it) {
        const int base = ((it * 5 + wave * 3) & 15) * 1024;        // walks the 32 KiB, stays 12 KiB clear of the end
        v4i a[8], b[4];
#pragma unroll
        for (int mi = 0; mi < 8; ++mi) a[mi] = *reinterpret_cast<const v4i*>(p + ((base + mi * 1024) & 16383));
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) b[ni] = *reinterpret_cast<const v4i*>(p + 16384 + ((base + ni * 1024) & 16383));
#pragma unroll
        for (int mi = 0; mi < 8; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[mi][ni][r];
    if (s == 0x7fffffff && sink) sink[0] = s;
}

// The same for the A4W4 kernel: v_mfma_f32_16x16x128_f8f6f4 on FP6 operands that hold INT4-like codes (bell-shaped in
// [-7, 7], encoded as E2M3), 8 waves per CU, every step reads the 8 + 4 tiles of a 128 x 64 wave tile from LDS -- one
// 16-byte and one 8-byte read per lane and tile, 18 KiB per wave and step -- and issues its 32 matrix instructions
// over 128 elements of the contraction.  No global loads, no barriers, no epilogue.
typedef int calib_v8i __attribute__((ext_vector_type(8)));
typedef float calib_v4f __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(512)
calib_mfma_f6_lds_kernel(int iters, int* __restrict__ sink) {
    constexpr int kRecords = 2048;                                  // lane slots: 16 bytes + 8 bytes each
    __shared__ __align__(16) uint8_t lds[kRecords * 24];
    uint8_t* lo = lds;                                              // [kRecords][16]
    uint8_t* hi = lds + kRecords * 16;                              // [kRecords][8]
    for (int rec = threadIdx.x; rec < kRecords; rec += 512) {
        uint64_t w[3] = {0ull, 0ull, 0ull};                         // the slot's 32 fields of 6 bits
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const uint32_t r = calib_hash((uint32_t)rec * 32u + j + blockIdx.x * 7919u);
            const int q = ((int)((r & 63) + ((r >> 6) & 63) + ((r >> 12) & 63) + ((r >> 18) & 63)) - 126) / 18;
            const int mag = q < 0 ? -q : q;
            const uint64_t e = ((0x1E1C1A1814100800ull >> (8 * mag)) & 0xFFull) | (q < 0 ? 32ull : 0ull);
            const int bit = 6 * j;
            w[bit >> 6] |= e << (bit & 63);
            if ((bit & 63) > 58) w[(bit >> 6) + 1] |= e >> (64 - (bit & 63));
        }
        reinterpret_cast<uint64_t*>(lo)[rec * 2] = w[0];
        reinterpret_cast<uint64_t*>(lo)[rec * 2 + 1] = w[1];
        reinterpret_cast<uint64_t*>(hi)[rec] = w[2];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    calib_v4f acc[8][4];
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mi][ni][r] = 0.0f;
    auto tile = [&](int first_record) {
        const int rec = (first_record + lane) & (kRecords - 1);
        const uint4 l = *reinterpret_cast<const uint4*>(lo + rec * 16);
        const uint2 h = *reinterpret_cast<const uint2*>(hi + rec * 8);
        calib_v8i v;
        v[0] = (int)l.x; v[1] = (int)l.y; v[2] = (int)l.z; v[3] = (int)l.w;
        v[4] = (int)h.x; v[5] = (int)h.y; v[6] = 0; v[7] = 0;
        return v;
    };
    for (int it = 0; it < iters; ++it) {
        const int base = ((it * 5 + wave * 3) & 31) * 64;
        calib_v8i a[8], b[4];
#pragma unroll
        for (int mi = 0; mi < 8; ++mi) a[mi] = tile(base + mi * 64);
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) b[ni] = tile(base + 1024 + ni * 64);
#pragma unroll
        for (int mi = 0; mi < 8; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[mi], b[ni], acc[mi][ni], 2, 2, 0, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[mi][ni][r];
    if (s == 12345.678f && sink) sink[0] = 1;
}

int calib_blocks() {
    int dev = 0, n_cu = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    return n_cu;
}

}  // namespace

hipError_t launch_calib_read(const void* src, int64_t bytes, unsigned long long* sink, hipStream_t stream) {
    calib_read_kernel<<<dim3((unsigned)(calib_blocks() * 8)), dim3(kCalibThreads), 0, stream>>>(
        static_cast<const u32x4*>(src), bytes / 16, sink);
    return hipGetLastError();
}

hipError_t launch_calib_copy(const void* src, void* dst, int64_t bytes, hipStream_t stream) {
    calib_copy_kernel<<<dim3((unsigned)(calib_blocks() * 8)), dim3(kCalibThreads), 0, stream>>>(
        static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
    return hipGetLastError();
}

// returns the number of integer operations (2 per multiply-add) the launch performs through *ops
hipError_t launch_calib_mfma_i8(int iters, int data_mode, int* sink, double* ops, hipStream_t stream) {
    const int blocks = calib_blocks();
    if (data_mode == 2) {
        calib_mfma_lds_kernel<<<dim3((unsigned)blocks), dim3(512), 0, stream>>>(iters, sink);
        if (ops) *ops = (double)blocks * 8.0 * (double)iters * 32.0 * (2.0 * 16 * 16 * 64);
        return hipGetLastError();
    }
    if (data_mode == 3) {
        calib_mfma16_kernel<<<dim3((unsigned)blocks), dim3(512), 0, stream>>>(iters, sink);
        if (ops) *ops = (double)blocks * 8.0 * (double)iters * 32.0 * (2.0 * 16 * 16 * 64);
        return hipGetLastError();
    }
    calib_mfma_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(iters, data_mode, sink);
    if (ops) *ops = (double)blocks * 4.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 32);
    return hipGetLastError();
}

// returns the number of operations (2 per multiply-add) the launch performs through *ops
hipError_t launch_calib_mfma_f6(int iters, int* sink, double* ops, hipStream_t stream) {
    const int blocks = calib_blocks();
    calib_mfma_f6_lds_kernel<<<dim3((unsigned)blocks), dim3(512), 0, stream>>>(iters, sink);
    if (ops) *ops = (double)blocks * 8.0 * (double)iters * 32.0 * (2.0 * 16 * 16 * 128);
    return hipGetLastError();
}

}  // namespace cq
