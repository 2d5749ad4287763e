// Internal launcher interface between the C-ABI layer and the gfx950 kernels.
// Every launcher enqueues on `stream`, allocates nothing and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace cq {

// binary16 bit pattern <-> binary32 (widening is exact; narrowing rounds to nearest even)
__device__ __forceinline__ float h2f(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}
__device__ __forceinline__ uint32_t f2h(float f) {
    return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)f);
}

// two binary32 values -> packed binary16 pair, each rounded to nearest even (one v_cvt_pk_f16_f32)
__device__ __forceinline__ uint32_t pack_half2(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, f16x2));
}

// A binary32 value that must be rounded on its own before it is converted to binary16: passing
// it through an empty asm keeps the compiler from folding the multiply that produced it into a
// mixed-precision multiply-convert, which would round once where the specification rounds twice.
__device__ __forceinline__ float rounded_f32(float v) {
    asm volatile("" : "+v"(v));
    return v;
}

// Library-owned device state comes in kStateSlots pieces; a stream keeps the slot it is given on
// first use (-1: none left, or a handle that stands for several streams -- the caller then takes
// the path that clears its accumulators with a kernel of its own first).
// A launch's total thread count has to stay below 2^32: the runtime forms it in 32 bits, and a larger
// grid silently runs only as many blocks as the low 32 bits give.  Launchers check this first and
// return hipErrorInvalidValue with nothing enqueued (reported as a size over the limit).
inline bool grid_fits(int64_t blocks, int threads) {
    return blocks >= 1 && blocks * threads < ((int64_t)1 << 32);
}

// Rows per block of the quantize / count / analysis kernels = 32 * nb (8 waves x nb batches of 4 rows, nb <= 16).
// Two of these blocks fit a CU, and a launch is fastest when all its blocks are resident at once, with as little
// work each as that allows: the smallest nb >= 2 that gives at most 512 blocks (measured over a dozen shapes, for
// the count-only form too, whose blocks all end with an atomic on one word: within 2 % of the best nb everywhere;
// "at least 512 blocks, nb a power of two" lost up to 20 % on shapes whose chunk count is not a power of two).
// One-batch blocks spend most of their time forming scale factors and are left to problems that would otherwise
// fill less than the chip.  n_chunks = column chunks of 512, times matrices in a batch.
inline int quantize_batches_per_wave(int64_t n_chunks, int T) {
    auto n_blocks_for = [&](int n) { return n_chunks * ((T + 32 * n - 1) / (32 * n)); };
    const int nb_max = T >= 512 ? 16 : (T + 31) / 32;
    int nb = nb_max < 2 ? nb_max : 2;
    while (nb < nb_max && n_blocks_for(nb) > 512) ++nb;
    if (nb == 2 && n_blocks_for(2) < 200) nb = 1;
    return nb;
}

constexpr int kStateSlots = 16;
int stream_slot(hipStream_t stream);

// A kernel that needs more dynamic LDS than the default limit has to be told so once per device.
// `done` is a bit mask of the devices (ordinal < 64) on which that has happened for this kernel; devices with
// a larger ordinal are simply told every time.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// t[0..T), c[0..I) <- 0 ; then one pass over X accumulating both maxima.
// B matrices of T rows, matrix_stride elements apart (B = 1: a plain matrix); t is [B*T], c is [B*I].
hipError_t launch_absmax(const uint16_t* X, int B, int T, int I, int64_t ldx, int64_t matrix_stride, float* t,
                         float* c, hipStream_t stream);

// a_i = t_i^alpha / qmax, b_j = c_j^(1-alpha) (binary64 pow, one rounding); counters[0..n) <- 0.
hipError_t launch_scale_finalize(const float* t, const float* c, int T, int I, float alpha, int qmax,
                                 float* a, float* b, unsigned long long* counters, int n_counters,
                                 hipStream_t stream);

// "Remove Kernel" matrix and the Table 1 indicators; counters = {Z, #{c_j >= t_i}, #{B~ < B}}.
// a, b: work vectors that receive the scale factors, or both null (the kernel then forms the factors itself).
// Clears the counters on the stream first.
hipError_t launch_kernel_analysis(const uint16_t* X, int T, int I, int64_t ldx, const float* t,
                                  const float* c, float* a, float* b, float alpha, int qmax,
                                  uint16_t* xrk, unsigned long long* counters, hipStream_t stream);


// The same with the work vectors in the library's static device array (T, I <= CQ_ANALYSIS_STATIC_MAX, else
// hipErrorInvalidValue with nothing enqueued).  Calls that overlap on one device race on that array.
hipError_t launch_kernel_analysis_static(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c,
                                         float alpha, int qmax, uint16_t* xrk, unsigned long long* counters,
                                         hipStream_t stream);

// Scale factors (as launch_scale_finalize: a, b are outputs), then fused quantize / dequantize / zero
// count, in one kernel.  codes or xhat may be null (count only = both null).
// B matrices as in launch_absmax; t, a are [B*T], c, b are [B*I], codes / xhat are [B*T][...].
hipError_t launch_quantize(const uint16_t* X, int B, int T, int I, int64_t ldx, int64_t matrix_stride, const float* t,
                           const float* c, float alpha, int bits, float* a, float* b, void* codes, uint16_t* xhat,
                           unsigned long long* zero_count, hipStream_t stream);

// packed nibbles [n_bytes] -> int8 codes [2 * n_bytes]
hipError_t launch_unpack_int4(const uint8_t* packed, int64_t n_bytes, int8_t* codes, hipStream_t stream);

// Maxima, then scale factors + quantize / dequantize / zero count: launch_absmax followed by launch_quantize.
hipError_t launch_absmax_quantize(const uint16_t* X, int T, int I, int64_t ldx, float alpha, int bits, float* t,
                                  float* c, float* a, float* b, void* codes, uint16_t* xhat,
                                  unsigned long long* zero_count, hipStream_t stream);

// The same result from one kernel that reads X once and holds it in registers and LDS across a grid barrier
// (vector layout only).  hipErrorNotSupported, with nothing enqueued, when the matrix does not fit on chip or the
// stream has no barrier state of its own.
hipError_t launch_absmax_quantize_single_read(const uint16_t* X, int T, int I, int64_t ldx, float alpha, int bits, float* t,
                                  float* c, float* a, float* b, void* codes, uint16_t* xhat,
                                  unsigned long long* zero_count, hipStream_t stream);
// polls a block of the single-read kernel makes at its grid barrier before it gives up (test hook)
void set_fused_barrier_polls(unsigned polls);

hipError_t launch_weight_quantize(const uint16_t* W, int I, int O, const float* fold, int qmax,
                                  int8_t* qw, float* w_scale, hipStream_t stream);

hipError_t launch_weight_quantize_grouped(const uint16_t* W, int I, int O, const float* fold, int group, int qmax,
                                          int8_t* qw, float* w_scale, uint16_t* wdq, hipStream_t stream);

hipError_t launch_w8a8_linear(const int8_t* qx, const float* row_scale, const int8_t* qw,
                              const float* w_scale, int T, int I, int O, uint16_t* Y, int64_t ldy,
                              int32_t* acc_debug, hipStream_t stream);

// CrossQuant step inside the GEMM's activation load (X binary16 -> Y, no codes in memory); a, b receive the factors.
hipError_t launch_quantize_linear(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c,
                                  float alpha, int bits, float* a, float* b, const int8_t* qw, const float* w_scale,
                                  int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug, hipStream_t stream);

// INT4 codes as FP6 fragments (32 rows x 64 columns per 1536-byte fragment) and the A4W4 linear layer on them.
hipError_t launch_quantize_fp6(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c, float alpha,
                               float* a, float* b, void* packed, uint16_t* xhat, unsigned long long* zero_count,
                               hipStream_t stream);
int64_t fp6_packed_bytes(int64_t R, int64_t K);
int64_t fp6_packed_weight_bytes(int64_t O, int64_t K);
hipError_t launch_pack_fp6(const void* codes, int src_format, bool weights, int R, int K, void* packed,
                           hipStream_t stream);
hipError_t launch_w4a4_linear(const void* qx6, const float* row_scale, const void* qw6, const float* w_scale, int T,
                              int I, int O, uint16_t* Y, int64_t ldy, int32_t* acc_debug, hipStream_t stream);

// Roofline calibration (plain read, plain copy, MFMA-only loop); bytes is a multiple of 16.
hipError_t launch_calib_read(const void* src, int64_t bytes, unsigned long long* sink, hipStream_t stream);
hipError_t launch_calib_copy(const void* src, void* dst, int64_t bytes, hipStream_t stream);
hipError_t launch_calib_mfma_i8(int iters, int data_mode, int* sink, double* ops, hipStream_t stream);
hipError_t launch_calib_mfma_f6(int iters, int* sink, double* ops, hipStream_t stream);

}  // namespace cq
