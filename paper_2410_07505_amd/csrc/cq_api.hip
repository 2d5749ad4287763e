// C-ABI entry points: argument validation on the host, then kernel launches on the caller's
// stream.  No allocation and no host synchronisation.  The library does hold a little process-wide
// state, all of it behind these calls: the table that gives every stream handle a slot of device-side
// accumulators (cq_slots.hip: the quantize kernel's zero-count words, the counters of the absmax launch
// that clears for itself, with the values they reach kept on the host, the barrier words of the
// single-read kernel and its poll limit), the device addresses of those and of the static work array of
// crossquant_kernel_analysis_static, and one flag per kernel and device saying that the kernel has been
// allowed its dynamic LDS size.
#include "../../include/crossquant.h"
#include "../../include/crossquant_bench.h"

#include <cmath>

#include "cq_kernels.h"

namespace {

inline bool dim_ok(int64_t v) { return v >= 1 && v <= CQ_MAX_DIM; }
inline bool aligned(const void* p, uintptr_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

int check_matrix(const void* X, int64_t T, int64_t I, int64_t ldx) {
    if (!X) return CQ_ERR_NULL;
    if (!dim_ok(T) || !dim_ok(I) || ldx < I || ldx > CQ_MAX_DIM) return CQ_ERR_SHAPE;
    if (T * I > CQ_MAX_ELEMS || T * ldx > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    if (!aligned(X, 2)) return CQ_ERR_ALIGN;
    return CQ_OK;
}

// [B][S][I] tensor: sequence b starts batch_stride elements after sequence b-1
int check_batch(const void* X, int64_t B, int64_t S, int64_t I, int64_t ldx, int64_t batch_stride) {
    if (int s = check_matrix(X, S, I, ldx)) return s;
    if (!dim_ok(B) || B * S > CQ_MAX_DIM || B * I > CQ_MAX_DIM) return CQ_ERR_SHAPE;
    if (batch_stride < (S - 1) * ldx + I || batch_stride > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    if (B * S * I > CQ_MAX_ELEMS || (B - 1) * batch_stride > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    return CQ_OK;
}

int check_quant_params(float alpha, int bits, int64_t I) {
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (bits == 4 && (I & 1)) return CQ_ERR_BITS;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return CQ_ERR_ALPHA;   // also rejects NaN
    return CQ_OK;
}

// do two float vectors share any element?
inline bool overlap(const float* p, int64_t n, const float* q, int64_t m) { return p < q + m && q < p + n; }

// hipErrorInvalidValue is what the launchers return, before enqueuing anything, for a grid whose total
// thread count would not fit in 32 bits
inline int from_hip(hipError_t e) {
    return e == hipSuccess ? CQ_OK : (e == hipErrorInvalidValue ? CQ_ERR_SHAPE : CQ_ERR_HIP);
}

}  // namespace

extern "C" {

int crossquant_absmax(const void* X, int64_t T, int64_t I, int64_t ldx, float* t, float* c, void* stream) {
    if (!t || !c) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (!aligned(t, 4) || !aligned(c, 4)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_absmax(static_cast<const uint16_t*>(X), 1, (int)T, (int)I, ldx, 0, t, c,
                                      static_cast<hipStream_t>(stream)));
}

int crossquant_absmax_batched(const void* X, int64_t B, int64_t S, int64_t I, int64_t ldx, int64_t batch_stride,
                              float* t, float* c, void* stream) {
    if (!t || !c) return CQ_ERR_NULL;
    if (int s = check_batch(X, B, S, I, ldx, batch_stride)) return s;
    if (!aligned(t, 4) || !aligned(c, 4)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_absmax(static_cast<const uint16_t*>(X), (int)B, (int)S, (int)I, ldx, batch_stride, t, c,
                                      static_cast<hipStream_t>(stream)));
}

int crossquant_quantize(const void* X, int64_t T, int64_t I, int64_t ldx, const float* t, const float* c,
                        float alpha, int bits, void* codes, void* xhat, float* row_scale, float* col_scale,
                        unsigned long long* zero_count, void* stream) {
    if (!t || !c || !codes || !row_scale || !col_scale) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (int s = check_quant_params(alpha, bits, I)) return s;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(xhat, 2) || !aligned(zero_count, 8))
        return CQ_ERR_ALIGN;
    if (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I)) return CQ_ERR_ALIAS;
    return from_hip(cq::launch_quantize(static_cast<const uint16_t*>(X), 1, (int)T, (int)I, ldx, 0, t, c, alpha, bits,
                                        row_scale, col_scale, codes, static_cast<uint16_t*>(xhat), zero_count,
                                        static_cast<hipStream_t>(stream)));
}

int crossquant_quantize_batched(const void* X, int64_t B, int64_t S, int64_t I, int64_t ldx, int64_t batch_stride,
                                const float* t, const float* c, float alpha, int bits, void* codes, void* xhat,
                                float* row_scale, float* col_scale, unsigned long long* zero_count, void* stream) {
    if (!t || !c || !row_scale || !col_scale) return CQ_ERR_NULL;
    if (!codes && (xhat || !zero_count)) return CQ_ERR_NULL;      // codes == NULL: count only
    if (int s = check_batch(X, B, S, I, ldx, batch_stride)) return s;
    if (int s = check_quant_params(alpha, bits, codes ? I : 0)) return s;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(xhat, 2) || !aligned(zero_count, 8))
        return CQ_ERR_ALIGN;
    if (overlap(t, B * S, row_scale, B * S) || overlap(c, B * I, col_scale, B * I)) return CQ_ERR_ALIAS;
    return from_hip(cq::launch_quantize(static_cast<const uint16_t*>(X), (int)B, (int)S, (int)I, ldx, batch_stride, t, c,
                                        alpha, bits, row_scale, col_scale, codes, static_cast<uint16_t*>(xhat),
                                        zero_count, static_cast<hipStream_t>(stream)));
}

int crossquant_absmax_quantize(const void* X, int64_t T, int64_t I, int64_t ldx, float alpha, int bits, float* t,
                               float* c, void* codes, void* xhat, float* row_scale, float* col_scale,
                               unsigned long long* zero_count, void* stream) {
    if (!t || !c || !codes || !row_scale || !col_scale) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (int s = check_quant_params(alpha, bits, I)) return s;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(xhat, 2) || !aligned(zero_count, 8))
        return CQ_ERR_ALIGN;
    if (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I)) return CQ_ERR_ALIAS;
    return from_hip(cq::launch_absmax_quantize(static_cast<const uint16_t*>(X), (int)T, (int)I, ldx, alpha, bits, t, c,
                                               row_scale, col_scale, codes, static_cast<uint16_t*>(xhat), zero_count,
                                               static_cast<hipStream_t>(stream)));
}

int crossquant_absmax_quantize_single_read(const void* X, int64_t T, int64_t I, int64_t ldx, float alpha, int bits,
                                           float* t, float* c, void* codes, void* xhat, float* row_scale,
                                           float* col_scale, unsigned long long* zero_count, void* stream) {
    if (!t || !c || !codes || !row_scale || !col_scale) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (int s = check_quant_params(alpha, bits, I)) return s;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(xhat, 2) || !aligned(zero_count, 8))
        return CQ_ERR_ALIGN;
    if (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I)) return CQ_ERR_ALIAS;
    // the register-resident kernel only takes the vector layout
    if (!aligned(X, 16) || ldx % 8 != 0 || I % 8 != 0 || !aligned(codes, 8) || !aligned(xhat, 16))
        return CQ_ERR_UNSUPPORTED;
    const hipError_t e = cq::launch_absmax_quantize_single_read(
        static_cast<const uint16_t*>(X), (int)T, (int)I, ldx, alpha, bits, t, c, row_scale, col_scale, codes,
        static_cast<uint16_t*>(xhat), zero_count, static_cast<hipStream_t>(stream));
    if (e == hipErrorNotSupported) return CQ_ERR_UNSUPPORTED;
    return from_hip(e);
}

void crossquant_debug_set_barrier_polls(unsigned polls) { cq::set_fused_barrier_polls(polls); }

int crossquant_kernel_count(const void* X, int64_t T, int64_t I, int64_t ldx, const float* t, const float* c,
                            float alpha, int bits, float* row_scale, float* col_scale,
                            unsigned long long* zero_count, void* stream) {
    if (!t || !c || !zero_count) return CQ_ERR_NULL;
    if ((row_scale == nullptr) != (col_scale == nullptr)) return CQ_ERR_NULL;     // both or neither
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return CQ_ERR_ALPHA;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(zero_count, 8))
        return CQ_ERR_ALIGN;
    if (row_scale && (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I))) return CQ_ERR_ALIAS;
    return from_hip(cq::launch_quantize(static_cast<const uint16_t*>(X), 1, (int)T, (int)I, ldx, 0, t, c, alpha, bits,
                                        row_scale, col_scale, nullptr, nullptr, zero_count,
                                        static_cast<hipStream_t>(stream)));
}

int crossquant_kernel_analysis(const void* X, int64_t T, int64_t I, int64_t ldx, const float* t, const float* c,
                               float alpha, int bits, void* xrk, float* row_scale, float* col_scale,
                               unsigned long long* counters, void* stream) {
    if (!t || !c || !counters) return CQ_ERR_NULL;
    if ((row_scale == nullptr) != (col_scale == nullptr)) return CQ_ERR_NULL;     // both or neither
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return CQ_ERR_ALPHA;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(xrk, 2) || !aligned(counters, 8))
        return CQ_ERR_ALIGN;
    // the factors are written by one kernel while the next one still reads t and c
    if (row_scale && (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I))) return CQ_ERR_ALIAS;
    const int qmax = (1 << (bits - 1)) - 1;
    return from_hip(cq::launch_kernel_analysis(static_cast<const uint16_t*>(X), (int)T, (int)I, ldx, t, c,
                                               row_scale, col_scale, alpha, qmax, static_cast<uint16_t*>(xrk),
                                               counters, static_cast<hipStream_t>(stream)));
}

int crossquant_kernel_analysis_static(const void* X, int64_t T, int64_t I, int64_t ldx, const float* t, const float* c,
                                      float alpha, int bits, void* xrk, unsigned long long* counters, void* stream) {
    if (!t || !c || !counters) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (T > CQ_ANALYSIS_STATIC_MAX || I > CQ_ANALYSIS_STATIC_MAX) return CQ_ERR_SHAPE;
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return CQ_ERR_ALPHA;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(xrk, 2) || !aligned(counters, 8)) return CQ_ERR_ALIGN;
    const int qmax = (1 << (bits - 1)) - 1;
    return from_hip(cq::launch_kernel_analysis_static(static_cast<const uint16_t*>(X), (int)T, (int)I, ldx, t, c, alpha,
                                                      qmax, static_cast<uint16_t*>(xrk), counters,
                                                      static_cast<hipStream_t>(stream)));
}

int crossquant_unpack_int4(const void* packed, int64_t T, int64_t I, int8_t* codes, void* stream) {
    if (!packed || !codes) return CQ_ERR_NULL;
    if (!dim_ok(T) || !dim_ok(I) || (I & 1) || T * I > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    return from_hip(cq::launch_unpack_int4(static_cast<const uint8_t*>(packed), T * (I / 2), codes,
                                           static_cast<hipStream_t>(stream)));
}

int crossquant_weight_quantize(const void* W, int64_t I, int64_t O, const float* fold, int bits, int8_t* qw,
                               float* w_scale, void* stream) {
    if (!W || !qw || !w_scale) return CQ_ERR_NULL;
    if (!dim_ok(I) || !dim_ok(O) || I * O > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (!aligned(W, 2) || !aligned(w_scale, 4) || !aligned(fold, 4)) return CQ_ERR_ALIGN;
    const int qmax = (1 << (bits - 1)) - 1;
    return from_hip(cq::launch_weight_quantize(static_cast<const uint16_t*>(W), (int)I, (int)O, fold, qmax, qw,
                                               w_scale, static_cast<hipStream_t>(stream)));
}

int crossquant_weight_quantize_grouped(const void* W, int64_t I, int64_t O, const float* fold, int64_t group,
                                       int bits, int8_t* qw, float* w_scale, void* w_dq, void* stream) {
    if (!W || !qw || !w_scale) return CQ_ERR_NULL;
    if (!dim_ok(I) || !dim_ok(O) || I * O > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    if (group < 1 || group > I || I % group != 0) return CQ_ERR_SHAPE;
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (!aligned(W, 2) || !aligned(w_scale, 4) || !aligned(fold, 4) || !aligned(w_dq, 2)) return CQ_ERR_ALIGN;
    const int qmax = (1 << (bits - 1)) - 1;
    return from_hip(cq::launch_weight_quantize_grouped(static_cast<const uint16_t*>(W), (int)I, (int)O, fold,
                                                       (int)group, qmax, qw, w_scale,
                                                       static_cast<uint16_t*>(w_dq), static_cast<hipStream_t>(stream)));
}

int crossquant_w8a8_linear(const int8_t* qx, const float* row_scale, const int8_t* qw, const float* w_scale,
                           int64_t T, int64_t I, int64_t O, void* Y, int64_t ldy, int32_t* acc_debug,
                           void* stream) {
    if (!qx || !row_scale || !qw || !w_scale || !Y) return CQ_ERR_NULL;
    if (!dim_ok(T) || !dim_ok(I) || !dim_ok(O) || ldy < O || ldy > CQ_MAX_DIM) return CQ_ERR_SHAPE;
    if (T * I > CQ_MAX_ELEMS || I * O > CQ_MAX_ELEMS || T * ldy > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    if (I > 133000) return CQ_ERR_SHAPE;     // 127 * 127 * I must fit the int32 accumulator
    if (!aligned(row_scale, 4) || !aligned(w_scale, 4) || !aligned(Y, 2) || !aligned(acc_debug, 4))
        return CQ_ERR_ALIGN;
    return from_hip(cq::launch_w8a8_linear(qx, row_scale, qw, w_scale, (int)T, (int)I, (int)O,
                                           static_cast<uint16_t*>(Y), ldy, acc_debug,
                                           static_cast<hipStream_t>(stream)));
}

int crossquant_quantize_linear_fused(const void* X, int64_t T, int64_t I, int64_t ldx, const float* t, const float* c,
                                     float alpha, int bits, const int8_t* qw, const float* w_scale, int64_t O, void* Y,
                                     int64_t ldy, float* row_scale, float* col_scale, int32_t* acc_debug, void* stream) {
    if (!t || !c || !qw || !w_scale || !Y || !row_scale || !col_scale) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (!dim_ok(O) || ldy < O || ldy > CQ_MAX_DIM) return CQ_ERR_SHAPE;
    if (I * O > CQ_MAX_ELEMS || T * ldy > CQ_MAX_ELEMS || I > 133000) return CQ_ERR_SHAPE;
    if (bits != 4 && bits != 8) return CQ_ERR_BITS;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return CQ_ERR_ALPHA;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) || !aligned(w_scale, 4) ||
        !aligned(Y, 2) || !aligned(acc_debug, 4))
        return CQ_ERR_ALIGN;
    if (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I)) return CQ_ERR_ALIAS;
    // only the layout of a real layer: whole K steps, vector loads
    if (I % 128 != 0 || ldx % 8 != 0 || !aligned(X, 16) || !aligned(qw, 16) || !aligned(col_scale, 16))
        return CQ_ERR_UNSUPPORTED;
    return from_hip(cq::launch_quantize_linear(static_cast<const uint16_t*>(X), (int)T, (int)I, ldx, t, c, alpha, bits,
                                               row_scale, col_scale, qw, w_scale, (int)O, static_cast<uint16_t*>(Y),
                                               ldy, acc_debug, static_cast<hipStream_t>(stream)));
}

int64_t crossquant_fp6_packed_bytes(int64_t R, int64_t K) {
    if (!dim_ok(R) || !dim_ok(K) || K % 128 != 0) return -1;
    return cq::fp6_packed_bytes(R, K);
}

int64_t crossquant_fp6_packed_weight_bytes(int64_t O, int64_t K) {
    if (!dim_ok(O) || !dim_ok(K) || K % 128 != 0) return -1;
    return cq::fp6_packed_weight_bytes(O, K);
}

static int pack_fp6(const void* codes, int src_format, bool weights, int64_t R, int64_t K, void* packed, void* stream) {
    if (!codes || !packed) return CQ_ERR_NULL;
    if (!dim_ok(R) || !dim_ok(K) || R * K > CQ_MAX_ELEMS) return CQ_ERR_SHAPE;
    if (src_format != 8 && src_format != 4) return CQ_ERR_BITS;
    if (K % 128 != 0) return CQ_ERR_UNSUPPORTED;
    if (!aligned(codes, 16) || !aligned(packed, 16)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_pack_fp6(codes, src_format, weights, (int)R, (int)K, packed,
                                        static_cast<hipStream_t>(stream)));
}

int crossquant_pack_fp6(const void* codes, int src_format, int64_t R, int64_t K, void* packed, void* stream) {
    return pack_fp6(codes, src_format, false, R, K, packed, stream);
}

int crossquant_pack_fp6_weights(const void* codes, int src_format, int64_t O, int64_t K, void* packed, void* stream) {
    return pack_fp6(codes, src_format, true, O, K, packed, stream);
}

int crossquant_quantize_fp6(const void* X, int64_t T, int64_t I, int64_t ldx, const float* t, const float* c,
                            float alpha, void* packed, void* xhat, float* row_scale, float* col_scale,
                            unsigned long long* zero_count, void* stream) {
    if (!t || !c || !packed || !row_scale || !col_scale) return CQ_ERR_NULL;
    if (int s = check_matrix(X, T, I, ldx)) return s;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return CQ_ERR_ALPHA;
    if (!aligned(t, 4) || !aligned(c, 4) || !aligned(row_scale, 4) || !aligned(col_scale, 4) ||
        !aligned(xhat, 2) || !aligned(zero_count, 8))
        return CQ_ERR_ALIGN;
    if (I % 128 != 0 || !aligned(packed, 16)) return CQ_ERR_UNSUPPORTED;
    if (overlap(t, T, row_scale, T) || overlap(c, I, col_scale, I)) return CQ_ERR_ALIAS;
    return from_hip(cq::launch_quantize_fp6(static_cast<const uint16_t*>(X), (int)T, (int)I, ldx, t, c, alpha, row_scale,
                                            col_scale, packed, static_cast<uint16_t*>(xhat), zero_count,
                                            static_cast<hipStream_t>(stream)));
}

int crossquant_w4a4_linear(const void* qx_fp6, const float* row_scale, const void* qw_fp6, const float* w_scale,
                           int64_t T, int64_t I, int64_t O, void* Y, int64_t ldy, int32_t* acc_debug, void* stream) {
    if (!qx_fp6 || !row_scale || !qw_fp6 || !w_scale || !Y) return CQ_ERR_NULL;
    if (!dim_ok(T) || !dim_ok(I) || !dim_ok(O) || ldy < O || ldy > CQ_MAX_DIM) return CQ_ERR_SHAPE;
    if (T * O > CQ_MAX_ELEMS || T * ldy > CQ_MAX_ELEMS || T * I > CQ_MAX_ELEMS || I * O > CQ_MAX_ELEMS)
        return CQ_ERR_SHAPE;
    if (I > (1 << 18)) return CQ_ERR_SHAPE;                 // 49 * I must stay below 2^24 (exact in binary32)
    if (!aligned(row_scale, 4) || !aligned(w_scale, 4) || !aligned(Y, 2) || !aligned(acc_debug, 4)) return CQ_ERR_ALIGN;
    if (I % 128 != 0 || O % 8 != 0 || ldy % 8 != 0 || !aligned(qx_fp6, 16) || !aligned(qw_fp6, 16) ||
        !aligned(Y, 16) || !aligned(w_scale, 16) || !aligned(acc_debug, 16) || ldy >= ((int64_t)1 << 22))
        return CQ_ERR_UNSUPPORTED;
    return from_hip(cq::launch_w4a4_linear(qx_fp6, row_scale, qw_fp6, w_scale, (int)T, (int)I, (int)O,
                                           static_cast<uint16_t*>(Y), ldy, acc_debug,
                                           static_cast<hipStream_t>(stream)));
}

int crossquant_calib_read(const void* src, int64_t bytes, unsigned long long* sink, void* stream) {
    if (!src) return CQ_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return CQ_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(sink, 8)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_calib_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

int crossquant_calib_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (!src || !dst) return CQ_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return CQ_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_calib_copy(src, dst, bytes, static_cast<hipStream_t>(stream)));
}

int crossquant_calib_mfma_i8(int iters, int data_mode, int* sink, double* ops, void* stream) {
    if (iters < 1 || iters > (1 << 20)) return CQ_ERR_SHAPE;
    if (data_mode < 0 || data_mode > 3) return CQ_ERR_UNSUPPORTED;
    if (!aligned(sink, 4)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_calib_mfma_i8(iters, data_mode, sink, ops, static_cast<hipStream_t>(stream)));
}

int crossquant_calib_mfma_f6(int iters, int* sink, double* ops, void* stream) {
    if (iters < 1 || iters > (1 << 20)) return CQ_ERR_SHAPE;
    if (!aligned(sink, 4)) return CQ_ERR_ALIGN;
    return from_hip(cq::launch_calib_mfma_f6(iters, sink, ops, static_cast<hipStream_t>(stream)));
}

const char* crossquant_status_string(int status) {
    switch (status) {
        case CQ_OK: return "ok";
        case CQ_ERR_NULL: return "a required pointer is NULL";
        case CQ_ERR_SHAPE: return "invalid shape or leading dimension";
        case CQ_ERR_BITS: return "bits must be 8, or 4 with an even number of channels";
        case CQ_ERR_ALPHA: return "alpha must lie in [0, 1]";
        case CQ_ERR_ALIGN: return "pointer alignment violated";
        case CQ_ERR_UNSUPPORTED: return "unsupported request";
        case CQ_ERR_HIP: return "kernel launch failed";
        case CQ_ERR_ALIAS: return "an output vector overlaps an input vector";
        default: return "unknown status";
    }
}

int crossquant_version(void) { return 200; }      // 0.2.0: the A4W4 weight operand has its own row order

}  // extern "C"
