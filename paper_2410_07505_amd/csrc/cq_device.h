// Device-side building blocks shared by the streaming kernels (absmax, quantize, fused).
#pragma once
#include "cq_kernels.h"

namespace cq {

constexpr int kLanes = 64;
constexpr int kColsPerWave = kLanes * 8;          // a wave owns 512 columns: 8 halfs (16 bytes) per lane
constexpr float kMagic = 12582912.0f;             // 1.5 * 2^23: adding it rounds to nearest-even integer
constexpr float kTieTol = 1.9073486328125e-06f;   // 2^-19

typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// packed maximum of two pairs of 16-bit patterns (|x| of binary16 orders like an unsigned integer)
__device__ __forceinline__ uint32_t pkmax(uint32_t a, uint32_t b) {
    us2 r = __builtin_elementwise_max(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b));
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ uint32_t half_bits_to_float_bits(uint32_t h) { return __float_as_uint(h2f(h)); }

__device__ __forceinline__ uint32_t shx(uint32_t v, int off) { return (uint32_t)__shfl_xor((int)v, off, kLanes); }

// 8 halfs starting at column j of a row; columns >= I read as zero.
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

// Per-lane maximum |x| of a 16-byte piece (a 16-bit pattern), also folded into four packed
// running column maxima.
__device__ __forceinline__ uint32_t absmax8(const uint4& v, uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3) {
    const uint32_t x0 = v.x & 0x7FFF7FFFu, x1 = v.y & 0x7FFF7FFFu;
    const uint32_t x2 = v.z & 0x7FFF7FFFu, x3 = v.w & 0x7FFF7FFFu;
    c0 = pkmax(c0, x0);
    c1 = pkmax(c1, x1);
    c2 = pkmax(c2, x2);
    c3 = pkmax(c3, x3);
    const uint32_t m = pkmax(pkmax(x0, x1), pkmax(x2, x3));
    return max(m & 0xFFFFu, m >> 16);
}

// rm[g] = this lane's maximum over its 8 columns of row g (a 16-bit pattern).  Returns, in lane
// l with (l & 7) == 0, the maximum over all 64 lanes of row (l >> 3).  A transposed butterfly:
// every exchange step halves the number of rows a lane still carries (7 shuffles for 8 rows).
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

// ---- scale factors of the CrossQuant step (binary64 pow, one rounding to binary32).
// pow(x, 0) = 1 for every x and pow(x, 1) = x are exact in any correct pow; they are written out
// so that the two special exponents (per-column and per-token steps) never depend on it.
__device__ __forceinline__ float row_factor(float t, double al, int qmax) {
    const double ti = (double)t;
    const double p = (al == 0.0) ? 1.0 : (al == 1.0 ? ti : pow(ti, al));
    return (float)(p / (double)qmax);
}
__device__ __forceinline__ float col_factor(float c, double al) {
    const double cj = (double)c;
    const double e = 1.0 - al;
    const double p = (e == 0.0) ? 1.0 : (e == 1.0 ? cj : pow(cj, e));
    return (float)p;
}

// Scale factors of one block of 512 threads, shared through LDS: thread k forms the factor of column col0 + k
// (lds_b[k]; 0 past the last column) and, if the block has that many rows, of row row0 + k (lds_a[k]; 0 past
// the last row).  a_out / b_out (nullable): where the caller wants them written as well.  Every block that
// needs a factor computes the same bits from the same inputs.  The caller synchronises the block afterwards.
__device__ __forceinline__ void block_scale_factors(const float* __restrict__ t_vec, const float* __restrict__ c_vec,
                                                    double alpha, int qmax, int T, int I, int col0, int row0,
                                                    int rows_per_block, float* lds_a, float* lds_b,
                                                    float* __restrict__ a_out, float* __restrict__ b_out) {
    const int k = (int)threadIdx.x;
    const int j = col0 + k;
    float bj = 0.0f;
    if (j < I) {
        bj = col_factor(c_vec[j], alpha);
        if (b_out) b_out[j] = bj;
    }
    lds_b[k] = bj;
    const int r = row0 + k;
    float ar = 0.0f;
    if (k < rows_per_block && r < T) {
        ar = row_factor(t_vec[r], alpha, qmax);
        if (a_out) a_out[r] = ar;
    }
    lds_a[k] = ar;
}

__device__ __forceinline__ float safe_rcp(float v) { return (v == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(v); }

__device__ __forceinline__ float half_lo(uint32_t w) { return h2f(w & 0xFFFFu); }
__device__ __forceinline__ float half_hi(uint32_t w) { return h2f(w >> 16); }

// Output stores of the streaming kernels: written through to memory at device scope (sc1) instead
// of being left dirty in the caches.  Measured on the 4096 x 8192 layer against plain and
// non-temporal stores: the quantize kernel itself is 3 us (8 %) faster, and the matrix kernel that
// reads the codes next 5 us.  The compiler offers no way to ask for this policy, hence the
// assembly; it cannot see a store in it, so the two wait states the hardware needs before the data
// registers of a wide store may be overwritten are added by hand.
__device__ __forceinline__ void store_through(uint32_t v, uint32_t* dst) {
    asm volatile("global_store_dword %0, %1, off sc1\n\ts_nop 1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(u32x2 v, u32x2* dst) {
    asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(u32x4 v, u32x4* dst) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(dst), "v"(v) : "memory");
}

// bytes 0 of four words -> one word
__device__ __forceinline__ uint32_t pack_bytes(uint32_t u0, uint32_t u1, uint32_t u2, uint32_t u3) {
    const uint32_t p01 = __builtin_amdgcn_perm(u1, u0, 0x0c0c0400u);
    const uint32_t p23 = __builtin_amdgcn_perm(u3, u2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(p23, p01, 0x05040100u);
}

// ---- one lane's 8 elements of one row.  On return q[e] = q_e and m[e] = kMagic + q_e with
// q_e = clamp(rne(fl32(x_e / fl32(a * b[e]))), +-qmax), identical to dividing every element.
// The quotient is first approximated as x * (1/a) * (1/b) (ra, rb: reciprocals within 1 ulp, 0
// where the factor is 0), which lies within 2^-21 relative of the correctly rounded quotient
// (two reciprocals at 2^-23, the rounding of their product and of a * b at 2^-24, and the
// quotient's own; 2^-20.7 even if each reciprocal were a further half ulp off).  The product is
// never formed on its own: fma(x, k, 1.5 * 2^23) rounds it straight to the nearest-even integer
// (the sum's ulp is 1), q = that - 1.5 * 2^23 is the code, and a second fma, x * k - q, gives the
// distance from it.  The integer can differ from the exact one only if the approximation lies
// within the bound of a rounding tie k + 1/2: lanes test |x k - q| + (|q| + 1) * 2^-19 >= 1/2
// (a 3x to 4x margin) and also |q| > qmax (a code that needs clamping: only with caller-supplied
// maxima below the data's), and a wave in which any lane trips recomputes its eight elements with
// the exact division and the clamp.  Both fmas read the binary16 value directly (v_fma_mix_f32).
// The bound needs ra * rb and a * b to be normal numbers: `tiny` (any factor of this lane's piece
// below kTinyFactor, possible only with caller-supplied maxima far below anything binary16 data
// can produce) sends the piece to the exact division as well.
constexpr float kTinyFactor = 8.673617379884035e-19f;   // 2^-60: both products stay within 2^+-120

__device__ __forceinline__ bool tiny_factor(float f) { return f != 0.0f && f < kTinyFactor; }

// The fast part: m, q from the reciprocals; returns whether this wave's row piece has to be redone exactly
// (wave-uniform).
__device__ __forceinline__ bool quantize8_fast(const uint4& v, float ra, const float (&rb)[8], float qmax,
                                               float (&m)[8], float (&q)[8], bool tiny) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    _Float16 h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = __builtin_bit_cast(_Float16, (unsigned short)(w[e >> 1] >> (16 * (e & 1))));
    float score = 0.0f;                                 // max over the 8 elements of |x k - q| + |q| * tol
    float big = 0.0f;                                   // max over the 8 elements of |q|
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float k = ra * rb[e];
        m[e] = __builtin_fmaf((float)h[e], k, kMagic);
        q[e] = m[e] - kMagic;
        const float f = __builtin_fmaf((float)h[e], k, -q[e]);
        score = __builtin_fmaxf(score, __builtin_fmaf(__builtin_fabsf(q[e]), kTieTol, __builtin_fabsf(f)));
        big = __builtin_fmaxf(big, __builtin_fabsf(q[e]));
    }
    // !(big <= qmax) also catches a NaN from an overflowed product
    return __any(score >= 0.5f - kTieTol || !(big <= qmax) || tiny);
}
// The exact part: the correctly rounded division and the clamp, for all 8 elements.
__device__ __forceinline__ void quantize8_exact(const uint4& v, float a, const float (&b)[8], float qmax,
                                                float (&m)[8], float (&q)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = (float)__builtin_bit_cast(_Float16, (unsigned short)(w[e >> 1] >> (16 * (e & 1))));
        const float D = a * b[e];
        float rt = (D == 0.0f) ? 0.0f : x / D;
        rt = __builtin_amdgcn_fmed3f(rt, -qmax, qmax);
        m[e] = rt + kMagic;
        q[e] = m[e] - kMagic;
    }
}
__device__ __forceinline__ void quantize8(const uint4& v, float a, float ra, const float (&b)[8],
                                          const float (&rb)[8], float qmax, float (&m)[8], float (&q)[8],
                                          bool tiny) {
    if (quantize8_fast(v, ra, rb, qmax, m, q, tiny)) quantize8_exact(v, a, b, qmax, m, q);   // rare
}

// Count-only form of quantize8: how many of the wave's 8 x 64 elements of one row have a non-zero code.
// q = rne(fl32(x / fl32(a b))) is 0 exactly when the quotient is at most 1/2 (a tie rounds to the even
// 0), so the sign of d = fma(|x|, 1/b, -a/2) decides, unless the two sides are within 2^-20 of each
// other: |x| / b differs from (x / fl32(a b)) a by at most 2^-22 relative (reciprocal, rounding of
// a b, the quotient's own rounding; the fma's single rounding never changes its sign).  A wave in
// which any lane comes that close, or has a factor so small that products leave the normal range,
// recounts the row piece with the exact division.  ha = a / 2 (exact), tol = ha * 2^-19.
__device__ __forceinline__ uint32_t count_row8_wave(const uint4& v, float a, float ha, float tol, const float (&b)[8],
                                                    const float (&rb)[8], float qmax, bool tiny) {
    float x[8];
    x[0] = half_lo(v.x); x[1] = half_hi(v.x);
    x[2] = half_lo(v.y); x[3] = half_hi(v.y);
    x[4] = half_lo(v.z); x[5] = half_hi(v.z);
    x[6] = half_lo(v.w); x[7] = half_hi(v.w);
    uint32_t nz = 0u;
    unsigned long long close = 0ull;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float d = __builtin_fmaf(__builtin_fabsf(x[e]), rb[e], -ha);
        nz += (uint32_t)__builtin_popcountll(__ballot(d > 0.0f));
        close |= __ballot(__builtin_fabsf(d) <= tol);
    }
    if (close != 0ull || __any(tiny)) {                 // rare: exact division for this wave's row piece
        nz = 0u;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float D = a * b[e];
            float rt = (D == 0.0f) ? 0.0f : x[e] / D;
            rt = __builtin_amdgcn_fmed3f(rt, -qmax, qmax);
            nz += (uint32_t)__builtin_popcountll(__ballot(rt + kMagic != kMagic));
        }
    }
    return nz;
}

// The same decision counted per lane: every lane returns how many of its own 8 elements have a non-zero code, and
// the kernel adds the lanes up once at its end.  A compare and an add-with-carry per element and one running
// minimum of |d| for the closeness test, all vector instructions: the form above hands every compare mask to the
// scalar unit (population count, add, or), which the four SIMDs of a CU share; in the streaming count-only kernel
// that was 1.6 scalar instructions per vector instruction.
__device__ __forceinline__ uint32_t count_row8_lane(const uint4& v, float a, float ha, float tol, const float (&b)[8],
                                                    const float (&rb)[8], float qmax, bool tiny) {
    float x[8];
    x[0] = half_lo(v.x); x[1] = half_hi(v.x);
    x[2] = half_lo(v.y); x[3] = half_hi(v.y);
    x[4] = half_lo(v.z); x[5] = half_hi(v.z);
    x[6] = half_lo(v.w); x[7] = half_hi(v.w);
    uint32_t nz = 0u;
    float nearest = __builtin_inff();
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float d = __builtin_fmaf(__builtin_fabsf(x[e]), rb[e], -ha);
        // nz += d > 0, as a compare and an add of its carry (written out: from "nz += d > 0 ? 1 : 0" the compiler
        // builds a bit mask of the eight compares with shifts and ors and counts its bits, three times the work)
        asm("v_cmp_lt_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, 0, %0, vcc" : "+v"(nz) : "v"(d) : "vcc");
        nearest = __builtin_fminf(nearest, __builtin_fabsf(d));
    }
    if (__any(nearest <= tol || tiny)) {                // rare: exact division for this wave's row piece
        nz = 0u;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float D = a * b[e];
            float rt = (D == 0.0f) ? 0.0f : x[e] / D;
            rt = __builtin_amdgcn_fmed3f(rt, -qmax, qmax);
            nz += (rt + kMagic != kMagic) ? 1u : 0u;
        }
    }
    return nz;
}

// number of non-zero codes among the whole wave's m[0..8): one compare per element, the counting is
// scalar (population count of the compare mask).  Only active lanes are counted.
__device__ __forceinline__ uint32_t count_nonzero8_wave(const float (&m)[8]) {
    uint32_t nz = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) nz += (uint32_t)__builtin_popcountll(__ballot(m[e] != kMagic));
    return nz;
}

// The same per lane, for the streaming kernel, which adds the lanes up once at its end: a compare and an add of
// its carry per element and nothing for the scalar unit, which the four SIMDs of a CU share.
__device__ __forceinline__ uint32_t count_nonzero8_lane(const float (&m)[8]) {
    uint32_t nz = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        asm("v_cmp_neq_f32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, 0, %0, vcc" : "+v"(nz) : "v"(m[e]), "v"(kMagic) : "vcc");
    return nz;
}

// number of non-zero codes among m[0..8) (as a float: exact far below 2^24)
__device__ __forceinline__ float count_nonzero8(const float (&m)[8]) {
    float nz = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) nz += __builtin_fminf(__builtin_fabsf(m[e] - kMagic), 1.0f);
    return nz;
}

// ---- buffer access for the streaming kernels.  A row piece is addressed as a raw buffer: its base and its
// length in bytes sit in scalar registers, every lane adds its own byte offset, and the hardware's range check
// does the masking: a load at or past the end returns 0, a store there is dropped.  Only used where a lane's
// piece lies entirely inside or entirely outside the row (no partial pieces).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t row_buffer(const void* base, int bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);   // raw, 32-bit data
}
constexpr int kWriteThrough = 16;     // cache policy sc1: written through to memory at device scope (see store_through)
__device__ __forceinline__ uint4 buffer_load16(rsrc_t r, int byte_offset) {
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, 0));
}

// INT8 codes of 8 elements as 8 bytes (the low mantissa byte of kMagic + q is q in two's complement)
__device__ __forceinline__ u32x2 pack_codes_i8(const float (&m)[8]) {
    uint32_t u[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = __float_as_uint(m[e]);
    return u32x2{pack_bytes(u[0], u[1], u[2], u[3]), pack_bytes(u[4], u[5], u[6], u[7])};
}
// INT4 codes of 8 elements as 4 bytes: two's-complement nibbles, even column in the low nibble
__device__ __forceinline__ uint32_t pack_codes_i4(const float (&m)[8]) {
    uint32_t u[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = __float_as_uint(m[e]);
    uint32_t w0 = pack_bytes(u[0], u[1], u[2], u[3]) & 0x0F0F0F0Fu;
    uint32_t w1 = pack_bytes(u[4], u[5], u[6], u[7]) & 0x0F0F0F0Fu;
    w0 |= w0 >> 4;                 // bytes 0 and 2 now hold two nibbles each
    w1 |= w1 >> 4;
    return __builtin_amdgcn_perm(w1, w0, 0x06040200u);
}
// dequantized values fl16(fl32(q * fl32(a * b))) of 8 elements as 16 bytes
__device__ __forceinline__ u32x4 pack_xhat(const float (&q)[8], float a, const float (&b)[8]) {
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = rounded_f32(q[e] * (a * b[e]));
    return u32x4{pack_half2(y[0], y[1]), pack_half2(y[2], y[3]), pack_half2(y[4], y[5]), pack_half2(y[6], y[7])};
}

// INT8 codes: 8 bytes at dst
__device__ __forceinline__ void store_codes_i8(const float (&m)[8], uint8_t* dst, bool vec_ok, int nvalid) {
    uint32_t u[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = __float_as_uint(m[e]);
    if (vec_ok && nvalid == 8) {
        store_through(pack_codes_i8(m), reinterpret_cast<u32x2*>(dst));
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < nvalid) dst[e] = (uint8_t)(u[e] & 0xFFu);
    }
}

// INT4 codes: 4 bytes at dst, two's-complement nibbles, even column in the low nibble
__device__ __forceinline__ void store_codes_i4(const float (&m)[8], uint8_t* dst, bool vec_ok, int nvalid) {
    uint32_t u[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = __float_as_uint(m[e]);
    uint32_t w0 = pack_bytes(u[0], u[1], u[2], u[3]) & 0x0F0F0F0Fu;
    uint32_t w1 = pack_bytes(u[4], u[5], u[6], u[7]) & 0x0F0F0F0Fu;
    w0 |= w0 >> 4;                 // bytes 0 and 2 now hold two nibbles each
    w1 |= w1 >> 4;
    const uint32_t w = __builtin_amdgcn_perm(w1, w0, 0x06040200u);
    if (vec_ok && nvalid == 8) {
        store_through(w, reinterpret_cast<uint32_t*>(dst));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (2 * e < nvalid) dst[e] = (uint8_t)((w >> (8 * e)) & 0xFFu);  // the channel count is even
    }
}

// INT4 codes as FP6 E2M3 fragments, the operand format of the A4W4 matrix kernel: a fragment is 32
// rows x 64 columns = 1536 bytes, fragments ordered [row / 32][column / 64]; fragment lane
// (row & 31) + 32 * ((column / 32) & 1) holds 32 consecutive columns as a 192-bit little-endian
// stream of 6-bit fields, its first 16 bytes at fragment + 16 * lane, the last 8 at fragment + 1024
// + 8 * lane.  The wave's lanes 4g .. 4g+3 hold the 32 columns of group g (8 each): their 48-bit
// pieces are gathered with three shuffles; lane 4g stores the 16 bytes, lane 4g+2 the 8 bytes.
// E2M3 of an integer 0..7 is the top of its binary32 pattern: (bits >> 20) - 0x3F0 (0 for 0).
// `group_ok`: the group's columns exist (I % 64 == 0: all or none).  frags_per_row = I / 64.
__device__ __forceinline__ void store_codes_fp6(const float (&m)[8], uint8_t* packed, int row, int first_col,
                                                int lane, int frags_per_row, bool group_ok) {
    uint32_t e[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float q = m[k] - kMagic;                                   // the code, exact
        const int mag = (int)(__float_as_uint(__builtin_fabsf(q)) >> 20) - 0x3F0;
        e[k] = (uint32_t)max(mag, 0) | (q < 0.0f ? 32u : 0u);
    }
    const uint32_t lo = e[0] | (e[1] << 6) | (e[2] << 12) | (e[3] << 18) | (e[4] << 24) | (e[5] << 30);
    const uint32_t hi = (e[5] >> 2) | (e[6] << 4) | (e[7] << 10);        // 16 bits
    const uint32_t lo1 = (uint32_t)__shfl_down((int)lo, 1, kLanes), hi1 = (uint32_t)__shfl_down((int)hi, 1, kLanes);
    const uint32_t lo2 = (uint32_t)__shfl_down((int)lo, 2, kLanes);
    const int q4 = lane & 3, g = lane >> 2;
    const int col = first_col + 32 * g;                                  // first column of the group
    const int64_t frag = (int64_t)(row >> 5) * frags_per_row + (col >> 6);
    const int flane = (row & 31) + 32 * ((col >> 5) & 1);
    uint8_t* f = packed + frag * 1536;
    // plain (cacheable) stores: a 128-byte line of a fragment is completed by 8 (or 16) different rows,
    // so the pieces have to meet in L2 before they leave for memory
    if (group_ok && q4 == 0)
        *reinterpret_cast<u32x4*>(f + flane * 16) = u32x4{lo, hi | (lo1 << 16), (lo1 >> 16) | (hi1 << 16), lo2};
    if (group_ok && q4 == 2)
        *reinterpret_cast<u32x2*>(f + 1024 + flane * 8) = u32x2{hi | (lo1 << 16), (lo1 >> 16) | (hi1 << 16)};
}

// The same fragments written four rows at a time (rows 4 k .. 4 k + 3 of one matrix, as the streaming kernel
// works on them): a lane keeps its 48 bits of each of the four rows, then the quad transposes them (two
// exchange steps of quad-permute register moves, no LDS) so that lane 4 g + u holds the whole 24-byte record of
// row u, and each lane stores one 16-byte and one 8-byte piece: a quad writes 64 and 32 contiguous bytes where
// the row-by-row form writes four scattered 16-byte and 8-byte pieces.
struct Fp6Batch {
    uint32_t lo[4], hi[4];      // this lane's fields of rows 0 .. 3: 32 + 16 bits each
};
template <int CTRL>
__device__ __forceinline__ uint32_t quad_permute(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, CTRL, 0xF, 0xF, true);
}
// r[k] = this lane's value of row k  ->  r[k] = the value lane k of the quad had for row (lane & 3)
__device__ __forceinline__ void quad_transpose(uint32_t (&r)[4], int lane) {
    const bool odd = lane & 1, up = lane & 2;
    // neighbours exchange: an even lane ends up with rows 0 and 2 of both lanes, an odd lane with rows 1 and 3
    const uint32_t g01 = quad_permute<0xB1>(odd ? r[0] : r[1]);         // lanes 1 0 3 2
    const uint32_t g23 = quad_permute<0xB1>(odd ? r[2] : r[3]);
    const uint32_t a01 = odd ? g01 : r[0], b01 = odd ? r[1] : g01;
    const uint32_t a23 = odd ? g23 : r[2], b23 = odd ? r[3] : g23;
    // pairs exchange: lanes 0, 1 give away their rows 2, 3 and lanes 2, 3 their rows 0, 1
    const uint32_t ga = quad_permute<0x4E>(up ? a01 : a23);             // lanes 2 3 0 1
    const uint32_t gb = quad_permute<0x4E>(up ? b01 : b23);
    r[0] = up ? ga : a01;
    r[1] = up ? gb : b01;
    r[2] = up ? a23 : ga;
    r[3] = up ? b23 : gb;
}
// Four INT4 codes (two's-complement bytes, -7 .. 7) -> their four E2M3 patterns packed into 24 bits.  Byte-wise:
// |q| = (q ^ mask) + sign bit with mask = 0xFF in negative bytes (no carry can cross a byte: |q| <= 7); the E2M3
// pattern of 0 .. 7 is one lookup in an 8-byte table (v_perm_b32 takes its selector bytes 0 .. 7 from the codes
// themselves); bit 5 is the sign.  Then the four 6-bit fields are squeezed together in two steps.
__device__ __forceinline__ uint32_t fp6_fields4(uint32_t w) {
    const uint32_t s = w & 0x80808080u;
    const uint32_t ones = s >> 7;
    const uint32_t mask = s | (s - ones);                               // 0xFF where negative
    const uint32_t mag = (w ^ mask) + ones;
    uint32_t e = __builtin_amdgcn_perm(0x1E1C1A18u, 0x14100800u, mag);  // 0 8 16 20 | 24 26 28 30
    e |= ones << 5;
    const uint32_t y = (e & 0x003F003Fu) | ((e & 0x3F003F00u) >> 2);    // two 12-bit fields in the half words
    return (y & 0xFFFu) | ((y >> 4) & 0xFFF000u);
}
// row u (0..3) of the batch: the lane's 8 codes as rounding-step values m
__device__ __forceinline__ void fp6_batch_row(Fp6Batch& out, const float (&m)[8], int u) {
    const u32x2 w = pack_codes_i8(m);
    const uint32_t f0 = fp6_fields4(w.x), f1 = fp6_fields4(w.y);        // 24 bits each
    out.lo[u] = f0 | (f1 << 24);
    out.hi[u] = f1 >> 8;                                                // 16 bits
}
// rows row4 .. row4 + 3 (row4 % 4 == 0); rows_ok: bit u set if row row4 + u exists; group_ok: the lane's columns exist.
// The four rows lie in one row of fragments, which is addressed as a raw buffer (frags_per_row * 1536 bytes).
// Must be called by the whole wave (the transposition exchanges registers between lanes).
__device__ __forceinline__ void fp6_batch_store(Fp6Batch& out, uint8_t* packed, int row4, int first_col, int lane,
                                                int frags_per_row, uint32_t rows_ok, bool group_ok) {
    quad_transpose(out.lo, lane);
    quad_transpose(out.hi, lane);
    // the group's 192-bit record of this lane's row: four lanes' 32 + 16 bits one after the other
    const uint32_t d1 = out.hi[0] | (out.lo[1] << 16), d2 = (out.lo[1] >> 16) | (out.hi[1] << 16);
    const uint32_t d4 = out.hi[2] | (out.lo[3] << 16), d5 = (out.lo[3] >> 16) | (out.hi[3] << 16);
    const int u = lane & 3, g = lane >> 2;
    const int col = first_col + 32 * g;
    const int flane = ((row4 + u) & 31) + 32 * ((col >> 5) & 1);
    const bool ok = group_ok && ((rows_ok >> u) & 1u);
    const rsrc_t frow = row_buffer(packed + (int64_t)(row4 >> 5) * frags_per_row * 1536, frags_per_row * 1536);
    // a lane that must not store points past the buffer's end: the hardware's range check drops its stores
    const int off = ok ? (col >> 6) * 1536 : 0x7FFF0000;
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{out.lo[0], d1, d2, out.lo[2]}, frow, off + flane * 16, 0, kWriteThrough);
    __builtin_amdgcn_raw_buffer_store_b64(u32x2{d4, d5}, frow, off + 1024 + flane * 8, 0, kWriteThrough);
}

// dequantized values fl16(fl32(q * fl32(a * b))): 16 bytes at dst
__device__ __forceinline__ void store_xhat(const float (&q)[8], float a, const float (&b)[8], uint16_t* dst,
                                           bool vec_ok, int nvalid) {
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = rounded_f32(q[e] * (a * b[e]));
    if (vec_ok && nvalid == 8) {
        store_through(u32x4{pack_half2(y[0], y[1]), pack_half2(y[2], y[3]), pack_half2(y[4], y[5]), pack_half2(y[6], y[7])},
                      reinterpret_cast<u32x4*>(dst));
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < nvalid) dst[e] = (uint16_t)f2h(y[e]);
    }
}

}  // namespace cq
