// Pieces shared by the matrix-core GEMM kernels (INT8 codes, and INT4 codes carried as FP6).
#pragma once
#include "cq_kernels.h"

namespace cq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int BM = 256, BN = 256;   // block tile (tokens x output channels)
constexpr int kXcds = 8;            // block ids are dealt round-robin to this many L2 domains
constexpr int kGroupM = 4;          // tile-rows walked together (8, 16 and 1 measured slower)

// s_waitcnt immediate for gfx9-family encodings: vmcnt in bits 3:0 and 15:14, expcnt 6:4 (7 = no
// wait), lgkmcnt 11:8 (15 = no wait)
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 0xF) | ((vm >> 4) << 14) | (7 << 4) | (lgkm << 8); }

// Block id -> output tile.  Consecutive block ids land on different XCDs, so ids are first
// de-interleaved by XCD (each XCD gets a contiguous range of tiles, hence its own L2 sees a compact
// patch), then walked in groups of kGroupM tile-rows so that concurrently resident tiles share A
// rows and B columns.  Returns false for the padding blocks of the last XCD range.
// position L of the walk -> tile
__device__ __forceinline__ void tile_of_index(int L, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    const int group_sz = kGroupM * tiles_n;
    const int g = L / group_sz;
    const int gm = min(kGroupM, tiles_m - g * kGroupM);
    const int in_g = L - g * group_sz;
    tile_m = g * kGroupM + in_g % gm;
    tile_n = in_g / gm;
}
__device__ __forceinline__ bool tile_of_block(int block, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const int L = (block % kXcds) * per_xcd + block / kXcds;
    if (L >= total) return false;
    tile_of_index(L, tiles_m, tiles_n, tile_m, tile_n);
    return true;
}

// Store policy of Y: up to 64 MiB it is written with plain stores, beyond that written through as a stream (see
// epilogue_rows_store).  Measured in a layer step: 2048 x 11008 outputs (43 MiB) 84.1 -> 82.5 us for the matrix
// kernel with plain stores and no change after it; 4096 x 20480 (160 MiB) and 4096 x 28672 (224 MiB) make the
// absmax call that follows 1.5 and 6 us slower with plain stores.
inline bool y_stays_cached(int T, int O) { return (int64_t)T * O * 2 <= (int64_t)64 << 20; }

// ---- Epilogue of the ring kernels, whose accumulator tiles are 16 x 16 (v_mfma_i32_16x16x64_i8 for INT8 codes,
// v_mfma_f32_16x16x128_f8f6f4 for INT4 codes carried as FP6; row0 / col0: first token / channel of the wave): lane l
// holds channel l & 15 of each tile and, in register r, token 4 (l >> 4) + r.  The kernel assigns the rows of its G weight tiles so that lane l's channels
// are the G consecutive ones G (l & 15) + ni: the G binary16 results of one token are 2 G adjacent bytes of Y, the
// 16 lanes of a group cover 32 G contiguous bytes of a token row (whole 128-byte lines for G = 4), and they are
// stored straight from registers, with no pass through LDS.  The wave's outputs are addressed as one raw buffer that
// ends with the last valid element, so the hardware's range check drops the rows past T; a lane whose channels lie
// past O gets an offset beyond any buffer.  No store is predicated: a wave always issues exactly 32 of them, which
// the kernel's hand-counted waits rely on.
// A lane needs the row factors of 4 consecutive tokens at a time; they go through 512 bytes of wave-private LDS
// (each lane requests two of its wave's 128 before the last step of the contraction).
template <int G>
struct EpilogueScales16 {
    float a_own[2];        // row factors of tokens row0 + lane and row0 + 64 + lane
    float s[G];            // column steps of channels col0 + G (lane & 15) + ni
};
template <int G>
__device__ __forceinline__ void epilogue16_load_scales(EpilogueScales16<G>& sc, const float* __restrict__ row_scale,
                                                       const float* __restrict__ w_scale, int T, int O, int row0, int col0,
                                                       int lane) {
    sc.a_own[0] = row_scale[min(row0 + lane, T - 1)];                 // rows >= T are never stored
    sc.a_own[1] = row_scale[min(row0 + 64 + lane, T - 1)];
#pragma unroll
    for (int ni = 0; ni < G; ++ni) sc.s[ni] = w_scale[min(col0 + G * (lane & 15) + ni, O - 1)];
}

constexpr int kEpilogue16Stores = 32;     // buffer stores per wave and tile (8 accumulator tiles x 4 registers)

// STREAM: Y is written through to memory as a stream (sc1 nt).  It is not read again here, and the memory-side cache
// is left without hundreds of MiB of dirty lines, so the kernel that runs next reads its cold input faster (64 MiB:
// 4 us less; of the policies tried -- plain, nt, sc1, sc1 nt, sc0 nt, sc0 sc1 nt -- this one gave the shortest
// following absmax + quantize calls).  A small Y (see y_stays_cached) fits the memory-side cache next to everything
// else of its layer: plain stores then, which make the kernel itself 2-3 % faster on such layers and change nothing
// after it.  DEBUG: the raw accumulators are stored as well (predicated stores; no fixed count then).
template <int WTN, int G, bool DEBUG, bool STREAM, typename ACC>
__device__ __forceinline__ void epilogue16_store(ACC (&acc)[8][G], float* a_lds, const EpilogueScales16<G>& sc,
                                                 uint16_t* __restrict__ Y, int64_t ldy, int32_t* __restrict__ acc_debug,
                                                 int T, int O, int row0, int col0, int lane) {
    static_assert(G == 2 || G == 4, "two or four channels per lane");
    static_assert(WTN == 16 * G, "G tiles of 16 channels");
    constexpr int kPolicy = STREAM ? 18 : 0;             // sc1 (16) | nt (2)
    const int fr = lane & 15, grp = lane >> 4;
    a_lds[lane] = sc.a_own[0];
    a_lds[64 + lane] = sc.a_own[1];
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));      // wave-private: the writes above are done
    const int o_loc = G * fr;                            // first of this lane's G channels
    // the wave's 128 x WTN outputs as a buffer: rows [row0, T) and channels [col0, O) of them exist
    const int n_rows = min(128, T - row0), n_cols = min(WTN, O - col0);
    const int pitch = (int)ldy * 2;                      // bytes; 128 rows of it stay below 2^31 (checked by the launcher)
    const int bytes = (n_rows > 0 && n_cols > 0) ? (n_rows - 1) * pitch + n_cols * 2 : 0;
    const __amdgpu_buffer_rsrc_t yb =
        __builtin_amdgcn_make_buffer_rsrc(Y + (int64_t)row0 * ldy + col0, 0, bytes, 0x00020000);   // raw, 32-bit data
    // O % 8 == 0 on this path: a lane's G channels exist or not together
    const bool o_ok = o_loc < n_cols;
    const uint32_t lane_off = o_ok ? (uint32_t)(4 * grp * pitch + o_loc * 2) : 0x80000000u;
#pragma unroll
    for (int mi = 0; mi < 8; ++mi) {
        const float4 a4 = *reinterpret_cast<const float4*>(a_lds + 16 * mi + 4 * grp);
        const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float y[G];
#pragma unroll
            for (int ni = 0; ni < G; ++ni) {
                y[ni] = (float)acc[mi][ni][r] * av[r];
                y[ni] = rounded_f32(y[ni] * sc.s[ni]);
            }
            const int off = (int)(lane_off + (uint32_t)((16 * mi + r) * pitch));
            if (G == 4) {
                typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
                __builtin_amdgcn_raw_buffer_store_b64(u32x2v{pack_half2(y[0], y[1]), pack_half2(y[G - 2], y[G - 1])}, yb, off, 0,
                                                      kPolicy);
            } else {
                __builtin_amdgcn_raw_buffer_store_b32(pack_half2(y[0], y[1]), yb, off, 0, kPolicy);
            }
            if (DEBUG) {
                const int t_loc = 16 * mi + 4 * grp + r;
                if (row0 + t_loc < T && o_ok) {
                    int32_t* d = acc_debug + (int64_t)(row0 + t_loc) * O + col0 + o_loc;
                    // (binary32 accumulators of the FP6 kernel hold exact integers)
                    if (G == 4)
                        *reinterpret_cast<int4*>(d) = make_int4((int)acc[mi][0][r], (int)acc[mi][1][r], (int)acc[mi][G - 2][r],
                                                                (int)acc[mi][G - 1][r]);
                    else
                        *reinterpret_cast<int2*>(d) = make_int2((int)acc[mi][0][r], (int)acc[mi][1][r]);
                }
            }
        }
    }
}

}  // namespace
}  // namespace cq
