// Pieces shared by the matrix-core GEMM kernels (INT8 codes, and INT4 codes carried as FP6).
#pragma once
#include "cq_kernels.h"

namespace cq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

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

// Epilogue of the A4W4 kernel, which is on the 32 x 32 FP6 instruction.  Scaled binary16 results go through LDS
// (free once the K loop has ended on a barrier with no reads outstanding) so that every global store is a full
// 16 bytes per lane and a wave writes whole 128-byte row pieces.  row0 / col0: first token / channel of this wave.
// The accumulators are in the instruction's natural orientation (activation fragment as the first
// operand): lane l holds one output channel per 32 x 32 tile and, in register r of the tile, token
// 8 (r / 4) + 4 (l >> 5) + (r & 3).  The kernel assigns the rows of its NI weight fragments so that lane l's
// channels are NI consecutive ones, NI (l & 31) + ni: with NI = 2 a lane packs two binary16 results of one token
// into a word without any exchange between lanes.  A lane needs 64 different row factors; they go through a small
// wave-private piece of LDS behind the staging areas (each lane requests two of its wave's 128 before the last step
// of the contraction, stores them when the loop is over and reads them back four at a time).  Results are staged
// token row by token row (a half wave writes 128 or 64 contiguous bytes of one token) and leave as whole 128-byte
// pieces.
template <int NI>
struct EpilogueScalesRows {
    float a_own[2];        // row factors of tokens row0 + lane and row0 + 64 + lane
    float s[NI];           // column steps of channels col0 + NI (lane & 31) + ni
};
// SPLIT (NI = 2): the lane's two channels are (lane & 31) and 32 + (lane & 31) -- weight fragments of 32
// consecutive rows, as the FP6 operand format has them -- instead of two adjacent ones.
template <int NI, bool SPLIT = false>
__device__ __forceinline__ void epilogue_rows_load_scales(EpilogueScalesRows<NI>& sc, const float* __restrict__ row_scale,
                                                          const float* __restrict__ w_scale, int T, int O, int row0,
                                                          int col0, int lane) {
    sc.a_own[0] = row_scale[min(row0 + lane, T - 1)];                 // rows >= T are never stored
    sc.a_own[1] = row_scale[min(row0 + 64 + lane, T - 1)];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
        sc.s[ni] = w_scale[min(col0 + (SPLIT ? (lane & 31) + 32 * ni : NI * (lane & 31) + ni), O - 1)];
}

constexpr int epilogue_rows_pitch(int wtn) { return wtn * 2 + 16; }   // bytes per staged token row
// LDS the epilogue needs for n_waves waves of 128 x wtn outputs: staging areas, then 512 bytes of row factors per wave
constexpr int epilogue_rows_lds(int n_waves, int wtn) { return n_waves * (128 * epilogue_rows_pitch(wtn) + 512); }

// Second half of the epilogue: a wave reads its staged rows back and stores them as whole 16-byte pieces.
template <int WTN, bool SPLIT>
__device__ __forceinline__ void epilogue_rows_flush(const int8_t* stage, uint16_t* __restrict__ Y, int64_t ldy, int T, int O,
                                                    int row0, int col0, int lane, bool y_cached) {
    constexpr int kRowPitch = epilogue_rows_pitch(WTN);
    // each wave reads back only what it wrote itself: no barrier, just its own LDS writes done
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
    auto store16 = [&](int trow, int col, u32x4v v) {
        if (row0 + trow < T && col0 + col < O) {
            uint16_t* dst = Y + (int64_t)(row0 + trow) * ldy + col0 + col;
            // Y is not read again here and whole 128-byte pieces leave at once: written through to memory
            // as a stream (sc1 nt).  The GEMM itself does not care, but the memory-side cache is left
            // without 224 MiB of dirty lines, so the kernel that runs next reads its cold input faster
            // (64 MiB: 4 us less; of the policies tried -- plain, nt, sc1, sc1 nt, sc0 nt, sc0 sc1 nt --
            // this one gave the shortest following absmax + quantize calls).
            // (The compiler offers no way to ask for this policy, hence the assembly; it cannot see a
            // store in it, so the two wait states the hardware needs before the data registers of a
            // 16-byte store may be overwritten are added by hand.)
            // A small Y (see y_stays_cached) fits the memory-side cache next to everything else of its layer: plain
            // stores then, which make the kernel itself 2-3 % faster on such layers and change nothing after it.
            if (y_cached) *reinterpret_cast<u32x4v*>(dst) = v;
            else asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(dst), "v"(v) : "memory");
        }
    };
    if (SPLIT) {
        // a lane takes 8 words of a row (channels 8 p .. 8 p + 7 in the low halves, 32 + 8 p .. in the high halves)
        // and stores them as two 16-byte pieces
        const int p = lane & 3, rsub = lane >> 2;
#pragma unroll
        for (int i = 0; i < 128 / 16; ++i) {
            const int trow = i * 16 + rsub;
            const uint4 w0 = *reinterpret_cast<const uint4*>(stage + trow * kRowPitch + p * 32);
            const uint4 w1 = *reinterpret_cast<const uint4*>(stage + trow * kRowPitch + p * 32 + 16);
            auto lows = [](uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); };
            auto highs = [](uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); };
            store16(trow, 8 * p, u32x4v{lows(w0.x, w0.y), lows(w0.z, w0.w), lows(w1.x, w1.y), lows(w1.z, w1.w)});
            store16(trow, 32 + 8 * p, u32x4v{highs(w0.x, w0.y), highs(w0.z, w0.w), highs(w1.x, w1.y), highs(w1.z, w1.w)});
        }
    } else {
        constexpr int kLanesPerRow = WTN * 2 / 16;           // 16-byte pieces per staged row (8 or 4)
        constexpr int kRowsPerInst = 64 / kLanesPerRow;
        const int piece = lane % kLanesPerRow, rsub = lane / kLanesPerRow;
#pragma unroll
        for (int i = 0; i < 128 / kRowsPerInst; ++i) {
            const int trow = i * kRowsPerInst + rsub;
            const uint4 v = *reinterpret_cast<const uint4*>(stage + trow * kRowPitch + piece * 16);
            store16(trow, piece * 8, u32x4v{v.x, v.y, v.z, v.w});
        }
    }
}

template <typename ACC, int WTN, int NI, int NWAVES, bool SPLIT = false>
__device__ __forceinline__ void epilogue_rows_store(ACC (&acc)[4][NI], int8_t* lds, const EpilogueScalesRows<NI>& sc,
                                                    uint16_t* __restrict__ Y, int64_t ldy,
                                                    int32_t* __restrict__ acc_debug, int T, int O, int row0, int col0,
                                                    int lane, int wave, bool y_cached) {
    static_assert(NI == 1 || NI == 2, "one or two channels per lane");
    static_assert(!SPLIT || (NI == 2 && WTN == 64), "the split form is the 128 x 64 wave tile");
    constexpr int kRowPitch = epilogue_rows_pitch(WTN);
    int8_t* stage = lds + wave * (128 * kRowPitch);
    float* a_lds = reinterpret_cast<float*>(lds + NWAVES * (128 * kRowPitch) + wave * 512);
    const int frag_half = lane >> 5, ch = lane & 31;
    a_lds[lane] = sc.a_own[0];
    a_lds[64 + lane] = sc.a_own[1];
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));      // wave-private: the writes above are done
    // SPLIT: word ch of a staged row holds channels ch and 32 + ch; they are taken apart again on the way out
    const int o_loc = SPLIT ? ch : NI * ch;              // first of this lane's NI channels
    const bool o_ok = col0 + o_loc < O;                  // O % 8 == 0 on this path: adjacent channels exist or not together
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        float4 a4[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) a4[g] = *reinterpret_cast<const float4*>(a_lds + mi * 32 + 8 * g + 4 * frag_half);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float av[4] = {a4[g].x, a4[g].y, a4[g].z, a4[g].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t_loc = mi * 32 + 8 * g + 4 * frag_half + j;
                float y[NI];
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    y[ni] = (float)acc[mi][ni][4 * g + j] * av[j];
                    y[ni] = rounded_f32(y[ni] * sc.s[ni]);
                }
                int8_t* dst = stage + t_loc * kRowPitch + (SPLIT ? ch * 4 : o_loc * 2);
                if (NI == 2) *reinterpret_cast<uint32_t*>(dst) = pack_half2(y[0], y[NI - 1]);   // one conversion for the pair
                else *reinterpret_cast<uint16_t*>(dst) = (uint16_t)f2h(y[0]);
                if (acc_debug && row0 + t_loc < T && o_ok) {
                    int32_t* d = acc_debug + (int64_t)(row0 + t_loc) * O + col0 + o_loc;
                    if (SPLIT) {
                        d[0] = (int)acc[mi][0][4 * g + j];
                        if (col0 + o_loc + 32 < O) d[32] = (int)acc[mi][NI - 1][4 * g + j];
                    } else if (NI == 2) {
                        *reinterpret_cast<int2*>(d) = make_int2((int)acc[mi][0][4 * g + j], (int)acc[mi][NI - 1][4 * g + j]);
                    } else {
                        *d = (int)acc[mi][0][4 * g + j];
                    }
                }
            }
        }
    }
    epilogue_rows_flush<WTN, SPLIT>(stage, Y, ldy, T, O, row0, col0, lane, y_cached);
}

// ---- Epilogue for the 16 x 16 x 64 instruction (INT8 kernel): lane l holds channel l & 15 of each 16 x 16 tile and,
// in register r, token 4 (l >> 4) + r.  The kernel assigns the rows of its G weight tiles so that lane l's channels
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
template <int WTN, int G, bool DEBUG, bool STREAM>
__device__ __forceinline__ void epilogue16_store(v4i (&acc)[8][G], float* a_lds, const EpilogueScales16<G>& sc,
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
                    if (G == 4)
                        *reinterpret_cast<int4*>(d) = make_int4(acc[mi][0][r], acc[mi][1][r], acc[mi][G - 2][r], acc[mi][G - 1][r]);
                    else
                        *reinterpret_cast<int2*>(d) = make_int2(acc[mi][0][r], acc[mi][1][r]);
                }
            }
        }
    }
}

}  // namespace
}  // namespace cq
