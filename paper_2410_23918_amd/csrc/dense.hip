// The materialising path (the appendix on inference throughput, "level 2"): the weight of the
// loaded prefix is restored once per call to a dense fp16 matrix
//
//     Wd[o][j] = ( sum_i S_i[o][j] * (U_i V_i^T)[o][j] ) / s[j]        (Eq. 8, Eq. 4 folded into the columns)
//
// in caller-owned memory (k_tile<true> in panel.hip), and the batch then meets it in one dense
// product Y = X Wd^T on the matrix cores (k_gemm below).  Restoring costs the same per weight
// element whatever the batch, so for prefill-sized batches this beats rebuilding weight tiles per
// token tile; the price is out x in x 2 bytes of scratch, shared by all stacks of a model.
//
// k_gemm: one workgroup (8 wavefronts, two per SIMD) owns 256 output rows x 256 tokens and walks
// the input columns in chunks of 64.  Both operand chunks (256 x 64 each, rows of the dense weight
// and rows of x as they lie in memory) go through LDS, double buffered; every thread requests its
// eight 16-byte pieces of a chunk two chunks before they are written to LDS, so all global loads
// of a wavefront have the same, long time to arrive (loads return in order: one late load would
// hold up every younger one).  A wavefront owns 128 rows x 64 tokens: per step of 16 columns it
// reads four weight and two activation fragments from LDS (rows padded by 16 bytes, conflict-free
// 128-bit reads) and issues eight v_mfma_f32_32x32x16_f16; the other wavefront of the SIMD covers
// the read latency.  One LDS-only barrier per chunk.  The fp16 output tile is turned in LDS and
// leaves in 16-byte pieces.  Workgroup ids map to tiles so that all token tiles of a row tile run
// on one XCD (one L2 pulls that part of the weight).  Two more instantiations, with tiles of 128
// rows x 256 tokens and of 128 x 128, fill the chip for shapes with few tiles (row slabs, small
// batches; chosen per launch on the host).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "kparams.h"
#include "layout.h"

namespace bitstack {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kGemmRows = 256;              // output rows per workgroup (128 in the narrow variant)
constexpr int kGemmTokens = 256;            // tokens per workgroup
constexpr int kGemmKc = 64;                 // input columns per chunk
constexpr int kGemmLd = kGemmKc + 8;        // fp16 per LDS row (+8: bank spread for 128-bit reads)
constexpr int kGemmTile = 256 * kGemmLd;    // fp16 per operand tile
constexpr int kGemmLds = 2 * 2 * kGemmTile * 2;   // bytes: two buffers x {weight tile, activation tile}
constexpr int kGemmYLd = 256 + 8;           // fp16 per LDS row of the output tile
static_assert(256 * kGemmYLd * 2 <= kGemmLds, "the output tile reuses the operand buffers");
constexpr int kGemmLdsSmall = kGemmLds / 2;       // the 128 x 128 variant: half-height tiles
static_assert(128 * kGemmYLd * 2 <= kGemmLdsSmall && 4 * 64 * 64 * 4 <= kGemmLdsSmall,
              "its output tile and the exchange of the column halves reuse the operand buffers");

__global__ __launch_bounds__(256) void k_dense_zero(uint4* w, size_t n16) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i < n16) w[i] = make_uint4(0, 0, 0, 0);
}

// RJ: 32-row fragments per wavefront.  4: the 256-row tile described above.  2: a 128-row tile
// (wavefront tile 64 rows x 64 tokens, four matrix instructions per step), for shapes whose
// 256-row tiles would leave half of the compute units without a workgroup.
// KSPLIT (with RJ = 2): a tile of 128 rows x 128 tokens for products too small to fill the chip
// with the wider tiles (a slab of 2048 rows x 2048 tokens is 256 of these).  The wavefront tile
// stays 64 x 64 (one LDS fragment per matrix instruction, as in the 128-row variant): wavefronts
// 0-3 take the first 32 columns of every chunk, wavefronts 4-7 the other 32, and the two halves
// are added through LDS after the loop.
template <int RJ, bool KSPLIT>
__global__ __launch_bounds__(512, KSPLIT ? 4 : 1) void k_gemm(KParams p) {
    static_assert(!KSPLIT || RJ == 2, "the 128 x 128 tile is built from 64 x 64 wavefront tiles");
    constexpr int ROWS = KSPLIT ? 128 : 64 * RJ;
    constexpr int TOKS = KSPLIT ? 128 : kGemmTokens;
    constexpr int STEPS = KSPLIT ? 2 : 4;   // 16-column steps of a chunk per wavefront
    // fp16 per operand tile in LDS: 128 rows in the 128 x 128 variant, so that two of its workgroups
    // (74 KB each, at most 128 registers per lane) fit a compute unit
    constexpr int TILE = (KSPLIT ? 128 : 256) * kGemmLd;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* const wl = reinterpret_cast<_Float16*>(smem);   // [buffer][256 rows][kGemmLd]
    _Float16* const xl = wl + 2 * TILE;                        // [buffer][256 tokens][kGemmLd]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hl = lane >> 5, ln = lane & 31;
    // my 64 tokens and 32 RJ rows inside the workgroup's tile (and, KSPLIT, my half of every chunk)
    const int tg = KSPLIT ? (wave & 1) : (wave & 3), rg = KSPLIT ? ((wave >> 1) & 1) : (wave >> 2);
    const int kh = KSPLIT ? (wave >> 2) : 0;

    // Workgroup ids are dealt round-robin to the 8 XCDs: all token tiles of a row tile go to one
    // XCD, so that a weight tile is pulled into one L2 only.
    const int ntt = (p.batch + TOKS - 1) / TOKS, nrt = (p.out + ROWS - 1) / ROWS;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rt = xcd + 8 * (slot / ntt), tt = slot % ntt;
    if (rt >= nrt) return;
    const int row0 = rt * ROWS, tok0 = tt * TOKS;
    const int nkc = p.in / kGemmKc;   // a multiple of 4

    // both tiles of a chunk: thread (row tid/8 + 64 i, 16-byte piece tid%8), i = 0..3 (weight
    // rows: i < RJ; tokens: i < 2 in the 128-token tile); rows and tokens past the end repeat the
    // last one (computed, never stored)
    const unsigned char* const wbase = reinterpret_cast<const unsigned char*>(p.wdense);
    const unsigned char* const xbase = reinterpret_cast<const unsigned char*>(p.x);
    // (scalar variables and macros on purpose: arrays or structs of 128 bytes of load results
    // are left in scratch memory by the compiler here)
    auto off_of = [&](int first, int i, int limit) -> unsigned {
        return unsigned((size_t(min(first + (tid >> 3) + 64 * i, limit - 1)) * p.in + (tid & 7) * 8) * 2);
    };
    const unsigned wo0 = off_of(row0, 0, p.out), wo1 = off_of(row0, 1, p.out), wo2 = off_of(row0, 2, p.out),
                   wo3 = off_of(row0, 3, p.out);
    const unsigned xo0 = off_of(tok0, 0, p.batch), xo1 = off_of(tok0, 1, p.batch), xo2 = off_of(tok0, 2, p.batch),
                   xo3 = off_of(tok0, 3, p.batch);
    const int dst = (tid >> 3) * kGemmLd + (tid & 7) * 8;
    auto ld16 = [&](const unsigned char* base, unsigned off) -> uint4 {
        return *reinterpret_cast<const uint4*>(base + off);
    };
    auto st16 = [&](_Float16* tile, int buf, int i, uint4 v) {
        *reinterpret_cast<uint4*>(tile + buf * TILE + dst + 64 * i * kGemmLd) = v;
    };
#define BS_GEMM_LOAD(S, KC)                                                                \
    {                                                                                      \
        const unsigned c = unsigned(min((KC), nkc - 1)) * (kGemmKc * 2);                   \
        w##S##0 = ld16(wbase, wo0 + c);                                                    \
        w##S##1 = ld16(wbase, wo1 + c);                                                    \
        if constexpr (RJ == 4) {                                                           \
            w##S##2 = ld16(wbase, wo2 + c);                                                \
            w##S##3 = ld16(wbase, wo3 + c);                                                \
        }                                                                                  \
        x##S##0 = ld16(xbase, xo0 + c);                                                    \
        x##S##1 = ld16(xbase, xo1 + c);                                                    \
        if constexpr (!KSPLIT) {                                                           \
            x##S##2 = ld16(xbase, xo2 + c);                                                \
            x##S##3 = ld16(xbase, xo3 + c);                                                \
        }                                                                                  \
    }
#define BS_GEMM_WRITE(S, BUF)                                                              \
    {                                                                                      \
        st16(wl, BUF, 0, w##S##0);                                                         \
        st16(wl, BUF, 1, w##S##1);                                                         \
        if constexpr (RJ == 4) {                                                           \
            st16(wl, BUF, 2, w##S##2);                                                     \
            st16(wl, BUF, 3, w##S##3);                                                     \
        }                                                                                  \
        st16(xl, BUF, 0, x##S##0);                                                         \
        st16(xl, BUF, 1, x##S##1);                                                         \
        if constexpr (!KSPLIT) {                                                           \
            st16(xl, BUF, 2, x##S##2);                                                     \
            st16(xl, BUF, 3, x##S##3);                                                     \
        }                                                                                  \
    }
    // fragments of step s (16 columns) of the chunk in buffer buf: weight rows j*32.., tokens t*32..
    const _Float16* const wfr = wl + (rg * (32 * RJ) + ln) * kGemmLd + 8 * hl + kh * 32;
    const _Float16* const xfr = xl + (tg * 64 + ln) * kGemmLd + 8 * hl + kh * 32;
    auto wfrag = [&](int buf, int s, int j) -> v8h {
        return *reinterpret_cast<const v8h*>(wfr + buf * TILE + j * 32 * kGemmLd + s * 16);
    };
    auto xfrag = [&](int buf, int s, int t) -> v8h {
        return *reinterpret_cast<const v8h*>(xfr + buf * TILE + t * 32 * kGemmLd + s * 16);
    };

    v16f acc[RJ][2];   // [row fragment][token group]
#pragma unroll
    for (int j = 0; j < RJ; ++j)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][t][v] = 0.0f;

    uint4 wA0, wA1, wA2 = {}, wA3 = {}, xA0, xA1, xA2 = {}, xA3 = {}, wB0, wB1, wB2 = {}, wB3 = {}, xB0, xB1, xB2 = {}, xB3 = {};
    BS_GEMM_LOAD(A, 0)
    BS_GEMM_LOAD(B, 1)
    BS_GEMM_WRITE(A, 0)
    BS_GEMM_LOAD(A, 2)
    lds_barrier();

    // The 128 x 256 tile has registers to spare (165 of 256): its fragments are read one step ahead of
    // their use.  The other two tiles would spill with that (256 / 128 registers, 56 / 76 bytes of
    // scratch: 8 % and 2x slower), so they read a step's fragments at its start.
    constexpr bool kAhead = RJ == 2 && !KSPLIT;
    // One chunk from buffer BUF: at step 1 the chunk after it (already in registers T) goes to the
    // other buffer and the chunk two further on is requested, so every global load has two chunks
    // to arrive.  The barrier at the end makes the other buffer readable and protects this one
    // from the writes of the chunk after next.  Fragments are read at the start of their step;
    // the second wavefront of the SIMD covers that latency.
#define BS_GEMM_CHUNK(KC, BUF, S)                                                          \
    {                                                                                      \
        v8h bn[RJ], an[2];                                                                 \
        if constexpr (kAhead) {                                                            \
            _Pragma("unroll") for (int j = 0; j < RJ; ++j) bn[j] = wfrag(BUF, 0, j);       \
            _Pragma("unroll") for (int t = 0; t < 2; ++t) an[t] = xfrag(BUF, 0, t);        \
        }                                                                                  \
        _Pragma("unroll") for (int s = 0; s < STEPS; ++s) {                                \
            if (s == 1) {                                                                  \
                BS_GEMM_WRITE(S, (BUF) ^ 1)                                                \
                BS_GEMM_LOAD(S, (KC) + 3)                                                  \
            }                                                                              \
            v8h b[RJ], a[2];                                                               \
            if constexpr (kAhead) {                                                        \
                _Pragma("unroll") for (int j = 0; j < RJ; ++j) b[j] = bn[j];               \
                _Pragma("unroll") for (int t = 0; t < 2; ++t) a[t] = an[t];                \
                if (s + 1 < STEPS) {                                                       \
                    _Pragma("unroll") for (int j = 0; j < RJ; ++j) bn[j] = wfrag(BUF, s + 1, j); \
                    _Pragma("unroll") for (int t = 0; t < 2; ++t) an[t] = xfrag(BUF, s + 1, t);  \
                }                                                                          \
            } else {                                                                       \
                _Pragma("unroll") for (int j = 0; j < RJ; ++j) b[j] = wfrag(BUF, s, j);    \
                _Pragma("unroll") for (int t = 0; t < 2; ++t) a[t] = xfrag(BUF, s, t);     \
            }                                                                              \
            __builtin_amdgcn_sched_barrier(0); /* requests before the step's arithmetic */ \
            _Pragma("unroll") for (int j = 0; j < RJ; ++j) {                               \
                acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0], b[j], acc[j][0], 0, 0, 0); \
                acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1], b[j], acc[j][1], 0, 0, 0); \
            }                                                                              \
            __builtin_amdgcn_sched_barrier(0);                                             \
        }                                                                                  \
        lds_barrier();                                                                     \
    }
    for (int kc = 0; kc < nkc; kc += 2) {
        BS_GEMM_CHUNK(kc, 0, B)
        BS_GEMM_CHUNK(kc + 1, 1, A)
    }
#undef BS_GEMM_CHUNK
#undef BS_GEMM_LOAD
#undef BS_GEMM_WRITE

    if constexpr (KSPLIT) {
        // the two column halves meet: wavefronts 4-7 park their tiles in LDS (the operand buffers are
        // free: the loop's last barrier has passed), wavefronts 0-3 add them to theirs
        float* const red = reinterpret_cast<float*>(smem) + (wave & 3) * (64 * 64) + lane;   // [4][64 registers][64 lanes]
        if (kh == 1) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) red[((j * 2 + t) * 16 + v) * 64] = acc[j][t][v];
        }
        lds_barrier();
        if (kh == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[j][t][v] += red[((j * 2 + t) * 16 + v) * 64];
        }
        lds_barrier();   // read before the output tile below overwrites it
    }
    const bool owner = kh == 0;   // wavefronts that hold finished sums
    // C[i = token][n = row]: lane (row ln), register v holds token 8*(v/4) + 4*hl + v%4 of the group
    if (p.y_f32) {
        if (!owner) return;
#pragma unroll
        for (int j = 0; j < RJ; ++j)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tok = tok0 + tg * 64 + t * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                    const int row = row0 + rg * (32 * RJ) + j * 32 + ln;
                    if (tok < p.batch && row < p.out) static_cast<float*>(p.y)[size_t(tok) * p.y_ld + row] = acc[j][t][v];
                }
        return;
    }
    // fp16 output: the tile is turned in LDS (the operand buffers are free now; the loop's last
    // barrier has passed) so that it leaves in 16-byte pieces, 2 ROWS contiguous bytes per token,
    // instead of 2-byte pieces
    _Float16* const yl = reinterpret_cast<_Float16*>(smem);   // [TOKS tokens][kGemmYLd]
    if (owner) {
#pragma unroll
        for (int j = 0; j < RJ; ++j)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    yl[(tg * 64 + t * 32 + 8 * (v >> 2) + 4 * hl + (v & 3)) * kGemmYLd + rg * (32 * RJ) + j * 32 + ln] =
                        _Float16(acc[j][t][v]);
    }
    lds_barrier();
    __half* const y = static_cast<__half*>(p.y);
    constexpr int PIECES = ROWS / 8;   // 16-byte pieces per token
#pragma unroll 4
    for (int k = 0; k < TOKS * PIECES / 512; ++k) {
        const int idx = tid + 512 * k, tok = idx / PIECES, piece = idx % PIECES;
        const uint4 v = *reinterpret_cast<const uint4*>(yl + tok * kGemmYLd + piece * 8);
        if (tok0 + tok < p.batch && row0 + piece * 8 < p.out)
            *reinterpret_cast<uint4*>(y + size_t(tok0 + tok) * p.y_ld + row0 + piece * 8) = v;
    }
}

hipError_t launch_dense_zero(const LaunchArgs& a, hipStream_t st) {
    const size_t n16 = size_t(a.geo.out) * size_t(a.geo.in) * 2 / 16;
    hipLaunchKernelGGL(k_dense_zero, dim3(unsigned((n16 + 255) / 256)), dim3(256), 0, st,
                       static_cast<uint4*>(a.wdense), n16);
    return hipGetLastError();
}

// Cost model of the product (microseconds, fitted to measurements): a round of workgroups takes
// in x (a + b x the fraction of the 256 compute units that have a workgroup) - a partly filled
// chip runs each tile faster (clock, shared caches) - with (a, b) = (0.0196, 0.0148) for 256-row
// tiles, (0.0111, 0.0089) for 128-row tiles and (0.0068, 0.0032) for 128 x 128 tiles.  The
// launcher takes the cheapest tile.
enum GemmTile { kTile256 = 1, kTile128 = 2, kTile128x128 = 3 };
static std::atomic<int> g_forced_tile{0};   // measurement hook: 0 = the estimate's choice
void dense_force_tile(int tile) { g_forced_tile = tile; }

static double tile_rounds_time_us(int out, int in, int batch, int tile) {
    const int rows = tile == kTile256 ? 256 : 128, toks = tile == kTile128x128 ? 128 : kGemmTokens;
    const int tiles = ((out + rows - 1) / rows) * ((batch + toks - 1) / toks);
    const double a = tile == kTile256 ? 0.0196 : tile == kTile128 ? 0.0111 : 0.0068;
    const double b = tile == kTile256 ? 0.0148 : tile == kTile128 ? 0.0089 : 0.0032;
    const int full = tiles / 256, rest = tiles % 256;
    return in * (full * (a + b) + (rest ? a + b * rest / 256.0 : 0.0));
}
static int dense_tile(int out, int in, int batch) {
    const int forced = g_forced_tile.load();
    if (forced >= kTile256 && forced <= kTile128x128) return forced;
    int best = kTile256;
    for (int t = kTile128; t <= kTile128x128; ++t)
        if (tile_rounds_time_us(out, in, batch, t) < tile_rounds_time_us(out, in, batch, best)) best = t;
    return best;
}
double dense_time_us(int out, int in, int batch) {
    // never below one pass over both operands at ~3.5 TB/s (few tokens: every tile reads its own rows
    // of the weight once and nothing is reused)
    const double t = tile_rounds_time_us(out, in, batch, dense_tile(out, in, batch));
    const double stream = (double(out) + batch) * in * 2.0 / 3.5e6;
    return t > stream ? t : stream;
}

hipError_t launch_dense(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    if (a.batch < 1 || p.wdense == nullptr) return hipErrorInvalidValue;
    if (a.rows) {
        // a slab of rows: the dense matrix holds rows [row_begin, row_begin + rows) of the weight, the
        // outputs go to the same columns of y (whose token rows stay the stack's full width apart)
        if (a.row_begin % 256 || a.row_begin < 0 || a.row_begin >= a.geo.out) return hipErrorInvalidValue;
        p.out = a.rows < a.geo.out - a.row_begin ? a.rows : a.geo.out - a.row_begin;
        p.y = static_cast<unsigned char*>(p.y) + size_t(a.row_begin) * (a.y_f32 ? 4 : 2);
    }
    if (size_t(p.batch) * p.in * 2 > 0xffffffffull || size_t(p.out) * p.in * 2 > 0xffffffffull)
        return hipErrorInvalidValue;   // 32-bit byte offsets into x and the dense weight
    static std::atomic<bool> attr_set{false};   // setting the attribute twice is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<4, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<2, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<2, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsSmall);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tile = dense_tile(p.out, p.in, p.batch);
    const int rows = tile == kTile256 ? 256 : 128, toks = tile == kTile128x128 ? 128 : kGemmTokens;
    const int ntt = (p.batch + toks - 1) / toks, nrt = (p.out + rows - 1) / rows;
    const unsigned wgs = unsigned(8 * ((nrt + 7) / 8) * ntt);
    if (tile == kTile128x128)
        hipLaunchKernelGGL((k_gemm<2, true>), dim3(wgs), dim3(512), kGemmLdsSmall, st, p);
    else if (tile == kTile128)
        hipLaunchKernelGGL((k_gemm<2, false>), dim3(wgs), dim3(512), kGemmLds, st, p);
    else
        hipLaunchKernelGGL((k_gemm<4, false>), dim3(wgs), dim3(512), kGemmLds, st, p);
    return hipGetLastError();
}

}  // namespace bitstack
