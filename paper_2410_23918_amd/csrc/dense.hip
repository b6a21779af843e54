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
// k_gemm: one workgroup (8 wavefronts) owns 256 output rows x 256 tokens and walks the input
// columns in chunks of 64.  The weight chunk (256 x 64) goes through LDS, double buffered, loaded
// two chunks ahead into registers; the activations come straight from memory in fragment order
// (k_xpack), requested four steps ahead.  A wavefront owns 128 rows x 64 tokens: per step of 16
// columns it reads four weight fragments from LDS and two activation fragments from its ring and
// issues eight v_mfma_f32_32x32x16_f16.  One LDS-only barrier per chunk.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "kparams.h"
#include "layout.h"

namespace bitstack {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kGemmRows = 256;              // output rows per workgroup
constexpr int kGemmTokens = 256;            // tokens per workgroup
constexpr int kGemmKc = 64;                 // input columns per chunk
constexpr int kGemmLd = kGemmKc + 8;        // fp16 per LDS row (+8: bank spread for 128-bit reads)
constexpr int kGemmBuf = kGemmRows * kGemmLd;   // fp16 per buffer
constexpr int kGemmLds = 2 * kGemmBuf * 2;  // bytes
constexpr int kGemmPd = 4;                  // activation fragments are requested this many steps ahead

__global__ __launch_bounds__(256) void k_dense_zero(uint4* w, size_t n16) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i < n16) w[i] = make_uint4(0, 0, 0, 0);
}

__global__ __launch_bounds__(512) void k_gemm(KParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* const wl = reinterpret_cast<_Float16*>(smem);   // [2][256][kGemmLd]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hl = lane >> 5, ln = lane & 31;
    const int tg = wave & 3, rg = wave >> 2;   // my 64 tokens and 128 rows inside the workgroup's tile

    // Workgroup ids are dealt round-robin to the 8 XCDs: all token tiles of a row tile go to one
    // XCD, so that a weight tile is pulled into one L2 only.
    const int ntt = (p.batch + kGemmTokens - 1) / kGemmTokens, nrt = (p.out + kGemmRows - 1) / kGemmRows;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rt = xcd + 8 * (slot / ntt), tt = slot % ntt;
    if (rt >= nrt) return;
    const int row0 = rt * kGemmRows, tok0 = tt * kGemmTokens + tg * 64;
    const int nkc = p.in / kGemmKc;   // a multiple of 4

    // activation fragments of my two token groups: [group][in / 16][64 lanes][8]
    const int last_group = (p.batch - 1) / 32;
    const _Float16* xg[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
        xg[t] = reinterpret_cast<const _Float16*>(p.xpack) +
                (size_t(min(tok0 / 32 + t, last_group)) * (p.in / 16) * 64 + lane) * 8;
    const int nks = p.in / 16;
    auto xfrag = [&](int t, int ks) -> v8h {
        return *reinterpret_cast<const v8h*>(xg[t] + size_t(min(ks, nks - 1)) * 512);
    };

    // weight chunk: thread (row tid/8 + 64 i, 16-byte piece tid%8), i = 0..3
    const _Float16* const wd = reinterpret_cast<const _Float16*>(p.wdense);
    const _Float16* wsrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        wsrc[i] = wd + size_t(min(row0 + (tid >> 3) + 64 * i, p.out - 1)) * p.in + (tid & 7) * 8;
    _Float16* const wdst = wl + (tid >> 3) * kGemmLd + (tid & 7) * 8;
    struct WIn {
        uint4 v[4];
    };
    auto load_w = [&](int kc) -> WIn {
        WIn w;
        const int c = min(kc, nkc - 1) * kGemmKc;
#pragma unroll
        for (int i = 0; i < 4; ++i) w.v[i] = *reinterpret_cast<const uint4*>(wsrc[i] + c);
        return w;
    };
    auto write_w = [&](const WIn& w, int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(wdst + buf * kGemmBuf + 64 * i * kGemmLd) = w.v[i];
    };
    // fragment j (32 rows) of my 128 rows, step s (16 columns) of the chunk in buffer buf
    const _Float16* const wfr = wl + (rg * 128 + ln) * kGemmLd + 8 * hl;
    auto wfrag = [&](int buf, int s, int j) -> v8h {
        return *reinterpret_cast<const v8h*>(wfr + buf * kGemmBuf + j * 32 * kGemmLd + s * 16);
    };

    v16f acc[4][2];   // [row fragment][token group]
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][t][v] = 0.0f;

    WIn wA = load_w(0);
    WIn wB = load_w(1);
    v8h ring[kGemmPd][2];
#pragma unroll
    for (int k = 0; k < kGemmPd; ++k) {
        ring[k][0] = xfrag(0, k);
        ring[k][1] = xfrag(1, k);
    }
    write_w(wA, 0);
    wA = load_w(2);
    lds_barrier();
    v8h b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = wfrag(0, 0, j);

    // One chunk from buffer BUF: at step 1 the chunk after it (already in registers W) goes to the
    // other buffer and the chunk two further on is requested; the barrier after step 2 makes the
    // other buffer readable for the prefetch at step 3 and protects this buffer from the next
    // chunk's writes.
#define BS_GEMM_CHUNK(KC, BUF, W)                                                          \
    {                                                                                      \
        _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                    \
            const int ks = (KC) * 4 + s;                                                   \
            const v8h a0 = ring[s][0], a1 = ring[s][1];                                    \
            ring[s][0] = xfrag(0, ks + kGemmPd);                                           \
            ring[s][1] = xfrag(1, ks + kGemmPd);                                           \
            if (s == 1) {                                                                  \
                write_w(W, (BUF) ^ 1);                                                     \
                W = load_w((KC) + 3);                                                      \
            }                                                                              \
            __builtin_amdgcn_sched_barrier(0); /* keep the requests ahead of the step's arithmetic */ \
            v8h nb[4];                                                                     \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                  \
                nb[j] = (s < 3) ? wfrag(BUF, s + 1, j) : wfrag((BUF) ^ 1, 0, j);           \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                \
                acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b[j], acc[j][0], 0, 0, 0); \
                acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b[j], acc[j][1], 0, 0, 0); \
            }                                                                              \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) b[j] = nb[j];                    \
            if (s == 2) lds_barrier();                                                     \
            __builtin_amdgcn_sched_barrier(0);                                             \
        }                                                                                  \
    }
    static_assert(kGemmPd == 4, "the ring is indexed by the step inside a chunk");
    for (int kc = 0; kc < nkc; kc += 2) {
        BS_GEMM_CHUNK(kc, 0, wB)
        BS_GEMM_CHUNK(kc + 1, 1, wA)
    }
#undef BS_GEMM_CHUNK

    // C[i = token][n = row]: lane (row ln), register v holds token 8*(v/4) + 4*hl + v%4 of the group
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tok = tok0 + t * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                const int row = row0 + rg * 128 + j * 32 + ln;
                if (tok < p.batch && row < p.out) store_y(p, size_t(tok) * p.out + row, acc[j][t][v]);
            }
}

hipError_t launch_dense_zero(const LaunchArgs& a, hipStream_t st) {
    const size_t n16 = size_t(a.geo.out) * size_t(a.geo.in) * 2 / 16;
    hipLaunchKernelGGL(k_dense_zero, dim3(unsigned((n16 + 255) / 256)), dim3(256), 0, st,
                       static_cast<uint4*>(a.wdense), n16);
    return hipGetLastError();
}

hipError_t launch_dense(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    if (a.batch < 1 || p.xpack == nullptr || p.wdense == nullptr) return hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    launch_xpack(p, st);
    const int ntt = (p.batch + kGemmTokens - 1) / kGemmTokens, nrt = (p.out + kGemmRows - 1) / kGemmRows;
    const unsigned wgs = unsigned(8 * ((nrt + 7) / 8) * ntt);
    hipLaunchKernelGGL(k_gemm, dim3(wgs), dim3(512), kGemmLds, st, p);
    return hipGetLastError();
}

}  // namespace bitstack
