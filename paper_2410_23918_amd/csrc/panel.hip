// Batch / prefill kernel: Y = W' X'^T with the weight tile W' rebuilt in LDS, never in HBM.
//
//     W'[o][j] = sum_i S_i[o][j] * (U_i V_i^T)[o][j]              (Eq. 8),   X' = X diag(1/s)   (Eq. 4)
//
// For more than a couple of tokens the factored form used by the decode kernel costs 16 matrix-
// core operations per sign bit and token; rebuilding the weight costs a fixed amount per weight
// element and is then reused by every token of the tile (the paper's own fused restore-and-
// multiply variant, its "level 5", pays the same redundant restoration once per token tile).
//
// One workgroup (4 wavefronts) owns 64 output rows x TN tokens and walks the input columns in
// chunks of 256 (one sign unit per 32 rows):
//   1. x/s for the chunk goes to LDS as fp16, token-major;
//   2. for every loaded block: V's chunk is transposed into LDS (column-major ranks), the
//      magnitude tile (U V^T)^T is formed 32 columns x 32 rows at a time with
//      v_mfma_f32_32x32x16_f16 (K = the 16 ranks) so that a lane holds, for one output row, 16
//      columns that all live in one 32-bit sign word of that row; the sign is applied as
//      "add where the bit is set" (bit-field extract, and, add) and S = 2B - 1 is undone at the
//      end with the plain sum of the magnitude tiles, accumulated for free by the matrix cores;
//   3. the fp16 weight tile (64 x 256) goes to LDS and meets the activation tile on the matrix
//      cores (fp32 accumulate).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "kparams.h"
#include "layout.h"

namespace bitstack {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kPanelRows = 64;        // output rows per workgroup
constexpr int kPanelLd = 264;         // fp16 elements per LDS row of a 256-column tile (+8: bank spread)

template <int TN>
__global__ __launch_bounds__(256) void k_panel(KParams p) {
    constexpr int TG = TN / 32;       // token groups of 32
    constexpr int TGW = TG / 2;       // token groups per wavefront in the GEMM stage
    static_assert(TN == 64 || TN == 128, "token tile");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* xt = reinterpret_cast<_Float16*>(smem);                                    // [TN][kPanelLd]
    _Float16* wt = xt + TN * kPanelLd;                                                   // [64][kPanelLd]
    _Float16* vt = wt + kPanelRows * kPanelLd;                                           // [2][256][16]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hl = lane >> 5, ln = lane & 31;
    const int row_tile0 = blockIdx.x * kPanelRows;
    const int tok0 = blockIdx.y * TN;
    const int nch = p.in / kChunkCols;

    // reconstruction role of this wavefront: 32 rows x 128 columns of the 64 x 256 tile
    const int rg = wave & 1, chalf = wave >> 1;
    const int rrow = row_tile0 + rg * 32 + ln;             // my output row while reconstructing
    const bool rrow_ok = rrow < p.out;
    const int rrow_c = rrow_ok ? rrow : p.out - 1;         // clamped for loads

    // GEMM role: row group rg, token groups chalf, chalf + 2, ...
    v16f yacc[TGW];
#pragma unroll
    for (int k = 0; k < TGW; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) yacc[k][v] = 0.0f;

    for (int ch = 0; ch < nch; ++ch) {
        // ---- 1. activation tile x/s -> LDS (fp16, token-major)
        for (int idx = tid; idx < TN * 32; idx += 256) {   // 8 columns per item
            const int t = idx >> 5, c8 = (idx & 31) * 8;
            v8h o;
            if (tok0 + t < p.batch) {
                const uint4 raw = *reinterpret_cast<const uint4*>(p.x + size_t(tok0 + t) * p.in + ch * kChunkCols + c8);
                const __half* h = reinterpret_cast<const __half*>(&raw);
                const float4 r0 = *reinterpret_cast<const float4*>(p.rs + ch * kChunkCols + c8);
                const float4 r1 = *reinterpret_cast<const float4*>(p.rs + ch * kChunkCols + c8 + 4);
                const float rr[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
#pragma unroll
                for (int k = 0; k < 8; ++k) o[k] = _Float16(__half2float(h[k]) * rr[k]);
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) o[k] = _Float16(0.0f);
            }
            *reinterpret_cast<v8h*>(xt + t * kPanelLd + c8) = o;
        }

        // ---- 2. weight tile: sum over blocks of sign (.) (U V^T), 32 rows x 128 columns per wave
        v16f acc2[4], msum[4];
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc2[w4][v] = msum[w4][v] = 0.0f;

        for (int i = 0; i < p.n_loaded; ++i) {
            const unsigned char* blk = p.blocks + size_t(i) * p.block_stride;
            // V chunk (256 columns x 16 ranks) -> LDS, column-major ranks
            {
                const __half* vsrc = reinterpret_cast<const __half*>(blk + p.off_v) + size_t(ch) * 4096 + tid * 16;
                const uint4 a = reinterpret_cast<const uint4*>(vsrc)[0], b = reinterpret_cast<const uint4*>(vsrc)[1];
                const unsigned vw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                const int pos = tid >> 4, r = tid & 15;
                const int g = pos & 1, t = pos >> 1;
                _Float16* dst = vt + (i & 1) * 4096 + r;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int col = g * 128 + (e >> 2) * 32 + (e & 3) * 8 + t;
                    const unsigned short bits = (e & 1) ? (vw[e >> 1] >> 16) : (vw[e >> 1] & 0xFFFFu);
                    reinterpret_cast<unsigned short*>(dst)[col * 16] = bits;
                }
            }
            // my row's sign words for this column half, my row's U (ranks 8*hl .. 8*hl+7)
            const uint4 sw = *reinterpret_cast<const uint4*>(
                blk + (size_t(rrow_c >> 5) * nch + ch) * kUnitBytes + (chalf * 32 + (rrow_c & 31)) * 16);
            const unsigned words[4] = {sw.x, sw.y, sw.z, sw.w};
            const v8h uf = *reinterpret_cast<const v8h*>(blk + p.off_u + size_t(rrow_c) * 32 + hl * 16);
            __syncthreads();   // V chunk of block i is in LDS (buffer i & 1)
            const _Float16* vb = vt + (i & 1) * 4096;
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4) {
                const int col = chalf * 128 + w4 * 32 + ln;
                const v8h vf = *reinterpret_cast<const v8h*>(vb + col * 16 + hl * 8);
                v16f z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                // C[i = column][n = row]: lane (row ln), register v holds column 8*(v/4) + 4*hl + v%4
                const v16f m = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, uf, z, 0, 0, 0);
                msum[w4] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, uf, msum[w4], 0, 0, 0);
                const int wrd = int(words[w4]);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int bit = 8 * (v >> 2) + 4 * hl + (v & 3);
                    // all-ones where the sign bit is set (+1), zero otherwise
                    const int mask = (hl == 0) ? __builtin_amdgcn_sbfe(wrd, 8 * (v >> 2) + (v & 3), 1)
                                               : __builtin_amdgcn_sbfe(wrd, 8 * (v >> 2) + 4 + (v & 3), 1);
                    (void)bit;
                    acc2[w4][v] += __int_as_float(__float_as_int(m[v]) & mask);
                }
            }
        }
        // W' = 2 * (sum over set bits) - (sum of all magnitude tiles) -> fp16 tile in LDS
        __syncthreads();       // previous chunk's GEMM has finished reading wt
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int col = chalf * 128 + w4 * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                wt[(rg * 32 + ln) * kPanelLd + col] = _Float16(2.0f * acc2[w4][v] - msum[w4][v]);
            }
        __syncthreads();       // xt and wt complete

        // ---- 3. Y tile += W' tile (64 x 256) * X'^T (256 x TN)
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) {
            const v8h af = *reinterpret_cast<const v8h*>(wt + (rg * 32 + ln) * kPanelLd + ks * 16 + hl * 8);
#pragma unroll
            for (int k = 0; k < TGW; ++k) {
                const int tg = chalf + 2 * k;
                const v8h bf = *reinterpret_cast<const v8h*>(xt + (tg * 32 + ln) * kPanelLd + ks * 16 + hl * 8);
                yacc[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, yacc[k], 0, 0, 0);
            }
        }
        __syncthreads();       // xt, wt free for the next chunk
    }

    // ---- store: C[i = row][n = token]: lane (token ln), register v holds row 8*(v/4) + 4*hl + v%4
#pragma unroll
    for (int k = 0; k < TGW; ++k) {
        const int tok = tok0 + (chalf + 2 * k) * 32 + ln;
        if (tok < p.batch) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row_tile0 + rg * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                if (row < p.out) store_y(p, size_t(tok) * p.out + row, yacc[k][v]);
            }
        }
    }
}

template <int TN>
static hipError_t launch_panel_t(const KParams& p, hipStream_t st) {
    const size_t smem = size_t(TN + kPanelRows) * kPanelLd * 2 + 2 * 4096 * 2;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_panel<TN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(smem));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((p.out + kPanelRows - 1) / kPanelRows, (p.batch + TN - 1) / TN);
    hipLaunchKernelGGL((k_panel<TN>), grid, dim3(256), smem, st, p);
    return hipGetLastError();
}

hipError_t launch_panel(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    if (a.batch > 64) return launch_panel_t<128>(p, st);
    return launch_panel_t<64>(p, st);
}

}  // namespace bitstack
