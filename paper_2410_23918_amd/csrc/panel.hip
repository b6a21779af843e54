// Batch / prefill kernel: Y = W' X'^T with the weight tile W' rebuilt in LDS, never in HBM.
//
//     W'[o][j] = sum_i S_i[o][j] * (U_i V_i^T)[o][j]              (Eq. 8),   X' = X diag(1/s)   (Eq. 4)
//
// For more than a couple of tokens the factored form used by the decode kernel costs 16 matrix-
// core operations per sign bit and token; rebuilding the weight costs a fixed amount per weight
// element and is then reused by every token of the tile (the paper's own fused restore-and-
// multiply variant, its "level 5", pays the same redundant restoration once per token tile).
//
// One workgroup (4 wavefronts) owns 64 output rows x up to 512 tokens and walks the input columns
// in chunks of 256 (one sign unit per 32 rows):
//   1. for every loaded block: V's chunk is transposed into LDS (column-major ranks), the
//      tile (U V^T)^T is formed 32 columns x 32 rows at a time with v_mfma_f32_32x32x16_f16
//      (K = the 16 ranks) so that a lane holds, for one output row, 16 columns that all live in
//      one 32-bit sign word of that row; the sign enters as a +-1.0 multiplier built from the bit
//      (bit-field extract, and-or, fused multiply-add).  The block's V values, sign words and U
//      row are fetched one block ahead of their use;
//   2. the fp16 weight tile (64 x 256) goes to LDS;
//   3. per tile of 128 tokens: x/s for the chunk goes to LDS as fp16, token-major, and meets the
//      weight tile on the matrix cores (fp32 accumulate).  The weight tile is built once per
//      chunk for all token tiles of the workgroup.
#include <hip/hip_fp16.h>
#include <type_traits>
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "kparams.h"
#include "layout.h"

namespace bitstack {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kPanelRows = 64;        // output rows per workgroup
constexpr int kPanelLd = 264;         // fp16 elements per LDS row of a 256-column tile (+8: bank spread)

// A V chunk (256 columns x 16 ranks) in LDS, kept in the order it has in memory: 16 panel positions
// (t, g) x 16 ranks, one row of 16 columns (32 B) each.  Rows are spaced 48 B and positions 784 B so
// that both the 128-bit row writes and the 16-bit gathers "one column, 8 ranks" spread over all banks.
constexpr int kFusedMaxBatch = kSmallBatch;   // above this the weight-tile kernels are used
constexpr int kVRow = 48;
constexpr int kVPos = 16 * kVRow + 16;

// TT token tiles of 128 tokens per workgroup: the weight tile is rebuilt once per column chunk
// and reused for all of them (accumulators: 32 registers per tile and lane).
template <int TT>
__global__ __launch_bounds__(256) void k_panel(KParams p) {
    constexpr int TN = 128;           // tokens per activation tile in LDS
    constexpr int TGW = 2;            // 32-token groups per wavefront and tile in the GEMM stage
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* xt = reinterpret_cast<_Float16*>(smem);                                    // [TN][kPanelLd]
    _Float16* wt = xt + TN * kPanelLd;                                                   // [64][kPanelLd]
    _Float16* vt = wt + kPanelRows * kPanelLd;                                           // [2][256][16]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hl = lane >> 5, ln = lane & 31;
    const int row_tile0 = blockIdx.x * kPanelRows;
    const int tok_base = blockIdx.y * (TN * TT);
    const int nch = p.in / kChunkCols;

    // reconstruction role of this wavefront: 32 rows x 128 columns of the 64 x 256 tile
    const int rg = wave & 1, chalf = wave >> 1;
    const int rrow = row_tile0 + rg * 32 + ln;             // my output row while reconstructing
    const int rrow_c = rrow < p.out ? rrow : p.out - 1;    // clamped for loads

    // GEMM role: row group rg, token groups chalf and chalf + 2 of every token tile
    v16f yacc[TT][TGW];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int k = 0; k < TGW; ++k)
#pragma unroll
            for (int v = 0; v < 16; ++v) yacc[tt][k][v] = 0.0f;

    // per-block inputs of the reconstruction, fetched one block ahead
    struct BlockIn {
        uint4 va, vb;   // my 16 V values (one panel position, one rank)
        uint4 sw;       // my row's four sign words of this column half
        v8h uf;         // my row's U, ranks 8*hl .. 8*hl+7
    };
    auto fetch = [&](int i, int ch) -> BlockIn {
        BlockIn b;
        const unsigned char* blk = p.blocks + size_t(min(i, p.n_loaded - 1)) * p.block_stride;
        const uint4* vsrc = reinterpret_cast<const uint4*>(reinterpret_cast<const __half*>(blk + p.off_v) +
                                                           size_t(ch) * 4096 + tid * 16);
        b.va = vsrc[0];
        b.vb = vsrc[1];
        b.sw = *reinterpret_cast<const uint4*>(blk + (size_t(rrow_c >> 5) * nch + ch) * kUnitBytes +
                                               (chalf * 32 + (rrow_c & 31)) * 16);
        b.uf = *reinterpret_cast<const v8h*>(blk + p.off_u + size_t(rrow_c) * 32 + hl * 16);
        return b;
    };

    for (int ch = 0; ch < nch; ++ch) {
        // ---- weight tile: sum over blocks of sign (.) (U V^T), 32 rows x 128 columns per wave
        v16f acc2[4];
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc2[w4][v] = 0.0f;

        BlockIn cur = fetch(0, ch);
        for (int i = 0; i < p.n_loaded; ++i) {
            const BlockIn nxt = fetch(i + 1, ch);   // clamped: the last one is fetched twice
            // V chunk (256 columns x 16 ranks) -> LDS, column-major ranks
            {
                const unsigned vw[8] = {cur.va.x, cur.va.y, cur.va.z, cur.va.w, cur.vb.x, cur.vb.y, cur.vb.z, cur.vb.w};
                const int pos = tid >> 4, r = tid & 15;
                const int g = pos & 1, t = pos >> 1;
                unsigned short* dst = reinterpret_cast<unsigned short*>(vt + (i & 1) * 4096 + r);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int col = g * 128 + (e >> 2) * 32 + (e & 3) * 8 + t;
                    dst[col * 16] = (e & 1) ? (unsigned short)(vw[e >> 1] >> 16) : (unsigned short)(vw[e >> 1] & 0xFFFFu);
                }
            }
            const unsigned words[4] = {cur.sw.x, cur.sw.y, cur.sw.z, cur.sw.w};
            const v8h uf = cur.uf;
            lds_barrier();     // V chunk of block i is in LDS (buffer i & 1); next block's loads stay in flight
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
                // one shift puts my 16 columns' bits at 8*(v/4) + v%4 for both lane halves;
                // inverted, so that a set bit marks a negative sign
                const int wrd = int(~words[w4] >> (4 * hl));
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int neg = __builtin_amdgcn_sbfe(wrd, 8 * (v >> 2) + (v & 3), 1);   // all-ones or zero
                    const float sgn = __int_as_float((neg & int(0x80000000u)) | 0x3f800000);   // -1.0f or +1.0f
                    acc2[w4][v] = __builtin_fmaf(m[v], sgn, acc2[w4][v]);
                }
            }
            cur = nxt;
        }
        // W' tile -> fp16 in LDS
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int col = chalf * 128 + w4 * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                wt[(rg * 32 + ln) * kPanelLd + col] = _Float16(acc2[w4][v]);
            }

        // ---- token tiles: x/s -> LDS, then Y tile += W' tile (64 x 256) * X'^T (256 x 128)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int tok0 = tok_base + tt * TN;
            if (tok0 < p.batch) {          // uniform over the workgroup
                for (int idx = tid; idx < TN * 32; idx += 256) {   // 8 columns per item
                    const int t = idx >> 5, c8 = (idx & 31) * 8;
                    v8h o;
                    if (tok0 + t < p.batch) {
                        const uint4 raw =
                            *reinterpret_cast<const uint4*>(p.x + size_t(tok0 + t) * p.in + ch * kChunkCols + c8);
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
                __syncthreads();       // xt (and, first time round, wt) complete
#pragma unroll
                for (int ks = 0; ks < 16; ++ks) {
                    const v8h af = *reinterpret_cast<const v8h*>(wt + (rg * 32 + ln) * kPanelLd + ks * 16 + hl * 8);
#pragma unroll
                    for (int k = 0; k < TGW; ++k) {
                        const int tg = chalf + 2 * k;
                        const v8h bf = *reinterpret_cast<const v8h*>(xt + (tg * 32 + ln) * kPanelLd + ks * 16 + hl * 8);
                        yacc[tt][k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, yacc[tt][k], 0, 0, 0);
                    }
                }
                __syncthreads();       // xt free for the next tile, wt for the next chunk
            }
        }
    }

    // ---- store: C[i = row][n = token]: lane (token ln), register v holds row 8*(v/4) + 4*hl + v%4
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int k = 0; k < TGW; ++k) {
            const int tok = tok_base + tt * TN + (chalf + 2 * k) * 32 + ln;
            if (tok < p.batch) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_tile0 + rg * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                    if (row < p.out) store_y(p, size_t(tok) * p.out + row, yacc[tt][k][v]);
                }
            }
        }
}

template <int TT>
static hipError_t launch_panel_t(const KParams& p, hipStream_t st) {
    const size_t smem = size_t(128 + kPanelRows) * kPanelLd * 2 + 2 * 4096 * 2;
    static std::atomic<bool> attr_set{false};   // setting the attribute twice is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_panel<TT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(smem));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((p.out + kPanelRows - 1) / kPanelRows, (p.batch + 128 * TT - 1) / (128 * TT));
    hipLaunchKernelGGL((k_panel<TT>), grid, dim3(256), smem, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Small batches (up to 64 tokens): no weight tile is kept at all.  Each block's signed 32 x 32
// tile goes straight from the accumulator registers of the magnitude product into the B operand
// of the product with the activations, so the sum over blocks (Eq. 8) happens inside the fp32
// accumulators of Y on the matrix cores:
//
//     Y[t][o] += sum_j X'[t][j] * ( S_i[o][j] * (U_i V_i^T)[o][j] )      for every block i
//
// The magnitude product is laid out C[i = column][n = row]: a lane holds one row and 16 columns
// 8*(v/4) + 4*half + v%4 of the tile, exactly the "K index on registers, N index on lanes" shape
// of a B operand whose K runs over columns.  Registers v and v + 8 sit 16 columns apart, i.e.
// 16 bits apart in the row's sign word, so one shift lines both sign bits up with the sign bits
// of a packed fp16 pair and one three-input bit operation flips them: 1.5 vector instructions per
// weight element and block (convert-pack, shift, xor-and).  K slots are permuted the same way in
// the activation fragments, which are built once per column chunk and stay in registers for all
// blocks.
//
// One workgroup = 64 output rows x 32 tokens; 8 wavefronts = 2 teams (even / odd column chunks)
// x 4 column quarters of a chunk; every wavefront handles both 32-row groups, so one V fragment
// and one activation fragment serve two products.  The eight partial Y tiles meet in LDS at the
// end.  More than 32 tokens: blockIdx.y walks the token groups (the signed tiles are rebuilt per
// group; the weight-tile kernel above takes over where that stops paying).
//
// Nothing in the main loop is shared between wavefronts, so it has no barrier: each wavefront
// turns its own 64 columns of V from "16 columns of one rank" rows into "8 ranks of one column"
// fragments through a private piece of LDS (LDS operations of one wavefront execute in order), and
// keeps its own 64 columns of x/s there.  The U rows of all loaded blocks (2 KiB per block) are
// cached in LDS once.
//
// A step is one (column chunk, block) pair of a team, chunks outermost.  Inputs travel three
// steps deep and are never copied between registers while in flight (a copy would wait for the
// load): three named register sets rotate through a loop unrolled three times.
//   step s:  V(s+1) registers -> LDS -> V(s+1) fragments | compute block s from signs(s), U(s),
//            fragments(s) | issue loads of signs(s+2), V(s+3)
constexpr int kVtStride = 68;                       // dwords between panel positions t in the private V piece
constexpr int kVPriv = 8 * kVtStride * 4;           // bytes per private V buffer (8 t x 16 ranks x 8 columns)
constexpr int kXPrivLd = 72;                        // fp16 per token row of the private x/s piece (64 + 8)
constexpr int kXPriv = 32 * kXPrivLd * 2;           // bytes
constexpr int kFusedFixedLds = 8 * (2 * kVPriv + kXPriv);
constexpr int kFusedMaxBlocks = (160 * 1024 - kFusedFixedLds) / 2048 - 1;   // U cache: 2 KiB per block

__global__ __launch_bounds__(512) void k_fused(KParams p) {
    constexpr int XPT = 4;   // tokens per lane when staging activations
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int team = wave >> 2, cw = wave & 3;
    const int hl = lane >> 5, ln = lane & 31;
    unsigned char* const vpriv = smem + wave * (2 * kVPriv + kXPriv);
    _Float16* const xpriv = reinterpret_cast<_Float16*>(vpriv + 2 * kVPriv);
    unsigned char* const ucache = smem + kFusedFixedLds;   // [block][64 rows][32 B]
    // column chunks of this workgroup: all of them, or one of ksplit ranges (blockIdx.z) when there are
    // too few row tiles to fill the chip; the partial results then meet in the workspace (see the end)
    const int ksplit = max(p.n_ks, 1);
    const int nch_all = p.in / kChunkCols;
    const int c_lo = int(blockIdx.z) * nch_all / ksplit, nch = (int(blockIdx.z) + 1) * nch_all / ksplit;   // [c_lo, nch)
    const int iters = (nch - c_lo + 1) / 2;
    const int n = p.n_loaded;
    const int total = iters * n;
    const int rt0 = blockIdx.x * 2, nrt = p.out / kTileRows;
    const int rtc[2] = {min(rt0, nrt - 1), min(rt0 + 1, nrt - 1)};   // clamped for loads
    const int tok0 = blockIdx.y * 32;

    // ---- U rows of my 64 output rows, all blocks -> LDS
    for (int idx = tid; idx < n * 128; idx += 512) {
        const int i = idx >> 7, piece = idx & 127;         // 16-byte pieces: row = piece / 2
        const int row = rtc[piece >> 6] * kTileRows + ((piece >> 1) & 31);
        *reinterpret_cast<uint4*>(ucache + idx * 16) = *reinterpret_cast<const uint4*>(
            p.blocks + size_t(i) * p.block_stride + p.off_u + size_t(row) * 32 + (piece & 1) * 16);
    }

    // ---- activations: x/s of my 64 columns of one chunk as fp16 in my LDS piece, token-major
    struct XIn {
        uint4 x[XPT];
        float4 r0, r1;
    };
    const int cg = lane & 7, tl = lane >> 3;   // staging role: 8 columns, tokens tl, tl + 8, ...
    auto fetch_x = [&](int it) -> XIn {         // chunk of my team's iteration `it`, clamped
        XIn v;
        const int col = min(c_lo + 2 * it + team, nch - 1) * kChunkCols + cw * 64 + cg * 8;
#pragma unroll
        for (int m = 0; m < XPT; ++m)
            v.x[m] = *reinterpret_cast<const uint4*>(p.x + size_t(min(tok0 + tl + 8 * m, p.batch - 1)) * p.in + col);
        v.r0 = *reinterpret_cast<const float4*>(p.rs + col);
        v.r1 = *reinterpret_cast<const float4*>(p.rs + col + 4);
        return v;
    };
    auto store_x = [&](XIn v, int it) {         // a team without a chunk left (odd chunk count) gets zeros
        const float rr[8] = {v.r0.x, v.r0.y, v.r0.z, v.r0.w, v.r1.x, v.r1.y, v.r1.z, v.r1.w};
        const bool valid = c_lo + 2 * it + team < nch;
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int tok = tl + 8 * m;
            const float on = (valid && tok0 + tok < p.batch) ? 1.0f : 0.0f;
            const __half* h = reinterpret_cast<const __half*>(&v.x[m]);
            v8h o;
#pragma unroll
            for (int k = 0; k < 8; ++k) o[k] = _Float16(__half2float(h[k]) * rr[k] * on);
            *reinterpret_cast<v8h*>(xpriv + tok * kXPrivLd + cg * 8) = o;
        }
    };
    // activation fragments, K slots in the order the signed tile has them:
    // slot 2p <-> column 8*mf + 4*hl + p, slot 2p + 1 <-> that + 16
    v8h afr[2][2];
    auto build_afr = [&]() {
#pragma unroll
        for (int tile = 0; tile < 2; ++tile)
#pragma unroll
            for (int mf = 0; mf < 2; ++mf) {
                const _Float16* src = xpriv + ln * kXPrivLd + tile * 32 + mf * 8 + 4 * hl;
                const uint2 lo = *reinterpret_cast<const uint2*>(src);
                const uint2 hi = *reinterpret_cast<const uint2*>(src + 16);
                const unsigned w[4] = {(lo.x & 0xFFFFu) | (hi.x << 16), (lo.x >> 16) | (hi.x & 0xFFFF0000u),
                                       (lo.y & 0xFFFFu) | (hi.y << 16), (lo.y >> 16) | (hi.y & 0xFFFF0000u)};
                afr[tile][mf] = __builtin_bit_cast(v8h, w);
            }
    };

    // ---- per-step inputs: signs and V of one (chunk, block) step, both through one buffer descriptor
    // over the loaded blocks (less than 4 GiB, checked by the launcher): the address of a load is a
    // per-lane constant plus a scalar offset that moves by one block stride per step, so no vector
    // instruction and only a handful of scalar ones go into addresses.
    struct Pos {
        int i, ch;              // block, chunk (past the last step the last chunk is read again, harmlessly)
        unsigned off_s, off_v;  // scalar offsets of the step's sign units and V panel
    };
    const unsigned stride32 = unsigned(p.block_stride), off_v32 = unsigned(p.off_v);
    auto pos_at = [&](int it, int i) -> Pos {
        Pos q;
        q.i = i;
        q.ch = min(c_lo + 2 * it + team, nch - 1);
        q.off_s = unsigned(i) * stride32 + unsigned(q.ch) * kUnitBytes;
        q.off_v = unsigned(i) * stride32 + off_v32 + unsigned(q.ch) * 8192u;
        return q;
    };
    auto advance = [&](Pos q) -> Pos {
        if (++q.i == n) {
            q.i = 0;
            q.ch = min(q.ch + 2, nch - 1);
            q.off_s = unsigned(q.ch) * kUnitBytes;
            q.off_v = off_v32 + unsigned(q.ch) * 8192u;
        } else {
            q.off_s += stride32;
            q.off_v += stride32;
        }
        return q;
    };
    __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(p.blocks), 0,
                                                                   unsigned(n) * stride32, 0x00020000);
    typedef int v4i_ __attribute__((ext_vector_type(4)));
    typedef int v2i_ __attribute__((ext_vector_type(2)));
    // V: my wavefront needs, of every row (t, g, r) with g = my column half, the 8 columns
    // e = 8*(cw&1) .. +7, i.e. 16 of its 32 bytes; lane L takes rows (t = L/8, r = 2*(L%8) and + 1)
    struct VIn {
        v4i_ a, b;
    };
    const unsigned voff = unsigned((((lane >> 3) * 2 + (cw >> 1)) * 16 + 2 * (lane & 7)) * 32 + (cw & 1) * 16);
    auto fetch_v = [&](Pos q) -> VIn {
        VIn v;
        v.a = __builtin_amdgcn_raw_buffer_load_b128(brs, voff, q.off_v, 0);
        v.b = __builtin_amdgcn_raw_buffer_load_b128(brs, voff + 32, q.off_v, 0);
        return v;
    };
    struct SIn {
        v2i_ w[2];   // per row group: my row's two sign words of my 64 columns
    };
    const unsigned soff[2] = {unsigned((size_t(rtc[0]) * nch_all) * kUnitBytes + ((cw >> 1) * 32 + ln) * 16 + (cw & 1) * 8),
                              unsigned((size_t(rtc[1]) * nch_all) * kUnitBytes + ((cw >> 1) * 32 + ln) * 16 + (cw & 1) * 8)};
    auto fetch_s = [&](Pos q) -> SIn {
        SIn v;
        v.w[0] = __builtin_amdgcn_raw_buffer_load_b64(brs, soff[0], q.off_s, 0);
        v.w[1] = __builtin_amdgcn_raw_buffer_load_b64(brs, soff[1], q.off_s, 0);
        return v;
    };

    // my private V piece, transposed on the way in: dword address of (t, column e, rank pair) =
    // t * kVtStride + e * 8 + pair.  A lane arrives with ranks 2j and 2j + 1 of eight columns (two
    // columns per register) and scatters them as sixteen 16-bit writes; a fragment "one column, 8 ranks"
    // is then one 128-bit read (the stride of 68 keeps the writes to two lanes per bank).
    unsigned short* const vdst = reinterpret_cast<unsigned short*>(vpriv) + ((lane >> 3) * kVtStride + (lane & 7)) * 2;
    int vsrc_off[2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
        const int b = ln >> 3, t = ln & 7, e = tile * 4 + b;   // e: column of my 8 within a row
        vsrc_off[tile] = (t * kVtStride + e * 8 + 4 * hl) * 4;
    }
    auto stage_v = [&](VIn v, int buf) {
        unsigned short* const d = vdst + buf * (kVPriv / 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned a = unsigned(v.a[i]), b = unsigned(v.b[i]);   // rank 2j / 2j + 1, columns 2i (low half) and 2i + 1
            d[(2 * i) * 16] = static_cast<unsigned short>(a);
            d[(2 * i) * 16 + 1] = static_cast<unsigned short>(b);
            d[(2 * i + 1) * 16] = static_cast<unsigned short>(a >> 16);
            d[(2 * i + 1) * 16 + 1] = static_cast<unsigned short>(b >> 16);
        }
    };
    auto read_vf = [&](int buf, int tile) -> v8h {
        // A operand of the magnitude product: my column's ranks 8*hl .. 8*hl + 7
        return *reinterpret_cast<const v8h*>(vpriv + buf * kVPriv + vsrc_off[tile]);
    };
    auto read_u = [&](int i, int rg) -> v8h {   // my row's U, ranks 8*hl .. 8*hl + 7
        return *reinterpret_cast<const v8h*>(ucache + ((i * 64 + rg * 32 + ln) * 2 + hl) * 16);
    };

    v16f yacc[2];
#pragma unroll
    for (int rg = 0; rg < 2; ++rg)
#pragma unroll
        for (int v = 0; v < 16; ++v) yacc[rg][v] = 0.0f;

    // per-lane shifts that bring the sign bits of a register pair (word bits 8*mf + k + 4*hl and that + 16)
    // to bits 15 and 31
    unsigned sh[2][4];
#pragma unroll
    for (int mf = 0; mf < 2; ++mf)
#pragma unroll
        for (int k = 0; k < 4; ++k) sh[mf][k] = unsigned(15 - 8 * mf - k - 4 * hl);

    auto compute = [&](const SIn& sg, v8h uf0, v8h uf1, v8h vf0, v8h vf1) {
        // magnitude tile C[i = column][n = row]: lane (row ln), register v holds column 8*(v/4) + 4*hl + v%4
        auto magnitude = [&](int tile, int rg) -> v16f {
            v16f z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.0f;
            return __builtin_amdgcn_mfma_f32_32x32x16_f16(tile ? vf1 : vf0, rg ? uf1 : uf0, z, 0, 0, 0);
        };
        auto apply = [&](const v16f& m, int tile, int rg) {
            const unsigned wrd = unsigned(tile ? sg.w[rg].y : sg.w[rg].x);
#pragma unroll
            for (int mf = 0; mf < 2; ++mf) {
                unsigned r4[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                    h2 c;
                    c[0] = _Float16(m[4 * mf + k]);
                    c[1] = _Float16(m[4 * mf + k + 8]);
                    // a cleared bit marks a negative sign
                    const unsigned flip = ~(wrd << sh[mf][k]) & 0x80008000u;
                    r4[k] = __builtin_bit_cast(unsigned, c) ^ flip;
                }
                yacc[rg] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afr[tile][mf], __builtin_bit_cast(v8h, r4), yacc[rg], 0, 0, 0);
            }
        };
        // the magnitude product of the next (tile, row group) is issued before the vector work on the
        // current one, which then covers its latency
        v16f m0 = magnitude(0, 0);
        v16f m1 = magnitude(0, 1);
        apply(m0, 0, 0);
        m0 = magnitude(1, 0);
        apply(m1, 0, 1);
        m1 = magnitude(1, 1);
        apply(m0, 1, 0);
        apply(m1, 1, 1);
        // left to itself the scheduler clusters the matrix-core instructions (two or three in a row, then
        // runs of 30-40 vector instructions); one of them per nine vector instructions keeps both pipes fed
#pragma unroll
        for (int i = 0; i < 12; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one matrix-core instruction
            __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);   // nine vector instructions
        }
    };

    // ---- prologue: steps 0..2 on their way, chunk 0's activations and V(0) fragments ready
    Pos q = pos_at(0, 0);
    VIn vA = fetch_v(q);
    SIn sA = fetch_s(q);
    q = advance(q);
    VIn vB = fetch_v(q);
    SIn sB = fetch_s(q);
    q = advance(q);
    VIn vC = fetch_v(q);
    SIn sC = fetch_s(q);
    q = advance(q);          // q: position of step s + 3
    store_x(fetch_x(0), 0);
    stage_v(vA, 0);
    v8h vf0 = read_vf(0, 0), vf1 = read_vf(0, 1);
    build_afr();
    XIn xn = fetch_x(1);
    __syncthreads();         // U cache complete

    int ci = 0, it = 0;      // block index inside the chunk, team iteration
    // one step; CUR: set in use, NXT: set whose V goes to LDS now.  V(s+3) lands in CUR's V registers
    // (V(s) left them one step ago), signs(s+3) in CUR's sign registers once the step has used them
#define BS_FUSED_STEP(S, CUR, NXT, FAR)                                                    \
    {                                                                                      \
        const v8h uf0 = read_u(ci, 0), uf1 = read_u(ci, 1);                                \
        stage_v(v##NXT, ((S) + 1) & 1);                                                    \
        const v8h vn0 = read_vf(((S) + 1) & 1, 0), vn1 = read_vf(((S) + 1) & 1, 1);        \
        if (ci == 0 && (S) > 0) {                                                          \
            store_x(xn, it);                                                               \
            build_afr();                                                                   \
            xn = fetch_x(it + 1);                                                          \
        }                                                                                  \
        v##CUR = fetch_v(q);                                                               \
        compute(s##CUR, uf0, uf1, vf0, vf1);                                               \
        s##CUR = fetch_s(q);                                                               \
        q = advance(q);                                                                    \
        vf0 = vn0;                                                                         \
        vf1 = vn1;                                                                         \
        if (++ci == n) {                                                                   \
            ci = 0;                                                                        \
            ++it;                                                                          \
        }                                                                                  \
    }
    // The step count is rounded up to a multiple of three without branches around the steps (a
    // branch would make the compiler wait for every load in flight): the extra steps start a new
    // "chunk" past the last one, whose activations are written as zeros, so they add nothing.
    for (int s = 0; s < total; s += 3) {
        BS_FUSED_STEP(s, A, B, C)
        BS_FUSED_STEP(s + 1, B, C, A)
        BS_FUSED_STEP(s + 2, C, A, B)
    }
#undef BS_FUSED_STEP

    // ---- the eight partial tiles meet in LDS; C[i = token][n = row]: lane (row ln),
    //      register v holds token 8*(v/4) + 4*hl + v%4 of the group
    float* red = reinterpret_cast<float*>(smem);   // [8][16][64]
    float* const mine = p.part + size_t(blockIdx.z) * p.batch * p.out;   // my rows of the workspace (ksplit > 1)
#pragma unroll
    for (int rg = 0; rg < 2; ++rg) {
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * 64 + lane] = yacc[rg][v];
        __syncthreads();
        for (int o = tid; o < 1024; o += 512) {
            const int v = o >> 6, l = o & 63;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < 8; ++w) sum += red[(w * 16 + v) * 64 + l];
            const int tok = tok0 + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
            const int row = (rt0 + rg) * kTileRows + (l & 31);
            if (tok < p.batch && row < p.out) {
                if (ksplit == 1)
                    store_y(p, size_t(tok) * p.out + row, sum);
                else   // write-through: the reader may sit on another XCD
                    __hip_atomic_store(mine + size_t(tok) * p.out + row, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    if (ksplit == 1) return;

    // ---- column split: the last workgroup of this (row tile, token group) adds the ksplit partial
    //      tiles in a fixed order and stores y (same protocol as the decode kernel: write-through
    //      stores, one relaxed agent-scope counter after a barrier, agent-scope loads by the last one)
    unsigned* const flag = reinterpret_cast<unsigned*>(smem + 32768);
    // vmcnt(0), other counters left alone: each wavefront's write-through stores above have been
    // acknowledged before it reaches the barrier, so the counter below is bumped only once every
    // partial value of this workgroup is visible at agent scope
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    unsigned* const ctr = p.ctr + blockIdx.y * gridDim.x + blockIdx.x;
    if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = (old + 1u == unsigned(ksplit)) ? 1u : 0u;
    }
    __syncthreads();
    if (*flag) {
        // thread = (token of the group, 4 consecutive rows of the 64)
        const int tok = tok0 + (tid >> 4), row = rt0 * kTileRows + 4 * (tid & 15);
        if (tok < p.batch && row < p.out) {   // out is a multiple of 32: a quad is inside or outside as a whole
            const unsigned span = unsigned(size_t(ksplit) * p.batch * p.out * 4);
            __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(p.part, 0, span, 0x00020000);
            constexpr int kAgentScope = 16;   // sc1
            typedef int v4i_ __attribute__((ext_vector_type(4)));
            v4i_ v[8];
#pragma unroll
            for (int z = 0; z < 8; ++z)
                v[z] = __builtin_amdgcn_raw_buffer_load_b128(
                    prs, z < ksplit ? unsigned(((size_t(z) * p.batch + tok) * p.out + row) * 4) : span, 0, kAgentScope);
            float o4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int z = 0; z < 8; ++z)
#pragma unroll
                for (int k = 0; k < 4; ++k) o4[k] += __int_as_float(v[z][k]);
#pragma unroll
            for (int k = 0; k < 4; ++k) store_y(p, size_t(tok) * p.out + row + k, o4[k]);
        }
        if (tid == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

static bool fused_fits(const KParams& p) {   // U cache in LDS; one 32-bit buffer descriptor over the loaded blocks
    return p.n_loaded <= kFusedMaxBlocks && size_t(p.n_loaded) * p.block_stride < (size_t(1) << 32);
}

constexpr int kFusedMaxSplit = 8;

// few row tiles: split the columns over several workgroups per tile (at least two chunks each;
// the workspace must hold a partial row per split and token, the counters one slot per tile)
int small_batch_split(int out, int in, int batch, int part_slots) {
    const int wgs = ((out + 2 * kTileRows - 1) / (2 * kTileRows)) * ((batch + 31) / 32);
    if (wgs >= 192 || wgs > kCounterSlots) return 1;
    int ksplit = 256 / wgs;
    ksplit = ksplit < kFusedMaxSplit ? ksplit : kFusedMaxSplit;
    const int by_chunks = (in / kChunkCols) / 2, by_space = part_slots / batch;
    ksplit = ksplit < by_chunks ? ksplit : by_chunks;
    ksplit = ksplit < by_space ? ksplit : by_space;
    return ksplit > 1 ? ksplit : 1;
}

static hipError_t launch_fused(KParams p, hipStream_t st) {
    const size_t smem = size_t(kFusedFixedLds) + size_t(p.n_loaded) * 2048;
    static std::atomic<bool> attr_set{false};   // setting the attribute twice is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_fused),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kFusedFixedLds + kFusedMaxBlocks * 2048);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((p.out + 2 * kTileRows - 1) / (2 * kTileRows), (p.batch + 31) / 32);
    p.n_ks = small_batch_split(p.out, p.in, p.batch, p.part_slots);
    grid.z = p.n_ks;
    hipLaunchKernelGGL(k_fused, grid, dim3(512), smem, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Many tokens (prefill): the weight tile is kept, but built the way the small-batch kernel builds
// its signed tiles.  Per block, the signed fp16 tile (same 1.5 vector instructions per element) is
// multiplied by a permuted identity on the matrix cores, which adds it to an fp32 accumulator tile
// in the same register layout; after the last block the tile is scaled by 1/s (Eq. 4 moved from the
// activations to the weight columns, so that activation fragments come from memory untouched),
// rounded to fp16 and parked in LDS.  Then every wavefront multiplies the two parked tiles (64 rows
// x 2 x 256 columns) with its own 64 of the workgroup's 512 tokens.  Same teams, private LDS
// pieces, U cache and three-deep input rotation as k_fused; two LDS-only barriers per pair of
// column chunks.
// Activations of a large batch, once per call, into the order the product stage reads them:
// fragment (token group of 32, 16 columns) = 64 lanes x 8 values, lane (token ln, half hl) holding
// columns 8*hl .. 8*hl + 7.  A wavefront then fetches a fragment as 1 KiB of consecutive memory
// instead of 32-byte pieces of 32 token rows.  Tokens past the batch are zero.
__global__ __launch_bounds__(256) void k_xpack(const __half* x, __half* xp, int batch, int in) {
    const int frags_per_group = in / 16;
    const size_t item = size_t(blockIdx.x) * 256 + threadIdx.x;          // one lane of one fragment
    const size_t total = size_t((batch + 31) / 32) * frags_per_group * 64;
    if (item >= total) return;
    const int lane = int(item & 63);
    const size_t frag = item >> 6;
    const int ks = int(frag % frags_per_group), tgp = int(frag / frags_per_group);
    const int tok = tgp * 32 + (lane & 31);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (tok < batch) v = *reinterpret_cast<const uint4*>(x + size_t(tok) * in + ks * 16 + 8 * (lane >> 5));
    *reinterpret_cast<uint4*>(xp + item * 8) = v;
}

void launch_xpack(const KParams& p, hipStream_t st) {
    const size_t lanes = size_t((p.batch + 31) / 32) * (p.in / 16) * 64;
    hipLaunchKernelGGL(k_xpack, dim3(unsigned((lanes + 255) / 256)), dim3(256), 0, st, p.x, p.xpack, p.batch, p.in);
}

constexpr int kTileFixedLds = 8 * 2 * kVPriv + 2 * kPanelRows * kPanelLd * 2;
constexpr int kTileMaxBlocks = (160 * 1024 - kTileFixedLds) / 2048 - 1;
constexpr int kTileTokens = 512;   // tokens per workgroup

// kRestore: the same construction of the weight tile, but the parked tiles are copied to a dense
// fp16 matrix W' diag(1/s) [out][in] in memory instead of being multiplied with activations (the
// restoring step of the appendix on inference throughput, "level 2"); blockIdx.y then selects a
// range of chunk pairs instead of a token tile.
template <bool kRestore>
__global__ __launch_bounds__(512) void k_tile(KParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int team = wave >> 2, cw = wave & 3;
    const int hl = lane >> 5, ln = lane & 31;
    unsigned char* const vpriv = smem + wave * (2 * kVPriv);
    _Float16* const wt = reinterpret_cast<_Float16*>(smem + 8 * 2 * kVPriv);   // [team][64][kPanelLd]
    unsigned char* const ucache = smem + kTileFixedLds;                         // [block][64 rows][32 B]
    const int nch = p.in / kChunkCols;
    const int iters = (nch + 1) / 2;
    const int n = p.n_loaded;
    const int its_per_wg = kRestore ? (iters + int(gridDim.y) - 1) / int(gridDim.y) : iters;
    const int it_first = kRestore ? int(blockIdx.y) * its_per_wg : 0;
    const int it_end = min(iters, it_first + its_per_wg);
    if (it_first >= it_end) return;
    const int total = (it_end - it_first) * n;
    const int rt0 = blockIdx.x * 2 + (kRestore ? p.row_begin / kTileRows : 0), nrt = p.out / kTileRows;
    const int rtc[2] = {min(rt0, nrt - 1), min(rt0 + 1, nrt - 1)};   // clamped for loads
    const int tok_w = kRestore ? 0 : blockIdx.y * kTileTokens + wave * 64;   // my first token in the product stage

    for (int idx = tid; idx < n * 128; idx += 512) {   // U rows of my 64 output rows, all blocks -> LDS
        const int i = idx >> 7, piece = idx & 127;
        const int row = rtc[piece >> 6] * kTileRows + ((piece >> 1) & 31);
        *reinterpret_cast<uint4*>(ucache + idx * 16) = *reinterpret_cast<const uint4*>(
            p.blocks + size_t(i) * p.block_stride + p.off_u + size_t(row) * 32 + (piece & 1) * 16);
    }

    // per-step inputs through one buffer descriptor over the loaded blocks, as in k_fused: per-lane
    // constant plus a scalar offset that moves by one block stride per step
    struct Pos {
        int i, ch;
        unsigned off_s, off_v;
    };
    const unsigned stride32 = unsigned(p.block_stride), off_v32 = unsigned(p.off_v);
    auto pos_at = [&](int it, int i) -> Pos {
        Pos q;
        q.i = i;
        q.ch = min(2 * it + team, nch - 1);
        q.off_s = unsigned(i) * stride32 + unsigned(q.ch) * kUnitBytes;
        q.off_v = unsigned(i) * stride32 + off_v32 + unsigned(q.ch) * 8192u;
        return q;
    };
    auto advance = [&](Pos q) -> Pos {
        if (++q.i == n) {
            q.i = 0;
            q.ch = min(q.ch + 2, nch - 1);
            q.off_s = unsigned(q.ch) * kUnitBytes;
            q.off_v = off_v32 + unsigned(q.ch) * 8192u;
        } else {
            q.off_s += stride32;
            q.off_v += stride32;
        }
        return q;
    };
    __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(p.blocks), 0,
                                                                   unsigned(n) * stride32, 0x00020000);
    typedef int v4i_ __attribute__((ext_vector_type(4)));
    typedef int v2i_ __attribute__((ext_vector_type(2)));
    struct VIn {
        v4i_ a, b;
    };
    const unsigned voff = unsigned((((lane >> 3) * 2 + (cw >> 1)) * 16 + 2 * (lane & 7)) * 32 + (cw & 1) * 16);
    auto fetch_v = [&](Pos q) -> VIn {
        VIn v;
        v.a = __builtin_amdgcn_raw_buffer_load_b128(brs, voff, q.off_v, 0);
        v.b = __builtin_amdgcn_raw_buffer_load_b128(brs, voff + 32, q.off_v, 0);
        return v;
    };
    struct SIn {
        v2i_ w[2];
    };
    const unsigned soff[2] = {unsigned((size_t(rtc[0]) * nch) * kUnitBytes + ((cw >> 1) * 32 + ln) * 16 + (cw & 1) * 8),
                              unsigned((size_t(rtc[1]) * nch) * kUnitBytes + ((cw >> 1) * 32 + ln) * 16 + (cw & 1) * 8)};
    auto fetch_s = [&](Pos q) -> SIn {
        SIn v;
        v.w[0] = __builtin_amdgcn_raw_buffer_load_b64(brs, soff[0], q.off_s, 0);
        v.w[1] = __builtin_amdgcn_raw_buffer_load_b64(brs, soff[1], q.off_s, 0);
        return v;
    };
    // private V piece transposed on the way in, as in k_fused: (t, column e, rank pair) at dword
    // t * kVtStride + e * 8 + pair; sixteen 16-bit writes per lane, one 128-bit read per fragment
    unsigned short* const vdst = reinterpret_cast<unsigned short*>(vpriv) + ((lane >> 3) * kVtStride + (lane & 7)) * 2;
    int vsrc_off[2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
        const int b = ln >> 3, t = ln & 7, e = tile * 4 + b;
        vsrc_off[tile] = (t * kVtStride + e * 8 + 4 * hl) * 4;
    }
    auto stage_v = [&](VIn v, int buf) {
        unsigned short* const d = vdst + buf * (kVPriv / 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned a = unsigned(v.a[i]), b = unsigned(v.b[i]);
            d[(2 * i) * 16] = static_cast<unsigned short>(a);
            d[(2 * i) * 16 + 1] = static_cast<unsigned short>(b);
            d[(2 * i + 1) * 16] = static_cast<unsigned short>(a >> 16);
            d[(2 * i + 1) * 16 + 1] = static_cast<unsigned short>(b >> 16);
        }
    };
    auto read_vf = [&](int buf, int tile) -> v8h {
        return *reinterpret_cast<const v8h*>(vpriv + buf * kVPriv + vsrc_off[tile]);
    };
    auto read_u = [&](int i, int rg) -> v8h {
        return *reinterpret_cast<const v8h*>(ucache + ((i * 64 + rg * 32 + ln) * 2 + hl) * 16);
    };

    // permuted identities: A[i'][slot s of half hl] = 1 where i' is the column that slot s of the
    // signed tile holds (8*mf + 4*hl + s/2 + 16*(s%2)), so that identity x tile = tile in the
    // accumulator layout "register v <-> column 8*(v/4) + 4*hl + v%4"
    v8h ident[2];
#pragma unroll
    for (int mf = 0; mf < 2; ++mf)
#pragma unroll
        for (int sl = 0; sl < 8; ++sl)
            ident[mf][sl] = _Float16(ln == 8 * mf + 4 * hl + (sl >> 1) + 16 * (sl & 1) ? 1.0f : 0.0f);

    v16f wacc[2][2];   // [tile][row group]: the weight tile of this chunk, fp32 (starts at a chunk's first block)
    v16f yacc[2][2];   // [row group][token group of my 64 tokens]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) yacc[a][b][v] = 0.0f;

    // shifts that bring the sign bits of a register pair (word bits 8*mf + k + 4*hl and that + 16) to
    // bits 15 and 31: per lane (eight registers) where registers are to spare, else the word is moved
    // down by 4*hl first and the shifts are immediates
    constexpr bool kLaneShift = kRestore;
    unsigned sh[2][4];
#pragma unroll
    for (int mf = 0; mf < 2; ++mf)
#pragma unroll
        for (int k = 0; k < 4; ++k) sh[mf][k] = unsigned(15 - 8 * mf - k) - (kLaneShift ? unsigned(4 * hl) : 0u);

    // first = the chunk's first block: the accumulator starts from zero instead of being cleared
    // beforehand, so that its 64 registers are free during the product stage
    auto magnitude = [&](int tb, v8h uf0, v8h uf1, v8h vf0, v8h vf1) -> v16f {
        v16f z;
#pragma unroll
        for (int v = 0; v < 16; ++v) z[v] = 0.0f;
        return __builtin_amdgcn_mfma_f32_32x32x16_f16((tb >> 1) ? vf1 : vf0, (tb & 1) ? uf1 : uf0, z, 0, 0, 0);
    };
    auto sign_and_add = [&](auto first, int tb, const v16f& m, const SIn& sg) {
        const int tile = tb >> 1, rg = tb & 1;
        const unsigned wrd = unsigned(tile ? sg.w[rg].y : sg.w[rg].x) >> (kLaneShift ? 0 : 4 * hl);
#pragma unroll
        for (int mf = 0; mf < 2; ++mf) {
            unsigned r4[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                h2 c;
                c[0] = _Float16(m[4 * mf + k]);
                c[1] = _Float16(m[4 * mf + k + 8]);
                const unsigned flip = ~(wrd << sh[mf][k]) & 0x80008000u;   // a cleared bit marks a negative sign
                r4[k] = __builtin_bit_cast(unsigned, c) ^ flip;
            }
            if (decltype(first)::value && mf == 0) {
                v16f z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                wacc[tile][rg] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ident[mf], __builtin_bit_cast(v8h, r4), z, 0, 0, 0);
            } else {
                wacc[tile][rg] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ident[mf], __builtin_bit_cast(v8h, r4),
                                                                        wacc[tile][rg], 0, 0, 0);
            }
        }
    };
    // tile-blocks tb = 2 * tile + row group
    auto rebuild = [&](auto first, const SIn& sg, v8h uf0, v8h uf1, v8h vf0, v8h vf1) {
        if (kRestore) {
            // registers to spare: the magnitude product of the next tile-block is issued before the
            // vector work on the current one, which then covers its latency
            v16f m0 = magnitude(0, uf0, uf1, vf0, vf1);
            v16f m1 = magnitude(1, uf0, uf1, vf0, vf1);
            sign_and_add(first, 0, m0, sg);
            m0 = magnitude(2, uf0, uf1, vf0, vf1);
            sign_and_add(first, 1, m1, sg);
            m1 = magnitude(3, uf0, uf1, vf0, vf1);
            sign_and_add(first, 2, m0, sg);
            sign_and_add(first, 3, m1, sg);
        } else {
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) sign_and_add(first, tb, magnitude(tb, uf0, uf1, vf0, vf1), sg);
        }
    };

    // end of a chunk: park my piece of W' diag(1/s) in LDS, then the product stage for both teams' chunks
    auto flush_and_multiply = [&](int it) {
        const int ch = min(2 * it + team, nch - 1);
#pragma unroll
        for (int tile = 0; tile < 2; ++tile)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int c = cw * 64 + tile * 32 + 8 * q4 + 4 * hl;   // first of 4 consecutive columns
                const float4 r = *reinterpret_cast<const float4*>(p.rs + ch * kChunkCols + c);
#pragma unroll
                for (int rg = 0; rg < 2; ++rg) {
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    h4 o;
                    o[0] = _Float16(wacc[tile][rg][4 * q4 + 0] * r.x);
                    o[1] = _Float16(wacc[tile][rg][4 * q4 + 1] * r.y);
                    o[2] = _Float16(wacc[tile][rg][4 * q4 + 2] * r.z);
                    o[3] = _Float16(wacc[tile][rg][4 * q4 + 3] * r.w);
                    *reinterpret_cast<h4*>(wt + (team * kPanelRows + rg * 32 + ln) * kPanelLd + c) = o;
                }
            }
        lds_barrier();   // both tiles parked
        if (kRestore) {
            __half* const wd = static_cast<__half*>(p.wdense);
            for (int idx = tid; idx < 2 * kPanelRows * 32; idx += 512) {   // 16-byte pieces, a row's 32 in a row
                const int tm = idx >> 11, r = (idx >> 5) & 63, piece = idx & 31;
                const int chc = 2 * it + tm, row = (rt0 + (r >> 5)) * kTileRows + (r & 31);
                if (chc < nch && row < p.out)
                    *reinterpret_cast<uint4*>(wd + size_t(row - p.row_begin) * p.in + chc * kChunkCols + piece * 8) =
                        *reinterpret_cast<const uint4*>(wt + (tm * kPanelRows + r) * kPanelLd + piece * 8);
            }
        } else if (tok_w < p.batch) {
            // fragments of my two token groups: [group][in / 16][64 lanes][8]
            const __half* xrow[2];
#pragma unroll
            for (int tg = 0; tg < 2; ++tg)
                xrow[tg] = p.xpack + (size_t(min(tok_w / 32 + tg, (p.batch - 1) / 32)) * (p.in / 16) * 64 + lane) * 8;
            // activation fragments are requested PD steps ahead of their use (they come from L2 or
            // beyond), weight fragments one step ahead (LDS); a step = 16 columns of one of the two tiles
            constexpr int PD = 8;
            const int nks = (2 * it + 1 < nch) ? 32 : 16;   // odd chunk count: the second team's last tile is not a chunk
            const __half* const x0 = xrow[0] + size_t(2 * it) * 16 * 512;
            const __half* const x1 = xrow[1] + size_t(2 * it) * 16 * 512;
            auto wfrag = [&](int ks, int rg) -> v8h {
                return *reinterpret_cast<const v8h*>(wt + ((ks >> 4) * kPanelRows + rg * 32 + ln) * kPanelLd + (ks & 15) * 16 + 8 * hl);
            };
            v8h ring[PD][2];
#pragma unroll
            for (int k = 0; k < PD; ++k) {
                ring[k][0] = *reinterpret_cast<const v8h*>(x0 + size_t(k) * 512);
                ring[k][1] = *reinterpret_cast<const v8h*>(x1 + size_t(k) * 512);
            }
            v8h b0 = wfrag(0, 0), b1 = wfrag(0, 1);
            for (int kb = 0; kb < nks; kb += PD) {   // nks is a multiple of PD
#pragma unroll
                for (int k = 0; k < PD; ++k) {
                    const int ks = kb + k;
                    const v8h a0 = ring[k][0], a1 = ring[k][1];
                    const int kn = min(ks + PD, nks - 1);
                    ring[k][0] = *reinterpret_cast<const v8h*>(x0 + size_t(kn) * 512);
                    ring[k][1] = *reinterpret_cast<const v8h*>(x1 + size_t(kn) * 512);
                    const int k1 = min(ks + 1, nks - 1);
                    const v8h nb0 = wfrag(k1, 0), nb1 = wfrag(k1, 1);
                    yacc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b0, yacc[0][0], 0, 0, 0);
                    yacc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b0, yacc[0][1], 0, 0, 0);
                    yacc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b1, yacc[1][0], 0, 0, 0);
                    yacc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b1, yacc[1][1], 0, 0, 0);
                    b0 = nb0;
                    b1 = nb1;
                }
            }
        }
        lds_barrier();   // tiles free for the next pair of chunks
    };

    Pos q = pos_at(it_first, 0);
    VIn vA = fetch_v(q);
    SIn sA = fetch_s(q);
    q = advance(q);
    VIn vB = fetch_v(q);
    SIn sB = fetch_s(q);
    q = advance(q);
    VIn vC = fetch_v(q);
    // Signs of step s + 3 are requested once step s has used its own (into the same registers) where
    // registers are to spare; else signs run one step behind V (step s + 2 at the start of step s, into
    // the third set) and need a position of their own.
    constexpr bool kSignsLate = kRestore;
    Pos qs = q;       // position of step s + 2
    SIn sC;
    if (kSignsLate) sC = fetch_s(q);
    q = advance(q);   // position of step s + 3
    stage_v(vA, 0);
    v8h vf0 = read_vf(0, 0), vf1 = read_vf(0, 1);
    __syncthreads();   // U cache complete

    int ci = 0, it = it_first;
#define BS_TILE_STEP(S, CUR, NXT, FAR)                                                     \
    {                                                                                      \
        const v8h uf0 = read_u(ci, 0), uf1 = read_u(ci, 1);                                \
        stage_v(v##NXT, ((S) + 1) & 1);                                                    \
        const v8h vn0 = read_vf(((S) + 1) & 1, 0), vn1 = read_vf(((S) + 1) & 1, 1);        \
        if (!kSignsLate) {                                                                 \
            s##FAR = fetch_s(qs);                                                          \
            qs = advance(qs);                                                              \
        }                                                                                  \
        v##CUR = fetch_v(q);                                                               \
        if (ci == 0)                                                                       \
            rebuild(std::true_type{}, s##CUR, uf0, uf1, vf0, vf1);                         \
        else                                                                               \
            rebuild(std::false_type{}, s##CUR, uf0, uf1, vf0, vf1);                        \
        if (kSignsLate) s##CUR = fetch_s(q);                                               \
        q = advance(q);                                                                    \
        vf0 = vn0;                                                                         \
        vf1 = vn1;                                                                         \
        if (++ci == n) {                                                                   \
            ci = 0;                                                                        \
            if (it < it_end) flush_and_multiply(it);                                       \
            ++it;                                                                          \
        }                                                                                  \
    }
    // steps past the last one (count rounded up to a multiple of three) only touch wacc
    for (int s = 0; s < total; s += 3) {
        BS_TILE_STEP(s, A, B, C)
        BS_TILE_STEP(s + 1, B, C, A)
        BS_TILE_STEP(s + 2, C, A, B)
    }
#undef BS_TILE_STEP

    if (kRestore) return;
    // C[i = token][n = row]: lane (row ln), register v holds token 8*(v/4) + 4*hl + v%4 of the group
#pragma unroll
    for (int rg = 0; rg < 2; ++rg)
#pragma unroll
        for (int tg = 0; tg < 2; ++tg)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tok = tok_w + tg * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
                const int row = (rt0 + rg) * kTileRows + ln;
                if (tok < p.batch && row < p.out) store_y(p, size_t(tok) * p.out + row, yacc[rg][tg][v]);
            }
}

static bool tile_fits(const KParams& p) {   // U cache in LDS; one 32-bit buffer descriptor over the loaded blocks
    return p.n_loaded <= kTileMaxBlocks && p.xpack != nullptr && size_t(p.n_loaded) * p.block_stride < (size_t(1) << 32);
}

static hipError_t launch_tile(const KParams& p, hipStream_t st) {
    const size_t smem = size_t(kTileFixedLds) + size_t(p.n_loaded) * 2048;
    static std::atomic<bool> attr_set{false};   // setting the attribute twice is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tile<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kTileFixedLds + kTileMaxBlocks * 2048);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    launch_xpack(p, st);
    dim3 grid((p.out + 2 * kTileRows - 1) / (2 * kTileRows), (p.batch + kTileTokens - 1) / kTileTokens);
    hipLaunchKernelGGL(k_tile<false>, grid, dim3(512), smem, st, p);
    return hipGetLastError();
}

// W' diag(1/s) of the loaded prefix as a dense fp16 matrix [out][in] (row-major) at a.wdense.
// Estimated duration of restoring `rows` rows (microseconds) and the number of column slices per row
// tile pair it assumes: rounds of 256 workgroups x (chunk pairs per workgroup x (~0.93 us per block +
// ~2.5 us for the flush) + ~3 us fixed) (a slab of 2048 rows of 28672x8192: ~40 us inside a run of
// slabs, the whole matrix 520-600).
double restore_time_us(int rows, int in, int n_loaded, int* slices_out) {
    const int iters = (in / kChunkCols + 1) / 2;
    const int row_wgs = (rows + 2 * kTileRows - 1) / (2 * kTileRows);
    int slices = 1;
    double best = 0.0;
    for (int sl = 1; sl <= iters; sl *= 2) {
        const int per = (iters + sl - 1) / sl;
        const double t = double((row_wgs * sl + 255) / 256) * (per * (0.93 * n_loaded + 2.5) + 3.0);
        if (sl == 1 || t < best) {
            best = t;
            slices = sl;
        }
    }
    if (slices_out) *slices_out = slices;
    return best;
}

hipError_t launch_restore(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    if (a.n_loaded < 1 || !restore_fits(p.block_stride, a.n_loaded) || p.wdense == nullptr) return hipErrorInvalidValue;
    const size_t smem = size_t(kTileFixedLds) + size_t(p.n_loaded) * 2048;
    static std::atomic<bool> attr_set{false};   // setting the attribute twice is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tile<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kTileFixedLds + kTileMaxBlocks * 2048);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // Column slices per row tile pair: few, long workgroups pay the fixed costs (copy of the U
    // rows, first loads, ~3 us) less often, many short ones fill the last round of the 256
    // compute units better (restore_time_us).
    const int slab_rows = a.rows ? a.rows : p.out;
    if (a.row_begin % 256 || a.row_begin < 0 || a.row_begin >= p.out || slab_rows < 1) return hipErrorInvalidValue;
    const int rows = min(slab_rows, p.out - a.row_begin);
    const int row_wgs = (rows + 2 * kTileRows - 1) / (2 * kTileRows);
    int slices = 1;
    restore_time_us(rows, p.in, p.n_loaded, &slices);
    hipLaunchKernelGGL(k_tile<true>, dim3(row_wgs, slices), dim3(512), smem, st, p);
    return hipGetLastError();
}
int restore_max_blocks() { return kTileMaxBlocks; }
// U cache in LDS; the kernel reaches the loaded blocks through one buffer descriptor with 32-bit offsets
bool restore_fits(size_t block_stride, int n_loaded) {
    return n_loaded <= kTileMaxBlocks && size_t(n_loaded) * block_stride < (size_t(1) << 32);
}

// Estimated durations (microseconds, constants fitted to measurements).  k_fused: per round of
// 256 workgroups ~8 us fixed + ~0.80 us per block and pair of column chunks of a workgroup; later
// workgroups start as earlier ones end, so rounds beyond the first count fractionally.
double fused_time_us(int out, int in, int batch, int n_loaded, int part_slots) {
    const int row_tiles = (out + 2 * kTileRows - 1) / (2 * kTileRows), chunk_pairs = (in / kChunkCols + 1) / 2;
    const int split = small_batch_split(out, in, batch, part_slots);
    const int wgs = row_tiles * ((batch + 31) / 32) * split;
    const double rounds = wgs <= 256 ? 1.0 : wgs / 256.0;
    return rounds * (8.0 + 0.80 * n_loaded * ((chunk_pairs + split - 1) / split)) + (split > 1 ? 4.0 : 0.0);
}
// k_tile: per pair of column chunks ~0.9 us per block for the rebuild + 12-14 us for the product
// (14 when several token tiles of a row tile run at once, 6.5 up to 256 tokens, where only one
// wavefront per SIMD has tokens to multiply); 15 % less of both when the chip is not full.
double tile_time_us(int out, int in, int batch, int n_loaded) {
    const int row_tiles = (out + 2 * kTileRows - 1) / (2 * kTileRows), chunk_pairs = (in / kChunkCols + 1) / 2;
    const int wgs = row_tiles * ((batch + kTileTokens - 1) / kTileTokens);
    const double rounds = wgs <= 256 ? 1.0 : wgs / 256.0, scale = wgs <= 256 ? 0.85 : 1.0;
    return rounds * (15.0 + chunk_pairs * scale * (0.9 * n_loaded + (batch > 512 ? 14.0 : batch > 256 ? 12.0 : 6.5)));
}

hipError_t launch_panel(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    if (a.n_loaded < 1 || a.batch < 1) return hipErrorInvalidValue;
    // 33..64 tokens: k_fused rebuilds the signed tiles twice; with many row tiles the weight-tile
    // kernel, which rebuilds once, is the cheaper one
    if (a.batch > 32 && a.batch <= kFusedMaxBatch && fused_fits(p) && tile_fits(p) &&
        tile_time_us(p.out, p.in, p.batch, p.n_loaded) < fused_time_us(p.out, p.in, p.batch, p.n_loaded, p.part_slots))
        return launch_tile(p, st);
    if (a.batch <= kFusedMaxBatch && fused_fits(p)) return launch_fused(p, st);
    if (a.batch > kFusedMaxBatch && tile_fits(p)) return launch_tile(p, st);
    if (a.batch > 256) return launch_panel_t<4>(p, st);
    if (a.batch > 128) return launch_panel_t<2>(p, st);
    return launch_panel_t<1>(p, st);
}

}  // namespace bitstack
