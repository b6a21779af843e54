// HIP kernels (gfx950 / CDNA4) for the BitStack linear layer
//     y = ( sum_i S_i (.) (U_i V_i^T) ) diag(1/s) x          (Eq. 4 + Eq. 8)
// evaluated from the packed residual blocks, never materialising the weight.
//
// Decode kernel (one token).  Per block the method needs, for every output row o
// and rank r, the signed sum  Z[o,r] = sum_j S[o,j] * T[j,r]  with the V-scaled
// activation panel  T[j,r] = V[j,r] * x[j]/s[j]  (per-rank identity
// (S (.) u v^T) x = u (.) (S (v (.) x))), followed by  y[o] += sum_r U[o,r] Z[o,r].
// Z is a dense contraction with a 1-bit operand, 16 multiply-adds per sign bit, so
// it runs on the matrix cores (v_mfma_i32_32x32x32_i8):
//   * sign operand: the packed words are turned into int8 operands with a single
//     bitwise AND per four signs (mask 0x01010101 << t keeps bit t of every byte,
//     value 0 or 2^t); the device layout is chosen so that this is all it takes.
//   * panel operand: T is quantised per (block, column slab) to 16-bit fixed point
//     against the slab's exact max |T|, pre-shifted by 2^-(3 - t%4) so that all
//     column classes of a nibble land on one scale, and split into a high and a
//     low signed byte: 16 ranks x {hi, lo} = the 32 rows of the A operand.
//   * accumulation is exact int32 (the high-nibble classes are brought down with
//     one shift of the sign words, so a single accumulator set serves all eight
//     classes); S = 2B - 1 is undone with the exact integer column sums of the panel.
// Work is split over (block, column slab, row slab) workgroups.  Each writes its
// fp32 partial sums to its own workspace row; the last workgroup to arrive for a
// row slab (one agent-scope counter per slab) adds the rows up in a fixed order,
// rounds once and stores y, so the result does not depend on arrival order.
// (Floating-point atomics across the chip's eight L2s proved far slower than the
// whole sign stream, and a fence per thread slower still.)
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kernels.h"
#include "kparams.h"
#include "layout.h"

namespace bitstack {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef short v2s __attribute__((ext_vector_type(2)));

#ifdef BITSTACK_TRACE
// Development aid (off in the shipped build): wave 0 of every workgroup stamps the
// constant-rate clock at phase boundaries.
__device__ unsigned long long g_trace[8192 * 8];
#define BS_TRACE2(role, i)                                                            \
    do {                                                                             \
        if (lane == 0 && (wave == 0 || wave == kConsumers) && blockIdx.x < 1024 && (i) < 24) \
            g_trace2[(blockIdx.x * 2 + (role)) * 24 + (i)] = wall_clock64();          \
    } while (0)
__device__ unsigned long long g_trace2[1024 * 2 * 24];
extern "C" int bitstack_debug_trace2(unsigned long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace2), size_t(n) * 8);
}
#define BS_TRACE(i)                                                                  \
    do {                                                                             \
        if (tid == 0 && blockIdx.x < 8192) g_trace[blockIdx.x * 8 + (i)] = wall_clock64(); \
    } while (0)
extern "C" int bitstack_debug_trace(unsigned long long* host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), size_t(n) * 8);
}
#else
#define BS_TRACE(i) do { } while (0)
#define BS_TRACE2(role, i) do { } while (0)
#endif

DecodeTuning& decode_tuning() {
    static DecodeTuning t;
    return t;
}

// ---------------------------------------------------------------- y = 0 (no block loaded)
__global__ void k_zero(KParams p) {
    size_t n = size_t(p.batch) * p.out;
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += size_t(gridDim.x) * blockDim.x)
        store_y(p, i, 0.0f);
}

hipError_t launch_zero(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    size_t n = size_t(a.batch) * a.geo.out;
    int blocks = int((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_zero, dim3(blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------- read-stream probe
// Reads a buffer once with 128-bit loads and folds it into one word per thread: the
// achievable HBM read rate that the decode kernel's sign stream is measured against.
__global__ __launch_bounds__(256) void k_stream_read(const uint4* __restrict__ src, size_t n16, unsigned* sink) {
    uint4 a = {0, 0, 0, 0};
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        a.x ^= v0.x ^ v1.x ^ v2.x ^ v3.x;
        a.y ^= v0.y ^ v1.y ^ v2.y ^ v3.y;
        a.z ^= v0.z ^ v1.z ^ v2.z ^ v3.z;
        a.w ^= v0.w ^ v1.w ^ v2.w ^ v3.w;
    }
    for (; i < n16; i += stride) {
        const uint4 v = src[i];
        a.x ^= v.x; a.y ^= v.y; a.z ^= v.z; a.w ^= v.w;
    }
    const unsigned r = a.x ^ a.y ^ a.z ^ a.w;
    if (r == 0x9E3779B9u) sink[0] = r;  // practically never; keeps the loads alive
}

hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int blocks, hipStream_t st) {
    hipLaunchKernelGGL(k_stream_read, dim3(blocks), dim3(256), 0, st, static_cast<const uint4*>(buf),
                       bytes / 16, static_cast<unsigned*>(sink));
    return hipGetLastError();
}

// ---------------------------------------------------------------- reference kernel
// One wavefront per output row, up to 8 tokens per pass, plain fp32 vector math:
// restores each weight element m = sum_r U[o,r] V[j,r] with its sign and multiplies
// by x/s.  Slow (16 FMAs per sign bit on the vector ALUs) but independent of every
// trick the fast kernels use; serves any batch.
constexpr int kRefTokens = 8;

__global__ __launch_bounds__(256) void k_reference(KParams p) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int tok0 = blockIdx.y * kRefTokens;
    if (row >= p.out) return;
    const int ntok = min(kRefTokens, p.batch - tok0);
    float acc[kRefTokens];
#pragma unroll
    for (int b = 0; b < kRefTokens; ++b) acc[b] = 0.0f;
    for (int i = 0; i < p.n_loaded; ++i) {
        const unsigned char* blk = p.blocks + size_t(i) * p.block_stride;
        const uint32_t* sw = reinterpret_cast<const uint32_t*>(blk);
        const __half* V = reinterpret_cast<const __half*>(blk + p.off_v);
        const __half* U = reinterpret_cast<const __half*>(blk + p.off_u) + size_t(row) * kRank;
        float u[kRank];
#pragma unroll
        for (int r = 0; r < kRank; ++r) u[r] = __half2float(U[r]);
        for (int col = lane; col < p.in; col += 64) {
            const uint32_t word = sw[sign_word_index(p.in, row, col >> 5)];
            const bool plus = (word >> (col & 31)) & 1u;
            const size_t vb = v_index(col, 0);
            float m = 0.0f;
#pragma unroll
            for (int r = 0; r < kRank; ++r) m = fmaf(u[r], __half2float(V[vb + size_t(r) * 16]), m);
            m = plus ? m : -m;
            const float rsj = p.rs[col];
#pragma unroll
            for (int b = 0; b < kRefTokens; ++b)
                if (b < ntok) acc[b] = fmaf(m, __half2float(p.x[size_t(tok0 + b) * p.in + col]) * rsj, acc[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < kRefTokens; ++b) {
        float v = acc[b];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0 && b < ntok) store_y(p, size_t(tok0 + b) * p.out + row, v);
    }
}

hipError_t launch_reference(const LaunchArgs& a, hipStream_t st) {
    KParams p = make_params(a);
    dim3 grid((a.geo.out + 3) / 4, (a.batch + kRefTokens - 1) / kRefTokens);
    hipLaunchKernelGGL(k_reference, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------- decode kernel
constexpr float kQMax = 32512.0f;  // |q| <= 127*256: the high byte stays in int8 after +128 rounding
constexpr int kMaxBlocksPerWg = 32;
constexpr int kMaxPre = 8;           // blocks per workgroup whose slab maxima are ready at the first barrier
constexpr int kConsumers = 8;      // wavefronts that stream signs through the matrix cores
constexpr int kProducers = 4;      // wavefronts that build the panel fragments
constexpr int kTilesPerWave = 4;   // 32-row tiles per consumer wavefront
constexpr int kDecodeRows = kConsumers * kTilesPerWave * kTileRows;   // rows per workgroup (1024)

__device__ __forceinline__ float wave_max(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// One workgroup owns a row slab (1024 rows) and a column slab (KS columns) and walks
// through every n_bg-th block of the loaded prefix, keeping its fp32 results in
// registers.  The twelve wavefronts are specialised:
//   * producers (4, one per SIMD) build, for the next block, the int8 panel
//     fragments of the slab in LDS (double buffered), the integer column sums and a
//     copy of the U rows;
//   * consumers (8, two per SIMD) own 128 rows each.  Their only global loads are the
//     sign units, issued unconditionally (buffer loads whose out-of-range lanes
//     return zero without touching memory) one block ahead into a register window,
//     so the in-order memory counter never makes them wait for anything younger
//     than the unit they need: 16 KiB per wavefront, 128 KiB per compute unit in
//     flight, which is what the HBM pipe needs to stay full.  Per unit: 8 masks x
//     (4 ANDs + 1 matrix-core instruction).  Per block: a short epilogue folds the
//     int32 accumulators into running fp32 sums using U, scale and column sums from
//     LDS.
// One barrier per block separates "fragments of block q+1 written" from "fragments of
// block q read".
// raw V values of GG consecutive 16-value panel groups (one thread's share of a slab)
template <int GG>
struct RawT {
    uint4 v[GG][2];
};

template <int KS>
__global__ __launch_bounds__((kConsumers + kProducers) * 64, 3) void k_decode_old(KGroup grp) {
    constexpr int NCH = KS / kChunkCols;   // sign chunks per slab
    constexpr int R = kTilesPerWave;       // 32-row tiles per consumer wavefront
    constexpr int RS = kDecodeRows;
    constexpr int PT = kProducers * 64;    // producer threads
    constexpr int NT = (kConsumers + kProducers) * 64;
    constexpr int G = KS / PT;             // 16-value panel groups per producer thread
    static_assert(KS % PT == 0 && G >= 1, "slab must give every producer thread whole groups");
    constexpr int FRAG_BYTES = KS * 32;
    constexpr int U_BYTES = RS * 32;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    v4i* frag0 = reinterpret_cast<v4i*>(smem);                                   // [2][NCH*8][64] x 16 B
    uint4* ulds = reinterpret_cast<uint4*>(smem + 2 * FRAG_BYTES);               // [2][RS][2] x 16 B
    float* xs = reinterpret_cast<float*>(smem + 2 * FRAG_BYTES + 2 * U_BYTES);   // [KS]
    float* amax_w = xs + KS;                                                     // [kProducers][kMaxBlocksPerWg]
    int* cs = reinterpret_cast<int*>(amax_w + kProducers * kMaxBlocksPerWg);     // [3][32]
    unsigned* flag = reinterpret_cast<unsigned*>(cs + 96);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool producer = wave >= kConsumers;
    const int ptid = tid - kConsumers * 64;   // producer thread index (valid when producer)

    // which stack of the group this workgroup serves (uniform)
    int gi = 0;
    while (gi + 1 < grp.count && blockIdx.x >= grp.base[gi + 1]) ++gi;
    const KParams& p = grp.s[gi];
    // workgroup id -> work item, contiguous ranges of items per XCD (ids are dealt
    // round-robin to the 8 XCDs), so that the workgroups sharing a V slab share an L2.
    // The id range of a stack is padded to a multiple of 8; ids past the last item leave.
    const unsigned local = blockIdx.x - grp.base[gi];
    const unsigned q8 = (grp.base[gi + 1] - grp.base[gi]) >> 3;
    const unsigned item = (local & 7u) * q8 + (local >> 3);
    if (item >= unsigned(p.n_rs) * unsigned(p.n_ks) * unsigned(p.n_bg)) return;
    const int rs_i = item % p.n_rs;
    const int ks_i = (item / p.n_rs) % p.n_ks;
    const int bg_i = item / (p.n_rs * p.n_ks);
    const int slot_i = bg_i * p.n_ks + ks_i;   // this workgroup's partial-sum row
    const int nb = (p.n_loaded - bg_i + p.n_bg - 1) / p.n_bg;   // blocks bg_i, bg_i + n_bg, ...

    const int nch_total = p.in / kChunkCols;
    const int c0 = ks_i * NCH;               // first chunk of this slab
    const int k0 = c0 * kChunkCols;
    const int n_rt = p.out / kTileRows;
    const int row0 = rs_i * RS;
    auto block_index = [&](int q) { return bg_i + q * p.n_bg; };
    auto block_ptr = [&](int q) { return p.blocks + size_t(block_index(q)) * p.block_stride; };

    auto amax_of = [&](int q) {
        float a = amax_w[q];
#pragma unroll
        for (int w = 1; w < kProducers; ++w) a = fmaxf(a, amax_w[w * kMaxBlocksPerWg + q]);
        return a;
    };

    // quantise block q's slab of the panel from raw V into fragment buffer (q & 1): thread ti of a
    // team of KS / GG threads takes the GG consecutive 16-value groups ti * GG ..: panel position
    // (ti * GG) / 16 (one 32-column operand of one class) and the ranks rk0 .. rk0 + GG - 1.
    // The producers use it with 4 groups per thread; block 0 is done by the consumers (twice the
    // threads, idle until their first signs arrive) from the raw values they fetched at entry.
    auto quantise = [&](int ti, int q, const auto raw) {
        constexpr int GG = int(sizeof(raw.v) / sizeof(raw.v[0]));
        v4i* frag = frag0 + (q & 1) * (FRAG_BYTES / 16);
        int* csq = cs + (q % 3) * 32;
        const float amax = amax_of(q);
        const float inv = amax > 0.0f ? (kQMax / 32767.0f) / amax : 0.0f;
        const int gbase = ti * GG;             // first group of this thread
        const int pos = gbase >> 4, rk0 = gbase & 15;
        const int g = pos & 1, t = (pos >> 1) & 7, c = pos >> 4;
        // the sign byte of class t is 2^(t%4) (high-nibble classes are shifted down by
        // the consumers): pre-dividing by it puts every class on one scale,
        // (sign byte) * q = 32512 * T / amax
        const int tc = t & 3;
        const float f = inv * __int_as_float((127 - tc) << 23);   // inv * 2^-tc
        float xf[16];
        {
            const float4* xg = reinterpret_cast<const float4*>(xs + pos * 16);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float4 v = xg[k];
                xf[4 * k] = v.x * f; xf[4 * k + 1] = v.y * f; xf[4 * k + 2] = v.z * f; xf[4 * k + 3] = v.w * f;
            }
        }
        int sums[GG][2];
#pragma unroll
        for (int m = 0; m < GG; ++m) {
            const uint4 va = raw.v[m][0], vb = raw.v[m][1];
            const unsigned vw[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
            unsigned qq[8];
#pragma unroll
            for (int e2 = 0; e2 < 8; ++e2) {
                typedef _Float16 h2v __attribute__((ext_vector_type(2)));
                const h2v h = __builtin_bit_cast(h2v, vw[e2]);
                // + 128 (in units of the 16-bit code) rides along in the multiply-add that also converts
                // the fp16 factor: the high byte of q + 128 is round(q / 256), the low byte q ^ 0x80
                constexpr float kHalfByte = 128.0f / 32767.0f;
                const v2s qv = __builtin_amdgcn_cvt_pknorm_i16(__builtin_fmaf(float(h[0]), xf[2 * e2], kHalfByte),
                                                               __builtin_fmaf(float(h[1]), xf[2 * e2 + 1], kHalfByte));
                qq[e2] = __builtin_bit_cast(unsigned, qv);
            }
            v4i H, L;
            int sH = 0, sL = 0;
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4) {
                const unsigned hi = __builtin_amdgcn_perm(qq[2 * w4 + 1], qq[2 * w4], 0x07050301u);
                const unsigned lo = __builtin_amdgcn_perm(qq[2 * w4 + 1], qq[2 * w4], 0x06040200u) ^ 0x80808080u;
                H[w4] = int(hi);
                L[w4] = int(lo);
                sH = __builtin_amdgcn_sdot4(int(hi), 0x01010101, sH, false);
                sL = __builtin_amdgcn_sdot4(int(lo), 0x01010101, sL, false);
            }
            sums[m][0] = sH << tc;
            sums[m][1] = sL << tc;
            const int r = rk0 + m;
            const int lane_hi = g * 32 + 8 * (r >> 2) + (r & 3);
            frag[(c * 8 + t) * 64 + lane_hi] = H;
            frag[(c * 8 + t) * 64 + lane_hi + 4] = L;
        }
        // integer column sums of the quantised panel per rank and byte half: add up the
        // lanes that hold the same ranks (lane bits above log2(16 / GG)), then one LDS
        // atomic per rank, half and wavefront
        constexpr int RSTEP = 16 / GG;   // lanes per full set of ranks
#pragma unroll
        for (int m = 0; m < GG; ++m)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                int v = sums[m][h];
#pragma unroll
                for (int off = RSTEP; off < 64; off <<= 1) v += __shfl_xor(v, off);
                sums[m][h] = v;
            }
        if (lane < RSTEP) {
#pragma unroll
            for (int m = 0; m < GG; ++m) {
                atomicAdd(&csq[rk0 + m], sums[m][0]);
                atomicAdd(&csq[16 + rk0 + m], sums[m][1]);
            }
        }
    };

    BS_TRACE(0);
    // Both roles pass the same barriers: P1 (x/s slab and the first blocks' maxima in LDS), P2
    // (remaining maxima; only if the workgroup has more than kMaxPre blocks), P3 (block 0
    // staged, by the consumers), then one per block.
    if (producer) {
        // ============================================================== producers
        // one producer wave shares a SIMD with two consumer waves that are almost never
        // stalled; without a raised issue priority it only gets their leftovers
        __builtin_amdgcn_s_setprio(2);
        constexpr int PER = U_BYTES / 16 / PT;   // 16-byte pieces of U per producer thread
        constexpr int XP = KS / PT;              // consecutive panel positions per producer thread
        // Raw V slab and U rows of a block are fetched one stage ahead (always issued, for
        // a block index clamped to the last one, so that the in-order memory counter lets
        // the older set be consumed while the younger one is still in flight).
        using Raw = RawT<G>;
        struct URows {
            uint4 u[PER];
        };
        static_assert(G == 4 || G == 2 || G == 1, "group mapping");
        auto load_raw = [&](int q) -> Raw {
            Raw raw;
            const unsigned char* blk = block_ptr(max(min(q, nb - 1), 0));
            const uint4* vsl = reinterpret_cast<const uint4*>(blk + p.off_v) + size_t(c0) * 256 * 2 +
                               size_t(ptid) * G * 2;
#pragma unroll
            for (int m = 0; m < G; ++m) {
                raw.v[m][0] = vsl[m * 2];
                raw.v[m][1] = vsl[m * 2 + 1];
            }
            // keep these loads where they are: scheduled below the code that consumes the
            // older set, the consumer of that set would have to drain them as well
            __builtin_amdgcn_sched_barrier(0);
            return raw;
        };
        auto load_u = [&](int q) -> URows {
            URows ur;
            const unsigned char* blk = block_ptr(max(min(q, nb - 1), 0));
            // rows past the end of the matrix: re-read the last valid piece (never used for output)
            const uint4* usrc = reinterpret_cast<const uint4*>(blk + p.off_u);
            const int last_piece = p.out * 2 - 1;
#pragma unroll
            for (int k = 0; k < PER; ++k) ur.u[k] = usrc[min(row0 * 2 + ptid + k * PT, last_piece)];
            __builtin_amdgcn_sched_barrier(0);
            return ur;
        };
        auto store_u = [&](int q, const URows ur) {
            uint4* udst = ulds + (q & 1) * (U_BYTES / 16);
#pragma unroll
            for (int k = 0; k < PER; ++k) udst[ptid + k * PT] = ur.u[k];
        };
        // ---- activation slab x/s in panel order (once per workgroup); the per-channel
        // maxima of my first blocks and block 0's raw data are requested at the same time
        if (ptid < 96) cs[ptid] = 0;
        constexpr int NPRE = kMaxPre;   // blocks whose maxima are fetched before the first barrier
        struct alignas(XP * 2) HVec {
            __half h[XP];
        };
        HVec hv[NPRE];
        float xv[XP], rv[XP];
#pragma unroll
        for (int m = 0; m < XP; ++m) {
            const int idx = ptid * XP + m;
            const int e = idx & 15, g = (idx >> 4) & 1, t = (idx >> 5) & 7, c = idx >> 8;
            const int col = k0 + panel_col(c, t, g, e);
            xv[m] = __half2float(p.x[col]);
            rv[m] = p.rs[col];
        }
#pragma unroll
        for (int k = 0; k < NPRE; ++k) {
            const __half* vm = p.vmax + size_t(block_index(min(k, nb - 1))) * p.in + size_t(c0) * kChunkCols +
                               ptid * XP;
            hv[k] = *reinterpret_cast<const HVec*>(vm);
        }
        // ---- exact max |V[j][r] * xs[j]| over the slab for each of my blocks:
        //      max_j |xs[j]| * max_r |V[j][r]|, the inner maximum stored at pack time.
        //      The first NPRE blocks are done from registers before the first barrier.
        float xa[XP];
#pragma unroll
        for (int m = 0; m < XP; ++m) {
            const float v = xv[m] * rv[m];
            xs[ptid * XP + m] = v;
            xa[m] = fabsf(v);
        }
        auto slab_max = [&](int qb) {
#pragma unroll
            for (int k = 0; k < NPRE; ++k) {
                if (qb + k < nb) {
                    float a = 0.0f;
#pragma unroll
                    for (int m = 0; m < XP; ++m) a = fmaxf(a, xa[m] * __half2float(hv[k].h[m]));
                    a = wave_max(a);
                    if (lane == 0) amax_w[(wave - kConsumers) * kMaxBlocksPerWg + qb + k] = a;
                }
            }
        };
        BS_TRACE2(1, 16);
        slab_max(0);
        BS_TRACE2(1, 17);
        lds_barrier();   // P1
        BS_TRACE(1);
        BS_TRACE2(1, 18);
        if (nb > NPRE) {   // same for the whole workgroup
            for (int qb = NPRE; qb < nb; qb += NPRE) {
#pragma unroll
                for (int k = 0; k < NPRE; ++k) {
                    const __half* vm = p.vmax + size_t(block_index(min(qb + k, nb - 1))) * p.in +
                                       size_t(c0) * kChunkCols + ptid * XP;
                    hv[k] = *reinterpret_cast<const HVec*>(vm);
                }
                slab_max(qb);
            }
            lds_barrier();   // P2
        }
        BS_TRACE(2);
        Raw ra;
        Raw rb = load_raw(1);
        BS_TRACE2(1, 19);
        lds_barrier();   // P3 (block 0 is staged by the consumers)
        BS_TRACE2(1, 22);
        BS_TRACE(3);
        // interval q: stage block q + 1 (raw V already here), fetch block q + 2's raw V
        for (int q = 0; q < nb; q += 2) {
            BS_TRACE2(1, 2 * q);
            if (ptid < 32) cs[((q + 2) % 3) * 32 + ptid] = 0;   // last read two barriers ago
            ra = load_raw(q + 2);
            if (q + 1 < nb) {
                quantise(ptid, q + 1, rb);
                store_u(q + 1, load_u(q + 1));   // producers have slack: latency exposed here is free
            }
            BS_TRACE2(1, 2 * q + 1);
            lds_barrier();
            if (q + 1 < nb) {
                BS_TRACE2(1, 2 * q + 2);
                if (ptid < 32) cs[((q + 3) % 3) * 32 + ptid] = 0;
                rb = load_raw(q + 3);
                if (q + 2 < nb) {
                    quantise(ptid, q + 2, ra);
                    store_u(q + 2, load_u(q + 2));
                }
                BS_TRACE2(1, 2 * q + 3);
                lds_barrier();
            }
        }
    } else {
        // ============================================================== consumers
        // sign window: win[c][tl] holds unit (chunk c, tile tl) of the current block until it
        // is used, then the same unit of the next block
        v4i win[NCH][R];
        unsigned soff[R];   // byte offset of (tile, first chunk of slab, lane) inside a block
        const unsigned sign_bytes = p.sign_bytes_total;   // bytes covered by the buffer descriptor
        __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(p.blocks), 0, sign_bytes, 0x00020000);
        // per-lane offset of (block q, tile tl, first chunk of the slab); for a block or tile
        // that does not exist an offset just past the descriptor (reads as zero, no traffic;
        // even unchecked it would stay inside the image)
        const unsigned skip_off = sign_bytes + unsigned(lane) * 16u;
        auto unit_off = [&](int q, int tl) -> unsigned {
            const bool ok = q < nb && soff[tl] != 0xFFFFFFFFu;
            return ok ? unsigned(block_index(q)) * unsigned(p.block_stride) + soff[tl] : skip_off;
        };
        float yacc[R];
#pragma unroll
        for (int tl = 0; tl < R; ++tl) {
            const int rt = rs_i * (kConsumers * R) + wave * R + tl;
            soff[tl] = rt < n_rt ? unsigned((size_t(rt) * nch_total + c0) * kUnitBytes) + unsigned(lane) * 16u
                                 : 0xFFFFFFFFu;
            yacc[tl] = 0.0f;
        }

        // Two tiles at a time (32 accumulator registers) against the whole slab, so that the
        // sign window, not the accumulators, gets the registers.
        auto compute = [&](int q) {
            const v4i* frag = frag0 + (q & 1) * (FRAG_BYTES / 16);
            const int part = lane >> 5;   // epilogue: 0 = high bytes, 1 = low bytes
            const float dq = amax_of(q) / kQMax;
            const int* csq = cs + (q % 3) * 32 + part * 16;
            const uint4* ub = ulds + (q & 1) * (U_BYTES / 16) + (wave * R * kTileRows + (lane & 31)) * 2;
#pragma unroll
            for (int tp = 0; tp < R; tp += 2) {
                v16i acc[2];
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[k][v] = 0;
                unsigned noff[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) noff[k] = unit_off(q + 1, tp + k);
                v4i Tf = frag[lane];
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        // next fragment is requested before this one is used (LDS latency
                        // hidden behind the matrix-core instructions of this one; requesting two
                        // steps ahead measured no faster)
                        v4i Tn = Tf;
                        if (c * 8 + t + 1 < NCH * 8) Tn = frag[(c * 8 + t + 1) * 64 + lane];
                        const int mask = 0x01010101 << (t & 3);
                        if (t == 4) {   // high-nibble classes: bit 4+t' of a byte becomes bit t'
#pragma unroll
                            for (int k = 0; k < 2; ++k)
#pragma unroll
                                for (int w = 0; w < 4; ++w)
                                    win[c][tp + k][w] = int(unsigned(win[c][tp + k][w]) >> 4);
                        }
#pragma unroll
                        for (int k = 0; k < 2; ++k) {
                            const v4i B = win[c][tp + k] & mask;
                            acc[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Tf, B, acc[k], 0, 0, 0);
                        }
                        Tf = Tn;
                    }
                    // this chunk's window slots now take the same chunk of the next block (not
                    // earlier: old and new contents would both need registers)
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int k = 0; k < 2; ++k)
                        win[c][tp + k] =
                            __builtin_amdgcn_raw_buffer_load_b128(rsrc, noff[k] + c * kUnitBytes, 0, 0);
                }
                // epilogue: undo S = 2B - 1, weight by U, reduce over ranks
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int tl = tp + k;
                    const uint4 ua = ub[tl * kTileRows * 2], uc = ub[tl * kTileRows * 2 + 1];
                    const unsigned uw[8] = {ua.x, ua.y, ua.z, ua.w, uc.x, uc.y, uc.z, uc.w};
                    float sum = 0.0f;
#pragma unroll
                    for (int r2 = 0; r2 < 8; ++r2) {
                        const __half2 h = *reinterpret_cast<const __half2*>(&uw[r2]);
                        const int z0 = (acc[k][2 * r2] << 1) - csq[2 * r2];
                        const int z1 = (acc[k][2 * r2 + 1] << 1) - csq[2 * r2 + 1];
                        sum = fmaf(float(z0), __low2float(h), sum);
                        sum = fmaf(float(z1), __high2float(h), sum);
                    }
                    const float other = __shfl_xor(sum, 32);
                    yacc[tl] = fmaf(256.0f * sum + other, dq, yacc[tl]);   // meaningful in lanes 0..31
                }
            }
        };

        // Block 0 is staged by the consumers: they have twice the producers' threads, two
        // wavefronts per SIMD, and nothing else to do until their first signs arrive (0.7 us
        // against 3.5 us in the producers).  Its raw V values and U rows are requested first, then
        // the whole sign window of block 0 (loads return in order: what is needed first is asked
        // for first).  Issuing the window takes until ~6 us after entry when every compute unit
        // asks at once (requests are accepted at the rate data returns); asking for half of it
        // here and the rest at the start of block 0, or for all of it after the barriers,
        // measured 2-5 % slower.
        constexpr int CT = kConsumers * 64;
        constexpr int CG = KS >= CT ? KS / CT : 1;   // 16-value groups per consumer thread
        constexpr int CACT = KS / CG;                // consumer threads that quantise
        constexpr int UPER = U_BYTES / 16 / CT;
        static_assert(UPER == 4, "four named registers below (an array of load results ends up in scratch memory)");
        RawT<CG> r0;
        uint4 u00, u01, u02, u03;
        {
            const unsigned char* blk = block_ptr(0);
            const uint4* vsl = reinterpret_cast<const uint4*>(blk + p.off_v) + size_t(c0) * 256 * 2 +
                               size_t(min(tid, CACT - 1)) * CG * 2;
#pragma unroll
            for (int m = 0; m < CG; ++m) {
                r0.v[m][0] = vsl[m * 2];
                r0.v[m][1] = vsl[m * 2 + 1];
            }
            const uint4* usrc = reinterpret_cast<const uint4*>(blk + p.off_u);
            const int last_piece = p.out * 2 - 1;   // rows past the end: re-read the last valid piece
            u00 = usrc[min(row0 * 2 + tid, last_piece)];
            u01 = usrc[min(row0 * 2 + tid + CT, last_piece)];
            u02 = usrc[min(row0 * 2 + tid + 2 * CT, last_piece)];
            u03 = usrc[min(row0 * 2 + tid + 3 * CT, last_piece)];
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int tl = 0; tl < R; ++tl)
                win[c][tl] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, unit_off(0, tl) + c * kUnitBytes, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        BS_TRACE2(0, 16);
        ulds[tid] = u00;
        ulds[tid + CT] = u01;
        ulds[tid + 2 * CT] = u02;
        ulds[tid + 3 * CT] = u03;
        BS_TRACE2(0, 17);
        lds_barrier();   // P1
        BS_TRACE2(0, 18);
        BS_TRACE(1);
        if (nb > kMaxPre) lds_barrier();   // P2
        BS_TRACE(2);
        BS_TRACE2(0, 19);
        if (tid < CACT) quantise(tid, 0, r0);
        BS_TRACE2(0, 20);
        lds_barrier();   // P3
        BS_TRACE2(0, 21);
        BS_TRACE(3);
        for (int q = 0; q < nb; ++q) {
            BS_TRACE2(0, 2 * q);
            compute(q);
            BS_TRACE2(0, 2 * q + 1);
            lds_barrier();
        }
        BS_TRACE(4);
        // ---- partial sums out (agent-scope, write-through stores: the reader may sit on another XCD)
#pragma unroll
        for (int tl = 0; tl < R; ++tl) {
            const int row = row0 + (wave * R + tl) * kTileRows + lane;
            if (lane < 32 && row < p.out)
                __hip_atomic_store(&p.part[size_t(slot_i) * p.out + row], yacc[tl], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- the last workgroup of this row slab adds the partial rows and stores y.
    // Ordering: every wave's stores above are complete when it passes the barrier
    // (workgroup-scope release = wait for the vector memory counter), they are
    // write-through, and the counter increment is issued only after that; the
    // finishing workgroup reads the rows back with agent-scope loads after an
    // agent-scope acquire.  No cache-wide write-back or invalidate is paid by the
    // other workgroups (those cost more than the whole sign stream of a block).
    __syncthreads();
    BS_TRACE(5);
    if (tid == 0) {
        const unsigned expected = unsigned(p.n_ks) * unsigned(p.n_bg);
        const unsigned old = __hip_atomic_fetch_add(&p.ctr[rs_i], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = (old + 1u == expected) ? 1u : 0u;
    }
    __syncthreads();
    BS_TRACE(6);
    if (*flag) {
        // One pass with every load in flight at once: thread = (4 consecutive rows, a third of
        // the slots), 128-bit loads; the three partial sums meet in LDS.  Fixed summation order,
        // so the result does not depend on which workgroup arrived last.  The loads carry agent
        // scope themselves (they miss in every cache that is not coherent across XCDs, where rows
        // written during an earlier call may still sit), so no cache invalidate is paid.
        static_assert(NT == 768 && RS == 1024, "finisher mapping: 256 row quads x 3 slot groups");
        const int nslots = p.n_ks * p.n_bg;
        const int rq = tid & 255, sg = tid >> 8;
        const int row = row0 + 4 * rq;
        const bool live = row < p.out;   // out is a multiple of 32: a quad is inside or outside as a whole
        float4 tot = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        {
            // descriptor over this row slab's column of the workspace; slots past the end or rows
            // past the matrix get an offset beyond it (reads as zero, no traffic)
            const unsigned span = unsigned(size_t(nslots) * p.out * 4);
            __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(p.part, 0, span, 0x00020000);
            constexpr int kAgentScope = 16;   // sc1
            constexpr int MAXK = 24;          // slots per group and round
            for (int base = 0; base < nslots; base += 3 * MAXK) {
                v4i v[MAXK];
#pragma unroll
                for (int k = 0; k < MAXK; ++k) {
                    const int sl = base + 3 * k + sg;
                    const unsigned off = (live && sl < nslots) ? unsigned((size_t(sl) * p.out + row) * 4) : span;
                    v[k] = __builtin_amdgcn_raw_buffer_load_b128(prs, off, 0, kAgentScope);
                }
#pragma unroll
                for (int k = 0; k < MAXK; ++k) {
                    tot.x += __int_as_float(v[k][0]); tot.y += __int_as_float(v[k][1]);
                    tot.z += __int_as_float(v[k][2]); tot.w += __int_as_float(v[k][3]);
                }
            }
        }
        float4* red = reinterpret_cast<float4*>(smem);   // [3][256]; fragments are dead by now
        red[sg * 256 + rq] = tot;
        __syncthreads();
        if (sg == 0 && live) {
            const float4 a = red[rq], b2 = red[256 + rq], c = red[512 + rq];
            const float o4[4] = {(a.x + b2.x) + c.x, (a.y + b2.y) + c.y, (a.z + b2.z) + c.z, (a.w + b2.w) + c.w};
            if (p.y_f32) {
                *reinterpret_cast<float4*>(static_cast<float*>(p.y) + row) = make_float4(o4[0], o4[1], o4[2], o4[3]);
            } else {
                __half2 h01 = __floats2half2_rn(o4[0], o4[1]), h23 = __floats2half2_rn(o4[2], o4[3]);
                uint2 pk;
                pk.x = *reinterpret_cast<unsigned*>(&h01);
                pk.y = *reinterpret_cast<unsigned*>(&h23);
                *reinterpret_cast<uint2*>(static_cast<__half*>(p.y) + row) = pk;
            }
        }
        if (tid == 0) __hip_atomic_store(&p.ctr[rs_i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    BS_TRACE(7);
}

template <int KS>
static hipError_t launch_decode_t(KGroup& grp, int bg_req, hipStream_t st) {
    // block groups: enough workgroups to fill the chip once (one per compute unit), few
    // enough that each walks through several blocks and amortises its prologue and tail
    int total_pairs = 0;
    for (int i = 0; i < grp.count; ++i) {
        KParams& p = grp.s[i];
        p.n_rs = (p.out + kDecodeRows - 1) / kDecodeRows;
        p.n_ks = p.in / KS;
        total_pairs += p.n_rs * p.n_ks;
    }
    // Merged launches: the stacks of a group differ in height (Section 2.2: the sorted universal
    // stack leaves every weight stack its own number of blocks), and the launch lasts as long as
    // its slowest workgroup.  So every stack gets block groups in proportion to its height:
    // the smallest number of blocks per workgroup T for which all workgroups still fit on the
    // chip in one round, and ceil(n_loaded / T) groups per stack.
    int blocks_per_wg = 0;
    if (grp.count > 1 && bg_req <= 0) {
        long work = 0;
        int tallest = 1;
        for (int i = 0; i < grp.count; ++i) {
            work += long(grp.s[i].n_rs) * grp.s[i].n_ks * grp.s[i].n_loaded;
            tallest = tallest > grp.s[i].n_loaded ? tallest : grp.s[i].n_loaded;
        }
        for (int t = int((work + 255) / 256); t <= tallest; ++t) {
            long wgs = 0;
            bool workspace_ok = true;   // members sharing a stack share its partial-row slots
            for (int i = 0; i < grp.count; ++i) {
                wgs += long(grp.s[i].n_rs) * grp.s[i].n_ks * ((grp.s[i].n_loaded + t - 1) / t);
                int slots = 0;
                for (int j = 0; j < grp.count; ++j)
                    if (grp.s[j].blocks == grp.s[i].blocks) slots += grp.s[j].n_ks * ((grp.s[j].n_loaded + t - 1) / t);
                workspace_ok = workspace_ok && slots <= grp.s[i].part_slots;
            }
            blocks_per_wg = t;
            if (wgs <= 256 && workspace_ok) break;
        }
        if (blocks_per_wg < 1) blocks_per_wg = 1;
    }
    unsigned next = 0;
    int part_shift[kMaxGroup] = {}, ctr_shift[kMaxGroup] = {};
    for (int i = 0; i < grp.count; ++i) {
        KParams& p = grp.s[i];
        int bg = bg_req;
        if (blocks_per_wg > 0) {
            bg = (p.n_loaded + blocks_per_wg - 1) / blocks_per_wg;
        } else if (bg <= 0) {
            // largest group count that still fits on the chip in one round; among those prefer
            // one that gives every workgroup the same number of blocks
            bg = 256 / total_pairs;
            if (bg < 1) bg = 1;
            if (bg > p.n_loaded) bg = p.n_loaded;
            for (int cand = bg; cand >= 1 && cand * 4 >= bg * 3; --cand)
                if (p.n_loaded % cand == 0) {
                    bg = cand;
                    break;
                }
        }
        if (bg > p.n_loaded) bg = p.n_loaded;
        while ((p.n_loaded + bg - 1) / bg > kMaxBlocksPerWg) ++bg;
        p.n_bg = bg;
        // Members that share a stack (several tokens of a small batch in one launch) share its
        // split-accumulation workspace: each gets its own partial rows and arrival counters
        // behind those of the members before it.
        int slots_before = 0, ctrs_before = 0;
        for (int j = 0; j < i; ++j)
            if (grp.s[j].blocks == p.blocks) {
                slots_before += grp.s[j].n_ks * grp.s[j].n_bg;
                ctrs_before += grp.s[j].n_rs;
            }
        if (ctrs_before + p.n_rs > kCounterSlots || slots_before + p.n_ks * bg > p.part_slots)
            return hipErrorInvalidValue;   // nothing has been launched
        part_shift[i] = slots_before;
        ctr_shift[i] = ctrs_before;
        grp.base[i] = next;
        next += (unsigned(p.n_rs * p.n_ks) * unsigned(bg) + 7u) & ~7u;
    }
    for (int i = 0; i < grp.count; ++i) {   // (after the loop above, which compares the unshifted pointers)
        grp.s[i].part += size_t(part_shift[i]) * grp.s[i].out;
        grp.s[i].part_slots -= part_shift[i];
        grp.s[i].ctr += ctr_shift[i];
    }
    for (int i = grp.count; i <= kMaxGroup; ++i) grp.base[i] = next;
    const size_t smem = size_t(KS) * 68 + 2 * size_t(kDecodeRows) * 32 + size_t(kProducers) * kMaxBlocksPerWg * 4 +
                        96 * 4 + 16;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_old<KS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(smem));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_decode_old<KS>), dim3(next), dim3((kConsumers + kProducers) * 64), smem, st, grp);
    return hipGetLastError();
}

hipError_t launch_decode_group_old(const LaunchArgs* a, int count, hipStream_t st) {
    if (count < 1 || count > kMaxGroup) return hipErrorInvalidValue;
    const DecodeTuning& tn = decode_tuning();
    int ks = tn.legacy_kslab;
    if (ks == 0) ks = a[0].geo.min_slab;
    KGroup grp;
    grp.count = count;
    for (int i = 0; i < count; ++i) {
        if (a[i].batch != 1 || a[i].n_loaded < 1) return hipErrorInvalidValue;
        // the workspace of an image is sized for its own min_slab; one kernel, one slab width
        if (ks < a[i].geo.min_slab || a[i].geo.in % ks) return hipErrorInvalidValue;
        const size_t sign_span = size_t(a[i].geo.n) * a[i].geo.block_stride;
        if (sign_span + 4096 >= (size_t(1) << 32)) return hipErrorInvalidValue;   // 32-bit buffer offsets
        grp.s[i] = make_params(a[i]);
        grp.s[i].sign_bytes_total = unsigned(sign_span);
    }
    for (int i = count; i < kMaxGroup; ++i) grp.s[i] = grp.s[0];
    if (ks == 1024) return launch_decode_t<1024>(grp, tn.bgroups.load(), st);
    if (ks == 512) return launch_decode_t<512>(grp, tn.bgroups.load(), st);
    if (ks == 256) return launch_decode_t<256>(grp, tn.bgroups.load(), st);
    return hipErrorInvalidValue;
}


}  // namespace bitstack
