// Batch-1 decode kernel of the BitStack linear layer (gfx950 / CDNA4)
//     y = ( sum_i S_i (.) (U_i V_i^T) ) diag(1/s) x          (Eq. 4 + Eq. 8)
// evaluated from the packed residual blocks, never materialising the weight.
//
// Per block the method needs, for every output row o and rank r, the signed sum
//     Z[o,r] = sum_j S[o,j] * T[j,r],     T[j,r] = V[j,r] * x[j]/s[j]
// (per-rank identity (S (.) u v^T) x = u (.) (S (v (.) x))), followed by
// y[o] += sum_r U[o,r] Z[o,r].  Z is a dense contraction with a 1-bit operand, 16
// multiply-adds per sign bit, so it runs on the matrix cores (v_mfma_i32_32x32x32_i8):
//   * sign operand: the packed words become int8 operands with one bitwise AND per
//     four signs (mask 0x01010101 << t keeps bit t of every byte, value 0 or 2^t;
//     the device layout is chosen so that this is all it takes; the high-nibble
//     classes are brought down with one shift per word);
//   * panel operand: T is quantised per (block, column range of the workgroup) to
//     16-bit fixed point against the range's exact max |T|, pre-divided by the class
//     weight 2^(t mod 4) so that all column classes land on one scale, and split into
//     a high and a low signed byte: 16 ranks x {hi, lo} = the 32 rows of the A operand;
//   * accumulation is exact int32 over the whole column range of a block; S = 2B - 1
//     is undone with the exact integer column sums of the quantised panel.
//
// One workgroup = 8 wavefronts (two per SIMD, up to 256 registers each), R x 256
// output rows, a range of 256-column chunks, and every n_bg-th block of the loaded
// prefix.  Time is cut into intervals of one block x 1024 columns.  All wavefronts
// do the same work:
//   * sign stream: each owns R tiles of 32 rows; its only loads in the main loop
//     besides a few small ones are the sign units, requested one interval ahead into
//     a register window (R x 4 units = 16 KiB at R = 4) right after the unit that
//     occupied the slot has been used.  One 1 KiB panel fragment read from LDS serves
//     R matrix-core instructions.
//   * panel: at the end of interval i every thread quantises 32 values of interval
//     i + 1's panel (raw V values requested at the start of interval i, i.e. before
//     the window refills: loads return in order, so waiting for them never waits for
//     a sign unit that is not needed yet) into the other fragment buffer.
//   * epilogue once per block (not per interval): the int32 sums of the whole column
//     range are folded into running fp32 row sums with the block's U rows, which each
//     wavefront reads for its own rows straight from memory.
// One LDS-only barrier per interval.  Partial rows of the workgroups that share a row
// slab meet in a workspace; the last one to arrive adds them in a fixed order.
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


namespace {

constexpr float kQMax = 32512.0f;   // |q| <= 127*256: the high byte stays in int8 after +128 rounding
constexpr int kMaxChunkExp = 3;     // finest chunk scale: 2^-3 of the range's
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kPieceChunks = 4;                          // sign chunks per interval
constexpr int kPieceCols = kPieceChunks * kChunkCols;    // 1024
constexpr int kFragBytes = kPieceCols * 32;              // one fragment buffer
constexpr int kXsFloats = kDecodeMaxRangeChunks * kChunkCols;
// LDS layout (bytes from the start): two fragment buffers, the x/s table of the range, the maxima per
// block and (16 bits each) per (block, chunk, column class), three column-sum buffers, the smallest of
// those maxima per block, four flag words
constexpr int kLdsXs = 2 * kFragBytes;
constexpr int kLdsAmax = kLdsXs + kXsFloats * 4;
constexpr int kLdsAmaxStep = kLdsAmax + kDecodeMaxBlocksPerWg * 4;
constexpr int kLdsColSums = kLdsAmaxStep + kDecodeMaxBlocksPerWg * kDecodeMaxRangeChunks * 8 * 2;
constexpr int kLdsAmin = kLdsColSums + 3 * 32 * 4;
constexpr int kLdsFlags = kLdsAmin + kDecodeMaxBlocksPerWg * 4;
constexpr int kLdsBytes = kLdsFlags + 16;

// maximum over each aligned group of 32 lanes, in all its lanes (values >= 0: compared as integers).
// Four rotations inside the rows of 16 lanes, then one exchange between the two rows: no LDS atomics,
// which serialise lane by lane when many lanes name one address.
__device__ __forceinline__ int group32_max(int v) {
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false));   // row_ror:8
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, false));   // row_ror:4
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x122, 0xF, 0xF, false));   // row_ror:2
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x121, 0xF, 0xF, false));   // row_ror:1
    return max(v, __builtin_amdgcn_ds_swizzle(v, 0x401F));                   // lane ^ 16
}

__device__ __forceinline__ int group32_min(int v) {
    v = min(v, __builtin_amdgcn_update_dpp(0x7FFFFFFF, v, 0x128, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(0x7FFFFFFF, v, 0x124, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(0x7FFFFFFF, v, 0x122, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(0x7FFFFFFF, v, 0x121, 0xF, 0xF, false));
    return min(v, __builtin_amdgcn_ds_swizzle(v, 0x401F));
}

// maximum over each aligned group of 4 lanes, in all its lanes
__device__ __forceinline__ int quad_max(int v) {
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false));   // quad_perm:[1,0,3,2]
    return max(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false)); // quad_perm:[2,3,0,1]
}

__device__ __forceinline__ void wait_all_vector_memory() {
    // vmcnt(0) with the other counters left alone: every global load and store this
    // wavefront has issued is complete (stores: written through when they carry agent scope)
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

}  // namespace

template <int R, int EARLY>
__global__ __launch_bounds__(kThreads, 2) void k_decode(KGroup grp) {
    constexpr int RS = R * 256;   // rows per workgroup

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    v4i* frag0 = reinterpret_cast<v4i*>(smem);                              // [2][32 fragments][64 lanes] x 16 B
    float* xs = reinterpret_cast<float*>(smem + kLdsXs);                    // [range columns], panel order
    int* amax_i = reinterpret_cast<int*>(smem + kLdsAmax);                  // [blocks], float bits
    unsigned short* amax_s = reinterpret_cast<unsigned short*>(smem + kLdsAmaxStep);   // [blocks][chunks * 8 classes]
    int* cs = reinterpret_cast<int*>(smem + kLdsColSums);                   // [3][32]
    int* amin_i = reinterpret_cast<int*>(smem + kLdsAmin);                  // [blocks]: smallest (chunk, class) maximum
    unsigned* flag = reinterpret_cast<unsigned*>(smem + kLdsFlags);         // [0] finisher flag, [1] max |x/s| bits

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

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
    const int c_lo = ks_i * p.ks_chunks;                                  // first chunk of this range
    const int rc = min(p.ks_chunks, nch_total - c_lo);                    // chunks in it
    const int npc = (rc + kPieceChunks - 1) / kPieceChunks;               // intervals per block
    const int n_int = nb * npc;
    const int n_rt = p.out / kTileRows;
    const int row0 = rs_i * RS;
    auto block_index = [&](int q) { return bg_i + q * p.n_bg; };

    // ---------------------------------------------------------------- small loads first
    // (everything requested before the sign window, so that waiting for it never waits for signs)
    // x/s of the range: a thread takes 8 consecutive columns (same chunk, half, word and byte
    // row; classes t = 0..7), up to two such octets
    const int n_oct = rc * (kChunkCols / 8);
    uint4 xo[2];
    float4 ro[2][2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int o8 = min(tid + k * kThreads, n_oct - 1);
        const int col = c_lo * kChunkCols + o8 * 8;
        xo[k] = *reinterpret_cast<const uint4*>(p.x + col);
        ro[k][0] = *reinterpret_cast<const float4*>(p.rs + col);
        ro[k][1] = *reinterpret_cast<const float4*>(p.rs + col + 4);
    }
    // raw V values of the 32 panel values this thread quantises per interval: two consecutive
    // 16-value groups; group index tid*2 + m inside the interval = (position tid >> 3, ranks
    // 2*(tid & 7) + m); position = chunk*16 + class*2 + half
    struct Raw {
        uint4 v[2][2];
    };
    const int my_chunk = tid >> 7;   // chunk of the interval this thread's groups belong to (wave-uniform)
    auto load_raw = [&](int i) -> Raw {
        // interval i (clamped to the last one: an unused, harmless load keeps the number of
        // loads in flight the same on every path)
        const int ii = min(i, n_int - 1);
        const int q = ii / npc, pc = ii - q * npc;
        const int ch = min(c_lo + pc * kPieceChunks + my_chunk, c_lo + rc - 1);
        const unsigned char* blk = p.blocks + size_t(block_index(q)) * p.block_stride;
        const uint4* vsl = reinterpret_cast<const uint4*>(blk + p.off_v) + size_t(ch) * 256 * 2 + size_t(tid & 127) * 4;
        Raw raw;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            raw.v[m][0] = vsl[m * 2];
            raw.v[m][1] = vsl[m * 2 + 1];
        }
        __builtin_amdgcn_sched_barrier(0);
        return raw;
    };
    Raw raw = load_raw(0);       // interval 0, quantised in the prologue
    // The two wavefronts of a SIMD share its issue port and the older one is served first: it
    // finishes an interval's matrix-core work well before the younger one.  So the younger one
    // (wavefronts 4..7) quantises its share of the next panel at the start of an interval, while
    // the older one streams, and the older one at the end, while the younger one streams.
    const bool late_wave = __builtin_amdgcn_readfirstlane(tid) >= kThreads / 2;
    // per-channel maxima of V (8 channels per task) for the range maxima below; the first kPreTasks
    // tasks of a thread are requested here, ahead of the sign window
    constexpr int kPreTasks = 4;
    const int per_block = rc * 32;   // 8-channel pieces of the range
    const int tasks = nb * per_block;
    auto vmax_ptr = [&](int t0) {
        const int q = t0 / per_block, o8 = t0 - q * per_block;
        return reinterpret_cast<const uint4*>(p.vmax + size_t(block_index(q)) * p.in + size_t(c_lo) * kChunkCols + o8 * 8);
    };
    uint4 hvp[kPreTasks];
#pragma unroll
    for (int k = 0; k < kPreTasks; ++k) hvp[k] = *vmax_ptr(min(tid + k * kThreads, tasks - 1));
    __builtin_amdgcn_sched_barrier(0);

    // ---------------------------------------------------------------- sign window
    // win[c][tl] holds unit (chunk c of the interval, tile tl) until it is used, then the same
    // slot of the next interval
    v4i win[kPieceChunks][R];
    unsigned soff[R];   // byte offset of (tile, first chunk of the range, lane) inside a block
    const unsigned sign_bytes = p.sign_bytes_total;   // bytes covered by the buffer descriptor
    __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(p.blocks), 0, sign_bytes, 0x00020000);
    // per-lane offset just past the descriptor: such a load returns zero without touching memory
    const unsigned skip_off = 0x80000000u + unsigned(lane) * 16u;
    float yacc[R];
#pragma unroll
    for (int tl = 0; tl < R; ++tl) {
        const int rt = rs_i * (kWaves * R) + wave * R + tl;
        soff[tl] = rt < n_rt ? unsigned((size_t(rt) * nch_total + c_lo) * kUnitBytes) + unsigned(lane) * 16u : skip_off;
        yacc[tl] = 0.0f;
    }
    // scalar part of a unit's address: block and first chunk of interval i
    auto interval_base = [&](int i) -> unsigned {
        const int q = i / npc, pc = i - q * npc;
        return unsigned(block_index(q)) * unsigned(p.block_stride) + unsigned(pc * kPieceChunks) * kUnitBytes;
    };
    auto chunks_of = [&](int i) -> int {   // valid chunks of interval i
        const int pc = i % npc;
        return min(kPieceChunks, rc - pc * kPieceChunks);
    };
    // A slot whose next unit does not exist (no next interval, chunk past the range, tile past the
    // matrix) is still loaded, from an offset beyond the descriptor: the number of loads in flight
    // stays the same on every path.  The offset is made invalid arithmetically (top bit; the
    // descriptor covers less than 2 GiB), not by selecting between two loads.
    auto request = [&](int i, int c) __attribute__((always_inline)) {   // window slots of chunk c <- interval i
        const bool ok = i < n_int && c < chunks_of(min(i, n_int - 1));
        const unsigned sb = interval_base(min(i, n_int - 1)) + unsigned(c) * kUnitBytes;
        const unsigned oob = ok ? 0u : 0x80000000u;
#pragma unroll
        for (int tl = 0; tl < R; ++tl)
            win[c][tl] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, soff[tl] | oob, sb, 0);
    };
#pragma unroll
    for (int c = 0; c < EARLY; ++c) request(0, c);
    __builtin_amdgcn_sched_barrier(0);

    // ---------------------------------------------------------------- x/s table, range maxima
    if (tid < 96) cs[tid] = 0;
    if (tid < kDecodeMaxBlocksPerWg) {
        amax_i[tid] = 0;
        amin_i[tid] = 0x7F800000;   // +infinity
    }
    if (tid == 0) flag[1] = 0;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int o8 = tid + k * kThreads;
        if (o8 < n_oct) {
            // octet o8 = (chunk, half g, word w, byte row b); its 8 columns are the classes t = 0..7
            const int ch = o8 >> 5, g = (o8 >> 4) & 1, e = o8 & 15;
            const unsigned xw[4] = {xo[k].x, xo[k].y, xo[k].z, xo[k].w};
            const float rr[8] = {ro[k][0].x, ro[k][0].y, ro[k][0].z, ro[k][0].w,
                                 ro[k][1].x, ro[k][1].y, ro[k][1].z, ro[k][1].w};
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const __half2 h = *reinterpret_cast<const __half2*>(&xw[t >> 1]);
                const float xv = (t & 1) ? __high2float(h) : __low2float(h);
                xs[((ch * 8 + t) * 2 + g) * 16 + e] = xv * rr[t];
            }
        }
    }
    lds_barrier();   // P1: x/s table complete, tables cleared
    {
        // exact max |V[j][r] * xs[j]| over the range for each of my blocks:
        // max_j |xs[j]| * max_r |V[j][r]|, the inner maximum stored at pack time (panel order)
        auto fold = [&](int t0, const uint4 hv) {
            const int q = t0 / per_block, o8 = t0 - q * per_block;
            const float4 xa = *reinterpret_cast<const float4*>(xs + o8 * 8);
            const float4 xb = *reinterpret_cast<const float4*>(xs + o8 * 8 + 4);
            const unsigned hw[4] = {hv.x, hv.y, hv.z, hv.w};
            const float xx[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
            float a = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const __half2 h = *reinterpret_cast<const __half2*>(&hw[k]);
                a = fmaxf(a, fabsf(xx[2 * k]) * __low2float(h));
                a = fmaxf(a, fabsf(xx[2 * k + 1]) * __high2float(h));
            }
            float xm = 0.0f;   // largest |x/s| (the same for every block: taken from block 0's tasks)
#pragma unroll
            for (int k = 0; k < 8; ++k) xm = fmaxf(xm, fabsf(xx[k]));
            // (non-negative floats order like their bit patterns.)  The 4 tasks of a (chunk, column class)
            // step sit in one aligned group of 4 lanes: its maximum, rounded up to 16 bits, is kept for
            // the step's exponent.  Range maximum, smallest step maximum and the largest |x/s| go through
            // groups of 32 lanes first, so that few lanes touch the shared words.
            const int sa = ((quad_max(__float_as_int(a)) + 0xFFFF) >> 16) << 16;
            if ((lane & 3) == 0) amax_s[q * (kDecodeMaxRangeChunks * 8) + (o8 >> 2)] = (unsigned short)(sa >> 16);
            const int ga = group32_max(__float_as_int(a)), gn = group32_min(sa), gx = group32_max(__float_as_int(xm));
            if ((lane & 31) == 0) {
                atomicMax(&amax_i[q], ga);
                atomicMin(&amin_i[q], gn);
                if (q == 0) atomicMax(reinterpret_cast<int*>(&flag[1]), gx);
            }
        };
#pragma unroll
        for (int k = 0; k < kPreTasks; ++k)
            if (tid + k * kThreads < tasks) fold(tid + k * kThreads, hvp[k]);
        // tall walks over wide ranges: the rest on demand (these loads wait for the early sign units too)
        for (int t0 = tid + kPreTasks * kThreads; t0 < tasks; t0 += kThreads) fold(t0, *vmax_ptr(t0));
    }
    lds_barrier();   // P2: maxima complete
    // The quantiser multiplies in fp16: V[j][r] * (x[j]/s[j] * scale).  The second factor stays below
    // 8 / max_r |V[j][r]|, which only leaves fp16's range for channels whose V entries are all tiny
    // (< 1.3e-4) while x/s is huge; a block where that can happen takes the fp32 quantiser instead.
    auto needs_fp32 = [&](int q) -> bool {
        const float amax = __int_as_float(amax_i[q]);
        return !(__int_as_float(int(flag[1])) * float(1 << kMaxChunkExp) <= 60000.0f * amax);
    };

    // Quiet columns next to loud ones (a few activation channels far above the rest: the case
    // activation-aware scaling, Eq. 3-4, is there for) keep their precision.  A step = the 32 columns of
    // one class t in one chunk (one panel fragment, one matrix-core instruction per tile).  A step whose
    // maximum is at least four times below the range's is quantised 2^e times finer, e = 2 or 3.  The
    // integer sums of a block stay on ONE scale, 2^-E of the range's with E the largest e of the block:
    // a step with e < E gets its sign bytes 2^(E - e) times larger instead (a rotate of the chunk's sign
    // words when the shift changes, the mask moves along).  For activations without such channels every
    // e and E is 0 and nothing changes.
    auto exp_of = [&](int a, int b) -> int {   // float bits, a >= 0, b >= 0: floor(log2(a / b)), as 0, 2 or 3
        const int e = (a >> 23) - (b >> 23) - ((a & 0x7FFFFF) < (b & 0x7FFFFF) ? 1 : 0);
        return e >= 2 ? min(e, kMaxChunkExp) : 0;
    };
    auto step_exp = [&](int q, int cr, int t) -> int {   // block q of this workgroup, chunk cr of its range, class t: e
        return exp_of(amax_i[q], int(amax_s[q * (kDecodeMaxRangeChunks * 8) + cr * 8 + t]) << 16);
    };
    auto block_exp = [&](int q) -> int { return exp_of(amax_i[q], amin_i[q]); };   // E: the quietest step's e

    // quantise this thread's two groups of interval i into fragment buffer (i & 1)
    auto quantise = [&](int i, const Raw& rw) __attribute__((always_inline)) {
        const int q = i / npc, pc = i - q * npc;
        if (my_chunk >= min(kPieceChunks, rc - pc * kPieceChunks)) return;   // chunk past the range (wave-uniform)
        v4i* frag = frag0 + (i & 1) * (kFragBytes / 16);
        int* csq = cs + (q % 3) * 32;
        const float amax = __int_as_float(amax_i[q]);
        // (an approximate reciprocal will do: any scale a hair below 1 / amax keeps the codes in range,
        // and the epilogue multiplies by amax itself)
        const float inv = amax > 0.0f ? (kQMax / 32767.0f) * __builtin_amdgcn_rcpf(amax) : 0.0f;
        const int pos = tid >> 3, rk0 = (tid & 7) * 2;
        const int g = pos & 1, t = (pos >> 1) & 7, c = pos >> 4;
        // this step's exponent e and the shift E - e of its sign bytes
        const int ce = step_exp(q, pc * kPieceChunks + my_chunk, t);
        const int cs_shift = block_exp(q) - ce;
        // the sign byte of class t is 2^(t%4) (high-nibble classes are shifted down before use):
        // pre-dividing by it puts every class on one scale, (sign byte) * q = 32512 * 2^ce * T / amax
        const int tc = t & 3;
        const float f = inv * __int_as_float((127 + ce - tc) << 23);   // inv * 2^(ce - tc)
        // uniform over the workgroup.  Blocks with outlier channels (E > 0) also take the fp32 variant:
        // there the loud chunks set the error, and fp32 arithmetic keeps it a third lower
        const bool fp32_path = needs_fp32(q) || block_exp(q) != 0;
        const float4* xg = reinterpret_cast<const float4*>(xs + (pc * kPieceChunks * 16 + pos) * 16);
        typedef _Float16 h2v __attribute__((ext_vector_type(2)));
        // + 128 (in units of the 16-bit code) rides along in the multiply-add: the high byte of
        // q + 128 is round(q / 256), the low byte q ^ 0x80
        constexpr float kHalfByte = 128.0f / 32767.0f;
        h2v xh[8];
        float xf[16];
        if (!fp32_path) {
            // the 16 channel factors of this position as fp16 pairs (round to nearest).  fp16 arithmetic
            // keeps 11 significant bits per panel value (the class pre-division already leaves the worst
            // class 13): the error of y grows from 2.2e-4 to 3.5e-4 of max |y|, for less than half the
            // instructions of the fp32 variant.
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float4 v = xg[k];
                xh[2 * k][0] = _Float16(v.x * f); xh[2 * k][1] = _Float16(v.y * f);
                xh[2 * k + 1][0] = _Float16(v.z * f); xh[2 * k + 1][1] = _Float16(v.w * f);
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float4 v = xg[k];
                xf[4 * k] = v.x * f; xf[4 * k + 1] = v.y * f; xf[4 * k + 2] = v.z * f; xf[4 * k + 3] = v.w * f;
            }
        }
        int sums[2][2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const uint4 va = rw.v[m][0], vb = rw.v[m][1];
            const unsigned vw[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
            unsigned qq[8];
            if (!fp32_path) {
                const h2v bias = {_Float16(kHalfByte), _Float16(kHalfByte)};
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) {
                    const h2v pr = __builtin_elementwise_fma(__builtin_bit_cast(h2v, vw[e2]), xh[e2], bias);
                    const unsigned pu = __builtin_bit_cast(unsigned, pr);
                    // both halves of one register to signed 16-bit fixed point: round(clamp(p, -1, 1) * 32767)
                    asm("v_cvt_pknorm_i16_f16 %0, %1, %1 op_sel:[0,1,0]" : "=v"(qq[e2]) : "v"(pu));
                }
            } else {
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) {
                    const h2v h = __builtin_bit_cast(h2v, vw[e2]);
                    const v2s qv = __builtin_amdgcn_cvt_pknorm_i16(__builtin_fmaf(float(h[0]), xf[2 * e2], kHalfByte),
                                                                   __builtin_fmaf(float(h[1]), xf[2 * e2 + 1], kHalfByte));
                    qq[e2] = __builtin_bit_cast(unsigned, qv);
                }
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
            // column sums on the block's scale, like the sign bytes of this chunk
            sums[m][0] = sH << (tc + cs_shift);
            sums[m][1] = sL << (tc + cs_shift);
            const int r = rk0 + m;
            const int lane_hi = g * 32 + 8 * (r >> 2) + (r & 3);
            frag[(c * 8 + t) * 64 + lane_hi] = H;
            frag[(c * 8 + t) * 64 + lane_hi + 4] = L;
        }
        // integer column sums of the quantised panel per rank and byte half: the lanes that hold the
        // same ranks differ in lane bits 3..5.  Bit 3 is added up in registers (a rotation by 8 within the
        // row of 16 lanes), the four rows go to LDS as they are: one atomic per rank, half and row
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                sums[m][h] += __builtin_amdgcn_update_dpp(0, sums[m][h], 0x128 /* row_ror:8 */, 0xF, 0xF, false);
        if ((lane & 8) == 0) {
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                atomicAdd(&csq[rk0 + m], sums[m][0]);
                atomicAdd(&csq[16 + rk0 + m], sums[m][1]);
            }
        }
    };

    // interval 1's V values (used first by the wavefronts that quantise at the start of an interval):
    // requested only now, so that the requests of the prologue that matter sooner (x, maxima, the
    // first panel's V, the first sign units) do not share the compute unit's memory queue with them
    Raw raw_cur = load_raw(1);
    quantise(0, raw);
#pragma unroll
    for (int c = EARLY; c < kPieceChunks; ++c) request(0, c);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();   // P3: interval 0 staged

    // ---------------------------------------------------------------- main loop
    v16i acc[R];
    // One interval: block q, piece pc of the column range.  LAST = the piece that ends the block
    // (two instantiations, so that the number of loads in flight is the same on every path
    // through a given instantiation and the memory waits the compiler places are exact).
    auto interval = [&](int i, int q, int pc, auto last_tag) __attribute__((always_inline)) {
        constexpr bool LAST = decltype(last_tag)::value;
        const int nvalid = min(kPieceChunks, rc - pc * kPieceChunks);
        // shifts E - e of this interval's 32 steps (uniform): lane c*8 + t looks step (c, t) up, two
        // ballots carry the two bits of every shift
        unsigned shift_lo, shift_hi;
        {
            const int cr = min(pc * kPieceChunks + ((lane >> 3) & 3), rc - 1);
            const int my = lane < 32 ? block_exp(q) - step_exp(q, cr, lane & 7) : 0;
            shift_lo = unsigned(__builtin_amdgcn_ballot_w64((my & 1) != 0));
            shift_hi = unsigned(__builtin_amdgcn_ballot_w64((my & 2) != 0));
        }
        // column sums of block q + 2 start from zero: that buffer was last read in the epilogue of
        // block q - 1 (at least one barrier ago) and is first added to one barrier from now or later
        if (LAST && tid < 32) cs[((q + 2) % 3) * 32 + tid] = 0;
        if (late_wave && i + 1 < n_int) quantise(i + 1, raw_cur);
        // small loads, requested before the window refills: raw V of the interval this wavefront
        // quantises next (at the end of this interval, or at the start of the next one) and, for the
        // epilogue, the U rows of its tiles
        raw_cur = load_raw(i + (late_wave ? 2 : 1));
        uint4 ur[R][2];
        if constexpr (LAST) {
            const uint4* usrc =
                reinterpret_cast<const uint4*>(p.blocks + size_t(block_index(q)) * p.block_stride + p.off_u);
            const int last_row = p.out - 1;   // rows past the end re-read the last one (never stored)
#pragma unroll
            for (int tl = 0; tl < R; ++tl) {
                const int row = min(row0 + (wave * R + tl) * kTileRows + (lane & 31), last_row);
                ur[tl][0] = usrc[row * 2];
                ur[tl][1] = usrc[row * 2 + 1];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const v4i* frag = frag0 + (i & 1) * (kFragBytes / 16);
        v4i Tf = frag[lane];
#pragma unroll
        for (int c = 0; c < kPieceChunks; ++c) {
            if (c < nvalid) {
                int rot = 0;   // how far this chunk's sign words are rotated left at the moment
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    // the next fragment is requested before this one is used
                    v4i Tn = Tf;
                    if (c * 8 + t + 1 < kPieceChunks * 8) Tn = frag[(c * 8 + t + 1) * 64 + lane];
                    // sign bytes of this step are 2^(t%4 + sh): the words are rotated left by sh (rare: only
                    // in a block where some steps are quantised finer than this one)
                    const int sh = int((shift_lo >> (c * 8 + t)) & 1u) | int((shift_hi >> (c * 8 + t)) & 1u) << 1;
                    if (sh != rot) {
                        const unsigned by = unsigned(32 - (sh - rot)) & 31u;   // rotate right by this much
#pragma unroll
                        for (int tl = 0; tl < R; ++tl)
#pragma unroll
                            for (int w = 0; w < 4; ++w)
                                win[c][tl][w] = int(__builtin_amdgcn_alignbit(unsigned(win[c][tl][w]), unsigned(win[c][tl][w]), by));
                        rot = sh;
                    }
                    const int mask = 0x01010101 << ((t & 3) + sh);
                    if (t == 4) {   // high-nibble classes: bit 4+t' of a byte goes where bit t' was (a rotate:
                                    // the rotates above may have moved bits of the last byte to the front)
#pragma unroll
                        for (int tl = 0; tl < R; ++tl)
#pragma unroll
                            for (int w = 0; w < 4; ++w)
                                win[c][tl][w] = int(__builtin_amdgcn_alignbit(unsigned(win[c][tl][w]), unsigned(win[c][tl][w]), 4));
                    }
#pragma unroll
                    for (int tl = 0; tl < R; ++tl) {
                        const v4i B = win[c][tl] & mask;
                        acc[tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Tf, B, acc[tl], 0, 0, 0);
                    }
                    Tf = Tn;
                }
            }
            // this chunk's window slots now take the same chunk of the next interval (not
            // earlier: old and new contents would both need registers)
            __builtin_amdgcn_sched_barrier(0);
            request(i + 1, c);
        }
        if constexpr (LAST) {
            // epilogue: undo S = 2B - 1, weight by U, reduce over ranks.  Sums and column sums are on the
            // block's scale, 2^-E of the range's.
            const int part = lane >> 5;   // 0 = high bytes, 1 = low bytes
            const float dq = __int_as_float(amax_i[q]) * (1.0f / kQMax) * __int_as_float((127 - block_exp(q)) << 23);
            const int* csq = cs + (q % 3) * 32 + part * 16;
            float sum[R];
#pragma unroll
            for (int tl = 0; tl < R; ++tl) sum[tl] = 0.0f;
#pragma unroll
            for (int r2 = 0; r2 < 8; ++r2) {
                const int c0 = csq[2 * r2], c1 = csq[2 * r2 + 1];
#pragma unroll
                for (int tl = 0; tl < R; ++tl) {
                    const unsigned uw = r2 < 4 ? (r2 == 0 ? ur[tl][0].x : r2 == 1 ? ur[tl][0].y : r2 == 2 ? ur[tl][0].z : ur[tl][0].w)
                                               : (r2 == 4 ? ur[tl][1].x : r2 == 5 ? ur[tl][1].y : r2 == 6 ? ur[tl][1].z : ur[tl][1].w);
                    const __half2 h = *reinterpret_cast<const __half2*>(&uw);
                    const int z0 = (acc[tl][2 * r2] << 1) - c0;
                    const int z1 = (acc[tl][2 * r2 + 1] << 1) - c1;
                    sum[tl] = fmaf(float(z0), __low2float(h), sum[tl]);
                    sum[tl] = fmaf(float(z1), __high2float(h), sum[tl]);
                }
            }
#pragma unroll
            for (int tl = 0; tl < R; ++tl) {
                const float other = __shfl_xor(sum[tl], 32);
                yacc[tl] = fmaf(256.0f * sum[tl] + other, dq, yacc[tl]);   // meaningful in lanes 0..31
            }
        }
        if (!late_wave && i + 1 < n_int) quantise(i + 1, raw_cur);
        lds_barrier();
    };
    {
        int i = 0;
        for (int q = 0; q < nb; ++q) {
#pragma unroll
            for (int tl = 0; tl < R; ++tl)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tl][v] = 0;
            for (int pc = 0; pc + 1 < npc; ++pc, ++i) interval(i, q, pc, std::false_type{});
            interval(i, q, npc - 1, std::true_type{});
            ++i;
        }
    }

    // ---------------------------------------------------------------- split accumulation
    // partial sums out (agent-scope, write-through stores: the reader may sit on another XCD)
#pragma unroll
    for (int tl = 0; tl < R; ++tl) {
        const int row = row0 + (wave * R + tl) * kTileRows + lane;
        if (lane < 32 && row < p.out)
            __hip_atomic_store(&p.part[size_t(slot_i) * p.out + row], yacc[tl], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    // The last workgroup of this row slab adds the partial rows and stores y.  Ordering: every
    // wavefront waits for its own stores (they are write-through: complete means visible to
    // agent-scope loads anywhere on the device) before the barrier; only then is the arrival
    // counter bumped.  The finishing workgroup reads the rows back with agent-scope loads, which
    // miss in every cache that is not coherent across XCDs.  No cache-wide write-back or
    // invalidate is paid by anybody (those cost more than the whole sign stream of a block).
    wait_all_vector_memory();
    __syncthreads();
    if (tid == 0) {
        const unsigned expected = unsigned(p.n_ks) * unsigned(p.n_bg);
        const unsigned old = __hip_atomic_fetch_add(&p.ctr[rs_i * kCounterStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = (old + 1u == expected) ? 1u : 0u;
    }
    __syncthreads();
    // Few partial rows per slab and one row per thread (R = 2): every thread adds up its row over all
    // slots, their loads in flight together, in slot order (fixed: the result does not depend on
    // which workgroup arrived last); no LDS, no barrier.  Measured 0.45 us faster than the general
    // path below at 32 slots, and slower beyond (a second round of loads) and with two rows per thread.
    if (R == 2 && *flag && p.n_ks * p.n_bg <= 32) {
        const int nslots = p.n_ks * p.n_bg;
        const int row = row0 + tid;
        const bool live = row < p.out;
        const unsigned span = unsigned(size_t(nslots) * p.out * 4);
        __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(p.part, 0, span, 0x00020000);
        constexpr int kAgentScope = 16;   // sc1
        int v[32];
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const unsigned off = (live && k < nslots) ? unsigned((size_t(k) * p.out + row) * 4) : span;
            v[k] = __builtin_amdgcn_raw_buffer_load_b32(prs, off, 0, kAgentScope);
        }
        float tot = 0.0f;
#pragma unroll
        for (int k = 0; k < 32; ++k) tot += __int_as_float(v[k]);   // slots past the end read as zero
        if (live) store_y(p, size_t(row), tot);
        if (tid == 0) __hip_atomic_store(&p.ctr[rs_i * kCounterStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else
    if (*flag) {
        // One pass with every load in flight at once: thread = (4 consecutive rows, every NSG-th
        // slot), 128-bit loads; the NSG partial sums of a row quad meet in LDS.  Fixed summation
        // order, so the result does not depend on which workgroup arrived last.
        constexpr int NQ = RS / 4;          // row quads
        constexpr int NSG = kThreads / NQ;  // slot groups (2 or 4)
        const int nslots = p.n_ks * p.n_bg;
        const int rq = tid % NQ, sg = tid / NQ;
        const int row = row0 + 4 * rq;
        const bool live = row < p.out;   // out is a multiple of 32: a quad is inside or outside as a whole
        float4 tot = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        {
            // descriptor over the workspace rows of this stack; slots past the end or rows past
            // the matrix get an offset beyond it (reads as zero, no traffic)
            const unsigned span = unsigned(size_t(nslots) * p.out * 4);
            __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(p.part, 0, span, 0x00020000);
            constexpr int kAgentScope = 16;   // sc1
            constexpr int MAXK = 16;          // slots per group and round
            for (int base = 0; base < nslots; base += NSG * MAXK) {
                v4i v[MAXK];
#pragma unroll
                for (int k = 0; k < MAXK; ++k) {
                    const int sl = base + NSG * k + sg;
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
        float4* red = reinterpret_cast<float4*>(smem);   // [NSG][NQ]; the fragments are dead by now
        red[sg * NQ + rq] = tot;
        __syncthreads();
        if (sg == 0 && live) {
            float4 a = red[rq];
#pragma unroll
            for (int k = 1; k < NSG; ++k) {
                const float4 b = red[k * NQ + rq];
                a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            }
            if (p.y_f32) {
                *reinterpret_cast<float4*>(static_cast<float*>(p.y) + row) = a;
            } else {
                __half2 h01 = __floats2half2_rn(a.x, a.y), h23 = __floats2half2_rn(a.z, a.w);
                uint2 pk;
                pk.x = *reinterpret_cast<unsigned*>(&h01);
                pk.y = *reinterpret_cast<unsigned*>(&h23);
                *reinterpret_cast<uint2*>(static_cast<__half*>(p.y) + row) = pk;
            }
        }
        if (tid == 0) __hip_atomic_store(&p.ctr[rs_i * kCounterStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}


// ======================================================================== host side
namespace {

struct MemberPlan {
    int n_rs, n_ks, ks_chunks, n_bg;
};
struct DecodePlan {
    int tiles;            // R
    MemberPlan m[kMaxGroup];
    long wgs;
    double us;            // estimate
};

// Measured on MI355X: an interval (one block x 1024 columns x R*256 rows) and the epilogue
// of a block per workgroup, the fixed part of a launch, and the finisher's read of the partial rows.
constexpr double kIntervalUs4 = 4.7, kIntervalUs2 = 2.7, kEpilogueUs = 0.25, kFixedUs = 7.0;
constexpr double kFinisherUsPerKiB = 1.0 / 110.0, kFinisherLatencyUs = 1.2, kArrivalUs = 0.03;

// The work split of one launch: tiles per wavefront R, chunks per column range, and per member
// the number of block groups.  Every member reads the same x, so they share `in`.  The stacks of
// a group differ in height (Section 2.2: the sorted universal stack leaves every weight stack
// its own number of blocks) and a launch lasts as long as its slowest workgroup, so every stack
// gets block groups in proportion to its height: the smallest number of blocks per workgroup T
// for which all workgroups fit on the chip in one round (and in the stacks' workspaces), and
// ceil(n_loaded / T) groups per stack.  Among the candidate (R, range) pairs the one with the
// smallest estimated duration is taken.  Members that share a stack (several tokens of a small
// batch) share its workspace.
bool plan_decode(const LaunchArgs* a, int count, DecodePlan* best) {
    const DecodeTuning& tn = decode_tuning();
    const int chunks = a[0].geo.in / kChunkCols;
    bool found = false;
    for (int R = 4; R >= 2; R -= 2) {
        if (tn.tiles.load() && tn.tiles.load() != R) continue;
        int last_ksc = 0;
        for (int want_ks = 1; want_ks <= chunks; ++want_ks) {
            int ksc = (chunks + want_ks - 1) / want_ks;
            if (chunks >= kPieceChunks) ksc = (ksc + kPieceChunks - 1) / kPieceChunks * kPieceChunks;
            if (tn.ks_chunks.load()) ksc = tn.ks_chunks.load();
            if (ksc > kDecodeMaxRangeChunks || ksc == last_ksc || ksc < 1) {
                if (tn.ks_chunks.load()) break;
                continue;
            }
            last_ksc = ksc;
            const int n_ks = (chunks + ksc - 1) / ksc;
            const int npc = (ksc + kPieceChunks - 1) / kPieceChunks;
            DecodePlan pl;
            pl.tiles = R;
            long work = 0;
            int tallest = 1;
            for (int i = 0; i < count; ++i) {
                pl.m[i].n_rs = (a[i].geo.out + R * 256 - 1) / (R * 256);
                pl.m[i].n_ks = n_ks;
                pl.m[i].ks_chunks = ksc;
                const long pairs = long(pl.m[i].n_rs) * n_ks;
                work += pairs * a[i].n_loaded;
                tallest = tallest > a[i].n_loaded ? tallest : a[i].n_loaded;
            }
            auto workspace_ok = [&](int T) {
                for (int i = 0; i < count; ++i) {
                    int slots = 0, ctrs = 0;
                    for (int j = 0; j < count; ++j)
                        if (a[j].image == a[i].image && a[j].ws_part == a[i].ws_part) {
                            slots += pl.m[j].n_ks * ((a[j].n_loaded + T - 1) / T);
                            ctrs += pl.m[j].n_rs;
                        }
                    const int have = a[i].ws_part ? a[i].ws_part_slots : a[i].geo.part_slots;
                    if (slots > have || ctrs * kCounterStride > kCounterSlots) return false;
                }
                return true;
            };
            int T = 0;
            long wgs = 0;
            const int forced_bg = count == 1 ? tn.bgroups.load() : 0;
            if (forced_bg > 0) {
                const int bg = forced_bg < a[0].n_loaded ? forced_bg : a[0].n_loaded;
                T = (a[0].n_loaded + bg - 1) / bg;
                if (T > kDecodeMaxBlocksPerWg || !workspace_ok(T)) continue;
            } else {
                for (int t = int((work + 255) / 256); t <= tallest; ++t) {
                    if (t < 1) continue;
                    long w = 0;
                    for (int i = 0; i < count; ++i) w += long(pl.m[i].n_rs) * n_ks * ((a[i].n_loaded + t - 1) / t);
                    if (w <= 256 && workspace_ok(t)) {
                        T = t;
                        break;
                    }
                }
                // more row slab / column range pairs than compute units: every workgroup walks its whole
                // stack and the launch takes several rounds
                if (T == 0 && workspace_ok(tallest)) T = tallest;
                if (T == 0 || T > kDecodeMaxBlocksPerWg) continue;
            }
            int max_slots = 0;
            for (int i = 0; i < count; ++i) {
                pl.m[i].n_bg = (a[i].n_loaded + T - 1) / T;
                wgs += long(pl.m[i].n_rs) * n_ks * pl.m[i].n_bg;
                const int slots = n_ks * pl.m[i].n_bg;
                max_slots = max_slots > slots ? max_slots : slots;
            }
            const double rounds = double((wgs + 255) / 256);
            pl.wgs = wgs;
            pl.us = kFixedUs + rounds * T * (npc * (R == 4 ? kIntervalUs4 : kIntervalUs2) + kEpilogueUs) +
                    kFinisherLatencyUs + max_slots * (R * 256 * 4 / 1024.0) * kFinisherUsPerKiB + max_slots * kArrivalUs;
            if (!found || pl.us < best->us) {
                *best = pl;
                found = true;
            }
            if (tn.ks_chunks.load()) break;
        }
    }
    return found;
}

template <int R, int EARLY>
hipError_t launch_variant(const KGroup& grp, unsigned wgs, hipStream_t st) {
    const size_t smem = size_t(kLdsBytes);
    static std::atomic<int> attr_state{0};   // per instantiation; setting the attribute twice is harmless
    if (attr_state.load(std::memory_order_acquire) == 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode<R, EARLY>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(smem));
        if (e != hipSuccess) return e;
        attr_state.store(1, std::memory_order_release);
    }
    hipLaunchKernelGGL((k_decode<R, EARLY>), dim3(wgs), dim3(kThreads), smem, st, grp);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_group(const LaunchArgs* a, int count, hipStream_t st) {
    DecodeLaunch d;
    const hipError_t e = prepare_decode_group(a, count, &d);
    return e != hipSuccess ? e : run_decode_launch(d, st);
}

// Work split and argument block of one launch (host only, nothing is enqueued).
hipError_t prepare_decode_group(const LaunchArgs* a, int count, DecodeLaunch* d) {
    if (count < 1 || count > kMaxGroup) return hipErrorInvalidValue;
    const DecodeTuning& tn = decode_tuning();
    for (int i = 0; i < count; ++i) {
        if (a[i].batch != 1 || a[i].n_loaded < 1 || a[i].geo.in != a[0].geo.in) return hipErrorInvalidValue;
        const size_t sign_span = size_t(a[i].geo.n) * a[i].geo.block_stride;
        if (sign_span + 4096 >= (size_t(1) << 31)) return hipErrorInvalidValue;   // 31-bit buffer offsets
    }
    DecodePlan pl;
    if (!plan_decode(a, count, &pl)) return hipErrorInvalidValue;   // nothing has been launched
    KGroup& grp = d->grp;
    grp.count = count;
    unsigned next = 0;
    for (int i = 0; i < count; ++i) {
        KParams& p = grp.s[i];
        p = make_params(a[i]);
        p.sign_bytes_total = unsigned(size_t(a[i].geo.n) * a[i].geo.block_stride);
        p.n_rs = pl.m[i].n_rs;
        p.n_ks = pl.m[i].n_ks;
        p.ks_chunks = pl.m[i].ks_chunks;
        p.n_bg = pl.m[i].n_bg;
        // Members that share a stack (several tokens of a small batch in one launch) share its
        // split-accumulation workspace: each gets its own partial rows and arrival counters
        // behind those of the members before it.
        int slots_before = 0, ctrs_before = 0;
        for (int j = 0; j < i; ++j)
            if (a[j].image == a[i].image && a[j].ws_part == a[i].ws_part) {
                slots_before += pl.m[j].n_ks * pl.m[j].n_bg;
                ctrs_before += pl.m[j].n_rs;
            }
        p.part += size_t(slots_before) * p.out;
        p.part_slots -= slots_before;
        p.ctr += ctrs_before * kCounterStride;
        grp.base[i] = next;
        next += (unsigned(p.n_rs * p.n_ks) * unsigned(p.n_bg) + 7u) & ~7u;
    }
    for (int i = count; i < kMaxGroup; ++i) grp.s[i] = grp.s[0];
    for (int i = count; i <= kMaxGroup; ++i) grp.base[i] = next;
    int early = tn.early.load();
    if (early < 0) early = 2;
    d->wgs = next;
    d->tiles = pl.tiles;
    d->early = early;
    return hipSuccess;
}

hipError_t run_decode_launch(const DecodeLaunch& d, hipStream_t st) {
    const KGroup& grp = d.grp;
    const unsigned next = d.wgs;
    const int early = d.early;
    if (d.tiles == 4) {
        if (early >= 4) return launch_variant<4, 4>(grp, next, st);
        if (early >= 2) return launch_variant<4, 2>(grp, next, st);
        if (early >= 1) return launch_variant<4, 1>(grp, next, st);
        return launch_variant<4, 0>(grp, next, st);
    }
    if (early >= 4) return launch_variant<2, 4>(grp, next, st);
    if (early >= 2) return launch_variant<2, 2>(grp, next, st);
    if (early >= 1) return launch_variant<2, 1>(grp, next, st);
    return launch_variant<2, 0>(grp, next, st);
}

// ---- the entry point that allocates nothing: workspace in a static device array
// (for callers that cannot call hipMalloc or lend a workspace: code under graph capture, serving
// loops).  Every device the library runs on holds its own copy until the process ends.  All calls on
// a device share it: calls that overlap in time on one device race.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];   // per device: device address of `scratch`

__global__ void k_clear_counters(unsigned* ctr, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) ctr[i] = 0u;
}
}  // namespace

hipError_t launch_decode_static(const LaunchArgs& a, hipStream_t st) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    unsigned char* base = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!base) {
        // first call on this device: the array's name is a host-side stand-in, its device address
        // comes from the runtime.  The counters must start at zero (the kernels leave them at zero):
        // cleared once by a small kernel on the caller's stream, ahead of the first launch.
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        base = static_cast<unsigned char*>(ptr);
        hipLaunchKernelGGL(k_clear_counters, dim3((kCounterSlots + 255) / 256), dim3(256), 0, st,
                           reinterpret_cast<unsigned*>(base + kStaticPartBytes), kCounterSlots);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev].store(base, std::memory_order_release);
    }
    LaunchArgs b = a;
    b.ws_part = reinterpret_cast<float*>(base);
    b.ws_ctr = reinterpret_cast<unsigned*>(base + kStaticPartBytes);
    b.ws_part_slots = int(kStaticPartBytes / (size_t(a.geo.out) * 4));
    if (b.ws_part_slots < 1) return hipErrorOutOfMemory;
    DecodePlan pl;
    if (!plan_decode(&b, 1, &pl)) return hipErrorOutOfMemory;   // no work split fits the array
    return launch_decode_group(&b, 1, st);
}

// Estimated duration (microseconds) of one decode launch with m tokens of one stack; 0: the
// launcher would refuse (workspace too small for m tokens).
static double decode_launch_time_us(const Geometry& g, int m, int n_loaded) {
    LaunchArgs a[kMaxGroup];
    for (int i = 0; i < m; ++i) {
        a[i].x = a[i].y = nullptr;
        a[i].image = nullptr;   // all members share one stack
        a[i].geo = g;
        a[i].batch = 1;
        a[i].n_loaded = n_loaded;
        a[i].y_f32 = false;
    }
    DecodePlan pl;
    if (!plan_decode(a, m, &pl)) return 0.0;
    // The work-split estimate prices intervals whose sign units are there; big stacks are bound by the
    // stream instead: ~4.4 TB/s from memory for one token, and every further member streams the
    // units again, from the L2s and the last-level cache at best (measured 2.7-3.9 TB/s over all
    // members' bytes), after ~9 us of the fixed part that overlaps with nothing.
    const double bytes = double(m) * n_loaded * (double(g.out) * g.in / 8.0);
    const double stream_us = 9.0 + bytes / (m == 1 ? 4.4e6 : 3.3e6);
    return pl.us > stream_us ? pl.us : stream_us;
}

// How a small batch is cut into launches of one to four tokens: the cut with the smallest
// estimated total (three tokens of a tall stack can be cheaper as 2 + 1 than as one launch whose
// workgroups each walk the whole stack).  Batches beyond kPlanTokens start with launches of the
// size that is cheapest per token.  sizes[] (kPlanTokens entries) receives the launch sizes of
// the planned tail in order; *head_launches launches of *head_size tokens come before it.
constexpr int kPlanTokens = 64;
static double plan_decode_tokens(const Geometry& g, int batch, int n_loaded, int* sizes, int* n_launches,
                                 int* head_size, int* head_launches) {
    double t_of[kMaxGroup + 1] = {};
    int m_best = 1;
    for (int m = 1; m <= kMaxGroup; ++m) {
        t_of[m] = decode_launch_time_us(g, m, n_loaded);
        if (t_of[m] > 0.0 && (t_of[m_best] == 0.0 || t_of[m] / m < t_of[m_best] / m_best)) m_best = m;
    }
    int heads = 0;
    while (batch - heads * m_best > kPlanTokens) ++heads;
    const int rest = batch - heads * m_best;
    // best[b]: cheapest way to run b tokens; take[b]: size of its last launch
    double best[kPlanTokens + 1];
    int take[kPlanTokens + 1];
    best[0] = 0.0;
    take[0] = 1;
    for (int b = 1; b <= rest; ++b) {
        best[b] = -1.0;
        take[b] = 1;
        for (int m = 1; m <= kMaxGroup && m <= b; ++m) {
            if (t_of[m] == 0.0 || best[b - m] < 0.0) continue;
            const double t = best[b - m] + t_of[m];
            if (best[b] < 0.0 || t < best[b]) {
                best[b] = t;
                take[b] = m;
            }
        }
    }
    int n = 0;
    for (int b = rest; b > 0; b -= take[b])
        if (sizes) sizes[n++] = take[b];
    if (n_launches) *n_launches = n;
    if (head_size) *head_size = m_best;
    if (head_launches) *head_launches = heads;
    return heads * t_of[m_best] + best[rest];
}

double decode_tokens_time_us(const Geometry& g, int batch, int n_loaded) {
    return plan_decode_tokens(g, batch, n_loaded, nullptr, nullptr, nullptr, nullptr);
}

// A small batch through the decode kernel: one to four tokens per launch, each a member of the
// group with its own x row, y row and share of the stack's workspace.
hipError_t launch_decode_tokens(const LaunchArgs& a, hipStream_t st) {
    const size_t xbytes = size_t(a.geo.in) * 2, ybytes = size_t(a.geo.out) * (a.y_f32 ? 4 : 2);
    int sizes[kPlanTokens], n_launches = 0, head_size = 1, head_launches = 0;
    plan_decode_tokens(a.geo, a.batch, a.n_loaded, sizes, &n_launches, &head_size, &head_launches);
    int b = 0;
    for (int l = 0; l < head_launches + n_launches; ++l) {
        const int count = l < head_launches ? head_size : sizes[l - head_launches];
        LaunchArgs t[kMaxGroup];
        for (int i = 0; i < count; ++i) {
            t[i] = a;
            t[i].batch = 1;
            t[i].x = static_cast<const unsigned char*>(a.x) + size_t(b + i) * xbytes;
            t[i].y = static_cast<unsigned char*>(a.y) + size_t(b + i) * ybytes;
        }
        hipError_t e = launch_decode_group(t, count, st);
        if (e == hipErrorInvalidValue && count > 1) {
            // refused before anything was launched (e.g. a forced tuning the plan does not know): one by one
            e = hipSuccess;
            for (int i = 0; i < count && e == hipSuccess; ++i) e = launch_decode_group(t + i, 1, st);
        }
        if (e != hipSuccess) return e;
        b += count;
    }
    return hipSuccess;
}

}  // namespace bitstack
