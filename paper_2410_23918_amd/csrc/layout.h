// Private device layout of a packed BitStack weight stack (gfx950).
//
// A residual block (BitStack, Section 2.1.2 and Eq. 9) holds a 1-bit sign matrix
// S (out x in) and fp16 factors U (out x k), V (in x k), k = 16.  On the device a
// block is one contiguous, self-contained range of exactly Eq. 9's byte count:
//
//   [ sign tiles : out*in/8 B ][ V panels : in*32 B ][ U rows : out*32 B ]
//
// Sign tiles.  The matrix is cut into units of 32 rows x 256 columns = 1 KiB,
// stored unit-major [row_tile][column_chunk].  Inside a unit, lane L = g*32 + j
// of a 64-wide wavefront owns 16 bytes: the four canonical uint32 words that hold
// columns [g*128, g*128+128) of row j.  One 128-bit load per lane therefore reads
// the unit fully coalesced, and the lane ends up with exactly the bytes the int8
// matrix-core instruction wants as its 32-column operand: masking the four words
// with 0x01010101 << t leaves, in every byte, bit t of that byte (value 0 or 2^t),
// i.e. the signs of the 32 columns {g*128 + w*32 + b*8 + t}.  Eight masks (t=0..7)
// consume the whole unit with one bitwise AND per four signs.
//
// V panels.  V is stored so that the 16 values of rank r that meet one such
// 32-column operand are contiguous: index (((chunk*8 + t)*2 + g)*16 + r)*16 + e,
// e = w*4 + b, column = chunk*256 + g*128 + w*32 + b*8 + t.
//
// U rows.  Plain row-major [out][16].
//
// The image of a whole stack is
//   [ 1/s : in floats ][ block 0 ] ... [ block n-1 ][ row maxima ][ partial sums ][ counters ][ activation scratch ]
// with every part 256-byte aligned.  "Row maxima" is derived data, not part of a
// block: per block and input channel j, max_r |V[j][r]| as fp16 in panel order; it
// lets the decode kernel find the exact max |V[j][r] * x[j]/s[j]| of a column slab
// from one value per channel instead of sixteen.  The partial-sum workspace holds
// one fp32 row of `out` values per workgroup that shares a row slab.  Images packed
// for more than 64 tokens per call end with a scratch area of max_batch x in fp16
// values, where the prefill kernel keeps the activations in fragment order.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define BS_HD __host__ __device__ inline
#else
#define BS_HD inline
#endif

namespace bitstack {

constexpr int kRank = 16;
constexpr int kTileRows = 32;      // rows per sign unit
constexpr int kChunkCols = 256;    // columns per sign unit
constexpr int kUnitBytes = 1024;
constexpr int kCounterSlots = 16384; // split-accumulation arrival counters (uint32 each)
constexpr int kCounterStride = 32;   // the decode kernel keeps one counter per 128-byte line
constexpr int kSmallBatch = 64;     // batches up to this size need no activation scratch

struct Geometry {
    int out, in, n, max_batch;
    size_t off_rs;       // float[in], 1/s
    size_t off_blocks;   // n blocks of block_stride bytes
    size_t block_stride; // == Eq. 9 bytes
    size_t off_v;        // inside a block: V panels
    size_t off_u;        // inside a block: U rows
    size_t off_vmax;     // fp16[n][in], max_r |V[j][r]| in panel order
    size_t off_part;     // float[part_slots][out] split-accumulation workspace
    int part_slots;      // n * (in / min_slab)
    int min_slab;        // smallest column slab the decode kernel may use with this image
    size_t off_ctr;      // uint32[kCounterSlots], zero between calls
    size_t off_xpack;    // fp16 activations of a large batch in matrix-core fragment order (max_batch > 64 only)
    size_t xpack_bytes;
    size_t total;
};

BS_HD size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

BS_HD bool shape_ok(int out, int in, int k) {
    return k == kRank && out > 0 && in > 0 && out % kTileRows == 0 && in % kChunkCols == 0;
}

BS_HD Geometry make_geometry(int out, int in, int n, int max_batch) {
    Geometry g;
    g.out = out; g.in = in; g.n = n; g.max_batch = max_batch;
    size_t signs = size_t(out) * size_t(in) / 8;
    g.off_v = signs;
    g.off_u = signs + size_t(in) * kRank * 2;
    g.block_stride = g.off_u + size_t(out) * kRank * 2;
    g.off_rs = 0;
    g.off_blocks = align256(size_t(in) * 4);
    g.min_slab = (in % 1024 == 0) ? 1024 : (in % 512 == 0) ? 512 : 256;
    g.part_slots = (n > 0 ? n : 1) * (in / g.min_slab);
    g.off_vmax = align256(g.off_blocks + size_t(n) * g.block_stride);
    g.off_part = align256(g.off_vmax + size_t(n) * size_t(in) * 2);
    g.off_ctr = align256(g.off_part + size_t(g.part_slots) * size_t(out) * 4);
    g.off_xpack = align256(g.off_ctr + size_t(kCounterSlots) * 4);
    g.xpack_bytes = max_batch > kSmallBatch ? size_t((max_batch + 31) / 32 * 32) * size_t(in) * 2 : 0;
    g.total = align256(g.off_xpack + g.xpack_bytes);
    return g;
}

// word index (in uint32 units from the start of the block's sign area) of the
// canonical word (row, word_in_row)
BS_HD size_t sign_word_index(int in, int row, int word) {
    int rt = row / kTileRows, j = row % kTileRows;
    int ch = word / 8, g = (word % 8) / 4, w = word % 4;
    size_t unit = size_t(rt) * size_t(in / kChunkCols) + size_t(ch);
    return unit * (kUnitBytes / 4) + size_t(g * 32 + j) * 4 + size_t(w);
}

// element index (in fp16 units from the start of the block's V area) of V[col][r]
BS_HD size_t v_index(int col, int r) {
    int ch = col / kChunkCols, c = col % kChunkCols;
    int g = c / 128, w = (c % 128) / 32, b = (c % 32) / 8, t = c % 8;
    int e = w * 4 + b;
    return ((((size_t(ch) * 8 + t) * 2 + g) * 16 + r) * 16) + size_t(e);
}

// index of channel col in a per-channel array kept in panel order
BS_HD size_t panel_index(int col) {
    int ch = col / kChunkCols, c = col % kChunkCols;
    int g = c / 128, w = (c % 128) / 32, b = (c % 32) / 8, t = c % 8;
    return ((size_t(ch) * 8 + t) * 2 + g) * 16 + size_t(w * 4 + b);
}

// inverse view used by the kernels: column of (chunk, t, g, e)
BS_HD int panel_col(int ch, int t, int g, int e) {
    return ch * kChunkCols + g * 128 + (e >> 2) * 32 + (e & 3) * 8 + t;
}

}  // namespace bitstack
