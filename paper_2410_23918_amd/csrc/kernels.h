// Internal interface between the C-ABI host code and the HIP kernels.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "layout.h"

namespace bitstack {

struct LaunchArgs {
    const void* x;         // device fp16 [batch][in]
    void* y;               // device [batch][out], fp16 or fp32
    unsigned char* image;  // packed stack (device)
    Geometry geo;
    int batch;
    int n_loaded;
    bool y_f32;
    void* wdense = nullptr;  // device fp16 [out][in]: the restored weight of the materialising path
    // split-accumulation workspace outside the image (the entry point that allocates nothing):
    // partial rows (ws_part_slots rows of out floats) and arrival counters (kCounterSlots words)
    float* ws_part = nullptr;
    unsigned* ws_ctr = nullptr;
    int ws_part_slots = 0;
    // materialising path in row slabs: rows [row_begin, row_begin + rows) only (rows = 0: all);
    // wdense then holds that slab, row-major [rows][in]; both are multiples of 256
    int row_begin = 0, rows = 0;
};

// Limits of the decode kernel's work split
constexpr int kDecodeMaxRangeChunks = 32;   // 256-column chunks per workgroup (x/s table in LDS)
constexpr int kDecodeMaxBlocksPerWg = 32;   // blocks a workgroup walks through

// Tunables of the decode kernel (0 = choose by shape); measurement hooks, set through the
// bench-only entry point.  Atomics: a call may read them while another thread sets them.
struct DecodeTuning {
    std::atomic<int> tiles{0};      // 32-row tiles per wavefront: 2 or 4 (512 or 1024 rows per workgroup)
    std::atomic<int> ks_chunks{0};  // 256-column chunks per workgroup
    std::atomic<int> bgroups{0};    // block groups (workgroups per row slab / column range pair)
    std::atomic<int> early{-1};     // chunks of the first sign window requested before the prologue's arithmetic
};
DecodeTuning& decode_tuning();

hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int blocks, hipStream_t st);
hipError_t launch_zero(const LaunchArgs& a, hipStream_t st);
hipError_t launch_reference(const LaunchArgs& a, hipStream_t st);
// up to 4 batch-1 calls that read the same activation vector in one launch
hipError_t launch_decode_group(const LaunchArgs* a, int count, hipStream_t st);
// a.batch tokens through the decode kernel, up to four per launch
hipError_t launch_decode_tokens(const LaunchArgs& a, hipStream_t st);
// One token with the split-accumulation workspace in the library's static device array instead of
// the image's.  hipErrorOutOfMemory: the stack's rows do not fit the array (nothing launched).
constexpr size_t kStaticPartBytes = size_t(4) << 20;   // partial rows
constexpr size_t kStaticScratchBytes = kStaticPartBytes + size_t(kCounterSlots) * 4;
hipError_t launch_decode_static(const LaunchArgs& a, hipStream_t st);
double decode_tokens_time_us(const Geometry& g, int batch, int n_loaded);
hipError_t launch_panel(const LaunchArgs& a, hipStream_t st);
// materialising path: W' diag(1/s) of the loaded prefix -> a.wdense; then y = x wdense^T
hipError_t launch_restore(const LaunchArgs& a, hipStream_t st);
hipError_t launch_dense_zero(const LaunchArgs& a, hipStream_t st);
hipError_t launch_dense(const LaunchArgs& a, hipStream_t st);
// k_gemm's tile choice (128-row tiles or 256-row ones) and its estimated duration
void dense_force_tile(int tile);   // measurement hook: 1 = 256-row tiles, 2 = 128-row tiles, 3 = 128 x 128 tiles, 0 = the estimate's choice
double dense_time_us(int out, int in, int batch);
double restore_time_us(int rows, int in, int n_loaded, int* slices_out);   // and the column slices its launcher takes
// estimated durations of the two batch kernels (microseconds); launch_panel takes the cheaper one
// for 33..64 tokens
double fused_time_us(int out, int in, int batch, int n_loaded, int part_slots);
double tile_time_us(int out, int in, int batch, int n_loaded);
int restore_max_blocks();
// can the restore kernel take n_loaded blocks of this stride? (block count, and their bytes below 4 GiB)
bool restore_fits(size_t block_stride, int n_loaded);
// decomposition on the device (decompose.hip): W fp32 [out][in], s fp32 [in] (device copy inside the
// workspace), outputs canonical sign words and fp16 factors on the device
size_t decompose_workspace_bytes(int out, int in, int slices);
int decompose_slices(int out, int in);
hipError_t launch_decompose(const float* W, const float* s, int out, int in, int n, int iters, uint32_t* sign_words,
                            __half* U, __half* V, unsigned char* workspace, hipStream_t st);
// one block from canonical device arrays into slot `slot` of a packed image (same bytes as the host packer)
hipError_t launch_pack_block_device(const Geometry& g, unsigned char* image, int slot, const uint32_t* sign_words,
                                    const uint16_t* U, const uint16_t* V, hipStream_t st);
// column split the small-batch kernel uses for this shape (1 = none)
int small_batch_split(int out, int in, int batch, int part_slots);

}  // namespace bitstack
