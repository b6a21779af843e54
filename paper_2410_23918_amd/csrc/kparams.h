// Kernel parameter block shared by the HIP kernels of the library.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "layout.h"

namespace bitstack {

struct KParams {
    const __half* x;      // [batch][in]
    void* y;              // [batch][out]
    const float* rs;      // [in]   1/s
    const unsigned char* blocks;
    size_t block_stride, off_v, off_u;
    const __half* vmax;   // [n][in] max_r |V[j][r]|, panel order
    float* part;          // [part_slots][out] partial sums
    int part_slots;
    unsigned sign_bytes_total;  // n * block_stride: extent of the buffer descriptor over the blocks
    int n_bg;             // block groups: a workgroup walks blocks bg, bg + n_bg, ...
    unsigned* ctr;        // arrival counters (zero between calls)
    int out, in, batch, n_loaded;
    int n_rs, n_ks;       // row slabs, column ranges per block
    int ks_chunks;        // 256-column chunks per column range (the last range may be shorter)
    int y_f32;
    __half* xpack;        // activation scratch in fragment order (null if the image has none)
    void* wdense;         // fp16 [out][in]: restored weight (materialising path only)
    int row_begin;        // materialising path in row slabs: first row of the slab wdense holds
    int y_ld;             // elements between two token rows of y (the stack's out, also when p.out is a slab's)
};

// Several decode calls that read the same activation vector, merged into one launch: workgroup
// ids [base[i], base[i + 1]) belong to stack i (ranges padded to multiples of 8, so that the id
// modulo 8 -- the XCD a workgroup lands on -- means the same for every stack).
constexpr int kMaxGroup = 4;
struct KGroup {
    KParams s[kMaxGroup];
    unsigned base[kMaxGroup + 1];
    int count;
};

// One decode launch, fully prepared: the kernel's argument block, its grid and the variant
// (tiles per wavefront, chunks of the first window requested early).  Made once, launched many times.
struct DecodeLaunch {
    KGroup grp;
    unsigned wgs;
    int tiles, early;
};
hipError_t prepare_decode_group(const LaunchArgs* a, int count, DecodeLaunch* d);
hipError_t run_decode_launch(const DecodeLaunch& d, hipStream_t st);

inline KParams make_params(const LaunchArgs& a) {
    KParams p;
    p.x = static_cast<const __half*>(a.x);
    p.y = a.y;
    p.rs = reinterpret_cast<const float*>(a.image + a.geo.off_rs);
    p.blocks = a.image + a.geo.off_blocks;
    p.block_stride = a.geo.block_stride;
    p.off_v = a.geo.off_v;
    p.off_u = a.geo.off_u;
    p.vmax = reinterpret_cast<const __half*>(a.image + a.geo.off_vmax);
    p.part = a.ws_part ? a.ws_part : reinterpret_cast<float*>(a.image + a.geo.off_part);
    p.part_slots = a.ws_part ? a.ws_part_slots : a.geo.part_slots;
    p.n_bg = 1;
    p.ctr = a.ws_part ? a.ws_ctr : reinterpret_cast<unsigned*>(a.image + a.geo.off_ctr);
    p.out = a.geo.out;
    p.in = a.geo.in;
    p.batch = a.batch;
    p.n_loaded = a.n_loaded;
    p.n_rs = p.n_ks = 0;
    p.ks_chunks = 0;
    p.y_f32 = a.y_f32 ? 1 : 0;
    p.xpack = a.geo.xpack_bytes ? reinterpret_cast<__half*>(a.image + a.geo.off_xpack) : nullptr;
    p.wdense = a.wdense;
    p.row_begin = a.row_begin;
    p.y_ld = a.geo.out;
    return p;
}

// p.x [batch][in] -> p.xpack in matrix-core fragment order (tokens padded with zeros to a multiple of 32)
void launch_xpack(const KParams& p, hipStream_t st);

__device__ __forceinline__ void store_y(const KParams& p, size_t idx, float v) {
    if (p.y_f32)
        static_cast<float*>(p.y)[idx] = v;
    else
        static_cast<__half*>(p.y)[idx] = __float2half_rn(v);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load of the wavefront (its fence covers all address spaces), which
// would drain loads that were issued ahead on purpose (the decode kernel's sign window, the
// batch kernel's next-block inputs).
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

}  // namespace bitstack
