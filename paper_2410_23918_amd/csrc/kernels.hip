// HIP kernels (gfx950 / CDNA4) for the BitStack linear layer
//     y = ( sum_i S_i (.) (U_i V_i^T) ) diag(1/s) x          (Eq. 4 + Eq. 8)
// that are not on the fast path: the zero fill for an empty prefix, the read-stream probe the
// measurements are priced against, and a plain second implementation of the forward pass for
// tests.  The batch-1 kernel is in decode.hip, the batch kernels in panel.hip.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "kparams.h"
#include "layout.h"

namespace bitstack {

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

}  // namespace bitstack
