// The compression half of the method on the device: activation-aware scaling (Eq. 3-4) and the
// iterative absolute value decomposition (Section 2.1.2, Eq. 5-7; the decomposition loop of the
// overall algorithm in the appendix).  Per block i:
//
//     S_i = sign(R_i)  (sign(0) = +1),   |R_i| ~ U_i V_i^T  (top k = 16 singular triplets, sqrt(sigma)
//     split of Eq. 2, factors rounded to fp16),   R_{i+1} = R_i - S_i (.) (U_i V_i^T)   (Eq. 6)
//
// "SVD" is a block power (subspace) iteration with k + 16 columns followed by a Rayleigh-Ritz
// step; any method that returns the leading triplets is a valid reading.  The two tall products
// per round, |R| X and |R|^T Y, run on the bf16 matrix cores from bf16 copies of |R| (written once
// per block, row-major and transposed); the product of the Rayleigh-Ritz step, which fixes U and V,
// reads the fp32 residual (|.| applied as it is loaded); sums are fp32, the 32 x 32 Gram /
// Cholesky / eigenvalue problems fp64.  The sign matrix is never materialised.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "kernels.h"
#include "layout.h"

namespace bitstack {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kL = 32;        // subspace width: rank 16 + 16 columns of oversampling
constexpr int kDcTile = 128;  // output indices per workgroup of the tall products
constexpr int kDcChunk = 32;  // reduction indices per LDS stage

__global__ __launch_bounds__(256) void k_dc_scale(const float* W, const float* s, float* R, size_t total, int in) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i < total) R[i] = W[i] * s[i % size_t(in)];
}

// start vectors: any full-rank matrix will do; a counter-based hash keeps it reproducible
__global__ __launch_bounds__(256) void k_dc_random(float* X, size_t total, unsigned seed) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= total) return;
    unsigned h = unsigned(i) * 2654435761u ^ seed;
    h ^= h >> 16; h *= 0x85ebca6bu; h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    X[i] = float(int(h >> 8) - (1 << 23)) * (1.0f / float(1 << 23));
}

// fp32 -> bf16, round to nearest even (the residual is finite)
__device__ __forceinline__ unsigned short bf16_of(float x) {
    const unsigned u = __float_as_uint(x);
    return (unsigned short)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// canonical sign words of the residual: bit b of word w of a row = (R[row][32 w + b] >= 0),
// -0.0 and 0.0 both count as +1.  One wavefront per 64 consecutive columns of a row.
__global__ __launch_bounds__(256) void k_dc_signs(const float* R, uint32_t* words, int out, int in) {
    const size_t wid = size_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int groups = in / 64;
    if (wid >= size_t(out) * groups) return;   // whole wavefront
    const size_t row = wid / groups, cg = wid % groups;
    const float x = R[row * in + cg * 64 + lane];
    const unsigned long long m = __ballot(!(x < 0.0f));
    if (lane == 0) {
        words[row * (in / 32) + cg * 2] = uint32_t(m);
        words[row * (in / 32) + cg * 2 + 1] = uint32_t(m >> 32);
    }
}

// Tall products with A = |R| (out x in, row-major), kL columns on the other side, on the fp32
// matrix cores (v_mfma_f32_32x32x2_f32: 32 output indices x 32 columns, two reduction indices
// per instruction).
//   TRANS = false:  P[slice][o][c] = sum_{j in slice} |R[o][j]| X[j][c]     (M = out, K = in)
//   TRANS = true :  P[slice][j][c] = sum_{o in slice} |R[o][j]| X[o][c]     (M = in,  K = out)
// A workgroup (4 wavefronts) owns 128 output indices and one slice of the reduction range; the
// residual chunk goes to LDS as As[reduction index][output index] (|.| applied on the way), so
// that an operand is 32 consecutive floats for either orientation.  The slices are added up by
// the kernel that reads the product.
template <bool TRANS>
__global__ __launch_bounds__(256) void k_dc_mul(const float* R, const float* X, float* P, int out, int in,
                                                int chunks_per_slice) {
    __shared__ float As[kDcChunk][kDcTile + 4];
    __shared__ float Xs[kDcChunk][kL];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hl = lane >> 5, ln = lane & 31;
    const int M = TRANS ? in : out, K = TRANS ? out : in;
    const int m0 = blockIdx.x * kDcTile;
    const int chunks = K / kDcChunk;
    const int c_begin = blockIdx.y * chunks_per_slice;
    const int c_end = min(chunks, c_begin + chunks_per_slice);
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int ch = c_begin; ch < c_end; ++ch) {
        const int k0 = ch * kDcChunk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (!TRANS) {
                const int m = idx >> 3, q = idx & 7;   // row m0 + m, columns k0 + 4 q ..
                if (m0 + m < M) v = *reinterpret_cast<const float4*>(R + size_t(m0 + m) * in + k0 + 4 * q);
                As[4 * q + 0][m] = fabsf(v.x);
                As[4 * q + 1][m] = fabsf(v.y);
                As[4 * q + 2][m] = fabsf(v.z);
                As[4 * q + 3][m] = fabsf(v.w);
            } else {
                const int kk = idx >> 5, q = idx & 31;   // row k0 + kk, columns m0 + 4 q ..
                if (m0 + 4 * q < M) v = *reinterpret_cast<const float4*>(R + size_t(k0 + kk) * in + m0 + 4 * q);
                *reinterpret_cast<float4*>(&As[kk][4 * q]) = make_float4(fabsf(v.x), fabsf(v.y), fabsf(v.z), fabsf(v.w));
            }
        }
        {
            const int kk = tid >> 3, q = tid & 7;
            *reinterpret_cast<float4*>(&Xs[kk][4 * q]) = *reinterpret_cast<const float4*>(X + size_t(k0 + kk) * kL + 4 * q);
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kDcChunk; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[kk + hl][wave * 32 + ln], Xs[kk + hl][ln], acc, 0, 0, 0);
        __syncthreads();
    }
    // D[i = output index][n = column]: lane (column ln), register v holds index 8*(v/4) + 4*hl + v%4
    float* Ps = P + size_t(blockIdx.y) * M * kL;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = m0 + wave * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
        if (m < M) Ps[size_t(m) * kL + ln] = acc[v];
    }
}

// |R| as bf16, twice: Rh[o][j] and its transpose RhT[j][o], for the power rounds' tall products
// (half the bytes of the fp32 residual, and a reduction index that is contiguous in memory for
// either orientation).  64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void k_dc_half(const float* R, unsigned short* Rh, unsigned short* RhT, int out, int in) {
    __shared__ unsigned short Ts[64][64 + 2];
    const int tid = threadIdx.x;
    const int o0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, r = idx >> 4, q = idx & 15;   // row o0 + r, columns j0 + 4 q ..
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (o0 + r < out) v = *reinterpret_cast<const float4*>(R + size_t(o0 + r) * in + j0 + 4 * q);
        const unsigned short h[4] = {bf16_of(fabsf(v.x)), bf16_of(fabsf(v.y)), bf16_of(fabsf(v.z)), bf16_of(fabsf(v.w))};
        if (o0 + r < out)
            *reinterpret_cast<uint2*>(Rh + size_t(o0 + r) * in + j0 + 4 * q) =
                make_uint2(unsigned(h[0]) | unsigned(h[1]) << 16, unsigned(h[2]) | unsigned(h[3]) << 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) Ts[4 * q + e][r] = h[e];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, c = idx >> 4, q = idx & 15;   // column j0 + c, rows o0 + 4 q ..
        if (o0 + 4 * q < out)   // out is a multiple of 32: a group of four rows is inside or outside as a whole
            *reinterpret_cast<uint2*>(RhT + size_t(j0 + c) * out + o0 + 4 * q) =
                make_uint2(unsigned(Ts[c][4 * q]) | unsigned(Ts[c][4 * q + 1]) << 16,
                           unsigned(Ts[c][4 * q + 2]) | unsigned(Ts[c][4 * q + 3]) << 16);
    }
}

// The power rounds' tall products on the bf16 matrix cores: P[slice][m][c] = sum_{k in slice}
// A[m][k] X[k][c] with A = Rh (M = out, K = in) or RhT (M = in, K = out), row-major with K
// contiguous, X (K x kL, fp32) rounded to bf16 as it is staged.  A perturbation of |R| and of the
// iterate of 2^-9 relative per element turns the subspace the rounds converge to by far less than
// the oversampling and the Rayleigh-Ritz step, which works on the fp32 residual, absorb.  A
// workgroup (4 wavefronts) owns 128 output indices and one slice of the reduction range, 64
// reduction indices per LDS stage (K is a multiple of 32: a last half stage is filled with zeros).
constexpr int kHChunk = 64;
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(256) void k_dc_mulh(const unsigned short* A, const float* X, float* P, int M, int K,
                                                 int chunks_per_slice) {
    __shared__ __attribute__((aligned(16))) unsigned short As[kDcTile][kHChunk + 8];   // [m][k]
    __shared__ __attribute__((aligned(16))) unsigned short Xs[kL][kHChunk + 8];        // [c][k]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hl = lane >> 5, ln = lane & 31;
    const int m0 = blockIdx.x * kDcTile;
    const int chunks = (K + kHChunk - 1) / kHChunk;
    const int c_begin = blockIdx.y * chunks_per_slice;
    const int c_end = min(chunks, c_begin + chunks_per_slice);
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int ch = c_begin; ch < c_end; ++ch) {
        const int k0 = ch * kHChunk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i, m = idx >> 3, q = idx & 7;   // row m0 + m, reduction indices k0 + 8 q ..
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (m0 + m < M && k0 + 8 * q < K) v = *reinterpret_cast<const uint4*>(A + size_t(m0 + m) * K + k0 + 8 * q);
            *reinterpret_cast<uint4*>(&As[m][8 * q]) = v;
        }
        {
            const int kk = tid >> 2, cq = tid & 3;   // reduction index k0 + kk, columns 8 cq ..
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (k0 + kk < K) {
                a = *reinterpret_cast<const float4*>(X + size_t(k0 + kk) * kL + 8 * cq);
                b = *reinterpret_cast<const float4*>(X + size_t(k0 + kk) * kL + 8 * cq + 4);
            }
            const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) Xs[8 * cq + e][kk] = bf16_of(x[e]);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kHChunk / 16; ++s) {
            const v8bf a = *reinterpret_cast<const v8bf*>(&As[wave * 32 + ln][16 * s + 8 * hl]);
            const v8bf b = *reinterpret_cast<const v8bf*>(&Xs[ln][16 * s + 8 * hl]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    // D[i = output index][n = column]: lane (column ln), register v holds index 8*(v/4) + 4*hl + v%4
    float* Ps = P + size_t(blockIdx.y) * M * kL;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = m0 + wave * 32 + 8 * (v >> 2) + 4 * hl + (v & 3);
        if (m < M) Ps[size_t(m) * kL + ln] = acc[v];
    }
}

// Y = sum of the product's slices (written out) and this workgroup's part of Y^T Y in fp64:
// 128 rows of Y (m x kL) per workgroup in four stages of 32, every thread four columns of one row
// with the loads of all slices in flight together.  The parts are added up in a fixed order by
// the kernel that consumes the Gram matrix (no atomics: the decomposition is reproducible bit for
// bit).  Gpart == nullptr: only the sum is wanted.
constexpr int kGramRows = 128;
__global__ __launch_bounds__(256) void k_dc_gram(const float* P, int slices, float* Y, int m, double* Gpart) {
    __shared__ float Ys[32][kL + 1];
    const int tid = threadIdx.x, r = tid >> 3, cq = tid & 7;
    const int i = tid >> 3, jg = tid & 7;
    const size_t n = size_t(m) * kL;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int st = 0; st < kGramRows / 32; ++st) {
        const int row = blockIdx.x * kGramRows + st * 32 + r;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < m) {
            const float* src = P + size_t(row) * kL + 4 * cq;
            int sl = 0;
            for (; sl + 4 <= slices; sl += 4) {
                const float4 a = *reinterpret_cast<const float4*>(src + size_t(sl) * n);
                const float4 b = *reinterpret_cast<const float4*>(src + size_t(sl + 1) * n);
                const float4 c = *reinterpret_cast<const float4*>(src + size_t(sl + 2) * n);
                const float4 d = *reinterpret_cast<const float4*>(src + size_t(sl + 3) * n);
                v.x += (a.x + b.x) + (c.x + d.x); v.y += (a.y + b.y) + (c.y + d.y);
                v.z += (a.z + b.z) + (c.z + d.z); v.w += (a.w + b.w) + (c.w + d.w);
            }
            for (; sl < slices; ++sl) {
                const float4 a = *reinterpret_cast<const float4*>(src + size_t(sl) * n);
                v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
            }
            *reinterpret_cast<float4*>(Y + size_t(row) * kL + 4 * cq) = v;
        }
        if (Gpart == nullptr) continue;   // same for the whole grid
        Ys[r][4 * cq] = v.x; Ys[r][4 * cq + 1] = v.y; Ys[r][4 * cq + 2] = v.z; Ys[r][4 * cq + 3] = v.w;
        __syncthreads();
#pragma unroll 8
        for (int q = 0; q < 32; ++q) {
            const double yi = double(Ys[q][i]);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += yi * double(Ys[q][4 * jg + e]);
        }
        __syncthreads();
    }
    if (Gpart == nullptr) return;
    double* dst = Gpart + size_t(blockIdx.x) * (kL * kL) + i * kL + 4 * jg;
#pragma unroll
    for (int e = 0; e < 4; ++e) dst[e] = acc[e];
}

// the Gram matrix from its parts, in a fixed order, into LDS: 1024 threads, one entry each, the loads
// of up to 32 parts in flight together (one trip to memory per 32 parts instead of one per four)
constexpr int kSmallThreads = kL * kL;
__device__ __forceinline__ void gram_sum(const double* Gpart, int parts, double (*Gs)[kL + 1]) {
    const int e = threadIdx.x;
    double acc = 0.0;
    for (int p0 = 0; p0 < parts; p0 += 32) {
        double v[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) v[u] = p0 + u < parts ? Gpart[size_t(p0 + u) * (kL * kL) + e] : 0.0;
#pragma unroll
        for (int u = 0; u < 32; ++u) acc += v[u];   // the order of the additions is fixed
    }
    Gs[e / kL][e % kL] = acc;
}

// G = L L^T (Cholesky, L lower triangular) so that Q = Y L^-T has orthonormal columns; the kernel that
// applies it solves Q L^T = Y row by row.  Right-looking, one thread per matrix entry, fp64: at step
// j the threads of column j publish their entries (final after the updates of the earlier steps)
// and thread (j, j) the reciprocal of the pivot and its square root; after one barrier column j of
// L is raw / sqrt(pivot) and every entry below and right of the pivot takes its rank-one update.
// No chain of dependent operations longer than one division per step.
//   Lout: kL x kL fp32, row-major, L[r][c] for c < r, and 1 / L[r][r] on the diagonal (what the
//   substitution multiplies by); all zero for an all-zero Y (no direction to normalise: Q = 0).
__global__ __launch_bounds__(kSmallThreads) void k_dc_chol(const double* Gpart, int parts, float* Lout) {
    __shared__ double Gs[kL][kL + 1];
    __shared__ double colj[2][kL];
    __shared__ double piv[2][2];
    const int t = threadIdx.x, r = t / kL, c = t % kL;
    gram_sum(Gpart, parts, Gs);
    __syncthreads();
    double tr = 0.0;
#pragma unroll
    for (int k = 0; k < kL; ++k) tr += Gs[k][k];
    if (!(tr > 0.0)) {   // uniform over the workgroup
        Lout[t] = 0.f;
        return;
    }
    // a tiny ridge keeps the factorisation defined if the columns are (numerically) dependent
    const double ridge = tr * 1e-13;
    double a = Gs[r][c] + (r == c ? ridge : 0.0);
    double mine = 0.0;   // my entry of L (r > c), or 1 / L[r][r]
    for (int j = 0; j < kL; ++j) {
        const int b = j & 1;
        if (c == j && r >= j) {
            colj[b][r] = a;
            if (r == j) {
                const double d = a > 0.0 ? a : ridge;
                const double inv = 1.0 / d;
                piv[b][0] = inv;
                piv[b][1] = sqrt(inv);
            }
        }
        __syncthreads();
        if (c == j && r >= j) mine = r == j ? piv[b][1] : a * piv[b][1];   // 1 / sqrt(d), or a_rj / sqrt(d)
        if (c > j && r >= c) a -= colj[b][r] * colj[b][c] * piv[b][0];
    }
    Lout[t] = r >= c ? float(mine) : 0.f;
}

// Q L^T = Y for every row of Y (m x kL), L as k_dc_chol leaves it (reciprocal pivots on the diagonal):
// q_c = (y_c - sum_{i < c} q_i L[c][i]) / L[c][c].  One row per thread, L in LDS (all lanes read the
// same entry: a broadcast).  Y and Q may be the same array.
__global__ __launch_bounds__(256) void k_dc_solve(const float* Y, const float* Lg, float* Q, int m) {
    __shared__ __attribute__((aligned(16))) float Ls[kL][kL];
    for (int idx = threadIdx.x; idx < kL * kL; idx += 256) Ls[idx / kL][idx % kL] = Lg[idx];
    __syncthreads();
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= m) return;
    float q[kL];
#pragma unroll
    for (int g = 0; g < kL / 4; ++g) {
        const float4 v = *reinterpret_cast<const float4*>(Y + size_t(r) * kL + 4 * g);
        q[4 * g] = v.x; q[4 * g + 1] = v.y; q[4 * g + 2] = v.z; q[4 * g + 3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < kL; ++c) {
        float v = q[c];
#pragma unroll
        for (int i = 0; i < c; ++i) v = fmaf(-q[i], Ls[c][i], v);
        q[c] = v * Ls[c][c];
    }
#pragma unroll
    for (int g = 0; g < kL / 4; ++g)
        *reinterpret_cast<float4*>(Q + size_t(r) * kL + 4 * g) = make_float4(q[4 * g], q[4 * g + 1], q[4 * g + 2], q[4 * g + 3]);
}

// Q[r][c] = sum_i Y[r][i] T[i][c], c < NC; fp32 or fp16 (round to nearest even) output
template <int NC, bool HALF_OUT>
__global__ __launch_bounds__(256) void k_dc_apply(const float* Y, const float* T, void* Qv, int m) {
    __shared__ float Ts[kL][NC];
    for (int idx = threadIdx.x; idx < kL * NC; idx += 256) Ts[idx / NC][idx % NC] = T[idx];
    __syncthreads();
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= m) return;
    float y[kL];
#pragma unroll
    for (int q = 0; q < kL / 4; ++q) {
        const float4 v = *reinterpret_cast<const float4*>(Y + size_t(r) * kL + 4 * q);
        y[4 * q] = v.x; y[4 * q + 1] = v.y; y[4 * q + 2] = v.z; y[4 * q + 3] = v.w;
    }
    float o[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) o[c] = 0.f;
#pragma unroll
    for (int i = 0; i < kL; ++i)
#pragma unroll
        for (int c = 0; c < NC; ++c) o[c] = fmaf(y[i], Ts[i][c], o[c]);
    if (HALF_OUT) {
        __half* Q = static_cast<__half*>(Qv);
#pragma unroll
        for (int c = 0; c < NC; ++c) Q[size_t(r) * NC + c] = __float2half_rn(o[c]);
    } else {
        float* Q = static_cast<float*>(Qv);
#pragma unroll
        for (int c = 0; c < NC; ++c) Q[size_t(r) * NC + c] = o[c];
    }
}

// Rayleigh-Ritz step.  With Q orthonormal (out x kL) and Z = |R|^T Q (in x kL), G = Z^T Z =
// H diag(sigma^2) H^T gives the leading triplets of |R|: left vectors Q H, right vectors
// Z H diag(1/sigma).  Tu = H_k diag(sqrt(sigma)), Tv = H_k diag(1/sqrt(sigma)) (Eq. 2's split):
// U = Q Tu, V = Z Tv.  Jacobi rotations in fp64 in the round-robin ordering: 31 rounds of 16
// disjoint pairs per sweep, the 16 rotations of a round applied together by 512 threads, one per
// (line, pair); all 1024 add up the parts of G first.
__global__ __launch_bounds__(kSmallThreads) void k_dc_ritz(const double* Gpart, int parts, float* Tu, float* Tv, int k) {
    __shared__ double A[kL][kL + 1];
    __shared__ double H[kL][kL + 1];
    __shared__ double cs[kL / 2][2];
    __shared__ int pq[kL / 2][2];
    __shared__ int order[kL];
    __shared__ double offd[kL];
    const int t = threadIdx.x;
    gram_sum(Gpart, parts, A);
    H[t / kL][t % kL] = (t / kL == t % kL) ? 1.0 : 0.0;
    __syncthreads();
    // thread (line r, pair e) of the first 512 applies rotation e of a round to line r
    const int r = t >> 4, e = t & (kL / 2 - 1);
    for (int sweep = 0; sweep < 10; ++sweep) {
        // converged?  (off-diagonal mass against the trace; falls quadratically once small)
        if (t < kL) {
            double o = 0.0;
            for (int c = 0; c < kL; ++c) o += (c == t) ? 0.0 : A[t][c] * A[t][c];
            offd[t] = o;
        }
        __syncthreads();
        double off = 0.0, tr = 0.0;
        for (int c = 0; c < kL; ++c) {
            off += offd[c];
            tr += fabs(A[c][c]);
        }
        __syncthreads();
        if (off <= 1e-26 * tr * tr) break;   // same for every thread
        for (int round = 0; round < kL - 1; ++round) {
            if (t < kL / 2) {
                // pair t of this round: (kL - 1, round) and ((round + t) mod 31, (round - t) mod 31)
                int p = (t == 0) ? kL - 1 : (round + t) % (kL - 1);
                int q = (t == 0) ? round : (round - t + (kL - 1)) % (kL - 1);
                if (p > q) {
                    const int x = p;
                    p = q;
                    q = x;
                }
                const double apq = A[p][q], app = A[p][p], aqq = A[q][q];
                double c = 1.0, s = 0.0;
                if (fabs(apq) > 1e-300 && fabs(apq) > 1e-18 * sqrt(fabs(app * aqq))) {
                    const double tau = (aqq - app) / (2.0 * apq);
                    const double tt = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
                    c = 1.0 / sqrt(1.0 + tt * tt);
                    s = tt * c;
                }
                pq[t][0] = p;
                pq[t][1] = q;
                cs[t][0] = c;
                cs[t][1] = s;
            }
            __syncthreads();
            // the 16 pairs of a round are disjoint: 512 threads, one (line, pair) each
            const int p = pq[e][0], q = pq[e][1];
            const double c = cs[e][0], sn = cs[e][1];
            if (t < kL * kL / 2) {   // columns p, q of A and H: row r
                const double ap = A[r][p], aq = A[r][q], hp = H[r][p], hq = H[r][q];
                A[r][p] = c * ap - sn * aq;
                A[r][q] = sn * ap + c * aq;
                H[r][p] = c * hp - sn * hq;
                H[r][q] = sn * hp + c * hq;
            }
            __syncthreads();
            if (t < kL * kL / 2) {   // rows p, q of A: column r
                const double ap = A[p][r], aq = A[q][r];
                A[p][r] = c * ap - sn * aq;
                A[q][r] = sn * ap + c * aq;
            }
            __syncthreads();
        }
    }
    if (t == 0) {   // eigenvalues in descending order
        bool used[kL];
        for (int i = 0; i < kL; ++i) used[i] = false;
        for (int r = 0; r < kL; ++r) {
            int best = -1;
            for (int i = 0; i < kL; ++i)
                if (!used[i] && (best < 0 || A[i][i] > A[best][best])) best = i;
            used[best] = true;
            order[r] = best;
        }
    }
    __syncthreads();
    if (t < kL)
        for (int r = 0; r < k; ++r) {
            const int e = order[r];
            const double lam = A[e][e] > 0.0 ? A[e][e] : 0.0;
            const double sig = sqrt(lam);
            const double rt = sqrt(sig);
            Tu[t * k + r] = float(H[t][e] * rt);
            Tv[t * k + r] = rt > 0.0 ? float(H[t][e] / rt) : 0.f;
        }
}

// R <- R - sign(R) (.) (U V^T) with the factors as stored (fp16); 32 rows x 64 columns per workgroup
__global__ __launch_bounds__(256) void k_dc_update(float* R, const __half* U, const __half* V, int out, int in) {
    __shared__ float Us[32][kRank + 1];
    __shared__ float Vs[64][kRank + 1];
    const int tid = threadIdx.x;
    const int o0 = blockIdx.y * 32, j0 = blockIdx.x * 64;
    for (int idx = tid; idx < 32 * kRank; idx += 256) {
        const int r = idx / kRank, c = idx % kRank;
        Us[r][c] = (o0 + r < out) ? __half2float(U[size_t(o0 + r) * kRank + c]) : 0.f;
    }
    for (int idx = tid; idx < 64 * kRank; idx += 256) {
        const int r = idx / kRank, c = idx % kRank;
        Vs[r][c] = (j0 + r < in) ? __half2float(V[size_t(j0 + r) * kRank + c]) : 0.f;
    }
    __syncthreads();
    const int jl = tid & 63, rg = tid >> 6;   // column, group of 8 rows
    if (j0 + jl >= in) return;
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const int o = o0 + rg * 8 + rr;
        if (o >= out) break;
        float m = 0.f;
#pragma unroll
        for (int r = 0; r < kRank; ++r) m = fmaf(Us[rg * 8 + rr][r], Vs[jl][r], m);
        const size_t at = size_t(o) * in + j0 + jl;
        const float x = R[at];
        R[at] = (x < 0.0f) ? x + m : x - m;
    }
}

size_t decompose_workspace_bytes(int out, int in, int slices) {
    const size_t mx = size_t(out > in ? out : in);
    size_t b = align256(size_t(out) * in * 4);               // R
    b += 2 * align256(size_t(out) * in * 2);                 // |R| as bf16 and its transpose
    b += 2 * align256(size_t(out) * kL * 4);                 // Y, Q (out side)
    b += 2 * align256(size_t(in) * kL * 4);                  // Z, Qz (in side)
    b += align256(size_t(slices) * mx * kL * 4);             // partial products
    b += align256(((mx + kGramRows - 1) / kGramRows) * size_t(kL * kL * 8)) + 3 * align256(kL * kL * 4);  // Gram parts, T, Tu, Tv
    return b;
}

int decompose_slices(int out, int in) {
    // enough workgroups for 256 compute units: 128 output indices x one slice each
    const int tiles = ((out < in ? out : in) + kDcTile - 1) / kDcTile;
    int s = 1;
    while (tiles * s < 512 && s < 16) s *= 2;
    return s;
}

hipError_t launch_decompose(const float* W, const float* s, int out, int in, int n, int iters, uint32_t* sign_words,
                            __half* U, __half* V, unsigned char* ws, hipStream_t st) {
    const int slices = decompose_slices(out, in);
    const size_t mx = size_t(out > in ? out : in);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        unsigned char* p = ws + off;
        off += align256(bytes);
        return p;
    };
    float* R = reinterpret_cast<float*>(take(size_t(out) * in * 4));
    unsigned short* Rh = reinterpret_cast<unsigned short*>(take(size_t(out) * in * 2));
    unsigned short* RhT = reinterpret_cast<unsigned short*>(take(size_t(out) * in * 2));
    float* Y = reinterpret_cast<float*>(take(size_t(out) * kL * 4));
    float* Q = reinterpret_cast<float*>(take(size_t(out) * kL * 4));
    float* Z = reinterpret_cast<float*>(take(size_t(in) * kL * 4));
    float* Qz = reinterpret_cast<float*>(take(size_t(in) * kL * 4));
    float* P = reinterpret_cast<float*>(take(size_t(slices) * mx * kL * 4));
    double* G = reinterpret_cast<double*>(take(((mx + kGramRows - 1) / kGramRows) * size_t(kL * kL * 8)));
    float* T = reinterpret_cast<float*>(take(kL * kL * 4));
    float* Tu = reinterpret_cast<float*>(take(kL * kL * 4));
    float* Tv = reinterpret_cast<float*>(take(kL * kL * 4));

    const size_t total = size_t(out) * in;
    hipLaunchKernelGGL(k_dc_scale, dim3(unsigned((total + 255) / 256)), dim3(256), 0, st, W, s, R, total, in);

    // P = slices of |R| X  (X: in x kL)  or of  |R|^T X  (X: out x kL)
    // (exact: from the fp32 residual; otherwise from its bf16 copies, which the power rounds use)
    auto mul = [&](bool trans, const float* X, bool exact) {
        const int M = trans ? in : out, K = trans ? out : in;
        dim3 grid((M + kDcTile - 1) / kDcTile, slices);
        if (exact) {
            const int chunks = K / kDcChunk;
            const int per = (chunks + slices - 1) / slices;
            if (trans)
                hipLaunchKernelGGL(k_dc_mul<true>, grid, dim3(256), 0, st, R, X, P, out, in, per);
            else
                hipLaunchKernelGGL(k_dc_mul<false>, grid, dim3(256), 0, st, R, X, P, out, in, per);
        } else {
            const int chunks = (K + kHChunk - 1) / kHChunk;
            const int per = (chunks + slices - 1) / slices;
            hipLaunchKernelGGL(k_dc_mulh, grid, dim3(256), 0, st, trans ? RhT : Rh, X, P, M, K, per);
        }
    };
    // the product in P, added up into raw (m x kL), columns made orthonormal into dst: Cholesky
    // QR with the Gram matrix in fp64 (factor, then a triangular solve per row); a second pass
    // (twice = orthonormal to rounding) where asked
    auto orth = [&](float* raw, float* dst, int m, bool twice) {
        const int parts = (m + kGramRows - 1) / kGramRows;
        hipLaunchKernelGGL(k_dc_gram, dim3(parts), dim3(256), 0, st, P, slices, raw, m, G);
        hipLaunchKernelGGL(k_dc_chol, dim3(1), dim3(kSmallThreads), 0, st, G, parts, T);
        hipLaunchKernelGGL(k_dc_solve, dim3((m + 255) / 256), dim3(256), 0, st, raw, T, dst, m);
        if (twice) {
            hipLaunchKernelGGL(k_dc_gram, dim3(parts), dim3(256), 0, st, dst, 1, raw, m, G);
            hipLaunchKernelGGL(k_dc_chol, dim3(1), dim3(kSmallThreads), 0, st, G, parts, T);
            hipLaunchKernelGGL(k_dc_solve, dim3((m + 255) / 256), dim3(256), 0, st, raw, T, dst, m);
        }
    };

    for (int i = 0; i < n; ++i) {
        uint32_t* sw = sign_words + size_t(i) * out * (in / 32);
        __half* Ui = U + size_t(i) * out * kRank;
        __half* Vi = V + size_t(i) * in * kRank;
        const size_t waves = size_t(out) * (in / 64);
        hipLaunchKernelGGL(k_dc_signs, dim3(unsigned((waves + 3) / 4)), dim3(256), 0, st, R, sw, out, in);
        if (iters > 0)
            hipLaunchKernelGGL(k_dc_half, dim3(in / 64, (out + 63) / 64), dim3(256), 0, st, R, Rh, RhT, out, in);
        // start: random X (in x kL) -> Y = |R| X -> Q
        hipLaunchKernelGGL(k_dc_random, dim3(unsigned((size_t(in) * kL + 255) / 256)), dim3(256), 0, st, Qz,
                           size_t(in) * kL, 0x9e3779b9u * unsigned(i + 1));
        mul(false, Qz, iters == 0);
        orth(Y, Q, out, iters == 0);
        // one round = |R| |R|^T applied to Q; only Q is made orthonormal again (the product in
        // between spreads the columns' lengths by sigma_0 / sigma_31 ~ 30, far inside fp32)
        for (int it = 0; it < iters; ++it) {
            mul(true, Q, false);
            hipLaunchKernelGGL(k_dc_gram, dim3((in + kGramRows - 1) / kGramRows), dim3(256), 0, st, P, slices, Z, in, static_cast<double*>(nullptr));
            mul(false, Z, false);
            orth(Y, Q, out, it == iters - 1);
        }
        mul(true, Q, true);   // the Rayleigh-Ritz step sees the fp32 residual
        hipLaunchKernelGGL(k_dc_gram, dim3((in + kGramRows - 1) / kGramRows), dim3(256), 0, st, P, slices, Z, in, G);
        hipLaunchKernelGGL(k_dc_ritz, dim3(1), dim3(kSmallThreads), 0, st, G, (in + kGramRows - 1) / kGramRows, Tu, Tv, kRank);
        hipLaunchKernelGGL((k_dc_apply<kRank, true>), dim3((out + 255) / 256), dim3(256), 0, st, Q, Tu, Ui, out);
        hipLaunchKernelGGL((k_dc_apply<kRank, true>), dim3((in + 255) / 256), dim3(256), 0, st, Z, Tv, Vi, in);
        hipLaunchKernelGGL(k_dc_update, dim3((in + 63) / 64, (out + 31) / 32), dim3(256), 0, st, R, Ui, Vi, out, in);
    }
    return hipGetLastError();
}

// One block from canonical device arrays (what launch_decompose writes) into its slot of a packed
// image: sign words re-tiled, V into panel order, U copied, and the per-channel maxima of V.
// The same index functions as the host-side packer; the result is byte for byte the same.
__global__ __launch_bounds__(256) void k_pack_signs(const uint32_t* csw, uint32_t* dsw, int out, int in) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    const int wpr = in / 32;
    if (i >= size_t(out) * wpr) return;
    const int o = int(i / wpr), w = int(i % wpr);
    dsw[sign_word_index(in, o, w)] = csw[i];
}

__global__ __launch_bounds__(256) void k_pack_factors(const uint16_t* cu, const uint16_t* cv, uint16_t* du, uint16_t* dv,
                                                      uint16_t* vm, int out, int in) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < in) {
        uint16_t m = 0;
#pragma unroll
        for (int r = 0; r < kRank; ++r) {
            const uint16_t h = cv[size_t(i) * kRank + r];
            dv[v_index(i, r)] = h;
            uint16_t a = h & 0x7FFFu;
            if (a > 0x7C00u) a = 0x7C00u;   // NaN payloads: treat as infinity
            if (a > m) m = a;
        }
        vm[panel_index(i)] = m;
    }
    if (i < out) {
        const uint4* src = reinterpret_cast<const uint4*>(cu + size_t(i) * kRank);
        uint4* dst = reinterpret_cast<uint4*>(du + size_t(i) * kRank);
        dst[0] = src[0];
        dst[1] = src[1];
    }
}

hipError_t launch_pack_block_device(const Geometry& g, unsigned char* image, int slot, const uint32_t* csw,
                                    const uint16_t* cu, const uint16_t* cv, hipStream_t st) {
    unsigned char* blk = image + g.off_blocks + size_t(slot) * g.block_stride;
    uint16_t* vm = reinterpret_cast<uint16_t*>(image + g.off_vmax) + size_t(slot) * g.in;
    const size_t words = size_t(g.out) * (g.in / 32);
    hipLaunchKernelGGL(k_pack_signs, dim3(unsigned((words + 255) / 256)), dim3(256), 0, st, csw,
                       reinterpret_cast<uint32_t*>(blk), g.out, g.in);
    const int mx = g.out > g.in ? g.out : g.in;
    hipLaunchKernelGGL(k_pack_factors, dim3((mx + 255) / 256), dim3(256), 0, st, cu, cv,
                       reinterpret_cast<uint16_t*>(blk + g.off_u), reinterpret_cast<uint16_t*>(blk + g.off_v), vm, g.out,
                       g.in);
    return hipGetLastError();
}

}  // namespace bitstack
