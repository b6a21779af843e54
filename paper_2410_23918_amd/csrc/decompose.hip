// The compression half of the method on the device: activation-aware scaling (Eq. 3-4) and the
// iterative absolute value decomposition (Section 2.1.2, Eq. 5-7; the decomposition loop of the
// overall algorithm in the appendix).  Per block i:
//
//     S_i = sign(R_i)  (sign(0) = +1),   |R_i| ~ U_i V_i^T  (top k = 16 singular triplets, sqrt(sigma)
//     split of Eq. 2, factors rounded to fp16),   R_{i+1} = R_i - S_i (.) (U_i V_i^T)   (Eq. 6)
//
// "SVD" is a block power (subspace) iteration with k + 16 columns followed by a Rayleigh-Ritz
// step; any method that returns the leading triplets is a valid reading.  Everything is fp32 on
// the vector ALUs except the 32 x 32 Gram / eigenvalue problems, which are fp64.  The two tall
// products per iteration, |R| X and |R|^T Y, read the fp32 residual once each and are bound by
// that read; |.| is applied as the residual is loaded, the sign matrix is never materialised.
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

// the Gram matrix from its parts, in a fixed order, into LDS (256 threads, four entries each)
__device__ __forceinline__ void gram_sum4(const double* Gpart, int parts, double (*Gs)[kL + 1]) {
    const int e0 = threadIdx.x * 4;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    typedef double d2 __attribute__((ext_vector_type(2)));
    int p = 0;
    for (; p + 4 <= parts; p += 4) {   // four parts' loads in flight together; the order of the additions is fixed
        d2 lo[4], hi[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const d2* src = reinterpret_cast<const d2*>(Gpart + size_t(p + u) * (kL * kL) + e0);
            lo[u] = src[0];
            hi[u] = src[1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a0 += lo[u][0]; a1 += lo[u][1]; a2 += hi[u][0]; a3 += hi[u][1];
        }
    }
    for (; p < parts; ++p) {
        const double* src = Gpart + size_t(p) * (kL * kL) + e0;
        a0 += src[0]; a1 += src[1]; a2 += src[2]; a3 += src[3];
    }
    const int row = e0 / kL, col = e0 % kL;
    Gs[row][col] = a0; Gs[row][col + 1] = a1; Gs[row][col + 2] = a2; Gs[row][col + 3] = a3;
}

// G = C^T C (Cholesky, C upper triangular), T = C^-1, so that Y T has orthonormal columns.
// 256 threads add up the parts of G; then 32 of them factorise in fp64: thread t keeps row t of
// the lower factor in registers, finished rows are published through LDS (one barrier per column).
__global__ __launch_bounds__(256) void k_dc_chol_inv(const double* Gpart, int parts, float* T) {
    __shared__ double Gs[kL][kL + 1];
    __shared__ double Lr[kL][kL + 1];
    const int t = threadIdx.x;
    gram_sum4(Gpart, parts, Gs);
    __syncthreads();
    if (t >= 64) return;   // the factorisation is one wavefront's work; its barriers then cost little
    double a[kL];
    if (t < kL) {
        Lr[t][t] = Gs[t][t];   // the diagonal, for the trace
#pragma unroll
        for (int c = 0; c < kL; ++c) a[c] = Gs[t][c];
    }
    __syncthreads();
    double tr = 0.0;
    for (int c = 0; c < kL; ++c) tr += Lr[c][c];
    if (!(tr > 0.0)) {   // Y = 0 (an all-zero residual): no direction to normalise, Q = 0
        if (t < kL)
            for (int c = 0; c < kL; ++c) T[t * kL + c] = 0.f;
        return;
    }
    // a tiny ridge keeps the factorisation defined if the columns are (numerically) dependent
    const double ridge = tr * 1e-13;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kL; ++j) {
        if (t == j) {
            double d = a[j] + ridge;
#pragma unroll
            for (int k = 0; k < j; ++k) d -= a[k] * a[k];
            a[j] = sqrt(d > 0.0 ? d : ridge);
#pragma unroll
            for (int k = 0; k <= j; ++k) Lr[j][k] = a[k];
        }
        __syncthreads();
        if (t > j && t < kL) {
            double v = a[j];
#pragma unroll
            for (int k = 0; k < j; ++k) v -= a[k] * Lr[j][k];
            a[j] = v / Lr[j][j];
        }
    }
    __syncthreads();
    // column t of L^-1 by forward substitution (in registers), T = C^-1 = (L^-1)^T
    if (t < kL) {
        double li[kL];
#pragma unroll
        for (int r = 0; r < kL; ++r) {
            double v = (r == t) ? 1.0 : 0.0;
#pragma unroll
            for (int k = 0; k < r; ++k) v -= (k >= t) ? Lr[r][k] * li[k] : 0.0;
            li[r] = (r < t) ? 0.0 : v / Lr[r][r];
        }
#pragma unroll
        for (int c = 0; c < kL; ++c) T[t * kL + c] = float(li[c]);
    }
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
    auto mul = [&](bool trans, const float* X) {
        const int M = trans ? in : out, K = trans ? out : in;
        const int chunks = K / kDcChunk;
        const int per = (chunks + slices - 1) / slices;
        dim3 grid((M + kDcTile - 1) / kDcTile, slices);
        if (trans)
            hipLaunchKernelGGL(k_dc_mul<true>, grid, dim3(256), 0, st, R, X, P, out, in, per);
        else
            hipLaunchKernelGGL(k_dc_mul<false>, grid, dim3(256), 0, st, R, X, P, out, in, per);
    };
    // the product in P, added up into raw (m x kL), columns made orthonormal into dst: Cholesky
    // QR with the Gram matrix in fp64; a second pass (twice = orthonormal to rounding) where asked
    auto orth = [&](float* raw, float* dst, int m, bool twice) {
        const int parts = (m + kGramRows - 1) / kGramRows;
        hipLaunchKernelGGL(k_dc_gram, dim3(parts), dim3(256), 0, st, P, slices, raw, m, G);
        hipLaunchKernelGGL(k_dc_chol_inv, dim3(1), dim3(256), 0, st, G, parts, T);
        hipLaunchKernelGGL((k_dc_apply<kL, false>), dim3((m + 255) / 256), dim3(256), 0, st, raw, T, dst, m);
        if (twice) {
            hipLaunchKernelGGL(k_dc_gram, dim3(parts), dim3(256), 0, st, dst, 1, raw, m, G);
            hipLaunchKernelGGL(k_dc_chol_inv, dim3(1), dim3(256), 0, st, G, parts, T);
            hipLaunchKernelGGL((k_dc_apply<kL, false>), dim3((m + 255) / 256), dim3(256), 0, st, raw, T, dst, m);
        }
    };

    for (int i = 0; i < n; ++i) {
        uint32_t* sw = sign_words + size_t(i) * out * (in / 32);
        __half* Ui = U + size_t(i) * out * kRank;
        __half* Vi = V + size_t(i) * in * kRank;
        const size_t waves = size_t(out) * (in / 64);
        hipLaunchKernelGGL(k_dc_signs, dim3(unsigned((waves + 3) / 4)), dim3(256), 0, st, R, sw, out, in);
        // start: random X (in x kL) -> Y = |R| X -> Q
        hipLaunchKernelGGL(k_dc_random, dim3(unsigned((size_t(in) * kL + 255) / 256)), dim3(256), 0, st, Qz,
                           size_t(in) * kL, 0x9e3779b9u * unsigned(i + 1));
        mul(false, Qz);
        orth(Y, Q, out, iters == 0);
        // one round = |R| |R|^T applied to Q; only Q is made orthonormal again (the product in
        // between spreads the columns' lengths by sigma_0 / sigma_31 ~ 30, far inside fp32)
        for (int it = 0; it < iters; ++it) {
            mul(true, Q);
            hipLaunchKernelGGL(k_dc_gram, dim3((in + kGramRows - 1) / kGramRows), dim3(256), 0, st, P, slices, Z, in, static_cast<double*>(nullptr));
            mul(false, Z);
            orth(Y, Q, out, it == iters - 1);
        }
        mul(true, Q);
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
