// Dense factorisations the trusted side needs to build a fresh mixing matrix
// (Section 3.2 step 1.2; Table 3's "A-gen (QR)" step; Section 3.2.1 Mitigation 1):
//   - blocked Householder QR with explicit Q (orthogonal A),
//   - row-pivoted blocked LU and an explicit inverse (non-orthogonal A),
//   - a kappa_2 estimate by power iteration (the "generate and verify" check).
// Everything is float and deterministic: reductions run in a fixed order, no atomics.
//
// Both factorisations use column panels of width 16.  A panel is factorised by ONE workgroup
// that keeps its rows in registers (thread t owns rows t, t+NTHR, ...), so the per-column
// reductions cost a couple of barriers and no memory traffic.  The rank-16 updates of the
// trailing matrix are bandwidth-bound and run on the vector ALUs.
#include "gelo_internal.h"

namespace gelo {
namespace {

constexpr int NB = kPanel;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum of NB per-thread values over the workgroup, result broadcast to every thread.
// red: [NW][NB] floats, fin: [NB] floats of LDS.  Two barriers; callers separate successive
// uses by at least one more barrier (the panel loops do).
template <int NW>
__device__ __forceinline__ void block_sum_vec(float (&v)[NB], float* red, float* fin) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        const float t = wave_sum(v[s]);
        if (lane == 0) red[wave * NB + s] = t;
    }
    __syncthreads();
    if (tid < NB) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) t += red[w * NB + tid];
        fin[tid] = t;
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NB; ++s) v[s] = fin[s];
}

// ------------------------------------------------------------------ QR panel --
// Factorises the m x 16 panel at Mp (row stride ld) in place (R on and above the diagonal,
// reflector tails below, as in LAPACK), and writes for the block reflector I - V T V^T:
// Vc = V with explicit unit diagonal and zeros above, VT = V T, VTt = V T^T (m x 16 each,
// row stride ld), and rdiag[0:16] = diag(R).  Reflector j: beta = -sign(alpha) ||x||,
// tau = (beta - alpha)/beta, v = x / (alpha - beta) below the diagonal; a zero column gets tau = 0.
template <int NTHR, int R>
__global__ __launch_bounds__(NTHR)
void qr_panel_kernel(float* Mp, float* Vc, float* VT, float* VTt, float* rdiag, int64_t ld, int m) {
    constexpr int NW = NTHR / 64;
    __shared__ float red[NW * NB];
    __shared__ float fin[NB];
    __shared__ float Tm[NB][NB];
    __shared__ float tau_s[NB];
    __shared__ float alpha_s;

    const int tid = threadIdx.x;
    float P[R][NB];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r < m) {
#pragma unroll
            for (int c4 = 0; c4 < NB / 4; ++c4) {
                const float4 v = *reinterpret_cast<const float4*>(Mp + (int64_t)r * ld + c4 * 4);
                P[i][c4 * 4 + 0] = v.x; P[i][c4 * 4 + 1] = v.y; P[i][c4 * 4 + 2] = v.z; P[i][c4 * 4 + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int c = 0; c < NB; ++c) P[i][c] = 0.f;
        }
    }
    if (tid < NB) {
#pragma unroll
        for (int c = 0; c < NB; ++c) Tm[tid][c] = 0.f;
    }

#pragma unroll
    for (int j = 0; j < NB; ++j) {
        // ||x below the diagonal||^2 and alpha = x_0
        float part[NB];
#pragma unroll
        for (int s = 0; s < NB; ++s) part[s] = 0.f;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = tid + i * NTHR;
            if (r > j && r < m) part[0] = fmaf(P[i][j], P[i][j], part[0]);
        }
        if (tid == j) alpha_s = P[0][j];
        block_sum_vec<NW>(part, red, fin);
        const float xnorm2 = part[0];
        const float alpha = alpha_s;
        float beta = alpha, tau = 0.f, scale = 0.f;
        if (xnorm2 > 0.f) {
            beta = -copysignf(sqrtf(fmaf(alpha, alpha, xnorm2)), alpha);
            tau = (beta - alpha) / beta;
            scale = 1.0f / (alpha - beta);
        }
        // form v_j in place and the dot products of v_j with every other panel column
        // (columns s > j: the update; columns s < j hold v_s there: the Gram entries T needs)
        float vr[R];
#pragma unroll
        for (int s = 0; s < NB; ++s) part[s] = 0.f;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = tid + i * NTHR;
            float v = 0.f;
            if (r < m) {
                if (r > j) { P[i][j] *= scale; v = P[i][j]; }
                else if (r == j) { P[i][j] = beta; v = 1.f; }
            }
            vr[i] = v;
#pragma unroll
            for (int s = 0; s < NB; ++s)
                if (s != j) part[s] = fmaf(v, P[i][s], part[s]);
        }
        block_sum_vec<NW>(part, red, fin);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const float tv = tau * vr[i];
#pragma unroll
            for (int s = j + 1; s < NB; ++s) P[i][s] = fmaf(-tv, part[s], P[i][s]);
        }
        // column j of T: T[a][j] = -tau_j sum_{b<j} T[a][b] (v_b . v_j), T[j][j] = tau_j
        if (tid < NB) {
            if (tid < j) {
                float t = 0.f;
#pragma unroll
                for (int b = 0; b < j; ++b) t = fmaf(Tm[tid][b], part[b], t);
                Tm[tid][j] = -tau * t;
            } else if (tid == j) {
                Tm[j][j] = tau;
                tau_s[j] = tau;
                rdiag[j] = beta;
            }
        }
        __syncthreads();
    }

    // write back the factored panel and the three reflector blocks
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r >= m) continue;
        float v[NB], vt[NB], vtt[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) v[c] = r > c ? P[i][c] : (r == c ? 1.f : 0.f);
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            float a = 0.f, b = 0.f;
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                if (k <= c) a = fmaf(v[k], Tm[k][c], a);     // (V T)[r][c]
                if (k >= c) b = fmaf(v[k], Tm[c][k], b);     // (V T^T)[r][c]
            }
            vt[c] = a; vtt[c] = b;
        }
        float* mp = Mp + (int64_t)r * ld;
        float* vc = Vc + (int64_t)r * ld;
        float* vtp = VT + (int64_t)r * ld;
        float* vttp = VTt + (int64_t)r * ld;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4) {
            *reinterpret_cast<float4*>(mp + c4 * 4) = make_float4(P[i][c4 * 4], P[i][c4 * 4 + 1], P[i][c4 * 4 + 2], P[i][c4 * 4 + 3]);
            *reinterpret_cast<float4*>(vc + c4 * 4) = make_float4(v[c4 * 4], v[c4 * 4 + 1], v[c4 * 4 + 2], v[c4 * 4 + 3]);
            *reinterpret_cast<float4*>(vtp + c4 * 4) = make_float4(vt[c4 * 4], vt[c4 * 4 + 1], vt[c4 * 4 + 2], vt[c4 * 4 + 3]);
            *reinterpret_cast<float4*>(vttp + c4 * 4) = make_float4(vtt[c4 * 4], vtt[c4 * 4 + 1], vtt[c4 * 4 + 2], vtt[c4 * 4 + 3]);
        }
    }
}

// ------------------------------------------------------- skinny rank-16 kernels --
constexpr int SK_COLS = 64;      // columns per workgroup
constexpr int SK_ROWS = 256;     // rows per workgroup (chunk)

// Wpart[chunk][i][col] = sum over the chunk's rows r of V[r][i] * C[r][col]
__global__ __launch_bounds__(256)
void vt_c_partial_kernel(const float* V, int64_t ldv, const float* C, int64_t ldc, int rows, int cols,
                         float* Wpart, int64_t ldw) {
    __shared__ float Vs[SK_ROWS][NB];
    __shared__ float red[4][NB][SK_COLS];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * SK_ROWS;
    {   // row tid of the chunk: 16 contiguous floats
        const int r = r0 + tid;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < rows) v = *reinterpret_cast<const float4*>(V + (int64_t)r * ldv + c4 * 4);
            *reinterpret_cast<float4*>(&Vs[tid][c4 * 4]) = v;
        }
    }
    __syncthreads();
    const int lc = tid & 63, rg = tid >> 6;
    const int col = blockIdx.x * SK_COLS + lc;
    float acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = 0.f;
    if (col < cols) {
        const int rbeg = r0 + rg * 64;
        const int rend = (rbeg + 64 < rows) ? rbeg + 64 : rows;
        for (int r = rbeg; r < rend; ++r) {
            const float c = C[(int64_t)r * ldc + col];
            const float* vs = Vs[r - r0];
#pragma unroll
            for (int i = 0; i < NB; ++i) acc[i] = fmaf(vs[i], c, acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) red[rg][i][lc] = acc[i];
    __syncthreads();
    if (col < cols) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i = rg * 4 + t;
            const float s = (red[0][i][lc] + red[1][i][lc]) + (red[2][i][lc] + red[3][i][lc]);
            Wpart[((int64_t)blockIdx.y * NB + i) * ldw + col] = s;
        }
    }
}

// W[i][col] = sum_chunk Wpart[chunk][i][col], chunks added in index order
__global__ __launch_bounds__(256)
void reduce_w_kernel(const float* Wpart, int chunks, int cols, int64_t ldw, float* W) {
    const int col = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (col >= cols) return;
    float s = 0.f;
    for (int c = 0; c < chunks; ++c) s += Wpart[((int64_t)c * NB + i) * ldw + col];
    W[(int64_t)i * ldw + col] = s;
}

// C[r][col] -= sum_i L[r][i] * W[i][col]
__global__ __launch_bounds__(256)
void rank16_update_kernel(const float* L, int64_t ldl, const float* W, int64_t ldw, float* C, int64_t ldc,
                          int rows, int cols) {
    __shared__ float Ls[SK_ROWS][NB];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * SK_ROWS;
    {
        const int r = r0 + tid;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < rows) v = *reinterpret_cast<const float4*>(L + (int64_t)r * ldl + c4 * 4);
            *reinterpret_cast<float4*>(&Ls[tid][c4 * 4]) = v;
        }
    }
    __syncthreads();
    const int lc = tid & 63, rg = tid >> 6;
    const int col = blockIdx.x * SK_COLS + lc;
    if (col >= cols) return;
    float w[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) w[i] = W[(int64_t)i * ldw + col];
    const int rbeg = r0 + rg * 64;
    const int rend = (rbeg + 64 < rows) ? rbeg + 64 : rows;
    for (int r = rbeg; r < rend; ++r) {
        const float* ls = Ls[r - r0];
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NB; ++i) s = fmaf(ls[i], w[i], s);
        C[(int64_t)r * ldc + col] -= s;
    }
}

__global__ __launch_bounds__(256)
void set_identity_kernel(float* X, int64_t ld, int n_pad) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (c < ld && r < n_pad) X[(int64_t)r * ld + c] = (r == c) ? 1.f : 0.f;
}

__global__ __launch_bounds__(256)
void pad_matrix_kernel(float* M, int64_t ld, int n, int n_pad, int identity_block) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (c >= ld || r >= n_pad) return;
    if (r >= n || c >= n) M[(int64_t)r * ld + c] = (identity_block && r == c) ? 1.f : 0.f;
}

// ------------------------------------------------------------------ LU panel --
// Row-pivoted LU of the m x 16 panel at Mp, in place (unit-lower multipliers below the diagonal).
// piv[j] = panel-local row swapped with row j (first largest |value|).  *flag is set on a zero pivot.
template <int NTHR, int R>
__global__ __launch_bounds__(NTHR)
void lu_panel_kernel(float* Mp, int64_t ld, int m, int* piv, int row_offset, int* flag) {
    constexpr int NW = NTHR / 64;
    __shared__ float red_v[NW];
    __shared__ int red_i[NW];
    __shared__ float rowbuf[2][NB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float P[R][NB];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r < m) {
#pragma unroll
            for (int c4 = 0; c4 < NB / 4; ++c4) {
                const float4 v = *reinterpret_cast<const float4*>(Mp + (int64_t)r * ld + c4 * 4);
                P[i][c4 * 4 + 0] = v.x; P[i][c4 * 4 + 1] = v.y; P[i][c4 * 4 + 2] = v.z; P[i][c4 * 4 + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int c = 0; c < NB; ++c) P[i][c] = 0.f;
        }
    }

#pragma unroll
    for (int j = 0; j < NB; ++j) {
        // pivot search over rows >= j: largest |value|, smallest row on ties
        float bv = -1.f;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = tid + i * NTHR;
            if (r >= j && r < m) {
                const float a = fabsf(P[i][j]);
                if (a > bv) { bv = a; bi = r; }       // rows visited in increasing order per thread
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oi = __shfl_xor(bi, off, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { red_v[wave] = bv; red_i[wave] = bi; }
        __syncthreads();
        bv = red_v[0]; bi = red_i[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            const float ov = red_v[w];
            const int oi = red_i[w];
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        const int pr = bi < m ? bi : j;
        // exchange rows j and pr through LDS
        if (tid == j) {
#pragma unroll
            for (int c = 0; c < NB; ++c) rowbuf[0][c] = P[0][c];
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            if (tid + i * NTHR == pr) {
#pragma unroll
                for (int c = 0; c < NB; ++c) rowbuf[1][c] = P[i][c];
            }
        }
        __syncthreads();
        if (pr != j) {
            if (tid == j) {
#pragma unroll
                for (int c = 0; c < NB; ++c) P[0][c] = rowbuf[1][c];
            }
#pragma unroll
            for (int i = 0; i < R; ++i) {
                if (tid + i * NTHR == pr) {
#pragma unroll
                    for (int c = 0; c < NB; ++c) P[i][c] = rowbuf[0][c];
                }
            }
        }
        float prow[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) prow[c] = rowbuf[1][c];
        if (tid == 0) piv[j] = row_offset + pr;
        const float pivot = prow[j];
        if (pivot != 0.f) {
            const float inv = 1.0f / pivot;
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int r = tid + i * NTHR;
                if (r > j && r < m) {
                    const float l = P[i][j] * inv;
                    P[i][j] = l;
#pragma unroll
                    for (int c = j + 1; c < NB; ++c) P[i][c] = fmaf(-l, prow[c], P[i][c]);
                }
            }
        } else if (tid == 0) {
            *flag = 1;
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r >= m) continue;
        float* mp = Mp + (int64_t)r * ld;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4)
            *reinterpret_cast<float4*>(mp + c4 * 4) = make_float4(P[i][c4 * 4], P[i][c4 * 4 + 1], P[i][c4 * 4 + 2], P[i][c4 * 4 + 3]);
    }
}

// applies the 16 row interchanges of one panel (global rows row0 + j <-> piv[j]) to columns [cbeg, cend)
__global__ __launch_bounds__(256)
void swap_rows_kernel(float* M, int64_t ld, int row0, const int* piv, int cbeg, int cend) {
    const int c = cbeg + blockIdx.x * 256 + threadIdx.x;
    if (c >= cend) return;
#pragma unroll 1
    for (int j = 0; j < NB; ++j) {
        const int p = piv[j];
        if (p != row0 + j) {
            const float a = M[(int64_t)(row0 + j) * ld + c];
            const float b = M[(int64_t)p * ld + c];
            M[(int64_t)(row0 + j) * ld + c] = b;
            M[(int64_t)p * ld + c] = a;
        }
    }
}

// B[0:16, col] <- T^-1 B[0:16, col] for the 16 x 16 triangle T (row stride ldt):
// UPPER = false: unit lower triangle; UPPER = true: upper triangle with its diagonal.
template <bool UPPER>
__global__ __launch_bounds__(256)
void tri_solve_kernel(const float* T, int64_t ldt, float* B, int64_t ldb, int cols) {
    __shared__ float Ts[NB][NB];
    const int tid = threadIdx.x;
    Ts[tid >> 4][tid & 15] = T[(int64_t)(tid >> 4) * ldt + (tid & 15)];
    __syncthreads();
    const int col = blockIdx.x * 256 + tid;
    if (col >= cols) return;
    float x[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) x[i] = B[(int64_t)i * ldb + col];
    if (!UPPER) {
#pragma unroll
        for (int i = 1; i < NB; ++i)
#pragma unroll
            for (int k = 0; k < i; ++k) x[i] = fmaf(-Ts[i][k], x[k], x[i]);
    } else {
#pragma unroll
        for (int i = NB - 1; i >= 0; --i) {
#pragma unroll
            for (int k = i + 1; k < NB; ++k) x[i] = fmaf(-Ts[i][k], x[k], x[i]);
            x[i] /= Ts[i][i];
        }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) B[(int64_t)i * ldb + col] = x[i];
}

// ------------------------------------------------------------ power iteration --
// y[row] = (M[row, 0:n] . x) / ||x||, one wave per row
__global__ __launch_bounds__(256)
void matvec_unit_kernel(const float* M, int64_t ld, int n, const float* x, float* y) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n) return;
    float ss = 0.f, dot = 0.f;
    const float* mr = M + (int64_t)row * ld;
    for (int c = lane; c < n; c += 64) {
        const float xv = x[c];
        ss = fmaf(xv, xv, ss);
        dot = fmaf(mr[c], xv, dot);
    }
    ss = wave_sum(ss);
    dot = wave_sum(dot);
    if (lane == 0) y[row] = dot * rsqrtf(ss);
}

__global__ __launch_bounds__(256)
void start_vector_kernel(float* x, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        uint32_t h = (uint32_t)i * 2654435761u + 0x9E3779B9u;   // fixed pseudo-random signs and sizes
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        x[i] = ((h & 1u) ? 1.f : -1.f) * (0.5f + (float)((h >> 8) & 0xFFFF) * (1.0f / 65536.0f));
    }
}

// out[0] = ||xa|| * ||xi||  (sigma_max estimate times 1/sigma_min estimate); out[1], out[2] the factors
__global__ __launch_bounds__(1024)
void kappa_finish_kernel(const float* xa, const float* xi, int n, float* out) {
    __shared__ float ra[16], ri[16];
    const int tid = threadIdx.x;
    float a = 0.f, b = 0.f;
    for (int i = tid; i < n; i += 1024) { a = fmaf(xa[i], xa[i], a); b = fmaf(xi[i], xi[i], b); }
    a = wave_sum(a); b = wave_sum(b);
    if ((tid & 63) == 0) { ra[tid >> 6] = a; ri[tid >> 6] = b; }
    __syncthreads();
    if (tid == 0) {
        float sa = 0.f, sb = 0.f;
        for (int w = 0; w < 16; ++w) { sa += ra[w]; sb += ri[w]; }
        out[1] = sqrtf(sa); out[2] = sqrtf(sb);
        out[0] = sqrtf(sa) * sqrtf(sb);
    }
}

template <int NTHR>
hipError_t launch_qr_panel(int rows_per_thread, float* Mp, float* Vc, float* VT, float* VTt, float* rdiag,
                           int64_t ld, int m, hipStream_t s) {
    switch (rows_per_thread) {
#define GELO_CASE(RR) case RR: hipLaunchKernelGGL((qr_panel_kernel<NTHR, RR>), dim3(1), dim3(NTHR), 0, s, Mp, Vc, VT, VTt, rdiag, ld, m); break;
        GELO_CASE(1) GELO_CASE(2) GELO_CASE(3) GELO_CASE(4) GELO_CASE(5)
#undef GELO_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int NTHR>
hipError_t launch_lu_panel(int rows_per_thread, float* Mp, int64_t ld, int m, int* piv, int row_offset,
                           int* flag, hipStream_t s) {
    switch (rows_per_thread) {
#define GELO_CASE(RR) case RR: hipLaunchKernelGGL((lu_panel_kernel<NTHR, RR>), dim3(1), dim3(NTHR), 0, s, Mp, ld, m, piv, row_offset, flag); break;
        GELO_CASE(1) GELO_CASE(2) GELO_CASE(3) GELO_CASE(4) GELO_CASE(5)
#undef GELO_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t rank16_update(const float* L, int64_t ldl, const float* W, int64_t ldw, float* C, int64_t ldc,
                         int rows, int cols, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    hipLaunchKernelGGL(rank16_update_kernel, dim3((cols + SK_COLS - 1) / SK_COLS, (rows + SK_ROWS - 1) / SK_ROWS),
                       dim3(256), 0, s, L, ldl, W, ldw, C, ldc, rows, cols);
    return hipGetLastError();
}

// W (16 x cols, row stride ws.ld) = V^T C over `rows` rows
hipError_t vt_c(const FactorWorkspace& ws, const float* V, const float* C, int64_t ldc, int rows, int cols,
                hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const int chunks = (rows + SK_ROWS - 1) / SK_ROWS;
    if (chunks > ws.wpart_chunks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(vt_c_partial_kernel, dim3((cols + SK_COLS - 1) / SK_COLS, chunks), dim3(256), 0, s,
                       V, ws.ld, C, ldc, rows, cols, ws.Wpart, ws.ld);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_w_kernel, dim3((cols + 255) / 256, NB), dim3(256), 0, s,
                       ws.Wpart, chunks, cols, ws.ld, ws.W);
    return hipGetLastError();
}

#define GELO_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

}  // namespace

size_t factor_workspace_bytes(int n) {
    const int64_t n_pad = round_up(n, NB), ld = round_up(n, 64);
    const int64_t chunks = (n_pad + SK_ROWS - 1) / SK_ROWS;
    int64_t floats = 5 * n_pad * ld + chunks * NB * ld + NB * ld + n_pad + 4 * ld + 64;
    return (size_t)floats * sizeof(float) + (size_t)(n_pad + 64) * sizeof(int) + 4096;
}

void factor_workspace_carve(void* base, int n, FactorWorkspace* ws) {
    const int64_t n_pad = round_up(n, NB), ld = round_up(n, 64);
    const int64_t chunks = (n_pad + SK_ROWS - 1) / SK_ROWS;
    float* p = (float*)base;
    auto take = [&](int64_t count) { float* q = p; p += round_up(count, 64); return q; };
    ws->M = take(n_pad * ld);
    ws->X = take(n_pad * ld);
    ws->Vc = take(n_pad * ld);
    ws->VT = take(n_pad * ld);
    ws->VTt = take(n_pad * ld);
    ws->Wpart = take(chunks * NB * ld);
    ws->W = take(NB * ld);
    ws->rdiag = take(n_pad);
    ws->vec = take(4 * ld);
    ws->scalars = take(16);
    ws->piv = (int*)take(n_pad);
    ws->flag = (int*)take(16);
    ws->n_pad = (int)n_pad;
    ws->ld = ld;
    ws->wpart_chunks = (int)chunks;
}

__global__ void zero_ints_kernel(int* p, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0;
}

hipError_t zero_ints(int* p, int count, hipStream_t stream) {
    hipLaunchKernelGGL(zero_ints_kernel, dim3((count + 255) / 256), dim3(256), 0, stream, p, count);
    return hipGetLastError();
}

hipError_t set_identity(float* X, int64_t ld, int n_pad, hipStream_t stream) {
    hipLaunchKernelGGL(set_identity_kernel, dim3((unsigned)((ld + 255) / 256), n_pad), dim3(256), 0, stream, X, ld, n_pad);
    return hipGetLastError();
}

hipError_t pad_matrix(float* M, int64_t ld, int n, int n_pad, int identity_block, hipStream_t stream) {
    hipLaunchKernelGGL(pad_matrix_kernel, dim3((unsigned)((ld + 255) / 256), n_pad), dim3(256), 0, stream,
                       M, ld, n, n_pad, identity_block);
    return hipGetLastError();
}

hipError_t householder_qr(const FactorWorkspace& ws, hipStream_t s) {
    const int n_pad = ws.n_pad;
    const int64_t ld = ws.ld;
    const int panels = n_pad / NB;
    // factorise: panel, then trailing columns C <- (I - V T V^T)^T C = C - (V T^T)(V^T C)
    for (int p = 0; p < panels; ++p) {
        const int c0 = p * NB, m = n_pad - c0;
        const int64_t off = (int64_t)c0 * ld + c0;
        if (m <= 256 * 5) GELO_TRY(launch_qr_panel<256>((m + 255) / 256, ws.M + off, ws.Vc + off, ws.VT + off, ws.VTt + off, ws.rdiag + c0, ld, m, s));
        else GELO_TRY(launch_qr_panel<1024>((m + 1023) / 1024, ws.M + off, ws.Vc + off, ws.VT + off, ws.VTt + off, ws.rdiag + c0, ld, m, s));
        const int cols = n_pad - c0 - NB;
        if (cols > 0) {
            float* C = ws.M + off + NB;
            GELO_TRY(vt_c(ws, ws.Vc + off, C, ld, m, cols, s));
            GELO_TRY(rank16_update(ws.VTt + off, ld, ws.W, ld, C, ld, m, cols, s));
        }
    }
    // accumulate Q = H_0 H_1 ... : start from I, apply the block reflectors last to first; block p
    // only touches the trailing (n_pad - c0)^2 corner, which is still the identity elsewhere
    GELO_TRY(set_identity(ws.X, ld, n_pad, s));
    for (int p = panels - 1; p >= 0; --p) {
        const int c0 = p * NB, m = n_pad - c0;
        const int64_t off = (int64_t)c0 * ld + c0;
        float* C = ws.X + off;
        GELO_TRY(vt_c(ws, ws.Vc + off, C, ld, m, m, s));
        GELO_TRY(rank16_update(ws.VT + off, ld, ws.W, ld, C, ld, m, m, s));
    }
    return hipSuccess;
}

hipError_t lu_inverse(const FactorWorkspace& ws, hipStream_t s) {
    const int n_pad = ws.n_pad;
    const int64_t ld = ws.ld;
    const int panels = n_pad / NB;
    GELO_TRY(zero_ints(ws.flag, 1, s));
    GELO_TRY(set_identity(ws.X, ld, n_pad, s));
    for (int p = 0; p < panels; ++p) {
        const int c0 = p * NB, m = n_pad - c0;
        const int64_t off = (int64_t)c0 * ld + c0;
        if (m <= 256 * 5) GELO_TRY(launch_lu_panel<256>((m + 255) / 256, ws.M + off, ld, m, ws.piv + c0, c0, ws.flag, s));
        else GELO_TRY(launch_lu_panel<1024>((m + 1023) / 1024, ws.M + off, ld, m, ws.piv + c0, c0, ws.flag, s));
        // the same interchanges on the rest of the matrix and on the right-hand side (X ends up as P)
        if (c0 > 0) {
            hipLaunchKernelGGL(swap_rows_kernel, dim3((c0 + 255) / 256), dim3(256), 0, s, ws.M, ld, c0, ws.piv + c0, 0, c0);
            GELO_TRY(hipGetLastError());
        }
        const int cols = n_pad - c0 - NB;
        if (cols > 0) {
            hipLaunchKernelGGL(swap_rows_kernel, dim3((cols + 255) / 256), dim3(256), 0, s, ws.M, ld, c0, ws.piv + c0, c0 + NB, n_pad);
            GELO_TRY(hipGetLastError());
        }
        hipLaunchKernelGGL(swap_rows_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, s, ws.X, ld, c0, ws.piv + c0, 0, n_pad);
        GELO_TRY(hipGetLastError());
        if (cols > 0) {
            float* U12 = ws.M + off + NB;
            hipLaunchKernelGGL(tri_solve_kernel<false>, dim3((cols + 255) / 256), dim3(256), 0, s, ws.M + off, ld, U12, ld, cols);
            GELO_TRY(hipGetLastError());
            GELO_TRY(rank16_update(ws.M + off + (int64_t)NB * ld, ld, U12, ld, U12 + (int64_t)NB * ld, ld, m - NB, cols, s));
        }
    }
    // L Y = P
    for (int p = 0; p < panels; ++p) {
        const int c0 = p * NB;
        const int64_t off = (int64_t)c0 * ld + c0;
        float* Xb = ws.X + (int64_t)c0 * ld;
        hipLaunchKernelGGL(tri_solve_kernel<false>, dim3((n_pad + 255) / 256), dim3(256), 0, s, ws.M + off, ld, Xb, ld, n_pad);
        GELO_TRY(hipGetLastError());
        GELO_TRY(rank16_update(ws.M + off + (int64_t)NB * ld, ld, Xb, ld, Xb + (int64_t)NB * ld, ld, n_pad - c0 - NB, n_pad, s));
    }
    // U X = Y
    for (int p = panels - 1; p >= 0; --p) {
        const int c0 = p * NB;
        const int64_t off = (int64_t)c0 * ld + c0;
        float* Xb = ws.X + (int64_t)c0 * ld;
        hipLaunchKernelGGL(tri_solve_kernel<true>, dim3((n_pad + 255) / 256), dim3(256), 0, s, ws.M + off, ld, Xb, ld, n_pad);
        GELO_TRY(hipGetLastError());
        GELO_TRY(rank16_update(ws.M + c0, ld, Xb, ld, ws.X, ld, c0, n_pad, s));
    }
    return hipSuccess;
}

hipError_t kappa_estimate(const float* A, const float* Ainv, int64_t lda, int n, const FactorWorkspace& ws,
                          int iterations, hipStream_t s) {
    const int64_t ld = ws.ld;
    // transposes into the (now free) factorisation buffers
    GELO_TRY(emit_matrix(A, lda, nullptr, n, ld, nullptr, nullptr, ws.M, nullptr, s));
    GELO_TRY(emit_matrix(Ainv, lda, nullptr, n, ld, nullptr, nullptr, ws.X, nullptr, s));
    const dim3 grid((n + 3) / 4), block(256);
    float* x = ws.vec;
    float* y = ws.vec + ld;
    float* xa = ws.vec + 2 * ld;
    float* xi = ws.vec + 3 * ld;
    for (int op = 0; op < 2; ++op) {
        const float* Mf = op == 0 ? A : Ainv;            // forward operator
        const float* Mt = op == 0 ? ws.M : ws.X;         // its transpose
        const int64_t ldf = lda;
        float* last = op == 0 ? xa : xi;
        hipLaunchKernelGGL(start_vector_kernel, dim3((n + 255) / 256), dim3(256), 0, s, x, n);
        GELO_TRY(hipGetLastError());
        for (int it = 0; it < iterations; ++it) {
            hipLaunchKernelGGL(matvec_unit_kernel, grid, block, 0, s, Mf, ldf, n, x, y);
            GELO_TRY(hipGetLastError());
            float* dst = (it + 1 == iterations) ? last : x;
            hipLaunchKernelGGL(matvec_unit_kernel, grid, block, 0, s, Mt, ld, n, y, dst);
            GELO_TRY(hipGetLastError());
        }
    }
    hipLaunchKernelGGL(kappa_finish_kernel, dim3(1), dim3(1024), 0, s, xa, xi, n, ws.scalars);
    return hipGetLastError();
}

}  // namespace gelo
