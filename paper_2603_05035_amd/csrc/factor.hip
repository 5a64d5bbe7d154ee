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
#include <type_traits>
#include <utility>

#include "gelo_internal.h"

namespace gelo {
namespace {

constexpr int NB = kPanel;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
    (f(std::integral_constant<int, Is>{}), ...);
}
// compile-time loop: the body sees its index as a constant, so register arrays stay in registers
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int PATTERN>
__device__ __forceinline__ float swizzle(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), PATTERN));
}

// Index of the value that lane `lane` ends up holding after wave_reduce16.
__device__ __forceinline__ int reduce16_slot(int lane) {
    return ((lane >> 2) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 1) & 1) * 2 + (lane & 1);
}

// Sums 16 per-lane values over the 64 lanes of a wave in ~50 instructions: each exchange step
// halves the number of values a lane carries (the lane keeps the half its partner does not),
// so after four steps inside a row of 16 lanes every lane holds ONE value, summed over its row;
// two more exchanges add the four rows.  Returns, in every lane, the wave total of value
// reduce16_slot(lane).  All 64 lanes must be active.  The order of additions is fixed.
__device__ __forceinline__ float wave_reduce16(const float (&t)[NB], int lane) {
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4, b3 = lane & 8;
    float a[8], c[4], e[2];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float keep = b0 ? t[2 * k + 1] : t[2 * k];
        const float give = b0 ? t[2 * k] : t[2 * k + 1];
        a[k] = keep + dpp_mov<0xB1>(give);              // lane ^ 1  (quad_perm [1,0,3,2])
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float keep = b1 ? a[2 * k + 1] : a[2 * k];
        const float give = b1 ? a[2 * k] : a[2 * k + 1];
        c[k] = keep + dpp_mov<0x4E>(give);              // lane ^ 2  (quad_perm [2,3,0,1])
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float keep = b3 ? c[2 * k + 1] : c[2 * k];
        const float give = b3 ? c[2 * k] : c[2 * k + 1];
        e[k] = keep + dpp_mov<0x128>(give);             // lane ^ 8  (row_ror:8)
    }
    const float keep = b2 ? e[1] : e[0];
    const float give = b2 ? e[0] : e[1];
    float f = keep + swizzle<0x101F>(give);             // lane ^ 4
    f += swizzle<0x401F>(f);                            // lane ^ 16
    f += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, f)));
    return f;
}

template <int LANE>
__device__ __forceinline__ float lane_value(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), LANE));
}

// ------------------------------------------------------------------ QR panel --
// Factorises the m x 16 panel at Mp (row stride ld) in place (R on and above the diagonal,
// reflector tails below, as in LAPACK), and writes for the block reflector I - V T V^T:
// Vc = V with explicit unit diagonal and zeros above (m x 16, row stride ld), T (16 x 16,
// dense row-major at Tg) and rdiag[0:16] = diag(R).  Reflector j: beta = -sign(alpha) ||x||,
// tau = (beta - alpha)/beta, v = x / (alpha - beta) below the diagonal; a zero tail gets tau = 0.
//
// One workgroup reduction and one barrier per column: with x the column below the diagonal,
// t[s] = x . P[below, s] for all 16 columns s gives the tail norm (s = j) and, with the broadcast
// pivot row, v . P[:, s] = scale * t[s] + P[j][s], which is both the update coefficient (s > j)
// and the Gram entry v_s . v_j that the T factor needs (s < j).  After the reduction lane s of
// every wave holds the quantities of column s; the update coefficients are then read into
// scalar registers.  The column loop is unrolled so that all register indices are constants.
// Mp: the panel's first 16 x 16 tile; the tiles of the rows below follow at 256 floats each
// (element (r, c) at Mp[(r / 16) * 256 + c * 16 + r % 16]).  The reflector block is written twice,
// compactly: Vr[r * 16 + c] (row-major, the A operand of C += V W') and Vt in the same tiles as
// the panel (the A operand of W = V^T C), both with explicit unit diagonal and zeros above.
template <int NTHR, int R>
__device__ __forceinline__ void qr_panel_body(float* Mp, float* Vr, float* Vt, float* Tg, float* rdiag, int m) {
    constexpr int NW = NTHR / 64;
    __shared__ float red[2][NW][NB];
    __shared__ float prow[2][NB];
    __shared__ float Z[NB][NB];          // Z[j][s] = v_j . (column s) at step j
    __shared__ float tau_s[NB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15;
    const int slot = reduce16_slot(lane);
    float P[R][NB];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        const int64_t at = (int64_t)(r >> 4) * 256 + (r & 15);
#pragma unroll
        for (int c = 0; c < NB; ++c) P[i][c] = r < m ? Mp[at + c * 16] : 0.f;             // 16 consecutive lanes, consecutive addresses
    }

    // Rows at or beyond m hold zeros and stay zero, rows tid + i NTHR with i > 0 lie below every
    // diagonal entry of the panel: only register row 0 needs a test against j, and that test is a
    // select, so the column loop is straight-line code.
    static_for<NB>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        constexpr int pb = j & 1;                       // LDS buffers alternate between columns
        float t[NB];
        {
            const float x = tid > j ? P[0][j] : 0.f;
#pragma unroll
            for (int s = 0; s < NB; ++s) t[s] = x * P[0][s];
        }
#pragma unroll
        for (int i = 1; i < R; ++i) {
            const float x = P[i][j];
#pragma unroll
            for (int s = 0; s < NB; ++s) t[s] = fmaf(x, P[i][s], t[s]);
        }
        if (tid == j) {                                 // row j is register row 0 of thread j
#pragma unroll
            for (int s = 0; s < NB; ++s) prow[pb][s] = P[0][s];
        }
        const float part = wave_reduce16(t, lane);
        if (lane < NB) red[pb][wave][slot] = part;
        __syncthreads();
        float tot = red[pb][0][li];                     // lane (li) now works on column li
#pragma unroll
        for (int w = 1; w < NW; ++w) tot += red[pb][w][li];
        const float pr = prow[pb][li];
        const float xnorm2 = lane_value<j>(tot);
        const float alpha = lane_value<j>(pr);
        // beta = -sign(alpha) sqrt(alpha^2 + |x|^2), tau = (beta - alpha) / beta, scale = 1 / (alpha - beta); the
        // hardware square root and reciprocals (1 ulp) keep this dependent chain short.  A zero tail: tau = 0.
        const bool tail = xnorm2 > 0.f;
        const float nrm = __builtin_amdgcn_sqrtf(fmaf(alpha, alpha, xnorm2));
        const float beta = tail ? -copysignf(nrm, alpha) : alpha;
        const float tau = tail ? (beta - alpha) * __builtin_amdgcn_rcpf(beta) : 0.f;
        const float scale = tail ? __builtin_amdgcn_rcpf(alpha - beta) : 0.f;
        const float wl = fmaf(scale, tot, pr);          // v_j . (column li)
        if (tid < NB) {
            Z[j][tid] = wl;
            if (tid == 0) { tau_s[j] = tau; rdiag[j] = beta; }
        }
        float w[NB];
        static_for<NB>([&](auto sc) {
            constexpr int s = decltype(sc)::value;
            if constexpr (s > j) w[s] = lane_value<s>(wl);
        });
        {
            // register row 0: below the diagonal v = x * scale, on it v = 1 and the entry becomes beta, above it nothing
            const float v = tid > j ? P[0][j] * scale : (tid == j ? 1.f : 0.f);
            P[0][j] = tid > j ? v : (tid == j ? beta : P[0][j]);
            const float tv = tau * v;
#pragma unroll
            for (int s = j + 1; s < NB; ++s) P[0][s] = fmaf(-tv, w[s], P[0][s]);
        }
#pragma unroll
        for (int i = 1; i < R; ++i) {
            const float v = P[i][j] * scale;
            P[i][j] = v;
            const float tv = tau * v;
#pragma unroll
            for (int s = j + 1; s < NB; ++s) P[i][s] = fmaf(-tv, w[s], P[i][s]);
        }
    });
    __syncthreads();

    // T by the forward recurrence T[a][j] = -tau_j sum_{b<j} T[a][b] (v_b . v_j), T[j][j] = tau_j;
    // lane a of the first wave carries row a.
    if (tid < NB) {
        float Trow[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) Trow[c] = 0.f;
        static_for<NB>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            float acc = 0.f;
#pragma unroll
            for (int bb = 0; bb < j; ++bb) acc = fmaf(Trow[bb], Z[j][bb], acc);
            const float tj = tau_s[j];
            Trow[j] = tid < j ? -tj * acc : (tid == j ? tj : 0.f);
        });
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4)
            *reinterpret_cast<float4*>(Tg + tid * NB + c4 * 4) =
                make_float4(Trow[c4 * 4], Trow[c4 * 4 + 1], Trow[c4 * 4 + 2], Trow[c4 * 4 + 3]);
    }

    // write back the factored panel and the clean reflector block
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r < m) {
#pragma unroll
            for (int c4 = 0; c4 < NB / 4; ++c4) {
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = c4 * 4 + e;
                    v[e] = r > c ? P[i][c] : (r == c ? 1.f : 0.f);
                    Mp[(int64_t)(r >> 4) * 256 + c * 16 + (r & 15)] = P[i][c];
                    Vt[(int64_t)(r >> 4) * 256 + c * 16 + (r & 15)] = v[e];
                }
                *reinterpret_cast<float4*>(Vr + (int64_t)r * NB + c4 * 4) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

template <int NTHR, int R>
__global__ __launch_bounds__(NTHR)
void qr_panel_kernel(float* Mp, float* Vr, float* Vt, float* Tg, float* rdiag, int m) {
    qr_panel_body<NTHR, R>(Mp, Vr, Vt, Tg, rdiag, m);
}

// ------------------------------------------------------- skinny rank-16 kernels --
// Both work on tiles of 128 rows x 64 columns with 128 threads: thread (ct, rt) owns 4 adjacent
// columns (one 16-byte access per row) of the 16 rows rt, rt+8, ...
constexpr int SK_COLS = 64;
constexpr int SK_ROWS = 128;
constexpr int SK_THREADS = 128;

// Wpart[tile][i][col] = sum over the rows r of tile blockIdx.y of V[r][i] * C[r][col]
__global__ __launch_bounds__(SK_THREADS)
void vt_c_partial_kernel(const float* V, int64_t ldv, const float* C, int64_t ldc, int rows, int cols,
                         float* Wpart, int64_t ldw) {
    __shared__ __attribute__((aligned(16))) float Vs[SK_ROWS][NB];
    __shared__ __attribute__((aligned(16))) float red[8][NB][SK_COLS];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * SK_ROWS;
#pragma unroll
    for (int t = 0; t < 4; ++t) {                   // 128 rows x 4 chunks of 16 bytes
        const int id = tid + t * SK_THREADS;
        const int r = id >> 2, c4 = id & 3;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < rows) v = *reinterpret_cast<const float4*>(V + (int64_t)(r0 + r) * ldv + c4 * 4);
        *reinterpret_cast<float4*>(&Vs[r][c4 * 4]) = v;
    }
    __syncthreads();
    const int ct = tid & 15, rt = tid >> 4;
    const int col = blockIdx.x * SK_COLS + ct * 4;
    float acc[NB][4];
#pragma unroll
    for (int i = 0; i < NB; ++i) { acc[i][0] = acc[i][1] = acc[i][2] = acc[i][3] = 0.f; }
    if (col < cols) {
        float4 c[16];
#pragma unroll
        for (int ii = 0; ii < 16; ++ii) {
            const int r = r0 + rt + 8 * ii;
            c[ii] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < rows) c[ii] = *reinterpret_cast<const float4*>(C + (int64_t)r * ldc + col);
        }
#pragma unroll
        for (int ii = 0; ii < 16; ++ii) {
            const float* vs = Vs[rt + 8 * ii];
#pragma unroll
            for (int i4 = 0; i4 < NB / 4; ++i4) {
                const float4 v = *reinterpret_cast<const float4*>(vs + i4 * 4);
                const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[i4 * 4 + e][0] = fmaf(vv[e], c[ii].x, acc[i4 * 4 + e][0]);
                    acc[i4 * 4 + e][1] = fmaf(vv[e], c[ii].y, acc[i4 * 4 + e][1]);
                    acc[i4 * 4 + e][2] = fmaf(vv[e], c[ii].z, acc[i4 * 4 + e][2]);
                    acc[i4 * 4 + e][3] = fmaf(vv[e], c[ii].w, acc[i4 * 4 + e][3]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i)
        *reinterpret_cast<float4*>(&red[rt][i][ct * 4]) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    __syncthreads();
    // 16 x 64 outputs of this tile, 8 per thread, each the sum of 8 partials in a fixed order
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int id = tid + t * SK_THREADS;        // 0..255: (i, 4-column group)
        const int i = id >> 4, cg = id & 15;
        const int ocol = blockIdx.x * SK_COLS + cg * 4;
        if (ocol < cols) {
            float4 s = *reinterpret_cast<const float4*>(&red[0][i][cg * 4]);
#pragma unroll
            for (int g = 1; g < 8; ++g) {
                const float4 q = *reinterpret_cast<const float4*>(&red[g][i][cg * 4]);
                s.x += q.x; s.y += q.y; s.z += q.z; s.w += q.w;
            }
            *reinterpret_cast<float4*>(Wpart + ((int64_t)blockIdx.y * NB + i) * ldw + ocol) = s;
        }
    }
}

// W[0:16, strip] = op(T) * sum_tile Wpart[tile][0:16, strip] for the 64-column strip blockIdx.x;
// tiles are added in index order; op(T) = T^T if t_transposed.
__global__ __launch_bounds__(SK_THREADS)
void reduce_apply_kernel(const float* Wpart, int tiles, int cols, int64_t ldw, const float* T, int t_transposed,
                         float* W) {
    __shared__ __attribute__((aligned(16))) float Wsum[NB][SK_COLS];
    __shared__ float Ts[NB][NB];
    const int tid = threadIdx.x;
    if (tid < NB) {
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4)
            *reinterpret_cast<float4*>(&Ts[tid][c4 * 4]) = *reinterpret_cast<const float4*>(T + tid * NB + c4 * 4);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int id = tid + t * SK_THREADS;
        const int i = id >> 4, cg = id & 15;
        const int ocol = blockIdx.x * SK_COLS + cg * 4;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ocol < cols) {
#pragma unroll 4
            for (int tl = 0; tl < tiles; ++tl) {
                const float4 q = *reinterpret_cast<const float4*>(Wpart + ((int64_t)tl * NB + i) * ldw + ocol);
                s.x += q.x; s.y += q.y; s.z += q.z; s.w += q.w;
            }
        }
        *reinterpret_cast<float4*>(&Wsum[i][cg * 4]) = s;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int id = tid + t * SK_THREADS;
        const int i = id >> 4, cg = id & 15;
        const int ocol = blockIdx.x * SK_COLS + cg * 4;
        if (ocol < cols) {
            float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const float tk = t_transposed ? Ts[k][i] : Ts[i][k];       // (T^T W)[i] or (T W)[i]
                const float4 q = *reinterpret_cast<const float4*>(&Wsum[k][cg * 4]);
                o.x = fmaf(tk, q.x, o.x); o.y = fmaf(tk, q.y, o.y); o.z = fmaf(tk, q.z, o.z); o.w = fmaf(tk, q.w, o.w);
            }
            *reinterpret_cast<float4*>(W + (int64_t)i * ldw + ocol) = o;
        }
    }
}

// C[r][col] -= sum_i L[r][i] * W[i][col]
__global__ __launch_bounds__(SK_THREADS)
void rank16_update_kernel(const float* L, int64_t ldl, const float* W, int64_t ldw, float* C, int64_t ldc,
                          int rows, int cols) {
    __shared__ __attribute__((aligned(16))) float Ls[SK_ROWS][NB];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * SK_ROWS;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int id = tid + t * SK_THREADS;
        const int r = id >> 2, c4 = id & 3;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < rows) v = *reinterpret_cast<const float4*>(L + (int64_t)(r0 + r) * ldl + c4 * 4);
        *reinterpret_cast<float4*>(&Ls[r][c4 * 4]) = v;
    }
    __syncthreads();
    const int ct = tid & 15, rt = tid >> 4;
    const int col = blockIdx.x * SK_COLS + ct * 4;
    if (col >= cols) return;
    float4 w[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) w[i] = *reinterpret_cast<const float4*>(W + (int64_t)i * ldw + col);
    float4 c[16];
#pragma unroll
    for (int ii = 0; ii < 16; ++ii) {
        const int r = r0 + rt + 8 * ii;
        c[ii] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < rows) c[ii] = *reinterpret_cast<const float4*>(C + (int64_t)r * ldc + col);
    }
#pragma unroll
    for (int ii = 0; ii < 16; ++ii) {
        const int r = r0 + rt + 8 * ii;
        const float* ls = Ls[rt + 8 * ii];
        float4 s = c[ii];
#pragma unroll
        for (int i4 = 0; i4 < NB / 4; ++i4) {
            const float4 l = *reinterpret_cast<const float4*>(ls + i4 * 4);
            const float lv[4] = {l.x, l.y, l.z, l.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s.x = fmaf(-lv[e], w[i4 * 4 + e].x, s.x);
                s.y = fmaf(-lv[e], w[i4 * 4 + e].y, s.y);
                s.z = fmaf(-lv[e], w[i4 * 4 + e].z, s.z);
                s.w = fmaf(-lv[e], w[i4 * 4 + e].w, s.w);
            }
        }
        if (r < rows) *reinterpret_cast<float4*>(C + (int64_t)r * ldc + col) = s;
    }
}

// ------------------------------------------------- fused block-reflector update --
// C <- C - V op(T) V^T C for a 16-column strip of C per workgroup, in ONE pass over C: the strip
// (m x 16, m a multiple of 16) lives in registers as 16 x 16 blocks in the accumulator layout of
// v_mfma_f32_16x16x4_f32, so the same registers serve as the B operand of W = V^T C (K = rows)
// and as the accumulator of C -= V W' (K = the 16 reflectors).  Wave w of 8 owns blocks
// w, w+8, ...; the 8 partial W are added in wave order (fixed order, reproducible), then
// W' = -op(T) W is formed once per strip.
// Layouts, chosen so that every global access of a wave is one contiguous kilobyte, 16 bytes per
// lane: the strip is a column of 16 x 16 tiles (256 floats each, [column][row] inside: the four
// rows 4 g .. 4 g + 3 a lane owns are adjacent), the reflectors come in the same tiles (Vt) for the
// first product and as Vr[r * 16 + i] for the second.
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int NBLK>
__device__ __forceinline__ void reflect_strip_body(const float* __restrict__ Vr, const float* __restrict__ Vt,
                                                   const float* __restrict__ T, int t_transposed, float* Cs, int nblocks) {
    __shared__ float Wp[8][NB][NB];
    __shared__ float Ws[NB][NB];
    __shared__ float Wn[NB][NB];
    __shared__ float Ts[NB][NB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    if (tid < NB * NB) Ts[tid >> 4][tid & 15] = T[tid];

    float* Cl = Cs + c * 16 + 4 * g;                         // this lane's column, its first row of tile 0
    const float* Vtl = Vt + c * 16 + 4 * g;                  // reflector c, same rows
    const float* Vrl = Vr + (int64_t)c * NB + 4 * g;         // row c of a block, reflectors 4 g ..
    // Blocks past the end are clamped to the last one for every load (a valid address, no branch) and
    // take no part: their strip registers are zero and they are not stored.  All loads of a phase are
    // issued ahead of the MFMAs that use them, in groups of GRP blocks, double-buffered: a load
    // consumed right behind its issue would expose one memory latency per block.
    constexpr int GRP = 5, NG = NBLK / GRP;
    static_assert(NBLK % GRP == 0, "blocks per wave must be a multiple of the load group");
    const int last = nblocks - 1;
    f32x4_t cr[NBLK];
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
        const int blk = wave + 8 * b;
        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(Cl + 256 * (blk < nblocks ? blk : last));
        const bool valid = blk < nblocks;
        cr[b] = f32x4_t{valid ? v[0] : 0.f, valid ? v[1] : 0.f, valid ? v[2] : 0.f, valid ? v[3] : 0.f};
    }
    // W_partial[i][col] = sum over this wave's rows of V[r][i] C[r][col]; MFMA (b, v) contracts the four
    // rows 16 blk + 4 kk + v (kk = lane / 16): A = V[row][lane % 16], B = the strip register itself
    f32x4_t w0 = {0.f, 0.f, 0.f, 0.f}, w1 = {0.f, 0.f, 0.f, 0.f};
    f32x4_t va[2][GRP];
    auto load_vt = [&](int grp) {
#pragma unroll
        for (int q = 0; q < GRP; ++q) {
            const int blk = wave + 8 * (grp * GRP + q);
            va[grp & 1][q] = *reinterpret_cast<const f32x4_t*>(Vtl + 256 * (blk < nblocks ? blk : last));
        }
    };
    load_vt(0);
#pragma unroll
    for (int grp = 0; grp < NG; ++grp) {
        if (grp + 1 < NG) load_vt(grp + 1);
#pragma unroll
        for (int q = 0; q < GRP; ++q) {
            const int b = grp * GRP + q;
            const f32x4_t a = va[grp & 1][q];
            w0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], cr[b][0], w0, 0, 0, 0);
            w1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], cr[b][1], w1, 0, 0, 0);
            w0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], cr[b][2], w0, 0, 0, 0);
            w1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], cr[b][3], w1, 0, 0, 0);
        }
    }
    // the reflector rows of the second product do not depend on W: fetch the first group before the barriers
    auto load_vr = [&](int grp) {
#pragma unroll
        for (int q = 0; q < GRP; ++q) {
            const int blk = wave + 8 * (grp * GRP + q);
            va[grp & 1][q] = *reinterpret_cast<const f32x4_t*>(Vrl + (int64_t)(16 * (blk < nblocks ? blk : last)) * NB);
        }
    };
    load_vr(0);
#pragma unroll
    for (int v = 0; v < 4; ++v) Wp[wave][4 * g + v][c] = w0[v] + w1[v];      // accumulator row 4 g + v, column c
    __syncthreads();
    if (tid < NB * NB) {
        const int i = tid >> 4, cc = tid & 15;
        float sum = Wp[0][i][cc];
#pragma unroll
        for (int w = 1; w < 8; ++w) sum += Wp[w][i][cc];
        Ws[i][cc] = sum;
    }
    __syncthreads();
    if (tid < NB * NB) {
        const int i = tid >> 4, cc = tid & 15;
        float o = 0.f;
#pragma unroll
        for (int k = 0; k < NB; ++k) o = fmaf(t_transposed ? Ts[k][i] : Ts[i][k], Ws[k][cc], o);
        Wn[i][cc] = -o;
    }
    __syncthreads();
    // C_block += V_block W': MFMA q contracts reflectors 4 kk + q; A = V[16 blk + lane % 16][4 kk + q]
    float bq[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) bq[q] = Wn[4 * g + q][c];
#pragma unroll
    for (int grp = 0; grp < NG; ++grp) {
        if (grp + 1 < NG) load_vr(grp + 1);
#pragma unroll
        for (int q = 0; q < GRP; ++q) {
            const int b = grp * GRP + q;
            const int blk = wave + 8 * b;
            const f32x4_t a4 = va[grp & 1][q];
            cr[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[0], bq[0], cr[b], 0, 0, 0);
            cr[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[1], bq[1], cr[b], 0, 0, 0);
            cr[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[2], bq[2], cr[b], 0, 0, 0);
            cr[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[3], bq[3], cr[b], 0, 0, 0);
            if (blk < nblocks) *reinterpret_cast<f32x4_t*>(Cl + 256 * blk) = cr[b];
        }
    }
}

template <int NBLK>
__global__ __launch_bounds__(512)
void reflect_strip_kernel(const float* __restrict__ Vr, const float* __restrict__ Vt, const float* __restrict__ T,
                          int t_transposed, float* C, int64_t strip_stride, int nblocks) {
    reflect_strip_body<NBLK>(Vr, Vt, T, t_transposed, C + (int64_t)blockIdx.x * strip_stride, nblocks);
}

// One launch per QR step p.  The chain of panel factorisations (one workgroup each) is the
// critical path, so the launch that applies block reflector p also factorises panel p + 1:
//   workgroup 0        updates the 16 columns of panel p + 1, then factorises them;
//   the next `wide`    update the remaining trailing columns of the matrix;
//   the last `acc`     update all columns of the accumulated transposed orthogonal factor
//                      X <- (I - V T^T V^T) X  (X starts as the identity, ends as Q^T).
// Every strip reads only V_p, T_p and its own columns; panel p + 1 writes its own columns, the
// other pair of reflector buffers and its own T, so the workgroups of one launch never touch the
// same data.  Waves of workgroup 0 that the panel does not use leave after the strip.
struct QrStepArgs {
    const float* Vr; const float* Vt;    // reflector block p in both layouts (see reflect_strip_body)
    const float* T;                      // its 16 x 16 triangle
    float* C;                            // tile (row block of c0, column block of c0 + 16) of the matrix: panel p + 1 first
    float* X;                            // tile (row block of c0, column block 0) of the accumulator
    int64_t strip_stride;                // floats between the tiles of neighbouring column blocks
    int nblocks;                         // rows / 16 of step p
    int wide, acc;                       // strip counts
    float* Vr_next; float* Vt_next; float* Tnext; float* rdiag_next;   // outputs of panel p + 1
    int m_next;                          // its row count (0: no further panel)
};

template <int NTHR, int R, int NBLK>
__global__ __launch_bounds__(512)
void qr_step_kernel(QrStepArgs a) {
    const int b = blockIdx.x;
    float* Cs = b <= a.wide ? a.C + (int64_t)b * a.strip_stride : a.X + (int64_t)(b - 1 - a.wide) * a.strip_stride;
    reflect_strip_body<NBLK>(a.Vr, a.Vt, a.T, 1, Cs, a.nblocks);
    if (b != 0 || a.m_next <= 0) return;
    __threadfence_block();
    __syncthreads();                     // the strip's stores are visible to the whole workgroup
    if (threadIdx.x >= NTHR) return;
    qr_panel_body<NTHR, R>(a.C + 256, a.Vr_next, a.Vt_next, a.Tnext, a.rdiag_next, a.m_next);   // one tile (16 rows) further down
}

// zeroes what lies beyond n x n of the tiled matrix M (n_pad x n_pad) and sets the tiled X to the identity
__global__ __launch_bounds__(256)
void qr_prepare_kernel(float* M, float* X, int n, int n_pad) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;          // index into the tiled arrays
    if (i >= (int64_t)n_pad * n_pad) return;
    const int nbr = n_pad >> 4;
    const int tile = (int)(i >> 8), in = (int)(i & 255);
    const int r = (tile % nbr) * 16 + (in & 15), c = (tile / nbr) * 16 + (in >> 4);
    if (r >= n || c >= n) M[i] = 0.f;
    X[i] = r == c ? 1.f : 0.f;
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

    // rolled loop with the columns rotated by one per step (current column = slot 0), as in the QR panel
#pragma unroll 1
    for (int j = 0; j < NB; ++j) {
        // pivot search over rows >= j: largest |value|, smallest row on ties
        float bv = -1.f;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = tid + i * NTHR;
            if (r >= j && r < m) {
                const float a = fabsf(P[i][0]);
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
        const float pivot = prow[0];
        const int live = NB - j;
        if (pivot != 0.f) {
            const float inv = 1.0f / pivot;
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int r = tid + i * NTHR;
                if (r > j && r < m) {
                    const float l = P[i][0] * inv;
                    P[i][0] = l;
#pragma unroll
                    for (int c = 1; c < NB; ++c) if (c < live) P[i][c] = fmaf(-l, prow[c], P[i][c]);
                }
            }
        } else if (tid == 0) {
            *flag = 1;
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const float first = P[i][0];
#pragma unroll
            for (int c = 0; c < NB - 1; ++c) P[i][c] = P[i][c + 1];
            P[i][NB - 1] = first;
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
hipError_t launch_qr_panel(int rows_per_thread, float* Mp, float* Vr, float* Vt, float* Tg, float* rdiag, int m,
                           hipStream_t s) {
    switch (rows_per_thread) {
#define GELO_CASE(RR) case RR: hipLaunchKernelGGL((qr_panel_kernel<NTHR, RR>), dim3(1), dim3(NTHR), 0, s, Mp, Vr, Vt, Tg, rdiag, m); break;
        GELO_CASE(1) GELO_CASE(2) GELO_CASE(3) GELO_CASE(4) GELO_CASE(5)
        GELO_CASE(6) GELO_CASE(7) GELO_CASE(8) GELO_CASE(9) GELO_CASE(10)
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
                       dim3(SK_THREADS), 0, s, L, ldl, W, ldw, C, ldc, rows, cols);
    return hipGetLastError();
}

// W (16 x cols, row stride ws.ld) = op(T) V^T C over `rows` rows; op(T) = T^T if t_transposed
hipError_t vt_c(const FactorWorkspace& ws, const float* V, const float* T, int t_transposed, const float* C,
                int64_t ldc, int rows, int cols, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const int chunks = (rows + SK_ROWS - 1) / SK_ROWS;
    if (chunks > ws.wpart_chunks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(vt_c_partial_kernel, dim3((cols + SK_COLS - 1) / SK_COLS, chunks), dim3(SK_THREADS), 0, s,
                       V, ws.ld, C, ldc, rows, cols, ws.Wpart, ws.ld);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_apply_kernel, dim3((cols + SK_COLS - 1) / SK_COLS), dim3(SK_THREADS), 0, s,
                       ws.Wpart, chunks, cols, ws.ld, T, t_transposed, ws.W);
    return hipGetLastError();
}

// C (rows x cols, rows and cols multiples of 16) <- (I - V op(T) V^T) C with op(T) = T^T if t_transposed
// C (tiled, rows x cols, both multiples of 16; C points at the first tile, strip_stride floats between column blocks)
// <- (I - V op(T) V^T) C
hipError_t apply_block_reflector(const float* Vr, const float* Vt, const float* T, int t_transposed,
                                 float* C, int64_t strip_stride, int rows, int cols, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    if (rows % NB != 0 || cols % NB != 0) return hipErrorInvalidValue;
    const int nblocks = rows / NB;
    const dim3 grid(cols / NB), block(512);
    const int per_wave = (nblocks + 7) / 8;
    if (per_wave <= 5) hipLaunchKernelGGL(reflect_strip_kernel<5>, grid, block, 0, s, Vr, Vt, T, t_transposed, C, strip_stride, nblocks);
    else if (per_wave <= 10) hipLaunchKernelGGL(reflect_strip_kernel<10>, grid, block, 0, s, Vr, Vt, T, t_transposed, C, strip_stride, nblocks);
    else if (per_wave <= 20) hipLaunchKernelGGL(reflect_strip_kernel<20>, grid, block, 0, s, Vr, Vt, T, t_transposed, C, strip_stride, nblocks);
    else if (per_wave <= 40) hipLaunchKernelGGL(reflect_strip_kernel<40>, grid, block, 0, s, Vr, Vt, T, t_transposed, C, strip_stride, nblocks);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

#define GELO_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

}  // namespace

size_t factor_workspace_bytes(int n) {
    const int64_t n_pad = round_up(n, NB), ld = round_up(n, 64);
    const int64_t chunks = (n_pad + SK_ROWS - 1) / SK_ROWS;
    int64_t floats = 3 * n_pad * ld + n_pad * NB + chunks * NB * ld + NB * ld + n_pad + 4 * ld + 64;
    return (size_t)floats * sizeof(float) + (size_t)(n_pad + ld + 128) * sizeof(int) + 8192;
}

void factor_workspace_carve(void* base, int n, FactorWorkspace* ws) {
    const int64_t n_pad = round_up(n, NB), ld = round_up(n, 64);
    const int64_t chunks = (n_pad + SK_ROWS - 1) / SK_ROWS;
    float* p = (float*)base;
    auto take = [&](int64_t count) { float* q = p; p += round_up(count, 64); return q; };
    ws->M = take(n_pad * ld);
    ws->X = take(n_pad * ld);
    ws->Vc = take(n_pad * ld);
    ws->Tmat = take(n_pad * NB);
    ws->Wpart = take(chunks * NB * ld);
    ws->W = take(NB * ld);
    ws->rdiag = take(n_pad);
    ws->vec = take(4 * ld);
    ws->scalars = take(16);
    ws->piv = (int*)take(n_pad);
    ws->flag = (int*)take(16);
    ws->counters = (int*)take(ld / SK_COLS + 1);
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

namespace {

template <int NTHR, int R, int NBLK>
hipError_t launch_qr_step_t(const QrStepArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((qr_step_kernel<NTHR, R, NBLK>), dim3(1 + a.wide + a.acc), dim3(512), 0, s, a);
    return hipGetLastError();
}

// Can a panel with R rows per thread (NTHR threads) meet strips with NBLK blocks per wave (PREV: the
// next smaller strip variant)?  The next panel has 16 (nblocks - 1) rows, so only a few pairs occur.
constexpr bool qr_step_pair_occurs(int NTHR, int R, int NBLK, int PREV) {
    const int min_nb = (R - 1) * NTHR / NB + 2, max_nb = R * NTHR / NB + 1;
    return (min_nb + 7) / 8 <= NBLK && (max_nb + 7) / 8 > PREV;
}

template <int NTHR, int R>
hipError_t launch_qr_step_r(int per_wave, const QrStepArgs& a, hipStream_t s) {
    if (per_wave <= 5) { if constexpr (qr_step_pair_occurs(NTHR, R, 5, 0)) return launch_qr_step_t<NTHR, R, 5>(a, s); }
    else if (per_wave <= 10) { if constexpr (qr_step_pair_occurs(NTHR, R, 10, 5)) return launch_qr_step_t<NTHR, R, 10>(a, s); }
    else if (per_wave <= 20) { if constexpr (qr_step_pair_occurs(NTHR, R, 20, 10)) return launch_qr_step_t<NTHR, R, 20>(a, s); }
    else if (per_wave <= 40) { if constexpr (qr_step_pair_occurs(NTHR, R, 40, 20)) return launch_qr_step_t<NTHR, R, 40>(a, s); }
    return hipErrorInvalidValue;
}

hipError_t launch_qr_step(const QrStepArgs& a, hipStream_t s) {
    const int per_wave = (a.nblocks + 7) / 8;
    const int m = a.m_next;
    if (m <= 1024) {
        switch ((m + 255) / 256) {
            case 0: case 1: return launch_qr_step_r<256, 1>(per_wave, a, s);
            case 2: return launch_qr_step_r<256, 2>(per_wave, a, s);
            case 3: return launch_qr_step_r<256, 3>(per_wave, a, s);
            default: return launch_qr_step_r<256, 4>(per_wave, a, s);
        }
    }
    switch ((m + 511) / 512) {
        case 3: return launch_qr_step_r<512, 3>(per_wave, a, s);
        case 4: return launch_qr_step_r<512, 4>(per_wave, a, s);
        case 5: return launch_qr_step_r<512, 5>(per_wave, a, s);
        case 6: return launch_qr_step_r<512, 6>(per_wave, a, s);
        case 7: return launch_qr_step_r<512, 7>(per_wave, a, s);
        case 8: return launch_qr_step_r<512, 8>(per_wave, a, s);
        case 9: return launch_qr_step_r<512, 9>(per_wave, a, s);
        case 10: return launch_qr_step_r<512, 10>(per_wave, a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t householder_qr(const FactorWorkspace& ws, int n, hipStream_t s) {
    const int n_pad = ws.n_pad;
    const int nbr = n_pad / NB;                               // tile rows (= tile columns)
    const int64_t strip_stride = (int64_t)nbr * 256;
    const int panels = nbr;
    // block reflector p is only needed while step p runs: two compact pairs of buffers alternate
    float* Vr[2] = {ws.Vc, ws.Vc + (int64_t)n_pad * NB};
    float* Vt[2] = {ws.Vc + 2 * (int64_t)n_pad * NB, ws.Vc + 3 * (int64_t)n_pad * NB};
    {
        const int64_t elems = (int64_t)n_pad * n_pad;
        hipLaunchKernelGGL(qr_prepare_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, s, ws.M, ws.X, n, n_pad);
        GELO_TRY(hipGetLastError());
    }
    // panel 0 on its own; then one launch per step: trailing update + accumulation of Q^T with block
    // reflector p, and in the same launch the factorisation of panel p + 1
    {
        const int m = n_pad;
        if (m <= 1024) GELO_TRY(launch_qr_panel<256>((m + 255) / 256, ws.M, Vr[0], Vt[0], ws.Tmat, ws.rdiag, m, s));
        else GELO_TRY(launch_qr_panel<512>((m + 511) / 512, ws.M, Vr[0], Vt[0], ws.Tmat, ws.rdiag, m, s));
    }
    for (int p = 0; p < panels; ++p) {
        const int c0 = p * NB, m = n_pad - c0;
        const int cols = n_pad - c0 - NB;
        QrStepArgs a;
        a.Vr = Vr[p & 1]; a.Vt = Vt[p & 1]; a.T = ws.Tmat + (int64_t)p * NB * NB;
        a.X = ws.X + (int64_t)p * 256;                        // tile (p, 0)
        a.strip_stride = strip_stride; a.nblocks = m / NB; a.acc = nbr;
        if (cols <= 0) {                      // last block reflector: only the accumulator is left
            GELO_TRY(apply_block_reflector(a.Vr, a.Vt, a.T, 1, a.X, strip_stride, m, n_pad, s));
            break;
        }
        a.C = ws.M + (int64_t)(p + 1) * strip_stride + (int64_t)p * 256;      // tile (p, p + 1)
        a.wide = cols / NB - 1;
        a.Vr_next = Vr[(p + 1) & 1]; a.Vt_next = Vt[(p + 1) & 1];
        a.Tnext = ws.Tmat + (int64_t)(p + 1) * NB * NB; a.rdiag_next = ws.rdiag + c0 + NB;
        a.m_next = m - NB;
        GELO_TRY(launch_qr_step(a, s));
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
    GELO_TRY(emit_matrix(A, lda, 0, nullptr, n, ld, nullptr, nullptr, ws.M, nullptr, s));
    GELO_TRY(emit_matrix(Ainv, lda, 0, nullptr, n, ld, nullptr, nullptr, ws.X, nullptr, s));
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
