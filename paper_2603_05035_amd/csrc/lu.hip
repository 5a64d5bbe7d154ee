// Row-pivoted blocked LU, the explicit inverse and the kappa_2 estimate (Lanczos) behind the non-orthogonal
// mixing matrices (Section 3.2.1, Mitigation 1: a well-conditioned non-orthogonal A, generated and
// verified; Section 3.2 eq. 3 needs A^-1 explicitly so that un-mixing is one GEMM).
// Everything is float and deterministic: reductions run in a fixed order, no atomics.
//
// Two block levels.  Column panels are 16 wide and factorised by ONE workgroup that keeps its rows
// in registers; eight panels make an outer block of 128 columns.  Inside a block each launch applies
// panel i to the block's remaining columns (16-column chunks, matrix cores) and, in workgroup 0,
// factorises panel i + 1 right behind the update of its own chunk, so the chain of panels is the
// critical path and nothing else.  The row interchanges of a panel never run one after another
// through memory: the panel writes them as ONE gather list (at most 32 rows change place), which
// the next launch applies to all other columns in one round trip.  After a block, its two diagonal
// triangles are inverted (one workgroup each); U12 = L11^-1 U12 and the trailing update are float
// GEMMs with K = 128.  The inverse then is two block substitutions (GEMMs again, the right-hand
// side of the forward one kept triangular) and one column permutation.
#include "gelo_internal.h"

namespace gelo {
namespace {

constexpr int NB = kPanel;
constexpr int BW = kLuBlock;
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ------------------------------------------------------------------ LU panel --
// Row-pivoted LU of the m x 16 panel at Mp (row stride ld), in place: unit-lower multipliers below
// the diagonal, U on and above it.  Thread t keeps rows t, t + NTHR, ... in registers.
// Rows do not move while the panel is factorised: a pivot row is only marked as used, and the
// positions that LAPACK's sequence of interchanges (row j <-> pivot of step j) would give every row
// are worked out once at the end, when the rows are written back to those positions.  The same
// bookkeeping gives the gather list for the rest of the matrix: gat[e] = destination row,
// gat[32 + e] = source row (both global, -1 = unused entry), new row dst = old row src.
// perm (global row indices) follows the same gather.  Pivot = largest |value|, smallest row on ties;
// a zero (or NaN-only) pivot column sets *flag and is left unscaled.
// Two barriers per column: one for the pivot search, one for the broadcast of the pivot row.
template <int NTHR, int R>
__device__ __forceinline__ void lu_panel_body(float* Mp, int64_t ld, int m, int row_offset, int* gat, int* perm,
                                              int* flag) {
    constexpr int NW = NTHR / 64;
    __shared__ unsigned long long keys[NW];
    __shared__ __attribute__((aligned(16))) float prow[NB];
    __shared__ int qlist[NB];
    __shared__ int gd[32], gs[32];
    __shared__ int pos_of[kMaxN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float P[R][NB];
    unsigned used = 0;                       // bit i: register row i is absent or already a pivot row
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
            used |= 1u << i;
        }
    }

    static_for<NB>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        // largest |value| among the rows not used yet; key = (|value| bits, ~row): one 64-bit maximum
        float bv = -1.f;
        int bi = 0;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const float a = fabsf(P[i][j]);
            const bool take = !((used >> i) & 1u) && a > bv;
            bv = take ? a : bv;
            bi = take ? i : bi;
        }
        unsigned long long key = bv < 0.f ? 0ull
            : (((unsigned long long)__float_as_uint(bv) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)(tid + bi * NTHR)));
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long o = __shfl_xor(key, off, 64);
            key = o > key ? o : key;
        }
        if (lane == 0) keys[wave] = key;
        __syncthreads();
        unsigned long long best = keys[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) { const unsigned long long o = keys[w]; best = o > best ? o : best; }
        const bool none = best == 0ull;
        const int q = none ? 0 : (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));     // the pivot row
        const int q_slot = q / NTHR, q_tid = q % NTHR;
        if (tid == q_tid) {
            // the pivot row's columns j..15 (all the update reads) go to LDS.  The empty asm hides that the
            // stored values are loads of P: the compiler would otherwise merge the R stores into one whose
            // address is picked at run time, and an array indexed that way stays in scratch memory.
            static_for<R>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                if (i == q_slot) {
#pragma unroll
                    for (int c = j; c < NB; ++c) {
                        float v = P[i][c];
                        asm volatile("" : "+v"(v));
                        prow[c] = v;
                    }
                }
            });
            used |= 1u << q_slot;
        }
        if (tid == 0) qlist[j] = q;
        __syncthreads();
        float pr[NB];
#pragma unroll
        for (int c = j; c < NB; ++c) pr[c] = prow[c];
        const float pivot = pr[j];
        const bool nz = !none && pivot != 0.f;
        float inv = __builtin_amdgcn_rcpf(pivot);
        inv = fmaf(fmaf(-pivot, inv, 1.0f), inv, inv);        // one Newton step: the reciprocal to the last bit or so
        inv = nz ? inv : 0.f;
        if (!nz && tid == 0) *flag = 1;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const bool live = !((used >> i) & 1u);
            const float l = live ? P[i][j] * inv : 0.f;
            P[i][j] = live ? l : P[i][j];
#pragma unroll
            for (int c = j + 1; c < NB; ++c) P[i][c] = fmaf(-l, pr[c], P[i][c]);
        }
    });

    // where LAPACK's interchanges put every row
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r < m) pos_of[r] = r;
    }
    if (tid < 32) { gd[tid] = -1; gs[tid] = -1; }
    __syncthreads();
    if (wave == 0) {
        // The 16 interchanges replayed by one wave, all state in registers: lane t < 16 carries top = the row
        // now at position t; rows that left the top 16 (always rows that started there) sit at far positions,
        // one (fpos, frow) pair per lane f < nf; every other row is still where it started.
        int top = lane, fpos = -1, frow = -1, nf = 0;
        const int qv = qlist[lane & 15];
        static_for<NB>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int q = __builtin_amdgcn_readlane(qv, j);
            const unsigned long long mt = __ballot(lane >= j && lane < NB && top == q);
            const unsigned long long mf = __ballot(lane < nf && frow == q);
            int pq = q;                                    // position of the pivot row before this interchange
            if (mt) pq = __ffsll(mt) - 1;
            else if (mf) pq = __shfl(fpos, __ffsll(mf) - 1, 64);
            const int w = __builtin_amdgcn_readlane(top, j);
            if (lane == j) top = q;
            if (pq < NB) {
                if (lane == pq && pq != j) top = w;
            } else {
                const unsigned long long mp = __ballot(lane < nf && fpos == pq);
                const int f = mp ? __ffsll(mp) - 1 : nf;
                nf += mp ? 0 : 1;
                if (lane == f) { fpos = pq; frow = w; }
            }
        });
        if (lane < NB) { pos_of[top] = lane; gd[lane] = row_offset + lane; gs[lane] = row_offset + top; }
        if (lane < nf) { pos_of[frow] = fpos; gd[NB + lane] = row_offset + fpos; gs[NB + lane] = row_offset + frow; }
    }
    __syncthreads();
    int pv = 0;
    if (tid < 32) {
        gat[tid] = gd[tid]; gat[32 + tid] = gs[tid];
        if (gs[tid] >= 0) pv = perm[gs[tid]];
    }
    __syncthreads();
    if (tid < 32 && gd[tid] >= 0) perm[gd[tid]] = pv;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int r = tid + i * NTHR;
        if (r >= m) continue;
        float* mp = Mp + (int64_t)pos_of[r] * ld;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4)
            *reinterpret_cast<float4*>(mp + c4 * 4) = make_float4(P[i][c4 * 4], P[i][c4 * 4 + 1], P[i][c4 * 4 + 2], P[i][c4 * 4 + 3]);
    }
}

template <int NTHR, int R>
__global__ __launch_bounds__(NTHR)
void lu_panel_kernel(float* Mp, int64_t ld, int m, int row_offset, int* gat, int* perm, int* flag) {
    lu_panel_body<NTHR, R>(Mp, ld, m, row_offset, gat, perm, flag);
}

// ------------------------------------------------------ one panel on one chunk --
// Applies the panel at (pc, pc) (already factorised, its interchanges in gat) to the 16 columns
// from col0 on: the interchanges, U_chunk = L11^-1 * top block, then C -= L21 * U_chunk over all
// rows below (v_mfma_f32_16x16x4_f32, one 16 x 16 block of rows per MFMA group).  512 threads.
// The MFMA sums over k in the order 4 g + e (g = lane / 16, e = the MFMA's number): then a lane's
// A values are the 16 bytes L[row][4 g .. 4 g + 3].
__device__ __forceinline__ void lu_chunk_body(float* M, int64_t ld, const int* gat, int pc, int col0, int n_pad) {
    __shared__ float L11[NB][NB + 1];
    __shared__ float Us[NB][NB];
    __shared__ int cg[64];
    const int tid = threadIdx.x;
    if (tid < 64) cg[tid] = gat[tid];
    __syncthreads();
    {
        const int e = tid >> 4, c = tid & 15;             // 32 entries x 16 columns
        const int src = cg[32 + e], dst = cg[e];
        float v = 0.f;
        if (src >= 0) v = M[(int64_t)src * ld + col0 + c];
        __syncthreads();                                  // every row is read before any is overwritten
        if (dst >= 0) M[(int64_t)dst * ld + col0 + c] = v;
    }
    __threadfence_block();
    __syncthreads();
    if (tid < NB * NB) L11[tid >> 4][tid & 15] = M[(int64_t)(pc + (tid >> 4)) * ld + pc + (tid & 15)];
    float x[NB];
    if (tid < NB) {
#pragma unroll
        for (int i = 0; i < NB; ++i) x[i] = M[(int64_t)(pc + i) * ld + col0 + tid];
    }
    __syncthreads();
    if (tid < NB) {
#pragma unroll
        for (int i = 1; i < NB; ++i)
#pragma unroll
            for (int k = 0; k < i; ++k) x[i] = fmaf(-L11[i][k], x[k], x[i]);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            Us[i][tid] = x[i];
            M[(int64_t)(pc + i) * ld + col0 + tid] = x[i];
        }
    }
    __syncthreads();
    const int lane = tid & 63, wave = tid >> 6;
    const int cc = lane & 15, g = lane >> 4;
    float bq[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) bq[e] = -Us[4 * g + e][cc];
    const int nblk = (n_pad - pc) / NB - 1;
    constexpr int UN = 4;                                 // blocks in flight per wave
    for (int b0 = wave; b0 < nblk; b0 += 8 * UN) {
        f32x4_t a4[UN], acc[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int b = b0 + 8 * u;
            const int rb = pc + NB + NB * (b < nblk ? b : nblk - 1);      // clamped: a valid address, no branch
            a4[u] = *reinterpret_cast<const f32x4_t*>(M + (int64_t)(rb + cc) * ld + pc + 4 * g);
            const float* cp = M + (int64_t)(rb + 4 * g) * ld + col0 + cc;
            acc[u] = f32x4_t{cp[0], cp[ld], cp[2 * ld], cp[3 * ld]};
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int b = b0 + 8 * u;
            acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[u][0], bq[0], acc[u], 0, 0, 0);
            acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[u][1], bq[1], acc[u], 0, 0, 0);
            acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[u][2], bq[2], acc[u], 0, 0, 0);
            acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[u][3], bq[3], acc[u], 0, 0, 0);
            if (b < nblk) {
                float* cp = M + (int64_t)(pc + NB + NB * b + 4 * g) * ld + col0 + cc;
                cp[0] = acc[u][0]; cp[ld] = acc[u][1]; cp[2 * ld] = acc[u][2]; cp[3 * ld] = acc[u][3];
            }
        }
    }
}

// The interchanges of one panel on a window of 128 columns; columns in [excl_lo, excl_hi) are
// somebody else's.  512 threads: 4 groups of 8 list entries x 128 columns.
__device__ __forceinline__ void lu_gather_body(float* M, int64_t ld, const int* gat, int window, int n_pad,
                                               int excl_lo, int excl_hi) {
    __shared__ int cg[64];
    const int tid = threadIdx.x;
    if (tid < 64) cg[tid] = gat[tid];
    __syncthreads();
    const int col = window * 128 + (tid & 127), eg = tid >> 7;
    const bool on = col < n_pad && !(col >= excl_lo && col < excl_hi);
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int src = cg[32 + eg * 8 + k];
        v[k] = (on && src >= 0) ? M[(int64_t)src * ld + col] : 0.f;
    }
    __syncthreads();                                      // every row is read before any is overwritten
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int dst = cg[eg * 8 + k];
        if (on && dst >= 0) M[(int64_t)dst * ld + col] = v[k];
    }
}

// One launch per panel inside an outer block (not its first panel):
//   workgroup 0             applies the previous panel (at pc) to the next 16 columns, then factorises them;
//   workgroups < nchunks    apply it to the other 16-column chunks of the block;
//   the rest                apply its interchanges to every column outside [pc, block_end).
// No two workgroups touch the same columns.
struct LuStepArgs {
    float* M; int64_t ld; int n_pad;
    int pc;                   // first row / column of the previous panel
    int block_end;            // first column behind the outer block
    int nchunks;              // (block_end - pc - 16) / 16 >= 1
    const int* gat_prev;      // interchanges of the previous panel
    int* gat_next;            // written by the panel factorised here
    int* perm; int* flag;
};

template <int NTHR, int R>
__global__ __launch_bounds__(512)
void lu_step_kernel(LuStepArgs a) {
    const int b = blockIdx.x;
    if (b >= a.nchunks) {
        lu_gather_body(a.M, a.ld, a.gat_prev, b - a.nchunks, a.n_pad, a.pc, a.block_end);
        return;
    }
    lu_chunk_body(a.M, a.ld, a.gat_prev, a.pc, a.pc + NB * (1 + b), a.n_pad);
    if (b != 0) return;
    __threadfence_block();
    __syncthreads();                     // the chunk's stores are visible to the whole workgroup
    if (threadIdx.x >= NTHR) return;
    const int pn = a.pc + NB;
    lu_panel_body<NTHR, R>(a.M + (int64_t)pn * a.ld + pn, a.ld, a.n_pad - pn, pn, a.gat_next, a.perm, a.flag);
}

// -------------------------------------------------------- triangle inverses --
// X = T^-1 for a w x w triangle (w <= 128, row stride ldt); thread j computes column j by block
// substitution with 16 x 16 blocks: the triangle sits in LDS (row i contiguous, read 16 bytes at a
// time, all lanes the same address), the 16 entries of the current block row in registers, the
// finished part of the column in LDS (Xl, read and written by its own thread only).
// UPPER = false: unit lower triangle; true: upper with its diagonal.  Beyond w the triangle is taken
// as the identity.  Out: row-major, pitch BW.  128 threads.
template <bool UPPER>
__device__ __forceinline__ void tri_inverse_body(const float* T, int64_t ldt, int w, float* out, float* Ts, float* Xl) {
    const int tid = threadIdx.x;
#pragma unroll 1
    for (int i0 = 0; i0 < BW; i0 += NB) {                  // 16 rows of loads in flight
        float v[NB];
#pragma unroll
        for (int ii = 0; ii < NB; ++ii) {
            const int i = i0 + ii;
            v[ii] = (i < w && tid < w) ? T[(int64_t)i * ldt + tid] : 0.f;
        }
#pragma unroll
        for (int ii = 0; ii < NB; ++ii) {
            const int i = i0 + ii;
            const bool keep = i < w && tid < w && (UPPER ? tid >= i : tid < i);
            Ts[i * BW + tid] = keep ? v[ii] : (i == tid ? 1.f : 0.f);
        }
    }
    __syncthreads();
    constexpr int NBLK = BW / NB;
#pragma unroll 1
    for (int s = 0; s < NBLK; ++s) {
        const int ib = UPPER ? NBLK - 1 - s : s;
        const float* Trow = Ts + ib * NB * BW;            // the 16 rows of this block row
        float acc[NB];
#pragma unroll
        for (int ii = 0; ii < NB; ++ii) acc[ii] = ib * NB + ii == tid ? 1.f : 0.f;
#pragma unroll 1
        for (int t = 0; t < s; ++t) {                      // the block rows solved so far
            const int kb = UPPER ? NBLK - 1 - t : t;
            float xk[NB];
#pragma unroll
            for (int kk = 0; kk < NB; ++kk) xk[kk] = Xl[(kb * NB + kk) * BW + tid];
#pragma unroll
            for (int ii = 0; ii < NB; ++ii)
#pragma unroll
                for (int k4 = 0; k4 < NB / 4; ++k4) {
                    const float4 tv = *reinterpret_cast<const float4*>(Trow + ii * BW + kb * NB + k4 * 4);
                    acc[ii] = fmaf(-tv.x, xk[k4 * 4 + 0], acc[ii]);
                    acc[ii] = fmaf(-tv.y, xk[k4 * 4 + 1], acc[ii]);
                    acc[ii] = fmaf(-tv.z, xk[k4 * 4 + 2], acc[ii]);
                    acc[ii] = fmaf(-tv.w, xk[k4 * 4 + 3], acc[ii]);
                }
        }
        const float* Td = Trow + ib * NB;                  // the diagonal block
        if (!UPPER) {
#pragma unroll
            for (int ii = 1; ii < NB; ++ii)
#pragma unroll
                for (int kk = 0; kk < ii; ++kk) acc[ii] = fmaf(-Td[ii * BW + kk], acc[kk], acc[ii]);
        } else {
#pragma unroll
            for (int ii = NB - 1; ii >= 0; --ii) {
#pragma unroll
                for (int kk = ii + 1; kk < NB; ++kk) acc[ii] = fmaf(-Td[ii * BW + kk], acc[kk], acc[ii]);
                acc[ii] /= Td[ii * BW + ii];
            }
        }
#pragma unroll
        for (int ii = 0; ii < NB; ++ii) {
            const int i = ib * NB + ii;
            Xl[i * BW + tid] = acc[ii];
            if (i < w && tid < w) out[i * BW + tid] = acc[ii];
        }
    }
}

// After the last panel of an outer block (first column c0, width w): workgroup 0 inverts L11,
// workgroup 1 inverts U11 (128 threads each), the others apply the last panel's interchanges to
// every column outside the block.  The block's own columns left of that panel belong to L11, so
// workgroup 0 moves those rows itself before it reads the triangle.
__global__ __launch_bounds__(512)
void lu_block_finish_kernel(float* M, int64_t ld, int n_pad, int c0, int w, const int* gat, float* Linv, float* Uinv) {
    extern __shared__ __attribute__((aligned(16))) float Ts[];
    __shared__ int cg[64];
    const int b = blockIdx.x, tid = threadIdx.x;
    if (b >= 2) {
        lu_gather_body(M, ld, gat, b - 2, n_pad, c0, c0 + w);
        return;
    }
    if (b == 0) {
        if (tid < 64) cg[tid] = gat[tid];
        __syncthreads();
        const int width = w - NB;                          // columns [c0, c0 + width), 32 list entries each
        float v[7];
#pragma unroll
        for (int k = 0; k < 7; ++k) {
            const int id = tid + 512 * k;
            const int e = width > 0 ? id / width : 32, c = width > 0 ? id % width : 0;
            const int src = e < 32 ? cg[32 + e] : -1;
            v[k] = src >= 0 ? M[(int64_t)src * ld + c0 + c] : 0.f;
        }
        __syncthreads();                                   // every row is read before any is overwritten
#pragma unroll
        for (int k = 0; k < 7; ++k) {
            const int id = tid + 512 * k;
            const int e = width > 0 ? id / width : 32, c = width > 0 ? id % width : 0;
            const int dst = e < 32 ? cg[e] : -1;
            if (dst >= 0) M[(int64_t)dst * ld + c0 + c] = v[k];
        }
        __threadfence_block();
        __syncthreads();
    }
    if (tid >= BW) return;
    const float* T = M + (int64_t)c0 * ld + c0;
    if (b == 0) tri_inverse_body<false>(T, ld, w, Linv, Ts, Ts + BW * BW);
    else tri_inverse_body<true>(T, ld, w, Uinv, Ts, Ts + BW * BW);
}

// X[r, perm[c]] <- X[r, c]: one row per workgroup, through LDS
__global__ __launch_bounds__(256)
void permute_columns_kernel(float* X, int64_t ld, int n_pad, const int* perm) {
    __shared__ float row[kMaxN];
    float* xr = X + (int64_t)blockIdx.x * ld;
    for (int c = threadIdx.x; c < n_pad; c += 256) row[perm[c]] = xr[c];
    __syncthreads();
    for (int c = threadIdx.x; c < n_pad; c += 256) xr[c] = row[c];
}

__global__ __launch_bounds__(256)
void iota_kernel(int* p, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = i;
}

// ------------------------------------------------------------------ Lanczos --
// sigma_max of a matrix M from a few steps of the Lanczos recurrence on M^T M (no
// reorthogonalisation: the largest Ritz value converges first and never overshoots).  The two
// operators the condition number needs, A and A^-1, share every launch.
constexpr int kLanczosMax = 32;      // coefficient slots per operator

// Two matrix-vector products per launch, one wave per row: rows [0, n) give ya = Ma xa,
// rows [n, 2n) give yb = Mb xb.
__global__ __launch_bounds__(256)
void matvec_pair_kernel(const float* Ma, int64_t lda, const float* xa, float* ya,
                        const float* Mb, int64_t ldb, const float* xb, float* yb, int n) {
    int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= 2 * n) return;
    const bool second = row >= n;
    row -= second ? n : 0;
    const float* mr = second ? Mb + (int64_t)row * ldb : Ma + (int64_t)row * lda;
    const float* x = second ? xb : xa;
    float dot = 0.f;
    for (int c = lane; c < n; c += 64) dot = fmaf(mr[c], x[c], dot);
    dot = wave_sum(dot);
    if (lane == 0) (second ? yb : ya)[row] = dot;
}

// sum over the 1024 threads of a workgroup, the same value in every thread, fixed order
__device__ __forceinline__ float block_sum_1024(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();                                   // red may still be read from the previous call
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) s += red[w];
    return s;
}

constexpr int kVecPerThread = kMaxN / 1024;            // 5

// Workgroup o (0: A, 1: A^-1) owns the vectors at vec + o * 4 * ld: v, v_prev, y, w.
// step < 0: v = a fixed pseudo-random unit vector, v_prev = 0.
// step >= 0: alpha = w . v, r = w - alpha v - beta_prev v_prev, beta = |r|, v_prev = v, v = r / beta;
//            tri[o][0][step] = alpha, tri[o][1][step] = beta.
__global__ __launch_bounds__(1024)
void lanczos_vector_kernel(float* vec, int64_t ld, int n, float* tri, int step) {
    __shared__ float red[16];
    const int tid = threadIdx.x, o = blockIdx.x;
    float* v = vec + (int64_t)o * 4 * ld;
    float* vp = v + ld;
    const float* w = v + 3 * ld;
    float* tr = tri + o * 2 * kLanczosMax;
    float x[kVecPerThread], xp[kVecPerThread], r[kVecPerThread];
    if (step < 0) {
        float ss = 0.f;
#pragma unroll
        for (int k = 0; k < kVecPerThread; ++k) {
            const int i = tid + 1024 * k;
            uint32_t h = (uint32_t)i * 2654435761u + 0x9E3779B9u;   // fixed pseudo-random signs and sizes
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            x[k] = i < n ? ((h & 1u) ? 1.f : -1.f) * (0.5f + (float)((h >> 8) & 0xFFFF) * (1.0f / 65536.0f)) : 0.f;
            ss = fmaf(x[k], x[k], ss);
        }
        const float inv = rsqrtf(block_sum_1024(ss, red));
#pragma unroll
        for (int k = 0; k < kVecPerThread; ++k) {
            const int i = tid + 1024 * k;
            if (i < n) { v[i] = x[k] * inv; vp[i] = 0.f; }
        }
        return;
    }
    float dot = 0.f;
#pragma unroll
    for (int k = 0; k < kVecPerThread; ++k) {
        const int i = tid + 1024 * k;
        x[k] = i < n ? v[i] : 0.f;
        xp[k] = i < n ? vp[i] : 0.f;
        r[k] = i < n ? w[i] : 0.f;
        dot = fmaf(r[k], x[k], dot);
    }
    const float alpha = block_sum_1024(dot, red);
    const float beta_prev = step > 0 ? tr[kLanczosMax + step - 1] : 0.f;
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < kVecPerThread; ++k) {
        r[k] = fmaf(-beta_prev, xp[k], fmaf(-alpha, x[k], r[k]));
        ss = fmaf(r[k], r[k], ss);
    }
    const float beta = sqrtf(block_sum_1024(ss, red));
    const float inv = beta > 0.f ? 1.0f / beta : 0.f;
#pragma unroll
    for (int k = 0; k < kVecPerThread; ++k) {
        const int i = tid + 1024 * k;
        if (i < n) { vp[i] = x[k]; v[i] = r[k] * inv; }
    }
    if (tid == 0) { tr[step] = alpha; tr[kLanczosMax + step] = beta; }
}

// Largest eigenvalue of the symmetric tridiagonal matrix (alpha[0..k), beta[0..k-1)) by bisection on
// the Sturm count; out[0] = sqrt(lambda_A lambda_Ainv) = the kappa_2 estimate, out[1], out[2] its factors.
__global__ __launch_bounds__(64)
void lanczos_finish_kernel(const float* tri, int k, float* out) {
    __shared__ float sig[2];
    const int o = threadIdx.x;
    if (o < 2) {
        const float* al = tri + o * 2 * kLanczosMax;
        const float* be = al + kLanczosMax;
        float hi = 0.f;
        for (int i = 0; i < k; ++i) {
            const float g = fabsf(al[i]) + (i > 0 ? fabsf(be[i - 1]) : 0.f) + (i + 1 < k ? fabsf(be[i]) : 0.f);
            hi = fmaxf(hi, g);
        }
        float lo = 0.f;
        for (int it = 0; it < 48; ++it) {
            const float mid = 0.5f * (lo + hi);
            int below = 0;                              // eigenvalues below mid
            float d = 1.f;
            for (int i = 0; i < k; ++i) {
                const float b2 = i > 0 ? be[i - 1] * be[i - 1] : 0.f;
                d = al[i] - mid - b2 / d;
                if (fabsf(d) < 1e-30f) d = -1e-30f;
                below += d < 0.f;
            }
            if (below == k) hi = mid; else lo = mid;
        }
        sig[o] = sqrtf(0.5f * (lo + hi));
    }
    __syncthreads();
    if (threadIdx.x == 0) { out[1] = sig[0]; out[2] = sig[1]; out[0] = sig[0] * sig[1]; }
}

#define GELO_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

// the panel at (pc, pc) with m rows, alone (first panel of an outer block)
hipError_t launch_lu_panel(float* Mp, int64_t ld, int m, int row_offset, int* gat, int* perm, int* flag, hipStream_t s) {
#define GELO_CASE(NT, RR) hipLaunchKernelGGL((lu_panel_kernel<NT, RR>), dim3(1), dim3(NT), 0, s, Mp, ld, m, row_offset, gat, perm, flag); break;
    if (m <= 1024) {
        switch ((m + 255) / 256) {
            case 0: case 1: GELO_CASE(256, 1)
            case 2: GELO_CASE(256, 2)
            case 3: GELO_CASE(256, 3)
            default: GELO_CASE(256, 4)
        }
    } else {
        switch ((m + 511) / 512) {
            case 3: GELO_CASE(512, 3)
            case 4: GELO_CASE(512, 4)
            case 5: GELO_CASE(512, 5)
            case 6: GELO_CASE(512, 6)
            case 7: GELO_CASE(512, 7)
            case 8: GELO_CASE(512, 8)
            case 9: GELO_CASE(512, 9)
            case 10: GELO_CASE(512, 10)
            default: return hipErrorInvalidValue;
        }
    }
#undef GELO_CASE
    return hipGetLastError();
}

hipError_t launch_lu_step(const LuStepArgs& a, hipStream_t s) {
    const int m = a.n_pad - a.pc - NB;                    // rows of the panel factorised in this launch
    const dim3 grid(a.nchunks + (a.n_pad + 127) / 128);
#define GELO_CASE(NT, RR) hipLaunchKernelGGL((lu_step_kernel<NT, RR>), grid, dim3(512), 0, s, a); break;
    if (m <= 1024) {
        switch ((m + 255) / 256) {
            case 0: case 1: GELO_CASE(256, 1)
            case 2: GELO_CASE(256, 2)
            case 3: GELO_CASE(256, 3)
            default: GELO_CASE(256, 4)
        }
    } else {
        switch ((m + 511) / 512) {
            case 3: GELO_CASE(512, 3)
            case 4: GELO_CASE(512, 4)
            case 5: GELO_CASE(512, 5)
            case 6: GELO_CASE(512, 6)
            case 7: GELO_CASE(512, 7)
            case 8: GELO_CASE(512, 8)
            case 9: GELO_CASE(512, 9)
            case 10: GELO_CASE(512, 10)
            default: return hipErrorInvalidValue;
        }
    }
#undef GELO_CASE
    return hipGetLastError();
}

hipError_t gemm(const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc, int M, int N, int K,
                bool subtract, hipStream_t s) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    GemmOperands g;
    g.A = A; g.lda = lda;
    g.B0 = B; g.ldb0 = ldb; g.K0 = K;
    g.B1 = B; g.ldb1 = ldb;
    g.C = C; g.ldc = ldc;
    g.M = M; g.N = N; g.K = K;
    g.subtract = subtract;
    return gemm_f32(g, s);
}

constexpr size_t kTriangleLds = 2 * (size_t)BW * BW * sizeof(float);      // the triangle and its inverse

}  // namespace

hipError_t lu_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(lu_block_finish_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kTriangleLds);
}

hipError_t lu_inverse(const FactorWorkspace& ws, hipStream_t s) {
    const int n_pad = ws.n_pad;
    const int64_t ld = ws.ld;
    float* M = ws.M;
    float* X = ws.X;
    float* Linv = ws.Dinv;
    float* Uinv = ws.Dinv + (int64_t)n_pad * BW;
    GELO_TRY(zero_ints(ws.flag, 1, s));
    hipLaunchKernelGGL(iota_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, s, ws.perm, n_pad);
    GELO_TRY(hipGetLastError());
    GELO_TRY(set_identity(X, ld, n_pad, s));

    // P A = L U
    int panel = 0;
    for (int c0 = 0; c0 < n_pad; c0 += BW) {
        const int w = n_pad - c0 < BW ? n_pad - c0 : BW;
        const int block_end = c0 + w;
        GELO_TRY(launch_lu_panel(M + (int64_t)c0 * ld + c0, ld, n_pad - c0, c0, ws.gat + 64 * (panel & 1), ws.perm, ws.flag, s));
        for (int pc = c0; pc + NB < block_end; pc += NB) {
            LuStepArgs a;
            a.M = M; a.ld = ld; a.n_pad = n_pad; a.pc = pc; a.block_end = block_end;
            a.nchunks = (block_end - pc - NB) / NB;
            a.gat_prev = ws.gat + 64 * (panel & 1);
            a.gat_next = ws.gat + 64 * ((panel + 1) & 1);
            a.perm = ws.perm; a.flag = ws.flag;
            GELO_TRY(launch_lu_step(a, s));
            ++panel;
        }
        hipLaunchKernelGGL(lu_block_finish_kernel, dim3(2 + (n_pad + 127) / 128), dim3(512), kTriangleLds, s,
                           M, ld, n_pad, c0, w, ws.gat + 64 * (panel & 1), Linv + (int64_t)c0 * BW, Uinv + (int64_t)c0 * BW);
        GELO_TRY(hipGetLastError());
        ++panel;
        const int rest = n_pad - block_end;
        // U12 = L11^-1 U12 (in place), then A22 -= L21 U12
        GELO_TRY(gemm(Linv + (int64_t)c0 * BW, BW, M + (int64_t)c0 * ld + block_end, ld,
                      M + (int64_t)c0 * ld + block_end, ld, w, rest, w, false, s));
        GELO_TRY(gemm(M + (int64_t)block_end * ld + c0, ld, M + (int64_t)c0 * ld + block_end, ld,
                      M + (int64_t)block_end * ld + block_end, ld, rest, rest, w, true, s));
    }
    // L Y = I: block row b of Y is zero right of its diagonal block
    for (int c0 = 0; c0 < n_pad; c0 += BW) {
        const int w = n_pad - c0 < BW ? n_pad - c0 : BW;
        const int block_end = c0 + w;
        GELO_TRY(gemm(Linv + (int64_t)c0 * BW, BW, X + (int64_t)c0 * ld, ld, X + (int64_t)c0 * ld, ld, w, block_end, w, false, s));
        GELO_TRY(gemm(M + (int64_t)block_end * ld + c0, ld, X + (int64_t)c0 * ld, ld, X + (int64_t)block_end * ld, ld,
                      n_pad - block_end, block_end, w, true, s));
    }
    // U Z = Y
    for (int c0 = (n_pad - 1) / BW * BW; c0 >= 0; c0 -= BW) {
        const int w = n_pad - c0 < BW ? n_pad - c0 : BW;
        GELO_TRY(gemm(Uinv + (int64_t)c0 * BW, BW, X + (int64_t)c0 * ld, ld, X + (int64_t)c0 * ld, ld, w, n_pad, w, false, s));
        GELO_TRY(gemm(M + c0, ld, X + (int64_t)c0 * ld, ld, X, ld, c0, n_pad, w, true, s));
    }
    // A^-1 = Z P
    hipLaunchKernelGGL(permute_columns_kernel, dim3(n_pad), dim3(256), 0, s, X, ld, n_pad, ws.perm);
    return hipGetLastError();
}

hipError_t kappa_estimate(const float* A, const float* Ainv, int64_t lda, int n, const FactorWorkspace& ws,
                          int steps, hipStream_t s) {
    const int64_t ld = ws.ld;
    if (steps < 1 || steps > kLanczosMax) return hipErrorInvalidValue;
    if (steps > n) steps = n;
    // transposes into the (now free) factorisation buffers
    GELO_TRY(emit_matrix(A, lda, 0, nullptr, n, ld, nullptr, nullptr, ws.M, nullptr, s));
    GELO_TRY(emit_matrix(Ainv, lda, 0, nullptr, n, ld, nullptr, nullptr, ws.X, nullptr, s));
    const dim3 grid((2 * n + 3) / 4), block(256);
    float* va = ws.vec;            float* ya = va + 2 * ld;   float* wa = va + 3 * ld;
    float* vi = ws.vec + 4 * ld;   float* yi = vi + 2 * ld;   float* wi = vi + 3 * ld;
    hipLaunchKernelGGL(lanczos_vector_kernel, dim3(2), dim3(1024), 0, s, ws.vec, ld, n, ws.tri, -1);
    GELO_TRY(hipGetLastError());
    for (int j = 0; j < steps; ++j) {
        // w = M^T (M v) for M = A and M = Ainv, then one step of the recurrence for both
        hipLaunchKernelGGL(matvec_pair_kernel, grid, block, 0, s, A, lda, va, ya, Ainv, lda, vi, yi, n);
        GELO_TRY(hipGetLastError());
        hipLaunchKernelGGL(matvec_pair_kernel, grid, block, 0, s, ws.M, ld, ya, wa, ws.X, ld, yi, wi, n);
        GELO_TRY(hipGetLastError());
        hipLaunchKernelGGL(lanczos_vector_kernel, dim3(2), dim3(1024), 0, s, ws.vec, ld, n, ws.tri, j);
        GELO_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(lanczos_finish_kernel, dim3(1), dim3(64), 0, s, ws.tri, steps, ws.scalars);
    return hipGetLastError();
}

}  // namespace gelo
