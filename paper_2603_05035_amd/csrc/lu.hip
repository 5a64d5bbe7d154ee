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
// the next launch applies to all other columns in one round trip.  The inverses of the block's two
// diagonal triangles grow by one block row / column per launch beside the panel chain; after the
// block, U12 = L11^-1 U12 and the trailing update are float GEMMs with K = 128.  The inverse then is two block substitutions (GEMMs again, the right-hand
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
    __shared__ __attribute__((aligned(16))) float stage[NW][64 * (NB + 4)];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t prow_addr = (uint32_t)(size_t)prow;       // its LDS byte address
    float P[R][NB];
    unsigned used = 0;                       // bit i: register row i is absent or already a pivot row
    // A thread owns whole rows (64 bytes of the row-major matrix each), but a load in which every lane
    // reads a different row touches 64 cache lines.  So the 64 rows of a wave travel through an LDS
    // stage: four lanes read one row together (16 lines per load), then every lane picks up its row.
    constexpr int SP = NB + 4;               // stage pitch, floats
    float* st = stage[wave];
    const int srow = lane >> 2, schunk = (lane & 3) * 4;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int base = i * NTHR + 64 * wave;
        float4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rr = base + 16 * q + srow;
            v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rr < m) v[q] = *reinterpret_cast<const float4*>(Mp + (int64_t)rr * ld + schunk);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<float4*>(&st[(16 * q + srow) * SP + schunk]) = v[q];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4) {
            const float4 x = *reinterpret_cast<const float4*>(&st[lane * SP + c4 * 4]);
            P[i][c4 * 4 + 0] = x.x; P[i][c4 * 4 + 1] = x.y; P[i][c4 * 4 + 2] = x.z; P[i][c4 * 4 + 3] = x.w;
        }
        __builtin_amdgcn_wave_barrier();
        if (base + lane >= m) used |= 1u << i;
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
            // the pivot row's columns j..15 (all the update reads) go to LDS.  The stores are written as
            // instructions: left to the compiler, the R alternatives are merged into one store whose source
            // is picked at run time, and an array indexed that way stays in scratch memory.
            static_for<R>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                if (i == q_slot) {
                    static_for<NB - j>([&](auto cc) {
                        constexpr int c = j + decltype(cc)::value;
                        const float val = P[i][c];
                        const uint32_t addr = prow_addr;
                        asm volatile("ds_write_b32 %0, %1 offset:%2" :: "v"(addr), "v"(val), "n"(c * 4) : "memory");
                    });
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
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
#pragma unroll
        for (int j = 0; j < NB; ++j) {
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
        }
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
    for (int i = 0; i < R; ++i) {            // back through the stage, every row to its new position
        const int base = i * NTHR + 64 * wave;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4)
            *reinterpret_cast<float4*>(&st[lane * SP + c4 * 4]) = make_float4(P[i][c4 * 4], P[i][c4 * 4 + 1], P[i][c4 * 4 + 2], P[i][c4 * 4 + 3]);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rr = base + 16 * q + srow;
            const float4 x = *reinterpret_cast<const float4*>(&st[(16 * q + srow) * SP + schunk]);
            if (rr < m) *reinterpret_cast<float4*>(Mp + (int64_t)pos_of[rr] * ld + schunk) = x;
        }
        __builtin_amdgcn_wave_barrier();
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
    __shared__ float X0[NB][NB];          // the chunk's top block after the interchanges
    __shared__ float Us[NB][NB];
    __shared__ int cg[64];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int cc = lane & 15, g = lane >> 4;
    // nothing below the panel's top block moves any more: L11 and the first rows of L21 are fetched
    // together with the interchange list
    float l11 = 0.f;
    if (tid < 64) cg[tid] = gat[tid];
    if (tid < NB * NB) l11 = M[(int64_t)(pc + (tid >> 4)) * ld + pc + (tid & 15)];
    const int nblk = (n_pad - pc) / NB - 1;
    constexpr int UN = 4;                                 // blocks in flight per wave
    f32x4_t a4[2][UN], acc[2][UN];
    auto rowbase = [&](int b) { return pc + NB + NB * (b < nblk ? b : nblk - 1); };     // clamped: a valid address, no branch
    auto load_l = [&](int buf, int b0) {
#pragma unroll
        for (int u = 0; u < UN; ++u)
            a4[buf][u] = *reinterpret_cast<const f32x4_t*>(M + (int64_t)(rowbase(b0 + 8 * u) + cc) * ld + pc + 4 * g);
    };
    auto load_c = [&](int buf, int b0) {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const float* cp = M + (int64_t)(rowbase(b0 + 8 * u) + 4 * g) * ld + col0 + cc;
            acc[buf][u] = f32x4_t{cp[0], cp[ld], cp[2 * ld], cp[3 * ld]};
        }
    };
    load_l(0, wave);
    __syncthreads();
    {
        const int e = tid >> 4, c = tid & 15;             // 32 entries x 16 columns
        const int src = cg[32 + e], dst = cg[e];
        float v = 0.f;
        if (src >= 0) v = M[(int64_t)src * ld + col0 + c];
        if (tid < NB * NB) L11[tid >> 4][tid & 15] = l11;
        __syncthreads();                                  // every row is read before any is overwritten
        if (dst >= 0) M[(int64_t)dst * ld + col0 + c] = v;
        if (e < NB) X0[e][c] = v;                         // entries 0..15 are the rows pc .. pc + 15
    }
    __threadfence_block();
    __syncthreads();
    load_c(0, wave);                                      // in flight while the first 16 lanes solve the top block
    if (tid < NB) {
        float x[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) x[i] = X0[i][tid];
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
    float bq[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) bq[e] = -Us[4 * g + e][cc];
    auto update = [&](auto bufc, int b0) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int b = b0 + 8 * u;
            f32x4_t r = acc[buf][u];
            r = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[buf][u][0], bq[0], r, 0, 0, 0);
            r = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[buf][u][1], bq[1], r, 0, 0, 0);
            r = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[buf][u][2], bq[2], r, 0, 0, 0);
            r = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[buf][u][3], bq[3], r, 0, 0, 0);
            if (b < nblk) {
                float* cp = M + (int64_t)(pc + NB + NB * b + 4 * g) * ld + col0 + cc;
                cp[0] = r[0]; cp[ld] = r[1]; cp[2 * ld] = r[2]; cp[3 * ld] = r[3];
            }
        }
    };
    // two groups per trip, so that the buffer indices are constants: the next group's loads are
    // issued before the current group's MFMAs and stores
    for (int b0 = wave; b0 < nblk; b0 += 16 * UN) {
        const bool second = b0 + 8 * UN < nblk;
        if (second) { load_l(1, b0 + 8 * UN); load_c(1, b0 + 8 * UN); }
        update(std::integral_constant<int, 0>{}, b0);
        if (b0 + 16 * UN < nblk) { load_l(0, b0 + 16 * UN); load_c(0, b0 + 16 * UN); }
        if (second) update(std::integral_constant<int, 1>{}, b0 + 8 * UN);
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

// ------------------------------------------ inverses of the diagonal triangles --
// The inverses of the two 128 x 128 triangles of an outer block (L11 unit lower, U11 upper) are
// what turns the block's triangular solves into GEMMs.  They grow with the block: once panel ib is
// factorised, block row ib of L11^-1 and block column ib of U11^-1 depend only on finished data,
// so two spare workgroups of the next launch compute them beside the panel chain.
// Both results are row-major with pitch BW; entries outside the triangles are written as zeros.

// Block row ib of Linv = L11^-1.  First the interchanges of panel ib are applied to the block's
// columns left of that panel (those entries belong to L11 and nobody else touches them in this
// launch); then thread j < 128 computes column j of the block row:
// Linv[ib][:, j] = Lii^-1 (E[ib][:, j] - sum_{kb < ib} L[ib][kb] Linv[kb][:, j]).  512 threads.
__device__ __forceinline__ void linv_block_row(float* M, int64_t ld, int c0, int ib, int w, const int* gat, float* Linv) {
    __shared__ float Lr[NB][BW + 1];
    __shared__ int cg[64];
    const int tid = threadIdx.x;
    const int width = NB * ib;                             // columns [c0, c0 + width) lie left of panel ib
    if (tid < 64) cg[tid] = gat[tid];
    __syncthreads();
    {
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
    }
    __threadfence_block();
    __syncthreads();
    const int cols = width + NB;                           // block row ib of L11: 16 rows x cols
    for (int id = tid; id < NB * cols; id += 512) {
        const int ii = id / cols, k = id - ii * cols;
        Lr[ii][k] = M[(int64_t)(c0 + width + ii) * ld + c0 + k];
    }
    __syncthreads();
    if (tid >= BW || tid >= w) return;
    const int j = tid;
    float acc[NB];
#pragma unroll
    for (int ii = 0; ii < NB; ++ii) acc[ii] = width + ii == j ? 1.f : 0.f;
    if (j < cols) {
#pragma unroll 1
        for (int kb = 0; kb < ib; ++kb) {
            float xk[NB];
#pragma unroll
            for (int kk = 0; kk < NB; ++kk) xk[kk] = Linv[(kb * NB + kk) * BW + j];
#pragma unroll
            for (int ii = 0; ii < NB; ++ii)
#pragma unroll
                for (int kk = 0; kk < NB; ++kk) acc[ii] = fmaf(-Lr[ii][kb * NB + kk], xk[kk], acc[ii]);
        }
#pragma unroll
        for (int ii = 1; ii < NB; ++ii)
#pragma unroll
            for (int kk = 0; kk < ii; ++kk) acc[ii] = fmaf(-Lr[ii][width + kk], acc[kk], acc[ii]);
    }
#pragma unroll
    for (int ii = 0; ii < NB; ++ii) Linv[(width + ii) * BW + j] = acc[ii];
}

// Block column ib of Uinv = U11^-1: Uinv[ib][ib] = Uii^-1 and, above it,
// Uinv[0:ib][ib] = -Uinv[0:ib][0:ib] (U[0:ib][ib] Uii^-1); zeros below.  Thread j < 128 owns row j.
__device__ __forceinline__ void uinv_block_col(const float* M, int64_t ld, int c0, int ib, int w, float* Uinv) {
    __shared__ float Uc[BW][NB + 1];                       // U[0 : 16 (ib + 1)][panel ib]
    __shared__ float Dii[NB][NB + 1];
    __shared__ float Y[BW][NB + 1];
    const int tid = threadIdx.x;
    const int above = NB * ib;
    for (int id = tid; id < (above + NB) * NB; id += 512) {
        const int r = id >> 4, c = id & 15;
        Uc[r][c] = M[(int64_t)(c0 + r) * ld + c0 + above + c];
    }
    __syncthreads();
    if (tid < NB) {                                        // column tid of Uii^-1 by back substitution
        float x[NB];
#pragma unroll
        for (int i = NB - 1; i >= 0; --i) {
            float t = i == tid ? 1.f : 0.f;
#pragma unroll
            for (int k = i + 1; k < NB; ++k) t = fmaf(-Uc[above + i][k], x[k], t);
            x[i] = t / Uc[above + i][i];
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) Dii[i][tid] = x[i];
    }
    __syncthreads();
    if (tid < above) {                                     // Y = U[0:ib][ib] Uii^-1, row tid
        float y[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) y[c] = 0.f;
#pragma unroll
        for (int m = 0; m < NB; ++m) {
            const float u = Uc[tid][m];
#pragma unroll
            for (int c = 0; c < NB; ++c) y[c] = fmaf(u, Dii[m][c], y[c]);
        }
#pragma unroll
        for (int c = 0; c < NB; ++c) Y[tid][c] = y[c];
    }
    __syncthreads();
    if (tid >= BW || tid >= w) return;
    const int j = tid;
    float z[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) z[c] = 0.f;
    if (j < above) {
#pragma unroll 1
        for (int kb = j >> 4; kb < ib; ++kb) {             // row j of Uinv is zero left of its diagonal
            float uk[NB];
#pragma unroll
            for (int k4 = 0; k4 < NB / 4; ++k4) {
                const float4 t = *reinterpret_cast<const float4*>(Uinv + j * BW + kb * NB + k4 * 4);
                uk[k4 * 4 + 0] = t.x; uk[k4 * 4 + 1] = t.y; uk[k4 * 4 + 2] = t.z; uk[k4 * 4 + 3] = t.w;
            }
#pragma unroll
            for (int kk = 0; kk < NB; ++kk)
#pragma unroll
                for (int c = 0; c < NB; ++c) z[c] = fmaf(-uk[kk], Y[kb * NB + kk][c], z[c]);
        }
    } else if (j < above + NB) {
#pragma unroll
        for (int c = 0; c < NB; ++c) z[c] = Dii[j - above][c];
    }
#pragma unroll
    for (int c4 = 0; c4 < NB / 4; ++c4)
        *reinterpret_cast<float4*>(Uinv + j * BW + above + c4 * 4) = make_float4(z[c4 * 4], z[c4 * 4 + 1], z[c4 * 4 + 2], z[c4 * 4 + 3]);
}

// One launch per panel inside an outer block (not its first panel):
//   workgroup 0             applies the previous panel (at pc) to the next 16 columns, then factorises them;
//   workgroups < nchunks    apply it to the other 16-column chunks of the block;
//   the next two            extend the inverses of the block's triangles by the previous panel's block row / column
//                           (the first of them also moves the block's own rows left of that panel);
//   the rest                apply its interchanges to every column outside the block.
// No two workgroups touch the same data.
struct LuStepArgs {
    float* M; int64_t ld; int n_pad;
    int c0, w;                // the outer block: first column, width
    int pc;                   // first row / column of the previous panel
    int nchunks;              // (c0 + w - pc - 16) / 16 >= 1
    const int* gat_prev;      // interchanges of the previous panel
    int* gat_next;            // written by the panel factorised here
    int* perm; int* flag;
    float* Linv; float* Uinv; // inverses of this block's triangles (pitch BW)
};

template <int NTHR, int R>
__global__ __launch_bounds__(512)
void lu_step_kernel(LuStepArgs a) {
    const int b = blockIdx.x;
    if (b >= a.nchunks) {
        const int ib = (a.pc - a.c0) / NB;
        if (b == a.nchunks) linv_block_row(a.M, a.ld, a.c0, ib, a.w, a.gat_prev, a.Linv);
        else if (b == a.nchunks + 1) uinv_block_col(a.M, a.ld, a.c0, ib, a.w, a.Uinv);
        else lu_gather_body(a.M, a.ld, a.gat_prev, b - a.nchunks - 2, a.n_pad, a.c0, a.c0 + a.w);
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

// After the last panel of an outer block: the last block row / column of the two inverses
// (workgroups 0 and 1), and that panel's interchanges on every column outside the block.
__global__ __launch_bounds__(512)
void lu_block_finish_kernel(float* M, int64_t ld, int n_pad, int c0, int w, const int* gat, float* Linv, float* Uinv) {
    const int b = blockIdx.x;
    const int ib = w / NB - 1;
    if (b == 0) linv_block_row(M, ld, c0, ib, w, gat, Linv);
    else if (b == 1) uinv_block_col(M, ld, c0, ib, w, Uinv);
    else lu_gather_body(M, ld, gat, b - 2, n_pad, c0, c0 + w);
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

// Largest eigenvalue of the symmetric tridiagonal matrix (alpha[0..k), beta[0..k-1)) by sectioning on
// the Sturm count: one wave, lanes 0..31 work on A, lanes 32..63 on A^-1; each round every lane counts
// the eigenvalues below its own trial value (32 trial values per bracket), and the bracket shrinks to
// the interval between the last trial with an eigenvalue at or above it and the first one above all.
// out[0] = sqrt(lambda_A lambda_Ainv) = the kappa_2 estimate, out[1], out[2] its factors.
__global__ __launch_bounds__(64)
void lanczos_finish_kernel(const float* tri, int k, float* out) {
    __shared__ float co[2 * 2 * kLanczosMax];
    const int lane = threadIdx.x, o = lane >> 5, l = lane & 31;
    co[lane] = tri[lane]; co[lane + 64] = tri[lane + 64];
    __syncthreads();
    const float* al = co + o * 2 * kLanczosMax;
    const float* be = al + kLanczosMax;
    float hi = 0.f;
    for (int i = 0; i < k; ++i) {
        const float gsh = fabsf(al[i]) + (i > 0 ? fabsf(be[i - 1]) : 0.f) + (i + 1 < k ? fabsf(be[i]) : 0.f);
        hi = fmaxf(hi, gsh);
    }
    float lo = 0.f;
    for (int round = 0; round < 6; ++round) {
        const float step = (hi - lo) * (1.0f / 32.0f);
        const float x = lo + step * (float)(l + 1);        // l = 31: the current upper end
        int below = 0;                                     // eigenvalues below x
        float d = 1.f;
        for (int i = 0; i < k; ++i) {
            const float b2 = i > 0 ? be[i - 1] * be[i - 1] : 0.f;
            d = al[i] - x - b2 * __builtin_amdgcn_rcpf(d);
            if (fabsf(d) < 1e-30f) d = -1e-30f;
            below += d < 0.f;
        }
        const unsigned long long all = __ballot(below == k);
        const unsigned half = (unsigned)(all >> (32 * o));  // this operator's lanes
        const int first = half ? __ffs(half) - 1 : 31;      // first trial above every eigenvalue
        hi = lo + step * (float)(first + 1);
        lo = lo + step * (float)first;
    }
    const float sigma = sqrtf(0.5f * (lo + hi));
    const float s0 = __shfl(sigma, 0, 64), s1 = __shfl(sigma, 32, 64);
    if (lane == 0) { out[1] = s0; out[2] = s1; out[0] = s0 * s1; }
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
    const dim3 grid(a.nchunks + 2 + (a.n_pad + 127) / 128);
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

}  // namespace

hipError_t lu_init() {         // brings this file's code onto the device (see factor_init)
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&permute_columns_kernel));
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
            a.M = M; a.ld = ld; a.n_pad = n_pad; a.c0 = c0; a.w = w; a.pc = pc;
            a.nchunks = (block_end - pc - NB) / NB;
            a.Linv = Linv + (int64_t)c0 * BW; a.Uinv = Uinv + (int64_t)c0 * BW;
            a.gat_prev = ws.gat + 64 * (panel & 1);
            a.gat_next = ws.gat + 64 * ((panel + 1) & 1);
            a.perm = ws.perm; a.flag = ws.flag;
            GELO_TRY(launch_lu_step(a, s));
            ++panel;
        }
        hipLaunchKernelGGL(lu_block_finish_kernel, dim3(2 + (n_pad + 127) / 128), dim3(512), 0, s,
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
