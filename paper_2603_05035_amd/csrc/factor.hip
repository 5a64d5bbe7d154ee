// Blocked Householder QR with explicit Q: the orthogonal mixing matrix the trusted side draws
// for every batch (Section 3.2 step 1.2; Table 3's "A-gen (QR)" step), and the workspace shared
// with the LU path.  Everything is float and deterministic: reductions run in a fixed order, no
// atomics.
//
// Column panels are 16 wide.  A panel is factorised by ONE workgroup that keeps its rows in
// registers (thread t owns rows t, t+NTHR, ...), so the per-column reductions cost one barrier
// and no memory traffic; the block reflectors are applied on the matrix cores.
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
// Factorises the m x 16 panel at Mp (read only; R on and above the diagonal and the reflector tails below, as
// in LAPACK, exist in registers only) and writes for the block reflector I - V T V^T:
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
// UPDATE = false builds every reflector from the column as it stands in memory - the later columns of the panel do
// not see the earlier reflectors - which is what the product of directly drawn reflectors needs (householder_qr with
// `direct`): the same reflector formulas, the same T, no factorisation.
template <int NTHR, int R, bool UPDATE = true>
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
            if constexpr (UPDATE) {
#pragma unroll
                for (int s = j + 1; s < NB; ++s) P[0][s] = fmaf(-tv, w[s], P[0][s]);
            }
        }
#pragma unroll
        for (int i = 1; i < R; ++i) {
            const float v = P[i][j] * scale;
            P[i][j] = v;
            const float tv = tau * v;
            if constexpr (UPDATE) {
#pragma unroll
                for (int s = j + 1; s < NB; ++s) P[i][s] = fmaf(-tv, w[s], P[i][s]);
            }
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

    // write the clean reflector block in its two layouts (the factored panel itself - R and the reflector tails -
    // is not stored: nobody reads these columns again, the diagonal of R went to rdiag)
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
                    Vt[(int64_t)(r >> 4) * 256 + c * 16 + (r & 15)] = v[e];
                }
                *reinterpret_cast<float4*>(Vr + (int64_t)r * NB + c4 * 4) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

template <int NTHR, int R>
__global__ __launch_bounds__(NTHR)
void qr_panel_kernel(float* Mp, float* Vr, float* Vt, float* Tg, float* rdiag, int m, int64_t batch_stride) {
    const int64_t off = (int64_t)blockIdx.y * batch_stride;
    qr_panel_body<NTHR, R>(Mp + off, Vr + off, Vt + off, Tg + off, rdiag + off, m);
}

// All the panels of a matrix at once, every reflector from the raw column (grid x = panel, grid y = matrix): panel p
// is the tile column p from its diagonal tile down, 16 (panels - p) rows; its reflector block goes where
// householder_qr keeps panel p's (Vr side by side in Vc, Vt in place of the panel, T and diag(R) in their arrays).
template <int NTHR, int R>
__global__ __launch_bounds__(NTHR)
void direct_panels_kernel(float* M, float* Vc, float* Tmat, float* rdiag, int nbr, int64_t batch_stride) {
    const int p = blockIdx.x;
    const int64_t off = (int64_t)blockIdx.y * batch_stride;
    float* Mp = M + off + (int64_t)p * nbr * 256 + (int64_t)p * 256;
    qr_panel_body<NTHR, R, false>(Mp, Vc + off + (int64_t)p * nbr * 16 * NB, Mp, Tmat + off + (int64_t)p * NB * NB, rdiag + off + p * NB, (nbr - p) * NB);
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

// One block reflector I - V op(T) V^T as a strip sees it: V in both layouts, its triangle, and `shift`, the
// number of 16-row blocks by which its first row lies below the strip's first row (a strip that applies several
// reflectors of a block of panels in one pass starts at the oldest one's first row).
struct Reflector { const float* Vr; const float* Vt; const float* T; int shift; int plain_t; };
// plain_t: op(T) = T (the reflector itself, I - V T V^T: what forming Q applies) instead of T^T (its transpose: what
// the factorisation applies to the columns behind it); honoured by reflect_strip_lds_body only
// (the pointers are those of the first matrix of a batch; `off` below is the distance to this workgroup's matrix)

constexpr int kBulkFromCount = 2;         // from this many factorisations side by side the block strips get launches of their own
constexpr int kPanelRows256 = 1024;      // panels of up to this many rows are factorised by 256 threads, longer ones by 512
constexpr int kMaxDelay = 4;             // panels per block of the delayed update: most reflectors a strip pass of the factorisation applies
constexpr int kMaxProduct = 8;           // most reflectors a strip pass applies while Q is formed (qr_bulk_kernel: all reflectors exist by then,
                                         // so the passes can be longer: measured 10% less time for the same reflectors than passes of four)

// a tile of zeros: what a strip block reads in place of a reflector block that does not exist for it
__device__ __attribute__((aligned(1024))) float g_zero_tile[256];

// NS neighbouring 16-column strips per workgroup (`strips` of them exist: the last may be missing at the end of a
// range; the tiles of neighbouring strips lie `strip_stride` floats apart).  With two strips every reflector block a
// wave fetches feeds twice the matrix instructions, at twice the registers; measured equal to two one-strip
// workgroups per compute unit (reflect_strip_lds_body), which is what the launches of many matrices use, so only
// NS = 1 is instantiated at present.  Each strip's arithmetic is the same whichever way strips are grouped.
template <int NBLK, int NS>
__device__ __forceinline__ void reflect_strip_body(const Reflector* refl, int count, int64_t off, float* Cs,
                                                   int64_t strip_stride, int strips, int nblocks) {
    constexpr int NC = NB * NS;                              // columns per workgroup
    __shared__ float Wp[2][8][NB][NC];                       // the waves' partial W, alternating between reflectors
    __shared__ float Ts[2][NB][NB];
    // the wave index as a scalar: block numbers and their offsets then live in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;

    float* Cl = Cs + c * 16 + 4 * g;                         // this lane's column, its first row of tile 0
    // Blocks past the end take no part: their strip registers are zero, they meet the zero tile instead of a
    // reflector block (so they are still zero when the next reflector of a block of panels comes), and they are
    // not stored; their loads are clamped to the last block (a valid address, no branch).  A missing second
    // strip is all zeros and not stored either.
    const int last = nblocks - 1;
    f32x4_t cr[NS][NBLK];
#pragma unroll
    for (int st = 0; st < NS; ++st) {
        const bool have = st < strips;
        const float* Csl = Cl + (have ? st * strip_stride : 0);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int blk = wave + 8 * b;
            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(Csl + 256 * (blk < nblocks ? blk : last));
            const bool valid = have && blk < nblocks;
            cr[st][b] = f32x4_t{valid ? v[0] : 0.f, valid ? v[1] : 0.f, valid ? v[2] : 0.f, valid ? v[3] : 0.f};
        }
    }
    // The reflector operands stream through two register groups of GRP blocks.  Per reflector there are 2 NG
    // groups, first those of the tiled layout (W = V^T C), then those of the row layout (C += V W'); group j
    // uses register group j % 2, and as soon as a group has been consumed the group two places further on -
    // of the next reflector, if this one has no more - is requested into the same registers.  Two groups are
    // always on their way, across the barriers and from one reflector to the next: a load consumed right behind
    // its issue would expose one memory latency per group.
    constexpr int GRP = (NBLK == 20 && NS == 1) ? 10 : 5, NG = NBLK / GRP;
    static_assert(NBLK % GRP == 0, "blocks per wave must be a multiple of the load group");
    f32x4_t va[2][GRP];
    const float* zero_l = g_zero_tile + c * 16 + 4 * g;
    auto request = [&](const Reflector& R, auto jc) {
        constexpr int j = decltype(jc)::value, phase = j / NG, grp = j % NG;
        // Vt: reflector c, this lane's four rows of the block; Vr: row c of the block, reflectors 4 g ..
        const float* base = (phase == 0 ? R.Vt : R.Vr) + off + c * 16 + 4 * g;
#pragma unroll
        for (int k = 0; k < GRP; ++k) {
            const int blk = wave + 8 * (grp * GRP + k), vb = blk - R.shift;      // strip block blk meets reflector block blk - shift
            const float* src = (vb >= 0 && blk <= last) ? base + 256 * vb : zero_l;
            va[j & 1][k] = *reinterpret_cast<const f32x4_t*>(src);
        }
    };
    // the triangle of a reflector is fetched one reflector ahead (needed behind its second barrier only), so that
    // no wait for it ever stands between a request and the products that use older requests
    float t_next = tid < NB * NB ? refl[0].T[off + tid] : 0.f;
    request(refl[0], std::integral_constant<int, 0>{});
    request(refl[0], std::integral_constant<int, 1>{});
    // (the loop over the reflectors is unrolled: the waits for the requests then count exactly what is outstanding)
    static_for<kMaxDelay>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        if (q >= count) return;
        const Reflector R = refl[q];
        const bool more = q + 1 < count;
        const Reflector Rn = more ? refl[q + 1] : R;
        auto request_behind = [&](auto jc) {                  // the group two places behind group j
            constexpr int j = decltype(jc)::value;
            if constexpr (j + 2 < 2 * NG) request(R, std::integral_constant<int, j + 2>{});
            else if (more) request(Rn, std::integral_constant<int, j + 2 - 2 * NG>{});
        };
        const float t_mine = t_next;
        // W_partial[i][col] = sum over this wave's rows of V[r][i] C[r][col]; MFMA (b, v) contracts the four
        // rows 16 blk + 4 kk + v (kk = lane / 16): A = V[row][lane % 16], B = the strip register itself.
        f32x4_t w0[NS], w1[NS];
#pragma unroll
        for (int st = 0; st < NS; ++st) { w0[st] = f32x4_t{0.f, 0.f, 0.f, 0.f}; w1[st] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }
        static_for<NG>([&](auto gc) {
            constexpr int grp = decltype(gc)::value;
#pragma unroll
            for (int k = 0; k < GRP; ++k) {
                const int b = grp * GRP + k;
                const f32x4_t a = va[grp & 1][k];
                if (wave + 8 * b > last) continue;            // a block past the end (wave-uniform): nothing to add
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    w0[st] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], cr[st][b][0], w0[st], 0, 0, 0);
                    w1[st] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], cr[st][b][1], w1[st], 0, 0, 0);
                }
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    w0[st] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], cr[st][b][2], w0[st], 0, 0, 0);
                    w1[st] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], cr[st][b][3], w1[st], 0, 0, 0);
                }
            }
            request_behind(gc);
        });
        if (tid < NB * NB) { if (R.plain_t) Ts[q & 1][tid & 15][tid >> 4] = t_mine; else Ts[q & 1][tid >> 4][tid & 15] = t_mine; }
        if (more && tid < NB * NB) t_next = Rn.T[off + tid];
#pragma unroll
        for (int st = 0; st < NS; ++st)
#pragma unroll
            for (int v = 0; v < 4; ++v) Wp[q & 1][wave][4 * g + v][st * NB + c] = w0[st][v] + w1[st][v];     // accumulator row 4 g + v, column c
        __syncthreads();
        // ONE barrier per reflector: every wave adds the eight partial W (in wave order) for the entries it needs as
        // an operand and forms W' = -T^T W itself, on the matrix cores: step s contracts reflectors 4 s + kk,
        // A = T[4 s + kk][lane % 16], B = W[4 s + kk][lane % 16]; the result arrives in the accumulator layout,
        // which is the operand layout of the second product.  (The partial sums and the triangle alternate between
        // two buffers: a wave may be a whole reflector ahead of another one that is still reading.)
        // C_block += V_block W': MFMA k contracts reflectors 4 kk + k; A = V[16 blk + lane % 16][4 kk + k]
        float bq[NS][4];
        {
            float ta[4];
#pragma unroll
            for (int sx = 0; sx < 4; ++sx) ta[sx] = Ts[q & 1][4 * sx + g][c];
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                f32x4_t wn = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int sx = 0; sx < 4; ++sx) {
                    float sum = Wp[q & 1][0][4 * sx + g][st * NB + c];
#pragma unroll
                    for (int w = 1; w < 8; ++w) sum += Wp[q & 1][w][4 * sx + g][st * NB + c];
                    wn = __builtin_amdgcn_mfma_f32_16x16x4f32(ta[sx], sum, wn, 0, 0, 0);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) bq[st][k] = -wn[k];
            }
        }
        static_for<NG>([&](auto gc) {
            constexpr int grp = decltype(gc)::value, j = NG + grp;
#pragma unroll
            for (int k = 0; k < GRP; ++k) {
                const int b = grp * GRP + k;
                const f32x4_t a4 = va[j & 1][k];
                if (wave + 8 * b > last) continue;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int st = 0; st < NS; ++st)
                        cr[st][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[kk], bq[st][kk], cr[st][b], 0, 0, 0);
            }
            request_behind(std::integral_constant<int, j>{});
        });
    });
#pragma unroll
    for (int st = 0; st < NS; ++st) {
        if (st < strips) {
            float* Csl = Cl + st * strip_stride;
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int blk = wave + 8 * b;
                if (blk < nblocks) *reinterpret_cast<f32x4_t*>(Csl + 256 * blk) = cr[st][b];
            }
        }
    }
}

// The same strip for launches that hold nothing but strips (several factorisations side by side: see
// householder_qr).  There the strips' own phases - read the strip, matrix instructions, write it - must overlap
// BETWEEN workgroups of a compute unit, which takes two workgroups per unit, that is at most 128 registers per
// lane.  So the reflector blocks do not pass through registers: each wave fetches them straight into a small
// ring in LDS (direct-to-LDS loads; a block is one contiguous kilobyte in either layout, and lane l's 16 bytes
// land at 16 l, which is where it reads them back as the instruction's operand).  One 16-column strip per
// workgroup, arithmetic and summation order exactly those of reflect_strip_body.
__device__ __forceinline__ void fetch_block_to_lds(const void* gptr, uint32_t lds_addr) {      // lds_addr wave-uniform (travels in M0)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(gptr), "s"(lds_addr) : "memory", "m0");
}
template <int N> __device__ __forceinline__ void wait_fetches() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

template <int NBLK>
__device__ __forceinline__ void reflect_strip_lds_body(const Reflector* refl, int count, int64_t off, float* Cs, int nblocks) {
    constexpr int GRP = NBLK % 3 == 0 ? 3 : NBLK % 2 == 0 ? 2 : 1, NG = NBLK / GRP;      // blocks per fetch group, groups per product
    constexpr int DEPTH = 2;                                         // ring slots per wave: one group in use, one on its way
    __shared__ __attribute__((aligned(1024))) float ring[8][DEPTH][GRP][256];
    __shared__ float Wp[2][8][NB][NB];
    __shared__ float Ts[2][NB][NB];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;
    float* Cl = Cs + c * 16 + 4 * g;
    const int last = nblocks - 1;
    if (count < 1) return;                                           // no reflector: the strip stays as it is (and is not loaded at all)
    // The strip's own blocks arrive group by group behind the first product of the first reflector, each requested
    // two groups ahead of its use, so that a workgroup starts on the matrix cores after two groups instead of
    // after the whole strip.  (Blocks past the end load the last block again - a valid address, a fixed number of
    // loads - and are never used: the products and the stores skip them.)
    f32x4_t cr[NBLK];
    auto load_strip = [&](auto gc) {
        constexpr int grp = decltype(gc)::value;
        if constexpr (grp < NG) {
#pragma unroll
            for (int k = 0; k < GRP; ++k) {
                const int blk = wave + 8 * (grp * GRP + k);
                // the strip passes through once: keep it out of the way of the reflectors, which every strip of the matrix re-reads from L2
                cr[grp * GRP + k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(Cl + 256 * (blk < nblocks ? blk : last)));
            }
        }
    };
    const uint32_t ring_addr = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)&ring[wave][0][0][0]);
    const float* mine = &ring[wave][0][0][0] + lane * 4;                 // this lane's operand inside a block
    const float* zero_l = g_zero_tile + c * 16 + 4 * g;
    // Group j of reflector q (first the NG groups of the tiled layout, then the NG of the row layout) is number
    // u = 2 NG q + j of the strip and goes to ring slot u % DEPTH.  Before a wave waits for group u it requests group
    // u + 1 into the slot that group u - 1 has just left: one group is on its way while one is in use, across the
    // barriers and from one reflector to the next.
    auto request = [&](const Reflector& R, auto uc) {
        constexpr int u = decltype(uc)::value, j = u % (2 * NG), phase = j / NG, grp = j % NG;
        const float* base = (phase == 0 ? R.Vt : R.Vr) + off + c * 16 + 4 * g;
#pragma unroll
        for (int k = 0; k < GRP; ++k) {
            const int blk = wave + 8 * (grp * GRP + k), vb = blk - R.shift;
            const float* src = (vb >= 0 && blk <= last) ? base + 256 * vb : zero_l;
            fetch_block_to_lds(src, ring_addr + (uint32_t)(((u % DEPTH) * GRP + k) * 1024));
        }
    };
    float t_next = tid < NB * NB ? refl[0].T[off + tid] : 0.f;
    load_strip(std::integral_constant<int, 0>{});
    load_strip(std::integral_constant<int, 1>{});
    request(refl[0], std::integral_constant<int, 0>{});
    static_for<kMaxProduct>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        if (q >= count) return;
        const Reflector R = refl[q];
        const bool more = q + 1 < count;
        const Reflector Rn = more ? refl[q + 1] : R;
        // Fetches (and the strip's loads) are counted in issue order, so block k of group j has landed once no more
        // are outstanding than were issued behind it: the rest of its group, the strip group that went out with the
        // request for group j + 1 (first product of the first reflector only), and group j + 1 itself - which does
        // not exist behind the last group of the last reflector.  (Any other load of this wave in between only makes
        // the wait longer.)
        auto landed = [&](auto jc, auto kc) {
            constexpr int j = decltype(jc)::value, k = decltype(kc)::value;
            constexpr int own = GRP - 1 - k, strip = (q == 0 && j + 2 < NG) ? GRP : 0;
            if constexpr (j + 1 < 2 * NG) wait_fetches<own + strip + GRP>();
            else { if (more) wait_fetches<own + GRP>(); else wait_fetches<own>(); }
        };
        auto request_ahead = [&](auto jc) {                   // the next group, into the slot consumed last
            constexpr int j = decltype(jc)::value, nj = j + 1;
            if constexpr (nj < 2 * NG) request(R, std::integral_constant<int, 2 * NG * q + nj>{});
            else if (more) request(Rn, std::integral_constant<int, 2 * NG * q + nj>{});
        };
        const float t_mine = t_next;
        f32x4_t w0 = {0.f, 0.f, 0.f, 0.f}, w1 = {0.f, 0.f, 0.f, 0.f};
        static_for<NG>([&](auto gc) {
            constexpr int grp = decltype(gc)::value;
            if constexpr (q == 0) load_strip(std::integral_constant<int, grp + 2>{});
            request_ahead(gc);
            static_for<GRP>([&](auto kc) {
                constexpr int k = decltype(kc)::value, b = grp * GRP + k;
                if (wave + 8 * b > last) return;              // a block past the end (wave-uniform): its fetch was the zero tile
                landed(gc, kc);
                const f32x4_t a = *reinterpret_cast<const f32x4_t*>(mine + (((2 * NG * q + grp) % DEPTH) * GRP + k) * 256);
                w0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], cr[b][0], w0, 0, 0, 0);
                w1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], cr[b][1], w1, 0, 0, 0);
                w0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], cr[b][2], w0, 0, 0, 0);
                w1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], cr[b][3], w1, 0, 0, 0);
            });
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the operands are in registers before their ring slot is refilled
        });
        if (tid < NB * NB) { if (R.plain_t) Ts[q & 1][tid & 15][tid >> 4] = t_mine; else Ts[q & 1][tid >> 4][tid & 15] = t_mine; }
        if (more && tid < NB * NB) t_next = Rn.T[off + tid];
#pragma unroll
        for (int v = 0; v < 4; ++v) Wp[q & 1][wave][4 * g + v][c] = w0[v] + w1[v];
        __syncthreads();
        float bq[4];                                          // W' = -T^T W, formed by every wave (see reflect_strip_body)
        {
            f32x4_t wn = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sx = 0; sx < 4; ++sx) {
                float sum = Wp[q & 1][0][4 * sx + g][c];
#pragma unroll
                for (int w = 1; w < 8; ++w) sum += Wp[q & 1][w][4 * sx + g][c];
                wn = __builtin_amdgcn_mfma_f32_16x16x4f32(Ts[q & 1][4 * sx + g][c], sum, wn, 0, 0, 0);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) bq[k] = -wn[k];
        }
        static_for<NG>([&](auto gc) {
            constexpr int grp = decltype(gc)::value, j = NG + grp;
            request_ahead(std::integral_constant<int, j>{});
            static_for<GRP>([&](auto kc) {
                constexpr int k = decltype(kc)::value, b = grp * GRP + k;
                if (wave + 8 * b > last) return;
                landed(std::integral_constant<int, j>{}, kc);
                const f32x4_t a4 = *reinterpret_cast<const f32x4_t*>(mine + (((2 * NG * q + j) % DEPTH) * GRP + k) * 256);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) cr[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[kk], bq[kk], cr[b], 0, 0, 0);
            });
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        });
    });
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
        const int blk = wave + 8 * b;
        if (blk < nblocks) __builtin_nontemporal_store(cr[b], reinterpret_cast<f32x4_t*>(Cl + 256 * blk));
    }
}

// A block of panels applied to `outer` strips from Cout (the factorisation: the columns behind a finished block)
// or to `acc` strips from X (forming Q), for `count` matrices, one strip per workgroup.  Which workgroup takes which strip of which matrix is chosen for the
// L2s: workgroups are dealt to the 8 accelerator dies in turn (die = workgroup number mod 8), every strip of a matrix
// reads that matrix's reflectors (1.1 MB for a block of four) and a die's L2 holds 4 MB - so a die works through
// whole matrices one after the other (matrices die, die + 8, ...; with fewer than 8 matrices the dies that share a
// matrix split its strips) instead of meeting all `count` sets of reflectors at once.  A count that is not a
// multiple of 8 is dealt in two parts: whole rounds of 8 matrices, one per die, then the remaining count % 8
// matrices with their strips split over the dies that share each (20 matrices: two rounds, then 4 matrices on two
// dies each - a die works off 2.5 matrices' strips, not 3).
struct QrBulkArgs {
    Reflector refl[kMaxProduct]; int pending;
    float* Cout; float* X; int outer, acc;
    int64_t strip_stride; int nb_block; int64_t batch_stride; int count;
};
// workgroups per die that the deal needs
inline int qr_bulk_slots(int strips, int count) {
    const int rounds = count / 8, rest = count % 8;
    int slots = rounds * strips;
    if (rest > 0) {
        const int dies = 8 / rest;                           // the fewest dies any of the remaining matrices gets
        slots += (strips + dies - 1) / dies;
    }
    return slots;
}

template <int NBLK>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4)))
void qr_bulk_kernel(QrBulkArgs a) {
    const int die = blockIdx.x & 7, slot = blockIdx.x >> 3, strips = a.outer + a.acc;
    const int rounds = a.count >> 3, rest = a.count & 7;
    int matrix, b;
    if (slot < rounds * strips) { matrix = die + 8 * (slot / strips); b = slot % strips; }
    else {
        if (rest == 0) return;
        const int mr = die % rest;
        const int sharing = (8 - mr + rest - 1) / rest;      // dies with die % rest == mr
        matrix = 8 * rounds + mr;
        b = (slot - rounds * strips) * sharing + die / rest;
    }
    if (matrix >= a.count || b >= strips) return;
    const int64_t off = (int64_t)matrix * a.batch_stride;
    float* Cs = b < a.outer ? a.Cout + (int64_t)b * a.strip_stride : a.X + (int64_t)(b - a.outer) * a.strip_stride;
    reflect_strip_lds_body<NBLK>(a.refl, a.pending, off, Cs + off, a.nb_block);
}

// Strips of more than 160 blocks (columns of more than 2560 rows) do not fit the 128 registers of qr_bulk_kernel:
// the same pass with the strip and the reflector groups in registers (reflect_strip_body), one workgroup per
// compute unit; grid x = strip of X, grid y = matrix.
template <int NBLK>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void qr_long_strips_kernel(QrBulkArgs a) {
    const int64_t off = (int64_t)blockIdx.y * a.batch_stride;
    reflect_strip_body<NBLK, 1>(a.refl, a.pending, off, a.X + off + (int64_t)blockIdx.x * a.strip_stride, a.strip_stride, 1, a.nb_block);
}

// One launch per QR step p.  The chain of panel factorisations (one workgroup each) is the critical path, so
// the launch that follows the factorisation of panel p also factorises panel p + 1.  Panels come in blocks of
// D (delayed update): inside a block only the block's own columns see each new reflector at once; the rest of
// the matrix is read and written ONCE per block, by strips that apply the block's D reflectors in a row while
// they hold their columns in registers.  That divides the memory traffic of the factorisation, which is what
// bounds several factorisations running side by side, by almost D.
//   workgroup 0          applies reflector p to the 16 columns of panel p + 1, then factorises them;
//   `inner` workgroups   (inside a block) apply reflector p to the block's later panels and to the first panel
//                        of the next block: its columns then lack only the newest reflector when workgroup 0
//                        gets to them, as everywhere else on the chain;
//   `outer`              (a block has just been finished) apply its reflectors to the columns beyond panel p + 1.
// Every strip reads only reflectors and its own columns; panel p + 1 writes its own columns, reflector buffers
// no strip of this launch reads, and its own T: the workgroups of one launch never touch the same data.  Waves
// of workgroup 0 that the panel does not use leave after the strip.  Q is formed afterwards (householder_qr).
struct QrStepArgs {
    Reflector refl[kMaxDelay];           // the current block's reflectors so far; shift = position in the block
    int pending;                         // how many of them (the newest is refl[pending - 1], reflector p)
    int block_done;                      // panel p is the last of its block (or of the matrix)
    float* C0;                           // the columns of panel p + 1: tile (row block p, column block p + 1)
    float* Cin;                          // tile (row block p, column block p + 2): `inner` strips from here
    float* Cout;                         // tile (row block of the block's first panel, column block p + 2): `outer` strips
    int64_t strip_stride;                // floats between the tiles of neighbouring column blocks
    int nb_single, nb_block;             // rows / 16 below the first row of reflector p / of the block's first reflector
    int inner, outer;                    // strip counts
    float* Vr_next; float* Vt_next; float* Tnext; float* rdiag_next;   // outputs of panel p + 1
    int m_next;                          // its row count (0: no further panel)
    int64_t batch_stride;                // floats from one matrix's workspace to the next one's (grid y = matrix)
};

template <int NTHR, int R, int NBLK, int NS>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(NBLK >= 10 ? 2 : 4, NBLK >= 10 ? 2 : 4)))
void qr_step_kernel(QrStepArgs a) {
    const int b = blockIdx.x;
    const int64_t off = (int64_t)blockIdx.y * a.batch_stride;
    const Reflector* newest = a.refl + (a.pending - 1);
    if (b == 0) {
        if (a.m_next <= 0) return;
        {
            Reflector single = *newest; single.shift = 0;
            reflect_strip_body<NBLK, 1>(&single, 1, off, a.C0 + off, 0, 1, a.nb_single);
        }
        __threadfence_block();
        __syncthreads();                 // the strip's stores are visible to the whole workgroup
        if (threadIdx.x >= NTHR) return;
        // the panel starts one tile (16 rows) below reflector p's first row
        float* Mp = a.C0 + off + 256;
        qr_panel_body<NTHR, R>(Mp, a.Vr_next + off, a.Vt_next + off, a.Tnext + off, a.rdiag_next + off, a.m_next);
        return;
    }
    if (b <= a.inner) {
        Reflector single = *newest; single.shift = 0;
        reflect_strip_body<NBLK, 1>(&single, 1, off, a.Cin + off + (int64_t)(b - 1) * a.strip_stride, 0, 1, a.nb_single);
        return;
    }
    // the strips behind the block, NS neighbours per workgroup
    const int first = (b - 1 - a.inner) * NS, strips = a.outer - first < NS ? a.outer - first : NS;
    reflect_strip_body<NBLK, NS>(a.refl, a.pending, off, a.Cout + off + (int64_t)first * a.strip_stride, a.strip_stride, strips, a.nb_block);
}

// zeroes what lies beyond n x n of the tiled matrix M (n_pad x n_pad) and sets the tiled X to the identity
__global__ __launch_bounds__(256)
void qr_prepare_kernel(float* M, float* X, int n, int n_pad, int64_t batch_stride) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;          // index into the tiled arrays
    if (i >= (int64_t)n_pad * n_pad) return;
    M += (int64_t)blockIdx.y * batch_stride; X += (int64_t)blockIdx.y * batch_stride;
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

template <int NTHR>
hipError_t launch_qr_panel(int rows_per_thread, float* Mp, float* Vr, float* Vt, float* Tg, float* rdiag, int m,
                           int count, int64_t batch_stride, hipStream_t s) {
    switch (rows_per_thread) {
#define GELO_CASE(RR) case RR: hipLaunchKernelGGL((qr_panel_kernel<NTHR, RR>), dim3(1, count), dim3(NTHR), 0, s, Mp, Vr, Vt, Tg, rdiag, m, batch_stride); break;
        GELO_CASE(1) GELO_CASE(2) GELO_CASE(3) GELO_CASE(4) GELO_CASE(5)
        GELO_CASE(6) GELO_CASE(7) GELO_CASE(8) GELO_CASE(9) GELO_CASE(10)
#undef GELO_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int NTHR>
hipError_t launch_direct_panels(int rows_per_thread, const FactorWorkspace& ws, int nbr, int count, int64_t batch_stride, hipStream_t s) {
    switch (rows_per_thread) {
#define GELO_CASE(RR) case RR: hipLaunchKernelGGL((direct_panels_kernel<NTHR, RR>), dim3(nbr, count), dim3(NTHR), 0, s, ws.M, ws.Vc, ws.Tmat, ws.rdiag, nbr, batch_stride); break;
        GELO_CASE(1) GELO_CASE(2) GELO_CASE(3) GELO_CASE(4) GELO_CASE(5)
        GELO_CASE(6) GELO_CASE(7) GELO_CASE(8) GELO_CASE(9) GELO_CASE(10)
#undef GELO_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

#define GELO_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

}  // namespace

size_t factor_workspace_bytes(int n) {
    const int64_t n_pad = round_up(n, NB), ld = round_up(n, 64);
    const int64_t floats = 3 * n_pad * ld + n_pad * NB + 2 * n_pad * kLuBlock + n_pad + 8 * ld + 256 + 64;
    return (size_t)floats * sizeof(float) + (size_t)(n_pad + 256) * sizeof(int) + 8192;
}

void factor_workspace_carve(void* base, int n, FactorWorkspace* ws) {
    const int64_t n_pad = round_up(n, NB), ld = round_up(n, 64);
    float* p = (float*)base;
    auto take = [&](int64_t count) { float* q = p; p += round_up(count, 64); return q; };
    ws->M = take(n_pad * ld);
    ws->X = take(n_pad * ld);
    ws->Vc = take(n_pad * ld);
    ws->Tmat = take(n_pad * NB);
    ws->Dinv = take(2 * n_pad * kLuBlock);
    ws->rdiag = take(n_pad);
    ws->vec = take(8 * ld);
    ws->tri = take(128);
    ws->scalars = take(16);
    ws->perm = (int*)take(n_pad);
    ws->gat = (int*)take(128);
    ws->flag = (int*)take(16);
    ws->n_pad = (int)n_pad;
    ws->ld = ld;
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
hipError_t launch_qr_step_t(const QrStepArgs& a, int count, hipStream_t s) {
    hipLaunchKernelGGL((qr_step_kernel<NTHR, R, NBLK, 1>), dim3(1 + a.inner + a.outer, count), dim3(512), 0, s, a);
    return hipGetLastError();
}

// Can a panel with R rows per thread (NTHR threads) meet strips with NBLK blocks per wave (PREV: the next
// smaller strip variant)?  The next panel has 16 (nb_single - 1) rows and the longest strip of the launch
// nb_single .. nb_single + kMaxDelay - 1 blocks, so only a few pairs occur.
constexpr bool qr_step_pair_occurs(int NTHR, int R, int NBLK, int PREV) {
    const int min_nb = (R - 1) * NTHR / NB + 2, max_nb = R * NTHR / NB + 1 + (kMaxDelay - 1);
    return (min_nb + 7) / 8 <= NBLK && (max_nb + 7) / 8 > PREV;
}

template <int NTHR, int R>
hipError_t launch_qr_step_r(int per_wave, const QrStepArgs& a, int count, hipStream_t s) {
    if (per_wave <= 5) { if constexpr (qr_step_pair_occurs(NTHR, R, 5, 0)) return launch_qr_step_t<NTHR, R, 5>(a, count, s); }
    else if (per_wave <= 10) { if constexpr (qr_step_pair_occurs(NTHR, R, 10, 5)) return launch_qr_step_t<NTHR, R, 10>(a, count, s); }
    else if (per_wave <= 20) { if constexpr (qr_step_pair_occurs(NTHR, R, 20, 10)) return launch_qr_step_t<NTHR, R, 20>(a, count, s); }
    else if (per_wave <= 40) { if constexpr (qr_step_pair_occurs(NTHR, R, 40, 20)) return launch_qr_step_t<NTHR, R, 40>(a, count, s); }
    return hipErrorInvalidValue;
}

template <int NBLK>
hipError_t launch_qr_bulk_t(const QrBulkArgs& b, int count, hipStream_t s) {
    hipLaunchKernelGGL((qr_bulk_kernel<NBLK>), dim3(8 * qr_bulk_slots(b.outer + b.acc, count)), dim3(512), 0, s, b);
    return hipGetLastError();
}

// strips of at most 160 blocks only (20 per wave: what fits 128 registers)
constexpr int kBulkMaxBlocks = 160;
hipError_t launch_qr_bulk(const QrBulkArgs& b, int count, hipStream_t s) {
    // blocks per wave in steps of two: a strip kernel sized for 20 blocks spends a third more time on a strip of 11
    // than one sized for 12 (it still requests and waits for the blocks that do not exist)
    const int per_wave = (b.nb_block + 7) / 8;
    switch ((per_wave + 1) / 2) {
        case 0: case 1: return launch_qr_bulk_t<2>(b, count, s);
        case 2: return launch_qr_bulk_t<4>(b, count, s);
        case 3: return launch_qr_bulk_t<6>(b, count, s);
        case 4: return launch_qr_bulk_t<8>(b, count, s);
        case 5: return launch_qr_bulk_t<10>(b, count, s);
        case 6: return launch_qr_bulk_t<12>(b, count, s);
        case 7: return launch_qr_bulk_t<14>(b, count, s);
        case 8: return launch_qr_bulk_t<16>(b, count, s);
        case 9: return launch_qr_bulk_t<18>(b, count, s);
        case 10: return launch_qr_bulk_t<20>(b, count, s);
        default: break;
    }
    if (per_wave <= 40 && b.outer == 0) {
        hipLaunchKernelGGL((qr_long_strips_kernel<40>), dim3(b.acc, count), dim3(512), 0, s, b);
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

hipError_t launch_qr_step(const QrStepArgs& a, int count, hipStream_t s) {
    const int longest = (a.block_done && a.outer > 0) ? a.nb_block : a.nb_single;
    const int per_wave = (longest + 7) / 8;
    const int m = a.m_next;
    // (256 or 512 threads per panel made no difference at 2150 rows: what a column costs beyond its rows -
    // reduction, broadcast, the scalar chain - is latency, not issue slots)
    if (m <= kPanelRows256) {
        switch ((m + 255) / 256) {
            case 0: case 1: return launch_qr_step_r<256, 1>(per_wave, a, count, s);
            case 2: return launch_qr_step_r<256, 2>(per_wave, a, count, s);
            case 3: return launch_qr_step_r<256, 3>(per_wave, a, count, s);
            default: return launch_qr_step_r<256, 4>(per_wave, a, count, s);
        }
    }
    switch ((m + 511) / 512) {
        case 3: return launch_qr_step_r<512, 3>(per_wave, a, count, s);
        case 4: return launch_qr_step_r<512, 4>(per_wave, a, count, s);
        case 5: return launch_qr_step_r<512, 5>(per_wave, a, count, s);
        case 6: return launch_qr_step_r<512, 6>(per_wave, a, count, s);
        case 7: return launch_qr_step_r<512, 7>(per_wave, a, count, s);
        case 8: return launch_qr_step_r<512, 8>(per_wave, a, count, s);
        case 9: return launch_qr_step_r<512, 9>(per_wave, a, count, s);
        case 10: return launch_qr_step_r<512, 10>(per_wave, a, count, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t householder_qr(const FactorWorkspace& ws, int n, int count, int64_t batch_stride, hipStream_t s, bool direct) {
    if (count < 1 || count > 65535) return hipErrorInvalidValue;
    const int n_pad = ws.n_pad;
    const int nbr = n_pad / NB;                               // tile rows (= tile columns)
    const int64_t strip_stride = (int64_t)nbr * 256;
    const int panels = nbr;
    // Panels per block of the delayed update; the reflectors of two blocks are alive at a time (the finished
    // block is being applied while the next one's first panel is written), each n_pad x 16 in two layouts, all
    // inside the n_pad x ld floats of ws.Vc.
    const int D = ws.ld >= 64 * kMaxDelay ? kMaxDelay : (ws.ld >= 128 ? 2 : 1);
    // Every panel's reflector block is kept until the end: the row-major copies side by side in ws.Vc (n_pad x 16 each,
    // n_pad x n_pad in all), the tiled copies IN PLACE of the panels they came from (a factored panel is dead: nobody
    // reads those columns of M again, and the panel kernel has all its rows in registers before it writes).
    const int64_t set_floats = (int64_t)n_pad * NB;
    auto Vr_of = [&](int p) { return ws.Vc + (int64_t)p * set_floats; };
    auto Vt_of = [&](int p) { return ws.M + (int64_t)p * strip_stride + (int64_t)p * 256; };
    // Q is formed AFTER the factorisation, last block first: block b then only meets the columns from its own first
    // one on - the rest of H_b+1 ... H_N is still the identity there - which is 4/3 n^3 operations instead of the
    // 2 n^3 of carrying Q^T along with the factorisation.
    {
        const int64_t elems = (int64_t)n_pad * n_pad;
        hipLaunchKernelGGL(qr_prepare_kernel, dim3((unsigned)((elems + 255) / 256), count), dim3(256), 0, s, ws.M, ws.X, n, n_pad, batch_stride);
        GELO_TRY(hipGetLastError());
    }
    if (direct) {
        // every panel's reflectors from the raw columns, in one launch: nothing to factorise, no chain of panels
        const int m = n_pad;
        if (m <= kPanelRows256) GELO_TRY(launch_direct_panels<256>((m + 255) / 256, ws, nbr, count, batch_stride, s));
        else GELO_TRY(launch_direct_panels<512>((m + 511) / 512, ws, nbr, count, batch_stride, s));
    }
    // panel 0 on its own; then one launch per step
    if (!direct) {
        const int m = n_pad;
        if (m <= kPanelRows256) GELO_TRY(launch_qr_panel<256>((m + 255) / 256, ws.M, Vr_of(0), Vt_of(0), ws.Tmat, ws.rdiag, m, count, batch_stride, s));
        else GELO_TRY(launch_qr_panel<512>((m + 511) / 512, ws.M, Vr_of(0), Vt_of(0), ws.Tmat, ws.rdiag, m, count, batch_stride, s));
    }
    for (int p = 0; p < panels && !direct; ++p) {
        const int p0 = p / D * D, i = p - p0;                 // first panel of p's block, p's position in it
        const bool last = p + 1 == panels;
        const int block_end = p0 + D < panels ? p0 + D : panels;     // one past the block's last panel
        QrStepArgs a;
        a.pending = i + 1;
        for (int q = 0; q <= i; ++q) {
            a.refl[q].Vr = Vr_of(p0 + q); a.refl[q].Vt = Vt_of(p0 + q);
            a.refl[q].T = ws.Tmat + (int64_t)(p0 + q) * NB * NB; a.refl[q].shift = q; a.refl[q].plain_t = 0;
        }
        a.block_done = (p + 1 == block_end) ? 1 : 0;
        a.strip_stride = strip_stride;
        a.nb_single = nbr - p; a.nb_block = nbr - p0;
        a.C0 = last ? ws.M : ws.M + (int64_t)(p + 1) * strip_stride + (int64_t)p * 256;
        a.Cin = ws.M + (int64_t)(p + 2 < nbr ? p + 2 : 0) * strip_stride + (int64_t)p * 256;
        a.Cout = ws.M + (int64_t)(p + 2 < nbr ? p + 2 : 0) * strip_stride + (int64_t)p0 * 256;
        // the block's panels behind p + 1 and the first panel of the next block
        a.inner = a.block_done ? 0 : (block_end < nbr ? block_end : nbr - 1) - (p + 1);
        a.outer = (a.block_done && p + 2 < nbr) ? nbr - (p + 2) : 0;
        a.Vr_next = Vr_of(p + 1); a.Vt_next = Vt_of(p + 1);
        a.Tnext = ws.Tmat + (int64_t)(p + 1) * NB * NB; a.rdiag_next = ws.rdiag + (p + 1) * NB;
        a.m_next = last ? 0 : n_pad - (p + 1) * NB;
        a.batch_stride = batch_stride;
        // Several matrices side by side: the strips that apply a finished block get a launch of their own (two
        // workgroups per compute unit, which the panel's registers rule out in the step kernel).  One matrix
        // alone keeps them beside workgroup 0: there the launch count and the chain of panels are what matters.
        // Either way every column sees the same arithmetic.
        if (count >= kBulkFromCount && a.block_done && a.outer > 0 && a.nb_block <= kBulkMaxBlocks) {
            QrBulkArgs b;
            for (int q = 0; q < kMaxProduct; ++q) b.refl[q] = a.refl[q < a.pending ? q : 0];
            b.pending = a.pending; b.Cout = a.Cout; b.X = a.Cout; b.outer = a.outer; b.acc = 0;
            b.strip_stride = strip_stride; b.nb_block = a.nb_block; b.batch_stride = batch_stride; b.count = count;
            GELO_TRY(launch_qr_bulk(b, count, s));
            a.outer = 0;
            if (last) continue;                               // no panel left: the step launch would be empty
        }
        GELO_TRY(launch_qr_step(a, count, s));
    }
    {
        // X = I so far.  Block by block from the last: X[p0:, p0:] <- H_p0 (H_p0+1 (... X[p0:, p0:])), one 16-column
        // strip per workgroup, the block's reflectors newest first, each as I - V T V^T.
        // (passes of kMaxProduct reflectors where the strips fit qr_bulk_kernel; the longer strips' kernel takes kMaxDelay.
        // Columns that a pass meets before their own block's turn hold the identity below the pass's first row: the
        // reflectors beyond their block leave them as they are, bit for bit, so the grouping does not show in Q.)
        const int Dq = nbr <= kBulkMaxBlocks ? (ws.ld >= 64 * kMaxProduct ? kMaxProduct : D) : D;
        for (int p0 = (panels - 1) / Dq * Dq; p0 >= 0; p0 -= Dq) {
            const int pend = panels - p0 < Dq ? panels - p0 : Dq;
            QrBulkArgs b;
            for (int q = 0; q < kMaxProduct; ++q) {
                const int src = q < pend ? pend - 1 - q : 0;
                b.refl[q].Vr = Vr_of(p0 + src); b.refl[q].Vt = Vt_of(p0 + src);
                b.refl[q].T = ws.Tmat + (int64_t)(p0 + src) * NB * NB; b.refl[q].shift = src; b.refl[q].plain_t = 1;
            }
            b.pending = pend; b.Cout = ws.X; b.X = ws.X + (int64_t)p0 * strip_stride + (int64_t)p0 * 256;
            b.outer = 0; b.acc = nbr - p0;
            b.strip_stride = strip_stride; b.nb_block = nbr - p0; b.batch_stride = batch_stride; b.count = count;
            GELO_TRY(launch_qr_bulk(b, count, s));
        }
    }
    return hipSuccess;
}


// Brings this file's code onto the device (the runtime loads a code object on its first use, which allocates
// device memory): contexts do this when they are created, so that no later call does.
hipError_t factor_init() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&qr_prepare_kernel));
}

}  // namespace gelo
