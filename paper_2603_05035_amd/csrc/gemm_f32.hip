// float GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32), used by the
// single-precision GELO chain (Section 3.2, eqs. 1-3): C[M x N] = A[M x K] * B[K x N],
// all row-major, B optionally split into two row segments ([H ; S]); optionally C <- C - A * B.
// A tile reads all of its B columns before it stores, so with M <= 128 the product may
// overwrite B in place (C == B0, K == M): the LU path's multiplications by a diagonal-block inverse
// (those shapes take the short kernel at the end of this file, which has the same property).
//
// A workgroup of 4 waves owns a 128 x 128 tile and walks K in steps of 16
// through double-buffered LDS; a wave owns 64 x 64 as 2 x 2 accumulators.
// A lane reads four consecutive k of its A row with one 16-byte LDS read and
// spends them on four successive MFMAs; the matching B values are single
// dwords, contiguous across lanes.
#include "gelo_internal.h"

namespace gelo {
namespace {

typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int NT = 256;
constexpr int A_PITCH = BK + 4;    // floats: 80-byte rows, conflict-free 16-byte reads down a column of rows
constexpr int B_PITCH = BN + 4;

struct F32Args {
    const float* A;  int64_t lda;
    const float* B0; int64_t ldb0; int K0;
    const float* B1; int64_t ldb1;
    float* C;        int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int subtract;              // C <- C - A B (the LU's trailing and substitution updates)
};

__global__ __launch_bounds__(NT)
void gemm_f32_kernel(F32Args g) {
    __shared__ __attribute__((aligned(16))) float As[2][BM * A_PITCH];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK * B_PITCH];

    // XCD-contiguous tile runs, N fastest inside a run (A row panel stays in that XCD's L2)
    const int total = g.tiles_m * g.tiles_n;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int base = total >> 3, rem = total & 7;
    const int lid = xcd * base + (xcd < rem ? xcd : rem) + slot;
    const int tm = lid / g.tiles_n, tn = lid % g.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int j = lane & 31, grp = lane >> 5;
    const int KA = (g.K + 3) & ~3;
    const int k_tiles = (g.K + BK - 1) / BK;

    f32x4_t a_stage[2], b_stage[2];

    auto load_global = [&](int kt) {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int id = tid + i * NT;
            {   // A: 128 rows x 4 chunks
                const int r = id >> 2, c = id & 3;
                int row = m0 + r;
                row = row < g.M ? row : g.M - 1;
                const int gk = k0 + c * 4;
                f32x4_t v = {0.f, 0.f, 0.f, 0.f};
                if (gk < KA) v = *reinterpret_cast<const f32x4_t*>(g.A + (int64_t)row * g.lda + gk);
                a_stage[i] = v;
            }
            {   // B: 16 rows x 32 chunks
                const int r = id >> 5, c = id & 31;
                const int gk = k0 + r, gn = n0 + c * 4;
                f32x4_t v = {0.f, 0.f, 0.f, 0.f};
                if (gk < g.K && gn < g.N) {
                    const float* p = gk < g.K0 ? g.B0 + (int64_t)gk * g.ldb0 + gn
                                               : g.B1 + (int64_t)(gk - g.K0) * g.ldb1 + gn;
                    v = *reinterpret_cast<const f32x4_t*>(p);
                }
                b_stage[i] = v;
            }
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int id = tid + i * NT;
            *reinterpret_cast<f32x4_t*>(&As[buf][(id >> 2) * A_PITCH + (id & 3) * 4]) = a_stage[i];
            *reinterpret_cast<f32x4_t*>(&Bs[buf][(id >> 5) * B_PITCH + (id & 31) * 4]) = b_stage[i];
        }
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < k_tiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < k_tiles) load_global(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            f32x4_t a4[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                a4[mt] = *reinterpret_cast<const f32x4_t*>(
                    &As[buf][(wm * 64 + mt * 32 + j) * A_PITCH + ks * 8 + grp * 4]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float b1[2];
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    b1[nt] = Bs[buf][(ks * 8 + grp * 4 + e) * B_PITCH + wn * 64 + nt * 32 + j];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[mt][e], b1[nt], acc[mt][nt], 0, 0, 0);
            }
        }
        if (kt + 1 < k_tiles) store_lds(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int col = n0 + wn * 64 + nt * 32 + j;
            if (col < g.N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * 64 + mt * 32 + 8 * (v >> 2) + 4 * grp + (v & 3);
                    if (row < g.M) {
                        float* cp = g.C + (int64_t)row * g.ldc + col;
                        *cp = g.subtract ? *cp - acc[mt][nt][v] : acc[mt][nt][v];
                    }
                }
            }
        }
}

// M <= 128 and K <= 128 (K a multiple of 16): the LU path's multiplications by the inverse of a
// diagonal block.  One 128 x 128 tile per 128 columns would leave most of the chip idle and each
// tile bound by the float MFMA rate of its one CU, so the tiles here are 128 x 32 (four times as
// many workgroups, a wave owns 32 x 32), and with so few K steps both panels of the tile are
// fetched at once (all loads in flight together) and stored to LDS behind ONE barrier.
constexpr int SN = 32;             // tile width
constexpr int KP = 132;            // LDS pitch of the A panel, floats (conflict-free as A_PITCH is)
constexpr int SP = SN + 4;         // LDS pitch of the B panel
constexpr size_t kShortLds = ((size_t)BM * KP + (size_t)BM * SP) * sizeof(float);

__global__ __launch_bounds__(NT)
void gemm_f32_short_kernel(F32Args g) {
    extern __shared__ __attribute__((aligned(16))) float panels[];
    float* As = panels;                 // [row][k]
    float* Bs = panels + BM * KP;       // [k][col]
    const int n0 = blockIdx.x * SN;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, grp = lane >> 5;
    const int kc = g.K >> 2;            // 16-byte chunks per A row

    f32x4_t a_st[16], b_st[4];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int id = tid + i * NT;
        const int r = id / kc, c = id - r * kc;
        const int row = r < g.M ? r : g.M - 1;
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
        if (r < BM) v = *reinterpret_cast<const f32x4_t*>(g.A + (int64_t)row * g.lda + c * 4);
        a_st[i] = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + i * NT;
        const int r = id >> 3, c = id & 7;
        const int gn = n0 + c * 4;
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
        if (r < g.K && gn < g.N) v = *reinterpret_cast<const f32x4_t*>(g.B0 + (int64_t)r * g.ldb0 + gn);
        b_st[i] = v;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int id = tid + i * NT;
        const int r = id / kc, c = id - r * kc;
        if (r < BM) *reinterpret_cast<f32x4_t*>(&As[r * KP + c * 4]) = a_st[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + i * NT;
        *reinterpret_cast<f32x4_t*>(&Bs[(id >> 3) * SP + (id & 7) * 4]) = b_st[i];
    }
    __syncthreads();

    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const int k_steps = g.K >> 3;
    for (int ks = 0; ks < k_steps; ++ks) {
        const f32x4_t a4 = *reinterpret_cast<const f32x4_t*>(&As[(wave * 32 + j) * KP + ks * 8 + grp * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[e], Bs[(ks * 8 + grp * 4 + e) * SP + j], acc, 0, 0, 0);
    }
    const int col = n0 + j;
    if (col < g.N) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = wave * 32 + 8 * (v >> 2) + 4 * grp + (v & 3);
            if (row < g.M) {
                float* cp = g.C + (int64_t)row * g.ldc + col;
                *cp = g.subtract ? *cp - acc[v] : acc[v];
            }
        }
    }
}

}  // namespace

hipError_t gemm_f32_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_f32_short_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kShortLds);
}

hipError_t gemm_f32(const GemmOperands& o, hipStream_t stream) {
    if (o.M <= 0 || o.N <= 0 || o.K <= 0) return hipSuccess;
    F32Args a;
    a.A = (const float*)o.A;   a.lda = o.lda;
    a.B0 = (const float*)o.B0; a.ldb0 = o.ldb0; a.K0 = o.K0;
    a.B1 = (const float*)o.B1; a.ldb1 = o.ldb1;
    a.C = (float*)o.C;         a.ldc = o.ldc;
    a.M = o.M; a.N = o.N; a.K = o.K;
    a.tiles_m = (o.M + BM - 1) / BM;
    a.tiles_n = (o.N + BN - 1) / BN;
    a.subtract = o.subtract ? 1 : 0;
    if (o.M <= BM && o.K <= 128 && o.K % 16 == 0 && o.K0 >= o.K)
        hipLaunchKernelGGL(gemm_f32_short_kernel, dim3((o.N + SN - 1) / SN), dim3(NT), kShortLds, stream, a);
    else
        hipLaunchKernelGGL(gemm_f32_kernel, dim3(a.tiles_m * a.tiles_n), dim3(NT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace gelo
