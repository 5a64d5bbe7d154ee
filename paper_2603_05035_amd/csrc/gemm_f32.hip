// float GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32), used by the
// single-precision GELO chain (Section 3.2, eqs. 1-3): C[M x N] = A[M x K] * B[K x N],
// all row-major, B optionally split into two row segments ([H ; S]); optionally C <- C - A * B.
// A tile reads all of its B columns before it stores, so with M <= 128 the product may
// overwrite B in place (C == B0, K == M): the LU path's multiplications by a diagonal-block inverse
// (those shapes take the short kernel at the end of this file, which has the same property).
//
// A workgroup of 4 waves owns a 128 x 96, 128 x 128 or 128 x 192 tile (whichever fills whole
// rounds of the chip's CUs best) and walks K in steps of 32 through double-buffered LDS.  A lane
// reads four consecutive k of its A row with one 16-byte LDS read and spends them on four
// successive MFMAs; the matching B values are single dwords, contiguous across lanes; the
// fragments of the next 8 k are read while the MFMAs of the current 8 run.
#include "gelo_internal.h"

namespace gelo {
namespace {

typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BK = 32;
constexpr int NT = 256;
constexpr int A_PITCH = BK + 4;    // floats: 144-byte rows, conflict-free 16-byte reads down a column of rows

struct F32Args {
    const float* A;  int64_t lda;
    const float* B0; int64_t ldb0; int K0;
    const float* B1; int64_t ldb1;
    float* C;        int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int subtract;              // C <- C - A B (the LU's trailing and substitution updates)
};

// BN = 96, 128 or 192: the tile width is picked per shape so that the tile count fills whole rounds of the chip's CUs.
// WAVES_M x (4 / WAVES_M) waves: 2 x 2 for the wide tiles, 4 x 1 (a wave owns 32 rows x 96 columns) for the narrow one,
// whose LDS footprint lets two workgroups share a CU and cover each other's barrier and LDS-store phases.
template <int BN, int WAVES_M>
__global__ __launch_bounds__(NT)
void gemm_f32_kernel(F32Args g) {
    constexpr int B_PITCH = BN + 4;
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int WROWS = BM / WAVES_M, WCOLS = BN / WAVES_N;
    constexpr int MTM = WROWS / 32;              // 32-row MFMA blocks per wave
    constexpr int NTN = WCOLS / 32;              // 32-column MFMA blocks per wave
    constexpr int BCH = BN / 4;                  // 16-byte chunks per B row
    constexpr int BLD = BK * BCH / NT;           // B chunks per thread and K step
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
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int j = lane & 31, grp = lane >> 5;
    const int KA = (g.K + 3) & ~3;
    const int k_tiles = (g.K + BK - 1) / BK;

    // the arguments the loads need, by value (scalar registers)
    const float* B0 = g.B0;
    const float* B1 = g.B1;
    const int64_t ldb0 = g.ldb0, ldb1 = g.ldb1;
    const int K0 = g.K0, Kd = g.K, Nd = g.N;

    f32x4_t a_stage[4], b_stage[BLD];

    auto load_global = [&](int kt) {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + i * NT;
            {   // A: 128 rows x 8 chunks
                const int r = id >> 3, c = id & 7;
                int row = m0 + r;
                row = row < g.M ? row : g.M - 1;
                const int gk = k0 + c * 4;
                f32x4_t v = {0.f, 0.f, 0.f, 0.f};
                if (gk < KA) v = *reinterpret_cast<const f32x4_t*>(g.A + (int64_t)row * g.lda + gk);
                a_stage[i] = v;
            }
        }
        // B: 32 rows x BN / 4 chunks.  A K step that lies in one row segment of B (the common case) takes its
        // base pointer from scalar registers; picking B0 or B1 per lane makes the compiler fetch the pointer
        // itself from the argument block with a vector load, one exposed memory latency per chunk.
        const bool seg0 = k0 + BK <= K0, seg1 = k0 >= K0;
        if (seg0 || seg1) {
            const float* base = seg0 ? B0 + (int64_t)k0 * ldb0 : B1 + (int64_t)(k0 - K0) * ldb1;
            const int64_t ldb = seg0 ? ldb0 : ldb1;
#pragma unroll
            for (int i = 0; i < BLD; ++i) {
                const int id = tid + i * NT;
                const int r = id / BCH, c = id - r * BCH;
                const int gn = n0 + c * 4;
                f32x4_t v = {0.f, 0.f, 0.f, 0.f};
                if (k0 + r < Kd && gn < Nd) v = *reinterpret_cast<const f32x4_t*>(base + (int64_t)r * ldb + gn);
                b_stage[i] = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < BLD; ++i) {
                const int id = tid + i * NT;
                const int r = id / BCH, c = id - r * BCH;
                const int gk = k0 + r, gn = n0 + c * 4;
                const bool first = gk < K0;
                const int64_t off = first ? (int64_t)gk * ldb0 : (int64_t)(gk - K0) * ldb1;
                f32x4_t v = {0.f, 0.f, 0.f, 0.f};
                if (gk < Kd && gn < Nd) {
                    if (first) v = *reinterpret_cast<const f32x4_t*>(B0 + off + gn);
                    else v = *reinterpret_cast<const f32x4_t*>(B1 + off + gn);
                }
                b_stage[i] = v;
            }
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + i * NT;
            *reinterpret_cast<f32x4_t*>(&As[buf][(id >> 3) * A_PITCH + (id & 7) * 4]) = a_stage[i];
        }
#pragma unroll
        for (int i = 0; i < BLD; ++i) {
            const int id = tid + i * NT;
            const int r = id / BCH, c = id - r * BCH;
            *reinterpret_cast<f32x4_t*>(&Bs[buf][r * B_PITCH + c * 4]) = b_stage[i];
        }
    };

    f32x16_t acc[MTM][NTN];
#pragma unroll
    for (int a = 0; a < MTM; ++a)
#pragma unroll
        for (int b = 0; b < NTN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < k_tiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < k_tiles) load_global(kt + 1);
        // fragments of sub-step ks + 1 are read while the 16 MFMAs of sub-step ks run
        f32x4_t a4[2][MTM];
        float b1[2][4][NTN];
        auto load_frags = [&](int fb, int ks) {
#pragma unroll
            for (int mt = 0; mt < MTM; ++mt)
                a4[fb][mt] = *reinterpret_cast<const f32x4_t*>(
                    &As[buf][(wm * WROWS + mt * 32 + j) * A_PITCH + ks * 8 + grp * 4]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int nt = 0; nt < NTN; ++nt)
                    b1[fb][e][nt] = Bs[buf][(ks * 8 + grp * 4 + e) * B_PITCH + wn * WCOLS + nt * 32 + j];
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 8; ++ks) {
            const int fb = ks & 1;
            if (ks + 1 < BK / 8) load_frags(fb ^ 1, ks + 1);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int mt = 0; mt < MTM; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NTN; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[fb][mt][e], b1[fb][e][nt], acc[mt][nt], 0, 0, 0);
        }
        if (kt + 1 < k_tiles) store_lds(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int mt = 0; mt < MTM; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTN; ++nt) {
            const int col = n0 + wn * WCOLS + nt * 32 + j;
            if (col < g.N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * WROWS + mt * 32 + 8 * (v >> 2) + 4 * grp + (v & 3);
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
    a.subtract = o.subtract ? 1 : 0;
    if (o.M <= BM && o.K <= 128 && o.K % 16 == 0 && o.K0 >= o.K) {
        a.tiles_n = (o.N + SN - 1) / SN;
        hipLaunchKernelGGL(gemm_f32_short_kernel, dim3(a.tiles_n), dim3(NT), kShortLds, stream, a);
        return hipGetLastError();
    }
    // Tile width.  Large K: 128 x 96 tiles, two workgroups per CU (cost: rounds of 512 tiles), unless a wider
    // tile wastes less of its last round over the 256 CUs; short K (the LU's updates, bound by the
    // read-modify-write of C): the wide tiles only.
    constexpr int kCus = 256;
    auto tiles = [&](int bn) { return a.tiles_m * ((o.N + bn - 1) / bn); };
    const int64_t cost96 = (int64_t)((tiles(96) + 2 * kCus - 1) / (2 * kCus)) * 2 * 96 * 85 / 100;      // measured: 15% faster per flop
    const int64_t cost128 = (int64_t)((tiles(128) + kCus - 1) / kCus) * 128, cost192 = (int64_t)((tiles(192) + kCus - 1) / kCus) * 192;
    if (o.K >= 512 && cost96 <= cost128 && cost96 <= cost192) {
        a.tiles_n = (o.N + 95) / 96;
        hipLaunchKernelGGL((gemm_f32_kernel<96, 4>), dim3(a.tiles_m * a.tiles_n), dim3(NT), 0, stream, a);
    } else if (cost192 < cost128) {
        a.tiles_n = (o.N + 191) / 192;
        hipLaunchKernelGGL((gemm_f32_kernel<192, 2>), dim3(a.tiles_m * a.tiles_n), dim3(NT), 0, stream, a);
    } else {
        a.tiles_n = (o.N + 127) / 128;
        hipLaunchKernelGGL((gemm_f32_kernel<128, 2>), dim3(a.tiles_m * a.tiles_n), dim3(NT), 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace gelo
