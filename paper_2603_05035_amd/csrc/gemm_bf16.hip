// bf16 x bf16 -> bf16 GEMM with fp32 accumulation on the gfx950 matrix cores.
//
// One kernel serves the three products of the GELO chain (Section 3.2, eqs. 1-3):
// mix U = A [H;S], project Y = U W and unmix Z = A^-1 Y.  All operands are
// row-major, so the right-hand operand arrives with the contraction index as
// its slow axis; the kernel turns 8x4 register blocks of it around with byte
// permutes to feed v_mfma_f32_32x32x16_bf16, whose lanes want 8 consecutive
// contraction elements each.
//
// Work decomposition: a workgroup owns a BM x BN tile of C and walks K in
// steps of 64 through a double-buffered LDS stage; a wave owns WM x 128 of the
// tile as (WM/32) x 4 accumulators of 32 x 32.  The four accumulators along N
// are column-interleaved (lane j of accumulator c holds column 4j + c), which
// makes both the LDS reads of B (8 bytes per lane) and the stores of C (4
// bf16 per lane and row) contiguous across lanes.
#include "gelo_internal.h"

namespace gelo {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BK = 64;
constexpr int WN = 128;
constexpr int A_PITCH = BK + 8;   // bf16 elements; 144-byte rows keep 16-byte row reads conflict-free

struct Bf16Args {
    const uint16_t* A;  int64_t lda;
    const uint16_t* B0; int64_t ldb0; int K0;
    const uint16_t* B1; int64_t ldb1;
    uint16_t* C;        int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int narrow_cols = 0;        // mixed-width launch only: tile columns of width 192 after tiles_n columns of width 256
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v = {(__bf16)lo, (__bf16)hi};      // round-to-nearest-even
    return __builtin_bit_cast(uint32_t, v);
}

// Workgroups are dealt to the 8 XCDs round-robin; give each XCD (own L2) a contiguous run of
// tiles, and inside a run walk a group of tile-rows before moving along N so that tiles in flight
// share A row panels and B column panels.  The tile-rows are split into equal groups of at most 8
// (9 rows -> 5 + 4, not 8 + 1): a short last group would hand one XCD a whole row of tiles, i.e.
// all of B.  Measured on the 2150 x 12288 x 4096 projection, L2 fills drop from 474 MB to 376 MB
// per launch; the run time does not change (the fills are served at a fraction of peak bandwidth).
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int* tm, int* tn) {
    const int total = tiles_m * tiles_n;
    const int xcd = bid & 7, slot = bid >> 3;
    const int base = total >> 3, rem = total & 7;
    const int lid = xcd * base + (xcd < rem ? xcd : rem) + slot;
    const int groups = (tiles_m + 7) >> 3;
    const int group_m = (tiles_m + groups - 1) / groups;
    const int per_group = group_m * tiles_n;
    const int group = lid / per_group;
    const int first_m = group * group_m;
    const int gsz = (tiles_m - first_m) < group_m ? (tiles_m - first_m) : group_m;
    const int in_group = lid - group * per_group;
    *tm = first_m + in_group % gsz;
    *tn = in_group / gsz;
}

template <int BM, int BN, int WM>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64)
void gemm_bf16_kernel(Bf16Args g) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * WAVES_N * 64;
    constexpr int MT = WM / 32;
    constexpr int A_TILE = BM * A_PITCH;
    constexpr int B_TILE = BK * BN;
    constexpr int A_CHUNKS = BM * (BK / 8) / NT;
    constexpr int B_CHUNKS = BK * (BN / 8) / NT;
    static_assert(BM * (BK / 8) % NT == 0 && BK * (BN / 8) % NT == 0, "tile / thread mismatch");

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* As = smem;
    uint16_t* Bs = smem + 2 * A_TILE;

    int tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int j = lane & 31, grp = lane >> 5;
    const int KA = (g.K + 7) & ~7;
    const int k_tiles = (g.K + BK - 1) / BK;
    const bool n_full = n0 + BN <= g.N;

    // per-thread element offsets of the chunks it stages (rows clamped into the matrix)
    int a_off[A_CHUNKS], a_lds[A_CHUNKS], b_row[B_CHUNKS], b_col[B_CHUNKS], b_lds[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        const int id = tid + i * NT;
        const int r = id >> 3, c = id & 7;
        int row = m0 + r;
        row = row < g.M ? row : g.M - 1;
        a_off[i] = row * (int)g.lda + c * 8;
        a_lds[i] = r * A_PITCH + c * 8;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
        const int id = tid + i * NT;
        b_row[i] = id / (BN / 8);
        b_col[i] = n0 + (id % (BN / 8)) * 8;
        b_lds[i] = b_row[i] * BN + (id % (BN / 8)) * 8;
    }

    u32x4_t a_stage[A_CHUNKS], b_stage[B_CHUNKS];

    auto load_global = [&](int kt) {
        const int k0 = kt * BK;
        const bool fast = n_full && (k0 + BK <= g.K) && (k0 + BK <= g.K0 || k0 >= g.K0);
        if (fast) {
            const uint16_t* ap = g.A + k0;
            const uint16_t* bp; int64_t ldb;
            if (k0 < g.K0) { bp = g.B0 + (int64_t)k0 * g.ldb0; ldb = g.ldb0; }
            else { bp = g.B1 + (int64_t)(k0 - g.K0) * g.ldb1; ldb = g.ldb1; }
#pragma unroll
            for (int i = 0; i < A_CHUNKS; ++i) a_stage[i] = *reinterpret_cast<const u32x4_t*>(ap + a_off[i]);
#pragma unroll
            for (int i = 0; i < B_CHUNKS; ++i) b_stage[i] = *reinterpret_cast<const u32x4_t*>(bp + b_row[i] * ldb + b_col[i]);
        } else {
#pragma unroll
            for (int i = 0; i < A_CHUNKS; ++i) {
                const int c8 = ((tid + i * NT) & 7) * 8;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (k0 + c8 < KA) v = *reinterpret_cast<const u32x4_t*>(g.A + k0 + a_off[i]);
                a_stage[i] = v;
            }
#pragma unroll
            for (int i = 0; i < B_CHUNKS; ++i) {
                const int gk = k0 + b_row[i], gn = b_col[i];
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (gk < g.K && gn < g.N) {
                    const uint16_t* p = gk < g.K0 ? g.B0 + (int64_t)gk * g.ldb0 + gn
                                                  : g.B1 + (int64_t)(gk - g.K0) * g.ldb1 + gn;
                    v = *reinterpret_cast<const u32x4_t*>(p);
                }
                b_stage[i] = v;
            }
        }
    };
    auto store_lds = [&](int buf) {
        uint16_t* as = As + buf * A_TILE;
        uint16_t* bs = Bs + buf * B_TILE;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<u32x4_t*>(as + a_lds[i]) = a_stage[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<u32x4_t*>(bs + b_lds[i]) = b_stage[i];
    };

    f32x16_t acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0.f;

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < k_tiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < k_tiles) load_global(kt + 1);

        const uint16_t* as = As + buf * A_TILE + (wm * WM + j) * A_PITCH + grp * 8;
        const uint16_t* bs = Bs + buf * B_TILE + (grp * 8) * BN + wn * WN + 4 * j;

        bf16x8_t a_frag[2][MT];
        u32x2_t b_raw[2][8];
        auto load_frags = [&](int fb, int ks) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                a_frag[fb][mt] = *reinterpret_cast<const bf16x8_t*>(as + mt * 32 * A_PITCH + ks * 16);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                b_raw[fb][i] = *reinterpret_cast<const u32x2_t*>(bs + (ks * 16 + i) * BN);
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int fb = ks & 1;
            if (ks + 1 < BK / 16) load_frags(fb ^ 1, ks + 1);     // next step's fragments fly under this step's MFMAs
            bf16x8_t b_frag[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                u32x4_t t;
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    t[m] = __builtin_amdgcn_perm(b_raw[fb][2 * m + 1][c >> 1], b_raw[fb][2 * m][c >> 1], sel);
                b_frag[c] = __builtin_bit_cast(bf16x8_t, t);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[mt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_frag[fb][mt], b_frag[c], acc[mt][c], 0, 0, 0);
        }

        if (kt + 1 < k_tiles) store_lds(buf ^ 1);
        __syncthreads();
    }

    const int col = n0 + wn * WN + 4 * j;
    if (col < g.N) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * WM + mt * 32 + 8 * (v >> 2) + 4 * grp + (v & 3);
                if (row < g.M) {
                    u32x2_t out;
                    out[0] = pack_bf16x2(acc[mt][0][v], acc[mt][1][v]);
                    out[1] = pack_bf16x2(acc[mt][2][v], acc[mt][3][v]);
                    *reinterpret_cast<u32x2_t*>(g.C + (int64_t)row * g.ldc + col) = out;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Fast path: 256 x BN tile (BN = 256 or 192), 8 waves (wave tile 64 x BN/2), K step 64, two LDS
// stages filled by direct-to-LDS loads (global_load_lds_dwordx4: no staging registers, no
// ds_write), one barrier per K step.
//   A rows (128 bytes per stage) keep their 16-byte chunks XOR-swizzled so that the 16-byte
//     fragment reads of 16 consecutive rows hit distinct banks.
//   B rows (2 BN bytes, K-major as in memory) are read with ds_read_b64_tr_b16, which hands every
//     lane the four K-consecutive values of one column: the MFMA operand layout, with no
//     permutes.  The 16-byte chunks of a row are permuted (XOR for BN = 256, rotation for
//     BN = 192, see b_chunk_pos) so that the four rows one transposing read touches are spread
//     over all banks (measured: zero conflicts in the main loop).
//   The MFMA operands are swapped (B fragment first), so the accumulators hold blocks of C^T and a
//     lane owns 4 consecutive columns of one row; the epilogue goes through LDS once more so that
//     the global stores are 16 bytes per lane over whole row segments.
// Out-of-range rows of A and columns of B are clamped to valid addresses (their products land in
// outputs that are never stored); rows of B beyond K are fetched from a block of zeros and A is zero
// in columns [K, round_up(K, 64)) (required by the dispatcher), so the K tail contributes exact zeros
// whatever the data holds.  Measured on the 2150 x 12288 x 4096 projection against the
// alternatives that were tried: K step 32 with four stages and prefetch distance 3 (-4 %),
// per-lane address arithmetic for the fetches (-5 %), v_perm transposition of B in registers
// with direct stores (-9 %).  BN = 192 exists for the tile count: 2048 x 12288 is 384 tiles of
// 256 x 256 (1.5 rounds on 256 CUs, so 2) but 512 of 256 x 192 (exactly 2 rounds of 0.87 the cost).
namespace dma {

constexpr int BM = 256, BKS = 64, STAGES = 2;
constexpr int A_BYTES = BM * BKS * 2;           // 32 KB per stage, rows of 128 B
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
template <int BN> constexpr int lds_bytes() { return STAGES * (A_BYTES + BKS * BN * 2); }

// sixteen zero bytes: what the rows of B beyond the contraction length are fetched from, so that a NaN or
// Inf in the last valid row cannot reach the accumulators through 0 x Inf
__device__ __align__(16) const uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};

// lds_addr must be wave-uniform (it travels in M0); lane l's 16 bytes land at lds_addr + 16 l
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(gptr), "s"(lds_addr) : "memory", "m0");
}

// position (in 16-byte chunks) of chunk c of B row r inside the row, and its inverse.  BN = 256: rows r .. r + 3
// of a transposing read differ in bits 1-2 of the 32-byte unit; BN = 192 (row pitch 384 bytes = 1.5 bank rounds):
// rows r + 2, r + 3 are rotated by 64 bytes, which puts the four 64-byte spans on the four quarters of the banks.
template <int BN> __device__ __forceinline__ int b_chunk_pos(int r, int c) {
    if (BN == 256) return c ^ ((((r & 3) << 1) | ((r >> 3) & 1)) << 1);
    const int p = c + 4 * ((r >> 1) & 1);
    return p >= BN / 8 ? p - BN / 8 : p;
}
template <int BN> __device__ __forceinline__ int b_chunk_of_pos(int r, int pos) {
    if (BN == 256) return pos ^ ((((r & 3) << 1) | ((r >> 3) & 1)) << 1);
    const int c = pos - 4 * ((r >> 1) & 1);
    return c < 0 ? c + BN / 8 : c;
}

template <int BN>
__device__ __forceinline__ void tile_body(const Bf16Args& g, uint8_t* lds, int m0, int n0) {
    constexpr int NCT = BN / 64;
    constexpr int ROWB = BN * 2;
    constexpr int B_BYTES = BKS * ROWB;
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int NBD = B_BYTES / 8192;
    constexpr int CPR = ROWB / 16;
    constexpr int EPI_PITCH = BN + 16;
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)lds);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int j = lane & 31, grp = lane >> 5;
    auto uni32 = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    auto uni64 = [&](int64_t x) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((int)(uint32_t)x), hi = __builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    const int K = uni32(g.K), K0 = uni32(g.K0);
    const int T = (K + BKS - 1) / BKS;
    const int64_t ldb0 = uni64(g.ldb0), ldb1 = uni64(g.ldb1);
    const uint16_t* B0p = (const uint16_t*)uni64((int64_t)g.B0);
    const uint16_t* B1p = (const uint16_t*)uni64((int64_t)g.B1);

    const uint16_t* a_src[4];
    const uint16_t* b0_src[NBD];
    const uint16_t* b1_src[NBD];
    int b_krow[NBD], b_gn[NBD];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int blk = wave * 4 + i;
        const int row = blk * 8 + (lane >> 3), cp = lane & 7;
        const int c = cp ^ ((row ^ (row >> 3)) & 7);
        int grow = m0 + row; grow = grow < g.M ? grow : g.M - 1;
        a_src[i] = g.A + (int64_t)grow * g.lda + c * 8;
    }
#pragma unroll
    for (int i = 0; i < NBD; ++i) {
        const int e = (wave * NBD + i) * 64 + lane;             // 16-byte unit of the B stage this lane fills
        const int br = e / CPR, cpos = e - br * CPR;
        const int bc = b_chunk_of_pos<BN>(br, cpos);
        int gn = n0 + bc * 8; gn = gn < g.N ? gn : g.N - 8;
        b_krow[i] = br; b_gn[i] = gn;
        b0_src[i] = B0p + (int64_t)br * ldb0 + gn;
        b1_src[i] = B1p + (int64_t)(br - K0) * ldb1 + gn;
    }

    auto issue = [&](int t) {
        const int k0 = t * BKS;
        const uint32_t st = lds_base + (t & 1) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16(a_src[i] + k0, st + (wave * 4 + i) * 1024);
        const uint32_t sb = st + A_BYTES + wave * NBD * 1024;
        if (k0 + BKS <= K0) {
            const int64_t off = (int64_t)k0 * ldb0;
#pragma unroll
            for (int i = 0; i < NBD; ++i) dma16(b0_src[i] + off, sb + i * 1024);
        } else if (k0 >= K0 && k0 + BKS <= K) {
            const int64_t off = (int64_t)k0 * ldb1;
#pragma unroll
            for (int i = 0; i < NBD; ++i) dma16(b1_src[i] + off, sb + i * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < NBD; ++i) {
                int gk = k0 + b_krow[i];
                const bool beyond = gk >= K;                      // rows past the contraction length read zeros
                gk = beyond ? K - 1 : gk;
                const bool first = gk < K0;
                const uint16_t* base = first ? B0p : B1p;
                const int64_t off = first ? (int64_t)gk * ldb0 : (int64_t)(gk - K0) * ldb1;
                dma16(beyond ? (const uint16_t*)g_zero16 : base + off + b_gn[i], sb + i * 1024);
            }
        }
    };

    const int a_row0 = wm * 64 + j;
    const int a_sw = (j ^ (j >> 3)) & 7;
    const uint32_t a_frag_off0 = a_row0 * 128;
    const int s16 = lane & 15, G = lane >> 4;
    const int kg = G >> 1, nh = G & 1;
    const int rl = kg * 8 + (s16 >> 2);                          // row of the first read; later reads add multiples of 4
    uint32_t b_off[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int m = wn * (NCT * 2) + ct * 2 + nh;
        b_off[ct] = A_BYTES + rl * ROWB + b_chunk_pos<BN>(rl, 2 * m) * 16 + (s16 & 3) * 8;
    }

    f32x16_t acc[2][NCT];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int c = 0; c < NCT; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0.f;

    constexpr bool DEFER = BN == 256;
    bf16x8_t a_frag[2][2];
    bf16x8_t b_frag[2][NCT];
    auto mfma_group = [&](int fb) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int c = 0; c < NCT; ++c)
                acc[mt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b_frag[fb][c], a_frag[fb][mt], acc[mt][c], 0, 0, 0);
    };

    issue(0);
    for (int t = 0; t < T; ++t) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        // The two waves of a SIMD (w and w + 4) would otherwise both spend the start of the K step issuing
        // fetches while the matrix pipe idles: with the wide tile the second one issues after its first two
        // MFMA groups instead (measured +3 %; no gain with the narrow tile).
        constexpr bool STAGGER = BN == 256;
        if ((!STAGGER || wave < 4) && t + 1 < T) issue(t + 1);
        const uint8_t* st = lds + (t & 1) * STAGE_BYTES;
        auto load_frags = [&](int fb, int ks) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                a_frag[fb][mt] = *reinterpret_cast<const bf16x8_t*>(st + a_frag_off0 + mt * 32 * 128 + (((ks * 2 + grp) ^ a_sw ^ (mt * 4)) * 16));
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(st + b_off[ct] + ks * 16 * ROWB));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(st + b_off[ct] + ks * 16 * ROWB + 4 * ROWB));
                const s16x8_t both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                b_frag[fb][ct] = __builtin_bit_cast(bf16x8_t, both);
            }
        };
        if (DEFER) {
            // The matrix instructions of a K step's last fragment group wait until the next barrier has been
            // passed: behind it every wave then has NCT * 2 of them ready in registers while the first fragments
            // of the new stage are still on their way from LDS (the stage they came from is free to be refilled:
            // its last fragments were read before the barrier).  Measured +2 ... 9 % with the wide tile, nothing
            // with the narrow one.
            load_frags(0, 0);
            if (t > 0) mfma_group(1);
            load_frags(1, 1);
            mfma_group(0);
            if (STAGGER && wave >= 4 && t + 1 < T) issue(t + 1);
            load_frags(0, 2);
            mfma_group(1);
            load_frags(1, 3);
            mfma_group(0);
        } else {
            load_frags(0, 0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int fb = ks & 1;
                if (ks + 1 < 4) load_frags(fb ^ 1, ks + 1);
                mfma_group(fb);
                if (STAGGER && wave >= 4 && ks == 1 && t + 1 < T) issue(t + 1);
            }
        }
    }
    if (DEFER) mfma_group(1);

    __builtin_amdgcn_s_barrier();
    uint8_t* patch = lds + wave * (32 * EPI_PITCH);
    const int rr = lane >> 4, cc = lane & 15;
    const int col = n0 + wn * (BN / 2) + cc * 8;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2_t out;
                out[0] = pack_bf16x2(acc[mt][ct][4 * q], acc[mt][ct][4 * q + 1]);
                out[1] = pack_bf16x2(acc[mt][ct][4 * q + 2], acc[mt][ct][4 * q + 3]);
                *reinterpret_cast<u32x2_t*>(patch + j * EPI_PITCH + (ct * 32 + 8 * q + 4 * grp) * 2) = out;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (cc < BN / 16) {
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int r = it * 4 + rr;
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(patch + r * EPI_PITCH + cc * 16);
                const int row = m0 + wm * 64 + mt * 32 + r;
                if (row < g.M && col < g.N) *reinterpret_cast<u32x4_t*>(g.C + (int64_t)row * g.ldc + col) = v;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

template <int BN>
__global__ __launch_bounds__(512)
void gemm_bf16_dma_kernel(Bf16Args g) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    int tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, &tm, &tn);
    tile_body<BN>(g, lds, tm * BM, tn * BN);
}

// Both tile widths in one launch: tiles_n columns of 256-wide tiles first (low block ids start first),
// then narrow_cols columns of 192-wide tiles.  For a tile count between one and two rounds of the
// chip's CUs this ends after one wide plus one narrow tile time instead of two wide ones.
__global__ __launch_bounds__(512)
void gemm_bf16_dma_mixed_kernel(Bf16Args g) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int wide_tiles = g.tiles_m * g.tiles_n;
    int tm, tn;
    if ((int)blockIdx.x < wide_tiles) {
        tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, &tm, &tn);
        tile_body<256>(g, lds, tm * BM, tn * 256);
    } else {
        tile_of_block(blockIdx.x - wide_tiles, g.tiles_m, g.narrow_cols, &tm, &tn);
        tile_body<192>(g, lds, tm * BM, g.tiles_n * 256 + tn * 192);
    }
}

// Several independent products of at most one tile row each in one launch: grid y picks the product (its
// arguments travel by value), grid x its tile.
struct Bf16Batch { Bf16Args g[kGemmBatchMax]; };

template <int BN>
__global__ __launch_bounds__(512)
void gemm_bf16_dma_batched_kernel(Bf16Batch b) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const Bf16Args& g = b.g[blockIdx.y];
    if ((int)blockIdx.x >= g.tiles_m * g.tiles_n) return;
    int tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, &tm, &tn);
    tile_body<BN>(g, lds, tm * BM, tn * BN);
}

}  // namespace dma

// ---------------------------------------------------------------------------------------------
// Skinny path (M <= 128: decode-shaped batches).  The product is bound by streaming B once.  A
// workgroup takes ALL rows and BN = 32 NCT columns; K steps of 64 run through a ring of LDS stages
// filled by the same direct-to-LDS loads as the fast path (whole 128-byte lines of A and B).  The
// CONTRACTION of a K step is split over the four waves: wave w multiplies rows 16 w .. 16 w + 15 of
// B's stage with the matching 32 bytes of every row of A, so nothing is read from LDS twice (with the
// rows split over the waves instead, every wave read all of B and the reads took as long as the
// fetches).  One barrier per K step; the fragments of step t + 1 are read while the matrix
// instructions of step t run.  Rows of A beyond M are not fetched (their lanes are masked; what the
// matrix cores make of the stale LDS words lands in rows that are never stored).  The four partial
// sums meet in LDS after the loop and are added in wave order.
//
// Two shapes of launch.  Measured on MI355X, one CU streams at most 26 - 28 GB/s from HBM whatever
// the depth of its ring (3 to 13 stages made no difference, nor did a panel-contiguous copy of B),
// and every byte of A a CU fetches (all of A, once per workgroup) counts against the same limit:
// 68 x 12288 x 4096 took 30 us on 192 workgroups of 64 columns, 20 us with 8 rows.
//  - NCT = 2 (64 columns), all of K per workgroup: no workspace, any shape.
//  - NCT = 6 (192 columns = three whole 128-byte lines per row of B), K cut into `slices` ranges of
//    K steps so that columns x slices fills the chip: every CU streams its share of B and only
//    1 / slices of A.  The workgroups write float partial sums; a second small kernel adds them in
//    slice order (fixed order, no atomics) and rounds to bf16.
namespace skinny {

constexpr int BKS = 64, NWAVES = 4, KW = BKS / NWAVES;
constexpr int EPI_COLS = 64, EPI_PITCH = EPI_COLS + 4;           // floats; 272-byte rows: 16-byte writes of 16 rows hit distinct banks

template <int RT, int NCT> struct Cfg {                          // RT = row tiles of 32, NCT = column tiles of 32
    static constexpr int BN = 32 * NCT;
    static constexpr int ROWB = BN * 2, CPR = ROWB / 16;         // bytes / 16-byte chunks per row of B's stage
    static constexpr int NBD = BKS * ROWB / 1024 / NWAVES;       // B fetches per wave and K step
    static constexpr int PER = RT + NBD;                         // fetches per wave and K step
    static constexpr int A_BYTES = RT * 32 * 128;
    static constexpr int STAGE_BYTES = A_BYTES + BKS * ROWB;
    static constexpr int STAGES_LDS = (156 * 1024) / STAGE_BYTES;              // what fits in LDS
    static constexpr int STAGES_CNT = 63 / PER + 1;                            // a wave can count 63 fetches in flight
    static constexpr int STAGES = STAGES_LDS < STAGES_CNT ? (STAGES_LDS < 8 ? STAGES_LDS : 8) : (STAGES_CNT < 8 ? STAGES_CNT : 8);
    static constexpr int DIST = STAGES - 1;
    static constexpr int EPI_BYTES = NWAVES * RT * 32 * EPI_PITCH * 4;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES > EPI_BYTES ? STAGES * STAGE_BYTES : EPI_BYTES;
    static_assert(DIST >= 2, "the ring must hold the step being read, the next one and one in flight");
    static_assert(BKS * ROWB % (1024 * NWAVES) == 0 && NCT % 2 == 0, "stage / wave mismatch");
};

// position (in 16-byte chunks) of chunk c of B row r inside the row: rows r + 2, r + 3 of a transposing read are
// rotated by 64 bytes (for 128-byte rows: their halves swap), which puts the four rows of a read on distinct banks
template <int CPR> __device__ __forceinline__ int chunk_pos(int r, int c) { const int p = c + 4 * ((r >> 1) & 1); return p >= CPR ? p - CPR : p; }
template <int CPR> __device__ __forceinline__ int chunk_of_pos(int r, int pos) { const int c = pos - 4 * ((r >> 1) & 1); return c < 0 ? c + CPR : c; }

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
template <int PER, int MAXL> __device__ __forceinline__ void wait_later(int later) {
    // allow `later` (<= MAXL) younger K steps of PER fetches each to stay in flight
    if constexpr (MAXL == 0) { wait_vmcnt<0>(); }
    else { if (later >= MAXL) wait_vmcnt<PER * MAXL>(); else wait_later<PER, MAXL - 1>(later); }
}

struct SkinnyArgs {
    Bf16Args g;
    float* partial;             // SPLIT: slices x M x ldp floats
    int64_t ldp;
    int slices;
};

template <int RT, int NCT, bool SPLIT>
__global__ __launch_bounds__(NWAVES * 64)
void gemm_bf16_skinny_kernel(SkinnyArgs sa) {
    using C = Cfg<RT, NCT>;
    const Bf16Args& g = sa.g;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)lds);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, grp = lane >> 5;
    auto uni32 = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    auto uni64 = [&](int64_t x) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((int)(uint32_t)x), hi = __builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    const int K = uni32(g.K), K0 = uni32(g.K0);
    const int T_all = (K + BKS - 1) / BKS;
    // consecutive workgroups take the slices of one column group: the workgroups of one XCD (every eighth) then share
    // few slices of A in their L2
    const int slices = SPLIT ? uni32(sa.slices) : 1;
    const int slice = SPLIT ? (int)(blockIdx.x % (unsigned)slices) : 0;
    const int n0 = (SPLIT ? (int)(blockIdx.x / (unsigned)slices) : (int)blockIdx.x) * C::BN;
    const int t_first = SPLIT ? (int)((int64_t)T_all * slice / slices) : 0;
    const int T = (SPLIT ? (int)((int64_t)T_all * (slice + 1) / slices) : T_all) - t_first;       // K steps of this workgroup
    const int64_t ldb0 = uni64(g.ldb0), ldb1 = uni64(g.ldb1);
    const uint16_t* B0p = (const uint16_t*)uni64((int64_t)g.B0);
    const uint16_t* B1p = (const uint16_t*)uni64((int64_t)g.B1);

    // A: the 4 RT blocks of 8 rows x 128 bytes are dealt to the waves (wave w: blocks w, w + 4, ...); chunk c of row r
    // lands at position c ^ swizzle(r).  Lanes of rows beyond M stay off, except lane 0, so that every fetch is issued
    // and counted.
    const uint16_t* a_src[RT];
    bool a_on[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        const int row = (wave + 4 * i) * 8 + (lane >> 3), cp = lane & 7;
        const int c = cp ^ ((row ^ (row >> 3)) & 7);
        a_on[i] = row < g.M || lane == 0;
        a_src[i] = g.A + (int64_t)(row < g.M ? row : 0) * g.lda + c * 8;
    }
    // B: the stage's 16-byte units in order, NBD kilobytes per wave
    const uint16_t* b0_src[C::NBD];
    const uint16_t* b1_src[C::NBD];
    int b_krow[C::NBD], b_gn[C::NBD];
#pragma unroll
    for (int i = 0; i < C::NBD; ++i) {
        const int e = (wave * C::NBD + i) * 64 + lane;
        const int br = e / C::CPR, cpos = e - br * C::CPR;
        const int bc = chunk_of_pos<C::CPR>(br, cpos);
        int gn = n0 + bc * 8; gn = gn < g.N ? gn : g.N - 8;
        b_krow[i] = br; b_gn[i] = gn;
        b0_src[i] = B0p + (int64_t)br * ldb0 + gn;
        b1_src[i] = B1p + (int64_t)(br - K0) * ldb1 + gn;
    }

    auto issue = [&](int t, int slot) {                          // t counts this workgroup's K steps
        const int k0 = (t_first + t) * BKS;
        const uint32_t st = lds_base + slot * C::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            if ((wave + 4 * i) * 8 + 8 <= g.M) dma::dma16(a_src[i] + k0, st + (wave + 4 * i) * 1024);       // wave-uniform: a whole block
            else if (a_on[i]) dma::dma16(a_src[i] + k0, st + (wave + 4 * i) * 1024);
        }
        const uint32_t sb = st + C::A_BYTES + wave * C::NBD * 1024;
        if (k0 + BKS <= K0) {
            const int64_t off = (int64_t)k0 * ldb0;
#pragma unroll
            for (int i = 0; i < C::NBD; ++i) dma::dma16(b0_src[i] + off, sb + i * 1024);
        } else if (k0 >= K0 && k0 + BKS <= K) {
            const int64_t off = (int64_t)k0 * ldb1;
#pragma unroll
            for (int i = 0; i < C::NBD; ++i) dma::dma16(b1_src[i] + off, sb + i * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < C::NBD; ++i) {
                int gk = k0 + b_krow[i];
                const bool beyond = gk >= K;                      // rows past the contraction length read zeros
                gk = beyond ? K - 1 : gk;
                const bool first = gk < K0;
                const uint16_t* base = first ? B0p : B1p;
                const int64_t off = first ? (int64_t)gk * ldb0 : (int64_t)(gk - K0) * ldb1;
                dma::dma16(beyond ? (const uint16_t*)dma::g_zero16 : base + off + b_gn[i], sb + i * 1024);
            }
        }
    };

    // fragment addresses inside a stage: the wave's 16 contraction rows
    uint32_t a_off[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        const int row = i * 32 + j;
        a_off[i] = row * 128 + (((wave * 2 + grp) ^ ((row ^ (row >> 3)) & 7)) * 16);
    }
    const int s16 = lane & 15, nh = (lane >> 4) & 1;
    const int rl = wave * KW + grp * 8 + (s16 >> 2);             // row of the first transposing read; the second is 4 below
    uint32_t b_off[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
        b_off[ct] = C::A_BYTES + rl * C::ROWB + chunk_pos<C::CPR>(rl, ct * 4 + nh * 2) * 16 + (s16 & 3) * 8;
    struct Frags { bf16x8_t a[RT], b[NCT]; };
    auto read_frags = [&](int slot, Frags& f) {
        const uint8_t* st = lds + slot * C::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < RT; ++i) f.a[i] = *reinterpret_cast<const bf16x8_t*>(st + a_off[i]);
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            typedef dma::s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
            const dma::s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(st + b_off[ct]));
            const dma::s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(st + b_off[ct] + 4 * C::ROWB));
            const dma::s16x8_t both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            f.b[ct] = __builtin_bit_cast(bf16x8_t, both);
        }
    };

    f32x16_t acc[RT][NCT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int c = 0; c < NCT; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][c][v] = 0.f;

    int slot_issue = 0, slot_read = 0;
    auto next_slot = [](int s) { return s + 1 == C::STAGES ? 0 : s + 1; };
#pragma unroll
    for (int t = 0; t < C::DIST; ++t) if (t < T) { issue(t, slot_issue); slot_issue = next_slot(slot_issue); }

    Frags cur, nxt;
    if (T > 0) {
        const int later = (T - 1) < (C::DIST - 1) ? (T - 1) : (C::DIST - 1);
        wait_later<C::PER, C::DIST - 1>(later);
        __builtin_amdgcn_s_barrier();                          // step 0 has landed for every wave
        read_frags(slot_read, cur); slot_read = next_slot(slot_read);
    }
    // step t: behind the barrier step t + 1 has landed for every wave and nobody reads the slot of step t - 1 any
    // more: refill that slot, start reading step t + 1, multiply step t
    for (int t = 0; t < T; ++t) {
        if (t + 1 < T) {
            const int left = T - 2 - t;
            wait_later<C::PER, C::DIST - 2>(left < C::DIST - 2 ? left : C::DIST - 2);
        }
        __builtin_amdgcn_s_barrier();
        if (t + C::DIST < T) { issue(t + C::DIST, slot_issue); slot_issue = next_slot(slot_issue); }
        nxt = cur;
        if (t + 1 < T) { read_frags(slot_read, nxt); slot_read = next_slot(slot_read); }
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct)
                acc[i][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.b[ct], cur.a[i], acc[i][ct], 0, 0, 0);
        cur = nxt;
    }

    // acc[i][ct][v] = partial C[row 32 i + lane % 32][col ct*32 + 8 (v / 4) + 4 (lane / 32) + v % 4] over the wave's share of K.
    // 64 columns at a time: every wave lays its share down, then all threads add the four in wave order.
    float* ep = reinterpret_cast<float*>(lds) + wave * (RT * 32 * EPI_PITCH);
    const float* all = reinterpret_cast<const float*>(lds);
    const int rr = tid >> 3, cc = tid & 7;
#pragma unroll
    for (int cp = 0; cp < NCT / 2; ++cp) {
        __syncthreads();                                       // the ring (first pass) or the previous pass is no longer read
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16_t& a = acc[i][cp * 2 + c2];
                    const f32x4_t v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                    *reinterpret_cast<f32x4_t*>(ep + (i * 32 + j) * EPI_PITCH + c2 * 32 + 8 * q + 4 * grp) = v;
                }
        __syncthreads();
        const int col = n0 + cp * EPI_COLS + cc * 8;
#pragma unroll
        for (int it = 0; it < RT; ++it) {
            const int row = it * 32 + rr;
            f32x4_t s0 = *reinterpret_cast<const f32x4_t*>(all + row * EPI_PITCH + cc * 8);
            f32x4_t s1 = *reinterpret_cast<const f32x4_t*>(all + row * EPI_PITCH + cc * 8 + 4);
#pragma unroll
            for (int w = 1; w < NWAVES; ++w) {                   // fixed order: wave 0 + wave 1 + wave 2 + wave 3
                s0 += *reinterpret_cast<const f32x4_t*>(all + (w * RT * 32 + row) * EPI_PITCH + cc * 8);
                s1 += *reinterpret_cast<const f32x4_t*>(all + (w * RT * 32 + row) * EPI_PITCH + cc * 8 + 4);
            }
            if (row < g.M && col < g.N) {
                if (SPLIT) {
                    float* dst = sa.partial + ((int64_t)slice * g.M + row) * sa.ldp + col;
                    *reinterpret_cast<f32x4_t*>(dst) = s0;
                    *reinterpret_cast<f32x4_t*>(dst + 4) = s1;
                } else {
                    u32x4_t out;
                    out[0] = pack_bf16x2(s0[0], s0[1]); out[1] = pack_bf16x2(s0[2], s0[3]);
                    out[2] = pack_bf16x2(s1[0], s1[1]); out[3] = pack_bf16x2(s1[2], s1[3]);
                    *reinterpret_cast<u32x4_t*>(g.C + (int64_t)row * g.ldc + col) = out;
                }
            }
        }
    }
}

// C[row][col .. col + 7] = bf16(partial[0] + partial[1] + ... in slice order); one thread per 8 columns
__global__ __launch_bounds__(256)
void skinny_reduce_kernel(const float* __restrict__ partial, int64_t ldp, int slices, int M, int N, uint16_t* __restrict__ Cout, int64_t ldc) {
    const int chunks = N >> 3;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= (int64_t)M * chunks) return;
    const int row = (int)(id / chunks), col = (int)(id - (int64_t)row * chunks) * 8;
    const float* src = partial + (int64_t)row * ldp + col;
    f32x4_t s0 = *reinterpret_cast<const f32x4_t*>(src), s1 = *reinterpret_cast<const f32x4_t*>(src + 4);
    for (int s = 1; s < slices; ++s) {
        const float* q = src + (int64_t)s * M * ldp;
        s0 += *reinterpret_cast<const f32x4_t*>(q);
        s1 += *reinterpret_cast<const f32x4_t*>(q + 4);
    }
    u32x4_t out;
    out[0] = pack_bf16x2(s0[0], s0[1]); out[1] = pack_bf16x2(s0[2], s0[3]);
    out[2] = pack_bf16x2(s1[0], s1[1]); out[3] = pack_bf16x2(s1[2], s1[3]);
    *reinterpret_cast<u32x4_t*>(Cout + (int64_t)row * ldc + col) = out;
}

}  // namespace skinny

template <int BM, int BN, int WM>
constexpr size_t smem_bytes() { return 2 * (size_t)(BM * A_PITCH + BK * BN) * sizeof(uint16_t); }

template <int BM, int BN, int WM>
hipError_t launch(const GemmOperands& o, hipStream_t stream) {
    Bf16Args a;
    a.A = (const uint16_t*)o.A;   a.lda = o.lda;
    a.B0 = (const uint16_t*)o.B0; a.ldb0 = o.ldb0; a.K0 = o.K0;
    a.B1 = (const uint16_t*)o.B1; a.ldb1 = o.ldb1;
    a.C = (uint16_t*)o.C;         a.ldc = o.ldc;
    a.M = o.M; a.N = o.N; a.K = o.K;
    a.tiles_m = (o.M + BM - 1) / BM;
    a.tiles_n = (o.N + BN - 1) / BN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    const size_t lds_bytes = smem_bytes<BM, BN, WM>();
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM>), dim3(a.tiles_m * a.tiles_n), dim3(NT),
                       lds_bytes, stream, a);
    return hipGetLastError();
}

template <int BM, int BN, int WM>
hipError_t allow_big_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<BM, BN, WM>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<BM, BN, WM>());
}

}  // namespace

// Split launch of the skinny path: how many ranges of K steps a column group of 192 is cut into so that
// groups x slices comes close to the chip's 256 CUs (1: not worth it), and the float workspace it needs.
int gemm_bf16_skinny_slices(int M, int N, int K) {
    // Measured: with 128 or more column groups of 64 the launch that keeps all of K in a workgroup is as fast (68 x
    // 12288 x 4096: 30 us either way; 68 x 4096 x 4096: 28 -> 20 us; 68 x 4096 x 11008: 70 -> 29 us); beyond three
    // row tiles the 192-column accumulators no longer fit the registers.
    if (M > 96 || N < 192 || (N + 63) / 64 > 128) return 1;
    const int groups = (N + 191) / 192;
    const int T = (K + 63) / 64;
    int slices = 256 / groups;
    if (slices > T / 4) slices = T / 4;                  // at least four K steps per slice
    return slices < 2 ? 1 : slices;
}
int64_t gemm_bf16_skinny_ldp(int N) { return ((int64_t)N + 7) & ~(int64_t)7; }
size_t gemm_bf16_skinny_ws_bytes(int M, int N, int K) {
    const int slices = gemm_bf16_skinny_slices(M, N, K);
    return slices > 1 ? (size_t)slices * M * gemm_bf16_skinny_ldp(N) * sizeof(float) : 0;
}

namespace {

template <int RT, int NCT, bool SPLIT>
hipError_t allow_skinny_lds() {
    using C = skinny::Cfg<RT, NCT>;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&skinny::gemm_bf16_skinny_kernel<RT, NCT, SPLIT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
}

template <int RT>
hipError_t launch_skinny(const Bf16Args& a, hipStream_t stream) {
    using C = skinny::Cfg<RT, 2>;
    skinny::SkinnyArgs sa{a, nullptr, 0, 1};
    hipLaunchKernelGGL((skinny::gemm_bf16_skinny_kernel<RT, 2, false>), dim3((a.N + C::BN - 1) / C::BN), dim3(skinny::NWAVES * 64),
                       (size_t)C::LDS_BYTES, stream, sa);
    return hipGetLastError();
}

// column groups of 192 x `slices` ranges of K steps, partial sums in `ws`, then the reduction
template <int RT>
hipError_t launch_skinny_split(const Bf16Args& a, int slices, float* ws, hipStream_t stream) {
    using C = skinny::Cfg<RT, 6>;
    const int groups = (a.N + C::BN - 1) / C::BN;
    const int64_t ldp = gemm_bf16_skinny_ldp(a.N);
    skinny::SkinnyArgs sa{a, ws, ldp, slices};
    hipLaunchKernelGGL((skinny::gemm_bf16_skinny_kernel<RT, 6, true>), dim3(groups * slices), dim3(skinny::NWAVES * 64),
                       (size_t)C::LDS_BYTES, stream, sa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t items = (int64_t)a.M * (a.N >> 3);
    hipLaunchKernelGGL(skinny::skinny_reduce_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, stream,
                       (const float*)ws, ldp, slices, a.M, a.N, a.C, a.ldc);
    return hipGetLastError();
}

}  // namespace

hipError_t gemm_bf16_init() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dma::gemm_bf16_dma_kernel<256>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, dma::lds_bytes<256>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dma::gemm_bf16_dma_kernel<192>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, dma::lds_bytes<192>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dma::gemm_bf16_dma_mixed_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, dma::lds_bytes<256>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dma::gemm_bf16_dma_batched_kernel<256>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, dma::lds_bytes<256>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dma::gemm_bf16_dma_batched_kernel<192>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, dma::lds_bytes<192>());
    if (e != hipSuccess) return e;
    e = allow_big_lds<256, 256, 64>();
    if (e != hipSuccess) return e;
    e = allow_skinny_lds<1, 2, false>();
    if (e == hipSuccess) e = allow_skinny_lds<2, 2, false>();
    if (e == hipSuccess) e = allow_skinny_lds<3, 2, false>();
    if (e == hipSuccess) e = allow_skinny_lds<4, 2, false>();
    if (e == hipSuccess) e = allow_skinny_lds<1, 6, true>();
    if (e == hipSuccess) e = allow_skinny_lds<2, 6, true>();
    if (e == hipSuccess) e = allow_skinny_lds<3, 6, true>();
    if (e != hipSuccess) return e;
    return allow_big_lds<128, 128, 32>();
}

namespace {

template <int BN>
hipError_t launch_dma(const GemmOperands& o, hipStream_t stream) {
    Bf16Args a;
    a.A = (const uint16_t*)o.A;   a.lda = o.lda;
    a.B0 = (const uint16_t*)o.B0; a.ldb0 = o.ldb0; a.K0 = o.K0;
    a.B1 = (const uint16_t*)o.B1; a.ldb1 = o.ldb1;
    a.C = (uint16_t*)o.C;         a.ldc = o.ldc;
    a.M = o.M; a.N = o.N; a.K = o.K;
    a.tiles_m = (o.M + dma::BM - 1) / dma::BM;
    a.tiles_n = (o.N + BN - 1) / BN; a.narrow_cols = 0;
    hipLaunchKernelGGL(dma::gemm_bf16_dma_kernel<BN>, dim3(a.tiles_m * a.tiles_n), dim3(512),
                       (size_t)dma::lds_bytes<BN>(), stream, a);
    return hipGetLastError();
}

}  // namespace

// Tile choice (measured on MI355X): 256-row tiles with 8 waves (two per SIMD) win for every shape
// of the chain whose M exceeds one small tile; the width is the one with the shorter schedule on
// the chip's 256 CUs (one tile per CU at a time; a 192-wide tile costs 0.87 of a 256-wide one).
// Tiny M (decode-shaped batches) takes 128 x 128 with 4 waves so that N alone can spread the work.
hipError_t gemm_bf16(const GemmOperands& o, hipStream_t stream) {
    if (o.M <= 0 || o.N <= 0 || o.K <= 0) return hipSuccess;
    if (o.subtract) return hipErrorInvalidValue;       // float only
    if ((int64_t)o.M * o.lda >= (int64_t)1 << 31) return hipErrorInvalidValue;   // the generic kernel keeps 32-bit element offsets into A
    if (o.M > 128 && o.N >= 8 && (o.a_zero_padded || o.K % dma::BKS == 0)) {
        constexpr int kCus = 256;
        constexpr double kNarrow = 0.87;         // measured cost of a 192-wide tile relative to a 256-wide one
        const int64_t tiles_m = (o.M + dma::BM - 1) / dma::BM;
        const int64_t t256 = tiles_m * ((o.N + 255) / 256), t192 = tiles_m * ((o.N + 191) / 192);
        const double cost256 = (double)((t256 + kCus - 1) / kCus), cost192 = kNarrow * (double)((t192 + kCus - 1) / kCus);
        // mixed: at most one round of wide tiles and two rounds in all, so that every CU runs at most wide + narrow
        int best_a = -1, best_b = 0;
        if (t256 > kCus && tiles_m <= kCus) {
            int64_t best_width = 0;
            for (int64_t a = std::min<int64_t>(o.N / 256, kCus / tiles_m); a >= 1; --a) {
                const int64_t rest = o.N - a * 256;
                const int64_t b = rest > 0 ? (rest + 191) / 192 : 0;
                if (b == 0 || tiles_m * (a + b) > 2 * kCus) continue;
                const int64_t width = a * 256 + b * 192;
                if (best_a < 0 || width < best_width) { best_a = (int)a; best_b = (int)b; best_width = width; }
            }
        }
        const double cost_mixed = best_a > 0 ? 1.0 + kNarrow : 1e30;
        if (cost_mixed < cost256 && cost_mixed < cost192) {
            Bf16Args a;
            a.A = (const uint16_t*)o.A;   a.lda = o.lda;
            a.B0 = (const uint16_t*)o.B0; a.ldb0 = o.ldb0; a.K0 = o.K0;
            a.B1 = (const uint16_t*)o.B1; a.ldb1 = o.ldb1;
            a.C = (uint16_t*)o.C;         a.ldc = o.ldc;
            a.M = o.M; a.N = o.N; a.K = o.K;
            a.tiles_m = (int)tiles_m; a.tiles_n = best_a; a.narrow_cols = best_b;
            hipLaunchKernelGGL(dma::gemm_bf16_dma_mixed_kernel, dim3((unsigned)(tiles_m * (best_a + best_b))), dim3(512),
                               (size_t)dma::lds_bytes<256>(), stream, a);
            return hipGetLastError();
        }
        return cost192 < cost256 ? launch_dma<192>(o, stream) : launch_dma<256>(o, stream);
    }
    if (o.M > 128) return launch<256, 256, 64>(o, stream);
    if (o.N >= 8 && (o.a_zero_padded || o.K % skinny::BKS == 0)) {
        Bf16Args a;
        a.A = (const uint16_t*)o.A;   a.lda = o.lda;
        a.B0 = (const uint16_t*)o.B0; a.ldb0 = o.ldb0; a.K0 = o.K0;
        a.B1 = (const uint16_t*)o.B1; a.ldb1 = o.ldb1;
        a.C = (uint16_t*)o.C;         a.ldc = o.ldc;
        a.M = o.M; a.N = o.N; a.K = o.K;
        a.tiles_m = 1; a.tiles_n = (o.N + 63) / 64;
        const int slices = gemm_bf16_skinny_slices(o.M, o.N, o.K);
        if (slices > 1 && o.N % 8 == 0 && o.splitk_ws && o.splitk_ws_bytes >= gemm_bf16_skinny_ws_bytes(o.M, o.N, o.K)) {
            float* ws = (float*)o.splitk_ws;
            switch ((o.M + 31) / 32) {
                case 1: return launch_skinny_split<1>(a, slices, ws, stream);
                case 2: return launch_skinny_split<2>(a, slices, ws, stream);
                default: return launch_skinny_split<3>(a, slices, ws, stream);
            }
        }
        switch ((o.M + 31) / 32) {
            case 1: return launch_skinny<1>(a, stream);
            case 2: return launch_skinny<2>(a, stream);
            case 3: return launch_skinny<3>(a, stream);
            default: return launch_skinny<4>(a, stream);
        }
    }
    return launch<128, 128, 32>(o, stream);
}

// One launch for all the products of a block-diagonal mix or unmix.  The tile width is the one with the shorter
// schedule on the chip's CUs over ALL products (a 192-wide tile costs 0.87 of a 256-wide one).
hipError_t gemm_bf16_batched(const GemmOperands* ops, int count, hipStream_t stream) {
    if (count < 1 || count > kGemmBatchMax) return hipErrorInvalidValue;
    const int N = ops[0].N;
    for (int i = 0; i < count; ++i) {
        const GemmOperands& o = ops[i];
        if (o.M < 1 || o.M > dma::BM || o.K < 1 || o.N != N || N < 8 || N % 8 != 0 || o.subtract) return hipErrorInvalidValue;
        if (!(o.a_zero_padded || o.K % dma::BKS == 0)) return hipErrorInvalidValue;
    }
    constexpr int kCus = 256;
    const int64_t t256 = (int64_t)count * ((N + 255) / 256), t192 = (int64_t)count * ((N + 191) / 192);
    const bool narrow = 0.87 * (double)((t192 + kCus - 1) / kCus) < (double)((t256 + kCus - 1) / kCus);
    const int BN = narrow ? 192 : 256;
    dma::Bf16Batch b;
    for (int i = 0; i < count; ++i) {
        const GemmOperands& o = ops[i];
        Bf16Args& a = b.g[i];
        a.A = (const uint16_t*)o.A;   a.lda = o.lda;
        a.B0 = (const uint16_t*)o.B0; a.ldb0 = o.ldb0; a.K0 = o.K0;
        a.B1 = (const uint16_t*)o.B1; a.ldb1 = o.ldb1;
        a.C = (uint16_t*)o.C;         a.ldc = o.ldc;
        a.M = o.M; a.N = o.N; a.K = o.K;
        a.tiles_m = 1; a.tiles_n = (N + BN - 1) / BN; a.narrow_cols = 0;
    }
    for (int i = count; i < kGemmBatchMax; ++i) b.g[i] = b.g[0];
    const dim3 grid((unsigned)((N + BN - 1) / BN), (unsigned)count);
    if (narrow) hipLaunchKernelGGL(dma::gemm_bf16_dma_batched_kernel<192>, grid, dim3(512), (size_t)dma::lds_bytes<192>(), stream, b);
    else hipLaunchKernelGGL(dma::gemm_bf16_dma_batched_kernel<256>, grid, dim3(512), (size_t)dma::lds_bytes<256>(), stream, b);
    return hipGetLastError();
}

}  // namespace gelo
