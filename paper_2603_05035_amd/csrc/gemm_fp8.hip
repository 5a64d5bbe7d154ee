// The accelerator's projection Y = U W (Section 3.2, eq. 2) with both operands stored as 8-bit floats
// (OCP FP8 E4M3; the paper's Conclusion lists FP8 / INT8 numerics as the next thing to characterise) on the
// gfx950 matrix cores: v_mfma_f32_32x32x64_f8f6f4, float accumulation, bf16 result.  Twice the matrix rate of
// the bf16 path for the same bytes fetched per unit time.
//
//   U (per batch)   one scale per row (token):  U8[i][k] = e4m3(U[i][k] * 448 / max_k |U[i][k]|)
//   W (static)      one scale per column:       W8[j][k] = e4m3(W[k][j] * 448 / max_k |W[k][j]|), stored
//                   TRANSPOSED (p x d), so that both operands have the contraction index contiguous and
//                   every fragment is two 16-byte LDS reads (no transposing reads)
//   Y[i][j] = (sum_k U8[i][k] W8[j][k]) * su[i] * sw[j],  su = max / 448, sw likewise
//
// Rounding is round-to-nearest-even onto the E4M3 grid with gradual underflow, done with integer
// arithmetic on the float bit pattern so that every code is defined by this file alone; the scaled value
// never exceeds 448 * (1 + 2^-23), which rounds to 448.
#include "gelo_internal.h"

namespace gelo {
namespace {

typedef int i32x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits(uint32_t h) { return __uint_as_float(h << 16); }

// float -> E4M3 code (1 sign, 4 exponent bits with bias 7, 3 fraction bits; largest finite value 448 = 0x7E),
// round to nearest even, saturating, subnormals spaced 2^-9
__device__ __forceinline__ uint32_t e4m3_code(float t) {
    const uint32_t bits = __float_as_uint(t);
    const uint32_t sign = (bits >> 24) & 0x80u;
    const float a = fabsf(t);
    uint32_t code;
    if (a < 0.015625f) {                                     // below 2^-6: multiples of 2^-9; 8 of them is the first normal
        code = (uint32_t)rintf(a * 512.0f);
    } else {
        uint32_t m = __float_as_uint(a);
        m += 0x7FFFFu + ((m >> 20) & 1u);                    // round the 23-bit fraction to 3 bits, ties to even
        const uint32_t e = (m >> 23) - 120u;                 // rebias: 127 -> 7
        code = (e << 3) | ((m >> 20) & 7u);
        code = code > 0x7Eu ? 0x7Eu : code;                  // saturate at 448 (0x7F would be NaN)
    }
    return sign | code;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// One workgroup per row of X (bf16, cols a multiple of 8): scale[row] = max |x| / 448 (1 for an all-zero row),
// codes[row][c] = e4m3(x * (448 / max)).
__global__ __launch_bounds__(256)
void quantize_rows_kernel(const uint16_t* X, int64_t ld, int cols, uint8_t* codes, int64_t ldq, float* scale) {
    __shared__ float part[4];
    const int row = blockIdx.x, tid = threadIdx.x;
    const uint16_t* xr = X + (int64_t)row * ld;
    float amax = 0.f;
    for (int c = tid * 8; c < cols; c += 256 * 8) {
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(xr + c);
#pragma unroll
        for (int t = 0; t < 4; ++t) amax = fmaxf(amax, fmaxf(fabsf(bf16_bits(v[t] & 0xFFFFu)), fabsf(bf16_bits(v[t] >> 16))));
    }
    amax = wave_max(amax);
    if ((tid & 63) == 0) part[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    const float inv = amax > 0.f ? 448.0f / amax : 1.0f;
    if (tid == 0) scale[row] = amax > 0.f ? amax / 448.0f : 1.0f;
    for (int c = tid * 8; c < cols; c += 256 * 8) {
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(xr + c);
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            lo |= e4m3_code(bf16_bits(v[t] & 0xFFFFu) * inv) << (16 * t);
            lo |= e4m3_code(bf16_bits(v[t] >> 16) * inv) << (16 * t + 8);
            hi |= e4m3_code(bf16_bits(v[t + 2] & 0xFFFFu) * inv) << (16 * t);
            hi |= e4m3_code(bf16_bits(v[t + 2] >> 16) * inv) << (16 * t + 8);
        }
        *reinterpret_cast<u32x2_t*>(codes + (int64_t)row * ldq + c) = u32x2_t{lo, hi};
    }
}

// W (d x p, bf16) -> codes transposed (p x d) and one scale per column.  A workgroup takes 64 columns: thread
// (c = tid % 64, g = tid / 64) first finds the column maximum over rows g, g + 4, ..., then quantises 16
// consecutive rows of its column at a time and writes them as one 16-byte piece of the transposed row.
__global__ __launch_bounds__(256)
void quantize_weight_kernel(const uint16_t* W, int64_t ldw, int d, int p, uint8_t* codes, float* scale) {
    __shared__ float part[4][64];
    const int tid = threadIdx.x, c = tid & 63, g = tid >> 6;
    const int col = blockIdx.x * 64 + c;
    const bool live = col < p;
    const uint16_t* wc = W + (live ? col : p - 1);
    float amax = 0.f;
    for (int r = g; r < d; r += 4) amax = fmaxf(amax, fabsf(bf16_bits(wc[(int64_t)r * ldw])));
    part[g][c] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(part[0][c], part[1][c]), fmaxf(part[2][c], part[3][c]));
    const float inv = amax > 0.f ? 448.0f / amax : 1.0f;
    if (g == 0 && live) scale[col] = amax > 0.f ? amax / 448.0f : 1.0f;
    for (int r0 = g * 16; r0 < d; r0 += 64) {                // d is a multiple of 128
        u32x4_t out;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) word |= e4m3_code(bf16_bits(wc[(int64_t)(r0 + 4 * q + b) * ldw]) * inv) << (8 * b);
            out[q] = word;
        }
        if (live) *reinterpret_cast<u32x4_t*>(codes + (int64_t)col * d + r0) = out;
    }
}

// ---------------------------------------------------------------------------------------- the product --
// Same frame as the bf16 kernel of gemm_bf16.hip: 256 x 256 tile, 8 waves (wave tile 64 x 128), two LDS stages
// filled by direct-to-LDS loads, one barrier per K step, XOR-swizzled 16-byte chunks, MFMA operands swapped so
// that a lane owns columns of one row, epilogue through LDS.  What differs: a K step is 128 contraction values
// (128 bytes per row: the same bytes per step as 64 bf16 values), both operands are row tiles with the
// contraction index contiguous, and a fragment is 32 consecutive bytes.
struct Fp8Args {
    const uint8_t* A; int64_t lda; const float* sa;      // M x K codes, row scales
    const uint8_t* B; int64_t ldb; const float* sb;      // N x K codes (the transposed weight), column scales of the product
    uint16_t* C; int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n;
};

constexpr int BM = 256, BN = 256, BKB = 128, TILE_BYTES = 256 * BKB, STAGE_BYTES = 2 * TILE_BYTES;

__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(gptr), "s"(lds_addr) : "memory", "m0");
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

// XCD-aware tile walk: each of the 8 XCDs gets a contiguous run of tiles, tile rows in balanced groups of at most 8
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

__global__ __launch_bounds__(512)
void gemm_fp8_kernel(Fp8Args g) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    int tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int j = lane & 31, grp = lane >> 5;
    const int T = g.K / BKB;                                  // K is a multiple of 128 (checked by the launcher)

    // fetch: a 1 KB block is 8 rows x 128 bytes; lane l brings chunk position l % 8 of row l / 8, which holds
    // logical chunk (position ^ swizzle(row)).  Rows beyond the matrix are clamped (their products are never stored).
    const uint8_t* a_src[4];
    const uint8_t* b_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (wave * 4 + i) * 8 + (lane >> 3), cp = lane & 7;
        const int c = cp ^ ((row ^ (row >> 3)) & 7);
        int ga = m0 + row; ga = ga < g.M ? ga : g.M - 1;
        int gb = n0 + row; gb = gb < g.N ? gb : g.N - 1;
        a_src[i] = g.A + (int64_t)ga * g.lda + c * 16;
        b_src[i] = g.B + (int64_t)gb * g.ldb + c * 16;
    }
    auto issue = [&](int t) {
        const int k0 = t * BKB;
        const uint32_t st = lds_base + (t & 1) * STAGE_BYTES + (wave * 4) * 1024;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16(a_src[i] + k0, st + i * 1024);
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16(b_src[i] + k0, st + TILE_BYTES + i * 1024);
    };

    const int sw = (j ^ (j >> 3)) & 7;
    const uint32_t a_off = (wm * 64 + j) * BKB;
    const uint32_t b_off = TILE_BYTES + (wn * 128 + j) * BKB;

    f32x16_t acc[2][4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0.f;

    i32x8_t a_frag[2][2], b_frag[2][4];
    issue(0);
    for (int t = 0; t < T; ++t) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        if (t + 1 < T) issue(t + 1);
        const uint8_t* st = lds + (t & 1) * STAGE_BYTES;
        // a fragment: the 32 contraction bytes 64 ks + 32 grp .. of the lane's row = logical chunks 4 ks + 2 grp, + 1
        auto load_frags = [&](int fb, int ks) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int s = sw ^ (mt * 4);
                const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(st + a_off + mt * 32 * BKB + (((ks * 4 + grp * 2) ^ s) * 16));
                const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(st + a_off + mt * 32 * BKB + (((ks * 4 + grp * 2 + 1) ^ s) * 16));
                a_frag[fb][mt] = i32x8_t{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                const int s = sw ^ ((ct & 1) * 4);
                const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(st + b_off + ct * 32 * BKB + (((ks * 4 + grp * 2) ^ s) * 16));
                const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(st + b_off + ct * 32 * BKB + (((ks * 4 + grp * 2 + 1) ^ s) * 16));
                b_frag[fb][ct] = i32x8_t{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
        };
        load_frags(0, 0);
        load_frags(1, 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[mt][c] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b_frag[ks][c], a_frag[ks][mt], acc[mt][c], 0, 0, 0, 0, 0, 0);
    }

    // acc[mt][ct][v] = C[row 64 wm + 32 mt + lane % 32][col 128 wn + 32 ct + 8 (v / 4) + 4 (lane / 32) + v % 4]
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    constexpr int EPI_PITCH = BN + 16;
    uint8_t* patch = lds + wave * (32 * EPI_PITCH);
    const int rr = lane >> 4, cc = lane & 15;
    const int col = n0 + wn * 128 + cc * 8;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        int srow = m0 + wm * 64 + mt * 32 + j; srow = srow < g.M ? srow : g.M - 1;
        const float sa = g.sa[srow];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int sc = n0 + wn * 128 + ct * 32 + 8 * q + 4 * grp; sc = sc + 4 <= g.N ? sc : g.N - 4;
                const f32x4_t sb = *reinterpret_cast<const f32x4_t*>(g.sb + sc);
                u32x2_t out;
                out[0] = pack_bf16x2(acc[mt][ct][4 * q] * (sa * sb[0]), acc[mt][ct][4 * q + 1] * (sa * sb[1]));
                out[1] = pack_bf16x2(acc[mt][ct][4 * q + 2] * (sa * sb[2]), acc[mt][ct][4 * q + 3] * (sa * sb[3]));
                *reinterpret_cast<u32x2_t*>(patch + j * EPI_PITCH + (ct * 32 + 8 * q + 4 * grp) * 2) = out;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = it * 4 + rr;
            const u32x4_t v = *reinterpret_cast<const u32x4_t*>(patch + r * EPI_PITCH + cc * 16);
            const int row = m0 + wm * 64 + mt * 32 + r;
            if (row < g.M && col < g.N) *reinterpret_cast<u32x4_t*>(g.C + (int64_t)row * g.ldc + col) = v;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

}  // namespace

hipError_t gemm_fp8_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_fp8_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               2 * STAGE_BYTES);
}

hipError_t quantize_rows_e4m3(const void* X, int64_t ld, int rows, int cols, uint8_t* codes, int64_t ldq, float* scale,
                              hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    if (cols % 8 != 0 || ldq < cols) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quantize_rows_kernel, dim3(rows), dim3(256), 0, stream, (const uint16_t*)X, ld, cols, codes, ldq, scale);
    return hipGetLastError();
}

hipError_t quantize_weight_e4m3(const void* W, int64_t ldw, int d, int p, uint8_t* codes, float* scale, hipStream_t stream) {
    if (d % 128 != 0 || p < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quantize_weight_kernel, dim3((p + 63) / 64), dim3(256), 0, stream, (const uint16_t*)W, ldw, d, p, codes, scale);
    return hipGetLastError();
}

hipError_t gemm_fp8(const uint8_t* A, int64_t lda, const float* sa, const uint8_t* B, int64_t ldb, const float* sb,
                    void* C, int64_t ldc, int M, int N, int K, hipStream_t stream) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    if (K % BKB != 0 || N % 8 != 0 || N < 8 || lda % 16 != 0 || ldb % 16 != 0) return hipErrorInvalidValue;
    Fp8Args g;
    g.A = A; g.lda = lda; g.sa = sa; g.B = B; g.ldb = ldb; g.sb = sb; g.C = (uint16_t*)C; g.ldc = ldc;
    g.M = M; g.N = N; g.K = K;
    g.tiles_m = (M + BM - 1) / BM; g.tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(gemm_fp8_kernel, dim3(g.tiles_m * g.tiles_n), dim3(512), (size_t)2 * STAGE_BYTES, stream, g);
    return hipGetLastError();
}

}  // namespace gelo
