// Decode-shaped batches (n = n_data + k_shield <= 128): the trusted side's two latency-bound steps as
// single launches.
//
//   small_sample   draws the secrets of MANY batches at once (Section 3.2 step 1.2: a fresh A per batch; a
//                  decode step needs one per layer, and A does not depend on the data, so a whole step's
//                  worth is drawn ahead in one launch).  One workgroup per matrix: Philox Gaussian straight
//                  into LDS, unblocked Householder QR there, A = Q diag(sign r_ii) and its transpose written
//                  out; one more workgroup per shield direction row.
//   small_mix      shield rows (row-norm statistic of H, exact-norm scaling; Section 3.2.1 eqs. 7-8) and
//                  U = A [H ; S] (eq. 1) in one launch.
//
// Both replace chains of 4 - 8 launches of the general kernels, each of which costs more in launch latency
// than in work at this size.
#include "gelo_internal.h"

namespace gelo {
namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// leading dimension (floats) of a column in LDS: a multiple of 4 (16-byte reads), four times an odd number so
// that the 16-byte reads of 16 neighbouring columns fall on distinct banks
__host__ __device__ inline int small_ldc(int n) { return 4 * (2 * ((n + 7) / 8) + 1); }

struct SmallSampleArgs {
    SmallSampleTargets t;
    uint32_t key0, key1, c1_mix, c1_shield;
    uint64_t first_batch;
    int n, k, d;
    int64_t ldk;
};

// Thread c owns column c of W = [G | I] (n x 2 n, column-major in LDS).  Step j applies the reflector of column
// j to every later column: each thread walks rows j + 1 .. n - 1 of the pivot column (the same address for all
// threads: a broadcast) and of its own column twice - once for v^T a and |x|^2, once for the update - and
// needs nobody else's result: one barrier per column, no reductions.  The right half ends as Q^T.
__global__ __launch_bounds__(256)
void small_sample_kernel(SmallSampleArgs a) {
    extern __shared__ __attribute__((aligned(16))) float W[];
    __shared__ float rdiag[kSmallMaxN];
    __shared__ float wave_part[4];
    const int per_item = 1 + a.k;
    const int item = blockIdx.x / per_item, role = blockIdx.x - item * per_item;
    const uint64_t batch = a.first_batch + (uint64_t)item;
    PhiloxStream ps;
    ps.key0 = a.key0; ps.key1 = a.key1; ps.c2 = (uint32_t)batch; ps.c3 = (uint32_t)(batch >> 32);
    char* block = (char*)a.t.block[item];
    if (role > 0) {
        ps.c1 = a.c1_shield;
        shield_direction_row((float*)(block + a.t.off_GS), a.d, role - 1, ps, (float*)(block + a.t.off_gsnorm), wave_part);
        return;
    }
    const int n = a.n, ldc = small_ldc(n), tid = threadIdx.x;
    // G: element e = r n + c is output e % 4 of Philox block e / 4; the right half starts as the identity;
    // rows n .. ldc - 1 of every column are zero (the 16-byte reads of a column's tail run into them)
    for (int i = tid; i < 2 * n * ldc; i += 256) {
        const int c = i / ldc, r = i - c * ldc;
        W[i] = (c >= n && r == c - n) ? 1.f : 0.f;
    }
    __syncthreads();
    const int total = n * n;
    for (int q = tid; q * 4 < total; q += 256) {
        uint32_t c0 = (uint32_t)q, c1 = a.c1_mix, c2 = ps.c2, c3 = ps.c3;
        philox4x32_10(c0, c1, c2, c3, ps.key0, ps.key1);
        float z[4];
        box_muller(c0, c1, &z[0], &z[1]);
        box_muller(c2, c3, &z[2], &z[3]);
        int e = q * 4;
        int r = e / n, c = e - r * n;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (e + t < total) W[c * ldc + r] = z[t];
            if (++c == n) { c = 0; ++r; }
        }
    }
    __syncthreads();

    const int c = tid;
    float* mine = W + c * ldc;
    for (int j = 0; j < n; ++j) {
        const float* piv = W + j * ldc;
        if (c > j && c < 2 * n) {
            const float alpha = piv[j];
            const float top = mine[j];
            const int r0 = (j + 1) & ~3;
            // four independent partial sums each, and the loop unrolled: a lone wave per SIMD has nothing else to hide
            // the LDS latency behind
            f32x4_t sp = {0.f, 0.f, 0.f, 0.f}, qp = {0.f, 0.f, 0.f, 0.f};
            {
                // only the first chunk can reach above the tail
                f32x4_t x = *reinterpret_cast<const f32x4_t*>(piv + r0);
                const f32x4_t y = *reinterpret_cast<const f32x4_t*>(mine + r0);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float xt = r0 + t > j ? x[t] : 0.f;
                    sp[t] = xt * y[t];
                    qp[t] = xt * xt;
                }
            }
#pragma unroll 4
            for (int r = r0 + 4; r < n; r += 4) {
                const f32x4_t x = *reinterpret_cast<const f32x4_t*>(piv + r);
                const f32x4_t y = *reinterpret_cast<const f32x4_t*>(mine + r);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    sp[t] = fmaf(x[t], y[t], sp[t]);
                    qp[t] = fmaf(x[t], x[t], qp[t]);
                }
            }
            const float s = (sp[0] + sp[1]) + (sp[2] + sp[3]);
            const float q = (qp[0] + qp[1]) + (qp[2] + qp[3]);
            // beta = -sign(alpha) sqrt(alpha^2 + |x|^2), tau = (beta - alpha) / beta, v = x / (alpha - beta) below a
            // unit entry; a zero tail gives the identity (tau = 0)
            const bool tail = q > 0.f;
            const float nrm = __builtin_amdgcn_sqrtf(fmaf(alpha, alpha, q));
            const float beta = tail ? -copysignf(nrm, alpha) : alpha;
            const float tau = tail ? (beta - alpha) * __builtin_amdgcn_rcpf(beta) : 0.f;      // hardware reciprocals (1 ulp), as in the
            const float scale = tail ? __builtin_amdgcn_rcpf(alpha - beta) : 0.f;             // panel kernel of the blocked QR
            const float w = fmaf(scale, s, top);                       // v^T (column c)
            const float tw = tau * w;
            mine[j] = top - tw;
            const float f = tw * scale;
            {
                const f32x4_t x = *reinterpret_cast<const f32x4_t*>(piv + r0);
                f32x4_t y = *reinterpret_cast<const f32x4_t*>(mine + r0);
#pragma unroll
                for (int t = 0; t < 4; ++t) y[t] = r0 + t > j ? fmaf(-f, x[t], y[t]) : y[t];
                *reinterpret_cast<f32x4_t*>(mine + r0) = y;
            }
#pragma unroll 4
            for (int r = r0 + 4; r < n; r += 4) {
                const f32x4_t x = *reinterpret_cast<const f32x4_t*>(piv + r);
                f32x4_t y = *reinterpret_cast<const f32x4_t*>(mine + r);
#pragma unroll
                for (int t = 0; t < 4; ++t) y[t] = fmaf(-f, x[t], y[t]);
                *reinterpret_cast<f32x4_t*>(mine + r) = y;
            }
            if (c == j + 1) rdiag[j] = beta;                           // the diagonal of R: (alpha, x) becomes (beta, 0)
        }
        __syncthreads();
    }

    // column n + i of W is row i of Q.  A = Q diag(sign r_ii); A^-1 = A^T; both zero beyond column n.
    float* A32 = (float*)(block + a.t.off_A32);
    float* Ai32 = (float*)(block + a.t.off_Ainv32);
    uint16_t* A16 = a.t.off_A16 >= 0 ? (uint16_t*)(block + a.t.off_A16) : nullptr;
    uint16_t* Ai16 = a.t.off_A16 >= 0 ? (uint16_t*)(block + a.t.off_Ainv16) : nullptr;
    const int ldk = (int)a.ldk;
    for (int e = tid; e < n * ldk; e += 256) {
        const int i = e / ldk, cc = e - i * ldk;
        float x = 0.f, xt = 0.f;
        if (cc < n) {
            x = W[(n + i) * ldc + cc];
            if (rdiag[cc] < 0.f) x = -x;
            xt = W[(n + cc) * ldc + i];
            if (rdiag[i] < 0.f) xt = -xt;
        }
        A32[e] = x;
        Ai32[e] = xt;
        if (A16) {
            const __bf16 h = (__bf16)x, ht = (__bf16)xt;
            A16[e] = __builtin_bit_cast(uint16_t, h);
            Ai16[e] = __builtin_bit_cast(uint16_t, ht);
        }
    }
}

// ---------------------------------------------------------------------------------------------- mix --
struct SmallMixArgs {
    const uint16_t* A16; int64_t ldk;
    const uint16_t* H; int64_t ldh;
    const float* GS; const float* gsnorm; const float* rownorm;
    int stat_kind; float shield_scale;
    int n_data, k, d;
    uint16_t* S; uint16_t* U; int64_t ldu;
};

constexpr int MIX_BN = 64;           // columns of U per workgroup
constexpr int MIX_KP = 128 + 8;      // pitch (bf16) of a column of the transposed operand tile in LDS

// One workgroup: 64 columns of U.  The operand tile [H ; S] (n x 64) is stored transposed in LDS (column-major,
// K contiguous) so that a lane's eight contraction values are one 16-byte read; wave w owns rows 32 w .. 32 w + 31
// of U and reads its rows of A straight from memory (A is zero beyond column n up to its pitch).
__global__ __launch_bounds__(256)
void small_mix_kernel(SmallMixArgs a) {
    __shared__ __attribute__((aligned(16))) uint16_t Bt[MIX_BN * MIX_KP];
    __shared__ float norms[kSmallMaxN];
    __shared__ float factor[kSmallMaxN];
    __shared__ float stat_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = a.n_data + a.k, c0 = blockIdx.x * MIX_BN;
    const int kp = (n + 15) & ~15;
    const int j = lane & 31, grp = lane >> 5;

    // Every load from memory is issued before anything waits: the kernel is a chain of a few dependent steps, and
    // one memory latency per step would be most of its run time.
    const float my_norm = (a.k > 0 && tid < a.n_data) ? a.rownorm[tid] : 0.f;
    const float my_gsnorm = tid < a.k ? a.gsnorm[tid] : 1.f;
    constexpr int HR = kSmallMaxN * (MIX_BN / 8) / 256;          // 16-byte chunks of H per thread: at most 4
    u32x4_t hreg[HR];
#pragma unroll
    for (int it = 0; it < HR; ++it) {
        const int i = tid + it * 256;
        const int r = i >> 3, col = c0 + (i & 7) * 8;
        hreg[it] = u32x4_t{0u, 0u, 0u, 0u};
        if (r < a.n_data && col < a.d) hreg[it] = *reinterpret_cast<const u32x4_t*>(a.H + (int64_t)r * a.ldh + col);
    }
    constexpr int GR = 4;                                        // shield values per thread held in registers (k <= 16)
    float gsv[GR];
#pragma unroll
    for (int it = 0; it < GR; ++it) {
        const int i = tid + it * 256;
        const int r = i / MIX_BN, col = c0 + (i - r * MIX_BN);
        gsv[it] = (r < a.k && col < a.d) ? a.GS[(int64_t)r * a.d + col] : 0.f;
    }
    bf16x8_t af[kSmallMaxN / 16];
    {
        int arow = wave * 32 + j; arow = arow < n ? arow : n - 1;
        const uint16_t* ap = a.A16 + (int64_t)arow * a.ldk + grp * 8;
#pragma unroll
        for (int ks = 0; ks < kSmallMaxN / 16; ++ks)
            if (ks * 16 < kp && wave * 32 < n) af[ks] = *reinterpret_cast<const bf16x8_t*>(ap + ks * 16);
    }

    if (a.k > 0) {
        if (tid < a.n_data) norms[tid] = my_norm;
        __syncthreads();
        if (a.stat_kind == 0) {
            // median by rank: every value counts the (value, index) pairs below it; the two of middle rank meet in the mean
            if (tid < a.n_data) {
                const uint32_t mine = __float_as_uint(my_norm);
                int below = 0;
                for (int i = 0; i < a.n_data; ++i) {
                    const uint32_t o = __float_as_uint(norms[i]);
                    below += (o < mine || (o == mine && i < tid)) ? 1 : 0;
                }
                if (below == (a.n_data - 1) / 2) factor[0] = my_norm;
                if (below == a.n_data / 2) factor[1] = my_norm;
            }
            __syncthreads();
            if (tid == 0) stat_s = 0.5f * (factor[0] + factor[1]);
        } else if (tid == 0) {
            float s = 0.f;
            for (int i = 0; i < a.n_data; ++i) s += norms[i];
            stat_s = s / (float)a.n_data;
        }
        __syncthreads();
        const float m = stat_s;
        __syncthreads();
        if (tid < a.k) factor[tid] = a.shield_scale * m / my_gsnorm;
    }
    // zero the K padding of the tile, then fill it: rows of H as 16-byte chunks of 8 columns, shield rows scaled on the way
    for (int i = tid; i < MIX_BN * (MIX_KP / 2); i += 256) reinterpret_cast<uint32_t*>(Bt)[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < HR; ++it) {
        const int i = tid + it * 256;
        const int r = i >> 3, ch = i & 7;
        if (r < a.n_data && c0 + ch * 8 < a.d) {                 // d is a multiple of 8: a chunk is inside or outside
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Bt[(ch * 8 + 2 * t) * MIX_KP + r] = (uint16_t)(hreg[it][t] & 0xFFFFu);
                Bt[(ch * 8 + 2 * t + 1) * MIX_KP + r] = (uint16_t)(hreg[it][t] >> 16);
            }
        }
    }
    for (int i = tid, it = 0; i < a.k * MIX_BN; i += 256, ++it) {
        const int r = i / MIX_BN, cc = i - r * MIX_BN;
        const int col = c0 + cc;
        if (col >= a.d) continue;
        float gsx;
        switch (it) { case 0: gsx = gsv[0]; break; case 1: gsx = gsv[1]; break; case 2: gsx = gsv[2]; break; case 3: gsx = gsv[3]; break;
                      default: gsx = a.GS[(int64_t)r * a.d + col]; }
        const __bf16 h = (__bf16)(gsx * factor[r]);
        const uint16_t bits = __builtin_bit_cast(uint16_t, h);
        a.S[(int64_t)r * a.d + col] = bits;
        Bt[cc * MIX_KP + a.n_data + r] = bits;
    }
    __syncthreads();
    if (wave * 32 >= n) return;
    // v_mfma_f32_32x32x16_bf16: lane l supplies row l % 32 of A and column l % 32 of B, contraction values
    // 8 (l / 32) .. + 7; it receives column l % 32, rows 8 (v / 4) + 4 (l / 32) + v % 4
    f32x16_t acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < kSmallMaxN / 16; ++ks) {
        if (ks * 16 < kp) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8_t bf = *reinterpret_cast<const bf16x8_t*>(Bt + (t * 32 + j) * MIX_KP + ks * 16 + grp * 8);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks], bf, acc[t], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int col = c0 + t * 32 + j;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = wave * 32 + 8 * (v >> 2) + 4 * grp + (v & 3);
            if (row < n && col < a.d) {
                const __bf16 h = (__bf16)acc[t][v];
                a.U[(int64_t)row * a.ldu + col] = __builtin_bit_cast(uint16_t, h);
            }
        }
    }
}

}  // namespace

hipError_t small_init() {
    const int ldc = small_ldc(kSmallMaxN);
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&small_sample_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               2 * kSmallMaxN * ldc * (int)sizeof(float));
}

hipError_t small_sample(const SmallSampleTargets& t, int count, uint64_t first_batch, PhiloxStream ps, uint32_t c1_shield,
                        int n, int k, int d, int64_t ldk, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    if (count > kSmallMaxBatch || n < 1 || n > kSmallMaxN || k < 0 || ldk < n) return hipErrorInvalidValue;
    SmallSampleArgs a;
    a.t = t;
    a.key0 = ps.key0; a.key1 = ps.key1; a.c1_mix = ps.c1; a.c1_shield = c1_shield;
    a.first_batch = first_batch;
    a.n = n; a.k = k; a.d = d; a.ldk = ldk;
    const size_t lds = (size_t)2 * n * small_ldc(n) * sizeof(float);
    hipLaunchKernelGGL(small_sample_kernel, dim3((unsigned)(count * (1 + k))), dim3(256), lds, stream, a);
    return hipGetLastError();
}

hipError_t small_mix(const uint16_t* A16, int64_t ldk, const uint16_t* H, int64_t ldh, const float* GS, const float* gsnorm,
                     const float* rownorm, int stat_kind, float shield_scale, int n_data, int k, int d,
                     uint16_t* S, uint16_t* U, int64_t ldu, hipStream_t stream) {
    const int n = n_data + k;
    if (n < 1 || n > kSmallMaxN || d < 8 || d % 8 != 0 || ldk < ((n + 15) & ~15)) return hipErrorInvalidValue;
    SmallMixArgs a;
    a.A16 = A16; a.ldk = ldk; a.H = H; a.ldh = ldh; a.GS = GS; a.gsnorm = gsnorm; a.rownorm = rownorm;
    a.stat_kind = stat_kind; a.shield_scale = shield_scale; a.n_data = n_data; a.k = k; a.d = d;
    a.S = S; a.U = U; a.ldu = ldu;
    hipLaunchKernelGGL(small_mix_kernel, dim3((unsigned)((d + MIX_BN - 1) / MIX_BN)), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace gelo
