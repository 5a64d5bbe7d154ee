// Structured orthogonal mixing: A = P_R (B D_{R-1} P_{R-1}) ... (B D_0 P_0) with random row
// permutations P_r, random sign flips D_r and B the normalised Walsh-Hadamard transform on the
// row blocks given by the binary expansion of n (largest block first).  The paper's Conclusion
// names structured orthogonal transforms as the way to cheaper fresh mixing and gives no
// construction; this one is the library's own.  Every factor is orthogonal, so A^-1 = A^T, and
// applying A or A^T to a column costs O(n log n) additions instead of n^2 multiply-adds.
//
// A and A^T are never formed.  One workgroup owns a strip of CW columns of the operand, keeps all
// n rows of it in LDS (float), and runs every permutation, sign flip and butterfly stage there:
// the operand is read from HBM once and the result written once, which is what bounds the kernel
// from below; the butterflies are plain vector additions (a +-1 matrix product on the matrix cores
// would be no faster in float and the work is not a contraction worth reshaping).
#include "gelo_internal.h"

namespace gelo {
namespace {

constexpr uint32_t kStreamPerm = 3, kStreamSign = 4;   // Philox streams of the sort keys / the signs
constexpr uint32_t kSignBit = 0x80000000u;

// ------------------------------------------------------------------ the random tables --
// Permutation b sorts n Philox words (stream kStreamPerm, sub-stream b) as (key, index) pairs:
// entry j is the index of the j-th smallest pair.  Each index finds its rank by counting the pairs
// below it - n^2 comparisons, spread over n / 64 workgroups, no sorting network and no
// ambiguity among equal keys.  The sign of position j in round b < rounds is the top bit of word
// j of stream kStreamSign, sub-stream b.  table[b * n + j] = index | sign bit.
__global__ __launch_bounds__(256)
void structured_tables_kernel(uint32_t* table, int n, int rounds, PhiloxStream ps) {
    extern __shared__ __align__(16) uint32_t keys[];         // n rounded up to 4
    __shared__ int part_count[4][64];
    const int b = blockIdx.y, tid = threadIdx.x;
    for (int q = tid; q * 4 < n; q += 256) {
        uint32_t c0 = (uint32_t)q, c1 = (kStreamPerm << 8) | (uint32_t)b, c2 = ps.c2, c3 = ps.c3;
        philox4x32_10(c0, c1, c2, c3, ps.key0, ps.key1);
        // past the end: the largest key, so that with its index >= n such a pair is above every real one
        keys[4 * q] = c0;
        keys[4 * q + 1] = 4 * q + 1 < n ? c1 : 0xFFFFFFFFu;
        keys[4 * q + 2] = 4 * q + 2 < n ? c2 : 0xFFFFFFFFu;
        keys[4 * q + 3] = 4 * q + 3 < n ? c3 : 0xFFFFFFFFu;
    }
    __syncthreads();
    const int slot = tid & 63, part = tid >> 6;
    const int i = blockIdx.x * 64 + slot;
    int below = 0;
    if (i < n) {
        const uint32_t ki = keys[i];
        const uint4* keys4 = reinterpret_cast<const uint4*>(keys);
        const int quads = (n + 3) / 4, chunk = (quads + 3) / 4;
        const int lo = part * chunk, hi = min(quads, lo + chunk);
        // (key, index) pairs compared as 64-bit numbers: no branch on equal keys
        const uint64_t mine = ((uint64_t)ki << 32) | (uint32_t)i;
        auto is_below = [&](uint32_t kk, int k) { return ((((uint64_t)kk << 32) | (uint32_t)k) < mine) ? 1 : 0; };
#pragma unroll 8
        for (int qd = lo; qd < hi; ++qd) {                   // every lane reads the same four keys: a broadcast
            const uint4 kk = keys4[qd];
            below += is_below(kk.x, 4 * qd) + is_below(kk.y, 4 * qd + 1) + is_below(kk.z, 4 * qd + 2) + is_below(kk.w, 4 * qd + 3);
        }
    }
    part_count[part][slot] = below;
    __syncthreads();
    if (part != 0 || i >= n) return;
    const int rank = part_count[0][slot] + part_count[1][slot] + part_count[2][slot] + part_count[3][slot];
    uint32_t sign = 0;
    if (b < rounds) {
        uint32_t c0 = (uint32_t)(rank >> 2), c1 = (kStreamSign << 8) | (uint32_t)b, c2 = ps.c2, c3 = ps.c3;
        philox4x32_10(c0, c1, c2, c3, ps.key0, ps.key1);
        const int w = rank & 3;
        const uint32_t word = w == 0 ? c0 : w == 1 ? c1 : w == 2 ? c2 : c3;
        sign = word & kSignBit;
    }
    table[(int64_t)b * n + rank] = (uint32_t)i | sign;
}

// ------------------------------------------------------------------------ the transform --
struct StructuredArgs {
    const void* in0; int64_t ld0; int rows0;   // rows [0, rows0) of the operand
    const void* in1; int64_t ld1;              // rows [rows0, n) (the shield rows of a mix)
    void* out; int64_t ldo; int rows_out;      // result rows >= rows_out are not stored
    const uint32_t* table;                     // (rounds + 1) x n, see structured_tables_kernel
    int n, ncols, rounds, inverse;
};

// Row r of the strip sits at LDS row r + r / 16: one empty row after every 16.  Without it the first
// butterfly pass, whose neighbouring lanes hold neighbouring groups of 16 rows, would put them all on
// the same banks; with it every pass is free of bank conflicts, and the LDS rows of a butterfly
// first + j 2^s0 are the first one plus offsets that depend on j and s0 only (lds_offset): one
// address per item, the rest scalar.
__device__ __forceinline__ int lds_row(int r) { return r + (r >> 4); }
__device__ __forceinline__ int lds_offset(int j, int s0) { return (j << s0) + ((j << s0) >> 4); }
inline size_t lds_rows(int n) { const size_t p = (size_t)round_up(n, 16); return p + p / 16; }

// exponent of the block of row r < n: the highest bit in which r and n differ (there n has a one:
// r lies in the block that this bit of n stands for)
__device__ __forceinline__ int block_exponent(int r, int n) { return 31 - __clz(r ^ n); }

// 2^(-e/2): the normalisation of a Walsh-Hadamard block of 2^e rows
__device__ __forceinline__ float block_scale(int e) {
    return ldexpf((e & 1) ? 0.70710678118654752f : 1.0f, -(e >> 1));
}

__device__ __forceinline__ float4 scaled(float4 v, float s) { return make_float4(v.x * s, v.y * s, v.z * s, v.w * s); }
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float4 sub4(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v = {(__bf16)lo, (__bf16)hi};                  // round to nearest even
    return __builtin_bit_cast(uint32_t, v);
}

template <typename T>
__device__ __forceinline__ float4 load_quad(const T* p);
template <>
__device__ __forceinline__ float4 load_quad<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <>
__device__ __forceinline__ float4 load_quad<uint16_t>(const uint16_t* p) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u),
                       __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xFFFF0000u));
}
__device__ __forceinline__ void store_quad(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store_quad(uint16_t* p, float4 v) {
    *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
}

// NS butterfly stages s0 .. s0 + NS - 1 on the 2^NS rows first + j 2^s0 of quad column q, which the
// caller knows to lie in one block of at least 2^(s0 + NS) rows (so bits s0 .. s0 + NS - 1 of `first`
// are zero, which is what makes lds_offset exact): registers, one LDS read and one write per row.
template <int QW, int NS>
__device__ __forceinline__ void butterfly_rows(float4* X, int first, int s0, int q) {
    constexpr int RW = 1 << NS;
    float4* x0 = X + lds_row(first) * QW + q;
    float4 v[RW];
#pragma unroll
    for (int j = 0; j < RW; ++j) v[j] = x0[lds_offset(j, s0) * QW];
#pragma unroll
    for (int k = 0; k < NS; ++k)
#pragma unroll
        for (int j = 0; j < RW; ++j)
            if (!(j & (1 << k))) {
                const float4 a = v[j], c = v[j | (1 << k)];
                v[j] = add4(a, c);
                v[j | (1 << k)] = sub4(a, c);
            }
#pragma unroll
    for (int j = 0; j < RW; ++j) x0[lds_offset(j, s0) * QW] = v[j];
}

// One pass of the block Walsh-Hadamard transform: stages s0 .. s0 + NS - 1 (stage s pairs rows 2^s
// apart and applies to a row only while s is below its block's exponent).  A work item is one quad
// of columns of the 2^NS rows base + j 2^s0.  Usually their aligned range of 2^(s0 + NS) rows lies
// in one block and the item is one butterfly.  At the end of the strip it straddles smaller blocks:
// then it is cut, block by block, into the shorter butterflies each block still needs in this pass
// (blocks come in decreasing size, so every piece starts at a multiple of its own length).
template <int QW, int NS>
__device__ __forceinline__ void hadamard_pass(float4* X, int n, int s0) {
    constexpr int RW = 1 << NS;
    const int tid = threadIdx.x;
    const int span = RW << s0;
    const int groups = ((n + span - 1) / span) << s0;        // items per quad column
#pragma unroll 1
    for (int t = tid; t < groups * QW; t += 512) {
        const int q = t % QW, gi = t / QW;
        const int base = ((gi >> s0) << (s0 + NS)) | (gi & ((1 << s0) - 1));
        if (base >= n) continue;
        if (block_exponent(base, n) >= s0 + NS) {
            butterfly_rows<QW, NS>(X, base, s0, q);
            continue;
        }
#pragma unroll 1
        for (int j0 = 0; j0 < RW;) {
            const int first = base + (j0 << s0);
            if (first >= n) break;
            const int ns = block_exponent(first, n) - s0;    // stages this block still needs; below NS here
            if (ns <= 0) break;                              // and no later block needs any
            if (NS > 3 && ns == 3) butterfly_rows<QW, 3>(X, first, s0, q);
            else if (NS > 2 && ns == 2) butterfly_rows<QW, 2>(X, first, s0, q);
            else butterfly_rows<QW, 1>(X, first, s0, q);
            j0 += 1 << ns;
        }
    }
}

// B: all passes, four stages at a time and what is left in the last.  Leaves the strip unnormalised;
// the factor 2^(-e/2) of each row is applied where the row is read next (the permutation that
// follows, or the store).
template <int QW>
__device__ __forceinline__ void block_hadamard(float4* X, int n) {
    const int top = 31 - __clz(n);                           // exponent of the largest block
#pragma unroll 1
    for (int s0 = 0; s0 < top; s0 += 4) {
        const int ns = min(4, top - s0);
        if (ns == 4) hadamard_pass<QW, 4>(X, n, s0);
        else if (ns == 3) hadamard_pass<QW, 3>(X, n, s0);
        else if (ns == 2) hadamard_pass<QW, 2>(X, n, s0);
        else hadamard_pass<QW, 1>(X, n, s0);
        __syncthreads();
    }
}

constexpr int kMaxQuads = 20;      // quads per thread: a strip has fewer than 512 x 20 of them (160 KB of LDS)

// T: float or uint16_t (bf16 bits).  CW columns per workgroup, 512 threads, lds_rows(n) x CW floats of LDS.
// In the permutations between the rounds a thread owns whole rows of the strip (rows tid, tid + 512, ...):
// one table entry, one sign, one scale and one pair of row addresses serve all the columns of a row.
template <typename T, int CW>
__global__ __launch_bounds__(512)
void structured_apply_kernel(StructuredArgs a) {
    constexpr int QW = CW / 4;
    constexpr int RP = kMaxQuads / QW;                       // rows per thread at most
    static_assert(RP >= 1, "strip too wide for one row per thread");
    extern __shared__ float4 X[];
    const int tid = threadIdx.x, n = a.n, R = a.rounds;
    // consecutive strips go to consecutive workgroups of ONE accelerator die (workgroups are dealt
    // round-robin over the 8 dies): neighbours in a row share cache lines of the operand
    const int nstrips = (a.ncols + CW - 1) / CW, per_die = (nstrips + 7) / 8;
    const int strip = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (strip >= nstrips) return;
    const int col0 = strip * CW;
    const int quads = min(QW, (a.ncols - col0) / 4);         // a ragged last strip has fewer
    const int total = n * QW;
    const uint32_t* tab_in = a.table + (int64_t)(a.inverse ? R : 0) * n;
    const uint32_t* tab_out = a.table + (int64_t)(a.inverse ? 0 : R) * n;

    // ---- load: forward x[j] = sign_0[j] in[perm_0[j]];  transposed x[perm_R[j]] = in[j]
    // Here and in the store a work item is one quad of one row, quads of a row on neighbouring lanes:
    // a wave's access touches 16 rows, not 64.  Unrolled over the thread's items so that its table
    // reads, then its operand loads, overlap.
    {
        uint32_t entry[kMaxQuads];
#pragma unroll
        for (int it = 0; it < kMaxQuads; ++it) {
            const int t = tid + 512 * it;
            entry[it] = t < total ? tab_in[t / QW] : 0u;
        }
        float4 v[kMaxQuads];
#pragma unroll
        for (int it = 0; it < kMaxQuads; ++it) {
            const int t = tid + 512 * it;
            const int q = t % QW, j = t / QW;
            if (t < total && q < quads) {
                const int src = a.inverse ? j : (int)(entry[it] & ~kSignBit);
                const T* row = src < a.rows0 ? (const T*)a.in0 + (int64_t)src * a.ld0 : (const T*)a.in1 + (int64_t)(src - a.rows0) * a.ld1;
                v[it] = load_quad<T>(row + col0 + 4 * q);
            }
        }
#pragma unroll
        for (int it = 0; it < kMaxQuads; ++it) {
            const int t = tid + 512 * it;
            const int q = t % QW, j = t / QW;
            if (t < total && q < quads) {
                const int dst = a.inverse ? (int)(entry[it] & ~kSignBit) : j;
                X[lds_row(dst) * QW + q] = scaled(v[it], (entry[it] & kSignBit) ? -1.f : 1.f);
            }
        }
    }
    __syncthreads();

    // ---- rounds: B, then (all but the last) sign flip and permutation of the next round
#pragma unroll 1
    for (int r = 1; r <= R; ++r) {
        block_hadamard<QW>(X, n);
        if (r == R) break;
        const uint32_t* tab = a.table + (int64_t)(a.inverse ? R - r : r) * n;
        float4 held[RP][QW];
        int where[RP];                                       // LDS row each held row goes to
#pragma unroll
        for (int it = 0; it < RP; ++it) {
            const int j = tid + 512 * it;
            if (j < n) {
                const uint32_t entry = tab[j];
                const int other = (int)(entry & ~kSignBit);
                const int src = a.inverse ? j : other, dst = a.inverse ? other : j;
                const float s = block_scale(block_exponent(src, n));
                const float f = (entry & kSignBit) ? -s : s;
                const float4* xr = X + lds_row(src) * QW;
#pragma unroll
                for (int q = 0; q < QW; ++q) held[it][q] = scaled(xr[q], f);
                where[it] = lds_row(dst) * QW;
            }
        }
        __syncthreads();                                     // every row is read before any is overwritten
#pragma unroll
        for (int it = 0; it < RP; ++it)
            if (tid + 512 * it < n) {
#pragma unroll
                for (int q = 0; q < QW; ++q) X[where[it] + q] = held[it][q];
            }
        __syncthreads();
    }

    // ---- store: forward out[j] = x[perm_R[j]];  transposed out[perm_0[j]] = sign_0[j] x[j]
    {
        // index arithmetic redone from an opaque copy of the thread number: values shared with the load
        // phase would otherwise stay in registers across the whole kernel and spill
        int tid_s = tid;
        asm volatile("" : "+v"(tid_s));
        uint32_t entry[kMaxQuads];
#pragma unroll
        for (int it = 0; it < kMaxQuads; ++it) {
            const int t = tid_s + 512 * it;
            entry[it] = t < total ? tab_out[t / QW] : 0u;
        }
#pragma unroll
        for (int it = 0; it < kMaxQuads; ++it) {
            const int t = tid_s + 512 * it;
            const int q = t % QW, j = t / QW;
            if (t >= total || q >= quads) continue;
            const int other = (int)(entry[it] & ~kSignBit);
            const int src = a.inverse ? j : other, dst = a.inverse ? other : j;
            if (dst >= a.rows_out) continue;
            const float s = block_scale(block_exponent(src, n));
            const float4 v = scaled(X[lds_row(src) * QW + q], (entry[it] & kSignBit) ? -s : s);
            store_quad((T*)a.out + (int64_t)dst * a.ldo + col0 + 4 * q, v);
        }
    }
}

int g_lds_cap = 0;                 // bytes of LDS one workgroup may use (set by structured_init)

template <typename T, int CW>
hipError_t allow_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&structured_apply_kernel<T, CW>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, g_lds_cap);
}

template <typename T, int CW>
hipError_t launch_apply(const StructuredArgs& a, size_t lds, hipStream_t s) {
    const int nstrips = (a.ncols + CW - 1) / CW;
    hipLaunchKernelGGL((structured_apply_kernel<T, CW>), dim3(((nstrips + 7) / 8) * 8), dim3(512), lds, s, a);
    return hipGetLastError();
}

// 16 columns per workgroup while the strip fits in LDS (2400 rows), then 8 (4816 rows), then 4.  (Half-size
// workgroups, two per CU, so that one's loads overlap the other's butterflies, were 8% slower: the
// kernel is bound by vector-ALU issue, not by its memory phases.)  Short strips (decode-shaped
// batches of at most 512 rows) take 64 columns: a workgroup's fixed cost - a dozen barriers and four
// dependent trips to memory - is then paid by 64 instead of 256 or 768 workgroups.
template <typename T>
hipError_t dispatch_apply(const StructuredArgs& a, hipStream_t s) {
    const size_t rows = lds_rows(a.n);
    if (a.n <= 512 && a.ncols >= 2048) return launch_apply<T, 64>(a, rows * 256, s);
    if (rows * 64 <= (size_t)g_lds_cap) return launch_apply<T, 16>(a, rows * 64, s);
    if (rows * 32 <= (size_t)g_lds_cap) return launch_apply<T, 8>(a, rows * 32, s);
    if (rows * 16 <= (size_t)g_lds_cap) return launch_apply<T, 4>(a, rows * 16, s);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t structured_init() {
    int dev = 0, cap = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cap, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;
    g_lds_cap = cap < 160 * 1024 ? cap : 160 * 1024;
    if (g_lds_cap < 64 * 1024) return hipErrorInvalidDevice;
    if ((e = allow_lds<float, 64>()) != hipSuccess) return e;
    if ((e = allow_lds<uint16_t, 64>()) != hipSuccess) return e;
    if ((e = allow_lds<float, 16>()) != hipSuccess) return e;
    if ((e = allow_lds<float, 8>()) != hipSuccess) return e;
    if ((e = allow_lds<float, 4>()) != hipSuccess) return e;
    if ((e = allow_lds<uint16_t, 16>()) != hipSuccess) return e;
    if ((e = allow_lds<uint16_t, 8>()) != hipSuccess) return e;
    return allow_lds<uint16_t, 4>();
}

int structured_max_rows() { return g_lds_cap / 16 / 17 * 16; }   // 4 columns of floats per row, one padding row per 16

hipError_t structured_tables(uint32_t* table, int n, int rounds, PhiloxStream ps, hipStream_t s) {
    const size_t lds = (size_t)round_up(n, 4) * sizeof(uint32_t);
    hipLaunchKernelGGL(structured_tables_kernel, dim3((n + 63) / 64, rounds + 1), dim3(256), lds, s, table, n, rounds, ps);
    return hipGetLastError();
}

hipError_t structured_apply(const StructuredOperands& o, int is_bf16, hipStream_t s) {
    StructuredArgs a;
    a.in0 = o.in0; a.ld0 = o.ld0; a.rows0 = o.rows0;
    a.in1 = o.in1 ? o.in1 : o.in0; a.ld1 = o.in1 ? o.ld1 : o.ld0;
    a.out = o.out; a.ldo = o.ldo; a.rows_out = o.rows_out;
    a.table = o.table; a.n = o.n; a.ncols = o.ncols; a.rounds = o.rounds; a.inverse = o.transposed ? 1 : 0;
    return is_bf16 ? dispatch_apply<uint16_t>(a, s) : dispatch_apply<float>(a, s);
}

}  // namespace gelo
