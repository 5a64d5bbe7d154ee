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
constexpr int kThreads = 640;                          // of a transform workgroup: ten waves

// ------------------------------------------------------------------ the random tables --
// Permutation b sorts n Philox words (stream kStreamPerm, sub-stream b) as (key, index) pairs:
// entry j is the index of the j-th smallest pair.  Each index finds its rank by counting the pairs
// below it - n^2 comparisons, spread over n / 64 workgroups, no sorting network and no
// ambiguity among equal keys.  The sign of position j in round b < rounds is the top bit of word
// j of stream kStreamSign, sub-stream b.  table[b * np + j] = index | sign bit (np = n rounded up to 4
// words: every table starts on a 16-byte boundary).  Behind the rounds + 1 tables lie their inverses, which
// the transposed transform gathers by: table[(rounds + 1 + b) * np + index] = j | the same sign bit.
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
    const int np = (n + 3) & ~3;
    table[(int64_t)b * np + rank] = (uint32_t)i | sign;
    table[(int64_t)(rounds + 1 + b) * np + i] = (uint32_t)rank | sign;
}

// ------------------------------------------------------------------------ the transform --
struct StructuredArgs {
    const void* in0; int64_t ld0; int rows0;   // rows [0, rows0) of the operand
    const void* in1; int64_t ld1;              // rows [rows0, n) (the shield rows of a mix)
    void* out; int64_t ldo; int rows_out;      // result rows >= rows_out are not stored
    const uint32_t* table;                     // 2 (rounds + 1) tables, see structured_tables_kernel
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

// An item whose 2^NS rows base + j 2^s0 straddle blocks too small for all NS stages (the end of the strip):
// cut, block by block, into the shorter butterflies each block still needs in this pass (blocks come in
// decreasing size, so every piece starts at a multiple of its own length).  (All pieces in registers at
// once, every pair under a condition of its own, was tried: several times slower.)
template <int QW, int NS>
__device__ __forceinline__ void straddling_item(float4* X, int n, int base, int s0, int q) {
    constexpr int RW = 1 << NS;
#pragma unroll 1
    for (int j0 = 0; j0 < RW;) {
        const int first = base + (j0 << s0);
        if (first >= n) break;
        const int ns = block_exponent(first, n) - s0;        // stages this block still needs; below NS here
        if (ns <= 0) break;                                  // and no later block needs any
        if (NS > 3 && ns == 3) butterfly_rows<QW, 3>(X, first, s0, q);
        else if (NS > 2 && ns == 2) butterfly_rows<QW, 2>(X, first, s0, q);
        else butterfly_rows<QW, 1>(X, first, s0, q);
        j0 += 1 << ns;
    }
}

// One pass of the block Walsh-Hadamard transform: stages s0 .. s0 + NS - 1 (stage s pairs rows 2^s
// apart and applies to a row only while s is below its block's exponent).  A work item is one quad
// of columns of the 2^NS rows base + j 2^s0.  Usually their aligned range of 2^(s0 + NS) rows lies
// in one block and the item is one butterfly.  At the end of the strip it straddles smaller blocks
// (straddling_item).
template <int QW, int NS>
__device__ __forceinline__ void hadamard_pass(float4* X, int n, int s0) {
    constexpr int RW = 1 << NS;
    const int tid = threadIdx.x;
    const int span = RW << s0;
    const int groups = ((n + span - 1) / span) << s0;        // items per quad column
#pragma unroll 1
    for (int t = tid; t < groups * QW; t += kThreads) {
        const int q = t % QW, gi = t / QW;
        const int base = ((gi >> s0) << (s0 + NS)) | (gi & ((1 << s0) - 1));
        if (base >= n) continue;
        if (block_exponent(base, n) >= s0 + NS) {
            butterfly_rows<QW, NS>(X, base, s0, q);
            continue;
        }
        straddling_item<QW, NS>(X, n, base, s0, q);
    }
}

// The passes of B from stage s0 on, four stages at a time and what is left in the last.  Leaves the strip
// unnormalised; the factor 2^(-e/2) of each row is applied where the row is read next (the gather
// that follows, or the store).
template <int QW>
__device__ __forceinline__ void block_hadamard_from(float4* X, int n, int first_s0) {
    const int top = 31 - __clz(n);                           // exponent of the largest block
#pragma unroll 1
    for (int s0 = first_s0; s0 < top; s0 += 4) {
        const int ns = min(4, top - s0);
        if (ns == 4) hadamard_pass<QW, 4>(X, n, s0);
        else if (ns == 3) hadamard_pass<QW, 3>(X, n, s0);
        else if (ns == 2) hadamard_pass<QW, 2>(X, n, s0);
        else hadamard_pass<QW, 1>(X, n, s0);
        __syncthreads();
    }
}

// Stages 0 .. 3 of B on 16 consecutive rows of one block that a thread holds in registers.
__device__ __forceinline__ void first_stages(float4 (&v)[16]) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (!(j & (1 << k))) {
                const float4 a = v[j], c = v[j | (1 << k)];
                v[j] = add4(a, c);
                v[j | (1 << k)] = sub4(a, c);
            }
}

// 16-byte pieces of a table a thread carries from memory to LDS: the narrower the strip, the more rows it may have
constexpr int table_pieces(int cw) { return cw == 4 ? 4 : cw == 8 ? 2 : 1; }

// T: float or uint16_t (bf16 bits).  CW columns per workgroup, kThreads threads; LDS holds lds_rows(n) x CW
// floats and, behind them, one table of round_up(n, 4) words.
//
// Both directions are gathers: with the table T_s of step s (forward: permutation s and its signs; transposed:
// the inverse of permutation R - s with the signs carried along) every step reads new[j] = +-scale x old[T_s[j]].
// A thread owns ONE item of the gathers: 16 consecutive rows of one quad of columns (the dispatcher only picks
// strip widths with at most kThreads such items).  It gathers its rows into registers - from memory in step 0,
// from the strip in the steps between the rounds -, runs the first four butterfly stages of the round there
// and writes the rows back in place: the permutation between two rounds costs no pass of its own and the
// first pass of every round no trip through LDS.  The table of the next step is fetched from memory before
// the passes of a round and parked in LDS behind them.
template <typename T, int CW>
__global__ __launch_bounds__(kThreads)
void structured_apply_kernel(StructuredArgs a) {
    constexpr int QW = CW / 4;
    extern __shared__ float4 X[];
    const int tid = threadIdx.x, n = a.n, R = a.rounds;
    const int np = (n + 3) & ~3;                             // words per table
    uint32_t* tbl = reinterpret_cast<uint32_t*>(X + (size_t)lds_row(((n + 15) & ~15)) * QW);
    // consecutive strips go to consecutive workgroups of ONE accelerator die (workgroups are dealt
    // round-robin over the 8 dies): neighbours in a row share cache lines of the operand
    const int nstrips = (a.ncols + CW - 1) / CW, per_die = (nstrips + 7) / 8;
    const int strip = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (strip >= nstrips) return;
    const int col0 = strip * CW;
    const int quads = min(QW, (a.ncols - col0) / 4);         // a ragged last strip has fewer
    // table of step s: forward table s; transposed the inverse table R - s (they lie behind the R + 1 forward ones)
    auto table_of = [&](int s) { return a.table + (int64_t)(a.inverse ? (R + 1) + (R - s) : s) * np; };

    // The items of the last 16-row group - the ones that may straddle small blocks and then take the slow
    // path - go to the last wave when the others leave it idle, so that the slow path runs beside the
    // common one instead of behind it in a wave that has both.
    const int groups = (n + 15) >> 4, last0 = (groups - 1) * QW;
    int item = tid;
    if (last0 <= kThreads - 64) {
        const int l = tid - (kThreads - 64);
        item = l >= 0 ? (l < QW ? last0 + l : groups * QW) : (tid < last0 ? tid : groups * QW);
    }
    const int q = item % QW, base = (item / QW) * 16;
    const bool active = base < n;
    // the 16 rows of an item usually lie in one block of at least 16 rows: then the first four stages run in
    // registers.  The item at the end of the strip straddles the blocks of 8, 4, 2, 1 rows: it is written back
    // as gathered and takes one more trip through LDS (a thread reads back only what it wrote itself; kept a
    // branch with memory accesses on purpose: merged into the common path as selects it slowed every thread)
    const bool whole = active && block_exponent(base, n) >= 4;
    float4 v[16];

    // ---- step 0: rows gathered from memory, first stages of round 1
    if (active) {
        const uint32_t* t0 = table_of(0) + base;
        uint4 e4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) e4[i] = base + 4 * i < n ? *reinterpret_cast<const uint4*>(t0 + 4 * i) : make_uint4(0u, 0u, 0u, 0u);
        const uint32_t e[16] = {e4[0].x, e4[0].y, e4[0].z, e4[0].w, e4[1].x, e4[1].y, e4[1].z, e4[1].w,
                                e4[2].x, e4[2].y, e4[2].z, e4[2].w, e4[3].x, e4[3].y, e4[3].z, e4[3].w};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (base + j < n && q < quads) {
                const int src = (int)(e[j] & ~kSignBit);
                const T* row = src < a.rows0 ? (const T*)a.in0 + (int64_t)src * a.ld0 : (const T*)a.in1 + (int64_t)(src - a.rows0) * a.ld1;
                v[j] = load_quad<T>(row + col0 + 4 * q);
            }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = scaled(v[j], (e[j] & kSignBit) ? -1.f : 1.f);
        if (whole) first_stages(v);
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (base + j < n) X[lds_row(base + j) * QW + q] = v[j];
        if (!whole) straddling_item<QW, 4>(X, n, base, 0, q);
    }
    __syncthreads();

#pragma unroll 1
    for (int r = 1; r <= R; ++r) {
        // the table of the step behind this round: on its way while the passes run
        constexpr int TQ = table_pieces(CW);                 // 16-byte pieces per thread
        const uint4* tn = reinterpret_cast<const uint4*>(table_of(r));
        uint4 tpre[TQ];
#pragma unroll
        for (int it = 0; it < TQ; ++it) {
            const int i = tid + kThreads * it;
            tpre[it] = 4 * i < n ? tn[i] : make_uint4(0u, 0u, 0u, 0u);
        }
        block_hadamard_from<QW>(X, n, 4);
#pragma unroll
        for (int it = 0; it < TQ; ++it) {
            const int i = tid + kThreads * it;
            if (4 * i < n) reinterpret_cast<uint4*>(tbl)[i] = tpre[it];
        }
        __syncthreads();
        if (r == R) break;
        // ---- step r: rows gathered from the strip (sign and the normalisation of B applied on the way),
        //      all reads before any write, first stages of round r + 1
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = make_float4(0.f, 0.f, 0.f, 0.f);     // (defined on every path: not live across the passes)
        if (active) {
            uint4 e4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) e4[i] = base + 4 * i < n ? *reinterpret_cast<const uint4*>(tbl + base + 4 * i) : make_uint4(0u, 0u, 0u, 0u);
            const uint32_t e[16] = {e4[0].x, e4[0].y, e4[0].z, e4[0].w, e4[1].x, e4[1].y, e4[1].z, e4[1].w,
                                    e4[2].x, e4[2].y, e4[2].z, e4[2].w, e4[3].x, e4[3].y, e4[3].z, e4[3].w};
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (base + j < n) {
                    const int src = (int)(e[j] & ~kSignBit);
                    const float s = block_scale(block_exponent(src, n));
                    v[j] = scaled(X[lds_row(src) * QW + q], (e[j] & kSignBit) ? -s : s);
                }
            }
        }
        __syncthreads();
        if (active) {
            if (whole) first_stages(v);
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (base + j < n) X[lds_row(base + j) * QW + q] = v[j];
            if (!whole) straddling_item<QW, 4>(X, n, base, 0, q);
        }
        __syncthreads();
    }

    // ---- step R: out[j] = scale x strip[T_R[j]]; result rows from rows_out on are not stored (nor read)
    const int out_items = min(a.rows_out, n) * QW;
#pragma unroll 4
    for (int t = tid; t < out_items; t += kThreads) {
        const int qq = t % QW, j = t / QW;
        if (qq >= quads) continue;
        const uint32_t e = tbl[j];
        const int src = (int)(e & ~kSignBit);
        const float s = block_scale(block_exponent(src, n));
        const float4 w = scaled(X[lds_row(src) * QW + qq], (e & kSignBit) ? -s : s);
        store_quad((T*)a.out + (int64_t)j * a.ldo + col0 + 4 * qq, w);
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
    hipLaunchKernelGGL((structured_apply_kernel<T, CW>), dim3(((nstrips + 7) / 8) * 8), dim3(kThreads), lds, s, a);
    return hipGetLastError();
}

// LDS a workgroup needs for a strip of cw columns (the strip as float, one table behind it), or 0 when
// that width cannot serve n rows: the strip must fit and its 16-row x 4-column items must not outnumber
// the threads (a thread owns one)
size_t strip_lds_bytes(int n, int cw) {
    const size_t bytes = lds_rows(n) * (size_t)cw * 4 + (size_t)round_up(n, 4) * 4;
    const int items = (n + 15) / 16 * (cw / 4);
    const bool table_fits = round_up(n, 4) / 4 <= (int64_t)table_pieces(cw) * kThreads;
    return (bytes <= (size_t)g_lds_cap && items <= kThreads && table_fits) ? bytes : 0;
}

// The widest strip that fits: 16 columns per workgroup up to 2272 rows, then 8 (4304 rows), then 4.  (Half-size
// workgroups, two per CU, so that one's loads overlap the other's butterflies, were 8% slower.)  Short strips
// (decode-shaped batches of at most 512 rows) take 64 columns: a workgroup's fixed cost - a dozen barriers and
// three dependent trips to memory - is then paid by 64 instead of 256 or 768 workgroups.
template <typename T>
hipError_t dispatch_apply(const StructuredArgs& a, hipStream_t s) {
    size_t lds;
    if (a.n <= 512 && a.ncols >= 2048 && (lds = strip_lds_bytes(a.n, 64)) != 0) return launch_apply<T, 64>(a, lds, s);
    if ((lds = strip_lds_bytes(a.n, 16)) != 0) return launch_apply<T, 16>(a, lds, s);
    if ((lds = strip_lds_bytes(a.n, 8)) != 0) return launch_apply<T, 8>(a, lds, s);
    if ((lds = strip_lds_bytes(a.n, 4)) != 0) return launch_apply<T, 4>(a, lds, s);
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

int structured_max_rows() {                // the narrowest strip: 4 columns of floats per row, one padding row per 16, the table
    int n = g_lds_cap / 21 / 16 * 16 + 16;
    while (n > 16 && strip_lds_bytes(n, 4) == 0) n -= 16;
    return n;
}

size_t structured_table_words(int n, int rounds) { return (size_t)2 * (rounds + 1) * (size_t)round_up(n, 4); }

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
