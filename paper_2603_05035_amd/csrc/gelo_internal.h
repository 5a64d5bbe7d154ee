// Internal declarations shared by the HIP translation units of the GELO library.
// Launchers validate nothing: the C ABI layer (api.hip) checks shapes, alignment
// and bounds on the host before any kernel is enqueued.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace gelo {

constexpr int kPanel = 16;          // column-panel width of the QR / LU factorisations
constexpr int kMaxN = 5120;         // 512 threads x 10 register-resident rows in the panel kernels
constexpr int kLuBlock = 128;       // outer block width of the LU: trailing updates are GEMMs with K = 128

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
    (f(std::integral_constant<int, Is>{}), ...);
}
// compile-time loop: the body sees its index as a constant, so register arrays stay in registers
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

// ---------------------------------------------------------------- GEMMs ----
// C[M x N] = A[M x K] * B[K x N], row-major.  B is given as two row segments:
// rows [0, K0) come from B0 (ldb0), rows [K0, K) from B1 (ldb1); this is how
// [H ; S] is consumed without a concatenated copy.  Requirements checked by the
// caller: N % 8 == 0; every pointer 16-byte aligned; leading dimensions multiples
// of 8 (bf16) / 4 (f32); A readable and ZERO in columns [K, round_up(K, 8)).
struct GemmOperands {
    const void* A;  int64_t lda;
    const void* B0; int64_t ldb0; int K0;
    const void* B1; int64_t ldb1;
    void* C;        int64_t ldc;
    int M, N, K;
    bool a_zero_padded = false;   // A is readable and zero in columns [K, round_up(K, 64))
    bool subtract = false;        // float only: C <- C - A * B instead of C <- A * B
    void* splitk_ws = nullptr;    // bf16, M <= 128: float workspace for a launch that cuts K over workgroups (optional;
    size_t splitk_ws_bytes = 0;   //   at least gemm_bf16_skinny_ws_bytes(M, N, K), 16-byte aligned)
};
size_t gemm_bf16_skinny_ws_bytes(int M, int N, int K);    // 0: such a launch is not used for this shape
int gemm_bf16_skinny_slices(int M, int N, int K);
int64_t gemm_bf16_skinny_ldp(int N);
hipError_t gemm_bf16(const GemmOperands& g, hipStream_t stream);
// `count` (1..kGemmBatchMax) independent bf16 products in ONE launch (grid y = product): the blocks of a block-diagonal
// mix or unmix.  Every product needs what the fast path of gemm_bf16 needs (N >= 8 and a multiple of 8, A zero-padded
// or K a multiple of 64) and M <= 256 (one tile row); all share N.  hipErrorInvalidValue otherwise.
constexpr int kGemmBatchMax = 20;
hipError_t gemm_bf16_batched(const GemmOperands* g, int count, hipStream_t stream);
hipError_t gemm_f32(const GemmOperands& g, hipStream_t stream);
hipError_t gemm_bf16_init();        // one-time kernel attribute set-up (large dynamic LDS)
hipError_t gemm_f32_init();
hipError_t lu_init();
hipError_t factor_init();
hipError_t sampler_init();

// 8-bit float projection (OCP FP8 E4M3 operands, float accumulation, bf16 result) --------------------------
// codes[r][c] = e4m3(X[r][c] * 448 / max_c |X[r][c]|) (ldq bytes per row), scale[r] = max / 448 (1 for a zero row); X bf16
hipError_t quantize_rows_e4m3(const void* X, int64_t ld, int rows, int cols, uint8_t* codes, int64_t ldq, float* scale,
                              hipStream_t stream);
// W (d x p bf16) -> codes[j][k] (p x d, the transpose) with one scale per column j of W; d a multiple of 128
hipError_t quantize_weight_e4m3(const void* W, int64_t ldw, int d, int p, uint8_t* codes, float* scale, hipStream_t stream);
// C[M x N] (bf16) = (A[M x K] . B[N x K]^T) * sa[i] * sb[j]; codes row-major with lda / ldb bytes per row (multiples of
// 16, at least K), K a multiple of 128, N a multiple of 8; sb 16-byte aligned
hipError_t gemm_fp8(const uint8_t* A, int64_t lda, const float* sa, const uint8_t* B, int64_t ldb, const float* sb,
                    void* C, int64_t ldc, int M, int N, int K, hipStream_t stream);
hipError_t gemm_fp8_init();

// --------------------------------------------------------------- sampler ---
struct PhiloxStream {
    uint32_t key0, key1;            // seed low / high
    uint32_t c1, c2, c3;            // (stream << 8 | attempt), batch id low, batch id high
};
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies
// and a word permutation, key advanced by Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}
// top 23 bits of a word -> (2 m + 1) 2^-24: exact in float, strictly inside (0, 1)
__device__ __forceinline__ float uniform_open01(uint32_t w) {
    return (float)(2u * (w >> 9) + 1u) * 5.9604644775390625e-08f;
}
// Box-Muller: two N(0, 1) values from two words
__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float* z0, float* z1) {
    const float radius = sqrtf(-2.0f * logf(uniform_open01(wa)));
    float s, c;
    sincospif(2.0f * uniform_open01(wb), &s, &c);
    *z0 = radius * c;
    *z1 = radius * s;
}
// Row i of the k x d shield directions (row-major, pitch d, element e = i d + c is output e % 4 of Philox block
// e / 4) and its norm, by one 256-thread workgroup; wave_part: 4 floats of LDS.  Partial sums of squares are
// added in a fixed order (lanes by halving, then the four waves in turn).
__device__ __forceinline__ void shield_direction_row(float* GS, int d, int i, PhiloxStream ps, float* gsnorm, float* wave_part) {
    const int tid = threadIdx.x;
    const int quads = d / 4;                                  // d is a multiple of 8
    float ss = 0.f;
    for (int ql = tid; ql < quads; ql += 256) {
        uint32_t c0 = (uint32_t)(i * quads + ql), c1 = ps.c1, c2 = ps.c2, c3 = ps.c3;
        philox4x32_10(c0, c1, c2, c3, ps.key0, ps.key1);
        float4 z;
        box_muller(c0, c1, &z.x, &z.y);
        box_muller(c2, c3, &z.z, &z.w);
        *reinterpret_cast<float4*>(GS + (int64_t)i * d + 4 * ql) = z;
        ss = fmaf(z.x, z.x, ss); ss = fmaf(z.y, z.y, ss); ss = fmaf(z.z, z.z, ss); ss = fmaf(z.w, z.w, ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((tid & 63) == 0) wave_part[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) gsnorm[i] = sqrtf(((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3]);
}
// The QR works on 16 x 16 tiles: a tile is 256 contiguous floats ordered [column in tile][row in
// tile], tiles are ordered column-block major; element (r, c) of a matrix with `tile_rows` tile
// rows sits at the index below.  A wave that owns a tile in the accumulator layout of
// v_mfma_f32_16x16x4_f32 (lane = 16 g + c holds rows 4 g .. 4 g + 3 of column c) then reads or
// writes it as ONE contiguous kilobyte, 16 bytes per lane.
__host__ __device__ inline int64_t qr_tile_index(int r, int c, int tile_rows) {
    return ((int64_t)(c >> 4) * tile_rows + (r >> 4)) * 256 + (c & 15) * 16 + (r & 15);
}
// out = scale * N(0,1) for r < rows, c < cols; element e = r*cols + c is output e % 4 of Philox
// block e / 4 (counter word 0 = block index).  tiled == 0: out[r * ld + c]; tiled != 0: the same
// element goes to out[qr_tile_index(r, c, ld)] (ld = number of tile rows); tiled == 2: the same, but pieces of 16 rows x
// 256 columns that lie wholly above the diagonal are left as they are (for a reader of the lower triangle only).
hipError_t fill_normal(float* out, int64_t ld, int rows, int cols, PhiloxStream ps, float scale,
                       int tiled, hipStream_t stream);
// words[4 i .. 4 i + 3] = the four output words of Philox block first_block + i (counter word 0), 16-byte aligned
// calibrate.hip: matrix instructions from registers only (0: bf16 32x32x16, 1: E4M3 32x32x64)
size_t matrix_rate_scratch_bytes();
hipError_t matrix_rate_launch(int fp8, int iters, float* scratch, double* flop, hipStream_t stream);
hipError_t philox_words(uint32_t* words, uint32_t first_block, uint32_t blocks, PhiloxStream ps, hipStream_t stream);
// GS[k x d] (pitch d) = N(0,1) with fill_normal's element order, gsnorm[i] = || GS[i, :] ||_2; d % 8 == 0
hipError_t shield_directions(float* GS, int k, int d, PhiloxStream ps, float* gsnorm, hipStream_t stream);
// dst[r * ldd + c] += scale * src[r * lds + c] over an rows x cols block
hipError_t axpy_matrix(float* dst, int64_t ldd, const float* src, int64_t lds, int rows, int cols,
                       float scale, hipStream_t stream);
// norms[r] = || X[r, 0:cols] ||_2, X float or bf16
hipError_t row_norms(const void* X, int is_bf16, int64_t ld, int rows, int cols, float* norms,
                     hipStream_t stream);
// out[0], out[1] = the two middle elements of v[0:count] (stat 0: their mean is the median; the same
// element twice when count is odd) or twice its mean (stat 1); consumers take 0.5 (out[0] + out[1])
hipError_t norm_statistic(const float* v, int count, int stat, float* out, hipStream_t stream);
// S[i, :] = G[i, :] * (scale * 0.5 (stat[0] + stat[1]) / gnorm[i]), written as float or bf16 (lds elements per row)
hipError_t make_shields(const float* G, int64_t ldg, const float* gnorm, const float* stat, float scale,
                        int k, int d, void* S, int is_bf16, int64_t lds, hipStream_t stream);
// Writes an n x n float matrix (src, optional per-column sign flip from `rdiag` < 0) into the
// mixing buffers: dst32 / dst16 get the matrix, dstT32 / dstT16 its transpose (any may be null).
// Every destination has `ldd` elements per row and its columns [n, ldd) are zero-filled.
// src_tiled == 0: src is row-major with pitch lds; src_tiled != 0: src holds the matrix in 16 x 16
// tiles with lds tile rows (what householder_qr leaves in ws.X).
hipError_t emit_matrix(const float* src, int64_t lds, int src_tiled, const float* rdiag, int n, int64_t ldd,
                       float* dst32, uint16_t* dst16, float* dstT32, uint16_t* dstT16,
                       hipStream_t stream);
// dense float copy out[r * cols + c] = (float) src[r * ld + c]
hipError_t export_dense(const void* src, int is_bf16, int64_t ld, int rows, int cols, float* out,
                        hipStream_t stream);

// ------------------------------------------- decode-shaped batches (n <= 128) --
constexpr int kSmallMaxN = 128;      // one workgroup holds [G | I] (n x 2 n floats) in LDS up to this n
constexpr int kSmallMaxBatch = 48;   // mixing objects one launch of small_sample draws
// Buffers of the mixing objects a batched draw fills, all of one shape: the same offsets into each block.
struct SmallSampleTargets {
    void* block[kSmallMaxBatch];
    int64_t off_A32, off_Ainv32, off_A16, off_Ainv16, off_GS, off_gsnorm;    // off_A16 < 0: no bf16 copies
};
// For item i < count: batch id = first_batch + i; A = Q diag(sign r_ii) of the Householder QR of its n x n Philox
// Gaussian (stream c1 of ps; ps.c2 / ps.c3 are ignored), written with its transpose (float, and bf16 if wanted;
// ldk elements per row, zero beyond column n), and the k x d shield directions with their norms (stream c1_shield).
// One launch: a workgroup per matrix and one per shield row.  n <= kSmallMaxN, count <= kSmallMaxBatch.
hipError_t small_sample(const SmallSampleTargets& t, int count, uint64_t first_batch, PhiloxStream ps, uint32_t c1_shield,
                        int n, int k, int d, int64_t ldk, hipStream_t stream);
hipError_t small_init();
// bf16, n <= kSmallMaxN: shield rows and U = A [H ; S] in one launch.  rownorm: the n_data row norms of H (ignored
// when k == 0); stat_kind 0 median / 1 mean; S (k x d bf16, pitch d) is written too.  d % 8 == 0.
hipError_t small_mix(const uint16_t* A16, int64_t ldk, const uint16_t* H, int64_t ldh, const float* GS, const float* gsnorm,
                     const float* rownorm, int stat_kind, float shield_scale, int n_data, int k, int d,
                     uint16_t* S, uint16_t* U, int64_t ldu, hipStream_t stream);

// ------------------------------------------------- structured orthogonal A --
constexpr int kStructuredRounds = 3;
// table: the rounds + 1 permutations (low 31 bits) and sign flips (top bit) of one structured
// A = P_R (B D_{R-1} P_{R-1}) ... (B D_0 P_0), drawn from the Philox streams of (seed, batch id) in ps
// (ps.c1 is not used: the streams are fixed), each in round_up(n, 4) words, and behind them the rounds + 1
// inverse permutations with the same signs (what the transposed transform gathers by):
// structured_table_words(n, rounds) words in all.
hipError_t structured_tables(uint32_t* table, int n, int rounds, PhiloxStream ps, hipStream_t stream);
size_t structured_table_words(int n, int rounds);
// out = A x (transposed == 0) or A^T x (transposed != 0) for the n x ncols operand x whose rows
// [0, rows0) come from in0 and rows [rows0, n) from in1 (may be null when rows0 == n); result rows
// >= rows_out are dropped.  float or bf16 throughout; ncols a multiple of 4 and every row start
// 16-byte (float) / 8-byte (bf16) aligned; n <= structured_max_rows().
struct StructuredOperands {
    const void* in0; int64_t ld0; int rows0;
    const void* in1; int64_t ld1;
    void* out; int64_t ldo; int rows_out;
    const uint32_t* table;
    int n, ncols, rounds;
    bool transposed;
};
hipError_t structured_apply(const StructuredOperands& o, int is_bf16, hipStream_t stream);
hipError_t structured_init();
int structured_max_rows();

// --------------------------------------------------------- factorisations --
// Workspace for one n_pad x ld float problem (n_pad = round_up(n, kPanel), ld = round_up(n, 64)).
struct FactorWorkspace {
    float* M;        // the matrix being factorised (G, then R + reflectors / L\U)
    float* X;        // the result being accumulated (Q, or A^-1)
    float* Vc;       // QR: two alternating pairs of compact reflector blocks (n_pad x 16 and 16 x n_pad)
    float* Tmat;     // per panel: the 16 x 16 triangle T of the block reflector I - V T V^T
    float* Dinv;     // LU: inverses of the diagonal blocks of L, then of U (pitch kLuBlock, n_pad rows each)
    float* rdiag;    // n_pad: diagonal of R
    float* vec;      // 8 * ld floats: the Lanczos vectors of the condition estimate
    float* tri;      // its tridiagonal coefficients (2 operators x (alpha, beta) x 32)
    int*   perm;     // LU: perm[i] = row of the input that the interchanges brought to row i
    int*   gat;      // LU: two alternating lists of 32 (destination, source) row pairs, one per panel
    int*   flag;     // singular-pivot flag
    float* scalars;  // [0] kappa estimate, [1] sigma_max, [2] 1 / sigma_min
    int n_pad; int64_t ld;
};
size_t factor_workspace_bytes(int n);
void factor_workspace_carve(void* base, int n, FactorWorkspace* ws);

// ws.M holds an n x n matrix in 16 x 16 tiles (qr_tile_index with n_pad / 16 tile rows; what lies
// beyond n need not be initialised).  On return ws.X holds the orthogonal factor Q of its Householder
// QR in the same tiled layout (identity in the padding block), ws.M and ws.Vc the reflectors, and
// ws.rdiag the diagonal of R.  `count` > 1 factorises that many matrices side by side in the same launches (grid y):
// matrix i's workspace is the one carved at `batch_stride` floats times i behind ws's (same n for all).
// `direct`: the reflectors are NOT those of a factorisation: reflector k is built from column k of ws.M as it
// stands (rows k onward), so ws.X becomes the product H_0 H_1 ... H_{n-1} of directly drawn reflectors and
// ws.rdiag the values beta_k those reflectors map their columns to; no chain of dependent panels.
hipError_t householder_qr(const FactorWorkspace& ws, int n, int count, int64_t batch_stride, hipStream_t stream, bool direct = false);
// ws.M holds an n_pad x n_pad matrix with an identity block in the padding.  On return ws.X holds
// its inverse (via row-pivoted LU), *ws.flag != 0 if a zero pivot was met.
hipError_t lu_inverse(const FactorWorkspace& ws, hipStream_t stream);
// kappa_2 estimate of the n x n matrix A (lda) with inverse Ainv: sigma_max of both by `steps`
// (at most 32) Lanczos steps on A^T A and Ainv^T Ainv; uses ws.M / ws.X as scratch for the two
// transposes; result in ws.scalars[0].
hipError_t kappa_estimate(const float* A, const float* Ainv, int64_t lda, int n, const FactorWorkspace& ws,
                          int steps, hipStream_t stream);
hipError_t set_identity(float* X, int64_t ld, int n_pad, hipStream_t stream);
hipError_t zero_ints(int* p, int count, hipStream_t stream);
// zero rows/cols [n, n_pad) of M; optionally put ones on that part of the diagonal
hipError_t pad_matrix(float* M, int64_t ld, int n, int n_pad, int identity_block, hipStream_t stream);

}  // namespace gelo
