// Trusted-side sampling kernels: the Philox4x32-10 Gaussian source for the mixing
// matrix A and the shield directions (Section 3.2 step 1.2; Section 3.2.1
// Mitigation 2), the row-norm statistic of H that sets the shield scale, and the
// kernels that write A / A^-1 into the layouts the GEMMs read.
#include "gelo_internal.h"

namespace gelo {
namespace {

__global__ __launch_bounds__(256)
void fill_normal_kernel(float* out, int64_t ld, int rows, int cols, PhiloxStream ps, float scale, int tiled) {
    const int64_t total = (int64_t)rows * cols;
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q * 4 >= total) return;
    uint32_t c0 = (uint32_t)q, c1 = ps.c1, c2 = ps.c2, c3 = ps.c3;
    philox4x32_10(c0, c1, c2, c3, ps.key0, ps.key1);
    float z[4];
    box_muller(c0, c1, &z[0], &z[1]);
    box_muller(c2, c3, &z[2], &z[3]);
    int64_t e = q * 4;
    int r = (int)(e / cols), c = (int)(e % cols);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (e + t < total) out[tiled ? qr_tile_index(r, c, (int)ld) : (int64_t)r * ld + c] = scale * z[t];
        if (++c == cols) { c = 0; ++r; }
    }
}

// The same values into the QR's 16 x 16 tiles (qr_tile_index).  Element e = r cols + c is output e % 4 of
// Philox block e / 4, so a block's four values are neighbours in a ROW while a tile keeps a COLUMN's 16 rows
// together: written straight from the registers every store of a wave would touch 64 cache lines.  A workgroup
// instead takes 16 rows x 256 columns, computes the blocks that cover each of its row segments (one more per
// row than the segment holds when its ends fall inside blocks), sets the values down in LDS and writes the 16
// tiles out as they lie in memory, 16 bytes per lane.
__global__ __launch_bounds__(256)
void fill_normal_tiled_kernel(float* out, int tile_rows, int rows, int cols, PhiloxStream ps, float scale, int lower_only) {
    constexpr int CW = 256, PITCH = CW + 1, PER_ROW = CW / 4 + 1;
    __shared__ float tile[16 * PITCH];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * 16, c0 = blockIdx.x * CW;
    if (lower_only && c0 >= r0 + 16) return;                 // every column of this piece lies to the right of every row's diagonal entry
    const int width = min(CW, cols - c0);
    for (int idx = tid; idx < 16 * PER_ROW; idx += 256) {
        const int ri = idx / PER_ROW, bi = idx - ri * PER_ROW;
        const int r = r0 + ri;
        if (r >= rows) break;
        const uint32_t e_first = (uint32_t)r * (uint32_t)cols + (uint32_t)c0, e_last = e_first + (uint32_t)width - 1u;
        const uint32_t b = e_first / 4u + (uint32_t)bi;
        if (4u * b > e_last) continue;
        uint32_t w0 = b, w1 = ps.c1, w2 = ps.c2, w3 = ps.c3;
        philox4x32_10(w0, w1, w2, w3, ps.key0, ps.key1);
        float z[4];
        box_muller(w0, w1, &z[0], &z[1]);
        box_muller(w2, w3, &z[2], &z[3]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t e = 4u * b + (uint32_t)t;
            if (e >= e_first && e <= e_last) tile[ri * PITCH + (int)(e - e_first)] = scale * z[t];
        }
    }
    __syncthreads();
    // float4 item: rows 4 g .. 4 g + 3 of column c of the strip (16 bytes of a tile: index (c & 15) * 16 + 4 g)
    for (int it = tid; it < CW * 4; it += 256) {
        const int c = it >> 2, g = it & 3;
        if (c >= width) continue;
        float* dst = out + qr_tile_index(r0 + 4 * g, c0 + c, tile_rows);
        const float* src = tile + (4 * g) * PITCH + c;
        if (r0 + 4 * g + 3 < rows) {
            *reinterpret_cast<float4*>(dst) = make_float4(src[0], src[PITCH], src[2 * PITCH], src[3 * PITCH]);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (r0 + 4 * g + t < rows) dst[t] = src[t * PITCH];
        }
    }
}

// Raw generator output for bitwise checks: words[4 i .. 4 i + 3] = the four words of block first + i.
__global__ __launch_bounds__(256)
void philox_words_kernel(uint32_t* words, uint32_t first, uint32_t blocks, PhiloxStream ps) {
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= blocks) return;
    uint32_t c0 = first + i, c1 = ps.c1, c2 = ps.c2, c3 = ps.c3;
    philox4x32_10(c0, c1, c2, c3, ps.key0, ps.key1);
    *reinterpret_cast<uint4*>(words + 4 * (size_t)i) = make_uint4(c0, c1, c2, c3);
}

// The k x d shield directions (row-major, pitch d, the same element-to-Philox-word map as
// fill_normal_kernel) and their norms in one launch: one workgroup per row, partial sums of squares
// added in a fixed order (lanes by halving, then the four waves in turn).
__global__ __launch_bounds__(256)
void shield_directions_kernel(float* GS, int d, PhiloxStream ps, float* gsnorm) {
    __shared__ float wave_part[4];
    shield_direction_row(GS, d, blockIdx.x, ps, gsnorm, wave_part);
}

__global__ __launch_bounds__(256)
void axpy_matrix_kernel(float* dst, int64_t ldd, const float* src, int64_t lds, int rows, int cols, float scale) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (c < cols && r < rows) dst[(int64_t)r * ldd + c] += scale * src[(int64_t)r * lds + c];
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }

// one wave per row, fixed summation order
template <bool BF16>
__global__ __launch_bounds__(256)
void row_norms_kernel(const void* X, int64_t ld, int rows, int cols, float* norms) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= rows) return;
    float s = 0.f;
    if (BF16) {
        const uint16_t* p = (const uint16_t*)X + (int64_t)row * ld;
#pragma unroll 8
        for (int c = lane * 8; c < cols; c += 64 * 8) {          // unrolled: the loads of eight steps fly together
            const uint4 v = *reinterpret_cast<const uint4*>(p + c);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float lo = bf16_bits_to_float(w[t] & 0xFFFFu), hi = bf16_bits_to_float(w[t] >> 16);
                s = fmaf(lo, lo, s);
                s = fmaf(hi, hi, s);
            }
        }
    } else {
        const float* p = (const float*)X + (int64_t)row * ld;
#pragma unroll 8
        for (int c = lane * 4; c < cols; c += 64 * 4) {
            const float4 v = *reinterpret_cast<const float4*>(p + c);
            s = fmaf(v.x, v.x, s); s = fmaf(v.y, v.y, s); s = fmaf(v.z, v.z, s); s = fmaf(v.w, v.w, s);
        }
    }
    s = wave_sum(s);
    if (lane == 0) norms[row] = sqrtf(s);
}

// Mean of v[0:count]: single workgroup, tree sum in a fixed order.
__global__ __launch_bounds__(1024)
void mean_kernel(const float* v, int count, float* out) {
    __shared__ float buf[1024];
    const int tid = threadIdx.x;
    float s = 0.f;
    for (int i = tid; i < count; i += 1024) s += v[i];
    buf[tid] = s;
    __syncthreads();
    for (int half = 512; half > 0; half >>= 1) {
        if (tid < half) buf[tid] += buf[tid + half];
        __syncthreads();
    }
    if (tid == 0) { out[0] = buf[0] / (float)count; out[1] = out[0]; }
}

// Median of v[0:count] (non-negative floats, whose order is that of their bit patterns) as its two
// middle elements: out[0] = element of rank (count - 1) / 2, out[1] = element of rank count / 2 (the
// same element when count is odd); the median is their mean.  Every element finds its rank by
// counting the (value, index) pairs below its own - count^2 comparisons spread over count / 16
// workgroups - and the two that hit the middle ranks write themselves out: no sorting, no atomics,
// and exactly one writer per slot.
__global__ __launch_bounds__(256)
void median_parts_kernel(const float* v, int count, float* out) {
    // 16 elements per workgroup, each counted by 16 threads over a sixteenth of the keys: the count is a chain of
    // dependent compare-and-add steps, so its length per thread, not the number of workgroups, sets the time
    constexpr int EL = 16, PARTS = 256 / EL;
    extern __shared__ __align__(16) uint32_t keys[];        // count rounded up to 4; the padding holds the largest key
    __shared__ int part_count[PARTS][EL];
    const int tid = threadIdx.x;
    const int padded = (count + 3) & ~3;
    for (int i = tid; i < padded; i += 256) keys[i] = i < count ? __float_as_uint(v[i]) : 0xFFFFFFFFu;
    __syncthreads();
    const int slot = tid % EL, part = tid / EL;
    const int i = blockIdx.x * EL + slot;
    int below = 0;
    if (i < count) {
        const uint4* keys4 = reinterpret_cast<const uint4*>(keys);
        const int quads = padded / 4, chunk = (quads + PARTS - 1) / PARTS;
        const int lo = part * chunk, hi = min(quads, lo + chunk);
        const uint64_t mine = ((uint64_t)keys[i] << 32) | (uint32_t)i;
        auto is_below = [&](uint32_t kk, int k) { return ((((uint64_t)kk << 32) | (uint32_t)k) < mine) ? 1 : 0; };
#pragma unroll 8
        for (int qd = lo; qd < hi; ++qd) {
            const uint4 kk = keys4[qd];
            below += is_below(kk.x, 4 * qd) + is_below(kk.y, 4 * qd + 1) + is_below(kk.z, 4 * qd + 2) + is_below(kk.w, 4 * qd + 3);
        }
    }
    part_count[part][slot] = below;
    __syncthreads();
    if (part != 0 || i >= count) return;
    int rank = 0;
#pragma unroll
    for (int q = 0; q < PARTS; ++q) rank += part_count[q][slot];
    if (rank == (count - 1) / 2) out[0] = __uint_as_float(keys[i]);
    if (rank == count / 2) out[1] = __uint_as_float(keys[i]);
}

template <bool BF16>
__global__ __launch_bounds__(256)
void make_shields_kernel(const float* G, int64_t ldg, const float* gnorm, const float* stat, float scale,
                         int d, void* S, int64_t lds) {
    const int i = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= d) return;
    const float f = scale * (0.5f * (stat[0] + stat[1])) / gnorm[i];
    const float x = G[(int64_t)i * ldg + c] * f;
    if (BF16) ((__bf16*)S)[(int64_t)i * lds + c] = (__bf16)x;
    else ((float*)S)[(int64_t)i * lds + c] = x;
}

// 32 x 32 tiles through LDS so that both the matrix and its transpose are written row-contiguously.
// Grid covers ceil(ldd/32) x ceil(ldd/32) tiles; everything outside n x n is written as zero.
__global__ __launch_bounds__(256)
void emit_matrix_kernel(const float* src, int64_t lds, int src_tiled, const float* rdiag, int n, int64_t ldd,
                        float* dst32, uint16_t* dst16, float* dstT32, uint16_t* dstT16) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8) {
        const int r = r0 + i, c = c0 + tx;
        float x = 0.f;
        if (r < n && c < n) {
            x = src_tiled ? src[qr_tile_index(r, c, (int)lds)] : src[(int64_t)r * lds + c];
            if (rdiag != nullptr && rdiag[c] < 0.f) x = -x;
        }
        tile[i][tx] = x;
        if (r < n && c < ldd) {
            if (dst32) dst32[(int64_t)r * ldd + c] = x;
            if (dst16) { __bf16 h = (__bf16)x; dst16[(int64_t)r * ldd + c] = __builtin_bit_cast(uint16_t, h); }
        }
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int r = c0 + i, c = r0 + tx;                       // row of the transpose = column of src
        const float x = tile[tx][i];
        if (r < n && c < ldd) {
            if (dstT32) dstT32[(int64_t)r * ldd + c] = x;
            if (dstT16) { __bf16 h = (__bf16)x; dstT16[(int64_t)r * ldd + c] = __builtin_bit_cast(uint16_t, h); }
        }
    }
}

// The same for a source in the factorisations' 16 x 16 tiles, 64 x 64 elements per workgroup: a wave reads a whole
// source tile at a time (one contiguous kilobyte, 16 bytes per lane: four rows of a column), and both the matrix and
// its transpose leave in pieces of four elements per lane over whole 64-element row segments.  ldd % 64 == 0.
__global__ __launch_bounds__(256)
void emit_tiled_kernel(const float* src, int tile_rows, const float* rdiag, int n, int64_t ldd,
                       float* dst32, uint16_t* dst16, float* dstT32, uint16_t* dstT16) {
    __shared__ float tile[64][65];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    for (int t = wave; t < 16; t += 4) {                         // source tile (t & 3, t >> 2) of the 4 x 4 in this piece
        const int cl = (t >> 2) * 16 + (lane >> 2), rl = (t & 3) * 16 + (lane & 3) * 4;
        const int r = r0 + rl, c = c0 + cl;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < n && c < n) {
            v = *reinterpret_cast<const float4*>(src + qr_tile_index(r, c, tile_rows));
            if (rdiag != nullptr && rdiag[c] < 0.f) v = make_float4(-v.x, -v.y, -v.z, -v.w);
            if (r + 1 >= n) v.y = 0.f;
            if (r + 2 >= n) v.z = 0.f;
            if (r + 3 >= n) v.w = 0.f;
        }
        tile[rl][cl] = v.x; tile[rl + 1][cl] = v.y; tile[rl + 2][cl] = v.z; tile[rl + 3][cl] = v.w;
    }
    __syncthreads();
    auto pack4 = [](float a, float b, float c, float d) {
        typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
        const bf16x4_t h = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
        return __builtin_bit_cast(uint2, h);
    };
    for (int item = tid; item < 64 * 16; item += 256) {
        const int i = item >> 4, q = (item & 15) * 4;
        {                                                        // row r0 + i of the matrix, columns c0 + q ..
            const int r = r0 + i, c = c0 + q;
            if (r < n && c < ldd) {
                const float a = tile[i][q], b = tile[i][q + 1], cc = tile[i][q + 2], d = tile[i][q + 3];
                if (dst32) *reinterpret_cast<float4*>(dst32 + (int64_t)r * ldd + c) = make_float4(a, b, cc, d);
                if (dst16) *reinterpret_cast<uint2*>(dst16 + (int64_t)r * ldd + c) = pack4(a, b, cc, d);
            }
        }
        {                                                        // row c0 + i of the transpose, columns r0 + q ..
            const int r = c0 + i, c = r0 + q;
            if (r < n && c < ldd) {
                const float a = tile[q][i], b = tile[q + 1][i], cc = tile[q + 2][i], d = tile[q + 3][i];
                if (dstT32) *reinterpret_cast<float4*>(dstT32 + (int64_t)r * ldd + c) = make_float4(a, b, cc, d);
                if (dstT16) *reinterpret_cast<uint2*>(dstT16 + (int64_t)r * ldd + c) = pack4(a, b, cc, d);
            }
        }
    }
}

template <bool BF16>
__global__ __launch_bounds__(256)
void export_dense_kernel(const void* src, int64_t ld, int rows, int cols, float* out) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (c >= cols || r >= rows) return;
    float x;
    if (BF16) x = bf16_bits_to_float(((const uint16_t*)src)[(int64_t)r * ld + c]);
    else x = ((const float*)src)[(int64_t)r * ld + c];
    out[(int64_t)r * cols + c] = x;
}

}  // namespace

hipError_t fill_normal(float* out, int64_t ld, int rows, int cols, PhiloxStream ps, float scale,
                       int tiled, hipStream_t stream) {
    const int64_t quads = ((int64_t)rows * cols + 3) / 4;
    if (quads == 0) return hipSuccess;
    if (tiled && (int64_t)rows * cols < ((int64_t)1 << 32)) {
        hipLaunchKernelGGL(fill_normal_tiled_kernel, dim3((cols + 255) / 256, (rows + 15) / 16), dim3(256), 0, stream,
                           out, (int)ld, rows, cols, ps, scale, tiled == 2 ? 1 : 0);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(fill_normal_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream,
                       out, ld, rows, cols, ps, scale, tiled);
    return hipGetLastError();
}

hipError_t philox_words(uint32_t* words, uint32_t first_block, uint32_t blocks, PhiloxStream ps, hipStream_t stream) {
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(philox_words_kernel, dim3((blocks + 255u) / 256u), dim3(256), 0, stream, words, first_block, blocks, ps);
    return hipGetLastError();
}

hipError_t shield_directions(float* GS, int k, int d, PhiloxStream ps, float* gsnorm, hipStream_t stream) {
    if (k <= 0) return hipSuccess;
    hipLaunchKernelGGL(shield_directions_kernel, dim3(k), dim3(256), 0, stream, GS, d, ps, gsnorm);
    return hipGetLastError();
}

hipError_t axpy_matrix(float* dst, int64_t ldd, const float* src, int64_t lds, int rows, int cols,
                       float scale, hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    hipLaunchKernelGGL(axpy_matrix_kernel, dim3((cols + 255) / 256, rows), dim3(256), 0, stream,
                       dst, ldd, src, lds, rows, cols, scale);
    return hipGetLastError();
}

hipError_t row_norms(const void* X, int is_bf16, int64_t ld, int rows, int cols, float* norms,
                     hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    const dim3 grid((rows + 3) / 4), block(256);
    if (is_bf16) hipLaunchKernelGGL(row_norms_kernel<true>, grid, block, 0, stream, X, ld, rows, cols, norms);
    else hipLaunchKernelGGL(row_norms_kernel<false>, grid, block, 0, stream, X, ld, rows, cols, norms);
    return hipGetLastError();
}

hipError_t norm_statistic(const float* v, int count, int stat, float* out, hipStream_t stream) {
    if (count <= 0) return hipErrorInvalidValue;
    if (stat == 1) hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(1024), 0, stream, v, count, out);
    else hipLaunchKernelGGL(median_parts_kernel, dim3((count + 15) / 16), dim3(256), (size_t)((count + 3) & ~3) * sizeof(uint32_t),
                            stream, v, count, out);
    return hipGetLastError();
}

hipError_t make_shields(const float* G, int64_t ldg, const float* gnorm, const float* stat, float scale,
                        int k, int d, void* S, int is_bf16, int64_t lds, hipStream_t stream) {
    if (k <= 0) return hipSuccess;
    const dim3 grid((d + 255) / 256, k), block(256);
    if (is_bf16) hipLaunchKernelGGL(make_shields_kernel<true>, grid, block, 0, stream, G, ldg, gnorm, stat, scale, d, S, lds);
    else hipLaunchKernelGGL(make_shields_kernel<false>, grid, block, 0, stream, G, ldg, gnorm, stat, scale, d, S, lds);
    return hipGetLastError();
}

hipError_t emit_matrix(const float* src, int64_t lds, int src_tiled, const float* rdiag, int n, int64_t ldd,
                       float* dst32, uint16_t* dst16, float* dstT32, uint16_t* dstT16, hipStream_t stream) {
    if (src_tiled && ldd % 64 == 0) {
        const int t64 = (int)(ldd / 64);
        hipLaunchKernelGGL(emit_tiled_kernel, dim3(t64, t64), dim3(256), 0, stream,
                           src, (int)lds, rdiag, n, ldd, dst32, dst16, dstT32, dstT16);
        return hipGetLastError();
    }
    const int t = (int)((ldd + 31) / 32);
    hipLaunchKernelGGL(emit_matrix_kernel, dim3(t, t), dim3(256), 0, stream,
                       src, lds, src_tiled, rdiag, n, ldd, dst32, dst16, dstT32, dstT16);
    return hipGetLastError();
}

hipError_t export_dense(const void* src, int is_bf16, int64_t ld, int rows, int cols, float* out,
                        hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const dim3 grid((cols + 255) / 256, rows), block(256);
    if (is_bf16) hipLaunchKernelGGL(export_dense_kernel<true>, grid, block, 0, stream, src, ld, rows, cols, out);
    else hipLaunchKernelGGL(export_dense_kernel<false>, grid, block, 0, stream, src, ld, rows, cols, out);
    return hipGetLastError();
}

hipError_t sampler_init() {    // brings this file's code onto the device (see factor_init)
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&fill_normal_kernel));
}

}  // namespace gelo
