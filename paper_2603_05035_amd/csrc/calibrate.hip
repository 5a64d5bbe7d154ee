// What the matrix cores deliver when nothing else is in the way: every wave of every compute unit issues
// independent matrix instructions from registers, in the mix of one K step of the projection kernels (eight
// accumulator tiles per wave, two waves per SIMD).  No memory, no LDS, no barrier.  The published peaks (Section
// 4.2's "fraction of peak" is quoted against them) assume the top clock; under this load the chip settles lower,
// so this rate is the ceiling a kernel can be held against.  A measurement aid: nothing in the protocol calls it.
#include "gelo_internal.h"

namespace gelo {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));

constexpr int kRateWorkgroups = 256, kRateThreads = 512, kGroup = 32;     // matrix instructions per wave and loop pass

// FP8: 0 = v_mfma_f32_32x32x16_bf16, 1 = v_mfma_f32_32x32x64_f8f6f4 on E4M3 operands
template <int FP8>
__global__ __launch_bounds__(kRateThreads)
void matrix_rate_kernel(float* out, int iters, uint32_t seed) {
    const int tid = threadIdx.x;
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    // Operands like real data - the power the matrix cores draw, and with it the clock they are given, depends on
    // how many operand bits change from one instruction to the next: four "A" and two "B" fragments per wave
    // (one K step of a 128 x 64 wave tile), every element with a random sign and mantissa and a magnitude between
    // 2^-3 and 2^4 (bf16), or a random E4M3 code with the top exponent bit clear (no NaN code).
    auto hash = [](uint32_t x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; };
    i32x8_t frag[6];
#pragma unroll
    for (int f = 0; f < 6; ++f)
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const uint32_t h = hash(seed + 977u * (uint32_t)(blockIdx.x * kRateThreads + tid) + 31u * (uint32_t)(f * 8 + v));
            if constexpr (FP8) frag[f][v] = (int)(h & 0xBFBFBFBFu);
            else {
                auto half = [](uint32_t b) { return (b & 0x8000u) | ((0x7Cu + ((b >> 8) & 7u)) << 7) | (b & 0x7Fu); };
                frag[f][v] = (int)(half(h) | (half(h >> 16) << 16));
            }
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < kGroup / 8; ++g)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const i32x8_t a = frag[i >> 1], b = frag[4 + (i & 1)];
                if constexpr (FP8) {
                    acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, acc[i], 0, 0, 0, 0, 0, 0);
                } else {
                    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
                    // the four K groups of a K step take different halves of the fragments in turn
                    const u32x4_t ah = {(uint32_t)a[(g & 1) * 4], (uint32_t)a[(g & 1) * 4 + 1], (uint32_t)a[(g & 1) * 4 + 2], (uint32_t)a[(g & 1) * 4 + 3]};
                    const u32x4_t bh = {(uint32_t)b[(g >> 1) * 4], (uint32_t)b[(g >> 1) * 4 + 1], (uint32_t)b[(g >> 1) * 4 + 2], (uint32_t)b[(g >> 1) * 4 + 3]};
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bh), __builtin_bit_cast(bf16x8_t, ah), acc[i], 0, 0, 0);
                }
            }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += acc[i][0] + acc[i][7] + acc[i][15];
    out[blockIdx.x * kRateThreads + tid] = sum;
}

}  // namespace

size_t matrix_rate_scratch_bytes() { return (size_t)kRateWorkgroups * kRateThreads * sizeof(float); }

// Enqueues one launch; flop = what it executes.
hipError_t matrix_rate_launch(int fp8, int iters, float* scratch, double* flop, hipStream_t stream) {
    if (fp8) hipLaunchKernelGGL(matrix_rate_kernel<1>, dim3(kRateWorkgroups), dim3(kRateThreads), 0, stream, scratch, iters, 7u);
    else hipLaunchKernelGGL(matrix_rate_kernel<0>, dim3(kRateWorkgroups), dim3(kRateThreads), 0, stream, scratch, iters, 7u);
    const double per_instr = 2.0 * 32 * 32 * (fp8 ? 64 : 16);
    *flop = per_instr * kGroup * (double)iters * (kRateThreads / 64) * kRateWorkgroups;
    return hipGetLastError();
}

}  // namespace gelo
