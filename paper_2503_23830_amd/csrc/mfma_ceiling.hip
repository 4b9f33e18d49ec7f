// What the matrix cores of this machine sustain on v_mfma_f32_32x32x16_bf16 alone: every
// wavefront loops over register-resident MFMAs, nothing else.  Two operand sets:
//   ones       every operand element is 1.0 (almost no switching activity in the multipliers)
//   random     eight A and eight B register sets holding N(0,1) bf16 values, a different pair
//              in every instruction (the data attention sees)
// The gap between the two is the power limit: it is the context for the "fraction of the
// 2.5 PFLOP/s dense bf16 peak" the attention kernels report.  Usage: mfma_ceiling [ms_target]
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                               \
    do {                                                                    \
        hipError_t e_ = (x);                                                \
        if (e_ != hipSuccess) {                                             \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));         \
            exit(1);                                                        \
        }                                                                   \
    } while (0)

constexpr int kSets = 8;

__global__ __launch_bounds__(256) void mfma_loop(const u32x4 *__restrict__ src, float *out, int iters, int random)
{
    bf16x8 a[kSets], b[kSets];
    for (int i = 0; i < kSets; ++i) {
        const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
        a[i] = __builtin_bit_cast(bf16x8, random ? src[(threadIdx.x * kSets + i) * 2] : ones);
        b[i] = __builtin_bit_cast(bf16x8, random ? src[(threadIdx.x * kSets + i) * 2 + 1] : ones);
    }
    f32x16 acc[4];
    for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kSets; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + j) % kSets], b[(i + 2 * j) % kSets], acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

int main(int argc, char **argv)
{
    const double ms_target = argc > 1 ? atof(argv[1]) : 100.0;
    std::vector<uint16_t> h(256 * kSets * 16);
    uint64_t st = 0x9E3779B97F4A7C15ull;
    auto next = [&]() { st ^= st << 13; st ^= st >> 7; st ^= st << 17; return (double)(st >> 11) / 9007199254740992.0 + 1e-12; };
    for (auto &x : h) {
        const float z = (float)(sqrt(-2.0 * log(next())) * cos(6.283185307179586 * next()));
        uint32_t bits;
        memcpy(&bits, &z, 4);
        x = (uint16_t)(bits >> 16);
    }
    u32x4 *src;
    float *out;
    const int wgs = 2048;  // 8 wavefronts per SIMD
    CK(hipMalloc(&src, h.size() * 2));
    CK(hipMemcpy(src, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    CK(hipMalloc(&out, 4 * 256 * wgs));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    for (int random = 0; random < 2; ++random) {
        int iters = 2000;
        for (int rep = 0; rep < 3; ++rep) {
            CK(hipEventRecord(e0, 0));
            hipLaunchKernelGGL(mfma_loop, dim3(wgs), dim3(256), 0, 0, src, out, iters, random);
            CK(hipEventRecord(e1, 0));
            CK(hipEventSynchronize(e1));
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            const double flop = (double)wgs * 4 * iters * kSets * 4 * 2.0 * 32 * 32 * 16;
            printf("%s operands: %d workgroups x 4 wavefronts, %.1f ms: %.1f TFLOP/s\n", random ? "random" : "ones  ", wgs,
                   ms, flop / ms / 1e9);
            iters = (int)(iters * ms_target / ms) + 1;  // the later repetitions run about ms_target
        }
    }
    return 0;
}
