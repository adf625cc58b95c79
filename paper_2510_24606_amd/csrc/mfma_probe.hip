// Measurement aid of libdhsa: sustained rate of the bf16 MFMA instruction the
// attention kernel is built on (v_mfma_f32_32x32x16_bf16), with nothing else in
// the loop.  The attention kernel's "% of MFMA peak" is priced against the
// published 2.5 PFLOP/s; this probe shows what the same chip sustains when the
// matrix unit alone runs flat out.  With operands that never change the unit
// reaches the published rate; with random operands (all bits toggling, as in
// real attention) the chip lowers its clock to stay inside its power limit and
// sustains markedly less -- which bounds any kernel that feeds the unit real data.
#include <hip/hip_runtime.h>

#include "dhsa.h"

namespace dhsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeSets = 8;      // operand sets rotated through (random mode)
constexpr int kProbeBlocks = 512;  // 2 workgroups of 4 waves per CU

__device__ __forceinline__ float probe_rand(unsigned &s) {
    s = s * 1664525u + 1013904223u;
    return ((s >> 8) * (1.0f / 8388608.0f) - 1.0f) * 2.0f;   // uniform in [-2, 2)
}

// words[0..1]: shader cycles and 100 MHz ticks of one wave around its loop
__global__ __launch_bounds__(256) void k_mfma_probe(float *sink, unsigned long long *words, int iters, int random) {
    bf16x8 a[kProbeSets], b[kProbeSets];
    unsigned seed = threadIdx.x * 7919u + blockIdx.x * 104729u + 1u;
#pragma unroll
    for (int j = 0; j < kProbeSets; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[j][i] = (__bf16)(random ? probe_rand(seed) : 0.5f);
            b[j][i] = (__bf16)(random ? probe_rand(seed) : 0.25f);
        }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int x = 0; x < 16; ++x) acc[j][x] = 0.f;
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(4 * r + j) % kProbeSets], b[(4 * r + j) % kProbeSets],
                                                                 acc[j], 0, 0, 0);
    }
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        words[0] = c1 - c0;
        words[1] = r1 - r0;
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int x = 0; x < 16; ++x) s += acc[j][x];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace dhsa

extern "C" __attribute__((visibility("default"))) dhsa_status dhsa_mfma_probe(int random_operands, int iters,
                                                                              void *scratch_dev, size_t scratch_bytes,
                                                                              double *tflops_host,
                                                                              double *shader_mhz_host, void *stream) {
    using namespace dhsa;
    if (!scratch_dev || !tflops_host) return DHSA_ERR_NULL;
    if (iters < 1 || iters > (1 << 22)) return DHSA_ERR_SHAPE;
    if (scratch_bytes < dhsa_mfma_probe_scratch_bytes()) return DHSA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long *words = (unsigned long long *)scratch_dev;
    float *sink = (float *)((char *)scratch_dev + 256);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return DHSA_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return DHSA_ERR_HIP; }
    dhsa_status st = DHSA_OK;
    hipLaunchKernelGGL(k_mfma_probe, dim3(kProbeBlocks), dim3(256), 0, s, sink, words, iters < 64 ? iters : 64,
                       random_operands);   // untimed first launch
    if (hipEventRecord(e0, s) != hipSuccess) st = DHSA_ERR_HIP;
    hipLaunchKernelGGL(k_mfma_probe, dim3(kProbeBlocks), dim3(256), 0, s, sink, words, iters, random_operands);
    if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess)
        st = DHSA_ERR_HIP;
    float ms = 0.f;
    unsigned long long w[2] = {0, 0};
    if (st == DHSA_OK && (hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
                          hipMemcpy(w, words, sizeof(w), hipMemcpyDeviceToHost) != hipSuccess))
        st = DHSA_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != DHSA_OK) return st;
    const double flop = (double)kProbeBlocks * 4 * (double)iters * 16 * (2.0 * 32 * 32 * 16);
    *tflops_host = flop / (ms * 1e-3) / 1e12;
    if (shader_mhz_host) *shader_mhz_host = w[1] ? (double)w[0] / (double)w[1] * 100.0 : 0.0;
    return DHSA_OK;
}

extern "C" __attribute__((visibility("default"))) size_t dhsa_mfma_probe_scratch_bytes(void) {
    return 256 + (size_t)dhsa::kProbeBlocks * 256 * sizeof(float);
}
