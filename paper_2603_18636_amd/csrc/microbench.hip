// Measurement aids, not part of the method: what this GPU sustains on the two resources the
// roofline figures of the attention and row-mover kernels are quoted against.
//   svoo_microbench_mfma_bf16   register-resident v_mfma_f32_32x32x16_bf16 chains, nothing else
//   svoo_microbench_copy        16-byte grid-stride copy
#include "common.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define MB_THREADS 256          // 4 waves, one per SIMD
#define MB_MFMA_PER_ITER 16
#define MB_MFMA_FLOPS (2.0 * 32 * 32 * 16)

// Four independent accumulator chains per wave, so the matrix pipeline never waits on its own
// result; operands stay in registers.  The clock the chip holds depends on how many operand bits
// toggle, so the operands are either pseudo-random (like real data) or one constant.
__global__ void __launch_bounds__(MB_THREADS) mfma_chain_kernel(int iters, int random_operands, float* sink) {
    const unsigned tid = blockIdx.x * MB_THREADS + threadIdx.x;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned ha = (tid * 131u + c * 17u + e + 1u) * 2654435761u;
            const unsigned hb = (tid * 31u + c * 7u + e + 5u) * 2246822519u;
            const float fa = random_operands ? (float)(ha >> 16) / 32768.f - 1.f : 0.5f;
            const float fb = random_operands ? (float)(hb >> 16) / 32768.f - 1.f : 0.5f;
            a[c][e] = (__bf16)(0.25f * fa);
            b[c][e] = (__bf16)(0.25f * fb);
        }
    f32x16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < MB_MFMA_PER_ITER; ++c)
            acc[c % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c % 8], b[(c / 2) % 8], acc[c % 4], 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) r += acc[t][e];
    sink[tid] = r;
}

// Each workgroup walks 16 KB chunks; a thread has four 16-byte loads in flight before it stores.
__global__ void __launch_bounds__(256) copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 1024;
    for (size_t base = (size_t)blockIdx.x * 1024; base < n16; base += stride) {
        const size_t i = base + threadIdx.x;
        if (base + 1024 <= n16) {
            const uint4 a = src[i], b = src[i + 256], c = src[i + 512], d = src[i + 768];
            dst[i] = a;
            dst[i + 256] = b;
            dst[i + 512] = c;
            dst[i + 768] = d;
        } else {
            for (size_t t = i; t < n16; t += 256) dst[t] = src[t];
        }
    }
}

extern "C" int svoo_microbench_mfma_bf16(int32_t workgroups, int32_t iters, int32_t random_operands, float* sink,
                                         double* flops, void* hip_stream) {
    if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || !sink) return SVOO_ERR_INVALID_ARG;
    if (((uintptr_t)sink & 3) != 0) return SVOO_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_chain_kernel, dim3(workgroups), dim3(MB_THREADS), 0, (hipStream_t)hip_stream, (int)iters,
                       (int)random_operands, sink);
    if (hipGetLastError() != hipSuccess) return SVOO_ERR_HIP;
    if (flops) *flops = (double)workgroups * (MB_THREADS / 64) * (double)iters * MB_MFMA_PER_ITER * MB_MFMA_FLOPS;
    return SVOO_OK;
}

extern "C" int svoo_microbench_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
    if (!src || !dst || bytes == 0 || bytes % 16 != 0) return SVOO_ERR_INVALID_ARG;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) != 0) return SVOO_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    size_t wgs = (n16 + 1023) / 1024;
    if (wgs > 4096) wgs = 4096;
    hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)src,
                       (uint4*)dst, n16);
    return hipGetLastError() == hipSuccess ? SVOO_OK : SVOO_ERR_HIP;
}
