// Measurement aids, not part of the method: what this GPU sustains on the two resources the
// roofline figures of the attention and row-mover kernels are quoted against.
//   svoo_microbench_mfma_bf16   register-resident v_mfma_f32_32x32x16_bf16 chains, nothing else
//   svoo_microbench_copy        16-byte grid-stride copy
//   svoo_microbench_attn_tile   the data movement of one attention tile step through the LDS, piece by piece
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

// ---------------------------------------------------------------------------------------------
// What one 64-key tile step of the bf16 attention kernel (d = 128, four waves of 32 query rows, two
// workgroups per CU) moves through the LDS, without the softmax arithmetic: per wave 16 K fragment
// reads (ds_read_b128), 32 V fragment reads (transposing ds_read_b64_tr_b16), 8 direct global->LDS
// loads of 1 KB (the workgroup's 32 KB tile, out of L2), and the 32 matrix instructions they feed --
// any subset, chosen by `parts` (bit 0 K reads, 1 V reads, 2 direct loads, 3 matrix instructions).
// Same LDS layout, swizzles and read addresses as the attention kernel; one barrier per step.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

template <int PARTS>
__global__ void __launch_bounds__(256, 2) attn_tile_skeleton_kernel(const unsigned char* __restrict__ src, int iters, float* sink) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];   // 2 buffers x (16 KB K tile + 16 KB V tile)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, j = lane % 32, h = lane / 32;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    const unsigned char* base = src + (size_t)(blockIdx.x % 64) * 65536;      // 4 MB over the grid: stays in L2
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8 b;
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = (__bf16)(0.25f * ((float)(((tid * 131u + e + 1u) * 2654435761u) >> 16) / 32768.f - 1.f));
    uint4 keep = make_uint4(0, 0, 0, 0);
    int koff[8], voff[2][4];
#pragma unroll
    for (int c = 0; c < 8; ++c) koff[c] = j * 256 + (((2 * c + h) ^ (j % 16)) * 16);
    {
        const int s = lane % 16, blk = lane / 16;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int rho = 8 * u + 4 * (blk / 2) + s / 4, chunk = 4 * db + 2 * (blk % 2) + (s % 4) / 2;
                voff[u][db] = rho * 256 + ((chunk ^ ((rho % 4) << 2)) * 16) + (s % 2) * 8;
            }
    }
    if (PARTS & 3) {     // the reads below need defined data in both buffers
        for (int e = tid; e < 65536 / 16; e += 256) ((uint4*)smem)[e] = ((const uint4*)base)[e];
        __syncthreads();
    }
    for (int it = 0; it < iters; ++it) {
        const int buf = it & 1;
        if (PARTS & 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t row = (uint32_t)(((it * 37 + wave * 4 + i) * 4 + lane / 16) & 127);
                const uint32_t off = row * 256 + (lane % 16) * 16;
                load_rows_to_lds_16(off, base, lds0 + (buf ^ 1) * 32768 + (wave * 4 + i) * 1024);
                load_rows_to_lds_16(off, base + 32768, lds0 + (buf ^ 1) * 32768 + 16384 + (wave * 4 + i) * 1024);
            }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                bf16x8 a = b;
                if (PARTS & 1)
                    a = __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) uint4*)(uintptr_t)(uint32_t)(
                                                       lds0 + buf * 32768 + kb * 8192 + koff[c]));
                if (PARTS & 8) {
                    acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[kb], 0, 0, 0);
                } else {
                    const uint4 u = __builtin_bit_cast(uint4, a);
                    keep.x += u.x;
                    keep.y ^= u.w;
                }
            }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    bf16x8 a = b;
                    if (PARTS & 2) {
                        const uint32_t cst = lds0 + buf * 32768 + 16384 + (32 * kb + 16 * t) * 256;
                        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                            (__attribute__((address_space(3))) bf16x4*)(uintptr_t)(uint32_t)(cst + voff[0][db]));
                        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                            (__attribute__((address_space(3))) bf16x4*)(uintptr_t)(uint32_t)(cst + voff[1][db]));
                        a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
                    if (PARTS & 8) {
                        acc[(t + db) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[(t + db) & 1], 0, 0, 0);
                    } else {
                        const uint4 u = __builtin_bit_cast(uint4, a);
                        keep.z += u.x;
                        keep.w ^= u.w;
                    }
                }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    float r = (float)(keep.x + keep.y + keep.z + keep.w);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) r += acc[i][e];
    sink[blockIdx.x * 256 + tid] = r;
}

template <int PARTS>
static int launch_tile_skeleton(const void* src, int iters, float* sink, hipStream_t stream) {
    static unsigned char opted_in[SVOO_MAX_DEVICES];
    if (!opt_in_dynamic_lds((const void*)attn_tile_skeleton_kernel<PARTS>, 65536, opted_in)) return SVOO_ERR_HIP;
    hipLaunchKernelGGL(attn_tile_skeleton_kernel<PARTS>, dim3(512), dim3(256), 65536, stream, (const unsigned char*)src, iters, sink);
    return hipGetLastError() == hipSuccess ? SVOO_OK : SVOO_ERR_HIP;
}

extern "C" int svoo_microbench_attn_tile(int32_t parts, int32_t iters, const void* src, float* sink, void* hip_stream) {
    if (parts < 1 || parts > 15 || iters < 1 || !src || !sink || !aligned16(src)) return SVOO_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    switch (parts) {
        case 1: return launch_tile_skeleton<1>(src, iters, sink, stream);
        case 2: return launch_tile_skeleton<2>(src, iters, sink, stream);
        case 3: return launch_tile_skeleton<3>(src, iters, sink, stream);
        case 4: return launch_tile_skeleton<4>(src, iters, sink, stream);
        case 7: return launch_tile_skeleton<7>(src, iters, sink, stream);
        case 8: return launch_tile_skeleton<8>(src, iters, sink, stream);
        case 11: return launch_tile_skeleton<11>(src, iters, sink, stream);
        case 15: return launch_tile_skeleton<15>(src, iters, sink, stream);
        default: return SVOO_ERR_INVALID_ARG;     // the other subsets are not instantiated
    }
}
