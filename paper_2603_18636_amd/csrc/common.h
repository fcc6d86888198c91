// Shared host/device helpers of libsvoo (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "svoo.h"

#define SVOO_MAX_K 1024
#define SVOO_WAVE 64

// ---------------------------------------------------------------------------------------------
// bf16 <-> float (bit-level; bf16 is the upper half of an IEEE binary32)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Direct global -> LDS load, 16 bytes per lane: lane l of the wave lands at LDS byte address
// lds_addr + 16 l (lds_addr wave-uniform).  Issued through inline assembly on purpose: the compiler
// then does not track an asynchronous LDS write and puts no "wait for every outstanding load" in
// front of later LDS reads of OTHER buffers, which would undo the prefetch.  Ordering against the
// reads of the buffer being filled is the caller's job (s_waitcnt vmcnt(..) followed by a barrier).
// m0 is on the clobber list so that the compiler never carries a value of its own in m0 across the
// statement (it treats m0 as reserved and says so with a warning, silenced here).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_global_to_lds_16(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(__builtin_amdgcn_readfirstlane(lds_addr))
                 : "memory", "m0");
}

// The same with a wave-uniform 64-bit base address (kept in scalar registers) and a 32-bit byte
// offset per lane.
__device__ __forceinline__ void load_rows_to_lds_16(uint32_t byte_offset, const void* uniform_base, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(byte_offset), "s"(uniform_base), "s"(__builtin_amdgcn_readfirstlane(lds_addr))
                 : "memory", "m0");
}
#pragma clang diagnostic pop

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// ---------------------------------------------------------------------------------------------
// host-side helpers
// ---------------------------------------------------------------------------------------------
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

static inline int elem_size(int dtype) { return dtype == SVOO_BF16 ? 2 : 4; }

// Shape checks shared by every entry point.  Returns SVOO_OK or the error to hand back.
static inline int check_shape(const svoo_shape* s, bool need_clusters) {
    if (!s) return SVOO_ERR_INVALID_ARG;
    if (s->bh < 1 || s->n < 1 || s->n > (1 << 24)) return SVOO_ERR_INVALID_ARG;
    if ((long long)s->bh * s->n > 0x7fffffffLL) return SVOO_ERR_INVALID_ARG;
    if (s->dtype != SVOO_BF16 && s->dtype != SVOO_F32) return SVOO_ERR_UNSUPPORTED;
    if (s->d != 64 && s->d != 128) return SVOO_ERR_UNSUPPORTED;
    if (need_clusters) {
        if (s->kq < 1 || s->kk < 1 || s->kq > SVOO_MAX_K || s->kk > SVOO_MAX_K) return SVOO_ERR_INVALID_ARG;
        if (s->kq > s->n || s->kk > s->n) return SVOO_ERR_INVALID_ARG;
    }
    return SVOO_OK;
}

// Bump allocator over the caller's workspace; every block 256-byte aligned.
struct WsCarver {
    char* base;
    size_t used;
    explicit WsCarver(void* p) : base((char*)p), used(0) {}
    template <typename T>
    T* take(size_t count) {
        T* r = (T*)(base + used);
        used += align_up(count * sizeof(T), 256);
        return r;
    }
};

static inline int launch_status() { return hipGetLastError() == hipSuccess ? SVOO_OK : SVOO_ERR_HIP; }

// Kernels that use more than 64 KB of dynamic LDS must opt in through a function attribute, once
// per kernel and device.  `done` is a per-kernel-instantiation table (one flag per device ordinal);
// racing first calls from two host threads both set the attribute, which is harmless.
#define SVOO_MAX_DEVICES 64
static inline bool opt_in_dynamic_lds(const void* kernel, int bytes, unsigned char (&done)[SVOO_MAX_DEVICES]) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (dev >= 0 && dev < SVOO_MAX_DEVICES && done[dev]) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    if (dev >= 0 && dev < SVOO_MAX_DEVICES) done[dev] = 1;
    return true;
}

// ---------------------------------------------------------------------------------------------
// internal entry points shared between translation units
// ---------------------------------------------------------------------------------------------
// Stable counting sort of labels [bh, n] into perm / offsets (and counts, nullable).
// chunk_hist: scratch int32 [bh * sort_chunks(n) * n_clusters].
size_t sort_scratch_ints(int bh, int n, int n_clusters);
int sort_labels(int bh, int n, int n_clusters, const int32_t* labels, int32_t* perm, int32_t* offsets,
                int32_t* counts, int32_t* chunk_hist, hipStream_t stream);
