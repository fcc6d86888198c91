// Bidirectional co-clustering (Algorithm 1): assignment, centroid update and the driver loop.
//
// Assignment of one side ("own") against the other ("opp").  Algorithm 1 asks for
//   L_i = argmin_j || Norm(x_i C_opp^T) - Norm(c_own_j C_opp^T) ||_2 .
// With row-wise L2 Norm, p^ = P / nx (nx = max(||P||, eps)) and pbar^_j the normalised anchor row,
//   ||p^ - pbar^_j||^2 = ||p^||^2 + b_j - 2 <x, W_j> / nx ,   W_j = C_opp^T pbar^_j ,  b_j = ||pbar^_j||^2
// so the N x K_opp affinity matrix never has to exist: W (K_own x d) is built once per half-step
// and every token needs one d-length dot product per own-side centroid.  b_j is exactly 1 unless
// ||c_own_j C_opp^T|| < eps (a degenerate anchor, e.g. an all-zero centroid); slices without
// such anchors reduce to argmax_j <x, W_j>.  Slices with one take the general form, which needs
// nx^2 = x^T (C_opp^T C_opp) x per token.
//
// Every decision is taken in float64: tokens are exact in float64, W is float64, accumulation is
// float64 in a fixed order.
#include <type_traits>

#include "common.h"

#define NORM_FLOOR 1e-12

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
__global__ void fill_i32_kernel(int32_t* p, int32_t v, size_t count) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

template <typename T>
__device__ __forceinline__ double load_as_f64(const T* p);
template <>
__device__ __forceinline__ double load_as_f64<uint16_t>(const uint16_t* p) { return (double)bf16_to_f32(*p); }
template <>
__device__ __forceinline__ double load_as_f64<float>(const float* p) { return (double)*p; }

// two consecutive elements as float64 (4-byte / 8-byte aligned address)
template <typename T>
__device__ __forceinline__ void load_pair(const T* p, double& a, double& b);
template <>
__device__ __forceinline__ void load_pair<uint16_t>(const uint16_t* p, double& a, double& b) {
    const uint32_t u = *(const uint32_t*)p;
    a = (double)__uint_as_float(u << 16);
    b = (double)__uint_as_float(u & 0xffff0000u);
}
template <>
__device__ __forceinline__ void load_pair<float>(const float* p, double& a, double& b) {
    const float2 u = *(const float2*)p;
    a = (double)u.x;
    b = (double)u.y;
}

// The per-slice words the next assignment accumulates into (degenerate flag, largest row norm, queue
// length) are cleared by the kernel that precedes it in the stream, not by a launch of their own.
__device__ __forceinline__ void clear_words(int32_t* clear, int clear_n) {
    if (clear && blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < clear_n; i += blockDim.x) clear[i] = 0;
}

// c64[b, c, :] = x[b, idx[b, c], :]   or   c64 = (double) init_c
template <typename T>
__global__ void init_centroids_kernel(const T* __restrict__ x, const int32_t* __restrict__ idx,
                                      const float* __restrict__ init_c, double* __restrict__ c64, int n, int k,
                                      int d, int32_t* __restrict__ clear, int clear_n) {
    const int b = blockIdx.y, c = blockIdx.x, t = threadIdx.x;
    clear_words(clear, clear_n);
    if (t >= d) return;
    double v;
    if (init_c) {
        v = (double)init_c[((size_t)b * k + c) * d + t];
    } else {
        int i = idx[(size_t)b * k + c];
        i = i < 0 ? 0 : (i >= n ? n - 1 : i);
        v = load_as_f64<T>(x + ((size_t)b * n + i) * d + t);
    }
    c64[((size_t)b * k + c) * d + t] = v;
}

__global__ void f64_to_f32_kernel(const double* __restrict__ src, float* __restrict__ dst, size_t count) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = (float)src[i];
}

__global__ void f32_to_f64_kernel(const float* __restrict__ src, double* __restrict__ dst, size_t count) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = (double)src[i];
}

// ---------------------------------------------------------------------------------------------
// Small batched float64 GEMM with arbitrary strides: C[m, n] = sum_k A(m, k) * B(k, n), on the
// float64 matrix instruction (v_mfma_f64_16x16x4_f64): one wave per 16 x 32 output tile, operands
// straight from global memory (the matrices are a few hundred KB and sit in L2) -- lane (i, kq) =
// (lane % 16, lane / 16) supplies A(m0 + i, k) and B(k, n0 + i), B(k, n0 + 16 + i) for the two
// contraction indices k = k0 + 2 kq, k0 + 2 kq + 1 of a block of 8 (any assignment of indices to
// the instruction's four contraction slots is valid as long as A and B agree); accumulator v of
// the lane holds C(m0 + kq + 4 v, n0 + i).  AK2 / BK2: the lane's two A / B values are adjacent
// in memory and 16-byte aligned, so one load fetches both.
// Used for G = C_opp^T C_opp (needed by slices with a degenerate anchor only; the other two small
// products of a half-step are inside anchor_w_kernel).
// ---------------------------------------------------------------------------------------------
struct GemmArgs {
    const double* a;
    const double* b;
    double* c;
    int m, n, k;
    long long a_batch, b_batch, c_batch;
    int a_sm, a_sk, b_sk, b_sn;
    const int32_t* only_if;   // nullable: per-batch flag; the batch is skipped when it is 0
};

typedef __attribute__((ext_vector_type(4))) double f64x4;

template <bool K2>
__device__ __forceinline__ void load_k_pair(const double* __restrict__ row, int k, int k_end, int sk, double& v0,
                                            double& v1) {
    if (K2 && k + 1 < k_end) {
        const double2 t = *(const double2*)(row + k);
        v0 = t.x;
        v1 = t.y;
    } else {
        v0 = k < k_end ? row[(size_t)k * sk] : 0.0;
        v1 = k + 1 < k_end ? row[(size_t)(k + 1) * sk] : 0.0;
    }
}

template <bool AK2, bool BK2>
__global__ void __launch_bounds__(64) gemm_f64_kernel(GemmArgs g) {
    if (g.only_if && g.only_if[blockIdx.z] == 0) return;
    const double* a = g.a + (size_t)blockIdx.z * g.a_batch;
    const double* b = g.b + (size_t)blockIdx.z * g.b_batch;
    double* c = g.c + (size_t)blockIdx.z * g.c_batch;
    const int lane = threadIdx.x, i = lane % 16, kq = lane / 16;
    const int m0 = blockIdx.y * 16, n0 = blockIdx.x * 32;
    // rows / columns past the edge read row / column 0: their products only reach outputs that are not stored
    const double* ap = a + (size_t)(m0 + i < g.m ? m0 + i : 0) * g.a_sm;
    const double* bp0 = b + (size_t)(n0 + i < g.n ? n0 + i : 0) * g.b_sn;
    const double* bp1 = b + (size_t)(n0 + 16 + i < g.n ? n0 + 16 + i : 0) * g.b_sn;
    f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
    for (int k00 = 0; k00 < g.k; k00 += 32) {     // four blocks of 8 per trip: their loads are in flight together
        double a0[4], a1[4], b00[4], b01[4], b10[4], b11[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k00 + 8 * u + 2 * kq;       // past the end: zeros
            load_k_pair<AK2>(ap, k, g.k, g.a_sk, a0[u], a1[u]);
            load_k_pair<BK2>(bp0, k, g.k, g.b_sk, b00[u], b01[u]);
            load_k_pair<BK2>(bp1, k, g.k, g.b_sk, b10[u], b11[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0[u], b00[u], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0[u], b10[u], acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1[u], b01[u], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1[u], b11[u], acc1, 0, 0, 0);
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int m = m0 + kq + 4 * v;
        if (m < g.m) {
            if (n0 + i < g.n) c[(size_t)m * g.n + n0 + i] = acc0[v];
            if (n0 + 16 + i < g.n) c[(size_t)m * g.n + n0 + 16 + i] = acc1[v];
        }
    }
}

static void launch_gemm(const GemmArgs& g, int batch, hipStream_t stream) {
    dim3 grid((g.n + 31) / 32, (g.m + 15) / 16, batch);
    const bool ak2 = g.a_sk == 1 && g.a_sm % 2 == 0 && g.a_batch % 2 == 0 && ((uintptr_t)g.a & 15) == 0;
    const bool bk2 = g.b_sk == 1 && g.b_sn % 2 == 0 && g.b_batch % 2 == 0 && ((uintptr_t)g.b & 15) == 0;
    if (ak2 && bk2)
        hipLaunchKernelGGL((gemm_f64_kernel<true, true>), grid, dim3(64), 0, stream, g);
    else if (ak2)
        hipLaunchKernelGGL((gemm_f64_kernel<true, false>), grid, dim3(64), 0, stream, g);
    else if (bk2)
        hipLaunchKernelGGL((gemm_f64_kernel<false, true>), grid, dim3(64), 0, stream, g);
    else
        hipLaunchKernelGGL((gemm_f64_kernel<false, false>), grid, dim3(64), 0, stream, g);
}

// ---------------------------------------------------------------------------------------------
// Tiled float64 contraction of a 64-token tile against the rows of a matrix B [rows_b, D]:
//   MODE_ARGMAX    B = W; per token the row j maximising the score, lowest j on ties
//   MODE_QUADFORM  B = G (D x D, symmetric); per token x^T G x
// 256 threads = 16 x 16; thread (ty, tx) owns tokens 4ty..4ty+3 and B rows 4tx..4tx+3 of the
// current 64-row block.  The token tile stays in LDS as float64 for the whole kernel.
// ---------------------------------------------------------------------------------------------
enum { MODE_ARGMAX = 0, MODE_QUADFORM = 1 };

template <typename T, int D, int MODE>
__global__ void __launch_bounds__(256)
token_tile_kernel(const T* __restrict__ x, const double* __restrict__ bmat, int rows_b,
                  const double* __restrict__ bterm, const int32_t* __restrict__ flags,
                  const double* __restrict__ nx2, const int32_t* __restrict__ list,
                  const int32_t* __restrict__ list_count, int32_t force_general, int32_t* __restrict__ labels,
                  double* __restrict__ quad_out, int n) {
    extern __shared__ double smem[];
    double* xs = smem;                 // [D][65]
    double* ws = smem + D * 65;        // [16][65]
    double* red_s = ws + 16 * 65;      // [64][16]
    int32_t* red_j = (int32_t*)(red_s + 64 * 16);  // [64][16]
    int32_t* tok = red_j + 64 * 16;    // [64]

    const int b = blockIdx.y;
    const int count = list ? list_count[b] : n;
    // nx^2 is only consumed by slices with a degenerate anchor unless the caller forces it
    if (MODE == MODE_QUADFORM && !force_general && flags[b] == 0) return;
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    // one tile per workgroup when the grid covers every tile; a smaller grid walks the tiles
    for (int t0 = blockIdx.x * 64; t0 < count; t0 += gridDim.x * 64) {
    __syncthreads();   // the previous tile's last LDS reads are done
    if (tid < 64) {
        const int p = t0 + tid;
        tok[tid] = p < count ? (list ? list[(size_t)b * n + p] : p) : -1;
    }
    __syncthreads();
    // stage the token tile: thread -> token tid/4, elements part*4 .. +3 of every 16-chunk
    {
        const int token = tid / 4, part = tid % 4;
        const int ti = tok[token];
        const T* src = x + ((size_t)b * n + (ti < 0 ? 0 : ti)) * D;
        for (int kc = 0; kc < D; kc += 16)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int col = kc + part * 4 + e;
                xs[col * 65 + token] = ti < 0 ? 0.0 : load_as_f64<T>(src + col);
            }
    }
    const bool general = MODE == MODE_ARGMAX && (force_general || flags[b] != 0);
    double nx_tok[4] = {0, 0, 0, 0};
    if (general) {
        for (int a = 0; a < 4; ++a) {
            const int ti = tok[ty * 4 + a];
            const double v = (ti < 0 || !nx2) ? 1.0 : nx2[(size_t)b * n + ti];   // no nx2: plain k-means scores
            const double r = sqrt(v > 0.0 ? v : 0.0);
            nx_tok[a] = r > NORM_FLOOR ? r : NORM_FLOOR;
        }
    }
    double best[4];
    int bestj[4] = {0, 0, 0, 0};
    double quad[4] = {0, 0, 0, 0};
    for (int a = 0; a < 4; ++a) best[a] = -INFINITY;
    const double* bm = bmat + (size_t)b * rows_b * D;
    const double* bt = bterm ? bterm + (size_t)b * rows_b : nullptr;

    for (int r0 = 0; r0 < rows_b; r0 += 64) {
        double acc[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[a][e] = 0.0;
        for (int kc = 0; kc < D; kc += 16) {
            __syncthreads();
            {
                const int row = tid / 4, part = tid % 4;
                const int j = r0 + row;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    ws[(part * 4 + e) * 65 + row] = j < rows_b ? bm[(size_t)j * D + kc + part * 4 + e] : 0.0;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                double xa[4], wb[4];
#pragma unroll
                for (int a = 0; a < 4; ++a) xa[a] = xs[(kc + kk) * 65 + ty * 4 + a];
#pragma unroll
                for (int e = 0; e < 4; ++e) wb[e] = ws[kk * 65 + tx * 4 + e];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[a][e] = fma(xa[a], wb[e], acc[a][e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = r0 + tx * 4 + e;
            if (j < rows_b) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    if (MODE == MODE_ARGMAX) {
                        const double val = general ? 2.0 * acc[a][e] - nx_tok[a] * bt[j] : acc[a][e];
                        if (val > best[a]) {
                            best[a] = val;
                            bestj[a] = j;
                        }
                    } else {
                        quad[a] = fma(acc[a][e], xs[j * 65 + ty * 4 + a], quad[a]);
                    }
                }
            }
        }
    }
    __syncthreads();
    for (int a = 0; a < 4; ++a) {
        red_s[(ty * 4 + a) * 16 + tx] = MODE == MODE_ARGMAX ? best[a] : quad[a];
        red_j[(ty * 4 + a) * 16 + tx] = bestj[a];
    }
    __syncthreads();
    if (tid < 64 && tok[tid] >= 0) {
        if (MODE == MODE_ARGMAX) {
            double bv = red_s[tid * 16];
            int bj = red_j[tid * 16];
            for (int u = 1; u < 16; ++u) {
                const double v = red_s[tid * 16 + u];
                const int j = red_j[tid * 16 + u];
                if (v > bv || (v == bv && j < bj)) {
                    bv = v;
                    bj = j;
                }
            }
            labels[(size_t)b * n + tok[tid]] = bj;
        } else {
            double s = 0.0;
            for (int u = 0; u < 16; ++u) s += red_s[tid * 16 + u];
            quad_out[(size_t)b * n + tok[tid]] = s;
        }
    }
    }   // tile loop
}

// ---------------------------------------------------------------------------------------------
// Float64 decision for the queued tokens of the matrix-core pre-filter: one workgroup per token
// (strided over the queue), one thread per centroid (j = tid, tid + 256, ...).  The token sits in
// LDS; thread j walks column j of the TRANSPOSED score matrix W^T [d, k_own], so that the 256
// threads read consecutive doubles, and adds the d products in index order -- the same fixed
// order, hence the same bits, as token_tile_kernel<MODE_ARGMAX>.  No cross-lane sums; one
// (value, index) reduction per token at the end.
// ---------------------------------------------------------------------------------------------
#define LIST_BATCH 32   // loads of W^T in flight per thread
template <typename T, int D>
__global__ void __launch_bounds__(256)
assign_list_kernel(const T* __restrict__ x, const double* __restrict__ wt, int k_own,
                   const double* __restrict__ bterm, const int32_t* __restrict__ flags,
                   const double* __restrict__ nx2, const int32_t* __restrict__ list,
                   const int32_t* __restrict__ list_count, int32_t force_general, int32_t* __restrict__ labels,
                   int n) {
    __shared__ double xs[D];
    __shared__ double best_v[4];
    __shared__ int32_t best_j[4];
    const int b = blockIdx.y, tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    int count = list_count[b];
    count = count > n ? n : count;
    const bool general = force_general || flags[b] != 0;
    const double* wb = wt + (size_t)b * D * k_own;
    for (int p = blockIdx.x; p < count; p += gridDim.x) {
        int ti = list[(size_t)b * n + p];
        ti = ti < 0 ? 0 : (ti >= n ? n - 1 : ti);
        if (tid < D) xs[tid] = load_as_f64<T>(x + ((size_t)b * n + ti) * D + tid);
        double nx = 0.0;
        if (general) {
            const double v = nx2 ? nx2[(size_t)b * n + ti] : 1.0;   // no nx2: plain k-means scores
            const double r = sqrt(v > 0.0 ? v : 0.0);
            nx = r > NORM_FLOOR ? r : NORM_FLOOR;
        }
        __syncthreads();
        double best = -INFINITY;
        int bj = 0x7fffffff;
        for (int j = tid; j < k_own; j += 256) {         // ascending j per thread: ">" keeps the lowest index
            const double* wc = wb + j;
            double sum = 0.0;
            // LIST_BATCH loads in flight, then their products: the fence keeps the compiler from turning the
            // batch into one load and one wait at a time (the loads are long round trips)
#pragma unroll 1
            for (int c0 = 0; c0 < D; c0 += LIST_BATCH) {
                double wv[LIST_BATCH];
#pragma unroll
                for (int u = 0; u < LIST_BATCH; ++u) wv[u] = wc[(size_t)(c0 + u) * k_own];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < LIST_BATCH; ++u) sum = fma(xs[c0 + u], wv[u], sum);
                __builtin_amdgcn_sched_barrier(0);
            }
            const double val = general ? 2.0 * sum - nx * bterm[(size_t)b * k_own + j] : sum;
            if (val > best || bj == 0x7fffffff) {
                best = val;
                bj = j;
            }
        }
        // (value, index) maximum, lowest index among equal values: within the wave, then across the four
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const double ov = __shfl_xor(best, off);
            const int oj = __shfl_xor(bj, off);
            if (oj != 0x7fffffff && (bj == 0x7fffffff || ov > best || (ov == best && oj < bj))) {
                best = ov;
                bj = oj;
            }
        }
        if (lane == 0) {
            best_v[wave] = best;
            best_j[wave] = bj;
        }
        __syncthreads();
        if (tid == 0) {
            double bv = best_v[0];
            int jj = best_j[0];
            for (int u = 1; u < 4; ++u)
                if (best_j[u] != 0x7fffffff && (jj == 0x7fffffff || best_v[u] > bv || (best_v[u] == bv && best_j[u] < jj))) {
                    bv = best_v[u];
                    jj = best_j[u];
                }
            labels[(size_t)b * n + ti] = jj == 0x7fffffff ? 0 : jj;
        }
        __syncthreads();
    }
}

template <int D>
static constexpr size_t token_tile_lds() {
    return (size_t)(D * 65 + 16 * 65 + 64 * 16) * sizeof(double) + (64 * 16 + 64) * sizeof(int32_t);
}

template <typename T, int D, int MODE>
static void launch_token_tile(const T* x, const double* bmat, int rows_b, const double* bterm, const int32_t* flags,
                              const double* nx2, const int32_t* list, const int32_t* list_count, int force_general,
                              int32_t* labels, double* quad_out, int bh, int n, hipStream_t stream) {
    auto kern = token_tile_kernel<T, D, MODE>;
    static unsigned char opted_in[SVOO_MAX_DEVICES];
    if (!opt_in_dynamic_lds((const void*)kern, (int)token_tile_lds<D>(), opted_in))
        return;   // the failure stays recorded as HIP's last error: the caller's launch_status() reports it
    // The quadratic form is skipped by every slice without a degenerate anchor unless it is forced:
    // a small grid that walks the tiles keeps that common case at a few microseconds.
    const int tiles = (n + 63) / 64;
    const bool mostly_skipped = MODE == MODE_QUADFORM && !force_general;
    dim3 grid(mostly_skipped && tiles > 64 ? 64 : tiles, bh);
    hipLaunchKernelGGL(kern, grid, dim3(256), token_tile_lds<D>(), stream, x, bmat, rows_b, bterm, flags, nx2, list,
                       list_count, force_general, labels, quad_out, n);
}

template <int MODE>
static void dispatch_token_tile(const svoo_shape* s, const void* x, const double* bmat, int rows_b,
                                const double* bterm, const int32_t* flags, const double* nx2, const int32_t* list,
                                const int32_t* list_count, int force_general, int32_t* labels, double* quad_out,
                                hipStream_t stream) {
    if (s->dtype == SVOO_BF16) {
        if (s->d == 128)
            launch_token_tile<uint16_t, 128, MODE>((const uint16_t*)x, bmat, rows_b, bterm, flags, nx2, list,
                                                   list_count, force_general, labels, quad_out, s->bh, s->n, stream);
        else
            launch_token_tile<uint16_t, 64, MODE>((const uint16_t*)x, bmat, rows_b, bterm, flags, nx2, list,
                                                  list_count, force_general, labels, quad_out, s->bh, s->n, stream);
    } else {
        if (s->d == 128)
            launch_token_tile<float, 128, MODE>((const float*)x, bmat, rows_b, bterm, flags, nx2, list, list_count,
                                                force_general, labels, quad_out, s->bh, s->n, stream);
        else
            launch_token_tile<float, 64, MODE>((const float*)x, bmat, rows_b, bterm, flags, nx2, list, list_count,
                                               force_general, labels, quad_out, s->bh, s->n, stream);
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 matrix-core pre-filter for the assignment (bf16 tokens only).
//
// W is split into two bf16 terms, W = W_hi + W_lo + r with |r| <= 2^-17 |W| element-wise; tokens
// are exact in bf16, so  f_j = <x, W_hi_j> + <x, W_lo_j>  (fp32 accumulation on the matrix cores)
// satisfies |f_j - <x, W_j>| <= eps ||x|| ||W_j|| with eps covering the split remainder and the
// fp32 accumulation of 2 d products.  If best - second > 2 eps ||x|| max_j ||W_j|| the fast
// argmax is the exact argmax; otherwise (and for every token of a slice with a degenerate
// anchor) the token is queued and the float64 kernel decides.  Equal scores have gap 0 and are
// therefore always decided by the float64 kernel, which breaks ties towards the lowest index.
//
// Tokens are the B operand (one token per lane column, loaded straight from global memory into
// registers, 64 tokens per wave), W blocks of 32 centroids are the A operand, streamed through
// LDS with direct global->LDS loads and an XOR swizzle, double buffered.  S^T layout: lane
// (j, h) holds for token j the centroids 32 cb + 8 (v/4) + 4 h + v%4.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
#define ASSIGN_LIST_WGS 256   // workgroups per slice that share the queue of undecided tokens
#define FAST_EPS 3.1e-5f   // 2^-16 + 256 * 2^-24, twice the analytic bound for d <= 128

// The split of a float64 score matrix for the pre-filter as a launch of its own (k-means, where W is the
// centroid array itself): 16 rows per workgroup (one wave takes four of them), one atomic per workgroup;
// also writes W^T in float64
template <int D>
__global__ void __launch_bounds__(256)
split_w_kernel(const double* __restrict__ w64, uint16_t* __restrict__ whi, uint16_t* __restrict__ wlo,
               double* __restrict__ wt, int32_t* __restrict__ wmax_bits, int k_own) {
    __shared__ float wave_max[4];
    const int b = blockIdx.y, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    float mx = 0.f;
    for (int r = 0; r < 4; ++r) {
        const int j = blockIdx.x * 16 + wave * 4 + r;
        if (j >= k_own) break;                         // uniform per wave
        double sq = 0.0;
        for (int t = lane; t < D; t += 64) {
            const size_t o = ((size_t)b * k_own + j) * D + t;
            const double v = w64[o];
            const uint16_t hb = f32_to_bf16((float)v);
            whi[o] = hb;
            wlo[o] = f32_to_bf16((float)(v - (double)bf16_to_f32(hb)));
            wt[((size_t)b * D + t) * k_own + j] = v;       // W^T [d, k_own] for the float64 queue kernel
            sq = fma(v, v, sq);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
        float nrm = (float)sqrt(sq);
        nrm = nrm * 1.0000002f + 1e-37f;   // round up
        if (!(nrm < 3.0e38f)) nrm = 3.0e38f;
        mx = fmaxf(mx, nrm);
    }
    if (lane == 0) wave_max[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float m = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
        atomicMax(&wmax_bits[b], __float_as_int(m));   // non-negative floats order like their bit patterns
    }
}

// Everything the assignment needs from the centroids, for 16 own-side centroids per workgroup:
//   P    = C_own[16 rows] C_opp^T          (float64 matrix instruction, tiles kept in LDS)
//   P^   = rows of P divided by max(||row||, floor);  b_j, degenerate flag
//   W    = P^ C_opp                        (16 x D)
//   and, for bf16 tokens, W's two-term bf16 split, W^T and the slice's largest row norm.
// One launch instead of GEMM, normalisation, GEMM and split; the K_own x K_opp matrix never leaves
// the chip.  Eight waves: wave w owns the column tiles w, w + 8, .. of each product and two rows of
// the row-wise steps.  Lane (i, kq) = (lane % 16, lane / 16) feeds row / column i and the contraction
// indices k0 + 2 kq, k0 + 2 kq + 1 of a block of 8; accumulator v holds row kq + 4 v, column i.
#define ANCHOR_WAVES 8
template <int D>
__global__ void __launch_bounds__(64 * ANCHOR_WAVES)
anchor_w_kernel(const double* __restrict__ c_own, const double* __restrict__ c_opp, int k_own, int k_opp,
                double* __restrict__ w64, double* __restrict__ bterm, int32_t* __restrict__ flags,
                uint16_t* __restrict__ whi, uint16_t* __restrict__ wlo, double* __restrict__ wt,
                int32_t* __restrict__ wmax_bits) {
    extern __shared__ __attribute__((aligned(16))) double anchor_lds[];
    constexpr int NW = ANCHOR_WAVES, RPW = 16 / NW;      // rows per wave in the row-wise steps
    __shared__ float wave_max[NW];
    const int pitch = ((k_opp + 31) / 32) * 32 + 2;     // even: 16-byte aligned pairs; columns past k_opp hold 0
    double* ps = anchor_lds;                            // [16][pitch]
    double* wtile = anchor_lds + 16 * pitch;            // [16][D + 2]
    const int b = blockIdx.y, row0 = blockIdx.x * 16;
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, i = lane % 16, kq = lane / 16;
    const double* co = c_own + (size_t)b * k_own * D;
    const double* cp = c_opp + (size_t)b * k_opp * D;

    // ---- P tile
    {
        const double* arow = co + (size_t)(row0 + i < k_own ? row0 + i : k_own - 1) * D + 2 * kq;
        double2 a[D / 8];
#pragma unroll
        for (int kb = 0; kb < D / 8; ++kb) a[kb] = *(const double2*)(arow + 8 * kb);
        for (int ct = wave; ct * 16 < k_opp; ct += NW) {
            const int n = ct * 16 + i;
            const double* brow = cp + (size_t)(n < k_opp ? n : k_opp - 1) * D + 2 * kq;
            f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kb = 0; kb < D / 8; ++kb) {
                const double2 bb = *(const double2*)(brow + 8 * kb);
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[kb].x, bb.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[kb].y, bb.y, acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) ps[(kq + 4 * v) * pitch + n] = n < k_opp ? acc[v] : 0.0;
        }
        const int filled = ((k_opp + 15) / 16) * 16, rest = pitch - filled;
        for (int e = threadIdx.x; e < 16 * rest; e += 64 * NW) ps[(e / rest) * pitch + filled + e % rest] = 0.0;
    }
    __syncthreads();
    // ---- row-wise L2 normalisation, b_j, degenerate flag
    for (int r = 0; r < RPW; ++r) {
        double* row = ps + (RPW * wave + r) * pitch;
        double sq = 0.0;
        for (int c = lane; c < k_opp; c += 64) sq = fma(row[c], row[c], sq);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
        const double nrm = sqrt(sq);
        const double div = nrm > NORM_FLOOR ? nrm : NORM_FLOOR;
        for (int c = lane; c < k_opp; c += 64) row[c] = row[c] / div;
        const int j = row0 + RPW * wave + r;
        if (lane == 0 && j < k_own) {
            const bool degenerate = !(nrm >= NORM_FLOOR);
            const double q = nrm / NORM_FLOOR;
            bterm[(size_t)b * k_own + j] = degenerate ? q * q : 1.0;
            if (degenerate) atomicOr(&flags[b], 1);
        }
    }
    __syncthreads();
    // ---- W tile = P^ C_opp: wave w owns the 16-column tiles w, w + NW, ..; the next trip's operands are
    // requested before the current trip's matrix instructions
    {
        constexpr int TILES = D / 16, NT = (TILES + NW - 1) / NW;
        if (wave < TILES) {
            f64x4 acc[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = f64x4{0.0, 0.0, 0.0, 0.0};
            const double* prow = ps + i * pitch + 2 * kq;
            double b0[4][NT], b1[4][NT];
            auto fetch = [&](int k00, double (&f0)[4][NT], double (&f1)[4][NT]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int k = k00 + 8 * u + 2 * kq;
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const int col = (wave + NW * t) * 16 + i;
                        const bool cv = wave + NW * t < TILES;
                        f0[u][t] = cv && k < k_opp ? cp[(size_t)k * D + col] : 0.0;
                        f1[u][t] = cv && k + 1 < k_opp ? cp[(size_t)(k + 1) * D + col] : 0.0;
                    }
                }
            };
            fetch(0, b0, b1);
            for (int k00 = 0; k00 < k_opp; k00 += 32) {
                double n0[4][NT], n1[4][NT];
                fetch(k00 + 32, n0, n1);          // past the end: zeros, no loads
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const double2 pa = *(const double2*)(prow + k00 + 8 * u);
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(pa.x, b0[u][t], acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(pa.y, b1[u][t], acc[t], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        b0[u][t] = n0[u][t];
                        b1[u][t] = n1[u][t];
                    }
            }
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (wave + NW * t < TILES)
#pragma unroll
                    for (int v = 0; v < 4; ++v) wtile[(kq + 4 * v) * (D + 2) + (wave + NW * t) * 16 + i] = acc[t][v];
        }
    }
    __syncthreads();
    // ---- outputs: W, and for the matrix-core pre-filter its bf16 split, W^T and the largest row norm
    float mx = 0.f;
    for (int r = 0; r < RPW; ++r) {
        const int j = row0 + RPW * wave + r;
        if (j >= k_own) break;                         // uniform per wave
        double sq = 0.0;
        for (int t = lane; t < D; t += 64) {
            const size_t o = ((size_t)b * k_own + j) * D + t;
            const double v = wtile[(RPW * wave + r) * (D + 2) + t];
            w64[o] = v;
            if (whi) {
                const uint16_t hb = f32_to_bf16((float)v);
                whi[o] = hb;
                wlo[o] = f32_to_bf16((float)(v - (double)bf16_to_f32(hb)));
                wt[((size_t)b * D + t) * k_own + j] = v;
            }
            sq = fma(v, v, sq);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
        float nrm = (float)sqrt(sq);
        nrm = nrm * 1.0000002f + 1e-37f;   // round up
        if (!(nrm < 3.0e38f)) nrm = 3.0e38f;
        mx = fmaxf(mx, nrm);
    }
    if (whi) {
        if (lane == 0) wave_max[wave] = mx;
        __syncthreads();
        if (threadIdx.x == 0) {
            float m = wave_max[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) m = fmaxf(m, wave_max[w]);
            atomicMax(&wmax_bits[b], __float_as_int(m));   // non-negative floats order like their bit patterns
        }
    }
}

template <int D>
static void launch_anchor_w(const double* c_own, const double* c_opp, int k_own, int k_opp, int bh, double* w64,
                            double* bterm, int32_t* flags, uint16_t* whi, uint16_t* wlo, double* wt,
                            int32_t* wmax_bits, hipStream_t stream) {
    auto kern = anchor_w_kernel<D>;
    const int pitch = ((k_opp + 31) / 32) * 32 + 2;
    const int lds = (16 * pitch + 16 * (D + 2)) * (int)sizeof(double);
    // the LDS need grows with k_opp: opt in once for the largest (k_opp = 1024) so that the flag holds for every call
    constexpr int lds_max = (16 * (SVOO_MAX_K + 2) + 16 * (D + 2)) * (int)sizeof(double);
    static unsigned char opted_in[SVOO_MAX_DEVICES];
    if (!opt_in_dynamic_lds((const void*)kern, lds_max, opted_in))
        return;   // stays recorded as HIP's last error: the caller's launch_status() reports it
    hipLaunchKernelGGL(kern, dim3((k_own + 15) / 16, bh), dim3(64 * ANCHOR_WAVES), lds, stream, c_own, c_opp, k_own,
                       k_opp, w64, bterm, flags, whi, wlo, wt, wmax_bits);
}

// BIAS: score_j = <x, W_j> - half_sq[j] (k-means on raw rows: W = C, half_sq = ||c_j||^2 / 2, one
// float per centroid, slices padded to a multiple of 32 entries); the margin then also covers the
// float32 rounding of the bias and of the subtraction.
template <int D, bool BIAS>
__global__ void __launch_bounds__(256, 2)
assign_mfma_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ whi, const uint16_t* __restrict__ wlo,
                   const int32_t* __restrict__ wmax_bits, const int32_t* __restrict__ flags,
                   const float* __restrict__ half_sq, int32_t* __restrict__ labels, int32_t* __restrict__ list,
                   int32_t* __restrict__ list_count, int n, int k_own) {
    constexpr int DC = D / 16, CPR = D / 8, ROWB = D * 2;
    constexpr int HALF = 32 * ROWB;          // one 32-centroid block of W_hi (or W_lo)
    constexpr int RPL = 64 / CPR;            // rows per wave-load
    constexpr int LPW = (32 / RPL) / 4;      // wave-loads per wave for one half block
    __shared__ __attribute__((aligned(1024))) unsigned char wl[2 * 2 * HALF];   // [buf][hi|lo][32][ROWB]
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid % 64, j = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);     // uniform: what derives from it stays scalar
    const int t0 = blockIdx.x * 256 + 64 * wave;
    const unsigned char* whb = (const unsigned char*)whi + (size_t)b * k_own * ROWB;
    const unsigned char* wlb = (const unsigned char*)wlo + (size_t)b * k_own * ROWB;
    const int n_blocks = (k_own + 31) / 32;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(wl));

    auto issue_block = [&](int cb, int buf) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int rl = (wave * LPW + i) * RPL + lane / CPR;     // row of the block, 0..31
            int row = 32 * cb + rl;
            row = row < k_own ? row : k_own - 1;
            const int chunk = (lane % CPR) ^ (rl % CPR);
            const uint32_t goff = (uint32_t)row * ROWB + chunk * 16;
            const uint32_t loff = lds0 + buf * 2 * HALF + (wave * LPW + i) * RPL * ROWB;
            load_rows_to_lds_16(goff, whb, loff);
            load_rows_to_lds_16(goff, wlb, loff + HALF);
        }
    };
    issue_block(0, 0);

    // token fragments and squared norms (the norm only scales the margin below, whose constant has a factor
    // of two in hand: the packed dot product's own rounding does not matter).  Rows past the end are read
    // from the last token instead of being predicated; their results are never stored.
    bf16x8_t xf[2][DC];
    float xn2[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int tok = t0 + 32 * tb + j;
        const uint4* src = (const uint4*)(x + ((size_t)b * n + (tok < n ? tok : n - 1)) * D);
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < DC; ++c) {
            const uint4 u = src[2 * c + h];
            xf[tb][c] = __builtin_bit_cast(bf16x8_t, u);
            const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bf16x2_t pr = __builtin_bit_cast(bf16x2_t, wds[e]);
                acc = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, acc, false);
            }
        }
        const int ai = __float_as_int(acc);
        auto r = __builtin_amdgcn_permlane32_swap(ai, ai, false, false);
        xn2[tb] = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    int koff[DC];
#pragma unroll
    for (int c = 0; c < DC; ++c) koff[c] = j * ROWB + (((2 * c + h) ^ (j % CPR)) * 16);
    // the compiler's wait for the token loads must not end up inside the block loop
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int c = 0; c < DC; ++c) asm volatile("" ::"v"(xf[tb][c]));

    float best[2] = {-INFINITY, -INFINITY}, second[2] = {-INFINITY, -INFINITY};
    int bidx[2] = {0, 0}, lidx[2] = {0, 0};
    for (int cb = 0; cb < n_blocks; ++cb) {
        const int buf = cb & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (cb + 1 < n_blocks) issue_block(cb + 1, buf ^ 1);
        const unsigned char* base = wl + buf * 2 * HALF;
        f32x16_t acc[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tb][v] = 0.f;
#pragma unroll
        for (int c = 0; c < DC; ++c) {
            const bf16x8_t ah = __builtin_bit_cast(bf16x8_t, *(const uint4*)(base + koff[c]));
            const bf16x8_t al = __builtin_bit_cast(bf16x8_t, *(const uint4*)(base + HALF + koff[c]));
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, xf[tb][c], acc[tb], 0, 0, 0);
                acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, xf[tb][c], acc[tb], 0, 0, 0);
            }
        }
        const int cbase = 32 * cb;      // uniform; the lane's own offset 4 h is added to the winner once, after the loop
        if (BIAS) {
            const float4* hb = (const float4*)(half_sq + (size_t)b * (32 * n_blocks) + cbase + 4 * h);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 t = hb[2 * g];
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    acc[tb][4 * g] -= t.x;
                    acc[tb][4 * g + 1] -= t.y;
                    acc[tb][4 * g + 2] -= t.z;
                    acc[tb][4 * g + 3] -= t.w;
                }
            }
        }
        if (cbase + 32 > k_own) {       // only the last block can hold centroids past the end: they never win
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (cbase + 4 * h + 8 * (v / 4) + (v % 4) >= k_own) acc[tb][v] = -INFINITY;
        }
        // best, second best and the winner: one median, one compare and two selects per score (selects instead
        // of a maximum keep the compiler from canonicalising every score first).  Inside the block only the
        // winner's position in the block is tracked (a small constant per score); the centroid index is
        // updated once per block, if the best moved.  The two token groups are independent chains and are
        // interleaved so that no select waits on its compare.
        float before[2] = {best[0], best[1]};
#pragma unroll
        for (int v = 0; v < 16; ++v)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const float val = acc[tb][v];
                second[tb] = __builtin_amdgcn_fmed3f(best[tb], second[tb], val);
                const bool up = val > best[tb];
                lidx[tb] = up ? 8 * (v / 4) + (v % 4) : lidx[tb];
                best[tb] = up ? val : best[tb];
            }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) bidx[tb] = best[tb] > before[tb] ? cbase + lidx[tb] : bidx[tb];
    }
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) bidx[tb] += 4 * h;
    const float wmax = __int_as_float(wmax_bits[b]);
    const bool degenerate = flags[b] != 0;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        auto rb = __builtin_amdgcn_permlane32_swap(__float_as_int(best[tb]), __float_as_int(best[tb]), false, false);
        auto rs = __builtin_amdgcn_permlane32_swap(__float_as_int(second[tb]), __float_as_int(second[tb]), false, false);
        auto ri = __builtin_amdgcn_permlane32_swap(bidx[tb], bidx[tb], false, false);
        // for lanes < 32: [0] is the own value, [1] the other half's
        const float b0 = __int_as_float(rb[0]), b1 = __int_as_float(rb[1]);
        const float s0 = __int_as_float(rs[0]), s1 = __int_as_float(rs[1]);
        const float fb = fmaxf(b0, b1);
        const float fs = fmaxf(fminf(b0, b1), fmaxf(s0, s1));
        const int fi = b0 >= b1 ? (int)ri[0] : (int)ri[1];
        const int tok = t0 + 32 * tb + j;
        if (h == 0 && tok < n) {
            const float xw = sqrtf(xn2[tb]) * wmax;
            const float margin = BIAS ? 2.0f * (FAST_EPS * xw + 2.4e-7f * (0.5f * wmax * wmax + xw))   // 2^-22
                                      : 2.0f * FAST_EPS * xw;
            const bool sure = (fb - fs) > margin;          // false for NaN as well
            labels[(size_t)b * n + tok] = fi;
            if (degenerate || !sure) {
                const int pos = atomicAdd(&list_count[b], 1);
                if (pos >= 0 && pos < n) list[(size_t)b * n + pos] = tok;   // always true when the counter started at zero
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Centroid update: C[j] = mean of the member rows, float64 sums in a fixed order.
// One workgroup per (cluster, slice); members are perm[offsets[j] .. offsets[j+1]) in ascending
// token order.  256 threads = G row-groups of D/8 lanes; a lane adds elements 8l .. 8l+7 (one
// 16-byte load for bf16) of the rows g, g+G, g+2G, ... of its group, then the G partial sums are
// added in group order.
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void load8_as_f64(const T* p, double (&v)[8]);
template <>
__device__ __forceinline__ void load8_as_f64<uint16_t>(const uint16_t* p, double (&v)[8]) {
    const uint4 u = *(const uint4*)p;
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = (double)__uint_as_float(w[e] << 16);
        v[2 * e + 1] = (double)__uint_as_float(w[e] & 0xffff0000u);
    }
}
template <>
__device__ __forceinline__ void load8_as_f64<float>(const float* p, double (&v)[8]) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

#define CU_ROWS 8   // rows in flight per lane (4: 41 us, 8: 38 us, 12: 43 us per launch at 12 x 75,600 x 128 bf16; was 47 with 2)
template <typename T, int D>
__global__ void __launch_bounds__(256)
centroid_update_kernel(const T* __restrict__ x, const int32_t* __restrict__ perm,
                       const int32_t* __restrict__ offsets, double* __restrict__ c64, float* __restrict__ c32,
                       int32_t* __restrict__ counts, int n, int k, int32_t* __restrict__ clear, int clear_n) {
    clear_words(clear, clear_n);
    constexpr int LANES = D / 8;
    constexpr int GROUPS = 256 / LANES;
    __shared__ double part[GROUPS][D];
    const int b = blockIdx.y, j = blockIdx.x;
    const int lane = threadIdx.x % LANES, grp = threadIdx.x / LANES;
    int beg = offsets[(size_t)b * (k + 1) + j], end = offsets[(size_t)b * (k + 1) + j + 1];
    beg = beg < 0 ? 0 : beg;
    end = end > n ? n : end;
    const int32_t* pm = perm + (size_t)b * n;
    auto member = [&](int pos) {       // a permutation entry outside [0, n) must not leave the tensor
        const int t = pm[pos];
        return t < 0 ? 0 : (t >= n ? n - 1 : t);
    };
    const T* xb = x + (size_t)b * n * D + 8 * lane;
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int p = beg + grp;
    // ROWS rows in flight per lane (the kernel is bound by the latency of its scattered 256-byte reads),
    // added in row order whatever the batch size, so the sums do not depend on it
    auto batch = [&](auto rows_c) {
        constexpr int ROWS = decltype(rows_c)::value;
        for (; p + (ROWS - 1) * GROUPS < end; p += ROWS * GROUPS) {
            double a[ROWS][8];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) load8_as_f64<T>(xb + (size_t)member(p + r * GROUPS) * D, a[r]);
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e) s[e] += a[r][e];
        }
    };
    batch(std::integral_constant<int, CU_ROWS>{});
    batch(std::integral_constant<int, 2>{});
    if (p < end) {
        double a0[8];
        load8_as_f64<T>(xb + (size_t)member(p) * D, a0);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += a0[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[grp][8 * lane + e] = s[e];
    __syncthreads();
    const int cnt = end - beg;
    if (threadIdx.x < D) {
        const size_t o = ((size_t)b * k + j) * D + threadIdx.x;
        if (cnt > 0) {
            double t = part[0][threadIdx.x];
            for (int g = 1; g < GROUPS; ++g) t += part[g][threadIdx.x];
            c64[o] = t / (double)cnt;
        }
        if (c32) c32[o] = (float)c64[o];
    }
    if (threadIdx.x == 0 && counts) counts[(size_t)b * k + j] = cnt;
}

// clear / clear_n: words to zero for the assignment that follows in the stream (nullable)
static void launch_centroid_update(const svoo_shape* s, const void* x, const int32_t* perm, const int32_t* offsets,
                                   double* c64, float* c32, int32_t* counts, int k, int32_t* clear, int clear_n,
                                   hipStream_t stream) {
    dim3 grid(k, s->bh);
    if (s->dtype == SVOO_BF16) {
        if (s->d == 128)
            hipLaunchKernelGGL((centroid_update_kernel<uint16_t, 128>), grid, dim3(256), 0, stream, (const uint16_t*)x,
                               perm, offsets, c64, c32, counts, s->n, k, clear, clear_n);
        else
            hipLaunchKernelGGL((centroid_update_kernel<uint16_t, 64>), grid, dim3(256), 0, stream, (const uint16_t*)x,
                               perm, offsets, c64, c32, counts, s->n, k, clear, clear_n);
    } else {
        if (s->d == 128)
            hipLaunchKernelGGL((centroid_update_kernel<float, 128>), grid, dim3(256), 0, stream, (const float*)x, perm,
                               offsets, c64, c32, counts, s->n, k, clear, clear_n);
        else
            hipLaunchKernelGGL((centroid_update_kernel<float, 64>), grid, dim3(256), 0, stream, (const float*)x, perm,
                               offsets, c64, c32, counts, s->n, k, clear, clear_n);
    }
}

// ---------------------------------------------------------------------------------------------
// Objective (diagnostic): D_i = ||p^_i||^2 + b_L - 2 <x_i, W_L> / nx_i, summed per slice in a
// fixed order.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
objective_terms_kernel(const T* __restrict__ x, const double* __restrict__ w, const double* __restrict__ bterm,
                       const double* __restrict__ nx2, const int32_t* __restrict__ labels,
                       double* __restrict__ terms, int n, int k_own, int d) {
    const int b = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int l = labels[(size_t)b * n + i];
    const T* xr = x + ((size_t)b * n + i) * d;
    const double* wr = w + ((size_t)b * k_own + l) * d;
    double s = 0.0;
    for (int c = 0; c < d; ++c) s = fma(load_as_f64<T>(xr + c), wr[c], s);
    const double v = nx2[(size_t)b * n + i];
    const double r = sqrt(v > 0.0 ? v : 0.0);
    const double nx = r > NORM_FLOOR ? r : NORM_FLOOR;
    const double pn2 = (r * r) / (nx * nx);
    terms[(size_t)b * n + i] = pn2 + bterm[(size_t)b * k_own + l] - 2.0 * s / nx;
}

__global__ void __launch_bounds__(1024)
objective_sum_kernel(const double* __restrict__ terms, double* __restrict__ out, int n, int out_stride) {
    __shared__ double red[1024];
    const int b = blockIdx.x, t = threadIdx.x;
    double s = 0.0;
    for (int i = t; i < n; i += 1024) s += terms[(size_t)b * n + i];
    red[t] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    if (t == 0) out[(size_t)b * out_stride] = red[0];
}

// ---------------------------------------------------------------------------------------------
// Independent k-means on raw rows: argmin_j ||x - c_j||^2 = argmax_j 2 <x, c_j> - ||c_j||^2, i.e.
// the same scoring kernels with W = C, anchor term ||c_j||^2 and token norm 1.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(128)
kmeans_prep_kernel(const double* __restrict__ c64, double* __restrict__ bterm, float* __restrict__ half_sq, int k,
                   int kpad, int d) {
    __shared__ double red[128];
    const int b = blockIdx.y, j = blockIdx.x, t = threadIdx.x;
    double v = 0.0;
    if (j < k && t < d) v = c64[((size_t)b * k + j) * d + t];
    red[t] = v * v;
    __syncthreads();
    for (int s = 64; s > 0; s >>= 1) {
        if (t < s) red[t] += red[t + s];
        __syncthreads();
    }
    if (t == 0) {
        if (j < k) bterm[(size_t)b * k + j] = red[0];
        half_sq[(size_t)b * kpad + j] = j < k ? (float)(0.5 * red[0]) : 0.f;
    }
}

// terms[i] = ||x_i - c_{L_i}||^2, summed term by term
template <typename T>
__global__ void __launch_bounds__(256)
kmeans_inertia_terms_kernel(const T* __restrict__ x, const double* __restrict__ c64,
                            const int32_t* __restrict__ labels, double* __restrict__ terms, int n, int k, int d) {
    const int b = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int l = labels[(size_t)b * n + i];
    const T* xr = x + ((size_t)b * n + i) * d;
    const double* cr = c64 + ((size_t)b * k + l) * d;
    double s = 0.0;
    for (int c = 0; c < d; ++c) {
        const double df = load_as_f64<T>(xr + c) - cr[c];
        s = fma(df, df, s);
    }
    terms[(size_t)b * n + i] = s;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct ClusterWs {
    double *c64q, *c64k, *w64, *wt64, *gram, *bterm, *nx2, *terms;
    uint16_t *whi, *wlo;
    float* half_sq;
    int32_t *flags, *wmax_bits, *list_count, *list, *perm, *offsets, *chunk_hist;
    size_t bytes;
};

static ClusterWs carve_cluster_ws(const svoo_shape* s, void* ws) {
    WsCarver c(ws);
    ClusterWs w;
    const size_t bh = s->bh, kmax = s->kq > s->kk ? s->kq : s->kk;
    w.c64q = c.take<double>(bh * s->kq * s->d);
    w.c64k = c.take<double>(bh * s->kk * s->d);
    w.w64 = c.take<double>(bh * kmax * s->d);
    w.wt64 = c.take<double>(bh * kmax * s->d);
    w.gram = c.take<double>(bh * (size_t)s->d * s->d);
    w.bterm = c.take<double>(bh * kmax);
    w.nx2 = c.take<double>(bh * (size_t)s->n);
    w.terms = c.take<double>(bh * (size_t)s->n);
    w.whi = c.take<uint16_t>(bh * kmax * s->d);
    w.wlo = c.take<uint16_t>(bh * kmax * s->d);
    w.half_sq = c.take<float>(bh * ((kmax + 31) / 32 * 32));
    w.flags = c.take<int32_t>(3 * bh);      // flags | wmax_bits | list_count, cleared by one fill
    w.wmax_bits = w.flags + bh;
    w.list_count = w.flags + 2 * bh;
    w.list = c.take<int32_t>(bh * (size_t)s->n);
    w.perm = c.take<int32_t>(bh * (size_t)s->n);
    w.offsets = c.take<int32_t>(bh * (kmax + 1));
    w.chunk_hist = c.take<int32_t>(sort_scratch_ints(s->bh, s->n, (int)kmax));
    w.bytes = c.used;
    return w;
}

size_t cluster_ws_bytes(const svoo_shape* s) { return carve_cluster_ws(s, nullptr).bytes; }

// One half-step's assignment: labels of x against own-side centroids through opp-side anchors.
// want_nx2: also fill w.nx2 (needed for the objective) even if no anchor is degenerate.
// words_cleared: the preceding kernel of the stream has zeroed w.flags / wmax_bits / list_count.
static int assign_side(const svoo_shape* s, const ClusterWs& w, const void* x, const double* c_own, int k_own,
                       const double* c_opp, int k_opp, int32_t* labels, bool want_nx2, bool words_cleared,
                       hipStream_t stream) {
    const int d = s->d, bh = s->bh;
    if (!words_cleared)
        hipLaunchKernelGGL(fill_i32_kernel, dim3((3 * bh + 255) / 256), dim3(256), 0, stream, w.flags, 0,
                           (size_t)3 * bh);
    // W = Norm(C_own C_opp^T) C_opp with b_j and the degenerate flags; for bf16 tokens also the split of W,
    // its transpose and the largest row norm for the matrix-core pre-filter
    {
        const bool bf16 = s->dtype == SVOO_BF16;
        uint16_t* whi = bf16 ? w.whi : nullptr;
        if (d == 128)
            launch_anchor_w<128>(c_own, c_opp, k_own, k_opp, bh, w.w64, w.bterm, w.flags, whi, w.wlo, w.wt64,
                                 w.wmax_bits, stream);
        else
            launch_anchor_w<64>(c_own, c_opp, k_own, k_opp, bh, w.w64, w.bterm, w.flags, whi, w.wlo, w.wt64,
                                w.wmax_bits, stream);
    }
    // G[a, b] = sum_c c_opp[c, a] * c_opp[c, b]
    // (only slices with a degenerate anchor need it, unless the objective is wanted)
    GemmArgs g3 = {c_opp, c_opp, w.gram, d, d, k_opp, (long long)k_opp * d, (long long)k_opp * d, (long long)d * d,
                   1, d, d, 1, want_nx2 ? nullptr : w.flags};
    launch_gemm(g3, bh, stream);
    // nx^2 = x^T G x: every workgroup of a slice without degenerate anchors exits at once unless the
    // objective wants it, so the launch sequence never depends on device-side flags.
    dispatch_token_tile<MODE_QUADFORM>(s, x, w.gram, d, nullptr, w.flags, nullptr, nullptr, nullptr, want_nx2 ? 1 : 0,
                                       nullptr, w.nx2, stream);
    if (s->dtype == SVOO_BF16) {
        // matrix-core pre-filter decides the clear cases; float64 decides the queued rest
        dim3 agrid((s->n + 255) / 256, bh);
        if (d == 128) {
            hipLaunchKernelGGL((assign_mfma_kernel<128, false>), agrid, dim3(256), 0, stream, (const uint16_t*)x, w.whi,
                               w.wlo, w.wmax_bits, w.flags, nullptr, labels, w.list, w.list_count, s->n, k_own);
        } else {
            hipLaunchKernelGGL((assign_mfma_kernel<64, false>), agrid, dim3(256), 0, stream, (const uint16_t*)x, w.whi,
                               w.wlo, w.wmax_bits, w.flags, nullptr, labels, w.list, w.list_count, s->n, k_own);
        }
        dim3 lgrid(s->n < ASSIGN_LIST_WGS ? s->n : ASSIGN_LIST_WGS, bh);
        if (d == 128)
            hipLaunchKernelGGL((assign_list_kernel<uint16_t, 128>), lgrid, dim3(256), 0, stream, (const uint16_t*)x,
                               w.wt64, k_own, w.bterm, w.flags, w.nx2, w.list, w.list_count, 0, labels, s->n);
        else
            hipLaunchKernelGGL((assign_list_kernel<uint16_t, 64>), lgrid, dim3(256), 0, stream, (const uint16_t*)x,
                               w.wt64, k_own, w.bterm, w.flags, w.nx2, w.list, w.list_count, 0, labels, s->n);
    } else {
        dispatch_token_tile<MODE_ARGMAX>(s, x, w.w64, k_own, w.bterm, w.flags, w.nx2, nullptr, nullptr, 0, labels,
                                         nullptr, stream);
    }
    return launch_status();
}

static void launch_objective(const svoo_shape* s, const ClusterWs& w, const void* x, int k_own,
                             const int32_t* labels, double* out, int out_stride, hipStream_t stream) {
    dim3 grid((s->n + 255) / 256, s->bh);
    if (s->dtype == SVOO_BF16)
        hipLaunchKernelGGL(objective_terms_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t*)x, w.w64,
                           w.bterm, w.nx2, labels, w.terms, s->n, k_own, s->d);
    else
        hipLaunchKernelGGL(objective_terms_kernel<float>, grid, dim3(256), 0, stream, (const float*)x, w.w64, w.bterm,
                           w.nx2, labels, w.terms, s->n, k_own, s->d);
    hipLaunchKernelGGL(objective_sum_kernel, dim3(s->bh), dim3(1024), 0, stream, w.terms, out, s->n, out_stride);
}

static void launch_init_centroids(const svoo_shape* s, const void* x, const int32_t* idx, const float* init_c,
                                  double* c64, int k, int32_t* clear, int clear_n, hipStream_t stream) {
    dim3 grid(k, s->bh);
    if (s->dtype == SVOO_BF16)
        hipLaunchKernelGGL(init_centroids_kernel<uint16_t>, grid, dim3(128), 0, stream, (const uint16_t*)x, idx, init_c,
                           c64, s->n, k, s->d, clear, clear_n);
    else
        hipLaunchKernelGGL(init_centroids_kernel<float>, grid, dim3(128), 0, stream, (const float*)x, idx, init_c, c64,
                           s->n, k, s->d, clear, clear_n);
}

// perm_* / *_offsets (all four or none): the cluster-order layout of the returned labels, which the
// last iteration's centroid updates need anyway
static int cocluster_impl(const svoo_shape* shape, const void* q, const void* k, const int32_t* init_q_idx,
                          const int32_t* init_k_idx, const float* init_cq, const float* init_ck, int32_t iters,
                          int32_t* labels_q, int32_t* labels_k, float* cq, float* ck, int32_t* counts_q,
                          int32_t* counts_k, double* objective, int32_t* perm_q, int32_t* q_offsets, int32_t* perm_k,
                          int32_t* k_offsets, void* ws, size_t ws_bytes, void* hip_stream) {
    int st = check_shape(shape, true);
    if (st != SVOO_OK) return st;
    if (!q || !k || !labels_q || !labels_k || !cq || !ck || !counts_q || !counts_k || !ws)
        return SVOO_ERR_INVALID_ARG;
    if ((!init_q_idx && !init_cq) || (!init_k_idx && !init_ck)) return SVOO_ERR_INVALID_ARG;
    if (iters < 1 || iters > 1000) return SVOO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || (((uintptr_t)ws) & 255u) != 0) return SVOO_ERR_INVALID_ARG;
    if (shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    const ClusterWs w = carve_cluster_ws(shape, ws);
    if (ws_bytes < w.bytes) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;

    launch_init_centroids(shape, q, init_q_idx, init_cq, w.c64q, shape->kq, nullptr, 0, stream);
    launch_init_centroids(shape, k, init_k_idx, init_ck, w.c64k, shape->kk, w.flags, 3 * shape->bh, stream);
    for (int it = 0; it < iters; ++it) {
        const bool last = it == iters - 1;
        // Step A: keys against query anchors (old C_q), own centroids old C_k.
        st = assign_side(shape, w, k, w.c64k, shape->kk, w.c64q, shape->kq, labels_k, objective != nullptr, true,
                         stream);
        if (st != SVOO_OK) return st;
        if (objective)
            launch_objective(shape, w, k, shape->kk, labels_k, objective + (size_t)it * 2, iters * 2, stream);
        int32_t* pk = last && perm_k ? perm_k : w.perm;
        int32_t* ok = last && perm_k ? k_offsets : w.offsets;
        st = sort_labels(shape->bh, shape->n, shape->kk, labels_k, pk, ok, nullptr, w.chunk_hist, stream);
        if (st != SVOO_OK) return st;
        launch_centroid_update(shape, k, pk, ok, w.c64k, last ? ck : nullptr, last ? counts_k : nullptr, shape->kk,
                               w.flags, 3 * shape->bh, stream);
        // Step B: queries against the NEW key anchors, own centroids the OLD C_q.
        st = assign_side(shape, w, q, w.c64q, shape->kq, w.c64k, shape->kk, labels_q, objective != nullptr, true,
                         stream);
        if (st != SVOO_OK) return st;
        if (objective)
            launch_objective(shape, w, q, shape->kq, labels_q, objective + (size_t)it * 2 + 1, iters * 2, stream);
        int32_t* pq = last && perm_q ? perm_q : w.perm;
        int32_t* oq = last && perm_q ? q_offsets : w.offsets;
        st = sort_labels(shape->bh, shape->n, shape->kq, labels_q, pq, oq, nullptr, w.chunk_hist, stream);
        if (st != SVOO_OK) return st;
        launch_centroid_update(shape, q, pq, oq, w.c64q, last ? cq : nullptr, last ? counts_q : nullptr, shape->kq,
                               w.flags, 3 * shape->bh, stream);
    }
    return launch_status();
}

extern "C" int svoo_cocluster(const svoo_shape* shape, const void* q, const void* k, const int32_t* init_q_idx,
                              const int32_t* init_k_idx, const float* init_cq, const float* init_ck, int32_t iters,
                              int32_t* labels_q, int32_t* labels_k, float* cq, float* ck, int32_t* counts_q,
                              int32_t* counts_k, double* objective, void* ws, size_t ws_bytes, void* hip_stream) {
    return cocluster_impl(shape, q, k, init_q_idx, init_k_idx, init_cq, init_ck, iters, labels_q, labels_k, cq, ck,
                          counts_q, counts_k, objective, nullptr, nullptr, nullptr, nullptr, ws, ws_bytes, hip_stream);
}

extern "C" int svoo_cocluster_sorted(const svoo_shape* shape, const void* q, const void* k, const int32_t* init_q_idx,
                                     const int32_t* init_k_idx, const float* init_cq, const float* init_ck,
                                     int32_t iters, int32_t* labels_q, int32_t* labels_k, float* cq, float* ck,
                                     int32_t* counts_q, int32_t* counts_k, double* objective, int32_t* perm_q,
                                     int32_t* q_offsets, int32_t* perm_k, int32_t* k_offsets, void* ws,
                                     size_t ws_bytes, void* hip_stream) {
    if (!perm_q || !q_offsets || !perm_k || !k_offsets) return SVOO_ERR_INVALID_ARG;
    return cocluster_impl(shape, q, k, init_q_idx, init_k_idx, init_cq, init_ck, iters, labels_q, labels_k, cq, ck,
                          counts_q, counts_k, objective, perm_q, q_offsets, perm_k, k_offsets, ws, ws_bytes,
                          hip_stream);
}

extern "C" int svoo_assign(const svoo_shape* shape, const void* x, const float* c_own, int32_t k_own,
                           const float* c_opp, int32_t k_opp, int32_t* labels, void* ws, size_t ws_bytes,
                           void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!x || !c_own || !c_opp || !labels || !ws) return SVOO_ERR_INVALID_ARG;
    if (k_own < 1 || k_opp < 1 || k_own > SVOO_MAX_K || k_opp > SVOO_MAX_K) return SVOO_ERR_INVALID_ARG;
    if (!aligned16(x) || (((uintptr_t)ws) & 255u) != 0 || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    svoo_shape s = *shape;
    s.kq = k_own;  // carve with own side in the "q" slot, opp side in the "k" slot
    s.kk = k_opp;
    const ClusterWs w = carve_cluster_ws(&s, ws);
    if (ws_bytes < w.bytes) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t n_own = (size_t)s.bh * k_own * s.d, n_opp = (size_t)s.bh * k_opp * s.d;
    hipLaunchKernelGGL(f32_to_f64_kernel, dim3((n_own + 255) / 256), dim3(256), 0, stream, c_own, w.c64q, n_own);
    hipLaunchKernelGGL(f32_to_f64_kernel, dim3((n_opp + 255) / 256), dim3(256), 0, stream, c_opp, w.c64k, n_opp);
    return assign_side(&s, w, x, w.c64q, k_own, w.c64k, k_opp, labels, false, false, stream);
}

// One Lloyd assignment: labels of x against centroids c64 [bh, k, d].
static int kmeans_assign(const svoo_shape* s, const ClusterWs& w, const void* x, const double* c64, int k,
                         int32_t* labels, hipStream_t stream) {
    const int d = s->d, bh = s->bh, kpad = (k + 31) / 32 * 32;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((3 * bh + 255) / 256), dim3(256), 0, stream, w.flags, 0,
                       (size_t)3 * bh);
    hipLaunchKernelGGL(kmeans_prep_kernel, dim3(kpad, bh), dim3(128), 0, stream, c64, w.bterm, w.half_sq, k, kpad, d);
    if (s->dtype == SVOO_BF16) {
        dim3 sgrid((k + 15) / 16, bh), agrid((s->n + 255) / 256, bh), lgrid(s->n < ASSIGN_LIST_WGS ? s->n : ASSIGN_LIST_WGS, bh);
        if (d == 128) {
            hipLaunchKernelGGL(split_w_kernel<128>, sgrid, dim3(256), 0, stream, c64, w.whi, w.wlo, w.wt64, w.wmax_bits, k);
            hipLaunchKernelGGL((assign_mfma_kernel<128, true>), agrid, dim3(256), 0, stream, (const uint16_t*)x, w.whi,
                               w.wlo, w.wmax_bits, w.flags, w.half_sq, labels, w.list, w.list_count, s->n, k);
            hipLaunchKernelGGL((assign_list_kernel<uint16_t, 128>), lgrid, dim3(256), 0, stream, (const uint16_t*)x,
                               w.wt64, k, w.bterm, w.flags, nullptr, w.list, w.list_count, 1, labels, s->n);
        } else {
            hipLaunchKernelGGL(split_w_kernel<64>, sgrid, dim3(256), 0, stream, c64, w.whi, w.wlo, w.wt64, w.wmax_bits, k);
            hipLaunchKernelGGL((assign_mfma_kernel<64, true>), agrid, dim3(256), 0, stream, (const uint16_t*)x, w.whi,
                               w.wlo, w.wmax_bits, w.flags, w.half_sq, labels, w.list, w.list_count, s->n, k);
            hipLaunchKernelGGL((assign_list_kernel<uint16_t, 64>), lgrid, dim3(256), 0, stream, (const uint16_t*)x,
                               w.wt64, k, w.bterm, w.flags, nullptr, w.list, w.list_count, 1, labels, s->n);
        }
    } else {
        dispatch_token_tile<MODE_ARGMAX>(s, x, c64, k, w.bterm, w.flags, nullptr, nullptr, nullptr, 1, labels, nullptr,
                                         stream);
    }
    return launch_status();
}

// workspace layout of svoo_kmeans: the co-clustering layout with the centroids in the "q" slot
static svoo_shape kmeans_ws_shape(const svoo_shape* shape, int k) {
    svoo_shape s = *shape;
    s.kq = k;
    s.kk = 1;
    return s;
}

size_t kmeans_ws_bytes(const svoo_shape* shape, int k) {
    const svoo_shape s = kmeans_ws_shape(shape, k);
    return carve_cluster_ws(&s, nullptr).bytes;
}

extern "C" int svoo_kmeans(const svoo_shape* shape, const void* x, int32_t k, const int32_t* init_idx,
                           const float* init_c, int32_t iters, int32_t* labels, float* c, int32_t* counts,
                           double* inertia, void* ws, size_t ws_bytes, void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!x || !labels || !c || !counts || !ws || (!init_idx && !init_c)) return SVOO_ERR_INVALID_ARG;
    if (k < 1 || k > SVOO_MAX_K || k > shape->n || iters < 1 || iters > 1000) return SVOO_ERR_INVALID_ARG;
    if (!aligned16(x) || (((uintptr_t)ws) & 255u) != 0 || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    const svoo_shape s = kmeans_ws_shape(shape, k);
    const ClusterWs w = carve_cluster_ws(&s, ws);
    if (ws_bytes < w.bytes) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;
    launch_init_centroids(&s, x, init_idx, init_c, w.c64q, k, nullptr, 0, stream);
    for (int it = 0; it < iters; ++it) {
        const bool last = it == iters - 1;
        st = kmeans_assign(&s, w, x, w.c64q, k, labels, stream);
        if (st != SVOO_OK) return st;
        if (inertia) {
            dim3 grid((s.n + 255) / 256, s.bh);
            if (s.dtype == SVOO_BF16)
                hipLaunchKernelGGL(kmeans_inertia_terms_kernel<uint16_t>, grid, dim3(256), 0, stream,
                                   (const uint16_t*)x, w.c64q, labels, w.terms, s.n, k, s.d);
            else
                hipLaunchKernelGGL(kmeans_inertia_terms_kernel<float>, grid, dim3(256), 0, stream, (const float*)x,
                                   w.c64q, labels, w.terms, s.n, k, s.d);
            hipLaunchKernelGGL(objective_sum_kernel, dim3(s.bh), dim3(1024), 0, stream, w.terms, inertia + it, s.n,
                               iters);
        }
        st = sort_labels(s.bh, s.n, k, labels, w.perm, w.offsets, nullptr, w.chunk_hist, stream);
        if (st != SVOO_OK) return st;
        launch_centroid_update(&s, x, w.perm, w.offsets, w.c64q, last ? c : nullptr, last ? counts : nullptr, k,
                               nullptr, 0, stream);
    }
    return launch_status();
}
