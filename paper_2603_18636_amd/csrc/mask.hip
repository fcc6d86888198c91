// Top Block-Pair Selection: which key blocks each query block attends to.
//
// One workgroup per (query block r, slice b), all arithmetic in float64 (the matrix is K_q x K_k;
// the cost is nothing next to the attention it prunes):
//   a_j  = scale * <cq[r], ck[j]>            coarse block estimate A_bar = C_q C_k^T
//   w_j  = n_j exp(a_j - max) / Z            softmax over non-empty key blocks, weighted by size
//   rank_j = position of j in the order by descending w, equal weights by lower index (bitonic sort in LDS)
//   m    = shortest sorted prefix with cumulative weight >= tau, summed sequentially in that order
//   b    = ceil(keep * K_k) (a product within 1e-6 K_k of an integer counts as that integer);
//          kept = (keep > theta ? min(m, b) : max(m, b)) clamped to [1, #live]
#include "common.h"

#define MASK_THREADS 256
#define MASK_PER_THREAD (SVOO_MAX_K / MASK_THREADS)

// A_bar[b, r, j] = <cq[b, r], ck[b, j]> in float64, the d products added in index order (32 x 32
// output tile per workgroup, 2 x 2 per thread), so that the selection kernel reads one coalesced
// row instead of every workgroup re-reading all key centroids.
__global__ void __launch_bounds__(256)
block_estimate_kernel(const float* __restrict__ cq, const float* __restrict__ ck, double* __restrict__ abar, int kq,
                      int kk, int d) {
    __shared__ double as[16][33];
    __shared__ double bs[16][33];
    const int b = blockIdx.z, m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const float* a = cq + (size_t)b * kq * d;
    const float* bm = ck + (size_t)b * kk * d;
    double acc[2][2] = {{0, 0}, {0, 0}};
    for (int k0 = 0; k0 < d; k0 += 16) {
        for (int e = threadIdx.x; e < 512; e += 256) {
            const int c = e % 16, r = e / 16;
            as[c][r] = (m0 + r < kq) ? (double)a[(size_t)(m0 + r) * d + k0 + c] : 0.0;
            bs[c][r] = (n0 + r < kk) ? (double)bm[(size_t)(n0 + r) * d + k0 + c] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const double a0 = as[c][ty * 2], a1 = as[c][ty * 2 + 1];
            const double b0 = bs[c][tx * 2], b1 = bs[c][tx * 2 + 1];
            acc[0][0] = fma(a0, b0, acc[0][0]);
            acc[0][1] = fma(a0, b1, acc[0][1]);
            acc[1][0] = fma(a1, b0, acc[1][0]);
            acc[1][1] = fma(a1, b1, acc[1][1]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {
            const int m = m0 + ty * 2 + i, n = n0 + tx * 2 + j;
            if (m < kq && n < kk) abar[((size_t)b * kq + m) * kk + n] = acc[i][j];
        }
}

__global__ void __launch_bounds__(MASK_THREADS)
block_mask_kernel(const double* __restrict__ abar, const int32_t* __restrict__ counts_q,
                  const int32_t* __restrict__ counts_k, const float* __restrict__ keep, double tau, double theta,
                  double scale, int32_t* __restrict__ block_count, int32_t* __restrict__ block_list,
                  uint8_t* __restrict__ bitmap, int kq, int kk, int d) {
    __shared__ double w[SVOO_MAX_K];
    __shared__ double w_sorted[SVOO_MAX_K];
    __shared__ int32_t ord[SVOO_MAX_K];
    __shared__ int32_t rank_s[SVOO_MAX_K];
    __shared__ double red[MASK_THREADS];
    __shared__ int32_t scan[MASK_THREADS];
    __shared__ int32_t n_keep_s;

    const int b = blockIdx.y, r = blockIdx.x, t = threadIdx.x;
    const size_t row_off = ((size_t)b * kq + r) * kk;
    const int nq = counts_q[(size_t)b * kq + r];
    if (nq <= 0) {  // empty query block: nothing kept
        for (int j = t; j < kk; j += MASK_THREADS) {
            block_list[row_off + j] = -1;
            if (bitmap) bitmap[row_off + j] = 0;
        }
        if (t == 0) block_count[(size_t)b * kq + r] = 0;
        return;
    }

    // logits and their maximum over non-empty key blocks
    double a[MASK_PER_THREAD];
    int nk[MASK_PER_THREAD];
    double mx = -INFINITY;
    int live_local = 0;
#pragma unroll
    for (int u = 0; u < MASK_PER_THREAD; ++u) {
        const int j = t + u * MASK_THREADS;
        a[u] = 0.0;
        nk[u] = 0;
        if (j < kk) {
            nk[u] = counts_k[(size_t)b * kk + j];
            a[u] = scale * abar[row_off + j];
            if (nk[u] > 0) {
                mx = a[u] > mx ? a[u] : mx;
                ++live_local;
            }
        }
    }
    red[t] = mx;
    scan[t] = live_local;
    __syncthreads();
    for (int s = MASK_THREADS / 2; s > 0; s >>= 1) {
        if (t < s) {
            red[t] = red[t + s] > red[t] ? red[t + s] : red[t];
            scan[t] += scan[t + s];
        }
        __syncthreads();
    }
    mx = red[0];
    const int n_live = scan[0];
    __syncthreads();
    if (n_live == 0) {  // no key at all: keep nothing
        for (int j = t; j < kk; j += MASK_THREADS) {
            block_list[row_off + j] = -1;
            if (bitmap) bitmap[row_off + j] = 0;
        }
        if (t == 0) block_count[(size_t)b * kq + r] = 0;
        return;
    }

    // unnormalised weights, their sum in a fixed order (index order inside a thread, then a tree)
    double e[MASK_PER_THREAD];
    double zs = 0.0;
#pragma unroll
    for (int u = 0; u < MASK_PER_THREAD; ++u) {
        e[u] = nk[u] > 0 ? (double)nk[u] * exp(a[u] - mx) : 0.0;
        zs += e[u];
    }
    red[t] = zs;
    __syncthreads();
    for (int s = MASK_THREADS / 2; s > 0; s >>= 1) {
        if (t < s) red[t] += red[t + s];
        __syncthreads();
    }
    const double z = red[0];
#pragma unroll
    for (int u = 0; u < MASK_PER_THREAD; ++u) {
        const int j = t + u * MASK_THREADS;
        if (j < kk) w[j] = nk[u] > 0 ? e[u] / z : -1.0;  // -1 marks an empty key block
    }
    __syncthreads();

    // position in the descending order (ties: lower index first; empty blocks after all live ones)
    if (kk <= MASK_THREADS) {
        // few blocks: count, per block, the blocks that come before it (one block per thread)
        if (t < kk) {
            const double wj = w[t];
            int rk = 0;
            for (int o = 0; o < kk; ++o) {
                const double wo = w[o];
                rk += (wo > wj || (wo == wj && o < t)) ? 1 : 0;
            }
            ord[rk] = t;
        }
        __syncthreads();
    } else {
        // many blocks: bitonic sort of the block ids in LDS, compared through their weights
        int P = 1;
        while (P < kk) P <<= 1;
        for (int i = t; i < P; i += MASK_THREADS) ord[i] = i < kk ? i : -1;     // -1 pads up to a power of two
        __syncthreads();
        auto before = [&](int x, int y) {     // does x come before y in the order?
            const double wx = x < 0 ? -2.0 : w[x], wy = y < 0 ? -2.0 : w[y];
            return wx > wy || (wx == wy && (unsigned)x < (unsigned)y);
        };
        for (int k2 = 2; k2 <= P; k2 <<= 1)
            for (int j2 = k2 >> 1; j2 > 0; j2 >>= 1) {
                for (int i = t; i < P; i += MASK_THREADS) {
                    const int ixj = i ^ j2;
                    if (ixj > i) {
                        const int x = ord[i], y = ord[ixj];
                        const bool forward = (i & k2) == 0;
                        if (forward ? before(y, x) : before(x, y)) {
                            ord[i] = y;
                            ord[ixj] = x;
                        }
                    }
                }
                __syncthreads();
            }
    }
    for (int i = t; i < kk; i += MASK_THREADS) {
        const int j = ord[i];
        if (j >= 0) {
            rank_s[j] = i;
            w_sorted[i] = w[j];
        }
    }
    __syncthreads();
    int rank[MASK_PER_THREAD];
#pragma unroll
    for (int u = 0; u < MASK_PER_THREAD; ++u) {
        const int j = t + u * MASK_THREADS;
        rank[u] = (j < kk && nk[u] > 0) ? rank_s[j] : -1;
    }

    if (t == 0) {
        int m = n_live;
        if (tau < 1.0) {
            double csum = 0.0;
            for (int i = 0; i < n_live; ++i) {
                csum += w_sorted[i];
                if (csum >= tau) {
                    m = i + 1;
                    break;
                }
            }
        }
        // keep arrives as a float32: a decimal ratio whose product with K_k is an integer (0.3 x 20)
        // sits a hair above it, so a product within 1e-6 K_k of an integer is that integer
        const double kp = (double)keep[b];
        const double prod = kp * (double)kk, nearest = rint(prod);
        const int budget = fabs(prod - nearest) <= 1e-6 * (double)kk ? (int)nearest : (int)ceil(prod);
        int n_keep = kp > theta ? (m < budget ? m : budget) : (m > budget ? m : budget);
        n_keep = n_keep > n_live ? n_live : n_keep;
        n_keep = n_keep < 1 ? 1 : n_keep;
        n_keep_s = n_keep;
        block_count[(size_t)b * kq + r] = n_keep;
    }
    __syncthreads();
    const int n_keep = n_keep_s;

    // compact the kept ids in ascending order: thread t owns ids t, t+256, ...; do it per stripe
    int base = 0;
    for (int u = 0; u < MASK_PER_THREAD && u * MASK_THREADS < kk; ++u) {   // stripes past kk hold nothing
        const int j = t + u * MASK_THREADS;
        const int kept = (j < kk && rank[u] >= 0 && rank[u] < n_keep) ? 1 : 0;
        if (j < kk && bitmap) bitmap[row_off + j] = (uint8_t)kept;
        scan[t] = kept;
        __syncthreads();
        for (int s = 1; s < MASK_THREADS; s <<= 1) {
            const int v = t >= s ? scan[t - s] : 0;
            __syncthreads();
            scan[t] += v;
            __syncthreads();
        }
        if (kept) block_list[row_off + base + scan[t] - 1] = j;
        base += scan[MASK_THREADS - 1];
        __syncthreads();
    }
    for (int j = n_keep + t; j < kk; j += MASK_THREADS) block_list[row_off + j] = -1;
}

size_t mask_ws_bytes(const svoo_shape* s) { return align_up((size_t)s->bh * s->kq * s->kk * sizeof(double), 256); }

extern "C" int svoo_block_mask(const svoo_shape* shape, const float* cq, const float* ck, const int32_t* counts_q,
                               const int32_t* counts_k, const float* keep, float tau, float theta, float scale,
                               int32_t* block_count, int32_t* block_list, uint8_t* bitmap, void* ws, size_t ws_bytes,
                               void* hip_stream) {
    int st = check_shape(shape, true);
    if (st != SVOO_OK) return st;
    if (!cq || !ck || !counts_q || !counts_k || !keep || !block_count || !block_list) return SVOO_ERR_INVALID_ARG;
    if (!(tau > 0.0f) || !(tau <= 1.0f) || !(scale == scale) || !(theta == theta)) return SVOO_ERR_INVALID_ARG;
    if (shape->bh > 65535 || !ws || (((uintptr_t)ws) & 255u) != 0) return SVOO_ERR_INVALID_ARG;
    if (ws_bytes < mask_ws_bytes(shape)) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;
    double* abar = (double*)ws;
    hipLaunchKernelGGL(block_estimate_kernel, dim3((shape->kk + 31) / 32, (shape->kq + 31) / 32, shape->bh), dim3(256), 0,
                       stream, cq, ck, abar, shape->kq, shape->kk, shape->d);
    hipLaunchKernelGGL(block_mask_kernel, dim3(shape->kq, shape->bh), dim3(MASK_THREADS), 0, stream, abar, counts_q,
                       counts_k, keep, (double)tau, (double)theta, (double)scale, block_count, block_list, bitmap,
                       shape->kq, shape->kk, shape->d);
    return launch_status();
}
