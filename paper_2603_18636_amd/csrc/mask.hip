// Top Block-Pair Selection: which key blocks each query block attends to.
//
// One workgroup per (query block r, slice b), all arithmetic in float64 (the matrix is K_q x K_k;
// the cost is nothing next to the attention it prunes):
//   a_j  = scale * <cq[r], ck[j]>            coarse block estimate A_bar = C_q C_k^T
//   w_j  = n_j exp(a_j - max) / Z            softmax over non-empty key blocks, weighted by size
//   rank_j = #{j' : w_j' > w_j, or equal and j' < j}     (position in the descending order)
//   m    = shortest sorted prefix with cumulative weight >= tau, summed sequentially in that order
//   b    = ceil(keep * K_k);  kept = (keep > theta ? min(m, b) : max(m, b)) clamped to [1, #live]
#include "common.h"

#define MASK_THREADS 256
#define MASK_PER_THREAD (SVOO_MAX_K / MASK_THREADS)

__global__ void __launch_bounds__(MASK_THREADS)
block_mask_kernel(const float* __restrict__ cq, const float* __restrict__ ck, const int32_t* __restrict__ counts_q,
                  const int32_t* __restrict__ counts_k, const float* __restrict__ keep, double tau, double theta,
                  double scale, int32_t* __restrict__ block_count, int32_t* __restrict__ block_list,
                  uint8_t* __restrict__ bitmap, int kq, int kk, int d) {
    __shared__ double w[SVOO_MAX_K];
    __shared__ double w_sorted[SVOO_MAX_K];
    __shared__ double qrow[128];
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
    if (t < d) qrow[t] = (double)cq[((size_t)b * kq + r) * d + t];
    __syncthreads();

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
            const float* kr = ck + ((size_t)b * kk + j) * d;
            double s = 0.0;
            for (int c = 0; c < d; ++c) s = fma(qrow[c], (double)kr[c], s);
            a[u] = scale * s;
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

    // rank in the descending order (ties: lower index first); empty blocks are not ranked
    int rank[MASK_PER_THREAD];
#pragma unroll
    for (int u = 0; u < MASK_PER_THREAD; ++u) {
        const int j = t + u * MASK_THREADS;
        rank[u] = -1;
        if (j < kk && nk[u] > 0) {
            const double wj = w[j];
            int rk = 0;
            for (int o = 0; o < kk; ++o) {
                const double wo = w[o];
                rk += (wo > wj || (wo == wj && o < j)) ? 1 : 0;
            }
            rank[u] = rk;
            w_sorted[rk] = wj;
        }
    }
    __syncthreads();

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
        const double kp = (double)keep[b];
        const int budget = (int)ceil(kp * (double)kk);
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
    for (int u = 0; u < MASK_PER_THREAD; ++u) {
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

extern "C" int svoo_block_mask(const svoo_shape* shape, const float* cq, const float* ck, const int32_t* counts_q,
                               const int32_t* counts_k, const float* keep, float tau, float theta, float scale,
                               int32_t* block_count, int32_t* block_list, uint8_t* bitmap, void* ws, size_t ws_bytes,
                               void* hip_stream) {
    (void)ws;
    (void)ws_bytes;
    int st = check_shape(shape, true);
    if (st != SVOO_OK) return st;
    if (!cq || !ck || !counts_q || !counts_k || !keep || !block_count || !block_list) return SVOO_ERR_INVALID_ARG;
    if (!(tau > 0.0f) || !(tau <= 1.0f) || !(scale == scale) || !(theta == theta)) return SVOO_ERR_INVALID_ARG;
    if (shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    hipLaunchKernelGGL(block_mask_kernel, dim3(shape->kq, shape->bh), dim3(MASK_THREADS), 0, (hipStream_t)hip_stream,
                       cq, ck, counts_q, counts_k, keep, (double)tau, (double)theta, (double)scale, block_count,
                       block_list, bitmap, shape->kq, shape->kk, shape->d);
    return launch_status();
}
