// Cluster-contiguous layout: stable counting sort of labels, row gather (permute) and row
// scatter (un-permute).  Pure integer work and data movement; HBM-bandwidth bound.
//
// Sort of one slice (n tokens, K bins), three launches:
//   hist     one wave per 512-token chunk counts its labels in LDS (integer atomics) and writes a
//            K-entry histogram for the chunk
//   scan     one workgroup per slice: per bin, exclusive prefix over chunks (bin-major, chunk-minor
//            order = stable order), bin totals = cluster sizes, exclusive scan of totals = offsets
//   scatter  one wave per chunk walks its tokens 64 at a time in index order; lanes with equal
//            labels find each other with one ballot per label bit and are ranked by lane, so equal
//            labels keep ascending token order
#include "common.h"

#define SORT_CHUNK 512
#define SORT_WAVES 4

static inline int sort_chunks(int n) { return (n + SORT_CHUNK - 1) / SORT_CHUNK; }

size_t sort_scratch_ints(int bh, int n, int n_clusters) {
    return (size_t)bh * sort_chunks(n) * n_clusters;
}

__device__ __forceinline__ int clamp_label(int l, int k) { return l < 0 ? 0 : (l >= k ? k - 1 : l); }

__global__ void __launch_bounds__(SORT_WAVES* SVOO_WAVE)
sort_hist_kernel(const int32_t* __restrict__ labels, int32_t* __restrict__ chunk_hist, int n, int k, int nchunks) {
    extern __shared__ int32_t lds[];
    const int wave = threadIdx.x / SVOO_WAVE, lane = threadIdx.x % SVOO_WAVE;
    const int b = blockIdx.y;
    const int chunk = blockIdx.x * SORT_WAVES + wave;
    int32_t* hist = lds + wave * k;
    for (int j = lane; j < k; j += SVOO_WAVE) hist[j] = 0;
    __syncthreads();
    if (chunk < nchunks) {
        const int32_t* lab = labels + (size_t)b * n;
        const int start = chunk * SORT_CHUNK;
        for (int g = 0; g < SORT_CHUNK / SVOO_WAVE; ++g) {
            int i = start + g * SVOO_WAVE + lane;
            if (i < n) atomicAdd(&hist[clamp_label(lab[i], k)], 1);
        }
    }
    __syncthreads();
    if (chunk < nchunks) {
        int32_t* out = chunk_hist + ((size_t)b * nchunks + chunk) * k;
        for (int j = lane; j < k; j += SVOO_WAVE) out[j] = hist[j];
    }
}

// One workgroup of 1024 threads per slice.  The threads form G = 1024 / K' groups (K' = bins rounded
// up to a multiple of 64); group g owns a contiguous range of chunks, thread (g, j) bin j of them.
// Pass 1 totals each (group, bin); the group totals are prefixed per bin; pass 2 rewrites the chunk
// histograms as exclusive prefixes.  Then the bin totals are scanned over bins for the offsets.
__global__ void __launch_bounds__(1024)
sort_scan_kernel(int32_t* __restrict__ chunk_hist, int32_t* __restrict__ offsets, int32_t* __restrict__ counts,
                 int k, int nchunks) {
    __shared__ int32_t tot[1024];
    __shared__ int32_t scan[1024];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int kp = (k + 63) / 64 * 64;
    const int groups = 1024 / kp;            // >= 1 because k <= 1024
    const int g = tid / kp, j = tid % kp;
    const bool live = g < groups && j < k;
    const int cpg = (nchunks + groups - 1) / groups;
    const int c0 = g * cpg, c1 = (c0 + cpg < nchunks) ? c0 + cpg : nchunks;
    int32_t* h = chunk_hist + (size_t)b * nchunks * k;
    int sum = 0;
    if (live) {
#pragma unroll 8
        for (int c = c0; c < c1; ++c) sum += h[(size_t)c * k + j];
    }
    tot[tid] = live ? sum : 0;
    __syncthreads();
    int base = 0, total = 0;
    if (live) {
        for (int gg = 0; gg < groups; ++gg) {
            const int v = tot[gg * kp + j];
            base += gg < g ? v : 0;
            total += v;
        }
        int running = base;
#pragma unroll 8
        for (int c = c0; c < c1; ++c) {
            const int v = h[(size_t)c * k + j];
            h[(size_t)c * k + j] = running;
            running += v;
        }
    }
    const int mine = (live && g == 0) ? total : 0;   // bin totals, one thread per bin
    const bool owner = live && g == 0;
    // scan over bins: owners sit at tid = j < kp <= 1024
    scan[tid] = (tid < kp) ? mine : 0;
    __syncthreads();
    for (int s = 1; s < 1024; s <<= 1) {
        int v = (tid >= s) ? scan[tid - s] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    if (owner) {
        offsets[(size_t)b * (k + 1) + j] = scan[j] - total;
        if (counts) counts[(size_t)b * k + j] = total;
        if (j == k - 1) offsets[(size_t)b * (k + 1) + k] = scan[j];
    }
}

__global__ void __launch_bounds__(SORT_WAVES* SVOO_WAVE)
sort_scatter_kernel(const int32_t* __restrict__ labels, const int32_t* __restrict__ chunk_hist,
                    const int32_t* __restrict__ offsets, int32_t* __restrict__ perm, int n, int k, int nchunks) {
    extern __shared__ int32_t lds[];
    const int wave = threadIdx.x / SVOO_WAVE, lane = threadIdx.x % SVOO_WAVE;
    const int b = blockIdx.y;
    const int chunk = blockIdx.x * SORT_WAVES + wave;
    const bool active = chunk < nchunks;
    int32_t* cnt = lds + wave * k;
    if (active) {
        const int32_t* base = chunk_hist + ((size_t)b * nchunks + chunk) * k;
        const int32_t* off = offsets + (size_t)b * (k + 1);
        for (int j = lane; j < k; j += SVOO_WAVE) cnt[j] = off[j] + base[j];
    }
    __syncthreads();
    const int32_t* lab = labels + (size_t)b * n;
    int32_t* out = perm + (size_t)b * n;
    const int start = chunk * SORT_CHUNK;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    int label_bits = 0;
    while ((1 << label_bits) < k) ++label_bits;
    int mine[SORT_CHUNK / SVOO_WAVE];     // all of the lane's labels requested at once
#pragma unroll
    for (int g = 0; g < SORT_CHUNK / SVOO_WAVE; ++g) {
        const int i = start + g * SVOO_WAVE + lane;
        mine[g] = (active && i < n) ? clamp_label(lab[i], k) : -1;
    }
#pragma unroll
    for (int g = 0; g < SORT_CHUNK / SVOO_WAVE; ++g) {
        const int i = start + g * SVOO_WAVE + lane;
        const int label = mine[g];
        const bool valid = label >= 0;
        // lanes with my label: one ballot per label bit, no loop over the distinct labels
        unsigned long long same = __ballot(valid);
        for (int bit = 0; bit < label_bits; ++bit) {
            const bool set = (label >> bit) & 1;
            const unsigned long long bal = __ballot(set);
            same &= set ? bal : ~bal;
        }
        int first = 0;
        if (valid) {
            first = cnt[label];
            const int pos = first + __popcll(same & lt_mask);
            if (pos >= 0 && pos < n) out[pos] = i;     // always true for the histogram of these labels
        }
        __builtin_amdgcn_wave_barrier();
        if (valid && (same & lt_mask) == 0) cnt[label] = first + __popcll(same);   // lowest lane of each label
        __builtin_amdgcn_wave_barrier();   // cnt belongs to this wave alone: no workgroup barrier needed
    }
}

int sort_labels(int bh, int n, int k, const int32_t* labels, int32_t* perm, int32_t* offsets, int32_t* counts,
                int32_t* chunk_hist, hipStream_t stream) {
    const int nchunks = sort_chunks(n);
    dim3 grid((nchunks + SORT_WAVES - 1) / SORT_WAVES, bh);
    const size_t lds = (size_t)SORT_WAVES * k * sizeof(int32_t);
    hipLaunchKernelGGL(sort_hist_kernel, grid, dim3(SORT_WAVES * SVOO_WAVE), lds, stream, labels, chunk_hist, n, k,
                       nchunks);
    hipLaunchKernelGGL(sort_scan_kernel, dim3(bh), dim3(1024), 0, stream, chunk_hist, offsets, counts, k, nchunks);
    hipLaunchKernelGGL(sort_scatter_kernel, grid, dim3(SORT_WAVES * SVOO_WAVE), lds, stream, labels, chunk_hist,
                       offsets, perm, n, k, nchunks);
    return launch_status();
}

// ---------------------------------------------------------------------------------------------
// Row gather / scatter: every lane moves 16 bytes; a row of d elements takes row_bytes/16 lanes.
// ---------------------------------------------------------------------------------------------
struct RowPtrs {
    const uint4* src[4];
    uint4* dst[4];
};

// dst[b, p] = src[b, perm[b, p]]   (GATHER=true)    dst[b, perm[b, p]] = src[b, p]   (GATHER=false)
template <bool GATHER>
__global__ void __launch_bounds__(256)
move_rows_kernel(RowPtrs ptrs, const int32_t* __restrict__ perm, int n, int vec_per_row, int rows_per_block) {
    const int b = blockIdx.z, t = blockIdx.y;
    const int row_in_block = threadIdx.x / vec_per_row;
    const int v = threadIdx.x % vec_per_row;
    const int p = blockIdx.x * rows_per_block + row_in_block;
    if (row_in_block >= rows_per_block || p >= n) return;
    int token = perm[(size_t)b * n + p];
    token = token < 0 ? 0 : (token >= n ? n - 1 : token);   // an entry outside [0, n) must not leave the tensor
    const uint4* src = ptrs.src[t] + (size_t)b * n * vec_per_row;
    uint4* dst = ptrs.dst[t] + (size_t)b * n * vec_per_row;
    if (GATHER)
        dst[(size_t)p * vec_per_row + v] = src[(size_t)token * vec_per_row + v];
    else
        dst[(size_t)token * vec_per_row + v] = src[(size_t)p * vec_per_row + v];
}

template <bool GATHER>
static int move_rows(const svoo_shape* s, int n_tensors, const RowPtrs& ptrs, const int32_t* perm,
                     hipStream_t stream) {
    if (n_tensors == 0) return SVOO_OK;
    const int vec_per_row = s->d * elem_size(s->dtype) / 16;  // 8, 16 or 32
    const int rows_per_block = 256 / vec_per_row;
    dim3 grid((s->n + rows_per_block - 1) / rows_per_block, n_tensors, s->bh);
    hipLaunchKernelGGL(move_rows_kernel<GATHER>, grid, dim3(256), 0, stream, ptrs, perm, s->n, vec_per_row,
                       rows_per_block);
    return launch_status();
}

extern "C" int svoo_permute(const svoo_shape* shape, const int32_t* labels, int32_t n_clusters, int32_t n_tensors,
                            const void* const* src, void* const* dst, int32_t* perm, int32_t* offsets, void* ws,
                            size_t ws_bytes, void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!labels || !perm || !offsets || !ws) return SVOO_ERR_INVALID_ARG;
    if (n_clusters < 1 || n_clusters > SVOO_MAX_K) return SVOO_ERR_INVALID_ARG;
    if (n_tensors < 0 || n_tensors > 4) return SVOO_ERR_INVALID_ARG;
    if (n_tensors > 0 && (!src || !dst)) return SVOO_ERR_INVALID_ARG;
    if (shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    RowPtrs ptrs = {};
    for (int t = 0; t < n_tensors; ++t) {
        if (!src[t] || !dst[t] || !aligned16(src[t]) || !aligned16(dst[t]) || src[t] == dst[t])
            return SVOO_ERR_INVALID_ARG;
        ptrs.src[t] = (const uint4*)src[t];
        ptrs.dst[t] = (uint4*)dst[t];
    }
    if ((((uintptr_t)ws) & 255u) != 0) return SVOO_ERR_INVALID_ARG;
    const size_t need = align_up(sort_scratch_ints(shape->bh, shape->n, n_clusters) * sizeof(int32_t), 256);
    if (ws_bytes < need) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;
    st = sort_labels(shape->bh, shape->n, n_clusters, labels, perm, offsets, nullptr, (int32_t*)ws, stream);
    if (st != SVOO_OK) return st;
    return move_rows<true>(shape, n_tensors, ptrs, perm, stream);
}

extern "C" int svoo_gather(const svoo_shape* shape, const int32_t* perm, int32_t n_tensors, const void* const* src,
                           void* const* dst, void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!perm || !src || !dst || n_tensors < 1 || n_tensors > 4 || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    RowPtrs ptrs = {};
    for (int t = 0; t < n_tensors; ++t) {
        if (!src[t] || !dst[t] || !aligned16(src[t]) || !aligned16(dst[t]) || src[t] == dst[t])
            return SVOO_ERR_INVALID_ARG;
        ptrs.src[t] = (const uint4*)src[t];
        ptrs.dst[t] = (uint4*)dst[t];
    }
    return move_rows<true>(shape, n_tensors, ptrs, perm, (hipStream_t)hip_stream);
}

extern "C" int svoo_unpermute(const svoo_shape* shape, const void* src_sorted, const int32_t* perm, void* dst,
                              void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!src_sorted || !perm || !dst || src_sorted == dst) return SVOO_ERR_INVALID_ARG;
    if (!aligned16(src_sorted) || !aligned16(dst)) return SVOO_ERR_INVALID_ARG;
    if (shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    RowPtrs ptrs = {};
    ptrs.src[0] = (const uint4*)src_sorted;
    ptrs.dst[0] = (uint4*)dst;
    return move_rows<false>(shape, 1, ptrs, perm, (hipStream_t)hip_stream);
}
