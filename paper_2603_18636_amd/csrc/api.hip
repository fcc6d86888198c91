// Entry points that launch nothing: status strings, version, workspace sizing.
#include "common.h"

size_t cluster_ws_bytes(const svoo_shape* s);
size_t attn_ws_bytes(const svoo_shape* s);
size_t kmeans_ws_bytes(const svoo_shape* s, int k);
size_t mask_ws_bytes(const svoo_shape* s);

extern "C" const char* svoo_status_string(int status) {
    switch (status) {
        case SVOO_OK: return "ok";
        case SVOO_ERR_INVALID_ARG: return "invalid argument";
        case SVOO_ERR_UNSUPPORTED: return "unsupported head dimension or dtype";
        case SVOO_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SVOO_ERR_HIP: return "HIP launch failed";
        case SVOO_ERR_STATIC_LIMIT: return "shape exceeds the fixed scratch of the allocation-free entry point";
        default: return "unknown status";
    }
}

extern "C" int32_t svoo_version(void) { return 200; }

extern "C" size_t svoo_permute_workspace_bytes(const svoo_shape* shape, int32_t n_clusters) {
    if (check_shape(shape, false) != SVOO_OK || n_clusters < 1 || n_clusters > SVOO_MAX_K) return 0;
    return align_up(sort_scratch_ints(shape->bh, shape->n, n_clusters) * sizeof(int32_t), 256);
}

extern "C" size_t svoo_workspace_bytes(const svoo_shape* shape) {
    if (check_shape(shape, true) != SVOO_OK) return 0;
    size_t need = cluster_ws_bytes(shape);
    const int kmax = shape->kq > shape->kk ? shape->kq : shape->kk;
    const size_t sort_need = align_up(sort_scratch_ints(shape->bh, shape->n, kmax) * sizeof(int32_t), 256);
    if (sort_need > need) need = sort_need;
    const size_t attn_need = attn_ws_bytes(shape);
    if (attn_need > need) need = attn_need;
    const size_t km_need = kmeans_ws_bytes(shape, kmax);   // svoo_kmeans with k = kq or kk
    if (km_need > need) need = km_need;
    const size_t mask_need = mask_ws_bytes(shape);
    if (mask_need > need) need = mask_need;
    return need;
}
