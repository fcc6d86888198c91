// Block-sparse flash attention over kept (query block, key block) pairs, and the dense baseline.
//
// Work item = one tile of up to BM consecutive sorted query rows inside ONE query block r.  Its
// keys are the rows of the kept key blocks of r, treated as one logical stream (segment after
// segment), cut into tiles of KT keys; only the last tile of the stream is ragged.  Online softmax
// (running max and sum per query row) makes one pass over the stream.
//
// bf16 kernel (CDNA4 matrix cores, v_mfma_f32_32x32x16_bf16), NW waves x 32 query rows:
//   S^T = K_tile Q^T      A operand: K rows from LDS, B operand: Q, resident in registers
//   O^T += V_tile^T P^T   A operand: V^T, read from the row-major V tile with transposing LDS reads,
//                          B operand: P^T taken straight from the S^T accumulators
// Computing the transposes puts one query per lane: the softmax row reductions are in-lane plus a
// single exchange between lane l and l+32, and the probabilities are already laid out as the next
// MFMA's B operand.  The block-sparse launch uses 4 waves (128 rows: query blocks hold a few hundred
// rows, so larger tiles waste more of their last tile than they save); the dense launch uses 8 waves
// (256 rows), which halves the K/V traffic out of L2 per flop (each K/V tile is fetched once per
// workgroup).
//
// f32 kernel: 4 lanes per query row, plain float32 FMAs, same schedule and key stream.
#include <type_traits>

#include "common.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define ATT_THREADS 256
#define KT 64                 // keys per tile
#define K_PITCH 272           // bytes per K row in LDS (256 + 16 pad)
#define VT_PITCH 144          // bytes per V^T row in LDS (KT*2 + 16 pad)
#define LOG2E 1.4426950408889634f

// ---------------------------------------------------------------------------------------------
// schedule: tile_prefix[b, r] = number of query tiles of blocks < r  (kq + 1 entries per slice)
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
attn_schedule_kernel(const int32_t* __restrict__ q_offsets, int32_t* __restrict__ tile_prefix, int kq, int bm,
                     int n) {
    __shared__ int32_t scan[1024];
    const int b = blockIdx.x, r = threadIdx.x;
    int tiles = 0;
    if (r < kq) {
        int lo = q_offsets[(size_t)b * (kq + 1) + r], hi = q_offsets[(size_t)b * (kq + 1) + r + 1];
        lo = lo < 0 ? 0 : (lo > n ? n : lo);          // the same clamps as where the tile is set up
        hi = hi < 0 ? 0 : (hi > n ? n : hi);
        const int len = hi - lo;
        tiles = len > 0 ? (len + bm - 1) / bm : 0;
    }
    scan[r] = tiles;
    __syncthreads();
    for (int s = 1; s < 1024; s <<= 1) {
        const int v = r >= s ? scan[r - s] : 0;
        __syncthreads();
        scan[r] += v;
        __syncthreads();
    }
    if (r < kq) {
        tile_prefix[(size_t)b * (kq + 1) + r] = scan[r] - tiles;
        if (r == kq - 1) tile_prefix[(size_t)b * (kq + 1) + kq] = scan[r];
    }
}

// Trivial one-block clustering for the dense baseline: offsets {0, n}, one kept block.
__global__ void dense_layout_kernel(int32_t* __restrict__ offsets, int32_t* __restrict__ block_count,
                                    int32_t* __restrict__ block_list, int n, int bh) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= bh) return;
    offsets[2 * b] = 0;
    offsets[2 * b + 1] = n;
    block_count[b] = 1;
    block_list[b] = 0;
}

struct AttnArgs {
    const void* q;
    const void* k;
    const void* v;
    void* out;
    float* lse;
    const int32_t* q_offsets;
    const int32_t* k_offsets;
    const int32_t* block_count;
    const int32_t* block_list;
    const int32_t* tile_prefix;
    const int32_t* q_perm;   // nullable: q / out / lse are in token order, sorted row p is token q_perm[p]
    int n, kq, kk;
    float scale;
};

// a permutation entry outside [0, n) must not turn into an access outside the tensor
__device__ __forceinline__ int clamp_row(int r, int n) { return r < 0 ? 0 : (r >= n ? n - 1 : r); }

struct TileInfo {
    int q0, qn;    // first sorted query row of the tile, number of valid rows
    int r;         // query block
    int total;     // keys in the logical stream
    int n_seg;
};

// Which tile is this workgroup?  blockIdx.x is spread round-robin over the 8 XCDs by the
// hardware.  The REAL tiles (their number is only known on the device; the grid is sized for the
// worst case) are dealt out in 8 equal contiguous ranges, one per XCD, so that every XCD gets the
// same share and the tiles of one query block, which read the same keys, run next to each other
// on one XCD and its L2.  Returns -1 for a workgroup without work.
__device__ __forceinline__ int logical_tile_index(int total_tiles) {
    const int per_xcd = (total_tiles + 7) / 8;
    const int xcd = blockIdx.x % 8, i = blockIdx.x / 8;
    const int slot = xcd * per_xcd + i;
    return (i < per_xcd && slot < total_tiles) ? slot : -1;
}

// Fills seg_start / seg_cum in LDS and returns the tile description; false if there is no work.
// seg_cum has n_seg + 1 entries (exclusive prefix of segment lengths); scan is NT ints of scratch.
template <int NT>
__device__ __forceinline__ bool setup_tile(const AttnArgs& a, int bm, int32_t* seg_start, int32_t* seg_cum,
                                           int32_t* scan, TileInfo& ti) {
    constexpr int SPT = SVOO_MAX_K / NT;   // consecutive segments owned by one thread
    const int b = blockIdx.y, tid = threadIdx.x;
    const int32_t* tp = a.tile_prefix + (size_t)b * (a.kq + 1);
    const int slot = logical_tile_index(tp[a.kq]);
    if (slot < 0) return false;
    int lo = 0, hi = a.kq;  // last r with tp[r] <= slot
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tp[mid] <= slot) lo = mid; else hi = mid;
    }
    // skip empty query blocks that share the same prefix value: take the last r with tp[r] <= slot
    const int r = lo;
    const int32_t* qo = a.q_offsets + (size_t)b * (a.kq + 1);
    const int t = slot - tp[r];
    ti.r = r;
    // offsets come from the caller: whatever they hold, rows stay inside [0, n)
    const long long q0l = (long long)qo[r] + (long long)t * bm;
    const int q0 = q0l < 0 ? 0 : (q0l >= a.n ? a.n - 1 : (int)q0l);
    int q1 = qo[r + 1];
    q1 = q1 < 0 ? 0 : (q1 > a.n ? a.n : q1);
    ti.q0 = q0;
    const int rem = q1 - q0;
    ti.qn = rem < bm ? (rem < 0 ? 0 : rem) : bm;
    int cnt = a.block_count[(size_t)b * a.kq + r];
    cnt = cnt < 0 ? 0 : (cnt > a.kk ? a.kk : cnt);
    const int32_t* bl = a.block_list + ((size_t)b * a.kq + r) * a.kk;
    const int32_t* ko = a.k_offsets + (size_t)b * (a.kk + 1);
    int len[SPT], start[SPT], local = 0;
#pragma unroll
    for (int u = 0; u < SPT; ++u) {
        const int i = tid * SPT + u;
        len[u] = 0;
        start[u] = 0;
        if (i < cnt) {
            int j = bl[i];
            j = j < 0 ? 0 : (j >= a.kk ? a.kk - 1 : j);
            int s0 = ko[j], s1 = ko[j + 1];
            s0 = s0 < 0 ? 0 : (s0 > a.n ? a.n : s0);
            s1 = s1 > a.n ? a.n : s1;
            start[u] = s0;
            len[u] = s1 > s0 ? s1 - s0 : 0;
        }
        local += len[u];
    }
    // Prefix sums that saturate at n: distinct key blocks never hold more than n keys, so nothing changes
    // for a valid block list; a list with repeated or overlapping blocks cannot overflow the sums or make
    // them decrease, which is what the walk along the stream relies on to end.
    const int cap = a.n;
    local = local < cap ? local : cap;
    scan[tid] = local;
    __syncthreads();
    for (int s = 1; s < NT; s <<= 1) {
        const int v = tid >= s ? scan[tid - s] : 0;
        __syncthreads();
        const int t = scan[tid] + v;
        scan[tid] = t < cap ? t : cap;
        __syncthreads();
    }
    int run = tid > 0 ? scan[tid - 1] : 0;
#pragma unroll
    for (int u = 0; u < SPT; ++u) {
        const int i = tid * SPT + u;
        if (i < cnt) {
            seg_start[i] = start[u];
            seg_cum[i] = run;
        }
        run += len[u];
        run = run < cap ? run : cap;
    }
    ti.total = scan[NT - 1];
    ti.n_seg = cnt;
    if (tid == 0) seg_cum[cnt] = ti.total;
    __syncthreads();
    return true;
}

// Sorted key row of logical stream position p (p < total): last segment s with seg_cum[s] <= p.
__device__ __forceinline__ int stream_row(const int32_t* seg_start, const int32_t* seg_cum, int n_seg, int p) {
    int lo = 0, hi = n_seg;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (seg_cum[mid] <= p) lo = mid; else hi = mid;
    }
    return seg_start[lo] + (p - seg_cum[lo]);
}

// ---------------------------------------------------------------------------------------------
// bf16 matrix-core kernel, head dimension D (64 or 128), BM = 32 NW query rows per workgroup
//
// LDS: K and V tiles of 64 keys, row-major [key][D], NBUF buffers of each, filled by direct
// global->LDS 16-byte loads (no register staging).  A wave-load writes 1 KB = lane-consecutive
// 16-byte slots, so the 16-byte chunk c of tile row r is fetched by the lane whose slot is
// c ^ swizzle(r): an XOR swizzle (by row for K, by row on 32-byte granules for V) that makes both
// kinds of reads below conflict-free.
//   K operand: ds_read_b128, lane (j, h) reads row 32 kb + j, chunk 2 c + h.
//   V operand: ds_read_b64_tr_b16 (transposing read): within a 16-lane block the lane s points at
//              4 consecutive d-columns of key row (s / 4); the lane i receives, for d-column i of
//              the block, the 4 keys -- exactly the layout of the MFMA A operand of V^T.
// The S^T accumulator of lane (j, h) holds, for query j, the keys 32 kb + 8 (v/4) + 4 h + v%4,
// so 8 consecutive accumulators (v = 8t .. 8t+7) are two runs of 4 consecutive keys, which is
// what two transposing reads deliver.
// ---------------------------------------------------------------------------------------------
// Kernel shape: NW waves of 32 query rows, NBUF K/V tile buffers in LDS (measured on MI355X at
// 12 x 75,600 x 128):
//   dense baseline : 8 waves x 3 buffers, one workgroup per CU.  256 rows per workgroup halve the
//                    K/V traffic out of L2 per flop; a 4th buffer does not help.
//   block-sparse   : 4 waves x 2 buffers, two workgroups per CU.  Query blocks are a few hundred
//                    rows, so 128-row tiles waste fewer rows in the last tile of a block than 256.
#define SVOO_SPARSE_NW 4
#define SVOO_SPARSE_NBUF 2
#define DENSE_NW 8
#define DENSE_NBUF 3
#define RESCALE_LOG2 8.0f   // the running max is only raised when it is exceeded by 2^8

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
    f32x2 x = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

template <int D, int NBUF>
struct AttnLds {
    static constexpr int ROWB = D * 2;            // bytes per K/V row
    static constexpr int TILE = KT * ROWB;        // bytes per tile
    static constexpr int SEG_BYTES = (2 * SVOO_MAX_K + 8) * 4;
    static constexpr int BYTES = SEG_BYTES + 2 * NBUF * TILE;   // seg tables + NBUF x (K tile + V tile)
};

template <int D, int NW, int NBUF>
__global__ void __launch_bounds__(64 * NW, 8 / NW)
sparse_attn_bf16_kernel(AttnArgs a) {
    constexpr int NT = 64 * NW, BM = 32 * NW;
    constexpr int DC = D / 16;        // 16-wide contraction chunks of QK^T
    constexpr int DB = D / 32;        // 32-row blocks of O^T
    constexpr int CPR = D / 8;        // 16-byte chunks per row
    constexpr int ROWB = AttnLds<D, NBUF>::ROWB;
    constexpr int TILE = AttnLds<D, NBUF>::TILE;
    constexpr int RPL = 64 / CPR;     // tile rows covered by one wave-load (1 KB)
    constexpr int RW = KT / NW;       // tile rows owned by one wave
    constexpr int LPW = RW / RPL;     // wave-loads per wave per tile and tensor
    static_assert(LPW >= 1 && RW <= 16 && NBUF >= 2 && NBUF <= 4, "wave-load geometry");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    unsigned char* k_lds = smem;                     // [NBUF][TILE]
    unsigned char* v_lds = smem + NBUF * TILE;       // [NBUF][TILE]
    int32_t* seg_start = (int32_t*)(smem + 2 * NBUF * TILE);
    int32_t* seg_cum = seg_start + SVOO_MAX_K;
    int32_t* scan = (int32_t*)smem;               // setup scratch, aliases the K tiles

    TileInfo ti;
    if (!setup_tile<NT>(a, BM, seg_start, seg_cum, scan, ti)) return;
    const int b = blockIdx.y, tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);    // uniform: keeps everything derived from it scalar
    const int lane = tid % 64, j = lane % 32, h = lane / 32;
    const uint16_t* qg = (const uint16_t*)a.q + (size_t)b * a.n * D;
    const unsigned char* kg = (const unsigned char*)a.k + (size_t)b * a.n * ROWB;
    const unsigned char* vg = (const unsigned char*)a.v + (size_t)b * a.n * ROWB;
    const int total = ti.total;
    const int n_tiles = (total + KT - 1) / KT;

    // V swizzle (in 16-byte chunk units): one transposing read touches, per half wave, 4 key rows x
    // 2 adjacent 32-byte column segments; XOR-ing the 64-byte granule index with the row spreads
    // those 8 segments over all banks (K keeps the 16-byte swizzle by row).
    auto vswz = [](int rho) { return ((rho / (256 / ROWB)) % (ROWB / 64)) << 2; };
    // ---- key-stream walk: this lane tracks tile row RW*wave + lane%RW from tile to tile
    int seg = 0, seg_end = 0, seg_delta = 0;
    if (total > 0) {
        seg_end = seg_cum[1];
        seg_delta = seg_start[0] - seg_cum[0];
    }
    // The key rows of a tile are looked up (segment walk through LDS tables, then a lane exchange)
    // one tile ahead of their use, while matrix instructions of the current tile are in flight, so
    // that issuing the loads right after the barrier costs address arithmetic only.
    int next_rows[LPW];
    auto prepare_tile = [&](int t) {          // call with t = 0, 1, 2, ... in order
        int p = t * KT + RW * wave + (lane % RW);
        p = p < total ? p : total - 1;        // rows past the end re-read the last key (masked later)
        while (p >= seg_end) {                // terminates: p < total = seg_cum[n_seg]
            ++seg;
            seg_end = seg_cum[seg + 1];
            seg_delta = seg_start[seg] - seg_cum[seg];
        }
        const int myrow = p + seg_delta;
#pragma unroll
        for (int i = 0; i < LPW; ++i) next_rows[i] = __shfl(myrow, i * RPL + lane / CPR);
    };
    // Tile row rho = RW wave + i RPL + lane / CPR is fetched by this lane's i-th wave-load; the three terms
    // occupy disjoint bits, so the swizzled 16-byte chunk of load i is that of load 0 XOR a constant
    // (K) or the same (V: its swizzle only looks at row bits below RPL).  The loads take the slice's
    // base address as a scalar and a 32-bit byte offset per lane: one shift-add per load, no 64-bit
    // address arithmetic in vector registers.
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    const uint32_t kx0 = (uint32_t)(((lane % CPR) ^ ((RW * wave + lane / CPR) % CPR)) * 16);
    const uint32_t vx0 = (uint32_t)(((lane % CPR) ^ vswz(RW * wave + lane / CPR)) * 16);
    auto issue_prepared = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const uint32_t row_off = (uint32_t)next_rows[i] * ROWB;      // < 2^32: n <= 2^24 rows of at most 256 bytes
            const uint32_t koffs = row_off + (kx0 ^ (uint32_t)(((i * RPL) % CPR) * 16));
            const uint32_t voffs = row_off + vx0;
            const uint32_t loff = lds0 + buf * TILE + (RW * wave + i * RPL) * ROWB;
            load_rows_to_lds_16(koffs, kg, loff);
            load_rows_to_lds_16(voffs, vg, loff + NBUF * TILE);
        }
    };

    // ---- which rows / which keys this wave works on.
    // Normal tile: wave w owns rows 32w .. 32w+31 and every key.  Tile with at most half the rows
    // (the last tile of a query block, often): the waves split the KEYS instead -- wave group g
    // takes the (g % 2)-th 32-key block of every tile for rows 32 (w % row_waves) .., and the
    // partial results are merged at the end -- so that a short tile costs about half the time, not
    // all of it.  With 4 waves and at most 32 rows there are four groups: groups 0, 1 take the two
    // blocks of the even tiles, groups 2, 3 those of the odd tiles.
    const int kgroups = (NW >= 4 && ti.qn <= BM / 2) ? ((NW == 4 && ti.qn <= BM / 4) ? 4 : 2) : 1;
    const bool split = kgroups > 1;
    const int row_waves = NW / kgroups;
    const int kgrp = wave / row_waves;
    const int rwave = wave % row_waves;
    const bool alternate = kgroups == 4;     // this wave computes every other tile only
    const int parity = kgrp / 2;
    // ---- Q fragments: query row (rwave, j), contraction elements 16c + 8h .. +7
    const int qrow = 32 * rwave + j;
    const bool qvalid = qrow < ti.qn;
    const bool wave_active = 32 * rwave < ti.qn;
    bf16x8 qf[DC];
    {
        int qtok = ti.q0 + (qvalid ? qrow : 0);
        if (a.q_perm) qtok = clamp_row(a.q_perm[(size_t)b * a.n + qtok], a.n);
        const uint4* src = (const uint4*)(qg + (size_t)qtok * D);
#pragma unroll
        for (int c = 0; c < DC; ++c) {
            uint4 u = qvalid ? src[2 * c + h] : make_uint4(0, 0, 0, 0);
            qf[c] = __builtin_bit_cast(bf16x8, u);
        }
    }
    // ---- per-lane LDS read offsets (bytes inside a tile; kb, t and buffer add constants)
    int koff[DC];            // K: row j, chunk (2c + h) ^ (j % CPR)
#pragma unroll
    for (int c = 0; c < DC; ++c) koff[c] = j * ROWB + (((2 * c + h) ^ (j % CPR)) * 16);
    int voff[2][DB];         // V: transposing read u of block db
    {
        const int s = lane % 16, blk = lane / 16;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const int rho = 8 * u + 4 * (blk / 2) + s / 4;            // + 32 kb + 16 t
                const int chunk = 4 * db + 2 * (blk % 2) + (s % 4) / 2;
                voff[u][db] = rho * ROWB + ((chunk ^ vswz(rho)) * 16) + (s % 2) * 8;
            }
    }

    // key-split waves read "their" 32-key block of every tile: fold its offset into the addresses.
    // The offsets are turned into absolute LDS byte addresses here, once, so that inside the loop a
    // read is "address register + immediate" with nothing left to add.
    const int kb_off = 32 * (kgrp % 2);
    const int k_base = (int)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)k_lds;
    const int v_base = (int)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)v_lds;
#pragma unroll
    for (int c = 0; c < DC; ++c) {
        koff[c] += kb_off * ROWB + k_base;
        asm volatile("" : "+v"(koff[c]));  // keep the sum in the register: no re-adding per tile
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            voff[u][db] += kb_off * ROWB + v_base;
            asm volatile("" : "+v"(voff[u][db]));
        }

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    const float c2 = a.scale * LOG2E;
    const float th_raw = RESCALE_LOG2 / c2;
    float m_used = -INFINITY;   // reference max (raw logits) the probabilities are scaled by
    float lsum = 0.f;           // this lane's share of the row sum

    // One tile (64 keys) out of LDS buffer BUF; MODE 0 = both 32-key blocks, 1 = one block (the
    // key-split wave's own block, whose offset is already folded into the read addresses).  LDS reads are issued in batches ahead of the matrix
    // instructions that consume them (the LDS latency is ~100 cycles, one MFMA is 32):
    //   S phase   K fragments in batches of DC/2, two batches in flight
    //   softmax   V fragments of the first block are fetched while S finishes
    //   PV phase  first block's MFMAs run while the second block's V fragments arrive and its
    //             exponentials are computed
    auto tile_body = [&](auto bufc, auto modec, int kt) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int MODE = decltype(modec)::value;
        constexpr int KB0 = 0;
        constexpr int NKB = MODE == 0 ? 2 : 1;       // number of blocks
        constexpr int HB = DC / 2;
        auto kfrag = [&](int kb, int c) {
            const uint32_t addr = (uint32_t)(koff[c] + BUF * TILE + kb * 32 * ROWB);
            return __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) uint4*)(uintptr_t)addr);
        };
        auto vfrag = [&](int kb, int t, int db) {
            const int cst = BUF * TILE + (32 * kb + 16 * t) * ROWB;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                (__attribute__((address_space(3))) bf16x4*)(uintptr_t)(uint32_t)(voff[0][db] + cst));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                (__attribute__((address_space(3))) bf16x4*)(uintptr_t)(uint32_t)(voff[1][db] + cst));
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        };
        f32x16 s[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
        bf16x8 fa[HB], fb[HB];
        bf16x8 vf[2][DB];
#pragma unroll
        for (int c = 0; c < HB; ++c) fa[c] = kfrag(KB0, c);
#pragma unroll
        for (int c = 0; c < HB; ++c) fb[c] = kfrag(KB0, HB + c);
        if (NKB == 2) {
#pragma unroll
            for (int c = 0; c < HB; ++c) {
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c], qf[c], s[0], 0, 0, 0);
                fa[c] = kfrag(1, c);
            }
#pragma unroll
            for (int c = 0; c < HB; ++c) {
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c], qf[HB + c], s[0], 0, 0, 0);
                fb[c] = kfrag(1, HB + c);
            }
        }
        // V fragments of the first block start arriving while the last block of S is computed
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < DB; ++db) vf[t][db] = vfrag(KB0, t, db);
#pragma unroll
        for (int c = 0; c < HB; ++c)
            s[NKB - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c], qf[c], s[NKB - 1], 0, 0, 0);
#pragma unroll
        for (int c = 0; c < HB; ++c)
            s[NKB - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c], qf[HB + c], s[NKB - 1], 0, 0, 0);
        // scheduling pipeline of this block: 2 batches of K reads, then every MFMA paired with the
        // LDS read(s) that refill its operand registers / prefetch V
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * HB, 0);
        if (NKB == 2) {
#pragma unroll
            for (int i = 0; i < 2 * HB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 2 * HB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (2 * 2 * DB) / (2 * HB), 0);
        }
        // ragged last tile: keys past the end of the stream get -inf
        if (kt == n_tiles - 1 && (total % KT) != 0) {
            const int base = kt * KT + 4 * h;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (base + kb_off + 32 * kb + 8 * (v / 4) + (v % 4) >= total) s[kb][v] = -INFINITY;
        }
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
        {
            const int mi = __float_as_int(mx);
            auto r = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
            mx = fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
        }
        if (__any(mx > m_used + th_raw)) {
            const float m_new = fmaxf(m_used, mx);
            const float alpha = __builtin_amdgcn_exp2f((m_used - m_new) * c2);   // 0 on the first tile
            m_used = m_new;
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        }
        // a key-split wave may have seen only masked keys so far (-inf reference): keep exp2 finite
        const float mb = (MODE != 0 && m_used == -INFINITY) ? 0.f : m_used * c2;
        const bf16x2 ones2 = __builtin_bit_cast(bf16x2, 0x3f803f80u);
        auto probs = [&](int kb, int t) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * t + 2 * e], c2, -mb));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * t + 2 * e + 1], c2, -mb));
                w[e] = pack2_bf16(p0, p1);
                // the row sum takes the two ROUNDED probabilities, the same values the second
                // contraction multiplies: one dot-product instruction with (1, 1) instead of two adds
                lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e]), ones2, lsum, false);
            }
            return __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
        };
        // ---- O^T += V^T P^T, block by block
        bf16x8 pf[2];
        pf[0] = probs(0, 0);
        pf[1] = probs(0, 1);
        if (NKB == 2) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][db], pf[t], o[db], 0, 0, 0);
                    vf[t][db] = vfrag(1, t, db);
                }
            pf[0] = probs(1, 0);
            pf[1] = probs(1, 1);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < DB; ++db)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][db], pf[t], o[db], 0, 0, 0);
        constexpr int PVALU = 48;   // VALU/transcendental instructions of one 32-key block's probabilities
        // pipeline: exponentials of the first block, then (two-block tiles) each MFMA of block 0
        // paired with two V reads of block 1 and a slice of block 1's exponentials, then the rest
        __builtin_amdgcn_sched_group_barrier(0x402, PVALU, 0);
        if (NKB == 2) {
#pragma unroll
            for (int i = 0; i < 2 * DB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x402, PVALU / (2 * DB), 0);
            }
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * DB, 0);
    };

    // Have the Q fragments arrive here: otherwise the compiler's wait for them sits inside the tile
    // loop as "wait for every outstanding load" and is paid again on every tile, against the prefetch.
#pragma unroll
    for (int c = 0; c < DC; ++c) asm volatile("" ::"v"(qf[c]));
    // Prefetch distance NBUF-1 tiles.  Loads complete in order, so "all but the newest tiles'
    // loads" is a constant outstanding-load count while tiles are still being issued.
    for (int t = 0; t < NBUF - 1 && t < n_tiles; ++t) {
        prepare_tile(t);
        issue_prepared(t);
    }
    if (NBUF - 1 < n_tiles) prepare_tile(NBUF - 1);
    auto run_tiles = [&](auto modec) {
        auto step = [&](auto bufc, int kt) {
            constexpr int BUF = decltype(bufc)::value;
            // tiles kt+1 .. kt+NBUF-2 (those that exist) may stay in flight; loads complete in order
            const int ahead = n_tiles - 1 - kt < NBUF - 2 ? n_tiles - 1 - kt : NBUF - 2;
            if (NBUF >= 4 && ahead == 2)
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * 2 * LPW) : "memory");
            else if (NBUF >= 3 && ahead == 1)
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPW) : "memory");
            else
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();    // tile kt has landed for every wave; everyone is done with tile kt-1's buffer
            if (kt + NBUF - 1 < n_tiles) issue_prepared((BUF + NBUF - 1) % NBUF);
            if (wave_active && (!alternate || (kt & 1) == parity)) tile_body(bufc, modec, kt);
            if (kt + NBUF < n_tiles) prepare_tile(kt + NBUF);
        };
        for (int kt = 0; kt < n_tiles; kt += NBUF) {
            step(std::integral_constant<int, 0>{}, kt);
            if (kt + 1 < n_tiles) step(std::integral_constant<int, 1>{}, kt + 1);
            if (NBUF > 2 && kt + 2 < n_tiles) step(std::integral_constant<int, 2 % NBUF>{}, kt + 2);
            if (NBUF > 3 && kt + 3 < n_tiles) step(std::integral_constant<int, 3 % NBUF>{}, kt + 3);
        }
    };
    if (split)
        run_tiles(std::integral_constant<int, 1>{});
    else
        run_tiles(std::integral_constant<int, 0>{});

    // ---- epilogue: (merge key-split partials,) normalise, transpose through LDS, store whole rows.
    // Lane (j, h) holds O[q = j][d = 32 db + 8 (v/4) + 4 h + v%4].
    float ltot;
    {
        const int li = __float_as_int(lsum);
        auto r = __builtin_amdgcn_permlane32_swap(li, li, false, false);
        ltot = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    __syncthreads();   // all waves are done with the K/V tiles
    if (split) {
        // groups 1.. park (O, m, l) in LDS; group 0 folds them into its own partial result
        constexpr int PARK = (16 * DB + 2) * 64;
        static_assert((NW == 4 ? 3 : NW / 2) * PARK * 4 <= AttnLds<D, NBUF>::BYTES, "parked partials exceed the LDS");
        if (kgrp > 0 && wave_active) {
            float* park = (float*)smem + ((kgrp - 1) * row_waves + rwave) * PARK;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) park[(16 * db + v) * 64 + lane] = o[db][v];
            park[(16 * DB) * 64 + lane] = m_used;
            park[(16 * DB + 1) * 64 + lane] = ltot;
        }
        __syncthreads();
        if (kgrp == 0 && wave_active) {
            for (int g = 1; g < kgroups; ++g) {
                const float* park = (const float*)smem + ((g - 1) * row_waves + rwave) * PARK;
                const float m_b = park[(16 * DB) * 64 + lane], l_b = park[(16 * DB + 1) * 64 + lane];
                const float m_new = fmaxf(m_used, m_b);
                const float sa = m_used == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_used - m_new) * c2);
                const float sb = m_b == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_b - m_new) * c2);
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[db][v] = o[db][v] * sa + park[(16 * db + v) * 64 + lane] * sb;
                ltot = ltot * sa + l_b * sb;
                m_used = m_new;
            }
        }
        __syncthreads();   // the staging below reuses the same LDS
    }
    const bool writer = wave_active && kgrp == 0;
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    unsigned char* stage = smem + wave * (32 * ROWB);      // 32 rows x ROWB per wave, inside the K buffers
    if (writer) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                w.x = pack2_bf16(o[db][4 * g] * inv, o[db][4 * g + 1] * inv);
                w.y = pack2_bf16(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
                const int chunk = 4 * db + g;                  // 16-byte chunk holding d = 32 db + 8 g ..
                *(uint2*)(stage + j * ROWB + ((chunk ^ (j % CPR)) * 16) + 8 * h) = w;
            }
        __builtin_amdgcn_wave_barrier();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        unsigned char* og = (unsigned char*)a.out + (size_t)b * a.n * ROWB;
        const int row0 = ti.q0 + 32 * rwave;               // first sorted row of this wave
        const int rows_here = ti.qn - 32 * rwave;          // valid rows of this wave
        const int32_t* pm = a.q_perm ? a.q_perm + (size_t)b * a.n : nullptr;
#pragma unroll
        for (int i = 0; i < (32 * CPR) / 64; ++i) {
            const int e = i * 64 + lane;
            const int r = e / CPR, c = e % CPR;
            if (r < rows_here) {
                const uint4 val = *(const uint4*)(stage + r * ROWB + ((c ^ (r % CPR)) * 16));
                const int dst = pm ? clamp_row(pm[row0 + r], a.n) : row0 + r;
                *(uint4*)(og + (size_t)dst * ROWB + c * 16) = val;
            }
        }
        if (a.lse && qvalid && h == 0) {
            const int dst = pm ? clamp_row(pm[ti.q0 + qrow], a.n) : ti.q0 + qrow;
            a.lse[(size_t)b * a.n + dst] =
                ltot > 0.f ? (m_used * c2 + log2f(ltot)) * 0.6931471805599453f : -INFINITY;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// float32 kernel: 64 query rows per workgroup, 4 lanes per row, each lane owns D/4 columns
// (interleaved in groups of 4: lane part p owns columns 16 c + 4 p .. +3), keys staged 32 at a time
// ---------------------------------------------------------------------------------------------
#define BM_F32 64
#define KT_F32 32

template <int D>
__global__ void __launch_bounds__(ATT_THREADS)
sparse_attn_f32_kernel(AttnArgs a) {
    constexpr int NC = D / 16;  // float4 chunks per lane
    __shared__ int32_t seg_start[SVOO_MAX_K];
    __shared__ int32_t seg_cum[SVOO_MAX_K + 1];
    __shared__ int32_t scan[ATT_THREADS];
    __shared__ int32_t rowidx[KT_F32];
    __shared__ float4 k_lds[KT_F32 * D / 4];
    __shared__ float4 v_lds[KT_F32 * D / 4];

    TileInfo ti;
    if (!setup_tile<ATT_THREADS>(a, BM_F32, seg_start, seg_cum, scan, ti)) return;
    const int b = blockIdx.y, tid = threadIdx.x;
    const int qrow = tid / 4, part = tid % 4;
    const bool qvalid = qrow < ti.qn;
    const float4* qg = (const float4*)a.q + (size_t)b * a.n * (D / 4);
    const float4* kg = (const float4*)a.k + (size_t)b * a.n * (D / 4);
    const float4* vg = (const float4*)a.v + (size_t)b * a.n * (D / 4);
    float4 qv[NC], ov[NC];
    int qtok = ti.q0 + (qvalid ? qrow : 0);     // token whose row this is: gathered / scattered through q_perm
    if (a.q_perm) qtok = clamp_row(a.q_perm[(size_t)b * a.n + qtok], a.n);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        qv[c] = qvalid ? qg[(size_t)qtok * (D / 4) + 4 * c + part] : make_float4(0, 0, 0, 0);
        ov[c] = make_float4(0, 0, 0, 0);
    }
    float m = -INFINITY, lsum = 0.f;
    const int n_tiles = (ti.total + KT_F32 - 1) / KT_F32;
    for (int kt = 0; kt < n_tiles; ++kt) {
        __syncthreads();
        if (tid < KT_F32) {
            const int p = kt * KT_F32 + tid;
            rowidx[tid] = p < ti.total ? stream_row(seg_start, seg_cum, ti.n_seg, p) : -1;
        }
        __syncthreads();
        for (int e = tid; e < KT_F32 * D / 4; e += ATT_THREADS) {
            const int row = e / (D / 4), col = e % (D / 4);
            const int g = rowidx[row];
            k_lds[e] = g >= 0 ? kg[(size_t)g * (D / 4) + col] : make_float4(0, 0, 0, 0);
            v_lds[e] = g >= 0 ? vg[(size_t)g * (D / 4) + col] : make_float4(0, 0, 0, 0);
        }
        __syncthreads();
        const int valid = ti.total - kt * KT_F32 < KT_F32 ? ti.total - kt * KT_F32 : KT_F32;
        float sc[KT_F32];
        float mx = -INFINITY;
#pragma unroll
        for (int key = 0; key < KT_F32; ++key) {
            float s = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 kv = k_lds[key * (D / 4) + 4 * c + part];
                s = fmaf(qv[c].x, kv.x, s);
                s = fmaf(qv[c].y, kv.y, s);
                s = fmaf(qv[c].z, kv.z, s);
                s = fmaf(qv[c].w, kv.w, s);
            }
            s += __shfl_xor(s, 1);
            s += __shfl_xor(s, 2);
            s = key < valid ? s * a.scale : -INFINITY;
            sc[key] = s;
            mx = fmaxf(mx, s);
        }
        const float m_new = fmaxf(m, mx);
        const float alpha = expf(m - m_new);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            ov[c].x *= alpha;
            ov[c].y *= alpha;
            ov[c].z *= alpha;
            ov[c].w *= alpha;
        }
#pragma unroll
        for (int key = 0; key < KT_F32; ++key) {
            const float p = expf(sc[key] - m_new);
            lsum += p;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 vv = v_lds[key * (D / 4) + 4 * c + part];
                ov[c].x = fmaf(p, vv.x, ov[c].x);
                ov[c].y = fmaf(p, vv.y, ov[c].y);
                ov[c].z = fmaf(p, vv.z, ov[c].z);
                ov[c].w = fmaf(p, vv.w, ov[c].w);
            }
        }
    }
    if (qvalid) {
        const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
        float4* og = (float4*)a.out + ((size_t)b * a.n + qtok) * (D / 4);
#pragma unroll
        for (int c = 0; c < NC; ++c)
            og[4 * c + part] = make_float4(ov[c].x * inv, ov[c].y * inv, ov[c].z * inv, ov[c].w * inv);
        if (a.lse && part == 0) a.lse[(size_t)b * a.n + qtok] = lsum > 0.f ? m + logf(lsum) : -INFINITY;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
size_t attn_ws_bytes(const svoo_shape* s) {
    // tile_prefix for the sparse call; the dense call adds a 1-block layout
    const size_t kq = s->kq > 1 ? s->kq : 1;
    return align_up((size_t)s->bh * (kq + 1) * 4, 256) + 3 * align_up((size_t)s->bh * 2 * 4, 256);
}

template <int D, int NW, int NBUF>
static int launch_bf16(dim3 grid, const AttnArgs& a, hipStream_t stream) {
    auto kern = sparse_attn_bf16_kernel<D, NW, NBUF>;
    constexpr int lds_bytes = AttnLds<D, NBUF>::BYTES;
    static unsigned char opted_in[SVOO_MAX_DEVICES];
    if (!opt_in_dynamic_lds((const void*)kern, lds_bytes, opted_in)) return SVOO_ERR_HIP;
    hipLaunchKernelGGL(kern, grid, dim3(64 * NW), lds_bytes, stream, a);
    return SVOO_OK;
}

// dense = one-block layout: every workgroup reads the same key stream
static int launch_sparse(const svoo_shape* s, AttnArgs& a, int32_t* tile_prefix, bool dense, hipStream_t stream) {
    const int bm = s->dtype == SVOO_BF16 ? 32 * (dense ? DENSE_NW : SVOO_SPARSE_NW) : BM_F32;
    hipLaunchKernelGGL(attn_schedule_kernel, dim3(s->bh), dim3(1024), 0, stream, a.q_offsets, tile_prefix, a.kq, bm,
                       s->n);
    a.tile_prefix = tile_prefix;
    int gx = (s->n + bm - 1) / bm + a.kq;
    gx = (gx + 7) / 8 * 8;
    dim3 grid(gx, s->bh);
    int st = SVOO_OK;
    if (s->dtype == SVOO_BF16) {
        if (s->d == 128)
            st = dense ? launch_bf16<128, DENSE_NW, DENSE_NBUF>(grid, a, stream)
                       : launch_bf16<128, SVOO_SPARSE_NW, SVOO_SPARSE_NBUF>(grid, a, stream);
        else
            st = dense ? launch_bf16<64, DENSE_NW, DENSE_NBUF>(grid, a, stream)
                       : launch_bf16<64, SVOO_SPARSE_NW, SVOO_SPARSE_NBUF>(grid, a, stream);
        if (st != SVOO_OK) return st;
    } else {
        if (s->d == 128)
            hipLaunchKernelGGL(sparse_attn_f32_kernel<128>, grid, dim3(ATT_THREADS), 0, stream, a);
        else
            hipLaunchKernelGGL(sparse_attn_f32_kernel<64>, grid, dim3(ATT_THREADS), 0, stream, a);
    }
    return launch_status();
}

static int sparse_attn_entry(const svoo_shape* shape, const void* q_sorted, const void* k_sorted,
                             const void* v_sorted, const int32_t* q_perm, const int32_t* q_offsets,
                             const int32_t* k_offsets, const int32_t* block_count, const int32_t* block_list,
                             float scale, void* out_sorted, float* lse, void* ws, size_t ws_bytes, void* hip_stream) {
    int st = check_shape(shape, true);
    if (st != SVOO_OK) return st;
    if (!q_sorted || !k_sorted || !v_sorted || !q_offsets || !k_offsets || !block_count || !block_list ||
        !out_sorted || !ws)
        return SVOO_ERR_INVALID_ARG;
    if (!aligned16(q_sorted) || !aligned16(k_sorted) || !aligned16(v_sorted) || !aligned16(out_sorted) ||
        (((uintptr_t)ws) & 255u) != 0)
        return SVOO_ERR_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < 1e30f) || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    if (ws_bytes < attn_ws_bytes(shape)) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    AttnArgs a = {q_sorted, k_sorted, v_sorted, out_sorted, lse, q_offsets, k_offsets, block_count, block_list,
                  nullptr, q_perm, shape->n, shape->kq, shape->kk, scale};
    return launch_sparse(shape, a, (int32_t*)ws, false, (hipStream_t)hip_stream);
}

extern "C" int svoo_block_sparse_attn(const svoo_shape* shape, const void* q_sorted, const void* k_sorted,
                                      const void* v_sorted, const int32_t* q_offsets, const int32_t* k_offsets,
                                      const int32_t* block_count, const int32_t* block_list, float scale,
                                      void* out_sorted, float* lse, void* ws, size_t ws_bytes, void* hip_stream) {
    return sparse_attn_entry(shape, q_sorted, k_sorted, v_sorted, nullptr, q_offsets, k_offsets, block_count,
                             block_list, scale, out_sorted, lse, ws, ws_bytes, hip_stream);
}

// ---------------------------------------------------------------------------------------------
// The same call for callers that cannot allocate or hand over a workspace (code under HIP graph
// capture, tight serving loops): the query-tile schedule, the only scratch the attention needs,
// lives in a file-scope device array.  In host code the array's NAME is a stand-in, not a device
// address: its address on the current device comes from hipGetSymbolAddress, once per device, and
// only that pointer is ever handed to a kernel.
// ---------------------------------------------------------------------------------------------
#define STATIC_SCRATCH_INTS (256 * 1024)     // 1 MiB per GPU: room for bh * (kq + 1) <= 262,144 schedule entries
static __device__ __align__(256) int32_t scratch[STATIC_SCRATCH_INTS];
static int32_t* scratch_ptr[SVOO_MAX_DEVICES];   // device address of `scratch`, per device ordinal

static int32_t* static_scratch_on_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SVOO_MAX_DEVICES) return nullptr;
    int32_t* p = __atomic_load_n(&scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        void* sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return nullptr;
        p = (int32_t*)sym;
        __atomic_store_n(&scratch_ptr[dev], p, __ATOMIC_RELEASE);   // two racing first calls store the same address
    }
    return p;
}

extern "C" int svoo_block_sparse_attn_static(const svoo_shape* shape, const void* q_sorted, const void* k_sorted,
                                             const void* v_sorted, const int32_t* q_offsets,
                                             const int32_t* k_offsets, const int32_t* block_count,
                                             const int32_t* block_list, float scale, void* out_sorted, float* lse,
                                             void* hip_stream) {
    int st = check_shape(shape, true);
    if (st != SVOO_OK) return st;
    if (!q_sorted || !k_sorted || !v_sorted || !q_offsets || !k_offsets || !block_count || !block_list || !out_sorted)
        return SVOO_ERR_INVALID_ARG;
    if (!aligned16(q_sorted) || !aligned16(k_sorted) || !aligned16(v_sorted) || !aligned16(out_sorted))
        return SVOO_ERR_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < 1e30f) || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    if ((long long)shape->bh * (shape->kq + 1) > STATIC_SCRATCH_INTS) return SVOO_ERR_STATIC_LIMIT;
    int32_t* tile_prefix = static_scratch_on_current_device();
    if (!tile_prefix) return SVOO_ERR_HIP;
    AttnArgs a = {q_sorted, k_sorted, v_sorted, out_sorted, lse, q_offsets, k_offsets, block_count, block_list,
                  nullptr, nullptr, shape->n, shape->kq, shape->kk, scale};
    // the schedule kernel rewrites every entry this shape uses, so nothing of an earlier call needs clearing
    return launch_sparse(shape, a, tile_prefix, false, (hipStream_t)hip_stream);
}

extern "C" int svoo_block_sparse_attn_tokens(const svoo_shape* shape, const void* q, const int32_t* q_perm,
                                             const void* k_sorted, const void* v_sorted, const int32_t* q_offsets,
                                             const int32_t* k_offsets, const int32_t* block_count,
                                             const int32_t* block_list, float scale, void* out, float* lse,
                                             void* ws, size_t ws_bytes, void* hip_stream) {
    if (!q_perm) return SVOO_ERR_INVALID_ARG;
    return sparse_attn_entry(shape, q, k_sorted, v_sorted, q_perm, q_offsets, k_offsets, block_count, block_list,
                             scale, out, lse, ws, ws_bytes, hip_stream);
}

extern "C" int svoo_attn(const svoo_shape* shape, const void* q, const void* k, const void* v, float scale, void* out,
                         float* lse, void* ws, size_t ws_bytes, void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!q || !k || !v || !out || !ws) return SVOO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (((uintptr_t)ws) & 255u) != 0)
        return SVOO_ERR_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < 1e30f) || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    svoo_shape s = *shape;
    s.kq = 1;
    s.kk = 1;
    if (ws_bytes < attn_ws_bytes(&s)) return SVOO_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;
    WsCarver c(ws);
    int32_t* tile_prefix = c.take<int32_t>((size_t)s.bh * 2);
    int32_t* offsets = c.take<int32_t>((size_t)s.bh * 2);
    int32_t* block_count = c.take<int32_t>((size_t)s.bh);
    int32_t* block_list = c.take<int32_t>((size_t)s.bh);
    hipLaunchKernelGGL(dense_layout_kernel, dim3((s.bh + 255) / 256), dim3(256), 0, stream, offsets, block_count,
                       block_list, s.n, s.bh);
    AttnArgs a = {q, k, v, out, lse, offsets, offsets, block_count, block_list, nullptr, nullptr, s.n, 1, 1, scale};
    return launch_sparse(&s, a, tile_prefix, true, stream);
}

// ---------------------------------------------------------------------------------------------
// Attention recall of a partition + block mask, per token, from the two log-sum-exp outputs:
// the share of the dense softmax mass that falls on the kept keys is exp(LSE_kept - LSE_all).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
row_recall_kernel(const float* __restrict__ lse_kept_sorted, const float* __restrict__ lse_all,
                  const int32_t* __restrict__ q_perm, float* __restrict__ recall, int n) {
    const int b = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
    if (p >= n) return;
    const int tok = clamp_row(q_perm[(size_t)b * n + p], n);
    recall[(size_t)b * n + tok] = expf(lse_kept_sorted[(size_t)b * n + p] - lse_all[(size_t)b * n + tok]);
}

extern "C" int svoo_row_recall(const svoo_shape* shape, const float* lse_kept_sorted, const float* lse_all,
                               const int32_t* q_perm, float* recall, void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!lse_kept_sorted || !lse_all || !q_perm || !recall || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    hipLaunchKernelGGL(row_recall_kernel, dim3((shape->n + 255) / 256, shape->bh), dim3(256), 0,
                       (hipStream_t)hip_stream, lse_kept_sorted, lse_all, q_perm, recall, shape->n);
    return launch_status();
}
