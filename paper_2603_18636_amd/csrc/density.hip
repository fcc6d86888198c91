// Offline profiling: attention density of one head's attention map (paper Sec. 4.1, the offline
// profiling module; the equation defining d_{l,h}).
//
// For a query row i with logits s_t = <q_i, k_t> and p_t = softmax_t(scale * s_t) over all n keys,
// the row's prefix length is the size of the shortest descending-sorted prefix of p whose sum
// reaches tau.  Nothing is sorted: the prefix is { t : s_t >= theta_i } plus, when several keys
// tie at theta_i, as many of them as are needed, and theta_i is found by bisection on the logit
// value.  Every bisection step is one pass over all keys that accumulates, per row, the count and
// the mass of { s_t >= mid }:
//
//   pass 0      row maximum m and minimum of the logits
//   pass 1      Z = sum_t 2^((s_t - m) c2)  (c2 = scale * log2 e) and the key count
//   pass 2...   mass / count above mid;  invariant  M(lo) >= tau Z > M(hi)
//
// until lo and hi enclose a single key, or are adjacent floats (ties).  The logits are recomputed
// in every pass by the same instruction sequence, so they are bit-identical from pass to pass and
// the bisection is consistent.  Masses are added in float32 inside a tile and in float64 across
// tiles.
//
// bf16 inputs: S^T = K Q^T on v_mfma_f32_32x32x16_bf16, one query per lane column, 128 query rows
// per workgroup, K in 64-key LDS tiles filled by direct global->LDS loads (same swizzle as the
// attention kernel).  A row sample that yields fewer workgroups than the chip has compute units
// (the offline profiling samples rows) would leave one wave per SIMD with nothing to hide its
// latencies behind: such launches split the keys KS ways inside the workgroup (4 KS waves, wave
// (rg, ks) takes the tiles ks, ks + KS, ... for row group rg) and combine the KS partial results
// of a pass through LDS in the fixed order ks = 0, 1, ...  float32 inputs: a plain kernel, one
// workgroup per row.
#include <type_traits>

#include "common.h"

#define LOG2E_F 1.4426950408889634f
#define DEN_KT 64
#define DEN_MAX_PASSES 48   // 2 + at most ~34 halvings of a float interval; a hard stop

typedef __attribute__((ext_vector_type(8))) __bf16 den_bf16x8;
typedef __attribute__((ext_vector_type(16))) float den_f32x16;

struct DensityArgs {
    const void* q;
    const void* k;
    const int32_t* rows;     // nullable: query row indices shared by all slices
    int32_t* prefix_len;     // [bh, n_rows]
    int32_t* passes;         // nullable [bh]: most passes over the keys any workgroup of the slice made
    int n, n_rows;
    float scale, tau;
};

// next representable float above x (x finite or +inf)
__device__ __forceinline__ float next_up(float x) {
    if (!(x < INFINITY)) return x;
    uint32_t u = __float_as_uint(x);
    if ((u << 1) == 0) return __uint_as_float(1u);          // +-0 -> smallest subnormal
    return __uint_as_float((u >> 31) ? u - 1 : u + 1);
}

// Per-row bisection state, identical in the two lanes (or all threads) that share a row.
struct RowState {
    float m, mn, nmb, thr, lo, hi;
    double target, m_hi;
    int c_lo, c_hi;
    bool done;
};

__device__ __forceinline__ void row_state_init(RowState& r) {
    r.m = -INFINITY; r.mn = INFINITY; r.nmb = 0.f; r.thr = -3.4028234e38f; r.lo = 0.f; r.hi = 0.f;
    r.target = 0.0; r.m_hi = 0.0; r.c_lo = 0; r.c_hi = 0; r.done = false;
}

// End of a pass: fold the pass result (row max/min, or mass and count above thr) into the state.
__device__ __forceinline__ void row_state_step(RowState& r, int pass, float mx, float mn, double mass, int cnt,
                                               float c2, float tau) {
    if (pass == 0) {
        r.m = mx;
        r.mn = mn;
        r.nmb = -mx * c2;
        return;
    }
    if (pass == 1) {
        r.target = (double)tau * mass;
        r.c_lo = cnt;
        r.c_hi = 0;
        r.m_hi = 0.0;
        r.lo = r.mn;
        r.hi = next_up(r.m);
    } else if (!r.done) {
        if (mass >= r.target) {
            r.lo = r.thr;
            r.c_lo = cnt;
        } else {
            r.hi = r.thr;
            r.c_hi = cnt;
            r.m_hi = mass;
        }
    }
    if (!r.done) {
        if (r.c_lo - r.c_hi <= 1) {
            r.done = true;
        } else {
            const float mid = r.lo + 0.5f * (r.hi - r.lo);
            if (mid > r.lo && mid < r.hi)
                r.thr = mid;
            else
                r.done = true;        // adjacent floats (or not finite): every key left ties at lo
        }
    }
}

__device__ __forceinline__ int row_state_result(const RowState& r, float c2, int n) {
    const int ties = r.c_lo - r.c_hi;
    int take = ties;
    if (ties > 1) {
        const float p = __builtin_amdgcn_exp2f(fmaf(r.lo, c2, r.nmb));
        const double need = r.target - r.m_hi;
        double t = p > 0.f ? ceil(need / (double)p) : (double)ties;
        t = t < 1.0 ? 1.0 : (t > (double)ties ? (double)ties : t);
        take = (int)t;
    }
    int len = r.c_hi + (take < 1 ? 1 : take);
    return len < 1 ? 1 : (len > n ? n : len);
}

// per-row partial result of one pass, one per key split
struct PassPartial {
    float mx, mn;
    int cnt, pad;
    double mass;
};

template <int D, int KS, int NBUF>
static constexpr size_t density_lds_bytes() {
    return (size_t)NBUF * KS * DEN_KT * D * 2 + (KS > 1 ? (size_t)KS * 128 * sizeof(PassPartial) : 0);
}

template <int D, int KS, int NBUF>
__global__ void __launch_bounds__(256 * KS)
density_bf16_kernel(DensityArgs a) {
    constexpr int DC = D / 16, CPR = D / 8, ROWB = D * 2, TILE = DEN_KT * ROWB, STAGE = KS * TILE;
    constexpr int RPL = 64 / CPR;             // tile rows covered by one wave-load (1 KB)
    constexpr int LPW = (DEN_KT / 4) / RPL;   // wave-loads per wave and step (a quarter of one tile)
    static_assert(NBUF == 2 || NBUF == 3, "two or three stages");
    extern __shared__ __attribute__((aligned(1024))) unsigned char k_lds[];
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid % 64, j = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64), rg = wave % 4, ks = wave / 4;
    const int n = a.n;
    const int rloc = 32 * rg + j;
    const int ridx = blockIdx.x * 128 + rloc;
    const bool rvalid = ridx < a.n_rows;
    int qrow = rvalid ? (a.rows ? a.rows[ridx] : ridx) : 0;
    qrow = qrow < 0 ? 0 : (qrow >= n ? n - 1 : qrow);
    const unsigned char* kg = (const unsigned char*)a.k + (size_t)b * n * ROWB;
    const int n_tiles = (n + DEN_KT - 1) / DEN_KT;
    const int n_steps = (n_tiles + KS - 1) / KS;     // a step = KS tiles, one per key split

    // wave (rg, ks) fetches quarter rg of the tile its key split consumes in step `step`
    auto issue = [&](int step, int buf) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int rl = (rg * LPW + i) * RPL + lane / CPR;       // tile row
            int row = (step * KS + ks) * DEN_KT + rl;
            row = row < n ? row : n - 1;                            // rows past the end are masked or unused
            const int chunk = (lane % CPR) ^ (rl % CPR);
            load_global_to_lds_16(kg + (size_t)row * ROWB + chunk * 16,
                                  lds_address(k_lds) + buf * STAGE + ks * TILE + (rg * LPW + i) * RPL * ROWB);
        }
    };
#pragma unroll
    for (int p = 0; p < NBUF - 1; ++p) issue(p % n_steps, p);

    den_bf16x8 qf[DC];
    {
        const uint4* src = (const uint4*)((const uint16_t*)a.q + ((size_t)b * n + qrow) * D);
#pragma unroll
        for (int c = 0; c < DC; ++c) qf[c] = __builtin_bit_cast(den_bf16x8, rvalid ? src[2 * c + h] : make_uint4(0, 0, 0, 0));
    }
    int koff[DC];
#pragma unroll
    for (int c = 0; c < DC; ++c) koff[c] = j * ROWB + (((2 * c + h) ^ (j % CPR)) * 16);
    // the compiler's wait for the Q loads must not end up inside the tile loop
#pragma unroll
    for (int c = 0; c < DC; ++c) asm volatile("" ::"v"(qf[c]));

    const float c2 = a.scale * LOG2E_F;
    RowState st;
    row_state_init(st);
    float mx = -INFINITY, mn = INFINITY;
    double mass = 0.0;
    int cnt = 0;
    int pass = 0, step = 0;
    // steps are consumed in one running sequence g = pass * n_steps + step; step g sits in stage
    // g % NBUF and the next NBUF - 1 steps are in flight or landed
    for (int g = 0;; ++g) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW * (NBUF - 2)) : "memory");   // all but the newest steps' loads
        __syncthreads();
        {
            int ns = step + NBUF - 1;
            ns = ns >= n_steps ? ns % n_steps : ns;      // wraps into the next pass (n_steps may be 1 or 2)
            issue(ns, (g + NBUF - 1) % NBUF);
        }
        const int kt = step * KS + ks;
        if (kt < n_tiles) {
            const unsigned char* base = k_lds + (g % NBUF) * STAGE + ks * TILE;
            den_f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
            for (int c = 0; c < DC; ++c) {
                const den_bf16x8 a0 = __builtin_bit_cast(den_bf16x8, *(const uint4*)(base + koff[c]));
                const den_bf16x8 a1 = __builtin_bit_cast(den_bf16x8, *(const uint4*)(base + 32 * ROWB + koff[c]));
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[c], s[0], 0, 0, 0);
                s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[c], s[1], 0, 0, 0);
            }
            const bool ragged = kt == n_tiles - 1 && (n % DEN_KT) != 0;
            if (pass == 0) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const bool valid = !ragged || kt * DEN_KT + 32 * kb + 8 * (v / 4) + 4 * h + (v % 4) < n;
                        mx = fmaxf(mx, valid ? s[kb][v] : -INFINITY);
                        mn = fminf(mn, valid ? s[kb][v] : INFINITY);
                    }
            } else {
                float ts = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const bool valid = !ragged || kt * DEN_KT + 32 * kb + 8 * (v / 4) + 4 * h + (v % 4) < n;
                        const float sv = s[kb][v];
                        const float p = __builtin_amdgcn_exp2f(fmaf(sv, c2, st.nmb));
                        const bool ge = valid && sv >= st.thr;
                        ts += ge ? p : 0.f;
                        cnt += ge ? 1 : 0;
                    }
                mass += (double)ts;
            }
        }
        if (++step == n_steps) {
            // both half-waves hold half of each row's keys: exchange and combine
            {
                auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(mx), __float_as_int(mx), false, false);
                mx = fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
                r = __builtin_amdgcn_permlane32_swap(__float_as_int(mn), __float_as_int(mn), false, false);
                mn = fminf(__int_as_float(r[0]), __int_as_float(r[1]));
                r = __builtin_amdgcn_permlane32_swap(cnt, cnt, false, false);
                cnt = (int)r[0] + (int)r[1];
                const long long mb = __double_as_longlong(mass);
                const int lo32 = (int)(mb & 0xffffffffLL), hi32 = (int)(mb >> 32);
                auto rl = __builtin_amdgcn_permlane32_swap(lo32, lo32, false, false);
                auto rh = __builtin_amdgcn_permlane32_swap(hi32, hi32, false, false);
                const double m0 = __longlong_as_double(((long long)(int)rh[0] << 32) | (unsigned int)rl[0]);
                const double m1 = __longlong_as_double(((long long)(int)rh[1] << 32) | (unsigned int)rl[1]);
                mass = m0 + m1;      // (own, other) in one half, (other, own) in the other: same sum
            }
            if constexpr (KS > 1) {
                // the key splits of a row group exchange their partial results; every wave then adds
                // them in the order ks = 0, 1, ..., so all of them step the same row state
                PassPartial* part = (PassPartial*)(k_lds + (size_t)NBUF * STAGE);
                if (h == 0) part[ks * 128 + rloc] = PassPartial{mx, mn, cnt, 0, mass};
                __syncthreads();
                PassPartial t = part[rloc];
#pragma unroll
                for (int o = 1; o < KS; ++o) {
                    const PassPartial u = part[o * 128 + rloc];
                    t.mx = fmaxf(t.mx, u.mx);
                    t.mn = fminf(t.mn, u.mn);
                    t.cnt += u.cnt;
                    t.mass += u.mass;
                }
                mx = t.mx; mn = t.mn; cnt = t.cnt; mass = t.mass;
            }
            row_state_step(st, pass, mx, mn, mass, cnt, c2, a.tau);
            mass = 0.0;
            cnt = 0;
            step = 0;
            ++pass;
            // also orders this pass's reads of the partial results before the next pass's writes
            const int all_done = __syncthreads_and((st.done || !rvalid) ? 1 : 0);
            if (all_done || pass >= DEN_MAX_PASSES) break;
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // loads issued for the pass that never ran
    if (a.passes && tid == 0) atomicMax(&a.passes[b], pass);
    if (rvalid && h == 0 && ks == 0) a.prefix_len[(size_t)b * a.n_rows + ridx] = row_state_result(st, c2, n);
}

template <int D, int KS, int NBUF>
static int launch_density_bf16(const DensityArgs& a, int bh, hipStream_t stream) {
    static unsigned char opted_in[SVOO_MAX_DEVICES];
    constexpr int lds = (int)density_lds_bytes<D, KS, NBUF>();
    auto kern = density_bf16_kernel<D, KS, NBUF>;
    if (!opt_in_dynamic_lds((const void*)kern, lds, opted_in)) return SVOO_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((a.n_rows + 127) / 128, bh), dim3(256 * KS), lds, stream, a);
    return SVOO_OK;
}

// Fewer workgroups than the chip can hold at one per compute unit (or two): split the keys inside
// the workgroup so that every SIMD still has several waves.
template <int D>
static int dispatch_density_bf16(const DensityArgs& a, int bh, hipStream_t stream) {
    const long long wgs = (long long)((a.n_rows + 127) / 128) * bh;
    if (wgs <= 256) return launch_density_bf16<D, 4, 2>(a, bh, stream);
    if (wgs <= 512) return launch_density_bf16<D, 2, 2>(a, bh, stream);
    return launch_density_bf16<D, 1, 3>(a, bh, stream);
}

// ---------------------------------------------------------------------------------------------
// float32 inputs (and a plain reference shape of the same algorithm): one workgroup per query
// row, every thread owns the keys tid, tid + 256, ...; logits by a fixed-order FMA chain.
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(256)
density_rowwise_kernel(DensityArgs a) {
    __shared__ float qs[D];
    __shared__ float red_f[2][256];
    __shared__ double red_d[256];
    __shared__ int red_i[256];
    const int b = blockIdx.y, ridx = blockIdx.x, tid = threadIdx.x, n = a.n;
    int qrow = a.rows ? a.rows[ridx] : ridx;
    qrow = qrow < 0 ? 0 : (qrow >= n ? n - 1 : qrow);
    const T* qg = (const T*)a.q + ((size_t)b * n + qrow) * D;
    const T* kg = (const T*)a.k + (size_t)b * n * D;
    auto as_f32 = [](const T* p) -> float {
        if constexpr (std::is_same<T, float>::value) return *p;
        else return bf16_to_f32(*(const uint16_t*)p);
    };
    if (tid < D) qs[tid] = as_f32(qg + tid);
    __syncthreads();
    const float c2 = a.scale * LOG2E_F;
    RowState st;
    row_state_init(st);
    int pass = 0;
    for (; pass < DEN_MAX_PASSES; ++pass) {
        float mx = -INFINITY, mn = INFINITY;
        double mass = 0.0;
        int cnt = 0;
        for (int t = tid; t < n; t += 256) {
            const T* kr = kg + (size_t)t * D;
            float sv = 0.f;
            for (int c = 0; c < D; ++c) sv = fmaf(qs[c], as_f32(kr + c), sv);
            if (pass == 0) {
                mx = fmaxf(mx, sv);
                mn = fminf(mn, sv);
            } else if (sv >= st.thr) {
                mass += (double)__builtin_amdgcn_exp2f(fmaf(sv, c2, st.nmb));
                ++cnt;
            }
        }
        red_f[0][tid] = mx;
        red_f[1][tid] = mn;
        red_d[tid] = mass;
        red_i[tid] = cnt;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if (tid < w) {
                red_f[0][tid] = fmaxf(red_f[0][tid], red_f[0][tid + w]);
                red_f[1][tid] = fminf(red_f[1][tid], red_f[1][tid + w]);
                red_d[tid] += red_d[tid + w];
                red_i[tid] += red_i[tid + w];
            }
            __syncthreads();
        }
        row_state_step(st, pass, red_f[0][0], red_f[1][0], red_d[0], red_i[0], c2, a.tau);
        __syncthreads();
        if (st.done) break;          // uniform: every thread holds the same state
    }
    if (a.passes && tid == 0) atomicMax(&a.passes[b], pass + 1 < DEN_MAX_PASSES ? pass + 1 : DEN_MAX_PASSES);
    if (tid == 0) a.prefix_len[(size_t)b * a.n_rows + ridx] = row_state_result(st, c2, n);
}

// density[b] = mean_i prefix_len[b, i] / n: integer sum in a fixed order, one division
__global__ void __launch_bounds__(1024)
density_mean_kernel(const int32_t* __restrict__ prefix_len, double* __restrict__ density, int n_rows, int n) {
    __shared__ long long red[1024];
    const int b = blockIdx.x, t = threadIdx.x;
    long long s = 0;
    for (int i = t; i < n_rows; i += 1024) s += prefix_len[(size_t)b * n_rows + i];
    red[t] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    if (t == 0) density[b] = (double)red[0] / ((double)n_rows * (double)n);
}

__global__ void density_clear_kernel(int32_t* p, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0;
}

extern "C" int svoo_attention_density(const svoo_shape* shape, const void* q, const void* k, const int32_t* rows,
                                      int32_t n_rows, float tau, float scale, int32_t* prefix_len, double* density,
                                      int32_t* passes, void* hip_stream) {
    int st = check_shape(shape, false);
    if (st != SVOO_OK) return st;
    if (!q || !k || !prefix_len || !density) return SVOO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || shape->bh > 65535) return SVOO_ERR_INVALID_ARG;
    if (n_rows < 1 || n_rows > shape->n || (!rows && n_rows != shape->n)) return SVOO_ERR_INVALID_ARG;
    if (!(tau > 0.0f) || !(tau <= 1.0f) || !(scale > 0.0f) || !(scale < 1e30f)) return SVOO_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    DensityArgs a = {q, k, rows, prefix_len, passes, shape->n, n_rows, scale, tau};
    if (passes)
        hipLaunchKernelGGL(density_clear_kernel, dim3((shape->bh + 255) / 256), dim3(256), 0, stream, passes, shape->bh);
    if (shape->dtype == SVOO_BF16) {
        st = shape->d == 128 ? dispatch_density_bf16<128>(a, shape->bh, stream)
                             : dispatch_density_bf16<64>(a, shape->bh, stream);
        if (st != SVOO_OK) return st;
    } else {
        dim3 grid(n_rows, shape->bh);
        if (shape->d == 128)
            hipLaunchKernelGGL((density_rowwise_kernel<float, 128>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((density_rowwise_kernel<float, 64>), grid, dim3(256), 0, stream, a);
    }
    hipLaunchKernelGGL(density_mean_kernel, dim3(shape->bh), dim3(1024), 0, stream, prefix_len, density, n_rows,
                       shape->n);
    return launch_status();
}
