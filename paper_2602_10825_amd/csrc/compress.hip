// KV-cache compression at a chunk commit (Sec. 3.3, Eq. (10)-(12); App. C.1, C.2).
//
// Kernels, all stream-ordered, float64 arithmetic, no floating-point atomics:
//   key_stats      pass 1 over K: per token 1/max(||k||,1e-12) and k^.k^; per block the
//                  partial sum of normalised keys                      (HBM-bound)
//   sum_partials   per head: fixed-order sum of the block partials -> s = sum_i k^_i
//   mean_sim       pass 2 over K: r_j = (k^_j . s - k^_j . k^_j) / L   (HBM-bound), the
//                  linear-time form of the diagonal-zeroed column mean of Eq. (11)
//   score_select   per head: softmax over r (Eq. (11)), max-pooled importance (Eq. (10)),
//                  score (Eq. (12)) -> order-preserving 64-bit keys; radix select of the
//                  budget-th largest key, started at the most significant bit in which
//                  the keys differ and finished on the few candidates left, in LDS; ordered
//                  compaction of the kept positions (ties: lower position wins; ascending)
//   gather_rows / copy_back   move kept K and V rows to positions [0, budget)
// A 16-lane group owns one token row in the two passes over K (16-byte loads, a full
// row per group), so a token's values never depend on where it sits in the launch.
#include "fc_common.hpp"

#pragma clang fp contract(off)

namespace {

constexpr int kThreads = 256;
constexpr int kGroups = kThreads / 16;
constexpr int kSelThreads = 1024;
constexpr int kItems = 8;

// ---- per-lane slice of one token row, widened exactly to float64 ---------------------
template <typename T, int D>
__device__ __forceinline__ void load_slice(const T* row, int u, double (&x)[D / 16]) {
    constexpr int EL = D / 16;
    const T* p = row + u * EL;
    if constexpr (sizeof(T) == 2 && EL == 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        float f[8];
        unpack16(v, f, bf16_t());
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (double)f[e];
    } else if constexpr (sizeof(T) == 2 && EL == 4) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        x[0] = (double)bf16lo_to_f32(v.x); x[1] = (double)bf16hi_to_f32(v.x);
        x[2] = (double)bf16lo_to_f32(v.y); x[3] = (double)bf16hi_to_f32(v.y);
    } else {
#pragma unroll
        for (int e = 0; e < EL; e += 4) {
            const float4 v = *reinterpret_cast<const float4*>(p + e);
            x[e] = (double)v.x; x[e + 1] = (double)v.y; x[e + 2] = (double)v.z; x[e + 3] = (double)v.w;
        }
    }
}

// all-reduce over the 16 lanes of a group; every lane ends with identical bits
__device__ __forceinline__ double group_sum(double v) {
    v += __shfl_xor(v, 1, 16);
    v += __shfl_xor(v, 2, 16);
    v += __shfl_xor(v, 4, 16);
    v += __shfl_xor(v, 8, 16);
    return v;
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void key_stats_kernel(
    const T* __restrict__ k_cache, int64_t head_stride, int64_t tok_stride, int L,
    double2* __restrict__ tokinfo, double* __restrict__ psum) {
    constexpr int EL = D / 16;
    const int h = blockIdx.y;
    const int g = threadIdx.x / 16, u = threadIdx.x % 16;
    const T* base = k_cache + (int64_t)h * head_stride;
    double acc[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[e] = 0.0;
    for (int j = blockIdx.x * kGroups + g; j < L; j += gridDim.x * kGroups) {
        double x[EL];
        load_slice<T, D>(base + (int64_t)j * tok_stride, u, x);
        double n2 = 0.0;
#pragma unroll
        for (int e = 0; e < EL; ++e) n2 = fma(x[e], x[e], n2);
        n2 = group_sum(n2);
        const double nrm = sqrt(n2);
        const double inv = 1.0 / fmax(nrm, 1e-12);
        if (u == 0) tokinfo[(int64_t)h * L + j] = make_double2(inv, (n2 * inv) * inv);
#pragma unroll
        for (int e = 0; e < EL; ++e) acc[e] += x[e] * inv;
    }
    __shared__ double sh[kGroups][D];
#pragma unroll
    for (int e = 0; e < EL; ++e) sh[g][u * EL + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < D) {
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < kGroups; ++k) t += sh[k][threadIdx.x];
        psum[((int64_t)h * gridDim.x + blockIdx.x) * D + threadIdx.x] = t;
    }
}

// s = sum over blocks of the partial sums, in a fixed order: thread (slice, e) adds the
// partials b = slice, slice + SL, ... ; the SL slice sums are then added in slice order.
template <int D>
__global__ __launch_bounds__(1024) void sum_partials_kernel(const double* __restrict__ psum,
                                                            int nblk, double* __restrict__ ssum) {
    constexpr int SL = 1024 / D;
    const int h = blockIdx.x, e = threadIdx.x % D, sl = threadIdx.x / D;
    const double* p = psum + (int64_t)h * nblk * D + e;
    double t = 0.0;
    int b = sl;
    for (; b + 3 * SL < nblk; b += 4 * SL) {
        const double v0 = p[(int64_t)b * D], v1 = p[(int64_t)(b + SL) * D];
        const double v2 = p[(int64_t)(b + 2 * SL) * D], v3 = p[(int64_t)(b + 3 * SL) * D];
        t += v0; t += v1; t += v2; t += v3;
    }
    for (; b < nblk; b += SL) t += p[(int64_t)b * D];
    __shared__ double sh[SL][D];
    sh[sl][e] = t;
    __syncthreads();
    if (sl == 0) {
        double tot = 0.0;
#pragma unroll
        for (int k = 0; k < SL; ++k) tot += sh[k][e];
        ssum[h * D + e] = tot;
    }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void mean_sim_kernel(
    const T* __restrict__ k_cache, int64_t head_stride, int64_t tok_stride, int L,
    const double2* __restrict__ tokinfo, const double* __restrict__ ssum,
    double* __restrict__ r, double* __restrict__ pmax) {
    constexpr int EL = D / 16;
    const int h = blockIdx.y;
    const int g = threadIdx.x / 16, u = threadIdx.x % 16;
    const T* base = k_cache + (int64_t)h * head_stride;
    double s[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) s[e] = ssum[h * D + u * EL + e];
    const double dL = (double)L;
    double rmax = -1.0e300;
    for (int j = blockIdx.x * kGroups + g; j < L; j += gridDim.x * kGroups) {
        double x[EL];
        load_slice<T, D>(base + (int64_t)j * tok_stride, u, x);
        double dot = 0.0;
#pragma unroll
        for (int e = 0; e < EL; ++e) dot = fma(x[e], s[e], dot);
        dot = group_sum(dot);
        if (u == 0) {
            const double2 ti = tokinfo[(int64_t)h * L + j];
            const double rj = (dot * ti.x - ti.y) / dL;
            r[(int64_t)h * L + j] = rj;
            rmax = fmax(rmax, rj);
        }
    }
    __shared__ double shm[kGroups];
    if (u == 0) shm[g] = rmax;
    __syncthreads();
    if (threadIdx.x == 0) {
        double m = shm[0];
#pragma unroll
        for (int k = 1; k < kGroups; ++k) m = fmax(m, shm[k]);
        pmax[(int64_t)h * gridDim.x + blockIdx.x] = m;
    }
}

// ---- block-wide helpers for the per-head selection kernel (1024 threads) --------------
__device__ __forceinline__ double block_max_d(double v, double* sh) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, FC_WAVE));
    const int w = threadIdx.x / FC_WAVE;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[w] = v;
    __syncthreads();
    double m = sh[0];
    for (int k = 1; k < kSelThreads / FC_WAVE; ++k) m = fmax(m, sh[k]);
    return m;
}

// fixed-shape tree: deterministic for a given block size
__device__ __forceinline__ double block_sum_d(double v, double* sh) {
    __syncthreads();
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = kSelThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    return sh[0];
}

__device__ __forceinline__ uint64_t score_key(double score) {
    if (score == 0.0) score = 0.0;  // -0 -> +0
    const uint64_t b = (uint64_t)__double_as_longlong(score);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

constexpr int kDigitBits = 11;
constexpr int kBins = 1 << kDigitBits;
constexpr int kCand = 4096;   // candidates resolved in LDS
constexpr int kUnroll = 8;    // independent loads in flight per thread in the selection scans

__device__ __forceinline__ uint64_t block_reduce_u64(uint64_t v, bool want_max, uint64_t* sh) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t w = (uint64_t)__shfl_xor((long long)v, o, FC_WAVE);
        v = want_max ? (w > v ? w : v) : (w < v ? w : v);
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x / FC_WAVE] = v;
    __syncthreads();
    uint64_t m = sh[0];
    for (int k = 1; k < kSelThreads / FC_WAVE; ++k) m = want_max ? (sh[k] > m ? sh[k] : m) : (sh[k] < m ? sh[k] : m);
    return m;
}

// From a histogram of `nb` <= 2048 bins (counts of the current candidates by digit), find the
// bin that holds the `need`-th largest candidate and the number of candidates in higher
// bins.  All 1024 threads take part: thread t owns the two bins nb-1-2t and nb-2-2t, a block
// scan in descending bin order gives the count above each, and the one thread whose bin
// straddles `need` publishes the answer.  (A single thread walking the bins would pay one
// LDS round trip per bin.)
__device__ __forceinline__ void pick_bin_parallel(const uint32_t* hist, int nb, uint32_t need,
                                                  uint32_t* wsum, uint64_t prefix, int shift,
                                                  uint64_t* out_prefix, uint32_t* out_need,
                                                  uint32_t* out_count) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid / FC_WAVE;
    const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
    const uint32_t h0 = (b0 >= 0) ? hist[b0] : 0u;
    const uint32_t h1 = (b1 >= 0) ? hist[b1] : 0u;
    uint32_t inc = h0 + h1;   // inclusive scan over threads (= descending bins)
#pragma unroll
    for (int o = 1; o < FC_WAVE; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o, FC_WAVE);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    uint32_t above = inc - (h0 + h1);
    for (int w = 0; w < wave; ++w) above += wsum[w];
    if (b0 >= 0 && above < need && need <= above + h0) {
        *out_prefix = prefix | ((uint64_t)b0 << shift);
        *out_need = need - above;
        *out_count = h0;
    } else if (b1 >= 0 && above + h0 < need && need <= above + h0 + h1) {
        *out_prefix = prefix | ((uint64_t)b1 << shift);
        *out_need = need - above - h0;
        *out_count = h1;
    }
}

// Histogram increment that survives skew: the digits most lanes of a wavefront share are
// counted once per wavefront (up to four rounds of leader election); the rest go one by one.
__device__ __forceinline__ void hist_add(uint32_t* hist, bool in, uint32_t dgt) {
    uint64_t act = __ballot(in);
#pragma unroll 1
    for (int round = 0; round < 4 && act; ++round) {
        const int leader = __ffsll((long long)act) - 1;
        const uint32_t d0 = __shfl(dgt, leader, FC_WAVE);
        const uint64_t same = __ballot(in && dgt == d0);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
        in = in && (dgt != d0);
        act &= ~same;
    }
    if (in) atomicAdd(&hist[dgt], 1u);
}

// Append `k` to an LDS list from the lanes with `take`; one counter update per wavefront.
__device__ __forceinline__ void list_append(uint64_t* list, uint32_t* counter, bool take, uint64_t k) {
    const uint64_t m = __ballot(take);
    if (m == 0) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((long long)m) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = __shfl(base, leader, FC_WAVE);
    if (take) list[base + __popcll(m & ((1ull << lane) - 1ull))] = k;
}

__global__ __launch_bounds__(kSelThreads) void score_select_kernel(
    const double* __restrict__ r_all, const float* __restrict__ mass_all,
    const double* __restrict__ pmax_all, int nblk, int L, int budget, int pool_k, double lambda,
    double* __restrict__ etmp_all, uint64_t* __restrict__ keys_all, int32_t* __restrict__ kept_all) {
    const int h = blockIdx.x;
    const int tid = threadIdx.x;
    const double* r = r_all + (int64_t)h * L;
    const float* mass = mass_all + (int64_t)h * L;
    double* etmp = etmp_all + (int64_t)h * L;
    uint64_t* keys = keys_all + (int64_t)h * L;
    int32_t* kept = kept_all + (int64_t)h * budget;

    __shared__ double shd[kSelThreads];
    __shared__ uint64_t shu[kSelThreads / FC_WAVE];
    __shared__ uint32_t hist[kBins];
    __shared__ uint64_t cand[kCand];
    __shared__ uint32_t wtot[2][kSelThreads / FC_WAVE];
    __shared__ uint64_t sh_prefix;
    __shared__ uint32_t sh_need, sh_count, sh_ncand;

    // Eq. (11): softmax over the token index of r.  max r comes from the block maxima of
    // the pass that produced r.
    double mx = -1.0e300;
    for (int i = tid; i < nblk; i += kSelThreads) mx = fmax(mx, pmax_all[(int64_t)h * nblk + i]);
    mx = block_max_d(mx, shd);
    // All scans below fetch kUnroll independent elements per thread before using them: one
    // block per head is latency-bound otherwise.
    double z = 0.0;
    for (int base = 0; base < L; base += kSelThreads * kUnroll) {
        double rv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = base + u * kSelThreads + tid;
            rv[u] = (j < L) ? r[j] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = base + u * kSelThreads + tid;
            if (j < L) {
                const double e = exp(rv[u] - mx);
                etmp[j] = e;
                z += e;
            }
        }
    }
    z = block_sum_d(z, shd);

    // Eq. (10) + Eq. (12) -> sortable keys; their min and max bound the bits that matter
    const int half = pool_k / 2;
    uint64_t kmin = ~0ull, kmax = 0ull;
    for (int base = 0; base < L; base += kSelThreads * kUnroll) {
        double ev[kUnroll];
        float imp[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = base + u * kSelThreads + tid;
            ev[u] = (j < L) ? etmp[j] : 0.0;
            imp[u] = (j < L) ? mass[j] : 0.f;
        }
        for (int d = 1; d <= half; ++d) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int j = base + u * kSelThreads + tid;
                if (j < L) {
                    const float lo = (j - d >= 0) ? mass[j - d] : imp[u];
                    const float hi = (j + d < L) ? mass[j + d] : imp[u];
                    imp[u] = fmaxf(imp[u], fmaxf(lo, hi));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = base + u * kSelThreads + tid;
            if (j < L) {
                const double red = ev[u] / z;
                const double a = lambda * (double)imp[u];
                const double b = (1.0 - lambda) * red;
                const uint64_t k = score_key(a - b);
                keys[j] = k;
                kmin = k < kmin ? k : kmin;
                kmax = k > kmax ? k : kmax;
            }
        }
    }
    kmin = block_reduce_u64(kmin, false, shu);
    kmax = block_reduce_u64(kmax, true, shu);
    __syncthreads();

    // Radix select of the budget-th largest key.  All keys agree above bit `top`.
    uint64_t thr;
    uint32_t need = (uint32_t)budget;
    const uint64_t diff = kmin ^ kmax;
    if (diff == 0) {
        thr = kmax;   // every score is the same: keep the first `budget` positions
    } else {
        const int top = 63 - __clzll((long long)diff);
        int rem = top + 1;                                         // undecided low bits
        uint64_t prefix = (rem == 64) ? 0ull : (kmax >> rem) << rem;
        bool in_lds = false;
        uint32_t ncand = 0;
        while (rem > 0) {
            const int w = in_lds ? (rem < 8 ? rem : 8) : (rem < kDigitBits ? rem : kDigitBits);
            const int shift = rem - w;
            const int nb = 1 << w;
            for (int i = tid; i < nb; i += kSelThreads) hist[i] = 0;
            __syncthreads();
            const uint64_t himask = (rem == 64) ? 0ull : (~0ull << rem);
            if (in_lds) {
                for (uint32_t i0 = 0; i0 < ncand; i0 += kSelThreads) {
                    const uint32_t i = i0 + tid;
                    const uint64_t k = (i < ncand) ? cand[i] : ~prefix;
                    hist_add(hist, i < ncand && (k & himask) == prefix, (uint32_t)(k >> shift) & (nb - 1));
                }
            } else {
                for (int base = 0; base < L; base += kSelThreads * kUnroll) {
                    uint64_t kv[kUnroll];
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        const int j = base + u * kSelThreads + tid;
                        kv[u] = (j < L) ? keys[j] : ~prefix;   // padding never matches the prefix
                    }
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u)
                        hist_add(hist, (kv[u] & himask) == prefix && base + u * kSelThreads + tid < L,
                                 (uint32_t)(kv[u] >> shift) & (nb - 1));
                }
            }
            __syncthreads();
            if (tid == 0) sh_ncand = 0;
            pick_bin_parallel(hist, nb, need, wtot[0], prefix, shift, &sh_prefix, &sh_need, &sh_count);
            __syncthreads();
            prefix = sh_prefix;
            need = sh_need;
            rem = shift;
            // few candidates left: pull them into LDS and finish there
            if (!in_lds && rem > 0 && sh_count <= (uint32_t)kCand) {
                const uint64_t hm = ~0ull << rem;
                for (int base = 0; base < L; base += kSelThreads * kUnroll) {
                    uint64_t kv[kUnroll];
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        const int j = base + u * kSelThreads + tid;
                        kv[u] = (j < L) ? keys[j] : 0ull;
                    }
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u)
                        list_append(cand, &sh_ncand,
                                    (kv[u] & hm) == prefix && base + u * kSelThreads + tid < L, kv[u]);
                }
                __syncthreads();
                ncand = sh_ncand;
                in_lds = true;
            }
        }
        thr = prefix;
    }

    // ordered compaction: position = #greater before + min(#equal before, need)
    uint32_t run_gt = 0, run_eq = 0;
    const int wave = tid / FC_WAVE, lane = tid & 63;
    for (int base = 0; base < L; base += kSelThreads * kItems) {
        const int j0 = base + tid * kItems;
        uint32_t fgt = 0, feq = 0;  // bit masks over the thread's items
        uint64_t kv[kItems];
#pragma unroll
        for (int i = 0; i < kItems; ++i) kv[i] = (j0 + i < L) ? keys[j0 + i] : 0ull;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            if (j0 + i < L) {
                fgt |= (kv[i] > thr) ? (1u << i) : 0u;
                feq |= (kv[i] == thr) ? (1u << i) : 0u;
            }
        }
        const uint32_t cg = __popc(fgt), ce = __popc(feq);
        // inclusive wave scans
        uint32_t sg = cg, se = ce;
#pragma unroll
        for (int o = 1; o < FC_WAVE; o <<= 1) {
            const uint32_t tg = __shfl_up(sg, o, FC_WAVE);
            const uint32_t te = __shfl_up(se, o, FC_WAVE);
            if (lane >= o) { sg += tg; se += te; }
        }
        __syncthreads();
        if (lane == 63) { wtot[0][wave] = sg; wtot[1][wave] = se; }
        __syncthreads();
        uint32_t pg = run_gt, pe = run_eq, allg = 0, alle = 0;
        for (int w = 0; w < kSelThreads / FC_WAVE; ++w) {
            if (w < wave) { pg += wtot[0][w]; pe += wtot[1][w]; }
            allg += wtot[0][w];
            alle += wtot[1][w];
        }
        uint32_t gt_before = pg + sg - cg;
        uint32_t eq_before = pe + se - ce;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const bool g = (fgt >> i) & 1u, e = (feq >> i) & 1u;
            if (g || (e && eq_before < need)) {
                const uint32_t pos = gt_before + (eq_before < need ? eq_before : need);
                kept[pos] = j0 + i;
            }
            gt_before += g ? 1u : 0u;
            eq_before += e ? 1u : 0u;
        }
        run_gt += allg;
        run_eq += alle;
    }
}

__global__ void iota_kernel(int32_t* kept, int H, int n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)H * n) kept[i] = (int32_t)(i % n);
}

// ---- compaction: kept rows -> staging -> positions [0, budget) ------------------------
// rows are `vpr` 16-byte vectors; a row whose position does not change is skipped.
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(
    const uint4* __restrict__ k_cache, const uint4* __restrict__ v_cache, int64_t head_stride_v,
    int64_t tok_stride_v, int vpr, int budget, const int32_t* __restrict__ kept,
    uint4* __restrict__ stage_k, uint4* __restrict__ stage_v) {
    const int h = blockIdx.y;
    const int64_t total = (int64_t)budget * vpr;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int s = (int)(i / vpr), v = (int)(i % vpr);
        const int src = kept[(int64_t)h * budget + s];
        if (src == s) continue;
        const int64_t a = h * head_stride_v + (int64_t)src * tok_stride_v + v;
        const int64_t d = ((int64_t)h * budget + s) * vpr + v;
        stage_k[d] = k_cache[a];
        stage_v[d] = v_cache[a];
    }
}

__global__ __launch_bounds__(kThreads) void copy_back_kernel(
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, int64_t head_stride_v,
    int64_t tok_stride_v, int vpr, int budget, const int32_t* __restrict__ kept,
    const uint4* __restrict__ stage_k, const uint4* __restrict__ stage_v) {
    const int h = blockIdx.y;
    const int64_t total = (int64_t)budget * vpr;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int s = (int)(i / vpr), v = (int)(i % vpr);
        if (kept[(int64_t)h * budget + s] == s) continue;
        const int64_t a = h * head_stride_v + (int64_t)s * tok_stride_v + v;
        const int64_t d = ((int64_t)h * budget + s) * vpr + v;
        k_cache[a] = stage_k[d];
        v_cache[a] = stage_v[d];
    }
}

struct WsLayout {
    size_t tokinfo, r, keys, psum, ssum, pmax, stage_k, stage_v, total;
    int nblk;
};

WsLayout layout(int H, int L, int d, int budget, fc_dtype dtype) {
    WsLayout w;
    int nblk = (L + kGroups * 8 - 1) / (kGroups * 8);
    const int cap = 2048 / (H > 0 ? H : 1);
    if (nblk > cap) nblk = cap;
    if (nblk < 1) nblk = 1;
    w.nblk = nblk;
    const size_t esz = (dtype == FC_BF16) ? 2 : 4;
    size_t off = 0;
    w.tokinfo = off; off += fc_align_up((size_t)H * L * 16);
    w.r = off;       off += fc_align_up((size_t)H * L * 8);
    w.keys = off;    off += fc_align_up((size_t)H * L * 8);
    w.psum = off;    off += fc_align_up((size_t)H * nblk * d * 8);
    w.ssum = off;    off += fc_align_up((size_t)H * d * 8);
    w.pmax = off;    off += fc_align_up((size_t)H * nblk * 8);
    const size_t b = (budget < L) ? (size_t)budget : 0;
    w.stage_k = off; off += fc_align_up((size_t)H * b * d * esz);
    w.stage_v = off; off += fc_align_up((size_t)H * b * d * esz);
    w.total = off;
    return w;
}

template <typename T, int D>
int launch_typed(const FcCompressArgs& a, hipStream_t s) {
    const WsLayout w = layout(a.H_k, a.L_k, a.d, a.budget, a.dtype);
    char* ws = reinterpret_cast<char*>(a.ws);
    double2* tokinfo = reinterpret_cast<double2*>(ws + w.tokinfo);
    double* r = reinterpret_cast<double*>(ws + w.r);
    uint64_t* keys = reinterpret_cast<uint64_t*>(ws + w.keys);
    double* psum = reinterpret_cast<double*>(ws + w.psum);
    double* ssum = reinterpret_cast<double*>(ws + w.ssum);
    double* pmax = reinterpret_cast<double*>(ws + w.pmax);
    double* etmp = reinterpret_cast<double*>(tokinfo);   // token info is dead once r exists
    uint4* stage_k = reinterpret_cast<uint4*>(ws + w.stage_k);
    uint4* stage_v = reinterpret_cast<uint4*>(ws + w.stage_v);
    const T* kc = reinterpret_cast<const T*>(a.k_cache);

    key_stats_kernel<T, D><<<dim3(w.nblk, a.H_k), kThreads, 0, s>>>(kc, a.head_stride, a.tok_stride,
                                                                   a.L_k, tokinfo, psum);
    FC_LAUNCH_CHECK();
    sum_partials_kernel<D><<<a.H_k, 1024, 0, s>>>(psum, w.nblk, ssum);
    FC_LAUNCH_CHECK();
    mean_sim_kernel<T, D><<<dim3(w.nblk, a.H_k), kThreads, 0, s>>>(kc, a.head_stride, a.tok_stride,
                                                                  a.L_k, tokinfo, ssum, r, pmax);
    FC_LAUNCH_CHECK();
    score_select_kernel<<<a.H_k, kSelThreads, 0, s>>>(r, a.mass, pmax, w.nblk, a.L_k, a.budget,
                                                      a.pool_k, a.lambda, etmp, keys, a.kept);
    FC_LAUNCH_CHECK();
    const int vpr = D * (int)sizeof(T) / 16;
    const int64_t hs = a.head_stride * (int64_t)sizeof(T) / 16, ts = a.tok_stride * (int64_t)sizeof(T) / 16;
    int gx = (int)(((int64_t)a.budget * vpr + kThreads * 4 - 1) / (kThreads * 4));
    gx = gx < 1 ? 1 : (gx > 4096 ? 4096 : gx);
    gather_rows_kernel<<<dim3(gx, a.H_k), kThreads, 0, s>>>(
        (const uint4*)a.k_cache, (const uint4*)a.v_cache, hs, ts, vpr, a.budget, a.kept, stage_k, stage_v);
    FC_LAUNCH_CHECK();
    copy_back_kernel<<<dim3(gx, a.H_k), kThreads, 0, s>>>((uint4*)a.k_cache, (uint4*)a.v_cache, hs, ts,
                                                          vpr, a.budget, a.kept, stage_k, stage_v);
    FC_LAUNCH_CHECK();
    return FC_OK;
}

}  // namespace

size_t fc_compress_workspace(int H_k, int L_k, int d, int budget, fc_dtype dtype) {
    return layout(H_k, L_k, d, budget, dtype).total;
}

int fc_launch_compress(const FcCompressArgs& a, hipStream_t s) {
    if (a.budget >= a.L_k) {  // cache-filling phase: nothing to drop
        const int64_t n = (int64_t)a.H_k * a.L_k;
        iota_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(a.kept, a.H_k, a.L_k);
        FC_LAUNCH_CHECK();
        return FC_OK;
    }
    if (a.dtype == FC_BF16) {
        if (a.d == 128) return launch_typed<bf16_t, 128>(a, s);
        if (a.d == 64) return launch_typed<bf16_t, 64>(a, s);
    } else {
        if (a.d == 128) return launch_typed<float, 128>(a, s);
        if (a.d == 64) return launch_typed<float, 64>(a, s);
    }
    return FC_UNSUPPORTED;
}
