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
//                  budget-th largest key; ordered compaction of the kept positions
//                  (ties: lower position wins; output ascending)
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

template <int D>
__global__ void sum_partials_kernel(const double* __restrict__ psum, int nblk,
                                    double* __restrict__ ssum) {
    const int h = blockIdx.x, e = threadIdx.x;
    double t = 0.0;
    for (int b = 0; b < nblk; ++b) t += psum[((int64_t)h * nblk + b) * D + e];
    ssum[h * D + e] = t;
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void mean_sim_kernel(
    const T* __restrict__ k_cache, int64_t head_stride, int64_t tok_stride, int L,
    const double2* __restrict__ tokinfo, const double* __restrict__ ssum,
    double* __restrict__ r) {
    constexpr int EL = D / 16;
    const int h = blockIdx.y;
    const int g = threadIdx.x / 16, u = threadIdx.x % 16;
    const T* base = k_cache + (int64_t)h * head_stride;
    double s[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) s[e] = ssum[h * D + u * EL + e];
    const double dL = (double)L;
    for (int j = blockIdx.x * kGroups + g; j < L; j += gridDim.x * kGroups) {
        double x[EL];
        load_slice<T, D>(base + (int64_t)j * tok_stride, u, x);
        double dot = 0.0;
#pragma unroll
        for (int e = 0; e < EL; ++e) dot = fma(x[e], s[e], dot);
        dot = group_sum(dot);
        if (u == 0) {
            const double2 ti = tokinfo[(int64_t)h * L + j];
            r[(int64_t)h * L + j] = (dot * ti.x - ti.y) / dL;
        }
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

__global__ __launch_bounds__(kSelThreads) void score_select_kernel(
    const double* __restrict__ r_all, const float* __restrict__ mass_all, int L, int budget,
    int pool_k, double lambda, uint64_t* __restrict__ keys_all, int32_t* __restrict__ kept_all) {
    const int h = blockIdx.x;
    const int tid = threadIdx.x;
    const double* r = r_all + (int64_t)h * L;
    const float* mass = mass_all + (int64_t)h * L;
    uint64_t* keys = keys_all + (int64_t)h * L;
    int32_t* kept = kept_all + (int64_t)h * budget;

    __shared__ double shd[kSelThreads];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wtot[2][kSelThreads / FC_WAVE];
    __shared__ uint64_t sh_prefix;
    __shared__ uint32_t sh_need;

    // Eq. (11): softmax over the token index of r
    double mx = -1.0e300;
    for (int j = tid; j < L; j += kSelThreads) mx = fmax(mx, r[j]);
    mx = block_max_d(mx, shd);
    double z = 0.0;
    for (int j = tid; j < L; j += kSelThreads) z += exp(r[j] - mx);
    z = block_sum_d(z, shd);

    // Eq. (10) + Eq. (12) -> sortable keys
    const int half = pool_k / 2;
    for (int j = tid; j < L; j += kSelThreads) {
        const int lo = (j - half > 0) ? j - half : 0;
        const int hi = (j + half < L - 1) ? j + half : L - 1;
        float imp = mass[lo];
        for (int u = lo + 1; u <= hi; ++u) imp = fmaxf(imp, mass[u]);
        const double red = exp(r[j] - mx) / z;
        const double a = lambda * (double)imp;
        const double b = (1.0 - lambda) * red;
        keys[j] = score_key(a - b);
    }
    __syncthreads();

    // radix select: the budget-th largest key, 8 bits per pass from the top
    uint64_t prefix = 0;
    uint32_t need = (uint32_t)budget;
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint64_t himask = (shift == 56) ? 0ull : (~0ull << (shift + 8));
        for (int j0 = 0; j0 < L; j0 += kSelThreads) {
            const int j = j0 + tid;
            const bool in = (j < L) && ((keys[j] & himask) == prefix);
            const uint32_t dgt = in ? (uint32_t)((keys[j] >> shift) & 255u) : 0u;
            // wave-aggregate the common case of one shared digit
            const uint64_t act = __ballot(in);
            if (act) {
                const int leader = __ffsll((long long)act) - 1;
                const uint32_t d0 = __shfl(dgt, leader, FC_WAVE);
                const uint64_t same = __ballot(in && dgt == d0);
                if (same == act) {
                    if ((tid & 63) == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(act));
                } else if (in) {
                    atomicAdd(&hist[dgt], 1u);
                }
            }
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0;
            int b = 255;
            for (; b > 0; --b) {
                if (cum + hist[b] >= need) break;
                cum += hist[b];
            }
            sh_prefix = prefix | ((uint64_t)b << shift);
            sh_need = need - cum;
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
    }
    const uint64_t thr = prefix;  // budget-th largest key; keep `need` of its copies

    // ordered compaction: position = #greater before + min(#equal before, need)
    uint32_t run_gt = 0, run_eq = 0;
    const int wave = tid / FC_WAVE, lane = tid & 63;
    for (int base = 0; base < L; base += kSelThreads * kItems) {
        const int j0 = base + tid * kItems;
        uint32_t fgt = 0, feq = 0;  // bit masks over the thread's items
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            if (j0 + i < L) {
                const uint64_t k = keys[j0 + i];
                fgt |= (k > thr) ? (1u << i) : 0u;
                feq |= (k == thr) ? (1u << i) : 0u;
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
    size_t tokinfo, r, keys, psum, ssum, stage_k, stage_v, total;
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
    uint4* stage_k = reinterpret_cast<uint4*>(ws + w.stage_k);
    uint4* stage_v = reinterpret_cast<uint4*>(ws + w.stage_v);
    const T* kc = reinterpret_cast<const T*>(a.k_cache);

    key_stats_kernel<T, D><<<dim3(w.nblk, a.H_k), kThreads, 0, s>>>(kc, a.head_stride, a.tok_stride,
                                                                   a.L_k, tokinfo, psum);
    FC_LAUNCH_CHECK();
    sum_partials_kernel<D><<<a.H_k, D, 0, s>>>(psum, w.nblk, ssum);
    FC_LAUNCH_CHECK();
    mean_sim_kernel<T, D><<<dim3(w.nblk, a.H_k), kThreads, 0, s>>>(kc, a.head_stride, a.tok_stride,
                                                                  a.L_k, tokinfo, ssum, r);
    FC_LAUNCH_CHECK();
    score_select_kernel<<<a.H_k, kSelThreads, 0, s>>>(r, a.mass, a.L_k, a.budget, a.pool_k,
                                                      a.lambda, keys, a.kept);
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
