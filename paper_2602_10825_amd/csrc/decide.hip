// Change metric, reuse decision and gather (Sec. 3.2, Eq. (5) and Eq. (8)); also the uniform
// policy of Fig. 2 (top) as a mode of the decision kernel.
//
// Three stream-ordered kernels:
//   1. decide_reduce   streaming pass over x_cur / x_prev: per block partial sums of
//                      |x_cur - x_prev| and |x_prev| in float64 (HBM-bound, 16-byte loads,
//                      contiguous segment per block, no atomics -> deterministic).
//   2. decide_finalize one block: fixed-order sum of the partials, Eq. (8) per chunk,
//                      ascending recompute list and count.
//   3. gather_chunks   block copies x_cur[idx[r]] -> x_compact[r] for r < n_recompute
//                      (the count is read on the device: no host round trip).
#include <atomic>

#include "fc_common.hpp"

namespace {

constexpr int kThreads = 256;

template <typename T>
__device__ __forceinline__ void accum_vec(const uint4& c, const uint4& p, double (&n)[4],
                                          double (&d)[4]) {
    float fc[Elem<T>::kVec], fp[Elem<T>::kVec];
    unpack16(c, fc, T());
    unpack16(p, fp, T());
#pragma unroll
    for (int e = 0; e < Elem<T>::kVec; ++e) {
        const double a = (double)fc[e];
        const double b = (double)fp[e];
        n[e & 3] += fabs(a - b);
        d[e & 3] += fabs(b);
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void decide_reduce_kernel(
    const T* __restrict__ x_cur, const T* __restrict__ x_prev, int64_t chunk_elems, int bpc,
    double* __restrict__ partial) {
    const int chunk = blockIdx.x / bpc;
    const int bi = blockIdx.x % bpc;
    const int tid = threadIdx.x;
    const T* c = x_cur + (int64_t)chunk * chunk_elems;
    const T* p = x_prev + (int64_t)chunk * chunk_elems;
    double n[4] = {0.0, 0.0, 0.0, 0.0};
    double d[4] = {0.0, 0.0, 0.0, 0.0};
    if (VEC) {
        constexpr int V = Elem<T>::kVec;
        const int64_t nvec = chunk_elems / V;
        const int64_t seg = (nvec + bpc - 1) / bpc;
        const int64_t lo = (int64_t)bi * seg;
        const int64_t hi = (lo + seg < nvec) ? lo + seg : nvec;
        const uint4* c4 = reinterpret_cast<const uint4*>(c);
        const uint4* p4 = reinterpret_cast<const uint4*>(p);
        int64_t i = lo + tid;
        for (; i + 3 * kThreads < hi; i += 4 * kThreads) {
            uint4 cv[4], pv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                cv[u] = nt_load16(c4 + i + u * kThreads);
                pv[u] = nt_load16(p4 + i + u * kThreads);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) accum_vec<T>(cv[u], pv[u], n, d);
        }
        for (; i < hi; i += kThreads) {
            const uint4 cv = nt_load16(c4 + i);
            const uint4 pv = nt_load16(p4 + i);
            accum_vec<T>(cv, pv, n, d);
        }
        if (bi == 0) {  // elements past the last whole vector
            const int64_t t = nvec * V + tid;
            if (t < chunk_elems) {
                const double a = (double)Elem<T>::to_f32(c[t]);
                const double b = (double)Elem<T>::to_f32(p[t]);
                n[0] += fabs(a - b);
                d[0] += fabs(b);
            }
        }
    } else {
        const int64_t seg = (chunk_elems + bpc - 1) / bpc;
        const int64_t lo = (int64_t)bi * seg;
        const int64_t hi = (lo + seg < chunk_elems) ? lo + seg : chunk_elems;
        for (int64_t i = lo + tid; i < hi; i += kThreads) {
            const double a = (double)Elem<T>::to_f32(c[i]);
            const double b = (double)Elem<T>::to_f32(p[i]);
            n[0] += fabs(a - b);
            d[0] += fabs(b);
        }
    }
    double ns = (n[0] + n[1]) + (n[2] + n[3]);
    double ds = (d[0] + d[1]) + (d[2] + d[3]);
    ns = wave_sum(ns);
    ds = wave_sum(ds);
    __shared__ double sh[2][kThreads / FC_WAVE];
    const int w = tid / FC_WAVE;
    if ((tid & (FC_WAVE - 1)) == 0) { sh[0][w] = ns; sh[1][w] = ds; }
    __syncthreads();
    if (tid == 0) {
        double a = 0.0, b = 0.0;
#pragma unroll
        for (int k = 0; k < kThreads / FC_WAVE; ++k) { a += sh[0][k]; b += sh[1][k]; }
        partial[2 * (int64_t)blockIdx.x] = a;
        partial[2 * (int64_t)blockIdx.x + 1] = b;
    }
}

__global__ __launch_bounds__(kThreads) void decide_finalize_kernel(
    const double* __restrict__ partial, int A, int bpc, const int32_t* __restrict__ step_idx,
    int warmup_m, double eps, double* __restrict__ acc, double* __restrict__ l1rel,
    uint8_t* __restrict__ mask, int32_t* __restrict__ idx, int32_t* __restrict__ n_rec,
    int uniform) {
    __shared__ double tot[2][FC_MAX_ACTIVE];
    __shared__ double acc_in[FC_MAX_ACTIVE];
    __shared__ int32_t step_in[FC_MAX_ACTIVE];
    const int tid = threadIdx.x;
    // the policy's own inputs are requested first, so that their latency overlaps the sums
    if (tid >= kThreads - FC_MAX_ACTIVE) {
        const int i = tid - (kThreads - FC_MAX_ACTIVE);
        if (i < A) step_in[i] = step_idx[i];
        if (i < (uniform ? 1 : A)) acc_in[i] = acc[i];
    }
    // one wavefront per chunk (chunks i, i + 4, ...): lane-strided sums of the block partials,
    // then a fixed shuffle tree -- no block-wide barriers inside the loop
    const int wave = tid / FC_WAVE, lane = tid % FC_WAVE;
    for (int i = wave; i < A; i += kThreads / FC_WAVE) {
        double a = 0.0, b = 0.0;
        for (int k = lane; k < bpc; k += FC_WAVE) {
            a += partial[2 * ((int64_t)i * bpc + k)];
            b += partial[2 * ((int64_t)i * bpc + k) + 1];
        }
        a = wave_sum(a);
        b = wave_sum(b);
        if (lane == 0) { tot[0][i] = a; tot[1][i] = b; }
    }
    __syncthreads();
    if (tid == 0 && uniform) {
        // Fig. 2, top: the chunks past warm-up share one metric, accumulator and decision
        double num = 0.0, den = 0.0;
        int old = 0;
        for (int i = 0; i < A; ++i)
            if (step_in[i] >= warmup_m) { num += tot[0][i]; den += tot[1][i]; ++old; }
        double f = 0.0;
        double rel = __longlong_as_double(0x7ff8000000000000LL);   // NaN: no chunk to measure
        if (old) {
            rel = (den == 0.0) ? __longlong_as_double(0x7ff0000000000000LL) : num / den;
            const double a = acc_in[0] + rel;
            f = (a > eps) ? 0.0 : a;
        }
        acc[0] = f;
        if (l1rel) l1rel[0] = rel;
        int cnt = 0;
        for (int i = 0; i < A; ++i) {
            const bool rec = (step_in[i] < warmup_m) || (f == 0.0);
            mask[i] = rec ? 1 : 0;
            if (rec) idx[cnt++] = i;
        }
        for (int i = cnt; i < A; ++i) idx[i] = -1;
        *n_rec = cnt;
    } else if (tid == 0) {
        int cnt = 0;
        for (int i = 0; i < A; ++i) {
            const double num = tot[0][i], den = tot[1][i];
            const double rel = (den == 0.0) ? __longlong_as_double(0x7ff0000000000000LL) : num / den;
            double f;
            if (step_in[i] < warmup_m) {
                f = 0.0;                       // case 1: warm-up steps never reuse
            } else {
                const double a = acc_in[i] + rel;
                f = (a > eps) ? 0.0 : a;       // case 2 / case 3
            }
            const bool rec = (f == 0.0);
            acc[i] = f;
            if (l1rel) l1rel[i] = rel;
            mask[i] = rec ? 1 : 0;
            if (rec) idx[cnt++] = i;
        }
        for (int i = cnt; i < A; ++i) idx[i] = -1;
        *n_rec = cnt;
    }
}

__global__ __launch_bounds__(kThreads) void gather_chunks_kernel(
    const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t chunk_vecs,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_rec) {
    const int nr = *n_rec;
    if ((int)blockIdx.y >= nr) return;
    const int r = nr - 1 - blockIdx.y;   // the metric pass read the last chunks last: they may still be cached
    const int c = idx[r];
    if ((unsigned)c >= gridDim.y) return;
    const uint4* s = src + (int64_t)c * chunk_vecs;
    uint4* d = dst + (int64_t)r * chunk_vecs;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < chunk_vecs; i += stride)
        d[i] = s[i];
}

// byte-granular variant for chunks whose size is not a multiple of 16 bytes
__global__ __launch_bounds__(kThreads) void gather_chunks_bytes_kernel(
    const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int64_t chunk_bytes,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_rec) {
    const int nr = *n_rec;
    if ((int)blockIdx.y >= nr) return;
    const int r = nr - 1 - blockIdx.y;
    const int c = idx[r];
    if ((unsigned)c >= gridDim.y) return;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < chunk_bytes; i += stride)
        dst[(int64_t)r * chunk_bytes + i] = src[(int64_t)c * chunk_bytes + i];
}

template <typename T>
int launch_typed(const FcDecideArgs& a, hipStream_t s) {
    const int bpc = fc_decide_blocks_per_chunk(a.A, a.chunk_elems, a.dtype);
    double* partial = reinterpret_cast<double*>(a.ws);
    const int64_t chunk_bytes = a.chunk_elems * (int64_t)sizeof(T);
    const bool vec = (chunk_bytes % 16 == 0) && ((uintptr_t)a.x_cur % 16 == 0) &&
                     ((uintptr_t)a.x_prev % 16 == 0);
    const dim3 grid(a.A * bpc);
    if (vec)
        decide_reduce_kernel<T, true><<<grid, kThreads, 0, s>>>(
            (const T*)a.x_cur, (const T*)a.x_prev, a.chunk_elems, bpc, partial);
    else
        decide_reduce_kernel<T, false><<<grid, kThreads, 0, s>>>(
            (const T*)a.x_cur, (const T*)a.x_prev, a.chunk_elems, bpc, partial);
    FC_LAUNCH_CHECK();
    decide_finalize_kernel<<<1, kThreads, 0, s>>>(partial, a.A, bpc, a.step_idx, a.warmup_m,
                                                  a.eps, a.acc, a.l1rel, a.mask, a.idx, a.n_rec, a.uniform);
    FC_LAUNCH_CHECK();
    if (a.x_compact) {
        const bool cvec = vec && ((uintptr_t)a.x_compact % 16 == 0);
        if (cvec) {
            const int64_t vecs = chunk_bytes / 16;
            int gx = (int)((vecs + kThreads * 4 - 1) / (kThreads * 4));
            gx = gx < 1 ? 1 : (gx > 1024 ? 1024 : gx);
            gather_chunks_kernel<<<dim3(gx, a.A), kThreads, 0, s>>>(
                (const uint4*)a.x_cur, (uint4*)a.x_compact, vecs, a.idx, a.n_rec);
        } else {
            int gx = (int)((chunk_bytes + kThreads * 16 - 1) / (kThreads * 16));
            gx = gx < 1 ? 1 : (gx > 1024 ? 1024 : gx);
            gather_chunks_bytes_kernel<<<dim3(gx, a.A), kThreads, 0, s>>>(
                (const uint8_t*)a.x_cur, (uint8_t*)a.x_compact, chunk_bytes, a.idx, a.n_rec);
        }
        FC_LAUNCH_CHECK();
    }
    return FC_OK;
}

}  // namespace

int fc_decide_blocks_per_chunk(int A, int64_t chunk_elems, fc_dtype dtype) {
    // about 8 blocks per compute unit over the whole launch, at least 4 KB of each operand
    // per block-iteration
    const int vec = (dtype == FC_BF16) ? 8 : 4;
    int64_t want = 2048 / A;
    int64_t max_useful = (chunk_elems / vec + kThreads - 1) / kThreads;
    if (max_useful < 1) max_useful = 1;
    if (want > max_useful) want = max_useful;
    if (want < 1) want = 1;
    return (int)want;
}

int fc_launch_decide(const FcDecideArgs& a, hipStream_t s) {
    return a.dtype == FC_BF16 ? launch_typed<bf16_t>(a, s) : launch_typed<float>(a, s);
}

// ---- library-owned scratch for the entry point that allocates nothing ---------------------
// The block partials of decide_reduce, for callers that cannot bring a workspace.  Every GPU
// the library runs on holds its own copy of the array for the life of the process.  In host
// code the array's name is only a stand-in for the symbol: the device address comes from
// hipGetSymbolAddress, is looked up once per device (with that device current) and is what
// the kernels receive.
static __device__ __align__(256) unsigned char scratch[FC_DECIDE_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
}  // namespace

int fc_decide_scratch(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FC_HIP_ERROR;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // racing first calls on one device look the same address up twice: harmless
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FC_HIP_ERROR;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return FC_OK;
}
