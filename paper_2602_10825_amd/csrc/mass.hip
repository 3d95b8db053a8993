// Per-key attention mass (importance), Sec. 3.3 Eq. (9), over an observation window of
// query rows (App. C.2: the last 50 tokens of the last denoising chunk).
//
//   mass[h_k, j] = 1/(W*G) * sum over rows w and the G query heads of key head h_k of
//                  softmax_j(q_w . k_j * scale), the softmax running over j < mass_len only.
//
// Two passes over the keys, both with one thread per key holding its key in registers:
//   mass_stats  per-row running (max, sum-exp) per wavefront            -> partials
//   mass_lse    per-row merge of the partials (fixed order)             -> log2-sum-exp
//   mass_cols   per key: sum over rows of exp2(s - lse), fixed order    -> mass
// Rows are processed in groups of at most 64; groups accumulate into mass in launch
// order, so the result is deterministic.  No atomics.
#include "fc_common.hpp"

namespace {

constexpr int kKeys = 256;   // keys (threads) per block
constexpr int kRowGroup = 64;
constexpr float kNegBig = -1.0e30f;
constexpr float kLog2e = 1.4426950408889634f;

template <typename T, int D>
__device__ __forceinline__ void load_key(const T* kp, float (&k)[D]) {
    constexpr int V = Elem<T>::kVec;
    const uint4* p = reinterpret_cast<const uint4*>(kp);
#pragma unroll
    for (int e = 0; e < D / V; ++e) {
        float f[V];
        unpack16(p[e], f, T());
#pragma unroll
        for (int u = 0; u < V; ++u) k[e * V + u] = f[u];
    }
}

// Row w of the current group, head h -> pointer; handles the "tail of the last compact
// block" addressing when n_rec is given.
struct RowSrc {
    const void* q; int64_t row0; int H_q; int D;
};

__device__ __forceinline__ bool resolve_rows(const FcMassArgs& a, int64_t& row0) {
    if (a.n_rec) {
        const int R = *a.n_rec;
        if (R <= 0 || a.rec_idx[R - 1] != a.A - 1) return false;
        row0 = (int64_t)R * a.L_c - a.W;
    } else {
        row0 = 0;
    }
    return true;
}

template <typename T, int D>
__device__ __forceinline__ void stage_rows(const FcMassArgs& a, int64_t row0, int w0, int nw,
                                           int h, float (*qs)[D]) {
    for (int i = threadIdx.x; i < nw * D; i += kKeys) {
        const int w = i / D, e = i % D;
        const T* src = (const T*)a.q_base + ((row0 + w0 + w) * a.H_q + h) * D + e;
        qs[w][e] = Elem<T>::to_f32(*src);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(kKeys) void mass_stats_kernel(FcMassArgs a, int w0, int nw, int np,
                                                           float* __restrict__ pm,
                                                           float* __restrict__ pl) {
    int64_t row0;
    if (!resolve_rows(a, row0)) return;
    const int h = blockIdx.y;
    const int hk = h / (a.H_q / a.H_k);
    const int tid = threadIdx.x;
    const int j = blockIdx.x * kKeys + tid;
    const bool ok = j < a.mass_len;
    __shared__ float qs[kRowGroup][D];
    stage_rows<T, D>(a, row0, w0, nw, h, qs);
    float k[D];
    load_key<T, D>((const T*)a.k_cache + (int64_t)hk * a.head_stride +
                       (int64_t)(ok ? j : a.mass_len - 1) * a.tok_stride, k);
    __syncthreads();
    const float c2 = a.scale * kLog2e;
    const int wave = tid / FC_WAVE, lane = tid % FC_WAVE;
    const int slot = blockIdx.x * (kKeys / FC_WAVE) + wave;
    for (int w = 0; w < nw; ++w) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < D; ++e) s = fmaf(k[e], qs[w][e], s);
        s = ok ? s * c2 : kNegBig;
        const float mx = wave_max_all(s);
        const float sum = wave_sum_all(__builtin_amdgcn_exp2f(s - mx));
        if (lane == 0) {
            pm[((int64_t)h * kRowGroup + w) * np + slot] = mx;
            pl[((int64_t)h * kRowGroup + w) * np + slot] = sum;
        }
    }
}

__global__ __launch_bounds__(kRowGroup) void mass_lse_kernel(const float* __restrict__ pm,
                                                             const float* __restrict__ pl, int nw,
                                                             int np, float* __restrict__ lse2,
                                                             const int32_t* n_rec,
                                                             const int32_t* rec_idx, int A) {
    if (n_rec) {
        const int R = *n_rec;
        if (R <= 0 || rec_idx[R - 1] != A - 1) return;
    }
    const int h = blockIdx.x, w = threadIdx.x;
    if (w >= nw) return;
    const float* m = pm + ((int64_t)h * kRowGroup + w) * np;
    const float* l = pl + ((int64_t)h * kRowGroup + w) * np;
    float mx = kNegBig;
    for (int i = 0; i < np; ++i) mx = fmaxf(mx, m[i]);
    float sum = 0.f;
    for (int i = 0; i < np; ++i) sum += l[i] * __builtin_amdgcn_exp2f(m[i] - mx);
    lse2[h * kRowGroup + w] = mx + __builtin_amdgcn_logf(sum);
}

template <typename T, int D>
__global__ __launch_bounds__(kKeys) void mass_cols_kernel(FcMassArgs a, int w0, int nw,
                                                          const float* __restrict__ lse2,
                                                          int first) {
    const int hk = blockIdx.y;
    const int tid = threadIdx.x;
    const int j = blockIdx.x * kKeys + tid;
    const bool ok = j < a.mass_len;
    int64_t row0;
    if (!resolve_rows(a, row0)) {
        if (ok) a.mass[(int64_t)hk * a.mass_len + j] = __uint_as_float(0x7fc00000u);
        return;
    }
    const int G = a.H_q / a.H_k;
    __shared__ float qs[kRowGroup][D];
    float k[D];
    load_key<T, D>((const T*)a.k_cache + (int64_t)hk * a.head_stride +
                       (int64_t)(ok ? j : a.mass_len - 1) * a.tok_stride, k);
    const float c2 = a.scale * kLog2e;
    float acc = 0.f;
    for (int g = 0; g < G; ++g) {
        const int h = hk * G + g;
        __syncthreads();
        stage_rows<T, D>(a, row0, w0, nw, h, qs);
        __syncthreads();
        for (int w = 0; w < nw; ++w) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < D; ++e) s = fmaf(k[e], qs[w][e], s);
            acc += __builtin_amdgcn_exp2f(s * c2 - lse2[h * kRowGroup + w]);
        }
    }
    if (ok) {
        const float contrib = acc / (float)(a.W * G);
        float* dst = a.mass + (int64_t)hk * a.mass_len + j;
        *dst = first ? contrib : *dst + contrib;
    }
}

template <typename T, int D>
int launch_typed(const FcMassArgs& a, hipStream_t s) {
    const int nkb = (a.mass_len + kKeys - 1) / kKeys;
    const int np = nkb * (kKeys / FC_WAVE);
    float* pm = reinterpret_cast<float*>(a.ws);
    float* pl = pm + (size_t)a.H_q * kRowGroup * np;
    float* lse2 = pl + (size_t)a.H_q * kRowGroup * np;
    for (int w0 = 0; w0 < a.W; w0 += kRowGroup) {
        const int nw = (a.W - w0 < kRowGroup) ? a.W - w0 : kRowGroup;
        mass_stats_kernel<T, D><<<dim3(nkb, a.H_q), kKeys, 0, s>>>(a, w0, nw, np, pm, pl);
        FC_LAUNCH_CHECK();
        mass_lse_kernel<<<a.H_q, kRowGroup, 0, s>>>(pm, pl, nw, np, lse2, a.n_rec, a.rec_idx, a.A);
        FC_LAUNCH_CHECK();
        mass_cols_kernel<T, D><<<dim3(nkb, a.H_k), kKeys, 0, s>>>(a, w0, nw, lse2, w0 == 0 ? 1 : 0);
        FC_LAUNCH_CHECK();
    }
    return FC_OK;
}

}  // namespace

size_t fc_mass_workspace(int W, int H_q, int mass_len) {
    (void)W;
    const size_t nkb = ((size_t)mass_len + kKeys - 1) / kKeys;
    const size_t np = nkb * (kKeys / FC_WAVE);
    return fc_align_up(((size_t)2 * H_q * kRowGroup * np + (size_t)H_q * kRowGroup) * sizeof(float));
}

int fc_launch_mass(const FcMassArgs& a, hipStream_t s) {
    if (a.dtype == FC_BF16) {
        if (a.d == 128) return launch_typed<bf16_t, 128>(a, s);
        if (a.d == 64) return launch_typed<bf16_t, 64>(a, s);
    } else {
        if (a.d == 128) return launch_typed<float, 128>(a, s);
        if (a.d == 64) return launch_typed<float, 64>(a, s);
    }
    return FC_UNSUPPORTED;
}
