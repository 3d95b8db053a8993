// Per-key attention mass (importance), Sec. 3.3 Eq. (9), over an observation window of
// query rows (App. C.2: the last 50 tokens of the last denoising chunk).
//
//   mass[h_k, j] = 1/(W*G) * sum over rows w and the G query heads of key head h_k of
//                  softmax_j(q_w . k_j * scale), the softmax running over j < mass_len only.
//
// Two passes over the keys (the softmax normaliser of a row is known only after all keys):
//   stats  per-row running (max, sum-exp) per block of keys             -> partials
//   lse    (between them) per row: the partials merged, fixed order     -> log2-sum-exp
//   cols   per key: sum over rows of exp2(s - lse), fixed order         -> mass
// bf16: both passes use v_mfma_f32_32x32x16_bf16 on 128-key tiles staged through LDS by
// coalesced 16-byte loads (the passes are bound by the two reads of K), each in the
// orientation that makes its reduction in-lane: stats forms S^T = K Q^T (one row per lane,
// its keys in registers: the row's max and sum need no exchange, 8 partials per row are
// merged once per block); cols forms S = Q K^T (one key per lane, the 64 padded rows in
// registers: the key's sum over rows is in-lane).  fp32: one thread per key with its key in
// registers, fp32 FMA.
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
        if (R <= 0 || R > a.A || a.rec_idx[R - 1] != a.A - 1) return false;
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
        if (R <= 0 || R > A || rec_idx[R - 1] != A - 1) return;
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


// ---- bf16: matrix-core passes -------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 128;            // keys per tile: 4 wavefronts x 32 keys
constexpr int kTilesPerBlock = 8;      // at most
constexpr int kMinTilesPerBlock = 4;
constexpr int kSpan = kTile * kTilesPerBlock;
constexpr int kNT = 256;
constexpr float kPosBig = 1.0e30f;

template <int D>
struct __attribute__((aligned(16))) MassSmem {
    // rows padded by 16 bytes: the 16-byte fragment reads of 32 consecutive rows then fall
    // on distinct LDS banks.  The 16-byte alignment is what lets them be single ds_read_b128.
    __attribute__((aligned(16))) bf16_t q[kRowGroup][D + 8];
    union __attribute__((aligned(16))) {
        __attribute__((aligned(16))) bf16_t k[kTile][D + 8];
        float merge[2][32][17];          // (max, sum) partials of the rows, after the tile loop
    };
    float lse[kRowGroup];
    float acc[kSpan];
};

template <int D>
__device__ __forceinline__ void stage_q_bf16(const FcMassArgs& a, int64_t row0, int w0, int nw, int h,
                                             bf16_t (*qs)[D + 8]) {
    constexpr int PR = D / 8;   // 16-byte pieces per row
    for (int i = threadIdx.x; i < kRowGroup * PR; i += kNT) {
        const int w = i / PR, c = i % PR;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (w < nw)
            v = *reinterpret_cast<const uint4*>((const bf16_t*)a.q_base +
                                                ((row0 + w0 + w) * a.H_q + h) * D + c * 8);
        *reinterpret_cast<uint4*>(&qs[w][c * 8]) = v;
    }
}

// 128-key tile -> registers (coalesced: consecutive threads take consecutive 16-byte pieces);
// rows past mass_len re-read the last valid row and are masked by the callers.
template <int D>
__device__ __forceinline__ void fetch_ktile(const FcMassArgs& a, const bf16_t* kh, int j0,
                                            u32x4_native (&kr)[D / 16]) {
    constexpr int PR = D / 8;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) {
        const int p = threadIdx.x + kNT * i;
        int j = j0 + p / PR;
        j = j < a.mass_len ? j : a.mass_len - 1;
        kr[i] = *reinterpret_cast<const u32x4_native*>(kh + (int64_t)j * a.tok_stride + (p % PR) * 8);
    }
}
template <int D>
__device__ __forceinline__ void store_ktile(bf16_t (*ks)[D + 8], const u32x4_native (&kr)[D / 16]) {
    constexpr int PR = D / 8;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) {
        const int p = threadIdx.x + kNT * i;
        *reinterpret_cast<u32x4_native*>(&ks[p / PR][(p % PR) * 8]) = kr[i];
    }
}

// S[row][key] for the 64 staged rows and this wavefront's 32 keys of the tile:
// s[rb][r] = row rb*32 + (r/4)*8 + (lane/32)*4 + r%4, key = wave*32 + lane%32.
template <int D>
__device__ __forceinline__ void tile_scores(const MassSmem<D>& sm, int wave, int lane,
                                            f32x16_t (&s)[2]) {
    const int n = lane & 31, half = lane >> 5;
    bf16x8_t kf[D / 16];
#pragma unroll
    for (int kb = 0; kb < D / 16; ++kb)
        kf[kb] = *reinterpret_cast<const bf16x8_t*>(&sm.k[wave * 32 + n][kb * 16 + half * 8]);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        f32x16_t c = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            const bf16x8_t qf =
                *reinterpret_cast<const bf16x8_t*>(&sm.q[rb * 32 + n][kb * 16 + half * 8]);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[kb], c, 0, 0, 0);
        }
        s[rb] = c;
    }
}

// S^T[key][row] for this wavefront's 32 keys of the tile and the 64 staged rows (the operands
// of tile_scores swapped): st[rb][r] = key wave*32 + (r/4)*8 + (lane/32)*4 + r%4,
// row rb*32 + lane%32 -- one observation row per lane, so its max and sum are in-lane.
template <int D>
__device__ __forceinline__ void tile_scores_t(const MassSmem<D>& sm, int wave, int lane,
                                              f32x16_t (&st)[2]) {
    const int n = lane & 31, half = lane >> 5;
    bf16x8_t kf[D / 16];
#pragma unroll
    for (int kb = 0; kb < D / 16; ++kb)
        kf[kb] = *reinterpret_cast<const bf16x8_t*>(&sm.k[wave * 32 + n][kb * 16 + half * 8]);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        f32x16_t c = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            const bf16x8_t qf =
                *reinterpret_cast<const bf16x8_t*>(&sm.q[rb * 32 + n][kb * 16 + half * 8]);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf, c, 0, 0, 0);
        }
        st[rb] = c;
    }
}

// Pass 1: per observation row, max and sum of exp2 over this block's span of keys.
template <int D>
__global__ __launch_bounds__(kNT, 2) void mass_stats_bf16_kernel(FcMassArgs a, int nrg, int np, int tpb,
                                                              float* __restrict__ pm,
                                                              float* __restrict__ pl) {
    int64_t row0;
    if (!resolve_rows(a, row0)) return;
    __shared__ __attribute__((aligned(16))) MassSmem<D> sm;
    const int h = blockIdx.y;
    const int hk = h / (a.H_q / a.H_k);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 31, half = lane >> 5;
    const bf16_t* kh = (const bf16_t*)a.k_cache + (int64_t)hk * a.head_stride;
    const int span = tpb * kTile;
    const int jb = blockIdx.x * span;
    const int left = a.mass_len - jb;
    const int nt = left >= span ? tpb : (left + kTile - 1) / kTile;
    const float c2 = a.scale * kLog2e;
    // row groups of 64 observation rows, one after the other: the block re-reads its own key
    // span (resident in L2 / Infinity Cache after the first group) instead of the whole K
    for (int rg = 0; rg < nrg; ++rg) {
    const int w0 = rg * kRowGroup;
    const int nw = (a.W - w0 < kRowGroup) ? a.W - w0 : kRowGroup;
    __syncthreads();
    u32x4_native kr[D / 16];
    fetch_ktile<D>(a, kh, jb, kr);             // on its way while the rows are staged
    stage_q_bf16<D>(a, row0, w0, nw, h, sm.q);
    float m[2] = {kNegBig, kNegBig}, l[2] = {0.f, 0.f};   // of row rb*32 + n over this lane's keys
    for (int t = 0; t < nt; ++t) {
        __syncthreads();
        store_ktile<D>(sm.k, kr);
        __syncthreads();
        if (t + 1 < nt) fetch_ktile<D>(a, kh, jb + (t + 1) * kTile, kr);   // never another block's tile
        f32x16_t st[2];
        tile_scores_t<D>(sm, wave, lane, st);
        const int key0 = jb + t * kTile + wave * 32 + half * 4;   // + (r/4)*8 + r%4
        if (key0 - half * 4 + 32 <= a.mass_len) {     // all 32 keys of this wavefront are real
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                float tm = st[rb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tm = fmaxf(tm, st[rb][r]);
                const float mn = fmaxf(m[rb], tm * c2);
                float acc = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc += __builtin_amdgcn_exp2f(fmaf(st[rb][r], c2, -mn));
                l[rb] = fmaf(l[rb], __builtin_amdgcn_exp2f(m[rb] - mn), acc);
                m[rb] = mn;
            }
        } else {                                      // the ragged end of the scored range
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                float tm = kNegBig;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (key0 + (r >> 2) * 8 + (r & 3) < a.mass_len) tm = fmaxf(tm, st[rb][r] * c2);
                const float mn = fmaxf(m[rb], tm);
                float acc = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (key0 + (r >> 2) * 8 + (r & 3) < a.mass_len)
                        acc += __builtin_amdgcn_exp2f(fmaf(st[rb][r], c2, -mn));
                // no real key yet (m and mn both at the floor): keep l = 0
                l[rb] = (mn > kNegBig) ? fmaf(l[rb], __builtin_amdgcn_exp2f(m[rb] - mn), acc) : 0.f;
                m[rb] = mn;
            }
        }
    }
    // merge the 8 partials of every row (4 wavefronts x 2 lane halves), in a fixed order
    __syncthreads();
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        sm.merge[0][rb * 16 + (n >> 1)][(n & 1) * 8 + wave * 2 + half] = m[rb];
        sm.merge[1][rb * 16 + (n >> 1)][(n & 1) * 8 + wave * 2 + half] = l[rb];
    }
    __syncthreads();
    if (tid < kRowGroup) {
        const int q = tid;   // rb*32 + n
        const float* mp = &sm.merge[0][(q >> 5) * 16 + ((q & 31) >> 1)][(q & 1) * 8];
        const float* lp = &sm.merge[1][(q >> 5) * 16 + ((q & 31) >> 1)][(q & 1) * 8];
        float mx = kNegBig;
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, mp[i]);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += lp[i] * __builtin_amdgcn_exp2f(mp[i] - mx);
        pm[(((int64_t)h * nrg + rg) * kRowGroup + q) * np + blockIdx.x] = mx;
        pl[(((int64_t)h * nrg + rg) * kRowGroup + q) * np + blockIdx.x] = sum;
    }
    }   // row groups
}

// Between the passes: log2-sum-exp of every observation row over all keys, from the blocks'
// partials.  One block per (row group, query head); four lanes per row take every fourth
// partial (loads batched four deep) and merge in a fixed order.  Padding rows get a huge
// normaliser: their terms vanish.
__global__ __launch_bounds__(kNT) void mass_lse_bf16_kernel(const float* __restrict__ pm,
                                                            const float* __restrict__ pl, int nrg, int np,
                                                            int W, float* __restrict__ lse2) {
    const int rg = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int w0 = rg * kRowGroup;
    const int nw = (W - w0 < kRowGroup) ? W - w0 : kRowGroup;
    const int row = tid >> 2, part = tid & 3;
    const float* m = pm + (((int64_t)h * nrg + rg) * kRowGroup + row) * np;
    const float* l = pl + (((int64_t)h * nrg + rg) * kRowGroup + row) * np;
    float mx = kNegBig, sum = 0.f;
    for (int i0 = part; i0 < np; i0 += 16) {
        float mi[4], li[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + 4 * u;
            mi[u] = i < np ? m[i] : kNegBig;
            li[u] = i < np ? l[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float mn = fmaxf(mx, mi[u]);
            sum = sum * __builtin_amdgcn_exp2f(mx - mn) + li[u] * __builtin_amdgcn_exp2f(mi[u] - mn);
            mx = mn;
        }
    }
#pragma unroll
    for (int o = 1; o < 4; o <<= 1) {
        const float mo = __shfl_xor(mx, o, FC_WAVE), so = __shfl_xor(sum, o, FC_WAVE);
        const float mn = fmaxf(mx, mo);
        // the lower lane's term first on both sides, so partners agree bit for bit
        const float lo = (part & o) ? so * __builtin_amdgcn_exp2f(mo - mn) : sum * __builtin_amdgcn_exp2f(mx - mn);
        const float hi = (part & o) ? sum * __builtin_amdgcn_exp2f(mx - mn) : so * __builtin_amdgcn_exp2f(mo - mn);
        sum = lo + hi;
        mx = mn;
    }
    if (part == 0)
        lse2[((int64_t)h * nrg + rg) * kRowGroup + row] = row < nw ? mx + __builtin_amdgcn_logf(sum) : kPosBig;
}

template <int D>
__global__ __launch_bounds__(kNT, 2) void mass_cols_bf16_kernel(FcMassArgs a, int nrg, int tpb,
                                                             const float* __restrict__ lse2) {
    const int hk = gridDim.y - 1 - blockIdx.y;   // the first pass read the last heads last: they may still be cached
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int span = tpb * kTile;
    const int jb = blockIdx.x * span;
    const int left = a.mass_len - jb;
    const int nkeys = left >= span ? span : left;
    int64_t row0;
    if (!resolve_rows(a, row0)) {
        for (int i = tid; i < nkeys; i += kNT)
            a.mass[(int64_t)hk * a.mass_len + jb + i] = __uint_as_float(0x7fc00000u);
        return;
    }
    __shared__ __attribute__((aligned(16))) MassSmem<D> sm;
    const int G = a.H_q / a.H_k;
    const bf16_t* kh = (const bf16_t*)a.k_cache + (int64_t)hk * a.head_stride;
    const int nt = (nkeys + kTile - 1) / kTile;
    const float c2 = a.scale * kLog2e;
    for (int i = tid; i < kSpan; i += kNT) sm.acc[i] = 0.f;
    for (int rg = 0; rg < nrg; ++rg)
    for (int g = 0; g < G; ++g) {
        const int h = hk * G + g;
        const int w0 = rg * kRowGroup;
        const int nw = (a.W - w0 < kRowGroup) ? a.W - w0 : kRowGroup;
        __syncthreads();
        u32x4_native kr[D / 16];
        fetch_ktile<D>(a, kh, jb, kr);         // on its way while the rows are staged
        stage_q_bf16<D>(a, row0, w0, nw, h, sm.q);
        if (tid < kRowGroup) sm.lse[tid] = lse2[((int64_t)h * nrg + rg) * kRowGroup + tid];
        __syncthreads();
        float lr[2][16];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                lr[rb][r] = sm.lse[rb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)];
        for (int t = 0; t < nt; ++t) {
            __syncthreads();
            store_ktile<D>(sm.k, kr);
            __syncthreads();
            if (t + 1 < nt) fetch_ktile<D>(a, kh, jb + (t + 1) * kTile, kr);   // never another block's tile
            f32x16_t s[2];
            tile_scores<D>(sm, wave, lane, s);
            float v = 0.f;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) v += __builtin_amdgcn_exp2f(s[rb][r] * c2 - lr[rb][r]);
            v += __shfl_xor(v, 32, FC_WAVE);
            if (lane < 32) sm.acc[t * kTile + wave * 32 + lane] += v;   // one owner per key
        }
    }
    __syncthreads();
    const float inv = 1.0f / (float)(a.W * G);
    for (int i = tid; i < nkeys; i += kNT) {
        a.mass[(int64_t)hk * a.mass_len + jb + i] = sm.acc[i] * inv;
    }
}

// ---- bf16, more than one group of 64 observation rows (frame-level queries, App. D.2.1) ------
// With many row groups the product S = Q K^T is real matrix work, and the two kernels above would
// stage every key tile again for every row group.  Here the loop order is: chunks of kNR row
// groups, inside them the key tiles of the block's span, inside a tile the row groups of the
// chunk.  A key tile is staged once per chunk and its MFMA fragments stay in registers across the
// chunk's row groups; the row groups' queries pass through a double buffer in LDS (the next group
// is on its way from L2 while the current one is multiplied; asking two groups ahead gained
// nothing), one barrier per (tile, row group).
// Both passes form S^T = K Q^T (one observation row per lane): pass 1 keeps the running (max,
// sum) of the chunk's row groups in registers, pass 2 adds exp2(s - lse) over the chunk's row
// groups per lane and reduces over the 32 rows of the lanes once per tile and chunk.
constexpr int kNR = 4;

template <int D>
struct __attribute__((aligned(16))) MassWideSmem {
    __attribute__((aligned(16))) bf16_t q[2][kRowGroup][D + 8];
    union __attribute__((aligned(16))) {
        __attribute__((aligned(16))) bf16_t k[kTile][D + 8];
        float merge[2][32][17];
    };
    float lse[kNR][kRowGroup];
    float acc[kSpan];
};

template <int D>
__device__ __forceinline__ void fetch_q_wide(const FcMassArgs& a, int64_t row0, int rg, int h,
                                             u32x4_native (&qr)[kRowGroup * (D / 8) / kNT]) {
    constexpr int PR = D / 8;
    const int w0 = rg * kRowGroup;
    const int nw = (a.W - w0 < kRowGroup) ? a.W - w0 : kRowGroup;
#pragma unroll
    for (int i = 0; i < kRowGroup * PR / kNT; ++i) {
        const int p = threadIdx.x + kNT * i;
        const int w = p / PR, c = p % PR;
        const int wc = w < nw ? w : 0;     // padding rows: a valid row is read, zeros are stored
        u32x4_native v = *reinterpret_cast<const u32x4_native*>(
            (const bf16_t*)a.q_base + ((row0 + w0 + wc) * a.H_q + h) * D + c * 8);
        if (w >= nw) v = u32x4_native{0u, 0u, 0u, 0u};
        qr[i] = v;
    }
}
template <int D>
__device__ __forceinline__ void store_q_wide(bf16_t (*qs)[D + 8], const u32x4_native (&qr)[kRowGroup * (D / 8) / kNT]) {
    constexpr int PR = D / 8;
#pragma unroll
    for (int i = 0; i < kRowGroup * PR / kNT; ++i) {
        const int p = threadIdx.x + kNT * i;
        *reinterpret_cast<u32x4_native*>(&qs[p / PR][(p % PR) * 8]) = qr[i];
    }
}

// S^T[key][row] of this wavefront's 32 keys (fragments kf, in registers) and the 64 staged rows:
// st[rb][r] = key (r/4)*8 + (lane/32)*4 + r%4 of the wavefront's 32, row rb*32 + lane%32.
template <int D>
__device__ __forceinline__ void scores_t_wide(const bf16x8_t (&kf)[D / 16], const bf16_t (*qs)[D + 8],
                                              int lane, f32x16_t (&st)[2]) {
    const int n = lane & 31, half = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        f32x16_t c = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            const bf16x8_t qf = *reinterpret_cast<const bf16x8_t*>(&qs[rb * 32 + n][kb * 16 + half * 8]);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf, c, 0, 0, 0);
        }
        st[rb] = c;
    }
}

template <int D>
__global__ __launch_bounds__(kNT, 2) void mass_stats_wide_kernel(FcMassArgs a, int nrg, int np, int tpb,
                                                              float* __restrict__ pm,
                                                              float* __restrict__ pl) {
    int64_t row0;
    if (!resolve_rows(a, row0)) return;
    __shared__ __attribute__((aligned(16))) MassWideSmem<D> sm;
    const int h = blockIdx.y;
    const int hk = h / (a.H_q / a.H_k);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 31, half = lane >> 5;
    const bf16_t* kh = (const bf16_t*)a.k_cache + (int64_t)hk * a.head_stride;
    const int span = tpb * kTile;
    const int jb = blockIdx.x * span;
    const int left = a.mass_len - jb;
    const int nt = left >= span ? tpb : (left + kTile - 1) / kTile;
    const float c2 = a.scale * kLog2e;
    for (int rc = 0; rc < nrg; rc += kNR) {
        const int ncr = nrg - rc < kNR ? nrg - rc : kNR;
        float m[kNR][2], l[kNR][2];
#pragma unroll
        for (int g = 0; g < kNR; ++g) { m[g][0] = m[g][1] = kNegBig; l[g][0] = l[g][1] = 0.f; }
        u32x4_native kr[D / 16];
        u32x4_native qr[kRowGroup * (D / 8) / kNT];
        fetch_ktile<D>(a, kh, jb, kr);
        fetch_q_wide<D>(a, row0, rc, h, qr);
        bf16x8_t kf[D / 16];
        for (int t = 0; t < nt; ++t) {
            __syncthreads();                       // the last tile's fragments are in registers everywhere
            store_ktile<D>(sm.k, kr);
            if (t + 1 < nt) fetch_ktile<D>(a, kh, jb + (t + 1) * kTile, kr);
            const int key0 = jb + t * kTile + wave * 32 + half * 4;   // + (r/4)*8 + r%4
            const bool full = key0 - half * 4 + 32 <= a.mass_len;
#pragma unroll
            for (int g = 0; g < kNR; ++g) {
                if (g < ncr) {                     // uniform over the block
                    const int buf = (t * ncr + g) & 1;
                    store_q_wide<D>(sm.q[buf], qr);
                    __syncthreads();
                    if (g == 0) {
#pragma unroll
                        for (int kb = 0; kb < D / 16; ++kb)
                            kf[kb] = *reinterpret_cast<const bf16x8_t*>(&sm.k[wave * 32 + n][kb * 16 + half * 8]);
                    }
                    if (!(t == nt - 1 && g == ncr - 1))     // the next pair's queries, on their way from L2
                        fetch_q_wide<D>(a, row0, rc + (g + 1) % ncr, h, qr);
                    f32x16_t st[2];
                    scores_t_wide<D>(kf, sm.q[buf], lane, st);
                    if (full) {                    // all 32 keys of this wavefront are real
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb) {
                            float tm = st[rb][0];
#pragma unroll
                            for (int r = 1; r < 16; ++r) tm = fmaxf(tm, st[rb][r]);
                            const float mn = fmaxf(m[g][rb], tm * c2);
                            float acc = 0.f;
#pragma unroll
                            for (int r = 0; r < 16; ++r) acc += __builtin_amdgcn_exp2f(fmaf(st[rb][r], c2, -mn));
                            l[g][rb] = fmaf(l[g][rb], __builtin_amdgcn_exp2f(m[g][rb] - mn), acc);
                            m[g][rb] = mn;
                        }
                    } else {                       // the ragged end of the scored range
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb) {
                            float tm = kNegBig;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (key0 + (r >> 2) * 8 + (r & 3) < a.mass_len) tm = fmaxf(tm, st[rb][r] * c2);
                            const float mn = fmaxf(m[g][rb], tm);
                            float acc = 0.f;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (key0 + (r >> 2) * 8 + (r & 3) < a.mass_len)
                                    acc += __builtin_amdgcn_exp2f(fmaf(st[rb][r], c2, -mn));
                            // no real key yet (m and mn both at the floor): keep l = 0
                            l[g][rb] = (mn > kNegBig) ? fmaf(l[g][rb], __builtin_amdgcn_exp2f(m[g][rb] - mn), acc) : 0.f;
                            m[g][rb] = mn;
                        }
                    }
                }
            }
        }
        // merge the 8 partials of every row (4 wavefronts x 2 lane halves), in a fixed order
#pragma unroll
        for (int g = 0; g < kNR; ++g) {
            if (g < ncr) {
                __syncthreads();
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    sm.merge[0][rb * 16 + (n >> 1)][(n & 1) * 8 + wave * 2 + half] = m[g][rb];
                    sm.merge[1][rb * 16 + (n >> 1)][(n & 1) * 8 + wave * 2 + half] = l[g][rb];
                }
                __syncthreads();
                if (tid < kRowGroup) {
                    const int q = tid;   // rb*32 + n
                    const float* mp = &sm.merge[0][(q >> 5) * 16 + ((q & 31) >> 1)][(q & 1) * 8];
                    const float* lp = &sm.merge[1][(q >> 5) * 16 + ((q & 31) >> 1)][(q & 1) * 8];
                    float mx = kNegBig;
#pragma unroll
                    for (int i = 0; i < 8; ++i) mx = fmaxf(mx, mp[i]);
                    float sum = 0.f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) sum += lp[i] * __builtin_amdgcn_exp2f(mp[i] - mx);
                    pm[(((int64_t)h * nrg + rc + g) * kRowGroup + q) * np + blockIdx.x] = mx;
                    pl[(((int64_t)h * nrg + rc + g) * kRowGroup + q) * np + blockIdx.x] = sum;
                }
            }
        }
        __syncthreads();     // the merge area is the key tile of the next chunk
    }
}

template <int D>
__global__ __launch_bounds__(kNT, 2) void mass_cols_wide_kernel(FcMassArgs a, int nrg, int tpb,
                                                             const float* __restrict__ lse2) {
    const int hk = gridDim.y - 1 - blockIdx.y;   // the first pass read the last heads last
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 31, half = lane >> 5;
    const int span = tpb * kTile;
    const int jb = blockIdx.x * span;
    const int left = a.mass_len - jb;
    const int nkeys = left >= span ? span : left;
    int64_t row0;
    if (!resolve_rows(a, row0)) {
        for (int i = tid; i < nkeys; i += kNT)
            a.mass[(int64_t)hk * a.mass_len + jb + i] = __uint_as_float(0x7fc00000u);
        return;
    }
    __shared__ __attribute__((aligned(16))) MassWideSmem<D> sm;
    const int G = a.H_q / a.H_k;
    const bf16_t* kh = (const bf16_t*)a.k_cache + (int64_t)hk * a.head_stride;
    const int nt = (nkeys + kTile - 1) / kTile;
    const float c2 = a.scale * kLog2e;
    for (int i = tid; i < kSpan; i += kNT) sm.acc[i] = 0.f;
    for (int gq = 0; gq < G; ++gq) {
        const int h = hk * G + gq;
        for (int rc = 0; rc < nrg; rc += kNR) {
            const int ncr = nrg - rc < kNR ? nrg - rc : kNR;
            __syncthreads();                       // the previous chunk's normalisers are no longer read
            for (int i = tid; i < ncr * kRowGroup; i += kNT)
                sm.lse[i / kRowGroup][i % kRowGroup] = lse2[((int64_t)h * nrg + rc) * kRowGroup + i];
            u32x4_native kr[D / 16];
            u32x4_native qr[kRowGroup * (D / 8) / kNT];
            fetch_ktile<D>(a, kh, jb, kr);
            fetch_q_wide<D>(a, row0, rc, h, qr);
            bf16x8_t kf[D / 16];
            for (int t = 0; t < nt; ++t) {
                __syncthreads();
                store_ktile<D>(sm.k, kr);
                if (t + 1 < nt) fetch_ktile<D>(a, kh, jb + (t + 1) * kTile, kr);
                float ka[16];                      // this lane's rows' share of the 16 keys it sees
#pragma unroll
                for (int r = 0; r < 16; ++r) ka[r] = 0.f;
#pragma unroll
                for (int g = 0; g < kNR; ++g) {
                    if (g < ncr) {
                        const int buf = (t * ncr + g) & 1;
                        store_q_wide<D>(sm.q[buf], qr);
                        __syncthreads();
                        if (g == 0) {
#pragma unroll
                            for (int kb = 0; kb < D / 16; ++kb)
                                kf[kb] = *reinterpret_cast<const bf16x8_t*>(&sm.k[wave * 32 + n][kb * 16 + half * 8]);
                        }
                        if (!(t == nt - 1 && g == ncr - 1))
                            fetch_q_wide<D>(a, row0, rc + (g + 1) % ncr, h, qr);
                        f32x16_t st[2];
                        scores_t_wide<D>(kf, sm.q[buf], lane, st);
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb) {
                            const float ls = sm.lse[g][rb * 32 + n];   // padding rows: huge, their terms vanish
#pragma unroll
                            for (int r = 0; r < 16; ++r) ka[r] += __builtin_amdgcn_exp2f(fmaf(st[rb][r], c2, -ls));
                        }
                    }
                }
                // over the 32 rows of the lanes (fixed exchange pattern), then one owner per key
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = ka[r];
#pragma unroll
                    for (int o = 1; o < 32; o <<= 1) v += __shfl_xor(v, o, FC_WAVE);
                    ka[r] = v;
                }
                if (n == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sm.acc[t * kTile + wave * 32 + (r >> 2) * 8 + half * 4 + (r & 3)] += ka[r];
                }
            }
        }
    }
    __syncthreads();
    const float inv = 1.0f / (float)(a.W * G);
    for (int i = tid; i < nkeys; i += kNT) a.mass[(int64_t)hk * a.mass_len + jb + i] = sm.acc[i] * inv;
}

// Tiles per block, 4 to 8: blocks of one launch take about the same time, so they run in rounds
// of as many blocks as the chip holds (two per compute unit); the span is chosen so that the
// last round is as full as possible (the MAGI-1-like layer: 3528 blocks of 4 tiles fill 6.9
// rounds of 512, where 1776 blocks of 8 tiles left the fourth round half empty).
inline int mass_tiles_per_block(int mass_len, int heads) {
    const int64_t slots = 512;
    int best = kTilesPerBlock;
    double best_eff = -1.0;
    for (int tpb = kTilesPerBlock; tpb >= kMinTilesPerBlock; --tpb) {
        const int64_t blocks = (int64_t)heads * ((mass_len + tpb * kTile - 1) / (tpb * kTile));
        const int64_t rounds = (blocks + slots - 1) / slots;
        const double eff = (double)blocks / (double)(rounds * slots);
        if (eff > best_eff + 0.02) { best_eff = eff; best = tpb; }   // longer spans unless clearly fuller
    }
    return best;
}

template <int D>
int launch_bf16(const FcMassArgs& a, hipStream_t s) {
    const int tpb = mass_tiles_per_block(a.mass_len, a.H_q);
    const int np = (a.mass_len + tpb * kTile - 1) / (tpb * kTile);
    const int nrg = (a.W + kRowGroup - 1) / kRowGroup;
    float* pm = reinterpret_cast<float*>(a.ws);
    float* pl = pm + (size_t)a.H_q * nrg * kRowGroup * np;
    float* lse2 = pl + (size_t)a.H_q * nrg * kRowGroup * np;
    if (nrg > 1)
        mass_stats_wide_kernel<D><<<dim3(np, a.H_q), kNT, 0, s>>>(a, nrg, np, tpb, pm, pl);
    else
        mass_stats_bf16_kernel<D><<<dim3(np, a.H_q), kNT, 0, s>>>(a, nrg, np, tpb, pm, pl);
    FC_LAUNCH_CHECK();
    mass_lse_bf16_kernel<<<dim3(nrg, a.H_q), kNT, 0, s>>>(pm, pl, nrg, np, a.W, lse2);
    FC_LAUNCH_CHECK();
    if (nrg > 1)
        mass_cols_wide_kernel<D><<<dim3(np, a.H_k), kNT, 0, s>>>(a, nrg, tpb, lse2);
    else
        mass_cols_bf16_kernel<D><<<dim3(np, a.H_k), kNT, 0, s>>>(a, nrg, tpb, lse2);
    FC_LAUNCH_CHECK();
    return FC_OK;
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
    // fp32 path: one row group at a time, a partial per wavefront of 64 keys
    const size_t nkb = ((size_t)mass_len + kKeys - 1) / kKeys;
    const size_t np = nkb * (kKeys / FC_WAVE);
    const size_t f32 = ((size_t)2 * H_q * kRowGroup * np + (size_t)H_q * kRowGroup) * sizeof(float);
    // bf16 path: all row groups in one launch, a partial per block span of keys
    const size_t nrg = ((size_t)(W > 0 ? W : 1) + kRowGroup - 1) / kRowGroup;
    const size_t nps = ((size_t)mass_len + kMinTilesPerBlock * kTile - 1) / (kMinTilesPerBlock * kTile);
    const size_t bf16 = ((size_t)2 * H_q * nrg * kRowGroup * nps + (size_t)H_q * nrg * kRowGroup) * sizeof(float);
    return fc_align_up(f32 > bf16 ? f32 : bf16);
}

int fc_launch_mass(const FcMassArgs& a, hipStream_t s) {
    if (a.dtype == FC_BF16) {
        if (a.d == 128) return launch_bf16<128>(a, s);
        if (a.d == 64) return launch_bf16<64>(a, s);
    } else {
        if (a.d == 128) return launch_typed<float, 128>(a, s);
        if (a.d == 64) return launch_typed<float, 64>(a, s);
    }
    return FC_UNSUPPORTED;
}
