// KV-cache compression at a chunk commit (Sec. 3.3, Eq. (10)-(12); App. C.1, C.2).
//
// Kernels, all stream-ordered, float64 arithmetic, no floating-point atomics:
//   key_stats      pass 1 over K: per token 1/max(||k||,1e-12); per block the partial sum of
//                  normalised keys
//   mean_sim       s = sum_i k^_i from the block partials (fixed order), then pass 2 over K:
//                  the token's norm again (same operations, same bits: cheaper than a side
//                  stream of 16 bytes per token written by pass 1 and read here), then
//                  r_j = (k^_j . s - k^_j . k^_j) / L, the linear-time form of the
//                  diagonal-zeroed column mean of Eq. (11); writes e_j = exp(r_j) and block
//                  partial sums of e.  (The softmax of Eq. (11) is shift-invariant and
//                  |r_j| <= 1 + 1/L, so no max is subtracted.)  Also per block the smallest
//                  and largest e and importance value: the bounds score_keys starts from.
//   score_keys     Red_j = e_j / sum e (Eq. (11)), max-pooled importance (Eq. (10)), score
//                  (Eq. (12)) -> order-preserving 64-bit keys; and the histogram of the first
//                  11 bits below the bits that all keys of the head share, which it knows
//                  before it has the keys: the score is monotone in e and in the importance,
//                  rounding included, so the same operations on their extremes bound it
//   select         per head: radix select of the budget-th largest key: a few blocks gather
//                  the chosen bin's keys in parallel, the last one to finish ends the select
//                  on them in LDS
//   write_kept     ordered compaction of the kept positions (ties: lower position wins;
//                  output ascending); blocks exchange their counts through one word each
//   compact_rows   move the kept K and V rows to positions [0, budget) IN PLACE, one pass of
//                  64-row tiles drawn from a ticket counter; a tile stores only after the
//                  lower tiles that read from its rows have loaded them
// A 16-lane group owns one token row in the two passes over K (16-byte loads, a full
// row per group), so a token's values never depend on where it sits in the launch.
#include "fc_common.hpp"

#pragma clang fp contract(off)

namespace {

constexpr int kThreads = 256;
constexpr int kGroups = kThreads / 16;
constexpr int kSelThreads = 1024;
constexpr int kItems = 8;
constexpr int kTokBlk = kThreads * kItems;   // tokens per block in the per-token kernels
constexpr int kDigitBits = 11;
constexpr int kBins = 1 << kDigitBits;
constexpr int kCand = 4096;   // candidates resolved in LDS
constexpr int kUnroll = 8;    // independent loads in flight per thread in the selection scans

// ---- bookkeeping of the in-place compaction (kernels further down) ----------------------
constexpr int kTileRows = 64;
constexpr uint32_t kSpinLimit = 1u << 24;

// Words of the sync area (uint32), all reset earlier in the call:
//   [0]                                  status word (non-zero: a bounded wait ran out)
//   [64 * (h + 1)]                       ticket counter of head h (one per 256-byte line:
//                                        atomics on one line serialise)
//   [64 * (H + 1) + h * ntile + t]       "tile t of head h has been read"
//   [64 * (H + 1) + (H + h) * ntile + t] source row of the last destination row of tile t
__host__ __device__ inline size_t sync_words(int H, int ntile) { return (size_t)2 * H * ntile + 64 * ((size_t)H + 1); }
__device__ __forceinline__ uint32_t* sync_flags(uint32_t* sync, int H, int ntile, int h) {
    return sync + 64 * (H + 1) + (int64_t)h * ntile;
}
__device__ __forceinline__ int32_t* sync_tile_last(uint32_t* sync, int H, int ntile, int h) {
    return reinterpret_cast<int32_t*>(sync + 64 * (H + 1) + (int64_t)(H + h) * ntile);
}


// ---- per-lane slice of one token row: raw bits held in registers, widened exactly ------
template <typename T, int D>
struct Slice {
    static constexpr int EL = D / 16;                       // elements per lane
    static constexpr int NW = EL * (int)sizeof(T) / 4;      // 32-bit words per lane
    typedef uint32_t raw_t __attribute__((ext_vector_type(NW)));
    static __device__ __forceinline__ raw_t load(const T* row, int u) {
        return *reinterpret_cast<const raw_t*>(row + u * EL);
    }
    static __device__ __forceinline__ void widen(const raw_t& r, double (&x)[EL]) {
        if constexpr (sizeof(T) == 8) {
#pragma unroll
            for (int e = 0; e < EL; ++e) x[e] = __hiloint2double((int)r[2 * e + 1], (int)r[2 * e]);
        } else if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                x[2 * w] = (double)bf16lo_to_f32(r[w]);
                x[2 * w + 1] = (double)bf16hi_to_f32(r[w]);
            }
        } else {
#pragma unroll
            for (int w = 0; w < NW; ++w) x[w] = (double)__uint_as_float(r[w]);
        }
    }
};

// Sixteen sums over the 16 lanes of a group, one wanted per lane (lane u wants the sum of
// v[u]): in the step for lane bit b a lane keeps the half of its values whose index has bit b
// like its own, hands the other half to its partner and adds what it receives -- 15 exchanges
// instead of the 64 of sixteen all-reduces.  Every sum is added up along the same tree over
// the lanes (bit 1, 2, 4, 8), so its bits do not depend on which token it belongs to.
__device__ __forceinline__ double group_sum_scatter(double (&v)[16], int u) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {    // lane bit 1 <-> value index bit 1: pairs (2i, 2i+1)
        const bool up = u & 1;
        const double keep = up ? v[2 * i + 1] : v[2 * i], give = up ? v[2 * i] : v[2 * i + 1];
        v[i] = keep + __shfl_xor(give, 1, 16);          // v[i] now belongs to index 2i + (u&1)
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {    // bit 2: indices 4i + (u&1) and 4i + 2 + (u&1)
        const bool up = u & 2;
        const double keep = up ? v[2 * i + 1] : v[2 * i], give = up ? v[2 * i] : v[2 * i + 1];
        v[i] = keep + __shfl_xor(give, 2, 16);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {    // bit 4
        const bool up = u & 4;
        const double keep = up ? v[2 * i + 1] : v[2 * i], give = up ? v[2 * i] : v[2 * i + 1];
        v[i] = keep + __shfl_xor(give, 4, 16);
    }
    {                                // bit 8
        const bool up = u & 8;
        const double keep = up ? v[1] : v[0], give = up ? v[0] : v[1];
        return keep + __shfl_xor(give, 8, 16);
    }
}

// Eight sums over the 16 lanes of a group: lanes u and u + 8 both end with the sum of v[u % 8]
// (three halving steps as above, then one exchange between the two halves of the group).
__device__ __forceinline__ double group_sum_scatter8(double (&v)[8], int u) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool up = u & 1;
        const double keep = up ? v[2 * i + 1] : v[2 * i], give = up ? v[2 * i] : v[2 * i + 1];
        v[i] = keep + __shfl_xor(give, 1, 16);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const bool up = u & 2;
        const double keep = up ? v[2 * i + 1] : v[2 * i], give = up ? v[2 * i] : v[2 * i + 1];
        v[i] = keep + __shfl_xor(give, 2, 16);
    }
    const bool up = u & 4;
    const double keep = up ? v[1] : v[0], give = up ? v[0] : v[1];
    const double half = keep + __shfl_xor(give, 4, 16);
    // the lower lane's term first on both sides, so both lanes get the same bits
    const double other = __shfl_xor(half, 8, 16);
    return (u & 8) ? other + half : half + other;
}

// The two passes over K.  A group of 16 lanes takes R consecutive tokens per round (R = 16 or
// 8): all R row slices are requested first, the per-token sums are reduced over the group so
// that lane u ends with token u's, and lane u finishes token u (square root, reciprocal,
// exponential) -- one token per lane instead of every lane repeating the same float64 work.
// With R = 8 the widened rows of pass 1 stay in registers for their second use.  Rows past the
// end of the head re-read its last row (branch-free loads) and are given weight zero.
template <typename T, int D, int R>
__device__ __forceinline__ void load_round(typename Slice<T, D>::raw_t (&raw)[R], const T* base,
                                           int64_t tok_stride, int j0, int L, int u) {
    const int jb = j0 < L ? j0 : L - 1;         // a round wholly past the end re-reads the last row
    const int room = L - 1 - jb;                // rows of this round that exist beyond the first
    const T* rb = base + (int64_t)jb * tok_stride;
#pragma unroll
    for (int i = 0; i < R; ++i)
        raw[i] = Slice<T, D>::load(rb + (int64_t)(i < room ? i : room) * tok_stride, u);
}

template <int R>
__device__ __forceinline__ double scatter_sum(double (&v)[R], int u) {
    if constexpr (R == 16) return group_sum_scatter(v, u);
    else return group_sum_scatter8(v, u);
}

template <typename T, int D, int R>
__global__ __launch_bounds__(kThreads) void key_stats_kernel(
    const T* __restrict__ k_cache, int64_t head_stride, int64_t tok_stride, int L,
    double* __restrict__ psum) {
    typedef Slice<T, D> S;
    constexpr int EL = S::EL;
    constexpr bool KEEP = (R == 8);   // the widened rows stay in registers between the two uses
    const int h = blockIdx.y;
    const int g = threadIdx.x / 16, u = threadIdx.x % 16;
    const T* base = k_cache + (int64_t)h * head_stride;
    double acc[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[e] = 0.0;
    const int stride = gridDim.x * kGroups * R;
    auto round = [&](typename S::raw_t (&raw)[R], int j0) {
        double xs[KEEP ? R : 1][EL];
        double part[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            double x[EL];
            S::widen(raw[i], x);
            double n2 = 0.0;
#pragma unroll
            for (int e = 0; e < EL; ++e) n2 = fma(x[e], x[e], n2);
            part[i] = n2;
            if constexpr (KEEP) {
#pragma unroll
                for (int e = 0; e < EL; ++e) xs[i][e] = x[e];
            }
        }
        const double mine = scatter_sum<R>(part, u);
        const double inv_mine = 1.0 / fmax(sqrt(mine), 1e-12);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            double inv = __shfl(inv_mine, i, 16);
            inv = (j0 + i < L) ? inv : 0.0;   // rows past the end were re-reads of the last row
            if constexpr (KEEP) {
#pragma unroll
                for (int e = 0; e < EL; ++e) acc[e] = fma(xs[i][e], inv, acc[e]);
            } else {
                double x[EL];
                asm volatile("" : "+v"(raw[i]));   // widen again here rather than keep R rows of doubles live
                S::widen(raw[i], x);
#pragma unroll
                for (int e = 0; e < EL; ++e) acc[e] = fma(x[e], inv, acc[e]);
            }
        }
    };
    // the rows of the next round are requested before the current round is worked on: with the
    // two or three wavefronts per SIMD that the registers allow, nothing else hides their latency
    // (rounds of 16 rows of wider storage would need more registers than a wavefront has)
    if constexpr (R == 8) {
        typename S::raw_t ra[R], rb[R];
        int j0 = (blockIdx.x * kGroups + g) * R;
        if (j0 < L) load_round<T, D, R>(ra, base, tok_stride, j0, L, u);
        for (; j0 < L; j0 += 2 * stride) {
            if (j0 + stride < L) load_round<T, D, R>(rb, base, tok_stride, j0 + stride, L, u);
            __builtin_amdgcn_sched_barrier(0);
            round(ra, j0);
            if (j0 + stride < L) {
                if (j0 + 2 * stride < L) load_round<T, D, R>(ra, base, tok_stride, j0 + 2 * stride, L, u);
                __builtin_amdgcn_sched_barrier(0);
                round(rb, j0 + stride);
            }
        }
    } else {
        for (int j0 = (blockIdx.x * kGroups + g) * R; j0 < L; j0 += stride) {
            typename S::raw_t raw[R];
            load_round<T, D, R>(raw, base, tok_stride, j0, L, u);
            round(raw, j0);
        }
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

// Pass 2: r_j = (k^_j . s - k^_j . k^_j) / L for every token, e_j = exp(r_j) and the block's
// partial sum of e.  Every block first adds up the head's few block partials of pass 1 itself,
// in block order (s = sum_i k^_i; the same bits in every block), which saves a launch.
template <typename T, int D, int R, typename MT>
__global__ __launch_bounds__(kThreads) void mean_sim_kernel(
    const T* __restrict__ k_cache, int64_t head_stride, int64_t tok_stride, int L,
    const double* __restrict__ psum, int npart,
    double* __restrict__ e_out, double* __restrict__ pz, const MT* __restrict__ mass_all,
    double* __restrict__ pstat, uint32_t* __restrict__ hist_all) {
    typedef Slice<T, D> S;
    constexpr int EL = S::EL;
    const int h = gridDim.y - 1 - blockIdx.y;   // pass 1 read the last heads last: they may still be cached
    const int g = threadIdx.x / 16, u = threadIdx.x % 16;
    const T* base = k_cache + (int64_t)h * head_stride;
    if (blockIdx.x == 0)   // the first-digit histogram that score_keys adds to
        for (int i = threadIdx.x; i < kBins; i += kThreads) hist_all[(int64_t)h * kBins + i] = 0u;
    __shared__ double sh_s[D];
    if (threadIdx.x < D) {
        const double* p = psum + (int64_t)h * npart * D + threadIdx.x;
        double t = 0.0;
        int b = 0;
        for (; b + 8 <= npart; b += 8) {      // eight loads in flight, added in block order
            double v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = p[(int64_t)(b + q) * D];
#pragma unroll
            for (int q = 0; q < 8; ++q) t += v[q];
        }
        for (; b < npart; ++b) t += p[(int64_t)b * D];
        sh_s[threadIdx.x] = t;
    }
    __syncthreads();
    double s[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) s[e] = sh_s[u * EL + e];
    const double dL = (double)L;
    double zsum = 0.0;
    // Bounds for score_keys (which needs the range of the scores before it has the scores):
    // smallest and largest e of this block's tokens and smallest and largest importance of a
    // slice of the head; `odd` notes a value that is not finite.
    const double kInf = __longlong_as_double(0x7ff0000000000000LL);
    double emin = kInf, emax = -kInf, mmin = kInf, mmax = -kInf;
    bool odd = false;
    // this block's share of the head's importance values: requested now, looked at after the
    // pass over the rows, so that their latency is not a prologue in front of it
    constexpr int MP = 12;
    const MT* mass = mass_all + (int64_t)h * L;
    const int mj0 = blockIdx.x * kThreads + threadIdx.x, mstride = gridDim.x * kThreads;
    MT mv[MP];
#pragma unroll
    for (int q = 0; q < MP; ++q) {
        const int j = mj0 + q * mstride;
        mv[q] = mass[j < L ? j : L - 1];
    }
    __builtin_amdgcn_sched_barrier(0);
    const int stride = gridDim.x * kGroups * R;
    for (int j0 = (blockIdx.x * kGroups + g) * R; j0 < L; j0 += stride) {
        typename S::raw_t raw[R];
        load_round<T, D, R>(raw, base, tok_stride, j0, L, u);
        const bool have = u < R && j0 + u < L;
        double part[R], part2[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            double x[EL];
            S::widen(raw[i], x);
            double dot = 0.0, n2 = 0.0;
#pragma unroll
            for (int e = 0; e < EL; ++e) dot = fma(x[e], s[e], dot);
#pragma unroll
            for (int e = 0; e < EL; ++e) n2 = fma(x[e], x[e], n2);   // as in pass 1, bit for bit
            part[i] = dot;
            part2[i] = n2;
        }
        const double mine = scatter_sum<R>(part, u);
        const double n2 = scatter_sum<R>(part2, u);
        if (have) {
            const double inv = 1.0 / fmax(sqrt(n2), 1e-12);
            const double2 ti = make_double2(inv, (n2 * inv) * inv);
            const double ej = exp((mine * ti.x - ti.y) / dL);
            e_out[(int64_t)h * L + j0 + u] = ej;
            zsum += ej;
            odd = odd || !(ej - ej == 0.0);
            emin = ej < emin ? ej : emin;
            emax = ej > emax ? ej : emax;
        }
    }
#pragma unroll
    for (int q = 0; q < MP; ++q) {
        if (mj0 + q * mstride < L) {
            const double m = (double)mv[q];
            odd = odd || !(m - m == 0.0);
            mmin = m < mmin ? m : mmin;
            mmax = m > mmax ? m : mmax;
        }
    }
    for (int j = mj0 + MP * mstride; j < L; j += mstride) {   // long heads: the rest
        const double m = (double)mass[j];
        odd = odd || !(m - m == 0.0);
        mmin = m < mmin ? m : mmin;
        mmax = m > mmax ? m : mmax;
    }
    __shared__ double shz[kThreads];
    __shared__ double shb[kThreads / FC_WAVE][4];
    __shared__ int sh_odd;
    if (threadIdx.x == 0) sh_odd = 0;
    shz[threadIdx.x] = zsum;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {   // minima and maxima: any order gives the same value
        emin = fmin(emin, __shfl_xor(emin, o, FC_WAVE));
        emax = fmax(emax, __shfl_xor(emax, o, FC_WAVE));
        mmin = fmin(mmin, __shfl_xor(mmin, o, FC_WAVE));
        mmax = fmax(mmax, __shfl_xor(mmax, o, FC_WAVE));
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        double* b = shb[threadIdx.x / FC_WAVE];
        b[0] = emin; b[1] = emax; b[2] = mmin; b[3] = mmax;
    }
    if (odd) sh_odd = 1;
    __syncthreads();
    if (threadIdx.x < 64) {   // fixed order: four strided terms per lane, then the lanes in order
        double z = (shz[threadIdx.x] + shz[threadIdx.x + 64]) + (shz[threadIdx.x + 128] + shz[threadIdx.x + 192]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) z += __shfl_down(z, o, FC_WAVE);
        if (threadIdx.x == 0) {
            pz[(int64_t)h * gridDim.x + blockIdx.x] = z;
            double* st = pstat + ((int64_t)h * gridDim.x + blockIdx.x) * 4;
            double v[4] = {shb[0][0], shb[0][1], shb[0][2], shb[0][3]};
            for (int w = 1; w < kThreads / FC_WAVE; ++w) {
                v[0] = fmin(v[0], shb[w][0]); v[1] = fmax(v[1], shb[w][1]);
                v[2] = fmin(v[2], shb[w][2]); v[3] = fmax(v[3], shb[w][3]);
            }
            // a value that is not finite anywhere in the block: the record says so with a NaN
            st[0] = sh_odd ? __longlong_as_double(0x7ff8000000000000LL) : v[0];
            st[1] = v[1]; st[2] = v[2]; st[3] = v[3];
        }
    }
}

// fixed-shape tree over the block: deterministic, and identical in every block that runs it
template <int NT>
__device__ __forceinline__ double block_sum_fixed(double v, double* sh) {
    __syncthreads();
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = NT / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    return sh[0];
}

template <int NT>
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
    for (int k = 1; k < NT / FC_WAVE; ++k) m = want_max ? (sh[k] > m ? sh[k] : m) : (sh[k] < m ? sh[k] : m);
    return m;
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

__device__ __forceinline__ uint64_t score_key(double score) {
    if (score == 0.0) score = 0.0;  // -0 -> +0
    const uint64_t b = (uint64_t)__double_as_longlong(score);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}


// ---- keys: Eq. (10)-(12) per token, fully parallel ------------------------------------
template <typename MT>   // importance as given (float) or pooled over a key group (double)
__global__ __launch_bounds__(kThreads) void score_keys_kernel(
    const double* __restrict__ e_all, const MT* __restrict__ mass_all,
    const double* __restrict__ pz_all, const double* __restrict__ pstat_all, int nblkz, int L, int pool_k,
    double lambda, uint64_t* __restrict__ keys_all, uint64_t* __restrict__ krange,
    uint32_t* __restrict__ hist_all, uint32_t* __restrict__ sync, int ntile, uint32_t* __restrict__ selsync,
    uint64_t* __restrict__ agg_all) {
    const int h = blockIdx.y, tid = threadIdx.x;
    const double* e = e_all + (int64_t)h * L;
    const MT* mass = mass_all + (int64_t)h * L;
    uint64_t* keys = keys_all + (int64_t)h * L;
    __shared__ double shd[kThreads];
    __shared__ double sh_bound[4];
    __shared__ int sh_odd;
    __shared__ uint32_t hist[kBins];
    if (blockIdx.x == 0) {   // state later kernels of this call start from: tile flags, tickets
        uint32_t* flags = sync_flags(sync, gridDim.y, ntile, h);
        for (int i = tid; i < ntile; i += kThreads) flags[i] = 0u;
        if (tid == 0) sync[64 * (h + 1)] = 0u;
        if (h == 0 && tid == 0) sync[0] = 0u;
        if (tid < 3) selsync[h * 64 + tid] = 0u;
        for (int i = tid; i < (int)gridDim.x; i += kThreads) agg_all[(int64_t)h * gridDim.x + i] = 0ull;
    }
    // Z = sum_j e_j: the block partials of the pass that wrote e, in a fixed order
    double z = 0.0;
    for (int i = tid; i < nblkz; i += kThreads) z += pz_all[(int64_t)h * nblkz + i];
    z = block_sum_fixed<kThreads>(z, shd);
    // The range of the head's scores, before any score: e and the pooled importance of every
    // token lie between the head's smallest and largest, and every operation from there to the
    // score is monotone, rounding included, so the same operations on the extremes bound the
    // scores from both sides.  All keys of the head then agree in the bits above the first in
    // which the keys of the two bounds differ; the 11 bits below are counted here.
    if (tid < FC_WAVE) {
        const double kInf = __longlong_as_double(0x7ff0000000000000LL);
        double v[4] = {kInf, -kInf, kInf, -kInf};
        bool odd = false;
        for (int i = tid; i < nblkz; i += FC_WAVE) {
            const double* st = pstat_all + ((int64_t)h * nblkz + i) * 4;
            odd = odd || (st[0] != st[0]);
            v[0] = fmin(v[0], st[0]); v[1] = fmax(v[1], st[1]);
            v[2] = fmin(v[2], st[2]); v[3] = fmax(v[3], st[3]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            v[0] = fmin(v[0], __shfl_xor(v[0], o, FC_WAVE)); v[1] = fmax(v[1], __shfl_xor(v[1], o, FC_WAVE));
            v[2] = fmin(v[2], __shfl_xor(v[2], o, FC_WAVE)); v[3] = fmax(v[3], __shfl_xor(v[3], o, FC_WAVE));
        }
        const bool any_odd = __ballot(odd) != 0ull;
        if (tid == 0) {
            sh_bound[0] = v[0]; sh_bound[1] = v[1]; sh_bound[2] = v[2]; sh_bound[3] = v[3];
            sh_odd = any_odd ? 1 : 0;
        }
    }
    __syncthreads();
    uint64_t klo = 0ull, khi = ~0ull;   // a value that is not finite somewhere: no common bits assumed
    if (!sh_odd && z - z == 0.0) {
        const double a_lo = lambda * sh_bound[2], a_hi = lambda * sh_bound[3];
        const double b_lo = (1.0 - lambda) * (sh_bound[0] / z), b_hi = (1.0 - lambda) * (sh_bound[1] / z);
        klo = score_key(a_lo - b_hi);
        khi = score_key(a_hi - b_lo);
    }
    const uint64_t kdiff = klo ^ khi;
    const int rem = kdiff ? 64 - __clzll((long long)kdiff) : 0;
    const int wbits = rem < kDigitBits ? rem : kDigitBits;
    const int shift = rem - wbits;
    if (blockIdx.x == 0 && tid == 0) { krange[2 * h] = klo; krange[2 * h + 1] = khi; }
    for (int i = tid; i < kBins; i += kThreads) hist[i] = 0u;
    __syncthreads();

    const int half = pool_k / 2;
    const int j0 = blockIdx.x * kTokBlk;
    double ev[kItems];
    MT imp[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int j = j0 + i * kThreads + tid;
        ev[i] = (j < L) ? e[j] : 0.0;
        imp[i] = (j < L) ? mass[j] : (MT)0;
    }
    for (int d = 1; d <= half; ++d) {   // Eq. (10): window max, -inf outside [0, L)
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int j = j0 + i * kThreads + tid;
            if (j < L) {
                const MT lo = (j - d >= 0) ? mass[j - d] : imp[i];
                const MT hi = (j + d < L) ? mass[j + d] : imp[i];
                const MT nb = lo > hi ? lo : hi;
                imp[i] = imp[i] > nb ? imp[i] : nb;
            }
        }
    }
    uint64_t kv[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int j = j0 + i * kThreads + tid;
        kv[i] = 0ull;
        if (j < L) {
            const double red = ev[i] / z;                    // Eq. (11)
            const double a = lambda * (double)imp[i];
            const double b = (1.0 - lambda) * red;
            kv[i] = score_key(a - b);                        // Eq. (12)
            keys[j] = kv[i];
        }
    }
    if (rem == 0) return;   // every score of the head is the same: nothing to count
#pragma unroll
    for (int i = 0; i < kItems; ++i)
        hist_add(hist, j0 + i * kThreads + tid < L, (uint32_t)(kv[i] >> shift) & ((1u << wbits) - 1u));
    __syncthreads();
    for (int i = tid; i < kBins; i += kThreads)
        if (hist[i]) atomicAdd(&hist_all[(int64_t)h * kBins + i], hist[i]);
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

// ---- per head: finish the radix select -> threshold key and the number of its copies kept.
// A few blocks per head.  Every block reads the first-digit histogram and picks the same bin.
// If that bin holds at most kCand keys (the usual case), the blocks scan the head's keys in
// parallel and append the bin's keys to a list in global memory; the block that finishes last
// (an integer count, nobody waits) pulls the list into LDS and finishes the select there.
// Otherwise -- many equal or nearly equal scores -- block 0 goes on alone with further
// histogram passes over global memory.  The list is written and read with agent-scope
// accesses: its writers may sit on other XCDs, whose L2 this block does not see.
// selsync[h * 64 + 0] = length of the list, [+1] = blocks done, [+2] = ticket of write_kept.
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const uint64_t* __restrict__ keys_all, const uint64_t* __restrict__ krange,
    const uint32_t* __restrict__ hist_all, int L, int budget, uint64_t* __restrict__ sel,
    uint64_t* __restrict__ cand_all, uint32_t* __restrict__ selsync) {
    const int h = blockIdx.y, part = blockIdx.x, nparts = gridDim.x;
    const int tid = threadIdx.x;
    const uint64_t* keys = keys_all + (int64_t)h * L;
    __shared__ uint64_t shu[kSelThreads / FC_WAVE];
    __shared__ uint32_t hist[kBins];
    __shared__ uint64_t cand[kCand];
    __shared__ uint32_t wtot[kSelThreads / FC_WAVE];
    __shared__ uint64_t sh_prefix, sh_thr;
    __shared__ uint32_t sh_need, sh_count, sh_ncand;
    __shared__ int sh_last;

    const uint64_t kmin = krange[2 * h], kmax = krange[2 * h + 1];   // bounds on the head's keys
    uint32_t need = (uint32_t)budget;
    const uint64_t diff = kmin ^ kmax;
    if (diff == 0) {   // every score is the same: keep the first `budget` positions
        if (part == 0 && tid == 0) { sel[2 * h] = kmax; sel[2 * h + 1] = need; }
        return;
    }
    int rem = 64 - __clzll((long long)diff);                   // undecided low bits
    uint64_t prefix = (rem == 64) ? 0ull : (kmax >> rem) << rem;
    {   // first digit: counted by score_keys_kernel
        const int w = rem < kDigitBits ? rem : kDigitBits;
        const int shift = rem - w;
        const int nb = 1 << w;
        for (int i = tid; i < nb; i += kSelThreads) hist[i] = hist_all[(int64_t)h * kBins + i];
        __syncthreads();
        pick_bin_parallel(hist, nb, need, wtot, prefix, shift, &sh_prefix, &sh_need, &sh_count);
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        rem = shift;
    }
    bool in_lds = false;
    uint32_t ncand = 0;
    uint32_t count = sh_count;        // keys in the bin chosen last
    if (rem > 0 && count <= (uint32_t)kCand) {
        uint64_t* cand_g = cand_all + (int64_t)h * kCand;
        uint32_t* cnt = &selsync[h * 64];
        const uint64_t hm = ~0ull << rem;
        const int lane = tid & 63;
        for (int base = part * kSelThreads * kUnroll; base < L; base += nparts * kSelThreads * kUnroll) {
            uint64_t kv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int j = base + u * kSelThreads + tid;
                kv[u] = (j < L) ? keys[j] : 0ull;
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const bool take = (kv[u] & hm) == prefix && base + u * kSelThreads + tid < L;
                const uint64_t m = __ballot(take);
                if (m == 0) continue;
                const int leader = __ffsll((long long)m) - 1;
                uint32_t at = 0;
                if (lane == leader)
                    at = __hip_atomic_fetch_add(cnt, (uint32_t)__popcll(m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                at = __shfl(at, leader, FC_WAVE);
                if (take) {
                    const uint32_t pos = at + __popcll(m & ((1ull << lane) - 1ull));
                    if (pos < (uint32_t)kCand)   // cannot be more than the histogram counted
                        __hip_atomic_store(&cand_g[pos], kv[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this block's part of the list is out
        __syncthreads();
        if (tid == 0)
            sh_last = __hip_atomic_fetch_add(&selsync[h * 64 + 1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                      (uint32_t)(nparts - 1);
        __syncthreads();
        if (!sh_last) return;
        ncand = __hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (ncand > (uint32_t)kCand) ncand = kCand;
        for (uint32_t i = tid; i < ncand; i += kSelThreads)
            cand[i] = __hip_atomic_load(&cand_g[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        in_lds = true;
    } else if (part != 0) {
        return;       // threshold already decided, or too many candidates: block 0 goes on alone
    }
    for (;;) {
        // few candidates left and still in global memory: pull them into LDS and finish there
        if (!in_lds && rem > 0 && count <= (uint32_t)kCand) {
            if (tid == 0) sh_ncand = 0;
            __syncthreads();
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
        // one candidate left in the chosen bin: it is the threshold, whatever its low bits
        if (in_lds && rem > 0 && count == 1u) {
            const uint64_t hm = ~0ull << rem;
            for (uint32_t i = tid; i < ncand; i += kSelThreads)
                if ((cand[i] & hm) == prefix) sh_thr = cand[i];
            __syncthreads();
            prefix = sh_thr;
            rem = 0;
        }
        if (rem == 0) break;
        const int w = in_lds ? (rem < 8 ? rem : 8) : (rem < kDigitBits ? rem : kDigitBits);
        const int shift = rem - w;
        const int nb = 1 << w;
        const uint64_t himask = (rem == 64) ? 0ull : (~0ull << rem);
        for (int i = tid; i < nb; i += kSelThreads) hist[i] = 0;
        __syncthreads();
        if (in_lds) {
            for (uint32_t i0 = 0; i0 < ncand; i0 += kSelThreads) {
                const uint32_t i = i0 + tid;
                const uint64_t k = (i < ncand) ? cand[i] : 0ull;
                hist_add(hist, i < ncand && (k & himask) == prefix, (uint32_t)(k >> shift) & (nb - 1));
            }
        } else {
            for (int base = 0; base < L; base += kSelThreads * kUnroll) {
                uint64_t kv[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int j = base + u * kSelThreads + tid;
                    kv[u] = (j < L) ? keys[j] : 0ull;
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
                    hist_add(hist, (kv[u] & himask) == prefix && base + u * kSelThreads + tid < L,
                             (uint32_t)(kv[u] >> shift) & (nb - 1));
            }
        }
        __syncthreads();
        pick_bin_parallel(hist, nb, need, wtot, prefix, shift, &sh_prefix, &sh_need, &sh_count);
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        count = sh_count;
        rem = shift;
    }
    if (tid == 0) {
        sel[2 * h] = prefix;
        sel[2 * h + 1] = need;
    }
}

// ---- ordered compaction of the kept positions: position = #greater before + min(#equal
//      before, need).  A block (2048 tokens, drawn from the head's ticket counter so that lower
//      blocks are always already running) publishes how many of its keys lie above and at the
//      threshold, in one 64-bit word with a valid bit, and then adds up the words of the blocks
//      below it -- they publish before they look at anyone else's, so every wait ends.
__global__ __launch_bounds__(kThreads) void write_kept_kernel(const uint64_t* __restrict__ keys_all,
                                                              const uint64_t* __restrict__ sel, int L,
                                                              int budget, int32_t* __restrict__ kept_all,
                                                              uint32_t* __restrict__ sync, int ntile,
                                                              uint32_t* __restrict__ selsync,
                                                              uint64_t* __restrict__ agg_all) {
    const int h = blockIdx.y, tid = threadIdx.x;
    const int wave = tid / FC_WAVE, lane = tid & 63;
    const uint64_t* keys = keys_all + (int64_t)h * L;
    int32_t* kept = kept_all + (int64_t)h * budget;
    int32_t* tile_last = sync_tile_last(sync, gridDim.y, ntile, h);   // for the compaction that follows
    uint64_t* agg = agg_all + (int64_t)h * gridDim.x;
    const uint64_t thr = sel[2 * h];
    const uint32_t need = (uint32_t)sel[2 * h + 1];
    __shared__ uint32_t wtot[2][kThreads / FC_WAVE];
    __shared__ int sh_blk;
    if (tid == 0)
        sh_blk = (int)__hip_atomic_fetch_add(&selsync[h * 64 + 2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int blk = sh_blk;
    const int first = blk * kTokBlk;

    const int j0 = first + tid * kItems;   // contiguous items per thread: order = position
    uint32_t fgt = 0, feq = 0;
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
    uint32_t sg = cg, se = ce;   // inclusive wave scans
#pragma unroll
    for (int o = 1; o < FC_WAVE; o <<= 1) {
        const uint32_t tg = __shfl_up(sg, o, FC_WAVE);
        const uint32_t te = __shfl_up(se, o, FC_WAVE);
        if (lane >= o) { sg += tg; se += te; }
    }
    if (lane == 63) { wtot[0][wave] = sg; wtot[1][wave] = se; }
    __syncthreads();
    uint32_t gt_before = sg - cg, eq_before = se - ce;
    uint32_t tot_g = 0, tot_e = 0;
#pragma unroll
    for (int w = 0; w < kThreads / FC_WAVE; ++w) {
        if (w < wave) { gt_before += wtot[0][w]; eq_before += wtot[1][w]; }
        tot_g += wtot[0][w];
        tot_e += wtot[1][w];
    }
    if (tid == 0)
        __hip_atomic_store(&agg[blk], (1ull << 63) | ((uint64_t)tot_g << 32) | (uint64_t)tot_e, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    // what lies below this block
    uint32_t ng = 0, ne = 0;
    bool ok = true;
    for (int b = tid; b < blk; b += kThreads) {
        uint64_t v = __hip_atomic_load(&agg[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t spins = 0;
        while (!(v >> 63)) {
            if (++spins > kSpinLimit) { ok = false; break; }
            __builtin_amdgcn_s_sleep(2);
            v = __hip_atomic_load(&agg[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        ng += (uint32_t)(v >> 32) & 0x7fffffffu;
        ne += (uint32_t)v;
    }
    if (!ok) atomicOr(&sync[0], 2u);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { ng += __shfl_xor(ng, o, FC_WAVE); ne += __shfl_xor(ne, o, FC_WAVE); }
    __syncthreads();
    if (lane == 0) { wtot[0][wave] = ng; wtot[1][wave] = ne; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kThreads / FC_WAVE; ++w) { gt_before += wtot[0][w]; eq_before += wtot[1][w]; }
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const bool g = (fgt >> i) & 1u, e = (feq >> i) & 1u;
        if (g || (e && eq_before < need)) {
            const uint32_t pos = gt_before + (eq_before < need ? eq_before : need);
            kept[pos] = j0 + i;
            if ((pos + 1) % kTileRows == 0 || (int)pos == budget - 1) tile_last[pos / kTileRows] = j0 + i;
        }
        gt_before += g ? 1u : 0u;
        eq_before += e ? 1u : 0u;
    }
}

__global__ void iota_kernel(int32_t* kept, int H, int n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)H * n) kept[i] = (int32_t)(i % n);
}

// ---- in-place compaction ---------------------------------------------------------------
// Rows are VPR 16-byte vectors; a tile is 64 destination rows of one head.  The launch is a
// fixed number of blocks that draw tiles from ONE ticket counter until it runs out: ticket g is
// tile g / H of head g % H, so a head's tiles are drawn in ascending order while consecutive
// tickets -- the tiles in flight at any moment -- are spread over all heads and seldom depend
// on one another.  Tile t may overwrite rows that a lower tile of its head still has to read
// (sources never lie below their destination): it stores only after every lower tile whose
// last source row reaches into its rows has published "read".
// A block works on its tiles in a two-stage pipeline: while the rows of the current tile are
// on their way it draws the next ticket, and it requests the next tile's row indices and what
// it needs to know about that tile's predecessors (their last source row, their flag) before it
// waits and stores the current one.  Every wait ends: a tile waits only for tiles of lower
// tickets; such a tile is held by a running block either as its current tile (published as soon
// as its rows have arrived, before that block waits for anything) or as its next tile, which
// becomes current once that block's current tile -- drawn earlier still -- is done; following
// the waits leads strictly back in drawing order, so there is no cycle.
template <int VPR>
__global__ __launch_bounds__(kThreads) void compact_rows_kernel(
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, int64_t head_stride_v,
    int64_t tok_stride_v, int H, int L, int budget, int ntile, const int32_t* __restrict__ kept_all,
    uint32_t* __restrict__ sync) {
    constexpr int LDN = kTileRows * VPR / kThreads;   // vectors per thread per matrix
    constexpr int RPP = kThreads / VPR;               // rows per pass
    __shared__ uint32_t sh_ticket;
    const int tid = threadIdx.x;
    const int lrow = tid / VPR, lcol = tid % VPR;
    const uint32_t total = (uint32_t)ntile * (uint32_t)H;
    uint32_t* ticket = &sync[64];

    // what a tile needs before its rows can be requested
    struct Tile {
        int h, tile;
        int src[LDN];
        int t_first, last_first;      // the nearest lower tile this thread looks at, its last source row
        uint32_t flag_first;          // and its "read" flag as seen when the indices were requested
    };
    auto request = [&](uint32_t g, Tile& T) {
        T.h = (int)(g % (uint32_t)H);
        T.tile = (int)(g / (uint32_t)H);
        const int32_t* kept = kept_all + (int64_t)T.h * budget;
#pragma unroll
        for (int p = 0; p < LDN; ++p) {
            const int s = T.tile * kTileRows + p * RPP + lrow;
            T.src[p] = (s < budget) ? kept[s] : -1;
        }
        T.t_first = T.tile - 1 - tid;
        T.last_first = -1;
        T.flag_first = 1u;
        if (T.t_first >= 0) {
            T.last_first = sync_tile_last(sync, H, ntile, T.h)[T.t_first];
            T.flag_first = __hip_atomic_load(&sync_flags(sync, H, ntile, T.h)[T.t_first], __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    if (tid == 0) sh_ticket = atomicAdd(ticket, 1u);
    __syncthreads();
    uint32_t g = sh_ticket;
    if (g >= total) return;
    Tile cur;
    request(g, cur);
    for (;;) {
        const int row0 = cur.tile * kTileRows;
        uint4* kh = k_cache + cur.h * head_stride_v;
        uint4* vh = v_cache + cur.h * head_stride_v;
        uint32_t* flags = sync_flags(sync, H, ntile, cur.h);
        const int32_t* tile_last = sync_tile_last(sync, H, ntile, cur.h);
        u32x4_native kr[LDN], vr[LDN];   // native vectors: the arrays stay in registers
#pragma unroll
        for (int p = 0; p < LDN; ++p) {
            const int s = row0 + p * RPP + lrow;
            if (cur.src[p] >= L) cur.src[p] = -1;   // never read outside the compressed range
            if (cur.src[p] == s) cur.src[p] = -1;   // already in place
            // branch-free: a row that is not moved loads row 0 instead (in range, value unused),
            // so that all loads of the tile are in flight together
            const int64_t a = (int64_t)(cur.src[p] >= 0 ? cur.src[p] : 0) * tok_stride_v + lcol;
            kr[p] = *reinterpret_cast<const u32x4_native*>(kh + a);
            vr[p] = *reinterpret_cast<const u32x4_native*>(vh + a);
        }
        uint32_t g_next = 0;
        if (tid == 0) g_next = atomicAdd(ticket, 1u);           // travels with the rows
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // the rows are in registers
        if (tid == 0) sh_ticket = g_next;
        __syncthreads();
        // No fence: nothing this block wrote has to become visible -- only the ORDER "rows
        // loaded, then flag" matters, and the loads have returned.  (A release fence here would
        // write back the whole L2 of this XCD, once per tile.)
        if (tid == 0) __hip_atomic_fetch_or(&flags[cur.tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        g_next = sh_ticket;
        const bool more = g_next < total;
        Tile nxt;
        if (more) request(g_next, nxt);       // on its way while this tile waits and stores
        // Lower tiles whose last (= largest) source row is >= row0 read from this tile's rows.
        // The last source rows ascend with the tile, so each thread walks down from its nearest
        // tile and stops at the first one that ends below row0.
        bool ok = true;
        int t = cur.t_first, last = cur.last_first;
        uint32_t flag = cur.flag_first;
        while (t >= 0 && last >= row0) {
            uint32_t spins = 0;
            while (flag == 0u) {
                if (++spins > kSpinLimit) { ok = false; break; }
                __builtin_amdgcn_s_sleep(2);
                flag = __hip_atomic_load(&flags[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            t -= kThreads;
            if (t >= 0) {
                last = tile_last[t];
                flag = __hip_atomic_load(&flags[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (!ok) atomicOr(&sync[0], 1u);
        __syncthreads();
#pragma unroll
        for (int p = 0; p < LDN; ++p) {
            const int s = row0 + p * RPP + lrow;
            if (cur.src[p] >= 0) {
                const int64_t a = (int64_t)s * tok_stride_v + lcol;
                // streaming stores: written the ordinary way, up to a cache's worth of these rows
                // stays behind as dirty lines and is written back during whichever kernel runs
                // next (a following pass over 460 MB of cold keys: 118 us instead of 90)
                __builtin_nontemporal_store(kr[p], reinterpret_cast<u32x4_native*>(kh + a));
                __builtin_nontemporal_store(vr[p], reinterpret_cast<u32x4_native*>(vh + a));
            }
        }
        if (!more) break;
        cur = nxt;
    }
}

// What compact_rows starts from, for the calls that bring their own kept list: zeroed tickets,
// flags and status word, and every tile's last source row.  grid = (blocks, H).
__global__ __launch_bounds__(kThreads) void prep_compact_kernel(uint32_t* __restrict__ sync, int H, int ntile,
                                                                const int32_t* __restrict__ kept_all,
                                                                int budget, int L) {
    const int h = blockIdx.y;
    uint32_t* flags = sync_flags(sync, H, ntile, h);
    int32_t* tile_last = sync_tile_last(sync, H, ntile, h);
    for (int t = blockIdx.x * kThreads + threadIdx.x; t < ntile; t += gridDim.x * kThreads) {
        flags[t] = 0u;
        const int e = ((t + 1) * kTileRows < budget ? (t + 1) * kTileRows : budget) - 1;
        tile_last[t] = kept_all[(int64_t)h * budget + e];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sync[64 * (h + 1)] = 0u;
        if (h == 0) sync[0] = 0u;
    }
    (void)L;
}

// Blocks of the compaction: two per compute unit, never more than there are tiles.  Measured on
// the MAGI-1-like cache (24 x 37440 rows of 256 bytes moved): 2048 blocks 215 us, 1024 200 us,
// 512 186 us, 256 197 us -- fewer streams in flight keep more of each open DRAM page in use.
unsigned compact_grid(int ntile, int H) {
    const int64_t tiles = (int64_t)ntile * H;
    return (unsigned)(tiles < 512 ? tiles : 512);
}

struct WsLayout {
    size_t e, keys, psum, pz, pstat, krange, hist, sel, cand, selsync, agg, sync, total;
    int nblk, nb2, ntile;
};

WsLayout layout(int H, int L, int d, int budget, fc_dtype dtype) {
    WsLayout w;
    int nblk = (L + kGroups * 16 - 1) / (kGroups * 16);   // one round of 16 tokens per group
    // three blocks per compute unit over all heads: the passes run at what the memory system
    // gives for one large read stream with small per-token side streams, whatever the launch
    // shape (512 to 4096 blocks were within 3 % of each other), so the partials stay few
    const int cap = 768 / (H > 0 ? H : 1) > 0 ? 768 / (H > 0 ? H : 1) : 1;
    if (nblk > cap) nblk = cap;
    if (nblk < 1) nblk = 1;
    w.nblk = nblk;
    w.nb2 = (L + kTokBlk - 1) / kTokBlk;
    const size_t esz = (dtype == FC_BF16) ? 2 : 4;
    size_t off = 0;
    w.e = off;       off += fc_align_up((size_t)H * L * 8);
    w.keys = off;    off += fc_align_up((size_t)H * L * 8);
    w.psum = off;    off += fc_align_up((size_t)H * nblk * d * 8);
    w.pz = off;      off += fc_align_up((size_t)H * nblk * 8);
    w.pstat = off;   off += fc_align_up((size_t)H * nblk * 32);
    w.krange = off;  off += fc_align_up((size_t)H * 16);
    w.hist = off;    off += fc_align_up((size_t)H * kBins * 4);
    w.sel = off;     off += fc_align_up((size_t)H * 16);
    w.cand = off;    off += fc_align_up((size_t)H * kCand * 8);
    w.selsync = off; off += fc_align_up((size_t)H * 64 * 4);
    w.agg = off;     off += fc_align_up((size_t)H * w.nb2 * 8);
    w.ntile = (((budget < L) ? budget : L) + kTileRows - 1) / kTileRows;
    w.sync = off;    off += fc_align_up(sync_words(H, w.ntile) * 4);
    (void)esz;
    w.total = off;
    return w;
}

template <typename T, int D, typename MT>
int launch_typed(const FcCompressArgs& a, const MT* mass, hipStream_t s, bool compact = true) {
    const WsLayout w = layout(a.H_k, a.L_k, a.d, a.budget, a.dtype);
    if constexpr (sizeof(T) <= 4) {   // (the float64 instantiation scores pooled keys: no rows to move)
        if (a.phase == 2) {           // rows only: the kept list is the caller's
            uint32_t* sync2 = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(a.ws) + w.sync);
            prep_compact_kernel<<<dim3((w.ntile + kThreads - 1) / kThreads, a.H_k), kThreads, 0, s>>>(
                sync2, a.H_k, w.ntile, a.kept, a.budget, a.L_k);
            FC_LAUNCH_CHECK();
            constexpr int VPR2 = D * (int)sizeof(T) / 16;
            const int64_t hs2 = a.head_stride * (int64_t)sizeof(T) / 16, ts2 = a.tok_stride * (int64_t)sizeof(T) / 16;
            compact_rows_kernel<VPR2><<<dim3(compact_grid(w.ntile, a.H_k)), kThreads, 0, s>>>(
                (uint4*)a.k_cache, (uint4*)a.v_cache, hs2, ts2, a.H_k, a.L_k, a.budget, w.ntile, a.kept, sync2);
            FC_LAUNCH_CHECK();
            return FC_OK;
        }
    }
    char* ws = reinterpret_cast<char*>(a.ws);
    double* e = reinterpret_cast<double*>(ws + w.e);
    uint64_t* keys = reinterpret_cast<uint64_t*>(ws + w.keys);
    double* psum = reinterpret_cast<double*>(ws + w.psum);
    double* pz = reinterpret_cast<double*>(ws + w.pz);
    double* pstat = reinterpret_cast<double*>(ws + w.pstat);
    uint64_t* krange = reinterpret_cast<uint64_t*>(ws + w.krange);
    uint32_t* hist = reinterpret_cast<uint32_t*>(ws + w.hist);
    uint64_t* sel = reinterpret_cast<uint64_t*>(ws + w.sel);
    uint64_t* cand = reinterpret_cast<uint64_t*>(ws + w.cand);
    uint32_t* selsync = reinterpret_cast<uint32_t*>(ws + w.selsync);
    uint64_t* agg = reinterpret_cast<uint64_t*>(ws + w.agg);
    uint32_t* sync = reinterpret_cast<uint32_t*>(ws + w.sync);
    const T* kc = reinterpret_cast<const T*>(a.k_cache);

    // rounds of 8 tokens for two-byte storage (the widened rows stay in registers), of 16 otherwise
    constexpr int R = sizeof(T) == 2 ? 8 : 16;
    key_stats_kernel<T, D, R><<<dim3(w.nblk, a.H_k), kThreads, 0, s>>>(kc, a.head_stride, a.tok_stride,
                                                                      a.L_k, psum);
    FC_LAUNCH_CHECK();
    mean_sim_kernel<T, D, R, MT><<<dim3(w.nblk, a.H_k), kThreads, 0, s>>>(
        kc, a.head_stride, a.tok_stride, a.L_k, psum, w.nblk, e, pz, mass, pstat, hist);
    FC_LAUNCH_CHECK();
    score_keys_kernel<MT><<<dim3(w.nb2, a.H_k), kThreads, 0, s>>>(e, mass, pz, pstat, w.nblk, a.L_k, a.pool_k,
                                                              a.lambda, keys, krange, hist, sync, w.ntile,
                                                              selsync, agg);
    FC_LAUNCH_CHECK();
    const int nparts = w.nb2 < 8 ? w.nb2 : 8;     // blocks per head that scan for the candidates
    select_kernel<<<dim3(nparts, a.H_k), kSelThreads, 0, s>>>(keys, krange, hist, a.L_k, a.budget, sel, cand,
                                                             selsync);
    FC_LAUNCH_CHECK();
    write_kept_kernel<<<dim3(w.nb2, a.H_k), kThreads, 0, s>>>(keys, sel, a.L_k, a.budget, a.kept, sync, w.ntile,
                                                              selsync, agg);
    FC_LAUNCH_CHECK();
    if (!compact || a.phase == 1) return FC_OK;   // scoring and selection only
    if constexpr (sizeof(T) <= 4) {
        constexpr int VPR = D * (int)sizeof(T) / 16;
        const int64_t hs = a.head_stride * (int64_t)sizeof(T) / 16, ts = a.tok_stride * (int64_t)sizeof(T) / 16;
        compact_rows_kernel<VPR><<<dim3(compact_grid(w.ntile, a.H_k)), kThreads, 0, s>>>(
            (uint4*)a.k_cache, (uint4*)a.v_cache, hs, ts, a.H_k, a.L_k, a.budget, w.ntile, a.kept, sync);
        FC_LAUNCH_CHECK();
    }
    return FC_OK;
}

// ---- key granularity above the token (frame- or chunk-level keys, App. D.2.1) ------------
// Group g = tokens [g*group, (g+1)*group): its key is the mean key, its importance the mean
// mass, both float64 sums in a fixed order divided by the group size and kept as float64.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void group_pool_kernel(
    const T* __restrict__ k_cache, int64_t head_stride, int64_t tok_stride, int group, int G,
    const float* __restrict__ mass, int L, double* __restrict__ k_pooled,
    double* __restrict__ mass_pooled) {
    typedef Slice<T, D> S;
    constexpr int EL = S::EL;
    const int g = blockIdx.x, h = blockIdx.y;
    const int r0 = threadIdx.x / 16, u = threadIdx.x % 16;
    const T* base = k_cache + (int64_t)h * head_stride + (int64_t)g * group * tok_stride;
    double acc[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[e] = 0.0;
    for (int r = r0; r < group; r += kGroups) {
        double x[EL];
        S::widen(S::load(base + (int64_t)r * tok_stride, u), x);
#pragma unroll
        for (int e = 0; e < EL; ++e) acc[e] += x[e];
    }
    __shared__ double sh[kGroups][D];
    __shared__ double shm[kThreads];
#pragma unroll
    for (int e = 0; e < EL; ++e) sh[r0][u * EL + e] = acc[e];
    double m = 0.0;
    for (int r = threadIdx.x; r < group; r += kThreads) m += (double)mass[(int64_t)h * L + (int64_t)g * group + r];
    m = block_sum_fixed<kThreads>(m, shm);   // includes the barrier that publishes sh
    if (threadIdx.x < D) {
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < kGroups; ++k) t += sh[k][threadIdx.x];
        k_pooled[((int64_t)h * G + g) * D + threadIdx.x] = t / (double)group;
    }
    if (threadIdx.x == 0) mass_pooled[(int64_t)h * G + g] = m / (double)group;
}

// kept groups -> kept token positions
__global__ __launch_bounds__(kThreads) void expand_groups_kernel(
    const int32_t* __restrict__ kept_groups, int n_groups, int group, int32_t* __restrict__ kept) {
    const int h = blockIdx.y;
    const int64_t n = (int64_t)n_groups * group;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads)
        kept[(int64_t)h * n + i] = kept_groups[(int64_t)h * n_groups + i / group] * group + (int32_t)(i % group);
}

struct GroupedLayout {
    size_t k_pooled, mass_pooled, kept_groups, inner, sync, total;
    int G, Bg, ntile;
};

GroupedLayout grouped_layout(int H, int L, int d, int budget, int group) {
    GroupedLayout w;
    w.G = L / group;
    w.Bg = budget / group;
    w.ntile = (budget + kTileRows - 1) / kTileRows;
    size_t off = 0;
    w.k_pooled = off;    off += fc_align_up((size_t)H * w.G * d * 8);
    w.mass_pooled = off; off += fc_align_up((size_t)H * w.G * 8);
    w.kept_groups = off; off += fc_align_up((size_t)H * (w.Bg > 0 ? w.Bg : 1) * 4);
    w.inner = off;       off += layout(H, w.G, d, w.Bg > 0 ? w.Bg : 1, FC_F32).total;
    w.sync = off;        off += fc_align_up(sync_words(H, w.ntile) * 4);
    w.total = off;
    return w;
}

template <typename T, int D>
int launch_grouped(const FcCompressArgs& a, hipStream_t s) {
    const GroupedLayout w = grouped_layout(a.H_k, a.L_k, a.d, a.budget, a.group);
    char* ws = reinterpret_cast<char*>(a.ws);
    double* k_pooled = reinterpret_cast<double*>(ws + w.k_pooled);
    double* mass_pooled = reinterpret_cast<double*>(ws + w.mass_pooled);
    int32_t* kept_groups = reinterpret_cast<int32_t*>(ws + w.kept_groups);
    uint32_t* sync = reinterpret_cast<uint32_t*>(ws + w.sync);
    group_pool_kernel<T, D><<<dim3(w.G, a.H_k), kThreads, 0, s>>>(
        (const T*)a.k_cache, a.head_stride, a.tok_stride, a.group, w.G, a.mass, a.L_k, k_pooled,
        mass_pooled);
    FC_LAUNCH_CHECK();
    // the token-level scoring and selection, run on the groups
    FcCompressArgs b = a;
    b.k_cache = k_pooled; b.v_cache = k_pooled;
    b.head_stride = (int64_t)w.G * D; b.tok_stride = D; b.dtype = FC_F32;
    b.L_k = w.G; b.budget = w.Bg; b.mass = nullptr; b.kept = kept_groups; b.ws = ws + w.inner;
    b.group = 1;
    const int st = launch_typed<double, D, double>(b, mass_pooled, s, false);
    if (st != FC_OK) return st;
    int gx = (int)(((int64_t)w.Bg * a.group + kThreads * 4 - 1) / (kThreads * 4));
    gx = gx < 1 ? 1 : (gx > 256 ? 256 : gx);
    expand_groups_kernel<<<dim3(gx, a.H_k), kThreads, 0, s>>>(kept_groups, w.Bg, a.group, a.kept);
    FC_LAUNCH_CHECK();
    prep_compact_kernel<<<dim3((w.ntile + kThreads - 1) / kThreads, a.H_k), kThreads, 0, s>>>(
        sync, a.H_k, w.ntile, a.kept, a.budget, a.L_k);
    FC_LAUNCH_CHECK();
    constexpr int VPR = D * (int)sizeof(T) / 16;
    const int64_t hs = a.head_stride * (int64_t)sizeof(T) / 16, ts = a.tok_stride * (int64_t)sizeof(T) / 16;
    compact_rows_kernel<VPR><<<dim3(compact_grid(w.ntile, a.H_k)), kThreads, 0, s>>>(
        (uint4*)a.k_cache, (uint4*)a.v_cache, hs, ts, a.H_k, a.L_k, a.budget, w.ntile, a.kept, sync);
    FC_LAUNCH_CHECK();
    return FC_OK;
}

}  // namespace

size_t fc_compress_grouped_workspace(int H_k, int L_k, int d, int budget, int group) {
    return grouped_layout(H_k, L_k, d, budget, group).total;
}

size_t fc_compress_status_offset(int H_k, int L_k, int d, int budget, int group, fc_dtype dtype) {
    if (group > 1) return grouped_layout(H_k, L_k, d, budget, group).sync;
    return layout(H_k, L_k, d, budget, dtype).sync;
}

size_t fc_compress_workspace(int H_k, int L_k, int d, int budget, fc_dtype dtype) {
    return layout(H_k, L_k, d, budget, dtype).total;
}

int fc_launch_compress(const FcCompressArgs& a, hipStream_t s) {
    if (a.budget >= a.L_k) {  // cache-filling phase: nothing to drop
        if (a.phase == 2) return FC_OK;   // every row is already in place
        const int64_t n = (int64_t)a.H_k * a.L_k;
        iota_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(a.kept, a.H_k, a.L_k);
        FC_LAUNCH_CHECK();
        return FC_OK;
    }
    if (a.group > 1) {
        if (a.dtype == FC_BF16) {
            if (a.d == 128) return launch_grouped<bf16_t, 128>(a, s);
            if (a.d == 64) return launch_grouped<bf16_t, 64>(a, s);
        } else {
            if (a.d == 128) return launch_grouped<float, 128>(a, s);
            if (a.d == 64) return launch_grouped<float, 64>(a, s);
        }
        return FC_UNSUPPORTED;
    }
    if (a.dtype == FC_BF16) {
        if (a.d == 128) return launch_typed<bf16_t, 128, float>(a, a.mass, s);
        if (a.d == 64) return launch_typed<bf16_t, 64, float>(a, a.mass, s);
    } else {
        if (a.d == 128) return launch_typed<float, 128, float>(a, a.mass, s);
        if (a.d == 64) return launch_typed<float, 64, float>(a, a.mass, s);
    }
    return FC_UNSUPPORTED;
}
