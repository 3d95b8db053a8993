// K/V scatter of the recompute chunks into their cache slots, and the fp32 chunk-causal
// attention kernel (Sec. 3.3; softmax(q K^T d^-1/2) V with a chunk-granular causal mask).
//
// The fp32 kernel is the small-problem path (FC_F32): one thread owns one query row
// (q and the output row live in registers), a block of 128 rows shares 32-key K/V tiles
// through LDS, and the softmax is updated online once per group of 8 keys.
#include "fc_common.hpp"

namespace {

// ------------------------------------------------------------------ K/V scatter
// new [rows, H_k, d] token-major  ->  cache[h][slot + t][0..d)
__global__ __launch_bounds__(256) void scatter_kv_kernel(
    const uint4* __restrict__ k_new, const uint4* __restrict__ v_new, uint4* __restrict__ k_cache,
    uint4* __restrict__ v_cache, int64_t head_stride_v, int64_t tok_stride_v, int H_k, int vpr,
    int L_c, FcScatterArgs args) {
    const int r = blockIdx.y;
    if (r >= *args.n_rec) return;
    const int c = args.rec_idx[r];
    if ((unsigned)c >= (unsigned)args.A) return;   // not a chunk: skipped, never followed
    const int64_t slot = args.active_off[c];
    const int64_t per_chunk = (int64_t)L_c * H_k * vpr;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < per_chunk; i += stride) {
        const int v = (int)(i % vpr);
        const int h = (int)((i / vpr) % H_k);
        const int64_t t = i / ((int64_t)vpr * H_k);
        const int64_t dst = h * head_stride_v + (slot + t) * tok_stride_v + v;
        k_cache[dst] = k_new[(int64_t)r * per_chunk + i];
        v_cache[dst] = v_new[(int64_t)r * per_chunk + i];
    }
}

// ------------------------------------------------------------------ fp32 attention
constexpr int kRows = 128;   // query rows (threads) per block
constexpr int kTile = 32;    // keys per LDS tile
constexpr float kNegBig = -1.0e30f;

template <int D>
__global__ __launch_bounds__(kRows) void attend_f32_kernel(FcAttendArgs a) {
    const int r = blockIdx.z;
    if (r >= *a.n_rec) return;
    const int c = a.rec_idx[r];
    if ((unsigned)c >= (unsigned)a.A) return;
    const int h = blockIdx.y;
    const int hk = h / (a.H_q / a.H_k);
    const int tid = threadIdx.x;
    const int row_in_chunk = blockIdx.x * kRows + tid;
    const bool row_ok = row_in_chunk < a.L_c;
    const int64_t row = (int64_t)r * a.L_c + (row_ok ? row_in_chunk : a.L_c - 1);
    const float c2 = a.scale * 1.4426950408889634f;  // fold log2(e): exp(x) = exp2(x*log2 e)

    __shared__ float Ks[kTile][D];
    __shared__ float Vs[kTile][D];

    float q[D], o[D];
    {
        const float4* qp = reinterpret_cast<const float4*>((const float*)a.q + (row * a.H_q + h) * D);
#pragma unroll
        for (int e = 0; e < D / 4; ++e) {
            const float4 v = qp[e];
            q[4 * e] = v.x * c2; q[4 * e + 1] = v.y * c2; q[4 * e + 2] = v.z * c2; q[4 * e + 3] = v.w * c2;
        }
#pragma unroll
        for (int e = 0; e < D; ++e) o[e] = 0.f;
    }
    float m = kNegBig, l = 0.f;

    const float* kbase = (const float*)a.k_cache + (int64_t)hk * a.head_stride;
    const float* vbase = (const float*)a.v_cache + (int64_t)hk * a.head_stride;

    // segments of visible keys: clean region, then active chunks 0..c
    for (int sgi = -1; sgi <= c; ++sgi) {
        const int seg_start = (sgi < 0) ? 0 : a.active_off[sgi];
        const int seg_len = (sgi < 0) ? a.L_clean : a.L_c;
        for (int t0 = 0; t0 < seg_len; t0 += kTile) {
            const int nvalid = (seg_len - t0 < kTile) ? seg_len - t0 : kTile;
            __syncthreads();
            for (int i = tid; i < kTile * (D / 4); i += kRows) {
                const int j = i / (D / 4), e = i % (D / 4);
                const int jj = (j < nvalid) ? j : nvalid - 1;
                const int64_t pos = (int64_t)(seg_start + t0 + jj) * a.tok_stride;
                reinterpret_cast<float4*>(&Ks[j][0])[e] = reinterpret_cast<const float4*>(kbase + pos)[e];
                reinterpret_cast<float4*>(&Vs[j][0])[e] = reinterpret_cast<const float4*>(vbase + pos)[e];
            }
            __syncthreads();
#pragma unroll 1
            for (int g = 0; g < kTile; g += 8) {
                if (g >= nvalid) break;
                float s[8];
                float mx = m;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    float acc = 0.f;
#pragma unroll
                    for (int e = 0; e < D; ++e) acc = fmaf(q[e], Ks[g + u][e], acc);
                    s[u] = (g + u < nvalid) ? acc : kNegBig;
                    mx = fmaxf(mx, s[u]);
                }
                const float alpha = __builtin_amdgcn_exp2f(m - mx);
                float psum = 0.f;
#pragma unroll
                for (int u = 0; u < 8; ++u) { s[u] = __builtin_amdgcn_exp2f(s[u] - mx); psum += s[u]; }
                l = l * alpha + psum;
                m = mx;
#pragma unroll
                for (int e = 0; e < D; ++e) {
                    float acc = o[e] * alpha;
#pragma unroll
                    for (int u = 0; u < 8; ++u) acc = fmaf(s[u], Vs[g + u][e], acc);
                    o[e] = acc;
                }
            }
        }
    }
    if (row_ok) {
        const float inv = 1.0f / l;
        float4* op = reinterpret_cast<float4*>((float*)a.out + (row * a.H_q + h) * D);
#pragma unroll
        for (int e = 0; e < D / 4; ++e)
            op[e] = make_float4(o[4 * e] * inv, o[4 * e + 1] * inv, o[4 * e + 2] * inv, o[4 * e + 3] * inv);
        if (a.lse)
            a.lse[(int64_t)h * a.A * a.L_c + row] = (m + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    }
}

}  // namespace

int fc_launch_scatter_kv(const FcScatterArgs& a, hipStream_t s) {
    const int esz = (a.dtype == FC_BF16) ? 2 : 4;
    const int vpr = a.d * esz / 16;                       // 16-byte vectors per row
    const int64_t hs = a.head_stride * esz / 16, ts = a.tok_stride * esz / 16;
    const int64_t per_chunk = (int64_t)a.L_c * a.H_k * vpr;
    int gx = (int)((per_chunk + 256 * 4 - 1) / (256 * 4));
    gx = gx < 1 ? 1 : (gx > 2048 ? 2048 : gx);
    scatter_kv_kernel<<<dim3(gx, a.A), 256, 0, s>>>((const uint4*)a.k_new, (const uint4*)a.v_new,
                                                     (uint4*)a.k_cache, (uint4*)a.v_cache, hs, ts,
                                                     a.H_k, vpr, a.L_c, a);
    FC_LAUNCH_CHECK();
    return FC_OK;
}

int fc_launch_attend_f32(const FcAttendArgs& a, hipStream_t s) {
    const dim3 grid((a.L_c + kRows - 1) / kRows, a.H_q, a.A);
    if (a.d == 64)
        attend_f32_kernel<64><<<grid, kRows, 0, s>>>(a);
    else if (a.d == 128)
        attend_f32_kernel<128><<<grid, kRows, 0, s>>>(a);
    else
        return FC_UNSUPPORTED;
    FC_LAUNCH_CHECK();
    return FC_OK;
}
