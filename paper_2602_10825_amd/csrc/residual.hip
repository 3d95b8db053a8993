// Cached-activation reuse around a skipped forward pass (Sec. 3.2: a chunk whose f is not
// zero reuses its cached activations).  The cache holds, per active chunk, output minus
// input of the layer stack at the chunk's last recompute:
//   recompute chunk c = idx[r]:  residual[c] = y_compact[r] - x[c],  out[c] = y_compact[r]
//   reused chunk c:              out[c] = x[c] + residual[c]
// One streaming pass, HBM-bound: 16-byte loads/stores, one grid row per chunk; whether a
// chunk is recomputed is read from the device-resident list, so no host round trip.
// Arithmetic: operands widened exactly to float64, one float64 add/subtract, ONE rounding to
// the storage type (bf16: float64 -> float32 toward zero with a sticky last bit, then to
// nearest even -- equal to rounding the float64 value directly).
#include "fc_common.hpp"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float f64_to_f32_round_to_odd(double v) {
    const float f = __double2float_rz(v);
    uint32_t u = __float_as_uint(f);
    if ((double)f != v) u |= 1u;   // inexact: mark "strictly between two floats"
    return __uint_as_float(u);
}

template <typename T> __device__ __forceinline__ T round_store(double v);
template <> __device__ __forceinline__ float round_store<float>(double v) { return (float)v; }
template <> __device__ __forceinline__ bf16_t round_store<bf16_t>(double v) {
    return f32_to_bf16(f64_to_f32_round_to_odd(v));
}

template <typename T>
__device__ __forceinline__ uint4 pack16(const double (&v)[Elem<T>::kVec]);
template <> __device__ __forceinline__ uint4 pack16<float>(const double (&v)[4]) {
    return make_uint4(__float_as_uint((float)v[0]), __float_as_uint((float)v[1]),
                      __float_as_uint((float)v[2]), __float_as_uint((float)v[3]));
}
template <> __device__ __forceinline__ uint4 pack16<bf16_t>(const double (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w[i] = (uint32_t)round_store<bf16_t>(v[2 * i]) | ((uint32_t)round_store<bf16_t>(v[2 * i + 1]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// compact row of chunk c in the recompute list, or -1
__device__ __forceinline__ int compact_row(const int32_t* idx, const int32_t* n_rec, int c) {
    const int R = min(*n_rec, (int)gridDim.y);   // the list never has more entries than chunks
    for (int r = 0; r < R; ++r)
        if (idx[r] == c) return r;
    return -1;
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void residual_apply_kernel(
    const T* x_cur, const T* __restrict__ y_compact, T* residual,
    T* out, int64_t chunk_elems, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ n_rec) {
    constexpr int V = Elem<T>::kVec;
    const int c = blockIdx.y;
    // without y_compact there is nothing to store: every chunk is treated as reused
    const int r = y_compact ? compact_row(idx, n_rec, c) : -1;
    const T* x = x_cur + (int64_t)c * chunk_elems;
    T* res = residual + (int64_t)c * chunk_elems;
    T* o = out + (int64_t)c * chunk_elems;
    const T* y = (r >= 0) ? y_compact + (int64_t)r * chunk_elems : nullptr;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (VEC) {
        const int64_t nvec = chunk_elems / V;
        const uint4* x4 = reinterpret_cast<const uint4*>(x);
        uint4* r4 = reinterpret_cast<uint4*>(res);
        uint4* o4 = reinterpret_cast<uint4*>(o);
        // U vectors of each operand in flight per thread: all loads of a round go out before its
        // arithmetic and stores (one vector per round left a third of the copy rate unused)
        constexpr int U = 4;
        if (r >= 0) {
            const uint4* y4 = reinterpret_cast<const uint4*>(y);
            for (int64_t i0 = t0; i0 < nvec; i0 += U * stride) {
                uint4 xv[U], yv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t i = i0 + u * stride < nvec ? i0 + u * stride : i0;
                    xv[u] = nt_load16(x4 + i);
                    yv[u] = nt_load16(y4 + i);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t i = i0 + u * stride;
                    if (i >= nvec) break;
                    float xf[V], yf[V];
                    unpack16(xv[u], xf, T());
                    unpack16(yv[u], yf, T());
                    double d[V];
#pragma unroll
                    for (int e = 0; e < V; ++e) d[e] = (double)yf[e] - (double)xf[e];
                    r4[i] = pack16<T>(d);
                    o4[i] = yv[u];
                }
            }
        } else {
            for (int64_t i0 = t0; i0 < nvec; i0 += U * stride) {
                uint4 xv[U], rv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t i = i0 + u * stride < nvec ? i0 + u * stride : i0;
                    xv[u] = nt_load16(x4 + i);
                    rv[u] = nt_load16(r4 + i);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t i = i0 + u * stride;
                    if (i >= nvec) break;
                    float xf[V], rf[V];
                    unpack16(xv[u], xf, T());
                    unpack16(rv[u], rf, T());
                    double d[V];
#pragma unroll
                    for (int e = 0; e < V; ++e) d[e] = (double)xf[e] + (double)rf[e];
                    o4[i] = pack16<T>(d);
                }
            }
        }
    }
    // scalar path: everything when unaligned, else the elements past the last whole vector
    const int64_t first = VEC ? (chunk_elems / V) * V : 0;
    for (int64_t i = first + t0; i < chunk_elems; i += stride) {
        const double xv = (double)Elem<T>::to_f32(x[i]);
        if (r >= 0) {
            res[i] = round_store<T>((double)Elem<T>::to_f32(y[i]) - xv);
            o[i] = y[i];
        } else {
            o[i] = round_store<T>(xv + (double)Elem<T>::to_f32(res[i]));
        }
    }
}

template <typename T>
int launch_typed(const FcResidualArgs& a, hipStream_t s) {
    const int64_t bytes = a.chunk_elems * (int64_t)sizeof(T);
    const bool vec = (bytes % 16 == 0) && ((uintptr_t)a.x_cur % 16 == 0) &&
                     ((uintptr_t)a.residual % 16 == 0) && ((uintptr_t)a.out % 16 == 0) &&
                     ((uintptr_t)a.y_compact % 16 == 0);
    const int64_t units = vec ? bytes / 16 : a.chunk_elems;
    int gx = (int)((units + kThreads * 4 - 1) / (kThreads * 4));
    gx = gx < 1 ? 1 : (gx > 2048 / a.A ? 2048 / a.A : gx);
    const dim3 grid(gx, a.A);
    if (vec)
        residual_apply_kernel<T, true><<<grid, kThreads, 0, s>>>(
            (const T*)a.x_cur, (const T*)a.y_compact, (T*)a.residual, (T*)a.out, a.chunk_elems,
            a.idx, a.n_rec);
    else
        residual_apply_kernel<T, false><<<grid, kThreads, 0, s>>>(
            (const T*)a.x_cur, (const T*)a.y_compact, (T*)a.residual, (T*)a.out, a.chunk_elems,
            a.idx, a.n_rec);
    FC_LAUNCH_CHECK();
    return FC_OK;
}

}  // namespace

int fc_launch_residual(const FcResidualArgs& a, hipStream_t s) {
    return a.dtype == FC_BF16 ? launch_typed<bf16_t>(a, s) : launch_typed<float>(a, s);
}
