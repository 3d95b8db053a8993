// Shared device helpers and the internal launcher interface of libflowcache (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flowcache.h"

#define FC_WAVE 64

typedef uint16_t bf16_t;  // raw bfloat16 bits

// ---- bf16 <-> f32 -------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) {
    return __uint_as_float(pair & 0xffff0000u);
}
// round-to-nearest-even, finite inputs
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kVec = 4;  // elements per 16-byte load
    __device__ static __forceinline__ float to_f32(float v) { return v; }
    __device__ static __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int kVec = 8;
    __device__ static __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
    __device__ static __forceinline__ bf16_t from_f32(float v) { return f32_to_bf16(v); }
};

// Unpack one 16-byte vector into kVec floats.
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[4], float) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[8], bf16_t) {
    f[0] = bf16lo_to_f32(v.x); f[1] = bf16hi_to_f32(v.x);
    f[2] = bf16lo_to_f32(v.y); f[3] = bf16hi_to_f32(v.y);
    f[4] = bf16lo_to_f32(v.z); f[5] = bf16hi_to_f32(v.z);
    f[6] = bf16lo_to_f32(v.w); f[7] = bf16hi_to_f32(v.w);
}

// 16-byte streaming load (data that is read once: keep it out of the way of resident lines)
typedef uint32_t u32x4_native __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load16(const uint4* p) {
    const u32x4_native v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_native*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- wavefront (64 lanes) reductions --------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, FC_WAVE);
    return v;  // valid in lane 0
}
__device__ __forceinline__ float wave_max_all(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, FC_WAVE));
    return v;
}
__device__ __forceinline__ float wave_sum_all(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, FC_WAVE);
    return v;
}

static inline size_t fc_align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

#define FC_HIP_TRY(expr)                          \
    do {                                          \
        hipError_t e__ = (expr);                  \
        if (e__ != hipSuccess) return FC_HIP_ERROR; \
    } while (0)

#define FC_LAUNCH_CHECK()                                   \
    do {                                                    \
        if (hipGetLastError() != hipSuccess) return FC_HIP_ERROR; \
    } while (0)

// ---- internal launchers (argument checking is done by the callers in api.hip) -------
struct FcDecideArgs {
    const void* x_cur; const void* x_prev; fc_dtype dtype; int A; int64_t chunk_elems;
    const int32_t* step_idx; int warmup_m; double eps; double* acc; double* l1rel;
    uint8_t* mask; int32_t* idx; int32_t* n_rec; void* x_compact; void* ws;
    int uniform;   // 1: one shared accumulator acc[0] / l1rel[0] for all chunks past warm-up
};
int fc_decide_blocks_per_chunk(int A, int64_t chunk_elems, fc_dtype dtype);
int fc_launch_decide(const FcDecideArgs& a, hipStream_t s);
// device address, on the current device, of the library's own FC_DECIDE_SCRATCH_BYTES of scratch
int fc_decide_scratch(void** ptr);

struct FcResidualArgs {
    const void* x_cur; const void* y_compact; void* residual; void* out; fc_dtype dtype;
    int A; int64_t chunk_elems; const int32_t* idx; const int32_t* n_rec;
};
int fc_launch_residual(const FcResidualArgs& a, hipStream_t s);

struct FcAttendArgs {
    const void* q; void* out; float* lse;
    const void* k_cache; const void* v_cache; int64_t head_stride; int64_t tok_stride;
    fc_dtype dtype; int H_q; int H_k; int d; int L_c; int L_clean; int A;
    int32_t active_off[FC_MAX_ACTIVE];
    const int32_t* rec_idx; const int32_t* n_rec; float scale;
};
int fc_launch_attend_f32(const FcAttendArgs& a, hipStream_t s);
int fc_launch_attend_bf16(const FcAttendArgs& a, hipStream_t s);

struct FcScatterArgs {
    const void* k_new; const void* v_new; void* k_cache; void* v_cache;
    int64_t head_stride; int64_t tok_stride; fc_dtype dtype; int H_k; int d; int L_c; int A;
    int32_t active_off[FC_MAX_ACTIVE];
    const int32_t* rec_idx; const int32_t* n_rec;
};
int fc_launch_scatter_kv(const FcScatterArgs& a, hipStream_t s);

struct FcMassArgs {
    const void* q_base;        // [rows, H_q, d]
    const int32_t* n_rec;      // when non-null: rows come from the tail of compact block *n_rec-1
    const int32_t* rec_idx;    //   and that block must hold chunk A-1
    int A; int L_c;
    int W;                     // number of observation rows
    const void* k_cache; int64_t head_stride; int64_t tok_stride; fc_dtype dtype;
    int H_q; int H_k; int d; int mass_len; float scale; float* mass; void* ws;
};
size_t fc_mass_workspace(int W, int H_q, int mass_len);
int fc_launch_mass(const FcMassArgs& a, hipStream_t s);

struct FcCompressArgs {
    void* k_cache; void* v_cache; int64_t head_stride; int64_t tok_stride; fc_dtype dtype;
    int H_k; int d; int L_k; int budget; const float* mass; int pool_k; double lambda;
    int32_t* kept; void* ws;
    int group;   // > 1: keys scored and kept in groups of this many consecutive tokens
    int phase;   // 0: score, select and move rows; 1: score and select only; 2: move rows only
};
size_t fc_compress_grouped_workspace(int H_k, int L_k, int d, int budget, int group);
size_t fc_compress_status_offset(int H_k, int L_k, int d, int budget, int group, fc_dtype dtype);
size_t fc_compress_workspace(int H_k, int L_k, int d, int budget, fc_dtype dtype);
int fc_launch_compress(const FcCompressArgs& a, hipStream_t s);
