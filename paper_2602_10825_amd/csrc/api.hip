// C-ABI entry points of libflowcache: argument validation (before any HIP call), workspace
// carving and kernel launches.  See include/flowcache.h for the contract of every call.
#include <cmath>
#include <cstring>

#include "fc_common.hpp"

namespace {

inline bool bad_dtype(fc_dtype t) { return t != FC_F32 && t != FC_BF16; }
inline int esize(fc_dtype t) { return t == FC_BF16 ? 2 : 4; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int check_kv_layout(const void* k_cache, const void* v_cache, int64_t head_stride,
                    int64_t tok_stride, int64_t positions, fc_dtype dtype, int H_k, int d) {
    if (!k_cache || !v_cache) return FC_INVALID_ARGUMENT;
    if (bad_dtype(dtype) || H_k < 1 || positions < 1) return FC_INVALID_ARGUMENT;
    if (d != 64 && d != 128) return FC_UNSUPPORTED;
    if (tok_stride < d || head_stride < positions * tok_stride) return FC_INVALID_ARGUMENT;
    if (tok_stride > (1 << 24)) return FC_UNSUPPORTED;   // kernels keep in-tile byte offsets in 32 bits
    const int per16 = 16 / esize(dtype);
    if (tok_stride % per16 != 0 || head_stride % per16 != 0) return FC_UNSUPPORTED;
    if (!aligned16(k_cache) || !aligned16(v_cache)) return FC_UNSUPPORTED;
    return FC_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

const char* flowcache_status_string(int status) {
    switch (status) {
        case FC_OK: return "ok";
        case FC_INVALID_ARGUMENT: return "invalid argument";
        case FC_UNSUPPORTED: return "unsupported shape or dtype";
        case FC_WORKSPACE_TOO_SMALL: return "workspace too small";
        case FC_HIP_ERROR: return "HIP runtime error";
        default: return "unknown status";
    }
}

int flowcache_version(void) { return 100; }

// ------------------------------------------------------------------ chunk_decide
size_t flowcache_chunk_decide_workspace(int A, int64_t chunk_elems) {
    if (A < 1 || A > FC_MAX_ACTIVE || chunk_elems < 1) return 0;
    // the bf16 launch never uses fewer blocks than the fp32 one would need space for
    const int b0 = fc_decide_blocks_per_chunk(A, chunk_elems, FC_F32);
    const int b1 = fc_decide_blocks_per_chunk(A, chunk_elems, FC_BF16);
    const int bpc = b0 > b1 ? b0 : b1;
    return fc_align_up((size_t)A * bpc * 2 * sizeof(double));
}

int flowcache_chunk_decide(const void* x_cur, const void* x_prev, fc_dtype dtype, int A,
                           int64_t chunk_elems, const int32_t* step_idx, int warmup_m,
                           double eps, double* acc, double* l1rel, uint8_t* recompute_mask,
                           int32_t* recompute_idx, int32_t* n_recompute, void* x_compact,
                           void* workspace, size_t workspace_bytes, fc_stream stream) {
    if (!x_cur || !x_prev || !step_idx || !acc || !recompute_mask || !recompute_idx ||
        !n_recompute || !workspace)
        return FC_INVALID_ARGUMENT;
    if (bad_dtype(dtype) || A < 1 || A > FC_MAX_ACTIVE || chunk_elems < 1 || warmup_m < 0)
        return FC_INVALID_ARGUMENT;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return FC_INVALID_ARGUMENT;
    if (workspace_bytes < flowcache_chunk_decide_workspace(A, chunk_elems))
        return FC_WORKSPACE_TOO_SMALL;
    FcDecideArgs a{x_cur, x_prev, dtype, A, chunk_elems, step_idx, warmup_m, eps, acc, l1rel,
                   recompute_mask, recompute_idx, n_recompute, x_compact, workspace, 0};
    return fc_launch_decide(a, (hipStream_t)stream);
}

int flowcache_chunk_decide_noalloc(const void* x_cur, const void* x_prev, fc_dtype dtype, int A,
                                   int64_t chunk_elems, const int32_t* step_idx, int warmup_m,
                                   double eps, double* acc, double* l1rel,
                                   uint8_t* recompute_mask, int32_t* recompute_idx,
                                   int32_t* n_recompute, void* x_compact, fc_stream stream) {
    if (!x_cur || !x_prev || !step_idx || !acc || !recompute_mask || !recompute_idx || !n_recompute)
        return FC_INVALID_ARGUMENT;
    if (bad_dtype(dtype) || A < 1 || A > FC_MAX_ACTIVE || chunk_elems < 1 || warmup_m < 0)
        return FC_INVALID_ARGUMENT;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return FC_INVALID_ARGUMENT;
    // the block partials of this launch must fit the library's own scratch
    if (flowcache_chunk_decide_workspace(A, chunk_elems) > (size_t)FC_DECIDE_SCRATCH_BYTES)
        return FC_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    const int st = fc_decide_scratch(&ws);
    if (st != FC_OK) return st;
    FcDecideArgs a{x_cur, x_prev, dtype, A, chunk_elems, step_idx, warmup_m, eps, acc, l1rel,
                   recompute_mask, recompute_idx, n_recompute, x_compact, ws, 0};
    return fc_launch_decide(a, (hipStream_t)stream);
}

int flowcache_uniform_decide(const void* x_cur, const void* x_prev, fc_dtype dtype, int A,
                             int64_t chunk_elems, const int32_t* step_idx, int warmup_m,
                             double eps, double* acc_global, double* l1rel,
                             uint8_t* recompute_mask, int32_t* recompute_idx,
                             int32_t* n_recompute, void* x_compact, void* workspace,
                             size_t workspace_bytes, fc_stream stream) {
    if (!x_cur || !x_prev || !step_idx || !acc_global || !recompute_mask || !recompute_idx ||
        !n_recompute || !workspace)
        return FC_INVALID_ARGUMENT;
    if (bad_dtype(dtype) || A < 1 || A > FC_MAX_ACTIVE || chunk_elems < 1 || warmup_m < 0)
        return FC_INVALID_ARGUMENT;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return FC_INVALID_ARGUMENT;
    if (workspace_bytes < flowcache_chunk_decide_workspace(A, chunk_elems))
        return FC_WORKSPACE_TOO_SMALL;
    FcDecideArgs a{x_cur, x_prev, dtype, A, chunk_elems, step_idx, warmup_m, eps, acc_global,
                   l1rel, recompute_mask, recompute_idx, n_recompute, x_compact, workspace, 1};
    return fc_launch_decide(a, (hipStream_t)stream);
}

int flowcache_residual_apply(const void* x_cur, const void* y_compact, void* residual, void* out,
                             fc_dtype dtype, int A, int64_t chunk_elems,
                             const int32_t* recompute_idx, const int32_t* n_recompute,
                             fc_stream stream) {
    if (!x_cur || !residual || !out || !recompute_idx || !n_recompute) return FC_INVALID_ARGUMENT;
    if (bad_dtype(dtype) || A < 1 || A > FC_MAX_ACTIVE || chunk_elems < 1)
        return FC_INVALID_ARGUMENT;
    FcResidualArgs a{x_cur, y_compact, residual, out, dtype, A, chunk_elems, recompute_idx,
                     n_recompute};
    return fc_launch_residual(a, (hipStream_t)stream);
}

// ------------------------------------------------------------------ attention mass
size_t flowcache_attention_mass_workspace(int W, int H_q, int H_k, int d, int mass_len) {
    (void)H_k; (void)d;
    if (W < 1 || H_q < 1 || mass_len < 1) return 0;
    return fc_mass_workspace(W, H_q, mass_len);
}

int flowcache_attention_mass(const void* q_obs, int W, const void* k_cache,
                             int64_t kv_head_stride, int64_t kv_tok_stride, fc_dtype dtype,
                             int H_q, int H_k, int d, int mass_len, float softmax_scale,
                             float* mass, void* workspace, size_t workspace_bytes,
                             fc_stream stream) {
    if (!q_obs || !mass || !workspace || W < 1 || H_q < 1) return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, k_cache, kv_head_stride, kv_tok_stride, mass_len, dtype, H_k, d);
    if (st != FC_OK) return st;
    if (H_q % H_k != 0) return FC_INVALID_ARGUMENT;
    if (!(softmax_scale >= 0.f) || !std::isfinite(softmax_scale)) return FC_INVALID_ARGUMENT;
    if (!aligned16(q_obs)) return FC_UNSUPPORTED;
    if (workspace_bytes < fc_mass_workspace(W, H_q, mass_len)) return FC_WORKSPACE_TOO_SMALL;
    FcMassArgs m{};
    m.q_base = q_obs; m.n_rec = nullptr; m.rec_idx = nullptr; m.A = 0; m.L_c = 0; m.W = W;
    m.k_cache = k_cache; m.head_stride = kv_head_stride; m.tok_stride = kv_tok_stride;
    m.dtype = dtype; m.H_q = H_q; m.H_k = H_k; m.d = d; m.mass_len = mass_len;
    m.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)d);
    m.mass = mass; m.ws = workspace;
    return fc_launch_mass(m, (hipStream_t)stream);
}

// ------------------------------------------------------------------ scatter_kv
namespace {
int check_slots(int A, int L_c, int L_clean, int capacity, const int32_t* active_off) {
    // slots: inside [L_clean, capacity], L_c long, pairwise disjoint
    for (int i = 0; i < A; ++i) {
        const int64_t lo = active_off[i];
        if (lo < L_clean || lo + L_c > capacity) return FC_INVALID_ARGUMENT;
        for (int j = 0; j < i; ++j) {
            const int64_t lj = active_off[j];
            if (lo < lj + L_c && lj < lo + L_c) return FC_INVALID_ARGUMENT;
        }
    }
    return FC_OK;
}
}  // namespace

int flowcache_scatter_kv(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                         int64_t kv_head_stride, int64_t kv_tok_stride, int capacity,
                         fc_dtype dtype, int H_k, int d, int L_c, int L_clean, int A,
                         const int32_t* active_off, const int32_t* recompute_idx,
                         const int32_t* n_recompute, fc_stream stream) {
    if (!k_new || !v_new || !active_off || !recompute_idx || !n_recompute) return FC_INVALID_ARGUMENT;
    if (A < 1 || A > FC_MAX_ACTIVE || L_c < 1 || L_clean < 0 || capacity < 1) return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, v_cache, kv_head_stride, kv_tok_stride, capacity, dtype, H_k, d);
    if (st != FC_OK) return st;
    st = check_slots(A, L_c, L_clean, capacity, active_off);
    if (st != FC_OK) return st;
    if (!aligned16(k_new) || !aligned16(v_new)) return FC_UNSUPPORTED;
    FcScatterArgs sc{};
    sc.k_new = k_new; sc.v_new = v_new; sc.k_cache = k_cache; sc.v_cache = v_cache;
    sc.head_stride = kv_head_stride; sc.tok_stride = kv_tok_stride; sc.dtype = dtype;
    sc.H_k = H_k; sc.d = d; sc.L_c = L_c; sc.A = A;
    std::memcpy(sc.active_off, active_off, sizeof(int32_t) * A);
    sc.rec_idx = recompute_idx; sc.n_rec = n_recompute;
    return fc_launch_scatter_kv(sc, (hipStream_t)stream);
}

// ------------------------------------------------------------------ attend
size_t flowcache_attend_workspace(int A, int L_c, int H_q, int H_k, int d, int mass_len,
                                  int obs_window) {
    (void)H_k; (void)d;
    if (A < 1 || L_c < 1 || H_q < 1) return 0;
    size_t need = 256;
    if (mass_len > 0) {
        const int W = (obs_window <= 0 || obs_window > L_c) ? L_c : obs_window;
        need += fc_mass_workspace(W, H_q, mass_len);
    }
    return need;
}

int flowcache_attend(const void* q, const void* k_new, const void* v_new, void* k_cache,
                     void* v_cache, int64_t kv_head_stride, int64_t kv_tok_stride,
                     int capacity, fc_dtype dtype, int H_q, int H_k, int d, int L_c,
                     int L_clean, int A, const int32_t* active_off,
                     const int32_t* recompute_idx, const int32_t* n_recompute,
                     float softmax_scale, void* out, float* lse, float* mass, int mass_len,
                     int obs_window, void* workspace, size_t workspace_bytes,
                     fc_stream stream) {
    if (!q || !out || !active_off || !recompute_idx || !n_recompute) return FC_INVALID_ARGUMENT;
    if ((k_new == nullptr) != (v_new == nullptr)) return FC_INVALID_ARGUMENT;
    if (A < 1 || A > FC_MAX_ACTIVE || L_c < 1 || L_clean < 0 || H_q < 1 || capacity < 1)
        return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, v_cache, kv_head_stride, kv_tok_stride, capacity, dtype, H_k, d);
    if (st != FC_OK) return st;
    if (H_q % H_k != 0) return FC_INVALID_ARGUMENT;
    if (!(softmax_scale >= 0.f) || !std::isfinite(softmax_scale)) return FC_INVALID_ARGUMENT;
    if ((int64_t)A * L_c > INT32_MAX) return FC_UNSUPPORTED;
    st = check_slots(A, L_c, L_clean, capacity, active_off);
    if (st != FC_OK) return st;
    if (!aligned16(q) || !aligned16(out) || (k_new && (!aligned16(k_new) || !aligned16(v_new))))
        return FC_UNSUPPORTED;
    if (mass) {
        if (mass_len < 1 || mass_len > capacity || obs_window < 0 || !workspace)
            return FC_INVALID_ARGUMENT;
    }
    if (workspace_bytes < flowcache_attend_workspace(A, L_c, H_q, H_k, d, mass ? mass_len : 0, obs_window) &&
        mass)
        return FC_WORKSPACE_TOO_SMALL;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)d);
    hipStream_t s = (hipStream_t)stream;

    if (k_new) {
        st = flowcache_scatter_kv(k_new, v_new, k_cache, v_cache, kv_head_stride, kv_tok_stride,
                                  capacity, dtype, H_k, d, L_c, L_clean, A, active_off,
                                  recompute_idx, n_recompute, stream);
        if (st != FC_OK) return st;
    }

    FcAttendArgs at{};
    at.q = q; at.out = out; at.lse = lse; at.k_cache = k_cache; at.v_cache = v_cache;
    at.head_stride = kv_head_stride; at.tok_stride = kv_tok_stride; at.dtype = dtype;
    at.H_q = H_q; at.H_k = H_k; at.d = d; at.L_c = L_c; at.L_clean = L_clean; at.A = A;
    std::memcpy(at.active_off, active_off, sizeof(int32_t) * A);
    at.rec_idx = recompute_idx; at.n_rec = n_recompute; at.scale = scale;
    st = (dtype == FC_BF16) ? fc_launch_attend_bf16(at, s) : fc_launch_attend_f32(at, s);
    if (st != FC_OK) return st;

    if (mass) {
        FcMassArgs m{};
        m.q_base = q; m.n_rec = n_recompute; m.rec_idx = recompute_idx; m.A = A; m.L_c = L_c;
        m.W = (obs_window <= 0 || obs_window > L_c) ? L_c : obs_window;
        m.k_cache = k_cache; m.head_stride = kv_head_stride; m.tok_stride = kv_tok_stride;
        m.dtype = dtype; m.H_q = H_q; m.H_k = H_k; m.d = d; m.mass_len = mass_len;
        m.scale = scale; m.mass = mass; m.ws = workspace;
        st = fc_launch_mass(m, s);
        if (st != FC_OK) return st;
    }
    return FC_OK;
}

// ------------------------------------------------------------------ kv_compress
size_t flowcache_kv_compress_grouped_workspace(int H_k, int L_k, int d, int budget, int group,
                                               fc_dtype dtype) {
    if (H_k < 1 || L_k < 1 || budget < 1 || group < 1 || (d != 64 && d != 128) || bad_dtype(dtype))
        return 0;
    if (L_k % group != 0 || budget % group != 0) return 0;
    if (group == 1) return fc_compress_workspace(H_k, L_k, d, budget, dtype);
    return fc_compress_grouped_workspace(H_k, L_k, d, budget, group);
}

int flowcache_kv_compress_grouped(void* k_cache, void* v_cache, int64_t kv_head_stride,
                                  int64_t kv_tok_stride, fc_dtype dtype, int H_k, int d, int L_k,
                                  int budget, int group, const float* mass, int pool_k,
                                  double lambda, int32_t* kept_idx, void* workspace,
                                  size_t workspace_bytes, fc_stream stream) {
    if (!mass || !kept_idx || !workspace) return FC_INVALID_ARGUMENT;
    if (L_k < 1 || budget < 1 || group < 1) return FC_INVALID_ARGUMENT;
    if (L_k % group != 0 || budget % group != 0) return FC_INVALID_ARGUMENT;
    if (pool_k < 1 || pool_k % 2 == 0) return FC_INVALID_ARGUMENT;
    if (!(lambda >= 0.0 && lambda <= 1.0)) return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, v_cache, kv_head_stride, kv_tok_stride, L_k, dtype, H_k, d);
    if (st != FC_OK) return st;
    if (workspace_bytes < flowcache_kv_compress_grouped_workspace(H_k, L_k, d, budget, group, dtype))
        return FC_WORKSPACE_TOO_SMALL;
    FcCompressArgs c{k_cache, v_cache, kv_head_stride, kv_tok_stride, dtype, H_k, d, L_k, budget,
                     mass, pool_k, lambda, kept_idx, workspace, group, 0};
    return fc_launch_compress(c, (hipStream_t)stream);
}

size_t flowcache_kv_compress_status_offset(int H_k, int L_k, int d, int budget, int group,
                                           fc_dtype dtype) {
    if (H_k < 1 || L_k < 1 || budget < 1 || group < 1 || (d != 64 && d != 128) || bad_dtype(dtype))
        return (size_t)-1;
    if (L_k % group != 0 || budget % group != 0) return (size_t)-1;
    return fc_compress_status_offset(H_k, L_k, d, budget, group, dtype);
}

size_t flowcache_kv_compress_workspace(int H_k, int L_k, int d, int budget, fc_dtype dtype) {
    if (H_k < 1 || L_k < 1 || budget < 1 || (d != 64 && d != 128) || bad_dtype(dtype)) return 0;
    return fc_compress_workspace(H_k, L_k, d, budget, dtype);
}

int flowcache_kv_compress(void* k_cache, void* v_cache, int64_t kv_head_stride,
                          int64_t kv_tok_stride, fc_dtype dtype, int H_k, int d, int L_k,
                          int budget, const float* mass, int pool_k, double lambda,
                          int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                          fc_stream stream) {
    if (!mass || !kept_idx || !workspace) return FC_INVALID_ARGUMENT;
    if (L_k < 1 || budget < 1) return FC_INVALID_ARGUMENT;
    if (pool_k < 1 || pool_k % 2 == 0) return FC_INVALID_ARGUMENT;
    if (!(lambda >= 0.0 && lambda <= 1.0)) return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, v_cache, kv_head_stride, kv_tok_stride, L_k, dtype, H_k, d);
    if (st != FC_OK) return st;
    if (workspace_bytes < fc_compress_workspace(H_k, L_k, d, budget, dtype))
        return FC_WORKSPACE_TOO_SMALL;
    FcCompressArgs c{k_cache, v_cache, kv_head_stride, kv_tok_stride, dtype, H_k, d, L_k, budget,
                     mass, pool_k, lambda, kept_idx, workspace, 1, 0};
    return fc_launch_compress(c, (hipStream_t)stream);
}

int flowcache_kv_select(const void* k_cache, int64_t kv_head_stride, int64_t kv_tok_stride,
                        fc_dtype dtype, int H_k, int d, int L_k, int budget, const float* mass,
                        int pool_k, double lambda, int32_t* kept_idx, void* workspace,
                        size_t workspace_bytes, fc_stream stream) {
    if (!mass || !kept_idx || !workspace) return FC_INVALID_ARGUMENT;
    if (L_k < 1 || budget < 1) return FC_INVALID_ARGUMENT;
    if (pool_k < 1 || pool_k % 2 == 0) return FC_INVALID_ARGUMENT;
    if (!(lambda >= 0.0 && lambda <= 1.0)) return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, k_cache, kv_head_stride, kv_tok_stride, L_k, dtype, H_k, d);
    if (st != FC_OK) return st;
    if (workspace_bytes < fc_compress_workspace(H_k, L_k, d, budget, dtype))
        return FC_WORKSPACE_TOO_SMALL;
    // the selection phase only reads K
    FcCompressArgs c{const_cast<void*>(k_cache), const_cast<void*>(k_cache), kv_head_stride,
                     kv_tok_stride, dtype, H_k, d, L_k, budget, mass, pool_k, lambda, kept_idx,
                     workspace, 1, 1};
    return fc_launch_compress(c, (hipStream_t)stream);
}

int flowcache_kv_compact(void* k_cache, void* v_cache, int64_t kv_head_stride,
                         int64_t kv_tok_stride, fc_dtype dtype, int H_k, int d, int L_k,
                         int budget, const int32_t* kept_idx, void* workspace,
                         size_t workspace_bytes, fc_stream stream) {
    if (!kept_idx || !workspace) return FC_INVALID_ARGUMENT;
    if (L_k < 1 || budget < 1) return FC_INVALID_ARGUMENT;
    int st = check_kv_layout(k_cache, v_cache, kv_head_stride, kv_tok_stride, L_k, dtype, H_k, d);
    if (st != FC_OK) return st;
    if (workspace_bytes < fc_compress_workspace(H_k, L_k, d, budget, dtype))
        return FC_WORKSPACE_TOO_SMALL;
    FcCompressArgs c{k_cache, v_cache, kv_head_stride, kv_tok_stride, dtype, H_k, d, L_k, budget,
                     nullptr, 1, 0.0, const_cast<int32_t*>(kept_idx), workspace, 1, 2};
    return fc_launch_compress(c, (hipStream_t)stream);
}

#pragma GCC visibility pop
}  // extern "C"
