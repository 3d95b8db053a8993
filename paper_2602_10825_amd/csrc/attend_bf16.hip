// bf16 chunk-causal flash attention on the CDNA4 matrix cores (Sec. 3.3:
// softmax(q K^T d^-1/2) V, clean KV cache + active chunks 0..c visible to chunk c).
//
// One workgroup = 256 query rows of one head of one recompute chunk, 4 wavefronts of
// 64 rows each.  Per 64-key tile:
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K fragment from LDS, B = Q fragment held
//                 in registers.  Computing the transpose puts one query per lane
//                 (column = lane % 32) and 16 keys of each 32-key block in that lane's
//                 accumulator registers, so the row max / row sum are in-lane reductions
//                 plus one exchange with lane ^ 32.
//   P   = exp2(S^T * scale*log2(e) - m)  fp32, online max / sum, cast to bf16 in place:
//                 the accumulator layout already is the B-operand layout of the next
//                 product (contraction index = key, with a fixed permutation of the keys
//                 inside each 16-key group that V's LDS layout mirrors).
//   O^T += V^T P^T  A = V^T fragment from LDS (V is stored transposed, keys permuted).
// K/V tiles are fetched with 16-byte global loads one tile ahead of the compute.
// Work-groups are mapped so that the 32 compute units of one XCD work on the same head
// and chunk at the same time and share the K/V stream through that XCD's L2.
#include "fc_common.hpp"

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BQ = 256;      // query rows per workgroup
constexpr int BK = 64;       // keys per tile
constexpr int NT = 256;      // threads
constexpr int NXCD = 8;
constexpr float kNegBig = -1.0e30f;

// position of key `kk` (0..63) inside a row of the transposed V tile: the 8 keys that one
// lane half contributes to one 16-key contraction step sit contiguously.
__device__ __forceinline__ int vt_pos(int kk) {
    const int kb = kk >> 5, w = kk & 31;
    const int blk8 = w >> 3, hh = (w >> 2) & 1, ilo = w & 3;
    return kb * 32 + (blk8 >> 1) * 16 + hh * 8 + (blk8 & 1) * 4 + ilo;
}

struct TileIter {
    int sgi, start, len, t0;
    bool done;
};

template <int D>
__global__ __launch_bounds__(NT) void attend_bf16_kernel(FcAttendArgs a, int tiles, int per) {
    constexpr int KS = D / 16;        // contraction steps of Q K^T
    constexpr int DVB = D / 32;       // 32-wide blocks of the value dimension
    constexpr int KROW = D + 8;       // padded K row (bf16 elements)
    constexpr int VROW = BK + 8;      // padded V^T row
    constexpr int VPR = D / 8;        // 16-byte vectors per K/V row
    constexpr int LD = BK * VPR / NT; // global loads per thread per tile (K, and again V)

    const int bid = blockIdx.x;
    const int xcd = bid % NXCD, slot = bid / NXCD;
    const int rank = slot / per;
    const int item = xcd * per + slot % per;
    if (item >= a.H_q * tiles) return;
    const int R = *a.n_rec;
    if (rank >= R) return;
    const int r = R - 1 - rank;               // heaviest (latest) chunk first
    const int c = a.rec_idx[r];
    const int h = item / tiles, tile = item % tiles;
    const int hk = h / (a.H_q / a.H_k);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, hh = lane >> 5;

    __shared__ __attribute__((aligned(16))) bf16_t Ks[BK * KROW];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[D * VROW];

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds Q[q = l32][16*step + 8*hh ..+8)
    bf16x8_t qf[2][KS];
    int row_in_chunk[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        int rc = tile * BQ + wave * 64 + qb * 32 + l32;
        row_in_chunk[qb] = rc;
        if (rc > a.L_c - 1) rc = a.L_c - 1;
        const bf16_t* qp = (const bf16_t*)a.q + (((int64_t)r * a.L_c + rc) * a.H_q + h) * D + 8 * hh;
#pragma unroll
        for (int st = 0; st < KS; ++st)
            qf[qb][st] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * st);
    }

    f32x16_t o[2][DVB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int dv = 0; dv < DVB; ++dv)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[qb][dv][i] = 0.f;
    float m[2] = {kNegBig, kNegBig};
    float lsum[2] = {0.f, 0.f};
    const float c2 = a.scale * 1.4426950408889634f;

    const bf16_t* kbase = (const bf16_t*)a.k_cache + (int64_t)hk * a.head_stride;
    const bf16_t* vbase = (const bf16_t*)a.v_cache + (int64_t)hk * a.head_stride;

    // ---- iterator over 64-key tiles of the visible, merged segments
    TileIter it;
    auto next_segment = [&](TileIter& t) {
        while (t.sgi <= c) {
            int start = (t.sgi < 0) ? 0 : a.active_off[t.sgi];
            int len = (t.sgi < 0) ? a.L_clean : a.L_c;
            ++t.sgi;
            while (t.sgi <= c && a.active_off[t.sgi] == start + len) { len += a.L_c; ++t.sgi; }
            if (len > 0) { t.start = start; t.len = len; t.t0 = 0; return; }
        }
        t.done = true;
    };
    it.sgi = -1; it.start = 0; it.len = 0; it.t0 = 0; it.done = false;
    next_segment(it);

    uint4 kreg[LD], vreg[LD];
    auto prefetch = [&](const TileIter& t) {
        const int nvalid = (t.len - t.t0 < BK) ? t.len - t.t0 : BK;
#pragma unroll
        for (int p = 0; p < LD; ++p) {
            const int idx = p * NT + tid;
            int row = idx / VPR;
            const int col = idx % VPR;
            if (row > nvalid - 1) row = nvalid - 1;
            const int64_t off = (int64_t)(t.start + t.t0 + row) * a.tok_stride + col * 8;
            kreg[p] = *reinterpret_cast<const uint4*>(kbase + off);
            vreg[p] = *reinterpret_cast<const uint4*>(vbase + off);
        }
    };
    if (!it.done) prefetch(it);

    while (!it.done) {
        const int nvalid = (it.len - it.t0 < BK) ? it.len - it.t0 : BK;
        // advance the iterator (scalar work) before the barrier
        it.t0 += BK;
        if (it.t0 >= it.len) next_segment(it);

        __syncthreads();  // every wave is done reading the previous tile
#pragma unroll
        for (int p = 0; p < LD; ++p) {
            const int idx = p * NT + tid;
            const int row = idx / VPR, col = idx % VPR;
            *reinterpret_cast<uint4*>(&Ks[row * KROW + col * 8]) = kreg[p];
            const int pos = vt_pos(row);
            const uint32_t w[4] = {vreg[p].x, vreg[p].y, vreg[p].z, vreg[p].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                Vt[(col * 8 + 2 * e) * VROW + pos] = (bf16_t)(w[e] & 0xffffu);
                Vt[(col * 8 + 2 * e + 1) * VROW + pos] = (bf16_t)(w[e] >> 16);
            }
        }
        __syncthreads();
        if (!it.done) prefetch(it);

        // ---- S^T = K Q^T : acc[qb][kb], lane: query l32, keys kb*32 + (r/4)*8 + hh*4 + r%4
        f32x16_t sacc[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[qb][kb][i] = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int st = 0; st < KS; ++st) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(
                    &Ks[(kb * 32 + l32) * KROW + 16 * st + 8 * hh]);
                sacc[0][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][st], sacc[0][kb], 0, 0, 0);
                sacc[1][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[1][st], sacc[1][kb], 0, 0, 0);
            }
        }
        if (nvalid < BK) {  // ragged tail of a segment: mask the keys past its end
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = kb * 32 + (i >> 2) * 8 + hh * 4 + (i & 3);
                    if (key >= nvalid) { sacc[0][kb][i] = kNegBig; sacc[1][kb][i] = kNegBig; }
                }
        }

        // ---- online softmax, P^T packed to bf16 (B operand of the next product)
        bf16x8_t pf[2][4];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mx = sacc[qb][0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[qb][kb][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, FC_WAVE));
            const float mnew = fmaxf(m[qb], mx * c2);
            const float alpha = __builtin_amdgcn_exp2f(m[qb] - mnew);
            m[qb] = mnew;
            float ps = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[qb][kb][i], c2, -mnew));
                    ps += p;
                    pf[qb][kb * 2 + (i >> 3)][i & 7] = (__bf16)p;
                }
            lsum[qb] = lsum[qb] * alpha + ps;
#pragma unroll
            for (int dv = 0; dv < DVB; ++dv)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[qb][dv][i] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int dv = 0; dv < DVB; ++dv) {
                const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(
                    &Vt[(dv * 32 + l32) * VROW + t * 16 + hh * 8]);
                o[0][dv] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[0][t], o[0][dv], 0, 0, 0);
                o[1][dv] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[1][t], o[1][dv], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: normalise, store O (bf16) and the row log-sum-exp
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float ltot = lsum[qb] + __shfl_xor(lsum[qb], 32, FC_WAVE);
        const float inv = 1.0f / ltot;
        if (row_in_chunk[qb] < a.L_c) {
            const int64_t row = (int64_t)r * a.L_c + row_in_chunk[qb];
            bf16_t* op = (bf16_t*)a.out + (row * a.H_q + h) * D;
#pragma unroll
            for (int dv = 0; dv < DVB; ++dv)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int e0 = dv * 32 + g * 8 + hh * 4;
                    uint2 pk;
                    pk.x = (uint32_t)f32_to_bf16(o[qb][dv][4 * g] * inv) |
                           ((uint32_t)f32_to_bf16(o[qb][dv][4 * g + 1] * inv) << 16);
                    pk.y = (uint32_t)f32_to_bf16(o[qb][dv][4 * g + 2] * inv) |
                           ((uint32_t)f32_to_bf16(o[qb][dv][4 * g + 3] * inv) << 16);
                    *reinterpret_cast<uint2*>(op + e0) = pk;
                }
            if (a.lse && hh == 0)
                a.lse[(int64_t)h * a.A * a.L_c + row] =
                    (m[qb] + __builtin_amdgcn_logf(ltot)) * 0.6931471805599453f;
        }
    }
}

}  // namespace

int fc_launch_attend_bf16(const FcAttendArgs& a, hipStream_t s) {
    const int tiles = (a.L_c + BQ - 1) / BQ;
    const int items = a.H_q * tiles;
    const int per = (items + NXCD - 1) / NXCD;
    const dim3 grid((unsigned)(NXCD * per * a.A));
    if (a.d == 128)
        attend_bf16_kernel<128><<<grid, NT, 0, s>>>(a, tiles, per);
    else if (a.d == 64)
        attend_bf16_kernel<64><<<grid, NT, 0, s>>>(a, tiles, per);
    else
        return FC_UNSUPPORTED;
    FC_LAUNCH_CHECK();
    return FC_OK;
}
