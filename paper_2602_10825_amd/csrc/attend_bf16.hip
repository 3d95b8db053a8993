// bf16 chunk-causal flash attention on the CDNA4 matrix cores (Sec. 3.3:
// softmax(q K^T d^-1/2) V, clean KV cache + active chunks 0..c visible to chunk c).
//
// One workgroup = 256 query rows of one head of one recompute chunk: 8 wavefronts of 32 rows,
// two per SIMD with 256 registers each (a single wavefront per SIMD cannot issue fast enough:
// one instruction per four cycles, and the matrix, vector and LDS streams of this loop add up
// to about 290 instructions per tile).  Per 64-key tile:
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K fragment from LDS, B = Q fragment held
//                 in registers.  Computing the transpose puts one query per lane
//                 (column = lane % 32) and 16 keys of each 32-key block in that lane's
//                 accumulator registers, so the row max / row sum are in-lane reductions
//                 plus one exchange with lane ^ 32.
//   P   = exp2(S^T * scale*log2(e) - m)  fp32, cast to bf16 in place: the accumulator
//                 layout already is the B-operand layout of the next product (contraction
//                 index = key, with a fixed permutation of the keys inside each 16-key
//                 group that V's LDS layout mirrors).  The row sums are taken over the
//                 ROUNDED weights (v_dot2c_f32_bf16 with a vector of ones), i.e. over
//                 exactly the weights V is multiplied with.
//   O^T += V^T P^T  A = V^T fragment read from the row-major V tile with the transposing
//                 LDS load ds_read_b64_tr_b16 (each 16-lane group turns 4 keys x 16 dv into
//                 16 lanes x 4 keys), two loads per 8-key fragment.
// The reference point m of the exponent is NOT the running row max: it is raised (and O, l
// rescaled) only when some row sum of a tile exceeds 2^40, which the sums reveal for free.
// exp2(S c2 - m) then stays far inside the fp32 / bf16 exponent range, the final O / l is
// unchanged, and the steady state carries no row-max reduction and no rescale at all.
// The first tile always takes the raise path once (m starts at -1e30).
// O += V P of tile j-1 is issued together with the exp2 / sum / pack of tile j, so the
// matrix cores work while the vector ALU turns S into P.  K/V tiles are fetched with 16-byte
// global loads one tile ahead (wavefront-uniform tile base + 32-bit lane offset) and live in a
// ring of three LDS buffers (tile j-1 still feeds O += V P while tile j+1 is being written):
// one barrier per tile.  The visible key segments are listed once per workgroup in LDS, so
// stepping to the next tile is branch-free.
// Work-groups are mapped so that the 32 compute units of one XCD work on the same head
// and chunk at the same time and share the K/V stream through that XCD's L2.
#include "fc_common.hpp"

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BQ = 256;      // query rows per workgroup
constexpr int BK = 64;       // keys per tile
constexpr int NXCD = 8;
constexpr float kNegBig = -1.0e30f;

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

// Transposing LDS load: within each group of 16 lanes, lane s passes the address of 4
// consecutive bf16; lane i receives element (i % 4) of the data addressed by lanes
// i/4, i/4 + 4, i/4 + 8, i/4 + 12.
__device__ __forceinline__ s16x4_t lds_read_tr(const bf16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4_t __attribute__((address_space(3)))*)(p));
}

struct TileIter {
    int sgi, start, len, t0;
    bool done;
};

// Tile -> registers.  The tile's first row is a wavefront-uniform base; each lane adds a 32-bit
// byte offset (precomputed for full tiles, clamped to the last valid row for a ragged one).
template <int LD, int ROWS_PER_PASS>
__device__ __forceinline__ void prefetch_tile(u32x4_native (&kreg)[LD], u32x4_native (&vreg)[LD],
                                              const bf16_t* kbase, const bf16_t* vbase,
                                              const TileIter& t, int64_t tok_stride, int ld_row,
                                              int ld_col, const uint32_t (&voff_full)[LD]) {
    const int nvalid = (t.len - t.t0 < BK) ? t.len - t.t0 : BK;
    const int64_t tile_off = (int64_t)(t.start + t.t0) * tok_stride;
    const char* kt = reinterpret_cast<const char*>(kbase + tile_off);
    const char* vt = reinterpret_cast<const char*>(vbase + tile_off);
#pragma unroll
    for (int p = 0; p < LD; ++p) {
        uint32_t voff = voff_full[p];
        if (nvalid < BK) {
            int row = p * ROWS_PER_PASS + ld_row;
            if (row > nvalid - 1) row = nvalid - 1;
            voff = ((uint32_t)row * (uint32_t)tok_stride + (uint32_t)ld_col * 8u) * 2u;
        }
        kreg[p] = *reinterpret_cast<const u32x4_native*>(kt + voff);
        vreg[p] = *reinterpret_cast<const u32x4_native*>(vt + voff);
    }
}

template <int LD, int ROWS_PER_PASS>
__device__ __forceinline__ void stage_tile(const u32x4_native (&kreg)[LD], const u32x4_native (&vreg)[LD],
                                           bf16_t* Kb, bf16_t* Vb, int krow, int vrow, int ld_row,
                                           int ld_col) {
#pragma unroll
    for (int p = 0; p < LD; ++p) {
        const int row = p * ROWS_PER_PASS + ld_row;
        *reinterpret_cast<u32x4_native*>(&Kb[row * krow + ld_col * 8]) = kreg[p];
        *reinterpret_cast<u32x4_native*>(&Vb[row * vrow + ld_col * 8]) = vreg[p];
    }
}

constexpr int NT = 64 * (BQ / 32);   // 8 wavefronts of 32 query rows, two per SIMD

template <int D>
__global__ __launch_bounds__(NT) void attend_bf16_kernel(FcAttendArgs a, int tiles, int per) {
    constexpr int KS = D / 16;        // contraction steps of Q K^T
    constexpr int DVB = D / 32;       // 32-wide blocks of the value dimension
    constexpr int KROW = D + 8;       // padded K row (bf16): 16-byte fragment reads of 16
                                      // consecutive keys fall in distinct banks
    constexpr int VROW = D + 32;      // padded V row: the 4 key rows of one transposing
                                      // load fall in disjoint bank quarters
    constexpr int VPR = D / 8;        // 16-byte vectors per K/V row
    constexpr int LD = BK * VPR / NT; // global loads per thread per tile (K, and again V)
    constexpr float kTooBig = 1.0995116e12f;  // 2^40: a row sum above this triggers a raise of m

    const int bid = blockIdx.x;
    const int xcd = bid % NXCD, slot = bid / NXCD;
    const int rank = slot / per;
    const int item = xcd * per + slot % per;
    if (item >= a.H_q * tiles) return;
    const int R = min(*a.n_rec, a.A);         // a count or an entry outside the valid range
    if (rank >= R) return;                    // (a caller's mistake) is skipped, never followed
    const int r = R - 1 - rank;               // heaviest (latest) chunk first
    const int c = a.rec_idx[r];
    if ((unsigned)c >= (unsigned)a.A) return;
    const int h = item / tiles, tile = item % tiles;
    const int hk = h / (a.H_q / a.H_k);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // wave: scalar
    const int l32 = lane & 31, hh = lane >> 5;

    constexpr int NBUF = 3;
    __shared__ __attribute__((aligned(16))) bf16_t Ks[NBUF][BK * KROW];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[NBUF][BK * VROW];

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds Q[q = l32][16*step + 8*hh ..+8)
    bf16x8_t qf[KS];
    const int row_in_chunk = tile * BQ + wave * 32 + l32;
    {
        const int rc = row_in_chunk > a.L_c - 1 ? a.L_c - 1 : row_in_chunk;
        const bf16_t* qp = (const bf16_t*)a.q + (((int64_t)r * a.L_c + rc) * a.H_q + h) * D + 8 * hh;
#pragma unroll
        for (int st = 0; st < KS; ++st) qf[st] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * st);
    }

    f32x16_t o[DVB];
#pragma unroll
    for (int dv = 0; dv < DVB; ++dv)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dv][i] = 0.f;
    float m = kNegBig, lsum = 0.f;
    const float c2 = a.scale * 1.4426950408889634f;

    const bf16_t* kbase = (const bf16_t*)a.k_cache + (int64_t)hk * a.head_stride;
    const bf16_t* vbase = (const bf16_t*)a.v_cache + (int64_t)hk * a.head_stride;

    // ---- visible key segments (clean region, then active chunks 0..c; adjacent ones merged),
    //      listed once so that stepping to the next 64-key tile is branch-free in the main loop
    __shared__ int seg_start[FC_MAX_ACTIVE + 2], seg_len[FC_MAX_ACTIVE + 2];
    __shared__ int seg_count;
    if (tid == 0) {
        int n = 0, sgi = -1;
        while (sgi <= c) {
            int start = (sgi < 0) ? 0 : a.active_off[sgi];
            int len = (sgi < 0) ? a.L_clean : a.L_c;
            ++sgi;
            while (sgi <= c && a.active_off[sgi] == start + len) { len += a.L_c; ++sgi; }
            if (len > 0) { seg_start[n] = start; seg_len[n] = len; ++n; }
        }
        seg_start[n] = seg_start[n - 1];   // sentinel: a valid range for the fetch past the end
        seg_len[n] = seg_len[n - 1];
        seg_count = n;
    }
    __syncthreads();
    const int nseg = __builtin_amdgcn_readfirstlane(seg_count);
    TileIter it;
    it.sgi = 0;
    it.start = __builtin_amdgcn_readfirstlane(seg_start[0]);
    it.len = __builtin_amdgcn_readfirstlane(seg_len[0]);
    it.t0 = 0;
    it.done = false;

    // Global -> register prefetch of one tile (rows past the end of a segment are clamped
    // to its last row) and its later store to LDS.
    u32x4_native kreg[LD], vreg[LD];
    const int ld_row = tid / VPR, ld_col = tid % VPR;
    uint32_t voff_full[LD];
#pragma unroll
    for (int p = 0; p < LD; ++p)
        voff_full[p] = ((uint32_t)(p * (NT / VPR) + ld_row) * (uint32_t)a.tok_stride + (uint32_t)ld_col * 8u) * 2u;
    // per-lane offsets of the fragment reads
    const int k_frag_off = l32 * KROW + 8 * hh;
    // transposing V read: lane s of a 16-lane group addresses key (s/4), dv 4*(s%4) of the
    // group's 4-key x 16-dv patch; groups 0/1 cover dv 0-15 / 16-31, lane half = key half
    const int l16 = lane & 15;
    const int v_frag_off = (hh * 4 + (l16 >> 2)) * VROW + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;

    // S^T = K Q^T of the tile in LDS buffer `BUF` (NV valid keys).
    // sacc[kb]: lane holds query l32, keys kb*32 + (i/4)*8 + hh*4 + i%4.
    f32x16_t sacc[2];
    float mx;
#define FC_QK(BUF, NV)                                                                        \
    {                                                                                         \
        const bf16_t* Kb_ = Ks[BUF];                                                          \
        _Pragma("unroll") for (int st = 0; st < KS; ++st) {                                   \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) { /* 2 independent chains */     \
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(                       \
                    &Kb_[kb * 32 * KROW + k_frag_off + 16 * st]);                             \
                if (st == 0) {                                                                \
                    f32x16_t z;                                                               \
                    _Pragma("unroll") for (int i = 0; i < 16; ++i) z[i] = 0.f;                \
                    sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], z, 0, 0, 0); \
                } else {                                                                      \
                    sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sacc[kb], 0, 0, 0); \
                }                                                                             \
            }                                                                                 \
        }                                                                                     \
        /* issue order: 8 fragment reads ahead of the matrix-core chain that uses them */     \
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);                                    \
        _Pragma("unroll") for (int g = 0; g < (2 * KS - 8) / 2; ++g) {                        \
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                \
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                \
        }                                                                                     \
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                    \
        if ((NV) < BK) { /* ragged tail of a segment: mask the keys past its end */           \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                  \
                _Pragma("unroll") for (int i = 0; i < 16; ++i) {                              \
                    const int key = kb * 32 + (i >> 2) * 8 + hh * 4 + (i & 3);                \
                    if (key >= (NV)) sacc[kb][i] = kNegBig;                                   \
                }                                                                             \
        }                                                                                     \
    }
    // scaled row max of S (only needed when m has to be raised)
#define FC_ROWMAX()                                                                           \
    {                                                                                         \
        float v = fmaxf(sacc[0][0], sacc[1][0]);                                              \
        _Pragma("unroll") for (int i = 1; i < 16; ++i)                                        \
            v = fmaxf(v, fmaxf(sacc[0][i], sacc[1][i]));                                      \
        v = fmaxf(v, __shfl_xor(v, 32, FC_WAVE));                                             \
        mx = v * c2;                                                                          \
    }
    // P^T = exp2(S^T c2 - m) packed to bf16 (B operand of O^T += V^T P^T) and its row sums
#define FC_EXP(PF, PS)                                                                        \
    {                                                                                         \
        const float mneg = -m;                                                                \
        const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};                                   \
        float ps0 = 0.f, ps1 = 0.f;                                                           \
        _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                      \
            _Pragma("unroll") for (int i = 0; i < 16; i += 4) {                               \
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], c2, mneg));     \
                const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i + 1], c2, mneg)); \
                const float p2 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i + 2], c2, mneg)); \
                const float p3 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i + 3], c2, mneg)); \
                const bf16x2_t lo = {(__bf16)p0, (__bf16)p1};                                 \
                const bf16x2_t hi = {(__bf16)p2, (__bf16)p3};                                 \
                /* the sums run over the ROUNDED weights, the ones V is multiplied with */     \
                ps0 = __builtin_amdgcn_fdot2_f32_bf16(lo, ones, ps0, false);                  \
                ps1 = __builtin_amdgcn_fdot2_f32_bf16(hi, ones, ps1, false);                  \
                PF[kb * 2 + (i >> 3)][i & 7] = lo[0];                                     \
                PF[kb * 2 + (i >> 3)][(i & 7) + 1] = lo[1];                               \
                PF[kb * 2 + (i >> 3)][(i & 7) + 2] = hi[0];                               \
                PF[kb * 2 + (i >> 3)][(i & 7) + 3] = hi[1];                               \
            }                                                                                 \
        PS = ps0 + ps1;                                                                       \
    }
    // Fetch the tile `it` points at into registers and step the iterator.
#define FC_FETCH_NEXT()                                                                       \
    {                                                                                         \
        pending = !it.done;                                                                   \
        nv_pending = (it.len - it.t0 < BK) ? it.len - it.t0 : BK;                             \
        prefetch_tile<LD, NT / VPR>(kreg, vreg, kbase, vbase, it, a.tok_stride, ld_row, ld_col, \
                                    voff_full);                                               \
        {                                                                                     \
            const bool last = it.t0 + BK >= it.len;          /* leaving this segment */       \
            const int nsg = (pending && last) ? it.sgi + 1 : it.sgi;                          \
            it.t0 = (!pending || last) ? 0 : it.t0 + BK;                                      \
            it.sgi = nsg;                                                                     \
            it.start = __builtin_amdgcn_readfirstlane(seg_start[nsg]);                        \
            it.len = __builtin_amdgcn_readfirstlane(seg_len[nsg]);                            \
            it.done = nsg >= nseg;                                                            \
        }                                                                                     \
    }

    // O^T += V^T P^T for the tile in V buffer VBUF: 16-key steps t, value blocks dv
#define FC_PV(PP, VBUF)                                                                       \
    {                                                                                         \
        const bf16_t* Vb_ = (VBUF) + v_frag_off;                                              \
        _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                       \
            _Pragma("unroll") for (int dv = 0; dv < DVB; ++dv) {                              \
                const bf16_t* vp = Vb_ + t * 16 * VROW + dv * 32;                             \
                const s16x4_t lo = lds_read_tr(vp);                                           \
                const s16x4_t hi = lds_read_tr(vp + 8 * VROW);                                \
                const s16x8_t v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);   \
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, v8);                         \
                o[dv] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, PP[t], o[dv], 0, 0, 0);   \
            }                                                                                 \
        }                                                                                     \
    }

    bool pending;
    int nv_pending, nv_cur = BK;
    bf16x8_t pprev[4];   // P of the previous tile, not yet multiplied into O
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < 8; ++i) pprev[t][i] = (__bf16)0.f;
    // buffer 2 plays "tile -1" in the first step: its V must be finite (P is zero there)
    for (int i = tid; i < BK * VROW / 8; i += NT)
        reinterpret_cast<uint4*>(Vs[2])[i] = make_uint4(0, 0, 0, 0);
    sacc[0] = sacc[1] = o[0];   // zeros (unused until tile 0)

    FC_FETCH_NEXT();                                                     // tile 0 -> registers
    int b = 2, bprev = 1, bnext = 0;
    bool first = true;

    // Inner loop = steady state: stage the next tile, S = K Q^T, then O += V P(previous
    // tile) on the matrix cores while the vector ALU turns S into P.  It is left when a row
    // sum shows that m must be raised; the outer loop does that (true row max of the tile,
    // rescale of O and l -- the pending P of the previous tile has already been applied in
    // the old scale --, P recomputed) and re-enters.
    for (;;) {
        if (!first) {
            FC_ROWMAX()
            {
                const float mnew = fmaxf(m, mx);
                const float alpha = __builtin_amdgcn_exp2f(m - mnew);
                m = mnew;
                lsum *= alpha;
#pragma unroll
                for (int dv = 0; dv < DVB; ++dv)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[dv][i] *= alpha;
            }
            FC_EXP(pprev, psum)
        }
        first = false;
        bool finished = false;
        bool raise = false;
        do {
            lsum += psum;
            if (!pending) { finished = true; break; }
            // ---- next tile: registers -> LDS (that buffer's tile j-2 is fully consumed)
            stage_tile<LD, NT / VPR>(kreg, vreg, Ks[bnext], Vs[bnext], KROW, VROW, ld_row, ld_col);
            __syncthreads();
            bprev = b;
            b = bnext;
            bnext = (bnext == NBUF - 1) ? 0 : bnext + 1;
            nv_cur = nv_pending;
            FC_FETCH_NEXT();
            // The wavefront in its matrix-core-only phase outranks its SIMD sibling that is
            // in the mixed phase: the sibling's vector work fills the gaps, and the two
            // reach the next barrier closer together.
            FC_QK(b, nv_cur);
            __builtin_amdgcn_s_setprio(2);
            // ---- matrix cores: O += V P(j-1);  vector ALU: P(j) = exp2(S(j) c2 - m), row
            //      sums, bf16 pack
            bf16x8_t pf[4];
            FC_PV(pprev, Vs[bprev])
            FC_EXP(pf, psum)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                // anchor: P must be computed here, next to the matrix-core work, not be
                // sunk to the loop latch where nothing would overlap it
                asm volatile("" : "+v"(pf[t]));
                pprev[t] = pf[t];
            }
            // issue order: V fragments are read 4 fragments (8 loads) ahead of their use
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
            for (int f = 0; f < 4 * DVB; ++f) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (f + 4 < 4 * DVB) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_s_setprio(0);
            raise = __any(psum > kTooBig);
        } while (!raise);
        if (finished) break;
    }
    FC_PV(pprev, Vs[b])                                                  // drain the pipeline
#undef FC_PV
#undef FC_QK
#undef FC_ROWMAX
#undef FC_EXP
#undef FC_FETCH_NEXT

    // ---- epilogue: normalise, store O (bf16) and the row log-sum-exp
    {
        const float ltot = lsum + __shfl_xor(lsum, 32, FC_WAVE);
        const float inv = 1.0f / ltot;
        if (row_in_chunk < a.L_c) {
            const int64_t row = (int64_t)r * a.L_c + row_in_chunk;
            bf16_t* op = (bf16_t*)a.out + (row * a.H_q + h) * D;
#pragma unroll
            for (int dv = 0; dv < DVB; ++dv)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int e0 = dv * 32 + g * 8 + hh * 4;
                    uint2 pk;
                    pk.x = (uint32_t)f32_to_bf16(o[dv][4 * g] * inv) |
                           ((uint32_t)f32_to_bf16(o[dv][4 * g + 1] * inv) << 16);
                    pk.y = (uint32_t)f32_to_bf16(o[dv][4 * g + 2] * inv) |
                           ((uint32_t)f32_to_bf16(o[dv][4 * g + 3] * inv) << 16);
                    *reinterpret_cast<uint2*>(op + e0) = pk;
                }
            if (a.lse && hh == 0)
                a.lse[(int64_t)h * a.A * a.L_c + row] =
                    (m + __builtin_amdgcn_logf(ltot)) * 0.6931471805599453f;
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
