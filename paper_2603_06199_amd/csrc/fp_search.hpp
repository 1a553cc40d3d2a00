// Stage (i): key-block mean pooling and the fused block-score kernel (Sec. 3.1-3.2, Alg. 1),
// and stage (ii): the max-based threshold with ballot compaction (Sec. 3.4, Alg. 2).
#pragma once
#include "fp_device.hpp"

namespace fp {

// ---------------------------------------------------------------------------------------------
// Alg. 1 stage 1.  One workgroup per (key block, KV head): 128 keys x D dims are read once,
// coalesced (D/8 lanes cover one key row), summed in fp32 and reduced through LDS.
// The mean is multiplied by c = tau*log2(e) here, once per pooled key, so that the score kernel's
// products come out as base-2 logits, and stored as two bf16 planes, hi = bf16(c*mean) and
// lo = bf16(c*mean - hi): fed to bf16 MFMA twice they keep ~16 mantissa bits of the pooled key.
// Next to the planes go two norms per pooled key: |hi + lo|_2 (bounds every logit against it by
// Cauchy-Schwarz) and |lo|_2 (bounds what a product with the hi plane alone leaves out).
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void pool_k_kernel(const uint16_t *__restrict__ K,
                                                     const KeyBlockRec *__restrict__ kblk, int hkv, float c,
                                                     uint16_t *__restrict__ kb_hi, uint16_t *__restrict__ kb_lo,
                                                     float2 *__restrict__ kb_norm) {
    constexpr int CPR = kChunks<D>;   // lanes per key row
    constexpr int RG = 256 / CPR;     // key rows per pass
    __shared__ float red[RG][D + 4];
    __shared__ float2 nrm[4];
    const int r = blockIdx.x, hk = blockIdx.y;
    const KeyBlockRec bi = kblk[r];
    const int t = threadIdx.x, chunk = t % CPR, rg = t / CPR;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    const uint4 *base = reinterpret_cast<const uint4 *>(K);
    for (int k = rg; k < bi.y; k += RG) {
        const uint4 v = base[((size_t)(bi.x + k) * hkv + hk) * CPR + chunk];
        acc[0] += bf16lo(v.x); acc[1] += bf16hi(v.x);
        acc[2] += bf16lo(v.y); acc[3] += bf16hi(v.y);
        acc[4] += bf16lo(v.z); acc[5] += bf16hi(v.z);
        acc[6] += bf16lo(v.w); acc[7] += bf16hi(v.w);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[rg][chunk * 8 + j] = acc[j];
    __syncthreads();
    if (t < D) {   // whole waves: D is a multiple of 64
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < RG; ++i) s += red[i][t];
        const float v = (s / (float)bi.y) * c;
        const __bf16 hi = (__bf16)v;
        const __bf16 lo = (__bf16)(v - (float)hi);
        const size_t o = ((size_t)r * hkv + hk) * D + t;
        kb_hi[o] = __builtin_bit_cast(uint16_t, hi);
        kb_lo[o] = __builtin_bit_cast(uint16_t, lo);
        const float both = (float)hi + (float)lo;
        const float n2 = wave_sum(both * both), l2 = wave_sum((float)lo * (float)lo);
        if ((t & 63) == 0) nrm[t >> 6] = make_float2(n2, l2);
    }
    __syncthreads();
    if (t == 0) {
        float n2 = 0.f, l2 = 0.f;
#pragma unroll
        for (int i = 0; i < D / 64; ++i) {
            n2 += nrm[i].x;
            l2 += nrm[i].y;
        }
        kb_norm[(size_t)r * hkv + hk] = make_float2(sqrtf(n2), sqrtf(l2));
    }
}

// ---------------------------------------------------------------------------------------------
// Alg. 1 stages 2 and 3, fused.  One workgroup of 4 waves per (q-block row, KV head, pair of
// query heads): wave w owns query head 2*chunk + w/2 of the group and queries 64*(w%2)..+63 of
// the tile, kept in registers as MFMA A-fragments (64 VGPRs).  Pooled keys stream through LDS in
// tiles of 32 blocks (hi and lo planes, shared by the four waves): direct global->LDS loads one
// tile ahead into two swizzled, unpadded buffers.  For each tile a wave computes its 64 x 32
// logits with 32 MFMAs (2 query sub-tiles x 8 k-slices x {hi, lo}); the result layout puts one
// pooled key per lane column, so the reduction over the query axis (Eq. 1-2) is in-register plus
// one lane exchange.  The two waves of a head then merge their results through a small LDS
// mailbox, one step later.  Each block pair's (m, S) is kept in LDS as one float,
// t = m + log2 S = log2 sum_i 2^x_i; after the last tile the row is brought to a common
// reference (Eq. 3), normalised (Eq. 4) and written once.  Nothing of size L x L/B ever exists.
//
// Two forms of the reduction.  Eq. 1-2 take the pair's max first so that the exponentials cannot
// overflow.  When every logit of the row is known to be small, |x| <= max_i|q_i| * max_J|kbar_J|
// < 100 (Cauchy-Schwarz on norms the kernel has anyway), 2^x cannot overflow or underflow in
// fp32, the max is not needed as a reference and t = log2 sum_i 2^x_i is taken directly: one
// exponential and one add per logit instead of max, subtract, exponential, add.  The pair's max
// is also what Eq. 4's eps is scaled against, so this form is taken only when eps is too small
// to change an fp32 result (the row total is >= 1).  Otherwise, and on ragged q-blocks, the
// kernel follows Eq. 1-2 literally.
//
// SELECT (search + selection in one pass) runs long rows on the hi plane alone, which halves
// the MFMA work and leaves each t_J with an error of at most eps_J = max_i|q_i| * |lo_J|, then
// re-scores exactly (both planes, the same instruction sequence as the plain kernel) the few
// block pairs on which a decision could hinge: those that may hold the row max, and those whose
// interval [t_J - eps_J, t_J + eps_J] straddles the threshold.  Every other pair is decided with
// a margin, so the lists are those of exact scores.
// ---------------------------------------------------------------------------------------------
template <int D> constexpr int kSearchPlane = 32 * 2 * D;           // one plane (hi or lo) of a 32-row tile, unpadded
template <int D> constexpr int kSearchTile = 2 * kSearchPlane<D>;   // hi + lo
constexpr int kSearchBufs = 2;
// A q-block of BLK queries of one head takes BLK/64 waves (64 queries each); the workgroup's four
// waves serve 4/(BLK/64) query heads of one KV group: 4 at block 64, 2 at 128, 1 at 256.
template <int BLK> constexpr int kSearchWavesPerHead = BLK / 64;
template <int BLK> constexpr int kSearchHeads = 4 / kSearchWavesPerHead<BLK>;
// [step parity][head][posting wave][pooled key] (max, sum): every wave of a head but its first posts
template <int BLK> constexpr int kSearchMailbox =
    2 * kSearchHeads<BLK> * (kSearchWavesPerHead<BLK> > 1 ? kSearchWavesPerHead<BLK> - 1 : 1) * 32 * 8;
template <int D, int BLK> constexpr int kSearchStageBytes = kSearchBufs * kSearchTile<D> + kSearchMailbox<BLK>;
constexpr int kSearchRowHeader = 64;                   // per-head row maxima and prologue exchange, ahead of the rows
constexpr int kSearchCandBytes = 4 * (32 + 4) * 4;     // SELECT: candidate tile indices + count per head
constexpr float kSearchSafeLogit = 100.f;              // |x| below this: 2^x needs no reference point in fp32
constexpr float kSearchEpsNoop = 0x1p-26f;             // eps below this cannot change an fp32 row total >= 1
constexpr int kSearchExactTiles = 4;                   // SELECT: rows of up to this many tiles run both planes throughout

// 64 x 32 logits of one pooled-key tile: acc[qt] = Q[qt] (hi + lo)^T, or Q[qt] hi^T.  baddr =
// buffer base + the lane's row and swizzled chunk for k-slice 0; slice ks (dims 16ks..16ks+15, chunks
// 2ks and 2ks+1) sits at baddr ^ (ks << 5) because the chunk permutation is an XOR.
template <int D, bool BOTH>
__device__ __forceinline__ void search_mma(const char *smem, uint32_t baddr, const bf16x8 (&qa)[2][D / 16], f32x16 (&acc)[2]) {
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[qt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        const char *bp = smem + (baddr ^ (uint32_t)(ks << 5));
        const bf16x8 bh = *reinterpret_cast<const bf16x8 *>(bp);
        acc[0] = mfma32(qa[0][ks], bh, acc[0]);
        acc[1] = mfma32(qa[1][ks], bh, acc[1]);
        if (BOTH) {
            const bf16x8 bl = *reinterpret_cast<const bf16x8 *>(bp + kSearchPlane<D>);
            acc[0] = mfma32(qa[0][ks], bl, acc[0]);
            acc[1] = mfma32(qa[1][ks], bl, acc[1]);
        }
    }
}

// Eq. 1-2 for the 32 pooled keys of a tile over this wave's 64 queries: per lane column, max and
// sum of 2^(x - max); lanes l and l^32 hold the two halves of a column.  Queries at or past
// nq (ragged last q-block; q0 = the wave's first query) are left out; a wave with no valid query
// returns (-inf, 0), which the merge below treats as empty.
template <bool RAGGED>
__device__ __forceinline__ float2 search_reduce(f32x16 (&acc)[2], int nq, int q0, int half) {
    if (RAGGED) {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (q0 + 32 * qt + 8 * (i >> 2) + 4 * half + (i & 3) >= nq) acc[qt][i] = -INFINITY;
    }
    float mx = max3(acc[0][0], acc[1][0], acc[0][1]);
    mx = fmaxf(mx, acc[1][1]);
#pragma unroll
    for (int i = 2; i < 16; i += 2) {
        mx = max3(mx, acc[0][i], acc[1][i]);
        mx = max3(mx, acc[0][i + 1], acc[1][i + 1]);
    }
    mx = halves_max(mx);
    const float ms = RAGGED ? (mx == -INFINITY ? 0.f : mx) : mx;   // all queries missing: every term is 2^-inf = 0
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s0 += fast_exp2(acc[0][i] - ms);
        s1 += fast_exp2(acc[1][i] - ms);
    }
    float sum = s0 + s1;
    sum = halves_sum(sum);
    return make_float2(mx, sum);
}

// The same sum with reference point 0 (all logits known to be small): (0, sum_i 2^x_i).
__device__ __forceinline__ float2 search_reduce_small(const f32x16 (&acc)[2]) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s0 += fast_exp2(acc[0][i]);
        s1 += fast_exp2(acc[1][i]);
    }
    float sum = s0 + s1;
    sum = halves_sum(sum);
    return make_float2(0.f, sum);
}

// (max, sum) of the union of two query sets: bring both sums to the common max.
__device__ __forceinline__ float2 search_merge(float2 a, float2 b) {
    const float m = fmaxf(a.x, b.x);
    const float sa = a.y > 0.f ? a.y * fast_exp2(a.x - m) : 0.f;
    const float sb = b.y > 0.f ? b.y * fast_exp2(b.x - m) : 0.f;
    return make_float2(m, sa + sb);
}

// Largest squared norm among this wave's 64 query rows: each lane holds half of the dims of two
// rows (the other half is in lane l^32), two bf16 per v_dot2.
template <int D>
__device__ __forceinline__ float search_qnorm2(const bf16x8 (&qa)[2][D / 16]) {
    float n2[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        float a = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                bf16x2 p;
                p[0] = qa[qt][ks][e];
                p[1] = qa[qt][ks][e + 1];
                a = __builtin_amdgcn_fdot2_f32_bf16(p, p, a, false);
            }
        n2[qt] = halves_sum(a);
    }
    return wave_max(fmaxf(n2[0], n2[1]));
}

// Selection parameters of the fused variant (Alg. 2 applied to the row while it is still in LDS).
struct SelectArgs {
    float alpha;
    int sinkB, winB;
    int32_t *idx, *cnt;
};

template <int D, int BLK, bool SELECT>
__global__ __launch_bounds__(256, D > 128 ? 2 : (SELECT ? 3 : 4)) void search_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ kb_hi, const uint16_t *__restrict__ kb_lo,
    const float2 *__restrict__ kb_norm, const RowRec *__restrict__ rows_ranked, const int32_t *__restrict__ order,
    int m_total, int n_max, int n_pad, int hq, int hkv, int g, int nchunk, float eps, float *__restrict__ scores,
    SelectArgs sel) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int KS = D / 16;            // k-slices of one MFMA row of fragments
    constexpr int LPW = D / 32;           // wave-wide 1 KB loads per wave and tile (both planes: 4 waves x LPW)
    constexpr int RPL = kRowsPerLoad<D>;  // pooled-key rows one such load covers
    constexpr int LPR = kChunks<D>;       // lanes per row
    constexpr int WPH = kSearchWavesPerHead<BLK>;   // waves per query head
    constexpr int HPW = kSearchHeads<BLK>;          // query heads per workgroup
    constexpr int NPOST = WPH > 1 ? WPH - 1 : 1;    // mailbox slots per head and pooled key
    float2 *mbox = reinterpret_cast<float2 *>(smem + kSearchBufs * kSearchTile<D>);
    float *mtop = reinterpret_cast<float *>(smem + kSearchStageBytes<D, BLK>);   // [head] max of the row's pair maxima
    float *xchg = mtop + 4;                                              // [wave] prologue exchange: query norm, key norm
    float *ms_all = mtop + kSearchRowHeader / sizeof(float);

    const int per_row = hkv * nchunk;
    const int rank = blockIdx.x / per_row;
    const int rem = blockIdx.x - rank * per_row;
    const int hk = rem / nchunk, ch = rem - hk * nchunk;
    const int r = order[rank];
    const RowRec bi = rows_ranked[rank];
    const int I = bi.I;
    const int tid = threadIdx.x, l = tid & 63, half = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, held in a scalar register
    const int hd = w / WPH, qh = w % WPH;   // head within the workgroup, 64-query part within the head
    const int hg = ch * HPW + hd;
    const bool active = hg < g;
    const int h = hk * g + (active ? hg : g - 1);
    float *ms = ms_all + (size_t)hd * n_pad;   // the row: t_J = m_J + log2 S_J per block pair
    const float2 *knorm = kb_norm + (size_t)bi.kb_row0 * hkv + hk;   // pooled key J of the row: knorm[J * hkv]

    // Query fragments: qa[qt][ks] covers queries 64qh + 32qt + l%32, dims 16ks + 8(l/32)..+7.
    bf16x8 qa[2][KS];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        int row = 64 * qh + 32 * qt + (l & 31);
        row = row < bi.q_len ? row : bi.q_len - 1;   // rows past a ragged end are masked in the reduction
        const uint16_t *qp = Q + ((size_t)(bi.q_tok0 + row) * hq + h) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qa[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
    }
    // Largest pooled-key norm of the row's causal blocks (for the bound on the logits).
    float kmax = 0.f;
    for (int J = tid; J <= I; J += 256) kmax = fmaxf(kmax, knorm[(size_t)J * hkv].x);

    // Tile loads: D/8 wave-wide instructions per tile (2 planes x D/16 groups of 512/D rows), D/32
    // per wave (head dimension 128: 16 instructions, 4 per wave, 4 rows each).  Instruction
    // q = LPW w + i covers plane q / (2 LPW), rows RPL (q % (2 LPW)) + l / LPR; lane l fills LDS
    // position l % LPR of its row, i.e. fetches global chunk (l % LPR) ^ (row & kSwz).  Rows past the diagonal
    // (J > I) are clamped to I: they are computed and dropped.  A row that runs on the hi plane
    // alone does not load the other one (waves 2 and 3 then issue nothing).
    const int ntile = I / 32 + 1;
    const bool ragged = bi.q_len < BLK;
    // the hi-plane pass and its re-scoring are laid out for two waves per head (block 128)
    const bool hi_only = SELECT && BLK == 128 && !ragged && ntile > kSearchExactTiles && sel.alpha > 0.f;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(FP_LDS(char) *)smem;
    const uint32_t row_bytes = (uint32_t)hkv * D * 2;
    const size_t pl_off = ((size_t)bi.kb_row0 * hkv + hk) * D * 2;
    const char *pl_base = reinterpret_cast<const char *>(w < 2 ? kb_hi : kb_lo) + pl_off;
    int ld_row[LPW];
    uint32_t ld_col[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        ld_row[i] = RPL * ((LPW * w + i) % (2 * LPW)) + l / LPR;
        ld_col[i] = (uint32_t)(((l % LPR) ^ (ld_row[i] & kSwz<D>)) * 16);
    }
#define FP_LOAD_TILE(jt)                                                                                  \
    do {                                                                                                  \
        if (!hi_only || w < 2) {                                                                          \
            const uint32_t dst_ = lds_base + (uint32_t)(((jt) % kSearchBufs) * kSearchTile<D>) + (w >> 1) * kSearchPlane<D>; \
            _Pragma("unroll") for (int i_ = 0; i_ < LPW; ++i_) {                                          \
                int J_ = 32 * (jt) + ld_row[i_];                                                          \
                J_ = J_ <= I ? J_ : I;                                                                    \
                load_to_lds(pl_base, (uint32_t)J_ * row_bytes + ld_col[i_], dst_ + ((LPW * w + i_) % (2 * LPW)) * 1024); \
            }                                                                                             \
        }                                                                                                 \
    } while (0)

    // B-fragment address inside a buffer: row l%32, chunk (2ks + half) ^ (row & kSwz) = 2ks ^ (half ^ (row & kSwz)).
    const int brow = l & 31;
    const uint32_t b_frag = (uint32_t)(brow * 2 * D + ((half ^ (brow & kSwz<D>)) << 4));
#define FP_BUF(jt) ((uint32_t)(((jt) % kSearchBufs) * kSearchTile<D>))

    // Prologue: tile 0 (and the older Q and norm loads) landed; the waves exchange their largest
    // query norm (per head) and pooled-key norm (per workgroup).
    FP_LOAD_TILE(0);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qa[qt][ks]));   // Q has landed before the loop
    FP_WAIT_VMCNT(0);
    {
        const float qn = sqrtf(search_qnorm2<D>(qa));
        kmax = wave_max(kmax);
        if (l == 0) {
            xchg[2 * w] = qn;
            xchg[2 * w + 1] = kmax;
        }
    }
    __syncthreads();
    // wave-uniform values, moved to scalar registers so that the branches on them are scalar too
    float qn_head = xchg[2 * (hd * WPH)];
#pragma unroll
    for (int i = 1; i < WPH; ++i) qn_head = fmaxf(qn_head, xchg[2 * (hd * WPH + i)]);
    const float qnorm = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qn_head)));   // all queries of the head's q-block
    kmax = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(fmaxf(fmaxf(xchg[1], xchg[3]), fmaxf(xchg[5], xchg[7])))));
    // small: no logit of this row can leave (-100, 100), and eps is a rounding no-op
    const bool small = !ragged && qnorm * kmax * 1.01f < kSearchSafeLogit && eps <= kSearchEpsNoop;

    // Step jt: tile jt is complete in LDS.  Issue tile jt+1 into the other buffer (its readers,
    // step jt-1's MFMAs, are behind the barrier), compute and reduce tile jt; the upper query half
    // posts its (max, sum) in the mailbox, the lower half merges the previous tile's post with
    // its own pair from the previous step and files the result; wait for tile jt+1.
    float2 prev = make_float2(-INFINITY, 0.f);
    float m_top = -INFINITY;
    // slot of (step parity, posting wave qh >= 1) for this head and lane
#define FP_MBOX(par_, qh_) mbox[(((par_) * HPW + hd) * NPOST + ((qh_) - 1)) * 32 + l]
#define FP_FILE(SMALL, Jp_, par_)                                                                         \
    do {                                                                                                  \
        float2 mg_ = prev;                                                                                \
        _Pragma("unroll") for (int p_ = 1; p_ < WPH; ++p_) {                                              \
            const float2 post_ = FP_MBOX(par_, p_);                                                       \
            if (SMALL) mg_.y += post_.y;                                                                  \
            else mg_ = search_merge(mg_, post_);                                                          \
        }                                                                                                 \
        if (SMALL) {                                                                                      \
            ms[Jp_] = __log2f(mg_.y);                                                                     \
        } else {                                                                                          \
            ms[Jp_] = mg_.x + __log2f(mg_.y);                                                             \
            m_top = fmaxf(m_top, mg_.x);                                                                  \
        }                                                                                                 \
    } while (0)
#define FP_STEP(RAGGED, SMALL, BOTH, jt)                                                                  \
    do {                                                                                                  \
        const int jt_ = (jt);                                                                             \
        if (jt_ + 1 < ntile) FP_LOAD_TILE(jt_ + 1);                                                       \
        if (active) {                                                                                     \
            f32x16 acc_[2];                                                                               \
            search_mma<D, BOTH>(smem, FP_BUF(jt_) + b_frag, qa, acc_);                                       \
            const float2 v_ = SMALL ? search_reduce_small(acc_) : search_reduce<RAGGED>(acc_, bi.q_len, 64 * qh, half); \
            if (l < 32) {                                                                                 \
                if (qh) {                                                                                 \
                    FP_MBOX(jt_ & 1, qh) = v_;                                                            \
                } else {                                                                                  \
                    const int Jp_ = 32 * (jt_ - 1) + l;                                                   \
                    if (jt_ > 0 && Jp_ <= I) FP_FILE(SMALL, Jp_, (jt_ - 1) & 1);                          \
                    prev = v_;                                                                            \
                }                                                                                         \
            }                                                                                             \
        }                                                                                                 \
        FP_WAIT_VMCNT(0);                                                                                 \
        __syncthreads();                                                                                  \
    } while (0)

    if (ragged) {
        for (int jt = 0; jt < ntile; ++jt) FP_STEP(true, false, true, jt);
    } else if (hi_only) {
        if (small) {
            for (int jt = 0; jt < ntile; ++jt) FP_STEP(false, true, false, jt);
        } else {
            for (int jt = 0; jt < ntile; ++jt) FP_STEP(false, false, false, jt);
        }
    } else if (small) {
        for (int jt = 0; jt < ntile; ++jt) FP_STEP(false, true, true, jt);
    } else {
        for (int jt = 0; jt < ntile; ++jt) FP_STEP(false, false, true, jt);
    }
#undef FP_STEP
    // the last tile's merge (its post is behind the loop's final barrier), then everyone meets once
    // more so that both waves of a head see the complete row
    if (active && qh == 0) {
        const int Jp = 32 * (ntile - 1) + l;
        if (l < 32 && Jp <= I) FP_FILE(small, Jp, (ntile - 1) & 1);
        m_top = wave_max(m_top);
        if (l == 0) mtop[hd] = m_top;
    }
    __syncthreads();

    // ------------------------------------------------------------------------------------------
    // SELECT on the hi plane: exact re-scoring of the pairs a decision could hinge on.
    // With eps_J >= |t_J(hi) - t_J(exact)|:  T_lo = max_J (t_J - eps_J) <= T <= T_hi = max_J (t_J + eps_J);
    // a pair is a candidate if it may hold the row max (t_J + eps_J >= T_lo) or if it is not kept
    // anyway (sink, window) and its interval meets [T_lo + log2 alpha, T_hi + log2 alpha].  The
    // scanning wave of each head (its lower query half) collects up to 32 candidates per pass, in
    // ascending order; the head's two waves gather those pooled keys (both planes) into the head's
    // tile buffer and run the plain kernel's instruction sequence on them; the exact t_J replaces
    // the approximate one.  The pass count is uniform over the workgroup (the heads' candidate counts meet in
    // LDS), so every wave takes the same barriers.
    // ------------------------------------------------------------------------------------------
    float T_exact = -INFINITY;   // scanning wave: max of the re-scored t_J
    if (SELECT && hi_only) {
        int32_t *cand = reinterpret_cast<int32_t *>(ms_all + (size_t)HPW * n_pad) + hd * 36;   // [32] indices, [32] = count
        const float la = __log2f(sel.alpha);
        float lo_t = -INFINITY, hi_t = -INFINITY;
        // eps_J = qn |lo_J| + slack; the slack stands for the fp32 accumulation noise of the two
        // instruction sequences (one plane, two planes), which scales with the size of the logits
        const float qn = qnorm * 1.004f;
        const float slack = 0x1p-15f + 0x1p-18f * qnorm * kmax;
        if (active && qh == 0) {
            for (int J = l; J <= I; J += 64) {
                const float tj = ms[J];
                const float ej = qn * knorm[(size_t)J * hkv].y + slack;
                lo_t = fmaxf(lo_t, tj - ej);
                hi_t = fmaxf(hi_t, tj + ej);
            }
            lo_t = wave_max(lo_t);
            hi_t = wave_max(hi_t);
        }
        const float thr_lo = lo_t + la - 0x1p-14f, thr_hi = hi_t + la + 0x1p-14f;
        int J_scan = 0;
        // If no pair that the threshold decides (sink and window blocks are kept anyway) has an
        // interval that meets [T_lo, T_hi] + log2 alpha, every decision already has a margin against
        // any T in [T_lo, T_hi]: nothing is re-scored, not even the pairs that may hold the max, and
        // the row's approximate max stands in for T below.
        if (active && qh == 0) {
            bool hinge = false;
            float t_apx = -INFINITY;
            for (int J = l; J <= I; J += 64) {
                const float tj = ms[J];
                const float ej = qn * knorm[(size_t)J * hkv].y + slack;
                const bool structural = (J < sel.sinkB) || (I - J < sel.winB);
                hinge |= !structural && tj + ej >= thr_lo && tj - ej <= thr_hi;
                t_apx = fmaxf(t_apx, tj);
            }
            if (__ballot(hinge) == 0ull) {
                J_scan = I + 1;
                T_exact = t_apx;   // reduced over the wave after the loop
            }
        }
        for (;;) {
            if (qh == 0) {
                int have = 0, first = 0;
                if (active) {
                    while (J_scan <= I && have < 32) {
                        const int J = J_scan + l;
                        bool c = false;
                        if (J <= I) {
                            const float tj = ms[J];
                            const float ej = qn * knorm[(size_t)J * hkv].y + slack;
                            const bool structural = (J < sel.sinkB) || (I - J < sel.winB);
                            c = (tj + ej >= lo_t) || (!structural && tj + ej >= thr_lo && tj - ej <= thr_hi);
                        }
                        const unsigned long long bal = __ballot(c);
                        const int slot = have + __builtin_popcountll(bal & ((1ull << l) - 1ull));
                        if (c && slot < 32) cand[slot] = J;
                        const int found = __builtin_popcountll(bal);
                        if (have == 0 && found > 0) first = J_scan + __builtin_ctzll(bal);
                        if (have + found > 32) {
                            // the tile is full inside this chunk: resume right after the last index taken
                            unsigned long long b = bal;
                            for (int k = have; k < 31; ++k) b &= b - 1;   // drop the (32 - have - 1) lowest set bits
                            J_scan += __builtin_ctzll(b) + 1;
                            have = 32;
                        } else {
                            have += found;
                            J_scan += 64;
                        }
                    }
                    if (l >= have && l < 32) cand[l] = first;   // pad the tile with a valid row
                }
                if (l == 0) cand[32] = have;
            }
            __syncthreads();
            const int32_t *cand0 = reinterpret_cast<int32_t *>(ms_all + (size_t)HPW * n_pad);
            const int n0 = cand0[32], n1 = cand0[36 + 32];
            if (n0 == 0 && n1 == 0) break;
            const int nmine = hd ? n1 : n0;
            if (nmine > 0) {   // wave qh gathers plane qh of the head's tile: 2 LPW instructions of RPL rows
                const char *pb = reinterpret_cast<const char *>(qh ? kb_lo : kb_hi) + pl_off;
                const uint32_t dst = lds_base + (uint32_t)(hd * kSearchTile<D> + qh * kSearchPlane<D>);
#pragma unroll
                for (int i = 0; i < 2 * LPW; ++i) {
                    const int row = RPL * i + l / LPR;
                    const int J = cand[row];
                    load_to_lds(pb, (uint32_t)J * row_bytes + (uint32_t)(((l % LPR) ^ (row & kSwz<D>)) * 16), dst + i * 1024);
                }
            }
            FP_WAIT_VMCNT(0);
            __syncthreads();
            float2 v = make_float2(-INFINITY, 0.f);
            if (nmine > 0) {
                f32x16 acc[2];
                search_mma<D, true>(smem, (uint32_t)(hd * kSearchTile<D>) + b_frag, qa, acc);
                v = small ? search_reduce_small(acc) : search_reduce<false>(acc, bi.q_len, 64 * qh, half);
                if (qh && l < 32) mbox[hd * 32 + l] = v;
            }
            __syncthreads();
            if (nmine > 0 && qh == 0 && l < nmine) {
                const float2 post = mbox[hd * 32 + l];
                float tj;
                if (small) {
                    tj = __log2f(v.y + post.y);
                } else {
                    const float2 mg = search_merge(v, post);
                    tj = mg.x + __log2f(mg.y);
                }
                ms[cand[l]] = tj;
                T_exact = fmaxf(T_exact, tj);
            }
            // the next pass rewrites cand and the tile buffers: its scan starts after this barrier's
            // readers are done because the scanning wave itself is the last reader of cand here, and
            // the gathers of the next pass are issued after the barrier that follows the scan
        }
        T_exact = wave_max(T_exact);
    }
#undef FP_LOAD_TILE
#undef FP_BUF
#undef FP_FILE
#undef FP_MBOX
    if (!active) return;
    if (SELECT && qh) return;   // the list is compacted by one wave per head
    // Eq. 3-4.  With M the max of the row's pair maxima, S'_J = S_J 2^(m_J - M) and the score is
    // S'_J / (sum_K S'_K + eps).  The row holds t_J = m_J + log2 S_J (half the LDS of the pair), so
    // the same ratio is formed relative to T = max_J t_J: S'_J = 2^(t_J - T) * 2^(T - M), i.e.
    // score_J = 2^(t_J - T) / (sum_K 2^(t_K - T) + eps * 2^(M - T)), where M <= T because S_J >= 1.
    float Tm = -INFINITY;
    if (SELECT && hi_only) {
        Tm = T_exact;   // every pair that can hold the max was re-scored
    } else {
        for (int J = l; J <= I; J += 64) Tm = fmaxf(Tm, ms[J]);
        Tm = wave_max(Tm);
    }
    float tot = 0.f;
    for (int J = l; J <= I; J += 64) tot += fast_exp2(ms[J] - Tm);
    tot = wave_sum(tot);
    const float denom = tot + (small ? 0.f : eps * fast_exp2(mtop[hd] - Tm));
    if (!SELECT) {   // the head's waves share the sequence's columns; columns past its last key block are left alone
        float *out = scores + ((size_t)h * m_total + r) * n_max;
        for (int J = l + 64 * qh; J < bi.n_kb; J += 64 * WPH) out[J] = J <= I ? fast_exp2(ms[J] - Tm) / denom : 0.f;
        return;
    }
    // Fused Alg. 2: the normalised scores (the same fp32 expression as above) replace the row in
    // LDS; threshold from their max; ballot compaction as in threshold_kernel below.  Each lane
    // re-reads only what it wrote.  On a row that ran on the hi plane, an entry that was not
    // re-scored lies outside the threshold's uncertainty interval, so comparing its approximate
    // value gives the decision of the exact one.
    float mx = -INFINITY;
    for (int J = l; J <= I; J += 64) {
        const float p = fast_exp2(ms[J] - Tm) / denom;
        ms[J] = p;
        mx = fmaxf(mx, p);
    }
    mx = wave_max(mx);
    const float thr = __fmul_rn(sel.alpha, mx);
    int32_t *lst = sel.idx + ((size_t)h * m_total + r) * n_max;
    int count = 0;
    for (int base = 0; base <= I; base += 64) {
        const int J = base + l;
        bool keep = false;
        if (J <= I) keep = (ms[J] >= thr) || (J < sel.sinkB) || (I - J < sel.winB);
        const unsigned long long bal = __ballot(keep);
        if (keep) lst[count + __builtin_popcountll(bal & ((1ull << l) - 1ull))] = J;
        count += __builtin_popcountll(bal);
    }
    if (l == 0) sel.cnt[(size_t)h * m_total + r] = count;
}

// ---------------------------------------------------------------------------------------------
// Alg. 2.  One wave per (head, q-block row).  Pass 1 reads the row's causal part once from HBM
// with coalesced loads, keeps it in LDS and takes the row max with a wave reduction.  Pass 2
// reads the row back from LDS, 64 candidates at a time: the keep decision
// (score >= alpha*max, or sink, or window) becomes a ballot; the popcount of the lower lanes is
// each kept block's slot, so the ascending list comes out without a sort or a scan over memory.
// ---------------------------------------------------------------------------------------------
constexpr int kThresholdWaves = 4;   // rows per workgroup

template <bool VEC>   // VEC: rows start on 16-byte boundaries (n_max % 4 == 0, aligned base)
__global__ __launch_bounds__(256) void threshold_kernel(const float *__restrict__ scores,
                                                        const RowRec *__restrict__ rows, int m_total, int n_max,
                                                        int n_pad, int hq, float alpha, int sinkB, int winB,
                                                        int32_t *__restrict__ idx, int32_t *__restrict__ cnt) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int wv = threadIdx.x >> 6;
    const int wave = blockIdx.x * kThresholdWaves + wv;
    const int l = threadIdx.x & 63;
    if (wave >= hq * m_total) return;   // no barrier in this kernel: waves are independent
    float *buf = reinterpret_cast<float *>(smem) + (size_t)wv * n_pad;
    const int r = wave % m_total;   // wave = h*m_total + r
    const int I = rows[r].I;
    const float *row = scores + (size_t)wave * n_max;
    int32_t *out = idx + (size_t)wave * n_max;

    float mx = -INFINITY;
    if (VEC) {
        // 16 bytes per lane and up to eight loads in flight per wave; the last vector may reach up to three
        // entries past the diagonal (still inside the row), which are left out of the max.
        const float4 *row4 = reinterpret_cast<const float4 *>(row);
        float4 *buf4 = reinterpret_cast<float4 *>(buf);
#pragma unroll 8
        for (int j4 = l; 4 * j4 <= I; j4 += 64) {
            const float4 v = row4[j4];
            buf4[j4] = v;
            const int J = 4 * j4;
            mx = fmaxf(mx, v.x);
            if (J + 1 <= I) mx = fmaxf(mx, v.y);
            if (J + 2 <= I) mx = fmaxf(mx, v.z);
            if (J + 3 <= I) mx = fmaxf(mx, v.w);
        }
    } else {
        for (int J = l; J <= I; J += 64) {
            const float v = row[J];
            buf[J] = v;
            mx = fmaxf(mx, v);
        }
    }
    mx = wave_max(mx);
    const float thr = __fmul_rn(alpha, mx);   // one fp32 rounding, as the reference decision

    int count = 0;
    for (int base = 0; base <= I; base += 64) {
        const int J = base + l;
        bool keep = false;
        if (J <= I) keep = (buf[J] >= thr) || (J < sinkB) || (I - J < winB);
        const unsigned long long bal = __ballot(keep);
        if (keep) out[count + __builtin_popcountll(bal & ((1ull << l) - 1ull))] = J;
        count += __builtin_popcountll(bal);
    }
    if (l == 0) cnt[wave] = count;
}

}  // namespace fp
