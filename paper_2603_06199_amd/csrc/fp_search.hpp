// Stage (i): key-block mean pooling and the fused block-score kernel (Sec. 3.1-3.2, Alg. 1),
// and stage (ii): the max-based threshold with ballot compaction (Sec. 3.4, Alg. 2).
#pragma once
#include "fp_device.hpp"

namespace fp {

// ---------------------------------------------------------------------------------------------
// Alg. 1 stage 1.  One workgroup per (key block, KV head): 128 keys x 128 dims are read once,
// coalesced (16 lanes cover one 256-byte key row), summed in fp32 and reduced through LDS.
// The mean is stored as two bf16 planes, hi = bf16(mean) and lo = bf16(mean - hi), so that the
// score kernel can feed it to bf16 MFMA twice and keep ~16 mantissa bits of the pooled key.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pool_k_kernel(const uint16_t *__restrict__ K,
                                                     const KeyBlockRec *__restrict__ kblk, int hkv,
                                                     uint16_t *__restrict__ kb_hi, uint16_t *__restrict__ kb_lo) {
    __shared__ float red[16][kHeadDim + 4];
    const int r = blockIdx.x, hk = blockIdx.y;
    const KeyBlockRec bi = kblk[r];
    const int t = threadIdx.x, chunk = t & 15, rg = t >> 4;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    const uint4 *base = reinterpret_cast<const uint4 *>(K);
    for (int k = rg; k < bi.y; k += 16) {
        const uint4 v = base[((size_t)(bi.x + k) * hkv + hk) * 16 + chunk];
        acc[0] += bf16lo(v.x); acc[1] += bf16hi(v.x);
        acc[2] += bf16lo(v.y); acc[3] += bf16hi(v.y);
        acc[4] += bf16lo(v.z); acc[5] += bf16hi(v.z);
        acc[6] += bf16lo(v.w); acc[7] += bf16hi(v.w);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[rg][chunk * 8 + j] = acc[j];
    __syncthreads();
    if (t < kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += red[i][t];
        const float mean = s / (float)bi.y;
        const __bf16 hi = (__bf16)mean;
        const __bf16 lo = (__bf16)(mean - (float)hi);
        const size_t o = ((size_t)r * hkv + hk) * kHeadDim + t;
        kb_hi[o] = __builtin_bit_cast(uint16_t, hi);
        kb_lo[o] = __builtin_bit_cast(uint16_t, lo);
    }
}

// ---------------------------------------------------------------------------------------------
// Alg. 1 stages 2 and 3, fused.  One workgroup of 4 waves per (q-block row, KV head, pair of
// query heads): wave w owns query head 2*chunk + w/2 of the group and queries 64*(w%2)..+63 of
// the tile, kept in registers as MFMA A-fragments (64 VGPRs).  Pooled keys stream through LDS in
// tiles of 32 blocks (hi and lo planes, shared by the four waves): direct global->LDS loads one
// tile ahead into two swizzled, unpadded buffers.  For each tile a wave computes its 64 x 32
// logits with 32 MFMAs (2 query sub-tiles x 8 k-slices x {hi, lo}); the result layout puts one
// pooled key per lane column, so the reduction over the query axis (Eq. 1-2: max, then sum of
// 2^(x - max)) is in-register plus one lane exchange.  The two waves of a head then merge their
// (max, sum) pairs through a small LDS mailbox, one step later.  Registers and LDS leave room
// for two to four workgroups per CU (two at 4096 blocks per sequence, four up to 1000): waves of
// different workgroups share a SIMD without sharing a barrier, so one's MFMAs overlap the
// other's reduction.  Each block pair's (m, S) is kept in LDS as one float, m + log2 S; after the
// last tile the row is brought to a common reference (Eq. 3), normalised (Eq. 4) and written once.
// Nothing of size L x L/B ever exists.
// ---------------------------------------------------------------------------------------------
constexpr int kSearchPlane = 32 * 256;                 // one plane (hi or lo) of a 32-row tile, unpadded
constexpr int kSearchTile = 2 * kSearchPlane;          // hi + lo
constexpr int kSearchBufs = 2;
constexpr int kSearchHeads = 2;                        // query heads per workgroup
constexpr int kSearchMailbox = 2 * kSearchHeads * 32 * 8;   // [step parity][head][pooled key] (max, sum)
constexpr int kSearchStageBytes = kSearchBufs * kSearchTile + kSearchMailbox;
constexpr int kSearchRowHeader = 16;                   // per-head row maxima, ahead of the rows

// 64 x 32 logits of one pooled-key tile: acc[qt] = Q[qt] (hi + lo)^T.  baddr = buffer base + the
// lane's row and swizzled chunk for k-slice 0 (slice ks sits at baddr ^ (ks << 5)).
__device__ __forceinline__ void search_mma(const char *smem, uint32_t baddr, const bf16x8 (&qa)[2][8], f32x16 (&acc)[2]) {
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[qt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const char *bp = smem + (baddr ^ (uint32_t)(ks << 5));
        const bf16x8 bh = *reinterpret_cast<const bf16x8 *>(bp);
        const bf16x8 bl = *reinterpret_cast<const bf16x8 *>(bp + kSearchPlane);
        acc[0] = mfma32(qa[0][ks], bh, acc[0]);
        acc[1] = mfma32(qa[1][ks], bh, acc[1]);
        acc[0] = mfma32(qa[0][ks], bl, acc[0]);
        acc[1] = mfma32(qa[1][ks], bl, acc[1]);
    }
}

// Eq. 1-2 for the 32 pooled keys of a tile over this wave's 64 queries: per lane column, max and
// sum of 2^(c x - c max); lanes l and l^32 hold the two halves of a column.  Queries at or past
// nq (ragged last q-block; q0 = the wave's first query) are left out; a wave with no valid query
// returns (-inf, 0), which the merge below treats as empty.
template <bool RAGGED>
__device__ __forceinline__ float2 search_reduce(f32x16 (&acc)[2], float c, int nq, int q0, int half) {
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
    const float mc = mx * c;
    const float mcs = RAGGED ? (mx == -INFINITY ? 0.f : mc) : mc;   // all queries missing: every term is 2^-inf = 0
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s0 += fast_exp2(__builtin_fmaf(acc[0][i], c, -mcs));
        s1 += fast_exp2(__builtin_fmaf(acc[1][i], c, -mcs));
    }
    float sum = s0 + s1;
    sum = halves_sum(sum);
    return make_float2(mc, sum);
}

// (max, sum) of the union of two query sets: bring both sums to the common max.
__device__ __forceinline__ float2 search_merge(float2 a, float2 b) {
    const float m = fmaxf(a.x, b.x);
    const float sa = a.y > 0.f ? a.y * fast_exp2(a.x - m) : 0.f;
    const float sb = b.y > 0.f ? b.y * fast_exp2(b.x - m) : 0.f;
    return make_float2(m, sa + sb);
}

// Selection parameters of the fused variant (Alg. 2 applied to the row while it is still in LDS).
struct SelectArgs {
    float alpha;
    int sinkB, winB;
    int32_t *idx, *cnt;
};

template <bool SELECT>
__global__ __launch_bounds__(256, 4) void search_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ kb_hi, const uint16_t *__restrict__ kb_lo,
    const RowRec *__restrict__ rows_ranked, const int32_t *__restrict__ order, int m_total, int n_max, int n_pad,
    int hq, int hkv, int g, int nchunk, float c /* tau*log2(e) */, float eps, float *__restrict__ scores,
    SelectArgs sel) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float2 *mbox = reinterpret_cast<float2 *>(smem + kSearchBufs * kSearchTile);
    float *mtop = reinterpret_cast<float *>(smem + kSearchStageBytes);   // [head] max of the row's pair maxima
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
    const int hd = w >> 1, qh = w & 1;
    const int hg = ch * kSearchHeads + hd;
    const bool active = hg < g;
    const int h = hk * g + (active ? hg : g - 1);
    float *ms = ms_all + (size_t)hd * n_pad;   // the row: t_J = m_J + log2 S_J per block pair

    // Query fragments: qa[qt][ks] covers queries 64qh + 32qt + l%32, dims 16ks + 8(l/32)..+7.
    bf16x8 qa[2][8];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        int row = 64 * qh + 32 * qt + (l & 31);
        row = row < bi.q_len ? row : bi.q_len - 1;   // rows past a ragged end are masked in the reduction
        const uint16_t *qp = Q + ((size_t)(bi.q_tok0 + row) * hq + h) * kHeadDim + 8 * half;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qa[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
    }

    // Tile loads: 16 wave-wide instructions per tile (2 planes x 8 groups of 4 rows), 4 per wave.
    // Instruction q = 4w + i covers plane q/8, rows 4(q%8) + l/16; lane l fills LDS position l%16
    // of its row, i.e. fetches global chunk (l%16) ^ (row & 15).  Rows past the diagonal
    // (J > I) are clamped to I: they are computed and dropped.
    const int ntile = I / 32 + 1;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(FP_LDS(char) *)smem;
    const uint32_t row_bytes = (uint32_t)hkv * kHeadDim * 2;
    const char *pl_base = reinterpret_cast<const char *>(w < 2 ? kb_hi : kb_lo) + ((size_t)bi.kb_row0 * hkv + hk) * kHeadDim * 2;
    int ld_row[4];
    uint32_t ld_col[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ld_row[i] = 4 * ((4 * w + i) & 7) + (l >> 4);
        ld_col[i] = (uint32_t)(((l & 15) ^ (ld_row[i] & 15)) * 16);
    }
#define FP_LOAD_TILE(jt)                                                                                  \
    do {                                                                                                  \
        const uint32_t dst_ = lds_base + (uint32_t)(((jt) % kSearchBufs) * kSearchTile) + (w >> 1) * kSearchPlane; \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                                \
            int J_ = 32 * (jt) + ld_row[i_];                                                              \
            J_ = J_ <= I ? J_ : I;                                                                        \
            load_to_lds(pl_base, (uint32_t)J_ * row_bytes + ld_col[i_], dst_ + ((4 * w + i_) & 7) * 1024); \
        }                                                                                                 \
    } while (0)

    // B-fragment address inside a buffer: row l%32, chunk (2ks + half) ^ (row & 15).
    const int brow = l & 31;
    const uint32_t b_frag =
        (uint32_t)(brow * 256 + ((((brow >> 1) & 7) << 5) | ((half ^ (brow & 1)) << 4)));
#define FP_BUF(jt) ((uint32_t)(((jt) % kSearchBufs) * kSearchTile))

    // Prologue: tile 0 (and the older Q loads) landed.
    FP_LOAD_TILE(0);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qa[qt][ks]));   // Q has landed before the loop
    FP_WAIT_VMCNT(0);
    __syncthreads();

    // Step jt: tile jt is complete in LDS.  Issue tile jt+1 into the other buffer (its readers,
    // step jt-1's MFMAs, are behind the barrier), compute and reduce tile jt; the upper query half
    // posts its (max, sum) in the mailbox, the lower half merges the previous tile's post with
    // its own pair from the previous step and files the result; wait for tile jt+1.
    float2 prev = make_float2(-INFINITY, 0.f);
    float m_top = -INFINITY;
#define FP_STEP(RAGGED, jt)                                                                               \
    do {                                                                                                  \
        const int jt_ = (jt);                                                                             \
        if (jt_ + 1 < ntile) FP_LOAD_TILE(jt_ + 1);                                                       \
        if (active) {                                                                                     \
            f32x16 acc_[2];                                                                               \
            search_mma(smem, FP_BUF(jt_) + b_frag, qa, acc_);                                             \
            const float2 v_ = search_reduce<RAGGED>(acc_, c, bi.q_len, 64 * qh, half);                        \
            if (l < 32) {                                                                                 \
                if (qh) {                                                                                 \
                    mbox[((jt_ & 1) * kSearchHeads + hd) * 32 + l] = v_;                                             \
                } else {                                                                                  \
                    const int Jp_ = 32 * (jt_ - 1) + l;                                                   \
                    if (jt_ > 0 && Jp_ <= I) {                                                            \
                        const float2 mg_ = search_merge(prev, mbox[(((jt_ - 1) & 1) * kSearchHeads + hd) * 32 + l]); \
                        ms[Jp_] = mg_.x + __log2f(mg_.y);                                                 \
                        m_top = fmaxf(m_top, mg_.x);                                                      \
                    }                                                                                     \
                    prev = v_;                                                                            \
                }                                                                                         \
            }                                                                                             \
        }                                                                                                 \
        FP_WAIT_VMCNT(0);                                                                                 \
        __syncthreads();                                                                                  \
    } while (0)

    if (bi.q_len < kBlock) {
        for (int jt = 0; jt < ntile; ++jt) FP_STEP(true, jt);
    } else {
        for (int jt = 0; jt < ntile; ++jt) FP_STEP(false, jt);
    }
#undef FP_LOAD_TILE
#undef FP_BUF
#undef FP_STEP
    // the last tile's merge (its post is behind the loop's final barrier), then everyone meets once
    // more so that both waves of a head see the complete (m, S) row
    if (active && qh == 0) {
        const int Jp = 32 * (ntile - 1) + l;
        if (l < 32 && Jp <= I) {
            const float2 mg = search_merge(prev, mbox[(((ntile - 1) & 1) * kSearchHeads + hd) * 32 + l]);
            ms[Jp] = mg.x + __log2f(mg.y);
            m_top = fmaxf(m_top, mg.x);
        }
        m_top = wave_max(m_top);
        if (l == 0) mtop[hd] = m_top;
    }
    __syncthreads();
    if (!active) return;
    if (SELECT && qh) return;   // the list is compacted by one wave per head
    // Eq. 3-4.  With M the max of the row's pair maxima, S'_J = S_J 2^(m_J - M) and the score is
    // S'_J / (sum_K S'_K + eps).  The row holds t_J = m_J + log2 S_J (half the LDS of the pair), so
    // the same ratio is formed relative to T = max_J t_J: S'_J = 2^(t_J - T) * 2^(T - M), i.e.
    // score_J = 2^(t_J - T) / (sum_K 2^(t_K - T) + eps * 2^(M - T)), where M <= T because S_J >= 1.
    float Tm = -INFINITY;
    for (int J = l; J <= I; J += 64) Tm = fmaxf(Tm, ms[J]);
    Tm = wave_max(Tm);
    float tot = 0.f;
    for (int J = l; J <= I; J += 64) tot += fast_exp2(ms[J] - Tm);
    tot = wave_sum(tot);
    const float denom = tot + eps * fast_exp2(mtop[hd] - Tm);
    if (!SELECT) {   // each wave writes half of the sequence's columns; columns past its last key block are left alone
        float *out = scores + ((size_t)h * m_total + r) * n_max;
        for (int J = l + 64 * qh; J < bi.n_kb; J += 128) out[J] = J <= I ? fast_exp2(ms[J] - Tm) / denom : 0.f;
        return;
    }
    // Fused Alg. 2: the normalised scores (the same fp32 expression as above, so the decisions are
    // those of the two-kernel path) replace the row in LDS; threshold from their max; ballot
    // compaction as in threshold_kernel below.  Each lane re-reads only what it wrote.
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
        // 16 bytes per lane and four loads in flight per wave; the last vector may reach up to three
        // entries past the diagonal (still inside the row), which are left out of the max.
        const float4 *row4 = reinterpret_cast<const float4 *>(row);
        float4 *buf4 = reinterpret_cast<float4 *>(buf);
#pragma unroll 4
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
