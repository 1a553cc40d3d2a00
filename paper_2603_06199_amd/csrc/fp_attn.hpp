// Stage (iii): index-driven block-sparse attention (Sec. 3.5, Alg. 3) and, from the same
// template, full causal attention.  bf16 MFMA for both contractions, fp32 online softmax.
#pragma once
#include "fp_device.hpp"

namespace fp {

// LDS: three K buffers and two V buffers of one 64-key tile (64 rows x 2D bytes, unpadded) each.
// Tiles are written by direct global->LDS loads (16 B per lane, lane i lands at base + 16 i), so
// bank conflicts are avoided by permuting the 16-byte chunks inside a row instead of padding
// (stated for head dimension 128, 16 chunks per row; the masks shrink with the row for 64):
//   K row r keeps chunk c at position c ^ (r & 15): the A-fragment reads of 16 consecutive rows
//     at one chunk index then hit 16 different bank groups;
//   V row r keeps chunk c at position c ^ 4 (r & 3): the four rows a transpose read touches per
//     lane group then hit four different 64-byte bank groups.
// Head dimension 128: 16 KB tiles, 80 KB, two workgroups per CU.  64: 40 KB.  256: 32 KB tiles,
// all 160 KB of a CU, one workgroup (its accumulators and query fragments need 512 registers).
// A workgroup has one wave per 32 queries of its q-block part, four at most; a 64-query block gets
// two waves and 32-key tiles (40 KB, four workgroups per CU), so that every wave still loads 16
// rows of each tile and no wave repeats another's queries.
template <int BLK> constexpr int kAttnWaves = BLK < 128 ? BLK / 32 : 4;
template <int BLK> constexpr int kAttnTileKeys = 16 * kAttnWaves<BLK>;
template <int D> constexpr int kAttnRowBytes = 2 * D;
template <int D, int KT> constexpr int kAttnTile = KT * kAttnRowBytes<D>;   // 16384 at D = 128, 64 keys
constexpr int kAttnKBufs = 3, kAttnVBufs = 2;
template <int D, int KT> constexpr int kAttnVBase = kAttnKBufs * kAttnTile<D, KT>;
template <int D, int BLK> constexpr int kAttnLds = (kAttnKBufs + kAttnVBufs) * kAttnTile<D, kAttnTileKeys<BLK>>;   // 81920 at D = 128
template <int D> constexpr int kAttnVSwz = (D / 32 - 1 < 3 ? D / 32 - 1 : 3);     // V rows: chunk ^ 4 (r & kAttnVSwz)

// ds_read_b64_tr_b16: within each group of 16 lanes the 16 x 4 b16 values addressed by the
// lanes (lane j supplies 4 consecutive b16) are exchanged so that lane i receives, in element e,
// the value that lane 4e + i/4 addressed at position i%4.  With lane j pointing at row (j/4)
// and columns 4*(j%4)..+3 of a row-major 4 x 16 patch, lane i ends up with column i of the four
// rows: exactly the key-contiguous fragment the PV product needs from a row-major V tile.
__device__ __forceinline__ s16x4 lds_read_tr(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((FP_LDS(s16x4) *)(FP_LDS(char) *)p);
}

/*
 * One workgroup (4 waves) per (query head, q-block row); wave w owns queries 32w..32w+31 of the
 * block.  Alg. 3's loop over the listed blocks runs as a loop over 64-key tiles (two per block)
 * whose addresses come straight from the index list: an unlisted block costs no instruction.
 * (Other block sizes: a 256-query block is two such workgroups over four tiles per block, a
 * 64-query block one workgroup of two waves over two 32-key tiles per block; the counts below are
 * for 64-key tiles.)
 *
 * Per tile and wave:
 *   S^T = K Q^T  (keys x queries, 16 MFMA 32x32x16): the query index is the lane column, so the
 *         row max and row sum of the softmax are reductions over a lane's own registers plus one
 *         exchange between the wave's halves;
 *   causal mask only if the tile belongs to the diagonal block (Alg. 3, is_diag);
 *   online softmax in base 2: p = 2^(c*s - c*m) with m a reference point that follows the row
 *         max lazily (see attn_new_max), so the accumulator is rescaled a few times per row;
 *   O^T += V^T P^T (16 MFMA): P^T is already in B-operand layout (registers of S^T, packed to
 *         bf16), V^T fragments come from the row-major V tile through LDS transpose reads.
 *
 * Software pipeline inside the wave: in step t the wave first issues the QK^T MFMAs of tile t+1
 * and only then runs the softmax of tile t (VALU) and the PV MFMAs of tile t, so the matrix
 * pipe works on t+1 while the vector ALU exponentiates t.  The S^T registers alternate between
 * two sets (steps are unrolled in pairs).  K therefore runs one tile ahead of V in LDS: step t
 * reads K[t+1] and V[t] and issues the direct-to-LDS loads of V[t+1] and K[t+3]; K has three
 * buffers, V two; one barrier per step.
 *
 * Work order: blockIdx -> (XCD, slot).  Consecutive workgroup ids land on different XCDs, each
 * with its own L2; slot k of XCD x takes query head k%g of super-item (k/g)*8 + x, where a
 * super-item is (KV head, row rank), KV head outermost, and rows are ranked heaviest (largest I)
 * first.  The g query heads that share a KV head run on one XCD at about the same time and find
 * each other's K/V tiles in its L2; the eight XCDs work on eight neighbouring rows of the same KV
 * head, so one head's K and V (128 MiB each at 512K tokens) are what the last-level cache holds
 * at a time, not every head's.
 */
// Block of key tile t: entry t / TPB of the list (TPB tiles per block), the entry index kept
// below nb and the block id inside [0, I].
template <bool SPARSE, int TPB>
__device__ __forceinline__ int attn_tile_block(const int32_t *list, int t, int I, int nb) {
    int li = t / TPB;
    li = li < nb ? li : nb - 1;
    if (!SPARSE) return li;
    const int b = list[li];
    return b < 0 ? 0 : (b > I ? I : b);
}

// S^T (KT keys x 32 queries) of one K tile: s0 = keys 0..31, s1 = keys 32..63 (untouched for a 32-key tile).
// kaddr = buffer base + the lane's row and swizzled chunk for k-slice 0; slice ks sits at kaddr ^ (ks << 5).
template <int D, int KT>
__device__ __forceinline__ void attn_qk(const char *smem, uint32_t kaddr, const bf16x8 (&qb)[D / 16], f32x16 &s0, f32x16 &s1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) { s0[i] = 0.f; if (KT > 32) s1[i] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        const char *kp = smem + (kaddr ^ (uint32_t)(ks << 5));
        const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(kp);
        s0 = mfma32(a0, qb[ks], s0);
        if (KT > 32) {
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(kp + 32 * kAttnRowBytes<D>);
            s1 = mfma32(a1, qb[ks], s1);
        }
    }
}

// Causal mask of a diagonal tile: key 8(i/4) + i%4 (+32 for s1) is in this lane's future if it
// exceeds lim = query - tile offset - 4*half.
template <int KT>
__device__ __forceinline__ void attn_mask(f32x16 &s0, f32x16 &s1, int lim) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int kk = 8 * (i >> 2) + (i & 3);
        if (kk > lim) s0[i] = -INFINITY;
        if (KT > 32 && kk + 32 > lim) s1[i] = -INFINITY;
    }
}

// Row max of one tile's S^T: half of the tile's keys are in this lane, the rest in lane^32.
template <int KT>
__device__ __forceinline__ float attn_rowmax(const f32x16 &s0, const f32x16 &s1) {
    if (KT == 32) {
        float ta = max3(s0[0], s0[1], s0[2]);
#pragma unroll
        for (int i = 3; i < 15; i += 2) ta = max3(ta, s0[i], s0[i + 1]);
        return halves_max(fmaxf(ta, s0[15]));
    }
    float ta = max3(s0[0], s0[1], s0[2]), tb = max3(s1[0], s1[1], s1[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) {
        ta = max3(ta, s0[i], s0[i + 1]);
        tb = max3(tb, s1[i], s1[i + 1]);
    }
    const float tm = max3(ta, s0[15], fmaxf(tb, s1[15]));
    return halves_max(tm);
}

// Online-softmax bookkeeping for a new tile max.  m_run is the reference point of the
// exponentials, not necessarily the true running max: it is moved (and the accumulator and the
// row sum rescaled) only when some row's max has outgrown it by more than kAttnLazy in the base-2
// exponent (wave-uniform test).  Until then p = 2^(c*s - c*m_run) may reach 2^kAttnLazy, which
// fp32 sums and bf16 operands hold without loss; O = acc / l and lse = c*m_run + log2 l do not
// depend on the reference point.  With 32 rows per wave an exact-max rule would fire on most
// tiles of a short row; this one fires a few times per row at most.
constexpr float kAttnLazy = 8.0f;
template <int NDT>
__device__ __forceinline__ void attn_new_max(float tm, float c, float &m_run, float &l_run, f32x16 (&acc)[NDT]) {
    const float m_new = fmaxf(m_run, tm);
    if (__ballot((m_new - m_run) * c > kAttnLazy)) {
        const float a = fast_exp2((m_run - m_new) * c);
        l_run *= a;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[dt][i] *= a;
        m_run = m_new;
    }
}

// p = 2^(c*s - c*m), rounded to bf16 and laid out as the B operand of the PV product; the row sum
// is taken over the fp32 values before rounding, so lse does not inherit bf16's 2^-9 rounding.
template <int KT>
__device__ __forceinline__ void attn_exp(const f32x16 &s0, const f32x16 &s1, float c, float mc, float &l_run,
                                         bf16x8 (&pb)[2][2]) {
    float la = 0.f, lb = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float pa = fast_exp2(__builtin_fmaf(s0[i], c, -mc));
        la += pa;
        pb[0][i >> 3][i & 7] = (__bf16)pa;
        if (KT > 32) {
            const float pq = fast_exp2(__builtin_fmaf(s1[i], c, -mc));
            lb += pq;
            pb[1][i >> 3][i & 7] = (__bf16)pq;
        }
    }
    l_run += la + lb;
}

// O^T += V^T P^T for one KT-key tile: V^T fragments by transpose reads of the row-major V tile.
// vaddr[dt] = buffer base + the lane's row/column offsets with the swizzle of d-tile dt folded in.
template <int D, int KT>
__device__ __forceinline__ void attn_pv(const char *smem, const uint32_t (&vaddr)[D / 32], const bf16x8 (&pb)[2][2],
                                        f32x16 (&acc)[D / 32]) {
#pragma unroll
    for (int kt2 = 0; kt2 < KT / 32; ++kt2)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) {
                const char *vp = smem + vaddr[dt] + (32 * kt2 + 16 * j) * kAttnRowBytes<D>;
                const s16x4 lo = lds_read_tr(vp);
                const s16x4 hi = lds_read_tr(vp + 8 * kAttnRowBytes<D>);
                const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[dt] = mfma32(__builtin_bit_cast(bf16x8, a), pb[kt2][j], acc[dt]);
            }
}

template <int D, int BLK, bool SPARSE>
__global__ __launch_bounds__(64 * kAttnWaves<BLK>, D > 128 ? 1 : 2) void attn_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ cnt, const RowRec *__restrict__ rows_ranked,
    const int32_t *__restrict__ order, int m_total, int n_max, int hq, int hkv, int g, int T, float c,
    uint16_t *__restrict__ O, float *__restrict__ lse) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int KS = D / 16;            // k-slices of the QK^T contraction
    constexpr int NDT = D / 32;           // 32-wide tiles of the head dimension in the output
    constexpr int KT = kAttnTileKeys<BLK>;   // keys per tile: 64, or 32 for the two-wave workgroup of a 64-query block
    constexpr int LPT = D / 32;           // wave-wide 1 KB loads per wave and tile (16 rows per wave)
    constexpr int RPL = kRowsPerLoad<D>;  // rows one such load covers
    constexpr int LPR = kChunks<D>;       // lanes (= 16-byte chunks) per row
    constexpr int RB = kAttnRowBytes<D>;
    constexpr int TPB = BLK / KT;                     // key tiles per key block: 2 or 4
    constexpr int QS = BLK > 128 ? BLK / 128 : 1;     // workgroups per (head, q-block), 128 queries each
    static_assert(TPB % 2 == 0, "the two register sets of the pipeline alternate over an even tile count");

    const int x = blockIdx.x & 7, k0 = blockIdx.x >> 3;
    const int sub = k0 % QS, k = k0 / QS;             // which 128 queries of the q-block
    const int s = (k / g) * 8 + x, hg = k % g;
    if (s >= m_total * hkv) return;
    // KV head outermost: the rows of one KV head run together, so the K/V of one head (not of all
    // heads at once) is what the last-level cache has to hold
    const int hk = s / m_total, rank = s - hk * m_total;
    const int r = order[rank];               // both tables are indexed by rank: one round trip
    const RowRec bi = rows_ranked[rank];
    const int h = hk * g + hg;
    const int I = bi.I;                  // diagonal key block (q-block index + KV prefix blocks)
    const int seq_tok0 = bi.k_tok0;      // K/V tokens of the sequence: seq_tok0 .. last_tok
    const int last_tok = bi.k_end - 1;

    const int tid = threadIdx.x, l = tid & 63, half = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, held in a scalar register
    const int q_local = 32 * w + (l & 31);
    const int qoff = 128 * sub;                               // the workgroup's first query within the q-block
    const int q_len = bi.q_len - qoff < 128 ? bi.q_len - qoff : 128;   // its valid queries
    if (q_len <= 0) return;                                   // a ragged q-block that ends before this part
    const int q_tok0 = bi.q_tok0 + qoff;

    // The first two list entries are fetched together with the count (the memory is there whatever
    // the count says), so that the first tile loads do not wait for a second round trip.
    int nb = I + 1, b0 = 0, b1 = 1;
    const int32_t *list = nullptr;
    if (SPARSE) {
        list = idx + ((size_t)h * m_total + r) * n_max;
        nb = cnt[(size_t)h * m_total + r];
        b0 = list[0];
        b1 = list[n_max > 1 ? 1 : 0];
        nb = nb < 0 ? 0 : (nb > I + 1 ? I + 1 : nb);
    }
    b0 = b0 < 0 ? 0 : (b0 > I ? I : b0);
    b1 = b1 < 0 ? 0 : (b1 > I ? I : b1);
    // Tiles: TPB per listed block.  Of the diagonal block (only the last entry can be it) this part
    // of the q-block needs the tiles up to its own last query, 2 (sub + 1) of them; that is fewer than
    // TPB only for the first half of a 256-query block.  The count is even in every case.
    int ntiles = TPB * nb;
    if (TPB > 2 && nb > 0 && 2 * (sub + 1) < TPB) {
        const int bl = SPARSE ? list[nb - 1] : nb - 1;
        if (bl >= I) ntiles -= TPB - 2 * (sub + 1);
    }

    if (ntiles == 0) {   // empty list: O = 0, lse = -inf (uniform exit, before any barrier)
        if (q_local < q_len) {
            uint16_t *op = O + ((size_t)(q_tok0 + q_local) * hq + h) * D + (D / 2) * half;
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < D / 16; ++i) *reinterpret_cast<u32x4 *>(op + 8 * i) = z;
            if (lse != nullptr && half == 0) lse[(size_t)h * T + q_tok0 + q_local] = -INFINITY;
        }
        return;
    }

#define FP_TILE_BLOCK(t) attn_tile_block<SPARSE, TPB>(list, (t), I, nb)

    // Q^T B-fragments: query 32w + l%32, dims 16ks + 8*half..+7.  The loads are written as
    // assembly so that their completion is counted here and not by the compiler, which cannot see
    // the tile loads queued behind them and would wait for those too: the prologue waits once,
    // with the exact count, for the fragments and the first K tile together.
    bf16x8 qb[KS];
    {
        int row = q_local < q_len ? q_local : q_len - 1;
        const uint16_t *qp = Q + ((size_t)(q_tok0 + row) * hq + h) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=&v"(qb[ks]) : "v"(qp), "n"(32 * ks) : "memory");
    }

    // Tile loads.  One wave-wide instruction moves RPL = 512/D rows (1 KB); wave w loads rows
    // 16w + RPL i + l/LPR (i < LPT) of a K or V tile (head dimension 128: 4 rows per instruction,
    // rows 16w + 4i + l/16).  Lane l fills LDS position l % LPR of its row, i.e. it fetches the
    // global chunk (l % LPR) ^ swizzle(row).  The global address is a wave-uniform base (first token
    // of the tile, KV head) plus a per-lane 32-bit byte offset.  Only a tile that reaches past
    // the end of its sequence (ragged last block) needs per-row clamping; its base is clamped
    // too, so the unsigned row offsets can never wrap.
    const uint32_t row_bytes = (uint32_t)hkv * D * 2;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(FP_LDS(char) *)smem;
    const int ld_row = 16 * w + l / LPR;   // + RPL i
    const int ld_pos = l % LPR;
    const char *Kb = reinterpret_cast<const char *>(K) + (size_t)hk * D * 2;
    const char *Vb = reinterpret_cast<const char *>(V) + (size_t)hk * D * 2;
    uint32_t ld_kcol[LPT], ld_vcol[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int row = ld_row + RPL * i;
        ld_kcol[i] = (uint32_t)((ld_pos ^ (row & kSwz<D>)) * 16);
        ld_vcol[i] = (uint32_t)((ld_pos ^ (4 * (row & kAttnVSwz<D>))) * 16);
    }
    // Clamped load of sub-tile sub_ of block blk_: every row is kept at or before the sequence's last token.
#define FP_LOAD(Xb, col_, blk_, sub_, ldsoff_)                                                            \
    do {                                                                                                  \
        const int tok0_ = seq_tok0 + (blk_) * BLK + (sub_) * KT;                                          \
        const int base_tok_ = tok0_ < last_tok ? tok0_ : last_tok;                                        \
        const char *base_ = Xb + (size_t)base_tok_ * row_bytes;                                           \
        const uint32_t dst_ = lds_base + (ldsoff_) + 16 * w * RB;                                         \
        _Pragma("unroll") for (int i_ = 0; i_ < LPT; ++i_) {                                              \
            int tok_ = tok0_ + ld_row + RPL * i_;                                                         \
            tok_ = tok_ < last_tok ? tok_ : last_tok; /* keys past the end are masked as future */        \
            const uint32_t ro_ = (uint32_t)(tok_ - base_tok_) * row_bytes; /* tok_ >= base_tok_ */        \
            load_to_lds(base_, ro_ + col_[i_], dst_ + i_ * 1024);                                         \
        }                                                                                                 \
    } while (0)
    // K tile t lives in K buffer t % 3, V tile t in V buffer t % 2.
#define FP_KBUF(t) ((uint32_t)(((t) % kAttnKBufs) * kAttnTile<D, KT>))
#define FP_VBUF(par) ((uint32_t)(kAttnVBase<D, KT> + (par) * kAttnTile<D, KT>))
    // Outside the main loop the tile index is kept at the row's last tile: a prefetch past the end
    // of the list re-reads that tile into a buffer nobody reads.
#define FP_LOAD_SAFE(Xb, col_, t, ldsoff_)                                                                \
    do {                                                                                                  \
        const int ts_ = (t) < ntiles ? (t) : ntiles - 1;                                                  \
        FP_LOAD(Xb, col_, FP_TILE_BLOCK(ts_), (ts_ % TPB), ldsoff_);                                      \
    } while (0)
    // The plain steps of the main loop load tiles known to lie before the diagonal block, hence
    // complete: no per-row clamp, and the address is a byte offset carried from step to step (see
    // the loop): off_ = offset of the tile's first row from the KV head's base.
#define FP_LOAD_AT(Xb, col_, off_, ldsoff_)                                                               \
    do {                                                                                                  \
        const char *base_ = Xb + (off_);                                                                  \
        const uint32_t dst_ = lds_base + (ldsoff_) + 16 * w * RB;                                         \
        _Pragma("unroll") for (int i_ = 0; i_ < LPT; ++i_)                                                \
            load_to_lds(base_, (uint32_t)(ld_row + RPL * i_) * row_bytes + col_[i_], dst_ + i_ * 1024);   \
    } while (0)
    // Offset of tile u given its list entry; the block id is kept inside the blocks that are complete
    // in memory (those before the diagonal one, and the diagonal one unless the sequence ends inside
    // it), so that even a malformed (non-ascending) list cannot make a plain load reach past the sequence.
    const bool diag_full = seq_tok0 + (I + 1) * BLK - 1 <= last_tok;
    const int ent_max = diag_full ? I : I - 1;
#define FP_ENT_OFF(ent_, u)                                                                               \
    ((uint64_t)(uint32_t)(seq_tok0 + ((ent_) < 0 ? 0 : ((ent_) < ent_max ? (ent_) : ent_max)) * BLK + ((u) % TPB) * KT) * row_bytes)

    f32x16 acc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_run = -INFINITY;   // reference point of the exponentials (raw dot-product units), see attn_new_max
    float l_run = 0.f;         // this lane's share of the running row sum

    // Fragment addresses inside a buffer.  K: rows l%32 and 32 + l%32, chunk
    // (2ks + half) ^ (row & kSwz) = 2ks ^ (half ^ (row & kSwz)); rows 32 apart share the permutation.
    const int krow = l & 31;
    const uint32_t k_frag = (uint32_t)(krow * RB + ((half ^ (krow & kSwz<D>)) << 4));
    // V transpose reads: row 32kt + 16j + 4half + e (+8), e = (l%16)/4 = row & 3; 8-byte unit at
    // dims 32dt + 16gq + 4cc, i.e. chunk 4dt + 2gq + cc/2, stored at chunk ^ 4(e & kAttnVSwz)
    // = 4(dt ^ (e & kAttnVSwz)) + ...
    uint32_t v_frag[NDT];
    {
        const int e = (l & 15) >> 2, gq = (l & 31) >> 4, cc = l & 3;
        const uint32_t vb = (uint32_t)((4 * half + e) * RB + (2 * gq + (cc >> 1)) * 16 + 8 * (cc & 1));
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) v_frag[dt] = vb + (uint32_t)((dt ^ (e & kAttnVSwz<D>)) * 64);
    }
    // Causal limit of tile t for this lane: on the diagonal block, key kk of the tile is in the
    // lane's future if kk > query - tile offset (and keys past a ragged end lie beyond every stored
    // query); elsewhere nothing is masked.
#define FP_LIM(t) (FP_TILE_BLOCK(t) == I ? qoff + q_local - ((t) % TPB) * KT - 4 * half : 2 * KT)

    // Prologue: S^T of tile 0 with its row max; on leaving it K[1] and V[0] are in, K[2] on its way.
    FP_LOAD(Kb, ld_kcol, b0, 0, FP_KBUF(0));
    FP_LOAD(Vb, ld_vcol, b0, 0, FP_VBUF(0));
    FP_LOAD(Kb, ld_kcol, b0, 1, FP_KBUF(1));   // ntiles >= 2
    if (TPB == 2) FP_LOAD(Kb, ld_kcol, (nb > 1 ? b1 : b0), (nb > 1 ? 0 : 1), FP_KBUF(2));
    else FP_LOAD(Kb, ld_kcol, b0, 2, FP_KBUF(2));
    FP_WAIT_VMCNT(3 * LPT);   // Q and K[0] are in; V[0], K[1] and K[2] keep landing under the first QK^T
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qb[ks]));   // uses of Q stay behind the wait
    __syncthreads();
    f32x16 sA0, sA1, sB0, sB1;
    attn_qk<D, KT>(smem, FP_KBUF(0) + k_frag, qb, sA0, sA1);
    attn_mask<KT>(sA0, sA1, b0 == I ? qoff + q_local - 4 * half : 2 * KT);
    m_run = attn_rowmax<KT>(sA0, sA1);   // finite: key 0 of tile 0 is visible to every query
    FP_WAIT_VMCNT(LPT);
    __syncthreads();

    // Step t.  On entry K[t+1] and V[t] are complete in LDS, K[t+2] may still be landing, S^T(t) is
    // in (c0, c1) and its row max is already folded into m_run (accumulator rescaled).  The step
    // issues V[t+1] into the buffer V[t-1] used and K[t+3] into the buffer K[t] used (all waves are
    // past step t-1's barrier, which was their last reader) and ends by waiting for everything but
    // K[t+3].  Every variant is straight-line code, so that the scheduler can interleave the QK^T
    // MFMAs of tile t+1 with the exponentials of tile t, and the PV MFMAs of tile t with the max of
    // tile t+1:
    //   MAIN  tile t+1 needs no mask, tiles t+1 and t+3 are complete in memory: cheap loads;
    //   TAIL  row-clamped loads and the (branch-free) causal limit of tile t+1;
    //   PEN   the last but one step: as TAIL without a K prefetch, ends with nothing in flight;
    //   LAST  exponentials and PV of the last tile only.
    // PAR is the parity of t (steps come in pairs that start at an even t): V tile t sits in V
    // buffer PAR.  KB_NEXT / KB_LOAD are the K buffers of tile t+1 (read) and t+3 (loaded); VOFF /
    // KOFF the byte offsets of tiles t+1 / t+3 (MAIN only).
    // A tile of the diagonal block that lies wholly in a wave's future needs no special case: its
    // logits are all -inf, which leaves the max alone and contributes zeros.
    enum { MAIN = 0, TAIL = 1, PEN = 2, LAST = 3 };
#define FP_STEP(MODE, PAR, t, c0, c1, n0, n1, VOFF, KOFF, KB_NEXT, KB_LOAD)                                \
    do {                                                                                                  \
        const int t_ = (t);                                                                               \
        if (MODE == MAIN) {                                                                               \
            FP_LOAD_AT(Vb, ld_vcol, VOFF, FP_VBUF(1 - PAR));                                              \
            FP_LOAD_AT(Kb, ld_kcol, KOFF, KB_LOAD);                                                       \
        } else if (MODE != LAST) {                                                                        \
            FP_LOAD_SAFE(Vb, ld_vcol, t_ + 1, FP_VBUF(1 - PAR));                                          \
            if (MODE == TAIL) FP_LOAD_SAFE(Kb, ld_kcol, t_ + 3, KB_LOAD);                                 \
        }                                                                                                 \
        bf16x8 pb_[2][2];                                                                                 \
        attn_exp<KT>(c0, c1, c, m_run * c, l_run, pb_);                                                   \
        if (MODE != LAST) attn_qk<D, KT>(smem, (KB_NEXT) + k_frag, qb, n0, n1);                           \
        {                                                                                                 \
            uint32_t va_[NDT];                                                                            \
            _Pragma("unroll") for (int dt_ = 0; dt_ < NDT; ++dt_) va_[dt_] = FP_VBUF(PAR) + v_frag[dt_];  \
            attn_pv<D, KT>(smem, va_, pb_, acc);                                                          \
        }                                                                                                 \
        if (MODE != LAST) {                                                                               \
            if (MODE != MAIN) attn_mask<KT>(n0, n1, FP_LIM(t_ + 1));                                      \
            attn_new_max<NDT>(attn_rowmax<KT>(n0, n1), c, m_run, l_run, acc);                             \
            if (MODE == PEN) FP_WAIT_VMCNT(0);                                                            \
            else FP_WAIT_VMCNT(LPT);                                                                      \
            __syncthreads();                                                                              \
        }                                                                                                 \
    } while (0)

    // Tiles before the diagonal block are complete (only a sequence's last block can be partial,
    // and a row only meets it as its diagonal); the list is ascending, so only its last block can
    // be the diagonal one: the first n_plain tiles need no mask.  A pair of MAIN steps (t, t+1)
    // computes S^T of tiles t+1 and t+2 without a mask and loads tiles t+1 .. t+4 without a clamp:
    // t+2 < n_plain, and t+4 has to exist and be complete, which the diagonal block is unless the
    // sequence ends inside it (then t+4 < n_plain).  ntiles and n_plain are even, and so is the
    // number of MAIN steps, so the register roles of the two S^T tiles alternate evenly.
    const int n_plain = FP_TILE_BLOCK(ntiles - 1) == I ? TPB * (nb - 1) : ntiles;
    const int t_main = diag_full ? (n_plain - 2 < ntiles - 4 ? n_plain - 2 : ntiles - 4) : n_plain - 4;   // <= 0: none
    int t = 0;
    if (t_main > 0) {
        // Addresses of the main loop, carried instead of recomputed: o1..o3 = offsets of tiles t+1..t+3,
        // e4 = list entry of tile t+4, fetched one pair of steps before it is needed (a list read is a
        // scalar memory load; waiting for it inside a step would stall the wave at the step's start);
        // kb0..kb2 = K buffers of tiles t..t+2.  Tile t+5 is the odd neighbour of t+4 in one block.
        // (Tiles 0..4 lie in the first 4 / TPB + 1 list entries; the first two are already here.)
#define FP_ENT(u) ((u) / TPB == 0 ? b0 : ((u) / TPB == 1 ? b1 : (SPARSE ? list[(u) / TPB < nb ? (u) / TPB : nb - 1] : (u) / TPB)))
        uint64_t o1 = FP_ENT_OFF(FP_ENT(1), 1), o2 = FP_ENT_OFF(FP_ENT(2), 2), o3 = FP_ENT_OFF(FP_ENT(3), 3);
        int e4 = FP_ENT(4);
        uint32_t kb0 = FP_KBUF(0), kb1 = FP_KBUF(1), kb2 = FP_KBUF(2);
        for (; t < t_main; t += 2) {
            const int u6 = (t + 6) / TPB < nb ? (t + 6) / TPB : nb - 1;
            const int e6 = SPARSE ? list[u6] : u6;
            FP_STEP(MAIN, 0, t, sA0, sA1, sB0, sB1, o1, o3, kb1, kb0);
            const uint64_t o4 = FP_ENT_OFF(e4, t + 4);
            FP_STEP(MAIN, 1, t + 1, sB0, sB1, sA0, sA1, o2, o4, kb2, kb1);
            o1 = o3;
            o2 = o4;
            o3 = o4 + (uint64_t)KT * row_bytes;
            e4 = e6;
            const uint32_t kb_ = kb0;
            kb0 = kb2;
            kb2 = kb1;
            kb1 = kb_;
        }
#undef FP_ENT
    }
    for (; t < ntiles - 2; t += 2) {
        FP_STEP(TAIL, 0, t, sA0, sA1, sB0, sB1, 0, 0, FP_KBUF(t + 1), FP_KBUF(t + 3));
        FP_STEP(TAIL, 1, t + 1, sB0, sB1, sA0, sA1, 0, 0, FP_KBUF(t + 2), FP_KBUF(t + 4));
    }
    FP_STEP(PEN, 0, t, sA0, sA1, sB0, sB1, 0, 0, FP_KBUF(t + 1), 0);
    FP_STEP(LAST, 1, t + 1, sB0, sB1, sA0, sA1, 0, 0, 0, 0);

    // O = acc / l, lse = m + log2 l (Alg. 3, final normalisation); rows past a ragged end are not stored.
    // Each lane holds 4 consecutive dims of one query per accumulator group, which would make every
    // global store touch 64 different rows.  The wave's 32 x D output tile is therefore turned
    // through LDS (its own 32 rows of the K buffers: their last reader and their last incoming load
    // finished before the barrier of the last-but-one step) into 16-byte pieces, D/8 lanes per row.
    // Chunk c of row q is kept at chunk c ^ (q & kSwz) so that neither side meets a bank conflict.
    const float l_tot = halves_sum(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    {
        char *ob = smem + w * (32 * RB);
        const int qrow = l & 31;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)(acc[dt][4 * q4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(ob + qrow * RB + (((4 * dt + q4) ^ (qrow & kSwz<D>)) << 4) + 8 * half) = o;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int pc = l % LPR;
#pragma unroll
        for (int i = 0; i < 32 / RPL; ++i) {
            const int orow = RPL * i + l / LPR;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(ob + orow * RB + (pc << 4));
            if (32 * w + orow < q_len)
                *reinterpret_cast<u32x4 *>(O + ((size_t)(q_tok0 + 32 * w + orow) * hq + h) * D + ((pc ^ (orow & kSwz<D>)) << 3)) = v;
        }
    }
    if (q_local < q_len && lse != nullptr && half == 0)
        lse[(size_t)h * T + q_tok0 + q_local] = l_tot > 0.f ? m_run * c + __log2f(l_tot) : -INFINITY;
#undef FP_TILE_BLOCK
#undef FP_LOAD
#undef FP_LOAD_SAFE
#undef FP_LOAD_AT
#undef FP_ENT_OFF
#undef FP_LIM
#undef FP_KBUF
#undef FP_VBUF
#undef FP_STEP
}

}  // namespace fp
