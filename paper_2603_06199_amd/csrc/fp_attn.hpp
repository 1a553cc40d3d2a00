// Stage (iii): index-driven block-sparse attention (Sec. 3.5, Alg. 3) and, from the same
// template, full causal attention.  bf16 MFMA for both contractions, fp32 online softmax.
#pragma once
#include "fp_device.hpp"

namespace fp {

// LDS tiles of 64 keys.  K rows are padded to 272 bytes so that the 16-byte A-fragment reads of
// 16 consecutive rows fall on 16 distinct 4-bank groups; V rows are padded to 320 bytes so that
// the 4 rows a transpose read touches per lane group fall on 4 distinct 16-bank groups.
constexpr int kAttnTileKeys = 64;
constexpr int kAttnKStride = 272;
constexpr int kAttnVStride = 320;
constexpr int kAttnKTile = kAttnTileKeys * kAttnKStride;   // 17408
constexpr int kAttnVTile = kAttnTileKeys * kAttnVStride;   // 20480
constexpr int kAttnLds = 2 * kAttnKTile + 2 * kAttnVTile;  // 75776: two workgroups per CU

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
 *
 * Per tile and wave:
 *   S^T = K Q^T  (keys x queries, 16 MFMA 32x32x16): the query index is the lane column, so the
 *         row max and row sum of the softmax are reductions over a lane's own registers plus one
 *         exchange with lane^32;
 *   causal mask only if the tile belongs to the diagonal block (Alg. 3, is_diag);
 *   online softmax in base 2: p = 2^(c*s - c*m), the accumulator is rescaled only when some
 *         row's max moved;
 *   O^T += V^T P^T (16 MFMA): P^T is already in B-operand layout (registers of S^T, packed to
 *         bf16), V^T fragments come from the row-major V tile through LDS transpose reads.
 *
 * K/V tiles are staged global -> registers -> LDS one tile ahead, and the global loads are
 * issued two tiles ahead, with one barrier per tile.
 *
 * Work order: blockIdx -> (XCD, slot).  Consecutive workgroup ids land on different XCDs, each
 * with its own L2; slot k of XCD x takes query head k%g of super-item (k/g)*8 + x, where a
 * super-item is (row rank, KV head) and rows are ranked heaviest (largest I) first.  The g query
 * heads that share a KV head, and neighbouring rows of that KV head, therefore run on one XCD
 * at about the same time and find each other's K/V tiles in its L2.
 */
template <bool SPARSE>
__device__ __forceinline__ int attn_tile_block(const int32_t *list, int t, int I) {
    if (!SPARSE) return t >> 1;
    const int b = list[t >> 1];
    return b < 0 ? 0 : (b > I ? I : b);
}

template <bool SPARSE>
__global__ __launch_bounds__(256, 2) void attn_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ cnt, const BlockRec *__restrict__ blk,
    const int32_t *__restrict__ order, int m_total, int n_max, int hq, int hkv, int g, int T, float c,
    uint16_t *__restrict__ O, float *__restrict__ lse) {
    __shared__ __attribute__((aligned(16))) char smem[kAttnLds];

    const int x = blockIdx.x & 7, k = blockIdx.x >> 3;
    const int s = (k / g) * 8 + x, hg = k % g;
    if (s >= m_total * hkv) return;
    const int rank = s / hkv, hk = s - rank * hkv;
    const int r = order[rank];
    const int h = hk * g + hg;
    const BlockRec bi = blk[r];
    const int I = r - bi.z;
    const int seq_tok0 = bi.x - I * kBlock;
    const int last_tok = bi.w - 1;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, half = l >> 5;

    int nb = I + 1;
    const int32_t *list = nullptr;
    if (SPARSE) {
        list = idx + ((size_t)h * m_total + r) * n_max;
        nb = cnt[(size_t)h * m_total + r];
        nb = nb < 0 ? 0 : (nb > I + 1 ? I + 1 : nb);
    }
    const int ntiles = 2 * nb;

#define FP_TILE_BLOCK(t) attn_tile_block<SPARSE>(list, (t), I)

    // Q^T B-fragments: query 32w + l%32, dims 16ks + 8*half..+7.
    bf16x8 qb[8];
    {
        int row = 32 * w + (l & 31);
        row = row < bi.y ? row : bi.y - 1;
        const uint16_t *qp = Q + ((size_t)(bi.x + row) * hq + h) * kHeadDim + 8 * half;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qb[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
    }

    // Staging: thread (row = tid/16 + 16i, chunk = tid%16) moves 16 bytes of K and of V.
    u32x4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
    const int st_row = tid >> 4, st_chunk = tid & 15;
    // Loads use a wave-uniform base (first token of the tile, KV head) plus a per-thread 32-bit
    // byte offset, so the address is one scalar pair + one VGPR.  Only a tile that reaches past
    // the end of its sequence (ragged last block) needs per-row clamping.
    const uint32_t row_bytes = (uint32_t)hkv * kHeadDim * 2;
    const uint32_t st_off = (uint32_t)st_row * row_bytes + (uint32_t)st_chunk * 16;
    const char *Kb = reinterpret_cast<const char *>(K) + (size_t)hk * kHeadDim * 2;
    const char *Vb = reinterpret_cast<const char *>(V) + (size_t)hk * kHeadDim * 2;
#define FP_LOAD_ROW(i_, kr_, vr_)                                                                         \
    {                                                                                                     \
        uint32_t o_ = st_off + 16u * (i_) * row_bytes;                                                    \
        if (ragged_) {                                                                                    \
            int tok_ = tok0_ + st_row + 16 * (i_);                                                        \
            tok_ = tok_ < last_tok ? tok_ : last_tok; /* keys past the end are masked as future keys */   \
            o_ = (uint32_t)(tok_ - base_tok_) * row_bytes + (uint32_t)st_chunk * 16; /* tok_ >= base_tok_ */ \
        }                                                                                                 \
        kr_ = *reinterpret_cast<const u32x4 *>(kbase_ + o_);                                              \
        vr_ = *reinterpret_cast<const u32x4 *>(vbase_ + o_);                                              \
    }
#define FP_LOAD_TILE(t)                                                                                   \
    do {                                                                                                  \
        const int tok0_ = seq_tok0 + FP_TILE_BLOCK(t) * kBlock + ((t) & 1) * kAttnTileKeys;               \
        const bool ragged_ = tok0_ + kAttnTileKeys - 1 > last_tok;                                        \
        /* the base never lies past the sequence end, so the unsigned row offsets cannot wrap */          \
        const int base_tok_ = tok0_ < last_tok ? tok0_ : last_tok;                                        \
        const char *kbase_ = Kb + (size_t)base_tok_ * row_bytes;                                          \
        const char *vbase_ = Vb + (size_t)base_tok_ * row_bytes;                                          \
        FP_LOAD_ROW(0, kr0, vr0) FP_LOAD_ROW(1, kr1, vr1) FP_LOAD_ROW(2, kr2, vr2) FP_LOAD_ROW(3, kr3, vr3) \
    } while (0)
#define FP_STORE_ROW(i_, kr_, vr_)                                                                        \
    *reinterpret_cast<u32x4 *>(kd_ + 16 * (i_) * kAttnKStride) = kr_;                                     \
    *reinterpret_cast<u32x4 *>(vd_ + 16 * (i_) * kAttnVStride) = vr_;
#define FP_STORE_TILE(buf)                                                                                \
    do {                                                                                                  \
        char *kd_ = smem + (buf) * kAttnKTile + st_row * kAttnKStride + st_chunk * 16;                    \
        char *vd_ = smem + 2 * kAttnKTile + (buf) * kAttnVTile + st_row * kAttnVStride + st_chunk * 16;   \
        FP_STORE_ROW(0, kr0, vr0) FP_STORE_ROW(1, kr1, vr1) FP_STORE_ROW(2, kr2, vr2) FP_STORE_ROW(3, kr3, vr3) \
    } while (0)

    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_run = -INFINITY;   // running row max of the raw dot products (before scaling by c)
    float l_run = 0.f;         // this lane's share of the running row sum

    const int q_local = 32 * w + (l & 31);
    if (ntiles == 0) {   // empty list: O = 0, lse = -inf (uniform exit, before any barrier)
        if (q_local < bi.y) {
            uint16_t *op = O + ((size_t)(bi.x + q_local) * hq + h) * kHeadDim + 64 * half;
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4 *>(op + 8 * i) = z;
            if (lse != nullptr && half == 0) lse[(size_t)h * T + bi.x + q_local] = -INFINITY;
        }
        return;
    }
    FP_LOAD_TILE(0);
    // Pin the Q fragments here: the loads must have landed before the tile loop, otherwise the
    // compiler keeps a wait on vector-memory loads inside the loop's MFMA section, which in steady
    // state would wait for the K/V prefetch issued moments earlier.
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qb[ks]));
    FP_STORE_TILE(0);
    if (ntiles > 1) FP_LOAD_TILE(1);
    __syncthreads();

    const int k_frag = (l & 31) * kAttnKStride + half * 16;
    // transpose-read base: row 4*half + (l%16)/4, dims 16*((l%32)/16) + 4*(l%4)
    const int v_frag = 2 * kAttnKTile + (4 * half + ((l & 15) >> 2)) * kAttnVStride + (16 * ((l & 31) >> 4) + 4 * (l & 3)) * 2;

    for (int t = 0; t < ntiles; ++t) {
        const int cur = t & 1;
        if (t + 1 < ntiles) FP_STORE_TILE(cur ^ 1);
        if (t + 2 < ntiles) FP_LOAD_TILE(t + 2);

        const int koff = (t & 1) * kAttnTileKeys;
        const bool diag = FP_TILE_BLOCK(t) == I;
        if (!(diag && koff > 32 * w + 31)) {   // a diagonal tile wholly in this wave's future is skipped
            f32x16 s0, s1;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
            const char *kt = smem + cur * kAttnKTile + k_frag;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(kt + ks * 32);
                const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(kt + 32 * kAttnKStride + ks * 32);
                s0 = mfma32(a0, qb[ks], s0);
                s1 = mfma32(a1, qb[ks], s1);
            }
            if (diag) {
                // key (koff + 32kt + 8(i/4) + 4half + i%4) is in the future of query q_local
                const int lim = q_local - koff - 4 * half;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kk = 8 * (i >> 2) + (i & 3);
                    if (kk > lim) s0[i] = -INFINITY;
                    if (kk + 32 > lim) s1[i] = -INFINITY;
                }
            }
            float ta = max3(s0[0], s0[1], s0[2]), tb = max3(s1[0], s1[1], s1[2]);
#pragma unroll
            for (int i = 3; i < 15; i += 2) {
                ta = max3(ta, s0[i], s0[i + 1]);
                tb = max3(tb, s1[i], s1[i + 1]);
            }
            float tm = max3(ta, s0[15], max3(tb, s1[15], s1[15]));
            tm = fmaxf(tm, __shfl_xor(tm, 32));
            const float m_new = fmaxf(m_run, tm);
            if (__ballot(m_new > m_run)) {
                const float a = fast_exp2((m_run - m_new) * c);
                l_run *= a;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[dt][i] *= a;
                m_run = m_new;
            }
            const float mc = m_run * c;
            // p = 2^(c*s - c*m), rounded to bf16 for the PV product; the row sum is taken over the
            // rounded values (the ones that multiply V), two per VALU op.
            bf16x8 pb[2][2];
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                bf16x2 a, b;
                a[0] = (__bf16)fast_exp2(__builtin_fmaf(s0[i], c, -mc));
                a[1] = (__bf16)fast_exp2(__builtin_fmaf(s0[i + 1], c, -mc));
                b[0] = (__bf16)fast_exp2(__builtin_fmaf(s1[i], c, -mc));
                b[1] = (__bf16)fast_exp2(__builtin_fmaf(s1[i + 1], c, -mc));
                l_run = add_pair(a, l_run);
                l_run = add_pair(b, l_run);
                pb[0][i >> 3][i & 7] = a[0];
                pb[0][i >> 3][(i & 7) + 1] = a[1];
                pb[1][i >> 3][i & 7] = b[0];
                pb[1][i >> 3][(i & 7) + 1] = b[1];
            }
            const char *vt = smem + cur * kAttnVTile + v_frag;
#pragma unroll
            for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const char *vp = vt + (32 * kt2 + 16 * j) * kAttnVStride;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        const s16x4 lo = lds_read_tr(vp + dt * 64);
                        const s16x4 hi = lds_read_tr(vp + 8 * kAttnVStride + dt * 64);
                        const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        acc[dt] = mfma32(__builtin_bit_cast(bf16x8, a), pb[kt2][j], acc[dt]);
                    }
                }
        }
        __syncthreads();
    }

    // O = acc / l, lse = m + log2 l (Alg. 3, final normalisation); rows past a ragged end are not stored.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (q_local < bi.y) {
        uint16_t *op = O + ((size_t)(bi.x + q_local) * hq + h) * kHeadDim + 4 * half;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)(acc[dt][4 * q4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(op + 32 * dt + 8 * q4) = o;
            }
        if (lse != nullptr && half == 0)
            lse[(size_t)h * T + bi.x + q_local] = l_tot > 0.f ? m_run * c + __log2f(l_tot) : -INFINITY;
    }
#undef FP_TILE_BLOCK
#undef FP_LOAD_TILE
#undef FP_STORE_TILE
#undef FP_LOAD_ROW
#undef FP_STORE_ROW
}

}  // namespace fp
