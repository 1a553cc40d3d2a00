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
__global__ __launch_bounds__(256) void pool_k_kernel(const uint16_t *__restrict__ K, const BlockRec *__restrict__ blk,
                                                     int hkv, uint16_t *__restrict__ kb_hi,
                                                     uint16_t *__restrict__ kb_lo) {
    __shared__ float red[16][kHeadDim + 4];
    const int r = blockIdx.x, hk = blockIdx.y;
    const BlockRec bi = blk[r];
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
// Alg. 1 stages 2 and 3, fused.  One workgroup per (q-block row, KV head, group of 4 query
// heads); wave w owns query head 4*chunk + w of the group and keeps that head's whole 128x128
// query tile in registers as MFMA A-fragments (128 VGPRs).  Pooled keys stream through LDS in
// tiles of 32 blocks (hi and lo planes, shared by the four waves, double buffered).  For each
// tile a wave computes the 128 x 32 logits with 64 MFMAs (4 query sub-tiles x 8 k-slices x
// {hi, lo}); the result layout puts one pooled key per lane column, so the reduction over the
// query axis (Eq. 1-2: max, then sum of 2^(x - max)) is in-register plus one lane exchange.
// (m, S) per block pair stay in LDS; after the last tile the wave takes the row max, rescales
// (Eq. 3) and writes the normalised row (Eq. 4) once.  Nothing of size L x L/B ever exists.
// ---------------------------------------------------------------------------------------------
constexpr int kSearchKbStride = 272;                      // bytes per pooled-key row in LDS (256 + 16 pad)
constexpr int kSearchPlane = 32 * kSearchKbStride;        // one plane (hi or lo) of a 32-row tile
constexpr int kSearchStage = 2 * kSearchPlane;            // hi + lo
constexpr int kSearchStageBytes = 2 * kSearchStage;       // double buffered

__global__ __launch_bounds__(256, 1) void search_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ kb_hi, const uint16_t *__restrict__ kb_lo,
    const BlockRec *__restrict__ blk, const int32_t *__restrict__ order, int m_total, int n_max, int n_pad, int hq,
    int hkv, int g, int nchunk, float c /* tau*log2(e) */, float eps, float *__restrict__ scores) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float2 *ms_all = reinterpret_cast<float2 *>(smem + kSearchStageBytes);

    const int per_row = hkv * nchunk;
    const int rank = blockIdx.x / per_row;
    const int rem = blockIdx.x - rank * per_row;
    const int hk = rem / nchunk, ch = rem - hk * nchunk;
    const int r = order[rank];
    const BlockRec bi = blk[r];
    const int I = r - bi.z;
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int hg = ch * 4 + w;
    const bool active = hg < g;
    const int h = hk * g + (active ? hg : g - 1);
    float2 *ms = ms_all + (size_t)w * n_pad;

    // Query tile as A-fragments: qa[qt][ks] covers queries 32qt + l%32, dims 16ks + 8(l/32)..+7.
    bf16x8 qa[4][8];
    {
        const int half = l >> 5;
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            int row = 32 * qt + (l & 31);
            row = row < bi.y ? row : bi.y - 1;   // rows past a ragged end are masked below
            const uint16_t *qp = Q + ((size_t)(bi.x + row) * hq + h) * kHeadDim + 8 * half;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) qa[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
        }
    }

    const int ntile = I / 32 + 1;
    u32x4 sg0, sg1, sg2, sg3;
    // Stage loader: 1024 16-byte chunks per tile (2 planes x 32 rows x 16 chunks), 4 per thread:
    // thread -> (plane = i/2, row = tid/16 + 16*(i%2), col = tid%16) for i = 0..3
    const int st_row = tid >> 4, st_col = tid & 15;
#define FP_LOAD_ROW(i_, sg_)                                                                              \
    {                                                                                                     \
        int J_ = jbase_ + 16 * ((i_) & 1);                                                                \
        J_ = J_ <= I ? J_ : I; /* columns past the diagonal are computed and dropped */                   \
        sg_ = *reinterpret_cast<const u32x4 *>((((i_) >> 1) ? kb_lo : kb_hi) +                            \
                                               ((size_t)(bi.z + J_) * hkv + hk) * kHeadDim + st_col * 8); \
    }
#define FP_LOAD_TILE(jt)                                                                                  \
    do {                                                                                                  \
        const int jbase_ = 32 * (jt) + st_row;                                                            \
        FP_LOAD_ROW(0, sg0) FP_LOAD_ROW(1, sg1) FP_LOAD_ROW(2, sg2) FP_LOAD_ROW(3, sg3)                   \
    } while (0)
#define FP_STORE_ROW(i_, sg_)                                                                             \
    *reinterpret_cast<u32x4 *>(sd_ + ((i_) >> 1) * kSearchPlane + 16 * ((i_) & 1) * kSearchKbStride) = sg_;
#define FP_STORE_TILE(buf)                                                                                \
    do {                                                                                                  \
        char *sd_ = smem + (buf) * kSearchStage + st_row * kSearchKbStride + st_col * 16;                 \
        FP_STORE_ROW(0, sg0) FP_STORE_ROW(1, sg1) FP_STORE_ROW(2, sg2) FP_STORE_ROW(3, sg3)               \
    } while (0)

    FP_LOAD_TILE(0);
    // Pin the Q fragments: their loads must have landed before the tile loop, or the compiler
    // leaves waits on vector-memory loads between the loop's MFMAs (which in steady state would
    // wait for the pooled-key prefetch issued just before).
#pragma unroll
    for (int qt = 0; qt < 4; ++qt)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qa[qt][ks]));
    FP_STORE_TILE(0);
    if (ntile > 1) FP_LOAD_TILE(1);
    __syncthreads();

    const int frag_off = (l & 31) * kSearchKbStride + (l >> 5) * 16;
    for (int jt = 0; jt < ntile; ++jt) {
        const int cur = jt & 1;
        if (jt + 1 < ntile) FP_STORE_TILE(cur ^ 1);
        if (jt + 2 < ntile) FP_LOAD_TILE(jt + 2);
        if (active) {
            f32x16 acc[4];
#pragma unroll
            for (int qt = 0; qt < 4; ++qt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[qt][i] = 0.f;
            const char *tile = smem + cur * kSearchStage + frag_off;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 bh = *reinterpret_cast<const bf16x8 *>(tile + ks * 32);
                const bf16x8 bl = *reinterpret_cast<const bf16x8 *>(tile + kSearchPlane + ks * 32);
#pragma unroll
                for (int qt = 0; qt < 4; ++qt) acc[qt] = mfma32(qa[qt][ks], bh, acc[qt]);
#pragma unroll
                for (int qt = 0; qt < 4; ++qt) acc[qt] = mfma32(qa[qt][ks], bl, acc[qt]);
            }
            if (bi.y < kBlock) {   // ragged last q-block: leave missing queries out of max and sum
#pragma unroll
                for (int qt = 0; qt < 4; ++qt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int row = 32 * qt + 8 * (i >> 2) + 4 * (l >> 5) + (i & 3);
                        if (row >= bi.y) acc[qt][i] = -INFINITY;
                    }
            }
            float mx = max3(acc[0][0], acc[1][0], acc[2][0]);
            mx = max3(mx, acc[3][0], acc[3][0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) {
                mx = max3(mx, acc[0][i], acc[1][i]);
                mx = max3(mx, acc[2][i], acc[3][i]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mc = mx * c;
            float sum = 0.f;
#pragma unroll
            for (int qt = 0; qt < 4; ++qt)
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += fast_exp2(__builtin_fmaf(acc[qt][i], c, -mc));
            sum += __shfl_xor(sum, 32);
            const int J = 32 * jt + (l & 31);
            if (l < 32 && J <= I) ms[J] = make_float2(mc, sum);
        }
        __syncthreads();
    }

#undef FP_LOAD_TILE
#undef FP_STORE_TILE
#undef FP_LOAD_ROW
#undef FP_STORE_ROW
    if (!active) return;
    // Eq. 3-4: row max of the pair maxima, rescale, normalise, write the row once.
    float M = -INFINITY;
    for (int J = l; J <= I; J += 64) M = fmaxf(M, ms[J].x);
    M = wave_max(M);
    float tot = 0.f;
    for (int J = l; J <= I; J += 64) {
        const float2 v = ms[J];
        tot += v.y * fast_exp2(v.x - M);
    }
    tot = wave_sum(tot);
    const float denom = tot + eps;
    float *out = scores + ((size_t)h * m_total + r) * n_max;
    for (int J = l; J < n_max; J += 64) {
        float p = 0.f;
        if (J <= I) {
            const float2 v = ms[J];
            p = (v.y * fast_exp2(v.x - M)) / denom;
        }
        out[J] = p;
    }
}

// ---------------------------------------------------------------------------------------------
// Alg. 2.  One wave per (head, q-block row).  Pass 1: row max over J <= I with coalesced loads
// and a wave reduction.  Pass 2: 64 candidates at a time, the keep decision
// (score >= alpha*max, or sink, or window) becomes a ballot; the popcount of the lower lanes is
// each kept block's slot, so the ascending list comes out without a sort or a scan over memory.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void threshold_kernel(const float *__restrict__ scores,
                                                        const BlockRec *__restrict__ blk, int m_total, int n_max,
                                                        int hq, float alpha, int sinkB, int winB,
                                                        int32_t *__restrict__ idx, int32_t *__restrict__ cnt) {
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    if (wave >= hq * m_total) return;
    const int r = wave % m_total;   // wave = h*m_total + r
    const int I = r - blk[r].z;
    const float *row = scores + (size_t)wave * n_max;
    int32_t *out = idx + (size_t)wave * n_max;

    float mx = -INFINITY;
    for (int J = l; J <= I; J += 64) mx = fmaxf(mx, row[J]);
    mx = wave_max(mx);
    const float thr = __fmul_rn(alpha, mx);   // one fp32 rounding, as the reference decision

    int count = 0;
    for (int base = 0; base <= I; base += 64) {
        const int J = base + l;
        bool keep = false;
        if (J <= I) keep = (row[J] >= thr) || (J < sinkB) || (I - J < winB);
        const unsigned long long bal = __ballot(keep);
        if (keep) out[count + __builtin_popcountll(bal & ((1ull << l) - 1ull))] = J;
        count += __builtin_popcountll(bal);
    }
    if (l == 0) cnt[wave] = count;
}

}  // namespace fp
