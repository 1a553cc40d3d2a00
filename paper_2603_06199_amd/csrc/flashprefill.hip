// Host side of the C ABI declared in include/flashprefill.h: shape validation, the plan
// (device tables + workspace) and the kernel launches.  gfx950 only.
#include "../../include/flashprefill.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "fp_attn.hpp"
#include "fp_device.hpp"
#include "fp_search.hpp"

// Built-in scratch for fp_block_search_static: the two pooled-key planes of one call.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and host calls use the per-device address.
constexpr size_t kStaticScratchBytes = FP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of the calling thread's current device's copy of `scratch`; looked up once per device.
// `device` must be the current device.  Returns nullptr on failure.
void *static_scratch(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[device] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}

// (m, S) of one row for 2 heads must fit the score kernel's LDS next to its tile buffers
// (2 x 16 KB + 1 KB + 2 x 8 B x blocks <= 160 KB would allow more; 4096 blocks = 512K tokens)
constexpr int kMaxBlocksPerSeq = 4096;

struct Layout {
    int m_total = 0, n_max = 0, kb_total = 0;
    std::vector<int32_t> row_offset;   // first q-block row of each sequence
    std::vector<int32_t> kb_offset;    // first key block of each sequence among all key blocks
    std::vector<int32_t> prefix_blocks;
};

fp_status check_shape(const fp_shape *s, Layout *out) {
    if (s == nullptr || s->cu_seqlens == nullptr) return FP_ERR_INVALID_ARG;
    if (s->nseq < 1 || s->hq < 1 || s->hkv < 1 || s->hq % s->hkv != 0) return FP_ERR_INVALID_ARG;
    const int32_t *cuk = s->cu_seqlens_k ? s->cu_seqlens_k : s->cu_seqlens;
    if (s->cu_seqlens[0] != 0 || cuk[0] != 0) return FP_ERR_INVALID_ARG;
    for (int i = 0; i < s->nseq; ++i)
        if (s->cu_seqlens[i + 1] <= s->cu_seqlens[i] || cuk[i + 1] <= cuk[i]) return FP_ERR_INVALID_ARG;
    if (!(s->scale == s->scale) || std::isinf(s->scale)) return FP_ERR_INVALID_ARG;
    // head dimension 64 / 128 / 256 at block 128; block 64 / 256 at head dimension 128
    if (!(((s->head_dim == 64 || s->head_dim == 256) && s->block == 128) ||
          (s->head_dim == 128 && (s->block == 64 || s->block == 128 || s->block == 256))))
        return FP_ERR_UNSUPPORTED;
    Layout L;
    L.row_offset.assign((size_t)s->nseq + 1, 0);
    L.kb_offset.assign((size_t)s->nseq + 1, 0);
    L.prefix_blocks.assign((size_t)s->nseq, 0);
    for (int i = 0; i < s->nseq; ++i) {
        const int64_t qlen = (int64_t)s->cu_seqlens[i + 1] - s->cu_seqlens[i];
        const int64_t klen = (int64_t)cuk[i + 1] - cuk[i];
        const int64_t prefix = klen - qlen;
        if (prefix < 0) return FP_ERR_INVALID_ARG;
        if (prefix % s->block != 0) return FP_ERR_UNSUPPORTED;
        const int64_t nkb = (klen + s->block - 1) / s->block;
        if (nkb > kMaxBlocksPerSeq) return FP_ERR_UNSUPPORTED;
        L.n_max = std::max<int>(L.n_max, (int)nkb);
        L.prefix_blocks[i] = (int32_t)(prefix / s->block);
        L.row_offset[i + 1] = L.row_offset[i] + (int32_t)((qlen + s->block - 1) / s->block);
        L.kb_offset[i + 1] = L.kb_offset[i] + (int32_t)nkb;
    }
    L.m_total = L.row_offset[s->nseq];
    L.kb_total = L.kb_offset[s->nseq];
    if (out) *out = std::move(L);
    return FP_OK;
}

int search_stage_bytes(int head_dim, int block) {
    if (head_dim == 64) return fp::kSearchStageBytes<64, 128>;
    if (head_dim == 256) return fp::kSearchStageBytes<256, 128>;
    return block == 64 ? fp::kSearchStageBytes<128, 64> : block == 128 ? fp::kSearchStageBytes<128, 128> : fp::kSearchStageBytes<128, 256>;
}
int search_heads_per_wg(int block) { return block == 64 ? 4 : block == 128 ? 2 : 1; }

template <int D, int BLK>
bool set_lds_ceilings() {
    const int search_lds_max = fp::kSearchStageBytes<D, BLK> + fp::kSearchRowHeader +
                               fp::kSearchHeads<BLK> * kMaxBlocksPerSeq * (int)sizeof(float) + fp::kSearchCandBytes;
    bool ok = hipFuncSetAttribute(reinterpret_cast<const void *>(fp::search_kernel<D, BLK, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, search_lds_max) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(fp::search_kernel<D, BLK, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, search_lds_max) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(fp::attn_kernel<D, BLK, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, fp::kAttnLds<D, BLK>) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(fp::attn_kernel<D, BLK, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, fp::kAttnLds<D, BLK>) == hipSuccess;
    return ok;
}

}  // namespace

struct fp_plan {
    int device = 0;
    int nseq = 0, hq = 0, hkv = 0, g = 0, T = 0;   // T: query tokens
    int head_dim = 0, block = 0;
    int m_total = 0, n_max = 0, kb_total = 0;
    float c = 0.f;                    // tau * log2(e)
    fp::RowRec *d_rows = nullptr;     // [m_total]
    int32_t *d_order = nullptr;       // [m_total] rows, most causal key blocks first
    fp::RowRec *d_rows_ranked = nullptr;   // [m_total] d_rows permuted by d_order
    fp::KeyBlockRec *d_kblk = nullptr;     // [kb_total]
    uint16_t *d_kb_hi = nullptr;      // [kb_total, hkv, 128] bf16
    uint16_t *d_kb_lo = nullptr;
    float2 *d_kb_norm = nullptr;      // [kb_total, hkv] (|pooled key|, |its lo plane|)
    void *workspace = nullptr;        // the one device buffer all of the above are carved from
    bool owns_workspace = false;      // true: allocated by fp_plan_create, freed by fp_plan_destroy
    size_t search_lds = 0;
    int n_pad = 0;
};

namespace {

// The plan's device memory is one buffer: row records by row and by rank, the rank order, the
// key-block records and the two pooled-key planes, each part starting on a 256-byte boundary.
constexpr size_t kWsAlign = 256;
struct WorkspaceMap {
    size_t rows = 0, rows_ranked = 0, order = 0, kblk = 0, kb_hi = 0, kb_lo = 0, kb_norm = 0, total = 0;
};
WorkspaceMap workspace_map(const Layout &L, int hkv, int head_dim) {
    WorkspaceMap m;
    size_t off = 0;
    auto take = [&off](size_t bytes) {
        const size_t at = off;
        off += (bytes + kWsAlign - 1) / kWsAlign * kWsAlign;
        return at;
    };
    const size_t kb_bytes = (size_t)L.kb_total * hkv * head_dim * sizeof(uint16_t);
    m.rows = take((size_t)L.m_total * sizeof(fp::RowRec));
    m.rows_ranked = take((size_t)L.m_total * sizeof(fp::RowRec));
    m.order = take((size_t)L.m_total * sizeof(int32_t));
    m.kblk = take((size_t)L.kb_total * sizeof(fp::KeyBlockRec));
    m.kb_hi = take(kb_bytes);
    m.kb_lo = take(kb_bytes);
    m.kb_norm = take((size_t)L.kb_total * hkv * sizeof(float2));
    m.total = off;
    return m;
}

}  // namespace

extern "C" {

const char *fp_status_string(fp_status s) {
    switch (s) {
        case FP_OK: return "ok";
        case FP_ERR_INVALID_ARG: return "invalid argument";
        case FP_ERR_UNSUPPORTED: return "unsupported shape (head_dim 64, 128 or 256 with block 128, or head_dim 128 with block 64 or 256; at most 4096 blocks per sequence; a KV prefix a multiple of the block)";
        case FP_ERR_DEVICE: return "HIP device error";
        case FP_ERR_NOMEM: return "out of host memory";
        case FP_ERR_STATIC_LIMIT:
            return "shape needs more pooled-key scratch than the library's built-in array holds (fp_block_search_static: "
                   "key blocks x Hkv <= 16384 at head_dim 128); use fp_block_search";
        case FP_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned (see fp_workspace_bytes)";
    }
    return "unknown status";
}

fp_status fp_layout(const fp_shape *shape, int32_t *m_total, int32_t *n_max, int32_t *row_offset) {
    Layout L;
    const fp_status st = check_shape(shape, &L);
    if (st != FP_OK) return st;
    if (m_total) *m_total = L.m_total;
    if (n_max) *n_max = L.n_max;
    if (row_offset) std::copy(L.row_offset.begin(), L.row_offset.end(), row_offset);
    return FP_OK;
}

size_t fp_workspace_bytes(const fp_shape *shape) {
    Layout L;
    if (check_shape(shape, &L) != FP_OK) return 0;
    return workspace_map(L, shape->hkv, shape->head_dim).total;
}

void fp_plan_destroy(fp_plan *p) {
    if (p == nullptr) return;
    if (p->owns_workspace && p->workspace != nullptr) {
        int prev = 0;
        const bool have_prev = hipGetDevice(&prev) == hipSuccess;
        if (hipSetDevice(p->device) == hipSuccess) (void)hipFree(p->workspace);
        if (have_prev) (void)hipSetDevice(prev);
    }
    delete p;
}

fp_status fp_plan_create(const fp_shape *shape, int device, fp_plan **out) {
    return fp_plan_create_in(shape, device, nullptr, 0, out);
}

fp_status fp_plan_create_in(const fp_shape *shape, int device, void *workspace, size_t workspace_bytes, fp_plan **out) {
    if (out == nullptr) return FP_ERR_INVALID_ARG;
    *out = nullptr;
    Layout L;
    const fp_status st = check_shape(shape, &L);
    if (st != FP_OK) return st;
    const WorkspaceMap wm = workspace_map(L, shape->hkv, shape->head_dim);
    if (workspace != nullptr && (workspace_bytes < wm.total || reinterpret_cast<uintptr_t>(workspace) % kWsAlign != 0))
        return FP_ERR_WORKSPACE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return FP_ERR_DEVICE;

    fp_plan *p = new (std::nothrow) fp_plan();
    if (p == nullptr) return FP_ERR_NOMEM;
    p->device = device;
    p->nseq = shape->nseq;
    p->hq = shape->hq;
    p->hkv = shape->hkv;
    p->g = shape->hq / shape->hkv;
    p->head_dim = shape->head_dim;
    p->block = shape->block;
    p->T = shape->cu_seqlens[shape->nseq];
    p->m_total = L.m_total;
    p->n_max = L.n_max;
    p->kb_total = L.kb_total;
    const float tau = shape->scale > 0.f ? shape->scale : 1.0f / std::sqrt((float)shape->head_dim);
    p->c = tau * fp::kLog2e;
    p->n_pad = (L.n_max + 31) / 32 * 32;
    p->search_lds = (size_t)search_stage_bytes(shape->head_dim, shape->block) + fp::kSearchRowHeader +
                    (size_t)search_heads_per_wg(shape->block) * p->n_pad * sizeof(float) + fp::kSearchCandBytes;

    const int32_t *cuk = shape->cu_seqlens_k ? shape->cu_seqlens_k : shape->cu_seqlens;
    std::vector<fp::RowRec> rows((size_t)L.m_total);
    std::vector<fp::KeyBlockRec> kblk((size_t)L.kb_total);
    for (int s = 0; s < shape->nseq; ++s) {
        const int a = shape->cu_seqlens[s], b = shape->cu_seqlens[s + 1];
        for (int r = L.row_offset[s]; r < L.row_offset[s + 1]; ++r) {
            const int Iq = r - L.row_offset[s];
            const int t0 = a + Iq * shape->block;
            fp::RowRec rec;
            rec.q_tok0 = t0;
            rec.q_len = std::min(shape->block, b - t0);
            rec.I = Iq + L.prefix_blocks[s];
            rec.kb_row0 = L.kb_offset[s];
            rec.k_tok0 = cuk[s];
            rec.k_end = cuk[s + 1];
            rec.n_kb = L.kb_offset[s + 1] - L.kb_offset[s];
            rec.pad1 = 0;
            rows[(size_t)r] = rec;
        }
        for (int j = L.kb_offset[s]; j < L.kb_offset[s + 1]; ++j) {
            const int t0 = cuk[s] + (j - L.kb_offset[s]) * shape->block;
            kblk[(size_t)j] = make_int2(t0, std::min(shape->block, cuk[s + 1] - t0));
        }
    }
    // Heaviest rows first: a row's work grows with the number of its causal key blocks.
    std::vector<int32_t> order((size_t)L.m_total);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t x, int32_t y) { return rows[(size_t)x].I > rows[(size_t)y].I; });

    std::vector<fp::RowRec> rows_ranked((size_t)L.m_total);
    for (int i = 0; i < L.m_total; ++i) rows_ranked[(size_t)i] = rows[(size_t)order[(size_t)i]];

    int prev = 0;
    (void)hipGetDevice(&prev);
    bool ok = hipSetDevice(device) == hipSuccess;
    if (workspace != nullptr) {
        p->workspace = workspace;
    } else {
        ok = ok && hipMalloc(&p->workspace, wm.total) == hipSuccess;
        p->owns_workspace = ok;
    }
    ok = ok && static_scratch(device) != nullptr;   // set-up of the built-in scratch, once per device
    if (ok) {
        char *base = static_cast<char *>(p->workspace);
        p->d_rows = reinterpret_cast<fp::RowRec *>(base + wm.rows);
        p->d_rows_ranked = reinterpret_cast<fp::RowRec *>(base + wm.rows_ranked);
        p->d_order = reinterpret_cast<int32_t *>(base + wm.order);
        p->d_kblk = reinterpret_cast<fp::KeyBlockRec *>(base + wm.kblk);
        p->d_kb_hi = reinterpret_cast<uint16_t *>(base + wm.kb_hi);
        p->d_kb_lo = reinterpret_cast<uint16_t *>(base + wm.kb_lo);
        p->d_kb_norm = reinterpret_cast<float2 *>(base + wm.kb_norm);
    }
    ok = ok && hipMemcpy(p->d_rows, rows.data(), rows.size() * sizeof(fp::RowRec), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_kblk, kblk.data(), kblk.size() * sizeof(fp::KeyBlockRec), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_order, order.data(), order.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_rows_ranked, rows_ranked.data(), rows.size() * sizeof(fp::RowRec), hipMemcpyHostToDevice) == hipSuccess;
    // The dynamic-LDS ceilings are per kernel, not per plan: they are set to what the largest
    // supported shape needs, so that plans of different sizes can be alive together.
    ok = ok && set_lds_ceilings<64, 128>() && set_lds_ceilings<128, 64>() && set_lds_ceilings<128, 128>() &&
         set_lds_ceilings<128, 256>() && set_lds_ceilings<256, 128>();
    const int thr_lds_max = fp::kThresholdWaves * kMaxBlocksPerSeq * (int)sizeof(float);
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(fp::threshold_kernel<true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, thr_lds_max) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(fp::threshold_kernel<false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, thr_lds_max) == hipSuccess;
    (void)hipSetDevice(prev);
    if (!ok) {
        (void)hipGetLastError();
        fp_plan_destroy(p);
        return FP_ERR_DEVICE;
    }
    *out = p;
    return FP_OK;
}

static fp_status launch_status() { return hipGetLastError() == hipSuccess ? FP_OK : FP_ERR_DEVICE; }

// Kernels are enqueued on the calling thread's current device, which must be the plan's.
static bool on_plan_device(const fp_plan *p) {
    int cur = -1;
    return hipGetDevice(&cur) == hipSuccess && cur == p->device;
}

extern "C++" {
template <int D, int BLK>
static fp_status launch_search_d(fp_plan *p, const void *Q, const void *K, float eps, float *scores,
                                 const fp::SelectArgs *sel, hipStream_t st, uint16_t *kb_hi, uint16_t *kb_lo,
                                 float2 *kb_norm) {
    fp::pool_k_kernel<D><<<dim3(p->kb_total, p->hkv), 256, 0, st>>>(static_cast<const uint16_t *>(K), p->d_kblk, p->hkv,
                                                                     p->c, kb_hi, kb_lo, kb_norm);
    const int nchunk = (p->g + fp::kSearchHeads<BLK> - 1) / fp::kSearchHeads<BLK>;
    const dim3 grid(p->m_total * p->hkv * nchunk);
    const uint16_t *q = static_cast<const uint16_t *>(Q);
    if (sel != nullptr)
        fp::search_kernel<D, BLK, true><<<grid, 256, p->search_lds, st>>>(q, kb_hi, kb_lo, kb_norm, p->d_rows_ranked, p->d_order,
                                                                     p->m_total, p->n_max, p->n_pad, p->hq, p->hkv, p->g, nchunk,
                                                                     eps, nullptr, *sel);
    else
        fp::search_kernel<D, BLK, false><<<grid, 256, p->search_lds, st>>>(q, kb_hi, kb_lo, kb_norm, p->d_rows_ranked, p->d_order,
                                                                      p->m_total, p->n_max, p->n_pad, p->hq, p->hkv, p->g, nchunk,
                                                                      eps, scores, fp::SelectArgs{});
    return launch_status();
}
}  // extern "C++"

// Alg. 1 stage 1 and stages 2-3; `sel` non-null selects the variant that applies Alg. 2 in place.
static fp_status launch_search(fp_plan *p, const void *Q, const void *K, float eps, float *scores,
                               const fp::SelectArgs *sel, void *hip_stream, uint16_t *kb_hi = nullptr,
                               uint16_t *kb_lo = nullptr, float2 *kb_norm = nullptr) {
    if (!on_plan_device(p)) return FP_ERR_DEVICE;
    if (kb_hi == nullptr) {   // the plan's own pooled-key planes
        kb_hi = p->d_kb_hi;
        kb_lo = p->d_kb_lo;
        kb_norm = p->d_kb_norm;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    switch (p->head_dim) {
        case 64: return launch_search_d<64, 128>(p, Q, K, eps, scores, sel, st, kb_hi, kb_lo, kb_norm);
        case 256: return launch_search_d<256, 128>(p, Q, K, eps, scores, sel, st, kb_hi, kb_lo, kb_norm);
        default: break;
    }
    switch (p->block) {
        case 64: return launch_search_d<128, 64>(p, Q, K, eps, scores, sel, st, kb_hi, kb_lo, kb_norm);
        case 256: return launch_search_d<128, 256>(p, Q, K, eps, scores, sel, st, kb_hi, kb_lo, kb_norm);
        default: return launch_search_d<128, 128>(p, Q, K, eps, scores, sel, st, kb_hi, kb_lo, kb_norm);
    }
}

static bool params_ok(const fp_params *params) {
    return params != nullptr && params->sink_tokens >= 0 && params->window_tokens >= 0 && params->alpha == params->alpha;
}

fp_status fp_block_search(fp_plan *p, const void *Q, const void *K, float eps, float *scores, void *hip_stream) {
    if (p == nullptr || Q == nullptr || K == nullptr || scores == nullptr || !(eps >= 0.f)) return FP_ERR_INVALID_ARG;
    return launch_search(p, Q, K, eps, scores, nullptr, hip_stream);
}

fp_status fp_block_search_static(fp_plan *p, const void *Q, const void *K, float eps, float *scores, void *hip_stream) {
    if (p == nullptr || Q == nullptr || K == nullptr || scores == nullptr || !(eps >= 0.f)) return FP_ERR_INVALID_ARG;
    const size_t plane = ((size_t)p->kb_total * p->hkv * p->head_dim * sizeof(uint16_t) + kWsAlign - 1) / kWsAlign * kWsAlign;
    const size_t norms = (size_t)p->kb_total * p->hkv * sizeof(float2);
    if (2 * plane + norms > kStaticScratchBytes) return FP_ERR_STATIC_LIMIT;
    if (!on_plan_device(p)) return FP_ERR_DEVICE;
    char *base = static_cast<char *>(static_scratch(p->device));
    if (base == nullptr) return FP_ERR_DEVICE;
    return launch_search(p, Q, K, eps, scores, nullptr, hip_stream, reinterpret_cast<uint16_t *>(base),
                         reinterpret_cast<uint16_t *>(base + plane), reinterpret_cast<float2 *>(base + 2 * plane));
}

fp_status fp_search_select(fp_plan *p, const void *Q, const void *K, float eps, const fp_params *params, int32_t *idx,
                           int32_t *cnt, void *hip_stream) {
    if (p == nullptr || Q == nullptr || K == nullptr || idx == nullptr || cnt == nullptr || !(eps >= 0.f) || !params_ok(params))
        return FP_ERR_INVALID_ARG;
    fp::SelectArgs sel;
    sel.alpha = params->alpha;
    sel.sinkB = (params->sink_tokens + p->block - 1) / p->block;
    sel.winB = (params->window_tokens + p->block - 1) / p->block;
    sel.idx = idx;
    sel.cnt = cnt;
    return launch_search(p, Q, K, eps, nullptr, &sel, hip_stream);
}

fp_status fp_threshold(fp_plan *p, const float *scores, const fp_params *params, int32_t *idx, int32_t *cnt,
                       void *hip_stream) {
    if (p == nullptr || scores == nullptr || idx == nullptr || cnt == nullptr || !params_ok(params))
        return FP_ERR_INVALID_ARG;
    if (!on_plan_device(p)) return FP_ERR_DEVICE;
    const int sinkB = (params->sink_tokens + p->block - 1) / p->block;
    const int winB = (params->window_tokens + p->block - 1) / p->block;
    const int rows = p->hq * p->m_total;
    const int n_pad = (p->n_max + 63) / 64 * 64;
    const dim3 grid((rows + fp::kThresholdWaves - 1) / fp::kThresholdWaves);
    const size_t lds = (size_t)fp::kThresholdWaves * n_pad * sizeof(float);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (p->n_max % 4 == 0 && reinterpret_cast<uintptr_t>(scores) % 16 == 0)
        fp::threshold_kernel<true><<<grid, 64 * fp::kThresholdWaves, lds, st>>>(scores, p->d_rows, p->m_total, p->n_max, n_pad, p->hq,
                                                                               params->alpha, sinkB, winB, idx, cnt);
    else
        fp::threshold_kernel<false><<<grid, 64 * fp::kThresholdWaves, lds, st>>>(scores, p->d_rows, p->m_total, p->n_max, n_pad, p->hq,
                                                                                params->alpha, sinkB, winB, idx, cnt);
    return launch_status();
}

extern "C++" {
template <int D, int BLK>
static fp_status launch_attn_d(fp_plan *p, bool sparse, const void *Q, const void *K, const void *V, const int32_t *idx,
                               const int32_t *cnt, void *O, float *lse, hipStream_t st) {
    const int n_super = p->m_total * p->hkv;
    const int grid = (n_super + 7) / 8 * 8 * p->g * (BLK > 128 ? BLK / 128 : 1);   // a 256-query block takes two workgroups
    const uint16_t *q = static_cast<const uint16_t *>(Q), *k = static_cast<const uint16_t *>(K),
                   *v = static_cast<const uint16_t *>(V);
    uint16_t *o = static_cast<uint16_t *>(O);
    if (sparse)
        fp::attn_kernel<D, BLK, true><<<dim3(grid), 64 * fp::kAttnWaves<BLK>, fp::kAttnLds<D, BLK>, st>>>(q, k, v, idx, cnt, p->d_rows_ranked, p->d_order, p->m_total,
                                                                          p->n_max, p->hq, p->hkv, p->g, p->T, p->c, o, lse);
    else
        fp::attn_kernel<D, BLK, false><<<dim3(grid), 64 * fp::kAttnWaves<BLK>, fp::kAttnLds<D, BLK>, st>>>(q, k, v, nullptr, nullptr, p->d_rows_ranked, p->d_order,
                                                                           p->m_total, p->n_max, p->hq, p->hkv, p->g, p->T, p->c, o, lse);
    return launch_status();
}
}  // extern "C++"

static fp_status launch_attn(fp_plan *p, bool sparse, const void *Q, const void *K, const void *V, const int32_t *idx,
                             const int32_t *cnt, void *O, float *lse, void *hip_stream) {
    if (!on_plan_device(p)) return FP_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    switch (p->head_dim) {
        case 64: return launch_attn_d<64, 128>(p, sparse, Q, K, V, idx, cnt, O, lse, st);
        case 256: return launch_attn_d<256, 128>(p, sparse, Q, K, V, idx, cnt, O, lse, st);
        default: break;
    }
    switch (p->block) {
        case 64: return launch_attn_d<128, 64>(p, sparse, Q, K, V, idx, cnt, O, lse, st);
        case 256: return launch_attn_d<128, 256>(p, sparse, Q, K, V, idx, cnt, O, lse, st);
        default: return launch_attn_d<128, 128>(p, sparse, Q, K, V, idx, cnt, O, lse, st);
    }
}

fp_status fp_sparse_prefill(fp_plan *p, const void *Q, const void *K, const void *V, const int32_t *idx,
                            const int32_t *cnt, void *O, float *lse, void *hip_stream) {
    if (p == nullptr || Q == nullptr || K == nullptr || V == nullptr || idx == nullptr || cnt == nullptr || O == nullptr)
        return FP_ERR_INVALID_ARG;
    return launch_attn(p, true, Q, K, V, idx, cnt, O, lse, hip_stream);
}

fp_status fp_dense_prefill(fp_plan *p, const void *Q, const void *K, const void *V, void *O, float *lse,
                           void *hip_stream) {
    if (p == nullptr || Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return FP_ERR_INVALID_ARG;
    return launch_attn(p, false, Q, K, V, nullptr, nullptr, O, lse, hip_stream);
}

}  // extern "C"
