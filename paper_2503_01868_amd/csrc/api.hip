// C ABI of the library: argument validation (before any HIP call), kernel selection, tuning options.
#include <string.h>

#include <mutex>

#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {

namespace {
std::mutex g_tuning_mu;
Tuning g_tuning;                   // process-wide options, guarded by g_tuning_mu
thread_local Tuning t_tuning;      // what the entry point running on this thread sees
thread_local int t_depth = 0;      // entry points on this thread's stack (one that is composed of others nests)
}  // namespace

const Tuning& tuning() { return t_tuning; }

// Only the outermost entry point copies: the calls it is composed of see the options it saw.
TuningSnapshot::TuningSnapshot() {
    if (t_depth++ == 0) {
        std::lock_guard<std::mutex> lock(g_tuning_mu);
        t_tuning = g_tuning;
    }
}
TuningSnapshot::~TuningSnapshot() { --t_depth; }

namespace {

constexpr int kCopyBlock = 256;
constexpr int kCopyPerLane = 4;  // 16-byte words per lane

__global__ __launch_bounds__(kCopyBlock) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                          int64_t n16) {
    const int64_t base = (int64_t)blockIdx.x * (kCopyBlock * kCopyPerLane) + threadIdx.x;
    uint4 r[kCopyPerLane];
#pragma unroll
    for (int i = 0; i < kCopyPerLane; ++i) {
        const int64_t idx = base + (int64_t)i * kCopyBlock;
        if (idx < n16) r[i] = src[idx];
    }
#pragma unroll
    for (int i = 0; i < kCopyPerLane; ++i) {
        const int64_t idx = base + (int64_t)i * kCopyBlock;
        if (idx < n16) dst[idx] = r[i];
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlaps2(const void* a, int64_t abytes, const void* b, int64_t bbytes) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + (uintptr_t)bbytes && y < x + (uintptr_t)abytes;
}

bool overlaps(const void* a, const void* b, int64_t bytes) { return overlaps2(a, bytes, b, bytes); }

// A device buffer an entry point reads or writes.
struct Range {
    const void* p;
    int64_t bytes;
};

int64_t filter_bytes(int64_t D, int32_t group, int32_t lh) { return (D / group) * (int64_t)lh * (int64_t)sizeof(float); }

// Every written buffer must be disjoint from every other buffer of the call (activations, filter tables, filter
// gradient, workspace alike).  Empty ranges never overlap anything.
hy_status check_disjoint(const Range* rd, int n_rd, const Range* wr, int n_wr) {
    for (int o = 0; o < n_wr; ++o) {
        if (wr[o].bytes <= 0) continue;
        for (int i = 0; i < n_rd; ++i)
            if (rd[i].bytes > 0 && overlaps2(wr[o].p, wr[o].bytes, rd[i].p, rd[i].bytes)) return HY_ERR_ALIGN;
        for (int o2 = o + 1; o2 < n_wr; ++o2)
            if (wr[o2].bytes > 0 && overlaps2(wr[o].p, wr[o].bytes, wr[o2].p, wr[o2].bytes)) return HY_ERR_ALIGN;
    }
    return HY_OK;
}

// A filter table the call reads: fp32 [D/group, lh].
struct FilterArg {
    const float* p;
    int32_t group, lh;
};

// Checks shared by every convolution entry point.  `ins`/`outs` hold activation pointers, `hs` the fp32 filter
// tables the call reads; lh and group are those of the inner filter.
hy_status validate(const void* const* ins, int n_in, void* const* outs, int n_out, const FilterArg* hs,
                   int n_h, int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype) {
    for (int i = 0; i < n_in; ++i)
        if (!ins[i]) return HY_ERR_NULL;
    for (int i = 0; i < n_out; ++i)
        if (!outs[i]) return HY_ERR_NULL;
    for (int i = 0; i < n_h; ++i)
        if (!hs[i].p) return HY_ERR_NULL;
    if (B < 0 || L < 0 || D < 0 || lh < 1 || group < 1) return HY_ERR_SHAPE;
    if (D % group != 0) return HY_ERR_SHAPE;
    if (dtype != HY_F32 && dtype != HY_BF16) return HY_ERR_DTYPE;
    for (int i = 0; i < n_in; ++i)
        if (!aligned16(ins[i])) return HY_ERR_ALIGN;
    for (int i = 0; i < n_out; ++i)
        if (!aligned16(outs[i])) return HY_ERR_ALIGN;
    for (int i = 0; i < n_h; ++i)
        if (!aligned16(hs[i].p)) return HY_ERR_ALIGN;
    // sizes must stay addressable with signed 64-bit byte offsets
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (B > 0 && L > 0 && D > 0) {
        if (L > INT64_MAX / D || B > INT64_MAX / (L * D) || B * L * D > INT64_MAX / esz) return HY_ERR_SHAPE;
        const int64_t bytes = B * L * D * esz;
        Range rd[16], wr[4];
        int n_rd = 0;
        for (int i = 0; i < n_in; ++i) rd[n_rd++] = Range{ins[i], bytes};
        for (int i = 0; i < n_h; ++i)
            if (hs[i].group >= 1 && hs[i].lh >= 1 && D % hs[i].group == 0)  // (else the caller reports the shape)
                rd[n_rd++] = Range{hs[i].p, filter_bytes(D, hs[i].group, hs[i].lh)};
        for (int o = 0; o < n_out; ++o) wr[o] = Range{outs[o], bytes};
        return check_disjoint(rd, n_rd, wr, n_out);
    }
    return HY_OK;
}

bool empty(int64_t B, int64_t L, int64_t D) { return B == 0 || L == 0 || D == 0; }

// ---- scratch of hyena_li_fwd_static: device memory that lives in the code object, one copy per GPU, held until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the device address
// it yields (per device) is what kernels, copies and fills get.
constexpr int64_t kLiStaticScratchBytes = HYENA_LI_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[kLiStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, resolved on first use there

// Address of the current device's copy of `scratch` (resolved once per device, with that device current).
hy_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HY_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return HY_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HY_OK;
}

}  // namespace
}  // namespace hy

using namespace hy;

namespace {

// Extra checks of the sequence-shard entry points: the layout arguments, and the overlap rules on what a shard call
// really touches (batch items a stride apart; k and v from `history` rows before their pointer).
hy_status validate_shard(const void* q, const void* k, const void* v, const float* h, void* y, int64_t B, int64_t L,
                         int64_t D, int32_t lh, int32_t group, int32_t dtype, int64_t stride_kv, int64_t stride_qy,
                         int32_t history) {
    if (history < 0 || stride_kv < 0 || stride_qy < 0) return HY_ERR_SHAPE;
    if (empty(B, L, D)) return HY_OK;
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (history > (INT64_MAX / esz - L * D) / D) return HY_ERR_SHAPE;
    const int64_t item_kv = (L + history) * D, item_qy = L * D;  // elements of one batch item's rows
    if (B > 1 && (stride_kv < item_kv || stride_qy < item_qy)) return HY_ERR_SHAPE;
    // every batch item starts on a 16-byte boundary
    if (B > 1 && ((stride_kv * esz) % 16 != 0 || (stride_qy * esz) % 16 != 0)) return HY_ERR_ALIGN;
    if (B > 1 && (stride_kv > (INT64_MAX / esz - item_kv) / (B - 1) || stride_qy > (INT64_MAX / esz - item_qy) / (B - 1)))
        return HY_ERR_SHAPE;
    const int64_t span_kv = ((B - 1) * stride_kv + L * D) * esz, span_qy = ((B - 1) * stride_qy + L * D) * esz;
    const int64_t back = (int64_t)history * D * esz;
    const Range rd[4] = {{q, span_qy},
                         {static_cast<const char*>(k) - back, span_kv + back},
                         {static_cast<const char*>(v) - back, span_kv + back},
                         {h, filter_bytes(D, group, lh)}};
    const Range wr[1] = {{y, span_qy}};
    return check_disjoint(rd, 4, wr, 1);
}

hy_status gated_fwd(bool mr_first, const void* q, const void* k, const void* v, const float* h, void* y, int64_t B,
                    int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, void* hip_stream,
                    bool shard = false, int64_t stride_kv = 0, int64_t stride_qy = 0, int32_t history = 0) {
    TuningSnapshot snap;
    const void* ins[3] = {q, k, v};
    void* outs[1] = {y};
    const FilterArg hs[1] = {{h, group, lh}};
    hy_status rc = validate(ins, 3, outs, 1, hs, 1, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (shard) {
        rc = validate_shard(q, k, v, h, y, B, L, D, lh, group, dtype, stride_kv, stride_qy, history);
        if (rc != HY_OK) return rc;
    }
    if (empty(B, L, D)) return HY_OK;
    ConvPtrs p{q, k, v, h, y};
    ConvShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype), true};
    if (shard) {
        s.bstride_kv = B > 1 ? stride_kv : L * D;
        s.bstride_qy = B > 1 ? stride_qy : L * D;
        s.history = history;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    rc = mr_first ? launch_mr_mfma(p, s, st) : HY_ERR_UNSUPPORTED;
    // short filters (that the grouped matrix-core path does not take) are the SE kernels' business
    if (rc == HY_ERR_UNSUPPORTED && (lh <= 8 || !mr_first)) {
        if (se_walk_preferred(s)) return launch_se_walk(&p, 1, s, st);
        rc = launch_stencil(&p, 1, s, st);
    }
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_cp4(p, s, st);
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_cp_mfma(p, s, st);
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_direct(&p, 1, s, st);
    return rc;
}

// Argument checks shared by hyena_li_fwd and its static-scratch form.
hy_status li_validate(const void* q, const void* k, const void* v, const float* R, const float* lambda, void* y,
                      int64_t B, int64_t L, int64_t D, int32_t order, int32_t group, int32_t dtype) {
    const void* ins[3] = {q, k, v};
    void* outs[1] = {y};
    const FilterArg hs[2] = {{R, group, order}, {lambda, group, order}};
    return validate(ins, 3, outs, 1, hs, 2, B, L, D, order, group, dtype);
}

// The workspace of a call must be present, aligned, large enough and disjoint from every other buffer.
hy_status check_workspace(const void* ws, int64_t ws_bytes, int64_t need, const Range* others, int n_others) {
    if (need <= 0) return HY_OK;
    if (!ws) return HY_ERR_NULL;
    if (!aligned16(ws)) return HY_ERR_ALIGN;
    if (ws_bytes < need) return HY_ERR_SHAPE;
    const Range w{ws, need};
    return check_disjoint(others, n_others, &w, 1);
}

}  // namespace

extern "C" {

hy_status hyena_se_fwd(const void* q, const void* k, const void* v, const float* h, void* y, int64_t B, int64_t L,
                       int64_t D, int32_t lh, int32_t group, int32_t dtype, void* hip_stream) {
    return gated_fwd(false, q, k, v, h, y, B, L, D, lh, group, dtype, hip_stream);
}

hy_status hyena_se_fwd_shard(const void* q, const void* k, const void* v, const float* h, void* y, int64_t B,
                             int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, int64_t batch_stride_kv,
                             int64_t batch_stride_qy, int32_t history, void* hip_stream) {
    return gated_fwd(false, q, k, v, h, y, B, L, D, lh, group, dtype, hip_stream, true, batch_stride_kv,
                     batch_stride_qy, history);
}

hy_status hyena_mr_fwd_shard(const void* q, const void* k, const void* v, const float* h, void* y, int64_t B,
                             int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, int64_t batch_stride_kv,
                             int64_t batch_stride_qy, int32_t history, void* hip_stream) {
    return gated_fwd(true, q, k, v, h, y, B, L, D, lh, group, dtype, hip_stream, true, batch_stride_kv,
                     batch_stride_qy, history);
}

hy_status hyena_mr_fwd(const void* q, const void* k, const void* v, const float* h, void* y, int64_t B, int64_t L,
                       int64_t D, int32_t lh, int32_t group, int32_t dtype, void* hip_stream) {
    return gated_fwd(true, q, k, v, h, y, B, L, D, lh, group, dtype, hip_stream);
}

hy_status hyena_featurize_fwd(const void* x, const float* h, void* y, int64_t B, int64_t L, int64_t D, int32_t lh,
                              int32_t group, int32_t dtype, void* hip_stream) {
    TuningSnapshot snap;
    const void* ins[1] = {x};
    void* outs[1] = {y};
    const FilterArg hs[1] = {{h, group, lh}};
    hy_status rc = validate(ins, 1, outs, 1, hs, 1, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (empty(B, L, D)) return HY_OK;
    ConvPtrs p{nullptr, x, nullptr, h, y};
    ConvShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype), false};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (se_walk_preferred(s, 1)) return launch_se_walk(&p, 1, s, st);  // long sequences: the tile walker
    rc = launch_stencil(&p, 1, s, st);
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_direct(&p, 1, s, st);
    return rc;
}

hy_status hyena_featurize3_fwd(const void* q, const void* k, const void* v, const float* hq, const float* hk,
                               const float* hv, void* qo, void* ko, void* vo, int64_t B, int64_t L, int64_t D,
                               int32_t lh, int32_t group, int32_t dtype, void* hip_stream) {
    TuningSnapshot snap;
    const void* ins[3] = {q, k, v};
    void* outs[3] = {qo, ko, vo};
    const FilterArg hs[3] = {{hq, group, lh}, {hk, group, lh}, {hv, group, lh}};
    hy_status rc = validate(ins, 3, outs, 3, hs, 3, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (empty(B, L, D)) return HY_OK;
    ConvPtrs p[3] = {{nullptr, q, nullptr, hq, qo}, {nullptr, k, nullptr, hk, ko}, {nullptr, v, nullptr, hv, vo}};
    ConvShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype), false};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (se_walk_preferred(s, 3)) return launch_se_walk(p, 3, s, st);
    rc = launch_stencil(p, 3, s, st);
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_direct(p, 3, s, st);
    return rc;
}

int64_t hyena_chain_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh,
                                    int32_t group, int32_t dtype) {
    if (B < 0 || L < 0 || D < 0 || lf < 1 || lh < 1 || feat_group < 1 || group < 1) return -1;
    if (D % group != 0 || D % feat_group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    ChainShape s{B, L, D, lf, feat_group, lh, group, static_cast<hy_dtype>(dtype)};
    if (empty(B, L, D) || chain4_supported(s)) return 0;
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (L > INT64_MAX / D || B > INT64_MAX / (L * D) || B * L * D > INT64_MAX / (3 * esz)) return -1;
    return 3 * B * L * D * esz;
}

hy_status hyena_chain_fwd(const void* q, const void* k, const void* v, const float* hq, const float* hk,
                          const float* hv, const float* h, void* y, void* workspace, int64_t workspace_bytes,
                          int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh, int32_t group,
                          int32_t dtype, void* hip_stream) {
    TuningSnapshot snap;
    const void* ins[3] = {q, k, v};
    void* outs[1] = {y};
    const FilterArg hs[4] = {{hq, feat_group, lf}, {hk, feat_group, lf}, {hv, feat_group, lf}, {h, group, lh}};
    hy_status rc = validate(ins, 3, outs, 1, hs, 4, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (lf < 1 || feat_group < 1 || D % feat_group != 0 || workspace_bytes < 0) return HY_ERR_SHAPE;
    if (empty(B, L, D)) return HY_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ChainShape cs{B, L, D, lf, feat_group, lh, group, static_cast<hy_dtype>(dtype)};
    if (chain4_supported(cs)) {
        ChainPtrs cp{q, k, v, hq, hk, hv, h, y};
        return launch_chain4(cp, cs, st);
    }
    // two-kernel path through the caller's workspace
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (B * L * D > INT64_MAX / (3 * esz)) return HY_ERR_SHAPE;
    const int64_t bytes = B * L * D * esz;
    const Range others[8] = {{q, bytes}, {k, bytes}, {v, bytes}, {y, bytes},
                             {hq, filter_bytes(D, feat_group, lf)}, {hk, filter_bytes(D, feat_group, lf)},
                             {hv, filter_bytes(D, feat_group, lf)}, {h, filter_bytes(D, group, lh)}};
    rc = check_workspace(workspace, workspace_bytes, 3 * bytes, others, 8);
    if (rc != HY_OK) return rc;
    char* ws = static_cast<char*>(workspace);
    ConvPtrs f[3] = {{nullptr, q, nullptr, hq, ws}, {nullptr, k, nullptr, hk, ws + bytes}, {nullptr, v, nullptr, hv, ws + 2 * bytes}};
    ConvShape fs{B, L, D, lf, feat_group, static_cast<hy_dtype>(dtype), false};
    rc = se_walk_preferred(fs, 3) ? launch_se_walk(f, 3, fs, st) : launch_stencil(f, 3, fs, st);
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_direct(f, 3, fs, st);
    if (rc != HY_OK) return rc;
    ConvPtrs m{ws, ws + bytes, ws + 2 * bytes, h, y};
    ConvShape ms{B, L, D, lh, group, static_cast<hy_dtype>(dtype), true};
    rc = launch_mr_mfma(m, ms, st);
    if (rc == HY_ERR_UNSUPPORTED) rc = launch_direct(&m, 1, ms, st);
    return rc;
}

hy_status hyena_chain_fwd_shard(const void* q, const void* k, const void* v, const float* hq, const float* hk,
                                const float* hv, const float* h, void* y, int64_t B, int64_t L, int64_t D, int32_t lf,
                                int32_t feat_group, int32_t lh, int32_t group, int32_t dtype, int64_t batch_stride_in,
                                int64_t batch_stride_y, int32_t history, void* hip_stream) {
    TuningSnapshot snap;
    const void* ins[3] = {q, k, v};
    void* outs[1] = {y};
    const FilterArg hs[4] = {{hq, feat_group, lf}, {hk, feat_group, lf}, {hv, feat_group, lf}, {h, group, lh}};
    hy_status rc = validate(ins, 3, outs, 1, hs, 4, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (lf < 1 || feat_group < 1 || D % feat_group != 0) return HY_ERR_SHAPE;
    if (history < 0 || batch_stride_in < 0 || batch_stride_y < 0) return HY_ERR_SHAPE;
    if (empty(B, L, D)) return HY_OK;
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (history > (INT64_MAX / esz - L * D) / D) return HY_ERR_SHAPE;
    const int64_t item_in = (L + history) * D, item_y = L * D;
    if (B > 1) {
        if (batch_stride_in < item_in || batch_stride_y < item_y) return HY_ERR_SHAPE;
        if ((batch_stride_in * esz) % 16 != 0 || (batch_stride_y * esz) % 16 != 0) return HY_ERR_ALIGN;
        if (batch_stride_in > (INT64_MAX / esz - item_in) / (B - 1) || batch_stride_y > (INT64_MAX / esz - item_y) / (B - 1))
            return HY_ERR_SHAPE;
    }
    const int64_t back = (int64_t)history * D * esz;
    const int64_t span_in = ((B - 1) * (B > 1 ? batch_stride_in : 0) + L * D) * esz + back;
    const int64_t span_y = ((B - 1) * (B > 1 ? batch_stride_y : 0) + L * D) * esz;
    const Range rd[7] = {{static_cast<const char*>(q) - back, span_in}, {static_cast<const char*>(k) - back, span_in},
                         {static_cast<const char*>(v) - back, span_in}, {hq, filter_bytes(D, feat_group, lf)},
                         {hk, filter_bytes(D, feat_group, lf)}, {hv, filter_bytes(D, feat_group, lf)},
                         {h, filter_bytes(D, group, lh)}};
    const Range wr[1] = {{y, span_y}};
    rc = check_disjoint(rd, 7, wr, 1);
    if (rc != HY_OK) return rc;
    ChainShape cs{B, L, D, lf, feat_group, lh, group, static_cast<hy_dtype>(dtype)};
    cs.bstride_in = B > 1 ? batch_stride_in : 0;
    cs.bstride_y = B > 1 ? batch_stride_y : 0;
    cs.history = history;
    if (!chain4_supported(cs)) return HY_ERR_UNSUPPORTED;  // shards exist on the single-kernel path only
    ChainPtrs cp{q, k, v, hq, hk, hv, h, y};
    return launch_chain4(cp, cs, static_cast<hipStream_t>(hip_stream));
}

int64_t hyena_li_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t order, int32_t group, int32_t dtype) {
    TuningSnapshot snap;
    if (B < 0 || L < 0 || D < 0 || order < 1 || group < 1 || D % group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    if (empty(B, L, D)) return 0;
    LiShape s{B, L, D, order, group, static_cast<hy_dtype>(dtype)};
    return li_workspace_bytes(s);
}

hy_status hyena_li_fwd(const void* q, const void* k, const void* v, const float* R, const float* lambda, void* y,
                       void* workspace, int64_t workspace_bytes, int64_t B, int64_t L, int64_t D, int32_t order,
                       int32_t group, int32_t dtype, void* hip_stream) {
    TuningSnapshot snap;
    hy_status rc = li_validate(q, k, v, R, lambda, y, B, L, D, order, group, dtype);
    if (rc != HY_OK) return rc;
    if (workspace_bytes < 0) return HY_ERR_SHAPE;
    if (order > 64) return HY_ERR_UNSUPPORTED;
    if (empty(B, L, D)) return HY_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    LiPtrs p{q, k, v, R, lambda, y};
    LiShape s{B, L, D, order, group, static_cast<hy_dtype>(dtype)};
    if (li_mfma_supported(s)) {
        const int64_t bytes = B * L * D * 2;
        const int64_t nf = filter_bytes(D, group, order);
        const Range others[6] = {{q, bytes}, {k, bytes}, {v, bytes}, {y, bytes}, {R, nf}, {lambda, nf}};
        rc = check_workspace(workspace, workspace_bytes, li_workspace_bytes(s), others, 6);
        if (rc != HY_OK) return rc;
        return launch_li_mfma(p, s, workspace, st);
    }
    return launch_li_direct(p, s, st);
}

hy_status hyena_li_fwd_carry(const void* q, const void* k, const void* v, const float* R, const float* lambda, void* y,
                             const float* state_in, float* state_out, void* workspace, int64_t workspace_bytes,
                             int64_t B, int64_t L, int64_t D, int32_t order, int32_t group, int32_t dtype,
                             void* hip_stream) {
    TuningSnapshot snap;
    hy_status rc = li_validate(q, k, v, R, lambda, y, B, L, D, order, group, dtype);
    if (rc != HY_OK) return rc;
    if (workspace_bytes < 0) return HY_ERR_SHAPE;
    if ((state_in && !aligned16(state_in)) || (state_out && !aligned16(state_out))) return HY_ERR_ALIGN;
    LiPtrs p{q, k, v, R, lambda, y, state_in, state_out};
    LiShape s{B, L, D, order, group, static_cast<hy_dtype>(dtype)};
    // states exist in the matrix-core scan only; an empty call would have to copy state_in to state_out
    if (!li_mfma_supported(s) || empty(B, L, D)) return HY_ERR_UNSUPPORTED;
    if (state_out && L % 32 != 0) return HY_ERR_UNSUPPORTED;
    const int64_t bytes = B * L * D * 2;
    const int64_t nf = filter_bytes(D, group, order);
    const int64_t sb = B * D * 64;  // bytes of a state: B * (D / 16) records of 256 floats
    const Range rd[6] = {{q, bytes}, {k, bytes}, {v, bytes}, {R, nf}, {lambda, nf}, {state_in, state_in ? sb : 0}};
    const Range wr[2] = {{y, bytes}, {state_out, state_out ? sb : 0}};
    rc = check_disjoint(rd, 6, wr, 2);
    if (rc != HY_OK) return rc;
    const Range others[8] = {{q, bytes}, {k, bytes}, {v, bytes}, {y, bytes}, {R, nf}, {lambda, nf},
                             {state_in, state_in ? sb : 0}, {state_out, state_out ? sb : 0}};
    rc = check_workspace(workspace, workspace_bytes, li_workspace_bytes(s), others, 8);
    if (rc != HY_OK) return rc;
    return launch_li_mfma(p, s, workspace, static_cast<hipStream_t>(hip_stream));
}

int64_t hyena_li_state_bytes(int64_t B, int64_t D) { return (B < 0 || D < 0 || D % 16 != 0) ? -1 : B * D * 64; }

int64_t hyena_li_state_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t order, int32_t group, int32_t dtype) {
    TuningSnapshot snap;
    if (B < 0 || L < 0 || D < 0 || order < 1 || group < 1 || D % group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    LiShape s{B, L, D, order, group, static_cast<hy_dtype>(dtype)};
    return li_state_workspace_bytes(s);
}

hy_status hyena_li_state(const void* k, const void* v, const float* lambda, const float* state_in, float* state_out,
                         void* workspace, int64_t workspace_bytes, int64_t B, int64_t L, int64_t D, int32_t order,
                         int32_t group, int32_t dtype, void* hip_stream) {
    TuningSnapshot snap;
    if (!state_out) return HY_ERR_NULL;
    // validated like a forward call whose q is k, whose residues are the poles and whose only output is the state
    const void* ins[2] = {k, v};
    const FilterArg hs[1] = {{lambda, group, order}};
    hy_status rc = validate(ins, 2, nullptr, 0, hs, 1, B, L, D, order, group, dtype);
    if (rc != HY_OK) return rc;
    if (workspace_bytes < 0) return HY_ERR_SHAPE;
    if ((state_in && !aligned16(state_in)) || !aligned16(state_out)) return HY_ERR_ALIGN;
    LiShape s{B, L, D, order, group, static_cast<hy_dtype>(dtype)};
    if (!li_mfma_supported(s) || empty(B, L, D) || L % 32 != 0) return HY_ERR_UNSUPPORTED;
    const int64_t bytes = B * L * D * 2;
    const int64_t nf = filter_bytes(D, group, order);
    const int64_t sb = B * D * 64;
    const Range rd[4] = {{k, bytes}, {v, bytes}, {lambda, nf}, {state_in, state_in ? sb : 0}};
    const Range wr[1] = {{state_out, sb}};
    rc = check_disjoint(rd, 4, wr, 1);
    if (rc != HY_OK) return rc;
    const Range others[5] = {{k, bytes}, {v, bytes}, {lambda, nf}, {state_in, state_in ? sb : 0}, {state_out, sb}};
    rc = check_workspace(workspace, workspace_bytes, li_state_workspace_bytes(s), others, 5);
    if (rc != HY_OK) return rc;
    LiPtrs p{nullptr, k, v, nullptr, lambda, nullptr, state_in, state_out};
    return launch_li_state(p, s, workspace, static_cast<hipStream_t>(hip_stream));
}

hy_status hyena_li_state_fold(const float* states, int64_t n_states, int64_t steps, const float* lambda,
                              const float* state_in, float* state_out, int64_t B, int64_t D, int32_t order,
                              int32_t group, void* hip_stream) {
    TuningSnapshot snap;
    if (!lambda || !state_out || (n_states > 0 && !states)) return HY_ERR_NULL;
    if (B < 0 || D < 0 || n_states < 0 || steps < 0 || order < 1 || group < 1 || D % group != 0) return HY_ERR_SHAPE;
    if (D % 16 != 0 || order > 16) return HY_ERR_UNSUPPORTED;
    if (!aligned16(states) || !aligned16(lambda) || !aligned16(state_out) || (state_in && !aligned16(state_in)))
        return HY_ERR_ALIGN;
    if (B == 0 || D == 0) return HY_OK;
    if (B > (INT64_MAX / 64) / D || (n_states > 0 && n_states > INT64_MAX / (B * D * 64))) return HY_ERR_SHAPE;
    const int64_t sb = B * D * 64;
    const Range rd[3] = {{states, n_states * sb}, {lambda, filter_bytes(D, group, order)}, {state_in, state_in ? sb : 0}};
    const Range wr[1] = {{state_out, sb}};
    hy_status rc = check_disjoint(rd, 3, wr, 1);
    if (rc != HY_OK) return rc;
    return launch_li_state_fold(states, n_states, steps, lambda, state_in, state_out, B, D, order, group,
                                static_cast<hipStream_t>(hip_stream));
}

hy_status hyena_li_fwd_static(const void* q, const void* k, const void* v, const float* R, const float* lambda,
                              void* y, int64_t B, int64_t L, int64_t D, int32_t order, int32_t group, int32_t dtype,
                              void* hip_stream) {
    TuningSnapshot snap;
    hy_status rc = li_validate(q, k, v, R, lambda, y, B, L, D, order, group, dtype);
    if (rc != HY_OK) return rc;
    if (order > 64) return HY_ERR_UNSUPPORTED;
    if (empty(B, L, D)) return HY_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    LiPtrs p{q, k, v, R, lambda, y};
    LiShape s{B, L, D, order, group, static_cast<hy_dtype>(dtype)};
    if (!li_mfma_supported(s)) return launch_li_direct(p, s, st);  // the plain recurrence needs no scratch
    const int64_t need = li_workspace_bytes(s);
    if (need > kLiStaticScratchBytes) return HY_ERR_SCRATCH;
    void* ws = nullptr;
    if (need > 0) {
        rc = static_scratch(&ws);
        if (rc != HY_OK) return rc;
    }
    // Nothing has to be cleared: pass 1 writes the end state of every tile but the last of each sequence, and pass 2
    // reads exactly those records, so no byte is read that this call has not written.
    return launch_li_mfma(p, s, ws, st);
}

int64_t hyena_bwd_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype) {
    TuningSnapshot snap;
    if (B < 0 || L < 0 || D < 0 || lh < 1 || group < 1 || D % group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    if (empty(B, L, D)) return 0;
    BwdShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype)};
    if (bwd_stencil_supported(s)) return bwd_walk_preferred(s) ? bwd_walk_workspace_bytes(s) : bwd_stencil_workspace_bytes(s);
    if (mr_bwd_supported(s)) return mr_bwd_workspace_bytes(s);
    if (cp4_bwd_supported(s)) return cp4_bwd_workspace_bytes(s);
    return 0;
}

int64_t hyena_bwd_shard_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype) {
    TuningSnapshot snap;
    if (B < 0 || L < 0 || D < 0 || lh < 1 || group < 1 || D % group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    if (empty(B, L, D)) return 0;
    BwdShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype)};
    s.shard_call = true;
    if (bwd_stencil_supported(s)) return bwd_walk_preferred(s) ? bwd_walk_workspace_bytes(s) : bwd_stencil_workspace_bytes(s);
    if (mr_bwd_supported(s)) return mr_bwd_workspace_bytes(s);
    if (cp4_bwd_supported(s)) return cp4_bwd_workspace_bytes(s);
    return 0;
}

// Layout of a sequence-shard backward call (all zero: the plain dense call).
struct BwdShard {
    int64_t stride_kv = 0, stride_gq = 0, stride_out = 0;
    int32_t history = 0, future = 0;
    bool on = false;
};

static hy_status gated_bwd(const void* dy, const void* q, const void* k, const void* v, const float* h, void* dq,
                           void* dk, void* dv, float* dh, void* workspace, int64_t workspace_bytes, int64_t B,
                           int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, void* hip_stream,
                           const BwdShard& sh = BwdShard()) {
    TuningSnapshot snap;
    const void* ins[4] = {dy, q, k, v};
    void* outs[3] = {dq, dk, dv};
    const FilterArg hs[2] = {{h, group, lh}, {dh, group, lh}};
    hy_status rc = validate(ins, 4, outs, 3, hs, 2, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (workspace_bytes < 0) return HY_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t nh = filter_bytes(D, group, lh);
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    int64_t bytes = B * L * D * esz;
    // what the call really touches: [front, front + span) around each pointer
    int64_t back_kv = 0, span_kv = bytes, span_gq = bytes, span_out = bytes;
    if (sh.on) {
        if (sh.history < 0 || sh.future < 0 || sh.stride_kv < 0 || sh.stride_gq < 0 || sh.stride_out < 0) return HY_ERR_SHAPE;
        if (!empty(B, L, D)) {
            const int64_t lim = (INT64_MAX / esz - L * D) / D;
            if (sh.history > lim || sh.future > lim) return HY_ERR_SHAPE;
            const int64_t item_kv = (L + sh.history) * D, item_gq = (L + sh.future) * D, item_out = L * D;
            if (B > 1) {
                if (sh.stride_kv < item_kv || sh.stride_gq < item_gq || sh.stride_out < item_out) return HY_ERR_SHAPE;
                if ((sh.stride_kv * esz) % 16 != 0 || (sh.stride_gq * esz) % 16 != 0 || (sh.stride_out * esz) % 16 != 0)
                    return HY_ERR_ALIGN;
                const int64_t cap = (INT64_MAX / esz - item_kv - item_gq) / (B - 1);
                if (sh.stride_kv > cap || sh.stride_gq > cap || sh.stride_out > cap) return HY_ERR_SHAPE;
            }
            back_kv = (int64_t)sh.history * D * esz;
            span_kv = ((B - 1) * (B > 1 ? sh.stride_kv : 0) + item_kv) * esz;
            span_gq = ((B - 1) * (B > 1 ? sh.stride_gq : 0) + item_gq) * esz;
            span_out = ((B - 1) * (B > 1 ? sh.stride_out : 0) + item_out) * esz;
            const Range rd[5] = {{dy, span_gq}, {q, span_gq}, {static_cast<const char*>(k) - back_kv, span_kv},
                                 {static_cast<const char*>(v) - back_kv, span_kv}, {h, nh}};
            const Range wr[3] = {{dq, span_out}, {dk, span_out}, {dv, span_out}};
            rc = check_disjoint(rd, 5, wr, 3);
            if (rc != HY_OK) return rc;
        }
    }
    const void* k_front = static_cast<const char*>(k) - back_kv;
    const void* v_front = static_cast<const char*>(v) - back_kv;
    // dh is written: disjoint from the filter and from every activation, read or written
    const Range reads[8] = {{h, nh}, {dy, span_gq}, {q, span_gq}, {k_front, span_kv}, {v_front, span_kv},
                            {dq, span_out}, {dk, span_out}, {dv, span_out}};
    const Range dh_range{dh, nh};
    if (check_disjoint(reads, 8, &dh_range, 1) != HY_OK) return HY_ERR_ALIGN;
    if (empty(B, L, D)) {
        // an empty batch has a zero filter gradient: one small fill launch, nothing else
        return launch_bwd_zero_dh(dh, D, lh, group, st);
    }
    BwdPtrs p{dy, q, k, v, h, dq, dk, dv, dh};
    BwdShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype)};
    if (sh.on) {
        s.bstride_kv = B > 1 ? sh.stride_kv : 0;
        s.bstride_gq = B > 1 ? sh.stride_gq : 0;
        s.bstride_out = B > 1 ? sh.stride_out : 0;
        s.history = sh.history;
        s.future = sh.future;
        s.shard_call = true;
    }
    const bool stencil = bwd_stencil_supported(s);
    const bool mfma = !stencil && mr_bwd_supported(s);
    const bool cp4 = !stencil && !mfma && cp4_bwd_supported(s);
    const bool walk = stencil && bwd_walk_preferred(s);
    if (stencil || mfma || cp4) {
        const int64_t need = walk ? bwd_walk_workspace_bytes(s)
                                  : (stencil ? bwd_stencil_workspace_bytes(s)
                                             : (mfma ? mr_bwd_workspace_bytes(s) : cp4_bwd_workspace_bytes(s)));
        const Range others[9] = {{dy, span_gq}, {q, span_gq}, {k_front, span_kv}, {v_front, span_kv}, {dq, span_out},
                                 {dk, span_out}, {dv, span_out}, {h, nh}, {dh, nh}};
        rc = check_workspace(workspace, workspace_bytes, need, others, 9);
        if (rc != HY_OK) return rc;
        if (walk) return launch_bwd_walk(p, s, workspace, st);
        if (stencil) return launch_bwd_stencil(p, s, workspace, st);
        if (mfma) return launch_mr_bwd(p, s, workspace, st);  // medium grouped filters: one pass on the matrix cores
        return launch_cp4_bwd(p, s, workspace, st);           // medium filters of single channels or small groups
    }
    return launch_bwd_direct(p, s, st);
}

hy_status hyena_se_bwd(const void* dy, const void* q, const void* k, const void* v, const float* h, void* dq, void* dk,
                       void* dv, float* dh, void* workspace, int64_t workspace_bytes, int64_t B, int64_t L, int64_t D,
                       int32_t lh, int32_t group, int32_t dtype, void* hip_stream) {
    return gated_bwd(dy, q, k, v, h, dq, dk, dv, dh, workspace, workspace_bytes, B, L, D, lh, group, dtype, hip_stream);
}

hy_status hyena_mr_bwd(const void* dy, const void* q, const void* k, const void* v, const float* h, void* dq, void* dk,
                       void* dv, float* dh, void* workspace, int64_t workspace_bytes, int64_t B, int64_t L, int64_t D,
                       int32_t lh, int32_t group, int32_t dtype, void* hip_stream) {
    return gated_bwd(dy, q, k, v, h, dq, dk, dv, dh, workspace, workspace_bytes, B, L, D, lh, group, dtype, hip_stream);
}

int64_t hyena_featurize_bwd_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype) {
    TuningSnapshot snap;
    if (B < 0 || L < 0 || D < 0 || lh < 1 || group < 1 || D % group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    if (empty(B, L, D)) return 0;
    BwdShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype)};
    s.gated = false;
    return bwd_stencil_supported(s) ? bwd_stencil_workspace_bytes(s) : 0;
}

hy_status hyena_featurize_bwd(const void* dy, const void* x, const float* h, void* dx, float* dh, void* workspace,
                              int64_t workspace_bytes, int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group,
                              int32_t dtype, void* hip_stream) {
    TuningSnapshot snap;
    const void* ins[2] = {dy, x};
    void* outs[1] = {dx};
    const FilterArg hs[2] = {{h, group, lh}, {dh, group, lh}};
    hy_status rc = validate(ins, 2, outs, 1, hs, 2, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (workspace_bytes < 0) return HY_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t nh = filter_bytes(D, group, lh);
    const int64_t bytes = B * L * D * (dtype == HY_F32 ? 4 : 2);
    // dh is written: disjoint from the filter and from every activation, read or written
    const Range reads[4] = {{h, nh}, {dy, bytes}, {x, bytes}, {dx, bytes}};
    const Range dh_range{dh, nh};
    if (check_disjoint(reads, 4, &dh_range, 1) != HY_OK) return HY_ERR_ALIGN;
    if (empty(B, L, D)) return launch_bwd_zero_dh(dh, D, lh, group, st);
    BwdPtrs p{dy, nullptr, x, nullptr, h, nullptr, dx, nullptr, dh};
    BwdShape s{B, L, D, lh, group, static_cast<hy_dtype>(dtype)};
    s.gated = false;
    if (bwd_stencil_supported(s)) {
        const Range others[5] = {{dy, bytes}, {x, bytes}, {dx, bytes}, {h, nh}, {dh, nh}};
        rc = check_workspace(workspace, workspace_bytes, bwd_stencil_workspace_bytes(s), others, 5);
        if (rc != HY_OK) return rc;
        return launch_bwd_stencil(p, s, workspace, st);
    }
    return launch_bwd_direct(p, s, st);
}

// The operator chain's backward as a composition of the calls above, through the caller's workspace:
// [q', k', v' | dq', dk', dv' | workspace of the inner calls].
namespace {
int64_t align256(int64_t n) { return (n + 255) / 256 * 256; }
int64_t chain_bwd_inner_ws(int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh, int32_t group,
                           int32_t dtype) {
    const int64_t a = hyena_bwd_workspace_bytes(B, L, D, lh, group, dtype);
    const int64_t b = hyena_featurize_bwd_workspace_bytes(B, L, D, lf, feat_group, dtype);
    if (a < 0 || b < 0) return -1;
    return a > b ? a : b;
}
}  // namespace

int64_t hyena_chain_bwd_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh,
                                        int32_t group, int32_t dtype) {
    TuningSnapshot snap;
    if (B < 0 || L < 0 || D < 0 || lf < 1 || lh < 1 || feat_group < 1 || group < 1) return -1;
    if (D % group != 0 || D % feat_group != 0) return -1;
    if (dtype != HY_F32 && dtype != HY_BF16) return -1;
    if (empty(B, L, D)) return 0;
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (L > INT64_MAX / D || B > INT64_MAX / (L * D) || B * L * D > (INT64_MAX / 8) / esz) return -1;
    const int64_t inner = chain_bwd_inner_ws(B, L, D, lf, feat_group, lh, group, dtype);
    if (inner < 0) return -1;
    return 6 * align256(B * L * D * esz) + inner;
}

hy_status hyena_chain_bwd(const void* dy, const void* q, const void* k, const void* v, const float* hq, const float* hk,
                          const float* hv, const float* h, void* dq, void* dk, void* dv, float* dhq, float* dhk,
                          float* dhv, float* dh, void* workspace, int64_t workspace_bytes, int64_t B, int64_t L,
                          int64_t D, int32_t lf, int32_t feat_group, int32_t lh, int32_t group, int32_t dtype,
                          void* hip_stream) {
    TuningSnapshot snap;
    const void* ins[4] = {dy, q, k, v};
    void* outs[3] = {dq, dk, dv};
    const FilterArg hs[8] = {{hq, feat_group, lf}, {hk, feat_group, lf}, {hv, feat_group, lf}, {h, group, lh},
                             {dhq, feat_group, lf}, {dhk, feat_group, lf}, {dhv, feat_group, lf}, {dh, group, lh}};
    hy_status rc = validate(ins, 4, outs, 3, hs, 8, B, L, D, lh, group, dtype);
    if (rc != HY_OK) return rc;
    if (lf < 1 || feat_group < 1 || D % feat_group != 0 || workspace_bytes < 0) return HY_ERR_SHAPE;
    const int64_t nf = filter_bytes(D, feat_group, lf), nh = filter_bytes(D, group, lh);
    const int64_t esz = dtype == HY_F32 ? 4 : 2;
    if (!empty(B, L, D) && B * L * D > (INT64_MAX / 8) / esz) return HY_ERR_SHAPE;
    const int64_t bytes = B * L * D * esz;
    // every filter gradient is written: disjoint from everything else the call touches
    const Range all[15] = {{dy, bytes}, {q, bytes}, {k, bytes}, {v, bytes}, {dq, bytes}, {dk, bytes}, {dv, bytes},
                           {hq, nf}, {hk, nf}, {hv, nf}, {h, nh}, {dhq, nf}, {dhk, nf}, {dhv, nf}, {dh, nh}};
    for (int i = 11; i < 15; ++i) {
        Range rest[14];
        int n = 0;
        for (int j = 0; j < 15; ++j)
            if (j != i) rest[n++] = all[j];
        if (check_disjoint(rest, n, &all[i], 1) != HY_OK) return HY_ERR_ALIGN;
    }
    if (empty(B, L, D)) {
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        float* const fg[3] = {dhq, dhk, dhv};
        for (float* g : fg) {
            rc = launch_bwd_zero_dh(g, D, lf, feat_group, st);
            if (rc != HY_OK) return rc;
        }
        return launch_bwd_zero_dh(dh, D, lh, group, st);
    }
    const int64_t inner = chain_bwd_inner_ws(B, L, D, lf, feat_group, lh, group, dtype);
    if (inner < 0) return HY_ERR_SHAPE;
    const int64_t slot = align256(bytes);
    rc = check_workspace(workspace, workspace_bytes, 6 * slot + inner, all, 15);
    if (rc != HY_OK) return rc;
    char* const ws = static_cast<char*>(workspace);
    void* const qf = ws, * const kf = ws + slot, * const vf = ws + 2 * slot;               // q', k', v'
    void* const gq = ws + 3 * slot, * const gk = ws + 4 * slot, * const gv = ws + 5 * slot;  // dq', dk', dv'
    void* const iw = inner > 0 ? ws + 6 * slot : nullptr;
    rc = hyena_featurize3_fwd(q, k, v, hq, hk, hv, qf, kf, vf, B, L, D, lf, feat_group, dtype, hip_stream);
    if (rc != HY_OK) return rc;
    rc = hyena_mr_bwd(dy, qf, kf, vf, h, gq, gk, gv, dh, iw, inner, B, L, D, lh, group, dtype, hip_stream);
    if (rc != HY_OK) return rc;
    rc = hyena_featurize_bwd(gq, q, hq, dq, dhq, iw, inner, B, L, D, lf, feat_group, dtype, hip_stream);
    if (rc != HY_OK) return rc;
    rc = hyena_featurize_bwd(gk, k, hk, dk, dhk, iw, inner, B, L, D, lf, feat_group, dtype, hip_stream);
    if (rc != HY_OK) return rc;
    return hyena_featurize_bwd(gv, v, hv, dv, dhv, iw, inner, B, L, D, lf, feat_group, dtype, hip_stream);
}

hy_status hyena_se_bwd_shard(const void* dy, const void* q, const void* k, const void* v, const float* h, void* dq,
                             void* dk, void* dv, float* dh, void* workspace, int64_t workspace_bytes, int64_t B,
                             int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, int64_t batch_stride_kv,
                             int64_t batch_stride_gq, int64_t batch_stride_out, int32_t history, int32_t future,
                             void* hip_stream) {
    BwdShard sh;
    sh.stride_kv = batch_stride_kv; sh.stride_gq = batch_stride_gq; sh.stride_out = batch_stride_out;
    sh.history = history; sh.future = future; sh.on = true;
    return gated_bwd(dy, q, k, v, h, dq, dk, dv, dh, workspace, workspace_bytes, B, L, D, lh, group, dtype, hip_stream, sh);
}

hy_status hyena_mr_bwd_shard(const void* dy, const void* q, const void* k, const void* v, const float* h, void* dq,
                             void* dk, void* dv, float* dh, void* workspace, int64_t workspace_bytes, int64_t B,
                             int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, int64_t batch_stride_kv,
                             int64_t batch_stride_gq, int64_t batch_stride_out, int32_t history, int32_t future,
                             void* hip_stream) {
    return hyena_se_bwd_shard(dy, q, k, v, h, dq, dk, dv, dh, workspace, workspace_bytes, B, L, D, lh, group, dtype,
                              batch_stride_kv, batch_stride_gq, batch_stride_out, history, future, hip_stream);
}

hy_status hyena_stream_copy(const void* src, void* dst, int64_t bytes, void* hip_stream) {
    if (!src || !dst) return HY_ERR_NULL;
    if (bytes < 0 || bytes % 16 != 0) return HY_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst) || (bytes > 0 && overlaps(src, dst, bytes))) return HY_ERR_ALIGN;
    if (bytes == 0) return HY_OK;
    const int64_t n16 = bytes / 16;
    const int64_t per_block = kCopyBlock * kCopyPerLane;
    const int64_t nb = (n16 + per_block - 1) / per_block;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel(copy_kernel, dim3((uint32_t)nb), dim3(kCopyBlock), static_cast<hipStream_t>(hip_stream),
                         static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
}

hy_status hyena_stream_gate(const void* q, const void* k, const void* v, void* y, int64_t B, int64_t L, int64_t D,
                            int32_t strip_channels, int64_t rows, int32_t depth, int32_t waves, void* hip_stream) {
    const void* ins[3] = {q, k, v};
    void* outs[1] = {y};
    hy_status rc = validate(ins, 3, outs, 1, nullptr, 0, B, L, D, 1, 1, HY_BF16);
    if (rc != HY_OK) return rc;
    if (rows < 0 || rows > 0x7fff0000LL || D % 8 != 0) return HY_ERR_SHAPE;
    if (strip_channels != 0 && strip_channels != 64 && strip_channels != 128 && strip_channels != 256)
        return HY_ERR_UNSUPPORTED;
    if (strip_channels != 0 && D % strip_channels != 0) return HY_ERR_SHAPE;
    if (depth != 0 && depth != 1 && depth != 2 && depth != 3 && depth != 4 && depth != 6 && depth != 8)
        return HY_ERR_UNSUPPORTED;
    // 4, 8 or 16 waves, at most one wave per 16 channels of the strip (the linear stream has no such choice)
    if (waves != 0 && (strip_channels == 0 || (waves != 4 && waves != 8 && waves != 16) || waves * 16 > strip_channels))
        return HY_ERR_UNSUPPORTED;
    if (empty(B, L, D)) return HY_OK;
    return launch_stream_gate(q, k, v, y, B, L, D, strip_channels, rows, depth, waves,
                              static_cast<hipStream_t>(hip_stream));
}

hy_status hyena_set_option(const char* name, int32_t value) {
    if (!name) return HY_ERR_NULL;
    if (value < 0) return HY_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    Tuning& t = g_tuning;
    if (strcmp(name, "se_vec") == 0) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return HY_ERR_SHAPE;
        t.se_vec = value;
    } else if (strcmp(name, "se_rows") == 0) {
        t.se_rows = value;
    } else if (strcmp(name, "mr_rows") == 0) {
        if (value % 32 != 0) return HY_ERR_SHAPE;
        t.mr_rows = value;
    } else if (strcmp(name, "mr_waves") == 0) {
        if (value != 0 && value != 4 && value != 8 && value != 16) return HY_ERR_SHAPE;
        t.mr_waves = value;
    } else if (strcmp(name, "se_walk") == 0) {
        if (value > 2) return HY_ERR_SHAPE;
        t.se_walk = value;
    } else {
        return HY_ERR_UNSUPPORTED;
    }
    return HY_OK;
}

const char* hyena_status_string(int32_t status) {
    switch (status) {
        case HY_OK: return "ok";
        case HY_ERR_NULL: return "null pointer argument";
        case HY_ERR_SHAPE: return "invalid shape or size argument";
        case HY_ERR_DTYPE: return "unknown dtype";
        case HY_ERR_ALIGN: return "pointer not 16-byte aligned, or a written buffer overlaps another buffer of the call";
        case HY_ERR_UNSUPPORTED: return "no kernel for this problem";
        case HY_ERR_LAUNCH: return "HIP launch error";
        case HY_ERR_SCRATCH: return "problem needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

int32_t hyena_version(void) { return 310; }

}  // extern "C"
