// Host-side launch interface between the C ABI (api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "hyena.h"

namespace hy {

// One convolution problem; up to three are batched into a launch (blockIdx.y selects).
struct ConvPtrs {
    const void* q;   // post-gate, unused when not gated
    const void* k;   // pre-gate operand, or the plain input x when not gated
    const void* v;   // pre-gate operand, unused when not gated
    const float* h;  // [D/group, lh] fp32
    void* y;
    // optional second post-gate and output, y2 = q2 * (h * (k*v)), from the same convolution (only where
    // cp4_dual_supported says so)
    const void* q2 = nullptr;
    void* y2 = nullptr;
};

struct ConvShape {
    int64_t B, L, D;
    int32_t lh, group;
    hy_dtype dtype;
    bool gated;
    // true: the convolution runs towards the past, y[t] = q[t] * sum_j h[j] k[t+j] v[t+j] (terms with t+j >= L
    // vanish): the transposed operator the backward pass needs.  Only launch_cp4 implements it.
    bool reversed = false;
    // One rank's share of a sequence-sharded call (Sec. 4, point-to-point scheme): consecutive batch items are
    // `bstride_kv` elements apart in k and v and `bstride_qy` in q and y (0: L * D, dense), and `history` rows of
    // k and v in front of row 0 hold the steps that precede the shard (the left neighbour's last rows); what lies
    // before them is zero.  Implemented by launch_stencil, launch_se_walk (history 0 or >= 8), launch_mr_mfma,
    // launch_cp4 and launch_direct.  In reversed time the history rows lie BEHIND row L - 1.  `bstride_y` (0: as
    // q) gives y a batch stride of its own; only launch_cp4 takes it.
    int64_t bstride_kv = 0, bstride_qy = 0;
    int32_t history = 0;
    int64_t bstride_y = 0;
    int64_t stride_kv() const { return bstride_kv > 0 ? bstride_kv : L * D; }
    int64_t stride_qy() const { return bstride_qy > 0 ? bstride_qy : L * D; }
    int64_t stride_y() const { return bstride_y > 0 ? bstride_y : stride_qy(); }
    bool sharded() const { return history != 0 || stride_kv() != L * D || stride_qy() != L * D || stride_y() != L * D; }
};

// The operator chain: featurize q, k, v (filters hq, hk, hv), then the gated medium convolution with h.
struct ChainPtrs {
    const void* q;
    const void* k;
    const void* v;
    const float* hq;
    const float* hk;
    const float* hv;
    const float* h;
    void* y;
};

struct ChainShape {
    int64_t B, L, D;
    int32_t lf, feat_group, lh, group;
    hy_dtype dtype;
    // One rank's share of a sequence-sharded call: `history` rows of q, k and v in front of row 0 hold data (zeros
    // before them); batch items are `bstride_in` elements apart in q, k, v and `bstride_y` in y (0: L * D).
    // Only launch_chain4 implements it.
    int64_t bstride_in = 0, bstride_y = 0;
    int32_t history = 0;
    int64_t stride_in() const { return bstride_in > 0 ? bstride_in : L * D; }
    int64_t stride_y() const { return bstride_y > 0 ? bstride_y : L * D; }
};

// Backward of the gated convolution.
struct BwdPtrs {
    const void* dy;
    const void* q;
    const void* k;
    const void* v;
    const float* h;
    void* dq;
    void* dk;
    void* dv;
    float* dh;  // [D/group, lh] fp32, overwritten
};

struct BwdShape {
    int64_t B, L, D;
    int32_t lh, group;
    hy_dtype dtype;
    // One rank's share of a sequence-sharded backward call: `history` rows of k and v in front of row 0 and `future`
    // rows of dy and q behind row L - 1 hold the neighbours' steps (zeros beyond them); batch items are
    // `bstride_kv` / `bstride_gq` / `bstride_out` elements apart in k, v / dy, q / dq, dk, dv (0: L * D, dense).
    // Implemented by every backward launcher.
    int64_t bstride_kv = 0, bstride_gq = 0, bstride_out = 0;
    int32_t history = 0, future = 0;
    bool gated = true;        // false: backward of the ungated featurizer convolution (x = k, dx = dk; no q, v, dq, dv);
                              // stencil and general kernels only
    bool shard_call = false;  // came in through a shard entry point: the kernels' shard variants, whatever the values
    int64_t stride_kv() const { return bstride_kv > 0 ? bstride_kv : L * D; }
    int64_t stride_gq() const { return bstride_gq > 0 ? bstride_gq : L * D; }
    int64_t stride_out() const { return bstride_out > 0 ? bstride_out : L * D; }
    bool sharded() const { return shard_call; }
};

// Hyena-LI forward: filter given by residues R and poles lam, fp32 [D/group, order] each.
struct LiPtrs {
    const void* q;
    const void* k;
    const void* v;
    const float* R;
    const float* lam;
    void* y;
    // optional (matrix-core scan only): the running sums at the step before the call's first step, and where to
    // leave them after its last step; fp32 [B][D/16][64][4], element [b][g][16 lq + li][r] = sum of exponential
    // n = 4 lq + r of channel 16 g + li
    const float* state_in = nullptr;
    float* state_out = nullptr;
};

struct LiShape {
    int64_t B, L, D;
    int32_t order, group;
    hy_dtype dtype;
};

struct Tuning {
    int se_vec = 0;
    int se_rows = 0;
    int mr_rows = 0;
    int mr_waves = 0;
    int se_walk = 0;  // 0: by size, 1: always the walking SE kernel where it applies, 2: never
};
// The options as the calling thread's current entry point sees them.  Every extern "C" function that sizes or
// launches anything starts with a TuningSnapshot, which copies the process-wide options under a lock into a
// thread-local; all code below the ABI reads only that copy, so within one call the tile choice that sizes a
// workspace and the one the launch uses cannot differ, whatever other threads set meanwhile.
const Tuning& tuning();

// Tiles per sequence when `base` workgroups cover one tile of every batch item (and problem): one workgroup per
// compute unit.  Kernels whose workgroups are bound by what one compute unit can stream pay the full time of a
// round of 256 workgroups that is partly empty, so where that choice leaves a round under 90% full (batches that
// do not divide 256) they take the finer cut, up to four rounds, that fills its rounds best while a tile keeps
// `min_rows` steps (measured: MR backward at B = 3 48% -> 53% of peak, three featurizers at B = 4 1192 -> 1040 us).
inline int64_t tiles_filling_rounds(int64_t base, int64_t L, int64_t min_rows) {
    int64_t tiles = 256 / base;
    if (tiles < 1) tiles = 1;
    auto fill = [&](int64_t t) { return (double)(base * t) / (double)(((base * t + 255) / 256) * 256); };
    int64_t best = tiles;
    for (int64_t t = tiles; fill(best) < 0.9 && base * t <= 1024 && (L + t - 1) / t >= min_rows; ++t)
        if (fill(t) > fill(best) + 1e-9) best = t;
    return best;
}
struct TuningSnapshot {
    TuningSnapshot();
    ~TuningSnapshot();
    TuningSnapshot(const TuningSnapshot&) = delete;
    TuningSnapshot& operator=(const TuningSnapshot&) = delete;
};

// Short-filter streaming stencil on the vector ALUs.  HY_ERR_UNSUPPORTED when lh is above its limit.
hy_status launch_stencil(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st);
// Short-filter kernel for long sequences (bf16, gated, lh <= 8, D % 128 == 0) on the MR kernel's data-movement
// skeleton; se_walk_preferred() says whether the dispatcher should take it for this shape.
// Ungated (featurizer) calls may bring up to three problems that share the shape (as launch_stencil does).
bool se_walk_preferred(const ConvShape& s, int nprob = 1);
hy_status launch_se_walk(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st);
// General fp32 direct convolution: any lh, any group, both dtypes.
hy_status launch_direct(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st);
// Block-Toeplitz contraction on bf16 MFMA.  HY_ERR_UNSUPPORTED outside its domain.
hy_status launch_mr_mfma(const ConvPtrs& p, const ConvShape& s, hipStream_t st);
// Chunk-parallel block-Toeplitz contraction on bf16 MFMA for filters not shared by 16 channels (any group).
// HY_ERR_UNSUPPORTED outside cp_mfma_supported().
bool cp_mfma_supported(const ConvShape& s);
hy_status launch_cp_mfma(const ConvPtrs& p, const ConvShape& s, hipStream_t st);
// The same on the batched 4x4x4 MFMA: 256 channels per workgroup, lh <= 129.  HY_ERR_UNSUPPORTED outside cp4_supported().
bool cp4_supported(const ConvShape& s);
// whether launch_cp4 also takes ConvPtrs::q2 / y2 for this shape (the long-filter kernel does)
bool cp4_dual_supported(const ConvShape& s);
hy_status launch_cp4(const ConvPtrs& p, const ConvShape& s, hipStream_t st);
// Whole chain in one pass over q, k, v, featurizers on the matrix cores too (batched 4x4x4 products, taps as bf16
// head + remainder).  HY_ERR_UNSUPPORTED outside chain4_supported().
bool chain4_supported(const ChainShape& s);
hy_status launch_chain4(const ChainPtrs& p, const ChainShape& s, hipStream_t st);
// Hyena-LI as a two-pass chunked scan on bf16 MFMA (end-of-tile states in `ws`), and the plain recurrence.
bool li_mfma_supported(const LiShape& s);
int64_t li_workspace_bytes(const LiShape& s);
hy_status launch_li_mfma(const LiPtrs& p, const LiShape& s, void* ws, hipStream_t st);
// The running sums after the call's steps alone (k, v only; L % 32 == 0; matrix-core scan's domain), and the fold of
// several stretches' zero-start end states [n][B][D/16][64][4] into the state after them.
int64_t li_state_workspace_bytes(const LiShape& s);
hy_status launch_li_state(const LiPtrs& p, const LiShape& s, void* ws, hipStream_t st);
hy_status launch_li_state_fold(const float* states, int64_t n, int64_t steps, const float* lam, const float* state_in,
                               float* state_out, int64_t B, int64_t D, int32_t order, int32_t group, hipStream_t st);
hy_status launch_li_direct(const LiPtrs& p, const LiShape& s, hipStream_t st);
// Backward, short filters: fused streaming pass + reduction of partial filter gradients held in `ws`.
bool bwd_stencil_supported(const BwdShape& s);
int64_t bwd_stencil_workspace_bytes(const BwdShape& s);
hy_status launch_bwd_stencil(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st);
// Backward, short bf16 filters on long stretches of time: the same arithmetic on the tile-walking data movement
// (256 channels per workgroup, 16-row chunks through LDS); bwd_walk_preferred() says when the dispatcher takes it.
bool bwd_walk_preferred(const BwdShape& s);
int64_t bwd_walk_workspace_bytes(const BwdShape& s);
hy_status launch_bwd_walk(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st);
// Backward, any shape (no workspace).
hy_status launch_bwd_direct(const BwdPtrs& p, const BwdShape& s, hipStream_t st);
// Backward on the matrix cores for medium grouped bf16 filters: dq, dk, dv and dh in one pass over dy, q, k, v.
bool mr_bwd_supported(const BwdShape& s);
int64_t mr_bwd_rows(const BwdShape& s);
int64_t mr_bwd_workspace_bytes(const BwdShape& s);
hy_status launch_mr_bwd(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st);
// Backward on the matrix cores for medium bf16 filters not shared by 16 channels (any group): dq and dk, dv from the
// chunk-parallel forward kernel (forwards, and twice towards the past), dh as a per-channel correlation on the
// batched 4x4x4 products; `ws` holds the partial filter gradients.
bool cp4_bwd_supported(const BwdShape& s);
int64_t cp4_bwd_workspace_bytes(const BwdShape& s);
hy_status launch_cp4_bwd(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st);
// dh[g][j] = sum over nsets partial sets and over `group` adjacent rows of a set; a set is [n_rows][lh].
hy_status launch_dh_reduce(const float* partial, float* dh, int64_t nsets, int64_t n_rows, int32_t lh, int32_t group,
                           hipStream_t st);
// dh := 0 (the filter gradient of an empty batch).
hy_status launch_bwd_zero_dh(float* dh, int64_t D, int32_t lh, int32_t group, hipStream_t st);
// Bandwidth yardstick y = q*k*v (bf16): strip = 0 streams linearly, 64 / 128 / 256 walks column strips of that many
// channels down time in `rows`-step tiles (0 = one workgroup per compute unit), `depth` chunks of loads in flight,
// `waves` waves per workgroup (0 = strip / 16).
hy_status launch_stream_gate(const void* q, const void* k, const void* v, void* y, int64_t B, int64_t L, int64_t D,
                             int32_t strip, int64_t rows, int32_t depth, int32_t waves, hipStream_t st);

// Launches `kernel` and returns the status of THIS launch as hipLaunchKernel reports it.  The thread's sticky
// "last error" is neither read nor cleared: an error left behind by an earlier, unrelated HIP call of the caller
// cannot make a healthy launch look failed, and stays there for the caller to find.
template <typename... KArgs>
inline hy_status launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t st,
                               std::decay_t<KArgs>... args) {
    void* ptrs[] = {static_cast<void*>(&args)...};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, st);
    return e == hipSuccess ? HY_OK : HY_ERR_LAUNCH;
}

}  // namespace hy
