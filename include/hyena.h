/*
 * hyena.h -- C ABI of the MI355X (gfx950) forward kernels for the StripedHyena 2 short and medium
 * gated causal convolutions (Hyena-SE and Hyena-MR) and their featurizer convolutions.
 *
 * Common conventions for every entry point
 *   - Activations are dense [B, L, D] row-major tensors with the channel index D contiguous; element
 *     type is given by `dtype` (HY_F32: IEEE binary32, HY_BF16: bfloat16).
 *   - Filters are fp32 for both dtypes, [D / group, lh] row-major, tap index contiguous; tap 0
 *     multiplies the current sample and tap j the sample j steps in the past (the FIR definition of
 *     Sec. 3.1, Eq. 2).  Channel c uses filter c / group (contiguous groups, Sec. 2.2).
 *   - Every pointer is a DEVICE pointer owned by the caller, 16-byte aligned.  A buffer the call writes
 *     (an output, the filter gradient, the workspace) must not overlap any other buffer of the call,
 *     activations and filter tables alike: HY_ERR_ALIGN.  The library allocates nothing, keeps no
 *     state between calls besides the tuning options below, launches on `hip_stream` (a hipStream_t,
 *     NULL = default stream) and never synchronises.
 *   - Left boundary: zero padding, separately for each batch item (terms with t - j < 0 vanish).
 *   - Errors: a status code is returned, nothing is thrown and nothing aborts.  All argument checks
 *     run before the first HIP call, so they work on a machine without a GPU.  B, L or D equal to 0
 *     is a valid empty problem and returns HY_OK without launching (the backward entry points still
 *     issue one small launch that sets the filter gradient to zero).
 *   - HY_ERR_LAUNCH reports the launch of this very call (the return value of hipLaunchKernel); the
 *     thread's sticky HIP error state is neither read nor cleared.
 */
#ifndef HYENA_H
#define HYENA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hy_status {
    HY_OK = 0,
    HY_ERR_NULL = 1,        /* a required pointer is NULL */
    HY_ERR_SHAPE = 2,       /* negative size, lh < 1, group < 1, or D not a multiple of group */
    HY_ERR_DTYPE = 3,       /* dtype is not one of hy_dtype */
    HY_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned, or a written buffer overlaps another buffer */
    HY_ERR_UNSUPPORTED = 5, /* valid problem, but no kernel in this build handles it */
    HY_ERR_LAUNCH = 6,      /* the HIP runtime reported an error at launch */
    HY_ERR_SCRATCH = 7      /* the problem needs more scratch than the library's static buffer holds */
} hy_status;

/* Storage types.  Entry points take the value as a plain int32_t so that any integer a caller passes is
 * well defined and can be rejected with HY_ERR_DTYPE. */
typedef enum hy_dtype { HY_F32 = 0, HY_BF16 = 1 } hy_dtype;

/*
 * Hyena-SE inner operator, forward (Sec. 2.1 Eq. 1 last line without the dense M; Algorithm 1 with
 * both optional gates on; FIR sum of Sec. 3.1 Eq. 2):
 *     y[b,t,c] = q[b,t,c] * sum_{j=0}^{min(lh-1,t)} h[c/group, j] * k[b,t-j,c] * v[b,t-j,c]
 * Meant for short filters (the paper runs lh = 4..7, always below 14): a fused streaming stencil on
 * the vector ALUs, fp32 arithmetic, one rounding at the store (two kernels with identical results, one
 * for short and one for long sequences, chosen by problem size).  Any lh >= 1 is accepted; filters
 * longer than 8 taps take the chunk-parallel matrix-core path described under hyena_mr_fwd when it
 * applies, else a slower general kernel.  q,k,v,y: [B,L,D] of `dtype`; h: fp32 [D/group, lh].
 */
hy_status hyena_se_fwd(const void *q, const void *k, const void *v, const float *h, void *y,
                       int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype,
                       void *hip_stream);

/*
 * Hyena-MR inner operator, forward: same formula as hyena_se_fwd, meant for filters of length in
 * the hundreds shared by groups of channels (paper default lh = 128, group = 16).  For HY_BF16 with
 * group a multiple of 16, D a multiple of 64 and lh <= 513 the convolution is evaluated as the
 * block-Toeplitz contraction of Sec. 3.1 (hat y_n = sum_k H_k hat x_{n-k}) on bf16 matrix cores with
 * fp32 accumulation: u = k*v is rounded once to bf16, h is rounded once to bf16, the output is
 * rounded once at the store.  For HY_BF16 with any other group size (down to one filter per
 * channel) the same contraction runs chunk-parallel (App. A.1), with the Toeplitz operands per
 * channel and consecutive chunks of a channel as the columns of the product: 4-step chunks on the
 * batched 4x4 matrix instruction when D is a multiple of 128 and lh <= 129, else 16-step chunks on
 * the 16x16 instruction when D is a multiple of 64 and lh <= 145; same roundings.  Every other valid
 * combination (HY_F32, other widths, longer filters) runs a general fp32 vector-ALU kernel.
 * On the matrix-core paths a source sample shares a product with the structural zeros of the Toeplitz
 * operand, so a non-finite k*v (Inf, NaN) makes outputs non-finite within the same 32-step block also
 * BEFORE its own time step and in all channels of its group slice; finite inputs are never affected.
 */
hy_status hyena_mr_fwd(const void *q, const void *k, const void *v, const float *h, void *y,
                       int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype,
                       void *hip_stream);

/*
 * One rank's share of a sequence-sharded forward call (Sec. 4, the point-to-point scheme for FIR filters: a
 * rank needs, beyond its own steps, only the last lh - 1 steps of k and v of its left neighbour).  Same
 * operator as hyena_se_fwd / hyena_mr_fwd on the shard's L steps,
 *     y[b,t,c] = q[b,t,c] * sum_{j<lh} h[c/group, j] * k[b,t-j,c] * v[b,t-j,c],   t = 0 .. L-1,
 * except that rows t - j < 0 are not all zero: the `history` rows in front of row 0 of k and v (device memory
 * at negative offsets from the pointers, i.e. the neighbour's rows received in front of the shard, or simply
 * the preceding rows when the shard is a window of a longer tensor) hold real steps; rows before those are
 * zero.  history = 0 is the start of a sequence; history >= lh - 1 an interior shard; values in between are
 * a shard that begins fewer than lh - 1 steps into the sequence.
 * Layout: row t of batch item b of k and v is at element offset b * batch_stride_kv + t * D from the pointer,
 * of q and y at b * batch_stride_qy + t * D (D contiguous as everywhere); the strides are ignored when B = 1,
 * else batch_stride_kv >= (L + history) * D, batch_stride_qy >= L * D (HY_ERR_SHAPE) and both a multiple of
 * 16 bytes (HY_ERR_ALIGN).  The overlap rules apply to the memory really touched (history rows included).
 * Kernels: the short-filter stencil and tile walker, the grouped matrix-core kernel, the batched 4x4x4
 * chunk-parallel kernel for medium filters that are not shared by 16 channels, and the general kernel for every
 * other shape.
 * Results of a sequence computed in shards equal the unsharded call's up to the rounding order of the fp32
 * sums (bit for bit on the short-filter paths, whose tap order is fixed).
 * No collective is issued here: exchanging the halo rows is the caller's business.
 */
hy_status hyena_se_fwd_shard(const void *q, const void *k, const void *v, const float *h, void *y,
                             int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype,
                             int64_t batch_stride_kv, int64_t batch_stride_qy, int32_t history,
                             void *hip_stream);
hy_status hyena_mr_fwd_shard(const void *q, const void *k, const void *v, const float *h, void *y,
                             int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype,
                             int64_t batch_stride_kv, int64_t batch_stride_qy, int32_t history,
                             void *hip_stream);

/*
 * Hyena-LI inner operator, forward (Sec. 2.1, the "long implicit" filter; gates as in Eq. 1 / Algorithm 1):
 *     y[b,t,c] = q[b,t,c] * sum_{j=0}^{t} h[c/group, j] * k[b,t-j,c] * v[b,t-j,c],
 *     h[g, j]  = sum_{n=0}^{order-1} R[g,n] * lambda[g,n]^j         (the paper's h_t with t = j + 1)
 * The filter is as long as the sequence and is never materialised: the sum of exponentials is evaluated
 * in its recurrent form, as a chunked scan whose per-chunk products run on the bf16 matrix cores with
 * fp32 accumulation (HY_BF16, group a multiple of 16, D a multiple of 64); u = k*v and the first 32
 * filter values are rounded once to bf16; the running sums stay in fp32 and, like the powers of the
 * poles that feed and read them, enter the products with 16 significant bits (two bf16 parts), so that
 * filters whose exponentials nearly cancel keep their accuracy.  Other valid combinations (fp32 storage, other
 * group sizes or widths, more than 16 exponentials) run the plain recurrence, one lane per channel, with its
 * running sums in fp64.  1 <= order <= 64, else HY_ERR_UNSUPPORTED; the matrix-core scan takes order <= 16.
 * q,k,v,y: [B,L,D] of `dtype` (device); R, lambda: fp32 [D/group, order] (device).  |lambda| <= 1 is the
 * caller's business: larger poles overflow like the definition does.
 * workspace: device memory of at least hyena_li_workspace_bytes(...) bytes, 16-byte aligned, disjoint
 * from every argument, owned by the caller, contents undefined afterwards; may be NULL when that size
 * is 0.  workspace_bytes is its size: HY_ERR_SHAPE if too small or negative.
 */
hy_status hyena_li_fwd(const void *q, const void *k, const void *v, const float *R, const float *lambda,
                       void *y, void *workspace, int64_t workspace_bytes, int64_t B, int64_t L, int64_t D,
                       int32_t order, int32_t group, int32_t dtype, void *hip_stream);

/* Bytes of workspace hyena_li_fwd needs for this problem under the current tuning options (0 when the
 * sequence is scanned in one piece or by the general kernel), -1 if the arguments are not a valid
 * problem.  Host-only. */
int64_t hyena_li_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t order, int32_t group,
                                 int32_t dtype);

/*
 * hyena_li_fwd on one stretch of a longer sequence (Sec. 2.1: the filter is a sum of real exponentials, so
 * everything before a step acts on it through `order` running sums per channel; a sequence cut into stretches,
 * in time on one GPU or across ranks, hands those sums from one stretch to the next).  The outputs are those
 * of hyena_li_fwd on the whole sequence restricted to this stretch, up to rounding.
 * state_in:  running sums s[n] = sum_{i < first step} lambda_n^(first step - 1 - i) * k[i] * v[i] left by the steps
 *            before this call, or NULL at the start of a sequence (zeros).
 * state_out: where to leave the sums after this call's last step, or NULL; requires L to be a multiple of 32.
 * Both are device arrays of hyena_li_state_bytes(B, D) bytes, fp32 [B][D/16][64][4]: element
 * [b][g][16*lq + li][r] belongs to exponential n = 4*lq + r (0 for n >= order) of channel 16*g + li; 16-byte
 * aligned, disjoint from every other argument (HY_ERR_ALIGN).  state_out of one call is state_in of the next.
 * Matrix-core scan only: HY_BF16, group a multiple of 16, D a multiple of 64, order <= 16, B, L, D >= 1; anything
 * else returns HY_ERR_UNSUPPORTED.  workspace as for hyena_li_fwd (same size query).
 */
hy_status hyena_li_fwd_carry(const void *q, const void *k, const void *v, const float *R, const float *lambda,
                             void *y, const float *state_in, float *state_out, void *workspace,
                             int64_t workspace_bytes, int64_t B, int64_t L, int64_t D, int32_t order, int32_t group,
                             int32_t dtype, void *hip_stream);

/* Bytes of a Hyena-LI state for hyena_li_fwd_carry: B * D * 64; -1 if D is not a multiple of 16.  Host-only. */
int64_t hyena_li_state_bytes(int64_t B, int64_t D);

/*
 * The two calls that let the stretches of a Hyena-LI sequence run at the same time (Sec. 4 applied to the recurrent
 * form of Sec. 2.1: ranks exchange `order` running sums per channel instead of a halo).
 *
 * hyena_li_state: the running sums after the call's L steps, from k and v alone (no q, no y): what
 * hyena_li_fwd_carry would leave in state_out, at the cost of one read of k and v.  state_in as there (NULL: the
 * sequence starts here); L a multiple of 32; bf16, group % 16 == 0, D % 64 == 0, order <= 16
 * (else HY_ERR_UNSUPPORTED).  workspace: hyena_li_state_workspace_bytes(...) bytes.
 *
 * hyena_li_state_fold: given the end states of n_states consecutive stretches of `steps` steps each, every one
 * walked from a zero state (states: fp32 [n_states][B][D/16][64][4], the layout above), the state after all of
 * them:  state_out = Lambda^(n_states * steps) state_in + sum_i Lambda^((n_states - 1 - i) * steps) states[i]
 * (state_in NULL: zero; n_states = 0: state_out = state_in or zero).  Powers of the poles by repeated squaring in
 * fp32.  A rank that holds stretch r of a sequence calls hyena_li_state on its k, v with a zero state, gathers
 * everyone's result, folds those of stretches 0 .. r-1 and passes the outcome to hyena_li_fwd_carry as state_in.
 * Both calls are asynchronous on hip_stream and allocate nothing; every written buffer must be disjoint from the
 * others (HY_ERR_ALIGN).
 */
hy_status hyena_li_state(const void *k, const void *v, const float *lambda, const float *state_in, float *state_out,
                         void *workspace, int64_t workspace_bytes, int64_t B, int64_t L, int64_t D, int32_t order,
                         int32_t group, int32_t dtype, void *hip_stream);
int64_t hyena_li_state_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t order, int32_t group, int32_t dtype);
hy_status hyena_li_state_fold(const float *states, int64_t n_states, int64_t steps, const float *lambda,
                              const float *state_in, float *state_out, int64_t B, int64_t D, int32_t order,
                              int32_t group, void *hip_stream);

/*
 * hyena_li_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and bit-identical
 * results; the end-of-tile states of the scan go to a buffer of HYENA_LI_STATIC_SCRATCH_BYTES = 4 MiB that is
 * part of the library's code object (one copy per GPU, held until the process ends) instead of a caller's
 * workspace.  The call allocates nothing, frees nothing and calls no allocating routine.
 * Limit: a problem whose hyena_li_workspace_bytes(...) exceeds that size returns HY_ERR_SCRATCH and launches
 * nothing.  With the built-in tile choice the scan never needs more than 4 MiB (one workgroup per compute
 * unit: B * tiles * D / 256 <= 256 records of 16 KiB), so this only happens with a small "mr_rows" option.
 * All calls on one GPU share that GPU's buffer: two calls that overlap in time on the same GPU (different
 * streams, or different threads) race on it and give wrong results; calls in stream order are safe, and no
 * call depends on what an earlier one left behind.  The buffer's device address is looked up once per GPU,
 * on the first call made while that GPU is current; make that first call outside graph capture.
 */
#define HYENA_LI_STATIC_SCRATCH_BYTES (4 * 1024 * 1024)
hy_status hyena_li_fwd_static(const void *q, const void *k, const void *v, const float *R, const float *lambda,
                              void *y, int64_t B, int64_t L, int64_t D, int32_t order, int32_t group,
                              int32_t dtype, void *hip_stream);

/*
 * Featurizer convolution, forward (Sec. 2.1 Eq. 1, first three lines: the short explicit filters
 * h_T, h_H, h_K applied to the projected q, k, v; no gating):
 *     y[b,t,c] = sum_{j=0}^{min(lh-1,t)} h[c/group, j] * x[b,t-j,c]
 * x,y: [B,L,D] of `dtype`; h: fp32 [D/group, lh].
 */
hy_status hyena_featurize_fwd(const void *x, const float *h, void *y, int64_t B, int64_t L,
                              int64_t D, int32_t lh, int32_t group, int32_t dtype,
                              void *hip_stream);

/*
 * The three featurizer convolutions of Eq. 1 in one launch: qo = hq * q, ko = hk * k, vo = hv * v,
 * each as hyena_featurize_fwd.  All six tensors share one shape and dtype, the three filters share
 * lh and group.
 */
hy_status hyena_featurize3_fwd(const void *q, const void *k, const void *v, const float *hq,
                               const float *hk, const float *hv, void *qo, void *ko, void *vo,
                               int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group,
                               int32_t dtype, void *hip_stream);

/*
 * The Hyena-MR operator chain of Sec. 2.1 Eq. 1 without its dense projections, forward:
 *     q' = hq * q,  k' = hk * k,  v' = hv * v      (featurizers: lf taps, filters [D/feat_group, lf])
 *     y[b,t,c] = q'[b,t,c] * sum_{j=0}^{min(lh-1,t)} h[c/group, j] * k'[b,t-j,c] * v'[b,t-j,c]
 * For HY_BF16 with group a multiple of 16, D a multiple of 128, lh <= 129 and lf <= 9 this is ONE kernel:
 * q, k, v are read once, y is written once, q', k', v' stay on chip in fp32 (u = k'v' is rounded once to
 * bf16 for the matrix cores, y once at the store); `workspace` is not touched and may be NULL.  The
 * featurizers run on the matrix cores too (per-channel Toeplitz products, App. A.1; the bf16 inputs enter
 * exactly, each fp32 tap as a bf16 head plus a bf16 remainder, i.e. to 16 mantissa bits, fp32 accumulation).
 * Every other valid problem is run as hyena_featurize3_fwd into `workspace` followed by hyena_mr_fwd;
 * `workspace` must then hold 3*B*L*D elements of `dtype` (16-byte aligned, disjoint from all other
 * arguments), the featurized tensors are rounded to `dtype` there.  hyena_chain_workspace_bytes tells
 * which case applies; workspace_bytes is the size of `workspace` (HY_ERR_SHAPE if negative or too small).
 * q,k,v,y: [B,L,D] of `dtype`; hq,hk,hv: fp32 [D/feat_group, lf]; h: fp32 [D/group, lh].
 */
hy_status hyena_chain_fwd(const void *q, const void *k, const void *v, const float *hq, const float *hk,
                          const float *hv, const float *h, void *y, void *workspace, int64_t workspace_bytes,
                          int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh,
                          int32_t group, int32_t dtype, void *hip_stream);

/*
 * Bytes of workspace hyena_chain_fwd needs for this problem: 0 when the single-kernel path applies,
 * 3*B*L*D*sizeof(dtype) otherwise, -1 if the arguments are not a valid problem.  Host-only, no HIP call.
 */
int64_t hyena_chain_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group,
                                    int32_t lh, int32_t group, int32_t dtype);

/*
 * One rank's share of a sequence-sharded hyena_chain_fwd call (Sec. 4, point-to-point scheme, for the whole
 * operator of Eq. 1): the shard's L steps, with `history` rows of q, k AND v in front of row 0 of each (device
 * memory at negative offsets) that hold the steps before the shard; rows before those are zero.  An interior
 * shard passes history >= (lh - 1) + (lf - 1): the medium filter reaches lh - 1 steps back into k' v', each of
 * which reaches lf - 1 steps further back into k and v (q' needs lf - 1); the first shard passes 0.
 * Row t of batch item b of q, k, v is at element offset b * batch_stride_in + t * D (>= (L + history) * D), of y
 * at b * batch_stride_y + t * D (>= L * D); ignored for B = 1; multiples of 16 bytes.
 * Single-kernel path only (HY_BF16, group a multiple of 16, D a multiple of 128, lh <= 129, lf <= 9): other
 * shapes return HY_ERR_UNSUPPORTED.  No workspace.
 */
hy_status hyena_chain_fwd_shard(const void *q, const void *k, const void *v, const float *hq, const float *hk,
                                const float *hv, const float *h, void *y, int64_t B, int64_t L, int64_t D,
                                int32_t lf, int32_t feat_group, int32_t lh, int32_t group, int32_t dtype,
                                int64_t batch_stride_in, int64_t batch_stride_y, int32_t history,
                                void *hip_stream);

/*
 * Backward of hyena_se_fwd / hyena_mr_fwd: gradients of y = q (.) (h * (k (.) v)) given dy = dLoss/dy.
 * With u = k*v, z = h * u (the forward sum of Sec. 3.1 Eq. 2) and g = dy*q:
 *     dq[b,t,c] = dy[b,t,c] * z[b,t,c]
 *     du[b,s,c] = sum_{j<lh, s+j<L} h[c/group, j] * g[b,s+j,c]
 *     dk = du * v,   dv = du * k
 *     dh[G,j]   = sum_b sum_{c in group G} sum_{t>=j} g[b,t,c] * u[b,t-j,c]
 * Structure as in the paper's backward (App. A.4, two passes): the main kernel produces dq, dk, dv and one
 * partial filter gradient per tile, written contiguously into `workspace`; a second kernel reduces them into dh.
 * dy,q,k,v,dq,dk,dv: [B,L,D] of `dtype`; h: fp32 [D/group, lh]; dh: fp32 [D/group, lh], overwritten.
 * `workspace` must hold hyena_bwd_workspace_bytes(...) bytes (16-byte aligned, disjoint from every other
 * argument; may be NULL when that is 0); it is scratch, its contents after the call are unspecified.
 * Arithmetic is fp32 throughout with one rounding per stored element; dh is summed in fp32, first within a
 * tile in time order, then over tiles and channels in index order (deterministic, no atomics).
 * Short filters (lh <= 8) run a fused streaming stencil.  Medium grouped bf16 filters (group a multiple of 16,
 * D a multiple of 64, 8 < lh <= 129) run on the matrix cores in ONE pass over dy, q, k, v that walks the sequence
 * from its end: dk, dv come from the block-Toeplitz scheme of the forward operator, causal in reversed time; dq
 * from the same Toeplitz operands applied to a window of u blocks, a few chunks late; dh is a second MFMA
 * contraction over the channels of a group (u and g = dy*q are rounded to bf16 for it, partial sums stay fp32).
 * Medium bf16 filters that are not shared by 16 channels (any other group size, D a multiple of 128, 8 < lh <= 129)
 * run chunk-parallel on the matrix cores (App. A.1): dq is the forward operator applied to (dy, k, v), dk and dv the
 * same kernel walking towards the past on g = dy*q (one launch each), dh a per-channel correlation of g and u on
 * the batched 4x4 matrix instruction (g and u rounded to bf16, partial sums fp32).
 * Everything else runs a general fp32 kernel.
 * hyena_se_bwd and hyena_mr_bwd are the same operation and differ only in which shapes they are tuned for.
 */
hy_status hyena_se_bwd(const void *dy, const void *q, const void *k, const void *v, const float *h, void *dq,
                       void *dk, void *dv, float *dh, void *workspace, int64_t workspace_bytes, int64_t B,
                       int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, void *hip_stream);
hy_status hyena_mr_bwd(const void *dy, const void *q, const void *k, const void *v, const float *h, void *dq,
                       void *dk, void *dv, float *dh, void *workspace, int64_t workspace_bytes, int64_t B,
                       int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype, void *hip_stream);

/*
 * Bytes of workspace the backward entry points need for this problem under the current tuning options
 * (0 for shapes served by the general kernel), -1 if the arguments are not a valid problem.  Host-only.
 */
int64_t hyena_bwd_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype);

/*
 * Backward of hyena_featurize_fwd: the featurizer convolutions of Eq. 1 (x' = h * x with Eq. 2, no gates) under
 * the chain rule, with the two-pass filter gradient of App. A.4.  Given dy = dLoss/dx':
 *     dx[b,s,c] = sum_{j<lh, s+j<L} h[c/group, j] * dy[b,s+j,c]
 *     dh[g, j]  = sum_b sum_{c in group g} sum_{t>=j} dy[b,t,c] * x[b,t-j,c]
 * dy, x, dx: device, [B, L, D] row-major of `dtype`, 16-byte aligned, dx distinct from dy and x; h, dh: device,
 * fp32 [D/group, lh], dh distinct from everything else (overlaps: HY_ERR_ALIGN).  Arithmetic as in
 * hyena_se_bwd: fp32 FMA chains in ascending tap order, one rounding per stored element of dx, fp32 partial filter
 * gradients per tile summed in fp64.  Filters of up to 8 taps run one fused streaming pass and need
 * hyena_featurize_bwd_workspace_bytes(...) bytes of device workspace (16-byte aligned, not overlapping any
 * argument; too small: HY_ERR_SHAPE); longer filters take the general kernels and need none.  An empty problem
 * (B, L or D zero) writes a zero dh and nothing else.  Asynchronous on hip_stream; never allocates.
 */
hy_status hyena_featurize_bwd(const void *dy, const void *x, const float *h, void *dx, float *dh, void *workspace,
                              int64_t workspace_bytes, int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group,
                              int32_t dtype, void *hip_stream);
int64_t hyena_featurize_bwd_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype);

/*
 * Backward of hyena_chain_fwd (Eq. 1 as a whole: q' = hq * q, k' = hk * k, v' = hv * v, y = q' (.) (h * (k' (.) v')))
 * by the chain rule, as a composition of the calls above on the caller's stream: hyena_featurize3_fwd recomputes
 * q', k', v'; hyena_mr_bwd gives dq', dk', dv' and dh; hyena_featurize_bwd, once per tensor, gives dq, dk, dv and
 * dhq, dhk, dhv.  The intermediate tensors live in the workspace in the activations' dtype (for bf16 they are
 * rounded to bf16 between the steps, as the forward's two-kernel path rounds q', k', v').
 * dy, q, k, v, dq, dk, dv: device, [B, L, D] of `dtype`; hq, hk, hv, dhq, dhk, dhv: fp32 [D/feat_group, lf];
 * h, dh: fp32 [D/group, lh]; the usual alignment and overlap rules (every gradient distinct from everything else).
 * workspace: hyena_chain_bwd_workspace_bytes(...) bytes (six tensors plus what the inner calls need), 16-byte
 * aligned, disjoint from every argument; too small: HY_ERR_SHAPE.  An empty problem writes zero filter gradients.
 */
hy_status hyena_chain_bwd(const void *dy, const void *q, const void *k, const void *v, const float *hq,
                          const float *hk, const float *hv, const float *h, void *dq, void *dk, void *dv,
                          float *dhq, float *dhk, float *dhv, float *dh, void *workspace, int64_t workspace_bytes,
                          int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh,
                          int32_t group, int32_t dtype, void *hip_stream);
int64_t hyena_chain_bwd_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lf, int32_t feat_group, int32_t lh,
                                        int32_t group, int32_t dtype);

/*
 * One rank's share of a sequence-sharded backward call (Sec. 4, point-to-point scheme; App. A.4).  Same
 * gradients as hyena_se_bwd / hyena_mr_bwd on the shard's L steps, with the neighbours' steps where the chain
 * rule reaches across the cuts: dq needs k and v of the `history` rows in front of row 0 (as the forward shard
 * call does), dk and dv need dy and q of the `future` rows behind row L - 1 (device memory directly after the
 * shard's rows of dy and q: the right neighbour's first rows); rows beyond those are zero.  history = 0 /
 * future = 0 mark the first / last shard of a sequence; interior shards pass lh - 1 for both.
 * dh receives THIS shard's share of the filter gradient: the shares of all shards of a sequence add up to the
 * gradient of the unsharded call (products that straddle a cut are counted by exactly one of the two shards;
 * which one depends on the kernel, the same for every shard of a given problem shape and dtype).
 * Layout: row t of batch item b is at element offset b * stride + t * D from the pointer, with
 * batch_stride_kv for k and v (>= (L + history) * D), batch_stride_gq for dy and q (>= (L + future) * D) and
 * batch_stride_out for dq, dk, dv (>= L * D); ignored when B = 1; multiples of 16 bytes (HY_ERR_ALIGN), too
 * small: HY_ERR_SHAPE.  The overlap rules apply to the memory really touched.
 * workspace: hyena_bwd_shard_workspace_bytes(...) bytes, for the shard's own B, L, D (every kernel that serves
 * hyena_se_bwd / hyena_mr_bwd also takes shards; the size is the one hyena_bwd_workspace_bytes gives for the same
 * arguments, asked through this function so that the pairing stays explicit).
 */
hy_status hyena_se_bwd_shard(const void *dy, const void *q, const void *k, const void *v, const float *h, void *dq,
                             void *dk, void *dv, float *dh, void *workspace, int64_t workspace_bytes, int64_t B,
                             int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype,
                             int64_t batch_stride_kv, int64_t batch_stride_gq, int64_t batch_stride_out,
                             int32_t history, int32_t future, void *hip_stream);
hy_status hyena_mr_bwd_shard(const void *dy, const void *q, const void *k, const void *v, const float *h, void *dq,
                             void *dk, void *dv, float *dh, void *workspace, int64_t workspace_bytes, int64_t B,
                             int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype,
                             int64_t batch_stride_kv, int64_t batch_stride_gq, int64_t batch_stride_out,
                             int32_t history, int32_t future, void *hip_stream);
int64_t hyena_bwd_shard_workspace_bytes(int64_t B, int64_t L, int64_t D, int32_t lh, int32_t group, int32_t dtype);

/*
 * Plain device-to-device streaming copy of `bytes` bytes (a multiple of 16) with the same launch
 * shape as the streaming kernels.  Used to measure the practical HBM ceiling and to calibrate
 * hardware byte counters; not part of the operator.
 */
hy_status hyena_stream_copy(const void *src, void *dst, int64_t bytes, void *hip_stream);

/*
 * Bandwidth yardstick with the operator's traffic and none of its arithmetic: y = q * k * v elementwise on bf16
 * [B, L, D] tensors (the gated convolution of Eq. 1 with a one-tap unit filter), three tensors read once and one
 * written once with the streaming hints the operator kernels use.  strip_channels = 0 streams the tensors
 * linearly; 64, 128 or 256 makes a workgroup walk a column strip of that many channels (128, 256 or 512 bytes
 * per row) down `rows` time steps (0 = tile length that gives one workgroup per compute unit), which is how the
 * matrix-core kernels move their data, with `depth` chunks of loads in flight per lane (1, 2, 3, 4, 6 or 8;
 * 0 = 2, what the operator kernels use; ignored by the linear stream) and one workgroup barrier per chunk.
 * `waves` = waves per workgroup: 0 = strip_channels / 16 (one wave per 16 channels, 32-row chunks: the operator
 * kernels' shape), or 4, 8, 16 with 16 * waves <= strip_channels (a chunk is then 512 * waves / strip_channels
 * rows: fewer, fatter streams per compute unit); must be 0 for the linear stream.  D must be a multiple of 8 and
 * of strip_channels.  Unsupported combinations return HY_ERR_UNSUPPORTED.  Not part of the operator: it measures
 * the practical ceiling a kernel with that access pattern can reach.
 */
hy_status hyena_stream_gate(const void *q, const void *k, const void *v, void *y, int64_t B, int64_t L, int64_t D,
                            int32_t strip_channels, int64_t rows, int32_t depth, int32_t waves, void *hip_stream);

/*
 * Tuning knobs (process-wide; 0 restores the built-in choice).  Thread-safe: every entry point takes one
 * consistent snapshot of all options when it is entered, so an option set by another thread during a call
 * affects later calls only; a *_workspace_bytes query and the call it sizes agree as long as no option that
 * matters to them is set in between (if one is, the call notices the short workspace: HY_ERR_SHAPE).  Names:
 *   "se_vec"   channels per lane in the SE / featurizer stencil (1, 2, 4 or 8)
 *   "se_rows"  time steps each lane walks (tile length in t)
 *   "mr_rows"  time steps per workgroup in the MR and chain kernels (multiple of 32)
 *   "mr_waves" waves (= 16-channel groups) per workgroup in the MR and Hyena-LI kernels (4, 8 or 16)
 *   "se_walk"  which kernel hyena_se_fwd takes for bf16 filters of up to 8 taps: 0 = by problem size,
 *              1 = always the long-sequence kernel (where D is a multiple of 128), 2 = always the stencil
 * Unknown names return HY_ERR_UNSUPPORTED.  Results depend on these only through rounding, within the
 * documented precision of each entry point.
 */
hy_status hyena_set_option(const char *name, int32_t value);

/* Static, NUL-terminated description of a status code. */
const char *hyena_status_string(int32_t status);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t hyena_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HYENA_H */
