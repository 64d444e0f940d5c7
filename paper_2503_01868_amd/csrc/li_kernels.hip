// Hyena-LI forward on gfx950: gated causal convolution with the long implicit filter of Sec. 2.1,
//   h[g, j] = sum_{n < order} R[g, n] * lambda[g, n]^j,   j = 0 .. L-1  (as long as the sequence).
// The filter is never materialised.  Because it is a sum of real exponentials, everything older than the
// current 32-step chunk acts through `order` running sums per channel (the recurrent form the paper
// mentions for this operator), and the whole operator becomes three small dense products per chunk:
//   z_chunk = T u_chunk + Q s,        T[t, i] = h[t - i] (lower triangular, 32 x 32: the H_0 of Sec. 3.1),
//                                      Q[t, n] = R_n lambda_n^(t+1),
//   s'      = Lambda^32 s + P u_chunk, P[n, i] = lambda_n^(31-i),   s[n, c] = sum_{i<=end} lambda_n^(end-i) u[i, c].
// With 16 channels of one filter group on a matrix tile (as in mr_kernels.hip) these are two
// v_mfma_f32_16x16x32_bf16 for T, one for P and two pairs of v_mfma_f32_16x16x16_bf16 for Q; s stays in fp32
// accumulators and enters the Q product split into a bf16 head and a bf16 remainder, so carrying the state
// over 10^5 steps costs no precision beyond the bf16 rounding of the coefficients.  The state product comes
// out with 4 consecutive n of one channel per lane, which is exactly the operand layout of the Q product:
// the state never leaves its registers.
//
// The recurrence runs along time, and one GPU needs more than B * D / 256 workgroups, so the sequence is cut
// into tiles and scanned in two passes (the classic chunked scan): pass 1 walks every tile but the last of
// each sequence with a zero start and leaves the tile's final state in a workspace (reads k and v only);
// pass 2 rebuilds its start state from the tiles before it, s_in = sum_tau Lambda^(rows * (tile-1-tau)) s_tau
// (a short Horner loop over 1 KiB records), and computes y.  With a single tile per sequence pass 1 is skipped.
// Data movement per chunk is that of mr_kernels.hip: whole row pieces, u and z through LDS, one barrier.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct LiArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* R;
    const float* lam;
    uint16_t* y;
    float* ws;              // [B][tiles_per_seq - 1][D / 16][64 lanes][4] end-of-tile states
    const float* s_in;      // [B][D / 16][64 lanes][4] running sums before the first step (nullptr: zero)
    float* s_out;           // same layout: running sums after the last step (nullptr: not wanted)
    int64_t L, D;
    int32_t order, group;
    int32_t rows;           // time steps per workgroup, multiple of 32
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / (16 NW)
};

constexpr int kChunk = 32;
constexpr int kMaxOrder = 16;

__device__ __forceinline__ float powi(float x, int e) {  // x^e, e >= 0, by squaring
    float r = 1.0f;
    while (e > 0) {
        if (e & 1) r *= x;
        x *= x;
        e >>= 1;
    }
    return r;
}

// kStateOnly: pass 1 (no q, no output, the tile's final state goes to the workspace).
template <int NW, int kPrefetch, bool kStateOnly>
__global__ __launch_bounds__(NW * 64, NW == 16 ? 4 : 2) void li_mfma_kernel(LiArgs a) {
    constexpr int PPR = 2 * NW;             // 16-byte pieces per staged row of u (bf16)
    constexpr int ZROW = 16 * NW * 4 + 16;  // bytes per staged row of z (fp32), padded against bank conflicts
    static_assert(NW % 4 == 0, "the LDS swizzle needs 8 pieces per row");
    __shared__ uint4 stage[2][kChunk * PPR];
    __shared__ __attribute__((aligned(16))) char zst[kStateOnly ? 1 : 2][kStateOnly ? 16 : kChunk * ZROW];
    __shared__ float rs[NW][kMaxOrder], ls[NW][kMaxOrder], hs[NW][kChunk];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const int li = lane % 16, lq = lane / 16;

    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tl = lb / a.ncb;
    const int tiles_run = kStateOnly ? a.tiles_per_seq - 1 : a.tiles_per_seq;  // pass 1 skips the last tile
    const int64_t b = tl / tiles_run;
    const int tile = (int)(tl % tiles_run);
    const int64_t t_start = (int64_t)tile * a.rows;
    const int64_t t_end = (t_start + a.rows < a.L) ? t_start + a.rows : a.L;
    const int nchunks = (int)((t_end - t_start + kChunk - 1) / kChunk);

    const int64_t D = a.D;
    const int64_t cblock0 = (int64_t)cb * 16 * NW;
    const int64_t c0 = cblock0 + 16 * w;
    const int64_t seq0 = b * a.L * D;

    const int lr = tid / PPR, lp = tid % PPR;
    const int64_t ld_off = cblock0 + 8 * lp;
    // unconditional, clamped loads (see mr_kernels.hip): rows past the end of the tile re-read its last row; loads
    // for chunk indices past the last chunk (results unused) all go to one 16-byte location of the tile
    const int64_t idle_off = (t_end - 1) * D + cblock0;
    auto load_kv = [&](int ci, Words<4>& kk, Words<4>& vv) {
        int64_t t = t_start + (int64_t)ci * kChunk + lr;
        t = t < t_end ? t : t_end - 1;
        const int64_t off = ci < nchunks ? t * D + ld_off : idle_off;
        kk = load_words_nt<4>(a.k + seq0 + off);
        vv = load_words_nt<4>(a.v + seq0 + off);
    };
    auto load_q = [&](int ci, Words<4>& qq) {
        int64_t t = t_start + (int64_t)ci * kChunk + lr;
        t = t < t_end ? t : t_end - 1;
        qq = load_words_nt<4>(a.q + seq0 + (ci < nchunks ? t * D + ld_off : idle_off));
    };

    Words<4> kpre[kPrefetch], vpre[kPrefetch], qpre[kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) {
        load_kv(i, kpre[i], vpre[i]);
        if constexpr (!kStateOnly)
            if (i + 1 < kPrefetch) load_q(i, qpre[i]);
    }

    // ---- per-wave filter set-up: residues and poles of the wave's group, taps 0..31 of the implicit filter
    {
        const int64_t g = c0 / a.group;
        if (lane < kMaxOrder) {
            rs[w][lane] = lane < a.order ? a.R[g * a.order + lane] : 0.0f;
            ls[w][lane] = lane < a.order ? a.lam[g * a.order + lane] : 0.0f;
        }
    }
    __syncthreads();
    // ---- start state: zero at the start of a sequence, else the Horner sum over the earlier tiles' end states,
    // sixteen records per round (the loads do not depend on the running sum, only the FMAs do; indices past the
    // last record are clamped so that the loads stay unconditional), so that up to sixteen earlier tiles cost one
    // memory latency.  Done before the operands are built, while few registers are live.
    // state layout: lane (li = channel, lq) holds s[n = 4lq + r][channel], r = 0..3
    f32x4_t s = {0.0f, 0.0f, 0.0f, 0.0f};
    const int64_t ws_wave = ((c0 / 16) * 64 + lane) * 4;  // this lane's 4 floats inside one (b, tile) record set
    const int64_t ws_tile = (D / 16) * 256;               // floats per (b, tile)
    if constexpr (!kStateOnly) {
        if (a.s_in) {  // a call that continues a sequence: what the steps before it left behind decays like any state
            const float4 c4 = *reinterpret_cast<const float4*>(a.s_in + b * ws_tile + ws_wave);
            s = f32x4_t{c4.x, c4.y, c4.z, c4.w};
        }
        float lam_rows[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) lam_rows[r] = powi(ls[w][4 * lq + r], a.rows);
        const float* wp = a.ws + b * (a.tiles_per_seq - 1) * ws_tile + ws_wave;
        for (int tau0 = 0; tau0 < tile; tau0 += 16) {
            float4 st[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int tau = tau0 + i < tile ? tau0 + i : tile - 1;
                st[i] = *reinterpret_cast<const float4*>(wp + tau * ws_tile);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (tau0 + i < tile) {
                    s[0] = lam_rows[0] * s[0] + st[i].x;
                    s[1] = lam_rows[1] * s[1] + st[i].y;
                    s[2] = lam_rows[2] * s[2] + st[i].z;
                    s[3] = lam_rows[3] * s[3] + st[i].w;
                }
            }
        }
    }

    if (lane < kChunk) {
        float hj = 0.0f;
        for (int n = 0; n < kMaxOrder; ++n) hj += rs[w][n] * powi(ls[w][n], lane);
        hs[w][lane] = hj;
    }
    __syncthreads();

    // T operands: tile x (steps 16x..16x+15 of the chunk) against the chunk's 32 source steps; lane (li = step,
    // lq = source octet), element e = h[16x + li - 8lq - e]
    bf16x8_t tz[2];
    if constexpr (!kStateOnly) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            Words<4> wds;
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const int i0 = 16 * x + li - 8 * lq - 2 * e2;
                const int i1 = i0 - 1;
                const float f0 = (i0 >= 0 && i0 < kChunk) ? hs[w][i0] : 0.0f;
                const float f1 = (i1 >= 0 && i1 < kChunk) ? hs[w][i1] : 0.0f;
                wds.w[e2] = pack_bf16x2(f0, f1);
            }
            tz[x] = __builtin_bit_cast(bf16x8_t, wds);
        }
    }
    // P operand: lane (li = n, lq = source octet), element e = lambda_n^(31 - 8lq - e), as a bf16 head and a bf16
    // remainder.  The exponentials of a filter may nearly cancel (close poles, residues of opposite sign); each
    // one's running sum therefore has to be accurate well beyond bf16, or the error of the individual terms shows
    // at full size in their small difference.  The same holds for the Q operands below.
    bf16x8_t pop, pop_lo;
    {
        const float ln = ls[w][li];
        Words<4> wds, wlo;
        float pw = powi(ln, 31 - 8 * lq - 7);  // smallest exponent of the lane (element 7), then multiply up
        float pe[8];
#pragma unroll
        for (int e = 7; e >= 0; --e) {
            pe[e] = pw;
            pw *= ln;
        }
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            wds.w[e2] = pack_bf16x2(pe[2 * e2], pe[2 * e2 + 1]);
            wlo.w[e2] = pack_bf16x2(pe[2 * e2] - bf16_lo(wds.w[e2]), pe[2 * e2 + 1] - bf16_hi(wds.w[e2]));
        }
        pop = __builtin_bit_cast(bf16x8_t, wds);
        pop_lo = __builtin_bit_cast(bf16x8_t, wlo);
    }
    float lam32[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) lam32[r] = powi(ls[w][4 * lq + r], kChunk);
    // Q operands: lane (li = step of tile x, lq), element e = R_n lambda_n^(16x + li + 1), n = 4lq + e
    s16x4_t qop[2], qop_lo[2];
    if constexpr (!kStateOnly) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            float qe[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) qe[e] = rs[w][4 * lq + e] * powi(ls[w][4 * lq + e], 16 * x + li + 1);
            Words<2> wds, wlo;
            wds.w[0] = pack_bf16x2(qe[0], qe[1]);
            wds.w[1] = pack_bf16x2(qe[2], qe[3]);
            wlo.w[0] = pack_bf16x2(qe[0] - bf16_lo(wds.w[0]), qe[1] - bf16_hi(wds.w[0]));
            wlo.w[1] = pack_bf16x2(qe[2] - bf16_lo(wds.w[1]), qe[3] - bf16_hi(wds.w[1]));
            qop[x] = __builtin_bit_cast(s16x4_t, wds);
            qop_lo[x] = __builtin_bit_cast(s16x4_t, wlo);
        }
    }

    const int swz = ((lr >> 3) & 3) << 1;
    const int st_idx = lr * PPR + (lp ^ swz);
    const int rd_piece = (2 * w + (li >> 3)) ^ (lq << 1);
    const int zwr_off = li * ZROW + (16 * w + 4 * lq) * 4;
    const int zrd_off = lr * ZROW + 8 * lp * 4;

    auto gate_store = [&](int ci, const Words<4>& qq) {
        const int64_t t = t_start + (int64_t)ci * kChunk + lr;
        if (t < t_end) {
            const char* zp = zst[ci & 1] + zrd_off;
            const float4 za = *reinterpret_cast<const float4*>(zp);
            const float4 zb = *reinterpret_cast<const float4*>(zp + 16);
            float qf[8];
            Pack<BF16, 8>::unpack(qq, qf);
            float y8[8] = {za.x * qf[0], za.y * qf[1], za.z * qf[2], za.w * qf[3],
                           zb.x * qf[4], zb.y * qf[5], zb.z * qf[6], zb.w * qf[7]};
            store_words_nt<4>(a.y + seq0 + t * D + ld_off, Pack<BF16, 8>::pack(y8));
        }
    };

    for (int base = 0; base < nchunks; base += kPrefetch) {
#pragma unroll
        for (int sgi = 0; sgi < kPrefetch; ++sgi) {
            const int ci = base + sgi;
            const bool live = ci < nchunks;
            {
                float kf[8], vf[8];
                Pack<BF16, 8>::unpack(kpre[sgi], kf);
                Pack<BF16, 8>::unpack(vpre[sgi], vf);
                Words<4> uu;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2)
                    uu.w[e2] = pack_bf16x2(kf[2 * e2] * vf[2 * e2], kf[2 * e2 + 1] * vf[2 * e2 + 1]);
                stage[ci & 1][st_idx] = make_uint4(uu.w[0], uu.w[1], uu.w[2], uu.w[3]);
            }
            load_kv(ci + kPrefetch, kpre[sgi], vpre[sgi]);

            __syncthreads();

            // transposed read: element e of this lane = u[row 8 lq + e][channel 16 w + li]
            bf16x8_t uw;
            {
                const uint16_t* s16 = reinterpret_cast<const uint16_t*>(stage[ci & 1]);
                Words<4> wds;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int r0 = 8 * lq + 2 * e2;
                    const uint32_t lo = s16[((r0 * PPR + rd_piece) << 3) + (li & 7)];
                    const uint32_t hi = s16[(((r0 + 1) * PPR + rd_piece) << 3) + (li & 7)];
                    wds.w[e2] = lo | (hi << 16);
                }
                uw = __builtin_bit_cast(bf16x8_t, wds);
            }

            if (live) {
                if constexpr (!kStateOnly) {
                    // carry-in: the state in two bf16 parts, head and remainder
                    const uint32_t h01 = pack_bf16x2(s[0], s[1]), h23 = pack_bf16x2(s[2], s[3]);
                    const uint32_t l01 = pack_bf16x2(s[0] - bf16_lo(h01), s[1] - bf16_hi(h01));
                    const uint32_t l23 = pack_bf16x2(s[2] - bf16_lo(h23), s[3] - bf16_hi(h23));
                    Words<2> hw, lw;
                    hw.w[0] = h01; hw.w[1] = h23;
                    lw.w[0] = l01; lw.w[1] = l23;
                    const s16x4_t shi = __builtin_bit_cast(s16x4_t, hw), slo = __builtin_bit_cast(s16x4_t, lw);
                    // smallest terms first: head of the state against the remainder of Q, remainder of the state
                    // against the head of Q, then the heads, then the chunk's own Toeplitz block.  The order of the
                    // two instruction shapes matters beyond rounding: a 16x16x16 product that accumulates onto the
                    // result of a 16x16x32 product issued fewer than 5 wait states earlier reads the register's
                    // previous contents on gfx950 (measured), and the compiler does not always leave that distance;
                    // 16x16x16 results feeding a 16x16x32 product are interlocked by the hardware.  Every 16x16x16
                    // product below accumulates onto zero or onto another 16x16x16 result, so the unsafe pair cannot
                    // arise from this source by data dependence; tests/test_isa_hazards.py checks the generated code
                    // of this file for the pair on every build.
                    f32x4_t acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(shi, qop_lo[0], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(shi, qop_lo[1], acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(slo, qop[0], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(slo, qop[1], acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(shi, qop[0], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(shi, qop[1], acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(uw, tz[0], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(uw, tz[1], acc1, 0, 0, 0);
                    char* zp = zst[ci & 1] + zwr_off;
                    *reinterpret_cast<float4*>(zp) = make_float4(acc0[0], acc0[1], acc0[2], acc0[3]);
                    *reinterpret_cast<float4*>(zp + 16 * ZROW) = make_float4(acc1[0], acc1[1], acc1[2], acc1[3]);
                }
                // state update: s' = Lambda^32 s + P u
                s[0] *= lam32[0];
                s[1] *= lam32[1];
                s[2] *= lam32[2];
                s[3] *= lam32[3];
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pop, uw, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pop_lo, uw, s, 0, 0, 0);
            }
            if constexpr (!kStateOnly) {
                const int prev = (sgi + kPrefetch - 1) % kPrefetch;
                if (ci > 0 && ci <= nchunks) gate_store(ci - 1, qpre[prev]);
                load_q(ci - 1 + kPrefetch, qpre[prev]);
            }
        }
    }
    if constexpr (!kStateOnly) {
        if (nchunks % kPrefetch == 0) {
            __syncthreads();
            gate_store(nchunks - 1, qpre[kPrefetch - 1]);
        }
        if (a.s_out && tile == a.tiles_per_seq - 1)  // (the launcher admits this only for L % 32 == 0: no padded rows)
            *reinterpret_cast<float4*>(a.s_out + b * ws_tile + ws_wave) = make_float4(s[0], s[1], s[2], s[3]);
    } else {
        float* wp = a.ws + (b * (a.tiles_per_seq - 1) + tile) * ws_tile + ws_wave;
        *reinterpret_cast<float4*>(wp) = make_float4(s[0], s[1], s[2], s[3]);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Folding states: out = Lambda^(steps of all records) s_in + sum_i Lambda^(steps after record i) rec_i, where every
// record is the end state of a stretch of `steps` steps walked from zero (`last_steps` for the last one).  This is
// the Horner sum of pass 2's start state as a kernel of its own: it turns the tile records of a state-only walk
// into the state after the walk, and the end states of several ranks' stretches into each rank's start state.
// One lane per float4 of a state ([B][D/16][64 lanes][4]: lane (li, lq) of a 16-channel block holds exponentials
// 4 lq .. 4 lq + 3 of channel li); records of one batch item are rec_stride_i floats apart, batch items rec_stride_b.
__device__ __forceinline__ float powi64(float x, int64_t e) {  // x^e, e >= 0, by squaring
    float r = 1.0f;
    while (e > 0) {
        if (e & 1) r *= x;
        x *= x;
        e >>= 1;
    }
    return r;
}

__global__ __launch_bounds__(256) void li_fold_kernel(const float* __restrict__ rec, int64_t n, int64_t rec_stride_b,
                                                      int64_t rec_stride_i, const float* __restrict__ lam,
                                                      const float* __restrict__ s_in, float* __restrict__ s_out, int64_t B,
                                                      int64_t D, int32_t order, int32_t group, int64_t steps,
                                                      int64_t last_steps) {
    const int64_t per_b = (D / 16) * 64;  // float4s of one batch item's state
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (x >= B * per_b) return;
    const int64_t b = x / per_b, within = x % per_b;
    const int lane = (int)(within % 64);
    const int64_t channel = (within / 64) * 16 + lane % 16;
    const float* lp = lam + (channel / group) * (int64_t)order;
    float pw[4], pl[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int nn = 4 * (lane / 16) + r;
        const float l = nn < order ? lp[nn] : 0.0f;
        pw[r] = powi64(l, steps);
        pl[r] = powi64(l, last_steps);
    }
    float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (s_in) s = *reinterpret_cast<const float4*>(s_in + x * 4);
    const float* rp = rec + b * rec_stride_b + within * 4;
    for (int64_t i0 = 0; i0 < n; i0 += 8) {
        float4 st[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {  // the loads do not depend on the running sum; past the end the last record repeats
            const int64_t ii = i0 + i < n ? i0 + i : n - 1;
            st[i] = *reinterpret_cast<const float4*>(rp + ii * rec_stride_i);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i0 + i < n) {
                const bool last = i0 + i == n - 1;
                s.x = (last ? pl[0] : pw[0]) * s.x + st[i].x;
                s.y = (last ? pl[1] : pw[1]) * s.y + st[i].y;
                s.z = (last ? pl[2] : pw[2]) * s.z + st[i].z;
                s.w = (last ? pl[3] : pw[3]) * s.w + st[i].w;
            }
        }
    }
    *reinterpret_cast<float4*>(s_out + x * 4) = s;
}

// ---------------------------------------------------------------------------------------------------------
// General kernel: the recurrence itself, one lane per (batch item, channel).  Any dtype, any group, up to
// kMaxOrderDirect exponentials; slow (B * D lanes in all), the correctness path for what the matrix-core kernel
// does not take.  The running sums and the output sum are kept in fp64: a slow pole (lambda close to 1) carries
// thousands of steps, and in fp32 one rounding per step and exponential would add up past the 1e-5 that fp32
// storage is held to; in fp64 the only roundings left are the final conversion of z and the gate.  The running
// sums live in registers (MAXO of them); residues and poles of the lane's group sit in LDS.
constexpr int kMaxOrderDirect = 64;

template <typename T, int MAXO>
__global__ __launch_bounds__(64) void li_direct_kernel(const void* qv, const void* kv, const void* vv, const float* R,
                                                       const float* lam, void* yv, int64_t B, int64_t L, int64_t D,
                                                       int32_t order, int32_t group) {
    __shared__ float rtab[MAXO][64], ltab[MAXO][64];  // [exponential][lane]: conflict-free per-lane columns
    const int64_t idx = (int64_t)blockIdx.x * 64 + threadIdx.x;
    const bool live = idx < B * D;
    const int64_t b = live ? idx / D : 0, c = live ? idx % D : 0;
    const int64_t g = c / group;
    double sn[MAXO];
#pragma unroll
    for (int n = 0; n < MAXO; ++n) {
        rtab[n][threadIdx.x] = n < order ? R[g * order + n] : 0.0f;
        ltab[n][threadIdx.x] = n < order ? lam[g * order + n] : 0.0f;
        sn[n] = 0.0;
    }
    if (!live) return;  // (each lane reads only its own column of the tables: no barrier needed)
    const char* qp = static_cast<const char*>(qv);
    const char* kp = static_cast<const char*>(kv);
    const char* vp = static_cast<const char*>(vv);
    char* yp = static_cast<char*>(yv);
    for (int64_t t = 0; t < L; ++t) {
        const int64_t off = ((b * L + t) * D + c) * T::kBytes;
        float qf[1], kf[1], vf[1];
        Pack<T, 1>::unpack(Pack<T, 1>::load(qp + off), qf);
        Pack<T, 1>::unpack(Pack<T, 1>::load(kp + off), kf);
        Pack<T, 1>::unpack(Pack<T, 1>::load(vp + off), vf);
        const double u = (double)kf[0] * (double)vf[0];
        double z = 0.0;
#pragma unroll
        for (int n = 0; n < MAXO; ++n) {
            sn[n] = __builtin_fma((double)ltab[n][threadIdx.x], sn[n], u);
            z = __builtin_fma((double)rtab[n][threadIdx.x], sn[n], z);
        }
        float y1[1] = {(float)((double)qf[0] * z)};
        Pack<T, 1>::store(yp + off, Pack<T, 1>::pack(y1));
    }
}

int64_t li_rows(const LiShape& s, int nw) {
    int64_t rows = tuning().mr_rows;
    const int64_t ncb = s.D / (16 * nw);
    if (rows <= 0) {
        int64_t tiles = 256 / (s.B * ncb);
        if (tiles < 1) tiles = 1;
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 4 * kChunk) rows = 4 * kChunk;
    }
    rows = (rows + kChunk - 1) / kChunk * kChunk;
    const int64_t cap = (s.L + kChunk - 1) / kChunk * kChunk;
    return rows > cap ? cap : rows;
}

int li_waves(const LiShape& s) {
    const int nw = tuning().mr_waves > 0 ? tuning().mr_waves : 16;
    // Left to itself, a problem that gives a 256-channel workgroup fewer than 512 steps takes 128-channel workgroups
    // (half as many tiles per sequence, twice as long): measured at B = 1, D = 4096: L = 2048 29.8 against 32.5 us,
    // L = 4096 45.8 against 48.6; from L = 8192 on the wide workgroup wins (76.2 against 79.2 us).
    if (tuning().mr_waves == 0 && tuning().mr_rows == 0 && s.D % 256 == 0 && li_rows(s, 16) < 512) return 8;
    // A batch that fills the chip with narrower workgroups of ONE tile per sequence takes them: a single pass moves
    // 8 bytes per output where the two-pass scan moves 12 (measured at L = 8192, D = 4096: B = 8 400 us with 8
    // waves against 445 with 16, B = 4 197 us with 4 waves against 241; B = 16 fills it with 16 waves: 695 us, 77%).
    // "Fills" means that at least three quarters of the compute units are busy in every round of 256 workgroups
    // (B = 6: 192 workgroups of 8 waves 309 us against 374; B = 3: 192 of 4 waves 165 us against 190).
    if (tuning().mr_waves == 0 && tuning().mr_rows == 0 && s.D % 256 == 0 && li_rows(s, 16) < s.L) {
        auto fills = [](int64_t wg) { return 4 * wg >= 3 * ((wg + 255) / 256) * 256; };
        if (fills(s.B * (s.D / 128))) return 8;
        if (fills(s.B * (s.D / 64))) return 4;
    }
    if (nw == 16 && s.D % 256 == 0) return 16;
    if (nw >= 8 && s.D % 128 == 0) return 8;
    return 4;
}

hy_status launch_fold(const float* rec, int64_t n, int64_t stride_b, int64_t stride_i, const float* lam, const float* s_in,
                      float* s_out, int64_t B, int64_t D, int32_t order, int32_t group, int64_t steps, int64_t last_steps,
                      hipStream_t st) {
    const int64_t items = B * (D / 16) * 64;
    const int64_t nb = (items + 255) / 256;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel(li_fold_kernel, dim3((uint32_t)nb), dim3(256), st, rec, n, stride_b, stride_i, lam, s_in, s_out, B,
                         D, order, group, steps, last_steps);
}

// State-only walk: pass 1 over EVERY tile (the kernel skips the last of `tiles_per_seq` tiles, so it is told of one
// more than there are), then the fold of the tile records.
template <int NW>
hy_status launch_li_state_nw(const LiPtrs& p, const LiShape& s, void* ws, hipStream_t st) {
    constexpr int PF = 2;
    LiArgs a;
    a.q = nullptr;
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.R = p.lam;  // the state does not depend on the residues; the kernel's set-up reads the table all the same
    a.lam = p.lam;
    a.y = nullptr;
    a.ws = static_cast<float*>(ws);
    a.s_in = nullptr;
    a.s_out = nullptr;
    a.L = s.L;
    a.D = s.D;
    a.order = s.order;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * NW));
    const int64_t rows = li_rows(s, NW);
    a.rows = (int32_t)rows;
    const int64_t tiles = (s.L + rows - 1) / rows;
    a.tiles_per_seq = (int32_t)(tiles + 1);
    const int64_t nb = s.B * tiles * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    const hy_status rc = launch_kernel((li_mfma_kernel<NW, PF, true>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
    if (rc != HY_OK) return rc;
    const int64_t ws_tile = (s.D / 16) * 256;
    return launch_fold(a.ws, tiles, tiles * ws_tile, ws_tile, p.lam, p.state_in, p.state_out, s.B, s.D, s.order, s.group,
                       rows, s.L - (tiles - 1) * rows, st);
}

template <int NW>
hy_status launch_li_nw(const LiPtrs& p, const LiShape& s, void* ws, hipStream_t st) {
    constexpr int PF = 2;
    LiArgs a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.R = p.R;
    a.lam = p.lam;
    a.y = static_cast<uint16_t*>(p.y);
    a.ws = static_cast<float*>(ws);
    a.s_in = p.state_in;
    a.s_out = p.state_out;
    a.L = s.L;
    a.D = s.D;
    a.order = s.order;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * NW));
    const int64_t rows = li_rows(s, NW);
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb2 = s.B * a.tiles_per_seq * a.ncb;
    const int64_t nb1 = s.B * (a.tiles_per_seq - 1) * a.ncb;
    if (nb2 > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    if (nb1 > 0) {
        const hy_status rc = launch_kernel((li_mfma_kernel<NW, PF, true>), dim3((uint32_t)nb1), dim3(NW * 64), st, a);
        if (rc != HY_OK) return rc;
    }
    return launch_kernel((li_mfma_kernel<NW, PF, false>), dim3((uint32_t)nb2), dim3(NW * 64), st, a);
}

}  // namespace

bool li_mfma_supported(const LiShape& s) {
    return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 64 == 0 && s.order >= 1 && s.order <= kMaxOrder &&
           s.L <= 0x7fffffffLL - 64;
}

int64_t li_workspace_bytes(const LiShape& s) {
    if (!li_mfma_supported(s) || s.B == 0 || s.L == 0 || s.D == 0) return 0;
    const int64_t rows = li_rows(s, li_waves(s));
    const int64_t tiles = (s.L + rows - 1) / rows;
    return s.B * (tiles - 1) * (s.D / 16) * 256 * (int64_t)sizeof(float);
}

hy_status launch_li_mfma(const LiPtrs& p, const LiShape& s, void* ws, hipStream_t st) {
    if (!li_mfma_supported(s)) return HY_ERR_UNSUPPORTED;
    // a last chunk with rows past the end would carry them into the state it leaves behind
    if (p.state_out && s.L % kChunk != 0) return HY_ERR_UNSUPPORTED;
    switch (li_waves(s)) {
        case 16: return launch_li_nw<16>(p, s, ws, st);
        case 8: return launch_li_nw<8>(p, s, ws, st);
        default: return launch_li_nw<4>(p, s, ws, st);
    }
}

int64_t li_state_workspace_bytes(const LiShape& s) {
    if (!li_mfma_supported(s) || s.B == 0 || s.L == 0 || s.D == 0) return 0;
    const int64_t rows = li_rows(s, li_waves(s));
    const int64_t tiles = (s.L + rows - 1) / rows;
    return s.B * tiles * (s.D / 16) * 256 * (int64_t)sizeof(float);
}

hy_status launch_li_state(const LiPtrs& p, const LiShape& s, void* ws, hipStream_t st) {
    if (!li_mfma_supported(s) || s.L % kChunk != 0 || !p.state_out) return HY_ERR_UNSUPPORTED;
    switch (li_waves(s)) {
        case 16: return launch_li_state_nw<16>(p, s, ws, st);
        case 8: return launch_li_state_nw<8>(p, s, ws, st);
        default: return launch_li_state_nw<4>(p, s, ws, st);
    }
}

hy_status launch_li_state_fold(const float* states, int64_t n, int64_t steps, const float* lam, const float* state_in,
                               float* state_out, int64_t B, int64_t D, int32_t order, int32_t group, hipStream_t st) {
    if (D % 16 != 0 || order < 1 || order > kMaxOrder) return HY_ERR_UNSUPPORTED;
    const int64_t per = (D / 16) * 256;  // floats of one batch item's state
    return launch_fold(states, n, per, B * per, lam, state_in, state_out, B, D, order, group, steps, steps, st);
}

hy_status launch_li_direct(const LiPtrs& p, const LiShape& s, hipStream_t st) {
    if (s.order < 1 || s.order > kMaxOrderDirect) return HY_ERR_UNSUPPORTED;
    const int64_t n = s.B * s.D;
    const int64_t nb = (n + 63) / 64;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)nb), block(64);
    const bool small = s.order <= kMaxOrder;
    if (s.dtype == HY_F32) {
        if (small)
            return launch_kernel((li_direct_kernel<F32, kMaxOrder>), grid, block, st, p.q, p.k, p.v, p.R, p.lam, p.y, s.B,
                                 s.L, s.D, s.order, s.group);
        return launch_kernel((li_direct_kernel<F32, kMaxOrderDirect>), grid, block, st, p.q, p.k, p.v, p.R, p.lam, p.y,
                             s.B, s.L, s.D, s.order, s.group);
    }
    if (small)
        return launch_kernel((li_direct_kernel<BF16, kMaxOrder>), grid, block, st, p.q, p.k, p.v, p.R, p.lam, p.y, s.B,
                             s.L, s.D, s.order, s.group);
    return launch_kernel((li_direct_kernel<BF16, kMaxOrderDirect>), grid, block, st, p.q, p.k, p.v, p.R, p.lam, p.y, s.B,
                         s.L, s.D, s.order, s.group);
}

}  // namespace hy
