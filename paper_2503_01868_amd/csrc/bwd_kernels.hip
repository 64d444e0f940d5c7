// Backward of the gated causal convolution  y = q (.) (h * (k (.) v))  for the vector-ALU paths.
//
// Given dy, with u = k*v, z = h * u, g = dy*q:
//     dq[t] = dy[t] * z[t]
//     du[s] = sum_{j<lh, s+j<L} h[j] * g[s+j]        (transposed = anti-causal convolution)
//     dk[s] = du[s] * v[s],  dv[s] = du[s] * k[s]
//     dh[G, j] = sum_b sum_{c in G} sum_{t>=j} g[b,t,c] * u[b,t-j,c]
// The filter gradient follows the two-pass scheme of the paper's backward (App. A.4): the main kernel
// accumulates a partial dh per tile next to dq, dk, dv and writes it out contiguously; a second small kernel
// reduces the partials (and the channels of a group).
//
//  * bwd_stencil_kernel: short filters (lh <= 8), one fused streaming pass.  A lane owns VEC adjacent
//    channels and walks one tile forward in time with everything in registers: the last lh-1 values of u
//    (for z), the last lh values of g (du is finished lh-1 steps late, when the newest g it needs has
//    arrived), a delay line of k and v for that lag, and VEC*lh partial sums for dh.  A tile reads lh-1
//    halo rows of k, v before its start and lh-1 halo rows of dy, q after its end.
//  * bwd_direct_kernel / dh_direct_kernel: any lh, any group, both dtypes.  Correctness path.
//
// kGated = false turns both paths into the backward of the featurizer convolutions of Eq. 1 (x' = h * x, no
// gates): u = x (the k pointer), g = dy, the only activation gradient is dx = du (the dk pointer); q, v, dq, dv are
// neither read nor written.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

// ------------------------------------------------------------------------------------- stencil
struct BwdStencilArgs {
    BwdPtrs p;
    float* partial;  // [B * tiles_per_seq][D * LH]
    int64_t L, D;
    int64_t skv, sgq, sout;  // elements between batch items in k, v / dy, q / dq, dk, dv
    int32_t hist, fut;       // rows of k, v in front of row 0 / of dy, q behind row L - 1 that hold data
    int64_t nvec, nitems;
    int32_t group, rows, tiles_per_seq;
};

constexpr int kBlock = 256;

template <typename T, int VEC, int LH, int R, bool kGated>
__global__ __launch_bounds__(kBlock) void bwd_stencil_kernel(BwdStencilArgs a) {
    using P = Pack<T, VEC>;
    using Raw = typename P::Raw;
    constexpr int W = LH - 1 + R;  // window length: LH-1 older steps plus the batch
    const int64_t item = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (item >= a.nitems) return;
    const int64_t cv = item % a.nvec;
    const int64_t tile = item / a.nvec;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t t0 = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t1 = (t0 + a.rows < a.L) ? t0 + a.rows : a.L;
    const int64_t L = a.L, D = a.D;
    const int64_t c = cv * VEC;
    const int64_t seq0 = b * a.sout + c, seq0kv = b * a.skv + c, seq0gq = b * a.sgq + c;
    const char* dyp = static_cast<const char*>(a.p.dy);
    const char* qp = static_cast<const char*>(a.p.q);
    const char* kp = static_cast<const char*>(a.p.k);
    const char* vp = static_cast<const char*>(a.p.v);
    char* dqp = static_cast<char*>(a.p.dq);
    char* dkp = static_cast<char*>(a.p.dk);
    char* dvp = static_cast<char*>(a.p.dv);

    float taps[VEC][LH], dh[VEC][LH];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const float* hp = a.p.h + ((c + e) / a.group) * (int64_t)LH;
#pragma unroll
        for (int j = 0; j < LH; ++j) {
            taps[e][j] = hp[j];
            dh[e][j] = 0.0f;
        }
    }

    // index i of a window = time (first step of the current batch) - (LH-1) + i
    float uw[VEC][W], gw[VEC][W], kd[VEC][W], vd[VEC][W];
#pragma unroll
    for (int i = 0; i < LH - 1; ++i) {
        const int64_t t = t0 - (LH - 1) + i;
        float kf[VEC], vf[VEC];
        if (t >= -(int64_t)a.hist) {
            const int64_t off = (seq0kv + t * D) * T::kBytes;
            P::unpack(P::load(kp + off), kf);
            if constexpr (kGated) {
                P::unpack(P::load(vp + off), vf);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) vf[e] = 1.0f;
            }
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) kf[e] = vf[e] = 0.0f;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            uw[e][i] = kf[e] * vf[e];
            gw[e][i] = 0.0f;
            kd[e][i] = kf[e];
            vd[e][i] = vf[e];
        }
    }

    // the walk covers the tile plus the LH-1 steps after it whose g still reaches into the tile
    const int64_t t_stop = L + a.fut;  // dy and q hold data up to here
    const int64_t t_walk = (t1 + (LH - 1) < t_stop) ? t1 + (LH - 1) : t_stop;
    Raw kr[R], vr[R], qr[R], gr[R];
    auto issue = [&](int64_t t) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            kr[r] = zero_words<P::kWords>();
            vr[r] = zero_words<P::kWords>();
            qr[r] = zero_words<P::kWords>();
            gr[r] = zero_words<P::kWords>();
            if (t + r < t_walk) {
                const int64_t off = (seq0gq + (t + r) * D) * T::kBytes;
                if constexpr (kGated) qr[r] = P::load_nt(qp + off);
                gr[r] = P::load_nt(dyp + off);
                if (t + r < t1) {
                    const int64_t offkv = (seq0kv + (t + r) * D) * T::kBytes;
                    kr[r] = P::load_nt(kp + offkv);
                    if constexpr (kGated) vr[r] = P::load_nt(vp + offkv);
                }
            }
        }
    };

    issue(t0);
    // du of step s is finished when step s + LH - 1 has been seen: run LH-1 steps past the tile end
    for (int64_t t = t0; t < t1 + (LH - 1); t += R) {
        Raw kc[R], vc[R], qc[R], gc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            kc[r] = kr[r];
            vc[r] = vr[r];
            qc[r] = qr[r];
            gc[r] = gr[r];
        }
        if (t + R < t1 + (LH - 1)) issue(t + R);

#pragma unroll
        for (int r = 0; r < R; ++r) {
            float kf[VEC], vf[VEC], qf[VEC], dyf[VEC];
            P::unpack(kc[r], kf);
            P::unpack(gc[r], dyf);
            if constexpr (kGated) {
                P::unpack(vc[r], vf);
                P::unpack(qc[r], qf);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) vf[e] = qf[e] = 1.0f;
            }
            const int64_t tt = t + r;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                uw[e][LH - 1 + r] = kf[e] * vf[e];
                gw[e][LH - 1 + r] = dyf[e] * qf[e];  // zero at and after the end of the sequence (loads skipped)
                kd[e][LH - 1 + r] = kf[e];
                vd[e][LH - 1 + r] = vf[e];
            }
            if (tt < t1) {  // dq and the filter-gradient partials of step tt
                float dqv[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    if constexpr (kGated) {
                        float z = taps[e][0] * uw[e][LH - 1 + r];
#pragma unroll
                        for (int j = 1; j < LH; ++j) z = __builtin_fmaf(taps[e][j], uw[e][LH - 1 + r - j], z);
                        dqv[e] = dyf[e] * z;
                    }
#pragma unroll
                    for (int j = 0; j < LH; ++j) dh[e][j] = __builtin_fmaf(gw[e][LH - 1 + r], uw[e][LH - 1 + r - j], dh[e][j]);
                }
                if constexpr (kGated) P::store_nt(dqp + (seq0 + tt * D) * T::kBytes, P::pack(dqv));
            }
            const int64_t s = tt - (LH - 1);  // the step whose du is complete now; window index r
            if (s >= t0 && s < t1) {
                float dkv[VEC], dvv[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    float du = taps[e][0] * gw[e][r];
#pragma unroll
                    for (int j = 1; j < LH; ++j) du = __builtin_fmaf(taps[e][j], gw[e][r + j], du);
                    dkv[e] = du * vd[e][r];
                    dvv[e] = du * kd[e][r];
                }
                P::store_nt(dkp + (seq0 + s * D) * T::kBytes, P::pack(dkv));
                if constexpr (kGated) P::store_nt(dvp + (seq0 + s * D) * T::kBytes, P::pack(dvv));
            }
        }
#pragma unroll
        for (int i = 0; i < LH - 1; ++i) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                uw[e][i] = uw[e][i + R];
                gw[e][i] = gw[e][i + R];
                kd[e][i] = kd[e][i + R];
                vd[e][i] = vd[e][i + R];
            }
        }
    }

    float* pp = a.partial + tile * (D * LH) + c * LH;
#pragma unroll
    for (int e = 0; e < VEC; ++e)
#pragma unroll
        for (int j = 0; j < LH; ++j) pp[e * LH + j] = dh[e][j];
}

// second pass: dh[g][j] = sum over partial sets and over the channels of group g.  A workgroup owns 64 outputs;
// its four waves each sum a contiguous quarter of the terms (fixed order: set, then channel of the group), wave 0
// adds the four quarters in order.  Deterministic, no atomics.  The sums run in fp64 (the adds are a negligible
// part of this kernel), so the reduction adds no rounding of its own to the fp32 partials.  With few terms per
// output (up to 8: single channels and a handful of tiles) a lane sums all of them for one of 256 outputs instead:
// a quarter of the workgroups, all loads of a lane in flight at once, no exchange.
template <int kRedParts>
__global__ __launch_bounds__(kBlock) void dh_reduce_kernel(const float* __restrict__ partial, float* __restrict__ dh,
                                                           int64_t nsets, int64_t D, int32_t lh, int32_t group) {
    constexpr int kRedOut = kBlock / kRedParts;
    __shared__ double red[kRedParts][kRedOut];
    const int o = threadIdx.x % kRedOut, part = threadIdx.x / kRedOut;
    const int64_t idx = (int64_t)blockIdx.x * kRedOut + o;  // (g, j)
    const int64_t n = (D / group) * lh;
    const int64_t idc = idx < n ? idx : n - 1;  // lanes past the end repeat the last output and do not store
    const int64_t g = idc / lh, j = idc % lh;
    const float* base = partial + (g * group) * lh + j;
    const int64_t total = nsets * group;
    const int64_t per = (total + kRedParts - 1) / kRedParts;
    const int64_t lo = part * per, hi = lo + per < total ? lo + per : total;
    double s = 0.0;
    // term x = set * group + c lives at base[set * D * lh + c * lh]; the offset is advanced term by term (one
    // division per lane instead of two per term).  Eight loads in flight at a time (they do not depend on the
    // running sum); past the end the last offset repeats, so that the loads stay unconditional.
    const int64_t set0 = lo / group;
    int32_t c = (int32_t)(lo - set0 * group);
    int64_t cur = set0 * (D * lh) + (int64_t)c * lh;
    const int64_t wrap = D * lh - (int64_t)(group - 1) * lh;
    for (int64_t x0 = lo; x0 < hi; x0 += 8) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            v[i] = base[cur];
            if (x0 + i + 1 < hi) {
                if (++c == group) {
                    c = 0;
                    cur += wrap;
                } else {
                    cur += lh;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (x0 + i < hi) s += (double)v[i];
    }
    if constexpr (kRedParts == 1) {
        if (idx < n) dh[idx] = (float)s;
        return;
    }
    red[part][o] = s;
    __syncthreads();
    if (part == 0 && idx < n) {
        double t = red[0][o];
#pragma unroll
        for (int r = 1; r < kRedParts; ++r) t += red[r][o];
        dh[idx] = (float)t;
    }
}

// ------------------------------------------------------------------------------------- general
constexpr int kRows = 8;
constexpr int kChan = 64;
constexpr int kRowLanes = 4;

struct BwdDirectArgs {
    BwdPtrs p;
    int64_t B, L, D;
    int64_t skv, sgq, sout;  // elements between batch items in k, v / dy, q / dq, dk, dv
    int32_t hist, fut;       // rows of k, v in front of row 0 / of dy, q behind row L - 1 that hold data
    int32_t lh, group;
};

// dq, dk, dv: one lane = one channel x kRows consecutive steps, sliding along the sources with the kRows
// matching taps in registers (backwards in time for z, forwards for du).
template <typename T, bool kGated>
__global__ __launch_bounds__(kChan* kRowLanes) void bwd_direct_kernel(BwdDirectArgs a) {
    using P = Pack<T, 1>;
    const int64_t b = blockIdx.z;
    const int64_t c = (int64_t)blockIdx.x * kChan + (threadIdx.x % kChan);
    const int64_t tf = ((int64_t)blockIdx.y * kRowLanes + threadIdx.x / kChan) * kRows;
    if (c >= a.D || tf >= a.L) return;
    const int64_t L = a.L;
    const int64_t tl = (tf + kRows - 1 < L - 1) ? tf + kRows - 1 : L - 1;
    const int lh = a.lh;
    const float* hp = a.p.h + (c / a.group) * (int64_t)lh;
    const char* dyp = static_cast<const char*>(a.p.dy);
    const char* qp = static_cast<const char*>(a.p.q);
    const char* kp = static_cast<const char*>(a.p.k);
    const char* vp = static_cast<const char*>(a.p.v);
    const int64_t seq0 = b * a.sout + c, seq0kv = b * a.skv + c, seq0gq = b * a.sgq + c;
    auto ld = [&](const char* base, int64_t s0, int64_t t) {
        float f[1];
        P::unpack(P::load(base + (s0 + t * a.D) * T::kBytes), f);
        return f[0];
    };

    float tw[kRows], acc[kRows], zz[kRows];
    if constexpr (kGated) {
        // z[tf + r] = sum_s h[tf + r - s] u[s], s ascending
        int64_t s = tf - (lh - 1);
        if (s < -(int64_t)a.hist) s = -(int64_t)a.hist;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int64_t j = tf + r - s;
            tw[r] = (j >= 0 && j < lh) ? hp[j] : 0.0f;
            acc[r] = 0.0f;
        }
        for (; s <= tl; ++s) {
            const float u = ld(kp, seq0kv, s) * ld(vp, seq0kv, s);
#pragma unroll
            for (int r = 0; r < kRows; ++r) acc[r] = __builtin_fmaf(tw[r], u, acc[r]);
#pragma unroll
            for (int r = kRows - 1; r > 0; --r) tw[r] = tw[r - 1];
            const int64_t j0 = tf - (s + 1);
            tw[0] = (j0 >= 0 && j0 < lh) ? hp[j0] : 0.0f;
        }
#pragma unroll
        for (int r = 0; r < kRows; ++r) zz[r] = acc[r];
    }

    // du[tf + r] = sum_t h[t - tf - r] g[t], t ascending from tf to tl + lh - 1
    int64_t t = tf;
    int64_t t_last = tl + (lh - 1);
    if (t_last > L + a.fut - 1) t_last = L + a.fut - 1;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t j = t - tf - r;
        tw[r] = (j >= 0 && j < lh) ? hp[j] : 0.0f;
        acc[r] = 0.0f;
    }
    for (; t <= t_last; ++t) {
        const float g = kGated ? ld(dyp, seq0gq, t) * ld(qp, seq0gq, t) : ld(dyp, seq0gq, t);
#pragma unroll
        for (int r = 0; r < kRows; ++r) acc[r] = __builtin_fmaf(tw[r], g, acc[r]);
        // next source: every tap index grows by one
#pragma unroll
        for (int r = kRows - 1; r > 0; --r) tw[r] = tw[r - 1];
        const int64_t j0 = t + 1 - tf;
        tw[0] = (j0 >= 0 && j0 < lh) ? hp[j0] : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (tf + r <= tl) {
            const int64_t off = (seq0 + (tf + r) * a.D) * T::kBytes;
            float o[1];
            if constexpr (kGated) {
                const float kf = ld(kp, seq0kv, tf + r), vf = ld(vp, seq0kv, tf + r), dyf = ld(dyp, seq0gq, tf + r);
                o[0] = dyf * zz[r];
                P::store(static_cast<char*>(a.p.dq) + off, P::pack(o));
                o[0] = acc[r] * vf;
                P::store(static_cast<char*>(a.p.dk) + off, P::pack(o));
                o[0] = acc[r] * kf;
                P::store(static_cast<char*>(a.p.dv) + off, P::pack(o));
            } else {
                o[0] = acc[r];
                P::store(static_cast<char*>(a.p.dk) + off, P::pack(o));
            }
        }
    }
}

// dh[g][j]: one workgroup per (group, tap); lanes stride over (b, t, channel of the group), then a tree sum.
// Products of fp32 factors and their sum are carried in fp64 (correctness path: the sum has B * L * group terms).
template <typename T, bool kGated>
__global__ __launch_bounds__(kBlock) void dh_direct_kernel(BwdDirectArgs a) {
    using P = Pack<T, 1>;
    __shared__ double red[kBlock];
    const int64_t g = blockIdx.x;
    const int64_t j = blockIdx.y;
    const int64_t L = a.L, D = a.D;
    const int group = a.group;
    const char* dyp = static_cast<const char*>(a.p.dy);
    const char* qp = static_cast<const char*>(a.p.q);
    const char* kp = static_cast<const char*>(a.p.k);
    const char* vp = static_cast<const char*>(a.p.v);
    auto ld = [&](const char* base, int64_t e) {
        float f[1];
        P::unpack(P::load(base + e * T::kBytes), f);
        return f[0];
    };
    // this call's share: g of its own steps against u up to `hist` steps before them
    const int64_t t_first = j > a.hist ? j - a.hist : 0;
    const int64_t span = (L - t_first) * group;  // (t, cc) pairs per batch item, channel fastest
    double s = 0.0;
    for (int64_t b = 0; b < a.B; ++b) {
        for (int64_t i = threadIdx.x; i < span; i += kBlock) {
            const int64_t t = t_first + i / group;
            const int64_t c = g * group + i % group;
            const int64_t at = b * a.sgq + t * D + c, src = b * a.skv + (t - j) * D + c;
            if constexpr (kGated)
                s = __builtin_fma((double)ld(dyp, at) * (double)ld(qp, at), (double)ld(kp, src) * (double)ld(vp, src), s);
            else
                s = __builtin_fma((double)ld(dyp, at), (double)ld(kp, src), s);
        }
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) a.p.dh[g * a.lh + j] = (float)red[0];
}

int stencil_rows(const BwdShape& s, int64_t nvec) {
    int rows = tuning().se_rows;
    if (rows <= 0) {
        const int64_t waves_per_row = (nvec + kWave - 1) / kWave;
        // Measured on MI355X (L = 8192, D = 4096): 256-step tiles run 10% faster than 128-step ones (half the
        // halo rows and half the partial filter gradients), as long as four waves per CU are left.
        // The featurizer variant holds half the loads and windows per lane and wants eight waves per CU (same
        // shape: 48.5 us with 128-step tiles, 66 us with 256).
        rows = 256;
        const int64_t want = s.gated ? 1024 : 2048;
        while (rows > 32 && s.B * ((s.L + rows - 1) / rows) * waves_per_row < want) rows >>= 1;
    }
    if (rows > s.L) rows = (int)s.L;
    if (rows < 1) rows = 1;
    return rows;
}

template <typename T>
constexpr int stencil_vec() { return T::kBytes == 2 ? 2 : 1; }

template <typename T, int LH>
hy_status launch_stencil_lh(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    constexpr int VEC = stencil_vec<T>();
    constexpr int R = 4;
    BwdStencilArgs a;
    a.p = p;
    a.partial = static_cast<float*>(ws);
    a.L = s.L;
    a.D = s.D;
    a.skv = s.stride_kv();
    a.sgq = s.stride_gq();
    a.sout = s.stride_out();
    a.hist = s.history;
    a.fut = s.future;
    a.group = s.group;
    a.nvec = s.D / VEC;
    a.rows = stencil_rows(s, a.nvec);
    a.tiles_per_seq = (int32_t)((s.L + a.rows - 1) / a.rows);
    a.nitems = s.B * a.tiles_per_seq * a.nvec;
    const int64_t nb = (a.nitems + kBlock - 1) / kBlock;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    const hy_status rc = s.gated
        ? launch_kernel((bwd_stencil_kernel<T, VEC, LH, R, true>), dim3((uint32_t)nb), dim3(kBlock), st, a)
        : launch_kernel((bwd_stencil_kernel<T, VEC, LH, R, false>), dim3((uint32_t)nb), dim3(kBlock), st, a);
    if (rc != HY_OK) return rc;
    const int64_t nsets = s.B * a.tiles_per_seq;
    return launch_dh_reduce(a.partial, p.dh, nsets, s.D, s.lh, s.group, st);
}

template <typename T>
hy_status launch_stencil_t(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    switch (s.lh) {
        case 1: return launch_stencil_lh<T, 1>(p, s, ws, st);
        case 2: return launch_stencil_lh<T, 2>(p, s, ws, st);
        case 3: return launch_stencil_lh<T, 3>(p, s, ws, st);
        case 4: return launch_stencil_lh<T, 4>(p, s, ws, st);
        case 5: return launch_stencil_lh<T, 5>(p, s, ws, st);
        case 6: return launch_stencil_lh<T, 6>(p, s, ws, st);
        case 7: return launch_stencil_lh<T, 7>(p, s, ws, st);
        case 8: return launch_stencil_lh<T, 8>(p, s, ws, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

template <typename T>
hy_status launch_direct_t(const BwdPtrs& p, const BwdShape& s, hipStream_t st) {
    BwdDirectArgs a;
    a.p = p;
    a.B = s.B; a.L = s.L; a.D = s.D; a.lh = s.lh; a.group = s.group;
    a.skv = s.stride_kv();
    a.sgq = s.stride_gq();
    a.sout = s.stride_out();
    a.hist = s.history;
    a.fut = s.future;
    const int64_t gx = (s.D + kChan - 1) / kChan;
    const int64_t gy = (s.L + kRows * kRowLanes - 1) / (kRows * kRowLanes);
    const int64_t G = s.D / s.group;
    if (gx > 0x7fffffffLL || gy > 65535 || s.B > 65535 || G > 0x7fffffffLL || s.lh > 65535) return HY_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)gx, (uint32_t)gy, (uint32_t)s.B), gridh((uint32_t)G, (uint32_t)s.lh);
    if (s.gated) {
        const hy_status rc = launch_kernel((bwd_direct_kernel<T, true>), grid, dim3(kChan * kRowLanes), st, a);
        if (rc != HY_OK) return rc;
        return launch_kernel((dh_direct_kernel<T, true>), gridh, dim3(kBlock), st, a);
    }
    const hy_status rc = launch_kernel((bwd_direct_kernel<T, false>), grid, dim3(kChan * kRowLanes), st, a);
    if (rc != HY_OK) return rc;
    return launch_kernel((dh_direct_kernel<T, false>), gridh, dim3(kBlock), st, a);
}

}  // namespace

bool bwd_stencil_supported(const BwdShape& s) {
    const int vec = s.dtype == HY_BF16 ? 2 : 1;
    return s.lh <= 8 && s.D % vec == 0;
}

int64_t bwd_stencil_workspace_bytes(const BwdShape& s) {
    const int vec = s.dtype == HY_BF16 ? 2 : 1;
    const int rows = stencil_rows(s, s.D / vec);
    const int64_t tiles = (s.L + rows - 1) / rows;
    return s.B * tiles * s.D * s.lh * (int64_t)sizeof(float);
}

hy_status launch_bwd_stencil(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    if (!bwd_stencil_supported(s)) return HY_ERR_UNSUPPORTED;
    return s.dtype == HY_BF16 ? launch_stencil_t<BF16>(p, s, ws, st) : launch_stencil_t<F32>(p, s, ws, st);
}

hy_status launch_dh_reduce(const float* partial, float* dh, int64_t nsets, int64_t n_rows, int32_t lh, int32_t group,
                           hipStream_t st) {
    const int64_t nout = (n_rows / group) * lh;
    if (nout == 0) return HY_OK;
    if (nsets * group <= 8)
        return launch_kernel(dh_reduce_kernel<1>, dim3((uint32_t)((nout + kBlock - 1) / kBlock)), dim3(kBlock), st, partial,
                             dh, nsets, n_rows, lh, group);
    return launch_kernel(dh_reduce_kernel<4>, dim3((uint32_t)((nout + kBlock / 4 - 1) / (kBlock / 4))), dim3(kBlock), st,
                         partial, dh, nsets, n_rows, lh, group);
}

hy_status launch_bwd_zero_dh(float* dh, int64_t D, int32_t lh, int32_t group, hipStream_t st) {
    const int64_t nout = (D / group) * lh;
    if (nout == 0) return HY_OK;
    // a reduction over zero partial sets writes zeros (a fill kernel, not a memset, so that callers may
    // capture the call in a HIP graph)
    return launch_kernel(dh_reduce_kernel<1>, dim3((uint32_t)((nout + kBlock - 1) / kBlock)), dim3(kBlock), st,
                         static_cast<const float*>(dh), dh, (int64_t)0, D, lh, group);
}

hy_status launch_bwd_direct(const BwdPtrs& p, const BwdShape& s, hipStream_t st) {
    return s.dtype == HY_BF16 ? launch_direct_t<BF16>(p, s, st) : launch_direct_t<F32>(p, s, st);
}

}  // namespace hy
