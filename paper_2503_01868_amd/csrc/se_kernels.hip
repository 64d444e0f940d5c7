// Hyena-SE / featurizer forward: fused streaming stencil for short filters (gfx950, vector ALUs).
//
// Each lane owns VEC adjacent channels and walks down `rows` time steps of one batch item.  The taps of
// its channels and the last LH-1 values of u = k*v sit in registers, so every input element is loaded
// exactly once per tile plus LH-1 halo rows of k and v at the tile start.  A wave covers 64*VEC
// adjacent channels of a row: every load and store is one contiguous, fully used segment.  Workgroups
// take tiles in launch order with the channel strip fastest, so the chip sweeps each tile row of the
// tensor left to right; loads and stores of the bulk rows carry the non-temporal hint.
// Arithmetic: fp32 multiply for the pre-gate, fp32 FMA chain over taps in ascending tap order, fp32
// multiply for the post-gate, one rounding to the storage type at the store.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

struct StencilArgs {
    ConvPtrs p[3];
    int64_t L, D;
    int64_t bstride_kv, bstride_qy;  // elements between batch items in k, v / in q, y
    int32_t hist;     // rows of k (and v) in front of row 0 that hold data
    int64_t nvec;    // D / VEC
    int64_t nitems;  // B * tiles_per_seq * nvec lanes of work
    int32_t group;
    int32_t rows;           // time steps per lane
    int32_t tiles_per_seq;  // ceil(L / rows)
    uint32_t nblocks;
};

constexpr int kStencilBlock = 256;

template <typename T, int VEC, int LH, int R, bool GATED>
__global__ __launch_bounds__(kStencilBlock) void stencil_kernel(StencilArgs a) {
    using P = Pack<T, VEC>;
    using Raw = typename P::Raw;
    const ConvPtrs pr = a.p[blockIdx.y];
    const int64_t item = (int64_t)blockIdx.x * kStencilBlock + threadIdx.x;
    if (item >= a.nitems) return;
    const int64_t cv = item % a.nvec;
    const int64_t tile = item / a.nvec;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t t0 = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t1 = (t0 + a.rows < a.L) ? t0 + a.rows : a.L;
    const int64_t c = cv * VEC;
    const int64_t D = a.D;

    const char* kp = static_cast<const char*>(pr.k);
    const char* vp = static_cast<const char*>(pr.v);
    const char* qp = static_cast<const char*>(pr.q);
    char* yp = static_cast<char*>(pr.y);
    const int64_t seq0 = b * a.bstride_qy + c;    // element offset of (b, 0, c) in q and y
    const int64_t seq0kv = b * a.bstride_kv + c;  // and in k and v

    // taps of this lane's channels
    float taps[VEC][LH];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const float* hp = pr.h + ((c + e) / a.group) * (int64_t)LH;
#pragma unroll
        for (int j = 0; j < LH; ++j) taps[e][j] = hp[j];
    }

    // win[e][i]: u at time (first row of the current batch) - (LH-1) + i
    float win[VEC][LH - 1 + R];
#pragma unroll
    for (int i = 0; i < LH - 1; ++i) {
        const int64_t t = t0 - (LH - 1) + i;
        float kf[VEC], vf[VEC];
        if (t >= -(int64_t)a.hist) {
            const int64_t off = (seq0kv + t * D) * T::kBytes;
            P::unpack(P::load(kp + off), kf);
            if constexpr (GATED) P::unpack(P::load(vp + off), vf);
#pragma unroll
            for (int e = 0; e < VEC; ++e) win[e][i] = GATED ? kf[e] * vf[e] : kf[e];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) win[e][i] = 0.0f;
        }
    }

    Raw kr[R], vr[R], qr[R];
    auto issue = [&](int64_t t) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (t + r < t1) {
                const int64_t off = (seq0kv + (t + r) * D) * T::kBytes;
                kr[r] = P::load_nt(kp + off);
                if constexpr (GATED) {
                    vr[r] = P::load_nt(vp + off);
                    qr[r] = P::load_nt(qp + (seq0 + (t + r) * D) * T::kBytes);
                }
            } else {
                kr[r] = zero_words<P::kWords>();
                if constexpr (GATED) {
                    vr[r] = zero_words<P::kWords>();
                    qr[r] = zero_words<P::kWords>();
                }
            }
        }
    };

    issue(t0);
    for (int64_t t = t0; t < t1; t += R) {
        Raw kc[R], vc[R], qc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            kc[r] = kr[r];
            if constexpr (GATED) {
                vc[r] = vr[r];
                qc[r] = qr[r];
            }
        }
        if (t + R < t1) issue(t + R);  // next batch is in flight while this one is computed

#pragma unroll
        for (int r = 0; r < R; ++r) {
            float kf[VEC], vf[VEC];
            P::unpack(kc[r], kf);
            if constexpr (GATED) P::unpack(vc[r], vf);
#pragma unroll
            for (int e = 0; e < VEC; ++e) win[e][LH - 1 + r] = GATED ? kf[e] * vf[e] : kf[e];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (t + r < t1) {
                float z[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    float acc = taps[e][0] * win[e][LH - 1 + r];
#pragma unroll
                    for (int j = 1; j < LH; ++j) acc = __builtin_fmaf(taps[e][j], win[e][LH - 1 + r - j], acc);
                    z[e] = acc;
                }
                if constexpr (GATED) {
                    float qf[VEC];
                    P::unpack(qc[r], qf);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) z[e] *= qf[e];
                }
                P::store_nt(yp + (seq0 + (t + r) * D) * T::kBytes, P::pack(z));
            }
        }
#pragma unroll
        for (int i = 0; i < LH - 1; ++i) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) win[e][i] = win[e][i + R];
        }
    }
}

template <typename T, int VEC, int LH, bool GATED>
hy_status launch_one(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    constexpr int R = 8;  // rows in flight per lane while the previous batch is computed
    StencilArgs a;
    for (int i = 0; i < 3; ++i) a.p[i] = p[i < nprob ? i : 0];
    a.L = s.L;
    a.D = s.D;
    a.bstride_kv = s.stride_kv();
    a.bstride_qy = s.stride_qy();
    a.hist = s.history;
    a.group = s.group;
    a.nvec = s.D / VEC;
    int rows = tuning().se_rows;
    if (rows <= 0) {
        // Tile length in t: 128 steps (halo re-reads 2.3% at lh = 7) when that still leaves about 8 waves
        // per CU, shorter powers of two for small problems.  Powers of two keep the spacing of the
        // concurrently walked tiles a power of two in memory, which measured best on MI355X.
        const int64_t waves_per_row = (a.nvec * nprob + kWave - 1) / kWave;
        rows = 128;
        while (rows > 32 && s.B * ((s.L + rows - 1) / rows) * waves_per_row < 2048) rows >>= 1;
    }
    if (rows > s.L) rows = (int)s.L;
    if (rows < 1) rows = 1;
    a.rows = rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    a.nitems = s.B * a.tiles_per_seq * a.nvec;
    const int64_t nb = (a.nitems + kStencilBlock - 1) / kStencilBlock;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    a.nblocks = (uint32_t)nb;
    return launch_kernel((stencil_kernel<T, VEC, LH, R, GATED>), dim3(a.nblocks, nprob), dim3(kStencilBlock), st, a);
}

template <typename T, int VEC, bool GATED>
hy_status by_lh(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    switch (s.lh) {
        case 1: return launch_one<T, VEC, 1, GATED>(p, nprob, s, st);
        case 2: return launch_one<T, VEC, 2, GATED>(p, nprob, s, st);
        case 3: return launch_one<T, VEC, 3, GATED>(p, nprob, s, st);
        case 4: return launch_one<T, VEC, 4, GATED>(p, nprob, s, st);
        case 5: return launch_one<T, VEC, 5, GATED>(p, nprob, s, st);
        case 6: return launch_one<T, VEC, 6, GATED>(p, nprob, s, st);
        case 7: return launch_one<T, VEC, 7, GATED>(p, nprob, s, st);
        case 8: return launch_one<T, VEC, 8, GATED>(p, nprob, s, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

template <typename T, bool GATED>
hy_status by_vec(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    constexpr int kMaxVec = 16 / T::kBytes;
    // 4 bytes per lane: narrow strips give the most waves per tile row; measured fastest for bf16 at D = 4096
    int vec = tuning().se_vec > 0 ? tuning().se_vec : (T::kBytes == 2 ? 2 : 1);
    if (vec > kMaxVec) vec = kMaxVec;
    while (vec > 1 && s.D % vec != 0) vec >>= 1;
    if constexpr (T::kBytes == 2) {
        if (vec == 8) return by_lh<T, 8, GATED>(p, nprob, s, st);
    }
    if (vec == 4) return by_lh<T, 4, GATED>(p, nprob, s, st);
    if (vec == 2) return by_lh<T, 2, GATED>(p, nprob, s, st);
    return by_lh<T, 1, GATED>(p, nprob, s, st);
}

}  // namespace

hy_status launch_stencil(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    if (s.lh > 8) return HY_ERR_UNSUPPORTED;
    if (s.dtype == HY_BF16)
        return s.gated ? by_vec<BF16, true>(p, nprob, s, st) : by_vec<BF16, false>(p, nprob, s, st);
    return s.gated ? by_vec<F32, true>(p, nprob, s, st) : by_vec<F32, false>(p, nprob, s, st);
}

}  // namespace hy
