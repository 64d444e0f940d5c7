// General forward kernel: direct causal FIR convolution with optional gating for any filter length and
// any group size, fp32 arithmetic on the vector ALUs.  It is the fallback behind every entry point for
// shapes the specialised kernels do not cover (fp32 Hyena-MR, group sizes that do not tile the matrix
// cores, filters longer than the specialised limits).  One lane = one channel x kRows consecutive
// outputs; it slides along the source samples keeping the kRows taps that meet them in registers, so
// each source sample and each tap is loaded once per lane.  Loads are coalesced over channels.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

constexpr int kRows = 8;
constexpr int kChan = 64;
constexpr int kRowLanes = 4;  // block = kChan x kRowLanes lanes, covers kChan channels x 32 rows

struct DirectArgs {
    ConvPtrs p[3];
    int64_t B, L, D;
    int64_t bstride_kv, bstride_qy;  // elements between batch items in k, v / in q, y
    int32_t hist;     // rows of k (and v) in front of row 0 that hold data
    int32_t lh, group;
};

template <typename T, bool GATED>
__global__ __launch_bounds__(kChan* kRowLanes) void direct_kernel(DirectArgs a) {
    using P = Pack<T, 1>;
    const int prob = blockIdx.z / (int)a.B;
    const int64_t b = blockIdx.z % (int)a.B;
    const ConvPtrs pr = a.p[prob];
    const int64_t c = (int64_t)blockIdx.x * kChan + (threadIdx.x % kChan);
    const int64_t tf = ((int64_t)blockIdx.y * kRowLanes + threadIdx.x / kChan) * kRows;  // first output row
    if (c >= a.D || tf >= a.L) return;
    const int64_t tl = (tf + kRows - 1 < a.L - 1) ? tf + kRows - 1 : a.L - 1;  // last output row
    const int lh = a.lh;
    const float* hp = pr.h + (c / a.group) * (int64_t)lh;
    const char* kp = static_cast<const char*>(pr.k);
    const char* vp = static_cast<const char*>(pr.v);
    const int64_t seq0 = b * a.bstride_qy + c, seq0kv = b * a.bstride_kv + c;

    int64_t s = tf - (lh - 1);
    if (s < -(int64_t)a.hist) s = -(int64_t)a.hist;
    // tw[r] = tap that links output row tf + r with source s: index (tf + r - s), zero outside [0, lh)
    float tw[kRows], acc[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t j = tf + r - s;
        tw[r] = (j >= 0 && j < lh) ? hp[j] : 0.0f;
        acc[r] = 0.0f;
    }
    for (; s <= tl; ++s) {
        const int64_t off = (seq0kv + s * a.D) * T::kBytes;
        float kf[1], vf[1];
        P::unpack(P::load(kp + off), kf);
        float u = kf[0];
        if constexpr (GATED) {
            P::unpack(P::load(vp + off), vf);
            u *= vf[0];
        }
#pragma unroll
        for (int r = 0; r < kRows; ++r) acc[r] = __builtin_fmaf(tw[r], u, acc[r]);
        // next source: every tap index drops by one
#pragma unroll
        for (int r = kRows - 1; r > 0; --r) tw[r] = tw[r - 1];
        const int64_t j0 = tf - (s + 1);
        tw[0] = (j0 >= 0 && j0 < lh) ? hp[j0] : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (tf + r <= tl) {
            const int64_t off = (seq0 + (tf + r) * a.D) * T::kBytes;
            float z[1] = {acc[r]};
            if constexpr (GATED) {
                float qf[1];
                P::unpack(P::load(static_cast<const char*>(pr.q) + off), qf);
                z[0] *= qf[0];
            }
            P::store(static_cast<char*>(pr.y) + off, P::pack(z));
        }
    }
}

template <typename T, bool GATED>
hy_status launch_t(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    DirectArgs a;
    for (int i = 0; i < 3; ++i) a.p[i] = p[i < nprob ? i : 0];
    a.B = s.B; a.L = s.L; a.D = s.D; a.lh = s.lh; a.group = s.group;
    a.bstride_kv = s.stride_kv();
    a.bstride_qy = s.stride_qy();
    a.hist = s.history;
    const int64_t gx = (s.D + kChan - 1) / kChan;
    const int64_t gy = (s.L + kRows * kRowLanes - 1) / (kRows * kRowLanes);
    const int64_t gz = s.B * nprob;
    if (gx > 0x7fffffffLL || gy > 65535 || gz > 65535) return HY_ERR_UNSUPPORTED;
    return launch_kernel((direct_kernel<T, GATED>), dim3((uint32_t)gx, (uint32_t)gy, (uint32_t)gz),
                       dim3(kChan * kRowLanes), st, a);
}

}  // namespace

hy_status launch_direct(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    if (s.dtype == HY_BF16)
        return s.gated ? launch_t<BF16, true>(p, nprob, s, st) : launch_t<BF16, false>(p, nprob, s, st);
    return s.gated ? launch_t<F32, true>(p, nprob, s, st) : launch_t<F32, false>(p, nprob, s, st);
}

}  // namespace hy
