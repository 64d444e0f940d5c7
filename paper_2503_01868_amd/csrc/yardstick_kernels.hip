// Bandwidth yardsticks: the operator's memory traffic with its arithmetic taken out.
//
//   y[t, c] = q[t, c] * k[t, c] * v[t, c]        (bf16 in, bf16 out; fp32 products, one rounding)
//
// i.e. the gated convolution with a one-tap unit filter: three tensors read once, one written once, 8 bytes per
// output like the real kernels, non-temporal loads and stores like theirs.  Two access patterns:
//   * linear: every lane takes 16-byte words at a workgroup-wide stride, the launch shape of hyena_stream_copy;
//   * strips: a workgroup of NW waves owns `strip` adjacent channels and `rows` time steps and walks down time in
//     chunks of 512 NW / strip rows (32 with strip = 16 NW, the operator kernels' shape), every lane loading one
//     16-byte piece of k, v, q per chunk `depth` chunks ahead (two in the operator kernels) with clamped
//     addresses, one workgroup barrier per chunk: the data movement of the matrix-core kernels (mr_kernels.hip and
//     its relatives), which read a [time][channel] tensor through column strips of 128, 256 or 512 bytes per row.
//     Fewer waves than strip / 16 make shorter chunks; with more chunks in flight per lane the bytes in flight per
//     compute unit stay the same (512-byte strips: 16 waves x 2 chunks, 8 x 4 and 4 x 8 all hold 96 KB).  The barrier is part of the pattern: it keeps the waves of a
//     workgroup on the same chunk, so that the workgroup asks for whole row pieces at a time; without it the waves
//     drift apart and 512-byte strips fall from 6.1 to 5.3 TB/s (MI355X, L = 131072, D = 4096).
// Measured against each other they give the practical ceilings the operator kernels are judged by: what a
// compute-free 3-read/1-write stream reaches on this machine, and what each strip width costs.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

__device__ __forceinline__ Words<4> gate3(const Words<4>& q, const Words<4>& k, const Words<4>& v) {
    float qf[8], kf[8], vf[8], y[8];
    Pack<BF16, 8>::unpack(q, qf);
    Pack<BF16, 8>::unpack(k, kf);
    Pack<BF16, 8>::unpack(v, vf);
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = qf[e] * (kf[e] * vf[e]);
    return Pack<BF16, 8>::pack(y);
}

constexpr int kLinBlock = 256;
constexpr int kLinPerLane = 4;  // 16-byte words per lane and tensor

__global__ __launch_bounds__(kLinBlock) void gate_linear_kernel(const uint4* __restrict__ q, const uint4* __restrict__ k,
                                                                const uint4* __restrict__ v, uint4* __restrict__ y,
                                                                int64_t n16) {
    const int64_t base = (int64_t)blockIdx.x * (kLinBlock * kLinPerLane) + threadIdx.x;
    Words<4> qr[kLinPerLane], kr[kLinPerLane], vr[kLinPerLane];
#pragma unroll
    for (int i = 0; i < kLinPerLane; ++i) {
        int64_t idx = base + (int64_t)i * kLinBlock;
        idx = idx < n16 ? idx : n16 - 1;  // clamped, unconditional loads
        kr[i] = load_words_nt<4>(k + idx);
        vr[i] = load_words_nt<4>(v + idx);
        qr[i] = load_words_nt<4>(q + idx);
    }
#pragma unroll
    for (int i = 0; i < kLinPerLane; ++i) {
        const int64_t idx = base + (int64_t)i * kLinBlock;
        if (idx < n16) store_words_nt<4>(y + idx, gate3(qr[i], kr[i], vr[i]));
    }
}

struct StripArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* y;
    int64_t L, D;
    int32_t rows;           // time steps per workgroup, multiple of 32
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / strip
};

// NW waves, PPR 16-byte pieces per row piece of the strip (strip = 8 PPR channels), kPrefetch chunks in flight
template <int NW, int PPR, int kPrefetch>
__global__ __launch_bounds__(NW * 64) void gate_strip_kernel(StripArgs a) {
    constexpr int kChunk = NW * 64 / PPR;  // rows per chunk
    const int tid = threadIdx.x;
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;  // channel block fastest, as in the operator kernels
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t t_start = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t_end = (t_start + a.rows < a.L) ? t_start + a.rows : a.L;
    const int nchunks = (int)((t_end - t_start + kChunk - 1) / kChunk);
    const int64_t D = a.D;
    const int64_t seq0 = b * a.L * D;
    const int lr = tid / PPR, lp = tid % PPR;
    const int64_t ld_off = (int64_t)cb * 8 * PPR + 8 * lp;

    // chunk indices past the last chunk load one 16-byte location for the whole workgroup, as in the operator kernels
    const int64_t idle_off = (t_end - 1) * D + (int64_t)cb * 8 * PPR;
    auto off_of = [&](int ci) {
        int64_t t = t_start + (int64_t)ci * kChunk + lr;
        t = t < t_end ? t : t_end - 1;
        return seq0 + (ci < nchunks ? t * D + ld_off : idle_off);
    };
    Words<4> qpre[kPrefetch], kpre[kPrefetch], vpre[kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) {
        const int64_t off = off_of(i);
        kpre[i] = load_words_nt<4>(a.k + off);
        vpre[i] = load_words_nt<4>(a.v + off);
        qpre[i] = load_words_nt<4>(a.q + off);
    }
    for (int base = 0; base < nchunks; base += kPrefetch) {
#pragma unroll
        for (int sgi = 0; sgi < kPrefetch; ++sgi) {
            const int ci = base + sgi;
            const Words<4> out = gate3(qpre[sgi], kpre[sgi], vpre[sgi]);
            const int64_t nxt = off_of(ci + kPrefetch);
            kpre[sgi] = load_words_nt<4>(a.k + nxt);
            vpre[sgi] = load_words_nt<4>(a.v + nxt);
            qpre[sgi] = load_words_nt<4>(a.q + nxt);
            __syncthreads();  // the operator kernels' one barrier per chunk (see the note at the top)
            const int64_t t = t_start + (int64_t)ci * kChunk + lr;
            if (ci < nchunks && t < t_end) store_words_nt<4>(a.y + seq0 + t * D + ld_off, out);
        }
    }
}

template <int NW, int PPR, int PF>
hy_status launch_strip_nw(const void* q, const void* k, const void* v, void* y, int64_t B, int64_t L, int64_t D,
                          int64_t rows, hipStream_t st) {
    constexpr int kChunk = NW * 64 / PPR;
    StripArgs a;
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.y = static_cast<uint16_t*>(y);
    a.L = L;
    a.D = D;
    a.ncb = (int32_t)(D / (8 * PPR));
    if (rows <= 0) {
        int64_t tiles = 256 / (B * a.ncb);  // one workgroup per compute unit, like the operator kernels
        if (tiles < 1) tiles = 1;
        rows = (L + tiles - 1) / tiles;
        if (rows < 128) rows = 128;
    }
    rows = (rows + kChunk - 1) / kChunk * kChunk;
    const int64_t cap = (L + kChunk - 1) / kChunk * kChunk;
    if (rows > cap) rows = cap;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((L + rows - 1) / rows);
    const int64_t nb = B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel((gate_strip_kernel<NW, PPR, PF>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
}

template <int NW, int PPR>
hy_status launch_strip_depth(const void* q, const void* k, const void* v, void* y, int64_t B, int64_t L, int64_t D,
                             int64_t rows, int32_t depth, hipStream_t st) {
    switch (depth) {
        case 0:
        case 2: return launch_strip_nw<NW, PPR, 2>(q, k, v, y, B, L, D, rows, st);
        case 1: return launch_strip_nw<NW, PPR, 1>(q, k, v, y, B, L, D, rows, st);
        case 3: return launch_strip_nw<NW, PPR, 3>(q, k, v, y, B, L, D, rows, st);
        case 4: return launch_strip_nw<NW, PPR, 4>(q, k, v, y, B, L, D, rows, st);
        case 6: return launch_strip_nw<NW, PPR, 6>(q, k, v, y, B, L, D, rows, st);
        case 8: return launch_strip_nw<NW, PPR, 8>(q, k, v, y, B, L, D, rows, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace

hy_status launch_stream_gate(const void* q, const void* k, const void* v, void* y, int64_t B, int64_t L, int64_t D,
                             int32_t strip, int64_t rows, int32_t depth, int32_t waves, hipStream_t st) {
    if (strip == 0) {
        const int64_t n16 = B * L * D / 8;
        const int64_t per_block = kLinBlock * kLinPerLane;
        const int64_t nb = (n16 + per_block - 1) / per_block;
        if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
        return launch_kernel(gate_linear_kernel, dim3((uint32_t)nb), dim3(kLinBlock), st, static_cast<const uint4*>(q),
                             static_cast<const uint4*>(k), static_cast<const uint4*>(v), static_cast<uint4*>(y), n16);
    }
    if (L > 0x7fff0000LL) return HY_ERR_UNSUPPORTED;
    if (waves == 0) waves = strip / 16;
    switch (strip * 100 + waves) {
        case 6404: return launch_strip_depth<4, 8>(q, k, v, y, B, L, D, rows, depth, st);
        case 12808: return launch_strip_depth<8, 16>(q, k, v, y, B, L, D, rows, depth, st);
        case 12804: return launch_strip_depth<4, 16>(q, k, v, y, B, L, D, rows, depth, st);
        case 25616: return launch_strip_depth<16, 32>(q, k, v, y, B, L, D, rows, depth, st);
        case 25608: return launch_strip_depth<8, 32>(q, k, v, y, B, L, D, rows, depth, st);
        case 25604: return launch_strip_depth<4, 32>(q, k, v, y, B, L, D, rows, depth, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
