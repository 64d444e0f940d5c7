// Fused Hyena-MR operator chain, forward (Sec. 2.1 Eq. 1 without the dense projections):
//     q' = hq * q,  k' = hk * k,  v' = hv * v          short per-channel featurizer convolutions
//     y  = q' (.) ( h * (k' (.) v') )                  grouped medium convolution with both gates
// in ONE pass over q, k, v: the three featurized tensors never touch HBM (4 instead of 10 tensor passes),
// and they stay in fp32 until the single bf16 rounding of u = k'v' that feeds the matrix cores.
//
// The medium convolution is the block-Toeplitz MFMA scheme of mr_kernels.hip (same operand mapping, same
// register-resident Toeplitz operands and source window).  Around it, per 32-step chunk, a workgroup of
// 8 waves (128 channels) runs two phases separated by two barriers:
//   phase 1  (a) lanes in "row" layout (one row, 8 channels) move the prefetched raw q, k, v of the NEXT chunk
//                from registers into a 3-chunk LDS ring;
//            (b) lanes in "column" layout (2 channels x 4 consecutive steps; taps of those channels in
//                registers) post-gate and store the PREVIOUS chunk: y = q' * z, z read from LDS;
//            (c) the same lanes featurize THIS chunk out of the ring (lf-1 steps of lookback come from the
//                previous chunk's slot), write u = k'v' as bf16 to the LDS source stage and keep q' in
//                registers for (b) of the next iteration;
//   phase 2  every wave reads its group's 32 x 16 block of u transposed, updates its register window,
//            issues the MFMAs and parks z (fp32) in LDS.
// Raw loads are whole 256-byte row pieces, 16 B per lane, prefetched several chunks ahead in registers
// with clamped addresses and no control flow around them.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

struct ChainArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* hq;
    const float* hk;
    const float* hv;
    const float* h;
    uint16_t* y;
    int64_t L, D;
    int32_t lh, group, feat_group;
    int32_t rows;           // time steps per workgroup, multiple of 32
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / 128
};

constexpr int kChunk = 32;
constexpr int kRing = 3;   // chunk slots of raw q, k, v kept in LDS
constexpr int kLook = 8;   // look-back rows stored in front of every slot (>= lf - 1)
constexpr int kSlotRows = kLook + kChunk;
constexpr int kSeg = 4;   // steps per column-layout lane: 8 segments per chunk

// kNW = waves per workgroup = 16-channel groups per workgroup (4 or 8)
template <int NKB, int LF, int PF, int kNW>
__global__ __launch_bounds__(kNW * 64, 2) void chain_mfma_kernel(ChainArgs a) {
    constexpr int kPPR = 2 * kNW;              // 16-byte pieces per row piece
    constexpr int kZRow = 16 * kNW * 4 + 16;   // bytes per staged row of z, padded
    constexpr int kPairs = 8 * kNW;            // channel pairs per workgroup
    constexpr int kTaps = 32 * NKB;
    static_assert(kSeg == 4 && LF >= 1 && LF - 1 <= kLook, "column lanes own 4 steps and look back at most 7");
    __shared__ uint4 raw[3][kRing * kSlotRows * kPPR];  // [tensor k,v,q][slot][look-back rows, chunk rows][piece]
    __shared__ uint4 ust[kChunk * kPPR];
    __shared__ __attribute__((aligned(16))) char zst[kChunk * kZRow];
    __shared__ float hs[kNW][kTaps];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const int li = lane % 16, lq = lane / 16;

    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t t_start = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t_end = (t_start + a.rows < a.L) ? t_start + a.rows : a.L;
    int64_t t_begin = t_start - (int64_t)kChunk * (NKB - 1);
    if (t_begin < 0) t_begin = 0;
    // chunk j covers steps tb(j) = t_begin + 32 (j - 1) ...; chunk 0 is the look-back chunk before the tile
    const int nch = (int)((t_end - t_begin + kChunk - 1) / kChunk);  // real chunks are j = 1 .. nch

    const int64_t D = a.D;
    const int64_t cblock0 = (int64_t)cb * 16 * kNW;
    const int64_t c0 = cblock0 + 16 * w;
    const int64_t seq0 = b * a.L * D;

    // ---- row layout: row lr of a chunk, 16-byte piece lp
    const int lr = tid / kPPR, lp = tid % kPPR;
    const int64_t ld_off = cblock0 + 8 * lp;
    const int64_t lo_kv = (t_begin - 8 > 0) ? t_begin - 8 : 0;  // oldest k, v step ever read
    const int64_t lo_q = (t_start - 8 > 0) ? t_start - 8 : 0;   // oldest q step ever read
    const uint32_t lane_off = (uint32_t)lr * (uint32_t)D + (uint32_t)(8 * lp);  // within a chunk, in elements
    auto load_raw = [&](int j, Words<4>& kk, Words<4>& vv, Words<4>& qq) {
        const int jc = j <= nch ? j : nch;
        const int64_t tb = t_begin + (int64_t)(jc - 1) * kChunk;
        // Only the addresses depend on the (uniform) case; the three loads themselves are unconditional.
        int64_t ok_, oq_;
        if (tb >= lo_kv && tb >= lo_q && tb + kChunk <= t_end) {
            // interior chunk: one scalar base plus a fixed per-lane offset
            ok_ = oq_ = seq0 + tb * D + cblock0 + lane_off;
        } else {
            int64_t t = tb + lr;
            t = t < t_end ? t : t_end - 1;
            ok_ = seq0 + (t > lo_kv ? t : lo_kv) * D + ld_off;
            oq_ = seq0 + (t > lo_q ? t : lo_q) * D + ld_off;
        }
        kk = load_words_nt<4>(a.k + ok_);
        vv = load_words_nt<4>(a.v + ok_);
        qq = load_words_nt<4>(a.q + oq_);
    };
    // Ring slot j % 3 holds chunk j behind kLook look-back rows (the last rows of chunk j - 1), so a featurizer
    // window never straddles slots.  The writer of a chunk therefore also drops its last kLook rows into the
    // look-back area of the next slot.  Steps before the start of the sequence are zeros (zero left padding
    // of every batch item).
    auto ring_write = [&](int j, const Words<4>& kk, const Words<4>& vv, const Words<4>& qq) {
        const int64_t t = t_begin + (int64_t)(j - 1) * kChunk + lr;
        const bool pad = t < 0;  // only ever true in chunk 0 of a tile that starts the sequence
        const uint4 k4 = pad ? make_uint4(0, 0, 0, 0) : make_uint4(kk.w[0], kk.w[1], kk.w[2], kk.w[3]);
        const uint4 v4 = pad ? make_uint4(0, 0, 0, 0) : make_uint4(vv.w[0], vv.w[1], vv.w[2], vv.w[3]);
        const uint4 q4 = pad ? make_uint4(0, 0, 0, 0) : make_uint4(qq.w[0], qq.w[1], qq.w[2], qq.w[3]);
        const int slot = __builtin_amdgcn_readfirstlane(j % kRing);
        const int idx = (slot * kSlotRows + kLook + lr) * kPPR + lp;
        raw[0][idx] = k4;
        raw[1][idx] = v4;
        raw[2][idx] = q4;
        if (lr >= kChunk - kLook) {  // whole waves
            const int nslot = slot == kRing - 1 ? 0 : slot + 1;
            const int nidx = (nslot * kSlotRows + lr - (kChunk - kLook)) * kPPR + lp;
            raw[0][nidx] = k4;
            raw[1][nidx] = v4;
            raw[2][nidx] = q4;
        }
    };

    Words<4> kpre[PF], vpre[PF], qpre[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) load_raw(i, kpre[i], vpre[i], qpre[i]);

    // ---- column layout: channels cblock0 + 2 cp, +1; steps 4 seg .. 4 seg + 3 of a chunk
    const int cp = tid % kPairs, seg = tid / kPairs;
    float tk_[2][LF], tv_[2][LF], tq_[2][LF];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int64_t f = ((cblock0 + 2 * cp + e) / a.feat_group) * (int64_t)LF;
#pragma unroll
        for (int i = 0; i < LF; ++i) {
            tk_[e][i] = a.hk[f + i];
            tv_[e][i] = a.hv[f + i];
            tq_[e][i] = a.hq[f + i];
        }
    }

    // ---- Toeplitz operands of this wave's group (see mr_kernels.hip)
    bf16x8_t tz[2 * NKB];
    {
        const float* hp = a.h + (c0 / a.group) * (int64_t)a.lh;
        for (int j = lane; j < kTaps; j += 64) hs[w][j] = (j < a.lh) ? hp[j] : 0.0f;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2 * NKB; ++i) {
            Words<4> wds;
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const int i0 = 16 * i + li - 8 * lq - 2 * e2;
                const int i1 = i0 - 1;
                const float f0 = (i0 >= 0 && i0 < kTaps) ? hs[w][i0] : 0.0f;
                const float f1 = (i1 >= 0 && i1 < kTaps) ? hs[w][i1] : 0.0f;
                wds.w[e2] = pack_bf16x2(f0, f1);
            }
            tz[i] = __builtin_bit_cast(bf16x8_t, wds);
        }
    }
    bf16x8_t uw[NKB];
    {
        Words<4> z = zero_words<4>();
#pragma unroll
        for (int m = 0; m < NKB; ++m) uw[m] = __builtin_bit_cast(bf16x8_t, z);
    }

    const int rd_piece = (2 * w + (li >> 3)) ^ (lq << 1);
    const int zwr_off = li * kZRow + (16 * w + 4 * lq) * 4;

    // One featurizer output set: x'[e][r] for channels e = 0, 1 and steps r = 0..3 of this lane, from the ring.
    auto featurize = [&](int tensor, int j, const float (&taps)[2][LF], float (&out)[2][4]) {
        const uint32_t* r32 = reinterpret_cast<const uint32_t*>(raw[tensor]);
        const int slot = __builtin_amdgcn_readfirstlane(j % kRing);
        const uint32_t* rp = r32 + (slot * kSlotRows + kLook + kSeg * seg - (LF - 1)) * (kPPR * 4) + cp;
        float win[2][LF - 1 + kSeg];
#pragma unroll
        for (int i = 0; i < LF - 1 + kSeg; ++i) {
            const uint32_t pr = rp[i * (kPPR * 4)];
            win[0][i] = bf16_lo(pr);
            win[1][i] = bf16_hi(pr);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int r = 0; r < kSeg; ++r) {
                float acc = taps[e][0] * win[e][LF - 1 + r];
#pragma unroll
                for (int i = 1; i < LF; ++i) acc = __builtin_fmaf(taps[e][i], win[e][LF - 1 + r - i], acc);
                out[e][r] = acc;
            }
    };

    float qf[2][4];  // q' of the chunk featurized last, consumed by the gate one iteration later
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int r = 0; r < 4; ++r) qf[e][r] = 0.0f;

    auto gate_store = [&](int j) {
        const int64_t tb = t_begin + (int64_t)(j - 1) * kChunk;
        if (j >= 1 && j <= nch && tb >= t_start) {  // uniform
#pragma unroll
            for (int r = 0; r < kSeg; ++r) {
                const int row = kSeg * seg + r;
                const int64_t t = tb + row;
                if (t < t_end) {
                    const float2 z2 = *reinterpret_cast<const float2*>(zst + row * kZRow + cp * 8);
                    const uint32_t y2 = pack_bf16x2(z2.x * qf[0][r], z2.y * qf[1][r]);
                    __builtin_nontemporal_store(y2, reinterpret_cast<uint32_t*>(a.y + seq0 + t * D + cblock0 + 2 * cp));
                }
            }
        }
    };

    // ring slots of the look-back chunk 0 and of chunk 1
    ring_write(0, kpre[0], vpre[0], qpre[0]);
    load_raw(PF, kpre[0], vpre[0], qpre[0]);
    ring_write(1, kpre[1 % PF], vpre[1 % PF], qpre[1 % PF]);
    load_raw(PF + 1, kpre[1 % PF], vpre[1 % PF], qpre[1 % PF]);
    __syncthreads();

    for (int jb = 1; jb <= nch; jb += PF) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int j = jb + s;
            const int stage = (s + 2) % PF;  // chunk j + 1 lives in stage (j + 1) % PF and jb = 1 (mod PF)
            const int64_t tb = t_begin + (int64_t)(j - 1) * kChunk;
            const bool live = j <= nch;
            const bool main_chunk = live && tb >= t_start;

            // ---------------- phase 1
            ring_write(j + 1, kpre[stage], vpre[stage], qpre[stage]);
            load_raw(j + 1 + PF, kpre[stage], vpre[stage], qpre[stage]);
            gate_store(j - 1);
            {
                float kf[2][4], vf[2][4];
                featurize(0, j, tk_, kf);
                featurize(1, j, tv_, vf);
                uint32_t* u32 = reinterpret_cast<uint32_t*>(ust);
#pragma unroll
                for (int r = 0; r < kSeg; ++r) {
                    const int row = kSeg * seg + r;
                    const int swz = ((row >> 3) & 3) << 1;
                    u32[row * (kPPR * 4) + ((((cp >> 2) ^ swz)) << 2) + (cp & 3)] =
                        pack_bf16x2(kf[0][r] * vf[0][r], kf[1][r] * vf[1][r]);
                }
                if (main_chunk) featurize(2, j, tq_, qf);  // uniform
            }
            __syncthreads();

            // ---------------- phase 2
#pragma unroll
            for (int m = NKB - 1; m > 0; --m) uw[m] = uw[m - 1];
            {
                const uint16_t* s16 = reinterpret_cast<const uint16_t*>(ust);
                Words<4> wds;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int r0 = 8 * lq + 2 * e2;
                    const uint32_t lo = s16[((r0 * kPPR + rd_piece) << 3) + (li & 7)];
                    const uint32_t hi = s16[(((r0 + 1) * kPPR + rd_piece) << 3) + (li & 7)];
                    wds.w[e2] = lo | (hi << 16);
                }
                uw[0] = __builtin_bit_cast(bf16x8_t, wds);
            }
            if (main_chunk) {
                f32x4_t acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int m = 0; m < NKB; ++m) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(uw[m], tz[2 * m], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(uw[m], tz[2 * m + 1], acc1, 0, 0, 0);
                }
                char* zp = zst + zwr_off;
                *reinterpret_cast<float4*>(zp) = make_float4(acc0[0], acc0[1], acc0[2], acc0[3]);
                *reinterpret_cast<float4*>(zp + 16 * kZRow) = make_float4(acc1[0], acc1[1], acc1[2], acc1[3]);
            }
            __syncthreads();
        }
    }
    if (nch % PF == 0) gate_store(nch);  // otherwise an idle iteration of the unrolled loop already did it
}

template <int NKB, int LF, int kNW>
hy_status launch_chain_nw(const ChainPtrs& p, const ChainShape& s, hipStream_t st) {
    constexpr int PF = 4;  // chunks of raw q, k, v in flight per lane; two waves per SIMD must fit
    ChainArgs a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.hq = p.hq;
    a.hk = p.hk;
    a.hv = p.hv;
    a.h = p.h;
    a.y = static_cast<uint16_t*>(p.y);
    a.L = s.L;
    a.D = s.D;
    a.lh = s.lh;
    a.group = s.group;
    a.feat_group = s.feat_group;
    a.ncb = (int32_t)(s.D / (16 * kNW));
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        const int64_t want = 256 * (8 / kNW);  // 8 waves per CU
        int64_t tiles = want / (s.B * a.ncb);
        if (tiles < 1) tiles = 1;
        rows = (s.L + tiles - 1) / tiles;
        const int64_t min_rows = 8LL * kChunk * (NKB > 1 ? NKB - 1 : 1);
        if (rows < min_rows) rows = min_rows;
    }
    rows = (rows + kChunk - 1) / kChunk * kChunk;
    if (rows > (s.L + kChunk - 1) / kChunk * kChunk) rows = (s.L + kChunk - 1) / kChunk * kChunk;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb = s.B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((chain_mfma_kernel<NKB, LF, PF, kNW>), dim3((uint32_t)nb), dim3(kNW * 64), 0, st, a);
    return launch_status();
}

template <int NKB, int LF>
hy_status launch_chain(const ChainPtrs& p, const ChainShape& s, hipStream_t st) {
    if (tuning().mr_waves == 4) return launch_chain_nw<NKB, LF, 4>(p, s, st);
    return launch_chain_nw<NKB, LF, 8>(p, s, st);
}

template <int NKB>
hy_status by_lf(const ChainPtrs& p, const ChainShape& s, hipStream_t st) {
    switch (s.lf) {
        case 1: return launch_chain<NKB, 1>(p, s, st);
        case 2: return launch_chain<NKB, 2>(p, s, st);
        case 3: return launch_chain<NKB, 3>(p, s, st);
        case 4: return launch_chain<NKB, 4>(p, s, st);
        case 5: return launch_chain<NKB, 5>(p, s, st);
        case 6: return launch_chain<NKB, 6>(p, s, st);
        case 7: return launch_chain<NKB, 7>(p, s, st);
        case 8: return launch_chain<NKB, 8>(p, s, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace

bool chain_fused_supported(const ChainShape& s) {
    return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 128 == 0 && s.lh <= 129 && s.lf >= 1 && s.lf <= 8;
}

hy_status launch_chain_fused(const ChainPtrs& p, const ChainShape& s, hipStream_t st) {
    if (!chain_fused_supported(s)) return HY_ERR_UNSUPPORTED;
    const int nkb = (s.lh - 1 + 31) / 32 + 1;
    switch (nkb) {
        case 1: return by_lf<1>(p, s, st);
        case 2: return by_lf<2>(p, s, st);
        case 3: return by_lf<3>(p, s, st);
        case 4: return by_lf<4>(p, s, st);
        case 5: return by_lf<5>(p, s, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
