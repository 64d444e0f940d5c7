// Fused Hyena-MR operator chain, forward (Sec. 2.1 Eq. 1 without the dense projections):
//     q' = hq * q,  k' = hk * k,  v' = hv * v          short per-channel featurizer convolutions
//     y  = q' (.) ( h * (k' (.) v') )                  grouped medium convolution with both gates
// with the featurizers on the matrix cores as well.  (An earlier kernel that evaluated the three short
// convolutions on the vector ALUs was bound by vector instruction issue and has been removed.)  Here every
// convolution is a Toeplitz product and the vector ALUs only gate, convert and transpose.
//
//   featurizers  one filter per channel, so chunks of one channel go on the matrix tile (App. A.1) with the batched
//                instruction v_mfma_f32_4x4x4_16B_bf16 as in cp4_kernels.hip: per tensor and 16 outputs of 16
//                channels, 3 products A_m X_m (A_m[i][k] = hf[4m + i - k], 8 steps of look-back, lf <= 9).  The
//                inputs are bf16 already; each fp32 tap enters as a bf16 head plus a bf16 remainder (two products
//                against the same X_m), which keeps 16 bits of the tap's mantissa.  q', k', v' come out in fp32.
//   medium conv  block-Toeplitz contraction of Sec. 3.1 as in mr_kernels.hip (register-resident operands for
//                d = 0, 16, 32, ..., register window of the last NKB source blocks), with the operands swapped
//                so that time is on the rows of the product: a lane ends up with 4 consecutive steps of one
//                channel, the layout the featurizer produces and the gate consumes.
// Everything on chip is laid out [channel][time].  A wave owns 16 channels for all products, so u = k'v' and q'
// never cross waves; only the raw inputs and y do.
//
// Twelve waves per workgroup and 128 channels: waves 0..7 multiply, waves 8..11 move data (16-byte row pieces of
// q, k, v from HBM, two rows packed per 4-byte LDS write into the channels' lines; y back the same way).  While
// the multipliers work on iteration j (32 steps) the movers store y of j-1 and stage the raw inputs of j+1; one
// barrier per iteration.  Raw lines hold 3 slots of 32 steps (j-1 for the look-back, j, j+1), y has 2 slots.
#include <type_traits>

#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct Chain4Args {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* hq;
    const float* hk;
    const float* hv;
    const float* h;
    uint16_t* y;
    int64_t L, D;
    int64_t bstride_in, bstride_y;  // elements between batch items in q, k, v / in y
    int32_t hist;                   // rows of q, k, v in front of row 0 that hold data
    int32_t lh, lf, group, feat_group;
    int32_t rows;           // time steps per workgroup, multiple of 32
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / 128
};

constexpr int kT = 32;           // steps per iteration
constexpr int kWM = 8;           // multiplier waves
constexpr int kWV = 4;           // mover waves
constexpr int kC = 16 * kWM;     // channels per workgroup
constexpr int kNF = 3;           // featurizer products per 16 outputs
constexpr int kRawSteps = 3 * kT;
// Line strides and skews in bytes, chosen with a bank-conflict probe for the access patterns named:
constexpr int kRawS = 224;       // raw line: 4-byte transposing writes (+8 per 8 channels), 8-byte operand reads
constexpr int kUS = 160;         // u line: 8-byte writes (4 steps), 16-byte operand reads (8 steps)
constexpr int kQS = 160;         // q' line (fp32): 16-byte writes and reads (4 steps)
constexpr int kYS = 80;          // y line: 8-byte writes (4 steps), 4-byte transposing reads (+136 per 8 channels)
constexpr int kYSkew = 136;

// PF = iterations of q, k, v in flight per mover lane (register stages); must divide 6.
template <int NKB, int PF>
__global__ __launch_bounds__((kWM + kWV) * 64, 3) void chain4_kernel(Chain4Args a) {
    static_assert(6 % PF == 0, "the stage index must be static in a loop unrolled by 6");
    constexpr int kTaps = 32 * NKB;
    __shared__ __attribute__((aligned(16))) char raw[3][kC * kRawS + (kC / 8) * 8];
    __shared__ __attribute__((aligned(16))) char ust[kC * kUS];
    __shared__ __attribute__((aligned(16))) char qst[kC * kQS];
    __shared__ __attribute__((aligned(16))) char yst[2][kC * kYS + (kC / 8) * kYSkew];
    static_assert(16 * kQS >= kTaps * 4, "a wave's q' lines double as the staging area of its filter");

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int ts32 = (int)((tile % a.tiles_per_seq) * (int64_t)a.rows);
    const int te32 = (ts32 + a.rows < a.L) ? ts32 + a.rows : (int)a.L;
    const int nit = (te32 - ts32 + kT - 1) / kT;
    // iteration idx holds steps ts32 + 32 (idx - NKB) ...: idx 0 is only looked back at, 1 .. NKB-1 fill the source
    // window of the medium convolution, NKB .. last produce output
    const int last = NKB + nit - 1;

    const uint32_t D32 = (uint32_t)a.D;
    const int64_t cblock0 = (int64_t)cb * kC;
    const int64_t seq0 = b * a.bstride_in, seq0y = b * a.bstride_y;
    const int t_old = -a.hist;  // oldest row that holds data; what lies before it counts as zeros
    using std::integral_constant;

    if (w < kWM) {
        // ================= multiplier waves
        const int blk = lane >> 2, l4 = lane & 3;    // featurizer products: channel blk, column l4 (4 steps)
        const int li = lane & 15, lq = lane >> 4;    // medium products: channel li, step quad / source octet lq
        const int cf = 16 * w + blk, cm = 16 * w + li;

        // ---- featurizer operands: tensor x (k, v, q), product m, head / remainder
        s16x4_t af[3][kNF][2];
        {
            const float* hf[3] = {a.hk, a.hv, a.hq};
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const float* hp = hf[x] + ((cblock0 + cf) / a.feat_group) * (int64_t)a.lf;
#pragma unroll
                for (int m = 0; m < kNF; ++m) {
                    float t4[4];  // t4[k] = hf[4m + i - k], i = l4
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        const int idx = 4 * m + l4 - kk;
                        t4[kk] = (idx >= 0 && idx < a.lf) ? hp[idx] : 0.0f;
                    }
                    Words<2> hi, lo;
                    hi.w[0] = pack_bf16x2(t4[0], t4[1]);
                    hi.w[1] = pack_bf16x2(t4[2], t4[3]);
                    lo.w[0] = pack_bf16x2(t4[0] - bf16_lo(hi.w[0]), t4[1] - bf16_hi(hi.w[0]));
                    lo.w[1] = pack_bf16x2(t4[2] - bf16_lo(hi.w[1]), t4[3] - bf16_hi(hi.w[1]));
                    af[x][m][0] = __builtin_bit_cast(s16x4_t, hi);
                    af[x][m][1] = __builtin_bit_cast(s16x4_t, lo);
                }
            }
        }
        // ---- Toeplitz operands of the medium filter: operand i serves d = 16 i; lane (li = output step, lq = source
        // octet), element e holds h[d + li - 8 lq - e], zero outside [0, lh).  The filter is staged in the wave's
        // own q' lines, which nothing else touches before the first iteration.
        bf16x8_t tz[2 * NKB];
        {
            float* hsw = reinterpret_cast<float*>(qst + (16 * w) * kQS);
            const float* hp = a.h + ((cblock0 + 16 * w) / a.group) * (int64_t)a.lh;
            for (int j = lane; j < kTaps; j += 64) hsw[j] = (j < a.lh) ? hp[j] : 0.0f;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 2 * NKB; ++i) {
                Words<4> wds;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int i0 = 16 * i + li - 8 * lq - 2 * e2;
                    const int i1 = i0 - 1;
                    const float f0 = (i0 >= 0 && i0 < kTaps) ? hsw[i0] : 0.0f;
                    const float f1 = (i1 >= 0 && i1 < kTaps) ? hsw[i1] : 0.0f;
                    wds.w[e2] = pack_bf16x2(f0, f1);
                }
                tz[i] = __builtin_bit_cast(bf16x8_t, wds);
            }
        }
        bf16x8_t uw[NKB];  // window of the last NKB source blocks of 32 steps
        {
            Words<4> z = zero_words<4>();
#pragma unroll
            for (int m = 0; m < NKB; ++m) uw[m] = __builtin_bit_cast(bf16x8_t, z);
        }

        // ---- lane offsets
        const int raw_line = cf * kRawS + (cf >> 3) * 8;
        const int raw_lane = raw_line + 8 * l4;                                  // position 4 l4
        const int raw_mix1 = raw_line + 2 * ((4 * l4 - 4 + kRawSteps) % kRawSteps);  // position 4 l4 - 4, wrapped
        const int raw_mix2 = raw_line + 2 * ((4 * l4 - 8 + kRawSteps) % kRawSteps);
        char* const u_wr = ust + cf * kUS + 8 * l4;
        char* const q_wr = qst + cf * kQS + 16 * l4;
        const char* const u_rd = ust + cm * kUS + 16 * lq;
        const char* const q_rd = qst + cm * kQS + 16 * lq;
        const int y_wr = cm * kYS + (cm >> 3) * kYSkew + 8 * lq;

        // one featurizer: 16 outputs (group g of the iteration in raw slot SL) of the lane's channel and column
        auto feat = [&](auto x_c, auto c0_c) {
            constexpr int X = decltype(x_c)::value;
            constexpr int C0 = decltype(c0_c)::value;  // ring position of the group's first step
            f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int m = 0; m < kNF; ++m) {
                const int c0 = (C0 - 4 * m + kRawSteps) % kRawSteps;
                int off;
                if (c0 <= kRawSteps - 16) off = raw_lane + 2 * c0;
                else if (c0 == kRawSteps - 4) off = raw_mix1;
                else off = raw_mix2;
                const uint2 bw = *reinterpret_cast<const uint2*>(raw[X] + off);
                Words<2> bb;
                bb.w[0] = bw.x; bb.w[1] = bw.y;
                const s16x4_t bv = __builtin_bit_cast(s16x4_t, bb);
                acc = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(af[X][m][0], bv, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(af[X][m][1], bv, acc, 0, 0, 0);
            }
            return acc;
        };

        auto mstep = [&](auto j6_c, int idx) {
            constexpr int J6 = decltype(j6_c)::value;   // idx mod 6
            constexpr int SL = J6 % 3;                  // raw slot of this iteration
            constexpr int YS = J6 & 1;                  // y slot
            const bool main_it = idx >= NKB;
            // featurize; u = k'v' in bf16 into the wave's u lines, q' in fp32 into its q' lines
            auto fgroup = [&](auto g_c) {
                constexpr int G = decltype(g_c)::value;
                using pos = integral_constant<int, kT * SL + 16 * G>;
                const f32x4_t kx = feat(integral_constant<int, 0>{}, pos{});
                const f32x4_t vx = feat(integral_constant<int, 1>{}, pos{});
                *reinterpret_cast<uint2*>(u_wr + 32 * G) =
                    make_uint2(pack_bf16x2(kx[0] * vx[0], kx[1] * vx[1]), pack_bf16x2(kx[2] * vx[2], kx[3] * vx[3]));
                if (main_it) {
                    const f32x4_t qx = feat(integral_constant<int, 2>{}, pos{});
                    *reinterpret_cast<float4*>(q_wr + 64 * G) = make_float4(qx[0], qx[1], qx[2], qx[3]);
                }
            };
            fgroup(integral_constant<int, 0>{});
            fgroup(integral_constant<int, 1>{});
            // medium convolution: the wave's own 32 x 16 block of u, 8 consecutive steps of a channel per lane
#pragma unroll
            for (int m = NKB - 1; m > 0; --m) uw[m] = uw[m - 1];
            {
                const uint4 t = *reinterpret_cast<const uint4*>(u_rd);
                Words<4> wds;
                wds.w[0] = t.x; wds.w[1] = t.y; wds.w[2] = t.z; wds.w[3] = t.w;
                uw[0] = __builtin_bit_cast(bf16x8_t, wds);
            }
            if (main_it) {
                f32x4_t acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int m = 0; m < NKB; ++m) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tz[2 * m], uw[m], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tz[2 * m + 1], uw[m], acc1, 0, 0, 0);
                }
                // the lane holds z of channel li at steps 4 lq .. + 3 and 16 + 4 lq .. + 3
                const float4 q0 = *reinterpret_cast<const float4*>(q_rd);
                const float4 q1 = *reinterpret_cast<const float4*>(q_rd + 64);
                char* yp = yst[YS] + y_wr;
                *reinterpret_cast<uint2*>(yp) =
                    make_uint2(pack_bf16x2(q0.x * acc0[0], q0.y * acc0[1]), pack_bf16x2(q0.z * acc0[2], q0.w * acc0[3]));
                *reinterpret_cast<uint2*>(yp + 32) =
                    make_uint2(pack_bf16x2(q1.x * acc1[0], q1.y * acc1[1]), pack_bf16x2(q1.z * acc1[2], q1.w * acc1[3]));
            }
            __syncthreads();
        };

        __syncthreads();  // raw inputs of iterations 0 and 1 are in place
        for (int idx = 1; idx <= last; idx += 6) {
            mstep(integral_constant<int, 1>{}, idx);
            if (idx + 1 <= last) mstep(integral_constant<int, 2>{}, idx + 1);
            if (idx + 2 <= last) mstep(integral_constant<int, 3>{}, idx + 2);
            if (idx + 3 <= last) mstep(integral_constant<int, 4>{}, idx + 3);
            if (idx + 4 <= last) mstep(integral_constant<int, 5>{}, idx + 4);
            if (idx + 5 <= last) mstep(integral_constant<int, 0>{}, idx + 5);
        }
    } else {
        // ================= mover waves: lane = 16-byte piece lp of rows 2 rp and 2 rp + 1 of an iteration
        const int mt = tid - kWM * 64;
        const int lp = mt & 15, rp = mt >> 4;
        const uint32_t ld_off = (uint32_t)(cblock0 + 8 * lp);
        const int raw_wr = (8 * lp) * kRawS + lp * 8 + 4 * rp;
        const int y_rd = (8 * lp) * kYS + lp * kYSkew + 4 * rp;

        auto row_addr = [&](int t) {  // clamped into the rows this tile may touch
            t = t < te32 ? t : te32 - 1;
            t = t > t_old ? t : t_old;
            return seq0 + ((int64_t)t * (int64_t)D32 + ld_off);
        };
        Words<4> kw[PF][2], vw[PF][2], qw[PF][2];
        auto load_rows = [&](int idx, Words<4> (&kk)[2], Words<4> (&vv)[2], Words<4> (&qq)[2]) {
            const int t0 = ts32 + (idx - NKB) * kT + 2 * rp;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int64_t off = row_addr(t0 + r);
                kk[r] = load_words_nt<4>(a.k + off);
                vv[r] = load_words_nt<4>(a.v + off);
                if (idx >= NKB - 1) qq[r] = load_words_nt<4>(a.q + off);  // the last window-filling iteration is q's look-back
            }
        };
        // two rows x 8 channels of one tensor, transposed: one dword (2 steps) per channel
        auto write_raw = [&](char* base, const Words<4> (&xx)[2], bool keep0, bool keep1) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t x0 = keep0 ? xx[0].w[p] : 0u, x1 = keep1 ? xx[1].w[p] : 0u;
                *reinterpret_cast<uint32_t*>(base + (2 * p) * kRawS) = (x0 & 0xffffu) | (x1 << 16);
                *reinterpret_cast<uint32_t*>(base + (2 * p + 1) * kRawS) = (x0 >> 16) | (x1 & 0xffff0000u);
            }
        };
        auto prepare = [&](int idx, int sl, Words<4> (&kk)[2], Words<4> (&vv)[2], Words<4> (&qq)[2]) {
            const int t = ts32 + (idx - NKB) * kT + 2 * rp;
            const int off = raw_wr + 2 * kT * sl;
            write_raw(raw[0] + off, kk, t >= t_old, t + 1 >= t_old);
            write_raw(raw[1] + off, vv, t >= t_old, t + 1 >= t_old);
            if (idx >= NKB - 1) write_raw(raw[2] + off, qq, t >= t_old, t + 1 >= t_old);
        };
        auto store_y = [&](int idx, int ys) {
            uint32_t yc[8];
            const char* yl = yst[ys] + y_rd;
#pragma unroll
            for (int c8 = 0; c8 < 8; ++c8) yc[c8] = *reinterpret_cast<const uint32_t*>(yl + c8 * kYS);
            Words<4> row0, row1;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                row0.w[p] = (yc[2 * p] & 0xffffu) | (yc[2 * p + 1] << 16);
                row1.w[p] = (yc[2 * p] >> 16) | (yc[2 * p + 1] & 0xffff0000u);
            }
            const int t = ts32 + (idx - NKB) * kT + 2 * rp;
            if (t < te32) store_words_nt<4>(a.y + seq0y + ((uint64_t)(uint32_t)t * D32 + ld_off), row0);
            if (t + 1 < te32) store_words_nt<4>(a.y + seq0y + ((uint64_t)(uint32_t)(t + 1) * D32 + ld_off), row1);
        };

#pragma unroll
        for (int i = 0; i < PF; ++i)
            if (i <= last) load_rows(i, kw[i], vw[i], qw[i]);
        __syncthreads();  // pairs with the multipliers' barrier around the filter staging
        prepare(0, 0, kw[0], vw[0], qw[0]);
        if (PF <= last) load_rows(PF, kw[0], vw[0], qw[0]);
        prepare(1, 1, kw[1 % PF], vw[1 % PF], qw[1 % PF]);
        if (1 + PF <= last) load_rows(1 + PF, kw[1 % PF], vw[1 % PF], qw[1 % PF]);
        __syncthreads();

        auto vstep = [&](auto j6_c, int idx) {
            constexpr int J6 = decltype(j6_c)::value;  // idx mod 6
            constexpr int ST = (J6 + 1) % PF;          // stage of iteration idx + 1
            if (idx - 1 >= NKB) store_y(idx - 1, (J6 + 1) & 1);
            if (idx + 1 <= last) {
                prepare(idx + 1, (J6 + 1) % 3, kw[ST], vw[ST], qw[ST]);
                if (idx + 1 + PF <= last) load_rows(idx + 1 + PF, kw[ST], vw[ST], qw[ST]);
            }
            __syncthreads();
        };
        for (int idx = 1; idx <= last; idx += 6) {
            vstep(integral_constant<int, 1>{}, idx);
            if (idx + 1 <= last) vstep(integral_constant<int, 2>{}, idx + 1);
            if (idx + 2 <= last) vstep(integral_constant<int, 3>{}, idx + 2);
            if (idx + 3 <= last) vstep(integral_constant<int, 4>{}, idx + 3);
            if (idx + 4 <= last) vstep(integral_constant<int, 5>{}, idx + 4);
            if (idx + 5 <= last) vstep(integral_constant<int, 0>{}, idx + 5);
        }
        store_y(last, last & 1);
    }
}

template <int NKB>
hy_status launch_chain4_nkb(const ChainPtrs& p, const ChainShape& s, hipStream_t st) {
    constexpr int PF = 3;  // 2 stages measured 1.7% slower; 6 do not fit the registers of three waves per SIMD
    Chain4Args a;
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
    a.bstride_in = s.stride_in();
    a.bstride_y = s.stride_y();
    a.hist = s.history;
    a.lh = s.lh;
    a.lf = s.lf;
    a.group = s.group;
    a.feat_group = s.feat_group;
    a.ncb = (int32_t)(s.D / kC);
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        const int64_t min_rows = 8LL * kT * (NKB > 1 ? NKB - 1 : 1);
        const int64_t tiles = tiles_filling_rounds(s.B * a.ncb, s.L, min_rows);  // one workgroup per CU
        rows = (s.L + tiles - 1) / tiles;
        if (rows < min_rows) rows = min_rows;
    }
    rows = (rows + kT - 1) / kT * kT;
    if (rows > (s.L + kT - 1) / kT * kT) rows = (s.L + kT - 1) / kT * kT;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb = s.B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel((chain4_kernel<NKB, PF>), dim3((uint32_t)nb), dim3((kWM + kWV) * 64), st, a);
}

}  // namespace

bool chain4_supported(const ChainShape& s) {
    return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % kC == 0 && s.lh >= 1 && s.lh <= 129 && s.lf >= 1 &&
           s.lf <= 9 && s.L <= 0x7fff0000LL && s.D <= 0x7fff0000LL;
}

hy_status launch_chain4(const ChainPtrs& p, const ChainShape& s, hipStream_t st) {
    if (!chain4_supported(s)) return HY_ERR_UNSUPPORTED;
    const int nkb = (s.lh - 1 + 31) / 32 + 1;
    switch (nkb) {
        case 1: return launch_chain4_nkb<1>(p, s, st);
        case 2: return launch_chain4_nkb<2>(p, s, st);
        case 3: return launch_chain4_nkb<3>(p, s, st);
        case 4: return launch_chain4_nkb<4>(p, s, st);
        case 5: return launch_chain4_nkb<5>(p, s, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
