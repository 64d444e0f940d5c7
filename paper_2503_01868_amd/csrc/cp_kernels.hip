// Chunk-parallel block-Toeplitz contraction on the gfx950 matrix cores (App. A.1): the gated causal
// convolution of Eq. 1 for filters that are NOT shared by 16 adjacent channels (d_g = 1, 2, 4, 8, ...),
// where the grouped kernel of mr_kernels.hip has no channel dimension to put on the matrix tile.
//
// Mapping.  For one channel, 16 consecutive chunks of 16 time steps are the columns of one product
//   Z[i, n] = sum_k A[i, k] * X[k, n],   i = step inside chunk n,  X[k, n] = u[16 n + 16 - K + k],
//   A[i, k] = h[K - 16 + i - k]  (zero outside [0, lh)),  K = 32 NKB >= lh + 15,
// i.e. [H_{NKB'} ... H_1 H_0] applied to the chunk and its predecessors (Sec. 3.1), with the same Toeplitz
// operand A for every chunk of the channel.  One v_mfma_f32_16x16x32_bf16 per 32 source steps yields 256
// outputs of the channel; A differs per channel, so channels are processed one after another by a wave.
//
// Memory has channels contiguous, the product wants time contiguous, so both directions go through LDS
// in [channel][time] order.  A workgroup (8 waves) owns 64 channels and `rows` time steps and walks them
// in iterations of 256 steps:
//   row phase   every lane owns 4 consecutive rows x 8 channels (16-byte global loads of k, v, q, issued one
//               iteration ahead), forms u = k*v, rounds to bf16 and writes, per channel, 4 steps (8 bytes) of
//               u into a per-channel ring of 256 + K steps and 4 steps of q into a [channel][256] buffer;
//   matrix phase wave w takes channels 8w..8w+7: per channel NKB x (A from a per-channel reversed-filter
//               table in LDS, 8 steps of u per lane with one 16-byte LDS read, one MFMA), then gates the 4
//               consecutive steps it holds with q and overwrites q by y in place;
//   store phase every lane reads back its 4 rows x 8 channels of y, re-forms rows and stores 16-byte pieces.
// Two barriers per 256 steps.  The ring keeps the last K steps, so the filter history costs no re-reads
// inside a tile; a tile that does not start the sequence first loads the K steps before it.
//
// A needs, per lane, 8 consecutive entries of the reversed filter starting at any offset; the table holds
// two bf16 copies per channel, shifted by one entry, so that every such window is four aligned dwords.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

struct CpArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* h;
    uint16_t* y;
    int64_t L, D;
    int32_t lh, group;
    int32_t rows;           // time steps per workgroup, multiple of 256
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / 64
};

constexpr int kC = 64;         // channels per workgroup
constexpr int kT = 256;        // steps per iteration: 16 chunks of 16
constexpr int kThreads = 512;  // 8 waves

template <int NKB>
__global__ __launch_bounds__(kThreads, 2) void cp_mfma_kernel(CpArgs a) {
    constexpr int kK = 32 * NKB;       // contraction length per chunk
    constexpr int kR = kT + kK;        // ring length in steps (multiple of 32)
    constexpr int kUS = kR * 2;        // bytes per channel line of u
    constexpr int kQS = kT * 2;        // bytes per channel line of q / y
    constexpr int kGW = 16 * NKB + 8;  // dwords per copy of the reversed filter
    // each block of 8 channels starts 16 bytes further than the line stride alone would put it: measured on
    // MI355X, the transposing 8-byte writes of a wave (8 row groups x 8 channel blocks) then run at the full
    // write rate of the LDS, against a quarter of it with blocks a multiple of 128 bytes apart
    __shared__ __attribute__((aligned(16))) char us[kC * kUS + (kC / 8) * 16];
    __shared__ __attribute__((aligned(16))) char qs[kC * kQS + (kC / 8) * 16];
    // reversed-filter tables, copy-major; the second copy starts 16 banks off the first, so that the even and
    // the odd lanes of a matrix-operand read (12 adjacent dwords of either copy) never meet in a bank
    constexpr int kGC = kC * kGW + (16 - (kC * kGW) % 32 + 32) % 32;
    __shared__ uint32_t gt[2 * kGC];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const int li = lane % 16, lq = lane / 16;

    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t t_start = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t_end = (t_start + a.rows < a.L) ? t_start + a.rows : a.L;
    const int nit = (int)((t_end - t_start + kT - 1) / kT);

    const int64_t D = a.D;
    const int64_t cblock0 = (int64_t)cb * kC;
    const int64_t seq0 = b * a.L * D;

    // ---- row layout: rows 4 rg .. 4 rg + 3 of an iteration, channels 8 lp .. 8 lp + 7 of the block
    const int lp = tid % 8, rg = tid / 8;
    const int64_t col = seq0 + cblock0 + 8 * lp;
    auto line_off = [](int c, int stride) { return c * stride + (c >> 3) * 16; };
    char* const u_lines = us + line_off(8 * lp, kUS);  // this lane's 8 channel lines are kUS apart
    char* const q_lines = qs + line_off(8 * lp, kQS) + 8 * rg;

    // Loads are unconditional; a row past the end of the tile re-reads the tile's last row.
    Words<4> kw[4], vw[4], qw[4];
    auto load_rows = [&](int it) {  // iteration it >= 1 covers steps t_start + 256 (it - 1) ...
        const int64_t t0 = t_start + (int64_t)(it - 1) * kT + 4 * rg;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int64_t t = t0 + r;
            t = t < t_end ? t : t_end - 1;
            const int64_t off = col + t * D;
            kw[r] = load_words_nt<4>(a.k + off);
            vw[r] = load_words_nt<4>(a.v + off);
            qw[r] = load_words_nt<4>(a.q + off);
        }
    };
    // u of 4 rows x 8 channels -> 8 ring lines, 4 steps (8 bytes) each; rows with keep[r] false become zeros
    auto write_u = [&](const Words<4> (&kk)[4], const Words<4> (&vv)[4], const bool (&keep)[4], int pos) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            float ulo[4], uhi[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ulo[r] = keep[r] ? bf16_lo(kk[r].w[p]) * bf16_lo(vv[r].w[p]) : 0.0f;
                uhi[r] = keep[r] ? bf16_hi(kk[r].w[p]) * bf16_hi(vv[r].w[p]) : 0.0f;
            }
            *reinterpret_cast<uint2*>(u_lines + (2 * p) * kUS + pos * 2) =
                make_uint2(pack_bf16x2(ulo[0], ulo[1]), pack_bf16x2(ulo[2], ulo[3]));
            *reinterpret_cast<uint2*>(u_lines + (2 * p + 1) * kUS + pos * 2) =
                make_uint2(pack_bf16x2(uhi[0], uhi[1]), pack_bf16x2(uhi[2], uhi[3]));
        }
    };

    load_rows(1);

    // ---- reversed filter tables: g[x] = h[K - 1 - x]; copy 0 holds (g[2x], g[2x+1]), copy 1 (g[2x+1], g[2x+2])
    for (int idx = tid; idx < kC * 2 * kGW; idx += kThreads) {
        const int c = idx / (2 * kGW);
        const int rem = idx % (2 * kGW);
        const int par = rem / kGW, x = rem % kGW;
        const float* hp = a.h + ((cblock0 + c) / a.group) * (int64_t)a.lh;
        const int j0 = kK - 1 - (2 * x + par);
        const float g0 = (j0 >= 0 && j0 < a.lh) ? hp[j0] : 0.0f;
        const float g1 = (j0 - 1 >= 0 && j0 - 1 < a.lh) ? hp[j0 - 1] : 0.0f;
        gt[par * kGC + c * kGW + x] = pack_bf16x2(g0, g1);
    }

    // ---- history: the K steps before the tile go to ring positions 256 - K .. 255 (whole waves take part)
    if (4 * rg >= kT - kK) {
        Words<4> kh[4], vh[4];
        bool keep[4];
        const int64_t t0 = t_start - kT + 4 * rg;  // < t_start; negative exactly when the tile starts the sequence
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t t = t0 + r >= 0 ? t0 + r : 0;
            kh[r] = load_words_nt<4>(a.k + col + t * D);
            vh[r] = load_words_nt<4>(a.v + col + t * D);
            keep[r] = t0 + r >= 0;  // zero left padding of every sequence
        }
        write_u(kh, vh, keep, 4 * rg);
    }

    // matrix-phase constants of this lane
    const uint32_t* const g_lane = gt + ((li & 1) ^ 1) * kGC + 8 * w * kGW + ((15 - li) >> 1) + 4 * lq;
    const int x_lane = 16 * li + 16 - kK + 8 * lq;  // ring position of the lane's first source octet, relative to wb
    const int qy_lane = (16 * li + 4 * lq) * 2;

    // The Toeplitz operands of the wave's 8 channels never change: the first kAR source blocks of each stay in
    // registers for the whole tile (the register file has room for 4 x 8 of them beside the row phase), the
    // rest is re-read from the tables every iteration.  Reading them all from LDS made the matrix phase
    // LDS-bound (8 of the 12 LDS cycles per product were operand A).
    constexpr int kAR = NKB < 4 ? NKB : 4;
    bf16x8_t ares[8][kAR];
    __syncthreads();  // tables complete
#pragma unroll
    for (int cc = 0; cc < 8; ++cc)
#pragma unroll
        for (int m = 0; m < kAR; ++m) {
            Words<4> aw;
#pragma unroll
            for (int d = 0; d < 4; ++d) aw.w[d] = g_lane[cc * kGW + 16 * m + d];
            ares[cc][m] = __builtin_bit_cast(bf16x8_t, aw);
        }

    int wb = 0;
    for (int it = 1; it <= nit; ++it) {
        wb += kT;
        if (wb >= kR) wb -= kR;
        const int64_t ts = t_start + (int64_t)(it - 1) * kT;

        // ---- row phase
        {
            bool keep[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) keep[r] = ts + 4 * rg + r < t_end;
            int pos = wb + 4 * rg;
            if (pos >= kR) pos -= kR;
            write_u(kw, vw, keep, pos);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t q0 = qw[0].w[p], q1 = qw[1].w[p], q2 = qw[2].w[p], q3 = qw[3].w[p];
                *reinterpret_cast<uint2*>(q_lines + (2 * p) * kQS) =
                    make_uint2((q0 & 0xffffu) | (q1 << 16), (q2 & 0xffffu) | (q3 << 16));
                *reinterpret_cast<uint2*>(q_lines + (2 * p + 1) * kQS) =
                    make_uint2((q0 >> 16) | (q1 & 0xffff0000u), (q2 >> 16) | (q3 & 0xffff0000u));
            }
        }
        load_rows(it + 1);
        __syncthreads();

        // ---- matrix phase: channels 8 w .. 8 w + 7
        {
            int x0 = wb + x_lane;
            if (x0 < 0) x0 += kR;
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                const int c = 8 * w + cc;
                const char* ul = us + line_off(c, kUS);
                const uint32_t* gl = g_lane + cc * kGW;
                f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
                int x = x0;
#pragma unroll
                for (int m = 0; m < NKB; ++m) {
                    if (x >= kR) x -= kR;
                    bf16x8_t av;
                    {
                        if (m < kAR) {
                            av = ares[cc][m < kAR ? m : 0];
                        } else {
                            Words<4> aw;
#pragma unroll
                            for (int d = 0; d < 4; ++d) aw.w[d] = gl[16 * m + d];
                            av = __builtin_bit_cast(bf16x8_t, aw);
                        }
                    }
                    const uint4 bw = *reinterpret_cast<const uint4*>(ul + x * 2);
                    Words<4> bww;
                    bww.w[0] = bw.x; bww.w[1] = bw.y; bww.w[2] = bw.z; bww.w[3] = bw.w;
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8_t, bww), acc, 0, 0, 0);
                    x += 32;
                }
                char* ql = qs + line_off(c, kQS) + qy_lane;
                const uint2 q4 = *reinterpret_cast<const uint2*>(ql);
                *reinterpret_cast<uint2*>(ql) = make_uint2(pack_bf16x2(bf16_lo(q4.x) * acc[0], bf16_hi(q4.x) * acc[1]),
                                                           pack_bf16x2(bf16_lo(q4.y) * acc[2], bf16_hi(q4.y) * acc[3]));
            }
        }
        __syncthreads();

        // ---- store phase
        {
            uint2 yc[8];
#pragma unroll
            for (int c8 = 0; c8 < 8; ++c8) yc[c8] = *reinterpret_cast<const uint2*>(q_lines + c8 * kQS);
            Words<4> row[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint2 e = yc[2 * p], o = yc[2 * p + 1];
                row[0].w[p] = (e.x & 0xffffu) | (o.x << 16);
                row[1].w[p] = (e.x >> 16) | (o.x & 0xffff0000u);
                row[2].w[p] = (e.y & 0xffffu) | (o.y << 16);
                row[3].w[p] = (e.y >> 16) | (o.y & 0xffff0000u);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t t = ts + 4 * rg + r;
                if (t < t_end) store_words_nt<4>(a.y + col + t * D, row[r]);
            }
        }
    }
}

template <int NKB>
hy_status launch_cp(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    CpArgs a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.h = p.h;
    a.y = static_cast<uint16_t*>(p.y);
    a.L = s.L;
    a.D = s.D;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / kC);
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        // about one workgroup per CU, but tiles of at least 8 iterations so that the history before a tile
        // (K steps of k and v) stays a few percent of its traffic
        int64_t tiles = 256 / (s.B * a.ncb);
        if (tiles < 1) tiles = 1;
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 8 * kT) rows = 8 * kT;
    }
    rows = (rows + kT - 1) / kT * kT;
    if (rows > (s.L + kT - 1) / kT * kT) rows = (s.L + kT - 1) / kT * kT;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb = s.B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel((cp_mfma_kernel<NKB>), dim3((uint32_t)nb), dim3(kThreads), st, a);
}

}  // namespace

bool cp_mfma_supported(const ConvShape& s) {
    return !s.sharded() && s.dtype == HY_BF16 && s.gated && s.D % kC == 0 && s.lh >= 1 && s.lh <= 32 * 5 - 15 &&
           s.L <= 0x7fffffffLL - 2 * kT;
}

hy_status launch_cp_mfma(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    if (!cp_mfma_supported(s)) return HY_ERR_UNSUPPORTED;
    const int nkb = (s.lh + 15 + 31) / 32;  // K = 32 nkb >= lh + 15
    switch (nkb) {
        case 1: return launch_cp<1>(p, s, st);
        case 2: return launch_cp<2>(p, s, st);
        case 3: return launch_cp<3>(p, s, st);
        case 4: return launch_cp<4>(p, s, st);
        case 5: return launch_cp<5>(p, s, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
