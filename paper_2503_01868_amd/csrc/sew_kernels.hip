// Hyena-SE forward for long sequences: the same gated short FIR as se_kernels.hip (Eq. 1 / Eq. 2, fp32
// arithmetic, one rounding at the store), on the data-movement skeleton of the Hyena-MR kernel.
//
// Why a second kernel: on MI355X the MR kernel's way of moving data -- one workgroup of 16 waves per CU that owns
// 256 channels (512-byte row pieces) and walks thousands of time steps in 32-row chunks, every lane loading one
// 16-byte piece of k, v and q per chunk two chunks ahead -- sustains 6.1-6.2 TB/s once the sequence is long
// (B*L >= 32K at D = 4096), while the register-delay-line stencil of se_kernels.hip, with its many short tiles,
// stays at 5.3-5.5 TB/s.  At B*L = 8192 the stencil wins (less halo, shorter ramp), so the dispatcher picks by size.
//
// Per chunk: a lane multiplies its k and v pieces (8 channels of one row) and writes u as fp32 into an LDS ring of
// three slots; every slot carries 8 look-back rows (the last rows of the chunk before it) in front of its 32 rows,
// written by the lanes that own those rows, so a lane's FIR window (rows r-lh+1..r of its own 8 channels) never
// straddles slots.  After one barrier the lane reads that window (lh x 32 bytes), runs the lh-tap FMA chain with
// its taps in registers, gates with the q piece it loaded itself and stores 16 bytes.  Three slots make the single
// barrier per chunk sufficient: chunk c+1 writes slot (c+1)%3 and the look-back rows of slot (c+2)%3, never the
// slot chunk c is still being read from.
//
// GATED = false is the featurizer convolution of Eq. 1 (x' = h * x, no gates) on the same skeleton: u is the input
// itself (the k pointer), nothing is read for v and q, and blockIdx.y selects one of up to three independent
// problems (q, k, v of the operator chain each with its own filter), so that the three featurizers are one launch.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

struct SewArgs {
    const uint16_t* q;
    const uint16_t* k[3];  // per problem (gated: one problem)
    const uint16_t* v;
    const float* h[3];
    uint16_t* y[3];
    int64_t L, D;
    int64_t bstride_kv, bstride_qy;  // elements between batch items in k, v / in q, y
    int32_t hist;           // rows of k and v in front of row 0 that hold data: 0 or >= kLook
    int32_t lh, group;
    int32_t rows;           // time steps per workgroup, multiple of 32
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / (16 NW)
};

constexpr int kChunk = 32;
constexpr int kLook = 8;  // look-back rows per slot, >= lh - 1

template <int LH, int NW, int kPrefetch, bool GATED>
__global__ __launch_bounds__(NW * 64, NW == 16 ? 4 : 2) void se_walk_kernel(SewArgs a) {
    static_assert(LH >= 1 && LH - 1 <= kLook, "the look-back rows must cover the filter");
    constexpr int PPR = 2 * NW;                 // 16-byte pieces of bf16 per row = lanes per row
    constexpr int ROWB = 16 * NW * 4;           // bytes per staged row of u (fp32)
    constexpr int SLOT = (kLook + kChunk) * ROWB;
    __shared__ __attribute__((aligned(16))) char ring[3 * SLOT];

    const int tid = threadIdx.x;
    const uint32_t lb = blockIdx.x;
    const int pi = GATED ? 0 : (int)blockIdx.y;
    const uint16_t* const kp = a.k[pi];
    const float* const hp0 = a.h[pi];
    uint16_t* const yp = a.y[pi];
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int ts32 = (int)((tile % a.tiles_per_seq) * (int64_t)a.rows);
    const int te32 = (ts32 + a.rows < a.L) ? ts32 + a.rows : (int)a.L;
    // one warm-up chunk in front of a tile that does not start the sequence; only its last 8 rows are real loads
    const bool warm = ts32 > 0 || a.hist > 0;
    const int tb32 = warm ? ts32 - kChunk : 0;
    const int nchunks = (te32 - tb32 + kChunk - 1) / kChunk;

    const int64_t D = a.D;
    const uint32_t D32 = (uint32_t)D;
    const int64_t cblock0 = (int64_t)cb * 16 * NW;
    const int64_t seq0 = b * a.bstride_qy, seq0kv = b * a.bstride_kv;
    const int lr = tid / PPR, lp = tid % PPR;
    const uint32_t ld_off = (uint32_t)(cblock0 + 8 * lp);
    const int t_lo = warm ? ts32 - kLook : 0;  // oldest row ever needed

    // unconditional, clamped loads: rows past the end of the tile re-read its last row; loads whose result is never
    // used (rows before the needed history, chunk indices past the last chunk, q of the warm-up chunk) all go to one
    // 16-byte location of the tile, the same for every lane of the workgroup (one cache line per wave; see
    // mr_kernels.hip)
    const uint64_t idle_off = (uint64_t)(uint32_t)(te32 - 1) * D32 + (uint32_t)cblock0;
    auto load_kv = [&](int ci, Words<4>& kk, Words<4>& vv) {
        int t = tb32 + ci * kChunk + lr;
        const bool used = ci < nchunks && t >= t_lo;
        t = t < te32 ? t : te32 - 1;
        const int64_t off = used ? (int64_t)t * (int64_t)D32 + ld_off : (int64_t)idle_off;
        kk = load_words_nt<4>(kp + seq0kv + off);
        if constexpr (GATED) vv = load_words_nt<4>(a.v + seq0kv + off);
    };
    auto load_q = [&](int ci, Words<4>& qq) {
        int t = tb32 + ci * kChunk + lr;
        const bool used = ci < nchunks && t >= ts32;
        t = t < te32 ? t : te32 - 1;
        qq = load_words_nt<4>(a.q + seq0 + (used ? (uint64_t)(uint32_t)t * D32 + ld_off : idle_off));
    };

    Words<4> kpre[kPrefetch], vpre[kPrefetch], qpre[kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) {
        load_kv(i, kpre[i], vpre[i]);
        if constexpr (GATED) load_q(i, qpre[i]);
    }

    // taps of this lane's 8 channels
    float tap[8][LH];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float* hp = hp0 + ((cblock0 + 8 * lp + c) / a.group) * (int64_t)LH;
#pragma unroll
        for (int j = 0; j < LH; ++j) tap[c][j] = hp[j];
    }

    // a tile that starts the sequence has zeros before it: clear the look-back rows of slot 0
    if (!warm) {
        for (int i = tid; i < kLook * ROWB / 16; i += NW * 64)
            reinterpret_cast<uint4*>(ring)[i] = make_uint4(0, 0, 0, 0);
    }

    const int lane_col = lp * 32;  // byte offset of this lane's 8 fp32 values inside a staged row

    for (int base = 0; base < nchunks; base += kPrefetch) {
#pragma unroll
        for (int sgi = 0; sgi < kPrefetch; ++sgi) {
            const int ci = base + sgi;
            const int slot = ci % 3;
            const int nslot = slot == 2 ? 0 : slot + 1;
            // u = k * v (fp32) -> this chunk's slot, and, for the chunk's last 8 rows, the next slot's look-back rows
            float uf[8];
            {
                float kf[8], vf[8];
                Pack<BF16, 8>::unpack(kpre[sgi], kf);
                if constexpr (GATED) {
                    Pack<BF16, 8>::unpack(vpre[sgi], vf);
#pragma unroll
                    for (int c = 0; c < 8; ++c) uf[c] = kf[c] * vf[c];
                } else {
#pragma unroll
                    for (int c = 0; c < 8; ++c) uf[c] = kf[c];
                }
            }
            {
                char* p = ring + slot * SLOT + (kLook + lr) * ROWB + lane_col;
                *reinterpret_cast<float4*>(p) = make_float4(uf[0], uf[1], uf[2], uf[3]);
                *reinterpret_cast<float4*>(p + 16) = make_float4(uf[4], uf[5], uf[6], uf[7]);
                if (lr >= kChunk - kLook) {  // whole waves
                    char* pn = ring + nslot * SLOT + (lr - (kChunk - kLook)) * ROWB + lane_col;
                    *reinterpret_cast<float4*>(pn) = make_float4(uf[0], uf[1], uf[2], uf[3]);
                    *reinterpret_cast<float4*>(pn + 16) = make_float4(uf[4], uf[5], uf[6], uf[7]);
                }
            }
            load_kv(ci + kPrefetch, kpre[sgi], vpre[sgi]);

            __syncthreads();

            const int t = tb32 + ci * kChunk + lr;
            if (ci < nchunks && t >= ts32 && t < te32) {  // the warm-up chunk and rows past the end produce no output
                float z[8];
#pragma unroll
                for (int c = 0; c < 8; ++c) z[c] = tap[c][0] * uf[c];
                const char* p = ring + slot * SLOT + (kLook + lr) * ROWB + lane_col;
#pragma unroll
                for (int j = 1; j < LH; ++j) {
                    const float4 wa = *reinterpret_cast<const float4*>(p - j * ROWB);
                    const float4 wb = *reinterpret_cast<const float4*>(p - j * ROWB + 16);
                    z[0] = __builtin_fmaf(tap[0][j], wa.x, z[0]);
                    z[1] = __builtin_fmaf(tap[1][j], wa.y, z[1]);
                    z[2] = __builtin_fmaf(tap[2][j], wa.z, z[2]);
                    z[3] = __builtin_fmaf(tap[3][j], wa.w, z[3]);
                    z[4] = __builtin_fmaf(tap[4][j], wb.x, z[4]);
                    z[5] = __builtin_fmaf(tap[5][j], wb.y, z[5]);
                    z[6] = __builtin_fmaf(tap[6][j], wb.z, z[6]);
                    z[7] = __builtin_fmaf(tap[7][j], wb.w, z[7]);
                }
                if constexpr (GATED) {
                    float qf[8];
                    Pack<BF16, 8>::unpack(qpre[sgi], qf);
#pragma unroll
                    for (int c = 0; c < 8; ++c) z[c] *= qf[c];
                }
                store_words_nt<4>(yp + seq0 + ((uint64_t)(uint32_t)t * D32 + ld_off), Pack<BF16, 8>::pack(z));
            }
            if constexpr (GATED) load_q(ci + kPrefetch, qpre[sgi]);
        }
    }
}

// Tiles per sequence: one workgroup per compute unit, rounds of 256 kept full (three featurizers at B = 4: 192
// workgroups on 256 compute units ran slower than the stencil, 768 run faster); a tile keeps 1024 steps.
int64_t walk_tiles(int64_t base, int64_t L) { return tiles_filling_rounds(base, L, 1024); }

template <int LH, int NW>
hy_status launch_sew_nw(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    constexpr int PF = 2;
    SewArgs a;
    a.q = static_cast<const uint16_t*>(p[0].q);
    a.v = static_cast<const uint16_t*>(p[0].v);
    for (int i = 0; i < 3; ++i) {
        const ConvPtrs& pp = p[i < nprob ? i : 0];
        a.k[i] = static_cast<const uint16_t*>(pp.k);
        a.h[i] = pp.h;
        a.y[i] = static_cast<uint16_t*>(pp.y);
    }
    a.L = s.L;
    a.D = s.D;
    a.bstride_kv = s.stride_kv();
    a.bstride_qy = s.stride_qy();
    a.hist = s.history;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * NW));
    int64_t rows = tuning().se_rows;
    if (rows <= 0) {
        const int64_t tiles = walk_tiles(nprob * s.B * a.ncb, s.L);
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 8 * kChunk) rows = 8 * kChunk;
    }
    rows = (rows + kChunk - 1) / kChunk * kChunk;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb = s.B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    if (s.gated) return launch_kernel((se_walk_kernel<LH, NW, PF, true>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
    return launch_kernel((se_walk_kernel<LH, NW, PF, false>), dim3((uint32_t)nb, (uint32_t)nprob), dim3(NW * 64), st, a);
}

template <int LH>
hy_status launch_sew_lh(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    if (s.D % 256 == 0 && tuning().mr_waves != 8) return launch_sew_nw<LH, 16>(p, nprob, s, st);
    return launch_sew_nw<LH, 8>(p, nprob, s, st);
}

}  // namespace

// The walking kernel pays off once every workgroup has a long stretch of time to walk.
bool se_walk_preferred(const ConvShape& s, int nprob) {
    if (s.dtype != HY_BF16 || s.lh < 1 || s.lh > 8 || s.D % 128 != 0) return false;
    if (nprob < 1 || nprob > 3 || (s.gated && nprob != 1)) return false;
    if (s.history != 0 && s.history < kLook) return false;  // a halo shorter than the look-back rows: the stencil's case
    if (s.L > 0x7fff0000LL || s.D > 0x7fff0000LL) return false;
    const int force = tuning().se_walk;
    if (force == 1) return true;
    if (force == 2) return false;
    // Measured at D = 4096, B = 1: the stencil wins at L = 8192 (512 steps per workgroup), the walker from
    // L = 16384 on (1024 steps per workgroup); short batch items never give a workgroup a long walk.
    const int nw = (s.D % 256 == 0 && tuning().mr_waves != 8) ? 16 : 8;
    const int64_t tiles = walk_tiles(nprob * s.B * (s.D / (16 * nw)), s.L);
    return (s.L + tiles - 1) / tiles >= 1024;
}

hy_status launch_se_walk(const ConvPtrs* p, int nprob, const ConvShape& s, hipStream_t st) {
    if (nprob < 1 || nprob > 3 || (s.gated && nprob != 1)) return HY_ERR_UNSUPPORTED;
    switch (s.lh) {
        case 1: return launch_sew_lh<1>(p, nprob, s, st);
        case 2: return launch_sew_lh<2>(p, nprob, s, st);
        case 3: return launch_sew_lh<3>(p, nprob, s, st);
        case 4: return launch_sew_lh<4>(p, nprob, s, st);
        case 5: return launch_sew_lh<5>(p, nprob, s, st);
        case 6: return launch_sew_lh<6>(p, nprob, s, st);
        case 7: return launch_sew_lh<7>(p, nprob, s, st);
        case 8: return launch_sew_lh<8>(p, nprob, s, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
