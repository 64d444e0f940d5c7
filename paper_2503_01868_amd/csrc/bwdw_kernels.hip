// Backward of the gated convolution for short filters (lh <= 7), bf16, on the data movement of the long-sequence
// forward kernel (sew_kernels.hip): a workgroup of 16 waves owns 256 adjacent channels (512-byte row pieces) and
// walks its stretch of time forwards in chunks of 16 rows, one barrier per chunk; a lane owns 4 channels of one row
// of the chunk (8-byte loads of dy, q, k, v issued three chunks ahead with clamped addresses, 8-byte stores).
//
//     u = k*v, g = dy*q (fp32, exact products of bf16 values)
//     dq[t] = dy[t] * sum_j h[j] u[t-j]              u of the last lh-1 rows: LDS ring with 8 look-back rows
//     du[s] = sum_j h[j] g[s+j], dk = du*v, dv = du*k   g of the next lh-1 rows: LDS ring with 8 look-ahead rows;
//                                                       du of a chunk is formed one chunk late, its k and v wait in
//                                                       registers
//     dh[c][j] += g[t] * u[t-j]                      the same u reads as dq; 4 x lh partial sums per lane
// Arithmetic is the vector-ALU backward's (bwd_kernels.hip): fp32 multiplies and FMA chains in ascending tap order,
// one rounding per stored element.  At the end the 16 lanes that share a channel quartet add their partial filter
// gradients through LDS in row order; the tile's partial goes to the workspace as [tile][D][lh] and dh_reduce_kernel
// sums tiles and the channels of a group (two passes, App. A.4).
// A tile reads lh-1 <= 8 rows of k, v before its start and of dy, q after its end.  A shard of a longer sequence
// (Sec. 4) is the same thing one level up: its first tile finds those rows of k, v in front of row 0, its last tile
// those of dy, q behind row L - 1 (as many as the call says hold data), and a product g[t] u[t-j] is counted by the
// call that owns step t, which is also the rule of the stencil kernel.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

struct BwdWalkArgs {
    const uint16_t* dy;
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* h;
    uint16_t* dq;
    uint16_t* dk;
    uint16_t* dv;
    float* partial;  // [B * tiles_per_seq][D][lh]
    int64_t L, D;
    int64_t skv, sgq, sout;  // elements between batch items in k, v / dy, q / dq, dk, dv
    int32_t hist, fut;       // rows of k, v in front of row 0 / of dy, q behind row L - 1 that hold data
    int32_t lh, group;
    int32_t rows, tiles_per_seq, ncb;
};

constexpr int kWaves = 16;
constexpr int kCh = 256;     // channels per workgroup
constexpr int kRowsC = 16;   // rows per chunk
constexpr int kLook = 8;     // look-back (u) / look-ahead (g) rows kept beside a chunk
constexpr int kRowB = kCh * 4;                      // bytes per staged fp32 row
constexpr int kSlot = (kRowsC + kLook) * kRowB;     // bytes per ring slot

template <int LH, int PF, bool kShard>
__global__ __launch_bounds__(kWaves * 64, 4) void bwd_walk_kernel(BwdWalkArgs a) {
    static_assert(LH >= 1 && LH - 1 <= kLook, "the extra rows must cover the filter");
    // u slot: rows 0..7 = the 8 rows before the chunk, rows 8..23 = the chunk; g slot: rows 0..15 = the chunk,
    // rows 16..23 = the 8 rows after it
    __shared__ __attribute__((aligned(16))) char ring[6 * kSlot];
    char* const uring = ring;
    char* const gring = ring + 3 * kSlot;

    const int tid = threadIdx.x;
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int L32 = (int)a.L;
    const int ts32 = (int)((tile % a.tiles_per_seq) * (int64_t)a.rows);
    const int te32 = (ts32 + a.rows < a.L) ? ts32 + a.rows : L32;
    // one chunk in front of a tile that does not start the sequence (k, v of its last rows), one more chunk behind
    // the tile (dy, q of its first rows; also the iteration that finishes du of the last chunk)
    const int t_old = kShard ? -a.hist : 0;        // oldest row of k, v that holds data
    const int t_end = kShard ? L32 + a.fut : L32;  // one past the newest row of dy, q that holds data
    const bool warm = ts32 > t_old;
    const int tb32 = warm ? ts32 - kRowsC : 0;
    const int nch = (te32 - tb32 + kRowsC - 1) / kRowsC + 1;

    const uint32_t D32 = (uint32_t)a.D;
    const int64_t cblock0 = (int64_t)cb * kCh;
    const int64_t seq0kv = b * a.skv, seq0gq = b * a.sgq, seq0out = b * a.sout;
    const int lr = tid >> 6, lp = tid & 63;          // row of the chunk, quartet of channels
    const uint32_t ld_off = (uint32_t)(cblock0 + 4 * lp);
    const int col = lp * 16;                          // byte offset of this lane's 4 fp32 values in a staged row

    // rows whose values are never used load one 8-byte location per workgroup instead (one cache line per wave)
    const int64_t idle_off = (int64_t)((uint64_t)(uint32_t)(te32 - 1) * D32 + (uint32_t)cblock0);
    auto row_of = [&](int ci) { return tb32 + ci * kRowsC + lr; };
    auto load_kv = [&](int ci, Words<2>& kk, Words<2>& vv) {
        const int t = row_of(ci);
        const bool used = ci < nch && t >= ts32 - (LH - 1) && t >= t_old && t < te32;
        const int64_t off = used ? (int64_t)t * (int64_t)D32 + ld_off : idle_off;  // t < 0: a shard's rows in front
        kk = load_words_nt<2>(a.k + seq0kv + off);
        vv = load_words_nt<2>(a.v + seq0kv + off);
    };
    auto load_g = [&](int ci, Words<2>& yy, Words<2>& qq) {
        const int t = row_of(ci);
        const bool used = ci < nch && t >= ts32 && t < te32 + (LH - 1) && t < t_end;
        const int64_t off = used ? (int64_t)t * (int64_t)D32 + ld_off : idle_off;
        yy = load_words_nt<2>(a.dy + seq0gq + off);
        qq = load_words_nt<2>(a.q + seq0gq + off);
    };

    Words<2> kpre[PF], vpre[PF], ypre[PF], qpre[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) {
        load_kv(i, kpre[i], vpre[i]);
        load_g(i, ypre[i], qpre[i]);
    }

    float tap[4][LH], dh[4][LH];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float* hp = a.h + ((cblock0 + 4 * lp + c) / a.group) * (int64_t)LH;
#pragma unroll
        for (int j = 0; j < LH; ++j) {
            tap[c][j] = hp[j];
            dh[c][j] = 0.0f;
        }
    }
    // zeros before a tile that starts the sequence: the look-back rows of the first chunk's slot
    if (!warm) {
        for (int i = tid; i < kLook * kRowB / 16; i += kWaves * 64) reinterpret_cast<uint4*>(uring)[i] = make_uint4(0, 0, 0, 0);
    }

    float kprev[4] = {0.0f, 0.0f, 0.0f, 0.0f}, vprev[4] = {0.0f, 0.0f, 0.0f, 0.0f};

    for (int base = 0; base < nch; base += PF) {
#pragma unroll
        for (int sgi = 0; sgi < PF; ++sgi) {
            const int ci = base + sgi;
            const int slot = ci % 3;
            const int nslot = slot == 2 ? 0 : slot + 1;
            const int pslot = slot == 0 ? 2 : slot - 1;
            const int t = row_of(ci);
            float kf[4], vf[4], yf[4], qf[4], uf[4], gf[4];
            Pack<BF16, 4>::unpack(kpre[sgi], kf);
            Pack<BF16, 4>::unpack(vpre[sgi], vf);
            Pack<BF16, 4>::unpack(ypre[sgi], yf);
            Pack<BF16, 4>::unpack(qpre[sgi], qf);
            // what lies outside the sequence, or outside what this tile may use, is zero
            const bool u_ok = ci < nch && t >= t_old && t < te32;
            const bool g_ok = ci < nch && t >= ts32 && t < t_end;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uf[c] = u_ok ? kf[c] * vf[c] : 0.0f;
                gf[c] = g_ok ? yf[c] * qf[c] : 0.0f;
            }
            {
                const float4 u4 = make_float4(uf[0], uf[1], uf[2], uf[3]);
                const float4 g4 = make_float4(gf[0], gf[1], gf[2], gf[3]);
                *reinterpret_cast<float4*>(uring + slot * kSlot + (kLook + lr) * kRowB + col) = u4;
                if (lr >= kRowsC - kLook)  // whole waves: the chunk's last 8 rows are the next chunk's look-back rows
                    *reinterpret_cast<float4*>(uring + nslot * kSlot + (lr - (kRowsC - kLook)) * kRowB + col) = u4;
                *reinterpret_cast<float4*>(gring + slot * kSlot + lr * kRowB + col) = g4;
                if (lr < kLook)  // the chunk's first 8 rows are the previous chunk's look-ahead rows
                    *reinterpret_cast<float4*>(gring + pslot * kSlot + (kRowsC + lr) * kRowB + col) = g4;
            }
            load_kv(ci + PF, kpre[sgi], vpre[sgi]);
            load_g(ci + PF, ypre[sgi], qpre[sgi]);

            __syncthreads();

            // dq and the filter-gradient partials of this chunk's row
            if (ci < nch && t >= ts32 && t < te32) {
                const char* up = uring + slot * kSlot + (kLook + lr) * kRowB + col;
                float z[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    z[c] = tap[c][0] * uf[c];
                    dh[c][0] = __builtin_fmaf(gf[c], uf[c], dh[c][0]);
                }
#pragma unroll
                for (int j = 1; j < LH; ++j) {
                    const float4 w4 = *reinterpret_cast<const float4*>(up - j * kRowB);
                    const float wv[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        z[c] = __builtin_fmaf(tap[c][j], wv[c], z[c]);
                        dh[c][j] = __builtin_fmaf(gf[c], wv[c], dh[c][j]);
                    }
                }
                float o[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = yf[c] * z[c];
                store_words_nt<2>(a.dq + seq0out + ((uint64_t)(uint32_t)t * D32 + ld_off), Pack<BF16, 4>::pack(o));
            }
            // du, dk, dv of the previous chunk's row: its g rows and the 8 after them are in the previous slot now
            const int tp = t - kRowsC;
            if (ci >= 1 && ci <= nch && tp >= ts32 && tp < te32) {
                const char* gp = gring + pslot * kSlot + lr * kRowB + col;
                float du[4];
                {
                    const float4 w4 = *reinterpret_cast<const float4*>(gp);
                    du[0] = tap[0][0] * w4.x; du[1] = tap[1][0] * w4.y; du[2] = tap[2][0] * w4.z; du[3] = tap[3][0] * w4.w;
                }
#pragma unroll
                for (int j = 1; j < LH; ++j) {
                    const float4 w4 = *reinterpret_cast<const float4*>(gp + j * kRowB);
                    du[0] = __builtin_fmaf(tap[0][j], w4.x, du[0]);
                    du[1] = __builtin_fmaf(tap[1][j], w4.y, du[1]);
                    du[2] = __builtin_fmaf(tap[2][j], w4.z, du[2]);
                    du[3] = __builtin_fmaf(tap[3][j], w4.w, du[3]);
                }
                float o1[4], o2[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    o1[c] = du[c] * vprev[c];
                    o2[c] = du[c] * kprev[c];
                }
                const uint64_t off = (uint64_t)(uint32_t)tp * D32 + ld_off;
                store_words_nt<2>(a.dk + seq0out + off, Pack<BF16, 4>::pack(o1));
                store_words_nt<2>(a.dv + seq0out + off, Pack<BF16, 4>::pack(o2));
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                kprev[c] = kf[c];
                vprev[c] = vf[c];
            }
        }
    }

    // ---- add the partial filter gradients of the 16 rows-lanes that share a channel quartet, in row order
    __syncthreads();  // all reads of the rings are done
    float* red = reinterpret_cast<float*>(ring);  // [lr][lp][4 * LH]
    constexpr int NV = 4 * LH;
    static_assert(kWaves * 64 * NV * 4 <= 6 * kSlot, "the partial sums must fit the rings");
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int j = 0; j < LH; ++j) red[(lr * 64 + lp) * NV + c * LH + j] = dh[c][j];
    __syncthreads();
    float* out = a.partial + ((int64_t)tile * a.D + cblock0 + 4 * lp) * LH;
    for (int idx = lr; idx < NV; idx += kWaves) {
        float s = 0.0f;
#pragma unroll
        for (int r = 0; r < kWaves; ++r) s += red[(r * 64 + lp) * NV + idx];
        out[idx] = s;  // idx = c * LH + j: channel 4 lp + c, tap j
    }
}

int64_t walk_rows(const BwdShape& s) {
    const int64_t ncb = s.D / kCh;
    int64_t rows = tuning().se_rows;
    if (rows <= 0) {
        int64_t tiles = 256 / (s.B * ncb);  // one workgroup per CU
        if (tiles < 1) tiles = 1;
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 8 * kRowsC) rows = 8 * kRowsC;
    }
    rows = (rows + kRowsC - 1) / kRowsC * kRowsC;
    const int64_t cap = (s.L + kRowsC - 1) / kRowsC * kRowsC;
    return rows > cap ? cap : rows;
}

template <int LH>
hy_status launch_walk_lh(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    constexpr int PF = LH >= 7 ? 2 : 3;  // chunks in flight per lane; the longest filters leave registers for two
    BwdWalkArgs a;
    a.dy = static_cast<const uint16_t*>(p.dy);
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.h = p.h;
    a.dq = static_cast<uint16_t*>(p.dq);
    a.dk = static_cast<uint16_t*>(p.dk);
    a.dv = static_cast<uint16_t*>(p.dv);
    a.partial = static_cast<float*>(ws);
    a.L = s.L;
    a.D = s.D;
    a.skv = s.stride_kv();
    a.sgq = s.stride_gq();
    a.sout = s.stride_out();
    a.hist = s.history;
    a.fut = s.future;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / kCh);
    a.rows = (int32_t)walk_rows(s);
    a.tiles_per_seq = (int32_t)((s.L + a.rows - 1) / a.rows);
    const int64_t nsets = s.B * a.tiles_per_seq;
    const int64_t nb = nsets * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    const hy_status rc = s.sharded()
        ? launch_kernel((bwd_walk_kernel<LH, PF, true>), dim3((uint32_t)nb), dim3(kWaves * 64), st, a)
        : launch_kernel((bwd_walk_kernel<LH, PF, false>), dim3((uint32_t)nb), dim3(kWaves * 64), st, a);
    if (rc != HY_OK) return rc;
    return launch_dh_reduce(static_cast<const float*>(ws), p.dh, nsets, s.D, s.lh, s.group, st);
}

}  // namespace

// bf16, lh <= 7 (eight taps do not fit 128 registers beside two chunks of loads), whole 256-channel blocks, and a
// stretch of at least 256 steps per workgroup to walk
bool bwd_walk_preferred(const BwdShape& s) {
    if (!s.gated || s.dtype != HY_BF16 || s.lh < 1 || s.lh > 7 || s.D % kCh != 0) return false;
    if (s.L > 0x7fff0000LL || s.D > 0x7fff0000LL) return false;
    const int force = tuning().se_walk;
    if (force == 1) return true;
    if (force == 2) return false;
    int64_t tiles = 256 / (s.B * (s.D / kCh));
    if (tiles < 1) tiles = 1;
    return (s.L + tiles - 1) / tiles >= 256;
}

int64_t bwd_walk_workspace_bytes(const BwdShape& s) {
    const int64_t rows = walk_rows(s);
    const int64_t tiles = (s.L + rows - 1) / rows;
    return s.B * tiles * s.D * s.lh * (int64_t)sizeof(float);
}

hy_status launch_bwd_walk(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    switch (s.lh) {
        case 1: return launch_walk_lh<1>(p, s, ws, st);
        case 2: return launch_walk_lh<2>(p, s, ws, st);
        case 3: return launch_walk_lh<3>(p, s, ws, st);
        case 4: return launch_walk_lh<4>(p, s, ws, st);
        case 5: return launch_walk_lh<5>(p, s, ws, st);
        case 6: return launch_walk_lh<6>(p, s, ws, st);
        case 7: return launch_walk_lh<7>(p, s, ws, st);
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
