// Backward of the gated convolution for filters that are NOT shared by 16 channels (one filter per channel or
// per small group), on the gfx950 matrix cores: the chunk-parallel scheme of App. A.1 applied to the backward
// structure of App. A.4.  With u = k*v, g = dy*q:
//     dq = dy (.) (h * u)                 the forward chunk-parallel kernel (cp4_kernels.hip) on (dy, k, v)
//     dk = v (.) (h *' g), dv = k (.) (h *' g),  (h *' g)[s] = sum_j h[j] g[s+j]
//                                         the same kernel walking time backwards, once per output (filters of
//                                         66 taps and more: once, with two post-gates and two outputs)
//     dh[c, j] = sum_{b, t} g[b,t,c] u[b,t-j,c]        this file: a per-channel correlation
//
// The correlation as batched 4 x 4 x 4 products (v_mfma_f32_4x4x4_16B_bf16: 16 independent blocks per
// instruction, one channel per block).  For a group of 4 steps starting at T (a multiple of 4) and lag block a:
//     D_a[i][r] += sum_k A[i][k] * B_a[k][r],   A[i][k] = g[T + i + k],   B_a[k][r] = u[T + k - 4 r - 16 a],
// so that entry (i, r) of accumulator a collects g[t] u[t - j] for the lag j = 16 a + 4 r + i over all t = T+i+k.
// B_a is four aligned 4-step pieces of the channel's u line (one 8-byte LDS read per lane, as in the forward
// kernel), and B_a of the group at T is B_0 of the group at T - 16 a: every operand is read from LDS once, as B_0
// of its group, and then stays in a register window of the last 4 (NA - 1) + 1 groups until its last lag block has
// used it (reading all NA operands per group from LDS made the LDS pipe the limit of this kernel).  A is a Hankel
// block of g whose rows start at consecutive steps, read as three aligned dwords and
// shifted by 16 bits in the odd rows.  Every (t, j) pair is produced exactly once, row i of a tile covering the
// steps [t0, t1) of T + k taking the g of [t0 + i, t1 + i): tiles partition the sum and need 3 steps of dy, q past
// their end and lh - 1 steps of k, v before their start.  The accumulators (4 registers per lag block) stay in
// registers for the whole tile and leave as dh[c][16 a + 4 r .. + 3], four adjacent floats per lane: the partial
// filter gradient of the tile, written out contiguously and reduced over tiles (and the channels of a group) by
// dh_reduce_kernel, the two-pass structure of App. A.4.
//
// A shard of a longer sequence (Sec. 4) is one more cut of the same kind: a call whose dy, q go on behind row
// L - 1 and whose k, v begin before row 0 counts the pair (t, j) when step t - (j mod 4) is one of its own, reads
// up to 3 of the rows behind it and up to lh - 1 of the rows in front, and the shares of all shards add up to the
// full gradient.  Where the call's last step is not the last step of a 4-step group, the entries of A that belong
// to the steps behind it are masked out (their g is real data there, not zeros).
//
// Data movement: 8 waves per 128 channels; per iteration of 64 steps every lane loads two rows x 8 channels of
// dy, q, k, v (16-byte pieces, one iteration ahead; two ahead do not fit the registers beside the operand
// window), forms g and u, rounds them to bf16 and writes them transposed into per-channel [time] lines in LDS
// (rings of 4 x 64 steps); the products of an iteration run one iteration late, when the 3 look-ahead steps of g
// are there.
#include <type_traits>

#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct Cp4DhArgs {
    const uint16_t* dy;
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    float* partial;  // [B * tiles_per_seq][D][lh]
    int64_t L, D;
    int64_t skv, sgq;  // elements between batch items in k, v / in dy, q
    int32_t hist, fut;  // rows of k, v in front of row 0 / of dy, q behind row L - 1 that hold data
    int32_t lh;
    int32_t rows;           // time steps per workgroup, multiple of 64
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / 128
};

constexpr int kT = 64;      // steps per iteration
constexpr int kNW = 8;      // waves per workgroup
constexpr int kC = 16 * kNW;  // channels per workgroup
constexpr int kRing = 256;  // ring length in steps (4 slots)
constexpr int kLine = 544;  // bytes per ring line: 256 steps, 4 steps of wrap-around copy, padding (8 banks per channel)

// NA = lag blocks of 16 = ceil(lh / 16)
template <int NA, bool kShard>
__global__ __launch_bounds__(kNW * 64, 1) void cp4_dh_kernel(Cp4DhArgs a) {
    constexpr int PPR = kC / 8;  // 16-byte pieces per row
    static_assert(kNW * 64 == PPR * (kT / 2), "one lane per (row pair, piece)");
    static_assert(16 * NA + 12 <= kRing - kT, "the lags must fit the ring behind the current slot");
    // every block of 8 channels starts 8 bytes further than the line stride puts it (bank spreading of the
    // transposing 4-byte writes)
    __shared__ __attribute__((aligned(16))) char uring[kC * kLine + (kC / 8) * 8];
    __shared__ __attribute__((aligned(16))) char gring[kC * kLine + (kC / 8) * 8];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int ts32 = (int)((tile % a.tiles_per_seq) * (int64_t)a.rows);
    const int te32 = (ts32 + a.rows < a.L) ? ts32 + a.rows : (int)a.L;
    const int L32 = (int)a.L;
    const int nit = (te32 - ts32 + kT - 1) / kT;  // iteration it = 1..nit holds steps ts32 + 64 (it - 1) ...

    const uint32_t D32 = (uint32_t)a.D;
    const int64_t cblock0 = (int64_t)cb * kC;
    const int64_t seq0kv = b * a.skv, seq0gq = b * a.sgq;
    const int t_old = kShard ? -a.hist : 0;       // oldest step of k, v that holds data
    const int t_end = kShard ? L32 + a.fut : L32;  // one past the newest step of dy, q that holds data
    auto line_off = [](int c, int stride) { return c * stride + (c >> 3) * 8; };

    // ---- row layout: rows 2 rp, 2 rp + 1 of an iteration, channels 8 lp .. 8 lp + 7 of the block
    const int lp = tid % PPR, rp = tid / PPR;
    const uint32_t ld_off = (uint32_t)(cblock0 + 8 * lp);
    char* const u_lines = uring + line_off(8 * lp, kLine) + 4 * rp;
    char* const g_lines = gring + line_off(8 * lp, kLine) + 4 * rp;

    // rows are clamped into what holds data; what lies outside it is zeroed when it is written to LDS
    auto row_kv = [&](int t) {
        t = t < L32 ? t : L32 - 1;
        t = t > t_old ? t : t_old;
        return seq0kv + ((int64_t)t * (int64_t)D32 + ld_off);
    };
    auto row_gq = [&](int t) {
        t = t < t_end ? t : t_end - 1;
        t = t > 0 ? t : 0;
        return seq0gq + ((int64_t)t * (int64_t)D32 + ld_off);
    };
    // x = a*b of 2 rows x 8 channels, transposed: one dword (2 steps) per channel at ring position `pos` + 2 rp
    auto write_prod = [&](char* lines, const Words<4> (&aa)[2], const Words<4> (&bb)[2], bool keep0, bool keep1, int pos) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float a0 = keep0 ? bf16_lo(aa[0].w[p]) * bf16_lo(bb[0].w[p]) : 0.0f;
            const float b0 = keep0 ? bf16_hi(aa[0].w[p]) * bf16_hi(bb[0].w[p]) : 0.0f;
            const float a1 = keep1 ? bf16_lo(aa[1].w[p]) * bf16_lo(bb[1].w[p]) : 0.0f;
            const float b1 = keep1 ? bf16_hi(aa[1].w[p]) * bf16_hi(bb[1].w[p]) : 0.0f;
            *reinterpret_cast<uint32_t*>(lines + (2 * p) * kLine + pos * 2) = pack_bf16x2(a0, a1);
            *reinterpret_cast<uint32_t*>(lines + (2 * p + 1) * kLine + pos * 2) = pack_bf16x2(b0, b1);
        }
    };

    constexpr int PF = 1;  // iterations of loads in flight; register stage it % PF holds the rows of iteration it
    Words<4> yw[PF][2], qw[PF][2], kw[PF][2], vw[PF][2];
    auto load_rows = [&](auto st_c, int it) {  // iteration it >= 1; one past the last iteration only its first rows matter
        constexpr int ST = decltype(st_c)::value;
        const int t0 = ts32 + (it - 1) * kT + 2 * rp;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int64_t off = row_kv(t0 + r), offg = row_gq(t0 + r);
            yw[ST][r] = load_words_nt<4>(a.dy + offg);
            qw[ST][r] = load_words_nt<4>(a.q + offg);
            kw[ST][r] = load_words_nt<4>(a.k + off);
            vw[ST][r] = load_words_nt<4>(a.v + off);
        }
    };

    // ---- history of u: the steps ts32 - 128 .. ts32 - 1 go to ring slots 3 and 0 (iteration it uses slot it & 3);
    // steps before the oldest row that holds data are zeros
    {
        Words<4> kh[2][2], vh[2][2];
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            const int t0 = ts32 - 2 * kT + hb * kT + 2 * rp;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int64_t off = row_kv(t0 + r);
                kh[hb][r] = load_words_nt<4>(a.k + off);
                vh[hb][r] = load_words_nt<4>(a.v + off);
            }
        }
        load_rows(std::integral_constant<int, 1 % PF>{}, 1);
        if constexpr (PF == 2) load_rows(std::integral_constant<int, 0>{}, 2);
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            const int t0 = ts32 - 2 * kT + hb * kT + 2 * rp;
            write_prod(u_lines, kh[hb], vh[hb], t0 >= t_old, t0 + 1 >= t_old, hb == 0 ? 3 * kT : 0);
        }
    }

    // ---- matrix-phase lane constants: block blk = channel, row / column index l4
    const int blk = lane >> 2, l4 = lane & 3;
    const int cw = 16 * w + blk;
    const char* const ul = uring + line_off(cw, kLine);
    const char* const gl = gring + line_off(cw, kLine) + 4 * (l4 >> 1);  // dword that holds step l4 (rounded down to even)
    const bool odd = (l4 & 1) != 0;
    const char* const u_lane = ul - 8 * l4;                              // column r = l4 reads 4 r steps further back
    const char* const u_mix0 = ul + 2 * ((0 - 4 * l4 + kRing) % kRing);  // positions that wrap for some lanes
    const char* const u_mix4 = ul + 2 * ((4 - 4 * l4 + kRing) % kRing);
    const char* const u_mix8 = ul + 2 * ((8 - 4 * l4 + kRing) % kRing);

    f32x4_t acc[NA];
#pragma unroll
    for (int x = 0; x < NA; ++x) acc[x] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // B_0 of the group at ring position 4 i sits in win[i]; all indices are compile-time constants, an entry is
    // dead 4 (NA - 1) groups after it was read
    constexpr int kWin = kRing / 4;
    s16x4_t win[kWin];
    auto read_b0 = [&](int c0) {  // ring position of column 0, a constant after unrolling
        const char* p;
        if (c0 >= 12) p = u_lane + 2 * c0;
        else if (c0 == 0) p = u_mix0;
        else if (c0 == 4) p = u_mix4;
        else p = u_mix8;
        const uint2 bw = *reinterpret_cast<const uint2*>(p);
        Words<2> bb;
        bb.w[0] = bw.x; bb.w[1] = bw.y;
        win[c0 / 4] = __builtin_bit_cast(s16x4_t, bb);
    };
    // the 4 (NA - 1) groups before ring position kT (the first iteration's), for its first products
    auto fill_history = [&]() {
        static_assert(4 * (NA - 1) <= 2 * (kT / 4), "the history lies in the two slots before the first iteration's");
#pragma unroll
        for (int i = 0; i < 4 * (NA - 1); ++i) read_b0((kT - 4 * (i + 1) + kRing) % kRing);
    };

    // one group of 4 steps whose first step sits at ring position P (a constant after unrolling); `rem` = steps from
    // there to the end of the tile (only a shard's last tile can end inside a group with real g behind it)
    auto group = [&](int P, int rem) {
        read_b0(P);
        // A: g[T + l4 .. T + l4 + 3], T at position P; the line carries a copy of positions 0..3 behind position 255,
        // so the window never wraps
        const char* gp = gl + 2 * P;
        const uint32_t d0 = *reinterpret_cast<const uint32_t*>(gp);
        const uint32_t d1 = *reinterpret_cast<const uint32_t*>(gp + 4);
        const uint32_t d2 = *reinterpret_cast<const uint32_t*>(gp + 8);
        Words<2> aw;
        aw.w[0] = odd ? __builtin_amdgcn_alignbit(d1, d0, 16) : d0;
        aw.w[1] = odd ? __builtin_amdgcn_alignbit(d2, d1, 16) : d1;
        if constexpr (kShard) {  // column k of A belongs to step T + k: keep it while that step is the tile's
            aw.w[0] &= rem >= 2 ? 0xffffffffu : (rem == 1 ? 0x0000ffffu : 0u);
            aw.w[1] &= rem >= 4 ? 0xffffffffu : (rem == 3 ? 0x0000ffffu : 0u);
        }
        const s16x4_t av = __builtin_bit_cast(s16x4_t, aw);
#pragma unroll
        for (int x = 0; x < NA; ++x)
            acc[x] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(av, win[((P - 16 * x + 4 * kRing) % kRing) / 4], acc[x], 0, 0, 0);
    };

    // products of the iteration whose first step sits at ring position WB; `left` = steps from there to the tile's end
    auto products = [&](auto wb_c, int left) {
        constexpr int WB = decltype(wb_c)::value;
#pragma unroll
        for (int n = 0; n < kT / 4; ++n) group(WB + 4 * n, left - 4 * n);
    };

    // iteration `it` (1 .. nit + 1): its rows go to ring slot it & 3; then the products of iteration it - 1
    auto step = [&](auto slot_c, int it) {
        constexpr int SL = decltype(slot_c)::value;  // it & 3
        constexpr int WB = kT * SL;
        constexpr int ST = SL % PF;
        {
            const int t = ts32 + (it - 1) * kT + 2 * rp;
            write_prod(u_lines, kw[ST], vw[ST], t < L32, t + 1 < L32, WB);
            write_prod(g_lines, yw[ST], qw[ST], t < t_end, t + 1 < t_end, WB);
            if constexpr (SL == 0) {  // positions 0..3 once more behind position 255 (read windows do not wrap)
                if (rp < 2) write_prod(g_lines, yw[ST], qw[ST], t < t_end, t + 1 < t_end, kRing);
            }
        }
        if (it + PF - 1 <= nit) load_rows(std::integral_constant<int, ST>{}, it + PF);
        __syncthreads();
        if constexpr (SL == 2) {
            if (it == 2) fill_history();  // the first products: iteration 1, ring slot 1
        }
        if (it >= 2) products(std::integral_constant<int, kT * ((SL + 3) & 3)>{}, te32 - (ts32 + (it - 2) * kT));
        __syncthreads();
    };
    using std::integral_constant;
    for (int it = 1; it <= nit + 1; it += 4) {
        step(integral_constant<int, 1>{}, it);
        if (it + 1 <= nit + 1) step(integral_constant<int, 2>{}, it + 1);
        if (it + 2 <= nit + 1) step(integral_constant<int, 3>{}, it + 2);
        if (it + 3 <= nit + 1) step(integral_constant<int, 0>{}, it + 3);
    }

    // ---- the lane holds dh[c][16 x + 4 l4 + i], i = 0..3
    float* out = a.partial + ((int64_t)tile * a.D + cblock0 + cw) * a.lh;
#pragma unroll
    for (int x = 0; x < NA; ++x) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = 16 * x + 4 * l4 + i;
            if (j < a.lh) out[j] = acc[x][i];
        }
    }
}

int64_t dh_rows(const BwdShape& s) {
    const int64_t ncb = s.D / kC;
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        const int64_t tiles = tiles_filling_rounds(s.B * ncb, s.L, 4 * kT);  // one workgroup per CU
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 4 * kT) rows = 4 * kT;
    }
    rows = (rows + kT - 1) / kT * kT;
    const int64_t cap = (s.L + kT - 1) / kT * kT;
    return rows > cap ? cap : rows;
}

template <int NA, bool kShard>
hy_status launch_dh_na(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    Cp4DhArgs a;
    a.dy = static_cast<const uint16_t*>(p.dy);
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.partial = static_cast<float*>(ws);
    a.L = s.L;
    a.D = s.D;
    a.skv = s.stride_kv();
    a.sgq = s.stride_gq();
    a.hist = s.history;
    a.fut = s.future;
    a.lh = s.lh;
    a.ncb = (int32_t)(s.D / kC);
    a.rows = (int32_t)dh_rows(s);
    a.tiles_per_seq = (int32_t)((s.L + a.rows - 1) / a.rows);
    const int64_t nsets = s.B * a.tiles_per_seq;
    const int64_t nb = nsets * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    hy_status rc = launch_kernel((cp4_dh_kernel<NA, kShard>), dim3((uint32_t)nb), dim3(kNW * 64), st, a);
    if (rc != HY_OK) return rc;
    return launch_dh_reduce(static_cast<const float*>(ws), p.dh, nsets, s.D, s.lh, s.group, st);
}

}  // namespace

bool cp4_bwd_supported(const BwdShape& s) {
    return s.gated && s.dtype == HY_BF16 && s.D % 128 == 0 && s.lh > 8 && s.lh <= 129 && s.L <= 0x7fff0000LL && s.D <= 0x7fff0000LL;
}

int64_t cp4_bwd_workspace_bytes(const BwdShape& s) {
    const int64_t rows = dh_rows(s);
    const int64_t tiles = (s.L + rows - 1) / rows;
    return s.B * tiles * s.D * s.lh * (int64_t)sizeof(float);
}

hy_status launch_cp4_bwd(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    if (!cp4_bwd_supported(s)) return HY_ERR_UNSUPPORTED;
    // dq: the forward operator on (dy, k, v); dk, dv: the operator towards the past on g = dy*q, gated by v and by k
    // (a shard: dq reaches back into the rows in front of k and v, dk and dv forward into the rows behind dy and q)
    ConvShape fwd{s.B, s.L, s.D, s.lh, s.group, s.dtype, true, false};
    ConvShape rev{s.B, s.L, s.D, s.lh, s.group, s.dtype, true, true};
    if (s.sharded()) {
        fwd.bstride_kv = s.stride_kv();
        fwd.bstride_qy = s.stride_gq();
        fwd.bstride_y = s.stride_out();
        fwd.history = s.history;
        rev.bstride_kv = s.stride_gq();
        rev.bstride_qy = s.stride_kv();
        rev.bstride_y = s.stride_out();
        rev.history = s.future;
    }
    hy_status rc = launch_cp4(ConvPtrs{p.dy, p.k, p.v, p.h, p.dq}, fwd, st);
    if (rc != HY_OK) return rc;
    if (cp4_dual_supported(rev)) {
        // filters of 66 taps and more: dk and dv from one launch with two post-gates
        rc = launch_cp4(ConvPtrs{p.v, p.dy, p.q, p.h, p.dk, p.k, p.dv}, rev, st);
        if (rc != HY_OK) return rc;
    } else {
        rc = launch_cp4(ConvPtrs{p.v, p.dy, p.q, p.h, p.dk}, rev, st);
        if (rc != HY_OK) return rc;
        rc = launch_cp4(ConvPtrs{p.k, p.dy, p.q, p.h, p.dv}, rev, st);
        if (rc != HY_OK) return rc;
    }
    const int na = (s.lh + 15) / 16;
    if (s.sharded()) {
        if (na <= 3) return launch_dh_na<3, true>(p, s, ws, st);
        if (na <= 5) return launch_dh_na<5, true>(p, s, ws, st);
        return launch_dh_na<9, true>(p, s, ws, st);
    }
    if (na <= 3) return launch_dh_na<3, false>(p, s, ws, st);
    if (na <= 5) return launch_dh_na<5, false>(p, s, ws, st);
    return launch_dh_na<9, false>(p, s, ws, st);
}

}  // namespace hy
