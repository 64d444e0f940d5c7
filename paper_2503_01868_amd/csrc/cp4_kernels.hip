// Gated causal convolution with one filter per channel (or per group of fewer than 16 channels) on the gfx950
// matrix cores, wide version: the chunk-parallel idea of App. A.1 -- put chunks of ONE channel on the matrix
// tile, reuse the channel's Toeplitz factors H_m (Sec. 3.1) for every chunk -- mapped to the batched small-tile
// instruction v_mfma_f32_4x4x4_16B_bf16, which multiplies 16 independent 4x4 blocks at once.
//
// Mapping.  A wave owns 16 channels, one per block.  For channel c and a group of 16 output steps starting at t0:
//   Z[i, j] = sum_m sum_k A_m[i, k] * X_m[k, j],     i, j, k = 0..3,   output step t0 + 4j + i,
//   A_m[i, k] = h_c[4m + i - k]   (zero outside [0, lh)),   X_m[k, j] = u_c[t0 + 4j - 4m + k],
// i.e. chunks of l_b = 4 steps, four chunks per product, and the block row [H_m ... H_1 H_0] of the channel applied
// to each of them; NBK = floor((lh + 2) / 4) + 1 products per 16 outputs.  All A_m of the wave's 16 channels stay in
// registers for the whole tile (2 VGPRs per m), so per product a lane only fetches 4 consecutive steps of u
// (8 bytes from LDS).  Small tiles are what makes this fit: a wave needs 16 steps of 16 channels at a time instead
// of 256 steps of one channel, so a workgroup of 16 waves can own 256 channels (512-byte row pieces, the access
// pattern of the grouped kernel in mr_kernels.hip) with a history ring of only 192 steps per channel in LDS, where
// the 16x16x32 mapping of cp_kernels.hip is confined to 64 channels (128-byte pieces).
//
// Data movement per iteration of 64 steps (memory has channels contiguous, the products want time contiguous):
//   row phase    a lane owns 2 rows x 8 channels (16-byte loads of k, v, q issued one iteration ahead), forms
//                u = k*v, rounds to bf16 and writes, per channel, 2 steps (4 bytes) into the channel's ring line,
//                and q likewise into a [channel][64] buffer;
//   matrix phase 4 groups x NBK products per wave, then the post-gate on the 4 consecutive steps a lane holds,
//                y overwriting q in place;
//   store phase  read back, re-form rows, 16-byte stores.
// The ring is 192 = 3 x 64 steps long, so the write position cycles through three values; the iteration loop is
// unrolled by three, which makes every LDS offset of the matrix phase a compile-time constant (no address
// arithmetic next to the products).  Valid for lh <= 129 (128 steps of history).
#include <type_traits>

#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct Cp4Args {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* h;
    uint16_t* y;
    const uint16_t* q2;  // second post-gate and output of the same convolution (dual kernels only)
    uint16_t* y2;
    int64_t L, D;
    int32_t lh, group;
    int32_t rows;           // time steps per workgroup, multiple of 64
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / (16 NW)
    int32_t rev;            // 1: step t of the kernel is row L - 1 - t of the tensors (the convolution then runs
                            // towards the past: the transposed operator of the backward pass)
    int64_t bstride_kv, bstride_qy, bstride_y;  // elements between batch items in k, v / in q (and q2) / in y (and y2)
    int32_t hist;           // steps of k and v before step 0 that hold data (a sequence shard's halo: rows in front
                            // of row 0, in reversed time rows behind row L - 1)
};

constexpr int kT = 64;    // steps per iteration
constexpr int kR = 192;   // ring length in steps = 3 kT >= kT + history
constexpr int kLS = 416;  // bytes per ring line (>= 2 kR, multiple of 32)
constexpr int kQS = 128;  // bytes per q/y line (2 kT)

// PF = iterations of k, v, q in flight per lane (register stages).
template <int NBK, int NW, int PF>
__global__ __launch_bounds__(NW * 64, NW == 16 ? 4 : 2) void cp4_kernel(Cp4Args a) {
    constexpr int kH = 4 * (NBK - 1);  // steps of history the products reach back
    constexpr int GP = 4;              // output groups per sweep over m
    static_assert(kH <= kR - kT, "history must fit the ring");
    constexpr int C = 16 * NW;         // channels per workgroup
    constexpr int PPR = 2 * NW;        // 16-byte pieces per row
    static_assert(NW * 64 == PPR * (kT / 2), "one lane per (row pair, piece)");
    // every block of 8 channels starts 8 bytes further than the line stride puts it (bank spreading of the
    // transposing 4-byte writes)
    __shared__ __attribute__((aligned(16))) char ring[C * kLS + (C / 8) * 8];
    __shared__ __attribute__((aligned(16))) char qy[C * kQS + (C / 8) * 8];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int ts32 = (int)((tile % a.tiles_per_seq) * (int64_t)a.rows);
    const int te32 = (ts32 + a.rows < a.L) ? ts32 + a.rows : (int)a.L;
    const int nit = (te32 - ts32 + kT - 1) / kT;

    const int64_t D = a.D;
    const uint32_t D32 = (uint32_t)D;
    const int64_t cblock0 = (int64_t)cb * C;
    const int64_t seq0 = b * a.bstride_qy, seq0kv = b * a.bstride_kv, seq0y = b * a.bstride_y;
    const int t_old = -a.hist;  // oldest row that holds data; what lies before it counts as zeros

    auto line_off = [](int c, int stride) { return c * stride + (c >> 3) * 8; };
    // step -> row of the tensors: t, or L - 1 - t = (t ^ -1) + L in reversed time
    const int rxor = a.rev ? -1 : 0, radd = a.rev ? (int)a.L : 0;
    auto phys = [&](int t) { return (uint32_t)((t ^ rxor) + radd); };

    // ---- row layout: rows 2 rp, 2 rp + 1 of an iteration, channels 8 lp .. 8 lp + 7 of the block
    const int lp = tid % PPR, rp = tid / PPR;
    const uint32_t ld_off = (uint32_t)(cblock0 + 8 * lp);
    char* const u_lines = ring + line_off(8 * lp, kLS) + 4 * rp;  // + ring base of the iteration * 2
    char* const q_lines = qy + line_off(8 * lp, kQS) + 4 * rp;

    Words<4> kw[PF][2], vw[PF][2], qw[PF][2];
    auto row_addr = [&](int t) {  // clamped into the rows this tile may touch
        t = t < te32 ? t : te32 - 1;
        t = t > t_old ? t : t_old;
        return (int64_t)((t ^ rxor) + radd) * (int64_t)D32 + ld_off;  // without the batch item's offset
    };
    auto load_rows = [&](int it, Words<4> (&kk)[2], Words<4> (&vv)[2], Words<4> (&qq)[2]) {
        const int t0 = ts32 + (it - 1) * kT + 2 * rp;  // iteration it >= 1 covers steps ts32 + 64 (it - 1) ...
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int64_t off = row_addr(t0 + r);
            kk[r] = load_words_nt<4>(a.k + seq0kv + off);
            vv[r] = load_words_nt<4>(a.v + seq0kv + off);
            qq[r] = load_words_nt<4>(a.q + seq0 + off);
        }
    };
    // u of 2 rows x 8 channels, transposed: one dword (2 steps) per channel into the ring at step position `pos`
    auto write_u = [&](const Words<4> (&kk)[2], const Words<4> (&vv)[2], bool keep0, bool keep1, int pos) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float a0 = keep0 ? bf16_lo(kk[0].w[p]) * bf16_lo(vv[0].w[p]) : 0.0f;
            const float b0 = keep0 ? bf16_hi(kk[0].w[p]) * bf16_hi(vv[0].w[p]) : 0.0f;
            const float a1 = keep1 ? bf16_lo(kk[1].w[p]) * bf16_lo(vv[1].w[p]) : 0.0f;
            const float b1 = keep1 ? bf16_hi(kk[1].w[p]) * bf16_hi(vv[1].w[p]) : 0.0f;
            *reinterpret_cast<uint32_t*>(u_lines + (2 * p) * kLS + pos * 2) = pack_bf16x2(a0, a1);
            *reinterpret_cast<uint32_t*>(u_lines + (2 * p + 1) * kLS + pos * 2) = pack_bf16x2(b0, b1);
        }
    };

#pragma unroll
    for (int i = 0; i < PF; ++i) load_rows(1 + i, kw[i], vw[i], qw[i]);

    // ---- Toeplitz operands of this lane: block = channel 16 w + lane / 4, row i = lane % 4, element k:
    // A_m[i][k] = h[4m + i - k]
    const int blk = lane >> 2, l4 = lane & 3;
    s16x4_t ares[NBK];
    {
        const float* hp = a.h + ((cblock0 + 16 * w + blk) / a.group) * (int64_t)a.lh;
        auto tapv = [&](int idx) { return (idx >= 0 && idx < a.lh) ? hp[idx] : 0.0f; };
#pragma unroll
        for (int m = 0; m < NBK; ++m) {
            float t4[4];  // t4[k] = h[4m + i - k]
            if (m >= 1 && 4 * m + 3 < a.lh) {
                // wholly inside [0, lh): h[4m + i - 3 .. 4m + i], four adjacent floats (4-byte aligned)
                const float* p = hp + 4 * m + l4 - 3;
                t4[3] = p[0]; t4[2] = p[1]; t4[1] = p[2]; t4[0] = p[3];
            } else {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) t4[kk] = tapv(4 * m + l4 - kk);
            }
            Words<2> wd;
            wd.w[0] = pack_bf16x2(t4[0], t4[1]);
            wd.w[1] = pack_bf16x2(t4[2], t4[3]);
            ares[m] = __builtin_bit_cast(s16x4_t, wd);
        }
    }

    // ---- history: the kH steps before the tile; steps ts32 - 128 + x sit at ring position (x + 128) % 192
    {
        Words<4> kh[2], vh[2];
#pragma unroll
        for (int hp2 = 0; hp2 < 2; ++hp2) {
            if (hp2 == 0 && kH <= kT) continue;  // short filters never reach the older half
            const int t0 = ts32 - 2 * kT + hp2 * kT + 2 * rp;
            const int t_lo = ts32 - kH;  // oldest step needed: older rows re-read it (unused)
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                int t = t0 + r;
                t = t > t_lo ? t : t_lo;
                const int64_t off = row_addr(t);
                kh[r] = load_words_nt<4>(a.k + seq0kv + off);
                vh[r] = load_words_nt<4>(a.v + seq0kv + off);
            }
            write_u(kh, vh, t0 >= t_old, t0 + 1 >= t_old, hp2 == 0 ? 2 * kT : 0);
        }
    }

    // ---- matrix-phase lane constants: block blk = channel, column j = l4
    const int cw = 16 * w + blk;
    const char* const rl = ring + line_off(cw, kLS);
    const char* const ring_lane = rl + 8 * l4;                            // position 4 j
    const char* const mix1 = rl + 2 * ((4 * l4 - 4 + kR) % kR);           // position 4 j - 4, wrapped per lane
    const char* const mix2 = rl + 2 * ((4 * l4 - 8 + kR) % kR);
    const char* const mix3 = rl + 2 * ((4 * l4 - 12 + kR) % kR);
    char* const qy_lane = qy + line_off(cw, kQS) + 8 * l4;

    auto phase = [&](auto wb_c, auto st_c, int it) {
        constexpr int WB = decltype(wb_c)::value;  // ring position of the iteration's first step
        constexpr int ST = decltype(st_c)::value;  // register stage holding this iteration's rows
        const int ts = ts32 + (it - 1) * kT;
        // ---- row phase
        {
            const int t = ts + 2 * rp;
            write_u(kw[ST], vw[ST], t < te32, t + 1 < te32, WB);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t q0 = qw[ST][0].w[p], q1 = qw[ST][1].w[p];
                *reinterpret_cast<uint32_t*>(q_lines + (2 * p) * kQS) = (q0 & 0xffffu) | (q1 << 16);
                *reinterpret_cast<uint32_t*>(q_lines + (2 * p + 1) * kQS) = (q0 >> 16) | (q1 & 0xffff0000u);
            }
        }
        load_rows(it + PF, kw[ST], vw[ST], qw[ST]);
        __syncthreads();

        // ---- matrix phase: 4 groups of 16 steps, NBK products each, all LDS offsets constant; GP groups share a
        // sweep over m (fewer accumulators and operands in flight where registers are short)
#pragma unroll
        for (int g0 = 0; g0 < 4; g0 += GP) {
            f32x4_t acc[GP];
#pragma unroll
            for (int g = 0; g < GP; ++g) acc[g] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int m = 0; m < NBK; ++m) {
#pragma unroll
                for (int g = 0; g < GP; ++g) {
                    const int c0 = WB + 16 * (g0 + g) - 4 * m;  // constant after unrolling: position of column 0
                    const char* p;
                    if (c0 >= 0) p = ring_lane + 2 * c0;
                    else if (c0 <= -16) p = ring_lane + 2 * (c0 + kR);
                    else if (c0 == -4) p = mix1;
                    else if (c0 == -8) p = mix2;
                    else p = mix3;
                    const uint2 bw = *reinterpret_cast<const uint2*>(p);
                    Words<2> bb;
                    bb.w[0] = bw.x; bb.w[1] = bw.y;
                    acc[g] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ares[m], __builtin_bit_cast(s16x4_t, bb), acc[g], 0, 0, 0);
                }
            }
#pragma unroll
            for (int g = 0; g < GP; ++g) {
                char* ql = qy_lane + 32 * (g0 + g);
                const uint2 q4 = *reinterpret_cast<const uint2*>(ql);
                *reinterpret_cast<uint2*>(ql) =
                    make_uint2(pack_bf16x2(bf16_lo(q4.x) * acc[g][0], bf16_hi(q4.x) * acc[g][1]),
                               pack_bf16x2(bf16_lo(q4.y) * acc[g][2], bf16_hi(q4.y) * acc[g][3]));
            }
        }
        __syncthreads();

        // ---- store phase
        {
            uint32_t yc[8];
#pragma unroll
            for (int c8 = 0; c8 < 8; ++c8) yc[c8] = *reinterpret_cast<const uint32_t*>(q_lines + c8 * kQS);
            Words<4> row0, row1;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                row0.w[p] = (yc[2 * p] & 0xffffu) | (yc[2 * p + 1] << 16);
                row1.w[p] = (yc[2 * p] >> 16) | (yc[2 * p + 1] & 0xffff0000u);
            }
            const int t = ts + 2 * rp;
            if (t < te32) store_words_nt<4>(a.y + seq0y + ((uint64_t)phys(t) * D32 + ld_off), row0);
            if (t + 1 < te32) store_words_nt<4>(a.y + seq0y + ((uint64_t)phys(t + 1) * D32 + ld_off), row1);
        }
    };

    // the ring position repeats every 3 iterations, the register stage every PF: unrolled by their common multiple
    using std::integral_constant;
    if constexpr (PF == 1) {
        for (int it = 1; it <= nit; it += 3) {
            phase(integral_constant<int, kT>{}, integral_constant<int, 0>{}, it);
            if (it + 1 <= nit) phase(integral_constant<int, 2 * kT>{}, integral_constant<int, 0>{}, it + 1);
            if (it + 2 <= nit) phase(integral_constant<int, 0>{}, integral_constant<int, 0>{}, it + 2);
        }
    } else {
        static_assert(PF == 2, "one or two stages");
        for (int it = 1; it <= nit; it += 6) {
            phase(integral_constant<int, kT>{}, integral_constant<int, 0>{}, it);
            if (it + 1 <= nit) phase(integral_constant<int, 2 * kT>{}, integral_constant<int, 1>{}, it + 1);
            if (it + 2 <= nit) phase(integral_constant<int, 0>{}, integral_constant<int, 0>{}, it + 2);
            if (it + 3 <= nit) phase(integral_constant<int, kT>{}, integral_constant<int, 1>{}, it + 3);
            if (it + 4 <= nit) phase(integral_constant<int, 2 * kT>{}, integral_constant<int, 0>{}, it + 4);
            if (it + 5 <= nit) phase(integral_constant<int, 0>{}, integral_constant<int, 1>{}, it + 5);
        }
    }
}

// ---- Wave-specialised version for the long filters (NBK >= 25), where the products take long enough that running
// them between the row and store phases of the same waves leaves the memory stream idle.  Twelve waves share 128
// channels: waves 0..7 only multiply (16 channels each, as above), waves 8..11 only move data (loads, u = k*v and
// q into LDS, y out of LDS).  While the multipliers work on iteration j, the movers store y of iteration j - 1 and
// prepare iteration j + 1; one barrier per iteration separates the steps.  The ring therefore has four slots of
// 64 steps (the products of iteration j read slots j-2, j-1, j while slot j+1 is written) and the q/y buffer two
// (a mover lane reads the y of iteration j - 1 and then writes the q of iteration j + 1 to the same addresses).
constexpr int kWM = 8;     // multiplier waves
constexpr int kWV = 4;     // mover waves
constexpr int kR4 = 256;   // ring length in steps, 4 kT
constexpr int kLS4 = 544;  // bytes per ring line (2 kR4 + 32: 8 banks per channel)
constexpr int kQS4 = 288;  // bytes per q/y line (2 slots x 2 kT + 32)

// DUAL: two post-gates and two outputs from one convolution, y = q * z and y2 = q2 * z (the backward pass needs
// dk = v * du and dv = k * du): a second q/y buffer, one more tensor loaded and one more stored per step.
template <int NBK, int PF, bool DUAL>
__global__ __launch_bounds__((kWM + kWV) * 64, 3) void cp4ws_kernel(Cp4Args a) {
    constexpr int kH = 4 * (NBK - 1);
    static_assert(kH <= 2 * kT, "history must fit two ring slots");
    static_assert(PF == 1 || PF == 2, "one or two stages");
    constexpr int C = 16 * kWM;  // channels per workgroup
    constexpr int PPR = C / 8;   // 16-byte pieces per row
    __shared__ __attribute__((aligned(16))) char ring[C * kLS4 + (C / 8) * 8];
    __shared__ __attribute__((aligned(16))) char qy[C * kQS4 + (C / 8) * 8];
    __shared__ __attribute__((aligned(16))) char qy2[DUAL ? C * kQS4 + (C / 8) * 8 : 16];

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int ts32 = (int)((tile % a.tiles_per_seq) * (int64_t)a.rows);
    const int te32 = (ts32 + a.rows < a.L) ? ts32 + a.rows : (int)a.L;
    const int nit = (te32 - ts32 + kT - 1) / kT;  // iterations 1..nit; iteration j holds steps ts32 + 64 (j - 1) ...

    const uint32_t D32 = (uint32_t)a.D;
    const int64_t cblock0 = (int64_t)cb * C;
    const int64_t seq0 = b * a.bstride_qy, seq0kv = b * a.bstride_kv, seq0y = b * a.bstride_y;
    const int t_old = -a.hist;  // oldest row that holds data; what lies before it counts as zeros
    auto line_off = [](int c, int stride) { return c * stride + (c >> 3) * 8; };
    const int rxor = a.rev ? -1 : 0, radd = a.rev ? (int)a.L : 0;  // step -> row, see cp4_kernel
    auto phys = [&](int t) { return (uint32_t)((t ^ rxor) + radd); };
    using std::integral_constant;

    if (w < kWM) {
        // ================= multiplier waves
        const int blk = lane >> 2, l4 = lane & 3;
        s16x4_t ares[NBK];
        {
            const float* hp = a.h + ((cblock0 + 16 * w + blk) / a.group) * (int64_t)a.lh;
            auto tapv = [&](int idx) { return (idx >= 0 && idx < a.lh) ? hp[idx] : 0.0f; };
#pragma unroll
            for (int m = 0; m < NBK; ++m) {
                float t4[4];  // t4[k] = h[4m + i - k]
                if (m >= 1 && 4 * m + 3 < a.lh) {
                    const float* p = hp + 4 * m + l4 - 3;
                    t4[3] = p[0]; t4[2] = p[1]; t4[1] = p[2]; t4[0] = p[3];
                } else {
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) t4[kk] = tapv(4 * m + l4 - kk);
                }
                Words<2> wd;
                wd.w[0] = pack_bf16x2(t4[0], t4[1]);
                wd.w[1] = pack_bf16x2(t4[2], t4[3]);
                ares[m] = __builtin_bit_cast(s16x4_t, wd);
            }
        }
        const int cw = 16 * w + blk;
        const char* const rl = ring + line_off(cw, kLS4);
        const char* const ring_lane = rl + 8 * l4;                    // position 4 j
        const char* const mix1 = rl + 2 * ((4 * l4 - 4 + kR4) % kR4);  // position 4 j - 4, wrapped per lane
        const char* const mix2 = rl + 2 * ((4 * l4 - 8 + kR4) % kR4);
        const char* const mix3 = rl + 2 * ((4 * l4 - 12 + kR4) % kR4);
        char* const qy_lane = qy + line_off(cw, kQS4) + 8 * l4;
        char* const qy2_lane = qy2 + line_off(cw, kQS4) + 8 * l4;

        auto mstep = [&](auto j4_c) {
            constexpr int J4 = decltype(j4_c)::value;  // iteration mod 4 = ring slot
            constexpr int WB = kT * J4;
            constexpr int SL = (J4 & 1) * 2 * kT;      // byte offset of the q/y slot
            f32x4_t acc[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) acc[g] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int m = 0; m < NBK; ++m) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c0 = (WB + 16 * g - 4 * m + 4 * kR4) % kR4;  // position of column 0, constant
                    const char* p;
                    if (c0 <= kR4 - 16) p = ring_lane + 2 * c0;
                    else if (c0 == kR4 - 4) p = mix1;
                    else if (c0 == kR4 - 8) p = mix2;
                    else p = mix3;
                    const uint2 bw = *reinterpret_cast<const uint2*>(p);
                    Words<2> bb;
                    bb.w[0] = bw.x; bb.w[1] = bw.y;
                    acc[g] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ares[m], __builtin_bit_cast(s16x4_t, bb), acc[g], 0, 0, 0);
                }
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                char* ql = qy_lane + SL + 32 * g;
                const uint2 q4 = *reinterpret_cast<const uint2*>(ql);
                *reinterpret_cast<uint2*>(ql) =
                    make_uint2(pack_bf16x2(bf16_lo(q4.x) * acc[g][0], bf16_hi(q4.x) * acc[g][1]),
                               pack_bf16x2(bf16_lo(q4.y) * acc[g][2], bf16_hi(q4.y) * acc[g][3]));
                if constexpr (DUAL) {
                    char* ql2 = qy2_lane + SL + 32 * g;
                    const uint2 p4 = *reinterpret_cast<const uint2*>(ql2);
                    *reinterpret_cast<uint2*>(ql2) =
                        make_uint2(pack_bf16x2(bf16_lo(p4.x) * acc[g][0], bf16_hi(p4.x) * acc[g][1]),
                                   pack_bf16x2(bf16_lo(p4.y) * acc[g][2], bf16_hi(p4.y) * acc[g][3]));
                }
            }
            __syncthreads();
        };

        __syncthreads();  // history and iteration 1 are in place
        for (int j = 1; j <= nit; j += 4) {
            mstep(integral_constant<int, 1>{});
            if (j + 1 <= nit) mstep(integral_constant<int, 2>{});
            if (j + 2 <= nit) mstep(integral_constant<int, 3>{});
            if (j + 3 <= nit) mstep(integral_constant<int, 0>{});
        }
    } else {
        // ================= mover waves: lane = piece lp of rows 2 rp, 2 rp + 1, 2 rp + 32, 2 rp + 33 of an iteration
        const int mt = tid - kWM * 64;
        const int lp = mt % PPR, rp = mt / PPR;
        const uint32_t ld_off = (uint32_t)(cblock0 + 8 * lp);
        char* const u_lines = ring + line_off(8 * lp, kLS4) + 4 * rp;
        char* const q_lines = qy + line_off(8 * lp, kQS4) + 4 * rp;
        char* const q2_lines = qy2 + line_off(8 * lp, kQS4) + 4 * rp;

        auto row_addr = [&](int t) {  // clamped into the rows this tile may touch
            t = t < te32 ? t : te32 - 1;
            t = t > t_old ? t : t_old;
            return (int64_t)((t ^ rxor) + radd) * (int64_t)D32 + ld_off;  // without the batch item's offset
        };
        // u of 2 rows x 8 channels, transposed: one dword (2 steps) per channel at ring position `pos` + 2 rp
        auto write_u = [&](const Words<4> (&kk)[2], const Words<4> (&vv)[2], bool keep0, bool keep1, int pos) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float a0 = keep0 ? bf16_lo(kk[0].w[p]) * bf16_lo(vv[0].w[p]) : 0.0f;
                const float b0 = keep0 ? bf16_hi(kk[0].w[p]) * bf16_hi(vv[0].w[p]) : 0.0f;
                const float a1 = keep1 ? bf16_lo(kk[1].w[p]) * bf16_lo(vv[1].w[p]) : 0.0f;
                const float b1 = keep1 ? bf16_hi(kk[1].w[p]) * bf16_hi(vv[1].w[p]) : 0.0f;
                *reinterpret_cast<uint32_t*>(u_lines + (2 * p) * kLS4 + pos * 2) = pack_bf16x2(a0, a1);
                *reinterpret_cast<uint32_t*>(u_lines + (2 * p + 1) * kLS4 + pos * 2) = pack_bf16x2(b0, b1);
            }
        };

        Words<4> kw[PF][2][2], vw[PF][2][2], qw[PF][2][2];  // [stage][half of the iteration][row of the pair]
        Words<4> pw[DUAL ? PF : 1][2][2];                  // the second gate
        auto load_rows = [&](int it, Words<4> (&kk)[2][2], Words<4> (&vv)[2][2], Words<4> (&qq)[2][2],
                             Words<4> (&pp)[2][2]) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int t0 = ts32 + (it - 1) * kT + 32 * hf + 2 * rp;
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int64_t off = row_addr(t0 + r);
                    kk[hf][r] = load_words_nt<4>(a.k + seq0kv + off);
                    vv[hf][r] = load_words_nt<4>(a.v + seq0kv + off);
                    qq[hf][r] = load_words_nt<4>(a.q + seq0 + off);
                    if constexpr (DUAL) pp[hf][r] = load_words_nt<4>(a.q2 + seq0 + off);
                }
            }
        };
        // a gate's 2 rows x 8 channels, transposed into its [channel][time] buffer
        auto write_gate = [&](char* ql, const Words<4> (&qq)[2]) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t q0 = qq[0].w[p], q1 = qq[1].w[p];
                *reinterpret_cast<uint32_t*>(ql + (2 * p) * kQS4) = (q0 & 0xffffu) | (q1 << 16);
                *reinterpret_cast<uint32_t*>(ql + (2 * p + 1) * kQS4) = (q0 >> 16) | (q1 & 0xffff0000u);
            }
        };
        // iteration `it` out of its register stage into ring position wb and q/y slot offset sl
        auto prepare = [&](int it, int wb, int sl, Words<4> (&kk)[2][2], Words<4> (&vv)[2][2], Words<4> (&qq)[2][2],
                           Words<4> (&pp)[2][2]) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int t = ts32 + (it - 1) * kT + 32 * hf + 2 * rp;
                write_u(kk[hf], vv[hf], t < te32, t + 1 < te32, wb + 32 * hf);
                write_gate(q_lines + sl + 64 * hf, qq[hf]);
                if constexpr (DUAL) write_gate(q2_lines + sl + 64 * hf, pp[hf]);
            }
        };
        auto store_one = [&](int it, int sl, const char* lines, uint16_t* dst) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                uint32_t yc[8];
                const char* ql = lines + sl + 64 * hf;
#pragma unroll
                for (int c8 = 0; c8 < 8; ++c8) yc[c8] = *reinterpret_cast<const uint32_t*>(ql + c8 * kQS4);
                Words<4> row0, row1;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    row0.w[p] = (yc[2 * p] & 0xffffu) | (yc[2 * p + 1] << 16);
                    row1.w[p] = (yc[2 * p] >> 16) | (yc[2 * p + 1] & 0xffff0000u);
                }
                const int t = ts32 + (it - 1) * kT + 32 * hf + 2 * rp;
                if (t < te32) store_words_nt<4>(dst + seq0y + ((uint64_t)phys(t) * D32 + ld_off), row0);
                if (t + 1 < te32) store_words_nt<4>(dst + seq0y + ((uint64_t)phys(t + 1) * D32 + ld_off), row1);
            }
        };
        auto store_y = [&](int it, int sl) {
            store_one(it, sl, q_lines, a.y);
            if constexpr (DUAL) store_one(it, sl, q2_lines, a.y2);
        };

        // history: steps ts32 - 128 .. ts32 - 65 into slot 3, ts32 - 64 .. ts32 - 1 into slot 0; its loads go out
        // first, the first iteration's behind them
        {
            const int t_lo = ts32 - kH;  // oldest step needed: older rows re-read it (unused)
            Words<4> kh[2][2][2], vh[2][2][2];
#pragma unroll
            for (int hb = (kH <= kT ? 1 : 0); hb < 2; ++hb) {
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const int t0 = ts32 - 2 * kT + hb * kT + 32 * hf + 2 * rp;
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        int t = t0 + r;
                        t = t > t_lo ? t : t_lo;
                        const int64_t off = row_addr(t);
                        kh[hb][hf][r] = load_words_nt<4>(a.k + seq0kv + off);
                        vh[hb][hf][r] = load_words_nt<4>(a.v + seq0kv + off);
                    }
                }
            }
            load_rows(1, kw[0], vw[0], qw[0], pw[0]);
#pragma unroll
            for (int hb = (kH <= kT ? 1 : 0); hb < 2; ++hb) {
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const int t0 = ts32 - 2 * kT + hb * kT + 32 * hf + 2 * rp;
                    write_u(kh[hb][hf], vh[hb][hf], t0 >= t_old, t0 + 1 >= t_old, (hb == 0 ? 3 * kT : 0) + 32 * hf);
                }
            }
        }
        if constexpr (PF == 2) {
            if (2 <= nit) load_rows(2, kw[1], vw[1], qw[1], pw[DUAL ? 1 : 0]);
        }
        prepare(1, kT, 2 * kT, kw[0], vw[0], qw[0], pw[0]);
        if (1 + PF <= nit) load_rows(1 + PF, kw[0], vw[0], qw[0], pw[0]);
        __syncthreads();

        auto vstep = [&](auto j4_c, int j) {
            constexpr int J4 = decltype(j4_c)::value;  // j mod 4
            constexpr int ST = J4 % PF;                // stage of iteration j + 1
            if (j >= 2) store_y(j - 1, ((J4 + 3) & 1) * 2 * kT);
            if (j + 1 <= nit) {
                prepare(j + 1, kT * ((J4 + 1) & 3), ((J4 + 1) & 1) * 2 * kT, kw[ST], vw[ST], qw[ST], pw[DUAL ? ST : 0]);
                if (j + 1 + PF <= nit) load_rows(j + 1 + PF, kw[ST], vw[ST], qw[ST], pw[DUAL ? ST : 0]);
            }
            __syncthreads();
        };
        for (int j = 1; j <= nit; j += 4) {
            vstep(integral_constant<int, 1>{}, j);
            if (j + 1 <= nit) vstep(integral_constant<int, 2>{}, j + 1);
            if (j + 2 <= nit) vstep(integral_constant<int, 3>{}, j + 2);
            if (j + 3 <= nit) vstep(integral_constant<int, 0>{}, j + 3);
        }
        store_y(nit, (nit & 1) * 2 * kT);
    }
}

template <int NBK, int NW, int PF>
hy_status launch_cp4_nw(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    Cp4Args a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.h = p.h;
    a.y = static_cast<uint16_t*>(p.y);
    a.q2 = nullptr;
    a.y2 = nullptr;
    a.L = s.L;
    a.D = s.D;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * NW));
    a.rev = s.reversed ? 1 : 0;
    a.bstride_kv = s.stride_kv();
    a.bstride_qy = s.stride_qy();
    a.bstride_y = s.stride_y();
    a.hist = s.history;
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        const int64_t tiles = tiles_filling_rounds(s.B * a.ncb, s.L, 4 * kT);  // one workgroup per CU
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 4 * kT) rows = 4 * kT;
    }
    rows = (rows + kT - 1) / kT * kT;
    if (rows > (s.L + kT - 1) / kT * kT) rows = (s.L + kT - 1) / kT * kT;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb = s.B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel((cp4_kernel<NBK, NW, PF>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
}

template <int NBK, int PF>
hy_status launch_cp4_ws(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    const bool dual = p.q2 != nullptr;
    Cp4Args a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.h = p.h;
    a.y = static_cast<uint16_t*>(p.y);
    a.q2 = static_cast<const uint16_t*>(p.q2);
    a.y2 = static_cast<uint16_t*>(p.y2);
    a.L = s.L;
    a.D = s.D;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * kWM));
    a.rev = s.reversed ? 1 : 0;
    a.bstride_kv = s.stride_kv();
    a.bstride_qy = s.stride_qy();
    a.bstride_y = s.stride_y();
    a.hist = s.history;
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        const int64_t tiles = tiles_filling_rounds(s.B * a.ncb, s.L, 4 * kT);  // one workgroup per CU
        rows = (s.L + tiles - 1) / tiles;
        if (rows < 4 * kT) rows = 4 * kT;
    }
    rows = (rows + kT - 1) / kT * kT;
    if (rows > (s.L + kT - 1) / kT * kT) rows = (s.L + kT - 1) / kT * kT;
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    const int64_t nb = s.B * a.tiles_per_seq * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    if (dual) return launch_kernel((cp4ws_kernel<NBK, PF, true>), dim3((uint32_t)nb), dim3((kWM + kWV) * 64), st, a);
    return launch_kernel((cp4ws_kernel<NBK, PF, false>), dim3((uint32_t)nb), dim3((kWM + kWV) * 64), st, a);
}

template <int NBK>
hy_status launch_cp4_nbk(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    // 16 waves (128 registers per lane) only where the operands of all products fit beside the rest; longer filters
    // run with 8 waves.  (Tried for them at 16 waves: accumulating two groups at a time with scheduling fences
    // fits the registers, but runs slower than 8 waves, 92 against 63 us at lh = 128.)
    if constexpr (NBK <= 17) {
        if (s.D % 256 == 0 && tuning().mr_waves != 8) return launch_cp4_nw<NBK, 16, 1>(p, s, st);
        // (a second register stage of loads in flight, PF = 2, measured no faster here)
        return launch_cp4_nw<NBK, 8, 1>(p, s, st);
    } else {
        // long filters: 8 multiplier waves + 4 mover waves (a kernel whose 8 waves load, multiply and store in turn
        // ran at the same speed and was removed)
        return launch_cp4_ws<NBK, 2>(p, s, st);
    }
}

}  // namespace

bool cp4_dual_supported(const ConvShape& s) { return cp4_supported(s) && (s.lh + 2) / 4 + 1 > 17; }

bool cp4_supported(const ConvShape& s) {
    return s.dtype == HY_BF16 && s.gated && s.D % 128 == 0 && s.lh >= 1 && s.lh <= 129 && s.L <= 0x7fff0000LL &&
           s.D <= 0x7fff0000LL;
}

hy_status launch_cp4(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    if (!cp4_supported(s)) return HY_ERR_UNSUPPORTED;
    if ((p.q2 != nullptr || p.y2 != nullptr) && !(p.q2 != nullptr && p.y2 != nullptr && cp4_dual_supported(s)))
        return HY_ERR_UNSUPPORTED;
    const int nbk = (s.lh + 2) / 4 + 1;  // products per 16 outputs; instantiated in steps of 8 (except the smallest)
    if (nbk <= 5) return launch_cp4_nbk<5>(p, s, st);
    if (nbk <= 9) return launch_cp4_nbk<9>(p, s, st);
    if (nbk <= 17) return launch_cp4_nbk<17>(p, s, st);
    if (nbk <= 25) return launch_cp4_nbk<25>(p, s, st);
    return launch_cp4_nbk<33>(p, s, st);
}

}  // namespace hy
