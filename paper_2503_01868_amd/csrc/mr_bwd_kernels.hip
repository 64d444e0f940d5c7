// Hyena-MR backward on the gfx950 matrix cores (bf16 operands, fp32 accumulation), ONE pass over the tensors.
//
// With u = k*v and g = dy*q the gradients of y = q (.) (h * u) are (Sec. 2.1 Eq. 1, Sec. 3.1 Eq. 2):
//     dq[t] = dy[t] * z[t],   z[t] = sum_j h[j] u[t-j]
//     du[s] = sum_j h[j] g[s+j],  dk = du (.) v,  dv = du (.) k
//     dh[j] = sum_{b, c in group, s} u[s] g[s+j]
// The kernel walks the sequence from its end, tau = L-1-t.  In tau the transposed convolution is causal,
// du'[tau] = sum_j h[j] g'[tau-j], so du is the forward block-Toeplitz scheme of mr_kernels.hip (Toeplitz operands
// in registers, register window of the last NKB source blocks, LDS transposition) with g in the role of u and two
// post-gates.  The forward sum is anti-causal in tau, z'[tau] = sum_j h[j] u'[tau+j]: the outputs of a chunk are
// complete once the NKB-1 chunks after it have arrived, so z (and dq) come out NKB-1 chunks late, from a second
// register window that holds the u blocks.  No second set of operands is needed: with the 32 source steps of a
// block fed in reversed order and the 16 output steps written in reversed order, the operand of the anti-causal
// product for output tile tau0 and source block sigma0 has the element h[(sigma0 - tau0 + 16) + n - k], which is the
// causal operand for the offset sigma0 - tau0 + 16.  dy waits NKB chunks for its z in a lane-private LDS ring.
// So dy, q, k, v are each read once and dq, dk, dv written once (7 tensor passes; with the forward kernel computing
// dq in a launch of its own it was 10).  A tile needs NKB-1 chunks of dy, q before it (for du) and NKB-1 chunks of
// k, v after it (for z).
// The filter gradient is a second contraction over the 16 channels of a group,
//     C_x[i][n] = sum_c u[tau_s + i, c] * g[tau_s - 16 x + n, c],    dh[16 x + i - n] += C_x[i][n],
// which is what v_mfma_f32_16x16x16_bf16 computes from plain row-major operands (4 adjacent channels of
// one row per lane): 2*(2 NKB - 1) extra MFMAs per chunk into 2 NKB - 1 accumulators that live in registers
// for the whole tile.  At the end of the tile each wave folds the diagonals of its accumulators into one
// partial dh row and writes it to the workspace (App. A.4: partial accumulation by block, written out
// contiguously); dh_reduce_kernel sums the partials.
// Four waves (64 channels) per workgroup, one wave per SIMD: operands, two windows, the filter-gradient
// accumulators and a deep prefetch need ~300 registers per lane.
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct MrBwdArgs {
    const uint16_t* dy;
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* h;
    uint16_t* dq;
    uint16_t* dk;
    uint16_t* dv;
    float* partial;  // [B * tiles_per_seq][D / 16][lh]: one row per (tile, 16-channel slice)
    int64_t L, D;
    int64_t skv, sgq, sout;  // elements between batch items in k, v / dy, q / dq, dk, dv
    int32_t hist, fut;       // rows of k, v in front of row 0 / of dy, q behind row L - 1 that hold data
    int32_t lh, group;
    int32_t rows, tiles_per_seq, ncb;
};

constexpr int kChunk = 32;

// kShard: the call is one rank's share of a sequence (halo rows next to the tensors, batch strides); the plain
// call's instantiation carries none of that arithmetic.
template <int NKB, int NW, int PF, bool kShard>
__global__ __launch_bounds__(NW * 64, 1) void mr_bwd_kernel(MrBwdArgs a) {
    constexpr int PPR = 2 * NW;              // 16-byte pieces per staged row
    constexpr int CPR = 2 * PPR;             // 8-byte chunks per staged row
    constexpr int kTaps = 32 * NKB;
    constexpr int ZROW = 16 * NW * 4 + 16;
    constexpr int ND = 2 * NKB - 1;          // 16-step offsets x with a tap 16 x + i - n inside [0, lh)
    constexpr int NSLOT = NKB + 1;           // chunks of g kept for the filter gradient (+1: no write/read overlap)
    constexpr int NR = NKB + 1;              // chunks of dy waiting for their z
    constexpr int LAG = NKB - 1;             // chunks between a chunk's arrival and its complete z
    static_assert(NW % 4 == 0, "the LDS swizzle needs 8 pieces per row");
    __shared__ uint4 gst[2][kChunk * PPR];             // g of the newest chunk, swizzled for the transposed read
    __shared__ uint4 utr[2][kChunk * PPR];             // u of the newest chunk, same layout (source of z)
    __shared__ uint2 gring[NSLOT][kChunk * CPR];       // g rows, 8-byte chunks XOR-swizzled by row
    __shared__ uint2 ust[2][kChunk * CPR];             // u rows of the current chunk, same layout (filter gradient)
    __shared__ uint4 dyring[NR][kChunk * PPR];         // raw dy pieces, written and read back by the same lane
    __shared__ __attribute__((aligned(16))) char zst[2][kChunk * ZROW];   // du, fp32 rows
    __shared__ __attribute__((aligned(16))) char zst2[2][kChunk * ZROW];  // z, fp32 rows
    __shared__ float hs[NW][kTaps];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const int li = lane % 16, lq = lane / 16;

    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t L = a.L, D = a.D;
    // everything below is in reversed time tau = L - 1 - t
    const int64_t t_start = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t_end = (t_start + a.rows < L) ? t_start + a.rows : L;
    // dy, q of the chunks before the tile feed its du; before tau = 0 lie the `fut` rows behind the sequence's end
    // that hold data (a shard's right halo), down to the first chunk boundary at or below them
    int64_t t_begin = t_start - (int64_t)kChunk * LAG;
    const int64_t t_floor = kShard ? -(((int64_t)a.fut + kChunk - 1) / kChunk) * kChunk : 0;
    if (t_begin < t_floor) t_begin = t_floor;
    const int64_t tau_lo = kShard ? -(int64_t)a.fut : 0;     // smallest reversed step at which dy and q hold data
    const int64_t tau_hi = kShard ? L + (int64_t)a.hist : L;  // k and v hold data below this reversed step
    // k, v of the LAG chunks after the tile feed its z; the walk always runs LAG chunks past the tile, also where
    // the sequence ends first (those chunks then hold zeros and load nothing)
    const int ntot = (int)((t_end - t_begin + kChunk - 1) / kChunk) + LAG;

    const int64_t cblock0 = (int64_t)cb * 16 * NW;
    const int64_t c0 = cblock0 + 16 * w;
    const int64_t seq0 = kShard ? b * a.sout : b * L * D;
    const int64_t seq0kv = kShard ? b * a.skv : seq0, seq0gq = kShard ? b * a.sgq : seq0;

    const int lr = tid / PPR, lp = tid % PPR;
    const int64_t ld_off = cblock0 + 8 * lp;
    // element offset of reversed step tau for this lane, without the batch item's offset
    auto row_off = [&](int64_t tau) { return (L - 1 - tau) * D + ld_off; };
    auto chunk_start = [&](int ci) { return t_begin + (int64_t)ci * kChunk; };
    auto in_tile = [&](int ci) {
        const int64_t t0 = chunk_start(ci);
        return ci >= 0 && t0 >= t_start && t0 < t_end;
    };
    // loads whose result is never used (chunk indices past the last chunk; k and v before the tile, dy and q after
    // it) all go to one 16-byte location of the tile, the same for every lane of the workgroup: one cache line per
    // wave
    const int64_t idle_off = (L - t_end) * D + cblock0;
    auto load_g = [&](int ci, Words<4>& yy, Words<4>& qq) {
        const int64_t t0 = chunk_start(ci);
        int64_t tau = t0 + lr;
        tau = tau < t_end ? tau : t_end - 1;
        if constexpr (kShard) tau = tau > tau_lo ? tau : tau_lo;  // rows past the data read its last row; their g is zeroed below
        const int64_t off = seq0gq + ((ci < ntot && t0 < t_end) ? row_off(tau) : idle_off);
        yy = load_words_nt<4>(a.dy + off);
        qq = load_words_nt<4>(a.q + off);
    };
    auto load_kv = [&](int ci, Words<4>& kk, Words<4>& vv) {
        const int64_t t0 = chunk_start(ci);
        int64_t tau = t0 + lr;
        tau = tau < tau_hi ? tau : tau_hi - 1;
        const int64_t off = seq0kv + ((ci < ntot && t0 >= t_start && t0 < tau_hi) ? row_off(tau) : idle_off);
        kk = load_words_nt<4>(a.k + off);
        vv = load_words_nt<4>(a.v + off);
    };

    Words<4> ypre[PF], qpre[PF], kpre[PF], vpre[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) {
        load_g(i, ypre[i], qpre[i]);
        if (i + 1 < PF) load_kv(i, kpre[i], vpre[i]);  // the last k, v stage is filled by the first iteration
    }

    // zero the g ring: slots of chunks before the start of the walk stand for steps past the end of the sequence
    for (int i = tid; i < NSLOT * kChunk * CPR; i += NW * 64) (&gring[0][0])[i] = make_uint2(0u, 0u);

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
    // gw[m]: g block of chunk ci - m, source steps in walk order; uw[m]: u block of chunk ci - m, source steps in
    // reversed order (element e of octet lq = step 31 - 8 lq - e of the chunk)
    bf16x8_t gw[NKB], uw[NKB];
    {
        Words<4> z = zero_words<4>();
#pragma unroll
        for (int m = 0; m < NKB; ++m) {
            gw[m] = __builtin_bit_cast(bf16x8_t, z);
            uw[m] = __builtin_bit_cast(bf16x8_t, z);
        }
    }
    f32x4_t cacc[ND];
#pragma unroll
    for (int x = 0; x < ND; ++x) cacc[x] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

    const int swz = ((lr >> 3) & 3) << 1;
    const int st_idx = lr * PPR + (lp ^ swz);
    const int rd_piece = (2 * w + (li >> 3)) ^ (lq << 1);          // rows 8 lq .. 8 lq + 7
    const int rd_piece_rev = (2 * w + (li >> 3)) ^ ((3 - lq) << 1);  // rows 31 - 8 lq - 7 .. 31 - 8 lq
    const int zwr_off = li * ZROW + (16 * w + 4 * lq) * 4;           // du: step li of a 16-step tile
    const int zwr_off_rev = (15 - li) * ZROW + (16 * w + 4 * lq) * 4;  // z: step 15 - li
    const int zrd_off = lr * ZROW + 8 * lp * 4;
    // 8-byte chunk layout: logical chunk c8 of row r sits at c8 ^ (r & 15)
    const int x8 = lr & 15;
    const int wr8a = lr * CPR + ((2 * lp) ^ x8), wr8b = lr * CPR + ((2 * lp + 1) ^ x8);
    const int rd8 = (4 * w + lq) ^ li;  // this lane's chunk in a row whose index is li (mod 16)

    // dk, dv of chunk ci (du staged one iteration earlier)
    auto gate_store_du = [&](int ci, const Words<4>& kk, const Words<4>& vv) {
        const int64_t tau = chunk_start(ci) + lr;
        if (in_tile(ci) && tau < t_end) {
            const char* zp = zst[ci & 1] + zrd_off;
            const float4 za = *reinterpret_cast<const float4*>(zp);
            const float4 zb = *reinterpret_cast<const float4*>(zp + 16);
            const float du[8] = {za.x, za.y, za.z, za.w, zb.x, zb.y, zb.z, zb.w};
            float kf[8], vf[8], o1[8], o2[8];
            Pack<BF16, 8>::unpack(kk, kf);
            Pack<BF16, 8>::unpack(vv, vf);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                o1[e] = du[e] * vf[e];
                o2[e] = du[e] * kf[e];
            }
            const int64_t off = seq0 + row_off(tau);
            store_words_nt<4>(a.dk + off, Pack<BF16, 8>::pack(o1));
            store_words_nt<4>(a.dv + off, Pack<BF16, 8>::pack(o2));
        }
    };
    // dq of chunk cq, whose z was staged in iteration cq + LAG (buffer parity of that iteration)
    auto gate_store_dq = [&](int cq) {
        const int64_t tau = chunk_start(cq) + lr;
        if (in_tile(cq) && tau < t_end) {
            const char* zp = zst2[(cq + LAG) & 1] + zrd_off;
            const float4 za = *reinterpret_cast<const float4*>(zp);
            const float4 zb = *reinterpret_cast<const float4*>(zp + 16);
            const uint4 raw = dyring[cq % NR][tid];
            Words<4> yy;
            yy.w[0] = raw.x; yy.w[1] = raw.y; yy.w[2] = raw.z; yy.w[3] = raw.w;
            float yf[8];
            Pack<BF16, 8>::unpack(yy, yf);
            float o[8] = {za.x * yf[0], za.y * yf[1], za.z * yf[2], za.w * yf[3],
                          zb.x * yf[4], zb.y * yf[5], zb.z * yf[6], zb.w * yf[7]};
            store_words_nt<4>(a.dq + seq0 + row_off(tau), Pack<BF16, 8>::pack(o));
        }
    };

    // one more iteration than chunks: the last chunk's du and the last finished z are gated one iteration late
    for (int base = 0; base < ntot + 1; base += PF) {
#pragma unroll
        for (int sgi = 0; sgi < PF; ++sgi) {
            const int ci = base + sgi;
            const int64_t t0 = chunk_start(ci);
            const bool main_chunk = in_tile(ci) && ci < ntot;
            const int slot = __builtin_amdgcn_readfirstlane(ci % NSLOT);

            // g = dy*q and u = k*v of this lane's row piece, rounded to bf16, into LDS; dy itself into its ring
            {
                float a8[8], b8[8];
                Pack<BF16, 8>::unpack(ypre[sgi], a8);
                Pack<BF16, 8>::unpack(qpre[sgi], b8);
                Words<4> gg;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) gg.w[e2] = pack_bf16x2(a8[2 * e2] * b8[2 * e2], a8[2 * e2 + 1] * b8[2 * e2 + 1]);
                if constexpr (kShard)
                    if (t0 + lr < tau_lo) gg = zero_words<4>();  // past the rows that hold data: zeros
                gst[ci & 1][st_idx] = make_uint4(gg.w[0], gg.w[1], gg.w[2], gg.w[3]);
                gring[slot][wr8a] = make_uint2(gg.w[0], gg.w[1]);
                gring[slot][wr8b] = make_uint2(gg.w[2], gg.w[3]);
                dyring[ci % NR][tid] = make_uint4(ypre[sgi].w[0], ypre[sgi].w[1], ypre[sgi].w[2], ypre[sgi].w[3]);
                Pack<BF16, 8>::unpack(kpre[sgi], a8);
                Pack<BF16, 8>::unpack(vpre[sgi], b8);
                Words<4> uu;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) uu.w[e2] = pack_bf16x2(a8[2 * e2] * b8[2 * e2], a8[2 * e2 + 1] * b8[2 * e2 + 1]);
                // z reaches over the end of the tile but not over the end of the sequence; the filter gradient
                // takes u of the tile only
                const bool in_seq = t0 + lr < tau_hi;
                const bool in_own = t0 + lr < t_end;
                utr[ci & 1][st_idx] = in_seq ? make_uint4(uu.w[0], uu.w[1], uu.w[2], uu.w[3]) : make_uint4(0u, 0u, 0u, 0u);
                ust[ci & 1][wr8a] = in_own ? make_uint2(uu.w[0], uu.w[1]) : make_uint2(0u, 0u);
                ust[ci & 1][wr8b] = in_own ? make_uint2(uu.w[2], uu.w[3]) : make_uint2(0u, 0u);
            }
            load_g(ci + PF, ypre[sgi], qpre[sgi]);

            __syncthreads();

#pragma unroll
            for (int m = NKB - 1; m > 0; --m) {
                gw[m] = gw[m - 1];
                uw[m] = uw[m - 1];
            }
            {
                const uint16_t* s16 = reinterpret_cast<const uint16_t*>(gst[ci & 1]);
                const uint16_t* u16 = reinterpret_cast<const uint16_t*>(utr[ci & 1]);
                Words<4> wds, wdu;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int r0 = 8 * lq + 2 * e2;
                    const uint32_t lo = s16[((r0 * PPR + rd_piece) << 3) + (li & 7)];
                    const uint32_t hi = s16[(((r0 + 1) * PPR + rd_piece) << 3) + (li & 7)];
                    wds.w[e2] = lo | (hi << 16);
                    const int rr = 31 - 8 * lq - 2 * e2;  // reversed: element 2 e2 = row rr, element 2 e2 + 1 = row rr - 1
                    const uint32_t ulo = u16[((rr * PPR + rd_piece_rev) << 3) + (li & 7)];
                    const uint32_t uhi = u16[(((rr - 1) * PPR + rd_piece_rev) << 3) + (li & 7)];
                    wdu.w[e2] = ulo | (uhi << 16);
                }
                gw[0] = __builtin_bit_cast(bf16x8_t, wds);
                uw[0] = __builtin_bit_cast(bf16x8_t, wdu);
            }

            if (main_chunk) {
                f32x4_t acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int m = 0; m < NKB; ++m) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gw[m], tz[2 * m], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gw[m], tz[2 * m + 1], acc1, 0, 0, 0);
                }
                char* zp = zst[ci & 1] + zwr_off;
                *reinterpret_cast<float4*>(zp) = make_float4(acc0[0], acc0[1], acc0[2], acc0[3]);
                *reinterpret_cast<float4*>(zp + 16 * ZROW) = make_float4(acc1[0], acc1[1], acc1[2], acc1[3]);

                // filter gradient: u rows 16 p + i of this chunk against g rows 16 p - 16 x + n
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const uint2 ua = ust[ci & 1][(16 * p + li) * CPR + rd8];
                    const s16x4_t av = __builtin_bit_cast(s16x4_t, ua);
#pragma unroll
                    for (int x = 0; x < ND; ++x) {
                        const int rel = 16 * p - 16 * x;                  // row of the g tile relative to this chunk
                        const int back = (31 - rel) / 32;                 // chunks back (0 for rel >= 0); rel <= 16
                        const int rin = rel + 32 * back;                  // row inside that chunk
                        int gs = slot - back;
                        if (gs < 0) gs += NSLOT;
                        const uint2 gb = gring[gs][(rin + li) * CPR + rd8];
                        cacc[x] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, __builtin_bit_cast(s16x4_t, gb), cacc[x], 0, 0, 0);
                    }
                }
            }
            // z of chunk ci - LAG: its source blocks ci - LAG .. ci are all in the window now.  Source block
            // ci - LAG + s sits s chunks after the output chunk: offset 32 s + 16 for the first 16 outputs,
            // 32 s for the second 16.
            if (ci < ntot && in_tile(ci - LAG)) {
                f32x4_t acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int s = 0; s < NKB; ++s) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(uw[LAG - s], tz[2 * s + 1], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(uw[LAG - s], tz[2 * s], acc1, 0, 0, 0);
                }
                char* zp = zst2[ci & 1] + zwr_off_rev;
                *reinterpret_cast<float4*>(zp) = make_float4(acc0[0], acc0[1], acc0[2], acc0[3]);
                *reinterpret_cast<float4*>(zp + 16 * ZROW) = make_float4(acc1[0], acc1[1], acc1[2], acc1[3]);
            }
            const int prev = (sgi + PF - 1) % PF;  // static after unrolling
            if (ci > 0 && ci <= ntot) {
                gate_store_du(ci - 1, kpre[prev], vpre[prev]);
                gate_store_dq(ci - 1 - LAG);
            }
            load_kv(ci - 1 + PF, kpre[prev], vpre[prev]);
        }
    }

    // ---- fold the diagonals: dh[16 x + i - n] += C_x[i][n]; the lane holds C_x[4 lq + r][li], r = 0..3
    __syncthreads();  // every wave is done with zst
    float* tilebuf = reinterpret_cast<float*>(zst[0]) + w * (16 * 17);  // this wave's 16 x 16 tile, row stride 17
    float* dhw = hs[w];                                                 // reuse: this wave's partial dh, kTaps floats
    for (int j = lane; j < kTaps; j += 64) dhw[j] = 0.0f;
#pragma unroll
    for (int x = 0; x < ND; ++x) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r = 0; r < 4; ++r) tilebuf[(4 * lq + r) * 17 + li] = cacc[x][r];
        __builtin_amdgcn_wave_barrier();
        if (lane < 31) {
            const int delta = lane - 15;  // i - n
            const int j = 16 * x + delta;
            if (j >= 0 && j < a.lh) {
                float s = 0.0f;
                for (int i = 0; i < 16; ++i) {
                    const int n = i - delta;
                    if (n >= 0 && n < 16) s += tilebuf[i * 17 + n];
                }
                dhw[j] += s;
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    float* out = a.partial + ((int64_t)tile * (D / 16) + (c0 / 16)) * a.lh;
    for (int j = lane; j < a.lh; j += 64) out[j] = dhw[j];
}

constexpr int kBwdWaves = 4;  // waves (16-channel slices) per workgroup

template <int NKB, int NW>
hy_status launch_nw(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st, int64_t* nsets) {
    constexpr int PF = 4;  // chunks of dy, q, k, v in flight per lane (measured: 3 and 6 are 2-8% slower)
    MrBwdArgs a;
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
    a.ncb = (int32_t)(s.D / (16 * NW));
    a.rows = (int32_t)mr_bwd_rows(s);
    a.tiles_per_seq = (int32_t)((s.L + a.rows - 1) / a.rows);
    *nsets = s.B * a.tiles_per_seq;
    const int64_t nb = *nsets * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    if (s.sharded()) return launch_kernel((mr_bwd_kernel<NKB, NW, PF, true>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
    return launch_kernel((mr_bwd_kernel<NKB, NW, PF, false>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
}

template <int NKB>
hy_status launch_nkb(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st, int64_t* nsets) {
    return launch_nw<NKB, kBwdWaves>(p, s, ws, st, nsets);
}

}  // namespace

bool mr_bwd_supported(const BwdShape& s) {
    return s.gated && s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 64 == 0 && s.lh > 8 && s.lh <= 129;
}

// time steps per workgroup: one workgroup per CU where the sequence allows it (same rule as the forward kernel)
int64_t mr_bwd_rows(const BwdShape& s) {
    const int64_t ncb = s.D / (16 * kBwdWaves);
    const int nkb = (s.lh - 1 + 31) / 32 + 1;
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        const int64_t base = s.B * ncb;
        const int64_t min_rows = 4LL * kChunk * (nkb > 1 ? nkb - 1 : 1);
        const int64_t tiles = tiles_filling_rounds(base, s.L, min_rows);  // one wave per SIMD: per-CU bound
        rows = (s.L + tiles - 1) / tiles;
        if (rows < min_rows) rows = min_rows;
    }
    rows = (rows + kChunk - 1) / kChunk * kChunk;
    const int64_t cap = (s.L + kChunk - 1) / kChunk * kChunk;
    return rows > cap ? cap : rows;
}

int64_t mr_bwd_workspace_bytes(const BwdShape& s) {
    const int64_t rows = mr_bwd_rows(s);
    const int64_t tiles = (s.L + rows - 1) / rows;
    return s.B * tiles * (s.D / 16) * s.lh * (int64_t)sizeof(float);
}

// dq, dk, dv and dh in one pass.  `ws` holds the partial filter gradients.
hy_status launch_mr_bwd(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st) {
    if (!mr_bwd_supported(s)) return HY_ERR_UNSUPPORTED;
    const int nkb = (s.lh - 1 + 31) / 32 + 1;
    int64_t nsets = 0;
    hy_status rc;
    switch (nkb) {
        case 2: rc = launch_nkb<2>(p, s, ws, st, &nsets); break;
        case 3: rc = launch_nkb<3>(p, s, ws, st, &nsets); break;
        case 4: rc = launch_nkb<4>(p, s, ws, st, &nsets); break;
        case 5: rc = launch_nkb<5>(p, s, ws, st, &nsets); break;
        default: return HY_ERR_UNSUPPORTED;
    }
    if (rc != HY_OK) return rc;
    // partial rows are per 16-channel slice: a group of `group` channels owns group/16 adjacent slices
    return launch_dh_reduce(static_cast<const float*>(ws), p.dh, nsets, s.D / 16, s.lh, s.group / 16, st);
}

}  // namespace hy
