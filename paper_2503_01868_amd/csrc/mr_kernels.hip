// Hyena-MR forward on the gfx950 matrix cores: block-Toeplitz contraction (Sec. 3.1, hat y_n = sum_k H_k
// hat x_{n-k}) with bf16 operands and fp32 accumulation, both gates fused (Algorithm 1).
//
// Mapping.  v_mfma_f32_16x16x32_bf16 computes a 16 x 16 tile from a 16 x 32 and a 32 x 16 operand.  Here
//   M = the 16 channels of one filter group slice,  N = 16 output time steps,  K = 32 source time steps:
//   Z^T[c, t] = sum_s U^T[c, s] * Tz^T[s, t],   Tz[t, s] = h[t - s]   (Eq. 3).
// Because Tz is Toeplitz, the operand for output tile t0 and source block s0 depends only on d = t0 - s0,
// so the 2*NKB operands d = 0, 16, 32, ... are built once per wave from h and stay in registers for the
// whole sequence: the filter is never re-read and no Toeplitz factor is ever materialised in memory.
// The source operand needs 8 consecutive time steps of one channel per lane while memory has channels
// contiguous, so u = k*v goes through LDS: written row-wise (16 B per lane), read column-wise.  With
// channels on M the accumulator of a lane holds 4 adjacent channels of one time step; z goes back through
// LDS as fp32 rows so that q is loaded and y is stored as whole row pieces, 16 bytes per lane, like k and v.
//
// A workgroup of NW waves owns 16*NW adjacent channels (wave w: channels 16w..16w+15, one filter) and
// `rows` time steps, and walks them in chunks of 32 steps.  Per chunk: the workgroup loads 32 x 16NW
// elements of k and v with full-line coalesced 16-byte loads (k, v and q are prefetched several chunks
// ahead in registers, so a chunk iteration never waits a full memory latency), multiplies, rounds u to bf16 and stores it to a double-buffered LDS stage; after one
// barrier each wave reads its group's 32 x 16 block transposed, pushes it into a register window of the
// last NKB blocks, issues 2*NKB MFMAs for the two 16-step output tiles of the chunk and parks z in LDS;
// the post-gate and store of a chunk run one iteration late, after the next barrier, so there is a
// single barrier per chunk.  A tile that does not start the sequence first runs NKB-1 warm-up chunks that
// only fill the window (the halo).
#include "hy_common.hpp"
#include "hy_launch.hpp"

namespace hy {
namespace {

struct MrArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const float* h;
    uint16_t* y;
    int64_t L, D;
    int64_t bstride_kv, bstride_qy;  // elements between batch items in k, v / in q, y
    int32_t hist;           // rows of k and v in front of row 0 that hold data (a sequence shard's left halo)
    int32_t lh, group;
    int32_t rows;           // time steps per workgroup, multiple of 32
    int32_t tiles_per_seq;  // ceil(L / rows)
    int32_t ncb;            // channel blocks = D / (16 NW)
};

constexpr int kChunk = 32;

// kPrefetch = chunks of k, v and q in flight per lane (registers).  Two waves per SIMD must fit (NKB = 13: 247
// registers); filters beyond 385 taps (NKB = 17: 34 operands and a window of 17 blocks, ~320 registers) run one wave
// per SIMD.
// kShard: the call is one rank's share of a sequence (history rows in front of k and v, batch strides); the plain
// call's instantiation carries none of that arithmetic.
template <int NKB, int NW, int kPrefetch, bool kShard>
__global__ __launch_bounds__(NW * 64, NW == 16 ? 4 : (NKB > 13 ? 1 : 2)) void mr_mfma_kernel(MrArgs a) {
    constexpr int PPR = 2 * NW;              // 16-byte pieces per staged row of u (bf16)
    constexpr int kTaps = 32 * NKB;          // >= lh
    constexpr int ZROW = 16 * NW * 4 + 16;   // bytes per staged row of z (fp32), padded against bank conflicts
    static_assert(NW % 4 == 0, "the LDS swizzle needs 8 pieces per row");
    __shared__ uint4 stage[2][kChunk * PPR];
    __shared__ __attribute__((aligned(16))) char zst[2][kChunk * ZROW];
    __shared__ float hs[NW][kTaps];

    const int tid = threadIdx.x;
    const int w = tid / 64, lane = tid % 64;
    const int li = lane % 16, lq = lane / 16;

    // launch order: channel block fastest, so neighbouring workgroups read neighbouring 32*NW-byte
    // pieces of the same rows and the chip sweeps whole rows
    const uint32_t lb = blockIdx.x;
    const int cb = lb % a.ncb;
    const int64_t tile = lb / a.ncb;
    const int64_t b = tile / a.tiles_per_seq;
    const int64_t t_start = (tile % a.tiles_per_seq) * (int64_t)a.rows;
    const int64_t t_end = (t_start + a.rows < a.L) ? t_start + a.rows : a.L;
    // warm-up chunks reach back to the first chunk boundary at or below the oldest row that holds data
    int64_t t_begin = t_start - (int64_t)kChunk * (NKB - 1);
    const int64_t t_floor = kShard ? -(((int64_t)a.hist + kChunk - 1) / kChunk) * kChunk : 0;
    if (t_begin < t_floor) t_begin = t_floor;
    const int nchunks = (int)((t_end - t_begin + kChunk - 1) / kChunk);

    const int64_t D = a.D;
    const int64_t cblock0 = (int64_t)cb * 16 * NW;  // first channel of the workgroup
    const int64_t c0 = cblock0 + 16 * w;            // first channel of this wave
    const int64_t seq0 = kShard ? b * a.bstride_qy : b * a.L * D, seq0kv = kShard ? b * a.bstride_kv : seq0;

    // cooperative coordinates of this lane: row lr of the chunk, 16-byte piece lp (8 channels) of the row;
    // used for the k, v, q loads and the y store, all of them whole 32*NW-byte row pieces
    const int lr = tid / PPR, lp = tid % PPR;
    // 32-bit lane arithmetic (the launcher admits L, D < 2^31): fewer live registers than 64-bit row offsets
    const uint32_t ld_off = (uint32_t)(cblock0 + 8 * lp);
    const uint32_t D32 = (uint32_t)D;
    const int tb32 = (int)t_begin, ts32 = (int)t_start, te32 = (int)t_end;
    // Every lane issues exactly three loads per chunk, with no control flow around them, so the loop keeps
    // kPrefetch chunks in flight without ever draining the queue.  Addresses are clamped instead:
    //  - rows past the end of the tile read the tile's last row (a source step >= t_end only reaches
    //    outputs >= t_end, which are never stored);
    //  - loads whose result is never used (chunk indices past the last chunk; q of warm-up chunks) all go to ONE
    //    16-byte location of the tile, the same for every lane of the workgroup, so that they cost one cache line
    //    per wave instead of a row piece per lane (with the streaming hint such re-reads may otherwise go all the
    //    way to memory: 2 of 20 chunk loads of a 512-step tile).
    const uint64_t idle_off = (uint64_t)(uint32_t)(te32 - 1) * D32 + (uint32_t)cblock0;
    //  - rows before the oldest row that holds data (a shard whose halo does not fill its first warm-up chunk) read
    //    that oldest row; their u is zeroed before it is staged.
    const int t_old = kShard ? -a.hist : 0;
    auto load_kv = [&](int ci, Words<4>& kk, Words<4>& vv) {
        int t = tb32 + ci * kChunk + lr;
        t = t < te32 ? t : te32 - 1;
        if constexpr (kShard) t = t > t_old ? t : t_old;
        const int64_t off = ci < nchunks ? (int64_t)t * (int64_t)D32 + ld_off : (int64_t)idle_off;
        kk = load_words_nt<4>(a.k + seq0kv + off);
        vv = load_words_nt<4>(a.v + seq0kv + off);
    };
    auto load_q = [&](int ci, Words<4>& qq) {
        const int t0 = tb32 + ci * kChunk;
        int tq = t0 + lr;
        tq = tq < te32 ? tq : te32 - 1;
        const uint64_t off = (ci < nchunks && t0 >= ts32) ? (uint64_t)(uint32_t)tq * D32 + ld_off : idle_off;
        qq = load_words_nt<4>(a.q + seq0 + off);
    };

    // start the first loads before anything else so their latency overlaps the filter set-up
    Words<4> kpre[kPrefetch], vpre[kPrefetch], qpre[kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) {
        load_kv(i, kpre[i], vpre[i]);
        if (i + 1 < kPrefetch) load_q(i, qpre[i]);  // the last q stage is filled by the first iteration
    }

    // ---- Toeplitz operands: operand i serves d = (output tile start) - (source block start) = 16 i; in it
    // lane (li = output step, lq = source octet), element e holds h[d + li - 8 lq - e] (zero outside
    // [0, lh)), rounded to bf16.  The wave's filter goes through LDS once so the gather is not 80 global loads.
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

    // ---- register window of the last NKB source blocks (block m starts 32 m steps before the chunk)
    bf16x8_t uw[NKB];
    {
        Words<4> z = zero_words<4>();
#pragma unroll
        for (int m = 0; m < NKB; ++m) uw[m] = __builtin_bit_cast(bf16x8_t, z);
    }

    const int swz = ((lr >> 3) & 3) << 1;
    const int st_idx = lr * PPR + (lp ^ swz);
    const int rd_piece = (2 * w + (li >> 3)) ^ (lq << 1);
    const int zwr_off = li * ZROW + (16 * w + 4 * lq) * 4;  // + 16 * ZROW for the second 16-step tile
    const int zrd_off = lr * ZROW + 8 * lp * 4;

    // Post-gate and store of a finished chunk: z comes back from LDS in row layout, so the lane multiplies
    // 8 adjacent channels of one row by q and writes 16 contiguous bytes.
    auto gate_store = [&](int ci, const Words<4>& qq) {
        const int t0 = tb32 + ci * kChunk;
        const int t = t0 + lr;
        if (t0 >= ts32 && t < te32) {
            const char* zp = zst[ci & 1] + zrd_off;
            const float4 za = *reinterpret_cast<const float4*>(zp);
            const float4 zb = *reinterpret_cast<const float4*>(zp + 16);
            float qf[8];
            Pack<BF16, 8>::unpack(qq, qf);
            float y8[8] = {za.x * qf[0], za.y * qf[1], za.z * qf[2], za.w * qf[3],
                           zb.x * qf[4], zb.y * qf[5], zb.z * qf[6], zb.w * qf[7]};
            store_words_nt<4>(a.y + seq0 + ((uint64_t)(uint32_t)t * D32 + ld_off), Pack<BF16, 8>::pack(y8));
        }
    };

    // q of chunk c lives in register stage c % kPrefetch until chunk c is gated (one iteration after its
    // MFMAs); only then is that stage refilled, so no loaded value is ever copied between registers.
    // The chunk loop is unrolled by the prefetch depth so that register stages are addressed statically;
    // iterations past the last chunk (at most kPrefetch-1) run empty but keep the barriers aligned.
    for (int base = 0; base < nchunks; base += kPrefetch) {
#pragma unroll
        for (int sgi = 0; sgi < kPrefetch; ++sgi) {
            const int ci = base + sgi;
            const int64_t t0 = t_begin + (int64_t)ci * kChunk;
            const bool main_chunk = t0 >= t_start && ci < nchunks;

            // u = k * v for this lane's 8 channels of one row -> bf16 -> LDS
            {
                float kf[8], vf[8];
                Pack<BF16, 8>::unpack(kpre[sgi], kf);
                Pack<BF16, 8>::unpack(vpre[sgi], vf);
                Words<4> uu;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2)
                    uu.w[e2] = pack_bf16x2(kf[2 * e2] * vf[2 * e2], kf[2 * e2 + 1] * vf[2 * e2 + 1]);
                if constexpr (kShard)
                    if (tb32 + ci * kChunk + lr < t_old) uu = zero_words<4>();  // before the data: zeros
                stage[ci & 1][st_idx] = make_uint4(uu.w[0], uu.w[1], uu.w[2], uu.w[3]);
            }
            // refill this register stage with the chunk kPrefetch ahead
            load_kv(ci + kPrefetch, kpre[sgi], vpre[sgi]);

            __syncthreads();  // u of this chunk and z of the previous chunk are now visible

            // transposed read: element e of this lane = u[row 8 lq + e][channel 16 w + li]
#pragma unroll
            for (int m = NKB - 1; m > 0; --m) uw[m] = uw[m - 1];
            {
                const uint16_t* s16 = reinterpret_cast<const uint16_t*>(stage[ci & 1]);
                Words<4> wds;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int r0 = 8 * lq + 2 * e2;
                    const uint32_t lo = s16[((r0 * PPR + rd_piece) << 3) + (li & 7)];
                    const uint32_t hi = s16[(((r0 + 1) * PPR + rd_piece) << 3) + (li & 7)];
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
                // the lane holds z for channels 16 w + 4 lq .. +3 at steps li and 16 + li of the chunk
                char* zp = zst[ci & 1] + zwr_off;
                *reinterpret_cast<float4*>(zp) = make_float4(acc0[0], acc0[1], acc0[2], acc0[3]);
                *reinterpret_cast<float4*>(zp + 16 * ZROW) = make_float4(acc1[0], acc1[1], acc1[2], acc1[3]);
            }
            const int prev = (sgi + kPrefetch - 1) % kPrefetch;  // static after unrolling
            if (ci > 0 && ci <= nchunks) gate_store(ci - 1, qpre[prev]);
            load_q(ci - 1 + kPrefetch, qpre[prev]);
        }
    }
    if (nchunks % kPrefetch == 0) {  // the last chunk's z has not been gated inside the loop
        __syncthreads();
        gate_store(nchunks - 1, qpre[kPrefetch - 1]);
    }
}

// Time steps per workgroup of NW waves and the number of workgroups that gives.
template <int NKB>
int64_t tile_rows(const ConvShape& s, int nw, int64_t* workgroups) {
    const int64_t ncb = s.D / (16 * nw);
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        // One workgroup per CU: measured on MI355X, few large workgroups that each stream a wide piece of
        // every row beat many small ones, and each extra tile costs (NKB-1)*32 halo steps of k and v.
        const int64_t want = 256;
        int64_t tiles = want / (s.B * ncb);
        if (tiles < 1) tiles = 1;
        rows = (s.L + tiles - 1) / tiles;
        const int64_t min_rows = 4LL * kChunk * (NKB > 1 ? NKB - 1 : 1);
        if (rows < min_rows) rows = min_rows;
    }
    rows = (rows + kChunk - 1) / kChunk * kChunk;
    if (rows > (s.L + kChunk - 1) / kChunk * kChunk) rows = (s.L + kChunk - 1) / kChunk * kChunk;
    *workgroups = s.B * ((s.L + rows - 1) / rows) * ncb;
    return rows;
}

template <int NKB, int NW>
hy_status launch_nkb_nw(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    constexpr int PF = 2;  // chunks of k, v, q in flight per lane: measured best on MI355X (deeper queues ran slower)
    MrArgs a;
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.h = p.h;
    a.y = static_cast<uint16_t*>(p.y);
    a.L = s.L;
    a.D = s.D;
    a.bstride_kv = s.stride_kv();
    a.bstride_qy = s.stride_qy();
    a.hist = s.history;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * NW));
    int64_t nb = 0;
    const int64_t rows = tile_rows<NKB>(s, NW, &nb);
    a.rows = (int32_t)rows;
    a.tiles_per_seq = (int32_t)((s.L + rows - 1) / rows);
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    if (s.sharded()) return launch_kernel((mr_mfma_kernel<NKB, NW, PF, true>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
    return launch_kernel((mr_mfma_kernel<NKB, NW, PF, false>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
}

template <int NKB>
hy_status launch_nkb(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    // Widest row piece per workgroup the width allows: 16 waves = 256 channels = 512 bytes of every row,
    // then 8, then 4.  Measured on MI355X (L = 131072): 694 us with 16 waves against 787 us with 8.
    if constexpr (NKB > 13) {
        return launch_nkb_nw<NKB, 4>(p, s, st);  // one wave per SIMD: 64 channels per workgroup
    } else {
        int nw = tuning().mr_waves > 0 ? tuning().mr_waves : 16;
        if (tuning().mr_waves == 0 && tuning().mr_rows == 0) {
            // Small problems: a tile cannot be shorter than four times its halo, so wide workgroups may leave
            // compute units idle.  Take the widest workgroup that still gives every compute unit one (measured
            // at B = 1, D = 4096, lh = 128: L = 4096 28.9 us with 8 waves against 33.0 with 16; L = 2048 16.3 us
            // with 4 waves against 19.8 / 28.3; L = 512 11.9 against 14.3 / 22.5; from L = 8192 on 16 waves win).
            // "Every" means three quarters of them: a batch of 3 gives 240 wide workgroups, which beat 192 narrow
            // ones by far (B = 3, L = 8192: 161 us with 4 waves, the old choice at a threshold of 256).
            constexpr int64_t kEnough = 192;
            int64_t wg = 0;
            const bool wide_ok = NKB <= 5 && s.D % 256 == 0;
            if (wide_ok) tile_rows<NKB>(s, 16, &wg);
            if (!wide_ok || wg < kEnough) {
                nw = 8;
                if (s.D % 128 == 0) tile_rows<NKB>(s, 8, &wg);
                if (s.D % 128 != 0 || wg < kEnough) nw = 4;
            }
        }
        if constexpr (NKB <= 5) {  // 16 waves only where the kernel fits 128 registers without spilling
            if (nw == 16 && s.D % 256 == 0) return launch_nkb_nw<NKB, 16>(p, s, st);
        }
        if (nw >= 8 && s.D % 128 == 0) return launch_nkb_nw<NKB, 8>(p, s, st);
        return launch_nkb_nw<NKB, 4>(p, s, st);
    }
}

}  // namespace

hy_status launch_mr_mfma(const ConvPtrs& p, const ConvShape& s, hipStream_t st) {
    if (s.dtype != HY_BF16 || !s.gated || s.group % 16 != 0 || s.D % 64 != 0 || s.lh > 513 || s.L > 0x7fff0000LL ||
        s.D > 0x7fff0000LL)
        return HY_ERR_UNSUPPORTED;
    const int nkb = (s.lh - 1 + 31) / 32 + 1;  // 32-step source blocks that can meet a 16-step output tile
    switch (nkb) {
        case 1: return launch_nkb<1>(p, s, st);
        case 2: return launch_nkb<2>(p, s, st);
        case 3: return launch_nkb<3>(p, s, st);
        case 4: return launch_nkb<4>(p, s, st);
        case 5: return launch_nkb<5>(p, s, st);
        case 6: return launch_nkb<6>(p, s, st);
        case 7: return launch_nkb<7>(p, s, st);
        case 8: return launch_nkb<8>(p, s, st);
        case 9: return launch_nkb<9>(p, s, st);
        case 10: case 11: case 12: case 13: return launch_nkb<13>(p, s, st);  // lh <= 385
        case 14: case 15: case 16: case 17: return launch_nkb<17>(p, s, st);  // lh <= 513
        default: return HY_ERR_UNSUPPORTED;
    }
}

}  // namespace hy
