// Hyena-MR backward on the gfx950 matrix cores (bf16 operands, fp32 accumulation).
//
// With u = k*v and g = dy*q the gradients of y = q (.) (h * u) are (Sec. 2.1 Eq. 1, Sec. 3.1 Eq. 2):
//     dq = dy (.) (h * u)                                   -> the forward kernel itself, called with q := dy
//     du[s] = sum_j h[j] g[s+j],  dk = du (.) v,  dv = du (.) k
//     dh[j] = sum_{b, c in group, s} u[s] g[s+j]
// This file holds the kernel for the last two lines.  In reversed time tau = L-1-t the transposed
// convolution is again causal, du'[tau] = sum_j h[j] g'[tau-j], so the kernel IS the forward block-Toeplitz
// scheme of mr_kernels.hip (same Toeplitz operands in registers, same source window, same LDS transposition,
// same clamped prefetch) walking the sequence from its end, with g in the role of u and two post-gates.
// The filter gradient is a second contraction over the 16 channels of a group,
//     C_x[i][n] = sum_c u[tau_s + i, c] * g[tau_s - 16 x + n, c],    dh[16 x + i - n] += C_x[i][n],
// which is what v_mfma_f32_16x16x16_bf16 computes from plain row-major operands (4 adjacent channels of
// one row per lane): 2*(2 NKB - 1) extra MFMAs per chunk into 2 NKB - 1 accumulators that live in registers
// for the whole tile.  At the end of the tile each wave folds the diagonals of its accumulators into one
// partial dh row and writes it to the workspace (App. A.4: partial accumulation by block, written out
// contiguously); dh_reduce_kernel sums the partials.
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
    uint16_t* dk;
    uint16_t* dv;
    float* partial;  // [B * tiles_per_seq][D / 16][lh]: one row per (tile, 16-channel slice)
    int64_t L, D;
    int32_t lh, group;
    int32_t rows, tiles_per_seq, ncb;
};

constexpr int kChunk = 32;

template <int NKB, int NW, int PF>
__global__ __launch_bounds__(NW * 64, 2) void mr_bwd_kernel(MrBwdArgs a) {
    constexpr int PPR = 2 * NW;              // 16-byte pieces per staged row
    constexpr int CPR = 2 * PPR;             // 8-byte chunks per staged row
    constexpr int kTaps = 32 * NKB;
    constexpr int ZROW = 16 * NW * 4 + 16;
    constexpr int ND = 2 * NKB - 1;          // 16-step offsets x with a tap 16 x + i - n inside [0, lh)
    constexpr int NSLOT = NKB + 1;           // chunks of g kept for the filter gradient (+1: no write/read overlap)
    __shared__ uint4 gst[2][kChunk * PPR];             // g of the newest chunk, swizzled for the transposed read
    __shared__ uint2 gring[NSLOT][kChunk * CPR];       // g rows, 8-byte chunks XOR-swizzled by row
    __shared__ uint2 ust[2][kChunk * CPR];             // u rows of the current chunk, same layout
    __shared__ __attribute__((aligned(16))) char zst[2][kChunk * ZROW];
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
    int64_t t_begin = t_start - (int64_t)kChunk * (NKB - 1);
    if (t_begin < 0) t_begin = 0;
    const int nchunks = (int)((t_end - t_begin + kChunk - 1) / kChunk);

    const int64_t cblock0 = (int64_t)cb * 16 * NW;
    const int64_t c0 = cblock0 + 16 * w;
    const int64_t seq0 = b * L * D;

    const int lr = tid / PPR, lp = tid % PPR;
    const int64_t ld_off = cblock0 + 8 * lp;
    // element offset of reversed step tau (clamped into the tile) for this lane
    auto row_off = [&](int64_t tau) {
        tau = tau < t_end ? tau : t_end - 1;
        return seq0 + (L - 1 - tau) * D + ld_off;
    };
    // loads whose result is never used (chunk indices past the last chunk; k and v of warm-up chunks) all go to one
    // 16-byte location of the tile, the same for every lane of the workgroup: one cache line per wave
    const int64_t idle_off = seq0 + (L - t_end) * D + cblock0;
    auto load_g = [&](int ci, Words<4>& yy, Words<4>& qq) {
        const int64_t off = ci < nchunks ? row_off(t_begin + (int64_t)ci * kChunk + lr) : idle_off;
        yy = load_words_nt<4>(a.dy + off);
        qq = load_words_nt<4>(a.q + off);
    };
    auto load_kv = [&](int ci, Words<4>& kk, Words<4>& vv) {  // warm-up chunks need no k, v
        const int64_t t0 = t_begin + (int64_t)ci * kChunk;
        const int64_t off = (ci < nchunks && t0 >= t_start) ? row_off(t0 + lr) : idle_off;
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
    bf16x8_t gw[NKB];
    {
        Words<4> z = zero_words<4>();
#pragma unroll
        for (int m = 0; m < NKB; ++m) gw[m] = __builtin_bit_cast(bf16x8_t, z);
    }
    f32x4_t cacc[ND];
#pragma unroll
    for (int x = 0; x < ND; ++x) cacc[x] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

    const int swz = ((lr >> 3) & 3) << 1;
    const int st_idx = lr * PPR + (lp ^ swz);
    const int rd_piece = (2 * w + (li >> 3)) ^ (lq << 1);
    const int zwr_off = li * ZROW + (16 * w + 4 * lq) * 4;
    const int zrd_off = lr * ZROW + 8 * lp * 4;
    // 8-byte chunk layout: logical chunk c8 of row r sits at c8 ^ (r & 15)
    const int x8 = lr & 15;
    const int wr8a = lr * CPR + ((2 * lp) ^ x8), wr8b = lr * CPR + ((2 * lp + 1) ^ x8);
    const int rd8 = (4 * w + lq) ^ li;  // this lane's chunk in a row whose index is li (mod 16)

    auto gate_store = [&](int ci, const Words<4>& kk, const Words<4>& vv) {
        const int64_t t0 = t_begin + (int64_t)ci * kChunk;
        const int64_t tau = t0 + lr;
        if (t0 >= t_start && tau < t_end) {
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
            const int64_t off = seq0 + (L - 1 - tau) * D + ld_off;
            store_words_nt<4>(a.dk + off, Pack<BF16, 8>::pack(o1));
            store_words_nt<4>(a.dv + off, Pack<BF16, 8>::pack(o2));
        }
    };

    for (int base = 0; base < nchunks; base += PF) {
#pragma unroll
        for (int sgi = 0; sgi < PF; ++sgi) {
            const int ci = base + sgi;
            const int64_t t0 = t_begin + (int64_t)ci * kChunk;
            const bool main_chunk = t0 >= t_start && ci < nchunks;
            const int slot = __builtin_amdgcn_readfirstlane(ci % NSLOT);

            // g = dy*q and u = k*v of this lane's row piece, rounded to bf16, into LDS
            {
                float a8[8], b8[8];
                Pack<BF16, 8>::unpack(ypre[sgi], a8);
                Pack<BF16, 8>::unpack(qpre[sgi], b8);
                Words<4> gg;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) gg.w[e2] = pack_bf16x2(a8[2 * e2] * b8[2 * e2], a8[2 * e2 + 1] * b8[2 * e2 + 1]);
                gst[ci & 1][st_idx] = make_uint4(gg.w[0], gg.w[1], gg.w[2], gg.w[3]);
                gring[slot][wr8a] = make_uint2(gg.w[0], gg.w[1]);
                gring[slot][wr8b] = make_uint2(gg.w[2], gg.w[3]);
                Pack<BF16, 8>::unpack(kpre[sgi], a8);
                Pack<BF16, 8>::unpack(vpre[sgi], b8);
                // u of steps past the end of the tile must not reach the filter gradient
                const bool live = t0 + lr < t_end;
                Words<4> uu;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2)
                    uu.w[e2] = live ? pack_bf16x2(a8[2 * e2] * b8[2 * e2], a8[2 * e2 + 1] * b8[2 * e2 + 1]) : 0u;
                ust[ci & 1][wr8a] = make_uint2(uu.w[0], uu.w[1]);
                ust[ci & 1][wr8b] = make_uint2(uu.w[2], uu.w[3]);
            }
            load_g(ci + PF, ypre[sgi], qpre[sgi]);

            __syncthreads();

#pragma unroll
            for (int m = NKB - 1; m > 0; --m) gw[m] = gw[m - 1];
            {
                const uint16_t* s16 = reinterpret_cast<const uint16_t*>(gst[ci & 1]);
                Words<4> wds;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int r0 = 8 * lq + 2 * e2;
                    const uint32_t lo = s16[((r0 * PPR + rd_piece) << 3) + (li & 7)];
                    const uint32_t hi = s16[(((r0 + 1) * PPR + rd_piece) << 3) + (li & 7)];
                    wds.w[e2] = lo | (hi << 16);
                }
                gw[0] = __builtin_bit_cast(bf16x8_t, wds);
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
            const int prev = (sgi + PF - 1) % PF;  // static after unrolling
            if (ci > 0 && ci <= nchunks) gate_store(ci - 1, kpre[prev], vpre[prev]);
            load_kv(ci - 1 + PF, kpre[prev], vpre[prev]);
        }
    }
    if (nchunks % PF == 0) {
        __syncthreads();
        gate_store(nchunks - 1, kpre[PF - 1], vpre[PF - 1]);
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

template <int NKB, int NW>
hy_status launch_nw(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st, int64_t* nsets) {
    constexpr int PF = 3;
    MrBwdArgs a;
    a.dy = static_cast<const uint16_t*>(p.dy);
    a.q = static_cast<const uint16_t*>(p.q);
    a.k = static_cast<const uint16_t*>(p.k);
    a.v = static_cast<const uint16_t*>(p.v);
    a.h = p.h;
    a.dk = static_cast<uint16_t*>(p.dk);
    a.dv = static_cast<uint16_t*>(p.dv);
    a.partial = static_cast<float*>(ws);
    a.L = s.L;
    a.D = s.D;
    a.lh = s.lh;
    a.group = s.group;
    a.ncb = (int32_t)(s.D / (16 * NW));
    a.rows = (int32_t)mr_bwd_rows(s);
    a.tiles_per_seq = (int32_t)((s.L + a.rows - 1) / a.rows);
    *nsets = s.B * a.tiles_per_seq;
    const int64_t nb = *nsets * a.ncb;
    if (nb > 0x7fffffffLL) return HY_ERR_UNSUPPORTED;
    return launch_kernel((mr_bwd_kernel<NKB, NW, PF>), dim3((uint32_t)nb), dim3(NW * 64), st, a);
}

template <int NKB>
hy_status launch_nkb(const BwdPtrs& p, const BwdShape& s, void* ws, hipStream_t st, int64_t* nsets) {
    if (s.D % 128 == 0) return launch_nw<NKB, 8>(p, s, ws, st, nsets);
    return launch_nw<NKB, 4>(p, s, ws, st, nsets);
}

}  // namespace

bool mr_bwd_supported(const BwdShape& s) {
    return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 64 == 0 && s.lh > 8 && s.lh <= 129;
}

// time steps per workgroup: one workgroup per CU where the sequence allows it (same rule as the forward kernel)
int64_t mr_bwd_rows(const BwdShape& s) {
    const int nw = s.D % 128 == 0 ? 8 : 4;
    const int64_t ncb = s.D / (16 * nw);
    const int nkb = (s.lh - 1 + 31) / 32 + 1;
    int64_t rows = tuning().mr_rows;
    if (rows <= 0) {
        int64_t tiles = 256 / (s.B * ncb);
        if (tiles < 1) tiles = 1;
        rows = (s.L + tiles - 1) / tiles;
        const int64_t min_rows = 4LL * kChunk * (nkb > 1 ? nkb - 1 : 1);
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

// dk, dv and dh (dq comes from the forward kernel).  `ws` holds the partial filter gradients.
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
