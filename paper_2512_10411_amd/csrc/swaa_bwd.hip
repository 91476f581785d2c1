// Backward pass of the SWA + sink (+ FA Decode rows) attention, gfx950: the
// gradients that SWA-aware fine-tuning (paper Sec. 3.2.2) needs, under the same
// mask as the forward kernels (Sec. 3.2.1 / Fig. 1b, Sec. 3.1.1 / Fig. 1a).
//
// With P_ij = exp(s_ij - lse_i) on the visible pairs and 0 elsewhere:
//
//   delta_i = <dO_i, O_i>                      (= sum_j P_ij dP_ij)
//   dV_j = sum_i P_ij dO_i                     dP_ij = <dO_i, v_j>
//   dS_ij = P_ij (dP_ij - delta_i)
//   dQ_i = scale sum_j dS_ij k_j               dK_j = scale sum_i dS_ij q_i
//
// Four kernels, no atomics, results independent of scheduling:
//   * swaa_bwd_delta_kernel: delta, one pass over dO and O.
//   * swaa_bwd_dq_kernel: a workgroup owns 256 query rows (the forward's work
//     decomposition and tile schedule), walks its visible KV tiles, recomputes
//     S^T = K Q^T and dP^T = V dO^T and accumulates dQ^T += K^T dS^T.
//   * swaa_bwd_dkv_kernel: a workgroup owns 128 keys of one KV head, walks
//     every query head of the GQA group and every 64-row query tile that can
//     see them, recomputes S = Q K^T and dP = dO V^T and accumulates
//     dV^T += dO^T P and dK^T += Q^T dS.  Key tiles that hold sink
//     keys are seen by every later row: their rows beyond the band are cut into
//     segments with a workgroup each, and
//   * swaa_bwd_sink_sum_kernel adds the fp32 partial sums of those key tiles.
// Each product is a v_mfma_f32_32x32x16_bf16 with the accumulator oriented so
// that the probabilities come out in the B-operand layout of the product that
// consumes them (as in the forward kernels); operands that a product needs
// transposed are read from row-major LDS tiles with ds_read_b64_tr_b16.
// P and dS are rounded to bf16 before the second products, sums are fp32.
// The kernels in this file stage tiles through registers (the templates, used for head
// dimension 64) or by LDS DMA (dK/dV for head dimension 128) and leave instruction scheduling
// to the compiler; dQ for head dimension 128 is the hand-pipelined kernel of
// swaa_bwd_dq_pipelined.hip.  All big kernels run two waves per SIMD.
#include <atomic>
#include <cmath>

#include "swaa_bwd.h"

#include <type_traits>

namespace swaa {
namespace {

constexpr int kBq = 64;  // query rows per tile of the dK/dV kernel
constexpr int kDqBlocks = 1;  // 32-row blocks per wave of the dQ kernel

template <int D>
struct BTile {
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kChunksPerThread = kBk * kChunksPerRow / kThreads;  // 64-row tile, 256 threads
    static constexpr int kStride = D + 8;  // bf16 elements per LDS row
    static constexpr int kElems = kBk * kStride;
};

// A operand "rows of the tile x 16 of the head dimension": row 32*rb + lane%32, elements 16*ks + 8*(lane/32) ..
template <int D>
__device__ __forceinline__ bf16x8 row_frag(const __bf16 *tile, int rb, int ks, int l32, int hf) {
    return *reinterpret_cast<const bf16x8 *>(&tile[(32 * rb + l32) * BTile<D>::kStride + 16 * ks + 8 * hf]);
}

// A operand "32 of the head dimension x 16 tile rows" (the tile transposed): head-dimension block db,
// tile rows 32*rb + 16*st + 4*(lane/32) + {0..3, 8..11} -- the order in which a 32x32 accumulator hands
// its rows to the next product as a B operand.
template <int D>
__device__ __forceinline__ bf16x8 col_frag(const __bf16 *tile, int rb, int st, int db, int lane) {
    const int hf = lane >> 5, grp = lane >> 4, j16 = lane & 15;
    const int row = 32 * rb + 16 * st + 4 * hf + (j16 >> 2);
    const int col = 32 * db + 16 * (grp & 1) + 4 * (j16 & 3);
    const __bf16 *a0 = &tile[row * BTile<D>::kStride + col];
    const __bf16 *a1 = a0 + 8 * BTile<D>::kStride;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(a0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(a1));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ bool visible(int i, int j, int W, int S, int P) {
    return (j <= i) && ((i >= P) || (j > i - W) || (j < S));
}
// The same without short-circuit evaluation, for code that must stay free of branches:
// per-element branches in the softmax stage of the dK/dV kernels (sixteen elements, several
// conditions each) cost more than all of the stage's arithmetic.
__device__ __forceinline__ bool visible_in_range(int i, int j, int N, int W, int S, int P) {
    return (i < N) & (j <= i) & ((i >= P) | (j > i - W) | (j < S));
}

// ---- delta_i = <dO_i, O_i> ---------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void swaa_bwd_delta_kernel(const BwdParams p) {
    constexpr int L = D / 8;  // lanes per row
    const long long rows = (long long)p.B * p.Hq * p.N;
    const long long row = (long long)blockIdx.x * (kThreads / L) + threadIdx.x / L;
    const int c = threadIdx.x % L;
    float acc = 0.f;
    if (row < rows) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(p.dout + row * D + 8 * c);
        const bf16x8 b = *reinterpret_cast<const bf16x8 *>(p.out + row * D + 8 * c);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
    }
#pragma unroll
    for (int w = L / 2; w > 0; w >>= 1) acc += __shfl_xor(acc, w, L);
    if (row < rows && c == 0) p.delta[row] = acc;
}

// ---- dQ ------------------------------------------------------------------------------
// QB: 32-row blocks per wave.  QB = 1 runs eight waves of 32 rows (two per SIMD, so that one
// wave's exponentials overlap the other's MFMAs), QB = 2 four waves of 64 rows.
template <int D, int QB>
__global__ __launch_bounds__(512 / QB, 1) void swaa_bwd_dq_kernel(const BwdParams p) {
    using T = BTile<D>;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int TH = 512 / QB;           // threads per workgroup
    constexpr int kRows = 32 * QB;         // query rows per wave
    constexpr int kCPT = kBk * T::kChunksPerRow / TH;  // 16-byte chunks of a tile per thread
    __shared__ __attribute__((aligned(16))) __bf16 Ks[T::kElems];
    __shared__ __attribute__((aligned(16))) __bf16 Vs[T::kElems];

    WorkItem wi;
    if (!decode_work(p.f, wi)) return;
    const int hpb = wi.hpb;
    const int rows_per_wg = kWgRows / hpb;
    const int N = p.N, W = p.f.W, S = p.f.S, P = p.f.P;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;

    const int head = wi.kvh * p.f.G + wi.h0 + (wave % hpb);
    const int wg_p0 = wi.pt * rows_per_wg;
    const int wg_p1 = min(N, wg_p0 + rows_per_wg) - 1;
    const int p0 = wg_p0 + (wave / hpb) * kRows;
    const bool wave_active = p0 < N;
    const int plast = min(p0 + kRows, N) - 1;

    const int band_lo = (wg_p1 >= P) ? 0 : max(0, wg_p0 - W + 1);
    const int t_band_lo = band_lo / kBk;
    const int t_hi = wg_p1 / kBk;
    const int n_sink_tiles = min((min(S, band_lo) + kBk - 1) / kBk, t_band_lo);
    const int wbound = window_bound(p0, kRows, W, P);

    const size_t kv_base = ((size_t)wi.b * p.Hkv + wi.kvh) * (size_t)N * D;
    const __bf16 *kg = p.f.k + kv_base;
    const __bf16 *vg = p.f.v + kv_base;
    const size_t q_base = ((size_t)wi.b * p.Hq + head) * (size_t)N * D;
    const size_t r_base = ((size_t)wi.b * p.Hq + head) * (size_t)N;

    // this wave's Q and dO rows as B operands, its rows' lse (log2 units) and delta
    bf16x8 qf[QB][KS], dof[QB][KS];
    float lse2[QB], dl[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = min(p0 + 32 * qb + l32, N - 1);
        const __bf16 *qs = p.f.q + q_base + (size_t)row * D + 8 * hf;
        const __bf16 *ds = p.dout + q_base + (size_t)row * D + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[qb][ks] = *reinterpret_cast<const bf16x8 *>(qs + 16 * ks);
            dof[qb][ks] = *reinterpret_cast<const bf16x8 *>(ds + 16 * ks);
        }
        lse2[qb] = p.f.lse[r_base + row] * 1.44269504088896340736f;
        dl[qb] = p.delta[r_base + row];
    }

    f32x16 dqacc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int e = 0; e < 16; ++e) dqacc[db][qb][e] = 0.f;

    u32x4 kreg[kCPT], vreg[kCPT];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int c = 0; c < kCPT; ++c) {
            const int id = c * TH + tid;
            const int row = min(t * kBk + id / T::kChunksPerRow, N - 1);
            const int col = (id % T::kChunksPerRow) * 8;
            kreg[c] = *reinterpret_cast<const u32x4 *>(kg + (size_t)row * D + col);
            vreg[c] = *reinterpret_cast<const u32x4 *>(vg + (size_t)row * D + col);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int c = 0; c < kCPT; ++c) {
            const int id = c * TH + tid;
            const int row = id / T::kChunksPerRow;
            const int col = (id % T::kChunksPerRow) * 8;
            *reinterpret_cast<u32x4 *>(&Ks[row * T::kStride + col]) = kreg[c];
            *reinterpret_cast<u32x4 *>(&Vs[row * T::kStride + col]) = vreg[c];
        }
    };
    auto next_tile = [&](int t) {
        int n = t + 1;
        if (n == n_sink_tiles && n < t_band_lo) n = t_band_lo;
        return n;
    };

    int t = (n_sink_tiles > 0) ? 0 : t_band_lo;
    load_tile(t);
    store_tile();
    __syncthreads();
    const float c2 = p.f.scale_log2;

    while (true) {
        const int tn = next_tile(t);
        const bool has_next = tn <= t_hi;
        if (has_next) load_tile(tn);

        const int k0 = t * kBk, k_last = k0 + kBk - 1;
        const bool in_future = k0 > plast;
        const bool before_band = (plast < P) && (k_last < p0 - W + 1) && (k0 >= S);
        if (wave_active && !in_future && !before_band) {
            const bool unmasked = (k_last <= p0) && ((k0 > wbound) || (k_last < S));

            // S^T = K Q^T and dP^T = V dO^T : [64 keys] x [64 queries]
            f32x16 sacc[2][QB], dpacc[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        sacc[kb][qb][e] = 0.f;
                        dpacc[kb][qb][e] = 0.f;
                    }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 ka = row_frag<D>(Ks, kb, ks, l32, hf);
                    const bf16x8 va = row_frag<D>(Vs, kb, ks, l32, hf);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        sacc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[qb][ks], sacc[kb][qb], 0, 0, 0);
                        dpacc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, dof[qb][ks], dpacc[kb][qb], 0, 0, 0);
                    }
                }

            // P^T = exp2(s c2 - lse2) on visible pairs, dS^T = P^T (dP^T - delta), packed to bf16
            bf16x8 dsf[2][QB][2];  // [kb][qb][16-key step]
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const int qpos = p0 + 32 * qb + l32;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int key = k0 + 32 * kb + 8 * (e / 4) + 4 * hf + (e % 4);
                        float pe = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][e], c2, -lse2[qb]));
                        if (!unmasked && !visible(qpos, key, W, S, P)) pe = 0.f;
                        dsf[kb][qb][e / 8][e % 8] = (__bf16)(pe * (dpacc[kb][qb][e] - dl[qb]));
                    }
            }

            // dQ^T += K^T dS^T
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int st = 0; st < 2; ++st)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const bf16x8 a = col_frag<D>(Ks, kb, st, db, lane);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            dqacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf[kb][qb][st], dqacc[db][qb], 0, 0, 0);
                    }
        }

        if (!has_next) break;
        __syncthreads();
        store_tile();
        __syncthreads();
        t = tn;
    }

    if (!wave_active) return;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = p0 + 32 * qb + l32;
        if (row >= N) continue;
        __bf16 *orow = p.dq + q_base + (size_t)row * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(dqacc[db][qb][4 * e4 + e] * p.f.scale);
                *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * e4 + 4 * hf) = o4;
            }
    }
}

// ---- dK, dV --------------------------------------------------------------------------
// Eight waves, two per SIMD (one wave's exponentials overlap the other's MFMAs): wave w owns
// the 32 keys 32*(w%4).. of the workgroup's 128 and the 32 rows 32*(w/4).. of every 64-row
// query tile; the two row halves are added through LDS at the end.  The workgroup's K and V
// rows stay in LDS for the whole kernel (B operands of S = Q K^T and dP = dO V^T), the query
// tile's Q and dO are staged per step and read both row-wise and transposed.
constexpr int kDkvThreads = 512;
template <int D>
struct DkvSmem {
    using T = BTile<D>;
    static constexpr int kKeyTileBytes = 128 * T::kStride * 2;  // K or V rows of the workgroup's keys
    static constexpr int kQTileBytes = T::kElems * 2;
    static constexpr int kK = 0, kV = kKeyTileBytes, kQ = 2 * kKeyTileBytes, kDO = kQ + kQTileBytes,
                         kL = kDO + kQTileBytes, kDl = kL + kBq * 4, kBytes = kDl + kBq * 4;
    static_assert(2 * kKeyTileBytes >= 4 * 32 * D * 4, "the K/V area doubles as the buffer of the final sum");
};

// Which key tile's main workgroup is block `bid` (the blocks before n_extra are sink
// segments)?  Workgroups are dealt to the eight dies round-robin, and each die has its own
// L2: every die gets a contiguous run of the (batch, KV head, key tile) list, so that the
// workgroups running side by side on a die hold neighbouring key tiles, whose query tiles
// largely coincide (tile T is read by key tile kt at its step T - 2 kt).  The Q and dO
// rows then come out of L2 instead of HBM: 0.8 GB instead of 4.6 GB per launch on the
// 16k-token benchmark layer.  The sink segments stay in front, dealt round-robin: a first
// attempt that gave them to one die lost more to the imbalance than the cache gave back.
// The launch rounds the number of main workgroups up to a multiple of the die count; ids
// past the list belong to workgroups that return at once.
__device__ __forceinline__ int dkv_main_item(unsigned bid, int n_extra) {
    const unsigned per_die = (gridDim.x - (unsigned)n_extra) / kXcds;
    return (int)((bid % kXcds) * per_die + (bid - (unsigned)n_extra) / kXcds);
}

template <int D>
__global__ __launch_bounds__(kDkvThreads, 1) void swaa_bwd_dkv_kernel(const BwdParams p) {
    using T = BTile<D>;
    using M = DkvSmem<D>;
    constexpr int KS = D / 16, DB = D / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __bf16 *Ks = reinterpret_cast<__bf16 *>(smem + M::kK);
    __bf16 *Vs = reinterpret_cast<__bf16 *>(smem + M::kV);
    __bf16 *Qs = reinterpret_cast<__bf16 *>(smem + M::kQ);
    __bf16 *dOs = reinterpret_cast<__bf16 *>(smem + M::kDO);
    float *Ls = reinterpret_cast<float *>(smem + M::kL);    // lse of the tile's rows, log2 units
    float *Dls = reinterpret_cast<float *>(smem + M::kDl);  // their delta

    const int N = p.N, W = p.f.W, S = p.f.S, P = p.f.P, G = p.f.G;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int kq = wave & 3, qb = wave >> 2;  // key block and row half of this wave
    // Work list: first the segments of the sink key tiles (rows beyond the band), then one
    // workgroup per key tile of 128 keys (band rows; for key tiles without sinks also the
    // generated rows).  Under a causal mask the first key tiles are seen by the most rows.
    const int n_kt = (N + 127) / 128;
    const int n_extra = p.B * p.Hkv * p.n_sink_kt * p.n_seg;
    const unsigned bid = blockIdx.x;
    int kt, pair, seg;  // seg: -1 for a key tile's main workgroup
    if ((int)bid < n_extra) {
        seg = bid % p.n_seg;
        kt = (bid / p.n_seg) % p.n_sink_kt;
        pair = bid / (p.n_seg * p.n_sink_kt);
    } else {
        const int id = dkv_main_item(bid, n_extra);
        if (id >= p.B * p.Hkv * n_kt) return;  // (the grid is rounded up to a multiple of eight)
        seg = -1;
        kt = id % n_kt;
        pair = id / n_kt;
    }
    const bool sink_kt = kt < p.n_sink_kt;  // results go to the partial-sum workspace
    const int b = pair / p.Hkv, kvh = pair % p.Hkv;
    const int k0 = kt * 128, k1 = min(k0 + 127, N - 1);  // the workgroup's keys
    const int kw0 = k0 + 32 * kq, kw1 = kw0 + 31;         // this wave's keys
    const int key = kw0 + l32;                            // this lane's key column
    const bool wave_active = kw0 < N;

    // the workgroup's K and V rows -> LDS (rows past the end repeat the last key; they stay invisible)
    {
        const size_t kv_base = ((size_t)b * p.Hkv + kvh) * (size_t)N * D;
#pragma unroll
        for (int c = 0; c < 128 * T::kChunksPerRow / kDkvThreads; ++c) {
            const int id = c * kDkvThreads + tid;
            const int row = id / T::kChunksPerRow, col = (id % T::kChunksPerRow) * 8;
            const size_t g = kv_base + (size_t)min(k0 + row, N - 1) * D + col;
            *reinterpret_cast<u32x4 *>(&Ks[row * T::kStride + col]) = *reinterpret_cast<const u32x4 *>(p.f.k + g);
            *reinterpret_cast<u32x4 *>(&Vs[row * T::kStride + col]) = *reinterpret_cast<const u32x4 *>(p.f.v + g);
        }
    }
    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            dkacc[db][e] = 0.f;
            dvacc[db][e] = 0.f;
        }

    // query tiles (64 rows) with a row that sees one of the workgroup's keys: the band tiles
    // tq_lo .. tq_band_hi, then -- if a key is a sink, or there are generated rows -- the rest.
    // For a sink key tile the rest is cut into segments: the main workgroup keeps the band.
    const int tq_last = (N - 1) / kBq;
    const int tq_band_hi = min(N - 1, k1 + W - 1) / kBq;
    int tq_lo = k0 / kBq;
    int n_band = tq_band_hi - tq_lo + 1;
    int tq_x = tq_last + 1, tq_x_end = tq_last;  // second range
    if (sink_kt) {
        if (seg >= 0) {
            n_band = 0;
            tq_x = tq_band_hi + 1 + seg * p.seg_tiles;
            tq_x_end = min(tq_last, tq_x + p.seg_tiles - 1);
        }
    } else if (P < N) {
        tq_x = max(tq_band_hi + 1, P / kBq);
    }
    const int n_tiles = n_band + max(0, tq_x_end - tq_x + 1);
    auto tile_of = [&](int n) { return n < n_band ? tq_lo + n : tq_x + (n - n_band); };

    const float c2 = p.f.scale_log2;
    constexpr int kCPT = kBk * T::kChunksPerRow / kDkvThreads;
    u32x4 qreg[kCPT], dreg[kCPT];
    float lreg = 0.f, dlreg = 0.f;
    auto load_tile = [&](int head, int tq) {
        const size_t base = ((size_t)b * p.Hq + head) * (size_t)N;
#pragma unroll
        for (int c = 0; c < kCPT; ++c) {
            const int id = c * kDkvThreads + tid;
            const int row = min(tq * kBq + id / T::kChunksPerRow, N - 1);
            const int col = (id % T::kChunksPerRow) * 8;
            qreg[c] = *reinterpret_cast<const u32x4 *>(p.f.q + (base + row) * D + col);
            dreg[c] = *reinterpret_cast<const u32x4 *>(p.dout + (base + row) * D + col);
        }
        if (tid < kBq) {
            const int row = min(tq * kBq + tid, N - 1);
            lreg = p.f.lse[base + row] * 1.44269504088896340736f;
            dlreg = p.delta[base + row];
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int c = 0; c < kCPT; ++c) {
            const int id = c * kDkvThreads + tid;
            const int row = id / T::kChunksPerRow;
            const int col = (id % T::kChunksPerRow) * 8;
            *reinterpret_cast<u32x4 *>(&Qs[row * T::kStride + col]) = qreg[c];
            *reinterpret_cast<u32x4 *>(&dOs[row * T::kStride + col]) = dreg[c];
        }
        if (tid < kBq) {
            Ls[tid] = lreg;
            Dls[tid] = dlreg;
        }
    };

    const int total = G * n_tiles;  // (head, tile) steps, head-major
    int step = 0;
    if (total > 0) {
        load_tile(kvh * G, tile_of(0));
        store_tile();
    }
    __syncthreads();

    while (total > 0) {
        const bool has_next = step + 1 < total;
        if (has_next) load_tile(kvh * G + (step + 1) / n_tiles, tile_of((step + 1) % n_tiles));

        const int tq = tile_of(step % n_tiles);
        const int i0 = tq * kBq + 32 * qb, i1 = i0 + 31;  // this wave's rows of the tile
        // can any of them see any key of this wave?
        const bool sees = (i0 < N) && (i1 >= kw0) && ((i0 < kw1 + W) || (kw0 < S) || (i1 >= P));
        if (wave_active && sees) {
            // all 32 x 32 pairs visible: rows at or below the keys' diagonal, inside every row's window
            // (or the keys are sinks, or the rows are generated tokens), and no row past the end
            const bool unmasked = (kw1 <= i0) && (i1 < N) && ((i1 - kw0 < W) || (kw1 < S) || (i0 >= P));

            // S = Q K^T and dP = dO V^T : [32 queries] x [32 keys]
            f32x16 sacc, dpacc;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                sacc[e] = 0.f;
                dpacc[e] = 0.f;
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag<D>(Qs, qb, ks, l32, hf),
                                                               row_frag<D>(Ks, kq, ks, l32, hf), sacc, 0, 0, 0);
                dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag<D>(dOs, qb, ks, l32, hf),
                                                                row_frag<D>(Vs, kq, ks, l32, hf), dpacc, 0, 0, 0);
            }

            // P and dS in the accumulator layout (row 8 (e/4) + 4 hf + e%4, column = this lane's key)
            bf16x8 pf[2], dsf[2];  // [16-row step]
            // (one uniform branch per tile, none per element: see visible_in_range)
            auto softmax_stage = [&](auto masked) {
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int r4 = 32 * qb + 8 * e4 + 4 * hf;
                    const float4 l4 = *reinterpret_cast<const float4 *>(&Ls[r4]);
                    const float4 d4 = *reinterpret_cast<const float4 *>(&Dls[r4]);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                    const float dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int e = 4 * e4 + x;
                        const int row = tq * kBq + r4 + x;
                        float pe = __builtin_amdgcn_exp2f(fmaf(sacc[e], c2, -lv[x]));
                        if (decltype(masked)::value) pe = visible_in_range(row, key, N, W, S, P) ? pe : 0.f;
                        pf[e / 8][e % 8] = (__bf16)pe;
                        dsf[e / 8][e % 8] = (__bf16)(pe * (dpacc[e] - dv4[x]));
                    }
                }
            };
            if (unmasked)
                softmax_stage(std::false_type{});
            else
                softmax_stage(std::true_type{});

            // dV^T += dO^T P,  dK^T += Q^T dS
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    dvacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(col_frag<D>(dOs, qb, st, db, lane), pf[st], dvacc[db], 0, 0, 0);
                    dkacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(col_frag<D>(Qs, qb, st, db, lane), dsf[st], dkacc[db], 0, 0, 0);
                }
        }

        if (!has_next) break;
        __syncthreads();
        store_tile();
        __syncthreads();
        ++step;
    }

    // ---- add the two row halves: waves 4..7 hand their sums to waves 0..3 through LDS
    // (the K/V area, which nobody reads any more), first dK, then dV ----
    float *xbuf = reinterpret_cast<float *>(smem);  // [4 key blocks][D][32 key columns]
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        __syncthreads();
        if (qb == 1) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int d = 32 * db + 8 * (e / 4) + 4 * hf + (e % 4);
                    xbuf[(kq * D + d) * 32 + l32] = which == 0 ? dkacc[db][e] : dvacc[db][e];
                }
        }
        __syncthreads();
        if (qb == 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int d = 32 * db + 8 * (e / 4) + 4 * hf + (e % 4);
                    const float other = xbuf[(kq * D + d) * 32 + l32];
                    if (which == 0)
                        dkacc[db][e] += other;
                    else
                        dvacc[db][e] += other;
                }
        }
    }
    if (qb != 0) return;

    if (sink_kt) {
        // fp32 partial sums of all 128 key columns (columns past the end hold zeros)
        float *slot = p.partial + ((((size_t)pair * p.n_sink_kt + kt) * (p.n_seg + 1) + (seg + 1)) * 2) * (size_t)(128 * D);
        float *pk = slot + (size_t)(32 * kq + l32) * D, *pv = pk + 128 * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const float4 k4 = {dkacc[db][4 * e4], dkacc[db][4 * e4 + 1], dkacc[db][4 * e4 + 2], dkacc[db][4 * e4 + 3]};
                const float4 v4 = {dvacc[db][4 * e4], dvacc[db][4 * e4 + 1], dvacc[db][4 * e4 + 2], dvacc[db][4 * e4 + 3]};
                *reinterpret_cast<float4 *>(pk + 32 * db + 8 * e4 + 4 * hf) = k4;
                *reinterpret_cast<float4 *>(pv + 32 * db + 8 * e4 + 4 * hf) = v4;
            }
    } else if (key < N) {
        const size_t row = (((size_t)b * p.Hkv + kvh) * (size_t)N + key) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 k4, v4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    k4[e] = (__bf16)(dkacc[db][4 * e4 + e] * p.f.scale);
                    v4[e] = (__bf16)dvacc[db][4 * e4 + e];
                }
                *reinterpret_cast<bf16x4 *>(p.dk + row + 32 * db + 8 * e4 + 4 * hf) = k4;
                *reinterpret_cast<bf16x4 *>(p.dv + row + 32 * db + 8 * e4 + 4 * hf) = v4;
            }
    }
}

// ---- dK, dV, head dimension 128: tiles by LDS DMA -------------------------------------------
// Same decomposition, arithmetic and summation order as swaa_bwd_dkv_kernel; what differs is
// how the tiles reach LDS and how they lie there.  K, V (once per workgroup) and the query
// tile's Q and dO (per step, two buffers each) travel HBM -> LDS with global_load_lds_dwordx4,
// no register staging and no store phase: one barrier per step instead of two.  Rows are 256
// bytes without padding; 16-byte chunk c of row r lies at chunk c ^ g(r), g(r) = ((r & 3) << 2)
// | ((r >> 2) & 3), applied on the global side of the copy.  That one layout serves both read
// patterns without bank conflicts: 16 consecutive rows reading the same logical chunk
// (ds_read_b128 row fragments: g takes 16 different values) and 4 consecutive rows reading the
// same 64 bytes (ds_read_b64_tr_b16 transposed fragments: the upper two bits of g differ).
// This kernel declares no static LDS: its dynamic LDS starts at address 0 and all LDS accesses
// below use plain byte addresses.
namespace dma128 {
constexpr int kD = 128, kRowBytes = 256;
constexpr int kAhead = 2;  // MFMAs between an LDS operand read and its use
constexpr int kKeyTileBytes = 128 * kRowBytes;  // 32 KiB: the workgroup's K rows, or V rows
constexpr int kQTileBytes = kBq * kRowBytes;    // 16 KiB
constexpr int kK = 0, kV = kKeyTileBytes, kQ = 2 * kKeyTileBytes, kDO = kQ + 2 * kQTileBytes, kL = kDO + 2 * kQTileBytes,
              kDl = kL + 2 * kBq * 4, kBytes = kDl + 2 * kBq * 4;
static_assert(2 * kKeyTileBytes >= 4 * 32 * kD * 4, "the K/V area doubles as the buffer of the final sum");
__device__ __forceinline__ bf16x8 lds16(uint32_t addr) {
    return *(const bf16x8 __attribute__((address_space(3))) *)(uintptr_t)addr;
}
__device__ __forceinline__ s16x4 lds8_tr(uint32_t addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(uintptr_t)addr);
}
}  // namespace dma128

__global__ __launch_bounds__(kDkvThreads, 1) void swaa_bwd_dkv_dma_kernel(const BwdParams p) {
    using namespace dma128;
    constexpr int D = kD, KS = D / 16, DB = D / 32;

    const int N = p.N, W = p.f.W, S = p.f.S, P = p.f.P, G = p.f.G;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int kq = wave & 3, qb = wave >> 2;  // key block and row half of this wave
    // (work list as in swaa_bwd_dkv_kernel)
    const int n_kt = (N + 127) / 128;
    const int n_extra = p.B * p.Hkv * p.n_sink_kt * p.n_seg;
    const unsigned bid = blockIdx.x;
    int kt, pair, seg;  // seg: -1 for a key tile's main workgroup
    if ((int)bid < n_extra) {
        seg = bid % p.n_seg;
        kt = (bid / p.n_seg) % p.n_sink_kt;
        pair = bid / (p.n_seg * p.n_sink_kt);
    } else {
        const int id = dkv_main_item(bid, n_extra);
        if (id >= p.B * p.Hkv * n_kt) return;  // (the grid is rounded up to a multiple of eight)
        seg = -1;
        kt = id % n_kt;
        pair = id / n_kt;
    }
    const bool sink_kt = kt < p.n_sink_kt;  // results go to the partial-sum workspace
    const int b = pair / p.Hkv, kvh = pair % p.Hkv;
    const int k0 = kt * 128, k1 = min(k0 + 127, N - 1);  // the workgroup's keys
    const int kw0 = k0 + 32 * kq, kw1 = kw0 + 31;         // this wave's keys
    const int key = kw0 + l32;                            // this lane's key column
    const bool wave_active = kw0 < N;

    // ---- HBM -> LDS copies: one wave instruction moves 64 x 16 bytes = 4 rows; the LDS side
    // is linear in the lane id, LDS address = M0 + 16 * lane.  Rows past the end of the
    // sequence repeat its last row (they stay invisible), so that the reads stay in bounds.
    const int lrow = lane >> 4, lchk = lane & 15;
    auto copy16 = [](const char *g, uint32_t lds) {
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds) : "memory");
    };
    // rows [4 ii, 4 ii + 4) of a tile whose first row is row `first` of a [N][D] matrix
    auto copy_rows = [&](const __bf16 *mat, int first, int ii, uint32_t tile) {
        const int r = 4 * ii + lrow;
        const int g = (lrow << 2) | (ii & 3);  // g(r): r & 3 = lrow, (r >> 2) & 3 = ii & 3
        const char *src = reinterpret_cast<const char *>(mat + (size_t)min(first + r, N - 1) * D) + ((lchk ^ g) << 4);
        copy16(src, tile + (uint32_t)(ii * 1024));
    };
    {
        const size_t kv_base = ((size_t)b * p.Hkv + kvh) * (size_t)N * D;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            copy_rows(p.f.k + kv_base, k0, 4 * wave + i, kK);
            copy_rows(p.f.v + kv_base, k0, 4 * wave + i, kV);
        }
    }
    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            dkacc[db][e] = 0.f;
            dvacc[db][e] = 0.f;
        }

    // query tiles (as in swaa_bwd_dkv_kernel)
    const int tq_last = (N - 1) / kBq;
    const int tq_band_hi = min(N - 1, k1 + W - 1) / kBq;
    int tq_lo = k0 / kBq;
    int n_band = tq_band_hi - tq_lo + 1;
    int tq_x = tq_last + 1, tq_x_end = tq_last;  // second range
    if (sink_kt) {
        if (seg >= 0) {
            n_band = 0;
            tq_x = tq_band_hi + 1 + seg * p.seg_tiles;
            tq_x_end = min(tq_last, tq_x + p.seg_tiles - 1);
        }
    } else if (P < N) {
        tq_x = max(tq_band_hi + 1, P / kBq);
    }
    const int n_tiles = n_band + max(0, tq_x_end - tq_x + 1);
    auto tile_of = [&](int n) { return n < n_band ? tq_lo + n : tq_x + (n - n_band); };

    const float c2 = p.f.scale_log2;
    float lreg = 0.f, dlreg = 0.f;
    // step `st` = (head, query tile): its Q and dO rows into buffer `buf`, its lse and delta into registers
    auto request_tile = [&](int st, int buf) {
        const int head = kvh * G + st / n_tiles, tq = tile_of(st % n_tiles);
        const size_t base = ((size_t)b * p.Hq + head) * (size_t)N;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            copy_rows(p.f.q + base * D, tq * kBq, 2 * wave + i, (uint32_t)(kQ + buf * kQTileBytes));
            copy_rows(p.dout + base * D, tq * kBq, 2 * wave + i, (uint32_t)(kDO + buf * kQTileBytes));
        }
        // (asked for here, first touched in publish_rows at the end of the step: any arithmetic on
        // them right away would make this wave wait for the loads, and with them for the copies above)
        if (tid < kBq) {
            const int row = min(tq * kBq + tid, N - 1);
            lreg = p.f.lse[base + row];
            dlreg = p.delta[base + row];
        }
    };
    auto publish_rows = [&](int buf) {
        if (tid < kBq) {
            *(float __attribute__((address_space(3))) *)(uintptr_t)(kL + buf * kBq * 4 + tid * 4) = lreg * 1.44269504088896340736f;
            *(float __attribute__((address_space(3))) *)(uintptr_t)(kDl + buf * kBq * 4 + tid * 4) = dlreg;
        }
    };

    // per-lane fragment addresses inside a tile (swizzle folded in)
    //  * row fragment, k-step ks: row 32 rb + l32, logical chunk 2 ks + hf:  row_lane ^ (ks << 5), + 32 rb rows
    //  * transposed fragment, 16-row step st, head-dimension block db: rows 32 rb + 16 st + 4 hf + j16/4 (lo)
    //    and 8 further (hi), logical chunk 4 db + 2 (grp & 1) + (j16 & 3) / 2:  col_lane ^ (db << 6), + rows
    const int gl = ((l32 & 3) << 2) | ((l32 >> 2) & 3);
    const uint32_t row_lane = (uint32_t)(l32 * kRowBytes + ((hf ^ gl) << 4));
    const int grp = lane >> 4, j16 = lane & 15;
    const int rr = 4 * hf + (j16 >> 2);
    const int cl = 2 * (grp & 1) + ((j16 & 3) >> 1);
    const uint32_t col_lo = (uint32_t)(rr * kRowBytes + ((((rr & 3) << 2) | (cl ^ hf)) << 4) + 8 * (j16 & 1));
    const uint32_t col_hi = (uint32_t)((rr + 8) * kRowBytes + ((((rr & 3) << 2) | (cl ^ (hf + 2))) << 4) + 8 * (j16 & 1));
    auto row_frag_at = [&](uint32_t tile, int rb, int ks) {
        return lds16(tile + (uint32_t)(32 * rb * kRowBytes) + (row_lane ^ (uint32_t)(ks << 5)));
    };
    auto col_frag_at = [&](uint32_t tile, int rb, int st, int db) {
        const uint32_t off = tile + (uint32_t)((32 * rb + 16 * st) * kRowBytes);
        const s16x4 lo = lds8_tr(off + (col_lo ^ (uint32_t)(db << 6)));
        const s16x4 hi = lds8_tr(off + (col_hi ^ (uint32_t)(db << 6)));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    const int total = G * n_tiles;  // (head, tile) steps, head-major
    if (total > 0) {
        request_tile(0, 0);
        publish_rows(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): this wave's copies have landed
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    for (int step = 0; step < total; ++step) {
        const int buf = step & 1;
        const bool has_next = step + 1 < total;
        // the other buffers were last read one step ago, before the barrier that ended it
        if (has_next) request_tile(step + 1, buf ^ 1);

        const uint32_t Qs = (uint32_t)(kQ + buf * kQTileBytes), dOs = (uint32_t)(kDO + buf * kQTileBytes);
        const int tq = tile_of(step % n_tiles);
        const int i0 = tq * kBq + 32 * qb, i1 = i0 + 31;  // this wave's rows of the tile
        // can any of them see any key of this wave?
        const bool sees = (i0 < N) && (i1 >= kw0) && ((i0 < kw1 + W) || (kw0 < S) || (i1 >= P));
        if (wave_active && sees) {
            // all 32 x 32 pairs visible: rows at or below the keys' diagonal, inside every row's window
            // (or the keys are sinks, or the rows are generated tokens), and no row past the end
            const bool unmasked = (kw1 <= i0) && (i1 < N) && ((i1 - kw0 < W) || (kw1 < S) || (i0 >= P));

            // S = Q K^T and dP = dO V^T : [32 queries] x [32 keys]
            f32x16 sacc, dpacc;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                sacc[e] = 0.f;
                dpacc[e] = 0.f;
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag_at(Qs, qb, ks), row_frag_at(kK, kq, ks), sacc, 0, 0, 0);
                dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag_at(dOs, qb, ks), row_frag_at(kV, kq, ks), dpacc, 0, 0, 0);
            }
            // operand reads run kAhead MFMAs ahead of their use (two reads per MFMA)
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
            for (int i = 0; i < 2 * KS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }

            // P and dS in the accumulator layout (row 8 (e/4) + 4 hf + e%4, column = this lane's key)
            bf16x8 pf[2], dsf[2];  // [16-row step]
            // (one uniform branch per tile, none per element: see visible_in_range)
            auto softmax_stage = [&](auto masked) {
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int r4 = 32 * qb + 8 * e4 + 4 * hf;
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    const f32x4 l4 = *(const f32x4 __attribute__((address_space(3))) *)(uintptr_t)(kL + buf * kBq * 4 + r4 * 4);
                    const f32x4 d4 = *(const f32x4 __attribute__((address_space(3))) *)(uintptr_t)(kDl + buf * kBq * 4 + r4 * 4);
                    const float lv[4] = {l4[0], l4[1], l4[2], l4[3]};
                    const float dv4[4] = {d4[0], d4[1], d4[2], d4[3]};
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int e = 4 * e4 + x;
                        const int row = tq * kBq + r4 + x;
                        float pe = __builtin_amdgcn_exp2f(fmaf(sacc[e], c2, -lv[x]));
                        if (decltype(masked)::value) pe = visible_in_range(row, key, N, W, S, P) ? pe : 0.f;
                        pf[e / 8][e % 8] = (__bf16)pe;
                        dsf[e / 8][e % 8] = (__bf16)(pe * (dpacc[e] - dv4[x]));
                    }
                }
            };
            if (unmasked)
                softmax_stage(std::false_type{});
            else
                softmax_stage(std::true_type{});

            // dV^T += dO^T P,  dK^T += Q^T dS
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    dvacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(col_frag_at(dOs, qb, st, db), pf[st], dvacc[db], 0, 0, 0);
                    dkacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(col_frag_at(Qs, qb, st, db), dsf[st], dkacc[db], 0, 0, 0);
                }
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 1);
#pragma unroll
            for (int i = 0; i < 4 * DB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
            }
        }

        if (has_next) publish_rows(buf ^ 1);
        // the next tile has landed (this wave's part, then everybody's), this one is free afterwards
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

    // ---- add the two row halves: waves 4..7 hand their sums to waves 0..3 through LDS
    // (the K/V area, which nobody reads any more), first dK, then dV ----
    // [4 key blocks][D][32 key columns] floats from LDS address 0
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        if (which) __syncthreads();
        if (qb == 1) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int d = 32 * db + 8 * (e / 4) + 4 * hf + (e % 4);
                    *(float __attribute__((address_space(3))) *)(uintptr_t)(((kq * D + d) * 32 + l32) * 4) =
                        which == 0 ? dkacc[db][e] : dvacc[db][e];
                }
        }
        __syncthreads();
        if (qb == 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int d = 32 * db + 8 * (e / 4) + 4 * hf + (e % 4);
                    const float other = *(const float __attribute__((address_space(3))) *)(uintptr_t)(((kq * D + d) * 32 + l32) * 4);
                    if (which == 0)
                        dkacc[db][e] += other;
                    else
                        dvacc[db][e] += other;
                }
        }
    }
    if (qb != 0) return;

    if (sink_kt) {
        // fp32 partial sums of all 128 key columns (columns past the end hold zeros)
        float *slot = p.partial + ((((size_t)pair * p.n_sink_kt + kt) * (p.n_seg + 1) + (seg + 1)) * 2) * (size_t)(128 * D);
        float *pk = slot + (size_t)(32 * kq + l32) * D, *pv = pk + 128 * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const float4 k4 = {dkacc[db][4 * e4], dkacc[db][4 * e4 + 1], dkacc[db][4 * e4 + 2], dkacc[db][4 * e4 + 3]};
                const float4 v4 = {dvacc[db][4 * e4], dvacc[db][4 * e4 + 1], dvacc[db][4 * e4 + 2], dvacc[db][4 * e4 + 3]};
                *reinterpret_cast<float4 *>(pk + 32 * db + 8 * e4 + 4 * hf) = k4;
                *reinterpret_cast<float4 *>(pv + 32 * db + 8 * e4 + 4 * hf) = v4;
            }
    } else if (key < N) {
        const size_t row = (((size_t)b * p.Hkv + kvh) * (size_t)N + key) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 k4, v4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    k4[e] = (__bf16)(dkacc[db][4 * e4 + e] * p.f.scale);
                    v4[e] = (__bf16)dvacc[db][4 * e4 + e];
                }
                *reinterpret_cast<bf16x4 *>(p.dk + row + 32 * db + 8 * e4 + 4 * hf) = k4;
                *reinterpret_cast<bf16x4 *>(p.dv + row + 32 * db + 8 * e4 + 4 * hf) = v4;
            }
    }
}

// dK, dV of the sink key tiles: sum of the band part and the segments, in a fixed order.
template <int D>
__global__ __launch_bounds__(kThreads) void swaa_bwd_sink_sum_kernel(const BwdParams p) {
    // one thread per 4 consecutive head-dimension elements of one key
    const long long per_kt = 128LL * D / 4;
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long total = (long long)p.B * p.Hkv * p.n_sink_kt * per_kt;
    if (idx >= total) return;
    const int e = (int)(idx % per_kt);
    const long long kt_id = idx / per_kt;  // pair * n_sink_kt + kt
    const int kt = (int)(kt_id % p.n_sink_kt);
    const long long pair = kt_id / p.n_sink_kt;
    const int key = kt * 128 + e / (D / 4);
    const int d = (e % (D / 4)) * 4;
    if (key >= p.N) return;
    const float *slot = p.partial + (kt_id * (p.n_seg + 1) * 2) * (size_t)(128 * D) + (size_t)(e / (D / 4)) * D + d;
    float4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s <= p.n_seg; ++s) {
        const float4 a = *reinterpret_cast<const float4 *>(slot + (size_t)s * 2 * 128 * D);
        const float4 c = *reinterpret_cast<const float4 *>(slot + (size_t)s * 2 * 128 * D + 128 * D);
        sk.x += a.x; sk.y += a.y; sk.z += a.z; sk.w += a.w;
        sv.x += c.x; sv.y += c.y; sv.z += c.z; sv.w += c.w;
    }
    const size_t row = ((size_t)pair * p.N + key) * D + d;
    bf16x4 k4 = {(__bf16)(sk.x * p.f.scale), (__bf16)(sk.y * p.f.scale), (__bf16)(sk.z * p.f.scale), (__bf16)(sk.w * p.f.scale)};
    bf16x4 v4 = {(__bf16)sv.x, (__bf16)sv.y, (__bf16)sv.z, (__bf16)sv.w};
    *reinterpret_cast<bf16x4 *>(p.dk + row) = k4;
    *reinterpret_cast<bf16x4 *>(p.dv + row) = v4;
}

template <int D>
hipError_t launch_bwd_d(const BwdParams &p, hipStream_t stream) {
    const long long rows = (long long)p.B * p.Hq * p.N;
    const int rows_per_block = kThreads / (D / 8);
    hipLaunchKernelGGL(swaa_bwd_delta_kernel<D>, dim3((unsigned)((rows + rows_per_block - 1) / rows_per_block)),
                       dim3(kThreads), 0, stream, p);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    // more than 64 KiB of LDS per workgroup has to be requested once per device
    static std::atomic<unsigned long long> configured{0};
    int dev = 0;
    err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    const unsigned long long bit = 1ull << (dev & 63);
    const bool first_time = !(configured.load(std::memory_order_acquire) & bit);
    if (D == 128)
        err = launch_bwd_dq_pipelined_d128(p, stream);  // swaa_bwd_dq_pipelined.hip
    else
        hipLaunchKernelGGL((swaa_bwd_dq_kernel<D, kDqBlocks>), dim3((unsigned)(p.f.chunk * kXcds)), dim3(512 / kDqBlocks), 0,
                           stream, p);
    if (err == hipSuccess) err = hipGetLastError();
    if (err != hipSuccess) return err;
    const long long n_kt = (p.N + 127) / 128;
    const long long pairs = (long long)p.B * p.Hkv;
    if (first_time) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&swaa_bwd_dkv_kernel<D>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, DkvSmem<D>::kBytes);
        if (err != hipSuccess) return err;
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&swaa_bwd_dkv_dma_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, dma128::kBytes);
        if (err != hipSuccess) return err;
        configured.fetch_or(bit, std::memory_order_release);
    }
    // sink segments first (the longest items), then the key tiles' main workgroups, their number
    // rounded up to a multiple of the die count (dkv_main_item)
    const long long n_main = (pairs * n_kt + kXcds - 1) / kXcds * kXcds;
    const dim3 dkv_grid((unsigned)(pairs * (long long)p.n_sink_kt * p.n_seg + n_main));
    if (D == 128)
        hipLaunchKernelGGL(swaa_bwd_dkv_dma_kernel, dkv_grid, dim3(kDkvThreads), dma128::kBytes, stream, p);
    else
        hipLaunchKernelGGL(swaa_bwd_dkv_kernel<D>, dkv_grid, dim3(kDkvThreads), DkvSmem<D>::kBytes, stream, p);
    err = hipGetLastError();
    if (err != hipSuccess || p.n_sink_kt == 0) return err;
    const long long threads = pairs * p.n_sink_kt * (128LL * D / 4);
    hipLaunchKernelGGL(swaa_bwd_sink_sum_kernel<D>, dim3((unsigned)((threads + kThreads - 1) / kThreads)), dim3(kThreads),
                       0, stream, p);
    return hipGetLastError();
}

}  // namespace

void plan_bwd(BwdParams &p) {
    const int N = p.N, W = p.f.W, S = p.f.S;
    p.n_sink_kt = 0;
    p.n_seg = 0;
    p.seg_tiles = 1;
    // rows beyond the band of the last sink key: only worth separate workgroups if there are any
    const int tq_last = (N - 1) / kBq;
    const int first_beyond = (min(N - 1, 127 + W - 1)) / kBq + 1;  // of key tile 0, the longest range
    if (S == 0 || first_beyond > tq_last) return;
    p.n_sink_kt = (min(S, N) + 127) / 128;
    const int range = tq_last - first_beyond + 1;
    // segments about as long as an ordinary key tile's band, but at most 512 of them in all
    const int band_tiles = (W + 127) / kBq + 1;
    long long seg = band_tiles;
    const long long groups = (long long)p.B * p.Hkv * p.n_sink_kt;
    while ((range + seg - 1) / seg * groups > 512) seg *= 2;
    p.seg_tiles = (int)seg;
    p.n_seg = (int)((range + seg - 1) / seg);
}

long long bwd_workspace_floats(const BwdParams &p, int D) {
    const long long rows = ((long long)p.B * p.Hq * p.N + 3) / 4 * 4;  // the partial sums start 16-byte aligned
    return rows + (long long)p.B * p.Hkv * p.n_sink_kt * (p.n_seg + 1) * 2 * 128 * D;
}

hipError_t launch_bwd(const BwdParams &p, int D, hipStream_t stream) {
    return D == 128 ? launch_bwd_d<128>(p, stream) : launch_bwd_d<64>(p, stream);
}

}  // namespace swaa
