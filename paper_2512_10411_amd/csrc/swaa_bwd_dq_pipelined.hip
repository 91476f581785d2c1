// dQ of the SWA + sink (+ FA Decode rows) attention, head dimension 128, gfx950: the
// software-pipelined version of swaa_bwd_dq_kernel (same formulas, see swaa_bwd.hip:
// dS_ij = P_ij (dP_ij - delta_i), dQ_i = scale sum_j dS_ij k_j under the mask of paper
// Sec. 3.2.1 / Fig. 1b and Sec. 3.1.1 / Fig. 1a; the gradients that SWA-aware fine-tuning,
// Sec. 3.2.2, needs).
//
// Built like the pipelined forward kernel: a workgroup owns 256 query rows on one KV head
// (the forward's work decomposition and tile schedule), eight waves of 32 rows, two per
// SIMD; K and V tiles of 64 keys travel HBM -> LDS by global_load_lds_dwordx4 into rings
// of three buffers, one barrier per tile.  A wave works on halves of 32 keys in three stages:
//   A  S^T = K Q^T and dP^T = V dO^T      16 MFMAs, Q and dO rows parked in AccVGPRs
//   B  dS^T = P^T (dP^T - delta), P^T = exp2(S^T c2 - lse) on visible pairs, packed to bf16
//   C  dQ^T += K^T dS^T                    8 MFMAs, dQ^T in AccVGPRs
// and a sub-step runs stage A of the following half with stage B of the current one
// interleaved by hand (MFMA, a chunk of vector work, MFMA, ...), then stage C of the
// current half.  The mask enters through the accumulator of the S^T chain (a tile of
// 0 / -inf, edge halves only), so invisible pairs give P = 0 exactly and stage B is the same
// for every half.  The MFMAs are written as inline assembly with the register file in the
// constraint (see swaa_tile_d128.h); tests/test_asm_hazards.py checks the wait-state rules
// on the generated code.  K and V tiles lie in LDS in the layout of the other LDS-DMA
// backward kernels: 256-byte rows, 16-byte chunk c of row r at chunk c ^ g(r),
// g(r) = ((r & 3) << 2) | ((r >> 2) & 3), which serves row fragments (ds_read_b128) and
// transposed fragments (ds_read_b64_tr_b16) without bank conflicts.
//
// This kernel declares no static LDS: its dynamic LDS starts at address 0 and all LDS
// accesses below use plain byte addresses.
#include <atomic>
#include <type_traits>

#include "swaa_bwd.h"
#include "swaa_tile_d128.h"

namespace swaa {
namespace {

constexpr int kQWaves = 8;
constexpr int kQThreads = 64 * kQWaves;
constexpr int kQRows = 32;                             // query rows per wave
constexpr int kQStages = 3;                            // tiles per ring
constexpr int kQTileBytes = kBk * kD * 2;              // 16 KiB
constexpr int kQVRing = kQStages * kQTileBytes;        // V ring follows the K ring
constexpr int kQSmemBytes = 2 * kQStages * kQTileBytes;  // 96 KiB
constexpr int kQAhead = 3;                             // MFMAs between an LDS fragment read and its use

// Per-lane byte offsets of the fragments inside one tile (swizzle folded in); a uniform
// offset (buffer, half, 16-key step) is added through the instruction's offset field.
struct DqLane {
    uint32_t row[kKS];     // row fragment, k-step ks: row lane%32, logical chunk 2 ks + lane/32
    uint32_t col_lo[kDB];  // transposed fragment, head-dimension block db: rows 4 hf + j16/4 ...
    uint32_t col_hi[kDB];  // ... and the rows 8 further
};

__device__ __forceinline__ DqLane make_dq_lane(int lane) {
    DqLane la;
    const int l32 = lane & 31, hf = lane >> 5;
    const int gl = ((l32 & 3) << 2) | ((l32 >> 2) & 3);
    const uint32_t row_lane = (uint32_t)(l32 * kRowBytes + ((hf ^ gl) << 4));
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) la.row[ks] = row_lane ^ (uint32_t)(ks << 5);
    const int grp = lane >> 4, j16 = lane & 15;
    const int rr = 4 * hf + (j16 >> 2);
    const int cl = 2 * (grp & 1) + ((j16 & 3) >> 1);
    const uint32_t lo = (uint32_t)(rr * kRowBytes + ((((rr & 3) << 2) | (cl ^ hf)) << 4) + 8 * (j16 & 1));
    const uint32_t hi = (uint32_t)((rr + 8) * kRowBytes + ((((rr & 3) << 2) | (cl ^ (hf + 2))) << 4) + 8 * (j16 & 1));
#pragma unroll
    for (int db = 0; db < kDB; ++db) {
        la.col_lo[db] = lo ^ (uint32_t)(db << 6);
        la.col_hi[db] = hi ^ (uint32_t)(db << 6);
    }
    // opaque: the compiler must add the buffers' constant offsets through the instructions'
    // offset fields, not precompute an address register per buffer and fragment
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) asm volatile("" : "+v"(la.row[ks]));
#pragma unroll
    for (int db = 0; db < kDB; ++db) asm volatile("" : "+v"(la.col_lo[db]), "+v"(la.col_hi[db]));
    return la;
}

// Uniform byte offsets of the three half tiles one sub-step touches.
struct DqHalves {
    uint32_t ak, av;  // stage A: K half and V half whose scores and dP are computed
    uint32_t ck;      // stage C: K half whose dS has just been formed
};

// Stage A slot i (0..15): even slots K row fragments (S^T chain), odd slots V row fragments
// (dP^T chain), k-step i / 2.  Stage C slot c (0..7): transposed K fragment, 16-key step
// c / 4, head-dimension block c % 4.
__device__ __forceinline__ bf16x8 load_a_slot(const DqLane &la, const DqHalves &h, int i) {
    return lds_read16(la.row[i / 2] + ((i & 1) ? h.av : h.ak));
}
__device__ __forceinline__ bf16x8 load_c_slot(const DqLane &la, const DqHalves &h, int c) {
    const uint32_t off = h.ck + (uint32_t)((c / kDB) * 16 * kRowBytes);
    const s16x4 lo = lds_read8_tr(la.col_lo[c % kDB] + off);
    const s16x4 hi = lds_read8_tr(la.col_hi[c % kDB] + off);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

struct DqScratch {
    float pe[16];
};
// Stage B, cut into 16 chunks: chunk c exponentiates element c; the subtraction, the product
// and the packing of a pair trail one chunk behind, so that no instruction waits on a
// transcendental issued just before it.
__device__ __forceinline__ void stage_b_chunk(int c, const f32x16 &s, const f32x16 &dp, float c2, float lse2, float dl,
                                              DqScratch &w, bf16x8 (&dsf)[2]) {
    w.pe[c] = __builtin_amdgcn_exp2f(fmaf(s[c], c2, -lse2));
    if (c >= 1) {
        const int e = c - 1;
        w.pe[e] *= dp[e] - dl;
        if (e & 1) {  // the pair (e-1, e) is complete: pack it
            dsf[e / 8][(e - 1) % 8] = (__bf16)w.pe[e - 1];
            dsf[e / 8][e % 8] = (__bf16)w.pe[e];
            if (e % 8 == 7) pin_p(dsf[e / 8]);
        }
    }
}
__device__ __forceinline__ void stage_b_tail(const f32x16 &dp, float dl, DqScratch &w, bf16x8 (&dsf)[2]) {
    w.pe[15] *= dp[15] - dl;
    dsf[1][6] = (__bf16)w.pe[14];
    dsf[1][7] = (__bf16)w.pe[15];
    // keep the packing here and two wait states away from the MFMAs that read it
    asm volatile("s_nop 1" : "+v"(dsf[0]), "+v"(dsf[1]));
}

// One sub-step: stage A of the half at (h.ak, h.av) into (s_next, dp_next), interleaved with
// stage B of (s_cur, dp_cur), then stage C of that half (K at h.ck).  mask_next / k0h_next:
// whether the half of stage A needs the mask, and its first key.
__device__ __forceinline__ void dq_substep(const DqLane &la, const DqHalves &h, const bf16x8 (&qf)[kKS],
                                           const bf16x8 (&dof)[kKS], f32x16 &s_next, f32x16 &dp_next, const f32x16 &s_cur,
                                           const f32x16 &dp_cur, f32x16 (&dq)[kDB], float c2, float lse2, float dl,
                                           bool mask_next, int k0h_next, int qpos, int W, int S, int hf) {
    DqScratch w;
    bf16x8 dsf[2];
    bf16x8 frag[16 + 8 + kQAhead];
#pragma unroll
    for (int i = 0; i < kQAhead; ++i) frag[i] = load_a_slot(la, h, i);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int n = i + kQAhead;
        frag[n] = n < 16 ? load_a_slot(la, h, n) : load_c_slot(la, h, n - 16);
        if (i == 0)
            qk_chain_start(s_next, frag[0], qf[0], mask_next, k0h_next, qpos, W, S, hf);
        else if (i == 1)
            mfma_s_first(dp_next, frag[1], dof[0]);
        else if ((i & 1) == 0)
            mfma_s(s_next, frag[i], qf[i / 2]);
        else
            mfma_s(dp_next, frag[i], dof[i / 2]);
        __builtin_amdgcn_sched_barrier(0);
        stage_b_chunk(i, s_cur, dp_cur, c2, lse2, dl, w, dsf);
        __builtin_amdgcn_sched_barrier(0);
    }
    stage_b_tail(dp_cur, dl, w, dsf);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int n = 16 + c + kQAhead;
        if (n < 24) frag[n] = load_c_slot(la, h, n - 16);
        mfma_acc(dq[c % kDB], frag[16 + c], dsf[c / kDB]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ __launch_bounds__(kQThreads, 2) void swaa_bwd_dq_pipelined_kernel(const BwdParams p) {
    WorkItem wi;
    if (!decode_work(p.f, wi)) return;
    const int hpb = wi.hpb;
    const int rows_per_wg = kWgRows / hpb;
    const int N = p.N, S = p.f.S, P = p.f.P;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l32 = lane & 31, hf = lane >> 5;

    const int head = wi.kvh * p.f.G + wi.h0 + (wave % hpb);
    const int wg_p0 = wi.pt * rows_per_wg;             // first row (= position) of the workgroup
    const int wg_p1 = min(N, wg_p0 + rows_per_wg) - 1;  // last valid one
    const int p0 = wg_p0 + (wave / hpb) * kQRows;       // first row of this wave
    const int qpos = p0 + l32;                          // this lane's query column
    // this lane's window: a generated token (position >= P) sees its whole prefix
    const int W = (qpos >= P) ? N : p.f.W;

    // visited KV tiles: sink tiles 0 .. n_sink_tiles-1, then band tiles t_band_lo .. t_hi
    const int band_lo = (wg_p1 >= P) ? 0 : max(0, wg_p0 - p.f.W + 1);
    const int t_band_lo = band_lo / kBk;
    const int t_hi = wg_p1 / kBk;
    const int n_sink_tiles = min((min(S, band_lo) + kBk - 1) / kBk, t_band_lo);
    const int J = n_sink_tiles + (t_hi - t_band_lo + 1);
    auto tile_of = [&](int j) { return j < n_sink_tiles ? j : j - n_sink_tiles + t_band_lo; };

    const size_t kv_base = ((size_t)wi.b * p.Hkv + wi.kvh) * (size_t)N * kD;
    const __bf16 *kg = p.f.k + kv_base;
    const __bf16 *vg = p.f.v + kv_base;
    const size_t q_base = ((size_t)wi.b * p.Hq + head) * (size_t)N * kD;
    const size_t r_base = ((size_t)wi.b * p.Hq + head) * (size_t)N;

    // ---- HBM -> LDS tile copies: one wave instruction moves 64 x 16 bytes = 4 rows, a wave
    // moves 8 rows of K and of V per tile; the LDS side is linear in the lane id (address =
    // M0 + 16 * lane), the swizzle is applied on the global side.  Rows past the end of the
    // sequence repeat its last row (they are masked), so that the reads stay in bounds.
    const int lrow = lane >> 4, lchk = lane & 15;
    auto copy16 = [](const char *g, uint32_t lds) {
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds) : "memory");
    };
    auto issue_tile = [&](int j, int buf) {
        if (j >= J) return;
        const int first = tile_of(j) * kBk;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ii = 2 * wave + i;
            const int r = 4 * ii + lrow;
            const int g = (lrow << 2) | (ii & 3);  // g(r): r & 3 = lrow, (r >> 2) & 3 = ii & 3
            const size_t off = (size_t)min(first + r, N - 1) * kD * 2 + (size_t)((lchk ^ g) << 4);
            const uint32_t l = (uint32_t)(buf * kQTileBytes + ii * 1024);
            copy16(reinterpret_cast<const char *>(kg) + off, l);
            copy16(reinterpret_cast<const char *>(vg) + off, (uint32_t)kQVRing + l);
        }
    };
    issue_tile(0, 0);
    issue_tile(1, 1);
    issue_tile(2, 2);

    // ---- this wave's Q and dO rows (B operands of stage A), parked in AccVGPRs; its rows'
    // lse (log2 units) and delta ----
    bf16x8 qf[kKS], dof[kKS];
    float lse2, dl;
    {
        const int row = min(p0 + l32, N - 1);
        const __bf16 *qs = p.f.q + q_base + (size_t)row * kD + 8 * hf;
        const __bf16 *ds = p.dout + q_base + (size_t)row * kD + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8 *>(qs + 16 * ks);
            dof[ks] = *reinterpret_cast<const bf16x8 *>(ds + 16 * ks);
        }
        lse2 = p.f.lse[r_base + row] * 1.44269504088896340736f;
        dl = p.delta[r_base + row];
    }
    // the idle cycles keep the copies two wait states away from the first MFMA that reads them
    asm volatile("s_nop 1"
                 : "+a"(qf[0]), "+a"(qf[1]), "+a"(qf[2]), "+a"(qf[3]), "+a"(qf[4]), "+a"(qf[5]), "+a"(qf[6]), "+a"(qf[7]));
    asm volatile("s_nop 1"
                 : "+a"(dof[0]), "+a"(dof[1]), "+a"(dof[2]), "+a"(dof[3]), "+a"(dof[4]), "+a"(dof[5]), "+a"(dof[6]),
                   "+a"(dof[7]));

    f32x16 dq[kDB];
#pragma unroll
    for (int db = 0; db < kDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) dq[db][e] = 0.f;
    pin_acc(dq);

    const DqLane la = make_dq_lane(lane);
    const float c2 = p.f.scale_log2;

    // A wave needs no mask on a 32-key half when all its keys are visible to all its 32
    // rows (see the forward kernel); a wave whose rows lie past the end masks everything.
    const int wbound = window_bound(p0, kQRows, p.f.W, P);
    auto half_masked = [&](int k0h) { return !((k0h + 31 <= p0) && ((k0h > wbound) || (k0h + 31 < S))); };

    // the first three tiles (those that exist) have landed: this wave's parts, then everybody's
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- pipeline prologue: stage A of the very first half ----
    f32x16 s_a, dp_a, s_b, dp_b;  // scores and dP of half 0 / half 1 of a tile
    {
        const int k0 = tile_of(0) * kBk;
        const DqHalves h = {0u, (uint32_t)kQVRing, 0u};
        qk_chain_start(s_a, load_a_slot(la, h, 0), qf[0], true, k0, qpos, W, S, hf);
        mfma_s_first(dp_a, load_a_slot(la, h, 1), dof[0]);
#pragma unroll
        for (int ks = 1; ks < kKS - 1; ++ks) {
            mfma_s(s_a, load_a_slot(la, h, 2 * ks), qf[ks]);
            mfma_s(dp_a, load_a_slot(la, h, 2 * ks + 1), dof[ks]);
        }
        mfma_s(s_a, load_a_slot(la, h, 2 * kKS - 2), qf[kKS - 1]);
        mfma_s_settled(dp_a, load_a_slot(la, h, 2 * kKS - 1), dof[kKS - 1]);  // (completes after the S^T chain's last)
    }

    // One step = one visited tile; the ring position R = j % 3 is a template argument, so
    // every LDS offset is a constant that folds into the instructions' offset fields.
    auto step = [&](auto ring_pos, int j) {
        constexpr int R = decltype(ring_pos)::value;
        constexpr int Rn = (R + 1) % kQStages;
        const int k0 = tile_of(j) * kBk;
        const int k0n = (j + 1 < J) ? tile_of(j + 1) * kBk : k0 + kBk;  // past the end: never used
        // dS of (j, half 0) | scores, dP of (j, half 1) ; dQ from (j, half 0)
        const DqHalves h1 = {R * kQTileBytes + kHalfBytes, kQVRing + R * kQTileBytes + kHalfBytes, R * kQTileBytes};
        dq_substep(la, h1, qf, dof, s_b, dp_b, s_a, dp_a, dq, c2, lse2, dl, half_masked(k0 + 32), k0 + 32, qpos, W, S, hf);
        // dS of (j, half 1) | scores, dP of (j+1, half 0) ; dQ from (j, half 1).  In the last
        // step "tile j+1" is whatever the next buffer holds: those results are never used.
        const DqHalves h2 = {Rn * kQTileBytes, kQVRing + Rn * kQTileBytes, R * kQTileBytes + kHalfBytes};
        dq_substep(la, h2, qf, dof, s_a, dp_a, s_b, dp_b, dq, c2, lse2, dl, half_masked(k0n), k0n, qpos, W, S, hf);

        // tile j+2 must have landed; tile j's buffers are free afterwards
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        asm volatile("" ::: "memory");  // no LDS access may be moved across the barrier
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue_tile(j + kQStages, R);
    };
    static_assert(kQStages == 3, "the loop below walks three ring positions");
    for (int j = 0;;) {
        step(std::integral_constant<int, 0>{}, j);
        if (++j >= J) break;
        step(std::integral_constant<int, 1>{}, j);
        if (++j >= J) break;
        step(std::integral_constant<int, 2>{}, j);
        if (++j >= J) break;
    }

    // ---- dQ = scale * accumulators -> bf16; a lane holds 4 consecutive elements of its row
    // per accumulator quad.  The accumulators must be settled first: the last MFMAs above
    // have no MFMA behind them.
    asm volatile("s_nop 15\n\ts_nop 7" : "+a"(dq[0]), "+a"(dq[1]), "+a"(dq[2]), "+a"(dq[3]));
    const int row = p0 + l32;
    if (row >= N) return;
    __bf16 *orow = p.dq + q_base + (size_t)row * kD;
#pragma unroll
    for (int db = 0; db < kDB; ++db)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            bf16x4 o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(dq[db][4 * e4 + e] * p.f.scale);
            *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * e4 + 4 * hf) = o4;
        }
}

}  // namespace

hipError_t launch_bwd_dq_pipelined_d128(const BwdParams &p, hipStream_t stream) {
    // more than 64 KiB of LDS per workgroup has to be requested once per device
    static std::atomic<unsigned long long> configured{0};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(configured.load(std::memory_order_acquire) & bit)) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&swaa_bwd_dq_pipelined_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kQSmemBytes);
        if (err != hipSuccess) return err;
        configured.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(swaa_bwd_dq_pipelined_kernel, dim3((unsigned)(p.f.chunk * kXcds)), dim3(kQThreads), kQSmemBytes, stream,
                       p);
    return hipGetLastError();
}

}  // namespace swaa
