// Software-pipelined SWA + sink attention forward, head dimension 128, gfx950.
//
// Same mask (paper Sec. 3.2.1 / Fig. 1b; full attention of Sec. 3.1.2 when the
// window covers the context) and the same work decomposition as the plain
// kernel: one workgroup = 256 query rows (4, 2 or 1 query heads x 64, 128 or
// 256 positions) on one KV head.  What differs:
//
//   * Eight waves of 32 query rows, two per SIMD.  A single wave cannot keep
//     the matrix pipe busy (back-to-back MFMAs of one wave issue about a third
//     slower than the pipe could take them, and every vector instruction beyond
//     four per MFMA adds to that); with two waves per SIMD one wave's
//     exponentials run while the other wave's MFMAs execute.  Each wave fits in
//     256 registers: O^T (64) and Q (32) in AccVGPRs, S^T, P^T and the K/V
//     fragments in VGPRs.
//   * K and V tiles (64 keys) travel HBM -> LDS with global_load_lds_dwordx4
//     (no register staging) into two rings of kStages tiles each, XOR-swizzled
//     in 16-byte chunks so that the MFMA operand reads are bank-conflict free.
//     One barrier per tile.  Q rows arrive the same way and O rows leave through
//     the same per-wave staging area, so that every HBM access of the kernel is a
//     full 256-byte row per 16 lanes.
//   * A wave works on half tiles of 32 keys in a three-stage pipeline: while
//     the softmax of half n runs on the VALU, the matrix pipe computes
//     S^T = K Q^T of half n+1 and O^T += V^T P^T of half n-1.  The interleaving
//     is fixed by hand with scheduling fences.  Every visited half goes through
//     the same pipeline; edge tiles use the variant that masks scores first.
//   * The softmax reference: softmax is invariant to the value subtracted
//     before the exponential, so the reference only has to keep exp2() inside
//     the fp32/bf16 range.  It is set from the first half a wave processes and
//     moves later only when a row sum shows that scores have outgrown it (or,
//     on edge tiles, when the maximum grows by more than 2^8); O and the row
//     sum are rescaled only then.  Results are mathematically unchanged; the
//     search for the row maximum and the rescale of the accumulator disappear
//     from the steady state.
//
// This kernel declares no static LDS: its dynamic LDS starts at address 0 and
// all LDS accesses below use plain byte addresses.
#include <atomic>
#include <type_traits>

#include "swaa_tile_d128.h"

namespace swaa {
namespace {

constexpr int kPWaves = 8;    // waves per workgroup
constexpr int kPThreads = 64 * kPWaves;
constexpr int kPRows = 32;  // query positions per wave
constexpr int kStages = 3;                            // tiles per ring: copies run one step ahead
constexpr int kTileBytes = kBk * kD * 2;              // 16 KiB
constexpr int kVRing = kStages * kTileBytes;          // V ring follows the K ring
constexpr int kStage = 2 * kStages * kTileBytes;      // per-wave staging areas follow the rings
constexpr int kStageBytes = kPRows * kD * 2;          // 8 KiB: a wave's 32 Q rows on the way in, O rows on the way out
constexpr int kSmemBytes = kStage + kPWaves * kStageBytes;  // 96 + 64 = 160 KiB, all of a CU's LDS
constexpr float kSumLimit = 1.0995116e12f;  // 2^40: a row sum that sends the workgroup back to the max-based path
constexpr float kSumFloor = 7.8886091e-31f;  // 2^-100: so does one this small (every score far below the reference)
constexpr int kPrefetch = 3;  // MFMAs between an LDS fragment read and its use

// ---- the pipelined sub-step, scheduled by hand -------------------------------------
// A sub-step issues 16 MFMAs, alternating S^T(n+1) += K Q^T (8, one chain) and
// O^T += V^T P^T(n-1) (8, four chains), and in their shadow the vector work of
// the softmax of half n, cut into 16 chunks.  Scheduling fences pin the order
// "MFMA, chunk, MFMA, chunk, ...".  LDS fragment reads are issued kPrefetch
// MFMAs ahead of their use, across the boundary between the two sub-steps of a
// step as well.
//
// The mask enters through the accumulator: on a half that is not fully visible
// to the wave's 32 rows the K Q^T chain starts from a tile of 0 / -inf instead
// of from zero, so invisible scores come out as -inf and their exponential is
// an exact 0.  A half that lies wholly outside a wave's rows (before its band,
// above its diagonal) therefore contributes nothing and needs no special case,
// and the softmax chunks are the same for every half.
//
// The softmax does not look for the row maximum: it keeps the reference it has
// (taken from the first half the wave sees).  exp2(s*c2 - mc) cannot overflow
// fp32 or bf16 unless a score exceeds the reference by more than 2^7 in the exp2
// domain, and the terms are never negative, so the final row sum bounds every
// term and every partial sum: if it reaches kSumLimit (or is not a number) the
// workgroup recomputes its rows with the max-based routine after the loop.  It
// does the same if a row sum comes out below kSumFloor: a row whose first half
// was invisible to it has reference 0, and if all its scores lie a hundred
// binary orders below that, its terms leave the range fp32 resolves.
// Everything else is "subtract, exponentiate, add, pack".
struct SoftmaxScratch {
    float pe[16];
};

// first score element handled by chunk c: 16 scores over chunks 0..13
__device__ __forceinline__ constexpr int chunk_first_elem(int c) { return c >= 14 ? 16 : (c * 16) / 14; }

__device__ __forceinline__ void softmax_chunk(int c, const f32x16 &s, float c2, RowState &st, SoftmaxScratch &w,
                                              bf16x8 (&pf)[2]) {
#pragma unroll
    for (int e = chunk_first_elem(c); e < chunk_first_elem(c + 1); ++e)
        w.pe[e] = __builtin_amdgcn_exp2f(fmaf(s[e], c2, -st.mc));
    // sums and packing trail one chunk behind, so that no instruction waits on
    // a transcendental issued just before it
    if (c >= 1 && c <= 14) {
#pragma unroll
        for (int e = chunk_first_elem(c - 1); e < chunk_first_elem(c); ++e) {
            st.l += w.pe[e];
            if (e & 1) {  // the pair (e-1, e) is complete: pack it
                pf[e / 8][(e - 1) % 8] = (__bf16)w.pe[e - 1];
                pf[e / 8][e % 8] = (__bf16)w.pe[e];
                if (e % 8 == 7) pin_p(pf[e / 8]);
            }
        }
    }
}

// ---- the divisor of O: column sums of the rounded P^T, on the matrix pipe -------------
// The P V contraction weights V with the bf16 entries of P^T, so O has to be
// divided by the sum of those (add_rounded_pair has the reason).  In this loop
// the vector ALU has no slot to spare for that sum, the matrix pipe has: a P^T
// fragment (B operand of the 32x32x16 MFMA: lane l holds eight keys of query
// column l % 32) is read as the B operand of a 16x16x32 MFMA, which takes lane l
// as column l % 16, k-group l / 16.  Against an A operand whose row 0 is ones on
// k-groups 0 and 2 and whose row 1 is ones on k-groups 1 and 3 (zero elsewhere),
// D[0][j] is the sum over the fragment's 16 keys of query column j and D[1][j]
// that of column 16 + j; lanes 0..15 hold them as elements 0 and 1.
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 rowsum_selector(int lane) {
    // A operand: lane l holds row l % 16, k-group l / 16
    const int m = lane & 15, kg = lane >> 4;
    const bool on = (m == 0 && (kg & 1) == 0) || (m == 1 && (kg & 1) == 1);
    bf16x8 a;
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = on ? (__bf16)1.f : (__bf16)0.f;
    return a;
}
__device__ __forceinline__ void mfma_rowsum(f32x4 &acc, const bf16x8 sel_acc, const bf16x8 pfrag) {
    asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "a"(sel_acc), "v"(pfrag));
}
// The sums of this lane's query column, from the two accumulators of the loop.
// (They must be settled: other MFMAs lie between the loop and this.)
__device__ __forceinline__ float rowsum_of_column(const f32x4 (&lsum)[2], int l32) {
    const float lo = __shfl(lsum[0][0] + lsum[1][0], l32 & 15);
    const float hi = __shfl(lsum[0][1] + lsum[1][1], l32 & 15);
    return l32 < 16 ? lo : hi;
}

// Uniform byte offsets of the LDS halves one sub-step touches.
struct HalfOffsets {
    uint32_t k, v;    // K half to multiply, V half to accumulate
    uint32_t nk, nv;  // the same for the following sub-step (fragment prefetch)
};

// Fragment slot i of a sub-step: even slots are K fragments (k-step i/2), odd
// slots V^T fragments ((i-1)/2 = 4*st + db); slots 16.. belong to the next sub-step.
__device__ __forceinline__ bf16x8 load_slot(const LaneAddr &la, const HalfOffsets &ho, int i) {
    const bool next = i >= 16;
    const int ii = next ? i - 16 : i;
    if ((ii & 1) == 0) return load_k_frag(la, next ? ho.nk : ho.k, ii / 2);
    return load_v_frag(la, next ? ho.nv : ho.v, (ii / 2) / kDB, (ii / 2) % kDB);
}

// fpre: the first kPrefetch fragments, already requested by the caller; on
// return it holds those of the following sub-step.  k0h_next / mask_next: first
// key of the half whose scores are computed here, and whether it needs the mask.
__device__ __forceinline__ void pipelined_substep(const LaneAddr &la, const HalfOffsets &ho, bf16x8 (&fpre)[kPrefetch],
                                                  const bf16x8 (&qf)[kKS], f32x16 &s_next, const f32x16 &s_cur,
                                                  bf16x8 (&p_cur)[2], const bf16x8 (&p_prev)[2], f32x16 (&o)[kDB],
                                                  RowState &st, f32x4 (&lsum)[2], const bf16x8 &sel, float c2,
                                                  bool mask_next, int k0h_next, int qpos, int W, int S, int hf) {
    SoftmaxScratch w;
    bf16x8 frag[16 + kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) frag[i] = fpre[i];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        frag[i + kPrefetch] = load_slot(la, ho, i + kPrefetch);
        if (i == 0)
            qk_chain_start(s_next, frag[i], qf[0], mask_next, k0h_next, qpos, W, S, hf);
        else if ((i & 1) == 0)
            mfma_s(s_next, frag[i], qf[i / 2]);
        else
            mfma_acc(o[(i / 2) % kDB], frag[i], p_prev[(i / 2) / kDB]);
        __builtin_amdgcn_sched_barrier(0);
        softmax_chunk(i, s_cur, c2, st, w, p_cur);
        if (i == 15) {  // P^T of this half is complete (and two MFMAs old)
            mfma_rowsum(lsum[0], sel, p_cur[0]);
            mfma_rowsum(lsum[1], sel, p_cur[1]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) fpre[i] = frag[16 + i];
}

__global__ __launch_bounds__(kPThreads, 2) void swaa_fwd_pipelined_kernel(const FwdParams p) {
    WorkItem wi;
    if (!decode_work(p, wi)) return;
    SeqGeom sg;
    if (!seq_geom(p, wi.b, sg)) return;
    const int hpb = wi.hpb;
    const int rows_per_wg = kWgRows / hpb;
    const int wg_r0 = wi.pt * rows_per_wg;  // first query row of the workgroup
    if (wg_r0 >= sg.nq) return;             // a shorter sequence of a packed batch
    const int Nq = sg.nq, Nk = sg.nk, S = p.S;
    const int pos_off = Nk - Nq;  // query row r sits at position pos_off + r

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform, and known to the compiler as such
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int hf = lane >> 5;

    const int head = wi.kvh * p.G + wi.h0 + (wave % hpb);
    const int r0 = wg_r0 + (wave / hpb) * kPRows;  // first query row of this wave
    const int wg_p0 = pos_off + wg_r0;             // positions of the workgroup's first ...
    const int wg_p1 = pos_off + min(Nq, wg_r0 + rows_per_wg) - 1;  // ... and last valid row
    const int p0 = pos_off + r0;                   // first position of this wave
    const int qpos = p0 + l32;                     // this lane's query column
    // this lane's window: a generated token (position >= P) sees its whole prefix
    const int W = (qpos >= p.P) ? Nk : p.W;

    // visited KV tiles: sink tiles 0 .. n_sink_tiles-1, then band tiles t_band_lo .. t_hi;
    // a workgroup that holds a generated token visits every tile up to its diagonal
    const int band_lo = (wg_p1 >= p.P) ? 0 : max(0, wg_p0 - p.W + 1);
    const int t_band_lo = band_lo / kBk;
    const int t_hi = wg_p1 / kBk;
    const int n_sink_tiles = min((min(S, band_lo) + kBk - 1) / kBk, t_band_lo);
    const int J = n_sink_tiles + (t_hi - t_band_lo + 1);
    auto tile_of = [&](int j) { return j < n_sink_tiles ? j : j - n_sink_tiles + t_band_lo; };

    const uint32_t k_rsb = (uint32_t)(p.k_sn * 2), v_rsb = (uint32_t)(p.v_sn * 2);  // row strides in bytes
    const __bf16 *kg = p.k + sg.k_batch * p.k_sb + (long long)wi.kvh * p.k_sh + sg.k_row0 * p.k_sn;
    const __bf16 *vg = p.v + sg.k_batch * p.v_sb + (long long)wi.kvh * p.v_sh + sg.k_row0 * p.v_sn;
    const __bf16 *qg = p.q + sg.q_batch * p.q_sb + (long long)head * p.q_sh + sg.q_row0 * p.q_sn;
    __bf16 *og = p.out + sg.q_batch * p.o_sb + (long long)head * p.o_sh + sg.q_row0 * p.o_sn;

    // ---- HBM -> LDS tile copies -------------------------------------------------
    // One wave instruction moves 64 x 16 bytes = 4 rows of the tile, a wave moves
    // 8 rows of K and of V per tile; the LDS side is linear in the lane id, the
    // swizzle is applied on the global side: LDS chunk (row, c') receives global
    // chunk c' ^ f(row) of that row, with f(row) = ((row & 7) << 1) | ((row >> 3) & 1)
    // for K (16 consecutive rows read the same logical chunk) and (row & 3) << 2
    // for V (4 consecutive rows read the same 64 bytes).
    const int lrow = lane >> 4;  // row within the 4-row group
    const int lchk = lane & 15;  // LDS chunk within the row
    // byte offset of this lane's 16 bytes from the tile's first row; row = 8*wave + 4*i + lrow
    const uint32_t chunk_k = (uint32_t)(lchk ^ (lrow << 1) ^ (wave & 1));
    const uint32_t voff_k = (uint32_t)(8 * wave + lrow) * k_rsb + (chunk_k << 4);
    const uint32_t voff_k1 = (uint32_t)(8 * wave + lrow + 4) * k_rsb + ((chunk_k ^ 8u) << 4);  // row & 7 = 4 + lrow
    const uint32_t voff_v = (uint32_t)(8 * wave + lrow) * v_rsb + (uint32_t)((lchk ^ (lrow << 2)) << 4);
    // LDS address = M0 + 16 * lane; global address = base + off.  Issued as assembly on
    // purpose: the compiler would otherwise make every later LDS read wait for the copy.
    auto copy16 = [](uint32_t off, const char *base, uint32_t lds) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds)
                     : "memory");
    };
    // The wave's two copies of one tile into ring buffer `buf`; base: the tile's first row in
    // HBM; ragged: the tile runs past the sequence's last row (only the last visited tile
    // can), and rows past the end repeat the last row -- they are masked later -- so that the
    // reads stay in bounds.
    auto copy_tile = [&](const char *base, int buf, int ring, bool is_k, bool ragged) {
        const uint32_t l = (uint32_t)(ring + buf * kTileBytes + 2 * wave * 1024);
        if (__builtin_expect(ragged, 0)) {
            const uint32_t rsb = is_k ? k_rsb : v_rsb;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                uint32_t off = is_k ? (i ? voff_k1 : voff_k) : voff_v + (uint32_t)(4 * i) * v_rsb;
                const int row = 8 * wave + 4 * i + lrow;
                off -= (uint32_t)max(t_hi * kBk + row - (Nk - 1), 0) * rsb;
                copy16(off, base, l + (uint32_t)(i * 1024));
            }
        } else if (is_k) {
            copy16(voff_k, base, l);
            copy16(voff_k1, base, l + 1024u);
        } else {
            copy16(voff_v, base, l);
            copy16(voff_v + 4u * v_rsb, base, l + 1024u);
        }
    };
    const int j_ragged = ((t_hi + 1) * kBk > Nk) ? J - 1 : -1;
    // any visited tile (the recomputation path)
    auto issue_tile = [&](int j, int buf, const __bf16 *src, int ring, bool is_k) {
        if (j >= J) return;
        const char *base = reinterpret_cast<const char *>(src) + (size_t)(tile_of(j) * kBk) * (is_k ? k_rsb : v_rsb);
        copy_tile(base, buf, ring, is_k, j == j_ragged);
    };
    auto issue_k = [&](int j, int buf) { issue_tile(j, buf, kg, 0, true); };
    auto issue_v = [&](int j, int buf) { issue_tile(j, buf, vg, kVRing, false); };
    // The pipeline asks for the visited tiles in order, so their addresses are kept as two
    // running pointers: a handful of scalar instructions per tile instead of a 64-bit
    // multiplication (every wave executes them, at the start of every step).
    struct TileStream {
        const char *next;   // first row of the next tile to copy
        size_t step, jump;  // bytes to the following tile: the usual one, and from the last sink tile to the band
        int plain;          // tiles to copy before the next one that needs a closer look
    };
    // A tile needs a closer look if it is the last sink tile before a jump, runs past the
    // sequence's end, or does not exist; all others take "copy, advance by one tile".
    auto special = [&](int j) { return j + 1 == n_sink_tiles || j == j_ragged || j >= J; };
    auto plain_from = [&](int j) {  // number of consecutive tiles from j on that are not special
        int e = J;
        if (j_ragged >= j) e = min(e, j_ragged);
        if (n_sink_tiles - 1 >= j) e = min(e, n_sink_tiles - 1);
        return max(e - j, 0);
    };
    auto make_stream = [&](const __bf16 *src, uint32_t rsb) {
        TileStream ts;
        ts.next = reinterpret_cast<const char *>(src) + (size_t)(tile_of(0) * kBk) * rsb;
        ts.step = (size_t)kBk * rsb;
        ts.jump = (size_t)(t_band_lo - n_sink_tiles + 1) * kBk * rsb;
        ts.plain = plain_from(0);
        return ts;
    };
    TileStream k_stream = make_stream(kg, k_rsb), v_stream = make_stream(vg, v_rsb);
    auto stream_tile = [&](TileStream &ts, int j, int buf, int ring, bool is_k) {
        if (__builtin_expect(--ts.plain >= 0, 1)) {
            const char *base = ts.next;
            ts.next += ts.step;
            copy_tile(base, buf, ring, is_k, false);
            return;
        }
        if (j >= J) return;  // (plain stays negative: every later call ends here)
        const char *base = ts.next;
        ts.next += (j + 1 == n_sink_tiles) ? ts.jump : ts.step;
        copy_tile(base, buf, ring, is_k, j == j_ragged);
        ts.plain = plain_from(j + 1);
    };
    auto stream_k = [&](int j, int buf) { stream_tile(k_stream, j, buf, 0, true); };
    auto stream_v = [&](int j, int buf) { stream_tile(v_stream, j, buf, kVRing, false); };

    // Step 0 multiplies an all-zero P^T with "the tile before the first": give that
    // V buffer (the last one of the ring, not yet a copy target) defined contents.
    {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < kTileBytes / 16; i += kPThreads)
            *(u32x4 __attribute__((address_space(3))) *)(uintptr_t)(kVRing + (kStages - 1) * kTileBytes + i * 16) = zero;
    }

    // ---- this wave's 32 Q rows: HBM -> its staging area, laid out like a K half tile ----
    const uint32_t stage = (uint32_t)(kStage + wave * kStageBytes);
    {
        const char *qb = reinterpret_cast<const char *>(qg);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 4 * i + lrow;
            const int f = ((4 * (i & 1) + lrow) << 1) | ((i >> 1) & 1);
            const char *g = qb + (size_t)min(r0 + row, Nq - 1) * (size_t)(p.q_sn * 2) + ((lchk ^ f) << 4);
            const uint32_t l = stage + (uint32_t)(i * 1024);
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(l) : "memory");
        }
    }
    // Tiles in the order they are needed.  A CU takes in about 64 bytes per cycle,
    // so the pipeline prologue below starts as soon as Q and K(0) are there (ten
    // copies per wave) and the other four tiles (eight copies) stream in behind it.
    stream_k(0, 0);
    stream_v(0, 0);
    stream_k(1, 1);
    stream_k(2, 2);
    stream_v(1, 1);

    f32x16 oacc[kDB];
#pragma unroll
    for (int db = 0; db < kDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
    pin_acc(oacc);

    // per-lane LDS read offsets inside a half tile (swizzle folded in)
    // (made opaque: otherwise the compiler precomputes "lane offset + buffer offset" for many
    // (buffer, fragment) pairs, parks those addresses in AccVGPRs and copies one back before
    // every read; this way the buffers' constant offsets go into the instructions' offset fields)
    LaneAddr la = make_lane_addr(lane, kVRing);
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) asm volatile("" : "+v"(la.k[ks]));
#pragma unroll
    for (int db = 0; db < kDB; ++db) asm volatile("" : "+v"(la.v[db]));

    const float c2 = p.scale_log2;

    f32x16 s_a, s_b;        // scores of half 0 / half 1 of a tile
    bf16x8 p_a[2], p_b[2];  // their P^T fragments
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        p_b[0][e] = (__bf16)0.f;
        p_b[1][e] = (__bf16)0.f;
    }
    pin_p(p_b[0]);
    pin_p(p_b[1]);
    f32x4 lsum[2];  // column sums of the rounded P^T (mfma_rowsum), one accumulator per fragment
#pragma unroll
    for (int e = 0; e < 4; ++e) lsum[0][e] = lsum[1][e] = 0.f;
    bf16x8 sel = rowsum_selector(lane);
    asm volatile("s_nop 1" : "+a"(lsum[0]), "+a"(lsum[1]), "+a"(sel));

    // A wave needs no mask on a 32-key half when all its keys are visible to all
    // its 32 rows: at or below the first row's diagonal, and inside the window of
    // its last prompt row (if it has one) or all sinks.
    const int wbound = window_bound(p0, kPRows, p.W, p.P);
    auto half_masked = [&](int k0h) { return !((k0h + 31 <= p0) && ((k0h > wbound) || (k0h + 31 < S))); };

    // (Worked out here, while the first copies travel.)
    // Steps [ja, jb) of this wave need no mask: band tiles t with both score halves of the
    // step (tile t half 1, tile t+1 half 0) inside every row's window and at or below the
    // first row's diagonal.  The two loops only run if the closed form is off.
    int ja, jb;
    {
        auto unmasked_step = [&](int j) {
            if (j < n_sink_tiles || j + 1 >= J) return false;
            const int k0 = tile_of(j) * kBk;
            return !half_masked(k0 + 32) && !half_masked(k0 + kBk);
        };
        const int t_min = max(((wbound - 32) >> 6) + 1, t_band_lo);  // 64 t + 32 > wbound
        const int t_max = min((p0 - 95) >> 6, t_hi - 1);             // 64 t + 64 + 31 <= p0
        ja = n_sink_tiles + (t_min - t_band_lo);
        jb = max(ja, n_sink_tiles + (t_max - t_band_lo) + 1);
        while (ja < jb && !unmasked_step(ja)) ++ja;
        while (jb > ja && !unmasked_step(jb - 1)) --jb;
    }
    const unsigned n_interior = (unsigned)(jb - ja);

    // this wave's Q and K(0) copies must have landed; V(0), K(1), K(2), V(1) -- those
    // of them that exist -- may still fly (two copies per tile)
    if (J >= 3)
        __builtin_amdgcn_s_waitcnt(0x0078);  // vmcnt(8) lgkmcnt(0)
    else if (J == 2)
        __builtin_amdgcn_s_waitcnt(0x0076);  // vmcnt(6) lgkmcnt(0)
    else
        __builtin_amdgcn_s_waitcnt(0x0072);  // vmcnt(2) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- Q fragments (B operand of S^T = K Q^T), parked in AccVGPRs -------------------
    bf16x8 qf[kKS];
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) qf[ks] = load_k_frag(la, stage, ks);
    // the idle cycles keep the copies two wait states away from the first MFMA that reads them
    asm volatile("s_nop 1"
                 : "+a"(qf[0]), "+a"(qf[1]), "+a"(qf[2]), "+a"(qf[3]), "+a"(qf[4]), "+a"(qf[5]), "+a"(qf[6]), "+a"(qf[7]));

    // ---- pipeline prologue: scores of the very first half, and the softmax reference ----
    // The reference is the largest visible score of that half (0 for a row that
    // sees none of its keys); from here on it only moves if a row sum overflows.
    RowState rs;
    rs.l = 0.f;
    rs.lb = 0.f;
    {
        const int k0 = tile_of(0) * kBk;
        qk_chain_start(s_a, load_k_frag(la, 0, 0), qf[0], true, k0, qpos, W, S, hf);
#pragma unroll
        for (int ks = 1; ks < kKS - 1; ++ks) mfma_s(s_a, load_k_frag(la, 0, ks), qf[ks]);
        mfma_s_settled(s_a, load_k_frag(la, 0, kKS - 1), qf[kKS - 1]);
        float mx = s_a[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s_a[e]);
        mx = half_swap_max(mx);
        rs.mc = (mx == -INFINITY) ? 0.f : mx * c2;
    }

    // step 0 reads V(0) and K(1): they must be there for every wave (K(2), V(1) may still fly)
    if (J >= 3)
        __builtin_amdgcn_s_waitcnt(0x0074);  // vmcnt(4) lgkmcnt(0)
    else if (J == 2)
        __builtin_amdgcn_s_waitcnt(0x0072);  // vmcnt(2) lgkmcnt(0)
    else
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // One step = one visited tile.  The ring position R = j % 3 is a template
    // argument, so every LDS offset below is a constant that folds into the
    // instructions' offset fields (no address arithmetic in the loop); the loop
    // walks the three instantiations in turn.
    bf16x8 fpre[kPrefetch];  // the first fragments of the coming sub-step, requested one sub-step ahead
    {
        const HalfOffsets h0 = {kHalfBytes, (kStages - 1) * kTileBytes + kHalfBytes, 0, 0};  // step 0, first sub-step
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) fpre[i] = load_slot(la, h0, i);
    }
    // checked: the step looks at its two score halves and masks them where needed.  In the
    // interior of a wave's band no half needs a mask, and the step skips that scalar
    // bookkeeping.
    auto step = [&](auto ring_pos, bool checked, int j) {
        constexpr int R = decltype(ring_pos)::value;
        constexpr int Rn = (R + 1) % kStages, Rp = (R + kStages - 1) % kStages;
        constexpr uint32_t kb_cur1 = R * kTileBytes + kHalfBytes;    // K(j), half 1
        constexpr uint32_t kb_next0 = Rn * kTileBytes;               // K(j+1), half 0
        constexpr uint32_t vb_prev1 = Rp * kTileBytes + kHalfBytes;  // V(j-1), half 1
        constexpr uint32_t vb_cur0 = R * kTileBytes;                 // V(j), half 0
        int k0 = 0, k0n = 0;
        bool mask1 = false, mask2 = false;
        if (__builtin_expect(checked, 0)) {
            k0 = tile_of(j) * kBk;
            k0n = (j + 1 < J) ? tile_of(j + 1) * kBk : k0 + kBk;  // past the end: scores never used
            mask1 = half_masked(k0 + 32);
            mask2 = half_masked(k0n);
        }

        // softmax of (j, half 0) | scores of (j, half 1) | P V of (j-1, half 1)
        const HalfOffsets h1 = {kb_cur1, vb_prev1, kb_next0, vb_cur0};
        pipelined_substep(la, h1, fpre, qf, s_b, s_a, p_a, p_b, oacc, rs, lsum, sel, c2, mask1, k0 + 32, qpos, W, S, hf);
        // softmax of (j, half 1) | scores of (j+1, half 0) | P V of (j, half 0); its last
        // fragment requests are the first ones of step j+1 (K(j+1) half 1, V(j) half 1: both
        // resident), so that they are under way while the waves meet at the barrier
        const HalfOffsets h2 = {kb_next0, vb_cur0, Rn * kTileBytes + kHalfBytes, R * kTileBytes + kHalfBytes};
        pipelined_substep(la, h2, fpre, qf, s_a, s_b, p_b, p_a, oacc, rs, lsum, sel, c2, mask2, k0n, qpos, W, S, hf);

        // K(j+2), V(j+1) must have landed; K(j) and V(j-1) are free afterwards
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        asm volatile("" ::: "memory");  // no LDS access may be moved across the barrier
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        stream_k(j + kStages, R);
        stream_v(j + kStages - 1, Rp);
    };
    static_assert(kStages == 3, "the loop below walks three ring positions");
    auto ring_step = [&](auto ring_pos, int j) { step(ring_pos, (unsigned)(j - ja) >= n_interior, j); };
    for (int j = 0;;) {
        ring_step(std::integral_constant<int, 0>{}, j);
        if (++j >= J) break;
        ring_step(std::integral_constant<int, 1>{}, j);
        if (++j >= J) break;
        ring_step(std::integral_constant<int, 2>{}, j);
        if (++j >= J) break;
    }
    // pipeline drain: P V of the last half (V(J-1) sits in buffer (J-1) % kStages)
    pv_half<true>(la, (uint32_t)(((J - 1) % kStages) * kTileBytes + kHalfBytes), p_b, oacc);

    // ---- scores outgrew the reference somewhere in this workgroup (inputs with
    // score jumps of tens of nats): recompute its rows with the max-based routine,
    // one tile at a time, no pipelining ------------------------------------------
    // (workgroup-wide OR through eight flag words at the start of the K ring,
    // which nobody reads any more after the loop's last barrier)
    // (the drain above waited for its own result, hence for the column sums issued before it)
    float l_row = half_swap_sum(rs.l);
    float lb_row = rowsum_of_column(lsum, l32);
    bool redo;
    {
        // a sum inside (kSumFloor, kSumLimit), tested on the bit pattern: positive floats order like
        // unsigned integers, and zero, infinity and every NaN pattern fall outside the interval
        // (the build does not honour NaNs in float comparisons).  Rows past the end of the
        // sequence (the ragged last tile; they may see no key at all) have no say.
        const bool in_range = (__float_as_uint(l_row) - (__float_as_uint(kSumFloor) + 1u)) <
                              (__float_as_uint(kSumLimit) - (__float_as_uint(kSumFloor) + 1u));
        const int mine = __any(!in_range && r0 + l32 < Nq) ? 1 : 0;
        if (lane == 0) *(int __attribute__((address_space(3))) *)(uintptr_t)(wave * 4) = mine;
        __syncthreads();
        int any = 0;
#pragma unroll
        for (int w = 0; w < kPWaves; ++w) any |= *(const int __attribute__((address_space(3))) *)(uintptr_t)(w * 4);
        redo = any != 0;
    }
    if (redo) {
#pragma unroll
        for (int db = 0; db < kDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
        pin_acc(oacc);
        rs.mc = -INFINITY;
        rs.l = 0.f;
        rs.lb = 0.f;
        for (int j = 0; j < J; ++j) {
            __syncthreads();  // everyone is done reading the previous tile
            issue_k(j, 0);
            issue_v(j, 0);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
#pragma unroll 1
            for (int hh = 0; hh < 2; ++hh) {
                float alpha;
                qk_half(la, (uint32_t)(hh * kHalfBytes), qf, s_a);
                softmax_half<true>(s_a, tile_of(j) * kBk + 32 * hh, qpos, W, S, hf, c2, rs, p_a, alpha);
                rescale(oacc, alpha);
                pv_half<true>(la, (uint32_t)(hh * kHalfBytes), p_a, oacc);
            }
        }
        row_sums(rs, l_row, lb_row);
    }

    // ---- epilogue: O / (sum of the rounded P) -> bf16 through the wave's staging area, so
    // that the stores to HBM are whole rows; lse = (mc + log2 l) * ln 2 -------------------
    // (the accumulators are settled: the last P V contraction above waited for its result)
    {
        const float inv_l = 1.f / lb_row;  // rows past the end: never stored
        const int fr = ((l32 & 7) << 1) | ((l32 >> 3) & 1);
        const uint32_t o_lane = stage + (uint32_t)(l32 * 256 + (fr << 4) + 8 * hf);
#pragma unroll
        for (int db = 0; db < kDB; ++db) {
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][4 * e4 + e] * inv_l);
                // d = 32 db + 8 e4 + 4 hf + (0..3): 16-byte chunk 4 db + e4 of row l32, swizzled like K
                *(bf16x4 __attribute__((address_space(3))) *)(uintptr_t)(o_lane ^ (uint32_t)((4 * db + e4) << 4)) = o4;
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 4 * i + lrow;
            const int f = ((4 * (i & 1) + lrow) << 1) | ((i >> 1) & 1);
            const u32x4 val = *(const u32x4 __attribute__((address_space(3))) *)(uintptr_t)(stage + i * 1024 + lane * 16);
            if (r0 + row < Nq) *reinterpret_cast<u32x4 *>(og + (size_t)(r0 + row) * p.o_sn + ((lchk ^ f) << 3)) = val;
        }
        if (hf == 0 && r0 + l32 < Nq)
            p.lse[sg.q_batch * p.lse_sb + (long long)head * p.lse_sh + sg.q_row0 + r0 + l32] =
                (rs.mc + __builtin_amdgcn_logf(l_row)) * 0.69314718055994530942f;
    }
}

}  // namespace

hipError_t launch_fwd_pipelined_d128(const FwdParams &p, hipStream_t stream) {
    // more than 64 KiB of LDS per workgroup has to be requested once per device
    static std::atomic<unsigned long long> configured{0};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(configured.load(std::memory_order_acquire) & bit)) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&swaa_fwd_pipelined_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes);
        if (err != hipSuccess) return err;
        configured.fetch_or(bit, std::memory_order_release);
    }
    const unsigned grid = (unsigned)(p.chunk * kXcds);
    hipLaunchKernelGGL(swaa_fwd_pipelined_kernel, dim3(grid), dim3(kPThreads), kSmemBytes, stream, p);
    return hipGetLastError();
}

}  // namespace swaa
