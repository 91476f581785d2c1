// Software-pipelined SWA + sink attention forward, head dimension 128, gfx950.
//
// Same mask (paper Sec. 3.2.1 / Fig. 1b; full attention of Sec. 3.1.2 when the
// window covers the context) as the plain kernel.  Design:
//
//   * A workgroup is FOUR waves of 32 query rows: 128 rows (4, 2 or 1 query heads
//     x 32, 64 or 128 positions) on one KV head, 64 KiB of LDS, 256 registers per
//     wave -- so TWO workgroups share a compute unit, one wave of each per SIMD.
//     A single wave cannot keep the matrix pipe busy (its exponentials, its tile
//     copies, its waits at the workgroup barrier and its start-up all leave the
//     pipe idle); two waves of DIFFERENT workgroups fill each other's gaps, and
//     because they meet at different barriers neither ever waits for the other:
//     one workgroup's prologue, epilogue and barrier waits run under the other's
//     matrix work.  (Eight waves of one workgroup, two per SIMD, are coupled by
//     their common barrier: the four that lose the arbitration for the matrix pipe
//     finish their step alone, and start-up and drain of a workgroup are not
//     overlapped with anything.)
//   * K and V tiles (64 keys) travel HBM -> LDS with global_load_lds_dwordx4 (no
//     register staging) into two rings of two tiles each, XOR-swizzled in 16-byte
//     chunks so that the MFMA operand reads are bank-conflict free.  One barrier
//     per tile.  O rows leave through the (then idle) rings, so that every store
//     to HBM is a full 256-byte row per 16 lanes; Q fragments are loaded straight
//     from HBM in operand layout and parked in AccVGPRs.
//   * A wave works on half tiles of 32 keys in a three-stage pipeline: while the
//     softmax of half n runs on the VALU, the matrix pipe computes S^T = K Q^T of
//     half n+1 and O^T += V^T P^T of half n-1.  The interleaving is fixed by hand
//     with scheduling fences.  A step of the loop is aligned to the tiles it
//     READS -- halves (2t-1, 2t) take both halves of K tile t and of V tile t-1 --
//     so a tile is dead when its step ends and two buffers per ring suffice.
//   * The softmax reference: softmax is invariant to the value subtracted before
//     the exponential, so the reference only has to keep exp2() inside the
//     fp32/bf16 range.  It is set from the first half a wave processes and does
//     not move in the loop; a workgroup whose row sums show that scores have
//     outgrown it recomputes its rows with the max-based routine.  Results are
//     mathematically unchanged; the search for the row maximum and the rescale of
//     the accumulator disappear from the steady state.
//
// This kernel declares no static LDS: its dynamic LDS starts at address 0 and
// all LDS accesses below use plain byte addresses.
#include <type_traits>

#include "swaa_tile_d128.h"

namespace swaa {
namespace {

constexpr int kPWaves = 4;    // waves per workgroup
constexpr int kPThreads = 64 * kPWaves;
constexpr int kPRows = 32;    // query positions per wave
constexpr int kPWgRows = kPWaves * kPRows;            // query rows (head x position) per workgroup
constexpr int kStages = 2;                            // tiles per ring
constexpr int kTileBytes = kBk * kD * 2;              // 16 KiB
constexpr int kVRing = kStages * kTileBytes;          // V ring follows the K ring
constexpr int kSmemBytes = 2 * kStages * kTileBytes;  // 64 KiB: two workgroups per compute unit
constexpr int kStageBytes = kPRows * kD * 2;          // 8 KiB: a wave's 32 O rows on the way out (inside the K ring)
constexpr float kSumLimit = 1.2089258e24f;  // 2^80: a row sum that sends the workgroup back to the max-based path
constexpr float kSumFloor = 7.8886091e-31f;  // 2^-100: so does one this small (every score far below the reference)
constexpr int kPrefetch = 3;  // MFMAs between an LDS fragment read and its use

// ---- the pipelined sub-step, scheduled by hand -------------------------------------
// A sub-step issues 16 MFMAs, alternating S^T(n+1) += K Q^T (8, one chain) and
// O^T += V^T P^T(n-1) (8, four chains), and in their shadow the vector work of
// the softmax of half n, cut into 16 chunks.  Scheduling fences pin the order
// "MFMA, chunk, MFMA, chunk, ...".  LDS fragment reads are issued kPrefetch
// MFMAs ahead of their use, across the boundary between the two sub-steps of a
// step as well (not across steps: the next step's tiles are only known to have
// landed after the barrier between them).
//
// The mask: a half that is not fully visible to the wave's 32 rows has its
// invisible scores replaced by -inf right before its softmax (a select, so
// whatever an invisible key row holds -- NaN, infinities, stale LDS contents
// of a tile that does not exist -- never reaches a row that must not see it);
// their exponential is an exact 0.  A half that lies wholly outside a wave's
// rows (before its band, above its diagonal, past the last tile) therefore
// contributes nothing and needs no special case, and the softmax chunks are the
// same for every half.
//
// The softmax does not look for the row maximum: it keeps the reference it has
// (taken from the first half the wave sees).  exp2(s*c2 - mc) cannot overflow
// fp32 or bf16 unless a score exceeds the reference by more than 2^7 in the exp2
// domain, and the terms are never negative, so the final row sum bounds every
// term and every partial sum: if it reaches kSumLimit (or is not a number) the
// workgroup recomputes its rows with the max-based routine after the loop.
// (2^80: scores up to 55 nats above the reference pass, and the products with V
// in the O accumulators stay inside fp32 for |v| < 2^47; bf16 carries eight bits
// of P at any magnitude, so nothing is lost by a reference far below the maximum.)  It
// does the same if a row sum comes out below kSumFloor: a row whose first half
// was invisible to it has reference 0, and if all its scores lie a hundred
// binary orders below that, its terms leave the range fp32 resolves.
// Everything else is "subtract, exponentiate, add, pack".
struct SoftmaxScratch {
    float pe[16];
};

// first score element handled by chunk c: 16 scores over chunks 0..13
__device__ __forceinline__ constexpr int chunk_first_elem(int c) { return c >= 14 ? 16 : (c * 16) / 14; }

template <bool kF16>
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
                const bf16x2 pr = pack_pair<kF16>(w.pe[e - 1], w.pe[e]);
                pf[e / 8][(e - 1) % 8] = pr[0];
                pf[e / 8][e % 8] = pr[1];
                if (e % 8 == 7) pin_p(pf[e / 8]);
            }
        }
    }
}

// Scores of keys a lane's query row must not see become -inf (a select: the old
// value, whatever it is, is dropped).  k0h: first key of the half.
__device__ __forceinline__ void mask_scores(f32x16 &s, int k0h, int qpos, int W, int S, int hf) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int key = k0h + 8 * (e / 4) + 4 * hf + (e % 4);
        const bool vis = (key <= qpos) && ((key > qpos - W) || (key < S));
        s[e] = vis ? s[e] : -INFINITY;
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

template <bool kF16>
__device__ __forceinline__ bf16x8 rowsum_selector(int lane) {
    // A operand: lane l holds row l % 16, k-group l / 16
    const int m = lane & 15, kg = lane >> 4;
    const bool on = (m == 0 && (kg & 1) == 0) || (m == 1 && (kg & 1) == 1);
    const bf16x2 one = pack_pair<kF16>(1.f, 1.f), zero = pack_pair<kF16>(0.f, 0.f);
    bf16x8 a;
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = on ? one[0] : zero[0];
    return a;
}
template <bool kF16>
__device__ __forceinline__ void mfma_rowsum(f32x4 &acc, const bf16x8 sel_acc, const bf16x8 pfrag) {
    if constexpr (kF16)
        asm("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "a"(sel_acc), "v"(pfrag));
    else
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

// kHasS: the scores of the following half are computed here (not in the last sub-step of a
//   workgroup, which issues the P V MFMAs only).
// kHasPV: there is a previous half whose P V product is due (not in the very first
//   sub-step of a workgroup, which issues the K Q^T MFMAs only).
// kLoadFirst: the first kPrefetch fragments are requested here (first sub-step of a
//   step); otherwise the caller passes them in fpre.
// kPrefetchNext: on return fpre holds the first fragments of the following sub-step.
// mask_cur / k0h_cur: whether the half whose softmax runs here (s_cur) needs the
//   mask, and its first key.
template <bool kF16, bool kHasS, bool kHasPV, bool kLoadFirst, bool kPrefetchNext>
__device__ __forceinline__ void pipelined_substep(const LaneAddr &la, const HalfOffsets &ho, bf16x8 (&fpre)[kPrefetch],
                                                  const bf16x8 (&qf)[kKS], f32x16 &s_next, f32x16 &s_cur,
                                                  bf16x8 (&p_cur)[2], const bf16x8 (&p_prev)[2], f32x16 (&o)[kDB],
                                                  RowState &st, f32x4 (&lsum)[2], const bf16x8 &sel, float c2,
                                                  bool mask_cur, int k0h_cur, int qpos, int W, int S, int hf) {
    SoftmaxScratch w;
    bf16x8 frag[16 + kPrefetch];
    auto wanted = [](int slot) __attribute__((always_inline)) { return (slot & 1) ? kHasPV : kHasS; };
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i)
        if (wanted(i)) frag[i] = kLoadFirst ? load_slot(la, ho, i) : fpre[i];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int nxt = i + kPrefetch;
        if ((nxt < 16 || kPrefetchNext) && (nxt >= 16 || wanted(nxt))) frag[nxt] = load_slot(la, ho, nxt);
        if ((i & 1) == 0) {
            if (kHasS) {
                if (i == 0)
                    mfma_s_first<kF16>(s_next, frag[i], qf[0]);
                else
                    mfma_s<kF16>(s_next, frag[i], qf[i / 2]);
            }
        } else if (kHasPV) {
            mfma_acc<kF16>(o[(i / 2) % kDB], frag[i], p_prev[(i / 2) / kDB]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (i == 0 && __builtin_expect(mask_cur, 0)) mask_scores(s_cur, k0h_cur, qpos, W, S, hf);
        softmax_chunk<kF16>(i, s_cur, c2, st, w, p_cur);
        if (i == 15) {  // P^T of this half is complete (and two MFMAs old)
            mfma_rowsum<kF16>(lsum[0], sel, p_cur[0]);
            mfma_rowsum<kF16>(lsum[1], sel, p_cur[1]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (kPrefetchNext) {
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) fpre[i] = frag[16 + i];
    }
}

// kF16: q, k, v and out hold IEEE binary16 instead of bfloat16 (the precision the paper serves
// its models in, Sec. 4.1.1).  Same kernel; what differs is the exponent range of P: binary16
// ends at 65504, so the reference is set 2^4 below the first half's largest score (later
// scores may exceed it by 2^12, about 8 nats, before a P overflows; smaller terms keep full
// precision down to 2^-18 of it and fade out through the subnormals), and a P that did
// overflow shows as a non-finite sum of the rounded P and sends the workgroup to the
// max-based second pass; so does a sum of rounded P below 2^-6 (a row without a visible
// key in its first half has reference 0, and if all its scores lie several nats below that
// its terms are subnormal or vanish).
// kPaged: k and v are a paged cache addressed through p.block_table (its own instantiation, so
// that the contiguous kernel carries none of the table arithmetic).
template <bool kF16, bool kPaged>
__global__ __launch_bounds__(kPThreads, 2) void swaa_fwd_pipelined_kernel(const FwdParams p) {
    WorkItem wi;
    if (!decode_work(p, wi)) return;
    SeqGeom sg;
    if (!seq_geom(p, wi.b, sg)) return;
    const int hpb = wi.hpb;
    const int rows_per_wg = kPWgRows / hpb;
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
    const int W = (qpos >= sg.n_prompt) ? Nk : p.W;

    const __bf16 *qg = p.q + sg.q_batch * p.q_sb + (long long)head * p.q_sh + sg.q_row0 * p.q_sn;

    // ---- this lane's Q fragments (B operand of S^T = K Q^T: query row l32, 16 bytes at
    // 32 ks + 16 hf), straight from HBM (ordinary loads: the compiler places their wait in
    // front of the first use; that wait also covers the tile copies issued below, which
    // it cannot see -- the loads complete in order) ----
    bf16x8 qf[kKS];
    {
        const char *qrow =
            reinterpret_cast<const char *>(qg) + (size_t)min(r0 + l32, Nq - 1) * (size_t)(p.q_sn * 2) + 16 * hf;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * ks);
    }

    // ---- the schedule, in halves of 32 keys: the halves that hold sink keys in front of the
    // band, then the halves from the one that holds the first row's first window key to the one
    // that holds the last row; a workgroup that holds a generated token visits every half up
    // to its diagonal.  Two consecutive visited halves make one 64-key tile of the rings (a
    // tile need not be 64 consecutive keys: the last sink half and the first band half share
    // one); an odd count is padded with a half past the last row, which no row can see.
    const int band_lo = (wg_p1 >= sg.n_prompt) ? 0 : max(0, wg_p0 - p.W + 1);
    const int hb_lo = band_lo >> 5, hb_hi = wg_p1 >> 5;
    const int n_sink_h = min((min(S, band_lo) + 31) >> 5, hb_lo);
    const int n_halves = n_sink_h + (hb_hi - hb_lo + 1);
    const int J = (n_halves + 1) >> 1;  // tiles
    // i-th visited half -> its index among all halves of the sequence (first key / 32); the
    // padding half comes out as hb_hi + 1
    auto half_of = [&](int i) __attribute__((always_inline)) { return i < n_sink_h ? i : i - n_sink_h + hb_lo; };

    const uint32_t k_rsb = (uint32_t)(p.k_sn * 2), v_rsb = (uint32_t)(p.v_sn * 2);  // row strides in bytes
    const __bf16 *kg = p.k + sg.k_batch * p.k_sb + (long long)wi.kvh * p.k_sh + sg.k_row0 * p.k_sn;
    const __bf16 *vg = p.v + sg.k_batch * p.v_sb + (long long)wi.kvh * p.v_sh + sg.k_row0 * p.v_sn;
    __bf16 *og = p.out + sg.q_batch * p.o_sb + (long long)head * p.o_sh + sg.q_row0 * p.o_sn;

    // ---- HBM -> LDS tile copies -------------------------------------------------
    // One wave instruction moves 64 x 16 bytes = 4 rows, a wave moves 16 rows of K and of V
    // per tile: waves 0, 1 the tile's first half, waves 2, 3 its second (instruction i of wave
    // w: rows 16 (w & 1) + 4 i + lrow of that half).  The LDS side is linear in the lane id,
    // the swizzle is applied on the global side: LDS chunk (row, c') receives global chunk
    // c' ^ f(row) of that row, with f(row) = ((row & 7) << 1) | ((row >> 3) & 1) for K (16
    // consecutive rows read the same logical chunk) and (row & 3) << 2 for V (4 consecutive
    // rows read the same 64 bytes).
    const int lrow = lane >> 4;  // row within the 4-row group
    const int lchk = lane & 15;  // LDS chunk within the row
    const int hslot = wave >> 1;  // which half of a tile this wave copies
    const int hrow0 = 16 * (wave & 1);
    // byte offsets of this lane's 16 bytes from the half's first row, minus 1024 i: the four
    // copies of a tile share one M0 value and use the instruction's offset field (1024 i), which
    // moves the LDS address and the global address alike
    uint32_t voff_k[4], voff_v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t row = (uint32_t)(hrow0 + 4 * i + lrow);
        // row & 7 = 4 (i & 1) + lrow, (row >> 3) & 1 = i >> 1
        const uint32_t fk = (uint32_t)(((4 * (i & 1) + lrow) << 1) | (i >> 1));
        voff_k[i] = row * k_rsb + (((uint32_t)lchk ^ fk) << 4) - (uint32_t)(1024 * i);
        voff_v[i] = row * v_rsb + (((uint32_t)lchk ^ (uint32_t)(lrow << 2)) << 4) - (uint32_t)(1024 * i);
    }
    // LDS address = M0 + offset field + 16 * lane; global address = base + off + offset field.
    // Issued as assembly on purpose: the compiler would otherwise make every later LDS read
    // wait for the copy.
    auto copy4 = [](const uint32_t (&vo)[4], const char *base, uint32_t lds) __attribute__((always_inline)) {
        asm volatile(
            "s_mov_b32 m0, %5\n\ts_nop 0\n\t"
            "global_load_lds_dwordx4 %0, %4\n\t"
            "global_load_lds_dwordx4 %1, %4 offset:1024\n\t"
            "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
            "global_load_lds_dwordx4 %3, %4 offset:3072" ::"v"(vo[0]),
            "v"(vo[1]), "v"(vo[2]), "v"(vo[3]), "s"(base), "s"(lds)
            : "memory");
    };
    const bool last_ragged = ((hb_hi + 1) << 5) > Nk;  // the last band half runs past the sequence's end
    // This wave's four copies of tile j (K or V) into ring buffer `buf`, from scratch: which
    // half, where it starts, whether its rows run past the sequence's last row (then they
    // repeat that row -- they are masked later -- so that the reads stay in bounds; the padding
    // half repeats the last real half).  A tile that does not exist is not copied.
    // (the table is only read while the kernel runs: addressed as constant memory, so that the
    // lookups are scalar loads -- as vector loads they would share the tile copies' counter, and
    // waiting for a table entry would mean waiting for every copy in flight)
    typedef const int __attribute__((address_space(4))) *TablePtr;
    const TablePtr bt = kPaged ? (TablePtr)(p.block_table + (size_t)wi.b * p.bt_stride) : nullptr;
    auto issue_tile = [&](int j, int buf, bool is_k) __attribute__((always_inline)) {
        if (2 * j >= n_halves) return;
        const int g = min(half_of(2 * j + hslot), hb_hi);
        const uint32_t rsb = is_k ? k_rsb : v_rsb;
        const uint32_t l = (uint32_t)((is_k ? 0 : kVRing) + buf * kTileBytes + wave * 4096);
        if constexpr (kPaged) {
            // Paged cache: this wave's 16 rows start at a multiple of 16, so they share a page and
            // the table lookup is uniform.  A block that starts past the last token is replaced by
            // the block that holds it, rows past it repeat it (all masked later); the page number
            // is clamped to the cache whatever the table says.
            const int key0 = min(32 * g + hrow0, (Nk - 1) & ~15);
            const int page = min(max(bt[key0 / p.page_size], 0), p.num_pages - 1);
            const char *base = reinterpret_cast<const char *>(is_k ? kg : vg) +
                               ((long long)page * (is_k ? p.k_sb : p.v_sb)) * 2 + (size_t)(key0 % p.page_size) * rsb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = 4 * i + lrow;  // row of the block, and how far it lies past the last token
                const uint32_t off = (is_k ? voff_k[i] : voff_v[i]) + (uint32_t)(1024 * i) -
                                     (uint32_t)(hrow0 + max(key0 + r - (Nk - 1), 0)) * rsb;
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base),
                             "s"(l + (uint32_t)(1024 * i))
                             : "memory");
            }
            return;
        }
        const char *base = reinterpret_cast<const char *>(is_k ? kg : vg) + (size_t)(32 * g) * rsb;
        if (__builtin_expect(last_ragged && g == hb_hi, 0)) {
            // (one M0 value per copy and no offset field: a clamped row may lie less than
            // 1024 i bytes behind the half's first row)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t off = (is_k ? voff_k[i] : voff_v[i]) + (uint32_t)(1024 * i) -
                                     (uint32_t)max(32 * g + hrow0 + 4 * i + lrow - (Nk - 1), 0) * rsb;
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base),
                             "s"(l + (uint32_t)(1024 * i))
                             : "memory");
            }
        } else {
            copy4(is_k ? voff_k : voff_v, base, l);
        }
    };
    auto issue_k = [&](int j, int buf) __attribute__((always_inline)) { issue_tile(j, buf, true); };
    auto issue_v = [&](int j, int buf) __attribute__((always_inline)) { issue_tile(j, buf, false); };

    // Tiles in the order they are needed: K(0) first, the other three stream in behind it.
    issue_k(0, 0);
    issue_v(0, 0);
    issue_k(1, 1);
    issue_v(1, 1);

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
    f32x4 lsum[2];  // column sums of the rounded P^T (mfma_rowsum), one accumulator per fragment
#pragma unroll
    for (int e = 0; e < 4; ++e) lsum[0][e] = lsum[1][e] = 0.f;
    bf16x8 sel = rowsum_selector<kF16>(lane);
    asm volatile("s_nop 1" : "+a"(lsum[0]), "+a"(lsum[1]), "+a"(sel));

    // A wave needs no mask on a 32-key half when all its keys are visible to all
    // its 32 rows: at or below the first row's diagonal, and inside the window of
    // its last prompt row (if it has one) or all sinks.
    const int wbound = window_bound(p0, kPRows, p.W, sg.n_prompt);
    auto half_masked = [&](int k0h) __attribute__((always_inline)) { return !((k0h + 31 <= p0) && ((k0h > wbound) || (k0h + 31 < S))); };

    // (Worked out here, while the first copies travel.)
    // Steps [ja, jb) of this wave need no mask.  Step t runs the softmax of the visited halves
    // 2 t - 1 and 2 t.  A band half g (keys 32 g .. 32 g + 31) lies inside every row's window
    // iff 32 g > wbound and at or below the first row's diagonal iff 32 g + 31 <= p0.
    // (Halves that need no mask because they hold sink keys only take the general step.)
    int ja, jb;
    {
        const int g_min = (wbound >> 5) + 1, g_max = (p0 - 31) >> 5;
        const int i_min = max(n_sink_h, g_min - hb_lo + n_sink_h);  // first unmasked band half
        const int i_max = min(g_max - hb_lo + n_sink_h, n_halves - 1);  // last one
        ja = (i_min + 2) >> 1;       // 2 t - 1 >= i_min
        jb = max(ja, (i_max >> 1) + 1);  // 2 t <= i_max
    }

    // The Q fragments move to AccVGPRs (the idle cycles keep the copies two wait states away
    // from the first MFMA that reads them).  The compiler waits for the loads here, hence
    // for every tile copy issued so far as well: K(0), V(0), K(1), V(1) have landed.
    asm volatile("s_nop 1"
                 : "+a"(qf[0]), "+a"(qf[1]), "+a"(qf[2]), "+a"(qf[3]), "+a"(qf[4]), "+a"(qf[5]), "+a"(qf[6]), "+a"(qf[7]));
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), should the compiler's own wait ever be weaker
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- pipeline prologue: scores of the very first half, and the softmax reference ----
    // The reference is the largest visible score of that half (0 for a row that
    // sees none of its keys); from here on it does not move.
    RowState rs;
    rs.l = 0.f;
    rs.lb = 0.f;
    {
        qk_half<kF16>(la, 0u, qf, s_a);
        mask_scores(s_a, 32 * half_of(0), qpos, W, S, hf);
        float mx = s_a[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s_a[e]);
        mx = half_swap_max(mx);
        rs.mc = (mx == -INFINITY) ? 0.f : mx * c2 - (kF16 ? 4.f : 0.f);
    }

    bf16x8 fpre[kPrefetch];  // first fragments of the second sub-step of a step, requested during the first
    // softmax of (tile 0, half 0) | scores of (tile 0, half 1); no P V product is due yet
    {
        const HalfOffsets h = {kHalfBytes, 0, 0, 0};
        pipelined_substep<kF16, true, false, true, false>(la, h, fpre, qf, s_b, s_a, p_a, p_b, oacc, rs, lsum, sel, c2, false, 0,
                                              qpos, W, S, hf);
    }
    // every wave is done with K(0), which is free afterwards
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue_k(2, 0);

    // Step t = 1 .. J - 1 reads K tile t (ring buffer t % 2) and V tile t - 1 (buffer
    // (t - 1) % 2).  The ring position R = t % 2 is a template argument, so every LDS offset
    // below is a constant that folds into the instructions' offset fields (no address
    // arithmetic in the loop).
    //
    // Two versions of the step.  The general one looks at the two halves whose softmax it
    // runs, masks them where needed, and works out the next copies from scratch (sink
    // halves, the jump to the band, the ragged last half, the end of the list).  The lean one
    // serves the interior of a wave's band, where no half needs a mask and the next tiles
    // simply follow the previous ones in memory.
    auto substeps = [&](auto ring_pos, bool mask_p, int k0p, bool mask_0, int k0) __attribute__((always_inline)) {
        constexpr int R = decltype(ring_pos)::value;
        constexpr uint32_t kb0 = R * kTileBytes, kb1 = kb0 + kHalfBytes;        // K(t)
        constexpr uint32_t vb0 = (1 - R) * kTileBytes, vb1 = vb0 + kHalfBytes;  // V(t-1)
        // softmax of (t-1, half 1) | scores of (t, half 0) | P V of (t-1, half 0)
        const HalfOffsets h1 = {kb0, vb0, kb1, vb1};
        pipelined_substep<kF16, true, true, true, true>(la, h1, fpre, qf, s_a, s_b, p_b, p_a, oacc, rs, lsum, sel, c2, mask_p,
                                                  k0p, qpos, W, S, hf);
        // softmax of (t, half 0) | scores of (t, half 1) | P V of (t-1, half 1)
        const HalfOffsets h2 = {kb1, vb1, 0, 0};
        pipelined_substep<kF16, true, true, false, false>(la, h2, fpre, qf, s_b, s_a, p_a, p_b, oacc, rs, lsum, sel, c2, mask_0,
                                                    k0, qpos, W, S, hf);
        // K(t+1), V(t) must have landed; K(t) and V(t-1) are free afterwards
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        asm volatile("" ::: "memory");  // no LDS access may be moved across the barrier
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto general_step = [&](auto ring_pos, int t) __attribute__((always_inline)) {
        constexpr int R = decltype(ring_pos)::value;
        const int k0p = 32 * half_of(2 * t - 1), k0 = 32 * half_of(2 * t);
        substeps(ring_pos, half_masked(k0p), k0p, half_masked(k0), k0);
        issue_k(t + 2, R);
        issue_v(t + 1, 1 - R);
    };
    // the lean step's copies: this wave's half of K tile t + 2 and of V tile t + 1
    const char *k_next = nullptr, *v_next = nullptr;
    // The lean step over a paged cache: the 16 rows a wave copies per tile lie in one page (page
    // sizes are multiples of 16), so a copy needs that page's number -- a block-table entry, a
    // scalar load.  It is asked for one step ahead: on entry (pg_k, in_k) are page and row
    // inside it of this wave's rows of K tile t + 2, (pg_v, in_v) those of V tile t + 1 (the
    // keys of K tile t + 1, so last step's pg_k), and the entry of tile t + 3 is requested
    // before the arithmetic and has landed when the step ends.
    int pg_k = 0, in_k = 0, pg_v = 0, in_v = 0, key_n = 0;
    auto paged_base = [&](bool is_k, int page, int in_page) __attribute__((always_inline)) {
        // (the row offsets in voff_* count from the half's first row: step back this wave's hrow0 rows;
        // the page number is clamped to the cache whatever the table says)
        page = min(max(page, 0), p.num_pages - 1);
        return reinterpret_cast<const char *>(is_k ? kg : vg) + ((long long)page * (is_k ? p.k_sb : p.v_sb)) * 2 +
               (long long)(in_page - hrow0) * (long long)(is_k ? k_rsb : v_rsb);
    };
    auto lean_step = [&](auto ring_pos) __attribute__((always_inline)) {
        constexpr int R = decltype(ring_pos)::value;
        int pg_n = 0, in_n = 0;
        if constexpr (kPaged) {
            key_n += kBk;
            const int kc = min(key_n, (Nk - 1) & ~15);  // (past the lean range the entry is asked for but not used)
            pg_n = bt[kc / p.page_size];
            in_n = kc % p.page_size;
        }
        substeps(ring_pos, false, 0, false, 0);
        if constexpr (kPaged) {
            k_next = paged_base(true, pg_k, in_k);
            v_next = paged_base(false, pg_v, in_v);
            pg_v = pg_k;
            in_v = in_k;
            pg_k = pg_n;
            in_k = in_n;
        }
        copy4(voff_k, k_next, (uint32_t)(R * kTileBytes + wave * 4096));
        k_next += (size_t)kBk * k_rsb;
        copy4(voff_v, v_next, (uint32_t)(kVRing + (1 - R) * kTileBytes + wave * 4096));
        v_next += (size_t)kBk * v_rsb;
    };
    static_assert(kStages == 2, "the loops below walk two ring positions");
    const std::integral_constant<int, 0> even{};
    const std::integral_constant<int, 1> odd{};
    // Lean steps: [ja, jb) needs no mask; the copies step t issues are the visited halves
    // 2 t + 2 .. 2 t + 5, which must be band halves (they are: 2 t - 1 >= n_sink_h) that exist
    // and do not run past the sequence's end.  The range starts at an odd step (steps run
    // in pairs: odd, even).
    const int lean_end = min(jb, ((n_halves - 6 - (last_ragged ? 1 : 0)) >> 1) + 1);
    const int lean_begin = ja | 1;
    bool lean_pending = lean_begin + 1 < lean_end;
    for (int t = 1; t < J;) {  // t is odd here
        if (lean_pending && t == lean_begin) {
            if constexpr (!kPaged) {
                k_next = reinterpret_cast<const char *>(kg) + (size_t)(32 * half_of(2 * t + 4 + hslot)) * k_rsb;
                v_next = reinterpret_cast<const char *>(vg) + (size_t)(32 * half_of(2 * t + 2 + hslot)) * v_rsb;
            } else {
                // (both tiles are band tiles inside the sequence: their keys are 64 apart)
                key_n = 32 * half_of(2 * t + 4 + hslot) + hrow0;
                pg_k = bt[key_n / p.page_size];
                in_k = key_n % p.page_size;
                pg_v = bt[(key_n - kBk) / p.page_size];
                in_v = (key_n - kBk) % p.page_size;
            }
            for (; t + 1 < lean_end; t += 2) {
                lean_step(odd);
                lean_step(even);
            }
            lean_pending = false;
        }
        general_step(odd, t);
        if (++t >= J) break;
        general_step(even, t);
        ++t;
    }
    // ---- tail: softmax of the last half | P V of the half before it, then the last P V ----
    {
        const uint32_t vb = (uint32_t)(((J - 1) & 1) * kTileBytes);  // V(J-1)
        const int k0l = 32 * half_of(2 * J - 1);
        const HalfOffsets h = {0, vb, 0, 0};
        pipelined_substep<kF16, false, true, true, false>(la, h, fpre, qf, s_a, s_b, p_b, p_a, oacc, rs, lsum, sel, c2,
                                                    half_masked(k0l), k0l, qpos, W, S, hf);
        // (the column sums of p_b, issued at the end of the sub-step, complete under these)
        pv_half<true, kF16>(la, vb + kHalfBytes, p_b, oacc);
    }

    // ---- scores outgrew the reference somewhere in this workgroup (inputs with
    // score jumps of tens of nats): recompute its rows with the max-based routine,
    // one tile at a time, no pipelining ------------------------------------------
    // (workgroup-wide OR through four flag words at the start of the V buffer that does NOT hold
    // the last tile: other waves may still be reading the last tile's V rows in their tail, and
    // the K ring becomes the O staging area right after the vote)
    // (what the rest of the kernel needs of the lane id is worked out again here, so that it
    // occupies no registers through the key loop)
    const int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int l32_e = lane_e & 31;
    float l_row = half_swap_sum(rs.l);
    float lb_row = rowsum_of_column(lsum, l32_e);
    bool redo;
    {
        // a sum inside (kSumFloor, kSumLimit), tested on the bit pattern: positive floats order like
        // unsigned integers, and zero, infinity and every NaN pattern fall outside the interval
        // (the build does not honour NaNs in float comparisons).  Rows past the end of the
        // sequence (the ragged last tile; they may see no key at all) have no say.
        const bool in_range = (__float_as_uint(l_row) - (__float_as_uint(kSumFloor) + 1u)) <
                              (__float_as_uint(kSumLimit) - (__float_as_uint(kSumFloor) + 1u));
        // binary16: a P beyond 65504 became infinity, and the sum of the rounded P with it; and a
        // row whose terms all sank into (or below) the subnormals has a small sum of rounded P
        // (a row that took its reference from a visible key has a term of 2^4)
        const bool p_sound = !kF16 || (__float_as_uint(lb_row) - 0x3c800000u) < (0x7f800000u - 0x3c800000u);  // [2^-6, inf)
        const int mine = __any(!(in_range && p_sound) && r0 + l32_e < Nq) ? 1 : 0;
        const uint32_t flag_base = (uint32_t)(kVRing + (J & 1) * kTileBytes);
        if (lane_e == 0) *(int __attribute__((address_space(3))) *)(uintptr_t)(flag_base + wave * 4) = mine;
        __syncthreads();
        int any = 0;
#pragma unroll
        for (int w = 0; w < kPWaves; ++w)
            any |= *(const int __attribute__((address_space(3))) *)(uintptr_t)(flag_base + w * 4);
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
        // tiles alternate between the two buffers of each ring: the copy of tile j + 1 travels
        // while tile j is worked on
        __syncthreads();  // everyone has read the vote (its flag words lie inside the V ring)
        issue_k(0, 0);
        issue_v(0, 0);
        for (int j = 0; j < J; ++j) {
            const uint32_t boff = (uint32_t)((j & 1) * kTileBytes);
            if (j + 1 < J) {
                issue_k(j + 1, (j + 1) & 1);
                issue_v(j + 1, (j + 1) & 1);
                __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8): all but the eight copies just issued
            } else {
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
            }
            __syncthreads();  // tile j has landed for every wave
#pragma unroll 1
            for (int hh = 0; hh < 2; ++hh) {
                float alpha;
                qk_half<kF16>(la, boff + (uint32_t)(hh * kHalfBytes), qf, s_a);
                softmax_half<true, kF16>(s_a, 32 * half_of(2 * j + hh), qpos, W, S, hf, c2, rs, p_a, alpha);
                rescale(oacc, alpha);
                pv_half<true, kF16>(la, boff + (uint32_t)(hh * kHalfBytes), p_a, oacc);
            }
            __syncthreads();  // everyone is done with this buffer: tile j + 2 is copied into it next
        }
        row_sums(rs, l_row, lb_row);
        // (after the loop's last barrier the rings are free: they become the O staging area below)
    }

    // ---- epilogue: O / (sum of the rounded P) -> bf16 through LDS (8 KiB per wave at the start
    // of the K ring, which nobody reads any more), so that the stores to HBM are whole rows;
    // lse = (mc + log2 l) * ln 2 -------------------
    {
        const int lane = lane_e, l32 = l32_e, hf = lane_e >> 5, lrow = lane_e >> 4, lchk = lane_e & 15;
        const uint32_t stage = (uint32_t)(wave * kStageBytes);
        const float inv_l = 1.f / lb_row;  // rows past the end: never stored
        const int fr = ((l32 & 7) << 1) | ((l32 >> 3) & 1);
        const uint32_t o_lane = stage + (uint32_t)(l32 * 256 + (fr << 4) + 8 * hf);
#pragma unroll
        for (int db = 0; db < kDB; ++db) {
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const bf16x2 lo = pack_pair<kF16>(oacc[db][4 * e4 + 0] * inv_l, oacc[db][4 * e4 + 1] * inv_l);
                const bf16x2 hi = pack_pair<kF16>(oacc[db][4 * e4 + 2] * inv_l, oacc[db][4 * e4 + 3] * inv_l);
                const bf16x4 o4 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
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
    if (p.wg_rows != kPWgRows) return hipErrorInvalidValue;  // the plan must be the one for this kernel's workgroups
    const unsigned grid = (unsigned)(p.chunk * kXcds);
    // (64 KiB of dynamic LDS is what a kernel gets without asking)
    static_assert(kSmemBytes <= 64 * 1024, "more would need hipFuncSetAttribute");
    const bool paged = p.block_table != nullptr;
    if (p.fp16 && paged)
        hipLaunchKernelGGL((swaa_fwd_pipelined_kernel<true, true>), dim3(grid), dim3(kPThreads), kSmemBytes, stream, p);
    else if (p.fp16)
        hipLaunchKernelGGL((swaa_fwd_pipelined_kernel<true, false>), dim3(grid), dim3(kPThreads), kSmemBytes, stream, p);
    else if (paged)
        hipLaunchKernelGGL((swaa_fwd_pipelined_kernel<false, true>), dim3(grid), dim3(kPThreads), kSmemBytes, stream, p);
    else
        hipLaunchKernelGGL((swaa_fwd_pipelined_kernel<false, false>), dim3(grid), dim3(kPThreads), kSmemBytes, stream, p);
    return hipGetLastError();
}

}  // namespace swaa
