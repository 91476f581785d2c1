// Decode-shape attention, head dimension 128, gfx950: the Nq newest tokens of a
// sequence attend to a cache of Nk keys and values (paper Sec. 3.1.1: all of
// them under FA Decode; their window plus the sink tokens of Sec. 3.2.1 when
// decoding stays on sliding-window attention).
//
// With a handful of query rows the cache is read once and nothing is reused:
// the bound is HBM bandwidth, and what matters is the number of bytes in flight.
//
//   * The G query heads x Nq rows of one (batch, KV head) pair are the 32
//     columns of an MFMA tile (more rows: more column tiles), so one pass over
//     K and V serves the whole GQA group.  Padding columns cost matrix-core
//     time only, of which there is plenty.
//   * The visited keys are cut into splits; a workgroup is ONE wave that owns a
//     three-stage ring of 32-key half tiles (K 8 KiB + V 8 KiB per stage) in
//     LDS, filled by global_load_lds_dwordx4 with whole 256-byte rows per 16
//     lanes.  No barriers: a wave waits on its own copies only.  48 KiB of LDS
//     per workgroup lets three of them share a CU: 96 KiB of copies in flight
//     per CU, 24 MiB over the chip.  (Workgroups that compute two column tiles
//     take a two-stage ring and run four to a CU: decode_stages.)
//   * Per half: all K and V^T operand fragments go from LDS to registers (V^T
//     through transposing reads), the copy of the half three ahead is issued into
//     the stage just emptied, and only then the arithmetic runs: S^T = K Q^T (8
//     MFMAs), max-based softmax (mask only on halves that are not fully visible),
//     O^T += V^T P^T (8 MFMAs).  The copies thus never wait for arithmetic.  The
//     query rows are loaded from HBM in operand layout and parked in AccVGPRs.
//   * The cache is a contiguous strided tensor or a paged one (a block table of
//     page numbers per sequence, pages of page_size tokens: the layout of a
//     serving engine's cache manager); sequences of a batch may have different
//     cache lengths (seq_lens): the splits are then planned on the device, in
//     proportion to the lengths (DecodeParams::ragged).
//   * Each workgroup leaves (O unnormalised, reference, row sum) for its valid
//     columns in the workspace; swaa_decode_merge_kernel combines the splits.
//
// The split kernel declares no static LDS: its dynamic LDS starts at address 0
// and all its LDS accesses use plain byte addresses.
#include <atomic>
#include <type_traits>

#include "swaa_decode.h"
#include "swaa_tile_d128.h"

namespace swaa {
namespace {

constexpr int kDStageBytes = 2 * kHalfBytes;          // K half, then V half
// Stages of the ring: three (48 KiB, three workgroups per CU) for one column tile per workgroup,
// where the copies in flight are what counts; two (32 KiB) for two tiles, whose 450 registers
// leave one wave per SIMD, so that four such workgroups fit a CU: those shapes are bound by the
// wave's own instruction stream, and a fourth wave per CU is a third more of it.
constexpr int decode_stages(int tiles) { return tiles == 2 ? 2 : 3; }
constexpr int decode_wgs_per_cu(int tiles) { return tiles == 2 ? 4 : 3; }
constexpr int kCopiesPerHalf = 16;                    // wave instructions per stage: 8 for K, 8 for V
constexpr int kMergeThreads = 1024;
constexpr int kRounds = 1;  // rounds of resident workgroups the split plan aims for

// ---- the split plan of a batch with per-sequence lengths, worked out by every workgroup of the
// split kernel (DecodeParams::ragged has the rules) ----
// Lane l keeps the halves that sequences l, 64 + l, ... visit (0 beyond the batch).
constexpr int kRaggedLaneRounds = kRaggedMaxBatch / 64;
struct RaggedHalves {
    unsigned n[kRaggedLaneRounds];
};
__device__ __forceinline__ RaggedHalves ragged_halves(const DecodeParams &p, int lane) {
    RaggedHalves h;
#pragma unroll
    for (int r = 0; r < kRaggedLaneRounds; ++r) {
        const int b = 64 * r + lane;
        const int nk = max(min(p.seq_lens[min(b, p.B - 1)], p.Nk), p.Nq);
        h.n[r] = b < p.B ? (unsigned)visited_halves(nk, p.Nq, p.W, p.S).n : 0u;
    }
    return h;
}
__device__ __forceinline__ unsigned ragged_halves_per_split(const DecodeParams &p, const RaggedHalves &h) {
    auto sum_over_sequences = [&](auto f) {
        unsigned mine = 0;
#pragma unroll
        for (int r = 0; r < kRaggedLaneRounds; ++r) mine += f(h.n[r]);
        return wave_read_lane(wave_inclusive_scan(mine), 63);
    };
    const unsigned target = (unsigned)p.units_target;
    const unsigned total = sum_over_sequences([](unsigned n) { return n; });
    unsigned hps = (total + target - 1) / target;
    hps = hps < 4u ? 4u : hps;
    // Rounding up per sequence can leave a few units more than the target, i.e. a handful of
    // workgroups in one more round than planned: lengthen the splits until the count fits (a
    // few steps; whatever they end on, the count stays below units_target + B).
    for (int it = 0; it < 4; ++it) {
        const unsigned units = sum_over_sequences([&](unsigned n) { return (n + hps - 1) / hps; });
        if (units <= target) break;
        const unsigned longer = (hps * units + target - 1) / target;
        hps = longer > hps ? longer : hps + 1;
    }
    return hps;
}
// The sequence and the split of unit `unit` of the list (sequence 0's splits, then sequence 1's, ...)
// and how many splits that sequence has; false beyond the list's end.
__device__ __forceinline__ bool ragged_find(const RaggedHalves &h, unsigned hps, unsigned unit, int &b, int &split, int &n_splits) {
    unsigned before = 0;
#pragma unroll
    for (int r = 0; r < kRaggedLaneRounds; ++r) {
        const unsigned mine = (h.n[r] + hps - 1) / hps;
        const unsigned incl = wave_inclusive_scan(mine);
        const unsigned in_round = wave_read_lane(incl, 63);
        if (unit - before < in_round) {
            const unsigned rel = unit - before;
            const int n = __popcll(__ballot(incl <= rel));  // sequences among these 64 that end at or before the unit
            const unsigned base = n ? wave_read_lane(incl, n - 1) : 0u;
            // (the same in all lanes; read through the first lane so that the compiler knows it
            // and keeps the addresses built from them in scalar registers)
            b = __builtin_amdgcn_readfirstlane(64 * r + n);
            split = __builtin_amdgcn_readfirstlane((int)(rel - base));
            n_splits = (int)wave_read_lane(mine, n);
            return true;
        }
        before += in_round;
    }
    return false;
}

// kPaged: k and v are a paged cache addressed through p.block_table (its own instantiation).
// kTiles: column tiles a workgroup computes from the same K and V fragments (1, or 2 when a pair
// has more than 32 query rows: two tiles in two workgroups would read every key twice).
template <bool kF16, bool kPaged, int kTiles>
__global__ __launch_bounds__(64) void swaa_decode_split_kernel(const DecodeParams p) {
    // Workgroups reach the eight dies round-robin; the list has fewer than 2^31 items: 32-bit
    // arithmetic, divisions as multiplications.  Sequences of one length: die x takes the x-th
    // contiguous chunk of the item list (a die streams neighbouring memory: 3 % faster on one
    // long sequence).  Per-sequence lengths: the units (sequence, split) x KV heads go to the
    // dies in turn, so that whatever the lengths every die gets its share of the long sequences.
    // Either way the column-tile groups of one (pair, split), which read the same keys, share a die.
    constexpr int kDStages = decode_stages(kTiles);
    const int lane = threadIdx.x;
    const unsigned items = (unsigned)p.wg_items;
    unsigned witem;
    if (p.ragged) {
        const unsigned per_round = kXcds * (unsigned)p.n_ctgroups;
        const unsigned round = fastdiv(blockIdx.x, p.div_per_round), rem = blockIdx.x - round * per_round;
        witem = round * per_round + (rem % kXcds) * (unsigned)p.n_ctgroups + rem / kXcds;
    } else {
        const unsigned chunk = (items + kXcds - 1) / kXcds;
        const unsigned slot = blockIdx.x / kXcds;
        witem = (blockIdx.x % kXcds) * chunk + slot;
        if (slot >= chunk) return;
    }
    if (witem >= items) return;
    const unsigned item_ct = fastdiv(witem, p.div_ctgroups);      // witem / n_ctgroups
    const int ctg = (int)(witem - item_ct * (unsigned)p.n_ctgroups);
    int b, kvh, split, halves_per_split;
    size_t slot0;  // workspace slot of the item's column tile 0
    if (p.ragged) {
        const unsigned unit = fastdiv(item_ct, p.div_hkv);        // (sequence, split) units, KV head innermost
        kvh = (int)(item_ct - unit * (unsigned)p.Hkv);
        const RaggedHalves rh = ragged_halves(p, lane);
        halves_per_split = __builtin_amdgcn_readfirstlane((int)ragged_halves_per_split(p, rh));
        int n_splits;
        if (!ragged_find(rh, (unsigned)halves_per_split, unit, b, split, n_splits)) return;  // beyond the true list
        slot0 = (size_t)item_ct * p.n_coltiles;
        // the sequence's first workgroup tells the merge kernel where its splits are (all lanes
        // store the same two words: a branch on the lane id here would make the compiler treat
        // what follows as lane-dependent, and the copies' base addresses must stay scalar)
        if (split == 0 && kvh == 0 && ctg == 0) {
            p.ws_units[2 * b] = (int)unit;
            p.ws_units[2 * b + 1] = n_splits;
        }
    } else {
        const unsigned upair = fastdiv(item_ct, p.div_splits);    // witem / (n_ctgroups * n_splits)
        split = (int)(item_ct - upair * (unsigned)p.n_splits);
        b = (int)fastdiv(upair, p.div_hkv);
        kvh = (int)upair - b * p.Hkv;
        halves_per_split = p.halves_per_split;
        slot0 = ((size_t)upair * p.n_splits + split) * p.n_coltiles;
    }
    // this workgroup's column tiles and the workspace slots of their partial results
    int ct[kTiles];
    bool tile_valid[kTiles];
    size_t item[kTiles];
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
        ct[j] = ctg * kTiles + j;
        tile_valid[j] = ct[j] < p.n_coltiles;  // (uniform; an odd number of tiles leaves the last workgroup one)
        item[j] = slot0 + min(ct[j], p.n_coltiles - 1);
    }

    const int l32 = lane & 31;
    const int hf = lane >> 5;
    // this sequence's cache length (at least the query rows themselves) and its visited halves
    // (read as constant memory -- nothing writes the lengths while the kernel runs -- so that it is
    // a scalar load whatever the kernel has stored before it)
    typedef const int __attribute__((address_space(4))) *ConstInts;
    const int Nk = p.seq_lens ? max(min(((ConstInts)p.seq_lens)[b], p.Nk), p.Nq) : p.Nk;
    const int W = p.W, S = p.S;
    const VisitedHalves vh = visited_halves(Nk, p.Nq, W, S);

    // this lane's query column in each tile: row c of the pair's G x Nq block (clamped: padding
    // columns repeat the last row and are never stored)
    bool col_valid[kTiles];
    int cc[kTiles], qpos[kTiles];
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
        const int c = ct[j] * 32 + l32;
        col_valid[j] = tile_valid[j] && c < p.cols;
        cc[j] = min(c, p.cols - 1);
        qpos[j] = Nk - p.Nq + (cc[j] % p.Nq);  // its position in the sequence
    }
    const int pos_min = Nk - p.Nq, pos_max = Nk - 1;

    const int h_begin = split * halves_per_split;
    const int n_mine = min(vh.n - h_begin, halves_per_split);
    if (n_mine <= 0) {
        // a shorter sequence has no keys for this split: an empty partial result (weight 0 in the merge)
#pragma unroll
        for (int j = 0; j < kTiles; ++j)
            if (col_valid[j] && hf == 0) {
                p.ws_ml[item[j] * 64 + l32] = -INFINITY;
                p.ws_ml[item[j] * 64 + 32 + l32] = 0.f;
            }
        return;
    }
    auto first_key = [&](int t) {
        const int h = h_begin + t;
        return 32 * (h < vh.n_sink ? h : h - vh.n_sink + vh.band0);
    };

    constexpr bool paged = kPaged;
    const uint32_t k_rsb = (uint32_t)(p.k_sn * 2), v_rsb = (uint32_t)(p.v_sn * 2);  // row strides in bytes
    const char *kg = reinterpret_cast<const char *>(p.k + (paged ? 0 : b * p.k_sb) + (long long)kvh * p.k_sh);
    const char *vg = reinterpret_cast<const char *>(p.v + (paged ? 0 : b * p.v_sb) + (long long)kvh * p.v_sh);
    // (the table is only read while the kernel runs: addressed as constant memory, so that the
    // lookups are scalar loads -- as vector loads they would share the tile copies' counter, and
    // waiting for a table entry would mean waiting for every copy in flight)
    typedef const int __attribute__((address_space(4))) *TablePtr;
    const TablePtr bt = paged ? (TablePtr)(p.block_table + (size_t)b * p.bt_stride) : nullptr;

    // ---- HBM -> LDS copies of one half: instruction i moves rows 4i .. 4i+3, 16 lanes
    // per row; the XOR swizzle of the operand reads is applied on the global side.  Rows
    // past the end of the cache repeat its last row (they are masked later). ----
    const int lrow = lane >> 4, lchk = lane & 15;
    // Paged cache: the block-table entries one half needs -- one if a page holds a multiple of 32
    // tokens, two for a multiple of 16, else none here (looked up per copy instruction).  They
    // are scalar loads with a long way to go, asked for one loop iteration before the copy.
    struct Pages {
        int a, b;
    };
    const int pages_per_half = !paged ? 0 : p.page_size % 32 == 0 ? 1 : p.page_size % 16 == 0 ? 2 : 0;
    auto lookup = [&](int t) __attribute__((always_inline)) {
        Pages pg{0, 0};
        if constexpr (paged) {
            if (pages_per_half != 0) {
                const int k0 = first_key(t);
                pg.a = bt[fastdiv((unsigned)k0, p.div_page)];
                pg.b = pages_per_half == 2 ? bt[fastdiv((unsigned)min(k0 + 16, Nk - 1), p.div_page)] : pg.a;
            }
        }
        return pg;
    };
    auto issue_half = [&](int t, int stage, const Pages pg) __attribute__((always_inline)) {
        const int k0 = first_key(t);
        const uint32_t lds = (uint32_t)(stage * kDStageBytes);
        if constexpr (paged) {
            if (pages_per_half == 0) {
                // page_size is a multiple of 4 only: the four rows of one instruction share a
                // page, so the page number is a uniform (scalar) table lookup per instruction
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int key4 = min(k0 + 4 * i, Nk - 1) & ~3;  // first row of the instruction, inside the cache
                    const unsigned pi = fastdiv((unsigned)key4, p.div_page);
                    const int page = min(max(bt[pi], 0), p.num_pages - 1);  // inside the cache whatever the table says
                    const int in_page = key4 - (int)pi * p.page_size;
                    const char *kb = kg + ((long long)page * p.k_sb + (long long)in_page * p.k_sn) * 2;
                    const char *vb = vg + ((long long)page * p.v_sb + (long long)in_page * p.v_sn) * 2;
                    const int row = min(key4 + lrow, Nk - 1) - key4;
                    const int fk = ((4 * (i & 1) + lrow) << 1) | ((i >> 1) & 1);
                    const uint32_t koff = (uint32_t)row * k_rsb + (uint32_t)((lchk ^ fk) << 4);
                    const uint32_t voff = (uint32_t)row * v_rsb + (uint32_t)((lchk ^ (lrow << 2)) << 4);
                    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(koff), "s"(kb),
                                 "s"(lds + (uint32_t)(i * 1024))
                                 : "memory");
                    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(vb),
                                 "s"(lds + (uint32_t)(kHalfBytes + i * 1024))
                                 : "memory");
                }
                return;
            }
            // page_size a multiple of 16: rows 0..15 of the half lie in one page, rows 16..31 in one
            // (the same one if page_size is a multiple of 32); their numbers came with `pg`.  Row
            // offsets count from the half's first row, so the second base steps back 16 rows; if
            // the cache ends inside the first 16 rows, every later row repeats its last row there.
            // (page strides and row strides of a paged cache fit 32 bits -- the entry point checks --
            // so each product is one 32 x 32 -> 64 bit multiplication, not the 64 x 64 bit one that
            // costs six: this arithmetic sits in front of every copy of the wave's only instruction stream)
            auto base_of = [](const char *g, long long sb, long long sn, int page, int row) __attribute__((always_inline)) {
                const long long elems = (long long)((unsigned long long)(unsigned)page * (unsigned)sb) + (long long)row * (int)sn;
                return g + 2 * elems;
            };
            const int in_a = k0 - (int)fastdiv((unsigned)k0, p.div_page) * p.page_size;
            const int page_a = min(max(pg.a, 0), p.num_pages - 1);
            const char *kb[2], *vb[2];
            kb[0] = kb[1] = base_of(kg, p.k_sb, p.k_sn, page_a, in_a);
            vb[0] = vb[1] = base_of(vg, p.v_sb, p.v_sn, page_a, in_a);
            if (pages_per_half == 2 && k0 + 16 <= Nk - 1) {
                const int in_b = k0 + 16 - (int)fastdiv((unsigned)(k0 + 16), p.div_page) * p.page_size;
                const int page_b = min(max(pg.b, 0), p.num_pages - 1);
                kb[1] = base_of(kg, p.k_sb, p.k_sn, page_b, in_b - 16);
                vb[1] = base_of(vg, p.v_sb, p.v_sn, page_b, in_b - 16);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = min(4 * i + lrow, Nk - 1 - k0);
                const int fk = ((4 * (i & 1) + lrow) << 1) | ((i >> 1) & 1);
                const uint32_t off = (uint32_t)row * k_rsb + (uint32_t)((lchk ^ fk) << 4);
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(kb[i / 4]),
                             "s"(lds + (uint32_t)(i * 1024))
                             : "memory");
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = min(4 * i + lrow, Nk - 1 - k0);
                const uint32_t off = (uint32_t)row * v_rsb + (uint32_t)((lchk ^ (lrow << 2)) << 4);
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(vb[i / 4]),
                             "s"(lds + (uint32_t)(kHalfBytes + i * 1024))
                             : "memory");
            }
            return;
        }
        const char *kb = kg + (size_t)k0 * k_rsb;  // uniform
        const char *vb = vg + (size_t)k0 * v_rsb;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = min(4 * i + lrow, Nk - 1 - k0);
            const int fk = ((4 * (i & 1) + lrow) << 1) | ((i >> 1) & 1);
            const uint32_t off = (uint32_t)row * k_rsb + (uint32_t)((lchk ^ fk) << 4);
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(kb),
                         "s"(lds + (uint32_t)(i * 1024))
                         : "memory");
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = min(4 * i + lrow, Nk - 1 - k0);
            const uint32_t off = (uint32_t)row * v_rsb + (uint32_t)((lchk ^ (lrow << 2)) << 4);
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(vb),
                         "s"(lds + (uint32_t)(kHalfBytes + i * 1024))
                         : "memory");
        }
    };
    const LaneAddr la = make_lane_addr(lane, 0);

    // ---- start-up: this lane's Q fragments (B operand of S^T = K Q^T: query row l32, 16 bytes at
    // 32 ks + 16 hf) straight from HBM with ordinary loads, then the first three halves into the
    // three stages.  The compiler places the wait for the Q loads in front of their first use,
    // and that wait covers the copies issued behind them as well (it cannot see them): a short
    // item has all its keys in flight at once and starts when they are there; a long one gives
    // away the head start of its first two steps, once. ----
    bf16x8 qf[kTiles][kKS];
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
        const char *qrow = reinterpret_cast<const char *>(p.q + ((size_t)b * p.Hq + (size_t)kvh * p.G) * p.Nq * kD) +
                           (size_t)cc[j] * kRowBytes + 16 * hf;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) qf[j][ks] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * ks);
    }
    issue_half(0, 0, lookup(0));
    if (n_mine >= 2) issue_half(1, 1, lookup(1));
    if (kDStages >= 3 && n_mine >= 3) issue_half(2, 2, lookup(2));
    // (the idle cycles keep the loads two wait states away from the first MFMA that reads them)
#pragma unroll
    for (int j = 0; j < kTiles; ++j)
        asm volatile("s_nop 1"
                     : "+a"(qf[j][0]), "+a"(qf[j][1]), "+a"(qf[j][2]), "+a"(qf[j][3]), "+a"(qf[j][4]), "+a"(qf[j][5]),
                       "+a"(qf[j][6]), "+a"(qf[j][7]));
    Pages pg_next = n_mine > kDStages ? lookup(kDStages) : Pages{0, 0};  // of the half the loop's first iteration issues

    f32x16 oacc[kTiles][kDB];
    RowState rs[kTiles];
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
#pragma unroll
        for (int db = 0; db < kDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[j][db][e] = 0.f;
        pin_acc(oacc[j]);
        rs[j].mc = -INFINITY;
        rs[j].l = 0.f;
        rs[j].lb = 0.f;
    }
    const float c2 = p.scale_log2;

    int stage = 0;
    for (int t = 0; t < n_mine; ++t) {
        // half t has landed when at most the copies of the halves issued after it are outstanding
        const int later = min(n_mine - 1 - t, kDStages - 1);
        if (later >= 2)
            asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
        else if (later == 1)
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        static_assert(kDStages <= 3 && kCopiesPerHalf == 16, "wait counts above");

        const uint32_t so = (uint32_t)(stage * kDStageBytes);
        const int k0h = first_key(t);
        // no mask when every key of the half is visible to every column: at or below the
        // oldest row's diagonal, and inside the newest row's window or all sinks
        const bool masked = !((k0h + 31 <= pos_min) && ((k0h > pos_max - W) || (k0h + 31 < S)));

        // all operand fragments of the half go to registers first; once they are there the
        // stage is free and the copy of the half three ahead leaves before any arithmetic
        bf16x8 kf[kKS], vf[2][kDB];
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) kf[ks] = load_k_frag(la, so, ks);
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < kDB; ++db) vf[st][db] = load_v_frag(la, so + kHalfBytes, st, db);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (t + kDStages < n_mine) issue_half(t + kDStages, stage, pg_next);
        if (t + kDStages + 1 < n_mine) pg_next = lookup(t + kDStages + 1);  // lands under this iteration's arithmetic

#pragma unroll
        for (int j = 0; j < kTiles; ++j) {
            if (j > 0 && !tile_valid[j]) continue;  // (uniform)
            f32x16 s;
            bf16x8 pf[2];
            float alpha;
            mfma_s_first<kF16>(s, kf[0], qf[j][0]);
#pragma unroll
            for (int ks = 1; ks < kKS - 1; ++ks) mfma_s<kF16>(s, kf[ks], qf[j][ks]);
            mfma_s_settled<kF16>(s, kf[kKS - 1], qf[j][kKS - 1]);
            if (masked)
                softmax_half<true, kF16>(s, k0h, qpos[j], W, S, hf, c2, rs[j], pf, alpha);
            else
                softmax_half<false, kF16>(s, k0h, qpos[j], W, S, hf, c2, rs[j], pf, alpha);
            rescale(oacc[j], alpha);
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int db = 0; db < kDB; ++db) {
                    if (st == 1 && db == kDB - 1)
                        mfma_acc_settled<kF16>(oacc[j][db], vf[st][db], pf[st]);  // the accumulators are read below / next time round
                    else
                        mfma_acc<kF16>(oacc[j][db], vf[st][db], pf[st]);
                }
        }
        stage = (stage + 1 == kDStages) ? 0 : stage + 1;
    }

    // ---- partial result of the valid columns: O^T accumulators (row d, column l32), reference, sum ----
    // The merge divides by the fp32 sums it combines; a partial O is the sum over the
    // rounded P, so it is stored scaled by l / (sum of the rounded P).
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
        float l_row, lb_row;
        row_sums(rs[j], l_row, lb_row);
        const float fix = lb_row > 0.f ? l_row / lb_row : 0.f;  // a column that saw no key: O = 0, l = 0
        if (col_valid[j]) {
            float *wo = p.ws_o + (item[j] * p.col_stride + l32) * kD;
#pragma unroll
            for (int db = 0; db < kDB; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    float4 o4;
                    o4.x = oacc[j][db][4 * e4 + 0] * fix;
                    o4.y = oacc[j][db][4 * e4 + 1] * fix;
                    o4.z = oacc[j][db][4 * e4 + 2] * fix;
                    o4.w = oacc[j][db][4 * e4 + 3] * fix;
                    *reinterpret_cast<float4 *>(wo + 32 * db + 8 * e4 + 4 * hf) = o4;
                }
            if (hf == 0) {
                p.ws_ml[item[j] * 64 + l32] = rs[j].mc;
                p.ws_ml[item[j] * 64 + 32 + l32] = l_row;
            }
        }
    }
}

// ---- merging the splits: out = sum_s 2^(mc_s - m) O_s / sum_s 2^(mc_s - m) l_s with m = max_s mc_s;
// lse = (m + log2 of the denominator) ln 2 ----
// One output row (b, hq, r) and where its partial results are: n_splits items, `step` workspace
// slots apart (times the column tiles), the first at slot0.
struct MergeRow {
    long long row;
    int ct, col;
    int n_splits;
    long long slot0, step;
};
__device__ __forceinline__ MergeRow merge_row(const DecodeParams &p, long long row) {
    MergeRow m;
    m.row = row;
    const int r = (int)(row % p.Nq);
    const int hq = (int)((row / p.Nq) % p.Hq);
    const int b = (int)(row / ((long long)p.Nq * p.Hq));
    const int kvh = hq / p.G;
    const int c = (hq % p.G) * p.Nq + r;
    m.ct = c / 32;
    m.col = c % 32;
    if (p.ragged) {  // (the device-side plan: the sequence's first split workgroup has left it here)
        m.n_splits = p.ws_units[2 * b + 1];
        m.slot0 = (long long)p.ws_units[2 * b] * p.Hkv + kvh;
        m.step = p.Hkv;
    } else {
        m.n_splits = p.n_splits;
        m.slot0 = ((long long)b * p.Hkv + kvh) * p.n_splits;
        m.step = 1;
    }
    return m;
}
__device__ __forceinline__ void merge_store(const DecodeParams &p, long long row, int d, float o, float l, float m) {
    if (p.fp16)
        reinterpret_cast<_Float16 *>(p.out)[(size_t)row * kD + d] = (_Float16)(o / l);
    else
        p.out[(size_t)row * kD + d] = (__bf16)(o / l);
    if (d == 0) p.lse[row] = (m + __builtin_amdgcn_logf(l)) * 0.69314718055994530942f;
}

// A whole workgroup of kMergeThreads on one row (many splits): red and lsum are its LDS.
__device__ __forceinline__ void merge_row_by_workgroup(const DecodeParams &p, const MergeRow &mr, float *red, float *lsum) {
    const int tid = threadIdx.x;
    const int n_splits = mr.n_splits, col = mr.col;
    auto item_of = [&](int s) { return (mr.slot0 + s * mr.step) * p.n_coltiles + mr.ct; };

    // largest reference over the splits: wave maxima by lane exchange, then one LDS round
    float m = -INFINITY;
    for (int s = tid; s < n_splits; s += kMergeThreads) m = fmaxf(m, p.ws_ml[item_of(s) * 64 + col]);
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) m = fmaxf(m, __shfl_xor(m, sh));
    if ((tid & 63) == 0) red[tid >> 6] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kMergeThreads / 64; ++w) m = fmaxf(m, red[w]);  // finite: every row sees at least its own key
    __syncthreads();

    // Four splits per round, their loads issued together.  A split that saw no visible
    // key has reference -inf and may not have written its O: it is loaded all the same
    // (the workspace is there) and left out of the sums by selection, not by a branch.
    const int d = tid % kD, g = tid / kD;
    constexpr int kGroups = kMergeThreads / kD;
    float acc = 0.f, l = 0.f;
    for (int s0 = g; s0 < n_splits; s0 += 4 * kGroups) {
        float mcs[4], ls[4], os[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u * kGroups;
            const bool there = s < n_splits;
            const long long it = item_of(there ? s : s0);
            mcs[u] = p.ws_ml[it * 64 + col];
            ls[u] = p.ws_ml[it * 64 + 32 + col];
            os[u] = p.ws_o[(it * p.col_stride + col) * kD + d];
            if (!there) mcs[u] = -INFINITY;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool empty = mcs[u] == -INFINITY;
            const float w = __builtin_amdgcn_exp2f(mcs[u] - m);
            l += empty ? 0.f : w * ls[u];
            acc += empty ? 0.f : w * os[u];
        }
    }
    red[tid] = acc;
    if (d == 0) lsum[g] = l;
    __syncthreads();
    if (g == 0) {
        float o = 0.f, lt = 0.f;
#pragma unroll
        for (int gg = 0; gg < kMergeThreads / kD; ++gg) {
            o += red[gg * kD + d];
            lt += lsum[gg];
        }
        merge_store(p, mr.row, d, o, lt, m);
    }
}

// 128 threads (one per head dimension element) on one row of at most kMergeRowSplits splits: every
// thread adds up the row's splits by itself -- no exchange between threads.
constexpr int kMergeRowSplits = 8;
__device__ __forceinline__ void merge_row_by_group(const DecodeParams &p, const MergeRow &mr, int d) {
    const long long item0 = mr.slot0 * p.n_coltiles + mr.ct, item_step = mr.step * p.n_coltiles;
    float mcs[kMergeRowSplits], ls[kMergeRowSplits], os[kMergeRowSplits];
    // (a split that saw no visible key has reference -inf and may not have written its O: loaded all
    // the same and left out by selection; splits beyond the row's repeat split 0 and count as empty)
#pragma unroll
    for (int s = 0; s < kMergeRowSplits; ++s) {
        const bool there = s < mr.n_splits;
        const long long it = item0 + (there ? s : 0) * item_step;
        mcs[s] = p.ws_ml[it * 64 + mr.col];
        ls[s] = p.ws_ml[it * 64 + 32 + mr.col];
        os[s] = p.ws_o[(it * p.col_stride + mr.col) * kD + d];
        if (!there) mcs[s] = -INFINITY;
    }
    float m = mcs[0];
#pragma unroll
    for (int s = 1; s < kMergeRowSplits; ++s) m = fmaxf(m, mcs[s]);  // finite: every row sees at least its own key
    float acc = 0.f, l = 0.f;
#pragma unroll
    for (int s = 0; s < kMergeRowSplits; ++s) {
        const bool empty = mcs[s] == -INFINITY;
        const float w = __builtin_amdgcn_exp2f(mcs[s] - m);
        l += empty ? 0.f : w * ls[s];
        acc += empty ? 0.f : w * os[s];
    }
    merge_store(p, mr.row, d, acc, l, m);
}

// Sequences of one length, more than kMergeRowSplits splits per pair: one workgroup per output row.
__global__ __launch_bounds__(kMergeThreads) void swaa_decode_merge_kernel(const DecodeParams p) {
    __shared__ float red[kMergeThreads];
    __shared__ float lsum[kMergeThreads / kD];
    merge_row_by_workgroup(p, merge_row(p, blockIdx.x), red, lsum);
}

// Sequences of one length, at most kMergeRowSplits splits per pair: kMergeThreads / 128 output rows
// per workgroup.  A batch of many sequences has thousands of rows of two or three splits each;
// one workgroup of 1024 threads per row spent most of the merge waiting for workgroup slots (64
// sequences x 8 new tokens: the call took 275 us, 70 of them here).
__global__ __launch_bounds__(kMergeThreads) void swaa_decode_merge_rows_kernel(const DecodeParams p) {
    const long long row = (long long)blockIdx.x * (kMergeThreads / kD) + threadIdx.x / kD;
    if (row >= (long long)p.B * p.Hq * p.Nq) return;
    merge_row_by_group(p, merge_row(p, row), threadIdx.x % kD);
}

// Per-sequence lengths: both at once.  The first n_small workgroups take kMergeThreads / 128 rows
// each and merge those of at most kMergeRowSplits splits, 128 threads per row.  The rows of the
// sequences with more splits -- there are at most (units_target + B) / (kMergeRowSplits + 1) such
// sequences -- are left to the workgroups behind them, one row each: workgroup n_small + k looks
// for the (k / (Hq Nq))-th such sequence in the plan the split kernel has left (a prefix sum of
// flags over the lanes, every wave for itself) and goes home if there is none.
__global__ __launch_bounds__(kMergeThreads) void swaa_decode_merge_ragged_kernel(const DecodeParams p, unsigned n_small) {
    __shared__ float red[kMergeThreads];
    __shared__ float lsum[kMergeThreads / kD];
    if (blockIdx.x < n_small) {
        const long long row = (long long)blockIdx.x * (kMergeThreads / kD) + threadIdx.x / kD;
        if (row >= (long long)p.B * p.Hq * p.Nq) return;
        const MergeRow mr = merge_row(p, row);
        if (mr.n_splits <= kMergeRowSplits) merge_row_by_group(p, mr, threadIdx.x % kD);
        return;
    }
    const unsigned k = blockIdx.x - n_small, rows_per_seq = (unsigned)(p.Hq * p.Nq);
    const unsigned want = k / rows_per_seq;  // the want-th sequence with many splits (from 0)
    const int lane = threadIdx.x & 63;
    unsigned before = 0;
    int b = -1;
    for (int c0 = 0; c0 < p.B; c0 += 64) {
        const bool many = c0 + lane < p.B && p.ws_units[2 * (c0 + lane) + 1] > kMergeRowSplits;
        const unsigned incl = wave_inclusive_scan(many ? 1u : 0u);
        const unsigned in_round = wave_read_lane(incl, 63);
        if (want - before < in_round) {
            b = c0 + __popcll(__ballot(incl <= want - before));
            break;
        }
        before += in_round;
    }
    if (b < 0) return;  // (the same in every wave of the workgroup)
    merge_row_by_workgroup(p, merge_row(p, (long long)b * rows_per_seq + (k - want * rows_per_seq)), red, lsum);
}

}  // namespace

void plan_decode(DecodeParams &p, bool ragged) {
    p.cols = p.G * p.Nq;
    p.n_coltiles = (p.cols + 31) / 32;
    p.col_stride = p.cols < 32 ? p.cols : 32;
    // an upper bound on the halves any sequence of at most Nk tokens visits (a shorter sequence's
    // band can straddle one half more than the longest one's): the splits are planned for it
    const int all = (p.Nk + 31) / 32;
    const int bound = (p.S + 31) / 32 + (p.W + p.Nq - 2) / 32 + 2;
    p.n_halves = all < bound ? all : bound;
    // kRounds rounds of three workgroups per CU (one round measured fastest: every split is
    // resident at once and streams for the whole launch), but no split shorter than four halves
    p.tiles_per_item = p.n_coltiles >= 2 ? 2 : 1;
    p.n_ctgroups = (p.n_coltiles + p.tiles_per_item - 1) / p.tiles_per_item;
    const long long groups = (long long)p.B * p.Hkv * p.n_ctgroups;
    p.div_ctgroups = make_fastdiv((unsigned)p.n_ctgroups);
    p.div_per_round = make_fastdiv((unsigned)(kXcds * p.n_ctgroups));
    p.div_hkv = make_fastdiv((unsigned)p.Hkv);
    p.ragged = ragged && p.B >= 2 && p.B <= kRaggedMaxBatch && (long long)p.B * p.n_halves < 0x7fffffffLL ? 1 : 0;
    if (p.ragged) {
        // Per-sequence lengths: kRaggedRounds rounds of resident workgroups' worth of (sequence,
        // split) units, cut on the device in proportion to the sequences' lengths; kTailRounds
        // with more (pair, column tile) groups than resident workgroups (see below).
        constexpr long long kRaggedRounds = 2, kRaggedTailRounds = 8;
        const long long resident = 256LL * decode_wgs_per_cu(p.tiles_per_item);
        const long long units = resident * (groups > resident ? kRaggedTailRounds : kRaggedRounds) / ((long long)p.Hkv * p.n_ctgroups);
        p.units_target = (int)(units < 1 ? 1 : units);
        // (at most units_target + B units by the rounding of the device's division, and no
        // sequence has more than ceil(n_halves / 4) splits)
        const long long most = (long long)p.B * ((p.n_halves + 3) / 4);
        p.max_units = (int)(p.units_target + p.B < most ? p.units_target + p.B : most);
        p.halves_per_split = p.n_splits = 0;
        p.div_splits = make_fastdiv(1u);
        p.wg_items = (long long)p.max_units * p.Hkv * p.n_ctgroups;
        p.items = (long long)p.max_units * p.Hkv * p.n_coltiles;
        return;
    }
    const long long target_items = 256LL * decode_wgs_per_cu(p.tiles_per_item) * kRounds;
    long long per_group = target_items / groups;
    // More (pair, column tile) groups than resident workgroups: one item per group would leave a
    // second round of a few long items streaming alone at the end (100 sequences x 8 KV heads
    // took 1.5 x the time of 96).  Many short items instead, kTailRounds rounds' worth: the
    // partly filled tail is then one short item long.
    constexpr long long kTailRounds = 8;
    if (per_group < 1) per_group = (kTailRounds * target_items + groups - 1) / groups;
    long long hps = (p.n_halves + per_group - 1) / per_group;
    if (hps < 4) hps = 4;
    p.halves_per_split = (int)hps;
    p.n_splits = (int)((p.n_halves + hps - 1) / hps);
    p.wg_items = groups * p.n_splits;
    p.items = (long long)p.B * p.Hkv * p.n_coltiles * p.n_splits;
    p.div_splits = make_fastdiv((unsigned)p.n_splits);
}

long long decode_workspace_floats(const DecodeParams &p) {
    // (per item O and 64 floats of references and row sums; ragged: two ints per sequence on top, rounded to 16 bytes)
    return p.items * ((long long)p.col_stride * kD + 64) + (p.ragged ? (2LL * p.B + 3) / 4 * 4 : 0);
}

// ---- scratch memory for callers that cannot allocate -----------------------------------
// swaa_attn_decode_static keeps the partial results of the key splits here instead of in
// a caller's workspace.  In host code the array's name is only a stand-in for the device
// object: its device address comes from hipGetSymbolAddress, asked once per device with
// that device current (every GPU the library runs on holds its own copy of the array at
// its own address until the process ends), and host code passes that address, never the
// name, to kernels.
static __device__ __align__(256) unsigned char scratch[kDecodeStaticScratchBytes];

hipError_t decode_static_scratch(void **ptr) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> address[kMaxDevices];  // zero-initialised
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *a = address[dev].load(std::memory_order_acquire);
    if (!a) {
        err = hipGetSymbolAddress(&a, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!a) return hipErrorInvalidSymbol;
        address[dev].store(a, std::memory_order_release);  // (two threads racing here store the same value)
    }
    *ptr = a;
    return hipSuccess;
}

hipError_t launch_decode(const DecodeParams &p, hipStream_t stream) {
    // (a whole number of rounds of 8 x column-tile groups covers both item orders)
    const long long per_round = (long long)kXcds * p.n_ctgroups;
    const long long chunk = (p.wg_items + kXcds - 1) / kXcds;
    const long long wgs = p.ragged ? (p.wg_items + per_round - 1) / per_round * per_round : chunk * kXcds;
    const dim3 grid((unsigned)wgs);
    const bool paged = p.block_table != nullptr;
    auto launch = [&](auto f16, auto pg, auto tiles) {
        hipLaunchKernelGGL((swaa_decode_split_kernel<decltype(f16)::value, decltype(pg)::value, decltype(tiles)::value>), grid,
                           dim3(64), decode_stages(decltype(tiles)::value) * kDStageBytes, stream, p);
    };
    auto pick_tiles = [&](auto f16, auto pg) {
        if (p.tiles_per_item == 2)
            launch(f16, pg, std::integral_constant<int, 2>{});
        else
            launch(f16, pg, std::integral_constant<int, 1>{});
    };
    if (p.fp16 && paged)
        pick_tiles(std::true_type{}, std::true_type{});
    else if (p.fp16)
        pick_tiles(std::true_type{}, std::false_type{});
    else if (paged)
        pick_tiles(std::false_type{}, std::true_type{});
    else
        pick_tiles(std::false_type{}, std::false_type{});
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const long long rows = (long long)p.B * p.Hq * p.Nq;
    constexpr int kRowsPerWg = kMergeThreads / kD;
    const unsigned n_small = (unsigned)((rows + kRowsPerWg - 1) / kRowsPerWg);
    if (p.ragged) {
        long long many = ((long long)p.units_target + p.B) / (kMergeRowSplits + 1);  // sequences that can have more splits
        many = many < p.B ? many : p.B;
        if (n_small + many * p.Hq * p.Nq > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(swaa_decode_merge_ragged_kernel, dim3(n_small + (unsigned)(many * p.Hq * p.Nq)), dim3(kMergeThreads),
                           0, stream, p, n_small);
    } else if (p.n_splits <= kMergeRowSplits) {
        hipLaunchKernelGGL(swaa_decode_merge_rows_kernel, dim3(n_small), dim3(kMergeThreads), 0, stream, p);
    } else {
        hipLaunchKernelGGL(swaa_decode_merge_kernel, dim3((unsigned)rows), dim3(kMergeThreads), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace swaa
