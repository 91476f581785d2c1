// Types, the kernel parameter block and the work decomposition shared by the
// attention-forward kernels of libswaa (gfx950 only).
#ifndef SWAA_COMMON_H_
#define SWAA_COMMON_H_

#include <hip/hip_runtime.h>

#include <cstdint>

namespace swaa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBk = 64;        // keys per KV tile
constexpr int kThreads = 256;  // plain kernels: 4 waves per workgroup ...
constexpr int kWaveRows = 64;  // ... of 64 query rows each (the pipelined kernel: 8 waves of 32)
constexpr int kWgRows = 256;   // query rows (head x position) per workgroup of the plain and backward kernels
constexpr int kXcds = 8;       // accelerator dies; workgroups are dealt to them round-robin

// Division of a number below 2^31 by a divisor fixed at launch, as a multiplication: with
// l = ceil(log2 d) and m = ceil(2^(31 + l) / d) (which fits 32 bits), n / d = (n * m) >> (31 + l)
// exactly: m d - 2^(31 + l) < d <= 2^l, so the product overshoots n / d by less than 1 / d.
// Every wave of every workgroup decodes its work item with three such divisions; done the long
// way they are about a hundred instructions in front of the first memory request.
struct FastDiv {
    unsigned m;
    int sh;  // negative: the divisor is 1
};
inline FastDiv make_fastdiv(unsigned d) {
    FastDiv f{0u, -1};
    if (d <= 1) return f;
    int l = 0;
    while ((1ull << l) < d) ++l;
    f.m = (unsigned)(((1ull << (31 + l)) + d - 1) / d);
    f.sh = l - 1;
    return f;
}
__host__ __device__ __forceinline__ unsigned fastdiv(unsigned n, const FastDiv f) {
    return f.sh < 0 ? n : (unsigned)(((unsigned long long)n * f.m) >> 32) >> f.sh;  // (the upper half of one 32 x 32 bit product)
}

struct FwdParams {
    const __bf16 *q;
    const __bf16 *k;
    const __bf16 *v;
    __bf16 *out;
    float *lse;
    // element strides of batch entry, head and row; the head dimension is contiguous
    long long q_sb, q_sh, q_sn;
    long long k_sb, k_sh, k_sn;
    long long v_sb, v_sh, v_sn;
    long long o_sb, o_sh, o_sn;
    long long lse_sb, lse_sh;  // rows contiguous
    // packed variable-length batches: device arrays of B + 1 row offsets along the row
    // axis (sequence b owns rows [cu[b], cu[b+1])), batch strides unused; or null
    const int *cu_q;
    const int *cu_k;
    // per-sequence prompt lengths (device, B ints) in place of P below, or null
    const int *n_prompts;
    // paged key/value cache (pipelined kernel only), or block_table null: token j of sequence b
    // lives in page block_table[b * bt_stride + j / page_size], row j % page_size; k, v then point
    // at page 0 and k_sb, v_sb are the page strides.  page_size is a multiple of 16.
    const int *block_table;
    int bt_stride, page_size, num_pages;
    int fp16;  // the 16-bit elements of q, k, v, out are IEEE binary16 instead of bfloat16 (plain kernel only)
    int B, Hq, Hkv;
    int Nq, Nk;  // query rows and keys per sequence (the largest ones when cu_q / cu_k are given)
    int W, S;    // clamped to [1, Nk] and [0, Nk]
    int P;       // rows at positions >= P are generated tokens and see every earlier key; clamped to [0, Nk]
    int G;       // Hq / Hkv
    float scale, scale_log2;
    // Work decomposition.  Per (batch, KV head) "pair" the G query heads are
    // cut into n4 groups of 4 heads, at most one group of 2 heads and at most
    // one single head; a workgroup is wg_rows query rows (head x position) on one
    // KV head: 4 heads x wg_rows/4 positions, 2 x wg_rows/2 or 1 x wg_rows.
    int wg_rows;  // 128 (forward kernels) or 256 (backward kernels)
    int n4, has2, has1;
    int nt_h4, nt_h2, nt_h1;  // row tiles of a sequence of Nq rows for workgroups of 4, 2 and 1 heads
    FastDiv div_tiles_per_pair, div_hkv, div_nt_h4;  // for the work-list decode of every workgroup
    int tiles_per_pair;
    long long total_items;
    long long chunk;  // work items per XCD
    // Packed batches whose total number of query rows the caller has stated: the work list holds
    // every sequence's own row tiles, one sequence after the other (no items for rows a shorter
    // sequence does not have); total_items and chunk are then upper bounds, the workgroups work
    // out the true ones from cu_q / cu_k (decode_work_packed).
    int packed_compact;
};

// One sequence as a workgroup sees it: the query rows are the newest nq of its nk
// tokens (row r sits at position nk - nq + r; nq = nk for a plain prefill).
struct SeqGeom {
    int nq, nk;
    int n_prompt;  // rows at positions >= n_prompt are generated tokens
    long long q_row0, k_row0;  // first row along the row axis of q / out / lse and of k / v
    long long q_batch, k_batch;  // batch index to multiply the batch strides with
};
__device__ __forceinline__ bool seq_geom(const FwdParams &p, int b, SeqGeom &g) {
    if (p.cu_q) {
        g.q_row0 = p.cu_q[b];
        g.nq = p.cu_q[b + 1] - (int)g.q_row0;
        g.q_batch = 0;
    } else {
        g.q_row0 = 0;
        g.nq = p.Nq;
        g.q_batch = b;
    }
    if (p.cu_k) {
        g.k_row0 = p.cu_k[b];
        g.nk = p.cu_k[b + 1] - (int)g.k_row0;
        g.k_batch = 0;
        if (p.block_table) g.k_row0 = 0;  // a paged cache: the offsets only give the lengths
    } else if (p.block_table) {
        g.k_row0 = 0;
        g.nk = p.Nk;
        g.k_batch = 0;
    } else {
        g.k_row0 = 0;
        g.nk = p.Nk;
        g.k_batch = b;
    }
    g.n_prompt = p.n_prompts ? max(p.n_prompts[b], 0) : p.P;
    g.nq = min(min(g.nq, p.Nq), g.nk);  // never more rows than the plan covers, nor than tokens
    g.nk = min(g.nk, p.Nk);
    return g.nq > 0;
}

// What one workgroup computes.
struct WorkItem {
    int b, kvh;  // batch entry, KV head
    int hpb;     // query heads in this workgroup: 4, 2 or 1
    int h0;      // first of them, relative to the GQA group
    int pt;      // row tile of 256/hpb rows
};

// Inclusive prefix sum of x over the 64 lanes of a wave, all of them active: four shift-and-add
// steps inside each row of 16 lanes (a lane without a source adds 0), then lane 15 of rows 0 and 2
// into rows 1 and 3, then lane 31 into rows 2 and 3 -- data-parallel-primitive operands of the
// vector adds, no trip through the LDS crossbar as with the shuffle functions.
__device__ __forceinline__ unsigned wave_inclusive_scan(unsigned x) {
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);  // row_shr:1
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);  // row_shr:2
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);  // row_shr:4
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);  // row_shr:8
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);  // row_bcast:15, rows 1 and 3
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);  // row_bcast:31, rows 2 and 3
    return x;
}
// Lane `src` (the same in all lanes) of x, as a uniform value.
__device__ __forceinline__ unsigned wave_read_lane(unsigned x, int src) {
    return (unsigned)__builtin_amdgcn_readlane((int)x, src);
}

// The work list of a packed batch, sequence by sequence: sequence b of nq_b query rows (the
// smaller of its rows, the plan's Nq and its keys -- what seq_geom makes of it) has Hkv pairs of
// n4 ceil(nq_b / r4) + has2 ceil(nq_b / r2) + has1 ceil(nq_b / r1) row tiles, r4 = wg_rows / 4
// and so on.  EVERY sequence's items are cut into eight contiguous chunks, one per XCD (XCD x
// works through chunk x of sequence 0, then chunk x of sequence 1, ...): the sequences' caches
// differ in length, so a chunk of the whole list would leave the long ones to one or two dies.
// Every wave reads the sequence lengths (64 per round, one per lane) and finds the sequence
// that holds its slot by a prefix sum of the chunk lengths over the lanes.
__device__ __forceinline__ bool decode_work_packed(const FwdParams &p, WorkItem &w) {
    const int lane = threadIdx.x & 63;
    const unsigned bid = blockIdx.x;
    const unsigned xcd = bid % kXcds, slot = bid / kXcds;
    const int s1 = p.wg_rows == 128 ? 7 : 8;  // log2 of the rows of a one-head tile (two heads: half, four: a quarter)
    auto rows_of = [&](int b) {  // nq_b of sequence b (0 for b >= B)
        if (b >= p.B) return 0;
        const int nq = p.cu_q[b + 1] - p.cu_q[b];
        const int nk = p.cu_k[b + 1] - p.cu_k[b];
        return max(0, min(min(nq, p.Nq), min(nk, p.Nk)));
    };
    auto tiles_of = [&](int nq) {  // row tiles of one pair
        return (unsigned)(p.n4 * ((nq + (1 << (s1 - 2)) - 1) >> (s1 - 2)) + p.has2 * ((nq + (1 << (s1 - 1)) - 1) >> (s1 - 1)) +
                          p.has1 * ((nq + (1 << s1) - 1) >> s1));
    };
    unsigned before = 0;
    for (int c0 = 0; c0 < p.B; c0 += 64) {
        const int nq = rows_of(c0 + lane);
        const unsigned incl = wave_inclusive_scan((tiles_of(nq) * (unsigned)p.Hkv + kXcds - 1) / kXcds);  // slots of this XCD up to and with the lane's sequence
        const unsigned in_round = wave_read_lane(incl, 63);
        if (slot - before < in_round) {
            const unsigned rel = slot - before;
            const int n = __popcll(__ballot(incl <= rel));  // sequences among these 64 that end at or before the slot
            const unsigned base = n ? wave_read_lane(incl, n - 1) : 0u;
            // (everything below is the same in all lanes, and read from one lane so that the
            // compiler knows it and keeps addresses built from it in scalar registers)
            const int nq_u = (int)wave_read_lane((unsigned)nq, n);
            const unsigned tpp_u = tiles_of(nq_u);
            const unsigned items_u = tpp_u * (unsigned)p.Hkv;
            unsigned r = xcd * ((items_u + kXcds - 1) / kXcds) + (rel - base);  // inside sequence c0 + n
            if (r >= items_u) return false;  // (the sequence's last chunks are shorter)
            w.b = c0 + n;
            w.kvh = (int)(r / tpp_u);
            r -= (unsigned)w.kvh * tpp_u;
            const unsigned nt4 = (unsigned)((nq_u + (1 << (s1 - 2)) - 1) >> (s1 - 2));
            const unsigned nt2 = (unsigned)((nq_u + (1 << (s1 - 1)) - 1) >> (s1 - 1));
            const unsigned nt1 = (unsigned)((nq_u + (1 << s1) - 1) >> s1);
            if (r < (unsigned)p.n4 * nt4) {
                const unsigned g = r / nt4;
                w.hpb = 4;
                w.h0 = 4 * (int)g;
                w.pt = (int)(nt4 - 1 - (r - g * nt4));
                return true;
            }
            r -= (unsigned)p.n4 * nt4;
            if (p.has2 && r < nt2) {
                w.hpb = 2;
                w.h0 = 4 * p.n4;
                w.pt = (int)(nt2 - 1 - r);
                return true;
            }
            if (p.has2) r -= nt2;
            w.hpb = 1;
            w.h0 = p.G - 1;
            w.pt = (int)(nt1 - 1 - r);
            return true;
        }
        before += in_round;
    }
    return false;
}

// Workgroups reach the 8 XCDs round-robin; XCD x takes the x-th contiguous
// chunk of the work list, so the position tiles of one KV head, whose K/V
// bands overlap, run behind the same L2.  Inside a pair, long rows go first.
__device__ __forceinline__ bool decode_work(const FwdParams &p, WorkItem &w) {
    if (p.packed_compact) return decode_work_packed(p, w);
    // (the entry points refuse work lists of 2^31 items or more: 32-bit arithmetic, whose
    // divisions cost a fraction of the 64-bit ones -- every wave of every workgroup pays them)
    const unsigned bid = blockIdx.x;
    const unsigned slot = bid / kXcds, chunk = (unsigned)p.chunk;
    const unsigned item = (bid % kXcds) * chunk + slot;
    if (slot >= chunk || item >= (unsigned)p.total_items) return false;
    const unsigned tpp = (unsigned)p.tiles_per_pair, hkv = (unsigned)p.Hkv;
    const unsigned pair = fastdiv(item, p.div_tiles_per_pair);
    unsigned r = item - pair * tpp;
    w.b = (int)fastdiv(pair, p.div_hkv);
    w.kvh = (int)(pair - (unsigned)w.b * hkv);
    const unsigned nt4 = (unsigned)p.nt_h4, nt2 = (unsigned)p.nt_h2;
    if (r < (unsigned)p.n4 * nt4) {
        const unsigned g = fastdiv(r, p.div_nt_h4);
        w.hpb = 4;
        w.h0 = 4 * (int)g;
        w.pt = (int)(nt4 - 1 - (r - g * nt4));
        return true;
    }
    r -= (unsigned)p.n4 * nt4;
    if (p.has2 && r < nt2) {
        w.hpb = 2;
        w.h0 = 4 * p.n4;
        w.pt = (int)(nt2 - 1 - r);
        return true;
    }
    if (p.has2) r -= nt2;
    w.hpb = 1;
    w.h0 = p.G - 1;
    w.pt = p.nt_h1 - 1 - (int)r;
    return true;
}

// Fills the work-decomposition fields (everything from wg_rows on) for sequences of
// `rows` query rows; needs B, Hkv and G.  False if the work list does not fit 31 bits.
inline bool plan_work(FwdParams &p, int rows, int wg_rows) {
    p.wg_rows = wg_rows;
    p.n4 = p.G / 4;
    p.has2 = (p.G % 4) >= 2 ? 1 : 0;
    p.has1 = p.G % 2;
    p.nt_h4 = (rows + wg_rows / 4 - 1) / (wg_rows / 4);
    p.nt_h2 = (rows + wg_rows / 2 - 1) / (wg_rows / 2);
    p.nt_h1 = (rows + wg_rows - 1) / wg_rows;
    p.tiles_per_pair = p.n4 * p.nt_h4 + p.has2 * p.nt_h2 + p.has1 * p.nt_h1;
    p.packed_compact = 0;
    p.total_items = (long long)p.B * p.Hkv * p.tiles_per_pair;
    p.div_tiles_per_pair = make_fastdiv((unsigned)p.tiles_per_pair);
    p.div_hkv = make_fastdiv((unsigned)p.Hkv);
    p.div_nt_h4 = make_fastdiv((unsigned)p.nt_h4);
    p.chunk = (p.total_items + kXcds - 1) / kXcds;
    return p.chunk * kXcds <= 0x7fffffffLL;
}

// The plan of a packed batch of B sequences with total_rows query rows in all (each at most
// `rows` long): the compact work list of decode_work_packed, bounded from above -- a sequence
// adds at most one partly filled tile per head group to total_rows / tile rows, and at most one
// slot per XCD for the rounding of its eight chunks.
inline bool plan_work_packed(FwdParams &p, int rows, int wg_rows, long long total_rows) {
    if (!plan_work(p, rows, wg_rows)) return false;
    if (wg_rows != 128 && wg_rows != 256) return true;  // (decode_work_packed knows these two; else the plain list)
    auto bound = [&](int tile_rows) { return (total_rows + tile_rows - 1) / tile_rows + p.B; };
    const long long tiles = p.n4 * bound(wg_rows / 4) + p.has2 * bound(wg_rows / 2) + p.has1 * bound(wg_rows);
    const long long items = (long long)p.Hkv * tiles;
    p.packed_compact = 1;
    p.chunk = (items + kXcds - 1) / kXcds + p.B;
    p.total_items = p.chunk * kXcds;
    return p.total_items <= 0x7fffffffLL;
}

// Row block [p0, p0 + rows): a key is inside the window of every prompt row of
// the block iff it lies above the returned bound (last prompt row minus W); a
// block of generated tokens only has no such bound.
__device__ __forceinline__ int window_bound(int p0, int rows, int W, int P) {
    return p0 >= P ? -(1 << 30) : min(p0 + rows - 1, P - 1) - W;
}

// Lanes l and l^32 hold partial results for the same query column.
__device__ __forceinline__ float half_swap_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Launchers (one per kernel family); return the HIP error of the launch.
// (the plain kernel: head dimensions 32 .. 256 in steps of 32 except 128; its workgroups hold
// fwd_simple_wg_rows(D) query rows)
hipError_t launch_fwd_simple(const FwdParams &p, int D, hipStream_t stream);
int fwd_simple_wg_rows(int D);
hipError_t launch_fwd_pipelined_d128(const FwdParams &p, hipStream_t stream);

}  // namespace swaa

#endif  // SWAA_COMMON_H_
