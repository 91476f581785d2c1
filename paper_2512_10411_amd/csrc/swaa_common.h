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
    int wg_rows;  // 256 (plain forward and backward kernels) or 128 (pipelined forward)
    int n4, has2, has1;
    int nt_h4, nt_h2, nt_h1;  // row tiles of a sequence of Nq rows for workgroups of 4, 2 and 1 heads
    FastDiv div_tiles_per_pair, div_hkv, div_nt_h4;  // for the work-list decode of every workgroup
    int tiles_per_pair;
    long long total_items;
    long long chunk;  // work items per XCD
};

// One sequence as a workgroup sees it: the query rows are the newest nq of its nk
// tokens (row r sits at position nk - nq + r; nq = nk for a plain prefill).
struct SeqGeom {
    int nq, nk;
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

// Workgroups reach the 8 XCDs round-robin; XCD x takes the x-th contiguous
// chunk of the work list, so the position tiles of one KV head, whose K/V
// bands overlap, run behind the same L2.  Inside a pair, long rows go first.
__device__ __forceinline__ bool decode_work(const FwdParams &p, WorkItem &w) {
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
    p.total_items = (long long)p.B * p.Hkv * p.tiles_per_pair;
    p.div_tiles_per_pair = make_fastdiv((unsigned)p.tiles_per_pair);
    p.div_hkv = make_fastdiv((unsigned)p.Hkv);
    p.div_nt_h4 = make_fastdiv((unsigned)p.nt_h4);
    p.chunk = (p.total_items + kXcds - 1) / kXcds;
    return p.chunk * kXcds <= 0x7fffffffLL;
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
