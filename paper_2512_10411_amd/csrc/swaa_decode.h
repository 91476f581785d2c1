// Decode-shape attention (few query rows against a long KV cache): parameter
// block, split plan and launchers.  Head dimension 128, gfx950.
#ifndef SWAA_DECODE_H_
#define SWAA_DECODE_H_

#include <hip/hip_runtime.h>

#include "swaa_common.h"

namespace swaa {

// The query rows of one (batch, KV head) pair -- G heads x Nq rows, contiguous
// in q -- are the columns of 32-wide column tiles.  The visited keys (sink
// halves, then the halves from the first row's window to the end of the cache;
// a half is 32 keys; `visited_halves` below) are cut into splits; one single-wave workgroup computes
// one (pair, column tile, split) item and leaves an unnormalised partial result
// in the workspace; a second kernel merges the splits.
struct DecodeParams {
    const __bf16 *q;
    const __bf16 *k;
    const __bf16 *v;
    __bf16 *out;
    float *lse;
    float *ws_o;   // [items][col_stride][128]: sum of 2^(s c2 - mc) v over the item's keys
    float *ws_ml;  // [items][2][32]: mc (softmax reference, log2 units) and l (sum of 2^(s c2 - mc))
    int *ws_units;  // ragged plans: [B][2], first (sequence, split) unit and number of splits of each sequence
    // Cache addressing, in elements; the head dimension is contiguous.
    //   contiguous: row `key` of (b, kvh) at  k + b * k_sb + kvh * k_sh + key * k_sn
    //   paged:      page = block_table[b * bt_stride + key / page_size] and the row at
    //               k + page * k_sb + kvh * k_sh + (key % page_size) * k_sn
    long long k_sb, k_sh, k_sn;
    long long v_sb, v_sh, v_sn;
    const int *block_table;  // device, or null for a contiguous cache
    int bt_stride, page_size, num_pages;
    const int *seq_lens;  // device, B cache lengths (each <= Nk), or null: every sequence holds Nk tokens
    int B, Hq, Hkv, G;
    int Nq, Nk;  // Nk: the (largest) cache length; the plan is made for it
    int W, S;    // clamped to [1, Nk] and [0, Nk]
    float scale_log2;
    int cols;        // G * Nq query rows per pair
    int n_coltiles;  // ceil(cols / 32)
    int col_stride;  // min(cols, 32): columns an item stores
    int n_halves;  // upper bound on the halves a sequence of at most Nk tokens visits
    int halves_per_split, n_splits;
    long long items;  // B * Hkv * n_coltiles * n_splits (ragged: max_units * Hkv * n_coltiles; below 2^31): partial results in the workspace
    // a workgroup computes tiles_per_item (1 or 2) column tiles of one (pair, split) from the same
    // K and V fragments; n_ctgroups = ceil(n_coltiles / tiles_per_item) of them per (pair, split)
    int tiles_per_item, n_ctgroups;
    long long wg_items;  // B * Hkv * n_ctgroups * n_splits (ragged: max_units * Hkv * n_ctgroups, an upper bound): workgroups that have work
    int fp16;         // elements of q, k, v, out are IEEE binary16 instead of bfloat16
    // Sequences of different lengths (seq_lens given, a batch of 2 .. kRaggedMaxBatch): the splits are
    // planned on the device.  Every wave adds up the halves all sequences visit, takes
    // halves_per_split = max(4, ceil(sum / units_target)) and gives sequence b ceil(halves_b /
    // halves_per_split) splits -- work in proportion to length, at most units_target + B
    // (sequence, split) units in all (max_units: the launch and the workspace are sized for it).
    // halves_per_split and n_splits above are then not used.
    int ragged;
    int units_target, max_units;
    // divisions every workgroup makes, as multiplications (FastDiv)
    FastDiv div_ctgroups, div_splits, div_hkv, div_page, div_per_round;
};

// The halves a sequence of nk cached tokens visits: halves 0 .. n_sink-1, then key halves band0 ..
struct VisitedHalves {
    int n_sink, band0, n;
};
__host__ __device__ inline VisitedHalves visited_halves(int nk, int nq, int W, int S) {
    VisitedHalves h;
    const int band_lo = (nk - nq) - W + 1 > 0 ? (nk - nq) - W + 1 : 0;  // first key of the oldest row's window
    h.band0 = band_lo / 32;
    const int sink_keys = S < band_lo ? S : band_lo;
    const int sink_halves = (sink_keys + 31) / 32;
    h.n_sink = sink_halves < h.band0 ? sink_halves : h.band0;
    h.n = h.n_sink + ((nk - 1) / 32 - h.band0 + 1);
    return h;
}

// Fills the plan fields (everything from `cols` on) from the shape fields.  ragged: the sequences
// may hold far fewer than Nk tokens each (seq_lens is given): the device-side plan described at
// DecodeParams::ragged, for batches of 2 .. kRaggedMaxBatch sequences (else the plan for Nk).
constexpr int kRaggedMaxBatch = 256;
void plan_decode(DecodeParams &p, bool ragged);
// Floats the workspace must hold for this plan.
long long decode_workspace_floats(const DecodeParams &p);

hipError_t launch_decode(const DecodeParams &p, hipStream_t stream);

// Size of the library's own scratch array (one per GPU) behind swaa_attn_decode_static,
// and its device address on the current device (looked up on the first call per device).
constexpr long long kDecodeStaticScratchBytes = 16LL << 20;
hipError_t decode_static_scratch(void **ptr);

}  // namespace swaa

#endif  // SWAA_DECODE_H_
