// Decode-shape attention (few query rows against a long KV cache): parameter
// block, split plan and launchers.  Head dimension 128, gfx950.
#ifndef SWAA_DECODE_H_
#define SWAA_DECODE_H_

#include <hip/hip_runtime.h>

namespace swaa {

// The query rows of one (batch, KV head) pair -- G heads x Nq rows, contiguous
// in q -- are the columns of 32-wide column tiles.  The visited keys (sink
// halves, then the halves from the first row's window to the end of the cache;
// a half is 32 keys) are cut into splits; one single-wave workgroup computes
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
    int B, Hq, Hkv, G;
    int Nq, Nk;
    int W, S;  // clamped to [1, Nk] and [0, Nk]
    float scale_log2;
    int cols;        // G * Nq query rows per pair
    int n_coltiles;  // ceil(cols / 32)
    int col_stride;  // min(cols, 32): columns an item stores
    int n_sink_halves, band_half0, n_halves;  // visited halves: sink halves 0.., then key halves band_half0..
    int halves_per_split, n_splits;
    long long items;  // B * Hkv * n_coltiles * n_splits
};

// Fills the plan fields (everything from `cols` on) from the shape fields.
void plan_decode(DecodeParams &p);
// Floats the workspace must hold for this plan.
long long decode_workspace_floats(const DecodeParams &p);

hipError_t launch_decode(const DecodeParams &p, hipStream_t stream);

}  // namespace swaa

#endif  // SWAA_DECODE_H_
