// Backward pass: parameter block and launcher.
#ifndef SWAA_BWD_H_
#define SWAA_BWD_H_

#include "swaa_common.h"

namespace swaa {

struct BwdParams {
    FwdParams f;  // q, k, v, lse, the mask and the forward's work decomposition; contiguous [B, H, N, D]
    const __bf16 *out;   // forward output
    const __bf16 *dout;  // upstream gradient, shaped like out
    __bf16 *dq;          // [B, Hq, N, D]
    __bf16 *dk;          // [B, Hkv, N, D]
    __bf16 *dv;          // [B, Hkv, N, D]
    float *delta;        // workspace, [B, Hq, N]
    int B, Hq, Hkv, N;
    // Key tiles (128 keys) that hold sink keys are seen by every later row.  Their rows
    // beyond the band are cut into n_seg segments of seg_tiles query tiles, each computed
    // by a workgroup of its own; the band part and the segments leave fp32 partial sums in
    // `partial` ([B*Hkv][n_sink_kt][n_seg + 1][2 (dK, dV)][128][D]) and a last kernel adds them.
    int n_sink_kt, n_seg, seg_tiles;
    float *partial;  // workspace, after delta
};

// Fills n_sink_kt, n_seg, seg_tiles from the shape and mask fields.
void plan_bwd(BwdParams &p);
// Floats of workspace the plan needs (delta + partial sums).
long long bwd_workspace_floats(const BwdParams &p, int D);

hipError_t launch_bwd(const BwdParams &p, int D, hipStream_t stream);
// dQ alone, head dimension 128, software-pipelined (swaa_bwd_dq_pipelined.hip); delta must be there
hipError_t launch_bwd_dq_pipelined_d128(const BwdParams &p, hipStream_t stream);

}  // namespace swaa

#endif  // SWAA_BWD_H_
