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
};

hipError_t launch_bwd(const BwdParams &p, int D, hipStream_t stream);

}  // namespace swaa

#endif  // SWAA_BWD_H_
