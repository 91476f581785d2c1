// Building blocks of the head-dimension-128 attention kernels of libswaa (gfx950):
// MFMA wrappers, LDS operand reads for K and V^T fragments of a 32-key half
// tile, the half-tile contractions and the max-based softmax of one half.
//
// LDS is addressed with plain byte addresses: kernels that include this file
// declare no static LDS, so their dynamic LDS starts at address 0.
#ifndef SWAA_TILE_D128_H_
#define SWAA_TILE_D128_H_

#include "swaa_common.h"

namespace swaa {

constexpr int kD = 128;
constexpr int kKS = kD / 16;  // k-steps of K Q^T
constexpr int kDB = kD / 32;  // 32-wide blocks of the head dimension
constexpr int kRowBytes = kD * 2;                 // one K, V, Q or O row
constexpr int kHalfBytes = 32 * kRowBytes;        // one 32-key half tile: 8 KiB
constexpr float kRefSlack = 8.f;  // log2 units a row maximum may exceed its reference before the reference moves

// ---- MFMA through inline assembly ------------------------------------------------
// The compiler cannot be told to keep some MFMA operands in AccVGPRs and others
// in VGPRs within one function, so every MFMA is written out with the register
// file in the constraint.  Consequences the code below has to honour itself:
//   (1) a vector instruction that writes an MFMA operand must be at least two
//       instructions ahead of the MFMA (hardware needs two wait states);
//   (2) a vector instruction that reads an MFMA result must wait for the MFMA
//       to finish.  The compiler may copy a result register right after the
//       statement that produced it, so the idle cycles belong into the same
//       asm statement as the last MFMA of a chain (*_settled below); settle_*
//       alone is only safe where other MFMAs lie between producer and reader.
// tests/test_asm_hazards.py checks both on the generated assembly.
// kF16: the 16-bit operands are IEEE binary16 instead of bfloat16.  Fragments are carried
// in bf16x8 registers either way (eight 16-bit lanes; only the MFMA's mnemonic and the
// float -> 16-bit conversions look at the format).
template <bool kF16 = false>
__device__ __forceinline__ void mfma_acc(f32x16 &acc, const bf16x8 a, const bf16x8 b) {
    if constexpr (kF16)
        asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// S^T accumulator: VGPR destination, Q operand read straight from AccVGPRs.
template <bool kF16 = false>
__device__ __forceinline__ void mfma_s(f32x16 &s, const bf16x8 kfrag, const bf16x8 q_acc) {
    if constexpr (kF16)
        asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(s) : "v"(kfrag), "a"(q_acc));
    else
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(kfrag), "a"(q_acc));
}
template <bool kF16 = false>
__device__ __forceinline__ void mfma_s_first(f32x16 &s, const bf16x8 kfrag, const bf16x8 q_acc) {
    if constexpr (kF16)
        asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(s) : "v"(kfrag), "a"(q_acc));
    else
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(kfrag), "a"(q_acc));
}
// Last MFMA of a chain whose result the vector ALU reads next.
template <bool kF16 = false>
__device__ __forceinline__ void mfma_s_settled(f32x16 &s, const bf16x8 kfrag, const bf16x8 q_acc) {
    if constexpr (kF16)
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 7" : "+v"(s) : "v"(kfrag), "a"(q_acc));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 7" : "+v"(s) : "v"(kfrag), "a"(q_acc));
}
template <bool kF16 = false>
__device__ __forceinline__ void mfma_acc_settled(f32x16 &acc, const bf16x8 a, const bf16x8 b) {
    if constexpr (kF16)
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 7" : "+a"(acc) : "v"(a), "v"(b));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 7" : "+a"(acc) : "v"(a), "v"(b));
}
// Two floats -> two 16-bit elements of the chosen format (round to nearest even), as the
// bit pattern of two fragment lanes.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <bool kF16>
__device__ __forceinline__ bf16x2 pack_pair(float a, float b) {
    if constexpr (kF16) {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        f16x2 h;
        h[0] = (_Float16)a;
        h[1] = (_Float16)b;
        return __builtin_bit_cast(bf16x2, h);
    } else {
        bf16x2 r;
        r[0] = (__bf16)a;
        r[1] = (__bf16)b;
        return r;
    }
}
// Makes the compiler hold `o` in AccVGPRs at this point (placed after every
// plain C++ write to the accumulators so that the value carried around the key
// loop never changes register file) and spaces those writes from the next MFMA.
__device__ __forceinline__ void pin_acc(f32x16 (&o)[kDB]) {
    asm volatile("s_nop 1" : "+a"(o[0]), "+a"(o[1]), "+a"(o[2]), "+a"(o[3]));
}
// Materialises a freshly packed P^T fragment here (the compiler would otherwise
// be free to sink the conversion down to the MFMA that reads it).
__device__ __forceinline__ void pin_p(bf16x8 &pf) { asm volatile("" : "+v"(pf)); }

// First MFMA of a K Q^T chain.  masked: start from the 0 / -inf visibility tile
// of the half whose first key is k0h; otherwise from zero.
__device__ __forceinline__ void qk_chain_start(f32x16 &s, const bf16x8 kfrag, const bf16x8 q_acc, bool masked, int k0h,
                                               int qpos, int W, int S, int hf) {
    if (__builtin_expect(masked, 0)) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int key = k0h + 8 * (e / 4) + 4 * hf + (e % 4);
            const bool vis = (key <= qpos) && ((key > qpos - W) || (key < S));
            s[e] = vis ? 0.f : -INFINITY;
        }
        asm volatile("s_nop 1" : "+v"(s));  // two wait states between these writes and the MFMA
        mfma_s(s, kfrag, q_acc);
    } else {
        mfma_s_first(s, kfrag, q_acc);
    }
}

// ---- LDS operand reads ---------------------------------------------------------------
__device__ __forceinline__ bf16x8 lds_read16(uint32_t addr) {
    return *(const bf16x8 __attribute__((address_space(3))) *)(uintptr_t)addr;
}
__device__ __forceinline__ s16x4 lds_read8_tr(uint32_t addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(uintptr_t)addr);
}

// Per-lane byte offsets of the MFMA A-operand fragments inside one 32-key half
// of a K or V tile, XOR swizzle folded in; a uniform buffer offset is added.
struct LaneAddr {
    uint32_t k[kKS];  // K fragment of k-step ks: row lane%32, 16-byte chunk 2*ks + lane/32
    uint32_t v[kDB];  // V^T fragment of head-dimension block db, 16-key step 0, keys 0..3
};

__device__ __forceinline__ bf16x8 load_k_frag(const LaneAddr &la, uint32_t boff, int ks) {
    return lds_read16(la.k[ks] + boff);
}
// two transposing reads: keys {0..3} and {8..11} of this half-wave's eight
__device__ __forceinline__ bf16x8 load_v_frag(const LaneAddr &la, uint32_t boff, int st, int db) {
    const uint32_t a0 = la.v[db] + boff;
    const s16x4 lo = lds_read8_tr(a0 + st * 16 * 256);
    const s16x4 hi = lds_read8_tr(a0 + st * 16 * 256 + 8 * 256);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// S^T (32 keys x 32 queries) = K_half Q^T; the result is ready for the vector ALU on return
template <bool kF16 = false>
__device__ __forceinline__ void qk_half(const LaneAddr &la, uint32_t kboff, const bf16x8 (&qf)[kKS], f32x16 &s) {
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) {
        const bf16x8 a = load_k_frag(la, kboff, ks);
        if (ks == 0)
            mfma_s_first<kF16>(s, a, qf[ks]);
        else if (ks < kKS - 1)
            mfma_s<kF16>(s, a, qf[ks]);
        else
            mfma_s_settled<kF16>(s, a, qf[ks]);
    }
}

// O^T (128 x 32 queries) += V_half^T P^T.  kSettle: the accumulators are ready for
// the vector ALU on return (all MFMAs complete in order, so waiting out the last
// one covers the four chains).
template <bool kSettle, bool kF16 = false>
__device__ __forceinline__ void pv_half(const LaneAddr &la, uint32_t vboff, const bf16x8 (&pf)[2], f32x16 (&o)[kDB]) {
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int db = 0; db < kDB; ++db) {
            const bf16x8 a = load_v_frag(la, vboff, st, db);
            if (kSettle && st == 1 && db == kDB - 1)
                mfma_acc_settled<kF16>(o[db], a, pf[st]);
            else
                mfma_acc<kF16>(o[db], a, pf[st]);
        }
    }
}

// Softmax state of one query column.  The column's 32 scores of a half are
// split over the lane pair (l32, l32 + 32); each lane keeps the sums over its
// own 16 scores, and row_sums adds the two shares when a total is needed.
struct RowState {
    float mc;  // softmax reference, in exp2 units (m * scale * log2 e); the same in both lanes
    float l;   // share of the sum of exp2(s * c2 - mc): the log-sum-exp comes from this one
    float lb;  // share of the sum of the same terms after rounding to bf16: the divisor of O
};

// acc + lo + hi for two entries of P as the P V contraction sees them.  The
// contraction weights V with the rounded entries, so O has to be divided by
// their sum: then the weights add up to one whatever the rounding did to them,
// and a row with a single visible key returns that key's V row exactly even
// when its reference is not its own score.  (Dividing by the fp32 sum leaves a
// relative error of up to 2^-9 in such a row, a whole bf16 step after the
// final rounding.)  One dot-product instruction per pair.
template <bool kF16 = false>
__device__ __forceinline__ float add_rounded_pair(float acc, bf16x2 pr) {
    if constexpr (kF16) {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        f16x2 one;
        one[0] = (_Float16)1.f;
        one[1] = (_Float16)1.f;
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pr), one, acc, false);
    } else {
        bf16x2 one;
        one[0] = (__bf16)1.f;
        one[1] = (__bf16)1.f;
        return __builtin_amdgcn_fdot2_f32_bf16(pr, one, acc, false);
    }
}

__device__ __forceinline__ void row_sums(const RowState &st, float &l, float &lb) {
    l = half_swap_sum(st.l);
    lb = half_swap_sum(st.lb);
}

// Max-based softmax of one half tile (edge tiles, first tile, and the rare
// half whose row sums outgrow the reference): optional mask, reference update
// with slack, exponentials, row sum, bf16 P^T fragments.  alpha is the factor
// the O accumulator must be multiplied with (1 when the reference stays).  The
// scores must be settled (qk_half leaves them so).
template <bool kMask, bool kF16 = false>
__device__ __forceinline__ void softmax_half(f32x16 &s, int k0h, int qpos, int W, int S, int hf, float c2, RowState &st,
                                             bf16x8 (&pf)[2], float &alpha) {
    if (kMask) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int key = k0h + 8 * (e / 4) + 4 * hf + (e % 4);
            const bool vis = (key <= qpos) && ((key > qpos - W) || (key < S));
            s[e] = vis ? s[e] : -INFINITY;
        }
    }
    float mx = s[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s[e]);
    mx = half_swap_max(mx);
    const float mc_old = st.mc;
    const float m_new = fmaxf(mc_old, mx * c2);
    const bool move = m_new > mc_old + kRefSlack;  // -inf never moves to -inf
    st.mc = move ? m_new : mc_old;
    const float mc_use = (kMask && st.mc == -INFINITY) ? 0.f : st.mc;
    alpha = move ? __builtin_amdgcn_exp2f(mc_old - mc_use) : 1.f;
    float rs = 0.f, rb = 0.f;
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[e], c2, -mc_use));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[e + 1], c2, -mc_use));
        rs += p0 + p1;
        const bf16x2 pr = pack_pair<kF16>(p0, p1);
        pf[e / 8][e % 8] = pr[0];
        pf[e / 8][e % 8 + 1] = pr[1];
        rb = add_rounded_pair<kF16>(rb, pr);
    }
    st.l = st.l * alpha + rs;  // (alpha is the same in both lanes of a column)
    st.lb = st.lb * alpha + rb;
    // keep the packing here and two wait states away from the MFMAs that read it
    asm volatile("s_nop 1" : "+v"(pf[0]), "+v"(pf[1]));
}

// (the accumulators must be settled: pv_half<true>, or other MFMAs since their last update)
__device__ __forceinline__ void rescale(f32x16 (&o)[kDB], float alpha) {
    if (__any(alpha != 1.f)) {
        // (pinned on entry too: the copies from the accumulator registers that the multiplications
        // need then stay inside this branch -- the compiler had moved all 64 of them in front of
        // it, into every trip round the key loop, taken or not)
        pin_acc(o);
#pragma unroll
        for (int db = 0; db < kDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
        pin_acc(o);
    }
}

// The per-lane offsets above; v_base is added to the V offsets (kernels whose V
// buffers sit behind their K buffers fold the distance in here).
__device__ __forceinline__ LaneAddr make_lane_addr(int lane, uint32_t v_base) {
    LaneAddr la;
    const int l32 = lane & 31, hf = lane >> 5;
    const int fr = ((l32 & 7) << 1) | ((l32 >> 3) & 1);
    const uint32_t k_lane = (uint32_t)(l32 * 256 + ((hf ^ fr) << 4));
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) la.k[ks] = k_lane ^ (uint32_t)(ks << 5);
    const int j16 = lane & 15, grp = lane >> 4;
    const int low2 = 2 * (grp & 1) + ((j16 & 3) >> 1);
    const uint32_t v_lane =
        v_base + (uint32_t)((4 * hf + (j16 >> 2)) * 256 + (((((j16 >> 2) & 3) << 2) | low2) << 4) + 8 * (j16 & 1));
#pragma unroll
    for (int db = 0; db < kDB; ++db) la.v[db] = v_lane ^ (uint32_t)(db << 6);
    return la;
}

}  // namespace swaa

#endif  // SWAA_TILE_D128_H_
