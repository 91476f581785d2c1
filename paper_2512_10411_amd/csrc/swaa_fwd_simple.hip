// Sliding-window + sink ("keep first k") attention forward for gfx950 (MI355X).
//
// The mask is the one of the paper's Sec. 3.2.1 / Fig. 1b (local window AND
// the initial k tokens, causal) and, with a window at least as long as the
// context, the full-attention layers of Sec. 3.1.2.  The tiling, the
// schedule and the register layout below are this library's own design for
// CDNA4; the paper only says that the mask lives inside a flash-style kernel.
//
// This is the plain kernel: it serves every head dimension that is a multiple of
// 32 up to 256 except 128, which has the software-pipelined kernel of its own.
//
// Shape of the kernel
//   * One workgroup = 4 wavefronts = 128 "query rows" that share one KV head:
//     hpb query heads (4, 2 or 1) x 128/hpb consecutive positions.  Each wave
//     owns 32 positions of one head, so K/V tiles staged in LDS are reused by
//     every query head of the GQA group and the dense band per wave is only
//     W + 32 keys wide.  Head dimensions up to 96 leave registers for three or
//     four such workgroups per CU; above 128, O^T and Q of 32 positions fill the
//     register file and one workgroup runs per CU.  (The kernel can also give a
//     wave 64 positions, 256 rows per workgroup: no instantiation uses it now.)
//   * KV tiles of 64 keys.  A workgroup visits only the tiles that hold sink
//     keys [0, S) or band keys (first position - W, last position]; a wave
//     skips the MFMA work of tiles that lie outside its own 64 positions' band
//     and applies the element mask only on tiles that cross an edge.
//   * S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K from LDS, B = Q kept in
//     registers): a lane then owns one query column, so the row maximum and
//     row sum are in-lane reductions plus one half-wave swap, and the bf16
//     P^T values are already in the B-operand layout of O^T += V^T P^T.
//   * V^T fragments come from row-major V in LDS through the transposing read
//     ds_read_b64_tr_b16.
//   * Online softmax in fp32 in the exp2 domain; O is rescaled only when some
//     row maximum in the wave moved.
#include <cmath>

#include "swaa_common.h"

namespace swaa {
namespace {

template <int D>
struct Tile {
    static constexpr int kChunksPerRow = D / 8;                        // 16-byte chunks
    static constexpr int kChunks = kBk * kChunksPerRow;                // per K or V tile
    static constexpr int kChunksPerThread = kChunks / kThreads;       // D / 32
    static_assert(D % 32 == 0 && D >= 32 && D <= 256, "head dimension: a multiple of 32 up to 256");
    static constexpr int kKStride = D + 8;                             // bf16 elements, K rows
    static constexpr int kVStride = D + 32;                            // bf16 elements, V rows
    static constexpr int kKElems = kBk * kKStride;
    static constexpr int kVElems = kBk * kVStride;
};

// Element types: bfloat16 (the library's main format) and IEEE binary16 (the paper serves its
// models in float16, Sec. 4.1.1).  Both share the 16-bit storage, the layouts and the MFMA shape.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
template <typename E>
struct Elem;
template <>
struct Elem<__bf16> {
    using x8 = bf16x8;
    using x4 = bf16x4;
    static __device__ __forceinline__ f32x16 mfma(x8 a, x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <>
struct Elem<_Float16> {
    using x8 = f16x8;
    using x4 = f16x4;
    static __device__ __forceinline__ f32x16 mfma(x8 a, x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

// QB: 32-row blocks of query positions per wave (1 in every instantiation; 2 is possible up to D = 128)
// Head dimensions up to kSmallD run 32 positions per wave and several workgroups per CU (the
// registers allow it), so that one wave's softmax runs under another's matrix instructions:
// measured against 64 positions per wave and one workgroup per CU, D = 64 is 1.25 - 1.37 x as
// fast, D = 96 1.15 - 1.24 x.  D = 160 still fits two workgroups per CU with a few registers
// spilled outside the loop (1.4 - 1.5 x); from 192 on the spills land inside it and cost more
// than the second workgroup brings.
constexpr int kSmallD = 96;
constexpr int min_blocks(int D) { return D <= 64 ? 4 : D <= kSmallD ? 3 : D <= 160 ? 2 : 1; }
template <int D, typename E, int QB>
__global__ __launch_bounds__(kThreads, min_blocks(D)) void swaa_fwd_kernel(const FwdParams p) {
    using T = Tile<D>;
    using X = Elem<E>;
    using x8 = typename X::x8;
    using x4 = typename X::x4;
    constexpr int KS = D / 16;  // k-steps of the QK^T contraction
    constexpr int DB = D / 32;  // 32-wide blocks of the head dimension
    constexpr int kWaveRows = 32 * QB;           // (hides the namespace's constants of the same names)
    constexpr int kWgRows = 4 * kWaveRows;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    E *Ks = reinterpret_cast<E *>(smem_raw);
    E *Vs = Ks + T::kKElems;

    WorkItem wi;
    if (!decode_work(p, wi)) return;
    const int b = wi.b, kvh = wi.kvh, hpb = wi.hpb, h0 = wi.h0, pt = wi.pt;
    SeqGeom sg;
    if (!seq_geom(p, b, sg)) return;
    const int rows_per_wg = kWgRows / hpb;
    const int wg_r0 = pt * rows_per_wg;  // first query row of the workgroup
    if (wg_r0 >= sg.nq) return;          // a shorter sequence of a packed batch
    const int Nq = sg.nq, Nk = sg.nk, W = p.W, S = p.S, P = sg.n_prompt;
    const int pos_off = Nk - Nq;  // query row r sits at position pos_off + r

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int hf = lane >> 5;  // which half of the wave

    const int head = kvh * p.G + h0 + (wave % hpb);
    const int r0 = wg_r0 + (wave / hpb) * kWaveRows;                // first query row of this wave
    const int wg_p0 = pos_off + wg_r0;                              // first position of the workgroup
    const int wg_p1 = pos_off + min(Nq, wg_r0 + rows_per_wg) - 1;   // last valid position
    const int p0 = pos_off + r0;                                    // first position of this wave
    const bool wave_active = r0 < Nq;
    const int plast = pos_off + min(r0 + kWaveRows, Nq) - 1;        // last valid position of this wave

    // ---- KV tiles this workgroup visits -------------------------------------
    // (a workgroup that holds a generated token visits every tile up to its diagonal)
    const int band_lo = (wg_p1 >= P) ? 0 : max(0, wg_p0 - W + 1);
    const int t_band_lo = band_lo / kBk;
    const int t_hi = wg_p1 / kBk;
    const int n_sink_tiles = min((min(S, band_lo) + kBk - 1) / kBk, t_band_lo);
    // tile order: 0 .. n_sink_tiles-1, then t_band_lo .. t_hi
    const int wbound = window_bound(p0, kWaveRows, W, P);

    const E *kg = reinterpret_cast<const E *>(p.k) + sg.k_batch * p.k_sb + (long long)kvh * p.k_sh + sg.k_row0 * p.k_sn;
    const E *vg = reinterpret_cast<const E *>(p.v) + sg.k_batch * p.v_sb + (long long)kvh * p.v_sh + sg.k_row0 * p.v_sn;
    const E *qg = reinterpret_cast<const E *>(p.q) + sg.q_batch * p.q_sb + (long long)head * p.q_sh + sg.q_row0 * p.q_sn;
    E *og = reinterpret_cast<E *>(p.out) + sg.q_batch * p.o_sb + (long long)head * p.o_sh + sg.q_row0 * p.o_sn;

    // ---- Q fragments (B operand of S^T = K Q^T), kept for the whole loop ----
    x8 qf[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = min(r0 + 32 * qb + l32, Nq - 1);
        const E *src = qg + (size_t)row * p.q_sn + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[qb][ks] = *reinterpret_cast<const x8 *>(src + 16 * ks);
    }

    f32x16 oacc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[db][qb][e] = 0.f;
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
    }

    // ---- staging: global -> registers -> LDS --------------------------------
    u32x4 kreg[T::kChunksPerThread], vreg[T::kChunksPerThread];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int c = 0; c < T::kChunksPerThread; ++c) {
            const int id = c * kThreads + tid;
            const int row = min(t * kBk + id / T::kChunksPerRow, Nk - 1);  // tail rows are masked later
            const int col = (id % T::kChunksPerRow) * 8;
            kreg[c] = *reinterpret_cast<const u32x4 *>(kg + (size_t)row * p.k_sn + col);
            vreg[c] = *reinterpret_cast<const u32x4 *>(vg + (size_t)row * p.v_sn + col);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int c = 0; c < T::kChunksPerThread; ++c) {
            const int id = c * kThreads + tid;
            const int row = id / T::kChunksPerRow;
            const int col = (id % T::kChunksPerRow) * 8;
            *reinterpret_cast<u32x4 *>(&Ks[row * T::kKStride + col]) = kreg[c];
            *reinterpret_cast<u32x4 *>(&Vs[row * T::kVStride + col]) = vreg[c];
        }
    };
    auto next_tile = [&](int t) {
        int n = t + 1;
        if (n == n_sink_tiles && n < t_band_lo) n = t_band_lo;
        return n;
    };

    int t = (n_sink_tiles > 0) ? 0 : t_band_lo;
    load_tile(t);
    store_tile();
    __syncthreads();

    const float c2 = p.scale_log2;

    while (true) {
        const int tn = next_tile(t);
        const bool has_next = tn <= t_hi;
        if (has_next) load_tile(tn);  // in flight while this tile is computed

        const int k0 = t * kBk;
        const int k_last = k0 + kBk - 1;
        // per-wave classification of the tile against this wave's 64 positions
        const bool in_future = k0 > plast;
        const bool before_band = (plast < P) && (k_last < p0 - W + 1) && (k0 >= S);
        if (wave_active && !in_future && !before_band) {
            const bool unmasked = (k_last <= p0) && ((k0 > wbound) || (k_last < S));

            // ---- S^T = K Q^T : [64 keys] x [64 queries] ----
            f32x16 sacc[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) sacc[kb][qb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const x8 a = *reinterpret_cast<const x8 *>(
                        &Ks[(32 * kb + l32) * T::kKStride + 16 * ks + 8 * hf]);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        sacc[kb][qb] = X::mfma(a, qf[qb][ks], sacc[kb][qb]);
                }
            }

            // ---- mask (edge tiles only) ----
            if (!unmasked) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const int qpos = p0 + 32 * qb + l32;
                    const int wq = (qpos >= P) ? Nk : W;  // a generated token's window is the whole prefix
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int key = k0 + 32 * kb + 8 * (e / 4) + 4 * hf + (e % 4);
                            const bool vis = (key <= qpos) && ((key > qpos - wq) || (key < S));
                            sacc[kb][qb][e] = vis ? sacc[kb][qb][e] : -INFINITY;
                        }
                }
            }

            // ---- online softmax; P^T packed to bf16 in B-operand order ----
            x8 pf[2][QB][2];  // [kb][qb][16-key step]
            float alpha[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = sacc[0][qb][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[kb][qb][e]);
                mx = half_swap_max(mx);
                const float m_new = fmaxf(m_run[qb], mx);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                alpha[qb] = __builtin_amdgcn_exp2f((m_run[qb] - m_use) * c2);
                const float mc = m_use * c2;
                float rs = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float pe = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][e], c2, -mc));
                        rs += pe;
                        pf[kb][qb][e / 8][e % 8] = (E)pe;
                    }
                }
                rs = half_swap_sum(rs);
                l_run[qb] = l_run[qb] * alpha[qb] + rs;
                m_run[qb] = m_new;
            }
            // rescale O only if some row maximum in this wave moved
            bool moved = false;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) moved = moved || (alpha[qb] != 1.f);
            if (__any(moved)) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                        for (int e = 0; e < 16; ++e) oacc[db][qb][e] *= alpha[qb];
            }

            // ---- O^T += V^T P^T ----
            // For the 16-key step (kb, st) the half-wave hf contracts over keys
            // 32kb + 16st + 4hf + {0..3, 8..11}, the order in which the S^T
            // accumulator hands them out; V^T must use the same order.
            const int grp = lane >> 4;  // 16-lane group of the transposing read
            const int j16 = lane & 15;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const int krow = 32 * kb + 16 * st + 4 * hf + (j16 >> 2);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const int col = 32 * db + 16 * (grp & 1) + 4 * (j16 & 3);
                        const E *a0 = &Vs[krow * T::kVStride + col];
                        const E *a1 = a0 + 8 * T::kVStride;
                        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3))) *)(a0));
                        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3))) *)(a1));
                        const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        const x8 a = __builtin_bit_cast(x8, av);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            oacc[db][qb] = X::mfma(a, pf[kb][qb][st], oacc[db][qb]);
                    }
                }
            }
        }

        if (!has_next) break;
        __syncthreads();  // every wave is done reading this tile
        store_tile();
        __syncthreads();
        t = tn;
    }

    // ---- epilogue: O / l -> bf16, lse = m*scale + ln(l) ----------------------
    if (!wave_active) return;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = r0 + 32 * qb + l32;
        if (row >= Nq) continue;
        const float inv_l = 1.f / l_run[qb];
        E *orow = og + (size_t)row * p.o_sn;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (E)(oacc[db][qb][4 * e4 + e] * inv_l);
                *reinterpret_cast<x4 *>(orow + 32 * db + 8 * e4 + 4 * hf) = o4;
            }
        }
        if (hf == 0)
            p.lse[sg.q_batch * p.lse_sb + (long long)head * p.lse_sh + sg.q_row0 + row] =
                (m_run[qb] * c2 + __builtin_amdgcn_logf(l_run[qb])) * 0.69314718055994530942f;
    }
}

}  // namespace

namespace {

template <int D, typename E>
hipError_t launch_one(const FwdParams &p, hipStream_t stream) {
    constexpr int QB = 1;
    using T = Tile<D>;
    constexpr int kBytes = (T::kKElems + T::kVElems) * 2;
    if (p.wg_rows != 4 * 32 * QB) return hipErrorInvalidValue;  // the plan must be the one for this instantiation
    auto kernel = swaa_fwd_kernel<D, E, QB>;
    if (kBytes > 64 * 1024) {
        // more than 64 KiB of dynamic LDS has to be asked for (harmless to repeat)
        const hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(p.chunk * kXcds)), dim3(kThreads), kBytes, stream, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_format(const FwdParams &p, hipStream_t stream) {
    return p.fp16 ? launch_one<D, _Float16>(p, stream) : launch_one<D, __bf16>(p, stream);
}

}  // namespace

int fwd_simple_wg_rows(int) { return 128; }

hipError_t launch_fwd_simple(const FwdParams &p, int D, hipStream_t stream) {
    switch (D) {
        case 32: return launch_format<32>(p, stream);
        case 64: return launch_format<64>(p, stream);
        case 96: return launch_format<96>(p, stream);
        case 160: return launch_format<160>(p, stream);
        case 192: return launch_format<192>(p, stream);
        case 224: return launch_format<224>(p, stream);
        case 256: return launch_format<256>(p, stream);
        default: return hipErrorInvalidValue;  // (128 has the pipelined kernel)
    }
}

}  // namespace swaa
