// C ABI of libswaa: argument checks, work decomposition, kernel choice.
#include <cmath>
#include <cstdint>
#include <cstring>

#include "swaa.h"
#include "swaa_common.h"
#include "swaa_bwd.h"
#include "swaa_decode.h"

using swaa::FwdParams;
using swaa::kXcds;

namespace {

// finite and > 0, tested on the bit pattern (independent of fast-math flags)
bool positive_finite(float x) {
    uint32_t u;
    std::memcpy(&u, &x, sizeof u);
    return (u >> 31) == 0 && ((u >> 23) & 0xffu) != 0xffu && (u << 1) != 0;
}

bool misaligned(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; }

}  // namespace

extern "C" {

long long swaa_visible_pairs(long long N, long long window, long long n_sink) {
    if (N < 1 || window < 1 || n_sink < 0) return -1;
    const long long W = window < N ? window : N;
    const long long M = N - W;  // rows whose window no longer reaches key 0
    long long pairs = W * (W + 1) / 2 + M * W;
    // row i = W - 1 + x (x = 1..M) has x keys in front of its window; min(x, S) are sinks
    const long long ramp = n_sink < M ? n_sink : M;
    pairs += ramp * (ramp + 1) / 2 + (M - ramp) * n_sink;
    return pairs;
}

long long swaa_visible_pairs_fa_decode(long long N, long long window, long long n_sink, long long n_prompt) {
    if (N < 1 || window < 1 || n_sink < 0 || n_prompt < 0) return -1;
    const long long P = n_prompt < N ? n_prompt : N;
    // the visible set of a prompt row does not depend on N; generated row i sees i + 1 keys
    const long long prompt_pairs = P > 0 ? swaa_visible_pairs(P, window, n_sink) : 0;
    return prompt_pairs + (N * (N + 1) - P * (P + 1)) / 2;
}

const char *swaa_status_string(int status) {
    switch (status) {
        case SWAA_OK: return "ok";
        case SWAA_ERR_NULL: return "null pointer argument";
        case SWAA_ERR_SHAPE: return "size, window, sink count, prompt length or scale out of range";
        case SWAA_ERR_UNSUPPORTED: return "unsupported head dimension or element type (forward: multiples of 32 up to 256; decode: 128; backward: 64 and 128)";
        case SWAA_ERR_ALIGN: return "pointer not 16-byte aligned";
        case SWAA_ERR_LAUNCH: return "HIP launch failed";
        case SWAA_ERR_WORKSPACE: return "workspace missing, misaligned or too small (or the call needs more scratch than the static array holds)";
        default: return "unknown status";
    }
}

int swaa_version(void) { return 130; }

namespace {

bool bad_stride(long long s, bool may_be_zero) {
    if (s == 0) return !may_be_zero;
    return s < 0 || (s % 8) != 0;  // row, head and batch starts stay 16-byte aligned
}

}  // namespace

int swaa_attn_fwd_ex(const swaa_fwd_args *a) {
    if (!a) return SWAA_ERR_NULL;
    if (!a->q.ptr || !a->k.ptr || !a->v.ptr || !a->out.ptr || !a->lse) return SWAA_ERR_NULL;
    const int B = a->B, Hq = a->Hq, Hkv = a->Hkv, D = a->D, Nq = a->Nq, Nk = a->Nk;
    if (B < 1 || Hq < 1 || Hkv < 1 || Nq < 1 || Nk < 1 || D < 1) return SWAA_ERR_SHAPE;
    if (Hq % Hkv != 0) return SWAA_ERR_SHAPE;
    if (a->window < 1 || a->n_sink < 0 || a->n_prompt < 0) return SWAA_ERR_SHAPE;
    if (!positive_finite(a->scale)) return SWAA_ERR_SHAPE;
    const bool packed = a->cu_seqlens_q != nullptr || a->cu_seqlens_k != nullptr;
    if (packed && (!a->cu_seqlens_q || !a->cu_seqlens_k)) return SWAA_ERR_NULL;
    if (!packed && Nq > Nk) return SWAA_ERR_SHAPE;  // the query rows are the newest Nq of Nk tokens
    if (D % 32 != 0 || D > 256) return SWAA_ERR_UNSUPPORTED;
    if (a->dtype != SWAA_BF16 && a->dtype != SWAA_F16) return SWAA_ERR_UNSUPPORTED;
    const bool paged = a->block_table != nullptr;
    if (paged && D != 128) return SWAA_ERR_UNSUPPORTED;
    if (paged && (a->page_size < 16 || a->page_size % 16 != 0 || a->num_pages < 1 || a->block_table_stride < 1))
        return SWAA_ERR_SHAPE;
    if (paged && (long long)a->block_table_stride * a->page_size < Nk) return SWAA_ERR_SHAPE;  // table too short for Nk tokens
    for (const swaa_tensor *t : {&a->q, &a->k, &a->v, &a->out}) {
        const bool kv = t == &a->k || t == &a->v;
        const int heads = kv ? Hkv : Hq;
        if (misaligned(t->ptr)) return SWAA_ERR_ALIGN;
        if (bad_stride(t->stride_n, false) || t->stride_n < D || t->stride_n >= (1LL << 22)) return SWAA_ERR_SHAPE;
        // (the batch stride of a paged k or v is the page stride)
        const bool one_block = (kv && paged) ? a->num_pages == 1 : (packed || B == 1);
        if (bad_stride(t->stride_h, heads == 1) || bad_stride(t->stride_b, one_block)) return SWAA_ERR_SHAPE;
    }
    if (paged && (reinterpret_cast<uintptr_t>(a->block_table) & 3u)) return SWAA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(a->lse) & 3u) != 0) return SWAA_ERR_ALIGN;
    if (a->lse_stride_h < 0 || a->lse_stride_b < 0) return SWAA_ERR_SHAPE;
    if (packed && ((reinterpret_cast<uintptr_t>(a->cu_seqlens_q) | reinterpret_cast<uintptr_t>(a->cu_seqlens_k)) & 3u))
        return SWAA_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(a->n_prompts) & 3u) return SWAA_ERR_ALIGN;

    FwdParams p{};
    p.q = static_cast<const __bf16 *>(a->q.ptr);
    p.k = static_cast<const __bf16 *>(a->k.ptr);
    p.v = static_cast<const __bf16 *>(a->v.ptr);
    p.out = static_cast<__bf16 *>(a->out.ptr);
    p.lse = a->lse;
    p.q_sb = a->q.stride_b; p.q_sh = a->q.stride_h; p.q_sn = a->q.stride_n;
    p.k_sb = a->k.stride_b; p.k_sh = a->k.stride_h; p.k_sn = a->k.stride_n;
    p.v_sb = a->v.stride_b; p.v_sh = a->v.stride_h; p.v_sn = a->v.stride_n;
    p.o_sb = a->out.stride_b; p.o_sh = a->out.stride_h; p.o_sn = a->out.stride_n;
    p.lse_sb = a->lse_stride_b; p.lse_sh = a->lse_stride_h;
    p.fp16 = a->dtype == SWAA_F16 ? 1 : 0;
    p.cu_q = a->cu_seqlens_q;
    p.cu_k = a->cu_seqlens_k;
    p.n_prompts = a->n_prompts;
    p.block_table = a->block_table;
    p.bt_stride = paged ? a->block_table_stride : 0;
    p.page_size = paged ? a->page_size : 1;
    p.num_pages = paged ? a->num_pages : 1;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.Nq = Nq; p.Nk = Nk;
    p.W = a->window < Nk ? a->window : Nk;
    p.S = a->n_sink < Nk ? a->n_sink : Nk;
    p.P = a->n_prompt < Nk ? a->n_prompt : Nk;
    p.G = Hq / Hkv;
    p.scale = a->scale;
    p.scale_log2 = a->scale * 1.44269504088896340736f;
    // the pipelined kernel (head dimension 128, either 16-bit format) runs workgroups of 128
    // rows, two per compute unit; other head dimensions run on the plain kernel
    const bool pipelined = D == 128;
    const int wg_rows = pipelined ? 128 : swaa::fwd_simple_wg_rows(D);
    if (a->total_rows_q < 0) return SWAA_ERR_SHAPE;
    if (packed && a->total_rows_q > 0 ? !swaa::plan_work_packed(p, Nq, wg_rows, a->total_rows_q) : !swaa::plan_work(p, Nq, wg_rows))
        return SWAA_ERR_SHAPE;

    hipStream_t s = static_cast<hipStream_t>(a->stream);
    const hipError_t err = pipelined ? swaa::launch_fwd_pipelined_d128(p, s) : swaa::launch_fwd_simple(p, D, s);
    return err == hipSuccess ? SWAA_OK : SWAA_ERR_LAUNCH;
}

int swaa_attn_fwd_fa_decode(const void *q, const void *k, const void *v, void *out, float *lse,
                            int B, int Hq, int Hkv, int N, int D, int window, int n_sink,
                            int n_prompt, float scale, void *stream) {
    if (!q || !k || !v || !out || !lse) return SWAA_ERR_NULL;
    if (B < 1 || Hq < 1 || Hkv < 1 || N < 1 || D < 1) return SWAA_ERR_SHAPE;
    // contiguous [B, H, N, D] tensors, every sequence N rows on N keys
    swaa_fwd_args a{};
    const long long nd = (long long)N * D;
    a.q = {const_cast<void *>(q), Hq * nd, nd, D};
    a.k = {const_cast<void *>(k), Hkv * nd, nd, D};
    a.v = {const_cast<void *>(v), Hkv * nd, nd, D};
    a.out = {out, Hq * nd, nd, D};
    a.lse = lse;
    a.lse_stride_b = (long long)Hq * N;
    a.lse_stride_h = N;
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.D = D;
    a.Nq = N; a.Nk = N;
    a.cu_seqlens_q = nullptr;
    a.cu_seqlens_k = nullptr;
    a.window = window; a.n_sink = n_sink; a.n_prompt = n_prompt;
    a.scale = scale;
    a.stream = stream;
    a.dtype = SWAA_BF16;
    a.block_table = nullptr;
    a.block_table_stride = a.page_size = a.num_pages = 0;
    return swaa_attn_fwd_ex(&a);
}

int swaa_attn_fwd(const void *q, const void *k, const void *v, void *out, float *lse,
                  int B, int Hq, int Hkv, int N, int D, int window, int n_sink,
                  float scale, void *stream) {
    // every row is a prompt token
    return swaa_attn_fwd_fa_decode(q, k, v, out, lse, B, Hq, Hkv, N, D, window, n_sink, N, scale, stream);
}

namespace {

// Shape checks shared by the two decode entry points; fills the shape fields and the plan.
int decode_plan(swaa::DecodeParams &p, int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink, bool ragged) {
    if (B < 1 || Hq < 1 || Hkv < 1 || Nq < 1 || Nk < 1 || D < 1) return SWAA_ERR_SHAPE;
    if (Hq % Hkv != 0 || Nq > Nk) return SWAA_ERR_SHAPE;
    if (window < 1 || n_sink < 0) return SWAA_ERR_SHAPE;
    if (D != 128) return SWAA_ERR_UNSUPPORTED;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.Nq = Nq; p.Nk = Nk;
    p.W = window < Nk ? window : Nk;
    p.S = n_sink < Nk ? n_sink : Nk;
    if ((long long)p.G * Nq > 0x7fffffffLL / 256) return SWAA_ERR_SHAPE;
    swaa::plan_decode(p, ragged);
    if (p.items + 64 > 0x7fffffffLL || (long long)B * Hq * Nq > 0x7fffffffLL)
        return SWAA_ERR_SHAPE;
    return SWAA_OK;
}

}  // namespace

long long swaa_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink) {
    swaa::DecodeParams p{};
    const int rc = decode_plan(p, B, Hq, Hkv, Nq, Nk, D, window, n_sink, false);
    return rc != SWAA_OK ? rc : swaa::decode_workspace_floats(p) * (long long)sizeof(float);
}

long long swaa_attn_decode_ex_workspace_bytes(const swaa_decode_args *a) {
    if (!a) return SWAA_ERR_NULL;
    swaa::DecodeParams p{};
    const int rc = decode_plan(p, a->B, a->Hq, a->Hkv, a->Nq, a->Nk, a->D, a->window, a->n_sink, a->seq_lens != nullptr);
    return rc != SWAA_OK ? rc : swaa::decode_workspace_floats(p) * (long long)sizeof(float);
}

namespace {

// Both decode entry points.  own_scratch: the partial results go to the library's static
// device array instead of the caller's workspace (whose two fields are then ignored).
int decode_call(const swaa_decode_args *a, bool own_scratch) {
    if (!a) return SWAA_ERR_NULL;
    if (!a->q || !a->k.ptr || !a->v.ptr || !a->out || !a->lse) return SWAA_ERR_NULL;
    swaa::DecodeParams p{};
    const int rc = decode_plan(p, a->B, a->Hq, a->Hkv, a->Nq, a->Nk, a->D, a->window, a->n_sink, a->seq_lens != nullptr);
    if (rc != SWAA_OK) return rc;
    if (!positive_finite(a->scale)) return SWAA_ERR_SHAPE;
    if (a->dtype != SWAA_BF16 && a->dtype != SWAA_F16) return SWAA_ERR_UNSUPPORTED;
    const bool paged = a->block_table != nullptr;
    if (paged && (a->page_size < 4 || a->page_size % 4 != 0 || a->num_pages < 1 || a->block_table_stride < 1))
        return SWAA_ERR_SHAPE;
    if (paged && (long long)a->block_table_stride * a->page_size < a->Nk) return SWAA_ERR_SHAPE;  // table too short for Nk tokens
    for (const swaa_tensor *t : {&a->k, &a->v}) {
        if (misaligned(t->ptr)) return SWAA_ERR_ALIGN;
        if (bad_stride(t->stride_n, false) || t->stride_n < a->D || t->stride_n >= (1LL << 22)) return SWAA_ERR_SHAPE;
        if (bad_stride(t->stride_h, a->Hkv == 1) || bad_stride(t->stride_b, paged ? a->num_pages == 1 : a->B == 1))
            return SWAA_ERR_SHAPE;
        if (paged && t->stride_b >= (1LL << 31)) return SWAA_ERR_SHAPE;  // a page of 4 GiB and more: not a page
    }
    if (misaligned(a->q) || misaligned(a->out)) return SWAA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(a->lse) & 3u) != 0) return SWAA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(a->seq_lens) | reinterpret_cast<uintptr_t>(a->block_table)) & 3u) return SWAA_ERR_ALIGN;
    const long long need = swaa::decode_workspace_floats(p) * (long long)sizeof(float);
    void *workspace = a->workspace;
    if (own_scratch) {
        if (need > swaa::kDecodeStaticScratchBytes) return SWAA_ERR_WORKSPACE;
        if (swaa::decode_static_scratch(&workspace) != hipSuccess) return SWAA_ERR_LAUNCH;
    } else if (!workspace || misaligned(workspace) || a->workspace_bytes < need) {
        return SWAA_ERR_WORKSPACE;
    }

    p.q = static_cast<const __bf16 *>(a->q);
    p.k = static_cast<const __bf16 *>(a->k.ptr);
    p.v = static_cast<const __bf16 *>(a->v.ptr);
    p.out = static_cast<__bf16 *>(a->out);
    p.lse = a->lse;
    p.k_sb = a->k.stride_b; p.k_sh = a->k.stride_h; p.k_sn = a->k.stride_n;
    p.v_sb = a->v.stride_b; p.v_sh = a->v.stride_h; p.v_sn = a->v.stride_n;
    p.block_table = a->block_table;
    p.bt_stride = a->block_table_stride;
    p.page_size = paged ? a->page_size : 1;
    p.num_pages = paged ? a->num_pages : 1;
    p.div_page = swaa::make_fastdiv((unsigned)p.page_size);
    p.seq_lens = a->seq_lens;
    p.ws_o = static_cast<float *>(workspace);
    p.ws_ml = p.ws_o + p.items * (long long)p.col_stride * 128;
    p.ws_units = reinterpret_cast<int *>(p.ws_ml + p.items * 64);
    p.fp16 = a->dtype == SWAA_F16 ? 1 : 0;
    p.scale_log2 = a->scale * 1.44269504088896340736f;
    const hipError_t err = swaa::launch_decode(p, static_cast<hipStream_t>(a->stream));
    return err == hipSuccess ? SWAA_OK : SWAA_ERR_LAUNCH;
}

// The argument block of a contiguous [B, Hkv, Nk, D] cache, every sequence Nk tokens long.
swaa_decode_args contiguous_decode_args(const void *q, const void *k, const void *v, void *out, float *lse, int B,
                                        int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink, float scale,
                                        void *stream) {
    swaa_decode_args a{};
    a.q = q;
    a.out = out;
    a.lse = lse;
    const long long nd = (long long)(Nk > 0 ? Nk : 0) * (D > 0 ? D : 0);
    a.k = {const_cast<void *>(k), (long long)(Hkv > 0 ? Hkv : 0) * nd, nd, D};
    a.v = {const_cast<void *>(v), (long long)(Hkv > 0 ? Hkv : 0) * nd, nd, D};
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.Nq = Nq; a.Nk = Nk; a.D = D;
    a.window = window; a.n_sink = n_sink; a.scale = scale;
    a.stream = stream;
    return a;
}

}  // namespace

int swaa_attn_decode_ex(const swaa_decode_args *a) { return decode_call(a, false); }

int swaa_attn_decode(const void *q, const void *k, const void *v, void *out, float *lse,
                     int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink,
                     float scale, void *workspace, long long workspace_bytes, void *stream) {
    if (!q || !k || !v || !out || !lse) return SWAA_ERR_NULL;
    swaa_decode_args a = contiguous_decode_args(q, k, v, out, lse, B, Hq, Hkv, Nq, Nk, D, window, n_sink, scale, stream);
    a.workspace = workspace;
    a.workspace_bytes = workspace_bytes;
    return decode_call(&a, false);
}

int swaa_attn_decode_static(const void *q, const void *k, const void *v, void *out, float *lse,
                            int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink,
                            float scale, void *stream) {
    if (!q || !k || !v || !out || !lse) return SWAA_ERR_NULL;
    const swaa_decode_args a =
        contiguous_decode_args(q, k, v, out, lse, B, Hq, Hkv, Nq, Nk, D, window, n_sink, scale, stream);
    return decode_call(&a, true);
}

static_assert(SWAA_DECODE_STATIC_SCRATCH_BYTES == swaa::kDecodeStaticScratchBytes, "the header states the array's size");

namespace {

// Shape and mask fields of the backward parameter block, and its plan.
int bwd_plan(swaa::BwdParams &p, int B, int Hq, int Hkv, int N, int D, int window, int n_sink, int n_prompt) {
    if (B < 1 || Hq < 1 || Hkv < 1 || N < 1 || D < 1) return SWAA_ERR_SHAPE;
    if (Hq % Hkv != 0) return SWAA_ERR_SHAPE;
    if (window < 1 || n_sink < 0 || n_prompt < 0) return SWAA_ERR_SHAPE;
    if (D != 64 && D != 128) return SWAA_ERR_UNSUPPORTED;
    FwdParams &f = p.f;
    f.fp16 = 0;
    f.B = B; f.Hq = Hq; f.Hkv = Hkv; f.Nq = N; f.Nk = N;
    f.W = window < N ? window : N;
    f.S = n_sink < N ? n_sink : N;
    f.P = n_prompt < N ? n_prompt : N;
    f.G = Hq / Hkv;
    if (!swaa::plan_work(f, N, swaa::kWgRows) || (long long)B * Hq * N > 0x7fffffffLL * 16) return SWAA_ERR_SHAPE;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N;
    swaa::plan_bwd(p);
    return SWAA_OK;
}

}  // namespace

long long swaa_attn_bwd_workspace_bytes(int B, int Hq, int Hkv, int N, int D, int window, int n_sink, int n_prompt) {
    swaa::BwdParams p{};
    const int rc = bwd_plan(p, B, Hq, Hkv, N, D, window, n_sink, n_prompt);
    if (rc != SWAA_OK) return rc;
    return swaa::bwd_workspace_floats(p, D) * (long long)sizeof(float);
}

int swaa_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                  const void *dout, void *dq, void *dk, void *dv,
                  int B, int Hq, int Hkv, int N, int D, int window, int n_sink, int n_prompt,
                  float scale, void *workspace, long long workspace_bytes, void *stream) {
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return SWAA_ERR_NULL;
    swaa::BwdParams p{};
    const int rc = bwd_plan(p, B, Hq, Hkv, N, D, window, n_sink, n_prompt);
    if (rc != SWAA_OK) return rc;
    if (!positive_finite(scale)) return SWAA_ERR_SHAPE;
    for (const void *ptr : {q, k, v, out, dout, (const void *)dq, (const void *)dk, (const void *)dv})
        if (misaligned(ptr)) return SWAA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(lse) & 3u) != 0) return SWAA_ERR_ALIGN;
    if (!workspace || misaligned(workspace) ||
        workspace_bytes < swaa::bwd_workspace_floats(p, D) * (long long)sizeof(float))
        return SWAA_ERR_WORKSPACE;

    FwdParams &f = p.f;
    f.q = static_cast<const __bf16 *>(q);
    f.k = static_cast<const __bf16 *>(k);
    f.v = static_cast<const __bf16 *>(v);
    f.lse = const_cast<float *>(lse);
    f.scale = scale;
    f.scale_log2 = scale * 1.44269504088896340736f;
    p.out = static_cast<const __bf16 *>(out);
    p.dout = static_cast<const __bf16 *>(dout);
    p.dq = static_cast<__bf16 *>(dq);
    p.dk = static_cast<__bf16 *>(dk);
    p.dv = static_cast<__bf16 *>(dv);
    p.delta = static_cast<float *>(workspace);
    // the partial sums follow delta, on a 16-byte boundary
    p.partial = p.delta + (((long long)B * Hq * N + 3) / 4) * 4;
    const hipError_t err = swaa::launch_bwd(p, D, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? SWAA_OK : SWAA_ERR_LAUNCH;
}

}  // extern "C"
