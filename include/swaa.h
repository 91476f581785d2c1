/*
 * swaa.h -- C ABI of libswaa: sliding-window attention with "keep first k" sink
 * tokens, prefill forward pass, for AMD MI355X (gfx950).
 *
 * The operation (paper Sec. 1: sliding window attention restricts each token
 * to a fixed-size local window; Sec. 3.2.1 and Fig. 1b: every later token
 * attends to its local window AND the initial k tokens, implemented as a mask
 * inside the attention kernel; Sec. 3.1.2 and Sec. 4.1.2: layers that keep
 * full attention are the same computation with a window at least as long as
 * the context).  For batch b, query head h, KV head g = h / (Hq / Hkv) and
 * query row i (0-based):
 *
 *     Vis(i)   = { j : 0 <= j <= i  and ( j > i - window  or  j < n_sink ) }
 *     s_j      = scale * <q[b,h,i,:], k[b,g,j,:]>
 *     lse[b,h,i]   = ln sum_{j in Vis(i)} exp(s_j)
 *     out[b,h,i,:] = sum_{j in Vis(i)} exp(s_j - lse[b,h,i]) * v[b,g,j,:]
 *
 * The window (i - window, i] holds `window` keys and includes the query's own
 * position; a key that is both a sink and inside the window counts once;
 * sinks are causal.  Inputs and `out` are bf16, products are accumulated in
 * fp32, `lse` is fp32 (natural logarithm of the scaled scores).
 *
 * All data pointers are DEVICE pointers owned by the caller; the library
 * neither allocates, frees nor retains them, keeps no state between calls and
 * is safe to call from several host threads.  Calls are asynchronous: work is
 * enqueued on `stream` and the function returns without synchronising.
 * Errors are reported through the return value only; every check happens
 * before anything is launched, so a failed call has touched no memory.
 */
#ifndef SWAA_H_
#define SWAA_H_

#ifdef __cplusplus
extern "C" {
#endif

typedef enum swaa_status {
    SWAA_OK = 0,
    SWAA_ERR_NULL = -1,        /* a required pointer is NULL */
    SWAA_ERR_SHAPE = -2,       /* a size, the window, the sink count, the prompt length or the scale is out of range */
    SWAA_ERR_UNSUPPORTED = -3, /* head dimension without a kernel instantiation */
    SWAA_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned */
    SWAA_ERR_LAUNCH = -5,      /* the HIP runtime refused the launch */
    SWAA_ERR_WORKSPACE = -6    /* the workspace is NULL, not 16-byte aligned or too small */
} swaa_status;

/*
 * Attention forward (the operation defined at the top of this file).
 *
 *   q    device, bf16 [B, Hq,  N, D], contiguous, 16-byte aligned, read only
 *   k    device, bf16 [B, Hkv, N, D], contiguous, 16-byte aligned, read only
 *   v    device, bf16 [B, Hkv, N, D], contiguous, 16-byte aligned, read only
 *   out  device, bf16 [B, Hq,  N, D], contiguous, 16-byte aligned, written;
 *        must not overlap q, k or v
 *   lse  device, fp32 [B, Hq, N], contiguous, written
 *   B, Hq, Hkv, N >= 1; Hq a multiple of Hkv (query head h reads KV head
 *        h / (Hq/Hkv)); N * D * max(Hq, Hkv) * B must fit in 2^62 elements
 *   D    head dimension: a multiple of 32 up to 256 (128 has the tuned, software-pipelined
 *        kernel; the others run on a plain tiled kernel)
 *   window  >= 1; any value >= N means full causal attention
 *   n_sink  >= 0; values >= N behave as N
 *   scale   finite and > 0 (callers normally pass 1/sqrt(D))
 *   stream  a hipStream_t, or NULL for the default stream
 *
 * Returns SWAA_OK or a negative swaa_status.
 */
int swaa_attn_fwd(const void *q, const void *k, const void *v, void *out, float *lse,
                  int B, int Hq, int Hkv, int N, int D, int window, int n_sink,
                  float scale, void *stream);

/*
 * Attention forward under the FA Decode mask (paper Sec. 3.1.1 and Fig. 1a:
 * the sliding window applies to the prefilling stage only; during decoding
 * each token reverts to full attention over all previous tokens).  The
 * sequence of N positions is the prompt followed by the generated tokens, as
 * when a whole conversation is processed in one pass:
 *
 *     Vis(i) = { j : 0 <= j <= i  and ( j > i - window  or  j < n_sink ) }   for i <  n_prompt
 *     Vis(i) = { j : 0 <= j <= i }                                           for i >= n_prompt
 *
 * and everything else as in swaa_attn_fwd, whose arguments, layouts, ownership
 * and error behaviour apply unchanged.
 *
 *   n_prompt  >= 0: number of leading prompt rows; values >= N mean that there
 *             are no generated rows (the call then equals swaa_attn_fwd), 0
 *             means full causal attention for every row
 *
 * Returns SWAA_OK or a negative swaa_status (n_prompt < 0: SWAA_ERR_SHAPE).
 */
int swaa_attn_fwd_fa_decode(const void *q, const void *k, const void *v, void *out, float *lse,
                            int B, int Hq, int Hkv, int N, int D, int window, int n_sink,
                            int n_prompt, float scale, void *stream);

/*
 * The general form of the two calls above: strided tensors, query rows that are
 * the newest Nq of Nk tokens (a chunk of a longer prefill whose earlier keys and
 * values are cached; row r sits at position Nk - Nq + r, as in swaa_attn_decode),
 * and packed batches of sequences of different lengths -- the calling
 * conventions of a serving engine (paper Sec. 4.1.1: vLLM; App. D: prefill and
 * decode tokens mixed in one batch).  The mask is that of
 * swaa_attn_fwd_fa_decode, in positions:
 *
 *     pos    = Nk - Nq + r
 *     Vis(r) = { j : 0 <= j <= pos  and ( pos >= n_prompt  or  j > pos - window  or  j < n_sink ) }
 *
 * A tensor is a device pointer to element [0, 0, 0, 0] plus the element strides
 * of batch entry, head and row; the D elements of a row are contiguous.  All
 * strides are multiples of 8 elements (row starts stay 16-byte aligned);
 * stride_n >= D and < 2^22.  [B, H, N, D], [B, N, H, D] and slices of either
 * are all expressible.  lse is fp32 with contiguous rows:
 * lse[b * lse_stride_b + h * lse_stride_h + r].
 *
 * Packed batches: when cu_seqlens_q and cu_seqlens_k (device arrays of B + 1
 * ints, both or neither) are given, sequence b owns rows
 * [cu_seqlens_q[b], cu_seqlens_q[b+1]) of q / out / lse and rows
 * [cu_seqlens_k[b], cu_seqlens_k[b+1]) of k / v along the row axis; batch
 * strides are ignored, and Nq, Nk are upper bounds on the sequence lengths
 * (rows beyond Nq are not computed).  A sequence with more query rows than keys
 * gets only its first Nk_b rows written; empty sequences are skipped.
 *
 * dtype selects the 16-bit element format of q, k, v and out: SWAA_BF16 (the
 * format of every other call) or SWAA_F16, which computes the same thing on
 * binary16 operands and rounds the probabilities and the output to binary16
 * (fp32 accumulation; runs on the plain kernel).
 *
 * Paged key/value cache (prefill of a chunk against a serving engine's cache, as
 * swaa_attn_decode_ex reads it): with block_table given, token j of sequence b
 * lives in page block_table[b][j / page_size], and its row of KV head kvh at
 * k.ptr + page * k.stride_b + kvh * k.stride_h + (j % page_size) * k.stride_n
 * (likewise v); page_size a multiple of 16, block_table_stride * page_size >= Nk,
 * num_pages = pages in the cache (page numbers are clamped to it).  With
 * cu_seqlens the keys' offsets only give each sequence's number of cached tokens
 * (cu_seqlens_k[b+1] - cu_seqlens_k[b]); q, out and lse stay packed.  Head
 * dimension 128 only (SWAA_ERR_UNSUPPORTED otherwise).
 *
 * Ownership, asynchrony and error reporting as for swaa_attn_fwd; the argument
 * block is read during the call only.  Without cu_seqlens, Nq <= Nk is required.
 */
typedef enum swaa_dtype {
    SWAA_BF16 = 0, /* bfloat16: every kernel */
    SWAA_F16 = 1   /* IEEE binary16 (the precision the paper serves in, Sec. 4.1.1) */
} swaa_dtype;

typedef struct swaa_tensor {
    void *ptr;
    long long stride_b, stride_h, stride_n;
} swaa_tensor;

typedef struct swaa_fwd_args {
    swaa_tensor q;   /* bf16, Hq heads, query rows; read only */
    swaa_tensor k;   /* bf16, Hkv heads, key rows; read only */
    swaa_tensor v;   /* bf16, Hkv heads, key rows; read only */
    swaa_tensor out; /* bf16, Hq heads, query rows; written; must not overlap the inputs */
    float *lse;      /* fp32, written */
    long long lse_stride_b, lse_stride_h;
    int B, Hq, Hkv, D;      /* D: a multiple of 32 up to 256 */
    int Nq, Nk;             /* query rows and keys per sequence (upper bounds for packed batches) */
    const int *cu_seqlens_q; /* device, B + 1 ints, or NULL */
    const int *cu_seqlens_k; /* device, B + 1 ints, or NULL */
    int window, n_sink;     /* as in swaa_attn_fwd */
    int n_prompt;           /* as in swaa_attn_fwd_fa_decode, in positions; >= Nk: no generated rows */
    float scale;
    void *stream;
    int dtype;              /* swaa_dtype of q, k, v and out */
    /* paged key/value cache (block_table NULL: k, v are tensors as described above) */
    const int *block_table; /* device, B rows of block_table_stride ints, or NULL */
    int block_table_stride, page_size, num_pages;
    /* Packed batches: the number of rows of the packed q tensor (at least cu_seqlens_q[B]; the
     * host cannot read that), or 0 if not known.  With it the launch holds one workgroup per row
     * tile a sequence really has instead of B times the longest sequence's: batches of very
     * different lengths run many times faster.  Rows beyond a total stated too small are not
     * computed.  Ignored for fixed-length batches. */
    long long total_rows_q;
    /* Per-sequence prompt lengths: device, B ints, or NULL.  With it sequence b takes
     * n_prompts[b] (negative values count as 0) in place of n_prompt: in a batch of a
     * serving engine every sequence has a prompt of its own (paper Sec. 3.1.1, FA Decode:
     * the window applies to prompt tokens only). */
    const int *n_prompts;
} swaa_fwd_args;

int swaa_attn_fwd_ex(const swaa_fwd_args *args);

/*
 * Number of visible (query, key) pairs per head under the mask of swaa_attn_fwd, i.e.
 * sum over i in [0, N) of |Vis(i)|; the benchmark counts 4*D floating-point
 * operations per pair (paper App. A: the cost of sliding window attention is
 * O(N * W)).  Host-only arithmetic; returns -1 on an invalid argument.
 */
long long swaa_visible_pairs(long long N, long long window, long long n_sink);

/* The same count under the FA Decode mask of swaa_attn_fwd_fa_decode. */
long long swaa_visible_pairs_fa_decode(long long N, long long window, long long n_sink, long long n_prompt);

/*
 * Decode-shape attention (paper Sec. 3.1.1: during auto-regressive generation
 * each new token attends to the cached keys and values of all previous tokens
 * -- FA Decode, window >= Nk -- or, when decoding stays on sliding-window
 * attention, to its local window and the first n_sink tokens of Sec. 3.2.1).
 * The Nq query rows are the newest tokens of a sequence of Nk tokens whose keys
 * and values, their own included, are in the cache: row r sits at position
 * pos = Nk - Nq + r and
 *
 *     Vis(r) = { j : 0 <= j <= pos  and ( j > pos - window  or  j < n_sink ) }
 *
 * with s_j, lse and out as in swaa_attn_fwd.
 *
 *   q    device, bf16 [B, Hq,  Nq, D], contiguous, 16-byte aligned, read only
 *   k,v  device, bf16 [B, Hkv, Nk, D], contiguous, 16-byte aligned, read only
 *   out  device, bf16 [B, Hq,  Nq, D], written; lse device, fp32 [B, Hq, Nq], written
 *   1 <= Nq <= Nk; D = 128; window, n_sink, scale, stream as in swaa_attn_fwd
 *   workspace  device scratch memory owned by the caller, 16-byte aligned, at
 *        least swaa_attn_decode_workspace_bytes(same shape arguments) bytes;
 *        holds the partial results of the key splits between the call's two
 *        kernels; contents before and after the call are meaningless, and calls
 *        that may overlap on the device need separate workspaces
 *
 * The library allocates nothing.  Returns SWAA_OK or a negative swaa_status;
 * SWAA_ERR_WORKSPACE if the workspace is NULL, misaligned or too small.
 */
int swaa_attn_decode(const void *q, const void *k, const void *v, void *out, float *lse,
                     int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink,
                     float scale, void *workspace, long long workspace_bytes, void *stream);

/*
 * The general form of swaa_attn_decode, for the caches of a serving engine
 * (paper Sec. 4.1.1: the models are served with vLLM, batch size 64): strided
 * or PAGED key/value caches and a batch of sequences with different cache
 * lengths.
 *
 *   q, out, lse   as in swaa_attn_decode (contiguous [B, Hq, Nq, D] / [B, Hq, Nq])
 *   seq_lens      device, B ints, or NULL: the number of cached tokens of each
 *                 sequence, the Nq newest included (values are clamped to [Nq, Nk]);
 *                 NULL: every sequence holds Nk tokens
 *   contiguous cache (block_table NULL): k, v are tensors as in swaa_fwd_args, key
 *                 row j of (b, kvh) at ptr + b * stride_b + kvh * stride_h + j * stride_n
 *   paged cache   block_table: device, B rows of block_table_stride ints; token j of
 *                 sequence b lives in page block_table[b][j / page_size], and its
 *                 row of KV head kvh at
 *                 ptr + page * stride_b + kvh * stride_h + (j % page_size) * stride_n;
 *                 page_size a multiple of 4, block_table_stride * page_size >= Nk,
 *                 num_pages = pages in the cache (page numbers are clamped to it)
 *   Nk            the largest cache length (an upper bound on seq_lens);
 *                 workspace of at least swaa_attn_decode_ex_workspace_bytes(args) bytes
 *
 * With seq_lens (and 2 <= B <= 256) the key splits are planned on the device from the
 * lengths themselves, so that every sequence gets splits in proportion to its length
 * and a batch with one long sequence among short ones still fills the chip; without,
 * they are planned for Nk.
 *   dtype         swaa_dtype of q, k, v and out: SWAA_BF16 (0, what a zeroed struct
 *                 and swaa_attn_decode select) or SWAA_F16, the precision the paper
 *                 serves in (Sec. 4.1.1); anything else: SWAA_ERR_UNSUPPORTED
 *
 * Everything else as in swaa_attn_decode.
 */
typedef struct swaa_decode_args {
    const void *q;
    void *out;
    float *lse;
    swaa_tensor k, v;
    const int *seq_lens;
    const int *block_table;
    int block_table_stride, page_size, num_pages;
    int B, Hq, Hkv, Nq, Nk, D;
    int window, n_sink;
    float scale;
    void *workspace;
    long long workspace_bytes;
    void *stream;
    int dtype;
} swaa_decode_args;

int swaa_attn_decode_ex(const swaa_decode_args *args);

/*
 * Bytes of workspace swaa_attn_decode needs for these shape arguments (a few
 * KiB per key split; host-only arithmetic), or a negative swaa_status if the
 * arguments are invalid.
 */
long long swaa_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink);

/*
 * The same for swaa_attn_decode_ex: reads the shape fields of args (B, Hq, Hkv, Nq, Nk,
 * D, window, n_sink) and whether seq_lens is NULL (per-sequence lengths take another
 * split plan, which may need more), nothing else, and no device memory.  Without
 * seq_lens the result equals swaa_attn_decode_workspace_bytes.
 */
long long swaa_attn_decode_ex_workspace_bytes(const swaa_decode_args *args);

/*
 * swaa_attn_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernels as swaa_attn_decode,
 * except that the partial results of the key splits go to a static device array
 * of SWAA_DECODE_STATIC_SCRATCH_BYTES inside the library instead of a workspace.
 * The call allocates and frees nothing; the array's device address is looked up
 * on the first call on each GPU (each GPU the library runs on holds its own copy
 * until the process ends).
 *
 *   - a shape whose swaa_attn_decode_workspace_bytes exceeds
 *     SWAA_DECODE_STATIC_SCRATCH_BYTES is refused with SWAA_ERR_WORKSPACE before
 *     anything is launched (use swaa_attn_decode with a workspace for those);
 *   - every call on a GPU shares that GPU's array: calls that may overlap on one
 *     GPU (two streams, two host threads) race on it and must be serialised by
 *     the caller; consecutive calls on one stream are fine.  The array keeps the
 *     last call's contents, and nothing in it has to be cleared between calls:
 *     every slot the merge kernel takes into account is written first by the same
 *     call's split kernel.
 */
#define SWAA_DECODE_STATIC_SCRATCH_BYTES (16LL << 20)
int swaa_attn_decode_static(const void *q, const void *k, const void *v, void *out, float *lse,
                            int B, int Hq, int Hkv, int Nq, int Nk, int D, int window, int n_sink,
                            float scale, void *stream);

/*
 * Backward pass of swaa_attn_fwd_fa_decode (and, with n_prompt >= N, of
 * swaa_attn_fwd): the gradients that fine-tuning under the sliding-window mask
 * (paper Sec. 3.2.2, with the structural masks of Sec. 3.1.1 and Sec. 3.2.1
 * applied during training) needs.  With P_ij = exp(s_ij - lse[i]) for j in
 * Vis(i) and 0 elsewhere, and dout the gradient with respect to out:
 *
 *     dv[j] = sum_i P_ij dout[i]
 *     dS_ij = P_ij ( <dout[i], v[j]> - <dout[i], out[i]> )
 *     dq[i] = scale * sum_j dS_ij k[j]        dk[j] = scale * sum_i dS_ij q[i]
 *
 * where dk and dv of a KV head sum over the Hq/Hkv query heads that read it.
 *
 *   q, k, v, out, lse   the forward call's inputs and results (same layouts)
 *   dout                device, bf16 [B, Hq, N, D], contiguous, read only
 *   dq                  device, bf16 [B, Hq,  N, D], written
 *   dk, dv              device, bf16 [B, Hkv, N, D], written
 *   D                   64 or 128; window, n_sink, n_prompt, scale, stream as in the forward call
 *   workspace           device scratch memory owned by the caller, 16-byte aligned, at
 *                       least swaa_attn_bwd_workspace_bytes(same shape and mask arguments)
 *                       bytes; calls that may overlap on the device need separate workspaces
 *
 * bf16 tensors 16-byte aligned; P and dS are rounded to bf16 before the second
 * products, all sums are fp32.  Deterministic (no atomics).  The library
 * allocates nothing.  Returns SWAA_OK or a negative swaa_status.
 */
int swaa_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                  const void *dout, void *dq, void *dk, void *dv,
                  int B, int Hq, int Hkv, int N, int D, int window, int n_sink, int n_prompt,
                  float scale, void *workspace, long long workspace_bytes, void *stream);

/*
 * Bytes of workspace swaa_attn_bwd needs (one float per query row, plus partial
 * sums for the key tiles that hold sink keys), or a negative swaa_status.
 */
long long swaa_attn_bwd_workspace_bytes(int B, int Hq, int Hkv, int N, int D, int window, int n_sink, int n_prompt);

/* Static description of a status code; never NULL, never freed. */
const char *swaa_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int swaa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SWAA_H_ */
