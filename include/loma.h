/*
 * loma.h -- C ABI of the LoMA attention hot path for AMD MI355X (gfx950).
 *
 * LoMA (Lossless Compressed Memory Attention) restructures a sequence into chunks of
 *     [ reading zone, R = t*c tokens | memory zone, t <m> tokens | repetition zone, R <r> tokens ]
 * (Sec. 4.1) and trains/generates under a block attention mask (Sec. 4.3, Eq. 1-3).
 * This library computes scaled-dot-product attention under that mask, in the two
 * forms the paper uses:
 *   - the training / compression-pass form over a whole restructured sample
 *     (loma_mask_attn_fwd), and
 *   - the generation form of Sec. 3.1 / Appendix A over a compressed KV cache
 *     (loma_decode_attn per generated token, loma_compress_step every R tokens).
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers (HIP, current device), 16-byte aligned,
 *     dense row-major tensors [B, H, L, head_dim] (length on axis 2, as in the
 *     appendix's cache).  The caller owns every buffer; the library borrows it
 *     until the work enqueued on `stream` has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue kernels and return; they never allocate, free or synchronise.
 *   - `dtype` selects the storage type of q/k/v/out and of the caches: LOMA_F32 or
 *     LOMA_BF16.  Arithmetic: bf16 inputs are multiplied on the matrix cores with
 *     fp32 accumulation, softmax in fp32, probabilities rounded to bf16 before the
 *     PV product; f32 inputs use fp32 throughout.  Outputs are written in `dtype`.
 *   - `scale` multiplies the scores before the softmax (the paper leaves 1/sqrt(d_k)
 *     implicit, Sec. 4.4); it must be finite and > 0.
 *   - head_dim must be a multiple of 8 in [8, 256].  bf16 with head_dim 64 or 128
 *     takes the MFMA kernels; everything else takes a slower generic kernel.
 *   - Return value: LOMA_OK, or a negative LOMA_ERR_* code.  Argument checking is
 *     done on the host before anything is enqueued; on error nothing was launched
 *     (LOMA_ERR_LAUNCH excepted, which reports a failed hipLaunch).
 *   - A masked (query, key) pair is excluded from the softmax: its weight is exactly
 *     0 (Eq. 8-9).  K/V rows that no row of a workgroup's block may see are never loaded,
 *     whatever they hold (NaN and Inf included).  One precondition: the reading-zone rows
 *     that FOLLOW a reading row inside the same block of 32..128 rows share that block's
 *     causal diagonal tiles, which the matrix cores multiply whole; there the hidden pair
 *     contributes 0 * V, which is 0 only for finite V.  K and V must therefore be finite
 *     wherever some row of the sample can see them (any finite value leaves the hidden
 *     rows' results bit-identical).
 */
#ifndef LOMA_H_
#define LOMA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LOMA_OK 0
#define LOMA_ERR_INVALID_ARG (-1) /* null/misaligned pointer, non-positive size, state the method forbids */
#define LOMA_ERR_UNSUPPORTED (-2) /* well-formed but outside what the kernels handle (dtype, head_dim, size) */
#define LOMA_ERR_WORKSPACE (-3)   /* workspace missing or smaller than the matching *_workspace_bytes() */
#define LOMA_ERR_LAUNCH (-4)      /* the HIP runtime refused a kernel launch */

#define LOMA_F32 0
#define LOMA_BF16 1

/* Position types of the memory tokens (Sec. 4.5; Appendix A, `position_type`). */
#define LOMA_POS_INTERMITTENT 0 /* Eq. 14: the last id of every group of c reading tokens */
#define LOMA_POS_CONTIGUOUS 1   /* the row numbers of the compressed cache */

/* Human-readable name of a status code; never NULL. */
const char* loma_status_string(int status);

/* ABI version of this library (bumped on any signature change). */
int loma_abi_version(void);

/*
 * Training / compression-pass form (Sec. 4.3 Eq. 1-3, Sec. 4.4 Eq. 5-7).
 *
 * q, k, v, out: [B, H, S, head_dim] with S = n_chunks * t * (2c + 1); row p of a
 * sequence lies in chunk y = p / s (s = t(2c+1)) at offset o = p % s.
 *   reading row  (o < R):        sees the memory zones of all chunks < y, and rows
 *                                0..o of its own reading zone (causal, self included);
 *   memory row   (R <= o < R+t): sees its chunk's whole reading and memory zone;
 *   repetition row (o >= R+t):   sees its chunk's memory zone and itself.
 * out[p] = sum_j softmax_j(scale * q[p].k[j]) v[j] over the visible j.
 * lse (optional, may be NULL): [B, H, S] float, log-sum-exp of the scaled visible scores.
 * Masked tiles are never loaded; the mask is derived from (chunk, zone), not stored.
 */
int loma_mask_attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                       int B, int H, int head_dim, int t, int c, int n_chunks,
                       float scale, int dtype, void* stream);

/*
 * Gradients of the training form: what fine-tuning under the mask needs from this operation
 * (Sec. 4.2: the loss L = L_LM + L_Repeat is back-propagated through the attention of Sec. 4.3-4.4;
 * the repetition rows reach the text only through their chunk's memory-zone K/V, so the
 * gradient that trains the memory tokens flows through exactly this operator).
 *
 *   q, k, v, out, dout, dq, dk, dv: [B, H, S, head_dim] in `dtype`, S = n_chunks * t * (2c + 1)
 *   lse: [B, H, S] float, as written by loma_mask_attn_fwd for the same q, k, scale (required)
 *   out: the forward output for the same inputs;  dout: gradient of the loss w.r.t. out.
 * With W_ij = exp(scale q_i.k_j - lse_i) on visible pairs and 0 on masked ones, and
 * delta_i = dout_i . out_i:
 *   dv_j = sum_i W_ij dout_i
 *   dq_i = scale sum_j W_ij (dout_i . v_j - delta_i) k_j
 *   dk_j = scale sum_i W_ij (dout_i . v_j - delta_i) q_i
 * Sums run over visible pairs only; masked tiles are never loaded.  Arithmetic as in the forward
 * pass: bf16 products on the matrix cores with fp32 accumulation (W and dA rounded to bf16 before
 * their products), fp32 throughout for f32 data.  dq, dk, dv are fully overwritten; they must not
 * alias an input.  Deterministic: every output row is summed by one owner, no atomics.
 * workspace: device scratch of at least loma_mask_attn_bwd_workspace_bytes(...) bytes (two
 * floats per row: dout . out and the rescaled lse; for some shapes also fp32 partial sums of the
 * memory-zone keys' dk, dv, added in a fixed order), 16-byte aligned; contents are don't-care on
 * entry and exit; calls sharing a workspace must be stream-ordered.
 */
int loma_mask_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                       const void* dout, void* dq, void* dk, void* dv,
                       int B, int H, int head_dim, int t, int c, int n_chunks,
                       float scale, int dtype,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace loma_mask_attn_bwd needs for this shape.  0 on invalid arguments.  Host-only. */
size_t loma_mask_attn_bwd_workspace_bytes(int B, int H, int head_dim, int t, int c, int n_chunks, int dtype);

/*
 * Generation form, compression boundary (Sec. 3.1 step 2-3; Appendix A, compress_last_chunk).
 *
 * Precondition: the reading zone is full (R = t*c live tokens).
 *   q_mem, k_mem, v_mem: [B, H, t, head_dim]   the t <m> tokens of this chunk
 *   k_read, v_read:      [B, H, R, head_dim]   the live reading zone
 *   out:                 [B, H, t, head_dim]   attention output of the <m> queries
 *   k_memcache, v_memcache: [B, H, mem_capacity, head_dim], rows [0, n_mem_chunks*t) valid
 * The t queries attend, unmasked, over [reading zone || the t <m> tokens' own K/V]
 * (row 2 of Eq. 1); they do NOT see older memory zones.  Then k_mem/v_mem are copied
 * into the memory cache at rows [n_mem_chunks*t, (n_mem_chunks+1)*t) (the appendix's
 * splice).  The library is stateless: afterwards the caller sets n_mem_chunks += 1
 * and read_fill = 0 (the reading zone is discarded).
 * Errors: (n_mem_chunks + 1) * t > mem_capacity -> LOMA_ERR_INVALID_ARG.
 */
int loma_compress_step(const void* q_mem, const void* k_mem, const void* v_mem,
                       const void* k_read, const void* v_read,
                       void* k_memcache, void* v_memcache, void* out,
                       int B, int H, int head_dim, int t, int c,
                       int n_mem_chunks, int mem_capacity,
                       float scale, int dtype, void* stream);

/*
 * Generation form, one new token per sequence (Sec. 3.1 step 1 and 3; Appendix A,
 * inference_input with one input token: the mask row is all ones over cache + self).
 *
 *   q:             [B, H, 1, head_dim]
 *   k_new, v_new:  [B, H, 1, head_dim] or both NULL
 *   k_memcache, v_memcache: [B, H, mem_capacity, head_dim], rows [0, n_mem_chunks*t) valid
 *                  (may be NULL when n_mem_chunks == 0)
 *   k_read, v_read:[B, H, R, head_dim], rows [0, read_fill) valid
 *   out:           [B, H, 1, head_dim]
 * With k_new/v_new: they are written to reading-zone row read_fill (requires
 * read_fill < R, the appendix's invariant) and the query attends over
 * n_mem_chunks*t + read_fill + 1 keys; the caller then sets read_fill += 1.
 * Without: the query attends over n_mem_chunks*t + read_fill keys (>= 1 required,
 * read_fill <= R) and the cache is not modified.
 * workspace: device scratch of at least loma_decode_workspace_bytes(...) bytes for the
 * split-K partial results (may be NULL when that function returns 0).  Contents are
 * don't-care on entry and exit; calls sharing a workspace must be stream-ordered.
 * The result is deterministic (fixed combine order, no atomics).
 */
int loma_decode_attn(const void* q, const void* k_new, const void* v_new,
                     const void* k_memcache, const void* v_memcache,
                     void* k_read, void* v_read, void* out,
                     int B, int H, int head_dim, int t, int c,
                     int n_mem_chunks, int mem_capacity, int read_fill,
                     float scale, int dtype,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * The decode step for callers that cannot allocate device memory and hold no workspace of their
 * own: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and same result, bit for bit, as loma_decode_attn, without `workspace`: the split-K
 * partial results go to a fixed array inside the library's device image
 * (loma_decode_static_scratch_bytes() bytes, 4 MiB, held by every GPU the library runs on until
 * the process ends).  Nothing is allocated or freed, here or in any library it calls.  Shapes
 * whose partial results do not fit (loma_decode_workspace_bytes(...) above that size) return
 * LOMA_ERR_UNSUPPORTED and launch nothing.  The array's address on a device is looked up on the
 * first call made with that device current (make that call outside graph capture).  Every call on
 * a GPU shares that GPU's array; its contents are don't-care between calls (every slot read was
 * written by the same call), but calls that overlap in time on one GPU (different streams) race.
 */
int loma_decode_attn_static(const void* q, const void* k_new, const void* v_new,
                            const void* k_memcache, const void* v_memcache,
                            void* k_read, void* v_read, void* out,
                            int B, int H, int head_dim, int t, int c,
                            int n_mem_chunks, int mem_capacity, int read_fill,
                            float scale, int dtype, void* stream);
size_t loma_decode_static_scratch_bytes(void);

/*
 * The decode step for n_layers independent caches of one shape in ONE launch (Sec. 3.1 steps 1
 * and 3 applied to every layer's cache of a model: the per-token cost the method is after is the
 * sum over the layers, and at small batch a launch per layer costs as much as the step itself).
 * Every tensor argument of loma_decode_attn becomes a DEVICE array of n_layers device pointers
 * (8-byte aligned; entry l points at layer l's tensor, laid out as there; the arrays and the
 * tensors are caller-owned and not checked on the host); k_new and v_new are both arrays or
 * both NULL; k_memcache/v_memcache may be NULL when n_mem_chunks == 0.  B, H, head_dim, t, c and
 * the cache state (n_mem_chunks, mem_capacity, read_fill) are shared by the layers.  Layer l's
 * result and its appended K/V row are bit-identical to a loma_decode_attn call on its tensors.
 * workspace: at least loma_decode_layers_workspace_bytes(...) bytes (n_layers blocks of the
 * single-call size).  bf16 with head_dim 64 or 128 only (else LOMA_ERR_UNSUPPORTED).
 */
int loma_decode_attn_layers(const void* const* q, const void* const* k_new, const void* const* v_new,
                            const void* const* k_memcache, const void* const* v_memcache,
                            void* const* k_read, void* const* v_read, void* const* out,
                            int n_layers, int B, int H, int head_dim, int t, int c,
                            int n_mem_chunks, int mem_capacity, int read_fill,
                            float scale, int dtype,
                            void* workspace, size_t workspace_bytes, void* stream);
size_t loma_decode_layers_workspace_bytes(int n_layers, int B, int H, int head_dim, int t, int c,
                                          int n_mem_chunks, int dtype);

/*
 * The decode step with grouped-query attention: H query heads, H_kv <= H key/value heads, query head h
 * reads the cache of KV head h / (H / H_kv) (Sec. 3.1 steps 1 and 3 on the cache layout of models
 * other than the paper's Llama-2-7B, which the conclusion claims the method carries over to; the
 * compressed cache then holds H_kv heads and a step streams it once for the H / H_kv queries that
 * share a head).  Arguments as loma_decode_attn with: q, out DEVICE [B, H, head_dim]; k_new, v_new
 * DEVICE [B, H_kv, head_dim] or both NULL; k_memcache, v_memcache DEVICE [B, H_kv, mem_capacity,
 * head_dim]; k_read, v_read DEVICE [B, H_kv, t*c, head_dim] (row read_fill of every KV head is
 * written when k_new is given).  H must be H_kv times 1, 2, 4 or 8 and the data bf16 with head_dim
 * 64 or 128 (else LOMA_ERR_UNSUPPORTED).  workspace: at least loma_decode_gqa_workspace_bytes(...)
 * bytes, caller-owned, 16-byte aligned.  Deterministic: fixed split plan, fixed merge order.
 */
int loma_decode_attn_gqa(const void* q, const void* k_new, const void* v_new,
                         const void* k_memcache, const void* v_memcache,
                         void* k_read, void* v_read, void* out,
                         int B, int H, int H_kv, int head_dim, int t, int c,
                         int n_mem_chunks, int mem_capacity, int read_fill,
                         float scale, int dtype,
                         void* workspace, size_t workspace_bytes, void* stream);
size_t loma_decode_gqa_workspace_bytes(int B, int H, int H_kv, int head_dim, int dtype);

/*
 * loma_decode_attn_gqa for n_layers caches in ONE launch: the tensor arguments become DEVICE arrays of
 * n_layers device pointers as in loma_decode_attn_layers (same alignment and NULL rules), shapes per
 * layer as in loma_decode_attn_gqa.  Layer l's result and appended rows are bit-identical to a
 * loma_decode_attn_gqa call on its tensors.  workspace: at least n_layers times
 * loma_decode_gqa_workspace_bytes(...) bytes.
 */
int loma_decode_attn_gqa_layers(const void* const* q, const void* const* k_new, const void* const* v_new,
                                const void* const* k_memcache, const void* const* v_memcache,
                                void* const* k_read, void* const* v_read, void* const* out,
                                int n_layers, int B, int H, int H_kv, int head_dim, int t, int c,
                                int n_mem_chunks, int mem_capacity, int read_fill,
                                float scale, int dtype,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Position ids (Sec. 4.5, Eq. 14; Appendix A).  Host-only arithmetic on HOST arrays; launches nothing.
 * The text is cut into reading zones of R = t*c tokens; reading token j of chunk i keeps its original id
 * i*R + j.  The t memory tokens of chunk i (i = number of chunks compressed before it) take
 *   LOMA_POS_INTERMITTENT: i*R + c-1, i*R + 2c-1, ..., i*R + tc-1   (Eq. 14 read with chunk length tc: ids inside
 *                          the chunk, the last one adjacent to the next chunk's first reading id)
 *   LOMA_POS_CONTIGUOUS:   i*t, i*t + 1, ..., i*t + t-1             (the appendix's mem_cursor + j)
 * Both are arithmetic progressions: first id ids[0], step ids[1] - ids[0] (c or 1), which is how the *_rope entry
 * points take them.  The paper gives no ids for repetition tokens; loma_sample_position_ids gives repetition
 * token j the id of the reading token it reproduces, i*R + j.
 *   loma_memory_position_ids: ids[0..t)               of chunk `chunk`
 *   loma_sample_position_ids: ids[0..n_chunks*t(2c+1)) of a whole restructured sample, row by row
 */
int loma_memory_position_ids(int t, int c, int chunk, int position_type, int* ids);
int loma_sample_position_ids(int t, int c, int n_chunks, int position_type, int* ids);

/*
 * The decode and compression steps with the rotary position embedding applied as q and k are loaded (the
 * paper's model, Llama-2, rotates q and k by their position ids before the scores; Sec. 4.5 designs the ids).
 * Same arguments and semantics as loma_decode_attn / loma_compress_step, except that q (q_mem) and k_new
 * (k_mem) arrive UNROTATED and the caches hold rotated K: the appended / spliced K rows are the rotated ones,
 * rounded to bf16 once.  Convention: head-dim element i < d/2 pairs with element i + d/2 and the pair turns by
 * pos * rope_theta^(-2i/d) (Llama's "rotate-half" form).
 *   decode:   pos is the id of the new token (the appendix's cursor); q and k_new turn by it.
 *   compress: memory token j turns by pos_first + j * pos_stride (see the position-id helpers above).
 *             `out` is used as scratch for the rotated queries before the results overwrite it, so it must
 *             not alias q_mem.
 * bf16 with head_dim 64 or 128 only (else LOMA_ERR_UNSUPPORTED); rope_theta > 0 (Llama-2: 10000).
 */
int loma_decode_attn_rope(const void* q, const void* k_new, const void* v_new,
                          const void* k_memcache, const void* v_memcache,
                          void* k_read, void* v_read, void* out,
                          int B, int H, int head_dim, int t, int c,
                          int n_mem_chunks, int mem_capacity, int read_fill,
                          float scale, int dtype, int pos, float rope_theta,
                          void* workspace, size_t workspace_bytes, void* stream);
int loma_compress_step_rope(const void* q_mem, const void* k_mem, const void* v_mem,
                            const void* k_read, const void* v_read,
                            void* k_memcache, void* v_memcache, void* out,
                            int B, int H, int head_dim, int t, int c,
                            int n_mem_chunks, int mem_capacity,
                            float scale, int dtype,
                            int pos_first, int pos_stride, float rope_theta, void* stream);

/*
 * Generation form, several new tokens per sequence at once: a prompt or a piece of one
 * (Appendix A: add_token_ids / inference_input with more than one input token, whose
 * mask is the lower triangle shifted by the cache length; the cost model T_infer(l, k)
 * of Sec. 3.1).  Same state and same arguments as loma_decode_attn, with n_new rows:
 *
 *   q, k_new, v_new, out: [B, H, n_new, head_dim]   (k_new, v_new required)
 * New token i (0 <= i < n_new) attends over all n_mem_chunks*t memory keys, the
 * read_fill live reading-zone rows and new tokens 0..i (itself included): exactly what
 * n_new successive loma_decode_attn calls would give.  k_new/v_new are written to
 * reading-zone rows [read_fill, read_fill + n_new); the caller then sets
 * read_fill += n_new and calls loma_compress_step when the zone is full.
 * Requires 1 <= n_new and read_fill + n_new <= t*c (a longer prompt is fed in pieces
 * with compression steps in between, as the appendix's driver loop does).
 * lse (optional, may be NULL): [B, H, n_new] float.  No workspace; deterministic.
 */
int loma_prefill_attn(const void* q, const void* k_new, const void* v_new,
                      const void* k_memcache, const void* v_memcache,
                      void* k_read, void* v_read, void* out, float* lse,
                      int B, int H, int head_dim, int t, int c,
                      int n_mem_chunks, int mem_capacity, int read_fill, int n_new,
                      float scale, int dtype, void* stream);

/*
 * Bytes of workspace loma_decode_attn needs for this shape at ANY read_fill in [0, R]
 * (with or without k_new).  0 on invalid arguments.  Host-only arithmetic.
 */
size_t loma_decode_workspace_bytes(int B, int H, int head_dim, int t, int c,
                                   int n_mem_chunks, int dtype);

/*
 * Host-only view of the mask pass's tile schedule (Sec. 4.3 mask -> work list), for
 * inspection and tests; launches nothing.
 *   loma_mask_schedule_size: number of workgroups the MFMA mask-pass kernel launches
 *     for this shape (0 if the shape does not take that kernel).
 *   loma_mask_schedule_item: decodes workgroup `block` into
 *     item[0] = b*H + h, item[1] = chunk, item[2] = zone (0 read, 1 memory, 2 repetition),
 *     item[3] = first row of the zone handled, item[4] = number of rows handled,
 *     item[5] = number of keys it visits;  returns 1 if the workgroup has work, 0 if it
 *     is padding, negative on bad arguments.
 */
long long loma_mask_schedule_size(int B, int H, int head_dim, int t, int c, int n_chunks, int dtype);
int loma_mask_schedule_item(int B, int H, int head_dim, int t, int c, int n_chunks, int dtype,
                            long long block, int item[6]);

#ifdef __cplusplus
}
#endif
#endif /* LOMA_H_ */
