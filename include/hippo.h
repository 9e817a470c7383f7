/*
 * hippo.h -- C ABI of the MI355X (gfx950) implementation of HIPPO's data-parallel hot path:
 * semantic-aware visual-token scoring and selection, construction of the pruned draft KV cache,
 * and the two attention calls that video parallel speculative decoding overlaps (draft decode over
 * the pruned cache, target verification of gamma+1 tokens over the full cache).
 *
 * The hot path proper:   hippo_score_tokens, hippo_select_gather_kv, hippo_draft_attention,
 *                        hippo_verify_attention (+ hippo_workspace_bytes, hippo_status_string).
 * Built around it:       hippo_score_tokens_layers (Eq. 2's layer sum in one call),
 *                        hippo_*_attention_append, hippo_*_attention_paged and
 *                        hippo_*_attention_fp8kv with hippo_quantize_kv_e4m3 (cache-format variants),
 *                        hippo_spec_verify (the speculative-sampling verdict of Eq. 1),
 *                        hippo_vpsd_* (host-side control of the parallel decoding rounds).
 *
 * Conventions common to every entry point
 *  - All data pointers are DEVICE pointers owned and allocated by the caller.  The library never
 *    allocates or frees device memory and never synchronises: it validates its arguments on the
 *    host, enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *    and returns.  Outputs are valid once the caller has synchronised that stream.  Calls on
 *    different streams may run concurrently as long as their outputs and workspaces are distinct.
 *  - The descriptor structs are HOST pointers, read before the call returns.
 *  - Every call returns a status (HIPPO_OK = 0).  Validation happens before any kernel is
 *    launched: on a non-zero status nothing has been enqueued and no output was touched.  No
 *    exception crosses the boundary.
 *  - `workspace` is device scratch of at least hippo_workspace_bytes(...) bytes, 256-byte aligned,
 *    private to the call until the stream has passed it.
 *  - Data pointers must be 16-byte aligned; strides are in elements and must keep every row
 *    16-byte aligned (multiples of 8 for bf16, of 4 for fp32).  head_dim is 64 or 128.
 *  - dtype: HIPPO_DTYPE_F32 or HIPPO_DTYPE_BF16 for q / K / V / emb / attention outputs (plus the
 *    8-bit cache type of the *_fp8kv calls and the gather, see enum hippo_dtype).  Scores,
 *    attention mass and log-sum-exp are always fp32, indices int32.  Accumulation is fp32;
 *    bf16 outputs are rounded to nearest even.
 */
#ifndef HIPPO_H_
#define HIPPO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum hippo_status {
  HIPPO_OK = 0,
  HIPPO_ERR_NULL_ARG = 1,            /* a required pointer is NULL */
  HIPPO_ERR_BAD_SHAPE = 2,           /* a size, count, stride or index range is invalid */
  HIPPO_ERR_BAD_DTYPE = 3,           /* dtype is not one the call supports */
  HIPPO_ERR_BAD_ALIGN = 4,           /* a pointer or stride breaks the 16-byte rule */
  HIPPO_ERR_WORKSPACE_TOO_SMALL = 5, /* workspace_bytes below hippo_workspace_bytes(...) */
  HIPPO_ERR_HIP = 6,                 /* a HIP runtime call (launch) failed */
  HIPPO_ERR_STATIC_SCRATCH_LIMIT = 7 /* hippo_verify_attention_static: the shapes need more scratch
                                        than hippo_static_scratch_bytes() */
};

enum hippo_dtype {
  HIPPO_DTYPE_F32 = 0,
  HIPPO_DTYPE_BF16 = 1,
  /* 8-bit floating-point CACHE elements (E4M3, see hippo_verify_attention_fp8kv): one byte each.
   * Accepted by the *_fp8kv attention calls, by hippo_select_gather_kv (rows are byte copies) and by
   * hippo_workspace_bytes for those calls; every other call answers BAD_DTYPE. */
  HIPPO_DTYPE_FP8_E4M3 = 2
};

enum hippo_call {
  HIPPO_CALL_SCORE_TOKENS = 0,
  HIPPO_CALL_SELECT_GATHER_KV = 1,
  HIPPO_CALL_DRAFT_ATTENTION = 2,
  HIPPO_CALL_VERIFY_ATTENTION = 3
};

/* which terms of the holistic score are enabled (the paper's ablation removes one at a time) */
enum hippo_score_flags {
  HIPPO_SCORE_ATTN = 1u,            /* global semantic relevance, Eq. 2 */
  HIPPO_SCORE_TEMP = 2u,            /* inter-frame temporal redundancy, Eq. 3-4 */
  HIPPO_SCORE_SPA = 4u,             /* intra-frame spatial redundancy, Eq. 5-6 */
  HIPPO_SCORE_ALL = 7u,
  HIPPO_SCORE_ACCUMULATE_ONLY = 8u  /* add this layer's attention mass into attn_mass_inout and stop
                                       (the outer layer sum of Eq. 2); no other output is written */
};

/* A K or V cache (or the q/out heads that go with it).
 * Element (b, hk, n, c) of a cache lives at base + b*stride_b + hk*stride_h + n*stride_n + c. */
typedef struct hippo_kv_desc {
  int32_t batch;
  int32_t n_q_heads;   /* H; multiple of n_kv_heads.  Query head h reads KV head h / (H / H_kv) */
  int32_t n_kv_heads;  /* H_kv */
  int32_t head_dim;    /* d_k: 64 or 128 */
  int32_t dtype;       /* enum hippo_dtype */
  int64_t stride_b, stride_h, stride_n;  /* elements; stride_n >= head_dim */
} hippo_kv_desc;

/* Where the video sits inside the sequence and how its tokens are arranged.
 * Visual token j = f*grid_h*grid_w + y*grid_w + x is cache row vis_offset + j.
 * Crops (Eq. 5-6) are non-overlapping crop_h x crop_w tiles of each frame anchored at (0,0);
 * tiles cut by the right / bottom edge keep the tokens they have. */
typedef struct hippo_video_desc {
  int32_t n_frames, grid_h, grid_w;
  int32_t vis_offset;
  int32_t crop_h, crop_w;           /* the paper uses 5 x 5; crop_h*crop_w <= 64 */
} hippo_video_desc;

const char* hippo_status_string(int status);

/* Bytes of workspace `call` needs for these shapes; never 0 for valid arguments, 0 if they are
 * invalid.  n_rows = l_txt for SCORE_TOKENS, q_len for the attention calls, ignored otherwise;
 * seq_len = number of valid cache rows (ctx_len + q_len for attention); k = tokens kept (select);
 * num_splits as passed to the attention call (0 = library's choice). */
size_t hippo_workspace_bytes(int32_t call, const hippo_kv_desc* kv, const hippo_video_desc* vid,
                             int32_t n_rows, int32_t seq_len, int32_t k, int32_t num_splits);

/*
 * Semantic-aware token scoring (Method, "Semantic-aware Token Preservation", Eq. 2-7).
 *   s_attn[j] = 1/(H l_txt) sum_h sum_i softmax_j(q_txt[i,h] . K_vid[j] / sqrt(d_k))      (Eq. 2,
 *               softmax over the N_v visual keys; one layer per call)
 *   s_temp[j] = 1 - mean over existing neighbour frames f-1, f+1 of the cosine between token j and
 *               the token at the same grid position there (1 if the video has one frame) (Eq. 3-4)
 *   s_spa[j]  = population variance over the tokens k of j's crop of cos(emb_j, emb_k)    (Eq. 5-6)
 *   scores[j] = sum over enabled terms of (s - mean_f) / std_f, statistics per frame, population
 *               std, a term with std_f = 0 contributes 0                                   (Eq. 7)
 * A zero-norm embedding has cosine 0 with everything.
 *
 * q_txt   [B, l_txt, H, d] contiguous, dtype kv->dtype: the text-prompt queries.
 * k_cache the cache whose keys guide pruning; rows [vis_offset, vis_offset + N_v) are read.
 * emb     [B, N_v, emb_dim] with token stride emb_stride_tok (batch stride N_v*emb_stride_tok),
 *         dtype kv->dtype, or NULL: then token j's embedding is its key vectors of all KV heads
 *         concatenated in head order (emb_dim, emb_stride_tok ignored).
 * attn_mass_inout [B, N_v] fp32 or NULL.  If non-NULL it holds the sum of s_attn over the layers
 *         already processed; this call adds its layer's s_attn to it and, unless ACCUMULATE_ONLY is
 *         set, uses the accumulated value as the attention term (a positive factor such as 1/N_L
 *         does not change Eq. 7's normalised value).
 * scores_out [B, N_v] fp32 (required unless ACCUMULATE_ONLY).
 * components_out optional [3, B, N_v] fp32: raw s_attn (this call's, or accumulated), s_temp, s_spa.
 * Errors: NULL_ARG, BAD_SHAPE (l_txt < 1, N_v < 1, vis_offset + N_v > seq_len, crop too large,
 *         no term enabled; beyond the launch limits: B * layers > 65535, more than 65535 frames,
 *         bf16 with N_v > 65535 * 256 tokens), BAD_DTYPE, BAD_ALIGN, WORKSPACE_TOO_SMALL, HIP.
 */
int hippo_score_tokens(const void* q_txt, int32_t l_txt,
                       const void* k_cache, const hippo_kv_desc* kv, int32_t seq_len,
                       const hippo_video_desc* vid,
                       const void* emb, int32_t emb_dim, int64_t emb_stride_tok,
                       uint32_t flags,
                       float* attn_mass_inout, float* scores_out, float* components_out,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same with Eq. 2's outer sum over layers done inside the call: the attention term is
 * sum over the n_layers given layers of that layer's s_attn (queries and keys of layer l from
 * q_txt_layers[l], k_cache_layers[l]; all layers share kv's shape and strides), swept in ONE launch per
 * pass instead of one call per layer.  q_txt_layers and k_cache_layers are HOST arrays of n_layers
 * device pointers (1 <= n_layers <= 64), read before the call returns.  When emb is NULL the
 * embedding terms use the keys of layer emb_layer.  attn_mass_inout, if given, is added to (and
 * updated with) the call's layer sum, exactly as for single calls.  hippo_score_tokens is this call
 * with one layer.  Workspace: hippo_score_layers_workspace_bytes(kv, vid, l_txt, n_layers).
 */
size_t hippo_score_layers_workspace_bytes(const hippo_kv_desc* kv, const hippo_video_desc* vid,
                                          int32_t l_txt, int32_t n_layers);
int hippo_score_tokens_layers(int32_t n_layers, const void* const* q_txt_layers, int32_t l_txt,
                              const void* const* k_cache_layers, int32_t emb_layer,
                              const hippo_kv_desc* kv, int32_t seq_len, const hippo_video_desc* vid,
                              const void* emb, int32_t emb_dim, int64_t emb_stride_tok,
                              uint32_t flags,
                              float* attn_mass_inout, float* scores_out, float* components_out,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Top-k retention and draft-cache construction (Method, end of "Holistic Score Fusion": keep the
 * top-k visual tokens by score; App. "Details of Experimental Setups": the pruned video features
 * are removed from the draft model's input, everything that is not video is kept whole).
 *   idx_out[b, :] = the k visual-token indices with the largest scores[b, :], listed in ascending
 *                   index order.  Equal scores (-0 == +0): the lower index wins.  NaN ranks below
 *                   every number.
 *   dst rows      = src rows [0, vis_offset) | src rows vis_offset + idx_out[b, .] | src rows
 *                   [vis_offset + N_v, src_len), for K and V and every KV head, bit copies.
 * scores [B, N_v] fp32.  1 <= k <= N_v.  src/dst descriptors must agree in batch, n_kv_heads,
 * head_dim and dtype (strides may differ); dst holds src_len - N_v + k rows.  k_src/v_src may be a
 * different model's cache than the one that was scored, and may be an 8-bit cache
 * (HIPPO_DTYPE_FP8_E4M3: the kept rows' codes are copied; the per-head multipliers stay valid).  k_dst/v_dst may be NULL together to get
 * the indices only.  src and dst must not overlap.
 * Errors: NULL_ARG, BAD_SHAPE (k out of range, video span outside src_len, descriptor mismatch),
 *         BAD_DTYPE, BAD_ALIGN, WORKSPACE_TOO_SMALL, HIP.
 */
int hippo_select_gather_kv(const float* scores, int32_t k,
                           const void* k_src, const void* v_src, const hippo_kv_desc* src,
                           int32_t src_len, const hippo_video_desc* vid,
                           void* k_dst, void* v_dst, const hippo_kv_desc* dst,
                           int32_t* idx_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Target verification attention (Preliminaries, "Speculative Decoding": the target model takes the
 * prefix plus the gamma draft tokens and emits p_0..p_gamma; Method, "Adaptive Decoding Strategy
 * Switching": in conservative mode it verifies x_1 alone, so any q_len >= 1 is accepted).
 *   out[b, i, h, :] = sum_n softmax_n(softmax_scale * q[b,i,h,:] . K[b,h/G,n,:]) V[b,h/G,n,:],
 *   n in [0, ctx_len + i]   -- the cache already holds the q_len new rows' own K/V at rows
 *   ctx_len .. ctx_len + q_len - 1, and new row i sees the context and new rows 0..i.
 * q, out [B, q_len, H, d] contiguous, dtype kv->dtype.  lse_out optional [B, H, q_len] fp32: natural
 * log of the softmax denominator (of the scaled logits).  softmax_scale <= 0 means 1/sqrt(d).
 * num_splits: how many slices the KV range is cut into (flash-decoding style), 0 = library's
 * choice; the result does not depend on it beyond rounding (fp32 caches: fp32 throughout; 16- and 8-bit
 * caches: each slice's output reaches the merge rounded to bf16, its statistics in fp32).
 * ctx_len >= 0, q_len >= 1.
 * Errors: NULL_ARG, BAD_SHAPE, BAD_DTYPE, BAD_ALIGN, WORKSPACE_TOO_SMALL, HIP.
 */
int hippo_verify_attention(const void* q, int32_t q_len,
                           const void* k_cache, const void* v_cache, const hippo_kv_desc* kv,
                           int32_t ctx_len, float softmax_scale, int32_t num_splits,
                           void* out, float* lse_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Draft-decode attention over the pruned cache (Preliminaries, "Speculative Decoding": the draft
 * model is invoked gamma times, one new token per forward).  Same contract, arguments, kernels and
 * split heuristic as hippo_verify_attention (measured: the matrix-unit kernel padded to one 16-row
 * block beats the vector-ALU kernel 4-9 x at G = 7 or 8 rows); the one difference is that its waves
 * do not raise their issue priority, so a verification running beside it keeps the right of way.  Running it on
 * the cache hippo_select_gather_kv built with k = N_v equals attention over the unpruned cache.
 */
int hippo_draft_attention(const void* q, int32_t q_len,
                          const void* k_cache, const void* v_cache, const hippo_kv_desc* kv,
                          int32_t ctx_len, float softmax_scale, int32_t num_splits,
                          void* out, float* lse_out,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * hippo_verify_attention for callers that can neither allocate device memory nor pass a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, result and errors as hippo_verify_attention minus the workspace pair; the split partials
 * live in an array that is part of the library's device image (hippo_static_scratch_bytes() = 8 MiB on
 * every GPU the library is used on, held until the process ends).  The call allocates and frees
 * nothing.  Shapes whose partials exceed the array (hippo_workspace_bytes(HIPPO_CALL_VERIFY_ATTENTION,
 * ...) > hippo_static_scratch_bytes(), e.g. many sequences with num_splits forced high) are refused
 * with HIPPO_ERR_STATIC_SCRATCH_LIMIT before anything is enqueued.  Every call on a GPU uses that
 * GPU's one array: calls must not overlap in time on one GPU (same stream, or ordered by events), or
 * they race.  Nothing in the array has to be cleared between calls, whatever the previous call left.
 * The array's device address is looked up on the first call on each device; hippo_static_scratch_init()
 * does that lookup for the current device ahead of time (call it before capturing a graph).
 */
size_t hippo_static_scratch_bytes(void);
int hippo_static_scratch_init(void);
int hippo_verify_attention_static(const void* q, int32_t q_len,
                                  const void* k_cache, const void* v_cache, const hippo_kv_desc* kv,
                                  int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                  void* out, float* lse_out, void* stream);

/*
 * The same two attention calls with the append of the new rows folded in (a cache-format variant for
 * decode loops: the gamma+1 rows the target verifies, or the one row the draft model decodes, come
 * straight from the K/V projection and would otherwise need a copy kernel of their own before the
 * attention launch).  k_new, v_new [B, q_len, H_kv, d] contiguous, dtype kv->dtype: the new rows'
 * keys and values.  The result is exactly that of hippo_verify_attention / hippo_draft_attention on
 * a cache whose rows ctx_len .. ctx_len + q_len - 1 hold them; the call also WRITES those rows into
 * k_cache / v_cache (bit copies), so the next call finds them there.  Rows below ctx_len are read
 * only.  k_new / v_new must not overlap the caches.  Everything else as above.
 * Errors: as above, plus NULL_ARG / BAD_ALIGN for k_new, v_new.
 */
int hippo_verify_attention_append(const void* q, int32_t q_len, const void* k_new, const void* v_new,
                                  void* k_cache, void* v_cache, const hippo_kv_desc* kv,
                                  int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                  void* out, float* lse_out,
                                  void* workspace, size_t workspace_bytes, void* stream);
int hippo_draft_attention_append(const void* q, int32_t q_len, const void* k_new, const void* v_new,
                                 void* k_cache, void* v_cache, const hippo_kv_desc* kv,
                                 int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                 void* out, float* lse_out,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same two attention calls over a cache stored in 8-bit floating point (a cache-format variant
 * the paper does not discuss: it halves the bytes these bandwidth-bound calls stream).  k_codes /
 * v_codes hold E4M3 codes (1 sign, 4 exponent, 3 mantissa bits, bias 7, finite-only: no infinities,
 * 0x7f / 0xff are NaN), one byte per element, laid out as kv describes with strides counted in
 * elements = bytes (multiples of 16).  k_scale / v_scale are DEVICE arrays [B, H_kv] of fp32
 * multipliers, all > 0: the cache entry is multiplier * decoded code.  kv->dtype must be
 * HIPPO_DTYPE_FP8_E4M3, the type of the cache; q and out are bf16.  The result is that of hippo_verify_attention /
 * hippo_draft_attention on the dequantised cache, computed with the same arithmetic as the bf16 path
 * (codes convert to bf16 exactly; the K multiplier joins the softmax scale, the V multiplier the
 * output).  Workspace: hippo_workspace_bytes with the same kv.  Caches are read only.
 * Errors: as hippo_verify_attention, plus NULL_ARG for the multipliers, BAD_DTYPE for any other
 * cache type.
 */
int hippo_verify_attention_fp8kv(const void* q, int32_t q_len, const void* k_codes, const void* v_codes,
                                 const float* k_scale, const float* v_scale, const hippo_kv_desc* kv,
                                 int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                 void* out, float* lse_out,
                                 void* workspace, size_t workspace_bytes, void* stream);
int hippo_draft_attention_fp8kv(const void* q, int32_t q_len, const void* k_codes, const void* v_codes,
                                const float* k_scale, const float* v_scale, const hippo_kv_desc* kv,
                                int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                void* out, float* lse_out,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Writer of that 8-bit cache format: rows [0, n_rows) of a bf16 or fp32 cache become E4M3 codes and
 * one multiplier per (batch element, KV head), separately for K and V:
 *     multiplier = max|x| / 448 over the head's n_rows x d entries (fp32; 1 when the maximum is 0)
 *     code       = the E4M3 value nearest to x / multiplier (fp32 division), ties to the even code
 * so the largest entry of every head maps to the largest code and nothing overflows.  src describes
 * k_src / v_src (dtype F32 or BF16), dst the code arrays (dtype FP8_E4M3, strides in bytes); both
 * agree in batch, n_kv_heads, head_dim.  k_scale / v_scale [B, H_kv] fp32 are OUTPUTS.  Inputs must
 * be finite (a NaN or infinity gives unspecified codes for its head).  Deterministic.  Workspace:
 * hippo_quantize_kv_workspace_bytes(src, n_rows).
 * Errors: NULL_ARG, BAD_DTYPE, BAD_SHAPE (descriptor mismatch, n_rows < 1), BAD_ALIGN,
 *         WORKSPACE_TOO_SMALL, HIP.
 */
size_t hippo_quantize_kv_workspace_bytes(const hippo_kv_desc* src, int32_t n_rows);
int hippo_quantize_kv_e4m3(const void* k_src, const void* v_src, const hippo_kv_desc* src, int32_t n_rows,
                           void* k_codes, void* v_codes, const hippo_kv_desc* dst,
                           float* k_scale, float* v_scale,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same two attention calls over a PAGED cache (a cache-format variant for serving stacks that
 * allocate the cache in fixed-size pages).  k_pool / v_pool are page pools; cache row n of sequence
 * b and KV head hk lives at element
 *     block_table[b * max_pages + n / page_size] * stride_page + (n % page_size) * stride_n + hk * stride_h
 * (+ c for head-dim element c), e.g. a [n_pool_pages, page_size, H_kv, d] pool has stride_page =
 * page_size * H_kv * d, stride_n = H_kv * d, stride_h = d.  block_table is a DEVICE array of int32,
 * [B, max_pages]; entries outside [0, n_pool_pages) are clamped into the pool (the result is then
 * meaningless, but no access leaves the pool).  page_size is a power of two, 16..256.  The result
 * is bit-identical to the contiguous call on the same rows.  A block stages the page numbers of its
 * KV slice in LDS, which bounds a slice to about 1000 pages: with num_splits forced very low on a
 * long cache the call returns BAD_SHAPE.  Use hippo_workspace_bytes with a hippo_kv_desc of the same
 * batch / heads / head_dim / dtype for the workspace size.
 * Errors: as hippo_verify_attention, plus BAD_SHAPE for a page size, table width or pool size
 * that does not fit, BAD_ALIGN for strides that break the 16-byte rule.
 */
typedef struct hippo_paged_kv_desc {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, dtype;
  int32_t page_size;        /* tokens per page */
  int32_t max_pages;        /* columns of block_table; >= ceil((ctx_len + q_len) / page_size) */
  int32_t n_pool_pages;     /* pages in the pool */
  int64_t stride_page, stride_n, stride_h;   /* elements */
} hippo_paged_kv_desc;

int hippo_verify_attention_paged(const void* q, int32_t q_len, const void* k_pool, const void* v_pool,
                                 const int32_t* block_table, const hippo_paged_kv_desc* kv,
                                 int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                 void* out, float* lse_out,
                                 void* workspace, size_t workspace_bytes, void* stream);
int hippo_draft_attention_paged(const void* q, int32_t q_len, const void* k_pool, const void* v_pool,
                                const int32_t* block_table, const hippo_paged_kv_desc* kv,
                                int32_t ctx_len, float softmax_scale, int32_t num_splits,
                                void* out, float* lse_out,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Speculative-sampling verification of one chain of gamma draft tokens per sequence
 * (Preliminaries, "Speculative Decoding": Eq. 1, the resampling rule below it, and the extra token
 * after a full acceptance; Method, "Adaptive Decoding Strategy Switching": conservative mode
 * verifies x_1 alone, i.e. gamma = 1).
 *   p_i = softmax(p_logits[b, i, :] / temperature), i = 0..gamma    target rows
 *   q_i = softmax(q_logits[b, i, :] / temperature), i = 0..gamma-1  draft rows; draft token
 *         x_i = draft_tokens[b, i] was sampled from q_i and is verified against p_i
 *   alpha_i = 1 if p_i[x_i] >= q_i[x_i] else p_i[x_i] / q_i[x_i]                          (Eq. 1)
 *   token i is accepted iff u_accept[b, i] < alpha_i; n_accept_out[b] = j = the first rejected
 *   position (gamma if none).  next_token_out[b] is drawn with u_sample[b] from
 *   max(0, p_j - q_j) / sum (from p_j if that sum is 0) after a rejection, from p_gamma otherwise:
 *   the first word t whose running sum r_0 + .. + r_t exceeds u_sample * sum(r), in index order.
 *   The caller emits x_0 .. x_{j-1} followed by next_token.
 * temperature == 0 is greedy decoding (the paper's evaluation setting): p_i is one-hot at the first
 *   maximum of its row, q_i one-hot at x_i, so alpha_i = [x_i == argmax p_i] and next_token is the
 *   argmax of row j; q_logits, u_accept and u_sample are not read and may be NULL.
 * alpha_out (optional) [B, gamma] fp32: alpha_i for every position, also after the first rejection.
 * A draft token outside [0, vocab) is rejected (alpha 0).  Logits may be -inf (masked words) but
 * not NaN or +inf, and every row needs a finite entry.  The uniforms are the caller's, in [0, 1).
 *
 * p_logits [B, gamma+1, p_stride_row], q_logits [B, gamma, q_stride_row], dtype F32 or BF16, row
 * strides in elements, >= vocab and keeping rows 16-byte aligned; the first `vocab` entries of a
 * row are read.  draft_tokens [B, gamma] int32, u_accept [B, gamma] fp32, u_sample [B] fp32,
 * outputs int32 [B].  0 <= gamma <= 64 (gamma = 0 just draws from p_0), vocab <= 2^20.
 * Sums are fp32; a word that the exact arithmetic would draw can be replaced by a neighbour in
 * the running sum only when u_sample * sum lies within fp32 rounding of the boundary between them.
 * Errors: NULL_ARG, BAD_SHAPE, BAD_DTYPE, BAD_ALIGN, WORKSPACE_TOO_SMALL, HIP.
 */
size_t hippo_spec_verify_workspace_bytes(int32_t batch, int32_t gamma, int32_t vocab, int32_t dtype);
int hippo_spec_verify(const void* p_logits, const void* q_logits, int32_t dtype,
                      int64_t p_stride_row, int64_t q_stride_row,
                      const int32_t* draft_tokens, const float* u_accept, const float* u_sample,
                      int32_t batch, int32_t gamma, int32_t vocab, float temperature,
                      int32_t* n_accept_out, int32_t* next_token_out, float* alpha_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Host-side control of video parallel speculative decoding (Method, "Video Parallel Speculative
 * Decoding").  No device work and no device pointers: every argument here is a HOST pointer.
 *
 * A round launches one target verification and, concurrently on another stream, draft decoding:
 *   optimistic mode   (the previous batch was fully accepted, or a prefill buffer exists): the target
 *                     verifies all n_pending buffered draft tokens while the draft model generates the
 *                     next gamma.  Full acceptance emits the verified tokens and the new batch becomes
 *                     the buffer (the extra token of serial speculative decoding is not taken: the draft
 *                     has already continued past it).  A rejection emits the accepted prefix plus the
 *                     target's replacement and discards every other draft; mode becomes conservative.
 *   conservative mode (a rejection occurred, nothing buffered): the draft model generates x_1; then
 *                     the target verifies x_1 alone while the draft generates x_2..x_gamma.  If x_1
 *                     is rejected drafting is aborted, the replacement is emitted and the mode stays;
 *                     if accepted, x_1 is emitted, x_2..x_gamma become the buffer and the mode becomes
 *                     optimistic.
 * (The paper fixes neither what happens to the extra token in the parallel modes nor how many
 * buffered tokens one verification takes; the above is this library's reading.)
 */
enum hippo_vpsd_mode { HIPPO_VPSD_CONSERVATIVE = 0, HIPPO_VPSD_OPTIMISTIC = 1 };
enum hippo_vpsd_policy { HIPPO_POLICY_AUTOREGRESSIVE = 0, HIPPO_POLICY_SERIAL_SD = 1, HIPPO_POLICY_VPSD = 2 };

typedef struct hippo_vpsd_state {
  int32_t gamma;            /* draft tokens per batch, 1..64 */
  int32_t mode;             /* enum hippo_vpsd_mode */
  int32_t n_pending;        /* drafted tokens waiting for verification */
  int32_t reserved;
  int64_t n_emitted;        /* tokens committed to the output so far */
  int64_t n_rounds, n_target_calls;
  int64_t n_draft_tokens;   /* draft forward passes so far (prefill buffer included) */
  int64_t n_draft_wasted;   /* draft tokens generated and then discarded */
  int64_t n_mode_switches;
} hippo_vpsd_state;

typedef struct hippo_vpsd_round {
  int32_t mode;             /* the mode this round runs in */
  int32_t draft_serial;     /* draft tokens to generate BEFORE the parallel phase (1 in conservative mode) */
  int32_t verify_len;       /* draft tokens the target verifies: hippo_verify_attention q_len = verify_len + 1,
                               hippo_spec_verify gamma = verify_len */
  int32_t draft_parallel;   /* draft tokens to generate concurrently with that verification */
} hippo_vpsd_round;

typedef struct hippo_vpsd_result {
  double time;              /* modelled wall time, in the unit of t_draft / t_target */
  double speedup;           /* n_emitted * t_target / time: against one target forward per token */
  int64_t n_emitted, n_rounds, n_target_calls, n_draft_tokens, n_draft_wasted, n_mode_switches;
  int64_t n_flags_used;
} hippo_vpsd_result;

/* Tokens the draft model can decode while the target model is still in prefill ("Synchronous
 * Draft-Target Prefill"): floor((t_prefill_target - t_prefill_draft) / t_draft_token), 0 if the
 * target is not slower; the paper's example (0.8 s, 0.2 s, 50 ms) gives 12.  -1 on invalid times. */
int32_t hippo_vpsd_prefill_buffer(double t_prefill_target, double t_prefill_draft, double t_draft_token);

/* Start of generation: n_prefill_buffer (0..64) draft tokens already buffered; optimistic if any. */
int hippo_vpsd_init(hippo_vpsd_state* state, int32_t gamma, int32_t n_prefill_buffer);
/* What to enqueue in the next round.  Does not change the state. */
int hippo_vpsd_plan(const hippo_vpsd_state* state, hippo_vpsd_round* round_out);
/* Account for the round's outcome: n_accept in [0, verify_len] as hippo_spec_verify reports it,
 * n_drafted_parallel = draft tokens actually produced concurrently (= draft_parallel unless
 * drafting was cut short by a rejection).  Errors: NULL_ARG, BAD_SHAPE (a round that is not the
 * one planned for this state, counts out of range, a fully accepted round whose new batch is
 * incomplete). */
int hippo_vpsd_commit(hippo_vpsd_state* state, const hippo_vpsd_round* round, int32_t n_accept,
                      int32_t n_drafted_parallel);

/* Timing model of a generation of at least n_tokens tokens under `policy`, with one draft forward
 * costing t_draft, one target forward (any verify width: it is memory-bound) t_target, and the
 * i-th verified draft token accepted iff accept[i] != 0 (flags beyond n_flags count as accepted;
 * one flag is consumed per token looked at, the rejected one included).
 *   AUTOREGRESSIVE: n_tokens target forwards.
 *   SERIAL_SD: per round gamma draft forwards, then one verification; emits n_accept + 1 tokens
 *     (Motivated Experiments, "Non-negligible Draft Latency": with t_target = 3 t_draft and gamma = 3
 *     the speedup is 2 when everything is accepted and 0.5 when every first token is rejected).
 *   VPSD: the state machine above; a fully accepted round costs draft_serial * t_draft +
 *     max(t_target, draft_parallel * t_draft), a round with a rejection draft_serial * t_draft +
 *     t_target (drafting is cut when the verdict arrives). */
int hippo_vpsd_simulate(int32_t policy, int32_t gamma, double t_draft, double t_target,
                        int32_t n_prefill_buffer, const uint8_t* accept, int64_t n_flags,
                        int64_t n_tokens, hippo_vpsd_result* result_out);

#ifdef __cplusplus
}
#endif
#endif /* HIPPO_H_ */
