// extern "C" boundary: argument validation, launch heuristics and workspace carving.  No kernel
// lives here.  Every check runs before the first launch, so a non-zero status means nothing was
// enqueued.
#include <math.h>

#include <atomic>

#include "common.h"

using namespace hippo;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int elem_bytes(int dtype) {
  return dtype == HIPPO_DTYPE_FP8_E4M3 ? 1 : (dtype == HIPPO_DTYPE_BF16 ? 2 : 4);
}

// allow_fp8: the call takes 8-bit caches (the fp8 attention calls, the gather, their workspace query)
int check_kv(const hippo_kv_desc* kv, bool allow_fp8 = false) {
  if (kv == nullptr) return HIPPO_ERR_NULL_ARG;
  if (kv->dtype != HIPPO_DTYPE_F32 && kv->dtype != HIPPO_DTYPE_BF16 &&
      !(allow_fp8 && kv->dtype == HIPPO_DTYPE_FP8_E4M3))
    return HIPPO_ERR_BAD_DTYPE;
  if (kv->batch < 1 || kv->n_kv_heads < 1 || kv->n_q_heads < 1) return HIPPO_ERR_BAD_SHAPE;
  if (kv->n_q_heads % kv->n_kv_heads != 0) return HIPPO_ERR_BAD_SHAPE;
  if (kv->head_dim != 64 && kv->head_dim != 128) return HIPPO_ERR_BAD_SHAPE;
  if (kv->stride_n < kv->head_dim || kv->stride_h < 0 || kv->stride_b < 0) return HIPPO_ERR_BAD_SHAPE;
  if (kv->stride_n > (1ll << 24)) return HIPPO_ERR_BAD_SHAPE;   // row offsets inside a tile stay 32-bit
  if (kv->batch > 65535 || kv->n_kv_heads > 65535) return HIPPO_ERR_BAD_SHAPE;
  const int per16 = 16 / elem_bytes(kv->dtype);
  if (kv->stride_n % per16 || kv->stride_h % per16 || kv->stride_b % per16) return HIPPO_ERR_BAD_ALIGN;
  return HIPPO_OK;
}

int check_video(const hippo_video_desc* v) {
  if (v == nullptr) return HIPPO_ERR_NULL_ARG;
  if (v->n_frames < 1 || v->grid_h < 1 || v->grid_w < 1 || v->vis_offset < 0) return HIPPO_ERR_BAD_SHAPE;
  if ((long long)v->n_frames * v->grid_h * v->grid_w > (1ll << 30)) return HIPPO_ERR_BAD_SHAPE;
  if (v->n_frames > 65535) return HIPPO_ERR_BAD_SHAPE;   // frames are a y dimension of the crop kernels' grids
  return HIPPO_OK;
}

// ---- attention planning -------------------------------------------------------------------------
struct AttnPlan {
  bool mfma;
  int R, row_chunk, n_chunks, S;
  size_t off_m, off_l, bytes;
};

int plan_attention(int call, const hippo_kv_desc* kv, int q_len, int n_total, int num_splits, AttnPlan* pl) {
  (void)call;   // draft and verify share one launch heuristic (they differ in wave priority only)
  if (q_len < 1 || n_total < q_len || num_splits < 0) return HIPPO_ERR_BAD_SHAPE;
  const int G = kv->n_q_heads / kv->n_kv_heads;
  if ((long long)G * q_len > 4096) return HIPPO_ERR_BAD_SHAPE;
  pl->R = G * q_len;
  pl->mfma = kv->dtype != HIPPO_DTYPE_F32;   // bf16 and 8-bit caches
  int tile, min_tiles_per_block;
  if (pl->mfma) {
    pl->row_chunk = pl->R >= 64 ? 64 : (pl->R + 15) / 16 * 16;
    tile = 32;
    min_tiles_per_block = 1;     // short caches are bound by latency, not bytes: thin slices on many compute
                                 // units win (1896 rows, 7 query rows: 59 slices of 32 rows beat 14 of 128 by 9 %)
  } else {
    pl->row_chunk = 32;
    tile = 32;
    min_tiles_per_block = 2;
  }
  pl->n_chunks = (pl->R + pl->row_chunk - 1) / pl->row_chunk;
  if ((long long)kv->batch * pl->n_chunks > 65535) return HIPPO_ERR_BAD_SHAPE;
  const int n_tiles = (n_total + tile - 1) / tile;
  int S = num_splits;
  if (S == 0) {
    // one block per compute unit (measured at the 16K configuration: 48 or 80-128 slices per KV head
    // are all slower than 64), but never slices thinner than one 32-token tile
    const long long per_split = (long long)kv->batch * kv->n_kv_heads * pl->n_chunks;
    S = (int)(kNumCU / per_split);          // rounded down: a block beyond the last compute unit would share one
    if (S < 1) S = 1;
    const int cap = n_tiles / min_tiles_per_block;
    if (S > cap) S = cap;
  }
  if (S > n_tiles) S = n_tiles;
  if (S < 1) S = 1;
  if (S > 1024) S = 1024;
  pl->S = S;
  const size_t slots = (size_t)kv->batch * kv->n_kv_heads * S;
  // the MFMA kernel hands its slices' outputs to the merge as bf16, the vector-ALU kernel as fp32
  const size_t o_bytes = align_up(slots * pl->R * kv->head_dim * (pl->mfma ? 2 : sizeof(float)), 256);
  const size_t ml_bytes = align_up(slots * pl->R * sizeof(float), 256);
  pl->off_m = o_bytes;
  pl->off_l = o_bytes + ml_bytes;
  pl->bytes = o_bytes + 2 * ml_bytes;
  return HIPPO_OK;
}

// what the cache-format variants add to a plain attention call
struct AttnExtra {
  bool append = false;
  const void* k_new = nullptr;
  const void* v_new = nullptr;
  const int32_t* block_table = nullptr;     // paged
  int page_size = 0, max_pages = 0, n_pool_pages = 0;
  long long page_stride = 0;
  bool fp8 = false;                         // E4M3 cache with per-(b, hk) multipliers
  const float* k_scale = nullptr;
  const float* v_scale = nullptr;
};

int attention_entry(int call, const void* q, int32_t q_len, const void* k_cache, const void* v_cache,
                    const hippo_kv_desc* kv, int32_t ctx_len, float softmax_scale, int32_t num_splits,
                    void* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream,
                    const AttnExtra& ex = AttnExtra()) {
  const bool append = ex.append;
  const void* k_new = ex.k_new;
  const void* v_new = ex.v_new;
  if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr || workspace == nullptr)
    return HIPPO_ERR_NULL_ARG;
  if (append && (k_new == nullptr || v_new == nullptr)) return HIPPO_ERR_NULL_ARG;
  if (ex.fp8 && (ex.k_scale == nullptr || ex.v_scale == nullptr)) return HIPPO_ERR_NULL_ARG;
  int rc = check_kv(kv, ex.fp8);
  if (rc != HIPPO_OK) return rc;
  if (ex.fp8 != (kv->dtype == HIPPO_DTYPE_FP8_E4M3)) return HIPPO_ERR_BAD_DTYPE;
  if (ctx_len < 0 || q_len < 1 || (long long)ctx_len + q_len > 0x7fffff00ll) return HIPPO_ERR_BAD_SHAPE;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return HIPPO_ERR_BAD_ALIGN;
  if (append && (!aligned16(k_new) || !aligned16(v_new))) return HIPPO_ERR_BAD_ALIGN;
  AttnPlan pl;
  rc = plan_attention(call, kv, q_len, ctx_len + q_len, num_splits, &pl);
  if (rc != HIPPO_OK) return rc;
  if (workspace_bytes < pl.bytes) return HIPPO_ERR_WORKSPACE_TOO_SMALL;
  int page_shift = 0;
  if (ex.block_table != nullptr) {
    while ((1 << page_shift) < ex.page_size) ++page_shift;
    // a block keeps the page numbers of its slice in LDS: bound the slice (32-token tiles, a ragged
    // tile at either end) by the staging area
    const long long tiles32 = ((long long)ctx_len + q_len + 31) / 32;
    const long long slice_tokens = (tiles32 / pl.S + 2) * 32;
    if (slice_tokens / ex.page_size + 2 > kMaxSlicePages) return HIPPO_ERR_BAD_SHAPE;
  }

  AttnParams p;
  p.q = q; p.k = k_cache; p.v = v_cache; p.out = out; p.lse = lse_out;
  p.part_o = workspace;
  p.part_m = reinterpret_cast<float*>(static_cast<char*>(workspace) + pl.off_m);
  p.part_l = reinterpret_cast<float*>(static_cast<char*>(workspace) + pl.off_l);
  p.B = kv->batch; p.q_len = q_len; p.H = kv->n_q_heads; p.Hkv = kv->n_kv_heads;
  p.G = kv->n_q_heads / kv->n_kv_heads; p.R = pl.R;
  p.ctx_len = ctx_len; p.n_total = ctx_len + q_len;
  p.sb = kv->stride_b; p.sh = kv->stride_h; p.sn = kv->stride_n;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)kv->head_dim);
  p.scale_log2 = scale * kLog2e;
  p.S = pl.S; p.row_chunk = pl.row_chunk; p.n_chunks = pl.n_chunks;
  p.wave_prio = call == HIPPO_CALL_VERIFY_ATTENTION ? 1 : 0;
  p.phase_per_head = 1.0f / (float)((long long)kv->batch * kv->n_kv_heads);
  p.k_new = append ? k_new : nullptr; p.v_new = append ? v_new : nullptr;
  p.k_w = const_cast<void*>(k_cache); p.v_w = const_cast<void*>(v_cache);
  p.block_table = ex.block_table; p.page_shift = page_shift; p.max_pages = ex.max_pages;
  p.n_pool_pages = ex.n_pool_pages; p.page_stride = ex.page_stride;
  p.k_scale = ex.fp8 ? ex.k_scale : nullptr; p.v_scale = ex.fp8 ? ex.v_scale : nullptr;
  // q and out of the 8-bit cache calls are bf16
  const int io_dtype = ex.fp8 ? (int)HIPPO_DTYPE_BF16 : kv->dtype;
  const hipError_t e = launch_attention(p, io_dtype, kv->head_dim, pl.mfma, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HIPPO_OK : HIPPO_ERR_HIP;
}

// ---- scoring planning ---------------------------------------------------------------------------
struct ScorePlan {
  int n_tile, n_rsplit;
  size_t off_row_l, off_row_lse, off_col, off_sa, off_st, off_ss, bytes;
};

int plan_score(const hippo_kv_desc* kv, const hippo_video_desc* vid, int l_txt, int n_layers, ScorePlan* pl) {
  if (l_txt < 1 || l_txt > (1 << 20)) return HIPPO_ERR_BAD_SHAPE;
  if (n_layers < 1 || n_layers > kMaxScoreLayers || (long long)kv->batch * n_layers > 65535) return HIPPO_ERR_BAD_SHAPE;
  const long long Nv = (long long)vid->n_frames * vid->grid_h * vid->grid_w;
  const int tile = score_token_tile(kv->dtype);
  pl->n_tile = (int)((Nv + tile - 1) / tile);
  if (pl->n_tile > 0x7fffffff / 2) return HIPPO_ERR_BAD_SHAPE;
  const size_t rows = (size_t)kv->batch * n_layers * kv->n_q_heads * l_txt;
  const size_t row_part = align_up(rows * pl->n_tile * sizeof(float), 256);
  const size_t row_lse = align_up(rows * sizeof(float), 256);
  pl->n_rsplit = score_row_splits(kv->dtype, (long long)pl->n_tile * kv->n_kv_heads * kv->batch * n_layers,
                                  l_txt * (kv->n_q_heads / kv->n_kv_heads));
  // launch limits of the sweeps (key tiles on grid y, row runs x (layer, batch element) on grid z; the
  // vector-ALU sweeps put KV heads on y) and of the row merge (32 rows per block)
  if (pl->n_tile > 65535 || (long long)kv->batch * n_layers * pl->n_rsplit > 65535 || kv->n_kv_heads > 65535 ||
      rows / 32 >= (1ull << 31))
    return HIPPO_ERR_BAD_SHAPE;
  const size_t col = align_up((size_t)kv->batch * n_layers * kv->n_kv_heads * pl->n_rsplit * Nv * sizeof(float), 256);
  const size_t vec = align_up((size_t)kv->batch * Nv * sizeof(float), 256);
  size_t o = 0;
  o += row_part;            pl->off_row_l = o;
  o += row_part;            pl->off_row_lse = o;
  o += row_lse;             pl->off_col = o;
  o += col;                 pl->off_sa = o;
  o += vec;                 pl->off_st = o;
  o += vec;                 pl->off_ss = o;
  o += vec;                 pl->bytes = o;
  return HIPPO_OK;
}

int check_crop(const hippo_video_desc* vid) {
  if (vid->crop_h < 1 || vid->crop_w < 1 || (long long)vid->crop_h * vid->crop_w > 64) return HIPPO_ERR_BAD_SHAPE;
  return HIPPO_OK;
}

// ---- speculative-sampling verification planning -------------------------------------------------
struct SpecPlan {
  int n_seg, n_rows;
  size_t off_cells, off_chosen, bytes;
};

int plan_spec(int batch, int gamma, int vocab, int dtype, SpecPlan* pl) {
  if (dtype != HIPPO_DTYPE_F32 && dtype != HIPPO_DTYPE_BF16) return HIPPO_ERR_BAD_DTYPE;
  if (batch < 1 || batch > 65535 || gamma < 0 || gamma > kSdMaxGamma || vocab < 1 || vocab > kSdMaxVocab)
    return HIPPO_ERR_BAD_SHAPE;
  pl->n_seg = (vocab + kSdSeg - 1) / kSdSeg;
  pl->n_rows = 2 * gamma + 1;
  const size_t stats = align_up((size_t)batch * pl->n_rows * pl->n_seg * sizeof(SegStat), 256);
  const size_t cells = align_up((size_t)batch * 2 * pl->n_seg * spec_cells_per_segment(dtype) * sizeof(float), 256);
  pl->off_cells = stats;
  pl->off_chosen = stats + cells;
  pl->bytes = stats + cells + align_up((size_t)batch * sizeof(Chosen), 256);
  return HIPPO_OK;
}

}  // namespace

// ---- scratch for callers that cannot allocate -----------------------------------------------------
// One array per GPU, part of the loaded code object: it exists from the moment the library is loaded on
// a device until the process ends.  In host code the name `scratch` is only a handle for the runtime's
// symbol lookup, never an address a kernel could use; the per-device address comes from
// hipGetSymbolAddress and is what every launch receives.
constexpr size_t kStaticScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // zero-initialised: not looked up yet

// address of the current device's copy of the array (looked up once per device), or null with *status set
void* static_scratch(int* status) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *status = HIPPO_ERR_HIP;
    return nullptr;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      *status = HIPPO_ERR_HIP;
      return nullptr;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // every thread finds the same address
  }
  *status = HIPPO_OK;
  return ptr;
}

}  // namespace

extern "C" {

const char* hippo_status_string(int status) {
  switch (status) {
    case HIPPO_OK: return "ok";
    case HIPPO_ERR_NULL_ARG: return "a required pointer is NULL";
    case HIPPO_ERR_BAD_SHAPE: return "invalid size, count, stride or index range";
    case HIPPO_ERR_BAD_DTYPE: return "unsupported dtype";
    case HIPPO_ERR_BAD_ALIGN: return "pointer or stride is not 16-byte aligned (workspace: 256)";
    case HIPPO_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than hippo_workspace_bytes()";
    case HIPPO_ERR_HIP: return "HIP runtime error at kernel launch";
    case HIPPO_ERR_STATIC_SCRATCH_LIMIT:
      return "the call needs more scratch than the library's static array holds (hippo_static_scratch_bytes())";
    default: return "unknown status";
  }
}

size_t hippo_workspace_bytes(int32_t call, const hippo_kv_desc* kv, const hippo_video_desc* vid,
                             int32_t n_rows, int32_t seq_len, int32_t k, int32_t num_splits) {
  (void)k;
  if (check_kv(kv, call != HIPPO_CALL_SCORE_TOKENS) != HIPPO_OK) return 0;
  switch (call) {
    case HIPPO_CALL_SCORE_TOKENS: {
      ScorePlan pl;
      if (check_video(vid) != HIPPO_OK || plan_score(kv, vid, n_rows, 1, &pl) != HIPPO_OK) return 0;
      return pl.bytes;
    }
    case HIPPO_CALL_SELECT_GATHER_KV:
      return 256;   // the selection keeps its state in LDS; a token amount keeps the contract uniform
    case HIPPO_CALL_DRAFT_ATTENTION:
    case HIPPO_CALL_VERIFY_ATTENTION: {
      AttnPlan pl;
      if (plan_attention(call, kv, n_rows, seq_len, num_splits, &pl) != HIPPO_OK) return 0;
      return pl.bytes;
    }
    default:
      return 0;
  }
}

size_t hippo_score_layers_workspace_bytes(const hippo_kv_desc* kv, const hippo_video_desc* vid, int32_t l_txt,
                                          int32_t n_layers) {
  ScorePlan pl;
  if (check_kv(kv) != HIPPO_OK || check_video(vid) != HIPPO_OK || plan_score(kv, vid, l_txt, n_layers, &pl) != HIPPO_OK)
    return 0;
  return pl.bytes;
}

int hippo_score_tokens_layers(int32_t n_layers, const void* const* q_txt_layers, int32_t l_txt,
                              const void* const* k_cache_layers, int32_t emb_layer, const hippo_kv_desc* kv,
                              int32_t seq_len, const hippo_video_desc* vid, const void* emb, int32_t emb_dim,
                              int64_t emb_stride_tok, uint32_t flags, float* attn_mass_inout, float* scores_out,
                              float* components_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (q_txt_layers == nullptr || k_cache_layers == nullptr || workspace == nullptr) return HIPPO_ERR_NULL_ARG;
  if (n_layers < 1 || n_layers > kMaxScoreLayers || emb_layer < 0 || emb_layer >= n_layers) return HIPPO_ERR_BAD_SHAPE;
  for (int l = 0; l < n_layers; ++l)
    if (q_txt_layers[l] == nullptr || k_cache_layers[l] == nullptr) return HIPPO_ERR_NULL_ARG;
  int rc = check_kv(kv);
  if (rc != HIPPO_OK) return rc;
  if ((rc = check_video(vid)) != HIPPO_OK) return rc;
  if ((rc = check_crop(vid)) != HIPPO_OK) return rc;
  const bool acc_only = (flags & HIPPO_SCORE_ACCUMULATE_ONLY) != 0;
  if (flags & ~(HIPPO_SCORE_ALL | HIPPO_SCORE_ACCUMULATE_ONLY)) return HIPPO_ERR_BAD_SHAPE;
  if (!acc_only && (flags & HIPPO_SCORE_ALL) == 0) return HIPPO_ERR_BAD_SHAPE;
  if (acc_only && attn_mass_inout == nullptr) return HIPPO_ERR_NULL_ARG;
  if (!acc_only && scores_out == nullptr) return HIPPO_ERR_NULL_ARG;
  const long long Nv = (long long)vid->n_frames * vid->grid_h * vid->grid_w;
  if (seq_len < 1 || (long long)vid->vis_offset + Nv > seq_len) return HIPPO_ERR_BAD_SHAPE;
  const int per16 = 16 / elem_bytes(kv->dtype);
  if (emb != nullptr) {
    if (emb_dim < 1 || emb_stride_tok < emb_dim) return HIPPO_ERR_BAD_SHAPE;
    if (emb_dim % per16) return HIPPO_ERR_BAD_SHAPE;
    if (emb_stride_tok % per16 || !aligned16(emb)) return HIPPO_ERR_BAD_ALIGN;
  }
  for (int l = 0; l < n_layers; ++l)
    if (!aligned16(q_txt_layers[l]) || !aligned16(k_cache_layers[l])) return HIPPO_ERR_BAD_ALIGN;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return HIPPO_ERR_BAD_ALIGN;
  ScorePlan pl;
  if ((rc = plan_score(kv, vid, l_txt, n_layers, &pl)) != HIPPO_OK) return rc;
  if (workspace_bytes < pl.bytes) return HIPPO_ERR_WORKSPACE_TOO_SMALL;

  ScoreParams p;
  p.q_txt = q_txt_layers[0]; p.k_cache = k_cache_layers[emb_layer]; p.emb = emb;
  p.n_layers = n_layers; p.Bz = kv->batch * n_layers;
  for (int l = 0; l < kMaxScoreLayers; ++l) {
    p.q_layers[l] = l < n_layers ? q_txt_layers[l] : nullptr;
    p.k_layers[l] = l < n_layers ? k_cache_layers[l] : nullptr;
  }
  p.B = kv->batch; p.L = l_txt; p.H = kv->n_q_heads; p.Hkv = kv->n_kv_heads;
  p.G = kv->n_q_heads / kv->n_kv_heads; p.D = kv->head_dim; p.dtype = kv->dtype;
  p.sb = kv->stride_b; p.sh = kv->stride_h; p.sn = kv->stride_n;
  p.F = vid->n_frames; p.gh = vid->grid_h; p.gw = vid->grid_w; p.P = vid->grid_h * vid->grid_w;
  p.Nv = (int)Nv; p.vis_off = vid->vis_offset; p.ch = vid->crop_h; p.cw = vid->crop_w;
  p.emb_dim = emb_dim; p.emb_stride_tok = emb_stride_tok; p.emb_stride_b = Nv * emb_stride_tok;
  p.flags = flags;
  p.attn_mass_inout = attn_mass_inout; p.scores_out = scores_out; p.components_out = components_out;
  char* ws = static_cast<char*>(workspace);
  p.row_m = reinterpret_cast<float*>(ws);
  p.row_l = reinterpret_cast<float*>(ws + pl.off_row_l);
  p.row_lse = reinterpret_cast<float*>(ws + pl.off_row_lse);
  p.col_part = reinterpret_cast<float*>(ws + pl.off_col);
  p.s_attn = reinterpret_cast<float*>(ws + pl.off_sa);
  p.s_temp = reinterpret_cast<float*>(ws + pl.off_st);
  p.s_spa = reinterpret_cast<float*>(ws + pl.off_ss);
  p.n_tile = pl.n_tile;
  p.n_rsplit = pl.n_rsplit;
  const hipError_t e = launch_score(p, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HIPPO_OK : HIPPO_ERR_HIP;
}

int hippo_score_tokens(const void* q_txt, int32_t l_txt, const void* k_cache, const hippo_kv_desc* kv,
                       int32_t seq_len, const hippo_video_desc* vid, const void* emb, int32_t emb_dim,
                       int64_t emb_stride_tok, uint32_t flags, float* attn_mass_inout, float* scores_out,
                       float* components_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (q_txt == nullptr || k_cache == nullptr) return HIPPO_ERR_NULL_ARG;
  const void* qs[1] = {q_txt};
  const void* ks[1] = {k_cache};
  return hippo_score_tokens_layers(1, qs, l_txt, ks, 0, kv, seq_len, vid, emb, emb_dim, emb_stride_tok, flags,
                                   attn_mass_inout, scores_out, components_out, workspace, workspace_bytes, stream);
}

int hippo_select_gather_kv(const float* scores, int32_t k, const void* k_src, const void* v_src,
                           const hippo_kv_desc* src, int32_t src_len, const hippo_video_desc* vid,
                           void* k_dst, void* v_dst, const hippo_kv_desc* dst, int32_t* idx_out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (scores == nullptr || idx_out == nullptr || workspace == nullptr) return HIPPO_ERR_NULL_ARG;
  int rc = check_video(vid);
  if (rc != HIPPO_OK) return rc;
  const long long Nv = (long long)vid->n_frames * vid->grid_h * vid->grid_w;
  if (k < 1 || k > Nv) return HIPPO_ERR_BAD_SHAPE;
  const bool do_gather = (k_dst != nullptr) || (v_dst != nullptr);
  if (do_gather && (k_dst == nullptr || v_dst == nullptr || k_src == nullptr || v_src == nullptr))
    return HIPPO_ERR_NULL_ARG;
  if (src == nullptr) return HIPPO_ERR_NULL_ARG;
  if ((rc = check_kv(src, true)) != HIPPO_OK) return rc;
  if (workspace_bytes < 256) return HIPPO_ERR_WORKSPACE_TOO_SMALL;
  SelectParams p;
  p.scores = scores; p.B = src->batch; p.Nv = (int)Nv; p.k = k; p.idx_out = idx_out;
  p.k_src = k_src; p.v_src = v_src; p.k_dst = nullptr; p.v_dst = nullptr;
  p.Hkv = src->n_kv_heads; p.D = src->head_dim; p.elem_bytes = elem_bytes(src->dtype);
  p.ssb = src->stride_b; p.ssh = src->stride_h; p.ssn = src->stride_n;
  p.dsb = p.dsh = p.dsn = 0;
  p.src_len = src_len; p.dst_len = 0; p.vis_off = vid->vis_offset;
  if (do_gather) {
    if (dst == nullptr) return HIPPO_ERR_NULL_ARG;
    if ((rc = check_kv(dst, true)) != HIPPO_OK) return rc;
    if (dst->batch != src->batch || dst->n_kv_heads != src->n_kv_heads || dst->head_dim != src->head_dim ||
        dst->dtype != src->dtype)
      return HIPPO_ERR_BAD_SHAPE;
    if (src_len < 1 || (long long)vid->vis_offset + Nv > src_len) return HIPPO_ERR_BAD_SHAPE;
    if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(k_dst) || !aligned16(v_dst))
      return HIPPO_ERR_BAD_ALIGN;
    p.k_dst = k_dst; p.v_dst = v_dst;
    p.dsb = dst->stride_b; p.dsh = dst->stride_h; p.dsn = dst->stride_n;
    p.dst_len = (int)(src_len - Nv + k);
  }
  const hipError_t e = launch_select_gather(p, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HIPPO_OK : HIPPO_ERR_HIP;
}

int hippo_verify_attention(const void* q, int32_t q_len, const void* k_cache, const void* v_cache,
                           const hippo_kv_desc* kv, int32_t ctx_len, float softmax_scale, int32_t num_splits,
                           void* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  return attention_entry(HIPPO_CALL_VERIFY_ATTENTION, q, q_len, k_cache, v_cache, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, workspace, workspace_bytes, stream);
}

int hippo_draft_attention(const void* q, int32_t q_len, const void* k_cache, const void* v_cache,
                          const hippo_kv_desc* kv, int32_t ctx_len, float softmax_scale, int32_t num_splits,
                          void* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  return attention_entry(HIPPO_CALL_DRAFT_ATTENTION, q, q_len, k_cache, v_cache, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, workspace, workspace_bytes, stream);
}

size_t hippo_static_scratch_bytes(void) { return kStaticScratchBytes; }

int hippo_static_scratch_init(void) {
  int rc = HIPPO_OK;
  static_scratch(&rc);
  return rc;
}

int hippo_verify_attention_static(const void* q, int32_t q_len, const void* k_cache, const void* v_cache,
                                  const hippo_kv_desc* kv, int32_t ctx_len, float softmax_scale,
                                  int32_t num_splits, void* out, float* lse_out, void* stream) {
  // every argument check that needs no device comes before the scratch lookup; the size check uses the
  // same plan as the launch
  if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr) return HIPPO_ERR_NULL_ARG;
  int rc = check_kv(kv);
  if (rc != HIPPO_OK) return rc;
  if (ctx_len < 0 || q_len < 1 || (long long)ctx_len + q_len > 0x7fffff00ll) return HIPPO_ERR_BAD_SHAPE;
  AttnPlan pl;
  if ((rc = plan_attention(HIPPO_CALL_VERIFY_ATTENTION, kv, q_len, ctx_len + q_len, num_splits, &pl)) != HIPPO_OK)
    return rc;
  if (pl.bytes > kStaticScratchBytes) return HIPPO_ERR_STATIC_SCRATCH_LIMIT;
  void* ws = static_scratch(&rc);
  if (ws == nullptr) return rc;
  // the split partials are written in full before the merge reads them: nothing has to start at zero
  return attention_entry(HIPPO_CALL_VERIFY_ATTENTION, q, q_len, k_cache, v_cache, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, ws, kStaticScratchBytes, stream);
}

size_t hippo_spec_verify_workspace_bytes(int32_t batch, int32_t gamma, int32_t vocab, int32_t dtype) {
  SpecPlan pl;
  return plan_spec(batch, gamma, vocab, dtype, &pl) == HIPPO_OK ? pl.bytes : 0;
}

int hippo_spec_verify(const void* p_logits, const void* q_logits, int32_t dtype, int64_t p_stride_row,
                      int64_t q_stride_row, const int32_t* draft_tokens, const float* u_accept,
                      const float* u_sample, int32_t batch, int32_t gamma, int32_t vocab, float temperature,
                      int32_t* n_accept_out, int32_t* next_token_out, float* alpha_out, void* workspace,
                      size_t workspace_bytes, void* stream) {
  SpecPlan pl;
  int rc = plan_spec(batch, gamma, vocab, dtype, &pl);
  if (rc != HIPPO_OK) return rc;
  if (!(temperature >= 0.f) || isinf(temperature)) return HIPPO_ERR_BAD_SHAPE;
  const bool greedy = temperature == 0.f;
  if (p_logits == nullptr || n_accept_out == nullptr || next_token_out == nullptr || workspace == nullptr)
    return HIPPO_ERR_NULL_ARG;
  if (gamma > 0 && (draft_tokens == nullptr || (!greedy && (q_logits == nullptr || u_accept == nullptr))))
    return HIPPO_ERR_NULL_ARG;
  if (!greedy && u_sample == nullptr) return HIPPO_ERR_NULL_ARG;
  if (p_stride_row < vocab || (gamma > 0 && !greedy && q_stride_row < vocab)) return HIPPO_ERR_BAD_SHAPE;
  const int per16 = 16 / elem_bytes(dtype);
  if (p_stride_row % per16 || !aligned16(p_logits) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return HIPPO_ERR_BAD_ALIGN;
  if (gamma > 0 && !greedy && (q_stride_row % per16 || !aligned16(q_logits))) return HIPPO_ERR_BAD_ALIGN;
  if (workspace_bytes < pl.bytes) return HIPPO_ERR_WORKSPACE_TOO_SMALL;

  SpecParams p;
  p.p_logits = p_logits; p.q_logits = q_logits; p.tokens = draft_tokens;
  p.u_accept = u_accept; p.u_sample = u_sample;
  p.B = batch; p.gamma = gamma; p.V = vocab; p.n_rows = pl.n_rows; p.n_seg = pl.n_seg;
  p.p_stride = p_stride_row; p.q_stride = q_stride_row;
  p.c = greedy ? 0.f : kLog2e / temperature;
  p.inv_temperature = greedy ? 0.0 : 1.0 / (double)temperature;
  p.n_accept = n_accept_out; p.next_token = next_token_out; p.alpha_out = alpha_out;
  char* ws = static_cast<char*>(workspace);
  p.stats = reinterpret_cast<SegStat*>(ws);
  p.cells = reinterpret_cast<float*>(ws + pl.off_cells);
  p.chosen = reinterpret_cast<Chosen*>(ws + pl.off_chosen);
  const hipError_t e = launch_spec_verify(p, dtype, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HIPPO_OK : HIPPO_ERR_HIP;
}

int hippo_verify_attention_append(const void* q, int32_t q_len, const void* k_new, const void* v_new,
                                  void* k_cache, void* v_cache, const hippo_kv_desc* kv, int32_t ctx_len,
                                  float softmax_scale, int32_t num_splits, void* out, float* lse_out,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (k_new == nullptr || v_new == nullptr) return HIPPO_ERR_NULL_ARG;
  AttnExtra ex;
  ex.append = true; ex.k_new = k_new; ex.v_new = v_new;
  return attention_entry(HIPPO_CALL_VERIFY_ATTENTION, q, q_len, k_cache, v_cache, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, workspace, workspace_bytes, stream, ex);
}

int hippo_draft_attention_append(const void* q, int32_t q_len, const void* k_new, const void* v_new,
                                 void* k_cache, void* v_cache, const hippo_kv_desc* kv, int32_t ctx_len,
                                 float softmax_scale, int32_t num_splits, void* out, float* lse_out,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (k_new == nullptr || v_new == nullptr) return HIPPO_ERR_NULL_ARG;
  AttnExtra ex;
  ex.append = true; ex.k_new = k_new; ex.v_new = v_new;
  return attention_entry(HIPPO_CALL_DRAFT_ATTENTION, q, q_len, k_cache, v_cache, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, workspace, workspace_bytes, stream, ex);
}

// paged caches: translate the pool descriptor into the per-row strides the kernels use
static int paged_entry(int call, const void* q, int32_t q_len, const void* k_pool, const void* v_pool,
                       const int32_t* block_table, const hippo_paged_kv_desc* pd, int32_t ctx_len,
                       float softmax_scale, int32_t num_splits, void* out, float* lse_out, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (pd == nullptr || block_table == nullptr) return HIPPO_ERR_NULL_ARG;
  if (pd->page_size < 16 || pd->page_size > 256 || (pd->page_size & (pd->page_size - 1))) return HIPPO_ERR_BAD_SHAPE;
  if (pd->n_pool_pages < 1 || pd->max_pages < 1 || ctx_len < 0 || q_len < 1) return HIPPO_ERR_BAD_SHAPE;
  if (((long long)ctx_len + q_len + pd->page_size - 1) / pd->page_size > pd->max_pages) return HIPPO_ERR_BAD_SHAPE;
  if (pd->n_kv_heads < 1 || pd->head_dim < 1 || pd->stride_n < pd->head_dim || pd->stride_h < 0)
    return HIPPO_ERR_BAD_SHAPE;
  // every element of a page lies inside the page's stride, so a clamped page number keeps every
  // access inside the pool
  if ((long long)(pd->page_size - 1) * pd->stride_n + (long long)(pd->n_kv_heads - 1) * pd->stride_h + pd->head_dim >
      pd->stride_page)
    return HIPPO_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(block_table) & 3u) return HIPPO_ERR_BAD_ALIGN;
  hippo_kv_desc kv;
  kv.batch = pd->batch; kv.n_q_heads = pd->n_q_heads; kv.n_kv_heads = pd->n_kv_heads;
  kv.head_dim = pd->head_dim; kv.dtype = pd->dtype;
  kv.stride_b = 0; kv.stride_h = pd->stride_h; kv.stride_n = pd->stride_n;
  const int per16 = 16 / (pd->dtype == HIPPO_DTYPE_BF16 ? 2 : 4);
  if (pd->stride_page % per16) return HIPPO_ERR_BAD_ALIGN;
  AttnExtra ex;
  ex.block_table = block_table; ex.page_size = pd->page_size; ex.max_pages = pd->max_pages;
  ex.n_pool_pages = pd->n_pool_pages; ex.page_stride = pd->stride_page;
  return attention_entry(call, q, q_len, k_pool, v_pool, &kv, ctx_len, softmax_scale, num_splits, out, lse_out,
                         workspace, workspace_bytes, stream, ex);
}

int hippo_verify_attention_paged(const void* q, int32_t q_len, const void* k_pool, const void* v_pool,
                                 const int32_t* block_table, const hippo_paged_kv_desc* kv, int32_t ctx_len,
                                 float softmax_scale, int32_t num_splits, void* out, float* lse_out,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  return paged_entry(HIPPO_CALL_VERIFY_ATTENTION, q, q_len, k_pool, v_pool, block_table, kv, ctx_len,
                     softmax_scale, num_splits, out, lse_out, workspace, workspace_bytes, stream);
}

int hippo_draft_attention_paged(const void* q, int32_t q_len, const void* k_pool, const void* v_pool,
                                const int32_t* block_table, const hippo_paged_kv_desc* kv, int32_t ctx_len,
                                float softmax_scale, int32_t num_splits, void* out, float* lse_out,
                                void* workspace, size_t workspace_bytes, void* stream) {
  return paged_entry(HIPPO_CALL_DRAFT_ATTENTION, q, q_len, k_pool, v_pool, block_table, kv, ctx_len,
                     softmax_scale, num_splits, out, lse_out, workspace, workspace_bytes, stream);
}

int hippo_verify_attention_fp8kv(const void* q, int32_t q_len, const void* k_codes, const void* v_codes,
                                 const float* k_scale, const float* v_scale, const hippo_kv_desc* kv,
                                 int32_t ctx_len, float softmax_scale, int32_t num_splits, void* out,
                                 float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  AttnExtra ex;
  ex.fp8 = true; ex.k_scale = k_scale; ex.v_scale = v_scale;
  return attention_entry(HIPPO_CALL_VERIFY_ATTENTION, q, q_len, k_codes, v_codes, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, workspace, workspace_bytes, stream, ex);
}

int hippo_draft_attention_fp8kv(const void* q, int32_t q_len, const void* k_codes, const void* v_codes,
                                const float* k_scale, const float* v_scale, const hippo_kv_desc* kv,
                                int32_t ctx_len, float softmax_scale, int32_t num_splits, void* out,
                                float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  AttnExtra ex;
  ex.fp8 = true; ex.k_scale = k_scale; ex.v_scale = v_scale;
  return attention_entry(HIPPO_CALL_DRAFT_ATTENTION, q, q_len, k_codes, v_codes, kv, ctx_len, softmax_scale,
                         num_splits, out, lse_out, workspace, workspace_bytes, stream, ex);
}

size_t hippo_quantize_kv_workspace_bytes(const hippo_kv_desc* src, int32_t n_rows) {
  if (check_kv(src) != HIPPO_OK || n_rows < 1) return 0;
  return align_up((size_t)src->batch * src->n_kv_heads * 2 * quant_slices(n_rows, src->head_dim) * sizeof(float), 256);
}

int hippo_quantize_kv_e4m3(const void* k_src, const void* v_src, const hippo_kv_desc* src, int32_t n_rows,
                           void* k_codes, void* v_codes, const hippo_kv_desc* dst, float* k_scale, float* v_scale,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (k_src == nullptr || v_src == nullptr || k_codes == nullptr || v_codes == nullptr || k_scale == nullptr ||
      v_scale == nullptr || workspace == nullptr)
    return HIPPO_ERR_NULL_ARG;
  int rc = check_kv(src);
  if (rc != HIPPO_OK) return rc;
  if ((rc = check_kv(dst, true)) != HIPPO_OK) return rc;
  if (dst->dtype != HIPPO_DTYPE_FP8_E4M3) return HIPPO_ERR_BAD_DTYPE;
  if (dst->batch != src->batch || dst->n_kv_heads != src->n_kv_heads || dst->head_dim != src->head_dim || n_rows < 1)
    return HIPPO_ERR_BAD_SHAPE;
  if (2 * (long long)src->n_kv_heads > 65535) return HIPPO_ERR_BAD_SHAPE;   // (KV head, K or V) is grid y
  if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(k_codes) || !aligned16(v_codes) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255u) || (reinterpret_cast<uintptr_t>(k_scale) & 3u) ||
      (reinterpret_cast<uintptr_t>(v_scale) & 3u))
    return HIPPO_ERR_BAD_ALIGN;
  if (workspace_bytes < hippo_quantize_kv_workspace_bytes(src, n_rows)) return HIPPO_ERR_WORKSPACE_TOO_SMALL;
  QuantParams p;
  p.k_src = k_src; p.v_src = v_src; p.k_dst = k_codes; p.v_dst = v_codes; p.k_scale = k_scale; p.v_scale = v_scale;
  p.partial = reinterpret_cast<float*>(workspace);
  p.B = src->batch; p.Hkv = src->n_kv_heads; p.D = src->head_dim; p.n_rows = n_rows;
  p.n_slices = quant_slices(n_rows, src->head_dim); p.src_dtype = src->dtype;
  p.ssb = src->stride_b; p.ssh = src->stride_h; p.ssn = src->stride_n;
  p.dsb = dst->stride_b; p.dsh = dst->stride_h; p.dsn = dst->stride_n;
  const hipError_t e = launch_quantize(p, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HIPPO_OK : HIPPO_ERR_HIP;
}

}  // extern "C"
