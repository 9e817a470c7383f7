// Shared device helpers and host-side launch parameter blocks of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hippo.h"

namespace hippo {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kNumCU = 256;        // MI355X compute units (8 XCDs x 32)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // one 16-byte load/store

// ---- bf16 <-> fp32 (raw 16-bit patterns; round to nearest even on the way down) ----------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // keep NaN a NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerVec = 4;  // elements in one 16-byte vector
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void unpack(const u32x4& v, float* o) {
    o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y);
    o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
  }
};
template <> struct Elem<uint16_t> {  // bf16 bits
  static constexpr int kPerVec = 8;
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_f32(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }
  static __device__ __forceinline__ void unpack(const u32x4& v, float* o) {
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
  }
};

// Maximum that propagates NaN (IEEE 754-2019 "maximum").  Unlike fmaxf it needs no quieting of its
// inputs, which the compiler otherwise performs with one extra instruction per operand that comes
// out of an MFMA, and nested calls fold into the three-input v_maximum3_f32.
__device__ __forceinline__ float max_nan(float a, float b) { return __builtin_elementwise_maximum(a, b); }
// maximum of N register values as a chain of three-input maxima: (N + 1) / 2 instructions
template <int N>
__device__ __forceinline__ float max_nan_of(const float (&v)[N]) {
  float m = v[0];
#pragma unroll
  for (int i = 1; i + 1 < N; i += 2) m = max_nan(max_nan(m, v[i]), v[i + 1]);
  if ((N - 1) % 2) m = max_nan(m, v[N - 1]);
  return m;
}

// ---- wavefront reductions and scans (results valid in every lane) ----------------------------
// Cross-lane steps inside the vector ALU (data-parallel primitives, DPP):
// A DPP operand reads another lane of the same 16-lane row (or, for the two row broadcasts, the last
// lane of the previous row / of the lower half) at no more than a few cycles; the generic shuffles
// go through the LDS crossbar (ds_bpermute), a round trip of ~100 cycles per step, which is what a
// lone wave's reduction or scan then consists of.  Lanes without a source lane, and rows outside
// ROW_MASK, read 0.
constexpr int kDppQuadXor1 = 0xB1;        // quad_perm [1,0,3,2]: lane ^ 1
constexpr int kDppQuadXor2 = 0x4E;        // quad_perm [2,3,0,1]: lane ^ 2
constexpr int kDppRowHalfMirror = 0x141;  // lane i of every 8 reads lane 7 - i
constexpr int kDppRowMirror = 0x140;      // lane i of every 16 reads lane 15 - i
constexpr int kDppRowShr = 0x110;         // + n: lane i reads lane i - n of its row
constexpr int kDppRowBcast15 = 0x142;     // lane 15 of a row to every lane of the next row
constexpr int kDppRowBcast31 = 0x143;     // lane 31 to every lane of the upper half
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ unsigned dpp_u32(unsigned v) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) { return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(v))); }

// Reduction over each 16-lane row, result in all its lanes.  After lane ^ 1 and lane ^ 2 a quad is
// uniform, so mirroring 8 lanes swaps its quads (= lane ^ 4) and mirroring the row swaps its halves.
template <typename Op>
__device__ __forceinline__ float row16_reduce(float v, Op op) {
  v = op(v, dpp_f32<kDppQuadXor1>(v));
  v = op(v, dpp_f32<kDppQuadXor2>(v));
  v = op(v, dpp_f32<kDppRowHalfMirror>(v));
  v = op(v, dpp_f32<kDppRowMirror>(v));
  return v;
}
__device__ __forceinline__ float row16_max(float v) { return row16_reduce(v, [](float a, float b) { return max_nan(a, b); }); }
__device__ __forceinline__ float row16_sum(float v) { return row16_reduce(v, [](float a, float b) { return a + b; }); }

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside the rows (row_shr 1, 2, 4, 8), then
// row 0's total into row 1 and row 2's into row 3, then the lower half's total into the upper half.
__device__ __forceinline__ unsigned wave_scan_incl(unsigned v) {
  v += dpp_u32<kDppRowShr + 1>(v);
  v += dpp_u32<kDppRowShr + 2>(v);
  v += dpp_u32<kDppRowShr + 4>(v);
  v += dpp_u32<kDppRowShr + 8>(v);
  v += dpp_u32<kDppRowBcast15, 0xa>(v);
  v += dpp_u32<kDppRowBcast31, 0xc>(v);
  return v;
}

// Reductions over the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48), result in every
// lane.  v_permlane16_swap / v_permlane32_swap exchange whole rows inside the vector ALU: called
// with the same value twice they return (even rows' value, odd rows' value) resp. (lower half's,
// upper half's) in every lane, so one swap and one max / add replace a trip through the LDS
// crossbar (ds_bpermute) per step.
__device__ __forceinline__ float rows4_max(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = max_nan(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return max_nan(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows4_sum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// over each half of the wavefront (lanes 0-31, lanes 32-63), result in all its lanes
__device__ __forceinline__ float half32_max(float v) {
  v = row16_max(v);
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return max_nan(__uint_as_float(a[0]), __uint_as_float(a[1]));
}
__device__ __forceinline__ float half32_sum(float v) {
  v = row16_sum(v);
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(a[0]) + __uint_as_float(a[1]);
}
// exact integer reduction (op associative and commutative: min, max, or, ...) over all 64 lanes
template <typename Op>
__device__ __forceinline__ int wave_reduce_i32(int v, Op op) {
  v = op(v, (int)dpp_u32<kDppQuadXor1>((unsigned)v));
  v = op(v, (int)dpp_u32<kDppQuadXor2>((unsigned)v));
  v = op(v, (int)dpp_u32<kDppRowHalfMirror>((unsigned)v));
  v = op(v, (int)dpp_u32<kDppRowMirror>((unsigned)v));
  auto a = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
  v = op((int)a[0], (int)a[1]);
  auto b = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
  return op((int)b[0], (int)b[1]);
}
// over all 64 lanes, result in every lane
__device__ __forceinline__ float wave_max(float v) { return rows4_max(row16_max(v)); }
__device__ __forceinline__ float wave_sum(float v) { return rows4_sum(row16_sum(v)); }

// r / G for 0 <= r < 2^20 without the integer division sequence (some forty instructions):
// (r + 1/2) * (1/G) lies at least 1/(2G) away from every integer, hundreds of times the rounding error
// of the two operations (checked exhaustively for every r below 2^20 and every G up to 256, with the
// reciprocal one unit in the last place off in either direction).
__device__ __forceinline__ int row_div_group(int r, float inv_g) { return (int)(((float)r + 0.5f) * inv_g); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- HBM -> LDS transfers without registers in between -------------------------------------------
// 16 bytes per lane from global memory straight into LDS at lds_addr + lane*16 (lds_addr uniform).
// Issued from inline assembly with hand-placed vmcnt waits: the compiler would otherwise wait for
// every outstanding transfer before each LDS read.
// NT marks the transfer non-temporal: the bytes are read once and must not displace what the caches
// could still serve (used for caches far larger than the chip's last-level cache).
template <bool NT = false>
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr) {
  // the address is wave-uniform by construction; readfirstlane tells the compiler so where its own
  // analysis cannot (it must end up in a scalar register to reach M0)
  const unsigned uniform_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  // M0 carries the LDS address; the statement puts back what M0 held before, so the compiler's own
  // uses of M0 (which an asm statement cannot declare as overwritten) are never disturbed
  unsigned saved_m0;
  if constexpr (NT)
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "v"(gptr), "s"(uniform_addr)
                 : "memory");
  else
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "v"(gptr), "s"(uniform_addr)
                 : "memory");
}
// A tile that such transfers fill is row-major and unpadded (a lane's 16 bytes land at base + lane*16);
// bank conflicts of the MFMA operand reads are avoided by fetching, for physical 16-byte chunk c of
// tile row r, logical chunk c ^ lds_row_swizzle(r).  D = bf16 elements per row.
template <int D>
__device__ __forceinline__ int lds_row_swizzle(int r) { return (r / (256 / (D * 2))) & (D / 8 - 1); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int N>
struct WaitLadder {   // s_waitcnt vmcnt(step * later) for a run-time, wave-uniform `later` in [0, N]
  template <int STEP>
  static __device__ __forceinline__ void run(int later) {
    if (later >= N) wait_vmcnt<(STEP * N > 63 ? 63 : STEP * N)>();
    else WaitLadder<N - 1>::template run<STEP>(later);
  }
};
template <>
struct WaitLadder<0> {
  template <int STEP>
  static __device__ __forceinline__ void run(int) { wait_vmcnt<0>(); }
};


// ---- host side ---------------------------------------------------------------------------------
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// One attention call, as the kernels see it.
struct AttnParams {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  float* lse;       // may be null
  void* part_o;     // [B, Hkv, S, R, D] unnormalised partial outputs: bf16 from the MFMA kernel, fp32 from the vector-ALU kernel
  float* part_m;    // [B, Hkv, S, R] running maxima (log2 domain)
  float* part_l;    // [B, Hkv, S, R] partial denominators
  int B, q_len, H, Hkv, G, R;
  int ctx_len, n_total;
  long long sb, sh, sn;   // element strides of K and V
  float scale_log2;       // softmax_scale * log2(e)
  int S;                  // number of KV splits
  int row_chunk;          // query rows handled by one block
  int n_chunks;           // ceil(R / row_chunk)
  int tiles_q, tiles_r;   // MFMA partial kernel: n_tiles / S and n_tiles % S (set by its launcher)
  float phase_per_head;   // 1 / (B * Hkv): (batch element, KV head) number i starts its slices i * this of the
                          // way in and wraps around; 0 = every slice is walked from its first tile
  int wave_prio;          // 1: the partial kernel's waves raise their issue priority (verification is
                          // the critical path of a decoding round; the draft call runs beside it)
  // appended-row fusion: when k_new is set, cache rows ctx_len .. ctx_len+q_len-1 are taken from
  // k_new / v_new [B, q_len, Hkv, D] instead of the cache, and one block copies them into the cache
  const void* k_new;
  const void* v_new;
  void* k_w;              // the caches again, writable
  void* v_w;
  // paged cache: when block_table is set, k / v point at page pools and cache row n of sequence b,
  // KV head hk lives at ((table[b][n >> page_shift] * page_stride) + (n & mask) * sn + hk * sh)
  const int32_t* block_table;   // [B, max_pages]
  int page_shift, max_pages, n_pool_pages;
  long long page_stride;        // elements
  // fp8 cache: when k_scale is set, k / v hold E4M3 codes (strides in bytes) and the cache entry is
  // code * k_scale[b, hk] (resp. v_scale); q and out stay bf16
  const float* k_scale;         // [B, Hkv]
  const float* v_scale;
};
constexpr int kMaxSlicePages = 1024;   // page-table entries a block stages in LDS

// Launchers, one per translation unit.  All return a hipError_t from hipGetLastError().
hipError_t launch_attention(const AttnParams& p, int dtype, int head_dim, bool use_mfma, hipStream_t st);

constexpr int kMaxScoreLayers = 64;   // layers whose s_attn sweeps can share one launch

struct ScoreParams {
  const void* q_txt;      // layer 0's (kept for the single-layer kernels)
  const void* k_cache;    // the cache whose keys act as the embedding when emb is null
  int n_layers;           // layers swept by this call (Eq. 2's outer sum)
  int Bz;                 // B * n_layers: (layer, batch element) pairs, the s_attn kernels' "batch"
  const void* q_layers[kMaxScoreLayers];   // [B, L, H, D] per layer
  const void* k_layers[kMaxScoreLayers];   // caches per layer (same strides)
  const void* emb;       // null => keys concatenated over KV heads
  int B, L, H, Hkv, G, D, dtype;
  long long sb, sh, sn;
  int F, gh, gw, P, Nv, vis_off, ch, cw;
  int emb_dim;
  long long emb_stride_tok, emb_stride_b;
  unsigned flags;
  float* attn_mass_inout;
  float* scores_out;
  float* components_out;
  // workspace pieces
  float* row_m;      // [n_tile, Bz, Hkv, L*G] partial row maxima (row r = i*G + g of a KV head)
  float* row_l;      // [n_tile, Bz, Hkv, L*G] partial row sums
  float* row_lse;    // [Bz, Hkv, L*G] final log2-domain row normaliser
  float* col_part;   // [Bz, Hkv * n_rsplit, Nv] column sums per layer, KV head and row run
  float* s_attn;     // [B, Nv]
  float* s_temp;     // [B, Nv]
  float* s_spa;      // [B, Nv]
  int n_tile;        // token tiles of pass 1
  int n_rsplit;      // runs the query rows of a KV head are cut into (one block each)
  // what every wave of the sweeps would otherwise divide out for itself (filled in by launch_score)
  int rows_per_split;            // rows of a run: whole 64-row chunks
  int q_step_i, q_step_g;        // 64 / G and 64 % G: how (i, g) of row r = i*G + g move from chunk to chunk
  int q_last_i, q_last_g;        // (i, g) of the KV head's last row
  int emb_run;                   // consecutive frames of one crop position that a block of the frame-run kernel owns
};
hipError_t launch_score(const ScoreParams& p, hipStream_t st);
int score_token_tile(int dtype);   // tokens per block in the s_attn passes
int score_row_splits(int dtype, long long blocks_unsplit, int rows_per_kv_head);

struct SelectParams {
  const float* scores;
  int B, Nv, k;
  int32_t* idx_out;
  const void* k_src;
  const void* v_src;
  void* k_dst;
  void* v_dst;
  int Hkv, D, elem_bytes;
  long long ssb, ssh, ssn, dsb, dsh, dsn;   // element strides
  int src_len, dst_len, vis_off;
};
hipError_t launch_select_gather(const SelectParams& p, hipStream_t st);

// ---- writer of the 8-bit cache format -----------------------------------------------------------
struct QuantParams {
  const void* k_src;
  const void* v_src;
  void* k_dst;            // E4M3 codes
  void* v_dst;
  float* k_scale;         // [B, Hkv] multipliers (outputs)
  float* v_scale;
  float* partial;         // workspace: [B, Hkv, 2, n_slices] slice maxima
  int B, Hkv, D, n_rows, n_slices, src_dtype;
  long long ssb, ssh, ssn, dsb, dsh, dsn;   // element strides (dst: bytes)
};
int quant_slices(int n_rows, int head_dim);
hipError_t launch_quantize(const QuantParams& p, hipStream_t st);

// ---- speculative-sampling verification ---------------------------------------------------------
constexpr int kSdSeg = 8192;        // vocabulary entries handled by one block
constexpr int kSdMaxGamma = 64;     // longest draft chain
constexpr int kSdMaxVocab = 1 << 20;

struct SegStat {   // statistics of one segment of one logits row
  float m;         // maximum logit (-inf if the segment is all -inf)
  float z;         // sum of exp2((x - m) * c) over the segment
  int arg;         // index (in the row) of the first maximum
  int pad;
};
struct Chosen {    // the row the next token is drawn from, and its normalisers
  int row;         // first rejected position, or gamma after a full acceptance
  int use_residual;
  float mp, inv_zp, mq, inv_zq;
  int pad0, pad1;
};

struct SpecParams {
  const void* p_logits;      // [B, gamma+1, p_stride]
  const void* q_logits;      // [B, gamma, q_stride]; unused when c == 0
  const int32_t* tokens;     // [B, gamma]
  const float* u_accept;     // [B, gamma]
  const float* u_sample;     // [B]
  int B, gamma, V;
  int n_rows;                // 2*gamma + 1 (target rows, then draft rows)
  int n_seg;                 // ceil(V / kSdSeg)
  long long p_stride, q_stride;
  float c;                   // log2(e) / temperature; 0 = greedy
  double inv_temperature;
  int32_t* n_accept;
  int32_t* next_token;
  float* alpha_out;          // may be null
  // workspace pieces
  SegStat* stats;            // [B, n_rows, n_seg]
  float* cells;              // [B, 2 (p, residual), n_seg * cells_per_segment]
  Chosen* chosen;            // [B]
};
hipError_t launch_spec_verify(const SpecParams& p, int dtype, hipStream_t st);
int spec_cells_per_segment(int dtype);

}  // namespace hippo
