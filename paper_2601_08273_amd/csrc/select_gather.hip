// Top-k retention and draft-cache construction (paper: Method, end of "Holistic Score Fusion":
// keep the top-k visual tokens; App. "Details of Experimental Setups": pruned video features are
// removed from the draft model's input, everything else is kept).
//
// Selection is exact and deterministic: scores map to order-preserving 32-bit keys, a 12/12/8-bit
// radix select finds the k-th largest key, and an index-ordered compaction emits every key above
// it plus the first (lowest-index) ties.  All counting is integer, so there is no run-to-run
// variation.
#include "common.h"

namespace hippo {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kKeysPerThread = 40;       // keys held in registers: sequences up to 40960 tokens
constexpr int kBins = 4096;              // 12-bit digits (the last pass uses 256 of them)
constexpr int kBinsPerThread = kBins / kSelThreads;

// larger score -> larger key; -0 == +0; NaN -> 0, below every number (-inf maps to 0x007fffff)
__device__ __forceinline__ uint32_t score_key(float x) {
  if (x != x) return 0u;
  uint32_t u = __float_as_uint(x);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive scan over the 1024 threads of the block (wave scan, then the 16 wave totals)
__device__ __forceinline__ unsigned block_incl_scan(unsigned v, unsigned* wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  __syncthreads();
  if (lane == 63) wave_tot[wave] = v;
  __syncthreads();
  unsigned off = 0;
  for (int w = 0; w < wave; ++w) off += wave_tot[w];
  return v + off;
}

// One block per sequence.  NC > 0: every thread keeps its keys (index c*1024 + tid, c < NC) in
// registers, so the scores are read from memory once and every loop over them is unrolled to the
// sequence's size class; NC = 0: any length, each pass re-reads the scores.
// Radix select with digits of 12, 12 and 8 bits: the wide first digit (sign, exponent, 3 mantissa
// bits) spreads scores of similar magnitude over many LDS bins, which keeps same-address atomic
// traffic low.  The compaction is index-ordered: per-(chunk, wave) counts, one scan, then each key
// computes its slot from the scan and its rank inside the wave.
template <int NC>
__global__ __launch_bounds__(kSelThreads) void topk_select(SelectParams p) {
  constexpr bool CACHED = NC > 0;
  __shared__ unsigned hist[kBins];
  __shared__ unsigned wave_tot[kSelWaves];
  __shared__ unsigned sh_prefix, sh_need;

  const int b = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const float* sc = p.scores + (long long)b * p.Nv;
  int32_t* out = p.idx_out + (long long)b * p.k;
  const int n_chunks = (p.Nv + kSelThreads - 1) / kSelThreads;

  unsigned keys[CACHED ? NC : 1];
  if (CACHED) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int i = c * kSelThreads + tid;
      keys[c] = (c < n_chunks && i < p.Nv) ? score_key(sc[i]) : 0u;
    }
  }
  auto key_at = [&](int c) -> unsigned {     // key of chunk c for this thread (index must be < Nv)
    return CACHED ? keys[c] : score_key(sc[c * kSelThreads + tid]);
  };

  // ---- radix select of the k-th largest key ----
  unsigned prefix = 0, need = (unsigned)p.k;   // `need` keys still wanted among those matching prefix
  const int shifts[3] = {20, 8, 0};
  const unsigned masks[3] = {0u, 0xfff00000u, 0xffffff00u};   // bits already decided
  const unsigned dmask[3] = {0xfffu, 0xfffu, 0xffu};
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    if (CACHED) {
#pragma unroll
      for (int c = 0; c < NC; ++c)
        if (c < n_chunks && c * kSelThreads + tid < p.Nv && (keys[c] & masks[pass]) == prefix)
          atomicAdd(&hist[(keys[c] >> shifts[pass]) & dmask[pass]], 1u);
    } else {
      for (int c = 0; c < n_chunks; ++c)
        if (c * kSelThreads + tid < p.Nv) {
          const unsigned key = key_at(c);
          if ((key & masks[pass]) == prefix) atomicAdd(&hist[(key >> shifts[pass]) & dmask[pass]], 1u);
        }
    }
    __syncthreads();
    // thread t looks at its kBinsPerThread bins from the top down, thread 0 holding the highest:
    // an inclusive scan over t then counts the keys in all higher bins
    const int top = kBins - 1 - kBinsPerThread * tid;
    unsigned hsum = 0;
#pragma unroll
    for (int q = 0; q < kBinsPerThread; ++q) hsum += hist[top - q];
    const unsigned incl = block_incl_scan(hsum, wave_tot);
    unsigned above = incl - hsum;                         // keys in bins above this thread's
    if (above < need && incl >= need) {                   // exactly one thread
      unsigned d = top;
#pragma unroll
      for (int q = 0; q < kBinsPerThread - 1; ++q) {
        const unsigned hh = hist[top - q];
        if (d == (unsigned)(top - q) && above + hh < need) { above += hh; d = top - q - 1; }
      }
      sh_prefix = prefix | (d << shifts[pass]);
      sh_need = need - above;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
  }
  const unsigned thr = prefix;      // the k-th largest key
  const unsigned need_eq = need;    // how many keys equal to it are kept (lowest indices first)

  // ---- compaction in index order ----
  // counts per (chunk, wave) in chunk-major order reuse the histogram storage: [2][n_chunks*16]
  unsigned* cnt_gt = hist;
  unsigned* cnt_eq = hist + kKeysPerThread * kSelWaves;
  __syncthreads();
  auto flags = [&](int c, bool& gt, bool& eq) {
    gt = eq = false;
    if (c * kSelThreads + tid < p.Nv) {
      const unsigned key = key_at(c);
      gt = key > thr;
      eq = key == thr;
    }
  };
  if (CACHED) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c < n_chunks) {
        bool gt, eq;
        flags(c, gt, eq);
        const unsigned long long bg = __ballot(gt), be = __ballot(eq);
        if (lane == 0) { cnt_gt[c * kSelWaves + wave] = __popcll(bg); cnt_eq[c * kSelWaves + wave] = __popcll(be); }
      }
    }
    __syncthreads();
    // exclusive scan of both count arrays in (chunk, wave) order; n_chunks * waves <= 640 entries,
    // handled kSelThreads at a time with a running carry
    const int n_ent = n_chunks * kSelWaves;
    unsigned carry_g = 0, carry_e = 0;
    for (int e0 = 0; e0 < n_ent; e0 += kSelThreads) {
      const int e = e0 + tid;
      const unsigned vg = e < n_ent ? cnt_gt[e] : 0u, ve = e < n_ent ? cnt_eq[e] : 0u;
      const unsigned ig = block_incl_scan(vg, wave_tot);
      const unsigned ie = block_incl_scan(ve, wave_tot);
      __syncthreads();
      if (e < n_ent) { cnt_gt[e] = carry_g + ig - vg; cnt_eq[e] = carry_e + ie - ve; }
      if (tid == kSelThreads - 1) { sh_prefix = ig; sh_need = ie; }
      __syncthreads();
      carry_g += sh_prefix;
      carry_e += sh_need;
      __syncthreads();
    }
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c < n_chunks) {
        bool gt, eq;
        flags(c, gt, eq);
        const unsigned long long bg = __ballot(gt), be = __ballot(eq);
        const unsigned gt_before = cnt_gt[c * kSelWaves + wave] + __popcll(bg & below);
        const unsigned eq_before = cnt_eq[c * kSelWaves + wave] + __popcll(be & below);
        if (gt || (eq && eq_before < need_eq)) out[gt_before + min(eq_before, need_eq)] = c * kSelThreads + tid;
      }
    }
  } else {
    // long sequences: chunk by chunk with running totals
    __shared__ unsigned run_gt, run_eq, wg[kSelWaves], we[kSelWaves];
    if (tid == 0) { run_gt = 0; run_eq = 0; }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int c = 0; c < n_chunks; ++c) {
      bool gt, eq;
      flags(c, gt, eq);
      const unsigned long long bg = __ballot(gt), be = __ballot(eq);
      const unsigned my_gt = __popcll(bg & below), my_eq = __popcll(be & below);
      if (lane == 0) { wg[wave] = __popcll(bg); we[wave] = __popcll(be); }
      __syncthreads();
      unsigned off_gt = run_gt, off_eq = run_eq;
      for (int w = 0; w < wave; ++w) { off_gt += wg[w]; off_eq += we[w]; }
      const unsigned gt_before = off_gt + my_gt, eq_before = off_eq + my_eq;
      if (gt || (eq && eq_before < need_eq)) out[gt_before + min(eq_before, need_eq)] = c * kSelThreads + tid;
      __syncthreads();
      if (tid == kSelThreads - 1) {
        run_gt = off_gt + my_gt + (gt ? 1u : 0u);
        run_eq = off_eq + my_eq + (eq ? 1u : 0u);
      }
      __syncthreads();
    }
  }
}

// dst row n of (b, hk): n < vis_off -> src n ; n < vis_off + k -> src vis_off + idx[n - vis_off] ;
// else src n - k + Nv.  One thread moves 16 bytes of K and of V.
__global__ __launch_bounds__(256) void gather_kv(SelectParams p) {
  const int vpr = p.D * p.elem_bytes / 16;                 // 16-byte vectors per row
  const long long total = (long long)p.B * p.Hkv * p.dst_len * vpr;
  for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total;
       e += (long long)gridDim.x * 256) {
    const int vec = (int)(e % vpr);
    long long r = e / vpr;
    const int n = (int)(r % p.dst_len);
    r /= p.dst_len;
    const int hk = (int)(r % p.Hkv), b = (int)(r / p.Hkv);
    int from;
    if (n < p.vis_off) from = n;
    else if (n < p.vis_off + p.k) from = p.vis_off + p.idx_out[(long long)b * p.k + (n - p.vis_off)];
    else from = n - p.k + p.Nv;
    const long long so = ((long long)b * p.ssb + (long long)hk * p.ssh + (long long)from * p.ssn) * p.elem_bytes;
    const long long dof = ((long long)b * p.dsb + (long long)hk * p.dsh + (long long)n * p.dsn) * p.elem_bytes;
    const u32x4 kv = *(const u32x4*)((const char*)p.k_src + so + vec * 16);
    const u32x4 vv = *(const u32x4*)((const char*)p.v_src + so + vec * 16);
    *(u32x4*)((char*)p.k_dst + dof + vec * 16) = kv;
    *(u32x4*)((char*)p.v_dst + dof + vec * 16) = vv;
  }
}

hipError_t launch_select_gather(const SelectParams& p, hipStream_t st) {
  const int n_chunks = (p.Nv + kSelThreads - 1) / kSelThreads;
#define HIPPO_TOPK(NC_) hipLaunchKernelGGL(topk_select<NC_>, dim3(p.B), dim3(kSelThreads), 0, st, p)
  if (n_chunks <= 2) HIPPO_TOPK(2);
  else if (n_chunks <= 4) HIPPO_TOPK(4);
  else if (n_chunks <= 8) HIPPO_TOPK(8);
  else if (n_chunks <= 16) HIPPO_TOPK(16);
  else if (n_chunks <= 24) HIPPO_TOPK(24);
  else if (n_chunks <= 32) HIPPO_TOPK(32);
  else if (n_chunks <= kKeysPerThread) HIPPO_TOPK(kKeysPerThread);
  else HIPPO_TOPK(0);
#undef HIPPO_TOPK
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.k_dst == nullptr) return e;
  const long long total = (long long)p.B * p.Hkv * p.dst_len * (p.D * p.elem_bytes / 16);
  long long blocks = (total + 255) / 256;
  if (blocks > 8 * 256 * 8) blocks = 8 * 256 * 8;
  hipLaunchKernelGGL(gather_kv, dim3((unsigned)blocks), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace hippo
