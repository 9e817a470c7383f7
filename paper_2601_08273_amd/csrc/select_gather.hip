// Top-k retention and draft-cache construction (paper: Method, end of "Holistic Score Fusion":
// keep the top-k visual tokens; App. "Details of Experimental Setups": pruned video features are
// removed from the draft model's input, everything else is kept).
//
// Selection is exact and deterministic: scores map to order-preserving 32-bit keys, a 4 x 8-bit
// radix select finds the k-th largest key, and an index-ordered compaction emits every key above
// it plus the first (lowest-index) ties.  All counting is integer, so there is no run-to-run
// variation.
#include "common.h"

namespace hippo {

constexpr int kSelThreads = 1024;

// larger score -> larger key; -0 == +0; NaN -> 0, below every number (-inf maps to 0x007fffff)
__device__ __forceinline__ uint32_t score_key(float x) {
  if (x != x) return 0u;
  uint32_t u = __float_as_uint(x);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kSelThreads) void topk_select(SelectParams p) {
  __shared__ unsigned hist[256];
  __shared__ unsigned sh_prefix, sh_need;
  __shared__ unsigned wave_gt[kSelThreads / 64], wave_eq[kSelThreads / 64];
  __shared__ unsigned run_gt, run_eq;

  const int b = blockIdx.x, tid = threadIdx.x;
  const float* sc = p.scores + (long long)b * p.Nv;
  int32_t* out = p.idx_out + (long long)b * p.k;

  // ---- radix select of the k-th largest key ----
  unsigned prefix = 0, need = (unsigned)p.k;   // `need` keys still wanted among those matching prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const unsigned hi_mask = (shift == 24) ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < p.Nv; i += kSelThreads) {
      const unsigned key = score_key(sc[i]);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      unsigned above = 0;
      int d = 255;
      for (; d > 0; --d) {
        if (above + hist[d] >= need) break;
        above += hist[d];
      }
      sh_prefix = prefix | ((unsigned)d << shift);
      sh_need = need - above;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    __syncthreads();
  }
  const unsigned thr = prefix;      // the k-th largest key
  const unsigned need_eq = need;    // how many keys equal to it are kept (lowest indices first)

  // ---- compaction in index order ----
  if (tid == 0) { run_gt = 0; run_eq = 0; }
  __syncthreads();
  const int lane = tid & 63, wave = tid >> 6;
  for (int base = 0; base < p.Nv; base += kSelThreads) {
    const int i = base + tid;
    unsigned key = 0;
    bool gt = false, eq = false;
    if (i < p.Nv) {
      key = score_key(sc[i]);
      gt = key > thr;
      eq = key == thr;
    }
    const unsigned long long bg = __ballot(gt), be = __ballot(eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    const unsigned my_gt = __popcll(bg & below), my_eq = __popcll(be & below);
    if (lane == 0) { wave_gt[wave] = __popcll(bg); wave_eq[wave] = __popcll(be); }
    __syncthreads();
    unsigned off_gt = run_gt, off_eq = run_eq;
    for (int w = 0; w < wave; ++w) { off_gt += wave_gt[w]; off_eq += wave_eq[w]; }
    const unsigned gt_before = off_gt + my_gt, eq_before = off_eq + my_eq;
    if (gt || (eq && eq_before < need_eq))
      out[gt_before + min(eq_before, need_eq)] = i;
    __syncthreads();
    if (tid == kSelThreads - 1) {
      run_gt = off_gt + my_gt + (gt ? 1u : 0u);
      run_eq = off_eq + my_eq + (eq ? 1u : 0u);
    }
    __syncthreads();
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
  hipLaunchKernelGGL(topk_select, dim3(p.B), dim3(kSelThreads), 0, st, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.k_dst == nullptr) return e;
  const long long total = (long long)p.B * p.Hkv * p.dst_len * (p.D * p.elem_bytes / 16);
  long long blocks = (total + 255) / 256;
  if (blocks > 8 * 256 * 8) blocks = 8 * 256 * 8;
  hipLaunchKernelGGL(gather_kv, dim3((unsigned)blocks), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace hippo
