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
constexpr int kHistStride = kBins + kBins / 64;   // padded histogram
__device__ __forceinline__ int hist_slot(int bin) { return bin + (bin >> 6); }

// larger score -> larger key; -0 == +0; NaN -> 1, below every number (-inf maps to 0x00800000).
// No score maps to key 0: a thread's slots past the end of the sequence hold 0, which lies below
// every real key, so with k <= N_v such a slot is never above or equal to the k-th largest key and
// no sweep over the cached keys has to ask whether a slot is real.
__device__ __forceinline__ uint32_t score_key(float x) {
  if (x != x) return 1u;
  uint32_t u = __float_as_uint(x);
  if ((u << 1) == 0u) u = 0u;
  return ((u & 0x80000000u) ? ~u : (u | 0x80000000u)) + 1u;      // at most 0xff800001 (+inf)
}

// One wave walks a histogram from the top bin down (no barriers inside): lane l owns the BPL bins
// below nb - 1 - BPL*l, read BATCH at a time so the LDS reads pipeline; an inclusive wave scan of
// the lane sums counts the keys in all higher bins; the lane in which the running count reaches
// `need` walks its bins again and publishes the digit and what is still needed inside it.
template <int BPL, int BATCH>
__device__ __forceinline__ void walk_histogram(const unsigned* h, int nb, int lane, unsigned prefix, unsigned need,
                                               int shift, unsigned* out_prefix, unsigned* out_need) {
  const int top = nb - 1 - BPL * lane;
  unsigned hsum = 0;
#pragma unroll 1
  for (int q0 = 0; q0 < BPL; q0 += BATCH) {
    unsigned v[BATCH];
#pragma unroll
    for (int q = 0; q < BATCH; ++q) v[q] = h[hist_slot(top - q0 - q)];
#pragma unroll
    for (int q = 0; q < BATCH; ++q) hsum += v[q];
  }
  const unsigned incl = wave_scan_incl(hsum);
  unsigned above = incl - hsum;                 // keys in bins above this lane's
  if (above < need && incl >= need) {           // exactly one lane
    int d = top;
    bool found = false;
#pragma unroll 1
    for (int q0 = 0; q0 < BPL; q0 += BATCH) {
      unsigned v[BATCH];
#pragma unroll
      for (int q = 0; q < BATCH; ++q) v[q] = h[hist_slot(top - q0 - q)];
#pragma unroll
      for (int q = 0; q < BATCH; ++q) {
        if (!found) {
          if (above + v[q] >= need) { found = true; d = top - q0 - q; }
          else above += v[q];
        }
      }
    }
    *out_prefix = prefix | ((unsigned)d << shift);
    *out_need = need - above;
  }
}

// Exclusive prefix of `mine` over the block's threads in thread order: a wave scan, the wave totals
// through LDS (one barrier), and the totals of the waves in front by a 16-lane row scan of the totals
// and one lane read.  tot = 16 words nobody else touches until the next barrier.
// sum of the totals of the waves in front of this one (wave_total is wave-uniform)
__device__ __forceinline__ unsigned waves_in_front(unsigned wave_total, unsigned* tot, int lane, int wave) {
  if (lane == 63) tot[wave] = wave_total;
  __syncthreads();
  unsigned t = tot[lane & (kSelWaves - 1)];
  t += dpp_u32<kDppRowShr + 1>(t);
  t += dpp_u32<kDppRowShr + 2>(t);
  t += dpp_u32<kDppRowShr + 4>(t);
  t += dpp_u32<kDppRowShr + 8>(t);
  static_assert(kSelWaves == 16, "the wave totals fill one 16-lane row");
  const int w = __builtin_amdgcn_readfirstlane(wave);
  return w > 0 ? (unsigned)__builtin_amdgcn_readlane((int)t, w - 1) : 0u;
}
__device__ __forceinline__ unsigned block_scan_excl(unsigned mine, unsigned* tot, int lane, int wave) {
  const unsigned incl = wave_scan_incl(mine);
  return incl - mine + waves_in_front((unsigned)__builtin_amdgcn_readlane((int)incl, 63), tot, lane, wave);
}

// One block per sequence.  NC > 0: every thread keeps NC keys in registers, so the scores are read
// from memory once and every loop over them is unrolled to the sequence's size class.  A wave owns
// 64 NC consecutive scores, dealt to its lanes VW at a time (slot c of lane l is score
// wave*64*NC + ((c / VW)*64 + l)*VW + c % VW), so that each load instruction of a wave reads one
// contiguous kilobyte; NC = 0: any length, keys strided over the threads, each pass re-reads them.
// Radix select with digits of 12, 12 and 8 bits: the wide first digit (sign, exponent, 3 mantissa
// bits) spreads scores of similar magnitude over many LDS bins, which keeps same-address atomic
// traffic low.  With cached keys, the keys that share the first digit with the k-th largest (a few
// hundred of 16K on scores of unit scale) are copied to an LDS list when they fit, and the second and
// third histogram are built from that list instead of from another sweep over every thread's keys.
// The compaction is index-ordered: when the keys are cached, one wave scan per group of VW slots plus
// one scan of the wave totals, per-(chunk, wave) ballots with running totals otherwise.
template <int NC>
__global__ __launch_bounds__(kSelThreads) void topk_select(SelectParams p) {
  constexpr bool CACHED = NC > 0;
  // one histogram per radix pass (12, 12, 8 bits); bin i lives at i + i/64, so that the 64 lanes of
  // the scanning wave, which own runs of 64 consecutive bins, hit different LDS banks
  constexpr int kHistWords = 2 * kHistStride + 256 + 4;
  constexpr int kListCap = kBins;            // candidate list: the first histogram's memory, once its digit is known
  __shared__ unsigned hist[kHistWords];
  __shared__ unsigned wave_tot[2][kSelWaves];
  __shared__ unsigned sh_prefix, sh_need, sh_bin_count, sh_list_n;

  const int b = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const float* sc = p.scores + (long long)b * p.Nv;
  int32_t* out = p.idx_out + (long long)b * p.k;
  const int n_chunks = (p.Nv + kSelThreads - 1) / kSelThreads;
  // CACHED: every load goes out before anything waits for one: 16-byte loads where the row allows,
  // addresses past the end pulled back inside (those slots are then set to 0), and the histograms are
  // cleared under the loads.
  constexpr int VW = !CACHED ? 1 : (NC % 4 == 0 ? 4 : (NC % 2 == 0 ? 2 : 1));    // slots dealt together
  constexpr int NV = CACHED ? NC / VW : 1;
  unsigned keys[CACHED ? NC : 1];            // first the scores' bits, then, in place, their keys
  const int wave_first = wave * 64 * NC;     // CACHED only
  auto slot_index = [&](int c) { return wave_first + ((c / VW) * 64 + lane) * VW + c % VW; };
  if (CACHED) {
    const bool vec_ok = (VW == 4) && (p.Nv % 4 == 0) && ((((long long)b * p.Nv) & 3) == 0) &&
                        ((reinterpret_cast<uintptr_t>(p.scores) & 15u) == 0);      // block-uniform
    if (vec_ok) {
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const u32x4 x = *(const u32x4*)(sc + min(slot_index(v * VW), p.Nv - 4));
        keys[v * VW] = x.x; keys[v * VW + 1 % VW] = x.y; keys[v * VW + 2 % VW] = x.z; keys[v * VW + 3 % VW] = x.w;
      }
    } else {
#pragma unroll
      for (int c = 0; c < NC; ++c) keys[c] = __float_as_uint(sc[min(slot_index(c), p.Nv - 1)]);
    }
  }
  for (int i = tid; i < kHistWords; i += kSelThreads) hist[i] = 0;
  if (tid == 0) sh_list_n = 0;
  if (CACHED) {
#pragma unroll
    for (int c = 0; c < NC; ++c) keys[c] = (slot_index(c) < p.Nv) ? score_key(__uint_as_float(keys[c])) : 0u;
  }
  // ---- radix select of the k-th largest key ----
  unsigned prefix = 0, need = (unsigned)p.k;   // `need` keys still wanted among those matching prefix
  const int shifts[3] = {20, 8, 0};
  const unsigned masks[3] = {0u, 0xfff00000u, 0xffffff00u};   // bits already decided
  const unsigned dmask[3] = {0xfffu, 0xfffu, 0xffu};
  bool listed = false;                         // block-uniform: the candidates are in the LDS list
  unsigned list_n = 0;
  unsigned* const list = hist;                 // the first histogram's words
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    unsigned* h = hist + (pass == 0 ? 0 : pass == 1 ? kHistStride : 2 * kHistStride);
    if (CACHED && pass > 0 && listed) {
      for (unsigned i = tid; i < list_n; i += kSelThreads) {
        const unsigned key = list[i];
        if ((key & masks[pass]) == prefix) atomicAdd(&h[hist_slot((key >> shifts[pass]) & dmask[pass])], 1u);
      }
    } else if (CACHED) {
#pragma unroll
      for (int c = 0; c < NC; ++c)        // (slots past the end would all hit bin 0: the first pass leaves them out)
        if ((keys[c] & masks[pass]) == prefix && (pass > 0 || keys[c] != 0u))
          atomicAdd(&h[hist_slot((keys[c] >> shifts[pass]) & dmask[pass])], 1u);
    } else {
      for (int c0 = 0; c0 < n_chunks; c0 += 8) {         // eight scores in flight per thread
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = sc[min((c0 + q) * kSelThreads + tid, p.Nv - 1)];
#pragma unroll
        for (int q = 0; q < 8; ++q)
          if ((c0 + q) * kSelThreads + tid < p.Nv) {
            const unsigned key = score_key(v[q]);
            if ((key & masks[pass]) == prefix) atomicAdd(&h[hist_slot((key >> shifts[pass]) & dmask[pass])], 1u);
          }
      }
    }
    __syncthreads();
    if (pass == 2) {
      if (wave == 0) walk_histogram<4, 4>(h, 256, lane, prefix, need, shifts[pass], &sh_prefix, &sh_need);
    } else {
      // all threads: thread t sums its 4 bins from the top down (thread 0 holds the highest), a block
      // scan counts the keys in all higher bins, and the one thread in which the running count reaches
      // `need` walks its bins again
      constexpr int BPT = kBins / kSelThreads;
      const int top = kBins - 1 - BPT * tid;
      unsigned hv[BPT], hsum = 0;
#pragma unroll
      for (int q = 0; q < BPT; ++q) { hv[q] = h[hist_slot(top - q)]; hsum += hv[q]; }
      unsigned above = block_scan_excl(hsum, wave_tot[pass], lane, wave);
      if (above < need && above + hsum >= need) {           // exactly one thread
        int d = top;
        unsigned in_bin = 0;
        bool found = false;
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
          if (!found) {
            if (above + hv[q] >= need) { found = true; d = top - q; in_bin = hv[q]; }
            else above += hv[q];
          }
        }
        sh_prefix = prefix | ((unsigned)d << shifts[pass]);
        sh_need = need - above;
        sh_bin_count = in_bin;
      }
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    if (CACHED && pass == 0 && sh_bin_count <= (unsigned)kListCap && prefix != 0u) {   // (digit 0 would match empty slots)
      // the keys that share the first digit with the k-th largest move to the list (the first
      // histogram is spent): per-thread count, wave scan, one LDS atomic per wave for its base.
      // The order of the list does not matter: only histograms are built from it.
      unsigned m = 0;
#pragma unroll
      for (int c = 0; c < NC; ++c) m += ((keys[c] & masks[1]) == prefix) ? 1u : 0u;
      const unsigned incl = wave_scan_incl(m);
      unsigned base = 0;
      if (lane == 63 && incl > 0) base = atomicAdd(&sh_list_n, incl);
      unsigned at = (unsigned)__builtin_amdgcn_readlane((int)base, 63) + incl - m;
      if (m > 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
          if ((keys[c] & masks[1]) == prefix) list[at++] = keys[c];
      }
      listed = true;
      list_n = sh_bin_count;
      __syncthreads();
    }
  }
  const unsigned thr = prefix;      // the k-th largest key
  const unsigned need_eq = need;    // how many keys equal to it are kept (lowest indices first)

  // ---- compaction in index order ----
  __syncthreads();
  if (CACHED) {
    // counts of keys above / equal to the threshold, packed (both fit 16 bits: a block caches at
    // most 40960 keys).  Index order inside a wave is (group of VW slots, lane, slot in the group):
    // one wave scan per group, a running total over the groups, then the totals of the waves in
    // front; every thread then writes its own survivors.
    unsigned excl[NV], run = 0;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      unsigned mine = 0;
#pragma unroll
      for (int e = 0; e < VW; ++e)
        mine += ((keys[v * VW + e] > thr) ? 0x10000u : 0u) + ((keys[v * VW + e] == thr) ? 1u : 0u);
      const unsigned incl = wave_scan_incl(mine);
      excl[v] = run + incl - mine;
      run += (unsigned)__builtin_amdgcn_readlane((int)incl, 63);
    }
    const unsigned in_front = waves_in_front(run, wave_tot[0], lane, wave);
    int32_t* const dst = out;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      unsigned gt_before = (in_front + excl[v]) >> 16, eq_before = (in_front + excl[v]) & 0xffffu;
#pragma unroll
      for (int e = 0; e < VW; ++e) {
        const unsigned key = keys[v * VW + e];
        const bool gt = key > thr, eq = key == thr;
        if (gt || (eq && eq_before < need_eq)) dst[gt_before + min(eq_before, need_eq)] = slot_index(v * VW + e);
        gt_before += gt ? 1u : 0u;
        eq_before += eq ? 1u : 0u;
      }
    }
  } else {
    // long sequences: chunk by chunk with running totals
    __shared__ unsigned run_gt, run_eq, wg[kSelWaves], we[kSelWaves];
    if (tid == 0) { run_gt = 0; run_eq = 0; }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    float ahead = sc[min(tid, p.Nv - 1)];                // the next chunk's score travels under this chunk's barriers
    for (int c = 0; c < n_chunks; ++c) {
      const float mine = ahead;
      if (c + 1 < n_chunks) ahead = sc[min((c + 1) * kSelThreads + tid, p.Nv - 1)];
      bool gt = false, eq = false;
      if (c * kSelThreads + tid < p.Nv) {
        const unsigned key = score_key(mine);
        gt = key > thr;
        eq = key == thr;
      }
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
// else src n - k + Nv.  One thread moves 16 bytes of K and of V.  Grid (rows x vectors, KV head, sequence):
// a row holds 2^vpr_shift 16-byte vectors (head dims 64 and 128 in 1, 2 or 4 bytes), so no thread divides.
__global__ __launch_bounds__(256) void gather_kv(SelectParams p, int vpr_shift) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int n = e >> vpr_shift, vec = e & ((1 << vpr_shift) - 1);
  if (n >= p.dst_len) return;
  const int hk = blockIdx.y, b = blockIdx.z;
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
  const int vpr = p.D * p.elem_bytes / 16;                 // 16-byte vectors per row: 4, 8, 16 or 32
  int vpr_shift = 0;
  while ((1 << vpr_shift) < vpr) ++vpr_shift;
  if ((1 << vpr_shift) != vpr || p.Hkv > 65535 || p.B > 65535) return hipErrorInvalidValue;
  const long long per_head = (long long)p.dst_len * vpr;
  if (per_head == 0) return hipSuccess;
  if ((per_head + 255) / 256 > 0x7fffffffll) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_kv, dim3((unsigned)((per_head + 255) / 256), p.Hkv, p.B), dim3(256), 0, st, p, vpr_shift);
  return hipGetLastError();
}

}  // namespace hippo
