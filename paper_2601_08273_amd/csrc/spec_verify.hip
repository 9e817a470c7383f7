// Speculative-sampling verification of a chain of gamma draft tokens (paper: Preliminaries,
// "Speculative Decoding", Eq. 1 and the resampling rule below it).
//
// Three launches, none of them a single-block walk over the vocabulary:
//   sd_row_stats : grid (segments, 2*gamma+1 rows, B).  Per 8192-word segment of a logits row:
//                  maximum, sum of exp relative to it, first argmax.
//   sd_cells     : grid (segments, B).  Every block merges the segment statistics (cheap, and it
//                  keeps the launch free of cross-block waits), evaluates Eq. 1 for all gamma
//                  positions and finds the first rejection j; then it turns its segment of
//                  max(0, p_j - q_j) (or of p_gamma after a full acceptance) into ordered
//                  partial sums, one per wave-contiguous "cell" of 64 lanes x one 16-byte vector.
//   sd_pick      : grid (B).  Ordered scan over the cell sums -> total mass and the cell in which
//                  the running sum first exceeds u * total; one wave re-evaluates that cell and
//                  finds the word (inverse CDF in index order).
// Greedy decoding (temperature 0) needs only the first launch over the target rows and a
// one-block-per-sequence comparison of argmax with the draft tokens.
//
// Arithmetic: probabilities and sums fp32 (exp2 with the temperature folded into the exponent
// scale); the gamma acceptance ratios of Eq. 1 are formed in double from the fp32 row sums, so the
// accept decision `u < alpha` is taken on a value with ~1e-6 relative error.
#include "common.h"

namespace hippo {

namespace {
// (largest value, lowest index among equals) of the lanes' candidates: an exact, order-independent
// choice, so the steps can run in any order -- inside the vector ALU: four in-row steps, two row swaps
__device__ __forceinline__ void better_of(float& m, int& arg, float om, int oa) {
  if (om > m || (om == m && oa < arg)) { m = om; arg = oa; }
}
template <int CTRL>
__device__ __forceinline__ void argmax_step(float& m, int& arg) {
  const float om = dpp_f32<CTRL>(m);
  const int oa = (int)dpp_u32<CTRL>((unsigned)arg);
  better_of(m, arg, om, oa);
}
__device__ __forceinline__ void row16_argmax(float& m, int& arg) {
  argmax_step<kDppQuadXor1>(m, arg);
  argmax_step<kDppQuadXor2>(m, arg);
  argmax_step<kDppRowHalfMirror>(m, arg);
  argmax_step<kDppRowMirror>(m, arg);
}
__device__ __forceinline__ void wave_argmax(float& m, int& arg) {
  row16_argmax(m, arg);
  {
    auto sm = __builtin_amdgcn_permlane16_swap(__float_as_uint(m), __float_as_uint(m), false, false);
    auto sa = __builtin_amdgcn_permlane16_swap((unsigned)arg, (unsigned)arg, false, false);
    m = __uint_as_float(sm[0]); arg = (int)sa[0];
    better_of(m, arg, __uint_as_float(sm[1]), (int)sa[1]);
  }
  {
    auto sm = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
    auto sa = __builtin_amdgcn_permlane32_swap((unsigned)arg, (unsigned)arg, false, false);
    m = __uint_as_float(sm[0]); arg = (int)sa[0];
    better_of(m, arg, __uint_as_float(sm[1]), (int)sa[1]);
  }
}


constexpr int kSdThreads = 256;
constexpr int kSdWaves = kSdThreads / 64;
constexpr int kSdPerThread = kSdSeg / kSdThreads;   // 32 logits per thread, held in registers
constexpr int kSdLdsStats = 1024;                   // segment statistics staged in LDS (16 KB)

template <typename T>
__device__ __forceinline__ void load_segment(const T* row, int v0, int V, float (&x)[kSdPerThread]) {
  constexpr int VEC = Elem<T>::kPerVec;
  constexpr int NV = kSdPerThread / VEC;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int idx = v0 + (j * kSdThreads + (int)threadIdx.x) * VEC;
    if (idx + VEC <= V) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(row + idx);
      Elem<T>::unpack(v, &x[j * VEC]);
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) x[j * VEC + e] = (idx + e < V) ? Elem<T>::load(row + idx + e) : -INFINITY;
    }
  }
}

// probability of a word from its logit and the row's statistics; the same expression, without
// contraction, in both kernels that evaluate it
__device__ __forceinline__ float word_prob(float x, float m, float c, float inv_z) {
#pragma clang fp contract(off)
  return fast_exp2((x - m) * c) * inv_z;
}
__device__ __forceinline__ float residual(float pp, float qq) {
#pragma clang fp contract(off)
  const float r = pp - qq;
  return r > 0.f ? r : 0.f;
}

template <typename T>
__global__ __launch_bounds__(kSdThreads) void sd_row_stats(SpecParams p) {
  __shared__ float sh_m[kSdWaves];
  __shared__ int sh_a[kSdWaves];
  __shared__ float sh_z[kSdWaves];
  const int seg = blockIdx.x, row = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* base = (row <= p.gamma)
      ? static_cast<const T*>(p.p_logits) + ((long long)b * (p.gamma + 1) + row) * p.p_stride
      : static_cast<const T*>(p.q_logits) + ((long long)b * p.gamma + (row - p.gamma - 1)) * p.q_stride;
  const int v0 = seg * kSdSeg;
  float x[kSdPerThread];
  load_segment<T>(base, v0, p.V, x);

  constexpr int VEC = Elem<T>::kPerVec;
  float m = -INFINITY;
  int arg = 0x7fffffff;
#pragma unroll
  for (int i = 0; i < kSdPerThread; ++i) {     // ascending index inside the thread: strict > keeps the first
    const int idx = v0 + ((i / VEC) * kSdThreads + tid) * VEC + (i % VEC);
    if (x[i] > m) { m = x[i]; arg = idx; }
  }
  wave_argmax(m, arg);
  if (lane == 0) { sh_m[wave] = m; sh_a[wave] = arg; }
  __syncthreads();
  m = sh_m[0]; arg = sh_a[0];
#pragma unroll
  for (int w = 1; w < kSdWaves; ++w)
    if (sh_m[w] > m || (sh_m[w] == m && sh_a[w] < arg)) { m = sh_m[w]; arg = sh_a[w]; }

  float z = 0.f;
  if (p.c > 0.f && m > -INFINITY) {
#pragma unroll
    for (int i = 0; i < kSdPerThread; ++i) z += fast_exp2((x[i] - m) * p.c);
  }
  z = wave_sum(z);
  if (lane == 0) sh_z[wave] = z;
  __syncthreads();
  if (tid == 0) {
    SegStat s;
    s.m = m; s.z = (sh_z[0] + sh_z[1]) + (sh_z[2] + sh_z[3]); s.arg = arg; s.pad = 0;
    p.stats[((long long)b * p.n_rows + row) * p.n_seg + seg] = s;
  }
}

// Eq. 1 for all positions, first rejection, and (sampling mode) the cell sums of the distribution
// the next token is drawn from.  Blocks of one sequence repeat the small first part identically.
template <typename T>
__global__ __launch_bounds__(kSdThreads) void sd_cells(SpecParams p) {
  __shared__ float sh_mp[kSdMaxGamma + 1], sh_zp[kSdMaxGamma + 1], sh_mq[kSdMaxGamma], sh_zq[kSdMaxGamma];
  __shared__ int sh_argp[kSdMaxGamma + 1];
  __shared__ int sh_rej[kSdMaxGamma];
  __shared__ int sh_j;
  __shared__ SegStat sh_stats[kSdLdsStats];
  const int seg = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool greedy = !(p.c > 0.f);
  const T* pl = static_cast<const T*>(p.p_logits) + (long long)b * (p.gamma + 1) * p.p_stride;
  const T* ql = static_cast<const T*>(p.q_logits) + (long long)b * p.gamma * p.q_stride;
  const SegStat* st = p.stats + (long long)b * p.n_rows * p.n_seg;

  // the few dependent loads first, so they overlap the statistics fetch
  int x = 0;
  float u = 0.f, lp_raw = 0.f, lq_raw = 0.f;
  if (tid < p.gamma) {
    x = p.tokens[(long long)b * p.gamma + tid];
    if (!greedy) {
      u = p.u_accept[(long long)b * p.gamma + tid];
      if (x >= 0 && x < p.V) {
        lp_raw = Elem<T>::load(pl + (long long)tid * p.p_stride + x);
        lq_raw = Elem<T>::load(ql + (long long)tid * p.q_stride + x);
      }
    }
  }
  // segment statistics of every row of this sequence: one parallel fetch into LDS when they fit
  const int n_stats = (greedy ? p.gamma + 1 : p.n_rows) * p.n_seg;
  const bool staged = n_stats <= kSdLdsStats;
  if (staged) {
    for (int i = tid; i < n_stats; i += kSdThreads) sh_stats[i] = st[i];
    __syncthreads();
  }
  // merged statistics of every row: one row per group of 16 lanes (lanes over segments), so the
  // merges run side by side instead of one thread walking each row
  {
    const int n_r = greedy ? p.gamma + 1 : p.n_rows;
    const int grp = tid >> 4, gl = tid & 15;
    for (int row = grp; row < n_r; row += kSdThreads / 16) {
      const SegStat* rs = staged ? sh_stats + row * p.n_seg : st + (long long)row * p.n_seg;
      float m = -INFINITY;
      int arg = 0x7fffffff;
      for (int i = gl; i < p.n_seg; i += 16) {
        const float sm_ = rs[i].m;
        const int sa_ = rs[i].arg;
        if (sm_ > m || (sm_ == m && sa_ < arg)) { m = sm_; arg = sa_; }
      }
      row16_argmax(m, arg);
      float z = 0.f;
      if (!greedy)
        for (int i = gl; i < p.n_seg; i += 16)
          if (rs[i].m > -INFINITY) z += rs[i].z * fast_exp2((rs[i].m - m) * p.c);
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) z += __shfl_xor(z, o, 64);
      if (gl == 0) {
        if (row <= p.gamma) { sh_mp[row] = m; sh_zp[row] = z; sh_argp[row] = arg; }
        else { sh_mq[row - p.gamma - 1] = m; sh_zq[row - p.gamma - 1] = z; }
      }
    }
  }
  __syncthreads();
  if (tid < p.gamma) {
    const float m = sh_mp[tid], z = sh_zp[tid];
    const int a = sh_argp[tid];
    double alpha;
    if (x < 0 || x >= p.V) {
      alpha = 0.0;                                        // not a word: rejected
    } else if (greedy) {
      alpha = (x == a) ? 1.0 : 0.0;
    } else {
      const float mq = sh_mq[tid], zq = sh_zq[tid];
      const double lp = (double)lp_raw - (double)m;
      const double lq = (double)lq_raw - (double)mq;
      // p[x] / q[x] = exp((lp - lq) / T) * zq / zp;  p[x] = 0 -> 0;  q[x] = 0 -> p >= q -> 1
      if (lp == -INFINITY) alpha = (lq == -INFINITY) ? 1.0 : 0.0;
      else if (lq == -INFINITY) alpha = 1.0;
      else {
        const double ratio = exp((lp - lq) * p.inv_temperature) * ((double)zq / (double)z);
        alpha = ratio >= 1.0 ? 1.0 : ratio;
      }
    }
    sh_rej[tid] = greedy ? (alpha == 0.0) : !((double)u < alpha);
    if (seg == 0 && p.alpha_out) p.alpha_out[(long long)b * p.gamma + tid] = (float)alpha;
  }
  __syncthreads();
  if (tid == 0) {
    int j = p.gamma;
    for (int i = p.gamma - 1; i >= 0; --i)
      if (sh_rej[i]) j = i;
    sh_j = j;
  }
  __syncthreads();
  const int j = sh_j;
  const bool rejected = j < p.gamma;
  if (greedy) {
    if (tid == 0) {
      p.n_accept[b] = j;
      p.next_token[b] = (sh_argp[j] >= 0 && sh_argp[j] < p.V) ? sh_argp[j] : 0;   // a row without a finite logit
    }
    return;
  }
  const float mp = sh_mp[j], inv_zp = 1.0f / sh_zp[j];
  const float mq = rejected ? sh_mq[j] : 0.f, inv_zq = rejected ? 1.0f / sh_zq[j] : 0.f;
  if (seg == 0 && tid == 0) {
    p.n_accept[b] = j;
    Chosen ch;
    ch.row = j; ch.use_residual = rejected; ch.mp = mp; ch.inv_zp = inv_zp; ch.mq = mq; ch.inv_zq = inv_zq;
    ch.pad0 = ch.pad1 = 0;
    p.chosen[b] = ch;
  }

  constexpr int VEC = Elem<T>::kPerVec;
  constexpr int NV = kSdPerThread / VEC;
  constexpr int CPS = NV * kSdWaves;             // cells per segment
  const int v0 = seg * kSdSeg;
  float xp[kSdPerThread];
  load_segment<T>(pl + (long long)j * p.p_stride, v0, p.V, xp);
  float sp[NV], sr[NV];
  if (rejected) {
    float xq[kSdPerThread];
    load_segment<T>(ql + (long long)j * p.q_stride, v0, p.V, xq);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      float a = 0.f, r = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float pp = word_prob(xp[v * VEC + e], mp, p.c, inv_zp);
        const float qq = word_prob(xq[v * VEC + e], mq, p.c, inv_zq);
        a += pp; r += residual(pp, qq);
      }
      sp[v] = a; sr[v] = r;
    }
  } else {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      float a = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) a += word_prob(xp[v * VEC + e], mp, p.c, inv_zp);
      sp[v] = a; sr[v] = 0.f;
    }
  }
  float* cells_p = p.cells + ((long long)b * 2 + 0) * p.n_seg * CPS + (long long)seg * CPS;
  float* cells_r = p.cells + ((long long)b * 2 + 1) * p.n_seg * CPS + (long long)seg * CPS;
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const float a = wave_sum(sp[v]);
    const float r = wave_sum(sr[v]);
    if (lane == 0) { cells_p[v * kSdWaves + wave] = a; cells_r[v * kSdWaves + wave] = r; }
  }
}

// inverse CDF over the ordered cell sums, then inside the chosen cell
template <typename T>
__global__ __launch_bounds__(kSdThreads) void sd_pick(SpecParams p) {
  constexpr int VEC = Elem<T>::kPerVec;
  constexpr int CPS = (kSdPerThread / VEC) * kSdWaves;
  __shared__ float sh_wave[kSdWaves];
  __shared__ int sh_first[kSdWaves], sh_last[kSdWaves];
  __shared__ float sh_before[kSdThreads];
  __shared__ float sh_total;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const Chosen ch = p.chosen[b];
  const int n_cells = p.n_seg * CPS;
  const int cpt = (n_cells + kSdThreads - 1) / kSdThreads;     // consecutive cells per thread
  const int c0 = tid * cpt, c1 = min(n_cells, c0 + cpt);

  int which = ch.use_residual;
  float local, incl, before, total;
  const float* cells;
  for (;;) {
    cells = p.cells + ((long long)b * 2 + which) * n_cells;
    local = 0.f;
    for (int c = c0; c < c1; ++c) local += cells[c];
    incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const float n = __shfl_up(incl, o, 64);
      if (lane >= o) incl += n;
    }
    __syncthreads();
    if (lane == 63) sh_wave[wave] = incl;
    __syncthreads();
    float off = 0.f;
    for (int w = 0; w < wave; ++w) off += sh_wave[w];
    before = off + (incl - local);
    if (tid == kSdThreads - 1) sh_total = off + incl;
    __syncthreads();
    total = sh_total;
    if (which == 1 && !(total > 0.f)) { which = 0; continue; }   // p_j == q_j after rounding: draw from p_j
    break;
  }
  const float target = p.u_sample[b] * total;

  // first cell whose inclusive running sum exceeds the target; last cell with mass as the fallback
  int first = 0x7fffffff, last = -1;
  float run = before, before_first = 0.f;
  for (int c = c0; c < c1; ++c) {
    const float v = cells[c];
    if (v > 0.f) last = c;
    if (first == 0x7fffffff && run + v > target && v > 0.f) { first = c; before_first = run; }
    run += v;
  }
  sh_before[tid] = before_first;
  int wf = first, wl = last;
  wf = wave_reduce_i32(wf, [](int a, int b) { return min(a, b); });
  wl = wave_reduce_i32(wl, [](int a, int b) { return max(a, b); });
  if (lane == 0) { sh_first[wave] = wf; sh_last[wave] = wl; }
  __syncthreads();
  if (wave != 0) return;
  int cell = min(min(sh_first[0], sh_first[1]), min(sh_first[2], sh_first[3]));
  float base;
  if (cell != 0x7fffffff) {
    base = sh_before[cell / cpt];
  } else {
    cell = max(max(sh_last[0], sh_last[1]), max(sh_last[2], sh_last[3]));
    base = -INFINITY;                       // rounding left no crossing: take the last word with mass
    if (cell < 0) {                         // no mass at all (a row without a finite logit)
      if (lane == 0) p.next_token[b] = 0;
      return;
    }
  }

  // one wave re-evaluates the cell: lane l holds VEC consecutive words
  const T* pl = static_cast<const T*>(p.p_logits) + ((long long)b * (p.gamma + 1) + ch.row) * p.p_stride;
  const T* ql = static_cast<const T*>(p.q_logits) + ((long long)b * p.gamma + ch.row) * p.q_stride;
  const int w0 = cell * 64 * VEC + lane * VEC;
  float val[VEC];
  float lane_sum = 0.f;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    float v = 0.f;
    if (w0 + e < p.V) {
      const float pp = word_prob(Elem<T>::load(pl + w0 + e), ch.mp, p.c, ch.inv_zp);
      v = pp;
      if (which == 1) v = residual(pp, word_prob(Elem<T>::load(ql + w0 + e), ch.mq, p.c, ch.inv_zq));
    }
    val[e] = v;
    lane_sum += v;
  }
  float incl_l = lane_sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float n = __shfl_up(incl_l, o, 64);
    if (lane >= o) incl_l += n;
  }
  float run_l = base + (incl_l - lane_sum);
  int hit = 0x7fffffff, last_w = -1;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    if (val[e] > 0.f) last_w = w0 + e;
    run_l += val[e];
    if (hit == 0x7fffffff && val[e] > 0.f && run_l > target) hit = w0 + e;
  }
  hit = wave_reduce_i32(hit, [](int a, int b) { return min(a, b); });
  last_w = wave_reduce_i32(last_w, [](int a, int b) { return max(a, b); });
  if (lane == 0) p.next_token[b] = (hit != 0x7fffffff) ? hit : (last_w >= 0 ? last_w : 0);
}

template <typename T>
hipError_t launch_typed(const SpecParams& p, hipStream_t st) {
  const bool greedy = !(p.c > 0.f);
  const int rows = greedy ? p.gamma + 1 : p.n_rows;
  sd_row_stats<T><<<dim3(p.n_seg, rows, p.B), kSdThreads, 0, st>>>(p);
  sd_cells<T><<<dim3(greedy ? 1 : p.n_seg, p.B), kSdThreads, 0, st>>>(p);
  if (!greedy) sd_pick<T><<<dim3(p.B), kSdThreads, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace

int spec_cells_per_segment(int dtype) {
  return (kSdPerThread / (dtype == HIPPO_DTYPE_BF16 ? 8 : 4)) * kSdWaves;
}

hipError_t launch_spec_verify(const SpecParams& p, int dtype, hipStream_t st) {
  return dtype == HIPPO_DTYPE_BF16 ? launch_typed<uint16_t>(p, st) : launch_typed<float>(p, st);
}

}  // namespace hippo
