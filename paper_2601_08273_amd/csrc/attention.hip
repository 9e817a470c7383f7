// Split-KV streaming attention for the draft-decode and target-verification calls
// (paper: Preliminaries, "Speculative Decoding"; the cost the paper attributes to reading large KV
// caches, App. "Details of Baselines").
//
// One launch streams each KV slice once for all R = G * q_len query rows that share a KV head
// (row r = i * G + g: new token i, query head g of the group), keeping an online-softmax state
// per row; a second small launch merges the slices.  Two partial kernels:
//   * attn_partial_mfma  -- bf16, MFMA 16x16x32: S^T = K Q^T puts the streamed tokens on the MFMA
//     M axis, so the score tile comes out in exactly the register layout the PV product
//     O^T = V^T P^T needs for its B operand; only V goes through a transposing LDS read.
//   * attn_partial_valu  -- fp32 or bf16 inputs, fp32 vector ALU; used for fp32 caches.
#include "common.h"

namespace hippo {

// =================================================================================================
// Vector-ALU partial kernel
// =================================================================================================
constexpr int kValuTile = 32;   // tokens per tile
constexpr int kValuRows = 32;   // query rows per block

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_partial_valu(AttnParams p) {
  constexpr int TT = kValuTile, RC = kValuRows;
  constexpr int NG = 256 / D;          // row groups in the PV phase
  constexpr int RPT = RC / NG;         // rows per thread in the PV phase
  constexpr int VPR = D / Elem<T>::kPerVec;  // 16-byte vectors per row

  __shared__ float Ks[TT][D + 1];
  __shared__ float Vs[TT][D];
  __shared__ float Qs[RC][D + 1];
  __shared__ float Ps[RC][TT];
  __shared__ float alpha_s[RC];

  const int tid = threadIdx.x;
  const int split = blockIdx.x, hk = blockIdx.y;
  const int b = blockIdx.z / p.n_chunks, chunk = blockIdx.z % p.n_chunks;
  const int r0 = chunk * RC;

  const T* kbase = (const T*)p.k + (long long)b * p.sb + (long long)hk * p.sh;
  const T* vbase = (const T*)p.v + (long long)b * p.sb + (long long)hk * p.sh;

  // stage the query rows of this chunk (zero rows beyond R)
  for (int e = tid; e < RC * D; e += 256) {
    const int rr = e / D, c = e % D, r = r0 + rr;
    float val = 0.f;
    if (r < p.R) {
      const int i = r / p.G, g = r % p.G;
      val = Elem<T>::load((const T*)p.q + (((long long)b * p.q_len + i) * p.H + hk * p.G + g) * D + c);
    }
    Qs[rr][c] = val;
  }

  // QK / softmax role: token = tid % 32, row group = tid / 32 -> rows rg + 8 * x
  const int tok = tid & 31, rg = tid >> 5;
  float m_run[4], l_run[4];
  int lim[4];
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    m_run[x] = -INFINITY;
    l_run[x] = 0.f;
    const int r = r0 + rg + 8 * x;
    lim[x] = (r < p.R) ? p.ctx_len + r / p.G : -1;   // last visible cache row
  }
  // PV role: column c, row group grp -> rows grp + NG * x
  const int c_pv = tid % D, grp = tid / D;
  float acc[RPT];
#pragma unroll
  for (int x = 0; x < RPT; ++x) acc[x] = 0.f;

  const int n_tiles = (p.n_total + TT - 1) / TT;
  const int t_lo = (int)((long long)split * n_tiles / p.S);
  const int t_hi = (int)((long long)(split + 1) * n_tiles / p.S);

  for (int t = t_lo; t < t_hi; ++t) {
    const int n0 = t * TT;
    __syncthreads();   // previous tile fully consumed (also orders the Q staging)
    for (int e = tid; e < TT * VPR; e += 256) {
      const int row = e / VPR, vec = e % VPR, n = n0 + row;
      float kf[Elem<T>::kPerVec], vf[Elem<T>::kPerVec];
      if (n < p.n_total) {
        const u32x4 kv4 = *(const u32x4*)(kbase + (long long)n * p.sn + vec * Elem<T>::kPerVec);
        const u32x4 vv4 = *(const u32x4*)(vbase + (long long)n * p.sn + vec * Elem<T>::kPerVec);
        Elem<T>::unpack(kv4, kf);
        Elem<T>::unpack(vv4, vf);
      } else {
#pragma unroll
        for (int u = 0; u < Elem<T>::kPerVec; ++u) kf[u] = vf[u] = 0.f;
      }
#pragma unroll
      for (int u = 0; u < Elem<T>::kPerVec; ++u) {
        Ks[row][vec * Elem<T>::kPerVec + u] = kf[u];
        Vs[row][vec * Elem<T>::kPerVec + u] = vf[u];
      }
    }
    __syncthreads();

    // logits of this thread's token against its 4 rows
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < D; ++c) {
      const float kc = Ks[tok][c];
#pragma unroll
      for (int x = 0; x < 4; ++x) s[x] = fmaf(kc, Qs[rg + 8 * x][c], s[x]);
    }
    const int n = n0 + tok;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      float sv = (n <= lim[x]) ? s[x] * p.scale_log2 : -INFINITY;
      float mx = sv;
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      const float m_new = fmaxf(m_run[x], mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float pv = fast_exp2(sv - m_safe);
      float ps = pv;
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) ps += __shfl_xor(ps, o, 64);
      const float a = fast_exp2(m_run[x] - m_safe);
      l_run[x] = l_run[x] * a + ps;
      m_run[x] = m_new;
      Ps[rg + 8 * x][tok] = pv;
      if (tok == 0) alpha_s[rg + 8 * x] = a;
    }
    __syncthreads();

#pragma unroll
    for (int x = 0; x < RPT; ++x) acc[x] *= alpha_s[grp + NG * x];
    for (int tt = 0; tt < TT; ++tt) {
      const float vv = Vs[tt][c_pv];
#pragma unroll
      for (int x = 0; x < RPT; ++x) acc[x] = fmaf(Ps[grp + NG * x][tt], vv, acc[x]);
    }
  }

  const long long slot = ((long long)b * p.Hkv + hk) * p.S + split;
#pragma unroll
  for (int x = 0; x < RPT; ++x) {
    const int r = r0 + grp + NG * x;
    if (r < p.R) p.part_o[(slot * p.R + r) * D + c_pv] = acc[x];
  }
  if (tok == 0) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int r = r0 + rg + 8 * x;
      if (r < p.R) {
        p.part_m[slot * p.R + r] = m_run[x];
        p.part_l[slot * p.R + r] = l_run[x];
      }
    }
  }
}

// =================================================================================================
// MFMA partial kernel (bf16)
// =================================================================================================
// Work decomposition: grid (S, H_kv, B * n_chunks); a block of 4 waves owns one KV slice and up to
// RB*16 query rows.  The slice is cut into 32-token tiles dealt round-robin to the waves; every
// wave runs its own online softmax over its tiles (no block barrier while streaming) and the four
// states are merged through LDS at the end.
//
// Register layouts (lane = j + 16*g, j = lane%16, g = lane/16), v_mfma_f32_16x16x32_bf16:
//   A operand: row j,  8 contraction elements of group g      B operand: column j, same 8 elements
//   D result : column j, rows 4g..4g+3
// S^T = K Q^T  -> D[token][qrow]: lane (qrow j, g) holds tokens 4g..4g+3 of a 16-token block.
// O^T = V^T P^T -> B operand wants, for column (qrow) j and group g, 8 contraction (token) values:
//   the two S^T blocks of a 32-token tile give exactly 8 per lane, so contraction slot 8g+e is
//   token (e/4)*16 + 4g + e%4; the V^T operand is read from LDS with the same token order.
// The contraction order of QK^T is likewise free: slot (ks, g, e) reads head-dim element
// (g*KS + ks)*8 + e of both K and Q, which makes each lane's K reads one contiguous run.
constexpr int kMfmaTile = 32;

template <int D>
struct MfmaSmem {
  static constexpr int kRowBytes = D * 2 + 16;                 // padded row: conflict-free 16-byte reads
  static constexpr int kTileBytes = kMfmaTile * kRowBytes;     // one K or V tile
  static constexpr int q_bytes(int rb) { return rb * 16 * kRowBytes; }
  static constexpr int stat_bytes(int rb) { return 2 * 4 * rb * 16 * 4; }   // m and l of 4 waves
  static constexpr int total(int rb) { return q_bytes(rb) + stat_bytes(rb) + 4 * 2 * kTileBytes; }
};

template <int D, int RB>
__global__ __launch_bounds__(256) void attn_partial_mfma(AttnParams p) {
  using SM = MfmaSmem<D>;
  constexpr int KS = D / 32;        // MFMA steps of QK^T
  constexpr int DB = D / 16;        // 16-row blocks of O^T
  constexpr int ROWB = SM::kRowBytes;
  constexpr int CPR = D / 8;        // 16-byte chunks per cache row
  constexpr int RPI = 64 / CPR;     // rows covered by one wave-wide 16-byte load
  constexpr int NLD = kMfmaTile / RPI;

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Qs = smem;
  float* stat_m = (float*)(smem + SM::q_bytes(RB));          // [4][RB*16]
  float* stat_l = stat_m + 4 * RB * 16;                      // [4][RB*16]
  unsigned char* stage = smem + SM::q_bytes(RB) + SM::stat_bytes(RB);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, hk = blockIdx.y;
  const int b = blockIdx.z / p.n_chunks, chunk = blockIdx.z % p.n_chunks;
  const int r0 = chunk * (RB * 16);

  unsigned char* Kt = stage + wave * 2 * SM::kTileBytes;
  unsigned char* Vt = Kt + SM::kTileBytes;

  // ---- stage Q (rows beyond R are zero) ----
  for (int e = tid; e < RB * 16 * CPR; e += 256) {
    const int rr = e / CPR, ch = e % CPR, r = r0 + rr;
    u32x4 val = (u32x4){0u, 0u, 0u, 0u};
    if (r < p.R) {
      const int i = r / p.G, gq = r % p.G;
      val = *(const u32x4*)((const uint16_t*)p.q +
                            (((long long)b * p.q_len + i) * p.H + hk * p.G + gq) * D + ch * 8);
    }
    *(u32x4*)(Qs + rr * ROWB + ch * 16) = val;
  }
  __syncthreads();

  const uint16_t* kbase = (const uint16_t*)p.k + (long long)b * p.sb + (long long)hk * p.sh;
  const uint16_t* vbase = (const uint16_t*)p.v + (long long)b * p.sb + (long long)hk * p.sh;

  int lim[RB];       // last cache row visible to this lane's query row of block rb
  float m_run[RB], l_run[RB];
  f32x4 acc[DB][RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = r0 + rb * 16 + j;
    // padding rows (zero queries) see everything: they stay finite and are never stored
    lim[rb] = (r < p.R) ? p.ctx_len + r / p.G : 0x7fffffff;
    m_run[rb] = -INFINITY;
    l_run[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db][rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const int n_tiles = (p.n_total + kMfmaTile - 1) / kMfmaTile;
  const int t_lo = (int)((long long)split * n_tiles / p.S);
  const int t_hi = (int)((long long)(split + 1) * n_tiles / p.S);

  const int ld_row = lane / CPR, ld_ch = lane % CPR;
  u32x4 kr[NLD], vr[NLD];
  const uint16_t* kld = kbase + ld_ch * 8;
  const uint16_t* vld = vbase + ld_ch * 8;
#define HIPPO_ISSUE_LOADS(T_)                                                        \
  _Pragma("unroll") for (int n = 0; n < NLD; ++n) {                                  \
    int row = (T_) * kMfmaTile + n * RPI + ld_row;                                   \
    row = row < p.n_total ? row : p.n_total - 1; /* in bounds; masked below */       \
    kr[n] = *(const u32x4*)(kld + (long long)row * p.sn);                            \
    vr[n] = *(const u32x4*)(vld + (long long)row * p.sn);                            \
  }

  int t = t_lo + wave;
  if (t < t_hi) { HIPPO_ISSUE_LOADS(t) }
  for (; t < t_hi; t += 4) {
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
      *(u32x4*)(Kt + (n * RPI + ld_row) * ROWB + ld_ch * 16) = kr[n];
      *(u32x4*)(Vt + (n * RPI + ld_row) * ROWB + ld_ch * 16) = vr[n];
    }
    if (t + 4 < t_hi) { HIPPO_ISSUE_LOADS(t + 4) }      // next tile streams in behind the math

    // ---- S^T = K Q^T for the two 16-token blocks ----
    f32x4 s[2][RB];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) s[tb][rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 kop[2];
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
        kop[tb] = *(const bf16x8*)(Kt + (tb * 16 + j) * ROWB + (g * KS + ks) * 16);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const bf16x8 qop = *(const bf16x8*)(Qs + (rb * 16 + j) * ROWB + (g * KS + ks) * 16);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
          s[tb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[tb], qop, s[tb][rb], 0, 0, 0);
      }
    }

    // ---- online softmax per query row (row = lane%16 of block rb) ----
    const int n0 = t * kMfmaTile;
    const bool need_mask = (n0 + kMfmaTile - 1) > p.ctx_len;
    bf16x8 pop[RB];
    float alpha[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float sv[8];
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float x = s[tb][rb][e] * p.scale_log2;
          if (need_mask && (n0 + tb * 16 + 4 * g + e) > lim[rb]) x = -INFINITY;
          sv[tb * 4 + e] = x;
        }
      float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                       fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[rb], mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      alpha[rb] = fast_exp2(m_run[rb] - m_safe);
      m_run[rb] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = fast_exp2(sv[e] - m_safe);
        // the PV product sees P rounded to bf16; sum the rounded value so numerator and
        // denominator stay consistent
        const __bf16 pb = (__bf16)pe;
        psum += (float)pb;
        pop[rb][e] = pb;
      }
      l_run[rb] = l_run[rb] * alpha[rb] + psum;           // per-lane share; groups g merged at the end
    }

    // ---- O^T += V^T P^T ----
    bool rescale = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) rescale |= (alpha[rb] != 1.f);
    if (__any(rescale)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[db][rb] *= alpha[rb];
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      bf16x8 vop;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int tl = (e >> 2) * 16 + 4 * g + (e & 3);
        vop[e] = *(const __bf16*)(Vt + tl * ROWB + (db * 16 + j) * 2);
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        acc[db][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop[rb], acc[db][rb], 0, 0, 0);
    }
  }

#undef HIPPO_ISSUE_LOADS
  // ---- merge the 4 waves ----
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    l_run[rb] += __shfl_xor(l_run[rb], 16, 64);
    l_run[rb] += __shfl_xor(l_run[rb], 32, 64);
    if (g == 0) stat_m[wave * RB * 16 + rb * 16 + j] = m_run[rb];
  }
  __syncthreads();   // all waves are done with their staging tiles, maxima published
  float m_blk[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mm = fmaxf(mm, stat_m[w * RB * 16 + rb * 16 + j]);
    m_blk[rb] = mm;
    const float f = (m_run[rb] == -INFINITY) ? 0.f : fast_exp2(m_run[rb] - mm);
    if (g == 0) stat_l[wave * RB * 16 + rb * 16 + j] = l_run[rb] * f;
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db][rb] *= f;
  }
  // tree: waves 2,3 -> LDS; waves 0,1 add; wave 1 -> LDS; wave 0 adds and writes out
  f32x4* xbuf = (f32x4*)stage;                              // [2][DB][RB][64]
  auto xbuf_at = [&](int slot, int db, int rb) { return xbuf + ((slot * DB + db) * RB + rb) * 64 + lane; };
  if (wave >= 2) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) *xbuf_at(wave - 2, db, rb) = acc[db][rb];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) acc[db][rb] += *xbuf_at(wave, db, rb);
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) *xbuf_at(0, db, rb) = acc[db][rb];
  }
  __syncthreads();
  if (wave == 0) {
    const long long slot = ((long long)b * p.Hkv + hk) * p.S + split;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int r = r0 + rb * 16 + j;
      if (r < p.R) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const f32x4 o = acc[db][rb] + *xbuf_at(0, db, rb);
          *(f32x4*)(p.part_o + (slot * p.R + r) * D + db * 16 + 4 * g) = o;
        }
        if (g == 0) {
          float ll = 0.f;
#pragma unroll
          for (int w = 0; w < 4; ++w) ll += stat_l[w * RB * 16 + rb * 16 + j];
          p.part_m[slot * p.R + r] = m_blk[rb];
          p.part_l[slot * p.R + r] = ll;
        }
      }
    }
  }
}

// =================================================================================================
// Merge of the KV slices: out = sum_s 2^(m_s - m*) o_s / sum_s 2^(m_s - m*) l_s
// =================================================================================================
template <typename T, int D>
__global__ __launch_bounds__(D) void attn_combine(AttnParams p) {
  const int r = blockIdx.x, hk = blockIdx.y, b = blockIdx.z, c = threadIdx.x;
  const long long slot0 = ((long long)b * p.Hkv + hk) * p.S;
  float mstar = -INFINITY;
  for (int s = 0; s < p.S; ++s) mstar = fmaxf(mstar, p.part_m[(slot0 + s) * p.R + r]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < p.S; ++s) {
    const float ms = p.part_m[(slot0 + s) * p.R + r];
    const float w = (ms == -INFINITY) ? 0.f : fast_exp2(ms - mstar);
    den = fmaf(w, p.part_l[(slot0 + s) * p.R + r], den);
    num = fmaf(w, p.part_o[((slot0 + s) * p.R + r) * D + c], num);
  }
  const int i = r / p.G, gq = r % p.G, h = hk * p.G + gq;
  Elem<T>::store((T*)p.out + (((long long)b * p.q_len + i) * p.H + h) * D + c, num / den);
  if (p.lse != nullptr && c == 0)
    p.lse[((long long)b * p.H + h) * p.q_len + i] = (mstar + __log2f(den)) * kLn2;
}

// =================================================================================================
// host launch
// =================================================================================================
template <int D, int RB>
static hipError_t launch_mfma(const AttnParams& p, hipStream_t st) {
  constexpr int smem = MfmaSmem<D>::total(RB);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_partial_mfma<D, RB>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(p.S, p.Hkv, p.B * p.n_chunks);
  hipLaunchKernelGGL((attn_partial_mfma<D, RB>), grid, dim3(256), smem, st, p);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_mfma_d(const AttnParams& p, hipStream_t st) {
  switch (p.row_chunk / 16) {
    case 1: return launch_mfma<D, 1>(p, st);
    case 2: return launch_mfma<D, 2>(p, st);
    case 3: return launch_mfma<D, 3>(p, st);
    default: return launch_mfma<D, 4>(p, st);
  }
}

template <typename T, int D>
static hipError_t launch_valu(const AttnParams& p, hipStream_t st) {
  dim3 grid(p.S, p.Hkv, p.B * p.n_chunks);
  hipLaunchKernelGGL((attn_partial_valu<T, D>), grid, dim3(256), 0, st, p);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_combine(const AttnParams& p, hipStream_t st) {
  hipLaunchKernelGGL((attn_combine<T, D>), dim3(p.R, p.Hkv, p.B), dim3(D), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_attention(const AttnParams& p, int dtype, int head_dim, bool use_mfma, hipStream_t st) {
  hipError_t e;
  if (dtype == HIPPO_DTYPE_BF16) {
    if (use_mfma) e = (head_dim == 128) ? launch_mfma_d<128>(p, st) : launch_mfma_d<64>(p, st);
    else e = (head_dim == 128) ? launch_valu<uint16_t, 128>(p, st) : launch_valu<uint16_t, 64>(p, st);
    if (e != hipSuccess) return e;
    return (head_dim == 128) ? launch_combine<uint16_t, 128>(p, st) : launch_combine<uint16_t, 64>(p, st);
  }
  e = (head_dim == 128) ? launch_valu<float, 128>(p, st) : launch_valu<float, 64>(p, st);
  if (e != hipSuccess) return e;
  return (head_dim == 128) ? launch_combine<float, 128>(p, st) : launch_combine<float, 64>(p, st);
}

}  // namespace hippo
