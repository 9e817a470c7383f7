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

// Phase timestamps for kernel tuning: compiled in only when HIPPO_TRACE is defined (never in the
// shipped library).  Lane 0 of every wave stores the shader clock at numbered points.
#ifdef HIPPO_TRACE
__device__ long long* g_hippo_trace;
#define HIPPO_TP(i_)                                                                              \
  if ((threadIdx.x & 63) == 0)                                                                    \
    g_hippo_trace[((((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 4 + \
                   (threadIdx.x >> 6)) * 16 + (i_)] = (long long)__builtin_readcyclecounter();
#else
#define HIPPO_TP(i_)
#endif

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
// Data path: K/V tiles go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no registers in
// between) into a private two-stage ring per wave, so a wave always has the next tile in flight
// while it works on the current one and the whole slice of a short context is requested at once.
// The DMA is issued from inline assembly with hand-placed vmcnt waits: the compiler would
// otherwise wait for every outstanding transfer before each LDS read.  A lane's 16 bytes land at
// (wave-uniform base) + lane*16, so a tile is stored row-major and unpadded; bank conflicts are
// avoided by fetching, for physical 16-byte chunk c of row r, logical chunk c ^ swz(r).
//
// Register layouts (lane = j + 16*g, j = lane%16, g = lane/16), v_mfma_f32_16x16x32_bf16:
//   A operand: row j,  8 contraction elements of group g      B operand: column j, same 8 elements
//   D result : column j, rows 4g..4g+3
// S^T = K Q^T  -> D[token][qrow]: lane (qrow j, g) holds tokens 4g..4g+3 of a 16-token block.
// O^T = V^T P^T -> B operand wants, for column (qrow) j and group g, 8 contraction (token) values:
//   the two S^T blocks of a 32-token tile give exactly 8 per lane, so contraction slot 8g+e is
//   token (e/4)*16 + 4g + e%4.  The matching V^T operand (row = head-dim element j, the same 8
//   tokens) comes from ds_read_b64_tr_b16, which hands lane j of a 16-lane group the j-th column
//   of a 4 x 16 block whose rows the lanes address 4 elements at a time.
// The contraction order of QK^T is likewise free: slot (ks, g, e) reads head-dim element
// (g*KS + ks)*8 + e of both K and Q, which makes each lane's K reads one contiguous run.
constexpr int kMfmaTile = 32;
constexpr int kStages = 2;            // per-wave ring depth
constexpr float kRescaleGap = 8.f;    // log2 units

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

template <int D>
struct MfmaSmem {
  static constexpr int kRowBytes = D * 2;                      // unpadded, swizzled rows
  static constexpr int kTileBytes = kMfmaTile * kRowBytes;     // one K or V tile
  static constexpr int kStageBytes = 2 * kTileBytes;           // K tile then V tile
  static constexpr int q_bytes(int rb) { return rb * 16 * kRowBytes; }
  static constexpr int stat_bytes(int rb) { return 2 * 4 * rb * 16 * 4; }   // m and l of 4 waves
  static constexpr int ring_bytes() { return 4 * kStages * kStageBytes; }
  static constexpr int total(int rb) { return q_bytes(rb) + stat_bytes(rb) + ring_bytes(); }
};

// 16 bytes per lane from global memory straight into LDS at lds_addr + lane*16 (lds_addr uniform)
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int D, int RB>
__global__ __launch_bounds__(256, 2) void attn_partial_mfma(AttnParams p) {
  using SM = MfmaSmem<D>;
  constexpr int KS = D / 32;        // MFMA steps of QK^T
  constexpr int DB = D / 16;        // 16-row blocks of O^T
  constexpr int ROWB = SM::kRowBytes;
  constexpr int CPR = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;     // rows covered by one wave-wide 16-byte transfer
  constexpr int NLD = kMfmaTile / RPI;   // transfers per K (or V) tile
  constexpr int RPS = 256 / ROWB;   // rows per 256 bytes of LDS (one pass over all banks)
  constexpr int NQ = RB * 16 / RPI; // transfers for the query block

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Qs = smem;
  float* stat_m = (float*)(smem + SM::q_bytes(RB));          // [4][RB*16]
  float* stat_l = stat_m + 4 * RB * 16;                      // [4][RB*16]
  unsigned char* ring = smem + SM::q_bytes(RB) + SM::stat_bytes(RB);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, hk = blockIdx.y;
  const int b = blockIdx.z / p.n_chunks, chunk = blockIdx.z % p.n_chunks;
  const int r0 = chunk * (RB * 16);

  unsigned char* my_ring = ring + wave * (kStages * SM::kStageBytes);
  const unsigned my_ring_addr = (unsigned)(uintptr_t)my_ring;    // LDS byte address (uniform)
  const unsigned q_addr = (unsigned)(uintptr_t)Qs;

  const char* kbase = (const char*)p.k + ((long long)b * p.sb + (long long)hk * p.sh) * 2;
  const char* vbase = (const char*)p.v + ((long long)b * p.sb + (long long)hk * p.sh) * 2;
  const long long row_bytes = p.sn * 2;

  // transfer n of a tile covers rows n*RPI + lane/CPR; this lane fills physical chunk lane%CPR
  const int ld_row = lane / CPR, ld_pc = lane % CPR;
  unsigned ld_off[NLD];
#pragma unroll
  for (int n = 0; n < NLD; ++n) {
    const int r = n * RPI + ld_row;
    ld_off[n] = (unsigned)(r * row_bytes + ((ld_pc ^ ((r / RPS) & (CPR - 1))) * 16));
  }

  const int n_tiles = (p.n_total + kMfmaTile - 1) / kMfmaTile;
  const int t_lo = (int)((long long)split * n_tiles / p.S);
  const int t_hi = (int)((long long)(split + 1) * n_tiles / p.S);
  const int t_first = t_lo + wave;
  const int n_my = (t_hi > t_first) ? (t_hi - t_first + 3) / 4 : 0;   // tiles of this wave

  // enqueue the K (which = 0) or V (which = 1) transfers of this wave's tile number i into ring
  // stage i % kStages
  auto issue_half = [&](int i, int which) {
    const long long row0 = (long long)(t_first + 4 * i) * kMfmaTile;
    const unsigned dst = my_ring_addr + (i % kStages) * SM::kStageBytes + which * SM::kTileBytes;
    const char* base = which ? vbase : kbase;
    if (row0 + kMfmaTile <= p.n_total) {
      const char* tp = base + row0 * row_bytes;
#pragma unroll
      for (int n = 0; n < NLD; ++n) dma16(tp + ld_off[n], dst + n * 1024);
    } else {   // ragged last tile: rows past the end re-read the last valid row (masked later)
#pragma unroll
      for (int n = 0; n < NLD; ++n) {
        const int r = n * RPI + ld_row;
        long long row = row0 + r;
        row = row < p.n_total ? row : p.n_total - 1;
        dma16(base + row * row_bytes + ((ld_pc ^ ((r / RPS) & (CPR - 1))) * 16), dst + n * 1024);
      }
    }
  };

  HIPPO_TP(0)
  // ---- prologue: K of tile 0, this wave's share of the query block, V of tile 0, tile 1 -- all in
  // flight at once.  Transfers complete in issue order, so "at most n outstanding" identifies
  // exactly which of them have landed.
  if (n_my > 0) issue_half(0, 0);
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    if ((n & 3) == wave) {       // wave-uniform
      const int rr = n * RPI + ld_row;
      int r = r0 + rr;
      r = r < p.R ? r : p.R - 1;                        // padding rows repeat the last real row
      const int i = r / p.G, gq = r % p.G;
      const char* src = (const char*)p.q + ((((long long)b * p.q_len + i) * p.H + hk * p.G + gq) * D) * 2 +
                        ((ld_pc ^ ((rr / RPS) & (CPR - 1))) * 16);
      dma16(src, q_addr + n * 1024);
    }
  }
  if (n_my > 0) issue_half(0, 1);
  if (n_my > 1) { issue_half(1, 0); issue_half(1, 1); }

  int lim[RB];       // last cache row visible to this lane's query row of block rb
  float m_run[RB], l_run[RB];
  f32x4 acc[DB][RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = r0 + rb * 16 + j;
    // padding rows see everything: they stay finite and are never stored
    lim[rb] = (r < p.R) ? p.ctx_len + r / p.G : 0x7fffffff;
    m_run[rb] = -INFINITY;
    l_run[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db][rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // per-lane LDS offsets of the MFMA operand reads (swizzle folded in)
  const int swz_k = (j / RPS) & (CPR - 1);            // rows tb*16 + j
  unsigned k_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_off[ks] = j * ROWB + (((g * KS + ks) ^ swz_k) * 16);
  const int v_row = 4 * g + (j >> 2);                  // + tb*16
  const int swz_v = (v_row / RPS) & (CPR - 1);
  unsigned v_off[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
    v_off[db] = v_row * ROWB + (((2 * db + ((j & 3) >> 1)) ^ swz_v) * 16) + (j & 1) * 8;

  // wait for K of tile 0 and the query block (V of tile 0 and tile 1 may still be in flight),
  // then publish Q
  if (n_my > 1) wait_vmcnt<3 * NLD>(); else if (n_my == 1) wait_vmcnt<NLD>(); else wait_vmcnt<0>();
  __syncthreads();
  HIPPO_TP(1)
  int trace_it = 0;
  (void)trace_it;

  for (int i = 0; i < n_my; ++i) {
    const bool has_next = (i + 1 < n_my);             // tile i+1 is already in flight
    if (i > 0) { if (has_next) wait_vmcnt<3 * NLD>(); else wait_vmcnt<NLD>(); }     // K landed
    const unsigned char* Kt = my_ring + (i % kStages) * SM::kStageBytes;
    const unsigned char* Vt = Kt + SM::kTileBytes;
    const int n0 = (t_first + 4 * i) * kMfmaTile;
    if (trace_it == 0) { HIPPO_TP(2) }

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
      for (int tb = 0; tb < 2; ++tb) kop[tb] = *(const bf16x8*)(Kt + tb * 16 * ROWB + k_off[ks]);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const bf16x8 qop = *(const bf16x8*)(Qs + rb * 16 * ROWB + k_off[ks]);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
          s[tb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[tb], qop, s[tb][rb], 0, 0, 0);
      }
    }
    if (trace_it == 0) { HIPPO_TP(3) }

    // ---- online softmax per query row (row = lane%16 of block rb) ----
    // The reference m_run of a row only moves when the tile maximum exceeds it by more than
    // kRescaleGap (log2 units): probabilities then stay below 2^kRescaleGap, well inside fp32 and
    // bf16 range, and the accumulators are rescaled a handful of times instead of once per tile.
    if ((n0 + kMfmaTile - 1) > p.ctx_len) {            // wave-uniform: tile touches the causal edge
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if ((n0 + tb * 16 + 4 * g + e) > lim[rb]) s[tb][rb][e] = -INFINITY;
    }
    bool grow = false;
    float mx[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float m8 = fmaxf(fmaxf(fmaxf(s[0][rb][0], s[0][rb][1]), fmaxf(s[0][rb][2], s[0][rb][3])),
                       fmaxf(fmaxf(s[1][rb][0], s[1][rb][1]), fmaxf(s[1][rb][2], s[1][rb][3])));
      m8 = fmaxf(m8, __shfl_xor(m8, 16, 64));
      m8 = fmaxf(m8, __shfl_xor(m8, 32, 64));
      mx[rb] = m8 * p.scale_log2;                      // scale > 0: max commutes with it
      grow |= mx[rb] > m_run[rb] + kRescaleGap;        // also true for the first finite maximum
    }
    if (__any(grow)) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const bool up = mx[rb] > m_run[rb] + kRescaleGap;
        const float a = up ? fast_exp2(m_run[rb] - mx[rb]) : 1.f;    // m_run = -inf -> 0
        if (up) m_run[rb] = mx[rb];
        l_run[rb] *= a;
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db][rb] *= a;
      }
    }
    bf16x8 pop[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float neg_m = (m_run[rb] == -INFINITY) ? 0.f : -m_run[rb];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // the PV product sees P rounded to bf16; sum the rounded value so numerator and
        // denominator stay consistent
        const __bf16 pb = (__bf16)fast_exp2(fmaf(s[e >> 2][rb][e & 3], p.scale_log2, neg_m));
        psum += (float)pb;
        pop[rb][e] = pb;
      }
      l_run[rb] += psum;                               // per-lane share; the 4 groups g meet at the end
    }
    if (trace_it == 0) { HIPPO_TP(4) }

    // ---- O^T += V^T P^T ----
    if (has_next) wait_vmcnt<2 * NLD>(); else wait_vmcnt<0>();                      // V landed
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(Vt + v_off[db]));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(Vt + 16 * ROWB + v_off[db]));
      const bf16x8 vop = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        acc[db][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop[rb], acc[db][rb], 0, 0, 0);
    }
    if (trace_it == 0) { HIPPO_TP(5) }
    ++trace_it;

    // the stage is free again: every LDS read of it has returned (the MFMAs consumed them)
    if (i + kStages < n_my) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      issue_half(i + kStages, 0);
      issue_half(i + kStages, 1);
    }
  }
  HIPPO_TP(6)

  // ---- merge the 4 waves: wave w reduces and stores head-dim blocks w, w+4, ... of all rows ----
  // every wave publishes its (m, l) and its unscaled accumulators; the ring is free by then
  // because each wave has drained its own transfers and the barrier orders the rest
  f32x4* xbuf = (f32x4*)ring;                               // [4 waves][DB][RB][64 lanes]
  auto xbuf_at = [&](int w, int db, int rb) { return xbuf + ((w * DB + db) * RB + rb) * 64 + lane; };
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    l_run[rb] += __shfl_xor(l_run[rb], 16, 64);
    l_run[rb] += __shfl_xor(l_run[rb], 32, 64);
    if (g == 0) {
      stat_m[wave * RB * 16 + rb * 16 + j] = m_run[rb];
      stat_l[wave * RB * 16 + rb * 16 + j] = l_run[rb];
    }
  }
  __syncthreads();   // (a) every wave is done reading its ring before anyone overwrites it
  HIPPO_TP(7)
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) *xbuf_at(wave, db, rb) = acc[db][rb];
  __syncthreads();   // (b) accumulators and statistics of all waves visible
  {
    const long long slot = ((long long)b * p.Hkv + hk) * p.S + split;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int r = r0 + rb * 16 + j;
      float mw[4], mm = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) { mw[w] = stat_m[w * RB * 16 + rb * 16 + j]; mm = fmaxf(mm, mw[w]); }
      float f[4], ll = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        f[w] = (mw[w] == -INFINITY) ? 0.f : fast_exp2(mw[w] - mm);
        ll = fmaf(f[w], stat_l[w * RB * 16 + rb * 16 + j], ll);
      }
#pragma unroll
      for (int dd = 0; dd < DB / 4; ++dd) {
        const int db = wave + 4 * dd;
        f32x4 o = *xbuf_at(0, db, rb) * f[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) o += *xbuf_at(w, db, rb) * f[w];
        if (r < p.R) *(f32x4*)(p.part_o + (slot * p.R + r) * D + db * 16 + 4 * g) = o;
      }
      if (wave == 0 && g == 0 && r < p.R) {
        p.part_m[slot * p.R + r] = mm;
        p.part_l[slot * p.R + r] = ll;
      }
    }
  }
  HIPPO_TP(8)
}

// =================================================================================================
// Merge of the KV slices: out = sum_s 2^(m_s - m*) o_s / sum_s 2^(m_s - m*) l_s
// One block per (query row, KV head, batch element).  The slices are spread over the threads: first
// the S weights (one slice per thread, block-wide max and sum), then thread (sg, vec) accumulates
// 16-byte vector `vec` of the row over slices sg, sg + NSG, ... and the NSG groups meet in LDS.
// =================================================================================================
constexpr int kMaxSplits = 1024;

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_combine(AttnParams p) {
  constexpr int VPR = D / 4;           // float4 vectors per row
  constexpr int NSG = 256 / VPR;       // slice groups
  __shared__ float w_s[kMaxSplits];
  __shared__ float red[8];
  __shared__ f32x4 acc_s[NSG][VPR];

  const int r = blockIdx.x, hk = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const long long slot0 = ((long long)b * p.Hkv + hk) * p.S;
  const int vec = tid % VPR, sg = tid / VPR;

  // the first PF slices of every group are fetched before the weights are known, so the whole
  // merge costs one trip to memory
  constexpr int PF = 8;
  f32x4 pre[PF];
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int s = sg + u * NSG;
    pre[u] = (s < p.S) ? *(const f32x4*)(p.part_o + ((slot0 + s) * p.R + r) * D + vec * 4)
                       : (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  float mloc = -INFINITY;
  for (int s = tid; s < p.S; s += 256) mloc = fmaxf(mloc, p.part_m[(slot0 + s) * p.R + r]);
  mloc = wave_max(mloc);
  if ((tid & 63) == 0) red[tid >> 6] = mloc;
  __syncthreads();
  const float mstar = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float dloc = 0.f;
  for (int s = tid; s < p.S; s += 256) {
    const float ms = p.part_m[(slot0 + s) * p.R + r];
    const float w = (ms == -INFINITY) ? 0.f : fast_exp2(ms - mstar);
    w_s[s] = w;
    dloc = fmaf(w, p.part_l[(slot0 + s) * p.R + r], dloc);
  }
  dloc = wave_sum(dloc);
  if ((tid & 63) == 0) red[4 + (tid >> 6)] = dloc;
  __syncthreads();
  const float den = red[4] + red[5] + red[6] + red[7];

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int s = sg + u * NSG;
    if (s < p.S) acc += pre[u] * w_s[s];
  }
#pragma unroll 4
  for (int s = sg + PF * NSG; s < p.S; s += NSG) {
    const f32x4 o = *(const f32x4*)(p.part_o + ((slot0 + s) * p.R + r) * D + vec * 4);
    acc += o * w_s[s];
  }
  acc_s[sg][vec] = acc;
  __syncthreads();
  if (tid < VPR) {
    f32x4 t = acc_s[0][tid];
#pragma unroll
    for (int g2 = 1; g2 < NSG; ++g2) t += acc_s[g2][tid];
    const float inv = 1.f / den;
    const int i = r / p.G, gq = r % p.G, h = hk * p.G + gq;
    T* o = (T*)p.out + (((long long)b * p.q_len + i) * p.H + h) * D + tid * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) Elem<T>::store(o + e, t[e] * inv);
    if (p.lse != nullptr && tid == 0)
      p.lse[((long long)b * p.H + h) * p.q_len + i] = (mstar + __log2f(den)) * kLn2;
  }
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
  hipLaunchKernelGGL((attn_combine<T, D>), dim3(p.R, p.Hkv, p.B), dim3(256), 0, st, p);
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
