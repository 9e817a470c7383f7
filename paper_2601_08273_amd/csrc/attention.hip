// Split-KV streaming attention for the draft-decode and target-verification calls
// (paper: Preliminaries, "Speculative Decoding"; the cost the paper attributes to reading large KV
// caches, App. "Details of Baselines").
//
// One launch streams each KV slice once for all R = G * q_len query rows that share a KV head
// (row r = i * G + g: new token i, query head g of the group), keeping an online-softmax state
// per row; a second small launch merges the slices.  Two partial kernels:
//   * attn_partial_grid  -- bf16, MFMA 16x16x32: S^T = K Q^T puts the streamed tokens on the MFMA
//     M axis, so the score tile comes out in exactly the register layout the PV product
//     O^T = V^T P^T needs for its B operand; only V goes through a transposing LDS read.
//     Instantiations of the same kernel cover the cache-format variants: rows appended by the
//     launch itself, paged caches, and caches of 8-bit floating-point codes (converted to bf16
//     after the LDS read).
//   * attn_partial_valu  -- fp32 or bf16 inputs, fp32 vector ALU; used for fp32 caches.
#include <atomic>
#include <type_traits>

#include "common.h"

namespace hippo {

// =================================================================================================
// Vector-ALU partial kernel
// =================================================================================================
// Appended-row fusion: the q_len new K/V rows of (b, hk) go from k_new / v_new [B, q_len, Hkv, D] into
// cache rows ctx_len.., bit for bit.  Called by one block per (b, hk) after its own transfers have
// drained; no block of this launch reads those cache rows (they all read k_new / v_new instead).
template <typename T, int D>
__device__ __forceinline__ void append_new_rows(const AttnParams& p, int b, int hk) {
  constexpr int VPR = D / Elem<T>::kPerVec;    // 16-byte pieces per row
  for (int e = threadIdx.x; e < p.q_len * VPR; e += blockDim.x) {
    const int nr = e / VPR, pc = e % VPR;
    const long long src = (((long long)b * p.q_len + nr) * p.Hkv + hk) * D + pc * Elem<T>::kPerVec;
    const long long dst = (long long)b * p.sb + (long long)hk * p.sh + (long long)(p.ctx_len + nr) * p.sn +
                          pc * Elem<T>::kPerVec;
    *(u32x4*)((T*)p.k_w + dst) = *(const u32x4*)((const T*)p.k_new + src);
    *(u32x4*)((T*)p.v_w + dst) = *(const u32x4*)((const T*)p.v_new + src);
  }
}

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
        const T* ks = kbase + (long long)n * p.sn;
        const T* vs = vbase + (long long)n * p.sn;
        if (p.block_table != nullptr) {                      // paged cache: page of row n, row inside it
          int pg = p.block_table[(long long)b * p.max_pages + (n >> p.page_shift)];
          pg = pg < 0 ? 0 : (pg >= p.n_pool_pages ? p.n_pool_pages - 1 : pg);
          const long long o = (long long)pg * p.page_stride + (long long)(n & ((1 << p.page_shift) - 1)) * p.sn +
                              (long long)hk * p.sh;
          ks = (const T*)p.k + o;
          vs = (const T*)p.v + o;
        }
        if (p.k_new != nullptr && n >= p.ctx_len) {          // a row that has not reached the cache yet
          const long long o = (((long long)b * p.q_len + (n - p.ctx_len)) * p.Hkv + hk) * D;
          ks = (const T*)p.k_new + o;
          vs = (const T*)p.v_new + o;
        }
        const u32x4 kv4 = *(const u32x4*)(ks + vec * Elem<T>::kPerVec);
        const u32x4 vv4 = *(const u32x4*)(vs + vec * Elem<T>::kPerVec);
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
      const float mx = half32_max(sv);
      const float m_new = max_nan(m_run[x], mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float pv = fast_exp2(sv - m_safe);
      const float ps = half32_sum(pv);
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
    if (r < p.R) ((float*)p.part_o)[(slot * p.R + r) * D + c_pv] = acc[x];
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
  if (p.k_new != nullptr && split == 0 && chunk == 0) append_new_rows<T, D>(p, b, hk);
}

// =================================================================================================
// MFMA partial kernel (bf16): helpers
// =================================================================================================
constexpr int kMfmaTile = 32;         // tokens per tile the host-side split heuristic counts in
constexpr float kRescaleGap = 8.f;    // log2 units, see the lazy rescale in the kernel

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// =================================================================================================
// MFMA partial kernel (bf16): query-row blocks x token groups
// =================================================================================================
// Grid (S, H_kv, B * n_chunks): a block owns one KV slice and up to RB*16 query rows, and has
// RB * TG waves.  Wave (rb, tg) owns query rows 16*rb..16*rb+15 and, of every "super-tile" of TG
// consecutive TT-token tiles, tile number tg.  A wave's state is one 16-row accumulator (32
// registers at d = 128), so 12-16 waves fit on a compute unit and hide each other's MFMA / LDS /
// exp latencies; at the end the TG states of a row block meet in LDS and wave (rb, tg) reduces and
// stores head-dim blocks tg, tg + TG, ...
//
// Data path: K/V tiles go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no registers in
// between) into one ring of NST super-tiles shared by the block; the first ISSUERS waves issue the
// transfers.  One block barrier per super-tile says both "it has landed" (every issuer waited for
// its own transfers first) and "everyone is done with the previous one" (whose stage is refilled
// right away).  A lane's 16 bytes land at (wave-uniform base) + lane*16, so a tile is stored
// row-major and unpadded; bank conflicts are avoided by fetching, for physical 16-byte chunk c of
// row r, logical chunk c ^ swz(r).
//
// Register layouts (lane = j + 16*g, j = lane%16, g = lane/16), v_mfma_f32_16x16x32_bf16:
//   A operand: row j,  8 contraction elements of group g      B operand: column j, same 8 elements
//   D result : column j, rows 4g..4g+3
// S^T = K Q^T  -> D[token][qrow]: lane (qrow j, g) holds tokens 4g..4g+3 of a 16-token block, which
//   is exactly what the B operand of O^T = V^T P^T wants (contraction slot 4g+e = token 4g+e; with
//   32-token tiles the second block supplies slots 4..7 of each lane).  The matching V^T operand
//   (row = head-dim element j, the same tokens) comes from ds_read_b64_tr_b16, which hands lane j
//   of a 16-lane group the j-th column of a 4 x 16 block whose rows the lanes address 4 elements at
//   a time.  The contraction order of QK^T is likewise free: slot (ks, g, e) reads head-dim element
//   (g*KS + ks)*8 + e of both K and Q, which makes each lane's K reads one contiguous run.
template <int D, int TG, int TT, int NST, int ES = 2>
struct GridSmem {
  static constexpr int kRowBytes = D * ES;                     // a cache row: ES bytes per element
  static constexpr int kTileBytes = TT * kRowBytes;
  static constexpr int kSuperBytes = TG * 2 * kTileBytes;      // TG x (K tile, V tile)
  static constexpr int q_bytes(int rb) { return rb * 16 * D * 2; }   // queries are always bf16
  static constexpr int stat_bytes(int rb) { return 2 * TG * rb * 16 * 4; }
  static constexpr int xbuf_bytes(int rb) { return rb * TG * (D / 16) * 1024; }   // merge staging
  static constexpr int ring_bytes(int rb) {
    return NST * kSuperBytes > xbuf_bytes(rb) ? NST * kSuperBytes : xbuf_bytes(rb);
  }
  static constexpr int total(int rb) { return q_bytes(rb) + stat_bytes(rb) + ring_bytes(rb); }
};

//
// fp8 cache (KV8): K and V rows are E4M3 codes, one byte per element, with one fp32 multiplier per
// (batch element, KV head); queries, probabilities and the MFMA operands stay bf16.  A code becomes
// a bf16 value exactly (4 significant bits), two per v_cvt_scalef32_pk_bf16_fp8, after the LDS read;
// the K multiplier joins the softmax scale and the V multiplier the slice's output.  Two layout
// changes keep the LDS reads at one instruction per operand: K operand row m of 16-token block tb
// is tile row 8*(m/4) + 4*tb + m%4, so the 8 probabilities a lane holds belong to 8 consecutive
// tokens 8g..8g+7, and ds_read_b64_tr_b8 (lane i of a 16-lane group addresses 8 bytes of row i/2,
// lane j receives column j of the 8 rows) then fetches exactly those 8 tokens of V^T in one read.
template <int D, bool KV8>
__device__ __forceinline__ int tile_swizzle(int r) {
  if constexpr (!KV8) return lds_row_swizzle<D>(r);
  // 128-byte rows: the K reads of 16 lanes touch rows {0-3, 8-11, 16-19, 24-27} (+4), the V reads of
  // 32 lanes 16 consecutive rows; both must spread over the 16 16-byte slots of 256 bytes
  else if constexpr (D == 128) return ((r >> 1) ^ ((r >> 3) & 2)) & 7;
  else return ((r >> 2) + (r >> 4)) & 3;               // 64-byte rows
}

// four E4M3 codes of one dword -> bf16, exact
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) int i32x2_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
__device__ __forceinline__ bf16x8 e4m3x8_to_bf16(int lo, int hi) {
  const bf16x2_t a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
  const bf16x2_t b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
  const bf16x2_t c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
  const bf16x2_t d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
  return __builtin_shufflevector(__builtin_shufflevector(a, b, 0, 1, 2, 3),
                                 __builtin_shufflevector(c, d, 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
}

// TT = tokens per tile (16 or 32), NST = ring stages (super-tiles resident in LDS)
// MODE: 0 = contiguous cache, 1 = contiguous cache with appended-row fusion, 2 = paged cache
template <int D, int RB, int TG, int TT, int NST, int MODE, bool KV8 = false, bool NT = false, bool ROT = false>
__global__ __launch_bounds__(RB * TG * 64) void attn_partial_grid(AttnParams p) {
  constexpr bool APPEND = MODE == 1, PAGED = MODE == 2;
  constexpr int ES = KV8 ? 1 : 2;                      // bytes per cache element
  using SM = GridSmem<D, TG, TT, NST, ES>;
  constexpr int WAVES = RB * TG;
  constexpr int KS = D / 32;
  constexpr int DB = D / 16;
  constexpr int TB = TT / 16;                          // 16-token blocks per tile
  constexpr int ROWB = SM::kRowBytes;
  constexpr int CPR = ROWB / 16;                       // 16-byte chunks per cache row
  constexpr int RPI = 64 / CPR;
  constexpr int NLD = TT / RPI;                        // transfers per K (or V) tile
  constexpr int QROWB = D * 2, QCPR = D / 8, QRPI = 64 / QCPR;   // the bf16 query block's layout
  constexpr int NQ = RB * 16 / QRPI;                   // transfers for the query block
  static_assert(!KV8 || (MODE == 0 && TT == 32), "the fp8 cache path: contiguous caches, 32-token tiles");
  constexpr int XFERS = TG * 2 * NLD;                  // transfers per super-tile
  constexpr int ISS0 = WAVES >= 8 ? 8 : (WAVES >= 4 ? 4 : (WAVES >= 2 ? 2 : 1));   // power of two <= WAVES
  constexpr int ISSUERS = XFERS < ISS0 ? XFERS : ISS0;
  constexpr int PER = XFERS / ISSUERS;                 // transfers per issuing wave per super-tile
  static_assert(XFERS % ISSUERS == 0 && PER * (NST - 1) <= 63, "transfer split");
  static_assert(DB % TG == 0, "head-dim blocks must split over the token groups");
  static_assert(TT == 16 || TT == 32, "tile size");

  // verification is the critical path of a decoding round: its waves win the issue arbitration
  // against the draft call's waves that share a compute unit with them
  if (p.wave_prio) __builtin_amdgcn_s_setprio(2);
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Qs = smem;
  float* stat_m = (float*)(smem + SM::q_bytes(RB));          // [TG][RB*16]
  float* stat_l = stat_m + TG * RB * 16;
  unsigned char* ring = smem + SM::q_bytes(RB) + SM::stat_bytes(RB);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rb = wave % RB, tg = wave / RB;
  const int j = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, hk = blockIdx.y;
  // (the usual single row chunk needs no division: nothing that can be avoided stands in front of the
  // block's first transfer)
  const int b = p.n_chunks == 1 ? (int)blockIdx.z : (int)(blockIdx.z / p.n_chunks);
  const int chunk = p.n_chunks == 1 ? 0 : (int)(blockIdx.z % p.n_chunks);
  const int r0 = chunk * (RB * 16);
  const float inv_g = __builtin_amdgcn_rcpf((float)p.G);

  // fp8 cache: the K multiplier scales the logits, the V multiplier the slice's output.  Fetched
  // first, through the scalar cache (a vector load here would sit behind every K/V transfer in the
  // same counter, and waiting for it would wait for the whole ring).
  float k_mult = 1.f, v_mult = 1.f;
  if constexpr (KV8) {
    const int bh = __builtin_amdgcn_readfirstlane(b * p.Hkv + hk);
    k_mult = p.k_scale[bh];
    v_mult = p.v_scale[bh];
  }
  const unsigned ring_addr = (unsigned)(uintptr_t)ring;
  const unsigned q_addr = (unsigned)(uintptr_t)Qs;
  // paged: the pools' base plus the head offset; the page and the row inside it are added per transfer
  const char* kbase = (const char*)p.k + ((PAGED ? 0ll : (long long)b * p.sb) + (long long)hk * p.sh) * ES;
  const char* vbase = (const char*)p.v + ((PAGED ? 0ll : (long long)b * p.sb) + (long long)hk * p.sh) * ES;
  const unsigned row_bytes = (unsigned)(p.sn * ES);        // the host caps the row stride at 2^24 elements
  const int ld_row = lane / CPR, ld_pc = lane % CPR;

  // the tiles are dealt to the S slices as evenly as possible, the first n_tiles % S slices taking
  // one more (32-bit arithmetic: this runs before the first transfer can be issued)
  const int tq = p.tiles_q, tr = p.tiles_r;   // n_tiles / S and n_tiles % S for this kernel's tile size, from the host
  const int t_lo = split * tq + min(split, tr);
  const int t_hi = t_lo + tq + (split < tr ? 1 : 0);
  const int n_blk = t_hi - t_lo;                           // tiles of this block
  const int n_super = (n_blk + TG - 1) / TG;
  // ROT (long slices): the softmax state does not care in which order a slice's tiles arrive, so every
  // (batch element, KV head) starts its slices at a different phase and wraps around.  Blocks that
  // would otherwise walk their slices in lockstep, a fixed stride apart, then spread over the memory
  // channels (4 sequences x 8 KV heads x 37K rows in 8 slices: 10 % faster).  The phase is this head's
  // share of the slice, in single precision: any value in range serves, and an integer division here
  // would sit in front of the block's first transfer.
  int phase = 0;
  if constexpr (ROT)
    phase = __builtin_amdgcn_readfirstlane(   // wave-uniform: keep it in a scalar register
        min((int)((float)(b * p.Hkv + hk) * (float)n_super * p.phase_per_head), max(n_super - 1, 0)));
  auto super_at = [&](int si) {
    if constexpr (!ROT) return si;
    const int x = si + phase;
    return x >= n_super ? x - n_super : x;
  };

  // issuing wave w moves transfers x = w*PER .. w*PER+PER-1 of a super-tile:
  //   x -> tile tt = x / (2 NLD), K or V = (x / NLD) & 1, 1 KB piece n = x % NLD
  // tiles past the block's range and rows past the cache's end re-read the block's last valid row
  // (a cache hit), so every super-tile costs every issuer exactly PER transfers
  const int row_cap = min(t_hi * TT, p.n_total) - 1;       // 32-bit row numbers: the host caps the cache length
  // paged: the page numbers of the rows this block streams, staged in LDS once (table entries
  // outside the pool are clamped into it, so a bad table cannot send a transfer out of bounds)
  int* page_s = (int*)(smem + SM::total(RB));
  const int page_mask = PAGED ? (1 << p.page_shift) - 1 : 0;
  const int slot_lo = PAGED ? (t_lo * TT) >> p.page_shift : 0;
  if (PAGED) {
    const int n_slots = n_blk > 0 ? (row_cap >> p.page_shift) - slot_lo + 1 : 0;
    for (int i = tid; i < n_slots && i < kMaxSlicePages; i += RB * TG * 64) {
      int pg = p.block_table[(long long)b * p.max_pages + slot_lo + i];
      pg = pg < 0 ? 0 : (pg >= p.n_pool_pages ? p.n_pool_pages - 1 : pg);
      page_s[i] = pg;
    }
    __syncthreads();
  }
  auto issue_super = [&](int si) {
    const unsigned dst = ring_addr + (si % NST) * SM::kSuperBytes;
    const int tile0 = t_lo + super_at(si) * TG;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int x = wave * PER + u;
      const int tt = x / (2 * NLD), which = (x / NLD) & 1, n = x % NLD;
      const int r = n * RPI + ld_row;
      const int row = min((tile0 + tt) * TT + r, row_cap);
      const char* src = (which ? vbase : kbase) + (unsigned long long)(unsigned)row * row_bytes;   // one 32 x 32 -> 64 multiply-add
      if (PAGED)
        src = (which ? vbase : kbase) + ((long long)page_s[(row >> p.page_shift) - slot_lo] * p.page_stride +
                                         (long long)(row & page_mask) * p.sn) * 2;
      if (APPEND && row >= p.ctx_len)                      // a row that has not reached the cache yet
        src = (const char*)(which ? p.v_new : p.k_new) +
              ((((long long)b * p.q_len + (row - p.ctx_len)) * p.Hkv + hk) * D) * 2;
      dma16<NT>(src + ((ld_pc ^ tile_swizzle<D, KV8>(r)) * 16), dst + (tt * 2 + which) * SM::kTileBytes + n * 1024);
    }
  };
  // ---- prologue: the first ring stage goes out before anything else (its bytes are the ones
  // the first products wait for), then the query block, then the remaining stages.  Transfers
  // complete in issue order, so the wait for super-tile 0 below also covers the query block. ----
  const bool issuer = wave < ISSUERS;
  int issued = n_super < NST ? n_super : NST;              // super-tiles requested so far
  // Appended rows: the block that copies them into the cache fetches them now, ahead of every transfer
  // (loads return in order, so the transfer counts waited for below are not disturbed), and stores them
  // after its slice: the copy's trip to memory hides behind the stream instead of following it.
  const bool appends = APPEND && split == 0 && chunk == 0;
  constexpr int APR = D / 8;                               // 16-byte pieces per bf16 row
  const bool append_early = appends && p.q_len * APR <= WAVES * 64;
  u32x4 app_k = {0u, 0u, 0u, 0u}, app_v = {0u, 0u, 0u, 0u};
  if (APPEND && append_early && (int)threadIdx.x < p.q_len * APR) {
    const long long src = (((long long)b * p.q_len + threadIdx.x / APR) * p.Hkv + hk) * D + (threadIdx.x % APR) * 8;
    app_k = *(const u32x4*)((const uint16_t*)p.k_new + src);
    app_v = *(const u32x4*)((const uint16_t*)p.v_new + src);
  }
  if (issuer && issued > 0) issue_super(0);
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    if ((n % WAVES) == wave) {
      const int rr = n * QRPI + lane / QCPR;
      int r = r0 + rr;
      r = r < p.R ? r : p.R - 1;                          // padding rows repeat the last real row
      const int i = row_div_group(r, inv_g), gq = r - i * p.G;
      const char* src = (const char*)p.q + ((((long long)b * p.q_len + i) * p.H + hk * p.G + gq) * D) * 2 +
                        (((lane % QCPR) ^ tile_swizzle<D, false>(rr)) * 16);
      dma16(src, q_addr + n * 1024);
    }
  }
  if (issuer)
    for (int si = 1; si < issued; ++si) issue_super(si);

  const int row = r0 + rb * 16 + j;                       // this lane's query row
  const int lim = (row < p.R) ? p.ctx_len + row_div_group(row, inv_g) : 0x7fffffff;
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) acc[db] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // bf16 cache: k_off[ks] is the lane's 16-byte K operand of contraction step ks in row j (the
  // query block uses the same offsets).  fp8 cache: a lane's KS*8 bytes of a row are NKC 16-byte
  // chunks, and k_off[tb * NKC + c] is chunk c in the permuted row of 16-token block tb.
  constexpr int NKC = KS / 2;
  constexpr int NKOFF = KV8 ? TB * NKC : KS;
  unsigned k_off[NKOFF];
  unsigned v_off[DB];
  if constexpr (!KV8) {
    const int swz_k = tile_swizzle<D, false>(j);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_off[ks] = j * ROWB + (((g * KS + ks) ^ swz_k) * 16);
    const int v_row = 4 * g + (j >> 2);
    const int swz_v = tile_swizzle<D, false>(v_row);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      v_off[db] = v_row * ROWB + (((2 * db + ((j & 3) >> 1)) ^ swz_v) * 16) + (j & 1) * 8;
  } else {
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int k_row = 8 * (j >> 2) + 4 * tb + (j & 3);
#pragma unroll
      for (int c = 0; c < NKC; ++c)
        k_off[tb * NKC + c] = k_row * ROWB + (((g * NKC + c) ^ tile_swizzle<D, true>(k_row)) * 16);
    }
    const int v_row = 8 * g + (j >> 1);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      v_off[db] = v_row * ROWB + ((db ^ tile_swizzle<D, true>(v_row)) * 16) + (j & 1) * 8;
  }
  // keep the swizzled lane offsets in registers: left to itself the compiler recomputes them from
  // (j, g) for every tile, which costs more vector instructions than the tile's arithmetic
#pragma unroll
  for (int i = 0; i < NKOFF; ++i) asm volatile("" : "+v"(k_off[i]));
#pragma unroll
  for (int db = 0; db < DB; ++db) asm volatile("" : "+v"(v_off[db]));
  const float scale_log2 = KV8 ? p.scale_log2 * k_mult : p.scale_log2;

  bf16x8 qop[KS];

  for (int si = 0; si < n_super; ++si) {
    // Transfers complete in issue order, so "at most PER * (super-tiles requested after si)
    // outstanding" means super-tile si (and Q) has landed.  Waves that issue no tile transfers
    // only ever have their share of Q in flight.
    if (issuer) WaitLadder<NST - 1>::template run<PER>(issued - 1 - si); else wait_vmcnt<0>();
    __syncthreads();           // super-tile si complete in LDS; everyone is past super-tile si-1
    if (si == 0) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        qop[ks] = *(const bf16x8*)(Qs + rb * 16 * QROWB + j * QROWB +
                                   (((g * KS + ks) ^ tile_swizzle<D, false>(j)) * 16));
    }
    if (si > 0 && issued < n_super) {                      // refill the stage just vacated
      if (issuer) issue_super(issued);
      ++issued;
    }
    const int ti = super_at(si) * TG + tg;                 // this wave's tile inside the block
    if (ti >= n_blk) continue;                             // ragged last super-tile

    const unsigned char* Kt = ring + (si % NST) * SM::kSuperBytes + tg * 2 * SM::kTileBytes;
    const unsigned char* Vt = Kt + SM::kTileBytes;
    const int n0 = (t_lo + ti) * TT;

    f32x4 s[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) s[tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if constexpr (!KV8) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          const bf16x8 kop = *(const bf16x8*)(Kt + tb * 16 * ROWB + k_off[ks]);
          s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qop[ks], s[tb], 0, 0, 0);
        }
    } else {
#pragma unroll
      for (int c = 0; c < NKC; ++c)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          const i32x4_t kraw = *(const i32x4_t*)(Kt + k_off[tb * NKC + c]);
          s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(kraw[0], kraw[1]), qop[2 * c], s[tb], 0, 0, 0);
          s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(kraw[2], kraw[3]), qop[2 * c + 1], s[tb], 0, 0, 0);
        }
    }

    if ((n0 + TT - 1) > p.ctx_len) {                     // tile touches the causal edge
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((n0 + (KV8 ? 8 * g + 4 * tb : tb * 16 + 4 * g) + e) > lim) s[tb][e] = -INFINITY;
    }
    float sv[TB * 4];
#pragma unroll
    for (int e = 0; e < TB * 4; ++e) sv[e] = s[e >> 2][e & 3];
    const float m8 = rows4_max(max_nan_of(sv));
    const float mx = m8 * scale_log2;                      // scale > 0: max commutes with it
    // lazy rescale: the reference m_run moves only when the tile maximum exceeds it by more than
    // kRescaleGap, so probabilities stay below 2^kRescaleGap and rescales are rare
    const bool up = mx > m_run + kRescaleGap;              // also true for the first finite maximum
    if (__any(up)) {
      const float a = up ? fast_exp2(m_run - mx) : 1.f;    // m_run = -inf -> 0
      if (up) m_run = mx;
      l_run *= a;
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] *= a;
    }
    const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
    // the PV product sees P rounded to bf16; the denominator sums the same rounded values.  Two
    // probabilities are rounded by one packed conversion and read back with a shift and a mask.
    unsigned pk[TB * 2];
    float psum = 0.f;
#pragma unroll
    for (int h = 0; h < TB * 2; ++h) {
      typedef __attribute__((ext_vector_type(2))) float f32x2_t;
      const f32x2_t x = {fast_exp2(fmaf(s[h >> 1][(2 * h) & 3], scale_log2, neg_m)),
                         fast_exp2(fmaf(s[h >> 1][(2 * h + 1) & 3], scale_log2, neg_m))};
      pk[h] = __builtin_bit_cast(unsigned, __builtin_convertvector(x, bf16x2_t));
      psum += __uint_as_float(pk[h] << 16) + __uint_as_float(pk[h] & 0xffff0000u);
    }
    l_run += psum;                                         // per-lane share; groups g meet at the end

    if (TB == 2) {
      const bf16x8 pop = __builtin_bit_cast(bf16x8, (i32x4_t){(int)pk[0], (int)pk[1], (int)pk[2 % (TB * 2)], (int)pk[3 % (TB * 2)]});
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        if constexpr (KV8) {
          const i32x2_t vraw = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
              (__attribute__((address_space(3))) i32x2_t*)(Vt + v_off[db]));
          acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(vraw[0], vraw[1]), pop, acc[db], 0, 0, 0);
        } else {
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(Vt + v_off[db]));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(Vt + (TB - 1) * 16 * ROWB + v_off[db]));
          const bf16x8 vop = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop, acc[db], 0, 0, 0);
        }
      }
    } else {
      const s16x4 pop = __builtin_bit_cast(s16x4, (i32x2_t){(int)pk[0], (int)pk[1]});
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const s16x4 vop = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(Vt + v_off[db]));
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vop, pop, acc[db], 0, 0, 0);
      }
    }
  }
  wait_vmcnt<0>();   // no transfer may still be writing LDS past this point

  // ---- merge the TG token groups of every row block ----
  l_run = rows4_sum(l_run);
  if (g == 0) {
    stat_m[tg * RB * 16 + rb * 16 + j] = m_run;
    stat_l[tg * RB * 16 + rb * 16 + j] = l_run;
  }
  f32x4* xbuf = (f32x4*)ring;                              // [WAVES][DB][64 lanes]
  __syncthreads();   // (a) every wave is done reading the ring before anyone overwrites it
  // a wave finishes head-dim blocks tg, tg + TG, ...: those stay in its registers, only the blocks
  // that other waves finish go through LDS.  The body is instantiated once per value of tg (it is
  // wave-uniform), so which blocks stay and which travel is known at compile time: straight-line
  // code whose LDS reads all go out before the first one is needed.
  const long long slot = ((long long)b * p.Hkv + hk) * p.S + split;
  auto finish = [&](auto tgc) {
    constexpr int TGC = decltype(tgc)::value;
#pragma unroll
    for (int db = 0; db < DB; ++db)
      if (db % TG != TGC) xbuf[(wave * DB + db) * 64 + lane] = acc[db];
    __syncthreads();   // (b) accumulators and statistics of all waves visible
    f32x4 other[TG][DB / TG];                                // [source wave group][own head-dim block]
#pragma unroll
    for (int w = 0; w < TG; ++w)
#pragma unroll
      for (int dd = 0; dd < DB / TG; ++dd)
        if (w != TGC) other[w][dd] = xbuf[((w * RB + rb) * DB + TGC + TG * dd) * 64 + lane];
    float mw[TG], mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < TG; ++w) { mw[w] = stat_m[w * RB * 16 + rb * 16 + j]; mm = max_nan(mm, mw[w]); }
    float f[TG], ll = 0.f;
#pragma unroll
    for (int w = 0; w < TG; ++w) {
      f[w] = (mw[w] == -INFINITY) ? 0.f : fast_exp2(mw[w] - mm);
      ll = fmaf(f[w], stat_l[w * RB * 16 + rb * 16 + j], ll);
    }
    if constexpr (KV8) {
#pragma unroll
      for (int w = 0; w < TG; ++w) f[w] *= v_mult;         // after the denominator took the plain weights
    }
#pragma unroll
    for (int dd = 0; dd < DB / TG; ++dd) {
      const int db = TGC + TG * dd;
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < TG; ++w) {
        if (w == TGC) o += acc[TGC + TG * dd] * f[w];
        else o += other[w][dd] * f[w];
      }
      // the slice's output leaves as bf16 (the merge weighs and sums it in fp32): half the bytes to write
      // here and to fetch in the merge, and the rounding is one more of the size the output's own has
      if (row < p.R) {
        typedef __attribute__((ext_vector_type(2))) float f32x2_t;
        const f32x2_t lo = {o[0], o[1]}, hi = {o[2], o[3]};
        uint2 w;
        w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2_t));
        w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2_t));
        *(uint2*)((uint16_t*)p.part_o + (slot * p.R + row) * D + db * 16 + 4 * g) = w;
      }
    }
    if (TGC == 0 && g == 0 && row < p.R) {
      p.part_m[slot * p.R + row] = mm;
      p.part_l[slot * p.R + row] = ll;
    }
  };
  static_assert(TG == 1 || TG == 2 || TG == 4, "token groups");
  if (tg == 0) finish(std::integral_constant<int, 0>());
  else if (tg == 1) finish(std::integral_constant<int, 1>());
  else if (tg == 2) finish(std::integral_constant<int, 2 % TG>());
  else finish(std::integral_constant<int, 3 % TG>());
  if (APPEND && appends) {
    if (append_early) {
      if ((int)threadIdx.x < p.q_len * APR) {
        const long long dst = (long long)b * p.sb + (long long)hk * p.sh +
                              (long long)(p.ctx_len + threadIdx.x / APR) * p.sn + (threadIdx.x % APR) * 8;
        *(u32x4*)((uint16_t*)p.k_w + dst) = app_k;
        *(u32x4*)((uint16_t*)p.v_w + dst) = app_v;
      }
    } else {
      append_new_rows<uint16_t, D>(p, b, hk);
    }
  }
}

// =================================================================================================
// Merge of the KV slices: out = sum_s 2^(m_s - m*) o_s / sum_s 2^(m_s - m*) l_s
// The slices' outputs o_s are fp32 (PO16 = false: the vector-ALU kernel's) or bf16 (the MFMA kernel's).
// One block per (query row, KV head, batch element).  The slices are spread over the threads: first
// the S weights (one slice per thread, block-wide max and sum), then thread (sg, vec) accumulates
// 16-byte vector `vec` of the row over slices sg, sg + NSG, ... and the NSG groups meet in LDS.
// =================================================================================================
constexpr int kMaxSplits = 1024;

// four consecutive elements of a slice's output; for bf16 the raw bits travel in the first two components
// until the weights are known (the loads must all be in flight before anything waits for one of them)
template <bool PO16>
__device__ __forceinline__ f32x4 part_o_load4(const void* base, long long elem) {
  if constexpr (!PO16) return *(const f32x4*)((const float*)base + elem);
  else {
    const uint2 w = *(const uint2*)((const uint16_t*)base + elem);
    return (f32x4){__uint_as_float(w.x), __uint_as_float(w.y), 0.f, 0.f};
  }
}
template <bool PO16>
__device__ __forceinline__ f32x4 part_o_widen(f32x4 raw) {
  if constexpr (!PO16) return raw;
  else {
    const unsigned x = __float_as_uint(raw[0]), y = __float_as_uint(raw[1]);
    return (f32x4){__uint_as_float(x << 16), __uint_as_float(x & 0xffff0000u), __uint_as_float(y << 16),
                   __uint_as_float(y & 0xffff0000u)};
  }
}

template <typename T, int D, bool PO16>
__global__ __launch_bounds__(256) void attn_combine(AttnParams p) {
  constexpr int VPR = D / 4;           // four-element vectors per row
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
    const int s = min(sg + u * NSG, p.S - 1);             // past the last slice: a harmless repeat, not used
    pre[u] = part_o_load4<PO16>(p.part_o, ((slot0 + s) * p.R + r) * D + vec * 4);
  }

  // where the row's output goes: worked out while the loads are in flight (the division would otherwise
  // stand between the last barrier and the store)
  const int i_row = r / p.G, h_row = hk * p.G + (r - i_row * p.G);
  long long out_at = (((long long)b * p.q_len + i_row) * p.H + h_row) * D + (tid % VPR) * 4;
  long long lse_at = ((long long)b * p.H + h_row) * p.q_len + i_row;
  asm volatile("" : "+v"(out_at), "+v"(lse_at));

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float mstar, den;
  if (p.S <= 64) {
    // up to 64 slices: every wave holds all slice statistics (one per lane), so the reference
    // maximum, the weights and the denominator need no LDS and no barrier; a weight reaches the
    // thread that needs it through a lane shuffle
    const int lane = tid & 63;
    const float ms = lane < p.S ? p.part_m[(slot0 + lane) * p.R + r] : -INFINITY;
    const float ls = lane < p.S ? p.part_l[(slot0 + lane) * p.R + r] : 0.f;
    mstar = wave_max(ms);
    const float w = (ms == -INFINITY) ? 0.f : fast_exp2(ms - mstar);
    den = wave_sum(w * ls);
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int sl = sg + u * NSG;                        // < 64 whenever it is < S
      const float ws = __shfl(w, sl & 63, 64);
      if (sl < p.S) acc += part_o_widen<PO16>(pre[u]) * ws;
    }
  } else {
    // this thread's first slice statistics ride in the same trip
    const float m0 = tid < p.S ? p.part_m[(slot0 + tid) * p.R + r] : -INFINITY;
    const float l0 = tid < p.S ? p.part_l[(slot0 + tid) * p.R + r] : 0.f;
    float mloc = m0;
    for (int s2 = tid + 256; s2 < p.S; s2 += 256) mloc = max_nan(mloc, p.part_m[(slot0 + s2) * p.R + r]);
    mloc = wave_max(mloc);
    if ((tid & 63) == 0) red[tid >> 6] = mloc;
    __syncthreads();
    mstar = max_nan(max_nan(red[0], red[1]), max_nan(red[2], red[3]));
    float dloc = 0.f;
    if (tid < p.S) {
      const float w = (m0 == -INFINITY) ? 0.f : fast_exp2(m0 - mstar);
      w_s[tid] = w;
      dloc = w * l0;
    }
    for (int s2 = tid + 256; s2 < p.S; s2 += 256) {
      const float ms = p.part_m[(slot0 + s2) * p.R + r];
      const float w = (ms == -INFINITY) ? 0.f : fast_exp2(ms - mstar);
      w_s[s2] = w;
      dloc = fmaf(w, p.part_l[(slot0 + s2) * p.R + r], dloc);
    }
    dloc = wave_sum(dloc);
    if ((tid & 63) == 0) red[4 + (tid >> 6)] = dloc;
    __syncthreads();
    den = red[4] + red[5] + red[6] + red[7];
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int sl = sg + u * NSG;
      if (sl < p.S) acc += part_o_widen<PO16>(pre[u]) * w_s[sl];
    }
#pragma unroll 4
    for (int sl = sg + PF * NSG; sl < p.S; sl += NSG) {
      const f32x4 o = part_o_widen<PO16>(part_o_load4<PO16>(p.part_o, ((slot0 + sl) * p.R + r) * D + vec * 4));
      acc += o * w_s[sl];
    }
  }
  acc_s[sg][vec] = acc;
  __syncthreads();
  if (tid < VPR) {
    f32x4 t = acc_s[0][tid];
#pragma unroll
    for (int g2 = 1; g2 < NSG; ++g2) t += acc_s[g2][tid];
    const float inv = 1.f / den;
    T* o = (T*)p.out + out_at;
    if constexpr (sizeof(T) == 2) {                        // four bf16 values: one 8-byte store
      typedef __attribute__((ext_vector_type(2))) float f32x2_t;
      const f32x2_t lo = {t[0] * inv, t[1] * inv}, hi = {t[2] * inv, t[3] * inv};
      uint2 w;
      w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2_t));
      w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2_t));
      *(uint2*)o = w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) Elem<T>::store(o + e, t[e] * inv);
    }
    if (p.lse != nullptr && tid == 0) p.lse[lse_at] = (mstar + __log2f(den)) * kLn2;
  }
}

// =================================================================================================
// host launch
// =================================================================================================
template <int D, int RB, int TG, int TT, int NST, int MODE, bool KV8 = false, bool NT = false, bool ROT = false>
static hipError_t launch_grid_mode(const AttnParams& p, hipStream_t st) {
  // the paged variant keeps its slice of the page table behind the ring
  constexpr int smem = GridSmem<D, TG, TT, NST, KV8 ? 1 : 2>::total(RB) + (MODE == 2 ? kMaxSlicePages * 4 : 0);
  // the attribute belongs to a (kernel, device) pair: set it once for each device this process uses
  static std::atomic<unsigned long long> attr_set{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (!(attr_set.load(std::memory_order_acquire) & bit)) {
    e = hipFuncSetAttribute((const void*)attn_partial_grid<D, RB, TG, TT, NST, MODE, KV8, NT, ROT>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set.fetch_or(bit, std::memory_order_release);
  }
  dim3 grid(p.S, p.Hkv, p.B * p.n_chunks);
  AttnParams q = p;                               // the slices' tile counts for this kernel's tile size
  const int n_tiles = (p.n_total + TT - 1) / TT;
  q.tiles_q = n_tiles / p.S;
  q.tiles_r = n_tiles % p.S;
  hipLaunchKernelGGL((attn_partial_grid<D, RB, TG, TT, NST, MODE, KV8, NT, ROT>), grid, dim3(RB * TG * 64), smem, st, q);
  return hipGetLastError();
}

// the appended-row and paged variants are separate instantiations, so the plain call carries none of
// their address selects
template <int D, int RB, int TG, int TT, int NST, bool NT = false, bool ROT = false>
static hipError_t launch_grid(const AttnParams& p, hipStream_t st) {
  if (p.block_table != nullptr) return launch_grid_mode<D, RB, TG, TT, NST, 2, false, NT, ROT>(p, st);
  if (p.k_new != nullptr) return launch_grid_mode<D, RB, TG, TT, NST, 1, false, NT, ROT>(p, st);
  return launch_grid_mode<D, RB, TG, TT, NST, 0, false, NT, ROT>(p, st);
}

// A call whose K and V exceed the chip's last-level cache (256 MB) streams them with non-temporal
// transfers: nothing of such a stream can be served from a cache again, and left to itself it evicts
// the query block, the split partials and the other stream's data (measured on 4 sequences x 8 KV
// heads x 37K rows, 608 MB: 6 % faster; at 34 MB the hint costs 5 %, so short streams do not use it).
static bool stream_exceeds_caches(const AttnParams& p, int head_dim, int elem_bytes) {
  return 2ll * p.B * p.Hkv * p.n_total * head_dim * elem_bytes > (256ll << 20);
}

// Short slices (a block owns only a handful of tiles, as at 16K context on 256 compute units) use
// 16-token tiles and a deeper ring; long slices use 32-token tiles, which halve the barrier count.
template <int D, int RB>
static hipError_t launch_grid_rb(const AttnParams& p, hipStream_t st) {
  const int tiles32_per_block = ((p.n_total + 31) / 32) / (p.S > 0 ? p.S : 1);
  const bool small_tiles = tiles32_per_block < 24;
  if (!small_tiles)
    return stream_exceeds_caches(p, D, 2) ? launch_grid<D, RB, 4, 32, 2, true, true>(p, st)
                                          : launch_grid<D, RB, 4, 32, 2, false, true>(p, st);
  // measured at the 16K configuration: with 3-4 row blocks, two token groups and a four-stage ring
  // (the whole slice in flight at once) beat four groups by ~8 %; the block merge moves half the data
  // four row blocks (49-64 query rows) over slices of 12-23 32-token tiles, the 33K long-video shape:
  // the per-tile work of the vector unit weighs most there, and 32-token tiles halve it per token
  if (RB == 4 && tiles32_per_block >= 12) return launch_grid<D, RB, 2, 32, 3>(p, st);
  if (RB >= 3) return launch_grid<D, RB, 2, 16, 4>(p, st);
  return launch_grid<D, RB, 4, 16, 3>(p, st);
}

// fp8 cache: 32-token tiles only; short slices keep the whole slice in flight (two token groups, four
// ring stages), long ones use four groups and two stages
template <int D, int RB>
static hipError_t launch_kv8_rb(const AttnParams& p, hipStream_t st) {
  const int tiles32_per_block = ((p.n_total + 31) / 32) / (p.S > 0 ? p.S : 1);
  if (tiles32_per_block < 24)
    return launch_grid_mode<D, RB, 2, 32, 4, 0, true>(p, st);
  if (stream_exceeds_caches(p, D, 1)) return launch_grid_mode<D, RB, 4, 32, 2, 0, true, true, true>(p, st);
  return launch_grid_mode<D, RB, 4, 32, 2, 0, true, false, true>(p, st);
}

template <int D>
static hipError_t launch_kv8_d(const AttnParams& p, hipStream_t st) {
  switch (p.row_chunk / 16) {
    case 1: return launch_kv8_rb<D, 1>(p, st);
    case 2: return launch_kv8_rb<D, 2>(p, st);
    case 3: return launch_kv8_rb<D, 3>(p, st);
    default: return launch_kv8_rb<D, 4>(p, st);
  }
}

template <int D>
static hipError_t launch_mfma_d(const AttnParams& p, hipStream_t st) {
  switch (p.row_chunk / 16) {
    case 1: return launch_grid_rb<D, 1>(p, st);
    case 2: return launch_grid_rb<D, 2>(p, st);
    case 3: return launch_grid_rb<D, 3>(p, st);
    default: return launch_grid_rb<D, 4>(p, st);
  }
}

template <typename T, int D>
static hipError_t launch_valu(const AttnParams& p, hipStream_t st) {
  dim3 grid(p.S, p.Hkv, p.B * p.n_chunks);
  hipLaunchKernelGGL((attn_partial_valu<T, D>), grid, dim3(256), 0, st, p);
  return hipGetLastError();
}

template <typename T, int D, bool PO16>
static hipError_t launch_combine(const AttnParams& p, hipStream_t st) {
  hipLaunchKernelGGL((attn_combine<T, D, PO16>), dim3(p.R, p.Hkv, p.B), dim3(256), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_attention(const AttnParams& p, int dtype, int head_dim, bool use_mfma, hipStream_t st) {
  hipError_t e;
  if (dtype == HIPPO_DTYPE_BF16) {
    if (p.k_scale != nullptr) e = (head_dim == 128) ? launch_kv8_d<128>(p, st) : launch_kv8_d<64>(p, st);
    else if (use_mfma) e = (head_dim == 128) ? launch_mfma_d<128>(p, st) : launch_mfma_d<64>(p, st);
    else return hipErrorInvalidValue;       // 16- and 8-bit caches have no vector-ALU path
    if (e != hipSuccess) return e;
    return (head_dim == 128) ? launch_combine<uint16_t, 128, true>(p, st) : launch_combine<uint16_t, 64, true>(p, st);
  }
  e = (head_dim == 128) ? launch_valu<float, 128>(p, st) : launch_valu<float, 64>(p, st);
  if (e != hipSuccess) return e;
  return (head_dim == 128) ? launch_combine<float, 128, false>(p, st) : launch_combine<float, 64, false>(p, st);
}

}  // namespace hippo
