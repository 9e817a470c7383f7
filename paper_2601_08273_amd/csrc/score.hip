// Semantic-aware token scoring (paper: Method, "Semantic-aware Token Preservation", Eq. 2-7).
//
//   s_attn  (Eq. 2)   two passes over the visual keys: pass 1 finds every text row's softmax
//                     normaliser over the N_v visual keys, pass 2 recomputes the logits and sums
//                     exp(z - lse_row) down the columns.  A block owns a tile of tokens (its keys
//                     stay in registers / LDS) and sweeps all L_txt*G query rows of the KV head.
//   s_temp, s_spa (Eq. 3-6)  one block per crop: the crop's embeddings and those of the same
//                     positions in the two neighbouring frames pass through LDS in channel chunks;
//                     the crop's Gram matrix and the temporal dot products accumulate in registers.
//   fusion (Eq. 7)    one block per frame: per-term mean / population std, z-scores summed.
#include "common.h"

namespace hippo {

// =================================================================================================
// s_attn, vector-ALU version (fp32 inputs).  PASS 1: row statistics; PASS 2: column sums.
// Block: 32 tokens x all rows (in chunks of 32); thread = (token tid%32, row group tid/32).
// =================================================================================================
constexpr int kSaValuTile = 32;

// Where pass 1 leaves the (max, sum) of query row r = i*G + g of KV head hk for token tile `tile`:
// tile-major slabs of all Bz*H*L rows in (bz, hk, r) order, so a block writes consecutive floats and
// the merge reads consecutive rows; bz = layer * B + b counts (layer, batch element) pairs when several
// layers are swept in one launch.  row_lse uses the same (bz, hk, r) order.
__device__ __forceinline__ long long sattn_part_at(const ScoreParams& p, int tile, int b, int hk, int r) {
  return (long long)tile * ((long long)p.Bz * p.H * p.L) + ((long long)b * p.Hkv + hk) * ((long long)p.L * p.G) + r;
}

template <typename T, int D, int PASS>
__global__ __launch_bounds__(256) void sattn_valu(ScoreParams p) {
  constexpr int TT = kSaValuTile, RC = 32;
  constexpr int VPR = D / Elem<T>::kPerVec;
  __shared__ float Ks[TT][D + 1];
  __shared__ float Qs[RC][D + 1];
  __shared__ float lse_s[RC];
  __shared__ float col_s[8][TT];

  const int tid = threadIdx.x, tok = tid & 31, rg = tid >> 5;
  const int tile = blockIdx.x, hk = blockIdx.y, bz = blockIdx.z;
  const int b = bz % p.B, layer = bz / p.B;          // several layers' sweeps share a launch
  const int n0 = tile * TT;
  const int Rs = p.L * p.G;
  const float scale_log2 = rsqrtf((float)D) * kLog2e;

  const T* kbase = (const T*)p.k_layers[layer] + (long long)b * p.sb + (long long)hk * p.sh +
                   (long long)p.vis_off * p.sn;
  const T* qlayer = (const T*)p.q_layers[layer];
  for (int e = tid; e < TT * VPR; e += 256) {
    const int row = e / VPR, vec = e % VPR, n = n0 + row;
    float kf[Elem<T>::kPerVec];
    if (n < p.Nv) {
      const u32x4 kv4 = *(const u32x4*)(kbase + (long long)n * p.sn + vec * Elem<T>::kPerVec);
      Elem<T>::unpack(kv4, kf);
    } else {
#pragma unroll
      for (int u = 0; u < Elem<T>::kPerVec; ++u) kf[u] = 0.f;
    }
#pragma unroll
    for (int u = 0; u < Elem<T>::kPerVec; ++u) Ks[row][vec * Elem<T>::kPerVec + u] = kf[u];
  }

  const bool tok_ok = (n0 + tok) < p.Nv;
  float col = 0.f;
  for (int r0 = 0; r0 < Rs; r0 += RC) {
    __syncthreads();
    for (int e = tid; e < RC * D; e += 256) {
      const int rr = e / D, c = e % D, r = r0 + rr;
      float val = 0.f;
      if (r < Rs) {
        const int i = r / p.G, gq = r % p.G;
        val = Elem<T>::load(qlayer + (((long long)b * p.L + i) * p.H + hk * p.G + gq) * D + c);
      }
      Qs[rr][c] = val;
    }
    if (PASS == 2 && tid < RC) {
      const int r = r0 + tid;
      float v = INFINITY;   // padding rows contribute exp2(-inf) = 0
      if (r < Rs) v = p.row_lse[((long long)bz * p.Hkv + hk) * Rs + r];
      lse_s[tid] = v;
    }
    __syncthreads();
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < D; ++c) {
      const float kc = Ks[tok][c];
#pragma unroll
      for (int x = 0; x < 4; ++x) s[x] = fmaf(kc, Qs[rg + 8 * x][c], s[x]);
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int r = r0 + rg + 8 * x;
      const float sv = tok_ok ? s[x] * scale_log2 : -INFINITY;
      if (PASS == 1) {
        const float mx = half32_max(sv);
        const float ps = half32_sum(fast_exp2(sv - mx));      // the tile always holds at least one valid token
        if (tok == 0 && r < Rs) {
          const long long at = sattn_part_at(p, tile, bz, hk, r);
          p.row_m[at] = mx;
          p.row_l[at] = ps;
        }
      } else {
        col += fast_exp2(sv - lse_s[rg + 8 * x]);
      }
    }
  }
  if (PASS == 2) {
    col_s[rg][tok] = col;
    __syncthreads();
    if (tid < TT && (n0 + tid) < p.Nv) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) t += col_s[w][tid];
      p.col_part[((long long)bz * p.Hkv + hk) * p.Nv + n0 + tid] = t;
    }
  }
}

// =================================================================================================
// s_attn, MFMA version (bf16).  Block = 8 waves x 32 tokens; each wave keeps its 32 keys as MFMA A
// operands in registers for the whole sweep over the query rows, which are staged through LDS in
// chunks of 64 rows.  Z^T = K Q^T: lane (row j, group g) holds tokens tb*16 + 4g + e.
// =================================================================================================
constexpr int kSaMfmaTile = 256;      // tokens per block
constexpr int kSaWaves = 8;           // waves per block, 32 tokens each: two waves per SIMD overlap MFMA and exp

template <int D, int PASS>
struct SattnSmem {
  static constexpr int RCH = 64;                 // query rows per LDS chunk
  static constexpr int ROWB = D * 2;             // unpadded rows, 16-byte pieces XOR-swizzled (lds_row_swizzle)
  static constexpr int RDEF = 256;               // pass 1 merges the waves' row statistics every RDEF rows
  __align__(16) unsigned char Qs[2][RCH * ROWB]; // two chunks: the next one lands while this one is multiplied
  float lse_s[2][RCH];
  float wm_s[PASS == 1 ? kSaWaves : 1][PASS == 1 ? RDEF : 1];
  float wl_s[PASS == 1 ? kSaWaves : 1][PASS == 1 ? RDEF : 1];
};

template <int D, int PASS>
__device__ __forceinline__ void sattn_mfma_body(const ScoreParams& p, SattnSmem<D, PASS>& sm, const int tile,
                                                const int vhk, const int bz) {
  const int b = bz % p.B, layer = bz / p.B;          // several layers' sweeps share a launch
  constexpr int NW = kSaWaves, NT = NW * 64;
  constexpr int TPW = kSaMfmaTile / NW;   // tokens per wave
  constexpr int TBW = TPW / 16;           // 16-token blocks per wave
  constexpr int KS = D / 32;
  constexpr int ROWB = SattnSmem<D, PASS>::ROWB;
  constexpr int CPR = D / 8;
  constexpr int RCH = SattnSmem<D, PASS>::RCH;
  constexpr int RDEF = SattnSmem<D, PASS>::RDEF;
  unsigned char* Qs = &sm.Qs[0][0];
  auto& wm_s = sm.wm_s;
  auto& wl_s = sm.wl_s;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int n0 = tile * kSaMfmaTile + wave * TPW;    // first token of this wave
  const int Rs = p.L * p.G;
  const float scale_log2 = rsqrtf((float)D) * kLog2e;
  // the query rows of a KV head are cut into n_rsplit runs of whole chunks; this block sweeps one
  // (vhk = KV head + H_kv * run)
  const int hk = vhk % p.Hkv, rs = vhk / p.Hkv;
  const int row_begin = rs * p.rows_per_split;
  const int row_end = min(Rs, row_begin + p.rows_per_split);

  const uint16_t* kbase = (const uint16_t*)p.k_layers[layer] + (long long)b * p.sb + (long long)hk * p.sh +
                          (long long)p.vis_off * p.sn;
  // This wave's keys as A operands: token tb*16 + j, head-dim elements (ks*4 + g)*8 .. +8 (which eight
  // elements ride in which slot of a contraction step is free as long as keys and queries agree).
  // An operand register wants 16 bytes of *its own* row in every lane; loaded that way, neighbouring
  // lanes read rows a whole row stride apart and the address unit takes a clock per lane (64 per
  // instruction: the 16 waves of a compute unit would queue there for 3.4 us with nothing to overlap).
  // So the keys are loaded as they lie in memory -- lane l takes piece l % CPR of row l / CPR, a
  // contiguous kilobyte per instruction -- and turned into operand layout through LDS: eight rows
  // at a time through this wave's own 8-row strip of query buffer 0 (swizzled like the query chunks;
  // the first query chunk lands in buffer 1 meanwhile), with no barrier, since a wave's LDS
  // operations complete in order and nobody else touches its strip before the first chunk barrier.
  constexpr int KRPI = 64 / CPR;                   // rows per load instruction
  constexpr int KNI = TPW / KRPI;                  // load instructions per wave
  constexpr int IPR = 8 / KRPI;                    // load instructions per 8-row round
  static_assert(TPW % 8 == 0 && 8 % KRPI == 0 && NW * 8 <= SattnSmem<D, PASS>::RCH, "key strips live in query buffer 0");
  u32x4 kraw[KNI];
#pragma unroll
  for (int i = 0; i < KNI; ++i) {
    int n = n0 + i * KRPI + lane / CPR;
    n = n < p.Nv ? n : p.Nv - 1;                     // in bounds; masked below
    kraw[i] = *(const u32x4*)(kbase + (long long)n * p.sn + (lane % CPR) * 8);
  }
  bool tok_ok[TBW][4];
#pragma unroll
  for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
    for (int e = 0; e < 4; ++e) tok_ok[tb][e] = (n0 + tb * 16 + 4 * g + e) < p.Nv;
  const bool wave_has_tokens = n0 < p.Nv;
  const bool wave_full = n0 + TPW <= p.Nv;

  float col[TBW][4];
#pragma unroll
  for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
    for (int e = 0; e < 4; ++e) col[tb][e] = 0.f;

  // Query rows are staged 64 at a time, straight from memory into LDS (16 bytes per lane, no
  // registers in between): a transfer fills 1 KB, i.e. 64 / CPR whole rows, and the chunk after the
  // current one is requested as soon as every wave has left the chunk before it, so its trip to
  // memory hides behind the MFMAs and a chunk costs one barrier.
  constexpr int RPI = 64 / CPR;                    // rows per transfer
  constexpr int XPW = RCH / RPI / NW;              // transfers per wave per chunk
  static_assert(RCH % (RPI * NW) == 0, "a chunk's transfers must split over the waves");
  static_assert(RCH == 64, "launch_score works out the chunk steps for 64-row chunks");
  constexpr int CHUNKB = RCH * ROWB;
  const unsigned qs_addr = (unsigned)(uintptr_t)Qs;
  float lse_reg = INFINITY;
  // Row r = i*G + g of the KV head lives at ((b*L + i)*H + hk*G + g)*D.  The (i, g) of the rows this
  // lane requests are carried from chunk to chunk (a chunk advances every row by RCH), so the
  // division by G happens once, not per chunk.  Rows past the end re-read the last row: pass 1 does
  // not write their statistics and pass 2 gives them an infinite normaliser.
  const uint16_t* qbase = (const uint16_t*)p.q_layers[layer] + ((long long)b * p.L * p.H + hk * p.G) * D;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  int qi[XPW], qg[XPW], qr[XPW];
  unsigned qpiece[XPW];                            // byte offset of this lane's piece inside its source row
  // (the chunk-to-chunk steps and the last row's coordinates come from the host, a lane's own first
  // division is a float reciprocal where the row numbers allow: 512 blocks x 8 waves dividing ten times
  // each kept every compute unit busy for 2.7 us before its first chunk was requested)
  const int step_i = p.q_step_i, step_g = p.q_step_g;
  const int last_i = p.q_last_i, last_g = p.q_last_g;
  const bool small_rows = Rs < (1 << 20);                       // block-uniform
  const float inv_g = __builtin_amdgcn_rcpf((float)p.G);
#pragma unroll
  for (int u = 0; u < XPW; ++u) {
    const int rr = (wave_u * XPW + u) * RPI + lane / CPR;       // row inside the chunk
    qr[u] = row_begin + rr;
    qi[u] = small_rows ? row_div_group(qr[u], inv_g) : qr[u] / p.G;
    qg[u] = qr[u] - qi[u] * p.G;
    qpiece[u] = (unsigned)(((lane % CPR) ^ lds_row_swizzle<D>(rr)) * 16);
  }
  auto request_chunk = [&](int buf, int r0) {    // must be called with r0 = row_begin, +RCH, +2 RCH, ...
#pragma unroll
    for (int u = 0; u < XPW; ++u) {
      const bool real = qr[u] < Rs;
      const int i = real ? qi[u] : last_i, g2 = real ? qg[u] : last_g;
      dma16((const char*)(qbase + ((long long)i * p.H + g2) * D) + qpiece[u],
            qs_addr + buf * CHUNKB + (wave_u * XPW + u) * 1024);
      qr[u] += RCH;
      qg[u] += step_g;
      const int carry = qg[u] >= p.G ? 1 : 0;
      qg[u] -= carry * p.G;
      qi[u] += step_i + carry;
    }
    if (PASS == 2 && tid < RCH) {
      const int r = r0 + tid;
      lse_reg = INFINITY;                     // padding rows contribute exp2(-inf) = 0
      if (r < Rs) lse_reg = p.row_lse[((long long)bz * p.Hkv + hk) * Rs + r];
    }
  };
  if (row_begin < row_end) request_chunk(1, row_begin);     // (every request is waited for at the top of its chunk)
  int buf = 1;
  bf16x8 kop[TBW][KS];
  {
    unsigned char* strip = Qs + __builtin_amdgcn_readfirstlane(wave) * (8 * ROWB);
    const int wr_row = lane / CPR;                                  // row of the round this lane's piece belongs to (+ ii * KRPI)
#pragma unroll
    for (int r = 0; r < TPW / 8; ++r) {
#pragma unroll
      for (int ii = 0; ii < IPR; ++ii) {
        const int row8 = ii * KRPI + wr_row;
        *(u32x4*)(strip + row8 * ROWB + (((lane % CPR) ^ lds_row_swizzle<D>(row8)) * 16)) = kraw[r * IPR + ii];
      }
      const int tb = r / 2, half = r % 2;                            // rows 8 * half .. of 16-token block tb
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 v = *(const bf16x8*)(strip + (j & 7) * ROWB + (((ks * 4 + g) ^ lds_row_swizzle<D>(j & 7)) * 16));
        if ((j >> 3) == half) kop[tb][ks] = v;
      }
    }
  }
  for (int r0 = row_begin; r0 < row_end; r0 += RCH, buf ^= 1) {
    wait_vmcnt<0>();                          // this wave's share of the chunk (and its normalisers) has arrived
    if (PASS == 2 && tid < RCH) sm.lse_s[buf][tid] = lse_reg;
    __syncthreads();                          // ... and everyone else's; everyone is done with the chunk before
    if (r0 + RCH < row_end) request_chunk(buf ^ 1, r0 + RCH);
    const unsigned char* Qc = Qs + buf * CHUNKB;
    const float* lse_c = sm.lse_s[buf];

    auto products = [&](int rb, f32x4 (&z)[TBW]) {
#pragma unroll
      for (int tb = 0; tb < TBW; ++tb) z[tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 qop = *(const bf16x8*)(Qc + (rb * 16 + j) * ROWB +
                                            (((ks * 4 + g) ^ lds_row_swizzle<D>(rb * 16 + j)) * 16));
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
          z[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[tb][ks], qop, z[tb], 0, 0, 0);
      }
    };
    auto reduce = [&](int rb, f32x4 (&z)[TBW]) {
      if (PASS == 1) {
        if (!wave_full) {                       // wave-uniform: only the ragged last wave masks
#pragma unroll
          for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (!tok_ok[tb][e]) z[tb][e] = -INFINITY;
        }
        float zv[TBW * 4];                      // the scale is positive: take the max of the raw logits
#pragma unroll
        for (int e = 0; e < TBW * 4; ++e) zv[e] = z[e >> 2][e & 3];
        float mx = rows4_max(max_nan_of(zv));
        mx *= scale_log2;
        const float neg_m = (mx == -INFINITY) ? 0.f : -mx;
        float ps = 0.f;
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
          for (int e = 0; e < 4; ++e) ps += fast_exp2(fmaf(z[tb][e], scale_log2, neg_m));
        ps = rows4_sum(ps);
        if (g == 0) {
          wm_s[wave][((r0 - row_begin) % RDEF) + rb * 16 + j] = mx;
          wl_s[wave][((r0 - row_begin) % RDEF) + rb * 16 + j] = ps;
        }
      } else {
        const float lse = lse_c[rb * 16 + j];
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
          for (int e = 0; e < 4; ++e) col[tb][e] += fast_exp2(fmaf(z[tb][e], scale_log2, -lse));
      }
    };
#pragma unroll
    for (int rb = 0; rb < RCH / 16; ++rb) {
      f32x4 z[TBW];
      products(rb, z);
      reduce(rb, z);
    }
    if (PASS == 1 && (((r0 - row_begin + RCH) % RDEF) == 0 || r0 + RCH >= row_end)) {
      // merge the waves' (max, sum) of the rows gathered since the last merge and write them out
      __syncthreads();
      const int base = r0 - ((r0 - row_begin) % RDEF);
      for (int rr = tid; rr < RDEF && base + rr < Rs && base + rr < r0 + RCH; rr += NT) {
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mm = max_nan(mm, wm_s[w][rr]);
        float ll = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w)
          ll += (wm_s[w][rr] == -INFINITY) ? 0.f : wl_s[w][rr] * fast_exp2(wm_s[w][rr] - mm);
        const long long at = sattn_part_at(p, tile, bz, hk, base + rr);  // consecutive rows: coalesced
        p.row_m[at] = mm;
        p.row_l[at] = ll;
      }
    }
  }
  if (PASS == 2 && wave_has_tokens) {
    // sum the 16 rows held by the lanes of each group g
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float v = row16_sum(col[tb][e]);
        if (j == 0 && tok_ok[tb][e])
          p.col_part[((long long)bz * p.Hkv * p.n_rsplit + vhk) * p.Nv + n0 + tb * 16 + 4 * g + e] = v;
      }
  }
}

// Launch order of the sweeps' blocks: KV head fastest, then key tile, then row run, then (layer,
// batch element).  Consecutive blocks go to consecutive XCDs, so with 1, 2, 4 or 8 KV heads an XCD
// sees the blocks of one or few heads only and its L2 fetches those heads' query rows instead of all
// of them (every block re-reads the query rows of its head and run); the blocks that sweep the other
// row run over the same 256 keys lie H_kv * n_tile places on -- on the same XCD, where the keys are.
// Grid (H_kv, n_tile, n_rsplit * Bz).
template <int D, int PASS>
__global__ __launch_bounds__(kSaWaves * 64) void sattn_mfma(ScoreParams p) {
  __shared__ SattnSmem<D, PASS> sm;
  const int rs = blockIdx.z % p.n_rsplit;
  sattn_mfma_body<D, PASS>(p, sm, blockIdx.y, blockIdx.x + p.Hkv * rs, blockIdx.z / p.n_rsplit);
}

// merge the per-tile row statistics: lse2 = m* + log2(sum_t l_t 2^(m_t - m*)).  A block takes 32
// consecutive rows; thread (row, slice s) merges tiles s, s+8, ... (loads issued 8 at a time), the 8
// slices of a row then merge through LDS.  Consecutive threads read consecutive rows of a tile's slab.
__global__ __launch_bounds__(256) void sattn_row_lse(ScoreParams p) {
  __shared__ float sm[8][32], sl[8][32];
  const long long rows = (long long)p.Bz * p.H * p.L;
  const int rl = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const long long row = (long long)blockIdx.x * 32 + rl;
  float mm = -INFINITY, ll = 0.f;
  if (row < rows) {
    for (int t0 = slice; t0 < p.n_tile; t0 += 64) {
      float m[8], l[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = t0 + 8 * u;
        m[u] = t < p.n_tile ? p.row_m[t * rows + row] : -INFINITY;
        l[u] = t < p.n_tile ? p.row_l[t * rows + row] : 0.f;
      }
      float mx = mm;
#pragma unroll
      for (int u = 0; u < 8; ++u) mx = max_nan(mx, m[u]);
      if (mx != -INFINITY) {
        ll *= fast_exp2(mm - mx);                 // mm = -inf: ll is 0 and exp2(-inf) = 0
#pragma unroll
        for (int u = 0; u < 8; ++u) ll += (m[u] != -INFINITY) ? l[u] * fast_exp2(m[u] - mx) : 0.f;
        mm = mx;
      }
    }
  }
  sm[slice][rl] = mm;
  sl[slice][rl] = ll;
  __syncthreads();
  if (slice == 0 && row < rows) {
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < 8; ++u) mx = max_nan(mx, sm[u][rl]);
    float tot = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) tot += (sm[u][rl] != -INFINITY) ? sl[u][rl] * fast_exp2(sm[u][rl] - mx) : 0.f;
    p.row_lse[row] = mx + __log2f(tot);
  }
}

// Sum over layers, KV heads and row runs of the column partials of token jj of batch element b, in index
// order, eight loads in flight at a time (a loop of one load and one add per turn would make every partial
// its own trip to memory).
__device__ __forceinline__ float sum_col_partials(const ScoreParams& p, int b, long long jj) {
  const int nvh = p.Hkv * p.n_rsplit;
  float a = 0.f;
  for (int layer = 0; layer < p.n_layers; ++layer)
    for (int hk0 = 0; hk0 < nvh; hk0 += 8) {
      float v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q)
        v[q] = p.col_part[(((long long)layer * p.B + b) * nvh + min(hk0 + q, nvh - 1)) * p.Nv + jj];
#pragma unroll
      for (int q = 0; q < 8; ++q) a += (hk0 + q < nvh) ? v[q] : 0.f;
    }
  return a;
}

// s_attn[b,j] = sum_hk col_part / (H L)  (+ running layer sum)
__global__ __launch_bounds__(256) void sattn_finalize(ScoreParams p) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)p.B * p.Nv) return;
  const int b = (int)(e / p.Nv), jj = (int)(e % p.Nv);
  float a = sum_col_partials(p, b, jj);
  a /= (float)p.H * (float)p.L;
  if (p.attn_mass_inout != nullptr) {
    a += p.attn_mass_inout[e];
    p.attn_mass_inout[e] = a;
  }
  p.s_attn[e] = a;
}

// =================================================================================================
// s_temp and s_spa: one block per (crop, frame, batch element)
// =================================================================================================
constexpr int kEmbChunk = 64;     // channels per LDS pass
constexpr int kMaxCrop = 64;      // tokens per crop

template <typename T>
__global__ __launch_bounds__(256) void emb_scores(ScoreParams p) {
  // E: this frame, previous frame, next frame.  G (the finished Gram matrix) reuses E's storage
  // once the channel sweep is over.
  __shared__ float e_raw[3 * kMaxCrop * (kEmbChunk + 1)];
  float (*E)[kMaxCrop][kEmbChunk + 1] = reinterpret_cast<float (*)[kMaxCrop][kEmbChunk + 1]>(e_raw);
  float (*G)[kMaxCrop + 1] = reinterpret_cast<float (*)[kMaxCrop + 1]>(e_raw);
  __shared__ float tdot[4][kMaxCrop];               // v.prev, |prev|^2, v.next, |next|^2
  __shared__ int tok_s[kMaxCrop];

  const int tid = threadIdx.x;
  const int ncx = (p.gw + p.cw - 1) / p.cw;
  const int cy = blockIdx.x / ncx, cx = blockIdx.x % ncx;
  const int f = blockIdx.y, b = blockIdx.z;
  const int y0 = cy * p.ch, x0 = cx * p.cw;
  const int mh = min(p.ch, p.gh - y0), mw = min(p.cw, p.gw - x0);
  const int M = mh * mw;
  if (tid < M) tok_s[tid] = f * p.P + (y0 + tid / mw) * p.gw + x0 + tid % mw;
  const bool has_prev = f > 0, has_next = f + 1 < p.F;

  const int de = p.emb ? p.emb_dim : p.Hkv * p.D;
  const int n_pairs = M * M;
  constexpr int PPT = kMaxCrop * kMaxCrop / 256;    // pairs per thread, worst case
  float gacc[PPT];
#pragma unroll
  for (int x = 0; x < PPT; ++x) gacc[x] = 0.f;
  float tacc = 0.f;                                  // threads [0,4*64): quantity tid/64 of token tid%64
  __syncthreads();

  constexpr int VPC = kEmbChunk / Elem<T>::kPerVec;  // vectors per chunk row
  for (int c0 = 0; c0 < de; c0 += kEmbChunk) {
    // ---- stage chunk [c0, c0+64) of the 3*M vectors ----
    for (int e = tid; e < 3 * M * VPC; e += 256) {
      const int which = e / (M * VPC), rem = e % (M * VPC);
      const int t = rem / VPC, vec = rem % VPC;
      const int c = c0 + vec * Elem<T>::kPerVec;
      float vals[Elem<T>::kPerVec];
#pragma unroll
      for (int u = 0; u < Elem<T>::kPerVec; ++u) vals[u] = 0.f;
      const bool present = (which == 0) || (which == 1 && has_prev) || (which == 2 && has_next);
      if (present && c < de) {
        const long long tokn = tok_s[t] + (which == 1 ? -p.P : (which == 2 ? p.P : 0));
        const T* src;
        if (p.emb) {
          src = (const T*)p.emb + (long long)b * p.emb_stride_b + tokn * p.emb_stride_tok + c;
        } else {
          const int hk = c / p.D, cc = c % p.D;
          src = (const T*)p.k_cache + (long long)b * p.sb + (long long)hk * p.sh +
                (p.vis_off + tokn) * p.sn + cc;
        }
        const u32x4 v4 = *(const u32x4*)src;
        Elem<T>::unpack(v4, vals);
      }
#pragma unroll
      for (int u = 0; u < Elem<T>::kPerVec; ++u) E[which][t][vec * Elem<T>::kPerVec + u] = vals[u];
    }
    __syncthreads();
    // ---- Gram of the crop ----
#pragma unroll
    for (int x = 0; x < PPT; ++x) {
      const int pr = tid + 256 * x;
      if (pr < n_pairs) {
        const int a = pr / M, c2 = pr % M;
        float s = 0.f;
#pragma unroll 8
        for (int c = 0; c < kEmbChunk; ++c) s = fmaf(E[0][a][c], E[0][c2][c], s);
        gacc[x] += s;
      }
    }
    // ---- temporal dot products and neighbour norms ----
    {
      const int qn = tid >> 6, t = tid & 63;
      if (t < M) {
        const int other = (qn < 2) ? 1 : 2;
        const float* ea = (qn & 1) ? E[other][t] : E[0][t];
        const float* eb = E[other][t];
        float s = 0.f;
#pragma unroll 8
        for (int c = 0; c < kEmbChunk; ++c) s = fmaf(ea[c], eb[c], s);
        tacc += s;
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int x = 0; x < PPT; ++x) {
    const int pr = tid + 256 * x;
    if (pr < n_pairs) G[pr / M][pr % M] = gacc[x];
  }
  tdot[tid >> 6][tid & 63] = tacc;
  __syncthreads();

  if (tid < M) {
    const int a = tid;
    const float na = G[a][a];
    // spatial: population variance of the cosine row
    float mu = 0.f;
    for (int c2 = 0; c2 < M; ++c2) {
      const float nb = G[c2][c2];
      const float cs = (na > 0.f && nb > 0.f) ? G[a][c2] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      mu += cs;
    }
    mu /= (float)M;
    float var = 0.f;
    for (int c2 = 0; c2 < M; ++c2) {
      const float nb = G[c2][c2];
      const float cs = (na > 0.f && nb > 0.f) ? G[a][c2] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      var = fmaf(cs - mu, cs - mu, var);
    }
    const long long o = (long long)b * p.Nv + tok_s[a];
    p.s_spa[o] = var / (float)M;
    // temporal
    float sum = 0.f;
    int cnt = 0;
    if (has_prev) {
      const float nb = tdot[1][a];
      sum += (na > 0.f && nb > 0.f) ? tdot[0][a] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      ++cnt;
    }
    if (has_next) {
      const float nb = tdot[3][a];
      sum += (na > 0.f && nb > 0.f) ? tdot[2][a] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      ++cnt;
    }
    p.s_temp[o] = 1.f - (cnt ? sum / (float)cnt : 0.f);
  }
}

// =================================================================================================
// s_temp and s_spa on MFMA (bf16): one block per (crop, frame, batch element), RBC*16 >= crop size.
// The crop's Gram matrix E E^T and the temporal products (E_f E_{f-1}^T, E_{f-1} E_{f-1}^T and the
// same for f+1, of which only the diagonals are used) are 16x16 output blocks of one and the same
// operand: a lane's A operand for row block rb -- token rb*16 + lane%16, 8 consecutive channels --
// is also the B operand for that block of columns, and it is read straight from global memory
// (16 bytes per lane; the 4 lane groups of a token cover 64 contiguous bytes).  The 16x16 blocks
// are dealt to the 4 waves, each sweeping all channels for its blocks, so nothing is reduced
// across waves; the finished Gram goes to LDS and one thread per token finishes Eq. 4 and Eq. 6.
// =================================================================================================
template <int RBC>
__global__ __launch_bounds__(256) void emb_scores_mfma(ScoreParams p) {
  constexpr int MP = RBC * 16;
  constexpr int N_GRAM = RBC * (RBC + 1) / 2;      // upper-triangle blocks
  constexpr int N_ITEMS = N_GRAM + 4 * RBC;        // + (prev dot, prev norm, next dot, next norm) x RBC
  __shared__ float G[MP][MP + 1];
  __shared__ float tdot[4][MP];                     // v.prev, |prev|^2, v.next, |next|^2
  __shared__ int tok_s[MP];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, g = lane >> 4;
  const int ncx = (p.gw + p.cw - 1) / p.cw;
  const int cy = blockIdx.x / ncx, cx = blockIdx.x % ncx;
  const int f = blockIdx.y, b = blockIdx.z;
  const int y0 = cy * p.ch, x0 = cx * p.cw;
  const int mh = min(p.ch, p.gh - y0), mw = min(p.cw, p.gw - x0);
  const int M = mh * mw;
  if (tid < MP) {
    const int t = tid < M ? tid : M - 1;            // padding slots repeat the last token
    tok_s[tid] = f * p.P + (y0 + t / mw) * p.gw + x0 + t % mw;
  }
  const bool has_prev = f > 0, has_next = f + 1 < p.F;
  const int de = p.emb ? p.emb_dim : p.Hkv * p.D;
  const int n_ks = (de + 31) / 32;
  __syncthreads();

  // operand of frame offset `df` (-1, 0, +1), row block rbk, channel step ks
  auto operand = [&](int df, int rbk, int ks) -> bf16x8 {
    const int c = ks * 32 + g * 8;
    if (c >= de) return (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
    const long long tokn = tok_s[rbk * 16 + j] + (long long)df * p.P;
    const uint16_t* src;
    if (p.emb) {
      src = (const uint16_t*)p.emb + (long long)b * p.emb_stride_b + tokn * p.emb_stride_tok + c;
    } else {
      const int hk = c / p.D, cc = c % p.D;
      src = (const uint16_t*)p.k_cache + (long long)b * p.sb + (long long)hk * p.sh +
            (p.vis_off + tokn) * p.sn + cc;
    }
    return *(const bf16x8*)src;
  };

  for (int item = wave; item < N_ITEMS; item += 4) {          // wave-uniform
    int da, db_, ra, rbk;                                      // frame offsets and row blocks of A and B
    int kind = -1;                                             // -1 Gram, 0..3 temporal quantity
    if (item < N_GRAM) {
      int bi = 0, rem = item;
      while (rem >= RBC - bi) { rem -= RBC - bi; ++bi; }
      ra = bi; rbk = bi + rem; da = 0; db_ = 0;
    } else {
      const int t = item - N_GRAM;
      kind = t / RBC;
      ra = rbk = t % RBC;
      const int dn = kind < 2 ? -1 : 1;
      if ((dn < 0 && !has_prev) || (dn > 0 && !has_next)) continue;
      da = (kind & 1) ? dn : 0;                                // norm: neighbour with itself
      db_ = dn;
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const bool same = (da == db_) && (ra == rbk);              // diagonal block: one operand serves both
    for (int ks0 = 0; ks0 < n_ks; ks0 += 8) {                  // 8 channel steps of loads in flight
      bf16x8 a[8], bb[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] = operand(da, ra, ks0 + u);
      if (same) {
#pragma unroll
        for (int u = 0; u < 8; ++u) bb[u] = a[u];
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) bb[u] = operand(db_, rbk, ks0 + u);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], bb[u], acc, 0, 0, 0);
    }
    // D[i][j']: this lane holds column j' = j, rows i = 4g..4g+3
    if (kind < 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        G[ra * 16 + 4 * g + e][rbk * 16 + j] = acc[e];
        G[rbk * 16 + j][ra * 16 + 4 * g + e] = acc[e];
      }
    } else if ((j >> 2) == g) {
      tdot[kind][ra * 16 + j] = acc[j & 3];
    }
  }
  __syncthreads();

  if (tid < M) {
    const int a = tid;
    const float na = G[a][a];
    float mu = 0.f;
    for (int c2 = 0; c2 < M; ++c2) {
      const float nb = G[c2][c2];
      mu += (na > 0.f && nb > 0.f) ? G[a][c2] / (sqrtf(na) * sqrtf(nb)) : 0.f;
    }
    mu /= (float)M;
    float var = 0.f;
    for (int c2 = 0; c2 < M; ++c2) {
      const float nb = G[c2][c2];
      const float cs = (na > 0.f && nb > 0.f) ? G[a][c2] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      var = fmaf(cs - mu, cs - mu, var);
    }
    const long long o = (long long)b * p.Nv + tok_s[a];
    p.s_spa[o] = var / (float)M;
    float sum = 0.f;
    int cnt = 0;
    if (has_prev) {
      const float nb = tdot[1][a];
      sum += (na > 0.f && nb > 0.f) ? tdot[0][a] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      ++cnt;
    }
    if (has_next) {
      const float nb = tdot[3][a];
      sum += (na > 0.f && nb > 0.f) ? tdot[2][a] / (sqrtf(na) * sqrtf(nb)) : 0.f;
      ++cnt;
    }
    p.s_temp[o] = 1.f - (cnt ? sum / (float)cnt : 0.f);
  }
}

// =================================================================================================
// s_temp and s_spa on MFMA, crops of at most 32 tokens (the paper's 5 x 5): channel-split variant.
// Same products as emb_scores_mfma, but here the waves split the CHANNELS in two halves and the
// neighbour frames between them (waves 0,1: Gram and previous frame; waves 2,3: next frame), so an
// operand is fetched at most twice per block; the two channel halves are summed through LDS.
// =================================================================================================
struct Emb32Smem {
  static constexpr int MP = 32;
  // blocks: Gram (0,0) (0,1) (1,1); then for prev and for next: dot rb0, dot rb1, norm rb0, norm rb1
  static constexpr int NBLK = 11;
  f32x4 red[2][3][64];                              // Gram blocks of the two channel halves
  float redd[2][NBLK - 3][16];                      // diagonals of the dot / norm blocks, likewise
  float G[MP][MP + 1];
  float tdot[4][MP];
  float inv_norm[MP];
  int tok_s[MP];
};

// One crop, computed by the 256 threads `tid` = 0..255 of a group; every thread of the block must
// call it (it contains block-wide barriers).  BATCH = channel steps whose operands are in flight.
template <int BATCH>
__device__ __forceinline__ void emb_mfma32_body(const ScoreParams& p, Emb32Smem& sm, const int tid,
                                                const int crop_in_frame, const int f, const int b) {
  constexpr int MP = Emb32Smem::MP;
  constexpr int NBLK = Emb32Smem::NBLK;
  auto& red = sm.red;
  auto& redd = sm.redd;
  auto& G = sm.G;
  auto& tdot = sm.tdot;
  auto& inv_norm = sm.inv_norm;
  auto& tok_s = sm.tok_s;

  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cg = wave & 1;                          // channel half: channel steps cg, cg+2, ...
  const int ig = wave >> 1;                         // 0: Gram + previous frame, 1: next frame
  const int j = lane & 15, g = lane >> 4;
  const int ncx = (p.gw + p.cw - 1) / p.cw;
  const int cy = crop_in_frame / ncx, cx = crop_in_frame % ncx;
  const int y0 = cy * p.ch, x0 = cx * p.cw;
  const int mh = min(p.ch, p.gh - y0), mw = min(p.cw, p.gw - x0);
  const int M = mh * mw;
  if (tid < MP) {
    const int t = tid < M ? tid : M - 1;            // padding slots repeat the last token
    tok_s[tid] = f * p.P + (y0 + t / mw) * p.gw + x0 + t % mw;
  }
  const bool has_prev = f > 0, has_next = f + 1 < p.F;
  const int de = p.emb ? p.emb_dim : p.Hkv * p.D;
  const int n_ks = (de + 31) / 32;
  __syncthreads();

  // frames without a neighbour re-read the frame itself (finite data, result unused)
  const int dnb = ig == 0 ? (has_prev ? -1 : 0) : (has_next ? 1 : 0);
  // Row pointers of this lane's two tokens (row blocks 0 and 1) in this frame and in the neighbour
  // frame, computed once; a channel step then only adds its channel offset.  With keys as the
  // embedding, channel c is element c % D of KV head c / D (D is a power of two).
  const uint16_t* row_cur[2];
  const uint16_t* row_nb[2];
  const int dsh = p.D == 128 ? 7 : 6;
#pragma unroll
  for (int rbk = 0; rbk < 2; ++rbk) {
    const long long tokn = tok_s[rbk * 16 + j];
    if (p.emb) {
      row_cur[rbk] = (const uint16_t*)p.emb + (long long)b * p.emb_stride_b + tokn * p.emb_stride_tok;
      row_nb[rbk] = row_cur[rbk] + (long long)dnb * p.P * p.emb_stride_tok;
    } else {
      row_cur[rbk] = (const uint16_t*)p.k_cache + (long long)b * p.sb + (p.vis_off + tokn) * p.sn;
      row_nb[rbk] = row_cur[rbk] + (long long)dnb * p.P * p.sn;
    }
  }
  const bool keys_as_emb = p.emb == nullptr;
  auto operand = [&](const uint16_t* row, int ks) -> bf16x8 {
    const int c = ks * 32 + g * 8;
    const bool ok = ks < n_ks && c < de;
    const int cs = ok ? c : 0;                         // a valid address either way; zeroed below
    const long long off = keys_as_emb ? (long long)(cs >> dsh) * p.sh + (cs & (p.D - 1)) : (long long)cs;
    const bf16x8 v = *(const bf16x8*)(row + off);
    return ok ? v : (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
  };

  f32x4 acc[7];   // ig 0: Gram x3, dot x2, norm x2;  ig 1: (unused x3), dot x2, norm x2
#pragma unroll
  for (int i = 0; i < 7; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int ks0 = cg; ks0 < n_ks; ks0 += 2 * BATCH) {   // BATCH channel steps of this wave per round
    bf16x8 cur[BATCH][2], nb[BATCH][2];
#pragma unroll
    for (int u = 0; u < BATCH; ++u)
#pragma unroll
      for (int rbk = 0; rbk < 2; ++rbk) {
        cur[u][rbk] = operand(row_cur[rbk], ks0 + 2 * u);
        nb[u][rbk] = operand(row_nb[rbk], ks0 + 2 * u);
      }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      if (ig == 0) {
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[u][0], cur[u][0], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[u][0], cur[u][1], acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[u][1], cur[u][1], acc[2], 0, 0, 0);
      }
#pragma unroll
      for (int rbk = 0; rbk < 2; ++rbk) {
        acc[3 + rbk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[u][rbk], nb[u][rbk], acc[3 + rbk], 0, 0, 0);
        acc[5 + rbk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(nb[u][rbk], nb[u][rbk], acc[5 + rbk], 0, 0, 0);
      }
    }
  }
  // D[i][j']: a lane holds column j' = j, rows i = 4g..4g+3; of the dot / norm blocks only the
  // diagonal (token with itself) is needed: lane (j, g = j/4), element j%4
  if (ig == 0) {
#pragma unroll
    for (int i = 0; i < 3; ++i) red[cg][i][lane] = acc[i];
  }
  if ((j >> 2) == g) {
#pragma unroll
    for (int i = 3; i < 7; ++i) {                    // 0,1 prev dot; 2,3 prev norm; 4,5 next dot; 6,7 next norm
      float* dst = &redd[cg][(ig == 0 ? 0 : 4) + i - 3][j];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((j & 3) == e) *dst = acc[i][e];
    }
  }
  __syncthreads();
  // sum the two channel halves: waves 0..2 finish one Gram block each, wave 3 the diagonals
  if (wave < 3) {
    const int blk = wave;
    const f32x4 v = red[0][blk][lane] + red[1][blk][lane];
    const int ra = blk == 2 ? 1 : 0, rbk = blk == 0 ? 0 : 1;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      G[ra * 16 + 4 * g + e][rbk * 16 + j] = v[e];
      G[rbk * 16 + j][ra * 16 + 4 * g + e] = v[e];
    }
  } else {
    for (int e = lane; e < (NBLK - 3) * 16; e += 64) {
      const int t = e >> 4, jj = e & 15;
      tdot[t >> 1][(t & 1) * 16 + jj] = redd[0][t][jj] + redd[1][t][jj];
    }
  }
  __syncthreads();
  if (tid < MP) inv_norm[tid] = G[tid][tid] > 0.f ? 1.f / sqrtf(G[tid][tid]) : 0.f;   // 0: zero-norm row
  __syncthreads();

  if (tid < M) {
    const int a = tid;
    const float ia = inv_norm[a];
    float mu = 0.f;
    for (int c2 = 0; c2 < M; ++c2) mu += G[a][c2] * ia * inv_norm[c2];
    mu /= (float)M;
    float var = 0.f;
    for (int c2 = 0; c2 < M; ++c2) {
      const float cs = G[a][c2] * ia * inv_norm[c2];
      var = fmaf(cs - mu, cs - mu, var);
    }
    const long long o = (long long)b * p.Nv + tok_s[a];
    p.s_spa[o] = var / (float)M;
    float sum = 0.f;
    int cnt = 0;
    if (has_prev) {
      const float nb2 = tdot[1][a];
      sum += (nb2 > 0.f) ? tdot[0][a] * ia / sqrtf(nb2) : 0.f;
      ++cnt;
    }
    if (has_next) {
      const float nb2 = tdot[3][a];
      sum += (nb2 > 0.f) ? tdot[2][a] * ia / sqrtf(nb2) : 0.f;
      ++cnt;
    }
    p.s_temp[o] = 1.f - (cnt ? sum / (float)cnt : 0.f);
  }
}

// =================================================================================================
// s_temp and s_spa on MFMA, crops of at most 32 tokens, at most 512 channels: frame-run variant.
// A block of eight waves owns ONE crop position over a run of consecutive frames, so a frame's crop
// is fetched once and serves as "this frame" for its Gram matrix (Eq. 5-6; its diagonal holds the
// norms) and as "the neighbour" of the frame before and after it (Eq. 3-4) -- against four fetches
// per crop when every (crop, frame) is a block of its own.  Wave w owns channels 64w .. 64w+63 (two
// MFMA channel steps) of all 32 rows; the eight partial Gram and dot blocks are summed through LDS.
// The operands travel HBM -> LDS by direct transfers, a lane fetching 16 bytes of a 128-byte row
// segment next to its neighbour's (an MFMA operand lane holds ITS OWN row, so fetching operands
// straight into registers makes neighbouring lanes read rows far apart, and the address unit then
// spends a clock per lane instead of a clock per four); the wave reads them back in operand layout
// from its own 4 KB strip, whose rows are XOR-swizzled against bank conflicts.  The strip then
// carries the wave's partial Gram blocks to the reduction, so the next frame's transfer is requested
// once the reduction has read them and lands under the rest of the frame's arithmetic.
// =================================================================================================
// 16 bytes of zeros in device memory: what a transfer lane fetches for channels beyond the last
__device__ __align__(16) const unsigned char g_zero_piece[16] = {0};

struct EmbRunSmem {
  static constexpr int MP = 32;
  static constexpr int NW = 8;
  __align__(16) unsigned char strip[NW][4096];      // operands in (32 rows x 128 B), then Gram partials out (3 x 64 x 16 B)
  float redd[NW][2][16];                            // diagonals of the (this frame) x (frame before) blocks
  float G[MP][MP + 1];
  float dotv[MP];
  float inv_norm[MP];
  int tok_s[MP];
};

// One crop position `pos` of batch element b over the frames f0 .. f0 + p.emb_run - 1 (cut at the
// video's end), by the 512 threads of a block; every thread must call it (block-wide barriers).
__device__ __forceinline__ void emb_run32_body(const ScoreParams& p, EmbRunSmem& sm, const int tid, const int pos,
                                               const int f0, const int b) {
  constexpr int MP = EmbRunSmem::MP;
  constexpr int NW = EmbRunSmem::NW;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, g = lane >> 4;
  const int ncx = (p.gw + p.cw - 1) / p.cw;
  const int cy = pos / ncx, cx = pos % ncx;
  const int y0 = cy * p.ch, x0 = cx * p.cw;
  const int mh = min(p.ch, p.gh - y0), mw = min(p.cw, p.gw - x0);
  const int M = mh * mw;
  if (tid < MP) {
    const int t = tid < M ? tid : M - 1;            // padding slots repeat the last token
    sm.tok_s[tid] = (y0 + t / mw) * p.gw + x0 + t % mw;   // token within its frame
  }
  const int f_end = min(f0 + p.emb_run, p.F);       // the run: frames f0 .. f_end - 1
  const int lo = max(f0 - 1, 0), hi = min(f_end, p.F - 1);   // frames fetched: the run and its neighbours
  const int de = p.emb ? p.emb_dim : p.Hkv * p.D;
  const bool keys_as_emb = p.emb == nullptr;
  const int dsh = p.D == 128 ? 7 : 6;
  __syncthreads();

  // Transfer i of a frame (0..3) brings rows 8i .. 8i+7 of the crop: lane l fetches, for strip
  // position l % 8 of row 8i + l / 8, the 16-byte piece (l % 8) ^ (row & 7) of the wave's 128 bytes.
  // With keys as the embedding, channel c is element c % D of KV head c / D (D is a power of two).
  // Pieces beyond the last channel are fetched from 16 bytes of zeros (and stay there from frame to
  // frame), so the operands need no masking.
  const uint16_t* src[4];
  const int c = wave * 64 + (((lane & 7) ^ ((lane >> 3) & 7)) * 8);   // (row & 7 is the same in all four transfers)
  const long long src_step = c >= de ? 0 : (long long)p.P * (keys_as_emb ? p.sn : p.emb_stride_tok);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const long long tokn = (long long)lo * p.P + sm.tok_s[i * 8 + (lane >> 3)];
    if (c >= de)
      src[i] = (const uint16_t*)g_zero_piece;
    else if (keys_as_emb)
      src[i] = (const uint16_t*)p.k_cache + (long long)b * p.sb + (p.vis_off + tokn) * p.sn +
               (long long)(c >> dsh) * p.sh + (c & (p.D - 1));
    else
      src[i] = (const uint16_t*)p.emb + (long long)b * p.emb_stride_b + tokn * p.emb_stride_tok + c;
  }
  unsigned char* strip = &sm.strip[wave][0];
  const unsigned strip_addr = (unsigned)(uintptr_t)strip;
  auto request_frame = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dma16(src[i], strip_addr + i * 1024);
      src[i] += src_step;
    }
  };
  // operand (row block rbk, channel step u of the wave): lane (j, g) holds piece 4u + g of row 16 rbk + j
  auto operand = [&](int rbk, int u) -> bf16x8 {
    return *(const bf16x8*)(strip + (rbk * 16 + j) * 128 + (((4 * u + g) ^ (j & 7)) * 16));
  };
  // 1 / sqrt(x) by the hardware's reciprocal square root (1 ulp), which ignores denormals: tiny
  // arguments are scaled by 2^64 first, the result by 2^32; 0 for a zero-norm row.  (The riding
  // blocks compete with the sweep for vector-instruction issue and nothing else, so what the crop's
  // closing arithmetic costs in instructions is what the embedding terms cost the launch.)
  auto inv_sqrt = [](float x) -> float {
    const bool tiny = x < 0x1p-60f;
    const float r = __builtin_amdgcn_rsqf(tiny ? x * 0x1p64f : x);
    return x > 0.f ? (tiny ? r * 0x1p32f : r) : 0.f;
  };
  const float inv_M = 1.f / (float)M;

  // state of the tokens' temporal term, kept by lane 0 of each 16-lane row (token a = tid / 16):
  // 1 / norm of the last two frames, and their dot product
  float inv_n1 = 0.f, inv_n2 = 0.f, dot1 = 0.f;
  const int a = tid >> 4, c0 = (tid & 15) * 2;
  const long long out_base = (long long)b * p.Nv + sm.tok_s[a];

  bf16x8 prev[2][2];                                // the operands of the frame before
#pragma unroll
  for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
    for (int u = 0; u < 2; ++u) prev[rbk][u] = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
  request_frame();
  for (int fr = lo; fr <= hi; ++fr) {
    f32x4 dot[2];
    bf16x8 cur[2][2];
    wait_vmcnt<0>();                                // the frame is in this wave's strip
#pragma unroll
    for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
      for (int u = 0; u < 2; ++u) cur[rbk][u] = operand(rbk, u);
    // D[i][j']: a lane holds column j' = j, rows i = 4g..4g+3.  The strip's operands are in registers
    // (a wave's LDS operations complete in order), so it can take the Gram partials at once
    // (one block at a time: few accumulators live beside the two frames' operands).  A neighbour frame
    // beyond the run is here for its norms and dot products: the diagonal blocks suffice.
    const bool own_frame = fr >= f0 && fr < f_end;  // (uniform)
#pragma unroll
    for (int i = 0; i < 3; ++i) {                    // Gram blocks (0,0) (0,1) (1,1)
      if (i == 1 && !own_frame) continue;
      f32x4 gram = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 2; ++u)
        gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[i >> 1][u], cur[(i + 1) >> 1][u], gram, 0, 0, 0);
      *(f32x4*)(strip + (i * 64 + lane) * 16) = gram;
    }
    dot[0] = dot[1] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        dot[rbk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[rbk][u], prev[rbk][u], dot[rbk], 0, 0, 0);
        prev[rbk][u] = cur[rbk][u];
      }
    // of a dot block only the diagonal (token with itself) is needed: lane (j, g = j/4), element j%4
    if ((j >> 2) == g) {
#pragma unroll
      for (int rbk = 0; rbk < 2; ++rbk) {
        float d = dot[rbk][0];
#pragma unroll
        for (int e = 1; e < 4; ++e)
          if ((j & 3) == e) d = dot[rbk][e];
        sm.redd[wave][rbk][j] = d;
      }
    }
    __syncthreads();
    // sum the eight channel slices in a fixed order: waves 0..2 one Gram block each (the diagonal
    // blocks also give the rows' 1 / norm), wave 3 the diagonals of the dot blocks
    if (wave < 3 && (own_frame || wave != 1)) {
      const int blk = wave;
      f32x4 v = *(const f32x4*)(&sm.strip[0][0] + (blk * 64 + lane) * 16);
#pragma unroll
      for (int w = 1; w < NW; ++w) v += *(const f32x4*)(&sm.strip[w][0] + (blk * 64 + lane) * 16);
      const int ra = blk == 2 ? 1 : 0, rbk = blk == 0 ? 0 : 1;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sm.G[ra * 16 + 4 * g + e][rbk * 16 + j] = v[e];
        sm.G[rbk * 16 + j][ra * 16 + 4 * g + e] = v[e];
      }
      if (blk != 1 && (j >> 2) == g) {              // D[j][j]: lane (j, g = j/4), element j%4
        float d = v[0];
#pragma unroll
        for (int e = 1; e < 4; ++e)
          if ((j & 3) == e) d = v[e];
        sm.inv_norm[ra * 16 + j] = inv_sqrt(d);
      }
    } else if (wave == 3 && lane < MP) {
      float d = sm.redd[0][lane >> 4][lane & 15];
#pragma unroll
      for (int w = 1; w < NW; ++w) d += sm.redd[w][lane >> 4][lane & 15];
      sm.dotv[lane] = d;
    }
    __syncthreads();
    if (fr < hi) request_frame();                   // the strips are free again: the next frame travels meanwhile

    // cosines of token a against tokens c0, c0 + 1 (16 lanes cover the crop; padding rows hold
    // finite values and are masked); Eq. 5-6: their variance -- for the run's own frames only
    const float ia = sm.inv_norm[a];
    float var = 0.f;
    if (own_frame) {
      const float cs0 = c0 < M ? sm.G[a][c0] * (ia * sm.inv_norm[c0]) : 0.f;
      const float cs1 = c0 + 1 < M ? sm.G[a][c0 + 1] * (ia * sm.inv_norm[c0 + 1]) : 0.f;
      const float mu = row16_sum(cs0 + cs1) * inv_M;
      const float d0 = c0 < M ? cs0 - mu : 0.f, d1 = c0 + 1 < M ? cs1 - mu : 0.f;
      var = row16_sum(fmaf(d0, d0, d1 * d1)) * inv_M;
    }
    if ((tid & 15) == 0 && a < M) {
      const float dcur = sm.dotv[a];                // <this frame, frame before>
      if (own_frame) p.s_spa[out_base + (long long)fr * p.P] = var;
      // Eq. 3-4 of the frame before, whose two neighbours are known now
      if (fr > lo && fr - 1 >= f0) {
        const float next = dcur * inv_n1 * ia, before = dot1 * inv_n1 * inv_n2;
        p.s_temp[out_base + (long long)(fr - 1) * p.P] = 1.f - (fr - 1 > 0 ? 0.5f * (next + before) : next);
      }
      inv_n2 = inv_n1;
      inv_n1 = ia;
      dot1 = dcur;
    }
  }
  // a run that reaches the video's last frame: that frame has no successor
  if ((tid & 15) == 0 && a < M && hi < f_end)
    p.s_temp[out_base + (long long)hi * p.P] = 1.f - (hi > 0 ? dot1 * inv_n1 * inv_n2 : 0.f);
}

// block number -> (crop position, run of frames, batch element), positions fastest
__device__ __forceinline__ void emb_run32_block(const ScoreParams& p, EmbRunSmem& sm, const unsigned blk) {
  const unsigned ncf = (unsigned)(((p.gh + p.ch - 1) / p.ch) * ((p.gw + p.cw - 1) / p.cw));   // crops per frame
  const unsigned n_runs = (unsigned)((p.F + p.emb_run - 1) / p.emb_run);
  const unsigned rest = blk / ncf, pos = blk - rest * ncf;
  const unsigned bb = rest / n_runs, run = rest - bb * n_runs;
  emb_run32_body(p, sm, threadIdx.x, (int)pos, (int)run * p.emb_run, (int)bb);
}

__global__ __launch_bounds__(512) void emb_scores_run32(ScoreParams p) {
  __shared__ EmbRunSmem sm;
  emb_run32_block(p, sm, blockIdx.x);
}

__global__ __launch_bounds__(256) void emb_scores_mfma32(ScoreParams p) {
  __shared__ Emb32Smem sm;
  emb_mfma32_body<4>(p, sm, threadIdx.x, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Pass 1 of s_attn and the embedding terms in ONE launch: the first n_sattn blocks run the
// (compute-bound) row-statistics sweep, two per compute unit; the remaining blocks run the crops and
// fill the third block slot of the compute units, so the memory-bound embedding work hides under the
// sweep instead of following it.  Three blocks fit a compute unit: 8 waves of at most 80 registers
// each and the larger of the shared-memory layouts.  RUNS: a riding block owns one crop position over
// a run of frames (up to 512 channels); otherwise it owns two crops, four waves each.
template <int D, bool RUNS>
__global__ __launch_bounds__(kSaWaves * 64, 6) void sattn_pass1_with_emb(ScoreParams p, int n_sattn) {
  static_assert(kSaWaves == EmbRunSmem::NW, "the riding blocks use the sweep's block size");
  union Smem {
    SattnSmem<D, 1> sa;
    EmbRunSmem run;
    Emb32Smem emb[2];
  };
  __shared__ Smem sm;
  const int blk = blockIdx.x;
  if (blk < n_sattn) {                       // the order of sattn_mfma's grid: KV head fastest, then key tile, ...
    const int hk = blk % p.Hkv, rest = blk / p.Hkv;
    const int tile = rest % p.n_tile, rest2 = rest / p.n_tile;
    sattn_mfma_body<D, 1>(p, sm.sa, tile, hk + p.Hkv * (rest2 % p.n_rsplit), rest2 / p.n_rsplit);
    return;
  }
  // (the host admits this launch only when its block count stays below 2^31: crop numbers fit 32 bits,
  // and 32-bit divisions are all that stands in front of a riding block's first load)
  if constexpr (RUNS) {
    emb_run32_block(p, sm.run, (unsigned)(blk - n_sattn));
  } else {
    const int ncf = ((p.gh + p.ch - 1) / p.ch) * ((p.gw + p.cw - 1) / p.cw);   // crops per frame
    const unsigned n_crops = (unsigned)ncf * (unsigned)p.F * (unsigned)p.B;
    const int half = threadIdx.x >> 8;
    unsigned crop = 2u * (unsigned)(blk - n_sattn) + (unsigned)half;
    if (crop >= n_crops) crop = n_crops - 1;       // odd count: the idle half repeats the last crop
    const unsigned fb = crop / (unsigned)ncf;
    const int c = (int)(crop - fb * (unsigned)ncf);
    const unsigned bb = fb / (unsigned)p.F;
    emb_mfma32_body<2>(p, sm.emb[half], threadIdx.x & 255, c, (int)(fb - bb * (unsigned)p.F), (int)bb);
  }
}

// =================================================================================================
// Eq. 7: per-frame z-scores, summed over the enabled terms.  One block per (frame, batch element).
// =================================================================================================
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void fuse_scores(ScoreParams p) {
  __shared__ float red[4];
  const int f = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const long long base = (long long)b * p.Nv + (long long)f * p.P;
  if (p.flags & HIPPO_SCORE_ATTN) {
    // s_attn[b,j] = sum_hk col_part / (H L) (+ the running layer sum), for this frame's tokens
    for (int i = tid; i < p.P; i += 256) {
      const long long e = base + i;
      const int jj = f * p.P + i;
      float a = sum_col_partials(p, b, jj);
      a /= (float)p.H * (float)p.L;
      if (p.attn_mass_inout != nullptr) {
        a += p.attn_mass_inout[e];
        p.attn_mass_inout[e] = a;
      }
      p.s_attn[e] = a;
    }
    __syncthreads();   // the block re-reads its own s_attn values below
  }
  const float* terms[3] = {p.s_attn, p.s_temp, p.s_spa};
  float mu[3], inv_sigma[3];
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    mu[t] = 0.f;
    inv_sigma[t] = 0.f;
    if (!(p.flags & (1u << t))) continue;
    float s = 0.f;
    for (int i = tid; i < p.P; i += 256) s += terms[t][base + i];
    mu[t] = block_sum_256(s, red) / (float)p.P;
    float v = 0.f;
    for (int i = tid; i < p.P; i += 256) {
      const float d = terms[t][base + i] - mu[t];
      v = fmaf(d, d, v);
    }
    const float var = block_sum_256(v, red) / (float)p.P;
    inv_sigma[t] = var > 0.f ? 1.f / sqrtf(var) : 0.f;
  }
  for (int i = tid; i < p.P; i += 256) {
    float sc = 0.f;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      if (!(p.flags & (1u << t))) continue;
      const float x = terms[t][base + i];
      sc += (x - mu[t]) * inv_sigma[t];
      if (p.components_out) p.components_out[(long long)t * p.B * p.Nv + base + i] = x;
    }
    p.scores_out[base + i] = sc;
  }
}

// The same for frames of at most 256 * NPT tokens: every value a thread needs is fetched in one
// batch and stays in registers, and the three terms share each of the two block reductions, so a
// frame costs one trip to memory instead of one per term and per moment.
template <int NPT>
__global__ __launch_bounds__(256) void fuse_scores_reg(ScoreParams p) {
  __shared__ float red[3][4];
  const int f = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long base = (long long)b * p.Nv + (long long)f * p.P;
  const bool on[3] = {(p.flags & HIPPO_SCORE_ATTN) != 0, (p.flags & HIPPO_SCORE_TEMP) != 0,
                      (p.flags & HIPPO_SCORE_SPA) != 0};
  float x[3][NPT];
#pragma unroll
  for (int u = 0; u < NPT; ++u) {
    const int i = tid + 256 * u;
    const bool ok = i < p.P;
    x[0][u] = x[1][u] = x[2][u] = 0.f;
    if (ok && on[1]) x[1][u] = p.s_temp[base + i];
    if (ok && on[2]) x[2][u] = p.s_spa[base + i];
    if (ok && on[0]) {
      float a = sum_col_partials(p, b, (long long)f * p.P + i);
      a /= (float)p.H * (float)p.L;
      if (p.attn_mass_inout != nullptr) {
        a += p.attn_mass_inout[base + i];
        p.attn_mass_inout[base + i] = a;
      }
      p.s_attn[base + i] = a;
      x[0][u] = a;
    }
  }
  auto reduce3 = [&](float (&v)[3]) {                  // block sums of three values at once
#pragma unroll
    for (int t = 0; t < 3; ++t) v[t] = wave_sum(v[t]);
    __syncthreads();
    if (lane == 0) { red[0][wave] = v[0]; red[1][wave] = v[1]; red[2][wave] = v[2]; }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 3; ++t) v[t] = (red[t][0] + red[t][1]) + (red[t][2] + red[t][3]);
  };
  float mu[3] = {0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 3; ++t)
#pragma unroll
    for (int u = 0; u < NPT; ++u) mu[t] += x[t][u];
  reduce3(mu);
  float var[3] = {0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    mu[t] /= (float)p.P;
#pragma unroll
    for (int u = 0; u < NPT; ++u) {
      const float d = (tid + 256 * u < p.P) ? x[t][u] - mu[t] : 0.f;
      var[t] = fmaf(d, d, var[t]);
    }
  }
  reduce3(var);
  float inv_sigma[3];
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    var[t] /= (float)p.P;
    inv_sigma[t] = (on[t] && var[t] > 0.f) ? 1.f / sqrtf(var[t]) : 0.f;
  }
#pragma unroll
  for (int u = 0; u < NPT; ++u) {
    const int i = tid + 256 * u;
    if (i >= p.P) continue;
    float sc = 0.f;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      if (!on[t]) continue;
      sc += (x[t][u] - mu[t]) * inv_sigma[t];
      if (p.components_out) p.components_out[(long long)t * p.B * p.Nv + base + i] = x[t][u];
    }
    p.scores_out[base + i] = sc;
  }
}

// =================================================================================================
// host launch
// =================================================================================================
int score_token_tile(int dtype) { return dtype == HIPPO_DTYPE_BF16 ? kSaMfmaTile : kSaValuTile; }

// Row splits of the s_attn sweeps (bf16 path): enough blocks for two per compute unit, which is what
// lets the MFMA and the exp work of different waves overlap; a split keeps at least two 64-row chunks.
// How many runs the query rows of a KV head are cut into (one block of the sweeps per run).  A compute
// unit holds two sweep blocks; measured at the 16K shape, two co-resident blocks take 2.1 us per 64-row
// chunk each, a block alone 1.29 us, and a block's start (keys, first chunk) 3.2 resp. 2.5 us.  The
// blocks are dealt to the compute units in rounds, so what counts is the busiest unit: ceil(blocks / 256)
// blocks, two at a time, an odd last one alone.  520 unsplit blocks of 28 chunks, for example, put a third
// block on a few units, which then start a 28-chunk sweep when all others are done (91 us against 81-83
// with three or four runs); 256 blocks of 14 chunks are best cut in two (one round, two blocks per unit).
int score_row_splits(int dtype, long long blocks_unsplit, int rows_per_kv_head) {
  if (dtype != HIPPO_DTYPE_BF16) return 1;
  const int chunks = (rows_per_kv_head + 63) / 64;
  int best = 1;
  double best_cost = 0.0;
  for (int rs = 1; rs <= 4; ++rs) {
    if (rs > 1 && chunks / rs < 2) break;                       // at least two chunks per block
    const int cpb = (chunks + rs - 1) / rs;                     // chunks per block
    const long long per_cu = (blocks_unsplit * rs + kNumCU - 1) / kNumCU;
    const double pair = cpb * 2.1 + 3.2, alone = cpb * 1.29 + 2.5;
    const double cost = (double)(per_cu / 2) * pair + (per_cu % 2 ? alone : 0.0);
    if (rs == 1 || cost < best_cost * 0.97) {                   // a finer cut has to pay for its extra column partials
      best = rs;
      best_cost = cost;
    }
  }
  return best;
}

template <typename T, int D>
static hipError_t launch_sattn_valu(const ScoreParams& p, hipStream_t st) {
  dim3 grid(p.n_tile, p.Hkv, p.Bz);
  hipLaunchKernelGGL((sattn_valu<T, D, 1>), grid, dim3(256), 0, st, p);
  const long long rows = (long long)p.Bz * p.H * p.L;
  hipLaunchKernelGGL(sattn_row_lse, dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, st, p);
  hipLaunchKernelGGL((sattn_valu<T, D, 2>), grid, dim3(256), 0, st, p);
  return hipGetLastError();
}

// riders: 0 = pass 1 in a launch of its own, else that many riding blocks (run_riders: of the frame-run kind)
template <int D>
static hipError_t launch_sattn_mfma(const ScoreParams& p, hipStream_t st, long long riders, bool run_riders) {
  if (p.n_tile > 65535 || (long long)p.n_rsplit * p.Bz > 65535) return hipErrorInvalidValue;
  dim3 grid(p.Hkv, p.n_tile, p.n_rsplit * p.Bz);
  if (riders > 0) {
    const long long n_sattn = (long long)p.n_tile * p.Hkv * p.n_rsplit * p.Bz;
    const dim3 fused((unsigned)(n_sattn + riders));
    if (run_riders)
      hipLaunchKernelGGL((sattn_pass1_with_emb<D, true>), fused, dim3(kSaWaves * 64), 0, st, p, (int)n_sattn);
    else
      hipLaunchKernelGGL((sattn_pass1_with_emb<D, false>), fused, dim3(kSaWaves * 64), 0, st, p, (int)n_sattn);
  } else {
    hipLaunchKernelGGL((sattn_mfma<D, 1>), grid, dim3(kSaWaves * 64), 0, st, p);
  }
  const long long rows = (long long)p.Bz * p.H * p.L;
  hipLaunchKernelGGL(sattn_row_lse, dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, st, p);
  hipLaunchKernelGGL((sattn_mfma<D, 2>), grid, dim3(kSaWaves * 64), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_score(const ScoreParams& p_in, hipStream_t st) {
  ScoreParams p = p_in;
  {
    const int rows = p.L * p.G, chunks = (rows + 63) / 64, rs = p.n_rsplit > 0 ? p.n_rsplit : 1;
    p.rows_per_split = (chunks + rs - 1) / rs * 64;
    p.q_step_i = 64 / p.G;
    p.q_step_g = 64 % p.G;
    p.q_last_i = (rows - 1) / p.G;
    p.q_last_g = (rows - 1) % p.G;
  }
  hipError_t e = hipSuccess;
  const bool accumulate_only = (p.flags & HIPPO_SCORE_ACCUMULATE_ONLY) != 0;
  // bf16 with the paper's small crops: the embedding terms ride in the launch of s_attn's pass 1
  const bool want_emb = (p.flags & (HIPPO_SCORE_TEMP | HIPPO_SCORE_SPA)) != 0;
  // bf16 crops of at most 32 tokens.  Up to 512 channels a block sweeps one crop position over a run
  // of frames; the runs are as long as still leaves every compute unit a block (at most 8 frames: a
  // run fetches its two neighbour frames on top of its own).  Wider embeddings: a block per two crops.
  const long long crops_per_frame = (long long)((p.gh + p.ch - 1) / p.ch) * ((p.gw + p.cw - 1) / p.cw);
  {
    const long long per_cu = crops_per_frame * p.F * p.B / kNumCU;
    p.emb_run = (int)std::max<long long>(1, std::min<long long>(std::min<long long>(8, p.F), per_cu));
  }
  const bool small_crops = p.dtype == HIPPO_DTYPE_BF16 && p.ch * p.cw <= 32;
  const bool emb_in_runs = small_crops && (p.emb ? p.emb_dim : p.Hkv * p.D) <= 512;
  const long long n_riders = emb_in_runs ? crops_per_frame * ((p.F + p.emb_run - 1) / p.emb_run) * p.B
                                         : (crops_per_frame * p.F * p.B + 1) / 2;
  const long long fused_blocks = (long long)p.n_tile * p.Hkv * p.n_rsplit * p.Bz + n_riders;
  const bool emb_rides = want_emb && !accumulate_only && (p.flags & HIPPO_SCORE_ATTN) && small_crops &&
                         fused_blocks < (1ll << 31);
  const long long riders = emb_rides ? n_riders : 0;
  if ((p.flags & HIPPO_SCORE_ATTN) || accumulate_only) {
    if (p.dtype == HIPPO_DTYPE_BF16)
      e = (p.D == 128) ? launch_sattn_mfma<128>(p, st, riders, emb_in_runs)
                       : launch_sattn_mfma<64>(p, st, riders, emb_in_runs);
    else
      e = (p.D == 128) ? launch_sattn_valu<float, 128>(p, st) : launch_sattn_valu<float, 64>(p, st);
    if (e != hipSuccess) return e;
    if (accumulate_only) {   // otherwise the fusion kernel finishes the attention mass itself
      const long long n = (long long)p.B * p.Nv;
      hipLaunchKernelGGL(sattn_finalize, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p);
      return hipGetLastError();
    }
  }
  if (want_emb && !emb_rides) {
    const int ncy = (p.gh + p.ch - 1) / p.ch, ncx = (p.gw + p.cw - 1) / p.cw;
    dim3 grid(ncy * ncx, p.F, p.B);
    if (p.dtype == HIPPO_DTYPE_BF16) {
      const int crop = p.ch * p.cw;
      if (emb_in_runs && n_riders < (1ll << 31))
        hipLaunchKernelGGL(emb_scores_run32, dim3((unsigned)n_riders), dim3(512), 0, st, p);
      else if (crop <= 32) hipLaunchKernelGGL(emb_scores_mfma32, grid, dim3(256), 0, st, p);
      else if (crop <= 48) hipLaunchKernelGGL(emb_scores_mfma<3>, grid, dim3(256), 0, st, p);
      else hipLaunchKernelGGL(emb_scores_mfma<4>, grid, dim3(256), 0, st, p);
    } else {
      hipLaunchKernelGGL(emb_scores<float>, grid, dim3(256), 0, st, p);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (p.P <= 256) hipLaunchKernelGGL(fuse_scores_reg<1>, dim3(p.F, p.B), dim3(256), 0, st, p);
  else if (p.P <= 1024) hipLaunchKernelGGL(fuse_scores_reg<4>, dim3(p.F, p.B), dim3(256), 0, st, p);
  else hipLaunchKernelGGL(fuse_scores, dim3(p.F, p.B), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace hippo
