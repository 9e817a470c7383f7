// Writer for the 8-bit cache format of the fp8 attention calls (a cache-format variant the paper
// does not discuss): a bf16 or fp32 K/V cache becomes E4M3 codes plus one fp32 multiplier per
// (batch element, KV head) and tensor.
//   multiplier = max|x| / 448 over the head's rows (1 when the maximum is 0)
//   code       = the E4M3 value nearest to x / multiplier, ties to the even code
// Two launches: every block reduces |x| over its slice of a head's rows; then every block reduces
// the (few) slice maxima of its head again, encodes its slice and block 0 stores the multiplier.
// No atomics, no ordering between blocks: the result is deterministic.
#include "common.h"

namespace hippo {

constexpr int kQuantThreads = 256;

// 16-byte source vectors per row and elements per vector, for T = float or bf16 bits
template <typename T>
__device__ __forceinline__ float vec_absmax(const u32x4& v) {
  float x[Elem<T>::kPerVec];
  Elem<T>::unpack(v, x);
  float m = 0.f;
#pragma unroll
  for (int i = 0; i < Elem<T>::kPerVec; ++i) m = fmaxf(m, fabsf(x[i]));   // NaN inputs are ignored
  return m;
}

__device__ __forceinline__ float block_max_256(float v, float* red) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// grid (n_slices, 2 * Hkv, B): blockIdx.y = 2 * hk + (0 = K, 1 = V)
template <typename T>
__global__ __launch_bounds__(kQuantThreads) void kv_absmax(QuantParams p) {
  __shared__ float red[4];
  const int which = blockIdx.y & 1, hk = blockIdx.y >> 1, b = blockIdx.z;
  const T* src = (const T*)(which ? p.v_src : p.k_src) + (long long)b * p.ssb + (long long)hk * p.ssh;
  constexpr int PV = Elem<T>::kPerVec;
  // a row holds 2^vshift 16-byte vectors (head dims 64 and 128): rows and vectors part by a shift,
  // the slice bounds are the only division of the kernel
  const int vshift = __builtin_ctz(p.D / PV), vmask = (1 << vshift) - 1;
  const long long n_vec = (long long)p.n_rows << vshift;
  const long long per = (n_vec + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per, hi = min(n_vec, lo + per);
  float m = 0.f;
  for (long long e0 = lo + threadIdx.x; e0 < hi; e0 += 4 * kQuantThreads) {
    u32x4 v[4];                                            // four loads in flight per thread
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long e = e0 + u * kQuantThreads;
      v[u] = (u32x4){0u, 0u, 0u, 0u};
      if (e < hi) v[u] = *(const u32x4*)(src + (e >> vshift) * p.ssn + ((int)e & vmask) * PV);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) m = fmaxf(m, vec_absmax<T>(v[u]));
  }
  m = block_max_256(m, red);
  if (threadIdx.x == 0) p.partial[((long long)(b * p.Hkv + hk) * 2 + which) * gridDim.x + blockIdx.x] = m;
}

// two floats -> two E4M3 codes in the low half of the result (round to nearest even)
__device__ __forceinline__ unsigned encode2(float a, float b) {
  return (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu;
}

template <typename T>
__global__ __launch_bounds__(kQuantThreads) void kv_encode(QuantParams p) {
  __shared__ float red[4];
  const int which = blockIdx.y & 1, hk = blockIdx.y >> 1, b = blockIdx.z;
  // the head's maximum from the slice maxima (at most kQuantThreads of them)
  const float* part = p.partial + ((long long)(b * p.Hkv + hk) * 2 + which) * gridDim.x;
  const float amax = block_max_256(threadIdx.x < gridDim.x ? part[threadIdx.x] : 0.f, red);
  const float mult = amax > 0.f ? amax / 448.0f : 1.0f;
  if (blockIdx.x == 0 && threadIdx.x == 0) (which ? p.v_scale : p.k_scale)[b * p.Hkv + hk] = mult;

  const T* src = (const T*)(which ? p.v_src : p.k_src) + (long long)b * p.ssb + (long long)hk * p.ssh;
  unsigned char* dst = (unsigned char*)(which ? p.v_dst : p.k_dst) + (long long)b * p.dsb + (long long)hk * p.dsh;
  constexpr int PV = Elem<T>::kPerVec;
  constexpr int SV = 16 / PV;                         // source vectors per 16 codes
  const int cshift = __builtin_ctz(p.D / 16), cmask = (1 << cshift) - 1;   // 2^cshift 16-byte code vectors per row
  const long long n_vec = (long long)p.n_rows << cshift;
  const long long per = (n_vec + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per, hi = min(n_vec, lo + per);
  for (long long e0 = lo + threadIdx.x; e0 < hi; e0 += 4 * kQuantThreads) {
    u32x4 raw[4][SV];                                      // every load of four code vectors in flight at once
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long e = min(e0 + u * kQuantThreads, hi - 1);     // past the slice: a repeat, not stored
      const long long row = e >> cshift;
      const int vec = (int)e & cmask;
#pragma unroll
      for (int s = 0; s < SV; ++s) raw[u][s] = *(const u32x4*)(src + row * p.ssn + vec * 16 + s * PV);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long e = e0 + u * kQuantThreads;
      if (e >= hi) break;
      float x[16];
#pragma unroll
      for (int s = 0; s < SV; ++s) Elem<T>::unpack(raw[u][s], x + s * PV);
      unsigned w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        w[i] = encode2(x[4 * i] / mult, x[4 * i + 1] / mult) | (encode2(x[4 * i + 2] / mult, x[4 * i + 3] / mult) << 16);
      u32x4 out;
      out.x = w[0]; out.y = w[1]; out.z = w[2]; out.w = w[3];
      *(u32x4*)(dst + (e >> cshift) * p.dsn + ((int)e & cmask) * 16) = out;
    }
  }
}

int quant_slices(int n_rows, int head_dim) {
  // about 16 KB of codes per block, at most one slice per thread of the second reduction
  const long long codes = (long long)n_rows * head_dim;
  long long n = (codes + 16383) / 16384;
  if (n < 1) n = 1;
  if (n > kQuantThreads) n = kQuantThreads;
  return (int)n;
}

hipError_t launch_quantize(const QuantParams& p, hipStream_t st) {
  dim3 grid(p.n_slices, 2 * p.Hkv, p.B);
  if (p.src_dtype == HIPPO_DTYPE_BF16) {
    hipLaunchKernelGGL(kv_absmax<uint16_t>, grid, dim3(kQuantThreads), 0, st, p);
    hipLaunchKernelGGL(kv_encode<uint16_t>, grid, dim3(kQuantThreads), 0, st, p);
  } else {
    hipLaunchKernelGGL(kv_absmax<float>, grid, dim3(kQuantThreads), 0, st, p);
    hipLaunchKernelGGL(kv_encode<float>, grid, dim3(kQuantThreads), 0, st, p);
  }
  return hipGetLastError();
}

}  // namespace hippo
