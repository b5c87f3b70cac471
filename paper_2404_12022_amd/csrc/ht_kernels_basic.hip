// Row-wise and integer kernels of the tree-verify step, plus dtype-generic reference-grade
// products and attention used by the fp32 model path (the bf16 hot path uses the MFMA kernels).
#include "ht_common.h"

namespace ht {

#define HT_DISPATCH_DTYPE(dtype, ...)                       \
  if ((dtype) == 0) { typedef float T; __VA_ARGS__ }        \
  else { typedef bf16_t T; __VA_ARGS__ }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ inline float wave_max_dpp(float x) {
  // quads, half rows and rows by data-parallel-primitive moves, then rows and halves of the wave by lane swaps
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true)));    // lanes 1 0 3 2
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true)));    // lanes 2 3 0 1
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, true)));   // half row mirrored
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, true)));   // row mirrored
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  u = __float_as_uint(x);
  auto r2 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r2[0]), __uint_as_float(r2[1]));
}
__device__ inline int wave_min_dpp(int x) {
  x = min(x, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true));
  x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true));
  x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x141, 0xf, 0xf, true));
  x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x140, 0xf, 0xf, true));
  auto r = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)x, false, false);
  x = min((int)r[0], (int)r[1]);
  auto r2 = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
  return min((int)r2[0], (int)r2[1]);
}

// block-wide sum for 256-thread blocks; `red` is __shared__ float[4]
__device__ inline float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ inline float block_max_256(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// ------------------------------------------------------------------------------------------------ embed
template <typename T>
__global__ void embed_kernel(const T* __restrict__ emb, const int32_t* __restrict__ tok, float* __restrict__ x, int d) {
  const int m = blockIdx.x;                     // blockIdx.y: which share of the row's columns
  const T* row = emb + (size_t)tok[m] * d;
  for (int c = blockIdx.y * blockDim.x + threadIdx.x; c < d; c += gridDim.y * blockDim.x)
    x[(size_t)m * d + c] = Conv<T>::load(row + c);
}
hipError_t launch_embed(int dtype, const void* emb, const int32_t* tok, float* x, int M, int d, hipStream_t s) {
  const int shares = d >= 2048 ? 4 : 1;         // a few workgroups per row: a row is one dependent round trip per pass
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(embed_kernel<T>, dim3(M, shares), dim3(256), 0, s, (const T*)emb, tok, x, d);)
  return hipGetLastError();
}

__global__ void copy_rows_kernel(const float* __restrict__ src, float* __restrict__ dst, size_t count) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) dst[i] = src[i];
}
hipError_t launch_load_rows(const float* src, float* x, int M, int d, hipStream_t s) {
  size_t count = (size_t)M * d;
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, src, x, count);
  return hipGetLastError();
}

template <typename T>
__global__ void convert_to_f32_kernel(const T* __restrict__ src, float* __restrict__ dst, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = Conv<T>::load(src + i);
}
hipError_t launch_convert_to_f32(int dtype, const void* src, float* dst, int n, hipStream_t s) {
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(convert_to_f32_kernel<T>, dim3((n + 255) / 256), dim3(256), 0, s,
                                              (const T*)src, dst, n);)
  return hipGetLastError();
}

// dst[i] = bf16(src[i]), four elements per thread (count a multiple of 4)
__global__ void convert_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, size_t quads) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= quads) return;
  const float4 v = *(const float4*)(src + i * 4);
  *(uint2*)(dst + i * 4) = pack4_bf16(v.x, v.y, v.z, v.w);
}
hipError_t launch_convert_to_bf16(const float* src, void* dst, size_t count, hipStream_t s) {
  if (count % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(convert_to_bf16_kernel, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, s, src, (bf16_t*)dst,
                     count / 4);
  return hipGetLastError();
}

__global__ void reduce_splits_kernel(const float* __restrict__ part, int nsplit, size_t stride, float* __restrict__ out) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= stride) return;
  float v = part[i];
  for (int sp = 1; sp < nsplit; ++sp) v += part[sp * stride + i];
  out[i] = v;
}
hipError_t launch_reduce_splits(const float* part, int nsplit, size_t stride, float* out, hipStream_t s) {
  hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)((stride + 255) / 256)), dim3(256), 0, s, part, nsplit, stride, out);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ residual + RMSNorm
// x[m] += sum over split-K partials of the previous projection (fixed order: deterministic), the
// updated residual is optionally saved (layer-t hidden states), then u[m] = x[m] * rsqrt(mean(x^2)+eps) * gain.
// One block of NT threads per row, four consecutive columns per thread and pass, every load of a pass
// issued before the first add so a row costs one memory round trip.
__device__ inline float block_sum_any(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += red[w];
  return t;
}

template <typename T, int NS>
__global__ void add_norm_kernel(float* __restrict__ x, const float* __restrict__ part, size_t part_stride,
                                const T* __restrict__ gain, T* __restrict__ u, float* __restrict__ save_h, int d,
                                float eps) {
  __shared__ float red[16];
  const int m = blockIdx.x;
  float* xr = x + (size_t)m * d;
  const float* pr = part + (size_t)m * d;
  float ss = 0.f;
  constexpr int MAXP = 4;                       // d <= MAXP * 4 * blockDim.x (checked by the launcher)
  float4 keep[MAXP];
#pragma unroll
  for (int p = 0; p < MAXP; ++p) {
    const int c = (p * blockDim.x + threadIdx.x) * 4;
    if (c < d) {
      float4 v = *(const float4*)(xr + c);
      float4 pv[NS > 0 ? NS : 1];
#pragma unroll
      for (int sp = 0; sp < NS; ++sp) pv[sp] = *(const float4*)(pr + sp * part_stride + c);
#pragma unroll
      for (int sp = 0; sp < NS; ++sp) { v.x += pv[sp].x; v.y += pv[sp].y; v.z += pv[sp].z; v.w += pv[sp].w; }
      if (NS) *(float4*)(xr + c) = v;
      if (save_h) *(float4*)(save_h + (size_t)m * d + c) = v;
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      keep[p] = v;
    }
  }
  ss = block_sum_any(ss, red);
  const float scale = 1.0f / sqrtf(ss / (float)d + eps);
  if (u) {
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
      const int c = (p * blockDim.x + threadIdx.x) * 4;
      if (c < d) {
        const float4 v = keep[p];
        T* dst = u + (size_t)m * d + c;
        Conv<T>::store(dst + 0, v.x * scale * Conv<T>::load(gain + c + 0));
        Conv<T>::store(dst + 1, v.y * scale * Conv<T>::load(gain + c + 1));
        Conv<T>::store(dst + 2, v.z * scale * Conv<T>::load(gain + c + 2));
        Conv<T>::store(dst + 3, v.w * scale * Conv<T>::load(gain + c + 3));
      }
    }
  }
}
// kNormParts blocks per row: block (m, q) owns columns q dq .. (q + 1) dq - 1, dq = d / kNormParts.
template <int NS>
__global__ void add_norm_parts_kernel(float* __restrict__ x, const float* __restrict__ part, size_t part_stride,
                                      const bf16_t* __restrict__ gain, bf16_t* __restrict__ u,
                                      float* __restrict__ save_h, float* __restrict__ ss_out, int d) {
  __shared__ float red[16];
  const int m = blockIdx.x, dq = d / kNormParts, c0 = blockIdx.y * dq;
  float* xr = x + (size_t)m * d;
  const float* pr = part + (size_t)m * d;
  float ss = 0.f;
  constexpr int MAXP = 4;                       // dq <= MAXP * 4 * blockDim.x (checked by the launcher)
#pragma unroll
  for (int p = 0; p < MAXP; ++p) {
    const int cl = (p * blockDim.x + threadIdx.x) * 4;
    if (cl < dq) {
      const int c = c0 + cl;
      float4 v = *(const float4*)(xr + c);
      float4 pv[NS > 0 ? NS : 1];
#pragma unroll
      for (int sp = 0; sp < NS; ++sp) pv[sp] = *(const float4*)(pr + sp * part_stride + c);
#pragma unroll
      for (int sp = 0; sp < NS; ++sp) { v.x += pv[sp].x; v.y += pv[sp].y; v.z += pv[sp].z; v.w += pv[sp].w; }
      if (NS) *(float4*)(xr + c) = v;
      if (save_h) *(float4*)(save_h + (size_t)m * d + c) = v;
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      if (u) {
        const uint2 g4 = *(const uint2*)(gain + c);
        *(uint2*)(u + (size_t)m * d + c) =
            pack4_bf16(v.x * __uint_as_float(g4.x << 16), v.y * __uint_as_float(g4.x & 0xffff0000u),
                       v.z * __uint_as_float(g4.y << 16), v.w * __uint_as_float(g4.y & 0xffff0000u));
      }
    }
  }
  ss = block_sum_any(ss, red);
  if (threadIdx.x == 0 && ss_out) ss_out[(size_t)m * kNormParts + blockIdx.y] = ss;
}
hipError_t launch_add_norm_parts(float* x, const float* part, int nsplit, size_t part_stride, const void* gain, void* u,
                                 float* save_h, float* ss, int M, int d, hipStream_t s) {
  if (d % (4 * kNormParts) || nsplit < 0 || nsplit > kMaxSplitK) return hipErrorInvalidValue;
  const int dq = d / kNormParts;
  int nt = 64;
  while (nt < 1024 && nt * 4 < dq) nt *= 2;
  if (dq > 16 * nt) return hipErrorInvalidValue;
#define HT_ADD_NORM_PARTS(NS)                                                                                      \
  case NS:                                                                                                         \
    hipLaunchKernelGGL((add_norm_parts_kernel<NS>), dim3(M, kNormParts), dim3(nt), 0, s, x, part, part_stride,     \
                       (const bf16_t*)gain, (bf16_t*)u, save_h, ss, d);                                            \
    break;
  switch (nsplit) {
    HT_ADD_NORM_PARTS(0) HT_ADD_NORM_PARTS(1) HT_ADD_NORM_PARTS(2) HT_ADD_NORM_PARTS(3) HT_ADD_NORM_PARTS(4)
    HT_ADD_NORM_PARTS(5) HT_ADD_NORM_PARTS(6) HT_ADD_NORM_PARTS(7) HT_ADD_NORM_PARTS(8)
  }
#undef HT_ADD_NORM_PARTS
  return hipGetLastError();
}

hipError_t launch_add_norm(int dtype, float* x, const float* part, int nsplit, size_t part_stride, const void* gain,
                           void* u, float* save_h, int M, int d, float eps, hipStream_t s) {
  if (d % 4 || nsplit < 0 || nsplit > kMaxSplitK) return hipErrorInvalidValue;
  int nt = 64;
  while (nt < 1024 && nt * 4 < d) nt *= 2;
  if (d > 16 * nt) return hipErrorInvalidValue;
#define HT_ADD_NORM(NS)                                                                                         \
  case NS:                                                                                                      \
    hipLaunchKernelGGL((add_norm_kernel<T, NS>), dim3(M), dim3(nt), 0, s, x, part, part_stride, (const T*)gain, \
                       (T*)u, save_h, d, eps);                                                                  \
    break;
  HT_DISPATCH_DTYPE(dtype, switch (nsplit) {
    HT_ADD_NORM(0) HT_ADD_NORM(1) HT_ADD_NORM(2) HT_ADD_NORM(3) HT_ADD_NORM(4) HT_ADD_NORM(5) HT_ADD_NORM(6)
    HT_ADD_NORM(7) HT_ADD_NORM(8)
  })
#undef HT_ADD_NORM
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ rotary
// cs[m][j] = (cos, sin) of (n + depth[m]) * base^(-2j/hd), evaluated in fp64 and rounded once.
__global__ void rope_table_kernel(float2* __restrict__ cs, const int32_t* __restrict__ depth, int n, int half,
                                  float base, const int32_t* __restrict__ n_dev) {
  n = cache_len(n, n_dev);
  const int m = blockIdx.x;
  const int j = threadIdx.x;
  if (j >= half) return;
  const double pos = (double)(n + (depth ? depth[m] : m));      // no depth table: row m at position n + m
  const double inv = exp(-(2.0 * (double)j / (double)(2 * half)) * log((double)base));
  double sn, cn;
  sincos(pos * inv, &sn, &cn);
  cs[(size_t)m * half + j] = make_float2((float)cn, (float)sn);
}
hipError_t launch_rope_table(float* cs, const int32_t* depth, int n, int M, int hd, float base, hipStream_t s,
                             const int32_t* n_dev) {
  hipLaunchKernelGGL(rope_table_kernel, dim3(M), dim3(hd / 2), 0, s, (float2*)cs, depth, n, hd / 2, base, n_dev);
  return hipGetLastError();
}

// Rotates q and k of row m at its tree position and appends k, v to cache slot n+m.
// Layouts: q[M][Hq][hd]; K cache [cap][Hkv][hd]; V cache [Hkv][hd][cap] (key index contiguous).
// The inputs may come as `nsplit` split-K partial sums `split_stride` elements apart (added in index order).
template <typename T, typename TIN>
__global__ void rope_append_kernel(const TIN* __restrict__ q_in, int q_stride, const TIN* __restrict__ k_in,
                                   int k_stride, const TIN* __restrict__ v_in, int v_stride, int nsplit,
                                   size_t split_stride, const float2* __restrict__ cs, T* __restrict__ q,
                                   T* __restrict__ kc, T* __restrict__ vc, int n, int Hq, int Hkv, int hd, int cap,
                                   int paired, const int32_t* __restrict__ n_dev) {
  n = cache_len(n, n_dev);
  const int m = blockIdx.x, hh = blockIdx.y, j = threadIdx.x, half = hd / 2;
  if (j >= half) return;
  const float2 c = cs[(size_t)m * half + j];
  if (hh < Hq + Hkv) {
    const TIN* src = hh < Hq ? q_in + (size_t)m * q_stride + (size_t)hh * hd
                             : k_in + (size_t)m * k_stride + (size_t)(hh - Hq) * hd;
    // paired: the q and k columns of a head come in the packed projection's order, every run of 8 features
    // followed by the run of their rotary partners
    const int ja = paired ? 16 * (j >> 3) + (j & 7) : j, jb = paired ? ja + 8 : j + half;
    float a = Conv<TIN>::load(src + ja), b = Conv<TIN>::load(src + jb);
    for (int sp = 1; sp < nsplit; ++sp) {
      a += Conv<TIN>::load(src + sp * split_stride + ja);
      b += Conv<TIN>::load(src + sp * split_stride + jb);
    }
    const float ra = a * c.x - b * c.y, rb = b * c.x + a * c.y;
    T* dst = hh < Hq ? q + ((size_t)m * Hq + hh) * hd : kc + ((size_t)(n + m) * Hkv + (hh - Hq)) * hd;
    Conv<T>::store(dst + j, ra);
    Conv<T>::store(dst + j + half, rb);
  } else {
    const int h = hh - Hq - Hkv;
    const TIN* src = v_in + (size_t)m * v_stride + (size_t)h * hd;
    float a = Conv<TIN>::load(src + j), b = Conv<TIN>::load(src + j + half);
    for (int sp = 1; sp < nsplit; ++sp) {
      a += Conv<TIN>::load(src + sp * split_stride + j);
      b += Conv<TIN>::load(src + sp * split_stride + j + half);
    }
    Conv<T>::store(vc + ((size_t)h * hd + j) * cap + n + m, a);
    Conv<T>::store(vc + ((size_t)h * hd + j + half) * cap + n + m, b);
  }
}
// The same, four feature pairs per thread (hd % 8 == 0): 16-byte loads of the partial sums, 8-byte stores of q
// and k.  blockIdx.x = row, 256 threads cover 256 / (hd / 8) heads.
template <typename TIN> __device__ inline void load4(const TIN* p, float (&v)[4]);
template <> __device__ inline void load4<float>(const float* p, float (&v)[4]) {
  const float4 t = *(const float4*)p;
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ inline void load4<bf16_t>(const bf16_t* p, float (&v)[4]) {
  const uint2 t = *(const uint2*)p;
  const bf16_t* h = (const bf16_t*)&t;
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = bf16_to_float(h[i]);
}
template <typename T> __device__ inline void store4(T* p, const float (&v)[4]);
template <> __device__ inline void store4<float>(float* p, const float (&v)[4]) {
  *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ inline void store4<bf16_t>(bf16_t* p, const float (&v)[4]) {
  *(uint2*)p = pack4_bf16(v[0], v[1], v[2], v[3]);
}

// One workgroup per (block of RB rows, head).  q and k heads: four feature pairs per thread and item, 16-byte loads,
// 8-byte stores.  v heads: the value cache is stored key-contiguous ([head][feature][slot]), so the rows go through LDS
// and every wavefront stores one feature of up to 64 consecutive rows at a time (a 2-byte store per row and feature
// straight from the row-major input touches a cache line of its own each).
template <typename T, typename TIN>
__global__ __launch_bounds__(256) void rope_append_rows_kernel(
    const TIN* __restrict__ q_in, int q_stride, const TIN* __restrict__ k_in, int k_stride, const TIN* __restrict__ v_in,
    int v_stride, int nsplit, size_t split_stride, const float* __restrict__ cs, T* __restrict__ q, T* __restrict__ kc,
    T* __restrict__ vc, int n, int M, int RB, int Hq, int Hkv, int hd, int cap, int paired,
    const int32_t* __restrict__ n_dev) {
  extern __shared__ __attribute__((aligned(16))) unsigned char rows_lds[];
  n = cache_len(n, n_dev);
  const int m0 = blockIdx.x * RB, hh = blockIdx.y, half = hd / 2;
  const int rows = M - m0 < RB ? M - m0 : RB;
  if (hh < Hq + Hkv) {
    const int per_row = half / 4;                          // items of four feature pairs
    for (int item = threadIdx.x; item < rows * per_row; item += 256) {
      const int m = m0 + item / per_row, j = (item % per_row) * 4;
      const TIN* src = hh < Hq ? q_in + (size_t)m * q_stride + (size_t)hh * hd
                               : k_in + (size_t)m * k_stride + (size_t)(hh - Hq) * hd;
      // paired: the q and k columns of a head come in the packed projection's order, every run of 8 features
      // followed by the run of their rotary partners
      const int ja = paired ? 16 * (j >> 3) + (j & 7) : j, jb = paired ? ja + 8 : j + half;
      float a[4], b[4];
      load4<TIN>(src + ja, a);
      load4<TIN>(src + jb, b);
      for (int sp = 1; sp < nsplit; ++sp) {
        float a2[4], b2[4];
        load4<TIN>(src + sp * split_stride + ja, a2);
        load4<TIN>(src + sp * split_stride + jb, b2);
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] += a2[i]; b[i] += b2[i]; }
      }
      const float4 c01 = *(const float4*)(cs + ((size_t)m * half + j) * 2), c23 = *(const float4*)(cs + ((size_t)m * half + j) * 2 + 4);
      const float c[4] = {c01.x, c01.z, c23.x, c23.z}, sn[4] = {c01.y, c01.w, c23.y, c23.w};
      float ra[4], rb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { ra[i] = a[i] * c[i] - b[i] * sn[i]; rb[i] = b[i] * c[i] + a[i] * sn[i]; }
      T* dst = hh < Hq ? q + ((size_t)m * Hq + hh) * hd : kc + ((size_t)(n + m) * Hkv + (hh - Hq)) * hd;
      store4<T>(dst + j, ra);
      store4<T>(dst + j + half, rb);
    }
    return;
  }
  // v head: rows into LDS (row stride hd + 2 elements: the column reads below fall on consecutive banks)
  const int h = hh - Hq - Hkv, ldr = hd + 2;
  T* tile = (T*)rows_lds;
  const int per_row = hd / 4;
  for (int item = threadIdx.x; item < rows * per_row; item += 256) {
    const int r = item / per_row, j = (item % per_row) * 4;
    const TIN* src = v_in + (size_t)(m0 + r) * v_stride + (size_t)h * hd + j;
    float a[4];
    load4<TIN>(src, a);
    for (int sp = 1; sp < nsplit; ++sp) {
      float a2[4];
      load4<TIN>(src + sp * split_stride, a2);
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] += a2[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) Conv<T>::store(tile + r * ldr + j + i, a[i]);
  }
  __syncthreads();
  // RB is 16, 32 or 64: a wavefront stores 64 / RB features of RB consecutive rows at a time
  const int r = threadIdx.x % RB, per_pass = 256 / RB;
  for (int e = threadIdx.x / RB; e < hd; e += per_pass)
    if (r < rows) vc[((size_t)h * hd + e) * cap + n + m0 + r] = tile[r * ldr + e];
}

// rows per workgroup of rope_append_rows_kernel: 16 (measured: blocks of 64 rows leave too few workgroups for passes of
// 64 - 128 rows, which are latency bound)
static int rope_rows_per_block(int dtype, int hd) { (void)dtype; (void)hd; return 16; }

hipError_t launch_rope_append(int dtype, const float* qkv, int nsplit, const float* cs, void* q, void* kc, void* vc,
                              int n, int M, int Hq, int Hkv, int hd, int cap, bool paired, hipStream_t s,
                              const int32_t* n_dev) {
  const int stride = (Hq + 2 * Hkv) * hd;
  if (hd % 8 == 0) {
    const int RB = rope_rows_per_block(dtype, hd);
    const size_t lds = (size_t)RB * (hd + 2) * (dtype == 0 ? 4 : 2);
    HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((rope_append_rows_kernel<T, float>), dim3((M + RB - 1) / RB, Hq + 2 * Hkv),
                                                dim3(256), lds, s, qkv, stride, qkv + (size_t)Hq * hd, stride,
                                                qkv + (size_t)(Hq + Hkv) * hd, stride, nsplit, (size_t)M * stride, cs,
                                                (T*)q, (T*)kc, (T*)vc, n, M, RB, Hq, Hkv, hd, cap, paired ? 1 : 0, n_dev);)
    return hipGetLastError();
  }
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((rope_append_kernel<T, float>), dim3(M, Hq + 2 * Hkv), dim3(hd / 2), 0,
                                              s, qkv, stride, qkv + (size_t)Hq * hd, stride,
                                              qkv + (size_t)(Hq + Hkv) * hd, stride, nsplit, (size_t)M * stride,
                                              (const float2*)cs, (T*)q, (T*)kc, (T*)vc, n, Hq, Hkv, hd, cap,
                                              paired ? 1 : 0, n_dev);)
  return hipGetLastError();
}
hipError_t launch_rope_append_split(int dtype, const void* q_in, const void* k_in, const void* v_in, const float* cs,
                                    void* q, void* kc, void* vc, int n, int M, int Hq, int Hkv, int hd, int cap,
                                    hipStream_t s) {
  if (hd % 8 == 0) {
    const int RB = rope_rows_per_block(dtype, hd);
    const size_t lds = (size_t)RB * (hd + 2) * (dtype == 0 ? 4 : 2);
    HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((rope_append_rows_kernel<T, T>), dim3((M + RB - 1) / RB, Hq + 2 * Hkv),
                                                dim3(256), lds, s, (const T*)q_in, Hq * hd, (const T*)k_in, Hkv * hd,
                                                (const T*)v_in, Hkv * hd, 1, (size_t)0, cs, (T*)q, (T*)kc, (T*)vc, n, M, RB, Hq,
                                                Hkv, hd, cap, 0, nullptr);)
    return hipGetLastError();
  }
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((rope_append_kernel<T, T>), dim3(M, Hq + 2 * Hkv), dim3(hd / 2), 0, s,
                                              (const T*)q_in, Hq * hd, (const T*)k_in, Hkv * hd, (const T*)v_in,
                                              Hkv * hd, 1, (size_t)0, (const float2*)cs, (T*)q, (T*)kc, (T*)vc, n, Hq, Hkv, hd,
                                              cap, 0, nullptr);)
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ SwiGLU gate
template <typename T>
__global__ void silu_mul_kernel(const float* __restrict__ gu, T* __restrict__ act, int f) {
  const int m = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= f) return;
  const float g = gu[(size_t)m * 2 * f + j], up = gu[(size_t)m * 2 * f + f + j];
  Conv<T>::store(act + (size_t)m * f + j, g / (1.0f + expf(-g)) * up);
}
hipError_t launch_silu_mul(int dtype, const float* gu, void* act, int M, int f, hipStream_t s) {
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(silu_mul_kernel<T>, dim3((f + 255) / 256, M), dim3(256), 0, s, gu,
                                              (T*)act, f);)
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ argmax / top-k
// (value, id) order: larger value first, lower id first on equal values.  NaN never wins.
__device__ inline bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// block-wide best for any block size that is a multiple of 64 (<= 1024); sv/si hold 16 entries
__device__ inline void block_best_any(float& v, int& i, float* sv, int* si) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(v, o, 64);
    int oi = __shfl_xor(i, o, 64);
    if (better(ov, oi, v, i)) { v = ov; i = oi; }
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = v; si[threadIdx.x >> 6] = i; }
  __syncthreads();
  v = sv[0]; i = si[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
    if (better(sv[w], si[w], v, i)) { v = sv[w]; i = si[w]; }
}

// g[row] = arg-max of a logit row, lowest id on ties.  1024 threads per row, 16-byte loads.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ z, int32_t* __restrict__ g, int V,
                                                      int vec) {
  __shared__ float sv[16];
  __shared__ int si[16];
  const float* row = z + (size_t)blockIdx.x * V;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  const int v4 = vec ? (V & ~3) : 0;            // vec: rows are 16-byte aligned
  for (int j = threadIdx.x * 4; j < v4; j += blockDim.x * 4) {
    const float4 q = *(const float4*)(row + j);
    if (better(q.x, j, bv, bi)) { bv = q.x; bi = j; }
    if (better(q.y, j + 1, bv, bi)) { bv = q.y; bi = j + 1; }
    if (better(q.z, j + 2, bv, bi)) { bv = q.z; bi = j + 2; }
    if (better(q.w, j + 3, bv, bi)) { bv = q.w; bi = j + 3; }
  }
  for (int j = v4 + threadIdx.x; j < V; j += blockDim.x)
    if (better(row[j], j, bv, bi)) { bv = row[j]; bi = j; }
  block_best_any(bv, bi, sv, si);
  if (threadIdx.x == 0) g[blockIdx.x] = bi == 0x7fffffff ? 0 : bi;
}
hipError_t launch_argmax(const float* z, int32_t* g, int M, int V, hipStream_t s) {
  const int vec = !((uintptr_t)z & 15) && !(V & 3);
  hipLaunchKernelGGL(argmax_kernel, dim3(M), dim3(1024), 0, s, z, g, V, vec);
  return hipGetLastError();
}

// cand[i][r], r < width[i+1]: the r-th entry of logit row i in (value desc, id asc) order.
// Two stages of the same selection: repeated block-wide arg-best over the entries that come strictly after
// the previous pick in that order.  Stage 1 runs it on kTopkSlices slices of the row in parallel and leaves
// each slice's best b entries in scratch (any of the row's top b is among its slice's top b); stage 2 runs
// it once more over those kTopkSlices * b survivors.
constexpr int kTopkSlices = 32;

template <bool FINAL>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ d, const float* __restrict__ sv_in,
                                                   const int32_t* __restrict__ si_in, float* __restrict__ sv_out,
                                                   int32_t* __restrict__ si_out, int32_t* __restrict__ cand,
                                                   const int32_t* __restrict__ width, int period, const int32_t* __restrict__ src_row,
                                                   int V) {
  __shared__ float sv[16];
  __shared__ int si[16];
  const int i = blockIdx.x, slice = blockIdx.y;
  const int b = width[i % period + 1];      // row i drafts the tree level i % period + 1
  // element range of this block: a slice of the logit row, or the survivors of all slices
  int lo, hi;
  if (FINAL) { lo = 0; hi = kTopkSlices * b; }
  else {
    const int per = (V + kTopkSlices - 1) / kTopkSlices;
    lo = slice * per;
    hi = lo + per < V ? lo + per : V;
  }
  float pv = INFINITY;
  int pi = -1;
  for (int r = 0; r < b; ++r) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int j = lo + threadIdx.x; j < hi; j += 256) {
      float v;
      int id;
      if (FINAL) { v = sv_in[(size_t)i * kTopkSlices * kMaxTopK + j]; id = si_in[(size_t)i * kTopkSlices * kMaxTopK + j]; }
      else { v = d[(size_t)(src_row ? src_row[i] : i) * V + j]; id = j; }
      const bool after = r == 0 || v < pv || (v == pv && id > pi);
      if (after && better(v, id, bv, bi)) { bv = v; bi = id; }
    }
    block_best_any(bv, bi, sv, si);
    if (threadIdx.x == 0) {
      if (FINAL) cand[i * kMaxTopK + r] = bi == 0x7fffffff ? 0 : bi;
      else {
        sv_out[(size_t)i * kTopkSlices * kMaxTopK + slice * b + r] = bi == 0x7fffffff ? -INFINITY : bv;
        si_out[(size_t)i * kTopkSlices * kMaxTopK + slice * b + r] = bi;
      }
    }
    pv = bv; pi = bi;
    __syncthreads();
  }
}
// The same two stages with the selection done by wavefronts on register-resident entries: every wavefront of a block
// takes a quarter of the block's entries (E per lane), picks its best b one by one (a wave-wide maximum by DPP moves,
// a ballot, the lowest id among equal values), the four lists meet in LDS and the first wavefront picks the best b
// of them the same way.  No block-wide barrier inside the rounds and no re-reading of the row.  The order is the
// total order (value descending, id ascending), so the result is that of `topk_kernel` bit for bit.
constexpr int kNoEntry = 0x7fffffff;       // id of an empty slot: loses against every real entry of the same value

template <int E>
__device__ inline void wave_select(float (&v)[E], int (&id)[E], int b, float* out_v, int* out_i) {
  const int lane = threadIdx.x & 63;
  for (int r = 0; r < b; ++r) {
    float bv = v[0];
    int bi = id[0];
#pragma unroll
    for (int e = 1; e < E; ++e)
      if (better(v[e], id[e], bv, bi)) { bv = v[e]; bi = id[e]; }
    const float top = wave_max_dpp(bv);
    const bool tie = bv == top;
    const uint64_t mask = __ballot(tie);
    int pick;
    if (mask & (mask - 1)) pick = wave_min_dpp(tie ? bi : kNoEntry);
    else pick = __builtin_amdgcn_readlane(bi, __builtin_amdgcn_readfirstlane(__builtin_ctzll(mask)));
    if (lane == 0) { out_v[r] = top; out_i[r] = pick; }
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (id[e] == pick) { v[e] = -INFINITY; id[e] = kNoEntry; }
  }
}

template <int E, bool FINAL>
__global__ __launch_bounds__(256) void topk_wave_kernel(const float* __restrict__ d, const float* __restrict__ sv_in,
                                                        const int32_t* __restrict__ si_in, float* __restrict__ sv_out,
                                                        int32_t* __restrict__ si_out, int32_t* __restrict__ cand,
                                                        const int32_t* __restrict__ width, int period,
                                                        const int32_t* __restrict__ src_row, int V) {
  __shared__ float list_v[5][kMaxTopK];
  __shared__ int list_i[5][kMaxTopK];
  const int i = blockIdx.x, slice = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = width[i % period + 1];      // row i drafts the tree level i % period + 1
  if (b <= 0) return;                       // uniform over the block
  int lo, hi;
  if (FINAL) { lo = 0; hi = kTopkSlices * b; }
  else {
    const int per = (V + kTopkSlices - 1) / kTopkSlices;
    lo = slice * per;
    hi = lo + per < V ? lo + per : V;
  }
  const int quarter = (hi - lo + 3) / 4;
  const int w0 = lo + wave * quarter, w1 = w0 + quarter < hi ? w0 + quarter : hi;
  const size_t base = FINAL ? (size_t)i * kTopkSlices * kMaxTopK : (size_t)(src_row ? src_row[i] : i) * V;
  float v[E];
  int id[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int j = w0 + lane + 64 * e;
    v[e] = -INFINITY;
    id[e] = kNoEntry;
    if (j < w1) {
      const float x = FINAL ? sv_in[base + j] : d[base + j];
      const int xi = FINAL ? si_in[base + j] : j;
      if (x == x && xi != kNoEntry) { v[e] = x; id[e] = xi; }      // NaN never wins
    }
  }
  wave_select<E>(v, id, b, list_v[wave], list_i[wave]);
  __syncthreads();
  if (wave) return;
  float v2[4];
  int id2[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v2[e] = lane < b ? list_v[e][lane] : -INFINITY;
    id2[e] = lane < b ? list_i[e][lane] : kNoEntry;
  }
  wave_select<4>(v2, id2, b, list_v[4], list_i[4]);
  if (lane < b) {                           // one wavefront: its LDS writes are ordered before these reads
    if (FINAL) cand[i * kMaxTopK + lane] = list_i[4][lane] == kNoEntry ? 0 : list_i[4][lane];
    else {
      sv_out[(size_t)i * kTopkSlices * kMaxTopK + slice * b + lane] = list_v[4][lane];
      si_out[(size_t)i * kTopkSlices * kMaxTopK + slice * b + lane] = list_i[4][lane];
    }
  }
}

// scratch: float[rows][kTopkSlices][kMaxTopK] followed by int32 of the same shape
size_t topk_scratch_bytes(int rows) { return (size_t)rows * kTopkSlices * kMaxTopK * 8; }
hipError_t launch_topk(const float* d, int32_t* cand, const int32_t* width, void* scratch, int rows, int period,
                       const int32_t* src_row, int V, hipStream_t s) {
  float* sv = (float*)scratch;
  int32_t* si = (int32_t*)(sv + (size_t)rows * kTopkSlices * kMaxTopK);
  // entries per lane of the first stage: a quarter of a slice over 64 lanes; of the second: a quarter of
  // kTopkSlices * b <= 2048 survivors
  const int per_lane = (((V + kTopkSlices - 1) / kTopkSlices + 3) / 4 + 63) / 64;
  const dim3 g1(rows, kTopkSlices), g2(rows, 1);
#define HT_TOPK_ARGS(in_v, in_i, out_v, out_i) d, in_v, in_i, out_v, out_i, cand, width, period, src_row, V
  if (per_lane <= 4)
    hipLaunchKernelGGL((topk_wave_kernel<4, false>), g1, dim3(256), 0, s, HT_TOPK_ARGS(nullptr, nullptr, sv, si));
  else if (per_lane <= 16)
    hipLaunchKernelGGL((topk_wave_kernel<16, false>), g1, dim3(256), 0, s, HT_TOPK_ARGS(nullptr, nullptr, sv, si));
  else          // very large vocabularies: block-wide selection, any row length
    hipLaunchKernelGGL(topk_kernel<false>, g1, dim3(256), 0, s, HT_TOPK_ARGS(nullptr, nullptr, sv, si));
  hipLaunchKernelGGL((topk_wave_kernel<8, true>), g2, dim3(256), 0, s, HT_TOPK_ARGS(sv, si, nullptr, nullptr));
#undef HT_TOPK_ARGS
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ tree build / accept / compact
__global__ void tree_build_kernel(const StepState* __restrict__ st, const int32_t* __restrict__ cand, TreeDev tree,
                                  int32_t* __restrict__ tok, int T) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= T) return;
  tok[v] = v == 0 ? st->root : cand[(tree.depth[v] - 1) * kMaxTopK + tree.rank[v]];
}
hipError_t launch_tree_build(const StepState* st, const int32_t* cand, TreeDev tree, int32_t* tok, int T,
                             hipStream_t s) {
  hipLaunchKernelGGL(tree_build_kernel, dim3((T + 63) / 64), dim3(64), 0, s, st, cand, tree, tok, T);
  return hipGetLastError();
}

// ---- tree chosen from the draft distributions
// lp[i][r] = log-softmax value of candidate r of draft row i:  z - (max + log(sum exp(z - max))) over the whole row.
// One block of 1024 threads per row; 16-byte loads when the row allows.
__global__ __launch_bounds__(1024) void cand_logprob_kernel(const float* __restrict__ d, const int32_t* __restrict__ cand,
                                                            int b, int V, int vec, float* __restrict__ lp) {
  __shared__ float red[16];
  const float* row = d + (size_t)blockIdx.x * V;
  const int v4 = vec ? (V & ~3) : 0;
  float peak = -INFINITY;
  for (int j = threadIdx.x * 4; j < v4; j += blockDim.x * 4) {
    const float4 q = *(const float4*)(row + j);
    peak = fmaxf(fmaxf(peak, fmaxf(q.x, q.y)), fmaxf(q.z, q.w));
  }
  for (int j = v4 + threadIdx.x; j < V; j += blockDim.x) peak = fmaxf(peak, row[j]);
  peak = wave_max(peak);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = peak;
  __syncthreads();
  peak = red[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) peak = fmaxf(peak, red[w]);
  float sum = 0.f;
  for (int j = threadIdx.x * 4; j < v4; j += blockDim.x * 4) {      // second pass: the row is in L2 now
    const float4 q = *(const float4*)(row + j);
    sum += (expf(q.x - peak) + expf(q.y - peak)) + (expf(q.z - peak) + expf(q.w - peak));
  }
  for (int j = v4 + threadIdx.x; j < V; j += blockDim.x) sum += expf(row[j] - peak);
  sum = block_sum_any(sum, red);
  const float lse = peak + logf(sum);
  if ((int)threadIdx.x < b) lp[blockIdx.x * kMaxTopK + threadIdx.x] = row[cand[blockIdx.x * kMaxTopK + threadIdx.x]] - lse;
}
hipError_t launch_cand_logprob(const float* d, const int32_t* cand, int rows, int b, int V, float* lp, hipStream_t s) {
  const int vec = !((uintptr_t)d & 15) && !(V & 3);
  hipLaunchKernelGGL(cand_logprob_kernel, dim3(rows), dim3(1024), 0, s, d, cand, b, V, vec, lp);
  return hipGetLastError();
}

// The T - 1 best nodes of the complete b-ary candidate tree of depth k in the order (score descending, depth
// ascending, rank path ascending), score = sum of lp along the path accumulated in float from the root down.
// A node never scores above its parent or its previous sibling, and each of the two comes first in that order, so
// the order is produced by a best-first walk: the frontier holds, for every node taken so far, its next sibling
// and (once) its first child; the best frontier entry becomes the next node.  The frontier never holds more than
// T <= 128 entries: slot j lives in the registers of lane j % 64 (two slots per lane), a round is one wave-wide
// maximum of the lanes' best scores, a ballot that names the winner (a second reduction over depth and path only
// when several lanes hold the best score), and register updates in two lanes: no barrier and no memory traffic
// inside the walk but the log-probability table in LDS.  Tables and tokens are written by all lanes at the end.
__device__ inline float not_nan(float v) { return v == v ? v : -INFINITY; }

// (depth, path) order of two frontier entries with equal scores
__device__ inline bool tie_first(int depth_a, uint64_t path_a, int depth_b, uint64_t path_b) {
  return depth_a != depth_b ? depth_a < depth_b : path_a < path_b;
}

__global__ __launch_bounds__(64) void tree_dynamic_kernel(const int32_t* __restrict__ root, const int32_t* __restrict__ cand,
                                                          const float* __restrict__ lp, int k, int b, int T,
                                                          TreeOut tree, int32_t* __restrict__ tok) {
  __shared__ float lp_s[kMaxTransfer * kMaxTopK];
  __shared__ int cand_s[kMaxTransfer * kMaxTopK];
  __shared__ int n_parent[kMaxTree], n_depth[kMaxTree], n_rank[kMaxTree];
  const int lane = threadIdx.x;
  for (int i = lane; i < k * kMaxTopK; i += 64) {
    const bool used = i % kMaxTopK < b;
    lp_s[i] = used ? not_nan(lp[i]) : -INFINITY;
    cand_s[i] = used ? cand[i] : 0;
  }
  for (int v = lane; v < kMaxTree; v += 64) {      // rows the walk does not reach (none, if the sizes were checked) hang under the root
    n_parent[v] = v ? 0 : -1;
    n_depth[v] = v ? 1 : 0;
    n_rank[v] = 0;
  }
  __syncthreads();
  // frontier slot: score, score of the parent, depth (0: empty), parent node, path = ranks from the root down, 6 bits
  // each, the last rank in the lowest digit
  float fs0 = -INFINITY, fs1 = -INFINITY, fb0 = 0.f, fb1 = 0.f;
  int fd0 = 0, fd1 = 0, fp0 = 0, fp1 = 0;
  uint64_t fq0 = 0, fq1 = 0;
  if (lane == 0) { fs0 = lp_s[0]; fd0 = 1; }      // first candidate of the first level, under the root
  int count = 1;
  for (int v = 1; v < T; ++v) {
    const bool second = fd1 != 0 && (fd0 == 0 || fs1 > fs0 || (fs1 == fs0 && tie_first(fd1, fq1, fd0, fq0)));
    const float s = second ? fs1 : fs0;
    const int d = second ? fd1 : fd0;
    const uint64_t q = second ? fq1 : fq0;
    const int par_l = second ? fp1 : fp0;
    const float best = wave_max_dpp(d ? s : -INFINITY);
    const bool top = d != 0 && s == best;
    uint64_t tied = __ballot(top);
    if (tied == 0) break;                          // frontier exhausted: uniform
    if (tied & (tied - 1)) {                       // several lanes hold the best score: depth, then path decide
      uint64_t key = top ? ((uint64_t)d << 48 | q) : ~0ull;
      uint64_t low = key;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const uint64_t other = __shfl_xor((unsigned long long)low, o, 64);
        low = other < low ? other : low;
      }
      tied = __ballot(key == low);
    }
    const int win = __builtin_amdgcn_readfirstlane(__builtin_ctzll(tied));
    const int depth = __builtin_amdgcn_readlane(d, win);
    const int par = __builtin_amdgcn_readlane(par_l, win);
    const float score = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), win));
    const uint64_t path = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(q >> 32), win) << 32 |
                          (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)q, win);
    const int r = (int)(path & 63);
    if (lane == 0) { n_parent[v] = par; n_depth[v] = depth; n_rank[v] = r; }
    if (lane == win) {                             // the next sibling takes the slot over
      const bool more = r + 1 < b;
      const float sib = more ? lp_s[(depth - 1) * kMaxTopK + r + 1] : 0.f;
      if (second) { fs1 = fb1 + sib; fq1 += 1; fd1 = more ? fd1 : 0; }
      else { fs0 = fb0 + sib; fq0 += 1; fd0 = more ? fd0 : 0; }
    }
    if (depth < k) {                               // the first child goes to a new slot
      if (lane == (count & 63)) {
        const float cs = score + lp_s[depth * kMaxTopK];
        if (count >> 6) { fs1 = cs; fb1 = score; fd1 = depth + 1; fp1 = v; fq1 = path << 6; }
        else { fs0 = cs; fb0 = score; fd0 = depth + 1; fp0 = v; fq0 = path << 6; }
      }
      ++count;
    }
  }
  __syncthreads();
  for (int v = lane; v < T; v += 64) {
    const int depth = n_depth[v], r = n_rank[v];
    tree.parent[v] = n_parent[v];
    tree.depth[v] = depth;
    tree.rank[v] = r;
    tok[v] = v ? cand_s[(depth - 1) * kMaxTopK + r] : *root;
    uint64_t mask[kMaskWords];
    for (int w = 0; w < kMaskWords; ++w) mask[w] = 0;
    for (int u = v, hop = 0; u >= 0 && hop <= kMaxTransfer; u = n_parent[u], ++hop)
      for (int w = 0; w < kMaskWords; ++w) mask[w] |= w == (u >> 6) ? 1ull << (u & 63) : 0ull;
    for (int w = 0; w < kMaskWords; ++w) tree.anc[(size_t)v * kMaskWords + w] = mask[w];
  }
}
hipError_t launch_tree_dynamic(const int32_t* root, const int32_t* cand, const float* lp, int k, int b, int T,
                               TreeOut tree, int32_t* tok, hipStream_t s) {
  hipLaunchKernelGGL(tree_dynamic_kernel, dim3(1), dim3(64), 0, s, root, cand, lp, k, b, T, tree, tok);
  return hipGetLastError();
}

// ---- distillation term of the training stage (Sec. 3.3)
// kl[p] = KL(softmax(z[row_a + p]) || softmax(z[row_b + p])) = sum_v A_v (log A_v - log B_v) for pairs p of logit
// rows.  One block of 1024 threads per pair: the two maxima, then the two sums of exponentials and the A-weighted sum
// of the shifted logit differences in one more pass.
__global__ __launch_bounds__(1024) void kl_rows_kernel(const float* __restrict__ z, int row_a, int row_b, int V, int vec,
                                                       float* __restrict__ kl) {
  __shared__ float red[16];
  const float* za = z + (size_t)(row_a + blockIdx.x) * V;
  const float* zb = z + (size_t)(row_b + blockIdx.x) * V;
  const int v4 = vec ? (V & ~3) : 0;
  float ma = -INFINITY, mb = -INFINITY;
  for (int j = threadIdx.x * 4; j < v4; j += blockDim.x * 4) {
    const float4 a = *(const float4*)(za + j), b = *(const float4*)(zb + j);
    ma = fmaxf(fmaxf(ma, fmaxf(a.x, a.y)), fmaxf(a.z, a.w));
    mb = fmaxf(fmaxf(mb, fmaxf(b.x, b.y)), fmaxf(b.z, b.w));
  }
  for (int j = v4 + threadIdx.x; j < V; j += blockDim.x) { ma = fmaxf(ma, za[j]); mb = fmaxf(mb, zb[j]); }
  auto block_max = [&](float v) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = red[0];
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) t = fmaxf(t, red[w]);
    return t;
  };
  ma = block_max(ma);
  mb = block_max(mb);
  float sa = 0.f, sb = 0.f, cross = 0.f;
  auto term = [&](float a, float b) {
    const float ea = expf(a - ma);
    sa += ea;
    sb += expf(b - mb);
    cross += ea * ((a - ma) - (b - mb));
  };
  for (int j = threadIdx.x * 4; j < v4; j += blockDim.x * 4) {
    const float4 a = *(const float4*)(za + j), b = *(const float4*)(zb + j);
    term(a.x, b.x); term(a.y, b.y); term(a.z, b.z); term(a.w, b.w);
  }
  for (int j = v4 + threadIdx.x; j < V; j += blockDim.x) term(za[j], zb[j]);
  sa = block_sum_any(sa, red);
  sb = block_sum_any(sb, red);
  cross = block_sum_any(cross, red);
  if (threadIdx.x == 0) kl[blockIdx.x] = cross / sa - logf(sa) + logf(sb);
}
hipError_t launch_kl_rows(const float* z, int row_a, int row_b, int pairs, int V, float* kl, hipStream_t s) {
  const int vec = !((uintptr_t)z & 15) && !(V & 3);
  hipLaunchKernelGGL(kl_rows_kernel, dim3(pairs), dim3(1024), 0, s, z, row_a, row_b, V, vec, kl);
  return hipGetLastError();
}

// One wavefront: each round, every lane tests a slice of the nodes for "child of cur carrying the
// greedy token after cur" and the lowest such node index wins.
__global__ void accept_kernel(StepState* __restrict__ st, TreeDev tree, const int32_t* __restrict__ tok,
                              const int32_t* __restrict__ g, int T, StepLog* __restrict__ log) {
  const int lane = threadIdx.x;
  int cur = 0, m = 1;
  if (lane == 0) { st->path[0] = 0; st->emitted[0] = tok[0]; }
  while (m < kMaxTransfer + 1) {
    const int want = g[cur];
    int best = 0x7fffffff;
    for (int c = cur + 1 + lane; c < T; c += 64)
      if (tree.parent[c] == cur && tok[c] == want) { best = c; break; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o, 64));
    if (best == 0x7fffffff) break;
    if (lane == 0) { st->path[m] = best; st->emitted[m] = tok[best]; }
    cur = best;
    ++m;
  }
  if (lane == 0) {
    st->m = m;
    st->next_root = g[cur];
    st->root = g[cur];
    if (log) {                       // device-resident loop: the host reads the steps and the cache length afterwards
      StepLog* e = log + st->log_count;
      e->m = m;
      for (int j = 0; j < m; ++j) e->emitted[j] = st->emitted[j];
      st->log_count += 1;
      st->n_old = st->n;
      st->n += m;
    }
  }
}
hipError_t launch_accept(StepState* st, TreeDev tree, const int32_t* tok, const int32_t* g, int T, hipStream_t s,
                         StepLog* log) {
  hipLaunchKernelGGL(accept_kernel, dim3(1), dim3(64), 0, s, st, tree, tok, g, T, log);
  return hipGetLastError();
}

// Moves the accepted rows to slots n..n+m-1 (ascending j; path[j] >= j so in place is safe) and makes
// the last accepted node's saved residual the next transfer source.  blockIdx.y = layer.
template <typename T>
__global__ void compact_kernel(const StepState* __restrict__ st, void* const* __restrict__ kcs,
                               void* const* __restrict__ vcs, int n, int row_elems, int cap,
                               const float* __restrict__ saved_h, size_t slot_stride, int slots,
                               float* __restrict__ h_src, int d, int n_from_state) {
  const int layer = blockIdx.y;
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = st->m;
  if (n_from_state) n = st->n_old;      // device-resident loop: the cache length before this acceptance
  if (e < row_elems) {
    T* kc = (T*)kcs[layer];
    T* vc = (T*)vcs[layer];
    for (int j = 0; j < m; ++j) {
      const int src = st->path[j];
      if (src == j) continue;
      kc[(size_t)(n + j) * row_elems + e] = kc[(size_t)(n + src) * row_elems + e];
      vc[(size_t)e * cap + n + j] = vc[(size_t)e * cap + n + src];
    }
  }
  if (layer < slots && e < d)       // one transfer source per distinct transfer layer (slots <= layers)
    h_src[(size_t)layer * d + e] = saved_h[layer * slot_stride + (size_t)st->path[m - 1] * d + e];
}
hipError_t launch_compact(int dtype, const StepState* st, void* const* kc, void* const* vc, int L, int n, int Hkv,
                          int hd, int cap, const float* saved_h, size_t slot_stride, int slots, float* h_src, int d,
                          hipStream_t s, bool n_from_state) {
  const int row = Hkv * hd;
  const int cols = row > d ? row : d;
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(compact_kernel<T>, dim3((cols + 255) / 256, L), dim3(256), 0, s, st, kc,
                                              vc, n, row, cap, saved_h, slot_stride, slots, h_src, d,
                                              n_from_state ? 1 : 0);)
  return hipGetLastError();
}

// saved_h holds one [rows, d] residual image per distinct transfer layer (`slot_stride` floats apart); the
// transfer sources h_src[slot][d] become the images' row `last`.  blockIdx.y = slot.
__global__ void prefill_finish_kernel(StepState* __restrict__ st, const int32_t* __restrict__ g,
                                      const float* __restrict__ saved_h, size_t slot_stride, float* __restrict__ h_src,
                                      int last, int d) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x, slot = blockIdx.y;
  if (e < d) h_src[(size_t)slot * d + e] = saved_h[slot * slot_stride + (size_t)last * d + e];
  if (e == 0 && slot == 0) { st->root = g[last]; st->next_root = g[last]; st->m = 0; }
}
hipError_t launch_prefill_finish(StepState* st, const int32_t* g, const float* saved_h, size_t slot_stride, int slots,
                                 float* h_src, int last, int d, hipStream_t s) {
  hipLaunchKernelGGL(prefill_finish_kernel, dim3((d + 255) / 256, slots), dim3(256), 0, s, st, g, saved_h, slot_stride,
                     h_src, last, d);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ hidden transfer
// pseudo[f][i][o] = sum_c W_i[o][c] h_f[c] for F source vectors h_f = h + row(f) * d, row(f) = src_rows[f] (or f
// when src_rows is NULL).  With several sources a wavefront produces four consecutive output features: the four
// weight rows are read fully coalesced (16 bytes per lane and row) and every 16-byte piece of a source, which
// comes from L2, serves all four (one feature per wavefront re-read the sources for every weight row: nine bytes
// of source per weight byte with four sources, 51 us against 28 us at d = 4096).  Sources go in groups of four (of
// sixteen from sixteen sources on, which walks the weight rows a quarter as often);
// one source alone has its own instance with one feature per wavefront.  Every (source,
// output) sum runs in the same order whatever F is, so one source alone and the same source among several give
// the same bits.
// Steps i0 .. i0 + gridDim.y - 1 are computed; the output row of (f, i) is f * row_stride + (i - i0).
// grid = (ceil(d / (4 R)), steps), block = 256.
template <typename T, int NF, int R>           // R output features per wavefront: a source piece is loaded once for all
__global__ void transfer_kernel(const float* __restrict__ h, const int32_t* __restrict__ src_rows, int F,
                                const void* const* __restrict__ ws, float* __restrict__ pseudo, int i0, int row_stride,
                                int d) {
  const int i = i0 + blockIdx.y;
  const int o0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * R;
  const int lane = threadIdx.x & 63;
  if (o0 >= d) return;
  const T* rows[R];
#pragma unroll
  for (int r = 0; r < R; ++r) rows[r] = (const T*)ws[i] + (size_t)(o0 + r < d ? o0 + r : d - 1) * d;
  constexpr int VEC = 16 / sizeof(T);
  for (int f0 = 0; f0 < F; f0 += NF) {
    const float* hp[NF];
#pragma unroll
    for (int j = 0; j < NF; ++j) {
      const int f = f0 + j < F ? f0 + j : F - 1;
      hp[j] = h + (size_t)(src_rows ? src_rows[f] : f) * d;
    }
    float acc[R][NF];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < NF; ++j) acc[r][j] = 0.f;
    for (int c = lane * VEC; c < d; c += 64 * VEC) {
      if (c + VEC <= d) {
        uint4 raw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) raw[r] = *(const uint4*)(rows[r] + c);
#pragma unroll
        for (int j = 0; j < NF; ++j) {
          float hv[VEC];
#pragma unroll
          for (int e = 0; e < VEC; e += 4) *(float4*)(hv + e) = *(const float4*)(hp[j] + c + e);
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const T* v = (const T*)&raw[r];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[r][j] += Conv<T>::load(v + e) * hv[e];
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int j = 0; j < NF; ++j)
            for (int e = 0; c + e < d; ++e) acc[r][j] += Conv<T>::load(rows[r] + c + e) * hp[j][c + e];
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < NF; ++j) {
        const float v = wave_sum(acc[r][j]);
        if (lane == 0 && f0 + j < F && o0 + r < d)
          pseudo[((size_t)(f0 + j) * row_stride + (i - i0)) * d + o0 + r] = v;
      }
  }
}
hipError_t launch_transfer(int dtype, const float* h, const int32_t* src_rows, int F, const void* const* w_dev,
                           float* pseudo, int i0, int steps, int row_stride, int d, hipStream_t s) {
  if (d % 4) return hipErrorInvalidValue;      // 16-byte pieces of the fp32 sources
  if (F == 1) {      // one source: its re-reads are cheap and one feature per wavefront spreads the rows wider
    HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((transfer_kernel<T, 1, 1>), dim3((d + 3) / 4, steps), dim3(256), 0, s, h,
                                                src_rows, F, w_dev, pseudo, i0, row_stride, d);)
  } else if (F < 16) {
    HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((transfer_kernel<T, 4, 4>), dim3((d + 15) / 16, steps), dim3(256), 0, s, h,
                                                src_rows, F, w_dev, pseudo, i0, row_stride, d);)
  } else {           // every node of a tree drafts: sixteen sources per walk over the weight rows (same sums, same order)
    HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL((transfer_kernel<T, 16, 4>), dim3((d + 15) / 16, steps), dim3(256), 0, s, h,
                                                src_rows, F, w_dev, pseudo, i0, row_stride, d);)
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ streaming probe
// Reads a buffer once the way the packed projections read their weights (every workgroup walks its own
// contiguous region, 8 KiB per step as eight nontemporal 1 KiB wavefront loads, eight steps in flight) and does
// nothing with the data: the time of this kernel is the floor for any weight stream of that size.
typedef unsigned int probe_u32x4_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const probe_u32x4_t* __restrict__ p, size_t vecs_per_group,
                                                          uint32_t* __restrict__ sink) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const probe_u32x4_t* base = p + (size_t)blockIdx.x * vecs_per_group + wave * 128 + lane;
  const size_t steps = vecs_per_group / 512;              // 512 vectors = 8 KiB per step
  probe_u32x4_t acc = {0, 0, 0, 0};
  for (size_t i = 0; i + 4 <= steps; i += 4) {
    probe_u32x4_t v[8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      v[2 * u] = __builtin_nontemporal_load(base + (i + u) * 512);
      v[2 * u + 1] = __builtin_nontemporal_load(base + (i + u) * 512 + 64);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;     // keeps the loads alive
}
// Reads floor(bytes / (groups * 32 KiB)) * groups * 32 KiB bytes; returns that count.
size_t launch_stream_read(const void* buf, size_t bytes, int groups, uint32_t* sink, hipStream_t s) {
  const size_t per_group = bytes / groups / 32768 * 32768;
  if (!per_group) return 0;
  hipLaunchKernelGGL(stream_read_kernel, dim3(groups), dim3(256), 0, s, (const probe_u32x4_t*)buf, per_group / 16, sink);
  return per_group * groups;
}

// ------------------------------------------------------------------------------------------------ matrix-core probe
// Nothing but independent matrix-core instructions on register operands, 32 accumulators of 16 x 16 (FORM 0:
// v_mfma_f32_16x16x32_bf16) or 8 of 32 x 32 (FORM 1: v_mfma_f32_32x32x16_bf16) per wavefront, two wavefronts per
// SIMD: the rate of this kernel is what a product kernel on that instruction can reach at best on this machine.
// The rate depends on the operand bits (the clock follows the power drawn), hence two kinds of operands.
typedef __bf16 probe_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float probe_f32x4_t __attribute__((ext_vector_type(4)));
typedef float probe_f32x16_t __attribute__((ext_vector_type(16)));
template <int FORM>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, int random_bits, uint32_t* __restrict__ sink) {
  // operands: small whole numbers (few bits toggle between lanes and instructions), or values in +-[1, 2) with
  // hashed sign and mantissa bits (what real activations and weights look like to the multipliers)
  probe_bf16x8_t a[4], b[8];
  auto fill = [&](int which, int j) -> __bf16 {
    if (!random_bits) return (__bf16)(float)((threadIdx.x * (which < 4 ? 1 : 3) + which + j) & 7);
    uint32_t h = (threadIdx.x * 64u + which * 8u + j) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    const unsigned short bits = (unsigned short)(0x3f80u | (h & 0x7fu) | ((h & 0x100u) << 7));
    return __builtin_bit_cast(__bf16, bits);
  };
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) a[i][j] = fill(i, j);
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) b[i][j] = fill(4 + i, j);
  float total = 0.f;
  if (FORM == 0) {
    probe_f32x4_t acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = probe_f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i % 4], b[i / 4], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) total += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  } else {
    probe_f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i % 2], b[i / 2], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) total += acc[i][j];
  }
  if (total == -1.25f) sink[0] = 1;                        // keeps the work alive (sums of whole numbers, or far from -1.25)
}
// Returns the floating-point operations of the launch (2 per multiply-add).
double launch_mfma_rate(int form, int iters, uint32_t* sink, hipStream_t s) {
  constexpr int kGroups = 512;                             // two workgroups of four wavefronts per compute unit
  if ((form & 1) == 0)
    hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(kGroups), dim3(256), 0, s, iters, form >> 1, sink);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(kGroups), dim3(256), 0, s, iters, form >> 1, sink);
  return (double)kGroups * 4 * iters * ((form & 1) == 0 ? 32 * 2.0 * 16 * 16 * 32 : 8 * 2.0 * 32 * 32 * 16);
}

// ------------------------------------------------------------------------------------------------ generic product
// out[m][n] = sum_k a[m][k] w[n][k], fp32 accumulation.  One wavefront per output feature n, rows in
// groups of 4.  Used by the fp32 model path and as the fallback for shapes the MFMA kernel rejects.
template <typename T>
__global__ void gemm_simple_kernel(const T* __restrict__ a, WeightSegs w, int M, int N, int K, float* __restrict__ out) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (n >= N) return;
  int seg = 0, local = n;
  while (seg + 1 < w.nseg && local >= w.rows[seg]) { local -= w.rows[seg]; ++seg; }
  const T* row = (const T*)w.w[seg] + (size_t)local * K;
  for (int m0 = 0; m0 < M; m0 += 4) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = lane; c < K; c += 64) {
      const float wv = Conv<T>::load(row + c);
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (m0 + r < M) acc[r] += wv * Conv<T>::load(a + (size_t)(m0 + r) * K + c);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = wave_sum(acc[r]);
      if (lane == 0 && m0 + r < M) out[(size_t)(m0 + r) * N + n] = v;
    }
  }
}
hipError_t launch_gemm_simple(int dtype, const void* a, WeightSegs w, int M, int N, int K, float* out, hipStream_t s) {
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(gemm_simple_kernel<T>, dim3((N + 3) / 4), dim3(256), 0, s, (const T*)a,
                                              w, M, N, K, out);)
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ generic attention
// One block per (query head, tree row).  Scores of all visible keys go to LDS, softmax in fp32, then
// every thread owns one (output element, key residue class).  Dynamic LDS: (n + M) floats + hd + 256.
template <typename T>
__global__ void attn_simple_kernel(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc, int cap,
                                   int n, int M, TreeDev tree, int Hq, int Hkv, int hd, T* __restrict__ out,
                                   const int32_t* __restrict__ n_dev) {
  extern __shared__ float smem[];
  __shared__ float red[4];
  n = cache_len(n, n_dev);             // at most the host's n, which sized the dynamic LDS
  const int h = blockIdx.x, m = blockIdx.y, hk = h / (Hq / Hkv), tid = threadIdx.x;
  const int S = n + M;
  float* sc = smem;            // [S]
  float* qs = smem + S;        // [hd]
  float* acc = qs + hd;        // [256]
  for (int e = tid; e < hd; e += 256) qs[e] = Conv<T>::load(q + ((size_t)m * Hq + h) * hd + e);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)hd);
  float mx = -INFINITY;
  for (int j = tid; j < S; j += 256) {
    bool vis = j < n;
    if (!vis) {
      const int u = j - n;
      vis = (tree.anc[(size_t)m * kMaskWords + (u >> 6)] >> (u & 63)) & 1ull;
    }
    float s = -INFINITY;
    if (vis) {
      const T* kr = kc + ((size_t)j * Hkv + hk) * hd;
      float dot = 0.f;
      for (int e = 0; e < hd; ++e) dot += qs[e] * Conv<T>::load(kr + e);
      s = dot * scale;
    }
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = block_max_256(mx, red);
  float sum = 0.f;
  for (int j = tid; j < S; j += 256) {
    const float p = sc[j] == -INFINITY ? 0.f : expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = block_sum_256(sum, red);
  const int groups = 256 / hd > 0 ? 256 / hd : 1;      // hd <= 256
  const int e = tid % hd, part = tid / hd;
  float o = 0.f;
  if (part < groups) {
    const T* vr = vc + ((size_t)hk * hd + e) * cap;
    for (int j = part; j < S; j += groups)
      if (sc[j] != 0.f) o += sc[j] * Conv<T>::load(vr + j);
  }
  acc[tid] = o;
  __syncthreads();
  if (tid < hd) {
    float t = 0.f;
    for (int p = 0; p < groups; ++p) t += acc[p * hd + tid];
    Conv<T>::store(out + (size_t)m * Hq * hd + (size_t)h * hd + tid, t / sum);
  }
}
hipError_t launch_attn_simple(int dtype, const void* q, const void* kc, const void* vc, int cap, int n, int M,
                              TreeDev tree, int Hq, int Hkv, int hd, void* out, hipStream_t s, const int32_t* n_dev) {
  const size_t smem = (size_t)(n + M + hd + 256) * sizeof(float);
  if (smem > 64 * 1024 || hd > 256) return hipErrorInvalidValue;
  HT_DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(attn_simple_kernel<T>, dim3(Hq, M), dim3(256), smem, s, (const T*)q,
                                              (const T*)kc, (const T*)vc, cap, n, M, tree, Hq, Hkv, hd, (T*)out, n_dev);)
  return hipGetLastError();
}

}  // namespace ht
