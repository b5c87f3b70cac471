// Skinny weight-streaming product for bf16 on CDNA4 matrix cores.
//
//   out[s][m][n] = sum_{k in split s} a[m][k] * w[n][k]        m < M <= 128, fp32 accumulate
//
// The weights are the big operand (N x K, streamed from HBM exactly once); the activations are a
// small panel (M x K) that every workgroup re-reads from L2.  Mapping on v_mfma_f32_16x16x32_bf16:
// weight rows are the MFMA "A" rows (16 output features per instruction), tokens are the "B"
// columns, so each lane ends with four consecutive output features of one token.
//
//   * A wavefront owns R blocks of 16 weight rows and streams them straight from global memory
//     into MFMA operand registers: per 64-wide K chunk a lane reads 32 contiguous bytes of its row,
//     four lanes cover a full 128-byte line, and a ring of PD chunks stays in flight per wavefront.
//     The contraction index inside a chunk is permuted the same way for both operands (lane group
//     g, step s  <->  k = 16 g + 8 s .. + 7), which is what makes those reads contiguous.
//   * The activation panel for the chunk is staged once per workgroup in LDS (rows padded to 144
//     bytes so 128-bit reads are bank-conflict free) and shared by the four wavefronts.
//   * Optional split-K over blockIdx.y writes partial sums that the consumer adds in a fixed order.
#include "ht_common.h"

namespace ht {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int KC = 64;                 // K elements per chunk
constexpr int ROWB = KC * 2 + 16;      // LDS row stride in bytes
constexpr int PD = 4;                  // weight chunks in flight per wavefront

union Frag {
  uint4 raw;
  bf16x8_t v;
};

template <int MT, int R>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const bf16_t* __restrict__ a, WeightSegs w, int M, int N, int K,
                                                        float* __restrict__ out, int nsplit) {
  constexpr int ROWS = MT * 16;
  constexpr int PIECES = ROWS * 8;                       // 16-byte pieces of the activation chunk
  constexpr int APASS = (PIECES + 255) / 256;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][ROWS * ROWB];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, g = lane >> 4;
  const int chunks = (K + KC - 1) / KC;
  const int c0 = (int)((long long)chunks * blockIdx.y / nsplit);
  const int c1 = (int)((long long)chunks * (blockIdx.y + 1) / nsplit);

  // weight rows of this wavefront
  const bf16_t* wrow[R];
  bool wvalid[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int rb = (blockIdx.x * 4 + wave) * R + r;
    int row = rb * 16 + r16;
    wvalid[r] = rb * 16 < N;
    int seg = 0;
    if (wvalid[r]) {
      while (seg + 1 < w.nseg && row >= w.rows[seg]) { row -= w.rows[seg]; ++seg; }
    } else {
      row = 0;
    }
    wrow[r] = (const bf16_t*)w.w[seg] + (size_t)row * K + g * 16;
  }

  auto load_w = [&](Frag (&dst)[R][2], int c) {
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const int k = c * KC + g * 16 + s * 8;
        if (wvalid[r] && k < K) dst[r][s].raw = *(const uint4*)(wrow[r] + c * KC + s * 8);
        else dst[r][s].raw = make_uint4(0, 0, 0, 0);
      }
  };
  auto load_a = [&](uint4 (&dst)[APASS], int c) {
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
      const int p = tid + i * 256;
      const int row = p >> 3, col = p & 7;
      const int k = c * KC + col * 8;
      if (p < PIECES && k < K) dst[i] = *(const uint4*)(a + (size_t)row * K + k);
      else dst[i] = make_uint4(0, 0, 0, 0);
    }
  };
  auto store_a = [&](const uint4 (&src)[APASS], int stage) {
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
      const int p = tid + i * 256;
      if (p < PIECES) *(uint4*)(&lds[stage][(p >> 3) * ROWB + (p & 7) * 16]) = src[i];
    }
  };

  floatx4_t acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[r][mt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  Frag wreg[PD][R][2];
  uint4 areg[APASS];
#pragma unroll
  for (int p = 0; p < PD; ++p)
    if (c0 + p < c1) load_w(wreg[p], c0 + p);
  if (c0 < c1) {
    load_a(areg, c0);
    store_a(areg, 0);
  }
  if (c0 + 1 < c1) load_a(areg, c0 + 1);
  __syncthreads();

  for (int cb = c0; cb < c1; cb += PD) {
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      const int c = cb + p;
      if (c < c1) {
        const int stage = p & 1;
        if (c + 1 < c1) store_a(areg, stage ^ 1);
        if (c + 2 < c1) load_a(areg, c + 2);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          Frag b[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            b[mt].raw = *(const uint4*)(&lds[stage][(mt * 16 + r16) * ROWB + g * 32 + s * 16]);
#pragma unroll
          for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[p][r][s].v, b[mt].v, acc[r][mt], 0, 0, 0);
        }
        if (c + PD < c1) load_w(wreg[p], c + PD);
        __syncthreads();
      }
    }
  }

  float* dst = out + (size_t)blockIdx.y * M * N;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int rb = (blockIdx.x * 4 + wave) * R + r;
    if (rb * 16 >= N) continue;
    const int n0 = rb * 16 + g * 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mt * 16 + r16;
      if (m < M) *(float4*)(dst + (size_t)m * N + n0) = make_float4(acc[r][mt][0], acc[r][mt][1], acc[r][mt][2], acc[r][mt][3]);
    }
  }
}

template <int MT>
hipError_t launch_mt(const bf16_t* a, const WeightSegs& w, int M, int N, int K, float* out, int nsplit, hipStream_t s) {
  const int rbs = N / 16;
  if (N >= 8192) {
    hipLaunchKernelGGL((gemm_mfma_kernel<MT, 2>), dim3((rbs + 7) / 8, nsplit), dim3(256), 0, s, a, w, M, N, K, out, nsplit);
  } else {
    hipLaunchKernelGGL((gemm_mfma_kernel<MT, 1>), dim3((rbs + 3) / 4, nsplit), dim3(256), 0, s, a, w, M, N, K, out, nsplit);
  }
  return hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(int M, int N, int K) { return M >= 1 && M <= 128 && N % 16 == 0 && K % 8 == 0 && N >= 16; }

int gemm_mfma_splits(int M, int N, int K) {
  (void)M;
  const int per_wg = N >= 8192 ? 128 : 64;
  const int tiles = (N + per_wg - 1) / per_wg;
  int s = 512 / tiles;
  const int chunks = (K + KC - 1) / KC;
  if (s > chunks / 4) s = chunks / 4;        // at least four chunks per split
  if (s > kMaxSplitK) s = kMaxSplitK;
  if (s < 1) s = 1;
  return s;
}

hipError_t launch_gemm_mfma(const void* a, WeightSegs w, int M, int N, int K, float* out, int nsplit, hipStream_t s) {
  const bf16_t* ap = (const bf16_t*)a;
  if (M <= 16) return launch_mt<1>(ap, w, M, N, K, out, nsplit, s);
  if (M <= 32) return launch_mt<2>(ap, w, M, N, K, out, nsplit, s);
  if (M <= 64) return launch_mt<4>(ap, w, M, N, K, out, nsplit, s);
  return launch_mt<8>(ap, w, M, N, K, out, nsplit, s);
}

}  // namespace ht
