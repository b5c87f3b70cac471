// Skinny weight-streaming product for bf16 on CDNA4 matrix cores.
//
//   out[m][n] = sum_k a[m][k] * w[n][k]        m < M <= 128 tokens, fp32 accumulate
//
// The weights are the big operand (N x K, read from HBM exactly once per pass); the activations are
// a small panel (M x K) that every workgroup re-reads from L2.  On v_mfma_f32_16x16x32_bf16 the weight
// rows are the MFMA "A" rows (16 output features per instruction) and the tokens are the "B" columns,
// so each lane ends with four consecutive output features of one token.
//
// Weight layout.  At model init every projection matrix is repacked once into MFMA-fragment order:
// fragment (rb, j) holds rows 16 rb .. 16 rb + 15 and columns 32 j .. 32 j + 31 as 64 lanes x 16 bytes
// (lane l: row l % 16, columns 8 (l / 16) .. + 7).  Eight row blocks form a tile; inside a tile the
// fragments are ordered K-step major (step j of row blocks 0..7, then step j+1, ..), so the workgroup that
// owns a tile reads one sequential stream of 8 KiB per K step while each wavefront load is still a fully
// coalesced 1 KiB that drops straight into MFMA operand registers: no LDS transpose, no partially used
// cache lines, sequential DRAM pages, and no two workgroups marching through memory at the same
// power-of-two stride (row-block-major order measured up to 15 % slower on a pure streaming test).  Row blocks can be ordered freely at pack time,
// and rows inside a block too: that is how gate and up rows meet in one wavefront for the fused SiLU epilogue and
// how a q or k feature meets its rotary partner inside one row block.
//
// The activation chunk (M x 64 columns) is staged once per workgroup in LDS (rows padded by 32 bytes:
// conflict-free 128-bit reads) and shared by the four wavefronts; a ring of PD weight chunks per
// wavefront stays in flight.  Split-K over blockIdx.y writes fp32 partial sums that the consumer adds
// in a fixed order (deterministic).
#include "ht_common.h"

namespace ht {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int kChunkCols = 64;         // K elements per activation chunk (128 for the 16-row instance)
constexpr int kRingDepth = 3;          // weight chunks in flight per wavefront
constexpr int kPadCols = 128;          // packed weights are zero-padded along K to a multiple of this
constexpr int kTileBlocks = 8;         // row blocks interleaved per K step in the packed layout
constexpr int kRowPad = 32;            // bytes added to every activation row in LDS, see gemm_packed_kernel

union Frag {
  uint4 raw;
  u32x4_t nat;
  bf16x8_t v;
};

enum { EPI_F32 = 0, EPI_SILU = 1, EPI_QKV = 2 };

// --------------------------------------------------------------------------------------------- repack
// dst fragment order from row-major segments.  One thread per 16-byte piece.
__global__ void repack_kernel(WeightSegs w, int K, int KS, int n_rb, int mode, int head_blocks,
                              bf16_t* __restrict__ dst) {
  const size_t piece = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int n_tiles = (n_rb + kTileBlocks - 1) / kTileBlocks;
  const size_t total = (size_t)n_tiles * KS * kTileBlocks * 64;
  if (piece >= total) return;
  const int lane = (int)(piece & 63);
  const size_t frag = piece >> 6;
  const int rbt = (int)(frag % kTileBlocks);
  const int j = (int)((frag / kTileBlocks) % KS);
  const int tile = (int)(frag / ((size_t)kTileBlocks * KS));
  const int rb = tile * kTileBlocks + rbt;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (rb < n_rb) {
    int grow = rb * 16 + (lane & 15);       // source row in the concatenated segments
    if (mode == 1) {               // two equal segments interleaved block by block (gate, up)
      grow = (rb & 1) * w.rows[0] + (rb >> 1) * 16 + (lane & 15);
    } else if (mode == 2) {        // q | k | v: block b of a q or k head holds features 8b .. 8b+7 (rows 0..7) and
      const int hb = head_blocks;  // their rotary partners hd/2 + 8b .. (rows 8..15); v heads keep their order
      const int qk_rbs = (w.rows[0] + w.rows[1]) / 16;
      if (rb < qk_rbs) {
        const int in_head = rb % hb, r = lane & 15;
        grow = (rb - in_head) * 16 + (r < 8 ? 8 * in_head + r : 8 * hb + 8 * in_head + r - 8);
      }
    }
    int seg = 0;
    while (seg + 1 < w.nseg && grow >= w.rows[seg]) { grow -= w.rows[seg]; ++seg; }
    const int row = grow;
    const int k = j * 32 + (lane >> 4) * 8;
    if (k < K) v = *(const uint4*)((const bf16_t*)w.w[seg] + (size_t)row * K + k);
  }
  *(uint4*)(dst + piece * 8) = v;
}

// --------------------------------------------------------------------------------------------- epilogues
// What a wavefront does with its finished sums acc[r][mt] (row block rb0 + r, token tile mt): the 1/rms factor of
// the token rows, then fp32 partial sums, SiLU(gate) * up, or rotary + q store / K,V append.
template <int MT, int R, int EPI>
__device__ __forceinline__ void finish_rows(floatx4_t (&acc)[R][MT], const float4 (&row_ss)[MT], int rb0, int wg1, int M,
                                            int N, void* __restrict__ outp, const QkvEpilogue& qe, const RowScale& rs,
                                            int row0, int split) {
  const int lane = threadIdx.x & 63, g = lane >> 4;
  const int r16 = row0 + (lane & 15);                    // token row of tile mt: mt * 16 + r16, counted over the whole pass
  if (rs.ss) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const float4 q4 = row_ss[mt];
      const float sc = __builtin_amdgcn_rsqf((q4.x + q4.y + q4.z + q4.w) * rs.inv_d + rs.eps);   // 1 ulp
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r][mt] *= sc;
    }
  }
  if (EPI == EPI_F32) {
    float* dst = (float*)outp + (size_t)split * M * N;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (rb0 + r >= wg1) continue;
      const int n0 = (rb0 + r) * 16 + g * 4;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r16;
        if (m < M)
          *(float4*)(dst + (size_t)m * N + n0) = make_float4(acc[r][mt][0], acc[r][mt][1], acc[r][mt][2], acc[r][mt][3]);
      }
    }
  } else if (EPI == EPI_SILU) {
    // row blocks come in pairs: block rb0 + 2 p holds gate rows, rb0 + 2 p + 1 the matching up rows: act = silu(gate) * up
    bf16_t* dst = (bf16_t*)outp;
    const int f = N / 2;
#pragma unroll
    for (int pr = 0; pr < R / 2; ++pr) {                  // (the launchers give this epilogue an even R)
      if (rb0 + 2 * pr + 1 >= wg1) continue;
      const int j0 = ((rb0 + 2 * pr) / 2) * 16 + g * 4;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r16;
        if (m < M) {
          float o[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float gt = acc[2 * pr][mt][i], up = acc[2 * pr + 1][mt][i];
            o[i] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * up;      // 1 ulp reciprocal, bf16 result
          }
          *(uint2*)(dst + (size_t)m * f + j0) = pack4_bf16(o[0], o[1], o[2], o[3]);
        }
      }
    }
  } else {
    // q | k | v rows.  Block b of a q or k head holds features 8b .. 8b+7 of the head in MFMA rows 0..7 and their
    // rotary partners (feature + hd/2) in rows 8..15, so lanes 0..31 end with the low halves and the lane 32 further
    // on with the partner of the same feature: one exchange, rotate by the row's position, store q or append k to
    // the cache.  v rows are appended to the slot-contiguous value cache.
    const int hd = qe.hd, half = hd / 2, hb = hd / 16, n_now = cache_len(qe.n, qe.n_dev);
    const int q_blocks = qe.Hq * hb, qk_blocks = q_blocks + qe.Hkv * hb;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int rb = rb0 + r;
      if (rb >= wg1) continue;                                  // uniform over the wavefront
      if (rb < qk_blocks) {
        const bool is_q = rb < q_blocks, upper = g >= 2;
        const int hrb = is_q ? rb : rb - q_blocks;
        const int h = hrb / hb, j = (hrb % hb) * 8 + (g & 1) * 4;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int m = mt * 16 + r16;
          float other[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(acc[r][mt][i], 32, 64);
          if (m < M) {
            const float4 c01 = *(const float4*)(qe.cs + ((size_t)m * half + j) * 2);
            const float4 c23 = *(const float4*)(qe.cs + ((size_t)m * half + j) * 2 + 4);
            const float cs_[8] = {c01.x, c01.y, c01.z, c01.w, c23.x, c23.y, c23.z, c23.w};
            float o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float x = upper ? other[i] : acc[r][mt][i], y = upper ? acc[r][mt][i] : other[i];
              const float co = cs_[2 * i], si = cs_[2 * i + 1];
              o[i] = upper ? y * co + x * si : x * co - y * si;
            }
            bf16_t* dst = is_q ? qe.q + ((size_t)m * qe.Hq + h) * hd + j
                               : qe.kc + ((size_t)(n_now + m) * qe.Hkv + h) * hd + j;
            *(uint2*)(dst + (upper ? half : 0)) = pack4_bf16(o[0], o[1], o[2], o[3]);
          }
        }
      } else {
        const int vb = rb - qk_blocks, h = vb / hb, e0 = (vb % hb) * 16 + g * 4;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int m = mt * 16 + r16;
          if (m < M) {
            const uint2 v4 = pack4_bf16(acc[r][mt][0], acc[r][mt][1], acc[r][mt][2], acc[r][mt][3]);
            bf16_t* col = qe.vc + ((size_t)h * hd + e0) * qe.cap + n_now + m;      // feature e0 + i is i * cap further on
            col[0] = (bf16_t)(v4.x & 0xffffu);
            col[(size_t)qe.cap] = (bf16_t)(v4.x >> 16);
            col[2 * (size_t)qe.cap] = (bf16_t)(v4.y & 0xffffu);
            col[3 * (size_t)qe.cap] = (bf16_t)(v4.y >> 16);
          }
        }
      }
    }
  }
}

// --------------------------------------------------------------------------------------------- product
// The hot loop is straight-line code (no predicated loads, no data-dependent branches) so that the
// compiler can keep exact outstanding-load counts and the weight ring really stays in flight: chunk
// indices past the end of this block's K range are clamped to its last chunk (a redundant, in-bounds
// reload that is never used), wavefront slots without a row block re-read one fragment (never stored), and
// activation columns past K are clamped into the row (they meet zero-padded weights).
template <int MT, int R, int WAVES, int EPI, int KC = kChunkCols, int PD = kRingDepth>
__global__ __launch_bounds__(64 * WAVES) void gemm_packed_kernel(const bf16_t* __restrict__ a,
                                                                 const bf16_t* __restrict__ wp, int M, int N, int K,
                                                                 int KS, void* __restrict__ outp, int nsplit,
                                                                 QkvEpilogue qe, RowScale rs, int row0) {
  constexpr int STEPS = KC / 32;                         // MFMA steps per chunk
  // LDS row stride in bytes.  Measured with the bank-conflict counter, a 128-bit operand read of the sixteen rows of
  // a fragment takes 4 cycles with rows padded by 32 bytes, 8 with 16 bytes of padding and 16 with none.
  constexpr int ROWB = KC * 2 + kRowPad;
  constexpr int THREADS = 64 * WAVES;
  constexpr int ROWS = MT * 16;
  constexpr int PIECES = ROWS * (KC / 8);                // 16-byte pieces of the activation chunk
  static_assert(PIECES >= THREADS, "every thread stages at least one piece of the activation chunk");
  constexpr int APASS = (PIECES + THREADS - 1) / THREADS;   // surplus threads of the last pass repeat the last piece
  constexpr int STAGE = ROWS * ROWB;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, g = lane >> 4;
  const int chunks = KS / STEPS;                         // KS is a multiple of STEPS (weights zero-padded)
  int c0, c1;
  even_share(chunks, nsplit, blockIdx.y, c0, c1);
  const int n_rb = N / 16;
  // The grid's workgroups share the row blocks evenly: workgroup b owns n_rb / G blocks, the first n_rb % G
  // workgroups one more (in whole pairs for the SiLU epilogue), at most R * WAVES of them (the launcher's
  // choice of G), R consecutive ones per wavefront.  A slot past the end of
  // the workgroup's range re-reads one fragment of its first block over and over (stride 0: cache hits, no HBM
  // traffic, same instruction stream) and stores nothing.
  constexpr int U = EPI == EPI_SILU ? 2 : 1;             // the SiLU epilogue needs both blocks of a (gate, up) pair
  const int units = (n_rb + U - 1) / U;
  int wg0, wg1;
  even_share(units, gridDim.x, blockIdx.x, wg0, wg1);
  wg0 *= U;
  wg1 *= U;
  const int rb0 = wg0 + wave * R;
  if (c0 >= c1) return;                                  // uniform over the block

  const u32x4_t* wbase[R];
  size_t wstep[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bool own = rb0 + r < wg1;
    const int rb = own ? rb0 + r : wg0;
    wbase[r] = (const u32x4_t*)wp + ((size_t)(rb / kTileBlocks) * KS * kTileBlocks + rb % kTileBlocks) * 64 + lane;
    wstep[r] = own ? (size_t)kTileBlocks * 64 : 0;
  }
  const int last = c1 - 1;
  // All workgroups walk K in the same order on purpose: they then pull the same activation lines from
  // L2 at about the same time, which keeps the small panel resident while the weights stream through
  // (a staggered walk measured 12 % slower).
  auto load_w = [&](Frag (&dst)[R][STEPS], int c) __attribute__((always_inline)) {
    c = c < last ? c : last;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int s = 0; s < STEPS; ++s)
        dst[r][s].nat = __builtin_nontemporal_load(wbase[r] + (size_t)(c * STEPS + s) * wstep[r]);
  };
  // activation pieces of this thread: row p / 16, 16-byte column p % 16 of the chunk
  const bf16_t* arow[APASS];
  int acol[APASS], alds[APASS];
#pragma unroll
  for (int i = 0; i < APASS; ++i) {
    int p = tid + i * THREADS;
    p = p < PIECES ? p : PIECES - 1;
    arow[i] = a + (size_t)(row0 + p / (KC / 8)) * K;
    acol[i] = (p % (KC / 8)) * 8;
    alds[i] = (p / (KC / 8)) * ROWB + (p % (KC / 8)) * 16;
  }
  auto load_a = [&](u32x4_t (&dst)[APASS], int c) __attribute__((always_inline)) {
    c = c < last ? c : last;
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
      int k = c * KC + acol[i];
      k = k < K - 8 ? k : K - 8;
      dst[i] = *(const u32x4_t*)(arow[i] + k);
    }
  };
  auto store_a = [&](const u32x4_t (&src)[APASS], int stage) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < APASS; ++i) *(u32x4_t*)(&lds[stage * STAGE + alds[i]]) = src[i];
  };

  floatx4_t acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[r][mt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // Rows of a panel that was stored without its 1/rms factor: the factor multiplies the finished sums instead
  // (every K split scales its partial sums by the same factor).  The sums of squares are fetched here, ahead of
  // the weight stream (they are the oldest loads, so no wait ever stalls on them), and turned into factors in the
  // epilogue.
  float4 row_ss[MT];
  if (rs.ss) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = row0 + mt * 16 + r16;
      row_ss[mt] = *(const float4*)(rs.ss + (size_t)(m < M ? m : M - 1) * kNormParts);
    }
  }

  // Loads retire in issue order, so everything is issued oldest-needed-first: at chunk c the ring holds
  // weights of chunks c .. c+PD-1 and activations of chunks c+1 .. c+PD; each iteration consumes the
  // oldest of both and issues activation chunk c+PD+1, then weight chunk c+PD.
  Frag wreg[PD][R][STEPS];
  u32x4_t areg[PD][APASS];
  {
    u32x4_t first[APASS];
    load_a(first, c0);
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      load_a(areg[p], c0 + 1 + p);
      load_w(wreg[p], c0 + p);
    }
    store_a(first, 0);
  }
  __syncthreads();

  auto body = [&](Frag (&wslot)[R][STEPS], u32x4_t (&aslot)[APASS], int c) __attribute__((always_inline)) {
    const int stage = (c - c0) & 1;
    const unsigned char* ab = &lds[stage * STAGE + r16 * ROWB + g * 16];
    // activation fragments are read one MFMA step ahead of their use
    Frag b[2][MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) b[0][mt].nat = *(const u32x4_t*)(ab + mt * 16 * ROWB);
    store_a(aslot, stage ^ 1);                 // activation chunk c+1 becomes visible after the barrier below
    load_a(aslot, c + PD + 1);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (s + 1 < STEPS) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b[(s + 1) & 1][mt].nat = *(const u32x4_t*)(ab + mt * 16 * ROWB + (s + 1) * 64);
      }
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wslot[r][s].v, b[s & 1][mt].v, acc[r][mt], 0, 0, 0);
    }
    load_w(wslot, c + PD);
    __syncthreads();
  };

  int c = c0;
  for (; c + PD <= c1; c += PD) {
#pragma unroll
    for (int p = 0; p < PD; ++p) body(wreg[p], areg[p], c + p);
  }
#pragma unroll
  for (int p = 0; p < PD - 1; ++p)
    if (c + p < c1) body(wreg[p], areg[p], c + p);                // uniform tail

  finish_rows<MT, R, EPI>(acc, row_ss, rb0, wg1, M, N, outp, qe, rs, row0, blockIdx.y);
}

// --------------------------------------------------------------------------------------------- product, many rows
// The same product tiled over the tokens as well, for passes of hundreds or thousands of rows (the forward pass of
// the training stage): a workgroup owns 4 R row blocks of the weights (four wavefronts, R each) and MT * 16 token
// rows, walks the whole K range, and the grid covers (row-block tiles) x (token tiles).  At R = 4, MT = 16 a
// workgroup does 256 x 256 outputs per 64 KB it takes in (32 KB of weights, 32 KB of tokens per 64 columns), so the
// matrix cores, not the memory path, set the pace.  Weights come straight into operand registers as before (ring of
// two chunks), the token chunk through registers into padded LDS (two stages, the chunk after next in flight), and
// the token operands are read from LDS four tiles at a time, one group ahead of the matrix cores.
// Workgroups are numbered so that those of one XCD (every eighth) share weight tiles: XCD x takes the row-block
// tiles x, x + 8, .. and runs all token tiles of one before the next, so a weight tile is fetched from HBM by one L2.
template <int MT, int R, int EPI, int AD = 2, int OCC = 1>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OCC, OCC))) void gemm_wide_kernel(const bf16_t* __restrict__ a, const bf16_t* __restrict__ wp, int M, int N,
                                                        int K, int KS, void* __restrict__ outp, QkvEpilogue qe, RowScale rs,
                                                        int n_tiles, int m_tiles) {
  constexpr int KC = 64, STEPS = 2, PD = 2;
  constexpr int ROWB = KC * 2 + kRowPad, ROWS = MT * 16, STAGE = ROWS * ROWB;
  constexpr int APASS = ROWS * (KC / 8) / 256;
  static_assert(ROWS * (KC / 8) % 256 == 0 && MT % 4 == 0, "whole passes of pieces; token tiles in groups of four");
  extern __shared__ __attribute__((aligned(16))) unsigned char wide_lds[];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, g = lane >> 4;
  // workgroup id -> (row-block tile, token tile), see above
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int tx = xcd + 8 * (slot / m_tiles), ty = slot % m_tiles;
  if (tx >= n_tiles) return;                             // uniform over the workgroup
  const int row0 = ty * ROWS;
  const int n_rb = N / 16;
  const int wg0 = tx * 4 * R, wg1 = wg0 + 4 * R < n_rb ? wg0 + 4 * R : n_rb;
  const int rb0 = wg0 + wave * R;
  const int chunks = KS / STEPS, last = chunks - 1;

  const u32x4_t* wbase[R];
  size_t wstep[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bool own = rb0 + r < wg1;
    const int rb = own ? rb0 + r : wg0;
    wbase[r] = (const u32x4_t*)wp + ((size_t)(rb / kTileBlocks) * KS * kTileBlocks + rb % kTileBlocks) * 64 + lane;
    wstep[r] = own ? (size_t)kTileBlocks * 64 : 0;
  }
  auto load_w = [&](Frag (&dst)[R][STEPS], int c) __attribute__((always_inline)) {
    c = c < last ? c : last;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int s = 0; s < STEPS; ++s) dst[r][s].nat = *(wbase[r] + (size_t)(c * STEPS + s) * wstep[r]);
  };
  // token pieces of this thread: pass i covers rows i * 32 + tid / 8, 16-byte column tid % 8
  const int arow0 = tid >> 3, acol = (tid & 7) * 8;
  const bf16_t* abase = a + acol;
  auto load_a = [&](u32x4_t (&dst)[APASS], int c) __attribute__((always_inline)) {
    c = c < last ? c : last;
    int k = c * KC;
    k = k + acol < K - 8 ? k : K - 8 - acol;               // columns past K meet zero-padded weights: any in-bounds piece
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
      int m = row0 + arow0 + i * 32;
      m = m < M ? m : M - 1;                                // rows past the pass: a valid row, results never stored
      dst[i] = *(const u32x4_t*)(abase + (size_t)m * K + k);
    }
  };
  auto store_a = [&](const u32x4_t (&src)[APASS], int stage) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < APASS; ++i)
      *(u32x4_t*)(wide_lds + stage * STAGE + (arow0 + i * 32) * ROWB + (tid & 7) * 16) = src[i];
  };

  floatx4_t acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[r][mt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  Frag wreg[PD][R][STEPS];
  u32x4_t areg[AD][APASS];
  {
    u32x4_t first[APASS];
    load_a(first, 0);
#pragma unroll
    for (int p = 0; p < AD; ++p) load_a(areg[p], 1 + p);
#pragma unroll
    for (int p = 0; p < PD; ++p) load_w(wreg[p], p);
    store_a(first, 0);
  }
  __syncthreads();

  auto body = [&](Frag (&wslot)[R][STEPS], u32x4_t (&aslot)[APASS], int c) __attribute__((always_inline)) {
    const int stage = c & 1;
    const unsigned char* ab = wide_lds + stage * STAGE + r16 * ROWB + g * 16;
    Frag b[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) b[0][j].nat = *(const u32x4_t*)(ab + j * 16 * ROWB);
    store_a(aslot, stage ^ 1);                 // token chunk c + 1 becomes visible after the barrier below
    load_a(aslot, c + AD + 1);
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
#pragma unroll
      for (int mg = 0; mg < MT / 4; ++mg) {
        constexpr int G = MT / 4;
        const int cur = (s * G + mg) & 1;
        if (s * G + mg + 1 < STEPS * G) {      // the next group of four token tiles, while these multiply
          const int ns = (s * G + mg + 1) / G, nm = (s * G + mg + 1) % G;
#pragma unroll
          for (int j = 0; j < 4; ++j) b[cur ^ 1][j].nat = *(const u32x4_t*)(ab + (nm * 4 + j) * 16 * ROWB + ns * 64);
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[r][mg * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wslot[r][s].v, b[cur][j].v, acc[r][mg * 4 + j], 0, 0, 0);
      }
    load_w(wslot, c + PD);
    __syncthreads();
  };
  static_assert(PD == 2 && (AD == 1 || AD == 2), "the loop below alternates two ring slots");
  int c = 0;
  for (; c + 2 <= chunks; c += 2) {
    body(wreg[0], areg[0], c);
    body(wreg[1], areg[AD - 1], c + 1);
  }
  if (c < chunks) body(wreg[0], areg[0], c);

  float4 row_ss[MT];
  if (rs.ss) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = row0 + mt * 16 + r16;
      row_ss[mt] = *(const float4*)(rs.ss + (size_t)(m < M ? m : M - 1) * kNormParts);
    }
  }
  finish_rows<MT, R, EPI>(acc, row_ss, rb0, wg1, M, N, outp, qe, rs, row0, 0);
}

// Workgroup shape.  R = 2 row blocks per wavefront when that still leaves >= 80 workgroups, else R = 1.
// Every workgroup re-reads the whole activation panel, and a compute unit ingests only ~45 GB/s (measured,
// weights + panel), so the fastest grid is the one closest to one workgroup on each of the 256 compute
// units: 3 wavefronts (6 row blocks) per workgroup when that gives <= 260 workgroups, else 4 (8 row
// blocks); split-K (gemm_mfma_splits) tops small-N grids up to about 256.
int rows_per_wave(int N) { return N / 16 / 8 >= 80 ? 2 : 1; }
int waves_per_group(int n_rb) { return (n_rb + 5) / 6 <= 260 ? 3 : 4; }

// With a token panel of more than 16 rows the panel a workgroup re-reads is no longer small beside its weight
// rows (64 weight rows against a 64-row panel: half of what it ingests).  When K is long enough to give every
// split 2048 columns, 128-row workgroups (R = 2, four wavefronts) on a deeper split-K halve that share at the
// same grid size: measured at M = 64, N x K = 5120 x 13824: 28.1 -> 25.5 us, 8192 x 28672: 83.7 -> 74.8 us,
// 10240 x 8192: 30.1 -> 28.1 us; at 4096 x 4096 and 4096 x 11008 (512 / 1376 columns per split) it loses or ties.
int wide_split(int M, int N, int K) {
  if (M <= 16) return 0;
  const int tiles = (N / 16 + 7) / 8;
  const int s = (256 + tiles / 2) / tiles;
  return s >= 2 && s <= kMaxSplitK && K / s >= 2048 ? s : 0;
}

template <int MT>
hipError_t launch_mt(const bf16_t* a, const PackedW& w, int M, void* out, int nsplit, int epi, const QkvEpilogue& qe,
                     const RowScale& rs, hipStream_t s, int row0) {
  const int n_rb = w.N / 16;
  const int KS = w.Kp / 32;
  constexpr int KC = MT == 1 ? 128 : kChunkCols;     // the chunk must give every thread at least one 16-byte piece
  if (epi == EPI_F32 && wide_split(M, w.N, w.K)) {
    hipLaunchKernelGGL((gemm_packed_kernel<MT, 2, 4, EPI_F32, KC>), dim3((n_rb + 7) / 8, nsplit), dim3(256), 0, s, a,
                       w.p, M, w.N, w.K, KS, out, nsplit, qe, rs, row0);
  } else if (epi == EPI_SILU || (epi == EPI_F32 && rows_per_wave(w.N) == 2)) {
    const bool three = waves_per_group(n_rb) == 3;
    // a grid just short of the 256 compute units is topped up to 256 (the kernel shares the row blocks evenly):
    // measured 32.3 -> 31.6 us at 22016 x 4096, M = 64, and 30.6 -> 29.2 us at M = 1
    int gx = three ? (n_rb + 5) / 6 : (n_rb + 7) / 8;
    if (gx >= 200 && gx < 256 && (epi == EPI_SILU || nsplit == 1)) gx = 256;
    const dim3 grid(gx, epi == EPI_SILU ? 1 : nsplit);
    if (epi == EPI_SILU) {
      if (three)
        hipLaunchKernelGGL((gemm_packed_kernel<MT, 2, 3, EPI_SILU, 128>), grid, dim3(192), 0, s, a, w.p, M, w.N, w.K, KS,
                           out, 1, qe, rs, row0);
      else
        hipLaunchKernelGGL((gemm_packed_kernel<MT, 2, 4, EPI_SILU, KC>), grid, dim3(256), 0, s, a, w.p, M, w.N, w.K, KS,
                           out, 1, qe, rs, row0);
    } else {
      if (three)
        hipLaunchKernelGGL((gemm_packed_kernel<MT, 2, 3, EPI_F32, 128>), grid, dim3(192), 0, s, a, w.p, M, w.N, w.K, KS,
                           out, nsplit, qe, rs, row0);
      else
        hipLaunchKernelGGL((gemm_packed_kernel<MT, 2, 4, EPI_F32, KC>), grid, dim3(256), 0, s, a, w.p, M, w.N, w.K, KS,
                           out, nsplit, qe, rs, row0);
    }
  } else if (epi == EPI_QKV) {
    // no split-K here, so one row block per wavefront and three or four wavefronts: 768 row blocks (a 4096-wide
    // model with full-size K/V heads) fill 256 workgroups exactly; measured 23.4 -> 21.6 us against two blocks
    // per wavefront in 192 workgroups of two
    const bool four = n_rb > 3 * 256;
    int gx = four ? (n_rb + 3) / 4 : (n_rb + 2) / 3;
    if (gx < 256 && n_rb >= 256) gx = 256;
    if (four)
      hipLaunchKernelGGL((gemm_packed_kernel<MT, 1, 4, EPI_QKV, KC>), dim3(gx, 1), dim3(256), 0, s, a, w.p, M, w.N, w.K,
                         KS, out, 1, qe, rs, row0);
    else
      hipLaunchKernelGGL((gemm_packed_kernel<MT, 1, 3, EPI_QKV, KC>), dim3(gx, 1), dim3(192), 0, s, a, w.p, M, w.N, w.K,
                         KS, out, 1, qe, rs, row0);
  } else {
    hipLaunchKernelGGL((gemm_packed_kernel<MT, 1, 4, EPI_F32, KC>), dim3((n_rb + 3) / 4, nsplit), dim3(256), 0, s, a,
                       w.p, M, w.N, w.K, KS, out, nsplit, qe, rs, row0);
  }
  return hipGetLastError();
}

// Rows [row0, row0 + rows) of a pass of M rows: the instance with the fewest token tiles that hold them.
hipError_t launch_rows(const bf16_t* ap, const PackedW& w, int rows, int M, void* out, int nsplit, int epi,
                       const QkvEpilogue& qe, const RowScale& rs, hipStream_t s, int row0) {
  if (rows <= 16) return launch_mt<1>(ap, w, M, out, nsplit, epi, qe, rs, s, row0);
  if (rows <= 32) return launch_mt<2>(ap, w, M, out, nsplit, epi, qe, rs, s, row0);
  if (rows <= 64) return launch_mt<4>(ap, w, M, out, nsplit, epi, qe, rs, s, row0);
  if (rows <= 80) return launch_mt<5>(ap, w, M, out, nsplit, epi, qe, rs, s, row0);   // a 64-node tree plus a few pseudo rows
  if (rows <= 96) return launch_mt<6>(ap, w, M, out, nsplit, epi, qe, rs, s, row0);
  return launch_mt<8>(ap, w, M, out, nsplit, epi, qe, rs, s, row0);
}

// A workgroup holds at most 128 token rows (accumulators and the activation ring are registers): a pass of more
// rows runs as two launches over the same weights, rows 0..127 and the rest, each writing its own rows of the
// same outputs.  The K split is the caller's and the same for both.
hipError_t launch_any(const void* a, const PackedW& w, int M, void* out, int nsplit, int epi, const QkvEpilogue& qe,
                      const RowScale& rs, hipStream_t s) {
  const bf16_t* ap = (const bf16_t*)a;
  if (M <= 128) return launch_rows(ap, w, M, M, out, nsplit, epi, qe, rs, s, 0);
  const hipError_t e = launch_rows(ap, w, 128, M, out, nsplit, epi, qe, rs, s, 0);
  return e != hipSuccess ? e : launch_rows(ap, w, M - 128, M, out, nsplit, epi, qe, rs, s, 128);
}

}  // namespace

bool gemm_mfma_supported(int M, int N, int K) { return M >= 1 && M <= kMaxRows && N % 16 == 0 && K % 8 == 0 && N >= 16; }

int packed_cols(int K) { return (K + kPadCols - 1) / kPadCols * kPadCols; }

size_t packed_weight_bytes(int N, int K) {
  const size_t rbs = (size_t)(N / 16 + kTileBlocks - 1) / kTileBlocks * kTileBlocks;
  return rbs * 16 * packed_cols(K) * sizeof(bf16_t);
}

int gemm_mfma_splits(int M, int N, int K) {
  if (const int wide = wide_split(M, N, K)) return wide;
  const int n_rb = N / 16;
  const int per_wg = rows_per_wave(N) == 2 ? 2 * waves_per_group(n_rb) : 4;      // row blocks per workgroup
  const int tiles = (n_rb + per_wg - 1) / per_wg;
  int s = (256 + tiles / 2) / tiles;         // nearest grid to 256 workgroups
  const int chunks = (K + 127) / 128;
  if (s > chunks / 4) s = chunks / 4;        // at least 512 columns per split
  if (s > kMaxSplitK) s = kMaxSplitK;
  if (s < 1) s = 1;
  return s;
}

hipError_t launch_repack(WeightSegs w, int K, int mode, int head_dim, void* dst, hipStream_t s) {
  int rows = 0;
  for (int i = 0; i < w.nseg; ++i) rows += w.rows[i];
  const int n_rb = rows / 16, KS = packed_cols(K) / 32;
  const size_t pieces = (size_t)((n_rb + kTileBlocks - 1) / kTileBlocks) * kTileBlocks * KS * 64;
  hipLaunchKernelGGL(repack_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, w, K, KS, n_rb, mode,
                     head_dim / 16, (bf16_t*)dst);
  return hipGetLastError();
}

hipError_t launch_gemm_packed(const void* a, PackedW w, int M, float* out, int nsplit, hipStream_t s, RowScale rs) {
  return launch_any(a, w, M, out, nsplit, EPI_F32, QkvEpilogue{}, rs, s);
}

hipError_t launch_gemm_packed_silu(const void* a, PackedW w, int M, void* act, hipStream_t s, RowScale rs) {
  return launch_any(a, w, M, act, 1, EPI_SILU, QkvEpilogue{}, rs, s);
}

namespace {
template <int EPI>
hipError_t launch_wide(const void* a, const PackedW& w, int M, void* out, const RowScale& rs, hipStream_t s) {
  constexpr int MT = 8, R = 4;                            // 128 tokens x 256 features per workgroup, two workgroups per unit
  const int n_tiles = (w.N / 16 + 4 * R - 1) / (4 * R), m_tiles = (M + MT * 16 - 1) / (MT * 16);
  const int lds = 2 * MT * 16 * (64 * 2 + kRowPad);
  hipLaunchKernelGGL((gemm_wide_kernel<MT, R, EPI, 1, 2>), dim3(8 * ((n_tiles + 7) / 8) * m_tiles), dim3(256), lds, s,
                     (const bf16_t*)a, w.p, M, w.N, w.K, w.Kp / 32, out, QkvEpilogue{}, rs, n_tiles, m_tiles);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_gemm_wide(const void* a, PackedW w, int M, float* out, hipStream_t s, RowScale rs) {
  return launch_wide<EPI_F32>(a, w, M, out, rs, s);
}
hipError_t launch_gemm_wide_silu(const void* a, PackedW w, int M, void* act, hipStream_t s, RowScale rs) {
  return launch_wide<EPI_SILU>(a, w, M, act, rs, s);
}

bool qkv_fusable(int head_dim) { return head_dim % 32 == 0; }

// The fused q|k|v product cannot split K, so its workgroups stay small (three or four row blocks); with few row
// blocks (70B-shaped grouped-query projections: 640) the 128-row split-K workgroups plus a separate rotary/append
// kernel are faster once the token panel is large (measured 41 us against 28 + 7 us at M = 64).
bool qkv_prefer_split(int M, int N) { return M > 16 && N / 16 / 4 < 176; }

hipError_t launch_gemm_packed_qkv(const void* a, PackedW w, int M, QkvEpilogue qe, hipStream_t s, RowScale rs) {
  return launch_any(a, w, M, nullptr, 1, EPI_QKV, qe, rs, s);
}

}  // namespace ht
