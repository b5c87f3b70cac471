// Tree-masked attention over the KV cache on CDNA4 matrix cores (bf16 in, fp32 softmax and sums).
//
//   out[m][h] = softmax_{j visible to m}( q[m][h] . K[j] / sqrt(hd) ) V[j]
//   visible(m) = cache slots 0 .. n-1  U  { n + u : u is m or an ancestor of m }          (ancestor bit masks)
//
// Everything is computed transposed so that no operand ever needs an LDS transpose:
//   S^T[key][query] = K[key][:] . Q[query][:]      MFMA "A" rows = keys   (K cache rows are contiguous in e)
//   O^T[e][query]  += V^T[e][key] . P[key][query]  MFMA "A" rows = e      (V cache is stored [head][e][slot],
//                                                                          so 8 consecutive keys are 16 bytes)
// K and V fragments are loaded from global memory straight into MFMA operand registers.  The 32 keys of
// a chunk are assigned to the two 16-row score blocks in the interleaved order key = 8 (r / 4) + 4 b + r % 4,
// which makes the eight scores a lane holds after the S MFMAs exactly the eight consecutive keys the P
// operand of the O MFMA wants: probabilities go from accumulator to operand registers without leaving the
// lane.  Online softmax runs per lane (a query column lives in 4 lanes: two xor-shuffles for the row max).
//
// A workgroup works on one query head and one slice of the keys.  Two kernels share this scheme:
//   attn_mfma_kernel (<= 16 rows): K and V fragments are loaded from global memory straight into MFMA
//     operand registers, the four wavefronts take 32-key chunks round-robin and merge (max, sum, O)
//     through LDS;
//   attn_tile_kernel (more rows): every wavefront owns 16 or 32 rows, 64-key tiles of K and V^T are staged
//     in LDS with fully coalesced loads and shared by the wavefronts (per-lane operand loads from global
//     memory cost one L1 tag lookup per lane and made the first version L1-bound).
// With more than one key slice the partials go to scratch and a small kernel combines them.
#include "ht_common.h"
#include <type_traits>

namespace ht {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

namespace {

union Frag {
  u32x4_t nat;
  bf16x8_t v;
  uint32_t u[4];
};

constexpr int kMaxSplits = 16;
constexpr float kRescaleStep = 8.0f;    // log2 units the running maximum may lag behind before accumulators are rescaled

template <int HD, int QB>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                                        const bf16_t* __restrict__ vc, int cap, int n, int M,
                                                        const uint64_t* __restrict__ anc, int Hq, int Hkv,
                                                        bf16_t* __restrict__ out, float* __restrict__ part_o,
                                                        float* __restrict__ part_ml, int nsplit, float scale_log2,
                                                        const int32_t* __restrict__ n_dev) {
  n = cache_len(n, n_dev);
  constexpr int ES = HD / 32;      // contraction steps of the score MFMAs
  constexpr int EB = HD / 16;      // 16-row blocks of O^T
  // LDS merge area: per wave, O accumulators [QB][EB][4][64], running max [QB][64], partial sums [QB][64]
  constexpr int O_FLOATS = QB * EB * 4 * 64;
  __shared__ float lds_o[4 * O_FLOATS];
  __shared__ float lds_m[4 * QB * 64];
  __shared__ float lds_l[4 * QB * 64];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, g = lane >> 4;
  const int h = blockIdx.x, hk = h / (Hq / Hkv);
  // the workgroup's wavefronts share QB row blocks and take every 4th chunk of the key slice
  const int m0 = blockIdx.y * QB * 16;
  const int split = blockIdx.z;
  const int S = n + M;
  const int chunks = (S + 31) / 32;
  int cs, ce;
  even_share(chunks, nsplit, split, cs, ce);

  // queries of this lane: token m0 + qb*16 + r16 (clamped for loads), e columns es*32 + g*8 ..
  Frag qf[QB][ES];
  uint64_t amask[QB][kMaskWords];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int m = m0 + qb * 16 + r16;
    const int mc = m < M ? m : M - 1;
    const bf16_t* qrow = q + ((size_t)mc * Hq + h) * HD + g * 8;
#pragma unroll
    for (int es = 0; es < ES; ++es) qf[qb][es].nat = *(const u32x4_t*)(qrow + es * 32);
#pragma unroll
    for (int wd = 0; wd < kMaskWords; ++wd) amask[qb][wd] = m < M ? anc[(size_t)m * kMaskWords + wd] : 0ull;
  }

  floatx4_t oacc[QB][EB];
  float mrun[QB], lrun[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    mrun[qb] = -INFINITY;
    lrun[qb] = 0.f;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) oacc[qb][eb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  }

  const bf16_t* kbase = kc + (size_t)hk * HD + g * 8;
  const bf16_t* vbase = vc + ((size_t)hk * HD + r16) * cap;

  // K fragments: row r of block b is key j0 + 8 (r / 4) + 4 b + r % 4 (clamped into the cache).
  // V^T fragments: rows e = eb*16 + r16, keys j0 + g*8 .. + 7 (clamped start keeps the load in bounds).
  auto load_kv = [&](Frag (&kf)[2][ES], Frag (&vf)[EB], int c) __attribute__((always_inline)) {
    const int j0 = c * 32;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      int key = j0 + (r16 >> 2) * 8 + b * 4 + (r16 & 3);
      key = key < cap ? key : cap - 1;
      const bf16_t* krow = kbase + (size_t)key * Hkv * HD;
#pragma unroll
      for (int es = 0; es < ES; ++es) kf[b][es].nat = *(const u32x4_t*)(krow + es * 32);
    }
    int kv = j0 + g * 8;
    kv = kv + 8 <= cap ? kv : cap - 8;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) vf[eb].nat = *(const u32x4_t*)(vbase + (size_t)eb * 16 * cap + kv);
  };

  auto process = [&](Frag (&kf)[2][ES], Frag (&vf)[EB], int c) __attribute__((always_inline)) {
    const int j0 = c * 32;
    if (j0 + 32 > S) {            // keys past the last tree row carry no defined values: zero them
      const int first_bad = S - (j0 + g * 8);       // elements >= first_bad are invalid
#pragma unroll
      for (int eb = 0; eb < EB; ++eb)
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
          uint32_t keep = 0;
          if (2 * w2 < first_bad) keep |= 0x0000ffffu;
          if (2 * w2 + 1 < first_bad) keep |= 0xffff0000u;
          vf[eb].u[w2] &= keep;
        }
    }
    const bool need_mask = j0 + 32 > n;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      floatx4_t s[2];
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        s[b] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int es = 0; es < ES; ++es)
          s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[b][es].v, qf[qb][es].v, s[b], 0, 0, 0);
      }
      // lane holds keys j0 + g*8 + t, t = 4 b + i  (raw scores; the softmax scale is folded into the exponent)
      float p[8];
      float cmax = -INFINITY;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        float v = s[t >> 2][t & 3];
        if (need_mask) {
          const int j = j0 + g * 8 + t;
          bool vis = j < n;
          if (!vis && j < S) {
            const int u = j - n;
            vis = (amask[qb][u >> 6] >> (u & 63)) & 1ull;
          }
          v = vis ? v : -INFINITY;
        }
        p[t] = v;
        cmax = fmaxf(cmax, v);
      }
      cmax = fmaxf(cmax, __shfl_xor(cmax, 16, 64));
      cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
      const float mnew = fmaxf(mrun[qb], cmax * scale_log2);       // running max in scaled (log2) units
      const float msafe = mnew == -INFINITY ? 0.f : mnew;
      float psum = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        p[t] = __builtin_amdgcn_exp2f(fmaf(p[t], scale_log2, -msafe));   // masked: exp2(-inf) = 0
        psum += p[t];
      }
      // the accumulators are rescaled only when some row of the wavefront saw a new maximum
      if (__any(mnew != mrun[qb])) {
        const float alpha = __builtin_amdgcn_exp2f(mrun[qb] - msafe);    // mrun = -inf -> 0
        lrun[qb] *= alpha;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) oacc[qb][eb] *= alpha;
        mrun[qb] = mnew;
      }
      lrun[qb] += psum;
      Frag pf;
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) {
        floatx2_t f2 = {p[2 * w2], p[2 * w2 + 1]};
        bf16x2_t b2 = __builtin_convertvector(f2, bf16x2_t);             // v_cvt_pk_bf16_f32 (RNE)
        pf.u[w2] = *(const uint32_t*)&b2;
      }
#pragma unroll
      for (int eb = 0; eb < EB; ++eb)
        oacc[qb][eb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[eb].v, pf.v, oacc[qb][eb], 0, 0, 0);
    }
  };

  // two register sets: the next chunk of this wavefront is in flight while the current one is multiplied
  {
    constexpr int STEP = 4;
    Frag kf0[2][ES], vf0[EB], kf1[2][ES], vf1[EB];
    int c = cs + wave;
    if (c < ce) load_kv(kf0, vf0, c);
    for (; c < ce; c += 2 * STEP) {
      if (c + STEP < ce) load_kv(kf1, vf1, c + STEP);
      process(kf0, vf0, c);
      if (c + STEP < ce) {
        if (c + 2 * STEP < ce) load_kv(kf0, vf0, c + 2 * STEP);
        process(kf1, vf1, c + STEP);
      }
    }
  }

  // ---- merge the four wavefronts
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    lds_m[(wave * QB + qb) * 64 + lane] = mrun[qb];
    lds_l[(wave * QB + qb) * 64 + lane] = lrun[qb];
#pragma unroll
    for (int eb = 0; eb < EB; ++eb)
#pragma unroll
      for (int i = 0; i < 4; ++i) lds_o[wave * O_FLOATS + ((qb * EB + eb) * 4 + i) * 64 + lane] = oacc[qb][eb][i];
  }
  __syncthreads();
  // wavefront w finalises e blocks w, w + 4, ..
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    float mw[4], mall = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mw[w] = lds_m[(w * QB + qb) * 64 + lane];
      mall = fmaxf(mall, mw[w]);
    }
    const float msafe = mall == -INFINITY ? 0.f : mall;
    float fw[4], lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      fw[w] = exp2f(mw[w] - msafe);
      lsum += fw[w] * lds_l[(w * QB + qb) * 64 + lane];
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    const int m = m0 + qb * 16 + r16;
    for (int eb = wave; eb < EB; eb += 4) {
      float o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) t += fw[w] * lds_o[w * O_FLOATS + ((qb * EB + eb) * 4 + i) * 64 + lane];
        o[i] = t;
      }
      if (m < M) {
        const int e0 = eb * 16 + g * 4;
        if (nsplit == 1) {
          const float inv = 1.0f / lsum;
          *(uint2*)(out + (size_t)m * Hq * HD + (size_t)h * HD + e0) =
              pack4_bf16(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
        } else {
          float* dst = part_o + (((size_t)h * nsplit + split) * M + m) * HD + e0;
          *(float4*)dst = make_float4(o[0], o[1], o[2], o[3]);
        }
      }
    }
    if (nsplit > 1 && wave == 0 && g == 0 && m < M) {
      float* ml = part_ml + (((size_t)h * nsplit + split) * M + m) * 2;
      ml[0] = mall;
      ml[1] = lsum;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// More than 16 rows: every wavefront owns one block of 16 rows and all wavefronts of the workgroup need the
// same keys, so the workgroup stages 64-key tiles of K ([key][e]) and V^T ([e][key]) in LDS with fully
// coalesced loads (whole 128/256-byte runs per row) and each wavefront reads its MFMA operands from there.
// The 16-byte pieces of a row are XOR-swizzled so that the 16 rows a fragment read touches fall into
// different banks.  The next tile is in flight in registers while the current one is multiplied.
// Tiles that lie entirely inside the cache (keys < n) run a loop body without any mask or tail code; only
// the last one to three tiles evaluate the ancestor masks and zero the V columns past the last tree row.

// max over lanes l, l ^ 16, l ^ 32, l ^ 48 with the two gfx950 half/row swaps (no LDS round trip)
__device__ __forceinline__ float max_over_groups(float x) {
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);      // rows (0,0,2,2) and (1,1,3,3)
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  u = __float_as_uint(x);
  auto r2 = __builtin_amdgcn_permlane32_swap(u, u, false, false);     // halves (lo,lo) and (hi,hi)
  return fmaxf(__uint_as_float(r2[0]), __uint_as_float(r2[1]));
}
__device__ __forceinline__ float sum_over_groups(float x) {
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  u = __float_as_uint(x);
  auto r2 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r2[0]) + __uint_as_float(r2[1]);
}

template <int HD, int QB, int NW>
__global__ __launch_bounds__(64 * NW) void attn_tile_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                                            const bf16_t* __restrict__ vc, int cap, int n, int M,
                                                            const uint64_t* __restrict__ anc, int Hq, int Hkv,
                                                            bf16_t* __restrict__ out, float* __restrict__ part_o,
                                                            float* __restrict__ part_ml, int nsplit, float scale_log2,
                                                            const int32_t* __restrict__ n_dev, int chunk) {
  n = cache_len(n, n_dev);
  // chunk > 0 (a whole causal sequence in one launch): the M rows come in chunks of `chunk` rows, and a chunk is a
  // pass of its own that sees the cache up to its first row plus its own rows through `anc` (the same masks for every
  // chunk).  Every workgroup walks all its keys (no key slices); with nsplit > 1 it leaves its result as slice 0 of
  // nsplit for a merge with slices that someone else writes.  Workgroups are taken from the last chunk backwards: the
  // longest key ranges start first.
  int gy = blockIdx.y, row_base = 0;
  const int Mtot = M;
  if (chunk > 0) {
    gy = gridDim.y - 1 - gy;
    row_base = gy * (NW * QB * 16) / chunk * chunk;
    n += row_base;
    q += (size_t)row_base * Hq * HD;
    out += (size_t)row_base * Hq * HD;
    M = M - row_base < chunk ? M - row_base : chunk;
    gy -= row_base / (NW * QB * 16);
  }
  constexpr int TK = 64;                 // keys per tile
  constexpr int ES = HD / 32, EB = HD / 16;
  constexpr int THREADS = 64 * NW;
  constexpr int PK = HD / 8;             // 16-byte pieces per K row
  constexpr int KPIECES = TK * PK, VPIECES = HD * (TK / 8);
  constexpr int KP = KPIECES / THREADS, VP = VPIECES / THREADS;
  static_assert(KPIECES % THREADS == 0 && VPIECES % THREADS == 0, "tile must divide over the threads");
  static_assert(THREADS % PK == 0 && THREADS % (TK / 8) == 0, "a thread keeps its column in every pass");
  constexpr int KROWS = THREADS / PK;    // key rows covered by one pass of K pieces
  constexpr int VROWS = THREADS / (TK / 8);
  constexpr int KBYTES = TK * HD * 2, VBYTES = HD * TK * 2;
  __shared__ __attribute__((aligned(16))) unsigned char lds[1][KBYTES + VBYTES];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, g = lane >> 4;
  const int h = blockIdx.x, hk = h / (Hq / Hkv);
  const int m0 = (gy * NW + wave) * QB * 16;
  const int split = chunk > 0 ? 0 : blockIdx.z;
  const int S = n + M;
  const int tiles = (S + TK - 1) / TK;
  int ts, te;
  even_share(tiles, chunk > 0 ? 1 : nsplit, split, ts, te);
  int tmid = n / TK;                     // tiles below tmid hold cache keys only
  tmid = tmid < ts ? ts : (tmid > te ? te : tmid);

  Frag qf[QB][ES];
  uint64_t amask[QB][kMaskWords];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int m = m0 + qb * 16 + r16;
    const int mc = m < M ? m : M - 1;
    const bf16_t* qrow = q + ((size_t)mc * Hq + h) * HD + g * 8;
#pragma unroll
    for (int es = 0; es < ES; ++es) qf[qb][es].nat = *(const u32x4_t*)(qrow + es * 32);
#pragma unroll
    for (int wd = 0; wd < kMaskWords; ++wd) amask[qb][wd] = m < M ? anc[(size_t)m * kMaskWords + wd] : 0ull;
  }
  floatx4_t oacc[QB][EB];
  float mrun[QB], lrun[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    mrun[qb] = -INFINITY;
    lrun[qb] = 0.f;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) oacc[qb][eb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  }

  // staging: in pass i a thread moves the K piece (row tid / PK + i * KROWS, column tid % PK) and the V piece
  // (row e = tid / 8 + i * VROWS, keys (tid % 8) * 8 ..); everything but the tile offset is loop invariant
  const int kl0 = tid / PK, kpc = tid % PK;
  const int ve0 = tid / (TK / 8), vpc = tid % (TK / 8);
  const bf16_t* kcol = kc + (size_t)hk * HD + kpc * 8;
  const bf16_t* vrow = vc + ((size_t)hk * HD + ve0) * cap;
  const unsigned krow_stride = (unsigned)(Hkv * HD);
  int klds[KP];
#pragma unroll
  for (int i = 0; i < KP; ++i) {
    const int kl = kl0 + i * KROWS;
    const int sw = ((((kl >> 3) & 3) << 2) | (kl & 3)) & (PK - 1);
    klds[i] = kl * (HD * 2) + ((kpc ^ sw) << 4);
  }
  static_assert(VROWS % 16 == 0, "the V swizzle of a thread's piece is the same in every pass");
  const int vlds0 = KBYTES + ve0 * (TK * 2) + ((vpc ^ ((ve0 >> 1) & 7)) << 4);     // pass i adds i * VROWS rows
  // The next tile is in flight in registers while the current one is multiplied out of LDS (a second register
  // set, two tiles in flight, measured slower: the staging side already runs near the streaming rate of the
  // memory system).
  u32x4_t kreg[KP], vreg[VP];
  auto load_tile = [&](int t) __attribute__((always_inline)) {
    const int j0 = t * TK;
#pragma unroll
    for (int i = 0; i < KP; ++i) {
      int key = j0 + kl0 + i * KROWS;
      key = key < cap ? key : cap - 1;
      kreg[i] = *(const u32x4_t*)(kcol + (unsigned)key * krow_stride);   // the launcher checks cap*Hkv*HD < 2^31
    }
    int kv = j0 + vpc * 8;
    kv = kv + 8 <= cap ? kv : cap - 8;
#pragma unroll
    for (int i = 0; i < VP; ++i) vreg[i] = *(const u32x4_t*)(vrow + (size_t)i * VROWS * cap + kv);
  };
  auto store_tile = [&](int stage, int t) __attribute__((always_inline)) {
    unsigned char* base = lds[stage];
#pragma unroll
    for (int i = 0; i < KP; ++i) *(u32x4_t*)(base + klds[i]) = kreg[i];
    const int valid = S - (t * TK + vpc * 8);           // keys of this thread's V pieces below S carry data
    if (t >= tmid && valid < 8) {                       // zero what lies past the last tree row
      uint32_t keep[4];
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) keep[w2] = (2 * w2 < valid ? 0x0000ffffu : 0u) | (2 * w2 + 1 < valid ? 0xffff0000u : 0u);
#pragma unroll
      for (int i = 0; i < VP; ++i)
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) vreg[i][w2] &= keep[w2];
    }
#pragma unroll
    for (int i = 0; i < VP; ++i) *(u32x4_t*)(base + vlds0 + i * VROWS * (TK * 2)) = vreg[i];
  };

  // fragment addresses inside a stage: K rows of score block b of the 32-key half `sub`, V^T pieces of `sub`
  int kfo[2], vfo[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) kfo[b] = ((r16 >> 2) * 8 + b * 4 + (r16 & 3)) * (HD * 2);   // interleaved key order
  const int ksw = r16 & (PK - 1);
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) vfo[sub] = KBYTES + r16 * (TK * 2) + (((sub * 4 + g) ^ ((r16 >> 1) & 7)) << 4);

  // One 64-key tile: 4 score blocks (two per 32-key half), one softmax update over the 16 scores a lane
  // holds, then the two halves' probabilities multiply V.
  auto process = [&](auto masked, int stage, int t) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked)::value;
    const unsigned char* base = lds[stage];
    const int j0 = t * TK;
    Frag kf[2][2][ES];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int es = 0; es < ES; ++es)
          kf[sub][b][es].nat = *(const u32x4_t*)(base + kfo[b] + sub * 32 * (HD * 2) + (((es * 4 + g) ^ ksw) << 4));
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      floatx4_t s[2][2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          s[sub][b] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int es = 0; es < ES; ++es)
            s[sub][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[sub][b][es].v, qf[qb][es].v, s[sub][b], 0, 0, 0);
        }
      // lane holds keys j0 + 32 sub + g*8 + tt, tt = 4 b + i (raw scores; the softmax scale is folded into
      // the exponent)
      float p[16];
#pragma unroll
      for (int x = 0; x < 16; ++x) p[x] = s[x >> 3][(x >> 2) & 1][x & 3];
      if (MASKED) {
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const int j = j0 + (x >> 3) * 32 + g * 8 + (x & 7);
          bool vis = j < n;
          if (!vis && j < S) {
            const int u = j - n;
            vis = (amask[qb][u >> 6] >> (u & 63)) & 1ull;
          }
          p[x] = vis ? p[x] : -INFINITY;
        }
      }
      float cmax = p[0];
#pragma unroll
      for (int x = 1; x < 16; ++x) cmax = fmaxf(cmax, p[x]);
      cmax = max_over_groups(cmax) * scale_log2;                   // in scaled (log2) units
      // The reference point of the exponentials only follows the running maximum when that grew by more
      // than kRescaleStep (probabilities stay below 2^kRescaleStep: exact in fp32 sums, same relative
      // precision in bf16), so the accumulators are rescaled once or twice per key slice, not per tile.
      const bool grow = cmax > mrun[qb] + kRescaleStep;            // mrun = -inf: true for any finite score
      if (__any(grow)) {
        const float mnew = grow ? cmax : mrun[qb];
        const float alpha = grow ? __builtin_amdgcn_exp2f(mrun[qb] - cmax) : 1.0f;   // mrun = -inf -> 0
        lrun[qb] *= alpha;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) oacc[qb][eb] *= alpha;
        mrun[qb] = mnew;
      }
      const float msafe = MASKED ? (mrun[qb] == -INFINITY ? 0.f : mrun[qb]) : mrun[qb];   // unmasked scores are finite
      float psum = 0.f;
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        p[x] = __builtin_amdgcn_exp2f(fmaf(p[x], scale_log2, -msafe));        // masked: exp2(-inf) = 0
        psum += p[x];
      }
      lrun[qb] += psum;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        Frag vf[EB];                        // read after the softmax: the K fragments are dead by now
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)     // rows e = eb * 16 + r16: (e >> 1) & 7 does not depend on eb
          vf[eb].nat = *(const u32x4_t*)(base + vfo[sub] + eb * 16 * (TK * 2));
        Frag pf;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
          floatx2_t f2 = {p[sub * 8 + 2 * w2], p[sub * 8 + 2 * w2 + 1]};
          bf16x2_t b2 = __builtin_convertvector(f2, bf16x2_t);                 // v_cvt_pk_bf16_f32 (RNE)
          pf.u[w2] = *(const uint32_t*)&b2;
        }
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
          oacc[qb][eb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[eb].v, pf.v, oacc[qb][eb], 0, 0, 0);
      }
    }
  };
  // One LDS stage of 32 KB: a second one (writing tile t + 1 while tile t is multiplied) measured slightly slower,
  // because it halves the workgroups a compute unit can hold, and other workgroups fill the two barriers' gaps.
  auto step = [&](auto masked, int t) __attribute__((always_inline)) {
    if (m0 < M) process(masked, 0, t);          // wavefronts past the last row only help staging
    __syncthreads();                            // everyone is done reading tile t
    if (t + 1 < te) store_tile(0, t + 1);
    if (t + 2 < te) load_tile(t + 2);
    __syncthreads();
  };

  if (ts < te) {
    load_tile(ts);
    store_tile(0, ts);
    if (ts + 1 < te) load_tile(ts + 1);
    __syncthreads();
    int t = ts;
    for (; t < tmid; ++t) step(std::false_type{}, t);
    for (; t < te; ++t) step(std::true_type{}, t);      // the few tiles that reach past the cache
  }

#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float lsum = sum_over_groups(lrun[qb]);
    const int m = m0 + qb * 16 + r16;
    if (m >= M) continue;
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) {
      const int e0 = eb * 16 + g * 4;
      if (nsplit == 1) {
        const float inv = 1.0f / lsum;
        bf16_t ob[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) ob[i] = float_to_bf16(oacc[qb][eb][i] * inv);
        *(uint2*)(out + (size_t)m * Hq * HD + (size_t)h * HD + e0) = *(const uint2*)ob;
      } else {
        float* dst = part_o + (((size_t)h * nsplit + split) * Mtot + row_base + m) * HD + e0;
        *(float4*)dst = make_float4(oacc[qb][eb][0], oacc[qb][eb][1], oacc[qb][eb][2], oacc[qb][eb][3]);
      }
    }
    if (nsplit > 1 && g == 0) {
      float* ml = part_ml + (((size_t)h * nsplit + split) * Mtot + row_base + m) * 2;
      ml[0] = mrun[qb];
      ml[1] = lsum;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// The tile scheme with a wavefront of its own for the loads, for long key ranges and grouped query heads.  One
// workgroup serves one key/value head and one key slice: NCW wavefronts each own a block of 16 query columns, a column
// being a (query head of the group, tree row) pair, so the query heads that share a key/value head also share its
// tiles (attn_tile_kernel stages them once per query head); one more wavefront does nothing but bring 64-key tiles of
// K and V^T from global memory straight into LDS (16-byte LDS-direct loads: no registers and no LDS stores in
// between), a ring of kStages tiles, one or two tiles ahead of the arithmetic.  One barrier per tile.  The LDS layout
// of a tile is that of attn_tile_kernel (XOR-swizzled 16-byte pieces); an LDS-direct load writes 64 consecutive
// pieces, so every lane picks the global piece that belongs at its place.  Same arithmetic in the same order as
// attn_tile_kernel: the two give the same bits.
template <int N> __device__ __forceinline__ void attn_wait_vm_then_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
__device__ __forceinline__ void attn_wait_lds_then_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int HD> struct RingShape {
  static constexpr int TK = 64;
  static constexpr int KBYTES = TK * HD * 2, VBYTES = HD * TK * 2, STAGE = KBYTES + VBYTES;
  static constexpr int NL = STAGE / 1024;                              // LDS-direct loads per tile
  static constexpr int AHEAD = 63 / NL < 2 ? 63 / NL : 2;              // tiles that may be in flight at a barrier
  static constexpr int STAGES = AHEAD + 2;
  static constexpr int LDS_BYTES = STAGES * STAGE;
};

template <int HD, int NCW>
__global__ __launch_bounds__(64 * (NCW + 1)) void attn_ring_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                                                   const bf16_t* __restrict__ vc, int cap, int n, int M,
                                                                   const uint64_t* __restrict__ anc, int Hq, int Hkv,
                                                                   bf16_t* __restrict__ out, float* __restrict__ part_o,
                                                                   float* __restrict__ part_ml, int nsplit, float scale_log2,
                                                                   const int32_t* __restrict__ n_dev) {
  n = cache_len(n, n_dev);
  using RS = RingShape<HD>;
  constexpr int TK = RS::TK, ES = HD / 32, EB = HD / 16, PK = HD / 8;
  constexpr int KBYTES = RS::KBYTES, STAGE = RS::STAGE, NL = RS::NL, NLK = KBYTES / 1024, AHEAD = RS::AHEAD, ST = RS::STAGES;
  static_assert(KBYTES % 1024 == 0 && RS::VBYTES % 1024 == 0, "whole LDS-direct loads per tile");
  extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, g = lane >> 4;
  const int hk = blockIdx.x, group = Hq / Hkv, split = blockIdx.z;
  const int S = n + M;
  const int tiles = (S + TK - 1) / TK;
  int ts, te;
  even_share(tiles, nsplit, split, ts, te);
  const bool empty = ts >= te;                            // a slice without tiles still leaves its (neutral) partials
  int tmid = n / TK;                                      // tiles below tmid hold cache keys only
  tmid = tmid < ts ? ts : (tmid > te ? te : tmid);
  const int iters = te - ts;
  const bool tail_tile = te == tiles && S % TK != 0;      // the slice ends with a tile that reaches past the last tree row

  if (wave == NCW) {
    // ---- load wavefront.  Piece li < NLK of a tile is K (64 / PK key rows), the others V^T (eight rows e of 64 keys)
    if (empty) return;
    const bf16_t* kbase = kc + (size_t)hk * HD;
    const bf16_t* vbase = vc + (size_t)hk * HD * cap;
    const unsigned krow_stride = (unsigned)(Hkv * HD);
    auto fetch = [&](int t, int stage) __attribute__((always_inline)) {
      t = t < te - 1 ? t : te - 1;                          // past the slice: a redundant in-bounds reload, never read
      const int j0 = t * TK;
      unsigned char* base = ring + stage * STAGE;
#pragma unroll
      for (int li = 0; li < NLK; ++li) {
        const int piece = li * 64 + lane, kl = piece / PK, pos = piece % PK;
        const int sw = ((((kl >> 3) & 3) << 2) | (kl & 3)) & (PK - 1);
        int key = j0 + kl;
        key = key < cap ? key : cap - 1;
        __builtin_amdgcn_global_load_lds(
            (const void __attribute__((address_space(1)))*)(kbase + (unsigned)key * krow_stride + (pos ^ sw) * 8),
            (void __attribute__((address_space(3)))*)(base + li * 1024), 16, 0, 0);
      }
#pragma unroll
      for (int li = 0; li < NL - NLK; ++li) {
        const int piece = li * 64 + lane, e = piece / (TK / 8), pos = piece % (TK / 8);
        int kv = j0 + (pos ^ ((e >> 1) & 7)) * 8;
        kv = kv + 8 <= cap ? kv : cap - 8;
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(vbase + (size_t)e * cap + kv),
                                         (void __attribute__((address_space(3)))*)(base + KBYTES + li * 1024), 16, 0, 0);
      }
    };
    // V columns of keys past the last tree row hold whatever the cache holds there: zeroed in LDS once the tile has
    // landed (their probabilities are zero, but zero times a stray NaN would not be)
    auto clear_tail = [&](int stage) __attribute__((always_inline)) {
      const int valid = S - (tiles - 1) * TK;               // keys of the tile that carry data, 1 .. TK - 1
      unsigned char* vb = ring + stage * STAGE + KBYTES;
      for (int idx = lane; idx < HD * (TK - valid); idx += 64) {
        const int e = idx / (TK - valid), key = valid + idx % (TK - valid);
        *(bf16_t*)(vb + e * (TK * 2) + (((key >> 3) ^ ((e >> 1) & 7)) << 4) + (key & 7) * 2) = 0;
      }
    };
#pragma unroll
    for (int p = 0; p < ST - 1; ++p) fetch(ts + p, p);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(AHEAD * NL) : "memory");      // tile ts has landed
    if (tail_tile && iters == 1) clear_tail(0);
    attn_wait_vm_then_barrier<AHEAD * NL>();
    int stage = ST - 1;
    for (int i = 0; i < iters; ++i) {
      fetch(ts + i + ST - 1, stage);                        // the stage the others finished before the last barrier
      stage = stage + 1 == ST ? 0 : stage + 1;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(AHEAD * NL) : "memory");    // tile ts + i + 1 has landed
      if (tail_tile && i + 2 == iters) clear_tail((i + 1) % ST);
      attn_wait_vm_then_barrier<AHEAD * NL>();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // nothing may still be writing LDS when the wavefront ends
    return;
  }

  // ---- arithmetic wavefronts: one block of 16 query columns each
  const int row_blocks = (M + 15) / 16, blocks = group * row_blocks;
  const int blk = blockIdx.y * NCW + wave;
  const bool live = blk < blocks;
  const int bc = live ? blk : blocks - 1;
  const int h = hk * group + bc / row_blocks, m0 = (bc % row_blocks) * 16;
  Frag qf[ES];
  uint64_t amask[kMaskWords];
  {
    const int m = m0 + r16, mc = m < M ? m : M - 1;
    const bf16_t* qrow = q + ((size_t)mc * Hq + h) * HD + g * 8;
#pragma unroll
    for (int es = 0; es < ES; ++es) qf[es].nat = *(const u32x4_t*)(qrow + es * 32);
#pragma unroll
    for (int wd = 0; wd < kMaskWords; ++wd) amask[wd] = m < M ? anc[(size_t)m * kMaskWords + wd] : 0ull;
  }
  floatx4_t oacc[EB];
  float mrun = -INFINITY, lrun = 0.f;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) oacc[eb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  int kfo[2], vfo[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) kfo[b] = ((r16 >> 2) * 8 + b * 4 + (r16 & 3)) * (HD * 2);   // interleaved key order
  const int ksw = r16 & (PK - 1);
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) vfo[sub] = KBYTES + r16 * (TK * 2) + (((sub * 4 + g) ^ ((r16 >> 1) & 7)) << 4);

  auto process = [&](auto masked, int stage, int t) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked)::value;
    const unsigned char* base = ring + stage * STAGE;
    const int j0 = t * TK;
    Frag kf[2][2][ES];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int es = 0; es < ES; ++es)
          kf[sub][b][es].nat = *(const u32x4_t*)(base + kfo[b] + sub * 32 * (HD * 2) + (((es * 4 + g) ^ ksw) << 4));
    floatx4_t s[2][2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        s[sub][b] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int es = 0; es < ES; ++es)
          s[sub][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[sub][b][es].v, qf[es].v, s[sub][b], 0, 0, 0);
      }
    float p[16];
#pragma unroll
    for (int x = 0; x < 16; ++x) p[x] = s[x >> 3][(x >> 2) & 1][x & 3];
    if (MASKED) {
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int j = j0 + (x >> 3) * 32 + g * 8 + (x & 7);
        bool vis = j < n;
        if (!vis && j < S) {
          const int u = j - n;
          vis = (amask[u >> 6] >> (u & 63)) & 1ull;
        }
        p[x] = vis ? p[x] : -INFINITY;
      }
    }
    float cmax = p[0];
#pragma unroll
    for (int x = 1; x < 16; ++x) cmax = fmaxf(cmax, p[x]);
    cmax = max_over_groups(cmax) * scale_log2;
    const bool grow = cmax > mrun + kRescaleStep;
    if (__any(grow)) {
      const float mnew = grow ? cmax : mrun;
      const float alpha = grow ? __builtin_amdgcn_exp2f(mrun - cmax) : 1.0f;
      lrun *= alpha;
#pragma unroll
      for (int eb = 0; eb < EB; ++eb) oacc[eb] *= alpha;
      mrun = mnew;
    }
    const float msafe = MASKED ? (mrun == -INFINITY ? 0.f : mrun) : mrun;
    float psum = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      p[x] = __builtin_amdgcn_exp2f(fmaf(p[x], scale_log2, -msafe));
      psum += p[x];
    }
    lrun += psum;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      Frag vf[EB];
#pragma unroll
      for (int eb = 0; eb < EB; ++eb) vf[eb].nat = *(const u32x4_t*)(base + vfo[sub] + eb * 16 * (TK * 2));
      Frag pf;
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) {
        floatx2_t f2 = {p[sub * 8 + 2 * w2], p[sub * 8 + 2 * w2 + 1]};
        bf16x2_t b2 = __builtin_convertvector(f2, bf16x2_t);
        pf.u[w2] = *(const uint32_t*)&b2;
      }
#pragma unroll
      for (int eb = 0; eb < EB; ++eb)
        oacc[eb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[eb].v, pf.v, oacc[eb], 0, 0, 0);
    }
  };

  if (!empty) {
    attn_wait_lds_then_barrier();                           // tile ts is in LDS
    int stage = 0, t = ts;
    for (; t < tmid; ++t) {
      if (live) process(std::false_type{}, stage, t);
      stage = stage + 1 == ST ? 0 : stage + 1;
      attn_wait_lds_then_barrier();
    }
    for (; t < te; ++t) {                                   // the few tiles that reach past the cache
      if (live) process(std::true_type{}, stage, t);
      stage = stage + 1 == ST ? 0 : stage + 1;
      attn_wait_lds_then_barrier();
    }
  }

  const float lsum = sum_over_groups(lrun);
  const int m = m0 + r16;
  if (!live || m >= M) return;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) {
    const int e0 = eb * 16 + g * 4;
    if (nsplit == 1) {
      const float inv = 1.0f / lsum;
      bf16_t ob[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) ob[i] = float_to_bf16(oacc[eb][i] * inv);
      *(uint2*)(out + (size_t)m * Hq * HD + (size_t)h * HD + e0) = *(const uint2*)ob;
    } else {
      float* dst = part_o + (((size_t)h * nsplit + split) * M + m) * HD + e0;
      *(float4*)dst = make_float4(oacc[eb][0], oacc[eb][1], oacc[eb][2], oacc[eb][3]);
    }
  }
  if (nsplit > 1 && g == 0) {
    float* ml = part_ml + (((size_t)h * nsplit + split) * M + m) * 2;
    ml[0] = mrun;
    ml[1] = lsum;
  }
}

// out[m][h] = sum_s exp2(m_s - m*) O_s / sum_s exp2(m_s - m*) l_s, splits added in index order.
// HD / 4 lanes per (row, head) pair, four output elements per lane; 256-thread blocks.
template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                         int nsplit, int M, int Hq, bf16_t* __restrict__ out) {
  constexpr int LANES = HD / 4, PAIRS = 256 / LANES;               // grid = (row groups of PAIRS rows, heads)
  const int h = blockIdx.y, m = blockIdx.x * PAIRS + threadIdx.x / LANES;
  const int e = (threadIdx.x % LANES) * 4;
  if (m >= M) return;
  float ms[kMaxSplits], mall = -INFINITY;
  for (int s = 0; s < nsplit; ++s) {
    ms[s] = part_ml[(((size_t)h * nsplit + s) * M + m) * 2];
    mall = fmaxf(mall, ms[s]);
  }
  const float msafe = mall == -INFINITY ? 0.f : mall;
  float l = 0.f;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < nsplit; ++s) {
    const size_t idx = ((size_t)h * nsplit + s) * M + m;
    const float f = __builtin_amdgcn_exp2f(ms[s] - msafe);          // exp2(-inf) = 0 for empty slices
    l += f * part_ml[idx * 2 + 1];
    const float4 v = *(const float4*)(part_o + idx * HD + e);
    o.x += f * v.x; o.y += f * v.y; o.z += f * v.z; o.w += f * v.w;
  }
  const float inv = __builtin_amdgcn_rcpf(l);
  *(uint2*)(out + (size_t)m * Hq * HD + (size_t)h * HD + e) = pack4_bf16(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
}

// One more slice for attn_merge_kernel: every row's own key and value, taken from buffers of their own (`ks`
// [M][Hkv][HD], `vs` [Hkv][HD][cap], as the rotary/append kernel writes them): m = q.k in scaled log2 units, l = 1,
// O = v.  One wavefront per (row, head), four heads per workgroup.
template <int HD>
__global__ __launch_bounds__(256) void attn_self_slice_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ ks,
                                                              const bf16_t* __restrict__ vs, int cap, int M, int Hq, int Hkv,
                                                              float scale_log2, float* __restrict__ part_o,
                                                              float* __restrict__ part_ml, int nsplit, int split) {
  constexpr int PER = HD / 64;
  const int m = blockIdx.x, h = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (h >= Hq) return;
  const int hk = h / (Hq / Hkv), e = lane * PER;
  float dot = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i)
    dot += bf16_to_float(q[((size_t)m * Hq + h) * HD + e + i]) * bf16_to_float(ks[((size_t)m * Hkv + hk) * HD + e + i]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
  const size_t idx = ((size_t)h * nsplit + split) * M + m;
#pragma unroll
  for (int i = 0; i < PER; ++i) part_o[idx * HD + e + i] = bf16_to_float(vs[((size_t)hk * HD + e + i) * cap + m]);
  if (lane == 0) {
    part_ml[idx * 2] = dot * scale_log2;
    part_ml[idx * 2 + 1] = 1.0f;
  }
}

// Work split.  M <= 16 rows (decode steps, pseudo rows): one row block, the four wavefronts of a workgroup
// split the keys of the slice and fragments come straight from global memory.  More rows: the tile kernel,
// each wavefront owning 16 rows (two row groups of workgroups above 64 rows).
struct AttnPlan { int qb, waves, groups, nsplit; bool tiled; int ring_waves; };

AttnPlan plan_attention(int M, int Hq, int Hkv, int S) {
  AttnPlan p;
  p.tiled = M > 16;
  p.qb = 1;                                       // 32 rows per wavefront measured slower (one wave per SIMD)
  p.waves = 4;
  p.ring_waves = 0;
  p.groups = p.tiled ? (M + p.waves * p.qb * 16 - 1) / (p.waves * p.qb * 16) : 1;
  const int units = p.tiled ? (S + 63) / 64 : (S + 31) / 32;     // tiles or chunks
  // Long key ranges, or query heads that share key/value heads: the ring kernel (measured at 128-wide heads, 64 rows:
  // 40 heads over 2112 keys 14.2 -> 13.2 us, 64 query on 8 key/value heads over 4160 keys 25.1 -> 20.7 us; 128 rows
  // of 32 heads over 4224 keys 23.7 -> 22.8 us; over 576 keys the tile kernel stays ahead, 7.0 against 7.3 us).  Its
  // three-tile ring fills the LDS of a compute unit, so the slices are cut for one workgroup per unit.
  // With four or more query heads per key/value head it also takes the passes of up to 16 rows (one-token step, draft
  // rows), whose own kernel streams the tiles once per query head.
  const int blocks = (Hq / Hkv) * ((M + 15) / 16);
  const int tiles = (S + 63) / 64;
  if (tiles >= 24 && M <= 128 && (p.tiled || Hq / Hkv >= 4)) {
    const int units = tiles;
    p.ring_waves = 4;      // eight wavefronts on half as many workgroups run as fast, but double the slices to merge
    p.groups = (blocks + p.ring_waves - 1) / p.ring_waves;
    int s = 256 / (Hkv * p.groups);
    if (s > units / 2) s = units / 2;
    if (s > kMaxSplits) s = kMaxSplits;
    p.nsplit = s < 1 ? 1 : s;
    return p;
  }
  int s = (512 + Hq * p.groups - 1) / (Hq * p.groups);           // about two workgroups per compute unit
  // per slice: every wavefront has work; slices of under four tiles only pay off on short caches (measured)
  const int min_units = !p.tiled ? 4 : (units >= 16 ? 4 : 2);
  if (s > units / min_units) s = units / min_units;
  if (s > kMaxSplits) s = kMaxSplits;
  if (s < 1) s = 1;
  p.nsplit = s;
  return p;
}

// The ring's LDS is more than a kernel may use without asking: asked for once per device (attn_mfma_prepare does it
// when a model is set up, so that no launch inside a stream capture has to).
template <int HD, int NCW>
hipError_t allow_ring_lds() {
  static bool allowed[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!allowed[dev]) {
    e = hipFuncSetAttribute((const void*)attn_ring_kernel<HD, NCW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            RingShape<HD>::LDS_BYTES);
    if (e != hipSuccess) return e;
    allowed[dev] = true;
  }
  return hipSuccess;
}

template <int HD, int NCW>
hipError_t launch_ring(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int cap, int n, int M, const uint64_t* anc, int Hq,
                       int Hkv, bf16_t* out, float* part_o, float* part_ml, const AttnPlan& p, float scale_log2, hipStream_t s,
                       const int32_t* n_dev) {
  constexpr int lds = RingShape<HD>::LDS_BYTES;            // above the 64 KB a kernel may use without asking
  const hipError_t ea = allow_ring_lds<HD, NCW>();
  if (ea != hipSuccess) return ea;
  hipLaunchKernelGGL((attn_ring_kernel<HD, NCW>), dim3(Hkv, p.groups, p.nsplit), dim3(64 * (NCW + 1)), lds, s, q, kc, vc, cap, n,
                     M, anc, Hq, Hkv, out, part_o, part_ml, p.nsplit, scale_log2, n_dev);
  return hipSuccess;
}

template <int HD>
hipError_t launch_hd(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int cap, int n, int M, const uint64_t* anc, int Hq,
                     int Hkv, bf16_t* out, void* scratch, const AttnPlan& p, hipStream_t s, const int32_t* n_dev) {
  float* part_o = (float*)scratch;
  float* part_ml = part_o + (size_t)Hq * kMaxSplits * M * HD;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  const dim3 grid(Hq, p.groups, p.nsplit);
#define HT_ATTN_ARGS q, kc, vc, cap, n, M, anc, Hq, Hkv, out, part_o, part_ml, p.nsplit, scale_log2, n_dev
  if (p.ring_waves) {
    const hipError_t e = launch_ring<HD, 4>(q, kc, vc, cap, n, M, anc, Hq, Hkv, out, part_o, part_ml, p, scale_log2, s, n_dev);
    if (e != hipSuccess) return e;
  } else if (!p.tiled) {
    hipLaunchKernelGGL((attn_mfma_kernel<HD, 1>), grid, dim3(256), 0, s, HT_ATTN_ARGS);
  } else {
    hipLaunchKernelGGL((attn_tile_kernel<HD, 1, 4>), grid, dim3(256), 0, s, HT_ATTN_ARGS, 0);
  }
#undef HT_ATTN_ARGS
  if (p.nsplit > 1)
    hipLaunchKernelGGL((attn_merge_kernel<HD>), dim3((M + 256 / (HD / 4) - 1) / (256 / (HD / 4)), Hq), dim3(256), 0, s,
                       part_o, part_ml, p.nsplit, M, Hq, out);
  return hipSuccess;
}

}  // namespace

bool attn_mfma_supported(int M, int Hq, int Hkv, int hd) {
  return (hd == 64 || hd == 128) && M >= 1 && M <= kMaxRows && Hq % Hkv == 0;
}

hipError_t attn_mfma_prepare(int hd) {
  if (hd == 128) return allow_ring_lds<128, 4>();
  if (hd == 64) return allow_ring_lds<64, 4>();
  return hipSuccess;
}

// A causal sequence of `rows` rows whose K/V are in the cache already (slot = position): row r sees the keys 0 .. r.
// One launch of the tile kernel, rows attending in chunks of kCausalChunk, a workgroup per (query head, 64 rows), every
// workgroup over all its keys.  `tree` holds the masks of a chain of at least kCausalChunk rows.
// With `self_k` / `self_v` ([rows][Hkv][hd] and [Hkv][hd][self_cap]) row r sees the keys 0 .. r of the cache and, on
// top, the key and value of its own row in those buffers: the cache part and the own part meet in the merge kernel
// (`scratch`: attn_causal_scratch_bytes).
namespace {
constexpr int kCausalChunk = 128;
template <int HD>
hipError_t launch_causal_hd(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int cap, int rows, const uint64_t* anc, int Hq,
                            int Hkv, bf16_t* out, const bf16_t* self_k, const bf16_t* self_v, int self_cap, void* scratch,
                            hipStream_t s) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  const dim3 grid(Hq, (rows + 63) / 64, 1);
  if (!self_k) {
    hipLaunchKernelGGL((attn_tile_kernel<HD, 1, 4>), grid, dim3(256), 0, s, q, kc, vc, cap, 0, rows, anc, Hq, Hkv, out,
                       nullptr, nullptr, 1, scale_log2, nullptr, kCausalChunk);
    return hipGetLastError();
  }
  float* part_o = (float*)scratch;
  float* part_ml = part_o + (size_t)Hq * 2 * rows * HD;
  hipLaunchKernelGGL((attn_tile_kernel<HD, 1, 4>), grid, dim3(256), 0, s, q, kc, vc, cap, 0, rows, anc, Hq, Hkv, out, part_o,
                     part_ml, 2, scale_log2, nullptr, kCausalChunk);
  hipLaunchKernelGGL((attn_self_slice_kernel<HD>), dim3(rows, (Hq + 3) / 4), dim3(256), 0, s, q, self_k, self_v, self_cap, rows,
                     Hq, Hkv, scale_log2, part_o, part_ml, 2, 1);
  hipLaunchKernelGGL((attn_merge_kernel<HD>), dim3((rows + 256 / (HD / 4) - 1) / (256 / (HD / 4)), Hq), dim3(256), 0, s, part_o,
                     part_ml, 2, rows, Hq, out);
  return hipGetLastError();
}
}  // namespace

size_t attn_causal_scratch_bytes(int rows, int Hq, int hd) {
  return ((size_t)Hq * 2 * rows * hd + (size_t)Hq * 2 * rows * 2) * sizeof(float) + 256;
}

hipError_t launch_attn_causal(const void* q, const void* kc, const void* vc, int cap, int rows, TreeDev tree, int Hq, int Hkv,
                              int hd, void* out, hipStream_t s, const void* self_k, const void* self_v, int self_cap,
                              void* scratch) {
  if ((size_t)cap * Hkv * hd >= ((size_t)1 << 31) || rows < 1 || rows > cap) return hipErrorInvalidValue;
  if ((self_k != nullptr) != (self_v != nullptr) || (self_k && (!scratch || self_cap < rows))) return hipErrorInvalidValue;
  const bf16_t *qp = (const bf16_t*)q, *kp = (const bf16_t*)kc, *vp = (const bf16_t*)vc;
  if (hd == 128)
    return launch_causal_hd<128>(qp, kp, vp, cap, rows, tree.anc, Hq, Hkv, (bf16_t*)out, (const bf16_t*)self_k,
                                 (const bf16_t*)self_v, self_cap, scratch, s);
  if (hd == 64)
    return launch_causal_hd<64>(qp, kp, vp, cap, rows, tree.anc, Hq, Hkv, (bf16_t*)out, (const bf16_t*)self_k,
                                (const bf16_t*)self_v, self_cap, scratch, s);
  return hipErrorInvalidValue;
}

size_t attn_mfma_scratch_bytes(int M, int Hq, int hd) {
  return ((size_t)Hq * kMaxSplits * M * hd + (size_t)Hq * kMaxSplits * M * 2) * sizeof(float) + 256;
}

hipError_t launch_attn_mfma(const void* q, const void* kc, const void* vc, int cap, int n, int M, TreeDev tree, int Hq,
                            int Hkv, int hd, void* out, void* scratch, hipStream_t s, const int32_t* n_dev) {
  if ((size_t)cap * Hkv * hd >= ((size_t)1 << 31)) return hipErrorInvalidValue;   // 32-bit element offsets inside a cache
  const AttnPlan p = plan_attention(M, Hq, Hkv, n + M);
  const bf16_t *qp = (const bf16_t*)q, *kp = (const bf16_t*)kc, *vp = (const bf16_t*)vc;
  const hipError_t e = hd == 128 ? launch_hd<128>(qp, kp, vp, cap, n, M, tree.anc, Hq, Hkv, (bf16_t*)out, scratch, p, s, n_dev)
                                 : launch_hd<64>(qp, kp, vp, cap, n, M, tree.anc, Hq, Hkv, (bf16_t*)out, scratch, p, s, n_dev);
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace ht
