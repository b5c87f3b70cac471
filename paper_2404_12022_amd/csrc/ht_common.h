// Internal declarations shared by the HIP sources of libht (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace ht {

typedef uint16_t bf16_t;   // raw bfloat16 bits

__host__ __device__ inline float bf16_to_float(bf16_t v) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)v << 16;
  return c.f;
}
// round-to-nearest-even; NaN stays NaN
__host__ __device__ inline bf16_t float_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40u);
  c.u += 0x7fffu + ((c.u >> 16) & 1u);
  return (bf16_t)(c.u >> 16);
}

// Four floats to four bf16 (8 bytes) with the gfx950 pair conversion (round-to-nearest-even, NaN stays NaN: the same
// values as float_to_bf16).
__device__ inline uint2 pack4_bf16(float a, float b, float c, float d) {
  typedef float f2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 b2_t __attribute__((ext_vector_type(2)));
  const b2_t lo = __builtin_convertvector(f2_t{a, b}, b2_t), hi = __builtin_convertvector(f2_t{c, d}, b2_t);
  uint2 r;
  r.x = *(const uint32_t*)&lo;
  r.y = *(const uint32_t*)&hi;
  return r;
}

// Share `total` items over `parts` owners as evenly as possible: owner i gets [lo, hi), the first total % parts
// owners one item more.  One 32-bit division (a 64-bit one is a few hundred instructions in front of a kernel's
// first load).
__device__ inline void even_share(unsigned total, unsigned parts, unsigned i, int& lo, int& hi) {
  const unsigned q = total / parts, rem = total - q * parts;
  lo = (int)(i * q + (i < rem ? i : rem));
  hi = lo + (int)q + (i < rem ? 1 : 0);
}

template <typename T> struct Conv;
template <> struct Conv<float> {
  __device__ static inline float load(const float* p) { return *p; }
  __device__ static inline void store(float* p, float v) { *p = v; }
};
template <> struct Conv<bf16_t> {
  __device__ static inline float load(const bf16_t* p) { return bf16_to_float(*p); }
  __device__ static inline void store(bf16_t* p, float v) { *p = float_to_bf16(v); }
};

constexpr int kMaxTree = 128;            // nodes of a tree (root included)
constexpr int kMaxRows = 256;            // rows of a pass: tree nodes plus the pseudo rows that ride along, or a prefill chunk
constexpr int kMaskWords = kMaxRows / 64;
constexpr int kMaxTopK = 64;
constexpr int kMaxTransfer = 8;
constexpr int kMaxSplitK = 8;
constexpr int kMaxLoopSteps = 64;        // steps per call of the device-resident loop

// Tree tables as the kernels see them (device pointers).
struct TreeDev {
  const int32_t* parent;     // [T]
  const int32_t* depth;      // [T]
  const int32_t* rank;       // [T]
  const uint64_t* anc;       // [rows][kMaskWords] bit u set iff row u is the row itself or an ancestor of it
};

// Device-resident decoder state written by the accept kernel and read back by the host.
struct StepState {
  int32_t root;                              // pending root token
  int32_t m;                                 // accepted count of the last step
  int32_t next_root;
  int32_t path[kMaxTransfer + 1];
  int32_t emitted[kMaxTransfer + 1];
  // device-resident loop (ht_decode_steps): cache length before / after the last acceptance, steps logged so far
  int32_t n_old, n, log_count;
  int32_t pad[1];
};
// what one step of the device-resident loop leaves for the host
struct StepLog {
  int32_t m;
  int32_t emitted[kMaxTransfer + 1];
};

// Cache length of a pass: kernels take the host's value `n` and, for the device-resident loop, a pointer that
// overrides it (NULL otherwise).  The host value then only has to be an upper bound (it sizes grids and LDS).
__device__ inline int cache_len(int n, const int32_t* n_dev) { return n_dev ? *n_dev : n; }

// One weight operand made of up to three row segments sharing K (Wq|Wk|Wv, Wgate|Wup).
struct WeightSegs {
  const void* w[3];
  int32_t rows[3];
  int32_t nseg;
};

// ------------------------------------------------------------------------------------------------
// launchers (definitions in the .hip files); all enqueue on `s` and return the launch status
// ------------------------------------------------------------------------------------------------
hipError_t launch_embed(int dtype, const void* emb, const int32_t* tok, float* x, int M, int d, hipStream_t s);
hipError_t launch_load_rows(const float* src, float* x, int M, int d, hipStream_t s);
// x[m] += sum_s part[s][m]; optional save; u[m] = rmsnorm(x[m]) * gain
hipError_t launch_add_norm(int dtype, float* x, const float* part, int nsplit, size_t part_stride, const void* gain,
                           void* u, float* save_h, int M, int d, float eps, hipStream_t s);
// The same with kNormParts workgroups per row (d a multiple of 4 kNormParts): each adds and stores its part of the
// row, leaves the sum of squares of that part in ss[m][part] and writes u[m] = x[m] * gain WITHOUT the 1/rms factor;
// the product that consumes u multiplies its output rows by RowScale::of(m) instead (bf16 only).
constexpr int kNormParts = 4;
hipError_t launch_add_norm_parts(float* x, const float* part, int nsplit, size_t part_stride, const void* gain, void* u,
                                 float* save_h, float* ss, int M, int d, hipStream_t s);
// 1 / rms of the rows of an activation panel written by launch_add_norm_parts; ss == NULL: rows are used as they are
struct RowScale {
  const float* ss = nullptr;
  float inv_d = 0.f, eps = 0.f;
};
// depth == NULL: row m sits at position n + m
hipError_t launch_rope_table(float* cs, const int32_t* depth, int n, int M, int hd, float base, hipStream_t s,
                             const int32_t* n_dev = nullptr);
// qkv may be `nsplit` split-K partial sums of [M][(Hq + 2 Hkv) hd] each
hipError_t launch_rope_append(int dtype, const float* qkv, int nsplit, const float* cs, void* q, void* kc, void* vc,
                              int n, int M, int Hq, int Hkv, int hd, int cap, bool paired, hipStream_t s,
                              const int32_t* n_dev = nullptr);
hipError_t launch_rope_append_split(int dtype, const void* q_in, const void* k_in, const void* v_in, const float* cs,
                                    void* q, void* kc, void* vc, int n, int M, int Hq, int Hkv, int hd, int cap,
                                    hipStream_t s);
hipError_t launch_silu_mul(int dtype, const float* gu, void* act, int M, int f, hipStream_t s);
hipError_t launch_argmax(const float* z, int32_t* g, int M, int V, hipStream_t s);
// cand[i] = top width[i % period + 1] entries of logit row src_row[i] (row i when src_row is NULL), i < rows;
// scratch: topk_scratch_bytes(rows) bytes for the per-slice survivors
size_t topk_scratch_bytes(int rows);
hipError_t launch_topk(const float* d, int32_t* cand, const int32_t* width, void* scratch, int rows, int period,
                       const int32_t* src_row, int V, hipStream_t s);
hipError_t launch_tree_build(const StepState* st, const int32_t* cand, TreeDev tree, int32_t* tok, int T, hipStream_t s);
// kl[p] = KL(softmax(z[row_a + p]) || softmax(z[row_b + p])), p < pairs, z rows of V floats (Sec. 3.3 loss term)
hipError_t launch_kl_rows(const float* z, int row_a, int row_b, int pairs, int V, float* kl, hipStream_t s);
// Tree chosen from the draft distributions: lp[k][kMaxTopK] = log-probabilities of the b best candidates of every
// draft row (whole-row log-softmax); then the T - 1 best nodes by (summed lp desc, depth asc, rank path asc) fill
// the tree tables and the token row.  T <= kMaxTree, 1 <= b <= kMaxTopK, 1 <= k <= kMaxTransfer and
// T - 1 <= b + b^2 + .. + b^k are the caller's to check.
struct TreeOut {
  int32_t *parent, *depth, *rank;
  uint64_t* anc;
};
hipError_t launch_cand_logprob(const float* d, const int32_t* cand, int rows, int b, int V, float* lp, hipStream_t s);
hipError_t launch_tree_dynamic(const int32_t* root /*device*/, const int32_t* cand, const float* lp, int k, int b, int T,
                               TreeOut tree, int32_t* tok, hipStream_t s);
// log != NULL (device-resident loop): the step is appended to log[st->log_count++] and st->n_old / st->n advance
hipError_t launch_accept(StepState* st, TreeDev tree, const int32_t* tok, const int32_t* g, int T, hipStream_t s,
                         StepLog* log = nullptr);
hipError_t launch_compact(int dtype, const StepState* st, void* const* kc, void* const* vc, int L, int n, int Hkv,
                          int hd, int cap, const float* saved_h, size_t slot_stride, int slots, float* h_src, int d,
                          hipStream_t s, bool n_from_state = false);
hipError_t launch_prefill_finish(StepState* st, const int32_t* g, const float* saved_h, size_t slot_stride, int slots,
                                 float* h_src, int last, int d, hipStream_t s);
// measurement aid: one pass over `buf` with the weight stream's access pattern; returns the bytes actually read
size_t launch_stream_read(const void* buf, size_t bytes, int groups, uint32_t* sink, hipStream_t s);
double launch_mfma_rate(int form, int iters, uint32_t* sink, hipStream_t s);
// pseudo[f * row_stride + (i - i0)] = W_i h_f for steps i0 <= i < i0 + steps and F sources
// h_f = h + (src_rows ? src_rows[f] : f) * d
hipError_t launch_transfer(int dtype, const float* h, const int32_t* src_rows, int F, const void* const* w_dev,
                           float* pseudo, int i0, int steps, int row_stride, int d, hipStream_t s);
hipError_t launch_convert_to_f32(int dtype, const void* src, float* dst, int n, hipStream_t s);
hipError_t launch_convert_to_bf16(const float* src, void* dst, size_t count, hipStream_t s);
// out[i] = sum_s part[s][i] in the fixed order s = 0, 1, ..
hipError_t launch_reduce_splits(const float* part, int nsplit, size_t stride, float* out, hipStream_t s);

// generic (any dtype, any shape) product: out[s=0][m][n] = sum_k a[m][k] w[n][k]
hipError_t launch_gemm_simple(int dtype, const void* a, WeightSegs w, int M, int N, int K, float* out, hipStream_t s);
// bf16 MFMA product over weights repacked into MFMA-fragment order (see ht_gemm_mfma.hip)
struct PackedW {
  const bf16_t* p;   // fragment-ordered copy
  int32_t N, K, Kp;  // rows (multiple of 16), columns, columns rounded up to packed_cols(K)
};
bool gemm_mfma_supported(int M, int N, int K);
int packed_cols(int K);
size_t packed_weight_bytes(int N, int K);
int gemm_mfma_splits(int M, int N, int K);
// mode 0: row blocks in natural order over the concatenated segments; mode 1: two equal segments
// interleaved block by block (gate block i, up block i, gate block i+1, ..); mode 2: segments (q, k, v), in
// every q and k head the 16-row block p is followed by its rotary partner block p + head_dim/32
hipError_t launch_repack(WeightSegs w, int K, int mode, int head_dim, void* dst, hipStream_t s);
// out[s][m][n], s < nsplit (split-K partial sums, fp32).  M <= kMaxRows; more than 128 rows run as two launches over
// the same weights (rows 0..127, then the rest).
hipError_t launch_gemm_packed(const void* a, PackedW w, int M, float* out, int nsplit, hipStream_t s,
                              RowScale rs = RowScale{});
// w packed with mode 1 from (gate, up): act[m][j] = silu(a.gate_j) * (a.up_j), bf16 [M][N/2]
hipError_t launch_gemm_packed_silu(const void* a, PackedW w, int M, void* act, hipStream_t s, RowScale rs = RowScale{});
// w packed with mode 2 from (q, k, v): rotary at the row's position, q rows to `q`, k/v rows appended to the
// caches at slot n + m (all bf16); cs is the (cos, sin) table [M][hd/2]
struct QkvEpilogue {
  const float* cs;
  bf16_t *q, *kc, *vc;
  int32_t n, Hq, Hkv, hd, cap;
  const int32_t* n_dev = nullptr;            // overrides n when set (device-resident loop)
};
// The same products tiled over the tokens too, for passes of any number of rows (the batched forward pass of the
// training stage): one launch, no K split.  out: fp32 [M][N]; act: bf16 [M][N/2] (w packed from (gate, up)).
hipError_t launch_gemm_wide(const void* a, PackedW w, int M, float* out, hipStream_t s, RowScale rs = RowScale{});
hipError_t launch_gemm_wide_silu(const void* a, PackedW w, int M, void* act, hipStream_t s, RowScale rs = RowScale{});
bool qkv_fusable(int head_dim);
bool qkv_prefer_split(int M, int N);
hipError_t launch_gemm_packed_qkv(const void* a, PackedW w, int M, QkvEpilogue qe, hipStream_t s,
                                  RowScale rs = RowScale{});

// attention over cache + tree rows; out[m][h*hd+e] in dtype
hipError_t launch_attn_simple(int dtype, const void* q, const void* kc, const void* vc, int cap, int n, int M,
                              TreeDev tree, int Hq, int Hkv, int hd, void* out, hipStream_t s,
                              const int32_t* n_dev = nullptr);
bool attn_mfma_supported(int M, int Hq, int Hkv, int hd);
size_t attn_mfma_scratch_bytes(int M, int Hq, int hd);
// once per device before the first launch that may sit inside a stream capture (kernel attributes)
hipError_t attn_mfma_prepare(int hd);
hipError_t launch_attn_mfma(const void* q, const void* kc, const void* vc, int cap, int n, int M, TreeDev tree, int Hq,
                            int Hkv, int hd, void* out, void* scratch, hipStream_t s, const int32_t* n_dev = nullptr);
hipError_t launch_attn_causal(const void* q, const void* kc, const void* vc, int cap, int rows, TreeDev tree, int Hq, int Hkv,
                              int hd, void* out, hipStream_t s, const void* self_k = nullptr, const void* self_v = nullptr,
                              int self_cap = 0, void* scratch = nullptr);
size_t attn_causal_scratch_bytes(int rows, int Hq, int hd);

}  // namespace ht
