// C ABI of libht: argument validation, workspace carving and the order in which the kernels of one
// decode step are enqueued.  All arithmetic lives in the kernels; nothing here touches tensor data
// on the host.
#include "../../include/ht.h"
#include "ht_common.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

using namespace ht;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HT_HIP(expr)                                                                              \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return fail(HT_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

size_t elem_size(int dtype) { return dtype == HT_F32 ? 4 : 2; }
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int padded_rows(int M) { return M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : M <= 128 ? 128 : 256; }

// Bump allocator over the workspace; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T> T* take(size_t count) {
    off = align_up(off, 256);
    T* p = base ? (T*)(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
  void* take_bytes(size_t bytes) { return take<char>(bytes); }
};

struct TreeTables {
  int32_t *parent, *depth, *rank;
  uint64_t* anc;
  TreeDev dev() const { return TreeDev{parent, depth, rank, anc}; }
  TreeOut out() const { return TreeOut{parent, depth, rank, anc}; }
};

struct Buffers {
  float* x;            // residual stream [Mp, d]
  void* u;             // normalised rows (dtype) [Mp, d]
  float* qkv;          // [Mp, (Hq + 2 Hkv) hd]
  void* q;             // rotated queries (dtype) [Mp, Hq hd]
  void* attn;          // attention output (dtype) [Mp, Hq hd]
  float* gu;           // gate | up [Mp, 2 f]
  void* act;           // silu(gate) * up (dtype) [Mp, f]
  float* part;         // split-K partial sums [kMaxSplitK][Mp][d]
  float* logits;       // [Mp, V]
  float* dlogits;      // draft logits [k, V]
  float* saved_h;      // residuals of the last verify pass at every distinct transfer layer [slots <= k][Mp, d]
  float* h_src;        // transfer sources [slots][d]
  float* pseudo;       // [k, d]
  float* cs;           // rotary table [Mp, hd/2] (cos, sin)
  float* ss;           // packed path: sums of squares of the rows of u, kNormParts parts per row [Mp][kNormParts]
  float* kl;           // training forward: KL term per position [max_cache]
  int32_t* train_rows; // training forward: source row of every pseudo row of the pass [kMaxTree]
  float* lp;           // log-probabilities of the candidates of the last draft [kMaxTransfer][kMaxTopK] (dynamic tree)
  int32_t *tok, *g, *cand, *width, *prompt;
  int32_t* fused_rows;   // tree nodes that get pseudo rows inside the verify pass [kMaxTree]
  int32_t* cand_fused;   // their candidates [fused node][k][kMaxTopK], at most kMaxRows (node, step) pairs
  int32_t* fused_src;    // logits row (past the tree rows) that holds the draft of (fused node, step) [kMaxRows]
  TreeTables tree, chain, train;   // the decoding tree; a chain (prefill, draft pass); the rows of a training pass
  StepState* state;
  StepLog* log;        // steps of the device-resident loop [kMaxLoopSteps]
  void** kc_ptrs;      // device array [L]
  void** vc_ptrs;
  void** wt_ptrs;      // device array [k]
  void* attn_scratch;
  void* topk_scratch;
  std::vector<void*> kc, vc;   // host copies of the per-layer cache pointers
  // bf16 only: projection weights repacked into MFMA-fragment order
  std::vector<PackedW> p_qkv, p_o, p_gu, p_down;
  PackedW p_head;
};

bool shapes_packable(const ht_config& c) {
  const int qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
  return c.dtype == HT_BF16 && qd % 16 == 0 && kvd % 16 == 0 && c.d_model % 16 == 0 && c.d_ffn % 16 == 0 &&
         c.vocab % 16 == 0;
}

void carve(const ht_config& c, Carver& cv, Buffers& b) {
  const size_t es = elem_size(c.dtype);
  const size_t Mp = padded_rows(c.max_tree > c.k ? c.max_tree : c.k);
  const size_t d = c.d_model, qd = (size_t)c.n_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim;
  b.x = cv.take<float>(Mp * d);
  b.u = cv.take_bytes(Mp * d * es);
  b.qkv = cv.take<float>((size_t)kMaxSplitK * Mp * (qd + 2 * kvd));
  b.q = cv.take_bytes(Mp * qd * es);
  b.attn = cv.take_bytes(Mp * qd * es);
  b.gu = cv.take<float>(Mp * 2 * c.d_ffn);
  b.act = cv.take_bytes(Mp * c.d_ffn * es);
  b.part = cv.take<float>((size_t)kMaxSplitK * Mp * d);
  b.logits = cv.take<float>(Mp * c.vocab);
  b.dlogits = cv.take<float>((size_t)padded_rows(c.k) * c.vocab);
  b.saved_h = cv.take<float>((size_t)c.k * Mp * d);
  b.h_src = cv.take<float>((size_t)c.k * d);
  b.pseudo = cv.take<float>((size_t)c.k * d);
  b.cs = cv.take<float>(Mp * c.head_dim);
  b.ss = cv.take<float>(Mp * kNormParts);
  b.lp = cv.take<float>((size_t)kMaxTransfer * kMaxTopK);
  b.kl = cv.take<float>(c.max_cache);
  b.train_rows = cv.take<int32_t>(kMaxTree);
  b.tok = cv.take<int32_t>(Mp);
  b.g = cv.take<int32_t>(Mp);
  b.cand = cv.take<int32_t>((size_t)kMaxTransfer * kMaxTopK);
  b.width = cv.take<int32_t>(kMaxTransfer + 2);
  b.prompt = cv.take<int32_t>(c.max_cache);
  b.fused_rows = cv.take<int32_t>(kMaxTree);
  b.cand_fused = cv.take<int32_t>((size_t)kMaxRows * kMaxTopK);
  b.fused_src = cv.take<int32_t>(kMaxRows);
  for (TreeTables* t : {&b.tree, &b.chain, &b.train}) {
    t->parent = cv.take<int32_t>(kMaxRows);
    t->depth = cv.take<int32_t>(kMaxRows);
    t->rank = cv.take<int32_t>(kMaxRows);
    t->anc = cv.take<uint64_t>((size_t)kMaxRows * kMaskWords);
  }
  b.state = cv.take<StepState>(1);
  b.log = cv.take<StepLog>(kMaxLoopSteps);
  b.kc_ptrs = cv.take<void*>(c.n_layers);
  b.vc_ptrs = cv.take<void*>(c.n_layers);
  b.wt_ptrs = cv.take<void*>(kMaxTransfer);
  b.topk_scratch = cv.take_bytes(topk_scratch_bytes(kMaxRows));
  b.attn_scratch = cv.take_bytes(attn_mfma_scratch_bytes((int)Mp, c.n_heads, c.head_dim));
  b.kc.resize(c.n_layers);
  b.vc.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    b.kc[l] = cv.take_bytes((size_t)c.max_cache * kvd * es);
    b.vc[l] = cv.take_bytes((size_t)c.max_cache * kvd * es);
  }
  if (shapes_packable(c)) {
    auto pk = [&](int N, int K) {
      return PackedW{(const bf16_t*)cv.take_bytes(packed_weight_bytes(N, K)), N, K, packed_cols(K)};
    };
    b.p_qkv.resize(c.n_layers);
    b.p_o.resize(c.n_layers);
    b.p_gu.resize(c.n_layers);
    b.p_down.resize(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
      b.p_qkv[l] = pk((int)(qd + 2 * kvd), (int)d);
      b.p_o[l] = pk((int)d, (int)qd);
      b.p_gu[l] = pk(2 * c.d_ffn, (int)d);
      b.p_down[l] = pk((int)d, c.d_ffn);
    }
    b.p_head = pk(c.vocab, (int)d);
  }
}

int check_config(const ht_config* c) {
  if (!c) return fail(HT_EINVAL, "config is NULL");
  if (c->n_layers < 2 || c->d_model < 8 || c->n_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 || c->d_ffn < 8 ||
      c->vocab < 2)
    return fail(HT_EINVAL, "non-positive or too small model dimension");
  if (c->dtype != HT_F32 && c->dtype != HT_BF16) return fail(HT_EINVAL, "dtype must be HT_F32 or HT_BF16");
  if (c->n_heads % c->n_kv_heads) return fail(HT_EINVAL, "n_heads must be a multiple of n_kv_heads");
  if (c->head_dim % 2 || c->head_dim > 256) return fail(HT_EINVAL, "head_dim must be even and <= 256");
  if (c->d_model % 8 || c->d_ffn % 8 || (c->n_heads * c->head_dim) % 8)
    return fail(HT_EINVAL, "d_model, d_ffn and n_heads*head_dim must be multiples of 8");
  if (c->k < 1 || c->k > HT_MAX_TRANSFER) return fail(HT_EINVAL, "k must be in 1..%d", HT_MAX_TRANSFER);
  for (int i = 0; i < c->k; ++i) {
    if (c->transfer_layer[i] < 1 || c->transfer_layer[i] >= c->n_layers)
      return fail(HT_EINVAL, "transfer_layer[%d]=%d outside 1..n_layers-1", i, c->transfer_layer[i]);
    if (i && c->transfer_layer[i] < c->transfer_layer[i - 1])
      return fail(HT_EINVAL, "transfer layers must not decrease (t_1 <= t_2 <= ..)");
  }
  if (c->max_tree < 1 || c->max_tree > HT_MAX_ROWS) return fail(HT_EINVAL, "max_tree must be in 1..%d", HT_MAX_ROWS);
  if (c->max_cache < 8 || c->max_cache % 8) return fail(HT_EINVAL, "max_cache must be a positive multiple of 8");
  if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return fail(HT_EINVAL, "rms_eps must be > 0 and rope_base > 1");
  return HT_OK;
}

}  // namespace

struct ht_model {
  ht_config cfg;
  const void *tok_emb, *final_norm, *lm_head;
  std::vector<const void*> attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down, w_transfer;
  Buffers b;
  int Mp = 0;
  int n = 0;
  int T = 0;
  bool has_tree = false, has_prefill = false, transfer_ready = false, verify_done = false;
  bool use_mfma = true;
  bool packed = false;          // bf16 projections run on the repacked weights
  bool qkv_fused = false;       // rotary + KV append run in the QKV projection's epilogue
  std::vector<char> layer_loaded;   // packed copy of each layer present
  bool head_loaded = false;
  std::vector<int32_t> depth, parent, rank;
  // transfer steps grouped by layer (Sec. 3.2: step i reads the hidden state of layer t_i): slot g covers steps
  // slot_first[g] .. slot_first[g] + slot_count[g] - 1, all at layer slot_layer[g]; slot_of_layer[l] = g or -1
  std::vector<int> slot_layer, slot_first, slot_count, slot_of_layer;
  std::vector<int32_t> fused;   // tree nodes with pseudo rows in the verify pass (empty: draft after accept only)
  int drafts_of = -1;           // index into `fused` of the node the last acceptance ended on, -1 if none
  int dyn_b = 0;                // > 0: every drafting step chooses its own tree among the dyn_b best candidates per level
  // pinned host staging
  int32_t* h_stage = nullptr;     // [max(max_cache, two table images)] + the pointer tables
  StepState* h_state = nullptr;
  // device-resident loop: while set, the kernels of a pass read the cache length here and `n` is an upper bound
  const int32_t* n_dev = nullptr;
};

namespace {

int product(ht_model* m, const void* a, WeightSegs w, int M, int N, int K, float* out, hipStream_t s) {
  HT_HIP(launch_gemm_simple(m->cfg.dtype, a, w, M, N, K, out, s));
  return HT_OK;
}

WeightSegs segs1(const void* w0, int r0) { return WeightSegs{{w0, nullptr, nullptr}, {r0, 0, 0}, 1}; }

int attention(ht_model* m, int layer, int n, int M, const TreeDev& tree, hipStream_t s) {
  const ht_config& c = m->cfg;
  Buffers& b = m->b;
  if (c.dtype == HT_BF16 && m->use_mfma && attn_mfma_supported(M, c.n_heads, c.n_kv_heads, c.head_dim)) {
    HT_HIP(launch_attn_mfma(b.q, b.kc[layer], b.vc[layer], c.max_cache, n, M, tree, c.n_heads, c.n_kv_heads, c.head_dim,
                            b.attn, b.attn_scratch, s, m->n_dev));
  } else {
    HT_HIP(launch_attn_simple(c.dtype, b.q, b.kc[layer], b.vc[layer], c.max_cache, n, M, tree, c.n_heads, c.n_kv_heads,
                              c.head_dim, b.attn, s, m->n_dev));
  }
  return HT_OK;
}

// Rows that join a pass on its way up.  kFromTree: under each of F tree nodes (b.fused_rows) the pseudo rows of
// every transfer step, W_i applied to the node's residual at layer t_i (Sec. 3.2), created when the pass reaches
// t_i: verification and the next candidates then come out of one forward (Fig. 2 caption, Sec. 3.4).
// kFromBuffer: the k rows of b.pseudo (draft pass after acceptance), row i joining at layer t_i.
// kTrainStep: one pseudo row per listed row (b.train_rows), made by the map of transfer step `step` alone when the
// pass reaches that step's layer (training stage, Sec. 3.3).
enum JoinMode { kNoJoin = 0, kFromTree = 1, kFromBuffer = 2, kTrainStep = 3 };

// Rows already in b.x (M of them, possibly none) go through blocks layer_from+1 .. L (0-based index
// layer_from .. L-1) together with the rows that join on the way, then the final norm and, if `logits` is given,
// the LM head and the row arg-max.  `tree` must describe all rows the pass ends with.
// layer_end >= 0: the pass stops after block layer_end (0-based index layer_end - 1) and leaves the finished residual
// rows in b.x (no final norm, no logits).
int run_pass(ht_model* m, const TreeDev& tree, int M, int layer_from, bool save_hidden, float* logits, int32_t* gout,
             hipStream_t s, JoinMode join = kNoJoin, int F = 0, int step = 0, int layer_end = -1) {
  const ht_config& c = m->cfg;
  Buffers& b = m->b;
  const int d = c.d_model, qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, f = c.d_ffn;
  const size_t es = elem_size(c.dtype), slot_stride = (size_t)m->Mp * d;
  size_t pstride = (size_t)M * d;
  const int n = m->n;
  int rc;
  const int joining = join == kFromTree ? F * c.k : join == kFromBuffer ? c.k : join == kTrainStep ? F : 0;
  HT_HIP(launch_rope_table(b.cs, tree.depth, n, M + joining, c.head_dim, c.rope_base, s, m->n_dev));
  int pending = 0;
  // Residual add + RMSNorm.  On packed weights the row is split over kNormParts workgroups (one workgroup per row
  // takes in its 80 KB at the pace of a single compute unit) and the 1/rms factor moves into the epilogue of the
  // product that reads u; everywhere else one workgroup normalises the whole row.
  const bool parts = m->packed && d % (4 * kNormParts) == 0;
  const RowScale rs = parts ? RowScale{b.ss, 1.0f / (float)d, c.rms_eps} : RowScale{};
  auto add_norm = [&](float* x, int nsplit, size_t stride, const void* gain, void* u, float* save, float* ss, int rows) {
    return parts ? launch_add_norm_parts(x, b.part, nsplit, stride, gain, u, save, ss, rows, d, s)
                 : launch_add_norm(c.dtype, x, b.part, nsplit, stride, gain, u, save, rows, d, c.rms_eps, s);
  };
  const int layer_stop = layer_end >= 0 ? layer_end : c.n_layers;
  for (int l = layer_from; l < layer_stop; ++l) {
    const int slot = m->slot_of_layer[l];
    if (M > 0) {
      float* save = (save_hidden && slot >= 0) ? b.saved_h + slot * slot_stride : nullptr;
      HT_HIP(add_norm(b.x, pending, pstride, m->attn_norm[l], b.u, save, b.ss, M));
    }
    if (join == kTrainStep) {
      if (l == c.transfer_layer[step]) {
        HT_HIP(launch_transfer(c.dtype, b.x, b.train_rows, F, (const void* const*)b.wt_ptrs, b.x + (size_t)M * d, step, 1,
                               1, d, s));
        HT_HIP(add_norm(b.x + (size_t)M * d, 0, 0, m->attn_norm[l], (char*)b.u + (size_t)M * d * es, nullptr,
                        b.ss + (size_t)M * kNormParts, F));
        M += F;
        pstride = (size_t)M * d;
      }
    } else if (join != kNoJoin && slot >= 0) {
      // the residual after l blocks is complete now: make the rows of this layer's transfer steps, normalise
      // them, go on wider
      const int i0 = m->slot_first[slot], cnt = m->slot_count[slot];
      int extra;
      if (join == kFromTree) {
        extra = F * cnt;                  // row of (node f, step i) = M + f * cnt + (i - i0)
        HT_HIP(launch_transfer(c.dtype, b.x, b.fused_rows, F, (const void* const*)b.wt_ptrs, b.x + (size_t)M * d, i0, cnt,
                               cnt, d, s));
      } else {
        extra = cnt;
        HT_HIP(launch_load_rows(b.pseudo + (size_t)i0 * d, b.x + (size_t)M * d, cnt, d, s));
      }
      HT_HIP(add_norm(b.x + (size_t)M * d, 0, 0, m->attn_norm[l], (char*)b.u + (size_t)M * d * es, nullptr,
                      b.ss + (size_t)M * kNormParts, extra));
      M += extra;
      pstride = (size_t)M * d;
    }
    if (M == 0) continue;
    if (m->qkv_fused && !qkv_prefer_split(M, qd + 2 * kvd)) {
      QkvEpilogue qe{b.cs, (bf16_t*)b.q, (bf16_t*)b.kc[l], (bf16_t*)b.vc[l], n, c.n_heads, c.n_kv_heads, c.head_dim,
                     c.max_cache, m->n_dev};
      HT_HIP(launch_gemm_packed_qkv(b.u, b.p_qkv[l], M, qe, s, rs));
    } else {
      int qsplit = 1;
      if (m->packed) {
        qsplit = gemm_mfma_splits(M, qd + 2 * kvd, d);
        HT_HIP(launch_gemm_packed(b.u, b.p_qkv[l], M, b.qkv, qsplit, s, rs));
      } else {
        WeightSegs qkv{{m->wq[l], m->wk[l], m->wv[l]}, {qd, kvd, kvd}, 3};
        if ((rc = product(m, b.u, qkv, M, qd + 2 * kvd, d, b.qkv, s))) return rc;
      }
      // weights packed for the fused epilogue keep their rotary-pair column order in the plain product's output
      HT_HIP(launch_rope_append(c.dtype, b.qkv, qsplit, b.cs, b.q, b.kc[l], b.vc[l], n, M, c.n_heads, c.n_kv_heads,
                                c.head_dim, c.max_cache, m->qkv_fused, s, m->n_dev));
    }
    if ((rc = attention(m, l, n, M, tree, s))) return rc;
    if (m->packed) {
      pending = gemm_mfma_splits(M, d, qd);
      HT_HIP(launch_gemm_packed(b.attn, b.p_o[l], M, b.part, pending, s));
    } else {
      pending = 1;
      if ((rc = product(m, b.attn, segs1(m->wo[l], d), M, d, qd, b.part, s))) return rc;
    }
    HT_HIP(add_norm(b.x, pending, pstride, m->ffn_norm[l], b.u, nullptr, b.ss, M));
    if (m->packed) {
      HT_HIP(launch_gemm_packed_silu(b.u, b.p_gu[l], M, b.act, s, rs));
      pending = gemm_mfma_splits(M, d, f);
      HT_HIP(launch_gemm_packed(b.act, b.p_down[l], M, b.part, pending, s));
    } else {
      WeightSegs gu{{m->w_gate[l], m->w_up[l], nullptr}, {f, f, 0}, 2};
      if ((rc = product(m, b.u, gu, M, 2 * f, d, b.gu, s))) return rc;
      HT_HIP(launch_silu_mul(c.dtype, b.gu, b.act, M, f, s));
      pending = 1;
      if ((rc = product(m, b.act, segs1(m->w_down[l], d), M, d, f, b.part, s))) return rc;
    }
  }
  if (layer_end >= 0) {      // fold the last block's partial sums into the residual and stop (u is scratch here)
    if (pending && M > 0) HT_HIP(add_norm(b.x, pending, pstride, m->attn_norm[layer_end], b.u, nullptr, b.ss, M));
    return HT_OK;
  }
  HT_HIP(add_norm(b.x, pending, pstride, m->final_norm, logits ? b.u : nullptr, nullptr, b.ss, M));
  if (logits) {
    if (m->packed) {
      HT_HIP(launch_gemm_packed(b.u, b.p_head, M, logits, 1, s, rs));      // vocab-sized N: never split
    } else if ((rc = product(m, b.u, segs1(m->lm_head, c.vocab), M, c.vocab, d, logits, s))) {
      return rc;
    }
    if (gout) HT_HIP(launch_argmax(logits, gout, M, c.vocab, s));
  }
  return HT_OK;
}

hipError_t pack_layer(ht_model* m, int l, const void* wq, const void* wk, const void* wv, const void* wo,
                      const void* wg, const void* wu, const void* wd, hipStream_t s) {
  const ht_config& c = m->cfg;
  const int qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, d = c.d_model, f = c.d_ffn;
  hipError_t e = launch_repack(WeightSegs{{wq, wk, wv}, {qd, kvd, kvd}, 3}, d, m->qkv_fused ? 2 : 0, c.head_dim,
                               (void*)m->b.p_qkv[l].p, s);
  if (e == hipSuccess) e = launch_repack(WeightSegs{{wo, nullptr, nullptr}, {d, 0, 0}, 1}, qd, 0, 0, (void*)m->b.p_o[l].p, s);
  if (e == hipSuccess) e = launch_repack(WeightSegs{{wg, wu, nullptr}, {f, f, 0}, 2}, d, 1, 0, (void*)m->b.p_gu[l].p, s);
  if (e == hipSuccess) e = launch_repack(WeightSegs{{wd, nullptr, nullptr}, {d, 0, 0}, 1}, f, 0, 0, (void*)m->b.p_down[l].p, s);
  return e;
}

bool all_loaded(const ht_model* m) {
  for (char c : m->layer_loaded)
    if (!c) return false;
  return m->head_loaded;
}

// host-side tree tables: depth, ancestor-or-self bit masks
void fill_tables(int T, const int32_t* parent, const int32_t* rank, int32_t* stage) {
  int32_t* sp = stage;                       // parent
  int32_t* sd = stage + kMaxRows;            // depth
  int32_t* sr = stage + 2 * kMaxRows;        // rank
  uint64_t* sa = (uint64_t*)(stage + 3 * kMaxRows);
  memset(stage, 0, sizeof(int32_t) * 3 * kMaxRows + sizeof(uint64_t) * kMaxRows * kMaskWords);
  for (int v = 0; v < T; ++v) {
    sp[v] = parent[v];
    sr[v] = rank ? rank[v] : 0;
    sd[v] = v == 0 ? 0 : sd[parent[v]] + 1;
    for (int wd = 0; wd < kMaskWords; ++wd) sa[v * kMaskWords + wd] = v == 0 ? 0 : sa[parent[v] * kMaskWords + wd];
    sa[v * kMaskWords + (v >> 6)] |= 1ull << (v & 63);
  }
}
constexpr size_t kTableInts = 3 * kMaxRows + 2 * kMaxRows * kMaskWords;   // int32 units of one table image

int upload_tables(const TreeTables& t, const int32_t* stage, hipStream_t s) {
  HT_HIP(hipMemcpyAsync(t.parent, stage, sizeof(int32_t) * kMaxRows, hipMemcpyHostToDevice, s));
  HT_HIP(hipMemcpyAsync(t.depth, stage + kMaxRows, sizeof(int32_t) * kMaxRows, hipMemcpyHostToDevice, s));
  HT_HIP(hipMemcpyAsync(t.rank, stage + 2 * kMaxRows, sizeof(int32_t) * kMaxRows, hipMemcpyHostToDevice, s));
  HT_HIP(hipMemcpyAsync(t.anc, stage + 3 * kMaxRows, sizeof(uint64_t) * kMaxRows * kMaskWords, hipMemcpyHostToDevice, s));
  return HT_OK;
}

int validate_tree(int T, const int32_t* parent, const int32_t* rank, int max_depth, int max_T) {
  if (T < 1 || T > max_T) return fail(HT_ETREE, "tree size %d outside 1..%d", T, max_T);
  if (!parent) return fail(HT_EINVAL, "parent is NULL");
  if (parent[0] != -1) return fail(HT_ETREE, "parent[0] must be -1");
  std::vector<int> depth(T, 0);
  for (int v = 1; v < T; ++v) {
    if (parent[v] < 0 || parent[v] >= v) return fail(HT_ETREE, "parent[%d]=%d must be in 0..%d", v, parent[v], v - 1);
    depth[v] = depth[parent[v]] + 1;
    if (depth[v] > max_depth) return fail(HT_ETREE, "node %d has depth %d > %d", v, depth[v], max_depth);
    if (rank) {
      if (rank[v] < 0 || rank[v] >= HT_MAX_TOPK) return fail(HT_ETREE, "rank[%d]=%d outside 0..%d", v, rank[v], HT_MAX_TOPK - 1);
      for (int u = 1; u < v; ++u)
        if (parent[u] == parent[v] && rank[u] == rank[v]) return fail(HT_ETREE, "siblings %d and %d share rank %d", u, v, rank[v]);
    }
  }
  return HT_OK;
}

// Nodes below the root of the complete b-ary tree of depth k, counted up to kMaxTree (more never matter).
int candidate_tree_room(int k, int b) {
  int room = 0, level = 1;
  for (int e = 0; e < k && room < kMaxTree; ++e) {
    level = level * b > kMaxTree ? kMaxTree : level * b;
    room += level;
  }
  return room < kMaxTree ? room : kMaxTree;
}

// Tokens of the tree from the candidates of the last draft: into the fixed tree, or (ht_set_dynamic_tree) into the
// tree this step chooses from the candidates' log-probabilities, which also rewrites the tree tables.
int build_tree(ht_model* m, hipStream_t s) {
  Buffers& b = m->b;
  const ht_config& c = m->cfg;
  if (!m->dyn_b) {
    HT_HIP(launch_tree_build(b.state, b.cand, b.tree.dev(), b.tok, m->T, s));
    return HT_OK;
  }
  HT_HIP(launch_cand_logprob(b.dlogits, b.cand, c.k, m->dyn_b, c.vocab, b.lp, s));
  HT_HIP(launch_tree_dynamic(&b.state->root, b.cand, b.lp, c.k, m->dyn_b, m->T, b.tree.out(), b.tok, s));
  return HT_OK;
}

}  // namespace

extern "C" {

const char* ht_last_error(void) { return g_err; }

int32_t ht_padded_rows(int32_t M) { return padded_rows(M); }

int ht_workspace_bytes(const ht_config* cfg, size_t* out_bytes) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!out_bytes) return fail(HT_EINVAL, "out_bytes is NULL");
  Carver cv(nullptr);
  Buffers b;
  carve(*cfg, cv, b);
  *out_bytes = align_up(cv.off, 256);
  return HT_OK;
}

int ht_init_model(const ht_config* cfg, const ht_weights* w, void* workspace, size_t workspace_bytes, void* stream,
                  ht_model** out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!w || !workspace || !out) return fail(HT_EINVAL, "NULL argument");
  if ((uintptr_t)workspace % 256) return fail(HT_EINVAL, "workspace must be 256-byte aligned");
  size_t need = 0;
  ht_workspace_bytes(cfg, &need);
  if (workspace_bytes < need) return fail(HT_EINVAL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  if (!w->tok_emb || !w->final_norm || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->ffn_norm ||
      !w->w_gate || !w->w_up || !w->w_down || !w->w_transfer)
    return fail(HT_EINVAL, "a weight pointer is NULL");
  const int L = cfg->n_layers;
  const char* env0 = getenv("HT_FORCE_SIMPLE");
  const bool can_defer = shapes_packable(*cfg) && !(env0 && env0[0] == '1');
  if (!w->lm_head && !can_defer) return fail(HT_EINVAL, "lm_head is NULL (deferred loading needs a packable bf16 model)");
  for (int l = 0; l < L; ++l) {
    if (!w->attn_norm[l] || !w->ffn_norm[l]) return fail(HT_EINVAL, "a norm gain of layer %d is NULL", l);
    const int given = !!w->wq[l] + !!w->wk[l] + !!w->wv[l] + !!w->wo[l] + !!w->w_gate[l] + !!w->w_up[l] + !!w->w_down[l];
    if (given != 7 && !(given == 0 && can_defer))
      return fail(HT_EINVAL, "layer %d: projection pointers must all be given (or all NULL for deferred loading of a "
                             "packable bf16 model)", l);
  }
  for (int i = 0; i < cfg->k; ++i)
    if (!w->w_transfer[i]) return fail(HT_EINVAL, "w_transfer[%d] is NULL", i);

  hipStream_t s = (hipStream_t)stream;
  ht_model* m = new ht_model();
  m->cfg = *cfg;
  m->tok_emb = w->tok_emb;
  m->final_norm = w->final_norm;
  m->lm_head = w->lm_head;
  m->attn_norm.assign(w->attn_norm, w->attn_norm + L);
  m->wq.assign(w->wq, w->wq + L);
  m->wk.assign(w->wk, w->wk + L);
  m->wv.assign(w->wv, w->wv + L);
  m->wo.assign(w->wo, w->wo + L);
  m->ffn_norm.assign(w->ffn_norm, w->ffn_norm + L);
  m->w_gate.assign(w->w_gate, w->w_gate + L);
  m->w_up.assign(w->w_up, w->w_up + L);
  m->w_down.assign(w->w_down, w->w_down + L);
  m->w_transfer.assign(w->w_transfer, w->w_transfer + cfg->k);
  m->Mp = padded_rows(cfg->max_tree > cfg->k ? cfg->max_tree : cfg->k);
  m->slot_of_layer.assign(L, -1);
  for (int i = 0; i < cfg->k; ++i) {
    if (i == 0 || cfg->transfer_layer[i] != cfg->transfer_layer[i - 1]) {
      m->slot_of_layer[cfg->transfer_layer[i]] = (int)m->slot_layer.size();
      m->slot_layer.push_back(cfg->transfer_layer[i]);
      m->slot_first.push_back(i);
      m->slot_count.push_back(0);
    }
    ++m->slot_count.back();
  }
  const char* env = getenv("HT_FORCE_SIMPLE");
  m->use_mfma = !(env && env[0] == '1');
  Carver cv(workspace);
  carve(*cfg, cv, m->b);

  auto cleanup = [&](int code) {
    if (m->h_stage) (void)hipHostFree(m->h_stage);
    if (m->h_state) (void)hipHostFree(m->h_state);
    delete m;
    return code;
  };
  size_t stage_ints = (size_t)cfg->max_cache > 2 * kTableInts ? (size_t)cfg->max_cache : 2 * kTableInts;
  stage_ints += 3 * (size_t)L * 2 + 64;     // per-layer pointer tables (as 8-byte entries) follow the ints
  hipError_t e = hipHostMalloc((void**)&m->h_stage, stage_ints * sizeof(int32_t) + 16, hipHostMallocDefault);
  if (e == hipSuccess) e = hipHostMalloc((void**)&m->h_state, sizeof(StepState), hipHostMallocDefault);
  if (e == hipSuccess) e = hipMemsetAsync(workspace, 0, need, s);
  if (e != hipSuccess) return cleanup(fail(HT_EHIP, "init allocation/clear failed: %s", hipGetErrorString(e)));

  if (e == hipSuccess && cfg->dtype == HT_BF16) e = attn_mfma_prepare(cfg->head_dim);
  if (e != hipSuccess) return cleanup(fail(HT_EHIP, "kernel set-up failed: %s", hipGetErrorString(e)));
  m->packed = m->use_mfma && shapes_packable(*cfg);
  m->qkv_fused = m->packed && qkv_fusable(cfg->head_dim);
  m->layer_loaded.assign(L, 0);
  if (m->packed) {
    for (int l = 0; l < L && e == hipSuccess; ++l)
      if (m->wq[l]) {
        e = pack_layer(m, l, m->wq[l], m->wk[l], m->wv[l], m->wo[l], m->w_gate[l], m->w_up[l], m->w_down[l], s);
        m->layer_loaded[l] = 1;
      }
    if (e == hipSuccess && m->lm_head) {
      e = launch_repack(WeightSegs{{m->lm_head, nullptr, nullptr}, {cfg->vocab, 0, 0}, 1}, cfg->d_model, 0, 0,
                        (void*)m->b.p_head.p, s);
      m->head_loaded = true;
    }
    if (e != hipSuccess) return cleanup(fail(HT_EHIP, "weight repack failed: %s", hipGetErrorString(e)));
  } else {
    m->layer_loaded.assign(L, 1);
    m->head_loaded = true;
  }

  // chain tables (prefill chunks and pseudo rows): row i has depth i and sees rows 0..i
  std::vector<int32_t> cp(kMaxRows);
  for (int i = 0; i < kMaxRows; ++i) cp[i] = i - 1;
  fill_tables(kMaxRows, cp.data(), nullptr, m->h_stage);
  if ((rc = upload_tables(m->b.chain, m->h_stage, s))) return cleanup(rc);
  // pointer tables
  void** hp = (void**)(m->h_stage + 2 * kTableInts);
  for (int l = 0; l < L; ++l) { hp[l] = m->b.kc[l]; hp[L + l] = m->b.vc[l]; }
  for (int i = 0; i < cfg->k; ++i) hp[2 * L + i] = (void*)m->w_transfer[i];
  e = hipMemcpyAsync(m->b.kc_ptrs, hp, sizeof(void*) * L, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(m->b.vc_ptrs, hp + L, sizeof(void*) * L, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(m->b.wt_ptrs, hp + 2 * L, sizeof(void*) * cfg->k, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return cleanup(fail(HT_EHIP, "init upload failed: %s", hipGetErrorString(e)));
  *out = m;
  return HT_OK;
}

int ht_load_layer(ht_model* m, int32_t layer, const void* wq, const void* wk, const void* wv, const void* wo,
                  const void* w_gate, const void* w_up, const void* w_down, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!m->packed) return fail(HT_EUNSUPPORTED, "deferred loading needs a bf16 model whose projections are packed");
  if (layer < 0 || layer >= m->cfg.n_layers) return fail(HT_EINVAL, "layer %d out of range", layer);
  if (!wq || !wk || !wv || !wo || !w_gate || !w_up || !w_down) return fail(HT_EINVAL, "NULL weight pointer");
  HT_HIP(pack_layer(m, layer, wq, wk, wv, wo, w_gate, w_up, w_down, (hipStream_t)stream));
  m->layer_loaded[layer] = 1;
  return HT_OK;
}

int ht_load_lm_head(ht_model* m, const void* lm_head, void* stream) {
  if (!m || !lm_head) return fail(HT_EINVAL, "NULL argument");
  if (!m->packed) return fail(HT_EUNSUPPORTED, "deferred loading needs a bf16 model whose projections are packed");
  HT_HIP(launch_repack(WeightSegs{{lm_head, nullptr, nullptr}, {m->cfg.vocab, 0, 0}, 1}, m->cfg.d_model, 0, 0,
                       (void*)m->b.p_head.p, (hipStream_t)stream));
  m->head_loaded = true;
  return HT_OK;
}

int ht_free_model(ht_model* m) {
  if (!m) return HT_OK;
  if (m->h_stage) (void)hipHostFree(m->h_stage);
  if (m->h_state) (void)hipHostFree(m->h_state);
  delete m;
  return HT_OK;
}

int ht_set_tree(ht_model* m, int32_t T, const int32_t* parent, const int32_t* rank, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!rank) return fail(HT_EINVAL, "rank is NULL");
  int rc = validate_tree(T, parent, rank, m->cfg.k, m->cfg.max_tree < kMaxTree ? m->cfg.max_tree : kMaxTree);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  HT_HIP(hipStreamSynchronize(s));           // staging buffer may still feed an earlier copy
  fill_tables(T, parent, rank, m->h_stage);
  int32_t* width = m->h_stage + kTableInts;
  for (int e = 0; e < kMaxTransfer + 2; ++e) width[e] = 0;
  const int32_t* depth = m->h_stage + kMaxRows;
  for (int v = 1; v < T; ++v)
    if (rank[v] + 1 > width[depth[v]]) width[depth[v]] = rank[v] + 1;
  if ((rc = upload_tables(m->b.tree, m->h_stage, s))) return rc;
  HT_HIP(hipMemcpyAsync(m->b.width, width, sizeof(int32_t) * (kMaxTransfer + 2), hipMemcpyHostToDevice, s));
  HT_HIP(hipStreamSynchronize(s));
  m->depth.assign(depth, depth + T);
  m->parent.assign(parent, parent + T);
  m->rank.assign(rank, rank + T);
  m->fused.clear();
  m->drafts_of = -1;
  m->dyn_b = 0;
  m->T = T;
  m->has_tree = true;
  m->verify_done = false;
  return HT_OK;
}

int ht_set_dynamic_tree(ht_model* m, int32_t T, int32_t b, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  const ht_config& c = m->cfg;
  if (T < 1 || T > c.max_tree || T > kMaxTree) return fail(HT_ETREE, "tree size %d outside 1..%d", T, c.max_tree);
  if (b < 1 || b > kMaxTopK) return fail(HT_ETREE, "%d candidates per level outside 1..%d", b, kMaxTopK);
  if (T - 1 > candidate_tree_room(c.k, b))
    return fail(HT_ETREE, "%d levels of %d candidates hold %d nodes, fewer than the %d asked for", c.k, b,
                candidate_tree_room(c.k, b), T - 1);
  hipStream_t s = (hipStream_t)stream;
  HT_HIP(hipStreamSynchronize(s));           // staging buffer may still feed an earlier copy
  // until the first step has chosen a tree the tables hold the root alone
  const int32_t root_parent = -1, root_rank = 0;
  fill_tables(1, &root_parent, &root_rank, m->h_stage);
  int32_t* width = m->h_stage + kTableInts;
  for (int e = 0; e < kMaxTransfer + 2; ++e) width[e] = e >= 1 && e <= c.k ? b : 0;
  int rc;
  if ((rc = upload_tables(m->b.tree, m->h_stage, s))) return rc;
  HT_HIP(hipMemcpyAsync(m->b.width, width, sizeof(int32_t) * (kMaxTransfer + 2), hipMemcpyHostToDevice, s));
  HT_HIP(hipStreamSynchronize(s));
  m->depth.clear();
  m->parent.clear();
  m->rank.clear();
  m->fused.clear();
  m->drafts_of = -1;
  m->dyn_b = b;
  m->T = T;
  m->has_tree = true;
  m->verify_done = false;
  return HT_OK;
}

int ht_set_fused_nodes(ht_model* m, int32_t count, const int32_t* nodes, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!m->has_tree) return fail(HT_ESTATE, "no tree: call ht_set_tree first");
  if (count < 0 || (count > 0 && !nodes)) return fail(HT_EINVAL, "bad node list");
  if (m->dyn_b) {
    // the tables belong to the tree of the last step and the host keeps no copy of it: nothing to rebuild
    if (count) return fail(HT_ESTATE, "a tree chosen anew at every step has no fixed nodes to draft from");
    m->fused.clear();
    m->drafts_of = -1;
    return HT_OK;
  }
  const ht_config& c = m->cfg;
  const int T = m->T, rows = T + count * c.k;
  if (rows > c.max_tree || rows > kMaxRows)
    return fail(HT_ECAPACITY, "%d tree rows + %d x %d pseudo rows exceed max_tree %d", T, count, c.k, c.max_tree);
  for (int f = 0; f < count; ++f) {
    if (nodes[f] < 0 || nodes[f] >= T) return fail(HT_ETREE, "fused node %d outside the tree", nodes[f]);
    for (int e = 0; e < f; ++e)
      if (nodes[e] == nodes[f]) return fail(HT_ETREE, "fused node %d listed twice", nodes[f]);
  }
  // the pass's row tables: the tree, then the pseudo rows in the order they join the pass: transfer layer by
  // transfer layer, node by node, step by step.  Pseudo row i of node v hangs under row i - 1 of v (the first
  // under v itself): it sits at v's position + i and sees what v sees, v's earlier pseudo rows and itself.
  std::vector<int32_t> parent(m->parent), rank(m->rank);
  auto row_of = [&](int f, int i) {            // i: 0-based transfer step
    int g = 0;
    while (i >= m->slot_first[g] + m->slot_count[g]) ++g;
    return T + count * m->slot_first[g] + f * m->slot_count[g] + (i - m->slot_first[g]);
  };
  for (size_t g = 0; g < m->slot_layer.size(); ++g)
    for (int f = 0; f < count; ++f)
      for (int i = m->slot_first[g]; i < m->slot_first[g] + m->slot_count[g]; ++i) {
        parent.push_back(i == 0 ? nodes[f] : row_of(f, i - 1));
        rank.push_back(0);
      }
  hipStream_t s = (hipStream_t)stream;
  HT_HIP(hipStreamSynchronize(s));           // staging buffer may still feed an earlier copy
  fill_tables(rows, parent.data(), rank.data(), m->h_stage);
  int rc;
  if ((rc = upload_tables(m->b.tree, m->h_stage, s))) return rc;
  int32_t* rows_stage = m->h_stage + kTableInts;
  int32_t* src_stage = rows_stage + kMaxRows;      // logits row, counted from the first pseudo row, of (node, step)
  for (int f = 0; f < count; ++f) {
    rows_stage[f] = nodes[f];
    for (int i = 0; i < c.k; ++i) src_stage[f * c.k + i] = row_of(f, i) - T;
  }
  if (count) {
    HT_HIP(hipMemcpyAsync(m->b.fused_rows, rows_stage, sizeof(int32_t) * count, hipMemcpyHostToDevice, s));
    HT_HIP(hipMemcpyAsync(m->b.fused_src, src_stage, sizeof(int32_t) * count * c.k, hipMemcpyHostToDevice, s));
  }
  HT_HIP(hipStreamSynchronize(s));
  m->fused.assign(nodes, nodes + count);
  m->drafts_of = -1;
  return HT_OK;
}

int ht_prefill(ht_model* m, const int32_t* tokens, int32_t n, void* stream) {
  if (!m || !tokens) return fail(HT_EINVAL, "NULL argument");
  const ht_config& c = m->cfg;
  if (!all_loaded(m)) return fail(HT_ESTATE, "deferred weights: ht_load_layer / ht_load_lm_head have not supplied every layer");
  if (n < 1) return fail(HT_EINVAL, "prompt must have at least one token");
  if (n > c.max_cache) return fail(HT_ECAPACITY, "prompt of %d tokens exceeds max_cache %d", n, c.max_cache);
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= c.vocab) return fail(HT_EINVAL, "token %d at %d outside the vocabulary", tokens[i], i);
  hipStream_t s = (hipStream_t)stream;
  HT_HIP(hipStreamSynchronize(s));
  memcpy(m->h_stage, tokens, sizeof(int32_t) * n);
  HT_HIP(hipMemcpyAsync(m->b.prompt, m->h_stage, sizeof(int32_t) * n, hipMemcpyHostToDevice, s));
  m->n = 0;
  m->has_prefill = m->transfer_ready = m->verify_done = false;
  const TreeDev chain = m->b.chain.dev();
  int rc;
  const int chunk = m->Mp < 128 ? m->Mp : 128;          // more rows a pass would only stream the weights twice
  for (int start = 0; start < n; start += chunk) {
    const int rows = n - start < chunk ? n - start : chunk;
    const bool last = start + rows == n;
    HT_HIP(launch_embed(c.dtype, m->tok_emb, m->b.prompt + start, m->b.x, rows, c.d_model, s));
    if ((rc = run_pass(m, chain, rows, 0, true, last ? m->b.logits : nullptr, m->b.g, s))) return rc;
    if (last)
      HT_HIP(launch_prefill_finish(m->b.state, m->b.g, m->b.saved_h, (size_t)m->Mp * c.d_model, (int)m->slot_layer.size(),
                                   m->b.h_src, rows - 1, c.d_model, s));
    m->n += rows;                              // chain rows are already in their final slots
  }
  HT_HIP(hipStreamSynchronize(s));
  m->has_prefill = true;
  return HT_OK;
}

int ht_training_forward(ht_model* m, int32_t step, const int32_t* tokens, int32_t n, float* kl_out, double* loss_out,
                        float* logits_hidden_out, float* logits_pseudo_out, void* stream) {
  if (!m || !tokens) return fail(HT_EINVAL, "NULL argument");
  const ht_config& c = m->cfg;
  if (!all_loaded(m)) return fail(HT_ESTATE, "deferred weights: ht_load_layer / ht_load_lm_head have not supplied every layer");
  if (step < 1 || step > c.k) return fail(HT_EINVAL, "transfer step %d outside 1..%d", step, c.k);
  if (n < step + 2) return fail(HT_EINVAL, "%d tokens give no loss term for step %d (at least %d needed)", n, step, step + 2);
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= c.vocab) return fail(HT_EINVAL, "token %d at %d outside the vocabulary", tokens[i], i);
  // A pass through blocks t+1..L holds C hidden rows whose K/V stay in the cache, `step` more hidden rows of lookahead
  // (the pseudo rows of the chunk see up to step - 1 positions ahead, the loss pairs up to `step`; the next pass
  // computes them again) and the chunk's C pseudo rows.
  const int room = c.max_tree < kMaxTree ? c.max_tree : kMaxTree;
  const int C = (room - step) / 2;
  if (C < 1) return fail(HT_ECAPACITY, "max_tree %d leaves no room for a chunk at step %d", c.max_tree, step);
  if (n + C > c.max_cache) return fail(HT_ECAPACITY, "%d tokens + %d pseudo rows exceed max_cache %d", n, C, c.max_cache);
  hipStream_t s = (hipStream_t)stream;
  Buffers& b = m->b;
  HT_HIP(hipStreamSynchronize(s));
  memcpy(m->h_stage, tokens, sizeof(int32_t) * n);
  HT_HIP(hipMemcpyAsync(b.prompt, m->h_stage, sizeof(int32_t) * n, hipMemcpyHostToDevice, s));
  HT_HIP(hipStreamSynchronize(s));           // the staging buffer takes the row tables next
  m->n = 0;
  m->has_prefill = m->transfer_ready = m->verify_done = false;
  m->drafts_of = -1;
  const int last_pseudo = n - step;          // pseudo rows exist for positions j <= n - step: all they may see is there
  const int terms = n - step - 1;            // loss terms j = 0 .. n - step - 2 (Sec. 3.3, upper limit of the sum)
  int shape_real = -1, shape_pseudo = -1, rc;
  std::vector<int32_t> parent, rows;
  const int t = c.transfer_layer[step - 1];
  // Blocks 1..t see hidden rows only, so they take two chunks (and the lookahead of the second) in one pass of up to
  // 2 C + step rows; their finished residual rows wait in the saved-hidden buffer while blocks t+1..L run the two
  // chunks one after the other, each with its pseudo rows.
  for (int b0 = 0; b0 < n; b0 += 2 * C) {
    const int low = n - b0 < 2 * C + step ? n - b0 : 2 * C + step;
    m->n = b0;
    HT_HIP(launch_embed(c.dtype, m->tok_emb, b.prompt + b0, b.x, low, c.d_model, s));
    if (t > 0 && (rc = run_pass(m, b.chain.dev(), low, 0, false, nullptr, nullptr, s, kNoJoin, 0, 0, t))) return rc;
    HT_HIP(launch_load_rows(b.x, b.saved_h, low, c.d_model, s));
    for (int c0 = b0; c0 < n && c0 < b0 + 2 * C; c0 += C) {
      const int real = n - c0 < C + step ? n - c0 : C + step;
      int pseudo = last_pseudo - c0 + 1;
      pseudo = pseudo < 0 ? 0 : pseudo > C ? C : pseudo;
      if (real != shape_real || pseudo != shape_pseudo) {
        // hidden rows form a chain; the pseudo row of in-pass position f hangs under hidden row f + step - 1: it then
        // sees hidden rows 0 .. f + step - 1 and itself and sits at position c0 + f + step (Sec. 3.3)
        parent.assign(real + pseudo, 0);
        rows.assign(pseudo > 0 ? pseudo : 1, 0);
        for (int r = 0; r < real; ++r) parent[r] = r - 1;
        for (int f = 0; f < pseudo; ++f) {
          parent[real + f] = f + step - 1;
          rows[f] = f;
        }
        HT_HIP(hipStreamSynchronize(s));       // earlier uploads have left the staging buffer
        fill_tables(real + pseudo, parent.data(), nullptr, m->h_stage);
        if ((rc = upload_tables(b.train, m->h_stage, s))) return rc;
        int32_t* rows_stage = m->h_stage + kTableInts;
        memcpy(rows_stage, rows.data(), sizeof(int32_t) * rows.size());
        HT_HIP(hipMemcpyAsync(b.train_rows, rows_stage, sizeof(int32_t) * rows.size(), hipMemcpyHostToDevice, s));
        shape_real = real;
        shape_pseudo = pseudo;
      }
      m->n = c0;
      HT_HIP(launch_load_rows(b.saved_h + (size_t)(c0 - b0) * c.d_model, b.x, real, c.d_model, s));
      if ((rc = run_pass(m, b.train.dev(), real, t, false, b.logits, nullptr, s, pseudo ? kTrainStep : kNoJoin, pseudo,
                         step - 1)))
        return rc;
      int pairs = terms - c0;
      pairs = pairs < 0 ? 0 : pairs > pseudo ? pseudo : pairs;
      if (pairs) HT_HIP(launch_kl_rows(b.logits, real, step, pairs, c.vocab, b.kl + c0, s));
      // the first `step` rows of a later pass were the lookahead of the pass before, whose loss terms used them: the
      // copy keeps that first version (in bf16 the two passes may round a row differently)
      const int seen = c0 > 0 ? step : 0;
      if (logits_hidden_out && real > seen)
        HT_HIP(hipMemcpyAsync(logits_hidden_out + (size_t)(c0 + seen) * c.vocab, b.logits + (size_t)seen * c.vocab,
                              sizeof(float) * (real - seen) * c.vocab, hipMemcpyDeviceToDevice, s));
      if (logits_pseudo_out && pseudo)
        HT_HIP(hipMemcpyAsync(logits_pseudo_out + (size_t)c0 * c.vocab, b.logits + (size_t)real * c.vocab,
                              sizeof(float) * pseudo * c.vocab, hipMemcpyDeviceToDevice, s));
      m->n = c0 + (real < C ? real : C);       // the lookahead rows are overwritten by the next pass
    }
  }
  float* h_kl = (float*)m->h_stage;
  HT_HIP(hipStreamSynchronize(s));
  HT_HIP(hipMemcpyAsync(h_kl, b.kl, sizeof(float) * terms, hipMemcpyDeviceToHost, s));
  HT_HIP(hipStreamSynchronize(s));
  double loss = 0.0;
  for (int j = 0; j < terms; ++j) {
    loss += (double)h_kl[j];
    if (kl_out) kl_out[j] = h_kl[j];
  }
  if (loss_out) *loss_out = loss;
  return HT_OK;
}

}  // extern "C" (reopened below)

// ---- the forward pass of the training stage over all positions at once ---------------------------------------------
namespace {
struct WideBuffers {
  float* x;            // residual stream [rows, d]
  void* u;             // normalised rows (bf16, before the 1/rms factor) [rows, d]
  float* qkv;          // [rows, (Hq + 2 Hkv) hd]
  void* q;             // rotated queries [rows, Hq hd]
  void* attn;          // attention output [rows, Hq hd]
  void* act;           // silu(gate) * up [rows, f]
  float* part;         // output of the O / down projection [rows, d]
  float* ss;           // sums of squares of the rows of u [rows, kNormParts]
  float* logits;       // [rows, V]
  float* cs;           // rotary table of positions 0 .. n [n + 1, hd / 2] (cos, sin), the same for every block
  void* self_k;        // the pseudo rows' own keys [n, Hkv hd] (rotated) and values [Hkv hd, self_cap]
  void* self_v;
  int self_cap;
  void* attn_scratch;  // the two slices of the pseudo rows' attention (cache part, own part)
  void* w_transfer;    // the step's transfer map in the streaming layout
  size_t total;
};

WideBuffers carve_wide(const ht_config& c, int n, void* base) {
  Carver cv(base);
  WideBuffers w;
  const size_t rows = 2 * (size_t)n, d = c.d_model, qd = (size_t)c.n_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim;
  w.x = cv.take<float>(rows * d);
  w.u = cv.take_bytes(rows * d * 2);
  w.qkv = cv.take<float>(rows * (qd + 2 * kvd));
  w.q = cv.take_bytes(rows * qd * 2);
  w.attn = cv.take_bytes(rows * qd * 2);
  w.act = cv.take_bytes(rows * c.d_ffn * 2);
  w.part = cv.take<float>(rows * d);
  w.ss = cv.take<float>(rows * kNormParts);
  w.logits = cv.take<float>(rows * c.vocab);
  w.cs = cv.take<float>(((size_t)n + 1) * c.head_dim);
  w.self_cap = (n + 63) / 64 * 64;
  w.self_k = cv.take_bytes((size_t)n * kvd * 2);
  w.self_v = cv.take_bytes(kvd * (size_t)w.self_cap * 2);
  w.attn_scratch = cv.take_bytes(attn_causal_scratch_bytes(n, c.n_heads, c.head_dim));
  w.w_transfer = cv.take_bytes(packed_weight_bytes((int)d, (int)d));
  w.total = align_up(cv.off, 256);
  return w;
}

}  // namespace

extern "C" int ht_training_workspace_bytes(const ht_config* cfg, int32_t n, size_t* out_bytes) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!out_bytes || n < 1) return fail(HT_EINVAL, "bad argument");
  *out_bytes = carve_wide(*cfg, n, nullptr).total;
  return HT_OK;
}

extern "C" int ht_training_forward_batched(ht_model* m, int32_t step, const int32_t* tokens, int32_t n, float* kl_out,
                                           double* loss_out, float* logits_hidden_out, float* logits_pseudo_out,
                                           void* train_ws, size_t train_ws_bytes, void* stream) {
  if (!m || !tokens || !train_ws) return fail(HT_EINVAL, "NULL argument");
  const ht_config& c = m->cfg;
  if (!m->packed || !m->qkv_fused)
    return fail(HT_EUNSUPPORTED, "the batched forward pass needs a bf16 model on packed weights with heads of a multiple of 32");
  if (c.d_model % (4 * kNormParts)) return fail(HT_EUNSUPPORTED, "d_model must be a multiple of %d", 4 * kNormParts);
  if (!attn_mfma_supported(kMaxRows, c.n_heads, c.n_kv_heads, c.head_dim))
    return fail(HT_EUNSUPPORTED, "head size %d has no matrix-core attention kernel", c.head_dim);
  if (!all_loaded(m)) return fail(HT_ESTATE, "deferred weights: ht_load_layer / ht_load_lm_head have not supplied every layer");
  if (step < 1 || step > c.k) return fail(HT_EINVAL, "transfer step %d outside 1..%d", step, c.k);
  if (n < step + 2) return fail(HT_EINVAL, "%d tokens give no loss term for step %d (at least %d needed)", n, step, step + 2);
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= c.vocab) return fail(HT_EINVAL, "token %d at %d outside the vocabulary", tokens[i], i);
  if (n > c.max_cache) return fail(HT_ECAPACITY, "%d tokens exceed max_cache %d", n, c.max_cache);
  if ((uintptr_t)train_ws % 256) return fail(HT_EINVAL, "workspace must be 256-byte aligned");
  const WideBuffers w = carve_wide(c, n, train_ws);
  if (train_ws_bytes < w.total) return fail(HT_EINVAL, "workspace has %zu bytes, %zu needed", train_ws_bytes, w.total);
  hipStream_t s = (hipStream_t)stream;
  Buffers& b = m->b;
  const int d = c.d_model, qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, f = c.d_ffn, L = c.n_layers;
  const int stride_qkv = qd + 2 * kvd;
  const int t = c.transfer_layer[step - 1];
  const int P = n - step + 1;                // pseudo states exist for positions j <= n - step
  const int terms = n - step - 1;            // loss terms j = 0 .. n - step - 2 (Sec. 3.3, upper limit of the sum)
  const RowScale rs{w.ss, 1.0f / (float)d, c.rms_eps};

  HT_HIP(hipStreamSynchronize(s));
  memcpy(m->h_stage, tokens, sizeof(int32_t) * n);
  HT_HIP(hipMemcpyAsync(b.prompt, m->h_stage, sizeof(int32_t) * n, hipMemcpyHostToDevice, s));
  HT_HIP(hipStreamSynchronize(s));           // the staging buffer takes the row tables next
  m->n = 0;
  m->has_prefill = m->transfer_ready = m->verify_done = false;
  m->drafts_of = -1;
  HT_HIP(launch_repack(WeightSegs{{m->w_transfer[step - 1], nullptr, nullptr}, {d, 0, 0}, 1}, d, 0, 0, w.w_transfer, s));
  const PackedW p_transfer{(const bf16_t*)w.w_transfer, d, d, packed_cols(d)};

  HT_HIP(launch_embed(c.dtype, m->tok_emb, b.prompt, w.x, n, d, s));
  HT_HIP(launch_rope_table(w.cs, nullptr, 0, n + 1, c.head_dim, c.rope_base, s));
  int rows = n, pending = 0;
  const TreeDev chain = b.chain.dev();
  for (int l = 0; l < L; ++l) {
    if (l == t) {
      // the residual after t blocks is complete once the last block's sums are in: pseudo states W_i h_j, j < P, as
      // one more product (sources rounded to bf16 like every other product's operand)
      if (pending) {
        HT_HIP(launch_add_norm_parts(w.x, w.part, 1, (size_t)rows * d, m->attn_norm[l], w.u, nullptr, w.ss, rows, d, s));
        pending = 0;
      }
      HT_HIP(launch_convert_to_bf16(w.x, w.u, (size_t)P * d, s));
      HT_HIP(launch_gemm_wide(w.u, p_transfer, P, w.x + (size_t)n * d, s));
      rows = n + P;
    }
    HT_HIP(launch_add_norm_parts(w.x, w.part, pending, (size_t)rows * d, m->attn_norm[l], w.u, nullptr, w.ss, rows, d, s));
    HT_HIP(launch_gemm_wide(w.u, b.p_qkv[l], rows, w.qkv, s, rs));
    // hidden rows: rotary at their own position, K/V to their own cache slot
    HT_HIP(launch_rope_append(c.dtype, w.qkv, 1, w.cs, w.q, b.kc[l], b.vc[l], 0, n, c.n_heads, c.n_kv_heads, c.head_dim,
                              c.max_cache, true, s));
    if (l >= t) {
      // Pseudo row j sits at position j + step and sees the hidden keys 0 .. j + step - 1 and itself (Sec. 3.3): as
      // row j + step - 1 of a causal launch over the hidden keys, with its own key and value, kept in buffers of their
      // own, as one more slice.  The step - 1 rows in front of pseudo row 0 are computed for nothing (their queries
      // are the last hidden rows'), and their outputs land on the last hidden rows of w.attn, which the hidden rows'
      // own launch below writes afterwards.
      const int lead = step - 1;
      HT_HIP(launch_rope_append(c.dtype, w.qkv + (size_t)n * stride_qkv, 1, w.cs + (size_t)step * c.head_dim,
                                (char*)w.q + (size_t)n * qd * 2, w.self_k, w.self_v, lead, P, c.n_heads, c.n_kv_heads,
                                c.head_dim, w.self_cap, true, s));
      HT_HIP(launch_attn_causal((char*)w.q + (size_t)(n - lead) * qd * 2, b.kc[l], b.vc[l], c.max_cache, n, chain, c.n_heads,
                                c.n_kv_heads, c.head_dim, (char*)w.attn + (size_t)(n - lead) * qd * 2, s, w.self_k, w.self_v,
                                w.self_cap, w.attn_scratch));
    }
    HT_HIP(launch_attn_causal(w.q, b.kc[l], b.vc[l], c.max_cache, n, chain, c.n_heads, c.n_kv_heads, c.head_dim, w.attn, s));
    HT_HIP(launch_gemm_wide(w.attn, b.p_o[l], rows, w.part, s));
    HT_HIP(launch_add_norm_parts(w.x, w.part, 1, (size_t)rows * d, m->ffn_norm[l], w.u, nullptr, w.ss, rows, d, s));
    HT_HIP(launch_gemm_wide_silu(w.u, b.p_gu[l], rows, w.act, s, rs));
    HT_HIP(launch_gemm_wide(w.act, b.p_down[l], rows, w.part, s));
    pending = 1;
  }
  HT_HIP(launch_add_norm_parts(w.x, w.part, pending, (size_t)rows * d, m->final_norm, w.u, nullptr, w.ss, rows, d, s));
  HT_HIP(launch_gemm_wide(w.u, b.p_head, rows, w.logits, s, rs));
  // term j pairs pseudo row j (logits row n + j) with the hidden state it stands for (logits row j + step)
  for (int j0 = 0; j0 < terms; j0 += 32768) {
    const int cnt = terms - j0 < 32768 ? terms - j0 : 32768;
    HT_HIP(launch_kl_rows(w.logits, n + j0, step + j0, cnt, c.vocab, b.kl + j0, s));
  }
  if (logits_hidden_out)
    HT_HIP(hipMemcpyAsync(logits_hidden_out, w.logits, sizeof(float) * (size_t)n * c.vocab, hipMemcpyDeviceToDevice, s));
  if (logits_pseudo_out)
    HT_HIP(hipMemcpyAsync(logits_pseudo_out, w.logits + (size_t)n * c.vocab, sizeof(float) * (size_t)P * c.vocab,
                          hipMemcpyDeviceToDevice, s));
  float* h_kl = (float*)m->h_stage;
  HT_HIP(hipStreamSynchronize(s));
  HT_HIP(hipMemcpyAsync(h_kl, b.kl, sizeof(float) * terms, hipMemcpyDeviceToHost, s));
  HT_HIP(hipStreamSynchronize(s));
  double loss = 0.0;
  for (int j = 0; j < terms; ++j) {
    loss += (double)h_kl[j];
    if (kl_out) kl_out[j] = h_kl[j];
  }
  if (loss_out) *loss_out = loss;
  return HT_OK;
}

extern "C" {

int ht_transfer(ht_model* m, const void* h_src, float* pseudo_out, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!h_src && !m->has_prefill) return fail(HT_ESTATE, "no saved hidden state: call ht_prefill first or pass h_src");
  hipStream_t s = (hipStream_t)stream;
  const ht_config& c = m->cfg;
  if (!h_src && !pseudo_out && m->drafts_of >= 0) return HT_OK;   // the verify pass already drafted from this node
  m->drafts_of = -1;
  const int slots = (int)m->slot_layer.size();
  if (h_src) HT_HIP(launch_convert_to_f32(c.dtype, h_src, m->b.h_src, slots * c.d_model, s));
  for (int g = 0; g < slots; ++g)       // step i reads the source of its own layer
    HT_HIP(launch_transfer(c.dtype, m->b.h_src + (size_t)g * c.d_model, nullptr, 1, (const void* const*)m->b.wt_ptrs,
                           m->b.pseudo + (size_t)m->slot_first[g] * c.d_model, m->slot_first[g], m->slot_count[g], 0,
                           c.d_model, s));
  if (pseudo_out)
    HT_HIP(hipMemcpyAsync(pseudo_out, m->b.pseudo, sizeof(float) * c.k * c.d_model, hipMemcpyDeviceToDevice, s));
  m->transfer_ready = true;
  return HT_OK;
}

int ht_tree_verify_step(ht_model* m, const int32_t* tree_tokens, int32_t* argmax_out, float* logits_out, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!m->has_tree) return fail(HT_ESTATE, "no tree: call ht_set_tree first");
  if (!m->has_prefill) return fail(HT_ESTATE, "empty cache: call ht_prefill first");
  if (!tree_tokens && !m->transfer_ready && m->drafts_of < 0)
    return fail(HT_ESTATE, "drafting needs a preceding ht_transfer");
  if (tree_tokens && m->dyn_b) return fail(HT_ESTATE, "a dynamic tree is drafted by the step itself: forced tokens need ht_set_tree");
  const ht_config& c = m->cfg;
  const int T = m->T, fused = (int)m->fused.size(), Mall = T + fused * c.k;
  const int rows = Mall > c.k ? Mall : c.k;
  if (m->n + rows > c.max_cache)
    return fail(HT_ECAPACITY, "cache_len %d + %d rows exceeds max_cache %d", m->n, rows, c.max_cache);
  hipStream_t s = (hipStream_t)stream;
  Buffers& b = m->b;
  int rc;
  if (tree_tokens) {
    HT_HIP(hipMemcpyAsync(b.tok, tree_tokens, sizeof(int32_t) * T, hipMemcpyDeviceToDevice, s));
  } else if (m->drafts_of >= 0 && !m->transfer_ready) {
    // the last verify pass carried pseudo rows for the node the acceptance ended on: its candidates are the tree
    HT_HIP(launch_tree_build(b.state, b.cand_fused + (size_t)m->drafts_of * c.k * kMaxTopK, b.tree.dev(), b.tok, T, s));
  } else {
    // draft: pseudo rows through blocks t+1..L as a chain at positions n, n+1, ..; their K/V land in
    // slots n.. and are overwritten by the verify pass below
    if ((rc = run_pass(m, b.chain.dev(), 0, c.transfer_layer[0], false, b.dlogits, nullptr, s, kFromBuffer))) return rc;
    HT_HIP(launch_topk(b.dlogits, b.cand, b.width, b.topk_scratch, c.k, c.k, nullptr, c.vocab, s));
    if ((rc = build_tree(m, s))) return rc;
  }
  HT_HIP(launch_embed(c.dtype, m->tok_emb, b.tok, b.x, T, c.d_model, s));
  if (!fused) {
    float* z = logits_out ? logits_out : b.logits;
    if ((rc = run_pass(m, b.tree.dev(), T, 0, true, z, b.g, s))) return rc;
  } else {
    // rows T.. of the logits are the draft distributions of the fused nodes (k rows per node)
    if ((rc = run_pass(m, b.tree.dev(), T, 0, true, b.logits, b.g, s, kFromTree, fused))) return rc;
    HT_HIP(launch_topk(b.logits + (size_t)T * c.vocab, b.cand_fused, b.width, b.topk_scratch, fused * c.k, c.k, b.fused_src,
                       c.vocab, s));
    if (logits_out)
      HT_HIP(hipMemcpyAsync(logits_out, b.logits, sizeof(float) * T * c.vocab, hipMemcpyDeviceToDevice, s));
  }
  if (argmax_out) HT_HIP(hipMemcpyAsync(argmax_out, b.g, sizeof(int32_t) * T, hipMemcpyDeviceToDevice, s));
  m->verify_done = true;
  m->transfer_ready = false;
  m->drafts_of = -1;
  return HT_OK;
}

int ht_accept_and_compact(ht_model* m, int32_t* n_accepted, int32_t* accepted_tokens, int32_t* next_root,
                          int32_t* path_out, void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!m->verify_done) return fail(HT_ESTATE, "ht_accept_and_compact must follow ht_tree_verify_step");
  hipStream_t s = (hipStream_t)stream;
  const ht_config& c = m->cfg;
  Buffers& b = m->b;
  HT_HIP(launch_accept(b.state, b.tree.dev(), b.tok, b.g, m->T, s));
  HT_HIP(launch_compact(c.dtype, b.state, b.kc_ptrs, b.vc_ptrs, c.n_layers, m->n, c.n_kv_heads, c.head_dim, c.max_cache,
                        b.saved_h, (size_t)m->Mp * c.d_model, (int)m->slot_layer.size(), b.h_src, c.d_model, s));
  HT_HIP(hipMemcpyAsync(m->h_state, b.state, sizeof(StepState), hipMemcpyDeviceToHost, s));
  HT_HIP(hipStreamSynchronize(s));
  const StepState& st = *m->h_state;
  if (st.m < 1 || st.m > c.k + 1) return fail(HT_EHIP, "accept kernel returned an impossible count %d", st.m);
  m->n += st.m;
  m->verify_done = false;
  m->drafts_of = -1;
  for (size_t f = 0; f < m->fused.size(); ++f)
    if (m->fused[f] == st.path[st.m - 1]) m->drafts_of = (int)f;
  if (n_accepted) *n_accepted = st.m;
  if (next_root) *next_root = st.next_root;
  for (int j = 0; j < st.m; ++j) {
    if (accepted_tokens) accepted_tokens[j] = st.emitted[j];
    if (path_out) path_out[j] = st.path[j];
  }
  return HT_OK;
}

// Device-resident loop (schedule: draft after acceptance).  Every kernel reads the cache length from the step state
// on the device, the acceptance kernel advances it and logs the step, and the host only waits once, at the end.
int ht_decode_steps(ht_model* m, int32_t steps, int32_t* n_accepted, int32_t* accepted_tokens, int32_t* next_root,
                    void* stream) {
  if (!m) return fail(HT_EINVAL, "model is NULL");
  if (!m->has_tree) return fail(HT_ESTATE, "no tree: call ht_set_tree first");
  if (!m->has_prefill) return fail(HT_ESTATE, "empty cache: call ht_prefill first");
  if (m->verify_done) return fail(HT_ESTATE, "a verify pass is waiting for ht_accept_and_compact");
  if (!m->fused.empty()) return fail(HT_ESTATE, "the loop drafts after acceptance: clear ht_set_fused_nodes first");
  if (steps < 1 || steps > kMaxLoopSteps) return fail(HT_EINVAL, "steps must be in 1..%d", kMaxLoopSteps);
  const ht_config& c = m->cfg;
  Buffers& b = m->b;
  const int T = m->T, rows = T > c.k ? T : c.k, n0 = m->n;
  if (n0 + steps * (c.k + 1) + rows > c.max_cache)
    return fail(HT_ECAPACITY, "cache_len %d + %d steps of up to %d tokens + %d rows exceeds max_cache %d", n0, steps,
                c.k + 1, rows, c.max_cache);
  hipStream_t s = (hipStream_t)stream;
  HT_HIP(hipStreamSynchronize(s));                     // the staging buffer below may still be in use
  int32_t* init = m->h_stage;
  init[0] = n0;                                        // n_old
  init[1] = n0;                                        // n
  init[2] = 0;                                         // log_count
  HT_HIP(hipMemcpyAsync(&b.state->n_old, init, 3 * sizeof(int32_t), hipMemcpyHostToDevice, s));
  struct Guard {
    ht_model* m;
    int n;
    ~Guard() { m->n_dev = nullptr; m->n = n; }
  } guard{m, n0};
  m->n_dev = &b.state->n;
  const int slots = (int)m->slot_layer.size();
  int rc;
  for (int st = 0; st < steps; ++st) {
    m->n = n0 + st * (c.k + 1);                        // upper bound of the cache length at this step: sizes grids only
    for (int g = 0; g < slots; ++g)
      HT_HIP(launch_transfer(c.dtype, b.h_src + (size_t)g * c.d_model, nullptr, 1, (const void* const*)b.wt_ptrs,
                             b.pseudo + (size_t)m->slot_first[g] * c.d_model, m->slot_first[g], m->slot_count[g], 0,
                             c.d_model, s));
    if ((rc = run_pass(m, b.chain.dev(), 0, c.transfer_layer[0], false, b.dlogits, nullptr, s, kFromBuffer))) return rc;
    HT_HIP(launch_topk(b.dlogits, b.cand, b.width, b.topk_scratch, c.k, c.k, nullptr, c.vocab, s));
    if ((rc = build_tree(m, s))) return rc;
    HT_HIP(launch_embed(c.dtype, m->tok_emb, b.tok, b.x, T, c.d_model, s));
    if ((rc = run_pass(m, b.tree.dev(), T, 0, true, b.logits, b.g, s))) return rc;
    HT_HIP(launch_accept(b.state, b.tree.dev(), b.tok, b.g, T, s, b.log));
    HT_HIP(launch_compact(c.dtype, b.state, b.kc_ptrs, b.vc_ptrs, c.n_layers, 0, c.n_kv_heads, c.head_dim, c.max_cache,
                          b.saved_h, (size_t)m->Mp * c.d_model, slots, b.h_src, c.d_model, s, true));
  }
  StepLog* h_log = (StepLog*)m->h_stage;
  HT_HIP(hipMemcpyAsync(h_log, b.log, sizeof(StepLog) * steps, hipMemcpyDeviceToHost, s));
  HT_HIP(hipMemcpyAsync(m->h_state, b.state, sizeof(StepState), hipMemcpyDeviceToHost, s));
  HT_HIP(hipStreamSynchronize(s));
  int total = 0;
  for (int st = 0; st < steps; ++st) {
    const int cnt = h_log[st].m;
    if (cnt < 1 || cnt > c.k + 1) return fail(HT_EHIP, "step %d of the loop logged an impossible count %d", st, cnt);
    if (n_accepted) n_accepted[st] = cnt;
    if (accepted_tokens)
      for (int j = 0; j < cnt; ++j) accepted_tokens[total + j] = h_log[st].emitted[j];
    total += cnt;
  }
  if (m->h_state->n != n0 + total || m->h_state->log_count != steps)
    return fail(HT_EHIP, "device cache length %d after the loop, expected %d", m->h_state->n, n0 + total);
  guard.n = n0 + total;
  m->transfer_ready = m->verify_done = false;
  m->drafts_of = -1;
  if (next_root) *next_root = m->h_state->next_root;
  return HT_OK;
}

int32_t ht_cache_len(const ht_model* m) { return m ? m->n : -1; }

int ht_get_buffer(const ht_model* m, int32_t which, int32_t layer, void** dev_ptr, size_t* bytes) {
  if (!m || !dev_ptr) return fail(HT_EINVAL, "NULL argument");
  const ht_config& c = m->cfg;
  const size_t es = elem_size(c.dtype);
  void* p = nullptr;
  size_t sz = 0;
  switch (which) {
    case HT_BUF_DRAFT_LOGITS: p = m->b.dlogits; sz = sizeof(float) * c.k * c.vocab; break;
    case HT_BUF_CANDIDATES: p = m->b.cand; sz = sizeof(int32_t) * c.k * kMaxTopK; break;
    case HT_BUF_TREE_TOKENS: p = m->b.tok; sz = sizeof(int32_t) * m->T; break;
    case HT_BUF_SAVED_HIDDEN:
    case HT_BUF_TRANSFER_SRC:            // `layer` selects the distinct transfer layer (0 = lowest)
      if (layer < 0 || layer >= (int)m->slot_layer.size()) return fail(HT_EINVAL, "transfer-layer slot %d out of range", layer);
      if (which == HT_BUF_SAVED_HIDDEN) { p = m->b.saved_h + (size_t)layer * m->Mp * c.d_model; sz = sizeof(float) * m->T * c.d_model; }
      else { p = m->b.h_src + (size_t)layer * c.d_model; sz = sizeof(float) * c.d_model; }
      break;
    case HT_BUF_PSEUDO: p = m->b.pseudo; sz = sizeof(float) * c.k * c.d_model; break;
    case HT_BUF_ROOT: p = &m->b.state->root; sz = sizeof(int32_t); break;
    case HT_BUF_FUSED_DRAFT_LOGITS:
      p = m->b.logits + (size_t)m->T * c.vocab;
      sz = sizeof(float) * m->fused.size() * c.k * c.vocab;
      break;
    case HT_BUF_FUSED_CANDIDATES: p = m->b.cand_fused; sz = sizeof(int32_t) * m->fused.size() * c.k * kMaxTopK; break;
    case HT_BUF_CANDIDATE_LOGPROBS: p = m->b.lp; sz = sizeof(float) * c.k * kMaxTopK; break;
    case HT_BUF_TREE_PARENT: p = m->b.tree.parent; sz = sizeof(int32_t) * m->T; break;
    case HT_BUF_TREE_RANK: p = m->b.tree.rank; sz = sizeof(int32_t) * m->T; break;
    case HT_BUF_K_CACHE:
    case HT_BUF_V_CACHE:
      if (layer < 0 || layer >= c.n_layers) return fail(HT_EINVAL, "layer %d out of range", layer);
      p = which == HT_BUF_K_CACHE ? m->b.kc[layer] : m->b.vc[layer];
      sz = (size_t)c.max_cache * c.n_kv_heads * c.head_dim * es;
      break;
    default: return fail(HT_EINVAL, "unknown buffer id %d", which);
  }
  *dev_ptr = p;
  if (bytes) *bytes = sz;
  return HT_OK;
}

// ------------------------------------------------------------------------------------------------ op level
namespace {
struct AttnScratch {
  int32_t *parent, *depth, *rank;
  uint64_t* anc;
  float* cs;
  void* q_rot;
  void* mfma;
  size_t total;
};
AttnScratch attn_scratch_layout(char* base, int T, int Hq, int hd, size_t es) {
  Carver cv(base);
  AttnScratch a;
  a.parent = cv.take<int32_t>(kMaxRows);
  a.depth = cv.take<int32_t>(kMaxRows);
  a.rank = cv.take<int32_t>(kMaxRows);
  a.anc = cv.take<uint64_t>((size_t)kMaxRows * kMaskWords);
  a.cs = cv.take<float>((size_t)padded_rows(T) * hd);
  a.q_rot = cv.take_bytes((size_t)padded_rows(T) * Hq * hd * es);
  a.mfma = cv.take_bytes(attn_mfma_scratch_bytes(padded_rows(T), Hq, hd));
  a.total = align_up(cv.off, 256);
  return a;
}
}  // namespace

size_t ht_tree_attention_scratch_bytes(int32_t T, int32_t Hq, int32_t hd) {
  if (T < 1 || T > kMaxRows || Hq < 1 || hd < 2) return 0;
  return attn_scratch_layout(nullptr, T, Hq, hd, 4).total;
}

int ht_tree_attention(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache, int32_t cap,
                      int32_t n, int32_t T, const int32_t* parent, int32_t Hq, int32_t Hkv, int32_t hd, int32_t dtype,
                      float rope_base, void* out, void* scratch, size_t scratch_bytes, void* stream) {
  if (!q || !k_cache || !v_cache || !out || !scratch) return fail(HT_EINVAL, "NULL argument");
  if ((k_new == nullptr) != (v_new == nullptr)) return fail(HT_EINVAL, "k_new and v_new must both be given or both be NULL");
  if (dtype != HT_F32 && dtype != HT_BF16) return fail(HT_EINVAL, "bad dtype");
  if (Hq < 1 || Hkv < 1 || Hq % Hkv || hd < 2 || hd % 2 || hd > 256) return fail(HT_EINVAL, "bad head shape");
  if (n < 0 || cap < 8 || cap % 8) return fail(HT_EINVAL, "cap must be a positive multiple of 8 and n >= 0");
  int rc;
  if (parent) {
    if ((rc = validate_tree(T, parent, nullptr, kMaxRows, kMaxRows))) return rc;
  } else if (T < 1 || T > kMaxRows) {
    return fail(HT_ETREE, "tree size %d outside 1..%d", T, kMaxRows);
  }
  if (n + T > cap) return fail(HT_ECAPACITY, "n + T = %d exceeds cap %d", n + T, cap);
  if (scratch_bytes < ht_tree_attention_scratch_bytes(T, Hq, hd)) return fail(HT_EINVAL, "scratch too small");
  if ((uintptr_t)scratch % 256) return fail(HT_EINVAL, "scratch must be 256-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  AttnScratch a = attn_scratch_layout((char*)scratch, T, Hq, hd, elem_size(dtype));
  TreeTables tt{a.parent, a.depth, a.rank, a.anc};
  if (parent) {                          // NULL: the tables an earlier call left in `scratch` are used again
    // The table image lives on this call's stack and goes up from pageable memory: the copies have left it when
    // hipMemcpyAsync returns, so the call keeps no state of its own between calls or threads.
    std::vector<int32_t> stage(kTableInts);
    fill_tables(T, parent, nullptr, stage.data());
    if ((rc = upload_tables(tt, stage.data(), s))) return rc;
  }
  const void* qq = q;
  if (k_new) {
    HT_HIP(launch_rope_table(a.cs, a.depth, n, T, hd, rope_base, s));
    HT_HIP(launch_rope_append_split(dtype, q, k_new, v_new, a.cs, a.q_rot, k_cache, v_cache, n, T, Hq, Hkv, hd, cap, s));
    qq = a.q_rot;
  }
  const char* env = getenv("HT_FORCE_SIMPLE");
  const bool simple = env && env[0] == '1';
  if (dtype == HT_BF16 && !simple && attn_mfma_supported(T, Hq, Hkv, hd)) {
    HT_HIP(launch_attn_mfma(qq, k_cache, v_cache, cap, n, T, tt.dev(), Hq, Hkv, hd, out, a.mfma, s));
  } else {
    HT_HIP(launch_attn_simple(dtype, qq, k_cache, v_cache, cap, n, T, tt.dev(), Hq, Hkv, hd, out, s));
  }
  return HT_OK;
}

int ht_mfma_rate_probe(int32_t form, int32_t iters, void* sink, double* flops, void* stream) {
  if (!sink) return fail(HT_EINVAL, "NULL argument");
  if (form < 0 || form > 3) return fail(HT_EINVAL, "form %d: 0 / 1 (16x16x32 / 32x32x16), + 2 for hashed operand bits", form);
  if (iters < 1 || iters > (1 << 20)) return fail(HT_EINVAL, "iters %d outside 1 .. 2^20", iters);
  const double f = launch_mfma_rate(form, iters, (uint32_t*)sink, (hipStream_t)stream);
  HT_HIP(hipGetLastError());
  if (flops) *flops = f;
  return HT_OK;
}

int ht_stream_read_probe(const void* buf, size_t bytes, void* sink, size_t* bytes_read, void* stream) {
  if (!buf || !sink) return fail(HT_EINVAL, "NULL argument");
  if ((uintptr_t)buf % 16) return fail(HT_EINVAL, "buffer must be 16-byte aligned");
  const size_t got = launch_stream_read(buf, bytes, 256, (uint32_t*)sink, (hipStream_t)stream);
  if (!got) return fail(HT_EINVAL, "buffer of %zu bytes is smaller than one pass (8 MiB)", bytes);
  HT_HIP(hipGetLastError());
  if (bytes_read) *bytes_read = got;
  return HT_OK;
}

size_t ht_weight_pack_bytes(int32_t N, int32_t K) {
  if (N < 16 || N % 16 || K < 8 || K % 8) return 0;
  return align_up(packed_weight_bytes(N, K), 256);
}

int ht_weight_pack(const void* w, int32_t N, int32_t K, void* packed, void* stream) {
  if (!w || !packed) return fail(HT_EINVAL, "NULL argument");
  if (!ht_weight_pack_bytes(N, K)) return fail(HT_EINVAL, "packing needs N %% 16 == 0 and K %% 8 == 0 (N=%d K=%d)", N, K);
  HT_HIP(launch_repack(segs1(w, N), K, 0, 0, packed, (hipStream_t)stream));
  return HT_OK;
}

int ht_gate_up_pack(const void* w_gate, const void* w_up, int32_t f, int32_t K, void* packed, void* stream) {
  if (!w_gate || !w_up || !packed) return fail(HT_EINVAL, "NULL argument");
  if (f < 16 || f % 16 || !ht_weight_pack_bytes(2 * f, K))
    return fail(HT_EINVAL, "packing needs f %% 16 == 0 and K %% 8 == 0 (f=%d K=%d)", f, K);
  HT_HIP(launch_repack(WeightSegs{{w_gate, w_up, nullptr}, {f, f, 0}, 2}, K, 1, 0, packed, (hipStream_t)stream));
  return HT_OK;
}

int ht_gate_up_silu_packed(const void* a, const void* packed, int32_t M, int32_t f, int32_t K, void* act_out,
                           void* stream) {
  if (!a || !packed || !act_out) return fail(HT_EINVAL, "NULL argument");
  if (M < 1 || M > kMaxRows || f < 16 || f % 16 || !ht_weight_pack_bytes(2 * f, K))
    return fail(HT_EINVAL, "bad shape M=%d f=%d K=%d", M, f, K);
  PackedW pw{(const bf16_t*)packed, 2 * f, K, packed_cols(K)};
  HT_HIP(launch_gemm_packed_silu(a, pw, M, act_out, (hipStream_t)stream));
  return HT_OK;
}

size_t ht_skinny_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || N < 1 || K < 1) return 0;
  return align_up((size_t)kMaxSplitK * M * N * sizeof(float), 256) + ht_weight_pack_bytes(N, K);
}

int ht_skinny_gemm_packed(const void* a, const void* packed, int32_t M, int32_t N, int32_t K, float* out, void* scratch,
                          size_t scratch_bytes, void* stream) {
  if (!a || !packed || !out) return fail(HT_EINVAL, "NULL argument");
  if (M < 1 || M > kMaxRows || !ht_weight_pack_bytes(N, K)) return fail(HT_EINVAL, "bad shape M=%d N=%d K=%d", M, N, K);
  hipStream_t s = (hipStream_t)stream;
  PackedW pw{(const bf16_t*)packed, N, K, packed_cols(K)};
  int sp = gemm_mfma_splits(M, N, K);
  if (sp > 1 && (!scratch || scratch_bytes < (size_t)sp * M * N * sizeof(float))) sp = 1;
  if (sp == 1) {
    HT_HIP(launch_gemm_packed(a, pw, M, out, 1, s));
  } else {
    HT_HIP(launch_gemm_packed(a, pw, M, (float*)scratch, sp, s));
    HT_HIP(launch_reduce_splits((const float*)scratch, sp, (size_t)M * N, out, s));
  }
  return HT_OK;
}

// ---- the packed product for callers that cannot allocate --------------------------------------------------------
// Split-K partial sums live in a device array of the library's own instead of a caller's scratch buffer.  Every
// GPU holds its own copy of the array at its own address: the address is asked for once per device, with that
// device current, and only that pointer (never the array's name) reaches kernels.
}  // extern "C" (reopened below the file-scope state)

namespace {
constexpr size_t kNoAllocScratchBytes = HT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each GPU, filled on first use

int noalloc_scratch(float** out) {
  int dev = -1;
  HT_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(HT_EUNSUPPORTED, "device index %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HT_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(HT_EHIP, "the library's scratch array has no address on device %d", dev);
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return HT_OK;
}
}  // namespace

extern "C" {

int ht_skinny_gemm_packed_noalloc(const void* a, const void* packed, int32_t M, int32_t N, int32_t K, float* out,
                                  void* stream) {
  if (!a || !packed || !out) return fail(HT_EINVAL, "NULL argument");
  if (M < 1 || M > kMaxRows || !ht_weight_pack_bytes(N, K)) return fail(HT_EINVAL, "bad shape M=%d N=%d K=%d", M, N, K);
  hipStream_t s = (hipStream_t)stream;
  PackedW pw{(const bf16_t*)packed, N, K, packed_cols(K)};
  const int sp = gemm_mfma_splits(M, N, K);          // the same split as ht_skinny_gemm_packed with enough scratch
  if (sp == 1) {
    HT_HIP(launch_gemm_packed(a, pw, M, out, 1, s));
    return HT_OK;
  }
  const size_t need = (size_t)sp * M * N * sizeof(float);
  if (need > kNoAllocScratchBytes)
    return fail(HT_ECAPACITY, "%d K splits of %d x %d partial sums need %zu bytes, the library's own scratch holds %zu",
                sp, M, N, need, kNoAllocScratchBytes);
  float* part = nullptr;
  int rc = noalloc_scratch(&part);
  if (rc) return rc;
  // every partial sum [split][m < M][n < N] is written before it is read: nothing has to start at zero
  HT_HIP(launch_gemm_packed(a, pw, M, part, sp, s));
  HT_HIP(launch_reduce_splits(part, sp, (size_t)M * N, out, s));
  return HT_OK;
}

int ht_skinny_gemm(const void* a, const void* w, int32_t M, int32_t N, int32_t K, int32_t dtype, float* out,
                   void* scratch, size_t scratch_bytes, void* stream) {
  if (!a || !w || !out) return fail(HT_EINVAL, "NULL argument");
  if (dtype != HT_F32 && dtype != HT_BF16) return fail(HT_EINVAL, "bad dtype");
  if (M < 1 || M > kMaxRows || N < 1 || K < 1) return fail(HT_EINVAL, "bad shape M=%d N=%d K=%d", M, N, K);
  hipStream_t s = (hipStream_t)stream;
  const char* env = getenv("HT_FORCE_SIMPLE");
  const bool simple = env && env[0] == '1';
  const size_t pb = ht_weight_pack_bytes(N, K);
  if (dtype == HT_BF16 && !simple && pb && scratch && scratch_bytes >= pb && (uintptr_t)scratch % 256 == 0) {
    int rc = ht_weight_pack(w, N, K, scratch, stream);
    if (rc) return rc;
    return ht_skinny_gemm_packed(a, scratch, M, N, K, out, (char*)scratch + pb, scratch_bytes - pb, stream);
  }
  HT_HIP(launch_gemm_simple(dtype, a, segs1(w, N), M, N, K, out, s));
  return HT_OK;
}

int ht_kl_divergence_rows(const float* z, int32_t row_a, int32_t row_b, int32_t pairs, int32_t V, float* kl, void* stream) {
  if (!z || !kl) return fail(HT_EINVAL, "NULL argument");
  if (row_a < 0 || row_b < 0 || pairs < 1 || pairs > 65535 || V < 1) return fail(HT_EINVAL, "bad shape pairs=%d V=%d", pairs, V);
  HT_HIP(launch_kl_rows(z, row_a, row_b, pairs, V, kl, (hipStream_t)stream));
  return HT_OK;
}

int ht_candidate_logprobs(const float* d, const int32_t* cand, int32_t rows, int32_t b, int32_t V, float* lp, void* stream) {
  if (!d || !cand || !lp) return fail(HT_EINVAL, "NULL argument");
  if (rows < 1 || rows > kMaxRows || b < 1 || b > kMaxTopK || V < 1) return fail(HT_EINVAL, "bad shape rows=%d b=%d V=%d", rows, b, V);
  HT_HIP(launch_cand_logprob(d, cand, rows, b, V, lp, (hipStream_t)stream));
  return HT_OK;
}

int ht_dynamic_tree(const float* lp, const int32_t* cand, const int32_t* root, int32_t k, int32_t b, int32_t T,
                    int32_t* parent, int32_t* depth, int32_t* rank, uint64_t* anc, int32_t* tokens, void* stream) {
  if (!lp || !cand || !root || !parent || !depth || !rank || !anc || !tokens) return fail(HT_EINVAL, "NULL argument");
  if (k < 1 || k > kMaxTransfer) return fail(HT_EINVAL, "k = %d outside 1..%d", k, kMaxTransfer);
  if (T < 1 || T > kMaxTree) return fail(HT_ETREE, "tree size %d outside 1..%d", T, kMaxTree);
  if (b < 1 || b > kMaxTopK) return fail(HT_ETREE, "%d candidates per level outside 1..%d", b, kMaxTopK);
  if (T - 1 > candidate_tree_room(k, b))
    return fail(HT_ETREE, "%d levels of %d candidates hold %d nodes, fewer than the %d asked for", k, b,
                candidate_tree_room(k, b), T - 1);
  HT_HIP(launch_tree_dynamic(root, cand, lp, k, b, T, TreeOut{parent, depth, rank, anc}, tokens, (hipStream_t)stream));
  return HT_OK;
}

}  // extern "C"
