// Stage object: buffer partitioning, the per-layer kernel sequences of forward
// and backward, gradient accumulation state, and the profiler.  C ABI in
// include/ah_stage.h.  Host code only enqueues kernels: on the caller's stream and, for the
// parts of backward that nothing downstream waits for, on a second stream joined back into it.
#include "ah_stage.h"
#include "capi_util.h"
#include "kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace ah;

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct ParamEntry { uint64_t off; int rows, cols; };  // cols == 0: tensor absent in this architecture

// byte offsets of one layer's saved activations
struct ActLayout {
  size_t x_in, a, qkv, o, lse, x_mid, c, u, g, stats1, stats2, bytes;
};

struct Workspace {
  size_t d0, d1, dmid, dbig, dsm, delta, part_n2, part_n1, part_b1, part_bqkv, rope, prof_x, prof_dy, prof_y, prof_dx, layer_ws, pend, vec_part, bytes;
};

// Output-gradient operands of one layer's four weight-gradient products, kept per (position in the group, layer)
// while those products wait for the rest of the group: byte offsets inside one such block.
struct PendLayout { size_t dy, dmid, du, dqkv, bytes; };
// Partial sums of one layer's vector gradients, shared by the micro-batches of a group (byte offsets in its block).
struct VecPartLayout { size_t n2, n1, b1, bqkv, bytes; };

}  // namespace

struct ah_stage {
  ah_stage_config_t cfg;
  ah_stage_buffers_t bufs;
  int T, h, nh, d, hl, F, L;
  bool llama, causal, recompute, res32;
  bool rope_in_gemm;  // the QKV product's tiles hold whole heads per wave: the rotary embedding runs in its epilogue
  float eps, rope_base;
  ParamEntry ptab[AH_P_COUNT];
  uint64_t layer_elems;
  ActLayout act;       // offsets inside one layer's block (x_in first)
  size_t slot_bytes;   // per in-flight micro-batch
  size_t per_layer_slot_bytes;
  Workspace ws;
  std::vector<char> busy;  // per slot: 0 empty, 1 forward done, 2 backward done and weight gradients pending
  bool overwrite_grads;   // next backward writes the vector gradients (and, undeferred, the matrices) instead of adding
  bool overwrite_wgrads;  // next weight-gradient product writes instead of adding
  // Deferred weight gradients: with group > 1 the four weight-gradient products of a layer run once per `group`
  // micro-batches, over the concatenation of their tokens, instead of once per micro-batch.
  int group;
  bool defer_matrix[4];         // by WgradWhich: small outputs stay undeferred (see plan())
  bool force_immediate;         // the profiler's per-layer timing runs undeferred
  PendLayout pend;
  VecPartLayout vpart;
  std::vector<int> pend_slots;  // slots of the micro-batches waiting, in backward order
  bool rope_ready;
  // optional per-call-site timing (ah_stage_trace_begin / _end)
  bool tracing;
  // Second stream for the work of backward that nothing downstream waits for (weight gradients, column-sum
  // reductions); created on first use, joined back into the caller's stream before every return.
  hipStream_t side;
  hipEvent_t sync_ev[8];
  bool side_ready, side_off;
  std::vector<hipEvent_t> ev_pool;           // pairs, in launch order
  std::vector<int> ev_site;                  // site of pair i
  std::vector<int> ev_mult;                  // micro-batches covered by the launch of pair i
  size_t ev_used;
};

namespace {

int validate(const ah_stage_config_t* c) {
  if (!c) return set_error(AH_EINVAL, "config is NULL");
  if (c->struct_size != sizeof(ah_stage_config_t)) return set_error(AH_EINVAL, "config.struct_size %u != %zu", c->struct_size, sizeof(ah_stage_config_t));
  if (c->arch != AH_ARCH_GPT && c->arch != AH_ARCH_LLAMA && c->arch != AH_ARCH_BERT) return set_error(AH_EINVAL, "unknown arch %d", c->arch);
  if (c->n_layers < 1 || c->n_layers > 1024) return set_error(AH_EINVAL, "n_layers %d out of range [1, 1024]", c->n_layers);
  if (c->tp_degree < 1 || c->tp_rank < 0 || c->tp_rank >= c->tp_degree) return set_error(AH_EINVAL, "bad tp_degree/tp_rank %d/%d", c->tp_degree, c->tp_rank);
  if (c->n_heads < 1 || c->ffn_hidden < 1 || c->hidden < 1 || c->seq_len < 1 || c->microbatch_size < 1)
    return set_error(AH_EINVAL, "sizes must be positive");
  if (c->n_heads % c->tp_degree || c->ffn_hidden % c->tp_degree) return set_error(AH_EINVAL, "tp_degree must divide n_heads and ffn_hidden");
  if (c->n_microbatches < 1) return set_error(AH_EINVAL, "n_microbatches must be >= 1");
  if (c->max_in_flight < 1 || c->max_in_flight > 4096) return set_error(AH_EINVAL, "max_in_flight %d out of range [1, 4096]", c->max_in_flight);
  if (c->recompute != 0 && c->recompute != 1) return set_error(AH_EINVAL, "recompute must be 0 or 1");
  if (c->residual_fp32 != 0 && c->residual_fp32 != 1) return set_error(AH_EINVAL, "residual_fp32 must be 0 or 1");
  if (c->wgrad_group < 0 || c->wgrad_group > kMaxGemmSegments) return set_error(AH_EINVAL, "wgrad_group %d out of range [0, %d]", c->wgrad_group, kMaxGemmSegments);
  if (c->wgrad_group > 1 && c->recompute) return set_error(AH_EINVAL, "wgrad_group > 1 keeps activations for the deferred products: recompute must be 0");
  if (c->wgrad_group > c->max_in_flight) return set_error(AH_EINVAL, "wgrad_group %d needs max_in_flight >= %d (a slot stays occupied until its group's weight gradients are taken)", c->wgrad_group, c->wgrad_group);
  if (c->norm_eps < 0 || c->rope_base < 0) return set_error(AH_EINVAL, "norm_eps and rope_base must be >= 0");
  if (c->head_dim != 64 && c->head_dim != 128) return set_error(AH_EUNSUPPORTED, "head_dim %d: only 64 and 128 are supported", c->head_dim);
  if (c->hidden % 128 || c->hidden > 16384) return set_error(AH_EUNSUPPORTED, "hidden %d must be a multiple of 128 and <= 16384", c->hidden);
  if (c->seq_len % 128) return set_error(AH_EUNSUPPORTED, "seq_len %d must be a multiple of 128", c->seq_len);
  const long hl = (long)(c->n_heads / c->tp_degree) * c->head_dim, F = c->ffn_hidden / c->tp_degree;
  if (hl % 128 || F % 128) return set_error(AH_EUNSUPPORTED, "local attention width %ld and local FFN width %ld must be multiples of 128", hl, F);
  if ((long)c->microbatch_size * c->seq_len > (1L << 24)) return set_error(AH_EUNSUPPORTED, "microbatch_size * seq_len too large");
  if (hl > 65536 || F > 262144) return set_error(AH_EUNSUPPORTED, "local widths too large");
  return AH_OK;
}

void plan(ah_stage* s, const ah_stage_config_t* c) {
  s->cfg = *c;
  s->L = c->n_layers;
  s->h = c->hidden;
  s->nh = c->n_heads / c->tp_degree;
  s->d = c->head_dim;
  s->hl = s->nh * s->d;
  s->F = c->ffn_hidden / c->tp_degree;
  s->T = c->microbatch_size * c->seq_len;
  s->llama = c->arch == AH_ARCH_LLAMA;
  s->causal = c->arch != AH_ARCH_BERT;
  s->recompute = c->recompute != 0;
  s->res32 = c->residual_fp32 != 0;
  s->group = c->wgrad_group > 1 ? c->wgrad_group : 1;
  {
    // A deferred product runs at the end of its group with a k axis G times as long.  That pays for the outputs
    // large enough for the 256-wide tiles (fewer fp32 passes over a large matrix, one prologue and epilogue).  A
    // small output, which gets 128 x 128 tiles that use a CU poorly on their own, is better taken per micro-batch:
    // the side stream runs it beside the rest of backward, and its read-modify-write is small anyway (measured on
    // the BERT-Large stage, whose matrices are all of that kind: 26.7 ms per step undeferred, 29.1 deferred).
    const char* e = getenv("AH_DEFER_MIN_TILE_AREA");  // tuning aid
    const int min_area = e ? atoi(e) : 256 * 128;
    const int Fu_ = (c->arch == AH_ARCH_LLAMA ? 2 : 1) * s->F;
    const int mn[4][2] = {{s->F, s->h}, {s->h, Fu_}, {s->hl, s->h}, {s->h, 3 * s->hl}};  // WG_FC2, WG_FC1, WG_WO, WG_QKV
    for (int i = 0; i < 4; i++) s->defer_matrix[i] = gemm_tile_area(mn[i][0], mn[i][1], GEMM_TN) >= min_area;
    // tuning and test aid: the choice given outright, bit i = matrix i (second MLP, first MLP, out-projection, QKV)
    if (const char* m = getenv("AH_DEFER_MATRICES"))
      for (int i = 0; i < 4; i++) s->defer_matrix[i] = (atoi(m) >> i) & 1;
  }
  {
    const int wc = gemm_min_wave_cols(s->T, 3 * s->hl, GEMM_NN);
    s->rope_in_gemm = s->llama && wc > 0 && wc % s->d == 0 && !getenv("AH_ROPE_KERNEL");  // the variable: tuning aid
  }
  s->eps = c->norm_eps > 0 ? c->norm_eps : (s->llama ? 1e-6f : 1e-5f);
  s->rope_base = c->rope_base > 0 ? c->rope_base : 10000.f;
  const int h = s->h, hl = s->hl, F = s->F;
  const size_t T = s->T;

  // ---- parameters: every tensor starts on a 128-element boundary (sizes are multiples of 128)
  uint64_t off = 0;
  auto put = [&](int which, int rows, int cols) {
    s->ptab[which] = {off, rows, cols};
    off += (uint64_t)rows * cols;
  };
  for (auto& e : s->ptab) e = {0, 0, 0};
  if (!s->llama) {
    put(AH_P_LN1_G, 1, h); put(AH_P_LN1_B, 1, h); put(AH_P_WQKV, h, 3 * hl); put(AH_P_BQKV, 1, 3 * hl);
    put(AH_P_WO, hl, h); put(AH_P_BO, 1, h); put(AH_P_LN2_G, 1, h); put(AH_P_LN2_B, 1, h);
    put(AH_P_W1, h, F); put(AH_P_B1, 1, F); put(AH_P_W2, F, h); put(AH_P_B2, 1, h);
  } else {
    put(AH_P_LN1_G, 1, h); put(AH_P_WQKV, h, 3 * hl); put(AH_P_WO, hl, h); put(AH_P_LN2_G, 1, h);
    put(AH_P_W1, h, 2 * F); put(AH_P_W2, F, h);
  }
  s->layer_elems = off;

  // ---- activations saved for backward, per layer
  const size_t Fu = s->llama ? 2 * (size_t)F : (size_t)F;  // width of the first MLP product
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align256(bytes); return r; };
  ActLayout& a = s->act;
  const size_t rsz = s->res32 ? 4 : 2;  // bytes per element of the residual stream
  a.x_in = take(T * h * rsz);
  const size_t keep_only_input = o;
  a.a = take(T * h * 2);
  a.qkv = take(T * 3 * hl * 2);
  a.o = take(T * hl * 2);
  a.lse = take(T * s->nh * 4);
  a.x_mid = take(T * h * rsz);
  a.c = take(T * h * 2);
  a.u = take(T * Fu * 2);
  a.g = take(T * F * 2);
  a.stats1 = take(T * 2 * 4);
  a.stats2 = take(T * 2 * 4);
  a.bytes = o;
  s->per_layer_slot_bytes = s->recompute ? keep_only_input : a.bytes;
  s->slot_bytes = s->per_layer_slot_bytes * s->L;

  // ---- workspace
  Workspace& w = s->ws;
  o = 0;
  w.d0 = take(T * h * 2);
  w.d1 = take(T * h * 2);
  w.dmid = take(T * h * 2);
  w.dbig = take(T * std::max<size_t>(Fu, 3 * hl) * 2);
  w.dsm = take(T * std::max<size_t>({(size_t)h, (size_t)hl, (size_t)F}) * 2);
  w.delta = take(T * s->nh * 4);
  // partial column sums: one region per producer, so that the reductions can trail behind on the side stream
  w.part_n2 = take((size_t)3 * norm_bwd_blocks(s->T) * h * 4);
  w.part_n1 = take((size_t)3 * norm_bwd_blocks(s->T) * h * 4);
  w.part_b1 = take(s->llama ? 0 : (size_t)colsum_blocks(s->T) * F * 4);
  w.part_bqkv = take(s->llama ? 0 : (size_t)colsum_blocks(s->T) * 3 * hl * 4);
  w.rope = take(s->llama ? (size_t)c->seq_len * s->d * 4 : 0);
  w.prof_x = take(T * h * 2);
  w.prof_dy = take(T * h * 2);
  w.prof_y = take(T * h * 2);
  w.prof_dx = take(T * h * 2);
  w.layer_ws = take(s->recompute ? a.bytes : 0);
  const size_t before_pend = o;
  o = 0;
  s->pend.dy = take(T * h * 2);
  s->pend.dmid = take(T * h * 2);
  s->pend.du = take(T * Fu * 2);
  s->pend.dqkv = take(T * 3 * hl * 2);
  s->pend.bytes = o;
  o = before_pend;
  w.pend = take(s->group > 1 ? (size_t)s->group * s->L * s->pend.bytes : 0);
  const size_t before_vec = o;
  o = 0;
  s->vpart.n2 = take((size_t)3 * norm_bwd_blocks(s->T) * h * 4);
  s->vpart.n1 = take((size_t)3 * norm_bwd_blocks(s->T) * h * 4);
  s->vpart.b1 = take(s->llama ? 0 : (size_t)colsum_blocks(s->T) * F * 4);
  s->vpart.bqkv = take(s->llama ? 0 : (size_t)colsum_blocks(s->T) * 3 * hl * 4);
  s->vpart.bytes = o;
  o = before_vec;
  w.vec_part = take(s->group > 1 ? (size_t)s->L * s->vpart.bytes : 0);
  w.bytes = o;
}

inline char* P(void* base, size_t off) { return (char*)base + off; }

// ------------------------------------------------------------------ small device helpers
__global__ void rope_table_kernel(float* cs, int S, int half, int d, double base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= S * half) return;
  const int pos = idx / half, i = idx % half;
  const double theta = exp(-(2.0 * i / d) * log(base));
  const double ang = pos * theta;
  cs[2 * idx] = (float)cos(ang);
  cs[2 * idx + 1] = (float)sin(ang);
}

__global__ void fill_pattern_kernel(__bf16* p, size_t n, uint32_t seed) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t x = (uint32_t)i * 2654435761u + seed;
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  p[i] = (__bf16)(((x & 0xffff) / 65536.0f - 0.5f) * 3.4641f);  // uniform, unit variance
}

// call sites that the trace distinguishes
enum Site {
  SITE_QKV_FWD, SITE_WO_FWD, SITE_FC1_FWD, SITE_FC2_FWD, SITE_FC2_WGRAD, SITE_FC2_DGRAD, SITE_FC1_WGRAD, SITE_FC1_DGRAD,
  SITE_WO_WGRAD, SITE_WO_DGRAD, SITE_QKV_WGRAD, SITE_QKV_DGRAD, SITE_ATTN_FWD, SITE_ATTN_BWD, SITE_NORM_FWD, SITE_NORM_BWD,
  SITE_COLSUM, SITE_ROPE, SITE_COUNT
};
const char* const kSiteNames[SITE_COUNT] = {
  "gemm_nn.qkv_fwd", "gemm_nn.wo_fwd", "gemm_nn.fc1_fwd", "gemm_nn.fc2_fwd", "gemm_tn.fc2_wgrad", "gemm_nt.fc2_dgrad",
  "gemm_tn.fc1_wgrad", "gemm_nt.fc1_dgrad", "gemm_tn.wo_wgrad", "gemm_nt.wo_dgrad", "gemm_tn.qkv_wgrad", "gemm_nt.qkv_dgrad",
  "attention_fwd", "attention_bwd", "norm_fwd", "norm_bwd", "colsum", "rope"};

// brackets the launches issued while it lives with an event pair when tracing
struct SiteTimer {
  ah_stage* s;
  hipStream_t st;
  size_t slot;
  SiteTimer(ah_stage* s_, int site, hipStream_t st_, int mult = 1) : s(s_), st(st_), slot((size_t)-1) {
    if (!s->tracing) return;
    if (s->ev_used + 2 > s->ev_pool.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return;
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
      s->ev_pool.push_back(a);
      s->ev_pool.push_back(b);
      s->ev_site.push_back(site);
      s->ev_mult.push_back(mult);
    } else {
      s->ev_site[s->ev_used / 2] = site;
      s->ev_mult[s->ev_used / 2] = mult;
    }
    slot = s->ev_used;
    s->ev_used += 2;
    (void)hipEventRecord(s->ev_pool[slot], st);
  }
  ~SiteTimer() {
    if (slot != (size_t)-1) (void)hipEventRecord(s->ev_pool[slot + 1], st);
  }
};

struct LayerPtrs {
  const char *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
  float *g_ln1_g, *g_ln1_b, *g_wqkv, *g_bqkv, *g_wo, *g_bo, *g_ln2_g, *g_ln2_b, *g_w1, *g_b1, *g_w2, *g_b2;
};

LayerPtrs layer_ptrs(const ah_stage* s, int layer) {
  LayerPtrs p;
  const char* pb = (const char*)s->bufs.params + (size_t)layer * s->layer_elems * 2;
  float* gb = (float*)s->bufs.grads + (size_t)layer * s->layer_elems;
  auto pp = [&](int w) -> const char* { return s->ptab[w].cols ? pb + s->ptab[w].off * 2 : nullptr; };
  auto gp = [&](int w) -> float* { return s->ptab[w].cols ? gb + s->ptab[w].off : nullptr; };
  p.ln1_g = pp(AH_P_LN1_G); p.ln1_b = pp(AH_P_LN1_B); p.wqkv = pp(AH_P_WQKV); p.bqkv = pp(AH_P_BQKV);
  p.wo = pp(AH_P_WO); p.bo = pp(AH_P_BO); p.ln2_g = pp(AH_P_LN2_G); p.ln2_b = pp(AH_P_LN2_B);
  p.w1 = pp(AH_P_W1); p.b1 = pp(AH_P_B1); p.w2 = pp(AH_P_W2); p.b2 = pp(AH_P_B2);
  p.g_ln1_g = gp(AH_P_LN1_G); p.g_ln1_b = gp(AH_P_LN1_B); p.g_wqkv = gp(AH_P_WQKV); p.g_bqkv = gp(AH_P_BQKV);
  p.g_wo = gp(AH_P_WO); p.g_bo = gp(AH_P_BO); p.g_ln2_g = gp(AH_P_LN2_G); p.g_ln2_b = gp(AH_P_LN2_B);
  p.g_w1 = gp(AH_P_W1); p.g_b1 = gp(AH_P_B1); p.g_w2 = gp(AH_P_W2); p.g_b2 = gp(AH_P_B2);
  return p;
}

// pointers to one layer's activations: the input always lives in the slot; the
// rest either in the slot (stored) or in the shared per-layer scratch (recompute)
struct ActPtrs { char *x_in, *a, *qkv, *o, *lse, *x_mid, *c, *u, *g, *stats1, *stats2; };

ActPtrs act_ptrs(const ah_stage* s, int slot, int layer) {
  char* slot_base = (char*)s->bufs.activations + (size_t)slot * s->slot_bytes + (size_t)layer * s->per_layer_slot_bytes;
  char* rest = s->recompute ? (char*)s->bufs.workspace + s->ws.layer_ws : slot_base;
  const ActLayout& a = s->act;
  ActPtrs p;
  p.x_in = slot_base + a.x_in;
  p.a = rest + a.a; p.qkv = rest + a.qkv; p.o = rest + a.o; p.lse = rest + a.lse; p.x_mid = rest + a.x_mid;
  p.c = rest + a.c; p.u = rest + a.u; p.g = rest + a.g; p.stats1 = rest + a.stats1; p.stats2 = rest + a.stats2;
  return p;
}

#define TIMED(site, expr)                \
  do {                                   \
    SiteTimer t_(s, site, st);           \
    g_where = #expr;                     \
    hipError_t e_ = (expr);              \
    if (e_ != hipSuccess) return e_;     \
  } while (0)

#define TRY(expr)                        \
  do {                                   \
    g_where = #expr;                     \
    hipError_t e_ = (expr);              \
    if (e_ != hipSuccess) return e_;     \
  } while (0)

hipError_t gemm(ah_stage* s, int site, GemmLayout lay, GemmEpilogue epi, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N,
                int K, const void* bias, const void* aux, int ld_aux, void* C2, int beta, hipStream_t st, float* colsum_part = nullptr,
                int colsum_acc = 0) {
  GemmArgs g = {};
  g.colsum_part = colsum_part; g.ld_colsum = N; g.colsum_acc = colsum_acc;
  g.A = A; g.B = B; g.C = C; g.C2 = C2; g.bias = bias; g.aux = aux;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.ld_aux = ld_aux; g.M = M; g.N = N; g.K = K; g.beta = beta;
  SiteTimer t(s, site, st);
  return launch_gemm(lay, epi, g, st);
}

// buffers one layer's backward writes its intermediate gradients to
struct BwdBufs { char *dmid, *du, *dqkv; };

BwdBufs pend_bufs(const ah_stage* s, int pos, int layer, char** dy_out) {
  char* b = (char*)s->bufs.workspace + s->ws.pend + ((size_t)pos * s->L + layer) * s->pend.bytes;
  if (dy_out) *dy_out = b + s->pend.dy;
  return {b + s->pend.dmid, b + s->pend.du, b + s->pend.dqkv};
}

// What a layer's backward does about its four weight-gradient products.
//   nseg == 0: takes them now, over this micro-batch alone (operands: this slot's activations and the BwdBufs);
//   nseg <  0: leaves them to a later call;
//   nseg >  0: takes them over the nseg micro-batches in slots[] (group positions 0 .. nseg - 1), whose token
//              axes are concatenated inside the product.
// Matrices that are never deferred (defer_matrix) are taken now whatever nseg says, with beta_now.
struct WgradPlan { int nseg; int slots[kMaxGemmSegments]; int beta, beta_now; };

enum WgradWhich { WG_FC2, WG_FC1, WG_WO, WG_QKV };

// Where a layer's backward leaves the partial column sums behind its vector gradients (biases, gains, offsets) and
// what it does with them.  Undeferred: the shared workspace regions, written (acc = 0) and folded into the gradient
// at once (finish).  Deferred: the layer's own regions, written by the first micro-batch of a group and added to by
// the others, folded once when the group closes.
struct VecPlan { float *n2, *n1, *b1, *bqkv; int acc; bool finish; int beta; };

VecPlan vec_plan(const ah_stage* s, int layer, bool deferred, int pos, bool closes, int beta_now, int beta_group) {
  char* wsb = (char*)s->bufs.workspace;
  if (!deferred)
    return {(float*)(wsb + s->ws.part_n2), (float*)(wsb + s->ws.part_n1), (float*)(wsb + s->ws.part_b1), (float*)(wsb + s->ws.part_bqkv),
            0, true, beta_now};
  char* b = wsb + s->ws.vec_part + (size_t)layer * s->vpart.bytes;
  return {(float*)(b + s->vpart.n2), (float*)(b + s->vpart.n1), (float*)(b + s->vpart.b1), (float*)(b + s->vpart.bqkv),
          pos > 0 ? 1 : 0, closes, beta_group};
}

// Folds one layer's partial sums into its vector gradients (the four reductions that end a layer's backward).
hipError_t finish_vectors(ah_stage* s, int layer, const VecPlan& vp, hipStream_t st);

// One weight-gradient product C[M, N] (+)= sum over the plan's micro-batches of act^T dY.
// A product over one micro-batch goes to `sd` (the side stream: beside the rest of backward it hides its tail and
// the launch gaps); a product over a whole group goes to `st`: it fills the chip for milliseconds, and next to it the
// kernels of the main chain only slow down (gpt7b_tp2, G = 8: 76.1 ms per step this way, 77.9 with the group's
// products on the side stream).
hipError_t wgrad(ah_stage* s, int site, int layer, WgradWhich which, const WgradPlan& wp, const void* act, const void* dY, float* C,
                 int M, int N, hipStream_t st, hipStream_t sd) {
  const bool now = wp.nseg == 0 || !s->defer_matrix[which];
  if (now && !act) return hipSuccess;  // a flush: this matrix was taken with each micro-batch
  if (!now && wp.nseg < 0) return hipSuccess;
  GemmArgs g = {};
  g.A = act; g.B = dY; g.C = C;
  g.lda = M; g.ldb = N; g.ldc = N; g.M = M; g.N = N; g.K = s->T; g.beta = now ? wp.beta_now : wp.beta;
  if (!now) {
    g.seg_k = s->T; g.n_seg = wp.nseg; g.K = s->T * wp.nseg;
    for (int i = 0; i < wp.nseg; i++) {
      const ActPtrs a = act_ptrs(s, wp.slots[i], layer);
      char* dy;
      const BwdBufs b = pend_bufs(s, i, layer, &dy);
      g.segA[i] = which == WG_FC2 ? a.g : which == WG_FC1 ? a.c : which == WG_WO ? a.o : a.a;
      g.segB[i] = which == WG_FC2 ? dy : which == WG_FC1 ? b.du : which == WG_WO ? b.dmid : b.dqkv;
    }
  }
  hipStream_t run_on = now ? sd : st;
  SiteTimer t(s, site, run_on, now ? 1 : wp.nseg);
  return launch_gemm(GEMM_TN, EPI_F32_ACC, g, run_on);
}

// One layer forward.  y == nullptr: stop after the activations backward needs
// (used when a layer is re-run inside backward).
hipError_t layer_forward(ah_stage* s, int layer, const ActPtrs& a, void* y, bool y_is_stage_output, hipStream_t st) {
  const LayerPtrs p = layer_ptrs(s, layer);
  const int T = s->T, h = s->h, hl = s->hl, F = s->F, B = s->cfg.microbatch_size, S = s->cfg.seq_len;
  // the residual stream (x_in, x_mid, the next layer's x_in) is bf16 or fp32; the stage's output y is always bf16
  const bool r32 = s->res32;
  const GemmEpilogue resid = r32 ? EPI_RESID_F32 : EPI_RESID;
  const GemmEpilogue resid_out = r32 ? (y_is_stage_output ? EPI_RESID_F32_OUT16 : EPI_RESID_F32) : EPI_RESID;
  TIMED(SITE_NORM_FWD, launch_norm_fwd(s->llama, a.x_in, p.ln1_g, p.ln1_b, a.a, (float*)a.stats1, T, h, s->eps, st, r32));
  if (s->llama && s->rope_in_gemm) {
    // rotary embedding on Q and K in the epilogue of their product, on the fp32 sums
    GemmArgs g = {};
    g.A = a.a; g.B = p.wqkv; g.C = a.qkv;
    g.lda = h; g.ldb = 3 * hl; g.ldc = 3 * hl; g.M = T; g.N = 3 * hl; g.K = h;
    g.rope_cs = (const float*)P(s->bufs.workspace, s->ws.rope); g.rope_S = S; g.rope_d = s->d; g.rope_cols = 2 * hl;
    SiteTimer t(s, SITE_QKV_FWD, st);
    TRY(launch_gemm(GEMM_NN, EPI_ROPE, g, st));
  } else {
    TRY(gemm(s, SITE_QKV_FWD, GEMM_NN, EPI_BF16, a.a, h, p.wqkv, 3 * hl, a.qkv, 3 * hl, T, 3 * hl, h, p.bqkv, nullptr, 0, nullptr, 0, st));
    if (s->llama) TIMED(SITE_ROPE, launch_rope(a.qkv, (const float*)P(s->bufs.workspace, s->ws.rope), T, S, s->nh, s->d, 1.f, st));
  }
  TIMED(SITE_ATTN_FWD, launch_attention_fwd(a.qkv, a.o, (float*)a.lse, B, S, s->nh, s->d, s->causal, st));
  TRY(gemm(s, SITE_WO_FWD, GEMM_NN, resid, a.o, hl, p.wo, h, a.x_mid, h, T, h, hl, p.bo, a.x_in, h, nullptr, 0, st));
  TIMED(SITE_NORM_FWD, launch_norm_fwd(s->llama, a.x_mid, p.ln2_g, p.ln2_b, a.c, (float*)a.stats2, T, h, s->eps, st, r32));
  if (!s->llama) {
    TRY(gemm(s, SITE_FC1_FWD, GEMM_NN, EPI_GELU, a.c, h, p.w1, F, a.u, F, T, F, h, p.b1, nullptr, 0, a.g, 0, st));
  } else {
    // gate | up product with silu(gate) * up taken in its epilogue from the fp32 accumulators (u = gate | up is kept for backward)
    GemmArgs g = {};
    g.A = a.c; g.B = p.w1; g.C = a.u; g.C2 = a.g;
    g.lda = h; g.ldb = 2 * F; g.ldc = 2 * F; g.ldc2 = F; g.swiglu_F = F; g.M = T; g.N = 2 * F; g.K = h;
    SiteTimer t(s, SITE_FC1_FWD, st);
    TRY(launch_gemm(GEMM_NN, EPI_SWIGLU, g, st));
  }
  if (y) TRY(gemm(s, SITE_FC2_FWD, GEMM_NN, resid_out, a.g, F, p.w2, h, y, h, T, h, F, p.b2, a.x_mid, h, nullptr, 0, st));
  return hipSuccess;
}

// Lets `to` wait for everything enqueued on `from` so far.  No-op when both are the same stream.
hipError_t stream_order(hipStream_t from, hipStream_t to, hipEvent_t ev) {
  if (from == to) return hipSuccess;
  hipError_t e = hipEventRecord(ev, from);
  return e != hipSuccess ? e : hipStreamWaitEvent(to, ev, 0);
}

// One layer backward.  `st` carries the chain every later kernel depends on (input gradients, attention,
// norms) and the weight-gradient products taken over a whole group; `sd` (the side stream, or st itself)
// carries the per-micro-batch weight-gradient GEMMs and the reductions behind the vector gradients, which only
// the caller's next use of the gradients waits for.  Each side launch is ordered after its producer on st, st
// waits for the side stream before a buffer the side stream still reads is rewritten (du, by attention backward,
// where dqkv shares its buffer) and at the end of the layer (workspace and, with recompute, the shared activation
// working set are reused by the next layer).  bb: where the intermediate gradients go; wp, vp: what happens to
// the matrix and vector gradients now (see WgradPlan, VecPlan).
hipError_t layer_backward(ah_stage* s, int layer, const ActPtrs& a, const void* dy, void* dx, const VecPlan& vp, const BwdBufs& bb,
                          const WgradPlan& wp, hipStream_t st, hipStream_t sd) {
  const LayerPtrs p = layer_ptrs(s, layer);
  const int T = s->T, h = s->h, hl = s->hl, F = s->F, B = s->cfg.microbatch_size, S = s->cfg.seq_len;
  const int Fu = s->llama ? 2 * F : F;
  char* wsb = (char*)s->bufs.workspace;
  char *dmid = bb.dmid, *du = bb.du, *dqkv = bb.dqkv, *dsm = wsb + s->ws.dsm;
  float *part_n2 = vp.n2, *part_n1 = vp.n1, *part_b1 = vp.b1, *part_bqkv = vp.bqkv;
  const int beta = vp.beta;
  float* delta = (float*)(wsb + s->ws.delta);
  const int nb = norm_bwd_blocks(T), cb = colsum_blocks(T);
  const bool rms = s->llama;
  hipEvent_t* ev = s->sync_ev;
#define ON_SIDE(site, expr)              \
  do {                                   \
    SiteTimer t_(s, site, sd);           \
    g_where = #expr;                     \
    hipError_t e_ = (expr);              \
    if (e_ != hipSuccess) return e_;     \
  } while (0)

  // second MLP matrix: dW2 += g^T dy ; input gradient of the activation
  TRY(stream_order(st, sd, ev[0]));  // dy is complete
  TRY(wgrad(s, SITE_FC2_WGRAD, layer, WG_FC2, wp, a.g, dy, p.g_w2, F, h, st, sd));
  if (!s->llama) {
    // du, and as a by-product of its epilogue the column sums of du per 64-row slab (for db1)
    TRY(gemm(s, SITE_FC2_DGRAD, GEMM_NT, EPI_GELU_BWD, dy, h, p.w2, h, du, F, T, F, h, nullptr, a.u, F, nullptr, 0, st, part_b1, vp.acc));
    TRY(stream_order(st, sd, ev[1]));
    if (vp.finish) ON_SIDE(SITE_COLSUM, launch_colsum_finish(part_b1, T / 64, F, p.g_b1, beta, sd));
  } else {
    // d(gate | up) straight from the product dm = dy Wd^T: the SwiGLU backward is the GEMM's epilogue
    GemmArgs g = {};
    g.A = dy; g.B = p.w2; g.C = du; g.aux = a.u;
    g.lda = h; g.ldb = h; g.ldc = 2 * F; g.ld_aux = 2 * F; g.swiglu_F = F; g.M = T; g.N = F; g.K = h;
    {
      SiteTimer t(s, SITE_FC2_DGRAD, st);
      TRY(launch_gemm(GEMM_NT, EPI_SWIGLU_BWD, g, st));
    }
    TRY(stream_order(st, sd, ev[1]));
  }
  TRY(wgrad(s, SITE_FC1_WGRAD, layer, WG_FC1, wp, a.c, du, p.g_w1, h, Fu, st, sd));
  TRY(gemm(s, SITE_FC1_DGRAD, GEMM_NT, EPI_BF16, du, Fu, p.w1, Fu, dsm, h, T, h, Fu, nullptr, nullptr, 0, nullptr, 0, st));  // dc
  // The side stream is done with du.  Only attention backward may have to wait for that, and only where dqkv
  // shares du's buffer; an event nobody waits for is not recorded.
  const bool du_reused = sd != st && dqkv == du;
  if (du_reused) TRY(hipEventRecord(ev[2], sd));
  // second norm backward; dx_mid = dy + norm_bwd(dc); column sums give d(gain), d(offset), d(b2)
  TIMED(SITE_NORM_BWD, launch_norm_bwd(rms, dsm, a.x_mid, (const float*)a.stats2, p.ln2_g, dy, dmid, part_n2, T, h, st, vp.acc, s->res32));
  TRY(stream_order(st, sd, ev[3]));
  if (vp.finish) {
    if (rms) ON_SIDE(SITE_COLSUM, launch_colsum_finish(part_n2, nb, h, p.g_ln2_g, beta, sd));
    else ON_SIDE(SITE_COLSUM, launch_colsum_finish3(part_n2, nb, h, p.g_ln2_g, p.g_ln2_b, p.g_b2, beta, sd));
  }
  // output projection
  TRY(wgrad(s, SITE_WO_WGRAD, layer, WG_WO, wp, a.o, dmid, p.g_wo, hl, h, st, sd));
  TRY(gemm(s, SITE_WO_DGRAD, GEMM_NT, EPI_BF16, dmid, h, p.wo, h, dsm, hl, T, hl, h, nullptr, nullptr, 0, nullptr, 0, st));  // do
  // attention (where dqkv shares its buffer with du: wait until the first MLP matrix's weight gradient has read it)
  if (du_reused) TRY(hipStreamWaitEvent(st, ev[2], 0));
  TIMED(SITE_ATTN_BWD, launch_attention_bwd(a.qkv, a.o, (const float*)a.lse, dsm, dqkv, delta, B, S, s->nh, s->d, s->causal, st));
  if (s->llama) TIMED(SITE_ROPE, launch_rope(dqkv, (const float*)P(s->bufs.workspace, s->ws.rope), T, S, s->nh, s->d, -1.f, st));
  TRY(stream_order(st, sd, ev[4]));
  if (!s->llama) {
    ON_SIDE(SITE_COLSUM, launch_colsum_partial(dqkv, T, 3 * hl, 3 * hl, part_bqkv, sd, vp.acc));
    if (vp.finish) ON_SIDE(SITE_COLSUM, launch_colsum_finish(part_bqkv, cb, 3 * hl, p.g_bqkv, beta, sd));
  }
  TRY(wgrad(s, SITE_QKV_WGRAD, layer, WG_QKV, wp, a.a, dqkv, p.g_wqkv, h, 3 * hl, st, sd));
  TRY(gemm(s, SITE_QKV_DGRAD, GEMM_NT, EPI_BF16, dqkv, 3 * hl, p.wqkv, 3 * hl, dsm, h, T, h, 3 * hl, nullptr, nullptr, 0, nullptr, 0, st));  // da
  // first norm backward; dx = dx_mid + norm_bwd(da); column sums give d(gain), d(offset), d(bo)
  TIMED(SITE_NORM_BWD, launch_norm_bwd(rms, dsm, a.x_in, (const float*)a.stats1, p.ln1_g, dmid, dx, part_n1, T, h, st, vp.acc, s->res32));
  TRY(stream_order(st, sd, ev[5]));
  if (vp.finish) {
    if (rms) ON_SIDE(SITE_COLSUM, launch_colsum_finish(part_n1, nb, h, p.g_ln1_g, beta, sd));
    else ON_SIDE(SITE_COLSUM, launch_colsum_finish3(part_n1, nb, h, p.g_ln1_g, p.g_ln1_b, p.g_bo, beta, sd));
  }
  TRY(stream_order(sd, st, ev[6]));  // join
#undef ON_SIDE
  return hipSuccess;
}

// The side stream and its events, created on the first backward pass (the device of the caller's buffers is
// current then).  AH_NO_SIDE_STREAM in the environment keeps everything on the caller's stream (tuning aid).
hipError_t ensure_side(ah_stage* s) {
  if (s->side_ready || s->side_off) return hipSuccess;
  if (getenv("AH_NO_SIDE_STREAM")) { s->side_off = true; return hipSuccess; }
  hipError_t e = hipStreamCreateWithFlags(&s->side, hipStreamNonBlocking);
  if (e != hipSuccess) return e;
  for (auto& v : s->sync_ev) {
    e = hipEventCreateWithFlags(&v, hipEventDisableTiming);
    if (e != hipSuccess) return e;
  }
  s->side_ready = true;
  return hipSuccess;
}

hipError_t ensure_rope(ah_stage* s, hipStream_t st) {
  if (!s->llama || s->rope_ready) return hipSuccess;
  const int S = s->cfg.seq_len, half = s->d / 2;
  hipLaunchKernelGGL(rope_table_kernel, dim3((S * half + 255) / 256), dim3(256), 0, st, (float*)P(s->bufs.workspace, s->ws.rope), S,
                     half, s->d, (double)s->rope_base);
  s->rope_ready = true;
  return hipGetLastError();
}

hipError_t stage_forward(ah_stage* s, int slot, const void* x, void* y, hipStream_t st, hipEvent_t* ev) {
  TRY(ensure_rope(s, st));
  if (s->res32) TRY(launch_widen(act_ptrs(s, slot, 0).x_in, x, (size_t)s->T * s->h, st));
  else TRY(launch_copy(act_ptrs(s, slot, 0).x_in, x, (size_t)s->T * s->h * 2, st));
  if (ev) TRY(hipEventRecord(ev[0], st));
  for (int l = 0; l < s->L; l++) {
    const ActPtrs a = act_ptrs(s, slot, l);
    void* out = (l + 1 < s->L) ? (void*)act_ptrs(s, slot, l + 1).x_in : y;
    TRY(layer_forward(s, l, a, out, l + 1 == s->L, st));
    if (ev) TRY(hipEventRecord(ev[l + 1], st));
  }
  return hipSuccess;
}

hipError_t finish_vectors(ah_stage* s, int layer, const VecPlan& vp, hipStream_t st) {
  const LayerPtrs p = layer_ptrs(s, layer);
  const int T = s->T, h = s->h, hl = s->hl, F = s->F, nb = norm_bwd_blocks(T), cb = colsum_blocks(T);
  if (s->llama) {
    TIMED(SITE_COLSUM, launch_colsum_finish(vp.n2, nb, h, p.g_ln2_g, vp.beta, st));
    TIMED(SITE_COLSUM, launch_colsum_finish(vp.n1, nb, h, p.g_ln1_g, vp.beta, st));
  } else {
    TIMED(SITE_COLSUM, launch_colsum_finish(vp.b1, T / 64, F, p.g_b1, vp.beta, st));
    TIMED(SITE_COLSUM, launch_colsum_finish3(vp.n2, nb, h, p.g_ln2_g, p.g_ln2_b, p.g_b2, vp.beta, st));
    TIMED(SITE_COLSUM, launch_colsum_finish(vp.bqkv, cb, 3 * hl, p.g_bqkv, vp.beta, st));
    TIMED(SITE_COLSUM, launch_colsum_finish3(vp.n1, nb, h, p.g_ln1_g, p.g_ln1_b, p.g_bo, vp.beta, st));
  }
  return hipSuccess;
}

// The gradients still owed to the micro-batches waiting in pend_slots (every layer's deferred weight-gradient
// products over them, and the vector gradients from the layers' partial sums); frees their slots.
hipError_t flush_wgrads(ah_stage* s, hipStream_t st) {
  const int n = (int)s->pend_slots.size();
  if (n == 0) return hipSuccess;
  WgradPlan wp = {};
  wp.nseg = n;
  wp.beta = s->overwrite_wgrads ? 0 : 1;
  for (int i = 0; i < n; i++) wp.slots[i] = s->pend_slots[i];
  const int h = s->h, hl = s->hl, F = s->F, Fu = s->llama ? 2 * F : F;
  for (int l = s->L - 1; l >= 0; l--) {
    const LayerPtrs p = layer_ptrs(s, l);
    TRY(wgrad(s, SITE_FC2_WGRAD, l, WG_FC2, wp, nullptr, nullptr, p.g_w2, F, h, st, st));
    TRY(wgrad(s, SITE_FC1_WGRAD, l, WG_FC1, wp, nullptr, nullptr, p.g_w1, h, Fu, st, st));
    TRY(wgrad(s, SITE_WO_WGRAD, l, WG_WO, wp, nullptr, nullptr, p.g_wo, hl, h, st, st));
    TRY(wgrad(s, SITE_QKV_WGRAD, l, WG_QKV, wp, nullptr, nullptr, p.g_wqkv, h, 3 * hl, st, st));
    TRY(finish_vectors(s, l, vec_plan(s, l, true, n, true, 0, wp.beta), st));
  }
  for (int i = 0; i < n; i++) s->busy[s->pend_slots[i]] = 0;
  s->pend_slots.clear();
  s->overwrite_wgrads = false;
  return hipSuccess;
}

// Backward of one micro-batch.  Undeferred, every layer takes its weight gradients at once.  Deferred
// (group > 1), the micro-batch's output-gradient operands are written into the pending block of its position in
// the group; the last micro-batch of a group takes the products for the whole group, layer by layer as its own
// backward passes each layer (so they overlap the rest of backward on the side stream), and frees the group's slots.
hipError_t stage_backward(ah_stage* s, int slot, const void* dy, void* dx, hipStream_t st, hipEvent_t* ev) {
  const int beta = s->overwrite_grads ? 0 : 1;
  char* wsb = (char*)s->bufs.workspace;
  const bool deferred = s->group > 1 && !s->force_immediate;
  const int pos = deferred ? (int)s->pend_slots.size() : 0;
  const bool closes_group = deferred && pos + 1 == s->group;
  WgradPlan wp = {};
  wp.nseg = !deferred ? 0 : closes_group ? s->group : -1;
  wp.beta = deferred ? (s->overwrite_wgrads ? 0 : 1) : beta;
  wp.beta_now = beta;
  if (closes_group) {
    for (int i = 0; i < pos; i++) wp.slots[i] = s->pend_slots[i];
    wp.slots[pos] = slot;
  }
  const void* cur = dy;
  TRY(ensure_side(s));
  // per-site timing wants one kernel at a time: a trace keeps everything on the caller's stream
  const bool streams_ok = s->side_ready && !s->tracing;
  // With every matrix deferred only the small reductions would be left for the side stream, and beside the main
  // chain they cost more than they hide (75.4 vs 75.1 ms per step): everything stays on the caller's stream then.
  const bool all_deferred = deferred && s->defer_matrix[0] && s->defer_matrix[1] && s->defer_matrix[2] && s->defer_matrix[3];
  const hipStream_t sd = (streams_ok && !all_deferred) ? s->side : st;
  if (deferred) {  // the caller may reuse dy once this call's work has run: keep a copy for the deferred product
    char* keep;
    (void)pend_bufs(s, pos, s->L - 1, &keep);
    TRY(launch_copy(keep, dy, (size_t)s->T * s->h * 2, st));
    cur = keep;
  }
  if (ev) TRY(hipEventRecord(ev[s->L], st));
  for (int l = s->L - 1; l >= 0; l--) {
    const ActPtrs a = act_ptrs(s, slot, l);
    if (s->recompute) TRY(layer_forward(s, l, a, nullptr, false, st));
    BwdBufs bb = {wsb + s->ws.dmid, wsb + s->ws.dbig, wsb + s->ws.dbig};
    void* out = (l == 0) ? dx : (void*)(wsb + ((l & 1) ? s->ws.d1 : s->ws.d0));
    if (deferred) {
      bb = pend_bufs(s, pos, l, nullptr);
      if (l > 0) {
        char* next_dy;
        (void)pend_bufs(s, pos, l - 1, &next_dy);
        out = next_dy;
      }
    }
    const VecPlan vp = vec_plan(s, l, deferred, pos, closes_group, beta, wp.beta);
    TRY(layer_backward(s, l, a, cur, out, vp, bb, wp, st, sd));
    cur = out;
    if (ev) TRY(hipEventRecord(ev[l], st));
  }
  s->overwrite_grads = false;
  if (!deferred) {
    s->overwrite_wgrads = false;
    s->busy[slot] = 0;
  } else if (closes_group) {
    for (int i = 0; i < pos; i++) s->busy[s->pend_slots[i]] = 0;
    s->busy[slot] = 0;
    s->pend_slots.clear();
    s->overwrite_wgrads = false;
  } else {
    s->pend_slots.push_back(slot);
    s->busy[slot] = 2;
  }
  return hipSuccess;
}

// A step with deferred weight gradients (group > 1) is not offered for HIP graph capture: replaying such a capture
// has ended in a host-side fault inside the graph launch whose cause is not known, so the two calls that belong to
// that mode refuse a capturing stream instead of recording something that may not replay.
int refuse_capture_of_groups(const ah_stage* s, hipStream_t st, const char* who) {
  if (s->group <= 1) return AH_OK;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cs) != hipSuccess) { (void)hipGetLastError(); return AH_OK; }  // the legacy default stream cannot be queried while another stream captures
  if (cs == hipStreamCaptureStatusNone) return AH_OK;
  return set_error(AH_EUNSUPPORTED, "%s: the stream is being captured into a HIP graph and wgrad_group is %d; graph capture is supported for wgrad_group <= 1 only", who, s->group);
}

float median(std::vector<float>& v) {
  std::sort(v.begin(), v.end());
  return v.empty() ? 0.f : v[v.size() / 2];
}

}  // namespace

extern "C" int ah_stage_query_sizes(const ah_stage_config_t* cfg, ah_stage_sizes_t* out) {
  if (!out) return set_error(AH_EINVAL, "ah_stage_query_sizes: out is NULL");
  int rc = validate(cfg);
  if (rc) return rc;
  ah_stage tmp;
  plan(&tmp, cfg);
  out->param_elems = tmp.layer_elems * tmp.L;
  out->param_bytes = out->param_elems * 2;
  out->grad_bytes = out->param_elems * 4;
  out->activation_bytes_per_slot = tmp.slot_bytes;
  out->activation_bytes_per_layer_per_slot = tmp.per_layer_slot_bytes;
  out->workspace_bytes = tmp.ws.bytes;
  return AH_OK;
}

extern "C" int ah_stage_create(const ah_stage_config_t* cfg, const ah_stage_buffers_t* bufs, ah_stage_t** out) {
  if (!out) return set_error(AH_EINVAL, "ah_stage_create: out is NULL");
  *out = nullptr;
  int rc = validate(cfg);
  if (rc) return rc;
  if (!bufs || !bufs->params || !bufs->grads || !bufs->activations || !bufs->workspace)
    return set_error(AH_EINVAL, "ah_stage_create: all four buffers are required");
  if (((uintptr_t)bufs->params | (uintptr_t)bufs->grads | (uintptr_t)bufs->activations | (uintptr_t)bufs->workspace) & 255)
    return set_error(AH_EINVAL, "ah_stage_create: buffers must be 256-byte aligned");
  ah_stage* s = new (std::nothrow) ah_stage();
  if (!s) return set_error(AH_ENOMEM, "ah_stage_create: out of host memory");
  plan(s, cfg);
  s->bufs = *bufs;
  s->busy.assign(cfg->max_in_flight, 0);
  s->overwrite_grads = true;
  s->overwrite_wgrads = true;
  s->force_immediate = false;
  s->rope_ready = false;
  s->side = nullptr;
  s->side_ready = false;
  s->side_off = false;
  s->tracing = false;
  s->ev_used = 0;
  *out = s;
  return AH_OK;
}

extern "C" int ah_stage_destroy(ah_stage_t* st) {
  if (st) {
    for (hipEvent_t e : st->ev_pool) (void)hipEventDestroy(e);
    if (st->side_ready) {
      (void)hipStreamSynchronize(st->side);
      for (hipEvent_t e : st->sync_ev) (void)hipEventDestroy(e);
      (void)hipStreamDestroy(st->side);
    }
  }
  delete st;
  return AH_OK;
}

extern "C" int ah_stage_param_layout(const ah_stage_t* st, int layer, int which, uint64_t* elem_offset, int32_t* rows, int32_t* cols) {
  if (!st || !elem_offset || !rows || !cols) return set_error(AH_EINVAL, "ah_stage_param_layout: NULL argument");
  if (layer < 0 || layer >= st->L || which < 0 || which >= AH_P_COUNT) return set_error(AH_EINVAL, "ah_stage_param_layout: layer %d / tensor %d out of range", layer, which);
  if (!st->ptab[which].cols) return set_error(AH_EINVAL, "ah_stage_param_layout: tensor %d does not exist in this architecture", which);
  *elem_offset = (uint64_t)layer * st->layer_elems + st->ptab[which].off;
  *rows = st->ptab[which].rows;
  *cols = st->ptab[which].cols;
  return AH_OK;
}

extern "C" int ah_stage_forward(ah_stage_t* st, int slot, const void* x, void* y, void* stream) {
  discard_stale_hip_error();
  if (!st || !x || !y) return set_error(AH_EINVAL, "ah_stage_forward: NULL argument");
  if (slot < 0 || slot >= (int)st->busy.size()) return set_error(AH_EINVAL, "ah_stage_forward: slot %d out of range [0, %zu)", slot, st->busy.size());
  if (st->busy[slot] == 2) return set_error(AH_ESTATE, "ah_stage_forward: slot %d holds a micro-batch whose weight gradients are pending (its group is not complete: ah_stage_flush_grads)", slot);
  if (st->busy[slot]) return set_error(AH_ESTATE, "ah_stage_forward: slot %d still holds a micro-batch awaiting backward", slot);
  int rc = hip_status(stage_forward(st, slot, x, y, (hipStream_t)stream, nullptr), "ah_stage_forward");
  if (rc == AH_OK) st->busy[slot] = 1;
  return rc;
}

extern "C" int ah_stage_backward(ah_stage_t* st, int slot, const void* dy, void* dx, void* stream) {
  discard_stale_hip_error();
  if (!st || !dy || !dx) return set_error(AH_EINVAL, "ah_stage_backward: NULL argument");
  if (slot < 0 || slot >= (int)st->busy.size()) return set_error(AH_EINVAL, "ah_stage_backward: slot %d out of range [0, %zu)", slot, st->busy.size());
  if (st->busy[slot] != 1) return set_error(AH_ESTATE, "ah_stage_backward: slot %d holds no forward pass awaiting backward", slot);
  if (int rc = refuse_capture_of_groups(st, (hipStream_t)stream, "ah_stage_backward")) return rc;
  return hip_status(stage_backward(st, slot, dy, dx, (hipStream_t)stream, nullptr), "ah_stage_backward");
}

extern "C" int ah_stage_flush_grads(ah_stage_t* st, void* stream) {
  discard_stale_hip_error();
  if (!st) return set_error(AH_EINVAL, "ah_stage_flush_grads: NULL argument");
  if (int rc = refuse_capture_of_groups(st, (hipStream_t)stream, "ah_stage_flush_grads")) return rc;
  return hip_status(flush_wgrads(st, (hipStream_t)stream), "ah_stage_flush_grads");
}

extern "C" int ah_stage_grads(ah_stage_t* st, float** dev_ptr, uint64_t* n_elems) {
  if (!st || !dev_ptr || !n_elems) return set_error(AH_EINVAL, "ah_stage_grads: NULL argument");
  *dev_ptr = (float*)st->bufs.grads;
  *n_elems = st->layer_elems * st->L;
  return AH_OK;
}

extern "C" int ah_stage_layer_input(ah_stage_t* st, int slot, int layer, const void** dev_ptr) {
  if (!st || !dev_ptr) return set_error(AH_EINVAL, "ah_stage_layer_input: NULL argument");
  if (slot < 0 || slot >= (int)st->busy.size()) return set_error(AH_EINVAL, "ah_stage_layer_input: slot %d out of range [0, %zu)", slot, st->busy.size());
  if (layer < 0 || layer >= st->L) return set_error(AH_EINVAL, "ah_stage_layer_input: layer %d out of range [0, %d)", layer, st->L);
  *dev_ptr = act_ptrs(st, slot, layer).x_in;
  return AH_OK;
}

extern "C" int ah_stage_zero_grads(ah_stage_t* st, void* /*stream*/) {
  if (!st) return set_error(AH_EINVAL, "ah_stage_zero_grads: NULL argument");
  if (!st->pend_slots.empty()) return set_error(AH_ESTATE, "ah_stage_zero_grads: %zu micro-batches still wait for their weight gradients (ah_stage_flush_grads first)", st->pend_slots.size());
  st->overwrite_grads = true;
  st->overwrite_wgrads = true;
  return AH_OK;
}

extern "C" int ah_stage_profile(ah_stage_t* st, int warmup, int iters, ah_stage_profile_t* out) {
  discard_stale_hip_error();
  if (!st || !out) return set_error(AH_EINVAL, "ah_stage_profile: NULL argument");
  if (out->struct_size != sizeof(ah_stage_profile_t)) return set_error(AH_EINVAL, "ah_stage_profile: struct_size mismatch");
  if (out->n_layers < st->L || !out->fwd_ms || !out->bwd_ms) return set_error(AH_EINVAL, "ah_stage_profile: fwd_ms/bwd_ms must hold n_layers entries");
  if (warmup < 0 || iters < 1 || iters > 10000) return set_error(AH_EINVAL, "ah_stage_profile: warmup >= 0 and 1 <= iters <= 10000 required");
  for (char b : st->busy)
    if (b) return set_error(AH_ESTATE, "ah_stage_profile: all slots must be empty");
  const int L = st->L, K = st->cfg.n_microbatches;
  char* wsb = (char*)st->bufs.workspace;
  __bf16* px = (__bf16*)(wsb + st->ws.prof_x);
  __bf16* pdy = (__bf16*)(wsb + st->ws.prof_dy);
  const size_t n = (size_t)st->T * st->h;
  hipStream_t s = nullptr;
  std::vector<hipEvent_t> ef(L + 1), eb(L + 1);
  hipEvent_t it0, it1;
  hipError_t e = hipSuccess;
  for (auto& v : ef) if (e == hipSuccess) e = hipEventCreate(&v);
  for (auto& v : eb) if (e == hipSuccess) e = hipEventCreate(&v);
  if (e == hipSuccess) e = hipEventCreate(&it0);
  if (e == hipSuccess) e = hipEventCreate(&it1);
  if (e != hipSuccess) return hip_status(e, "ah_stage_profile (events)");
  hipLaunchKernelGGL(fill_pattern_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, px, n, 1u);
  hipLaunchKernelGGL(fill_pattern_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, pdy, n, 2u);
  void* y = wsb + st->ws.prof_y;
  void* dx = wsb + st->ws.prof_dx;
  std::vector<std::vector<float>> tf(L), tb(L);
  std::vector<float> sf, sb, ti;
  st->force_immediate = true;  // a layer's backward time includes its weight gradients
  for (int it = 0; it < warmup + iters && e == hipSuccess; it++) {
    st->overwrite_grads = st->overwrite_wgrads = true;
    e = stage_forward(st, 0, px, y, s, ef.data());
    if (e == hipSuccess) e = stage_backward(st, 0, pdy, dx, s, eb.data());
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess || it < warmup) continue;
    float ms;
    for (int l = 0; l < L; l++) {
      (void)hipEventElapsedTime(&ms, ef[l], ef[l + 1]); tf[l].push_back(ms);
      (void)hipEventElapsedTime(&ms, eb[l + 1], eb[l]); tb[l].push_back(ms);
    }
    (void)hipEventElapsedTime(&ms, ef[0], ef[L]); sf.push_back(ms);
    (void)hipEventElapsedTime(&ms, eb[L], eb[0]); sb.push_back(ms);
  }
  st->force_immediate = false;
  // the iteration as configured: with deferred weight gradients each micro-batch of a group takes a slot of its own
  const int nslots = (int)st->busy.size();
  for (int it = 0; it < std::min(warmup, 2) + iters && e == hipSuccess; it++) {
    st->overwrite_grads = st->overwrite_wgrads = true;
    e = hipEventRecord(it0, s);
    for (int k = 0; k < K && e == hipSuccess; k++) {
      const int slot = st->group > 1 ? k % nslots : 0;
      e = stage_forward(st, slot, px, y, s, nullptr);
      if (e == hipSuccess) e = stage_backward(st, slot, pdy, dx, s, nullptr);
    }
    if (e == hipSuccess) e = flush_wgrads(st, s);
    if (e == hipSuccess) e = hipEventRecord(it1, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    float ms;
    if (e == hipSuccess && it >= std::min(warmup, 2)) { (void)hipEventElapsedTime(&ms, it0, it1); ti.push_back(ms); }
  }
  for (auto& v : ef) (void)hipEventDestroy(v);
  for (auto& v : eb) (void)hipEventDestroy(v);
  (void)hipEventDestroy(it0);
  (void)hipEventDestroy(it1);
  st->force_immediate = false;
  st->pend_slots.clear();
  std::fill(st->busy.begin(), st->busy.end(), 0);
  st->overwrite_grads = st->overwrite_wgrads = true;
  if (e != hipSuccess) return hip_status(e, "ah_stage_profile");
  for (int l = 0; l < L; l++) { out->fwd_ms[l] = median(tf[l]); out->bwd_ms[l] = median(tb[l]); }
  out->stage_fwd_ms = median(sf);
  out->stage_bwd_ms = median(sb);
  out->iteration_ms = median(ti);
  out->peak_activation_bytes = (uint64_t)st->busy.size() * st->slot_bytes + st->ws.bytes;
  out->activation_bytes_per_layer_per_slot = st->per_layer_slot_bytes;
  out->param_bytes = st->layer_elems * st->L * 2;
  out->grad_bytes = st->layer_elems * st->L * 4;
  return AH_OK;
}

extern "C" int ah_stage_trace_begin(ah_stage_t* st) {
  if (!st) return set_error(AH_EINVAL, "ah_stage_trace_begin: NULL argument");
  st->tracing = true;
  st->ev_used = 0;
  return AH_OK;
}

extern "C" int ah_stage_trace_end(ah_stage_t* st, ah_trace_entry_t* out, int capacity, int* n_out) {
  if (!st || !out || !n_out || capacity < 1) return set_error(AH_EINVAL, "ah_stage_trace_end: NULL argument or no capacity");
  if (!st->tracing) return set_error(AH_ESTATE, "ah_stage_trace_end: no trace in progress");
  st->tracing = false;
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) return hip_status(e, "ah_stage_trace_end");
  double total[SITE_COUNT] = {0};
  long launches[SITE_COUNT] = {0}, mults[SITE_COUNT] = {0};
  for (size_t i = 0; i + 1 < st->ev_used; i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, st->ev_pool[i], st->ev_pool[i + 1]) != hipSuccess) continue;
    total[st->ev_site[i / 2]] += ms;
    launches[st->ev_site[i / 2]]++;
    mults[st->ev_site[i / 2]] += st->ev_mult[i / 2];
  }
  st->ev_used = 0;
  // algorithmic work per launch: 2*M*N*K flops for the GEMMs, causal-half flops for masked attention (all S*S pairs without the mask)
  // (forward 4*d*S*(S+1)/2 per head, backward 2.5x that as executed by the recompute-in-tile scheme
  // counts as 2x model flops), bytes moved once for the bandwidth-bound kernels.
  const double T = st->T, h = st->h, hl = st->hl, F = st->F, Fu = st->llama ? 2.0 * st->F : st->F;
  const double S = st->cfg.seq_len, B = st->cfg.microbatch_size;
  const double attn = 4.0 * st->d * (st->causal ? S * (S + 1) / 2 : S * S) * st->nh * B;
  double flops[SITE_COUNT] = {0}, bytes[SITE_COUNT] = {0};
  flops[SITE_QKV_FWD] = flops[SITE_QKV_WGRAD] = flops[SITE_QKV_DGRAD] = 2 * T * h * 3 * hl;
  flops[SITE_WO_FWD] = flops[SITE_WO_WGRAD] = flops[SITE_WO_DGRAD] = 2 * T * hl * h;
  flops[SITE_FC1_FWD] = flops[SITE_FC1_WGRAD] = flops[SITE_FC1_DGRAD] = 2 * T * h * Fu;
  flops[SITE_FC2_FWD] = flops[SITE_FC2_WGRAD] = flops[SITE_FC2_DGRAD] = 2 * T * F * h;
  flops[SITE_ATTN_FWD] = attn;
  flops[SITE_ATTN_BWD] = 2 * attn;
  bytes[SITE_NORM_FWD] = 4 * T * h + 8 * T;
  bytes[SITE_NORM_BWD] = 8 * T * h + 8 * T;
  bytes[SITE_ROPE] = 2 * (2 * T * 2 * hl);
  int n = 0;
  for (int sidx = 0; sidx < SITE_COUNT && n < capacity; sidx++) {
    if (!launches[sidx]) continue;
    ah_trace_entry_t& o = out[n++];
    snprintf(o.name, sizeof o.name, "%s", kSiteNames[sidx]);
    o.launches = launches[sidx];
    o.total_ms = total[sidx];
    o.flops_per_launch = flops[sidx] * ((double)mults[sidx] / launches[sidx]);  // deferred weight gradients cover several micro-batches per launch
    o.bytes_per_launch = bytes[sidx];
  }
  *n_out = n;
  return AH_OK;
}

extern "C" int ah_attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int nh, int d, int causal, void* stream) {
  discard_stale_hip_error();
  if (!qkv || !o || !lse) return set_error(AH_EINVAL, "ah_attention_fwd: NULL pointer");
  if (B < 1 || nh < 1 || S < 1 || S % 128 || (d != 64 && d != 128)) return set_error(AH_EUNSUPPORTED, "ah_attention_fwd: need S %% 128 == 0 and d in {64, 128}");
  return hip_status(launch_attention_fwd(qkv, o, lse, B, S, nh, d, causal != 0, (hipStream_t)stream), "ah_attention_fwd");
}

extern "C" int ah_attention_bwd(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, float* delta, int B,
                                int S, int nh, int d, int causal, void* stream) {
  discard_stale_hip_error();
  if (!qkv || !o || !lse || !d_o || !dqkv || !delta) return set_error(AH_EINVAL, "ah_attention_bwd: NULL pointer");
  if (B < 1 || nh < 1 || S < 1 || S % 128 || (d != 64 && d != 128)) return set_error(AH_EUNSUPPORTED, "ah_attention_bwd: need S %% 128 == 0 and d in {64, 128}");
  return hip_status(launch_attention_bwd(qkv, o, lse, d_o, dqkv, delta, B, S, nh, d, causal != 0, (hipStream_t)stream), "ah_attention_bwd");
}

// ---- the entry point that allocates nothing: attention backward with its scratch in the device image
namespace {
// One copy per GPU, at its own address on each; in host code the name below is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) float scratch[AH_ATTENTION_STATIC_MAX_ROWS];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, looked up once
std::mutex g_scratch_mu;
}  // namespace

extern "C" int ah_attention_bwd_static(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, int B, int S,
                                       int nh, int d, int causal, void* stream) {
  discard_stale_hip_error();
  if (!qkv || !o || !lse || !d_o || !dqkv) return set_error(AH_EINVAL, "ah_attention_bwd_static: NULL pointer");
  if (B < 1 || nh < 1 || S < 1 || S % 128 || (d != 64 && d != 128)) return set_error(AH_EUNSUPPORTED, "ah_attention_bwd_static: need S %% 128 == 0 and d in {64, 128}");
  if ((long)B * nh * S > (long)AH_ATTENTION_STATIC_MAX_ROWS)
    return set_error(AH_EINVAL, "ah_attention_bwd_static: B * nh * S = %ld exceeds the fixed scratch of %d rows (use ah_attention_bwd with a caller-supplied buffer)", (long)B * nh * S, AH_ATTENTION_STATIC_MAX_ROWS);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_status(e, "ah_attention_bwd_static (hipGetDevice)");
  if (dev < 0 || dev >= kMaxDevices) return set_error(AH_EUNSUPPORTED, "ah_attention_bwd_static: device index %d out of range", dev);
  float* delta;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) return hip_status(e != hipSuccess ? e : hipErrorInvalidSymbol, "ah_attention_bwd_static (hipGetSymbolAddress)");
      g_scratch_ptr[dev] = (float*)p;
    }
    delta = g_scratch_ptr[dev];
  }
  return hip_status(launch_attention_bwd(qkv, o, lse, d_o, dqkv, delta, B, S, nh, d, causal != 0, (hipStream_t)stream), "ah_attention_bwd_static");
}
