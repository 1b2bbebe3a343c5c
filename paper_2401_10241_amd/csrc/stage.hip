// Host side of the zero-bubble stage library: the C ABI of include/zb_stage.h, the per-stage pass
// order of 1F1B / ZB-H1 / ZB-H2, the stash pools with the F -> B -> W life cycle, the pass
// executors and the post-validated optimizer protocol.  All arithmetic runs in the HIP kernels
// declared in zb_common.h; nothing here computes on the CPU.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <string>
#include <vector>

#include "../../include/zb_stage.h"
#include "zb_common.h"

using namespace zb;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

struct Bump {  // carves the arena; with base == nullptr it only measures
  char* base;
  size_t off = 0;
  explicit Bump(void* b) : base((char*)b) {}
  template <typename T> T* take(size_t bytes) {
    off = align_up(off);
    T* p = base ? (T*)(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

struct LayerOff {  // byte offsets inside one slot of each pool
  size_t fb_x, fb_qkv, fb_y1, fb_fh, fb_stats1, fb_stats2, fb_lse;
  size_t fw_a, fw_c, fw_u, fw_g;
  size_t bw_dqkv, bw_dy1, bw_dfh, bw_dy;
};

enum KClass {
  KC_GEMM_FWD = 0, KC_GEMM_DGRAD, KC_GEMM_WGRAD, KC_ATTN_FWD, KC_ATTN_BWD, KC_LN_FWD, KC_LN_BWD, KC_COLSUM,
  KC_FILL, KC_SUMSQ, KC_ADAMW_STEP, KC_ADAMW_ROLLBACK, KC_ADAMW_RESTEP, KC_TRANSPOSE, KC_EMBED, KC_LOSS, KC_COUNT
};
const char* const kClassNames[KC_COUNT] = {
    "gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attention_fwd", "attention_bwd", "layernorm_fwd", "layernorm_bwd",
    "bias_grad_colsum", "grad_zero_fill", "grad_sumsq", "adamw_step", "adamw_rollback", "adamw_restep",
    "weight_transpose", "embedding", "cross_entropy"};

struct ProfRec {
  int cls;
  hipEvent_t a, b;
};

}  // namespace

struct zb_stage {
  zb_config cfg;
  hipStream_t stream = nullptr;
  bool bf16 = true;
  bool group_w = true;
  bool fuse_bw = false;
  int chunks = 1;  // model chunks held by the stage (2: ZB-V); microbatch indices are then virtual, chunk-major
  int L = 0, h = 0, a = 0, ffn = 0, s = 0, b = 0, T = 0, d = 0;
  size_t esz = 2;

  // flat fp32 vectors: [layer][param], each tensor padded to 64 floats
  size_t flat_count = 0;
  std::vector<size_t> poff;  // L * ZB_P_COUNT
  size_t pcount[ZB_P_COUNT];
  float *theta = nullptr, *grad = nullptr, *adam_m = nullptr, *adam_v = nullptr;
  float *j_theta = nullptr, *j_m = nullptr, *j_v = nullptr;
  bf16_t* theta16 = nullptr;
  bf16_t* theta16_t = nullptr;  // the four weight matrices transposed ([out][in]), for the dgrad GEMMs

  char *in_x = nullptr, *in_dy = nullptr, *out_y = nullptr, *out_dx = nullptr;
  size_t act_bytes = 0;  // one [T, h] tensor

  char *fb_pool = nullptr, *fw_pool = nullptr, *bw_pool = nullptr;
  size_t fb_slot = 0, fw_slot = 0, bw_slot = 0;
  std::vector<LayerOff> lo;
  std::vector<int> free_fb, free_fw, free_bw, slot_fb, slot_fw, slot_bw;
  std::vector<unsigned char> done[3];
  int m = 0, iter = 0;

  // first / last stage (Sec. 5.1)
  int role = ZB_ROLE_MIDDLE, V = 0;
  size_t spoff[ZB_SP_COUNT], spcount[ZB_SP_COUNT];  // stage-level tensors in the flat vectors (count 0: absent)
  int *ids = nullptr, *perm = nullptr;  // [max_microbatches][T]: input ids (first) / target ids (last); sorted token order
  float *loss = nullptr, *row_loss = nullptr;
  size_t fb_logits = 0, fb_lse = 0, fb_statsf = 0, fw_z = 0, bw_dlogits = 0;  // last stage: offsets inside the stash slots
  float* SP(int i) const { return theta + spoff[i]; }
  float* SG(int i) const { return grad + spoff[i]; }
  const void* SWt(int i) const { return bf16 ? (const void*)(theta16 + spoff[i]) : (const void*)SP(i); }

  char* tmp = nullptr;  // [T, h] activation-gradient scratch
  float *dvec = nullptr, *ln_partials = nullptr, *staging = nullptr, *gemm_ws = nullptr;
  size_t staging_floats = 0, gemm_ws_floats = 0;
  double* partial_sq = nullptr;
  int* partial_nf = nullptr;
  OptDevState* opt = nullptr;
  OptHyper hp;

  std::string err;
  bool profiling = false;
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> ev_pool;
  double prof_flops[KC_COUNT], prof_bytes[KC_COUNT];

  float* P(int l, int i) const { return theta + poff[l * ZB_P_COUNT + i]; }
  float* G(int l, int i) const { return grad + poff[l * ZB_P_COUNT + i]; }
  const void* Wt(int l, int i) const {
    return bf16 ? (const void*)(theta16 + poff[l * ZB_P_COUNT + i]) : (const void*)P(l, i);
  }
  const void* WtT(int l, int i) const { return theta16_t + poff[l * ZB_P_COUNT + i]; }
};

namespace {

zb_status fail(zb_stage* st, zb_status code, const std::string& msg) {
  if (st) st->err = msg;
  return code;
}
#define ZB_HIP(st, expr)                                                                             \
  do {                                                                                               \
    hipError_t e__ = (expr);                                                                         \
    if (e__ != hipSuccess)                                                                           \
      return fail(st, ZB_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e__));               \
  } while (0)

struct ProfScope {  // brackets one kernel launch with events when profiling is on
  zb_stage* st;
  hipEvent_t b = nullptr;
  bool on;
  ProfScope(zb_stage* s, int cls, double flops, double bytes) : st(s), on(s->profiling) {
    if (!on) return;
    hipEvent_t a = take();
    b = take();
    if (!a || !b) { on = false; return; }
    st->prof.push_back({cls, a, b});
    st->prof_flops[cls] += flops;
    st->prof_bytes[cls] += bytes;
    (void)hipEventRecord(a, st->stream);
  }
  ~ProfScope() {
    if (on) (void)hipEventRecord(b, st->stream);
  }
  hipEvent_t take() {
    if (!st->ev_pool.empty()) {
      hipEvent_t e = st->ev_pool.back();
      st->ev_pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};

bool valid_shapes(const zb_config* c, std::string* why) {
  auto bad = [&](const char* m) { *why = m; return false; };
  if (!c) return bad("null config");
  if (c->layers < 1 || c->hidden < 1 || c->heads < 1 || c->ffn < 1 || c->seq < 1 || c->mb_size < 1)
    return bad("layers, hidden, heads, ffn, seq, mb_size must be positive");
  if (c->hidden % c->heads != 0) return bad("hidden must be a multiple of heads");
  if (c->hidden % 8 != 0 || c->ffn % 8 != 0) return bad("hidden and ffn must be multiples of 8");
  if (c->hidden > 8192) return bad("hidden above 8192 is not supported by the LayerNorm kernels");
  if (c->max_microbatches < 1 || c->max_pending_b < 1 || c->max_pending_w < 1 || c->max_inflight < 1)
    return bad("max_microbatches, max_pending_b, max_pending_w, max_inflight must be positive");
  if (c->dtype != ZB_FP32 && c->dtype != ZB_BF16) return bad("dtype must be ZB_FP32 or ZB_BF16");
  if ((long long)c->seq * c->mb_size > (1 << 24)) return bad("too many tokens per microbatch");
  if (c->chunks != 0 && c->chunks != 1 && c->chunks != 2) return bad("chunks must be 1 or 2");
  if (c->chunks == 2 && c->layers % 2 != 0) return bad("two chunks need an even number of layers");
  if (c->role != ZB_ROLE_MIDDLE && c->role != ZB_ROLE_FIRST && c->role != ZB_ROLE_LAST) return bad("unknown role");
  if (c->role != ZB_ROLE_MIDDLE) {
    if (c->chunks == 2) return bad("a first or last stage cannot hold two chunks");
    if (c->vocab < 1 || c->vocab > kEmbeddingMaxVocab) return bad("vocab must be in [1, 2^18]");
    if (c->role == ZB_ROLE_FIRST && (long long)c->seq * c->mb_size > kEmbeddingMaxTokens)
      return bad("a first stage takes at most 8192 tokens per microbatch");
  }
  return true;
}

// Lays the stage out in the arena (or just measures when arena == nullptr).
size_t layout(zb_stage* st, void* arena) {
  const zb_config& c = st->cfg;
  st->L = c.layers; st->h = c.hidden; st->a = c.heads; st->ffn = c.ffn; st->s = c.seq; st->b = c.mb_size;
  st->T = c.seq * c.mb_size; st->d = c.hidden / c.heads;
  st->bf16 = c.dtype == ZB_BF16;
  st->group_w = c.group_w != 0;
  st->fuse_bw = c.fuse_bw != 0;
  st->chunks = c.chunks == 2 ? 2 : 1;
  st->esz = st->bf16 ? 2 : 4;
  const size_t h = st->h, f = st->ffn, T = st->T;
  const size_t pc[ZB_P_COUNT] = {h, h, h * 3 * h, 3 * h, h * h, h, h, h, h * f, f, f * h, h};
  st->poff.assign((size_t)st->L * ZB_P_COUNT, 0);
  size_t o = 0;
  for (int l = 0; l < st->L; ++l)
    for (int i = 0; i < ZB_P_COUNT; ++i) {
      st->pcount[i] = pc[i];
      st->poff[l * ZB_P_COUNT + i] = o;
      o += align_up(pc[i], 64);
    }
  st->role = c.role;
  st->V = c.role == ZB_ROLE_MIDDLE ? 0 : c.vocab;
  for (int i = 0; i < ZB_SP_COUNT; ++i) st->spoff[i] = st->spcount[i] = 0;
  auto stage_tensor = [&](int i, size_t n) { st->spcount[i] = n; st->spoff[i] = o; o += align_up(n, 64); };
  if (c.role == ZB_ROLE_FIRST) {
    stage_tensor(ZB_SP_EMB_TOK, (size_t)st->V * h);
    stage_tensor(ZB_SP_EMB_POS, (size_t)st->s * h);
  } else if (c.role == ZB_ROLE_LAST) {
    stage_tensor(ZB_SP_LNF_G, h);
    stage_tensor(ZB_SP_LNF_B, h);
    stage_tensor(ZB_SP_W_HEAD, h * (size_t)st->V);
  }
  st->flat_count = o;

  Bump bp(arena);
  const size_t fb = o * sizeof(float);
  st->theta = bp.take<float>(fb);
  st->grad = bp.take<float>(fb);
  st->adam_m = bp.take<float>(fb);
  st->adam_v = bp.take<float>(fb);
  if (c.journal) {
    st->j_theta = bp.take<float>(fb);
    st->j_m = bp.take<float>(fb);
    st->j_v = bp.take<float>(fb);
  }
  if (st->bf16) {
    st->theta16 = bp.take<bf16_t>(o * sizeof(bf16_t));
    st->theta16_t = bp.take<bf16_t>(o * sizeof(bf16_t));
  }

  const size_t E = st->esz;
  st->act_bytes = align_up(T * h * E);
  const size_t io = st->act_bytes * (size_t)c.max_microbatches;
  st->in_x = bp.take<char>(io);
  st->in_dy = bp.take<char>(io);
  st->out_y = bp.take<char>(io);
  st->out_dx = bp.take<char>(io);

  st->lo.assign(st->L, LayerOff());
  size_t ofb = 0, ofw = 0, obw = 0;
  auto put = [&](size_t& cur, size_t bytes) { size_t p = cur; cur += align_up(bytes); return p; };
  for (int l = 0; l < st->L; ++l) {
    LayerOff& q = st->lo[l];
    q.fb_x = put(ofb, l == 0 ? 0 : T * h * E);
    q.fb_qkv = put(ofb, T * 3 * h * E);
    q.fb_y1 = put(ofb, T * h * E);
    q.fb_fh = put(ofb, T * f * E);
    q.fb_stats1 = put(ofb, T * 2 * sizeof(float));
    q.fb_stats2 = put(ofb, T * 2 * sizeof(float));
    q.fb_lse = put(ofb, (size_t)st->b * st->a * st->s * sizeof(float));
    q.fw_a = put(ofw, T * h * E);
    q.fw_c = put(ofw, T * h * E);
    q.fw_u = put(ofw, T * h * E);
    q.fw_g = put(ofw, T * f * E);
    q.bw_dqkv = put(obw, T * 3 * h * E);
    q.bw_dy1 = put(obw, T * h * E);
    q.bw_dfh = put(obw, T * f * E);
    q.bw_dy = put(obw, l == st->L - 1 ? 0 : T * h * E);
  }
  if (c.role == ZB_ROLE_LAST) {  // the head: logits and row statistics F -> B, its input F -> W, its output gradient B -> W
    st->fb_logits = put(ofb, T * (size_t)st->V * E);
    st->fb_lse = put(ofb, T * sizeof(float));
    st->fb_statsf = put(ofb, T * 2 * sizeof(float));
    st->fw_z = put(ofw, T * h * E);
    st->bw_dlogits = put(obw, T * (size_t)st->V * E);
  }
  st->fb_slot = ofb; st->fw_slot = ofw; st->bw_slot = obw;
  st->fb_pool = bp.take<char>(ofb * (size_t)c.max_pending_b);
  st->fw_pool = bp.take<char>(ofw * (size_t)c.max_inflight);
  st->bw_pool = bp.take<char>(obw * (size_t)c.max_pending_w);

  if (c.role != ZB_ROLE_MIDDLE) st->ids = bp.take<int>((size_t)c.max_microbatches * T * sizeof(int));
  if (c.role == ZB_ROLE_FIRST) st->perm = bp.take<int>((size_t)c.max_microbatches * T * sizeof(int));
  if (c.role == ZB_ROLE_LAST) {
    st->loss = bp.take<float>((size_t)c.max_microbatches * sizeof(float));
    st->row_loss = bp.take<float>(T * sizeof(float));
  }
  st->tmp = bp.take<char>(T * h * E);
  st->dvec = bp.take<float>((size_t)st->b * st->a * st->s * sizeof(float));
  {  // LayerNorm-backward partials; the bias-gradient column sums reuse it for their row slices
    size_t need = (size_t)kLnBwdSlices * 2 * h;
    const size_t all_dy = (size_t)h + f + h + 3 * h;  // the four dY of a layer side by side
    if ((size_t)kColsumSlices * all_dy > need) need = (size_t)kColsumSlices * all_dy;
    st->ln_partials = bp.take<float>(need * sizeof(float));
  }
  size_t stg = h * f;
  if (h * 3 * h > stg) stg = h * 3 * h;
  if (T * h > stg) stg = T * h;
  st->staging_floats = stg;
  st->staging = bp.take<float>(stg * sizeof(float));
  if (st->bf16) {  // split-K partial products of the N = hidden GEMMs (up to 4 K slices)
    st->gemm_ws_floats = (size_t)4 * T * h;
    st->gemm_ws = bp.take<float>(st->gemm_ws_floats * sizeof(float));
  }
  const size_t nsq = grad_sumsq_partials(st->flat_count);
  st->partial_sq = bp.take<double>(nsq * sizeof(double));
  st->partial_nf = bp.take<int>(nsq * sizeof(int));
  st->opt = bp.take<OptDevState>(sizeof(OptDevState));
  return align_up(bp.off);
}

void order_shape(int p, int sigma, int m, int kind, int* w, int* delta) {
  const int base = p - 1 - sigma;
  if (kind == ZB_H2) {
    *w = 2 * base < m ? 2 * base : m;
    *delta = 2 * sigma < m ? 2 * sigma : m;
  } else {
    *w = base < m ? base : m;
    *delta = kind == ZB_H1 ? (sigma < m ? sigma : m) : 0;
  }
}

zb_status check_sched_args(int p, int stage, int m, int kind) {
  if (p < 1 || stage < 0 || stage >= p || m < 1 || m > (1 << 20)) return ZB_EINVAL;
  if (kind != ZB_1F1B && kind != ZB_H1 && kind != ZB_H2) return ZB_EINVAL;
  return ZB_OK;
}

// Warm-up forwards, then (F, B, deferred W) triples, then the W tail.
void build_order(int p, int sigma, int m, int kind, std::vector<zb_op>* out) {
  int w, delta;
  order_shape(p, sigma, m, kind, &w, &delta);
  out->clear();
  out->reserve(3 * (size_t)m);
  for (int k = 0; k < w; ++k) out->push_back({ZB_PASS_F, k});
  for (int k = 0; k < m; ++k) {
    if (w + k < m) out->push_back({ZB_PASS_F, w + k});
    out->push_back({ZB_PASS_B, k});
    if (k >= delta) out->push_back({ZB_PASS_W, k - delta});
  }
  for (int k = m - delta; k < m; ++k) out->push_back({ZB_PASS_W, k});
}

// rows (= in features) and columns of weight matrix i
void weight_dims(const zb_stage* st, int i, int* rows, int* cols) {
  const int h = st->h, f = st->ffn;
  *rows = i == ZB_P_W2 ? f : h;
  *cols = i == ZB_P_WQKV ? 3 * h : i == ZB_P_W1 ? f : h;
}
const int kMatrices[4] = {ZB_P_WQKV, ZB_P_WO, ZB_P_W1, ZB_P_W2};

// refresh the transposed bf16 copy of one weight matrix (bf16 stages only)
hipError_t refresh_transposed(zb_stage* st, int l, int i) {
  if (!st->bf16) return hipSuccess;
  int rows, cols;
  weight_dims(st, i, &rows, &cols);
  const size_t off = st->poff[l * ZB_P_COUNT + i];
  return launch_transpose_bf16(st->theta16 + off, st->theta16_t + off, rows, cols, st->stream);
}

// Layers a (virtual) microbatch runs through: all of them, or with two chunks the first half of the stack
// for virtual microbatches 0 .. m/2-1 (chunk 0) and the second half for m/2 .. m-1 (chunk 1).
static void layer_range(const zb_stage* st, int mb, int* lo, int* hi) {
  if (st->chunks == 1) { *lo = 0; *hi = st->L - 1; return; }
  const int half = st->L / 2;
  if (mb < st->m / 2) { *lo = 0; *hi = half - 1; }
  else { *lo = half; *hi = st->L - 1; }
}

template <typename T> struct Exec {
  // B operand of a dgrad GEMM dIn[T, n_in] = dOut[T, k_out] * W^T with W = [n_in][k_out]
  static void dgrad_weight(zb_stage* st, GemmArgs* g, int l, int wi, int n_in, int k_out) {
    if (st->bf16) {  // transposed copy [k_out][n_in]: row-contiguous, as the MFMA kernel wants it
      g->B = st->WtT(l, wi);
      g->b_sk = n_in;
      g->b_sn = 1;
    } else {
      g->B = st->Wt(l, wi);
      g->b_sk = 1;
      g->b_sn = k_out;
    }
  }

  static hipError_t gemm(zb_stage* st, int cls, GemmArgs g) {
    g.workspace = st->gemm_ws;
    g.workspace_floats = st->gemm_ws_floats;
    double bytes = 0;
    const double E = sizeof(T);
    if (g.epilogue == EPI_ACCUM_F32) bytes = 8.0 * g.M * g.N + E * (double)g.K * ((double)g.M + g.N);
    else bytes = E * ((double)g.M * g.K + (double)g.K * g.N + (double)g.M * g.N);
    ProfScope ps(st, cls, 2.0 * g.M * g.N * g.K, bytes);
    return launch_gemm<T>(g, st->stream);
  }

  static zb_status forward(zb_stage* st, int mb) {
    const int h = st->h, f = st->ffn, T_ = st->T;
    hipStream_t s = st->stream;
    char* fb = st->fb_pool + st->fb_slot * (size_t)st->slot_fb[mb];
    char* fw = st->fw_pool + st->fw_slot * (size_t)st->slot_fw[mb];
    const T* x = (const T*)(st->in_x + st->act_bytes * (size_t)mb);
    const double E = sizeof(T);
    int l_lo, l_hi;
    layer_range(st, mb, &l_lo, &l_hi);
    if (st->role == ZB_ROLE_FIRST) {  // X0 = token row + position row, written where a middle stage receives X
      const int* ids = st->ids + (size_t)mb * T_;
      ProfScope ps(st, KC_EMBED, 0, 3 * E * T_ * h);
      ZB_HIP(st, launch_embedding_fwd<T>(ids, (const T*)st->SWt(ZB_SP_EMB_TOK), (const T*)st->SWt(ZB_SP_EMB_POS),
                                         (T*)(st->in_x + st->act_bytes * (size_t)mb), T_, h, st->s, s));
      ZB_HIP(st, launch_sort_tokens(ids, st->perm + (size_t)mb * T_, T_, s));  // for the table's gradient in W
    }
    bool ln1_done = false;  // LayerNorm 1 of the layer already written by the previous layer's last GEMM
    for (int l = l_lo; l <= l_hi; ++l) {
      const LayerOff& q = st->lo[l];
      T* A = (T*)(fw + q.fw_a);
      T* C = (T*)(fw + q.fw_c);
      T* U = (T*)(fw + q.fw_u);
      T* Gl = (T*)(fw + q.fw_g);
      T* QKV = (T*)(fb + q.fb_qkv);
      T* Y1 = (T*)(fb + q.fb_y1);
      T* Fh = (T*)(fb + q.fb_fh);
      float* st1 = (float*)(fb + q.fb_stats1);
      float* st2 = (float*)(fb + q.fb_stats2);
      float* lse = (float*)(fb + q.fb_lse);
      T* y = (l == l_hi) ? (T*)(st->out_y + st->act_bytes * (size_t)mb) : (T*)(fb + st->lo[l + 1].fb_x);
      if (!ln1_done) {
        ProfScope ps(st, KC_LN_FWD, 0, 2 * E * T_ * h + 8.0 * T_);
        ZB_HIP(st, launch_layernorm_fwd<T>(x, st->P(l, ZB_P_LN1_G), st->P(l, ZB_P_LN1_B), A, st1, T_, h,
                                            st->cfg.ln_eps, s));
      }
      GemmArgs g{};
      g.A = A; g.B = st->Wt(l, ZB_P_WQKV); g.M = T_; g.N = 3 * h; g.K = h;
      g.a_sm = h; g.a_sk = 1; g.b_sk = 3 * h; g.b_sn = 1;
      g.epilogue = EPI_BIAS; g.out0 = QKV; g.bias = st->P(l, ZB_P_BQKV);
      ZB_HIP(st, gemm(st, KC_GEMM_FWD, g));
      {
        AttnArgs aa{};
        aa.qkv = QKV; aa.out = C; aa.lse = lse; aa.b = st->b; aa.s = st->s; aa.a = st->a; aa.d = st->d;
        ProfScope ps(st, KC_ATTN_FWD, 4.0 * st->s * (double)st->s * st->b * h, E * 4.0 * T_ * h);
        ZB_HIP(st, launch_attention_fwd<T>(aa, s));
      }
      g = GemmArgs{};
      g.A = C; g.B = st->Wt(l, ZB_P_WO); g.M = T_; g.N = h; g.K = h;
      g.a_sm = h; g.a_sk = 1; g.b_sk = h; g.b_sn = 1;
      g.epilogue = EPI_BIAS_RESID; g.out0 = Y1; g.bias = st->P(l, ZB_P_BO); g.aux = x;
      bool ln2_done = false;  // LayerNorm 2 rides along with the projection GEMM where that runs as K slices
      g.ln_mode = 1; g.ln_gamma = st->P(l, ZB_P_LN2_G); g.ln_beta = st->P(l, ZB_P_LN2_B); g.ln_out = U;
      g.ln_stats = st2; g.ln_eps = st->cfg.ln_eps; g.ln_done = &ln2_done;
      ZB_HIP(st, gemm(st, KC_GEMM_FWD, g));
      if (!ln2_done) {
        ProfScope ps(st, KC_LN_FWD, 0, 2 * E * T_ * h + 8.0 * T_);
        ZB_HIP(st, launch_layernorm_fwd<T>(Y1, st->P(l, ZB_P_LN2_G), st->P(l, ZB_P_LN2_B), U, st2, T_, h,
                                            st->cfg.ln_eps, s));
      }
      g = GemmArgs{};
      g.A = U; g.B = st->Wt(l, ZB_P_W1); g.M = T_; g.N = f; g.K = h;
      g.a_sm = h; g.a_sk = 1; g.b_sk = f; g.b_sn = 1;
      g.epilogue = EPI_BIAS_GELU; g.out0 = Fh; g.out1 = Gl; g.bias = st->P(l, ZB_P_B1);
      ZB_HIP(st, gemm(st, KC_GEMM_FWD, g));
      g = GemmArgs{};
      g.A = Gl; g.B = st->Wt(l, ZB_P_W2); g.M = T_; g.N = h; g.K = f;
      g.a_sm = f; g.a_sk = 1; g.b_sk = h; g.b_sn = 1;
      g.epilogue = EPI_BIAS_RESID; g.out0 = y; g.bias = st->P(l, ZB_P_B2); g.aux = Y1;
      ln1_done = false;
      if (l < l_hi) {  // the next layer's LayerNorm 1 on the rows this GEMM finishes
        const LayerOff& qn = st->lo[l + 1];
        g.ln_mode = 1; g.ln_gamma = st->P(l + 1, ZB_P_LN1_G); g.ln_beta = st->P(l + 1, ZB_P_LN1_B);
        g.ln_out = fw + qn.fw_a; g.ln_stats = (float*)(fb + qn.fb_stats1); g.ln_eps = st->cfg.ln_eps;
        g.ln_done = &ln1_done;
      }
      ZB_HIP(st, gemm(st, KC_GEMM_FWD, g));
      x = y;
    }
    if (st->role == ZB_ROLE_LAST) {  // final LayerNorm, head, softmax cross-entropy against the targets
      T* Z = (T*)(fw + st->fw_z);
      T* logits = (T*)(fb + st->fb_logits);
      {
        ProfScope ps(st, KC_LN_FWD, 0, 2 * E * T_ * h + 8.0 * T_);
        ZB_HIP(st, launch_layernorm_fwd<T>(x, st->SP(ZB_SP_LNF_G), st->SP(ZB_SP_LNF_B), Z, (float*)(fb + st->fb_statsf),
                                            T_, h, st->cfg.ln_eps, s));
      }
      GemmArgs g{};
      g.A = Z; g.B = st->SWt(ZB_SP_W_HEAD); g.M = T_; g.N = st->V; g.K = h;
      g.a_sm = h; g.a_sk = 1; g.b_sk = st->V; g.b_sn = 1;
      g.epilogue = EPI_STORE; g.out0 = logits;
      ZB_HIP(st, gemm(st, KC_GEMM_FWD, g));
      ProfScope ps(st, KC_LOSS, 0, E * T_ * (double)st->V);
      ZB_HIP(st, launch_ce_fwd<T>(logits, st->ids + (size_t)mb * T_, (float*)(fb + st->fb_lse), st->row_loss,
                                  st->loss + mb, T_, st->V, s));
    }
    return ZB_OK;
  }

  // Last stage: the gradient that starts B.  dLogits = (softmax - onehot) / (tokens * m) is kept for W, goes
  // through the head and the final LayerNorm, and lands where a middle stage receives the upstream gradient.
  static zb_status head_backward(zb_stage* st, int mb) {
    const int h = st->h, T_ = st->T;
    hipStream_t s = st->stream;
    char* fb = st->fb_pool + st->fb_slot * (size_t)st->slot_fb[mb];
    char* bw = st->bw_pool + st->bw_slot * (size_t)st->slot_bw[mb];
    const double E = sizeof(T);
    T* dlogits = (T*)(bw + st->bw_dlogits);
    {
      ProfScope ps(st, KC_LOSS, 0, 2 * E * T_ * (double)st->V);
      ZB_HIP(st, launch_ce_bwd<T>((const T*)(fb + st->fb_logits), (const float*)(fb + st->fb_lse),
                                  st->ids + (size_t)mb * T_, dlogits, T_, st->V, 1.0f / ((float)T_ * (float)st->m), s));
    }
    GemmArgs g{};  // dZ = dLogits W_head^T
    g.A = dlogits; g.M = T_; g.N = h; g.K = st->V;
    g.a_sm = st->V; g.a_sk = 1;
    if (st->bf16) { g.B = st->theta16_t + st->spoff[ZB_SP_W_HEAD]; g.b_sk = h; g.b_sn = 1; }
    else { g.B = st->SP(ZB_SP_W_HEAD); g.b_sk = 1; g.b_sn = st->V; }
    g.epilogue = EPI_STORE; g.out0 = st->tmp;
    ZB_HIP(st, gemm(st, KC_GEMM_DGRAD, g));
    ProfScope ps(st, KC_LN_BWD, 0, 3 * E * T_ * h);
    ZB_HIP(st, launch_layernorm_bwd<T>((const T*)st->tmp, (const T*)(st->out_y + st->act_bytes * (size_t)mb),
                                        (const float*)(fb + st->fb_statsf), st->SP(ZB_SP_LNF_G), (const T*)nullptr,
                                        (T*)(st->in_dy + st->act_bytes * (size_t)mb), st->SG(ZB_SP_LNF_G),
                                        st->SG(ZB_SP_LNF_B), st->ln_partials, T_, h, s));
    return ZB_OK;
  }

  // Stage-level parameter gradients of the W pass of n microbatches (in the order given): the head's weight
  // gradient (last stage), the token and position tables' gradients (first stage).
  static zb_status end_stage_wgrad(zb_stage* st, const int* mbs, int n) {
    const int h = st->h, T_ = st->T;
    hipStream_t s = st->stream;
    const double E = sizeof(T);
    if (st->role == ZB_ROLE_LAST) {
      WgradMultiArgs w{};
      w.nprob = 1; w.ngroup = n; w.K = T_;
      w.M[0] = h; w.N[0] = st->V; w.outf[0] = st->SG(ZB_SP_W_HEAD);
      for (int i = 0; i < n; ++i) {
        w.a[i] = st->fw_pool + st->fw_slot * (size_t)st->slot_fw[mbs[i]] + st->fw_z;
        w.b[i] = st->bw_pool + st->bw_slot * (size_t)st->slot_bw[mbs[i]] + st->bw_dlogits;
      }
      ProfScope ps(st, KC_GEMM_WGRAD, 2.0 * h * st->V * T_ * n, 8.0 * h * st->V + E * (double)T_ * ((double)h + st->V) * n);
      ZB_HIP(st, launch_wgrad_multi<T>(w, s));
    } else if (st->role == ZB_ROLE_FIRST) {
      for (int i = 0; i < n; ++i) {
        const int mb = mbs[i];
        ProfScope ps(st, KC_EMBED, 0, 2 * E * T_ * h + 8.0 * T_ * h);
        ZB_HIP(st, launch_embedding_grad<T>((const T*)(st->out_dx + st->act_bytes * (size_t)mb),
                                            st->ids + (size_t)mb * T_, st->perm + (size_t)mb * T_,
                                            st->SG(ZB_SP_EMB_TOK), st->SG(ZB_SP_EMB_POS), T_, h, st->s, s));
      }
    }
    return ZB_OK;
  }

  // layers l_hi down to l_lo (the whole stack by default)
  static zb_status backward_input(zb_stage* st, int mb, int l_hi = -1, int l_lo = 0) {
    const int h = st->h, f = st->ffn, T_ = st->T;
    hipStream_t s = st->stream;
    char* fb = st->fb_pool + st->fb_slot * (size_t)st->slot_fb[mb];
    char* fw = st->fw_pool + st->fw_slot * (size_t)st->slot_fw[mb];
    char* bw = st->bw_pool + st->bw_slot * (size_t)st->slot_bw[mb];
    T* tmp = (T*)st->tmp;
    const double E = sizeof(T);
    int bottom, top;  // the layers this (virtual) microbatch runs through
    layer_range(st, mb, &bottom, &top);
    if (l_hi < 0) { l_hi = top; l_lo = bottom; }
    if (st->role == ZB_ROLE_LAST && l_hi == top) {
      zb_status rc = head_backward(st, mb);
      if (rc != ZB_OK) return rc;
    }
    for (int l = l_hi; l >= l_lo; --l) {
      const LayerOff& q = st->lo[l];
      // gradient entering layer l: the upstream gradient, or what layer l+1 left in the B->W stash
      const T* dy = l == top ? (const T*)(st->in_dy + st->act_bytes * (size_t)mb) : (const T*)(bw + q.bw_dy);
      const T* xl = l == bottom ? (const T*)(st->in_x + st->act_bytes * (size_t)mb) : (const T*)(fb + q.fb_x);
      const T* QKV = (const T*)(fb + q.fb_qkv);
      const T* Y1 = (const T*)(fb + q.fb_y1);
      const T* Fh = (const T*)(fb + q.fb_fh);
      const float* st1 = (const float*)(fb + q.fb_stats1);
      const float* st2 = (const float*)(fb + q.fb_stats2);
      float* lse = (float*)(fb + q.fb_lse);
      const T* C = (const T*)(fw + q.fw_c);
      T* dQKV = (T*)(bw + q.bw_dqkv);
      T* dY1 = (T*)(bw + q.bw_dy1);
      T* dFh = (T*)(bw + q.bw_dfh);
      T* dx = l == bottom ? (T*)(st->out_dx + st->act_bytes * (size_t)mb) : (T*)(bw + st->lo[l - 1].bw_dy);

      GemmArgs g{};  // dFh = (dY W2^T) * gelu'(Fh)
      g.A = dy; g.M = T_; g.N = f; g.K = h;
      g.a_sm = h; g.a_sk = 1; dgrad_weight(st, &g, l, ZB_P_W2, f, h);
      g.epilogue = EPI_DGELU; g.out0 = dFh; g.aux = Fh;
      ZB_HIP(st, gemm(st, KC_GEMM_DGRAD, g));
      g = GemmArgs{};  // dU = dFh W1^T
      g.A = dFh; g.M = T_; g.N = h; g.K = f;
      g.a_sm = f; g.a_sk = 1; dgrad_weight(st, &g, l, ZB_P_W1, h, f);
      g.epilogue = EPI_STORE; g.out0 = tmp;
      bool lnb_done = false;  // LayerNorm 2's backward on the rows this GEMM finishes (K slices only)
      g.ln_mode = 2; g.ln_x = Y1; g.ln_stats = const_cast<float*>(st2); g.ln_gamma = st->P(l, ZB_P_LN2_G);
      g.ln_resid = dy; g.ln_out = dY1; g.ln_dgamma = st->G(l, ZB_P_LN2_G); g.ln_dbeta = st->G(l, ZB_P_LN2_B);
      g.ln_partials = st->ln_partials; g.ln_done = &lnb_done;
      ZB_HIP(st, gemm(st, KC_GEMM_DGRAD, g));
      if (!lnb_done) {
        ProfScope ps(st, KC_LN_BWD, 0, 4 * E * T_ * h);
        ZB_HIP(st, launch_layernorm_bwd<T>(tmp, Y1, st2, st->P(l, ZB_P_LN2_G), dy, dY1, st->G(l, ZB_P_LN2_G),
                                            st->G(l, ZB_P_LN2_B), st->ln_partials, T_, h, s));
      }
      g = GemmArgs{};  // dC = dY1 Wo^T
      g.A = dY1; g.M = T_; g.N = h; g.K = h;
      g.a_sm = h; g.a_sk = 1; dgrad_weight(st, &g, l, ZB_P_WO, h, h);
      g.epilogue = EPI_STORE; g.out0 = tmp;
      ZB_HIP(st, gemm(st, KC_GEMM_DGRAD, g));
      {
        AttnArgs aa{};
        aa.qkv = QKV; aa.o = C; aa.dout = tmp; aa.lse = lse; aa.dqkv = dQKV; aa.dvec = st->dvec;
        aa.b = st->b; aa.s = st->s; aa.a = st->a; aa.d = st->d;
        ProfScope ps(st, KC_ATTN_BWD, 8.0 * st->s * (double)st->s * st->b * h, E * 8.0 * T_ * h);
        ZB_HIP(st, launch_attention_bwd<T>(aa, s));
      }
      g = GemmArgs{};  // dA = dQKV Wqkv^T
      g.A = dQKV; g.M = T_; g.N = h; g.K = 3 * h;
      g.a_sm = 3 * h; g.a_sk = 1; dgrad_weight(st, &g, l, ZB_P_WQKV, h, 3 * h);
      g.epilogue = EPI_STORE; g.out0 = tmp;
      lnb_done = false;  // LayerNorm 1's backward likewise
      g.ln_mode = 2; g.ln_x = xl; g.ln_stats = const_cast<float*>(st1); g.ln_gamma = st->P(l, ZB_P_LN1_G);
      g.ln_resid = dY1; g.ln_out = dx; g.ln_dgamma = st->G(l, ZB_P_LN1_G); g.ln_dbeta = st->G(l, ZB_P_LN1_B);
      g.ln_partials = st->ln_partials; g.ln_done = &lnb_done;
      ZB_HIP(st, gemm(st, KC_GEMM_DGRAD, g));
      if (!lnb_done) {
        ProfScope ps(st, KC_LN_BWD, 0, 4 * E * T_ * h);
        ZB_HIP(st, launch_layernorm_bwd<T>(tmp, xl, st1, st->P(l, ZB_P_LN1_G), dY1, dx, st->G(l, ZB_P_LN1_G),
                                            st->G(l, ZB_P_LN1_B), st->ln_partials, T_, h, s));
      }
    }
    return ZB_OK;
  }

  // W of n microbatches (1 <= n <= kGemmGroupMax, all of one chunk) for layers l_hi .. l_lo: the accumulate
  // GEMMs of as many whole layers as one launch takes (tiles of equal duration, so the partly filled last
  // round of workgroups is paid once per launch, not once per weight matrix), each summing its n operand
  // pairs in the order given.  The bias gradients (column sums of the same dY operands, microbatch by
  // microbatch in the same order) are taken by extra workgroups of that launch where the MFMA kernel runs it,
  // by the column-sum kernels otherwise.
  static zb_status wgrad_layers(zb_stage* st, const int* mbs, int n, int l_hi, int l_lo) {
    const int h = st->h, f = st->ffn, T_ = st->T;
    hipStream_t s = st->stream;
    const double E = sizeof(T);
    int bottom, top;  // the same for every microbatch given (the caller splits at chunk changes)
    layer_range(st, mbs[0], &bottom, &top);
    struct Lin { size_t fw_off, bw_off; bool top_dy; int kin, nout, wi, bi; };
    auto lins_of = [&](int l, Lin (&lins)[4]) {
      const LayerOff& q = st->lo[l];
      lins[0] = {q.fw_g, q.bw_dy, l == top, f, h, ZB_P_W2, ZB_P_B2};
      lins[1] = {q.fw_u, q.bw_dfh, false, h, f, ZB_P_W1, ZB_P_B1};
      lins[2] = {q.fw_c, q.bw_dy1, false, h, h, ZB_P_WO, ZB_P_BO};
      lins[3] = {q.fw_a, q.bw_dqkv, false, h, 3 * h, ZB_P_WQKV, ZB_P_BQKV};
    };
    auto dy_of = [&](const Lin& ln, int mb) -> const char* {
      const char* bw = st->bw_pool + st->bw_slot * (size_t)st->slot_bw[mb];
      return ln.top_dy ? (const char*)(st->in_dy + st->act_bytes * (size_t)mb) : bw + ln.bw_off;
    };
    int per_launch = kWgradMaxPairs / (4 * n);  // whole layers per launch
    if (per_launch > kWgradMaxProblems / 4) per_launch = kWgradMaxProblems / 4;
    if (per_launch < 1) per_launch = 1;
    std::vector<char> bias_in_launch(st->L, 0);
    for (int l1 = l_hi; l1 >= l_lo; l1 -= per_launch) {
      const int l0 = l1 - per_launch + 1 > l_lo ? l1 - per_launch + 1 : l_lo;
      WgradMultiArgs w{};
      bool bias_done = false;
      w.ngroup = n; w.K = T_; w.bias_done = &bias_done;
      double flops = 0, bytes = 0;
      for (int l = l1; l >= l0; --l) {
        Lin lins[4];
        lins_of(l, lins);
        for (const Lin& ln : lins) {
          const int q = w.nprob++;
          w.M[q] = ln.kin; w.N[q] = ln.nout; w.outf[q] = st->G(l, ln.wi); w.bias[q] = st->G(l, ln.bi);
          for (int i = 0; i < n; ++i) {
            const char* fw = st->fw_pool + st->fw_slot * (size_t)st->slot_fw[mbs[i]];
            w.a[q * n + i] = fw + ln.fw_off;
            w.b[q * n + i] = dy_of(ln, mbs[i]);
          }
          flops += 2.0 * ln.kin * ln.nout * T_ * n;
          bytes += 8.0 * ln.kin * ln.nout + E * (double)T_ * ((double)ln.kin + ln.nout) * n;
        }
      }
      {
        ProfScope ps(st, KC_GEMM_WGRAD, flops, bytes);
        ZB_HIP(st, launch_wgrad_multi<T>(w, s));
      }
      if (bias_done)
        for (int l = l1; l >= l0; --l) bias_in_launch[l] = 1;
    }
    for (int l = l_hi; l >= l_lo; --l) {
      if (bias_in_launch[l]) continue;  // the wgrad launch summed the columns of its dY operands itself
      Lin lins[4];
      lins_of(l, lins);
      for (int i = 0; i < n; ++i) {  // the four bias gradients: column sums of the same dY's
        const void* dys[4];
        float* dbs[4];
        int ns[4];
        for (int q = 0; q < 4; ++q) { dys[q] = dy_of(lins[q], mbs[i]); dbs[q] = st->G(l, lins[q].bi); ns[q] = lins[q].nout; }
        ProfScope ps(st, KC_COLSUM, 0, E * T_ * (double)(ns[0] + ns[1] + ns[2] + ns[3]));
        ZB_HIP(st, launch_colsum_accum_multi<T>(dys, dbs, ns, 4, st->ln_partials, T_, s));
      }
    }
    return ZB_OK;
  }

  static zb_status backward_weight(zb_stage* st, int mb, int l_hi = -1, int l_lo = 0) {
    int bottom, top;
    layer_range(st, mb, &bottom, &top);
    if (l_hi < 0) { l_hi = top; l_lo = bottom; }
    if (st->role == ZB_ROLE_LAST && l_hi == top) {
      zb_status rc = end_stage_wgrad(st, &mb, 1);
      if (rc != ZB_OK) return rc;
    }
    zb_status rc = wgrad_layers(st, &mb, 1, l_hi, l_lo);
    if (rc != ZB_OK) return rc;
    if (st->role == ZB_ROLE_FIRST && l_lo == bottom) rc = end_stage_wgrad(st, &mb, 1);
    return rc;
  }

  // The traditional single backward (Sec. 1): layer by layer, the input gradient and right after it the
  // parameter gradients of the same layer, while that layer's output gradients are still in the caches.
  static zb_status backward_fused(zb_stage* st, int mb) {
    int bottom, top;
    layer_range(st, mb, &bottom, &top);
    for (int l = top; l >= bottom; --l) {
      zb_status rc = backward_input(st, mb, l, l);
      if (rc != ZB_OK) return rc;
      if ((rc = backward_weight(st, mb, l, l)) != ZB_OK) return rc;
    }
    return ZB_OK;
  }

  // W of n microbatches (2 <= n <= kGemmGroupMax) of one chunk: every gradient is read and written once.
  static zb_status backward_weight_group(zb_stage* st, const int* mbs, int n) {
    int bottom, top;
    layer_range(st, mbs[0], &bottom, &top);
    if (st->role == ZB_ROLE_LAST) {
      zb_status rc = end_stage_wgrad(st, mbs, n);
      if (rc != ZB_OK) return rc;
    }
    zb_status rc = wgrad_layers(st, mbs, n, top, bottom);
    if (rc != ZB_OK) return rc;
    if (st->role == ZB_ROLE_FIRST) rc = end_stage_wgrad(st, mbs, n);
    return rc;
  }
};

zb_status check_pass(zb_stage* st, int pass, int mb) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  if (st->m <= 0) return fail(st, ZB_ESTATE, "zb_begin_iteration has not been called");
  if (mb < 0 || mb >= st->m) return fail(st, ZB_EINVAL, "microbatch index out of range");
  if (st->done[pass][mb]) return fail(st, ZB_EORDER, "pass already run for this microbatch in this iteration");
  if (pass == ZB_PASS_B && !st->done[ZB_PASS_F][mb]) return fail(st, ZB_EORDER, "B before F of the same microbatch");
  if (pass == ZB_PASS_W && !st->done[ZB_PASS_B][mb]) return fail(st, ZB_EORDER, "W before B of the same microbatch");
  return ZB_OK;
}

int take_slot(std::vector<int>& pool) {
  if (pool.empty()) return -1;
  int v = pool.back();
  pool.pop_back();
  return v;
}

struct TensorRef {
  bool typed;      // true: stored in the stage's data type; false: fp32
  void* ptr;
  size_t count;
  bool writable;
  bool is_param;   // also refresh the bf16 working copy
  size_t flat_off;
  bool is_ids;     // int32 token / target ids (host buffer int32 as well)
  int matrix_rows, matrix_cols;  // parameter that also has a transposed bf16 copy (0: none)
};

zb_status resolve(zb_stage* st, int what, int layer, int mb, TensorRef* r) {
  *r = TensorRef{};
  r->writable = true;
  if (what >= ZB_T_PARAM && what < ZB_T_ADAM_V + 16) {
    const int grp = what / 16, i = what % 16;
    if (i >= ZB_P_COUNT) return fail(st, ZB_EINVAL, "bad parameter index");
    if (layer < 0 || layer >= st->L) return fail(st, ZB_EINVAL, "layer out of range");
    float* base = grp == 0 ? st->theta : grp == 1 ? st->grad : grp == 2 ? st->adam_m : st->adam_v;
    r->typed = false;
    r->flat_off = st->poff[layer * ZB_P_COUNT + i];
    r->ptr = base + r->flat_off;
    r->count = st->pcount[i];
    r->is_param = grp == 0;
    if (grp == 0 && (i == ZB_P_WQKV || i == ZB_P_WO || i == ZB_P_W1 || i == ZB_P_W2)) weight_dims(st, i, &r->matrix_rows, &r->matrix_cols);
    return ZB_OK;
  }
  if (what >= ZB_T_INPUT_X && what <= ZB_T_OUTPUT_DX) {
    if (mb < 0 || mb >= st->cfg.max_microbatches) return fail(st, ZB_EINVAL, "microbatch out of range");
    char* base = what == ZB_T_INPUT_X ? st->in_x : what == ZB_T_INPUT_DY ? st->in_dy
               : what == ZB_T_OUTPUT_Y ? st->out_y : st->out_dx;
    r->typed = true;
    r->ptr = base + st->act_bytes * (size_t)mb;
    r->count = (size_t)st->T * st->h;
    r->writable = what == ZB_T_INPUT_X || what == ZB_T_INPUT_DY;
    return ZB_OK;
  }
  if (what == ZB_T_INPUT_IDS || what == ZB_T_TARGET_IDS) {
    if ((what == ZB_T_INPUT_IDS) != (st->role == ZB_ROLE_FIRST) || st->role == ZB_ROLE_MIDDLE)
      return fail(st, ZB_EINVAL, "input ids belong to a first stage, target ids to a last stage");
    if (mb < 0 || mb >= st->cfg.max_microbatches) return fail(st, ZB_EINVAL, "microbatch out of range");
    r->ptr = st->ids + (size_t)mb * st->T;
    r->count = (size_t)st->T;
    r->is_ids = true;
    return ZB_OK;
  }
  if (what == ZB_T_LOSS) {
    if (st->role != ZB_ROLE_LAST) return fail(st, ZB_EINVAL, "only a last stage computes a loss");
    if (mb < 0 || mb >= st->cfg.max_microbatches) return fail(st, ZB_EINVAL, "microbatch out of range");
    r->ptr = st->loss + mb;
    r->count = 1;
    r->writable = false;
    return ZB_OK;
  }
  if (what >= ZB_T_STAGE_PARAM && what < ZB_T_STAGE_ADAM_V + 8) {
    const int grp = (what - ZB_T_STAGE_PARAM) / 8, i = (what - ZB_T_STAGE_PARAM) % 8;
    if (i >= ZB_SP_COUNT || st->spcount[i] == 0) return fail(st, ZB_EINVAL, "this stage has no such stage-level parameter");
    float* base = grp == 0 ? st->theta : grp == 1 ? st->grad : grp == 2 ? st->adam_m : st->adam_v;
    r->flat_off = st->spoff[i];
    r->ptr = base + r->flat_off;
    r->count = st->spcount[i];
    r->is_param = grp == 0;
    if (grp == 0 && i == ZB_SP_W_HEAD) { r->matrix_rows = st->h; r->matrix_cols = st->V; }
    return ZB_OK;
  }
  if (what >= ZB_T_FLAT_PARAMS && what <= ZB_T_FLAT_ADAM_V) {
    float* base = what == ZB_T_FLAT_PARAMS ? st->theta : what == ZB_T_FLAT_GRADS ? st->grad
                : what == ZB_T_FLAT_ADAM_M ? st->adam_m : st->adam_v;
    r->typed = false;
    r->ptr = base;
    r->count = st->flat_count;
    r->writable = false;
    return ZB_OK;
  }
  return fail(st, ZB_EINVAL, "unknown tensor selector");
}

}  // namespace

extern "C" {

zb_status zb_config_defaults(zb_config* cfg) {
  if (!cfg) return ZB_EINVAL;
  memset(cfg, 0, sizeof(*cfg));
  cfg->mb_size = 1;
  cfg->dtype = ZB_BF16;
  cfg->journal = 1;
  cfg->group_w = 1;
  cfg->chunks = 1;
  cfg->ln_eps = 1e-5f;
  cfg->lr = 1e-4f; cfg->beta1 = 0.9f; cfg->beta2 = 0.95f; cfg->adam_eps = 1e-8f; cfg->weight_decay = 0.01f;
  cfg->clip = 1.0f;
  return ZB_OK;
}

zb_status zb_stage_arena_bytes(const zb_config* cfg, size_t* bytes) {
  std::string why;
  if (!bytes || !valid_shapes(cfg, &why)) return ZB_EINVAL;
  zb_stage tmp;
  tmp.cfg = *cfg;
  *bytes = layout(&tmp, nullptr);
  return ZB_OK;
}

zb_status zb_stage_init(const zb_config* cfg, zb_stage** out) {
  if (!out) return ZB_EINVAL;
  *out = nullptr;
  std::string why;
  if (!valid_shapes(cfg, &why)) return ZB_EINVAL;
  if (!cfg->arena || (reinterpret_cast<uintptr_t>(cfg->arena) & (kAlign - 1))) return ZB_EINVAL;
  if (!(cfg->beta1 > 0.f && cfg->beta1 < 1.f && cfg->beta2 > 0.f && cfg->beta2 < 1.f)) return ZB_EINVAL;
  zb_stage* st = new (std::nothrow) zb_stage();
  if (!st) return ZB_ENOMEM;
  st->cfg = *cfg;
  const size_t need = layout(st, cfg->arena);
  if (need > cfg->arena_bytes) {
    delete st;
    return ZB_ENOMEM;
  }
  st->stream = (hipStream_t)cfg->hip_stream;
  st->hp = OptHyper{cfg->lr, cfg->beta1, cfg->beta2, cfg->adam_eps, cfg->weight_decay, cfg->clip};
  for (int i = 0; i < KC_COUNT; ++i) st->prof_flops[i] = st->prof_bytes[i] = 0;
  // zero state: parameters, moments, gradients, journal, optimizer scalars
  hipError_t e = hipMemsetAsync(cfg->arena, 0, need, st->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(st->stream);
  if (e != hipSuccess) {
    delete st;
    return ZB_EDEVICE;
  }
  st->slot_fb.assign(cfg->max_microbatches, -1);
  st->slot_fw.assign(cfg->max_microbatches, -1);
  st->slot_bw.assign(cfg->max_microbatches, -1);
  *out = st;
  return ZB_OK;
}

zb_status zb_stage_free(zb_stage* st) {
  if (!st) return ZB_EINVAL;
  (void)hipStreamSynchronize(st->stream);
  for (auto& r : st->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto e : st->ev_pool) (void)hipEventDestroy(e);
  delete st;
  return ZB_OK;
}

zb_status zb_stage_flat_count(const zb_stage* st, size_t* count) {
  if (!st || !count) return ZB_EINVAL;
  *count = st->flat_count;
  return ZB_OK;
}

zb_status zb_begin_iteration(zb_stage* st, int32_t iter, int32_t m) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  if (m < 1 || m > st->cfg.max_microbatches) return fail(st, ZB_EINVAL, "m must be in [1, max_microbatches]");
  if (st->chunks == 2 && m % 2 != 0)
    return fail(st, ZB_EINVAL, "with two chunks m counts virtual microbatches (chunk * m/2 + microbatch): even");
  st->m = m;
  st->iter = iter;
  for (int c = 0; c < 3; ++c) st->done[c].assign(m, 0);
  st->free_fb.clear(); st->free_fw.clear(); st->free_bw.clear();
  for (int i = st->cfg.max_pending_b - 1; i >= 0; --i) st->free_fb.push_back(i);
  for (int i = st->cfg.max_inflight - 1; i >= 0; --i) st->free_fw.push_back(i);
  for (int i = st->cfg.max_pending_w - 1; i >= 0; --i) st->free_bw.push_back(i);
  ProfScope ps(st, KC_FILL, 0, 4.0 * st->flat_count);
  ZB_HIP(st, launch_fill_f32(st->grad, st->flat_count, 0.f, st->stream));
  return ZB_OK;
}

zb_status zb_forward(zb_stage* st, int32_t mb) {
  zb_status rc = check_pass(st, ZB_PASS_F, mb);
  if (rc != ZB_OK) return rc;
  if (st->free_fb.empty() || st->free_fw.empty())
    return fail(st, ZB_ENOMEM, "no free stash slot for F: raise max_pending_b / max_inflight");
  st->slot_fb[mb] = take_slot(st->free_fb);
  st->slot_fw[mb] = take_slot(st->free_fw);
  rc = st->bf16 ? Exec<bf16_t>::forward(st, mb) : Exec<float>::forward(st, mb);
  if (rc != ZB_OK) return rc;
  st->done[ZB_PASS_F][mb] = 1;
  return ZB_OK;
}

zb_status zb_backward_input(zb_stage* st, int32_t mb) {
  zb_status rc = check_pass(st, ZB_PASS_B, mb);
  if (rc != ZB_OK) return rc;
  if (st->free_bw.empty()) return fail(st, ZB_ENOMEM, "no free stash slot for B: raise max_pending_w");
  st->slot_bw[mb] = take_slot(st->free_bw);
  rc = st->bf16 ? Exec<bf16_t>::backward_input(st, mb) : Exec<float>::backward_input(st, mb);
  if (rc != ZB_OK) return rc;
  st->done[ZB_PASS_B][mb] = 1;
  st->free_fb.push_back(st->slot_fb[mb]);  // what only B needed is released (stream order keeps it safe)
  st->slot_fb[mb] = -1;
  return ZB_OK;
}

zb_status zb_backward_weight(zb_stage* st, int32_t mb) {
  zb_status rc = check_pass(st, ZB_PASS_W, mb);
  if (rc != ZB_OK) return rc;
  rc = st->bf16 ? Exec<bf16_t>::backward_weight(st, mb) : Exec<float>::backward_weight(st, mb);
  if (rc != ZB_OK) return rc;
  st->done[ZB_PASS_W][mb] = 1;
  st->free_fw.push_back(st->slot_fw[mb]);
  st->free_bw.push_back(st->slot_bw[mb]);
  st->slot_fw[mb] = st->slot_bw[mb] = -1;
  return ZB_OK;
}

zb_status zb_backward_fused(zb_stage* st, int32_t mb) {
  zb_status rc = check_pass(st, ZB_PASS_B, mb);
  if (rc != ZB_OK) return rc;
  if (st->free_bw.empty()) return fail(st, ZB_ENOMEM, "no free stash slot for B: raise max_pending_w");
  st->slot_bw[mb] = take_slot(st->free_bw);
  rc = st->bf16 ? Exec<bf16_t>::backward_fused(st, mb) : Exec<float>::backward_fused(st, mb);
  if (rc != ZB_OK) return rc;
  st->done[ZB_PASS_B][mb] = st->done[ZB_PASS_W][mb] = 1;
  st->free_fb.push_back(st->slot_fb[mb]);
  st->free_fw.push_back(st->slot_fw[mb]);
  st->free_bw.push_back(st->slot_bw[mb]);
  st->slot_fb[mb] = st->slot_fw[mb] = st->slot_bw[mb] = -1;
  return ZB_OK;
}

zb_status zb_backward_weight_group(zb_stage* st, const int32_t* mbs, int32_t n) {
  if (!st) return ZB_EINVAL;
  if (!mbs || n < 1) return fail(st, ZB_EINVAL, "no microbatches given");
  if (n == 1) return zb_backward_weight(st, mbs[0]);
  for (int i = 0; i < n; ++i) {
    zb_status rc = check_pass(st, ZB_PASS_W, mbs[i]);
    if (rc != ZB_OK) return rc;
    for (int j = 0; j < i; ++j)
      if (mbs[j] == mbs[i]) return fail(st, ZB_EORDER, "a microbatch appears twice in the group");
  }
  for (int i0 = 0, cnt = 0; i0 < n; i0 += cnt) {  // at most kGemmGroupMax operand pairs per GEMM, one chunk
    int lo0, hi0;
    layer_range(st, mbs[i0], &lo0, &hi0);
    cnt = 1;
    while (i0 + cnt < n && cnt < kGemmGroupMax) {
      int lo1, hi1;
      layer_range(st, mbs[i0 + cnt], &lo1, &hi1);
      if (lo1 != lo0) break;
      ++cnt;
    }
    zb_status rc;
    if (cnt == 1) rc = st->bf16 ? Exec<bf16_t>::backward_weight(st, mbs[i0]) : Exec<float>::backward_weight(st, mbs[i0]);
    else rc = st->bf16 ? Exec<bf16_t>::backward_weight_group(st, mbs + i0, cnt)
                       : Exec<float>::backward_weight_group(st, mbs + i0, cnt);
    if (rc != ZB_OK) return rc;
    for (int i = i0; i < i0 + cnt; ++i) {
      const int mb = mbs[i];
      st->done[ZB_PASS_W][mb] = 1;
      st->free_fw.push_back(st->slot_fw[mb]);
      st->free_bw.push_back(st->slot_bw[mb]);
      st->slot_fw[mb] = st->slot_bw[mb] = -1;
    }
  }
  return ZB_OK;
}

// Runs a stage order; with group_w, maximal runs of consecutive W entries go through the grouped W.
static zb_status run_ops(zb_stage* st, const zb_op* ops, size_t n) {
  std::vector<int32_t> run;
  for (size_t q = 0; q < n;) {
    const zb_op& op = ops[q];
    if (op.pass == ZB_PASS_W && st->group_w) {
      run.clear();
      while (q < n && ops[q].pass == ZB_PASS_W) run.push_back(ops[q++].mb);
      zb_status rc = zb_backward_weight_group(st, run.data(), (int32_t)run.size());
      if (rc != ZB_OK) return rc;
      continue;
    }
    if (st->fuse_bw && op.pass == ZB_PASS_B && q + 1 < n && ops[q + 1].pass == ZB_PASS_W && ops[q + 1].mb == op.mb) {
      zb_status rc = zb_backward_fused(st, op.mb);  // B_k W_k: the single backward of 1F1B
      if (rc != ZB_OK) return rc;
      q += 2;
      continue;
    }
    zb_status rc = op.pass == ZB_PASS_F ? zb_forward(st, op.mb)
                 : op.pass == ZB_PASS_B ? zb_backward_input(st, op.mb) : zb_backward_weight(st, op.mb);
    if (rc != ZB_OK) return rc;
    ++q;
  }
  return ZB_OK;
}

zb_status zb_schedule_order(int32_t p, int32_t stage, int32_t m, int32_t kind, zb_op* out, int32_t cap,
                            int32_t* n) {
  if (!n || check_sched_args(p, stage, m, kind) != ZB_OK) return ZB_EINVAL;
  *n = 3 * m;
  if (!out || cap < 3 * m) return ZB_EINVAL;
  std::vector<zb_op> ops;
  build_order(p, stage, m, kind, &ops);
  memcpy(out, ops.data(), ops.size() * sizeof(zb_op));
  return ZB_OK;
}

static void stash_need(const zb_op* ops, size_t n, int32_t* max_pending_b, int32_t* max_pending_w,
                       int32_t* max_inflight) {
  int nb = 0, nw = 0, mb_ = 0, mw_ = 0, mi_ = 0;
  for (size_t q = 0; q < n; ++q) {
    if (ops[q].pass == ZB_PASS_F) ++nb;
    else if (ops[q].pass == ZB_PASS_B) { --nb; ++nw; }
    else --nw;
    if (nb > mb_) mb_ = nb;
    if (nw > mw_) mw_ = nw;
    if (nb + nw > mi_) mi_ = nb + nw;
  }
  if (max_pending_b) *max_pending_b = mb_;
  if (max_pending_w) *max_pending_w = mw_;
  if (max_inflight) *max_inflight = mi_;
}

zb_status zb_schedule_stash_need(int32_t p, int32_t stage, int32_t m, int32_t kind, int32_t* max_pending_b,
                                 int32_t* max_pending_w, int32_t* max_inflight) {
  if (check_sched_args(p, stage, m, kind) != ZB_OK) return ZB_EINVAL;
  std::vector<zb_op> ops;
  build_order(p, stage, m, kind, &ops);
  stash_need(ops.data(), ops.size(), max_pending_b, max_pending_w, max_inflight);
  return ZB_OK;
}

// every (pass, mb) at most once, F before B before W of one microbatch, mb in [0, n/3)
static bool valid_stage_order(const zb_op* ops, int32_t n) {
  if (!ops || n < 0 || n % 3 != 0) return false;
  const int m = n / 3;
  std::vector<char> seen((size_t)n, 0);
  for (int q = 0; q < n; ++q) {
    const zb_op& op = ops[q];
    if (op.pass < 0 || op.pass > 2 || op.mb < 0 || op.mb >= m) return false;
    if (seen[(size_t)op.pass * m + op.mb]) return false;
    if (op.pass > 0 && !seen[(size_t)(op.pass - 1) * m + op.mb]) return false;
    seen[(size_t)op.pass * m + op.mb] = 1;
  }
  return true;
}

zb_status zb_order_stash_need(const zb_op* ops, int32_t n, int32_t* max_pending_b, int32_t* max_pending_w,
                              int32_t* max_inflight) {
  if (!ops || n < 0) return ZB_EINVAL;
  if (!valid_stage_order(ops, n)) return ZB_EORDER;
  stash_need(ops, (size_t)n, max_pending_b, max_pending_w, max_inflight);
  return ZB_OK;
}

zb_status zb_run_order(zb_stage* st, const zb_op* ops, int32_t n) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  if (!ops || n < 0) return fail(st, ZB_EINVAL, "no order given");
  if (n != 3 * st->m) return fail(st, ZB_ESTATE, "the order must hold 3m passes for zb_begin_iteration's m");
  if (!valid_stage_order(ops, n)) return fail(st, ZB_EORDER, "not a valid stage order");
  return run_ops(st, ops, (size_t)n);
}

zb_status zb_run_schedule(zb_stage* st, int32_t p, int32_t stage, int32_t m, int32_t kind) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  if (check_sched_args(p, stage, m, kind) != ZB_OK) return fail(st, ZB_EINVAL, "bad schedule arguments");
  if (m != st->m) return fail(st, ZB_ESTATE, "m differs from zb_begin_iteration's");
  std::vector<zb_op> ops;
  build_order(p, stage, m, kind, &ops);
  return run_ops(st, ops.data(), ops.size());
}

zb_status zb_optimizer_step_validated(zb_stage* st, const zb_global_state* gs, zb_step_report* report) {
  if (!st || !gs) return ZB_EINVAL;
  st->err.clear();
  if (!(gs->prev_sq >= 0.0) && !isnan(gs->prev_sq)) return fail(st, ZB_EINVAL, "prev_sq must not be negative");
  if (!(gs->rest_sq >= 0.0) && !isnan(gs->rest_sq)) return fail(st, ZB_EINVAL, "rest_sq must not be negative");
  hipStream_t s = st->stream;
  const size_t n = st->flat_count;
  const double n_d = (double)n;
  const int prev_nf = gs->prev_nonfinite ? 1 : 0, rest_nf = gs->rest_nonfinite ? 1 : 0;
  const double step_bytes = n_d * (16 + 12 + (st->j_theta ? 12 : 0) + (st->theta16 ? 2 : 0));
  {  // local state of this stage
    ProfScope ps(st, KC_SUMSQ, 0, 4.0 * n_d);
    ZB_HIP(st, launch_grad_sumsq(st->grad, n, st->partial_sq, st->partial_nf, st->opt, s));
  }
  // optimistic step controlled by the partially reduced state
  ZB_HIP(st, launch_decide_optimistic(st->opt, st->hp, gs->prev_sq, prev_nf, gs->force_optimistic ? 1 : 0, s));
  {
    ProfScope ps(st, KC_ADAMW_STEP, 0, step_bytes);
    ZB_HIP(st, launch_adamw_step(st->theta, st->adam_m, st->adam_v, st->grad, st->j_theta, st->j_m, st->j_v,
                                 st->theta16, n, st->hp, st->opt, s));
  }
  // validation against the fully reduced state; rollback and redo if the step was not legitimate
  ZB_HIP(st, launch_decide_validate(st->opt, st->hp, gs->prev_sq, gs->rest_sq, prev_nf, rest_nf, s));
  {
    ProfScope ps(st, KC_ADAMW_ROLLBACK, 0, n_d * (16 + 12 + (st->j_theta ? 12 : 0) + (st->theta16 ? 2 : 0)));
    ZB_HIP(st, launch_adamw_rollback(st->theta, st->adam_m, st->adam_v, st->grad, st->j_theta, st->j_m, st->j_v,
                                     st->theta16, n, st->hp, st->opt, s));
  }
  ZB_HIP(st, launch_decide_after_rollback(st->opt, st->hp, s));
  {
    ProfScope ps(st, KC_ADAMW_RESTEP, 0, n_d * (16 + 12 + (st->theta16 ? 2 : 0)));  // no journal after the validation
    ZB_HIP(st, launch_adamw_step(st->theta, st->adam_m, st->adam_v, st->grad, st->j_theta, st->j_m, st->j_v,
                                 st->theta16, n, st->hp, st->opt, s));
  }
  ZB_HIP(st, launch_clear_step(st->opt, s));
  if (st->bf16) {  // the dgrad GEMMs read the weights transposed
    ProfScope ps(st, KC_TRANSPOSE, 0, 4.0 * 12.0 * st->h * (double)st->h * st->L);
    for (int l = 0; l < st->L; ++l)
      for (int wi : kMatrices) ZB_HIP(st, refresh_transposed(st, l, wi));
    if (st->role == ZB_ROLE_LAST)
      ZB_HIP(st, launch_transpose_bf16(st->theta16 + st->spoff[ZB_SP_W_HEAD], st->theta16_t + st->spoff[ZB_SP_W_HEAD],
                                       st->h, st->V, s));
  }
  if (report) {
    OptDevState h;
    ZB_HIP(st, hipMemcpyAsync(&h, st->opt, sizeof(h), hipMemcpyDeviceToHost, s));
    ZB_HIP(st, hipStreamSynchronize(s));
    report->outcome = h.outcome;
    report->stepped_optimistically = h.stepped;
    report->local_sq = h.local_sq;
    report->global_norm = h.global_norm;
    report->clip_coef = h.clip_coef;
    report->t = h.t;
    report->alg1_mismatch_elems = h.mismatch;
  }
  return ZB_OK;
}

zb_status zb_get_tensor(zb_stage* st, int32_t what, int32_t layer, int32_t mb, void* host_dst, size_t bytes) {
  if (!st || !host_dst) return ZB_EINVAL;
  st->err.clear();
  TensorRef r;
  zb_status rc = resolve(st, what, layer, mb, &r);
  if (rc != ZB_OK) return rc;
  if (bytes != r.count * sizeof(float)) return fail(st, ZB_EINVAL, "bytes must be 4 * element count");
  hipStream_t s = st->stream;
  const void* src = r.ptr;
  if (r.typed && st->bf16) {
    if (r.count > st->staging_floats) return fail(st, ZB_ESTATE, "staging buffer too small");
    ZB_HIP(st, launch_convert_to_f32<bf16_t>((const bf16_t*)r.ptr, st->staging, r.count, s));
    src = st->staging;
  }
  ZB_HIP(st, hipMemcpyAsync(host_dst, src, bytes, hipMemcpyDeviceToHost, s));
  ZB_HIP(st, hipStreamSynchronize(s));
  return ZB_OK;
}

zb_status zb_set_tensor(zb_stage* st, int32_t what, int32_t layer, int32_t mb, const void* host_src, size_t bytes) {
  if (!st || !host_src) return ZB_EINVAL;
  st->err.clear();
  TensorRef r;
  zb_status rc = resolve(st, what, layer, mb, &r);
  if (rc != ZB_OK) return rc;
  if (!r.writable) return fail(st, ZB_EINVAL, "tensor is read-only");
  if (bytes != r.count * sizeof(float)) return fail(st, ZB_EINVAL, "bytes must be 4 * element count");
  hipStream_t s = st->stream;
  if (r.is_ids) {  // checked on the host: a kernel indexes the tables / the logits with these
    const int32_t* ids = (const int32_t*)host_src;
    for (size_t i = 0; i < r.count; ++i)
      if (ids[i] < 0 || ids[i] >= st->V) return fail(st, ZB_EINVAL, "id outside [0, vocab)");
  }
  if (r.typed && st->bf16) {
    if (r.count > st->staging_floats) return fail(st, ZB_ESTATE, "staging buffer too small");
    ZB_HIP(st, hipMemcpyAsync(st->staging, host_src, bytes, hipMemcpyHostToDevice, s));
    ZB_HIP(st, launch_convert_from_f32<bf16_t>(st->staging, (bf16_t*)r.ptr, r.count, s));
  } else {
    ZB_HIP(st, hipMemcpyAsync(r.ptr, host_src, bytes, hipMemcpyHostToDevice, s));
    if (r.is_param && st->bf16) {
      ZB_HIP(st, launch_convert_from_f32<bf16_t>((const float*)r.ptr, st->theta16 + r.flat_off, r.count, s));
      if (r.matrix_rows)  // the dgrad GEMMs read this matrix transposed
        ZB_HIP(st, launch_transpose_bf16(st->theta16 + r.flat_off, st->theta16_t + r.flat_off, r.matrix_rows,
                                         r.matrix_cols, s));
    }
  }
  ZB_HIP(st, hipStreamSynchronize(s));
  return ZB_OK;
}

zb_status zb_get_stash_columns(zb_stage* st, int32_t which, int32_t layer, int32_t mb, const int32_t* cols,
                               int32_t ncols, float* host_dst) {
  if (!st || !cols || !host_dst) return ZB_EINVAL;
  st->err.clear();
  if (which < ZB_S_QKV_IN || which > ZB_S_FC2_DOUT) return fail(st, ZB_EINVAL, "unknown stash selector");
  if (layer < 0 || layer >= st->L) return fail(st, ZB_EINVAL, "layer out of range");
  if (st->m <= 0 || mb < 0 || mb >= st->m) return fail(st, ZB_EINVAL, "microbatch out of range");
  if (!st->done[ZB_PASS_B][mb] || st->done[ZB_PASS_W][mb])
    return fail(st, ZB_EORDER, "the W stash of a microbatch exists between its B and its W");
  int lo_l, hi_l;
  layer_range(st, mb, &lo_l, &hi_l);
  if (layer < lo_l || layer > hi_l) return fail(st, ZB_EINVAL, "the microbatch does not run through this layer");
  const int h = st->h, f = st->ffn;
  const LayerOff& q = st->lo[layer];
  const char* fw = st->fw_pool + st->fw_slot * (size_t)st->slot_fw[mb];
  const char* bw = st->bw_pool + st->bw_slot * (size_t)st->slot_bw[mb];
  const char* src = nullptr;
  int width = h;
  switch (which) {
    case ZB_S_QKV_IN: src = fw + q.fw_a; break;
    case ZB_S_PROJ_IN: src = fw + q.fw_c; break;
    case ZB_S_FC1_IN: src = fw + q.fw_u; break;
    case ZB_S_FC2_IN: src = fw + q.fw_g; width = f; break;
    case ZB_S_QKV_DOUT: src = bw + q.bw_dqkv; width = 3 * h; break;
    case ZB_S_PROJ_DOUT: src = bw + q.bw_dy1; break;
    case ZB_S_FC1_DOUT: src = bw + q.bw_dfh; width = f; break;
    default:  // the top layer's FC2 output gradient is the upstream gradient itself
      src = layer == hi_l ? st->in_dy + st->act_bytes * (size_t)mb : bw + q.bw_dy;
      break;
  }
  if (ncols < 1 || (size_t)ncols * ((size_t)st->T + 1) > st->staging_floats)
    return fail(st, ZB_EINVAL, "ncols must be positive and tokens * ncols + ncols floats must fit the staging buffer");
  for (int c = 0; c < ncols; ++c)
    if (cols[c] < 0 || cols[c] >= width) return fail(st, ZB_EINVAL, "column index out of range");
  hipStream_t s = st->stream;
  int* dcols = reinterpret_cast<int*>(st->staging + (size_t)st->T * ncols);
  ZB_HIP(st, hipMemcpyAsync(dcols, cols, sizeof(int32_t) * (size_t)ncols, hipMemcpyHostToDevice, s));
  if (st->bf16) ZB_HIP(st, launch_gather_columns<bf16_t>((const bf16_t*)src, width, st->T, dcols, ncols, st->staging, s));
  else ZB_HIP(st, launch_gather_columns<float>((const float*)src, width, st->T, dcols, ncols, st->staging, s));
  ZB_HIP(st, hipMemcpyAsync(host_dst, st->staging, sizeof(float) * (size_t)st->T * ncols, hipMemcpyDeviceToHost, s));
  ZB_HIP(st, hipStreamSynchronize(s));
  return ZB_OK;
}

zb_status zb_inject(zb_stage* st, int32_t what, int32_t mb, int64_t elem, float value) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  if (what != ZB_T_INPUT_X && what != ZB_T_INPUT_DY) return fail(st, ZB_EINVAL, "only inputs can be injected");
  TensorRef r;
  zb_status rc = resolve(st, what, 0, mb, &r);
  if (rc != ZB_OK) return rc;
  if (elem < 0 || (size_t)elem >= r.count) return fail(st, ZB_EINVAL, "element out of range");
  if (st->bf16) ZB_HIP(st, launch_poke<bf16_t>((bf16_t*)r.ptr, (size_t)elem, value, st->stream));
  else ZB_HIP(st, launch_poke<float>((float*)r.ptr, (size_t)elem, value, st->stream));
  return ZB_OK;
}

zb_status zb_synchronize(zb_stage* st) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  ZB_HIP(st, hipStreamSynchronize(st->stream));
  return ZB_OK;
}

const char* zb_last_error(const zb_stage* st) { return st ? st->err.c_str() : "null stage"; }

zb_status zb_stage_model_flops(const zb_stage* st, int32_t m, double* flops) {
  if (!st || !flops || m < 0) return ZB_EINVAL;
  const double s = st->s, b = st->b, h = st->h;
  const double F = s * b * h * (24 * h + 4 * s), B = s * b * h * (24 * h + 8 * s), W = s * b * h * 24 * h;
  *flops = (double)(st->L / st->chunks) * m * (F + B + W);  // with two chunks m counts virtual microbatches
  if (st->role == ZB_ROLE_LAST) *flops += (double)m * 6.0 * s * b * h * (double)st->V;
  return ZB_OK;
}

zb_status zb_stage_stash_bytes(const zb_stage* st, double* m_b, double* m_w) {
  if (!st || !m_b || !m_w) return ZB_EINVAL;
  *m_b = (double)(st->fb_slot + st->fw_slot);
  *m_w = (double)(st->fw_slot + st->bw_slot);
  return ZB_OK;
}

zb_status zb_profile_enable(zb_stage* st, int32_t on) {
  if (!st) return ZB_EINVAL;
  st->err.clear();
  ZB_HIP(st, hipStreamSynchronize(st->stream));
  if (on) {
    for (auto& r : st->prof) { st->ev_pool.push_back(r.a); st->ev_pool.push_back(r.b); }
    st->prof.clear();
    for (int i = 0; i < KC_COUNT; ++i) st->prof_flops[i] = st->prof_bytes[i] = 0;
  }
  st->profiling = on != 0;
  return ZB_OK;
}

zb_status zb_profile_read(zb_stage* st, zb_kernel_stat* out, int32_t cap, int32_t* n) {
  if (!st || !n) return ZB_EINVAL;
  st->err.clear();
  ZB_HIP(st, hipStreamSynchronize(st->stream));
  double ms[KC_COUNT] = {0};
  long long cnt[KC_COUNT] = {0};
  for (const ProfRec& r : st->prof) {
    float t = 0.f;
    ZB_HIP(st, hipEventElapsedTime(&t, r.a, r.b));
    ms[r.cls] += t;
    cnt[r.cls] += 1;
  }
  int k = 0;
  for (int c = 0; c < KC_COUNT; ++c) {
    if (!cnt[c]) continue;
    if (out && k < cap) {
      memset(&out[k], 0, sizeof(out[k]));
      snprintf(out[k].name, sizeof(out[k].name), "%s", kClassNames[c]);
      out[k].launches = cnt[c];
      out[k].total_ms = ms[c];
      out[k].flops = st->prof_flops[c];
      out[k].bytes = st->prof_bytes[c];
    }
    ++k;
  }
  *n = k;
  return (out && k > cap) ? ZB_EINVAL : ZB_OK;
}

}  // extern "C"
