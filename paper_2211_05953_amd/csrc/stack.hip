// The rank's layer stack: workspace layout, parameter access, and the stream scheduler
// that issues one training step in breadth-first or depth-first order (Sec. 4.1, App. C).
//
// Workspace layout (all offsets 256-byte aligned, everything pre-allocated, App. D.2):
//   w32 | m | v | g32           fp32 master weights, Adam moments, main-grads  [P_total each]
//   w_lp                        bf16 copy of the weights (bf16 mode only)        [P_total]
//                               (dp_fs: a double buffer of two stages instead, App. D.1)
//   records                     stored activations, one record per (layer, micro-batch)
//                               (BF_CKPT_NONE) or one checkpoint per (layer, micro-batch)
//                               plus a single scratch record (BF_CKPT_LAYER)
//   backward temporaries, per-micro-batch gradient hand-off buffers, output scratch
// Parameters of a layer are contiguous and layers follow each other, so a stage is one
// contiguous range and its Adam step is one launch.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "common.h"
#include "schedule.h"

namespace bf {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v, size_t a = ALIGN) { return (v + a - 1) / a * a; }

struct Dims {
  int h, a, d, f, S_seq, L;
  size_t tensor_elems[BF_N_TENSORS];
  size_t tensor_off[BF_N_TENSORS];  // element offset inside a layer
  size_t layer_elems;               // padded
  // input / output layers (S_voc > 0): e_tok, e_pos, lnf_g, lnf_b, w_out after the last layer
  size_t voc_elems[BF_N_VOCAB_TENSORS];
  size_t voc_off[BF_N_VOCAB_TENSORS];  // element offset from the end of the layers
  size_t voc_total;
};

void fill_dims(const bf_config& c, Dims* D) {
  D->h = c.S_hidden; D->a = c.N_heads; D->d = c.S_head; D->f = c.S_mlp; D->S_seq = c.S_seq; D->L = c.N_layers;
  const size_t h = c.S_hidden, f = c.S_mlp;
  const size_t n[BF_N_TENSORS] = {h, h, h * 3 * h, 3 * h, h * h, h, h, h, h * f, f, f * h, h};
  size_t off = 0;
  for (int i = 0; i < BF_N_TENSORS; ++i) {
    D->tensor_elems[i] = n[i];
    D->tensor_off[i] = off;
    off += up(n[i], 128);  // 128 elements: 512 B in fp32, 256 B in bf16
  }
  D->layer_elems = off;
  const size_t V = c.S_voc > 0 ? (size_t)c.S_voc : 0;
  const size_t nv[BF_N_VOCAB_TENSORS] = {V * h, V ? (size_t)c.S_seq * h : 0, V ? h : 0, V ? h : 0, V * h};
  off = 0;
  for (int i = 0; i < BF_N_VOCAB_TENSORS; ++i) {
    D->voc_elems[i] = nv[i];
    D->voc_off[i] = off;
    off += up(nv[i], 128);
  }
  D->voc_total = off;
}

bool valid_config(const bf_config* c) {
  if (!c) { set_error("null config"); return false; }
  if (c->S_hidden < 1 || c->N_heads < 1 || c->S_head < 1 || c->S_mlp < 1 || c->S_seq < 1 || c->N_layers < 1 ||
      c->N_mb_max < 1 || c->S_mb_max < 1) { set_error("config: every size must be >= 1"); return false; }
  if ((int64_t)c->N_heads * c->S_head != c->S_hidden) { set_error("config: N_heads * S_head != S_hidden"); return false; }
  if (c->dtype != BF_FP32 && c->dtype != BF_BF16) { set_error("config: unknown dtype"); return false; }
  if (c->ckpt_mode != BF_CKPT_NONE && c->ckpt_mode != BF_CKPT_LAYER) { set_error("config: unknown ckpt_mode"); return false; }
  if (c->kernels != BF_KERNELS_AUTO && c->kernels != BF_KERNELS_PLAIN) { set_error("config: unknown kernels"); return false; }
  if (c->causal != 0 && c->causal != 1) { set_error("config: causal must be 0 or 1"); return false; }
  if (c->queue_depth < 0) { set_error("config: queue_depth < 0"); return false; }
  if (c->fuse_wgrad != 0 && c->fuse_wgrad != 1) { set_error("config: fuse_wgrad must be 0 or 1"); return false; }
  if (c->N_loop_min < 0 || c->N_loop_min > c->N_layers) { set_error("config: N_loop_min outside 0..N_layers"); return false; }
  if (c->S_voc < 0) { set_error("config: S_voc < 0"); return false; }
  if (c->dp_fs != 0 && c->dp_fs != 1) { set_error("config: dp_fs must be 0 or 1"); return false; }
  if (c->dp_fs && c->dtype != BF_BF16) { set_error("config: dp_fs reconstructs bf16 weights: dtype must be BF_BF16"); return false; }
  if ((int64_t)c->S_mb_max * c->S_seq > (1 << 24)) { set_error("config: S_mb_max * S_seq too large"); return false; }
  if (!(c->ln_eps > 0.f) || !(c->init_std >= 0.f)) { set_error("config: ln_eps must be > 0, init_std >= 0"); return false; }
  if (c->mb_chains < 0 || c->mb_chains > 2) { set_error("config: mb_chains must be 0, 1 or 2"); return false; }
  if (c->mb_chains == 2 && (c->fuse_wgrad != 1 || c->dp_fs || c->queue_depth || c->S_voc)) {
    set_error("config: mb_chains = 2 needs fuse_wgrad = 1, dp_fs = 0, queue_depth = 0 and S_voc = 0");
    return false;
  }
  return true;
}

// One stored-activation record (pointers into the workspace).
struct Record {
  char* a;     // LN1 output            [T, h]
  char* qkv;   //                       [T, 3h]
  char* ctx;   // attention output      [T, h]
  char* x1;    // x + attention branch  [T, h]
  char* c;     // LN2 output            [T, h]
  char* u;     // FC1 pre-activation    [T, f]
  char* g;     // GeLU(u)               [T, f]
  char* y;     // layer output = next layer's input (the checkpoint of the next layer) [T, h]
  float* ln1;  // mean, rstd            [T, 2]
  float* ln2;
  float* lse;  //                       [S_mb, N_heads, S_seq]
};

struct WsLayout {
  size_t P_layers, P_total;  // parameters of the layers; with the input / output layers
  size_t off_w32, off_m, off_v, off_g32, off_wlp;
  size_t half_bytes;       // dp_fs: one half of the weight double buffer
  size_t off_wlp_voc;      // dp_fs: bf16 copy of the input / output layers
  size_t off_lm, logits_bytes;  // S_voc > 0: buffers of the input / output layers
  size_t rec_bytes;        // one full record (without y)
  size_t y_bytes;          // one [T, h] tensor
  size_t off_records;      // NONE: L * N_mb_max full records (each with y); LAYER: 1 scratch record
  size_t n_full_records;
  size_t off_ckpt;         // LAYER: L * N_mb_max [T, h] tensors (outputs of each layer)
  size_t off_tmp;          // backward temporaries
  size_t off_tmp2;         // mb_chains = 2: the second chain's backward temporaries
  size_t off_g32b;         // mb_chains = 2: where the second chain accumulates its bias / LayerNorm gradients
  size_t off_grec;         // fused weight gradient: (layers per stage) * N_mb_max records {dy, du, dx1, dqkv}
  size_t grec_bytes;
  size_t off_wrec;         // with checkpointing: as many records {a, ctx, c, g}, the recomputed wgrad operands
  size_t wrec_bytes;
  size_t off_step;         // optimizer step count (one int)
  size_t off_bhand;        // 2 x N_mb_max [T, h] (two sets, alternating by stage)
  size_t off_scratch_out;  // [T, h] x 2: discarded outputs / ping-pong
  size_t total;
};

struct RecSizes { size_t a, qkv, ctx, x1, c, u, g, ln1, ln2, lse, total; };

RecSizes rec_sizes(const bf_config& c) {
  const size_t es = c.dtype == BF_BF16 ? 2 : 4;
  const size_t T = (size_t)c.S_mb_max * c.S_seq, h = c.S_hidden, f = c.S_mlp;
  RecSizes r;
  r.a = up(T * h * es); r.qkv = up(T * 3 * h * es); r.ctx = up(T * h * es); r.x1 = up(T * h * es);
  r.c = up(T * h * es); r.u = up(T * f * es); r.g = up(T * f * es);
  r.ln1 = up(T * 2 * 4); r.ln2 = up(T * 2 * 4); r.lse = up((size_t)c.S_mb_max * c.N_heads * c.S_seq * 4);
  r.total = r.a + r.qkv + r.ctx + r.x1 + r.c + r.u + r.g + r.ln1 + r.ln2 + r.lse;
  return r;
}

struct TmpSizes { size_t du, dc, dx1, dctx, dqkv, delta, ping, colpart, lnpart, attnpart, splitk, total; };

TmpSizes tmp_sizes_of(const bf_config& c);

// Asked for on every launch that uses the scratch areas: the last answer is kept per thread (a stack's configuration
// is one object that does not change, so the bytes compare equal from call to call).
TmpSizes tmp_sizes(const bf_config& c) {
  static thread_local bool have = false;
  static thread_local bf_config last_c;
  static thread_local TmpSizes last_t;
  if (have && std::memcmp(&last_c, &c, sizeof(bf_config)) == 0) return last_t;
  last_t = tmp_sizes_of(c);
  std::memcpy(&last_c, &c, sizeof(bf_config));
  have = true;
  return last_t;
}

TmpSizes tmp_sizes_of(const bf_config& c) {
  const size_t es = c.dtype == BF_BF16 ? 2 : 4;
  const size_t T = (size_t)c.S_mb_max * c.S_seq, h = c.S_hidden, f = c.S_mlp;
  TmpSizes t;
  t.du = up(T * f * es); t.dc = up(T * h * es); t.dx1 = up(T * h * es); t.dctx = up(T * h * es);
  t.dqkv = up(T * 3 * h * es); t.delta = up((size_t)c.S_mb_max * c.N_heads * c.S_seq * 4); t.ping = up(T * h * es);
  // partial column sums that a product's epilogue leaves per row of (at least 128-row) tiles: [T / 128][f] fp32
  t.colpart = up(((T + 127) / 128) * f * 4);
  // partial column sums of the one-pass LayerNorm backward: one row of [3][h] per workgroup
  t.lnpart = up(layernorm_bwd_part_elems((int)T, (int)h) * 4);
  // partial column sums of dqkv that the attention backward kernels leave per query / key block
  t.attnpart = up(attention_bwd_part_elems(c.S_mb_max, c.S_seq, c.N_heads, c.S_head) * 4);
  // fp32 planes of the products whose contraction is split (few tiles, long K): the largest such product of a layer
  size_t planes = 0;
  if (c.dtype == BF_BF16 && c.kernels == BF_KERNELS_AUTO) {
    const int Ti = (int)T, hi = (int)h, fi = (int)f;
    const int cand[6][5] = {{L_NN, E_BIAS, Ti, 3 * hi, hi},     {L_NN, E_BIAS_RES, Ti, hi, hi}, {L_NN, E_BIAS_RES, Ti, hi, fi},
                            {L_NT, E_NONE, Ti, hi, 3 * hi},     {L_NT, E_NONE, Ti, hi, hi},     {L_NT, E_NONE, Ti, hi, fi}};
    for (const auto& k : cand) {
      const int sl = gemm_splitk_slices(k[0], k[1], k[2], k[3], k[4]);
      if (sl > 1) planes = std::max(planes, (size_t)sl * k[2] * k[3]);
    }
  }
  t.splitk = up(planes * 4);
  t.total = t.du + t.dc + t.dx1 + t.dctx + t.dqkv + t.delta + 2 * t.ping + t.colpart + t.lnpart + t.attnpart + t.splitk;
  return t;
}

// The weight gradients of a stage can be taken as one product over all its micro-batches only
// when every micro-batch's activations are still stored (no checkpointing).
bool fuse_wgrad_possible(const bf_config& c) { return c.fuse_wgrad != 0; }

// Most layers a stage can have (sizes the per-stage buffers of the fused weight gradient).
int lps_max(const bf_config& c) {
  const int nl = c.N_loop_min > 0 ? c.N_loop_min : 1;
  return (c.N_layers + nl - 1) / nl;
}

void fill_layout(const bf_config& c, const Dims& D, WsLayout* Lo) {
  const size_t es = c.dtype == BF_BF16 ? 2 : 4;
  const size_t T = (size_t)c.S_mb_max * c.S_seq;
  Lo->P_layers = D.layer_elems * (size_t)c.N_layers;
  Lo->P_total = Lo->P_layers + D.voc_total;
  size_t off = 0;
  Lo->off_w32 = off; off += up(Lo->P_total * 4);
  Lo->off_m = off; off += up(Lo->P_total * 4);
  Lo->off_v = off; off += up(Lo->P_total * 4);
  Lo->off_g32 = off; off += up(Lo->P_total * 4);
  Lo->off_wlp = off;
  Lo->half_bytes = up((size_t)lps_max(c) * D.layer_elems * 2);
  Lo->off_wlp_voc = 0;
  if (c.dp_fs) {
    off += 2 * Lo->half_bytes;  // double buffer of two stages instead of every layer's copy
    Lo->off_wlp_voc = off;      // the input / output layers keep a resident copy
    off += up(D.voc_total * 2);
  } else if (c.dtype == BF_BF16) {
    off += up(Lo->P_total * 2);
  }
  Lo->rec_bytes = rec_sizes(c).total;
  Lo->y_bytes = up(T * c.S_hidden * es);
  Lo->off_records = off;
  const size_t slots = (size_t)c.N_layers * c.N_mb_max;
  if (c.ckpt_mode == BF_CKPT_NONE) {
    Lo->n_full_records = slots;
    off += slots * (Lo->rec_bytes + Lo->y_bytes);
    Lo->off_ckpt = off;
  } else {
    Lo->n_full_records = c.mb_chains == 2 ? 2 : 1;  // one scratch record per chain of micro-batches
    off += Lo->n_full_records * Lo->rec_bytes;
    Lo->off_ckpt = off;
    off += slots * Lo->y_bytes;
  }
  Lo->off_tmp = off; off += tmp_sizes(c).total;
  Lo->off_tmp2 = Lo->off_g32b = 0;
  if (c.mb_chains == 2) {
    Lo->off_tmp2 = off; off += tmp_sizes(c).total;
    Lo->off_g32b = off; off += up(Lo->P_layers * 4);
  }
  {
    TmpSizes t = tmp_sizes(c);
    RecSizes r = rec_sizes(c);
    const size_t stage_slots = (size_t)lps_max(c) * c.N_mb_max;
    Lo->grec_bytes = t.ping + t.du + t.dx1 + t.dqkv;
    Lo->off_grec = off;
    if (fuse_wgrad_possible(c)) off += stage_slots * Lo->grec_bytes;
    Lo->wrec_bytes = r.a + r.ctx + r.c + r.g;
    Lo->off_wrec = off;
    if (fuse_wgrad_possible(c) && c.ckpt_mode == BF_CKPT_LAYER) off += stage_slots * Lo->wrec_bytes;
  }
  Lo->off_bhand = off; off += 2 * (size_t)c.N_mb_max * Lo->y_bytes;
  Lo->off_scratch_out = off; off += 2 * Lo->y_bytes;
  // input / output layers: embedded inputs and loss gradients per micro-batch, the last layer's output,
  // its normalised form and the gradient of that, LayerNorm statistics, logits of one micro-batch, row losses
  Lo->off_lm = off;
  Lo->logits_bytes = up(T * (size_t)(c.S_voc > 0 ? c.S_voc : 0) * es);
  if (c.S_voc > 0) off += (2 * (size_t)c.N_mb_max + 3) * Lo->y_bytes + up(T * 8) + Lo->logits_bytes + up(T * 4);
  Lo->off_step = off; off += ALIGN;
  Lo->total = off;
}

}  // namespace
}  // namespace bf

using namespace bf;

struct bf_stack {
  bf_config cfg;
  Dims D;
  WsLayout Lo;
  char* ws;
  float *w32, *m, *v, *g32;
  bf16_t* wlp;            // resident bf16 copy (null in fp32 mode and with dp_fs)
  bf16_t* wlp_voc;        // dp_fs: resident bf16 copy of the input / output layers
  // dp_fs: the two halves of the weight buffer, the first layer / layer count each holds (-1: nothing
  // valid), the half and first layer the op being issued reads, and the events that order the halves
  bf16_t* fs_half[2];
  int fs_l0[2], fs_n[2];
  int fs_cur, fs_cur_l0;
  hipEvent_t fs_ready[2], fs_free[2];
  hipStream_t side;       // Adam and weight-reconstruction stream
  hipEvent_t ev_grad_ready, ev_side_done, ev_t0, ev_t1;
  std::vector<hipEvent_t> adam_ev;   // pairs of events per stage for timing
  std::vector<hipEvent_t> queue_ev;  // ring for the bounded launch queue
  std::vector<bf_event> trace;
  // per-kernel-class timing: event pairs around the launches of a step, every class (timing == 2) or
  // the weight-gradient products only (timing == 3); prof_mask has one bit per class
  bool prof_on;
  unsigned prof_mask;
  std::vector<hipEvent_t> prof_ev;
  struct ProfRec { int cls; double flops, bytes; };
  std::vector<ProfRec> prof_rec;
  int step;               // optimizer step counter (host mirror; the kernels read d_step)
  int* d_step;            // the same count on the device, bumped by a one-thread kernel at the start of an
                          // optimizer step: a step recorded in a HIP graph keeps counting when replayed
  bool have_grads;
  int device;
  // mb_chains = 2: the chain (0 or 1) whose op is being issued selects the backward temporaries and the arena the
  // bias / LayerNorm gradients go to; the second chain's stream; events for the fork at the start of a step, the two
  // directions of the meeting at a stage's end and the join at the step's end
  int chain;
  int chains_active;  // chains of the step being issued (1 outside a two-chain step)
  float* g32b;
  hipStream_t chain_st;
  hipEvent_t ev_chain[4];
};

namespace bf {
namespace {

float* param_ptr(bf_stack* s, float* arena, int layer, int tid) {
  if (tid >= BF_E_TOK) return arena + s->Lo.P_layers + s->D.voc_off[tid - BF_E_TOK];
  return arena + (size_t)layer * s->D.layer_elems + s->D.tensor_off[tid];
}

// bf16 copy of the master element at offset `off`, or null where there is none
bf16_t* lp_ptr(bf_stack* s, size_t off) {
  if (s->wlp) return s->wlp + off;
  if (s->wlp_voc && off >= s->Lo.P_layers) return s->wlp_voc + (off - s->Lo.P_layers);
  return nullptr;
}

// weight operand of the GEMMs: bf16 copy in bf16 mode, the master itself in fp32 mode
const void* weight_ptr(bf_stack* s, int layer, int tid) {
  if (tid >= BF_E_TOK) {
    float* m = param_ptr(s, s->w32, layer, tid);
    return s->cfg.dtype == BF_BF16 ? (const void*)lp_ptr(s, m - s->w32) : (const void*)m;
  }
  if (s->cfg.dp_fs)
    return s->fs_half[s->fs_cur] + (size_t)(layer - s->fs_cur_l0) * s->D.layer_elems + s->D.tensor_off[tid];
  const size_t off = (size_t)layer * s->D.layer_elems + s->D.tensor_off[tid];
  return s->cfg.dtype == BF_BF16 ? (const void*)(s->wlp + off) : (const void*)(s->w32 + off);
}

Record record_at(bf_stack* s, char* base) {
  RecSizes r = rec_sizes(s->cfg);
  Record R;
  char* p = base;
  R.a = p; p += r.a; R.qkv = p; p += r.qkv; R.ctx = p; p += r.ctx; R.x1 = p; p += r.x1; R.c = p; p += r.c;
  R.u = p; p += r.u; R.g = p; p += r.g; R.ln1 = (float*)p; p += r.ln1; R.ln2 = (float*)p; p += r.ln2;
  R.lse = (float*)p; p += r.lse;
  R.y = nullptr;
  return R;
}

// Record used by (layer, mb): its own slot without checkpointing, the scratch record (of the chain that is
// being issued) with.
Record record_for(bf_stack* s, int layer, int mb) {
  if (s->cfg.ckpt_mode == BF_CKPT_NONE) {
    const size_t slot = (size_t)layer * s->cfg.N_mb_max + mb;
    char* base = s->ws + s->Lo.off_records + slot * (s->Lo.rec_bytes + s->Lo.y_bytes);
    Record R = record_at(s, base);
    R.y = base + s->Lo.rec_bytes;
    return R;
  }
  Record R = record_at(s, s->ws + s->Lo.off_records + (s->chain ? s->Lo.rec_bytes : 0));
  R.y = s->ws + s->Lo.off_ckpt + ((size_t)layer * s->cfg.N_mb_max + mb) * s->Lo.y_bytes;
  return R;
}

struct Tmp { char *du, *dc, *dx1, *dctx, *dqkv, *ping[2]; float *delta, *colpart, *lnpart, *attnpart, *splitk; size_t splitk_elems; };

// Per (layer, micro-batch) gradients kept for the fused weight gradient of a stage.
struct GradRec { char *dy, *du, *dx1, *dqkv; };

// ls: index of the layer inside its stage
GradRec grad_rec(bf_stack* s, int ls, int mb) {
  TmpSizes t = tmp_sizes(s->cfg);
  char* p = s->ws + s->Lo.off_grec + ((size_t)ls * s->cfg.N_mb_max + mb) * s->Lo.grec_bytes;
  GradRec g;
  g.dy = p; p += t.ping; g.du = p; p += t.du; g.dx1 = p; p += t.dx1; g.dqkv = p;
  return g;
}

// With checkpointing the recomputed a / ctx / c / g of (layer in stage ls, micro-batch mb) are written
// here instead of the scratch record, so that they survive until the stage's weight-gradient products.
void redirect_wgrad_operands(bf_stack* s, int ls, int mb, Record* R) {
  RecSizes r = rec_sizes(s->cfg);
  char* p = s->ws + s->Lo.off_wrec + ((size_t)ls * s->cfg.N_mb_max + mb) * s->Lo.wrec_bytes;
  R->a = p; p += r.a; R->ctx = p; p += r.ctx; R->c = p; p += r.c; R->g = p;
}

Tmp tmp_of(bf_stack* s) {
  TmpSizes t = tmp_sizes(s->cfg);
  Tmp T;
  char* p = s->ws + (s->chain ? s->Lo.off_tmp2 : s->Lo.off_tmp);
  T.du = p; p += t.du; T.dc = p; p += t.dc; T.dx1 = p; p += t.dx1; T.dctx = p; p += t.dctx; T.dqkv = p; p += t.dqkv;
  T.delta = (float*)p; p += t.delta; T.ping[0] = p; p += t.ping; T.ping[1] = p; p += t.ping; T.colpart = (float*)p; p += t.colpart; T.lnpart = (float*)p; p += t.lnpart;
  T.attnpart = t.attnpart ? (float*)p : nullptr;
  p += t.attnpart;
  T.splitk = t.splitk ? (float*)p : nullptr;
  T.splitk_elems = t.splitk / 4;
  return T;
}

// Runs one kernel launcher; with profiling on, brackets it with a pair of events on its stream.
template <typename F>
bf_status timed(bf_stack* s, int cls, double flops, double bytes, hipStream_t st, F&& call) {
  if (!s->prof_on || !((s->prof_mask >> cls) & 1u)) return call();
  const size_t i = s->prof_rec.size();
  while (s->prof_ev.size() < 2 * (i + 1)) {
    hipEvent_t e;
    BF_HIP_CHECK(hipEventCreate(&e));
    s->prof_ev.push_back(e);
  }
  BF_HIP_CHECK(hipEventRecord(s->prof_ev[2 * i], st));
  bf_status r = call();
  if (r != BF_OK) return r;
  BF_HIP_CHECK(hipEventRecord(s->prof_ev[2 * i + 1], st));
  s->prof_rec.push_back({cls, flops, bytes});
  return BF_OK;
}

#define BF_TRY(expr)            \
  do {                          \
    bf_status s__ = (expr);     \
    if (s__ != BF_OK) return s__; \
  } while (0)

// ---- launchers with per-class accounting: algorithmic flops (MFMA-bound classes) and
// algorithmic HBM bytes (bandwidth-bound classes) of each launch
bf_status p_gemm(bf_stack* s, int layout, int epi, const GemmArgs& g, hipStream_t st) {
  const int cls = layout == L_NN ? BF_K_GEMM_FWD : layout == L_NT ? BF_K_GEMM_DGRAD : BF_K_GEMM_WGRAD;
  const double es = s->cfg.dtype == BF_BF16 ? 2 : 4;
  double bytes = es * ((double)g.M * g.K + (double)g.K * g.N) + (layout == L_TN ? (g.accumulate ? 8.0 : 4.0) : es) * g.M * g.N;
  const double nseg = g.n_seg > 1 ? g.n_seg : 1;
  if (nseg > 1) bytes = es * nseg * ((double)g.M * g.K + (double)g.K * g.N) + 4.0 * g.M * g.N;
  GemmArgs a = g;
  // Scratch for a split contraction; gemm() decides whether the product takes it.  Not with two chains of
  // micro-batches in flight: the other chain's kernels fill the compute units a product of few tiles leaves idle,
  // and the pass that adds the planes is saved (a 2048-wide stack: 38.3 -> 36.7 ms per step).
  a.shared_chip = s->chains_active == 2;  // and no 256 x 192 tile either, for the same reason
  if (layout != L_TN && s->chains_active == 1) {
    const Tmp t = tmp_of(s);
    a.splitk_ws = t.splitk;
    a.splitk_ws_elems = t.splitk_elems;
  }
  return timed(s, cls, 2.0 * g.M * g.N * g.K * nseg, bytes, st, [&] { return gemm(s->cfg.dtype, s->cfg.kernels, layout, epi, a, st); });
}
bf_status p_ln_fwd(bf_stack* s, int T, int h, const void* x, const float* g, const float* b, float eps, void* y, float* stats,
                   hipStream_t st) {
  const double es = s->cfg.dtype == BF_BF16 ? 2 : 4;
  return timed(s, BF_K_LN_FWD, 0.0, 2.0 * es * T * h, st, [&] { return layernorm_fwd(s->cfg.dtype, T, h, x, g, b, eps, y, stats, st); });
}
// dcs: null, or where the column sums of dx go (the bias gradient of the linear layer that produced x)
bf_status p_ln_bwd(bf_stack* s, int T, int h, const void* dy, const void* x, const float* g, const float* stats, const void* dres,
                   void* dx, float* dg, float* db, float* dcs, int acc, hipStream_t st) {
  const double es = s->cfg.dtype == BF_BF16 ? 2 : 4;
  return timed(s, BF_K_LN_BWD, 0.0, 4.0 * es * T * h, st, [&] {
    return layernorm_bwd(s->cfg.dtype, T, h, dy, x, g, stats, dres, dx, dg, db, acc, st, dcs, tmp_of(s).lnpart);
  });
}
bf_status p_colsum(bf_stack* s, int T, int N, const void* dY, float* out, int acc, hipStream_t st) {
  const double es = s->cfg.dtype == BF_BF16 ? 2 : 4;
  return timed(s, BF_K_COLSUM, 0.0, es * T * N, st, [&] { return colsum(s->cfg.dtype, T, N, dY, out, acc, st); });
}
bf_status p_attn_fwd(bf_stack* s, int S_mb, const void* qkv, void* ctx, float* lse, hipStream_t st) {
  const bf_config& c = s->cfg;
  const double full = 4.0 * c.S_seq * (double)S_mb * c.S_seq * c.S_hidden;
  return timed(s, BF_K_ATTN_FWD, c.causal ? full / 2 : full, 0.0, st, [&] {
    return attention_fwd(c.dtype, c.kernels, S_mb, c.S_seq, c.N_heads, c.S_head, c.causal, qkv, ctx, lse, st);
  });
}
// db_qkv: the QKV bias gradient (column sums of dqkv), taken on the way when `part` is there
bf_status p_attn_bwd(bf_stack* s, int S_mb, const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                     float* delta, float* db_qkv, float* part, int acc, hipStream_t st) {
  const bf_config& c = s->cfg;
  const double full = 4.0 * c.S_seq * (double)S_mb * c.S_seq * c.S_hidden;
  // algorithmic backward = 2.5 x forward (five score-sized products); the two-pass kernels run seven
  return timed(s, BF_K_ATTN_BWD, 2.5 * (c.causal ? full / 2 : full), 0.0, st, [&] {
    return attention_bwd(c.dtype, c.kernels, S_mb, c.S_seq, c.N_heads, c.S_head, c.causal, qkv, ctx, lse, dctx, dqkv, delta, st,
                         db_qkv, part, acc);
  });
}

// Forward of one layer on T tokens.  x: layer input; R: where the activations go; y: output.
// skip_fc2: recomputation before a backward does not need the layer output.
bf_status layer_forward(bf_stack* s, int layer, int S_mb, const void* x, const Record& R, void* y, bool skip_fc2,
                        hipStream_t st) {
  const bf_config& c = s->cfg;
  const int T = S_mb * c.S_seq, h = c.S_hidden, f = c.S_mlp, dt = c.dtype, kn = c.kernels;
  auto P = [&](int tid) { return param_ptr(s, s->w32, layer, tid); };
  BF_TRY(p_ln_fwd(s, T, h, x, P(BF_LN1_G), P(BF_LN1_B), c.ln_eps, R.a, R.ln1, st));
  GemmArgs g{};
  g = GemmArgs{T, 3 * h, h, R.a, weight_ptr(s, layer, BF_W_QKV), R.qkv, P(BF_B_QKV), nullptr, nullptr, 0};
  BF_TRY(p_gemm(s, L_NN, E_BIAS, g, st));
  BF_TRY(p_attn_fwd(s, S_mb, R.qkv, R.ctx, R.lse, st));
  g = GemmArgs{T, h, h, R.ctx, weight_ptr(s, layer, BF_W_O), R.x1, P(BF_B_O), x, nullptr, 0};
  BF_TRY(p_gemm(s, L_NN, E_BIAS_RES, g, st));
  BF_TRY(p_ln_fwd(s, T, h, R.x1, P(BF_LN2_G), P(BF_LN2_B), c.ln_eps, R.c, R.ln2, st));
  g = GemmArgs{T, f, h, R.c, weight_ptr(s, layer, BF_W_FC1), R.u, P(BF_B_FC1), nullptr, R.g, 0};
  BF_TRY(p_gemm(s, L_NN, E_BIAS_GELU, g, st));
  if (!skip_fc2) {
    g = GemmArgs{T, h, f, R.g, weight_ptr(s, layer, BF_W_FC2), y, P(BF_B_FC2), R.x1, nullptr, 0};
    BF_TRY(p_gemm(s, L_NN, E_BIAS_RES, g, st));
  }
  return BF_OK;
}

// Backward of one layer.  dy: gradient w.r.t. the layer output; dx: gradient w.r.t. its input.
// acc: 0 for the first micro-batch of the step (main-grads are overwritten), 1 afterwards.
// keep: null, or where du / dx1 / dqkv are kept for a later weight-gradient product over all the
// micro-batches of the stage (then no weight-matrix gradient is taken here).
// dy_summed: the column sums of dy (this layer's FC2 bias gradient) were taken by whoever produced dy.
// below_b_fc2: null, or the FC2 bias gradient of the layer that dx feeds: its column sums are taken here, on the way.
bf_status layer_backward(bf_stack* s, int layer, int S_mb, const void* x, const Record& R, const void* dy, void* dx,
                         int acc, const GradRec* keep, bool dy_summed, float* below_b_fc2, hipStream_t st) {
  const bf_config& c = s->cfg;
  const int T = S_mb * c.S_seq, h = c.S_hidden, f = c.S_mlp;
  Tmp t = tmp_of(s);
  char* du = keep ? keep->du : t.du;
  char* dx1 = keep ? keep->dx1 : t.dx1;
  char* dqkv = keep ? keep->dqkv : t.dqkv;
  auto P = [&](int tid) { return param_ptr(s, s->w32, layer, tid); };
  // the second chain of a two-chain step sums its bias / LayerNorm gradients in an arena of its own
  if (s->chain && !keep) { set_error("layer_backward: the second chain takes no weight-matrix gradients"); return BF_ESTATE; }
  auto G = [&](int tid) { return param_ptr(s, s->chain ? s->g32b : s->g32, layer, tid); };
  GemmArgs g{};
  // y = x1 + gelu(u) W_fc2 + b_fc2
  if (!keep) {
    g = GemmArgs{f, h, T, R.g, dy, G(BF_W_FC2), nullptr, nullptr, nullptr, acc};
    BF_TRY(p_gemm(s, L_TN, E_ACCUM, g, st));
  }
  if (!dy_summed) BF_TRY(p_colsum(s, T, h, dy, G(BF_B_FC2), acc, st));
  // du = (dy W_fc2^T) gelu'(u), and on the way the bias gradient of FC1, the column sums of du: taken in the
  // product's epilogue (per-tile partial sums, then a small fixed-order reduction) instead of a second pass over du
  g = GemmArgs{T, f, h, dy, weight_ptr(s, layer, BF_W_FC2), du, nullptr, R.u, nullptr, acc};
  g.colsum = G(BF_B_FC1);
  g.colsum_part = t.colpart;
  BF_TRY(p_gemm(s, L_NT, E_GELU_BWD, g, st));
  // u = c W_fc1 + b_fc1
  if (!keep) {
    g = GemmArgs{h, f, T, R.c, du, G(BF_W_FC1), nullptr, nullptr, nullptr, acc};
    BF_TRY(p_gemm(s, L_TN, E_ACCUM, g, st));
  }
  g = GemmArgs{T, h, f, du, weight_ptr(s, layer, BF_W_FC1), t.dc, nullptr, nullptr, nullptr, 0};
  BF_TRY(p_gemm(s, L_NT, E_NONE, g, st));
  // c = LN2(x1); dx1 = dy + LN2'(dc); the column sums of dx1 are the out-projection's bias gradient
  BF_TRY(p_ln_bwd(s, T, h, t.dc, R.x1, P(BF_LN2_G), R.ln2, dy, dx1, G(BF_LN2_G), G(BF_LN2_B), G(BF_B_O), acc, st));
  // x1 = x + ctx W_o + b_o
  if (!keep) {
    g = GemmArgs{h, h, T, R.ctx, dx1, G(BF_W_O), nullptr, nullptr, nullptr, acc};
    BF_TRY(p_gemm(s, L_TN, E_ACCUM, g, st));
  }
  g = GemmArgs{T, h, h, dx1, weight_ptr(s, layer, BF_W_O), t.dctx, nullptr, nullptr, nullptr, 0};
  BF_TRY(p_gemm(s, L_NT, E_NONE, g, st));
  // qkv = a W_qkv + b_qkv: the bias gradient is the column sum of dqkv, which the attention kernels take on their way out
  BF_TRY(p_attn_bwd(s, S_mb, R.qkv, R.ctx, R.lse, t.dctx, dqkv, t.delta, G(BF_B_QKV), t.attnpart, acc, st));
  if (!keep) {
    g = GemmArgs{h, 3 * h, T, R.a, dqkv, G(BF_W_QKV), nullptr, nullptr, nullptr, acc};
    BF_TRY(p_gemm(s, L_TN, E_ACCUM, g, st));
  }
  g = GemmArgs{T, h, 3 * h, dqkv, weight_ptr(s, layer, BF_W_QKV), t.dc, nullptr, nullptr, nullptr, 0};
  BF_TRY(p_gemm(s, L_NT, E_NONE, g, st));
  // a = LN1(x); dx = dx1 + LN1'(da); dx is the gradient arriving at the layer below, whose FC2 bias gradient is
  // its column sums
  BF_TRY(p_ln_bwd(s, T, h, t.dc, x, P(BF_LN1_G), R.ln1, dx1, dx, G(BF_LN1_G), G(BF_LN1_B), below_b_fc2, acc, st));
  return BF_OK;
}

// The four weight-matrix gradients of one layer as products over all N_mb micro-batches at once
// (breadth-first only: every micro-batch of the stage has been through its backward, Sec. 4.2).
// G = sum_m X_m^T dY_m is one long contraction, written once: no read-modify-write of the fp32
// main-grad per micro-batch.  dy0 / dy_stride: the layer's incoming gradients, micro-batch 0 and
// the distance (elements) between micro-batches.
bf_status layer_wgrad_fused(bf_stack* s, int layer, int ls, int S_mb, int N_mb, const void* dy0, size_t dy_stride,
                            hipStream_t st) {
  const bf_config& c = s->cfg;
  const int T = S_mb * c.S_seq, h = c.S_hidden, f = c.S_mlp;
  const size_t esz = c.dtype == BF_BF16 ? 2 : 4;
  Record R0 = record_for(s, layer, 0);
  size_t rec_stride = (s->Lo.rec_bytes + s->Lo.y_bytes) / esz;
  if (c.ckpt_mode == BF_CKPT_LAYER) {
    redirect_wgrad_operands(s, ls, 0, &R0);
    rec_stride = s->Lo.wrec_bytes / esz;
  }
  const GradRec K0 = grad_rec(s, ls, 0);
  const size_t grec_stride = s->Lo.grec_bytes / esz;
  auto G = [&](int tid) { return param_ptr(s, s->g32, layer, tid); };
  auto run = [&](int M, int N, const void* A, const void* B, size_t sb, float* out) {
    GemmArgs g{M, N, T, A, B, out, nullptr, nullptr, nullptr, 0};
    g.n_seg = N_mb;
    g.seg_stride_a = rec_stride;
    g.seg_stride_b = sb;
    return p_gemm(s, L_TN, E_ACCUM, g, st);
  };
  BF_TRY(run(f, h, R0.g, dy0, dy_stride, G(BF_W_FC2)));
  BF_TRY(run(h, f, R0.c, K0.du, grec_stride, G(BF_W_FC1)));
  BF_TRY(run(h, h, R0.ctx, K0.dx1, grec_stride, G(BF_W_O)));
  BF_TRY(run(h, 3 * h, R0.a, K0.dqkv, grec_stride, G(BF_W_QKV)));
  return BF_OK;
}

}  // namespace
}  // namespace bf

extern "C" {

const char* bf_last_error(void) { return bf::g_err; }

int64_t bf_param_count(const bf_config* cfg) {
  if (!valid_config(cfg)) return 0;
  Dims D;
  fill_dims(*cfg, &D);
  int64_t n = 0;
  for (int i = 0; i < BF_N_TENSORS; ++i) n += (int64_t)D.tensor_elems[i];
  n *= cfg->N_layers;
  for (int i = 0; i < BF_N_VOCAB_TENSORS; ++i) n += (int64_t)D.voc_elems[i];
  return n;
}

size_t bf_workspace_bytes(const bf_config* cfg) {
  if (!valid_config(cfg)) return 0;
  Dims D;
  WsLayout Lo;
  fill_dims(*cfg, &D);
  fill_layout(*cfg, D, &Lo);
  return Lo.total;
}

bf_status bf_create_stack(const bf_config* cfg, void* workspace, size_t bytes, void* stream, bf_stack** out) {
  if (!out) { set_error("bf_create_stack: out is null"); return BF_EINVAL; }
  *out = nullptr;
  if (!valid_config(cfg)) return BF_EINVAL;
  if (!workspace || ((uintptr_t)workspace & (ALIGN - 1))) { set_error("bf_create_stack: workspace null or not 256-byte aligned"); return BF_EINVAL; }
  bf_stack* s = new (std::nothrow) bf_stack();
  if (!s) { set_error("bf_create_stack: host allocation failed"); return BF_ENOMEM; }
  s->cfg = *cfg;
  fill_dims(*cfg, &s->D);
  fill_layout(*cfg, s->D, &s->Lo);
  if (bytes < s->Lo.total) {
    set_error("bf_create_stack: workspace has %zu bytes, %zu needed", bytes, s->Lo.total);
    delete s;
    return BF_ENOMEM;
  }
  s->ws = (char*)workspace;
  s->w32 = (float*)(s->ws + s->Lo.off_w32);
  s->m = (float*)(s->ws + s->Lo.off_m);
  s->v = (float*)(s->ws + s->Lo.off_v);
  s->g32 = (float*)(s->ws + s->Lo.off_g32);
  s->wlp = cfg->dtype == BF_BF16 && !cfg->dp_fs ? (bf16_t*)(s->ws + s->Lo.off_wlp) : nullptr;
  s->wlp_voc = cfg->dp_fs && cfg->S_voc > 0 ? (bf16_t*)(s->ws + s->Lo.off_wlp_voc) : nullptr;
  for (int i = 0; i < 2; ++i) {
    s->fs_half[i] = cfg->dp_fs ? (bf16_t*)(s->ws + s->Lo.off_wlp + i * s->Lo.half_bytes) : nullptr;
    s->fs_l0[i] = s->fs_n[i] = -1;
    s->fs_ready[i] = s->fs_free[i] = nullptr;
  }
  s->fs_cur = 0;
  s->fs_cur_l0 = 0;
  s->step = 0;
  s->d_step = (int*)(s->ws + s->Lo.off_step);
  s->have_grads = false;
  s->prof_on = false;
  s->prof_mask = 0;
  s->side = nullptr;
  s->ev_grad_ready = s->ev_side_done = s->ev_t0 = s->ev_t1 = nullptr;
  s->chain = 0;
  s->chains_active = 1;
  s->g32b = cfg->mb_chains == 2 ? (float*)(s->ws + s->Lo.off_g32b) : nullptr;
  s->chain_st = nullptr;
  for (auto& e : s->ev_chain) e = nullptr;
  hipStream_t st = (hipStream_t)stream;
  auto fail = [&](bf_status code) { bf_destroy_stack(s); return code; };
#define CK(expr)                                                                                  \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) { set_error("%s failed: %s", #expr, hipGetErrorString(e_)); return fail(BF_EDEVICE); } \
  } while (0)
  CK(hipGetDevice(&s->device));
  CK(hipStreamCreateWithFlags(&s->side, hipStreamNonBlocking));
  CK(hipEventCreateWithFlags(&s->ev_grad_ready, hipEventDisableTiming));
  CK(hipEventCreateWithFlags(&s->ev_side_done, hipEventDisableTiming));
  CK(hipEventCreate(&s->ev_t0));
  CK(hipEventCreate(&s->ev_t1));
  if (cfg->mb_chains == 2) {
    CK(hipStreamCreateWithFlags(&s->chain_st, hipStreamNonBlocking));
    for (auto& e : s->ev_chain) CK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  }
  if (cfg->dp_fs)
    for (int i = 0; i < 2; ++i) {
      CK(hipEventCreateWithFlags(&s->fs_ready[i], hipEventDisableTiming));
      CK(hipEventCreateWithFlags(&s->fs_free[i], hipEventDisableTiming));
    }
  s->adam_ev.resize(2 * (size_t)cfg->N_layers, nullptr);
  for (auto& e : s->adam_ev) CK(hipEventCreate(&e));
  if (cfg->queue_depth > 0) {
    s->queue_ev.resize(cfg->queue_depth, nullptr);
    for (auto& e : s->queue_ev) CK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  }
#undef CK
  // initialise: zero everything, then weights ~ N(0, init_std), LN gains 1
  const size_t P = s->Lo.P_total;
  bf_status r;
  if ((r = fill_f32(P, s->w32, 0.f, st)) != BF_OK || (r = fill_f32(P, s->m, 0.f, st)) != BF_OK ||
      (r = fill_f32(P, s->v, 0.f, st)) != BF_OK || (r = fill_f32(P, s->g32, 0.f, st)) != BF_OK ||
      (r = fill_f32(1, (float*)s->d_step, 0.f, st)) != BF_OK)  // integer 0 has the bit pattern of 0.f
    return fail(r);
  for (int l = 0; l < cfg->N_layers; ++l) {
    const int wt[4] = {BF_W_QKV, BF_W_O, BF_W_FC1, BF_W_FC2};
    for (int i = 0; i < 4; ++i) {
      const uint64_t sd = cfg->seed * 0x9E3779B97F4A7C15ull + (uint64_t)l * BF_N_TENSORS + wt[i];
      if ((r = init_normal(s->D.tensor_elems[wt[i]], param_ptr(s, s->w32, l, wt[i]), sd, cfg->init_std, st)) != BF_OK)
        return fail(r);
    }
    if ((r = fill_f32(s->D.tensor_elems[BF_LN1_G], param_ptr(s, s->w32, l, BF_LN1_G), 1.f, st)) != BF_OK) return fail(r);
    if ((r = fill_f32(s->D.tensor_elems[BF_LN2_G], param_ptr(s, s->w32, l, BF_LN2_G), 1.f, st)) != BF_OK) return fail(r);
  }
  if (cfg->S_voc > 0) {
    const int wt[3] = {BF_E_TOK, BF_E_POS, BF_W_OUT};
    for (int i = 0; i < 3; ++i) {
      const uint64_t sd = cfg->seed * 0x9E3779B97F4A7C15ull + (uint64_t)cfg->N_layers * BF_N_TENSORS + wt[i];
      if ((r = init_normal(s->D.voc_elems[wt[i] - BF_E_TOK], param_ptr(s, s->w32, 0, wt[i]), sd, cfg->init_std, st)) != BF_OK)
        return fail(r);
    }
    if ((r = fill_f32(s->D.voc_elems[BF_LNF_G - BF_E_TOK], param_ptr(s, s->w32, 0, BF_LNF_G), 1.f, st)) != BF_OK) return fail(r);
  }
  if (s->wlp && (r = cast_f32_to_bf16(P, s->w32, s->wlp, st)) != BF_OK) return fail(r);
  if (s->wlp_voc && (r = cast_f32_to_bf16(s->D.voc_total, s->w32 + s->Lo.P_layers, s->wlp_voc, st)) != BF_OK) return fail(r);
  hipError_t e = hipStreamSynchronize(st);
  if (e != hipSuccess) { set_error("bf_create_stack: initialisation failed: %s", hipGetErrorString(e)); return fail(BF_EDEVICE); }
  *out = s;
  return BF_OK;
}

bf_status bf_destroy_stack(bf_stack* s) {
  if (!s) return BF_OK;
  if (s->side) { (void)hipStreamSynchronize(s->side); (void)hipStreamDestroy(s->side); }
  if (s->chain_st) { (void)hipStreamSynchronize(s->chain_st); (void)hipStreamDestroy(s->chain_st); }
  for (hipEvent_t e : s->ev_chain) if (e) (void)hipEventDestroy(e);
  hipEvent_t evs[8] = {s->ev_grad_ready, s->ev_side_done, s->ev_t0, s->ev_t1,
                       s->fs_ready[0], s->fs_ready[1], s->fs_free[0], s->fs_free[1]};
  for (hipEvent_t e : evs) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : s->adam_ev) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : s->queue_ev) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : s->prof_ev) if (e) (void)hipEventDestroy(e);
  delete s;
  return BF_OK;
}

size_t bf_tensor_elems(const bf_stack* s, int tensor_id) {
  if (!s || tensor_id < 0 || tensor_id >= BF_N_TENSORS + BF_N_VOCAB_TENSORS) return 0;
  return tensor_id < BF_N_TENSORS ? s->D.tensor_elems[tensor_id] : s->D.voc_elems[tensor_id - BF_E_TOK];
}

static bf_status check_tensor(bf_stack* s, int layer, int tid, const void* host, size_t n) {
  if (!s || !host) { set_error("null stack or host pointer"); return BF_EINVAL; }
  const bool voc = tid >= BF_E_TOK && tid < BF_E_TOK + BF_N_VOCAB_TENSORS && s->cfg.S_voc > 0;
  // the input / output layers are addressed as pseudo-layer N_layers
  if (voc ? layer != s->cfg.N_layers : (layer < 0 || layer >= s->cfg.N_layers || tid < 0 || tid >= BF_N_TENSORS)) {
    set_error("bad layer %d or tensor id %d", layer, tid);
    return BF_EINVAL;
  }
  if (n != bf_tensor_elems(s, tid)) { set_error("tensor %d has %zu elements, caller passed %zu", tid, bf_tensor_elems(s, tid), n); return BF_EINVAL; }
  return BF_OK;
}

bf_status bf_set_params(bf_stack* s, int layer, int tid, const float* host_src, size_t n) {
  BF_TRY(check_tensor(s, layer, tid, host_src, n));
  BF_HIP_CHECK(hipDeviceSynchronize());
  float* dst = param_ptr(s, s->w32, layer, tid);
  BF_HIP_CHECK(hipMemcpy(dst, host_src, n * sizeof(float), hipMemcpyHostToDevice));
  if (bf16_t* lp = lp_ptr(s, dst - s->w32)) {
    BF_TRY(cast_f32_to_bf16(n, dst, lp, nullptr));
    BF_HIP_CHECK(hipDeviceSynchronize());
  }
  s->fs_l0[0] = s->fs_l0[1] = -1;  // dp_fs: whatever the double buffer holds is stale now
  return BF_OK;
}

static bf_status get_from(bf_stack* s, float* arena, int layer, int tid, float* host_dst, size_t n) {
  BF_TRY(check_tensor(s, layer, tid, host_dst, n));
  BF_HIP_CHECK(hipDeviceSynchronize());
  BF_HIP_CHECK(hipMemcpy(host_dst, param_ptr(s, arena, layer, tid), n * sizeof(float), hipMemcpyDeviceToHost));
  return BF_OK;
}

bf_status bf_get_params(bf_stack* s, int layer, int tid, float* host_dst, size_t n) {
  if (!s) { set_error("null stack"); return BF_EINVAL; }
  return get_from(s, s->w32, layer, tid, host_dst, n);
}

bf_status bf_get_grads(bf_stack* s, int layer, int tid, float* host_dst, size_t n) {
  if (!s) { set_error("null stack"); return BF_EINVAL; }
  if (!s->have_grads) { set_error("bf_get_grads: no step has run yet"); return BF_ESTATE; }
  return get_from(s, s->g32, layer, tid, host_dst, n);
}

bf_status bf_get_moments(bf_stack* s, int layer, int tid, int which, float* host_dst, size_t n) {
  if (!s) { set_error("null stack"); return BF_EINVAL; }
  if (which != 0 && which != 1) { set_error("bf_get_moments: which must be 0 or 1"); return BF_EINVAL; }
  return get_from(s, which ? s->v : s->m, layer, tid, host_dst, n);
}

bf_status bf_reset_optimizer(bf_stack* s) {
  if (!s) { set_error("null stack"); return BF_EINVAL; }
  BF_HIP_CHECK(hipDeviceSynchronize());
  BF_TRY(fill_f32(s->Lo.P_total, s->m, 0.f, nullptr));
  BF_TRY(fill_f32(s->Lo.P_total, s->v, 0.f, nullptr));
  BF_TRY(fill_f32(1, (float*)s->d_step, 0.f, nullptr));  // the bit pattern of integer 0
  BF_HIP_CHECK(hipDeviceSynchronize());
  s->step = 0;
  return BF_OK;
}

bf_status bf_get_trace(const bf_stack* s, bf_event* dst, size_t cap, size_t* n) {
  if (!s || !n) { set_error("bf_get_trace: null argument"); return BF_EINVAL; }
  *n = s->trace.size();
  if (dst) {
    const size_t k = cap < s->trace.size() ? cap : s->trace.size();
    if (k) memcpy(dst, s->trace.data(), k * sizeof(bf_event));
  }
  return BF_OK;
}

bf_status bf_schedule_trace(int schedule, int N_PP, int N_loop, int N_mb, int rank, int t_fwd, int t_bwd, bf_event* dst,
                            size_t cap, size_t* n, bf_sched_stats* stats) {
  std::vector<SchedOp> ops;
  std::string why;
  if (!rank_order(schedule, N_PP, N_loop, N_mb, rank, &ops, &why)) { set_error("%s", why.c_str()); return BF_EINVAL; }
  if (n) *n = ops.size();
  if (dst) {
    int live = 0;
    for (size_t i = 0; i < ops.size() && i < cap; ++i) {
      live += ops[i].op == 0 ? 1 : -1;
      dst[i] = bf_event{ops[i].op, ops[i].stage, ops[i].mb, live};
    }
  }
  if (stats) {
    std::vector<int64_t> peak;
    if (!simulate(schedule, N_PP, N_loop, N_mb, t_fwd, t_bwd, stats, &peak, &why)) { set_error("%s", why.c_str()); return BF_EINVAL; }
    stats->peak_live = peak[rank];
  }
  return BF_OK;
}

// One step of rank `rank` of an N_PP-deep looped pipeline.  chained: the rank's stages feed each
// other (N_PP = 1: x / dy / y / dx hold one tensor per micro-batch); otherwise every stage takes
// its input and incoming gradient from the caller's buffers and leaves its output and outgoing
// gradient there (one tensor per local stage and micro-batch), as a rank that receives from and
// sends to its neighbours would.
// lm: null, or the token ids, labels and loss output of a step with the input and output layers
// (chained only; x / dy / y / dx are then unused).
struct LmIO { const int32_t* tokens; const int32_t* labels; float* loss; };

static bf_status run_rank_step(bf_stack* s, int schedule, int N_PP, int rank, bool chained, int N_loop, int N_mb, int S_mb,
                               const void* x, const void* dy, void* y, void* dx, const LmIO* lm, int apply_optimizer,
                               int timing, void* stream, bf_step_report* report) {
  if (!s) { set_error("bf_run_step: null stack"); return BF_EINVAL; }
  const bf_config& c = s->cfg;
  if (schedule != BF_SCHED_BF && schedule != BF_SCHED_DF) { set_error("bf_run_step: unknown schedule %d", schedule); return BF_EINVAL; }
  if (timing < 0 || timing > 3) { set_error("bf_run_step: timing %d outside 0..3", timing); return BF_EINVAL; }
  if (N_loop < 1 || c.N_layers % N_loop) { set_error("bf_run_step: N_loop = %d must divide N_layers = %d", N_loop, c.N_layers); return BF_EINVAL; }
  if (N_mb < 1 || N_mb > c.N_mb_max) { set_error("bf_run_step: N_mb = %d outside 1..%d", N_mb, c.N_mb_max); return BF_EINVAL; }
  if (S_mb < 1 || S_mb > c.S_mb_max) { set_error("bf_run_step: S_mb = %d outside 1..%d", S_mb, c.S_mb_max); return BF_EINVAL; }
  if (!lm && (!x || !dy)) { set_error("bf_run_step: x and dy must not be null"); return BF_EINVAL; }
  int cur = -1;
  BF_HIP_CHECK(hipGetDevice(&cur));
  if (cur != s->device) { set_error("bf_run_step: stack lives on device %d, current device is %d", s->device, cur); return BF_EINVAL; }

  hipStream_t st = (hipStream_t)stream;
  const size_t es = c.dtype == BF_BF16 ? 2 : 4;
  const int per_stage = c.N_layers / N_loop;
  const size_t mb_bytes = (size_t)S_mb * c.S_seq * c.S_hidden * es;
  s->chain = 0;
  Tmp tmp = tmp_of(s);
  // gradient hand-off between stages: stage j reads set j & 1 and writes set (j - 1) & 1, so the
  // gradients a stage received stay intact until its fused weight-gradient products have run
  auto bhand = [&](int stage, int m) { return s->ws + s->Lo.off_bhand + ((size_t)(stage & 1) * c.N_mb_max + m) * s->Lo.y_bytes; };
  char* scratch_out = s->ws + s->Lo.off_scratch_out;
  // input / output layers: embedded input and loss gradient of every micro-batch, then one micro-batch's
  // last-layer output, its normalised form, the gradient of that, LayerNorm statistics, logits, row losses
  char* lm_base = s->ws + s->Lo.off_lm;
  auto emb_x = [&](int m) { return lm_base + (size_t)m * s->Lo.y_bytes; };
  auto dy_lm = [&](int m) { return lm_base + ((size_t)c.N_mb_max + m) * s->Lo.y_bytes; };
  char* y_top = lm_base + 2 * (size_t)c.N_mb_max * s->Lo.y_bytes;
  char* hn = y_top + s->Lo.y_bytes;
  char* dhn = hn + s->Lo.y_bytes;
  float* lnf_stats = (float*)(dhn + s->Lo.y_bytes);
  char* logits = (char*)lnf_stats + up((size_t)c.S_mb_max * c.S_seq * 8);
  float* row_loss = (float*)(logits + s->Lo.logits_bytes);
  const int T_mb = S_mb * c.S_seq;
  if (lm) {
    x = emb_x(0);
    dy = dy_lm(0);
    y = nullptr;
    dx = nullptr;
  }
  const bool fuse = schedule == BF_SCHED_BF && fuse_wgrad_possible(c) && per_stage <= lps_max(c);
  // Two chains: micro-batch m runs on stream m & 1, so two micro-batches of a stage are in flight side by side and a
  // kernel with fewer workgroups than the chip has compute units shares it with the other chain's.  Micro-batches
  // of one stage are independent of each other in both directions (Sec. 4.2), which is what breadth-first order
  // leaves room for, on a rank of a deeper pipeline as well (its order has every micro-batch of a stage in a row
  // too); depth-first order, the input / output layers and steps without caller buffers for the outputs (they
  // would share one scratch tensor) run as one chain.
  const int chains = c.mb_chains == 2 && fuse && !lm && N_mb >= 2 && y && dx ? 2 : 1;
  auto stream_of = [&](int m) { return chains == 2 && (m & 1) ? s->chain_st : st; };
  s->chains_active = chains;
  if (c.dp_fs && per_stage > lps_max(c)) {
    set_error("bf_run_step: dp_fs holds stages of up to %d layers (N_loop_min = %d), N_loop = %d gives %d", lps_max(c),
              c.N_loop_min, N_loop, per_stage);
    return BF_EINVAL;
  }

  std::vector<SchedOp> ops;
  std::string why;
  if (!rank_order(schedule, N_PP, N_loop, N_mb, rank, &ops, &why)) { set_error("%s", why.c_str()); return BF_EINVAL; }
  // local index of an op's stage: the rank holds the global stages ls * N_PP + rank (Sec. 4.1)
  auto local = [&](const SchedOp& o) { return o.stage / N_PP; };
  // the caller's tensor of (local stage, micro-batch)
  const size_t io_stride = lm ? s->Lo.y_bytes : mb_bytes;
  auto io_off = [&](int ls, int m) { return ((size_t)(chained ? 0 : ls) * N_mb + m) * io_stride; };

  // dp_fs: cut the order into intervals (runs of one stage in one direction) and decide, in order,
  // which half of the double buffer serves each and whether the stage has to be reconstructed into
  // it: a stage still resident is reused, otherwise it goes to the half the previous interval is
  // not reading, so that the reconstruction can run beside that interval (App. D.1).
  struct Interval { int stage, half; bool load; };
  std::vector<Interval> ivs;
  std::vector<int> iv_of(ops.size(), -1);
  if (c.dp_fs) {
    int l0h[2] = {s->fs_l0[0], s->fs_l0[1]}, nh[2] = {s->fs_n[0], s->fs_n[1]};
    for (size_t i = 0; i < ops.size(); ++i) {
      if (i == 0 || ops[i].stage != ops[i - 1].stage || ops[i].op != ops[i - 1].op) {
        const int l0 = local(ops[i]) * per_stage;
        Interval iv{local(ops[i]), 0, true};
        const int prev = ivs.empty() ? 1 : ivs.back().half;
        if (l0h[0] == l0 && nh[0] == per_stage) { iv.half = 0; iv.load = false; }
        else if (l0h[1] == l0 && nh[1] == per_stage) { iv.half = 1; iv.load = false; }
        else { iv.half = prev ^ 1; l0h[iv.half] = l0; nh[iv.half] = per_stage; }
        ivs.push_back(iv);
      }
      iv_of[i] = (int)ivs.size() - 1;
    }
  }
  int64_t n_recon = 0;
  // enqueue the reconstruction of interval j on the side stream, after everything issued so far
  // on the caller's stream (the earlier readers of that half, earlier optimizer steps)
  auto reconstruct = [&](int j) -> bf_status {
    const Interval& iv = ivs[j];
    const size_t off = (size_t)iv.stage * per_stage * s->D.layer_elems, n = (size_t)per_stage * s->D.layer_elems;
    BF_HIP_CHECK(hipEventRecord(s->fs_free[iv.half], st));
    BF_HIP_CHECK(hipStreamWaitEvent(s->side, s->fs_free[iv.half], 0));
    BF_TRY(timed(s, BF_K_RECONSTRUCT, 0.0, 6.0 * (double)n, s->side,
                 [&] { return cast_f32_to_bf16(n, s->w32 + off, s->fs_half[iv.half], s->side); }));
    BF_HIP_CHECK(hipEventRecord(s->fs_ready[iv.half], s->side));
    s->fs_l0[iv.half] = iv.stage * per_stage;
    s->fs_n[iv.half] = per_stage;
    ++n_recon;
    return BF_OK;
  };

  s->trace.clear();
  s->have_grads = false;
  s->prof_on = timing == 2 || timing == 3;
  s->prof_mask = timing == 2 ? ~0u : 1u << BF_K_GEMM_WGRAD;
  s->prof_rec.clear();
  if (apply_optimizer) {
    s->step += 1;
    BF_TRY(bump_step(s->d_step, st));
  }
  int live = 0;
  int64_t peak_live = 0;
  size_t n_adam = 0, qi = 0;
  if (timing) BF_HIP_CHECK(hipEventRecord(s->ev_t0, st));
  if (chains == 2) {
    // the second chain starts after everything the caller's stream holds so far
    BF_HIP_CHECK(hipEventRecord(s->ev_chain[0], st));
    BF_HIP_CHECK(hipStreamWaitEvent(s->chain_st, s->ev_chain[0], 0));
  }

  // where a stage meets the caller's buffers: the first layer's input and outgoing gradient, the
  // last layer's output and incoming gradient (chained: only the rank's first and last layer)
  auto is_bottom = [&](int layer) { return chained ? layer == 0 : layer % per_stage == 0; };
  auto is_top = [&](int layer) { return chained ? layer == c.N_layers - 1 : layer % per_stage == per_stage - 1; };
  // layer input of (layer, mb): the caller's x at a stage bottom, else the previous layer's stored output
  auto input_of = [&](int layer, int m) -> const void* {
    if (is_bottom(layer)) return (const char*)x + io_off(layer / per_stage, m);
    return record_for(s, layer - 1, m).y;
  };

  for (size_t oi = 0; oi < ops.size(); ++oi) {
    const SchedOp& op = ops[oi];
    const int ls = local(op), l0 = ls * per_stage, l1 = l0 + per_stage, m = op.mb;
    // the stream this op is issued on, and with it the set of temporaries and the arena of the small gradients
    hipStream_t os = stream_of(m);
    s->chain = chains == 2 ? m & 1 : 0;
    const int first = m < chains ? 0 : 1;  // 0: the chain's first micro-batch overwrites its gradient sums
    if (c.dp_fs && (oi == 0 || iv_of[oi] != iv_of[oi - 1])) {
      // a new interval starts: its weights must have arrived, and the next interval's are sent for
      const int j = iv_of[oi];
      if (j == 0 && ivs[0].load) BF_TRY(reconstruct(0));
      if (ivs[j].load) BF_HIP_CHECK(hipStreamWaitEvent(os, s->fs_ready[ivs[j].half], 0));
      s->fs_cur = ivs[j].half;
      s->fs_cur_l0 = l0;
      if (j + 1 < (int)ivs.size() && ivs[j + 1].load) BF_TRY(reconstruct(j + 1));
    }
    if (op.op == 0) {
      if (lm && l0 == 0) {
        if (m == 0)  // the token rows' gradients are added to, use by use: start from zero
          BF_TRY(fill_f32(s->D.voc_elems[0], param_ptr(s, s->g32, 0, BF_E_TOK), 0.f, os));
        BF_TRY(timed(s, BF_K_VOCAB, 0.0, (double)T_mb * c.S_hidden * (8.0 + es), os, [&] {
          return embedding_fwd(c.dtype, T_mb, c.S_seq, c.S_voc, c.S_hidden, lm->tokens + (size_t)m * T_mb,
                               param_ptr(s, s->w32, 0, BF_E_TOK), param_ptr(s, s->w32, 0, BF_E_POS), emb_x(m), os);
        }));
      }
      for (int l = l0; l < l1; ++l) {
        Record R = record_for(s, l, m);
        void* out = R.y;
        if (is_top(l)) out = lm ? y_top : y ? (char*)y + io_off(ls, m) : scratch_out;
        BF_TRY(layer_forward(s, l, S_mb, input_of(l, m), R, out, false, os));
        ++live;
      }
      if (lm && l1 == c.N_layers) {
        // output layer, loss and their backward at once: nothing downstream has to be waited for
        const int h = c.S_hidden, V = c.S_voc;
        float* gw = param_ptr(s, s->g32, 0, BF_W_OUT);
        BF_TRY(p_ln_fwd(s, T_mb, h, y_top, param_ptr(s, s->w32, 0, BF_LNF_G), param_ptr(s, s->w32, 0, BF_LNF_B), c.ln_eps, hn,
                        lnf_stats, os));
        GemmArgs g{T_mb, V, h, hn, weight_ptr(s, 0, BF_W_OUT), logits, nullptr, nullptr, nullptr, 0};
        BF_TRY(p_gemm(s, L_NT, E_NONE, g, os));
        const float scale = 1.0f / ((float)N_mb * (float)T_mb);
        BF_TRY(timed(s, BF_K_VOCAB, 0.0, 3.0 * es * T_mb * V, os, [&] {
          return ce_loss(c.dtype, T_mb, V, logits, lm->labels + (size_t)m * T_mb, scale, row_loss, lm->loss + m, os);
        }));
        g = GemmArgs{T_mb, h, V, logits, weight_ptr(s, 0, BF_W_OUT), dhn, nullptr, nullptr, nullptr, 0};
        BF_TRY(p_gemm(s, L_NN, E_NONE, g, os));
        g = GemmArgs{V, h, T_mb, logits, hn, gw, nullptr, nullptr, nullptr, m > 0};
        BF_TRY(p_gemm(s, L_TN, E_ACCUM, g, os));
        BF_TRY(p_ln_bwd(s, T_mb, h, dhn, y_top, param_ptr(s, s->w32, 0, BF_LNF_G), lnf_stats, nullptr, dy_lm(m),
                        param_ptr(s, s->g32, 0, BF_LNF_G), param_ptr(s, s->g32, 0, BF_LNF_B), nullptr, m > 0, os));
      }
    } else {
      for (int l = l1 - 1; l >= l0; --l) {
        Record R = record_for(s, l, m);
        const void* xin = input_of(l, m);
        if (c.ckpt_mode == BF_CKPT_LAYER) {
          if (fuse) redirect_wgrad_operands(s, l - l0, m, &R);
          BF_TRY(layer_forward(s, l, S_mb, xin, R, nullptr, true, os));
        }
        // gradient in: caller's dy for the last layer, the hand-off buffer at a stage top, else the ping-pong
        // (with the fused weight gradient every layer's incoming gradient is kept per micro-batch instead)
        const void* din;
        if (is_top(l)) din = (const char*)dy + io_off(ls, m);
        else if (l == l1 - 1) din = bhand(ls, m);
        else din = fuse ? grad_rec(s, l - l0, m).dy : tmp.ping[(l + 1) & 1];
        void* dout;
        if (is_bottom(l)) dout = dx ? (char*)dx + io_off(ls, m) : scratch_out + s->Lo.y_bytes;
        else if (l == l0) dout = bhand(ls - 1, m);
        else dout = fuse ? grad_rec(s, l - 1 - l0, m).dy : tmp.ping[l & 1];
        GradRec keep{};
        if (fuse) keep = grad_rec(s, l - l0, m);
        // A layer whose incoming gradient was written by the layer above on this rank (everything but the top of
        // the chain, or of a stage when the stages do not feed each other) has had its FC2 bias gradient taken there.
        const bool fed_from_above = !is_top(l);
        float* below = is_bottom(l) ? nullptr : param_ptr(s, s->chain ? s->g32b : s->g32, l - 1, BF_B_FC2);
        BF_TRY(layer_backward(s, l, S_mb, xin, R, din, dout, first, fuse ? &keep : nullptr, fed_from_above, below, os));
        --live;
      }
      if (lm && l0 == 0) {
        char* dxe = scratch_out + s->Lo.y_bytes;  // where layer 0 left the gradient of its input
        BF_TRY(timed(s, BF_K_VOCAB, 0.0, (double)T_mb * c.S_hidden * (es + 16.0), os, [&] {
          return embedding_bwd(c.dtype, S_mb, c.S_seq, c.S_voc, c.S_hidden, lm->tokens + (size_t)m * T_mb, dxe,
                               param_ptr(s, s->g32, 0, BF_E_TOK), param_ptr(s, s->g32, 0, BF_E_POS), m > 0, os);
        }));
      }
      if (fuse && m == N_mb - 1) {
        if (chains == 2) {
          // the stage's last micro-batch: wait for the other chain's, which the products below read
          BF_HIP_CHECK(hipEventRecord(s->ev_chain[1], stream_of(m + 1)));
          BF_HIP_CHECK(hipStreamWaitEvent(os, s->ev_chain[1], 0));
        }
        // every micro-batch of the stage is through: one weight-gradient product per matrix
        for (int l = l1 - 1; l >= l0; --l) {
          const void* dy0;
          size_t stride;
          if (is_top(l)) { dy0 = (const char*)dy + io_off(ls, 0); stride = io_stride / es; }
          else if (l == l1 - 1) { dy0 = bhand(ls, 0); stride = s->Lo.y_bytes / es; }
          else { dy0 = grad_rec(s, l - l0, 0).dy; stride = s->Lo.grec_bytes / es; }
          BF_TRY(layer_wgrad_fused(s, l, l - l0, S_mb, N_mb, dy0, stride, os));
        }
        if (chains == 2) {
          // the two chains' bias / LayerNorm gradient sums become one, always in this order
          const int small[8] = {BF_LN1_G, BF_LN1_B, BF_B_QKV, BF_B_O, BF_LN2_G, BF_LN2_B, BF_B_FC1, BF_B_FC2};
          size_t off[8], cnt[8];
          for (int k = 0; k < 8; ++k) { off[k] = s->D.tensor_off[small[k]]; cnt[k] = s->D.tensor_elems[small[k]]; }
          const size_t lo = (size_t)l0 * s->D.layer_elems;
          BF_TRY(add_segments(per_stage, s->D.layer_elems, 8, off, cnt, s->g32 + lo, s->g32b + lo, os));
          // the next stage's backward reuses the buffers those products read: the other chain goes on only now
          BF_HIP_CHECK(hipEventRecord(s->ev_chain[2], os));
          BF_HIP_CHECK(hipStreamWaitEvent(stream_of(m + 1), s->ev_chain[2], 0));
        }
      }
    }
    peak_live = live > peak_live ? live : peak_live;
    s->trace.push_back(bf_event{op.op, op.stage, m, live});

    if (op.op == 1 && m == N_mb - 1) {
      // this stage's gradient is final (Sec. 4.2: breadth-first groups the work by stage)
      if (apply_optimizer) {
        const size_t off = (size_t)l0 * s->D.layer_elems, n = (size_t)per_stage * s->D.layer_elems;
        // The update runs in line, on the stream that issued the stage's last backward (the caller's, unless the step
        // runs two chains of micro-batches), as soon as the stage's gradient is final.
        // (On a side stream, "beside" the backward of the earlier stages, it is slower: the products
        // hold every compute unit, so the two do not overlap but take turns, a product that shares
        // the chip with the update's workgroups runs in more rounds, and under the power limit an
        // overlap would buy nothing anyway.  Measured: 1 % at C3, 7 % at the bidirectional workload.)
        hipStream_t as = os;
        if (timing) BF_HIP_CHECK(hipEventRecord(s->adam_ev[2 * n_adam], as));
        BF_TRY(timed(s, BF_K_ADAM, 0.0, (double)n * (s->wlp ? 30.0 : 28.0), as, [&] {
          return adam_step(n, s->w32 + off, s->m + off, s->v + off, s->g32 + off, s->wlp ? s->wlp + off : nullptr, s->step,
                           s->d_step, c.lr, c.beta1, c.beta2, c.adam_eps, c.weight_decay, as);
        }));
        if (lm) {
          // the input layer steps with the first stage, the output layer with the last
          auto voc_range = [&](int first, int last) {
            const size_t o = s->Lo.P_layers + s->D.voc_off[first - BF_E_TOK];
            const size_t cnt = s->D.voc_off[last - BF_E_TOK] + s->D.voc_elems[last - BF_E_TOK] - s->D.voc_off[first - BF_E_TOK];
            return timed(s, BF_K_ADAM, 0.0, (double)cnt * (lp_ptr(s, o) ? 30.0 : 28.0), as, [&] {
              return adam_step(cnt, s->w32 + o, s->m + o, s->v + o, s->g32 + o, lp_ptr(s, o), s->step, s->d_step, c.lr, c.beta1, c.beta2,
                               c.adam_eps, c.weight_decay, as);
            });
          };
          if (l0 == 0) BF_TRY(voc_range(BF_E_TOK, BF_E_POS));
          if (l1 == c.N_layers) BF_TRY(voc_range(BF_LNF_G, BF_W_OUT));
        }
        // dp_fs: the halves hold this stage's old weights at most until here
        for (int i = 0; i < 2; ++i) if (s->fs_l0[i] == l0) s->fs_l0[i] = -1;
        if (timing) BF_HIP_CHECK(hipEventRecord(s->adam_ev[2 * n_adam + 1], as));
        ++n_adam;
      }
      s->trace.push_back(bf_event{2, op.stage, -1, live});
    }
    if (!s->queue_ev.empty()) {
      // bounded launch queue (App. D.2): wait for the op issued queue_depth ops ago
      hipEvent_t e = s->queue_ev[qi % s->queue_ev.size()];
      if (qi >= s->queue_ev.size()) BF_HIP_CHECK(hipEventSynchronize(e));
      BF_HIP_CHECK(hipEventRecord(e, os));
      ++qi;
    }
  }
  s->chain = 0;
  s->chains_active = 1;
  if (chains == 2) {
    // the step ends on the caller's stream
    BF_HIP_CHECK(hipEventRecord(s->ev_chain[3], s->chain_st));
    BF_HIP_CHECK(hipStreamWaitEvent(st, s->ev_chain[3], 0));
  }
  if (apply_optimizer && schedule == BF_SCHED_BF) {
    BF_HIP_CHECK(hipEventRecord(s->ev_side_done, s->side));
    BF_HIP_CHECK(hipStreamWaitEvent(st, s->ev_side_done, 0));
  }
  s->have_grads = true;

  if (report) {
    memset(report, 0, sizeof *report);
    const double T = (double)S_mb * c.S_seq, h = c.S_hidden, f = c.S_mlp;
    const double lin = 2.0 * T * (3 * h * h + h * h + 2 * h * f);
    const double att = 4.0 * c.S_seq * T * h;  // full S_seq x S_seq scores
    const double lm_ = (double)c.N_layers * N_mb;
    const double head = lm ? 2.0 * T * h * (double)c.S_voc * N_mb : 0.0;  // output projection, forward
    report->flops_model = 3.0 * (lin + att) * lm_ + 3.0 * head;
    report->flops_paper = 4.0 * (lin + att) * lm_ + 3.0 * head;  // Eq. compute: no recomputation of the output layer
    const double att_f = c.causal ? att / 2 : att;
    // backward attention runs 7 score-sized products (dq pass: S, dP, dQ; dk/dv pass: S, dP, dK, dV) vs 2 forward
    double exec = 3.0 * lin + att_f * (1.0 + 3.5);
    if (c.ckpt_mode == BF_CKPT_LAYER) exec += (lin - 2.0 * T * h * f) + att_f;
    report->flops_executed = exec * lm_ + 3.0 * head;
    report->peak_ckpt_count = peak_live;
    report->peak_ckpt_bytes = peak_live * (int64_t)mb_bytes;
    const double frac = (double)S_mb / c.S_mb_max;
    const int64_t rec_live = (int64_t)((double)(s->Lo.rec_bytes) * frac) + (int64_t)mb_bytes;
    report->peak_act_bytes = c.ckpt_mode == BF_CKPT_NONE ? peak_live * rec_live
                                                         : peak_live * (int64_t)mb_bytes + chains * (int64_t)((double)s->Lo.rec_bytes * frac);
    // The fused weight gradient keeps, per layer of the stage and micro-batch, the gradients {dy, du, dx1, dqkv}
    // (with checkpointing also the recomputed operands {a, ctx, c, g}) until the stage's products have run.  The
    // last stage's set is complete while every stored activation of the step is still alive, so it adds to the peak.
    int64_t kept = 0;
    if (fuse) {
      kept = (int64_t)per_stage * N_mb * (int64_t)((double)s->Lo.grec_bytes * frac);
      if (c.ckpt_mode == BF_CKPT_LAYER) kept += (int64_t)per_stage * N_mb * (int64_t)((double)s->Lo.wrec_bytes * frac);
    }
    report->fused_wgrad_bytes = kept;
    report->peak_act_bytes += kept;
    report->state_bytes = (int64_t)s->Lo.P_total * (c.dtype == BF_BF16 && !c.dp_fs ? 18 : 16) +
                          (c.dp_fs ? 2 * (int64_t)s->Lo.half_bytes : 0);
    report->n_weight_intervals = (int64_t)ivs.size();
    report->n_reconstruct = n_recon;
    report->reconstruct_bytes = n_recon * 6 * (int64_t)per_stage * (int64_t)s->D.layer_elems;
    report->weight_buffer_bytes = c.dp_fs ? 2 * (int64_t)s->Lo.half_bytes : 0;
    report->n_events = (int32_t)s->trace.size();
    report->mb_chains = chains;
  }
  if (timing) {
    BF_HIP_CHECK(hipEventRecord(s->ev_t1, st));
    BF_HIP_CHECK(hipEventSynchronize(s->ev_t1));
    if (report) {
      float ms = 0.f;
      BF_HIP_CHECK(hipEventElapsedTime(&ms, s->ev_t0, s->ev_t1));
      report->gpu_ms = ms;
      double am = 0;
      for (size_t i = 0; i < n_adam; ++i) {
        BF_HIP_CHECK(hipEventSynchronize(s->adam_ev[2 * i + 1]));
        BF_HIP_CHECK(hipEventElapsedTime(&ms, s->adam_ev[2 * i], s->adam_ev[2 * i + 1]));
        am += ms;
      }
      report->adam_ms = am;
      report->timed = 1;
      if (s->prof_on) BF_HIP_CHECK(hipStreamSynchronize(s->side));
      for (size_t i = 0; i < s->prof_rec.size(); ++i) {
        BF_HIP_CHECK(hipEventElapsedTime(&ms, s->prof_ev[2 * i], s->prof_ev[2 * i + 1]));
        const int k = s->prof_rec[i].cls;
        report->kernel_ms[k] += ms;
        report->kernel_launches[k] += 1;
        report->kernel_flops[k] += s->prof_rec[i].flops;
        report->kernel_bytes[k] += s->prof_rec[i].bytes;
      }
    }
  }
  return BF_OK;
}

bf_status bf_run_step(bf_stack* s, int schedule, int N_loop, int N_mb, int S_mb, const void* x, const void* dy, void* y,
                      void* dx, int apply_optimizer, int timing, void* stream, bf_step_report* report) {
  return run_rank_step(s, schedule, 1, 0, true, N_loop, N_mb, S_mb, x, dy, y, dx, nullptr, apply_optimizer, timing, stream,
                       report);
}

bf_status bf_run_lm_step(bf_stack* s, int schedule, int N_loop, int N_mb, int S_mb, const int32_t* tokens,
                         const int32_t* labels, float* loss, int apply_optimizer, int timing, void* stream,
                         bf_step_report* report) {
  if (!s) { set_error("bf_run_lm_step: null stack"); return BF_EINVAL; }
  if (s->cfg.S_voc <= 0) { set_error("bf_run_lm_step: the stack was created without input / output layers (S_voc = 0)"); return BF_ESTATE; }
  if (!tokens || !labels || !loss) { set_error("bf_run_lm_step: tokens, labels and loss must not be null"); return BF_EINVAL; }
  const LmIO lm{tokens, labels, loss};
  return run_rank_step(s, schedule, 1, 0, true, N_loop, N_mb, S_mb, nullptr, nullptr, nullptr, nullptr, &lm, apply_optimizer,
                       timing, stream, report);
}

bf_status bf_run_rank_step(bf_stack* s, int schedule, int N_PP, int rank, int N_loop, int N_mb, int S_mb, const void* x,
                           const void* dy, void* y, void* dx, int apply_optimizer, int timing, void* stream,
                           bf_step_report* report) {
  if (N_PP < 1 || rank < 0 || rank >= N_PP) { set_error("bf_run_rank_step: rank %d outside 0..N_PP-1 (N_PP = %d)", rank, N_PP); return BF_EINVAL; }
  return run_rank_step(s, schedule, N_PP, rank, false, N_loop, N_mb, S_mb, x, dy, y, dx, nullptr, apply_optimizer, timing, stream,
                       report);
}

}  // extern "C"
