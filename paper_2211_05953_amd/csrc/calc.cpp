// The paper's analytical efficiency model (Sec. 3, Sec. 4.2, Table 4.1, Sec. 3.5) as host functions.
#include "../../include/bf_calc.h"

namespace bf { void set_error(const char* fmt, ...); }

namespace {

bool valid(const bf_calc_config& c) {
  using bf::set_error;
  if (c.method < BF_METHOD_NO_PIPELINE || c.method > BF_METHOD_BREADTH_FIRST) { set_error("calc: unknown method %d", c.method); return false; }
  if (c.N_PP < 1 || c.N_loop < 1 || c.N_TP < 1 || c.N_mb < 1 || c.S_mb < 1 || c.N_layers < 0) { set_error("calc: sizes must be >= 1"); return false; }
  if (!(c.beta_net >= 0.0)) { set_error("calc: beta_net < 0"); return false; }
  if (c.method == BF_METHOD_NO_PIPELINE && (c.N_PP != 1 || c.N_loop != 1)) { set_error("calc: no pipeline means N_PP = N_loop = 1"); return false; }
  if (c.method == BF_METHOD_NON_LOOPED && c.N_loop != 1) { set_error("calc: a non-looped pipeline has N_loop = 1"); return false; }
  if (c.N_mb < c.N_PP) { set_error("calc: N_mb = %d < N_PP = %d", c.N_mb, c.N_PP); return false; }
  if (c.method == BF_METHOD_DEPTH_FIRST && c.N_mb % c.N_PP) { set_error("calc: depth-first needs N_mb %% N_PP == 0"); return false; }
  if (c.N_layers > 0 && c.N_layers % (c.N_PP * c.N_loop)) { set_error("calc: N_layers must be a multiple of N_PP N_loop"); return false; }
  return true;
}

// micro-batches whose backward a gradient reduction can run beside (Sec. 4.2): one without looping,
// a sequence of N_PP depth-first, the whole batch breadth-first
double overlapped_mbs(const bf_calc_config& c) {
  switch (c.method) {
    case BF_METHOD_DEPTH_FIRST: return c.N_PP;
    case BF_METHOD_BREADTH_FIRST: return c.N_mb;
    default: return 1.0;
  }
}

void eval(const bf_calc_config& c, bf_calc_point* p) {
  const double samples = (double)c.N_mb * c.S_mb;
  p->beta = samples / ((double)c.N_PP * c.N_TP);
  p->bubble = (double)(c.N_PP - 1) / ((double)c.N_mb * c.N_loop);
  // Table 4.1, "DP network": 2 units (reduce + reconstruct) per 1 / N_PP of the model, 3 when fully
  // sharded, times the repetitions; relative to plain data parallelism that is vol / 2.
  const double reps = c.sharded ? (double)c.N_mb / overlapped_mbs(c) : 1.0;
  const double vol = (c.sharded ? 1.5 : 1.0) * reps;
  p->net_ratio = vol * c.beta_net / samples;
  // Table 4.1, "DP overlap".  A repeated operation overlaps with its own micro-batches each time, so
  // the repetitions together can hide under the whole backward pass.
  const double tail = c.N_layers > 0 ? 1.0 - (double)c.N_PP / c.N_layers : 1.0;
  const double share = c.sharded ? 1.0 : overlapped_mbs(c) / c.N_mb;
  p->overlap_share = c.overlap ? tail * share : 0.0;
  const double over = p->net_ratio - p->overlap_share;
  p->net_overhead = over > 0.0 ? over : 0.0;
  p->efficiency = 1.0 / (1.0 + p->bubble + p->net_overhead);
}

}  // namespace

extern "C" {

bf_status bf_calc_efficiency(const bf_calc_config* cfg, bf_calc_point* out) {
  if (!cfg || !out) { bf::set_error("bf_calc_efficiency: null argument"); return BF_EINVAL; }
  if (!valid(*cfg)) return BF_EINVAL;
  eval(*cfg, out);
  return BF_OK;
}

bf_status bf_calc_efficiency_curve(const bf_calc_config* cfg, const int32_t* n_mb, size_t n, bf_calc_point* out) {
  if (!cfg || (n && (!n_mb || !out))) { bf::set_error("bf_calc_efficiency_curve: null argument"); return BF_EINVAL; }
  bf_calc_config probe = *cfg;
  probe.N_mb = cfg->N_PP > 0 ? cfg->N_PP : 1;  // the smallest count every method allows
  if (!valid(probe)) return BF_EINVAL;
  for (size_t i = 0; i < n; ++i) {
    bf_calc_config c = *cfg;
    c.N_mb = n_mb[i];
    if (valid(c)) {
      eval(c, &out[i]);
    } else {
      out[i] = bf_calc_point{0, 0, 0, 0, 0, -1.0};
    }
  }
  return BF_OK;
}

bf_status bf_calc_beta_threshold(const bf_calc_config* cfg, double* beta_out) {
  if (!cfg || !beta_out) { bf::set_error("bf_calc_beta_threshold: null argument"); return BF_EINVAL; }
  if (!valid(*cfg)) return BF_EINVAL;
  const bf_calc_config& c = *cfg;
  const double tail = c.N_layers > 0 ? 1.0 - (double)c.N_PP / c.N_layers : 1.0;
  if (!(tail > 0.0)) { bf::set_error("calc: one layer per pipeline rank leaves nothing to overlap with"); return BF_EINVAL; }
  // net_ratio <= overlap_share solved for the samples per data-parallel rank N_mb S_mb, then divided by N_PP N_TP
  const double factor = c.sharded ? 1.5 : 1.0;
  const double samples = factor * c.beta_net * c.N_mb / (overlapped_mbs(c) * tail);
  *beta_out = samples / ((double)c.N_PP * c.N_TP);
  return BF_OK;
}

bf_status bf_calc_cost_time(double beta, double N_gpu, double B_crit, double efficiency, double* cost, double* time) {
  if (!cost || !time) { bf::set_error("bf_calc_cost_time: null argument"); return BF_EINVAL; }
  if (!(beta > 0.0) || !(N_gpu > 0.0) || !(B_crit > 0.0) || !(efficiency > 0.0) || efficiency > 1.0) {
    bf::set_error("bf_calc_cost_time: beta, N_gpu, B_crit must be > 0 and efficiency in (0, 1]");
    return BF_EINVAL;
  }
  *cost = (1.0 + beta * N_gpu / B_crit) / efficiency;
  *time = *cost / N_gpu;
  return BF_OK;
}

}  // extern "C"
