// Host-only integer logic: the op order of a rank in a looped pipeline and a unit-time
// simulation of all ranks (Sec. 4.1; Eq. bubble, Eq. bubble_looped; App. C for N_PP = 1).
#include "schedule.h"

#include <algorithm>
#include <map>
#include <numeric>
#include <tuple>

namespace bf {

bool rank_order(int schedule, int N_PP, int N_loop, int N_mb, int rank, std::vector<SchedOp>* out, std::string* why) {
  out->clear();
  if (N_PP < 1 || N_loop < 1 || N_mb < 1 || rank < 0 || rank >= N_PP) {
    *why = "schedule: N_PP, N_loop, N_mb must be >= 1 and 0 <= rank < N_PP";
    return false;
  }
  if (schedule == BF_SCHED_BF) {
    if (N_mb < N_PP) {
      *why = "breadth-first schedule needs N_mb >= N_PP";
      return false;
    }
    // earlier stages first, every micro-batch through a stage before the next stage
    for (int l = 0; l < N_loop; ++l)
      for (int m = 0; m < N_mb; ++m) out->push_back({0, l * N_PP + rank, m});
    for (int l = N_loop - 1; l >= 0; --l)
      for (int m = 0; m < N_mb; ++m) out->push_back({1, l * N_PP + rank, m});
    return true;
  }
  if (schedule != BF_SCHED_DF) {
    *why = "schedule must be BF_SCHED_BF or BF_SCHED_DF";
    return false;
  }
  if (N_mb % N_PP) {
    *why = "depth-first schedule needs N_mb to be a multiple of N_PP";
    return false;
  }
  if (N_PP == 1) {
    // one device: a micro-batch finishes forward and backward before the next starts
    for (int m = 0; m < N_mb; ++m) {
      for (int l = 0; l < N_loop; ++l) out->push_back({0, l, m});
      for (int l = N_loop - 1; l >= 0; --l) out->push_back({1, l, m});
    }
    return true;
  }
  // Micro-batches travel in sequences of N_PP; inside a sequence the rank visits its
  // loops in order (reverse order for the backward).  Warm-up forwards, then one
  // forward / one backward alternately, then the remaining backwards.
  const int total = N_loop * N_mb, seq = N_PP * N_loop;
  auto slot = [&](int i, bool backward) {
    const int g = i / seq, r = i % seq;
    int l = r / N_PP;
    const int j = r % N_PP;
    if (backward) l = N_loop - 1 - l;
    return SchedOp{backward ? 1 : 0, l * N_PP + rank, g * N_PP + j};
  };
  int warm = N_loop == 1 ? N_PP - rank - 1 : 2 * (N_PP - rank - 1) + (N_loop - 1) * N_PP;
  warm = std::min(warm, total);
  int fi = 0, bi = 0;
  for (; fi < warm; ++fi) out->push_back(slot(fi, false));
  while (fi < total) {
    out->push_back(slot(fi++, false));
    out->push_back(slot(bi++, true));
  }
  while (bi < total) out->push_back(slot(bi++, true));
  return true;
}

bool simulate(int schedule, int N_PP, int N_loop, int N_mb, int t_fwd, int t_bwd, bf_sched_stats* stats,
              std::vector<int64_t>* peak_live, std::string* why) {
  if (t_fwd < 1 || t_bwd < 1) {
    *why = "schedule: t_fwd and t_bwd must be >= 1";
    return false;
  }
  std::vector<std::vector<SchedOp>> orders(N_PP);
  for (int r = 0; r < N_PP; ++r)
    if (!rank_order(schedule, N_PP, N_loop, N_mb, r, &orders[r], why)) return false;
  const int N_stage = N_PP * N_loop;
  std::vector<size_t> ptr(N_PP, 0);
  std::vector<int64_t> free_at(N_PP, 0);
  std::map<std::tuple<int, int, int>, int64_t> done;
  size_t remaining = 0;
  for (auto& o : orders) remaining += o.size();
  peak_live->assign(N_PP, 0);
  std::vector<int64_t> live(N_PP, 0);
  while (remaining) {
    bool progressed = false;
    for (int r = 0; r < N_PP; ++r) {
      while (ptr[r] < orders[r].size()) {
        const SchedOp& op = orders[r][ptr[r]];
        int64_t ready = 0;
        bool has_dep = true;
        std::tuple<int, int, int> dep;
        if (op.op == 0) {
          if (op.stage == 0) has_dep = false;
          else dep = std::make_tuple(0, op.stage - 1, op.mb);
        } else {
          dep = op.stage == N_stage - 1 ? std::make_tuple(0, op.stage, op.mb) : std::make_tuple(1, op.stage + 1, op.mb);
        }
        if (has_dep) {
          auto it = done.find(dep);
          if (it == done.end()) break;
          ready = it->second;
        }
        const int64_t start = std::max(free_at[r], ready);
        free_at[r] = start + (op.op == 0 ? t_fwd : t_bwd);
        done[std::make_tuple(op.op, op.stage, op.mb)] = free_at[r];
        if (op.op == 0) {
          ++live[r];
          (*peak_live)[r] = std::max((*peak_live)[r], live[r]);
        } else {
          --live[r];
        }
        ++ptr[r];
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) {
      *why = "schedule deadlocks";
      return false;
    }
  }
  const int64_t makespan = *std::max_element(free_at.begin(), free_at.end());
  const int64_t busy = (int64_t)N_loop * N_mb * (t_fwd + t_bwd);
  const int64_t idle = makespan - busy;
  const int64_t g = std::gcd(idle, busy);
  stats->makespan = makespan;
  stats->busy = busy;
  stats->bubble_num = idle / (g ? g : 1);
  stats->bubble_den = busy / (g ? g : 1);
  return true;
}

}  // namespace bf
