// Host-only schedule logic (no device code).
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/bf.h"

namespace bf {

struct SchedOp {
  int op;     // 0 forward, 1 backward
  int stage;  // global stage index l * N_PP + rank
  int mb;
};

// Ordered ops of one rank.  Returns false and fills *why on invalid arguments.
bool rank_order(int schedule, int N_PP, int N_loop, int N_mb, int rank, std::vector<SchedOp>* out, std::string* why);

// Unit-time simulation of all N_PP ranks; peak_live[r] = peak live stage inputs of rank r.
bool simulate(int schedule, int N_PP, int N_loop, int N_mb, int t_fwd, int t_bwd, bf_sched_stats* stats,
              std::vector<int64_t>* peak_live, std::string* why);

}  // namespace bf
