// Host-side slot scheduler of one Bamboo stage: 1F1B program with simulated
// bubbles and eager FRC, and the failover schedule (paper Sections 2, 4, 5.2).
#pragma once
#include <vector>

#include "../../include/bamboo_stage.h"

namespace bamboo {

struct Step {       // one computation of the 1F1B order
  bool backward;
  int mb;
};

int warmup_depth(int P, int s, int M);            // forwards before the first backward, minus one
int own_slot_count(int P, int s, int M);          // peak in-flight micro-batches of stage s
std::vector<Step> one_f_one_b(int P, int s, int M);

// Idle ticks of stage s before each of its computations and after the last one,
// from a zero-latency simulation of all P stages.
std::vector<int> idle_before(int P, int s, int M, int tick_F, int tick_B, int* tail);
// the same with a forward / backward duration per stage (P entries each): uneven partitions
std::vector<int> idle_before(int P, int s, int M, const int* tick_F, const int* tick_B, int* tail);

std::vector<bamboo_instr_t> build_program(const bamboo_cfg_t& c);
// per-stage durations; null arrays fall back to c.tick_F / c.tick_B for every stage
std::vector<bamboo_instr_t> build_program(const bamboo_cfg_t& c, const int* tick_F, const int* tick_B);
std::vector<bamboo_instr_t> build_failover_program(const bamboo_cfg_t& c, int k_fail);
// a whole iteration of the stage after it has taken over the victim's layers (adjacent stages, or the
// two nodes of pure data parallelism when P == 1)
std::vector<bamboo_instr_t> build_merged_program(const bamboo_cfg_t& c);
// wrap-around: the last stage takes over the lost first stage (cfg.wrap)
std::vector<bamboo_instr_t> build_wrap_failover_program(const bamboo_cfg_t& c, int k_fail);
std::vector<bamboo_instr_t> build_wrap_merged_program(const bamboo_cfg_t& c);
void wrap_victim_progress(const bamboo_cfg_t& c, int k_fail, int* n_fwd, int* n_bwd);

}  // namespace bamboo
