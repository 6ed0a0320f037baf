// Slot scheduler (host only, integers only).
//
// The 1F1B order with flush (Section 2) gives each stage a fixed sequence of
// forward and backward computations.  Each computation is preceded by its
// group's communication (Section 5.2: a group is leading communication followed
// by computation that needs no remote data).  Bubbles are not measured but
// simulated: all P stages are played on a zero-latency timeline and wherever
// this stage would wait for a neighbour a BUBBLE instruction is emitted.  FRC(k)
// goes on lane 1 right after FWD(k), i.e. before the stage starts talking to its
// successor, which is where the paper places it (Section 5.2 "Scheduling").
#include "schedule.h"

#include <algorithm>

namespace bamboo {

int warmup_depth(int P, int s, int M) { return std::min(P - 1 - s, M); }
int own_slot_count(int P, int s, int M) { return std::min(P - s, M); }

std::vector<Step> one_f_one_b(int P, int s, int M) {
  const int w = warmup_depth(P, s, M);
  std::vector<Step> seq;
  seq.reserve(2 * (size_t)M);
  int next_f = 0, next_b = 0;
  while (next_f < w) seq.push_back({false, next_f++});
  while (next_f < M) {
    seq.push_back({false, next_f++});
    seq.push_back({true, next_b++});
  }
  while (next_b < M) seq.push_back({true, next_b++});
  return seq;
}

std::vector<int> idle_before(int P, int s, int M, int tick_F, int tick_B, int* tail) {
  const std::vector<int> f(P, tick_F), b(P, tick_B);
  return idle_before(P, s, M, f.data(), b.data(), tail);
}

std::vector<int> idle_before(int P, int s, int M, const int* tick_F, const int* tick_B, int* tail) {
  // Play all P stages: a stage advances through its sequence whenever the same
  // micro-batch has finished on the neighbour it depends on (previous stage for
  // a forward, next stage for a backward).  fwd_end/bwd_end hold finishing times.
  std::vector<std::vector<Step>> seq(P);
  for (int st = 0; st < P; ++st) seq[st] = one_f_one_b(P, st, M);
  std::vector<std::vector<long>> fwd_end(P, std::vector<long>(M, -1)), bwd_end(P, std::vector<long>(M, -1));
  std::vector<size_t> cursor(P, 0);
  std::vector<long> clock(P, 0);
  std::vector<int> gaps(seq[s].size(), 0);
  for (bool moved = true; moved;) {
    moved = false;
    for (int st = 0; st < P; ++st) {
      while (cursor[st] < seq[st].size()) {
        const Step c = seq[st][cursor[st]];
        long ready = 0;
        if (!c.backward && st > 0) ready = fwd_end[st - 1][c.mb];
        if (c.backward && st < P - 1) ready = bwd_end[st + 1][c.mb];
        if (ready < 0) break;  // neighbour has not produced it yet
        const long t0 = std::max(clock[st], ready);
        if (st == s) gaps[cursor[st]] = (int)(t0 - clock[st]);
        clock[st] = t0 + (c.backward ? tick_B[st] : tick_F[st]);
        (c.backward ? bwd_end : fwd_end)[st][c.mb] = clock[st];
        ++cursor[st];
        moved = true;
      }
    }
  }
  *tail = (int)(*std::max_element(clock.begin(), clock.end()) - clock[s]);
  return gaps;
}

namespace {
bamboo_instr_t ins(int op, int lane, int mb, int arg) {
  bamboo_instr_t i;
  i.op = (uint8_t)op;
  i.lane = (uint8_t)lane;
  i.mb = (int16_t)mb;
  i.arg = arg;
  return i;
}

// what the previous computation produced is sent first, then what the next one
// needs is received
void group_head(std::vector<bamboo_instr_t>& out, const Step* prev, const Step* next, int P, int s) {
  if (prev) {
    if (!prev->backward && s < P - 1) out.push_back(ins(BAMBOO_SEND_ACT, 0, prev->mb, s + 1));
    if (prev->backward && s > 0) out.push_back(ins(BAMBOO_SEND_GRAD, 0, prev->mb, s - 1));
  }
  if (next) {
    if (!next->backward && s > 0) out.push_back(ins(BAMBOO_RECV_ACT, 0, next->mb, s - 1));
    if (next->backward && s < P - 1) out.push_back(ins(BAMBOO_RECV_GRAD, 0, next->mb, s + 1));
  }
}

void epilogue(std::vector<bamboo_instr_t>& out) {
  out.push_back(ins(BAMBOO_JOIN, 0, -1, -1));
  out.push_back(ins(BAMBOO_ALLREDUCE, 0, -1, 0));
  out.push_back(ins(BAMBOO_APPLY, 0, -1, 0));
}
}  // namespace

std::vector<bamboo_instr_t> build_program(const bamboo_cfg_t& c) { return build_program(c, nullptr, nullptr); }

std::vector<bamboo_instr_t> build_program(const bamboo_cfg_t& c, const int* tick_F, const int* tick_B) {
  const int P = c.P, s = c.stage_id, M = c.M;
  const std::vector<Step> seq = one_f_one_b(P, s, M);
  const int slots = own_slot_count(P, s, M);
  int tail = 0;
  const std::vector<int> uf(P, c.tick_F), ub(P, c.tick_B);
  const std::vector<int> gaps = idle_before(P, s, M, tick_F ? tick_F : uf.data(), tick_B ? tick_B : ub.data(), &tail);
  const bool frc = c.rc_mode != BAMBOO_RC_LFLB && c.n_shadow > 0;
  const bool eager_brc = c.rc_mode == BAMBOO_RC_EFEB && c.n_shadow > 0 && s < P - 1;
  std::vector<bamboo_instr_t> out;
  for (size_t j = 0; j < seq.size(); ++j) {
    if (eager_brc && seq[j].backward) {
      // eager BRC (Section 7.4): issued on lane 1 where the stage starts to wait for the successor's
      // backward of this micro-batch; its upstream gradient comes from the stage after the successor
      if (s + 2 < P) out.push_back(ins(BAMBOO_RECV_GRAD, 1, seq[j].mb, s + 2));
      out.push_back(ins(BAMBOO_BRC, 1, seq[j].mb, seq[j].mb));
    }
    if (gaps[j] > 0) out.push_back(ins(BAMBOO_BUBBLE, 0, -1, gaps[j]));
    group_head(out, j ? &seq[j - 1] : nullptr, &seq[j], P, s);
    const int k = seq[j].mb;
    if (seq[j].backward) {
      out.push_back(ins(BAMBOO_BWD, 0, k, k % slots));
    } else {
      out.push_back(ins(BAMBOO_FWD, 0, k, k % slots));
      if (frc) out.push_back(ins(BAMBOO_FRC, 1, k, k));
    }
  }
  group_head(out, seq.empty() ? nullptr : &seq.back(), nullptr, P, s);
  if (tail > 0) out.push_back(ins(BAMBOO_BUBBLE, 0, -1, tail));
  epilogue(out);
  return out;
}

// Failover schedule (Section 5.2 "Lazy BRC and Recovery").  The failure shows
// when the send of micro-batch k_fail's activation to the successor breaks.
//  1. JOIN the FRC lane up to FRC(k_fail): its stash is about to be consumed.
//  2. The successor's weight gradients of the micro-batches it had already
//     back-propagated are gone; BRC recomputes them, in micro-batch order, from
//     the upstream gradients the stage after the victim delivers again.
//  3. The remaining 1F1B computations of this stage, each merged with the
//     victim's computation of the same micro-batch.  Merge rules: communication
//     leads the group (1); victim<->shadow traffic disappears (2); the victim's
//     external traffic comes before the shadow's (3); backward work (BRC then
//     BWD) comes before forward work (FWD then FRC), so a backward that follows
//     a forward in 1F1B order opens a new group (4).
std::vector<bamboo_instr_t> build_failover_program(const bamboo_cfg_t& c, int k_fail) {
  const int P = c.P, s = c.stage_id, M = c.M;
  const std::vector<Step> seq = one_f_one_b(P, s, M);
  const int slots = own_slot_count(P, s, M);
  const bool far = s + 2 < P;  // the victim had a successor of its own
  size_t at = 0;
  int lost = 0;
  while (at < seq.size() && !(!seq[at].backward && seq[at].mb == k_fail)) lost += seq[at++].backward ? 1 : 0;
  std::vector<bamboo_instr_t> out;
  out.push_back(ins(BAMBOO_JOIN, 0, -1, k_fail));
  // Variants (Section 7.4): with eager BRC the lost gradients were never only the victim's, so
  // nothing is replayed; with lazy FRC nothing redundant exists yet, so FRC runs before every BRC
  // and the micro-batches the victim had forwarded but not back-propagated are forwarded again.
  if (c.rc_mode != BAMBOO_RC_EFEB)
    for (int k = 0; k < lost; ++k) {
      if (far) out.push_back(ins(BAMBOO_RECV_GRAD, 0, k, s + 2));
      if (c.rc_mode == BAMBOO_RC_LFLB) out.push_back(ins(BAMBOO_FRC, 0, k, k));
      out.push_back(ins(BAMBOO_BRC, 0, k, k));
    }
  if (c.rc_mode == BAMBOO_RC_LFLB)
    for (int k = lost; k <= k_fail; ++k) out.push_back(ins(BAMBOO_FRC, 0, k, k));
  std::vector<int> z_pending{k_fail};  // FRC outputs the far stage still has to get
  std::vector<int> gx_pending;          // input gradients not yet sent back
  size_t j = at + 1;
  bool done = false;
  while (!done) {
    // members of the next group: [backward] [forward] or a lone forward
    const Step* gb = nullptr;
    const Step* gf = nullptr;
    if (j < seq.size() && seq[j].backward) gb = &seq[j++];
    if (j < seq.size() && !seq[j].backward) gf = &seq[j++];
    done = !gb && !gf;
    if (far)
      for (int k : z_pending) out.push_back(ins(BAMBOO_SEND_ACT, 0, k, s + 2));
    z_pending.clear();
    if (gb && far) out.push_back(ins(BAMBOO_RECV_GRAD, 0, gb->mb, s + 2));
    if (s > 0)
      for (int k : gx_pending) out.push_back(ins(BAMBOO_SEND_GRAD, 0, k, s - 1));
    gx_pending.clear();
    if (gf && s > 0) out.push_back(ins(BAMBOO_RECV_ACT, 0, gf->mb, s - 1));
    if (gb) {
      out.push_back(ins(BAMBOO_BRC, 0, gb->mb, gb->mb));
      out.push_back(ins(BAMBOO_BWD, 0, gb->mb, gb->mb % slots));
      gx_pending.push_back(gb->mb);
    }
    if (gf) {
      out.push_back(ins(BAMBOO_FWD, 0, gf->mb, gf->mb % slots));
      out.push_back(ins(BAMBOO_FRC, 0, gf->mb, gf->mb));
      z_pending.push_back(gf->mb);
    }
  }
  epilogue(out);
  return out;
}

}  // namespace bamboo
