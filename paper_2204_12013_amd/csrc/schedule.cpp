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

namespace {
// Start and finishing time of every computation of every stage on the zero-latency timeline:
// t[stage][0 forward / 1 backward][micro-batch].
struct Timeline {
  std::vector<std::vector<long>> start[2], end[2];
  std::vector<long> clock;   // finishing time of each stage's last computation
};

// Play all P stages: a stage advances through its sequence whenever the same
// micro-batch has finished on the neighbour it depends on (previous stage for
// a forward, next stage for a backward).
Timeline play(int P, int M, const int* tick_F, const int* tick_B) {
  Timeline t;
  for (int d = 0; d < 2; ++d) {
    t.start[d].assign(P, std::vector<long>(M, -1));
    t.end[d].assign(P, std::vector<long>(M, -1));
  }
  t.clock.assign(P, 0);
  std::vector<std::vector<Step>> seq(P);
  for (int st = 0; st < P; ++st) seq[st] = one_f_one_b(P, st, M);
  std::vector<size_t> cursor(P, 0);
  for (bool moved = true; moved;) {
    moved = false;
    for (int st = 0; st < P; ++st) {
      while (cursor[st] < seq[st].size()) {
        const Step c = seq[st][cursor[st]];
        long ready = 0;
        if (!c.backward && st > 0) ready = t.end[0][st - 1][c.mb];
        if (c.backward && st < P - 1) ready = t.end[1][st + 1][c.mb];
        if (ready < 0) break;  // neighbour has not produced it yet
        const long t0 = std::max(t.clock[st], ready);
        t.start[c.backward][st][c.mb] = t0;
        t.clock[st] = t0 + (c.backward ? tick_B[st] : tick_F[st]);
        t.end[c.backward][st][c.mb] = t.clock[st];
        ++cursor[st];
        moved = true;
      }
    }
  }
  return t;
}
}  // namespace

std::vector<int> idle_before(int P, int s, int M, const int* tick_F, const int* tick_B, int* tail) {
  const Timeline t = play(P, M, tick_F, tick_B);
  const std::vector<Step> seq = one_f_one_b(P, s, M);
  std::vector<int> gaps(seq.size(), 0);
  long clock = 0;
  for (size_t j = 0; j < seq.size(); ++j) {
    gaps[j] = (int)(t.start[seq[j].backward][s][seq[j].mb] - clock);
    clock = t.end[seq[j].backward][s][seq[j].mb];
  }
  *tail = (int)(*std::max_element(t.clock.begin(), t.clock.end()) - t.clock[s]);
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

namespace {
// Merge rules (1)-(4) over the computations seq[from..]: members of a group are [backward] [forward]
// or a lone forward.  first_unsent: micro-batch whose FRC output the stage after the victim still
// has to get when the list starts (-1: none).
void merge_rest(std::vector<bamboo_instr_t>& out, const std::vector<Step>& seq, size_t from, int slots, int s,
                bool far, int first_unsent) {
  std::vector<int> z_pending;   // FRC outputs the far stage still has to get
  if (first_unsent >= 0) z_pending.push_back(first_unsent);
  std::vector<int> gx_pending;  // input gradients not yet sent back
  size_t j = from;
  bool done = false;
  while (!done) {
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
}
}  // namespace

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
  merge_rest(out, seq, at + 1, slots, s, far, k_fail);
  epilogue(out);
  return out;
}

// The merged stage's whole iteration: rule-(1)-(4) groups from the first computation on, nothing to
// join and nothing to replay (Section 5.2: until the pipeline is reconfigured the shadow node
// executes all of the victim's instructions).  With P == 1 the two merged nodes are data-parallel
// peers and there is no communication.
std::vector<bamboo_instr_t> build_merged_program(const bamboo_cfg_t& c) {
  const int P = c.P, s = c.stage_id, M = c.M;
  std::vector<bamboo_instr_t> out;
  merge_rest(out, one_f_one_b(P, s, M), 0, own_slot_count(P, s, M), s, s + 2 < P, -1);
  epilogue(out);
  return out;
}

// Wrap-around (Section 5.1): the last stage holds the replica of the first stage, which is lost.
// The last stage notices after FWD(k_fail) and its FRC.  Where the victim stood at that moment
// comes from the zero-latency timeline: it had finished n_fwd forwards and n_bwd backwards.
void wrap_victim_progress(const bamboo_cfg_t& c, int k_fail, int* n_fwd, int* n_bwd) {
  const int P = c.P, M = c.M;
  const std::vector<int> tf(P, c.tick_F), tb(P, c.tick_B);
  const Timeline t = play(P, M, tf.data(), tb.data());
  const long t_star = t.end[0][P - 1][k_fail];
  *n_fwd = *n_bwd = 0;
  for (int k = 0; k < M; ++k) {
    *n_fwd += t.end[0][0][k] <= t_star;
    *n_bwd += t.end[1][0][k] <= t_star;
  }
}

// The merged node is both ends of the pipeline, so no traffic turns internal unless P = 2.
// After the replay of the victim's finished backwards, what is left of the two stages' 1F1B
// sequences is merged by start time on the failure-free timeline (anything a computation needs
// started earlier there); on equal times backward work goes first, then the victim's.  Each
// sequence is already in time order, so this is a two-way merge.
// k_fail < 0: the whole iteration of the merged node (nothing to join, nothing to replay)
static std::vector<bamboo_instr_t> wrap_merge(const bamboo_cfg_t& c, int k_fail) {
  const int P = c.P, s = P - 1, M = c.M;
  const int slots = own_slot_count(P, s, M);
  const bool far = P > 2;
  const std::vector<int> tf(P, c.tick_F), tb(P, c.tick_B);
  const Timeline t = play(P, M, tf.data(), tb.data());
  int n_fwd = 0, n_bwd = 0;
  std::vector<bamboo_instr_t> out;
  std::vector<Step> own = one_f_one_b(P, s, M), vic;
  size_t io = 0;
  if (k_fail >= 0) {
    wrap_victim_progress(c, k_fail, &n_fwd, &n_bwd);
    out.push_back(ins(BAMBOO_JOIN, 0, -1, k_fail));
    // lazy FRC (Section 7.4): nothing redundant has run yet, so FRC precedes every replayed BRC, and the
    // victim's forwards that were done but not yet back-propagated are run again for their intermediates
    const bool lazy = c.rc_mode == BAMBOO_RC_LFLB;
    for (int k = 0; k < n_bwd; ++k) {
      if (far) out.push_back(ins(BAMBOO_RECV_GRAD, 0, k, 1));
      if (lazy) out.push_back(ins(BAMBOO_FRC, 0, k, k));
      out.push_back(ins(BAMBOO_BRC, 0, k, k));
    }
    if (lazy)
      for (int k = n_bwd; k <= k_fail; ++k) out.push_back(ins(BAMBOO_FRC, 0, k, k));
    // what is left: own sequence behind FWD(k_fail); victim forwards beyond k_fail, victim backwards from n_bwd
    while (!(!own[io].backward && own[io].mb == k_fail)) ++io;
    ++io;
  }
  for (const Step& v : one_f_one_b(P, 0, M))
    if (v.backward ? v.mb >= n_bwd : v.mb > k_fail) vic.push_back(v);
  size_t iv = 0;
  auto key = [&](const Step& st, int stage) { return t.start[st.backward][stage][st.mb]; };
  std::vector<bamboo_instr_t> owed;   // sends of the computation emitted last
  while (io < own.size() || iv < vic.size()) {
    bool take_victim;
    if (io >= own.size()) take_victim = true;
    else if (iv >= vic.size()) take_victim = false;
    else {
      const long tv = key(vic[iv], 0), to = key(own[io], s);
      if (tv != to) take_victim = tv < to;
      else if (vic[iv].backward != own[io].backward) take_victim = vic[iv].backward;
      else take_victim = true;
    }
    out.insert(out.end(), owed.begin(), owed.end());
    owed.clear();
    if (take_victim) {
      const Step v = vic[iv++];
      if (v.backward) {
        if (far) out.push_back(ins(BAMBOO_RECV_GRAD, 0, v.mb, 1));
        out.push_back(ins(BAMBOO_BRC, 0, v.mb, v.mb));
      } else {
        out.push_back(ins(BAMBOO_FRC, 0, v.mb, v.mb));
        if (far && v.mb >= n_fwd) owed.push_back(ins(BAMBOO_SEND_ACT, 0, v.mb, 1));
      }
    } else {
      const Step o = own[io++];
      if (o.backward) {
        out.push_back(ins(BAMBOO_BWD, 0, o.mb, o.mb % slots));
        if (far) owed.push_back(ins(BAMBOO_SEND_GRAD, 0, o.mb, s - 1));
      } else {
        if (far) out.push_back(ins(BAMBOO_RECV_ACT, 0, o.mb, s - 1));
        out.push_back(ins(BAMBOO_FWD, 0, o.mb, o.mb % slots));
      }
    }
  }
  out.insert(out.end(), owed.begin(), owed.end());
  epilogue(out);
  return out;
}

std::vector<bamboo_instr_t> build_wrap_failover_program(const bamboo_cfg_t& c, int k_fail) { return wrap_merge(c, k_fail); }
std::vector<bamboo_instr_t> build_wrap_merged_program(const bamboo_cfg_t& c) { return wrap_merge(c, -1); }

}  // namespace bamboo
