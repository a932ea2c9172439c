// Host-sanitizer driver for the planner (no HIP): reads problems from stdin, one per line
//   B H S W hint q_len cus L_0 .. L_{B-1}
// plans each, re-plans it with every length grown by one, and checks the partition the
// way the Python tests do in spirit (segments tile [0, ntiles) per sequence without gaps,
// slots dense), so that every vector the planner fills is walked under ASan / UBSan.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_2511_22481_amd/csrc/plan.h"

using namespace omniattn;

static int check(const HostPlan& hp) {
  std::vector<int> next((size_t)hp.prob.batch * hp.n_hb, 0);
  std::vector<char> slot_seen((size_t)hp.n_slots, 0);
  for (const Segment& s : hp.segs) {
    if (s.b < 0 || s.b >= hp.prob.batch || s.hb < 0 || s.hb >= hp.n_hb) return 1;
    int& pos = next[(size_t)s.b * hp.n_hb + s.hb];
    if (s.tile_lo != pos || s.tile_hi < s.tile_lo) return 2;
    pos = s.tile_hi;
    if (s.slot >= 0) {
      if (s.slot >= hp.n_slots || slot_seen[s.slot]) return 3;
      slot_seen[s.slot] = 1;
    }
    if (s.unit < 0 || s.unit + 1 >= (int)hp.unit_seg.size()) return 4;
  }
  for (int b = 0; b < hp.prob.batch; ++b)
    for (int hb = 0; hb < hp.n_hb; ++hb)
      if (next[(size_t)b * hp.n_hb + hb] != tile_layout(hp.seq_lens[b], hp.prob.sink, hp.window_union, hp.tile).count()) return 5;
  for (char c : slot_seen)
    if (!c) return 6;
  for (const CombineItem& it : hp.combine)
    if (it.slot0 < 0 || it.nslots < 2 || it.slot0 + it.nslots > hp.n_slots) return 7;
  return 0;
}

int main() {
  int B, H, S, W, hint, q_len, cus, n_ok = 0;
  while (std::scanf("%d %d %d %d %d %d %d", &B, &H, &S, &W, &hint, &q_len, &cus) == 7) {
    std::vector<int32_t> lens((size_t)B);
    int max_pages = 1;
    for (int b = 0; b < B; ++b) {
      if (std::scanf("%d", &lens[b]) != 1) return 90;
      max_pages = std::max(max_pages, (lens[b] + 1 + kPage - 1) / kPage);
    }
    omniattn_problem_t prob{};
    prob.batch = B;
    prob.num_heads = H;
    prob.qk_dim = kQK;
    prob.v_dim = kV;
    prob.page_size = kPage;
    prob.max_pages_per_seq = max_pages;
    prob.num_pages = (int64_t)B * max_pages;
    prob.sink = S;
    prob.window = W;
    prob.softmax_scale = 0.1f;
    prob.num_splits_hint = hint;
    prob.q_len = q_len;
    for (int round = 0; round < 2; ++round) {
      HostPlan hp;
      const int rc = build_host_plan(hp, prob, lens.data(), cus);
      if (rc != OMNIATTN_OK) {
        std::printf("plan rejected rc=%d\n", rc);
        return 91;
      }
      const int bad = check(hp);
      if (bad) {
        std::printf("partition check %d failed\n", bad);
        return 92;
      }
      for (int32_t& L : lens) L += 1;  // the next decode step
    }
    ++n_ok;
  }
  std::printf("ok %d\n", n_ok);
  return 0;
}
