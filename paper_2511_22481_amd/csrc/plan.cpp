// Work partition for sparse MLA decode (host only, no HIP calls).
#include "plan.h"

#include <algorithm>
#include <climits>
#include <cstring>

namespace omniattn {

namespace {

struct Item {
  int b, hb, ntiles;
};

// A segment carries a fixed cost (loading the query block, writing a result)
// worth about this many KV tiles.
constexpr int kSegFixedCost = 1;
// Do not leave slivers shorter than this many tiles unless the item itself is shorter.
constexpr int kMinSegTiles = 2;

// Greedy fill of units of capacity `cap`; returns the number of units used.
int fill_units(const std::vector<Item>& items, int cap, std::vector<Segment>* segs_out,
               std::vector<int32_t>* unit_seg_out) {
  std::vector<Segment> segs;
  std::vector<int32_t> unit_seg;
  unit_seg.push_back(0);
  int load = 0;
  auto close_unit = [&]() {
    if ((int)segs.size() > unit_seg.back()) {
      unit_seg.push_back((int32_t)segs.size());
      load = 0;
    }
  };
  for (const Item& it : items) {
    int done = 0;
    if (it.ntiles == 0) {  // empty retained set: one segment that only writes zeros / -inf
      if (load + kSegFixedCost > cap) close_unit();
      segs.push_back({it.b, it.hb, 0, 0, -1, (int32_t)unit_seg.size() - 1, 0, 0});
      load += kSegFixedCost;
      continue;
    }
    while (done < it.ntiles) {
      int rem = it.ntiles - done;
      int room = cap - load - kSegFixedCost;
      int need = std::min(rem, kMinSegTiles);
      if (room < need) {
        if (load == 0) room = need;  // capacity smaller than one minimal segment
        else { close_unit(); continue; }
      }
      int take = std::min(std::min(rem, room), kMaxSegTiles);
      // avoid leaving a sliver behind
      if (rem - take > 0 && rem - take < kMinSegTiles) take = std::max(1, rem - kMinSegTiles);
      segs.push_back({it.b, it.hb, done, done + take, -1, (int32_t)unit_seg.size() - 1, 0,
                      it.ntiles});
      done += take;
      load += take + kSegFixedCost;
      if (load >= cap) close_unit();
    }
  }
  close_unit();
  int n_units = (int)unit_seg.size() - 1;
  if (segs_out) {
    *segs_out = std::move(segs);
    *unit_seg_out = std::move(unit_seg);
  }
  return n_units;
}

}  // namespace

int build_host_plan(HostPlan& hp, const omniattn_problem_t& prob, const int32_t* seq_lens,
                    int num_cus) {
  if (!seq_lens) return OMNIATTN_EINVAL;
  if (prob.batch < 1 || prob.num_heads < 1 || prob.sink < 0 || prob.window < 0 ||
      prob.max_pages_per_seq < 1 || prob.num_pages < 1 || prob.num_splits_hint < 0 || num_cus < 1)
    return OMNIATTN_EINVAL;
  if (prob.qk_dim != kQK || prob.v_dim != kV || prob.page_size != kPage) return OMNIATTN_EUNSUPPORTED;
  if (prob.kv_dtype != OMNIATTN_BF16 && prob.kv_dtype != OMNIATTN_FP8_E4M3) return OMNIATTN_EUNSUPPORTED;
  if (prob.out_dtype != OMNIATTN_BF16 && prob.out_dtype != OMNIATTN_FP32) return OMNIATTN_EUNSUPPORTED;
  if (!(prob.softmax_scale == prob.softmax_scale)) return OMNIATTN_EINVAL;  // NaN
  if (prob.q_len < 0 || prob.q_len > 64) return OMNIATTN_EINVAL;
  const int q_len = prob.q_len > 1 ? prob.q_len : 1;
  if ((int64_t)prob.num_heads * q_len > (1 << 20)) return OMNIATTN_EUNSUPPORTED;
  for (int b = 0; b < prob.batch; ++b) {
    int64_t L = seq_lens[b];
    if (L < 0) return OMNIATTN_EINVAL;
    if (L > 0 && L < q_len) return OMNIATTN_EINVAL;  // every query needs its own token in the cache
    if ((L + kPage - 1) / kPage > prob.max_pages_per_seq) return OMNIATTN_EINVAL;
  }

  hp.prob = prob;
  hp.num_cus = num_cus;
  hp.seq_lens.assign(seq_lens, seq_lens + prob.batch);
  // Always four waves (one per SIMD), 32 heads each; waves past the last head idle along.
  hp.waves = 4;
  hp.head_block = hp.waves * kHeadsPerWave;
  hp.q_len = q_len;
  hp.tile = prob.kv_dtype == OMNIATTN_FP8_E4M3 ? kTileFp8 : kTile;
  hp.heads_total = prob.num_heads * q_len;
  // Several causal queries: query t keeps [0, S) and the W positions ending at its own token.
  // Over all queries that is [0, S) and (for W > 0) the W + q_len - 1 positions ending at L:
  // tiles are laid out for that union, the kernel masks per query.
  hp.window_union = prob.window > 0 ? (int)std::min<int64_t>((int64_t)prob.window + q_len - 1, INT32_MAX) : 0;
  hp.n_hb = (hp.heads_total + hp.head_block - 1) / hp.head_block;

  std::vector<Item> items;
  items.reserve((size_t)prob.batch * hp.n_hb);
  hp.retained_tokens = 0;
  int64_t total_cost = 0;
  for (int b = 0; b < prob.batch; ++b) {
    int L = seq_lens[b];
    int64_t sink_end = std::min<int64_t>(prob.sink, L);
    int64_t win_lo = std::max<int64_t>((int64_t)L - hp.window_union, 0);
    hp.retained_tokens += (win_lo <= sink_end) ? L : sink_end + (L - win_lo);
  }
  // sequence-major: the head blocks of one sequence read the same tiles; as neighbours they
  // land on one XCD (see the unit mapping in the kernel) and share its L2
  for (int b = 0; b < prob.batch; ++b)
    for (int hb = 0; hb < hp.n_hb; ++hb) {
      int n = tile_layout(seq_lens[b], prob.sink, hp.window_union, hp.tile).count();
      items.push_back({b, hb, n});
      total_cost += n + kSegFixedCost;
    }

  if (prob.num_splits_hint > 0) {
    hp.segs.clear();
    hp.unit_seg.assign(1, 0);
    for (const Item& it : items) {
      int pieces = std::max(1, std::min(prob.num_splits_hint, it.ntiles));
      pieces = std::max(pieces, (it.ntiles + kMaxSegTiles - 1) / kMaxSegTiles);
      for (int s = 0; s < pieces; ++s) {
        int lo = (int)((int64_t)it.ntiles * s / pieces);
        int hi = (int)((int64_t)it.ntiles * (s + 1) / pieces);
        hp.segs.push_back({it.b, it.hb, lo, hi, -1, (int32_t)hp.unit_seg.size() - 1, 0, it.ntiles});
        hp.unit_seg.push_back((int32_t)hp.segs.size());
      }
    }
  } else {
    int cap = (int)((total_cost + num_cus - 1) / num_cus);
    cap = std::max(cap, kSegFixedCost + 1);
    // splitting adds fixed costs, so the first capacity may need a few more units than CUs
    for (int iter = 0; iter < 64; ++iter) {
      if (fill_units(items, cap, nullptr, nullptr) <= num_cus) break;
      ++cap;
    }
    fill_units(items, cap, &hp.segs, &hp.unit_seg);
  }

  // partial slots for every (sequence, head block) cut into more than one segment
  hp.combine.clear();
  hp.n_slots = 0;
  hp.max_splits = 1;
  size_t i = 0;
  // segments of one item are consecutive in hp.segs by construction
  while (i < hp.segs.size()) {
    size_t j = i + 1;
    while (j < hp.segs.size() && hp.segs[j].b == hp.segs[i].b && hp.segs[j].hb == hp.segs[i].hb) ++j;
    int n = (int)(j - i);
    if (n > 1) {
      hp.combine.push_back({hp.segs[i].b, hp.segs[i].hb, hp.n_slots, n});
      for (size_t k = i; k < j; ++k) hp.segs[k].slot = hp.n_slots++;
      hp.max_splits = std::max(hp.max_splits, n);
    }
    i = j;
  }
  for (Segment& s : hp.segs) s.L = seq_lens[s.b];
  // workspace: lse of every partial row (fp32), then the partial rows in the output type
  const size_t rows = (size_t)hp.n_slots * hp.head_block;
  const size_t elt = prob.out_dtype == OMNIATTN_FP32 ? 4 : 2;
  hp.part_rows_offset = (rows * sizeof(float) + 255) & ~(size_t)255;
  hp.workspace_bytes = rows ? ((hp.part_rows_offset + rows * kV * elt + 255) & ~(size_t)255) : 0;
  return OMNIATTN_OK;
}

}  // namespace omniattn
