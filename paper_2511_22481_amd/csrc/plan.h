// Host-side plan for sparse MLA decode: retained ranges -> KV tiles -> work units.
//
// The retained set of a sequence of length L is the first S positions and the
// last W positions (paper section 3.2.1, second equation; 0-based and clipped
// to [0, L) here).  Tiles are TILE-token aligned pieces of the logical token
// axis that contain at least one retained position; because the set is at most
// two contiguous ranges, the tiles of a sequence are [0, ns) and [w0, w1) in
// units of TILE tokens, and only ns / w0 / w1 need to be known to enumerate
// them.  The device code re-derives ns / w0 from (L, S, W) with the same
// formulas (tile_layout below is shared by host and device).
#pragma once
#include <stdint.h>
#include <vector>

#include "../../include/omniattn.h"

#if defined(__HIPCC__)
#define OA_HD __host__ __device__
#else
#define OA_HD
#endif

namespace omniattn {

constexpr int kTile = 32;    // KV tokens per tile of a bf16 cache (divides the 128-token page)
constexpr int kTileFp8 = 64; // KV tokens per tile of an fp8 cache: the fp8 matrix instruction contracts 64 tokens
constexpr int kQK = OMNIATTN_QK_DIM;
constexpr int kV = OMNIATTN_V_DIM;
constexpr int kPage = OMNIATTN_PAGE;
constexpr int kHeadsPerWave = 32;
constexpr int kMaxSegTiles = 1024;  // tiles per segment (the kernel keeps a table of them in LDS)

struct TileLayout {
  int ns;   // tiles [0, ns) cover the sink range
  int w0;   // tiles [w0, w1) cover the recent range (w0 >= ns)
  int w1;
  OA_HD int count() const { return ns + (w1 > w0 ? w1 - w0 : 0); }
  // retained tile number i (ascending position) -> logical tile index
  OA_HD int logical(int i) const { return i < ns ? i : w0 + (i - ns); }
};

OA_HD inline TileLayout tile_layout(int L, int S, int W, int tile = kTile) {
  TileLayout t;
  if (L < 0) L = 0;
  int sink_end = S < L ? S : L;                 // sink range [0, sink_end)
  bool has_recent = W > 0 && L > 0;             // recent range [max(L - W, 0), L)
  int win_lo = L - W > 0 ? L - W : 0;
  t.ns = (sink_end + tile - 1) / tile;
  t.w1 = has_recent ? (L + tile - 1) / tile : 0;
  int w0 = has_recent ? win_lo / tile : 0;
  t.w0 = w0 > t.ns ? w0 : t.ns;                 // tiles shared with the sink range count once
  if (t.w0 > t.w1) t.w0 = t.w1;
  return t;
}

// Physically compressed cache: pages a sequence owns, and which of them holds a logical page.
// The first ceil(S/page) logical pages (those with sink tokens) are pinned; later logical pages
// share a ring of ceil(W/page) + 1 pages.  When logical page lp + ring opens (token position
// (lp + ring) * page), the newest token of logical page lp is ring * page - 127 >= W + 2
// positions back, outside the window, and it is no sink page: its page may be reused.
OA_HD inline int ring_pinned_pages(int S) { return S > 0 ? (S + kPage - 1) / kPage : 0; }
OA_HD inline int ring_ring_pages(int W) { return (W > 0 ? (W + kPage - 1) / kPage : 0) + 1; }
OA_HD inline int ring_slot(int S, int W, int lp) {
  const int ps = ring_pinned_pages(S);
  return lp < ps ? lp : ps + (lp - ps) % ring_ring_pages(W);
}

// One contiguous run of retained tiles of one (sequence, head block), processed
// by one work unit.  Layout is part of the ABI (omniattn_plan_get_segments).
struct Segment {
  int32_t b, hb, tile_lo, tile_hi, slot, unit, L, ntiles;
};

// One (sequence, head block) whose tiles were cut into several segments.
struct CombineItem {
  int32_t b, hb, slot0, nslots;
};

struct HostPlan {
  omniattn_problem_t prob;
  int num_cus = 0;
  int waves = 0;        // waves per work group; each owns 32 heads
  int head_block = 0;   // heads per work unit = 32 * waves
  int n_hb = 0;         // head blocks per sequence
  int tile = kTile;       // KV tokens per tile (kTile, or kTileFp8 for an fp8 cache)
  int q_len = 1;          // queries per sequence
  int heads_total = 0;    // q_len * num_heads rows of q per sequence ("virtual heads")
  int window_union = 0;   // window + q_len - 1: the union of the queries' windows ends at L
  int64_t retained_tokens = 0;
  int max_splits = 1;
  std::vector<int32_t> seq_lens;
  std::vector<Segment> segs;
  std::vector<int32_t> unit_seg;  // [n_units + 1] prefix into segs
  std::vector<CombineItem> combine;
  int n_slots = 0;
  size_t workspace_bytes = 0;
  size_t part_rows_offset = 0;  // byte offset of the partial rows inside the workspace
};

// Returns OMNIATTN_OK or an error code.
int build_host_plan(HostPlan& hp, const omniattn_problem_t& prob, const int32_t* seq_lens,
                    int num_cus);

}  // namespace omniattn
