// Launch interface between the C ABI (api.cpp) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace omniattn {

// A segment as the kernels read it: the planner's record with the two fields the device has
// no use for (work unit, tile count of the sequence) replaced by the partial slots of the
// segment's (sequence, head block): [slot0, slot0 + nslots) when it was cut, else nslots = 0.
struct DevSegment {
  int32_t b, hb, tile_lo, tile_hi, slot, slot0, L, nslots;
};
static_assert(sizeof(DevSegment) == sizeof(Segment), "same size as the planner's record");

// What a work unit reads first: its range of segments and a copy of the first of them,
// so that the kernel's first dependent load already yields a segment.
struct UnitHeader {
  int32_t seg_lo, seg_hi, pad0, pad1;
  DevSegment first;
};

struct DecodeParams {
  const uint16_t* q;
  const uint8_t* kv;
  const float* kv_scales;
  const int32_t* page_table;
  void* out;
  float* lse;
  void* part_o;     // [n_slots, head_block, 512] in the output type (bf16 or fp32)
  float* part_lse;  // [n_slots, head_block]
  const UnitHeader* units;
  const DevSegment* segs;
  int xcds;     // work group i runs on XCD i % xcds (1: no remapping)
  int H;        // rows of q per sequence: heads x queries
  int Hq, T;    // heads per query, queries per sequence (T >= 1)
  int Wu;       // W + T - 1: window of the union of the queries' kept sets
  int max_pages, S, W, head_block, out_fp32, n_units;
  float scale_log2;  // softmax_scale * log2(e)
};

struct CombineParams {
  const CombineItem* items;
  const void* part_o;
  const float* part_lse;
  void* out;
  float* lse;
  int H, head_block, out_fp32, n_items;
};

struct AppendParams {
  int32_t* seq_lens;
  const uint8_t* new_rows;
  const float* new_scales;
  const int32_t* seq_pages;
  uint8_t* kv;
  float* kv_scales;
  int32_t* page_table;
  int max_pages, S, W, ring_pages, row_bytes;  // row_bytes: 1152 (bf16) or 576 (fp8)
};
hipError_t launch_append(const AppendParams& p, int batch, hipStream_t stream);

// One-time per-process kernel attribute setup (large dynamic LDS).
hipError_t init_kernels();
// bf16 cache.  waves must be 4; grid = number of work units.
hipError_t launch_decode(const DecodeParams& p, int waves, int n_units, hipStream_t stream);
// fp8 cache: its own kernel (decode_fp8_kernel.hip), tiles of kTileFp8 tokens.
hipError_t init_fp8_kernel();
hipError_t launch_decode_fp8(const DecodeParams& p, int n_units, hipStream_t stream);
hipError_t launch_combine(const CombineParams& p, int n_items, hipStream_t stream);
// Copies `bytes` (rounded up to 16; both buffers are that large) from pinned host memory to
// device memory with a small kernel on `stream`.
hipError_t launch_copy16(void* dst, const void* src_pinned, size_t bytes, hipStream_t stream);
// Number of XCDs if work groups are dealt to them round-robin (work group i on XCD i % n),
// measured by a probe kernel on the current device; 1 if the pattern does not hold.
hipError_t probe_xcds(int* n_xcds);

}  // namespace omniattn
