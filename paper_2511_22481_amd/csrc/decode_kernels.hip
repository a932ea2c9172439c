// gfx950 kernels for sparse MLA decode over the OmniAttn retained set
// (paper section 3.2.1: softmax(q K_M^T * scale) V_M with M = sinks + recents):
// the main kernel for a bf16 cache (an fp8 cache has its own, decode_fp8_kernel.hip),
// the combine kernel and small helpers.
//
// Main kernel: one work group per work unit, WAVES waves, one wave per SIMD; each
// wave owns 32 heads and the full 512-wide output row of those heads.
//   a3  retained 32-token tiles stream into a ring of four LDS stages by direct
//       global->LDS 16-byte loads, two tiles ahead of the compute;
//   a4  S^T[token, head] = K_tile . Q^T on 32x32x16 bf16 MFMA, Q held in
//       registers as the B operand for the whole segment;
//   a5  positions outside the retained set get -inf (partial tiles only);
//   a6  softmax against a per-segment reference (see kRefSlack): a lane holds 16
//       tokens of one head, its partner lane (lane ^ 32) the other 16;
//   a7  O^T[col, head] += V^T . P^T on the same MFMA; the C layout of S^T is
//       exactly the B layout P^T needs, so P never leaves registers; V^T comes
//       from the same LDS tile through transposing LDS reads.  The PV MFMAs of
//       tile i-1 are issued interleaved with the softmax arithmetic of tile i;
//   a8  normalise, transpose through LDS, write bf16/fp32 rows + lse to the output
//       or, for a split sequence, to a partial slot (same type).
// Combine kernel (a9): merges the partials of sequences that were split.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "decode_common.h"

namespace omniattn {

constexpr int kRowBytes = kQK * 2;             // one token row in global memory (bf16)
constexpr int kChunksPerRow = kRowBytes / 16;  // 72

// LDS layout of one 32-token stage (36,864 bytes).  A token row is 72 chunks of
// 16 bytes: chunks 0..63 (the 512 value dims) and 64..71 (the 64 rope dims).
//   main part: row r at r * 1024; chunk c < 64 sits at position c ^ swz_main(r)
//   tail part: at kTailBase + r * 128; chunk 64 + c sits at position c ^ swz_tail(r)
// Splitting the row this way makes one direct global->LDS load instruction
// (64 lanes x 16 bytes = 1024 contiguous LDS bytes) fill exactly one main row,
// so a lane's global offset is a lane constant XOR a per-row constant.
// The XOR swizzles make both read patterns bank-conflict free: 16 consecutive
// rows at one chunk index (A-operand gather of K rows) land in 16 different
// 16-byte bank groups, and 4 consecutive rows x 64 bytes (one transposing read
// of V) land in the four quarters of the 64 banks.
constexpr int kMainRowBytes = 1024;
constexpr int kTailRowBytes = 128;
constexpr int kTailBase = kTile * kMainRowBytes;                      // 32,768
constexpr int kStageBytes = kTile * (kMainRowBytes + kTailRowBytes);  // 36,864
constexpr int kStages = 4;
constexpr int kTileTabBytes = kMaxSegTiles * 8;  // first global byte of every tile of the segment
constexpr int kJunkBytes = 4096;  // target of the direct loads issued for tiles that do not exist
constexpr int kLdsBytes = kStages * kStageBytes + 16 + kTileTabBytes + kJunkBytes;  // 16: retry flag
static_assert(kLdsBytes <= 160 * 1024, "LDS of one compute unit");
__host__ __device__ constexpr int swz_main(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
__host__ __device__ constexpr int swz_tail(int r) { return (r >> 1) & 7; }
// byte offset of chunk c (0..71) of row r inside a stage
__device__ __forceinline__ uint32_t lds_chunk(int r, int c) {
  return c < 64 ? r * kMainRowBytes + ((c ^ swz_main(r)) << 4)
                : kTailBase + r * kTailRowBytes + (((c - 64) ^ swz_tail(r)) << 4);
}

// Epilogue staging (reuses the stages): per wave 32 head rows of 1024 bytes + 16 pad.
constexpr int kOutRowBytes = 1024 + 16;
constexpr int kOutWaveBytes = kHeadsPerWave * kOutRowBytes;  // 33,280; x4 waves fits the stages

// Register files.  At one wave per SIMD a wave has 256 vector registers and 256
// accumulation registers.  The O^T tile (512 columns x 32 heads, fp32) fills the
// accumulation file exactly; Q (144 registers), S, P and operand fragments live in
// the vector file.  The MFMAs are written as assembly because only the assembly
// form lets the destination register file be chosen per instruction: S must not
// land in the accumulation file and O^T must never leave it.  Wait states the
// hardware does not interlock are supplied by hand: back-to-back MFMAs that
// accumulate into the same registers need none; a vector-ALU read of the result
// of an 8-pass MFMA needs 12 (settle_*()).
__device__ __forceinline__ void mfma_s_first(f32x16& s, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_s(f32x16& s, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(a), "v"(b));
}
__device__ __forceinline__ void settle_s(f32x16& s) { asm volatile("s_nop 11" : "+v"(s)); }
__device__ __forceinline__ void mfma_o(f32x16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// Every block of the O^T tile at once: nothing may read any of them before this point.
__device__ __forceinline__ void settle_o(f32x16 (&acc)[kV / 32]) {
  asm volatile("s_nop 11"
               : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]),
                 "+a"(acc[6]), "+a"(acc[7]), "+a"(acc[8]), "+a"(acc[9]), "+a"(acc[10]), "+a"(acc[11]),
                 "+a"(acc[12]), "+a"(acc[13]), "+a"(acc[14]), "+a"(acc[15]));
}

// Softmax reference.  exp2(x - r) is evaluated against a per-head reference r that is
// fixed for a whole segment (the maximum of the segment's first tile), not against a
// running maximum: softmax is invariant to r, so the only requirement is that exp2
// does not overflow.  That keeps every rescaling of the 256-register O^T tile out of
// the kernel.  The running maximum of all logits is tracked on the side; if some logit
// exceeded r by more than kRefSlack (2^64: far below fp32/bf16 overflow even after
// summing a million terms) the work group runs the same segment code a second time
// with r = that exact maximum, which cannot overflow.
constexpr float kRefSlack = 64.f;

// One head row of one (sequence, head block) that was cut into nslots partial results:
// out = sum_s w_s O_s with w_s = exp(lse_s - lse), lse = log sum_s exp(lse_s).  One wave per
// row, 64 lanes x 8 columns.  Partials are taken four at a time, all their loads in flight
// together, and folded into a running (maximum, sum, row) triple, so any number of partials
// takes one pass.  hl: the row inside the head block; orow: the row of out / lse.
template <bool OUT_FP32>
__device__ __forceinline__ void merge_row(const void* part_o, const float* part_lse, int slot0, int nslots,
                                          int head_block, int hl, int lane, void* out, float* lse_out, size_t orow) {
  constexpr int kBatch = 4;
  float m = -INFINITY, z = 0.f;
  float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int s0 = 0; s0 < nslots; s0 += kBatch) {
    float l[kBatch];
    f32x4 ra[kBatch], rb[kBatch];
    bf16x8 rh[kBatch];
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const bool ok = s0 + k < nslots;
      const size_t row = (size_t)(slot0 + (ok ? s0 + k : 0)) * head_block + hl;
      l[k] = ok ? part_lse[row] : -INFINITY;
      if constexpr (OUT_FP32) {
        const f32x4* src = (const f32x4*)((const float*)part_o + row * kV + lane * 8);
        ra[k] = src[0];
        rb[k] = src[1];
      } else {
        rh[k] = *(const bf16x8*)((const uint16_t*)part_o + row * kV + lane * 8);
      }
    }
    float mb = m;
#pragma unroll
    for (int k = 0; k < kBatch; ++k) mb = fmaxf(mb, l[k]);
    if (mb == -INFINITY) continue;  // nothing but empty partials so far
    const float keep = __expf(m - mb);  // 0 on the first batch (m = -inf)
    z *= keep;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] *= keep;
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const float w = __expf(l[k] - mb);  // 0 for a slot past the end
      z += w;
      if constexpr (OUT_FP32) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          o[c] = fmaf(w, ra[k][c], o[c]);
          o[4 + c] = fmaf(w, rb[k][c], o[4 + c]);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) o[c] = fmaf(w, (float)rh[k][c], o[c]);
      }
    }
    m = mb;
  }
  const float inv = z > 0.f ? 1.0f / z : 0.f;
  if (lane == 0) lse_out[orow] = z > 0.f ? m + __logf(z) : -INFINITY;
  if constexpr (OUT_FP32) {
    float* dst = (float*)out + orow * kV + lane * 8;
    *(f32x4*)dst = f32x4{o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
    *(f32x4*)(dst + 4) = f32x4{o[4] * inv, o[5] * inv, o[6] * inv, o[7] * inv};
  } else {
    bf16x8 v;
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = (__bf16)(o[k] * inv);
    *(bf16x8*)((uint16_t*)out + orow * kV + lane * 8) = v;
  }
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64, 1) void decode_kernel(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds_raw;  // LDS byte address of stage 0
  const uint32_t lds_flag = lds0 + kStages * kStageBytes;
  const uint32_t lds_tiles = lds_flag + 16;
  const uint32_t lds_junk = lds_tiles + kTileTabBytes;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  // Per-lane values are derived anew in each phase of a segment from a lane id that went
  // through an opaque move.  Computed once at kernel entry they would stay alive across the
  // MFMA loop, which has no registers to spare: the compiler would spill them, and every
  // spill reload waits for all vector-memory traffic, tile prefetches included.
  auto fresh_lane = [&]() {
    int l = lane;
    asm volatile("" : "+v"(l));
    return l;
  };

  constexpr int kRowsPerWave = kTile / WAVES;                  // 8, 16 or 32
  // direct loads per wave and tile: one per row plus one for the rope parts of 8 rows
  constexpr int kDmaPerTile = kRowsPerWave + kRowsPerWave / 8;

  // Work groups are dealt to the XCDs round-robin (p.xcds of them, measured on the device).
  // Consecutive work units (the pieces of one sequence, which read the same Q and exchange
  // their partial results) are mapped to work groups of one XCD so that they share its L2.
  const int per_xcd = (p.n_units + p.xcds - 1) / p.xcds;
  const int unit = ((int)blockIdx.x % p.xcds) * per_xcd + (int)blockIdx.x / p.xcds;
  if (unit >= p.n_units) return;
  // The unit's header (segment range and a copy of its first segment) in three 16-byte
  // loads issued together; the values are wave-uniform and moved to scalar registers.
  auto uniform4 = [](u32x4 v) {
    return u32x4{(uint32_t)__builtin_amdgcn_readfirstlane(v.x), (uint32_t)__builtin_amdgcn_readfirstlane(v.y),
                 (uint32_t)__builtin_amdgcn_readfirstlane(v.z), (uint32_t)__builtin_amdgcn_readfirstlane(v.w)};
  };
  static_assert(sizeof(UnitHeader) == 48 && sizeof(DevSegment) == 32, "header layout");
  const u32x4* hdr = (const u32x4*)(p.units + unit);
  const u32x4 hdr0 = hdr[0], hdr1 = hdr[1], hdr2 = hdr[2];
  const int seg_lo = __builtin_amdgcn_readfirstlane(hdr0.x), seg_hi = __builtin_amdgcn_readfirstlane(hdr0.y);

  for (int si = seg_lo; si < seg_hi; ++si) {
    u32x4 sg_a = hdr1, sg_b = hdr2;
    if (si != seg_lo) {
      const u32x4* sp = (const u32x4*)(p.segs + si);
      sg_a = sp[0];
      sg_b = sp[1];
    }
    sg_a = uniform4(sg_a);
    sg_b = uniform4(sg_b);
    const DevSegment sg = {(int32_t)sg_a.x, (int32_t)sg_a.y, (int32_t)sg_a.z, (int32_t)sg_a.w,
                           (int32_t)sg_b.x, (int32_t)sg_b.y, (int32_t)sg_b.z, (int32_t)sg_b.w};
    const int L = sg.L;
    const int h0 = sg.hb * p.head_block + wave * kHeadsPerWave;  // wave's first head
    const int lane_s = fresh_lane();
    const int n32 = lane_s & 31;  // head within the wave's 32 (B / C column)
    const int g = lane_s >> 5;    // k-group of the MFMA operands
    // Tiles cover the union of the queries' kept sets: [0, S) and the Wu = W + T - 1 positions
    // ending at L (one query: Wu = W).
    const TileLayout tl = tile_layout(L, p.S, p.Wu);
    const int n_tiles = sg.tile_hi - sg.tile_lo;
    // A tile counts as full when every query keeps all of its positions: the earliest query
    // sees a sequence of length L0 = L - (T - 1) and has the earliest window end, the latest
    // one the latest window start L - W.
    const int L0 = L - (p.T - 1);
    const int sink_end = p.S < L0 ? p.S : L0;

    auto tile_pos = [&](int it) { return tl.logical(sg.tile_lo + it) * kTile; };
    // ring position of a tile's stage
    // (unsigned: a signed remainder could be negative as far as the compiler knows, and it
    // then refuses to fold constant offsets into the LDS instructions built on these addresses)
    auto stage_of = [](int it) -> uint32_t { return (uint32_t)it & (kStages - 1); };
    auto tile_full = [&](int pos0) {
      return (pos0 + kTile <= sink_end) || (pos0 >= L - p.W && pos0 + kTile <= L0);
    };
    // ---- tile loader: wave w fills rows [w * kRowsPerWave, ...) of stage it & 3 ----
    // A tile is fetched by kDmaPerTile direct-load instructions per wave.  Exactly that
    // many are issued for every tile index, also for tiles past the segment's end and for
    // tiles filled through registers (partial tiles): those point at a junk region.
    // The count of loads in flight per tile is therefore a constant, which is what the
    // vmcnt-based wait_tile relies on, and the loop needs no branch per load.
    struct TileSrc {
      const uint8_t* gbase;   // first byte of the tile's rows in the cache (placeholder loads: page 0 of the cache)
      uint32_t lmain, ltail;  // LDS destinations of row 0 (main part, tail part)
      uint32_t mstride, tstride;  // 1024 / 128, or 0 for the junk target
    };
    auto prep_tile_e = [&](int it, uint32_t e_lo, uint32_t e_hi) -> TileSrc {
      TileSrc ts;
      // Placeholder loads read up to one tile's worth of bytes behind gbase: the cache's first
      // page (128 rows) always holds that much, which a small q tensor does not.
      ts.gbase = p.kv;
      ts.lmain = ts.ltail = lds_junk;
      ts.mstride = ts.tstride = 0;
      if (it >= n_tiles) return ts;
      // table entry: first global byte of the tile's rows; bit 0 = every position retained
      const bool full = e_lo & 1;
      const uint8_t* gbase = (const uint8_t*)(uintptr_t)(((uint64_t)e_hi << 32) | (e_lo & ~1u));
      const int stage = stage_of(it);
      const uint32_t lbase = lds0 + stage * kStageBytes;
      const int row_w0 = wave * kRowsPerWave;
      if (full) {
        ts.gbase = gbase;
        ts.lmain = lbase;
        ts.ltail = lbase + kTailBase;
        ts.mstride = kMainRowBytes;
        ts.tstride = kTailRowBytes;
      } else {
        // partial tile: rows outside the retained set are zero-filled, never loaded
        // (their contents are unspecified and 0 * NaN would poison the PV product)
        const int pos0 = tile_pos(it);
#pragma unroll 1
        for (int ci = lane; ci < kRowsPerWave * kChunksPerRow; ci += 64) {
          const int r = ci / kChunksPerRow;
          const int c = ci - r * kChunksPerRow;
          const int row = row_w0 + r;
          u32x4 v = {0, 0, 0, 0};
          if (retained(pos0 + row, L, p.S, p.Wu)) v = *(const u32x4*)(gbase + row * kRowBytes + (c << 4));
          *LDS_PTR(u32x4, lbase + lds_chunk(row, c)) = v;
        }
      }
      return ts;
    };
    // Direct load number k (0 .. kDmaPerTile-1) of a prepared tile.  Four consecutive main
    // rows share one LDS base (M0): the instruction's immediate offset (a multiple of the
    // 1024-byte LDS row) selects the row on the LDS side and is subtracted from the lane's
    // global offset.  The per-lane offset costs one XOR-and-add per load, computed from a
    // lane id that went through an opaque move: kept alive across the MFMA loop as loop
    // invariants the offsets would cost registers the loop does not have.
    auto dma_piece = [&](const TileSrc& ts, auto k_tag) {
      constexpr int k = decltype(k_tag)::value;
      uint32_t l16 = lane << 4;
      asm volatile("" : "+v"(l16));
      const int row_w0 = wave * kRowsPerWave;
      if constexpr (k < kRowsPerWave) {  // main part: one instruction per row; lane l fetches chunk l ^ swz_main(row)
        constexpr int imm = (k & 3) * kMainRowBytes;
        const int row = row_w0 + k;
        if constexpr ((k & 3) == 0) dma_set_lds_base(ts.lmain + row * ts.mstride);
        dma16<imm>(ts.gbase, (l16 ^ (swz_main(row) << 4)) + (row * kRowBytes - imm));
      } else {  // tail part: one instruction per 8 rows; lane l fetches row l / 8, rope chunk (l & 7) ^ swz
        const int r8 = row_w0 + 8 * (k - kRowsPerWave);
        const uint32_t row = r8 + (l16 >> 7);
        dma_set_lds_base(ts.ltail + r8 * ts.tstride);
        dma16<0>(ts.gbase, row * kRowBytes + ((64 + (((l16 >> 4) & 7) ^ swz_tail(row))) << 4));
      }
    };
    // Table entry of tile `it`.  The index is clamped to the table; entries at or past
    // n_tiles are stale and never interpreted (prep_tile_e checks the index first).
    auto tile_entry = [&](int it) -> u32x2 {
      return *LDS_PTR(u32x2, lds_tiles + (it < kMaxSegTiles ? it : kMaxSegTiles - 1) * 8);
    };
    auto prep_tile = [&](int it) -> TileSrc {
      const u32x2 e = tile_entry(it);
      return prep_tile_e(it, __builtin_amdgcn_readfirstlane(e.x), __builtin_amdgcn_readfirstlane(e.y));
    };
    auto issue_tile = [&](int it) {
      const TileSrc ts = prep_tile(it);
      [&]<int... K>(std::integer_sequence<int, K...>) {
        (dma_piece(ts, std::integral_constant<int, K>{}), ...);
      }(std::make_integer_sequence<int, kDmaPerTile>{});
    };
    // Wait for this wave's share of a tile: only the loads of the tile after it may still
    // be in flight.
    auto wait_tile = [&]() { wait_vm<kDmaPerTile>(); };

    // The page-table entries of the segment's tiles come first: the tile table and with it
    // the first direct loads depend on them.
    // Table: first global byte of every tile (bit 0: whole tile retained), kept in LDS: the
    // loop then needs no global load of its own besides the direct tile loads, whose
    // completion counter must not be disturbed by other vector-memory waits.
    constexpr int kTabPerThread = kMaxSegTiles / (WAVES * 64);
    int tid_s = tid;  // per segment, see fresh_lane
    asm volatile("" : "+v"(tid_s));
    int page_of[kTabPerThread];
    // Unconditional loads, so that all of a thread's entries are requested together instead
    // of one per branch: an index past the segment's tiles is clamped to its last tile, and
    // a segment without tiles reads (and ignores) a word of the plan instead.
    const int32_t* pt_row = n_tiles > 0 ? p.page_table + (size_t)sg.b * p.max_pages : (const int32_t*)p.units;
#pragma unroll
    for (int u = 0; u < kTabPerThread; ++u) {
      const int t = tid_s + u * WAVES * 64;
      const int tc = t < n_tiles ? t : n_tiles - 1;
      page_of[u] = pt_row[n_tiles > 0 ? tile_pos(tc) >> 7 : 0];
    }
    // ---- Q fragments: B operand, lane (head n32, g) holds d = 16 ks + 8 g .. + 8 ----
    // Requested right behind the page-table entries, so that they stream in while the tile
    // table is built and the first direct loads are issued; they are older than those
    // loads, so the wait for tile 0 covers them.
    bf16x8 qf[kQK / 16];
    auto load_q = [&]() {
      // heads past H (a partly filled wave) read the last real head; their results are never written
      const int head = h0 + n32;
      const uint16_t* qrow = p.q + ((size_t)sg.b * p.H + (head < p.H ? head : p.H - 1)) * kQK + g * 8;
#pragma unroll
      for (int ks = 0; ks < kQK / 16; ++ks)
        qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + ks * 16));
    };
    load_q();
#pragma unroll
    for (int u = 0; u < kTabPerThread; ++u) {
      const int t = tid_s + u * WAVES * 64;
      if (t < n_tiles) {
        const int pos0 = tile_pos(t);
        const uint64_t a = (uint64_t)(uintptr_t)p.kv +
                           ((uint64_t)page_of[u] * kPage + (pos0 & (kPage - 1))) * kRowBytes;
        *LDS_PTR(u32x2, lds_tiles + t * 8) = u32x2{(uint32_t)a | (uint32_t)tile_full(pos0), (uint32_t)(a >> 32)};
      }
    }
    if (tid == 0) *LDS_PTR(int, lds_flag) = 0;  // the retry vote at the segment's end
    __syncthreads();
    issue_tile(0);
    issue_tile(1);

    // LDS fragment requests kept in flight (the hand-over between iterations is written for 8)
    constexpr int kRing = 8;
    constexpr int kNK = kQK / 16;       // 36 MFMAs for S^T
    constexpr int kNV = 2 * (kV / 32);  // 32 MFMAs for O^T

    // The MFMAs are volatile assembly, which the scheduler does not move loads across, so
    // the LDS reads are software-pipelined by hand through one ring of kRing fragments:
    // the MFMAs of an iteration (36 for S^T of tile `it`, then 32 for PV of tile it-1)
    // consume the ring in order and each fragment is requested kRing MFMAs ahead.
    // LDS read addresses.  For a tile, 12 K-fragment and 8 V-fragment address registers
    // are formed once (XOR of the swizzle-dependent field, plus the stage base); every read
    // then only adds an immediate.  They are rebuilt per tile from bases that pass through
    // an opaque move, so that the compiler neither keeps them alive across tiles nor
    // spills them (a spill reload waits on the vector-memory counter and would drain the
    // tile prefetch).
    // QK^T A operand: token row n32, chunk 2 ks + g.  For ks < 32 the chunk position is
    // ((2 (ks & 7) + g) ^ swz) + 16 (ks >> 3); since 2 (ks & 7) has bit 0 clear, the byte
    // offset is am ^ ((ks & 7) << 5) plus a constant.
    uint32_t am = n32 * kMainRowBytes + ((g ^ swz_main(n32)) << 4);
    uint32_t at = kTailBase + n32 * kTailRowBytes + ((g ^ swz_tail(n32)) << 4);
    // PV A operand (V^T): each 16-lane group reads a 4-token x 16-column block transposed.
    // Lane row = 16 th + 8 hi + 4 g + (i16 >> 2); chunk = 4 cb + c_lane.  Chunk position =
    // ((cb & 3) * 4 + c_lane) ^ swz; the swizzle's upper two bits only touch the (cb & 3)
    // field, so the byte offset is vb{hi} ^ ((cb & 3) << 6) + (cb >> 2) * 256.
    uint32_t vb0, vb1;
    {
      const int i16 = lane_s & 15;
      const int c_lane = ((lane_s >> 4) & 1) * 2 + ((i16 & 3) >> 1);
      const int half8 = (i16 & 1) * 8;
      const int r0 = g * 4 + (i16 >> 2), r1 = 8 + r0;
      vb0 = r0 * kMainRowBytes + ((c_lane ^ swz_main(r0)) << 4) + half8;
      vb1 = r1 * kMainRowBytes + ((c_lane ^ swz_main(r1)) << 4) + half8;
    }
    auto launder_offsets = [&]() { asm volatile("" : "+v"(am), "+v"(at), "+v"(vb0), "+v"(vb1)); };
    struct KAddr { uint32_t a[12]; };
    struct VAddr { uint32_t a[8]; };
    auto k_addr = [&](uint32_t st) -> KAddr {
      KAddr r;
#pragma unroll
      for (int b = 0; b < 8; ++b) r.a[b] = (am ^ (b << 5)) + st;
#pragma unroll
      for (int b = 0; b < 4; ++b) r.a[8 + b] = (at ^ (b << 5)) + st;
      return r;
    };
    auto v_addr = [&](uint32_t st) -> VAddr {
      VAddr r;
#pragma unroll
      for (int cl = 0; cl < 4; ++cl) {
        r.a[cl] = (vb0 ^ (cl << 6)) + st;
        r.a[4 + cl] = (vb1 ^ (cl << 6)) + st;
      }
      return r;
    };
    auto load_k = [&](const KAddr& ka, int ks) -> bf16x8 {
      if (ks < 32) return *LDS_PTR(bf16x8, ka.a[ks & 7] + (ks >> 3) * 256);
      return *LDS_PTR(bf16x8, ka.a[8 + ks - 32]);
    };
    auto load_v = [&](const VAddr& va, int j) -> bf16x8 {  // j = th * 16 + cb
      const int th = j >> 4, cb = j & 15;
      const uint32_t imm = th * 16 * kMainRowBytes + (cb >> 2) * 256;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, va.a[cb & 3] + imm));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, va.a[4 + (cb & 3)] + imm));
      return __builtin_bit_cast(bf16x8, s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
    };
    // Per-lane validity bits of a partial tile: bit i = element i is a retained position
    // (element i is token (i/4)*8 + g*4 + i%4 of the tile).
    // With several queries per sequence the lane's head belongs to query tq, which sees a
    // sequence of length L - (T - 1 - tq) (derived here, on the rare path, rather than kept in
    // a register through the loop).
    auto valid_bits = [&](int pos0) -> uint32_t {
      int Lq = L;
      if (p.T > 1) {
        const int l = fresh_lane();
        int tq = (h0 + (l & 31)) / p.Hq;
        tq = tq < p.T ? tq : p.T - 1;  // lanes past the last head
        Lq = L - (p.T - 1 - tq);
      }
      uint32_t m = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        m |= (uint32_t)retained(pos0 + (i >> 2) * 8 + g * 4 + (i & 3), Lq, p.S, p.W) << i;
      return m;
    };
    // Logits are used in the log2 domain relative to the reference: t = s * c - ref (one
    // fused multiply-add).  A masked-out position gets the raw value that maps to t = -inf.
    const float c = p.scale_log2;
    const float masked_raw = c < 0.f ? INFINITY : -INFINITY;
    auto mask_partial = [&](f32x16& s, int pos0) {
      const uint32_t vbits = valid_bits(pos0);
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = (vbits >> i) & 1 ? s[i] : masked_raw;
    };

    float ref = 0.f, l_run = 0.f;
    float ref_exact = __builtin_nanf("");  // NaN: take the reference from the first tile
    f32x16 acc[kV / 32];

#pragma unroll 1
    for (int attempt = 0; attempt < 2; ++attempt) {
      if (attempt > 0) {
        // (Q is fetched again rather than kept alive across the whole first attempt)
        load_q();
        issue_tile(0);
        issue_tile(1);
      }
#pragma unroll
      for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
      float mt_all = -INFINITY;  // running maximum of this lane's t = s * c - ref

      if (n_tiles > 0) {
        // pn: bf16 weights of the tile whose S^T was computed last (the loop copies them to the
        // B operand registers of its PV MFMAs early in the next iteration); fr: the ring of
        // operand fragments requested ahead.
        bf16x8 pn[2], fr[kRing];
        f32x16 s;

        // ---- tile 0: S^T, reference, weights (no PV to overlap with yet) ----
        {
          wait_tile();  // tile 1 may still be in flight; Q is older than tile 0
          __syncthreads();
          launder_offsets();
          const KAddr ka0 = k_addr(lds0);
#pragma unroll
          for (int d = 0; d < kRing; ++d) fr[d] = load_k(ka0, d);
          issue_tile(2);
#pragma unroll
          for (int m = 0; m < kNK; ++m) {
            if (m == 0) mfma_s_first(s, fr[m % kRing], qf[m]);
            else mfma_s(s, fr[m % kRing], qf[m]);
            if (m + kRing < kNK) fr[m % kRing] = load_k(ka0, m + kRing);
          }
          settle_s(s);
          const int pos0 = tile_pos(0);
          if (!tile_full(pos0)) mask_partial(s, pos0);
          float mx = -INFINITY;
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[i] * c);
          if (ref_exact == ref_exact) {
            ref = ref_exact;
          } else {
            const float m2 = fmaxf(mx, __shfl_xor(mx, 32));
            // An integer reference makes weights computed against different references
            // differ by exact powers of two, so their bf16 roundings agree between
            // different partitions of the same sequence.  (-inf only if the data itself
            // holds -inf / NaN logits.)
            ref = m2 == -INFINITY ? 0.f : ceilf(m2);
          }
          float lsum = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float t = fmaf(s[i], c, -ref);
            mt_all = fmaxf(mt_all, t);
            const float e = __builtin_amdgcn_exp2f(t);
            lsum += e;
            pn[i >> 3][i & 7] = (__bf16)e;
          }
          l_run = lsum;
        }

        // ---- tiles 1 .. n-1 and the last PV as one continuous stream of MFMAs ----
        // Iteration `it` issues 68 MFMAs: S^T of tile `it` (36), then PV of tile it-1 (32),
        // with the softmax arithmetic of tile `it` and the direct loads of tile it+2 spread
        // between them.  With one wave per SIMD the wave's own instruction issue is the
        // scarce resource, and the matrix pipeline drains whenever the wave does anything
        // else for long.  So nothing is done between iterations: the operand ring is
        // continuous across them (fragment m lives in slot m % 8; the next iteration's first
        // eight fragments are requested behind MFMAs 63 .. 67 as their slots fall free: 4 .. 7
        // first, then 0 .. 3), the LDS addresses of the next iteration are formed a few at a
        // time behind MFMAs whose own addresses are no longer needed, and the barrier that
        // publishes tile it+1 sits behind MFMA 63, where the four fragments still in flight
        // were requested four MFMAs earlier.
        KAddr ka;  // K fragments of tile `it` (in use behind MFMAs 60 of the iteration before .. 27)
        VAddr va;  // V fragments of tile it-1 (in use behind MFMAs 20 .. 59)
        // table entry of tile it+2: requested behind MFMA 16 of the previous iteration, moved to
        // scalar registers behind MFMA 34, when it has long arrived
        u32x2 e_tab;
        uint32_t e_lo, e_hi;
        launder_offsets();
        if (n_tiles > 1) {
          wait_tile();
          __syncthreads();  // tile 1 is visible
          ka = k_addr(lds0 + kStageBytes);
#pragma unroll
          for (int d = 0; d < kRing; ++d) fr[d] = load_k(ka, d);
        }
        e_tab = tile_entry(3);
        e_lo = __builtin_amdgcn_readfirstlane(e_tab.x);
        e_hi = __builtin_amdgcn_readfirstlane(e_tab.y);

        auto body = [&](const int it) {
          const int stage = stage_of(it);
          const uint32_t st_prev = lds0 + stage_of(it - 1) * kStageBytes;
          const uint32_t st_next = lds0 + stage_of(it + 1) * kStageBytes;
          const TileSrc ts = prep_tile_e(it + 2, e_lo, e_hi);
          uint32_t full_word = 1;
          float lsum = 0.f, mt = -INFINITY;
          bf16x8 pf[2];  // weights of tile it-1, taken over from pn behind MFMA 2
          // One MFMA and what is issued behind it; m is a compile-time constant.
          auto step = [&](auto m_tag) {
            constexpr int m = decltype(m_tag)::value;
            constexpr int slot = m % kRing;
            if constexpr (m == 0) mfma_s_first(s, fr[slot], qf[m]);
            else if constexpr (m < kNK) mfma_s(s, fr[slot], qf[m]);
            else mfma_o(acc[(m - kNK) & 15], fr[slot], pf[(m - kNK) >> 4]);
            // the fragment eight MFMAs ahead: of this iteration, or (behind MFMAs 64 .. 67)
            // K fragments 0 .. 3 of tile it+1.  (After the last tile these read a stage that
            // holds nothing new; the values are never used.)
            if constexpr (m + kRing < kNK) fr[slot] = load_k(ka, m + kRing);
            else if constexpr (m + kRing < kNK + kNV) fr[slot] = load_v(va, m + kRing - kNK);
            else if constexpr (m >= 64) fr[slot] = load_k(ka, slot);
            if constexpr (m == 2) {
              pf[0] = pn[0];
              pf[1] = pn[1];
            }
            if constexpr (m == 30) full_word = *LDS_PTR(uint32_t, lds_tiles + it * 8);
            if constexpr (m == 16) e_tab = tile_entry(it + 3);
            if constexpr (m == 34) {
              e_lo = __builtin_amdgcn_readfirstlane(e_tab.x);
              e_hi = __builtin_amdgcn_readfirstlane(e_tab.y);
            }
            // the direct loads of tile it+2: one every four MFMAs of the S^T phase (whose MFMAs
            // leave issue slots free; the PV phase, with two LDS reads and a softmax element per
            // MFMA, has none to spare)
            if constexpr (m % 4 == 1 && m / 4 < kDmaPerTile) dma_piece(ts, std::integral_constant<int, m / 4>{});
            // LDS addresses, formed in registers whose previous contents are no longer needed:
            // V of tile it-1 behind MFMAs 20 .. 27 (K addresses 0 .. 3 are done with), the
            // next iteration's K behind MFMAs 60 .. 62
            if constexpr (m == 20) launder_offsets();
            if constexpr (m >= 20 && m < 24) va.a[m - 20] = (vb0 ^ ((m - 20) << 6)) + st_prev;
            if constexpr (m >= 24 && m < 28) va.a[m - 20] = (vb1 ^ ((m - 24) << 6)) + st_prev;
            // (opaque: otherwise the compiler may rebase these addresses on one another and pay
            // for it with an add in front of every LDS read instead of using the offset field)
            if constexpr (m >= 20 && m < 28) asm volatile("" : "+v"(va.a[m - 20]));
            if constexpr (m == 60) launder_offsets();
            if constexpr (m >= 60 && m < 63) {
              constexpr int q = m - 60;
#pragma unroll
              for (int b = 0; b < 4; ++b) {
                if constexpr (q < 2) ka.a[4 * q + b] = (am ^ ((4 * q + b) << 5)) + st_next;
                else ka.a[8 + b] = (at ^ (b << 5)) + st_next;
                asm volatile("" : "+v"(ka.a[q < 2 ? 4 * q + b : 8 + b]));
              }
            }
            if constexpr (m == 63) {
              // Tile it+1 becomes visible, and every wave is done with tile it-1 (its last
              // fragments were requested behind MFMA 59 and the barrier's fence waits for
              // them), whose stage the direct loads of the next iteration overwrite.
              wait_tile();
              __syncthreads();
#pragma unroll
              for (int d = 4; d < 8; ++d) fr[d] = load_k(ka, d);
            }
            constexpr int j = m - kNK;
            if constexpr (j == 0) {
              if (!(full_word & 1)) {  // wave-uniform and rare
                settle_s(s);
                mask_partial(s, tile_pos(it));
              }
            }
            // S^T may be read by the vector ALU 12 instructions after its last MFMA: the
            // 16 softmax elements of tile `it` are spread over PV MFMAs 4 .. 31 of tile it-1
            // (checked on the generated code at build time).
            constexpr int kFirst = 4;
            if constexpr (j >= kFirst) {
              constexpr int i = ((j - kFirst) * 16) / (kNV - kFirst), i1 = ((j + 1 - kFirst) * 16) / (kNV - kFirst);
              if constexpr (i1 > i) {  // at most one element per MFMA
                const float t = fmaf(s[i], c, -ref);
                mt = fmaxf(mt, t);
                const float e = __builtin_amdgcn_exp2f(t);
                lsum += e;
                pn[i >> 3][i & 7] = (__bf16)e;
              }
            }
          };
          [&]<int... M>(std::integer_sequence<int, M...>) {
            (step(std::integral_constant<int, M>{}), ...);
          }(std::make_integer_sequence<int, kNK + kNV>{});
          mt_all = fmaxf(mt_all, mt);
          l_run += lsum;
        };
#pragma unroll 1
        for (int it = 1; it < n_tiles; ++it) body(it);
        // ---- PV of the last tile (the one place where the ring starts empty) ----
        {
          launder_offsets();
          va = v_addr(lds0 + stage_of(n_tiles - 1) * kStageBytes);
#pragma unroll
          for (int d = 0; d < kRing; ++d) fr[d] = load_v(va, d);
#pragma unroll
          for (int j = 0; j < kNV; ++j) {
            mfma_o(acc[j & 15], fr[j % kRing], pn[j >> 4]);
            if (j + kRing < kNV) fr[j % kRing] = load_v(va, j + kRing);
          }
          settle_o(acc);  // the compiler may move the tile between registers right after this
        }
      }
      wait_vm<0>();  // the junk-region loads issued for tiles past the end

      // Did any head of the work group see its largest logit too far from its reference?  Too
      // far above, the weights could overflow; too far below (possible when the first tile
      // holds nothing for a query, so that its reference is 0), they underflow and the sum
      // loses its digits or vanishes.  Either way the segment is run again with the exact
      // maximum as reference.  (The flag was cleared before this segment's first barrier.)
      const float m2 = fmaxf(mt_all, __shfl_xor(mt_all, 32));
      const bool off = m2 > kRefSlack || (m2 < -kRefSlack && m2 != -INFINITY);
      if (attempt == 0 && __any(off) && (tid & 63) == 0) *LDS_PTR(int, lds_flag) = 1;
      __syncthreads();  // also: all reads of the stages are done before they are reused
      if (*LDS_PTR(int, lds_flag) == 0) break;
      ref_exact = m2 == -INFINITY ? 0.f : ref + ceilf(m2);
    }

    // ---- epilogue: normalise, transpose through LDS, write whole rows ----
    l_run += __shfl_xor(l_run, 32);
    // (l_run == 0: a head that keeps no position of this segment - possible only with several
    // queries per sequence, for a late query in a segment of early positions)
    const float inv = (n_tiles > 0 && l_run != 0.f) ? 1.0f / l_run : 0.f;
    const float lse = n_tiles > 0 ? (ref + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
    const bool final_out = sg.slot < 0;
    const uint32_t ost = lds0 + wave * kOutWaveBytes;  // this wave's staging rows
    const int heads_here = p.H - h0 < kHeadsPerWave ? p.H - h0 : kHeadsPerWave;  // may be <= 0
    const int lane_e = fresh_lane();
    const int n32e = lane_e & 31, ge = lane_e >> 5;
    if (n32e < heads_here && ge == 0) {
      if (final_out) p.lse[(size_t)sg.b * p.H + h0 + n32e] = lse;
      else p.part_lse[(size_t)sg.slot * p.head_block + wave * kHeadsPerWave + n32e] = lse;
    }
    // rows go to the output tensor, or (a split sequence) to this segment's partial slot;
    // both hold the output type
    const size_t row0 = final_out ? (size_t)sg.b * p.H + h0
                                  : (size_t)sg.slot * p.head_block + wave * kHeadsPerWave;
    if (!p.out_fp32) {
      // bf16: one round, a staged row is the head's 512 outputs (1024 bytes)
#pragma unroll
      for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          bf16x4 v = {(__bf16)(acc[cb][i4 * 4] * inv), (__bf16)(acc[cb][i4 * 4 + 1] * inv),
                      (__bf16)(acc[cb][i4 * 4 + 2] * inv), (__bf16)(acc[cb][i4 * 4 + 3] * inv)};
          *LDS_PTR(bf16x4, ost + n32e * kOutRowBytes + (cb * 32 + i4 * 8 + ge * 4) * 2) = v;
        }
      uint8_t* dst = (uint8_t*)(final_out ? p.out : p.part_o) + row0 * (kV * 2) + lane_e * 16;
#pragma unroll 4
      for (int h = 0; h < heads_here; ++h)
        *(u32x4*)(dst + (size_t)h * (kV * 2)) = *LDS_PTR(u32x4, ost + h * kOutRowBytes + lane_e * 16);
    } else {
      // fp32 rows: two rounds of 256 columns
      uint8_t* dst = (uint8_t*)(final_out ? p.out : p.part_o) + row0 * (kV * 4) + lane_e * 16;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
#pragma unroll
        for (int cb8 = 0; cb8 < 8; ++cb8)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const int cb = r * 8 + cb8;
            f32x4 v = {acc[cb][i4 * 4] * inv, acc[cb][i4 * 4 + 1] * inv, acc[cb][i4 * 4 + 2] * inv,
                       acc[cb][i4 * 4 + 3] * inv};
            *LDS_PTR(f32x4, ost + n32e * kOutRowBytes + (cb8 * 32 + i4 * 8 + ge * 4) * 4) = v;
          }
#pragma unroll 4
        for (int h = 0; h < heads_here; ++h)
          *(u32x4*)(dst + (size_t)h * (kV * 4) + r * 1024) =
              *LDS_PTR(u32x4, ost + h * kOutRowBytes + lane_e * 16);
      }
    }
    __syncthreads();  // staging rows are free again before the next segment's tiles arrive
  }
}

// Merge the partial results of one (sequence, head block): one work group per
// (combine item, group of 4 heads), one wave per head row (see merge_row).
// One instance per output type: with both in one kernel the registers of the fp32 path
// cost the bf16 path a third of its waves in flight, and this kernel lives on those.
template <bool OUT_FP32>
__global__ __launch_bounds__(256) void combine_kernel(CombineParams p) {
  const CombineItem it = p.items[blockIdx.x];
  const int hl = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int head = it.hb * p.head_block + hl;
  if (hl >= p.head_block || head >= p.H) return;
  merge_row<OUT_FP32>(p.part_o, p.part_lse, it.slot0, it.nslots, p.head_block, hl, threadIdx.x & 63, p.out, p.lse,
                      (size_t)it.b * p.H + head);
}

// Plan metadata from the plan's pinned host buffer (mapped into the device's address space)
// to its device copy, 16 bytes per thread.  A kernel rather than a copy command: a launch
// costs the host a few microseconds, a small asynchronous copy several times that.
__global__ __launch_bounds__(256) void copy16_kernel(u32x4* dst, const u32x4* src, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// One work group of 64 threads per probe block: the XCD the block runs on.
__global__ void xcd_probe_kernel(int* out) {
  if (threadIdx.x == 0) out[blockIdx.x] = (int)xcc_id();
}

template <int WAVES>
static hipError_t set_lds_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<WAVES>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

hipError_t init_kernels() {
  hipError_t e;
  if ((e = set_lds_attr<4>()) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_decode(const DecodeParams& p, int waves, int n_units, hipStream_t stream) {
  if (n_units <= 0) return hipSuccess;
  if (waves != 4) return hipErrorInvalidValue;
  if (p.xcds < 1) return hipErrorInvalidValue;
  // the grid is rounded up to a multiple of the XCD count (see the unit mapping in the kernel)
  dim3 grid(((n_units + p.xcds - 1) / p.xcds) * p.xcds), block(waves * 64);
  hipLaunchKernelGGL((decode_kernel<4>), grid, block, kLdsBytes, stream, p);
  return hipGetLastError();
}

hipError_t launch_combine(const CombineParams& p, int n_items, hipStream_t stream) {
  if (n_items <= 0) return hipSuccess;
  dim3 grid(n_items, (p.head_block + 3) / 4), block(256);
  if (p.out_fp32) hipLaunchKernelGGL(combine_kernel<true>, grid, block, 0, stream, p);
  else hipLaunchKernelGGL(combine_kernel<false>, grid, block, 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_copy16(void* dst, const void* src_pinned, size_t bytes, hipStream_t stream) {
  const int n = (int)((bytes + 15) / 16);
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(copy16_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, (u32x4*)dst, (const u32x4*)src_pinned, n);
  return hipGetLastError();
}

hipError_t probe_xcds(int* n_xcds) {
  constexpr int kBlocks = 64;
  *n_xcds = 1;
  int* d = nullptr;
  hipError_t e = hipMalloc((void**)&d, kBlocks * sizeof(int));
  if (e != hipSuccess) return e;
  int h[kBlocks];
  hipLaunchKernelGGL(xcd_probe_kernel, dim3(kBlocks), dim3(64), 0, 0, d);
  e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpy(h, d, sizeof(h), hipMemcpyDeviceToHost);
  (void)hipFree(d);
  if (e != hipSuccess) return e;
  int n = 0;
  for (int i = 0; i < kBlocks; ++i) n = h[i] + 1 > n ? h[i] + 1 : n;
  if (n < 1 || n > 16) return hipSuccess;
  for (int i = 0; i < kBlocks; ++i)
    if (h[i] != i % n) return hipSuccess;  // not round-robin: the kernel then does not remap
  *n_xcds = n;
  return hipSuccess;
}

}  // namespace omniattn
