// gfx950 kernel for sparse MLA decode over an fp8 (e4m3) latent cache with one fp32 scale
// per token (paper section 3.2.1: softmax(q K_M^T * scale) V_M with M = sinks + recents).
//
// The cache bytes are never widened: both contractions run on the 8-bit matrix instruction
// (32x32x64, twice the bf16 rate) straight out of the LDS tiles.
//   QK^T  The bf16 query row of a head is split once per segment into two e4m3 terms,
//         q = 2^e (hi + lo / 16): hi is q / 2^e rounded to e4m3 and lo 16 times the remainder,
//         rounded (the factor comes back as the block scale of the second matrix instruction).
//         With the row maximum scaled into [128, 256) every element that is not below 2^-14 of
//         the maximum is represented exactly (a bf16 significand is two e4m3 significands long),
//         smaller ones to 2^-22 of the maximum, so S^T = K hi + K lo carries fp32 accumulation
//         error only.  Two matrix instructions per
//         64 latent dims replace four bf16 ones and the K operand is read once for both.
//   PV    The weights of a head's 32 tokens of one tile half are rounded to e4m3 with one
//         power-of-two block scale (the B-side block scale of the scaled matrix instruction),
//         after the token's fp32 scale has been folded in; V is read raw through the 8-bit transposing
//         LDS read.  The output is normalised by the sum of the *rounded* weights, so the
//         rounding only perturbs the mix between tokens (a row with one dominant key is exact);
//         lse uses the exact sum.
// Everything else (work units, tile table, four-stage ring of direct global->LDS loads, fixed
// softmax reference with retry, epilogue, partial slots) follows the bf16 kernel; a tile here is
// 64 tokens (the same 36,864 bytes as a 32-token bf16 tile).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "decode_common.h"

namespace omniattn {

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(2))) unsigned short u16x2;

constexpr int kT8 = kTileFp8;                   // tokens per tile
constexpr int kRow8 = kQK;                      // bytes per token row
constexpr int kMain8 = 512, kTail8 = kQK - 512;  // value dims / rope dims of a row
constexpr int kChunks8 = kRow8 / 16;            // 36
constexpr int kTailBase8 = kT8 * kMain8;        // 32,768
constexpr int kStage8 = kT8 * kRow8;            // 36,864
constexpr int kStages8 = 4;
constexpr int kScale8 = kT8 * 4;                // fp32 scales of one tile
constexpr int kTileTab8 = kMaxSegTiles * 8;
constexpr int kJunk8 = 4096;
constexpr int kWaves8 = 4;
// stages | scale slots | per-wave weight scales and their reciprocals | retry flag | tile table | junk
constexpr int kLds8 = kStages8 * (kStage8 + kScale8) + kWaves8 * 2 * kScale8 + 16 + kTileTab8 + kJunk8;
static_assert(kLds8 <= 160 * 1024, "LDS of one compute unit");

// LDS layout of a stage: the first 512 bytes of the 64 rows (row r at 512 r), then their 64
// rope bytes (row r at 32,768 + 64 r).  16-byte chunk c of a row sits at position
// c ^ sw8_main(r) (c < 32, the XOR touches the low four bits) or 32 + ((c - 32) ^ sw8_tail(r)).
//   K operand (ds_read_b128, a row per lane, 16 consecutive rows at one chunk index): the sixteen
//   rows map to sixteen different 16-byte bank groups;
//   V^T operand (8-bit transposing read: per 32 lanes eight rows {8a + 4g + b} x two neighbouring
//   chunks): bit 0 of the swizzle depends on row bit 2 (= g, constant within a read), bits 1..3 on
//   (b, a), so the sixteen pieces again fall into sixteen different bank groups.
__host__ __device__ constexpr int sw8_main(int r) { return ((r & 3) << 1) | ((r >> 2) & 1) | (((r >> 3) & 1) << 3); }
__host__ __device__ constexpr int sw8_tail(int r) { return (r >> 2) & 3; }
__device__ __forceinline__ uint32_t lds_chunk8(int r, int c) {
  return c < 32 ? r * kMain8 + ((c ^ sw8_main(r)) << 4) : kTailBase8 + r * kTail8 + (((c - 32) ^ sw8_tail(r)) << 4);
}

// 8-bit matrix instructions (16 passes).  S^T goes to vector registers, O^T stays in the
// accumulation registers; a vector-ALU read of a result needs 19 wait states (settle8_*).
__device__ __forceinline__ void mfma8_s_first(f32x16& s, i32x8 a, i32x8 b) {
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0" : "=&v"(s) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma8_s(f32x16& s, i32x8 a, i32x8 b) {
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+v"(s) : "v"(a), "v"(b));
}
// s += a . (b * 2^-4): the low term of q is stored 16 times too large (kQLoShift), which keeps
// it out of the e4m3 subnormals for elements down to 2^-14 of the row's maximum
constexpr int kQLoShift = 4;
__device__ __forceinline__ void mfma8_s_lo(f32x16& s, i32x8 a, i32x8 b) {
  asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4" : "+v"(s) : "v"(a), "v"(b), "v"(127), "v"(127 - kQLoShift));
}
// acc += a . (b * 2^(sb - 127)).  Lane (column n, g) holds contraction indices 16 g .. 16 g + 15
// (bytes 0..15) and 32 + 16 g .. (bytes 16..31) of column n; byte 0 of its scale word applies to
// indices 32 g .. 32 g + 31 of that column, i.e. to bytes 16 g .. 16 g + 15 of both lanes of n (the A-side scale word is 127: 2^0; both scale words must be vector registers).
__device__ __forceinline__ void mfma8_o(f32x16& acc, i32x8 a, i32x8 b, int sb) {
  asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4" : "+a"(acc) : "v"(a), "v"(b), "v"(127), "v"(sb));
}
__device__ __forceinline__ void settle8_s(f32x16& s) { asm volatile("s_nop 15\n\ts_nop 3" : "+v"(s)); }
__device__ __forceinline__ void settle8_o(f32x16 (&acc)[kV / 32]) {
  asm volatile("s_nop 15\n\ts_nop 3"
               : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]),
                 "+a"(acc[6]), "+a"(acc[7]), "+a"(acc[8]), "+a"(acc[9]), "+a"(acc[10]), "+a"(acc[11]),
                 "+a"(acc[12]), "+a"(acc[13]), "+a"(acc[14]), "+a"(acc[15]));
}

constexpr float kRefSlack8 = 64.f;  // see the bf16 kernel: fixed softmax reference with retry

constexpr int kOutRowBytes8 = 1024 + 16;
constexpr int kOutWaveBytes8 = kHeadsPerWave * kOutRowBytes8;

}  // namespace

__global__ __launch_bounds__(kWaves8 * 64, 1) void decode_fp8_kernel(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  constexpr int WAVES = kWaves8;
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds_raw;
  const uint32_t lds_scales = lds0 + kStages8 * kStage8;
  const uint32_t lds_rscale = lds_scales + kStages8 * kScale8;
  const uint32_t lds_flag = lds_rscale + WAVES * 2 * kScale8;
  const uint32_t lds_tiles = lds_flag + 16;
  const uint32_t lds_junk = lds_tiles + kTileTab8;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // per-lane values are re-derived per phase from a lane id that went through an opaque
  // move, so that nothing computed at kernel entry stays alive across the loop
  auto fresh_lane = [&]() {
    int l = lane;
    asm volatile("" : "+v"(l));
    return l;
  };

  constexpr int kRowsPerWave = kT8 / WAVES;  // 16
  // direct loads per wave and tile: eight for the 512-byte parts of its 16 rows (two rows
  // each), one for their rope parts, one for the tile's 64 scales (wave 0; void elsewhere)
  constexpr int kDmaPerTile = kRowsPerWave / 2 + 2;

  const int per_xcd = (p.n_units + p.xcds - 1) / p.xcds;
  const int unit = ((int)blockIdx.x % p.xcds) * per_xcd + (int)blockIdx.x / p.xcds;
  if (unit >= p.n_units) return;
  auto uniform4 = [](u32x4 v) {
    return u32x4{(uint32_t)__builtin_amdgcn_readfirstlane(v.x), (uint32_t)__builtin_amdgcn_readfirstlane(v.y),
                 (uint32_t)__builtin_amdgcn_readfirstlane(v.z), (uint32_t)__builtin_amdgcn_readfirstlane(v.w)};
  };
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
    const int h0 = sg.hb * p.head_block + wave * kHeadsPerWave;
    const int lane_s = fresh_lane();
    const int n32 = lane_s & 31;  // head within the wave's 32 (B / C column); token row of the A operand
    const int g = lane_s >> 5;    // which 32 of the 64 contraction indices this lane holds
    const TileLayout tl = tile_layout(L, p.S, p.Wu, kT8);
    const int n_tiles = sg.tile_hi - sg.tile_lo;
    const int L0 = L - (p.T - 1);
    const int sink_end = p.S < L0 ? p.S : L0;

    auto tile_pos = [&](int it) { return tl.logical(sg.tile_lo + it) * kT8; };
    auto stage_of = [](int it) -> uint32_t { return (uint32_t)it & (kStages8 - 1); };
    auto tile_full = [&](int pos0) {
      return (pos0 + kT8 <= sink_end) || (pos0 >= L - p.W && pos0 + kT8 <= L0);
    };
    // ---- tile loader: wave w fills rows [16 w, 16 w + 16) of stage it & 3 ----
    // Exactly kDmaPerTile direct loads per wave are issued for every tile index (missing and
    // partial tiles: void loads into a junk region), so vmcnt(kDmaPerTile) is a tile-granular wait.
    struct TileSrc {
      const uint8_t* gbase;       // first byte of the tile's rows (void loads: page 0 of the cache)
      uint32_t lmain, ltail;      // LDS destinations of this wave's first row
      uint32_t on;                // 1: real tile, 0: void loads
      const float* sgbase;        // the tile's 64 scales in global memory
      uint32_t lscale;
    };
    auto prep_tile_e = [&](int it, uint32_t e_lo, uint32_t e_hi) -> TileSrc {
      TileSrc ts;
      ts.gbase = p.kv;  // the cache's first page holds a whole tile's worth of bytes
      ts.lmain = ts.ltail = lds_junk;
      ts.on = 0;
      ts.sgbase = nullptr;
      ts.lscale = lds_junk;
      if (it >= n_tiles) return ts;
      const bool full = e_lo & 1;
      const uint8_t* gbase = (const uint8_t*)(uintptr_t)(((uint64_t)e_hi << 32) | (e_lo & ~1u));
      const uint32_t lbase = lds0 + stage_of(it) * kStage8;
      const int row_w0 = wave * kRowsPerWave;
      const float* sbase = p.kv_scales + (gbase - p.kv) / kRow8;
      const uint32_t lscale = lds_scales + stage_of(it) * kScale8;
      if (full) {
        ts.gbase = gbase;
        ts.lmain = lbase + row_w0 * kMain8;
        ts.ltail = lbase + kTailBase8 + row_w0 * kTail8;
        ts.on = 1;
        ts.sgbase = sbase;
        ts.lscale = lscale;
      } else {
        // partial tile: rows outside the kept set are zero-filled, never loaded (their contents
        // are unspecified); such a position gets the smallest normal scale (its logit is -inf, its
        // weight 0, and it does not raise the bound on the tile's scales)
        const int pos0 = tile_pos(it);
#pragma unroll 1
        for (int ci = lane; ci < kRowsPerWave * kChunks8; ci += 64) {
          const int r = ci / kChunks8;
          const int c = ci - r * kChunks8;
          const int row = row_w0 + r;
          u32x4 v = {0, 0, 0, 0};
          if (retained(pos0 + row, L, p.S, p.Wu)) v = *(const u32x4*)(gbase + row * kRow8 + (c << 4));
          *LDS_PTR(u32x4, lbase + lds_chunk8(row, c)) = v;
        }
        if (lane < kRowsPerWave) {
          const int row = row_w0 + lane;
          *LDS_PTR(float, lscale + row * 4) = retained(pos0 + row, L, p.S, p.Wu) ? sbase[row] : 1.1754944e-38f;
        }
      }
      return ts;
    };
    auto dma_piece = [&](const TileSrc& ts, auto k_tag) {
      constexpr int k = decltype(k_tag)::value;
      uint32_t l = lane;
      asm volatile("" : "+v"(l));
      const int row_w0 = wave * kRowsPerWave;
      if constexpr (k < kRowsPerWave / 2) {
        // rows row_w0 + 2 k (lanes 0..31) and the next (lanes 32..63): lane fetches the chunk that
        // belongs at its LDS position.  The low four bits of the even row are those of 2 k.
        constexpr int imm = (k & 3) * 2 * kMain8;
        if constexpr ((k & 3) == 0) dma_set_lds_base(ts.lmain + ts.on * (2 * k * kMain8));
        const uint32_t hi = l >> 5;
        const uint32_t pos = ((l & 31) ^ (hi << 1) ^ sw8_main((2 * k) & 15)) << 4;
        const uint32_t off = ((row_w0 + 2 * k) * kRow8 + hi * kRow8 + pos) * ts.on + ((l << 4) & (ts.on - 1));
        dma16<imm>(ts.gbase, off - imm * ts.on);
      } else if constexpr (k == kRowsPerWave / 2) {
        // rope parts of the wave's 16 rows: lane fetches row l / 4, rope chunk (l & 3) ^ swizzle
        dma_set_lds_base(ts.ltail);
        const uint32_t row = row_w0 + (l >> 2);
        const uint32_t off = (row * kRow8 + ((32 + ((l & 3) ^ ((l >> 4) & 3))) << 4)) * ts.on + ((l << 4) & (ts.on - 1));
        dma16<0>(ts.gbase, off);
      } else {
        // the tile's 64 scales (wave 0)
        const bool real = ts.on != 0 && wave == 0;
        dma_set_lds_base(real ? ts.lscale : lds_junk);
        dma4(real ? (const uint8_t*)ts.sgbase : p.kv, l << 2);
      }
    };
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
    auto wait_tile = [&]() { wait_vm<kDmaPerTile>(); };

    // ---- page-table entries of the segment's tiles, tile table in LDS ----
    constexpr int kTabPerThread = kMaxSegTiles / (WAVES * 64);
    int tid_s = tid;
    asm volatile("" : "+v"(tid_s));
    int page_of[kTabPerThread];
    const int32_t* pt_row = n_tiles > 0 ? p.page_table + (size_t)sg.b * p.max_pages : (const int32_t*)p.units;
#pragma unroll
    for (int u = 0; u < kTabPerThread; ++u) {
      const int t = tid_s + u * WAVES * 64;
      const int tc = t < n_tiles ? t : n_tiles - 1;
      page_of[u] = pt_row[n_tiles > 0 ? tile_pos(tc) >> 7 : 0];
    }

    // ---- Q: the B operand of S^T.  Lane (head n32, g) holds dims 64 ks + 32 g .. + 31 of its
    // head for ks = 0..8, as two e4m3 terms of 32 bytes each per ks. ----
    // The rows are requested ahead of the first tiles and split behind them, so that the
    // conversion arithmetic runs while the tiles are on their way.
    i32x8 qh[kQK / 64], ql[kQK / 64];
    float c_head = 0.f;  // |softmax scale| * log2(e) * 2^e of the head's split (the sign goes into q)
    u32x4 raw[kQK / 64][4];
    auto request_q = [&]() {
      const int head = h0 + n32;
      const uint16_t* qrow = p.q + ((size_t)sg.b * p.H + (head < p.H ? head : p.H - 1)) * kQK + g * 32;
#pragma unroll
      for (int ks = 0; ks < kQK / 64; ++ks)
#pragma unroll
        for (int j = 0; j < 4; ++j) raw[ks][j] = *(const u32x4*)(qrow + ks * 64 + j * 8);
    };
    auto split_q = [&]() {
      // largest magnitude of the head's row: bf16 magnitudes order like unsigned integers
      u16x2 mx = {0, 0};
#pragma unroll
      for (int ks = 0; ks < kQK / 64; ++ks)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int k = 0; k < 4; ++k)
            mx = __builtin_elementwise_max(mx, __builtin_bit_cast(u16x2, raw[ks][j][k] & 0x7fff7fffu));
      uint32_t m = mx[0] > mx[1] ? mx[0] : mx[1];
      const uint32_t mo = __shfl_xor(m, 32);
      m = m > mo ? m : mo;
      // exponent e with max / 2^e in [128, 256); an all-zero (or denormal) row keeps e = 0,
      // Inf / NaN rows are scaled like the largest finite exponent and stay Inf / NaN
      int ex = (int)(m >> 7);
      ex = ex == 0 ? 0 : (ex > 254 ? 254 : ex) - 127 - 7;
      // a negative softmax scale is moved into q, so that a larger product is a larger logit
      const float inv_s = __builtin_amdgcn_ldexpf(p.scale_log2 < 0.f ? -1.0f : 1.0f, -ex);
      c_head = __builtin_amdgcn_ldexpf(fabsf(p.scale_log2), ex);
#pragma unroll
      for (int ks = 0; ks < kQK / 64; ++ks)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int k2 = 0; k2 < 2; ++k2) {
            // four values -> one dword of hi codes and one of lo codes
            int hi = 0, lo = 0;
            {
              const uint32_t pr = raw[ks][j][k2 * 2];
              const float x0 = __builtin_bit_cast(float, pr << 16) * inv_s;
              const float x1 = __builtin_bit_cast(float, pr & 0xffff0000u) * inv_s;
              hi = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, hi, false);
              const f32x2 back = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false);
              lo = __builtin_amdgcn_cvt_pk_fp8_f32((x0 - back[0]) * (float)(1 << kQLoShift), (x1 - back[1]) * (float)(1 << kQLoShift), lo, false);
            }
            {
              const uint32_t pr = raw[ks][j][k2 * 2 + 1];
              const float x0 = __builtin_bit_cast(float, pr << 16) * inv_s;
              const float x1 = __builtin_bit_cast(float, pr & 0xffff0000u) * inv_s;
              hi = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, hi, true);
              const f32x2 back = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
              lo = __builtin_amdgcn_cvt_pk_fp8_f32((x0 - back[0]) * (float)(1 << kQLoShift), (x1 - back[1]) * (float)(1 << kQLoShift), lo, true);
            }
            qh[ks][j * 2 + k2] = hi;
            ql[ks][j * 2 + k2] = lo;
          }
    };
    request_q();
#pragma unroll
    for (int u = 0; u < kTabPerThread; ++u) {
      const int t = tid_s + u * WAVES * 64;
      if (t < n_tiles) {
        const int pos0 = tile_pos(t);
        const uint64_t a = (uint64_t)(uintptr_t)p.kv + ((uint64_t)page_of[u] * kPage + (pos0 & (kPage - 1))) * kRow8;
        *LDS_PTR(u32x2, lds_tiles + t * 8) = u32x2{(uint32_t)a | (uint32_t)tile_full(pos0), (uint32_t)(a >> 32)};
      }
    }
    if (tid == 0) *LDS_PTR(int, lds_flag) = 0;
    __syncthreads();
    issue_tile(0);
    issue_tile(1);
    split_q();

    constexpr int kNK = 2 * 2 * (kQK / 64);  // 36 MFMAs for S^T: token half x 9 dim blocks x (hi, lo)
    constexpr int kNV = kV / 32;             // 16 MFMAs for O^T
    constexpr int kRing = 3;                 // operand fragments (32 bytes per lane) in flight

    // LDS read addresses (see the layout above).  K fragment (half h, dim block ks) of lane
    // (row n32, g): chunks 4 ks + 2 g and the next of row 32 h + n32.  V^T fragment (column
    // block cb, part pt) of lane l: tokens 16 pt + 8 a + 4 g + b with (a, b) from the lane's
    // position in its group of 16, chunk 2 cb + (group & 1).
    // One base register per operand and tile; the swizzle-dependent part of every read's
    // address is one XOR in front of it (the loop has no registers for a table of them).
    struct KAddr { uint32_t main, tail; };
    struct VAddr { uint32_t base; };
    auto k_addr = [&](uint32_t st) -> KAddr {
      const int l = fresh_lane();
      const int r32 = l & 31, gg = l >> 5;
      KAddr r;
      r.main = st + r32 * kMain8 + (((2 * gg) ^ sw8_main(r32)) << 4);
      r.tail = st + kTailBase8 + r32 * kTail8 + (((2 * gg) ^ sw8_tail(r32)) << 4);
      return r;
    };
    auto v_addr = [&](uint32_t st) -> VAddr {
      const int l = fresh_lane();
      const int ip = (l & 15) >> 1;
      const int rowlow = 8 * (ip >> 2) + 4 * (l >> 5) + (ip & 3);
      VAddr r;
      r.base = st + rowlow * kMain8 + ((((l >> 4) & 1) ^ sw8_main(rowlow)) << 4) + 8 * (l & 1);
      return r;
    };
    // (stage bases are multiples of 256 and the XORs touch bits 4 .. 7 only, so base ^ x is the
    // address with the swizzled field replaced)
    // fragment f = 9 h + ks of S^T
    auto load_k = [&](const KAddr& ka, int f) -> i32x8 {
      const int h = f / 9, ks = f % 9;
      i32x4 lo, hi;
      if (ks < 8) {
        const uint32_t imm = h * 32 * kMain8 + (ks >> 2) * 256;
        const uint32_t a = ka.main ^ ((ks & 3) << 6);
        lo = *LDS_PTR(i32x4, a + imm);
        hi = *LDS_PTR(i32x4, (a ^ 16u) + imm);
      } else {
        lo = *LDS_PTR(i32x4, ka.tail + h * 32 * kTail8);
        hi = *LDS_PTR(i32x4, (ka.tail ^ 16u) + h * 32 * kTail8);
      }
      return i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };
    auto load_v = [&](const VAddr& va, int cb) -> i32x8 {
      i32x8 r;
      const uint32_t a = va.base ^ ((cb & 7) << 5);
#pragma unroll
      for (int pt = 0; pt < 4; ++pt) {
        const i32x2 t = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(i32x2, a + (cb >> 3) * 256 + pt * 16 * kMain8));
        r[2 * pt] = t[0];
        r[2 * pt + 1] = t[1];
      }
      return r;
    };
    // Element i of half h of a lane's S^T is token 32 h + (i / 4) * 8 + 4 g + i % 4 of the tile.
    // Validity bits of a partial tile for this lane's head (several queries: the head's query
    // sees a sequence cut after its own token).
    auto valid_bits = [&](int pos0, int h) -> uint32_t {
      int Lq = L;
      if (p.T > 1) {
        const int l = fresh_lane();
        int tq = (h0 + (l & 31)) / p.Hq;
        tq = tq < p.T ? tq : p.T - 1;
        Lq = L - (p.T - 1 - tq);
      }
      uint32_t m = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        m |= (uint32_t)retained(pos0 + 32 * h + (i >> 2) * 8 + g * 4 + (i & 3), Lq, p.S, p.W) << i;
      return m;
    };
    // scales of the four tokens behind elements 4 q .. 4 q + 3 of half h
    auto scale_base = [&](uint32_t slot_base) -> uint32_t {
      uint32_t b = slot_base + g * 16;
      asm volatile("" : "+v"(b));
      return b;
    };
    auto tok4 = [&](uint32_t base, int h, int q) -> f32x4 { return *LDS_PTR(f32x4, base + h * 128 + q * 32); };
    auto tok2 = [&](uint32_t base, int h, int q, int w) -> f32x2 { return *LDS_PTR(f32x2, base + h * 128 + q * 32 + w * 8); };
    // Weight scales of the tile in `stage` and their reciprocals, for this wave's own use (lane =
    // token); returns es with every scale of the tile < 2^es (wave-uniform, at least -100).  The
    // weight of token j goes to the matrix instruction as round(w_j * scale_j), so a token whose
    // scale lies far below the tile's largest would underflow e4m3 and drop out of the rounded
    // weights' sum although its softmax weight counts.  Its weight scale is therefore raised to
    // 2^(es - 10): the sum stays right (also for a scale of zero), and its value row, at most
    // 2^-10 of the tile's largest values, enters the output that much too large at worst.  The
    // logits keep the true scale.
    // The maximum runs down each row of 16 lanes by shifted moves; the four row ends are read out
    // and combined on the scalar side.
    auto prep_rscale = [&](uint32_t stage) -> int {
      uint32_t l = lane;
      asm volatile("" : "+v"(l));
      const float sc = *LDS_PTR(float, lds_scales + stage * kScale8 + l * 4);
      uint32_t m = __builtin_bit_cast(uint32_t, sc) & 0x7fffffffu;  // positive floats order like integers
#define OA_ROW_SHR_MAX(n)                                                                        \
  {                                                                                              \
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x110 + (n), 0xf, 0xf, true); \
    m = m > o ? m : o;                                                                           \
  }
      OA_ROW_SHR_MAX(1) OA_ROW_SHR_MAX(2) OA_ROW_SHR_MAX(4) OA_ROW_SHR_MAX(8)
#undef OA_ROW_SHR_MAX
      const uint32_t a = __builtin_amdgcn_readlane(m, 15), b = __builtin_amdgcn_readlane(m, 31);
      const uint32_t c = __builtin_amdgcn_readlane(m, 47), d = __builtin_amdgcn_readlane(m, 63);
      const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
      int es = (int)((ab > cd ? ab : cd) >> 23) - 126;
      es = es < -100 ? -100 : es;
      // (a NaN scale reaches the output through the logits; here the maximum drops it)
      const float wsc = fmaxf(sc, __builtin_amdgcn_ldexpf(1.0f, es - 10));
      *LDS_PTR(float, lds_rscale + wave * 2 * kScale8 + l * 4) = wsc;
      *LDS_PTR(float, lds_rscale + wave * 2 * kScale8 + kScale8 + l * 4) = __builtin_amdgcn_rcpf(wsc);
      return es;
    };
    // Pass A over quads [q_lo, q_hi) of one half: raw logit -> u = s * scale_token, in place, or
    // -inf where the lane's validity bit is clear (two bit operations per element, without a
    // branch: a branch inside the MFMA stream costs the loop registers it does not have);
    // running maximum of u.
    auto pass_a = [&](f32x16& s, int h, uint32_t sbase, int q_lo, int q_hi, uint32_t vbits, float& mu) {
#pragma unroll
      for (int q = q_lo; q < q_hi; ++q) {
        const f32x4 sc = tok4(sbase, h, q);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int i = q * 4 + k;
          const uint32_t keep = (uint32_t)((int32_t)(vbits << (31 - i)) >> 31);  // all ones: valid
          const uint32_t ub = __builtin_bit_cast(uint32_t, s[i] * sc[k]);
          const float u = __builtin_bit_cast(float, (ub & keep) | (0xff800000u & ~keep));
          s[i] = u;
          mu = fmaxf(mu, u);
        }
      }
    };
    // max over the two lanes (l, l ^ 32) of a head
    // (v_permlane32_swap exchanges the first operand of lanes 32..63 with the second of lanes
    // 0..31.  Written as assembly: with the builtin the compiler drops the maximum of the two
    // results.  The wait states around it are the ones the compiler places for the builtin.)
    auto pair_max = [&](float x) -> float {
      float a = x, b = x;
      asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
      return fmaxf(a, b);
    };
    // Block exponent of a head's 32 weights of one tile half (mt: the largest t = u c - ref over
    // both lanes of the head): with kk = ceil(mt) - 8 + es (every token scale < 2^es), every
    // weight 2^(t - kk) * scale stays below 2^8 (e4m3 holds 448).
    auto block_exp = [&](float mt, int es) -> int {
      if (mt == -INFINITY) return 0;
      int kk = (int)ceilf(mt) - 8 + es;
      return kk < -126 ? -126 : (kk > 126 ? 126 : kk);
    };

    float ref = 0.f, l_run = 0.f, lq_run = 0.f;
    float ref_exact = __builtin_nanf("");
    f32x16 acc[kV / 32];

#pragma unroll 1
    for (int attempt = 0; attempt < 2; ++attempt) {
      if (attempt > 0) {
        request_q();
        issue_tile(0);
        issue_tile(1);
        split_q();
      }
#pragma unroll
      for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
      float mt_all = -INFINITY;
      l_run = 0.f;
      lq_run = 0.f;

      if (n_tiles > 0) {
        i32x8 pn, fr[kRing];  // pn: e4m3 weights of the tile at hand (B operand of its PV MFMAs)
        f32x16 s0, s1;        // S^T of the two token halves

        // Pass B over elements 4 q + 2 w, 4 q + 2 w + 1 of one half: u -> weight
        // 2^(u c - ref - kk) * scale, rounded to e4m3 into the lane's B operand (bytes 16 h + 4 q
        // + 2 w, + 1); exact and rounded sums.  sc, rs: the quad's weight scales (prep_rscale) and
        // their reciprocals.
        auto pass_b2 = [&](f32x16& s, auto h_tag, auto q_tag, auto w_tag, uint32_t sbase, uint32_t rbase, float rk,
                           float& lsum, float& lqsum) {
          constexpr int h = decltype(h_tag)::value, q = decltype(q_tag)::value, w = decltype(w_tag)::value;
          const f32x2 sc = tok2(sbase, h, q, w), rs = tok2(rbase, h, q, w);
          const float e0 = __builtin_amdgcn_exp2f(fmaf(s[q * 4 + 2 * w], c_head, -rk));
          const float e1 = __builtin_amdgcn_exp2f(fmaf(s[q * 4 + 2 * w + 1], c_head, -rk));
          lsum += e0 + e1;
          pn[h * 4 + q] = __builtin_amdgcn_cvt_pk_fp8_f32(e0 * sc[0], e1 * sc[1], pn[h * 4 + q], w);
          const f32x2 bk = __builtin_amdgcn_cvt_pk_f32_fp8(pn[h * 4 + q], w);
          lqsum = fmaf(bk[0], rs[0], lqsum);
          lqsum = fmaf(bk[1], rs[1], lqsum);
        };

        // One iteration per tile, 52 MFMAs: S^T of the tile (36; the first half's logits are
        // scaled behind the second half's MFMAs), its softmax, then its PV (16).  The direct loads
        // of tile it+2 go out behind the first MFMAs; the barrier that publishes tile it+1 sits
        // behind PV MFMA 11, and the first K fragments of tile it+1 are requested behind the last
        // four PV MFMAs, so the next iteration starts without waiting on LDS.
        // Operand ring of three fragments: K fragment f (= 9 half + dim block) lives in slot
        // (f + 1) % 3 and is requested behind the second MFMA of fragment f - 3; V^T fragment cb
        // lives in slot cb % 3, requested behind PV MFMA cb - 3.  PV MFMAs 13, 14, 15 free slots
        // 1, 2, 0 in the order the next tile's K fragments 0, 1, 2 take them.
        KAddr ka;
        VAddr va;
        u32x2 e_tab;
        uint32_t e_lo, e_hi;
        {
          wait_tile();  // tile 1 may still be in flight
          __syncthreads();
          ka = k_addr(lds0);
#pragma unroll
          for (int d = 0; d < kRing; ++d) fr[(d + 1) % kRing] = load_k(ka, d);
        }
        e_tab = tile_entry(2);
        e_lo = __builtin_amdgcn_readfirstlane(e_tab.x);
        e_hi = __builtin_amdgcn_readfirstlane(e_tab.y);

        auto body = [&](const int it) {
          const uint32_t st_cur = lds0 + stage_of(it) * kStage8;
          const uint32_t st_next = lds0 + stage_of(it + 1) * kStage8;
          const TileSrc ts = prep_tile_e(it + 2, e_lo, e_hi);
          // validity bits of the lane's 2 x 16 logits (a partial tile: wave-uniform and rare)
          const bool full = *LDS_PTR(uint32_t, lds_tiles + it * 8) & 1;
          uint32_t vb0 = ~0u, vb1 = ~0u;
          if (!full) {
            vb0 = valid_bits(tile_pos(it), 0);
            vb1 = valid_bits(tile_pos(it), 1);
          }
          float mu0 = -INFINITY, mu1 = -INFINITY, ls = 0.f, lq = 0.f, rk0 = 0.f, rk1 = 0.f;
          int es = 0, kk0 = 0, kk1 = 0, pn_s = 127;
          auto sb = [&]() { return scale_base(lds_scales + stage_of(it) * kScale8); };
          auto wb = [&]() { return scale_base(lds_rscale + wave * 2 * kScale8); };
          auto rb = [&]() { return scale_base(lds_rscale + wave * 2 * kScale8 + kScale8); };
          // the half's block exponent (the same in both lanes of a head) and what pass B subtracts
          auto close_half = [&](float& mu, int& kk, float& rk) {
            const float mt = pair_max(fmaf(mu, c_head, -ref));  // -inf stays -inf (c_head > 0)
            kk = block_exp(mt, es);
            rk = ref + (float)kk;
            mt_all = fmaxf(mt_all, mt);
          };
          auto step = [&](auto m_tag) {
            constexpr int m = decltype(m_tag)::value;
            if constexpr (m < kNK) {
              constexpr int f = m / 2, h = f / 9, ks = f % 9, term = m & 1, slot = (f + 1) % kRing;
              f32x16& s = h ? s1 : s0;
              if constexpr (ks == 0 && term == 0) mfma8_s_first(s, fr[slot], qh[0]);
              else if constexpr (term == 0) mfma8_s(s, fr[slot], qh[ks]);
              else mfma8_s_lo(s, fr[slot], ql[ks]);
              if constexpr (term == 1 && f + kRing < 18) fr[slot] = load_k(ka, f + kRing);
            } else {
              constexpr int cb = m - kNK;
              mfma8_o(acc[cb], fr[cb % kRing], pn, pn_s);
              if constexpr (cb + kRing < kNV) fr[cb % kRing] = load_v(va, cb + kRing);
            }
            if constexpr (m == 0) es = prep_rscale(stage_of(it));
            if constexpr (m == 4) e_tab = tile_entry(it + 3);
            // direct loads of tile it+2, one every second MFMA
            if constexpr (m % 2 == 1 && m / 2 < kDmaPerTile) dma_piece(ts, std::integral_constant<int, m / 2>{});
            if constexpr (m == 22) {
              e_lo = __builtin_amdgcn_readfirstlane(e_tab.x);
              e_hi = __builtin_amdgcn_readfirstlane(e_tab.y);
            }
            // ---- softmax of half 0, behind the MFMAs of half 1 (half 0 is complete behind MFMA
            // 17; three 16-pass MFMAs lie between it and the first read) ----
            if constexpr (m == 20) {
              asm volatile("" : "+v"(s0));  // nothing below reads S^T ahead of this point
              pass_a(s0, 0, sb(), 0, 2, vb0, mu0);
            }
            if constexpr (m == 21) pass_a(s0, 0, sb(), 2, 4, vb0, mu0);
            if constexpr (m == 22) {
              // The segment's reference, taken in its first tile from the first 32 positions
              // (selects, no branch): an integer, so that weights computed by different partitions
              // of a sequence differ by exact powers of two.
              {
                const float m2 = pair_max(mu0 * c_head);
                const float r0 = (m2 == -INFINITY || m2 != m2) ? 0.f : ceilf(m2);
                const float r1 = ref_exact == ref_exact ? ref_exact : r0;
                ref = it == 0 ? r1 : ref;
              }
              close_half(mu0, kk0, rk0);
            }
            if constexpr (m >= 23 && m < 31) {
              constexpr int q = (m - 23) / 2, w = (m - 23) & 1;
              pass_b2(s0, std::integral_constant<int, 0>{}, std::integral_constant<int, q>{}, std::integral_constant<int, w>{},
                      wb(), rb(), rk0, ls, lq);
            }
            if constexpr (m == 31) {
              l_run += __builtin_amdgcn_ldexpf(ls, kk0);
              lq_run += __builtin_amdgcn_ldexpf(lq, kk0);
              ls = 0.f;
              lq = 0.f;
            }
            if constexpr (m == kNK - 1) {
              // ---- softmax of half 1, between the two MFMA chains ----
              settle8_s(s1);
              pass_a(s1, 1, sb(), 0, 4, vb1, mu1);
              close_half(mu1, kk1, rk1);
              // the matrix instruction takes the block scale of half g from lane (head, g)
              {
                const int l = fresh_lane();
                pn_s = 127 + (l < 32 ? kk0 : kk1);
              }
              va = v_addr(st_cur);
#pragma unroll
              for (int d = 0; d < kRing; ++d) fr[d] = load_v(va, d);
              [&]<int... E>(std::integer_sequence<int, E...>) {
                (([&] {
                   constexpr int q = E / 2, w = E & 1;
                   pass_b2(s1, std::integral_constant<int, 1>{}, std::integral_constant<int, q>{},
                           std::integral_constant<int, w>{}, wb(), rb(), rk1, ls, lq);
                 }()),
                 ...);
              }(std::make_integer_sequence<int, 8>{});
              l_run += __builtin_amdgcn_ldexpf(ls, kk1);
              lq_run += __builtin_amdgcn_ldexpf(lq, kk1);
            }
            if constexpr (m == kNK + 12) {
              // Tile it+1 becomes visible, and every wave is done with tile it (its last V^T
              // fragments were requested behind PV MFMA 11; the barrier's fence waits for them)
              wait_tile();
              __syncthreads();
              ka = k_addr(st_next);
            }
            // K fragments 0 .. 2 of tile it+1 into slots 1, 2, 0 as the last PV MFMAs free them
            if constexpr (m >= kNK + 13) {
              constexpr int f = m - (kNK + 13);
              fr[(f + 1) % kRing] = load_k(ka, f);
            }
            // what was written behind this MFMA stays behind it: the scheduler otherwise gathers
            // the arithmetic of many steps in front of one MFMA and the matrix pipeline drains
            __builtin_amdgcn_sched_barrier(0);
          };
          [&]<int... M>(std::integer_sequence<int, M...>) {
            (step(std::integral_constant<int, M>{}), ...);
          }(std::make_integer_sequence<int, kNK + kNV>{});
        };
#pragma unroll 1
        for (int it = 0; it < n_tiles; ++it) body(it);
        settle8_o(acc);
      }
      wait_vm<0>();  // the void loads issued for tiles past the end

      const float m2 = fmaxf(mt_all, __shfl_xor(mt_all, 32));
      const bool off = m2 > kRefSlack8 || (m2 < -kRefSlack8 && m2 != -INFINITY);
      if (attempt == 0 && __any(off) && (tid & 63) == 0) *LDS_PTR(int, lds_flag) = 1;
      __syncthreads();  // also: all reads of the stages are done before they are reused
      if (*LDS_PTR(int, lds_flag) == 0) break;
      ref_exact = m2 == -INFINITY ? 0.f : ref + ceilf(m2);
    }

    // ---- epilogue: normalise by the rounded weights' sum, transpose through LDS, write rows ----
    l_run += __shfl_xor(l_run, 32);
    lq_run += __shfl_xor(lq_run, 32);
    const float inv = (n_tiles > 0 && lq_run != 0.f) ? 1.0f / lq_run : 0.f;
    const float lse = n_tiles > 0 ? (ref + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
    const bool final_out = sg.slot < 0;
    const uint32_t ost = lds0 + wave * kOutWaveBytes8;
    const int heads_here = p.H - h0 < kHeadsPerWave ? p.H - h0 : kHeadsPerWave;
    const int lane_e = fresh_lane();
    const int n32e = lane_e & 31, ge = lane_e >> 5;
    if (n32e < heads_here && ge == 0) {
      if (final_out) p.lse[(size_t)sg.b * p.H + h0 + n32e] = lse;
      else p.part_lse[(size_t)sg.slot * p.head_block + wave * kHeadsPerWave + n32e] = lse;
    }
    const size_t row0 = final_out ? (size_t)sg.b * p.H + h0
                                  : (size_t)sg.slot * p.head_block + wave * kHeadsPerWave;
    if (!p.out_fp32) {
#pragma unroll
      for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          bf16x4 v = {(__bf16)(acc[cb][i4 * 4] * inv), (__bf16)(acc[cb][i4 * 4 + 1] * inv),
                      (__bf16)(acc[cb][i4 * 4 + 2] * inv), (__bf16)(acc[cb][i4 * 4 + 3] * inv)};
          *LDS_PTR(bf16x4, ost + n32e * kOutRowBytes8 + (cb * 32 + i4 * 8 + ge * 4) * 2) = v;
        }
      uint8_t* dst = (uint8_t*)(final_out ? p.out : p.part_o) + row0 * (kV * 2) + lane_e * 16;
#pragma unroll 4
      for (int h = 0; h < heads_here; ++h)
        *(u32x4*)(dst + (size_t)h * (kV * 2)) = *LDS_PTR(u32x4, ost + h * kOutRowBytes8 + lane_e * 16);
    } else {
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
            *LDS_PTR(f32x4, ost + n32e * kOutRowBytes8 + (cb8 * 32 + i4 * 8 + ge * 4) * 4) = v;
          }
#pragma unroll 4
        for (int h = 0; h < heads_here; ++h)
          *(u32x4*)(dst + (size_t)h * (kV * 4) + r * 1024) =
              *LDS_PTR(u32x4, ost + h * kOutRowBytes8 + lane_e * 16);
      }
    }
    __syncthreads();
  }
}

hipError_t init_fp8_kernel() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_fp8_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kLds8);
}

hipError_t launch_decode_fp8(const DecodeParams& p, int n_units, hipStream_t stream) {
  if (n_units <= 0) return hipSuccess;
  if (p.xcds < 1) return hipErrorInvalidValue;
  dim3 grid(((n_units + p.xcds - 1) / p.xcds) * p.xcds), block(kWaves8 * 64);
  hipLaunchKernelGGL(decode_fp8_kernel, grid, block, kLds8, stream, p);
  return hipGetLastError();
}

}  // namespace omniattn
