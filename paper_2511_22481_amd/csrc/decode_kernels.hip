// gfx950 kernels for sparse MLA decode over the OmniAttn retained set
// (paper section 3.2.1: softmax(q K_M^T * scale) V_M with M = sinks + recents).
//
// Main kernel, one work group per work unit, WAVES waves, each wave owning 32
// heads and the full 512-wide output of those heads:
//   a3  retained 64-token tile -> LDS by direct global->LDS 16-byte loads
//       (double buffered), rows XOR-swizzled so that both later read patterns
//       are bank-conflict free;
//   a4  S^T[token, head] = K_tile . Q^T on 32x32x16 bf16 MFMA, Q held in
//       registers as the B operand for the whole segment;
//   a5  positions outside the retained set get -inf (partial tiles only);
//   a6  online softmax per head: a lane holds 16 tokens of one head per
//       32-token block, its partner lane (lane ^ 32) the other 16;
//   a7  O^T[col, head] += V^T . P^T on the same MFMA; the C layout of S^T is
//       exactly the B layout P^T needs, so P never leaves registers; V^T comes
//       from the same LDS tile through transposing LDS reads;
//   a8  normalise, write bf16/fp32 output + lse, or an fp32 partial.
// Combine kernel (a9): merges the partials of sequences that were split.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernels.h"

namespace omniattn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_PTR(T, byte_off) ((__attribute__((address_space(3))) T*)(uintptr_t)(byte_off))

constexpr int kRowBytes = kQK * 2;            // one token row in LDS (bf16)
constexpr int kChunksPerRow = kRowBytes / 16; // 72
constexpr int kTileBytes = kTile * kRowBytes; // 73,728
constexpr int kScaleBytes = kTile * 4;        // per-token fp32 scales of one tile (fp8 cache)
constexpr int kLdsBytes = 2 * kTileBytes + 2 * kScaleBytes + 16;  // + redo flag

// LDS layout of one 64-token tile (73,728 bytes).  A token row is 72 chunks of
// 16 bytes: chunks 0..63 (the 512 value dims) and 64..71 (the 64 rope dims).
//   main part: row r at r * 1024; chunk c < 64 sits at position c ^ swz_main(r)
//   tail part: at kTailBase + r * 128; chunk 64 + c sits at position c ^ swz_tail(r)
// Splitting the row this way makes one direct global->LDS load instruction
// (64 lanes x 16 bytes = 1024 contiguous LDS bytes) fill exactly one main row,
// so a lane's global offset is a lane constant plus a per-instruction constant.
// The XOR swizzles make both read patterns bank-conflict free: 16 consecutive
// rows at one chunk index (A-operand gather of K rows) land in 16 different
// 16-byte bank groups, and 4 consecutive rows x 64 bytes (one transposing read
// of V) land in the four quarters of the 64 banks.
constexpr int kMainRowBytes = 1024;
constexpr int kTailRowBytes = 128;
constexpr int kTailBase = kTile * kMainRowBytes;  // 65,536
__host__ __device__ constexpr int swz_main(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
__host__ __device__ constexpr int swz_tail(int r) { return (r >> 1) & 7; }
// byte offset of chunk c (0..71) of row r inside a tile buffer
__device__ __forceinline__ uint32_t lds_chunk(int r, int c) {
  return c < 64 ? r * kMainRowBytes + ((c ^ swz_main(r)) << 4)
                : kTailBase + r * kTailRowBytes + (((c - 64) ^ swz_tail(r)) << 4);
}

__device__ __forceinline__ bool retained(int j, int L, int S, int W) {
  return j < L && (j < S || j >= L - W);
}

// Register files.  At one wave per SIMD a wave has 256 vector registers and 256
// accumulation registers.  The O^T tile (512 columns x 32 heads, fp32) fills the
// accumulation file exactly; Q (144 registers), S, P and operand fragments live in
// the vector file.  The MFMAs are written as assembly because only the assembly
// form lets the destination register file be chosen per instruction: S must not
// land in the accumulation file and O^T must never leave it.  Wait states the
// hardware does not interlock are supplied by hand: back-to-back MFMAs that
// accumulate into the same registers need none; a vector-ALU read of the result
// of an 8-pass MFMA needs 12 (settle()).
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
__device__ __forceinline__ void settle_o(f32x16& acc) { asm volatile("s_nop 11" : "+a"(acc)); }

// Softmax reference.  exp2(x - r) is evaluated against a per-head reference r
// that is fixed for a whole segment (the maximum of the segment's first 32-token
// block), not against a running maximum: softmax is invariant to r, so the only
// requirement is that exp2 does not overflow.  That removes every rescaling of
// the 256-register O^T tile from the loop.  If a later logit exceeds r by more
// than kRefSlack (2^64 headroom below fp32/bf16 overflow even after summing a
// million terms) the segment is redone once with r = its exact maximum, found
// by a QK-only pass.
constexpr float kRefSlack = 64.f;

template <int WAVES, bool FP8>
__global__ __launch_bounds__(WAVES * 64, 1) void decode_kernel(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds_raw;  // LDS byte address of buffer 0
  const uint32_t lds_scales = lds0 + 2 * kTileBytes;
  const uint32_t lds_flag = lds_scales + 2 * kScaleBytes;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int n32 = lane & 31;  // head within the wave's 32 (B / C column)
  const int g = lane >> 5;    // k-group of the MFMA operands

  // ---- per-lane LDS read offsets (relative to a tile buffer) ----
  // QK^T A operand: token row n32 (+32 per block), chunk 2 ks + g.  For ks < 32 the
  // chunk position is ((2 (ks & 7) + g) ^ swz) + 16 (ks >> 3); since 2 (ks & 7) has
  // bit 0 clear, the byte offset is a_main ^ ((ks & 7) << 5) plus a constant.
  const uint32_t a_main = n32 * kMainRowBytes + ((g ^ swz_main(n32)) << 4);
  const uint32_t a_tail = kTailBase + n32 * kTailRowBytes + ((g ^ swz_tail(n32)) << 4);
  // PV A operand (V^T): each 16-lane group reads a 4-token x 16-column block transposed.
  // Lane row = 16 th + 8 hi + 4 g + (i16 >> 2); chunk = 4 cb + c_lane.
  const int i16 = lane & 15;
  const int c_lane = ((lane >> 4) & 1) * 2 + ((i16 & 3) >> 1);
  const int half8 = (i16 & 1) * 8;
  uint32_t v_off[2][4];  // [upper k-slots][cb & 3]; add (cb >> 2) * 256 + th * 16 rows
#pragma unroll
  for (int hi = 0; hi < 2; ++hi) {
    const int r = hi * 8 + g * 4 + (i16 >> 2);
#pragma unroll
    for (int cl = 0; cl < 4; ++cl)
      v_off[hi][cl] = r * kMainRowBytes + (((cl * 4 + c_lane) ^ swz_main(r)) << 4) + half8;
  }

  const int unit = blockIdx.x;
  const int seg_lo = p.unit_seg[unit], seg_hi = p.unit_seg[unit + 1];

  for (int si = seg_lo; si < seg_hi; ++si) {
    const Segment sg = p.segs[si];
    const int L = sg.L;
    const int h0 = sg.hb * p.head_block + wave * kHeadsPerWave;  // wave's first head
    const int head = h0 + n32;
    const bool head_ok = head < p.H;
    const TileLayout tl = tile_layout(L, p.S, p.W);
    const int n_tiles = sg.tile_hi - sg.tile_lo;
    const int sink_end = p.S < L ? p.S : L;

    // ---- Q fragments: B operand, lane (head n32, g) holds d = 16 ks + 8 g .. + 8 ----
    bf16x8 qf[kQK / 16];
    {
      // heads past H (a partly filled wave) read the last real head; their results are never written
      const uint16_t* qrow = p.q + ((size_t)sg.b * p.H + (head_ok ? head : p.H - 1)) * kQK + g * 8;
#pragma unroll
      for (int ks = 0; ks < kQK / 16; ++ks)
        qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + ks * 16));
    }

    // ---- tile loader: wave w fills its share of the tile's rows ----
    auto issue_tile = [&](int ti, int buf) {
      const int pos0 = tl.logical(ti) * kTile;
      const int page = p.page_table[(size_t)sg.b * p.max_pages + (pos0 >> 7)];
      const int slot0 = pos0 & (kPage - 1);
      const bool full = (pos0 + kTile <= sink_end) || (pos0 >= L - p.W && pos0 + kTile <= L);
      const uint32_t lbase = lds0 + buf * kTileBytes;
      if constexpr (!FP8) {
        const uint8_t* gbase = p.kv + ((size_t)page * kPage + slot0) * kRowBytes;
        constexpr int rows_per_wave = kTile / WAVES;  // 16, 32 or 64: a multiple of 16
        const int row_w0 = wave * rows_per_wave;
        if (full) {
          // The per-lane offsets below are loop invariant; recomputing them (an XOR and a
          // shift) is cheaper than keeping 18 of them alive across the MFMA loops, so the
          // lane id is passed through an opaque move that stops the compiler hoisting them.
          uint32_t l = lane;
          asm volatile("" : "+v"(l));
          // main part: one instruction per row; lane l fetches chunk l ^ swz_main(row)
#pragma unroll
          for (int j = 0; j < rows_per_wave; ++j) {
            const int row = row_w0 + j;
            const uint32_t off = row * kRowBytes + ((l ^ swz_main(j)) << 4);
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)(gbase + off),
                (void __attribute__((address_space(3)))*)(uintptr_t)(lbase + row * kMainRowBytes),
                16, 0, 0);
          }
          // tail part: one instruction per 8 rows; lane l fetches row l / 8, rope chunk (l & 7) ^ swz
#pragma unroll
          for (int k = 0; k < rows_per_wave / 8; ++k) {
            const uint32_t r8 = 8 * k + (l >> 3);  // row within the wave's share (row_w0 is a multiple of 16)
            const uint32_t off = (row_w0 + r8) * kRowBytes + ((64 + ((l & 7) ^ swz_tail(r8))) << 4);
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)(gbase + off),
                (void __attribute__((address_space(3)))*)(uintptr_t)(lbase + kTailBase +
                                                                     (row_w0 + 8 * k) * kTailRowBytes),
                16, 0, 0);
          }
        } else {
          // partial tile: rows outside the retained set are zero-filled, never loaded
          // (their contents are unspecified and 0 * NaN would poison the PV product)
#pragma unroll 1
          for (int ci = lane; ci < rows_per_wave * kChunksPerRow; ci += 64) {
            const int r = ci / kChunksPerRow;
            const int c = ci - r * kChunksPerRow;
            const int row = row_w0 + r;
            u32x4 v = {0, 0, 0, 0};
            if (retained(pos0 + row, L, p.S, p.W)) v = *(const u32x4*)(gbase + row * kRowBytes + (c << 4));
            *LDS_PTR(u32x4, lbase + lds_chunk(row, c)) = v;
          }
        }
      } else {
        // fp8 rows: 36 chunks of 16 codes; widen each code exactly to bf16, keep the
        // per-token scale aside (it multiplies the logit and the softmax weight).
        const uint8_t* gbase = p.kv + ((size_t)page * kPage + slot0) * kQK;
        constexpr int n_chunks = kTile * (kQK / 16);  // 2304
#pragma unroll 1
        for (int c0 = 0; c0 < n_chunks; c0 += WAVES * 64 * 3) {
          u32x4 raw[3];
#pragma unroll
          for (int u = 0; u < 3; ++u) {
            int ci = c0 + u * WAVES * 64 + tid;
            int row = ci / (kQK / 16);
            int cc = ci - row * (kQK / 16);
            raw[u] = u32x4{0, 0, 0, 0};
            if (full || retained(pos0 + row, L, p.S, p.W))
              raw[u] = *(const u32x4*)(gbase + row * kQK + cc * 16);
          }
#pragma unroll
          for (int u = 0; u < 3; ++u) {
            int ci = c0 + u * WAVES * 64 + tid;
            int row = ci / (kQK / 16);
            int cc = ci - row * (kQK / 16);
            uint32_t w[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(raw[u][k], false);
              f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(raw[u][k], true);
              bf16x2 blo = {(__bf16)lo.x, (__bf16)lo.y};
              bf16x2 bhi = {(__bf16)hi.x, (__bf16)hi.y};
              w[2 * k] = __builtin_bit_cast(uint32_t, blo);
              w[2 * k + 1] = __builtin_bit_cast(uint32_t, bhi);
            }
            *LDS_PTR(u32x4, lbase + lds_chunk(row, 2 * cc)) = u32x4{w[0], w[1], w[2], w[3]};
            *LDS_PTR(u32x4, lbase + lds_chunk(row, 2 * cc + 1)) = u32x4{w[4], w[5], w[6], w[7]};
          }
        }
        if (tid < kTile) {
          bool ok = full || retained(pos0 + tid, L, p.S, p.W);
          float sc = ok ? p.kv_scales[(size_t)page * kPage + slot0 + tid] : 0.f;
          *LDS_PTR(float, lds_scales + buf * kScaleBytes + tid * 4) = sc;
        }
      }
    };

    // One pass over the segment's tiles.  MAX_ONLY: only the per-head maximum of the
    // logits (log2 domain) is formed; otherwise the full softmax-weighted sum.
    f32x16 acc[kV / 32];
    float ref = 0.f, l_run = 0.f;
    bool overflow = false;

    auto run_pass = [&](auto max_only_tag, float ref_in) -> float {
      constexpr bool MAX_ONLY = decltype(max_only_tag)::value;
      float mx_all = -INFINITY;
      bool have_ref = !MAX_ONLY && ref_in == ref_in;  // NaN = choose from the first block
      ref = have_ref ? ref_in : 0.f;
      l_run = 0.f;
      overflow = false;
      if constexpr (!MAX_ONLY) {
#pragma unroll
        for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
      }
      if (n_tiles > 0) issue_tile(sg.tile_lo, 0);
#pragma unroll 1
      for (int it = 0; it < n_tiles; ++it) {
        const int buf = it & 1;
        const int ti = sg.tile_lo + it;
        __builtin_amdgcn_s_waitcnt(0);  // my loads / LDS writes for this tile are done
        __syncthreads();                // everyone's are; everyone finished reading the other buffer
        if (it + 1 < n_tiles) issue_tile(ti + 1, buf ^ 1);

        const uint32_t tb_base = lds0 + buf * kTileBytes;
        const int pos0 = tl.logical(ti) * kTile;
        const bool full = (pos0 + kTile <= sink_end) || (pos0 >= L - p.W && pos0 + kTile <= L);

        // The MFMAs are volatile assembly, which the scheduler does not move loads
        // across, so the LDS reads are software-pipelined by hand: each fragment is
        // requested kDepth MFMAs ahead of its use.
        auto load_k = [&](int tb, int ks) -> bf16x8 {
          if (ks < 32)
            return *LDS_PTR(bf16x8, tb_base + (a_main ^ ((ks & 7) << 5)) + (ks >> 3) * 256 +
                                        tb * 32 * kMainRowBytes);
          return *LDS_PTR(bf16x8, tb_base + (a_tail ^ ((ks - 32) << 5)) + tb * 32 * kTailRowBytes);
        };
        auto load_v = [&](int tb, int j) -> bf16x8 {  // j = th * 16 + cb
          const int th = j >> 4, cb = j & 15;
          const uint32_t base = tb_base + (tb * 32 + th * 16) * kMainRowBytes + (cb >> 2) * 256;
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, base + v_off[0][cb & 3]));
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, base + v_off[1][cb & 3]));
          return __builtin_bit_cast(
              bf16x8, (__attribute__((ext_vector_type(8))) short){lo[0], lo[1], lo[2], lo[3], hi[0],
                                                                  hi[1], hi[2], hi[3]});
        };
        constexpr int kDepth = 6;
        constexpr int kNK = kQK / 16;  // 36 MFMAs for S^T
        constexpr int kNV = 2 * (kV / 32);  // 32 MFMAs for O^T

#pragma unroll 1
        for (int tb = 0; tb < kTile / 32; ++tb) {
          bf16x8 kf[kDepth], vf[kDepth];
#pragma unroll
          for (int d = 0; d < kDepth; ++d) kf[d] = load_k(tb, d);

          // ---- S^T = K . Q^T ----
          f32x16 s;
#pragma unroll
          for (int ks = 0; ks < kNK; ++ks) {
            if (ks == 0) mfma_s_first(s, kf[ks % kDepth], qf[ks]);
            else mfma_s(s, kf[ks % kDepth], qf[ks]);
            if (ks + kDepth < kNK) kf[ks % kDepth] = load_k(tb, ks + kDepth);
            else if constexpr (!MAX_ONLY) vf[(ks + kDepth - kNK) % kDepth] = load_v(tb, ks + kDepth - kNK);
          }
          settle_s(s);

          // ---- logits in the log2 domain, per-token scale (fp8), mask ----
          // element i is token tb*32 + (i/4)*8 + g*4 + i%4 of the tile
          const uint32_t sc_base = lds_scales + buf * kScaleBytes + (tb * 32 + g * 4) * 4;
          float mx = -INFINITY;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float x = s[i] * p.scale_log2;
            if constexpr (FP8) x *= *LDS_PTR(float, sc_base + ((i >> 2) * 8 + (i & 3)) * 4);
            if (!full) {
              const int tok = tb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
              if (!retained(pos0 + tok, L, p.S, p.W)) x = -INFINITY;
            }
            s[i] = x;
            mx = fmaxf(mx, x);
          }
          if constexpr (MAX_ONLY) {
            mx_all = fmaxf(mx_all, mx);
            continue;
          }
          if (!have_ref) {  // wave-uniform: first block of the pass
            float m2 = fmaxf(mx, __shfl_xor(mx, 32));
            // a block may hold no retained token (its tile still does): wait for a finite maximum
            if (__any(m2 != -INFINITY)) {
              ref = m2 == -INFINITY ? 0.f : m2;
              have_ref = true;
            }
          }
          overflow |= __any(mx - ref > kRefSlack) != 0;

          bf16x8 pf[2];
          float lsum = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float e = __builtin_amdgcn_exp2f(s[i] - ref);
            lsum += e;
            if constexpr (FP8) e *= *LDS_PTR(float, sc_base + ((i >> 2) * 8 + (i & 3)) * 4);
            pf[i >> 3][i & 7] = (__bf16)e;
          }
          l_run += lsum;

          // ---- O^T += V^T . P^T ----
#pragma unroll
          for (int j = 0; j < kNV; ++j) {
            mfma_o(acc[j & 15], vf[j % kDepth], pf[j >> 4]);
            if (j + kDepth < kNV) vf[j % kDepth] = load_v(tb, j + kDepth);
          }
        }
      }
      __syncthreads();  // all reads of both buffers are done before anyone reuses them
      return mx_all;
    };

    run_pass(std::false_type{}, __builtin_nanf(""));
    // Did any wave see a logit too far above its reference?  Then redo with the exact maximum.
    if (tid == 0) *LDS_PTR(int, lds_flag) = 0;
    __syncthreads();
    if (overflow && lane == 0) *LDS_PTR(int, lds_flag) = 1;
    __syncthreads();
    if (*LDS_PTR(int, lds_flag) != 0) {
      float m = run_pass(std::true_type{}, 0.f);
      m = fmaxf(m, __shfl_xor(m, 32));
      run_pass(std::false_type{}, m == -INFINITY ? 0.f : m);
    }

    // ---- epilogue ----
#pragma unroll
    for (int cb = 0; cb < kV / 32; ++cb) settle_o(acc[cb]);
    l_run += __shfl_xor(l_run, 32);
    const float inv = n_tiles > 0 ? 1.0f / l_run : 0.f;
    const float lse = n_tiles > 0 ? (ref + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
    if (head_ok) {
      if (sg.slot < 0) {
        if (g == 0) p.lse[(size_t)sg.b * p.H + head] = lse;
        if (p.out_fp32) {
          float* o = (float*)p.out + ((size_t)sg.b * p.H + head) * kV;
#pragma unroll
          for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              f32x4 v = {acc[cb][i4 * 4] * inv, acc[cb][i4 * 4 + 1] * inv, acc[cb][i4 * 4 + 2] * inv,
                         acc[cb][i4 * 4 + 3] * inv};
              *(f32x4*)(o + cb * 32 + i4 * 8 + g * 4) = v;
            }
        } else {
          uint16_t* o = (uint16_t*)p.out + ((size_t)sg.b * p.H + head) * kV;
#pragma unroll
          for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              bf16x4 v = {(__bf16)(acc[cb][i4 * 4] * inv), (__bf16)(acc[cb][i4 * 4 + 1] * inv),
                          (__bf16)(acc[cb][i4 * 4 + 2] * inv), (__bf16)(acc[cb][i4 * 4 + 3] * inv)};
              *(bf16x4*)(o + cb * 32 + i4 * 8 + g * 4) = v;
            }
        }
      } else {
        const int hl = wave * kHeadsPerWave + n32;  // head within the block
        if (g == 0) p.part_lse[(size_t)sg.slot * p.head_block + hl] = lse;
        float* o = p.part_o + ((size_t)sg.slot * p.head_block + hl) * kV;
#pragma unroll
        for (int cb = 0; cb < kV / 32; ++cb)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            f32x4 v = {acc[cb][i4 * 4] * inv, acc[cb][i4 * 4 + 1] * inv, acc[cb][i4 * 4 + 2] * inv,
                       acc[cb][i4 * 4 + 3] * inv};
            *(f32x4*)(o + cb * 32 + i4 * 8 + g * 4) = v;
          }
      }
    }
  }
}

// Merge the partial results of one (sequence, head block): out = sum_s w_s O_s with
// w_s = exp(lse_s - lse), lse = log sum_s exp(lse_s).  One work group per
// (combine item, group of 4 heads); 64 lanes x 8 columns cover one head row.
__global__ __launch_bounds__(256) void combine_kernel(CombineParams p) {
  const CombineItem it = p.items[blockIdx.x];
  const int hl = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int head = it.hb * p.head_block + hl;
  if (hl >= p.head_block || head >= p.H) return;
  const int lane = threadIdx.x & 63;
  float m = -INFINITY;
  for (int s = 0; s < it.nslots; ++s)
    m = fmaxf(m, p.part_lse[(size_t)(it.slot0 + s) * p.head_block + hl]);
  float z = 0.f;
  for (int s = 0; s < it.nslots; ++s)
    z += expf(p.part_lse[(size_t)(it.slot0 + s) * p.head_block + hl] - m);
  const float tot = m + logf(z);
  float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int s = 0; s < it.nslots; ++s) {
    const size_t row = (size_t)(it.slot0 + s) * p.head_block + hl;
    const float w = expf(p.part_lse[row] - tot);
    const f32x4* src = (const f32x4*)(p.part_o + row * kV + lane * 8);
    f32x4 a = src[0], b = src[1];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      o[k] += w * a[k];
      o[4 + k] += w * b[k];
    }
  }
  const size_t orow = (size_t)it.b * p.H + head;
  if (lane == 0) p.lse[orow] = tot;
  if (p.out_fp32) {
    float* dst = (float*)p.out + orow * kV + lane * 8;
    *(f32x4*)dst = f32x4{o[0], o[1], o[2], o[3]};
    *(f32x4*)(dst + 4) = f32x4{o[4], o[5], o[6], o[7]};
  } else {
    bf16x8 v;
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = (__bf16)o[k];
    *(bf16x8*)((uint16_t*)p.out + orow * kV + lane * 8) = v;
  }
}


template <int WAVES, bool FP8>
static hipError_t set_lds_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<WAVES, FP8>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

hipError_t init_kernels() {
  hipError_t e;
  if ((e = set_lds_attr<1, false>()) != hipSuccess) return e;
  if ((e = set_lds_attr<2, false>()) != hipSuccess) return e;
  if ((e = set_lds_attr<4, false>()) != hipSuccess) return e;
  if ((e = set_lds_attr<1, true>()) != hipSuccess) return e;
  if ((e = set_lds_attr<2, true>()) != hipSuccess) return e;
  if ((e = set_lds_attr<4, true>()) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_decode(const DecodeParams& p, int waves, bool fp8, int n_units, hipStream_t stream) {
  if (n_units <= 0) return hipSuccess;
  dim3 grid(n_units), block(waves * 64);
#define OA_LAUNCH(W, F) \
  hipLaunchKernelGGL((decode_kernel<W, F>), grid, block, kLdsBytes, stream, p)
  if (!fp8) {
    if (waves == 4) OA_LAUNCH(4, false);
    else if (waves == 2) OA_LAUNCH(2, false);
    else if (waves == 1) OA_LAUNCH(1, false);
    else return hipErrorInvalidValue;
  } else {
    if (waves == 4) OA_LAUNCH(4, true);
    else if (waves == 2) OA_LAUNCH(2, true);
    else if (waves == 1) OA_LAUNCH(1, true);
    else return hipErrorInvalidValue;
  }
#undef OA_LAUNCH
  return hipGetLastError();
}

hipError_t launch_combine(const CombineParams& p, int n_items, hipStream_t stream) {
  if (n_items <= 0) return hipSuccess;
  dim3 grid(n_items, (p.head_block + 3) / 4), block(256);
  hipLaunchKernelGGL(combine_kernel, grid, block, 0, stream, p);
  return hipGetLastError();
}

}  // namespace omniattn
