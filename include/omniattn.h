/*
 * omniattn.h - C ABI of the MI355X (gfx950) sparse MLA decode library.
 *
 * One operation: decode-phase attention for absorbed multi-head latent
 * attention, restricted to the KV positions that OmniAttn's cache-compression
 * rule keeps.  For sequence b of length L_b the kept set is the first S
 * ("sink") positions and the last W ("recent") positions, as a set union
 * clipped to [0, L_b) (paper section 3.2.1, second equation, 0-based here),
 * and the result is softmax(q K_M^T * scale) V_M over that set (left-hand side
 * of the first equation of 3.2.1).  One (S, W) applies to every head of the
 * call (section 3.2.2: the layer, not the head, is the unit of compression).
 *
 * MLA layout (the paper only names MLA as compatible; shapes are the
 * DeepSeek-R1 absorbed decode form): each cached token is one latent row of
 * 576 numbers; the key is the whole row, the value is its first 512 numbers;
 * queries arrive already multiplied by the key up-projection.
 *
 * Conventions
 *   - All data pointers marked "device" are HIP device pointers owned by the
 *     caller; "host" pointers are ordinary memory.  The library owns only the
 *     plan object and the small device metadata it uploads for it.
 *   - `hip_stream` is a hipStream_t cast to void* (NULL = the null stream).
 *   - Every function returns 0 on success or a negative OMNIATTN_E* code.
 *     Nothing aborts and no C++ exception crosses this boundary.
 *   - The library is a HIP library: there is no CPU fallback.  On a machine
 *     without a usable GPU, omniattn_plan() and omniattn_decode() fail with
 *     OMNIATTN_EHIP; only the host-side planner (omniattn_plan_host) works.
 */
#ifndef OMNIATTN_H
#define OMNIATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OMNIATTN_QK_DIM 576
#define OMNIATTN_V_DIM 512
#define OMNIATTN_PAGE 128

enum { OMNIATTN_BF16 = 0, OMNIATTN_FP8_E4M3 = 1, OMNIATTN_FP32 = 2 };

enum {
  OMNIATTN_OK = 0,
  OMNIATTN_EINVAL = -1,       /* null pointer, bad shape, bad size            */
  OMNIATTN_EUNSUPPORTED = -2, /* dtype / head count / dims not supported      */
  OMNIATTN_EWORKSPACE = -3,   /* workspace missing or too small               */
  OMNIATTN_EHIP = -4,         /* a HIP call failed; see omniattn_last_hip_error */
  OMNIATTN_ENOMEM = -5,       /* host allocation failed                       */
  OMNIATTN_ESCRATCH = -6      /* plan too large for omniattn_decode_static    */
};

/* Size of the library-owned device buffer omniattn_decode_static works in. */
#define OMNIATTN_STATIC_SCRATCH_BYTES (40u << 20)

/* Statement of one decode problem.  Fixed by the plan; the tensors come later. */
typedef struct {
  int32_t batch;             /* B >= 1 sequences                                        */
  int32_t num_heads;         /* H >= 1 query heads sharing each sequence's latent cache */
  int32_t qk_dim;            /* must be 576                                             */
  int32_t v_dim;             /* must be 512 (value = first 512 numbers of a cache row)  */
  int32_t page_size;         /* must be 128 tokens                                      */
  int32_t max_pages_per_seq; /* row stride of page_table, in int32 elements             */
  int64_t num_pages;         /* pages in the pool (for validation of host inputs only)  */
  int32_t sink;              /* S = N_sink  >= 0                                        */
  int32_t window;            /* W = N_recent >= 0; S + W >= L_b means dense attention   */
  float softmax_scale;       /* multiplies q.k before the softmax                       */
  int32_t kv_dtype;          /* OMNIATTN_BF16 | OMNIATTN_FP8_E4M3 (OCP e4m3, finite-only;
                                one fp32 scale per token multiplies the whole row)      */
  int32_t out_dtype;         /* OMNIATTN_BF16 | OMNIATTN_FP32                           */
  int32_t num_splits_hint;   /* 0: the library balances work over the GPU's compute
                                units.  n > 0: every sequence's retained tiles are cut
                                into min(n, tiles) pieces (for tests of the split path) */
  int32_t q_len;             /* queries per sequence (the query matrix of the first equation
                                of 3.2.1 has K rows); 0 or 1: one.  T > 1: the queries are
                                the last T tokens of the sequence (all already in the cache
                                and counted in L_b >= T), query t = 0 .. T-1 sits at position
                                L_b - T + t and sees the keys before and at it: the kept-set
                                rule is applied to a sequence of length L_b - (T - 1 - t).
                                q, out and lse then carry [B, T, H, ...] (query-major)    */
} omniattn_problem_t;

typedef struct omniattn_plan_s omniattn_plan_t; /* opaque, library-owned */

/*
 * Steps a1/a2 of the path: build the retained ranges of every sequence (second
 * equation of 3.2.1), cut them into KV tiles, partition tiles into work units
 * and size the workspace.  `seq_lens_host` is a host array of B context
 * lengths L_b >= 0 (the token being decoded is already in the cache and is
 * counted).  Requires ceil(L_b/128) <= max_pages_per_seq.
 *
 * omniattn_plan      also copies the metadata to the current HIP device so that
 *                    omniattn_decode can run: device and pinned host buffers are
 *                    allocated here (hipMalloc, hipHostMalloc), the copy itself is
 *                    asynchronous on `hip_stream`, and decodes of this plan must be
 *                    ordered after it (same stream, or an event).  Work is balanced
 *                    over that device's CU count.
 * omniattn_plan_update  plans again for new lengths of the same problem (every decode
 *                    step changes every L_b) into the same object: host work, one
 *                    asynchronous copy from the plan's pinned buffer and one small
 *                    kernel on `hip_stream`; nothing is allocated and nothing
 *                    synchronises unless the new plan needs more metadata than any
 *                    before it.  The plan must not be in use by a decode on another
 *                    stream.  The workspace size may change: ask again.  On failure
 *                    for bad lengths the plan is unchanged.  A plan made by
 *                    omniattn_plan_host is planned again on the host only.
 * omniattn_plan_host builds the same plan for `num_cus` compute units without
 *                    touching HIP; such a plan can be inspected but
 *                    omniattn_decode on it returns OMNIATTN_EINVAL.
 * On failure *plan_out is set to NULL.
 */
int omniattn_plan(omniattn_plan_t** plan_out, const omniattn_problem_t* prob,
                  const int32_t* seq_lens_host, void* hip_stream);
int omniattn_plan_update(omniattn_plan_t* plan, const int32_t* seq_lens_host, void* hip_stream);
int omniattn_plan_host(omniattn_plan_t** plan_out, const omniattn_problem_t* prob,
                       const int32_t* seq_lens_host, int32_t num_cus);
void omniattn_plan_destroy(omniattn_plan_t* plan); /* NULL is allowed */

/* Introspection (host only, cheap). */
size_t omniattn_plan_workspace_bytes(const omniattn_plan_t* plan); /* may be 0 */
int64_t omniattn_plan_retained_tokens(const omniattn_plan_t* plan); /* sum_b |M_b| */
int32_t omniattn_plan_num_units(const omniattn_plan_t* plan);      /* grid of the main kernel */
int32_t omniattn_plan_num_segments(const omniattn_plan_t* plan);
int32_t omniattn_plan_num_partials(const omniattn_plan_t* plan);   /* partial results the combine kernel merges */
int32_t omniattn_plan_max_splits(const omniattn_plan_t* plan);     /* most pieces any one sequence was cut into */
int32_t omniattn_plan_num_splits(const omniattn_plan_t* plan);     /* the same number under its other name */
int32_t omniattn_plan_tile_tokens(const omniattn_plan_t* plan);    /* KV tokens per tile */
int32_t omniattn_plan_head_block(const omniattn_plan_t* plan);     /* heads per work unit */

/*
 * Copy out the plan's segments, 8 int32 each:
 *   [0] sequence b          [1] head block index     [2] first tile  [3] end tile
 *   [4] partial slot or -1  [5] work unit            [6] L_b         [7] tiles of b
 * Tiles are numbered along the sequence's retained tiles in ascending position.
 * Returns the number of segments written (<= cap) or a negative error.
 */
int32_t omniattn_plan_get_segments(const omniattn_plan_t* plan, int32_t* buf, int32_t cap);
/*
 * Logical token range [*lo, *hi) that retained tile `tile` of sequence `b`
 * spans (tile-aligned; the retained predicate still applies inside it).
 */
int omniattn_plan_tile_range(const omniattn_plan_t* plan, int32_t b, int32_t tile,
                             int32_t* lo, int32_t* hi);

/*
 * Steps a3-a9: gather retained tiles through the page table, QK^T, masking of
 * partial tiles, online softmax, PV, normalisation, and (when some sequence was
 * split) the combine pass.  Asynchronous on `hip_stream`; allocates nothing and
 * does not synchronise.  The current HIP device must be the one the plan was made on
 * (OMNIATTN_EINVAL otherwise).
 *
 *   q          device, bf16 [B, H, 576] contiguous (absorbed queries); [B, T, H, 576]
 *              for q_len = T > 1, and out / lse likewise [B, T, H, 512] / [B, T, H]
 *   kv_cache   device, bf16 or e4m3 bytes [num_pages, 128, 576] contiguous
 *   kv_scales  device, fp32 [num_pages, 128]; NULL unless kv_dtype is fp8.  Scales of
 *              retained tokens are finite and >= 0 (zero: a row of zeros).
 *   page_table device, int32 [B, max_pages_per_seq]; entry i of row b is the
 *              physical page of logical tokens [128 i, 128 i + 128).  Entries of
 *              pages that hold no retained token are never read.
 *   out        device, out_dtype [B, H, 512]
 *   lse        device, fp32 [B, H]: natural-log sum of exp(scale * q.k_j) over
 *              the retained j.  An empty retained set gives out = 0, lse = -inf.
 *   workspace  device, at least omniattn_plan_workspace_bytes(plan) bytes (partial
 *              rows of split sequences, in the output type, and their lse),
 *              256-byte aligned; may be NULL when that is 0.  Two decodes in
 *              flight at once need two workspaces.
 *
 * Slots outside the retained set, and pages not referenced, may hold anything
 * (NaN included) without effect.  Page ids of retained pages must lie in
 * [0, num_pages): the kernel does not check device-side contents.
 * Same plan + same inputs give bitwise identical results (nothing is accumulated atomically).
 * Arithmetic: bf16 cache - bf16 matrix products with fp32 accumulation, softmax weights
 * rounded to bf16.  fp8 cache - both products on the 8-bit matrix instruction; the query
 * enters as two e4m3 terms (exact for all but elements below 2^-14 of the row's largest), so
 * logits and lse carry fp32 accumulation error only; the softmax weights, with the token's
 * scale folded in, are rounded to e4m3 (relative 2^-4 per weight) and out is normalised by
 * the sum of the rounded weights.  A token whose scale is more than 2^10 below the largest
 * scale of its 64-token tile has its value row taken at 2^-10 of that largest scale (its
 * softmax weight counts in full).
 */
int omniattn_decode(const omniattn_plan_t* plan, const void* q, const void* kv_cache,
                    const float* kv_scales, const int32_t* page_table, void* out,
                    float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Same as omniattn_decode, and additionally records caller-owned HIP events
 * (hipEvent_t cast to void*, any may be NULL) on `hip_stream`: `ev_begin` before
 * the main kernel, `ev_main_end` after it, `ev_end` after the combine kernel
 * (recorded right after `ev_main_end` when the plan needs no combine).  For
 * benchmarks that report the main kernel's duration on its own; nothing is
 * allocated and nothing synchronises.
 */
int omniattn_decode_timed(const omniattn_plan_t* plan, const void* q, const void* kv_cache,
                          const float* kv_scales, const int32_t* page_table, void* out,
                          float* lse, void* workspace, size_t workspace_bytes, void* hip_stream,
                          void* ev_begin, void* ev_main_end, void* ev_end);

/*
 * For callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * same kernels and same results as omniattn_decode, but the partial rows of split
 * sequences go to a buffer of OMNIATTN_STATIC_SCRATCH_BYTES (40 MiB) that is part of the
 * library's device image; every GPU the library runs on holds it until the process ends.
 * The call allocates nothing and does not synchronise.  A plan whose
 * omniattn_plan_workspace_bytes() exceeds the buffer is refused with OMNIATTN_ESCRATCH
 * (nothing is launched).  All calls on one GPU share that GPU's buffer: two calls that
 * overlap in time on one GPU (different streams) race; calls on one stream are ordered.
 * Nothing in the buffer has to start at zero: every partial row is written by the main
 * kernel before the merge reads it.
 */
int omniattn_decode_static(const omniattn_plan_t* plan, const void* q, const void* kv_cache,
                           const float* kv_scales, const int32_t* page_table, void* out,
                           float* lse, void* hip_stream);
size_t omniattn_static_scratch_bytes(void);

/*
 * Physically compressed cache of a compressed layer.  Section 3.2.1 keeps only the
 * N_sink first and the N_recent last tokens of a sequence, so such a layer never has
 * to store more: a sequence owns omniattn_ring_pages(S, W) pages however long it
 * grows - ceil(S/128) pinned pages for the logical pages that hold sink tokens, and
 * a ring of ceil(W/128) + 1 pages which all later logical pages use in turn.  A ring
 * page is handed to a new logical page only when every token of its previous
 * logical page has left the window (see omniattn_ring_slot).  The decode entry
 * points need nothing new: the page table simply maps the retained logical pages to
 * these pages, and entries of logical pages that hold no retained token are never
 * read.
 * Several queries per sequence (q_len = T > 1): the earliest of the T queries keeps W
 * positions that end T - 1 tokens before the newest one, so the layer must keep the
 * W + T - 1 most recent tokens.  omniattn_ring_pages and omniattn_ring_slot are functions
 * of that effective window: pass window + T - 1 to them.  omniattn_ring_append reads q_len
 * from `prob` and adds T - 1 itself.
 *
 * omniattn_ring_slot   which of the sequence's own pages (0 .. ring_pages-1) holds
 *                      logical page `logical_page` (host, pure function; negative
 *                      arguments give -1).
 * omniattn_ring_append appends one token to every sequence of the batch (device
 *                      work on `hip_stream`, asynchronous, allocates nothing):
 *   prob       batch, max_pages_per_seq, sink, window, q_len, kv_dtype are used
 *   seq_lens   device int32 [B]: lengths before the call; each is incremented
 *   new_rows   device [B, 576] bf16, or e4m3 bytes for an fp8 cache
 *   new_scales device fp32 [B] for an fp8 cache, else NULL
 *   seq_pages  device int32 [B, omniattn_ring_pages(S, W + T - 1)]: the pool pages each
 *              sequence owns (distinct)
 *   kv_cache, kv_scales  the pool, as for omniattn_decode
 *   page_table device int32 [B, max_pages_per_seq]: entry L/128 of row b is written
 *              when the new token (position L) opens a logical page
 * A sequence whose length has reached 128 * max_pages_per_seq is left unchanged
 * (nothing written, length not incremented); the caller can see that from seq_lens.
 */
int32_t omniattn_ring_pages(int32_t sink, int32_t window);
int32_t omniattn_ring_slot(int32_t sink, int32_t window, int32_t logical_page);
int omniattn_ring_append(const omniattn_problem_t* prob, int32_t* seq_lens, const void* new_rows,
                         const float* new_scales, const int32_t* seq_pages, void* kv_cache,
                         float* kv_scales, int32_t* page_table, void* hip_stream);

const char* omniattn_strerror(int code);
/* Text of the last HIP error seen by the calling thread ("" if none). */
const char* omniattn_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OMNIATTN_H */
