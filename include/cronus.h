/*
 * cronus.h - C ABI of the MI355X (gfx950) mixed-iteration paged attention library.
 *
 * Scope: the attention work of one iteration of the chunked prefill instance of
 * Cronus (arXiv 2509.17357).  In that system the first part of a prompt is
 * prefilled on another GPU and its KV cache is transferred (section 4.2, steps 6-7:
 * the transfer takes the place of computing that prefix); the remainder runs as
 * chunked prefill, batched in the same iteration with single-token decodes of
 * earlier requests (section 4.4, "Chunked prefill"; Eq. 3 names the two attention
 * terms: continuation chunk against its prefill context, decodes against their
 * contexts).  The cache is managed in blocks of N_size tokens (Algorithm 1).
 *
 * Two operations:
 *   cronus_kv_append  - place K/V rows (a transferred prefix, or this iteration's new
 *                       tokens) into paged blocks through a block table.
 *   cronus_attn_mixed - causal attention of every sequence's chunk rows against
 *                       all of its cached keys, chunks and decodes in one launch.
 *
 * General rules
 *   - Every pointer says "host" or "device".  Device pointers are plain HIP device
 *     addresses on the current device.  The caller owns every buffer; the library
 *     never allocates or frees device memory and never allocates cache blocks.
 *   - All device work is enqueued on `hip_stream` (a hipStream_t cast to void*; NULL
 *     is the default stream).  No call synchronises the device.  Host arrays are
 *     consumed before the call returns.
 *   - Return value: a cronus_status.  Arguments are checked on the host before
 *     anything is launched: INVALID_ARG, UNSUPPORTED and WORKSPACE mean that nothing has
 *     been enqueued.  CRONUS_ERR_HIP reports a failed HIP runtime call; one-time set-up
 *     (kernel attributes, the plan buffers) precedes the first launch of a call, but a
 *     failed launch or event record can leave earlier kernels of the same call enqueued,
 *     and the outputs of that call are then undefined.
 *   - Device-side facts (CU count, kernel set-up, plan buffers) are kept per device and
 *     looked up for the device that is current in the calling thread; calls are
 *     serialised by one lock.
 *   - Block ids in block tables are NOT checked on the device: an id outside
 *     [0, num_blocks) or two rows mapped to one slot in a single call is undefined
 *     behaviour.  Table entries past ceil(len/16) are never read and may hold
 *     anything; cache slots past a sequence's length are never used as data.
 *
 * Paged cache layout (block_size = 16 tokens; E = element: bf16 = 2 bytes, or one
 * fp8 e4m3 code = 1 byte).  The layout is chosen so that every MFMA operand of the
 * attention kernel is one aligned 8-element chunk:
 *   K pool: [num_blocks][Hkv][D/8][16][8] E
 *       element (block b, head g, slot t, dim d) at
 *       (((b*Hkv + g)*(D/8) + d/8)*16 + t)*8 + d%8
 *       (a chunk = 8 consecutive d of one token; 16 tokens adjacent per chunk index)
 *   V pool: [num_blocks][Hkv][2][D][8] E
 *       element (b, g, t, d) at (((b*Hkv + g)*2 + t/8)*D + d)*8 + t%8
 *       (a chunk = 8 consecutive tokens of one d)
 *   One (block, head) is 16*D elements in either pool.
 * fp8 pools: real value = code_value * scale[g], one fp32 scale per KV head for K
 *   and one for V (OCP e4m3: no infinities, max 448).
 */
#ifndef CRONUS_H_
#define CRONUS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CRONUS_OK = 0,
  CRONUS_ERR_INVALID_ARG = 1, /* null pointer, negative size, lengths that do not fit the table */
  CRONUS_ERR_UNSUPPORTED = 2, /* head_dim not 64/128, block_size != 16, Hq % Hkv != 0, unknown dtype */
  CRONUS_ERR_WORKSPACE = 3,   /* workspace smaller than cronus_attn_mixed_workspace_bytes() */
  CRONUS_ERR_HIP = 4          /* a HIP runtime call failed */
} cronus_status;

typedef enum { CRONUS_KV_BF16 = 0, CRONUS_KV_FP8_E4M3 = 1 } cronus_kv_dtype;

typedef struct cronus_kv_cache {
  void* k_cache;        /* device; K pool, layout above                                  */
  void* v_cache;        /* device; V pool, layout above                                  */
  const float* k_scale; /* device fp32 [Hkv]; must be NULL for bf16, non-NULL for fp8    */
  const float* v_scale; /* device fp32 [Hkv]; same                                       */
  int64_t num_blocks;   /* blocks in each pool                                           */
  int32_t num_q_heads;  /* Hq                                                            */
  int32_t num_kv_heads; /* Hkv, divides Hq; q head h reads kv head h / (Hq/Hkv)          */
  int32_t head_dim;     /* D: 64 or 128                                                  */
  int32_t block_size;   /* 16                                                            */
  int32_t kv_dtype;     /* cronus_kv_dtype                                               */
} cronus_kv_cache;

/*
 * cronus_kv_append - scatter K/V rows into their paged blocks.
 * Section 4.2 (the transferred prefix is stored instead of computed) and the per-
 * iteration append of ordinary chunked prefill / decode; block granularity from
 * Algorithm 1.  Row r of sequence s (r = 0 .. cu_tokens[s+1]-cu_tokens[s]-1) is source
 * row cu_tokens[s]+r and goes to logical position p = start_pos[s]+r, that is block
 * block_tables[s*max_blocks_per_seq + p/16], slot p%16.  A prefix hand-off uses
 * start_pos = 0; appending an iteration's new tokens uses start_pos = tokens already
 * cached.  For an fp8 cache each element is quantised as
 * e4m3_rne(clamp(fp32(x) / scale[g], -448, 448)) with one IEEE fp32 division.
 *
 *   k_src, v_src : device, bf16 [n_tokens][Hkv][D], rows of all sequences back to back
 *   cu_tokens    : device, int32 [n_seqs+1], exclusive prefix sums, cu_tokens[0] = 0
 *   start_pos    : device, int32 [n_seqs]
 *   block_tables : device, int32 [n_seqs][max_blocks_per_seq]
 *   n_tokens     : total rows (= cu_tokens[n_seqs]); 0 is a no-op
 * Only the addressed slots are written.  The copy is bit-exact for bf16.
 * Errors: INVALID_ARG (null pointer, negative count), UNSUPPORTED (shape/dtype).
 */
int cronus_kv_append(const cronus_kv_cache* cache, const void* k_src, const void* v_src,
                     const int32_t* cu_tokens, const int32_t* start_pos,
                     const int32_t* block_tables, int32_t max_blocks_per_seq, int32_t n_seqs,
                     int32_t n_tokens, void* hip_stream);

/*
 * cronus_attn_mixed - attention of one mixed iteration (section 4.4; section 2 for
 * decode as one token against the whole cache).  Sequence s contributes
 * chunk_lens[s] query rows (1 = a decode, 0 = skipped) at logical positions
 * prefix_lens[s] .. prefix_lens[s]+chunk_lens[s]-1; keys/values of positions
 * [0, prefix_lens[s]+chunk_lens[s]) must already be in the cache.  Row i of head h:
 *     out[i,h,:] = softmax_j(sm_scale * <q[i,h,:], K[j,h/G,:]>, j <= prefix+i) . V[:,h/G,:]
 * computed with bf16 MFMA products, fp32 accumulation and fp32 softmax statistics;
 * the result is rounded to bf16.
 *
 *   q, out       : device, bf16 [total_q][Hq][D], total_q = sum(chunk_lens), batch order
 *   prefix_lens  : host, int32 [n_seqs]  (length already cached before this chunk)
 *   chunk_lens   : host, int32 [n_seqs]
 *   block_tables : device, int32 [n_seqs][max_blocks_per_seq]
 *   sm_scale     : softmax scale, normally 1/sqrt(D)
 *   workspace    : device, at least cronus_attn_mixed_workspace_bytes() bytes (never 0),
 *                  256-byte aligned; holds the partial results of key spans until they are
 *                  merged and, for an fp8 cache, a bf16 copy of the K/V of every sequence
 *                  whose chunk spans 16 or more tiles, or 8 or more behind 8192 or more
 *                  cached tokens (4 x Hkv x D bytes per cached or
 *                  new token of such a sequence, 1 GiB at most: sequences beyond that
 *                  are computed from the codes); contents are undefined afterwards;
 *                  must not be shared by calls that can overlap on the device
 * The work list is built on the host during the call and read by the kernels from
 * pinned, device-mapped host memory that the library owns (a ring of 8 buffers, grown on
 * demand, never freed; the ninth call in flight waits on the host for the first).  The main
 * kernel's work-groups stay resident and take their items from work queues whose heads (a
 * few integers per call in flight) live in a small static device array of the library; every
 * launch leaves its set of heads zero for the next one.
 * Errors: INVALID_ARG (null pointers, negative lengths, prefix+chunk >
 * 16*max_blocks_per_seq), UNSUPPORTED, WORKSPACE, HIP.
 */
int cronus_attn_mixed(const cronus_kv_cache* cache, const void* q, void* out,
                      const int32_t* prefix_lens, const int32_t* chunk_lens,
                      const int32_t* block_tables, int32_t max_blocks_per_seq, int32_t n_seqs,
                      float sm_scale, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * cronus_attn_mixed_static - cronus_attn_mixed for callers that cannot allocate: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * without the workspace, same kernels, same results; the call allocates no device or pinned
 * memory and calls no allocating HIP routine.  The plan image and the partial results live in
 * a static device array inside the library (64 MiB, CRONUS_STATIC_SCRATCH_BYTES; every GPU
 * that the library runs on holds its own copy until the process ends); the work list reaches
 * it as kernel arguments of small upload launches (about one per 48 work items) on
 * `hip_stream`.  The first call on a device looks up that device's address of the array and
 * sets the kernels' attributes (no allocation either).  On the host the planner keeps its
 * per-thread arrays (ordinary heap memory, grown to the largest batch the thread has planned).
 *   - CRONUS_ERR_WORKSPACE, nothing enqueued: the batch's plan image plus partial results
 *     exceed the array (about 4000 partial slots at head_dim 128; every benchmark batch fits).
 *   - fp8 cache: no bf16 copy is made (it would not fit); chunks of many tiles convert codes on
 *     the fly, so results can differ from cronus_attn_mixed's in the last bf16 bit.
 *   - Every call on a GPU uses that GPU's one array, which keeps the previous call's contents
 *     (nothing in it has to start at zero: a call reads only what it has written).  Calls on
 *     the same stream are ordered; calls that can overlap on one GPU (different streams or
 *     threads without ordering) race on it and must not be made.
 * Errors otherwise as cronus_attn_mixed.
 */
#define CRONUS_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int cronus_attn_mixed_static(const cronus_kv_cache* cache, const void* q, void* out,
                             const int32_t* prefix_lens, const int32_t* chunk_lens,
                             const int32_t* block_tables, int32_t max_blocks_per_seq,
                             int32_t n_seqs, float sm_scale, void* hip_stream);

/* Bytes of workspace cronus_attn_mixed needs for these lengths (host arrays); 0 on
 * invalid arguments.  Depends only on the shapes and lengths, not on cache contents. */
size_t cronus_attn_mixed_workspace_bytes(const cronus_kv_cache* cache, const int32_t* prefix_lens,
                                         const int32_t* chunk_lens, int32_t n_seqs);

/*
 * cronus_attn_mixed_plan_stats - how the work decomposition (mixed batch of section
 * 4.4 turned into tiles) would look for these lengths.  stats (host, int64[6]):
 * [0] work items launched, [1] of those that are wide (chunk) tiles, [2] split partial
 * results, [3] rows merged from partials, [4] work-groups of the merge kernel (0: it is
 * not launched), [5] cache blocks converted by the fp8 copy kernel (0: it is not
 * launched).  Returns a cronus_status.
 */
int cronus_attn_mixed_plan_stats(const cronus_kv_cache* cache, const int32_t* prefix_lens,
                                 const int32_t* chunk_lens, int32_t n_seqs, int64_t* stats);

/*
 * cronus_attn_mixed_plan_items - the work list itself, for inspection and tests (host
 * only, nothing is launched).  Writes up to `capacity` items, 11 int32 each: seq, kv_head,
 * head0, n_heads, q_tok0, n_tok, kv_begin, kv_end, partial, wide, queue.  The items form 8 queues, listed one after the other, each in the order in which
 * its items are taken: the main kernel's work-groups stay resident (one per CU) and take
 * items from the queue of the XCD they run on, then from the other queues.  wide >= 1: chunk
 * tile over keys [kv_begin, kv_end) (wide >= 2, fp8 cache only: it reads the launch's bf16
 * copy of its sequence, whose first block there is wide - 2); wide = 0: narrow item over
 * keys [kv_begin, kv_end); partial >= 0 when the item's result is merged with other spans
 * of the same rows.  Returns the number
 * of items of the plan (which may exceed capacity), or a negative cronus_status on invalid
 * arguments.  items may be NULL when capacity = 0.
 */
int64_t cronus_attn_mixed_plan_items(const cronus_kv_cache* cache, const int32_t* prefix_lens,
                                     const int32_t* chunk_lens, int32_t n_seqs, int32_t* items,
                                     int64_t capacity);

/*
 * cronus_kv_gather - the inverse of cronus_kv_append: export logical positions
 * [start_pos[s], start_pos[s] + n) of each sequence from its paged blocks into
 * contiguous rows (section 4.2: the partially prefilled prefix leaves the instance that
 * computed it as one contiguous KV cache buffer; the receiving side stores it with
 * cronus_kv_append).  Row r of sequence s (n = cu_tokens[s+1]-cu_tokens[s] rows) is
 * destination row cu_tokens[s]+r and comes from block
 * block_tables[s*max_blocks_per_seq + p/16], slot p%16, p = start_pos[s]+r.
 *
 *   k_dst, v_dst : device, [n_tokens][Hkv][D]; bf16 for a bf16 cache (bit-exact copy),
 *                  raw e4m3 codes (1 byte per element) for an fp8 cache: codes are
 *                  exported as stored, the scales travel separately
 *   cu_tokens, start_pos, block_tables : device, as for cronus_kv_append
 * Every destination row of the call is written in full; nothing else is.
 * Errors: INVALID_ARG (null pointer, negative count), UNSUPPORTED (shape/dtype), HIP.
 */
int cronus_kv_gather(const cronus_kv_cache* cache, void* k_dst, void* v_dst,
                     const int32_t* cu_tokens, const int32_t* start_pos,
                     const int32_t* block_tables, int32_t max_blocks_per_seq, int32_t n_seqs,
                     int32_t n_tokens, void* hip_stream);

/*
 * Execution-time models that the balancer uses (section 4.4): a partial prefill of L
 * tokens on the partial prefill instance takes k_p * L + b_p (Eq. 2); one chunked
 * prefill iteration whose prefill request has context L_ctx next to decode requests of
 * total context L_ctxd takes k_ctxp * L_ctx + k_ctxd * L_ctxd + b_c (Eq. 3).  All times
 * in one unit of the caller's choice.
 */
typedef struct cronus_balancer_model {
  double k_p, b_p;            /* Eq. 2 */
  double k_ctxp, k_ctxd, b_c; /* Eq. 3 */
  int32_t block_size;         /* N_size: tokens per KV block of the chunked prefill instance */
  int32_t batch_tokens;       /* B: most tokens batched into one iteration                   */
  int32_t n_candidates;       /* candidate split points, evenly spaced; 512 in Algorithm 1   */
} cronus_balancer_model;

/*
 * cronus_balancer_split - partial prefill length of one request (Algorithm 1 of the
 * appendix, with Eq. 1-3).  Host function; touches no device.
 *   l_in   : prompt length in tokens (> 0)
 *   n_d    : decode requests on the chunked prefill instance (0 <= n_d < batch_tokens);
 *            each iteration has n_p = batch_tokens - n_d prefill tokens
 *   l_ctxd : sum of those requests' context lengths (>= 0)
 *   n_free : free KV blocks of the chunked prefill instance (>= 0)
 *   l_p    : host, out; the chosen length, 1 <= *l_p <= l_in.  l_in itself when the
 *            prompt's ceil(l_in / N_size) blocks do not fit into n_free (the whole
 *            prompt is then prefilled on the partial prefill instance)
 *   t_prefill, t_chunked : host, out, may be NULL; the two modelled times for the
 *            returned length (on the capacity fallback l_p = l_in and t_chunked = 0)
 * Candidate j = 1..n_candidates is L_p = ceil(j * l_in / n_candidates); with
 * L_c = l_in - L_p, N_iter = ceil(L_c / n_p), L_last = L_p + floor(L_c / n_p) * n_p the
 * chunked time is N_iter * (k_ctxp * (l_in + L_last) / 2 + k_ctxd * l_ctxd + b_c), as
 * printed in Algorithm 1; the first candidate with the smallest |T_prefill - T_chunked|
 * wins.  Arithmetic is IEEE double without contraction, integers converted exactly.
 * Errors: INVALID_ARG (null model or l_p, values outside the ranges above, products
 * that would leave the exactly representable integer range).
 */
int cronus_balancer_split(const cronus_balancer_model* model, int64_t l_in, int64_t n_d,
                          int64_t l_ctxd, int64_t n_free, int64_t* l_p, double* t_prefill,
                          double* t_chunked);

/*
 * cronus_profile_events - measurement aid.  Handles are hipEvent_t cast to void*, created
 * by the caller with timing enabled.  While main_start and main_stop are set, every
 * cronus_attn_mixed launches its main attention kernel with them as the start and stop
 * events of that dispatch (hipExtLaunchKernel), on that call's stream:
 * hipEventElapsedTime(main_start, main_stop) is then the duration of that one kernel (within
 * a few microseconds of what a profiler's kernel trace shows for it).  A call may launch two
 * more kernels: the fp8 copy before the main kernel (cronus_attn_mixed_plan_stats [5] > 0) and
 * the merge after it ([4] > 0).  first_start, if set, becomes the start event of the copy
 * kernel when there is one, and last_stop the stop event of the merge kernel when there is
 * one; otherwise they are left untouched.  The whole attention of a call thus spans from
 * (copy ? first_start : main_start) to (merge ? last_stop : main_stop).  Pass four NULLs to
 * switch it off (the default).  Process-wide; not meant for concurrent callers.
 */
void cronus_profile_events(void* main_start, void* main_stop, void* first_start, void* last_stop);

/*
 * cronus_probe_mfma - measurement aid, not part of the attention path: the rate of
 * v_mfma_f32_32x32x16_bf16 (the instruction of both products of cronus_attn_mixed) that the
 * current GPU sustains when every CU issues nothing else.  Enqueues one kernel on hip_stream:
 * one work-group of 8 wavefronts per CU, each wavefront issuing iters x 32 independent MFMAs
 * on operand registers that hold small integer bit patterns (random_operands = 0) or random
 * bf16 values of magnitude 1/16 .. 1 (random_operands != 0: the switching activity of real
 * data; the clock a GPU holds under this load depends on it).  *flops_host receives the
 * floating-point operations of the launch (2 x 32 x 32 x 16 per MFMA); the caller times the
 * launch with events on the stream.  sink: DEVICE buffer of at least sink_floats floats that
 * receives the accumulators (one float per thread; cronus_probe_mfma_sink_floats()).
 * Returns CRONUS_OK, INVALID_ARG (iters < 1 or > 1 << 20, null pointers), WORKSPACE (sink
 * smaller than cronus_probe_mfma_sink_floats()), ERR_HIP.
 */
int cronus_probe_mfma(int random_operands, int iters, float* sink, size_t sink_floats, void* hip_stream,
                      double* flops_host);

/* Floats the sink of cronus_probe_mfma must hold on the current device (CUs x 512). */
size_t cronus_probe_mfma_sink_floats(void);

/* Static, NUL-terminated description of a cronus_status. */
const char* cronus_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int cronus_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CRONUS_H_ */
