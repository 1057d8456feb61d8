/*
 * pqcache.h -- C ABI of libpqcache: the decode-time hot path of PQ-based KV-cache
 * retrieval (PQCache, arxiv 2407.12820) for one attention layer on one AMD MI355X.
 *
 * What one decode step computes (paper, Section 3.1 steps 4-6; Algorithm 2,
 * "PQSearch", "AllKV = InitKV + TopkKV + LocalKV", attention):
 *
 *   1. look-up table: the decode query, cut into M partitions, is multiplied with
 *      every PQ centroid of its partition (Section 2.2, search phase);
 *   2. code scan: every cached token's approximate score is the sum over the
 *      partitions of the table entries its PQ code names;
 *   3. top-k: the K middle tokens with the largest approximate scores;
 *   4. the attended set is the initial window, those K tokens, the local window;
 *   5. softmax attention of every query head over the K/V rows of that set only.
 *
 * With grouped-query attention the G = Hq/Hkv query heads that share a KV head
 * share one selection: the group's score is the sum of its heads' scores.
 *
 * Notation: B sequences, Hq query heads, Hkv key/value heads, D = d_h head
 * dimension, N cached tokens, M partitions, C centroids per partition, Dm = D/M,
 * I/L initial/local window sizes, K retrieved tokens.  "Middle" tokens are
 * [I, N-L).  A "unit" is one (sequence, KV head) pair; units are independent.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers to contiguous row-major memory owned
 *     by the caller; inputs are read-only, outputs are fully overwritten.  16-byte
 *     alignment is required for every tensor pointer.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     only enqueue work on that stream: they never synchronise the host, never
 *     allocate or free device memory.  Results are ready when the stream reaches
 *     the end of the enqueued work.
 *   - Return value: PQC_OK (0) or a negative pqc_status.  Nothing throws or aborts.
 *   - A context is bound to one configuration and one workspace; it is not
 *     thread-safe, and calls that share a context must be ordered on one stream.
 *     Workspace contents are private to the library between calls.
 *   - Codes must satisfy code < C.  Tensors must hold finite values; the ranking
 *     of NaN scores is unspecified.
 *
 * Floating-point contract of the ranking (steps 1-3).  Scores are evaluated in
 * fp32 in this fixed order, so that a selection is reproducible bit for bit:
 *   qs[d]      = ((q_0[d] + q_1[d]) + ...)   over the group's heads, in head order;
 *   table[j,c] = fused multiply-add chain over e = 0..Dm-1 of qs[j*Dm+e]*cent[j,c,e],
 *                starting from 0;
 *   score[t]   = ((table[0,code0] + table[1,code1]) + table[2,code2]) + ...
 * Ties are broken towards the lower token index.
 */
#ifndef PQCACHE_H_
#define PQCACHE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pqc_ctx pqc_ctx; /* opaque, host memory, owned by the library */

typedef enum pqc_status {
  PQC_OK = 0,
  PQC_EINVAL = -1,      /* null pointer, malformed or inconsistent configuration   */
  PQC_EUNSUPPORTED = -2,/* well-formed configuration outside the supported shapes   */
  PQC_EWORKSPACE = -3,  /* workspace missing, misaligned or smaller than required   */
  PQC_EHIP = -4,        /* a HIP call failed; see pqc_last_hip_error()              */
  PQC_ESCRATCH = -5     /* pqc_decode_static: the shape needs more scratch memory    *
                         * than the library's static array holds                     */
} pqc_status;

typedef enum pqc_dtype { PQC_F32 = 0, PQC_BF16 = 1 } pqc_dtype;

/* Shape of one decode step.  Supported: head_dim = 128; pq_m in {1,2,4,8};
 * 1 <= pq_centroids <= 256; n_q_heads / n_kv_heads in {1,2,4,8};
 * n_init + topk + n_local <= n_tokens and >= 1; n_tokens <= 2^22;
 * B * Hkv <= 65535. */
typedef struct pqc_config {
  int32_t batch;         /* B                                                        */
  int32_t n_q_heads;     /* Hq                                                       */
  int32_t n_kv_heads;    /* Hkv, divides Hq                                          */
  int32_t head_dim;      /* D                                                        */
  int32_t n_tokens;      /* N, tokens in the K/V cache (same for every sequence)     */
  int32_t pq_m;          /* M, divides D                                             */
  int32_t pq_centroids;  /* C = 2^b (any value up to 256 is accepted)                */
  int32_t topk;          /* K, retrieved middle tokens per KV head                   */
  int32_t n_init;        /* I, always-attended first tokens                          */
  int32_t n_local;       /* L, always-attended most recent tokens                    */
  int32_t kv_dtype;      /* pqc_dtype of q, k_cache and v_cache                      */
  float softmax_scale;   /* factor on q.k before softmax; <= 0 means 1/sqrt(D)       */
  int32_t n_capacity;    /* tokens per (sequence, head) that k_cache, v_cache, keys  *
                          * and codes have room for, >= N: where the layouts below   *
                          * say [N] for these four tensors, the stride is n_capacity *
                          * and the first N entries are used.  0 means N (dense).    *
                          * At most 2^22.  A cache that grows by one token per       *
                          * decode step keeps its buffers and changes N alone        *
                          * (pqc_set_length).                                        */
} pqc_config;

/* Library version: major*10000 + minor*100 + patch. */
int pqc_version(void);

/* Static, human-readable text for a status code. */
const char* pqc_strerror(int status);

/* Bytes of device workspace a context of this configuration needs
 * (0 when the configuration is invalid or unsupported).  With n_capacity > n_tokens
 * the figure covers every length up to the capacity, so that the context can follow a
 * growing cache (pqc_set_length) in the same workspace. */
size_t pqc_workspace_bytes(const pqc_config* cfg);

/* Create a context.  `workspace` is device memory of at least
 * pqc_workspace_bytes(cfg) bytes, 256-byte aligned, which must stay valid and
 * untouched by the caller until pqc_destroy.  Host-only: enqueues nothing. */
int pqc_create(pqc_ctx** out, const pqc_config* cfg, void* workspace, size_t workspace_bytes);

/* Change the number of cached tokens N and the number of retrieved tokens K of an
 * existing context: the decode loop of Algorithm 2 appends one token per step to every
 * sequence, and the retrieval size follows the length (Section 4.1: a fixed share of
 * it).  All other fields, the capacity included, stay as created (a context created
 * without n_capacity has its first N as capacity).  Host-only, enqueues nothing; later
 * calls on the context use the new shape: out_idx is then [B][Hkv][I+K+L] with the new
 * K.  PQC_EINVAL when n_tokens exceeds the capacity or I + K + L exceeds n_tokens;
 * PQC_EWORKSPACE when the workspace given to pqc_create is too small for the new shape
 * (never the case when it was sized by pqc_workspace_bytes with the capacity set). */
int pqc_set_length(pqc_ctx* ctx, int32_t n_tokens, int32_t topk);

/* Free the host-side context (the workspace stays the caller's). NULL is allowed. */
void pqc_destroy(pqc_ctx* ctx);

/* hipError_t value of the last failed HIP call on this context (0 if none). */
int pqc_last_hip_error(const pqc_ctx* ctx);

/*
 * The whole decode step, steps 1-5 above (Algorithm 2: PQSearch, fetch of the
 * retrieved K/V, attention over initial + retrieved + local tokens).
 *
 *   q          [B][Hq][D]            kv_dtype   decode query of every head
 *   centroids  [B][Hkv][M][C][Dm]    f32        PQ centroids of the keys
 *   codes      [B][Hkv][N][M]        uint8      PQ codes of the keys
 *   k_cache    [B][Hkv][N][D]        kv_dtype
 *   v_cache    [B][Hkv][N][D]        kv_dtype
 *   out_idx    [B][Hkv][I+K+L]       int32      attended tokens: 0..I-1, then the K
 *                                               retrieved tokens (those above the
 *                                               threshold ascending, then the ones
 *                                               admitted at the threshold best first:
 *                                               compare as a set), then N-L..N-1
 *   out_attn   [B][Hq][D]            f32        attention output
 *
 * Codes of tokens inside the initial and local windows are ignored.
 *
 * The call enqueues kernel launches only (three; before a context's first call,
 * and after a call that failed, one more that clears the workspace) and a completed
 * call leaves the workspace as it found it.  It may therefore be recorded into a
 * HIP graph by stream capture and replayed, for instance one call per layer with
 * one context shared by all layers (Algorithm 2's loop over the layers); make one
 * ordinary call on the context first, so that the clearing launch is not recorded.
 */
int pqc_decode(pqc_ctx* ctx, const void* q, const float* centroids, const uint8_t* codes,
               const void* k_cache, const void* v_cache, int32_t* out_idx, float* out_attn,
               void* stream);

/* pqc_decode for a cache that has just received a token: besides the step, the code of that
 * token is written (Algorithm 2: the PQ search of a step and the code of the token that joins
 * the compressed part; Section 3.1: nearest centroid of each partition), inside the same three
 * launches -- nothing in the step reads it, so it costs no launch of its own.
 *   new_key   [B][Hkv][D]  kv_dtype   key of the token (e.g. its row of k_cache, copied)
 *   position  where its code goes: codes[b][h][position][0..M-1] (same result as
 *             pqc_pq_encode_token).  Must be a position whose code this call ignores: inside the
 *             initial or the local window, or at or beyond n_tokens (below the capacity);
 *             PQC_EINVAL otherwise.
 * Everything else as pqc_decode; `codes` is read and, at that one position, written. */
int pqc_decode_append(pqc_ctx* ctx, const void* q, const float* centroids, uint8_t* codes,
                      const void* k_cache, const void* v_cache, const void* new_key, int32_t position,
                      int32_t* out_idx, float* out_attn, void* stream);

/* pqc_decode for callers that cannot allocate device memory and hold no workspace: code that
 * runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * inputs, outputs, kernels and results as pqc_decode on a context of `cfg`; the workspace is a
 * device array inside the library, pqc_static_scratch_bytes() bytes (24 MiB) per GPU, which a
 * GPU holds from the library's first use on it until the process ends.  No context is needed
 * and the call allocates nothing, on the device or on the host; it enqueues the step's launches
 * preceded by one small fill kernel that clears the step's counters (the array keeps whatever
 * the last call left).
 *   - PQC_ESCRATCH when the step's workspace for n_tokens of cfg (never more than
 *     pqc_workspace_bytes(cfg)) exceeds pqc_static_scratch_bytes(); nothing is enqueued then.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two
 *     streams, two threads) race and give undefined results; order them on one stream.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress); make
 *     that call outside stream capture.
 * cfg is read at every call, so a growing cache needs no pqc_set_length here. */
size_t pqc_static_scratch_bytes(void);
int pqc_decode_static(const pqc_config* cfg, const void* q, const float* centroids, const uint8_t* codes,
                      const void* k_cache, const void* v_cache, int32_t* out_idx, float* out_attn,
                      void* stream);

/* The same step for PQ structures with two partitions of at most 64 centroids, where a
 * token's score takes one of C*C values (one per pair of codes): the threshold of the
 * top-k selection (Section 3.1 steps 4-5) then follows from the look-up table and from how
 * many tokens carry each pair, without a separate pass over the tokens.  Results are those
 * of pqc_decode (same scores, same selection, same attention).
 *   pair_counts [B][Hkv][C*C] uint32  tokens of the unit whose codes are (c0, c1), at index
 *                                     c0 + C*c1, over all N tokens: a statistic of `codes`
 *                                     alone, built by pqc_pair_counts and kept in step with
 *                                     appended codes by pqc_pair_counts_add (caller-owned)
 * PQC_EUNSUPPORTED unless pq_m == 2, pq_centroids <= 64 and the capacity (n_tokens when
 * none is given) is a multiple of 8.  pair_counts that do not belong to `codes` (a token
 * appended and not counted, or counted twice) give an unspecified selection; every write
 * still stays inside out_idx and out_attn. */
int pqc_decode_indexed(pqc_ctx* ctx, const void* q, const float* centroids, const uint8_t* codes,
                       const uint32_t* pair_counts, const void* k_cache, const void* v_cache,
                       int32_t* out_idx, float* out_attn, void* stream);

/* pqc_decode_indexed for a cache that has just received a token (as pqc_decode_append): on
 * entry pair_counts holds the first N tokens except the one at `position`, whose code does not
 * exist yet; the call writes that code and adds its pair to pair_counts, inside its own two
 * launches.  `position` as for pqc_decode_append. */
int pqc_decode_indexed_append(pqc_ctx* ctx, const void* q, const float* centroids, uint8_t* codes,
                              uint32_t* pair_counts, const void* k_cache, const void* v_cache,
                              const void* new_key, int32_t position, int32_t* out_idx, float* out_attn,
                              void* stream);

/* pair_counts of the first N tokens of a code tensor (fully overwritten), and the update for
 * the one code pair written at `position` (< capacity) of every unit: call it after
 * pqc_pq_encode_token for a position that was not counted before.  pqc_decode_indexed
 * expects the counts of exactly its N tokens, so in a growing cache every token is encoded
 * and counted when it is appended.  Need no context.  pq_m == 2 and pq_centroids <= 64. */
int pqc_pair_counts(const pqc_config* cfg, const uint8_t* codes, uint32_t* pair_counts, void* stream);
int pqc_pair_counts_add(const pqc_config* cfg, const uint8_t* codes, int32_t position, uint32_t* pair_counts,
                        void* stream);

/* Profiling aid: the kernels of pqc_decode one at a time.  phase 0 = histogram, 1 =
 * select + attention, 2 = finalize; calling phases 0, 1, 2 in this order with the same
 * arguments is exactly one pqc_decode (same kernels, same results).  It lets a harness
 * launch one phase for several contexts back to back between two events, which times
 * a kernel without an event in front of every launch.  A phase out of turn on a context
 * (not 0 after a complete step, not the successor of the phase before) is refused with
 * PQC_EINVAL and enqueues nothing; pqc_decode and the other calls start a new step whenever
 * they are called, whatever was left unfinished. */
#define PQC_DECODE_KERNELS 3
int pqc_decode_phase(pqc_ctx* ctx, int phase, const void* q, const float* centroids, const uint8_t* codes,
                     const void* k_cache, const void* v_cache, int32_t* out_idx, float* out_attn,
                     void* stream);

/* ---- the same path, one stage at a time (unit tests, per-kernel profiling) ---- */

/* Step 1 (Section 2.2 search / Section 3.1 step 4, "multiply the query with the PQ
 * centroids"):  table [B][Hkv][M][C] f32, per KV head (group-summed query). */
int pqc_lut(pqc_ctx* ctx, const void* q, const float* centroids, float* table, void* stream);

/* Step 2 (Section 3.1 step 4, "gather and reduce using PQ codes"):
 * scores [B][Hkv][N] f32; positions inside the initial and local windows hold -inf. */
int pqc_scan(pqc_ctx* ctx, const float* table, const uint8_t* codes, float* scores, void* stream);

/* Steps 3-4 (Section 3.1 steps 4-5, Section 3.2 top-k): from scores [B][Hkv][N] to
 * out_idx [B][Hkv][I+K+L] as in pqc_decode.  Window positions are not read. */
int pqc_topk(pqc_ctx* ctx, const float* scores, int32_t* out_idx, void* stream);

/* Step 5 (Section 2.1 attention restricted to the retrieved set, Section 3.1 step
 * 6): idx [B][Hkv][I+K+L] int32, every entry in [0, N) -> out_attn [B][Hq][D] f32.
 * Each listed K/V row is read once and shared by the G heads of its group. */
int pqc_gather_attn(pqc_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                    const int32_t* idx, float* out_attn, void* stream);

/* ---- PQ construction and maintenance (context-free; shapes come from cfg) ---- */

/* Bytes of device workspace pqc_pq_build needs (0 for an invalid configuration). */
size_t pqc_pq_build_workspace_bytes(const pqc_config* cfg);

/*
 * PQ construction (Section 2.2 index construction; Section 3.1 step 2): for every
 * (sequence, KV head, partition) Lloyd K-Means of the keys' sub-vectors into C
 * centroids.  Start: centroid c of partition j is the sub-vector of token
 * init_idx[b][h][j][c] (clamped into [0,N)).  `iters` rounds of (assign every token
 * to its nearest centroid in squared L2 distance, lowest index on ties; replace each
 * centroid by the mean of its members, an empty cluster keeps its centroid), then a
 * final assignment, so that the returned codes are the nearest centroids of the
 * returned centroids.  Distances are compared in fp32 (for bf16 keys through
 * |c|^2 - 2 x.c on the matrix cores, with fp32 accumulation of exact products), so a
 * token within fp32 rounding of two centroids may go to either; centroid sums are
 * exact integer sums of the keys rounded to 2^-20, hence independent of execution
 * order.
 *
 *   keys       [B][Hkv][N][D]        kv_dtype   (in)
 *   init_idx   [B][Hkv][M][C]        int32      (in)
 *   centroids  [B][Hkv][M][C][Dm]    f32        (out)
 *   codes      [B][Hkv][N][M]        uint8      (out)
 *   workspace  device memory, 256-byte aligned, >= pqc_pq_build_workspace_bytes(cfg)
 * The fields topk, n_init, n_local and softmax_scale of cfg are validated but unused.
 */
int pqc_pq_build(const pqc_config* cfg, const void* keys, const int32_t* init_idx, int32_t iters,
                 float* centroids, uint8_t* codes, void* workspace, size_t workspace_bytes,
                 void* stream);

/* Assignment step alone: codes[b][h][t][j] = nearest centroid of keys[b][h][t]'s j-th
 * sub-vector, for all N tokens (same arithmetic and tie rule as pqc_pq_build). */
int pqc_pq_assign(const pqc_config* cfg, const void* keys, const float* centroids, uint8_t* codes,
                  void* stream);

/* Code of one new token per (sequence, KV head) (Section 3.1: a token leaving the
 * local window is given the codes of its nearest centroids; Algorithm 2,
 * "PQArgNearest" then "Codes.append"):  key [B][Hkv][D] kv_dtype; writes
 * codes[b][h][position][0..M-1] inside the code tensor; 0 <= position < capacity (the
 * code of a token may be written as soon as the token exists: while the token is inside
 * the local window its code is ignored by pqc_decode). */
int pqc_pq_encode_token(const pqc_config* cfg, const void* key, const float* centroids,
                        uint8_t* codes, int32_t position, void* stream);

/* Block statistics for a block-level cache of hot K/V blocks (Section 3.4: after each
 * retrieval the cache is refreshed with the k_cache blocks that contain the most
 * retrieved tokens).  A block is block_tokens consecutive tokens, 1 <= block_tokens <= 2047;
 * nb = ceil(N / block_tokens) with N from cfg.
 *   idx     [B][Hkv][n_idx]  int32   listed tokens (e.g. out_idx of pqc_decode, or its
 *                                    retrieved part); entries outside [0, N) are skipped;
 *                                    the entries of one unit must be distinct
 *   counts  [B][Hkv][nb]     int32   listed tokens per block (fully overwritten)
 *   blocks  [B][Hkv][k_cache] int32  the k_cache blocks with the largest counts, a lower
 *                                    block index winning among equal counts, in the order
 *                                    in which pqc_block_cache_update serves them: fullest
 *                                    first, lower index first among equal counts; may be
 *                                    NULL when k_cache == 0.  0 <= k_cache <= nb.
 * Needs no context and no workspace.  PQC_EINVAL on null pointers or sizes out of range. */
int pqc_block_stats(const pqc_config* cfg, const int32_t* idx, int64_t n_idx, int32_t block_tokens,
                    int32_t k_cache, int32_t* counts, int32_t* blocks, void* stream);

/* Refresh of the block-level cache of Section 3.4: the retrieved tokens are looked up in the
 * cache, then the cache is refreshed with the k_cache blocks that hold the most retrieved
 * tokens, evicting by an LRU or an LFU policy.  The library keeps
 * the bookkeeping only: which blocks are resident, when each was last used and how often; the
 * K/V rows themselves already live in device memory here.  Per unit, the state is three
 * caller-owned arrays of n_slots entries, 1 <= n_slots <= 1024, updated in place:
 *   slot_block [B][Hkv][n_slots] int32  resident block, or -1 for an empty slot (initialise to -1)
 *   slot_stamp [B][Hkv][n_slots] int32  `step` of the block's last use
 *   slot_uses  [B][Hkv][n_slots] int32  steps in which the block was requested
 * Inputs of one step (both as written by pqc_block_stats for the same cfg and block_tokens):
 *   counts     [B][Hkv][nb]      int32  retrieved tokens per block
 *   blocks     [B][Hkv][k_cache] int32  requested blocks, distinct, served in this order;
 *                                       entries outside [0, nb) are skipped; 0 <= k_cache <= 1024
 *                                       (NULL allowed when 0)
 *   step       any int32 that grows from call to call
 * First the look-up: stats[b][h] = { retrieved tokens lying in blocks that are resident before
 * the refresh, requested blocks that are resident, blocks inserted, blocks evicted } (int32 x 4).
 * Then the refresh: a requested resident block gets stamp = step and uses + 1; a requested
 * absent block takes the lowest empty slot, else it replaces, among the slots holding no block
 * requested in this step, the one used longest ago (PQC_CACHE_LRU) or the one with the fewest
 * uses, the one used longest ago among those (PQC_CACHE_LFU), the lowest slot on remaining ties,
 * and starts with stamp = step, uses = 1; requests left when no such slot remains are dropped.
 * The paper names the two policies and leaves these details open.  Needs no context. */
#define PQC_CACHE_LRU 0
#define PQC_CACHE_LFU 1
int pqc_block_cache_update(const pqc_config* cfg, int32_t block_tokens, int32_t n_slots, int32_t policy,
                           int32_t step, const int32_t* counts, const int32_t* blocks, int32_t k_cache,
                           int32_t* slot_block, int32_t* slot_stamp, int32_t* slot_uses, int32_t* stats,
                           void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PQCACHE_H_ */
