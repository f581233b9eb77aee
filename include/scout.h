/*
 * scout.h -- C ABI of the MI355X-native GPU side of GPU-CPU collaborative
 * block-wise sparse decode attention (ScoutAttention, Sec. 3.2-3.4, Alg. 1).
 *
 * One decode step of one layer, as the paper states it (Sec. 3.2):
 *   1. score every KV block of every sequence by the query against the
 *      block's digest                                   -> score_blocks
 *   2. keep the top-k blocks under the token budget and split them by
 *      residency (Alg. 1: B_cpu = B_pred \ B_gpu)        -> select_topk
 *   3. attend, on the GPU, to the selected blocks that are GPU-resident,
 *      producing a partial result                        -> sparse_decode_attn
 *   4. merge that partial with the one the host computed for the offloaded
 *      selected blocks (FlashAttention rescaling)        -> merge_partials
 *   and, every few steps, after the layer's attention (Sec. 3.4), plan which
 *   offloaded blocks return to the GPU                   -> periodic_recall
 *
 * Conventions common to every entry point
 *   - Every pointer except `const scout_problem*` is DEVICE memory owned by
 *     the caller (recall_fetch and append_token also take pinned host memory).  The library allocates nothing, frees nothing and keeps no
 *     pointer after a call returns.  Scratch comes from the caller's
 *     workspace (`ws`, at least scout_workspace_bytes() bytes, 256-byte
 *     aligned).
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue
 *     work and return; they never synchronise.
 *   - Arguments are validated on the host before anything is launched.  A
 *     negative return code means nothing was launched and no output was
 *     written.  Device-side data (ctx_len, slots, counts) cannot be checked
 *     on the host: kernels clamp counts to their array bounds and skip slots
 *     outside [0, n_slots), so malformed device data gives wrong numbers,
 *     never an out-of-bounds access.
 *   - All tensors are dense, row-major, 16-byte aligned.
 *   - Same inputs give the same bits: no floating-point atomics anywhere.
 *
 * Symbols:  B sequences, Hq query heads, Hkv KV heads, G = Hq/Hkv, d head
 * dim, S tokens per block, nb_b = ceil(ctx_len[b]/S), "pair" = one
 * (sequence, KV head).  "e" is the element type selected by `dtype`.
 */
#ifndef SCOUT_H
#define SCOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SCOUT_OK = 0,
  SCOUT_EINVAL = -1,       /* null pointer, bad shape, misaligned pointer          */
  SCOUT_EUNSUPPORTED = -2, /* valid request outside what the kernels cover          */
  SCOUT_EWORKSPACE = -3,   /* workspace missing, misaligned or too small            */
  SCOUT_EHIP = -4,         /* the HIP runtime reported an error at launch           */
  SCOUT_ESCRATCH = -5      /* sparse_decode_attn_static: the problem needs more scratch
                              than SCOUT_STATIC_SCRATCH_BYTES                         */
};

enum { SCOUT_F32 = 0, SCOUT_BF16 = 1 };

typedef struct scout_problem {
  int32_t B, Hq, Hkv; /* Hq % Hkv == 0, G = Hq/Hkv <= 16; B * Hkv <= 65535
                         (B * Hq with per_head)                                    */
  int32_t d;          /* head dim: 64 or 128                                        */
  int32_t S;          /* tokens per block: 16, 32 or 64                             */
  int32_t dtype;      /* element type of q, k_pool, v_pool, digest, out             */
  int32_t max_blocks; /* row length of scores / block_table / digest, <= 16384      */
  int32_t k;          /* block budget per pair = token budget / S, 1 <= k <= 1024   */
  float sm_scale;     /* softmax scale; 0 means 1/sqrt(d)                           */
  int32_t n_sink;     /* always-kept blocks: the first n_sink blocks of a sequence  */
  int32_t n_tail;     /* and its last n_tail blocks that hold tokens (both >= 0)    */
  int32_t group_max;  /* block importance of a KV head: 0 = sum over its G query
                         heads (default), 1 = maximum over them                     */
  int32_t per_head;   /* 0 = one selection per KV head, shared by its G query heads
                         (default); 1 = every query head selects its own blocks:
                         scores, the sel_* / slot_gpu lists and the n_* counts
                         then have Hq where the layouts below say Hkv, while
                         digest, block_table, the pools and everything about
                         building, appending and recalling keep Hkv             */
  int32_t digest_kind; /* 0 = channel-wise min and max of a block's keys (default; the
                         digest layouts below), 1 = mean pooling: `digest` is then
                         f32 [B][Hkv][max_blocks][d], the SUM of the block's valid
                         keys in binary32 added in token order (an append is one
                         addition and equals a rebuild bit for bit), and a block's
                         importance is sum_h q_h . sum / count; not with group_max */
  int32_t tile_stride; /* elements from the tile of one pool slot to the tile of the next, in
                         k_pool and in v_pool alike.  0 = S * d: two dense pools
                         [n_slots][S][d].  2 * S * d with v_pool = k_pool + S * d is ONE pool
                         [n_slots][2][S][d] in which the K tile and the V tile of a slot lie
                         next to each other (one 16 KiB region per block instead of two 8 KiB
                         regions).  Otherwise >= S * d and a multiple of 8                  */
  const int32_t* ctx_len; /* DEVICE int32 [B]: tokens per sequence; blocks beyond
                             max_blocks are ignored                                  */
} scout_problem;

/* Library version, major*100 + minor. */
int scout_version(void);

/* Short static description of an error code. */
const char* scout_strerror(int code);

/* Bytes of workspace that any entry point may use for this problem. */
int scout_workspace_bytes(const scout_problem* p, size_t* bytes);

/*
 * Block digests (Sec. 2.2: channel-wise min and max pooling over the keys of
 * a block).  Builds the digest cache from keys laid out block by block.
 *   k_blocks  e  [B][Hkv][max_blocks][S][d]   keys of every block (any residency)
 *   digest    e  [B][Hkv][max_blocks][2][d]   out: [..][0] = min, [..][1] = max
 * Only the valid tokens of a block are pooled; rows of blocks >= nb_b are
 * left untouched.  Min/max never round, so the result is exact.
 */
int build_digests(const scout_problem* p, const void* k_blocks, void* digest, void* stream);

/*
 * Decode append (the digest of Sec. 2.2 kept current while the cache of
 * Sec. 3.2 grows): the key and value of the token that decode just produced
 * join every KV head of every sequence.  With t = ctx_len[b] before the call,
 * the token takes row r = t % S of block j = t / S:
 *   - r == 0 opens block j: block_table[b][g][j] = new_slot[b][g] (a pool slot,
 *     or -1 when the caller keeps the new block on the host) and both digest
 *     rows become the key; otherwise a digest element changes only where the
 *     key is strictly smaller (min row) or strictly larger (max row);
 *   - if the block's table entry is a slot in [0, n_slots), the key and value
 *     rows are written to row r of that slot's K and V tiles (a host-resident
 *     tail block is the caller's to extend);
 *   - if host_k / host_v are given, the rows are also written to the host's copy
 *     of every block, whatever the block's residency: with it the host always
 *     holds the whole cache, which is what recall_fetch reads from and why an
 *     eviction moves nothing;
 *   - ctx_len[b] becomes t + 1.
 * A sequence that already fills max_blocks blocks is left untouched.
 *   ctx_len      i32 [B]              in/out; the lengths to advance (normally
 *                                     the array p->ctx_len points to, which this
 *                                     call does not read through p)
 *   k_new, v_new e   [B][Hkv][d]
 *   new_slot     i32 [B][Hkv]         read only for sequences with r == 0
 *   digest       e   [B][Hkv][max_blocks][2][d]   in/out
 *   block_table  i32 [B][Hkv][max_blocks]         in/out
 *   k_pool, v_pool e [n_slots][S][d]              in/out
 *   host_k, host_v e [B][Hkv][max_blocks][S][d]   in/out, both or neither (NULL);
 *                  PINNED HOST memory that the GPU can address (or device memory)
 * Copies and comparisons only; the result is exact.
 */
int append_token(const scout_problem* p, int32_t* ctx_len, const void* k_new, const void* v_new,
                 const int32_t* new_slot, void* digest, int32_t* block_table, void* k_pool,
                 void* v_pool, int64_t n_slots, void* host_k, void* host_v, void* stream);

/*
 * Block importance (Sec. 2.2, Sec. 3.2, Alg. 1 TopK argument): for each pair
 * and block j, sum over the G query heads of the group and over channels c of
 * max(q[c]*min_j[c], q[c]*max_j[c])  (with group_max = 1: the maximum over the
 * heads of that sum over channels).  Unscaled.  Accumulated in binary64 and
 * rounded once to binary32.  The always-kept blocks (j < n_sink or
 * j >= nb_b - n_tail) get +inf instead, so that the selection keeps them first
 * (lower index first if the budget cannot hold them all); they count against k.
 *   q        e   [B][Hq][d]
 *   digest   e   [B][Hkv][max_blocks][2][d]
 *   scores   f32 [B][Hkv][max_blocks]          out; -inf for j >= nb_b
 */
int score_blocks(const scout_problem* p, const void* q, const void* digest, float* scores,
                 void* ws, size_t ws_bytes, void* stream);

/*
 * Top-k selection and residency split (Alg. 1: TopK, then B_pred \ B_gpu).
 * Per pair: the k_eff = min(k, nb_b) blocks that come first when ordered by
 * (score descending, block index ascending), reported in ascending index.
 *   scores       f32 [B][Hkv][max_blocks]
 *   block_table  i32 [B][Hkv][max_blocks]   pool slot (>= 0) of a GPU-resident
 *                                           block, -1 for a host-resident one
 *   sel_all      i32 [B][Hkv][k]   out: selected block indices, then -1
 *   sel_gpu      i32 [B][Hkv][k]   out: the resident ones, then -1
 *   slot_gpu     i32 [B][Hkv][k]   out: their pool slots, then -1
 *   n_gpu        i32 [B][Hkv]      out
 *   sel_host     i32 [B][Hkv][k]   out: the offloaded ones, then -1
 *   n_host       i32 [B][Hkv]      out
 * Integer and comparison work only; the result is exact.  NaN scores rank
 * below -inf.
 */
int select_topk(const scout_problem* p, const float* scores, const int32_t* block_table,
                int32_t* sel_all, int32_t* sel_gpu, int32_t* slot_gpu, int32_t* n_gpu,
                int32_t* sel_host, int32_t* n_host, void* ws, size_t ws_bytes, void* stream);

/*
 * GPU-side partial attention (Sec. 3.2; Alg. 1 GPUAttn): for every query head,
 * softmax(sm_scale * q.K^T) V over all valid tokens of the listed resident
 * blocks, returned as a partial result (o, m, l):  m = max logit (natural-log
 * units), l = sum exp(logit - m), o = sum exp(logit - m) v / l.
 * An empty list gives o = 0, m = -inf, l = 0.
 *   q         e   [B][Hq][d]
 *   k_pool    e   [n_slots][S][d]     one K tile per resident (pair, block)
 *   v_pool    e   [n_slots][S][d]
 *   sel_gpu   i32 [B][Hkv][k]         logical block index (masks a partial last block)
 *   slot_gpu  i32 [B][Hkv][k]         pool slot of the same entry
 *   n_gpu     i32 [B][Hkv]            entries used per pair (clamped to k)
 *   o         f32 [B][Hq][d], m f32 [B][Hq], l f32 [B][Hq]   out
 * Inputs are read in their stored type; products and sums are binary32 (the
 * bf16 kernel rounds softmax weights to bf16 before the value product).
 */
int sparse_decode_attn(const scout_problem* p, const void* q, const void* k_pool,
                       const void* v_pool, int64_t n_slots, const int32_t* sel_gpu,
                       const int32_t* slot_gpu, const int32_t* n_gpu, float* o, float* m,
                       float* l, void* ws, size_t ws_bytes, void* stream);

/*
 * sparse_decode_attn for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without `ws`, same kernels,
 * same results bit for bit.  The per-split partials that the two passes exchange
 * live in a buffer of SCOUT_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (every GPU the library runs on holds its own copy until the
 * process ends); the call allocates nothing, frees nothing and calls no
 * allocating routine.
 *   - A problem whose partials do not fit returns SCOUT_ESCRATCH and launches
 *     nothing.  They take about  B * Hkv * nsplit * G * (d + 2) * 4  bytes, where
 *     nsplit is the number of workgroups the library spreads a pair over: about
 *     256 / (B * Hkv) for bf16 with d = 128 (none at all from 192 pairs on, where
 *     a workgroup finishes its pair), at most 64.  All five benchmark
 *     configurations need at most 1.1 MiB.
 *   - The buffer's device address is looked up on the first call on each device
 *     (hipGetSymbolAddress); make that first call outside a graph capture.
 *   - Every call on a GPU uses that GPU's one buffer, which keeps the last
 *     call's contents.  Nothing in it has to be cleared between calls (each call
 *     writes every word it later reads), but two calls that overlap in time on
 *     one GPU (different streams, different threads) race: order them.
 */
#define SCOUT_STATIC_SCRATCH_BYTES (8u << 20)
int sparse_decode_attn_static(const scout_problem* p, const void* q, const void* k_pool,
                              const void* v_pool, int64_t n_slots, const int32_t* sel_gpu,
                              const int32_t* slot_gpu, const int32_t* n_gpu, float* o, float* m,
                              float* l, void* stream);

/*
 * First half of sparse_decode_attn on its own: the pass that streams the K/V
 * rows and leaves one partial per (pair, split) in the workspace; the small
 * combine pass that folds the splits is left out.  Same arguments; writes
 * nothing but the workspace.  It exists so that the bandwidth-bound kernel can
 * be timed alone.
 */
int scout_attn_partials(const scout_problem* p, const void* q, const void* k_pool,
                        const void* v_pool, int64_t n_slots, const int32_t* sel_gpu,
                        const int32_t* slot_gpu, const int32_t* n_gpu, void* ws, size_t ws_bytes,
                        void* stream);

/*
 * Second half to scout_attn_partials for a caller that starts the GPU's
 * attention before the host's partial has arrived (the layer-ahead pipeline of
 * Sec. 3.3): folds the per-split partials that the preceding
 * scout_attn_partials call (same problem, same workspace, same stream or
 * ordered after it) left in the workspace and merges them with the host's
 * partial (Alg. 1 Merge) in one pass, instead of exporting (o, m, l) and
 * merging in a further launch.  host_* may be all NULL; lse may be NULL.
 *   host_o f32 [B][Hq][d], host_m, host_l f32 [B][Hq];  out e [B][Hq][d];  lse f32 [B][Hq]
 * The attention mode must not be changed between the two calls.
 */
int scout_attn_finish(const scout_problem* p, const float* host_o, const float* host_m,
                      const float* host_l, void* out, float* lse, void* ws, size_t ws_bytes,
                      void* stream);

/*
 * Merge of two partial results (Alg. 1 Merge; FlashAttention rescaling):
 *   m* = max(m_a, m_b), w_x = l_x exp(m_x - m*), out = (w_a o_a + w_b o_b)/(w_a + w_b),
 *   lse = m* + ln(w_a + w_b).  A side with l = 0 has weight 0.
 *   o_a, o_b  f32 [B][Hq][d];  m_*, l_*  f32 [B][Hq];  side b may be all NULL
 *   out       e   [B][Hq][d]
 *   lse       f32 [B][Hq]   optional (may be NULL)
 */
int merge_partials(const scout_problem* p, const float* o_a, const float* m_a, const float* l_a,
                   const float* o_b, const float* m_b, const float* l_b, void* out, float* lse,
                   void* stream);

/*
 * Periodic recall plan (Sec. 3.4): rescore all blocks with the current query,
 * take the top-k set T, and with R the resident set of a pair:
 *   recall = T \ R (if larger than R \ T, its best-ranked |R \ T| members),
 *   evict  = the |recall| worst-ranked members of R \ T,
 * both ascending by block index; the i-th recalled block takes the slot of the
 * i-th evicted block and block_table is updated in place.  The caller copies
 * the recalled tiles into the returned slots before the next step's attention.
 *   block_table  i32 [B][Hkv][max_blocks]   in/out
 *   recall_blk, recall_slot, evict_blk  i32 [B][Hkv][k]   out, padded with -1
 *   n_recall     i32 [B][Hkv]   out
 */
int periodic_recall(const scout_problem* p, const void* q, const void* digest,
                    int32_t* block_table, int32_t* recall_blk, int32_t* recall_slot,
                    int32_t* evict_blk, int32_t* n_recall, void* ws, size_t ws_bytes,
                    void* stream);

/*
 * Data movement of a periodic recall (Sec. 3.4: the planned blocks return from
 * host memory after the layer's attention, off the critical path).  For every
 * pair and every i < n_recall, the K and V tiles of block recall_blk[i] are
 * copied from the source arrays into pool slot recall_slot[i]; the three plan
 * arrays are the ones periodic_recall wrote.  Launch it on a stream of its
 * own to keep it off the compute stream; the recalled blocks are first read by
 * the next step's attention.
 *   src_k, src_v  e [B][Hkv][max_blocks][S][d]   every block that may be
 *                 recalled, by logical index, in memory the GPU can address:
 *                 PINNED HOST memory (hipHostMalloc; read over the host link
 *                 by the kernel itself) or device memory
 *   recall_blk, recall_slot  i32 [B][Hkv][k];  n_recall  i32 [B][Hkv]   DEVICE
 *   k_pool, v_pool  e [n_slots][S][d]   in/out
 * Entries outside [0, max_blocks) x [0, n_slots) are skipped.  Pure copies.
 * Wave loads over the host link slow every kernel that runs at the same time
 * (measured: by 1.7 to 1.9 times); a transfer that is to overlap with compute
 * goes through recall_scatter below instead.
 */
int recall_fetch(const scout_problem* p, const void* src_k, const void* src_v,
                 const int32_t* recall_blk, const int32_t* recall_slot, const int32_t* n_recall,
                 void* k_pool, void* v_pool, int64_t n_slots, void* stream);

/*
 * The same recall (Sec. 3.4) for tiles that were brought over by a copy
 * engine: the host packs the planned tiles in plan order
 * (scout_host_stage_recall in scout_host.h), one contiguous asynchronous copy
 * moves the packed buffer into device memory, and this call puts the tiles into
 * their slots, device to device.  For every pair and every
 * i < min(n_recall, k), tile t = tile_off[pair] + i of the buffer (K rows at
 * byte t * 2 * tile, V rows at t * 2 * tile + tile, tile = S * d * sizeof(e))
 * goes to pool slot recall_slot[i]; entries whose recall_blk is outside
 * [0, max_blocks) or whose slot is outside [0, n_slots) are skipped, so the
 * result equals recall_fetch's.
 *   staged    e   [n_tiles][2][S][d]   DEVICE, 16-byte aligned
 *   tile_off  i32 [B][Hkv]             DEVICE: first tile of each pair (the
 *                                      exclusive prefix sum of min(n_recall, k))
 *   the other arguments as for recall_fetch
 * An entry whose tile index falls outside [0, n_tiles) moves nothing.
 */
int recall_scatter(const scout_problem* p, const void* staged, int64_t n_tiles, const int32_t* tile_off,
                   const int32_t* recall_blk, const int32_t* recall_slot, const int32_t* n_recall,
                   void* k_pool, void* v_pool, int64_t n_slots, void* stream);

/*
 * One whole layer-step (Sec. 3.2, steps 1-4 above) with the fewest launches:
 * score, select, attend, and combine the attention splits together with the
 * host partial.  Outputs are those of the four separate calls; host_* may be
 * all NULL (nothing offloaded).  sel_host / n_host tell the host which blocks
 * it has to cover for this query.  `scores` may be NULL for a caller that does
 * not need them (they then stay in the workspace or, where one workgroup does
 * the whole step of a pair, on the chip).  Launches: three where a pair is
 * spread over several workgroups (scoring; selection + attention; combine +
 * merge), one where the pairs alone fill the chip (bf16, d = 128, at least 192
 * pairs: every step of a pair in one workgroup).
 *
 * slot_gpu and n_gpu are read before they are written: what they hold on entry
 * is taken as a HINT of where this step's tiles will be (adjacent decode tokens
 * attend to highly overlapping sets of blocks, Sec. 1; a caller that keeps one set
 * of list buffers per layer hands over the previous step's lists by doing nothing).
 * While the selection runs, the kernel touches the tiles of the hinted slots
 * so that they are on their way from HBM.  The hint changes no result, whatever
 * it holds: counts are clamped to [0, k], slots outside [0, n_slots) are
 * skipped, nothing outside the pools is read, and the values read are dropped.
 * Buffers that were never written are a valid (useless) hint.  Only budgets up to
 * k = 128 use it.
 */
int scout_layer_step(const scout_problem* p, const void* q, const void* digest,
                     const int32_t* block_table, const void* k_pool, const void* v_pool,
                     int64_t n_slots, const float* host_o, const float* host_m,
                     const float* host_l, float* scores, int32_t* sel_all, int32_t* sel_gpu,
                     int32_t* slot_gpu, int32_t* n_gpu, int32_t* sel_host, int32_t* n_host,
                     void* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Tuning knob for measurements: force the attention kernel family, the split
 * count per pair and the workgroup size.  family: 0 = automatic, 1 = generic
 * vector-ALU kernel, 2 = MFMA kernel (bf16 and d = 128 only; otherwise
 * SCOUT_EUNSUPPORTED at the call), 3 = as 2, but scout_layer_step launches the
 * scoring and the selection on their own instead of inside the attention kernel,
 * 4 = as 2, but only the scoring on its own.
 * nsplit: 0 = automatic, else 1..64.
 * waves: 0 = automatic, else 4, 8 or 16 waves per workgroup (MFMA family).
 * The setting belongs to the calling thread (other threads keep their own).
 */
int scout_set_attn_mode(int family, int nsplit, int waves);

#ifdef __cplusplus
}
#endif
#endif /* SCOUT_H */
