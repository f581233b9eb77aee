/*
 * scout_host.h -- C ABI of the HOST side of GPU-CPU collaborative block-wise
 * sparse decode attention: the attention over the selected blocks that live
 * in host memory (ScoutAttention, Sec. 3.2; Alg. 1 CPUAttn), computed by a
 * pool of worker threads next to the data, so that only a partial result of
 * G*(d+2) floats per (sequence, KV head) pair crosses the host link instead
 * of the blocks themselves.  The call is asynchronous so that it can run one
 * layer ahead of the GPU (Sec. 3.3).
 *
 * Every pointer here is HOST memory owned by the caller and must stay valid
 * and unchanged from submit until the matching wait returns.  Symbols as in
 * scout.h; "e" is the element type selected by `dtype` (SCOUT_F32 = 0,
 * SCOUT_BF16 = 1).
 */
#ifndef SCOUT_HOST_H
#define SCOUT_HOST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct scout_host_worker scout_host_worker;

typedef struct scout_host_problem {
  int32_t B, Hq, Hkv; /* Hq % Hkv == 0, G = Hq/Hkv <= 16                       */
  int32_t d;          /* head dim, a multiple of 8, <= 256                     */
  int32_t S;          /* tokens per block, <= 64                               */
  int32_t dtype;      /* element type of q, k_blocks, v_blocks                 */
  int32_t max_blocks; /* row length of k_blocks / v_blocks                     */
  int32_t k;          /* row length of sel_host                                */
  float sm_scale;     /* softmax scale; 0 means 1/sqrt(d)                      */
} scout_host_problem;

/*
 * Start a pool of n_threads worker threads (>= 1).  Returns 0 and the handle,
 * or a negative code (-1 bad argument, -5 out of memory / thread start failed).
 */
int scout_host_create(int n_threads, scout_host_worker** out);

/* Stop the threads and free the pool.  Waits for the jobs handed in (the running one and the one behind it). */
void scout_host_destroy(scout_host_worker* w);

/*
 * Host-side partial attention (Sec. 3.2; Alg. 1 CPUAttn): for every query head,
 * softmax(sm_scale * q.K^T) V over all valid tokens of the listed blocks, as a
 * partial result in the convention of sparse_decode_attn: m = max logit
 * (natural-log units), l = sum exp(logit - m), o = sum exp(logit - m) v / l;
 * an empty list gives o = 0, m = -inf, l = 0.
 *   q         e   [B][Hq][d]      (the predicted query when run a layer ahead)
 *   k_blocks  e   [B][Hkv][max_blocks][S][d]   the host's copy of the blocks,
 *   v_blocks  e   same layout                   by logical block index
 *   sel_host  i32 [B][Hkv][k]     logical indices of the offloaded selected blocks
 *   n_host    i32 [B][Hkv]        entries used per pair (clamped to k)
 *   ctx_len   i32 [B]             tokens per sequence (masks a partial last block)
 *   o f32 [B][Hq][d], m f32 [B][Hq], l f32 [B][Hq]   out
 * Inputs are read in their stored type; products and sums are binary32.
 * Returns at once (0); -1 on a bad argument.  One job runs at a time, the
 * pairs being dealt to the threads; ONE more may be handed in while it runs and
 * starts when it ends (Alg. 1 spawns the job of layer i+1 before the GPU has
 * merged layer i's); -6 if one is waiting already.  The arrays of a job must
 * stay as they are until scout_host_wait has reported it.  Indices outside
 * [0, max_blocks) and blocks beyond the context are skipped.
 */
int scout_host_submit(scout_host_worker* w, const scout_host_problem* p, const void* q,
                      const void* k_blocks, const void* v_blocks, const int32_t* sel_host,
                      const int32_t* n_host, const int32_t* ctx_len, float* o, float* m, float* l);

/*
 * Pack the tiles of a recall plan for one contiguous transfer (Sec. 3.4: the
 * planned blocks return to the GPU asynchronously).  Over all pairs in order,
 * the tiles of the first min(n_recall[pair], k) plan entries are copied, by the
 * pool's threads, into `staged`: tile t = tile_off[pair] + i holds the K rows of
 * block recall_blk[pair][i] at byte t * 2 * tile and its V rows at
 * t * 2 * tile + tile (tile = S * d * sizeof(e)).  An entry outside
 * [0, max_blocks) keeps its place; nothing is written there.
 *   k_blocks, v_blocks  e [B][Hkv][max_blocks][S][d]   the host's copy of the blocks
 *   recall_blk  i32 [B][Hkv][k], n_recall i32 [B][Hkv]   the plan, copied to HOST memory
 *   staged      bytes, staged_bytes long: out (pinned memory if a copy engine is
 *               to read it); may be NULL if the plan is empty
 *   tile_off    i32 [B][Hkv]   out: first tile of each pair, written before the
 *               call returns
 *   total_tiles out: tiles in the packed buffer, written before the call returns
 * Only p's B, Hkv, d, S, dtype, max_blocks and k are read.  Asynchronous like
 * scout_host_submit and sharing its two places (one running, one behind it): 0
 * once the work is handed in (wait with scout_host_wait), -1 on a bad argument or
 * a buffer too small, -6 if a job is waiting already.
 */
int scout_host_stage_recall(scout_host_worker* w, const scout_host_problem* p, const void* k_blocks,
                            const void* v_blocks, const int32_t* recall_blk, const int32_t* n_recall,
                            void* staged, size_t staged_bytes, int32_t* tile_off, int64_t* total_tiles);

/*
 * Block until the OLDEST job not yet reported is done (0): jobs are reported in
 * the order they were handed in, one per call.  Returns 0 at once if none is
 * outstanding.  *seconds, if not NULL, receives the time from the job's start
 * on the threads to its last pair's completion (0 if none was outstanding).
 */
int scout_host_wait(scout_host_worker* w, double* seconds);

/* 1 if every job handed in has finished (or none was), else 0.  Never blocks. */
int scout_host_done(scout_host_worker* w);

#ifdef __cplusplus
}
#endif
#endif /* SCOUT_HOST_H */
