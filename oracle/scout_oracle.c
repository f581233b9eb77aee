/*
 * scout_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision CPU statement of what the GPU side of
 * GPU-CPU collaborative block-wise sparse decode attention computes
 * (ScoutAttention, Sec. 3.2 and Algorithm 1; digest as in Sec. 2.2).
 * It exists to be compared against: only tests, the smoke check and the
 * CPU-baseline leg of the benchmark may call it.  It shares no code, table
 * or helper with the HIP library and is never used as a fallback.
 *
 * Every function works on ONE (sequence, KV head) pair and, where a query
 * head is involved, on one head at a time, with scalar loops in the order
 * the definitions are written.  No blocking, fusion or reordering.
 *
 * Stored element types: ORC_F32 (IEEE binary32) and ORC_BF16 (the upper 16
 * bits of a binary32).  Both convert to binary64 exactly, and all arithmetic
 * after that conversion is binary64.
 *
 * Pins (tests/test_oracle_*.py): digest against an array min/max; score
 * against its upper-bound property, the one-token-block special case (plain
 * dot product), translation equivariance and a folded group form; selection
 * against a brute-force sort; partial attention against a library dense
 * attention routine when the selection covers everything, against closed
 * forms and against weight normalisation; merge against attention over the
 * union of a split; recall plan against brute-force set arithmetic; decode
 * append against the digest and the tiles of the finished sequence built in
 * one piece; recall transfer against plain slicing of the source array;
 * always-kept blocks against a brute-force statement of the same rule; the
 * max-over-heads score against an array computation and its G = 1 case.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };

static double ld(const void* p, int dtype, size_t i) {
  if (dtype == ORC_F32) return (double)((const float*)p)[i];
  uint32_t u = (uint32_t)((const uint16_t*)p)[i] << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static size_t esize(int dtype) { return dtype == ORC_F32 ? 4 : 2; }

/* Number of blocks that hold at least one valid token. */
int orc_num_blocks(int ctx_len, int S) { return (ctx_len + S - 1) / S; }

/*
 * Block digest (Sec. 2.2: channel-wise min and max pooling over the keys of
 * a block).  K is the pair's logical key matrix [ctx_len][d]; block j holds
 * tokens j*S .. min(ctx_len,(j+1)*S)-1.  Only valid tokens are pooled.
 * dig is [nb][2][d] in the storage type: row 0 the minimum, row 1 the
 * maximum.  Min/max never round, so the stored element is copied bit for bit.
 */
void orc_digest(int dtype, const void* K, int ctx_len, int S, int d, void* dig) {
  int nb = orc_num_blocks(ctx_len, S);
  size_t es = esize(dtype);
  for (int j = 0; j < nb; ++j) {
    int t0 = j * S, t1 = t0 + S < ctx_len ? t0 + S : ctx_len;
    for (int c = 0; c < d; ++c) {
      size_t imin = (size_t)t0 * d + c, imax = imin;
      for (int t = t0 + 1; t < t1; ++t) {
        size_t i = (size_t)t * d + c;
        if (ld(K, dtype, i) < ld(K, dtype, imin)) imin = i;
        if (ld(K, dtype, i) > ld(K, dtype, imax)) imax = i;
      }
      memcpy((char*)dig + (((size_t)j * 2 + 0) * d + c) * es, (const char*)K + imin * es, es);
      memcpy((char*)dig + (((size_t)j * 2 + 1) * d + c) * es, (const char*)K + imax * es, es);
    }
  }
}

/*
 * Block importance (Sec. 2.2 / Sec. 3.2: the query against each block's
 * digest; with a min/max digest the per-channel contribution is the larger of
 * q*min and q*max, which bounds q.k over the block from above).  The G query
 * heads that share the KV head contribute the sum of their estimates.
 * q is [G][d], dig is [nb][2][d]; s is [nb] in binary64, unscaled.
 */
void orc_score(int dtype, const void* q, const void* dig, int nb, int G, int d, double* s) {
  for (int j = 0; j < nb; ++j) {
    double sg = 0.0;
    for (int h = 0; h < G; ++h) {
      double sh = 0.0;
      for (int c = 0; c < d; ++c) {
        double qc = ld(q, dtype, (size_t)h * d + c);
        double lo = qc * ld(dig, dtype, ((size_t)j * 2 + 0) * d + c);
        double hi = qc * ld(dig, dtype, ((size_t)j * 2 + 1) * d + c);
        sh += lo > hi ? lo : hi;
      }
      sg += sh;
    }
    s[j] = sg;
  }
}

/* Total order used everywhere: higher score first, equal scores by lower index. */
typedef struct { double s; int j; } orc_key;
static int key_before(const void* a, const void* b) {
  const orc_key* x = (const orc_key*)a;
  const orc_key* y = (const orc_key*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return x->j < y->j ? -1 : (x->j > y->j ? 1 : 0);
}
static int int_up(const void* a, const void* b) {
  int x = *(const int*)a, y = *(const int*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

/*
 * Rank all nb blocks by the total order.  rank[i] = index of the i-th best.
 */
void orc_rank(const double* s, int nb, int* rank) {
  orc_key* keys = (orc_key*)malloc(sizeof(orc_key) * (size_t)(nb > 0 ? nb : 1));
  for (int j = 0; j < nb; ++j) { keys[j].s = s[j]; keys[j].j = j; }
  qsort(keys, (size_t)nb, sizeof(orc_key), key_before);
  for (int i = 0; i < nb; ++i) rank[i] = keys[i].j;
  free(keys);
}

/*
 * Top-k selection (Algorithm 1, the TopK step): the k_eff = min(k, nb) first
 * blocks of the ranking, reported in ascending block index.  sel has room for
 * k entries; unused entries are -1.  Returns k_eff.
 */
int orc_select(const double* s, int nb, int k, int* sel) {
  int* rank = (int*)malloc(sizeof(int) * (size_t)(nb > 0 ? nb : 1));
  orc_rank(s, nb, rank);
  int ke = k < nb ? k : nb;
  for (int i = 0; i < ke; ++i) sel[i] = rank[i];
  qsort(sel, (size_t)ke, sizeof(int), int_up);
  for (int i = ke; i < k; ++i) sel[i] = -1;
  free(rank);
  return ke;
}

/*
 * Residency split (Algorithm 1: the predicted blocks minus the GPU-resident
 * ones go to the host).  table[j] >= 0 is the pool slot of a resident block,
 * -1 marks a block kept in host memory.  Order (ascending index) is kept.
 */
void orc_split(const int* sel, int n_sel, const int* table, int k,
               int* sel_gpu, int* n_gpu, int* sel_host, int* n_host) {
  int ng = 0, nh = 0;
  for (int i = 0; i < n_sel; ++i) {
    if (table[sel[i]] >= 0) sel_gpu[ng++] = sel[i];
    else sel_host[nh++] = sel[i];
  }
  for (int i = ng; i < k; ++i) sel_gpu[i] = -1;
  for (int i = nh; i < k; ++i) sel_host[i] = -1;
  *n_gpu = ng;
  *n_host = nh;
}

/*
 * Partial attention of ONE query head over a set of blocks (Sec. 3.2: each
 * device attends to its share of the selected blocks and hands over an
 * intermediate result that a FlashAttention-style merge can combine).
 * K, V: the pair's logical [ctx_len][d] matrices; blocks: nblk logical block
 * indices; q_h: [d].  With x_t = sm_scale * q.k_t over every valid token t of
 * every listed block:  m = max x_t,  l = sum exp(x_t - m),
 * o = sum exp(x_t - m) v_t / l.  Empty set: o = 0, m = -inf, l = 0.
 */
void orc_partial_attn(int dtype, const void* q_h, const void* K, const void* V,
                      const int* blocks, int nblk, int ctx_len, int S, int d,
                      double sm_scale, double* o, double* m, double* l) {
  double mx = -INFINITY;
  for (int i = 0; i < nblk; ++i) {
    int t0 = blocks[i] * S, t1 = t0 + S < ctx_len ? t0 + S : ctx_len;
    for (int t = t0; t < t1; ++t) {
      double x = 0.0;
      for (int c = 0; c < d; ++c) x += ld(q_h, dtype, c) * ld(K, dtype, (size_t)t * d + c);
      x *= sm_scale;
      if (x > mx) mx = x;
    }
  }
  double sum = 0.0;
  for (int c = 0; c < d; ++c) o[c] = 0.0;
  for (int i = 0; i < nblk; ++i) {
    int t0 = blocks[i] * S, t1 = t0 + S < ctx_len ? t0 + S : ctx_len;
    for (int t = t0; t < t1; ++t) {
      double x = 0.0;
      for (int c = 0; c < d; ++c) x += ld(q_h, dtype, c) * ld(K, dtype, (size_t)t * d + c);
      x *= sm_scale;
      double p = exp(x - mx);
      sum += p;
      for (int c = 0; c < d; ++c) o[c] += p * ld(V, dtype, (size_t)t * d + c);
    }
  }
  if (sum > 0.0)
    for (int c = 0; c < d; ++c) o[c] /= sum;
  *m = mx;
  *l = sum;
}

/*
 * Merge of two partial results (Algorithm 1, the Merge step; the rescaling
 * rule of FlashAttention).  A side with l = 0 has weight 0 and its m is never
 * subtracted.  Both empty: out = 0, lse = -inf.
 */
void orc_merge(const double* o_a, double m_a, double l_a,
               const double* o_b, double m_b, double l_b, int d,
               double* out, double* lse) {
  double ms = -INFINITY;
  if (l_a > 0.0 && m_a > ms) ms = m_a;
  if (l_b > 0.0 && m_b > ms) ms = m_b;
  double wa = l_a > 0.0 ? l_a * exp(m_a - ms) : 0.0;
  double wb = l_b > 0.0 ? l_b * exp(m_b - ms) : 0.0;
  double ls = wa + wb;
  for (int c = 0; c < d; ++c) {
    double acc = 0.0;
    if (wa > 0.0) acc += wa * o_a[c];
    if (wb > 0.0) acc += wb * o_b[c];
    out[c] = ls > 0.0 ? acc / ls : 0.0;
  }
  *lse = ls > 0.0 ? ms + log(ls) : -INFINITY;
}

/*
 * Recall plan for one pair (Sec. 3.4: at a recall step, after the layer's
 * attention, the blocks that are important now but live in host memory are
 * brought back; the paper leaves the eviction rule open, the reading taken
 * here moves as little as possible).  With T the top-k set for the current
 * scores and R the resident set:
 *   recall  = T \ R; if it is larger than R \ T, only its best-ranked
 *             |R \ T| members are recalled;
 *   evict   = the |recall| worst-ranked members of R \ T;
 *   both are reported in ascending block index and the i-th recalled block
 *   takes the slot of the i-th evicted block; table is updated in place.
 * Arrays have room for k entries, unused entries are -1.  Returns n_recall.
 */
int orc_recall_plan(const double* s, int nb, int k, int* table,
                    int* recall_blk, int* recall_slot, int* evict_blk) {
  int* rank = (int*)malloc(sizeof(int) * (size_t)(nb > 0 ? nb : 1));
  orc_rank(s, nb, rank);
  int ke = k < nb ? k : nb;
  int n_missing = 0, n_spare = 0;
  for (int i = 0; i < ke; ++i)
    if (table[rank[i]] < 0) ++n_missing;
  for (int i = ke; i < nb; ++i)
    if (table[rank[i]] >= 0) ++n_spare;
  int n = n_missing < n_spare ? n_missing : n_spare;
  int nr = 0, ne = 0;
  for (int i = 0; i < ke && nr < n; ++i)          /* best-ranked missing first */
    if (table[rank[i]] < 0) recall_blk[nr++] = rank[i];
  for (int i = nb - 1; i >= ke && ne < n; --i)    /* worst-ranked spare first */
    if (table[rank[i]] >= 0) evict_blk[ne++] = rank[i];
  qsort(recall_blk, (size_t)n, sizeof(int), int_up);
  qsort(evict_blk, (size_t)n, sizeof(int), int_up);
  for (int i = 0; i < n; ++i) {
    recall_slot[i] = table[evict_blk[i]];
    table[recall_blk[i]] = recall_slot[i];
    table[evict_blk[i]] = -1;
  }
  for (int i = n; i < k; ++i) { recall_blk[i] = -1; recall_slot[i] = -1; evict_blk[i] = -1; }
  free(rank);
  return n;
}

/*
 * Decode append for one pair (the digest of Sec. 2.2 kept up to date while the
 * sequence of Sec. 3.2 grows by the token that decode just produced).
 * The token takes position t = ctx_len, row r = t % S of block j = t / S:
 *   - r == 0 opens block j: its table entry becomes new_slot (>= 0: a pool
 *     slot on the GPU, -1: the block lives on the host) and both digest rows
 *     become the key; otherwise a digest element is replaced only where the
 *     key is strictly smaller (row 0) or strictly larger (row 1);
 *   - if the block's table entry is a slot in [0, n_slots), the key and the
 *     value are written to row r of that slot's K and V tiles;
 *   - if the host keeps a copy of every block (host_k / host_v not NULL,
 *     [max_blocks][S][d] by logical index), the rows are written there as well,
 *     whatever the residency: the copy a later recall reads from and the reason
 *     an eviction has nothing to move.
 * dig is [max_blocks][2][d], table [max_blocks], the pools [n_slots][S][d].
 * Returns the new length: ctx_len + 1, or ctx_len unchanged (and nothing
 * written) when the sequence already fills max_blocks blocks.
 */
int orc_append(int dtype, int S, int d, int max_blocks, int ctx_len, const void* k_new,
               const void* v_new, int new_slot, void* dig, int* table, void* k_pool,
               void* v_pool, long n_slots, void* host_k, void* host_v) {
  if (ctx_len >= max_blocks * S) return ctx_len;
  size_t es = esize(dtype);
  int j = ctx_len / S, r = ctx_len % S;
  if (r == 0) table[j] = new_slot;
  char* dmin = (char*)dig + ((size_t)j * 2 + 0) * d * es;
  char* dmax = (char*)dig + ((size_t)j * 2 + 1) * d * es;
  for (int c = 0; c < d; ++c) {
    const char* kc = (const char*)k_new + (size_t)c * es;
    if (r == 0 || ld(k_new, dtype, c) < ld(dmin, dtype, c)) memcpy(dmin + (size_t)c * es, kc, es);
    if (r == 0 || ld(k_new, dtype, c) > ld(dmax, dtype, c)) memcpy(dmax + (size_t)c * es, kc, es);
  }
  int slot = table[j];
  if (slot >= 0 && slot < n_slots) {
    size_t row = ((size_t)slot * S + r) * d * es;
    memcpy((char*)k_pool + row, k_new, (size_t)d * es);
    memcpy((char*)v_pool + row, v_new, (size_t)d * es);
  }
  if (host_k != NULL && host_v != NULL) {   /* the host's copy of every block, [max_blocks][S][d] */
    size_t row = ((size_t)j * S + r) * d * es;
    memcpy((char*)host_k + row, k_new, (size_t)d * es);
    memcpy((char*)host_v + row, v_new, (size_t)d * es);
  }
  return ctx_len + 1;
}

/*
 * Data movement of a periodic recall for one pair (Sec. 3.4: the blocks the
 * plan names come back from host memory into the pool slots that the plan
 * freed).  src_k / src_v hold the pair's blocks by logical index,
 * [max_blocks][S][d]; entry i < n of the plan copies the K and V tiles of
 * block recall_blk[i] into slot recall_slot[i] of the pools [n_slots][S][d].
 * Entries outside [0, max_blocks) x [0, n_slots) are skipped.  Returns the
 * number of tiles copied (K and V count as one).
 */
int orc_recall_fetch(int dtype, int S, int d, int max_blocks, const void* src_k, const void* src_v,
                     const int* recall_blk, const int* recall_slot, int n, void* k_pool,
                     void* v_pool, long n_slots) {
  size_t tile = (size_t)S * d * esize(dtype);
  int copied = 0;
  for (int i = 0; i < n; ++i) {
    int blk = recall_blk[i], slot = recall_slot[i];
    if (blk < 0 || blk >= max_blocks || slot < 0 || slot >= n_slots) continue;
    memcpy((char*)k_pool + (size_t)slot * tile, (const char*)src_k + (size_t)blk * tile, tile);
    memcpy((char*)v_pool + (size_t)slot * tile, (const char*)src_v + (size_t)blk * tile, tile);
    ++copied;
  }
  return copied;
}

/*
 * Mean-pooled block digest (Sec. 2.2 names mean pooling over a block's keys as
 * the other common digest; a variant of the min/max digest the method uses).
 * It is stored as the SUM of the block's valid keys in binary32, added in token
 * order, so that an append extends it by one addition and a digest built at once
 * equals one grown token by token; the mean is sum / count where it is used.
 * K is [ctx_len][d]; out is f32 [ceil(ctx_len/S)][d].
 */
void orc_digest_sum(int dtype, const void* K, int ctx_len, int S, int d, float* out) {
  int nb = (ctx_len + S - 1) / S;
  for (int j = 0; j < nb; ++j) {
    int t0 = j * S, t1 = t0 + S < ctx_len ? t0 + S : ctx_len;
    for (int c = 0; c < d; ++c) {
      float sum = (float)ld(K, dtype, (size_t)t0 * d + c);
      for (int t = t0 + 1; t < t1; ++t) {
        volatile float next = sum + (float)ld(K, dtype, (size_t)t * d + c); /* one binary32 rounding per token */
        sum = next;
      }
      out[(size_t)j * d + c] = sum;
    }
  }
}

/* The append of one key to that digest: the token at position ctx_len opens block ctx_len / S with
 * its key, or is added to the block's sum (binary32).  sums is f32 [max_blocks][d].  Nothing happens
 * when the sequence already fills max_blocks blocks. */
void orc_append_sum(int dtype, int S, int d, int max_blocks, int ctx_len, const void* k_new, float* sums) {
  if (ctx_len >= max_blocks * S) return;
  int j = ctx_len / S, r = ctx_len % S;
  for (int c = 0; c < d; ++c) {
    float k = (float)ld(k_new, dtype, c);
    volatile float next = sums[(size_t)j * d + c] + k;
    sums[(size_t)j * d + c] = r == 0 ? k : next;
  }
}

/*
 * Block importance with the mean-pooled digest: the query against the block's
 * mean key, summed over the G query heads of the KV head,
 *   s_j = sum_h sum_c q[h][c] * sums[j][c] / count_j,
 * count_j the number of valid tokens of block j.  q is [G][d], sums f32 [nb][d].
 */
void orc_score_mean(int dtype, const void* q, const float* sums, int nb, int G, int d, int ctx_len, int S,
                    double* s) {
  for (int j = 0; j < nb; ++j) {
    int count = ctx_len - j * S;
    if (count > S) count = S;
    double acc = 0.0;
    for (int h = 0; h < G; ++h)
      for (int c = 0; c < d; ++c) acc += ld(q, dtype, (size_t)h * d + c) * (double)sums[(size_t)j * d + c];
    s[j] = acc / (double)count;
  }
}

/*
 * The same recall through a staging buffer (Sec. 3.4, asynchronous transfer:
 * the host packs the planned tiles so that they cross the host link as one
 * contiguous copy, the device then puts them into their slots).
 *
 * Stage (host side): over all pairs, the tiles named by the first
 * min(n_recall[pair], k) plan entries of each pair are packed in pair order,
 * entry order: tile t = tile_off[pair] + i holds K at byte t*2*tile and V at
 * t*2*tile + tile.  An entry whose block index is outside [0, max_blocks)
 * keeps its place but nothing is written there.  src_k / src_v are
 * [pairs][max_blocks][S][d], recall_blk is [pairs][k], tile_off is [pairs]
 * (out).  Returns the total number of tiles.
 */
long orc_recall_stage(int dtype, int S, int d, int max_blocks, int k, int pairs, const void* src_k,
                      const void* src_v, const int* recall_blk, const int* n_recall, void* staged,
                      int* tile_off) {
  size_t tile = (size_t)S * d * esize(dtype);
  long t = 0;
  for (int p = 0; p < pairs; ++p) {
    int n = n_recall[p];
    if (n < 0) n = 0;
    if (n > k) n = k;
    tile_off[p] = (int)t;
    for (int i = 0; i < n; ++i, ++t) {
      int blk = recall_blk[(size_t)p * k + i];
      if (blk < 0 || blk >= max_blocks) continue;
      size_t from = ((size_t)p * max_blocks + blk) * tile;
      memcpy((char*)staged + (size_t)t * 2 * tile, (const char*)src_k + from, tile);
      memcpy((char*)staged + (size_t)t * 2 * tile + tile, (const char*)src_v + from, tile);
    }
  }
  return t;
}

/*
 * Scatter (device side): entry i of a pair takes staged tile tile_off[pair] + i
 * to pool slot recall_slot[pair][i]; entries with a block index outside
 * [0, max_blocks) or a slot outside [0, n_slots) are skipped, as in
 * orc_recall_fetch.  Returns the number of tiles placed.
 */
long orc_recall_scatter(int dtype, int S, int d, int max_blocks, int k, int pairs, const void* staged,
                        const int* tile_off, const int* recall_blk, const int* recall_slot,
                        const int* n_recall, void* k_pool, void* v_pool, long n_slots) {
  size_t tile = (size_t)S * d * esize(dtype);
  long placed = 0;
  for (int p = 0; p < pairs; ++p) {
    int n = n_recall[p];
    if (n < 0) n = 0;
    if (n > k) n = k;
    for (int i = 0; i < n; ++i) {
      int blk = recall_blk[(size_t)p * k + i], slot = recall_slot[(size_t)p * k + i];
      if (blk < 0 || blk >= max_blocks || slot < 0 || slot >= n_slots) continue;
      size_t t = (size_t)tile_off[p] + i;
      memcpy((char*)k_pool + (size_t)slot * tile, (const char*)staged + t * 2 * tile, tile);
      memcpy((char*)v_pool + (size_t)slot * tile, (const char*)staged + t * 2 * tile + tile, tile);
      ++placed;
    }
  }
  return placed;
}

/*
 * Always-kept blocks (a variant of the selection rule of Alg. 1's TopK: the
 * first n_sink blocks of a sequence and the last n_tail blocks that hold
 * tokens are selected whatever their score).  They are given the score
 * +infinity, so the ordinary selection keeps them first, lower index first
 * among them if the budget cannot hold them all; they count against k.
 * s is [nb], changed in place.
 */
void orc_force_blocks(double* s, int nb, int n_sink, int n_tail) {
  for (int j = 0; j < nb; ++j)
    if (j < n_sink || j >= nb - n_tail) s[j] = INFINITY;
}

/*
 * Block importance with the group's heads combined by their maximum instead
 * of their sum (a variant of the selection argument of Alg. 1: a block matters
 * to the KV head if it matters to any of the query heads that share it).  Per
 * head the estimate is the one of orc_score: sum over channels of the larger
 * of q*min and q*max.  q is [G][d], dig is [nb][2][d]; s is [nb], unscaled.
 */
void orc_score_max(int dtype, const void* q, const void* dig, int nb, int G, int d, double* s) {
  for (int j = 0; j < nb; ++j) {
    double best = -INFINITY;
    for (int h = 0; h < G; ++h) {
      double sh = 0.0;
      for (int c = 0; c < d; ++c) {
        double qc = ld(q, dtype, (size_t)h * d + c);
        double lo = qc * ld(dig, dtype, ((size_t)j * 2 + 0) * d + c);
        double hi = qc * ld(dig, dtype, ((size_t)j * 2 + 1) * d + c);
        sh += lo > hi ? lo : hi;
      }
      if (sh > best) best = sh;
    }
    s[j] = best;
  }
}
