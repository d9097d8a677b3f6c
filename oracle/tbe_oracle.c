/*
 * CPU oracle for the cached embedding-bag training path.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP library and to be timed as the CPU baseline; nothing on
 * the product path may call it, and it shares no code with the HIP sources.
 *
 * What it computes (paper sections in brackets):
 *   - pooled lookup: for every (table, sample) bag, the sum of the looked-up rows
 *     [Section 2.1.1];
 *   - sparse backward with row-wise Adagrad: every distinct row of a batch receives the
 *     sum of the output gradients of the bags that looked it up (once per lookup), one
 *     accumulator per row [Section 2.1.2: optimizers with few states per row, Adagrad;
 *     Section 5.9: the GPU aggregates, runs the optimizer and updates the weights in the
 *     memory they live in during backward];
 *   - a one-level software cache of raw rows with tags and per-entry timestamps
 *     [Section 5.3.1], managed per batch in the order the paper lists [Section 5.5.2]:
 *     1) stamp the hits, 2) choose slots for the misses, 3) evict when no slot is free;
 *     a missed row is inserted into the cache from the lower tier and the least recently
 *     used row is written back to it [Section 5.5.4]; rows fetched for a batch stay in
 *     the cache until that batch has trained [Section 5.7].
 *
 * Readings where the paper is silent (the HIP path follows the same ones):
 *   - organisation: each table has its own W-way set-associative cache, set(r) = r mod S;
 *   - time = batch id k = 1, 2, ... given at prefetch; free entries carry timestamp -1;
 *   - inside one batch the distinct rows of a table are handled in two phases: all hits
 *     are stamped k first, then the misses in ascending row order; the victim of a miss
 *     is the way with the smallest timestamp < k, the lowest way among equals;
 *   - when every way of the set already carries timestamp k the row is not inserted
 *     ("bypass"): it is read from and updated in the lower tier directly;
 *   - prefetching D batches ahead [Section 5.7: rows fetched for a batch are not evicted before it
 *     has trained]: optional; the ways stamped k-D .. k-1 are then locked like those stamped k (the
 *     batches that would still be waiting for their training when batch k is fetched);
 *   - every evicted row is written back (rows are trained on after insertion, so all
 *     lines are dirty); flush writes back every valid line and keeps the tags;
 *   - row-wise Adagrad: m += mean_d(g_d^2); w_d -= lr * g_d / (sqrt(m) + eps), m starts
 *     wherever the caller's state array starts (0 in the tests), eps outside the root;
 *   - fp16 storage: rows are widened exactly, results are rounded to nearest even;
 *   - two-level exclusive cache [Section 5.3, 5.5.4]: a second, larger set-associative cache
 *     (set2(r) = r mod S2, same number of ways, timestamps of its own) sits between the first
 *     level and the lower tier; a row lives in exactly one of the three places.  Per batch,
 *     after the first level has decided: (A) every row the first level missed is looked up
 *     in the second level -- found and inserted into the first level: it moves up and its
 *     second-level entry becomes free; found but bypassed by the first level: it stays, is
 *     used in place and is stamped k; not found: it comes from / stays in the lower tier --
 *     then (B) the rows the first level evicted move down, in ascending row order, each into
 *     the way of its second-level set with the smallest timestamp < k - 1 (free first, lowest
 *     way among equals), stamped k; what that way held is written back to the lower tier;
 *     with no such way the row goes to the lower tier directly.  An entry stamped by this
 *     batch or the one before is thus never replaced: its data may still be on its way
 *     (the paper's pipelining rule, Section 5.7, applied to the second level, whose moves
 *     trail the decisions by a batch).  The second level is always LRU by the time a row
 *     entered it (or was last used in place);
 *   - deferred initialisation on read [Section 5.4.2]: with it enabled a row of the lower tier
 *     has no value until it is first read from there (a first-level miss that the second
 *     level does not hold); it is then given normal random values, std * z, z from a
 *     counter-based generator of (seed, table, row, element) -- so the values do not depend on
 *     the order of the reads and equal a table initialised in advance with the same
 *     generator: z is the centred sum of twelve 16-bit uniforms (three 64-bit hashes per
 *     element), the classic twelve-uniform approximation of a normal number (mean 0, variance
 *     1, |z| < 6) -- integer arithmetic up to one fp32 multiplication by std * 2^-17, which is
 *     fixed to fp32 so that both sides store bit-identical values (with max pooling a value
 *     that differed in its last bit could change which lookup supplies a maximum);
 *   - mean pooling, the second pooling mode the paper names [Section 2.1.1]: the pooled
 *     vector is the sum divided by the number of lookups of the bag (a row looked up twice
 *     counts twice; an empty bag gives zeros), so a lookup of a bag of L lookups hands
 *     1/L of the bag's output gradient to its row;
 *   - max pooling, the third pooling mode [Section 2.1.1]: element d of the pooled vector is
 *     the largest element d among the bag's rows (an empty bag gives zeros); in backward the
 *     bag's output gradient of element d goes to the lookup that supplied the maximum, the
 *     first such lookup of the bag when several tie, and to no other;
 *   - LFU, the other policy the paper tried [Section 5.5.2; it gives no details]: every
 *     entry also counts the lookups of its row since it was inserted (a row looked up c
 *     times in a batch adds c; the count saturates at INT32_MAX and is forgotten at
 *     eviction; free entries count 0).  The two phases, the lock of the ways stamped k
 *     and the bypass rule are those of LRU; only the choice of the victim differs: the
 *     smallest count, the smallest timestamp among equal counts, the lowest way after that.
 * All floating-point work is done in fp64 from the stored values and rounded once when
 * stored (fp32 state, fp32 or fp16 weights, fp32 pooled output).
 *
 * Plain C, no blocking or fusion: each function is the definition written out.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ERANGE (-2)
#define ORC_EORDER (-3)
#define ORC_ENOMEM (-4)

#define ORC_POOL_SUM 0
#define ORC_POOL_MEAN 1
#define ORC_POOL_MAX 2

#define ORC_LRU 0
#define ORC_LFU 1

typedef struct {
  int64_t rows;        /* H_t */
  int32_t dim;         /* D_t */
  int32_t dtype;       /* 0 = fp32, 1 = fp16 storage */
  void *weights;       /* caller-owned backing tier [rows, dim] */
  float *state;        /* caller-owned backing tier accumulator [rows] */
  int64_t cache_slots; /* S_t = cache_slots / ways (floor) */
} orc_table_spec;

typedef struct {
  int64_t lookups, uniques, hits, inserts, bypasses, evictions, hit_lookups;
} orc_stats;

typedef struct {
  int64_t rows;
  int32_t dim, dtype;
  void *weights;
  float *state;
  int64_t sets;
  int64_t *tag;     /* [sets*ways], -1 = free */
  int32_t *ts;      /* [sets*ways], -1 = free */
  int32_t *freq;    /* [sets*ways], lookups since insertion (kept under both policies, used by LFU) */
  void *lines;      /* [sets*ways, dim] in the storage type */
  float *line_state;/* [sets*ways] */
  /* second level (absent when sets2 == 0) */
  int64_t sets2;
  int64_t *tag2;    /* [sets2*ways], -1 = free */
  int32_t *ts2;     /* [sets2*ways], -1 = free */
  void *lines2;
  float *line_state2;
  int64_t l2_hits, l2_demotions, l2_evictions, l2_bypasses; /* of the last batch */
  unsigned char *initialised; /* deferred initialisation: [rows] 1 = the row has a value (null = off) */
  int32_t index;              /* table number (enters the generator) */
  float *peak;      /* [rows] bookkeeping for the tests, enters no result: the largest |element| a row has
                       held before or after any of its updates (0 = never updated) */
  /* last prefetched batch */
  int64_t n_uniq;
  int64_t *uniq;    /* sorted distinct rows */
  int64_t *mult;    /* lookups per distinct row */
  /* events of the last prefetch */
  int64_t n_hit, n_ins, n_byp;
  int64_t *hit_row;
  int64_t *ins_row, *ins_slot, *ins_old;
  int64_t *byp_row;
  int64_t cap;
  orc_stats st;
} orc_table;

typedef struct {
  int32_t T, ways;
  int32_t policy;      /* ORC_LRU or ORC_LFU */
  int32_t pooling;     /* ORC_POOL_SUM or ORC_POOL_MEAN */
  int deferred;        /* deferred initialisation on read */
  uint64_t init_seed;
  double init_std;
  orc_table *tab;
  int32_t k;           /* batch id of the last prefetch */
  int32_t B;
  int64_t N;
  int64_t *indices;
  int64_t *offsets;
  int64_t cap_idx, cap_off;
  int64_t *argmax;     /* max pooling: [B * sum of dims] lookup (position in indices) that supplied each maximum, -1 = empty bag */
  int64_t cap_arg;
  int forwarded, prefetched;
  int threads;
  int32_t lock1;       /* first level: ways stamped within the last `lock1` batches before the current one are locked
                          like the current batch's own (0 = only those; D = the rule of Section 5.7 for a pipeline
                          that fetches D batches ahead: a row fetched for a batch stays until that batch has trained) */
  int32_t lock2;       /* second level: entries stamped within the last `lock2` batches (the current one included)
                          are not replaced.  2 = the reading the library follows (this batch and the one before);
                          1 = the plain reading of Section 5.7 (this batch only), kept for the comparison of the two */
  orc_stats last, total;
  int64_t l2_last[4], l2_total[4]; /* hits, demotions, evictions, bypasses of the second level */
} orc;

/* ---------------- fp16 <-> fp64 ---------------- */

static double half_to_double(uint16_t h) {
  int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0) v = ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(m | 1024), e - 25);
  return s ? -v : v;
}

/* round to nearest, ties to even, straight from fp64 (no intermediate fp32) */
static uint16_t double_to_half(double x) {
  uint64_t b;
  memcpy(&b, &x, 8);
  uint16_t sign = (uint16_t)((b >> 48) & 0x8000u);
  int64_t e = (int64_t)((b >> 52) & 0x7ff);
  uint64_t m = b & ((1ull << 52) - 1);
  if (e == 0x7ff) return (uint16_t)(sign | 0x7c00u | (m ? 0x200u : 0));
  if (e == 0) return sign;
  int64_t he = e - 1023 + 15;
  if (he >= 31) return (uint16_t)(sign | 0x7c00u);
  if (he >= 1) {
    uint32_t r = (uint32_t)((he << 10) | (int64_t)(m >> 42));
    uint64_t rem = m & ((1ull << 42) - 1), half = 1ull << 41;
    if (rem > half || (rem == half && (r & 1))) r++;
    return (uint16_t)(sign | r);
  }
  uint64_t M = m | (1ull << 52);
  int64_t shift = 1051 - e; /* result in units of 2^-24 */
  if (shift >= 64) return sign;
  uint64_t q = M >> shift, rem = M & ((1ull << shift) - 1), half = 1ull << (shift - 1);
  if (rem > half || (rem == half && (q & 1))) q++;
  return (uint16_t)(sign | (uint16_t)q);
}

uint16_t orc_double_to_half(double x) { return double_to_half(x); }
double orc_half_to_double(uint16_t h) { return half_to_double(h); }

static double load_elem(const void *base, int dtype, int64_t i) {
  return dtype == 0 ? (double)((const float *)base)[i] : half_to_double(((const uint16_t *)base)[i]);
}
static void store_elem(void *base, int dtype, int64_t i, double v) {
  if (dtype == 0) ((float *)base)[i] = (float)v;
  else ((uint16_t *)base)[i] = double_to_half(v);
}
static size_t esize(int dtype) { return dtype == 0 ? 4 : 2; }

/* ---------------- life cycle ---------------- */

static void free_table(orc_table *t) {
  free(t->tag); free(t->ts); free(t->freq); free(t->lines); free(t->line_state);
  free(t->tag2); free(t->ts2); free(t->lines2); free(t->line_state2); free(t->initialised); free(t->peak);
  free(t->uniq); free(t->mult); free(t->hit_row); free(t->ins_row);
  free(t->ins_slot); free(t->ins_old); free(t->byp_row);
}

void orc_destroy(void *hp) {
  orc *h = (orc *)hp;
  if (!h) return;
  for (int t = 0; t < h->T; t++) free_table(&h->tab[t]);
  free(h->tab); free(h->indices); free(h->offsets); free(h->argmax); free(h);
}

void *orc_create(const orc_table_spec *specs, int32_t T, int32_t ways) {
  if (!specs || T <= 0 || ways <= 0) return NULL;
  orc *h = (orc *)calloc(1, sizeof(orc));
  if (!h) return NULL;
  h->T = T; h->ways = ways; h->threads = 1; h->lock1 = 0; h->lock2 = 2;
  h->tab = (orc_table *)calloc((size_t)T, sizeof(orc_table));
  for (int t = 0; t < T; t++) {
    orc_table *tb = &h->tab[t];
    const orc_table_spec *s = &specs[t];
    if (s->rows <= 0 || s->dim <= 0 || (s->dtype != 0 && s->dtype != 1) || !s->weights || !s->state ||
        s->cache_slots < 0) { orc_destroy(h); return NULL; }
    tb->rows = s->rows; tb->dim = s->dim; tb->dtype = s->dtype;
    tb->weights = s->weights; tb->state = s->state;
    tb->sets = s->cache_slots / ways;
    tb->peak = (float *)calloc((size_t)s->rows, sizeof(float));
    if (!tb->peak) { orc_destroy(h); return NULL; }
    int64_t slots = tb->sets * ways;
    if (slots > 0) {
      tb->tag = (int64_t *)malloc(sizeof(int64_t) * (size_t)slots);
      tb->ts = (int32_t *)malloc(sizeof(int32_t) * (size_t)slots);
      tb->freq = (int32_t *)calloc((size_t)slots, sizeof(int32_t));
      tb->lines = calloc((size_t)slots * (size_t)s->dim, esize(s->dtype));
      tb->line_state = (float *)calloc((size_t)slots, sizeof(float));
      if (!tb->tag || !tb->ts || !tb->freq || !tb->lines || !tb->line_state) { orc_destroy(h); return NULL; }
      for (int64_t i = 0; i < slots; i++) { tb->tag[i] = -1; tb->ts[i] = -1; }
    }
  }
  return h;
}

void orc_set_threads(void *hp, int n) { ((orc *)hp)->threads = n > 0 ? n : 1; }

/* second-level cache of slots2[t] entries per table (whole sets of `ways`); only before the first batch */
/* Batches before the current one whose first-level entries are locked as well (see orc.lock1); before the first batch. */
int orc_set_prefetch_lock(void *hp, int32_t batches) {
  orc *h = (orc *)hp;
  if (!h || batches < 0 || batches > 64) return ORC_EINVAL;
  if (h->k != 0) return ORC_EORDER;
  h->lock1 = batches;
  return ORC_OK;
}

/* Batches whose second-level entries are locked (see orc.lock2): 1 or 2, before the first batch. */
int orc_set_second_level_lock(void *hp, int32_t batches) {
  orc *h = (orc *)hp;
  if (!h || batches < 1 || batches > 2) return ORC_EINVAL;
  if (h->k != 0) return ORC_EORDER;
  h->lock2 = batches;
  return ORC_OK;
}

int orc_set_second_level(void *hp, const int64_t *slots2) {
  orc *h = (orc *)hp;
  if (!h || !slots2) return ORC_EINVAL;
  if (h->k != 0) return ORC_EORDER;
  for (int t = 0; t < h->T; t++) {
    orc_table *tb = &h->tab[t];
    if (slots2[t] < 0 || tb->sets2) return ORC_EINVAL;
    tb->sets2 = slots2[t] / h->ways;
    int64_t n = tb->sets2 * h->ways;
    if (n == 0) continue;
    tb->tag2 = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
    tb->ts2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    tb->lines2 = calloc((size_t)n * (size_t)tb->dim, esize(tb->dtype));
    tb->line_state2 = (float *)calloc((size_t)n, sizeof(float));
    if (!tb->tag2 || !tb->ts2 || !tb->lines2 || !tb->line_state2) return ORC_ENOMEM;
    for (int64_t i = 0; i < n; i++) { tb->tag2[i] = -1; tb->ts2[i] = -1; }
  }
  return ORC_OK;
}

/* ---------------- deferred initialisation: the counter-based generator ---------------- */

static uint64_t mix64(uint64_t x) { /* the finaliser of splitmix64 */
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

/* Element d of row r of table t: S = sum over twelve 16-bit fields f of (2 f + 1), minus 12 * 65536
 * -- an integer with mean 0; z = S / 2^17 has variance 1 (twelve uniforms on (0, 1) minus 6). */
static int32_t init_sum(uint64_t seed, int32_t t, int64_t r, int32_t d) {
  uint64_t table_key = mix64(seed ^ ((uint64_t)(t + 1) * 0xD1342543DE82EF95ull));
  int64_t s = -12 * 65536;
  for (int j = 0; j < 3; j++) {
    uint64_t h = mix64(table_key + (uint64_t)r * 0x2545F4914F6CDD1Dull + (uint64_t)d * 3u + (uint64_t)j);
    for (int f = 0; f < 4; f++) s += 2 * (int64_t)((h >> (16 * f)) & 0xFFFFu) + 1;
  }
  return (int32_t)s;
}
int32_t orc_init_sum(uint64_t seed, int32_t t, int64_t r, int32_t d) { return init_sum(seed, t, r, d); }
/* the value itself, in the precision the definition fixes: one fp32 product */
static float init_value(uint64_t seed, float std, int32_t t, int64_t r, int32_t d) {
  float scale = std * 0x1p-17f; /* exact */
  return (float)init_sum(seed, t, r, d) * scale;
}
float orc_init_value(uint64_t seed, float std, int32_t t, int64_t r, int32_t d) { return init_value(seed, std, t, r, d); }

/* first read of a row from the lower tier gives it its value */
static void ensure_initialised(const orc *h, orc_table *tb, int64_t r) {
  if (!tb->initialised || tb->initialised[r]) return;
  for (int d = 0; d < tb->dim; d++)
    store_elem(tb->weights, tb->dtype, r * tb->dim + d, (double)init_value(h->init_seed, (float)h->init_std, tb->index, r, d));
  tb->initialised[r] = 1;
}

/* rows get their values on first read from the lower tier; only before the first batch */
int orc_enable_deferred_init(void *hp, uint64_t seed, double std) {
  orc *h = (orc *)hp;
  if (!h || !(std >= 0.0)) return ORC_EINVAL;
  if (h->k != 0 || h->deferred) return ORC_EORDER;
  for (int t = 0; t < h->T; t++) {
    h->tab[t].initialised = (unsigned char *)calloc((size_t)h->tab[t].rows, 1);
    if (!h->tab[t].initialised) return ORC_ENOMEM;
    h->tab[t].index = t;
  }
  h->deferred = 1; h->init_seed = seed; h->init_std = std;
  return ORC_OK;
}

int orc_export_initialised(void *hp, int32_t t, unsigned char *out) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T || !out || !h->tab[t].initialised) return ORC_EINVAL;
  memcpy(out, h->tab[t].initialised, (size_t)h->tab[t].rows);
  return ORC_OK;
}

/* pooling mode; only before the first batch */
int orc_set_pooling(void *hp, int32_t pooling) {
  orc *h = (orc *)hp;
  if (!h || (pooling != ORC_POOL_SUM && pooling != ORC_POOL_MEAN && pooling != ORC_POOL_MAX)) return ORC_EINVAL;
  if (h->k != 0) return ORC_EORDER;
  h->pooling = pooling;
  return ORC_OK;
}

/* replacement policy; only before the first batch */
int orc_set_policy(void *hp, int32_t policy) {
  orc *h = (orc *)hp;
  if (!h || (policy != ORC_LRU && policy != ORC_LFU)) return ORC_EINVAL;
  if (h->k != 0) return ORC_EORDER;
  h->policy = policy;
  return ORC_OK;
}

/* ---------------- cache primitives ---------------- */

/* slot of row r in table tb's cache, or -1 when it is not cached */
static int64_t find_slot(const orc_table *tb, int ways, int64_t r) {
  if (tb->sets == 0) return -1;
  int64_t s = r % tb->sets;
  for (int w = 0; w < ways; w++)
    if (tb->tag[s * ways + w] == r) return s * ways + w;
  return -1;
}

/* slot of row r in table tb's second-level cache, or -1 */
static int64_t find_slot2(const orc_table *tb, int ways, int64_t r) {
  if (tb->sets2 == 0) return -1;
  int64_t s = r % tb->sets2;
  for (int w = 0; w < ways; w++)
    if (tb->tag2[s * ways + w] == r) return s * ways + w;
  return -1;
}

/* where row r lives: first-level line, second-level line or lower tier */
static void locate_row(orc_table *tb, int ways, int64_t r, void **base, int64_t *index, float **state) {
  int64_t slot = find_slot(tb, ways, r);
  if (slot >= 0) { *base = tb->lines; *index = slot; *state = &tb->line_state[slot]; return; }
  slot = find_slot2(tb, ways, r);
  if (slot >= 0) { *base = tb->lines2; *index = slot; *state = &tb->line_state2[slot]; return; }
  *base = tb->weights; *index = r; *state = &tb->state[r];
}

static void line2_to_backing(orc_table *tb, int64_t slot2, int64_t r) {
  size_t rb = (size_t)tb->dim * esize(tb->dtype);
  memcpy((char *)tb->weights + (size_t)r * rb, (char *)tb->lines2 + (size_t)slot2 * rb, rb);
  tb->state[r] = tb->line_state2[slot2];
}

static void line_to_backing(orc_table *tb, int64_t slot, int64_t r) {
  size_t rb = (size_t)tb->dim * esize(tb->dtype);
  memcpy((char *)tb->weights + (size_t)r * rb, (char *)tb->lines + (size_t)slot * rb, rb);
  tb->state[r] = tb->line_state[slot];
}
static void backing_to_line(orc_table *tb, int64_t slot, int64_t r) {
  size_t rb = (size_t)tb->dim * esize(tb->dtype);
  memcpy((char *)tb->lines + (size_t)slot * rb, (char *)tb->weights + (size_t)r * rb, rb);
  tb->line_state[slot] = tb->state[r];
}

static int32_t add_saturating(int32_t a, int64_t b) {
  int64_t v = (int64_t)a + b;
  return v > INT32_MAX ? INT32_MAX : (int32_t)v;
}

static int cmp_i64(const void *a, const void *b) {
  int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
  return x < y ? -1 : x > y;
}

static int grow(orc_table *tb, int64_t n) {
  if (n <= tb->cap) return 0;
  int64_t c = n + n / 2 + 16;
  int64_t **ptrs[] = {&tb->uniq, &tb->mult, &tb->hit_row, &tb->ins_row, &tb->ins_slot, &tb->ins_old, &tb->byp_row};
  for (unsigned i = 0; i < sizeof(ptrs) / sizeof(ptrs[0]); i++) {
    int64_t *p = (int64_t *)realloc(*ptrs[i], sizeof(int64_t) * (size_t)c);
    if (!p) return -1;
    *ptrs[i] = p;
  }
  tb->cap = c;
  return 0;
}

typedef struct { int64_t row, slot; } orc_victim;
static int cmp_victim(const void *a, const void *b) {
  int64_t x = ((const orc_victim *)a)->row, y = ((const orc_victim *)b)->row;
  return x < y ? -1 : x > y;
}

/* Second level, after the first level has taken its decisions for batch k (its tags are
 * already those of the new rows, the lines still hold the victims' data). */
static int second_level(orc *h, orc_table *tb) {
  const int W = h->ways;
  const int32_t k = h->k;
  const size_t rb = (size_t)tb->dim * esize(tb->dtype);
  tb->l2_hits = tb->l2_demotions = tb->l2_evictions = tb->l2_bypasses = 0;
  /* the victims' data leave their first-level lines */
  int64_t nv = 0;
  orc_victim *vic = (orc_victim *)malloc(sizeof(orc_victim) * (size_t)(tb->n_ins + 1));
  char *vdata = (char *)malloc(rb * (size_t)(tb->n_ins + 1));
  float *vstate = (float *)malloc(sizeof(float) * (size_t)(tb->n_ins + 1));
  if (!vic || !vdata || !vstate) { free(vic); free(vdata); free(vstate); return ORC_ENOMEM; }
  for (int64_t i = 0; i < tb->n_ins; i++) {
    if (tb->ins_old[i] < 0) continue;
    vic[nv].row = tb->ins_old[i]; vic[nv].slot = nv;
    memcpy(vdata + (size_t)nv * rb, (char *)tb->lines + (size_t)tb->ins_slot[i] * rb, rb);
    vstate[nv] = tb->line_state[tb->ins_slot[i]];
    nv++;
  }
  /* (A) the rows the first level missed, ascending: inserted ones ... */
  for (int64_t i = 0; i < tb->n_ins; i++) {
    int64_t r = tb->ins_row[i], slot = tb->ins_slot[i];
    int64_t s2 = find_slot2(tb, W, r);
    if (s2 >= 0) { /* found: moves up, its second-level entry becomes free */
      memcpy((char *)tb->lines + (size_t)slot * rb, (char *)tb->lines2 + (size_t)s2 * rb, rb);
      tb->line_state[slot] = tb->line_state2[s2];
      tb->tag2[s2] = -1; tb->ts2[s2] = -1;
      tb->l2_hits++;
    } else {
      ensure_initialised(h, tb, r);
      backing_to_line(tb, slot, r);
    }
  }
  /* ... and bypassed ones: used in place */
  for (int64_t j = 0; j < tb->n_byp; j++) {
    int64_t s2 = find_slot2(tb, W, tb->byp_row[j]);
    if (s2 >= 0) { tb->ts2[s2] = k; tb->l2_hits++; }
    else ensure_initialised(h, tb, tb->byp_row[j]);
  }
  /* (B) the evicted rows move down in ascending row order */
  qsort(vic, (size_t)nv, sizeof(orc_victim), cmp_victim);
  for (int64_t v = 0; v < nv; v++) {
    int64_t r = vic[v].row, src = vic[v].slot;
    int64_t s = r % tb->sets2;
    int way = -1;
    for (int w = 0; w < W; w++) {
      int32_t tw = tb->ts2[s * W + w];
      if (tw < k - (h->lock2 - 1) && (way < 0 || tw < tb->ts2[s * W + way])) way = w;
    }
    if (way < 0) { /* every way was stamped by this batch or the one before: straight to the lower tier */
      memcpy((char *)tb->weights + (size_t)r * rb, vdata + (size_t)src * rb, rb);
      tb->state[r] = vstate[src];
      tb->l2_bypasses++;
      continue;
    }
    int64_t s2 = s * W + way;
    if (tb->tag2[s2] >= 0) { line2_to_backing(tb, s2, tb->tag2[s2]); tb->l2_evictions++; }
    memcpy((char *)tb->lines2 + (size_t)s2 * rb, vdata + (size_t)src * rb, rb);
    tb->line_state2[s2] = vstate[src];
    tb->tag2[s2] = r; tb->ts2[s2] = k;
    tb->l2_demotions++;
  }
  free(vic); free(vdata); free(vstate);
  return 0;
}

/* One table, one batch: distinct rows, then the two-phase replacement pass. */
static int prefetch_table(orc *h, int t) {
  orc_table *tb = &h->tab[t];
  const int W = h->ways;
  const int32_t k = h->k;
  int64_t lo = h->offsets[(int64_t)t * h->B], hi = h->offsets[(int64_t)(t + 1) * h->B];
  int64_t n = hi - lo;
  memset(&tb->st, 0, sizeof(tb->st));
  tb->n_uniq = tb->n_hit = tb->n_ins = tb->n_byp = 0;
  tb->l2_hits = tb->l2_demotions = tb->l2_evictions = tb->l2_bypasses = 0; /* per batch, also when the table has no lookups */
  tb->st.lookups = n;
  if (n == 0) return 0;
  if (grow(tb, n)) return ORC_ENOMEM;
  /* distinct rows in ascending order with their multiplicities */
  int64_t *tmp = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
  if (!tmp) return ORC_ENOMEM;
  memcpy(tmp, h->indices + lo, sizeof(int64_t) * (size_t)n);
  qsort(tmp, (size_t)n, sizeof(int64_t), cmp_i64);
  int64_t u = 0;
  for (int64_t i = 0; i < n; i++) {
    if (i == 0 || tmp[i] != tmp[i - 1]) { tb->uniq[u] = tmp[i]; tb->mult[u] = 1; u++; }
    else tb->mult[u - 1]++;
  }
  free(tmp);
  tb->n_uniq = u;
  tb->st.uniques = u;
  /* phase 1: hits get the time of access */
  char *is_hit = (char *)calloc((size_t)u, 1);
  if (!is_hit) return ORC_ENOMEM;
  for (int64_t i = 0; i < u; i++) {
    int64_t slot = find_slot(tb, W, tb->uniq[i]);
    if (slot >= 0) {
      tb->ts[slot] = k;
      tb->freq[slot] = add_saturating(tb->freq[slot], tb->mult[i]);
      is_hit[i] = 1;
      tb->hit_row[tb->n_hit++] = tb->uniq[i];
      tb->st.hits++;
      tb->st.hit_lookups += tb->mult[i];
    }
  }
  /* phase 2: misses in ascending row order pick a slot, evicting if it is occupied */
  for (int64_t i = 0; i < u; i++) {
    if (is_hit[i]) continue;
    int64_t r = tb->uniq[i];
    int victim = -1;
    int64_t s = 0;
    if (tb->sets > 0) {
      s = r % tb->sets;
      for (int w = 0; w < W; w++) {
        int32_t tw = tb->ts[s * W + w], fw = tb->freq[s * W + w];
        if (tw >= 1 && tw >= k - h->lock1) continue; /* used by this batch (or one of the lock1 before it): locked;
                                                         a free way (-1) never is */
        if (victim < 0) { victim = w; continue; }
        int32_t tv = tb->ts[s * W + victim], fv = tb->freq[s * W + victim];
        if (h->policy == ORC_LFU ? (fw < fv || (fw == fv && tw < tv)) : (tw < tv)) victim = w;
      }
    }
    if (victim < 0) {
      tb->byp_row[tb->n_byp++] = r;
      tb->st.bypasses++;
      if (tb->sets2 == 0) ensure_initialised(h, tb, r); /* read from the lower tier directly */
      continue;
    }
    int64_t slot = s * W + victim;
    int64_t old = tb->tag[slot];
    if (old >= 0) tb->st.evictions++;
    if (tb->sets2 == 0) { /* one level: the victim goes to the lower tier, the row comes from it */
      if (old >= 0) line_to_backing(tb, slot, old);
      ensure_initialised(h, tb, r);
      backing_to_line(tb, slot, r);
    }
    tb->tag[slot] = r;
    tb->ts[slot] = k;
    tb->freq[slot] = add_saturating(0, tb->mult[i]);
    tb->ins_row[tb->n_ins] = r; tb->ins_slot[tb->n_ins] = slot; tb->ins_old[tb->n_ins] = old;
    tb->n_ins++;
    tb->st.inserts++;
  }
  free(is_hit);
  if (tb->sets2 > 0) return second_level(h, tb);
  return 0;
}

static void add_stats(orc_stats *a, const orc_stats *b) {
  a->lookups += b->lookups; a->uniques += b->uniques; a->hits += b->hits; a->inserts += b->inserts;
  a->bypasses += b->bypasses; a->evictions += b->evictions; a->hit_lookups += b->hit_lookups;
}

int orc_prefetch(void *hp, const int64_t *indices, const int64_t *offsets, int32_t B, int64_t N) {
  orc *h = (orc *)hp;
  if (!h || !offsets || B < 0 || N < 0 || (N > 0 && !indices)) return ORC_EINVAL;
  int64_t nb = (int64_t)h->T * B;
  if (offsets[0] != 0 || offsets[nb] != N) return ORC_EINVAL;
  for (int64_t i = 0; i < nb; i++) if (offsets[i + 1] < offsets[i]) return ORC_EINVAL;
  for (int t = 0; t < h->T; t++)
    for (int64_t j = offsets[(int64_t)t * B]; j < offsets[(int64_t)(t + 1) * B]; j++)
      if (indices[j] < 0 || indices[j] >= h->tab[t].rows) return ORC_ERANGE;
  if (N > h->cap_idx) { free(h->indices); h->indices = (int64_t *)malloc(sizeof(int64_t) * (size_t)N); h->cap_idx = N; }
  if (nb + 1 > h->cap_off) { free(h->offsets); h->offsets = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb + 1)); h->cap_off = nb + 1; }
  if ((N > 0 && !h->indices) || !h->offsets) return ORC_ENOMEM;
  if (N > 0) memcpy(h->indices, indices, sizeof(int64_t) * (size_t)N);
  memcpy(h->offsets, offsets, sizeof(int64_t) * (size_t)(nb + 1));
  h->B = B; h->N = N;
  h->k += 1;
  int rc = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(h->threads)
  for (int t = 0; t < h->T; t++) {
    int r = prefetch_table(h, t);
    if (r) {
#pragma omp critical
      rc = r;
    }
  }
  if (rc) return rc;
  memset(&h->last, 0, sizeof(h->last));
  for (int t = 0; t < h->T; t++) add_stats(&h->last, &h->tab[t].st);
  add_stats(&h->total, &h->last);
  memset(h->l2_last, 0, sizeof(h->l2_last));
  for (int t = 0; t < h->T; t++) {
    orc_table *tb = &h->tab[t];
    if (tb->sets2 == 0) continue;
    h->l2_last[0] += tb->l2_hits; h->l2_last[1] += tb->l2_demotions;
    h->l2_last[2] += tb->l2_evictions; h->l2_last[3] += tb->l2_bypasses;
  }
  for (int i = 0; i < 4; i++) h->l2_total[i] += h->l2_last[i];
  h->prefetched = 1; h->forwarded = 0;
  return ORC_OK;
}

/* out[b, col_t + d] = sum over the lookups of bag (t, b) of the row, read where it lives */
int orc_forward(void *hp, float *out) {
  orc *h = (orc *)hp;
  if (!h || !out) return ORC_EINVAL;
  if (!h->prefetched) return ORC_EORDER;
  int64_t sumD = 0;
  for (int t = 0; t < h->T; t++) sumD += h->tab[t].dim;
  int failed = 0;
  if (h->pooling == ORC_POOL_MAX && (int64_t)h->B * sumD > h->cap_arg) {
    free(h->argmax);
    h->cap_arg = (int64_t)h->B * sumD;
    h->argmax = (int64_t *)malloc(sizeof(int64_t) * (size_t)h->cap_arg);
    if (!h->argmax) { h->cap_arg = 0; return ORC_ENOMEM; }
  }
#pragma omp parallel for schedule(dynamic, 1) num_threads(h->threads)
  for (int t = 0; t < h->T; t++) {
    orc_table *tb = &h->tab[t];
    int64_t col = 0;
    for (int q = 0; q < t; q++) col += h->tab[q].dim;
    double *acc = (double *)malloc(sizeof(double) * (size_t)tb->dim);
    if (!acc) { failed = 1; continue; }
    for (int32_t b = 0; b < h->B; b++) {
      for (int d = 0; d < tb->dim; d++) acc[d] = 0.0;
      int64_t first = h->offsets[(int64_t)t * h->B + b];
      for (int64_t j = first; j < h->offsets[(int64_t)t * h->B + b + 1]; j++) {
        void *src; int64_t at; float *st_unused;
        locate_row(tb, h->ways, h->indices[j], &src, &at, &st_unused);
        int64_t base = at * tb->dim;
        if (h->pooling == ORC_POOL_MAX) { /* the first lookup supplies the maximum until a larger value comes */
          for (int d = 0; d < tb->dim; d++) {
            double v = load_elem(src, tb->dtype, base + d);
            if (j == first || v > acc[d]) { acc[d] = v; h->argmax[(int64_t)b * sumD + col + d] = j; }
          }
          continue;
        }
        for (int d = 0; d < tb->dim; d++) acc[d] += load_elem(src, tb->dtype, base + d);
      }
      if (h->pooling == ORC_POOL_MAX && first == h->offsets[(int64_t)t * h->B + b + 1])
        for (int d = 0; d < tb->dim; d++) h->argmax[(int64_t)b * sumD + col + d] = -1;
      int64_t L = h->offsets[(int64_t)t * h->B + b + 1] - h->offsets[(int64_t)t * h->B + b];
      double div = (h->pooling == ORC_POOL_MEAN && L > 0) ? (double)L : 1.0;
      for (int d = 0; d < tb->dim; d++) out[(int64_t)b * sumD + col + d] = (float)(acc[d] / div);
    }
    free(acc);
  }
  if (failed) return ORC_ENOMEM;
  h->forwarded = 1;
  return ORC_OK;
}

static int64_t lower_bound(const int64_t *a, int64_t n, int64_t v) {
  int64_t lo = 0, hi = n;
  while (lo < hi) { int64_t mid = (lo + hi) / 2; if (a[mid] < v) lo = mid + 1; else hi = mid; }
  return lo;
}

/* g_r = sum over lookups of r of grad_out[bag] (mean pooling: / lookups of the bag); m_r += mean(g^2); w_r -= lr*g/(sqrt(m_r)+eps) */
int orc_backward_update(void *hp, const float *grad_out, float lr, float eps) {
  orc *h = (orc *)hp;
  if (!h || !grad_out) return ORC_EINVAL;
  if (!h->forwarded) return ORC_EORDER;
  int64_t sumD = 0;
  for (int t = 0; t < h->T; t++) sumD += h->tab[t].dim;
  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(h->threads)
  for (int t = 0; t < h->T; t++) {
    orc_table *tb = &h->tab[t];
    int64_t col = 0;
    for (int q = 0; q < t; q++) col += h->tab[q].dim;
    int64_t U = tb->n_uniq;
    if (U == 0) continue;
    double *g = (double *)calloc((size_t)U * (size_t)tb->dim, sizeof(double));
    if (!g) { failed = 1; continue; }
    for (int32_t b = 0; b < h->B; b++) {
      int64_t L = h->offsets[(int64_t)t * h->B + b + 1] - h->offsets[(int64_t)t * h->B + b];
      double div = h->pooling == ORC_POOL_MEAN ? (double)L : 1.0;
      for (int64_t j = h->offsets[(int64_t)t * h->B + b]; j < h->offsets[(int64_t)t * h->B + b + 1]; j++) {
        int64_t u = lower_bound(tb->uniq, U, h->indices[j]);
        for (int d = 0; d < tb->dim; d++) {
          if (h->pooling == ORC_POOL_MAX && h->argmax[(int64_t)b * sumD + col + d] != j) continue;
          g[u * tb->dim + d] += (double)grad_out[(int64_t)b * sumD + col + d] / div;
        }
      }
    }
    for (int64_t u = 0; u < U; u++) {
      void *wbase; int64_t at; float *mptr;
      locate_row(tb, h->ways, tb->uniq[u], &wbase, &at, &mptr);
      int64_t base = at * tb->dim;
      double sq = 0.0;
      for (int d = 0; d < tb->dim; d++) sq += g[u * tb->dim + d] * g[u * tb->dim + d];
      double m = (double)*mptr + sq / (double)tb->dim;
      double denom = sqrt(m) + (double)eps;
      double pk = (double)tb->peak[tb->uniq[u]];
      for (int d = 0; d < tb->dim; d++) {
        double w = load_elem(wbase, tb->dtype, base + d);
        store_elem(wbase, tb->dtype, base + d, w - (double)lr * g[u * tb->dim + d] / denom);
        double w1 = load_elem(wbase, tb->dtype, base + d);
        if (fabs(w) > pk) pk = fabs(w);
        if (fabs(w1) > pk) pk = fabs(w1);
      }
      tb->peak[tb->uniq[u]] = (float)pk;
      *mptr = (float)m;
    }
    free(g);
  }
  if (failed) return ORC_ENOMEM;
  h->forwarded = 0; h->prefetched = 0;
  return ORC_OK;
}

/* every valid line (row and accumulator) goes to the lower tier; tags stay */
int orc_flush(void *hp) {
  orc *h = (orc *)hp;
  if (!h) return ORC_EINVAL;
  for (int t = 0; t < h->T; t++) {
    orc_table *tb = &h->tab[t];
    for (int64_t s = 0; s < tb->sets * h->ways; s++)
      if (tb->tag[s] >= 0) line_to_backing(tb, s, tb->tag[s]);
    for (int64_t s = 0; s < tb->sets2 * h->ways; s++)
      if (tb->tag2[s] >= 0) line2_to_backing(tb, s, tb->tag2[s]);
  }
  return ORC_OK;
}

/* ---------------- observation ---------------- */

int64_t orc_num_sets(void *hp, int32_t t) { return ((orc *)hp)->tab[t].sets; }
int64_t orc_num_sets2(void *hp, int32_t t) { return ((orc *)hp)->tab[t].sets2; }

int orc_export_second_level(void *hp, int32_t t, int64_t *tags, int32_t *ts) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T) return ORC_EINVAL;
  orc_table *tb = &h->tab[t];
  int64_t n = tb->sets2 * h->ways;
  if (n) { memcpy(tags, tb->tag2, sizeof(int64_t) * (size_t)n); memcpy(ts, tb->ts2, sizeof(int32_t) * (size_t)n); }
  return ORC_OK;
}

/* second-level counters: hits, demotions, evictions, bypasses -- of the last batch and in total */
int orc_get_second_level_stats(void *hp, int64_t *last4, int64_t *total4) {
  orc *h = (orc *)hp;
  if (!h) return ORC_EINVAL;
  if (last4) memcpy(last4, h->l2_last, sizeof(h->l2_last));
  if (total4) memcpy(total4, h->l2_total, sizeof(h->l2_total));
  return ORC_OK;
}
int32_t orc_batch_id(void *hp) { return ((orc *)hp)->k; }

int orc_export_cache_state(void *hp, int32_t t, int64_t *tags, int32_t *ts) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T) return ORC_EINVAL;
  orc_table *tb = &h->tab[t];
  int64_t n = tb->sets * h->ways;
  if (n) { memcpy(tags, tb->tag, sizeof(int64_t) * (size_t)n); memcpy(ts, tb->ts, sizeof(int32_t) * (size_t)n); }
  return ORC_OK;
}

/* Test hook: overwrite the per-entry lookup counts of a table (same layout as the export).  Lets a
 * test start from counts near INT32_MAX without replaying two billion lookups. */
int orc_import_cache_freq(void *hp, int32_t t, const int32_t *freq) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T || !freq) return ORC_EINVAL;
  memcpy(h->tab[t].freq, freq, sizeof(int32_t) * (size_t)(h->tab[t].sets * h->ways));
  return ORC_OK;
}

/* lookup counts of the entries (0 for free ones), same order as the tags */
int orc_export_cache_freq(void *hp, int32_t t, int32_t *freq) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T || !freq) return ORC_EINVAL;
  orc_table *tb = &h->tab[t];
  int64_t n = tb->sets * h->ways;
  if (n) memcpy(freq, tb->freq, sizeof(int32_t) * (size_t)n);
  return ORC_OK;
}

int orc_get_stats(void *hp, orc_stats *last, orc_stats *total) {
  orc *h = (orc *)hp;
  if (!h) return ORC_EINVAL;
  if (last) *last = h->last;
  if (total) *total = h->total;
  return ORC_OK;
}

/* events of the last prefetch: kind 0 = hits, 1 = inserts, 2 = bypasses.  With null
 * arrays returns the count; otherwise fills table[], row[] and, for inserts, slot[]
 * (table-local, set*ways + way) and old[] (row evicted from it, -1 if it was free). */
int64_t orc_events(void *hp, int kind, int64_t *table, int64_t *row, int64_t *slot, int64_t *old) {
  orc *h = (orc *)hp;
  int64_t n = 0;
  for (int t = 0; t < h->T; t++) {
    orc_table *tb = &h->tab[t];
    int64_t c = kind == 0 ? tb->n_hit : kind == 1 ? tb->n_ins : tb->n_byp;
    const int64_t *src = kind == 0 ? tb->hit_row : kind == 1 ? tb->ins_row : tb->byp_row;
    if (table && row)
      for (int64_t i = 0; i < c; i++) {
        table[n + i] = t; row[n + i] = src[i];
        if (kind == 1 && slot && old) { slot[n + i] = tb->ins_slot[i]; old[n + i] = tb->ins_old[i]; }
      }
    n += c;
  }
  return n;
}

/* max pooling, after a forward: out[b, col_t + d] = position inside bag (t, b) of the lookup that
 * supplied pooled element d (the first of several equal ones), -1 for an empty bag */
int orc_export_argmax(void *hp, int32_t *out) {
  orc *h = (orc *)hp;
  if (!h || !out) return ORC_EINVAL;
  if (h->pooling != ORC_POOL_MAX || !h->forwarded) return ORC_EORDER;
  int64_t sumD = 0, col = 0;
  for (int t = 0; t < h->T; t++) sumD += h->tab[t].dim;
  for (int t = 0; t < h->T; t++) {
    for (int32_t b = 0; b < h->B; b++)
      for (int d = 0; d < h->tab[t].dim; d++) {
        int64_t j = h->argmax[(int64_t)b * sumD + col + d];
        out[(int64_t)b * sumD + col + d] = j < 0 ? -1 : (int32_t)(j - h->offsets[(int64_t)t * h->B + b]);
      }
    col += h->tab[t].dim;
  }
  return ORC_OK;
}

/* bookkeeping for the tests: per row, the largest |element| it has held before or after any of its updates */
int orc_export_row_peak(void *hp, int32_t t, float *out) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T || !out) return ORC_EINVAL;
  memcpy(out, h->tab[t].peak, sizeof(float) * (size_t)h->tab[t].rows);
  return ORC_OK;
}

/* current value of a row and its accumulator, wherever they live */
int orc_read_row(void *hp, int32_t t, int64_t r, double *w, float *m) {
  orc *h = (orc *)hp;
  if (!h || t < 0 || t >= h->T || r < 0 || r >= h->tab[t].rows) return ORC_EINVAL;
  orc_table *tb = &h->tab[t];
  void *src; int64_t at; float *st;
  locate_row(tb, h->ways, r, &src, &at, &st);
  for (int d = 0; d < tb->dim; d++) w[d] = load_elem(src, tb->dtype, at * tb->dim + d);
  *m = *st;
  return ORC_OK;
}
