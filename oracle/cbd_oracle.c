/*
 * cbd_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-channel CPU statement of what the decoder computes:
 * frame-synchronous Viterbi token passing with beam pruning over a static
 * transducer, where a channel's context is a set of arc indices and a discount
 * offset that is added to a listed arc's weight at the moment the arc is
 * expanded (paper Sec. 1, Sec. 4.1: "boosting weight = original weight +
 * discount factor"; Sec. 3.2: every outgoing arc of every queued token is
 * expanded, candidates are pruned by a beam and re-queued; Sec. 1/2.2: the
 * partial hypothesis is the current best token sequence, no lattice).
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP library.
 *
 * The paper names beam pruning and recombination but prints no formulas for
 * them.  The reading taken here (every choice independent of visiting order):
 *
 *   key      A token of state d is (cost, arc).  Keys order by fp32 cost, then
 *            by the arc: lower source state first, then emitting before
 *            epsilon, then lower arc index (for rows whose emitting arcs come
 *            first this is "lowest arc index wins").  The start token's arc is
 *            NONE, after every real arc.
 *   weight   w'(a) = w[a] + offset if a is in the channel's set, else w[a]
 *            (one fp32 add; Sec. 4.1).
 *   reset    E = {start: (0, NONE)}, m = 0, F = epsilon closure of E.
 *   frame    1. prune F_{t-1}: best = min cost; a token dies if
 *               cost - best > beam; if max_active > 0 and more than max_active
 *               survive: bin = min(255, floor((cost-best) * (256/beam))),
 *               B = largest bin whose cumulative count <= max_active (0 if
 *               bin 0 alone exceeds it); a token survives iff bin <= B.
 *            2. emit: for each survivor (s, c) and arc a of s with ilabel != 0:
 *               cand = (c + w'(a)) - L[ilabel-1]; E[dst] = min key.
 *            3. m = min cost in E; drop entries with cost - m > beam.
 *            4. closure: least fixed point of relaxing cand = c + w'(a) over
 *               epsilon arcs, ignoring cand with cand - m > beam.
 *            5. the predecessor of a token reached by arc a is the final token
 *               of a's source state: in F_t if a is epsilon, else in F_{t-1}.
 *   best     argmin key over F_t (cost + final cost if asked).
 *
 * All arithmetic is IEEE fp32, in exactly the order written.  Compile with
 * -ffp-contract=off and without fast-math.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_NO_TOKENS 1
#define ORC_EPS_DIVERGED 2
#define ORC_BUFFER 3
#define ORC_INVALID 4

#define ARC_NONE (-1)

typedef struct orc_graph {
  int32_t S, A, P, start;
  const int32_t *row, *dst, *ilabel, *olabel; /* borrowed from the caller */
  const float *weight;
  const float *final_cost; /* may be NULL */
  int32_t *src;            /* owned: source state of each arc */
} orc_graph;

typedef struct orc_chan {
  const orc_graph *g;
  float beam;
  int32_t max_active;
  int32_t max_eps_iters;
  /* context: the set, kept three ways so the lookups can be compared */
  uint8_t *member;     /* [A] 1 if listed */
  int32_t *ctx_raw;    /* list as given */
  int32_t n_raw;
  int32_t *ctx_sorted; /* sorted, duplicates removed */
  int32_t n_sorted;
  float offset;
  int32_t lookup_mode; /* 0 membership array, 1 linear scan, 2 binary search */
  /* current table F_t as a list plus a dense state -> list position map */
  int32_t n, cap;
  int32_t *st, *ar;
  float *co;
  int32_t *where;      /* [S], -1 = absent */
  int32_t *prev_where; /* [S] positions in F_{t-1} */
  int32_t *prev_st;
  int32_t prev_n, prev_cap;
  int32_t frame_base, prev_frame_base; /* first record of F_t / F_{t-1} */
  /* back-pointer records */
  int32_t *rec_arc, *rec_prev;
  int64_t n_rec, rec_cap;
  /* bookkeeping */
  int32_t status;
  int32_t frames_done;
  float last_m, last_best;
  int64_t emit_arcs;   /* emitting arcs of surviving tokens, all frames */
  int64_t tokens_sum;  /* sum over frames of |F_t| */
  int64_t active_sum;  /* sum over frames of survivors of step 1 */
  int32_t tokens_max;
  uint8_t *alive;
  int32_t alive_cap;
} orc_chan;

/* ------------------------------------------------------------------ graph */

orc_graph *orc_graph_new(int32_t S, int32_t A, int32_t P, int32_t start, const int32_t *row,
                         const int32_t *dst, const int32_t *ilabel, const int32_t *olabel,
                         const float *weight, const float *final_cost) {
  if (S <= 0 || A < 0 || start < 0 || start >= S || row[0] != 0 || row[S] != A) return NULL;
  orc_graph *g = (orc_graph *)calloc(1, sizeof(orc_graph));
  g->S = S; g->A = A; g->P = P; g->start = start;
  g->row = row; g->dst = dst; g->ilabel = ilabel; g->olabel = olabel;
  g->weight = weight; g->final_cost = final_cost;
  g->src = (int32_t *)malloc(sizeof(int32_t) * (size_t)(A > 0 ? A : 1));
  for (int32_t s = 0; s < S; s++)
    for (int32_t a = row[s]; a < row[s + 1]; a++) g->src[a] = s;
  return g;
}

void orc_graph_free(orc_graph *g) {
  if (!g) return;
  free(g->src);
  free(g);
}

/* ---------------------------------------------------------------- ordering */

/* Does arc a1 come before arc a2 in the tie-break order? */
static int arc_before(const orc_graph *g, int32_t a1, int32_t a2) {
  if (a1 == a2) return 0;
  if (a1 == ARC_NONE) return 0;
  if (a2 == ARC_NONE) return 1;
  int32_t s1 = g->src[a1], s2 = g->src[a2];
  if (s1 != s2) return s1 < s2;
  int e1 = g->ilabel[a1] == 0, e2 = g->ilabel[a2] == 0;
  if (e1 != e2) return e1 < e2;
  return a1 < a2;
}

static int key_less(const orc_graph *g, float c1, int32_t a1, float c2, int32_t a2) {
  if (c1 < c2) return 1;
  if (c1 > c2) return 0;
  return arc_before(g, a1, a2);
}

/* ----------------------------------------------------------------- context */

static int cmp_i32(const void *x, const void *y) {
  int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
  return (a > b) - (a < b);
}

static int in_context(const orc_chan *ch, int32_t a) {
  if (ch->lookup_mode == 1) {
    for (int32_t i = 0; i < ch->n_raw; i++)
      if (ch->ctx_raw[i] == a) return 1;
    return 0;
  }
  if (ch->lookup_mode == 2) {
    int32_t lo = 0, hi = ch->n_sorted;
    while (lo < hi) {
      int32_t mid = lo + (hi - lo) / 2;
      if (ch->ctx_sorted[mid] < a) lo = mid + 1; else hi = mid;
    }
    return lo < ch->n_sorted && ch->ctx_sorted[lo] == a;
  }
  return ch->member[a];
}

/* Sec. 4.1: the boosted weight is the arc's weight plus the discount. */
static float biased_weight(const orc_chan *ch, int32_t a) {
  float w = ch->g->weight[a];
  if (ch->n_raw > 0 && in_context(ch, a)) w = w + ch->offset;
  return w;
}

int32_t orc_set_context(orc_chan *ch, const int32_t *arcs, int32_t n, float offset) {
  for (int32_t i = 0; i < n; i++)
    if (arcs[i] < 0 || arcs[i] >= ch->g->A) return ORC_INVALID;
  for (int32_t i = 0; i < ch->n_raw; i++) ch->member[ch->ctx_raw[i]] = 0;
  free(ch->ctx_raw); free(ch->ctx_sorted);
  ch->ctx_raw = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  ch->ctx_sorted = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  if (n > 0) memcpy(ch->ctx_raw, arcs, sizeof(int32_t) * (size_t)n);
  if (n > 0) memcpy(ch->ctx_sorted, arcs, sizeof(int32_t) * (size_t)n);
  ch->n_raw = n;
  qsort(ch->ctx_sorted, (size_t)n, sizeof(int32_t), cmp_i32);
  int32_t k = 0;
  for (int32_t i = 0; i < n; i++)
    if (i == 0 || ch->ctx_sorted[i] != ch->ctx_sorted[i - 1]) ch->ctx_sorted[k++] = ch->ctx_sorted[i];
  ch->n_sorted = k;
  for (int32_t i = 0; i < n; i++) ch->member[arcs[i]] = 1;
  ch->offset = offset;
  return ORC_OK;
}

void orc_set_lookup_mode(orc_chan *ch, int32_t mode) { ch->lookup_mode = mode; }

/* ----------------------------------------------------------------- channel */

orc_chan *orc_chan_new(const orc_graph *g, float beam, int32_t max_active, int32_t max_eps_iters) {
  orc_chan *ch = (orc_chan *)calloc(1, sizeof(orc_chan));
  ch->g = g; ch->beam = beam; ch->max_active = max_active;
  ch->max_eps_iters = max_eps_iters > 0 ? max_eps_iters : 64;
  ch->member = (uint8_t *)calloc((size_t)(g->A > 0 ? g->A : 1), 1);
  ch->where = (int32_t *)malloc(sizeof(int32_t) * (size_t)g->S);
  ch->prev_where = (int32_t *)malloc(sizeof(int32_t) * (size_t)g->S);
  for (int32_t s = 0; s < g->S; s++) { ch->where[s] = -1; ch->prev_where[s] = -1; }
  ch->status = ORC_NO_TOKENS; /* until reset */
  return ch;
}

void orc_chan_free(orc_chan *ch) {
  if (!ch) return;
  free(ch->member); free(ch->ctx_raw); free(ch->ctx_sorted);
  free(ch->st); free(ch->ar); free(ch->co); free(ch->where); free(ch->prev_where);
  free(ch->prev_st); free(ch->rec_arc); free(ch->rec_prev); free(ch->alive);
  free(ch);
}

static void table_reserve(orc_chan *ch, int32_t need) {
  if (need <= ch->cap) return;
  int32_t cap = ch->cap ? ch->cap : 1024;
  while (cap < need) cap *= 2;
  ch->st = (int32_t *)realloc(ch->st, sizeof(int32_t) * (size_t)cap);
  ch->ar = (int32_t *)realloc(ch->ar, sizeof(int32_t) * (size_t)cap);
  ch->co = (float *)realloc(ch->co, sizeof(float) * (size_t)cap);
  ch->cap = cap;
}

/* E[d] = min key.  Returns 1 if the table changed. */
static int relax(orc_chan *ch, int32_t d, float cand, int32_t a) {
  int32_t p = ch->where[d];
  if (p < 0) {
    table_reserve(ch, ch->n + 1);
    p = ch->n++;
    ch->where[d] = p;
    ch->st[p] = d; ch->co[p] = cand; ch->ar[p] = a;
    return 1;
  }
  if (key_less(ch->g, cand, a, ch->co[p], ch->ar[p])) {
    ch->co[p] = cand; ch->ar[p] = a;
    return 1;
  }
  return 0;
}

/* Step 4: relax epsilon arcs until nothing changes (Gauss-Seidel sweeps; the
 * fixed point does not depend on the order because fp32 addition is monotone). */
static void eps_closure(orc_chan *ch, float m) {
  const orc_graph *g = ch->g;
  int changed = 1, rounds = 0;
  while (changed && rounds < ch->max_eps_iters) {
    changed = 0;
    for (int32_t i = 0; i < ch->n; i++) { /* ch->n may grow during the sweep */
      int32_t s = ch->st[i];
      for (int32_t a = g->row[s]; a < g->row[s + 1]; a++) {
        if (g->ilabel[a] != 0) continue;
        float cand = ch->co[i] + biased_weight(ch, a);
        if (cand - m > ch->beam) continue;
        if (relax(ch, g->dst[a], cand, a)) changed = 1;
      }
    }
    rounds++;
  }
  if (changed) ch->status = ORC_EPS_DIVERGED;
}

/* Step 5: one record (arc, predecessor record) per token of F_t, in list order. */
static void write_records(orc_chan *ch) {
  const orc_graph *g = ch->g;
  int64_t need = ch->n_rec + ch->n;
  if (need > ch->rec_cap) {
    int64_t cap = ch->rec_cap ? ch->rec_cap : 4096;
    while (cap < need) cap *= 2;
    ch->rec_arc = (int32_t *)realloc(ch->rec_arc, sizeof(int32_t) * (size_t)cap);
    ch->rec_prev = (int32_t *)realloc(ch->rec_prev, sizeof(int32_t) * (size_t)cap);
    ch->rec_cap = cap;
  }
  int32_t base = (int32_t)ch->n_rec;
  for (int32_t i = 0; i < ch->n; i++) {
    int32_t a = ch->ar[i], prev = -1;
    if (a != ARC_NONE) {
      int32_t s = g->src[a];
      if (g->ilabel[a] == 0) prev = base + ch->where[s];
      else prev = ch->prev_frame_base + ch->prev_where[s];
    }
    ch->rec_arc[base + i] = a;
    ch->rec_prev[base + i] = prev;
  }
  ch->frame_base = base;
  ch->n_rec = need;
}

/* Make F_t the "previous" table. */
static void roll(orc_chan *ch) {
  for (int32_t i = 0; i < ch->prev_n; i++) ch->prev_where[ch->prev_st[i]] = -1;
  if (ch->n > ch->prev_cap) {
    ch->prev_cap = ch->cap;
    ch->prev_st = (int32_t *)realloc(ch->prev_st, sizeof(int32_t) * (size_t)ch->prev_cap);
  }
  for (int32_t i = 0; i < ch->n; i++) {
    ch->prev_st[i] = ch->st[i];
    ch->prev_where[ch->st[i]] = i;
    ch->where[ch->st[i]] = -1;
  }
  ch->prev_n = ch->n;
  ch->prev_frame_base = ch->frame_base;
}

int32_t orc_reset(orc_chan *ch) {
  for (int32_t i = 0; i < ch->prev_n; i++) ch->prev_where[ch->prev_st[i]] = -1;
  for (int32_t i = 0; i < ch->n; i++) ch->where[ch->st[i]] = -1;
  ch->prev_n = 0; ch->n = 0; ch->n_rec = 0;
  ch->frame_base = 0; ch->prev_frame_base = 0;
  ch->status = ORC_OK; ch->frames_done = 0;
  ch->emit_arcs = 0; ch->tokens_sum = 0; ch->active_sum = 0; ch->tokens_max = 0;
  relax(ch, ch->g->start, 0.0f, ARC_NONE);
  ch->last_m = 0.0f;
  eps_closure(ch, 0.0f);
  write_records(ch);
  float best = ch->co[0];
  for (int32_t i = 1; i < ch->n; i++) if (ch->co[i] < best) best = ch->co[i];
  ch->last_best = best;
  return ch->status;
}

/* Step 1 on a bare list of costs (exported so tests can pin it by hand).
 * alive[i] = 1 if token i survives.  Returns the number of survivors. */
int32_t orc_prune(const float *cost, int32_t n, float beam, int32_t max_active, uint8_t *alive,
                  float *best_out, int32_t *cut_bin_out) {
  if (cut_bin_out) *cut_bin_out = -1;
  if (n <= 0) return 0;
  float best = cost[0];
  for (int32_t i = 1; i < n; i++) if (cost[i] < best) best = cost[i];
  if (best_out) *best_out = best;
  int32_t survivors = 0;
  for (int32_t i = 0; i < n; i++) {
    alive[i] = !(cost[i] - best > beam);
    survivors += alive[i];
  }
  if (max_active > 0 && survivors > max_active && beam > 0.0f && beam < INFINITY) {
    int32_t hist[256];
    memset(hist, 0, sizeof(hist));
    float inv = 256.0f / beam;
    for (int32_t i = 0; i < n; i++) {
      if (!alive[i]) continue;
      int32_t bin = (int32_t)floorf((cost[i] - best) * inv);
      if (bin > 255) bin = 255;
      hist[bin]++;
    }
    int32_t B = 0, cum = 0;
    for (int32_t b = 0; b < 256; b++) {
      cum += hist[b];
      if (cum <= max_active) B = b; else break;
    }
    if (cut_bin_out) *cut_bin_out = B;
    survivors = 0;
    for (int32_t i = 0; i < n; i++) {
      if (!alive[i]) continue;
      int32_t bin = (int32_t)floorf((cost[i] - best) * inv);
      if (bin > 255) bin = 255;
      alive[i] = bin <= B;
      survivors += alive[i];
    }
  }
  return survivors;
}

/* One frame.  L = this frame's log-likelihood row, P floats. */
static void frame(orc_chan *ch, const float *L) {
  const orc_graph *g = ch->g;
  /* the table of the previous frame becomes read-only input */
  int32_t pn = ch->n;
  if (pn > ch->alive_cap) {
    ch->alive_cap = ch->cap;
    ch->alive = (uint8_t *)realloc(ch->alive, (size_t)ch->alive_cap);
  }
  float *pco = (float *)malloc(sizeof(float) * (size_t)(pn > 0 ? pn : 1));
  int32_t *pst = (int32_t *)malloc(sizeof(int32_t) * (size_t)(pn > 0 ? pn : 1));
  memcpy(pco, ch->co, sizeof(float) * (size_t)pn);
  memcpy(pst, ch->st, sizeof(int32_t) * (size_t)pn);
  roll(ch);
  ch->n = 0;
  /* 1. prune */
  int32_t act = orc_prune(pco, pn, ch->beam, ch->max_active, ch->alive, NULL, NULL);
  ch->active_sum += act;
  /* 2. emit */
  for (int32_t i = 0; i < pn; i++) {
    if (!ch->alive[i]) continue;
    int32_t s = pst[i];
    float c = pco[i];
    for (int32_t a = g->row[s]; a < g->row[s + 1]; a++) {
      int32_t il = g->ilabel[a];
      if (il == 0) continue;
      ch->emit_arcs++;
      float cand = (c + biased_weight(ch, a)) - L[il - 1];
      relax(ch, g->dst[a], cand, a);
    }
  }
  free(pco); free(pst);
  if (ch->n == 0) {
    ch->status = ORC_NO_TOKENS;
    ch->frame_base = (int32_t)ch->n_rec;
    ch->frames_done++;
    return;
  }
  /* 3. emission beam */
  float m = ch->co[0];
  for (int32_t i = 1; i < ch->n; i++) if (ch->co[i] < m) m = ch->co[i];
  int32_t k = 0;
  for (int32_t i = 0; i < ch->n; i++) {
    if (ch->co[i] - m > ch->beam) { ch->where[ch->st[i]] = -1; continue; }
    ch->st[k] = ch->st[i]; ch->co[k] = ch->co[i]; ch->ar[k] = ch->ar[i];
    ch->where[ch->st[k]] = k;
    k++;
  }
  ch->n = k;
  ch->last_m = m;
  /* 4. closure, 5. records */
  eps_closure(ch, m);
  write_records(ch);
  float best = ch->co[0];
  for (int32_t i = 1; i < ch->n; i++) if (ch->co[i] < best) best = ch->co[i];
  ch->last_best = best;
  ch->tokens_sum += ch->n;
  if (ch->n > ch->tokens_max) ch->tokens_max = ch->n;
  ch->frames_done++;
}

/* loglikes: n_frames rows of P floats, consecutive rows `stride` floats apart. */
int32_t orc_advance(orc_chan *ch, const float *loglikes, int32_t n_frames, int64_t stride) {
  for (int32_t f = 0; f < n_frames; f++) {
    if (ch->status != ORC_OK) break;
    frame(ch, loglikes + (int64_t)f * stride);
  }
  return ch->status;
}

/* Best token of the current table and its back-pointer path.
 * words/arcs: caller's buffers of `cap` entries (arcs may be NULL). */
int32_t orc_best_path(const orc_chan *ch, int32_t use_final, int32_t *words, int32_t *arcs, int32_t cap,
                      int32_t *n_words, int32_t *n_arcs, float *cost) {
  const orc_graph *g = ch->g;
  *n_words = 0; *n_arcs = 0; *cost = INFINITY;
  if (ch->status == ORC_EPS_DIVERGED) return ORC_EPS_DIVERGED;
  int32_t bi = -1; float bc = 0.0f;
  for (int32_t i = 0; i < ch->n; i++) {
    float c = ch->co[i];
    if (use_final && g->final_cost) c = c + g->final_cost[ch->st[i]];
    if (!(c < INFINITY)) continue;
    if (bi < 0 || key_less(g, c, ch->ar[i], bc, ch->ar[bi])) { bi = i; bc = c; }
  }
  if (bi < 0) return ORC_NO_TOKENS;
  *cost = bc;
  int32_t na = 0, nw = 0;
  for (int32_t r = ch->frame_base + bi; r >= 0; r = ch->rec_prev[r]) {
    int32_t a = ch->rec_arc[r];
    if (a == ARC_NONE) break;
    na++;
    if (g->olabel[a] != 0) nw++;
    /* zero-weight epsilon cycles can tie into a predecessor cycle: no path is that long */
    if (na > ch->n_rec) { *cost = INFINITY; return ORC_EPS_DIVERGED; }
  }
  *n_arcs = na; *n_words = nw;
  if (na > cap) return ORC_BUFFER;
  int32_t ia = na, iw = nw;
  for (int32_t r = ch->frame_base + bi; r >= 0; r = ch->rec_prev[r]) {
    int32_t a = ch->rec_arc[r];
    if (a == ARC_NONE) break;
    if (arcs) arcs[--ia] = a; else --ia;
    if (g->olabel[a] != 0) words[--iw] = g->olabel[a];
  }
  return ORC_OK;
}

/* Current table F_t (any order).  Returns its size; fills up to cap entries. */
int32_t orc_get_tokens(const orc_chan *ch, int32_t *states, float *costs, int32_t *arcs, int32_t cap) {
  int32_t k = ch->n < cap ? ch->n : cap;
  for (int32_t i = 0; i < k; i++) { states[i] = ch->st[i]; costs[i] = ch->co[i]; arcs[i] = ch->ar[i]; }
  return ch->n;
}

/* which: 0 emitting arcs expanded, 1 sum |F_t|, 2 sum survivors of step 1,
 * 3 max |F_t|, 4 frames done, 5 records written */
int64_t orc_stat(const orc_chan *ch, int32_t which) {
  switch (which) {
    case 0: return ch->emit_arcs;
    case 1: return ch->tokens_sum;
    case 2: return ch->active_sum;
    case 3: return ch->tokens_max;
    case 4: return ch->frames_done;
    case 5: return ch->n_rec;
    default: return -1;
  }
}

float orc_last_m(const orc_chan *ch) { return ch->last_m; }
float orc_last_best(const orc_chan *ch) { return ch->last_best; }
int32_t orc_status(const orc_chan *ch) { return ch->status; }
