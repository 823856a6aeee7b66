/*
 * CPU oracle for frame-synchronous WFST token-passing beam search over a CTC decoding graph.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded, scalar fp32
 * implementation used only to check the GPU decoder and to serve as a timed CPU baseline.
 * It shares no code with the GPU path and must never be called from the product path.
 *
 * What it follows (paper: "GPU-Accelerated WFST Beam Search Decoder for CTC-based Speech
 * Recognition"):
 *   - Section "Algorithm description": one iteration per acoustic frame with the stages
 *     ExpandArcs -> Prune -> store tokens and backpointers; the least-cost path is built
 *     from the stored backpointers afterwards.
 *   - Figure "Pseudo-code of Expand Arcs": new_cost = token cost + acoustic_cost[ilabel]
 *     + arc graph cost, for every token of the main queue and every out-arc.
 *   - Section "Offline inference": beam = largest allowed score gap from the best
 *     hypothesis; max-active = largest number of hypotheses, counted in graph states
 *     (states entered over epsilon arcs included).
 * The paper defers all remaining detail to earlier work.  The readings taken here:
 *   R1  ilabel 0 = epsilon; ilabel k>=1 reads log-likelihood column k-1; olabel 0 = none.
 *   R2  cost update is ((c + w) + (-loglike)) in fp32, in exactly that association.
 *   R3  recombination keeps, per destination state, the lexicographic minimum of
 *       (cost, global arc id); emitting arcs are numbered 0..Ae-1 in (source state,
 *       given order), epsilon arcs Ae..Ae+Ax-1 likewise.
 *   R4  a token is in the beam iff (c - best) <= beam, computed in fp32.
 *   R5  max-active uses a fixed 256-bin histogram over [best, best+beam]:
 *       bin(c) = clamp(floor((c-best) * (256/beam)), 0, 255); if more than max_active
 *       tokens are in the beam, only bins below k_keep survive, k_keep being the first bin
 *       at which the running count exceeds max_active, but never less than 1.
 *   R6  pruning is applied to the recombined emitting result; the epsilon closure then runs
 *       under the same, frozen, (best, k_keep) predicate and updates tokens in place.
 *   R7  candidates whose cost is not finite are discarded when created.
 *   R8  final choice: min over (cost + final_cost, state) if any token is final, else min
 *       over (cost, state) with the reached_final flag clear.
 *   R9  word boosting (Section "Word boosting" and the green lines of the Expand Arcs
 *       pseudo-code): on every arc, emitting or epsilon, whose olabel is in the utterance's
 *       boost table, the table's score is added after the other terms:
 *       ((c + w) + (-loglike)) + b[olabel], resp. (c + w) + b[olabel].
 *   R10 lattice output.  The paper only says that the stored tokens and backpointers let the
 *       host build "a lattice or least cost path" (Section "Algorithm description") and gives
 *       no definition, so this one is this build's own: the nodes are the tokens of all
 *       closed sets A_0..A_T; there is a link for every graph arc between two stored tokens
 *       (an emitting arc from a token of A_{t-1} to a token of A_t, read against row t-1; an
 *       epsilon arc between two tokens of the same A_t) whose cost through the arc,
 *       computed from the source token's stored cost exactly as in R2/R9, is finite and
 *       satisfies (cost - stored cost of the destination token) <= lattice_beam in fp32.
 *       The backpointer arcs are the links with difference 0.  Pinned by the tests only
 *       through what the definition implies (complete path set on unpruned micro graphs,
 *       best path = the decoder's); against the paper it is "parity unpinned".
 *   R11 cost offsets (an option; the paper is silent on cost renormalisation).  After the prune
 *       step of a frame, with b the best cost of the recombined set, every surviving token's
 *       cost c becomes (c - b) in fp32 and the closure's frozen predicate uses best = 0; the
 *       b's are summed in fp64 and the sum is added back to the cost that is reported:
 *       cost = (float)((double)c_final + sum).  Stored token costs (digests, dumps) are the
 *       rebased ones.  Costs then stay of the order of the beam however long the stream is.
 *       Pins: identical results on exactly representable (dyadic) inputs, and a smaller error
 *       against an fp64 trellis on a long stream.  In the lattice (R10) the cost of an emitting
 *       link into A_t is rebased like the tokens of A_t: (cost through the arc) - b_t.
 *
 *   R12 boosting acceptor with several states (Section "Word boosting": the graph is composed on
 *       the fly with a boosting acceptor B, TLG o B; the paper's B has one state, its figure
 *       "Example word boosting WFSA" shows the failure arc taken when no word arc matches, and
 *       its conclusions name phrase boosting as the extension).  B is a deterministic acceptor over
 *       OUTPUT labels: arcs (from, label, to, score), state 0 = root.  A token is a pair (graph
 *       state, B state); there is at most one token per pair and frame, so recombination,
 *       the epsilon closure and the stored sets are keyed by the pair.  On an arc with output label
 *       o != 0 taken by a token in B state b: if b has an arc on o, the token moves to its
 *       destination and the arc's score is added after the other terms (as in R9); otherwise the
 *       failure arc leads to the root at no cost and o is tried once more there (root arc on o:
 *       its destination and score; none: the token stays in the root, nothing is added).  Arcs
 *       without output label leave b unchanged.  A B with the single state 0 and self-loops is
 *       exactly the table of R9.  Final choice ties: lower graph state, then lower B state.
 *       Recombination ties (R3): two tokens of one graph state can take the SAME arc into the same
 *       pair (both fall back to the root, say); after (cost, arc id) the lower B state of the
 *       source token wins, which makes the order total again (an arc of the product is a graph
 *       arc plus the B state it is taken in).
 *       Digest of a token: the pair's B state enters the mix (0 leaves the R1-R11 digest unchanged).
 *
 * parity pins: see tests/test_oracle_*.py (exhaustive path enumeration, fp64 trellis
 * Viterbi, greedy CTC collapse on the normal CTC topology, closed-form histogram cases,
 * Dijkstra for the epsilon closure, traceback cost re-summation).  Absolute outputs are
 * "parity unpinned" against the paper itself: it prints no decoder output to compare to.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t num_states, start_state, num_classes;
  int64_t num_arcs;
  const int64_t *row_offsets;
  const int32_t *next_state, *ilabel, *olabel;
  const float *weight;
  const float *final_cost; /* NULL: every state final with cost 0 */
} oracle_graph;

typedef struct {
  int32_t S, start, V;
  int64_t Ae, Ax;
  int64_t *e_off, *x_off;                 /* [S+1] */
  int32_t *e_next, *e_il, *e_ol;          /* [Ae] */
  float *e_w;
  int32_t *x_next, *x_ol;                 /* [Ax] */
  float *x_w;
  int64_t *e_orig, *x_orig;               /* index of the arc in the caller's arrays */
  float *final_cost;                      /* [S] */
} oracle_prepared;

typedef struct {
  float beam;
  int32_t max_active;
  int32_t max_words;
  int32_t finalize;        /* 1: use final costs (R8); 0: best token regardless */
  int32_t worklist_order;  /* 0 FIFO, 1 LIFO, 2 seeded random pick */
  uint64_t order_seed;
  /* word boosting (Section "Word boosting"): table word id -> score of the single-state
   * boosting acceptor B; decoding behaves as if the graph were TLG o B */
  int32_t boost_n;
  const int32_t *boost_ids;
  const float *boost_scores;
  int32_t cost_offset;     /* R11: 1 = rebase the token costs to the best cost after every prune step */
  /* R12: boosting acceptor with bfst_states > 0 states (then the table above must be empty) */
  int32_t bfst_states, bfst_arcs;
  const int32_t *bfst_from, *bfst_label, *bfst_to;
  const float *bfst_score;
} oracle_opts;

typedef struct {
  int32_t nwords;
  float cost;
  int32_t flags;           /* bit0 reached_final, bit1 words truncated, bit2 dead */
  int32_t path_len;        /* number of arcs on the best path */
  int64_t counters[8];     /* see README of counters below */
} oracle_result;
/* counters: 0 sum |A_t| over expanded frames, 1 emitting arcs out of those sets,
 * 2 epsilon arcs out of every closed set (initial one included), 3 tokens that survive the
 * prune step (before the epsilon closure), 4 tokens stored (all closed sets), 5 frames where max-active pruned,
 * 6 frames where bin 0 alone exceeded max_active, 7 recombined destinations before pruning */

enum { FLAG_FINAL = 1, FLAG_TRUNC = 2, FLAG_DEAD = 4 };

/* ------------------------------------------------------------------ graph preparation */
void oracle_free(oracle_prepared *p) {
  if (!p) return;
  free(p->e_off); free(p->x_off); free(p->e_next); free(p->e_il); free(p->e_ol); free(p->e_w);
  free(p->x_next); free(p->x_ol); free(p->x_w); free(p->e_orig); free(p->x_orig);
  free(p->final_cost); free(p);
}

/* Returns NULL for a malformed graph (bad offsets, labels, destinations, non-finite weight,
 * or a cycle of epsilon arcs). */
oracle_prepared *oracle_prepare(const oracle_graph *g) {
  int32_t S = g->num_states;
  if (S <= 0 || g->start_state < 0 || g->start_state >= S || g->num_classes <= 0) return NULL;
  if (g->row_offsets[0] != 0 || g->row_offsets[S] != g->num_arcs) return NULL;
  for (int32_t s = 0; s < S; ++s)
    if (g->row_offsets[s + 1] < g->row_offsets[s]) return NULL;
  int64_t Ae = 0, Ax = 0;
  for (int64_t a = 0; a < g->num_arcs; ++a) {
    if (g->next_state[a] < 0 || g->next_state[a] >= S) return NULL;
    if (g->ilabel[a] < 0 || g->ilabel[a] > g->num_classes) return NULL;
    if (!isfinite(g->weight[a])) return NULL;
    if (g->ilabel[a] == 0) ++Ax; else ++Ae;
  }
  oracle_prepared *p = (oracle_prepared *)calloc(1, sizeof(*p));
  p->S = S; p->start = g->start_state; p->V = g->num_classes; p->Ae = Ae; p->Ax = Ax;
  p->e_off = (int64_t *)malloc(sizeof(int64_t) * (S + 1));
  p->x_off = (int64_t *)malloc(sizeof(int64_t) * (S + 1));
  p->e_next = (int32_t *)malloc(sizeof(int32_t) * (Ae + 1));
  p->e_il = (int32_t *)malloc(sizeof(int32_t) * (Ae + 1));
  p->e_ol = (int32_t *)malloc(sizeof(int32_t) * (Ae + 1));
  p->e_w = (float *)malloc(sizeof(float) * (Ae + 1));
  p->e_orig = (int64_t *)malloc(sizeof(int64_t) * (Ae + 1));
  p->x_next = (int32_t *)malloc(sizeof(int32_t) * (Ax + 1));
  p->x_ol = (int32_t *)malloc(sizeof(int32_t) * (Ax + 1));
  p->x_w = (float *)malloc(sizeof(float) * (Ax + 1));
  p->x_orig = (int64_t *)malloc(sizeof(int64_t) * (Ax + 1));
  p->final_cost = (float *)malloc(sizeof(float) * S);
  int64_t ne = 0, nx = 0;
  for (int32_t s = 0; s < S; ++s) {
    p->e_off[s] = ne; p->x_off[s] = nx;
    for (int64_t a = g->row_offsets[s]; a < g->row_offsets[s + 1]; ++a) {
      if (g->ilabel[a] == 0) {
        p->x_next[nx] = g->next_state[a]; p->x_ol[nx] = g->olabel[a];
        p->x_w[nx] = g->weight[a]; p->x_orig[nx] = a; ++nx;
      } else {
        p->e_next[ne] = g->next_state[a]; p->e_il[ne] = g->ilabel[a];
        p->e_ol[ne] = g->olabel[a]; p->e_w[ne] = g->weight[a]; p->e_orig[ne] = a; ++ne;
      }
    }
    p->final_cost[s] = g->final_cost ? g->final_cost[s] : 0.0f;
    if (isnan(p->final_cost[s])) { oracle_free(p); return NULL; }
  }
  p->e_off[S] = ne; p->x_off[S] = nx;
  /* epsilon sub-graph must be acyclic: Kahn's algorithm on in-degrees */
  int32_t *indeg = (int32_t *)calloc(S, sizeof(int32_t));
  int32_t *stack = (int32_t *)malloc(sizeof(int32_t) * S);
  for (int64_t a = 0; a < nx; ++a) indeg[p->x_next[a]]++;
  int32_t top = 0, seen = 0;
  for (int32_t s = 0; s < S; ++s) if (indeg[s] == 0) stack[top++] = s;
  while (top > 0) {
    int32_t s = stack[--top]; ++seen;
    for (int64_t a = p->x_off[s]; a < p->x_off[s + 1]; ++a)
      if (--indeg[p->x_next[a]] == 0) stack[top++] = p->x_next[a];
  }
  free(indeg); free(stack);
  if (seen != S) { oracle_free(p); return NULL; }
  return p;
}

int64_t oracle_num_emitting(const oracle_prepared *p) { return p->Ae; }
int64_t oracle_num_epsilon(const oracle_prepared *p) { return p->Ax; }
/* global arc id -> index of that arc in the arrays the caller passed to oracle_prepare */
int64_t oracle_arc_original_index(const oracle_prepared *p, int64_t gid) {
  if (gid < 0 || gid >= p->Ae + p->Ax) return -1;
  return gid < p->Ae ? p->e_orig[gid] : p->x_orig[gid - p->Ae];
}

/* ------------------------------------------------------------------ pruning rule (R4, R5) */
typedef struct { float best, beam, scale; int32_t k_keep; } cutoff_t;

static int32_t bin_of(float c, const cutoff_t *k) {
  if (k->beam == 0.0f) return 0;
  float x = floorf((c - k->best) * k->scale);
  if (!(x > 0.0f)) return 0;          /* negative gap, zero, or NaN from inf*0 */
  if (x > 255.0f) return 255;
  return (int32_t)x;
}
static int keep(float c, const cutoff_t *k) {
  return ((c - k->best) <= k->beam) && (bin_of(c, k) < k->k_keep);
}

/* Cutoff of a set of recombined costs.  Outputs best and k_keep; returns the number of
 * tokens in the beam.  hist_out (256 ints) may be NULL. */
int32_t oracle_cutoff(const float *costs, int32_t n, float beam, int32_t max_active,
                      float *best_out, int32_t *k_keep_out, int32_t *hist_out) {
  cutoff_t k; k.beam = beam; k.scale = 256.0f / beam; k.k_keep = 256;
  float best = INFINITY;
  for (int32_t i = 0; i < n; ++i) if (costs[i] < best) best = costs[i];
  k.best = best;
  int32_t hist[256]; memset(hist, 0, sizeof(hist));
  int32_t n_in = 0;
  for (int32_t i = 0; i < n; ++i)
    if ((costs[i] - best) <= beam) { hist[bin_of(costs[i], &k)]++; ++n_in; }
  int32_t k_keep = 256;
  if (n_in > max_active) {
    int64_t run = 0;
    for (int32_t j = 0; j < 256; ++j) { run += hist[j]; if (run > max_active) { k_keep = j; break; } }
    if (k_keep < 1) k_keep = 1;
  }
  *best_out = best; *k_keep_out = k_keep;
  if (hist_out) memcpy(hist_out, hist, sizeof(hist));
  return n_in;
}
int32_t oracle_keep(float c, float best, float beam, int32_t k_keep) {
  cutoff_t k; k.best = best; k.beam = beam; k.scale = 256.0f / beam; k.k_keep = k_keep;
  return keep(c, &k);
}

/* ------------------------------------------------------------------ token sets */
typedef struct { int32_t state; float cost; int32_t prev; int32_t arc;
                 int32_t b;      /* state of the boosting acceptor (R12); 0 without one */
                 int32_t link;   /* next token of the same graph state, or -1 */
} token_t;
typedef struct { token_t *t; int32_t n, cap; } tokvec;

static void tv_push(tokvec *v, token_t x) {
  if (v->n == v->cap) { v->cap = v->cap ? v->cap * 2 : 1024; v->t = (token_t *)realloc(v->t, sizeof(token_t) * v->cap); }
  v->t[v->n++] = x;
}
static float canon(float x) { return x == 0.0f ? 0.0f : x; }   /* -0.0 -> +0.0 */

/* One token per (graph state, B state).  head[s] starts the chain of the tokens of graph state s
 * (one per B state; a single token without a boosting acceptor), -1 if there is none. */
static int32_t tok_find(const tokvec *v, const int32_t *head, int32_t s, int32_t b) {
  for (int32_t q = head[s]; q >= 0; q = v->t[q].link) if (v->t[q].b == b) return q;
  return -1;
}
static int32_t tok_add(tokvec *v, int32_t *head, int32_t s, int32_t b, float cost, int32_t prev, int32_t arc) {
  token_t t = { s, cost, prev, arc, b, head[s] };
  head[s] = v->n;
  tv_push(v, t);
  return v->n - 1;
}

/* What an output label does to a token (R9, R12). */
typedef struct {
  const float *table;      /* R9: dense over output labels, or NULL */
  int32_t n_states, n_arcs;                     /* R12 */
  const int32_t *from, *label, *to; const float *score;
} booster;
/* arc of B out of state b on label o, or -1 */
static int32_t bfst_arc(const booster *B, int32_t b, int32_t o) {
  for (int32_t i = 0; i < B->n_arcs; ++i) if (B->from[i] == b && B->label[i] == o) return i;
  return -1;
}
/* Token in B state b takes an arc with output label o != 0: returns the new B state; *add says
 * whether a score is added and *score which. */
static int32_t boost_step(const booster *B, int32_t b, int32_t o, int *add, float *score) {
  *add = 0; *score = 0.0f;
  if (B->table) { *add = 1; *score = B->table[o]; return 0; }
  if (B->n_states <= 0) return 0;
  int32_t i = bfst_arc(B, b, o);
  if (i < 0 && b != 0) i = bfst_arc(B, 0, o);   /* failure arc to the root, then once more */
  if (i < 0) return 0;
  *add = 1; *score = B->score[i];
  return B->to[i];
}

static uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
static uint64_t rng_next(uint64_t *s) { *s += 0x9E3779B97F4A7C15ull; return mix64(*s); }

/* Epsilon closure (R6) of the token set `v` in place, under the frozen predicate `k`.
 * head[state] = chain of the state's tokens in v (tok_find).  The worklist is consumed from the
 * front (order 0), from the back (1) or at a seeded random position (2); `head_` only moves
 * in order 0.  The result does not depend on the order. */
static void eps_closure(const oracle_prepared *p, tokvec *v, int32_t *head, const cutoff_t *k,
                        int32_t order, uint64_t seed, const booster *B) {
  int32_t *wl = NULL; int32_t wn = 0, wcap = 0, head_ = 0;
  for (int32_t i = 0; i < v->n; ++i) {
    if (wn == wcap) { wcap = wcap ? wcap * 2 : 1024; wl = (int32_t *)realloc(wl, sizeof(int32_t) * wcap); }
    wl[wn++] = i;
  }
  while (head_ < wn) {
    int32_t j;
    if (order == 0) j = wl[head_++];
    else if (order == 1) j = wl[--wn];
    else { int32_t r = head_ + (int32_t)(rng_next(&seed) % (uint64_t)(wn - head_)); j = wl[r]; wl[r] = wl[--wn]; }
    int32_t s = v->t[j].state; float c = v->t[j].cost; int32_t b = v->t[j].b;
    for (int64_t a = p->x_off[s]; a < p->x_off[s + 1]; ++a) {
      float nc = canon(c + p->x_w[a]);
      int32_t nb = b;
      if (B && p->x_ol[a] != 0) {
        int add; float sc;
        nb = boost_step(B, b, p->x_ol[a], &add, &sc);
        if (add) nc = canon(nc + sc);
      }
      if (!(nc < INFINITY)) continue;
      if (!keep(nc, k)) continue;
      int32_t d = p->x_next[a]; int32_t gid = (int32_t)(p->Ae + a);
      int32_t q = tok_find(v, head, d, nb);
      if (q < 0) {
        q = tok_add(v, head, d, nb, nc, j, gid);
      } else if (nc < v->t[q].cost || (nc == v->t[q].cost && gid < v->t[q].arc) ||
                 (nc == v->t[q].cost && gid == v->t[q].arc && b < v->t[v->t[q].prev].b)) {
        v->t[q].cost = nc; v->t[q].prev = j; v->t[q].arc = gid;
      } else continue;
      if (wn == wcap) { wcap = wcap ? wcap * 2 : 1024; wl = (int32_t *)realloc(wl, sizeof(int32_t) * wcap); }
      wl[wn++] = q;
    }
  }
  free(wl);
}

/* Closure of an arbitrary seed set, exported for tests of R6.
 * in: n seed tokens (states distinct); out arrays must hold `cap` entries. Returns count or -1. */
int32_t oracle_eps_closure(const oracle_prepared *p, const int32_t *states, const float *costs,
                           int32_t n, float best, float beam, int32_t k_keep, int32_t order,
                           uint64_t seed, int32_t *out_states, float *out_costs,
                           int32_t *out_prev, int32_t *out_arc, int32_t cap) {
  cutoff_t k; k.best = best; k.beam = beam; k.scale = 256.0f / beam; k.k_keep = k_keep;
  int32_t *map = (int32_t *)malloc(sizeof(int32_t) * p->S);
  for (int32_t s = 0; s < p->S; ++s) map[s] = -1;
  tokvec v = { 0, 0, 0 };
  for (int32_t i = 0; i < n; ++i) tok_add(&v, map, states[i], 0, costs[i], -1, -1);
  eps_closure(p, &v, map, &k, order, seed, NULL);
  int32_t ret = v.n;
  if (ret > cap) ret = -1;
  else for (int32_t i = 0; i < v.n; ++i) {
    out_states[i] = v.t[i].state; out_costs[i] = v.t[i].cost;
    if (out_prev) out_prev[i] = v.t[i].prev;
    if (out_arc) out_arc[i] = v.t[i].arc;
  }
  free(v.t); free(map);
  return ret;
}

/* ------------------------------------------------------------------ the decoder */
typedef struct { int32_t prev, arc; } bp_t;

/*
 * Decode one utterance.  loglikes: [len][V] row-major (row stride `row_stride` floats).
 * words: [opts->max_words].  Optional outputs (NULL to skip):
 *   digest_count/digest_sum [len+1]: per closed token set A_0..A_len, its size and the sum
 *     over tokens of mix64((state<<32 | cost bits) ^ B state * 0x9E3779B97F4A7C15) modulo 2^64;
 *   path_arcs [path_cap]: global arc ids of the best path in order (res->path_len of them);
 *   dump_off [len+2], dump_states/dump_costs (and dump_bstates, may be NULL) [dump_cap]: every
 *     closed token set;
 *   frame_best [len+1]: with cost offsets (R11) the best cost b_t that the tokens of A_t were
 *     rebased by (0 for A_0, for empty sets and without offsets).
 * Returns 0, or -1 on bad arguments, -2 if a dump/path buffer is too small.
 */
int32_t oracle_decode(const oracle_prepared *p, const float *loglikes, int64_t row_stride,
                      int32_t len, const oracle_opts *o, int32_t *words, oracle_result *res,
                      int32_t *digest_count, uint64_t *digest_sum,
                      int32_t *path_arcs, int32_t path_cap,
                      int64_t *dump_off, int32_t *dump_states, float *dump_costs, int64_t dump_cap,
                      float *frame_best, int32_t *dump_bstates) {
  if (!p || !o || !res || len < 0 || o->max_words < 0 || !(o->beam >= 0.0f)) return -1;
  if (o->bfst_states > 0) {                     /* R12: a well-formed deterministic acceptor, and no table beside it */
    if (o->boost_n > 0 || o->bfst_arcs < 0) return -1;
    for (int32_t i = 0; i < o->bfst_arcs; ++i) {
      if (o->bfst_from[i] < 0 || o->bfst_from[i] >= o->bfst_states || o->bfst_to[i] < 0 ||
          o->bfst_to[i] >= o->bfst_states || o->bfst_label[i] <= 0 || !isfinite(o->bfst_score[i])) return -1;
      for (int32_t j = 0; j < i; ++j)
        if (o->bfst_from[j] == o->bfst_from[i] && o->bfst_label[j] == o->bfst_label[i]) return -1;
    }
  }
  memset(res, 0, sizeof(*res));
  int32_t rc = 0;
  int32_t *map = (int32_t *)malloc(sizeof(int32_t) * p->S);
  for (int32_t s = 0; s < p->S; ++s) map[s] = -1;
  bp_t **lat = (bp_t **)calloc((size_t)len + 1, sizeof(bp_t *));
  int32_t *lat_n = (int32_t *)calloc((size_t)len + 1, sizeof(int32_t));
  tokvec cur = { 0, 0, 0 }, nxt = { 0, 0, 0 };
  int64_t dump_used = 0;
  cutoff_t k; k.beam = o->beam; k.scale = 256.0f / o->beam;
  double offset_sum = 0.0;                      /* R11 */
  float *cost_buf = NULL; int32_t cost_cap = 0;
  /* boost table as a dense array over output labels (absent words add exactly 0) */
  float *boost = NULL;
  if (o->boost_n > 0) {
    int32_t max_ol = 0;
    for (int64_t a = 0; a < p->Ae; ++a) if (p->e_ol[a] > max_ol) max_ol = p->e_ol[a];
    for (int64_t a = 0; a < p->Ax; ++a) if (p->x_ol[a] > max_ol) max_ol = p->x_ol[a];
    boost = (float *)calloc((size_t)max_ol + 1, sizeof(float));
    for (int32_t i = 0; i < o->boost_n; ++i)
      if (o->boost_ids[i] > 0 && o->boost_ids[i] <= max_ol) boost[o->boost_ids[i]] = o->boost_scores[i];
  }

  booster Bst = { boost, o->bfst_states, o->bfst_arcs, o->bfst_from, o->bfst_label, o->bfst_to, o->bfst_score };
  const booster *B = (boost || o->bfst_states > 0) ? &Bst : NULL;

  if (frame_best) frame_best[0] = 0.0f;
  /* initial set: start token (in the root of B), closed over epsilon arcs with best = 0 and no bin limit */
  tok_add(&cur, map, p->start, 0, 0.0f, -1, -1);
  k.best = 0.0f; k.k_keep = 256;
  eps_closure(p, &cur, map, &k, o->worklist_order, o->order_seed, B);

  for (int32_t t = 0; t <= len; ++t) {
    /* ---- store the closed set A_t: backpointers, digest, counters, dump */
    lat_n[t] = cur.n;
    lat[t] = (bp_t *)malloc(sizeof(bp_t) * (cur.n ? cur.n : 1));
    uint64_t dsum = 0;
    for (int32_t i = 0; i < cur.n; ++i) {
      lat[t][i].prev = cur.t[i].prev; lat[t][i].arc = cur.t[i].arc;
      uint32_t cb; memcpy(&cb, &cur.t[i].cost, 4);
      dsum += mix64((((uint64_t)(uint32_t)cur.t[i].state << 32) | cb) ^
                    ((uint64_t)(uint32_t)cur.t[i].b * 0x9E3779B97F4A7C15ull));
      res->counters[2] += p->x_off[cur.t[i].state + 1] - p->x_off[cur.t[i].state];
    }
    res->counters[4] += cur.n;
    if (digest_count) digest_count[t] = cur.n;
    if (digest_sum) digest_sum[t] = dsum;
    if (dump_off) {
      dump_off[t] = dump_used;
      if (dump_used + cur.n > dump_cap) { rc = -2; goto done; }
      for (int32_t i = 0; i < cur.n; ++i) {
        dump_states[dump_used + i] = cur.t[i].state; dump_costs[dump_used + i] = cur.t[i].cost;
        if (dump_bstates) dump_bstates[dump_used + i] = cur.t[i].b;
      }
      dump_used += cur.n; dump_off[t + 1] = dump_used;
    }
    if (t == len) break;

    /* ---- ExpandArcs over emitting arcs + recombination (R2, R3) */
    const float *L = loglikes + (int64_t)t * row_stride;
    for (int32_t i = 0; i < cur.n; ++i) map[cur.t[i].state] = -1;
    nxt.n = 0;
    res->counters[0] += cur.n;
    for (int32_t i = 0; i < cur.n; ++i) {
      int32_t s = cur.t[i].state; float c = cur.t[i].cost; int32_t b = cur.t[i].b;
      res->counters[1] += p->e_off[s + 1] - p->e_off[s];
      for (int64_t a = p->e_off[s]; a < p->e_off[s + 1]; ++a) {
        float ac = -L[p->e_il[a] - 1];
        float nc = canon((c + p->e_w[a]) + ac);
        int32_t nb = b;
        if (B && p->e_ol[a] != 0) {
          int add; float sc;
          nb = boost_step(B, b, p->e_ol[a], &add, &sc);
          if (add) nc = canon(nc + sc);
        }
        if (!(nc < INFINITY)) continue;
        int32_t d = p->e_next[a]; int32_t q = tok_find(&nxt, map, d, nb);
        if (q < 0) tok_add(&nxt, map, d, nb, nc, i, (int32_t)a);
        else if (nc < nxt.t[q].cost || (nc == nxt.t[q].cost && (int32_t)a < nxt.t[q].arc) ||
                 (nc == nxt.t[q].cost && (int32_t)a == nxt.t[q].arc && b < cur.t[nxt.t[q].prev].b)) {
          nxt.t[q].cost = nc; nxt.t[q].prev = i; nxt.t[q].arc = (int32_t)a;
        }
      }
    }
    res->counters[7] += nxt.n;
    /* ---- Prune: beam from the best cost, max-active through the histogram (R4, R5): the
     * one cutoff routine, applied to the costs of the recombined set */
    if (nxt.n > cost_cap) { cost_cap = nxt.n * 2; cost_buf = (float *)realloc(cost_buf, sizeof(float) * cost_cap); }
    for (int32_t i = 0; i < nxt.n; ++i) cost_buf[i] = nxt.t[i].cost;
    float best; int32_t k_keep, hist[256];
    int32_t n_in = oracle_cutoff(cost_buf, nxt.n, o->beam, o->max_active, &best, &k_keep, hist);
    k.best = best; k.k_keep = k_keep;
    if (n_in > o->max_active) {
      res->counters[5]++;
      if (hist[0] > o->max_active) res->counters[6]++;
    }
    int32_t m = 0;
    for (int32_t i = 0; i < nxt.n; ++i) map[nxt.t[i].state] = -1;
    for (int32_t i = 0; i < nxt.n; ++i)
      if (keep(nxt.t[i].cost, &k)) {               /* survivors move up; their chains are rebuilt */
        nxt.t[m] = nxt.t[i]; nxt.t[m].link = map[nxt.t[m].state]; map[nxt.t[m].state] = m; ++m;
      }
    nxt.n = m;
    res->counters[3] += m;
    if (frame_best) frame_best[t + 1] = 0.0f;
    if (o->cost_offset && m > 0) {              /* R11 */
      for (int32_t i = 0; i < m; ++i) nxt.t[i].cost = canon(nxt.t[i].cost - best);
      offset_sum += (double)best;
      k.best = 0.0f;
      if (frame_best) frame_best[t + 1] = best;
    }
    /* ---- epsilon closure under the frozen predicate (R6) */
    eps_closure(p, &nxt, map, &k, o->worklist_order, o->order_seed + (uint64_t)t + 1, B);
    { tokvec tmp = cur; cur = nxt; nxt = tmp; }
  }

  /* ---- final choice (R8) and traceback */
  if (cur.n == 0) {
    res->flags = FLAG_DEAD; res->cost = INFINITY; res->nwords = 0; res->path_len = 0;
  } else {
    int32_t bi = -1; float bf = INFINITY; int any_final = 0;
    if (o->finalize) {
      for (int32_t i = 0; i < cur.n; ++i) {
        float f = cur.t[i].cost + p->final_cost[cur.t[i].state];
        if (!(f < INFINITY)) continue;
        if (bi < 0 || f < bf || (f == bf && cur.t[i].state < cur.t[bi].state) ||
            (f == bf && cur.t[i].state == cur.t[bi].state && cur.t[i].b < cur.t[bi].b)) { bi = i; bf = f; }
        any_final = 1;
      }
    }
    if (!any_final) {
      for (int32_t i = 0; i < cur.n; ++i) {
        float f = cur.t[i].cost;
        if (bi < 0 || f < bf || (f == bf && cur.t[i].state < cur.t[bi].state) ||
            (f == bf && cur.t[i].state == cur.t[bi].state && cur.t[i].b < cur.t[bi].b)) { bi = i; bf = f; }
      }
    }
    res->cost = o->cost_offset ? (float)((double)bf + offset_sum) : bf;
    res->flags = any_final ? FLAG_FINAL : 0;
    /* walk back: an epsilon arc's prev indexes the same frame, an emitting arc's the one before */
    int32_t plen = 0, pcap = 1024; int32_t *rev = (int32_t *)malloc(sizeof(int32_t) * pcap);
    int32_t f = len, i = bi;
    while (lat[f][i].arc >= 0) {
      int32_t a = lat[f][i].arc;
      if (plen == pcap) { pcap *= 2; rev = (int32_t *)realloc(rev, sizeof(int32_t) * pcap); }
      rev[plen++] = a;
      i = lat[f][i].prev;
      if ((int64_t)a < p->Ae) --f;
    }
    res->path_len = plen;
    int32_t nw = 0;
    for (int32_t q = plen - 1; q >= 0; --q) {
      int32_t a = rev[q];
      int32_t ol = (int64_t)a < p->Ae ? p->e_ol[a] : p->x_ol[a - p->Ae];
      if (ol != 0) { if (nw < o->max_words) words[nw++] = ol; else res->flags |= FLAG_TRUNC; }
    }
    res->nwords = nw;
    if (path_arcs) {
      if (plen > path_cap) rc = -2;
      else for (int32_t q = 0; q < plen; ++q) path_arcs[q] = rev[plen - 1 - q];
    }
    free(rev);
  }
done:
  for (int32_t t = 0; t <= len; ++t) free(lat[t]);
  free(lat); free(lat_n); free(cur.t); free(nxt.t); free(map); free(boost); free(cost_buf);
  return rc;
}

/*
 * Lattice links (R10) between the closed token sets of one utterance, which the caller got
 * from oracle_decode's dump (set_off [len+2], set_states, set_costs).  Outputs, one entry per
 * link, ordered by frame, then epsilon links before emitting links, then source token, then
 * arc: l_frame = t of the destination set A_t; l_src / l_dst = token positions inside their
 * sets (the source of an emitting link lies in A_{t-1}, of an epsilon link in A_t); l_arc =
 * global arc id (R3); l_cost = cost through the arc.  frame_best: NULL, or the per-set offsets
 * of a decode with cost offsets (R11).  Returns the number of links (only the first `cap` are
 * written), or -1 on bad arguments.
 */
int64_t oracle_lattice_links(const oracle_prepared *p, const float *loglikes, int64_t row_stride,
                             int32_t len, const oracle_opts *o, float lattice_beam,
                             const int64_t *set_off, const int32_t *set_states, const float *set_costs,
                             const float *frame_best,
                             int64_t cap, int32_t *l_frame, int32_t *l_src, int32_t *l_dst,
                             int32_t *l_arc, float *l_cost) {
  if (!p || !o || len < 0 || !set_off || !(lattice_beam >= 0.0f)) return -1;
  if (o->bfst_states > 0) return -1;            /* the lattice definition (R10) is over graph states only */
  float *boost = NULL;
  if (o->boost_n > 0) {
    int32_t max_ol = 0;
    for (int64_t a = 0; a < p->Ae; ++a) if (p->e_ol[a] > max_ol) max_ol = p->e_ol[a];
    for (int64_t a = 0; a < p->Ax; ++a) if (p->x_ol[a] > max_ol) max_ol = p->x_ol[a];
    boost = (float *)calloc((size_t)max_ol + 1, sizeof(float));
    for (int32_t i = 0; i < o->boost_n; ++i)
      if (o->boost_ids[i] > 0 && o->boost_ids[i] <= max_ol) boost[o->boost_ids[i]] = o->boost_scores[i];
  }
  int32_t *where = (int32_t *)malloc(sizeof(int32_t) * p->S);     /* state -> position in A_t */
  for (int32_t s = 0; s < p->S; ++s) where[s] = -1;
  int64_t n = 0;
#define PUT(T, I, J, A, C_) do { if (n < cap) { l_frame[n] = (T); l_src[n] = (I); l_dst[n] = (J); \
                                               l_arc[n] = (int32_t)(A); l_cost[n] = (C_); } ++n; } while (0)
  for (int32_t t = 0; t <= len; ++t) {
    const int32_t *S1 = set_states + set_off[t]; const float *C1 = set_costs + set_off[t];
    const int32_t n1 = (int32_t)(set_off[t + 1] - set_off[t]);
    for (int32_t j = 0; j < n1; ++j) where[S1[j]] = j;
    /* epsilon arcs between two tokens of A_t */
    for (int32_t i = 0; i < n1; ++i) {
      for (int64_t a = p->x_off[S1[i]]; a < p->x_off[S1[i] + 1]; ++a) {
        float nc = canon(C1[i] + p->x_w[a]);
        if (boost && p->x_ol[a] != 0) nc = canon(nc + boost[p->x_ol[a]]);
        const int32_t j = where[p->x_next[a]];
        if (!(nc < INFINITY) || j < 0) continue;
        if ((nc - C1[j]) <= lattice_beam) PUT(t, i, j, p->Ae + a, nc);
      }
    }
    /* emitting arcs from the tokens of A_{t-1}, against row t-1 */
    if (t > 0) {
      const int32_t *S0 = set_states + set_off[t - 1]; const float *C0 = set_costs + set_off[t - 1];
      const int32_t n0 = (int32_t)(set_off[t] - set_off[t - 1]);
      const float *L = loglikes + (int64_t)(t - 1) * row_stride;
      for (int32_t i = 0; i < n0; ++i) {
        for (int64_t a = p->e_off[S0[i]]; a < p->e_off[S0[i] + 1]; ++a) {
          float nc = canon((C0[i] + p->e_w[a]) + (-L[p->e_il[a] - 1]));
          if (boost && p->e_ol[a] != 0) nc = canon(nc + boost[p->e_ol[a]]);
          if (frame_best) nc = canon(nc - frame_best[t]);    /* into the cost base of A_t */
          const int32_t j = where[p->e_next[a]];
          if (!(nc < INFINITY) || j < 0) continue;
          if ((nc - C1[j]) <= lattice_beam) PUT(t, i, j, a, nc);
        }
      }
    }
    for (int32_t j = 0; j < n1; ++j) where[S1[j]] = -1;
  }
#undef PUT
  free(where); free(boost);
  return n;
}
