/*
 * TEST INFRASTRUCTURE -- plain, slow CPU oracle of the TACOS synthesis path.
 *
 * This file is the reference the HIP path is compared against.  It is NOT part of
 * the product: only the tests, the smoke check and the benchmark's cpu_baseline leg
 * may build, load or call it, and it shares no code, header, table or helper with
 * the HIP path.
 *
 * What it computes (paper: TACOS, arXiv 2304.05301):
 *   - link cost alpha + beta*n of the alpha-beta model (section "TACOS for
 *     Heterogeneous Networks"), in integer picoseconds;
 *   - the end-to-end synthesis loop of Algorithm 2 (expand the time-expanded network
 *     by one span, run the matching, repeat until no postcondition is unsatisfied),
 *     event-driven so that the spans of a heterogeneous network fall on the arrival
 *     times of its links;
 *   - the utilization-maximizing link-chunk matching of Algorithm 1 for one span, in
 *     the link-centric, deterministic form: destinations in turn, each destination's
 *     incoming idle links in ascending link id (or cheapest first, the paper's
 *     "Prioritizing Lower-cost Links", when asked), every link matched to the
 *     (r mod p)-th smallest chunk of the p chunks its source holds, its destination
 *     lacks and is not already receiving; r is Philox4x32-10 keyed by the seed and
 *     countered by (link, event, phase).  One chunk per link (section "Representing
 *     Collective Algorithms using TEN"), a chunk is delivered to an NPU once
 *     (Algorithm 1 marks it at match time);
 *   - Reduce-Scatter as the reversed All-Gather on the link-reversed topology and
 *     All-Reduce as Reduce-Scatter followed by All-Gather (paragraph "Collectives
 *     with Reduction Operations").
 *
 * Readings of points the paper leaves open are listed with the function they
 * affect.  No floating point is used anywhere.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors; unidirectional N-ring
 * = N-1 steps with a unique schedule; fully connected = 1 step; bidirectional ring
 * = ceil((N-1)/2) steps; ingress and diameter lower bounds; brute-force optimal
 * step counts for all strongly connected digraphs with N <= 4; an independent
 * schedule checker (validity, one chunk per link, maximality); RS/AR structure;
 * exact replays of two-NPU cases from the rule alone (equal and unequal link costs,
 * the latter with a span that matches nothing; parallel links for the postcondition-
 * centric draw); collective times and span counts of an independent implementation
 * for the 8x8-mesh All-Gather and the heterogeneous 4x4x8-torus All-Reduce.  Every
 * planted mistake of tests/test_oracle_mutants.py is noticed by a named pin.
 * The full-size 40,960-NPU result has no value pin of its own: parity unpinned
 * except by those invariants and bounds.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_NONE 0xFFFFFFFFu
#define ORC_INF  0xFFFFFFFFFFFFFFFFull

enum { ORC_ALL_GATHER = 0, ORC_REDUCE_SCATTER = 1, ORC_ALL_REDUCE = 2, ORC_BROADCAST = 3, ORC_REDUCE = 4 };
enum { ORC_OK = 0, ORC_E_INVAL = -1, ORC_E_UNREACHABLE = -2, ORC_E_OVERFLOW = -3, ORC_E_NOMEM = -4 };

typedef struct {
  uint64_t t_ps;
  uint32_t src, dst, chunk, link;
} orc_xfer_t;

typedef struct {
  uint64_t collective_time_ps;
  uint64_t n_xfers;        /* records of all passes                                   */
  uint64_t n_events;       /* matching sweeps of all passes                           */
  uint64_t n_attempts;     /* idle-link candidate evaluations of all passes           */
  uint64_t digest;         /* sum of orc_mix(t, link, chunk) over every record        */
  uint64_t pass_time_ps[2];
  uint64_t pass_events[2];
  uint64_t n_stored;       /* records kept in xfers (canonical order)                 */
  orc_xfer_t *xfers;
  uint64_t n_event_times;  /* event times of the LAST pass (diagnostics)              */
  uint64_t *event_times;
  uint32_t *event_matches; /* matches made at each of those events                    */
} orc_result_t;

/* ------------------------------------------------------------------ Philox4x32-10 */
/* Counter-based generator of Salmon, Moraes, Dror and Shaw (SC'11): ten rounds of
 * two 32x32->64 multiplies with a Weyl-sequence key schedule. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The random word that picks a chunk for `link` at matching sweep `event` of pass
 * `phase` (0 = forward/All-Gather pass, 1 = reversed pass of a Reduce-Scatter). */
static uint32_t draw(uint64_t seed, uint32_t link, uint32_t event, uint32_t phase)
{
  uint32_t ctr[4] = { link, event, phase, 0u };
  uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  return out[0];
}

/* The two random words of step i of destination d in the postcondition-centric
 * matching: word 0 picks the chunk, word 1 the source link. */
static void draw_pair(uint64_t seed, uint32_t d, uint32_t event, uint32_t phase, uint32_t i,
                      uint32_t *r_chunk, uint32_t *r_link)
{
  uint32_t ctr[4] = { d, event, phase + 2u, i };
  uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  *r_chunk = out[0];
  *r_link = out[1];
}

/* ------------------------------------------------------------------------ digest */
/* Order-independent schedule digest: every record contributes a 64-bit mix of its
 * start time, link id and chunk id; contributions add modulo 2^64. */
uint64_t orc_mix(uint64_t t_ps, uint32_t link, uint32_t chunk)
{
  uint64_t h = t_ps ^ ((((uint64_t)link << 32) | (uint64_t)chunk) * 0x9E3779B97F4A7C15ull);
  h ^= h >> 33; h *= 0xFF51AFD7ED558CCDull;
  h ^= h >> 33; h *= 0xC4CEB9FE1A85EC53ull;
  h ^= h >> 33;
  return h;
}

/* --------------------------------------------------------------------- link cost */
/* alpha + beta*n, rounded to the nearest picosecond (beta is given in fs/byte).
 * Returns 0 and leaves *cost alone if the value does not fit 64 bits. */
int orc_link_cost(uint64_t alpha_ps, uint64_t beta_fs_per_B, uint64_t chunk_bytes, uint64_t *cost)
{
  unsigned __int128 fs = (unsigned __int128)beta_fs_per_B * chunk_bytes + 500u;
  unsigned __int128 ps = fs / 1000u + alpha_ps;
  if (ps >= (unsigned __int128)ORC_INF) return 0;
  *cost = (uint64_t)ps;
  return 1;
}

/* Optional progress lines on stderr every `every` matching sweeps (0 = silent), for
 * runs that take minutes. */
static uint64_t g_progress_every = 0;
void orc_set_progress(uint64_t every) { g_progress_every = every; }

/* ------------------------------------------------------------------- one pass   */
typedef struct { uint64_t t; uint32_t link, chunk; } pass_rec_t;

typedef struct {
  pass_rec_t *rec; uint64_t n, cap;
  uint64_t *ev_time; uint32_t *ev_matches; uint64_t n_ev, cap_ev;
  uint64_t keep_first;   /* store the records with generation index in              */
  uint64_t keep_limit;   /*   [keep_first, keep_first+keep_limit); all are counted  */
  uint64_t n_total;      /* records generated                                       */
  uint64_t n_attempts;
  int      fwd;          /* forward pass: digest every record as it is generated   */
  uint64_t t_off;        /* time offset of the pass in the whole collective        */
  uint64_t digest;
} pass_out_t;

/* Which records of a forward pass are stored (all are counted and digested): by default the
 * window [keep_first, keep_first + keep_limit); with orc_set_keep_windows(stride, block),
 * stride > 0, the blocks of `block` records that start at keep_first + k * stride, k = 0, 1, ...
 * (samples spread over a run whose records do not fit memory). */
static uint64_t g_keep_stride = 0, g_keep_block = 0;
void orc_set_keep_windows(uint64_t stride, uint64_t block) { g_keep_stride = stride; g_keep_block = block; }

static int push_rec(pass_out_t *o, uint64_t t, uint32_t link, uint32_t chunk)
{
  o->n_total++;
  if (o->fwd) o->digest += orc_mix(t + o->t_off, link, chunk);
  if (o->n_total - 1 < o->keep_first || o->n >= o->keep_limit) return 1;
  if (o->fwd && g_keep_stride && (o->n_total - 1 - o->keep_first) % g_keep_stride >= g_keep_block) return 1;
  if (o->n == o->cap) {
    uint64_t nc = o->cap ? o->cap * 2 : 1024;
    pass_rec_t *p = (pass_rec_t *)realloc(o->rec, nc * sizeof(pass_rec_t));
    if (!p) return 0;
    o->rec = p; o->cap = nc;
  }
  o->rec[o->n].t = t; o->rec[o->n].link = link; o->rec[o->n].chunk = chunk;
  o->n++;
  return 1;
}

static int push_event(pass_out_t *o, uint64_t t, uint32_t matches)
{
  if (o->n_ev == o->cap_ev) {
    uint64_t nc = o->cap_ev ? o->cap_ev * 2 : 1024;
    uint64_t *p = (uint64_t *)realloc(o->ev_time, nc * sizeof(uint64_t));
    if (!p) return 0;
    o->ev_time = p;
    uint32_t *q = (uint32_t *)realloc(o->ev_matches, nc * sizeof(uint32_t));
    if (!q) return 0;
    o->ev_matches = q; o->cap_ev = nc;
  }
  o->ev_time[o->n_ev] = t; o->ev_matches[o->n_ev] = matches; o->n_ev++;
  return 1;
}

/* k-th (0-based) set bit of a non-zero word, counting from the least significant. */
static uint32_t kth_bit(uint64_t w, uint32_t k)
{
  while (k--) w &= w - 1;           /* drop the k lowest set bits */
  return (uint32_t)__builtin_ctzll(w);
}

/*
 * One All-Gather pass over the links (psrc[l] -> pdst[l]) with cost[l].
 *
 * State, in the paper's terms: held = precondition (chunks that have ARRIVED at an
 * NPU: only these qualify it as a source); inflight = chunks matched to an NPU and
 * not yet arrived (they only prevent a second delivery); carry/free_at = the chunk
 * on a link of the time-expanded network and the time the link is free again.
 *
 * Readings: a chunk that arrives at time t may be forwarded at t (arrivals are
 * applied before matching at the same event time); every idle link is tried at
 * every event, whether it became free now or earlier; event indices count the
 * matching sweeps of the pass from 0 and include sweeps that match nothing; chunk c
 * is owned by NPU c / chunks_per_npu.
 *
 * Emits (start time, link, chunk) in (time, link id) order.  *T = time of the last
 * arrival.  max_events > 0 stops after that many matching sweeps (prefix runs for
 * large inputs; *T is then the time reached and *complete = 0).
 */
static int ag_pass(uint32_t N, uint32_t L, const uint32_t *psrc, const uint32_t *pdst,
                   const uint64_t *cost, uint32_t cpn, uint64_t seed, uint32_t phase,
                   uint64_t max_events, int n_threads, int link_order, int matching,
                   pass_out_t *out, uint64_t *T, uint64_t *n_events, int *complete, uint32_t root)
{
  /* root == ORC_NONE: All-Gather, N*cpn chunks, chunk c owned by NPU c / cpn.
   * Otherwise Broadcast from `root`: cpn chunks, all held by the root at t = 0; the
   * postcondition is the same (every NPU holds every chunk). */
  const uint64_t C = (root == ORC_NONE) ? (uint64_t)N * cpn : (uint64_t)cpn;
  const uint64_t W = (C + 63) / 64;
  int rc = ORC_OK;
  const size_t n_words = (size_t)N * W;
  uint64_t *held = (uint64_t *)calloc(n_words > 0 ? n_words : 1, sizeof(uint64_t));
  uint64_t *inflight = (uint64_t *)calloc(n_words > 0 ? n_words : 1, sizeof(uint64_t));
  uint32_t *carry = (uint32_t *)malloc((L ? L : 1) * sizeof(uint32_t));
  uint32_t *fresh = (uint32_t *)malloc((L ? L : 1) * sizeof(uint32_t));
  uint64_t *free_at = (uint64_t *)calloc(L ? L : 1, sizeof(uint64_t));
  uint32_t *in_ptr = (uint32_t *)calloc((size_t)N + 2, sizeof(uint32_t));
  uint32_t *in_link = (uint32_t *)malloc((L ? L : 1) * sizeof(uint32_t));
  uint64_t *attempts_d = (uint64_t *)calloc(N ? N : 1, sizeof(uint64_t));
  if (!held || !inflight || !carry || !fresh || !free_at || !in_ptr || !in_link || !attempts_d) {
    rc = ORC_E_NOMEM; goto done;
  }
  /* incoming links of every destination, ascending link id (counting sort is stable) */
  for (uint32_t l = 0; l < L; ++l) in_ptr[pdst[l] + 1]++;
  for (uint32_t d = 0; d < N; ++d) in_ptr[d + 1] += in_ptr[d];
  {
    uint32_t *fill = (uint32_t *)malloc(((size_t)N + 1) * sizeof(uint32_t));
    if (!fill) { rc = ORC_E_NOMEM; goto done; }
    memcpy(fill, in_ptr, ((size_t)N + 1) * sizeof(uint32_t));
    for (uint32_t l = 0; l < L; ++l) in_link[fill[pdst[l]]++] = l;
    free(fill);
  }
  /* "Prioritizing Lower-cost Links": when asked, a destination's incoming links are
   * walked from the cheapest to the most expensive (ties by link id) instead of by
   * link id.  Insertion sort: stable, lists are short. */
  if (link_order == 1) {
    for (uint32_t d = 0; d < N; ++d)
      for (uint32_t j = in_ptr[d] + 1; j < in_ptr[d + 1]; ++j) {
        uint32_t l = in_link[j];
        uint32_t k = j;
        while (k > in_ptr[d] && cost[in_link[k - 1]] > cost[l]) { in_link[k] = in_link[k - 1]; k--; }
        in_link[k] = l;
      }
  }
  /* precondition of All-Gather: NPU i holds its own cpn chunks */
  if (root == ORC_NONE) {
  for (uint32_t i = 0; i < N; ++i)
    for (uint32_t j = 0; j < cpn; ++j) {
      uint64_t c = (uint64_t)i * cpn + j;
      held[(size_t)i * W + (c >> 6)] |= 1ull << (c & 63);
    }
  } else {
    /* precondition of Broadcast: the root holds all cpn chunks, nobody else any */
    for (uint32_t j = 0; j < cpn; ++j) held[(size_t)root * W + (j >> 6)] |= 1ull << (j & 63);
  }
  for (uint32_t l = 0; l < L; ++l) carry[l] = ORC_NONE;

  uint64_t remaining = (uint64_t)N * C - C;   /* unsatisfied postconditions */
  uint64_t t = 0;
  uint64_t event = 0;
  *complete = 0;
  for (;;) {
    /* 1. arrivals at time t: the precondition of the next span */
    for (uint32_t l = 0; l < L; ++l) {
      if (carry[l] != ORC_NONE && free_at[l] == t) {
        uint32_t c = carry[l], d = pdst[l];
        held[(size_t)d * W + (c >> 6)] |= 1ull << (c & 63);
        inflight[(size_t)d * W + (c >> 6)] &= ~(1ull << (c & 63));
        carry[l] = ORC_NONE;
        remaining--;
      }
    }
    /* 2. all postconditions satisfied? */
    if (remaining == 0) { *complete = 1; break; }
    if (max_events && event >= max_events) break;
    if (event > 0xFFFFFFFEull) { rc = ORC_E_OVERFLOW; goto done; }

    /* 3. matching for this span; destinations are independent of each other
     *    because sources are read from `held`, which step 3 does not modify */
    for (uint32_t l = 0; l < L; ++l) fresh[l] = ORC_NONE;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16) num_threads(n_threads)
#endif
    for (uint32_t d = 0; d < N; ++d) {
      const uint64_t *hd = held + (size_t)d * W;
      uint64_t *fd = inflight + (size_t)d * W;
      if (matching == 1) {
        /* Algorithm 1 as printed: unsatisfied postconditions (d, c) are visited in random
         * order, each is given a random in-neighbour that holds c and whose link is free.
         * Visiting a uniformly shuffled list and skipping the pairs no free link can
         * serve is the same as repeatedly drawing a chunk uniformly from the servable
         * ones (links are only ever used up), which is what is done here, with the draws
         * fixed by Philox(d, event, phase + 2, step). */
        for (uint32_t step = 0;; ++step) {
          uint64_t p = 0;
          for (uint64_t w = 0; w < W; ++w) {
            uint64_t any = 0;
            for (uint32_t j = in_ptr[d]; j < in_ptr[d + 1]; ++j) {
              uint32_t l = in_link[j];
              if (carry[l] == ORC_NONE && fresh[l] == ORC_NONE) any |= held[(size_t)psrc[l] * W + w];
            }
            p += (uint64_t)__builtin_popcountll(any & ~hd[w] & ~fd[w]);
          }
          attempts_d[d]++;
          if (p == 0) break;                 /* no free link can serve any missing chunk */
          uint32_t r_chunk, r_link;
          draw_pair(seed, d, (uint32_t)event, phase, step, &r_chunk, &r_link);
          uint32_t k = r_chunk % (uint32_t)p, c = ORC_NONE;
          for (uint64_t w = 0; w < W && c == ORC_NONE; ++w) {
            uint64_t any = 0;
            for (uint32_t j = in_ptr[d]; j < in_ptr[d + 1]; ++j) {
              uint32_t l = in_link[j];
              if (carry[l] == ORC_NONE && fresh[l] == ORC_NONE) any |= held[(size_t)psrc[l] * W + w];
            }
            uint64_t serv = any & ~hd[w] & ~fd[w];
            uint32_t pc = (uint32_t)__builtin_popcountll(serv);
            if (k < pc) c = (uint32_t)(w * 64) + kth_bit(serv, k);
            else k -= pc;
          }
          /* the free links whose source holds c, in list order (ascending link id, or
           * cheapest first); a random one, or with link_order 1 the cheapest */
          uint32_t n_hold = 0;
          for (uint32_t j = in_ptr[d]; j < in_ptr[d + 1]; ++j) {
            uint32_t l = in_link[j];
            if (carry[l] == ORC_NONE && fresh[l] == ORC_NONE &&
                (held[(size_t)psrc[l] * W + (c >> 6)] >> (c & 63) & 1ull)) n_hold++;
          }
          uint32_t pick = (link_order == 1) ? 0u : r_link % n_hold;
          for (uint32_t j = in_ptr[d]; j < in_ptr[d + 1]; ++j) {
            uint32_t l = in_link[j];
            if (carry[l] == ORC_NONE && fresh[l] == ORC_NONE &&
                (held[(size_t)psrc[l] * W + (c >> 6)] >> (c & 63) & 1ull)) {
              if (pick == 0) { fresh[l] = c; fd[c >> 6] |= 1ull << (c & 63); break; }
              pick--;
            }
          }
        }
        continue;
      }
      for (uint32_t j = in_ptr[d]; j < in_ptr[d + 1]; ++j) {
        uint32_t l = in_link[j];
        if (carry[l] != ORC_NONE) continue;            /* link busy */
        const uint64_t *hs = held + (size_t)psrc[l] * W;
        attempts_d[d]++;
        uint64_t p = 0;
        for (uint64_t w = 0; w < W; ++w)
          p += (uint64_t)__builtin_popcountll(hs[w] & ~hd[w] & ~fd[w]);
        if (p == 0) continue;                          /* nothing to send: no draw */
        uint32_t k = draw(seed, l, (uint32_t)event, phase) % (uint32_t)p;
        for (uint64_t w = 0; w < W; ++w) {
          uint64_t cand = hs[w] & ~hd[w] & ~fd[w];
          uint32_t pc = (uint32_t)__builtin_popcountll(cand);
          if (k < pc) {
            uint32_t c = (uint32_t)(w * 64) + kth_bit(cand, k);
            fd[w] |= 1ull << (c & 63);
            fresh[l] = c;
            break;
          }
          k -= pc;
        }
      }
    }
    /* commit the span's matches in link order: TEN[t][src][dst] <- chunk */
    uint32_t matches = 0;
    for (uint32_t l = 0; l < L; ++l) {
      if (fresh[l] == ORC_NONE) continue;
      if (cost[l] > ORC_INF - 1 - t) { rc = ORC_E_OVERFLOW; goto done; }
      carry[l] = fresh[l];
      free_at[l] = t + cost[l];
      if (!push_rec(out, t, l, fresh[l])) { rc = ORC_E_NOMEM; goto done; }
      matches++;
    }
    if (!push_event(out, t, matches)) { rc = ORC_E_NOMEM; goto done; }
    if (g_progress_every && event % g_progress_every == 0) {
      fprintf(stderr, "[oracle] sweep %llu t=%llu ps matches=%u remaining=%llu\n",
              (unsigned long long)event, (unsigned long long)t, matches, (unsigned long long)remaining);
      fflush(stderr);
    }

    /* 4. next span = earliest arrival; nothing in flight and work left = stall */
    uint64_t tn = ORC_INF;
    for (uint32_t l = 0; l < L; ++l)
      if (carry[l] != ORC_NONE && free_at[l] < tn) tn = free_at[l];
    if (tn == ORC_INF) { rc = ORC_E_UNREACHABLE; goto done; }
    t = tn;
    event++;
  }
  *T = t;
  *n_events = event;
  for (uint32_t d = 0; d < N; ++d) out->n_attempts += attempts_d[d];
done:
  free(held); free(inflight); free(carry); free(fresh); free(free_at);
  free(in_ptr); free(in_link); free(attempts_d);
  return rc;
}

/* --------------------------------------------------------------------- top level */
static int cmp_xfer(const void *a, const void *b)
{
  const orc_xfer_t *x = (const orc_xfer_t *)a, *y = (const orc_xfer_t *)b;
  if (x->t_ps != y->t_ps) return x->t_ps < y->t_ps ? -1 : 1;
  if (x->link != y->link) return x->link < y->link ? -1 : 1;
  return 0;
}

void orc_result_free(orc_result_t *r)
{
  if (!r) return;
  free(r->xfers); free(r->event_times); free(r->event_matches); free(r);
}

static void pass_out_free(pass_out_t *o) { free(o->rec); free(o->ev_time); free(o->ev_matches); }

/*
 * Synthesize `collective` on the topology given in CSR-by-source form (link id =
 * index into col_idx).
 *   max_events : 0 = run to completion; >0 = stop every pass after that many
 *                matching sweeps (prefix of a large run; time/digest then cover the
 *                prefix only and the result's collective_time is the time reached).
 *   keep_first, keep_xfers : of the forward (All-Gather) pass, store only the
 *                records with canonical index in [keep_first, keep_first+keep_xfers)
 *                (all are counted and digested); a reversed pass always keeps all.
 *   n_threads  : OpenMP threads for the destination loop of the matching step
 *                (1 = serial; only used when built with -fopenmp).
 *   link_order : 0 = a destination's incoming links are tried in ascending link id;
 *                1 = cheapest link first, ties by link id (the paper's "Prioritizing
 *                Lower-cost Links").  The random draw of a link does not depend on it.
 *   matching   : 0 = link-centric (every idle link draws a chunk); 1 = Algorithm 1 as
 *                printed, postcondition-centric (every missing chunk draws a source
 *                link); see the comment in ag_pass.
 *   root       : Broadcast / Reduce only (paragraph "Collectives with Reduction
 *                Operations": Reduce = the Broadcast synthesized on the reversed links,
 *                reversed back, exactly as Reduce-Scatter is obtained from All-Gather).
 *                Broadcast: the root's chunks_per_npu chunks reach every NPU; Reduce: the
 *                reverse.  Chunk ids are 0 .. chunks_per_npu-1.
 */
int orc_synthesize(uint32_t n_npus, const uint32_t *row_ptr, const uint32_t *col_idx,
                   const uint64_t *alpha_ps, const uint64_t *beta_fs_per_B,
                   uint32_t chunks_per_npu, uint64_t chunk_bytes, int collective,
                   uint64_t seed, uint64_t max_events, uint64_t keep_first,
                   uint64_t keep_xfers, int n_threads, int link_order, int matching,
                   uint32_t root, orc_result_t **result)
{
  if (!row_ptr || !result || n_npus == 0 || chunks_per_npu == 0 || chunk_bytes == 0)
    return ORC_E_INVAL;
  if (collective < ORC_ALL_GATHER || collective > ORC_REDUCE) return ORC_E_INVAL;
  const int rooted = collective == ORC_BROADCAST || collective == ORC_REDUCE;
  if (rooted && root >= n_npus) return ORC_E_INVAL;
  const uint32_t pass_root = rooted ? root : ORC_NONE;
  /* which passes: a reversed one (All-Gather / Broadcast on the reversed links, mapped
   * back in direction and time) and / or a forward one */
  const int has_rev = collective == ORC_REDUCE_SCATTER || collective == ORC_ALL_REDUCE || collective == ORC_REDUCE;
  const int has_fwd = collective == ORC_ALL_GATHER || collective == ORC_ALL_REDUCE || collective == ORC_BROADCAST;
  if (row_ptr[0] != 0) return ORC_E_INVAL;
  for (uint32_t i = 0; i < n_npus; ++i)
    if (row_ptr[i + 1] < row_ptr[i]) return ORC_E_INVAL;
  const uint32_t L = row_ptr[n_npus];
  if (L && (!col_idx || !alpha_ps || !beta_fs_per_B)) return ORC_E_INVAL;
  if ((rooted ? (uint64_t)chunks_per_npu : (uint64_t)n_npus * chunks_per_npu) >= 0xFFFFFFFFull) return ORC_E_INVAL;
  if (n_threads < 1) n_threads = 1;
  if (link_order != 0 && link_order != 1) return ORC_E_INVAL;
  if (matching != 0 && matching != 1) return ORC_E_INVAL;

  int rc = ORC_OK;
  uint32_t *src = (uint32_t *)malloc((L ? L : 1) * sizeof(uint32_t));
  uint64_t *cost = (uint64_t *)malloc((L ? L : 1) * sizeof(uint64_t));
  orc_result_t *res = (orc_result_t *)calloc(1, sizeof(orc_result_t));
  pass_out_t po[2];
  memset(po, 0, sizeof(po));
  if (!src || !cost || !res) { rc = ORC_E_NOMEM; goto fail; }
  for (uint32_t i = 0; i < n_npus; ++i)
    for (uint32_t l = row_ptr[i]; l < row_ptr[i + 1]; ++l) {
      if (col_idx[l] >= n_npus || col_idx[l] == i) { rc = ORC_E_INVAL; goto fail; }
      src[l] = i;
      if (!orc_link_cost(alpha_ps[l], beta_fs_per_B[l], chunk_bytes, &cost[l])) {
        rc = ORC_E_OVERFLOW; goto fail;
      }
    }

  int n_pass = 0;
  int complete_all = 1;
  uint64_t t_off = 0;
  /* Reduce-Scatter (alone or as the first half of All-Reduce): All-Gather on the
   * reversed links, then the schedule reversed in direction AND time, so that the
   * last hop of the reversed All-Gather becomes the first reduction hop. */
  if (has_rev) {
    pass_out_t *o = &po[n_pass];
    o->keep_limit = ~0ull;
    uint64_t T = 0, ne = 0; int complete = 0;
    rc = ag_pass(n_npus, L, col_idx, src, cost, chunks_per_npu, seed, 1u, max_events,
                 n_threads, link_order, matching, o, &T, &ne, &complete, pass_root);
    if (rc != ORC_OK) goto fail;
    complete_all &= complete;
    res->pass_time_ps[n_pass] = T; res->pass_events[n_pass] = ne;
    n_pass++;
    t_off = T;
  }
  if (has_fwd) {
    pass_out_t *o = &po[n_pass];
    o->keep_first = keep_first; o->keep_limit = keep_xfers;
    o->fwd = 1; o->t_off = t_off;
    uint64_t T = 0, ne = 0; int complete = 0;
    rc = ag_pass(n_npus, L, src, col_idx, cost, chunks_per_npu, seed, 0u, max_events,
                 n_threads, link_order, matching, o, &T, &ne, &complete, pass_root);
    if (rc != ORC_OK) goto fail;
    complete_all &= complete;
    res->pass_time_ps[n_pass] = T; res->pass_events[n_pass] = ne;
    n_pass++;
  }
  (void)complete_all;

  /* assemble the records in canonical order */
  uint64_t total_keep = 0;
  /* keep_xfers == 0: digest-only run (large inputs): the reversed pass is digested
   * from its raw records and not materialised */
  const int digest_only = (keep_xfers == 0);
  for (int p = 0; p < n_pass; ++p)
    if (!(digest_only && has_rev && p == 0)) total_keep += po[p].n;
  res->xfers = (orc_xfer_t *)malloc((total_keep ? total_keep : 1) * sizeof(orc_xfer_t));
  if (!res->xfers) { rc = ORC_E_NOMEM; goto fail; }
  uint64_t w = 0;
  int p = 0;
  if (has_rev) {
    /* reversed pass: a transfer that occupied link l during [t', t'+cost) of the
     * reversed All-Gather occupies the ORIGINAL link l (src -> dst) during
     * [T - t' - cost, T - t') of the Reduce-Scatter */
    const uint64_t T = res->pass_time_ps[0];
    const uint64_t first = w;
    if (digest_only) {
      for (uint64_t i = 0; i < po[0].n; ++i) {
        const pass_rec_t *r = &po[0].rec[i];
        res->digest += orc_mix(T - r->t - cost[r->link], r->link, r->chunk);
      }
    } else
    for (uint64_t i = 0; i < po[0].n; ++i) {
      const pass_rec_t *r = &po[0].rec[i];
      orc_xfer_t x;
      x.t_ps = T - r->t - cost[r->link];
      x.src = src[r->link]; x.dst = col_idx[r->link];
      x.chunk = r->chunk; x.link = r->link;
      res->xfers[w++] = x;
    }
    qsort(res->xfers + first, (size_t)(w - first), sizeof(orc_xfer_t), cmp_xfer);
    for (uint64_t i = first; i < w; ++i)
      res->digest += orc_mix(res->xfers[i].t_ps, res->xfers[i].link, res->xfers[i].chunk);
    res->n_xfers += po[0].n_total;
    p = 1;
  }
  if (has_fwd) {
    for (uint64_t i = 0; i < po[p].n; ++i) {
      const pass_rec_t *r = &po[p].rec[i];
      orc_xfer_t x;
      x.t_ps = r->t + t_off;
      x.src = src[r->link]; x.dst = col_idx[r->link];
      x.chunk = r->chunk; x.link = r->link;
      res->xfers[w++] = x;
    }
    res->n_xfers += po[p].n_total;
  }
  res->n_stored = w;
  if (has_fwd) res->digest += po[p].digest;
  for (int q = 0; q < n_pass; ++q) {
    res->collective_time_ps += res->pass_time_ps[q];
    res->n_events += res->pass_events[q];
    res->n_attempts += po[q].n_attempts;
  }
  /* event trace of the last pass */
  {
    pass_out_t *o = &po[n_pass - 1];
    res->n_event_times = o->n_ev;
    res->event_times = o->ev_time; o->ev_time = NULL;
    res->event_matches = o->ev_matches; o->ev_matches = NULL;
  }
  for (int q = 0; q < 2; ++q) pass_out_free(&po[q]);
  free(src); free(cost);
  *result = res;
  return ORC_OK;
fail:
  for (int q = 0; q < 2; ++q) pass_out_free(&po[q]);
  free(src); free(cost);
  orc_result_free(res);
  return rc;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
