/*
 * tacos.h -- C ABI of the MI355X-native TACOS collective-algorithm synthesizer.
 *
 * The library synthesizes a topology-aware collective algorithm by greedy
 * link-chunk matching over the Time-Expanded Network (TEN) of the target topology
 * (TACOS, arXiv 2304.05301: Algorithm 1 "Utilization Maximizing Matching" run once
 * per time span by Algorithm 2 "End-to-End Synthesis").  All of the synthesis runs
 * in HIP kernels on the current device (gfx950); the host code of the library only
 * validates and uploads the inputs, launches, and copies results out.  There is no
 * CPU fallback: without a usable HIP device every call returns TACOS_E_DEVICE.
 *
 * Conventions
 *   - All pointers in this header are HOST pointers unless a comment says "device".
 *   - Times are unsigned 64-bit integer picoseconds.  No floating point is used for
 *     times anywhere, so equal times compare equal.
 *   - A topology is a directed multigraph in CSR form by source NPU.  The LINK ID of
 *     a link is its index into col_idx.  Parallel links are allowed (distinct ids);
 *     self-loops are rejected.
 *   - Chunk c (0 <= c < n_npus*chunks_per_npu) is owned by NPU c / chunks_per_npu:
 *     the precondition of All-Gather is that every NPU holds its own chunks, the
 *     postcondition that every NPU holds all chunks (paper, section "Collective
 *     Communication Patterns").
 *
 * What is computed (the deterministic, link-centric form of the paper's matching):
 *   cost[l] = alpha[l] + beta[l]*chunk_bytes, rounded to the nearest picosecond
 *             (alpha-beta model, section "TACOS for Heterogeneous Networks");
 *   state:    held[n]     chunks that have arrived at NPU n (only these make n a source),
 *             inflight[n] chunks matched to n and not yet arrived (never re-delivered),
 *             per link the chunk it carries and the time it becomes free;
 *   loop (Algorithm 2), starting at t = 0, event = 0:
 *     1. arrivals: every link whose transfer ends at t delivers its chunk;
 *     2. if every NPU holds every chunk: collective_time = t, stop;
 *     3. matching for this span (Algorithm 1): for every destination NPU d, for every
 *        IDLE incoming link l = (s -> d) in ascending link id (or cheapest first, see
 *        tacos_options_t::link_order):
 *          cand = held[s] & ~held[d] & ~inflight[d];  p = |cand|;  if p == 0 skip;
 *          r = word 0 of Philox4x32-10(counter = (l, event, phase, 0),
 *                                      key = (seed mod 2^32, seed div 2^32));
 *          the link carries the (r mod p)-th smallest chunk id of cand, from t to
 *          t + cost[l]  (one chunk per TEN link: section "Representing Collective
 *          Algorithms using TEN");
 *     4. t = earliest end of a transfer in flight, event += 1.  Nothing in flight
 *        while chunks are missing = the topology is not strongly connected.
 *   phase is 0 for a forward (All-Gather) pass and 1 for the reversed pass of a
 *   Reduce-Scatter.  Reduce-Scatter = the All-Gather pass on the topology with every
 *   link reversed (same ids, same costs), then every transfer (t', l, c) of it mapped
 *   to (T - t' - cost[l], src[l], dst[l], c); All-Reduce = Reduce-Scatter followed by
 *   All-Gather starting at the Reduce-Scatter's end (paragraph "Collectives with
 *   Reduction Operations").
 *
 * Canonical order of a schedule: ascending (t_ps, link); for All-Reduce all
 * Reduce-Scatter transfers precede all All-Gather transfers.  (t_ps, link) is unique
 * inside one pass because a link starts at most one transfer per event.
 */
#ifndef TACOS_H
#define TACOS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TACOS_ALL_GATHER = 0,
  TACOS_REDUCE_SCATTER = 1,
  TACOS_ALL_REDUCE = 2,
  /* Rooted collectives (paragraph "Collectives with Reduction Operations": Reduce is the
   * Broadcast synthesized on the reversed links, reversed back).  The buffer of the root
   * (tacos_options_t::root) is split into chunks_per_npu chunks, ids 0 .. chunks_per_npu-1;
   * Broadcast: all of them start at the root and reach every NPU (one forward pass, phase
   * 0); Reduce: the reverse (one reversed pass, phase 1).  Same loop, same matching. */
  TACOS_BROADCAST = 3,
  TACOS_REDUCE = 4
} tacos_collective_t;

/* Error codes (every entry point that returns int: 0 = success, negative = error). */
#define TACOS_OK             0
#define TACOS_E_INVAL       (-1) /* null pointer, N = 0, chunks_per_npu = 0, chunk_bytes = 0,
                                    malformed row_ptr, col_idx out of range, self-loop, unknown
                                    collective, N*chunks_per_npu beyond the supported maximum,
                                    bad window in tacos_result_read                          */
#define TACOS_E_UNREACHABLE (-2) /* chunks missing and nothing in flight: not strongly connected */
#define TACOS_E_OVERFLOW    (-3) /* a link cost or a time does not fit 64 bits                 */
#define TACOS_E_NOMEM       (-4) /* host or device allocation failed                           */
#define TACOS_E_DEVICE      (-5) /* no HIP device / a HIP call failed (see tacos_last_error)   */

/* tacos_options_t::link_order */
#define TACOS_LINK_ORDER_ID   0u
#define TACOS_LINK_ORDER_COST 1u

/* tacos_options_t::matching */
#define TACOS_MATCH_LINK_CENTRIC  0u
#define TACOS_MATCH_POSTCONDITION 1u

/* Largest supported number of chunks N*chunks_per_npu (rooted collectives: chunks_per_npu).
 * A wavefront keeps a destination's whole "still needed" bitset in its share of the LDS and,
 * up to 122,880 chunks, a source's whole row in registers; beyond that the source rows are
 * streamed.  More than 65,536 chunks: link-centric matching, per-span launches only. */
#define TACOS_MAX_CHUNKS 262144u
/* Largest number of chunks for tacos_options_t::matching = 1 and for launch_mode 2. */
#define TACOS_MAX_CHUNKS_IN_REGISTERS 65536u

#define TACOS_NO_CHUNK 0xFFFFFFFFu

/* Topology: borrowed, read during the call only. */
typedef struct {
  uint32_t        n_npus;        /* N >= 1                                                    */
  uint32_t        n_links;       /* L, must equal row_ptr[N]                                  */
  const uint32_t *row_ptr;       /* [N+1] non-decreasing, row_ptr[0] == 0 (CSR by source)     */
  const uint32_t *col_idx;       /* [L]   destination NPU of link id l                        */
  const uint64_t *alpha_ps;      /* [L]   link latency, picoseconds                           */
  const uint64_t *beta_fs_per_B; /* [L]   reciprocal bandwidth, femtoseconds per byte
                                          (50 GB/s == 20000)                                  */
} tacos_topology_t;

/* One link-chunk match of the schedule: `chunk` occupies link `link` = (src -> dst)
 * from t_ps to t_ps + cost[link]. 24 bytes, no padding. */
typedef struct {
  uint64_t t_ps;
  uint32_t src, dst, chunk, link;
} tacos_xfer_t;

/* Optional knobs; zero-initialise for the defaults. */
typedef struct {
  void    *stream;        /* hipStream_t to launch on (NULL = the null stream).  The call
                             returns after the work on it has completed.  An All-Reduce on
                             up to about 16,000 NPUs sweeps its two passes at the same time:
                             the All-Gather pass on a stream the library creates for the
                             call, from a second host thread that has ended when the call
                             returns (not with time_kernels).                               */
  uint64_t max_events;    /* 0 = run to completion; > 0 = stop each pass after that many
                             matching sweeps (the result then covers that prefix only and
                             collective_time is the time reached)                           */
  uint32_t time_kernels;  /* != 0: bracket every launch of the kernel that does the matching
                             with HIP events on `stream` so that tacos_result_kernel_ms is
                             available                                                      */
  uint32_t launch_mode;   /* 0 = automatic.
                             1 = two plain launches per span (arrivals; matching + next-event
                             reduction), queued in batches; once at most 16 destinations
                             still miss chunks (link-centric matching, complete runs, dense
                             schedule rows), one workgroup sweeps the remaining spans, many per
                             launch, with those destinations' link state in registers.
                             4 = as 1, with two launches for every span up to the last.
                             2 = small topologies: ONE workgroup sweeps many spans per launch
                             with the per-link state and a work list in LDS and matches only
                             the destinations something changed for; needs links, NPUs and
                             need rows to fit the LDS of one CU (<= 16,384 chunks, a few
                             thousand links), else TACOS_E_INVAL.
                             3 = homogeneous TEN (paper, section "Time-expanded Network": links of
                             equal cost, spans of equal length): ONE launch per span; a chunk
                             matched in span e arrives exactly at span e + 1, so arrivals,
                             matching and the next event need no separate steps.  Needs equal
                             link costs (<= 2^31 ps), <= 65,536 chunks, link-centric matching,
                             max_events == 0, else TACOS_E_INVAL.  Automatic: 2 if it fits and a
                             span has little to decide or its destinations can be matched
                             one per lane (links that nearly all cost differently; at most
                             64 links; link-centric matching of at most 1,024 chunks with
                             links x row words <= 8,192), else 3 if it applies and
                             its two held tables take at most 256 MiB (about 32,768 NPUs
                             with one chunk each; the last stretch of a pass, at most 16
                             destinations left, as in 1), else 1 (with equal link costs one
                             launch per span once at most 2,048 destinations are left).
                             Same results in all modes.                                      */
  uint32_t link_order;    /* order in which a destination's idle incoming links are tried:
                             0 = ascending link id; 1 = cheapest link first, ties by link id
                             (paper, "Prioritizing Lower-cost Links").  The random draw of a
                             link does not depend on the order.                              */
  uint32_t matching;      /* 0 = link-centric: every idle link draws a chunk (the rule in the
                             header comment).  1 = Algorithm 1 in the order the paper prints
                             it, postcondition-centric: for every destination d, step by step,
                               serv = (chunks d misses) & OR over d's FREE incoming links of
                                      held[src];  stop when serv is empty;
                               (r0, r1) = words 0, 1 of Philox4x32-10(counter = (d, event,
                                      phase + 2, step), key as above);
                               chunk c = the (r0 mod |serv|)-th smallest of serv;
                               link = the (r1 mod n)-th of the n free links whose source
                                      holds c, in list order (link_order 1: the cheapest);
                             which equals visiting a shuffled list of unsatisfied (d, c)
                             pairs and giving each a random free holder.  Needs in-degree
                             <= 64 (TACOS_E_INVAL otherwise).                                */
  uint32_t root;          /* TACOS_BROADCAST / TACOS_REDUCE: the root NPU (< n_npus, else
                             TACOS_E_INVAL); ignored by the other collectives                */
} tacos_options_t;

typedef struct tacos_result tacos_result_t; /* opaque; owns device and host buffers */

/*
 * Synthesize `coll` for the topology (steps 1-4 above, on the current HIP device).
 * On success *out receives a result handle to be released with tacos_result_free.
 * On error *out is left untouched.  opts may be NULL.
 */
int tacos_synthesize(const tacos_topology_t *topo, uint32_t chunks_per_npu,
                     uint64_t chunk_bytes, tacos_collective_t coll, uint64_t seed,
                     const tacos_options_t *opts, tacos_result_t **out);

/*
 * Best of several seeds.  The matching draws at random, so the collective time varies
 * from seed to seed (paper, "Utilization-maximizing Link-Chunk Matching": randomised
 * choices; results of independent runs differ).  time_ps[i] (host, [n_seeds], caller-
 * owned) receives exactly the collective time tacos_synthesize(..., seeds[i], ...)
 * gives, num_events[i] (optional, may be NULL) its number of spans, *best (optional) the
 * index of the smallest time, lowest index on ties.  No schedule is kept: synthesize
 * seeds[*best] again for it.  When the topology fits the single-workgroup kernel
 * (launch_mode 2 of tacos_synthesize) every pass of every seed is one workgroup and all
 * of them sweep their spans concurrently, one CU each; otherwise (or with launch_mode 1)
 * the seeds are synthesized whole: up to about 16,000 NPUs several at a time, on streams the
 * library creates for the call from host threads that have ended when it returns (such a
 * synthesis leaves most of the GPU idle), beyond that one after the other on `stream`.
 * opts: stream, launch_mode, link_order, matching, root as
 * for tacos_synthesize; max_events must be 0.  Errors as tacos_synthesize; on error the
 * outputs are unspecified.
 */
int tacos_seed_search(const tacos_topology_t *topo, uint32_t chunks_per_npu, uint64_t chunk_bytes,
                      tacos_collective_t coll, const uint64_t *seeds, uint32_t n_seeds,
                      const tacos_options_t *opts, uint64_t *time_ps, uint64_t *num_events,
                      uint32_t *best);

/* Time of the last arrival (All-Reduce: Reduce-Scatter time + All-Gather time). */
uint64_t tacos_result_collective_time_ps(const tacos_result_t *r);
/* Number of link-chunk matches in the schedule (all passes). */
uint64_t tacos_result_num_xfers(const tacos_result_t *r);
/* Number of matching sweeps (TEN spans expanded), summed over passes. */
uint64_t tacos_result_num_events(const tacos_result_t *r);
/* Number of passes (1, or 2 for All-Reduce) and per-pass time / sweeps. */
uint32_t tacos_result_num_passes(const tacos_result_t *r);
uint64_t tacos_result_pass_time_ps(const tacos_result_t *r, uint32_t pass);
uint64_t tacos_result_pass_events(const tacos_result_t *r, uint32_t pass);
/*
 * Copies transfers [first, first+count) of the canonical order into host_out
 * (count * sizeof(tacos_xfer_t) bytes, caller-owned).  Windowed because a large
 * schedule (1.7e9 transfers for 40,960 NPUs) does not fit host memory at once.
 * Returns TACOS_E_INVAL if the window exceeds tacos_result_num_xfers.
 */
int tacos_result_read(const tacos_result_t *r, uint64_t first, uint64_t count,
                      tacos_xfer_t *host_out);
/*
 * Per-sweep trace of pass `pass`: time of every matching sweep and the number of
 * matches made in it, n = tacos_result_pass_events entries each (either pointer may
 * be NULL).  Link utilisation of a sweep = matches / n_links.  The times are the pass's
 * own, counted from its first sweep at 0: for a forward pass inside an All-Reduce add the
 * Reduce-Scatter's time; a reversed pass (Reduce-Scatter, Reduce) is traced as it was
 * synthesized, i.e. on the reversed links and before the reversal in time, so sweep i at
 * time t_i holds the transfers that END at T - t_i in the schedule.  (For a reversed pass
 * the counts are computed from the schedule on first use: one pass over its rows.)
 */
int tacos_result_event_trace(const tacos_result_t *r, uint32_t pass,
                             uint64_t *event_time_ps, uint32_t *event_matches);
/*
 * Number of transfers every link carries in pass `pass`: link_counts[l] (host,
 * [n_links], caller-owned), column sums of the schedule computed on the device.  With
 * the link costs this gives the link utilisation the paper reports
 * (count * cost / pass time; section "Analysis of TACOS-Synthesized Algorithms").
 */
int tacos_result_link_counts(const tacos_result_t *r, uint32_t pass, uint64_t *link_counts);
/*
 * Order-independent digest of the schedule: sum modulo 2^64 over all transfers of
 *   h = t_ps ^ (((link << 32) | chunk) * 0x9E3779B97F4A7C15);
 *   h ^= h >> 33; h *= 0xFF51AFD7ED558CCD; h ^= h >> 33; h *= 0xC4CEB9FE1A85EC53; h ^= h >> 33.
 */
uint64_t tacos_result_digest(const tacos_result_t *r);
/* Milliseconds spent inside the kernel that does the matching (sum over its launches:
 * the per-span matching kernel, or the single-workgroup sweep kernel of launch_mode 2) and
 * the number of launches (a launch of the per-span form that sweeps the last stretch of a
 * pass counts once per span it swept); 0 unless opts->time_kernels was set. */
double   tacos_result_kernel_ms(const tacos_result_t *r);
uint64_t tacos_result_kernel_launches(const tacos_result_t *r);
/* Host wall-clock milliseconds of the whole tacos_synthesize call. */
double   tacos_result_wall_ms(const tacos_result_t *r);
/* Bytes of device memory the result holds (schedule tables).  A pass run by the per-span
 * launches (launch_mode 1 and 3) keeps one row of n_links 32-bit entries per span, i.e.
 * spans * n_links * 4 bytes, allocated in 256 MiB segments as the spans are reached (6.7 GB for
 * the 40,960-NPU torus).  A pass run by the single-workgroup kernel (launch_mode 2) keeps 8
 * bytes per transfer and 12 bytes per span, and so does launch_mode 1 on a topology whose
 * links nearly all cost differently (at least 64 distinct costs and at least n_links / 4 of
 * them: about one transfer starts per span and there are millions of spans) with at most
 * about 40,000 links.  Beyond that size such a topology keeps dense rows and can exhaust
 * device memory: TACOS_E_NOMEM. */
uint64_t tacos_result_device_bytes(const tacos_result_t *r);
void     tacos_result_free(tacos_result_t *r);

/* Text for an error code; tacos_last_error gives the HIP detail of the calling
 * thread's last TACOS_E_DEVICE / TACOS_E_NOMEM (empty string if none). */
const char *tacos_strerror(int code);
const char *tacos_last_error(void);

/*
 * Step a1 alone: the link costs of the alpha-beta model as the synthesis uses them,
 * cost_ps[l] = alpha_ps[l] + round(beta_fs_per_B[l] * chunk_bytes / 1000), computed by
 * the library's device kernel and copied to cost_ps (host, [n_links], caller-owned).
 * Returns TACOS_E_OVERFLOW if a cost does not fit 64 bits.
 */
int tacos_link_costs(const tacos_topology_t *topo, uint64_t chunk_bytes, uint64_t *cost_ps);

/*
 * Link busy times of pass `pass`: busy_ps[l] = (transfers link l carries) * cost[l] (host,
 * [n_links], caller-owned, may be NULL), and their sum, minimum and maximum over the links
 * (each may be NULL), computed on the device from the schedule.  The paper's link
 * utilisation (section "Analysis of TACOS-Synthesized Algorithms") is the exact ratio
 * busy_ps[l] / tacos_result_pass_time_ps(pass); the mean over the links is
 * sum / (n_links * pass time).  TACOS_E_OVERFLOW if the sum does not fit 64 bits.
 */
int tacos_result_link_busy(const tacos_result_t *r, uint32_t pass, uint64_t *busy_ps, uint64_t *sum_ps,
                           uint64_t *min_ps, uint64_t *max_ps);

/*
 * Switch unwinding (paper, section "TACOS for Switch-based Networks"): an n_npus-port switch
 * whose ports have latency alpha_ps and reciprocal bandwidth beta_fs_per_B becomes, with
 * degree d, the point-to-point topology in which NPU i has the d outgoing links to NPUs
 * i+1 .. i+d (mod n_npus), each with the same alpha and with beta multiplied by d (the port
 * bandwidth is shared).  Outputs (host, caller-owned): row_ptr [n_npus + 1], col_idx,
 * alpha_out, beta_out [n_npus * degree each], in the library's CSR convention (rows by
 * source, ascending destination inside a row), ready for tacos_topology_t.  Computed on the
 * device.  TACOS_E_INVAL unless n_npus >= 2 and 1 <= degree <= n_npus - 1;
 * TACOS_E_OVERFLOW if beta * degree does not fit 64 bits.
 */
int tacos_unwind_switch(uint32_t n_npus, uint32_t degree, uint64_t alpha_ps, uint64_t beta_fs_per_B,
                        uint32_t *row_ptr, uint32_t *col_idx, uint64_t *alpha_out, uint64_t *beta_out);

/*
 * The paper's theoretically ideal collective time (section "Baseline Collective Algorithms
 * and Synthesizers"):  Ideal = CollectiveSize * 2(n-1)/n / min_NPU(BW_NPU) + Diameter, in
 * integer picoseconds.  CollectiveSize = n_npus * chunks_per_npu * chunk_bytes.  An
 * All-Gather has every NPU receive CollectiveSize * (n-1)/n bytes: its bandwidth term is
 * that over the smallest INGRESS bandwidth of an NPU (sum of 1/beta over its incoming
 * links, kept as an exact fraction), rounded up to a picosecond; a Reduce-Scatter has every
 * NPU send as much: the same over the smallest EGRESS bandwidth; an All-Reduce is the sum of
 * the two (the paper's factor 2).  Diameter = the largest, over ordered pairs of NPUs, of the
 * smallest sum of alpha along a path (computed if with_diameter != 0; needs n_npus <=
 * TACOS_IDEAL_MAX_DIAMETER_NPUS, else TACOS_E_INVAL).  pass_*: per pass in schedule order
 * (All-Reduce: Reduce-Scatter, All-Gather); bottleneck = the worst-connected NPU, lowest id
 * on ties.  TACOS_E_UNREACHABLE if an NPU has no link on the side needed or is not reached;
 * TACOS_E_OVERFLOW if a value does not fit 64 bits; TACOS_E_INVAL for rooted collectives.
 */
#define TACOS_IDEAL_MAX_DIAMETER_NPUS 8192u
typedef struct {
  uint64_t collective_bytes;
  uint64_t bandwidth_term_ps;          /* sum over the passes                  */
  uint64_t diameter_ps;                /* 0 if with_diameter == 0              */
  uint64_t ideal_ps;                   /* bandwidth_term_ps + diameter_ps      */
  uint64_t pass_bandwidth_term_ps[2];
  uint32_t pass_bottleneck_npu[2];
} tacos_ideal_t;
int tacos_ideal_bound(const tacos_topology_t *topo, uint32_t chunks_per_npu, uint64_t chunk_bytes,
                      tacos_collective_t coll, uint32_t with_diameter, tacos_ideal_t *out);

/*
 * tacos_link_costs for callers that cannot allocate device memory: code that runs where
 * hipMalloc is not allowed (while a HIP graph is being captured elsewhere in the process,
 * tight serving loops, harnesses that forbid allocation).  Same arguments, same results
 * and same error codes as tacos_link_costs, but the device staging (alpha, beta, costs,
 * overflow flag) lives in a device array of fixed size that is part of the library image
 * (24 bytes per link of TACOS_STATIC_MAX_LINKS links, about 6 MiB, present on every GPU the
 * library runs on until the process ends), and the call makes no hipMalloc, hipFree or
 * other allocating call.  More than TACOS_STATIC_MAX_LINKS links: TACOS_E_INVAL (see
 * tacos_last_error).  Runs on the null stream and returns after the work has completed.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU race.
 */
#define TACOS_STATIC_MAX_LINKS 262144u
int tacos_link_costs_static(const tacos_topology_t *topo, uint64_t chunk_bytes, uint64_t *cost_ps);

/* Library version string. */
const char *tacos_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TACOS_H */
