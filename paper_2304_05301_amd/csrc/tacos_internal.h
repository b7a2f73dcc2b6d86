// Internal interface between the host side of the library (tacos_api.cpp) and its
// HIP kernels (tacos_kernels.hip).  Not installed; the public ABI is include/tacos.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tacos {

constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint64_t kInf = 0xFFFFFFFFFFFFFFFFull;

// Status words written by the kernels into Ctl::status (0 = running / fine).
constexpr uint32_t kStUnreachable = 1;
constexpr uint32_t kStOverflow = 2;
constexpr uint32_t kStInternal = 3;

// Device-resident control block of one pass.  next_t is double-buffered by event
// parity: the matching kernel of event e min-reduces the end times of all transfers
// in flight into next_t[(e+1)&1]; the arrival kernel of event e+1 reads it as "now".
// The pass has ended when nothing is in flight after a span's matching: every NPU holds
// every chunk if no destination of that span still needed one (need_flag), else the
// topology is not strongly connected.
struct Ctl {
  unsigned long long next_t[2];
  unsigned long long remaining;  // single-workgroup kernel: unsatisfied postconditions (NPU, chunk)
  unsigned long long T;          // time of the last arrival, valid once done
  unsigned long long now;        // time of the span the arrival kernel processed last
  uint32_t done;
  uint32_t status;
  uint32_t n_events;             // matching sweeps run, valid once done
  uint32_t n_rec;                // single-workgroup kernel: schedule records written so far
  // Set by the matching of span e if a destination with an idle incoming link still misses a
  // chunk, read by the launch that follows, cleared one span ahead.  Two launches per span:
  // index e & 1 (set by match_kernel, read and cleared by arrive_kernel); homogeneous-TEN path:
  // index e % 3, with match_flag[e % 3] set if a link was matched in span e.
  uint32_t need_flag[4];
  uint32_t match_flag[4];
};

// HBM layout of the per-NPU held bitsets ("precondition" rows).
//
// A row has NP "pieces" of 1 KiB.  In piece i lane j of a wavefront owns the 16 bytes
// at byte offset i*1024 + j*16, so one global_load_dwordx4 per piece per lane reads the
// row fully coalesced.  Chunk ids are laid out LANE-MAJOR: lane j owns the 2*NP
// consecutive 64-bit words [j*2NP, (j+1)*2NP) of the logical bitset, word 2i+s of them
// sitting in half s of its 16 bytes of piece i.  So ascending chunk id = ascending
// (lane, piece, half, bit), and one wave prefix sum over per-lane popcounts locates
// the k-th candidate.  Bits of chunk ids >= C are stored as 1 ("held") in every row so
// that they never become candidates.
constexpr uint32_t kNoRoot = 0xFFFFFFFFu;

struct PassDev {
  uint32_t N, L, cpn, NP;
  uint32_t C;                      // chunks: N*cpn, or cpn for a rooted collective
  uint32_t root;                   // kNoRoot: NPU i owns chunks [i*cpn, (i+1)*cpn); else the root owns all C
  uint32_t phase;
  uint32_t seed_lo, seed_hi;
  uint32_t row_words;              // 64-bit words per row = NP*128
  uint32_t reversed;               // 1: schedule rows are keyed by ARRIVAL event
  uint32_t max_deg;                // largest in-degree of the pass orientation
  unsigned long long *held;        // [N][row_words]
  const uint32_t *in_ptr;          // [N+1]
  const uint32_t *in_link;         // [L] incoming links of each NPU, ascending link id
  const uint32_t *in_src;          // [L] their source NPUs (pass orientation)
  const unsigned short *in_src16;  // [L] the same as 16-bit values in LDS (single-workgroup kernel, when the
                                   //     in-list records themselves do not fit there), else null
  uint32_t in_rec_in_lds;          // single-workgroup kernel: in_rec points into LDS
  uint4 *in_rec;                   // [L] the in-lists as one record per entry: (link, source, cost lo, cost hi),
                                   //     written by the set-up kernel from in_link / in_src / cost
  const uint32_t *pos_dst;         // [L] destination NPU of in-list position j (pass orientation)
  uint32_t n_slots;                // processing slots in use (N, less the complete destinations the host dropped)
  uint32_t *dest_done;             // [N] set to 1 by the matching once the NPU holds every chunk; may be null
  const uint4 *slot_rec;           // [N] per processing slot: (destination d, in_ptr[d], in_ptr[d+1], 0); the
                                   //     destinations in processing order are a permutation of the NPUs
  const unsigned long long *cost;  // [L]
  uint32_t *carry;                 // [L] chunk in flight or kNone, indexed by IN-LIST POSITION j (so that a
                                   //     destination's links are contiguous and need no indirection)
  unsigned long long *free_at;     // [L] busy-until time, same indexing
  uint32_t *rnd;                   // [L] by in-list position: word 0 of Philox(link, current span, phase, 0),
                                   //     written by arrive_kernel for the link-centric match_kernel; else null
  // Per-span launches: the matching kernels min-reduce the end times of the transfers in flight
  // (a workgroup's four wavefronts through LDS, then one atomic, skipped if the word is already as
  // small) into kNextSlots words per span parity ([2][kNextSlots]); the arrivals kernel of the next
  // span takes the minimum of the words, publishes it as Ctl::next_t and clears the other parity.
  // The workgroups of a SHORT launch all finish together, every one of them then sees the word
  // still at infinity, and thousands of atomics on one address take tens of microseconds: such
  // launches spread over all the words (next_mask = kNextSlots - 1); long launches, whose first
  // finisher's value stops all the others, use the first word only (next_mask = 0; spreading
  // costs them a few per cent).  Null in the other modes.
  unsigned long long *next_slots;
  uint32_t next_mask;
  Ctl *ctl;
};
constexpr uint32_t kNextSlots = 64;

// a1: cost = alpha + round(beta*bytes/1000); *overflow set non-zero if any cost >= 2^64-1
void launch_link_cost(const unsigned long long *alpha, const unsigned long long *beta,
                      unsigned long long chunk_bytes, uint32_t L, unsigned long long *cost,
                      uint32_t *overflow, hipStream_t s);
// Homogeneous TEN (every link of the topology has the same cost, so all spans have the same
// length and a chunk matched in span e arrives exactly at span e + 1; paper, section
// "Time-expanded Network"): arrivals, matching and the next event collapse into ONE launch
// per span.  The held table is double-buffered: span e reads held[e & 1], which is complete
// as of that span, and every destination's wavefront brings its own row of the other table
// (one span behind) up to date for span e + 1 by setting the bits of the chunks that arrived
// now (matched in span e - 1, prev[(e - 1) & 1]) and of the ones it matches now.
struct UniformDev {
  unsigned long long *held[2];  // [N][row_words] each
  uint32_t *prev[2];            // [L] by in-list position: chunk matched in span e (prev[e & 1]) or kNone
  uint32_t *rnd[2];             // [L] by in-list position: word 0 of Philox(link, e, phase, 0) for span e
                                //     (rnd[e & 1]); link-centric matching only, else null
  unsigned long long cost;      // the common link cost: span e is at time e * cost
};
// prev = kNone, the random words of span 0 (p.held / p.carry / p.free_at / p.rnd are not used
// by this path; the control block and in_rec come from launch_init_pass)
void launch_uniform_init(const PassDev &p, const UniformDev &u, uint32_t mode, hipStream_t s);
// a3-a8 of span `event` in one launch.  row: schedule row of the span (forward pass), row_next:
// schedule row of span event + 1 (reversed pass: rows are keyed by arrival); the other is null.
// The pass has ended when the launch of span e finds that span e - 1 needed nothing.
// The state launch_arrive / launch_tail_sweep start span `event` (>= 1) from, out of the state the
// homogeneous-TEN form has after span event - 1: the chunks matched there are in flight until
// event * cost (carry, free_at, the next-event words, which the caller has set to kInf), the time
// and need flag of span event - 1 go to the places arrive_kernel reads them from.  The held table
// to go on with is u.held[(event - 1) & 1].
void launch_uniform_handover(const PassDev &p, const UniformDev &u, uint32_t event, hipStream_t s);
// The opposite direction, before the arrivals of span `event` (>= 1) on a topology of equal link
// costs: u.held[event & 1] is the table the launches with link state worked on (it receives the
// arrivals of the span), u.held[(event + 1) & 1] becomes a copy of it as it is before; the flags of
// span event - 1 are set here and all others cleared.  sched_row: the span's
// schedule row in a reversed pass, else null.
void launch_links_to_uniform(const PassDev &p, const UniformDev &u, uint32_t event, uint32_t *sched_row,
                             hipStream_t s);
void launch_match_uniform(const PassDev &p, const UniformDev &u, uint32_t event, uint32_t *row, uint32_t *row_next,
                          unsigned long long *event_time_slot, uint32_t mode, hipStream_t s);

// a1 for callers that may not allocate: the same kernel with its device staging in a
// file-scope device array (per GPU) instead of allocated buffers.  Host pointers in and out;
// L in [1, kStaticMaxLinks]; *h_overflow != 0 if a cost does not fit.  Calls no hipMalloc or
// hipFree; returns after the work on `s` has completed.  Calls that overlap on one GPU race.
constexpr uint32_t kStaticMaxLinks = 262144;
hipError_t link_cost_static(const unsigned long long *h_alpha, const unsigned long long *h_beta,
                            unsigned long long chunk_bytes, uint32_t L, unsigned long long *h_cost,
                            uint32_t *h_overflow, hipStream_t s);
// a2: precondition rows, idle links, control block
void launch_init_pass(const PassDev &p, hipStream_t s);
// a3 + a8 (consume): arrivals at the event's time; writes event_time_slot and, for a
// reversed pass, the arrivals into the schedule row of the event (rows are pre-filled with kNone)
// Compact schedule (recs != null, sched_row == null): a reversed pass appends its arrivals as
// (link, chunk) records at Ctl::n_rec; first_slot, if not null, receives the index of the
// span's first record.
void launch_arrive(const PassDev &p, uint32_t event, unsigned long long *event_time_slot,
                   uint32_t *sched_row, uint2 *recs, uint32_t *first_slot, hipStream_t s);
// a4-a8 (produce): termination test, matching for all destinations, min-reduction of
// the next event time; a forward pass writes its matches into the schedule row of the event
// (pre-filled with kNone).  Only the first p.n_slots processing slots are launched.
// mode 0: link-centric; 1: postcondition-centric with a random holder link; 2: postcondition-
// centric with the first holder of the incoming list (in-degree <= 64 for modes 1, 2)
void launch_match(const PassDev &p, uint32_t event, uint32_t *sched_row, uint32_t mode, hipStream_t s);
// Per-span launches with at most kTailSlots destinations left in the processing order (link-centric
// matching, dense schedule rows, in-degrees up to 64, rows of at most 8 pieces): one workgroup
// sweeps spans first_event .. first_event + n_spans - 1 (or up to the end of the pass) in ONE
// launch, arrivals and matching; rows0 / times0 are the schedule row and time slot of span
// first_event, the rows of the following spans row_stride words apart (same segment).  Leaves
// the state as launch_arrive + launch_match of those spans would.
constexpr uint32_t kTailSlots = 16;
hipError_t launch_tail_sweep(const PassDev &p, uint32_t first_event, uint32_t n_spans, uint32_t *rows0,
                             unsigned long long row_stride, unsigned long long *times0, hipStream_t s);
// The same with a compact schedule: a forward pass appends its matches as (link, chunk) records
// at Ctl::n_rec; first_next, if not null (reversed pass), receives the index at which the records
// of the next span (its arrivals) start.  Rows of at most 8 pieces.
void launch_match_compact(const PassDev &p, uint32_t event, uint2 *recs, uint32_t *first_next, uint32_t mode,
                          hipStream_t s);
// largest number of links whose compact schedule the epilogue can order (one LDS word per link)
uint32_t compact_schedule_max_links();
// a3-a8 fused for small topologies: ONE workgroup sweeps spans [first_event,
// first_event+n_events) with the per-link state in LDS (arrivals, termination test,
// matching of the destinations something changed for, next-event min-reduction) and
// returns early when the pass ends.  mode: as launch_match.  stop_event: the span at which only the arrivals are
// applied (prefix runs), or 0xFFFFFFFF.  The schedule is written as compact records: recs
// (the whole pass's (link, chunk) pairs, appended in span order; within a span in no
// particular order) and, per span from first_event on, span_first (index of the span's first
// record) and event_times.  A forward pass records matches, a reversed pass arrivals.
// out_ptr/out_dst: out-neighbour lists of the pass orientation.  sparse: about one transfer per
// span is expected (links that nearly all cost differently): the destinations of a span are then
// matched one per wavefront also where the shape would allow one per lane.
hipError_t launch_small_sweep(const PassDev &p, const uint32_t *out_ptr, const uint32_t *out_dst,
                              uint32_t first_event, uint32_t n_events, uint32_t stop_event,
                              uint2 *recs, uint32_t *span_first, unsigned long long *event_times, uint32_t mode,
                              bool sparse, hipStream_t s);
// Whether that kernel would match this shape's destinations one per LANE (link-centric matching,
// at most 1,024 chunks, held table and in-list records in LDS): then a span in which every
// link is matched costs it little more than a span with one transfer.
bool small_sweep_by_lane(uint32_t N, uint32_t L, uint32_t NP, uint32_t C, uint32_t mode);
// The same sweep for n_jobs independent passes of one shape at once, one workgroup each
// (jobs: device array); collective times only, no schedule rows.  p0: any of the jobs'
// PassDev (shape).  Every unfinished job advances by n_events spans from first_event.  sparse: as
// launch_small_sweep.
struct SmallJob {
  PassDev p;
  const uint32_t *out_ptr;
  const uint32_t *out_dst;
};
hipError_t launch_small_sweep_batch(const SmallJob *jobs, uint32_t n_jobs, const PassDev &p0,
                                    uint32_t first_event, uint32_t n_events, uint32_t mode, bool sparse,
                                    hipStream_t s);
// LDS the small-topology kernel needs, (size_t)-1 if the shape is not supported
size_t small_sweep_lds_bytes(uint32_t N, uint32_t L, uint32_t NP);
// epilogue: per-row match counts and the schedule digest of a block of rows; `digest` points at
// kDigestSlots partial sums, one every 16 words (128 bytes), which the caller adds up
constexpr uint32_t kDigestSlots = 256;
void launch_row_stats(const uint32_t *rows, uint32_t n_rows, uint32_t L,
                      const unsigned long long *row_time, unsigned long long t_base,
                      uint32_t reversed, uint32_t *row_count, unsigned long long *digest,
                      hipStream_t s);

// ---- compact schedules (single-workgroup kernel): n_rec records (link, chunk), the records of
// span e are [span_first[e], span_first[e + 1]), span_first has n_spans + 1 entries.
// epilogue: orders the records of every span by link id (workgroups of 256 threads, L * 4 bytes
// of LDS) and adds the schedule digest of all records into the kDigestSlots partial sums
void launch_compact_epilogue(uint2 *recs, const uint32_t *span_first, uint32_t n_spans, uint32_t L,
                             const unsigned long long *span_time, unsigned long long t_base, uint32_t reversed,
                             unsigned long long *digest, hipStream_t s);
// counts[l] += records on link l
void launch_compact_link_counts(const uint2 *recs, uint32_t n_rec, unsigned long long *counts, hipStream_t s);
// reversed pass: counts[k] += records that STARTED in span k (arrival span's time minus the link's cost)
void launch_compact_start_span_counts(const uint2 *recs, const uint32_t *span_first, uint32_t n_spans,
                                      const unsigned long long *span_time, const unsigned long long *cost,
                                      uint32_t *counts, hipStream_t s);

// reporting, reversed pass (rows keyed by arrival span): counts[k] += number of transfers of
// the block of rows [first_row, first_row + n_rows) that STARTED in span k, i.e. whose arrival
// time minus the link's cost is row_time[k]; row_time: times of all spans of the pass, ascending
void launch_start_span_counts(const uint32_t *rows, uint32_t first_row, uint32_t n_rows, uint32_t L,
                              const unsigned long long *row_time, const unsigned long long *cost,
                              uint32_t *counts, hipStream_t s);

// reporting: counts[l] += number of rows of the block in which link l carries a chunk
void launch_link_counts(const uint32_t *rows, uint32_t n_rows, uint32_t L, unsigned long long *counts,
                        hipStream_t s);

// ---- reporting and input pre-processing (tacos_report.hip)
// flags the kernels below OR into *flags
constexpr uint32_t kRepOverflow = 1;  // a value does not fit 64 bits
constexpr uint32_t kRepNoLink = 2;    // an NPU without a link on the side asked for / not reached
// switch unwinding: CSR of the degree-d unwinding of an n-NPU switch (device pointers)
void launch_unwind_switch(uint32_t n, uint32_t d, unsigned long long alpha, unsigned long long beta_d,
                          uint32_t *row_ptr, uint32_t *col_idx, unsigned long long *alpha_out,
                          unsigned long long *beta_out, hipStream_t s);
// bandwidth term of the Ideal on one side (ptr/beta: every NPU's incoming or outgoing links):
// out[0] = ceil(bytes / bandwidth of the worst-connected NPU) in ps, out[1] = that NPU;
// P, Q: [N] scratch (the NPU bandwidths as fractions)
void launch_bandwidth_term(uint32_t N, const uint32_t *ptr, const unsigned long long *beta, unsigned long long bytes,
                           unsigned long long *P, unsigned long long *Q, unsigned long long *out, uint32_t *flags,
                           hipStream_t s);
// latency diameter: *diameter = max over ordered pairs of the smallest alpha sum of a path
// (N * 8 + 16 bytes of LDS per workgroup: N <= 8192)
hipError_t launch_latency_diameter(uint32_t N, uint32_t L, const uint32_t *src, const uint32_t *dst,
                                   const unsigned long long *alpha, unsigned long long *diameter, uint32_t *flags,
                                   hipStream_t s);
// busy[l] = counts[l] * cost[l] (busy may be null); out[0..2] = sum, min, max over the links
void launch_link_busy(uint32_t L, const unsigned long long *counts, const unsigned long long *cost,
                      unsigned long long *busy, unsigned long long *out, uint32_t *flags, hipStream_t s);

}  // namespace tacos
