// Host side of the C ABI declared in include/tacos.h: input validation, upload, the
// launch loop over TEN spans, and windowed read-back of the schedule.  Everything the
// method computes (link costs, arrivals, matching, next-event reduction, schedule
// statistics) runs in the kernels of tacos_kernels.hip; this file holds no CPU
// implementation of any of it.

#include "../../include/tacos.h"
#include "tacos_internal.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <system_error>
#include <thread>
#include <utility>
#include <vector>

using tacos::Ctl;
using tacos::PassDev;

namespace {

thread_local std::string g_last_error;

struct HipFail {
  int code;
};

void hip_check(hipError_t e, const char *what, const char *file, int line)
{
  if (e == hipSuccess) return;
  char buf[512];
  std::snprintf(buf, sizeof buf, "%s failed: %s (%s:%d)", what, hipGetErrorString(e), file, line);
  g_last_error = buf;
  (void)hipGetLastError();
  throw HipFail{e == hipErrorOutOfMemory ? TACOS_E_NOMEM : TACOS_E_DEVICE};
}
#define HIP_TRY(expr) hip_check((expr), #expr, __FILE__, __LINE__)

// Owning device allocation.
struct DevBuf {
  void *p = nullptr;
  size_t bytes = 0;
  DevBuf() = default;
  explicit DevBuf(size_t n) { alloc(n); }
  DevBuf(const DevBuf &) = delete;
  DevBuf &operator=(const DevBuf &) = delete;
  DevBuf(DevBuf &&o) noexcept : p(o.p), bytes(o.bytes) { o.p = nullptr; o.bytes = 0; }
  DevBuf &operator=(DevBuf &&o) noexcept
  {
    if (this != &o) { reset(); p = o.p; bytes = o.bytes; o.p = nullptr; o.bytes = 0; }
    return *this;
  }
  ~DevBuf() { reset(); }
  void alloc(size_t n)
  {
    reset();
    HIP_TRY(hipMalloc(&p, n ? n : 1));
    bytes = n;
  }
  // for memory the caller can do without: false (and no pending HIP error) if there is none
  bool try_alloc(size_t n)
  {
    reset();
    if (hipMalloc(&p, n ? n : 1) != hipSuccess) {
      (void)hipGetLastError();
      p = nullptr;
      return false;
    }
    bytes = n;
    return true;
  }
  void reset()
  {
    if (p) (void)hipFree(p);
    p = nullptr;
    bytes = 0;
  }
  template <class T> T *as() const { return static_cast<T *>(p); }
};

// A stream of the library's own (default priority, not synchronizing with the null stream).
struct OwnedStream {
  hipStream_t s = nullptr;
  OwnedStream() { HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking)); }
  OwnedStream(const OwnedStream &) = delete;
  OwnedStream &operator=(const OwnedStream &) = delete;
  ~OwnedStream() { if (s) (void)hipStreamDestroy(s); }
};

// A host thread that is joined when it goes out of scope, also on an exception.
struct JoiningThread {
  std::thread t;
  template <class F> explicit JoiningThread(F &&f) : t(std::forward<F>(f)) {}
  JoiningThread(const JoiningThread &) = delete;
  JoiningThread &operator=(const JoiningThread &) = delete;
  ~JoiningThread() { if (t.joinable()) t.join(); }
};

struct PinnedCtl {
  Ctl *p = nullptr;
  PinnedCtl() { HIP_TRY(hipHostMalloc(reinterpret_cast<void **>(&p), sizeof(Ctl), hipHostMallocDefault)); }
  ~PinnedCtl() { if (p) (void)hipHostFree(p); }
};

struct PinnedBuf {
  void *p = nullptr;
  explicit PinnedBuf(size_t n) { HIP_TRY(hipHostMalloc(&p, n ? n : 1, hipHostMallocDefault)); }
  PinnedBuf(const PinnedBuf &) = delete;
  PinnedBuf &operator=(const PinnedBuf &) = delete;
  ~PinnedBuf() { if (p) (void)hipHostFree(p); }
};

// Seed search: passes per launch (one workgroup each), device bytes of their state, and
// spans every unfinished pass advances per launch.
constexpr size_t kSearchJobs = 2048;
constexpr size_t kSearchBytes = 16ull << 30;
constexpr uint64_t kSearchSpansPerLaunch = 1u << 16;

template <class T> void upload(DevBuf &b, const T *src, size_t n, hipStream_t s)
{
  b.alloc(n * sizeof(T));
  if (n) HIP_TRY(hipMemcpyAsync(b.p, src, n * sizeof(T), hipMemcpyHostToDevice, s));
}

// Largest size of the two held tables of the homogeneous-TEN path for which the automatic
// launch mode chooses it.
constexpr size_t kUniformAutoBytes = 256ull << 20;
// Largest held table of a pass for which independent passes (the halves of an All-Reduce, the
// seeds of a search) sweep at the same time on streams of their own.
constexpr size_t kConcurrentPassBytes = 48ull << 20;

// Schedule rows are stored in segments so that the number of spans need not be known
// up front: segment k holds rows [k*rows_per_seg, (k+1)*rows_per_seg) and their times.
constexpr size_t kSegmentBytes = 256ull << 20;

struct Segment {
  DevBuf rows;      // uint32 [rows_per_seg][L], chunk carried or TACOS_NO_CHUNK
  DevBuf row_time;  // uint64 [rows_per_seg], event time of the row
};

struct Pass {
  bool reversed = false;
  uint32_t L = 0;
  uint32_t rows_per_seg = 1;
  std::vector<Segment> segs;
  // Compact schedule (single-workgroup kernel): (link, chunk) records in span order instead of
  // one row of L entries per span; while the pass runs, a segment's `rows` holds one u32 per
  // span, the index of the span's first record.  After the pass: first / d_first
  // [n_rows + 1] and d_time [n_rows] are the whole pass's, the segments are released.
  bool compact = false;
  DevBuf recs, d_first, d_time;
  uint64_t n_rec = 0;
  std::vector<uint32_t> first;
  uint32_t row_stride() const { return compact ? 1u : L; }
  uint64_t T = 0;         // pass time
  uint64_t n_events = 0;  // matching sweeps
  uint64_t n_rows = 0;    // schedule rows that may hold records
  uint64_t t_off = 0;     // start of the pass inside the collective
  uint64_t n_xfers = 0;
  bool prefill = false;   // new segments are filled with TACOS_NO_CHUNK
  std::vector<uint64_t> row_time;   // [n_rows] by event index
  std::vector<uint32_t> row_count;  // [n_rows] by event index
  std::vector<uint64_t> canon_base; // [n_rows+1] prefix of counts in canonical row order
  // reversed pass: matches made in every span (row_count holds arrivals); filled on first use
  mutable std::vector<uint32_t> start_count;
  // canonical row k is event k of a forward pass, event n_rows-1-k of a reversed one
  uint64_t event_of(uint64_t k) const { return reversed ? n_rows - 1 - k : k; }
  uint64_t time_of_event(uint64_t e) const { return reversed ? T - row_time[e] : row_time[e] + t_off; }
};

}  // namespace

struct tacos_result {
  int device = 0;
  uint32_t N = 0, L = 0;
  std::vector<uint32_t> link_src, link_dst;  // original orientation
  std::vector<Pass> passes;
  uint64_t collective_time = 0, n_xfers = 0, n_events = 0, digest = 0;
  double kernel_ms = 0.0, wall_ms = 0.0;
  uint64_t kernel_launches = 0;
  uint64_t device_bytes = 0;
  DevBuf d_cost;  // [L] link costs, kept for the per-span trace of a reversed pass
};

namespace {

struct EventPool {
  std::vector<hipEvent_t> ev;
  ~EventPool() { for (auto e : ev) (void)hipEventDestroy(e); }
  void ensure(size_t n)
  {
    while (ev.size() < n) {
      hipEvent_t e;
      HIP_TRY(hipEventCreate(&e));
      ev.push_back(e);
    }
  }
};

// Destination processing order: breadth-first clusters of about kClusterSize NPUs.
// Purely a locality heuristic for the L2 caches; it never changes the result.
constexpr uint32_t kClusterSize = 512;

std::vector<uint32_t> cluster_order(uint32_t N, uint32_t L, const std::vector<uint32_t> &in_ptr,
                                    const std::vector<uint32_t> &in_src, const std::vector<uint32_t> &psrc,
                                    const std::vector<uint32_t> &pdst, std::vector<uint32_t> &out_ptr,
                                    std::vector<uint32_t> &out_dst)
{
  std::vector<uint32_t> order;
  order.reserve(N);
  // out-neighbour lists (CSR by psrc) next to the in-neighbour lists we already have
  out_ptr.assign(N + 1, 0);
  out_dst.assign(L, 0);
  for (uint32_t l = 0; l < L; ++l) out_ptr[psrc[l] + 1]++;
  for (uint32_t i = 0; i < N; ++i) out_ptr[i + 1] += out_ptr[i];
  {
    std::vector<uint32_t> fill(out_ptr.begin(), out_ptr.end() - 1);
    for (uint32_t l = 0; l < L; ++l) out_dst[fill[psrc[l]]++] = pdst[l];
  }
  std::vector<uint8_t> state(N, 0);  // 0 = free, 1 = queued in the current cluster, 2 = placed
  std::vector<uint32_t> queue;
  for (uint32_t seed = 0; seed < N; ++seed) {
    if (state[seed] != 0) continue;
    queue.clear();
    queue.push_back(seed);
    state[seed] = 1;
    size_t head = 0;
    uint32_t placed = 0;
    while (head < queue.size() && placed < kClusterSize) {
      const uint32_t u = queue[head++];
      state[u] = 2;
      order.push_back(u);
      placed++;
      for (uint32_t j = in_ptr[u]; j < in_ptr[u + 1]; ++j) {
        const uint32_t v = in_src[j];
        if (state[v] == 0) { state[v] = 1; queue.push_back(v); }
      }
      for (uint32_t j = out_ptr[u]; j < out_ptr[u + 1]; ++j) {
        const uint32_t v = out_dst[j];
        if (state[v] == 0) { state[v] = 1; queue.push_back(v); }
      }
    }
    for (; head < queue.size(); ++head) state[queue[head]] = 0;  // not placed: free again
  }
  return order;
}

// The graph of one pass orientation on the device: in-lists (ascending link id, or
// cheapest first), out-neighbour lists, link destinations, processing order.
struct PassGraph {
  uint32_t N = 0, L = 0, max_deg = 0;
  DevBuf in_ptr, in_link, in_src, in_rec, pos_dst, slot_rec, out_ptr, out_dst;
  std::vector<uint32_t> h_order, h_in_ptr;  // host copies, for dropping complete destinations
};

void build_pass_graph(uint32_t N, uint32_t L, const std::vector<uint32_t> &psrc, const std::vector<uint32_t> &pdst,
                      const std::vector<uint64_t> *order_cost, hipStream_t stream, PassGraph &g)
{
  g.N = N;
  g.L = L;
  // incoming links of every NPU in ascending link id (stable counting sort by destination)
  std::vector<uint32_t> in_ptr(N + 1, 0), in_link(L), in_src(L);
  for (uint32_t l = 0; l < L; ++l) in_ptr[pdst[l] + 1]++;
  for (uint32_t d = 0; d < N; ++d) in_ptr[d + 1] += in_ptr[d];
  {
    std::vector<uint32_t> fill(in_ptr.begin(), in_ptr.end() - 1);
    for (uint32_t l = 0; l < L; ++l) {
      const uint32_t j = fill[pdst[l]]++;
      in_link[j] = l;
      in_src[j] = psrc[l];
    }
  }
  if (order_cost) {
    // cheapest incoming link first, ties by link id ("Prioritizing Lower-cost Links");
    // the costs are the ones the device computed
    std::vector<uint32_t> tmp;
    for (uint32_t d = 0; d < N; ++d) {
      tmp.assign(in_link.begin() + in_ptr[d], in_link.begin() + in_ptr[d + 1]);
      std::stable_sort(tmp.begin(), tmp.end(),
                       [&](uint32_t a, uint32_t b) { return (*order_cost)[a] < (*order_cost)[b]; });
      for (size_t k = 0; k < tmp.size(); ++k) {
        in_link[in_ptr[d] + k] = tmp[k];
        in_src[in_ptr[d] + k] = psrc[tmp[k]];
      }
    }
  }

  // Processing order of the destinations: clusters grown breadth-first over the
  // (undirected) topology, so that NPUs that read each other's rows are matched close
  // together in time and on the same XCD.  Any permutation gives the same schedule.
  std::vector<uint32_t> out_ptr, out_dst;
  std::vector<uint32_t> order = cluster_order(N, L, in_ptr, in_src, psrc, pdst, out_ptr, out_dst);

  std::vector<uint32_t> slot_rec((size_t)N * 4), pos_dst(L);
  for (uint32_t k = 0; k < N; ++k) {
    const uint32_t d = order[k];
    slot_rec[4 * (size_t)k] = d; slot_rec[4 * (size_t)k + 1] = in_ptr[d]; slot_rec[4 * (size_t)k + 2] = in_ptr[d + 1];
  }
  for (uint32_t j = 0; j < L; ++j) pos_dst[j] = pdst[in_link[j]];
  g.h_order = order;
  g.h_in_ptr = in_ptr;
  for (uint32_t d = 0; d < N; ++d) g.max_deg = std::max(g.max_deg, in_ptr[d + 1] - in_ptr[d]);
  upload(g.slot_rec, slot_rec.data(), slot_rec.size(), stream);
  upload(g.pos_dst, pos_dst.data(), pos_dst.size(), stream);
  upload(g.in_ptr, in_ptr.data(), in_ptr.size(), stream);
  upload(g.in_link, in_link.data(), in_link.size(), stream);
  upload(g.in_src, in_src.data(), in_src.size(), stream);
  upload(g.out_ptr, out_ptr.data(), out_ptr.size(), stream);
  upload(g.out_dst, out_dst.data(), out_dst.size(), stream);
  g.in_rec.alloc((size_t)L * 16);
  // the uploads read host vectors that die with this scope
  HIP_TRY(hipStreamSynchronize(stream));
}

// Chunks of the collective: every NPU contributes cpn, or (rooted) the root's cpn alone.
uint32_t total_chunks(uint32_t N, uint32_t cpn, uint32_t root) { return root == tacos::kNoRoot ? N * cpn : cpn; }

// Per-pass device state descriptor over a graph; held / carry / free_at / ctl are the
// pass's own buffers.
PassDev make_pass_dev(const PassGraph &g, const DevBuf &d_cost, uint32_t cpn, uint32_t root, uint64_t seed,
                      uint32_t phase, bool reversed, unsigned long long *held, uint32_t *carry,
                      unsigned long long *free_at, Ctl *ctl)
{
  const uint32_t C = total_chunks(g.N, cpn, root);
  const uint32_t NP = (C + 8191u) / 8192u;
  PassDev p{};
  p.N = g.N; p.L = g.L; p.cpn = cpn; p.NP = NP; p.C = C; p.root = root; p.phase = phase;
  p.seed_lo = (uint32_t)(seed & 0xFFFFFFFFull); p.seed_hi = (uint32_t)(seed >> 32);
  p.row_words = NP * 128u; p.reversed = reversed ? 1u : 0u;
  p.max_deg = g.max_deg;
  p.held = held;
  p.in_ptr = g.in_ptr.as<uint32_t>(); p.in_link = g.in_link.as<uint32_t>();
  p.in_src = g.in_src.as<uint32_t>(); p.pos_dst = g.pos_dst.as<uint32_t>();
  p.in_rec = g.in_rec.as<uint4>();
  p.slot_rec = g.slot_rec.as<uint4>();
  p.n_slots = g.N;
  p.cost = d_cost.as<unsigned long long>();
  p.carry = carry; p.free_at = free_at;
  p.ctl = ctl;
  return p;
}

// Nearly every link with a cost of its own: spans then sit on about as many times as there are
// transfers, about one transfer per span.
bool nearly_all_costs_differ(const std::vector<uint64_t> &cost)
{
  std::vector<uint64_t> sorted(cost);
  std::sort(sorted.begin(), sorted.end());
  const size_t distinct = (size_t)(std::unique(sorted.begin(), sorted.end()) - sorted.begin());
  return distinct >= 64 && distinct * 4 >= cost.size();
}

// Whether the single-workgroup kernel can take this shape on the current device.
bool fits_small_kernel(uint32_t N, uint32_t L, uint32_t NP)
{
  int dev = 0, lds_max = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
  const size_t need = tacos::small_sweep_lds_bytes(N, L, NP);
  return need != (size_t)-1 && need <= (size_t)lds_max;
}

// Runs one All-Gather pass over links psrc[l] -> pdst[l] and stores its schedule rows.
int run_pass(uint32_t N, uint32_t L, const std::vector<uint32_t> &psrc, const std::vector<uint32_t> &pdst,
             const DevBuf &d_cost, uint32_t cpn, uint32_t root, uint64_t seed, uint32_t phase, bool reversed,
             uint64_t max_events, bool time_kernels, uint32_t launch_mode, const std::vector<uint64_t> *order_cost,
             uint32_t match_mode, uint64_t uniform_cost, bool many_costs, hipStream_t stream, tacos_result &res,
             Pass &pass)
{
  const uint32_t C = total_chunks(N, cpn, root);
  const uint32_t NP = (C + 8191u) / 8192u;
  pass.reversed = reversed;
  pass.L = L;
  pass.rows_per_seg = (uint32_t)std::max<size_t>(1, std::min<size_t>(kSegmentBytes / ((size_t)L * 4), 1u << 20));

  PassGraph g;
  build_pass_graph(N, L, psrc, pdst, order_cost, stream, g);
  // An NPU without incoming links (in this pass's orientation) never receives anything.  If it
  // misses a chunk, the sweep ends with postconditions left and nothing in flight: the topology
  // is not strongly connected (Algorithm 2 would expand the TEN for ever).  The per-span kernels
  // look for missing chunks through a destination's idle incoming links, which such an NPU does
  // not have, so the case is settled here, for every launch mode alike.
  for (uint32_t d = 0; d < N; ++d) {
    const bool misses_chunks = root == tacos::kNoRoot ? N > 1 : d != root;
    if (misses_chunks && g.h_in_ptr[d + 1] == g.h_in_ptr[d]) return TACOS_E_UNREACHABLE;
  }
  // Small topologies: one workgroup sweeps many spans with the link state in LDS.  Chosen
  // automatically when the shape fits (launch_mode 0), forced by launch_mode 2.
  bool small = false;
  if (launch_mode == 0 || launch_mode == 2) {
    small = fits_small_kernel(N, L, NP);
    if (!small && launch_mode == 2) {
      g_last_error = "launch_mode 2: links, NPUs and need rows do not fit the LDS of one workgroup";
      return TACOS_E_INVAL;
    }
    // Automatic: one workgroup is the fastest form while a span has little to decide (links that
    // nearly all cost differently: about one transfer per span; at most 64 links) or while its
    // destinations are matched one per lane (links x row words up to 8,192).  Where most links are
    // matched in most spans and a wavefront has to take the destinations one after the other, a
    // span costs it 0.75 us per 16 links: with equal link costs one launch per span is faster
    // (8 x 8 x 8 torus with 3 chunks per NPU: 12 against 176 us per span), with a few cost classes
    // two launches per span (4 x 4 x 8 heterogeneous torus with 16 chunks per NPU: 10 against 27).
    // (The postcondition-centric orders have no lane-per-destination form: 16 x 16 mesh with 8
    // chunks per NPU 57 against 12 us per span with two launches.)
    if (small && launch_mode == 0) {
      const bool by_lane = tacos::small_sweep_by_lane(N, L, NP, C, match_mode) && (uint64_t)L * ((C + 63u) / 64u) <= 8192u;
      if (!many_costs && !by_lane && L > 64) small = false;
    }
  }
  // Homogeneous TEN (all links cost the same): one launch per span on a double-buffered held
  // table; link-centric matching, rows that fit the registers, complete runs only.  Span e is
  // at time e * cost, which must not overflow for any span index.
  const uint32_t row_words = NP * 128u;
  const size_t held_bytes = (size_t)N * row_words * 8;
  const bool can_uniform = !small && uniform_cost != 0 && uniform_cost <= (1ull << 31) && NP <= 8 && match_mode == 0 &&
                           max_events == 0;
  // Chosen automatically while both tables fit the 256 MiB Infinity Cache: then it is 1.1x
  // (32,768 NPUs) to 1.6x (4,096 NPUs) faster than two launches per span; beyond that the
  // second table's traffic costs more than the saved launch (40,960 NPUs: 13 % slower).
  const bool uniform = can_uniform && (launch_mode == 3 || (launch_mode == 0 && 2 * held_bytes <= kUniformAutoBytes));
  if (launch_mode == 3 && !uniform) {
    g_last_error = "launch_mode 3 needs equal link costs of at most 2^31 ps, at most 65,536 chunks, link-centric "
                   "matching and a complete run";
    return TACOS_E_INVAL;
  }
  DevBuf d_held, d_carry, d_free_at, d_ctl;
  d_held.alloc(uniform ? 2 * held_bytes : held_bytes);
  d_carry.alloc((size_t)L * 4);
  d_free_at.alloc((size_t)L * 8);
  d_ctl.alloc(sizeof(Ctl));
  PassDev p = make_pass_dev(g, d_cost, cpn, root, seed, phase, reversed, d_held.as<unsigned long long>(),
                            d_carry.as<uint32_t>(), d_free_at.as<unsigned long long>(), d_ctl.as<Ctl>());
  // per-span launches: destinations that hold every chunk are dropped from the order
  DevBuf d_done;
  std::vector<uint32_t> h_done;
  uint32_t n_active = N;
  if (!small) {
    d_done.alloc((size_t)N * 4);
    HIP_TRY(hipMemsetAsync(d_done.p, 0, (size_t)N * 4, stream));
    p.dest_done = d_done.as<uint32_t>();
    h_done.assign(N, 0);
  }
  DevBuf d_next_slots;
  if (!small) {  // (the homogeneous-TEN form needs them once it hands over to the link-state form)
    d_next_slots.alloc((size_t)2 * tacos::kNextSlots * 8);
    p.next_slots = d_next_slots.as<unsigned long long>();
    p.next_mask = N <= 8192u ? tacos::kNextSlots - 1u : 0u;  // short launches spread over the words
  }
  tacos::launch_init_pass(p, stream);
  HIP_TRY(hipGetLastError());

  PinnedCtl host_ctl;
  EventPool pool;
  auto row_slot = [&](uint64_t e, uint32_t **row, unsigned long long **tslot) {
    const uint64_t k = e / pass.rows_per_seg;
    const size_t stride = pass.row_stride();
    while (pass.segs.size() <= k) {
      Segment s;
      s.rows.alloc((size_t)pass.rows_per_seg * stride * 4);
      s.row_time.alloc((size_t)pass.rows_per_seg * 8);
      if (pass.prefill) HIP_TRY(hipMemsetAsync(s.rows.p, 0xFF, s.rows.bytes, stream));  // TACOS_NO_CHUNK
      pass.segs.push_back(std::move(s));
    }
    const uint64_t i = e - k * pass.rows_per_seg;
    *row = pass.segs[k].rows.as<uint32_t>() + i * stride;
    *tslot = pass.segs[k].row_time.as<unsigned long long>() + i;
  };

  uint64_t e = 0;
  bool stopped = false;  // prefix run reached max_events
  // Per-span launches on a topology whose links nearly all cost differently: about one transfer
  // starts per span, so dense rows (one entry per link and span) would be almost empty and
  // millions of them long.  Such a pass keeps compact records as the single-workgroup kernel
  // does, provided the epilogue can order a span's records (one LDS word per link).
  const uint64_t n_transfers = (uint64_t)N * C - C;
  const bool compact_spans = !small && !uniform && many_costs && NP <= 8 && L <= tacos::compact_schedule_max_links() &&
                             n_transfers <= 0xFFFFFFFEull;
  pass.prefill = !small && !compact_spans;  // dense rows: the kernels write matches (a reversed pass: arrivals) only
  if (small || compact_spans) {
    // compact records: exactly one per unsatisfied postcondition of the pass
    pass.compact = true;
    pass.rows_per_seg = 1u << 20;
    if (n_transfers > 0xFFFFFFFEull) { g_last_error = "more than 2^32-2 transfers in a pass of the single-workgroup kernel"; return TACOS_E_INVAL; }
    pass.recs.alloc((size_t)std::max<uint64_t>(n_transfers, 1) * 8);
  }
  DevBuf d_rnd, d_prev;
  if (!small && match_mode == 0) {
    d_rnd.alloc((size_t)L * 4 * (uniform ? 2 : 1));
    p.rnd = d_rnd.as<uint32_t>();
  }
  tacos::UniformDev u{};
  if (uniform) {
    d_prev.alloc((size_t)L * 4 * 2);
    u.held[0] = d_held.as<unsigned long long>();
    u.held[1] = u.held[0] + (size_t)N * row_words;
    u.prev[0] = d_prev.as<uint32_t>();
    u.prev[1] = u.prev[0] + L;
    u.rnd[0] = d_rnd.as<uint32_t>();
    u.rnd[1] = u.rnd[0] + L;
    u.cost = uniform_cost;
    HIP_TRY(hipMemcpyAsync(u.held[1], u.held[0], held_bytes, hipMemcpyDeviceToDevice, stream));
    tacos::launch_uniform_init(p, u, match_mode, stream);
    HIP_TRY(hipGetLastError());
  }
  if (small) {
    for (;;) {
      if (e >= 0xFFFFFFFEull) { g_last_error = "more than 2^32-2 spans"; return TACOS_E_OVERFLOW; }
      uint32_t *row = nullptr;
      unsigned long long *tslot = nullptr;
      row_slot(e, &row, &tslot);
      // as many spans as the current segment still has rows for
      const uint64_t seg_end = (e / pass.rows_per_seg + 1) * pass.rows_per_seg;
      uint64_t n = std::min<uint64_t>(seg_end - e, 0xFFFFFFFEull - e);
      uint32_t stop_event = 0xFFFFFFFFu;
      if (max_events && e + n > max_events) { n = max_events - e + 1; stop_event = (uint32_t)max_events; }
      hipEvent_t ev0 = nullptr, ev1 = nullptr;
      if (time_kernels) {
        pool.ensure(2);
        ev0 = pool.ev[0]; ev1 = pool.ev[1];
        HIP_TRY(hipEventRecord(ev0, stream));
      }
      HIP_TRY(tacos::launch_small_sweep(p, g.out_ptr.as<uint32_t>(), g.out_dst.as<uint32_t>(), (uint32_t)e,
                                        (uint32_t)n, stop_event, pass.recs.as<uint2>(), row, tslot, match_mode,
                                        many_costs, stream));
      if (time_kernels) HIP_TRY(hipEventRecord(ev1, stream));
      HIP_TRY(hipMemcpyAsync(host_ctl.p, p.ctl, sizeof(Ctl), hipMemcpyDeviceToHost, stream));
      HIP_TRY(hipStreamSynchronize(stream));
      if (time_kernels) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, ev0, ev1));
        res.kernel_ms += ms;
        res.kernel_launches++;
      }
      e += n;
      if (host_ctl.p->done) break;
      if (stop_event != 0xFFFFFFFFu) { stopped = true; break; }
    }
  } else {
    // Link-centric passes with dense rows: once at most kTailSlots destinations are left in the
    // processing order, one single-workgroup launch sweeps many spans (tail_sweep_kernel), up
    // to the end of the row segment.  launch_mode 4 keeps two launches for every span.
    const bool tail_ok = launch_mode != 4 && !compact_spans && match_mode == 0 && NP <= 8 && max_events == 0 &&
                         p.max_deg >= 1u && p.max_deg <= 64u;
    // The homogeneous-TEN form (one launch per span) hands over to the link-state form for that
    // last stretch (automatic mode only; launch_mode 3 keeps one launch per span to the end).
    bool uniform_now = uniform;
    // ... and a pass that started with two launches per span because of its size goes over to
    // one launch per span once at most kLateUniformSlots destinations are left (automatic mode).
    constexpr uint32_t kLateUniformSlots = 2048;
    bool late_uniform_ok = launch_mode == 0 && !uniform && !compact_spans && uniform_cost != 0 &&
                           uniform_cost <= (1ull << 31) && NP <= 8 && match_mode == 0 && max_events == 0;
    DevBuf d_held_b, d_rnd_b;
    constexpr uint32_t kTailBatch = 1024;
    uint32_t batch = 8;
    for (;;) {
      size_t n_timed = 0;
      uint64_t tail_spans = 0;  // spans of this batch swept by a tail launch (then the whole batch)
      if (time_kernels) pool.ensure(2 * (size_t)batch);
      if (!uniform_now && late_uniform_ok && p.n_slots <= kLateUniformSlots && p.n_slots > tacos::kTailSlots && e >= 1) {
        late_uniform_ok = false;  // once
        // Equal link costs on a topology too large for two held tables beside each other in the
        // Infinity Cache: with few destinations left that no longer matters, and one launch per
        // span is half the launches.  The table so far becomes the one span e reads (it receives
        // the arrivals of span e), a copy of it the lagging one.  Without memory for the copy the
        // pass goes on as it is.
        if (d_held_b.try_alloc(held_bytes) && d_prev.try_alloc((size_t)L * 4 * 2) && d_rnd_b.try_alloc((size_t)L * 4 * 2)) {
          u.held[e & 1u] = d_held.as<unsigned long long>();
          u.held[(e + 1) & 1u] = d_held_b.as<unsigned long long>();
          u.prev[0] = d_prev.as<uint32_t>();
          u.prev[1] = u.prev[0] + L;
          u.rnd[0] = d_rnd_b.as<uint32_t>();
          u.rnd[1] = u.rnd[0] + L;
          u.cost = uniform_cost;
          uint32_t *row = nullptr;
          unsigned long long *tslot = nullptr;
          row_slot(e, &row, &tslot);
          tacos::launch_links_to_uniform(p, u, (uint32_t)e, reversed ? row : nullptr, stream);
          HIP_TRY(hipGetLastError());
          uniform_now = true;
        }
      }
      if (uniform_now && launch_mode == 0 && tail_ok && p.n_slots <= tacos::kTailSlots && e >= 1) {
        // state before the arrivals of span e: the table span e - 1 read, the chunks it matched in flight
        p.held = u.held[(e - 1) & 1u];
        HIP_TRY(hipMemsetAsync(p.next_slots, 0xFF, (size_t)2 * tacos::kNextSlots * 8, stream));  // kInf
        tacos::launch_uniform_handover(p, u, (uint32_t)e, stream);
        uniform_now = false;
      }
      if (!uniform_now && tail_ok && p.n_slots <= tacos::kTailSlots) {
        if (e >= 0xFFFFFFFEull) { g_last_error = "more than 2^32-2 spans"; return TACOS_E_OVERFLOW; }
        uint32_t *row = nullptr;
        unsigned long long *tslot = nullptr;
        row_slot(e, &row, &tslot);
        const uint64_t seg_end = (e / pass.rows_per_seg + 1) * pass.rows_per_seg;
        tail_spans = std::min<uint64_t>(std::min<uint64_t>(kTailBatch, seg_end - e), 0xFFFFFFFEull - e);
        if (time_kernels) HIP_TRY(hipEventRecord(pool.ev[0], stream));
        HIP_TRY(tacos::launch_tail_sweep(p, (uint32_t)e, (uint32_t)tail_spans, row, pass.row_stride(), tslot, stream));
        if (time_kernels) { HIP_TRY(hipEventRecord(pool.ev[1], stream)); n_timed = 1; }
        e += tail_spans;
      }
      for (uint32_t i = 0; i < batch && tail_spans == 0; ++i) {
        if (e >= 0xFFFFFFFEull) { g_last_error = "more than 2^32-2 spans"; return TACOS_E_OVERFLOW; }
        uint32_t *row = nullptr;
        unsigned long long *tslot = nullptr;
        row_slot(e, &row, &tslot);
        if (uniform_now) {
          uint32_t *row_next = nullptr;
          unsigned long long *tslot_next = nullptr;
          if (reversed) row_slot(e + 1, &row_next, &tslot_next);  // rows are keyed by arrival
          if (time_kernels) HIP_TRY(hipEventRecord(pool.ev[2 * n_timed], stream));
          tacos::launch_match_uniform(p, u, (uint32_t)e, reversed ? nullptr : row, row_next, tslot, match_mode, stream);
          if (time_kernels) { HIP_TRY(hipEventRecord(pool.ev[2 * n_timed + 1], stream)); n_timed++; }
          e++;
          continue;
        }
        if (compact_spans) {
          // `row` is the span's slot for the index of its first record: a forward pass's arrivals
          // kernel fills it; in a reversed pass (records = arrivals) the matching of the span before
          uint32_t *first_next = nullptr;
          unsigned long long *tslot_next = nullptr;
          if (reversed) row_slot(e + 1, &first_next, &tslot_next);
          tacos::launch_arrive(p, (uint32_t)e, tslot, nullptr, reversed ? pass.recs.as<uint2>() : nullptr,
                               (!reversed || e == 0) ? row : nullptr, stream);
          if (max_events && e >= max_events) { stopped = true; break; }
          if (time_kernels) HIP_TRY(hipEventRecord(pool.ev[2 * n_timed], stream));
          tacos::launch_match_compact(p, (uint32_t)e, pass.recs.as<uint2>(), first_next, match_mode, stream);
          if (time_kernels) { HIP_TRY(hipEventRecord(pool.ev[2 * n_timed + 1], stream)); n_timed++; }
          e++;
          continue;
        }
        tacos::launch_arrive(p, (uint32_t)e, tslot, reversed ? row : nullptr, nullptr, nullptr, stream);
        if (max_events && e >= max_events) { stopped = true; break; }
        if (time_kernels) HIP_TRY(hipEventRecord(pool.ev[2 * n_timed], stream));
        tacos::launch_match(p, (uint32_t)e, reversed ? nullptr : row, match_mode, stream);
        if (time_kernels) { HIP_TRY(hipEventRecord(pool.ev[2 * n_timed + 1], stream)); n_timed++; }
        e++;
      }
      HIP_TRY(hipGetLastError());
      HIP_TRY(hipMemcpyAsync(host_ctl.p, p.ctl, sizeof(Ctl), hipMemcpyDeviceToHost, stream));
      HIP_TRY(hipStreamSynchronize(stream));
      const bool done = host_ctl.p->done != 0;
      if (time_kernels && tail_spans) {
        // a tail launch counts once per span it swept
        const uint64_t e_first = e - tail_spans, e_end = host_ctl.p->n_events;
        const uint64_t useful = !done ? tail_spans : (e_end > e_first ? std::min<uint64_t>(tail_spans, e_end - e_first) : 0);
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, pool.ev[0], pool.ev[1]));
        if (useful) { res.kernel_ms += ms; res.kernel_launches += useful; }
      } else if (time_kernels) {
        // launches after the pass ended return at once; count the ones that did work
        const uint64_t e_first = e - n_timed, e_end = host_ctl.p->n_events;
        const uint64_t useful = !done ? n_timed : (e_end > e_first ? std::min<uint64_t>(n_timed, e_end - e_first) : 0);
        for (size_t i = 0; i < n_timed; ++i) {
          float ms = 0.f;
          HIP_TRY(hipEventElapsedTime(&ms, pool.ev[2 * i], pool.ev[2 * i + 1]));
          if (i < useful) { res.kernel_ms += ms; res.kernel_launches++; }
        }
      }
      if (done || stopped) break;
      batch = std::min<uint32_t>(batch * 2, 512);
      // Drop the destinations that are complete from the processing order once that
      // shrinks the launch by an eighth (the first slot always stays: it ends the pass).
      HIP_TRY(hipMemcpyAsync(h_done.data(), d_done.p, (size_t)N * 4, hipMemcpyDeviceToHost, stream));
      HIP_TRY(hipStreamSynchronize(stream));
      uint32_t alive = 0;
      for (uint32_t k = 0; k < N; ++k) alive += (k == 0 || !h_done[g.h_order[k]]) ? 1u : 0u;
      if (alive < n_active && alive + n_active / 8 <= n_active) {
        std::vector<uint32_t> rec((size_t)alive * 4, 0);
        size_t w = 0;
        for (uint32_t k = 0; k < N; ++k) {
          const uint32_t d = g.h_order[k];
          if (k != 0 && h_done[d]) continue;
          rec[w] = d; rec[w + 1] = g.h_in_ptr[d]; rec[w + 2] = g.h_in_ptr[d + 1];
          w += 4;
        }
        HIP_TRY(hipMemcpyAsync(g.slot_rec.p, rec.data(), rec.size() * 4, hipMemcpyHostToDevice, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        n_active = alive;
        p.n_slots = alive;
      }
    }
  }

  const Ctl &c = *host_ctl.p;
  if (c.status == tacos::kStUnreachable) return TACOS_E_UNREACHABLE;
  if (c.status == tacos::kStOverflow) return TACOS_E_OVERFLOW;
  if (c.status == tacos::kStInternal) {
    g_last_error = "internal: matching produced a chunk id out of range";
    return TACOS_E_DEVICE;
  }
  if (c.done) {
    pass.T = c.T;
    pass.n_events = c.n_events;
  } else {  // prefix run: time reached, sweeps run
    pass.T = c.next_t[max_events & 1u];
    pass.n_events = max_events;
  }
  pass.n_rows = reversed ? pass.n_events + 1 : pass.n_events;
  pass.n_rec = c.n_rec;
  // drop segments past the end (batches run ahead of the terminating span)
  const uint64_t used_segs = (pass.n_rows + pass.rows_per_seg - 1) / pass.rows_per_seg;
  while (pass.segs.size() > used_segs) pass.segs.pop_back();
  return TACOS_OK;
}

// Epilogue of a pass: event times to the host, per-row match counts and the digest.
void finish_pass(Pass &pass, uint64_t t_off, uint64_t *digest, hipStream_t stream)
{
  pass.t_off = t_off;
  pass.row_time.assign(pass.n_rows, 0);
  pass.row_count.assign(pass.n_rows, 0);
  const size_t digest_bytes = (size_t)tacos::kDigestSlots * 16 * 8;  // partial sums, one per cache line
  DevBuf d_digest(digest_bytes);
  HIP_TRY(hipMemsetAsync(d_digest.p, 0, digest_bytes, stream));
  const uint64_t t_base = pass.reversed ? pass.T : t_off;
  if (pass.compact) {
    // gather the spans' first-record indices and times, order every span's records by link
    // and digest them; the per-span segments are not needed afterwards
    pass.first.assign(pass.n_rows + 1, 0);
    for (size_t k = 0; k < pass.segs.size(); ++k) {
      const uint64_t first = (uint64_t)k * pass.rows_per_seg;
      if (first >= pass.n_rows) break;
      const size_t n = (size_t)std::min<uint64_t>(pass.rows_per_seg, pass.n_rows - first);
      HIP_TRY(hipMemcpyAsync(pass.first.data() + first, pass.segs[k].rows.p, n * 4, hipMemcpyDeviceToHost, stream));
      HIP_TRY(hipMemcpyAsync(pass.row_time.data() + first, pass.segs[k].row_time.p, n * 8, hipMemcpyDeviceToHost, stream));
    }
    HIP_TRY(hipStreamSynchronize(stream));
    pass.first[pass.n_rows] = (uint32_t)pass.n_rec;
    pass.segs.clear();
    upload(pass.d_first, pass.first.data(), pass.first.size(), stream);
    upload(pass.d_time, reinterpret_cast<const unsigned long long *>(pass.row_time.data()), pass.row_time.size(), stream);
    tacos::launch_compact_epilogue(pass.recs.as<uint2>(), pass.d_first.as<uint32_t>(), (uint32_t)pass.n_rows, pass.L,
                                   pass.d_time.as<unsigned long long>(), t_base, pass.reversed ? 1u : 0u,
                                   d_digest.as<unsigned long long>(), stream);
    HIP_TRY(hipGetLastError());
    for (uint64_t k = 0; k < pass.n_rows; ++k) pass.row_count[k] = pass.first[k + 1] - pass.first[k];
  }
  for (size_t k = 0; k < pass.segs.size(); ++k) {
    const uint64_t first = (uint64_t)k * pass.rows_per_seg;
    const uint32_t n = (uint32_t)std::min<uint64_t>(pass.rows_per_seg, pass.n_rows - first);
    DevBuf d_count((size_t)n * 4);
    HIP_TRY(hipMemsetAsync(d_count.p, 0, (size_t)n * 4, stream));
    tacos::launch_row_stats(pass.segs[k].rows.as<uint32_t>(), n, pass.L,
                            pass.segs[k].row_time.as<unsigned long long>(), t_base,
                            pass.reversed ? 1u : 0u, d_count.as<uint32_t>(),
                            d_digest.as<unsigned long long>(), stream);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(pass.row_time.data() + first, pass.segs[k].row_time.p, (size_t)n * 8,
                           hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipMemcpyAsync(pass.row_count.data() + first, d_count.p, (size_t)n * 4,
                           hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
  }
  std::vector<uint64_t> partial((size_t)tacos::kDigestSlots * 16);
  HIP_TRY(hipMemcpyAsync(partial.data(), d_digest.p, digest_bytes, hipMemcpyDeviceToHost, stream));
  HIP_TRY(hipStreamSynchronize(stream));
  for (uint32_t k = 0; k < tacos::kDigestSlots; ++k) *digest += partial[(size_t)k * 16];
  pass.canon_base.assign(pass.n_rows + 1, 0);
  for (uint64_t k = 0; k < pass.n_rows; ++k)
    pass.canon_base[k + 1] = pass.canon_base[k] + pass.row_count[pass.event_of(k)];
  pass.n_xfers = pass.canon_base[pass.n_rows];
}

bool is_rooted(int coll) { return coll == TACOS_BROADCAST || coll == TACOS_REDUCE; }
// a reversed pass (on the swapped orientation, mapped back in time) and / or a forward pass
bool has_reversed_pass(int coll) { return coll == TACOS_REDUCE_SCATTER || coll == TACOS_ALL_REDUCE || coll == TACOS_REDUCE; }
bool has_forward_pass(int coll) { return coll == TACOS_ALL_GATHER || coll == TACOS_ALL_REDUCE || coll == TACOS_BROADCAST; }

int validate(const tacos_topology_t *topo, uint32_t cpn, uint64_t chunk_bytes, int coll, const tacos_options_t *opts)
{
  if (!topo || !topo->row_ptr || topo->n_npus == 0 || cpn == 0 || chunk_bytes == 0) return TACOS_E_INVAL;
  if (coll < TACOS_ALL_GATHER || coll > TACOS_REDUCE) return TACOS_E_INVAL;
  if (is_rooted(coll) && opts && opts->root >= topo->n_npus) return TACOS_E_INVAL;
  const uint32_t N = topo->n_npus;
  if (topo->row_ptr[0] != 0) return TACOS_E_INVAL;
  for (uint32_t i = 0; i < N; ++i)
    if (topo->row_ptr[i + 1] < topo->row_ptr[i]) return TACOS_E_INVAL;
  const uint32_t L = topo->row_ptr[N];
  if (L != topo->n_links) return TACOS_E_INVAL;
  if (L && (!topo->col_idx || !topo->alpha_ps || !topo->beta_fs_per_B)) return TACOS_E_INVAL;
  if ((is_rooted(coll) ? (uint64_t)cpn : (uint64_t)N * cpn) > TACOS_MAX_CHUNKS) return TACOS_E_INVAL;
  for (uint32_t i = 0; i < N; ++i)
    for (uint32_t l = topo->row_ptr[i]; l < topo->row_ptr[i + 1]; ++l)
      if (topo->col_idx[l] >= N || topo->col_idx[l] == i) return TACOS_E_INVAL;
  return TACOS_OK;
}

int require_device(int *device)
{
  int n = 0;
  hipError_t e = hipGetDeviceCount(&n);
  if (e != hipSuccess || n <= 0) {
    g_last_error = std::string("no HIP device: ") + hipGetErrorString(e);
    (void)hipGetLastError();
    return TACOS_E_DEVICE;
  }
  e = hipGetDevice(device);
  if (e != hipSuccess) {
    g_last_error = std::string("hipGetDevice failed: ") + hipGetErrorString(e);
    return TACOS_E_DEVICE;
  }
  return TACOS_OK;
}

// a1 on the device; returns the device buffer and, if asked, a host copy.
int device_costs(const tacos_topology_t *topo, uint64_t chunk_bytes, hipStream_t stream, DevBuf &d_cost,
                 std::vector<uint64_t> *host_cost)
{
  const uint32_t L = topo->n_links;
  DevBuf d_alpha, d_beta, d_ovf(4);
  upload(d_alpha, reinterpret_cast<const unsigned long long *>(topo->alpha_ps), L, stream);
  upload(d_beta, reinterpret_cast<const unsigned long long *>(topo->beta_fs_per_B), L, stream);
  d_cost.alloc((size_t)L * 8);
  HIP_TRY(hipMemsetAsync(d_ovf.p, 0, 4, stream));
  tacos::launch_link_cost(d_alpha.as<unsigned long long>(), d_beta.as<unsigned long long>(), chunk_bytes, L,
                          d_cost.as<unsigned long long>(), d_ovf.as<uint32_t>(), stream);
  HIP_TRY(hipGetLastError());
  uint32_t ovf = 0;
  HIP_TRY(hipMemcpyAsync(&ovf, d_ovf.p, 4, hipMemcpyDeviceToHost, stream));
  if (host_cost) {
    host_cost->resize(L);
    if (L) HIP_TRY(hipMemcpyAsync(host_cost->data(), d_cost.p, (size_t)L * 8, hipMemcpyDeviceToHost, stream));
  }
  HIP_TRY(hipStreamSynchronize(stream));
  return ovf ? TACOS_E_OVERFLOW : TACOS_OK;
}

// Kernel matching mode from the options: 0 link-centric; 1 postcondition-centric, random
// holder; 2 postcondition-centric, first holder of the cheapest-first list.
int resolve_match_mode(const tacos_topology_t *topo, int coll, const tacos_options_t *opts, uint64_t n_chunks,
                       uint32_t *mode)
{
  *mode = 0;
  if (!opts || opts->matching == TACOS_MATCH_LINK_CENTRIC) return TACOS_OK;
  if (opts->matching != TACOS_MATCH_POSTCONDITION) return TACOS_E_INVAL;
  if (n_chunks > TACOS_MAX_CHUNKS_IN_REGISTERS) return TACOS_E_INVAL;  // streamed rows: link-centric only
  std::vector<uint32_t> deg_in(topo->n_npus, 0), deg_out(topo->n_npus, 0);
  for (uint32_t i = 0; i < topo->n_npus; ++i) {
    deg_out[i] = topo->row_ptr[i + 1] - topo->row_ptr[i];
    for (uint32_t l = topo->row_ptr[i]; l < topo->row_ptr[i + 1]; ++l) deg_in[topo->col_idx[l]]++;
  }
  for (uint32_t i = 0; i < topo->n_npus; ++i) {
    // the reversed pass of a Reduce-Scatter walks the out-links as incoming links
    const bool fwd = has_forward_pass(coll), rev = has_reversed_pass(coll);
    if ((fwd && deg_in[i] > 64) || (rev && deg_out[i] > 64)) return TACOS_E_INVAL;
  }
  *mode = opts->link_order == TACOS_LINK_ORDER_COST ? 2u : 1u;
  return TACOS_OK;
}

}  // namespace

extern "C" {

int tacos_synthesize(const tacos_topology_t *topo, uint32_t chunks_per_npu, uint64_t chunk_bytes,
                     tacos_collective_t coll, uint64_t seed, const tacos_options_t *opts,
                     tacos_result_t **out)
{
  g_last_error.clear();
  if (!out) return TACOS_E_INVAL;
  int rc = validate(topo, chunks_per_npu, chunk_bytes, (int)coll, opts);
  if (rc != TACOS_OK) return rc;
  const uint64_t max_events = opts ? opts->max_events : 0;
  if (max_events && has_reversed_pass((int)coll)) return TACOS_E_INVAL;
  if (opts && (opts->link_order > TACOS_LINK_ORDER_COST || opts->launch_mode > 4 ||
               opts->matching > TACOS_MATCH_POSTCONDITION))
    return TACOS_E_INVAL;
  // kernel variant: 0 link-centric; 1 postcondition-centric, random holder; 2 first holder
  uint32_t match_mode = 0;
  rc = resolve_match_mode(topo, (int)coll, opts,
                          is_rooted((int)coll) ? (uint64_t)chunks_per_npu : (uint64_t)topo->n_npus * chunks_per_npu,
                          &match_mode);
  if (rc != TACOS_OK) return rc;
  const bool time_kernels = opts && opts->time_kernels;
  const uint32_t launch_mode = opts ? opts->launch_mode : 0;
  const uint32_t root = is_rooted((int)coll) ? (opts ? opts->root : 0u) : tacos::kNoRoot;
  hipStream_t stream = opts ? static_cast<hipStream_t>(opts->stream) : nullptr;

  const auto wall0 = std::chrono::steady_clock::now();
  std::unique_ptr<tacos_result> res(new (std::nothrow) tacos_result);
  if (!res) return TACOS_E_NOMEM;
  rc = require_device(&res->device);
  if (rc != TACOS_OK) return rc;

  const uint32_t N = topo->n_npus, L = topo->n_links;
  try {
    res->N = N;
    res->L = L;
    res->link_src.resize(L);
    res->link_dst.assign(topo->col_idx, topo->col_idx + L);
    for (uint32_t i = 0; i < N; ++i)
      for (uint32_t l = topo->row_ptr[i]; l < topo->row_ptr[i + 1]; ++l) res->link_src[l] = i;

    const int n_pass = coll == TACOS_ALL_REDUCE ? 2 : 1;
    if (N == 1) {
      // a single NPU holds everything at t = 0: no span is expanded
      for (int i = 0; i < n_pass; ++i) {
        Pass ps;
        ps.reversed = has_reversed_pass((int)coll) && i == 0;
        ps.canon_base.assign(1, 0);
        res->passes.push_back(std::move(ps));
      }
    } else {
      if (L == 0) return TACOS_E_UNREACHABLE;
      DevBuf &d_cost = res->d_cost;
      std::vector<uint64_t> host_cost;
      const bool by_cost = opts && opts->link_order == TACOS_LINK_ORDER_COST;
      rc = device_costs(topo, chunk_bytes, stream, d_cost, &host_cost);
      if (rc != TACOS_OK) return rc;
      const std::vector<uint64_t> *order_cost = by_cost ? &host_cost : nullptr;
      // the common cost if every link costs the same (a homogeneous TEN), else 0
      uint64_t uniform_cost = host_cost[0];
      for (uint32_t l = 1; l < L && uniform_cost; ++l)
        if (host_cost[l] != host_cost[0]) uniform_cost = 0;
      const bool many_costs = !uniform_cost && nearly_all_costs_differ(host_cost);
      // reversed pass: every link (s -> d) is used as (d -> s), ids and costs unchanged
      auto run_one = [&](bool rev, hipStream_t st, Pass &ps) {
        return run_pass(N, L, rev ? res->link_dst : res->link_src, rev ? res->link_src : res->link_dst, d_cost,
                        chunks_per_npu, root, seed, rev ? 1u : 0u, rev, rev ? 0 : max_events, time_kernels, launch_mode,
                        order_cost, match_mode, uniform_cost, many_costs, st, *res, ps);
      };
      uint64_t t_off = 0;
      // All-Reduce: the Reduce-Scatter and the All-Gather pass do not depend on each other (the
      // All-Gather half equals the stand-alone All-Gather), and up to some ten thousand NPUs a
      // pass is bound by the latency of its launches, not by the GPU's throughput: the two then
      // sweep at the same time, the All-Gather pass on a stream of its own from a second host
      // thread (1.3 to 1.9 times faster between 128 and 16,384 NPUs).  Not where the passes' held
      // tables together (four of them with one launch per span) would no longer fit the Infinity
      // Cache (24,576 NPUs: 3 % slower, 32,768: 14 %; two 200-MB passes would gain 3 %), not for
      // a few thousand transfers (the second stream and thread cost 0.3 ms), and not with kernel
      // timing, which is to measure a kernel by itself.
      const uint32_t C_total = total_chunks(N, chunks_per_npu, root);
      const size_t held_bytes_pass = (size_t)N * ((C_total + 8191u) / 8192u) * 1024;
      if (coll == TACOS_ALL_REDUCE && !time_kernels && held_bytes_pass <= kConcurrentPassBytes &&
          (uint64_t)C_total * (N - 1) >= 4096) {
        res->passes.reserve(2);
        res->passes.emplace_back();
        res->passes.emplace_back();
        OwnedStream side;
        int rc_side = TACOS_OK;
        std::string err_side;
        {
          JoiningThread th([&] {
            try {
              HIP_TRY(hipSetDevice(res->device));
              rc_side = run_one(false, side.s, res->passes[1]);
            } catch (const HipFail &f) {
              rc_side = f.code;
            } catch (const std::bad_alloc &) {
              g_last_error = "host allocation failed";
              rc_side = TACOS_E_NOMEM;
            }
            err_side = g_last_error;
          });
          rc = run_one(true, stream, res->passes[0]);  // (th is joined on every way out of this block)
        }
        if (rc != TACOS_OK) return rc;
        if (rc_side != TACOS_OK) { g_last_error = err_side; return rc_side; }
        finish_pass(res->passes[0], 0, &res->digest, stream);
        finish_pass(res->passes[1], res->passes[0].T, &res->digest, stream);
      } else {
        if (has_reversed_pass((int)coll)) {
          res->passes.emplace_back();
          rc = run_one(true, stream, res->passes.back());
          if (rc != TACOS_OK) return rc;
          finish_pass(res->passes.back(), 0, &res->digest, stream);
          t_off = res->passes.back().T;
        }
        if (has_forward_pass((int)coll)) {
          res->passes.emplace_back();
          rc = run_one(false, stream, res->passes.back());
          if (rc != TACOS_OK) return rc;
          finish_pass(res->passes.back(), t_off, &res->digest, stream);
        }
      }
    }
    for (const Pass &ps : res->passes) {
      res->collective_time += ps.T;
      res->n_events += ps.n_events;
      res->n_xfers += ps.n_xfers;
      res->device_bytes += ps.recs.bytes + ps.d_first.bytes + ps.d_time.bytes;
      for (const Segment &sg : ps.segs) res->device_bytes += sg.rows.bytes + sg.row_time.bytes;
    }
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    g_last_error = "host allocation failed";
    return TACOS_E_NOMEM;
  } catch (const std::system_error &e) {  // a host thread could not be started
    g_last_error = std::string("host thread: ") + e.what();
    return TACOS_E_DEVICE;
  }
  res->wall_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - wall0).count();
  *out = res.release();
  return TACOS_OK;
}

int tacos_seed_search(const tacos_topology_t *topo, uint32_t chunks_per_npu, uint64_t chunk_bytes,
                      tacos_collective_t coll, const uint64_t *seeds, uint32_t n_seeds,
                      const tacos_options_t *opts, uint64_t *time_ps, uint64_t *num_events, uint32_t *best)
{
  g_last_error.clear();
  if (!seeds || n_seeds == 0 || !time_ps) return TACOS_E_INVAL;
  int rc = validate(topo, chunks_per_npu, chunk_bytes, (int)coll, opts);
  if (rc != TACOS_OK) return rc;
  if (opts && (opts->max_events != 0 || opts->link_order > TACOS_LINK_ORDER_COST || opts->launch_mode > 4 ||
               opts->matching > TACOS_MATCH_POSTCONDITION))
    return TACOS_E_INVAL;
  uint32_t match_mode = 0;
  rc = resolve_match_mode(topo, (int)coll, opts,
                          is_rooted((int)coll) ? (uint64_t)chunks_per_npu : (uint64_t)topo->n_npus * chunks_per_npu,
                          &match_mode);
  if (rc != TACOS_OK) return rc;
  const uint32_t launch_mode = opts ? opts->launch_mode : 0;
  const uint32_t root = is_rooted((int)coll) ? (opts ? opts->root : 0u) : tacos::kNoRoot;
  hipStream_t stream = opts ? static_cast<hipStream_t>(opts->stream) : nullptr;
  int device = 0;
  rc = require_device(&device);
  if (rc != TACOS_OK) return rc;

  const uint32_t N = topo->n_npus, L = topo->n_links;
  auto pick_best = [&]() {
    uint32_t b = 0;
    for (uint32_t i = 1; i < n_seeds; ++i)
      if (time_ps[i] < time_ps[b]) b = i;
    if (best) *best = b;
  };
  if (N == 1) {
    for (uint32_t i = 0; i < n_seeds; ++i) { time_ps[i] = 0; if (num_events) num_events[i] = 0; }
    pick_best();
    return TACOS_OK;
  }
  if (L == 0) return TACOS_E_UNREACHABLE;

  try {
    const uint32_t C = total_chunks(N, chunks_per_npu, root);
    const uint32_t NP = (C + 8191u) / 8192u;
    const bool concurrent = (launch_mode == 0 || launch_mode == 2) && fits_small_kernel(N, L, NP);
    if (!concurrent && launch_mode == 2) {
      g_last_error = "launch_mode 2: links, NPUs and need rows do not fit the LDS of one workgroup";
      return TACOS_E_INVAL;
    }
    if (!concurrent) {
      // Whole syntheses, each with its per-span launches.  Up to some ten thousand NPUs such a
      // synthesis is bound by the latency of its launches and leaves most of the GPU idle:
      // several host threads then take the seeds in turn, each on a stream of its own (8 seeds
      // on a 64 x 64 mesh 121 -> 47 ms with four threads; an All-Reduce already sweeps its two
      // passes at once and gets two).  A larger topology fills the GPU by itself: one seed after
      // the other on the caller's stream.
      auto one_seed = [&](uint32_t i, const tacos_options_t *o) {
        tacos_result_t *r = nullptr;
        const int c = tacos_synthesize(topo, chunks_per_npu, chunk_bytes, coll, seeds[i], o, &r);
        if (c != TACOS_OK) return c;
        time_ps[i] = r->collective_time;
        if (num_events) num_events[i] = r->n_events;
        tacos_result_free(r);
        return (int)TACOS_OK;
      };
      const size_t held_bytes_pass = (size_t)N * NP * 1024;
      const uint32_t n_threads = (held_bytes_pass <= kConcurrentPassBytes && (uint64_t)C * (N - 1) >= 4096)
                                     ? std::min<uint32_t>(coll == TACOS_ALL_REDUCE ? 2u : 4u, n_seeds) : 1u;
      if (n_threads <= 1) {
        for (uint32_t i = 0; i < n_seeds; ++i) {
          rc = one_seed(i, opts);
          if (rc != TACOS_OK) return rc;
        }
      } else {
        std::atomic<uint32_t> next{0};
        std::atomic<int> first_rc{TACOS_OK};
        std::mutex err_lock;
        std::string err;
        {
          std::vector<std::unique_ptr<JoiningThread>> workers;
          for (uint32_t w = 0; w < n_threads; ++w) {
            workers.emplace_back(new JoiningThread([&] {
              int c = TACOS_OK;
              try {
                HIP_TRY(hipSetDevice(device));
                OwnedStream own;
                tacos_options_t o{};
                if (opts) o = *opts;
                o.stream = own.s;
                for (uint32_t i = next.fetch_add(1); i < n_seeds && first_rc.load() == TACOS_OK; i = next.fetch_add(1))
                  if ((c = one_seed(i, &o)) != TACOS_OK) break;
              } catch (const HipFail &f) {
                c = f.code;
              } catch (const std::bad_alloc &) {
                g_last_error = "host allocation failed";
                c = TACOS_E_NOMEM;
              }
              if (c != TACOS_OK) {
                std::lock_guard<std::mutex> hold(err_lock);
                int expected = TACOS_OK;
                if (first_rc.compare_exchange_strong(expected, c)) err = g_last_error;
              }
            }));
          }
        }  // joined
        if (first_rc.load() != TACOS_OK) {
          g_last_error = err;
          return first_rc.load();
        }
      }
      pick_best();
      return TACOS_OK;
    }

    std::vector<uint32_t> link_src(L), link_dst(topo->col_idx, topo->col_idx + L);
    for (uint32_t i = 0; i < N; ++i)
      for (uint32_t l = topo->row_ptr[i]; l < topo->row_ptr[i + 1]; ++l) link_src[l] = i;
    DevBuf d_cost;
    std::vector<uint64_t> host_cost;
    const bool by_cost = opts && opts->link_order == TACOS_LINK_ORDER_COST;
    rc = device_costs(topo, chunk_bytes, stream, d_cost, &host_cost);
    if (rc != TACOS_OK) return rc;
    const std::vector<uint64_t> *order_cost = by_cost ? &host_cost : nullptr;
    const bool sparse = nearly_all_costs_differ(host_cost);  // as tacos_synthesize: one destination per wavefront
    const bool want_rev = has_reversed_pass((int)coll), want_fwd = has_forward_pass((int)coll);
    PassGraph g_rev, g_fwd;
    if (want_rev) build_pass_graph(N, L, link_dst, link_src, order_cost, stream, g_rev);
    if (want_fwd) build_pass_graph(N, L, link_src, link_dst, order_cost, stream, g_fwd);
    const uint32_t per_seed = (want_rev ? 1u : 0u) + (want_fwd ? 1u : 0u);

    // groups of seeds whose passes (one workgroup each) run in one launch
    const size_t row_bytes = (size_t)NP * 128u * 8u;
    const size_t job_bytes = (size_t)N * row_bytes + (size_t)L * 12 + sizeof(Ctl);
    const uint32_t group_seeds = (uint32_t)std::max<size_t>(1, std::min<size_t>(kSearchJobs / per_seed,
                                                                            kSearchBytes / (job_bytes * per_seed)));
    for (uint32_t s0 = 0; s0 < n_seeds; s0 += group_seeds) {
      const uint32_t ns = std::min(group_seeds, n_seeds - s0);
      const uint32_t n_jobs = ns * per_seed;
      DevBuf d_held((size_t)n_jobs * N * row_bytes), d_carry((size_t)n_jobs * L * 4),
          d_free((size_t)n_jobs * L * 8), d_ctl((size_t)n_jobs * sizeof(Ctl)), d_jobs;
      std::vector<tacos::SmallJob> jobs(n_jobs);
      for (uint32_t i = 0; i < ns; ++i) {
        for (uint32_t k = 0; k < per_seed; ++k) {
          const uint32_t j = i * per_seed + k;
          const bool rev = want_rev && k == 0;
          const PassGraph &g = rev ? g_rev : g_fwd;
          jobs[j].p = make_pass_dev(g, d_cost, chunks_per_npu, root, seeds[s0 + i], rev ? 1u : 0u, rev,
                                    d_held.as<unsigned long long>() + (size_t)j * N * (row_bytes / 8),
                                    d_carry.as<uint32_t>() + (size_t)j * L,
                                    d_free.as<unsigned long long>() + (size_t)j * L, d_ctl.as<Ctl>() + j);
          jobs[j].out_ptr = g.out_ptr.as<uint32_t>();
          jobs[j].out_dst = g.out_dst.as<uint32_t>();
          tacos::launch_init_pass(jobs[j].p, stream);
        }
      }
      HIP_TRY(hipGetLastError());
      upload(d_jobs, jobs.data(), jobs.size(), stream);
      HIP_TRY(hipStreamSynchronize(stream));
      PinnedBuf host_ctl((size_t)n_jobs * sizeof(Ctl));
      const Ctl *hc = static_cast<const Ctl *>(host_ctl.p);
      uint64_t e = 0;
      for (;;) {
        if (e >= 0xFFFFFFFEull) { g_last_error = "more than 2^32-2 spans"; return TACOS_E_OVERFLOW; }
        const uint32_t n = (uint32_t)std::min<uint64_t>(kSearchSpansPerLaunch, 0xFFFFFFFEull - e);
        HIP_TRY(tacos::launch_small_sweep_batch(d_jobs.as<tacos::SmallJob>(), n_jobs, jobs[0].p, (uint32_t)e, n,
                                                match_mode, sparse, stream));
        HIP_TRY(hipMemcpyAsync(host_ctl.p, d_ctl.p, (size_t)n_jobs * sizeof(Ctl), hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        e += n;
        bool all_done = true;
        for (uint32_t j = 0; j < n_jobs; ++j) all_done = all_done && hc[j].done != 0;
        if (all_done) break;
      }
      for (uint32_t j = 0; j < n_jobs; ++j) {
        if (hc[j].status == tacos::kStUnreachable) return TACOS_E_UNREACHABLE;
        if (hc[j].status == tacos::kStOverflow) return TACOS_E_OVERFLOW;
        if (hc[j].status == tacos::kStInternal) {
          g_last_error = "internal: matching produced a chunk id out of range";
          return TACOS_E_DEVICE;
        }
      }
      for (uint32_t i = 0; i < ns; ++i) {
        uint64_t T = 0, ev = 0;
        for (uint32_t k = 0; k < per_seed; ++k) { T += hc[i * per_seed + k].T; ev += hc[i * per_seed + k].n_events; }
        time_ps[s0 + i] = T;
        if (num_events) num_events[s0 + i] = ev;
      }
    }
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    g_last_error = "host allocation failed";
    return TACOS_E_NOMEM;
  } catch (const std::system_error &e) {  // a host thread could not be started
    g_last_error = std::string("host thread: ") + e.what();
    return TACOS_E_DEVICE;
  }
  pick_best();
  return TACOS_OK;
}

uint64_t tacos_result_collective_time_ps(const tacos_result_t *r) { return r ? r->collective_time : 0; }
uint64_t tacos_result_num_xfers(const tacos_result_t *r) { return r ? r->n_xfers : 0; }
uint64_t tacos_result_num_events(const tacos_result_t *r) { return r ? r->n_events : 0; }
uint32_t tacos_result_num_passes(const tacos_result_t *r) { return r ? (uint32_t)r->passes.size() : 0; }
uint64_t tacos_result_pass_time_ps(const tacos_result_t *r, uint32_t pass)
{
  return (r && pass < r->passes.size()) ? r->passes[pass].T : 0;
}
uint64_t tacos_result_pass_events(const tacos_result_t *r, uint32_t pass)
{
  return (r && pass < r->passes.size()) ? r->passes[pass].n_events : 0;
}
uint64_t tacos_result_digest(const tacos_result_t *r) { return r ? r->digest : 0; }
double tacos_result_kernel_ms(const tacos_result_t *r) { return r ? r->kernel_ms : 0.0; }
uint64_t tacos_result_kernel_launches(const tacos_result_t *r) { return r ? r->kernel_launches : 0; }
double tacos_result_wall_ms(const tacos_result_t *r) { return r ? r->wall_ms : 0.0; }
uint64_t tacos_result_device_bytes(const tacos_result_t *r) { return r ? r->device_bytes : 0; }

int tacos_result_event_trace(const tacos_result_t *r, uint32_t pass, uint64_t *event_time_ps,
                             uint32_t *event_matches)
{
  g_last_error.clear();
  if (!r || pass >= r->passes.size()) return TACOS_E_INVAL;
  const Pass &ps = r->passes[pass];
  // The rows of a reversed pass are keyed by the span a chunk ARRIVED in, so their counts are
  // arrivals per span; the matches per span are counted from the rows once, on first use.
  if (ps.reversed && event_matches && ps.n_events && ps.start_count.empty()) {
    try {
      int prev = 0;
      HIP_TRY(hipGetDevice(&prev));
      if (prev != r->device) HIP_TRY(hipSetDevice(r->device));
      DevBuf d_time((size_t)ps.n_rows * 8), d_counts((size_t)ps.n_rows * 4);
      HIP_TRY(hipMemcpy(d_time.p, ps.row_time.data(), (size_t)ps.n_rows * 8, hipMemcpyHostToDevice));
      HIP_TRY(hipMemset(d_counts.p, 0, (size_t)ps.n_rows * 4));
      if (ps.compact) {
        tacos::launch_compact_start_span_counts(ps.recs.as<uint2>(), ps.d_first.as<uint32_t>(), (uint32_t)ps.n_rows,
                                                d_time.as<unsigned long long>(), r->d_cost.as<unsigned long long>(),
                                                d_counts.as<uint32_t>(), nullptr);
        HIP_TRY(hipGetLastError());
      }
      for (size_t k = 0; k < ps.segs.size(); ++k) {
        const uint64_t first = (uint64_t)k * ps.rows_per_seg;
        if (first >= ps.n_rows) break;
        const uint32_t n = (uint32_t)std::min<uint64_t>(ps.rows_per_seg, ps.n_rows - first);
        tacos::launch_start_span_counts(ps.segs[k].rows.as<uint32_t>(), (uint32_t)first, n, ps.L,
                                        d_time.as<unsigned long long>(), r->d_cost.as<unsigned long long>(),
                                        d_counts.as<uint32_t>(), nullptr);
        HIP_TRY(hipGetLastError());
      }
      std::vector<uint32_t> counts(ps.n_rows);
      HIP_TRY(hipMemcpy(counts.data(), d_counts.p, (size_t)ps.n_rows * 4, hipMemcpyDeviceToHost));
      if (prev != r->device) HIP_TRY(hipSetDevice(prev));
      ps.start_count.swap(counts);
    } catch (const HipFail &f) {
      return f.code;
    } catch (const std::bad_alloc &) {
      return TACOS_E_NOMEM;
    }
  }
  // spans 0 .. E-1 of the pass, in the pass's own time (a reversed pass runs from its t = 0)
  for (uint64_t i = 0; i < ps.n_events; ++i) {
    if (event_time_ps) event_time_ps[i] = ps.row_time[i];
    if (event_matches) event_matches[i] = ps.reversed ? ps.start_count[i] : ps.row_count[i];
  }
  return TACOS_OK;
}

int tacos_result_read(const tacos_result_t *r, uint64_t first, uint64_t count, tacos_xfer_t *host_out)
{
  g_last_error.clear();
  if (!r || (count && !host_out)) return TACOS_E_INVAL;
  if (first > r->n_xfers || count > r->n_xfers - first) return TACOS_E_INVAL;
  if (count == 0) return TACOS_OK;
  try {
    int prev = 0;
    HIP_TRY(hipGetDevice(&prev));
    if (prev != r->device) HIP_TRY(hipSetDevice(r->device));
    std::vector<uint32_t> stage;
    uint64_t written = 0;
    uint64_t pass_base = 0;
    for (const Pass &ps : r->passes) {
      const uint64_t lo = std::max(first, pass_base), hi = std::min(first + count, pass_base + ps.n_xfers);
      if (lo < hi) {
        const uint64_t lfirst = lo - pass_base, lend = hi - pass_base;
        // first canonical row holding record lfirst
        uint64_t k = (uint64_t)(std::upper_bound(ps.canon_base.begin(), ps.canon_base.end(), lfirst) -
                                ps.canon_base.begin()) - 1;
        // last canonical row (exclusive) that holds a record below lend
        const uint64_t k_end = (uint64_t)(std::lower_bound(ps.canon_base.begin(), ps.canon_base.end(), lend) -
                                          ps.canon_base.begin());
        if (ps.compact) {
          // the spans of canonical rows [k, k_end) are consecutive (descending for a reversed
          // pass), so their records are one range of the record array
          const uint64_t e_a = ps.event_of(k), e_b = ps.event_of(k_end - 1);
          const uint64_t e_lo = std::min(e_a, e_b), e_hi = std::max(e_a, e_b) + 1;
          const uint32_t r_lo = ps.first[e_lo], r_hi = ps.first[e_hi];
          std::vector<uint2> recs_host((size_t)(r_hi - r_lo));
          if (r_hi > r_lo)
            HIP_TRY(hipMemcpy(recs_host.data(), ps.recs.as<uint2>() + r_lo, (size_t)(r_hi - r_lo) * 8, hipMemcpyDeviceToHost));
          for (uint64_t kk = k; kk < k_end; ++kk) {
            const uint64_t ee = ps.event_of(kk);
            const uint64_t t = ps.time_of_event(ee);
            uint64_t idx = ps.canon_base[kk];
            for (uint32_t i = ps.first[ee]; i < ps.first[ee + 1] && idx < lend; ++i, ++idx) {
              if (idx < lfirst) continue;
              const uint2 rc = recs_host[i - r_lo];
              tacos_xfer_t &x = host_out[written++];
              x.t_ps = t; x.src = r->link_src[rc.x]; x.dst = r->link_dst[rc.x]; x.chunk = rc.y; x.link = rc.x;
            }
          }
          pass_base += ps.n_xfers;
          continue;
        }
        const uint64_t block_rows = std::max<uint64_t>(1, (64ull << 20) / ((uint64_t)ps.L * 4));
        while (k < k_end) {
          // a block of canonical rows that is contiguous in one segment
          const uint64_t e = ps.event_of(k);
          const uint64_t seg = e / ps.rows_per_seg;
          uint64_t n = std::min(block_rows, k_end - k);
          uint64_t e_lo;
          if (!ps.reversed) {
            n = std::min(n, (seg + 1) * ps.rows_per_seg - e);
            e_lo = e;
          } else {
            n = std::min(n, e - seg * ps.rows_per_seg + 1);
            e_lo = e - n + 1;
          }
          stage.resize((size_t)n * ps.L);
          HIP_TRY(hipMemcpy(stage.data(),
                            ps.segs[seg].rows.as<uint32_t>() + (e_lo - seg * ps.rows_per_seg) * ps.L,
                            (size_t)n * ps.L * 4, hipMemcpyDeviceToHost));
          for (uint64_t q = 0; q < n; ++q) {
            const uint64_t kk = k + q, ee = ps.event_of(kk);
            if (ps.row_count[ee] == 0) continue;
            const uint32_t *row = stage.data() + (ee - e_lo) * ps.L;
            const uint64_t t = ps.time_of_event(ee);
            uint64_t idx = ps.canon_base[kk];
            for (uint32_t l = 0; l < ps.L && idx < lend; ++l) {
              const uint32_t c = row[l];
              if (c == TACOS_NO_CHUNK) continue;
              if (idx >= lfirst) {
                tacos_xfer_t &x = host_out[written++];
                x.t_ps = t; x.src = r->link_src[l]; x.dst = r->link_dst[l]; x.chunk = c; x.link = l;
              }
              idx++;
            }
          }
          k += n;
        }
      }
      pass_base += ps.n_xfers;
    }
    if (prev != r->device) HIP_TRY(hipSetDevice(prev));
    if (written != count) { g_last_error = "internal: window size mismatch"; return TACOS_E_DEVICE; }
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    return TACOS_E_NOMEM;
  }
  return TACOS_OK;
}

int tacos_result_link_counts(const tacos_result_t *r, uint32_t pass, uint64_t *link_counts)
{
  g_last_error.clear();
  if (!r || pass >= r->passes.size() || (r->L && !link_counts)) return TACOS_E_INVAL;
  const Pass &ps = r->passes[pass];
  if (r->L == 0) return TACOS_OK;
  try {
    int prev = 0;
    HIP_TRY(hipGetDevice(&prev));
    if (prev != r->device) HIP_TRY(hipSetDevice(r->device));
    DevBuf d_counts((size_t)r->L * 8);
    HIP_TRY(hipMemset(d_counts.p, 0, (size_t)r->L * 8));
    if (ps.compact) tacos::launch_compact_link_counts(ps.recs.as<uint2>(), (uint32_t)ps.n_rec, d_counts.as<unsigned long long>(), nullptr);
    for (size_t k = 0; k < ps.segs.size(); ++k) {
      const uint64_t first = (uint64_t)k * ps.rows_per_seg;
      if (first >= ps.n_rows) break;
      const uint32_t n = (uint32_t)std::min<uint64_t>(ps.rows_per_seg, ps.n_rows - first);
      tacos::launch_link_counts(ps.segs[k].rows.as<uint32_t>(), n, ps.L, d_counts.as<unsigned long long>(),
                                nullptr);
      HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipMemcpy(link_counts, d_counts.p, (size_t)r->L * 8, hipMemcpyDeviceToHost));
    if (prev != r->device) HIP_TRY(hipSetDevice(prev));
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    return TACOS_E_NOMEM;
  }
  return TACOS_OK;
}

int tacos_result_link_busy(const tacos_result_t *r, uint32_t pass, uint64_t *busy_ps, uint64_t *sum_ps,
                           uint64_t *min_ps, uint64_t *max_ps)
{
  g_last_error.clear();
  if (!r || pass >= r->passes.size()) return TACOS_E_INVAL;
  const Pass &ps = r->passes[pass];
  if (r->L == 0 || (ps.segs.empty() && !ps.compact)) {
    if (busy_ps) std::fill(busy_ps, busy_ps + r->L, 0ull);
    if (sum_ps) *sum_ps = 0;
    if (min_ps) *min_ps = 0;
    if (max_ps) *max_ps = 0;
    return TACOS_OK;
  }
  try {
    int prev = 0;
    HIP_TRY(hipGetDevice(&prev));
    if (prev != r->device) HIP_TRY(hipSetDevice(r->device));
    DevBuf d_counts((size_t)r->L * 8), d_busy((size_t)r->L * 8), d_out(3 * 8), d_flags(4);
    HIP_TRY(hipMemset(d_counts.p, 0, (size_t)r->L * 8));
    HIP_TRY(hipMemset(d_flags.p, 0, 4));
    if (ps.compact) tacos::launch_compact_link_counts(ps.recs.as<uint2>(), (uint32_t)ps.n_rec, d_counts.as<unsigned long long>(), nullptr);
    for (size_t k = 0; k < ps.segs.size(); ++k) {
      const uint64_t first = (uint64_t)k * ps.rows_per_seg;
      if (first >= ps.n_rows) break;
      const uint32_t n = (uint32_t)std::min<uint64_t>(ps.rows_per_seg, ps.n_rows - first);
      tacos::launch_link_counts(ps.segs[k].rows.as<uint32_t>(), n, ps.L, d_counts.as<unsigned long long>(), nullptr);
    }
    tacos::launch_link_busy(r->L, d_counts.as<unsigned long long>(), r->d_cost.as<unsigned long long>(),
                            d_busy.as<unsigned long long>(), d_out.as<unsigned long long>(), d_flags.as<uint32_t>(),
                            nullptr);
    HIP_TRY(hipGetLastError());
    uint64_t out3[3] = {0, 0, 0};
    uint32_t flags = 0;
    HIP_TRY(hipMemcpy(out3, d_out.p, sizeof out3, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(&flags, d_flags.p, 4, hipMemcpyDeviceToHost));
    if (busy_ps) HIP_TRY(hipMemcpy(busy_ps, d_busy.p, (size_t)r->L * 8, hipMemcpyDeviceToHost));
    if (prev != r->device) HIP_TRY(hipSetDevice(prev));
    if (flags & tacos::kRepOverflow) return TACOS_E_OVERFLOW;
    if (sum_ps) *sum_ps = out3[0];
    if (min_ps) *min_ps = out3[1];
    if (max_ps) *max_ps = out3[2];
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    return TACOS_E_NOMEM;
  }
  return TACOS_OK;
}

int tacos_unwind_switch(uint32_t n_npus, uint32_t degree, uint64_t alpha_ps, uint64_t beta_fs_per_B,
                        uint32_t *row_ptr, uint32_t *col_idx, uint64_t *alpha_out, uint64_t *beta_out)
{
  g_last_error.clear();
  if (!row_ptr || !col_idx || !alpha_out || !beta_out || n_npus < 2 || degree < 1 || degree > n_npus - 1)
    return TACOS_E_INVAL;
  const uint64_t n_links = (uint64_t)n_npus * degree;
  if (n_links > 0xFFFFFFFEull) return TACOS_E_INVAL;
  if (beta_fs_per_B != 0 && degree > ~0ull / beta_fs_per_B) return TACOS_E_OVERFLOW;
  int dev = 0;
  const int rc = require_device(&dev);
  if (rc != TACOS_OK) return rc;
  try {
    DevBuf d_ptr(((size_t)n_npus + 1) * 4), d_col(n_links * 4), d_alpha(n_links * 8), d_beta(n_links * 8);
    tacos::launch_unwind_switch(n_npus, degree, alpha_ps, beta_fs_per_B * degree, d_ptr.as<uint32_t>(),
                                d_col.as<uint32_t>(), d_alpha.as<unsigned long long>(),
                                d_beta.as<unsigned long long>(), nullptr);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpy(row_ptr, d_ptr.p, ((size_t)n_npus + 1) * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(col_idx, d_col.p, n_links * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(alpha_out, d_alpha.p, n_links * 8, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(beta_out, d_beta.p, n_links * 8, hipMemcpyDeviceToHost));
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    return TACOS_E_NOMEM;
  }
  return TACOS_OK;
}

int tacos_ideal_bound(const tacos_topology_t *topo, uint32_t chunks_per_npu, uint64_t chunk_bytes,
                      tacos_collective_t coll, uint32_t with_diameter, tacos_ideal_t *out)
{
  g_last_error.clear();
  if (!out) return TACOS_E_INVAL;
  int rc = validate(topo, chunks_per_npu, chunk_bytes, (int)coll, nullptr);
  if (rc != TACOS_OK) return rc;
  if (is_rooted((int)coll)) return TACOS_E_INVAL;
  const uint32_t N = topo->n_npus, L = topo->n_links;
  if (with_diameter && N > TACOS_IDEAL_MAX_DIAMETER_NPUS) {
    g_last_error = "tacos_ideal_bound: the latency diameter is computed for at most TACOS_IDEAL_MAX_DIAMETER_NPUS NPUs";
    return TACOS_E_INVAL;
  }
  // CollectiveSize and the bytes every NPU receives (sends): (n - 1) * chunks_per_npu * chunk_bytes
  const unsigned __int128 size = (unsigned __int128)N * chunks_per_npu * chunk_bytes;
  const unsigned __int128 moved = (unsigned __int128)(N - 1) * chunks_per_npu * chunk_bytes;
  if (size >> 64) return TACOS_E_OVERFLOW;
  tacos_ideal_t res{};
  res.collective_bytes = (uint64_t)size;
  if (N == 1) { *out = res; return TACOS_OK; }
  if (L == 0) return TACOS_E_UNREACHABLE;
  int dev = 0;
  rc = require_device(&dev);
  if (rc != TACOS_OK) return rc;
  try {
    // the links by destination (in-lists) next to the CSR by source: input marshalling
    std::vector<uint32_t> src(L), in_ptr(N + 1, 0);
    std::vector<uint64_t> in_beta(L);
    for (uint32_t i = 0; i < N; ++i)
      for (uint32_t l = topo->row_ptr[i]; l < topo->row_ptr[i + 1]; ++l) { src[l] = i; in_ptr[topo->col_idx[l] + 1]++; }
    for (uint32_t d = 0; d < N; ++d) in_ptr[d + 1] += in_ptr[d];
    {
      std::vector<uint32_t> fill(in_ptr.begin(), in_ptr.end() - 1);
      for (uint32_t l = 0; l < L; ++l) in_beta[fill[topo->col_idx[l]]++] = topo->beta_fs_per_B[l];
    }
    DevBuf d_in_ptr, d_in_beta, d_out_ptr, d_out_beta, d_P((size_t)N * 8), d_Q((size_t)N * 8), d_res(4 * 8), d_flags(4);
    upload(d_in_ptr, in_ptr.data(), in_ptr.size(), nullptr);
    upload(d_in_beta, reinterpret_cast<const unsigned long long *>(in_beta.data()), in_beta.size(), nullptr);
    upload(d_out_ptr, topo->row_ptr, (size_t)N + 1, nullptr);
    upload(d_out_beta, reinterpret_cast<const unsigned long long *>(topo->beta_fs_per_B), (size_t)L, nullptr);
    HIP_TRY(hipMemset(d_flags.p, 0, 4));
    HIP_TRY(hipMemset(d_res.p, 0, 4 * 8));
    const bool rs = has_reversed_pass((int)coll), ag = has_forward_pass((int)coll);
    int n_pass = 0;
    unsigned long long *res_dev = d_res.as<unsigned long long>();
    if (rs) {  // every NPU sends: egress side
      tacos::launch_bandwidth_term(N, d_out_ptr.as<uint32_t>(), d_out_beta.as<unsigned long long>(), (uint64_t)moved,
                                   d_P.as<unsigned long long>(), d_Q.as<unsigned long long>(), res_dev + 2 * n_pass,
                                   d_flags.as<uint32_t>(), nullptr);
      n_pass++;
    }
    if (ag) {  // every NPU receives: ingress side
      tacos::launch_bandwidth_term(N, d_in_ptr.as<uint32_t>(), d_in_beta.as<unsigned long long>(), (uint64_t)moved,
                                   d_P.as<unsigned long long>(), d_Q.as<unsigned long long>(), res_dev + 2 * n_pass,
                                   d_flags.as<uint32_t>(), nullptr);
      n_pass++;
    }
    HIP_TRY(hipGetLastError());
    DevBuf d_src, d_dst, d_alpha, d_diam(8);
    HIP_TRY(hipMemset(d_diam.p, 0, 8));
    if (with_diameter) {
      upload(d_src, src.data(), src.size(), nullptr);
      upload(d_dst, topo->col_idx, (size_t)L, nullptr);
      upload(d_alpha, reinterpret_cast<const unsigned long long *>(topo->alpha_ps), (size_t)L, nullptr);
      HIP_TRY(tacos::launch_latency_diameter(N, L, d_src.as<uint32_t>(), d_dst.as<uint32_t>(),
                                             d_alpha.as<unsigned long long>(), d_diam.as<unsigned long long>(),
                                             d_flags.as<uint32_t>(), nullptr));
    }
    uint64_t host_res[4] = {0, 0, 0, 0}, diam = 0;
    uint32_t flags = 0;
    HIP_TRY(hipMemcpy(host_res, d_res.p, sizeof host_res, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(&diam, d_diam.p, 8, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(&flags, d_flags.p, 4, hipMemcpyDeviceToHost));
    if (flags & tacos::kRepNoLink) return TACOS_E_UNREACHABLE;
    if (flags & tacos::kRepOverflow) return TACOS_E_OVERFLOW;
    for (int i = 0; i < n_pass; ++i) {
      res.pass_bandwidth_term_ps[i] = host_res[2 * i];
      res.pass_bottleneck_npu[i] = (uint32_t)host_res[2 * i + 1];
      if (res.bandwidth_term_ps + host_res[2 * i] < res.bandwidth_term_ps) return TACOS_E_OVERFLOW;
      res.bandwidth_term_ps += host_res[2 * i];
    }
    res.diameter_ps = diam;
    if (res.bandwidth_term_ps + diam < diam) return TACOS_E_OVERFLOW;
    res.ideal_ps = res.bandwidth_term_ps + diam;
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    return TACOS_E_NOMEM;
  }
  *out = res;
  return TACOS_OK;
}

void tacos_result_free(tacos_result_t *r)
{
  if (!r) return;
  int prev = 0;
  const int dev = r->device;
  const bool have = hipGetDevice(&prev) == hipSuccess;
  if (have && prev != dev) (void)hipSetDevice(dev);
  delete r;
  if (have && prev != dev) (void)hipSetDevice(prev);
}

int tacos_link_costs(const tacos_topology_t *topo, uint64_t chunk_bytes, uint64_t *cost_ps)
{
  g_last_error.clear();
  if (!topo || chunk_bytes == 0 || (topo->n_links && (!cost_ps || !topo->alpha_ps || !topo->beta_fs_per_B)))
    return TACOS_E_INVAL;
  int dev = 0;
  int rc = require_device(&dev);
  if (rc != TACOS_OK) return rc;
  if (topo->n_links == 0) return TACOS_OK;
  try {
    DevBuf d_cost;
    std::vector<uint64_t> host;
    rc = device_costs(topo, chunk_bytes, nullptr, d_cost, &host);
    if (rc != TACOS_OK) return rc;
    std::memcpy(cost_ps, host.data(), host.size() * 8);
  } catch (const HipFail &f) {
    return f.code;
  } catch (const std::bad_alloc &) {
    return TACOS_E_NOMEM;
  }
  return TACOS_OK;
}

int tacos_link_costs_static(const tacos_topology_t *topo, uint64_t chunk_bytes, uint64_t *cost_ps)
{
  g_last_error.clear();
  if (!topo || chunk_bytes == 0 || (topo->n_links && (!cost_ps || !topo->alpha_ps || !topo->beta_fs_per_B)))
    return TACOS_E_INVAL;
  if (topo->n_links > TACOS_STATIC_MAX_LINKS) {
    g_last_error = "tacos_link_costs_static: more than TACOS_STATIC_MAX_LINKS links";
    return TACOS_E_INVAL;
  }
  int dev = 0;
  const int rc = require_device(&dev);
  if (rc != TACOS_OK) return rc;
  if (topo->n_links == 0) return TACOS_OK;
  static_assert(TACOS_STATIC_MAX_LINKS == tacos::kStaticMaxLinks, "header and kernels disagree");
  uint32_t overflow = 0;
  const hipError_t e = tacos::link_cost_static(reinterpret_cast<const unsigned long long *>(topo->alpha_ps),
                                               reinterpret_cast<const unsigned long long *>(topo->beta_fs_per_B),
                                               chunk_bytes, topo->n_links,
                                               reinterpret_cast<unsigned long long *>(cost_ps), &overflow, nullptr);
  if (e != hipSuccess) {
    char buf[256];
    std::snprintf(buf, sizeof buf, "tacos_link_costs_static failed: %s", hipGetErrorString(e));
    g_last_error = buf;  // a fixed-size message: this entry point allocates nothing on the device
    (void)hipGetLastError();
    return TACOS_E_DEVICE;
  }
  return overflow ? TACOS_E_OVERFLOW : TACOS_OK;
}

const char *tacos_strerror(int code)
{
  switch (code) {
    case TACOS_OK: return "success";
    case TACOS_E_INVAL: return "invalid argument";
    case TACOS_E_UNREACHABLE: return "topology not strongly connected: chunks missing and nothing in flight";
    case TACOS_E_OVERFLOW: return "a link cost or a time does not fit 64 bits";
    case TACOS_E_NOMEM: return "out of host or device memory";
    case TACOS_E_DEVICE: return "no HIP device or a HIP call failed";
    default: return "unknown error code";
  }
}

const char *tacos_last_error(void) { return g_last_error.c_str(); }

const char *tacos_version(void) { return "tacos-mi355x 0.1 (gfx950)"; }

}  // extern "C"
