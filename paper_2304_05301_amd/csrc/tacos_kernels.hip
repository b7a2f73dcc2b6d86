// HIP kernels (gfx950, wave64) of the TACOS synthesis hot path.
//
// Paper: TACOS, arXiv 2304.05301.  One TEN span ("event") is processed by two launches:
//   arrive_kernel : the precondition update for the span (chunks whose transfer ends now
//                   become held), one thread per link; also the span's random words;
//   match_kernel  : Algorithm 1 (utilization-maximizing matching) in its link-centric
//                   deterministic form (or, MODE 1/2, in the postcondition-centric order
//                   the paper prints), one wavefront per destination NPU, plus the
//                   min-reduction that finds the next span of Algorithm 2.
// The host never sees the per-event state; it only queues launches and polls the
// control block once per batch of events.
// Small topologies: small_sweep_kernel, ONE workgroup that sweeps many spans with the
// link state in LDS; small_sweep_batch_kernel runs many such passes (seeds) at once.
//
// All arithmetic is integer.  Bitset layout: see PassDev in tacos_internal.h.

#include "tacos_internal.h"

#include <mutex>
#include <type_traits>

namespace tacos {

namespace {

typedef unsigned long long u64;
typedef uint32_t u32;

// Loads and stores with the address space spelled out.  The single-workgroup kernel keeps
// some arrays either in LDS or in device memory, decided at launch; through a generic
// pointer such an access becomes a FLAT instruction, and on gfx9 every wait for a flat load
// is s_waitcnt vmcnt(0) lgkmcnt(0): it also waits for all global loads, stores and atomics
// in flight, which is exactly what that kernel avoids.  With these, an LDS access is a ds_
// instruction and a device-memory access a global_ one.
#define TACOS_LDS __attribute__((address_space(3)))
#define TACOS_GLB __attribute__((address_space(1)))
typedef u32 u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32 lds_ld(const u32 *p) { return *(const TACOS_LDS u32 *)p; }
__device__ __forceinline__ u32 lds_ld(const unsigned short *p) { return *(const TACOS_LDS unsigned short *)p; }
__device__ __forceinline__ unsigned long long lds_ld(const unsigned long long *p)
{
  return *(const TACOS_LDS unsigned long long *)p;
}
__device__ __forceinline__ uint4 lds_ld(const uint4 *p)
{
  const u32x4_t v = *(const TACOS_LDS u32x4_t *)p;
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void lds_st(u32 *p, u32 v) { *(TACOS_LDS u32 *)p = v; }
__device__ __forceinline__ void lds_st(unsigned long long *p, unsigned long long v)
{
  *(TACOS_LDS unsigned long long *)p = v;
}
__device__ __forceinline__ u32 glb_ld(const u32 *p) { return *(const TACOS_GLB u32 *)p; }
__device__ __forceinline__ uint4 glb_ld(const uint4 *p)
{
  const u32x4_t v = *(const TACOS_GLB u32x4_t *)p;
  return make_uint4(v.x, v.y, v.z, v.w);
}
// link state and control block: in LDS for the single-workgroup kernel (IN_LDS), else in device memory
template <bool IN_LDS, class T> __device__ __forceinline__ auto state_ld(const T *p)
{
  if constexpr (IN_LDS) return lds_ld(p);
  else return *p;
}
template <bool IN_LDS, class T, class V> __device__ __forceinline__ void state_st(T *p, V v)
{
  if constexpr (IN_LDS) lds_st(p, (T)v);
  else *p = (T)v;
}

// ---------------------------------------------------------------- small helpers

__device__ __forceinline__ u32 uniform(u32 v) { return (u32)__builtin_amdgcn_readfirstlane((int)v); }

__device__ __forceinline__ u32 read_lane(u32 v, u32 lane)
{
  return (u32)__builtin_amdgcn_readlane((int)v, (int)lane);
}

// Inclusive prefix sum over the 64 lanes of a wavefront with DPP adds: a Hillis-Steele
// scan inside each row of 16 lanes (row_shr 1,2,4,8, zero fill), then lane 15 of rows 0/2
// is added to rows 1/3 (row_bcast:15) and lane 31 to rows 2 and 3 (row_bcast:31).
__device__ __forceinline__ u32 wave_inclusive_scan(u32 v)
{
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);
  v += (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);
  return v;
}

// Minimum over the 64 lanes (uniform result) with DPP moves: a reduction towards the last
// lane of each row of 16 (row_shr 1,2,4,8), then across rows (row_bcast:15, row_bcast:31);
// lanes a move does not reach keep the identity (all ones).  The result is read from lane 63.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ u64 dpp_min_step(u64 v)
{
  const u32 lo = (u32)__builtin_amdgcn_update_dpp(-1, (int)(u32)v, CTRL, ROW_MASK, 0xF, false);
  const u32 hi = (u32)__builtin_amdgcn_update_dpp(-1, (int)(u32)(v >> 32), CTRL, ROW_MASK, 0xF, false);
  const u64 o = ((u64)hi << 32) | lo;
  return o < v ? o : v;
}

__device__ __forceinline__ u64 wave_min64(u64 v)
{
  v = dpp_min_step<0x111, 0xF>(v);
  v = dpp_min_step<0x112, 0xF>(v);
  v = dpp_min_step<0x114, 0xF>(v);
  v = dpp_min_step<0x118, 0xF>(v);
  v = dpp_min_step<0x142, 0xA>(v);
  v = dpp_min_step<0x143, 0xC>(v);
  return ((u64)read_lane((u32)(v >> 32), 63) << 32) | read_lane((u32)v, 63);
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), word 0 of the output block.
__device__ __forceinline__ u32 philox4x32_10_word0(u32 c0, u32 c1, u32 c2, u32 c3, u32 k0, u32 k1)
{
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const u32 lo0 = 0xD2511F53u * c0, hi0 = __umulhi(0xD2511F53u, c0);
    const u32 lo1 = 0xCD9E8D57u * c2, hi1 = __umulhi(0xCD9E8D57u, c2);
    const u32 n0 = hi1 ^ c1 ^ k0;
    const u32 n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

// Physical 64-bit word index inside a row of logical bitset word w (lane-major layout).
__device__ __forceinline__ u32 phys_word(u32 w, u32 NP)
{
  const u32 nw = 2u * NP;
  const u32 ln = w / nw;
  const u32 idx = w - ln * nw;
  return (idx >> 1) * 128u + ln * 2u + (idx & 1u);
}

// ---------------------------------------------------------------- a1: link cost

// cost = alpha + (beta*bytes + 500)/1000 with a 128-bit intermediate.
__global__ void link_cost_kernel(const u64 *__restrict__ alpha, const u64 *__restrict__ beta,
                                 u64 chunk_bytes, u32 L, u64 *__restrict__ cost,
                                 u32 *__restrict__ overflow)
{
  const u32 l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= L) return;
  const u64 b = beta[l];
  u64 lo = b * chunk_bytes;
  u64 hi = __umul64hi(b, chunk_bytes);
  const u64 lo2 = lo + 500ull;
  if (lo2 < lo) hi += 1ull;
  lo = lo2;
  // (hi:lo) / 1000 by long division over 32-bit digits
  bool ovf = false;
  const u64 q3 = hi / 1000ull;            // would land above bit 63
  u64 rem = hi % 1000ull;
  if (q3 != 0) ovf = true;
  u64 cur = (rem << 32) | (lo >> 32);
  const u64 q1 = cur / 1000ull;
  rem = cur % 1000ull;
  cur = (rem << 32) | (lo & 0xFFFFFFFFull);
  const u64 q0 = cur / 1000ull;
  if (q1 >> 32) ovf = true;
  const u64 q = (q1 << 32) + q0;
  const u64 c = q + alpha[l];
  if (c < q || c == kInf) ovf = true;
  cost[l] = c;
  if (ovf) atomicOr(overflow, 1u);
}

// ---------------------------------------------------------------- a2: initial state

__global__ void init_rows_kernel(PassDev p)
{
  // one thread per physical 64-bit word of the held table
  const u64 gid = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  const u64 total = (u64)p.N * p.row_words;
  if (gid >= total) return;
  const u32 npu = (u32)(gid / p.row_words);
  const u32 ph = (u32)(gid - (u64)npu * p.row_words);
  const u32 piece = ph >> 7, ln = (ph & 127u) >> 1, half = ph & 1u;
  const u32 w = ln * 2u * p.NP + piece * 2u + half;  // logical word
  const u64 c0 = (u64)w * 64ull;
  // chunks the NPU holds at t = 0: [own_lo, own_hi)
  u64 own_lo = (u64)npu * p.cpn, own_hi = own_lo + p.cpn;
  if (p.root != kNoRoot) { own_lo = 0; own_hi = npu == p.root ? p.C : 0; }
  u64 bits = 0;
  for (u32 b = 0; b < 64; ++b) {
    const u64 c = c0 + b;
    if (c >= p.C || (c >= own_lo && c < own_hi)) bits |= 1ull << b;
  }
  p.held[gid] = bits;
}

__global__ void init_links_kernel(PassDev p)
{
  const u32 l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l < p.L) {
    p.carry[l] = kNone; p.free_at[l] = 0ull;
    // entry l of the in-lists gathered into one 16-byte record
    const u32 lk = p.in_link[l];
    const u64 cs = p.cost[lk];
    p.in_rec[l] = make_uint4(lk, p.in_src[l], (u32)cs, (u32)(cs >> 32));
  }
  if (l == 0) {
    Ctl *c = p.ctl;
    c->next_t[0] = 0ull;
    c->next_t[1] = kInf;
    c->remaining = (u64)p.N * p.C - p.C;
    c->T = 0ull;
    c->done = 0u;
    c->status = 0u;
    c->n_events = 0u;
    c->n_rec = 0u;
    c->now = 0ull;
    for (int i = 0; i < 4; ++i) { c->need_flag[i] = 0u; c->match_flag[i] = 0u; }
  }
  if (p.next_slots && l < 2u * kNextSlots) p.next_slots[l] = l == 0u ? 0ull : kInf;  // span 0 is at time 0
}

// Compact schedule records: (link, chunk) pairs appended in the order the spans are swept, at a
// record counter (in LDS for the single-workgroup kernel, Ctl::n_rec for the per-span launches on
// topologies whose links nearly all cost differently).  Null where the schedule is dense rows.
struct RecOut {
  uint2 *recs = nullptr;
  u32 *counter = nullptr;
};

// appends the lanes' records (lanes with has == true) behind one another
__device__ __forceinline__ void append_records(const RecOut &rec, bool has, u32 link, u32 chunk, int lane)
{
  const u64 m = __ballot(has);
  if (m == 0ull) return;
  const u32 first = (u32)__ffsll((long long)m) - 1u;
  u32 base = 0;
  if ((u32)lane == first) base = atomicAdd(rec.counter, (u32)__popcll(m));
  base = read_lane(base, first);
  if (has) rec.recs[base + (u32)__popcll(m & ((1ull << lane) - 1ull))] = make_uint2(link, chunk);
}

// ---------------------------------------------------------------- a3: arrivals

// The time of span `event`: the minimum of the words the matching of the span before reduced into
// (all of them, or only the first one: PassDev::next_mask).  Wave-uniform; all 64 lanes call it.
__device__ __forceinline__ u64 next_event_time(const PassDev &p, u32 event)
{
  const u64 *w = p.next_slots + (event & 1u) * kNextSlots;
  if (p.next_mask == 0u) return w[0];
  return wave_min64(w[threadIdx.x & 63u]);
}

// Compact schedules (recs != null; see RecOut): a reversed pass appends its arrivals as (link,
// chunk) records at ctl->n_rec; first_slot, if not null, receives the index of the span's first
// record (forward pass: the matching kernel appends the span's matches after this launch).
__global__ __launch_bounds__(256) void arrive_kernel(PassDev p, u32 event, u64 *event_time_slot,
                                                     u32 *__restrict__ sched_row, uint2 *__restrict__ recs,
                                                     u32 *__restrict__ first_slot)
{
  Ctl *ctl = p.ctl;
  // one thread per in-list position (the per-link state is kept in in-list order)
  const u32 l = blockIdx.x * 256u + threadIdx.x;
  // the link's state does not depend on the control block: have all loads in flight at once
  u32 c = kNone, d = 0, link = 0;
  u64 fa = 0;
  if (l < p.L) {
    c = p.carry[l]; fa = p.free_at[l]; d = p.pos_dst[l];
    if (sched_row || recs || p.rnd) link = p.in_link[l];
  }
  if (ctl->done) return;
  // the span's time: the earliest end of a transfer in flight (a8), reduced over the slots the
  // matching of the previous span min-reduced into
  const u64 t = next_event_time(p, event);
  if (blockIdx.x == 0 && threadIdx.x < kNextSlots) p.next_slots[((event + 1u) & 1u) * kNextSlots + threadIdx.x] = kInf;
  if (l == 0) {
    if (first_slot) *first_slot = ctl->n_rec;
    ctl->next_t[event & 1u] = t;
    if (t == kInf) {
      // a4 / a8: nothing is in flight after the previous span's matching.  If no destination
      // needed a chunk there, every postcondition is satisfied and the collective ended at
      // that span's time; else the topology is not strongly connected.
      if (event != 0u && ctl->need_flag[(event - 1u) & 1u] == 0u) {
        ctl->T = ctl->now;
        ctl->n_events = event - 1u;
      } else {
        ctl->status = kStUnreachable;
      }
      ctl->done = 1u;
    } else {
      *event_time_slot = t;
      ctl->now = t;
      ctl->next_t[(event + 1u) & 1u] = kInf;
      ctl->need_flag[event & 1u] = 0u;
    }
  }
  if (t == kInf) return;
  // a6, first half: this span's random word of every link (the matching kernel takes it
  // modulo the number of candidates); here all 64 lanes of a wavefront are in use
  if (p.rnd && l < p.L) p.rnd[l] = philox4x32_10_word0(link, event, p.phase, 0u, p.seed_lo, p.seed_hi);
  const bool arrived = (c != kNone) && (fa == t);
  if (arrived) {
    atomicOr(&p.held[(u64)d * p.row_words + phys_word(c >> 6, p.NP)], 1ull << (c & 63u));
    p.carry[l] = kNone;
  }
  if (sched_row && arrived) sched_row[link] = c;  // rows are pre-filled with kNone
  if (recs) append_records(RecOut{recs, &ctl->n_rec}, arrived, link, c, (int)(threadIdx.x & 63u));
}

// The same for the in-lists of the destinations still in the processing order only: once the
// host has dropped the complete destinations (nothing is or will be in flight to them, so
// their links never deliver again), a thread per (slot, position in the in-list), deg
// positions per slot.  On the meshes of the paper's scalability experiment the last third of
// a pass has a handful of active destinations among tens of thousands.
__global__ __launch_bounds__(256) void arrive_slots_kernel(PassDev p, u32 event, u64 *event_time_slot,
                                                           u32 *__restrict__ sched_row, uint2 *__restrict__ recs,
                                                           u32 *__restrict__ first_slot, u32 deg)
{
  Ctl *ctl = p.ctl;
  const u32 q = blockIdx.x * 256u + threadIdx.x;
  const u32 slot = q / deg, k = q - slot * deg;
  u32 c = kNone, d = 0, link = 0, j = 0;
  u64 fa = 0;
  bool valid = false;
  if (slot < p.n_slots) {
    const uint4 sr = p.slot_rec[slot];  // (destination, in-list begin, end)
    j = sr.y + k;
    if (j < sr.z) {
      valid = true;
      d = sr.x;
      c = p.carry[j]; fa = p.free_at[j];
      if (sched_row || recs || p.rnd) link = p.in_link[j];
    }
  }
  if (ctl->done) return;
  const u64 t = next_event_time(p, event);  // as arrive_kernel
  if (blockIdx.x == 0 && threadIdx.x < kNextSlots) p.next_slots[((event + 1u) & 1u) * kNextSlots + threadIdx.x] = kInf;
  if (q == 0) {
    if (first_slot) *first_slot = ctl->n_rec;
    ctl->next_t[event & 1u] = t;
    if (t == kInf) {  // as arrive_kernel
      if (event != 0u && ctl->need_flag[(event - 1u) & 1u] == 0u) {
        ctl->T = ctl->now;
        ctl->n_events = event - 1u;
      } else {
        ctl->status = kStUnreachable;
      }
      ctl->done = 1u;
    } else {
      *event_time_slot = t;
      ctl->now = t;
      ctl->next_t[(event + 1u) & 1u] = kInf;
      ctl->need_flag[event & 1u] = 0u;
    }
  }
  if (t == kInf) return;
  if (p.rnd && valid) p.rnd[j] = philox4x32_10_word0(link, event, p.phase, 0u, p.seed_lo, p.seed_hi);
  const bool arrived = valid && (c != kNone) && (fa == t);
  if (arrived) {
    atomicOr(&p.held[(u64)d * p.row_words + phys_word(c >> 6, p.NP)], 1ull << (c & 63u));
    p.carry[j] = kNone;
  }
  if (sched_row && arrived) sched_row[link] = c;
  if (recs) append_records(RecOut{recs, &ctl->n_rec}, arrived, link, c, (int)(threadIdx.x & 63u));
}

// ---------------------------------------------------------------- a4-a8: matching

// A lane's share of a bitset row (NDW dwords) held in native vector registers, so that
// the compiler can index it with a wave-uniform register index (s_set_gpr_idx) instead
// of a chain of selects or branches.  Indexable vectors come in 4/8/16/32 dwords; a row
// of 17..31 dwords is split into a 16-dword part and a remainder, one of 33..64 dwords into a
// 32-dword part and a remainder, so that few registers are wasted on padding.
template <int N> struct VecOf {
  typedef u32 type __attribute__((ext_vector_type(N <= 4 ? 4 : N <= 8 ? 8 : N <= 16 ? 16 : 32)));
};
// (Two separate vector variables rather than one struct: a struct of two vectors that
// is indexed dynamically ends up in scratch memory.)
template <int NDW> struct RowRegs {
  static_assert(NDW <= 64, "a lane's share of a row is at most 64 dwords");
  static constexpr bool kSplit = NDW > 16 && NDW != 32;
  static constexpr int kCut = NDW > 32 ? 32 : 16;  // dwords in part A of a split row
  static constexpr int kA = kSplit ? kCut : NDW;
  static constexpr int kB = kSplit ? NDW - kCut : 4;  // B is unused unless split
  typedef typename VecOf<kA>::type A;
  typedef typename VecOf<kB>::type B;
  static constexpr u32 kMaskA = sizeof(A) / 4 - 1;
  static constexpr u32 kMaskB = sizeof(B) / 4 - 1;
  template <int I> static __device__ __forceinline__ u32 get(const A &a, const B &b)
  {
    if constexpr (!kSplit || I < kCut) return a[I];
    else return b[I - kCut];
  }
  template <int I> static __device__ __forceinline__ void set(A &a, B &b, u32 x)
  {
    if constexpr (!kSplit || I < kCut) a[I] = x;
    else b[I - kCut] = x;
  }
  // i is wave-uniform: both parts are indexed and the scalar condition picks one
  static __device__ __forceinline__ u32 at(const A &a, const B &b, u32 i)
  {
    if constexpr (!kSplit) return a[i];
    else {
      const u32 x = a[i & kMaskA], y = b[(i - (u32)kCut) & kMaskB];
      return i < (u32)kCut ? x : y;
    }
  }
};

// compile-time loop over the dword indices of a row
template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// popcount(x) + acc in one VALU instruction (v_bcnt accumulates); written as asm so that
// the running count stays a dependent chain whose partial sums are the in-lane prefixes.
__device__ __forceinline__ u32 popc_acc(u32 x, u32 acc)
{
  u32 r;
  asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
  return r;
}

// Position of the k-th (0-based) set bit of the wave-uniform word (hi:lo): lane i of
// the wavefront computes the rank of bit i with v_mbcnt, the lane whose bit is set and
// whose rank equals k is the answer.
__device__ __forceinline__ u32 kth_set_bit_wave(u32 lo, u32 hi, u32 k)
{
  const u32 rank = __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
  const u64 hit = __ballot(rank == k) & (((u64)hi << 32) | lo);
  return (u32)__ffsll((long long)hit) - 1u;
}

// Where the matching reads the held rows from.
// RowsHbm: the table in device memory, swizzled rows of NP KiB (see PassDev).
struct RowsHbm {
  const u64 *held;
  u32 row_words;
  __device__ __forceinline__ uint4 load(u32 npu, int piece, int lane) const
  {
    return reinterpret_cast<const uint4 *>(held + (u64)npu * row_words)[piece * 64 + lane];
  }
  __device__ __forceinline__ u32 dword(u32 npu, u32 dw) const  // dw: dword index inside the row
  {
    return reinterpret_cast<const u32 *>(held + (u64)npu * row_words)[dw];
  }
};
// RowsLds: a copy of the table in LDS (single-workgroup kernel, small chunk counts) without
// the lanes that own no chunk id below C: a row is NP pieces of `lanes` 16-byte shares; the
// shares left out are all ones ("held", never a candidate) and are synthesized on load.
struct RowsLds {
  uint4 *base;
  u32 lanes;   // lanes of a wavefront that own a chunk id < C
  u32 row_u4;  // NP * lanes
  __device__ __forceinline__ uint4 load(u32 npu, int piece, int lane) const
  {
    uint4 v = make_uint4(~0u, ~0u, ~0u, ~0u);
    if ((u32)lane < lanes) v = base[npu * row_u4 + (u32)piece * lanes + (u32)lane];
    return v;
  }
  __device__ __forceinline__ u32 dword(u32 npu, u32 dw) const
  {
    const u32 share = dw >> 2, piece = share >> 6, ln = share & 63u;
    if (ln >= lanes) return ~0u;
    return reinterpret_cast<const u32 *>(&base[npu * row_u4 + piece * lanes + ln])[dw & 3u];
  }
  // the 64-bit word that holds chunk c in row npu (c < C)
  __device__ __forceinline__ u64 *word_of(u32 npu, u32 c, u32 NP) const
  {
    const u32 w = c >> 6, nw = 2u * NP;
    const u32 ln = w / nw, iw = w - ln * nw;
    return reinterpret_cast<u64 *>(&base[npu * row_u4 + (iw >> 1) * lanes + ln]) + (iw & 1u);
  }
};

// The link-centric draws of ONE destination for up to 64 of its incoming links (one per
// lane): for every link whose bit is set in `idle`, in ascending lane order,
//   cand = held[source] & need;  p = |cand|;  nothing if p == 0;
//   the link carries the (r mod p)-th smallest chunk of cand, which leaves `need`.
// s, r: the lane's link's source NPU and random word; need_lds: the destination's need row
// (this wavefront's NP*64 uint4 of LDS), updated in place.  Returns the lane's link's chunk or
// kNone.  Source rows land in two register buffers used in turn, so that the next link's
// row is in flight while the current link is decided; the candidate set is formed in place
// in the buffer.
// pre(): called once, after the first link's row has been asked for and before anything is
// decided (r is read only after it); returns false (wave-uniform) if nothing is to be drawn.
struct DrawNow {
  __device__ __forceinline__ bool operator()() const { return true; }
};
template <int NP, class Rows, class Pre = DrawNow>
__device__ __forceinline__ u32 draw_chunks(const Rows &rows, u32 s, const u32 &r, u64 idle, uint4 *need_lds, int lane,
                                           Pre &&pre = Pre())
{
  constexpr int NW = 2 * NP;
  constexpr int NDW = 4 * NP;
  typedef RowRegs<NDW> RT;
  u32 res = kNone;
  typename RT::A buf0_a, buf1_a;
  typename RT::B buf0_b, buf1_b;
  auto fetch = [&](typename RT::A &ba, typename RT::B &bb, u64 pending) {
    const u32 src = read_lane(s, (u32)__ffsll((long long)pending) - 1u);
    static_for<0, NP>([&](auto I) {
      constexpr int i = decltype(I)::value;
      const uint4 v = rows.load(src, i, lane);
      RT::template set<4 * i>(ba, bb, v.x); RT::template set<4 * i + 1>(ba, bb, v.y);
      RT::template set<4 * i + 2>(ba, bb, v.z); RT::template set<4 * i + 3>(ba, bb, v.w);
    });
  };
  auto decide = [&](typename RT::A &ca, typename RT::B &cb, typename RT::A &na, typename RT::B &nb) {
    const u32 b = (u32)__ffsll((long long)idle) - 1u;
    idle &= idle - 1ull;
    // cand = held[src] & need in place, with the running in-lane candidate counts
    u32 pre[NW];
    u32 cnt = 0;
    static_for<0, NP>([&](auto I) {
      constexpr int i = decltype(I)::value;
      const uint4 nd = need_lds[i * 64 + lane];
      const u32 c0 = RT::template get<4 * i>(ca, cb) & nd.x;
      const u32 c1 = RT::template get<4 * i + 1>(ca, cb) & nd.y;
      const u32 c2 = RT::template get<4 * i + 2>(ca, cb) & nd.z;
      const u32 c3 = RT::template get<4 * i + 3>(ca, cb) & nd.w;
      RT::template set<4 * i>(ca, cb, c0); RT::template set<4 * i + 1>(ca, cb, c1);
      RT::template set<4 * i + 2>(ca, cb, c2); RT::template set<4 * i + 3>(ca, cb, c3);
      cnt = popc_acc(c0, cnt);
      cnt = popc_acc(c1, cnt);
      pre[2 * i] = cnt;
      cnt = popc_acc(c2, cnt);
      cnt = popc_acc(c3, cnt);
      pre[2 * i + 1] = cnt;
    });
    // pin the candidate computation ahead of the next row's loads: it waits for THIS
    // row only, and the next row's latency hides behind the selection below
    asm volatile("" ::"v"(cnt));
    if (idle) fetch(na, nb, idle);
    const u32 incl = wave_inclusive_scan(cnt);
    const u32 pop = read_lane(incl, 63);
    if (pop != 0) {
      u32 k = read_lane(r, b) % pop;
      const u64 above = __ballot(incl > k);
      const u32 ln = (u32)__ffsll((long long)above) - 1u;
      k -= read_lane(incl - cnt, ln);
      // the owning lane's word, by a scalar walk over its in-lane prefixes (a vector search of
      // every lane's own words was measured: 2 % slower, the vector unit is the busier one here)
      u32 idx = 0, before = 0;
#pragma unroll
      for (int i = 0; i < NW - 1; ++i) {
        const u32 pi = read_lane(pre[i], ln);
        const u32 le = ((k - pi) >> 31) ^ 1u;
        idx += le;
        const u32 cand_before = pi * le;
        before = cand_before > before ? cand_before : before;
      }
      const u32 lo = read_lane(RT::at(ca, cb, 2u * idx), ln);
      const u32 hi = read_lane(RT::at(ca, cb, 2u * idx + 1u), ln);
      const u32 bit = kth_set_bit_wave(lo, hi, k - before);
      const u32 chunk = ((ln * (u32)NW + idx) << 6) + bit;
      // now in flight to d: one lane removes it from the LDS row
      if (lane == 0) {
        u32 *ptr = reinterpret_cast<u32 *>(&need_lds[(idx >> 1) * 64u + ln]) + ((idx & 1u) * 2u + (bit >> 5));
        *ptr &= ~(1u << (bit & 31u));
      }
      if ((u32)lane == b) res = chunk;
    }
  };
  if (idle) fetch(buf0_a, buf0_b, idle);
  if (!pre()) return kNone;
  while (idle) {
    decide(buf0_a, buf0_b, buf1_a, buf1_b);
    if (!idle) break;
    decide(buf1_a, buf1_b, buf0_a, buf0_b);
  }
  return res;
}

// Algorithm 1 for ONE destination d at TEN span `event` (time t), run by one wavefront.
// Returns (per lane) the earliest end time among the transfers in flight on the links
// this lane looked at; the caller min-reduces it.
//
// The destination's `need` row (chunks it neither holds nor is receiving) lives in LDS:
// one 1-KiB slab per piece, 16 bytes per lane, conflict-free ds_read_b128; need_lds
// points at this wavefront's private NP*64 uint4.  Source rows land in two register
// buffers used in turn, so that the next link's row is in flight while the current link
// is decided; the candidate set is formed in place in the buffer.
template <int NP, bool LATENCY_BOUND, class Rows>
__device__ __forceinline__ u64 match_destination(const PassDev &p, const Rows &rows, u32 d, u32 jb, u32 je, u32 event,
                                                     u64 t, u32 *__restrict__ sched_row, int lane, uint4 *need_lds,
                                                     const RecOut rec = RecOut(), u32 *wave_need = nullptr)
{
  constexpr int NW = 2 * NP;
  Ctl *ctl = p.ctl;
  u64 my_min = kInf;  // [jb, je) = d's in-list positions

  // LATENCY_BOUND (the single-workgroup kernel; few destinations per span): d's own row is
  // asked for together with the in-list records, before it is known whether any incoming
  // link is idle (one memory round trip instead of two, NP*4 more live registers), and the
  // links' random words are computed here.  Otherwise (one wavefront per destination of a
  // large topology, VALU- and bandwidth-bound) the random words were computed for all links
  // of the span by arrive_kernel, with every lane busy, and are read from p.rnd.
  uint4 own[NP];
  if constexpr (LATENCY_BOUND) {
#pragma unroll
    for (int i = 0; i < NP; ++i) own[i] = rows.load(d, i, lane);
  }

  u32 l0 = 0, s0 = 0, cr0 = kNone;
  u32 ry0 = 0;  // the record's source field: kept alive with the rest of the record (see below)
  u64 cs0 = 0;
  if (jb + lane < je) {
    uint4 rec;
    if constexpr (LATENCY_BOUND) rec = p.in_rec_in_lds ? lds_ld(p.in_rec + jb + lane) : glb_ld(p.in_rec + jb + lane);
    else rec = p.in_rec[jb + lane];
    cr0 = state_ld<LATENCY_BOUND>(&p.carry[jb + lane]);
    l0 = rec.x; ry0 = rec.y; cs0 = ((u64)rec.w << 32) | rec.z;
    // LATENCY_BOUND with the sources in LDS: the first source row can be asked for without
    // waiting for the record, i.e. in the same memory round trip as the record and d's own row.
    // (The empty asm keeps the two cases in separate branches: as a select, the source would
    // wait for the record in both.)
    if constexpr (LATENCY_BOUND) {
      if (p.in_src16) {
        s0 = lds_ld(p.in_src16 + jb + lane);
      } else {
        u32 y = rec.y;
        asm volatile("" : "+v"(y));
        s0 = y;
      }
    } else {
      s0 = rec.y;
    }
  }
  bool any_idle = __ballot(jb + lane < je && cr0 == kNone) != 0ull;
  for (u32 base = jb + 64; base < je && !any_idle; base += 64) {
    const u32 j = base + lane;
    any_idle = __ballot(j < je && state_ld<LATENCY_BOUND>(&p.carry[j < je ? j : jb]) == kNone) != 0ull;
  }

  bool need_any = false;
  bool need_ready = false;  // LATENCY_BOUND: the need row is set up behind the first row request
  auto setup_need = [&]() {
    need_ready = true;
    // need = ~held[d] & ~inflight[d], written to LDS; inflight[d] = the chunks on d's
    // busy incoming links, cleared by single-lane read-modify-writes
    u32 acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      uint4 v;
      if constexpr (LATENCY_BOUND) v = own[i];
      else v = rows.load(d, i, lane);
      v.x = ~v.x; v.y = ~v.y; v.z = ~v.z; v.w = ~v.w;
      need_lds[i * 64 + lane] = v;
      acc |= v.x | v.y | v.z | v.w;
    }
    need_any = __ballot(acc != 0u) != 0ull;  // before the in-flight bits are removed: a superset
    // d holds every chunk: nothing is or will be in flight to it, its links stay idle for
    // good, and the host may drop it from the processing order
    if (!need_any && p.dest_done && lane == 0) p.dest_done[d] = 1u;
    // (wave_need: the caller collects the flag per workgroup instead of one store per wavefront)
    if (need_any && lane == 0) {
      if (wave_need) *wave_need = 1u;
      else state_st<LATENCY_BOUND>(&ctl->need_flag[event & 1u], 1u);
    }
    for (u32 base = jb; base < je; base += 64) {
      const u32 j = base + lane;
      u32 cr = kNone;
      if (base == jb) cr = cr0;
      else if (j < je) cr = state_ld<LATENCY_BOUND>(&p.carry[j]);
      const u64 busy = __ballot(cr != kNone);
      if (busy && cr != kNone) {
        // every busy lane clears its own link's chunk (distinct chunks; dword updates
        // of one wavefront are applied in order by the LDS)
        const u32 w = cr >> 6;
        const u32 ln = w / (u32)NW;
        const u32 iw = w - ln * (u32)NW;
        u32 *ptr = reinterpret_cast<u32 *>(&need_lds[(iw >> 1) * 64u + ln]) + ((iw & 1u) * 2u + ((cr >> 5) & 1u));
        atomicAnd(ptr, ~(1u << (cr & 31u)));
      }
    }
  };
  if constexpr (!LATENCY_BOUND) {
    if (any_idle) setup_need();
  }

  // one block of up to 64 in-list entries, one per lane: (l, s, cr, cs) = the lane's link id,
  // source, chunk carried (kNone: idle) and cost
  auto block = [&](u32 base, u32 l, u32 s, u32 cr, u64 cs) {
    const u32 j = base + lane;
    const bool valid = j < je;
    u32 res = kNone;
    if constexpr (LATENCY_BOUND) {
      const u64 idle = __ballot(valid && cr == kNone);
      if (idle != 0ull && (need_any || !need_ready)) {
        u32 r = 0;
        res = draw_chunks<NP>(rows, s, r, idle, need_lds, lane, [&]() {
          if (!need_ready) {
            // d's own row and the records are first used here, behind the request for the first
            // source row, so that all three arrive in one memory round trip
            asm volatile("" ::: "memory");
#pragma unroll
            for (int i = 0; i < NP; ++i) asm volatile("" : "+v"(own[i].x), "+v"(own[i].y), "+v"(own[i].z), "+v"(own[i].w));
            setup_need();
          }
          // (an unused register of a load in flight would be reused at once, which waits for the load)
          asm volatile("" : "+v"(l) : "v"(ry0));
          r = philox4x32_10_word0(l, event, p.phase, 0u, p.seed_lo, p.seed_hi);
          return need_any;
        });
      }
    } else if (need_any) {
      const u64 idle = __ballot(valid && cr == kNone);
      const u32 r = valid ? p.rnd[j] : 0u;
      res = draw_chunks<NP>(rows, s, r, idle, need_lds, lane);
    }
    if (rec.recs) append_records(rec, valid && res != kNone, l, res, lane);
    if (valid) {
      if (sched_row && res != kNone) sched_row[l] = res;  // rows are pre-filled with kNone
      if (res != kNone) {
        if (res >= p.C) {
          state_st<LATENCY_BOUND>(&ctl->status, kStInternal);
          state_st<LATENCY_BOUND>(&ctl->done, 1u);
        } else if (cs > kInf - 1ull - t) {
          state_st<LATENCY_BOUND>(&ctl->status, kStOverflow);
          state_st<LATENCY_BOUND>(&ctl->done, 1u);
        } else {
          const u64 fa = t + cs;
          state_st<LATENCY_BOUND>(&p.carry[j], res);
          state_st<LATENCY_BOUND>(&p.free_at[j], fa);
          my_min = fa < my_min ? fa : my_min;
        }
      } else if (cr != kNone) {
        const u64 fa = state_ld<LATENCY_BOUND>(&p.free_at[j]);
        my_min = fa < my_min ? fa : my_min;
      }
    }
  };
  // the first block as straight-line code (no in-degree above 64 in practice): the values it
  // starts from are then not copied into loop variables, which would wait for their loads
  block(jb, l0, s0, cr0, cs0);
  for (u32 base = jb + 64; base < je; base += 64) {
    const u32 j = base + lane;
    u32 l = 0, s = 0, cr = kNone;
    u64 cs = 0;
    if (j < je) {
      uint4 rec;
      if constexpr (LATENCY_BOUND) rec = p.in_rec_in_lds ? lds_ld(p.in_rec + j) : glb_ld(p.in_rec + j);
      else rec = p.in_rec[j];
      cr = state_ld<LATENCY_BOUND>(&p.carry[j]);
      l = rec.x; s = rec.y; cs = ((u64)rec.w << 32) | rec.z;
    }
    block(base, l, s, cr, cs);
  }
  return my_min;
}

// Philox4x32-10, words 0 and 1 of the output block.
__device__ __forceinline__ void philox4x32_10_words01(u32 c0, u32 c1, u32 c2, u32 c3, u32 k0, u32 k1,
                                                      u32 &w0, u32 &w1)
{
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const u32 lo0 = 0xD2511F53u * c0, hi0 = __umulhi(0xD2511F53u, c0);
    const u32 lo1 = 0xCD9E8D57u * c2, hi1 = __umulhi(0xCD9E8D57u, c2);
    const u32 n0 = hi1 ^ c1 ^ k0;
    const u32 n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  w0 = c0;
  w1 = c1;
}

// Algorithm 1 in the order the paper prints it, for ONE destination d (in-degree <= 64),
// run by one wavefront: unsatisfied postconditions (d, c) are visited in random order and
// each is given a random in-neighbour that holds c and whose link is free.  Visiting a
// shuffled list and skipping the pairs no free link can serve equals drawing, step by
// step, a chunk uniformly from the servable ones (links are only used up), so each step
//   serv = need & OR_{free links} held[src];  c = (r0 mod |serv|)-th smallest of serv;
//   holders = free links whose source holds c (list order);  link = holders[r1 mod n]
//   (or the first holder when the list is sorted cheapest-first),
// with (r0, r1) = words 0, 1 of Philox(d, event, phase + 2, step; seed).
//
// Both cores below take the links of the destination one per lane (s: the lane's link's
// source NPU; free_links: the lanes whose link is free) and the need row in LDS, and return
// the chunk the lane's link carries or kNone.

// Any in-degree up to 64: the rows of the free links are re-streamed (from L2) in every step.
template <int NP, class Rows>
__device__ __forceinline__ u32 draw_pairs_streamed(const Rows &rows, u32 s, u64 free_links, u32 d, u32 event, u32 phase2,
                                                   u32 seed_lo, u32 seed_hi, bool first_holder, uint4 *need_lds,
                                                   int lane)
{
  constexpr int NW = 2 * NP;
  constexpr int NDW = 4 * NP;
  typedef RowRegs<NDW> RT;
  u32 res = kNone;
  for (u32 step = 0; free_links; ++step) {
    // serv = need & (OR of the rows of the free links), in registers
    typename RT::A acc_a = {};
    typename RT::B acc_b = {};
    u64 todo = free_links;
    while (todo) {
      const u32 b = (u32)__ffsll((long long)todo) - 1u;
      todo &= todo - 1ull;
      const u32 src = read_lane(s, b);
      static_for<0, NP>([&](auto I) {
        constexpr int i = decltype(I)::value;
        const uint4 v = rows.load(src, i, lane);
        RT::template set<4 * i>(acc_a, acc_b, RT::template get<4 * i>(acc_a, acc_b) | v.x);
        RT::template set<4 * i + 1>(acc_a, acc_b, RT::template get<4 * i + 1>(acc_a, acc_b) | v.y);
        RT::template set<4 * i + 2>(acc_a, acc_b, RT::template get<4 * i + 2>(acc_a, acc_b) | v.z);
        RT::template set<4 * i + 3>(acc_a, acc_b, RT::template get<4 * i + 3>(acc_a, acc_b) | v.w);
      });
    }
    u32 pre[NW];
    u32 cnt = 0;
    static_for<0, NP>([&](auto I) {
      constexpr int i = decltype(I)::value;
      const uint4 nd = need_lds[i * 64 + lane];
      const u32 c0 = RT::template get<4 * i>(acc_a, acc_b) & nd.x;
      const u32 c1 = RT::template get<4 * i + 1>(acc_a, acc_b) & nd.y;
      const u32 c2 = RT::template get<4 * i + 2>(acc_a, acc_b) & nd.z;
      const u32 c3 = RT::template get<4 * i + 3>(acc_a, acc_b) & nd.w;
      RT::template set<4 * i>(acc_a, acc_b, c0); RT::template set<4 * i + 1>(acc_a, acc_b, c1);
      RT::template set<4 * i + 2>(acc_a, acc_b, c2); RT::template set<4 * i + 3>(acc_a, acc_b, c3);
      cnt = popc_acc(c0, cnt);
      cnt = popc_acc(c1, cnt);
      pre[2 * i] = cnt;
      cnt = popc_acc(c2, cnt);
      cnt = popc_acc(c3, cnt);
      pre[2 * i + 1] = cnt;
    });
    const u32 incl = wave_inclusive_scan(cnt);
    const u32 pop = read_lane(incl, 63);
    if (pop == 0) break;  // no free link can serve any missing chunk
    u32 r0, r1;
    philox4x32_10_words01(d, event, phase2, step, seed_lo, seed_hi, r0, r1);
    u32 k = r0 % pop;
    const u64 above = __ballot(incl > k);
    const u32 ln = (u32)__ffsll((long long)above) - 1u;
    k -= read_lane(incl - cnt, ln);
    u32 idx = 0, before = 0;
#pragma unroll
    for (int i = 0; i < NW - 1; ++i) {
      const u32 pi = read_lane(pre[i], ln);
      const u32 le = ((k - pi) >> 31) ^ 1u;
      idx += le;
      const u32 cand_before = pi * le;
      before = cand_before > before ? cand_before : before;
    }
    const u32 lo = read_lane(RT::at(acc_a, acc_b, 2u * idx), ln);
    const u32 hi = read_lane(RT::at(acc_a, acc_b, 2u * idx + 1u), ln);
    const u32 bit = kth_set_bit_wave(lo, hi, k - before);
    const u32 chunk = ((ln * (u32)NW + idx) << 6) + bit;
    // which free links' sources hold the chunk: lane j tests its own source's dword
    const u32 dword = ((idx >> 1) * 128u + ln * 2u + (idx & 1u)) * 2u + (bit >> 5);
    bool holds = false;
    if ((free_links >> lane) & 1ull) {
      const u32 wv = rows.dword(s, dword);
      holds = (wv >> (bit & 31u)) & 1u;
    }
    const u64 holders = __ballot(holds);
    u32 pick;
    if (first_holder) pick = (u32)__ffsll((long long)holders) - 1u;
    else pick = kth_set_bit_wave((u32)holders, (u32)(holders >> 32), r1 % (u32)__popcll(holders));
    if ((u32)lane == pick) res = chunk;
    free_links &= ~(1ull << pick);
    if (lane == 0) {  // now in flight to d
      u32 *ptr = reinterpret_cast<u32 *>(&need_lds[(idx >> 1) * 64u + ln]) + ((idx & 1u) * 2u + (bit >> 5));
      *ptr &= ~(1u << (bit & 31u));
    }
  }
  return res;
}

// In-degree <= DEG (the links sit in lanes 0 .. DEG-1): the rows of all free links are read
// ONCE and stay in registers (DEG planes of a lane's share of a row), so that a step is
// register and LDS work only: OR of the planes & need, selection, and the holders of the chosen
// chunk from one dword of every plane; the plane of the link that was used is cleared.
template <int NP, int DEG, class Rows>
__device__ __forceinline__ u32 draw_pairs_planes(const Rows &rows, u32 s, u64 free_links, u32 d, u32 event, u32 phase2,
                                                 u32 seed_lo, u32 seed_hi, bool first_holder, uint4 *need_lds, int lane)
{
  constexpr int NW = 2 * NP;
  constexpr int NDW = 4 * NP;
  typedef RowRegs<NDW> RT;
  u32 res = kNone;
  typename RT::A pa[DEG];
  typename RT::B pb[DEG];
  static_for<0, DEG>([&](auto J) {
    constexpr int j = decltype(J)::value;
    pa[j] = typename RT::A{};
    pb[j] = typename RT::B{};
    if ((free_links >> j) & 1ull) {
      const u32 src = read_lane(s, (u32)j);
      static_for<0, NP>([&](auto I) {
        constexpr int i = decltype(I)::value;
        const uint4 v = rows.load(src, i, lane);
        RT::template set<4 * i>(pa[j], pb[j], v.x); RT::template set<4 * i + 1>(pa[j], pb[j], v.y);
        RT::template set<4 * i + 2>(pa[j], pb[j], v.z); RT::template set<4 * i + 3>(pa[j], pb[j], v.w);
      });
    }
  });
  // the random words of all steps at once: lane i computes the block of step i (a destination
  // takes at most one step per link, DEG <= 64), instead of one scalar block per step; word 1
  // is reduced modulo every possible number of holders 1 .. DEG here (divisions by constants),
  // four bits each
  u32 rw0, rw1;
  philox4x32_10_words01(d, event, phase2, (u32)lane, seed_lo, seed_hi, rw0, rw1);
  static_assert(DEG <= 8, "the packed remainders of word 1 take four bits per holder count");
  u32 rmods = 0;
  static_for<1, DEG + 1>([&](auto M) {
    constexpr u32 m = (u32)decltype(M)::value;
    rmods |= (rw1 % m) << (4u * (m - 1u));
  });
  for (u32 step = 0; free_links; ++step) {
    // serv = need & (OR of the planes), with the running in-lane candidate counts
    typename RT::A sa;
    typename RT::B sb;
    u32 pre[NW];
    u32 cnt = 0;
    static_for<0, NP>([&](auto I) {
      constexpr int i = decltype(I)::value;
      const uint4 nd = need_lds[i * 64 + lane];
      u32 o[4] = {0, 0, 0, 0};
      static_for<0, DEG>([&](auto J) {
        constexpr int j = decltype(J)::value;
        o[0] |= RT::template get<4 * i>(pa[j], pb[j]);
        o[1] |= RT::template get<4 * i + 1>(pa[j], pb[j]);
        o[2] |= RT::template get<4 * i + 2>(pa[j], pb[j]);
        o[3] |= RT::template get<4 * i + 3>(pa[j], pb[j]);
      });
      const u32 c0 = o[0] & nd.x, c1 = o[1] & nd.y, c2 = o[2] & nd.z, c3 = o[3] & nd.w;
      RT::template set<4 * i>(sa, sb, c0); RT::template set<4 * i + 1>(sa, sb, c1);
      RT::template set<4 * i + 2>(sa, sb, c2); RT::template set<4 * i + 3>(sa, sb, c3);
      cnt = popc_acc(c0, cnt);
      cnt = popc_acc(c1, cnt);
      pre[2 * i] = cnt;
      cnt = popc_acc(c2, cnt);
      cnt = popc_acc(c3, cnt);
      pre[2 * i + 1] = cnt;
    });
    const u32 incl = wave_inclusive_scan(cnt);
    const u32 pop = read_lane(incl, 63);
    if (pop == 0) break;  // no free link can serve any missing chunk
    const u32 k = read_lane(rw0, step) % pop;
    const u64 above = __ballot(incl > k);
    const u32 ln = (u32)__ffsll((long long)above) - 1u;
    // Every lane looks for rank k - (candidates in the lanes below it) among its own words with
    // vector compares; only the owning lane's answer is read.  (With three wavefronts per SIMD
    // the scalar unit's work does not hide behind the vector unit's: a walk driven by readlane
    // costs six scalar instructions per word.)
    const u32 kl = k - (incl - cnt);
    u32 idxv = 0, befv = 0;
#pragma unroll
    for (int i = 0; i < NW - 1; ++i) {
      const bool le = pre[i] <= kl;
      idxv += le ? 1u : 0u;
      befv = le ? pre[i] : befv;
    }
    const u32 idx = read_lane(idxv, ln);
    const u32 k2 = read_lane(kl - befv, ln);
    const u32 lo = read_lane(RT::at(sa, sb, 2u * idx), ln);
    const u32 hi = read_lane(RT::at(sa, sb, 2u * idx + 1u), ln);
    const u32 bit = kth_set_bit_wave(lo, hi, k2);
    const u32 chunk = ((ln * (u32)NW + idx) << 6) + bit;
    // holders: the planes (free links) that have the chunk's bit; every lane forms the mask from
    // its own dword dw of every plane, the owning lane's is read
    const u32 dw = 2u * idx + (bit >> 5);
    u32 hv = 0;
    static_for<0, DEG>([&](auto J) {
      constexpr int j = decltype(J)::value;
      hv |= ((RT::at(pa[j], pb[j], dw) >> (bit & 31u)) & 1u) << j;
    });
    const u32 holders = read_lane(hv, ln);
    u32 pick;
    if (first_holder) pick = (u32)__ffs((int)holders) - 1u;
    else {
      u32 m = holders;
      const u32 q0 = (read_lane(rmods, step) >> (4u * ((u32)__popc(holders) - 1u))) & 15u;
      for (u32 q = q0; q; --q) m &= m - 1u;  // drop the q lowest holders
      pick = (u32)__ffs((int)m) - 1u;
    }
    if ((u32)lane == pick) res = chunk;
    free_links &= ~(1ull << pick);
    static_for<0, DEG>([&](auto J) {  // a used link serves nothing more
      constexpr int j = decltype(J)::value;
      if (pick == (u32)j) {
        asm volatile("" ::: "memory");  // keeps this a (wave-uniform) branch: one plane is cleared, not all selected
        pa[j] = typename RT::A{};
        pb[j] = typename RT::B{};
      }
    });
    if (lane == 0) {  // now in flight to d
      u32 *ptr = reinterpret_cast<u32 *>(&need_lds[(idx >> 1) * 64u + ln]) + ((idx & 1u) * 2u + (bit >> 5));
      *ptr &= ~(1u << (bit & 31u));
    }
  }
  return res;
}

// The postcondition-centric matching of destination d at span `event` (time t): set-up of the
// need row, one of the two cores above, and the link state of the matched links.  Returns (per
// lane) the end time of the transfer on the lane's link, for the next-event reduction.
template <int NP, int DEG, class Rows>
__device__ __forceinline__ u64 match_destination_pairs(const PassDev &p, const Rows &rows, u32 d, u32 jb, u32 je,
                                                       u32 event, u64 t, u32 *__restrict__ sched_row, int lane,
                                                       uint4 *need_lds, bool first_holder, const RecOut rec = RecOut())
{
  constexpr int NW = 2 * NP;
  Ctl *ctl = p.ctl;
  u64 my_min = kInf;
  const bool valid = jb + lane < je;
  const u32 j = jb + (u32)lane;
  u32 l = 0, s = 0, cr = kNone;
  u64 cs = 0;
  if (valid) {
    const uint4 rec = p.in_rec_in_lds ? lds_ld(p.in_rec + j) : glb_ld(p.in_rec + j);
    cr = p.carry[j];
    l = rec.x; s = rec.y; cs = ((u64)rec.w << 32) | rec.z;
  }
  const u64 free_links = __ballot(valid && cr == kNone);
  u32 res = kNone;

  if (free_links) {
    u32 acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      uint4 v = rows.load(d, i, lane);
      v.x = ~v.x; v.y = ~v.y; v.z = ~v.z; v.w = ~v.w;
      need_lds[i * 64 + lane] = v;
      acc |= v.x | v.y | v.z | v.w;
    }
    const bool need_any = __ballot(acc != 0u) != 0ull;
    if (!need_any && p.dest_done && lane == 0) p.dest_done[d] = 1u;  // d holds every chunk
    if (need_any && lane == 0) ctl->need_flag[event & 1u] = 1u;
    if (cr != kNone) {  // chunks in flight to d are not needed
      const u32 w = cr >> 6;
      const u32 ln = w / (u32)NW;
      const u32 iw = w - ln * (u32)NW;
      u32 *ptr = reinterpret_cast<u32 *>(&need_lds[(iw >> 1) * 64u + ln]) + ((iw & 1u) * 2u + ((cr >> 5) & 1u));
      atomicAnd(ptr, ~(1u << (cr & 31u)));
    }
    if (need_any) {
      if (DEG > 0 && je - jb <= (u32)(DEG > 0 ? DEG : 1))
        res = draw_pairs_planes<NP, (DEG > 0 ? DEG : 1)>(rows, s, free_links, d, event, p.phase + 2u, p.seed_lo,
                                                         p.seed_hi, first_holder, need_lds, lane);
      else
        res = draw_pairs_streamed<NP>(rows, s, free_links, d, event, p.phase + 2u, p.seed_lo, p.seed_hi, first_holder,
                                      need_lds, lane);
    }
  }
  if (rec.recs) append_records(rec, valid && res != kNone, l, res, lane);
  if (valid) {
    if (sched_row && res != kNone) sched_row[l] = res;  // rows are pre-filled with kNone
    if (res != kNone) {
      if (res >= p.C) {
        ctl->status = kStInternal;
        ctl->done = 1u;
      } else if (cs > kInf - 1ull - t) {
        ctl->status = kStOverflow;
        ctl->done = 1u;
      } else {
        const u64 fa = t + cs;
        p.carry[j] = res;
        p.free_at[j] = fa;
        my_min = fa < my_min ? fa : my_min;
      }
    } else if (cr != kNone) {
      const u64 fa = p.free_at[j];
      my_min = fa < my_min ? fa : my_min;
    }
  }
  return my_min;
}

// MODE 0: link-centric matching; 1: postcondition-centric, random holder; 2: postcondition-
// centric, first holder of the (cheapest-first) list.
// (Five-piece rows, the 40,960-NPU workloads: the register allocator lands two registers
// above the 80 that allow 6 wavefronts per SIMD; asking for 6 costs no spill and is 7 %
// faster.  7 or 8 wavefronts per SIMD spill and are slower.)
// DEG (postcondition-centric modes): in-degrees up to DEG keep the rows of a destination's free
// links in registers (draw_pairs_planes); 0 = always re-stream them.
template <int NP, int MODE, int DEG>
__global__ __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu(MODE == 0 ? (NP == 5 ? 6 : 1) : (4 * NP * DEG >= 96 ? 3 : 1))))
void match_kernel(PassDev p, u32 event, u32 *__restrict__ sched_row)
{
  const int lane = threadIdx.x & 63;
  // Workgroups are handed to the 8 XCDs round-robin.  Give XCD x the contiguous slice
  // [x*per_xcd, (x+1)*per_xcd) of the processing order, so that destinations that are
  // close in the order (and share source rows) meet in the same L2.
  // The grid is a multiple of 8 workgroups; slots past N do nothing.
  const u32 per_xcd = gridDim.x >> 3;
  const u32 pos = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const u32 slot = uniform(pos * 4u + (threadIdx.x >> 6));
  Ctl *ctl = p.ctl;
  __shared__ uint4 need_lds[4 * NP * 64];
  __shared__ u64 wg_min[4];
  __shared__ u32 wg_need[4];
  u64 my_min = kInf;
  if (lane == 0) wg_need[threadIdx.x >> 6] = 0u;
  if (slot < p.n_slots && !ctl->done) {
    const uint4 sr = p.slot_rec[slot];  // (destination, its in-list begin, end)
    const u32 d = uniform(sr.x), jb = uniform(sr.y), je = uniform(sr.z);
    const u64 t = ctl->next_t[event & 1u];
    uint4 *my_need = need_lds + (threadIdx.x >> 6) * NP * 64;
    const RowsHbm rows{p.held, p.row_words};
    if constexpr (MODE == 0)
      my_min = match_destination<NP, false>(p, rows, d, jb, je, event, t, sched_row, lane, my_need, RecOut(),
                                            &wg_need[threadIdx.x >> 6]);
    else my_min = match_destination_pairs<NP, DEG>(p, rows, d, jb, je, event, t, sched_row, lane, my_need, MODE == 2);
  }
  // a8: next span = earliest end of a transfer in flight (min over all destinations): the
  // workgroup's four wavefronts through LDS, then one filtered atomic
  const u64 m = wave_min64(my_min);
  if (lane == 0) wg_min[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    if constexpr (MODE == 0) {
      if ((wg_need[0] | wg_need[1] | wg_need[2] | wg_need[3]) != 0u) ctl->need_flag[event & 1u] = 1u;
    }
    u64 mm = wg_min[0];
    mm = wg_min[1] < mm ? wg_min[1] : mm;
    mm = wg_min[2] < mm ? wg_min[2] : mm;
    mm = wg_min[3] < mm ? wg_min[3] : mm;
    if (mm != kInf) {
      u64 *nt = &p.next_slots[((event + 1u) & 1u) * kNextSlots + (pos & p.next_mask)];
      const u64 cur = __hip_atomic_load(nt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (mm < cur) atomicMin(nt, mm);
    }
  }
}

// The same with a compact schedule: the matches of a forward pass are appended as (link, chunk)
// records at ctl->n_rec; in a reversed pass (whose records are its arrivals, appended by the
// arrivals kernel of the next span) first_next receives the index that span's records start at.
// For topologies whose links all cost differently: about one match per span, millions of spans.
template <int NP, int MODE>
__global__ __launch_bounds__(256) void match_compact_kernel(PassDev p, u32 event, uint2 *__restrict__ recs,
                                                            u32 *__restrict__ first_next)
{
  const int lane = threadIdx.x & 63;
  const u32 per_xcd = gridDim.x >> 3;
  const u32 pos = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const u32 slot = uniform(pos * 4u + (threadIdx.x >> 6));
  Ctl *ctl = p.ctl;
  __shared__ uint4 need_lds[4 * NP * 64];
  __shared__ u64 wg_min[4];
  u64 my_min = kInf;
  if (slot < p.n_slots && !ctl->done) {
    const uint4 sr = p.slot_rec[slot];
    const u32 d = uniform(sr.x), jb = uniform(sr.y), je = uniform(sr.z);
    const u64 t = ctl->next_t[event & 1u];
    if (first_next && slot == 0u && lane == 0) *first_next = ctl->n_rec;
    uint4 *my_need = need_lds + (threadIdx.x >> 6) * NP * 64;
    const RecOut rec = p.reversed ? RecOut() : RecOut{recs, &ctl->n_rec};
    const RowsHbm rows{p.held, p.row_words};
    if constexpr (MODE == 0) my_min = match_destination<NP, false>(p, rows, d, jb, je, event, t, nullptr, lane, my_need, rec);
    else my_min = match_destination_pairs<NP, 0>(p, rows, d, jb, je, event, t, nullptr, lane, my_need, MODE == 2, rec);
  }
  const u64 m = wave_min64(my_min);  // as match_kernel
  if (lane == 0) wg_min[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    u64 mm = wg_min[0];
    mm = wg_min[1] < mm ? wg_min[1] : mm;
    mm = wg_min[2] < mm ? wg_min[2] : mm;
    mm = wg_min[3] < mm ? wg_min[3] : mm;
    if (mm != kInf) {
      u64 *nt = &p.next_slots[((event + 1u) & 1u) * kNextSlots + (pos & p.next_mask)];
      const u64 cur = __hip_atomic_load(nt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (mm < cur) atomicMin(nt, mm);
    }
  }
}

// ---------------------------------------------------------------- homogeneous TEN: one launch per span

__global__ void uniform_init_kernel(PassDev p, UniformDev u)
{
  const u32 j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= p.L) return;
  u.prev[0][j] = kNone;
  u.prev[1][j] = kNone;
  if (u.rnd[0]) u.rnd[0][j] = philox4x32_10_word0(p.in_link[j], 0u, p.phase, 0u, p.seed_lo, p.seed_hi);
}

// Algorithm 1 (link-centric form) for ONE destination d at span `event` of a homogeneous TEN,
// run by one wavefront.  Every incoming link is idle at the start of a span (the transfers of
// the previous span have just arrived) and nothing is in flight, so need = ~held[d].  Returns
// whether a link was matched.
template <int NP>
__device__ __forceinline__ bool match_destination_uniform(const PassDev &p, const UniformDev &u, u32 d, u32 jb, u32 je,
                                                          u32 event, u32 *__restrict__ sched_row,
                                                          u32 *__restrict__ sched_row_next, int lane, uint4 *need_lds)
{
  Ctl *ctl = p.ctl;
  const u64 *H = u.held[event & 1u];
  u64 *Hn = u.held[(event + 1u) & 1u] + (u64)d * p.row_words;
  const u32 *prev_in = u.prev[(event + 1u) & 1u];
  u32 *prev_out = u.prev[event & 1u];
  const u32 *rnd = u.rnd[event & 1u];
  const uint4 *hp = reinterpret_cast<const uint4 *>(H + (u64)d * p.row_words) + lane;
  // Everything that depends on the slot record only is asked for at once: d's own row, and for the
  // first 64 in-list entries the chunk that arrived now, the record and the span's random word.
  // (Launches of ten to thirty thousand destinations gain 3 to 6 % from the shorter chain of
  // memory round trips; smaller ones are bound by the instructions of the decisions.)
  uint4 own[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) own[i] = hp[i * 64];
  const bool valid0 = jb + (u32)lane < je;
  u32 pc0 = kNone, l0 = 0, s0 = 0, r0 = 0;
  if (valid0) {
    const u32 j = jb + (u32)lane;
    if (event != 0u) pc0 = prev_in[j];
    const uint4 rec = p.in_rec[j];
    l0 = rec.x; s0 = rec.y;
    r0 = rnd[j];
  }
  bool need_any = false;
  auto setup_need = [&]() {
    u32 acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      uint4 v = own[i];
      v.x = ~v.x; v.y = ~v.y; v.z = ~v.z; v.w = ~v.w;
      need_lds[i * 64 + lane] = v;
      acc |= v.x | v.y | v.z | v.w;
    }
    need_any = __ballot(acc != 0u) != 0ull;
    return need_any;
  };
  // one block of up to 64 in-list entries, one per lane; returns whether a link was matched
  auto finish_block = [&](u32 base, bool valid, u32 l, u32 res) {
    const u32 j = base + (u32)lane;
    if (valid) {
      prev_out[j] = res;
      if (res != kNone) {
        if (res >= p.C) {
          ctl->status = kStInternal;
          ctl->done = 1u;
        } else {
          if (sched_row) sched_row[l] = res;            // rows are pre-filled with kNone
          if (sched_row_next) sched_row_next[l] = res;  // reversed pass: keyed by arrival
          atomicOr(&Hn[phys_word(res >> 6, NP)], 1ull << (res & 63u));
        }
      }
    }
    return __ballot(res != kNone) != 0ull;
  };
  // The first block: the first source row is asked for as soon as the records are there and the
  // need row is set up behind that request.  (Asking for the rows of up to 8 links at once was
  // measured on rows of one and two pieces: no gain on 4,096 NPUs, where the launch is bound by
  // the instructions of the decisions, and 7 % slower with two pieces, where the registers cost
  // occupancy.)
  const u32 res0 = draw_chunks<NP>(RowsHbm{H, p.row_words}, s0, r0, __ballot(valid0), need_lds, lane, setup_need);
  // the chunks that arrived now are in held[event & 1] already; the other table lags a span
  bool had_prev = __ballot(pc0 != kNone) != 0ull;
  if (pc0 != kNone) atomicOr(&Hn[phys_word(pc0 >> 6, NP)], 1ull << (pc0 & 63u));
  for (u32 base = jb + 64u; base < je && event != 0u; base += 64u) {
    const u32 j = base + (u32)lane;
    const u32 pc = j < je ? prev_in[j] : kNone;
    if (pc != kNone) atomicOr(&Hn[phys_word(pc >> 6, NP)], 1ull << (pc & 63u));
    had_prev = had_prev || __ballot(pc != kNone) != 0ull;
  }
  if (!need_any) {
    // d holds every chunk; once its last arrivals are in both tables the host may drop it
    for (u32 base = jb; base < je; base += 64)
      if (base + (u32)lane < je) prev_out[base + lane] = kNone;
    if (!had_prev && p.dest_done && lane == 0) p.dest_done[d] = 1u;
    return false;
  }
  if (lane == 0) ctl->need_flag[event % 3u] = 1u;
  bool any = finish_block(jb, valid0, l0, res0);
  for (u32 base = jb + 64u; base < je; base += 64u) {  // in-degrees above 64
    const u32 j = base + (u32)lane;
    const bool valid = j < je;
    u32 l = 0, s = 0, r = 0;
    if (valid) {
      const uint4 rec = p.in_rec[j];
      l = rec.x; s = rec.y;
      r = rnd[j];
    }
    const u32 res = draw_chunks<NP>(RowsHbm{H, p.row_words}, s, r, __ballot(valid), need_lds, lane);
    any = finish_block(base, valid, l, res) || any;
  }
  return any;
}

template <int NP, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NP == 5 && MODE == 0 ? 6 : 1)))
void match_uniform_kernel(PassDev p, UniformDev u, u32 event, u32 *__restrict__ sched_row,
                          u32 *__restrict__ sched_row_next, u64 *__restrict__ event_time_slot)
{
  const int lane = threadIdx.x & 63;
  const u32 per_xcd = gridDim.x >> 3;  // as match_kernel: contiguous slices of the order per XCD
  const u32 pos = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const u32 slot = uniform(pos * 4u + (threadIdx.x >> 6));
  if (slot >= p.n_slots) return;
  const uint4 sr = p.slot_rec[slot];
  const u32 d = uniform(sr.x), jb = uniform(sr.y), je = uniform(sr.z);
  Ctl *ctl = p.ctl;
  if (ctl->done) return;
  if (event != 0u) {
    // a4 / a8: what the previous span found.  Nothing needed: the collective ended there.
    // Something needed and nothing matched: no transfer is in flight, the topology is not
    // strongly connected.
    const u32 pv = (event + 2u) % 3u;
    const u32 nf = ctl->need_flag[pv], mf = ctl->match_flag[pv];
    if (nf == 0u || mf == 0u) {
      if (slot == 0 && lane == 0) {
        if (nf == 0u) { ctl->T = (u64)(event - 1u) * u.cost; ctl->n_events = event - 1u; }
        else ctl->status = kStUnreachable;
        ctl->done = 1u;
      }
      return;
    }
  }
  if (slot == 0 && lane == 0) {
    const u32 nx = (event + 1u) % 3u;
    ctl->need_flag[nx] = 0u;
    ctl->match_flag[nx] = 0u;
    *event_time_slot = (u64)event * u.cost;
  }
  __shared__ uint4 need_lds[4 * NP * 64];
  uint4 *my_need = need_lds + (threadIdx.x >> 6) * NP * 64;
  const bool any = match_destination_uniform<NP>(p, u, d, jb, je, event, sched_row, sched_row_next, lane, my_need);
  if (any && lane == 0) ctl->match_flag[event % 3u] = 1u;
  // a6, first half, for the NEXT span.  All destinations in the launch: its wavefronts share out
  // the links, 64 each, so that every lane of the few wavefronts that do it is busy.  Once the
  // host has dropped complete destinations, only the links into the remaining ones can be
  // matched again: every wavefront draws for its own destination's in-list (sharing out ALL
  // links among a handful of wavefronts took tens of microseconds per span at the end of a pass
  // on a mesh).
  if (u.rnd[0]) {
    u32 *rnd_next = u.rnd[(event + 1u) & 1u];
    if (p.n_slots == p.N) {
      for (u32 q = slot * 64u + (u32)lane; q < p.L; q += p.n_slots * 64u)
        rnd_next[q] = philox4x32_10_word0(p.in_rec[q].x, event + 1u, p.phase, 0u, p.seed_lo, p.seed_hi);
    } else {
      for (u32 q = jb + (u32)lane; q < je; q += 64u)
        rnd_next[q] = philox4x32_10_word0(p.in_rec[q].x, event + 1u, p.phase, 0u, p.seed_lo, p.seed_hi);
    }
  }
}

// From the launches with link state to one launch per span (see launch_links_to_uniform): the
// chunks in flight (all matched in span event - 1: equal link costs) become the arrivals of span
// `event`: into the table that span reads, into the list the lagging table is brought up to date
// from, and (reversed pass) into the span's schedule row.
__global__ __launch_bounds__(256) void links_to_uniform_kernel(PassDev p, UniformDev u, u32 event,
                                                               u32 *__restrict__ sched_row)
{
  const u32 j = blockIdx.x * 256u + threadIdx.x;
  Ctl *ctl = p.ctl;
  if (j < p.L) {
    const u32 c = __hip_atomic_load(&p.carry[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const u32 link = p.in_link[j];
    u.prev[(event + 1u) & 1u][j] = c;
    u.prev[event & 1u][j] = kNone;
    u.rnd[event & 1u][j] = philox4x32_10_word0(link, event, p.phase, 0u, p.seed_lo, p.seed_hi);
    if (c != kNone) {
      atomicOr(&u.held[event & 1u][(u64)p.pos_dst[j] * p.row_words + phys_word(c >> 6, p.NP)], 1ull << (c & 63u));
      if (sched_row) sched_row[link] = c;  // rows are pre-filled with kNone
      ctl->match_flag[(event - 1u) % 3u] = 1u;
    }
  }
}

// the need flag of span event - 1 from where the launches with link state keep it to where one
// launch per span looks for it; every other flag cleared
__global__ void links_to_uniform_flags_kernel(Ctl *ctl, u32 event)
{
  // (An atomic load, i.e. a vector memory instruction: as a plain load of a uniform address this
  // becomes a scalar load, which the hardware does not order with the vector stores below; they
  // overtook it and it returned the cleared flag.)
  const u32 nf = __hip_atomic_load(&ctl->need_flag[(event - 1u) & 1u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int i = 0; i < 4; ++i) { ctl->need_flag[i] = 0u; ctl->match_flag[i] = 0u; }
  ctl->need_flag[(event - 1u) % 3u] = nf;
}

// From one launch per span to the launches with link state (see launch_uniform_handover).
__global__ __launch_bounds__(256) void uniform_handover_kernel(PassDev p, UniformDev u, u32 event)
{
  const u32 j = blockIdx.x * 256u + threadIdx.x;
  Ctl *ctl = p.ctl;
  const u64 t = (u64)event * u.cost;
  if (j < p.L) {
    const u32 c = __hip_atomic_load(&u.prev[(event - 1u) & 1u][j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    p.carry[j] = c;
    p.free_at[j] = c != kNone ? t : 0ull;
    if (c != kNone) {  // few links: the form changes when a handful of destinations are left
      u64 *nt = &p.next_slots[(event & 1u) * kNextSlots];
      if (__hip_atomic_load(nt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != t) atomicMin(nt, t);
    }
  }
  if (j == 0) {
    const u32 nf = __hip_atomic_load(&ctl->need_flag[(event - 1u) % 3u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ctl->now = t - u.cost;
    ctl->need_flag[(event - 1u) & 1u] = nf;
  }
}

// ---------------------------------------------------------------- rows of more than 8 pieces

// Link-centric matching for ONE destination when a row (more than 65,536 chunks) no longer
// fits a wavefront's registers: the source row is STREAMED.  Pass 1 reads it piece by piece,
// forms cand = piece & need on the fly and keeps only the lane's candidate count per piece
// (one byte each: a lane's share of a piece is 128 bits); the wave prefix sum over the lane
// totals finds the owning lane, its per-piece counts the owning piece; pass 2 reloads that
// one 16-byte share and selects the bit.  The need row (NP KiB) is in LDS as before.
// np <= kMaxStreamedPieces pieces; same results as match_destination.
constexpr u32 kMaxStreamedPieces = 32;
// (Rows of up to kMaxRegisterPieces pieces are matched with whole rows in registers: match_destination.)
constexpr u32 kMaxRegisterPieces = 15;

__device__ __forceinline__ u64 match_destination_streamed(const PassDev &p, u32 d, u32 jb, u32 je, u32 event,
                                                          u64 t, u32 *__restrict__ sched_row, int lane,
                                                          uint4 *need_lds)
{
  const u32 np = p.NP, nw = 2u * np;
  Ctl *ctl = p.ctl;
  u64 my_min = kInf;
  // clear chunk c in the LDS need row (lane-major layout: lane c/64/nw, word c/64 mod nw)
  auto need_word = [&](u32 c) {
    const u32 w = c >> 6;
    const u32 ln = w / nw;
    const u32 iw = w - ln * nw;
    return reinterpret_cast<u32 *>(&need_lds[(iw >> 1) * 64u + ln]) + ((iw & 1u) * 2u + ((c >> 5) & 1u));
  };
  bool any_idle = false;
  for (u32 base = jb; base < je && !any_idle; base += 64) {
    const u32 j = base + (u32)lane;
    any_idle = __ballot(j < je && p.carry[j < je ? j : jb] == kNone) != 0ull;
  }
  bool need_any = false;
  if (any_idle) {
    const uint4 *hp = reinterpret_cast<const uint4 *>(p.held + (u64)d * p.row_words) + lane;
    u32 acc = 0;
    for (u32 i = 0; i < np; ++i) {
      uint4 v = hp[i * 64u];
      v.x = ~v.x; v.y = ~v.y; v.z = ~v.z; v.w = ~v.w;
      need_lds[i * 64u + lane] = v;
      acc |= v.x | v.y | v.z | v.w;
    }
    need_any = __ballot(acc != 0u) != 0ull;
    if (!need_any && p.dest_done && lane == 0) p.dest_done[d] = 1u;
    if (need_any && lane == 0) ctl->need_flag[event & 1u] = 1u;
    for (u32 base = jb; base < je; base += 64) {  // chunks in flight to d are not needed
      const u32 j = base + (u32)lane;
      const u32 cr = j < je ? p.carry[j] : kNone;
      if (cr != kNone) atomicAnd(need_word(cr), ~(1u << (cr & 31u)));
    }
  }

  for (u32 base = jb; base < je; base += 64) {
    const u32 j = base + (u32)lane;
    const bool valid = j < je;
    u32 l = 0, s = 0, cr = kNone, r = 0;
    u64 cs = 0;
    if (valid) {
      const uint4 rec = p.in_rec[j];
      cr = p.carry[j];
      r = p.rnd[j];
      l = rec.x; s = rec.y; cs = ((u64)rec.w << 32) | rec.z;
    }
    u32 res = kNone;
    u64 idle = need_any ? __ballot(valid && cr == kNone) : 0ull;
    while (idle) {
      const u32 b = (u32)__ffsll((long long)idle) - 1u;
      idle &= idle - 1ull;
      const uint4 *sp = reinterpret_cast<const uint4 *>(p.held + (u64)read_lane(s, b) * p.row_words) + lane;
      // pass 1: candidate count of this lane per piece, packed four to a register; eight
      // pieces of the row are asked for at a time (few wavefronts fit beside the need rows,
      // so each keeps many loads in flight)
      u32 pc[kMaxStreamedPieces / 4];
      u32 cnt = 0;
#pragma unroll
      for (u32 g = 0; g < kMaxStreamedPieces / 4; ++g) pc[g] = 0;
#pragma unroll
      for (u32 h = 0; h < kMaxStreamedPieces / 8; ++h) {
        if (h * 8u < np) {
          uint4 v[8];
#pragma unroll
          for (u32 q = 0; q < 8; ++q)
            if (h * 8u + q < np) v[q] = sp[(h * 8u + q) * 64u];
#pragma unroll
          for (u32 q = 0; q < 8; ++q)
            if (h * 8u + q < np) {
              const uint4 nd = need_lds[(h * 8u + q) * 64u + lane];
              const u32 c = (u32)__popc(v[q].x & nd.x) + (u32)__popc(v[q].y & nd.y) + (u32)__popc(v[q].z & nd.z) +
                            (u32)__popc(v[q].w & nd.w);
              pc[h * 2u + (q >> 2)] |= c << (8u * (q & 3u));
              cnt += c;
            }
        }
      }
      const u32 incl = wave_inclusive_scan(cnt);
      const u32 pop = read_lane(incl, 63);
      if (pop == 0) continue;
      u32 k = read_lane(r, b) % pop;
      const u32 ln = (u32)__ffsll((long long)__ballot(incl > k)) - 1u;
      k -= read_lane(incl - cnt, ln);
      // the owning lane's piece: walk its per-piece counts (wave-uniform)
      u32 piece = 0;
      bool found = false;
#pragma unroll
      for (u32 g = 0; g < kMaxStreamedPieces / 4; ++g) {
        const u32 packed = read_lane(pc[g], ln);
#pragma unroll
        for (u32 q = 0; q < 4; ++q) {
          const u32 c = (packed >> (8u * q)) & 0xFFu;
          if (!found) {
            if (k < c) { piece = g * 4u + q; found = true; }
            else k -= c;
          }
        }
      }
      // pass 2: the owning lane's 16 bytes of that piece again
      uint4 cv = make_uint4(0, 0, 0, 0);
      if ((u32)lane == ln) {
        const uint4 v = sp[piece * 64u];
        const uint4 nd = need_lds[piece * 64u + lane];
        cv = make_uint4(v.x & nd.x, v.y & nd.y, v.z & nd.z, v.w & nd.w);
      }
      const u32 w0 = read_lane(cv.x, ln), w1 = read_lane(cv.y, ln), w2 = read_lane(cv.z, ln), w3 = read_lane(cv.w, ln);
      u32 dw = 0, word = w0;
      const u32 c0 = (u32)__popc(w0), c1 = (u32)__popc(w1), c2 = (u32)__popc(w2);
      if (k >= c0) { k -= c0; dw = 1; word = w1;
        if (k >= c1) { k -= c1; dw = 2; word = w2;
          if (k >= c2) { k -= c2; dw = 3; word = w3; } } }
      const u32 bit = kth_set_bit_wave(word, 0u, k);
      // dwords 0,1 of a lane's share are logical word 2*piece, dwords 2,3 word 2*piece+1
      const u32 chunk = ((ln * nw + 2u * piece + (dw >> 1)) << 6) + (dw & 1u) * 32u + bit;
      if (lane == 0) *need_word(chunk) &= ~(1u << (chunk & 31u));  // now in flight to d
      if ((u32)lane == b) res = chunk;
    }
    if (valid) {
      if (sched_row && res != kNone) sched_row[l] = res;  // rows are pre-filled with kNone
      if (res != kNone) {
        if (res >= p.C) {
          ctl->status = kStInternal;
          ctl->done = 1u;
        } else if (cs > kInf - 1ull - t) {
          ctl->status = kStOverflow;
          ctl->done = 1u;
        } else {
          const u64 fa = t + cs;
          p.carry[j] = res;
          p.free_at[j] = fa;
          my_min = fa < my_min ? fa : my_min;
        }
      } else if (cr != kNone) {
        const u64 fa = p.free_at[j];
        my_min = fa < my_min ? fa : my_min;
      }
    }
  }
  return my_min;
}

__global__ __launch_bounds__(256) void match_kernel_streamed(PassDev p, u32 event, u32 *__restrict__ sched_row)
{
  extern __shared__ __align__(16) unsigned char streamed_lds[];  // 4 wavefronts x NP KiB of need rows
  const int lane = threadIdx.x & 63;
  const u32 per_xcd = gridDim.x >> 3;  // as match_kernel
  const u32 pos = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const u32 slot = uniform(pos * 4u + (threadIdx.x >> 6));
  if (slot >= p.n_slots) return;
  const uint4 sr = p.slot_rec[slot];
  const u32 d = uniform(sr.x), jb = uniform(sr.y), je = uniform(sr.z);
  Ctl *ctl = p.ctl;
  if (ctl->done) return;
  const u64 t = ctl->next_t[event & 1u];
  uint4 *my_need = reinterpret_cast<uint4 *>(streamed_lds) + (size_t)(threadIdx.x >> 6) * p.NP * 64u;
  const u64 my_min = match_destination_streamed(p, d, jb, je, event, t, sched_row, lane, my_need);
  const u64 m = wave_min64(my_min);
  if (lane == 0 && m != kInf) {
    u64 *nt = &p.next_slots[((event + 1u) & 1u) * kNextSlots + (slot & p.next_mask)];
    const u64 cur = __hip_atomic_load(nt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (m < cur) atomicMin(nt, m);
  }
}

// ---------------------------------------------------------------- few chunks: a lane per destination

// Position of the k-th (0-based) set bit of x, k < popcount(x): binary search on popcounts.
__device__ __forceinline__ u32 kth_set_bit64(u64 x, u32 k)
{
  u32 pos = 0;
  u32 c = (u32)__popc((u32)x);
  u32 w = (u32)x;
  if (k >= c) { k -= c; pos = 32; w = (u32)(x >> 32); }
#pragma unroll
  for (u32 width = 16; width >= 1; width >>= 1) {
    const u32 lowbits = w & ((1u << width) - 1u);
    c = (u32)__popc(lowbits);
    if (k >= c) { k -= c; pos += width; w >>= width; }
    else w = lowbits;
  }
  return pos;
}

// Link-centric matching (Algorithm 1, as match_destination) when a bitset row is at most W
// 64-bit words (W * 64 chunks): ONE LANE per destination instead of one wavefront, every lane
// walking its own destination's idle incoming links in list order with its need row in
// registers, so that a wavefront matches 64 destinations at once.  Rows, in-list records and
// offsets and the link state are in LDS (single-workgroup kernel).  active: the lane has a
// destination d; all lanes of the wavefront must call this together.
template <int W>
__device__ __forceinline__ void match_destinations_by_lane(const PassDev &q, const RowsLds &rows, const u32 *in_ptr, u32 d,
                                                           bool active, u32 event, u64 t, const RecOut rec, int lane)
{
  Ctl *ctl = q.ctl;
  const u32 nw = 2u * rows.lanes;  // words of a row that hold chunk ids (NP = 1: lane j owns words 2j, 2j + 1)
  u32 jb = 0, deg = 0;
  if (active) { jb = in_ptr[d]; deg = in_ptr[d + 1] - jb; }
  u64 need[W];
  {
    const u64 *own = reinterpret_cast<const u64 *>(rows.base + d * rows.row_u4);
#pragma unroll
    for (int w = 0; w < W; ++w) need[w] = (active && (u32)w < nw) ? ~own[w] : 0ull;
  }
  bool any_idle = false;
  for (u32 jr = 0; jr < deg; ++jr) {  // chunks in flight to d are not needed
    const u32 c = q.carry[jb + jr];
    if (c == kNone) { any_idle = true; continue; }
#pragma unroll
    for (int w = 0; w < W; ++w)
      if ((c >> 6) == (u32)w) need[w] &= ~(1ull << (c & 63u));
  }
  u64 any = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) any |= need[w];
  if (any_idle && any != 0ull) ctl->need_flag[event & 1u] = 1u;
  for (u32 jr = 0; __ballot(jr < deg) != 0ull; ++jr) {
    bool has = false;
    u32 link = 0, chunk = kNone;
    const u32 j = jb + jr;
    if (jr < deg && any != 0ull && q.carry[j] == kNone) {
      const uint4 ir = lds_ld(q.in_rec + j);  // (link, source, cost lo, cost hi)
      const u64 *srow = reinterpret_cast<const u64 *>(rows.base + ir.y * rows.row_u4);
      u64 cand[W];
      u32 p = 0;
#pragma unroll
      for (int w = 0; w < W; ++w) {
        cand[w] = (u32)w < nw ? srow[w] & need[w] : 0ull;
        p += (u32)__popcll(cand[w]);
      }
      if (p != 0u) {
        u32 k = philox4x32_10_word0(ir.x, event, q.phase, 0u, q.seed_lo, q.seed_hi) % p;
        u32 wsel = 0;
        u64 word = 0;
        bool found = false;
#pragma unroll
        for (int w = 0; w < W; ++w) {
          const u32 c = (u32)__popcll(cand[w]);
          if (!found) {
            if (k < c) { found = true; wsel = (u32)w; word = cand[w]; }
            else k -= c;
          }
        }
        const u32 bit = kth_set_bit64(word, k);
        chunk = (wsel << 6) + bit;
#pragma unroll
        for (int w = 0; w < W; ++w)
          if (wsel == (u32)w) need[w] &= ~(1ull << bit);
        const u64 cs = ((u64)ir.w << 32) | ir.z;
        if (chunk >= q.C) {
          ctl->status = kStInternal;
          ctl->done = 1u;
        } else if (cs > kInf - 1ull - t) {
          ctl->status = kStOverflow;
          ctl->done = 1u;
        } else {
          q.carry[j] = chunk;
          q.free_at[j] = t + cs;
          has = true;
          link = ir.x;
        }
      }
    }
    if (rec.recs) append_records(rec, has, link, chunk, lane);
  }
}

// ---------------------------------------------------------------- small topologies

// One workgroup of 16 wavefronts sweeps many TEN spans without leaving the chip: the
// per-link state (chunk carried, busy-until time) and the work list live in LDS, the
// next event is a min-reduction over the busy-until times in LDS, and a span touches
// only the destinations something changed for.  Used when links, NPUs and the need slabs
// fit the LDS of one CU; such inputs are bound by the latency of a span, not by memory
// bandwidth (a heterogeneous topology has about one arrival per span).
//
// A destination d must be matched at a span only if a link into d became idle at it, or
// an in-neighbour of d gained a chunk at it (or at span 0): otherwise every idle link
// into d found no candidate the last time it was tried, its source holds nothing new and
// d needs nothing more than then.  No random number is drawn for a link without
// candidates, so skipping it cannot change the result.
//
// In LDS an idle link's busy-until time is kInf, so the next event is a plain minimum
// over the array, and a thread whose own links' minimum is not the span's time has no
// arrival to look for.  A span costs four workgroup barriers; three of them order LDS
// traffic only, so the global stores of schedule records are never waited for and the
// arrival atomics are waited for once, after the work list has been built.
//
// LDS layout (dynamic): u64 free_at[L rounded up to even] | u32 carry[L] | u32 stamp[N] |
// u32 work[N] | uint4 need[16][NP][64] | u64 next[2] | u32 counters[4] | Ctl shadow |
// and, each while it still fits: u32 pos_dst[L] | the held table without its padding lanes
// (RowsLds: N * ceil(C / 128) * 16 bytes when NP = 1) | uint4 in_rec[L], u32 in_ptr[N + 1] |
// u16 in_src[L] if in_rec does not fit.
// Link state is indexed by in-list position, as in HBM.  With the held table in LDS a span of
// a small topology touches device memory only to append schedule records.
__host__ __device__ inline size_t small_lds_bytes(u32 N, u32 L, u32 NP)
{
  size_t b = (((size_t)L + 1) & ~(size_t)1) * 8;
  b += ((size_t)L * 4 + 15) & ~(size_t)15;
  b += ((size_t)N * 4 + 15) & ~(size_t)15;
  b += ((size_t)N * 4 + 15) & ~(size_t)15;
  b += (size_t)16 * NP * 1024;
  b += 2 * 8 + 16;
  b += (sizeof(Ctl) + 15) & ~(size_t)15;
  return b;
}
constexpr size_t kLdsPerWorkgroup = 160 * 1024;  // gfx950

// Workgroup barrier that orders LDS traffic only: the wavefront's outstanding global
// stores and atomics are not waited for.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// TW > 0 (link-centric matching, NP = 1, rows of at most TW 64-bit words, held table and in-list
// records in LDS): destinations are matched one per LANE (match_destinations_by_lane).
template <int NP, int MODE, bool HELD_LDS, int TW>
__device__ __forceinline__ void small_sweep_body(const PassDev &p, const u32 *__restrict__ out_ptr,
                                                 const u32 *__restrict__ out_dst, u32 first_event,
                                                 u32 n_events, u32 stop_event, uint2 *__restrict__ recs,
                                                 u32 *__restrict__ span_first, u64 *__restrict__ event_times,
                                                 u32 dst_in_lds, u32 held_lanes, u32 rec_in_lds)
{
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const u32 Lp = (p.L + 1u) & ~1u;
  unsigned char *cur = lds_raw;
  u64 *s_free = reinterpret_cast<u64 *>(cur); cur += (size_t)Lp * 8;
  u32 *s_carry = reinterpret_cast<u32 *>(cur); cur += ((size_t)p.L * 4 + 15) & ~(size_t)15;
  u32 *s_stamp = reinterpret_cast<u32 *>(cur); cur += ((size_t)p.N * 4 + 15) & ~(size_t)15;
  u32 *s_work = reinterpret_cast<u32 *>(cur); cur += ((size_t)p.N * 4 + 15) & ~(size_t)15;
  uint4 *s_need = reinterpret_cast<uint4 *>(cur); cur += (size_t)16 * NP * 1024;
  u64 *s_next = reinterpret_cast<u64 *>(cur); cur += 2 * 8;  // next event time, one slot per span parity
  // [0] = destinations appended as out-neighbours, [1] = arrivals, [2] = schedule records
  // written so far in the pass, [3] = NPUs arrived at
  u32 *s_cnt = reinterpret_cast<u32 *>(cur); cur += 16;
  Ctl *s_ctl = reinterpret_cast<Ctl *>(cur); cur += (sizeof(Ctl) + 15) & ~(size_t)15;  // status / done of the matching code
  u32 *s_dst = reinterpret_cast<u32 *>(cur);
  if (dst_in_lds) cur += ((size_t)p.L * 4 + 15) & ~(size_t)15;
  // HELD_LDS: the held table itself, without the lanes that own no chunk (RowsLds)
  const RowsLds lrows{reinterpret_cast<uint4 *>(cur), held_lanes, (u32)NP * held_lanes};
  const RowsHbm grows{p.held, p.row_words};
  if constexpr (HELD_LDS) cur += (size_t)p.N * NP * held_lanes * 16;
  // rec_in_lds bit 0: the in-list records, bit 1: the in-list offsets, so that setting up a
  // destination costs one memory round trip less each
  uint4 *s_rec = reinterpret_cast<uint4 *>(cur); cur += (rec_in_lds & 1u) ? (size_t)p.L * 16 : 0;
  u32 *s_inptr = reinterpret_cast<u32 *>(cur); cur += (rec_in_lds & 2u) ? (((size_t)p.N + 1) * 4 + 15) & ~(size_t)15 : 0;
  // bit 2 (only without bit 0): the in-list sources alone, 16 bits each, so that a destination's
  // first source row is asked for together with its records instead of after them
  unsigned short *s_src16 = reinterpret_cast<unsigned short *>(cur);

  const u32 tid = threadIdx.x;
  const int lane = tid & 63;
  const u32 wave = tid >> 6;
  Ctl *ctl = p.ctl;
  if (ctl->done) return;
  for (u32 l = tid; l < Lp; l += 1024u) {
    const u32 c = l < p.L ? p.carry[l] : kNone;
    if (l < p.L) s_carry[l] = c;
    s_free[l] = c != kNone ? p.free_at[l] : kInf;
  }
  for (u32 n = tid; n < p.N; n += 1024u) s_stamp[n] = kNone;
  if (tid == 0) {
    s_cnt[0] = 0u; s_cnt[1] = 0u; s_cnt[3] = 0u;
    s_cnt[2] = ctl->n_rec;
    s_ctl->status = 0u; s_ctl->done = 0u;
    s_next[0] = kInf; s_next[1] = kInf;
  }
  if constexpr (HELD_LDS) {
    const uint4 *g = reinterpret_cast<const uint4 *>(p.held);
    for (u32 i = tid; i < p.N * lrows.row_u4; i += 1024u) {
      const u32 npu = i / lrows.row_u4, rem = i - npu * lrows.row_u4;
      const u32 piece = rem / held_lanes, ln = rem - piece * held_lanes;
      lrows.base[i] = g[(u64)npu * (p.row_words / 2u) + piece * 64u + ln];
    }
  }
  const RecOut rec_fwd = (recs && !p.reversed) ? RecOut{recs, &s_cnt[2]} : RecOut();
  if (dst_in_lds) {
    for (u32 l = tid; l < p.L; l += 1024u) s_dst[l] = p.pos_dst[l];
  }
  // (a branch per access rather than one pointer to either copy: see lds_ld)
  auto dst_of = [&](u32 l) { return dst_in_lds ? lds_ld(s_dst + l) : glb_ld(p.pos_dst + l); };
  PassDev q = p;  // the matching code works on the LDS copy of the link state
  q.carry = s_carry;
  q.free_at = s_free;
  q.ctl = s_ctl;
  if (rec_in_lds & 1u) {
    for (u32 l = tid; l < p.L; l += 1024u) s_rec[l] = p.in_rec[l];
    q.in_rec = s_rec;
    q.in_rec_in_lds = 1u;
  }
  if (rec_in_lds & 2u) {
    for (u32 n = tid; n <= p.N; n += 1024u) s_inptr[n] = p.in_ptr[n];
  }
  auto in_off = [&](u32 n) { return (rec_in_lds & 2u) ? lds_ld(s_inptr + n) : glb_ld(p.in_ptr + n); };
  if (rec_in_lds & 4u) {
    for (u32 l = tid; l < p.L; l += 1024u) s_src16[l] = (unsigned short)p.in_src[l];
    q.in_src16 = s_src16;
  }
  u64 t = ctl->next_t[first_event & 1u];
  u64 remaining = ctl->remaining;
  u32 e = first_event;
  bool finished = false;  // uniform
  __syncthreads();

  // a thread owns the link pairs (2*tid + 2048*i, +1); own_min = earliest busy-until of them
  auto own_min = [&]() {
    u64 m = kInf;
    for (u32 l = tid * 2u; l < Lp; l += 2048u) {
      const ulonglong2 f = *reinterpret_cast<const ulonglong2 *>(&s_free[l]);
      m = f.x < m ? f.x : m;
      m = f.y < m ? f.y : m;
    }
    return m;
  };
  u64 lm = own_min();

  for (; e < first_event + n_events; ++e) {
    // the span's records (a forward pass: its matches; a reversed one: its arrivals) begin here
    if (tid == 0 && event_times) { event_times[e - first_event] = t; span_first[e - first_event] = s_cnt[2]; }
    // ---- arrivals at t (a3): the NPUs a chunk arrived at start the work list
    if (lm == t) {
      for (u32 l2 = tid * 2u; l2 < Lp; l2 += 2048u) {
#pragma unroll
        for (u32 k = 0; k < 2u; ++k) {
          const u32 l = l2 + k;
          if (s_free[l] != t) continue;
          const u32 c = s_carry[l];
          const u32 d = dst_of(l);
          if constexpr (HELD_LDS) atomicOr(lrows.word_of(d, c, (u32)NP), 1ull << (c & 63u));
          else atomicOr(&p.held[(u64)d * p.row_words + phys_word(c >> 6, p.NP)], 1ull << (c & 63u));
          s_carry[l] = kNone;
          s_free[l] = kInf;
          atomicAdd(&s_cnt[1], 1u);
          if (p.reversed && recs) recs[atomicAdd(&s_cnt[2], 1u)] = make_uint2(p.in_link[l], c);
          if (atomicExch(&s_stamp[d], e) != e) s_work[atomicAdd(&s_cnt[3], 1u)] = d;
        }
      }
    }
    lds_barrier();
    // ---- every NPU whose state changed, and its out-neighbours, go on the work list
    //      once: one wavefront per NPU arrived at, one lane per out-neighbour
    const u32 n_arr = s_cnt[3];
    for (u32 i = wave; i < n_arr; i += 16u) {
      const u32 a = uniform(s_work[i]);
      const u32 ob = out_ptr[a], oe = out_ptr[a + 1];
      for (u32 j = ob + (u32)lane; j < oe; j += 64u) {
        const u32 o = out_dst[j];
        if (atomicExch(&s_stamp[o], e) != e) s_work[n_arr + atomicAdd(&s_cnt[0], 1u)] = o;
      }
    }
    __syncthreads();  // also: the arrival atomics have been performed
    remaining -= (u64)s_cnt[1];
    // ---- all postconditions satisfied? (a4)
    if (remaining == 0ull) {
      if (tid == 0) { ctl->T = t; ctl->n_events = e; ctl->done = 1u; }
      finished = true;
      break;
    }
    if (e == stop_event) break;  // prefix run: time reached is next_t[e & 1]
    // ---- matching (a5-a7) for the destinations on the work list (all of them at span 0)
    const u32 n_work = (e == 0u) ? p.N : n_arr + s_cnt[0];
    if constexpr (TW > 0) {
      for (u32 i0 = wave * 64u; i0 < n_work; i0 += 1024u) {
        const u32 i = i0 + (u32)lane;
        const bool active = i < n_work;
        const u32 d = active ? ((e == 0u) ? i : s_work[i]) : 0u;
        match_destinations_by_lane<(TW > 0 ? TW : 1)>(q, lrows, s_inptr, d, active, e, t, rec_fwd, lane);
      }
    } else
    for (u32 i = wave; i < n_work; i += 16u) {
      const u32 d = uniform((e == 0u) ? i : s_work[i]);
      const u32 jb = in_off(d), je = in_off(d + 1u);
      uint4 *my_need = s_need + wave * NP * 64;
      if constexpr (MODE == 0) {
        if constexpr (HELD_LDS) (void)match_destination<NP, true>(q, lrows, d, jb, je, e, t, nullptr, lane, my_need, rec_fwd);
        else (void)match_destination<NP, true>(q, grows, d, jb, je, e, t, nullptr, lane, my_need, rec_fwd);
      } else {
        if constexpr (HELD_LDS)
          (void)match_destination_pairs<NP, 8>(q, lrows, d, jb, je, e, t, nullptr, lane, my_need, MODE == 2, rec_fwd);
        else
          (void)match_destination_pairs<NP, 8>(q, grows, d, jb, je, e, t, nullptr, lane, my_need, MODE == 2, rec_fwd);
      }
    }
    lds_barrier();
    // ---- next span = earliest end of a transfer in flight (a8), reduced in LDS
    lm = own_min();
    const u64 wm = wave_min64(lm);
    if (lane == 0 && wm != kInf) atomicMin(&s_next[e & 1u], wm);
    if (tid == 0) { s_cnt[0] = 0u; s_cnt[1] = 0u; s_cnt[3] = 0u; s_next[(e + 1u) & 1u] = kInf; }
    lds_barrier();
    const u64 m = s_next[e & 1u];
    if (s_ctl->done) {  // an overflow flagged during matching
      if (tid == 0) { ctl->status = s_ctl->status; ctl->done = 1u; }
      finished = true;
      break;
    }
    if (m == kInf) {  // chunks missing and nothing in flight
      if (tid == 0) { ctl->status = kStUnreachable; ctl->done = 1u; }
      finished = true;
      break;
    }
    t = m;
  }
  // ---- hand the state back for the next launch
  __syncthreads();
  for (u32 l = tid; l < p.L; l += 1024u) { p.free_at[l] = s_free[l]; p.carry[l] = s_carry[l]; }
  if constexpr (HELD_LDS) {
    uint4 *g = reinterpret_cast<uint4 *>(p.held);
    for (u32 i = tid; i < p.N * lrows.row_u4; i += 1024u) {
      const u32 npu = i / lrows.row_u4, rem = i - npu * lrows.row_u4;
      const u32 piece = rem / held_lanes, ln = rem - piece * held_lanes;
      g[(u64)npu * (p.row_words / 2u) + piece * 64u + ln] = lrows.base[i];
    }
  }
  if (tid == 0 && !finished) ctl->next_t[e & 1u] = t;
  if (tid == 0) { ctl->remaining = remaining; ctl->n_rec = s_cnt[2]; }
}

template <int NP, int MODE, bool HELD_LDS, int TW>
__global__ __launch_bounds__(1024) void small_sweep_kernel(PassDev p, const u32 *__restrict__ out_ptr,
                                                           const u32 *__restrict__ out_dst, u32 first_event,
                                                           u32 n_events, u32 stop_event,
                                                           uint2 *__restrict__ recs, u32 *__restrict__ span_first,
                                                           u64 *__restrict__ event_times, u32 dst_in_lds, u32 held_lanes,
                                                           u32 rec_in_lds)
{
  small_sweep_body<NP, MODE, HELD_LDS, TW>(p, out_ptr, out_dst, first_event, n_events, stop_event, recs, span_first,
                                           event_times, dst_in_lds, held_lanes, rec_in_lds);
}

// Many independent passes at once (one per workgroup, each with its own seed, rows, link
// state and control block): only the collective times are wanted, no schedule is kept.
template <int NP, int MODE, bool HELD_LDS, int TW>
__global__ __launch_bounds__(1024) void small_sweep_batch_kernel(const SmallJob *__restrict__ jobs, u32 first_event,
                                                                 u32 n_events, u32 dst_in_lds, u32 held_lanes,
                                                                 u32 rec_in_lds)
{
  // (The job's pointers are read from memory, so the compiler cannot tell device memory from
  // LDS behind them and some of this kernel's accesses stay flat instructions.)
  const SmallJob &j = jobs[blockIdx.x];
  small_sweep_body<NP, MODE, HELD_LDS, TW>(j.p, j.out_ptr, j.out_dst, first_event, n_events, 0xFFFFFFFFu, nullptr,
                                           nullptr, nullptr, dst_in_lds, held_lanes, rec_in_lds);
}

// ---------------------------------------------------------------- last stretch of a pass: few destinations left

// Per-span launches, link-centric matching, dense schedule rows: once at most kTailSlots
// destinations are left in the processing order (on a mesh the corner NPUs, whose two or three
// incoming links need thousands of spans more than everyone else's), ONE workgroup sweeps many
// spans per launch, one wavefront per destination and one lane per incoming link (in-degrees up
// to 64).  The lane keeps its link's state (chunk carried, busy-until time) in registers and the
// wavefront its destination's need row in LDS for the whole launch: an arrival moves a chunk
// from "in flight" to "held", which leaves need = ~held & ~inflight as it is, and a match clears
// its bit, so after the set-up a span costs no read of d's own row, of the records or of the
// link state.  Arrivals are atomics on the held table in device memory as in arrive_kernel; a
// workgroup barrier separates them from the matching, whose source rows may belong to another
// wavefront's destination.  Span times, schedule rows, the control block and (on return) the
// link state and the next event time are written exactly as arrive_kernel and match_kernel
// write them, so the host may switch between the two forms at any span.
// rows0 / times0: schedule row and time slot of span first_event; the launch stays inside one
// row segment, row_stride apart.
template <int NP>
__global__ __launch_bounds__(64 * kTailSlots) void tail_sweep_kernel(PassDev p, u32 first_event, u32 n_spans,
                                                                     u32 *__restrict__ rows0, u64 row_stride,
                                                                     u64 *__restrict__ times0)
{
  constexpr int NW = 2 * NP;
  extern __shared__ __align__(16) unsigned char tail_lds[];  // kTailSlots need rows of NP KiB
  __shared__ u64 s_min[2][kTailSlots];
  __shared__ u32 s_need[2][kTailSlots];
  const int lane = threadIdx.x & 63;
  const u32 w = uniform(threadIdx.x >> 6);
  Ctl *ctl = p.ctl;
  if (ctl->done) return;
  uint4 *need_lds = reinterpret_cast<uint4 *>(tail_lds) + w * NP * 64;
  const RowsHbm rows{p.held, p.row_words};
  const bool active = w < p.n_slots;
  u32 d = 0, jb = 0, je = 0;
  if (active) {
    const uint4 sr = p.slot_rec[w];
    d = uniform(sr.x); jb = uniform(sr.y); je = uniform(sr.z);
  }
  const u32 j = jb + (u32)lane;
  const bool valid = active && j < je;
  u32 link = 0, src = 0, cr = kNone;
  u64 cs = 0, fa = 0;
  if (valid) {
    const uint4 rec = p.in_rec[j];
    link = rec.x; src = rec.y; cs = ((u64)rec.w << 32) | rec.z;
    cr = p.carry[j];
    fa = p.free_at[j];
  }
  if (active) {
    // need = ~held[d] & ~inflight[d] (as match_destination sets it up)
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      uint4 v = rows.load(d, i, lane);
      v.x = ~v.x; v.y = ~v.y; v.z = ~v.z; v.w = ~v.w;
      need_lds[i * 64 + lane] = v;
    }
    if (cr != kNone) {
      const u32 wd = cr >> 6;
      const u32 ln = wd / (u32)NW;
      const u32 iw = wd - ln * (u32)NW;
      u32 *ptr = reinterpret_cast<u32 *>(&need_lds[(iw >> 1) * 64u + ln]) + ((iw & 1u) * 2u + ((cr >> 5) & 1u));
      atomicAnd(ptr, ~(1u << (cr & 31u)));
    }
  }
  u64 t = next_event_time(p, first_event);  // time of the span at hand, kInf: nothing in flight
  u64 t_before = ctl->now;
  u32 need_before = first_event != 0u ? ctl->need_flag[(first_event - 1u) & 1u] : 1u;
  u32 i = 0;
  bool ended = false;  // uniform
  for (; i < n_spans; ++i) {
    const u32 event = first_event + i;
    if (threadIdx.x == 0) {  // as arrive_kernel
      ctl->next_t[event & 1u] = t;
      if (t == kInf) {
        if (event != 0u && need_before == 0u) {
          ctl->T = t_before;
          ctl->n_events = event - 1u;
        } else {
          ctl->status = kStUnreachable;
        }
        ctl->done = 1u;
      } else {
        times0[i] = t;
        ctl->now = t;
        ctl->next_t[(event + 1u) & 1u] = kInf;
      }
    }
    if (t == kInf) { ended = true; break; }
    u32 *row = rows0 + (u64)i * row_stride;
    // a3: arrivals on this wavefront's links
    if (valid && cr != kNone && fa == t) {
      atomicOr(&p.held[(u64)d * p.row_words + phys_word(cr >> 6, p.NP)], 1ull << (cr & 63u));
      if (p.reversed) row[link] = cr;  // rows are pre-filled with kNone
      cr = kNone;
    }
    __syncthreads();  // the arrival atomics of all wavefronts have been performed
    // a5-a7: matching
    const u64 idle = __ballot(valid && cr == kNone);
    u32 acc = 0;
    if (idle != 0ull) {
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        const uint4 v = need_lds[q * 64 + lane];
        acc |= v.x | v.y | v.z | v.w;
      }
    }
    const bool need_now = __ballot(acc != 0u) != 0ull;
    // what match_destination calls need_any: chunks d does not hold, in flight or not
    const bool need_any = need_now || __ballot(valid && cr != kNone) != 0ull;
    u32 res = kNone;
    if (idle != 0ull && need_now) {
      u32 r = 0;
      res = draw_chunks<NP>(rows, src, r, idle, need_lds, lane, [&]() {
        r = philox4x32_10_word0(link, event, p.phase, 0u, p.seed_lo, p.seed_hi);  // behind the first row request
        return true;
      });
    }
    if (idle != 0ull && !need_any && p.dest_done && lane == 0) p.dest_done[d] = 1u;
    if (valid && res != kNone) {
      if (res >= p.C) {
        ctl->status = kStInternal;
        ctl->done = 1u;
      } else if (cs > kInf - 1ull - t) {
        ctl->status = kStOverflow;
        ctl->done = 1u;
      } else {
        if (!p.reversed) row[link] = res;
        cr = res;
        fa = t + cs;
      }
    }
    // a8: next span = earliest end of a transfer in flight; the buffers alternate, so one
    // barrier per reduction is enough
    const u64 m = wave_min64((valid && cr != kNone) ? fa : kInf);
    if (lane == 0) {
      s_min[i & 1u][w] = m;
      s_need[i & 1u][w] = (idle != 0ull && need_any) ? 1u : 0u;
    }
    lds_barrier();
    const u64 tn = wave_min64((u32)lane < kTailSlots ? s_min[i & 1u][lane] : kInf);
    const u32 nd = __ballot((u32)lane < kTailSlots && s_need[i & 1u][lane] != 0u) != 0ull ? 1u : 0u;
    if (threadIdx.x == 0) ctl->need_flag[event & 1u] = nd;
    t_before = t;
    need_before = nd;
    t = tn;
  }
  // hand the state back: the link state, and the next event time where arrive_kernel looks for it
  if (valid) {
    p.carry[j] = cr;
    p.free_at[j] = fa;
  }
  if (!ended && threadIdx.x < kNextSlots)
    p.next_slots[((first_event + i) & 1u) * kNextSlots + threadIdx.x] = threadIdx.x == 0 ? t : kInf;
}

// ---------------------------------------------------------------- epilogue

__device__ __forceinline__ u64 mix_record(u64 t, u32 link, u32 chunk)
{
  u64 h = t ^ ((((u64)link << 32) | (u64)chunk) * 0x9E3779B97F4A7C15ull);
  h ^= h >> 33; h *= 0xFF51AFD7ED558CCDull;
  h ^= h >> 33; h *= 0xC4CEB9FE1A85EC53ull;
  h ^= h >> 33;
  return h;
}

// grid = n_rows * ceil(L / 2048) blocks; every block covers 2048 links of one schedule row;
// digest: kDigestSlots partial sums, 128 bytes apart, to be added up by the caller
__global__ __launch_bounds__(256) void row_stats_kernel(const u32 *__restrict__ rows, u32 L,
                                                        const u64 *__restrict__ row_time, u64 t_base,
                                                        u32 reversed, u32 blocks_per_row,
                                                        u32 *__restrict__ row_count,
                                                        u64 *__restrict__ digest)
{
  const u32 row = blockIdx.x / blocks_per_row;
  const u32 seg = blockIdx.x - row * blocks_per_row;
  const u64 rt = row_time[row];
  const u64 t = reversed ? t_base - rt : rt + t_base;
  const u32 *r = rows + (u64)row * L;
  u32 n = 0;
  u64 dg = 0;
  const u32 first = seg * 2048u;
#pragma unroll
  for (u32 i = 0; i < 8; ++i) {
    const u32 l = first + i * 256u + threadIdx.x;
    if (l < L) {
      const u32 c = r[l];
      if (c != kNone) { n++; dg += mix_record(t, l, c); }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    n += (u32)__shfl_xor((int)n, off, 64);
    const u32 lo = (u32)__shfl_xor((int)(u32)dg, off, 64);
    const u32 hi = (u32)__shfl_xor((int)(u32)(dg >> 32), off, 64);
    dg += ((u64)hi << 32) | lo;
  }
  // one atomic per workgroup; the digest goes to one of kDigestSlots partial sums, each on
  // a cache line of its own (a single address would serialise every workgroup of the grid)
  __shared__ u32 s_n[4];
  __shared__ u64 s_dg[4];
  if ((threadIdx.x & 63u) == 0) { s_n[threadIdx.x >> 6] = n; s_dg[threadIdx.x >> 6] = dg; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const u32 nb = s_n[0] + s_n[1] + s_n[2] + s_n[3];
    if (nb) {
      atomicAdd(&row_count[row], nb);
      atomicAdd(&digest[(blockIdx.x % kDigestSlots) * 16u], s_dg[0] + s_dg[1] + s_dg[2] + s_dg[3]);
    }
  }
}

// ---- compact schedules of the single-workgroup kernel

// One workgroup per span: brings the span's records into ascending link id (a link starts at
// most one transfer per span, so the records scatter into a row of L entries in LDS and are
// read back in order) and adds their digest contributions.  t = the span's time (forward
// pass, offset t_base) or t_base minus it (reversed pass: the records are arrivals).
__global__ __launch_bounds__(256) void compact_epilogue_kernel(uint2 *__restrict__ recs,
                                                               const u32 *__restrict__ span_first, u32 L,
                                                               const u64 *__restrict__ span_time, u64 t_base,
                                                               u32 reversed, u64 *__restrict__ digest)
{
  extern __shared__ __align__(16) unsigned char compact_lds[];
  u32 *row = reinterpret_cast<u32 *>(compact_lds);  // [L]
  __shared__ u32 s_off[257];
  __shared__ u64 s_dg[4];
  const u32 e = blockIdx.x;
  const u32 b0 = span_first[e], n = span_first[e + 1] - b0;
  if (n == 0) return;
  const u64 rt = span_time[e];
  const u64 t = reversed ? t_base - rt : rt + t_base;
  u64 dg = 0;
  for (u32 i = threadIdx.x; i < n; i += 256u) {
    const uint2 r = recs[b0 + i];
    dg += mix_record(t, r.x, r.y);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const u32 lo = (u32)__shfl_xor((int)(u32)dg, off, 64);
    const u32 hi = (u32)__shfl_xor((int)(u32)(dg >> 32), off, 64);
    dg += ((u64)hi << 32) | lo;
  }
  if ((threadIdx.x & 63u) == 0) s_dg[threadIdx.x >> 6] = dg;
  if (n > 1) {  // uniform over the workgroup
    for (u32 l = threadIdx.x; l < L; l += 256u) row[l] = kNone;
    __syncthreads();
    for (u32 i = threadIdx.x; i < n; i += 256u) {
      const uint2 r = recs[b0 + i];
      row[r.x] = r.y;
    }
    __syncthreads();
    // thread k owns links [k*per, (k+1)*per): count, exclusive prefix over the threads, write back
    const u32 per = (L + 255u) / 256u;
    const u32 l0 = threadIdx.x * per, l1 = l0 + per < L ? l0 + per : L;
    u32 cnt = 0;
    for (u32 l = l0; l < l1; ++l) cnt += row[l] != kNone ? 1u : 0u;
    s_off[threadIdx.x + 1] = cnt;
    if (threadIdx.x == 0) s_off[0] = 0u;
    __syncthreads();
    if (threadIdx.x == 0)
      for (u32 k = 1; k <= 256u; ++k) s_off[k] += s_off[k - 1];
    __syncthreads();
    u32 w = b0 + s_off[threadIdx.x];
    for (u32 l = l0; l < l1; ++l) {
      const u32 c = row[l];
      if (c != kNone) recs[w++] = make_uint2(l, c);
    }
  } else {
    __syncthreads();
  }
  if (threadIdx.x == 0) atomicAdd(&digest[(blockIdx.x % kDigestSlots) * 16u], s_dg[0] + s_dg[1] + s_dg[2] + s_dg[3]);
}

__global__ __launch_bounds__(256) void compact_link_count_kernel(const uint2 *__restrict__ recs, u32 n_rec,
                                                                 u64 *__restrict__ counts)
{
  const u32 i = blockIdx.x * 256u + threadIdx.x;
  if (i < n_rec) atomicAdd(&counts[recs[i].x], 1ull);
}

// One workgroup per span of a reversed pass: every record arrived in this span; it started in
// the span whose time is the arrival time minus the link's cost.
__global__ __launch_bounds__(256) void compact_start_span_kernel(const uint2 *__restrict__ recs,
                                                                 const u32 *__restrict__ span_first,
                                                                 const u64 *__restrict__ span_time,
                                                                 const u64 *__restrict__ cost, u32 *__restrict__ counts)
{
  const u32 e = blockIdx.x;
  const u32 b0 = span_first[e], n = span_first[e + 1] - b0;
  const u64 t_arr = span_time[e];
  for (u32 i = threadIdx.x; i < n; i += 256u) {
    const u64 t_start = t_arr - cost[recs[b0 + i].x];
    u32 lo = 0, hi = e;  // the first span with time >= t_start
    while (lo < hi) {
      const u32 mid = (lo + hi) >> 1;
      if (span_time[mid] < t_start) lo = mid + 1u;
      else hi = mid;
    }
    atomicAdd(&counts[lo], 1u);
  }
}

// grid = (ceil(L/256), n_rows): a thread looks at one entry of one schedule row of a reversed
// pass.  The row index is the span the chunk ARRIVED in; the span it was matched in is the one
// whose time is the arrival time minus the link's cost (every transfer starts at a span's
// time), found by binary search in the ascending span times.  Lanes of a wavefront that
// found the same span add to its counter once.
__global__ __launch_bounds__(256) void start_span_count_kernel(const u32 *__restrict__ rows, u32 first_row, u32 L,
                                                               const u64 *__restrict__ row_time,
                                                               const u64 *__restrict__ cost,
                                                               u32 *__restrict__ counts)
{
  const u32 l = blockIdx.x * 256u + threadIdx.x;
  const u32 r = first_row + blockIdx.y;
  u32 idx = kNone;
  if (l < L && rows[(u64)blockIdx.y * L + l] != kNone) {
    const u64 t_start = row_time[r] - cost[l];
    u32 lo = 0, hi = r;  // the first span with time >= t_start
    while (lo < hi) {
      const u32 mid = (lo + hi) >> 1;
      if (row_time[mid] < t_start) lo = mid + 1u;
      else hi = mid;
    }
    idx = lo;
  }
  u64 todo = __ballot(idx != kNone);
  const int lane = threadIdx.x & 63;
  while (todo) {
    const u32 first = (u32)__ffsll((long long)todo) - 1u;
    const u32 v = read_lane(idx, first);
    const u64 same = __ballot(idx == v);
    if ((u32)lane == first) atomicAdd(&counts[v], (u32)__popcll(same));
    todo &= ~same;
  }
}

// grid = (ceil(L/256), ceil(n_rows/64)): a thread sums 64 rows of one schedule column
__global__ __launch_bounds__(256) void link_count_kernel(const u32 *__restrict__ rows, u32 n_rows, u32 L,
                                                         u64 *__restrict__ counts)
{
  const u32 l = blockIdx.x * 256u + threadIdx.x;
  if (l >= L) return;
  const u32 r0 = blockIdx.y * 64u;
  const u32 r1 = r0 + 64u < n_rows ? r0 + 64u : n_rows;
  u32 n = 0;
  for (u32 r = r0; r < r1; ++r) n += rows[(u64)r * L + l] != kNone ? 1u : 0u;
  if (n) atomicAdd(&counts[l], (u64)n);
}

}  // namespace

// ---------------------------------------------------------------- launchers

void launch_link_cost(const u64 *alpha, const u64 *beta, u64 chunk_bytes, u32 L, u64 *cost,
                      u32 *overflow, hipStream_t s)
{
  if (L == 0) return;
  hipLaunchKernelGGL(link_cost_kernel, dim3((L + 255) / 256), dim3(256), 0, s, alpha, beta,
                     chunk_bytes, L, cost, overflow);
}

// ---------------------------------------------------------------- link costs without allocating
//
// Device staging of the entry point that may not allocate: the alpha and beta arrays, the
// costs and the overflow flag of up to kStaticMaxLinks links, in a file-scope device array.
// Every GPU the library runs on holds its own copy of the array (until the process ends) at
// its own address; host code never uses the array's name as an address, only the pointer
// hipGetSymbolAddress returned for the device that is current.
static __device__ __align__(256) unsigned char scratch[3ull * kStaticMaxLinks * 8ull + 256ull];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// the array's address on the current device, looked up once per device
hipError_t static_scratch(unsigned char **ptr)
{
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = static_cast<unsigned char *>(g_scratch_ptr[dev]);
  return hipSuccess;
}

__global__ void clear_word_kernel(u32 *w) { *w = 0u; }

}  // namespace

hipError_t link_cost_static(const u64 *h_alpha, const u64 *h_beta, u64 chunk_bytes, u32 L, u64 *h_cost,
                            u32 *h_overflow, hipStream_t s)
{
  if (L == 0 || L > kStaticMaxLinks) return hipErrorInvalidValue;
  unsigned char *base = nullptr;
  hipError_t e = static_scratch(&base);
  if (e != hipSuccess) return e;
  u64 *d_alpha = reinterpret_cast<u64 *>(base);
  u64 *d_beta = d_alpha + kStaticMaxLinks;
  u64 *d_cost = d_beta + kStaticMaxLinks;
  u32 *d_ovf = reinterpret_cast<u32 *>(d_cost + kStaticMaxLinks);
  const size_t bytes = (size_t)L * 8;
  if ((e = hipMemcpyAsync(d_alpha, h_alpha, bytes, hipMemcpyHostToDevice, s)) != hipSuccess) return e;
  if ((e = hipMemcpyAsync(d_beta, h_beta, bytes, hipMemcpyHostToDevice, s)) != hipSuccess) return e;
  // the array keeps the last call's contents: the flag has to start at zero (a fill kernel
  // rather than a memset node, so that the sequence may also be captured into a graph)
  hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, s, d_ovf);
  hipLaunchKernelGGL(link_cost_kernel, dim3((L + 255) / 256), dim3(256), 0, s, d_alpha, d_beta, chunk_bytes, L,
                     d_cost, d_ovf);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if ((e = hipMemcpyAsync(h_cost, d_cost, bytes, hipMemcpyDeviceToHost, s)) != hipSuccess) return e;
  if ((e = hipMemcpyAsync(h_overflow, d_ovf, 4, hipMemcpyDeviceToHost, s)) != hipSuccess) return e;
  return hipStreamSynchronize(s);
}

void launch_init_pass(const PassDev &p, hipStream_t s)
{
  const u64 total = (u64)p.N * p.row_words;
  hipLaunchKernelGGL(init_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
  hipLaunchKernelGGL(init_links_kernel, dim3((p.L + 255) / 256 + (p.L == 0)), dim3(256), 0, s, p);
}

void launch_arrive(const PassDev &p, u32 event, u64 *event_time_slot, u32 *sched_row, uint2 *recs, u32 *first_slot,
                   hipStream_t s)
{
  // few destinations left in the processing order: only their in-lists are looked at
  const u64 slot_threads = (u64)p.n_slots * p.max_deg;
  if (p.n_slots < p.N && p.max_deg >= 1u && p.max_deg <= 64u && slot_threads * 2ull <= (u64)p.L) {
    const u32 blocks = (u32)((slot_threads + 255ull) / 256ull);
    hipLaunchKernelGGL(arrive_slots_kernel, dim3(blocks ? blocks : 1u), dim3(256), 0, s, p, event, event_time_slot,
                       sched_row, recs, first_slot, p.max_deg);
    return;
  }
  hipLaunchKernelGGL(arrive_kernel, dim3((p.L + 255) / 256), dim3(256), 0, s, p, event,
                     event_time_slot, sched_row, recs, first_slot);
}

void launch_match_compact(const PassDev &p, u32 event, uint2 *recs, u32 *first_next, u32 mode, hipStream_t s)
{
  const u32 n_wg = (p.n_slots + 3u) / 4u;
  const dim3 grid(8u * ((n_wg + 7u) / 8u + (n_wg == 0u)), 1, 1), block(256);
#define TACOS_MATCH_COMPACT(NP_)                                                                              \
  if (mode == 0) hipLaunchKernelGGL((match_compact_kernel<NP_, 0>), grid, block, 0, s, p, event, recs, first_next);      \
  else if (mode == 1) hipLaunchKernelGGL((match_compact_kernel<NP_, 1>), grid, block, 0, s, p, event, recs, first_next); \
  else hipLaunchKernelGGL((match_compact_kernel<NP_, 2>), grid, block, 0, s, p, event, recs, first_next)
  switch (p.NP) {
    case 1: TACOS_MATCH_COMPACT(1); break;
    case 2: TACOS_MATCH_COMPACT(2); break;
    case 3: TACOS_MATCH_COMPACT(3); break;
    case 4: TACOS_MATCH_COMPACT(4); break;
    case 5: TACOS_MATCH_COMPACT(5); break;
    case 6: TACOS_MATCH_COMPACT(6); break;
    case 7: TACOS_MATCH_COMPACT(7); break;
    case 8: TACOS_MATCH_COMPACT(8); break;
    default: break;  // the host uses this path for rows of at most 8 pieces only
  }
#undef TACOS_MATCH_COMPACT
}

// Shapes whose register planes fit without spilling at three or more wavefronts per SIMD
// (a lane's share of a row is 4*NP dwords per plane): measured from the compiler's register
// counts; the other shapes re-stream the rows.
constexpr bool planes_fit(int np, int deg) { return (deg == 4 && np <= 6) || (deg == 6 && np <= 5) || (deg == 8 && np <= 4); }

template <int MODE, int DEG> static void launch_match_mode(const PassDev &p, u32 event, u32 *sched_row, hipStream_t s)
{
  const u32 n_wg = (p.n_slots + 3u) / 4u;
  const dim3 grid(8u * ((n_wg + 7u) / 8u + (n_wg == 0u)), 1, 1), block(256);
#define TACOS_MATCH(NP_)                                                                               \
  if constexpr (planes_fit(NP_, DEG))                                                                  \
    hipLaunchKernelGGL((match_kernel<NP_, MODE, DEG>), grid, block, 0, s, p, event, sched_row);        \
  else                                                                                                 \
    hipLaunchKernelGGL((match_kernel<NP_, MODE, 0>), grid, block, 0, s, p, event, sched_row)
  switch (p.NP) {
    case 1: TACOS_MATCH(1); break;
    case 2: TACOS_MATCH(2); break;
    case 3: TACOS_MATCH(3); break;
    case 4: TACOS_MATCH(4); break;
    case 5: TACOS_MATCH(5); break;
    case 6: TACOS_MATCH(6); break;
    case 7: TACOS_MATCH(7); break;
    case 8: TACOS_MATCH(8); break;
    default:
      // rows of 9..kMaxRegisterPieces pieces (up to 122,880 chunks), link-centric only: still whole
      // rows in registers, at two to four wavefronts per SIMD (16 pieces would need more than the
      // 64 KiB of LDS a kernel may declare for its four need rows)
      if constexpr (MODE == 0 && DEG == 0) {
        switch (p.NP) {
          case 9: TACOS_MATCH(9); break;
          case 10: TACOS_MATCH(10); break;
          case 11: TACOS_MATCH(11); break;
          case 12: TACOS_MATCH(12); break;
          case 13: TACOS_MATCH(13); break;
          case 14: TACOS_MATCH(14); break;
          case 15: TACOS_MATCH(15); break;
          default: break;  // rejected by the host before any launch
        }
      }
      break;
  }
#undef TACOS_MATCH
}

// postcondition-centric: the register-plane variant that covers the largest in-degree of the pass
template <int MODE> static void launch_match_pairs(const PassDev &p, u32 event, u32 *sched_row, hipStream_t s)
{
  if (p.max_deg <= 4) launch_match_mode<MODE, 4>(p, event, sched_row, s);
  else if (p.max_deg <= 6) launch_match_mode<MODE, 6>(p, event, sched_row, s);
  else if (p.max_deg <= 8) launch_match_mode<MODE, 8>(p, event, sched_row, s);
  else launch_match_mode<MODE, 0>(p, event, sched_row, s);
}

void launch_match(const PassDev &p, u32 event, u32 *sched_row, u32 mode, hipStream_t s)
{
  if (p.NP > kMaxRegisterPieces) {  // streamed rows (link-centric only; the host rejects the rest)
    const u32 n_wg = (p.n_slots + 3u) / 4u;
    const dim3 grid(8u * ((n_wg + 7u) / 8u + (n_wg == 0u)), 1, 1), block(256);
    const size_t lds = (size_t)4 * p.NP * 1024;
    // more than 64 KiB of dynamic LDS has to be allowed explicitly
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&match_kernel_streamed),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(match_kernel_streamed, grid, block, lds, s, p, event, sched_row);
    return;
  }
  if (mode == 0) launch_match_mode<0, 0>(p, event, sched_row, s);
  else if (mode == 1) launch_match_pairs<1>(p, event, sched_row, s);
  else launch_match_pairs<2>(p, event, sched_row, s);
}

hipError_t launch_tail_sweep(const PassDev &p, u32 first_event, u32 n_spans, u32 *rows0, u64 row_stride, u64 *times0,
                             hipStream_t s)
{
  if (p.n_slots > kTailSlots || p.max_deg > 64u || p.NP > 8u || n_spans == 0u) return hipErrorInvalidValue;
  const size_t lds = (size_t)kTailSlots * p.NP * 1024;
#define TACOS_TAIL(NP_)                                                                                      \
  {                                                                                                          \
    /* more than 64 KiB of dynamic LDS has to be allowed explicitly */                                       \
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tail_sweep_kernel<NP_>),        \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
    if (e != hipSuccess) return e;                                                                           \
    hipLaunchKernelGGL((tail_sweep_kernel<NP_>), dim3(1), dim3(64 * kTailSlots), lds, s, p, first_event, n_spans, rows0, \
                       row_stride, times0);                                                                  \
    return hipGetLastError();                                                                                \
  }
  switch (p.NP) {
    case 1: TACOS_TAIL(1)
    case 2: TACOS_TAIL(2)
    case 3: TACOS_TAIL(3)
    case 4: TACOS_TAIL(4)
    case 5: TACOS_TAIL(5)
    case 6: TACOS_TAIL(6)
    case 7: TACOS_TAIL(7)
    case 8: TACOS_TAIL(8)
    default: return hipErrorInvalidValue;
  }
#undef TACOS_TAIL
}

void launch_uniform_init(const PassDev &p, const UniformDev &u, uint32_t mode, hipStream_t s)
{
  (void)mode;
  hipLaunchKernelGGL(uniform_init_kernel, dim3((p.L + 255) / 256 + (p.L == 0)), dim3(256), 0, s, p, u);
}

// copy of the held table (200 MB on the large meshes, once per pass)
__global__ __launch_bounds__(256) void copy_table_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, u64 n)
{
  for (u64 i = (u64)blockIdx.x * 256u + threadIdx.x; i < n; i += (u64)gridDim.x * 256u) dst[i] = src[i];
}

void launch_links_to_uniform(const PassDev &p, const UniformDev &u, u32 event, u32 *sched_row, hipStream_t s)
{
  const u64 n16 = (u64)p.N * p.row_words / 2u;  // rows are multiples of 1 KiB
  hipLaunchKernelGGL(copy_table_kernel, dim3(256 * 8), dim3(256), 0, s, reinterpret_cast<uint4 *>(u.held[(event + 1u) & 1u]),
                     reinterpret_cast<const uint4 *>(u.held[event & 1u]), n16);
  hipLaunchKernelGGL(links_to_uniform_flags_kernel, dim3(1), dim3(1), 0, s, p.ctl, event);
  hipLaunchKernelGGL(links_to_uniform_kernel, dim3((p.L + 255) / 256 + (p.L == 0)), dim3(256), 0, s, p, u, event, sched_row);
}

void launch_uniform_handover(const PassDev &p, const UniformDev &u, u32 event, hipStream_t s)
{
  hipLaunchKernelGGL(uniform_handover_kernel, dim3((p.L + 255) / 256 + (p.L == 0)), dim3(256), 0, s, p, u, event);
}

void launch_match_uniform(const PassDev &p, const UniformDev &u, u32 event, u32 *row, u32 *row_next,
                          u64 *event_time_slot, u32 mode, hipStream_t s)
{
  (void)mode;  // link-centric only so far; the host sends the other orders down the general path
  const u32 n_wg = (p.n_slots + 3u) / 4u;
  const dim3 grid(8u * ((n_wg + 7u) / 8u + (n_wg == 0u)), 1, 1), block(256);
#define TACOS_UNIFORM(NP_) \
  hipLaunchKernelGGL((match_uniform_kernel<NP_, 0>), grid, block, 0, s, p, u, event, row, row_next, event_time_slot)
  switch (p.NP) {
    case 1: TACOS_UNIFORM(1); break;
    case 2: TACOS_UNIFORM(2); break;
    case 3: TACOS_UNIFORM(3); break;
    case 4: TACOS_UNIFORM(4); break;
    case 5: TACOS_UNIFORM(5); break;
    case 6: TACOS_UNIFORM(6); break;
    case 7: TACOS_UNIFORM(7); break;
    case 8: TACOS_UNIFORM(8); break;
    default: break;  // the host uses this path for rows of at most 8 pieces only
  }
#undef TACOS_UNIFORM
}

// LDS a workgroup may ask for on the current device (what the host's fit test compares
// against), never more than the 160 KiB of a gfx950 compute unit.
static size_t lds_limit()
{
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || v <= 0)
    return 64 * 1024;
  return (size_t)v < kLdsPerWorkgroup ? (size_t)v : kLdsPerWorkgroup;
}

// LDS of one single-workgroup launch: the link state, and while they still fit the held table
// (without its padding lanes) and the link destinations.
static size_t small_launch_lds(const PassDev &p, u32 *dst_in_lds, u32 *held_lanes, u32 *rec_in_lds)
{
  size_t lds = small_lds_bytes(p.N, p.L, p.NP);
  const size_t limit = lds_limit();
  const u32 lanes = (p.C + 128u * p.NP - 1u) / (128u * p.NP);
  const size_t held_bytes = (size_t)p.N * p.NP * lanes * 16;
  const size_t dst_bytes = ((size_t)p.L * 4 + 15) & ~(size_t)15;
  const size_t ptr_bytes = ((size_t)p.N + 1) * 4 + 15 & ~(size_t)15;
  const size_t rec_bytes = (size_t)p.L * 16;
  const size_t src16_bytes = ((size_t)p.L * 2 + 15) & ~(size_t)15;
  // in the order the kernel lays them out: link destinations, held table, in-list records
  *dst_in_lds = lds + dst_bytes <= limit ? 1u : 0u;
  if (*dst_in_lds) lds += dst_bytes;
  *held_lanes = lds + held_bytes <= limit ? lanes : 0u;
  if (*held_lanes) lds += held_bytes;
  *rec_in_lds = 0u;
  if (lds + ptr_bytes <= limit) { *rec_in_lds |= 2u; lds += ptr_bytes; }  // offsets first: they are small
  if (lds + rec_bytes <= limit) { *rec_in_lds |= 1u; lds += rec_bytes; }
  else if (p.N <= 65536u && lds + src16_bytes <= limit) { *rec_in_lds |= 4u; lds += src16_bytes; }
  return lds;
}

// Words per row (2, 4, 8, 16) of the lane-per-destination variant that takes this launch, or 0.
template <int NP, int MODE> static int tiny_words(u32 held_lanes, u32 rec_in_lds)
{
  if (NP != 1 || MODE != 0 || held_lanes == 0 || held_lanes > 8 || rec_in_lds != 3u) return 0;
  return held_lanes == 1 ? 2 : held_lanes == 2 ? 4 : held_lanes <= 4 ? 8 : 16;
}

template <int NP, int MODE, bool HELD_LDS, int TW>
static hipError_t launch_small_variant(const PassDev &p, const u32 *out_ptr, const u32 *out_dst, u32 first_event,
                                       u32 n_events, u32 stop_event, uint2 *recs, u32 *span_first, u64 *event_times,
                                       size_t lds, u32 dst_in_lds, u32 held_lanes, u32 rec_in_lds, hipStream_t s)
{
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&small_sweep_kernel<NP, MODE, HELD_LDS, TW>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((small_sweep_kernel<NP, MODE, HELD_LDS, TW>), dim3(1), dim3(1024), lds, s, p, out_ptr, out_dst,
                     first_event, n_events, stop_event, recs, span_first, event_times, dst_in_lds, held_lanes, rec_in_lds);
  return hipGetLastError();
}

template <int NP, int MODE>
static hipError_t launch_small_np(const PassDev &p, const u32 *out_ptr, const u32 *out_dst, u32 first_event,
                                  u32 n_events, u32 stop_event, uint2 *recs, u32 *span_first, u64 *event_times,
                                  bool sparse, hipStream_t s)
{
  u32 dst_in_lds = 0, held_lanes = 0, rec_in_lds = 0;
  const size_t lds = small_launch_lds(p, &dst_in_lds, &held_lanes, &rec_in_lds);
#define TACOS_VARIANT(H_, T_)                                                                                         \
  return launch_small_variant<NP, MODE, H_, T_>(p, out_ptr, out_dst, first_event, n_events, stop_event, recs, span_first, \
                                                event_times, lds, dst_in_lds, held_lanes, rec_in_lds, s)
  // sparse (about one transfer per span): a wavefront per destination decides the one or two
  // destinations of a span in a fraction of the time a single lane takes for each
  if constexpr (NP == 1 && MODE == 0) {
    switch (sparse ? 0 : tiny_words<NP, MODE>(held_lanes, rec_in_lds)) {
      case 2: TACOS_VARIANT(true, 2);
      case 4: TACOS_VARIANT(true, 4);
      case 8: TACOS_VARIANT(true, 8);
      case 16: TACOS_VARIANT(true, 16);
      default: break;
    }
  }
  if (held_lanes) TACOS_VARIANT(true, 0);
  TACOS_VARIANT(false, 0);
#undef TACOS_VARIANT
}

template <int NP, int MODE, bool HELD_LDS, int TW>
static hipError_t launch_batch_variant(const SmallJob *jobs, u32 n_jobs, u32 first_event, u32 n_events, size_t lds,
                                       u32 dst_in_lds, u32 held_lanes, u32 rec_in_lds, hipStream_t s)
{
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&small_sweep_batch_kernel<NP, MODE, HELD_LDS, TW>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((small_sweep_batch_kernel<NP, MODE, HELD_LDS, TW>), dim3(n_jobs), dim3(1024), lds, s, jobs,
                     first_event, n_events, dst_in_lds, held_lanes, rec_in_lds);
  return hipGetLastError();
}

template <int NP, int MODE>
static hipError_t launch_batch_np(const SmallJob *jobs, u32 n_jobs, const PassDev &p0, u32 first_event,
                                  u32 n_events, bool sparse, hipStream_t s)
{
  u32 dst_in_lds = 0, held_lanes = 0, rec_in_lds = 0;
  const size_t lds = small_launch_lds(p0, &dst_in_lds, &held_lanes, &rec_in_lds);
#define TACOS_VARIANT(H_, T_) \
  return launch_batch_variant<NP, MODE, H_, T_>(jobs, n_jobs, first_event, n_events, lds, dst_in_lds, held_lanes, rec_in_lds, s)
  if constexpr (NP == 1 && MODE == 0) {
    switch (sparse ? 0 : tiny_words<NP, MODE>(held_lanes, rec_in_lds)) {
      case 2: TACOS_VARIANT(true, 2);
      case 4: TACOS_VARIANT(true, 4);
      case 8: TACOS_VARIANT(true, 8);
      case 16: TACOS_VARIANT(true, 16);
      default: break;
    }
  }
  if (held_lanes) TACOS_VARIANT(true, 0);
  TACOS_VARIANT(false, 0);
#undef TACOS_VARIANT
}

hipError_t launch_small_sweep(const PassDev &p, const u32 *out_ptr, const u32 *out_dst, u32 first_event,
                              u32 n_events, u32 stop_event, uint2 *recs, u32 *span_first, u64 *event_times, u32 mode,
                              bool sparse, hipStream_t s)
{
#define TACOS_SMALL(NP_, M_) \
  return launch_small_np<NP_, M_>(p, out_ptr, out_dst, first_event, n_events, stop_event, recs, span_first, event_times, sparse, s)
  if (mode > 2) return hipErrorInvalidValue;
  switch (p.NP * 4 + mode) {
    case 4: TACOS_SMALL(1, 0);
    case 5: TACOS_SMALL(1, 1);
    case 6: TACOS_SMALL(1, 2);
    case 8: TACOS_SMALL(2, 0);
    case 9: TACOS_SMALL(2, 1);
    case 10: TACOS_SMALL(2, 2);
    default: return hipErrorInvalidValue;
  }
#undef TACOS_SMALL
}

hipError_t launch_small_sweep_batch(const SmallJob *jobs, u32 n_jobs, const PassDev &p0, u32 first_event,
                                    u32 n_events, u32 mode, bool sparse, hipStream_t s)
{
#define TACOS_BATCH(NP_, M_) return launch_batch_np<NP_, M_>(jobs, n_jobs, p0, first_event, n_events, sparse, s)
  if (mode > 2 || n_jobs == 0) return hipErrorInvalidValue;
  switch (p0.NP * 4 + mode) {
    case 4: TACOS_BATCH(1, 0);
    case 5: TACOS_BATCH(1, 1);
    case 6: TACOS_BATCH(1, 2);
    case 8: TACOS_BATCH(2, 0);
    case 9: TACOS_BATCH(2, 1);
    case 10: TACOS_BATCH(2, 2);
    default: return hipErrorInvalidValue;
  }
#undef TACOS_BATCH
}

bool small_sweep_by_lane(u32 N, u32 L, u32 NP, u32 C, u32 mode)
{
  if (NP != 1 || mode != 0) return false;
  PassDev p{};
  p.N = N; p.L = L; p.NP = NP; p.C = C;
  u32 dst_in_lds = 0, held_lanes = 0, rec_in_lds = 0;
  (void)small_launch_lds(p, &dst_in_lds, &held_lanes, &rec_in_lds);
  return tiny_words<1, 0>(held_lanes, rec_in_lds) != 0;
}

size_t small_sweep_lds_bytes(u32 N, u32 L, u32 NP) { return NP <= 2 ? small_lds_bytes(N, L, NP) : (size_t)-1; }

uint32_t compact_schedule_max_links() { return (uint32_t)((lds_limit() - 2048) / 4); }

void launch_compact_epilogue(uint2 *recs, const u32 *span_first, u32 n_spans, u32 L, const u64 *span_time, u64 t_base,
                             u32 reversed, u64 *digest, hipStream_t s)
{
  if (n_spans == 0) return;
  // more than 64 KiB of dynamic LDS has to be allowed explicitly
  if ((size_t)L * 4 > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&compact_epilogue_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)((size_t)L * 4));
  hipLaunchKernelGGL(compact_epilogue_kernel, dim3(n_spans), dim3(256), (size_t)L * 4, s, recs, span_first, L, span_time,
                     t_base, reversed, digest);
}

void launch_compact_link_counts(const uint2 *recs, u32 n_rec, u64 *counts, hipStream_t s)
{
  if (n_rec == 0) return;
  hipLaunchKernelGGL(compact_link_count_kernel, dim3((n_rec + 255) / 256), dim3(256), 0, s, recs, n_rec, counts);
}

void launch_compact_start_span_counts(const uint2 *recs, const u32 *span_first, u32 n_spans, const u64 *span_time,
                                      const u64 *cost, u32 *counts, hipStream_t s)
{
  if (n_spans == 0) return;
  hipLaunchKernelGGL(compact_start_span_kernel, dim3(n_spans), dim3(256), 0, s, recs, span_first, span_time, cost,
                     counts);
}

void launch_start_span_counts(const u32 *rows, u32 first_row, u32 n_rows, u32 L, const u64 *row_time,
                              const u64 *cost, u32 *counts, hipStream_t s)
{
  if (n_rows == 0 || L == 0) return;
  for (u32 r0 = 0; r0 < n_rows; r0 += 65535u) {  // grid.y limit
    const u32 nr = n_rows - r0 < 65535u ? n_rows - r0 : 65535u;
    hipLaunchKernelGGL(start_span_count_kernel, dim3((L + 255) / 256, nr), dim3(256), 0, s, rows + (u64)r0 * L,
                       first_row + r0, L, row_time, cost, counts);
  }
}

void launch_link_counts(const u32 *rows, u32 n_rows, u32 L, u64 *counts, hipStream_t s)
{
  if (n_rows == 0 || L == 0) return;
  // at most 65535 row blocks per launch (grid.y limit)
  for (u32 r0 = 0; r0 < n_rows; r0 += 65535u * 64u) {
    const u32 nr = n_rows - r0 < 65535u * 64u ? n_rows - r0 : 65535u * 64u;
    hipLaunchKernelGGL(link_count_kernel, dim3((L + 255) / 256, (nr + 63) / 64), dim3(256), 0, s,
                       rows + (u64)r0 * L, nr, L, counts);
  }
}

void launch_row_stats(const u32 *rows, u32 n_rows, u32 L, const u64 *row_time, u64 t_base,
                      u32 reversed, u32 *row_count, u64 *digest, hipStream_t s)
{
  if (n_rows == 0 || L == 0) return;
  const u32 bpr = (L + 2047) / 2048;
  // keep every launch below 2^31 blocks
  const u32 max_rows = 0x7FFFFFFFu / bpr;
  for (u32 r0 = 0; r0 < n_rows; r0 += max_rows) {
    const u32 nr = n_rows - r0 < max_rows ? n_rows - r0 : max_rows;
    hipLaunchKernelGGL(row_stats_kernel, dim3(nr * bpr), dim3(256), 0, s, rows + (u64)r0 * L, L,
                       row_time + r0, t_base, reversed, bpr, row_count + r0, digest);
  }
}

}  // namespace tacos
