// HIP kernels (gfx950, wave64) of the TACOS synthesis hot path.
//
// Paper: TACOS, arXiv 2304.05301.  One TEN span ("event") is processed by two launches:
//   arrive_kernel : the precondition update for the span (chunks whose transfer ends now
//                   become held), one thread per link;
//   match_kernel  : Algorithm 1 (utilization-maximizing matching) in its link-centric
//                   deterministic form, one wavefront per destination NPU, plus the
//                   min-reduction that finds the next span of Algorithm 2.
// The host never sees the per-event state; it only queues launches and polls the
// control block once per batch of events.
//
// All arithmetic is integer.  Bitset layout: see PassDev in tacos_internal.h.

#include "tacos_internal.h"

namespace tacos {

namespace {

typedef unsigned long long u64;
typedef uint32_t u32;

// ---------------------------------------------------------------- small helpers

__device__ __forceinline__ u32 uniform(u32 v) { return (u32)__builtin_amdgcn_readfirstlane((int)v); }

__device__ __forceinline__ u32 read_lane(u32 v, u32 lane)
{
  return (u32)__builtin_amdgcn_readlane((int)v, (int)lane);
}

__device__ __forceinline__ u64 read_lane64(u64 v, u32 lane)
{
  u32 lo = read_lane((u32)v, lane), hi = read_lane((u32)(v >> 32), lane);
  return ((u64)hi << 32) | lo;
}

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ u32 wave_inclusive_scan(u32 v, int lane)
{
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    u32 o = (u32)__shfl_up((int)v, off, 64);
    if (lane >= off) v += o;
  }
  return v;
}

__device__ __forceinline__ u64 wave_min64(u64 v)
{
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    u32 lo = (u32)__shfl_xor((int)(u32)v, off, 64);
    u32 hi = (u32)__shfl_xor((int)(u32)(v >> 32), off, 64);
    u64 o = ((u64)hi << 32) | lo;
    v = o < v ? o : v;
  }
  return v;
}

// Position of the k-th (0-based) set bit of w, k < popcount(w): binary search on the
// popcounts of the low halves.
__device__ __forceinline__ u32 kth_set_bit(u64 w, u32 k)
{
  u32 pos = 0;
#pragma unroll
  for (u32 s = 32; s >= 1; s >>= 1) {
    u64 low = (w >> pos) & ((1ull << s) - 1ull);
    u32 pc = (u32)__popcll(low);
    if (k >= pc) { k -= pc; pos += s; }
  }
  return pos;
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
  const u64 own_lo = (u64)npu * p.cpn, own_hi = own_lo + p.cpn;  // [own_lo, own_hi)
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
  if (l < p.L) { p.carry[l] = kNone; p.free_at[l] = 0ull; }
  if (l == 0) {
    Ctl *c = p.ctl;
    c->next_t[0] = 0ull;
    c->next_t[1] = kInf;
    c->remaining = (u64)p.N * p.C - p.C;
    c->T = 0ull;
    c->done = 0u;
    c->status = 0u;
    c->n_events = 0u;
    c->pad = 0u;
  }
}

// ---------------------------------------------------------------- a3: arrivals

__global__ __launch_bounds__(256) void arrive_kernel(PassDev p, u32 event, u64 *event_time_slot,
                                                     u32 *__restrict__ sched_row)
{
  Ctl *ctl = p.ctl;
  if (ctl->done) return;
  const u64 t = ctl->next_t[event & 1u];
  const u32 l = blockIdx.x * 256u + threadIdx.x;
  if (l == 0) {
    *event_time_slot = t;
    ctl->next_t[(event + 1u) & 1u] = kInf;
    if (t == kInf) {  // chunks missing (else done) and nothing in flight
      ctl->status = kStUnreachable;
      ctl->done = 1u;
    }
  }
  if (t == kInf) return;
  bool arrived = false;
  if (l < p.L) {
    const u32 c = p.carry[l];
    arrived = (c != kNone) && (p.free_at[l] == t);
    if (arrived) {
      const u32 d = p.link_dst[l];
      atomicOr(&p.held[(u64)d * p.row_words + phys_word(c >> 6, p.NP)], 1ull << (c & 63u));
      p.carry[l] = kNone;
    }
    if (sched_row) sched_row[l] = arrived ? c : kNone;
  }
  const u32 n = (u32)__popcll(__ballot(arrived));
  __shared__ u32 block_n;
  if (threadIdx.x == 0) block_n = 0;
  __syncthreads();
  if ((threadIdx.x & 63u) == 0 && n) atomicAdd(&block_n, n);
  __syncthreads();
  if (threadIdx.x == 0 && block_n) atomicAdd(&ctl->remaining, (u64)0 - (u64)block_n);
}

// ---------------------------------------------------------------- a4-a8: matching

template <int NW>
__device__ __forceinline__ void clear_chunk(u64 (&need)[NW], u32 c, int lane)
{
  // c is wave-uniform; lane-major layout: word w = c>>6 lives in lane w/NW at index w%NW
  const u32 w = c >> 6;
  const u32 ln = w / (u32)NW;
  const u32 idx = w - ln * (u32)NW;
  const u64 m = ~(1ull << (c & 63u));
#pragma unroll
  for (int i = 0; i < NW; ++i)
    if ((u32)i == idx && (u32)lane == ln) need[i] &= m;
}

template <int NP>
__global__ __launch_bounds__(256) void match_kernel(PassDev p, u32 event, u32 *__restrict__ sched_row)
{
  constexpr int NW = 2 * NP;  // 64-bit words of a row held by one lane
  const int lane = threadIdx.x & 63;
  const u32 d = uniform(blockIdx.x * 4u + (threadIdx.x >> 6));
  if (d >= p.N) return;
  Ctl *ctl = p.ctl;
  if (ctl->done) return;
  const u64 rem = ctl->remaining;
  const u64 t = ctl->next_t[event & 1u];
  if (rem == 0) {  // every postcondition satisfied: the collective ends now
    if (d == 0 && lane == 0) { ctl->T = t; ctl->n_events = event; ctl->done = 1u; }
    return;
  }

  const u32 jb = p.in_ptr[d], je = p.in_ptr[d + 1];
  const u32 k0 = p.seed_lo, k1 = p.seed_hi;

  // pass 1 over the incoming links: is any idle?  earliest end among the busy ones
  u64 my_min = kInf;
  bool any_idle = false;
  for (u32 base = jb; base < je; base += 64) {
    const u32 j = base + lane;
    bool idle = false;
    if (j < je) {
      const u32 l = p.in_link[j];
      const u32 cr = p.carry[l];
      idle = cr == kNone;
      if (!idle) { const u64 fa = p.free_at[l]; my_min = fa < my_min ? fa : my_min; }
    }
    any_idle |= __ballot(idle) != 0ull;
  }

  u64 need[NW];
  bool need_any = false;
  if (any_idle) {
    // need = ~held[d] & ~inflight[d]; inflight[d] = the chunks on d's busy incoming links
    const uint4 *hp = reinterpret_cast<const uint4 *>(p.held + (u64)d * p.row_words) + lane;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const uint4 v = hp[i * 64];
      need[2 * i] = ~(((u64)v.y << 32) | v.x);
      need[2 * i + 1] = ~(((u64)v.w << 32) | v.z);
    }
    for (u32 base = jb; base < je; base += 64) {
      const u32 j = base + lane;
      u32 cr = kNone;
      if (j < je) cr = p.carry[p.in_link[j]];
      u64 busy = __ballot(cr != kNone);
      while (busy) {
        const u32 b = (u32)__ffsll((long long)busy) - 1u;
        busy &= busy - 1ull;
        clear_chunk<NW>(need, read_lane(cr, b), lane);
      }
    }
    u64 acc = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) acc |= need[i];
    need_any = __ballot(acc != 0ull) != 0ull;
  }

  for (u32 base = jb; base < je; base += 64) {
    const u32 j = base + lane;
    const bool valid = j < je;
    u32 l = 0, s = 0, cr = kNone;
    u64 cs = 0;
    if (valid) { l = p.in_link[j]; s = p.in_src[j]; cr = p.carry[l]; cs = p.cost[l]; }
    u32 res = kNone;  // chunk matched to this lane's link in this span
    if (need_any) {
      u64 idle = __ballot(valid && cr == kNone);
      const u32 r = philox4x32_10_word0(l, event, p.phase, 0u, k0, k1);
      while (idle) {
        const u32 b = (u32)__ffsll((long long)idle) - 1u;
        idle &= idle - 1ull;
        const u32 src = read_lane(s, b);
        // cand = held[src] & need
        const uint4 *sp = reinterpret_cast<const uint4 *>(p.held + (u64)src * p.row_words) + lane;
        u64 cand[NW];
        u32 cnt = 0;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
          const uint4 v = sp[i * 64];
          cand[2 * i] = (((u64)v.y << 32) | v.x) & need[2 * i];
          cand[2 * i + 1] = (((u64)v.w << 32) | v.z) & need[2 * i + 1];
          cnt += (u32)__popcll(cand[2 * i]) + (u32)__popcll(cand[2 * i + 1]);
        }
        const u32 incl = wave_inclusive_scan(cnt, lane);
        const u32 pop = read_lane(incl, 63);
        if (pop == 0) continue;  // nothing this link could carry: no draw is consumed
        u32 k = read_lane(r, b) % pop;
        // owning lane = first lane whose inclusive count exceeds k
        const u64 above = __ballot(incl > k);
        const u32 ln = (u32)__ffsll((long long)above) - 1u;
        k -= read_lane(incl - cnt, ln);
        // owning word inside that lane (ascending word index = ascending chunk id)
        u32 idx = 0;
        u64 word = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
          const u64 w = read_lane64(cand[i], ln);
          const u32 pc = (u32)__popcll(w);
          if (word == 0) {
            if (k < pc) { word = w; idx = (u32)i; }
            else k -= pc;
          }
        }
        const u32 bit = kth_set_bit(word, k);
        const u32 chunk = ((ln * (u32)NW + idx) << 6) + bit;
        clear_chunk<NW>(need, chunk, lane);  // now in flight to d: later links skip it
        if ((u32)lane == b) res = chunk;
      }
    }
    if (valid) {
      if (sched_row) sched_row[l] = res;
      if (res != kNone) {
        if (cs > kInf - 1ull - t) {
          ctl->status = kStOverflow;
          ctl->done = 1u;
        } else {
          const u64 fa = t + cs;
          p.carry[l] = res;
          p.free_at[l] = fa;
          my_min = fa < my_min ? fa : my_min;
        }
      }
    }
  }

  // a8: next span = earliest end of a transfer in flight (min over all destinations)
  const u64 m = wave_min64(my_min);
  if (lane == 0 && m != kInf) {
    u64 *nt = &ctl->next_t[(event + 1u) & 1u];
    const u64 cur = __hip_atomic_load(nt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (m < cur) atomicMin(nt, m);
  }
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

// grid = n_rows * ceil(L / 2048) blocks; every block covers 2048 links of one schedule row
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
  if ((threadIdx.x & 63u) == 0 && n) {
    atomicAdd(&row_count[row], n);
    atomicAdd(digest, dg);
  }
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

void launch_init_pass(const PassDev &p, hipStream_t s)
{
  const u64 total = (u64)p.N * p.row_words;
  hipLaunchKernelGGL(init_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
  hipLaunchKernelGGL(init_links_kernel, dim3((p.L + 255) / 256 + (p.L == 0)), dim3(256), 0, s, p);
}

void launch_arrive(const PassDev &p, u32 event, u64 *event_time_slot, u32 *sched_row, hipStream_t s)
{
  hipLaunchKernelGGL(arrive_kernel, dim3((p.L + 255) / 256), dim3(256), 0, s, p, event,
                     event_time_slot, sched_row);
}

void launch_match(const PassDev &p, u32 event, u32 *sched_row, hipStream_t s)
{
  const dim3 grid((p.N + 3) / 4), block(256);
  switch (p.NP) {
    case 1: hipLaunchKernelGGL(match_kernel<1>, grid, block, 0, s, p, event, sched_row); break;
    case 2: hipLaunchKernelGGL(match_kernel<2>, grid, block, 0, s, p, event, sched_row); break;
    case 3: hipLaunchKernelGGL(match_kernel<3>, grid, block, 0, s, p, event, sched_row); break;
    case 4: hipLaunchKernelGGL(match_kernel<4>, grid, block, 0, s, p, event, sched_row); break;
    case 5: hipLaunchKernelGGL(match_kernel<5>, grid, block, 0, s, p, event, sched_row); break;
    case 6: hipLaunchKernelGGL(match_kernel<6>, grid, block, 0, s, p, event, sched_row); break;
    case 7: hipLaunchKernelGGL(match_kernel<7>, grid, block, 0, s, p, event, sched_row); break;
    case 8: hipLaunchKernelGGL(match_kernel<8>, grid, block, 0, s, p, event, sched_row); break;
    default: break;  // rejected by the host before any launch
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
