// HIP kernels (gfx950) around the synthesis: the paper's switch unwinding (input
// pre-processing) and the quantities it judges a schedule by (link busy times for the link
// utilisation, the two terms of its "Ideal" collective time).  All integer arithmetic.
//
// Paper, section "TACOS for Switch-based Networks": an N-NPU switch unwound with degree d
// gives every NPU i the d outgoing links to NPUs i+1 .. i+d (mod N), with alpha unchanged and
// beta multiplied by d.  Section "Baseline Collective Algorithms and Synthesizers":
//   Ideal = CollectiveSize * 2(n-1)/n / min over NPUs of BW_N + Diameter
// (bandwidth term: serialization at the worst-connected NPU; Diameter: smallest latency
// between the two farthest NPUs).  Section "Analysis of TACOS-Synthesized Algorithms": link
// utilisation over the execution of a collective.

#include "tacos_internal.h"

namespace tacos {

namespace {

typedef unsigned long long u64;
typedef uint32_t u32;

// ---------------------------------------------------------------- switch unwinding

// one thread per link (i, k), k = 1 .. d; the links of NPU i are written in ascending
// destination: the w = max(0, i + d - (N - 1)) destinations that wrap around come first
__global__ void unwind_switch_kernel(u32 n, u32 d, u64 alpha, u64 beta_d, u32 *__restrict__ row_ptr,
                                     u32 *__restrict__ col_idx, u64 *__restrict__ alpha_out, u64 *__restrict__ beta_out)
{
  const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (t <= n) row_ptr[t] = (u32)(t * d);
  if (t >= (u64)n * d) return;
  const u32 i = (u32)(t / d), k = (u32)(t - (u64)i * d) + 1u;
  const u32 w = i + d > n - 1u ? i + d - (n - 1u) : 0u;
  u32 dst = i + k, pos;
  if (dst < n) pos = w + (k - 1u);
  else { dst -= n; pos = dst; }
  const u64 at = (u64)i * d + pos;
  col_idx[at] = dst;
  alpha_out[at] = alpha;
  beta_out[at] = beta_d;
}

// ---------------------------------------------------------------- Ideal: bandwidth term

__device__ __forceinline__ u64 gcd64(u64 a, u64 b)
{
  while (b) { const u64 t = a % b; a = b; b = t; }
  return a;
}

// Bandwidth of an NPU = sum over its links (ptr/beta: the in-lists, or the out-lists) of
// 1/beta, as the exact fraction P/Q bytes per femtosecond: Q = lcm(beta), P = sum Q/beta.
// A link with beta == 0 makes the bandwidth infinite: (P, Q) = (1, 0).
__global__ void npu_bandwidth_kernel(u32 N, const u32 *__restrict__ ptr, const u64 *__restrict__ beta,
                                     u64 *__restrict__ P, u64 *__restrict__ Q, u32 *__restrict__ flags)
{
  const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  const u32 b0 = ptr[i], b1 = ptr[i + 1];
  if (b0 == b1) { atomicOr(flags, kRepNoLink); P[i] = 0; Q[i] = 1; return; }
  u64 q = 1;
  bool infinite = false, ovf = false;
  for (u32 l = b0; l < b1; ++l) {
    const u64 b = beta[l];
    if (b == 0) { infinite = true; continue; }
    const u64 m = q / gcd64(q, b);
    if (__umul64hi(m, b)) ovf = true;
    q = m * b;
  }
  u64 p = 0;
  if (!infinite && !ovf)
    for (u32 l = b0; l < b1; ++l) {
      const u64 add = q / beta[l];
      if (p + add < p) ovf = true;
      p += add;
    }
  if (ovf) atomicOr(flags, kRepOverflow);
  P[i] = infinite ? 1ull : p;
  Q[i] = infinite ? 0ull : q;
}

// time per byte a = Qa/Pa against b = Qb/Pb, exact (128-bit cross products)
__device__ __forceinline__ bool slower(u64 Pa, u64 Qa, u64 Pb, u64 Qb)
{
  const u64 ah = __umul64hi(Qa, Pb), al = Qa * Pb, bh = __umul64hi(Qb, Pa), bl = Qb * Pa;
  return ah > bh || (ah == bh && al > bl);
}

// The worst-connected NPU (largest time per byte Q/P, lowest id on ties) and the time it
// needs for `bytes`: ceil(bytes * Q / (P * 1000)) picoseconds.  One workgroup.
// out[0] = the time, out[1] = the NPU.
__global__ __launch_bounds__(256) void bottleneck_kernel(u32 N, const u64 *__restrict__ P, const u64 *__restrict__ Q,
                                                         u64 bytes, u64 *__restrict__ out, u32 *__restrict__ flags)
{
  __shared__ u64 sP[256], sQ[256];
  __shared__ u32 sI[256];
  u64 bp = 1, bq = 0;
  u32 bi = 0xFFFFFFFFu;
  for (u32 i = threadIdx.x; i < N; i += 256u) {
    const u64 p = P[i], q = Q[i];
    if (p == 0) continue;  // no link: flagged by the kernel before
    if (bi == 0xFFFFFFFFu || slower(p, q, bp, bq)) { bp = p; bq = q; bi = i; }
  }
  sP[threadIdx.x] = bp; sQ[threadIdx.x] = bq; sI[threadIdx.x] = bi;
  __syncthreads();
  if (threadIdx.x != 0) return;
  for (u32 k = 1; k < 256u; ++k) {
    if (sI[k] == 0xFFFFFFFFu) continue;
    if (bi == 0xFFFFFFFFu || slower(sP[k], sQ[k], bp, bq) || (!slower(bp, bq, sP[k], sQ[k]) && sI[k] < bi)) {
      bp = sP[k]; bq = sQ[k]; bi = sI[k];
    }
  }
  u64 term = 0;
  if (bi != 0xFFFFFFFFu && bq != 0) {
    if (__umul64hi(bp, 1000ull)) atomicOr(flags, kRepOverflow);
    const u64 dv = bp * 1000ull;
    // (hi:lo) = bytes * Q + dv - 1, then divided by dv, bit by bit
    u64 hi = __umul64hi(bytes, bq), lo = bytes * bq;
    const u64 lo2 = lo + (dv - 1ull);
    if (lo2 < lo) hi += 1ull;
    lo = lo2;
    u64 rem = 0, quo = 0;
    bool ovf = false;
    for (int b = 127; b >= 0; --b) {
      const u64 bit = b >= 64 ? (hi >> (b - 64)) & 1ull : (lo >> b) & 1ull;
      const bool carry = rem >> 63;
      rem = (rem << 1) | bit;
      if (carry || rem >= dv) {
        rem -= dv;
        if (b >= 64) ovf = true;
        else quo |= 1ull << b;
      }
    }
    if (ovf) atomicOr(flags, kRepOverflow);
    term = quo;
  }
  out[0] = term;
  out[1] = bi;
}

// ---------------------------------------------------------------- Ideal: latency diameter

// One workgroup per source NPU: label-correcting shortest paths over the link latencies with
// the distances in LDS (N * 8 bytes), swept until nothing changes; then the largest distance
// goes into *diameter.  An NPU that is not reached sets kRepNoLink.
__global__ __launch_bounds__(256) void latency_sssp_kernel(u32 N, u32 L, const u32 *__restrict__ src,
                                                           const u32 *__restrict__ dst, const u64 *__restrict__ alpha,
                                                           u64 *__restrict__ diameter, u32 *__restrict__ flags)
{
  extern __shared__ __align__(16) unsigned char sssp_lds[];
  u64 *dist = reinterpret_cast<u64 *>(sssp_lds);
  u32 *changed = reinterpret_cast<u32 *>(dist + N);
  const u32 s = blockIdx.x;
  for (u32 i = threadIdx.x; i < N; i += 256u) dist[i] = i == s ? 0ull : kInf;
  if (threadIdx.x == 0) changed[0] = 0u;
  __syncthreads();
  for (u32 it = 0; it <= N; ++it) {
    bool any = false;
    for (u32 l = threadIdx.x; l < L; l += 256u) {
      const u64 du = dist[src[l]];
      if (du == kInf) continue;
      const u64 a = alpha[l];
      if (a > kInf - 1ull - du) { atomicOr(flags, kRepOverflow); continue; }
      const u64 nd = du + a;
      if (nd < dist[dst[l]]) { atomicMin(&dist[dst[l]], nd); any = true; }
    }
    if (any) changed[0] = 1u;
    __syncthreads();
    const bool again = changed[0] != 0u;
    __syncthreads();
    if (!again) break;
    if (threadIdx.x == 0) changed[0] = 0u;
    __syncthreads();
  }
  u64 m = 0;
  for (u32 i = threadIdx.x; i < N; i += 256u) m = dist[i] > m ? dist[i] : m;
  if (m == kInf) atomicOr(flags, kRepNoLink);
  else atomicMax(diameter, m);
}

// ---------------------------------------------------------------- link busy times

// busy[l] = transfers carried * cost; out = (sum, min, max) over the links.  One workgroup
// strides over the links (a few hundred thousand at most).
__global__ __launch_bounds__(256) void link_busy_kernel(u32 L, const u64 *__restrict__ counts, const u64 *__restrict__ cost,
                                                        u64 *__restrict__ busy, u64 *__restrict__ out,
                                                        u32 *__restrict__ flags)
{
  __shared__ u64 s_sum[256], s_min[256], s_max[256];
  u64 sum = 0, mn = kInf, mx = 0;
  bool ovf = false;
  for (u32 l = threadIdx.x; l < L; l += 256u) {
    if (__umul64hi(counts[l], cost[l])) ovf = true;
    const u64 b = counts[l] * cost[l];
    if (busy) busy[l] = b;
    if (sum + b < sum) ovf = true;
    sum += b;
    mn = b < mn ? b : mn;
    mx = b > mx ? b : mx;
  }
  s_sum[threadIdx.x] = sum; s_min[threadIdx.x] = mn; s_max[threadIdx.x] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (u32 k = 1; k < 256u; ++k) {
      if (sum + s_sum[k] < sum) ovf = true;
      sum += s_sum[k];
      mn = s_min[k] < mn ? s_min[k] : mn;
      mx = s_max[k] > mx ? s_max[k] : mx;
    }
    out[0] = sum; out[1] = L ? mn : 0ull; out[2] = mx;
  }
  if (ovf) atomicOr(flags, kRepOverflow);
}

}  // namespace

void launch_unwind_switch(u32 n, u32 d, u64 alpha, u64 beta_d, u32 *row_ptr, u32 *col_idx, u64 *alpha_out, u64 *beta_out,
                          hipStream_t s)
{
  const u64 threads = (u64)n * d > (u64)n + 1 ? (u64)n * d : (u64)n + 1;
  hipLaunchKernelGGL(unwind_switch_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, n, d, alpha, beta_d,
                     row_ptr, col_idx, alpha_out, beta_out);
}

void launch_bandwidth_term(u32 N, const u32 *ptr, const u64 *beta, u64 bytes, u64 *P, u64 *Q, u64 *out, u32 *flags,
                           hipStream_t s)
{
  hipLaunchKernelGGL(npu_bandwidth_kernel, dim3((N + 255) / 256), dim3(256), 0, s, N, ptr, beta, P, Q, flags);
  hipLaunchKernelGGL(bottleneck_kernel, dim3(1), dim3(256), 0, s, N, P, Q, bytes, out, flags);
}

hipError_t launch_latency_diameter(u32 N, u32 L, const u32 *src, const u32 *dst, const u64 *alpha, u64 *diameter,
                                   u32 *flags, hipStream_t s)
{
  const size_t lds = (size_t)N * 8 + 16;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&latency_sssp_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(latency_sssp_kernel, dim3(N), dim3(256), lds, s, N, L, src, dst, alpha, diameter, flags);
  return hipGetLastError();
}

void launch_link_busy(u32 L, const u64 *counts, const u64 *cost, u64 *busy, u64 *out, u32 *flags, hipStream_t s)
{
  hipLaunchKernelGGL(link_busy_kernel, dim3(1), dim3(256), 0, s, L, counts, cost, busy, out, flags);
}

}  // namespace tacos
