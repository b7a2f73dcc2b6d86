// Bench-side probes (gfx950) for bench.py: what the memory system of THIS device delivers
// for the access pattern of the matching kernel, measured with no method arithmetic.
// Built to libbench_probe.so beside bench.py; never linked into libtacos_hip.so and shares
// no code with it (the product) or with the oracle.
//
//   probe_row_stream : every destination NPU's wavefront loads its own bitset row and the
//                      rows of all its in-neighbours (one 16-byte load per lane and KiB of
//                      row, fully coalesced), i.e. exactly the requests the matching kernel
//                      sends to L2 when every incoming link is idle, in the same
//                      destination order (breadth-first clusters handed to the 8 XCDs in
//                      contiguous slices), and only XORs the words together.  Its time is
//                      the floor the L2-to-CU path sets for one span.
//   probe_read_stream: a read-only pass over a large buffer (HBM streaming rate).
//   probe_copy       : a plain device-to-device copy kernel (read + write rate).
//
// All entry points take host pointers, allocate their own device buffers, time `iters`
// launches with HIP events on the null stream after one warm-up launch, and return 0 or
// the hipError_t that failed.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace {

#define PROBE_TRY(expr)                         \
  do {                                          \
    const hipError_t e_ = (expr);               \
    if (e_ != hipSuccess) { cleanup(); return (int)e_; } \
  } while (0)

template <int NP>
__global__ __launch_bounds__(256) void row_stream_kernel(const uint4 *__restrict__ rows, uint32_t n_slots,
                                                         const uint4 *__restrict__ slot_rec,
                                                         const uint32_t *__restrict__ in_src,
                                                         uint32_t *__restrict__ sink)
{
  const int lane = threadIdx.x & 63;
  const uint32_t per_xcd = gridDim.x >> 3;
  const uint32_t pos = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const uint32_t slot = pos * 4u + (threadIdx.x >> 6);
  if (slot >= n_slots) return;
  const uint4 sr = slot_rec[slot];  // (destination, its in-list begin, end)
  const uint32_t d = (uint32_t)__builtin_amdgcn_readfirstlane((int)sr.x);
  const uint32_t jb = (uint32_t)__builtin_amdgcn_readfirstlane((int)sr.y);
  const uint32_t je = (uint32_t)__builtin_amdgcn_readfirstlane((int)sr.z);
  uint32_t acc = 0;
  const uint4 *own = rows + (size_t)d * NP * 64 + lane;
  uint4 o[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) o[i] = own[i * 64];
  for (uint32_t base = jb; base < je; base += 64) {
    // lane j holds the source of in-list entry base + j; two rows are asked for at a time
    const uint32_t mine = base + (uint32_t)lane < je ? in_src[base + lane] : d;
    const uint32_t n = je - base < 64u ? je - base : 64u;
    for (uint32_t j = 0; j < n; j += 2) {
      const uint32_t s0 = (uint32_t)__builtin_amdgcn_readlane((int)mine, (int)j);
      const uint32_t s1 = (uint32_t)__builtin_amdgcn_readlane((int)mine, (int)(j + 1 < n ? j + 1 : j));
      const uint4 *p0 = rows + (size_t)s0 * NP * 64 + lane;
      const uint4 *p1 = rows + (size_t)s1 * NP * 64 + lane;
      uint4 a[NP], b[NP];
#pragma unroll
      for (int i = 0; i < NP; ++i) a[i] = p0[i * 64];
      if (j + 1 < n) {
#pragma unroll
        for (int i = 0; i < NP; ++i) b[i] = p1[i * 64];
      } else {
#pragma unroll
        for (int i = 0; i < NP; ++i) b[i] = make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < NP; ++i) acc ^= a[i].x ^ a[i].y ^ a[i].z ^ a[i].w ^ b[i].x ^ b[i].y ^ b[i].z ^ b[i].w;
    }
  }
#pragma unroll
  for (int i = 0; i < NP; ++i) acc ^= o[i].x ^ o[i].y ^ o[i].z ^ o[i].w;
  if (acc == 0x9E3779B9u) sink[slot] = acc;  // keeps the loads alive; practically never true
}

__global__ __launch_bounds__(256) void read_stream_kernel(const uint4 *__restrict__ src, size_t n_vec,
                                                          uint32_t *__restrict__ sink)
{
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n_vec)
{
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

__global__ void fill_kernel(uint32_t *p, size_t n, uint32_t seed)
{
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    p[i] = (uint32_t)(i * 2654435761u) ^ seed;
}

// Destination order: clusters of about 512 NPUs grown breadth-first over the undirected
// topology (the locality heuristic the matching kernel's launch uses as well).
std::vector<uint32_t> cluster_order(uint32_t N, const std::vector<uint32_t> &in_ptr, const std::vector<uint32_t> &in_src,
                                    const uint32_t *row_ptr, const uint32_t *col_idx)
{
  std::vector<uint32_t> order;
  order.reserve(N);
  std::vector<uint8_t> state(N, 0);
  std::vector<uint32_t> queue;
  for (uint32_t seed = 0; seed < N; ++seed) {
    if (state[seed]) continue;
    queue.assign(1, seed);
    state[seed] = 1;
    size_t head = 0;
    uint32_t placed = 0;
    while (head < queue.size() && placed < 512) {
      const uint32_t u = queue[head++];
      state[u] = 2;
      order.push_back(u);
      placed++;
      for (uint32_t j = in_ptr[u]; j < in_ptr[u + 1]; ++j)
        if (!state[in_src[j]]) { state[in_src[j]] = 1; queue.push_back(in_src[j]); }
      for (uint32_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j)
        if (!state[col_idx[j]]) { state[col_idx[j]] = 1; queue.push_back(col_idx[j]); }
    }
    for (; head < queue.size(); ++head) state[queue[head]] = 0;
  }
  return order;
}

template <int NP>
void launch_rows(const uint4 *rows, uint32_t N, const uint4 *slot_rec, const uint32_t *in_src, uint32_t *sink)
{
  const uint32_t n_wg = (N + 3u) / 4u;
  const dim3 grid(8u * ((n_wg + 7u) / 8u)), block(256);
  hipLaunchKernelGGL((row_stream_kernel<NP>), grid, block, 0, nullptr, rows, N, slot_rec, in_src, sink);
}

}  // namespace

extern "C" {

// Topology in CSR form by source (as the synthesis takes it); row_bytes = NP KiB, NP in 1..8.
// *mean_us: mean duration of one launch; *request_bytes: bytes the wavefronts ask L2 for per
// launch = sum over destinations of (1 + in-degree) * row_bytes.
int probe_row_stream(uint32_t n_npus, const uint32_t *row_ptr, const uint32_t *col_idx, uint32_t row_bytes,
                     uint32_t iters, double *mean_us, double *request_bytes)
{
  if (!row_ptr || !col_idx || !mean_us || !request_bytes || n_npus == 0 || iters == 0) return (int)hipErrorInvalidValue;
  const uint32_t NP = row_bytes / 1024u;
  if (NP < 1 || NP > 8 || NP * 1024u != row_bytes) return (int)hipErrorInvalidValue;
  const uint32_t N = n_npus, L = row_ptr[N];
  std::vector<uint32_t> in_ptr(N + 1, 0), in_src(L);
  for (uint32_t l = 0; l < L; ++l) in_ptr[col_idx[l] + 1]++;
  for (uint32_t d = 0; d < N; ++d) in_ptr[d + 1] += in_ptr[d];
  {
    std::vector<uint32_t> fill(in_ptr.begin(), in_ptr.end() - 1);
    for (uint32_t s = 0; s < N; ++s)
      for (uint32_t l = row_ptr[s]; l < row_ptr[s + 1]; ++l) in_src[fill[col_idx[l]]++] = s;
  }
  const std::vector<uint32_t> order = cluster_order(N, in_ptr, in_src, row_ptr, col_idx);
  std::vector<uint32_t> slot_rec((size_t)N * 4, 0);
  for (uint32_t k = 0; k < N; ++k) {
    slot_rec[4 * (size_t)k] = order[k];
    slot_rec[4 * (size_t)k + 1] = in_ptr[order[k]];
    slot_rec[4 * (size_t)k + 2] = in_ptr[order[k] + 1];
  }
  void *d_rows = nullptr, *d_order = nullptr, *d_in_ptr = nullptr, *d_in_src = nullptr, *d_sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&]() {
    (void)hipFree(d_rows); (void)hipFree(d_order); (void)hipFree(d_in_ptr); (void)hipFree(d_in_src); (void)hipFree(d_sink);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  const size_t table = (size_t)N * row_bytes;
  PROBE_TRY(hipMalloc(&d_rows, table));
  PROBE_TRY(hipMalloc(&d_order, (size_t)N * 16));
  PROBE_TRY(hipMalloc(&d_in_ptr, (size_t)(N + 1) * 4));
  PROBE_TRY(hipMalloc(&d_in_src, (size_t)(L ? L : 1) * 4));
  PROBE_TRY(hipMalloc(&d_sink, (size_t)N * 4));
  PROBE_TRY(hipMemcpy(d_order, slot_rec.data(), (size_t)N * 16, hipMemcpyHostToDevice));
  PROBE_TRY(hipMemcpy(d_in_ptr, in_ptr.data(), (size_t)(N + 1) * 4, hipMemcpyHostToDevice));
  if (L) PROBE_TRY(hipMemcpy(d_in_src, in_src.data(), (size_t)L * 4, hipMemcpyHostToDevice));
  hipLaunchKernelGGL(fill_kernel, dim3(4096), dim3(256), 0, nullptr, (uint32_t *)d_rows, table / 4, 0x1234567u);
  PROBE_TRY(hipGetLastError());
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  auto launch = [&]() {
    const uint4 *rows = (const uint4 *)d_rows;
    const uint4 *o = (const uint4 *)d_order;
    const uint32_t *is = (const uint32_t *)d_in_src;
    uint32_t *sink = (uint32_t *)d_sink;
    switch (NP) {
      case 1: launch_rows<1>(rows, N, o, is, sink); break;
      case 2: launch_rows<2>(rows, N, o, is, sink); break;
      case 3: launch_rows<3>(rows, N, o, is, sink); break;
      case 4: launch_rows<4>(rows, N, o, is, sink); break;
      case 5: launch_rows<5>(rows, N, o, is, sink); break;
      case 6: launch_rows<6>(rows, N, o, is, sink); break;
      case 7: launch_rows<7>(rows, N, o, is, sink); break;
      default: launch_rows<8>(rows, N, o, is, sink); break;
    }
  };
  launch();
  PROBE_TRY(hipGetLastError());
  PROBE_TRY(hipDeviceSynchronize());
  PROBE_TRY(hipEventRecord(e0, nullptr));
  for (uint32_t i = 0; i < iters; ++i) launch();
  PROBE_TRY(hipEventRecord(e1, nullptr));
  PROBE_TRY(hipEventSynchronize(e1));
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  *mean_us = (double)ms * 1e3 / iters;
  *request_bytes = ((double)N + (double)L) * row_bytes;
  cleanup();
  return 0;
}

static int stream_probe(size_t bytes, uint32_t iters, bool copy, double *gb_per_s)
{
  if (!gb_per_s || bytes < 4096 || iters == 0) return (int)hipErrorInvalidValue;
  void *a = nullptr, *b = nullptr, *sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&]() {
    (void)hipFree(a); (void)hipFree(b); (void)hipFree(sink);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  const size_t n_vec = bytes / 16;
  PROBE_TRY(hipMalloc(&a, n_vec * 16));
  if (copy) PROBE_TRY(hipMalloc(&b, n_vec * 16));
  PROBE_TRY(hipMalloc(&sink, 256));
  hipLaunchKernelGGL(fill_kernel, dim3(4096), dim3(256), 0, nullptr, (uint32_t *)a, n_vec * 4, 0x7654321u);
  PROBE_TRY(hipGetLastError());
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  const dim3 grid(256 * 16), block(256);
  auto launch = [&]() {
    if (copy) hipLaunchKernelGGL(copy_kernel, grid, block, 0, nullptr, (const uint4 *)a, (uint4 *)b, n_vec);
    else hipLaunchKernelGGL(read_stream_kernel, grid, block, 0, nullptr, (const uint4 *)a, n_vec, (uint32_t *)sink);
  };
  launch();
  PROBE_TRY(hipGetLastError());
  PROBE_TRY(hipDeviceSynchronize());
  PROBE_TRY(hipEventRecord(e0, nullptr));
  for (uint32_t i = 0; i < iters; ++i) launch();
  PROBE_TRY(hipEventRecord(e1, nullptr));
  PROBE_TRY(hipEventSynchronize(e1));
  float ms = 0.f;
  PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  const double moved = (double)n_vec * 16.0 * (copy ? 2.0 : 1.0);
  *gb_per_s = moved * iters / ((double)ms * 1e-3) / 1e9;
  cleanup();
  return 0;
}

// Read-only pass over `bytes` of device memory: GB/s read.
int probe_read_stream(uint64_t bytes, uint32_t iters, double *gb_per_s) { return stream_probe(bytes, iters, false, gb_per_s); }
// Device-to-device copy of `bytes`: GB/s read + written.
int probe_copy(uint64_t bytes, uint32_t iters, double *gb_per_s) { return stream_probe(bytes, iters, true, gb_per_s); }

}  // extern "C"
