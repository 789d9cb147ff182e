// Data side of the method on the device (gfx950, wave64).
//
//   partition kernels   Section V-A: one seeded permutation of the n data points, by ranking 64-bit keys; its first
//                       o entries are the shared subset O, the next k blocks of floor((n-o)/k) the private subsets
//                       S_j, and row j of the index array holds D_j = O u S_j (O first, permutation order).
//   gather_kernel       each worker's minibatch: B uniform draws (with replacement) from its own D_j at its local
//                       step, rows and labels copied from the resident data set into the step's input buffers.
//
// The permutation is found by counting, for every point, the points whose (key, index) pair is smaller: n^2
// comparisons, but exact, free of any ordering of equal work between threads, and done once per run
// (n = 60000 takes well under a millisecond of compares).  The gather is a plain row copy bound by HBM bandwidth.
#include <mutex>

#include "dw_internal.h"

// Scratch of dw_overlap_partition_static: keys and ranks of up to DW_STATIC_MAX_POINTS points, in the layout
// partition_scratch_bytes describes.  Every device the library runs on holds its own copy at its own address until the
// process ends; host code reaches it only through the address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[(size_t)DW_STATIC_MAX_POINTS * 12];

namespace dw {

namespace {

constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ inline uint64_t mix64_d(uint64_t x) {      // SplitMix64 output function
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

__global__ __launch_bounds__(256) void partition_keys_kernel(uint64_t* keys, int32_t* rank, int64_t n, uint64_t k1) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  keys[i] = mix64_d(k1 + kGamma * (uint64_t)(i + 1));
  rank[i] = 0;
}

// rank[i] += number of points j of this block row's slice with (key_j, j) < (key_i, i)
__global__ __launch_bounds__(256) void partition_rank_kernel(const uint64_t* keys, int32_t* rank, int64_t n,
                                                             int64_t slice) {
  __shared__ uint64_t tile[256];
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const uint64_t mine = i < n ? keys[i] : 0;
  const int64_t j0 = (int64_t)blockIdx.y * slice;
  const int64_t j1 = j0 + slice < n ? j0 + slice : n;
  int32_t cnt = 0;
  for (int64_t base = j0; base < j1; base += 256) {            // uniform trip count: every thread reaches the barriers
    const int64_t j = base + threadIdx.x;
    __syncthreads();
    tile[threadIdx.x] = j < j1 ? keys[j] : ~0ull;
    __syncthreads();
    const int lim = (int)(j1 - base < 256 ? j1 - base : 256);
    for (int t = 0; t < lim; ++t) {
      const uint64_t other = tile[t];
      cnt += (other < mine || (other == mine && base + t < i)) ? 1 : 0;
    }
  }
  if (i < n && cnt != 0) atomicAdd(&rank[i], cnt);
}

__global__ __launch_bounds__(256) void partition_scatter_kernel(const int32_t* rank, int32_t* index, int64_t n,
                                                                int64_t o, int64_t s, int k) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int64_t r = rank[i];
  const int64_t m = o + s;
  if (r < o) {
    for (int j = 0; j < k; ++j) index[(int64_t)j * m + r] = (int32_t)i;
  } else if (s > 0) {
    const int64_t q = r - o;
    const int64_t j = q / s;
    if (j < k) index[j * m + o + (q - j * s)] = (int32_t)i;
  }
}

struct GatherKeys { uint64_t key[DW_MAX_K]; };

// block (b, j): draw b of worker j, one row of row_vecs 16-byte pieces
__global__ __launch_bounds__(256) void gather_kernel(const uint4* data, const int32_t* labels, const int32_t* index,
                                                     int64_t n, int64_t m, int row_vecs, int B, GatherKeys keys,
                                                     uint64_t active_mask, uint4* x, int32_t* y) {
  const int j = blockIdx.y, b = blockIdx.x;
  if (!((active_mask >> j) & 1ull)) return;
  const uint64_t u = mix64_d(keys.key[j] + kGamma * (uint64_t)(b + 1));
  const int64_t pos = (int64_t)__umul64hi(u, (uint64_t)m);     // floor(u * m / 2^64)
  const int64_t idx = index[(int64_t)j * m + pos];
  const bool ok = idx >= 0 && idx < n;                         // an index outside the data set yields a zero row
  uint4* dst = x + ((int64_t)j * B + b) * row_vecs;
  if (ok) {
    const uint4* src = data + idx * row_vecs;
    for (int v = threadIdx.x; v < row_vecs; v += 256) dst[v] = src[v];
    if (threadIdx.x == 0) y[(int64_t)j * B + b] = labels[idx];
  } else {
    for (int v = threadIdx.x; v < row_vecs; v += 256) dst[v] = make_uint4(0u, 0u, 0u, 0u);
    if (threadIdx.x == 0) y[(int64_t)j * B + b] = -1;
  }
}

}  // namespace

size_t partition_scratch_bytes(int64_t n) {
  const size_t keys = ((size_t)n * 8 + 255) / 256 * 256;
  const size_t rank = ((size_t)n * 4 + 255) / 256 * 256;
  return keys + rank;
}

hipError_t launch_partition(int64_t n, int64_t o, int k, uint64_t seed, int32_t* index, void* scratch, hipStream_t s) {
  uint64_t* keys = reinterpret_cast<uint64_t*>(scratch);
  int32_t* rank = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(scratch) + ((size_t)n * 8 + 255) / 256 * 256);
  const unsigned nb = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(partition_keys_kernel, dim3(nb), dim3(256), 0, s, keys, rank, n, mix64_d(seed));
  // enough block rows to fill the chip when n is small; each covers a slice of the points compared against
  int64_t rows = 2048 / nb;
  if (rows < 1) rows = 1;
  if (rows > nb) rows = nb;
  int64_t slice = ((n + rows - 1) / rows + 255) / 256 * 256;
  rows = (n + slice - 1) / slice;
  hipLaunchKernelGGL(partition_rank_kernel, dim3(nb, (unsigned)rows), dim3(256), 0, s, keys, rank, n, slice);
  const int64_t sz = (n - o) / k;
  hipLaunchKernelGGL(partition_scatter_kernel, dim3(nb), dim3(256), 0, s, rank, index, n, o, sz, k);
  return hipGetLastError();
}

hipError_t launch_gather(const void* data, const int32_t* labels, const int32_t* index, int64_t n, int64_t m,
                         int row_bytes, int B, int k, const uint64_t* keys_host, uint64_t active_mask, void* x,
                         int32_t* y, hipStream_t s) {
  KernelScope ks(KC_GATHER, s);
  GatherKeys keys;
  for (int i = 0; i < DW_MAX_K; ++i) keys.key[i] = i < k ? keys_host[i] : 0;
  hipLaunchKernelGGL(gather_kernel, dim3((unsigned)B, (unsigned)k), dim3(256), 0, s,
                     reinterpret_cast<const uint4*>(data), labels, index, n, m, row_bytes / 16, B, keys, active_mask,
                     reinterpret_cast<uint4*>(x), y);
  return hipGetLastError();
}

// device address of `scratch` on the current device, looked up once per device
hipError_t static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {nullptr};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

}  // namespace dw

extern "C" int64_t dw_overlap_partition_static(int64_t n, int64_t o, int k, uint64_t seed, int32_t* d_index,
                                               void* stream) {
  if (n < 1 || o < 0 || o > n || k < 1 || k > DW_MAX_K) return DW_ERR_ARG;
  if (n > DW_STATIC_MAX_POINTS) return DW_ERR_TOO_LARGE;
  static_assert(sizeof(scratch) % 256 == 0, "the rank array starts at a multiple of 256 bytes");
  if (dw::partition_scratch_bytes(n) > sizeof(scratch)) return DW_ERR_TOO_LARGE;
  const int64_t sz = (n - o) / k;
  if (!d_index && o + sz > 0) return DW_ERR_NULL;
  void* d_scratch = nullptr;
  hipError_t e = dw::static_scratch(&d_scratch);
  if (e == hipSuccess) e = dw::launch_partition(n, o, k, seed, d_index, d_scratch, (hipStream_t)stream);
  if (e != hipSuccess) return dw::note_hip_error(e);
  return sz;
}
