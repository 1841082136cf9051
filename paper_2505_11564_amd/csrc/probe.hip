// Kernels of the widened rows: the weighted accumulation of the batch loop of
// Algorithm 1 and the Hessian-column statistics of the section "Banded
// Hessians" (counts of entries below thresholds, equal-width histogram of the
// absolute values).  All HBM-bound streaming passes.
#include <mutex>

#include "hf_internal.h"

namespace hf {

static inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// h <- w u (first batch) or h <- h + w u: the step "h += u |B|" with the
// division by N folded into w = |B| / N.
__global__ void scale_add_kernel(float* __restrict__ h, const float* __restrict__ u, float w, int first, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t n4 = n >> 2;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const float4 x = ((const float4*)u)[i];
    float4 y = first ? make_float4(0.f, 0.f, 0.f, 0.f) : ((const float4*)h)[i];
    y.x += w * x.x; y.y += w * x.y; y.z += w * x.z; y.w += w * x.w;
    ((float4*)h)[i] = y;
  }
  for (int64_t i = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    h[i] = (first ? 0.f : h[i]) + w * u[i];
}
hipError_t launch_scale_add(float* h, const float* u, float w, int first, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (((uintptr_t)h | (uintptr_t)u) & 15) return hipErrorInvalidValue;
  const int blocks = (int)std::min<int64_t>(cdiv64(n, 1024), 4096);
  hipLaunchKernelGGL(scale_add_kernel, dim3(blocks), dim3(256), 0, st, h, u, w, first, n);
  return hipGetLastError();
}

// ---- column statistics --------------------------------------------------------
// stats (uint64): [0, 17) bucket counts (bucket b: entries that reach exactly b of the sorted
// thresholds), [17] NaN entries; [24] bit pattern of the largest |h_i| (non-negative floats order
// like their bit patterns); [32, 32 + n_bins) histogram.

__device__ __forceinline__ unsigned wave_sum_u32(unsigned v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// Thresholds arrive sorted ascending (the host sorts them and undoes the permutation), so an
// entry's contribution is one bucket index b = #{k : |h_i| >= t_k}, found by a branch-free binary
// search over the (padded to 16, +inf) thresholds; each thread counts buckets in its own LDS
// column (no atomics, no bank conflicts: counter [bucket][thread]), and the per-threshold counts are
// the prefix sums of the bucket counts, formed on the host.  NaN entries land in bucket 16.
__global__ __launch_bounds__(256) void colstats_pass1_kernel(const float* __restrict__ h, int64_t n, ColThresholds thr,
                                                            int nt, unsigned long long* stats) {
  __shared__ unsigned cnt[18][256];
  __shared__ float redm[4];
  __shared__ float lt[CS_MAX_THRESHOLDS];
#pragma unroll
  for (int k = 0; k < 18; ++k) cnt[k][threadIdx.x] = 0;
  if (threadIdx.x < CS_MAX_THRESHOLDS) lt[threadIdx.x] = thr.t[threadIdx.x];
  __syncthreads();
  float mx = 0.f;
  auto take = [&](float x) {
    const float a = fabsf(x);
    int b;
    if (a == a) {
      mx = fmaxf(mx, a);
      // binary search: b in [0, 16]
      b = a >= lt[7] ? 8 : 0;
      b += a >= lt[b + 3] ? 4 : 0;
      b += a >= lt[b + 1] ? 2 : 0;
      b += a >= lt[b] ? 1 : 0;
      b += (b == 15 && a >= lt[15]) ? 1 : 0;
    } else {
      b = 17;
    }
    cnt[b][threadIdx.x] += 1;
  };
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  // scalar head up to the first 16-byte boundary, vector body, scalar tail
  const int64_t head = std::min<int64_t>(n, (int64_t)((16 - ((uintptr_t)h & 15)) & 15) / 4);
  const int64_t n4 = (n - head) >> 2;
  if (gid < head) take(h[gid]);
  const f32x4_t* h4 = (const f32x4_t*)(h + head);
  for (int64_t i = gid; i < n4; i += stride) {
    const f32x4_t x = __builtin_nontemporal_load(h4 + i);
    take(x.x); take(x.y); take(x.z); take(x.w);
  }
  for (int64_t i = head + (n4 << 2) + gid; i < n; i += stride) take(h[i]);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  {
    float m = mx;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_down(m, o, 64));
    if (lane == 0) redm[wave] = m;
  }
  __syncthreads();
  // bucket totals of the block: thread k < 18 sums row k
  if (threadIdx.x < 18) {
    unsigned long long s = 0;
    for (int t = 0; t < 256; ++t) s += cnt[threadIdx.x][(t + threadIdx.x) & 255];
    if (s) atomicAdd(stats + threadIdx.x, s);
  }
  if (threadIdx.x == 0) {
    const float m = fmaxf(fmaxf(redm[0], redm[1]), fmaxf(redm[2], redm[3]));
    atomicMax((unsigned*)(stats + 24), __float_as_uint(m));
  }
}

// Bin of |h_i|: floor(|h_i| * scale), scale = n_bins / max as one correctly rounded float32
// quotient; the maximum itself (and a product that is not a number, which needs an infinite
// maximum) lands in the last bin.  The maximum is the first pass's result, read from the counters
// (max_bits: its bit pattern), so no host round trip separates the passes; a column without a
// positive maximum (all zeros, or empty) leaves the bins untouched for the host to fill in.
__global__ __launch_bounds__(256) void colstats_hist_kernel(const float* __restrict__ h, int64_t n,
                                                           const unsigned long long* __restrict__ max_bits, int nb,
                                                           unsigned long long* hist) {
  __shared__ unsigned lh[CS_MAX_BINS];
  const float mx = __uint_as_float((unsigned)*max_bits);
  if (!(mx > 0.f)) return;
  const float scale = __fdiv_rn((float)nb, mx);
  for (int i = threadIdx.x; i < nb; i += 256) lh[i] = 0;
  __syncthreads();
  // consecutive entries of a thread that fall in the same bin are counted in a register and added
  // to LDS once per run: a column that is nearly all zeros (the case the paper reports) would
  // otherwise send every lane to the same LDS address
  int last = -1;
  unsigned run = 0;
  auto take = [&](float x) {
    const float a = fabsf(x);
    if (a == a) {
      const float s = __fmul_rn(a, scale);
      const int b = (s == s) ? (int)fminf(floorf(s), (float)(nb - 1)) : nb - 1;
      if (b == last) { ++run; }
      else {
        if (run) atomicAdd(&lh[last], run);
        last = b; run = 1;
      }
    }
  };
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t head = std::min<int64_t>(n, (int64_t)((16 - ((uintptr_t)h & 15)) & 15) / 4);
  const int64_t n4 = (n - head) >> 2;
  if (gid < head) take(h[gid]);
  const f32x4_t* h4 = (const f32x4_t*)(h + head);
  for (int64_t i = gid; i < n4; i += stride) {
    const f32x4_t x = __builtin_nontemporal_load(h4 + i);
    take(x.x); take(x.y); take(x.z); take(x.w);
  }
  for (int64_t i = head + (n4 << 2) + gid; i < n; i += stride) take(h[i]);
  if (run) atomicAdd(&lh[last], run);
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += 256)
    if (lh[i]) atomicAdd(hist + i, (unsigned long long)lh[i]);
}

// Each thread sees at most n / (blocks * 256) + 4 elements, so 32-bit per-thread
// and per-block counters cannot overflow for n < 2^40 with these grids.
static inline int colstats_blocks(int64_t n) { return (int)std::max<int64_t>(1, std::min<int64_t>(cdiv64(n, 4096), 2048)); }

hipError_t launch_colstats_pass1(const float* h, int64_t n, const ColThresholds& thr, int nt, unsigned long long* stats,
                                 hipStream_t st) {
  hipLaunchKernelGGL(colstats_pass1_kernel, dim3(colstats_blocks(n)), dim3(256), 0, st, h, n, thr, nt, stats);
  return hipGetLastError();
}
hipError_t launch_colstats_hist(const float* h, int64_t n, const unsigned long long* max_bits, int nb, unsigned long long* hist,
                                hipStream_t st) {
  hipLaunchKernelGGL(colstats_hist_kernel, dim3(colstats_blocks(n)), dim3(256), 0, st, h, n, max_bits, nb, hist);
  return hipGetLastError();
}

// ---- counters for callers that cannot allocate -------------------------------------
// A fixed array in the library's device image, one copy per GPU, held until the process ends.
// Host code must not hand the symbol itself to a kernel: its device address is looked up once per
// device (with that device current) and only that pointer is used afterwards.
static __device__ __align__(256) unsigned long long scratch[CS_STATS_WORDS];

hipError_t colstats_static_counters(unsigned long long** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static unsigned long long* ptr[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr[dev] = (unsigned long long*)p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

}  // namespace hf
