// Bandwidth-bound vector kernels of the Lanczos iteration (Algorithm 2 of the
// paper) and of the full orthogonalisation against a stored basis Q that
// Section "Memory Compute trade off" uses as its baseline.
//
// Per iteration, with w = H q_k already computed.
// Without a basis (three-term recurrence), r' = w - beta_{k-1} q_{k-1}, r = r' - alpha_k q_k:
//   lz3_dots      : alpha_k = <q_k, r'>, <r', r'>, <q_k, q_k>; r' is formed on the fly   (3R)
//   lz3_finish    : beta_k^2 = ||r||^2 = <r', r'> - alpha_k^2 (2 - <q_k, q_k>), an identity of the
//                   fp32 vectors as stored; where the difference has lost its digits
//   lz3_norm      : forms ||r||^2 explicitly (3R), else returns at once
//   lz3_normalise : q_{k+1} = (w - beta_{k-1} q_{k-1} - alpha_k q_k) / beta_k written over
//                   q_{k-1}                                                              (3R + 1W)
// With a stored basis the first Gram-Schmidt pass is applied to w itself (against q_0 .. q_k; with
// a bf16 basis q_k and q_{k-1} are taken from the fp32 working vectors): alpha_k is its k-th
// coefficient and the two three-term subtractions are part of the pass:
//   lz_qtr      : c = Q^T r      (k+1 dot products, Q read once)
//   lz_sub_qc   : r -= Q c;  beta_k = ||r||   (Q read once)
//   lz_scale    : q_{k+1} = r / beta_k, written to its basis row                          (1R + 1W)
// Scalars stay on the device (array `scal` of doubles) so consecutive kernels
// need no host round trip; the kernels that write q_{k+1} test beta_k against the
// tolerance (and the error flags of the product that made w) themselves and leave
// the state untouched when the iteration must not advance, so the host reads the
// scalars once, after everything has been enqueued.  Reductions: fp64 per-thread
// accumulators, one partial per block, summed in a fixed order by a small second
// kernel, so results are bitwise reproducible.
#include "hf_internal.h"
#include "lanczos.h"

namespace hf {

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ double block_sum_d(double v, double* red) {
  v = wave_sum_d(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// Streaming passes over n-vectors, 16 bytes per access, as measured at n = 1.2e8 .. 6.7e9:
//  - passes that only read (dot products) walk the vector with a grid-wide stride, two groups in
//    flight per thread, at most LZ_NBLK_VEC blocks (one partial sum each): 6.6-7.0 TB/s with
//    non-temporal loads (5.3-5.9 with plain ones, or with one contiguous run per block);
//  - passes that also write launch one thread per two groups (no loop; the thread's second group
//    lies half a vector further on): 6.0-6.6 TB/s with non-temporal loads and stores, against
//    4.0-5.1 for a looping grid of a few thousand blocks.
typedef float lz_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned lz_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 ldnt4(const float* p, int64_t i4) {
  const lz_f32x4 v = __builtin_nontemporal_load((const lz_f32x4*)p + i4);
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stnt4(float* p, int64_t i4, const float4& v) {
  lz_f32x4 x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, (lz_f32x4*)p + i4);
}
__device__ __forceinline__ void stnt_bf16x4(bf16* p, int64_t i4, const float4& v) {
  const bf16 o[4] = {(bf16)v.x, (bf16)v.y, (bf16)v.z, (bf16)v.w};
  __builtin_nontemporal_store(*(const lz_u32x2*)o, (lz_u32x2*)p + i4);
}

__device__ __forceinline__ float4 fnma4(float c, const float4& x, const float4& y) {  // y - c x
  return make_float4(fmaf(-c, x.x, y.x), fmaf(-c, x.y, y.y), fmaf(-c, x.z, y.z), fmaf(-c, x.w, y.w));
}
__device__ __forceinline__ float4 scale4(const float4& x, float c) { return make_float4(x.x * c, x.y * c, x.z * c, x.w * c); }
__device__ __forceinline__ double dot4(const float4& a, const float4& b) {
  return (double)a.x * b.x + (double)a.y * b.y + (double)a.z * b.z + (double)a.w * b.w;
}

// partials[block] = sum of z^2 over the groups the block visits
__global__ __launch_bounds__(256) void lz_sumsq_kernel(const float* __restrict__ z, int64_t n, double* __restrict__ partials) {
  __shared__ double red[4];
  double acc = 0.0;
  const int64_t n4 = n >> 2, step = (int64_t)gridDim.x * 256;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + step < n4; i += 2 * step) {
    const float4 a = ldnt4(z, i), b = ldnt4(z, i + step);
    acc += dot4(a, a) + dot4(b, b);
  }
  if (i < n4) { const float4 a = ldnt4(z, i); acc += dot4(a, a); }
  for (int64_t e = (n4 << 2) + (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += step) acc += (double)z[e] * z[e];
  acc = block_sum_d(acc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}

// Three-term recurrence, first pass (read only).  With r' = w - bprev qp formed on the fly
// (use_prev = 0: r' = w): partials[0][block] = <q, r'>, [1][block] = <r', r'>, [2][block] = <q, q>.
__global__ __launch_bounds__(256) void lz3_dots_kernel(const float* __restrict__ w, const float* __restrict__ q,
                                                       const float* __restrict__ qp, int64_t n, int use_prev, float bprev,
                                                       double* __restrict__ partials) {
  __shared__ double red[4];
  double a0 = 0.0, a1 = 0.0, a2 = 0.0;
  const int64_t n4 = n >> 2, step = (int64_t)gridDim.x * 256;
  auto take = [&](float4 rv, const float4& qv, const float4& pv) {
    if (use_prev) rv = fnma4(bprev, pv, rv);
    a0 += dot4(rv, qv); a1 += dot4(rv, rv); a2 += dot4(qv, qv);
  };
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + step < n4; i += 2 * step) {
    const float4 r0 = ldnt4(w, i), r1 = ldnt4(w, i + step), q0 = ldnt4(q, i), q1 = ldnt4(q, i + step);
    const float4 p0 = use_prev ? ldnt4(qp, i) : zero, p1 = use_prev ? ldnt4(qp, i + step) : zero;
    take(r0, q0, p0);
    take(r1, q1, p1);
  }
  if (i < n4) take(ldnt4(w, i), ldnt4(q, i), use_prev ? ldnt4(qp, i) : zero);
  for (int64_t e = (n4 << 2) + (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += step) {
    float rv = w[e];
    if (use_prev) rv = fmaf(-bprev, qp[e], rv);
    a0 += (double)rv * q[e]; a1 += (double)rv * rv; a2 += (double)q[e] * q[e];
  }
  a0 = block_sum_d(a0, red);
  a1 = block_sum_d(a1, red);
  a2 = block_sum_d(a2, red);
  if (threadIdx.x == 0) {
    partials[blockIdx.x] = a0;
    partials[gridDim.x + blockIdx.x] = a1;
    partials[2 * (int64_t)gridDim.x + blockIdx.x] = a2;
  }
}

// alpha_k and, from the three sums, ||r' - alpha q||^2 = <r',r'> - 2 alpha <q,r'> + alpha^2 <q,q>
// = <r',r'> - alpha^2 (2 - <q,q>): an identity of the fp32 vectors as the passes read them, so
// only the fp64 summation error (about 1e-15 <r',r'>) is amplified by the cancellation; below
// 1e-6 <r',r'> the norm is formed explicitly instead (scal[S_REDO] = 1 asks lz3_norm for it).
__global__ __launch_bounds__(256) void lz3_finish_kernel(const double* __restrict__ partials, int nblk, double* __restrict__ scal) {
  __shared__ double red[4];
  double s[3];
  for (int j = 0; j < 3; ++j) {
    double a = 0.0;
    for (int i = threadIdx.x; i < nblk; i += 256) a += partials[(int64_t)j * nblk + i];
    s[j] = block_sum_d(a, red);
  }
  if (threadIdx.x != 0) return;
  const double al = s[0], rest = s[1] - al * al * (2.0 - s[2]);
  scal[S_ALPHA] = al;
  if (rest > 1e-6 * s[1]) { scal[S_BETA] = sqrt(rest); scal[S_REDO] = 0.0; }
  else { scal[S_BETA] = 0.0; scal[S_REDO] = 1.0; }   // also taken when a sum is NaN
}

// Only when lz3_finish asked for it: partials[block] = ||w - bprev qp - alpha q||^2 (read only).
__global__ __launch_bounds__(256) void lz3_norm_kernel(const float* __restrict__ w, const float* __restrict__ q,
                                                       const float* __restrict__ qp, int64_t n, int use_prev, float bprev,
                                                       const double* __restrict__ scal, double* __restrict__ partials) {
  __shared__ double red[4];
  if (scal[S_REDO] == 0.0) return;
  const float al = (float)scal[S_ALPHA];
  double acc = 0.0;
  const int64_t n4 = n >> 2, step = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += step) {
    float4 rv = ldnt4(w, i);
    if (use_prev) rv = fnma4(bprev, ldnt4(qp, i), rv);
    rv = fnma4(al, ldnt4(q, i), rv);
    acc += dot4(rv, rv);
  }
  for (int64_t e = (n4 << 2) + (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += step) {
    float rv = w[e];
    if (use_prev) rv = fmaf(-bprev, qp[e], rv);
    rv = fmaf(-al, q[e], rv);
    acc += (double)rv * rv;
  }
  acc = block_sum_d(acc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}

// what 0: scal[S_Q0NORM] = sqrt(sum);
// 2 (after lz3_norm, only when it ran): scal[S_BETA] = sqrt(sum);
// 3 (after an orthogonalisation pass): scal[S_BETA] = sqrt(sum), redo flag set
//    iff this was the first pass and the norm fell below 1/sqrt(2) of its
//    value before the pass.
__global__ __launch_bounds__(256) void lz_finish_kernel(const double* partials, int nblk, int what, int pass,
                                                        double* scal) {
  __shared__ double red[4];
  if (what == 3 && pass == 1 && scal[S_REDO] == 0.0) return;
  if (what == 2 && scal[S_REDO] == 0.0) return;
  double s = 0.0;
  for (int i = threadIdx.x; i < nblk; i += 256) s += partials[i];
  s = block_sum_d(s, red);
  if (threadIdx.x != 0) return;
  if (what == 0) scal[S_Q0NORM] = sqrt(s);
  else if (what == 2) { scal[S_BETA] = sqrt(s); scal[S_REDO] = 0.0; }
  else {
    const double nb = sqrt(s);
    scal[S_BETA] = nb;
    scal[S_REDO] = (pass == 0 && nb < scal[S_NRM_BEFORE] * 0.70710678118654752) ? 1.0 : 0.0;
    scal[S_NRM_BEFORE] = nb;
  }
}

// Whether iteration k may write q_{k+1}: beta_k (scal[idx]) is a positive number not below the
// tolerance, and the product that made w reported no bad token / label (flags, may be NULL).
// The first thread of the grid also leaves the flags in scal[S_FLAG0], scal[S_FLAG1] for the host.
__device__ __forceinline__ bool lz_may_advance(double* scal, int idx, double tol, const int* flags) {
  const double b = scal[idx];
  bool ok = (b >= tol) && (b > 0.0);
  if (flags) {
    const int f0 = flags[0], f1 = flags[1];
    if (blockIdx.x == 0 && threadIdx.x == 0) { scal[S_FLAG0] = (double)f0; scal[S_FLAG1] = (double)f1; }
    ok = ok && f0 == 0 && f1 != 0;
  }
  return ok;
}

// Three-term recurrence, last pass: qp <- (w - bprev qp - alpha q) / beta (q_{k+1} over q_{k-1}), and
// optionally vb = its bf16 copy (the operand-type copy of the next Hessian-vector product's
// direction, which would otherwise cost that product a pass over q_{k+1}).  One thread per two
// 16-byte groups: i and i + gridDim.x * 256.
__global__ __launch_bounds__(256) void lz3_normalise_kernel(const float* __restrict__ w, const float* __restrict__ q,
                                                            float* __restrict__ qp, bf16* __restrict__ vb, int64_t n,
                                                            int use_prev, float bprev, double* scal, double tol,
                                                            const int* flags) {
  if (!lz_may_advance(scal, S_BETA, tol, flags)) return;
  const float al = (float)scal[S_ALPHA];
  const float inv = (float)(1.0 / scal[S_BETA]);
  const int64_t n4 = n >> 2, half = (int64_t)gridDim.x * 256;
  const int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x, i1 = i0 + half;
  const bool ok0 = i0 < n4, ok1 = i1 < n4;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 r0 = zero, r1 = zero, q0 = zero, q1 = zero, p0 = zero, p1 = zero;
  if (ok0) { r0 = ldnt4(w, i0); q0 = ldnt4(q, i0); if (use_prev) p0 = ldnt4(qp, i0); }
  if (ok1) { r1 = ldnt4(w, i1); q1 = ldnt4(q, i1); if (use_prev) p1 = ldnt4(qp, i1); }
  if (ok0) {
    if (use_prev) r0 = fnma4(bprev, p0, r0);
    r0 = scale4(fnma4(al, q0, r0), inv);
    stnt4(qp, i0, r0);
    if (vb) stnt_bf16x4(vb, i0, r0);
  }
  if (ok1) {
    if (use_prev) r1 = fnma4(bprev, p1, r1);
    r1 = scale4(fnma4(al, q1, r1), inv);
    stnt4(qp, i1, r1);
    if (vb) stnt_bf16x4(vb, i1, r1);
  }
  const int64_t e = (n4 << 2) + threadIdx.x;   // ragged tail: at most three elements, block 0
  if (blockIdx.x == 0 && e < n) {
    float rv = w[e];
    if (use_prev) rv = fmaf(-bprev, qp[e], rv);
    rv = fmaf(-al, q[e], rv) * inv;
    qp[e] = rv;
    if (vb) vb[e] = (bf16)rv;
  }
}

// q_{k+1} = src / scal[idx] into any of: dst (fp32 working vector), basis (its row of the stored
// basis, fp32 or bf16 rounded to nearest even), vb (bf16 copy for the next Hessian-vector product).
// One thread per two 16-byte groups.
template <typename BT>
__global__ __launch_bounds__(256) void lz_scale_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                       BT* __restrict__ basis, bf16* __restrict__ vb, int64_t n,
                                                       double* scal, int idx, double tol, const int* flags) {
  if (!lz_may_advance(scal, idx, tol, flags)) return;
  const float inv = (float)(1.0 / scal[idx]);
  const int64_t n4 = n >> 2, half = (int64_t)gridDim.x * 256;
  const int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x, i1 = i0 + half;
  const bool ok0 = i0 < n4, ok1 = i1 < n4;
  float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
  if (ok0) v0 = ldnt4(src, i0);
  if (ok1) v1 = ldnt4(src, i1);
  auto put = [&](int64_t i, float4 v) {
    v = scale4(v, inv);
    if (dst) stnt4(dst, i, v);
    if (basis) {
      if (sizeof(BT) == 4) stnt4((float*)basis, i, v);
      else stnt_bf16x4((bf16*)basis, i, v);
    }
    if (vb) stnt_bf16x4(vb, i, v);
  };
  if (ok0) put(i0, v0);
  if (ok1) put(i1, v1);
  const int64_t e = (n4 << 2) + threadIdx.x;
  if (blockIdx.x == 0 && e < n) {
    const float v = src[e] * inv;
    if (dst) dst[e] = v;
    if (basis) basis[e] = (BT)v;
    if (vb) vb[e] = (bf16)v;
  }
}

template <typename BT>
__device__ __forceinline__ float4 load4(const BT* p, int64_t i4);
template <>
__device__ __forceinline__ float4 load4<float>(const float* p, int64_t i4) { return ((const float4*)p)[i4]; }
template <>
__device__ __forceinline__ float4 load4<bf16>(const bf16* p, int64_t i4) {
  const uint2 u = ((const uint2*)p)[i4];
  float4 v;
  v.x = __uint_as_float(u.x << 16); v.y = __uint_as_float(u.x & 0xffff0000u);
  v.z = __uint_as_float(u.y << 16); v.w = __uint_as_float(u.y & 0xffff0000u);
  return v;
}

// Re-orthogonalisation kernels.  Both stream the basis once: the vectors are
// cut into slices of LZ_SLICE elements; a block keeps its slice of r in
// registers (16 floats per thread) and walks the stored vectors j = 0..nq-1,
// issuing 16 B loads for the whole slice of Q_j before using them, so every
// basis byte is read exactly once per kernel with many loads in flight and
// contiguous 16 KB / 8 KB runs per vector (measured best among 2K..16K); the loads of vector
// j+1 are issued before vector j is consumed.
constexpr int LZ_SLICE = 4096;            // elements per slice
constexpr int LZ_RPT = LZ_SLICE / 256;    // r elements per thread

typedef unsigned lz_u32x4 __attribute__((ext_vector_type(4)));
template <typename BT> struct QVec;
template <> struct QVec<float> {  // 4 elements per 16 B load, 16 loads per slice
  static constexpr int E = 4, U = LZ_RPT / 4;
  typedef lz_f32x4 raw;
  __device__ static __forceinline__ void unpack(const raw& q, float* o) { o[0] = q.x; o[1] = q.y; o[2] = q.z; o[3] = q.w; }
};
template <> struct QVec<bf16> {   // 8 elements per 16 B load, 8 loads per slice
  static constexpr int E = 8, U = LZ_RPT / 8;
  typedef lz_u32x4 raw;
  __device__ static __forceinline__ void unpack(const raw& q, float* o) {
    o[0] = __uint_as_float(q.x << 16); o[1] = __uint_as_float(q.x & 0xffff0000u);
    o[2] = __uint_as_float(q.y << 16); o[3] = __uint_as_float(q.y & 0xffff0000u);
    o[4] = __uint_as_float(q.z << 16); o[5] = __uint_as_float(q.z & 0xffff0000u);
    o[6] = __uint_as_float(q.w << 16); o[7] = __uint_as_float(q.w & 0xffff0000u);
  }
};

// Thread t owns elements base + (t + 256 u) E .. + E of the slice, u < U.
template <typename BT>
__device__ __forceinline__ void load_r_slice(const float* __restrict__ r, int64_t base, int64_t n, float (&rv)[LZ_RPT]) {
  typedef QVec<BT> V;
#pragma unroll
  for (int u = 0; u < V::U; ++u) {
    const int64_t e0 = base + (int64_t)(threadIdx.x + 256 * u) * V::E;
#pragma unroll
    for (int h = 0; h < V::E / 4; ++h) {
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e0 + h * 4 + 4 <= n) x = *(const float4*)(r + e0 + h * 4);
      else {
        float t4[4] = {0.f, 0.f, 0.f, 0.f};
        for (int q = 0; q < 4; ++q) if (e0 + h * 4 + q < n) t4[q] = r[e0 + h * 4 + q];
        x = make_float4(t4[0], t4[1], t4[2], t4[3]);
      }
      rv[u * V::E + h * 4 + 0] = x.x; rv[u * V::E + h * 4 + 1] = x.y;
      rv[u * V::E + h * 4 + 2] = x.z; rv[u * V::E + h * 4 + 3] = x.w;
    }
  }
}

template <typename BT>
__device__ __forceinline__ void load_q_slice(const BT* __restrict__ q, int64_t base, int64_t n, bool full,
                                             typename QVec<BT>::raw (&qv)[QVec<BT>::U]) {
  typedef QVec<BT> V;
#pragma unroll
  for (int u = 0; u < V::U; ++u) {
    const int64_t e0 = base + (int64_t)(threadIdx.x + 256 * u) * V::E;
    if (full || e0 + V::E <= n) {
      qv[u] = __builtin_nontemporal_load((const typename V::raw*)(q + e0));
    } else {
      BT t8[V::E];
      for (int k = 0; k < V::E; ++k) t8[k] = (e0 + k < n) ? q[e0 + k] : (BT)0.f;
      qv[u] = *(const typename V::raw*)t8;
    }
  }
}

// c_j = <Q_j, r>: partials[j * nblk + block] (fp64), summed by lz_qtr_finish_kernel.
// RR: one more result, c_nq = <r, r>.
// x0, x1 (optional, fp32 vectors): two more "rows" after the nq stored ones, results nq and nq + 1
// (x1 alone is not allowed); the <r, r> result then follows them.
template <typename BT, bool RR = false, bool XR = false>
__global__ __launch_bounds__(256) void lz_qtr_kernel(const BT* __restrict__ Q, int64_t ldq, const float* __restrict__ r,
                                                     int64_t n, int nq, int64_t nslices, const double* scal, int pass,
                                                     double* __restrict__ partials, const float* __restrict__ x0 = nullptr,
                                                     const float* __restrict__ x1 = nullptr) {
  typedef QVec<BT> V;
  extern __shared__ double accs[];  // [4 waves][na]
  if (pass == 1 && scal[S_REDO] == 0.0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nx = XR ? (x0 ? 1 : 0) + (x1 ? 1 : 0) : 0;
  const int na = nq + nx + (RR ? 1 : 0);
  for (int j = threadIdx.x; j < 4 * na; j += 256) accs[j] = 0.0;
  __syncthreads();
  for (int64_t sl = blockIdx.x; sl < nslices; sl += gridDim.x) {
    const int64_t base = sl * LZ_SLICE;
    const bool full = base + LZ_SLICE <= n;
    float rv[LZ_RPT];
    load_r_slice<BT>(r, base, n, rv);
    if (RR) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < LZ_RPT; ++k) s = fmaf(rv[k], rv[k], s);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (lane == 0) accs[wave * na + nq + nx] += (double)s;
    }
    // the fp32 rows, in r's register layout
    auto dot_x = [&](const float* __restrict__ x, int j) {
      float xv[LZ_RPT];
      load_r_slice<BT>(x, base, n, xv);
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < LZ_RPT; ++k) s = fmaf(xv[k], rv[k], s);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (lane == 0) accs[wave * na + j] += (double)s;
    };
    if constexpr (XR) {
      if (x0) dot_x(x0, nq);
      if (x1) dot_x(x1, nq + 1);
      if (nq == 0) continue;
    }
    auto dot_j = [&](const typename V::raw (&qv)[V::U], int j) {
      float s = 0.f;
#pragma unroll
      for (int u = 0; u < V::U; ++u) {
        float qf[V::E];
        V::unpack(qv[u], qf);
#pragma unroll
        for (int k = 0; k < V::E; ++k) s = fmaf(qf[k], rv[u * V::E + k], s);
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (lane == 0) accs[wave * na + j] += (double)s;
    };
    typename V::raw qa[V::U], qb[V::U];
    load_q_slice<BT>(Q, base, n, full, qa);
#pragma unroll 1
    for (int j = 0; j < nq; j += 2) {
      if (j + 1 < nq) load_q_slice<BT>(Q + (int64_t)(j + 1) * ldq, base, n, full, qb);
      dot_j(qa, j);
      if (j + 2 < nq) load_q_slice<BT>(Q + (int64_t)(j + 2) * ldq, base, n, full, qa);
      if (j + 1 < nq) dot_j(qb, j + 1);
    }
  }
  __syncthreads();
  for (int j = threadIdx.x; j < na; j += 256)
    partials[(int64_t)j * gridDim.x + blockIdx.x] = accs[j] + accs[na + j] + accs[2 * na + j] + accs[3 * na + j];
}

// After c = Q^T w and c_nq = <w, w> (w = H q_k, Q = q_0 .. q_k in fp32): alpha_k = c_k, and the
// norm that the three-term recurrence would have left before the orthogonalisation pass,
// ||w - alpha_k q_k - c_{k-1} q_{k-1}||, follows from the three numbers.  Where that difference
// has lost its digits (beta_k tiny against alpha_k) the norm is set to infinity, which makes the
// pass that follows ask for a second one.
__global__ void lz_direct_scal_kernel(const double* __restrict__ c, int nq, double* __restrict__ scal) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const double a = c[nq - 1], p = nq >= 2 ? c[nq - 2] : 0.0, ww = c[nq];
  const double rest = ww - a * a - p * p;
  scal[S_ALPHA] = a;
  scal[S_NRM_BEFORE] = rest > 1e-5 * ww ? sqrt(rest) : INFINITY;
  scal[S_REDO] = 0.0;
}

__global__ __launch_bounds__(256) void lz_qtr_finish_kernel(const double* partials, int nblk, const double* scal,
                                                            int pass, double* c) {
  __shared__ double red[4];
  if (pass == 1 && scal[S_REDO] == 0.0) return;
  const int j = blockIdx.x;
  double s = 0.0;
  for (int i = threadIdx.x; i < nblk; i += 256) s += partials[(int64_t)j * nblk + i];
  s = block_sum_d(s, red);
  if (threadIdx.x == 0) c[j] = s;
}

// r -= sum_j c_j Q_j, partial ||r||^2.
// x0, x1 (optional, fp32 vectors): two more rows with coefficients c[nq], c[nq + 1].
template <typename BT, bool XR = false>
__global__ __launch_bounds__(256) void lz_sub_qc_kernel(const BT* __restrict__ Q, int64_t ldq, float* __restrict__ r,
                                                        int64_t n, int nq, int64_t nslices, const double* __restrict__ c,
                                                        const double* scal, int pass, double* __restrict__ partials,
                                                        const float* __restrict__ x0 = nullptr, const float* __restrict__ x1 = nullptr) {
  typedef QVec<BT> V;
  extern __shared__ float cs[];
  __shared__ double red[4];
  if (pass == 1 && scal[S_REDO] == 0.0) return;
  const int nx = XR ? (x0 ? 1 : 0) + (x1 ? 1 : 0) : 0;
  for (int j = threadIdx.x; j < nq + nx; j += 256) cs[j] = (float)c[j];
  __syncthreads();
  double acc = 0.0;
  for (int64_t sl = blockIdx.x; sl < nslices; sl += gridDim.x) {
    const int64_t base = sl * LZ_SLICE;
    const bool full = base + LZ_SLICE <= n;
    float rv[LZ_RPT];
    load_r_slice<BT>(r, base, n, rv);
    auto sub_j = [&](const typename V::raw (&qv)[V::U], int j) {
      const float cj = cs[j];
#pragma unroll
      for (int u = 0; u < V::U; ++u) {
        float qf[V::E];
        V::unpack(qv[u], qf);
#pragma unroll
        for (int k = 0; k < V::E; ++k) rv[u * V::E + k] = fmaf(-cj, qf[k], rv[u * V::E + k]);
      }
    };
    auto sub_x = [&](const float* __restrict__ x, int j) {
      float xv[LZ_RPT];
      load_r_slice<BT>(x, base, n, xv);
      const float cj = cs[j];
#pragma unroll
      for (int k = 0; k < LZ_RPT; ++k) rv[k] = fmaf(-cj, xv[k], rv[k]);
    };
    if constexpr (XR) {
      if (x0) sub_x(x0, nq);
      if (x1) sub_x(x1, nq + 1);
    }
    if (!XR || nq > 0) {
      // three rows in flight ahead of the one being subtracted
      typename V::raw q0[V::U], q1[V::U], q2[V::U], q3[V::U];
      auto row = [&](int j) { return Q + (int64_t)j * ldq; };
      load_q_slice<BT>(row(0), base, n, full, q0);
      if (1 < nq) load_q_slice<BT>(row(1), base, n, full, q1);
      if (2 < nq) load_q_slice<BT>(row(2), base, n, full, q2);
#pragma unroll 1
      for (int j = 0; j < nq; j += 4) {
        if (j + 3 < nq) load_q_slice<BT>(row(j + 3), base, n, full, q3);
        sub_j(q0, j);
        if (j + 1 < nq) {
          if (j + 4 < nq) load_q_slice<BT>(row(j + 4), base, n, full, q0);
          sub_j(q1, j + 1);
        }
        if (j + 2 < nq) {
          if (j + 5 < nq) load_q_slice<BT>(row(j + 5), base, n, full, q1);
          sub_j(q2, j + 2);
        }
        if (j + 3 < nq) {
          if (j + 6 < nq) load_q_slice<BT>(row(j + 6), base, n, full, q2);
          sub_j(q3, j + 3);
        }
      }
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < V::U; ++u) {
      const int64_t e0 = base + (int64_t)(threadIdx.x + 256 * u) * V::E;
#pragma unroll
      for (int h = 0; h < V::E / 4; ++h) {
        const float* x = rv + u * V::E + h * 4;
        if (e0 + h * 4 + 4 <= n) {
          *(float4*)(r + e0 + h * 4) = make_float4(x[0], x[1], x[2], x[3]);
          s += x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
        } else {
          for (int q = 0; q < 4; ++q)
            if (e0 + h * 4 + q < n) { r[e0 + h * 4 + q] = x[q]; s += x[q] * x[q]; }
        }
      }
    }
    acc += (double)s;
  }
  acc = block_sum_d(acc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}

template <typename BT>
__global__ void lz_widen_kernel(const BT* src, float* dst, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = (float)src[i];
}

// ------------------------------------------------------------- launchers ----

// grid of a pass that only reads: grid-wide stride, two groups per thread in flight
static int vec_blocks(int64_t n) {
  const int64_t want = (n / 4 + 511) / 512;
  return (int)std::max<int64_t>(1, std::min<int64_t>(want, LZ_NBLK_VEC));
}
// grid of a pass that writes: one thread per two groups
static unsigned wide_blocks(int64_t n) { return (unsigned)std::max<int64_t>(1, (n / 4 + 511) / 512); }

hipError_t lz_norm_q0(const float* z, int64_t n, double* scal, double* partials, hipStream_t st) {
  const int nb = vec_blocks(n);
  hipLaunchKernelGGL(lz_sumsq_kernel, dim3(nb), dim3(256), 0, st, z, n, partials);
  hipLaunchKernelGGL(lz_finish_kernel, dim3(1), dim3(256), 0, st, partials, nb, 0, 0, scal);
  return hipGetLastError();
}

hipError_t lz3_update(const float* w, const float* q, float* qp, bf16* vb, int64_t n, int use_prev, double beta_prev,
                      double tol, const int* flags, double* scal, double* partials, hipStream_t st) {
  const int nb = vec_blocks(n);
  const float bp = (float)beta_prev;
  hipLaunchKernelGGL(lz3_dots_kernel, dim3(nb), dim3(256), 0, st, w, q, qp, n, use_prev, bp, partials);
  hipLaunchKernelGGL(lz3_finish_kernel, dim3(1), dim3(256), 0, st, partials, nb, scal);
  hipLaunchKernelGGL(lz3_norm_kernel, dim3(nb), dim3(256), 0, st, w, q, qp, n, use_prev, bp, scal, partials);
  hipLaunchKernelGGL(lz_finish_kernel, dim3(1), dim3(256), 0, st, partials, nb, 2, 0, scal);
  hipLaunchKernelGGL(lz3_normalise_kernel, dim3(wide_blocks(n)), dim3(256), 0, st, w, q, qp, vb, n, use_prev, bp, scal, tol, flags);
  return hipGetLastError();
}

hipError_t lz_scale(const float* src, float* dst, void* basis, int basis_bf16, bf16* vb, int64_t n, double* scal, int idx,
                    double tol, const int* flags, hipStream_t st) {
  const unsigned nb = wide_blocks(n);
  if (basis_bf16) hipLaunchKernelGGL(lz_scale_kernel<bf16>, dim3(nb), dim3(256), 0, st, src, dst, (bf16*)basis, vb, n, scal, idx, tol, flags);
  else hipLaunchKernelGGL(lz_scale_kernel<float>, dim3(nb), dim3(256), 0, st, src, dst, (float*)basis, vb, n, scal, idx, tol, flags);
  return hipGetLastError();
}

// r -= Q c for an fp32 basis of nq rows.  With bf16 copies of the rows at hand, rows 0 .. nq-3 are
// read from the copies (their coefficients are what rounding left of the orthogonality, so the
// rounding of a copy changes r far below its own last bit) and rows nq-2, nq-1, which carry
// beta_{k-1} and alpha_k, from the basis.
static void launch_sub_f32(const float* Q, const bf16* copies, int64_t ldq, float* r, int64_t n, int nq, int64_t nslices,
                           int nb, const double* c, const double* scal, int pass, double* partials, hipStream_t st) {
  const size_t sh = (size_t)nq * sizeof(float);
  if (copies && nq >= 3)
    hipLaunchKernelGGL((lz_sub_qc_kernel<bf16, true>), dim3(nb), dim3(256), sh, st, copies, ldq, r, n, nq - 2, nslices, c, scal,
                       pass, partials, Q + (int64_t)(nq - 2) * ldq, Q + (int64_t)(nq - 1) * ldq);
  else
    hipLaunchKernelGGL(lz_sub_qc_kernel<float>, dim3(nb), dim3(256), sh, st, Q, ldq, r, n, nq, nslices, c, scal, pass, partials);
}

hipError_t lz_reorth_pass(const void* Q, int basis_bf16, const bf16* copies, int64_t ldq, float* r, int64_t n, int nq, int pass,
                          double* scal, double* c, double* partials, hipStream_t st) {
  if (nq <= 0) return hipSuccess;
  const int64_t nslices = (n + LZ_SLICE - 1) / LZ_SLICE;
  const int nb = (int)std::max<int64_t>(1, std::min<int64_t>(nslices, LZ_NBLK));
  const size_t sh1 = (size_t)4 * nq * sizeof(double), sh2 = (size_t)nq * sizeof(float);
  if (basis_bf16) {
    hipLaunchKernelGGL(lz_qtr_kernel<bf16>, dim3(nb), dim3(256), sh1, st, (const bf16*)Q, ldq, r, n, nq, nslices, scal, pass, partials);
    hipLaunchKernelGGL(lz_qtr_finish_kernel, dim3(nq), dim3(256), 0, st, partials, nb, scal, pass, c);
    hipLaunchKernelGGL(lz_sub_qc_kernel<bf16>, dim3(nb), dim3(256), sh2, st, (const bf16*)Q, ldq, r, n, nq, nslices, c, scal, pass, partials);
  } else {
    hipLaunchKernelGGL(lz_qtr_kernel<float>, dim3(nb), dim3(256), sh1, st, (const float*)Q, ldq, r, n, nq, nslices, scal, pass, partials);
    hipLaunchKernelGGL(lz_qtr_finish_kernel, dim3(nq), dim3(256), 0, st, partials, nb, scal, pass, c);
    launch_sub_f32((const float*)Q, copies, ldq, r, n, nq, nslices, nb, c, scal, pass, partials, st);
  }
  hipLaunchKernelGGL(lz_finish_kernel, dim3(1), dim3(256), 0, st, partials, nb, 3, pass, scal);
  return hipGetLastError();
}

// First Gram-Schmidt pass straight on w = H q_k against an fp32 basis that holds q_0 .. q_k
// (nq = k + 1 rows): the coefficients of rows k and k - 1 are alpha_k and (up to rounding)
// beta_{k-1}, so the pass subsumes the three-term subtraction, which saves its two passes over the
// vectors.  Leaves alpha_k, ||r|| and the redo flag in scal as the three-term kernels followed by
// lz_reorth_pass(pass 0) do.  c: nq + 1 doubles, partials: (nq + 1) * LZ_NBLK doubles.
hipError_t lz_gs_first_pass(const float* Q, const bf16* copies, int64_t ldq, float* r, int64_t n, int nq, double* scal,
                            double* c, double* partials, hipStream_t st) {
  if (nq <= 0) return hipErrorInvalidValue;
  const int64_t nslices = (n + LZ_SLICE - 1) / LZ_SLICE;
  const int nb = (int)std::max<int64_t>(1, std::min<int64_t>(nslices, LZ_NBLK));
  const size_t sh1 = (size_t)4 * (nq + 1) * sizeof(double);
  hipLaunchKernelGGL((lz_qtr_kernel<float, true>), dim3(nb), dim3(256), sh1, st, Q, ldq, r, n, nq, nslices, scal, 0, partials);
  hipLaunchKernelGGL(lz_qtr_finish_kernel, dim3(nq + 1), dim3(256), 0, st, partials, nb, scal, 0, c);
  hipLaunchKernelGGL(lz_direct_scal_kernel, dim3(1), dim3(64), 0, st, c, nq, scal);
  launch_sub_f32(Q, copies, ldq, r, n, nq, nslices, nb, c, scal, 0, partials, st);
  hipLaunchKernelGGL(lz_finish_kernel, dim3(1), dim3(256), 0, st, partials, nb, 3, 0, scal);
  return hipGetLastError();
}

// The same with a bf16 basis: its rows k and k - 1 are rounded copies, so the pass takes q_k and
// q_{k-1} from the fp32 working vectors instead (alpha_k must come from the unrounded q_k) and the
// rounded rows 0 .. k-2 from the basis.  qkm1 is ignored for k = 0.
hipError_t lz_gs_first_pass_bf16(const bf16* Q, int64_t ldq, const float* qkm1, const float* qk, float* r, int64_t n, int k,
                                 double* scal, double* c, double* partials, hipStream_t st) {
  if (k < 0 || !qk || (k > 0 && !qkm1)) return hipErrorInvalidValue;
  const int64_t nslices = (n + LZ_SLICE - 1) / LZ_SLICE;
  const int nb = (int)std::max<int64_t>(1, std::min<int64_t>(nslices, LZ_NBLK));
  const int nqb = std::max(0, k - 1);  // rows taken from the basis
  const float* x0 = k > 0 ? qkm1 : qk;
  const float* x1 = k > 0 ? qk : nullptr;
  const size_t sh1 = (size_t)4 * (k + 2) * sizeof(double), sh2 = (size_t)(k + 1) * sizeof(float);
  hipLaunchKernelGGL((lz_qtr_kernel<bf16, true, true>), dim3(nb), dim3(256), sh1, st, Q, ldq, r, n, nqb, nslices, scal, 0, partials, x0, x1);
  hipLaunchKernelGGL(lz_qtr_finish_kernel, dim3(k + 2), dim3(256), 0, st, partials, nb, scal, 0, c);
  hipLaunchKernelGGL(lz_direct_scal_kernel, dim3(1), dim3(64), 0, st, c, k + 1, scal);
  hipLaunchKernelGGL((lz_sub_qc_kernel<bf16, true>), dim3(nb), dim3(256), sh2, st, Q, ldq, r, n, nqb, nslices, c, scal, 0, partials, x0, x1);
  hipLaunchKernelGGL(lz_finish_kernel, dim3(1), dim3(256), 0, st, partials, nb, 3, 0, scal);
  return hipGetLastError();
}

hipError_t lz_widen(const void* src, int is_bf16, float* dst, int64_t n, hipStream_t st) {
  const int nb = (int)std::max<int64_t>(1, std::min<int64_t>((n + 255) / 256, 8192));
  if (is_bf16) hipLaunchKernelGGL(lz_widen_kernel<bf16>, dim3(nb), dim3(256), 0, st, (const bf16*)src, dst, n);
  else hipLaunchKernelGGL(lz_widen_kernel<float>, dim3(nb), dim3(256), 0, st, (const float*)src, dst, n);
  return hipGetLastError();
}

}  // namespace hf
