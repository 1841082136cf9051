// Row-wise and pointwise operators of the Hessian-vector product, each in the
// two fused forms the forward-over-reverse evaluation of Algorithm 1 needs:
//   *_fwd : y and its tangent y_t (directional derivative along v)
//   *_bwd : the adjoint dx and its tangent dx_t, plus the H v block of the
//           operator's own parameters.
// For y = f(a):  y_t = f'(a) a_t;  da = f'(a) dy;  da_t = f'(a) dy_t + f''(a) a_t dy.
// All statistics and accumulations are fp32; AT is the storage type of
// activations that feed matrix products (float, or bf16 in bf16 mode).
#include "hf_internal.h"

#include <initializer_list>

namespace hf {

// ---------------------------------------------------------------- helpers ----

template <typename T>
__device__ __forceinline__ float ldf(const T* p, int64_t i) { return (float)p[i]; }
template <typename T>
__device__ __forceinline__ void stf(T* p, int64_t i, float v) { p[i] = (T)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Sum of N values per thread over a 256-thread block; result in every thread.
template <int N>
__device__ __forceinline__ void block_sum(float (&v)[N], float* red /* [4*N] */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = wave_sum(v[i]);
  __syncthreads();
  if (lane == 0)
#pragma unroll
    for (int i = 0; i < N; ++i) red[wave * N + i] = v[i];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = red[i] + red[N + i] + red[2 * N + i] + red[3 * N + i];
}

__device__ __forceinline__ float block_max(float v, float* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_max(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// 8 consecutive elements per thread: one 16 B access of bf16, two of fp32.
__device__ __forceinline__ void ld8(const float* p, int64_t i8, float (&o)[8]) {
  const float4 a = ((const float4*)p)[2 * i8], b = ((const float4*)p)[2 * i8 + 1];
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void ld8(const bf16* p, int64_t i8, float (&o)[8]) {
  const uint4 u = ((const uint4*)p)[i8];
  o[0] = __uint_as_float(u.x << 16); o[1] = __uint_as_float(u.x & 0xffff0000u);
  o[2] = __uint_as_float(u.y << 16); o[3] = __uint_as_float(u.y & 0xffff0000u);
  o[4] = __uint_as_float(u.z << 16); o[5] = __uint_as_float(u.z & 0xffff0000u);
  o[6] = __uint_as_float(u.w << 16); o[7] = __uint_as_float(u.w & 0xffff0000u);
}
__device__ __forceinline__ void st8(float* p, int64_t i8, const float (&v)[8]) {
  ((float4*)p)[2 * i8] = make_float4(v[0], v[1], v[2], v[3]);
  ((float4*)p)[2 * i8 + 1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void st8(bf16* p, int64_t i8, const float (&v)[8]) {
  bf16 o[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) o[q] = (bf16)v[q];
  ((uint4*)p)[i8] = *(const uint4*)o;
}
static inline bool all_aligned16(std::initializer_list<const void*> ps) {
  for (const void* x : ps) if (x && ((uintptr_t)x & 15)) return false;
  return true;
}

// ------------------------------------------------- attention row statistics ----
// Row i of a causal score matrix is covered by the parts 0 .. i/64 (64 columns each).
__global__ void attn_combine_kernel(int backward, const float* __restrict__ part, int NP, int M, int64_t rows,
                                    float* __restrict__ rstat) {
  const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= rows) return;
  const int np = (int)(row % M) / 64 + 1;
  const float* pr = part + row * NP * 3;
  if (backward) {
    float d = 0.f, dt = 0.f;
    for (int q = 0; q < np; ++q) { d += pr[q * 3]; dt += pr[q * 3 + 1]; }
    rstat[row * 3] = d; rstat[row * 3 + 1] = dt; rstat[row * 3 + 2] = 0.f;
    return;
  }
  float m = -INFINITY;
  for (int q = 0; q < np; ++q) m = fmaxf(m, pr[q * 3]);
  float l = 0.f, rr = 0.f;
  for (int q = 0; q < np; ++q) {
    const float w = __expf(pr[q * 3] - m);  // a part without a valid column has max -inf, weight 0
    l += pr[q * 3 + 1] * w;
    rr += pr[q * 3 + 2] * w;
  }
  const float inv = 1.f / l;
  rstat[row * 3] = m; rstat[row * 3 + 1] = inv; rstat[row * 3 + 2] = rr * inv;
}
hipError_t launch_attn_combine(int backward, const float* part, int NP, int M, int64_t rows, float* rstat, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)cdiv(rows, 256)), dim3(256), 0, st, backward, part, NP, M, rows, rstat);
  return hipGetLastError();
}

// delta = <dO, O>, delta_t = <dO_t, O> + <dO, O_t> per (token, head): the row sums sum_j P dP and
// sum_j (P_t dP + P dP_t) of the softmax adjoint, obtained without forming dP (O = P V, so
// sum_j P_ij (dO_i . V_j) = dO_i . O_i).  Operands are bf16 [T, D]; O takes its low-order half.
// One wavefront per token, 8 columns per lane; a head is dh / 8 adjacent lanes (a power of two).
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16* __restrict__ dO, const bf16* __restrict__ dO_t,
                                                         const bf16* __restrict__ O, const bf16* __restrict__ O_lo,
                                                         const bf16* __restrict__ O_t, int T, int S, int H, int dh,
                                                         float* __restrict__ rstat) {
  const int lane = threadIdx.x & 63;
  const int tok = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= T) return;
  const int D = H * dh, lph = dh >> 3;  // lanes per head
  const int b = tok / S, sq = tok % S;
  for (int c0 = 0; c0 < D; c0 += 512) {
    const int c = c0 + lane * 8;
    float d = 0.f, dt = 0.f;
    if (c < D) {
      float a[8], at[8], o[8], ol[8], ot[8];
      const int64_t i8 = ((int64_t)tok * D + c) >> 3;
      ld8(dO, i8, a); ld8(dO_t, i8, at); ld8(O, i8, o); ld8(O_t, i8, ot);
      if (O_lo) ld8(O_lo, i8, ol);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float of = O_lo ? o[q] + ol[q] : o[q];
        d += a[q] * of;
        dt += at[q] * of + a[q] * ot[q];
      }
    }
    for (int m = 1; m < lph; m <<= 1) { d += __shfl_xor(d, m, 64); dt += __shfl_xor(dt, m, 64); }
    if (c < D && (lane & (lph - 1)) == 0) {
      const int h = c / dh;
      float* dst = rstat + (((int64_t)b * H + h) * S + sq) * 3;
      dst[0] = d; dst[1] = dt; dst[2] = 0.f;
    }
  }
}
hipError_t launch_attn_delta(const void* dO, const void* dO_t, const void* O, const void* O_lo, const void* O_t, int T, int S,
                             int H, int dh, float* rstat, hipStream_t st) {
  const int lph = dh / 8;
  if (dh % 8 || (lph & (lph - 1)) || lph > 64 || (H * dh) % 8) return hipErrorNotSupported;
  if (!all_aligned16({dO, dO_t, O, O_lo, O_t})) return hipErrorNotSupported;
  hipLaunchKernelGGL(attn_delta_kernel, dim3((T + 3) / 4), dim3(256), 0, st, (const bf16*)dO, (const bf16*)dO_t, (const bf16*)O,
                     (const bf16*)O_lo, (const bf16*)O_t, T, S, H, dh, rstat);
  return hipGetLastError();
}

// ------------------------------------------------------------ fill / cast ----

__global__ void fill_f32_kernel(float* p, int64_t n, float val) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = val;
}
hipError_t launch_fill_f32(float* p, int64_t n, float val, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const int blocks = (int)std::min<int64_t>(cdiv(n, 256), 4096);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks), dim3(256), 0, st, p, n, val);
  return hipGetLastError();
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, bf16* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) {
      const float4 v = *(const float4*)(src + i);
      bf16 o[4] = {(bf16)v.x, (bf16)v.y, (bf16)v.z, (bf16)v.w};
      *(uint2*)(dst + i) = *(const uint2*)o;
    } else {
      for (int64_t j = i; j < n; ++j) dst[j] = (bf16)src[j];
    }
  }
}
hipError_t launch_f32_to_bf16(const float* src, bf16* dst, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const int blocks = (int)std::min<int64_t>(cdiv(n, 1024), 8192);
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(blocks), dim3(256), 0, st, src, dst, n);
  return hipGetLastError();
}

static inline int ew_blocks(int64_t n) { return (int)std::min<int64_t>(cdiv(n, 256), 16384); }
__global__ void cast_pair_vec_kernel(const float* a, const float* b, bf16* oa, bf16* ob, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
    float x[8], y[8];
    ld8(a, i, x); ld8(b, i, y);
    st8(oa, i, x); st8(ob, i, y);
  }
}
template <typename AT>
__global__ void cast_pair_kernel(const float* a, const float* b, AT* oa, AT* ob, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    oa[i] = (AT)a[i];
    ob[i] = (AT)b[i];
  }
}
// Second half of a k-split dual-output product: C = sum of the partial sums + bias + Cadd, in
// the output format of the unsplit kernel (fp32, or bf16 with an optional low-order half), for
// both results in one launch (blockIdx.y selects the result).
// VEC: four consecutive columns per thread (N, ldc multiples of 4, 16-byte aligned rows).
template <bool VEC>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(SplitKOut o0, SplitKOut o1, int splits, int M, int N, int64_t ldc,
                                                            int out_bf16) {
  const SplitKOut o = blockIdx.y ? o1 : o0;
  constexpr int W = VEC ? 4 : 1;
  const int64_t mn = (int64_t)M * N, nq = mn / W;
  const int ncol = N / W;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nq; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t m = i / ncol;
    const int n = (int)(i - m * ncol) * W;
    float v[W];
#pragma unroll
    for (int q = 0; q < W; ++q) v[q] = 0.f;
    for (int k = 0; k < splits; ++k) {
      const float* src = o.part + k * mn + m * N + n;
      if (VEC) {
        const float4 x = *(const float4*)src;
        v[0] += x.x; v[1 % W] += x.y; v[2 % W] += x.z; v[3 % W] += x.w;
      } else {
        v[0] += src[0];
      }
    }
#pragma unroll
    for (int q = 0; q < W; ++q) {
      if (o.bias_bf16) v[q] += (float)o.bias_bf16[n + q];
      if (o.bias_f32) v[q] += o.bias_f32[n + q];
    }
    const int64_t ci = m * ldc + n;
    if (o.Cadd) {
#pragma unroll
      for (int q = 0; q < W; ++q) v[q] += o.Cadd[ci + q];
    }
    if (out_bf16) {
#pragma unroll
      for (int q = 0; q < W; ++q) {
        const bf16 h = (bf16)v[q];
        ((bf16*)o.C)[ci + q] = h;
        if (o.C_lo) ((bf16*)o.C_lo)[ci + q] = (bf16)(v[q] - (float)h);
      }
    } else {
      if (VEC) *(float4*)((float*)o.C + ci) = make_float4(v[0], v[1 % W], v[2 % W], v[3 % W]);
      else ((float*)o.C)[ci] = v[0];
    }
  }
}
hipError_t launch_splitk_reduce(const SplitKOut& o0, const SplitKOut& o1, int splits, int M, int N, int64_t ldc, int out_bf16,
                                hipStream_t st) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (!o0.part || !o0.C || !o1.part || !o1.C || splits < 1) return hipErrorInvalidValue;
  const uintptr_t al = (uintptr_t)o0.part | (uintptr_t)o0.C | (uintptr_t)o0.Cadd | (uintptr_t)o1.part | (uintptr_t)o1.C |
                       (uintptr_t)o1.Cadd;
  const bool vec = N % 4 == 0 && ldc % 4 == 0 && (al & 15) == 0;
  const int64_t nq = (int64_t)M * N / (vec ? 4 : 1);
  dim3 grid((unsigned)ew_blocks(nq), 2);
  if (vec) hipLaunchKernelGGL(splitk_reduce_kernel<true>, grid, dim3(256), 0, st, o0, o1, splits, M, N, ldc, out_bf16);
  else hipLaunchKernelGGL(splitk_reduce_kernel<false>, grid, dim3(256), 0, st, o0, o1, splits, M, N, ldc, out_bf16);
  return hipGetLastError();
}

hipError_t launch_cast_pair(int bf, const float* a, const float* b, void* oa, void* ob, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (bf && n % 8 == 0 && all_aligned16({a, b, oa, ob})) {
    hipLaunchKernelGGL(cast_pair_vec_kernel, dim3(ew_blocks(n / 8)), dim3(256), 0, st, a, b, (bf16*)oa, (bf16*)ob, n / 8);
    return hipGetLastError();
  }
  const int blocks = (int)std::min<int64_t>(cdiv(n, 256), 8192);
  if (bf) hipLaunchKernelGGL(cast_pair_kernel<bf16>, dim3(blocks), dim3(256), 0, st, a, b, (bf16*)oa, (bf16*)ob, n);
  else hipLaunchKernelGGL(cast_pair_kernel<float>, dim3(blocks), dim3(256), 0, st, a, b, (float*)oa, (float*)ob, n);
  return hipGetLastError();
}

// -------------------------------------------------------------- embedding ----

template <typename PT>
__global__ void embed_fwd_kernel(const PT* wte, const PT* wpe, const float* wte_t, const float* wpe_t,
                                 const int32_t* tok, int S, int d, int vocab, float* x, float* x_t, int* err_flag) {
  const int t = blockIdx.x;
  int id = tok[t];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0) atomicOr(err_flag, 1);
    id = 0;
  }
  const int pos = t % S;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    float v = ldf(wte, (int64_t)id * d + c), vt = wte_t[(int64_t)id * d + c];
    if (wpe) {
      v += ldf(wpe, (int64_t)pos * d + c);
      vt += wpe_t[(int64_t)pos * d + c];
    }
    x[(int64_t)t * d + c] = v;
    x_t[(int64_t)t * d + c] = vt;
  }
}
hipError_t launch_embed_fwd(int bf, const void* wte, const void* wpe, const float* wte_t, const float* wpe_t,
                            const int32_t* tok, int T, int S, int d, int vocab, float* x, float* x_t, int* err_flag,
                            hipStream_t st) {
  if (bf) hipLaunchKernelGGL(embed_fwd_kernel<bf16>, dim3(T), dim3(256), 0, st, (const bf16*)wte, (const bf16*)wpe, wte_t, wpe_t, tok, S, d, vocab, x, x_t, err_flag);
  else hipLaunchKernelGGL(embed_fwd_kernel<float>, dim3(T), dim3(256), 0, st, (const float*)wte, (const float*)wpe, wte_t, wpe_t, tok, S, d, vocab, x, x_t, err_flag);
  return hipGetLastError();
}

__global__ void embed_bwd_kernel(const float* dx_t, const int32_t* tok, int S, int d, int vocab, float* out_wte, float* out_wpe) {
  const int t = blockIdx.x;
  int id = tok[t];
  if (id < 0 || id >= vocab) return;
  const int pos = t % S;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = dx_t[(int64_t)t * d + c];
    atomicAdd(out_wte + (int64_t)id * d + c, v);
    if (out_wpe) atomicAdd(out_wpe + (int64_t)pos * d + c, v);
  }
}
hipError_t launch_embed_bwd(const float* dx_t, const int32_t* tok, int T, int S, int d, int vocab, float* out_wte,
                            float* out_wpe, hipStream_t st) {
  hipLaunchKernelGGL(embed_bwd_kernel, dim3(T), dim3(256), 0, st, dx_t, tok, S, d, vocab, out_wte, out_wpe);
  return hipGetLastError();
}

// ------------------------------------------------------------------ norms ----
// LayerNorm: xh = (x - mu) rstd, y = gam xh + bet.  With s_t = mean(xh x_t):
//   xh_t = (x_t - mean(x_t) - xh s_t) rstd,  y_t = gam_t xh + gam xh_t + bet_t.
// RMSNorm is the same with mu = mean(x_t) = 0 and rstd = 1/sqrt(mean(x^2)+eps).
// stats row: [mu, rstd, mean(x_t), s_t].

template <typename PT, typename AT, bool RMS>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const float* __restrict__ x, const float* __restrict__ x_t,
                                                       const PT* gam, const PT* bet, const float* gam_t,
                                                       const float* bet_t, int d, float eps, AT* y, AT* y_t,
                                                       AT* y_lo, float* stats) {
  __shared__ float red[16];
  const int64_t row = blockIdx.x;
  const float* xr = x + row * d;
  const float* xtr = x_t + row * d;
  const float inv_d = 1.f / (float)d;
  float mu = 0.f, mxt = 0.f;
  if (!RMS) {
    float s[2] = {0.f, 0.f};
    for (int c = threadIdx.x; c < d; c += 256) { s[0] += xr[c]; s[1] += xtr[c]; }
    block_sum<2>(s, red);
    mu = s[0] * inv_d;
    mxt = s[1] * inv_d;
  }
  float s2[2] = {0.f, 0.f};
  for (int c = threadIdx.x; c < d; c += 256) {
    const float xc = xr[c] - mu;
    s2[0] += xc * xc;
    s2[1] += xc * xtr[c];
  }
  block_sum<2>(s2, red);
  const float rstd = rsqrtf(s2[0] * inv_d + eps);
  const float st = s2[1] * inv_d * rstd;  // mean(xh * x_t)
  for (int c = threadIdx.x; c < d; c += 256) {
    const float xh = (xr[c] - mu) * rstd;
    const float xht = (xtr[c] - mxt - xh * st) * rstd;
    const float g = ldf(gam, c);
    float yv = g * xh, yt = gam_t[c] * xh + g * xht;
    if (!RMS) { yv += ldf(bet, c); yt += bet_t[c]; }
    stf(y, row * d + c, yv);
    stf(y_t, row * d + c, yt);
    // optional low-order part: y = (AT)y + y_lo to about twice the mantissa
    if (y_lo) stf(y_lo, row * d + c, yv - (float)(AT)yv);
  }
  if (threadIdx.x == 0) {
    float4 o = make_float4(mu, rstd, mxt, st);
    *(float4*)(stats + row * 4) = o;
  }
}

// Same, one block per row with the row held in registers (NCH chunks of 4 columns per thread,
// d <= 1024 NCH): x and x_t are read once, 16 bytes at a time, and the bf16 results leave 8 bytes
// at a time.  Needs d % 4 == 0 and 16-byte (fp32) / 8-byte (bf16) aligned rows.
__device__ __forceinline__ float4 ldq(const float* p, int64_t i4) { return ((const float4*)p)[i4]; }
__device__ __forceinline__ float4 ldq(const bf16* p, int64_t i4) {
  const uint2 u = ((const uint2*)p)[i4];
  const bf16* h = (const bf16*)&u;
  return make_float4((float)h[0], (float)h[1], (float)h[2], (float)h[3]);
}
__device__ __forceinline__ void stq(float* p, int64_t i4, float4 v) { ((float4*)p)[i4] = v; }
__device__ __forceinline__ void stq(bf16* p, int64_t i4, float4 v) {
  const bf16 h[4] = {(bf16)v.x, (bf16)v.y, (bf16)v.z, (bf16)v.w};
  ((uint2*)p)[i4] = *(const uint2*)h;
}
__device__ __forceinline__ float4 lo_of(float4 v, float*) { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ float4 lo_of(float4 v, bf16*) {
  return make_float4(v.x - (float)(bf16)v.x, v.y - (float)(bf16)v.y, v.z - (float)(bf16)v.z, v.w - (float)(bf16)v.w);
}

template <typename PT, typename AT, bool RMS, int NCH>
__global__ __launch_bounds__(256) void norm_fwd_vec_kernel(const float* __restrict__ x, const float* __restrict__ x_t,
                                                           const PT* __restrict__ gam, const PT* __restrict__ bet,
                                                           const float* __restrict__ gam_t, const float* __restrict__ bet_t,
                                                           int d, float eps, AT* __restrict__ y, AT* __restrict__ y_t,
                                                           AT* __restrict__ y_lo, float* __restrict__ stats) {
  __shared__ float red[16];
  const int64_t row = blockIdx.x;
  const int d4 = d >> 2;
  const int64_t base4 = row * d4;
  const float inv_d = 1.f / (float)d;
  float4 xv[NCH], tv[NCH];
  float s[2] = {0.f, 0.f};
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c4 = j * 256 + threadIdx.x;
    xv[j] = make_float4(0.f, 0.f, 0.f, 0.f); tv[j] = xv[j];
    if (c4 < d4) {
      xv[j] = ldq(x, base4 + c4); tv[j] = ldq(x_t, base4 + c4);
      s[0] += (xv[j].x + xv[j].y) + (xv[j].z + xv[j].w);
      s[1] += (tv[j].x + tv[j].y) + (tv[j].z + tv[j].w);
    }
  }
  float mu = 0.f, mxt = 0.f;
  if (!RMS) {
    block_sum<2>(s, red);
    mu = s[0] * inv_d;
    mxt = s[1] * inv_d;
  }
  float s2[2] = {0.f, 0.f};
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c4 = j * 256 + threadIdx.x;
    if (c4 < d4) {
      xv[j].x -= mu; xv[j].y -= mu; xv[j].z -= mu; xv[j].w -= mu;
      s2[0] += (xv[j].x * xv[j].x + xv[j].y * xv[j].y) + (xv[j].z * xv[j].z + xv[j].w * xv[j].w);
      s2[1] += (xv[j].x * tv[j].x + xv[j].y * tv[j].y) + (xv[j].z * tv[j].z + xv[j].w * tv[j].w);
    }
  }
  block_sum<2>(s2, red);
  const float rstd = rsqrtf(s2[0] * inv_d + eps);
  const float st = s2[1] * inv_d * rstd;  // mean(xh * x_t)
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c4 = j * 256 + threadIdx.x;
    if (c4 < d4) {
      const float4 g = ldq(gam, c4), gt = ldq(gam_t, c4);
      float4 yv, yt;
#define HF_NFV(q)                                            \
  {                                                          \
    const float xh = xv[j].q * rstd;                         \
    const float xht = (tv[j].q - mxt - xh * st) * rstd;      \
    yv.q = g.q * xh;                                         \
    yt.q = gt.q * xh + g.q * xht;                            \
  }
      HF_NFV(x) HF_NFV(y) HF_NFV(z) HF_NFV(w)
#undef HF_NFV
      if (!RMS) {
        const float4 b = ldq(bet, c4), bt = ldq(bet_t, c4);
        yv.x += b.x; yv.y += b.y; yv.z += b.z; yv.w += b.w;
        yt.x += bt.x; yt.y += bt.y; yt.z += bt.z; yt.w += bt.w;
      }
      stq(y, base4 + c4, yv);
      stq(y_t, base4 + c4, yt);
      if (y_lo) stq(y_lo, base4 + c4, lo_of(yv, y_lo));
    }
  }
  if (threadIdx.x == 0) *(float4*)(stats + row * 4) = make_float4(mu, rstd, mxt, st);
}

hipError_t launch_norm_fwd(int bf, int rms, const float* x, const float* x_t, const void* gam, const void* bet,
                           const float* gam_t, const float* bet_t, int T, int d, float eps, void* y, void* y_t,
                           void* y_lo, float* stats, hipStream_t st) {
  {
    const uintptr_t a16 = (uintptr_t)x | (uintptr_t)x_t | (uintptr_t)gam_t | (uintptr_t)bet_t | (uintptr_t)stats;
    const uintptr_t ap = (uintptr_t)gam | (uintptr_t)bet | (uintptr_t)y | (uintptr_t)y_t | (uintptr_t)y_lo;
    if (d % 4 == 0 && d <= 8192 && (a16 & 15) == 0 && (ap & (bf ? 7 : 15)) == 0) {
      const int nch = (d / 4 + 255) / 256;
#define HF_NFV2(PT, AT, R, N) hipLaunchKernelGGL((norm_fwd_vec_kernel<PT, AT, R, N>), dim3(T), dim3(256), 0, st, x, x_t, (const PT*)gam, (const PT*)bet, gam_t, bet_t, d, eps, (AT*)y, (AT*)y_t, (AT*)y_lo, stats)
#define HF_NFV1(PT, AT, R) { if (nch <= 1) HF_NFV2(PT, AT, R, 1); else if (nch <= 2) HF_NFV2(PT, AT, R, 2); else if (nch <= 4) HF_NFV2(PT, AT, R, 4); else HF_NFV2(PT, AT, R, 8); }
      if (bf) { if (rms) HF_NFV1(bf16, bf16, true) else HF_NFV1(bf16, bf16, false) }
      else { if (rms) HF_NFV1(float, float, true) else HF_NFV1(float, float, false) }
#undef HF_NFV1
#undef HF_NFV2
      return hipGetLastError();
    }
  }
#define HF_NF(PT, AT, R) hipLaunchKernelGGL((norm_fwd_kernel<PT, AT, R>), dim3(T), dim3(256), 0, st, x, x_t, (const PT*)gam, (const PT*)bet, gam_t, bet_t, d, eps, (AT*)y, (AT*)y_t, (AT*)y_lo, stats)
  if (bf) { if (rms) HF_NF(bf16, bf16, true); else HF_NF(bf16, bf16, false); }
  else { if (rms) HF_NF(float, float, true); else HF_NF(float, float, false); }
#undef HF_NF
  return hipGetLastError();
}

// Adjoint of the norm with its tangent.  g = gam dy, g_t = gam_t dy + gam dy_t,
//   dx   = (g - mean(g) - xh mean(g xh)) rstd
//   dx_t = (g_t - mean(g_t) - xh_t mean(g xh) - xh mean(g_t xh + g xh_t)) rstd - dx s_t rstd
//   (Hv)_gam = sum_rows (dy_t xh + dy xh_t),  (Hv)_bet = sum_rows dy_t.
// Each block walks `rows_per_block` rows and keeps its column partial sums in
// registers, so the atomics on hv_gam / hv_bet are one per column per block.
constexpr int NORM_MAXC = 32;  // columns per thread: d <= 8192

template <typename PT, bool RMS>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const float* __restrict__ dy, const float* __restrict__ dy_t,
                                                       const float* __restrict__ x, const float* __restrict__ x_t,
                                                       const float* __restrict__ stats, const PT* gam,
                                                       const float* gam_t, int T, int d, int rows_per_block,
                                                       int accumulate, float* dx, float* dx_t, float* hv_gam,
                                                       float* hv_bet, bf16* dxb, bf16* dxb_t) {
  __shared__ float red[16];
  float pg[NORM_MAXC], pb[NORM_MAXC];
#pragma unroll
  for (int i = 0; i < NORM_MAXC; ++i) { pg[i] = 0.f; pb[i] = 0.f; }
  const float inv_d = 1.f / (float)d;
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(T, r0 + rows_per_block);
  for (int row = r0; row < r1; ++row) {
    const int64_t base = (int64_t)row * d;
    const float4 s = *(const float4*)(stats + (int64_t)row * 4);
    const float mu = s.x, rstd = s.y, mxt = s.z, st = s.w;
    float m[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = threadIdx.x; c < d; c += 256) {
      const float xh = (x[base + c] - mu) * rstd;
      const float xht = (x_t[base + c] - mxt - xh * st) * rstd;
      const float gm = ldf(gam, c);
      const float g = gm * dy[base + c];
      const float gt = gam_t[c] * dy[base + c] + gm * dy_t[base + c];
      m[0] += g; m[1] += g * xh; m[2] += gt; m[3] += gt * xh + g * xht;
    }
    block_sum<4>(m, red);
    float m1 = m[0] * inv_d, m2 = m[1] * inv_d, m1t = m[2] * inv_d, m2t = m[3] * inv_d;
    if (RMS) { m1 = 0.f; m1t = 0.f; }
    int ci = 0;
    for (int c = threadIdx.x; c < d; c += 256, ++ci) {
      const float xh = (x[base + c] - mu) * rstd;
      const float xht = (x_t[base + c] - mxt - xh * st) * rstd;
      const float gm = ldf(gam, c);
      const float dyv = dy[base + c], dytv = dy_t[base + c];
      const float g = gm * dyv;
      const float gt = gam_t[c] * dyv + gm * dytv;
      const float dxv = (g - m1 - xh * m2) * rstd;
      const float dxt = (gt - m1t - xht * m2 - xh * m2t) * rstd - dxv * st * rstd;
      float ov = dxv, ovt = dxt;
      if (accumulate) { ov += dx[base + c]; ovt += dx_t[base + c]; }
      dx[base + c] = ov; dx_t[base + c] = ovt;
      if (dxb) { dxb[base + c] = (bf16)ov; dxb_t[base + c] = (bf16)ovt; }
      pg[ci] += dytv * xh + dyv * xht;
      pb[ci] += dytv;
    }
  }
  int ci = 0;
  for (int c = threadIdx.x; c < d; c += 256, ++ci) {
    atomicAdd(hv_gam + c, pg[ci]);
    if (!RMS) atomicAdd(hv_bet + c, pb[ci]);
  }
}

// Vector variant for d % 4 == 0: each thread owns NCH groups of 4 consecutive
// columns (group j of thread t covers columns 4 (256 j + t) .. +3), keeps the
// row's four inputs in registers between the reduction and the write, and
// moves 16 bytes per access.
__device__ __forceinline__ float4 ld4(const float* p, int64_t i4) { return ((const float4*)p)[i4]; }
__device__ __forceinline__ float4 ld4(const bf16* p, int64_t i4) {
  const uint2 u = ((const uint2*)p)[i4];
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xffff0000u));
}

template <typename PT, bool RMS, int NCH>
__global__ __launch_bounds__(256) void norm_bwd_vec_kernel(const float* __restrict__ dy, const float* __restrict__ dy_t,
                                                           const float* __restrict__ x, const float* __restrict__ x_t,
                                                           const float* __restrict__ stats, const PT* gam,
                                                           const float* gam_t, int T, int d, int rows_per_block,
                                                           int accumulate, float* dx, float* dx_t, float* hv_gam,
                                                           float* hv_bet, float* part, bf16* dxb, bf16* dxb_t, float* hv_out) {
  __shared__ float red[16];
  const int d4 = d >> 2;
  float4 pg[NCH], pb[NCH], po[NCH], gm[NCH], gmt[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    pg[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    pb[j] = pg[j];
    po[j] = pg[j];
    const int c4 = j * 256 + threadIdx.x;
    gm[j] = c4 < d4 ? ld4(gam, c4) : pg[j];
    gmt[j] = c4 < d4 ? ld4(gam_t, c4) : pg[j];
  }
  const float inv_d = 1.f / (float)d;
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(T, r0 + rows_per_block);
  for (int row = r0; row < r1; ++row) {
    const int64_t base4 = (int64_t)row * d4;
    const float4 s = *(const float4*)(stats + (int64_t)row * 4);
    const float mu = s.x, rstd = s.y, mxt = s.z, st = s.w;
    float4 xh[NCH], xht[NCH], dv[NCH], dtv[NCH];
    float m[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int c4 = j * 256 + threadIdx.x;
      if (c4 < d4) {
        const float4 xv = ld4(x, base4 + c4), xtv = ld4(x_t, base4 + c4);
        dv[j] = ld4(dy, base4 + c4);
        dtv[j] = ld4(dy_t, base4 + c4);
#define HF_NBV(q)                                                         \
  {                                                                       \
    const float h = (xv.q - mu) * rstd;                                   \
    const float ht = (xtv.q - mxt - h * st) * rstd;                       \
    xh[j].q = h; xht[j].q = ht;                                           \
    const float g = gm[j].q * dv[j].q;                                    \
    const float gt = gmt[j].q * dv[j].q + gm[j].q * dtv[j].q;             \
    m[0] += g; m[1] += g * h; m[2] += gt; m[3] += gt * h + g * ht;        \
  }
        HF_NBV(x) HF_NBV(y) HF_NBV(z) HF_NBV(w)
#undef HF_NBV
      }
    }
    block_sum<4>(m, red);
    float m1 = m[0] * inv_d, m2 = m[1] * inv_d, m1t = m[2] * inv_d, m2t = m[3] * inv_d;
    if (RMS) { m1 = 0.f; m1t = 0.f; }
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int c4 = j * 256 + threadIdx.x;
      if (c4 < d4) {
        float4 o, ot;
#define HF_NBV(q)                                                                                   \
  {                                                                                                 \
    const float g = gm[j].q * dv[j].q;                                                              \
    const float gt = gmt[j].q * dv[j].q + gm[j].q * dtv[j].q;                                       \
    o.q = (g - m1 - xh[j].q * m2) * rstd;                                                           \
    ot.q = (gt - m1t - xht[j].q * m2 - xh[j].q * m2t) * rstd - o.q * st * rstd;                     \
    pg[j].q += dtv[j].q * xh[j].q + dv[j].q * xht[j].q;                                             \
    pb[j].q += dtv[j].q;                                                                            \
  }
        HF_NBV(x) HF_NBV(y) HF_NBV(z) HF_NBV(w)
#undef HF_NBV
        if (accumulate) {
          const float4 a = ld4(dx, base4 + c4), b = ld4(dx_t, base4 + c4);
          o.x += a.x; o.y += a.y; o.z += a.z; o.w += a.w;
          ot.x += b.x; ot.y += b.y; ot.z += b.z; ot.w += b.w;
        }
        ((float4*)dx)[base4 + c4] = o;
        ((float4*)dx_t)[base4 + c4] = ot;
        po[j].x += ot.x; po[j].y += ot.y; po[j].z += ot.z; po[j].w += ot.w;
        if (dxb) {  // operand-type copies for the products that consume the adjoint next
          const bf16 h[4] = {(bf16)o.x, (bf16)o.y, (bf16)o.z, (bf16)o.w}, ht[4] = {(bf16)ot.x, (bf16)ot.y, (bf16)ot.z, (bf16)ot.w};
          ((uint2*)dxb)[base4 + c4] = *(const uint2*)h;
          ((uint2*)dxb_t)[base4 + c4] = *(const uint2*)ht;
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = 4 * (j * 256 + threadIdx.x);
    if (c < d) {
      if (part) {  // per-block partial sums, summed by norm_colsum_kernel
        *(float4*)(part + ((size_t)blockIdx.x * 3) * d + c) = pg[j];
        if (!RMS) *(float4*)(part + ((size_t)blockIdx.x * 3 + 1) * d + c) = pb[j];
        if (hv_out) *(float4*)(part + ((size_t)blockIdx.x * 3 + 2) * d + c) = po[j];
      } else {
        if (hv_out) {
          atomicAdd(hv_out + c, po[j].x); atomicAdd(hv_out + c + 1, po[j].y);
          atomicAdd(hv_out + c + 2, po[j].z); atomicAdd(hv_out + c + 3, po[j].w);
        }
        atomicAdd(hv_gam + c, pg[j].x); atomicAdd(hv_gam + c + 1, pg[j].y);
        atomicAdd(hv_gam + c + 2, pg[j].z); atomicAdd(hv_gam + c + 3, pg[j].w);
        if (!RMS) {
          atomicAdd(hv_bet + c, pb[j].x); atomicAdd(hv_bet + c + 1, pb[j].y);
          atomicAdd(hv_bet + c + 2, pb[j].z); atomicAdd(hv_bet + c + 3, pb[j].w);
        }
      }
    }
  }
}

// Narrow rows (d <= 1024): one wavefront per row, so a block has four rows in
// flight and the row reductions are wave shuffles without a block barrier.
// Lane l owns the groups of 4 columns 4 (64 j + l) .. +3, j < NJ.  The column
// sums of the four waves meet in LDS and leave as one atomic per column per block.
template <typename PT, bool RMS, int NJ>
__global__ __launch_bounds__(256) void norm_bwd_wave_kernel(const float* __restrict__ dy, const float* __restrict__ dy_t,
                                                            const float* __restrict__ x, const float* __restrict__ x_t,
                                                            const float* __restrict__ stats, const PT* gam,
                                                            const float* gam_t, int T, int d, int rows_per_block,
                                                            int accumulate, float* dx, float* dx_t, float* hv_gam,
                                                            float* hv_bet, float* part, bf16* dxb, bf16* dxb_t, float* hv_out) {
  extern __shared__ float colred[];  // [2 or 3][4][d]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d4 = d >> 2;
  float4 pg[NJ], pb[NJ], po[NJ], gm[NJ], gmt[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    pg[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    pb[j] = pg[j];
    po[j] = pg[j];
    const int c4 = j * 64 + lane;
    gm[j] = c4 < d4 ? ld4(gam, c4) : pg[j];
    gmt[j] = c4 < d4 ? ld4(gam_t, c4) : pg[j];
  }
  const float inv_d = 1.f / (float)d;
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(T, r0 + rows_per_block);
  for (int row = r0 + wave; row < r1; row += 4) {
    const int64_t base4 = (int64_t)row * d4;
    const float4 s = *(const float4*)(stats + (int64_t)row * 4);
    const float mu = s.x, rstd = s.y, mxt = s.z, st = s.w;
    float4 xh[NJ], xht[NJ], dv[NJ], dtv[NJ];
    float m0 = 0.f, m1s = 0.f, m2s = 0.f, m3s = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c4 = j * 64 + lane;
      if (c4 < d4) {
        const float4 xv = ld4(x, base4 + c4), xtv = ld4(x_t, base4 + c4);
        dv[j] = ld4(dy, base4 + c4);
        dtv[j] = ld4(dy_t, base4 + c4);
#define HF_NBW(q)                                                       \
  {                                                                     \
    const float h = (xv.q - mu) * rstd;                                 \
    const float ht = (xtv.q - mxt - h * st) * rstd;                     \
    xh[j].q = h; xht[j].q = ht;                                         \
    const float g = gm[j].q * dv[j].q;                                  \
    const float gt = gmt[j].q * dv[j].q + gm[j].q * dtv[j].q;           \
    m0 += g; m1s += g * h; m2s += gt; m3s += gt * h + g * ht;           \
  }
        HF_NBW(x) HF_NBW(y) HF_NBW(z) HF_NBW(w)
#undef HF_NBW
      }
    }
    m0 = wave_sum(m0); m1s = wave_sum(m1s); m2s = wave_sum(m2s); m3s = wave_sum(m3s);
    float m1 = m0 * inv_d, m2 = m1s * inv_d, m1t = m2s * inv_d, m2t = m3s * inv_d;
    if (RMS) { m1 = 0.f; m1t = 0.f; }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c4 = j * 64 + lane;
      if (c4 < d4) {
        float4 o, ot;
#define HF_NBW(q)                                                                               \
  {                                                                                             \
    const float g = gm[j].q * dv[j].q;                                                          \
    const float gt = gmt[j].q * dv[j].q + gm[j].q * dtv[j].q;                                   \
    o.q = (g - m1 - xh[j].q * m2) * rstd;                                                       \
    ot.q = (gt - m1t - xht[j].q * m2 - xh[j].q * m2t) * rstd - o.q * st * rstd;                 \
    pg[j].q += dtv[j].q * xh[j].q + dv[j].q * xht[j].q;                                         \
    pb[j].q += dtv[j].q;                                                                        \
  }
        HF_NBW(x) HF_NBW(y) HF_NBW(z) HF_NBW(w)
#undef HF_NBW
        if (accumulate) {
          const float4 a = ld4(dx, base4 + c4), b = ld4(dx_t, base4 + c4);
          o.x += a.x; o.y += a.y; o.z += a.z; o.w += a.w;
          ot.x += b.x; ot.y += b.y; ot.z += b.z; ot.w += b.w;
        }
        ((float4*)dx)[base4 + c4] = o;
        ((float4*)dx_t)[base4 + c4] = ot;
        po[j].x += ot.x; po[j].y += ot.y; po[j].z += ot.z; po[j].w += ot.w;
        if (dxb) {  // operand-type copies for the products that consume the adjoint next
          const bf16 h[4] = {(bf16)o.x, (bf16)o.y, (bf16)o.z, (bf16)o.w}, ht[4] = {(bf16)ot.x, (bf16)ot.y, (bf16)ot.z, (bf16)ot.w};
          ((uint2*)dxb)[base4 + c4] = *(const uint2*)h;
          ((uint2*)dxb_t)[base4 + c4] = *(const uint2*)ht;
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c4 = j * 64 + lane;
    if (c4 < d4) {
      ((float4*)(colred + (size_t)wave * d))[c4] = pg[j];
      ((float4*)(colred + (size_t)(4 + wave) * d))[c4] = pb[j];
      if (hv_out) ((float4*)(colred + (size_t)(8 + wave) * d))[c4] = po[j];
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += 256) {
    if (hv_out) atomicAdd(hv_out + c, (colred[8 * d + c] + colred[9 * d + c]) + (colred[10 * d + c] + colred[11 * d + c]));
    const float sg = (colred[c] + colred[d + c]) + (colred[2 * d + c] + colred[3 * d + c]);
    const float sb = (colred[4 * d + c] + colred[5 * d + c]) + (colred[6 * d + c] + colred[7 * d + c]);
    if (part) {
      part[((size_t)blockIdx.x * 3) * d + c] = sg;
      if (!RMS) part[((size_t)blockIdx.x * 3 + 1) * d + c] = sb;
    } else {
      atomicAdd(hv_gam + c, sg);
      if (!RMS) atomicAdd(hv_bet + c, sb);
    }
  }
}

// hv[c] += sum over blocks of part[block][which][c]: grid (d / 256, groups, 3);
// each block sums its share of the partial rows and adds once per column.
__global__ void norm_colsum_kernel(const float* __restrict__ part, int nblocks, int d, float* hv_gam, float* hv_bet, float* hv_out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  const int which = blockIdx.z;
  float* hv = which == 0 ? hv_gam : which == 1 ? hv_bet : hv_out;
  if (!hv) return;
  const int per = (nblocks + gridDim.y - 1) / gridDim.y;
  const int b0 = blockIdx.y * per, b1 = min(nblocks, b0 + per);
  float s = 0.f;
  for (int b = b0; b < b1; ++b) s += part[((size_t)b * 3 + which) * d + c];
  if (b1 > b0) atomicAdd(hv + c, s);
}

hipError_t launch_norm_bwd(int bf, int rms, const float* dy, const float* dy_t, const float* x, const float* x_t,
                           const float* stats, const void* gam, const float* gam_t, int T, int d, int accumulate,
                           float* dx, float* dx_t, float* hv_gam, float* hv_bet, float* part, hipStream_t st, void* dxb_v,
                           void* dxb_t_v, float* hv_out) {
  if (d > 256 * NORM_MAXC) return hipErrorInvalidValue;
  bf16* dxb = (bf16*)dxb_v;
  bf16* dxb_t = (bf16*)dxb_t_v;
  if ((dxb == nullptr) != (dxb_t == nullptr) || (((uintptr_t)dxb | (uintptr_t)dxb_t) & 7)) return hipErrorInvalidValue;
  // part (optional): room for NORM_PART_BLOCKS x 3 x d floats; the vector kernels then leave their
  // column sums there and a second kernel adds them up (the atomics otherwise cost more than the rows)
  // hv_out (optional): also hv_out[c] += sum over rows of the dx_t written here, i.e. the H v block of
  // the bias of the linear layer whose output adjoint this is.
  auto finish = [&](int blocks) {
    hipLaunchKernelGGL(norm_colsum_kernel, dim3((d + 255) / 256, 16, hv_out ? 3 : (rms ? 1 : 2)), dim3(256), 0, st, part, blocks, d, hv_gam,
                       rms ? nullptr : hv_bet, hv_out);
    return hipGetLastError();
  };
  const bool vec_ok = d % 4 == 0 && all_aligned16({dy, dy_t, x, x_t, dx, dx_t, gam_t}) && ((uintptr_t)gam & (bf ? 7 : 15)) == 0;
  if (vec_ok && d <= 1024 && T >= 64) {
    const int rpb = std::max(4, (T / 512 + 3) / 4 * 4);
    const int blocks = (T + rpb - 1) / rpb;
    const int nj = (d / 4 + 63) / 64;
    part = nullptr;  // narrow rows: the atomics are cheaper than a second launch
    const size_t lds = (size_t)(hv_out ? 12 : 8) * d * sizeof(float);
#define HF_NBW2(PT, R, N) hipLaunchKernelGGL((norm_bwd_wave_kernel<PT, R, N>), dim3(blocks), dim3(256), lds, st, dy, dy_t, x, x_t, stats, (const PT*)gam, gam_t, T, d, rpb, accumulate, dx, dx_t, hv_gam, hv_bet, part, dxb, dxb_t, hv_out)
#define HF_NBW1(PT, R) { if (nj <= 1) HF_NBW2(PT, R, 1); else if (nj <= 2) HF_NBW2(PT, R, 2); else if (nj <= 3) HF_NBW2(PT, R, 3); else HF_NBW2(PT, R, 4); }
    if (bf) { if (rms) HF_NBW1(bf16, true) else HF_NBW1(bf16, false) }
    else { if (rms) HF_NBW1(float, true) else HF_NBW1(float, false) }
#undef HF_NBW1
#undef HF_NBW2
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    return part ? finish(blocks) : hipSuccess;
  }
  if (vec_ok) {
    const int rpb = std::max(1, T / 512);  // the column atomics at the end bound the block count
    const int blocks = (T + rpb - 1) / rpb;
    const int nch = (d / 4 + 255) / 256;
    if (blocks > NORM_PART_BLOCKS) part = nullptr;
#define HF_NBV2(PT, R, N) hipLaunchKernelGGL((norm_bwd_vec_kernel<PT, R, N>), dim3(blocks), dim3(256), 0, st, dy, dy_t, x, x_t, stats, (const PT*)gam, gam_t, T, d, rpb, accumulate, dx, dx_t, hv_gam, hv_bet, part, dxb, dxb_t, hv_out)
#define HF_NBV1(PT, R) { if (nch <= 1) HF_NBV2(PT, R, 1); else if (nch <= 2) HF_NBV2(PT, R, 2); else if (nch <= 4) HF_NBV2(PT, R, 4); else HF_NBV2(PT, R, 8); }
    if (bf) { if (rms) HF_NBV1(bf16, true) else HF_NBV1(bf16, false) }
    else { if (rms) HF_NBV1(float, true) else HF_NBV1(float, false) }
#undef HF_NBV1
#undef HF_NBV2
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    return part ? finish(blocks) : hipSuccess;
  }
  const int rpb = std::max(1, T / 512);
  const int blocks = (T + rpb - 1) / rpb;
#define HF_NB(PT, R) hipLaunchKernelGGL((norm_bwd_kernel<PT, R>), dim3(blocks), dim3(256), 0, st, dy, dy_t, x, x_t, stats, (const PT*)gam, gam_t, T, d, rpb, accumulate, dx, dx_t, hv_gam, hv_bet, dxb, dxb_t)
  if (bf) { if (rms) HF_NB(bf16, true); else HF_NB(bf16, false); }
  else { if (rms) HF_NB(float, true); else HF_NB(float, false); }
#undef HF_NB
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  return hv_out ? launch_colsum(0, dx_t, T, d, d, hv_out, st) : hipSuccess;
}

// ------------------------------------------------------------ activations ----

__device__ __forceinline__ void act_derivs(int act, float a, float& f, float& f1, float& f2) {
  if (act == ACT_TANH) {
    const float t = tanhf(a);
    f = t; f1 = 1.f - t * t; f2 = -2.f * t * f1;
  } else if (act == ACT_GELU_TANH) {
    // f = a/2 (1 + t), t = tanh u, u = c (a + k a^3):  t' = (1 - t^2) u',
    // t'' = (1 - t^2)(u'' - 2 t u'^2),  f' = (1 + t)/2 + a t'/2,  f'' = t' + a t''/2
    const float c = 0.79788456080286536f, k = 0.044715f;
    const float t = tanhf(c * (a + k * a * a * a));
    const float u1 = c * (1.f + 3.f * k * a * a), u2 = 6.f * k * c * a;
    const float s = 1.f - t * t;
    const float t1 = s * u1, t2 = s * (u2 - 2.f * t * u1 * u1);
    f = 0.5f * a * (1.f + t); f1 = 0.5f * (1.f + t) + 0.5f * a * t1; f2 = t1 + 0.5f * a * t2;
  } else {  // erf GELU: f = a Phi(a), f' = Phi + a phi, f'' = phi (2 - a^2)
    const float Phi = 0.5f * (1.f + erff(a * 0.70710678118654752f));
    const float phi = 0.39894228040143268f * __expf(-0.5f * a * a);
    f = a * Phi; f1 = Phi + a * phi; f2 = phi * (2.f - a * a);
  }
}

// a_lo / y_lo (optional): low-order parts, a = a + a_lo on input and
// y_lo = y - round(y) on output, so the primal chain keeps ~16 mantissa bits.
template <typename AT>
__global__ void act_fwd_kernel(int act, const AT* a, const AT* a_t, const AT* a_lo, AT* y, AT* y_t, AT* y_lo, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    float f, f1, f2;
    float av = ldf(a, i);
    if (a_lo) av += ldf(a_lo, i);
    act_derivs(act, av, f, f1, f2);
    stf(y, i, f);
    stf(y_t, i, f1 * ldf(a_t, i));
    if (y_lo) stf(y_lo, i, f - (float)(AT)f);
  }
}
template <typename AT>
__global__ void act_bwd_kernel(int act, const AT* a, const AT* a_t, const AT* dy, const AT* dy_t, AT* da, AT* da_t,
                               int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    float f, f1, f2;
    act_derivs(act, ldf(a, i), f, f1, f2);
    const float d = ldf(dy, i);
    stf(da, i, f1 * d);
    stf(da_t, i, f1 * ldf(dy_t, i) + f2 * ldf(a_t, i) * d);
  }
}

template <typename AT>
__global__ void act_fwd_vec_kernel(int act, const AT* a, const AT* a_t, const AT* a_lo, AT* y, AT* y_t, AT* y_lo, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
    float av[8], at[8], yv[8], yt[8], yl[8];
    ld8(a, i, av); ld8(a_t, i, at);
    if (a_lo) { float al[8]; ld8(a_lo, i, al);
#pragma unroll
      for (int q = 0; q < 8; ++q) av[q] += al[q]; }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      float f, f1, f2;
      act_derivs(act, av[q], f, f1, f2);
      yv[q] = f; yt[q] = f1 * at[q]; yl[q] = f - (float)(AT)f;
    }
    st8(y, i, yv); st8(y_t, i, yt);
    if (y_lo) st8(y_lo, i, yl);
  }
}
template <typename AT>
__global__ void act_bwd_vec_kernel(int act, const AT* a, const AT* a_t, const AT* dy, const AT* dy_t, AT* da, AT* da_t, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
    float av[8], at[8], d[8], dt[8], o[8], ot[8];
    ld8(a, i, av); ld8(a_t, i, at); ld8(dy, i, d); ld8(dy_t, i, dt);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      float f, f1, f2;
      act_derivs(act, av[q], f, f1, f2);
      o[q] = f1 * d[q]; ot[q] = f1 * dt[q] + f2 * at[q] * d[q];
    }
    st8(da, i, o); st8(da_t, i, ot);
  }
}
template <typename AT>
__global__ void swiglu_fwd_vec_kernel(const AT* g, const AT* g_t, const AT* u, const AT* u_t, const AT* g_lo, const AT* u_lo,
                                      AT* y, AT* y_t, AT* y_lo, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
    float gv[8], gt[8], uv[8], ut[8], yv[8], yt[8], yl[8];
    ld8(g, i, gv); ld8(g_t, i, gt); ld8(u, i, uv); ld8(u_t, i, ut);
    if (g_lo) { float a8[8], b8[8]; ld8(g_lo, i, a8); ld8(u_lo, i, b8);
#pragma unroll
      for (int q = 0; q < 8; ++q) { gv[q] += a8[q]; uv[q] += b8[q]; } }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float sg = 1.f / (1.f + __expf(-gv[q]));
      const float s = gv[q] * sg, s1 = sg + gv[q] * sg * (1.f - sg);
      yv[q] = s * uv[q]; yt[q] = s1 * gt[q] * uv[q] + s * ut[q]; yl[q] = yv[q] - (float)(AT)yv[q];
    }
    st8(y, i, yv); st8(y_t, i, yt);
    if (y_lo) st8(y_lo, i, yl);
  }
}
template <typename AT>
__global__ void swiglu_bwd_vec_kernel(const AT* g, const AT* g_t, const AT* u, const AT* u_t, const AT* dy, const AT* dy_t,
                                      AT* dg, AT* dg_t, AT* du, AT* du_t, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
    float gv[8], gt[8], uv[8], ut[8], d[8], dt[8], o1[8], o2[8], o3[8], o4[8];
    ld8(g, i, gv); ld8(g_t, i, gt); ld8(u, i, uv); ld8(u_t, i, ut); ld8(dy, i, d); ld8(dy_t, i, dt);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float sg = 1.f / (1.f + __expf(-gv[q]));
      const float dsg = sg * (1.f - sg);
      const float s = gv[q] * sg, s1 = sg + gv[q] * dsg, s2 = dsg * (2.f + gv[q] * (1.f - 2.f * sg));
      o1[q] = s1 * uv[q] * d[q];
      o3[q] = s * d[q];
      o2[q] = s2 * gt[q] * uv[q] * d[q] + s1 * ut[q] * d[q] + s1 * uv[q] * dt[q];
      o4[q] = s1 * gt[q] * d[q] + s * dt[q];
    }
    st8(dg, i, o1); st8(dg_t, i, o2); st8(du, i, o3); st8(du_t, i, o4);
  }
}

hipError_t launch_act_fwd(int bf, int act, const void* a, const void* a_t, const void* a_lo, void* y, void* y_t,
                          void* y_lo, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n % 8 == 0 && all_aligned16({a, a_t, a_lo, y, y_t, y_lo})) {
    const int nb = ew_blocks(n / 8);
    if (bf) hipLaunchKernelGGL(act_fwd_vec_kernel<bf16>, dim3(nb), dim3(256), 0, st, act, (const bf16*)a, (const bf16*)a_t, (const bf16*)a_lo, (bf16*)y, (bf16*)y_t, (bf16*)y_lo, n / 8);
    else hipLaunchKernelGGL(act_fwd_vec_kernel<float>, dim3(nb), dim3(256), 0, st, act, (const float*)a, (const float*)a_t, (const float*)a_lo, (float*)y, (float*)y_t, (float*)y_lo, n / 8);
    return hipGetLastError();
  }
  if (bf) hipLaunchKernelGGL(act_fwd_kernel<bf16>, dim3(ew_blocks(n)), dim3(256), 0, st, act, (const bf16*)a, (const bf16*)a_t, (const bf16*)a_lo, (bf16*)y, (bf16*)y_t, (bf16*)y_lo, n);
  else hipLaunchKernelGGL(act_fwd_kernel<float>, dim3(ew_blocks(n)), dim3(256), 0, st, act, (const float*)a, (const float*)a_t, (const float*)a_lo, (float*)y, (float*)y_t, (float*)y_lo, n);
  return hipGetLastError();
}
hipError_t launch_act_bwd(int bf, int act, const void* a, const void* a_t, const void* dy, const void* dy_t, void* da,
                          void* da_t, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n % 8 == 0 && all_aligned16({a, a_t, dy, dy_t, da, da_t})) {
    const int nb = ew_blocks(n / 8);
    if (bf) hipLaunchKernelGGL(act_bwd_vec_kernel<bf16>, dim3(nb), dim3(256), 0, st, act, (const bf16*)a, (const bf16*)a_t, (const bf16*)dy, (const bf16*)dy_t, (bf16*)da, (bf16*)da_t, n / 8);
    else hipLaunchKernelGGL(act_bwd_vec_kernel<float>, dim3(nb), dim3(256), 0, st, act, (const float*)a, (const float*)a_t, (const float*)dy, (const float*)dy_t, (float*)da, (float*)da_t, n / 8);
    return hipGetLastError();
  }
  if (bf) hipLaunchKernelGGL(act_bwd_kernel<bf16>, dim3(ew_blocks(n)), dim3(256), 0, st, act, (const bf16*)a, (const bf16*)a_t, (const bf16*)dy, (const bf16*)dy_t, (bf16*)da, (bf16*)da_t, n);
  else hipLaunchKernelGGL(act_bwd_kernel<float>, dim3(ew_blocks(n)), dim3(256), 0, st, act, (const float*)a, (const float*)a_t, (const float*)dy, (const float*)dy_t, (float*)da, (float*)da_t, n);
  return hipGetLastError();
}

// SwiGLU y = s(g) u with s(g) = g sigmoid(g):
//   s' = sig + g sig', s'' = sig' (2 + g (1 - 2 sig)), sig' = sig (1 - sig).
template <typename AT>
__global__ void swiglu_fwd_kernel(const AT* g, const AT* g_t, const AT* u, const AT* u_t, const AT* g_lo,
                                  const AT* u_lo, AT* y, AT* y_t, AT* y_lo, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    float gv = ldf(g, i), uv = ldf(u, i);
    if (g_lo) { gv += ldf(g_lo, i); uv += ldf(u_lo, i); }
    const float sg = 1.f / (1.f + __expf(-gv));
    const float s = gv * sg, s1 = sg + gv * sg * (1.f - sg);
    const float yv = s * uv;
    stf(y, i, yv);
    stf(y_t, i, s1 * ldf(g_t, i) * uv + s * ldf(u_t, i));
    if (y_lo) stf(y_lo, i, yv - (float)(AT)yv);
  }
}
template <typename AT>
__global__ void swiglu_bwd_kernel(const AT* g, const AT* g_t, const AT* u, const AT* u_t, const AT* dy, const AT* dy_t,
                                  AT* dg, AT* dg_t, AT* du, AT* du_t, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const float gv = ldf(g, i), uv = ldf(u, i), gt = ldf(g_t, i), ut = ldf(u_t, i);
    const float d = ldf(dy, i), dt = ldf(dy_t, i);
    const float sg = 1.f / (1.f + __expf(-gv));
    const float dsg = sg * (1.f - sg);
    const float s = gv * sg, s1 = sg + gv * dsg, s2 = dsg * (2.f + gv * (1.f - 2.f * sg));
    stf(dg, i, s1 * uv * d);
    stf(du, i, s * d);
    stf(dg_t, i, s2 * gt * uv * d + s1 * ut * d + s1 * uv * dt);
    stf(du_t, i, s1 * gt * d + s * dt);
  }
}
hipError_t launch_swiglu_fwd(int bf, const void* g, const void* g_t, const void* u, const void* u_t, const void* g_lo,
                             const void* u_lo, void* y, void* y_t, void* y_lo, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n % 8 == 0 && all_aligned16({g, g_t, u, u_t, g_lo, u_lo, y, y_t, y_lo})) {
    const int nb = ew_blocks(n / 8);
    if (bf) hipLaunchKernelGGL(swiglu_fwd_vec_kernel<bf16>, dim3(nb), dim3(256), 0, st, (const bf16*)g, (const bf16*)g_t, (const bf16*)u, (const bf16*)u_t, (const bf16*)g_lo, (const bf16*)u_lo, (bf16*)y, (bf16*)y_t, (bf16*)y_lo, n / 8);
    else hipLaunchKernelGGL(swiglu_fwd_vec_kernel<float>, dim3(nb), dim3(256), 0, st, (const float*)g, (const float*)g_t, (const float*)u, (const float*)u_t, (const float*)g_lo, (const float*)u_lo, (float*)y, (float*)y_t, (float*)y_lo, n / 8);
    return hipGetLastError();
  }
  if (bf) hipLaunchKernelGGL(swiglu_fwd_kernel<bf16>, dim3(ew_blocks(n)), dim3(256), 0, st, (const bf16*)g, (const bf16*)g_t, (const bf16*)u, (const bf16*)u_t, (const bf16*)g_lo, (const bf16*)u_lo, (bf16*)y, (bf16*)y_t, (bf16*)y_lo, n);
  else hipLaunchKernelGGL(swiglu_fwd_kernel<float>, dim3(ew_blocks(n)), dim3(256), 0, st, (const float*)g, (const float*)g_t, (const float*)u, (const float*)u_t, (const float*)g_lo, (const float*)u_lo, (float*)y, (float*)y_t, (float*)y_lo, n);
  return hipGetLastError();
}
hipError_t launch_swiglu_bwd(int bf, const void* g, const void* g_t, const void* u, const void* u_t, const void* dy,
                             const void* dy_t, void* dg, void* dg_t, void* du, void* du_t, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n % 8 == 0 && all_aligned16({g, g_t, u, u_t, dy, dy_t, dg, dg_t, du, du_t})) {
    const int nb = ew_blocks(n / 8);
    if (bf) hipLaunchKernelGGL(swiglu_bwd_vec_kernel<bf16>, dim3(nb), dim3(256), 0, st, (const bf16*)g, (const bf16*)g_t, (const bf16*)u, (const bf16*)u_t, (const bf16*)dy, (const bf16*)dy_t, (bf16*)dg, (bf16*)dg_t, (bf16*)du, (bf16*)du_t, n / 8);
    else hipLaunchKernelGGL(swiglu_bwd_vec_kernel<float>, dim3(nb), dim3(256), 0, st, (const float*)g, (const float*)g_t, (const float*)u, (const float*)u_t, (const float*)dy, (const float*)dy_t, (float*)dg, (float*)dg_t, (float*)du, (float*)du_t, n / 8);
    return hipGetLastError();
  }
  if (bf) hipLaunchKernelGGL(swiglu_bwd_kernel<bf16>, dim3(ew_blocks(n)), dim3(256), 0, st, (const bf16*)g, (const bf16*)g_t, (const bf16*)u, (const bf16*)u_t, (const bf16*)dy, (const bf16*)dy_t, (bf16*)dg, (bf16*)dg_t, (bf16*)du, (bf16*)du_t, n);
  else hipLaunchKernelGGL(swiglu_bwd_kernel<float>, dim3(ew_blocks(n)), dim3(256), 0, st, (const float*)g, (const float*)g_t, (const float*)u, (const float*)u_t, (const float*)dy, (const float*)dy_t, (float*)dg, (float*)dg_t, (float*)du, (float*)du_t, n);
  return hipGetLastError();
}

// ---------------------------------------------------------- causal softmax ----
// Row i of a [S,S] score matrix has i+1 live entries.  One wavefront per row.
//   p = softmax(s),  p_t = p (s_t - sum_j p_j s_t_j).  Entries j > i are 0.

template <typename AT>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const float* __restrict__ s, const float* __restrict__ s_t,
                                                          AT* p, AT* p_t, AT* p_lo, int64_t rows, int S) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int i = (int)(row % S);
  const float* sr = s + row * S;
  const float* str = s_t + row * S;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) mx = fmaxf(mx, sr[j]);
  mx = wave_max(mx);
  float sum = 0.f, dot = 0.f;
  for (int j = lane; j <= i; j += 64) {
    const float e = __expf(sr[j] - mx);
    sum += e;
    dot += e * str[j];
  }
  sum = wave_sum(sum);
  dot = wave_sum(dot);
  const float inv = 1.f / sum;
  dot *= inv;
  for (int j = lane; j < S; j += 64) {
    float pv = 0.f, pt = 0.f;
    if (j <= i) {
      pv = __expf(sr[j] - mx) * inv;
      pt = pv * (str[j] - dot);
    }
    stf(p, row * S + j, pv);
    stf(p_t, row * S + j, pt);
    if (p_lo) stf(p_lo, row * S + j, pv - (float)(AT)pv);
  }
}
hipError_t launch_softmax_fwd(int bf, const float* s, const float* s_t, void* p, void* p_t, void* p_lo, int nbh, int S,
                              hipStream_t st) {
  const int64_t rows = (int64_t)nbh * S;
  const int blocks = (int)cdiv(rows, 4);
  if (bf) hipLaunchKernelGGL(softmax_fwd_kernel<bf16>, dim3(blocks), dim3(256), 0, st, s, s_t, (bf16*)p, (bf16*)p_t, (bf16*)p_lo, rows, S);
  else hipLaunchKernelGGL(softmax_fwd_kernel<float>, dim3(blocks), dim3(256), 0, st, s, s_t, (float*)p, (float*)p_t, (float*)p_lo, rows, S);
  return hipGetLastError();
}

// delta = sum p dp; delta_t = sum (p_t dp + p dp_t);
// ds = p (dp - delta); ds_t = p_t (dp - delta) + p (dp_t - delta_t).
template <typename AT>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const AT* __restrict__ p, const AT* __restrict__ p_t,
                                                          const float* __restrict__ dp, const float* __restrict__ dp_t,
                                                          AT* ds, AT* ds_t, int64_t rows, int S) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int i = (int)(row % S);
  const int64_t b = row * S;
  float dl = 0.f, dlt = 0.f;
  for (int j = lane; j <= i; j += 64) {
    const float pv = ldf(p, b + j), pt = ldf(p_t, b + j);
    dl += pv * dp[b + j];
    dlt += pt * dp[b + j] + pv * dp_t[b + j];
  }
  dl = wave_sum(dl);
  dlt = wave_sum(dlt);
  for (int j = lane; j < S; j += 64) {
    float a = 0.f, at = 0.f;
    if (j <= i) {
      const float pv = ldf(p, b + j), pt = ldf(p_t, b + j);
      a = pv * (dp[b + j] - dl);
      at = pt * (dp[b + j] - dl) + pv * (dp_t[b + j] - dlt);
    }
    stf(ds, b + j, a);
    stf(ds_t, b + j, at);
  }
}
hipError_t launch_softmax_bwd(int bf, const void* p, const void* p_t, const float* dp, const float* dp_t, void* ds,
                              void* ds_t, int nbh, int S, hipStream_t st) {
  const int64_t rows = (int64_t)nbh * S;
  const int blocks = (int)cdiv(rows, 4);
  if (bf) hipLaunchKernelGGL(softmax_bwd_kernel<bf16>, dim3(blocks), dim3(256), 0, st, (const bf16*)p, (const bf16*)p_t, dp, dp_t, (bf16*)ds, (bf16*)ds_t, rows, S);
  else hipLaunchKernelGGL(softmax_bwd_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)p, (const float*)p_t, dp, dp_t, (float*)ds, (float*)ds_t, rows, S);
  return hipGetLastError();
}

// ------------------------------------------------------------------- RoPE ----
// Pair (i, i + dh/2) of every head is rotated by pos * theta^(-2i/dh); the
// tangent takes the same rotation, adjoints the transposed one.

template <typename AT>
__global__ void rope_kernel(const float* src, const float* src_t, int64_t lds, AT* dst, AT* dst_t, AT* dst_lo,
                            int64_t ldd, int T, int S, int n_head, int dh, float log2_theta, int inverse) {
  const int half = dh / 2;
  const int64_t total = (int64_t)T * n_head * half;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
    const int i = (int)(idx % half);
    const int h = (int)((idx / half) % n_head);
    const int64_t t = idx / ((int64_t)half * n_head);
    const int pos = (int)(t % S);
    const double ang = (double)pos * exp2(-2.0 * (double)i / (double)dh * (double)log2_theta);
    float sn = (float)sin(ang), cs = (float)cos(ang);
    if (inverse) sn = -sn;
    const int64_t a = t * lds + (int64_t)h * dh + i, b = a + half;
    const int64_t oa = t * ldd + (int64_t)h * dh + i, ob = oa + half;
    const float x1 = src[a], x2 = src[b];
    const float r1 = x1 * cs - x2 * sn, r2 = x2 * cs + x1 * sn;
    stf(dst, oa, r1);
    stf(dst, ob, r2);
    if (dst_lo) { stf(dst_lo, oa, r1 - (float)(AT)r1); stf(dst_lo, ob, r2 - (float)(AT)r2); }
    const float y1 = src_t[a], y2 = src_t[b];
    stf(dst_t, oa, y1 * cs - y2 * sn);
    stf(dst_t, ob, y2 * cs + y1 * sn);
  }
}
hipError_t launch_rope(int bf, const float* src, const float* src_t, int64_t lds, void* dst, void* dst_t, void* dst_lo,
                       int64_t ldd, int T, int S, int n_head, int dh, float theta, int inverse, hipStream_t st) {
  const int64_t total = (int64_t)T * n_head * (dh / 2);
  if (total <= 0) return hipSuccess;
  const float l2 = log2f(theta);
  if (bf) hipLaunchKernelGGL(rope_kernel<bf16>, dim3(ew_blocks(total)), dim3(256), 0, st, src, src_t, lds, (bf16*)dst, (bf16*)dst_t, (bf16*)dst_lo, ldd, T, S, n_head, dh, l2, inverse);
  else hipLaunchKernelGGL(rope_kernel<float>, dim3(ew_blocks(total)), dim3(256), 0, st, src, src_t, lds, (float*)dst, (float*)dst_t, (float*)dst_lo, ldd, T, S, n_head, dh, l2, inverse);
  return hipGetLastError();
}

// ------------------------------------------------ softmax cross-entropy ------
// L = mean over valid rows of lse(z) - z[y];  dz = (p - onehot)/N;
// dz_t = p (z_t - <p, z_t>)/N.  Ignored rows (label < 0) produce zeros.

__global__ void count_valid_kernel(const int32_t* labels, int T, int V, int* n_valid, int* err_flag) {
  int cnt = 0, bad = 0;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < T; i += gridDim.x * blockDim.x) {
    const int y = labels[i];
    cnt += (y >= 0);
    bad |= (y >= V);
  }
  float c = wave_sum((float)cnt);
  if ((threadIdx.x & 63) == 0 && c > 0.f) atomicAdd(n_valid, (int)c);
  if (bad) atomicOr(err_flag, 2);
}
hipError_t launch_count_valid(const int32_t* labels, int T, int V, int* n_valid, int* err_flag, hipStream_t st) {
  hipLaunchKernelGGL(count_valid_kernel, dim3((int)std::min<int64_t>(cdiv(T, 256), 256)), dim3(256), 0, st, labels, T, V, n_valid, err_flag);
  return hipGetLastError();
}

// Two passes over a row of logits (rows are 16-byte aligned: ldz % 64 == 0):
// an online-softmax pass that keeps (max, sum exp, sum exp * z_t) per thread,
// rescaled when the running maximum moves, then the pass that writes dz, dz_t.
__device__ __forceinline__ void st4f(float* p, int64_t i, float a, float b, float c, float d) { *(float4*)(p + i) = make_float4(a, b, c, d); }
__device__ __forceinline__ void st4f(bf16* p, int64_t i, float a, float b, float c, float d) {
  bf16 o[4] = {(bf16)a, (bf16)b, (bf16)c, (bf16)d};
  *(uint2*)(p + i) = *(const uint2*)o;
}

template <typename AT>
__global__ __launch_bounds__(256) void ce_kernel(const float* __restrict__ z, const float* __restrict__ z_t,
                                                 const int32_t* labels, const int* n_valid, int V, int64_t ldz, AT* dz,
                                                 AT* dz_t, float* loss_rows, float scale) {
  __shared__ float red[16];
  const int64_t row = blockIdx.x;
  const float* zr = z + row * ldz;
  const float* ztr = z_t + row * ldz;
  const int y = labels[row];
  const int V4 = V >> 2;
  if (y < 0 || y >= V) {
    for (int c = threadIdx.x; c < V4; c += 256) { st4f(dz, row * ldz + 4 * c, 0.f, 0.f, 0.f, 0.f); st4f(dz_t, row * ldz + 4 * c, 0.f, 0.f, 0.f, 0.f); }
    for (int c = 4 * V4 + threadIdx.x; c < V; c += 256) { stf(dz, row * ldz + c, 0.f); stf(dz_t, row * ldz + c, 0.f); }
    if (threadIdx.x == 0) loss_rows[row] = 0.f;
    return;
  }
  float m = -INFINITY, se = 0.f, sd = 0.f;
  for (int c = threadIdx.x; c < V4; c += 256) {
    const float4 x = ((const float4*)zr)[c], t = ((const float4*)ztr)[c];
    const float mn = fmaxf(fmaxf(m, fmaxf(x.x, x.y)), fmaxf(x.z, x.w));
    const float sc = __expf(m - mn);  // exp(-inf) = 0 on the first visit
    const float e0 = __expf(x.x - mn), e1 = __expf(x.y - mn), e2 = __expf(x.z - mn), e3 = __expf(x.w - mn);
    se = se * sc + ((e0 + e1) + (e2 + e3));
    sd = sd * sc + ((e0 * t.x + e1 * t.y) + (e2 * t.z + e3 * t.w));
    m = mn;
  }
  for (int c = 4 * V4 + threadIdx.x; c < V; c += 256) {
    const float x = zr[c], mn = fmaxf(m, x), sc = __expf(m - mn), e = __expf(x - mn);
    se = se * sc + e;
    sd = sd * sc + e * ztr[c];
    m = mn;
  }
  const float mx = block_max(m, red);
  float s[2];
  {
    const float sc = (m == -INFINITY) ? 0.f : __expf(m - mx);  // a thread that saw no column contributes nothing
    s[0] = se * sc;
    s[1] = sd * sc;
  }
  block_sum<2>(s, red);
  const float inv = 1.f / s[0];
  const float pz = s[1] * inv;
  const float invN = scale / (float)max(1, *n_valid);
  for (int c = threadIdx.x; c < V4; c += 256) {
    const float4 x = ((const float4*)zr)[c], t = ((const float4*)ztr)[c];
    const float p0 = __expf(x.x - mx) * inv, p1 = __expf(x.y - mx) * inv, p2 = __expf(x.z - mx) * inv, p3 = __expf(x.w - mx) * inv;
    const int c0 = 4 * c;
    st4f(dz, row * ldz + c0, (p0 - (c0 == y ? 1.f : 0.f)) * invN, (p1 - (c0 + 1 == y ? 1.f : 0.f)) * invN,
         (p2 - (c0 + 2 == y ? 1.f : 0.f)) * invN, (p3 - (c0 + 3 == y ? 1.f : 0.f)) * invN);
    st4f(dz_t, row * ldz + c0, p0 * (t.x - pz) * invN, p1 * (t.y - pz) * invN, p2 * (t.z - pz) * invN, p3 * (t.w - pz) * invN);
  }
  for (int c = 4 * V4 + threadIdx.x; c < V; c += 256) {
    const float pv = __expf(zr[c] - mx) * inv;
    stf(dz, row * ldz + c, (pv - (c == y ? 1.f : 0.f)) * invN);
    stf(dz_t, row * ldz + c, pv * (ztr[c] - pz) * invN);
  }
  if (threadIdx.x == 0) loss_rows[row] = logf(s[0]) + mx - zr[y];
}
// One pass over a row: 1024 threads hold the row of z and of z_t in registers (EPT chunks of four
// columns each, V <= 4096 EPT), so the logits are read once instead of twice.  Rows are 16-byte
// aligned (ldz % 64 == 0); the V % 4 last columns go through thread-private scalars.
template <typename AT, int EPT>
__global__ __launch_bounds__(1024) void ce_row_kernel(const float* __restrict__ z, const float* __restrict__ z_t,
                                                      const int32_t* __restrict__ labels, const int* __restrict__ n_valid,
                                                      int V, int64_t ldz, AT* __restrict__ dz, AT* __restrict__ dz_t,
                                                      float* __restrict__ loss_rows, float scale) {
  __shared__ float red[48];
  const int64_t row = blockIdx.x;
  const float* zr = z + row * ldz;
  const float* ztr = z_t + row * ldz;
  const int y = labels[row];
  const int V4 = V >> 2, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int ct = 4 * V4 + t;  // this thread's tail column (valid if < V)
  if (y < 0 || y >= V) {
    for (int c = t; c < V4; c += 1024) { st4f(dz, row * ldz + 4 * c, 0.f, 0.f, 0.f, 0.f); st4f(dz_t, row * ldz + 4 * c, 0.f, 0.f, 0.f, 0.f); }
    if (ct < V) { stf(dz, row * ldz + ct, 0.f); stf(dz_t, row * ldz + ct, 0.f); }
    if (t == 0) loss_rows[row] = 0.f;
    return;
  }
  float4 x[EPT], d[EPT];
  float xt = -INFINITY, dt = 0.f;
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int c = t + 1024 * j;
    x[j] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    d[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < V4) { x[j] = ((const float4*)zr)[c]; d[j] = ((const float4*)ztr)[c]; }
    m = fmaxf(m, fmaxf(fmaxf(x[j].x, x[j].y), fmaxf(x[j].z, x[j].w)));
  }
  if (ct < V) { xt = zr[ct]; dt = ztr[ct]; m = fmaxf(m, xt); }
  // block maximum over 16 waves
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  float mx = red[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) mx = fmaxf(mx, red[w]);
  float se = 0.f, sd = 0.f;
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    x[j].x = __expf(x[j].x - mx); x[j].y = __expf(x[j].y - mx); x[j].z = __expf(x[j].z - mx); x[j].w = __expf(x[j].w - mx);
    se += (x[j].x + x[j].y) + (x[j].z + x[j].w);
    sd += (x[j].x * d[j].x + x[j].y * d[j].y) + (x[j].z * d[j].z + x[j].w * d[j].w);
  }
  xt = __expf(xt - mx);  // exp(-inf) = 0 for a thread without a tail column
  se += xt; sd += xt * dt;
  se = wave_sum(se); sd = wave_sum(sd);
  if (lane == 0) { red[16 + wave] = se; red[32 + wave] = sd; }
  __syncthreads();
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) { s0 += red[16 + w]; s1 += red[32 + w]; }
  const float inv = 1.f / s0;
  const float pz = s1 * inv;
  const float invN = scale / (float)max(1, *n_valid);
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int c = t + 1024 * j;
    if (c < V4) {
      const float p0 = x[j].x * inv, p1 = x[j].y * inv, p2 = x[j].z * inv, p3 = x[j].w * inv;
      const int c0 = 4 * c;
      st4f(dz, row * ldz + c0, (p0 - (c0 == y ? 1.f : 0.f)) * invN, (p1 - (c0 + 1 == y ? 1.f : 0.f)) * invN,
           (p2 - (c0 + 2 == y ? 1.f : 0.f)) * invN, (p3 - (c0 + 3 == y ? 1.f : 0.f)) * invN);
      st4f(dz_t, row * ldz + c0, p0 * (d[j].x - pz) * invN, p1 * (d[j].y - pz) * invN, p2 * (d[j].z - pz) * invN,
           p3 * (d[j].w - pz) * invN);
    }
  }
  if (ct < V) {
    const float pv = xt * inv;
    stf(dz, row * ldz + ct, (pv - (ct == y ? 1.f : 0.f)) * invN);
    stf(dz_t, row * ldz + ct, pv * (dt - pz) * invN);
  }
  if (t == 0) loss_rows[row] = logf(s0) + mx - zr[y];
}

hipError_t launch_ce(int bf, const float* z, const float* z_t, const int32_t* labels, const int* n_valid, int T, int V,
                     int64_t ldz, void* dz, void* dz_t, float* loss_rows, float scale, hipStream_t st) {
  if (bf && V >= 8192 && ldz % 4 == 0) {  // wide rows: the two-pass kernel reads them twice
    if (V <= 4096 * 8) { hipLaunchKernelGGL((ce_row_kernel<bf16, 8>), dim3(T), dim3(1024), 0, st, z, z_t, labels, n_valid, V, ldz, (bf16*)dz, (bf16*)dz_t, loss_rows, scale); return hipGetLastError(); }
    if (V <= 4096 * 13) { hipLaunchKernelGGL((ce_row_kernel<bf16, 13>), dim3(T), dim3(1024), 0, st, z, z_t, labels, n_valid, V, ldz, (bf16*)dz, (bf16*)dz_t, loss_rows, scale); return hipGetLastError(); }
  }
  if (bf) hipLaunchKernelGGL(ce_kernel<bf16>, dim3(T), dim3(256), 0, st, z, z_t, labels, n_valid, V, ldz, (bf16*)dz, (bf16*)dz_t, loss_rows, scale);
  else hipLaunchKernelGGL(ce_kernel<float>, dim3(T), dim3(256), 0, st, z, z_t, labels, n_valid, V, ldz, (float*)dz, (float*)dz_t, loss_rows, scale);
  return hipGetLastError();
}

// out[0] = weight * mean over the valid rows (added to out[0] when accumulate); a batch without a
// valid label sets bit 2 of err_flag.
__global__ __launch_bounds__(256) void sum_rows_f64_kernel(const float* v, int n, const int* n_valid, double* out, double weight,
                                                           int accumulate, int* err_flag) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += (double)v[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const int nv = *n_valid;
    if (nv == 0) atomicOr(err_flag, 4);
    out[0] = (accumulate ? out[0] : 0.0) + weight * red[0] / (double)max(1, nv);
  }
}
hipError_t launch_sum_rows_f64(const float* v, int n, const int* n_valid, double* out, double weight, int accumulate,
                               int* err_flag, hipStream_t st) {
  hipLaunchKernelGGL(sum_rows_f64_kernel, dim3(1), dim3(256), 0, st, v, n, n_valid, out, weight, accumulate, err_flag);
  return hipGetLastError();
}

// ------------------------------------------------------------ column sums ----

template <typename AT>
__global__ void colsum_kernel(const AT* y, int T, int N, int64_t ld, int rows_per_block, float* out) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= N) return;
  const int r0 = blockIdx.y * rows_per_block, r1 = min(T, r0 + rows_per_block);
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += ldf(y, (int64_t)r * ld + c);
  atomicAdd(out + c, s);
}
// 8 consecutive columns per thread (16-byte loads of bf16, two of fp32), 8 row
// lanes per block that meet in LDS: one atomic per column per block.
template <typename AT>
__global__ __launch_bounds__(256) void colsum_vec_kernel(const AT* __restrict__ y, int T, int N, int64_t ld, int rows_per_block,
                                                         float* out) {
  __shared__ float red[8][256 + 8];
  const int cg = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int c = blockIdx.x * 256 + cg * 8;
  const int r0 = blockIdx.y * rows_per_block, r1 = min(T, r0 + rows_per_block);
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (c < N) {
    for (int r = r0 + rl; r < r1; r += 8) {
      float v[8];
      ld8(y + (int64_t)r * ld + c, 0, v);
#pragma unroll
      for (int q = 0; q < 8; ++q) s[q] += v[q];
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) red[rl][cg * 8 + q] = s[q];
  __syncthreads();
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col < N) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) t += red[k][threadIdx.x];
    atomicAdd(out + col, t);
  }
}

hipError_t launch_colsum(int is_bf16, const void* y, int T, int N, int64_t ld, float* out, hipStream_t st) {
  if (T <= 0 || N <= 0) return hipSuccess;
  if (N % 8 == 0 && ld % 8 == 0 && ((uintptr_t)y & 15) == 0 && T >= 256) {
    const int rows = 128;
    dim3 grid((N + 255) / 256, (T + rows - 1) / rows);
    if (is_bf16) hipLaunchKernelGGL(colsum_vec_kernel<bf16>, grid, dim3(256), 0, st, (const bf16*)y, T, N, ld, rows, out);
    else hipLaunchKernelGGL(colsum_vec_kernel<float>, grid, dim3(256), 0, st, (const float*)y, T, N, ld, rows, out);
    return hipGetLastError();
  }
  const int rpb = 64;
  dim3 grid((N + 255) / 256, (T + rpb - 1) / rpb);
  if (is_bf16) hipLaunchKernelGGL(colsum_kernel<bf16>, grid, dim3(256), 0, st, (const bf16*)y, T, N, ld, rpb, out);
  else hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)y, T, N, ld, rpb, out);
  return hipGetLastError();
}

}  // namespace hf
