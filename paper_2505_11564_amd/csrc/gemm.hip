// Matrix-product kernels of the Hessian-vector product (Algorithm 1 of the
// paper needs, per linear layer Y = X W: the forward product, its tangent
// X_t W + X W_t, the adjoint dY W^T, its tangent dY_t W^T + dY W_t^T, and the
// H v block X_t^T dY + X^T dY_t; attention needs the same forms per head).
//
// One launcher covers all of them: C = alpha (A0 op B0 + A1 op B1) + bias
// (+ Cadd), optionally batched over (batch, head) with strided operands so the
// per-head slices of the packed q|k|v activations are read in place.
//
//   gemm_bf16_kernel : bf16 operands, fp32 accumulate on the CDNA4 matrix
//                      cores (v_mfma_f32_32x32x16_bf16), LDS-staged tiles,
//                      register prefetch of the next k-slab.
//   gemm_f32_kernel  : fp32 operands, plain FMA, fully guarded; used by the
//                      fp32 parity configurations, which are launch-bound.
#include "hf_internal.h"
#include "gemm_params.h"

#include <cstdlib>

namespace hf {

// ------------------------------------------------------------------ fp32 ----

template <int BM, int BN, int BK>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmP p) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int t = threadIdx.x;
  const int tile = blockIdx.x;
  const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
  if (p.skip_upper && n0 > m0 + BM - 1) return;
  const int z = blockIdx.y, z1 = z / p.nb2, z2 = z % p.nb2;
  const int64_t offA = z1 * p.sA1 + z2 * p.sA2, offB = z1 * p.sB1 + (z2 / p.divB) * p.sB2, offC = z1 * p.sC1 + z2 * p.sC2;
  int kbeg = 0, kend = p.K;
  if (p.klimit == 1) kend = min(p.K, m0 + BM);
  if (p.klimit == 2) kbeg = (m0 / BK) * BK;
  const int tx = t % 16, ty = t / 16;
  float acc[4][4] = {};
  const int nterm = p.nterm;
  for (int term = 0; term < nterm; ++term) {
    const float* A = (const float*)p.A[term] + offA;
    const float* B = (const float*)p.B[term] + offB;
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
      for (int i = t; i < BM * BK; i += 256) {
        int m, k;
        if (p.transA) { m = i % BM; k = i / BM; } else { k = i % BK; m = i / BK; }
        const int gm = m0 + m, gk = k0 + k;
        float v = 0.f;
        if (gm < p.M && gk < kend) v = p.transA ? A[(int64_t)gk * p.lda + gm] : A[(int64_t)gm * p.lda + gk];
        As[k][m] = v;
      }
      for (int i = t; i < BN * BK; i += 256) {
        int n, k;
        if (p.transB) { k = i % BK; n = i / BK; } else { n = i % BN; k = i / BN; }
        const int gn = n0 + n, gk = k0 + k;
        float v = 0.f;
        if (gn < p.N && gk < kend) v = p.transB ? B[(int64_t)gn * p.ldb + gk] : B[(int64_t)gk * p.ldb + gn];
        Bs[k][n] = v;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < BK; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= p.N) continue;
      float v = p.alpha * acc[i][j];
      if (p.bias) v += p.bias_bf16 ? (float)((const bf16*)p.bias)[gn] : ((const float*)p.bias)[gn];
      if (p.bias_t) v += p.bias_t[gn];
      const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
      if (p.Cadd) v += p.Cadd[ci];
      if (p.out_bf16) {
            const bf16 hi = (bf16)v;
            ((bf16*)p.C)[ci] = hi;
            if (p.C_lo) ((bf16*)p.C_lo)[ci] = (bf16)(v - (float)hi);
          } else {
            ((float*)p.C)[ci] = v;
          }
    }
  }
}

// ------------------------------------------------------------------ bf16 ----

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;
constexpr int BKP = BK + 8;  // padded LDS row (80 B): conflict-free 16 B reads

// Global -> registers for a tile of R rows x BK k-values, destined for LDS
// laid out [row][k].  KC: the source is k-contiguous (element (r,k) at
// src[r*ld + k]); otherwise r-contiguous (src[k*ld + r]) and the 2 x 8 block a
// thread fetches is transposed in registers.
template <int R, bool KC>
__device__ __forceinline__ void tile_fetch(uint4 (&regs)[R / 64], const bf16* __restrict__ src, int64_t ld, int r0,
                                           int k0, int rmax, int kend, bool vec, int t) {
#pragma unroll
  for (int i = 0; i < R / 64; ++i) {
    if (KC) {
      const int c = t + i * 256;
      const int row = c >> 2, kc = (c & 3) * 8;
      const int gr = r0 + row, gk = k0 + kc;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (gr < rmax) {
        const bf16* ptr = src + (int64_t)gr * ld + gk;
        if (vec && gk + 8 <= kend) {
          v = *(const uint4*)ptr;
        } else {
          unsigned short e[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) e[q] = (gk + q < kend) ? ((const unsigned short*)ptr)[q] : (unsigned short)0;
          v.x = e[0] | ((unsigned)e[1] << 16); v.y = e[2] | ((unsigned)e[3] << 16);
          v.z = e[4] | ((unsigned)e[5] << 16); v.w = e[6] | ((unsigned)e[7] << 16);
        }
      }
      regs[i] = v;
    }
  }
  if (!KC) {
    // R/128 thread-items, each a pair of rows (2rp, 2rp+1) x 8 k-values
#pragma unroll
    for (int i = 0; i < R / 128; ++i) {
      const int c = t + i * 256;
      const int rp = c % (R / 2), kb = c / (R / 2);
      const int gr = r0 + 2 * rp, gk = k0 + kb * 8;
      unsigned w[8];
      if (vec && gr + 1 < rmax && gk + 8 <= kend) {
#pragma unroll
        for (int q = 0; q < 8; ++q) w[q] = *(const unsigned*)(src + (int64_t)(gk + q) * ld + gr);
      } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          unsigned lo = 0, hi = 0;
          if (gk + q < kend) {
            const unsigned short* ptr = (const unsigned short*)(src + (int64_t)(gk + q) * ld + gr);
            if (gr < rmax) lo = ptr[0];
            if (gr + 1 < rmax) hi = ptr[1];
          }
          w[q] = lo | (hi << 16);
        }
      }
      uint4 a, b;  // a: row 2rp, b: row 2rp+1
      a.x = (w[0] & 0xffffu) | (w[1] << 16); b.x = (w[0] >> 16) | (w[1] & 0xffff0000u);
      a.y = (w[2] & 0xffffu) | (w[3] << 16); b.y = (w[2] >> 16) | (w[3] & 0xffff0000u);
      a.z = (w[4] & 0xffffu) | (w[5] << 16); b.z = (w[4] >> 16) | (w[5] & 0xffff0000u);
      a.w = (w[6] & 0xffffu) | (w[7] << 16); b.w = (w[6] >> 16) | (w[7] & 0xffff0000u);
      regs[2 * i] = a;
      regs[2 * i + 1] = b;
    }
  }
}

template <int R, bool KC>
__device__ __forceinline__ void tile_store(const uint4 (&regs)[R / 64], bf16* lds, int t) {
  if (KC) {
#pragma unroll
    for (int i = 0; i < R / 64; ++i) {
      const int c = t + i * 256;
      *(uint4*)(lds + (c >> 2) * BKP + (c & 3) * 8) = regs[i];
    }
  } else {
#pragma unroll
    for (int i = 0; i < R / 128; ++i) {
      const int c = t + i * 256;
      const int rp = c % (R / 2), kb = c / (R / 2);
      *(uint4*)(lds + (2 * rp) * BKP + kb * 8) = regs[2 * i];
      *(uint4*)(lds + (2 * rp + 1) * BKP + kb * 8) = regs[2 * i + 1];
    }
  }
}

// Block tile BM x BN, 4 waves arranged (BM/WM) x (BN/WN), each wave WM x WN
// built from 32x32x16 MFMA tiles.
template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmP p) {
  static_assert((BM / WM) * (BN / WN) == 4, "four waves");
  __shared__ __attribute__((aligned(16))) bf16 As[BM * BKP];
  __shared__ __attribute__((aligned(16))) bf16 Bs[BN * BKP];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int tile = blockIdx.x;
  const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
  if (p.skip_upper && n0 > m0 + BM - 1) return;
  const int z = blockIdx.y, z1 = z / p.nb2, z2 = z % p.nb2;
  const int64_t offA = z1 * p.sA1 + z2 * p.sA2, offB = z1 * p.sB1 + (z2 / p.divB) * p.sB2, offC = z1 * p.sC1 + z2 * p.sC2;
  int kbeg = 0, kend = p.K;
  if (p.klimit == 1) kend = min(p.K, m0 + BM);
  if (p.klimit == 2) kbeg = (m0 / BK) * BK;
  const int wm0 = (wave / (BN / WN)) * WM, wn0 = (wave % (BN / WN)) * WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (kend - kbeg + BK - 1) / BK;
  const int nterm = p.nterm;
  const int total = nk * nterm;
  uint4 ra[BM / 64], rb[BN / 64];
  auto fetch = [&](int it) {
    const int term = it / nk, k0 = kbeg + (it % nk) * BK;
    const bf16* A = (const bf16*)p.A[term] + offA;
    const bf16* B = (const bf16*)p.B[term] + offB;
    // A is k-contiguous when not transposed; B (element (k,n)) when transposed.
    tile_fetch<BM, !TA>(ra, A, p.lda, m0, k0, p.M, kend, p.vecA, t);
    tile_fetch<BN, TB>(rb, B, p.ldb, n0, k0, p.N, kend, p.vecB, t);
  };
  if (total > 0) fetch(0);
  for (int it = 0; it < total; ++it) {
    __syncthreads();
    tile_store<BM, !TA>(ra, As, t);
    tile_store<BN, TB>(rb, Bs, t);
    __syncthreads();
    if (it + 1 < total) fetch(it + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *(const bf16x8*)(As + (wm0 + i * 32 + (lane & 31)) * BKP + kk * 16 + (lane >> 5) * 8);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *(const bf16x8*)(Bs + (wn0 + j * 32 + (lane & 31)) * BKP + kk * 16 + (lane >> 5) * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int gn = n0 + wn0 + j * 32 + (lane & 31);
    if (gn >= p.N) continue;
    float bsum = 0.f;
    if (p.bias) bsum += p.bias_bf16 ? (float)((const bf16*)p.bias)[gn] : ((const float*)p.bias)[gn];
    if (p.bias_t) bsum += p.bias_t[gn];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (gm >= p.M) continue;
        float v = p.alpha * acc[i][j][r] + bsum;
        const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
        if (p.Cadd) v += p.Cadd[ci];
        if (p.out_bf16) {
            const bf16 hi = (bf16)v;
            ((bf16*)p.C)[ci] = hi;
            if (p.C_lo) ((bf16*)p.C_lo)[ci] = (bf16)(v - (float)hi);
          } else {
            ((float*)p.C)[ci] = v;
          }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_bf16_cfg(const GemmP& p, dim3 grid, hipStream_t st) {
  if (!p.transA && !p.transB) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, false, false>), grid, dim3(256), 0, st, p);
  else if (!p.transA && p.transB) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, false, true>), grid, dim3(256), 0, st, p);
  else if (p.transA && !p.transB) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, true, false>), grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, true, true>), grid, dim3(256), 0, st, p);
  return hipGetLastError();
}

static bool aligned_to(const void* ptr, size_t a) { return ptr == nullptr || ((uintptr_t)ptr % a) == 0; }

static hipError_t launch_gemm_single(const Gemm& g, hipStream_t st);
static int prepare_single(const Gemm& g, GemmP& p);
static hipError_t launch_prepared(int kind, const Gemm& g, GemmP& p, hipStream_t st);

hipError_t launch_gemm(const Gemm& g, hipStream_t st) {
  if (!g.Ct) return launch_gemm_single(g, st);
  // dual output: one fused launch when the MFMA path applies, else two products
  if (g.M <= 0 || g.N <= 0 || g.nb1 <= 0 || g.nb2 <= 0) return hipSuccess;
  if (!g.At || !g.Bt || !g.A[0] || !g.B[0] || !g.C || ((g.Cadd || g.Cadd_t) && g.out_bf16)) return hipErrorInvalidValue;
  // Measured: the fused kernel wins only when the product alone cannot fill
  // the GPU (fewer than ~256 tiles of 128 x 128); larger products run faster
  // as two launches with their own tile shapes.
  const int64_t tiles128 = ((int64_t)(g.M + 127) / 128) * ((g.N + 127) / 128) * g.nb1 * g.nb2;
  if (g.epi != EPI_NONE && !g.in_bf16) return hipErrorInvalidValue;
  if (g.in_bf16 && g.M >= 8 && g.N >= 8 && (g.epi != EPI_NONE || tiles128 < 256)) {
    auto ok = [&](const void* x, int64_t ld, int64_t s1, int64_t s2, int rows_contig, int R) {
      return ((uintptr_t)x % 16) == 0 && ld % 8 == 0 && s1 % 8 == 0 && s2 % 8 == 0 && (!rows_contig || ld >= ((R + 7) / 8) * 8);
    };
    bool fast = ok(g.At, g.lda, g.sA1, g.sA2, g.transA, g.M) && ok(g.Bt, g.ldb, g.sB1, g.sB2, !g.transB, g.N);
    for (int i = 0; i < 3 && fast; ++i) {
      if (g.A[i]) fast = ok(g.A[i], g.lda, g.sA1, g.sA2, g.transA, g.M) && ok(g.B[i], g.ldb, g.sB1, g.sB2, !g.transB, g.N);
    }
    if (fast) {
      hipError_t e = launch_gemm_dual(g, st);
      if (e != hipErrorNotSupported) return e;
    }
  }
  if (g.epi != EPI_NONE) return hipErrorNotSupported;  // the caller takes the unfused path
  Gemm p = g;
  p.At = nullptr; p.Bt = nullptr; p.Ct = nullptr; p.Cadd_t = nullptr; p.bias_t = nullptr;
  Gemm t = g;
  t.At = nullptr; t.Bt = nullptr; t.Ct = nullptr; t.Cadd_t = nullptr;
  t.A[0] = g.At; t.B[0] = g.B[0]; t.A[1] = g.A[0]; t.B[1] = g.Bt; t.A[2] = nullptr; t.B[2] = nullptr;
  t.C = g.Ct; t.C_lo = nullptr; t.Cadd = g.Cadd_t; t.bias = nullptr;
  GemmP pp, pt;
  const int kp = prepare_single(p, pp), kt = prepare_single(t, pt);
  if (kp == 2 && kt == 2 && p.force_cfg < 0 && !p.allow_splitk) {
    const hipError_t e2 = launch_gemm_mfma_pair(pp, pt, g.nb1 * g.nb2, st);
    if (e2 != hipErrorNotSupported) return e2;
  }
  hipError_t e = launch_prepared(kp, p, pp, st);
  if (e != hipSuccess) return e;
  return launch_prepared(kt, t, pt, st);
}

// Validates a single-output description and fills the kernel parameters.  Returns 0: nothing to
// do, 1: fp32 kernel, 2: MFMA fast path, 3: register-staged bf16 fallback, -1: invalid.
static int prepare_single(const Gemm& g, GemmP& p) {
  if (g.M <= 0 || g.N <= 0 || g.nb1 <= 0 || g.nb2 <= 0) return 0;
  if (!g.A[0] || !g.B[0] || !g.C || (g.A[1] && !g.B[1]) || (g.A[2] && (!g.B[2] || !g.A[1])) || (g.Cadd && g.out_bf16) ||
      (g.C_lo && !g.out_bf16))
    return -1;
  p.nterm = 0;
  for (int i = 0; i < 3; ++i) { p.A[i] = g.A[i]; p.B[i] = g.B[i]; if (g.A[i]) p.nterm = i + 1; }
  p.C_lo = g.C_lo;
  p.C = g.C; p.Cadd = g.Cadd; p.bias = g.bias; p.bias_t = g.bias_t;
  p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
  p.transA = g.transA; p.transB = g.transB; p.nb2 = g.nb2;
  p.sA1 = g.sA1; p.sA2 = g.sA2; p.sB1 = g.sB1; p.sB2 = g.sB2; p.sC1 = g.sC1; p.sC2 = g.sC2;
  p.divB = g.divB > 0 ? g.divB : 1;
  p.alpha = g.alpha; p.out_bf16 = g.out_bf16; p.bias_bf16 = g.in_bf16;
  p.klimit = g.klimit; p.skip_upper = g.skip_upper;
  p.tiles_n = 0; p.vecA = p.vecB = 0;
  if (!g.in_bf16) return 1;
  // vector loaders: k-contiguous operands need 16 B alignment of every row
  // start and batch slice, r-contiguous ones 4 B.
  auto vec_ok = [&](const void* x0, const void* x1, const void* x2, int64_t ld, int64_t s1, int64_t s2, bool kcontig) {
    const int64_t q = kcontig ? 8 : 2;
    return aligned_to(x0, q * 2) && aligned_to(x1, q * 2) && aligned_to(x2, q * 2) && ld % q == 0 && s1 % q == 0 && s2 % q == 0;
  };
  p.vecA = vec_ok(g.A[0], g.A[1], g.A[2], g.lda, g.sA1, g.sA2, !g.transA);
  p.vecB = vec_ok(g.B[0], g.B[1], g.B[2], g.ldb, g.sB1, g.sB2, g.transB != 0);
  // Fast path: every operand row starts 16-byte aligned (both loaders move
  // 16 B chunks) and the problem is at least one tile's worth of work.
  auto fast_ok = [&](const void* x0, const void* x1, const void* x2, int64_t ld, int64_t s1, int64_t s2, int rows_contig, int R) {
    return aligned_to(x0, 16) && aligned_to(x1, 16) && aligned_to(x2, 16) && ld % 8 == 0 && s1 % 8 == 0 && s2 % 8 == 0 &&
           (!rows_contig || ld >= ((R + 7) / 8) * 8);
  };
  if (g.M >= 8 && g.N >= 8 && fast_ok(g.A[0], g.A[1], g.A[2], g.lda, g.sA1, g.sA2, g.transA, g.M) &&
      fast_ok(g.B[0], g.B[1], g.B[2], g.ldb, g.sB1, g.sB2, !g.transB, g.N))
    return 2;
  return 3;
}

static hipError_t launch_prepared(int kind, const Gemm& g, GemmP& p, hipStream_t st) {
  const int nb = g.nb1 * g.nb2;
  if (kind == 0) return hipSuccess;
  if (kind < 0) return hipErrorInvalidValue;
  if (kind == 1) {
    constexpr int BM = 64, BN = 64;
    p.tiles_n = (g.N + BN - 1) / BN;
    p.vecA = p.vecB = 0;
    dim3 grid(p.tiles_n * ((g.M + BM - 1) / BM), nb);
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, 16>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
  }
  if (kind == 2) return launch_gemm_mfma(p, nb, g.allow_splitk, g.force_cfg, g.force_ks, st, g.c_zeroed);
  constexpr int BM = 128, BN = 128;
  p.tiles_n = (g.N + BN - 1) / BN;
  dim3 grid(p.tiles_n * ((g.M + BM - 1) / BM), nb);
  return launch_bf16_cfg<BM, BN, 64, 64>(p, grid, st);
}

// Several single-output products in one launch where that pays (A^T B products with few output
// tiles each: the weight-gradient products of a layer of a small model); otherwise one by one.
hipError_t launch_gemm_group(const Gemm* gs, int n, hipStream_t st) {
  if (n >= 2 && n <= 4) {
    GemmP ps[4];
    bool ok = true;
    for (int i = 0; i < n && ok; ++i) {
      const Gemm& g = gs[i];
      ok = !g.Ct && g.nb1 == 1 && g.nb2 == 1 && g.allow_splitk && g.in_bf16 && g.force_cfg < 0 &&
           (g.c_zeroed || (g.Cadd && g.Cadd == (const float*)g.C)) && prepare_single(g, ps[i]) == 2;
    }
    if (ok) {
      const hipError_t e = launch_gemm_mfma_group(ps, n, st);
      if (e != hipErrorNotSupported) return e;
    }
  }
  for (int i = 0; i < n; ++i) {
    const hipError_t e = launch_gemm(gs[i], st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

static hipError_t launch_gemm_single(const Gemm& g, hipStream_t st) {
  GemmP p;
  const int kind = prepare_single(g, p);
  return launch_prepared(kind, g, p, st);
}

}  // namespace hf
