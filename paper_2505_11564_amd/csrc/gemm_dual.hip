// Dual-output matrix product: a primal product and its tangent in one launch.
//
//   C   = alpha (A B + A_lo B + A B_lo) + bias   + Cadd
//   C_t = alpha (A_t B + A B_t)         + bias_t + Cadd_t
//
// This is the product rule of every linear map of the Hessian-vector product
// (Y_t = X_t W + X W_t next to Y = X W; dX_t = dY_t W^T + dY W_t^T next to
// dX = dY W^T; the same for each attention product).  Computing both in one
// kernel loads the shared tiles A and B once (five or six operand tiles feed
// four or five products instead of six tiles feeding three in two launches)
// and halves the number of launches.  A_lo / B_lo are the optional low-order
// halves of the bf16 primal operands (primal forward chain only).
//
// Tile 128 x 128 x 32, four wavefronts (64 x 64 each), two accumulator sets in
// AGPRs, operands through the same direct global->LDS pipeline and LDS layouts
// as gemm_mfma_kernel.
#include "gemm_mfma_common.h"

namespace hf {

struct DualP {
  const void *A, *At, *Alo, *B, *Bt, *Blo;
  void *C, *Ct, *Clo;
  const float *Cadd, *Cadd_t;
  const void* bias;
  const float* bias_t;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int nb2;
  int64_t sA1, sA2, sB1, sB2, sC1, sC2;
  float alpha;
  int out_bf16, bias_bf16;
  int klimit, skip_upper;
};

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_dual_kernel(DualP p) {
  constexpr int BM = 128, BN = 128, KT = 32;
  constexpr int TILE = 128 * KT;  // elements per operand tile
  constexpr bool AKC = !TA, BKC = TB;
  constexpr int NI = TILE / 512 / 4;  // load instructions per wave per tile (2)
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  HF_LDS bf16* smem = (HF_LDS bf16*)smem_raw;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const bool hasAlo = p.Alo != nullptr, hasBlo = p.Blo != nullptr;
  const int ntile = 4 + (hasAlo ? 1 : 0) + (hasBlo ? 1 : 0);
  const int stage_el = ntile * TILE;
  // tile slots inside a stage
  const int sA = 0, sAt = TILE, sB = 2 * TILE, sBt = 3 * TILE;
  const int sAlo = 4 * TILE, sBlo = (hasAlo ? 5 : 4) * TILE;

  int tile = blockIdx.x;
  {
    const int nt = gridDim.x;
    if (nt >= 16) {
      const int per = nt / 8, rem = nt % 8;
      const int x = tile % 8, q = tile / 8;
      tile = x * per + min(x, rem) + q;
    }
  }
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  constexpr int GROUP_M = 8;
  int tm, tn;
  {
    const int band = GROUP_M * tiles_n;
    const int g = tile / band, first = g * GROUP_M;
    const int gsz = min(GROUP_M, tiles_m - first);
    const int in_band = tile - g * band;
    tm = first + in_band % gsz;
    tn = in_band / gsz;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  if (p.skip_upper && n0 > m0 + BM - 1) return;
  const int z = blockIdx.y, z1 = z / p.nb2, z2 = z % p.nb2;
  const int64_t offA = z1 * p.sA1 + z2 * p.sA2, offB = z1 * p.sB1 + z2 * p.sB2, offC = z1 * p.sC1 + z2 * p.sC2;
  int kbeg = 0, kend = p.K;
  if (p.klimit == 1) kend = min(p.K, m0 + BM);
  if (p.klimit == 2) kbeg = (m0 / 64) * 64;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  f32x16 accp[2][2], acct[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { accp[i][j][r] = 0.f; acct[i][j][r] = 0.f; }

  const int nfull = (kend - kbeg) / KT;
  const int ktail = (kend - kbeg) - nfull * KT;

  uint32_t voffA[NI], voffB[NI];
  slab_offsets<BM, AKC, KT>(voffA, p.lda, m0, p.M, wave, lane);
  slab_offsets<BN, BKC, KT>(voffB, p.ldb, n0, p.N, wave, lane);
  const int64_t stepA = (AKC ? (int64_t)KT : (int64_t)KT * p.lda) * 2;
  const int64_t stepB = (BKC ? (int64_t)KT : (int64_t)KT * p.ldb) * 2;
  const int64_t a0 = (offA + (AKC ? (int64_t)m0 * p.lda + kbeg : (int64_t)kbeg * p.lda + m0)) * 2;
  const int64_t b0 = (offB + (BKC ? (int64_t)n0 * p.ldb + kbeg : (int64_t)kbeg * p.ldb + n0)) * 2;
  int64_t curA = a0, curB = b0;  // byte offset of the next slab to issue (same for every A- / B-side operand)
  HF_LDS char* const smem_c = (HF_LDS char*)smem;
  const int wave_off = wave * (NI * 1024);
  auto issue = [&](int stage) {
    HF_LDS char* st = smem_c + (int64_t)stage * stage_el * 2 + wave_off;
    slab_issue<NI>((const char*)p.A + curA, voffA, st + sA * 2);
    slab_issue<NI>((const char*)p.At + curA, voffA, st + sAt * 2);
    slab_issue<NI>((const char*)p.B + curB, voffB, st + sB * 2);
    slab_issue<NI>((const char*)p.Bt + curB, voffB, st + sBt * 2);
    if (hasAlo) slab_issue<NI>((const char*)p.Alo + curA, voffA, st + sAlo * 2);
    if (hasBlo) slab_issue<NI>((const char*)p.Blo + curB, voffB, st + sBlo * 2);
    curA += stepA;
    curB += stepB;
  };
  auto compute = [&](int stage) {
    const HF_LDS bf16* st = smem + stage * stage_el;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      bf16x8 a[2], at[2], b[2], bt[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = frag_read<BM, AKC, KT>(st + sA, wm0 + i * 32, kk, lane);
        at[i] = frag_read<BM, AKC, KT>(st + sAt, wm0 + i * 32, kk, lane);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        b[j] = frag_read<BN, BKC, KT>(st + sB, wn0 + j * 32, kk, lane);
        bt[j] = frag_read<BN, BKC, KT>(st + sBt, wn0 + j * 32, kk, lane);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], accp[i][j], 0, 0, 0);
          acct[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[i], b[j], acct[i][j], 0, 0, 0);
          acct[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bt[j], acct[i][j], 0, 0, 0);
        }
      if (hasAlo) {
        bf16x8 al[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) al[i] = frag_read<BM, AKC, KT>(st + sAlo, wm0 + i * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], b[j], accp[i][j], 0, 0, 0);
      }
      if (hasBlo) {
        bf16x8 bl[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) bl[j] = frag_read<BN, BKC, KT>(st + sBlo, wn0 + j * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bl[j], accp[i][j], 0, 0, 0);
      }
    }
  };

  // two LDS stages: the loads of slab i+1 fly while slab i is multiplied
  if (nfull > 0) issue(0);
  for (int i0 = 0; i0 < nfull; i0 += 2) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int i = i0 + s;
      if (i < nfull) {
        HF_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (i + 1 < nfull) issue(s ^ 1);
        compute(s);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  if (ktail > 0) {
    const int k0 = kbeg + nfull * KT;
    __syncthreads();
    auto guarded = [&](const void* X, int slot, bool isA) {
      if (isA) slab_guarded<BM, AKC, KT>((const bf16*)X + offA, p.lda, m0, k0, p.M, kend, smem + slot, t);
      else slab_guarded<BN, BKC, KT>((const bf16*)X + offB, p.ldb, n0, k0, p.N, kend, smem + slot, t);
    };
    guarded(p.A, sA, true); guarded(p.At, sAt, true); guarded(p.B, sB, false); guarded(p.Bt, sBt, false);
    if (hasAlo) guarded(p.Alo, sAlo, true);
    if (hasBlo) guarded(p.Blo, sBlo, false);
    __syncthreads();
    compute(0);
  }

  // epilogue: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int gn = n0 + wn0 + j * 32 + (lane & 31);
    if (gn >= p.N) continue;
    float bp = 0.f, bt = 0.f;
    if (p.bias) bp = p.bias_bf16 ? (float)((const bf16*)p.bias)[gn] : ((const float*)p.bias)[gn];
    if (p.bias_t) bt = p.bias_t[gn];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (gm >= p.M) continue;
        const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
        float vp = p.alpha * accp[i][j][r] + bp;
        float vt = p.alpha * acct[i][j][r] + bt;
        if (p.Cadd) vp += p.Cadd[ci];
        if (p.Cadd_t) vt += p.Cadd_t[ci];
        if (p.out_bf16) {
          const bf16 hi = (bf16)vp;
          ((bf16*)p.C)[ci] = hi;
          if (p.Clo) ((bf16*)p.Clo)[ci] = (bf16)(vp - (float)hi);
          ((bf16*)p.Ct)[ci] = (bf16)vt;
        } else {
          ((float*)p.C)[ci] = vp;
          ((float*)p.Ct)[ci] = vt;
        }
      }
    }
  }
}

template <bool TA, bool TB>
static hipError_t launch_dual_one(const DualP& p, dim3 grid, int smem, hipStream_t st) {
  static bool attr_done = false;
  auto kern = gemm_dual_kernel<TA, TB>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 6 * 128 * 32 * 2 * 2);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
  return hipGetLastError();
}

// g.Ct != nullptr.  Returns hipErrorNotSupported when the description does not
// fit the canonical form; the caller then issues two single-output products.
hipError_t launch_gemm_dual(const Gemm& g, hipStream_t st) {
  DualP p;
  p.A = g.A[0]; p.B = g.B[0]; p.At = g.At; p.Bt = g.Bt; p.Alo = nullptr; p.Blo = nullptr;
  if (!g.At || !g.Bt) return hipErrorNotSupported;
  // optional low-order terms must be (A_lo, B) and (A, B_lo)
  for (int i = 1; i < 3; ++i) {
    if (!g.A[i]) continue;
    if (g.B[i] == g.B[0] && g.A[i] != g.A[0] && !p.Alo) p.Alo = g.A[i];
    else if (g.A[i] == g.A[0] && g.B[i] != g.B[0] && !p.Blo) p.Blo = g.B[i];
    else return hipErrorNotSupported;
  }
  p.C = g.C; p.Ct = g.Ct; p.Clo = g.C_lo; p.Cadd = g.Cadd; p.Cadd_t = g.Cadd_t; p.bias = g.bias; p.bias_t = g.bias_t;
  p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.nb2 = g.nb2;
  p.sA1 = g.sA1; p.sA2 = g.sA2; p.sB1 = g.sB1; p.sB2 = g.sB2; p.sC1 = g.sC1; p.sC2 = g.sC2;
  p.alpha = g.alpha; p.out_bf16 = g.out_bf16; p.bias_bf16 = 1; p.klimit = g.klimit; p.skip_upper = g.skip_upper;
  const int ntile = 4 + (p.Alo ? 1 : 0) + (p.Blo ? 1 : 0);
  const int smem = 2 * ntile * 128 * 32 * 2;
  const int64_t nt = ((g.M + 127) / 128) * (int64_t)((g.N + 127) / 128);
  dim3 grid((unsigned)nt, (unsigned)(g.nb1 * g.nb2), 1);
  if (!g.transA && !g.transB) return launch_dual_one<false, false>(p, grid, smem, st);
  if (!g.transA && g.transB) return launch_dual_one<false, true>(p, grid, smem, st);
  if (g.transA && !g.transB) return launch_dual_one<true, false>(p, grid, smem, st);
  return launch_dual_one<true, true>(p, grid, smem, st);
}

}  // namespace hf
