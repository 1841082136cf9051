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

// NT: operand tiles per stage: 4 (A, A_t, B, B_t), 5 (+ A_lo) or 6 (+ A_lo, B_lo).
template <bool TA, bool TB, int NT>
__global__ __launch_bounds__(256) void gemm_dual_kernel(DualP p) {
  constexpr int BM = 128, BN = 128, KT = 32;
  constexpr int TILE = 128 * KT;  // elements per operand tile
  constexpr bool AKC = !TA, BKC = TB;
  constexpr int NI = TILE / 512 / 4;  // load instructions per wave per tile (2)
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  HF_LDS bf16* smem = (HF_LDS bf16*)smem_raw;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  constexpr bool hasAlo = NT >= 5, hasBlo = NT >= 6;
  constexpr int stage_el = NT * TILE;
  // tile slots inside a stage
  constexpr int sA = 0, sAt = TILE, sB = 2 * TILE, sBt = 3 * TILE, sAlo = 4 * TILE, sBlo = 5 * TILE;

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
  // per-lane LDS byte addresses of the fragments inside an operand tile
  constexpr int NKK = KT / 16;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  uint32_t adA[AKC ? NKK : 1][2], adB[BKC ? NKK : 1][2];
#pragma unroll
  for (int kk = 0; kk < (AKC ? NKK : 1); ++kk)
#pragma unroll
    for (int i = 0; i < 2; ++i) adA[kk][i] = lds0 + frag_addr<BM, AKC, KT>(wm0 + i * 32, kk, lane);
#pragma unroll
  for (int kk = 0; kk < (BKC ? NKK : 1); ++kk)
#pragma unroll
    for (int j = 0; j < 2; ++j) adB[kk][j] = lds0 + frag_addr<BN, BKC, KT>(wn0 + j * 32, kk, lane);

  // Products of the slab in stage S; the fragments of k-step kk+1 are requested
  // as soon as those of step kk have landed (explicit reads and waits, see
  // gemm_mfma_common.h).
  auto compute = [&](auto stage_c) {
    constexpr int S = decltype(stage_c)::value;
    Frag<AKC> a[2][2], at[2][2], al[2][2];
    Frag<BKC> b[2][2], bt[2][2], bl[2][2];
    auto request = [&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      constexpr int offA = S * stage_el * 2 + (AKC ? 0 : kk * 16 * BM * 2);
      constexpr int offB = S * stage_el * 2 + (BKC ? 0 : kk * 16 * BN * 2);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[kk & 1][i].template read<offA + sA * 2, 4 * BM * 2>(adA[AKC ? kk : 0][i]);
        at[kk & 1][i].template read<offA + sAt * 2, 4 * BM * 2>(adA[AKC ? kk : 0][i]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        b[kk & 1][j].template read<offB + sB * 2, 4 * BN * 2>(adB[BKC ? kk : 0][j]);
        bt[kk & 1][j].template read<offB + sBt * 2, 4 * BN * 2>(adB[BKC ? kk : 0][j]);
      }
      if constexpr (hasAlo) {
#pragma unroll
        for (int i = 0; i < 2; ++i) al[kk & 1][i].template read<offA + sAlo * 2, 4 * BM * 2>(adA[AKC ? kk : 0][i]);
      }
      if constexpr (hasBlo) {
#pragma unroll
        for (int j = 0; j < 2; ++j) bl[kk & 1][j].template read<offB + sBlo * 2, 4 * BN * 2>(adB[BKC ? kk : 0][j]);
      }
    };
    request(std::integral_constant<int, 0>{});
    static_for<NKK>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value, c = kk & 1;
      __builtin_amdgcn_sched_barrier(0);
      lds_wait_all();
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[c][i].tie(); at[c][i].tie(); b[c][i].tie(); bt[c][i].tie();
        if constexpr (hasAlo) al[c][i].tie();
        if constexpr (hasBlo) bl[c][i].tie();
      }
      if constexpr (kk + 1 < NKK) request(std::integral_constant<int, kk + 1>{});
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i].get(), b[c][j].get(), accp[i][j], 0, 0, 0);
          acct[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[c][i].get(), b[c][j].get(), acct[i][j], 0, 0, 0);
          acct[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i].get(), bt[c][j].get(), acct[i][j], 0, 0, 0);
          if constexpr (hasAlo)
            accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[c][i].get(), b[c][j].get(), accp[i][j], 0, 0, 0);
          if constexpr (hasBlo)
            accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i].get(), bl[c][j].get(), accp[i][j], 0, 0, 0);
        }
    });
  };

  // two LDS stages: the loads of slab i+1 fly while slab i is multiplied
  if (nfull > 0) issue(0);
  for (int i0 = 0; i0 < nfull; i0 += 2) {
    static_for<2>([&](auto s_c) {
      constexpr int s = decltype(s_c)::value;
      const int i = i0 + s;
      if (i < nfull) {
        HF_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (i + 1 < nfull) issue(s ^ 1);
        compute(s_c);
        __builtin_amdgcn_sched_barrier(0);
      }
    });
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
    compute(std::integral_constant<int, 0>{});
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

template <bool TA, bool TB, int NT>
static hipError_t launch_dual_nt(const DualP& p, dim3 grid, hipStream_t st) {
  static bool attr_done = false;
  auto kern = gemm_dual_kernel<TA, TB, NT>;
  constexpr int smem = 2 * NT * 128 * 32 * 2;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
  return hipGetLastError();
}
template <bool TA, bool TB>
static hipError_t launch_dual_one(const DualP& p, dim3 grid, hipStream_t st) {
  if (p.Blo) return launch_dual_nt<TA, TB, 6>(p, grid, st);
  if (p.Alo) return launch_dual_nt<TA, TB, 5>(p, grid, st);
  return launch_dual_nt<TA, TB, 4>(p, grid, st);
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
  if (p.Blo && !p.Alo) return hipErrorNotSupported;
  const int64_t nt = ((g.M + 127) / 128) * (int64_t)((g.N + 127) / 128);
  dim3 grid((unsigned)nt, (unsigned)(g.nb1 * g.nb2), 1);
  if (!g.transA && !g.transB) return launch_dual_one<false, false>(p, grid, st);
  if (!g.transA && g.transB) return launch_dual_one<false, true>(p, grid, st);
  if (g.transA && !g.transB) return launch_dual_one<true, false>(p, grid, st);
  return launch_dual_one<true, true>(p, grid, st);
}

}  // namespace hf
