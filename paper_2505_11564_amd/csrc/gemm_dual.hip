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
  int nb2, divB;
  int64_t sA1, sA2, sB1, sB2, sC1, sC2;
  int64_t sCk;         // k-split (gridDim.z > 1): elements between the partial results of consecutive splits
  float alpha;
  int out_bf16, bias_bf16;
  int klimit, skip_upper;
  int epi;             // attention epilogue (EPI_* of hf_internal.h)
  int vec;             // C, Ct, Clo, E0, E1, Cadd, Cadd_t rows allow 16-byte accesses
  int NP;              // parts per row of `part`
  float* part;
  const float* rstat;
  const void *E0, *E1;
};

// NT: operand tiles per stage: 4 (A, A_t, B, B_t), 5 (+ A_lo) or 6 (+ A_lo, B_lo).
// NS: LDS stages (slabs in flight + 1).  The attention products have a k of one
// head dimension (2-4 slabs), so their variants keep every slab in flight.
// EPI: epilogue (EPI_* of hf_internal.h), compile-time.
template <bool TA, bool TB, int NT, int NS, int EPI>
__global__ __launch_bounds__(256, (EPI != EPI_NONE && NT == 4 && NS == 2 ? 2 : 1)) void gemm_dual_kernel(DualP p) {
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

  // Blocks are dealt round-robin to the 8 XCDs in launch order (x fastest).
  //  * Batched causal products (the attention scores): XCD c takes whole batch entries
  //    (heads) c, c + 8, ...  Every XCD then holds the same number of tiles on or below the
  //    diagonal (a column-wise split leaves XCD 0 with 8 times the work of XCD 7 at 8 x 8
  //    tiles), and a head's Q and K tiles are fetched by one L2 only.
  //  * Otherwise each XCD gets a contiguous range of tiles, so that neighbours share
  //    operand rows in its L2.
  int tile = blockIdx.x, z = blockIdx.y;
  {
    const int nt = gridDim.x;
    if (p.skip_upper && (gridDim.y & 7) == 0) {
      // launch-order index L: XCD L % 8, its r-th block; XCD c walks the tiles of batch entry c,
      // then of entry c + 8, ...
      const int L = blockIdx.y * nt + blockIdx.x, r = L >> 3;
      z = (r / nt) * 8 + (L & 7);
      tile = r % nt;
    } else if (nt >= 16) {
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
  const int z1 = z / p.nb2, z2 = z % p.nb2;
  // k-split (plain products only): split blockIdx.z takes a contiguous share of the full slabs and
  // writes its partial sums to its own slice of C / Ct; the last split also takes the ragged tail
  const int ksp = blockIdx.z, nks = gridDim.z;
  const int64_t offA = z1 * p.sA1 + z2 * p.sA2, offB = z1 * p.sB1 + (z2 / p.divB) * p.sB2,
                offC = z1 * p.sC1 + z2 * p.sC2 + ksp * p.sCk;
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

  const int nfull_all = (kend - kbeg) / KT;
  const int ktail = (ksp == nks - 1) ? (kend - kbeg) - nfull_all * KT : 0;
  const int it0 = (int)((int64_t)nfull_all * ksp / nks), nfull = (int)((int64_t)nfull_all * (ksp + 1) / nks) - it0;

  uint32_t voffA[NI], voffB[NI];
  slab_offsets<BM, AKC, KT>(voffA, p.lda, m0, p.M, wave, lane);
  slab_offsets<BN, BKC, KT>(voffB, p.ldb, n0, p.N, wave, lane);
  const int64_t stepA = (AKC ? (int64_t)KT : (int64_t)KT * p.lda) * 2;
  const int64_t stepB = (BKC ? (int64_t)KT : (int64_t)KT * p.ldb) * 2;
  const int64_t a0 = (offA + (AKC ? (int64_t)m0 * p.lda + kbeg : (int64_t)kbeg * p.lda + m0)) * 2 + it0 * stepA;
  const int64_t b0 = (offB + (BKC ? (int64_t)n0 * p.ldb + kbeg : (int64_t)kbeg * p.ldb + n0)) * 2 + it0 * stepB;
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

  // One wave per SIMD issues everything in order, so (as in gemm_mfma_kernel) the fragment reads
  // of the next k-step and the loads of a later slab are dealt out between the matrix
  // instructions, and the hand-over barrier of a slab sits before its last k-step: the matrix
  // instructions of that k-step (fragments already in registers) cover the first reads of the
  // next slab.  Fragment registers: two sets alternating by k-step, alive across slabs.
  static_assert(NKK == 2, "two k-steps per slab");
  constexpr int NFR = 2 * NT;       // fragments per k-step: two per operand tile
  constexpr int MQ = 4 * (NT - 1);  // matrix instructions per k-step (12, 16 or 20)
  constexpr int NLOAD = NT * NI;    // load instructions per wave per slab
  static_assert(NLOAD <= MQ, "at most one load per matrix instruction");
  Frag<AKC> fa[2][2], fat[2][2], fal[2][2];
  Frag<BKC> fb[2][2], fbt[2][2], fbl[2][2];
  // fragment f of k-step kk of the slab in stage S (+ run-time byte offset): operand tile f / 2
  // in the order A, A_t, B, B_t, A_lo, B_lo; row block f % 2
  auto request_one = [&](auto stage_c, auto kk_c, auto f_c, uint32_t dyn) {
    constexpr int S = decltype(stage_c)::value, kk = decltype(kk_c)::value, f = decltype(f_c)::value;
    constexpr int tl = f / 2, ix = f % 2, c = kk & 1;
    constexpr int offA = S * stage_el * 2 + (AKC ? 0 : kk * 16 * BM * 2);
    constexpr int offB = S * stage_el * 2 + (BKC ? 0 : kk * 16 * BN * 2);
    const uint32_t aA = adA[AKC ? kk : 0][ix] + dyn, aB = adB[BKC ? kk : 0][ix] + dyn;
    if constexpr (tl == 0) fa[c][ix].template read<offA + sA * 2, 4 * BM * 2>(aA);
    else if constexpr (tl == 1) fat[c][ix].template read<offA + sAt * 2, 4 * BM * 2>(aA);
    else if constexpr (tl == 2) fb[c][ix].template read<offB + sB * 2, 4 * BN * 2>(aB);
    else if constexpr (tl == 3) fbt[c][ix].template read<offB + sBt * 2, 4 * BN * 2>(aB);
    else if constexpr (tl == 4) fal[c][ix].template read<offA + sAlo * 2, 4 * BM * 2>(aA);
    else fbl[c][ix].template read<offB + sBlo * 2, 4 * BN * 2>(aB);
  };
  auto request = [&](auto stage_c, auto kk_c, uint32_t dyn) {
    static_for<NFR>([&](auto f_c) { request_one(stage_c, kk_c, f_c, dyn); });
  };
  auto landed = [&](auto kk_c) {
    constexpr int c = decltype(kk_c)::value & 1;
    __builtin_amdgcn_sched_barrier(0);
    lds_wait_all();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      fa[c][i].tie(); fat[c][i].tie(); fb[c][i].tie(); fbt[c][i].tie();
      if constexpr (hasAlo) fal[c][i].tie();
      if constexpr (hasBlo) fbl[c][i].tie();
    }
  };
  // load number l of the slab at the issue cursor, into LDS stage S
  auto issue_one = [&](auto stage_c, auto l_c) {
    constexpr int S = decltype(stage_c)::value, l = decltype(l_c)::value, tl = l / NI, j = l % NI;
    HF_LDS char* st = smem_c + S * stage_el * 2 + wave_off + j * 1024;
    const void* X = tl == 0 ? p.A : tl == 1 ? p.At : tl == 2 ? p.B : tl == 3 ? p.Bt : tl == 4 ? p.Alo : p.Blo;
    constexpr bool onA = (tl == 0 || tl == 1 || tl == 4);
    constexpr int slot = tl == 0 ? sA : tl == 1 ? sAt : tl == 2 ? sB : tl == 3 ? sBt : tl == 4 ? sAlo : sBlo;
    const char* src = (const char*)X + (onA ? curA + voffA[j] : curB + voffB[j]);
    __builtin_amdgcn_global_load_lds((const void*)src, (HF_LDS void*)(st + slot * 2), 16, 0, 0);
  };
  // The MQ matrix instructions of k-step kk, in the order A B, A_t B, A B_t, A_lo B, A B_lo (each over
  // the four 32 x 32 tiles, so that the two updates of an accumulator are four instructions apart).
  // With REQ the fragment reads of k-step RK of stage RS follow the first MQ/2 of them; with ISSUE
  // (PH = 0: first k-step of a pipeline iteration) one load of the slab at the cursor follows each
  // of the first NLOAD, into stage LS.
  auto mfmas = [&](auto kk_c, auto ph_c, auto issue_c, auto ls_c, auto req_c, auto rs_c, auto rk_c, uint32_t dyn) {
    constexpr int c = decltype(kk_c)::value & 1, PH = decltype(ph_c)::value;
    constexpr bool ISSUE = decltype(issue_c)::value, REQ = decltype(req_c)::value;
    static_for<MQ>([&](auto q_c) {
      constexpr int q = decltype(q_c)::value, ty = q / 4, i = (q % 4) / 2, j = q % 2;
      if constexpr (ty == 0) accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i].get(), fb[c][j].get(), accp[i][j], 0, 0, 0);
      else if constexpr (ty == 1) acct[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fat[c][i].get(), fb[c][j].get(), acct[i][j], 0, 0, 0);
      else if constexpr (ty == 2) acct[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i].get(), fbt[c][j].get(), acct[i][j], 0, 0, 0);
      else if constexpr (ty == 3) accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fal[c][i].get(), fb[c][j].get(), accp[i][j], 0, 0, 0);
      else accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i].get(), fbl[c][j].get(), accp[i][j], 0, 0, 0);
      if constexpr (REQ) {
        static_for<NFR>([&](auto f_c) {
          constexpr int f = decltype(f_c)::value;
          if constexpr ((f * MQ) / (2 * NFR) == q) request_one(rs_c, rk_c, f_c, dyn);
        });
      }
      if constexpr (ISSUE && PH == 0 && q < NLOAD) issue_one(ls_c, q_c);
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  // One pipeline iteration, entered after the barrier that publishes the slab in stage S and
  // frees stage LS: last k-step of the previous slab (covering this slab's first reads and,
  // with ISSUE, the loads of the slab NS-1 after this one), then this slab's first k-step.
  auto iteration = [&](auto stage_c, auto issue_c, auto ls_c, uint32_t dyn) {
    mfmas(I1{}, I0{}, issue_c, ls_c, std::true_type{}, stage_c, I0{}, dyn);
    landed(I0{});
    mfmas(I0{}, I1{}, issue_c, ls_c, std::true_type{}, stage_c, I1{}, dyn);
    landed(I1{});
    if constexpr (decltype(issue_c)::value) { curA += stepA; curB += stepB; }
  };
  // at most x slabs of loads may still be in flight (vmcnt counts instructions)
  auto wait_slabs = [&](int x) {
    if (x >= 3) HF_WAIT_VMCNT(3 * NLOAD);
    else if (x == 2) HF_WAIT_VMCNT(2 * NLOAD);
    else if (x == 1) HF_WAIT_VMCNT(NLOAD);
    else HF_WAIT_VMCNT(0);
  };
  // a whole slab already in LDS stage 0 (prologue, ragged tail): both k-steps
  auto first_slab = [&](auto last_c) {
    request(I0{}, I0{}, 0u);
    landed(I0{});
    mfmas(I0{}, I1{}, std::false_type{}, I0{}, std::true_type{}, I0{}, I1{}, 0u);
    landed(I1{});
    if constexpr (decltype(last_c)::value)
      mfmas(I1{}, I1{}, std::false_type{}, I0{}, std::false_type{}, I0{}, I0{}, 0u);
  };

#pragma unroll
  for (int s0 = 0; s0 < NS; ++s0)
    if (s0 < nfull) issue(s0);
  if (nfull > 0) {
    wait_slabs(min(NS, nfull) - 1);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    first_slab(std::false_type{});
    // iterations that still have a slab to prefetch (stage numbers are compile-time constants),
    // then the remaining ones with the stage as a run-time offset
    const int n_issue = max(0, nfull - NS);
    for (int j0 = 0; j0 < n_issue; j0 += NS) {
      static_for<NS>([&](auto s_c) {
        constexpr int s = decltype(s_c)::value;
        if (j0 + s < n_issue) {
          HF_WAIT_VMCNT((NS - 2) * NLOAD);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          iteration(std::integral_constant<int, (s + 1) % NS>{}, std::true_type{}, s_c, 0u);
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    }
    for (int j = n_issue; j + 1 < nfull; ++j) {
      wait_slabs(min(nfull - 2 - j, NS - 2));
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      iteration(I0{}, std::false_type{}, I0{}, (uint32_t)(((j + 1) % NS) * (stage_el * 2)));
      __builtin_amdgcn_sched_barrier(0);
    }
    mfmas(I1{}, I1{}, std::false_type{}, I0{}, std::false_type{}, I0{}, I0{}, 0u);
  }
  if constexpr (EPI != EPI_NONE && NT == 4) {
    // Low-order primal terms A_lo B and A B_lo (forward scores) as further
    // k-slabs of two operand tiles each, through the same two stages: the
    // kernel stays at four tiles per stage and two resident blocks per CU.
    static_assert(NS == 2, "the low-order loops assume two stages");
    auto lo_loop = [&](const void* Ax, const void* Bx) {
      int64_t cA = a0, cB = b0;
      auto issue_lo = [&](int stage) {
        HF_LDS char* st = smem_c + (int64_t)stage * stage_el * 2 + wave_off;
        slab_issue<NI>((const char*)Ax + cA, voffA, st + sA * 2);
        slab_issue<NI>((const char*)Bx + cB, voffB, st + sB * 2);
        cA += stepA;
        cB += stepB;
      };
      auto compute_lo = [&](auto stage_c) {
        constexpr int S = decltype(stage_c)::value;
        Frag<AKC> a[2][2];
        Frag<BKC> b[2][2];
        auto request = [&](auto kk_c) {
          constexpr int kk = decltype(kk_c)::value;
          constexpr int offA = S * stage_el * 2 + (AKC ? 0 : kk * 16 * BM * 2);
          constexpr int offB = S * stage_el * 2 + (BKC ? 0 : kk * 16 * BN * 2);
#pragma unroll
          for (int i = 0; i < 2; ++i) a[kk & 1][i].template read<offA + sA * 2, 4 * BM * 2>(adA[AKC ? kk : 0][i]);
#pragma unroll
          for (int j = 0; j < 2; ++j) b[kk & 1][j].template read<offB + sB * 2, 4 * BN * 2>(adB[BKC ? kk : 0][j]);
        };
        request(std::integral_constant<int, 0>{});
        static_for<NKK>([&](auto kk_c) {
          constexpr int kk = decltype(kk_c)::value, c = kk & 1;
          __builtin_amdgcn_sched_barrier(0);
          lds_wait_all();
#pragma unroll
          for (int i = 0; i < 2; ++i) { a[c][i].tie(); b[c][i].tie(); }
          if constexpr (kk + 1 < NKK) request(std::integral_constant<int, kk + 1>{});
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              accp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i].get(), b[c][j].get(), accp[i][j], 0, 0, 0);
        });
      };
      __builtin_amdgcn_s_barrier();  // every wave is done with both stages
      if (nfull > 0) issue_lo(0);
      for (int i0 = 0; i0 < nfull; i0 += 2) {
        static_for<2>([&](auto s_c) {
          constexpr int s = decltype(s_c)::value;
          const int i = i0 + s;
          if (i < nfull) {
            HF_WAIT_VMCNT(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            if (i + 1 < nfull) issue_lo(s ^ 1);
            compute_lo(s_c);
            __builtin_amdgcn_sched_barrier(0);
          }
        });
      }
    };
    if (p.Alo) lo_loop(p.Alo, p.B);
    if (p.Blo) lo_loop(p.A, p.Blo);
  }
  if (ktail > 0) {
    const int k0 = kbeg + nfull_all * KT;
    __syncthreads();
    auto guarded = [&](const void* X, int slot, bool isA) {
      if (isA) slab_guarded<BM, AKC, KT>((const bf16*)X + offA, p.lda, m0, k0, p.M, kend, smem + slot, t);
      else slab_guarded<BN, BKC, KT>((const bf16*)X + offB, p.ldb, n0, k0, p.N, kend, smem + slot, t);
    };
    guarded(p.A, sA, true); guarded(p.At, sAt, true); guarded(p.B, sB, false); guarded(p.Bt, sBt, false);
    if (hasAlo) guarded(p.Alo, sAlo, true);
    if (hasBlo) guarded(p.Blo, sBlo, false);
    __syncthreads();
    first_slab(std::true_type{});
  }

  // ---- epilogue -------------------------------------------------------------
  // An accumulator tile holds, per lane, column (lane & 31) and rows
  // 8*(r/4) + 4*(lane/32) + r%4.  Each wave stages 32 rows x 64 columns of both
  // results in LDS and walks them row-wise, 8 consecutive columns per lane (8
  // lanes per row), so that memory is touched 16 bytes at a time and the row
  // reductions of the attention epilogues are three cross-lane steps.
  constexpr int LDW = 64 + 4;
  HF_LDS float* stgP = (HF_LDS float*)smem + wave * (2 * 32 * LDW);
  HF_LDS float* stgT = stgP + 32 * LDW;
  float bp[2], bt[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int gn = n0 + wn0 + j * 32 + (lane & 31);
    bp[j] = 0.f; bt[j] = 0.f;
    if (gn < p.N) {
      if (p.bias) bp[j] = p.bias_bf16 ? (float)((const bf16*)p.bias)[gn] : ((const float*)p.bias)[gn];
      if (p.bias_t) bt[j] = p.bias_t[gn];
    }
  }
  constexpr int epi = EPI;
  const bool causal = p.skip_upper != 0;
  const int64_t zrow0 = (int64_t)z * p.M;
  auto xor8_sum = [](float v) { v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64); return v; };
  auto xor8_max = [](float v) {
    v = fmaxf(v, __shfl_xor(v, 1, 64)); v = fmaxf(v, __shfl_xor(v, 2, 64)); v = fmaxf(v, __shfl_xor(v, 4, 64));
    return v;
  };
  auto store8_bf16 = [&](void* X, int64_t ci, int gn, const float (&v)[8]) {
    if (p.vec && gn + 8 <= p.N) {
      bf16 o[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = (bf16)v[q];
      *(uint4*)((bf16*)X + ci) = *(const uint4*)o;
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (gn + q < p.N) ((bf16*)X)[ci + q] = (bf16)v[q];
    }
  };
  // Inputs of the attention epilogues (row statistics, P and P_t), requested
  // together before the staging so that one round trip covers all of them.  Epilogue pass (i, ps) of a lane
  // covers row m0 + wm0 + 32 i + 8 ps + lane/8, columns n0 + wn0 + 8 (lane%8) .. +7.
  // These variants require 16-byte aligned rows and N % 8 == 0 (checked by the
  // launcher), so a lane's 8 columns are valid together.
  constexpr bool kNeedStat = EPI == EPI_FWD_SOFTMAX || EPI == EPI_BWD_DS;
  constexpr bool kNeedP = EPI == EPI_BWD_STATS || EPI == EPI_BWD_DS;
  float pre_s[kNeedStat ? 8 : 1][3];
  uint4 pre_p[kNeedP ? 8 : 1], pre_pt[kNeedP ? 8 : 1];
  if constexpr (kNeedStat || kNeedP) {
    const int64_t zr = (int64_t)z * p.M;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int gm = m0 + wm0 + (e >> 2) * 32 + (e & 3) * 8 + (lane >> 3), gn = n0 + wn0 + (lane & 7) * 8;
      if constexpr (kNeedStat) {
        pre_s[e][0] = 0.f; pre_s[e][1] = 0.f; pre_s[e][2] = 0.f;
        if (gm < p.M) {
          const float* rs = p.rstat + (zr + gm) * 3;
          pre_s[e][0] = rs[0]; pre_s[e][1] = rs[1];
          if (EPI == EPI_FWD_SOFTMAX) pre_s[e][2] = rs[2];
        }
      }
      if constexpr (kNeedP) {
        pre_p[e] = make_uint4(0, 0, 0, 0); pre_pt[e] = pre_p[e];
        if (gm < p.M && gn < p.N) {
          const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
          pre_p[e] = *(const uint4*)((const bf16*)p.E0 + ci);
          pre_pt[e] = *(const uint4*)((const bf16*)p.E1 + ci);
        }
      }
    }
  }

  __syncthreads();  // every wave is done reading operand tiles
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int idx = ((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * LDW + j * 32 + (lane & 31);
        stgP[idx] = p.alpha * accp[i][j][r] + bp[j];
        stgT[idx] = p.alpha * acct[i][j][r] + bt[j];
      }
    __syncthreads();
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int row = ps * 8 + (lane >> 3), ch = lane & 7;
      const int gm = m0 + wm0 + i * 32 + row, gn = n0 + wn0 + ch * 8;
      const bool rowok = gm < p.M;
      typedef float f32x4_t __attribute__((ext_vector_type(4)));
      float vp[8], vt[8];
      {
        const f32x4_t a0 = *(const HF_LDS f32x4_t*)(stgP + row * LDW + ch * 8), a1 = *(const HF_LDS f32x4_t*)(stgP + row * LDW + ch * 8 + 4);
        const f32x4_t b0 = *(const HF_LDS f32x4_t*)(stgT + row * LDW + ch * 8), b1 = *(const HF_LDS f32x4_t*)(stgT + row * LDW + ch * 8 + 4);
        vp[0] = a0.x; vp[1] = a0.y; vp[2] = a0.z; vp[3] = a0.w; vp[4] = a1.x; vp[5] = a1.y; vp[6] = a1.z; vp[7] = a1.w;
        vt[0] = b0.x; vt[1] = b0.y; vt[2] = b0.z; vt[3] = b0.w; vt[4] = b1.x; vt[5] = b1.y; vt[6] = b1.z; vt[7] = b1.w;
      }
      const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
      bool ok[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) ok[q] = rowok && gn + q < p.N && (!causal || gn + q <= gm);
      if constexpr (epi == EPI_NONE) {
        if (!rowok || gn >= p.N) continue;
        if (p.vec && gn + 8 <= p.N) {
          if (p.Cadd) {
            const float4 c0 = *(const float4*)(p.Cadd + ci), c1 = *(const float4*)(p.Cadd + ci + 4);
            vp[0] += c0.x; vp[1] += c0.y; vp[2] += c0.z; vp[3] += c0.w; vp[4] += c1.x; vp[5] += c1.y; vp[6] += c1.z; vp[7] += c1.w;
          }
          if (p.Cadd_t) {
            const float4 c0 = *(const float4*)(p.Cadd_t + ci), c1 = *(const float4*)(p.Cadd_t + ci + 4);
            vt[0] += c0.x; vt[1] += c0.y; vt[2] += c0.z; vt[3] += c0.w; vt[4] += c1.x; vt[5] += c1.y; vt[6] += c1.z; vt[7] += c1.w;
          }
          if (p.out_bf16) {
            store8_bf16(p.C, ci, gn, vp);
            if (p.Clo) {
              float lo[8];
#pragma unroll
              for (int q = 0; q < 8; ++q) lo[q] = vp[q] - (float)(bf16)vp[q];
              store8_bf16(p.Clo, ci, gn, lo);
            }
            store8_bf16(p.Ct, ci, gn, vt);
          } else {
            *(float4*)((float*)p.C + ci) = make_float4(vp[0], vp[1], vp[2], vp[3]);
            *(float4*)((float*)p.C + ci + 4) = make_float4(vp[4], vp[5], vp[6], vp[7]);
            *(float4*)((float*)p.Ct + ci) = make_float4(vt[0], vt[1], vt[2], vt[3]);
            *(float4*)((float*)p.Ct + ci + 4) = make_float4(vt[4], vt[5], vt[6], vt[7]);
          }
        } else {
          for (int q = 0; q < 8; ++q) {
            if (gn + q >= p.N) break;
            float x = vp[q], xt = vt[q];
            if (p.Cadd) x += p.Cadd[ci + q];
            if (p.Cadd_t) xt += p.Cadd_t[ci + q];
            if (p.out_bf16) {
              const bf16 hi = (bf16)x;
              ((bf16*)p.C)[ci + q] = hi;
              if (p.Clo) ((bf16*)p.Clo)[ci + q] = (bf16)(x - (float)hi);
              ((bf16*)p.Ct)[ci + q] = (bf16)xt;
            } else {
              ((float*)p.C)[ci + q] = x;
              ((float*)p.Ct)[ci + q] = xt;
            }
          }
        }
      } else if constexpr (epi == EPI_FWD_STATS) {
        float m = -INFINITY;
#pragma unroll
        for (int q = 0; q < 8; ++q) if (ok[q]) m = fmaxf(m, vp[q]);
        m = xor8_max(m);
        float l = 0.f, rr = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q)
          if (ok[q]) { const float e = __expf(vp[q] - m); l += e; rr += e * vt[q]; }
        l = xor8_sum(l);
        rr = xor8_sum(rr);
        if (ch == 0 && rowok && n0 + wn0 < p.N) {
          float* dst = p.part + ((zrow0 + gm) * p.NP + (n0 + wn0) / 64) * 3;
          dst[0] = m; dst[1] = l; dst[2] = rr;
        }
      } else if constexpr (epi == EPI_FWD_SOFTMAX) {
        const float m = pre_s[i * 4 + ps][0], inv = pre_s[i * 4 + ps][1], rbar = pre_s[i * 4 + ps][2];
        if (!rowok || gn >= p.N) continue;
        float P[8], Pl[8], Pt[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          P[q] = ok[q] ? __expf(vp[q] - m) * inv : 0.f;
          Pt[q] = ok[q] ? P[q] * (vt[q] - rbar) : 0.f;
          Pl[q] = P[q] - (float)(bf16)P[q];
        }
        store8_bf16(p.C, ci, gn, P);
        if (p.Clo) store8_bf16(p.Clo, ci, gn, Pl);
        store8_bf16(p.Ct, ci, gn, Pt);
      } else {
        float P[8], Pt[8];
        {
          const uint4 u = pre_p[kNeedP ? i * 4 + ps : 0], w = pre_pt[kNeedP ? i * 4 + ps : 0];
          P[0] = __uint_as_float(u.x << 16); P[1] = __uint_as_float(u.x & 0xffff0000u);
          P[2] = __uint_as_float(u.y << 16); P[3] = __uint_as_float(u.y & 0xffff0000u);
          P[4] = __uint_as_float(u.z << 16); P[5] = __uint_as_float(u.z & 0xffff0000u);
          P[6] = __uint_as_float(u.w << 16); P[7] = __uint_as_float(u.w & 0xffff0000u);
          Pt[0] = __uint_as_float(w.x << 16); Pt[1] = __uint_as_float(w.x & 0xffff0000u);
          Pt[2] = __uint_as_float(w.y << 16); Pt[3] = __uint_as_float(w.y & 0xffff0000u);
          Pt[4] = __uint_as_float(w.z << 16); Pt[5] = __uint_as_float(w.z & 0xffff0000u);
          Pt[6] = __uint_as_float(w.w << 16); Pt[7] = __uint_as_float(w.w & 0xffff0000u);
        }
        if constexpr (epi == EPI_BWD_STATS) {
          float d = 0.f, dt = 0.f;
#pragma unroll
          for (int q = 0; q < 8; ++q)
            if (ok[q]) { d += P[q] * vp[q]; dt += Pt[q] * vp[q] + P[q] * vt[q]; }
          d = xor8_sum(d);
          dt = xor8_sum(dt);
          if (ch == 0 && rowok && n0 + wn0 < p.N) {
            float* dst = p.part + ((zrow0 + gm) * p.NP + (n0 + wn0) / 64) * 3;
            dst[0] = d; dst[1] = dt; dst[2] = 0.f;
          }
        } else {  // EPI_BWD_DS
          const float d = pre_s[kNeedStat ? i * 4 + ps : 0][0], dt = pre_s[kNeedStat ? i * 4 + ps : 0][1];
          if (!rowok || gn >= p.N) continue;
          float dS[8], dSt[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            dS[q] = ok[q] ? P[q] * (vp[q] - d) : 0.f;
            dSt[q] = ok[q] ? Pt[q] * (vp[q] - d) + P[q] * (vt[q] - dt) : 0.f;
          }
          store8_bf16(p.C, ci, gn, dS);
          store8_bf16(p.Ct, ci, gn, dSt);
        }
      }
    }
    __syncthreads();
  }
}

template <bool TA, bool TB, int NT, int NS, int EPI>
static hipError_t launch_dual_k(const DualP& p, dim3 grid, hipStream_t st) {
  static OncePerDevice once;
  auto kern = gemm_dual_kernel<TA, TB, NT, NS, EPI>;
  constexpr int smem_pipe = NS * NT * 128 * 32 * 2, smem_epi = 4 * 2 * 32 * (64 + 4) * 4;
  constexpr int smem = smem_pipe > smem_epi ? smem_pipe : smem_epi;
  static_assert(smem <= 160 * 1024, "LDS");
  if (hipError_t e = once.lds_limit((const void*)kern, smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
  return hipGetLastError();
}
// A launch of at most one block per CU cannot hide a slab's load latency behind another block, so
// it keeps two or three slabs in flight instead of one (the LDS is its own anyway).
template <bool TA, bool TB>
static hipError_t launch_dual_one(const DualP& p, dim3 grid, hipStream_t st) {
  const bool deep = (int64_t)grid.x * grid.y * grid.z <= 256 && p.K >= 256;
  if (p.Blo) return deep ? launch_dual_k<TA, TB, 6, 3, EPI_NONE>(p, grid, st) : launch_dual_k<TA, TB, 6, 2, EPI_NONE>(p, grid, st);
  if (p.Alo) return deep ? launch_dual_k<TA, TB, 5, 3, EPI_NONE>(p, grid, st) : launch_dual_k<TA, TB, 5, 2, EPI_NONE>(p, grid, st);
  return deep ? launch_dual_k<TA, TB, 4, 4, EPI_NONE>(p, grid, st) : launch_dual_k<TA, TB, 4, 2, EPI_NONE>(p, grid, st);
}
// Attention epilogues: A B^T products with k = head dimension.  Four operand
// tiles per stage and two stages (optional low-order terms run as further
// slabs), so that two blocks are resident per CU: with so short a k the
// per-block prologue and epilogue dominate and only a second block hides them.
template <int EPI>
static hipError_t launch_dual_att(const DualP& p, dim3 grid, hipStream_t st) {
  if (p.K % 32 != 0) return hipErrorNotSupported;  // the low-order loops have no ragged-k path
  return launch_dual_k<false, true, 4, 2, EPI>(p, grid, st);
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
  p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.nb2 = g.nb2; p.divB = g.divB > 0 ? g.divB : 1;
  p.sA1 = g.sA1; p.sA2 = g.sA2; p.sB1 = g.sB1; p.sB2 = g.sB2; p.sC1 = g.sC1; p.sC2 = g.sC2;
  p.alpha = g.alpha; p.out_bf16 = g.out_bf16; p.bias_bf16 = 1; p.klimit = g.klimit; p.skip_upper = g.skip_upper;
  p.epi = g.epi; p.part = g.part; p.rstat = g.rstat; p.E0 = g.E0; p.E1 = g.E1; p.NP = (g.N + 63) / 64;
  if (g.epi != EPI_NONE) {
    const bool stats = g.epi == EPI_FWD_STATS || g.epi == EPI_BWD_STATS;
    const bool reads = g.epi == EPI_BWD_STATS || g.epi == EPI_BWD_DS;
    if ((stats && !g.part) || (!stats && (!g.rstat || !g.out_bf16)) || (reads && (!g.E0 || !g.E1)) || g.Cadd || g.Cadd_t ||
        g.bias || g.bias_t)
      return hipErrorInvalidValue;
    if (g.transA || !g.transB) return hipErrorNotSupported;
  }
  {
    const int64_t q = (g.out_bf16 || g.epi != EPI_NONE) ? 8 : 4;
    auto al = [&](const void* x) { return x == nullptr || ((uintptr_t)x % 16) == 0; };
    p.vec = al(g.C) && al(g.Ct) && al(g.C_lo) && al(g.E0) && al(g.E1) && al(g.Cadd) && al(g.Cadd_t) && g.ldc % q == 0 &&
            g.sC1 % q == 0 && g.sC2 % q == 0;
  }
  if (p.Blo && !p.Alo) return hipErrorNotSupported;
  p.sCk = 0;
  const int64_t nt = ((g.M + 127) / 128) * (int64_t)((g.N + 127) / 128);
  dim3 grid((unsigned)nt, (unsigned)(g.nb1 * g.nb2), 1);
  // Few output tiles and a long k (a 7B-shaped layer at 512 tokens: 128 tiles, k = 4096 or 11008):
  // split k so that every CU holds one block; the partial sums go to fp32 scratch and a second
  // kernel adds them up and applies bias, addend and the output format.
  if (g.epi == EPI_NONE && g.ws && g.nb1 * g.nb2 == 1 && nt * 2 <= 256 && g.K >= 1024 && !g.klimit && !g.skip_upper) {
    const int64_t mn = (int64_t)g.M * g.N;
    const int ks = (int)std::min<int64_t>(std::min<int64_t>(256 / nt, g.K / 512), 8);
    if (ks >= 2 && 2 * ks * mn <= g.ws_elems) {
      DualP q = p;
      q.C = g.ws; q.Ct = g.ws + ks * mn; q.Clo = nullptr; q.Cadd = nullptr; q.Cadd_t = nullptr; q.bias = nullptr; q.bias_t = nullptr;
      q.out_bf16 = 0; q.ldc = g.N; q.sCk = mn; q.vec = (g.N % 4 == 0 && ((uintptr_t)g.ws % 16) == 0 && mn % 4 == 0) ? 1 : 0;
      grid.z = (unsigned)ks;
      hipError_t e;
      if (!g.transA && !g.transB) e = launch_dual_one<false, false>(q, grid, st);
      else if (!g.transA && g.transB) e = launch_dual_one<false, true>(q, grid, st);
      else if (g.transA && !g.transB) e = launch_dual_one<true, false>(q, grid, st);
      else e = launch_dual_one<true, true>(q, grid, st);
      if (e != hipSuccess) return e;
      SplitKOut o0, o1;
      o0.part = g.ws; o0.bias_bf16 = (const bf16*)g.bias; o0.Cadd = g.Cadd; o0.C = g.C; o0.C_lo = g.C_lo;
      o1.part = g.ws + ks * mn; o1.bias_f32 = g.bias_t; o1.Cadd = g.Cadd_t; o1.C = g.Ct;
      return launch_splitk_reduce(o0, o1, ks, g.M, g.N, g.ldc, g.out_bf16, st);
    }
  }
  if (g.epi != EPI_NONE) {
    if (!p.vec || g.N % 8 != 0) return hipErrorNotSupported;
    switch (g.epi) {
      case EPI_FWD_STATS: return launch_dual_att<EPI_FWD_STATS>(p, grid, st);
      case EPI_FWD_SOFTMAX: return launch_dual_att<EPI_FWD_SOFTMAX>(p, grid, st);
      case EPI_BWD_STATS: return launch_dual_att<EPI_BWD_STATS>(p, grid, st);
      case EPI_BWD_DS: return launch_dual_att<EPI_BWD_DS>(p, grid, st);
      default: return hipErrorInvalidValue;
    }
  }
  if (!g.transA && !g.transB) return launch_dual_one<false, false>(p, grid, st);
  if (!g.transA && g.transB) return launch_dual_one<false, true>(p, grid, st);
  if (g.transA && !g.transB) return launch_dual_one<true, false>(p, grid, st);
  return launch_dual_one<true, true>(p, grid, st);
}

}  // namespace hf
