// bf16 matrix-product kernel for the CDNA4 matrix cores (the performance core
// of the Hessian-vector product: every linear layer and every attention
// product of Algorithm 1's forward, backward and tangent passes lands here).
//
//   C = alpha (A0 op B0 + A1 op B1) + bias + Cadd      fp32 accumulate
//
// Design for gfx950:
//   * block tile BM x BN x 64, four wavefronts, each WM x WN made of
//     v_mfma_f32_32x32x16_bf16 tiles with accumulators resident in registers;
//   * operands go global -> LDS directly (global_load_lds, 16 B per lane, no
//     VGPR staging) into a double buffer, so the loads of k-slab i+1 are in
//     flight while slab i is multiplied; only s_waitcnt vmcnt + s_barrier
//     separate the stages;
//   * one wave per SIMD issues everything in order, so fragment reads and loads are
//     dealt out between the matrix instructions (a run of them in front of a k-step
//     leaves the matrix pipe idle), and the barrier that hands a stage over sits
//     before a slab's last k-step, whose matrix instructions cover the first
//     fragment reads of the next slab;
//   * an operand that is k-contiguous in memory is stored [row][64] with the
//     16 B chunks of a row XOR-swizzled by (row & 7), so the 16 B fragment
//     reads of 32 consecutive rows are bank-conflict free;
//   * an operand that is row-contiguous in memory (A^T or B) keeps its memory
//     order [k][row] in LDS and is read with ds_read_b64_tr_b16, which hands
//     each lane four consecutive k of its own column: no transposition pass
//     and no second copy of the weights;
//   * out-of-range rows/columns are clamped to a valid address (they only feed
//     outputs that are never stored); a ragged last k-slab is loaded through a
//     guarded path; optional split-K accumulates with fp32 atomics.
#include "gemm_mfma_common.h"

namespace hf {

// Pipeline: two LDS stages.  Iteration j waits for slab j+1, passes one barrier
// (every wave then holds the fragments of slab j's last k-step in registers, so
// slab j's stage is free), multiplies that last k-step and the first k-steps of
// slab j+1 while the loads of slab j+2 go to the freed stage.
// 128x128 tiles with 32-deep slabs are compiled for three resident blocks per
// CU (768 slots), which fits the 576- and 768-tile products of the small
// models in one round; the other shapes take what registers they need.
constexpr int cmin(int a, int b) { return a < b ? a : b; }

template <int BM, int BN, int KT, int NS>
constexpr int min_blocks() { return (BM == 128 && BN == 128 && KT == 32 && NS == 2) ? 3 : 1; }

// The body of the kernel: one block's product.  ks / nks: this block's part of a k-split.
// given_tile >= 0: the block's tile index is given (a launch that deals the tiles of several
// products to its blocks itself) instead of derived from the block index.
template <int BM, int BN, int WM, int WN, int KT, int NS, bool TA, bool TB, int FL>
__device__ __forceinline__ void gemm_mfma_body(const GemmP& p, const int ks, const int nks, const int given_tile = -1) {
  static_assert((BM / WM) * (BN / WN) == 4, "four waves");
  static_assert(NS == 2, "stages");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  HF_LDS bf16* smem = (HF_LDS bf16*)smem_raw;
  constexpr int A_EL = BM * KT, B_EL = BN * KT, STAGE = A_EL + B_EL;
  constexpr bool AKC = !TA, BKC = TB;
  constexpr int NLOAD = (BM + BN) * KT / 2048;  // load instructions per wave per slab

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);  // wave-uniform, kept in an SGPR
  // tile order: blocks are dealt round-robin to the 8 XCDs; give each XCD a
  // contiguous range of tiles so that neighbours share operand rows in its L2.
  // Batched causal products (attention, k clipped per tile row) instead give XCD c the whole
  // batch entries (heads) c, c + 8, ...: every XCD gets the same mix of long and short tile
  // rows, and a head's B operand (V, K, Q or dO) is fetched by one L2 only.
  int tile = blockIdx.x, z = blockIdx.y;
  if (given_tile >= 0) {
    tile = given_tile;
    z = 0;
  } else {
    const int nt = gridDim.x;
    if (p.klimit && (gridDim.y & 7) == 0) {
      // launch-order index L: XCD L % 8, its r-th block; XCD c walks the tiles of batch entry c,
      // then of entry c + 8, ...
      const int L = blockIdx.y * nt + blockIdx.x, r = L >> 3;
      z = (r / nt) * 8 + (L & 7);
      tile = r % nt;
    } else if (nt >= 16) {
      const int per = nt / 8, rem = nt % 8;
      const int x = tile % 8, q = tile / 8;
      // XCD x owns `per` (+1 if x < rem) consecutive tiles
      const int start = x * per + min(x, rem);
      tile = start + q;
    }
  }
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  // Grouped order: bands of GROUP_M tile rows, walked row-first inside a band,
  // so that a contiguous run of tiles (what one XCD executes at a time) covers
  // a near-square patch and shares both operand streams through its L2.
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
  // Causal products (k clipped to the tile row's triangle) cost in proportion to the row index.
  // The second half of the batch walks the rows in reverse, so that the two blocks a CU holds at a
  // time (ids b and b + half the grid) are a heavy and a light one.
  if (given_tile < 0 && p.klimit && blockIdx.y * 2 >= gridDim.y) tm = tiles_m - 1 - tm;
  const int m0 = tm * BM, n0 = tn * BN;
  if (p.skip_upper && n0 > m0 + BM - 1) return;
  const int z1 = z / p.nb2, z2 = z % p.nb2;
  const int64_t offA = z1 * p.sA1 + z2 * p.sA2, offB = z1 * p.sB1 + (z2 / p.divB) * p.sB2, offC = z1 * p.sC1 + z2 * p.sC2;
  int kbeg = 0, kend = p.K;
  if (p.klimit == 1) kend = min(p.K, m0 + BM);
  if (p.klimit == 2) kbeg = (m0 / 64) * 64;
  const int wm0 = (wave / (BN / WN)) * WM, wn0 = (wave % (BN / WN)) * WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nfull = (kend - kbeg) / KT;          // full slabs per term
  const int ktail = (kend - kbeg) - nfull * KT;  // ragged remainder
  const int nterm = p.nterm;
  // split-K: this block handles slabs [it0, it1) of the nterm*nfull full slabs
  const int total = nterm * nfull;
  const int it0 = (int)((int64_t)total * ks / nks), it1 = (int)((int64_t)total * (ks + 1) / nks);

  // Per-lane source offsets of this wave's load instructions (slab-invariant).
  constexpr int NIA = BM * KT / 2048, NIB = BN * KT / 2048;
  uint32_t voffA[NIA], voffB[NIB];
  slab_offsets<BM, AKC, KT>(voffA, p.lda, m0, p.M, wave, lane);
  slab_offsets<BN, BKC, KT>(voffB, p.ldb, n0, p.N, wave, lane);
  const int64_t stepA = (AKC ? (int64_t)KT : (int64_t)KT * p.lda) * 2;  // bytes per slab
  const int64_t stepB = (BKC ? (int64_t)KT : (int64_t)KT * p.ldb) * 2;
  auto slab_base = [&](const void* X, int64_t off, bool kc, int64_t ld, int r0, int k0) {
    return (const char*)X + (off + (kc ? (int64_t)r0 * ld + k0 : (int64_t)k0 * ld + r0)) * 2;
  };
  // issue-side cursor: runs NS-1 slabs ahead of the compute-side one
  int i_term = nfull > 0 ? it0 / nfull : 0, i_slab = nfull > 0 ? it0 % nfull : 0;
  const char* i_a = slab_base(p.A[i_term], offA, AKC, p.lda, m0, kbeg + i_slab * KT);
  const char* i_b = slab_base(p.B[i_term], offB, BKC, p.ldb, n0, kbeg + i_slab * KT);
  HF_LDS char* const smem_c = (HF_LDS char*)smem;
  auto issue = [&](int stage) {
    HF_LDS char* sa = smem_c + stage * (STAGE * 2);
    slab_issue<NIA>(i_a, voffA, sa + wave * (NIA * 1024));
    slab_issue<NIB>(i_b, voffB, sa + A_EL * 2 + wave * (NIB * 1024));
    i_a += stepA;
    i_b += stepB;
    if (++i_slab == nfull) {  // next term
      i_slab = 0;
      if (++i_term < nterm) {
        i_a = slab_base(p.A[i_term], offA, AKC, p.lda, m0, kbeg);
        i_b = slab_base(p.B[i_term], offB, BKC, p.ldb, n0, kbeg);
      }
    }
  };
  // Per-lane LDS byte addresses of this wave's fragments (stage 0): one per
  // k-step for a k-contiguous operand (the chunk swizzle depends on k), one in
  // all for a row-contiguous operand (k-steps are a constant offset apart).
  constexpr int NKK = KT / 16;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  uint32_t adA[AKC ? NKK : 1][TM], adB[BKC ? NKK : 1][TN];
#pragma unroll
  for (int kk = 0; kk < (AKC ? NKK : 1); ++kk)
#pragma unroll
    for (int i = 0; i < TM; ++i) adA[kk][i] = lds0 + frag_addr<BM, AKC, KT>(wm0 + i * 32, kk, lane);
#pragma unroll
  for (int kk = 0; kk < (BKC ? NKK : 1); ++kk)
#pragma unroll
    for (int j = 0; j < TN; ++j) adB[kk][j] = lds0 + A_EL * 2 + frag_addr<BN, BKC, KT>(wn0 + j * 32, kk, lane);

  // Issue-side helpers for loads interleaved with the products: load number L
  // of the next slab (A tiles first), and the cursor update after the last.
  auto issue_one = [&](auto stage_c, auto l_c) {
    constexpr int stage = decltype(stage_c)::value, L = decltype(l_c)::value;
    HF_LDS char* sa = smem_c + stage * (STAGE * 2);
    if constexpr (L < NIA)
      __builtin_amdgcn_global_load_lds((const void*)(i_a + voffA[L]), (HF_LDS void*)(sa + wave * (NIA * 1024) + L * 1024), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((const void*)(i_b + voffB[L - NIA]),
                                       (HF_LDS void*)(sa + A_EL * 2 + wave * (NIB * 1024) + (L - NIA) * 1024), 16, 0, 0);
  };
  auto issue_advance = [&]() {
    i_a += stepA;
    i_b += stepB;
    if (++i_slab == nfull) {  // next term
      i_slab = 0;
      if (++i_term < nterm) {
        i_a = slab_base(p.A[i_term], offA, AKC, p.lda, m0, kbeg);
        i_b = slab_base(p.B[i_term], offB, BKC, p.ldb, n0, kbeg);
      }
    }
  };

  // Fragment registers: two sets, alternating by k-step parity; they live
  // across slab boundaries (the last k-step of a slab is multiplied after the
  // barrier that hands over the next slab).
  constexpr int Q = TM * TN, QS = Q * NKK;  // matrix instructions per k-step / per slab
  static_assert(NLOAD * FL <= QS, "at most one load per matrix instruction");
  static_assert(NS == 2 && NKK % 2 == 0, "two LDS stages, an even number of k-steps per slab");
  Frag<AKC> fa[2][TM];
  Frag<BKC> fb[2][TN];
  // request fragment number f (A fragments first) of k-step kk of the slab in LDS stage S
  // (plus a run-time byte offset)
  constexpr int NF = TM + TN;
  auto request_one = [&](auto stage_c, auto kk_c, auto f_c, uint32_t dyn) {
    constexpr int S = decltype(stage_c)::value, kk = decltype(kk_c)::value, f = decltype(f_c)::value;
    constexpr int oA = S * STAGE * 2 + (AKC ? 0 : kk * 16 * BM * 2);
    constexpr int oB = S * STAGE * 2 + (BKC ? 0 : kk * 16 * BN * 2);
    if constexpr (f < TM) fa[kk & 1][f].template read<oA, 4 * BM * 2>(adA[AKC ? kk : 0][f] + dyn);
    else fb[kk & 1][f - TM].template read<oB, 4 * BN * 2>(adB[BKC ? kk : 0][f - TM] + dyn);
  };
  auto request = [&](auto stage_c, auto kk_c, uint32_t dyn) {
    static_for<NF>([&](auto f_c) { request_one(stage_c, kk_c, f_c, dyn); });
  };
  // every LDS read requested so far has landed; pins the fragments of k-step kk to this point
  auto landed = [&](auto kk_c) {
    constexpr int kk = decltype(kk_c)::value;
    __builtin_amdgcn_sched_barrier(0);
    lds_wait_all();
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[kk & 1][i].tie();
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[kk & 1][j].tie();
  };
  // The Q matrix instructions of k-step kk.  Everything else the wave has to issue is dealt out
  // between them, so that the matrix pipe never waits behind a run of memory instructions:
  //  * with REQ, the fragment reads of k-step RK of the slab in stage RS (into the other register
  //    set), one or two after each of the first Q/2 matrix instructions;
  //  * with ISSUE, this being phase PH (0 .. NKK-1) of a pipeline iteration, the NLOAD loads of
  //    the slab two ahead, at most one after each of the iteration's first QS / FL matrix
  //    instructions, into LDS stage LS.
  auto mfmas = [&](auto kk_c, auto ph_c, auto issue_c, auto ls_c, auto req_c, auto rs_c, auto rk_c, uint32_t dyn) {
    constexpr int kk = decltype(kk_c)::value, PH = decltype(ph_c)::value;
    constexpr bool ISSUE = decltype(issue_c)::value, REQ = decltype(req_c)::value;
    static_for<Q>([&](auto q_c) {
      constexpr int q = decltype(q_c)::value, g = PH * Q + q;
      acc[q / TN][q % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][q / TN].get(), fb[kk & 1][q % TN].get(),
                                                                    acc[q / TN][q % TN], 0, 0, 0);
      if constexpr (REQ) {
        static_for<NF>([&](auto f_c) {
          constexpr int f = decltype(f_c)::value;
          if constexpr ((f * Q) / (2 * NF) == q) request_one(rs_c, rk_c, f_c, dyn);
        });
      }
      constexpr int l0 = cmin((g * NLOAD * FL) / QS, NLOAD), l1 = cmin(((g + 1) * NLOAD * FL) / QS, NLOAD);
      if constexpr (ISSUE && l1 > l0) issue_one(ls_c, std::integral_constant<int, l0>{});
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  using I0 = std::integral_constant<int, 0>;
  // k-steps 0 .. NKK-2 of a slab whose k-step 0 has been requested: each waits for its
  // fragments and multiplies while the next k-step's are requested.  On return the fragments
  // of k-step NKK-1 are in registers and no LDS read is outstanding.
  auto ksteps = [&](auto stage_c, auto issue_c, auto ls_c, uint32_t dyn) {
    static_for<NKK - 1>([&](auto k_c) {
      constexpr int k = decltype(k_c)::value;
      landed(k_c);
      mfmas(k_c, std::integral_constant<int, k + 1>{}, issue_c, ls_c, std::true_type{}, stage_c,
            std::integral_constant<int, k + 1>{}, dyn);
    });
    landed(std::integral_constant<int, NKK - 1>{});
  };
  // One pipeline iteration, entered right after the barrier that publishes the slab in LDS
  // stage S: the matrix instructions of the previous slab's last k-step (its fragments are in
  // registers) cover this slab's first fragment reads; then k-steps 0 .. NKK-2 of this slab.
  // With ISSUE the loads of the slab after this one go to the other stage, which every wave
  // has finished reading before that barrier.
  auto iteration = [&](auto stage_c, auto issue_c, uint32_t dyn) {
    constexpr int S = decltype(stage_c)::value;
    using LS = std::integral_constant<int, 1 - S>;
    mfmas(std::integral_constant<int, NKK - 1>{}, I0{}, issue_c, LS{}, std::true_type{}, stage_c, I0{}, dyn);
    ksteps(stage_c, issue_c, LS{}, dyn);
    if constexpr (decltype(issue_c)::value) issue_advance();
  };

  const int nit = it1 - it0;
  if (nit > 0) {
    issue(0);
    if (nit > 1) {
      issue(1);
      HF_WAIT_VMCNT(NLOAD);
    } else {
      HF_WAIT_VMCNT(0);
    }
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    request(I0{}, I0{}, 0u);
    ksteps(I0{}, std::false_type{}, I0{}, 0u);
    // iterations that still have a slab to prefetch, unrolled by two so that the
    // LDS stage addresses are compile-time constants; then the last one, whose
    // stage is a run-time offset
    const int n_issue = max(0, nit - 2);
    for (int j0 = 0; j0 < n_issue; j0 += 2) {
      static_for<2>([&](auto s_c) {
        constexpr int s = decltype(s_c)::value;
        if (j0 + s < n_issue) {
          HF_WAIT_VMCNT(0);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          iteration(std::integral_constant<int, 1 - s>{}, std::true_type{}, 0u);
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    }
    if (nit > 1) {
      HF_WAIT_VMCNT(0);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      iteration(I0{}, std::false_type{}, (uint32_t)(((nit - 1) & 1) * (STAGE * 2)));
      __builtin_amdgcn_sched_barrier(0);
    }
    mfmas(std::integral_constant<int, NKK - 1>{}, I0{}, std::false_type{}, I0{}, std::false_type{}, I0{}, I0{}, 0u);
  }
  // ragged k remainder (handled by the last split only)
  if (ktail > 0 && ks == nks - 1) {
    for (int term = 0; term < nterm; ++term) {
      const bf16* A = (const bf16*)p.A[term] + offA;
      const bf16* B = (const bf16*)p.B[term] + offB;
      const int k0 = kbeg + nfull * KT;
      __syncthreads();
      slab_guarded<BM, AKC, KT>(A, p.lda, m0, k0, p.M, kend, smem, t);
      slab_guarded<BN, BKC, KT>(B, p.ldb, n0, k0, p.N, kend, smem + A_EL, t);
      __syncthreads();
      request(I0{}, I0{}, 0u);
      ksteps(I0{}, std::false_type{}, I0{}, 0u);
      mfmas(std::integral_constant<int, NKK - 1>{}, I0{}, std::false_type{}, I0{}, std::false_type{}, I0{}, I0{}, 0u);
    }
  }

  // epilogue.  An accumulator tile holds, per lane, column (lane & 31) and rows
  // 8*(r/4) + 4*(lane/32) + r%4.  Split-K adds with atomics straight from that
  // layout; otherwise each wave stages 32 x WN results in LDS and writes them
  // out row-wise, 8 consecutive columns (16 B of bf16, 32 B of fp32) per lane.
  const bool first = (ks == 0);
  float bsum[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int gn = n0 + wn0 + j * 32 + (lane & 31);
    bsum[j] = 0.f;
    if (first && gn < p.N) {
      if (p.bias) bsum[j] += p.bias_bf16 ? (float)((const bf16*)p.bias)[gn] : ((const float*)p.bias)[gn];
      if (p.bias_t) bsum[j] += p.bias_t[gn];
    }
  }
  if (nks > 1) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int gn = n0 + wn0 + j * 32 + (lane & 31);
      if (gn >= p.N) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int gm = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          if (gm >= p.M) continue;
          // C was zero-filled (or holds Cadd) by the launcher
          atomicAdd((float*)p.C + offC + (int64_t)gm * p.ldc + gn, p.alpha * acc[i][j][r] + bsum[j]);
        }
    }
    return;
  }
  constexpr int LDW = WN + 4;               // staging row stride (floats)
  constexpr int CPRW = WN / 8;              // 8-column chunks per staged row
  constexpr int RPP = 64 / CPRW;            // rows written per pass of the wave
  HF_LDS float* stg = (HF_LDS float*)smem + wave * (32 * LDW);
  const bool vec = p.vecA != 0;             // C (and Cadd / C_lo) rows are 16-byte aligned
  __syncthreads();                          // every wave is done reading operand tiles
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stg[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * LDW + j * 32 + (lane & 31)] = p.alpha * acc[i][j][r] + bsum[j];
    __syncthreads();
#pragma unroll
    for (int ps = 0; ps < 32 / RPP; ++ps) {
      const int row = ps * RPP + lane / CPRW, ch = lane % CPRW;
      const int gm = m0 + wm0 + i * 32 + row, gn = n0 + wn0 + ch * 8;
      if (gm < p.M && gn < p.N) {
        typedef float f32x4_t __attribute__((ext_vector_type(4)));
        const f32x4_t x0 = *(const HF_LDS f32x4_t*)(stg + row * LDW + ch * 8);
        const f32x4_t x1 = *(const HF_LDS f32x4_t*)(stg + row * LDW + ch * 8 + 4);
        float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
        if (vec && gn + 8 <= p.N) {
          if (p.Cadd) {
            const float4 c0 = *(const float4*)(p.Cadd + ci), c1 = *(const float4*)(p.Cadd + ci + 4);
            v[0] += c0.x; v[1] += c0.y; v[2] += c0.z; v[3] += c0.w; v[4] += c1.x; v[5] += c1.y; v[6] += c1.z; v[7] += c1.w;
          }
          if (p.out_bf16) {
            bf16 hi[8], lo[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) { hi[q] = (bf16)v[q]; lo[q] = (bf16)(v[q] - (float)hi[q]); }
            *(uint4*)((bf16*)p.C + ci) = *(const uint4*)hi;
            if (p.C_lo) *(uint4*)((bf16*)p.C_lo + ci) = *(const uint4*)lo;
          } else {
            *(float4*)((float*)p.C + ci) = make_float4(v[0], v[1], v[2], v[3]);
            *(float4*)((float*)p.C + ci + 4) = make_float4(v[4], v[5], v[6], v[7]);
          }
        } else {
          for (int q = 0; q < 8; ++q) {
            if (gn + q >= p.N) break;
            float x = v[q];
            if (p.Cadd) x += p.Cadd[ci + q];
            if (p.out_bf16) {
              const bf16 h = (bf16)x;
              ((bf16*)p.C)[ci + q] = h;
              if (p.C_lo) ((bf16*)p.C_lo)[ci + q] = (bf16)(x - (float)h);
            } else {
              ((float*)p.C)[ci + q] = x;
            }
          }
        }
      }
    }
    __syncthreads();
  }
}

template <int BM, int BN, int WM, int WN, int KT, int NS, bool TA, bool TB, int FL = 1>
__global__ __launch_bounds__(256, (min_blocks<BM, BN, KT, NS>())) void gemm_mfma_kernel(GemmP p) {
  gemm_mfma_body<BM, BN, WM, WN, KT, NS, TA, TB, FL>(p, blockIdx.z, gridDim.z);
}

// Two products of the same shape in one launch (a primal product and its tangent, each too
// small to fill the CUs with 256 x 256 tiles on its own): blockIdx.z selects the product.
struct GemmPair { GemmP g[2]; };
template <int BM, int BN, int WM, int WN, int KT, int NS, bool TA, bool TB, int FL = 1>
__global__ __launch_bounds__(256, (min_blocks<BM, BN, KT, NS>())) void gemm_mfma_pair_kernel(GemmPair pp) {
  gemm_mfma_body<BM, BN, WM, WN, KT, NS, TA, TB, FL>(pp.g[blockIdx.z], 0, 1);
}

// Up to four A^T B products (the weight-gradient products of one layer: few output tiles each, a
// long contraction over the tokens) as one launch of 256 x 256 tiles: block b works on part
// (b - first[g]) / tiles[g] of the k-split of tile (b - first[g]) % tiles[g] of product g and adds
// its result with atomics, so every C must hold zeros (or what the sum is added to) beforehand.
struct GemmGroup {
  GemmP g[4];
  int first[5];   // first block of each product; first[n] = number of blocks
  int tiles[4];
  int nks[4];
  int n;
};
template <int BM, int BN, int WM, int WN, int KT, int NS, bool TA, bool TB, int FL = 1>
__global__ __launch_bounds__(256, 1) void gemm_mfma_group_kernel(GemmGroup gg) {
  const int b = blockIdx.x;
  int g = 0;
  while (g + 1 < gg.n && b >= gg.first[g + 1]) ++g;
  const int local = b - gg.first[g];
  gemm_mfma_body<BM, BN, WM, WN, KT, NS, TA, TB, FL>(gg.g[g], local / gg.tiles[g], gg.nks[g], local % gg.tiles[g]);
}

template <int BM, int BN, int WM, int WN, int KT, int NS, bool TA, bool TB, int FL = 1>
static hipError_t launch_one(const GemmP& p, dim3 grid, hipStream_t st) {
  constexpr int smem_pipe = NS * (BM + BN) * KT * 2, smem_epi = 4 * 32 * (WN + 4) * 4;
  constexpr int smem = smem_pipe > smem_epi ? smem_pipe : smem_epi;
  static OncePerDevice once;
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, KT, NS, TA, TB, FL>;
  if (hipError_t e = once.lds_limit((const void*)kern, smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, int KT, int NS, int FL = 1>
static hipError_t launch_cfg(const GemmP& p, dim3 grid, hipStream_t st) {
  if (!p.transA && !p.transB) return launch_one<BM, BN, WM, WN, KT, NS, false, false, FL>(p, grid, st);
  if (!p.transA && p.transB) return launch_one<BM, BN, WM, WN, KT, NS, false, true, FL>(p, grid, st);
  if (p.transA && !p.transB) return launch_one<BM, BN, WM, WN, KT, NS, true, false, FL>(p, grid, st);
  return launch_one<BM, BN, WM, WN, KT, NS, true, true, FL>(p, grid, st);
}

// Tile configurations (index = force_cfg): block tile, slab depth.
struct TileCfg { int bm, bn; };
// 0: 256x256x64; 1: 128x128x64; 2: 128x128x32; 3: 256x128x64 and 4: 128x64x64 for products one
// attention head wide (N = 128 / N <= 64).  All but the last deal the loads of the next slab out
// over the first half of a slab's matrix instructions (FL = 2), which leaves them the second
// half to land; the 128x64 tile has too few matrix instructions per slab for that.
// (Three- and four-stage pipelines with 32-deep slabs were measured and were slower.)
static const TileCfg kCfg[] = {{256, 256}, {128, 128}, {128, 128}, {256, 128}, {128, 64}};
constexpr int kNumCfg = 5;

// Tile choice: the largest tile that still yields about two blocks per CU;
// split-K for products with few output tiles and a long k (the H v blocks).
static void choose_tile_and_split(const GemmP& p, int nb, int allow_splitk, int force_cfg, int force_ks, int& cfg_out, int& ks_out) {
  const int64_t M = p.M, N = p.N;
  auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn) * (int64_t)nb; };
  // Measured on MI355X: 256x256 tiles (one block per CU) reach 1.3-1.5 PFLOP/s when their count
  // fills the 256 CUs evenly, 128x128 tiles (two blocks per CU) 1.1-1.3 PFLOP/s; a product with
  // 384 tiles of 256x256 (1.5 rounds) is faster on the small tile.  A^T B products read both
  // operands through transposing LDS reads, which the small tile hides worse, so they keep the
  // large tile down to 160 tiles.  A row-contiguous B with a short k prefers 32-deep slabs
  // (the pipeline fills sooner).
  const int64_t t256 = tiles(256, 256);
  const bool even256 = t256 >= 256 && t256 * 100 >= ((t256 + 255) / 256) * 256 * 85;
  int cfg;
  if (force_cfg >= 0 && force_cfg < kNumCfg) cfg = force_cfg;
  else if (!p.transB && N <= 64 && M >= 128) cfg = 4;
  else if (!p.transB && N <= 128 && N > 64 && p.klimit) cfg = 1;  // causal: 128-row tiles pair up heavy and light rows
  else if (!p.transB && N <= 128 && N > 64 && tiles(256, 128) >= 128) cfg = 3;
  else if (p.transA && !p.transB) cfg = t256 >= 160 ? 0 : 1;
  else if (!p.transA && !p.transB) cfg = even256 ? 0 : (p.K >= 1536 ? 1 : 2);
  else cfg = even256 ? 0 : 1;
  const int bm = kCfg[cfg].bm, bn = kCfg[cfg].bn;
  const int64_t nt = tiles(bm, bn);
  int ks = 1;
  if (force_ks > 0) ks = force_ks;
  else if (allow_splitk && !p.out_bf16 && !p.klimit) {
    // Split k only while all blocks of the split product are resident at once (256 CUs, one block
    // of a 256-wide tile or two of the others each) and every split keeps at least 8 slabs: a split
    // costs a zero-fill and an atomic read-modify-write of C per part, which for short k outweighs
    // the parallelism (4096 x 4096 x 512: 45 us unsplit, 143 us split in two).
    const int64_t slots = (bm == 256) ? 256 : 512;
    const int slabs = p.nterm * (p.K / 64);
    if (nt * 2 <= slots) ks = (int)std::min<int64_t>(std::min<int64_t>(slots / nt, std::max(1, slabs / 8)), 16);
    // A very long k (the head adjoint: k = vocabulary, 1500 slabs) can afford more parts than
    // are resident at once: take the smallest count whose blocks fill whole rounds of the slots
    // (192 tiles x 8 = 3 x 512 instead of 384 of 512).  For shorter k the extra atomic passes
    // over C cost more than the fuller rounds gain (measured on the weight-gradient products).
    auto full_rounds = [&](int k2) { const int64_t rem = (nt * k2) % slots; return rem == 0 || rem >= slots - slots / 16; };
    if (slabs >= 512 && !full_rounds(ks)) {
      for (int k2 = ks + 1; k2 <= 16; ++k2)
        if (full_rounds(k2) && slabs / k2 >= 16) { ks = k2; break; }
    }
  }
  cfg_out = cfg; ks_out = ks;
}

// Whether launch_gemm_mfma would split k (and so add into C with atomics, which needs C zeroed) for an
// fp32-output A^T B product of this shape: lets a caller clear several results with one fill.
bool gemm_mfma_splits_k(int M, int N, int K, int nterm) {
  GemmP p = {};
  p.M = M; p.N = N; p.K = K; p.nterm = nterm; p.transA = 1; p.transB = 0; p.out_bf16 = 0; p.klimit = 0;
  int cfg, ks;
  choose_tile_and_split(p, 1, 1, -1, -1, cfg, ks);
  return ks > 1;
}

// c_zeroed: the caller has already cleared C (a split product then skips its own fill).
hipError_t launch_gemm_mfma(GemmP p, int nb, int allow_splitk, int force_cfg, int force_ks, hipStream_t st, int c_zeroed) {
  const int64_t M = p.M, N = p.N;
  auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn) * (int64_t)nb; };
  int cfg, ks;
  choose_tile_and_split(p, nb, allow_splitk, force_cfg, force_ks, cfg, ks);
  const int bm = kCfg[cfg].bm, bn = kCfg[cfg].bn;
  const int64_t nt = tiles(bm, bn);
  if (ks > 1) {
    // accumulate with atomics on top of Cadd (or zero)
    if (p.Cadd == nullptr) {
      if (p.ldc == p.N && nb == 1) {
        if (!c_zeroed) {
          hipError_t e = launch_fill_f32((float*)p.C, M * N, 0.f, st);
          if (e != hipSuccess) return e;
        }
      } else {
        ks = 1;
      }
    } else if (p.Cadd != (const float*)p.C) {
      ks = 1;
    }
  }
  p.tiles_n = (int)((N + bn - 1) / bn);
  {  // vectorised stores need 16-byte aligned rows of C (and of Cadd / C_lo)
    const int64_t q = p.out_bf16 ? 8 : 4;
    auto al = [&](const void* x) { return x == nullptr || ((uintptr_t)x % 16) == 0; };
    p.vecA = al(p.C) && al(p.Cadd) && al(p.C_lo) && p.ldc % q == 0 && p.sC1 % q == 0 && p.sC2 % q == 0;
  }
  dim3 grid((unsigned)(nt / nb), (unsigned)nb, (unsigned)ks);
  switch (cfg) {
    case 0: return launch_cfg<256, 256, 128, 128, 64, 2, 2>(p, grid, st);
    case 1: return launch_cfg<128, 128, 64, 64, 64, 2, 2>(p, grid, st);
    case 3: return launch_cfg<256, 128, 128, 64, 64, 2, 2>(p, grid, st);
    case 4: return launch_cfg<128, 64, 64, 32, 64, 2, 1>(p, grid, st);
    default: return launch_cfg<128, 128, 64, 64, 32, 2, 2>(p, grid, st);
  }
}

template <int BM, int BN, int WM, int WN, int KT, int NS, bool TA, bool TB, int FL>
static hipError_t launch_pair_one(const GemmPair& pp, dim3 grid, hipStream_t st) {
  constexpr int smem_pipe = NS * (BM + BN) * KT * 2, smem_epi = 4 * 32 * (WN + 4) * 4;
  constexpr int smem = smem_pipe > smem_epi ? smem_pipe : smem_epi;
  static OncePerDevice once;
  auto kern = gemm_mfma_pair_kernel<BM, BN, WM, WN, KT, NS, TA, TB, FL>;
  if (hipError_t e = once.lds_limit((const void*)kern, smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, pp);
  return hipGetLastError();
}
template <int BM, int BN, int WM, int WN, int KT, int NS, int FL>
static hipError_t launch_pair_cfg(const GemmPair& pp, dim3 grid, hipStream_t st) {
  const GemmP& a = pp.g[0];
  if (!a.transA && !a.transB) return launch_pair_one<BM, BN, WM, WN, KT, NS, false, false, FL>(pp, grid, st);
  if (!a.transA && a.transB) return launch_pair_one<BM, BN, WM, WN, KT, NS, false, true, FL>(pp, grid, st);
  if (a.transA && !a.transB) return launch_pair_one<BM, BN, WM, WN, KT, NS, true, false, FL>(pp, grid, st);
  return hipErrorNotSupported;
}

// A primal product and its tangent (same shape and layout) as one launch; blockIdx.z selects the
// product.  Two cases:
//  * not batched: 256 x 256 tiles, when the two together fill the 256 CUs evenly, in particular
//    when one alone does not (4096 x 2048: 128 + 128 tiles).  The term counts may differ (adjoint 1, its
//    tangent 2): the launch then lasts as long as the two-term blocks, still less than two
//    launches of 128 x 128 tiles;
//  * batched causal products one attention head wide (P V and O_t, dS K and dQ_t, ...): the
//    tiles a single launch would use; one launch instead of two short ones.
// Returns hipErrorNotSupported otherwise; the caller then launches the two products in turn.
hipError_t launch_gemm_mfma_pair(GemmP a, GemmP b, int nb, hipStream_t st) {
  if (a.M != b.M || a.N != b.N || a.K != b.K || a.transA != b.transA || a.transB != b.transB ||
      a.klimit != b.klimit || a.skip_upper || b.skip_upper || (a.transA && a.transB))
    return hipErrorNotSupported;
  GemmPair pp;
  pp.g[0] = a; pp.g[1] = b;
  auto finish = [&](int bn) {
    for (int i = 0; i < 2; ++i) {
      GemmP& p = pp.g[i];
      p.tiles_n = (p.N + bn - 1) / bn;
      const int64_t q = p.out_bf16 ? 8 : 4;
      auto al = [&](const void* x) { return x == nullptr || ((uintptr_t)x % 16) == 0; };
      p.vecA = al(p.C) && al(p.Cadd) && al(p.C_lo) && p.ldc % q == 0 && p.sC1 % q == 0 && p.sC2 % q == 0;
    }
  };
  if (a.klimit) {
    if (a.transB || a.N > 128 || a.M < 128) return hipErrorNotSupported;
    if (a.N > 64) {
      finish(128);
      dim3 grid((unsigned)((a.M + 127) / 128), (unsigned)nb, 2);
      return launch_pair_cfg<128, 128, 64, 64, 64, 2, 2>(pp, grid, st);
    }
    finish(64);
    dim3 grid((unsigned)((a.M + 127) / 128), (unsigned)nb, 2);
    return launch_pair_cfg<128, 64, 64, 32, 64, 2, 1>(pp, grid, st);
  }
  if (nb != 1) return hipErrorNotSupported;
  const int64_t t256 = ((int64_t)(a.M + 255) / 256) * ((a.N + 255) / 256);
  auto even = [](int64_t t) { return t >= 256 && t * 100 >= ((t + 255) / 256) * 256 * 85; };
  if (even(2 * t256) && a.K >= 512) {
    finish(256);
    dim3 grid((unsigned)t256, 1, 2);
    return launch_pair_cfg<256, 256, 128, 128, 64, 2, 2>(pp, grid, st);
  }
  // Products that take 128 x 128 tiles on their own (the small models' 576- and 768-tile
  // products): the same tiles, one launch instead of two 40 us ones.
  if (even(t256) || (a.transA && t256 >= 160) || a.N <= 128) return hipErrorNotSupported;
  const int64_t t128 = ((int64_t)(a.M + 127) / 128) * ((a.N + 127) / 128);
  if (t128 < 256 || t128 > 2048) return hipErrorNotSupported;
  finish(128);
  dim3 grid((unsigned)t128, 1, 2);
  if (!a.transA && !a.transB && a.K < 1536) return launch_pair_cfg<128, 128, 64, 64, 32, 2, 2>(pp, grid, st);
  return launch_pair_cfg<128, 128, 64, 64, 64, 2, 2>(pp, grid, st);
}

// The A^T B products ps[0..n) (fp32 results that are zero or hold what the sum is added to, no
// bias, operands on the fast path) as one launch.  hipErrorNotSupported: launch them one by one.
hipError_t launch_gemm_mfma_group(const GemmP* ps, int n, hipStream_t st) {
  if (n < 2 || n > 4) return hipErrorNotSupported;
  GemmGroup gg = {};
  gg.n = n;
  int64_t tiles_total = 0;
  int min_slabs = 1 << 30;
  for (int i = 0; i < n; ++i) {
    const GemmP& p = ps[i];
    if (!p.transA || p.transB || p.out_bf16 || p.klimit || p.skip_upper || p.bias || p.bias_t || p.C_lo) return hipErrorNotSupported;
    if (p.Cadd && p.Cadd != (const float*)p.C) return hipErrorNotSupported;
    if (p.ldc != p.N || p.K < 512) return hipErrorNotSupported;
    gg.g[i] = p;
    gg.g[i].tiles_n = (p.N + 255) / 256;
    gg.g[i].Cadd = nullptr;  // the parts add to C with atomics
    {
      auto al = [&](const void* x) { return x == nullptr || ((uintptr_t)x % 16) == 0; };
      gg.g[i].vecA = al(p.C) && p.ldc % 4 == 0;
    }
    gg.tiles[i] = ((p.M + 255) / 256) * ((p.N + 255) / 256);
    tiles_total += gg.tiles[i];
    min_slabs = std::min(min_slabs, p.K / 64);
  }
  if (tiles_total >= 256 || tiles_total < 16) return hipErrorNotSupported;
  // parts per tile: as many as keep all blocks resident at once (one per CU).  More rounds of
  // shorter parts were slower: a part ends with 65536 atomic adds, which cost as much as about 40
  // slabs of the product (756 blocks of 18 slabs: 262 us for the four products of a GPT-2-small
  // layer; 216 blocks of 64 slabs: see the kernel trace).
  int best = (int)(256 / tiles_total);
  while (best > 1 && min_slabs / best < 8) --best;
  if (best < 2) return hipErrorNotSupported;  // nothing is split: atomics would only cost
  int first = 0;
  for (int i = 0; i < n; ++i) {
    gg.first[i] = first;
    gg.nks[i] = best;
    first += gg.tiles[i] * best;
  }
  gg.first[n] = first;
  constexpr int smem_pipe = 2 * (256 + 256) * 64 * 2, smem_epi = 4 * 32 * (128 + 4) * 4;
  constexpr int smem = smem_pipe > smem_epi ? smem_pipe : smem_epi;
  static OncePerDevice once;
  auto kern = gemm_mfma_group_kernel<256, 256, 128, 128, 64, 2, true, false, 2>;
  if (hipError_t e = once.lds_limit((const void*)kern, smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)first), dim3(256), smem, st, gg);
  return hipGetLastError();
}

}  // namespace hf
