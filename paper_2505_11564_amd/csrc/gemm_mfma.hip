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
#include "hf_internal.h"
#include "gemm_params.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define HF_LDS __attribute__((address_space(3)))

constexpr int KT = 64;  // k-slab

// vmcnt(n) only (expcnt / lgkmcnt left at their maxima), gfx9 encoding.
#define HF_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((((n) & 0xF) | ((((n) >> 4) & 0x3) << 14) | (0x7 << 4) | (0xF << 8)))

// ---- LDS addressing ---------------------------------------------------------
// k-contiguous operand: element (r, k) at r*64 + ((k/8) ^ (r & 7))*8 + k%8.
__device__ __forceinline__ int lds_kc(int r, int k) { return r * KT + ((((k >> 3) ^ r) & 7) << 3) + (k & 7); }
// row-contiguous operand, R rows per k: element (k, r) at k*R + swizzled r.
// 16 B chunk index (r/8) has its bit 2 flipped on odd k (64 B windows of odd
// and even k rows fall on different halves of the banks).
__device__ __forceinline__ int lds_rc(int k, int r, int R) { return k * R + ((((r >> 3) ^ ((k & 1) << 2))) << 3) + (r & 7); }

// Issue the direct global->LDS loads of one k-slab of one operand.
// KC: k-contiguous source (element (r,k) at src[r*ld + k]); else (k,r) at src[k*ld + r].
template <int R, bool KC>
__device__ __forceinline__ void slab_issue(const bf16* __restrict__ src, int64_t ld, int r0, int k0, int rmax,
                                           HF_LDS bf16* lds, int wave, int lane) {
  constexpr int NI = R / 32;  // instructions per wave (each moves 64 chunks of 16 B)
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int P = (wave * NI + j) * 64 + lane;
    const bf16* g;
    if (KC) {
      const int row = P >> 3, pc = P & 7;
      const int lc = pc ^ (row & 7);
      const int gr = min(r0 + row, rmax - 1);
      g = src + (int64_t)gr * ld + k0 + lc * 8;
    } else {
      constexpr int CPR = R / 8;  // chunks per k-row
      const int krow = P / CPR, pc = P % CPR;
      const int lc = pc ^ ((krow & 1) << 2);
      const int gc = min(r0 + lc * 8, ((rmax - 1) >> 3) << 3);
      g = src + (int64_t)(k0 + krow) * ld + gc;
    }
    __builtin_amdgcn_global_load_lds((const void*)g, (HF_LDS void*)(lds + (wave * NI + j) * 512), 16, 0, 0);
  }
}

// Guarded load of a ragged k-slab (k in [k0, kend) valid, the rest zero).
template <int R, bool KC>
__device__ __forceinline__ void slab_guarded(const bf16* __restrict__ src, int64_t ld, int r0, int k0, int rmax, int kend,
                                             HF_LDS bf16* lds, int t) {
  for (int i = t; i < R * KT; i += 256) {
    int r, k;
    if (KC) { k = i & (KT - 1); r = i >> 6; } else { r = i % R; k = i / R; }
    const int gr = r0 + r, gk = k0 + k;
    bf16 v = (bf16)0.f;
    if (gr < rmax && gk < kend) v = KC ? src[(int64_t)gr * ld + gk] : src[(int64_t)gk * ld + gr];
    lds[KC ? lds_kc(r, k) : lds_rc(k, r, R)] = v;
  }
}

// Fragment (row = base + lane%32, k = kk*16 + (lane/32)*8 .. +8) of a slab.
template <int R, bool KC>
__device__ __forceinline__ bf16x8 frag_read(const HF_LDS bf16* lds, int rbase, int kk, int lane) {
  if (KC) {
    const int r = rbase + (lane & 31);
    const int c = kk * 2 + (lane >> 5);
    return *(const HF_LDS bf16x8*)(lds + r * KT + (((c ^ r) & 7) << 3));
  } else {
    // transpose read: 16 lanes address 4 k-rows x 16 columns (4 lanes per row,
    // 4 columns each); lane i of the group receives column i, 4 consecutive k.
    const int i = lane & 15, g = lane >> 4;
    const int kq = kk * 16 + (g >> 1) * 8 + (i >> 2);
    const int c = rbase + (g & 1) * 16 + (i & 3) * 4;
    const HF_LDS bf16* p0 = lds + kq * R + ((((c >> 3) ^ ((kq & 1) << 2))) << 3) + (c & 7);
    const HF_LDS bf16* p1 = p0 + 4 * R;  // k + 4: same parity, same swizzle
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((HF_LDS bf16x4*)p0);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((HF_LDS bf16x4*)p1);
    bf16x8 v;
    v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
    v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
    return v;
  }
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmP p) {
  static_assert((BM / WM) * (BN / WN) == 4, "four waves");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  HF_LDS bf16* smem = (HF_LDS bf16*)smem_raw;
  constexpr int A_EL = BM * KT, B_EL = BN * KT, STAGE = A_EL + B_EL;
  constexpr bool AKC = !TA, BKC = TB;
  constexpr int NLOAD = BM / 32 + BN / 32;  // load instructions per wave per slab

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  // tile order: blocks are dealt round-robin to the 8 XCDs; give each XCD a
  // contiguous range of tiles so that neighbours share operand rows in its L2.
  int tile = blockIdx.x;
  {
    const int nt = gridDim.x;
    if (nt >= 16) {
      const int per = nt / 8, rem = nt % 8;
      const int x = tile % 8, q = tile / 8;
      // XCD x owns `per` (+1 if x < rem) consecutive tiles
      const int start = x * per + min(x, rem);
      tile = start + q;
    }
  }
  const int tiles_m = (p.M + BM - 1) / BM;
  // column-major walk over tiles (consecutive tiles share the B columns)
  const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;
  if (p.skip_upper && n0 > m0 + BM - 1) return;
  const int z = blockIdx.y, z1 = z / p.nb2, z2 = z % p.nb2;
  const int64_t offA = z1 * p.sA1 + z2 * p.sA2, offB = z1 * p.sB1 + z2 * p.sB2, offC = z1 * p.sC1 + z2 * p.sC2;
  int kbeg = 0, kend = p.K;
  if (p.klimit == 1) kend = min(p.K, m0 + BM);
  if (p.klimit == 2) kbeg = (m0 / KT) * KT;
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
  const int ks = blockIdx.z, nks = gridDim.z;
  const int it0 = (int)((int64_t)total * ks / nks), it1 = (int)((int64_t)total * (ks + 1) / nks);

  auto issue = [&](int it, int buf) {
    const int term = it / nfull, k0 = kbeg + (it % nfull) * KT;
    const bf16* A = (const bf16*)p.A[term] + offA;
    const bf16* B = (const bf16*)p.B[term] + offB;
    HF_LDS bf16* sa = smem + buf * STAGE;
    slab_issue<BM, AKC>(A, p.lda, m0, k0, p.M, sa, wave, lane);
    slab_issue<BN, BKC>(B, p.ldb, n0, k0, p.N, sa + A_EL, wave, lane);
  };
  auto compute = [&](int buf) {
    const HF_LDS bf16* sa = smem + buf * STAGE;
    const HF_LDS bf16* sb = sa + A_EL;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = frag_read<BM, AKC>(sa, wm0 + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = frag_read<BN, BKC>(sb, wn0 + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  if (it0 < it1) issue(it0, 0);
  for (int it = it0; it < it1; ++it) {
    const int buf = (it - it0) & 1;
    if (it + 1 < it1) {
      issue(it + 1, buf ^ 1);
      HF_WAIT_VMCNT(NLOAD);
    } else {
      HF_WAIT_VMCNT(0);
    }
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    compute(buf);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
  }
  // ragged k remainder (handled by the last split only)
  if (ktail > 0 && ks == nks - 1) {
    for (int term = 0; term < nterm; ++term) {
      const bf16* A = (const bf16*)p.A[term] + offA;
      const bf16* B = (const bf16*)p.B[term] + offB;
      const int k0 = kbeg + nfull * KT;
      __syncthreads();
      slab_guarded<BM, AKC>(A, p.lda, m0, k0, p.M, kend, smem, t);
      slab_guarded<BN, BKC>(B, p.ldb, n0, k0, p.N, kend, smem + A_EL, t);
      __syncthreads();
      compute(0);
    }
  }

  // epilogue: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane/32) + r%4
  const bool first = (ks == 0);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int gn = n0 + wn0 + j * 32 + (lane & 31);
    if (gn >= p.N) continue;
    float bsum = 0.f;
    if (first) {
      if (p.bias) bsum += p.bias_bf16 ? (float)((const bf16*)p.bias)[gn] : ((const float*)p.bias)[gn];
      if (p.bias_t) bsum += p.bias_t[gn];
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (gm >= p.M) continue;
        float v = p.alpha * acc[i][j][r] + bsum;
        const int64_t ci = offC + (int64_t)gm * p.ldc + gn;
        if (nks > 1) {
          atomicAdd((float*)p.C + ci, v);  // C was zero-filled (or holds Cadd) by the launcher
        } else {
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
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB>
static hipError_t launch_one(const GemmP& p, dim3 grid, hipStream_t st) {
  constexpr int smem = 2 * (BM + BN) * KT * 2;
  static bool attr_done = false;
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, TA, TB>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const GemmP& p, dim3 grid, hipStream_t st) {
  if (!p.transA && !p.transB) return launch_one<BM, BN, WM, WN, false, false>(p, grid, st);
  if (!p.transA && p.transB) return launch_one<BM, BN, WM, WN, false, true>(p, grid, st);
  if (p.transA && !p.transB) return launch_one<BM, BN, WM, WN, true, false>(p, grid, st);
  return launch_one<BM, BN, WM, WN, true, true>(p, grid, st);
}

// Tile choice: the largest tile that still yields about two blocks per CU;
// split-K for products with few output tiles and a long k (the H v blocks).
hipError_t launch_gemm_mfma(GemmP p, int nb, int allow_splitk, int force_cfg, int force_ks, hipStream_t st) {
  const int64_t M = p.M, N = p.N;
  auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn) * (int64_t)nb; };
  int cfg;
  if (force_cfg >= 0) cfg = force_cfg;
  else if (tiles(256, 256) >= 384) cfg = 0;
  else if (tiles(256, 128) >= 320) cfg = 1;
  else cfg = 2;
  const int bm = cfg == 2 ? 128 : 256, bn = cfg == 0 ? 256 : 128;
  const int64_t nt = tiles(bm, bn);
  int ks = 1;
  if (force_ks > 0) ks = force_ks;
  else if (allow_splitk && !p.out_bf16 && !p.klimit && nt < 384) {
    const int slabs = p.nterm * (p.K / KT);
    ks = (int)std::min<int64_t>(std::max<int64_t>(1, (512 + nt - 1) / nt), std::max(1, slabs / 4));
    ks = std::min(ks, 16);
  }
  if (ks > 1) {
    // accumulate with atomics on top of Cadd (or zero)
    // (caller guarantees fp32 C; the fill is one small kernel)
    if (p.Cadd == nullptr) {
      // zero-fill C rows
      if (p.ldc == p.N && nb == 1) {
        hipError_t e = launch_fill_f32((float*)p.C, M * N, 0.f, st);
        if (e != hipSuccess) return e;
      } else {
        ks = 1;
      }
    } else if (p.Cadd != (const float*)p.C) {
      ks = 1;
    }
  }
  p.tiles_n = (int)((N + bn - 1) / bn);
  dim3 grid((unsigned)(nt / nb), (unsigned)nb, (unsigned)ks);
  if (cfg == 0) return launch_cfg<256, 256, 128, 128>(p, grid, st);
  if (cfg == 1) return launch_cfg<256, 128, 128, 64>(p, grid, st);
  return launch_cfg<128, 128, 64, 64>(p, grid, st);
}

}  // namespace hf
