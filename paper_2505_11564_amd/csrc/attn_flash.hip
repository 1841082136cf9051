// Causal softmax attention with its tangent, streamed tile by tile (bf16 operands, fp32
// accumulation): forward, and the backward sweep that recomputes the probabilities from saved row
// statistics, so that no S x S tensor ever reaches memory.  Section "Distributed Pearlmutter"
// (Algorithm 1) of the paper disables fused attention because its autograd kernel has no double
// backward; here the second-order terms are written out, per (batch, head), with c = 1/sqrt(dh):
//   S = c Q K^T            S_t = c (Q_t K^T + Q K_t^T)
//   P = softmax(S)         P_t = P (S_t - r),  r = rowsum(P S_t)
//   O = P V                O_t = P_t V + P V_t
//   dV = P^T dO            dV_t = P_t^T dO + P^T dO_t
//   dP = dO V^T            dP_t = dO_t V^T + dO V_t^T
//   dS = P (dP - delta)    dS_t = P_t (dP - delta) + P (dP_t - delta_t)
//   dQ = c dS K            dQ_t = c (dS_t K + dS K_t)
//   dK = c dS^T Q          dK_t = c (dS_t^T Q + dS^T Q_t)
// delta = rowsum(P dP) = <dO, O> and delta_t = <dO_t, O> + <dO, O_t> come from attn_delta_kernel.
// The primal scores and P V take the low-order halves of their bf16 operands as extra terms
// (A_hi B_hi + A_lo B_hi + A_hi B_lo); tangents and adjoints use the high halves.
//
// Kernel shapes (v_mfma_f32_32x32x16_bf16, 4 wavefronts of 64 lanes per block):
//   forward, dQ : a block owns 128 queries (32 per wave) of one head and walks the key tiles
//                 0 .. diagonal, 32 keys at a time, staged in LDS.  The products are formed
//                 transposed, S^T = K Q^T (32 keys x 32 queries per wave): the accumulator layout
//                 then has one query per lane (rows = keys spread over the 16 registers), so the
//                 softmax statistics are per lane plus one exchange between the lane halves, and
//                 the probabilities are already the B operand (k = keys) of O^T = V^T P^T; the
//                 k index of that product is a permutation of the keys that the A operand (V^T,
//                 read from LDS with transposing reads) follows.
//   dK, dV      : a block owns 128 keys (32 per wave) of one key/value head and walks the query
//                 tiles diagonal .. end (and the query heads of its group), with S = Q K^T formed
//                 untransposed so that one key sits per lane and P, dS are the B operands of
//                 dV^T = dO^T P and dK^T = Q^T dS.
// Online softmax: running maximum m, sum l and tangent sum per query; the forward saves
// (m + log l, r) per row, the backward recomputes P = exp(S - lse), P_t = P (S_t - r).
#include "gemm_mfma_common.h"

namespace hf {

namespace {

#define HF_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)
typedef unsigned at_u32x4 __attribute__((ext_vector_type(4)));
typedef float at_f32x4 __attribute__((ext_vector_type(4)));

// LDS tile of 32 rows x DH bf16, rows contiguous.  Two permutations of a row's 16-byte chunks:
// kc for tiles read as fragments with one tile row per lane (16 consecutive rows at one chunk
// index fall on 16 different bank groups), rc for tiles read with transposing reads (four
// consecutive rows at one column fall on four different quarters of the banks).
template <int DH>
__device__ __forceinline__ int kc_off(int r, int c) { return r * DH + ((c ^ ((r / (128 / DH)) & (DH / 8 - 1))) << 3); }
template <int DH>
__device__ __forceinline__ int rc_off(int r, int c) { return r * DH + ((c ^ rc_rot(r, DH)) << 3); }

// Fragment with tile rows on lanes: lane holds row lane % 32, columns kk*16 + (lane/32)*8 .. +8.
template <int DH>
__device__ __forceinline__ bf16x8 frag_rows(const HF_LDS bf16* tile, int lane, int kk) {
  return *(const HF_LDS bf16x8*)(tile + kc_off<DH>(lane & 31, kk * 2 + (lane >> 5)));
}
// Fragment with tile columns on lanes (the tile transposed): lane holds column rt*32 + lane % 32 and,
// as its 8 values, the tile rows ks*16 + {4G .. 4G+3, 8+4G .. 8+4G+3}, G = lane / 32: the order in
// which a 32x32 accumulator holds its rows in registers 8 ks .. 8 ks + 7 (row of register v:
// 8 (v/4) + 4 G + v % 4), so an accumulator tile converted to bf16 multiplies against it directly.
template <int DH>
__device__ __forceinline__ bf16x8 frag_cols(const HF_LDS bf16* tile, int lane, int rt, int ks) {
  const int i = lane & 15, g = lane >> 4;
  const int kq = ks * 16 + (g >> 1) * 4 + (i >> 2);
  const int c = rt * 32 + (g & 1) * 16 + (i & 3) * 4;
  const HF_LDS bf16* p0 = tile + kq * DH + ((((c >> 3) ^ rc_rot(kq, DH))) << 3) + (c & 7);
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((HF_LDS bf16x4*)p0);
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((HF_LDS bf16x4*)(p0 + 8 * DH));  // rows + 8: same rotation
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ bf16x8 pack8(const float* x) {
  bf16x8 v;
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = (bf16)x[j];
  return v;
}

// Global -> registers -> LDS staging of NT tiles of 32 rows x DH (16 bytes per thread and step;
// rows beyond rmax are clamped to the last valid row and masked by the caller).
template <int DH>
struct StageDim {
  static constexpr int CH = 4 * DH;               // 16-byte chunks per tile
  static constexpr int PER = (CH + 255) / 256;    // chunks per thread and tile
};
template <int DH, int I>
__device__ __forceinline__ void stage_load_one(at_u32x4 (&pre)[StageDim<DH>::PER], const bf16* src, int64_t ld, int r0, int rmax, int t) {
  constexpr int CH = StageDim<DH>::CH, PER = StageDim<DH>::PER;
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int idx = t + 256 * u;
    if (CH >= 256 || idx < CH) {
      const int row = idx / (DH / 8), c = idx % (DH / 8);
      const int rr = min(r0 + row, rmax - 1);
      pre[u] = *(const at_u32x4*)(src + (int64_t)rr * ld + c * 8);
    }
  }
}
// kc_tile / rc_tile: LDS tile that takes the chunks in the kc / rc permutation (-1: none)
template <int DH, int KC_TILE, int RC_TILE>
__device__ __forceinline__ void stage_store_one(const at_u32x4 (&pre)[StageDim<DH>::PER], HF_LDS bf16* sm, int t) {
  constexpr int CH = StageDim<DH>::CH, PER = StageDim<DH>::PER;
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int idx = t + 256 * u;
    if (CH >= 256 || idx < CH) {
      const int row = idx / (DH / 8), c = idx % (DH / 8);
      if (KC_TILE >= 0) *(HF_LDS at_u32x4*)(sm + KC_TILE * (32 * DH) + kc_off<DH>(row, c)) = pre[u];
      if (RC_TILE >= 0) *(HF_LDS at_u32x4*)(sm + RC_TILE * (32 * DH) + rc_off<DH>(row, c)) = pre[u];
    }
  }
}

// Four consecutive columns (col .. col+3) of row `row` of a [rows, ld] result, bf16 or fp32.
__device__ __forceinline__ void store4(void* base, int f32, int64_t row, int64_t ld, int col, float a, float b, float c, float d) {
  if (f32) {
    *(float4*)((float*)base + row * ld + col) = make_float4(a, b, c, d);
  } else {
    const bf16 o[4] = {(bf16)a, (bf16)b, (bf16)c, (bf16)d};
    *(uint2*)((bf16*)base + row * ld + col) = *(const uint2*)o;
  }
}

// block -> (batch * head index, tile rank): whole heads per XCD (launch order L goes to XCD L % 8, so
// head hh runs on XCD hh % 8 and its operands stay in that L2).  Rank 0 is a head's longest tile
// (work falls linearly with the rank), and the slots s = L / 8 of an XCD take the (head, rank) items
// longest first, which is what balances a launch whose later blocks start as earlier ones end.
// A launch of at most two resident blocks per CU starts all at once instead: the slots go round
// the XCD's 32 CUs (measured: slots s and s + 32 share a CU), so with N <= 64 items the 64 - N
// longest run alone and the others in pairs of a longer and a shorter one.
__device__ __forceinline__ bool block_map(int nheads, int ntiles, int occ, int& hh, int& tile) {
  constexpr int C = 32;  // CUs per XCD
  const int L = blockIdx.x, xcd = L & 7, s = L >> 3;
  const int nhx = (nheads + 7) >> 3, N = nhx * ntiles;
  int i = s;
  if (occ == 2 && N > C && N <= 2 * C) {
    const int P = N - C;  // CUs with two blocks: slots [0, P) and [C, N)
    i = s < P ? (2 * C - N) + s : (s < C ? s - P : N - 1 - (s - C));
  }
  tile = i / nhx;
  hh = (i % nhx) * 8 + xcd;
  return hh < nheads;
}

}  // namespace

// ---- direct global -> LDS staging and hand-scheduled fragment reads ------------------------
// A stage is a run of tiles (32 rows x DH, 64*DH bytes each); one global_load_lds instruction fills
// 1 KB of it (64 lanes x 16 bytes, consecutive), so instruction q of a stage covers bytes
// [q KB, (q+1) KB): tile q / (DH/16), chunks (q % (DH/16)) * 64 + lane.  The chunk permutation of
// a tile is applied on the source side: the lane that fills chunk slot s of row r fetches the
// logical chunk s ^ swz(r).  Wave w issues the instructions q = w, w + 4, ...
template <int DH>
struct LdsLoad {
  static constexpr int NI_T = DH / 16, CPR = DH / 8, RPI = 64 / CPR;
  // With a = q % NI_T, b = lane / CPR, slot = lane % CPR the lane fetches row a RPI + b and the chunk
  // slot ^ swz(row); both permutations split into a lane part and a part of a alone (rows on lanes:
  // swz = ((4 a) & (CPR - 1)) | b / (128 / DH); transposing reads: swz depends on b alone), so one
  // packed register per lane serves every instruction: b | (chunk, rows on lanes) << 8 | (chunk,
  // transposing reads) << 16.
  __device__ static __forceinline__ uint32_t lane_part(int lane) {
    const int b = lane / CPR, slot = lane % CPR;
    return (uint32_t)(b | ((slot ^ (b / (128 / DH))) << 8) | ((slot ^ rc_rot(b, DH)) << 16));
  }
  // row (0..31) and column (elements) for instruction q; rc: the tile is one for transposing reads
  __device__ static __forceinline__ void lane_chunk(uint32_t lp, int q, bool rc, int& row, int& col) {
    const int a = q % NI_T;
    row = a * RPI + (int)(lp & 255u);
    col = (int)((rc ? (lp >> 16) & 255u : ((lp >> 8) & 255u) ^ (uint32_t)((4 * a) & (CPR - 1))) << 3);
  }
};
// addr ^ IMM, kept where it is written (the fragment addresses of the k-steps and column tiles differ
// from the first one by one flipped bit field; forming them at the point of use costs an instruction
// and saves the registers that would hold them across the loop)
template <int IMM>
__device__ __forceinline__ uint32_t lds_xor(uint32_t addr) {
  if constexpr (IMM == 0) return addr;
  uint32_t r;
  asm volatile("v_xor_b32 %0, %1, %2" : "=v"(r) : "n"(IMM), "v"(addr));
  return r;
}
// Places a fragment in the accumulator half of the register file at this point (matrix instructions
// read their operands from either half; everything else needs the other one).
__device__ __forceinline__ void agpr_pin(bf16x8& v) { asm volatile("" : "+a"(v)); }
// Tile filled by load instruction wave + 4 i (NI_T instructions per tile): a constant of i wherever a
// tile takes a multiple of four instructions.
template <int NI_T>
__device__ __forceinline__ int tile_of(int wave, int i) { return NI_T % 4 == 0 ? (4 * i) / NI_T : (wave + 4 * i) / NI_T; }
template <int N>
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }

// Per-lane LDS byte offsets (relative to a tile) of the fragments a wave reads:
//   rows on lanes, k-step kk   : (kc_off(lane % 32, 2 kk + lane / 32)) * 2
//   columns on lanes, row tile rt : the address of frag_cols at ks = 0; ks adds 16 * DH * 2 bytes,
//                                   the second transposing read 8 * DH * 2 more
template <int DH>
__device__ __forceinline__ uint32_t addr_rows(int lane, int kk) { return (uint32_t)(kc_off<DH>(lane & 31, kk * 2 + (lane >> 5)) * 2); }
template <int DH>
__device__ __forceinline__ uint32_t addr_cols(int lane, int rt) {
  const int i = lane & 15, g = lane >> 4;
  const int kq = (g >> 1) * 4 + (i >> 2);
  const int c = rt * 32 + (g & 1) * 16 + (i & 3) * 4;
  return (uint32_t)((kq * DH + ((((c >> 3) ^ rc_rot(kq, DH))) << 3) + (c & 7)) * 2);
}

// ------------------------------------------------------------------ forward ----
// Two LDS stages of six tiles (K hi / lo / t with keys on lanes, V hi / lo / t for transposing
// reads), filled by direct global -> LDS loads one key tile ahead; one barrier per key tile.
// Fragment reads are issued one step ahead of the matrix instructions that use them.
// Online softmax with a lazy reference maximum: the running maximum is only moved (and the
// accumulators rescaled) when a tile exceeds it by more than 8, which keeps exp() below e^8.

// LO: the primal operands come as pairs of a high and a low half (extra terms, extra tiles).
template <int DH, bool LO>
__global__ __launch_bounds__(256, (DH <= 64 ? 2 : 1)) void attn_fwd_kernel(const AttnP p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  // tiles of a stage: K hi / (lo) / t with keys on lanes, V hi / (lo) / t for transposing reads
  constexpr int T_KD = LO ? 2 : 1, T_VH = LO ? 3 : 2, T_VL = 4, T_VD = LO ? 5 : 3, NT = LO ? 6 : 4;
  constexpr int TILE_B = 64 * DH, STAGE_B = NT * TILE_B, KS = DH / 16, RT = DH / 32;
  constexpr int NI = NT * (DH / 16) / 4;  // load instructions per wave and stage
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6) & 3;  // (masked so that tile indices below fold)
  const int nqt = (p.S + 127) / 128;
  int hh, tile;
  if (!block_map(p.B * p.H, nqt, DH <= 64 ? 2 : 1, hh, tile)) return;
  const int qt = nqt - 1 - tile;  // long rows first
  const int b = hh / p.H, h = hh % p.H, hk = h / p.grp;
  const int m0 = qt * 128, mw = m0 + wave * 32;
  const int64_t row0 = (int64_t)b * p.S;
  const int mq = mw + (lane & 31);            // this lane's query
  const int qm = min(mq, p.S - 1);

  bf16x8 qh[KS], ql[LO ? KS : 1], qd[KS];
  {
    const int64_t off = (row0 + qm) * p.ldq + (int64_t)h * DH + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      qh[kk] = *(const bf16x8*)(p.qkv + off + kk * 16);
      if constexpr (LO) ql[kk] = *(const bf16x8*)(p.qkv_lo + off + kk * 16);
      qd[kk] = *(const bf16x8*)(p.qkv_t + off + kk * 16);
    }
  }
  const int64_t ok = row0 * p.ldq + p.offK + (int64_t)hk * DH, ov = row0 * p.ldq + p.offV + (int64_t)hk * DH;
  const bf16 *const sKh = p.qkv + ok, *const sKl = LO ? p.qkv_lo + ok : nullptr, *const sKd = p.qkv_t + ok, *const sVh = p.qkv + ov,
             *const sVl = LO ? p.qkv_lo + ov : nullptr, *const sVd = p.qkv_t + ov;
  const uint32_t lp = LdsLoad<DH>::lane_part(lane);
  HF_LDS char* const smem_c = (HF_LDS char*)smem_raw;
  auto issue = [&](int stage, int r0) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int T = tile_of<DH / 16>(wave, i);  // (wave-uniform)
      const bf16* base = T == 0 ? sKh : T == T_KD ? sKd : T == T_VH ? sVh : T == T_VD ? sVd : (T == 1 ? sKl : sVl);
      int row, col;
      LdsLoad<DH>::lane_chunk(lp, wave + 4 * i, T >= T_VH, row, col);
      const int rr = min(r0 + row, p.S - 1);
      __builtin_amdgcn_global_load_lds((const void*)(base + ((int64_t)rr * p.ldq + col)),
                                       (HF_LDS void*)(smem_c + stage * STAGE_B + (wave + 4 * i) * 1024), 16, 0, 0);
    }
  };
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem_c;
  const uint32_t adK0 = lds0 + addr_rows<DH>(lane, 0), adV0 = lds0 + addr_cols<DH>(lane, 0);  // k-step kk: ^ kk << 5, column tile rt: ^ rt << 6

  f32x16 o[RT], a1[RT];
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) { o[i][v] = 0.f; a1[i][v] = 0.f; }
  float m_run = -INFINITY, l_run = 0.f, rs_run = 0.f;

  // the work of one key tile held in LDS stage S (compile-time)
  auto compute = [&](auto S_c, int n0) {
    constexpr int SB = decltype(S_c)::value * STAGE_B;
    f32x16 st, su;
#pragma unroll
    for (int v = 0; v < 16; ++v) { st[v] = 0.f; su[v] = 0.f; }
    bf16x8 kh[2], kl[2], kd[2];
    kh[0] = lds_read_b128<SB>(adK0); kd[0] = lds_read_b128<SB + T_KD * TILE_B>(adK0);
    if constexpr (LO) kl[0] = lds_read_b128<SB + TILE_B>(adK0);
    static_for<KS>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value, c = kk & 1, nx = c ^ 1;
      if constexpr (kk + 1 < KS) {
        const uint32_t ad = lds_xor<((kk + 1) << 5)>(adK0);
        kh[nx] = lds_read_b128<SB>(ad); kd[nx] = lds_read_b128<SB + T_KD * TILE_B>(ad);
        if constexpr (LO) kl[nx] = lds_read_b128<SB + TILE_B>(ad);
        lds_wait<(LO ? 3 : 2)>();
      } else {
        lds_wait<0>();
      }
      lds_tie(kh[c]); lds_tie(kd[c]);
      if constexpr (LO) lds_tie(kl[c]);
      st = HF_MFMA(kh[c], qh[kk], st);
      su = HF_MFMA(kd[c], qh[kk], su);
      if constexpr (LO) st = HF_MFMA(kl[c], qh[kk], st);
      su = HF_MFMA(kh[c], qd[kk], su);
      if constexpr (LO) st = HF_MFMA(kh[c], ql[kk], st);
      __builtin_amdgcn_sched_barrier(0);
    });
    // first V fragments on their way while the softmax arithmetic runs
    bf16x4 vh[2][2], vl[2][2], vd[2][2];
    auto req_v = [&](auto s_c, auto set_c) {
      constexpr int s = decltype(s_c)::value, set = decltype(set_c)::value;
      constexpr int rt = s % RT, ks = s / RT, OFF = SB + ks * 16 * DH * 2;
      const uint32_t ad = lds_xor<(rt << 6)>(adV0);
      vh[set][0] = lds_read_tr64<OFF + T_VH * TILE_B>(ad); vh[set][1] = lds_read_tr64<OFF + T_VH * TILE_B + 8 * DH * 2>(ad);
      vd[set][0] = lds_read_tr64<OFF + T_VD * TILE_B>(ad); vd[set][1] = lds_read_tr64<OFF + T_VD * TILE_B + 8 * DH * 2>(ad);
      if constexpr (LO) { vl[set][0] = lds_read_tr64<OFF + T_VL * TILE_B>(ad); vl[set][1] = lds_read_tr64<OFF + T_VL * TILE_B + 8 * DH * 2>(ad); }
    };
    req_v(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    // register v of this lane: key n0 + 8 (v/4) + 4 (lane/32) + v%4 against query mq
    float s[16], eu[16];
    float mx = -INFINITY;
    const bool diag = n0 + 31 > mw;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = n0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      s[v] = st[v] * p.scale;
      if (diag && key > mq) s[v] = -INFINITY;
      mx = fmaxf(mx, s[v]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // finite: key n0 <= mw <= mq is never masked
    if (__any(mx > m_run + 8.f)) {
      const float m_new = mx > m_run + 8.f ? mx : m_run;
      const float alpha = __expf(m_run - m_new);  // 0 on the first tile, 1 for lanes that keep their maximum
      l_run *= alpha;
      rs_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) { o[i][v] *= alpha; a1[i][v] *= alpha; }
    }
    float ls = 0.f, rsum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s[v] = __expf(s[v] - m_run);
      eu[v] = s[v] * (su[v] * p.scale);
      ls += s[v];
      rsum += eu[v];
    }
    l_run += ls;
    rs_run += rsum;
    bf16x8 eh[2], el[2], es[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      float lo8[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bf16 hi = (bf16)s[ks * 8 + j];
        eh[ks][j] = hi;
        lo8[j] = s[ks * 8 + j] - (float)hi;
      }
      if constexpr (LO) el[ks] = pack8(lo8);
      es[ks] = pack8(eu + ks * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
    static_for<2 * RT>([&](auto s_c) {
      constexpr int sI = decltype(s_c)::value, c = sI & 1, rt = sI % RT, ks = sI / RT;
      if constexpr (sI + 1 < 2 * RT) {
        req_v(std::integral_constant<int, sI + 1>{}, std::integral_constant<int, c ^ 1>{});
        lds_wait<(LO ? 6 : 4)>();
      } else {
        lds_wait<0>();
      }
      lds_tie(vh[c][0]); lds_tie(vh[c][1]); lds_tie(vd[c][0]); lds_tie(vd[c][1]);
      const bf16x8 a_h = __builtin_shufflevector(vh[c][0], vh[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8 a_d = __builtin_shufflevector(vd[c][0], vd[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
      o[rt] = HF_MFMA(a_h, eh[ks], o[rt]);
      a1[rt] = HF_MFMA(a_h, es[ks], a1[rt]);
      if constexpr (LO) o[rt] = HF_MFMA(a_h, el[ks], o[rt]);
      a1[rt] = HF_MFMA(a_d, eh[ks], a1[rt]);
      if constexpr (LO) {
        lds_tie(vl[c][0]); lds_tie(vl[c][1]);
        const bf16x8 a_l = __builtin_shufflevector(vl[c][0], vl[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
        o[rt] = HF_MFMA(a_l, eh[ks], o[rt]);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  const int n_end = min(p.S, m0 + 128);
  const int nkt = (n_end + 31) / 32;
  issue(0, 0);
  for (int kt0 = 0; kt0 < nkt; kt0 += 2) {
    static_for<2>([&](auto s_c) {
      constexpr int S = decltype(s_c)::value;
      const int kt = kt0 + S;
      if (kt < nkt) {
        const int n0 = kt * 32;
        HF_WAIT_VMCNT(0);                 // this wave's part of tile kt has landed
        __builtin_amdgcn_s_barrier();     // everyone's has, and stage 1 - S has been read for the last time
        __builtin_amdgcn_sched_barrier(0);
        if (kt + 1 < nkt) issue(1 - S, n0 + 32);
        // (wave-uniform) keys beyond this wave's diagonal, or a wave without a valid query: nothing to do
        if (n0 <= mw + 31 && mw < p.S) compute(s_c, n0);
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  }
  if (mw >= p.S) return;
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  const float rs = rs_run + __shfl_xor(rs_run, 32, 64);
  if (mq >= p.S) return;
  const float inv = 1.f / l, r = rs * inv;
  const int64_t orow = row0 + mq;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int col = h * DH + rt * 32 + 8 * g4 + 4 * (lane >> 5);
      float x[4], xl[4], xt[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float ov_ = o[rt][g4 * 4 + q];
        x[q] = ov_ * inv;
        xl[q] = x[q] - (float)(bf16)x[q];
        xt[q] = (a1[rt][g4 * 4 + q] - r * ov_) * inv;
      }
      store4(p.o, 0, orow, p.ldo, col, x[0], x[1], x[2], x[3]);
      if constexpr (LO) store4(p.o_lo, 0, orow, p.ldo, col, xl[0], xl[1], xl[2], xl[3]);
      store4(p.o_t, 0, orow, p.ldo, col, xt[0], xt[1], xt[2], xt[3]);
    }
  }
  if (lane < 32) {
    float* sp = p.stat + (((int64_t)b * p.H + h) * p.S + mq) * 2;
    sp[0] = m_run + __logf(l);
    sp[1] = r;
  }
}

// ---------------------------------------------------------------- backward: dQ ----
// Staged like the forward kernel: two LDS stages of seven tiles (K hi / lo / t and V hi / t with keys
// on lanes for the score-shaped products, K hi / t once more in the layout of transposing reads for
// dQ^T = K^T dS^T), filled by direct loads one key tile ahead, one barrier per key tile.

template <int DH, bool LO>
__global__ __launch_bounds__(256, (DH <= 64 ? 2 : 1)) void attn_bwd_q_kernel(const AttnP p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  // tiles of a stage: K hi / (lo) / t, V hi / t with keys on lanes; K hi / t for transposing reads
  constexpr int T_KD = LO ? 2 : 1, T_VH = T_KD + 1, T_VD = T_KD + 2, T_KHT = T_KD + 3, T_KDT = T_KD + 4, NT = T_KD + 5;
  constexpr int TILE_B = 64 * DH, STAGE_B = NT * TILE_B, KS = DH / 16, RT = DH / 32;
  constexpr int NQ = NT * (DH / 16), NI = (NQ + 3) / 4;  // load instructions per stage, per wave
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6) & 3;
  const int nqt = (p.S + 127) / 128;
  int hh, tile;
  if (!block_map(p.B * p.H, nqt, DH <= 64 ? 2 : 1, hh, tile)) return;
  const int qt = nqt - 1 - tile;
  const int b = hh / p.H, h = hh % p.H, hk = h / p.grp;
  const int m0 = qt * 128, mw = m0 + wave * 32;
  const int64_t row0 = (int64_t)b * p.S;
  const int mq = mw + (lane & 31);
  const int qm = min(mq, p.S - 1);

  bf16x8 qh[KS], ql[LO ? KS : 1], qd[KS], gh[KS], gd[KS];
  {
    const int64_t off = (row0 + qm) * p.ldq + (int64_t)h * DH + (lane >> 5) * 8;
    const int64_t offg = (row0 + qm) * p.lddo + (int64_t)h * DH + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      qh[kk] = *(const bf16x8*)(p.qkv + off + kk * 16);
      if constexpr (LO) ql[kk] = *(const bf16x8*)(p.qkv_lo + off + kk * 16);
      qd[kk] = *(const bf16x8*)(p.qkv_t + off + kk * 16);
      gh[kk] = *(const bf16x8*)(p.dO + offg + kk * 16);
      gd[kk] = *(const bf16x8*)(p.dO_t + offg + kk * 16);
    }
  }
  const int64_t srow = ((int64_t)b * p.H + h) * p.S + qm;
  const float lse = p.stat[srow * 2], rr = p.stat[srow * 2 + 1];
  const float dl = p.delta[srow * 3], dlt = p.delta[srow * 3 + 1];

  const int64_t ok = row0 * p.ldq + p.offK + (int64_t)hk * DH, ov = row0 * p.ldq + p.offV + (int64_t)hk * DH;
  const bf16 *const sKh = p.qkv + ok, *const sKl = LO ? p.qkv_lo + ok : nullptr, *const sKd = p.qkv_t + ok, *const sVh = p.qkv + ov, *const sVd = p.qkv_t + ov;
  const uint32_t lp = LdsLoad<DH>::lane_part(lane);
  HF_LDS char* const smem_c = (HF_LDS char*)smem_raw;
  auto issue = [&](int stage, int r0) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + 4 * i;  // (wave-uniform)
      if (NQ % 4 == 0 || q < NQ) {
        const int T = tile_of<DH / 16>(wave, i);
        const bf16* base = (T == 0 || T == T_KHT) ? sKh : (T == T_KD || T == T_KDT) ? sKd : T == T_VH ? sVh : T == T_VD ? sVd : sKl;
        int row, col;
        LdsLoad<DH>::lane_chunk(lp, q, T >= T_KHT, row, col);
        const int rr_ = min(r0 + row, p.S - 1);
        __builtin_amdgcn_global_load_lds((const void*)(base + ((int64_t)rr_ * p.ldq + col)),
                                         (HF_LDS void*)(smem_c + stage * STAGE_B + q * 1024), 16, 0, 0);
      }
    }
  };
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem_c;
  const uint32_t adK0 = lds0 + addr_rows<DH>(lane, 0), adT0 = lds0 + addr_cols<DH>(lane, 0);  // k-step kk: ^ kk << 5, column tile rt: ^ rt << 6

  f32x16 dq[RT], dqt[RT];
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dq[i][v] = 0.f; dqt[i][v] = 0.f; }

  auto compute = [&](auto S_c, int n0) {
    constexpr int SB = decltype(S_c)::value * STAGE_B;
    f32x16 st, su, dp, dpt;
#pragma unroll
    for (int v = 0; v < 16; ++v) { st[v] = 0.f; su[v] = 0.f; dp[v] = 0.f; dpt[v] = 0.f; }
    bf16x8 kh[2], kl[2], kd[2], vh[2], vd[2];
    auto req_k = [&](auto kk_c, auto set_c) {
      constexpr int kk = decltype(kk_c)::value, set = decltype(set_c)::value;
      const uint32_t ad = lds_xor<(kk << 5)>(adK0);
      kh[set] = lds_read_b128<SB>(ad); kd[set] = lds_read_b128<SB + T_KD * TILE_B>(ad);
      vh[set] = lds_read_b128<SB + T_VH * TILE_B>(ad); vd[set] = lds_read_b128<SB + T_VD * TILE_B>(ad);
      if constexpr (LO) kl[set] = lds_read_b128<SB + TILE_B>(ad);
    };
    req_k(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    static_for<KS>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value, c = kk & 1;
      if constexpr (kk + 1 < KS) {
        req_k(std::integral_constant<int, kk + 1>{}, std::integral_constant<int, c ^ 1>{});
        lds_wait<(LO ? 5 : 4)>();
      } else {
        lds_wait<0>();
      }
      lds_tie(kh[c]); lds_tie(kd[c]); lds_tie(vh[c]); lds_tie(vd[c]);
      if constexpr (LO) lds_tie(kl[c]);
      st = HF_MFMA(kh[c], qh[kk], st);
      su = HF_MFMA(kd[c], qh[kk], su);
      dp = HF_MFMA(vh[c], gh[kk], dp);       // dP^T = V dO^T
      dpt = HF_MFMA(vh[c], gd[kk], dpt);     // dP_t^T = V dO_t^T + V_t dO^T
      if constexpr (LO) st = HF_MFMA(kl[c], qh[kk], st);
      su = HF_MFMA(kh[c], qd[kk], su);
      dpt = HF_MFMA(vd[c], gh[kk], dpt);
      if constexpr (LO) st = HF_MFMA(kh[c], ql[kk], st);
      __builtin_amdgcn_sched_barrier(0);
    });
    // first transposed fragments on their way while the pointwise arithmetic runs
    bf16x4 th[2][2], td[2][2];
    auto req_t = [&](auto s_c, auto set_c) {
      constexpr int sI = decltype(s_c)::value, set = decltype(set_c)::value;
      constexpr int rt = sI % RT, ks = sI / RT, OFF = SB + ks * 16 * DH * 2;
      const uint32_t ad = lds_xor<(rt << 6)>(adT0);
      th[set][0] = lds_read_tr64<OFF + T_KHT * TILE_B>(ad); th[set][1] = lds_read_tr64<OFF + T_KHT * TILE_B + 8 * DH * 2>(ad);
      td[set][0] = lds_read_tr64<OFF + T_KDT * TILE_B>(ad); td[set][1] = lds_read_tr64<OFF + T_KDT * TILE_B + 8 * DH * 2>(ad);
    };
    req_t(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    // register v of this lane: key n0 + 8 (v/4) + 4 (lane/32) + v%4 against query mq
    float ds[16], dst_[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = n0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const float pr = key > mq ? 0.f : __expf(st[v] * p.scale - lse);
      const float pt = pr * (su[v] * p.scale - rr);
      ds[v] = pr * (dp[v] - dl);
      dst_[v] = pt * (dp[v] - dl) + pr * (dpt[v] - dlt);
    }
    bf16x8 dsb[2], dtb[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) { dsb[ks] = pack8(ds + ks * 8); dtb[ks] = pack8(dst_ + ks * 8); }
    __builtin_amdgcn_sched_barrier(0);
    static_for<2 * RT>([&](auto s_c) {
      constexpr int sI = decltype(s_c)::value, c = sI & 1, rt = sI % RT, ks = sI / RT;
      if constexpr (sI + 1 < 2 * RT) {
        req_t(std::integral_constant<int, sI + 1>{}, std::integral_constant<int, c ^ 1>{});
        lds_wait<4>();
      } else {
        lds_wait<0>();
      }
      lds_tie(th[c][0]); lds_tie(th[c][1]); lds_tie(td[c][0]); lds_tie(td[c][1]);
      const bf16x8 kT = __builtin_shufflevector(th[c][0], th[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8 kdT = __builtin_shufflevector(td[c][0], td[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
      dq[rt] = HF_MFMA(kT, dsb[ks], dq[rt]);
      dqt[rt] = HF_MFMA(kT, dtb[ks], dqt[rt]);
      dqt[rt] = HF_MFMA(kdT, dsb[ks], dqt[rt]);
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  const int n_end = min(p.S, m0 + 128);
  const int nkt = (n_end + 31) / 32;
  issue(0, 0);
  for (int kt0 = 0; kt0 < nkt; kt0 += 2) {
    static_for<2>([&](auto s_c) {
      constexpr int S = decltype(s_c)::value;
      const int kt = kt0 + S;
      if (kt < nkt) {
        const int n0 = kt * 32;
        HF_WAIT_VMCNT(0);                 // this wave's part of tile kt has landed
        __builtin_amdgcn_s_barrier();     // everyone's has, and stage 1 - S has been read for the last time
        __builtin_amdgcn_sched_barrier(0);
        if (kt + 1 < nkt) issue(1 - S, n0 + 32);
        if (n0 <= mw + 31 && mw < p.S) compute(s_c, n0);
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  }
  if (mq >= p.S) return;
  const int64_t orow = row0 + mq;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int col = h * DH + rt * 32 + 8 * g4 + 4 * (lane >> 5);
      store4(p.dq, p.dq_f32, orow, p.lddq, col, dq[rt][g4 * 4] * p.scale, dq[rt][g4 * 4 + 1] * p.scale, dq[rt][g4 * 4 + 2] * p.scale,
             dq[rt][g4 * 4 + 3] * p.scale);
      store4(p.dq_t, p.dq_f32, orow, p.lddq, col, dqt[rt][g4 * 4] * p.scale, dqt[rt][g4 * 4 + 1] * p.scale,
             dqt[rt][g4 * 4 + 2] * p.scale, dqt[rt][g4 * 4 + 3] * p.scale);
    }
  }
}

// ------------------------------------------------------------ backward: dK, dV ----
// WHAT & 1: dV, dV_t;  WHAT & 2: dK, dK_t.
// LDS: two stages of up to nine tiles, filled by direct loads one query tile ahead -- Q hi / lo / t
// with queries on lanes; dO, dO_t the same (dK only); copies of Q hi / t (dK) and of dO, dO_t (dV) in
// the layout of transposing reads -- and two small tiles of row statistics (lse, r, delta, delta_t
// per query), which go through registers two tiles ahead.  One barrier per query tile; the tiles of
// all query heads of a group form one sequence.

template <int DH, int WHAT, bool LO>
struct KvTiles {
  static constexpr bool DV = (WHAT & 1) != 0, DK = (WHAT & 2) != 0;
  static constexpr int T_QH = 0, T_QL = LO ? 1 : -1, T_QD = LO ? 2 : 1;
  static constexpr int T_GH = DK ? T_QD + 1 : -1, T_GD = DK ? T_QD + 2 : -1;
  static constexpr int NKC = T_QD + 1 + (DK ? 2 : 0);       // tiles with queries on lanes
  static constexpr int T_QHT = DK ? NKC : -1, T_QDT = DK ? NKC + 1 : -1;
  static constexpr int T_GHT = DV ? NKC + (DK ? 2 : 0) : -1, T_GDT = DV ? NKC + (DK ? 2 : 0) + 1 : -1;
  static constexpr int NT = NKC + (DK ? 2 : 0) + (DV ? 2 : 0);
  static constexpr int TILE_B = 64 * DH, STAGE_B = NT * TILE_B;
  static constexpr int STATS_B = 32 * 4 * 4;                // one statistics tile
  static constexpr int LDS_B = 2 * STAGE_B + 2 * STATS_B;
  // source of a tile: 0 Q hi, 1 Q lo, 2 Q t, 3 dO, 4 dO t
  __device__ static constexpr int src(int T) {
    return T == T_QH || T == T_QHT ? 0 : T == T_QL ? 1 : T == T_QD || T == T_QDT ? 2 : T == T_GH || T == T_GHT ? 3 : 4;
  }
};

template <int DH, int WHAT, bool LO>
__global__ __launch_bounds__(256, (DH <= 32 ? 2 : 1)) void attn_bwd_kv_kernel(const AttnP p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  typedef KvTiles<DH, WHAT, LO> L;
  constexpr bool DV = L::DV, DK = L::DK;
  constexpr int TILE_B = L::TILE_B, STAGE_B = L::STAGE_B, KS = DH / 16, RT = DH / 32;
  constexpr int NQ = L::NT * (DH / 16), NI = (NQ + 3) / 4;
  HF_LDS char* const smem_c = (HF_LDS char*)smem_raw;
  HF_LDS float* const stats = (HF_LDS float*)(smem_c + 2 * STAGE_B);  // [2][32 queries][4]

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6) & 3;
  const int nkb = (p.S + 127) / 128;
  const int Hkv = p.H / p.grp;
  int hh, kb;
  if (!block_map(p.B * Hkv, nkb, DH <= 32 ? 2 : 1, hh, kb)) return;  // key block 0 (the longest) first
  const int b = hh / Hkv, hk = hh % Hkv;
  const int k0 = kb * 128, kw = k0 + wave * 32;
  const int64_t row0 = (int64_t)b * p.S;
  const int nk = kw + (lane & 31);            // this lane's key
  const int nkc = min(nk, p.S - 1);

  bf16x8 kh[KS], kl[LO ? KS : 1], kd[KS], vh[DK ? KS : 1], vd[DK ? KS : 1];
  {
    const int64_t off = (row0 + nkc) * p.ldq + (int64_t)hk * DH + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      kh[kk] = *(const bf16x8*)(p.qkv + p.offK + off + kk * 16);
      if constexpr (LO) kl[kk] = *(const bf16x8*)(p.qkv_lo + p.offK + off + kk * 16);
      kd[kk] = *(const bf16x8*)(p.qkv_t + p.offK + off + kk * 16);
      if (DK) {
        vh[kk] = *(const bf16x8*)(p.qkv + p.offV + off + kk * 16);
        vd[kk] = *(const bf16x8*)(p.qkv_t + p.offV + off + kk * 16);
      }
    }
    if constexpr (DH == 128) {  // 160 registers of loop constants that only matrix instructions read: the accumulator file
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        agpr_pin(kh[kk]); agpr_pin(kd[kk]);
        if constexpr (LO) agpr_pin(kl[kk]);
        if (DK) { agpr_pin(vh[kk]); agpr_pin(vd[kk]); }
      }
    }
  }
  f32x16 dv[DV ? RT : 1], dvt[DV ? RT : 1], dk[DK ? RT : 1], dkt[DK ? RT : 1];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
#pragma unroll
    for (int i = 0; i < (DV ? RT : 1); ++i) { dv[i][v] = 0.f; dvt[i][v] = 0.f; }
#pragma unroll
    for (int i = 0; i < (DK ? RT : 1); ++i) { dk[i][v] = 0.f; dkt[i][v] = 0.f; }
  }
  const int nqs = (p.S - k0 + 31) / 32;  // query sub-tiles k0, k0 + 32, ... (k0 < S) of one head
  const int nit = nqs * p.grp;           // ... of all query heads of the group

  const uint32_t lp = LdsLoad<DH>::lane_part(lane);
  const bf16 *const pq = p.qkv, *const pql = LO ? p.qkv_lo : nullptr, *const pqt = p.qkv_t, *const pg = p.dO, *const pgt = p.dO_t;
  const int64_t ldq = p.ldq, lddo = p.lddo;
  auto issue = [&](int stage, int it) {
    const int j = it / nqs, r0 = k0 + (it - j * nqs) * 32;
    const int h = hk * p.grp + j;
    const int64_t oq = row0 * ldq + (int64_t)h * DH, og = row0 * lddo + (int64_t)h * DH;
    const bf16 *const sQh = pq + oq, *const sQl = pql + oq, *const sQd = pqt + oq, *const sGh = pg + og, *const sGd = pgt + og;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + 4 * i;  // (wave-uniform)
      if (NQ % 4 == 0 || q < NQ) {
        const int T = tile_of<DH / 16>(wave, i), sr = L::src(T);
        const bf16* base = sr == 0 ? sQh : sr == 1 ? sQl : sr == 2 ? sQd : sr == 3 ? sGh : sGd;
        const int64_t ld = sr >= 3 ? lddo : ldq;
        int row, col;
        LdsLoad<DH>::lane_chunk(lp, q, T >= L::NKC, row, col);
        const int rr_ = min(r0 + row, p.S - 1);
        __builtin_amdgcn_global_load_lds((const void*)(base + (rr_ * ld + col)),
                                         (HF_LDS void*)(smem_c + stage * STAGE_B + q * 1024), 16, 0, 0);
      }
    }
  };
  at_f32x4 spre = {0.f, 0.f, 0.f, 0.f};
  auto load_stats = [&](int it) {  // (threads 0..31)
    const int j = it / nqs, q0 = k0 + (it - j * nqs) * 32;
    const int64_t sbase = ((int64_t)b * p.H + hk * p.grp + j) * p.S;
    const int q = min(q0 + t, p.S - 1);
    spre = at_f32x4{p.stat[(sbase + q) * 2], p.stat[(sbase + q) * 2 + 1], p.delta[(sbase + q) * 3], p.delta[(sbase + q) * 3 + 1]};
  };
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem_c;
  const uint32_t adQ0 = lds0 + addr_rows<DH>(lane, 0), adT0 = lds0 + addr_cols<DH>(lane, 0);  // k-step kk: ^ kk << 5, column tile rt: ^ rt << 6

  auto compute = [&](auto S_c, int q0) {
    constexpr int SI = decltype(S_c)::value, SB = SI * STAGE_B;
    f32x16 st, su, dp, dpt;
#pragma unroll
    for (int v = 0; v < 16; ++v) { st[v] = 0.f; su[v] = 0.f; dp[v] = 0.f; dpt[v] = 0.f; }
    bf16x8 qa[2], qb[2], qc[2], ga[2], gb[2];
    auto req_q = [&](auto kk_c, auto set_c) {
      constexpr int kk = decltype(kk_c)::value, set = decltype(set_c)::value;
      const uint32_t ad = lds_xor<(kk << 5)>(adQ0);
      qa[set] = lds_read_b128<SB + L::T_QH * TILE_B>(ad); qc[set] = lds_read_b128<SB + L::T_QD * TILE_B>(ad);
      if constexpr (LO) qb[set] = lds_read_b128<SB + L::T_QL * TILE_B>(ad);
      if constexpr (DK) {
        ga[set] = lds_read_b128<SB + L::T_GH * TILE_B>(ad); gb[set] = lds_read_b128<SB + L::T_GD * TILE_B>(ad);
      }
    };
    // (fragments one step ahead of their use, except at head width 128, where the registers are all taken)
    constexpr bool AHEAD = DH <= 64;
    if constexpr (AHEAD) req_q(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    static_for<KS>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value, c = AHEAD ? (kk & 1) : 0;
      if constexpr (!AHEAD) {
        req_q(kk_c, std::integral_constant<int, 0>{});
        lds_wait<0>();
      } else if constexpr (kk + 1 < KS) {
        req_q(std::integral_constant<int, kk + 1>{}, std::integral_constant<int, c ^ 1>{});
        lds_wait<((LO ? 3 : 2) + (DK ? 2 : 0))>();
      } else {
        lds_wait<0>();
      }
      lds_tie(qa[c]); lds_tie(qc[c]);
      if constexpr (LO) lds_tie(qb[c]);
      if constexpr (DK) { lds_tie(ga[c]); lds_tie(gb[c]); }
      st = HF_MFMA(qa[c], kh[kk], st);
      su = HF_MFMA(qc[c], kh[kk], su);
      if constexpr (DK) {
        dp = HF_MFMA(ga[c], vh[kk], dp);       // dP = dO V^T
        dpt = HF_MFMA(gb[c], vh[kk], dpt);     // dP_t = dO_t V^T + dO V_t^T
      }
      if constexpr (LO) st = HF_MFMA(qb[c], kh[kk], st);
      su = HF_MFMA(qa[c], kd[kk], su);
      if constexpr (DK) dpt = HF_MFMA(ga[c], vd[kk], dpt);
      if constexpr (LO) st = HF_MFMA(qa[c], kl[kk], st);
      __builtin_amdgcn_sched_barrier(0);
    });
    // the products of the second half, in order: per key step ks, the dV products of the RT column
    // tiles, then the dK ones; each takes two transposed fragments (four reads)
    constexpr int UK = (DV ? RT : 0) + (DK ? RT : 0), NU = 2 * UK;
    bf16x4 ta[2][2], tb[2][2];
    auto req_t = [&](auto u_c, auto set_c) {
      constexpr int u = decltype(u_c)::value, set = decltype(set_c)::value;
      constexpr int ks = u / UK, w = u % UK;
      constexpr bool isV = DV && w < RT;
      constexpr int rt = isV ? w : w - (DV ? RT : 0);
      constexpr int TA = isV ? L::T_GHT : L::T_QHT, TB = isV ? L::T_GDT : L::T_QDT;
      constexpr int OFF = SB + ks * 16 * DH * 2;
      const uint32_t ad = lds_xor<(rt << 6)>(adT0);
      ta[set][0] = lds_read_tr64<OFF + TA * TILE_B>(ad); ta[set][1] = lds_read_tr64<OFF + TA * TILE_B + 8 * DH * 2>(ad);
      tb[set][0] = lds_read_tr64<OFF + TB * TILE_B>(ad); tb[set][1] = lds_read_tr64<OFF + TB * TILE_B + 8 * DH * 2>(ad);
    };
    if constexpr (AHEAD) req_t(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    // register v of this lane: query q0 + 8 (v/4) + 4 (lane/32) + v%4 against key nk
    float pr[16], pt[16], ds[DK ? 16 : 1], dsx[DK ? 16 : 1];
    const HF_LDS float* sq_base = stats + SI * 128;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int qi = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const at_f32x4 sq = *(const HF_LDS at_f32x4*)(sq_base + qi * 4);
      const int q = q0 + qi;
      pr[v] = (q < nk || q >= p.S) ? 0.f : __expf(st[v] * p.scale - sq.x);
      pt[v] = pr[v] * (su[v] * p.scale - sq.y);
      if constexpr (DK) {
        ds[v] = pr[v] * (dp[v] - sq.z);
        dsx[v] = pt[v] * (dp[v] - sq.z) + pr[v] * (dpt[v] - sq.w);
      }
    }
    bf16x8 pb[2], ptb[2], sb[DK ? 2 : 1], sxb[DK ? 2 : 1];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      pb[ks] = pack8(pr + ks * 8); ptb[ks] = pack8(pt + ks * 8);
      if constexpr (DK) { sb[ks] = pack8(ds + ks * 8); sxb[ks] = pack8(dsx + ks * 8); }
    }
    __builtin_amdgcn_sched_barrier(0);
    static_for<NU>([&](auto u_c) {
      constexpr int u = decltype(u_c)::value, c = AHEAD ? (u & 1) : 0;
      constexpr int ks = u / UK, w = u % UK;
      constexpr bool isV = DV && w < RT;
      constexpr int rt = isV ? w : w - (DV ? RT : 0);
      if constexpr (!AHEAD) {
        req_t(u_c, std::integral_constant<int, 0>{});
        lds_wait<0>();
      } else if constexpr (u + 1 < NU) {
        req_t(std::integral_constant<int, u + 1>{}, std::integral_constant<int, c ^ 1>{});
        lds_wait<4>();
      } else {
        lds_wait<0>();
      }
      lds_tie(ta[c][0]); lds_tie(ta[c][1]); lds_tie(tb[c][0]); lds_tie(tb[c][1]);
      const bf16x8 xa = __builtin_shufflevector(ta[c][0], ta[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8 xb = __builtin_shufflevector(tb[c][0], tb[c][1], 0, 1, 2, 3, 4, 5, 6, 7);
      if constexpr (isV) {
        dv[rt] = HF_MFMA(xa, pb[ks], dv[rt]);       // dV^T = dO^T P
        dvt[rt] = HF_MFMA(xa, ptb[ks], dvt[rt]);    // dV_t^T = dO^T P_t + dO_t^T P
        dvt[rt] = HF_MFMA(xb, pb[ks], dvt[rt]);
      } else {
        dk[rt] = HF_MFMA(xa, sb[ks], dk[rt]);       // dK^T = Q^T dS
        dkt[rt] = HF_MFMA(xa, sxb[ks], dkt[rt]);    // dK_t^T = Q^T dS_t + Q_t^T dS
        dkt[rt] = HF_MFMA(xb, sb[ks], dkt[rt]);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // statistics of tile 0 straight into their LDS tile, those of tile 1 into registers
  if (t < 32) {
    load_stats(0);
    *(HF_LDS at_f32x4*)(stats + t * 4) = spre;
    if (nit > 1) load_stats(1);
  }
  issue(0, 0);
  for (int it0 = 0; it0 < nit; it0 += 2) {
    static_for<2>([&](auto s_c) {
      constexpr int S = decltype(s_c)::value;
      const int it = it0 + S;
      if (it < nit) {
        const int qs = it % nqs, q0 = k0 + qs * 32;
        HF_WAIT_VMCNT(0);                 // this wave's part of tile `it` has landed (and the statistics in registers)
        lds_wait<0>();                    // ... and its statistics store of the previous turn
        __builtin_amdgcn_s_barrier();     // everyone's has, and stage 1 - S has been read for the last time
        __builtin_amdgcn_sched_barrier(0);
        if (it + 1 < nit) {
          issue(1 - S, it + 1);
          if (t < 32) {
            *(HF_LDS at_f32x4*)(stats + (1 - S) * 128 + t * 4) = spre;
            if (it + 2 < nit) load_stats(it + 2);
          }
        }
        // (wave-uniform) nothing to do where every query of the tile precedes this wave's keys
        if (!(q0 + 31 < kw || kw >= p.S)) compute(s_c, q0);
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  }
  if (nk >= p.S) return;
  const int64_t orow = row0 + nk;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int col = hk * DH + rt * 32 + 8 * g4 + 4 * (lane >> 5);
      if (DV) {
        store4(p.dv, p.dv_f32, orow, p.lddv, col, dv[rt][g4 * 4], dv[rt][g4 * 4 + 1], dv[rt][g4 * 4 + 2], dv[rt][g4 * 4 + 3]);
        store4(p.dv_t, p.dv_f32, orow, p.lddv, col, dvt[rt][g4 * 4], dvt[rt][g4 * 4 + 1], dvt[rt][g4 * 4 + 2], dvt[rt][g4 * 4 + 3]);
      }
      if (DK) {
        store4(p.dk, p.dk_f32, orow, p.lddk, col, dk[rt][g4 * 4] * p.scale, dk[rt][g4 * 4 + 1] * p.scale, dk[rt][g4 * 4 + 2] * p.scale,
               dk[rt][g4 * 4 + 3] * p.scale);
        store4(p.dk_t, p.dk_f32, orow, p.lddk, col, dkt[rt][g4 * 4] * p.scale, dkt[rt][g4 * 4 + 1] * p.scale,
               dkt[rt][g4 * 4 + 2] * p.scale, dkt[rt][g4 * 4 + 3] * p.scale);
      }
    }
  }
}

// ------------------------------------------------------------------ launchers ----

static bool attn_shape_ok(const AttnP& p) {
  const int dh = p.dh;
  if (dh != 32 && dh != 64 && dh != 128) return false;
  if (p.B <= 0 || p.H <= 0 || p.S <= 0 || p.grp <= 0 || p.H % p.grp) return false;
  if (p.ldq % 8 || p.offK % 8 || p.offV % 8) return false;
  return true;
}
static bool al16(const void* x) { return x != nullptr && ((uintptr_t)x & 15) == 0; }

bool attn_flash_supported(int dh, int64_t ldq, int64_t ldo) { return (dh == 32 || dh == 64 || dh == 128) && ldq % 8 == 0 && ldo % 8 == 0; }

// Up to head width 64 two blocks share a CU and the streamed kernels win at every size measured.  At
// 128 a block needs the whole register file; the kernels still win once a launch has a block for
// every CU (1.3B shape, 512 blocks: 14.2 against 16 ms per product), but not at a batch of one
// sequence (Llama-7B shape, 128 blocks: 1 % behind).
bool attn_flash_preferred(int dh, int64_t heads, int64_t S) { return dh <= 64 || heads * ((S + 127) / 128) >= 256; }

template <int DH, bool LO>
static hipError_t launch_fwd_t(const AttnP& p, unsigned grid, hipStream_t st) {
  constexpr int lds = 2 * (LO ? 6 : 4) * 64 * DH;  // two stages of six (four) tiles
  static OncePerDevice once;
  auto kern = attn_fwd_kernel<DH, LO>;
  if (lds > 64 * 1024)
    if (const hipError_t e = once.lds_limit((const void*)kern, lds); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p);
  return hipGetLastError();
}
template <int DH, bool LO>
static hipError_t launch_q_t(const AttnP& p, unsigned grid, hipStream_t st) {
  constexpr int lds = 2 * (LO ? 7 : 6) * 64 * DH;  // two stages of seven (six) tiles
  static OncePerDevice once;
  auto kern = attn_bwd_q_kernel<DH, LO>;
  if (lds > 64 * 1024)
    if (const hipError_t e = once.lds_limit((const void*)kern, lds); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p);
  return hipGetLastError();
}
template <int DH, int WHAT, bool LO>
static hipError_t launch_kv(const AttnP& p, unsigned grid, hipStream_t st) {
  constexpr int lds = KvTiles<DH, WHAT, LO>::LDS_B;
  static_assert(lds <= 160 * 1024, "LDS");
  static OncePerDevice once;
  auto kern = attn_bwd_kv_kernel<DH, WHAT, LO>;
  if (lds > 64 * 1024)
    if (const hipError_t e = once.lds_limit((const void*)kern, lds); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p);
  return hipGetLastError();
}

// p.qkv_lo == nullptr: the primal operands have no low-order halves (and no o_lo is written).
hipError_t launch_attn_fwd(const AttnP& p, hipStream_t st) {
  if (!attn_shape_ok(p) || p.ldo % 8) return hipErrorInvalidValue;
  const bool lo = p.qkv_lo != nullptr;
  if (!al16(p.qkv) || !al16(p.qkv_t) || !al16(p.o) || !al16(p.o_t) || !p.stat) return hipErrorInvalidValue;
  if (lo && (!al16(p.qkv_lo) || !al16(p.o_lo))) return hipErrorInvalidValue;
  const int nqt = (p.S + 127) / 128;
  const unsigned grid = (unsigned)(((p.B * p.H + 7) / 8) * 8 * nqt);
  if (p.dh == 32) return lo ? launch_fwd_t<32, true>(p, grid, st) : launch_fwd_t<32, false>(p, grid, st);
  if (p.dh == 64) return lo ? launch_fwd_t<64, true>(p, grid, st) : launch_fwd_t<64, false>(p, grid, st);
  return lo ? launch_fwd_t<128, true>(p, grid, st) : launch_fwd_t<128, false>(p, grid, st);
}

template <int DH, bool LO>
static hipError_t launch_bwd_t(const AttnP& p, unsigned gq, unsigned gk, hipStream_t st) {
  if (const hipError_t e = launch_q_t<DH, LO>(p, gq, st); e != hipSuccess) return e;
  if constexpr (DH <= 64) {
    return launch_kv<DH, 3, LO>(p, gk, st);
  } else {
    // at a head width of 128 the accumulators of dK and dV together exceed the register file:
    // one launch each, both recomputing the scores
    if (const hipError_t e1 = launch_kv<DH, 1, LO>(p, gk, st); e1 != hipSuccess) return e1;
    return launch_kv<DH, 2, LO>(p, gk, st);
  }
}

hipError_t launch_attn_bwd(const AttnP& p, hipStream_t st) {
  if (!attn_shape_ok(p) || p.lddo % 8) return hipErrorInvalidValue;
  const bool lo = p.qkv_lo != nullptr;
  if (!al16(p.qkv) || (lo && !al16(p.qkv_lo)) || !al16(p.qkv_t) || !al16(p.dO) || !al16(p.dO_t) || !p.stat || !p.delta) return hipErrorInvalidValue;
  if (!al16(p.dq) || !al16(p.dq_t) || !al16(p.dk) || !al16(p.dk_t) || !al16(p.dv) || !al16(p.dv_t)) return hipErrorInvalidValue;
  if (p.lddq % 4 || p.lddk % 4 || p.lddv % 4) return hipErrorInvalidValue;
  const int nqt = (p.S + 127) / 128;
  const unsigned gq = (unsigned)(((p.B * p.H + 7) / 8) * 8 * nqt);
  const unsigned gk = (unsigned)(((p.B * (p.H / p.grp) + 7) / 8) * 8 * nqt);
  if (p.dh == 32) return lo ? launch_bwd_t<32, true>(p, gq, gk, st) : launch_bwd_t<32, false>(p, gq, gk, st);
  if (p.dh == 64) return lo ? launch_bwd_t<64, true>(p, gq, gk, st) : launch_bwd_t<64, false>(p, gq, gk, st);
  return lo ? launch_bwd_t<128, true>(p, gq, gk, st) : launch_bwd_t<128, false>(p, gq, gk, st);
}

}  // namespace hf
