// Device helpers shared by the MFMA matrix-product kernels: LDS layouts,
// direct global->LDS slab loads, fragment reads (see gemm_mfma.hip for the
// design notes).
#pragma once
#include "hf_internal.h"
#include "gemm_params.h"

#include <type_traits>
#include <utility>
#include <atomic>

namespace hf {

// hipFuncSetAttribute acts on the current device, so "already done" is kept per device.
struct OncePerDevice {
  std::atomic<bool> done[64];
  OncePerDevice() { for (auto& d : done) d.store(false); }
  // Sets the dynamic-LDS limit of `kern` on the current device the first time it is asked to.
  hipError_t lds_limit(const void* kern, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool track = dev >= 0 && dev < 64;
    if (track && done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && track) done[dev].store(true, std::memory_order_release);
    return e;
  }
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define HF_LDS __attribute__((address_space(3)))

// vmcnt(n) only (expcnt / lgkmcnt left at their maxima), gfx9 encoding.
#define HF_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((((n) & 0xF) | ((((n) >> 4) & 0x3) << 14) | (0x7 << 4) | (0xF << 8)))

// ---- LDS addressing ---------------------------------------------------------
// The LDS of gfx950 serves 256 B per clock (64 banks): a 16 B fragment read is
// conflict-free when 16 consecutive lanes cover all 64 banks.
// k-contiguous operand, slab depth KT (64 or 32): row r holds KT/8 chunks of
// 16 B; 256/(2 KT) rows span the banks, so the chunk index is rotated by
// r / (128/KT).
template <int KT>
__device__ __forceinline__ int kc_chunk(int r, int c) { return (c ^ (r / (128 / KT))) & (KT / 8 - 1); }
template <int KT>
__device__ __forceinline__ int lds_kc(int r, int k) { return r * KT + (kc_chunk<KT>(r, k >> 3) << 3) + (k & 7); }
// row-contiguous operand, R rows per k: element (k, r) at k*R + swizzled r.
// The 64 B windows that one transpose read touches in four consecutive k rows
// are rotated by (k & 3) so that they fall on four different quarters of the
// banks (row strides are multiples of 256 B).
// (rows of fewer than 16 chunks keep the low bits of the rotation)
__device__ __forceinline__ int rc_rot(int k, int R) { return ((k & 3) << 2) & (R / 8 - 1); }
__device__ __forceinline__ int lds_rc(int k, int r, int R) { return k * R + ((((r >> 3) ^ rc_rot(k, R))) << 3) + (r & 7); }

// Direct global->LDS loads of one k-slab of one operand.  Each wave issues NI
// instructions per slab; instruction j moves 64 chunks of 16 B to the LDS
// chunks [(wave*NI + j)*64, +64).  The lane's source offset relative to the
// slab's (wave-uniform) base address does not change from slab to slab, so it
// is computed once (slab_offsets) and the per-slab work is one scalar base
// update plus NI load instructions (slab_issue).
// KC: k-contiguous source (element (r,k) at src[r*ld + k]); else (k,r) at src[k*ld + r].
template <int R, bool KC, int KT>
__device__ __forceinline__ void slab_offsets(uint32_t (&voff)[R * KT / 2048], int64_t ld, int r0, int rmax, int wave,
                                             int lane) {
  constexpr int NI = R * KT / 2048;
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int P = (wave * NI + j) * 64 + lane;
    if (KC) {
      constexpr int CPK = KT / 8;  // chunks per row
      const int row = P / CPK, pc = P % CPK;
      const int lc = kc_chunk<KT>(row, pc);
      const int gr = min(r0 + row, rmax - 1) - r0;  // clamped rows only feed outputs that are never stored
      voff[j] = (uint32_t)(((int64_t)gr * ld + lc * 8) * 2);
    } else {
      constexpr int CPR = R / 8;  // chunks per k-row
      const int krow = P / CPR, pc = P % CPR;
      const int lc = pc ^ rc_rot(krow, R);
      const int gc = min(r0 + lc * 8, ((rmax - 1) >> 3) << 3) - r0;
      voff[j] = (uint32_t)(((int64_t)krow * ld + gc) * 2);
    }
  }
}

template <int NI>
__device__ __forceinline__ void slab_issue(const char* base, const uint32_t (&voff)[NI], HF_LDS char* lds_wave) {
#pragma unroll
  for (int j = 0; j < NI; ++j)
    __builtin_amdgcn_global_load_lds((const void*)(base + voff[j]), (HF_LDS void*)(lds_wave + j * 1024), 16, 0, 0);
}

// Guarded load of a ragged k-slab (k in [k0, kend) valid, the rest zero).
template <int R, bool KC, int KT>
__device__ __forceinline__ void slab_guarded(const bf16* __restrict__ src, int64_t ld, int r0, int k0, int rmax, int kend,
                                             HF_LDS bf16* lds, int t) {
  for (int i = t; i < R * KT; i += 256) {
    int r, k;
    if (KC) { k = i % KT; r = i / KT; } else { r = i % R; k = i / R; }
    const int gr = r0 + r, gk = k0 + k;
    bf16 v = (bf16)0.f;
    if (gr < rmax && gk < kend) v = KC ? src[(int64_t)gr * ld + gk] : src[(int64_t)gk * ld + gr];
    lds[KC ? lds_kc<KT>(r, k) : lds_rc(k, r, R)] = v;
  }
}

// Fragment (row = base + lane%32, k = kk*16 + (lane/32)*8 .. +8) of a slab.
template <int R, bool KC, int KT>
__device__ __forceinline__ bf16x8 frag_read(const HF_LDS bf16* lds, int rbase, int kk, int lane) {
  if (KC) {
    const int r = rbase + (lane & 31);
    const int c = kk * 2 + (lane >> 5);
    return *(const HF_LDS bf16x8*)(lds + r * KT + (kc_chunk<KT>(r, c) << 3));
  } else {
    // transpose read: 16 lanes address 4 k-rows x 16 columns (4 lanes per row,
    // 4 columns each); lane i of the group receives column i, 4 consecutive k.
    const int i = lane & 15, g = lane >> 4;
    const int kq = kk * 16 + (g >> 1) * 8 + (i >> 2);
    const int c = rbase + (g & 1) * 16 + (i & 3) * 4;
    const HF_LDS bf16* p0 = lds + kq * R + ((((c >> 3) ^ rc_rot(kq, R))) << 3) + (c & 7);
    const HF_LDS bf16* p1 = p0 + 4 * R;  // k + 4: same k & 3, same swizzle
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((HF_LDS bf16x4*)p0);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((HF_LDS bf16x4*)p1);
    bf16x8 v;
    v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
    v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
    return v;
  }
}

// ---- explicit LDS fragment reads ---------------------------------------------
// The main loop issues its fragment reads as inline instructions and waits for
// them itself.  Left to the compiler, a transpose read that follows a
// global->LDS load is preceded by a wait for ALL outstanding vector-memory
// loads (it cannot prove that the two do not touch the same LDS bytes), which
// would serialise the slab prefetch with the products; here the stage being
// read and the stage being filled are disjoint by construction and ordered by
// the barrier at the top of each iteration.
// addr: byte address in LDS; OFF: compile-time byte offset (split into the
// 16-bit immediate and a part added to the address).
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
  bf16x8 v;
  constexpr int hi = OFF & ~0xFFFF, lo = OFF & 0xFFFF;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr + hi), "n"(lo));
  return v;
}
template <int OFF>
__device__ __forceinline__ bf16x4 lds_read_tr64(uint32_t addr) {
  bf16x4 v;
  constexpr int hi = OFF & ~0xFFFF, lo = OFF & 0xFFFF;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr + hi), "n"(lo));
  return v;
}
// All LDS reads issued so far have landed; the operands tie the fragments to
// this point so that nothing that uses them is moved above the wait.
__device__ __forceinline__ void lds_wait_all() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void lds_tie(bf16x8& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void lds_tie(bf16x4& v) { asm volatile("" : "+v"(v)); }

// Per-lane byte address (relative to the operand's slab in LDS) of the
// fragment rows rbase + lane%32 at k-step kk (k-contiguous layout) or at
// k-step 0 (row-contiguous layout, where k-step kk adds kk*16*R*2 bytes and
// the second half of the fragment another 4*R*2).
template <int R, bool KC, int KT>
__device__ __forceinline__ uint32_t frag_addr(int rbase, int kk, int lane) {
  if (KC) {
    const int r = rbase + (lane & 31);
    const int c = kk * 2 + (lane >> 5);
    return (uint32_t)((r * KT + (kc_chunk<KT>(r, c) << 3)) * 2);
  } else {
    const int i = lane & 15, g = lane >> 4;
    const int kq = (g >> 1) * 8 + (i >> 2);
    const int c = rbase + (g & 1) * 16 + (i & 3) * 4;
    return (uint32_t)((kq * R + ((((c >> 3) ^ rc_rot(kq, R))) << 3) + (c & 7)) * 2);
  }
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(<N-1>{}).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// One MFMA operand fragment (8 bf16 per lane) on its way from LDS: a single
// 16 B read for a k-contiguous operand, two transpose reads for a
// row-contiguous one.
template <bool KC>
struct Frag;
template <>
struct Frag<true> {
  bf16x8 v;
  template <int OFF, int KSTEP>
  __device__ __forceinline__ void read(uint32_t addr) { v = lds_read_b128<OFF>(addr); }
  __device__ __forceinline__ void tie() { lds_tie(v); }
  __device__ __forceinline__ bf16x8 get() const { return v; }
};
template <>
struct Frag<false> {
  bf16x4 lo, hi;
  template <int OFF, int KSTEP>
  __device__ __forceinline__ void read(uint32_t addr) {
    lo = lds_read_tr64<OFF>(addr);
    hi = lds_read_tr64<OFF + KSTEP>(addr);
  }
  __device__ __forceinline__ void tie() { lds_tie(lo); lds_tie(hi); }
  __device__ __forceinline__ bf16x8 get() const { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); }
};

}  // namespace hf
