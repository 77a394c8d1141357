// Shared device helpers of the MoE kernels: bf16 / FP8 conversions, 128-bit loads, the activation-fragment
// layout, the MFMA wrapper, the register software pipeline and the weight addressing.
// Part of the single translation unit moe_kernels.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cascade_moe.h"

namespace {

constexpr int kMaxTokens = 16;
constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 16;
constexpr int kMaxShared = 8;
constexpr int kGateCols = 16;  // columns of the per-slot gate table = MFMA N

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Index of the calling wavefront inside its workgroup, as a SCALAR: tid >> 6 is the same in all 64 lanes, but the
// compiler cannot know that, and everything derived from a per-lane value (loop bounds, base pointers of the
// wave's share of the work) would live in vector registers and be branched on through the EXEC mask.
__device__ __forceinline__ int wave_index(int tid) { return __builtin_amdgcn_readfirstlane(tid >> 6); }

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // keep NaN a NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// x = hi + lo (+ residual below 2^-17 |x|): both halves are exact bf16 numbers.
__device__ __forceinline__ void split_bf16(float x, uint16_t& hi, uint16_t& lo) {
  hi = f32_to_bf16(x);
  lo = f32_to_bf16(x - bf16_to_f32(hi));
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 128-bit global load; NT = streaming (non-temporal) hint for bytes that are read exactly once.
template <bool NT>
__device__ __forceinline__ uint4 ld128(const char* base, uint32_t byte_off) {
  if constexpr (NT) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + byte_off));
    return uint4{v.x, v.y, v.z, v.w};
  } else {
    return *reinterpret_cast<const uint4*>(base + byte_off);
  }
}

// Activation fragments.  The MFMA B operand of k-step s (32 k) wants, in lane (n = l%16, kg = l/16),
// the 8 values k = 32 s + 8 kg .. +7 of token column n.  Activations are therefore stored in that
// order — unit q = s*64 + kg*16 + n holds those 8 bf16 (16 bytes) — so a wave fetches the whole
// fragment of a k-step with ONE contiguous 1 KB load.  Token columns are padded to 16.
//
// Two arrangements of the bf16 hi + lo halves of the fp32 activations:
//   split   (T > 8)   two fragment arrays, hi and lo; column n = token n; two MFMAs per weight tile
//   packed  (T <= 8)  ONE array: column n < 8 = hi half of token n, column n + 8 = lo half of token n.
//                     MFMA columns are independent, so one MFMA yields the hi and the lo contribution
//                     in two columns, which the epilogue adds: half the fragment loads and half the
//                     MFMAs for every speculation length up to K = 7.
constexpr int kPackedTokens = 8;
__device__ __forceinline__ size_t frag_unit(int k8, int n) {  // k8 = k / 8
  return (size_t)(k8 >> 2) * 64 + (size_t)(k8 & 3) * 16 + n;
}

// Compact variant of the packed arrangement, used where fragment bytes are the bottleneck: per k-group only the
// `cols` = 2 T live columns (hi halves of tokens 0 .. T-1, then their lo halves) instead of 16, so a k-step is
// 64 * cols bytes.  With cols = 16 it is the packed arrangement itself.
__device__ __forceinline__ size_t frag_unit_compact(int k8, int c, int cols) {
  return (size_t)(k8 >> 2) * (4 * cols) + (size_t)(k8 & 3) * cols + c;
}

// FP8 weights: the 16 bytes a lane loads are its 8 codes of one k-step followed by its 8 codes of the
// next k-step.  Every E4M3 value is exactly a bf16 number, so the codes are widened in registers (two
// codes per instruction) and fed to the same bf16 MFMA; the per-row scale is applied to the fp32 sums.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
template <bool HI>
__device__ __forceinline__ uint32_t fp8x2_to_bf16x2(uint32_t v) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v, 1.0f, HI));
}
__device__ __forceinline__ void fp8x16_to_bf16(uint4 a, uint4& k0, uint4& k1) {
  k0 = uint4{fp8x2_to_bf16x2<false>(a.x), fp8x2_to_bf16x2<true>(a.x), fp8x2_to_bf16x2<false>(a.y),
             fp8x2_to_bf16x2<true>(a.y)};
  k1 = uint4{fp8x2_to_bf16x2<false>(a.z), fp8x2_to_bf16x2<true>(a.z), fp8x2_to_bf16x2<false>(a.w),
             fp8x2_to_bf16x2<true>(a.w)};
}

__device__ __forceinline__ f32x4 mfma_bf16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                  0, 0);
}

// ------------------------------------------------------------------------------------------
// Shared software pipeline of the two expert kernels.
//   NA  A tiles (16 rows) consumed per step, each with its own wave-uniform base pointer
//   NB  k-steps (32 k) one 128-bit weight load covers: 1 for bf16, 2 for FP8
//   P   pipeline depth (steps of loads in flight per wave)
// A stage holds one 128-bit load per tile plus the hi and lo activation fragments of its NB k-steps.
// ------------------------------------------------------------------------------------------
template <int NA, int NB, bool PK>
struct Stage {
  uint4 a[NA];
  uint4 bh[NB];
  uint4 bl[PK ? 1 : NB];  // unused when the halves are packed into bh
};

// Issue slots between the last MFMA of a code path and whatever comes after a branch.  A matrix-core result lands
// several slots after its instruction was issued; the compiler pads a too-early reader with s_nop, but its padding
// has been seen to fall short when the reader (typically a register-allocator copy of the accumulators) sits
// behind a TAKEN uniform branch — the wave then continues with the accumulator as it was before its last MFMA.
// So every conditionally executed group of MFMAs below ends with the padding itself, fenced so that nothing is
// scheduled across it.  (The generated code is also checked after every build: mfma_hazard_check.py.)
__device__ __forceinline__ void mfma_settle() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 7");
  __builtin_amdgcn_sched_barrier(0);
}

template <int NA, int NB, bool PK, int P, class Load, class Compute>
__device__ __forceinline__ void pipeline(int nst, Load load, Compute compute) {
  Stage<NA, NB, PK> st[P];
  // The prologue loads are unconditional (a short wave re-reads its last valid step): a load that
  // is issued on only some paths makes the compiler's wait counters pessimistic inside the loop.
  const int last = nst > 0 ? nst - 1 : 0;
#pragma unroll
  for (int p = 0; p < P; ++p) load(st[p], min(p, last));
  int s = 0;
  for (; s + 2 * P <= nst; s += P) {
#pragma unroll
    for (int p = 0; p < P; ++p) {
      compute(st[p]);
      load(st[p], s + p + P);
    }
  }
  mfma_settle();
#pragma unroll
  for (int p = 0; p < P; ++p)
    if (s + p < nst) {
      compute(st[p]);
      mfma_settle();
      if (s + p + P < nst) load(st[p], s + p + P);
    }
#pragma unroll
  for (int p = 0; p < P; ++p)
    if (s + P + p < nst) {
      compute(st[p]);
      mfma_settle();
    }
}

// ------------------------------------------------------------------------------------------
// Weight addressing.  A step of a 16-row tile is 1 KB: 16 rows x 32 k of bf16, or 16 rows x 64 k of FP8.
//   row-major [rows, K]:  lane (r, kg) reads 16 contiguous bytes of row tile*16 + r:
//                         bf16: k = 32 s + 8 kg .. + 7;   FP8: k = 64 s + 16 kg .. + 15
//   tiled              :  the same 1 KB stored contiguously, block index tile*(steps per row) + s, lane
//                         l at byte 16 l — what moe_pack_weights produces; one wave load = 1 KB contiguous
// An FP8 lane feeds its first 8 codes to one MFMA and its last 8 to the next.  In the tiled layout those are
// k-group kg of k-step 2s and of k-step 2s + 1; in the row-major one they are the adjacent k-groups 2 kg and
// 2 kg + 1 of the 64-k block.  A matrix product does not care in which order k is walked as long as both
// operands agree, so the row-major kernels fetch the matching activation units instead (frag_lane_off).
// ------------------------------------------------------------------------------------------
template <bool TILED, bool FP8>
struct WeightAddr {
  uint32_t lane_off, step_stride;
  size_t tile_stride;
  __device__ __forceinline__ WeightAddr(int K, int r, int kg, int lane) {
    if constexpr (TILED) {
      lane_off = lane * 16;
      step_stride = 1024;
      tile_stride = (size_t)(K >> (FP8 ? 6 : 5)) * 1024;
    } else if constexpr (FP8) {
      lane_off = (uint32_t)r * K + kg * 16;
      step_stride = 64;
      tile_stride = (size_t)16 * K;
    } else {
      lane_off = ((uint32_t)r * K + kg * 8) * 2;
      step_stride = 64;
      tile_stride = (size_t)16 * K * 2;
    }
  }
};

// Byte offset, inside the fragments of one pipeline step (NB k-steps of 1 KB), of the activation unit that lane
// (n, kg) multiplies with the b-th half of its weight load.
template <bool TILED, bool FP8>
__device__ __forceinline__ uint32_t frag_lane_off(int n, int kg, int lane, int b) {
  if constexpr (!TILED && FP8) {
    const int g = 2 * kg + b;  // k-group (8 k) inside the 64-k block
    return (uint32_t)((g >> 2) * 64 + (g & 3) * 16 + n) * 16;
  } else {
    return (uint32_t)lane * 16 + (uint32_t)b * 1024;
  }
}

}  // namespace
