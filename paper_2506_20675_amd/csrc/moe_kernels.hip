// MoE verification path for MI355X (gfx950): hand-written HIP kernels + the device half of the C ABI.
//
// One decode iteration of speculative decoding pushes T = K+1 tokens through each MoE layer
// (paper: Section 2.2); every token picks top_k experts on its own, and the layer's cost is the
// HBM traffic for the UNION of the picked experts (Section 1, Section 2.4).  The path below touches
// every unique expert's weights exactly once per step:
//
//   route_kernel   one workgroup (16 waves) per token: router logits (fp64 accumulate), top-k by rank
//                  counting, softmax gates, and the bf16 hi + lo activation fragments for the matrix cores
//   group_kernel   union of experts, per-expert token lists, slot tables for the expert kernels and the
//                  combine (for a single token, T = 1, route_kernel does this itself and the launch is skipped)
//   gateup_kernel  for each slot of the union: G = w1 X, U = w3 X, H = gate * silu(G) * U   (2/3 of bytes)
//   down_kernel    split-K partial sums of w2 H over (slot, k-chunk)                        (1/3 of bytes)
//   combine_kernel out[t] = sum of the slabs of token t's own picks, in pick order (deterministic, no atomics)
//
// The two FFN kernels are skinny GEMMs (at most 16 token columns) and purely HBM-bound.  They use
// v_mfma_f32_16x16x32_bf16 with the weight tile as the A operand: lane l holds 8 consecutive k of
// row l%16, k-group l/16, so one 128-bit global load per lane feeds one MFMA directly with no
// conversion and no cross-lane reduction; fp32 activations enter as hi + lo bf16 pairs (two MFMAs)
// so the result keeps ~fp32 accuracy.  The token dimension is the 16-wide N of the MFMA: all T <= 16
// tokens ride along with every weight byte, which is why a weight byte is read once per step no
// matter how many tokens share the expert.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "cascade_moe.h"

namespace {

constexpr int kMaxTokens = 16;
constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 16;
constexpr int kMaxShared = 8;
constexpr int kGateCols = 16;  // columns of the per-slot gate table = MFMA N

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

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
// Step 2: union of activated experts + per-expert token lists + the tables the expert kernels and
// the combine read.  One workgroup; thread a = one (token, pick) pair, thread e = one expert.
// ------------------------------------------------------------------------------------------
struct GroupArgs {
  const int32_t* ids;   // [T, top_k], the picks of one token distinct
  const float* gates;   // [T, top_k] or NULL (then no gate table is built)
  int T, top_k, E;
  int32_t *unique, *n_unique, *count, *offset, *assign;     // caller-visible outputs, each optional
  int32_t *n_unique_ws, *n_unique_extra, *slot_expert;      // tables for the expert kernels, each optional
  int32_t* tok_slot;                                        // [T, top_k] slot of the union each pick landed in
  float* slot_gate;                                         // [u_max, 16]
};

// Every thread of the workgroup must call this (it holds barriers); blockDim.x >= 256.
// s_ids_in / s_gates_in: the routing in LDS, or NULL to read g.ids / g.gates.
// A token picks an expert at most once, so expert e's token list is a 16-bit mask: pairs set their
// bit with an LDS atomic OR (commutative, so the result does not depend on arrival order), counts are
// popcounts, and lists come out in ascending token order by walking the set bits.
__device__ void group_body(const GroupArgs& g, const int* s_ids_in, const float* s_gates_in) {
  __shared__ int s_ids_own[kMaxTokens * kMaxTopK];
  __shared__ unsigned s_mask[kMaxExperts];
  __shared__ unsigned char s_pos[kMaxExperts * kMaxTokens];  // which pick i of token t chose expert e
  __shared__ int s_rank[kMaxExperts];
  __shared__ float s_row[kMaxExperts * kGateCols];           // gate table by slot, built in LDS
  __shared__ int s_cnt[4], s_uni[4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int E = g.E, A = g.T * g.top_k;
  const bool want_gates = g.slot_gate && (g.gates || s_gates_in);
  const int* s_ids = s_ids_in ? s_ids_in : s_ids_own;
  if (!s_ids_in && tid < A) s_ids_own[tid] = g.ids[tid];
  if (tid < E) s_mask[tid] = 0u;
  const int max_slots = A < E ? A : E;
  if (want_gates)
    for (int i = tid; i < max_slots * kGateCols; i += blockDim.x) s_row[i] = 0.f;
  __syncthreads();
  const int my_e = tid < A ? s_ids[tid] : -1;
  const int my_t = tid / g.top_k;
  const bool pair_ok = tid < A && (unsigned)my_e < (unsigned)E;
  if (pair_ok) {
    atomicOr(&s_mask[my_e], 1u << my_t);
    s_pos[my_e * kMaxTokens + my_t] = (unsigned char)(tid - my_t * g.top_k);
  }
  __syncthreads();
  const bool act = tid < 256;
  const int e = tid;
  unsigned m = (act && e < E) ? s_mask[e] : 0u;
  const int cnt = __popc(m);
  const int flag = cnt > 0;
  // inclusive scan of cnt inside the wave, ballot for the rank among live experts
  int incl = cnt;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  const unsigned long long bal = __ballot(flag);
  const int rank_in_wave = __popcll(bal & ((1ull << lane) - 1ull));
  if (act && lane == 63) s_cnt[wave] = incl;
  if (act && lane == 0) s_uni[wave] = __popcll(bal);
  __syncthreads();
  int cbase = 0, ubase = 0, n_unique = 0, total = 0;
  for (int w = 0; w < 4; ++w) {
    if (w < wave) {
      cbase += s_cnt[w];
      ubase += s_uni[w];
    }
    n_unique += s_uni[w];
    total += s_cnt[w];
  }
  if (act && e < E) {
    const int off = cbase + incl - cnt;
    const int rank = ubase + rank_in_wave;
    if (g.count) g.count[e] = cnt;
    if (g.offset) g.offset[e] = off;
    if (flag) {
      s_rank[e] = rank;
      if (g.unique) g.unique[rank] = e;
      if (g.slot_expert) g.slot_expert[rank] = e;
      if (g.assign) {
        int j = 0;
        while (m) {
          const int t = __ffs(m) - 1;
          m &= m - 1u;
          g.assign[off + j++] = t * g.top_k + s_pos[e * kMaxTokens + t];
        }
      }
    }
    if (e >= n_unique && g.unique) g.unique[e] = -1;
  }
  if (tid == 0) {
    if (g.offset) g.offset[E] = total;
    if (g.n_unique) *g.n_unique = n_unique;
    if (g.n_unique_ws) *g.n_unique_ws = n_unique;
    if (g.n_unique_extra) *g.n_unique_extra = n_unique;
  }
  __syncthreads();
  if (pair_ok) {
    const int slot = s_rank[my_e];
    if (g.tok_slot) g.tok_slot[tid] = slot;
    if (want_gates) s_row[slot * kGateCols + my_t] = s_gates_in ? s_gates_in[tid] : g.gates[tid];
  }
  if (!want_gates) return;
  __syncthreads();
  for (int i = tid; i < n_unique * kGateCols; i += blockDim.x) g.slot_gate[i] = s_row[i];
}

__global__ __launch_bounds__(256) void group_kernel(GroupArgs g) { group_body(g, nullptr, nullptr); }

// ------------------------------------------------------------------------------------------
// Step 1: router.
// ------------------------------------------------------------------------------------------
struct RouteArgs {
  const float* hidden;       // [T, d]
  const uint16_t* router_w;  // [E, d]
  int d, E, top_k, T, gate_mode;
  int32_t *ids_ws, *ids_out;  // [T, top_k]; *_out optional
  float *gates_ws, *gates_out;
  uint16_t *xf_hi, *xf_lo;    // activation fragments
};

// activations of token t -> bf16 hi/lo halves in fragment order (the MFMA B operand of the expert kernels)
__device__ __forceinline__ void split_token(const float* __restrict__ x, int d, int t, int first, int stride,
                                            uint16_t* __restrict__ xf_hi, uint16_t* __restrict__ xf_lo, bool packed) {
  for (int k8 = first; k8 < (d >> 3); k8 += stride) {
    const float4 v0 = *reinterpret_cast<const float4*>(x + k8 * 8);
    const float4 v1 = *reinterpret_cast<const float4*>(x + k8 * 8 + 4);
    const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint16_t h0, l0, h1, l1;
      split_bf16(v[2 * i], h0, l0);
      split_bf16(v[2 * i + 1], h1, l1);
      h[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
      l[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
    }
    const size_t q = frag_unit(k8, t);
    reinterpret_cast<uint4*>(xf_hi)[q] = uint4{h[0], h[1], h[2], h[3]};
    if (packed)
      reinterpret_cast<uint4*>(xf_hi)[q + kPackedTokens] = uint4{l[0], l[1], l[2], l[3]};
    else
      reinterpret_cast<uint4*>(xf_lo)[q] = uint4{l[0], l[1], l[2], l[3]};
  }
}

constexpr int kRouteWaves = 16;  // waves per token in route_kernel
constexpr int kRouteBatch = 8;   // expert rows one work item covers

// One work item of the router of one token: the 512-element chunk `chunk` of d against the expert
// rows e0 .. e0+7.  The activation loads and the (up to) 8 row loads are issued together — one round
// trip — and accumulated in fp64: fp32 x bf16 products are exact in double, so the top-k decision does
// not depend on the order of summation (beyond ~1e-13 relative).  The 64 lanes' partial sums are
// folded by a reduce-scatter butterfly (each exchange halves the experts a lane still carries: 4 + 2 +
// 1 exchanges, then 3 plain ones) instead of one 6-step butterfly per expert; lane 8*i then adds the
// sum of expert e0 + i to s_acc[e0 + i], the wave's own row of partial logits.
__device__ __forceinline__ void route_item(const float* __restrict__ x, const uint16_t* __restrict__ router_w, int d,
                                           int E, int lane, int chunk, int e0, double* s_acc) {
  const int j = chunk * 512 + lane * 8;
  const float4 x0 = *reinterpret_cast<const float4*>(x + j);
  const float4 x1 = *reinterpret_cast<const float4*>(x + j + 4);
  uint4 wv[kRouteBatch];
#pragma unroll
  for (int e = 0; e < kRouteBatch; ++e) {
    const int row = min(e0 + e, E - 1);  // past the last expert: re-read a valid row, result unused
    wv[e] = *reinterpret_cast<const uint4*>(router_w + (size_t)row * d + j);
  }
  const double xd[8] = {(double)x0.x, (double)x0.y, (double)x0.z, (double)x0.w,
                        (double)x1.x, (double)x1.y, (double)x1.z, (double)x1.w};
  double v[kRouteBatch];
#pragma unroll
  for (int e = 0; e < kRouteBatch; ++e) {
    double a = 0.0;
    a = fma(xd[0], (double)bf16_to_f32(wv[e].x & 0xffffu), a);
    a = fma(xd[1], (double)bf16_to_f32(wv[e].x >> 16), a);
    a = fma(xd[2], (double)bf16_to_f32(wv[e].y & 0xffffu), a);
    a = fma(xd[3], (double)bf16_to_f32(wv[e].y >> 16), a);
    a = fma(xd[4], (double)bf16_to_f32(wv[e].z & 0xffffu), a);
    a = fma(xd[5], (double)bf16_to_f32(wv[e].z >> 16), a);
    a = fma(xd[6], (double)bf16_to_f32(wv[e].w & 0xffffu), a);
    a = fma(xd[7], (double)bf16_to_f32(wv[e].w >> 16), a);
    v[e] = a;
  }
  // reduce-scatter: after the exchange over lane bit 5 a lane carries experts {0..3} or {4..7}, ...
  const bool b5 = lane & 32, b4 = lane & 16, b3 = lane & 8;
  double u4[4], u2[2], u1;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const double send = b5 ? v[i] : v[i + 4];
    const double keep = b5 ? v[i + 4] : v[i];
    u4[i] = keep + __shfl_xor(send, 32);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const double send = b4 ? u4[i] : u4[i + 2];
    const double keep = b4 ? u4[i + 2] : u4[i];
    u2[i] = keep + __shfl_xor(send, 16);
  }
  {
    const double send = b3 ? u2[0] : u2[1];
    const double keep = b3 ? u2[1] : u2[0];
    u1 = keep + __shfl_xor(send, 8);
  }
  u1 += __shfl_xor(u1, 4);
  u1 += __shfl_xor(u1, 2);
  u1 += __shfl_xor(u1, 1);
  const int idx = (b5 ? 4 : 0) + (b4 ? 2 : 0) + (b3 ? 1 : 0);
  if ((lane & 7) == 0 && e0 + idx < E) s_acc[e0 + idx] += u1;
}

// One workgroup (16 waves) per token.  The (chunk of d, batch of 8 experts) work items are dealt
// round-robin to the waves; partial logits meet in LDS and are summed in wave order.  Top-k by rank
// counting: thread e counts the logits that beat its own (larger, or equal with a lower index), the
// expert of rank i < top_k is pick i — no serial arg-max rounds.  Gates = softmax over the picked
// logits in fp32, summed in pick order.  With a single token in flight (T = 1, no speculation) this
// workgroup already sees the whole routing, so the expert-union step runs right here; with more
// tokens it needs the launch of its own that follows (group_kernel).
__global__ __launch_bounds__(64 * kRouteWaves) void route_kernel(RouteArgs g, GroupArgs grp) {
  __shared__ double s_part[kRouteWaves][kMaxExperts];
  __shared__ double s_logit[kMaxExperts];
  __shared__ int s_ids[kMaxTopK];
  __shared__ float s_sel[kMaxTopK];
  __shared__ float s_gates[kMaxTopK];
  __shared__ float s_prob[kMaxExperts];
  const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int E = g.E, top_k = g.top_k;
  const float* x = g.hidden + (size_t)t * g.d;
  const int n_batches = (E + kRouteBatch - 1) / kRouteBatch;
  const int n_full = g.d >> 9;  // whole 512-element chunks
  const int n_items = n_full * n_batches;
  for (int e = lane; e < E; e += 64) s_part[wave][e] = 0.0;  // the wave's own row: no barrier needed
  for (int it = wave; it < n_items; it += kRouteWaves)
    route_item(x, g.router_w, g.d, E, lane, it / n_batches, (it % n_batches) * kRouteBatch, s_part[wave]);
  if ((g.d & 511) && wave == kRouteWaves - 1) {
    // ragged tail of d (a multiple of 32 elements): lanes walk it 8 elements at a time
    for (int e = 0; e < E; ++e) {
      double a = 0.0;
      for (int j = (n_full << 9) + lane * 8; j < g.d; j += 512) {
        const uint4 w = *reinterpret_cast<const uint4*>(g.router_w + (size_t)e * g.d + j);
        const float4 x0 = *reinterpret_cast<const float4*>(x + j);
        const float4 x1 = *reinterpret_cast<const float4*>(x + j + 4);
        a = fma((double)x0.x, (double)bf16_to_f32(w.x & 0xffffu), a);
        a = fma((double)x0.y, (double)bf16_to_f32(w.x >> 16), a);
        a = fma((double)x0.z, (double)bf16_to_f32(w.y & 0xffffu), a);
        a = fma((double)x0.w, (double)bf16_to_f32(w.y >> 16), a);
        a = fma((double)x1.x, (double)bf16_to_f32(w.z & 0xffffu), a);
        a = fma((double)x1.y, (double)bf16_to_f32(w.z >> 16), a);
        a = fma((double)x1.z, (double)bf16_to_f32(w.w & 0xffffu), a);
        a = fma((double)x1.w, (double)bf16_to_f32(w.w >> 16), a);
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
      if (lane == 0) s_part[wave][e] += a;
    }
  }
  split_token(x, g.d, t, tid, 64 * kRouteWaves, g.xf_hi, g.xf_lo, g.T <= kPackedTokens);
  __syncthreads();
  if (tid < E) {
    double l = 0.0;
#pragma unroll
    for (int w = 0; w < kRouteWaves; ++w) l += s_part[w][tid];
    if (l != l) l = -INFINITY;  // a NaN logit is never preferred
    s_logit[tid] = l;
  }
  __syncthreads();
  if (tid < E) {
    const double mine = s_logit[tid];
    int rank = 0;
    for (int j = 0; j < E; ++j) {
      const double o = s_logit[j];  // same address in every lane: an LDS broadcast
      rank += (o > mine || (o == mine && j < tid)) ? 1 : 0;
    }
    if (rank < top_k) {
      s_ids[rank] = tid;
      s_sel[rank] = (float)mine;
    }
  }
  __syncthreads();
  const bool all = g.gate_mode == MOE_GATE_SOFTMAX_ALL;
  if (all) {  // exp(l_e - max) of every expert, for the denominator over all E
    if (tid < E) s_prob[tid] = expf((float)s_logit[tid] - s_sel[0]);
    __syncthreads();
  }
  if (tid < top_k) {
    // p_i = exp(l_i - l_0); denominator summed in pick order over the picks, or in expert order over all experts
    const float l0 = s_sel[0];
    float sum = 0.f;
    if (all)
      for (int e = 0; e < E; ++e) sum += s_prob[e];
    else
      for (int i = 0; i < top_k; ++i) sum += expf(s_sel[i] - l0);
    const float gate = expf(s_sel[tid] - l0) / sum;
    const int a = t * top_k + tid, id = s_ids[tid];
    g.ids_ws[a] = id;
    g.gates_ws[a] = gate;
    if (g.ids_out) g.ids_out[a] = id;
    if (g.gates_out) g.gates_out[a] = gate;
    s_gates[tid] = gate;
  }
  if (gridDim.x == 1) group_body(grp, s_ids, s_gates);  // begins with a barrier: the picks are in LDS by then
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
#pragma unroll
  for (int p = 0; p < P; ++p)
    if (s + p < nst) {
      compute(st[p]);
      if (s + p + P < nst) load(st[p], s + p + P);
    }
#pragma unroll
  for (int p = 0; p < P; ++p)
    if (s + P + p < nst) compute(st[p]);
}

// ------------------------------------------------------------------------------------------
// Weight addressing.  A step of a 16-row tile is 1 KB: 16 rows x 32 k of bf16, or 16 rows x 64 k of FP8.
//   row-major [rows, K]:  lane (r, kg) reads 16 B at row tile*16 + r, k = 32 s + 8 kg   (bf16 only)
//   tiled              :  the same 1 KB stored contiguously, block index tile*(steps per row) + s, lane
//                         l at byte 16 l — what moe_pack_weights produces; one wave load = 1 KB contiguous
// ------------------------------------------------------------------------------------------
template <bool TILED, bool FP8>
struct WeightAddr {
  uint32_t lane_off, step_stride;
  size_t tile_stride;
  __device__ __forceinline__ WeightAddr(int K, int r, int kg, int lane) {
    static_assert(TILED || !FP8, "FP8 weights are consumed in the tiled layout only");
    if constexpr (TILED) {
      lane_off = lane * 16;
      step_stride = 1024;
      tile_stride = (size_t)(K >> (FP8 ? 6 : 5)) * 1024;
    } else {
      lane_off = ((uint32_t)r * K + kg * 8) * 2;
      step_stride = 64;
      tile_stride = (size_t)16 * K * 2;
    }
  }
};

// ------------------------------------------------------------------------------------------
// Step 3: gate/up projections + SiLU*mul for every unique expert (and shared expert).
// grid = (row blocks of 16*R rows of ffn, min(E, T*top_k) + n_shared slots); block = W waves that split d.
// ------------------------------------------------------------------------------------------
struct GateupArgs {
  const void *w1, *w3, *sw1, *sw3;      // [E,ffn,d] / [n_shared,ffn,d], bf16 or FP8 codes
  const float *s1, *s3, *ss1, *ss3;     // FP8 only: per-row scales [E,ffn] / [n_shared,ffn]
  const uint16_t *xf_hi, *xf_lo;        // activation fragments, d*16 elements each
  const int32_t* n_unique;              // [1]        size of the union                   } written by the
  const int32_t* slot_expert;           // [u_max]    expert of slot u (ascending)        } grouping step
  const float* slot_gate;               // [u_max+n_shared, 16] gate of token column n, 0 = not routed
  uint16_t *hf_hi, *hf_lo;              // [u_max + n_shared] fragments of gate*silu(G)*U, ffn*16 elements each
  int d, ffn, T, routed_slots, u_max;   // routed_slots = min(E, T*top_k) slots in this grid
};

template <int R, int W, int P, bool TILED, bool NT, bool FP8, bool PK>
__global__ __launch_bounds__(64 * W) void gateup_kernel(GateupArgs g) {
  constexpr int NB = FP8 ? 2 : 1;
  __shared__ float4 red[W > 1 ? W * 2 * R * 64 : 1];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const char *W1, *W3;
  const float *S1 = nullptr, *S3 = nullptr;  // FP8: scale rows of this expert
  const size_t per = (size_t)g.ffn * g.d * (FP8 ? 1 : 2);
  float gate;
  int slot = blockIdx.y;  // slot of the union, or routed_slots + s for shared expert s
  if (slot < g.routed_slots) {
    // three independent loads (one round trip); the tables are in bounds for every slot of the grid
    const int nu = *g.n_unique;
    const int e = g.slot_expert[slot];
    gate = g.slot_gate[slot * kGateCols + (PK ? (r & (kPackedTokens - 1)) : r)];
    if (slot >= nu) return;  // beyond the union of this step
    W1 = reinterpret_cast<const char*>(g.w1) + e * per;
    W3 = reinterpret_cast<const char*>(g.w3) + e * per;
    if constexpr (FP8) {
      S1 = g.s1 + (size_t)e * g.ffn;
      S3 = g.s3 + (size_t)e * g.ffn;
    }
  } else {
    gate = 1.f;  // shared expert: every token, gate 1
    const int sh = slot - g.routed_slots;
    W1 = reinterpret_cast<const char*>(g.sw1) + sh * per;
    W3 = reinterpret_cast<const char*>(g.sw3) + sh * per;
    if constexpr (FP8) {
      S1 = g.ss1 + (size_t)sh * g.ffn;
      S3 = g.ss3 + (size_t)sh * g.ffn;
    }
    slot = g.u_max + sh;  // buffers keep shared experts after the largest union
  }
  const int ntiles = g.ffn >> 4, tile0 = blockIdx.x * R;
  const int nsteps = g.d >> (FP8 ? 6 : 5), chunk = (nsteps + W - 1) / W;
  const int nst = max(0, min(chunk, nsteps - wave * chunk));
  const int s_beg = min(wave * chunk, nsteps - 1);  // a wave without work still issues in-bounds loads

  const WeightAddr<TILED, FP8> wa(g.d, r, kg, lane);
  const char* base[2 * R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const size_t t = (size_t)min(tile0 + j, ntiles - 1);  // ragged last block: re-read a valid tile, result unused
    base[j] = W1 + t * wa.tile_stride + (size_t)s_beg * wa.step_stride;
    base[R + j] = W3 + t * wa.tile_stride + (size_t)s_beg * wa.step_stride;
  }
  const char* XH = reinterpret_cast<const char*>(g.xf_hi) + (size_t)s_beg * (1024 * NB);
  const char* XL = reinterpret_cast<const char*>(g.xf_lo) + (size_t)s_beg * (1024 * NB);
  const uint32_t b_off = lane * 16;

  f32x4 acc[2 * R];
#pragma unroll
  for (int j = 0; j < 2 * R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<2 * R, NB, PK, P>(
      nst,
      [&](Stage<2 * R, NB, PK>& st, int s) {
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) st.a[j] = ld128<NT>(base[j], wa.lane_off + (uint32_t)s * wa.step_stride);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          st.bh[b] = ld128<false>(XH, b_off + (uint32_t)(s * NB + b) * 1024);
          if constexpr (!PK) st.bl[b] = ld128<false>(XL, b_off + (uint32_t)(s * NB + b) * 1024);
        }
      },
      [&](const Stage<2 * R, NB, PK>& st) {
        if constexpr (FP8) {
#pragma unroll
          for (int j = 0; j < 2 * R; ++j) {
            uint4 k0, k1;
            fp8x16_to_bf16(st.a[j], k0, k1);
            acc[j] = mfma_bf16(k0, st.bh[0], acc[j]);
            if constexpr (!PK) acc[j] = mfma_bf16(k0, st.bl[0], acc[j]);
            acc[j] = mfma_bf16(k1, st.bh[1], acc[j]);
            if constexpr (!PK) acc[j] = mfma_bf16(k1, st.bl[1], acc[j]);
          }
        } else {
#pragma unroll
          for (int j = 0; j < 2 * R; ++j) acc[j] = mfma_bf16(st.a[j], st.bh[0], acc[j]);
          if constexpr (!PK) {
#pragma unroll
            for (int j = 0; j < 2 * R; ++j) acc[j] = mfma_bf16(st.a[j], st.bl[0], acc[j]);
          }
        }
      });

  // reduce the W k-slices through LDS, then wave w finishes tiles w, w+W, ...
  if constexpr (W > 1) {
#pragma unroll
    for (int j = 0; j < 2 * R; ++j)
      red[(wave * 2 * R + j) * 64 + lane] = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
    __syncthreads();
  }
  uint16_t* HH = g.hf_hi + (size_t)slot * g.ffn * 16;
  uint16_t* HL = g.hf_lo + (size_t)slot * g.ffn * 16;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    if (j % W != wave || tile0 + j >= ntiles) continue;
    float4 G, U;
    if constexpr (W > 1) {
      G = red[j * 64 + lane];
      U = red[(R + j) * 64 + lane];
      for (int w = 1; w < W; ++w) {
        const float4 g2 = red[(w * 2 * R + j) * 64 + lane], u2 = red[(w * 2 * R + R + j) * 64 + lane];
        G.x += g2.x, G.y += g2.y, G.z += g2.z, G.w += g2.w;
        U.x += u2.x, U.y += u2.y, U.z += u2.z, U.w += u2.w;
      }
    } else {
      G = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
      U = float4{acc[R + j][0], acc[R + j][1], acc[R + j][2], acc[R + j][3]};
    }
    if constexpr (PK) {  // column n + 8 carries the lo-half contribution of token n: fold it in
      G.x += __shfl_xor(G.x, 8), G.y += __shfl_xor(G.y, 8), G.z += __shfl_xor(G.z, 8), G.w += __shfl_xor(G.w, 8);
      U.x += __shfl_xor(U.x, 8), U.y += __shfl_xor(U.y, 8), U.z += __shfl_xor(U.z, 8), U.w += __shfl_xor(U.w, 8);
    }
    if constexpr (FP8) {  // the lane's four rows of the tile are consecutive: one 16-byte load per scale vector
      const float4 c1 = *reinterpret_cast<const float4*>(S1 + (tile0 + j) * 16 + kg * 4);
      const float4 c3 = *reinterpret_cast<const float4*>(S3 + (tile0 + j) * 16 + kg * 4);
      G.x *= c1.x, G.y *= c1.y, G.z *= c1.z, G.w *= c1.w;
      U.x *= c3.x, U.y *= c3.y, U.z *= c3.z, U.w *= c3.w;
    }
    if (r < g.T && (!PK || r < kPackedTokens) && gate != 0.f) {
      // lane holds rows 4*kg .. 4*kg+3 of the tile for token column r: four consecutive k of the
      // down projection, i.e. one half of a 16-byte fragment unit
      uint16_t hi[4], lo[4];
      split_bf16(gate * (G.x / (1.f + expf(-G.x))) * U.x, hi[0], lo[0]);
      split_bf16(gate * (G.y / (1.f + expf(-G.y))) * U.y, hi[1], lo[1]);
      split_bf16(gate * (G.z / (1.f + expf(-G.z))) * U.z, hi[2], lo[2]);
      split_bf16(gate * (G.w / (1.f + expf(-G.w))) * U.w, hi[3], lo[3]);
      const int k = (tile0 + j) * 16 + kg * 4;
      const size_t o = frag_unit(k >> 3, r) * 8 + (k & 4);
      *reinterpret_cast<uint2*>(HH + o) =
          uint2{(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
      *reinterpret_cast<uint2*>((PK ? HH + kPackedTokens * 8 : HL) + o) =
          uint2{(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 4: down projection, split-K over (expert, k-chunk).  The gate is already folded into H, so
// every slab is a plain partial sum of out.
// grid = (row blocks of 16*R rows of d, min(E, T*top_k) + n_shared slots, KS k-chunks); block = W waves
// splitting the chunk.
// ------------------------------------------------------------------------------------------
struct DownArgs {
  const void *w2, *sw2;           // [E,d,ffn] / [n_shared,d,ffn], bf16 or FP8 codes
  const float *s2, *ss2;          // FP8 only: per-row scales [E,d] / [n_shared,d]
  const uint16_t *hf_hi, *hf_lo;  // [u_max + n_shared] fragments, ffn*16 elements each
  const int32_t* n_unique;
  const int32_t* slot_expert;
  const float* slot_gate;
  float* partial;                 // [(u_max + n_shared)*KS, max_tokens, d]
  int d, ffn, T, routed_slots, u_max, max_tokens, KS;
};

template <int R, int W, int P, bool TILED, bool NT, bool FP8, bool PK>
__global__ __launch_bounds__(64 * W) void down_kernel(DownArgs g) {
  constexpr int NB = FP8 ? 2 : 1;
  __shared__ float4 red[W > 1 ? W * R * 64 : 1];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const int ks = blockIdx.z;
  int slot = blockIdx.y;
  const char* W2;
  const float* S2 = nullptr;
  const size_t per = (size_t)g.ffn * g.d * (FP8 ? 1 : 2);
  bool live;  // token column r contributes only if the token is routed to this expert
  if (slot < g.routed_slots) {
    const int nu = *g.n_unique;  // three independent loads, one round trip
    const int e = g.slot_expert[slot];
    // 0 also for the padded columns r >= T; packed: column n + 8 belongs to token n
    live = g.slot_gate[slot * kGateCols + (PK ? (r & (kPackedTokens - 1)) : r)] != 0.f;
    if (slot >= nu) return;
    W2 = reinterpret_cast<const char*>(g.w2) + e * per;
    if constexpr (FP8) S2 = g.s2 + (size_t)e * g.d;
  } else {
    live = (PK ? (r & (kPackedTokens - 1)) : r) < g.T;
    const int sh = slot - g.routed_slots;
    W2 = reinterpret_cast<const char*>(g.sw2) + sh * per;
    if constexpr (FP8) S2 = g.ss2 + (size_t)sh * g.d;
    slot = g.u_max + sh;
  }
  const int ntiles = g.d >> 4, tile0 = blockIdx.x * R;
  const int nsteps = g.ffn >> (FP8 ? 6 : 5), parts = g.KS * W, chunk = (nsteps + parts - 1) / parts;
  const int nst = max(0, min(chunk, nsteps - (ks * W + wave) * chunk));
  const int s_beg = min((ks * W + wave) * chunk, nsteps - 1);  // a wave without work still issues in-bounds loads

  const WeightAddr<TILED, FP8> wa(g.ffn, r, kg, lane);
  const char* base[R];
#pragma unroll
  for (int j = 0; j < R; ++j)
    base[j] = W2 + (size_t)min(tile0 + j, ntiles - 1) * wa.tile_stride + (size_t)s_beg * wa.step_stride;
  const char* HH =
      reinterpret_cast<const char*>(g.hf_hi) + ((size_t)slot * g.ffn * 16 + (size_t)s_beg * (512 * NB)) * 2;
  const char* HL =
      reinterpret_cast<const char*>(g.hf_lo) + ((size_t)slot * g.ffn * 16 + (size_t)s_beg * (512 * NB)) * 2;
  const uint32_t b_off = lane * 16;

  f32x4 acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<R, NB, PK, P>(
      nst,
      [&](Stage<R, NB, PK>& st, int s) {
#pragma unroll
        for (int j = 0; j < R; ++j) st.a[j] = ld128<NT>(base[j], wa.lane_off + (uint32_t)s * wa.step_stride);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          st.bh[b] = uint4{0u, 0u, 0u, 0u};
          if constexpr (!PK) st.bl[b] = uint4{0u, 0u, 0u, 0u};
          if (live) {  // H of a token that was not routed here was never written: do not read it
            st.bh[b] = ld128<false>(HH, b_off + (uint32_t)(s * NB + b) * 1024);
            if constexpr (!PK) st.bl[b] = ld128<false>(HL, b_off + (uint32_t)(s * NB + b) * 1024);
          }
        }
      },
      [&](const Stage<R, NB, PK>& st) {
        if constexpr (FP8) {
#pragma unroll
          for (int j = 0; j < R; ++j) {
            uint4 k0, k1;
            fp8x16_to_bf16(st.a[j], k0, k1);
            acc[j] = mfma_bf16(k0, st.bh[0], acc[j]);
            if constexpr (!PK) acc[j] = mfma_bf16(k0, st.bl[0], acc[j]);
            acc[j] = mfma_bf16(k1, st.bh[1], acc[j]);
            if constexpr (!PK) acc[j] = mfma_bf16(k1, st.bl[1], acc[j]);
          }
        } else {
#pragma unroll
          for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], st.bh[0], acc[j]);
          if constexpr (!PK) {
#pragma unroll
            for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], st.bl[0], acc[j]);
          }
        }
      });

  if constexpr (W > 1) {
#pragma unroll
    for (int j = 0; j < R; ++j) red[(wave * R + j) * 64 + lane] = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < R; ++j) {
    if (j % W != wave || tile0 + j >= ntiles) continue;
    float4 y;
    if constexpr (W > 1) {
      y = red[j * 64 + lane];
      for (int w = 1; w < W; ++w) {
        const float4 y2 = red[(w * R + j) * 64 + lane];
        y.x += y2.x, y.y += y2.y, y.z += y2.z, y.w += y2.w;
      }
    } else {
      y = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
    }
    if constexpr (PK)  // column n + 8 carries the lo-half contribution of token n
      y.x += __shfl_xor(y.x, 8), y.y += __shfl_xor(y.y, 8), y.z += __shfl_xor(y.z, 8), y.w += __shfl_xor(y.w, 8);
    if constexpr (FP8) {  // scaling each split-K partial sum by the row scale = scaling the whole sum
      const float4 c2 = *reinterpret_cast<const float4*>(S2 + (tile0 + j) * 16 + kg * 4);
      y.x *= c2.x, y.y *= c2.y, y.z *= c2.z, y.w *= c2.w;
    }
    if (live && (!PK || r < kPackedTokens)) {  // nobody reads the slab column of a token that was not routed here
      const size_t o = (((size_t)slot * g.KS + ks) * g.max_tokens + r) * g.d + (size_t)(tile0 + j) * 16 + kg * 4;
      *reinterpret_cast<float4*>(g.partial + o) = y;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 5: out[t] = sum over the token's own picks i = 0 .. top_k-1 (the slot each landed in comes from
// the grouping step), then the shared experts; k-chunks ascending inside each.  A fixed order — the
// order of the defining sum — so reruns are bit-identical and no floating-point atomics are needed.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ partial,
                                                      const int32_t* __restrict__ tok_slot, float* __restrict__ out,
                                                      int d, int T, int top_k, int u_max, int n_shared,
                                                      int max_tokens, int KS) {
  const int i = blockIdx.x * 256 + threadIdx.x;  // float4 index inside [T, d]
  const int per_tok = d >> 2;
  if (i >= T * per_tok) return;
  const int t = i / per_tok, c4 = i - t * per_tok;
  float4 s = float4{0.f, 0.f, 0.f, 0.f};
  const size_t slab = (size_t)max_tokens * d;
  const float* p0 = partial + (size_t)t * d + (size_t)c4 * 4;
  // flat walk over (pick, k-chunk): unrolled by 8 so that eight slab loads are in flight at a time
  const int n = (top_k + n_shared) * KS;
#pragma unroll 8
  for (int q = 0; q < n; ++q) {
    const int j = q / KS, k = q - j * KS;
    const int u = j < top_k ? tok_slot[t * top_k + j] : u_max + (j - top_k);
    const float4 v = *reinterpret_cast<const float4*>(p0 + ((size_t)u * KS + k) * slab);
    s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
  }
  *reinterpret_cast<float4*>(out + (size_t)t * d + (size_t)c4 * 4) = s;
}

// ------------------------------------------------------------------------------------------
// Chained stack: one workgroup per token finishes block l-1 and prepares block l in one pass over d:
//   x_l = x_{l-1} + (slabs of the token's picks, as in combine_kernel)      -> resid_out
//   n   = x_l / sqrt(mean(x_l^2) + eps) * gamma_l                           -> xn_out (the router's input)
// partial == NULL: no MoE term (first block: x_0 is the caller's input).  gamma == NULL: no
// normalisation (after the last block only the residual stream is wanted).
// ------------------------------------------------------------------------------------------
struct ChainArgs {
  const float* partial;
  const int32_t* tok_slot;
  const float* resid_in;   // [T, d]
  float* resid_out;        // [T, d] or NULL
  const uint16_t* gamma;   // [d] bf16 or NULL
  float* xn_out;           // [T, d] fp32 normalised output, or NULL
  uint16_t *xf_hi, *xf_lo; // or: the normalised output as bf16 hi/lo fragments (MFMA B operand), or NULL
  int d, T, top_k, u_max, n_shared, max_tokens, KS;
  float eps;
};
constexpr int kChainThreads = 1024;
constexpr int kChainVecs = 4;  // float4 per thread: d <= 4 * 4 * 1024

__global__ __launch_bounds__(kChainThreads) void chain_kernel(ChainArgs g) {
  __shared__ float s_ss[kChainThreads / 64];
  const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int per_tok = g.d >> 2;
  const size_t slab = (size_t)g.max_tokens * g.d;
  const int n = g.partial ? (g.top_k + g.n_shared) * g.KS : 0;
  float4 v[kChainVecs];
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < kChainVecs; ++q) {
    const int c4 = tid + q * kChainThreads;
    v[q] = float4{0.f, 0.f, 0.f, 0.f};
    if (c4 < per_tok) {
      const size_t o = (size_t)t * g.d + (size_t)c4 * 4;
      float4 m = float4{0.f, 0.f, 0.f, 0.f};  // the MoE term, summed as combine_kernel sums it
#pragma unroll 8
      for (int i = 0; i < n; ++i) {
        const int j = i / g.KS, k = i - j * g.KS;
        const int u = j < g.top_k ? g.tok_slot[t * g.top_k + j] : g.u_max + (j - g.top_k);
        const float4 p = *reinterpret_cast<const float4*>(g.partial + o + ((size_t)u * g.KS + k) * slab);
        m.x += p.x, m.y += p.y, m.z += p.z, m.w += p.w;
      }
      const float4 x = *reinterpret_cast<const float4*>(g.resid_in + o);
      v[q] = float4{x.x + m.x, x.y + m.y, x.z + m.z, x.w + m.w};
      if (g.resid_out) *reinterpret_cast<float4*>(g.resid_out + o) = v[q];
      ss += v[q].x * v[q].x + v[q].y * v[q].y + v[q].z * v[q].z + v[q].w * v[q].w;
    }
  }
  if (!g.gamma) return;  // uniform over the grid
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if (lane == 0) s_ss[wave] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < kChainThreads / 64; ++w) tot += s_ss[w];
  const float root = sqrtf(tot / (float)g.d + g.eps);
#pragma unroll
  for (int q = 0; q < kChainVecs; ++q) {
    const int c4 = tid + q * kChainThreads;
    if (c4 < per_tok) {
      const uint2 gb = *reinterpret_cast<const uint2*>(g.gamma + (size_t)c4 * 4);
      float4 y;
      y.x = (v[q].x / root) * bf16_to_f32(gb.x & 0xffffu);
      y.y = (v[q].y / root) * bf16_to_f32(gb.x >> 16);
      y.z = (v[q].z / root) * bf16_to_f32(gb.y & 0xffffu);
      y.w = (v[q].w / root) * bf16_to_f32(gb.y >> 16);
      if (g.xn_out) *reinterpret_cast<float4*>(g.xn_out + (size_t)t * g.d + (size_t)c4 * 4) = y;
      if (g.xf_hi) {  // this thread's 4 values are one half of the 8-value fragment unit k8 = c4 / 2
        uint16_t hi[4], lo[4];
        split_bf16(y.x, hi[0], lo[0]);
        split_bf16(y.y, hi[1], lo[1]);
        split_bf16(y.z, hi[2], lo[2]);
        split_bf16(y.w, hi[3], lo[3]);
        const bool packed = g.T <= kPackedTokens;
        const size_t o = frag_unit(c4 >> 1, t) * 8 + (c4 & 1) * 4;
        *reinterpret_cast<uint2*>(g.xf_hi + o) =
            uint2{(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
        *reinterpret_cast<uint2*>((packed ? g.xf_hi + kPackedTokens * 8 : g.xf_lo) + o) =
            uint2{(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Attention stub.  linear_kernel: out[t, row] = sum_k W[row, k] X[t, k] (+ resid[t, row]) for a tiled bf16
// matrix and activation fragments — the down projection without slots or slabs: one workgroup per 16-row
// tile, its 4 waves split K, LDS reduce, wave 0 writes.  grid = rows / 16.
// ------------------------------------------------------------------------------------------
struct LinearArgs {
  const uint16_t* w;             // [rows, K] tiled
  const uint16_t *xf_hi, *xf_lo; // fragments of X, K*16 elements each
  const float* resid;            // [T, rows] or NULL
  float* out;                    // [T, rows]
  int rows, K, T;
};

template <bool PK>
__global__ __launch_bounds__(256) void linear_kernel(LinearArgs g) {
  constexpr int W = 4, P = 6;
  __shared__ float4 red[W * 64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const int nsteps = g.K >> 5, chunk = (nsteps + W - 1) / W;
  const int nst = max(0, min(chunk, nsteps - wave * chunk));
  const int s_beg = min(wave * chunk, nsteps - 1);
  const char* base = reinterpret_cast<const char*>(g.w) + (size_t)blockIdx.x * nsteps * 1024 + (size_t)s_beg * 1024;
  const char* XH = reinterpret_cast<const char*>(g.xf_hi) + (size_t)s_beg * 1024;
  const char* XL = reinterpret_cast<const char*>(g.xf_lo) + (size_t)s_beg * 1024;
  const uint32_t off = lane * 16;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  pipeline<1, 1, PK, P>(
      nst,
      [&](Stage<1, 1, PK>& st, int s) {
        st.a[0] = ld128<true>(base, off + (uint32_t)s * 1024);
        st.bh[0] = ld128<false>(XH, off + (uint32_t)s * 1024);
        if constexpr (!PK) st.bl[0] = ld128<false>(XL, off + (uint32_t)s * 1024);
      },
      [&](const Stage<1, 1, PK>& st) {
        acc = mfma_bf16(st.a[0], st.bh[0], acc);
        if constexpr (!PK) acc = mfma_bf16(st.a[0], st.bl[0], acc);
      });
  red[wave * 64 + lane] = float4{acc[0], acc[1], acc[2], acc[3]};
  __syncthreads();
  if (wave != 0) return;
  float4 y = red[lane];
  for (int w = 1; w < W; ++w) {
    const float4 y2 = red[w * 64 + lane];
    y.x += y2.x, y.y += y2.y, y.z += y2.z, y.w += y2.w;
  }
  if constexpr (PK)
    y.x += __shfl_xor(y.x, 8), y.y += __shfl_xor(y.y, 8), y.z += __shfl_xor(y.z, 8), y.w += __shfl_xor(y.w, 8);
  if (r < g.T && (!PK || r < kPackedTokens)) {
    const size_t o = (size_t)r * g.rows + (size_t)blockIdx.x * 16 + kg * 4;  // the lane's 4 rows are consecutive
    if (g.resid) {
      const float4 x = *reinterpret_cast<const float4*>(g.resid + o);
      y.x += x.x, y.y += x.y, y.z += x.z, y.w += x.w;
    }
    *reinterpret_cast<float4*>(g.out + o) = y;
  }
}

// Attention core of the stub: one workgroup per query head.  q, k, v of its (kv) head for the T in-flight tokens
// sit in LDS; scores, the causal softmax and the weighted sum of values are plain fp32 loops in index order
// (T <= 16, head_dim <= 128: a few thousand multiply-adds per head).  The head's output goes out as bf16 hi/lo
// fragments, the B operand of the output projection.
struct AttnArgs {
  const float* qkv;               // [T, (H + 2 Hkv) dh]
  uint16_t *of_hi, *of_lo;        // fragments of concat_h(o), H*dh*16 elements each
  int T, H, Hkv, dh;
};

__global__ __launch_bounds__(256) void attn_core_kernel(AttnArgs g) {
  __shared__ float s_q[kMaxTokens * 128], s_k[kMaxTokens * 128], s_v[kMaxTokens * 128];
  __shared__ float s_p[kMaxTokens * kMaxTokens];
  const int h = blockIdx.x, tid = threadIdx.x, T = g.T, dh = g.dh;
  const int kvh = h / (g.H / g.Hkv), nq = g.H * dh, nkv = g.Hkv * dh, nout = nq + 2 * nkv;
  for (int i = tid; i < T * dh; i += 256) {
    const int t = i / dh, j = i - t * dh;
    const float* row = g.qkv + (size_t)t * nout;
    s_q[i] = row[h * dh + j];
    s_k[i] = row[nq + kvh * dh + j];
    s_v[i] = row[nq + nkv + kvh * dh + j];
  }
  __syncthreads();
  const float scale = 1.f / sqrtf((float)dh);
  for (int i = tid; i < T * T; i += 256) {
    const int t = i / T, u = i - t * T;
    if (u <= t) {
      float s = 0.f;
      for (int j = 0; j < dh; ++j) s += s_q[t * dh + j] * s_k[u * dh + j];
      s_p[t * kMaxTokens + u] = s * scale;
    }
  }
  __syncthreads();
  if (tid < T) {  // row tid: max, exponentials, sum in index order, normalise
    float* p = s_p + tid * kMaxTokens;
    float m = p[0];
    for (int u = 1; u <= tid; ++u) m = fmaxf(m, p[u]);
    float sum = 0.f;
    for (int u = 0; u <= tid; ++u) {
      p[u] = expf(p[u] - m);
      sum += p[u];
    }
    for (int u = 0; u <= tid; ++u) p[u] = p[u] / sum;
  }
  __syncthreads();
  const bool packed = T <= kPackedTokens;
  for (int i = tid; i < T * (dh >> 3); i += 256) {  // (token, unit of 8 output dims)
    const int t = i / (dh >> 3), j0 = (i - t * (dh >> 3)) * 8;
    float o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = 0.f;
    for (int u = 0; u <= t; ++u) {
      const float pu = s_p[t * kMaxTokens + u];
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] += pu * s_v[u * dh + j0 + j];
    }
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint16_t h0, l0, h1, l1;
      split_bf16(o[2 * j], h0, l0);
      split_bf16(o[2 * j + 1], h1, l1);
      hi[j] = (uint32_t)h0 | ((uint32_t)h1 << 16);
      lo[j] = (uint32_t)l0 | ((uint32_t)l1 << 16);
    }
    const size_t q = frag_unit((h * dh + j0) >> 3, t);
    reinterpret_cast<uint4*>(g.of_hi)[q] = uint4{hi[0], hi[1], hi[2], hi[3]};
    if (packed)
      reinterpret_cast<uint4*>(g.of_hi)[q + kPackedTokens] = uint4{lo[0], lo[1], lo[2], lo[3]};
    else
      reinterpret_cast<uint4*>(g.of_lo)[q] = uint4{lo[0], lo[1], lo[2], lo[3]};
  }
}

// One-off re-layout of a row-major [rows, K] bf16 matrix into the tiled order (see WeightAddr).
__global__ __launch_bounds__(256) void pack_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t rows,
                                                   int K) {
  const size_t nsteps = (size_t)(K >> 5), units = rows * (size_t)(K >> 3);
  for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < units; q += (size_t)gridDim.x * 256) {
    const size_t blk = q >> 6;
    const int l = (int)(q & 63), rr = l & 15, kk = l >> 4;
    const size_t tile = blk / nsteps, st = blk % nsteps;
    dst[q] = src[((tile * 16 + rr) * (size_t)K + st * 32 + kk * 8) >> 3];
  }
}

// The same for FP8 codes: a 1 KB block holds 16 rows x 64 k; unit l = (r, kg) = the 8 codes of k-step
// 2p followed by the 8 codes of k-step 2p+1.
__global__ __launch_bounds__(256) void pack_kernel_fp8(const uint2* __restrict__ src, uint4* __restrict__ dst,
                                                       size_t rows, int K) {
  const size_t npairs = (size_t)(K >> 6), units = rows * (size_t)(K >> 4);
  for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < units; q += (size_t)gridDim.x * 256) {
    const size_t blk = q >> 6;
    const int l = (int)(q & 63), rr = l & 15, kk = l >> 4;
    const size_t tile = blk / npairs, pr = blk % npairs;
    const size_t i0 = ((tile * 16 + rr) * (size_t)K + pr * 64 + kk * 8) >> 3;
    const uint2 a = src[i0], b = src[i0 + 4];
    dst[q] = uint4{a.x, a.y, b.x, b.y};
  }
}

// ------------------------------------------------------------------------------------------
// Measurement aid: plain coalesced read stream.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16_per_wave,
                                                          size_t n16, float* __restrict__ sink) {
  // every wave owns one contiguous chunk and keeps 8 non-temporal 1 KB loads in flight: the access
  // pattern that gave the highest read rate on this chip
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const size_t beg = wave * n16_per_wave;
  const size_t end = beg + n16_per_wave < n16 ? beg + n16_per_wave : n16;
  uint32_t acc = 0;
  size_t i = beg + lane;
  for (; i + 7 * 64 < end; i += 8 * 64) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld128<true>(reinterpret_cast<const char*>(src + i + 64 * u), 0);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < end; i += 64) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if (lane == 0) atomicXor(reinterpret_cast<unsigned int*>(sink) + (blockIdx.x & 4095), acc);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

// ------------------------------------------------------------------------------------------
// Host side of the device ABI
// ------------------------------------------------------------------------------------------
struct moe_ctx {
  moe_shape s;
  int device;
  int u_max;              // largest possible union: min(E, max_tokens * top_k)
  int ks_alloc;           // split-K slabs the partial buffer is sized for
  int plan_override[3];   // MOE_PLAN=guR,dnR,dnKS (tuning), zeros = automatic
  char* ws;
  size_t ws_bytes;
  uint16_t *xf_hi, *xf_lo, *hf_hi, *hf_lo;  // activation fragments (see frag_unit)
  int32_t *ids, *n_unique, *slot_expert, *tok_slot;
  float *gates, *slot_gate, *partial;
  float *xn, *resid[2];  // chained stack: normalised router input and the residual stream (ping-pong), [max_tokens, d]
  float *hbuf, *qkv;     // decoder stack: stream after the attention half [max_tokens, d]; q|k|v [max_tokens, (H+2Hkv) dh]
  uint16_t *af_hi, *af_lo;  // decoder stack: fragments of the attention output, H*dh*16 elements each
  bool profiling;
  std::vector<hipEvent_t> events;  // kProfMarks per profiled layer-step
};

namespace {

constexpr int kProfMarks = 5;  // events per profiled layer-step: route, gate/up, down, combine
constexpr int kWaves = 4;    // waves per workgroup in the expert kernels (they split K)
constexpr int kMaxKS = 16;   // largest split-K factor of the down projection

// Launch plan of the two expert kernels for one (T, weight layout).
//   gu_R, dn_R  weight tiles (16 rows) per wave; the pipeline depth is tied to it (fewer tiles ->
//               deeper pipeline, same bytes in flight per wave)
//   dn_KS       split-K factor of the down projection across workgroups
// Chosen from measurements on Mixtral-shaped layers (see plan_for).
struct Plan {
  int gu_R, dn_R, dn_KS;
};

int ks_cap_for(const moe_shape& s, bool fp8) {
  const int nsteps = s.ffn / (fp8 ? 64 : 32);
  int cap = 1;
  while (cap < kMaxKS && nsteps / (kWaves * cap * 2) >= 4) cap *= 2;  // every wave keeps >= 4 k-steps
  return cap;
}

Plan plan_for(const moe_ctx* c, int T, bool tiled, bool fp8) {
  const moe_shape& s = c->s;
  // expected number of live expert slots for T tokens under uniform routing (balls into bins)
  double miss = 1.0;
  for (int t = 0; t < T; ++t) miss *= 1.0 - (double)s.top_k / s.n_experts;
  const double slots = s.n_experts * (1.0 - miss) + s.n_shared;
  Plan p;
  p.gu_R = tiled ? 1 : ((s.ffn / 16 / 2) * kWaves * slots >= 1536 ? 2 : 1);
  const int cap = ks_cap_for(s, fp8);
  p.dn_R = 1;
  p.dn_KS = cap;
  // measured on Mixtral-shaped layers: 4 k-chunks per (row block, slot) is within 1 us of the best split for
  // every T (1 chunk loses 10 %, 8 chunks make the slab sum longer than they shorten the projection); grids
  // that already hold four thousand waves (many small experts) are not split, tiny grids are split further
  // until about a thousand waves are in flight
  for (int R : {4, 2, 1}) {
    const double per_ks = (double)((s.d / 16 + R - 1) / R) * kWaves * slots;
    int ks = 1;
    while (ks < cap && per_ks * ks < (ks < 4 ? 4096 : 1024)) ks *= 2;
    if (per_ks * ks >= 1024 || R == 1) {
      p.dn_R = R;
      p.dn_KS = ks;
      break;
    }
  }
  if (c->plan_override[0] > 0) {
    p.gu_R = c->plan_override[0];
    p.dn_R = c->plan_override[1];
    p.dn_KS = c->plan_override[2] < cap ? c->plan_override[2] : cap;
  }
  return p;
}

moe_status check_stream_device(const moe_ctx* c) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
  return dev == c->device ? MOE_OK : MOE_ERR_INVALID_ARG;
}

// profiling mode only: drop an event into the stream between kernels
void mark(moe_ctx* c, hipStream_t st) {
  if (!c->profiling) return;
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return;
  (void)hipEventRecord(e, st);
  c->events.push_back(e);
}

// Steps 1 and 2.  ids / gates / unique / n_unique / n_unique_extra: optional DEVICE outputs.
void launch_route_and_group(moe_ctx* c, const float* hidden, const uint16_t* router_w, int T, int32_t* ids,
                            float* gates, int32_t* unique, int32_t* n_unique, int32_t* n_unique_extra, hipStream_t st) {
  const moe_shape& s = c->s;
  RouteArgs ra{hidden, router_w, s.d, s.n_experts, s.top_k, T, s.gate_mode, c->ids, ids, c->gates, gates,
               c->xf_hi, c->xf_lo};
  GroupArgs ga{c->ids, c->gates, T, s.top_k, s.n_experts, unique, n_unique, nullptr, nullptr, nullptr,
               c->n_unique, n_unique_extra, c->slot_expert, c->tok_slot, c->slot_gate};
  hipLaunchKernelGGL(route_kernel, dim3(T), dim3(64 * kRouteWaves), 0, st, ra, ga);
  if (T > 1) hipLaunchKernelGGL(group_kernel, dim3(1), dim3(256), 0, st, ga);  // T = 1: done inside route_kernel
}

template <int R, int P>
void launch_gateup(const moe_ctx* c, const GateupArgs& a, hipStream_t st) {  // row-major bf16 weights
  const dim3 grid((c->s.ffn / 16 + R - 1) / R, a.routed_slots + c->s.n_shared);
  if (a.T <= kPackedTokens)
    hipLaunchKernelGGL((gateup_kernel<R, kWaves, P, false, false, false, true>), grid, dim3(64 * kWaves), 0, st, a);
  else
    hipLaunchKernelGGL((gateup_kernel<R, kWaves, P, false, false, false, false>), grid, dim3(64 * kWaves), 0, st, a);
}
// Tiled weights are read exactly once in contiguous 1 KB pieces -> streaming loads; row-major weights
// are read in 64-byte row segments whose cache lines are completed by the next k-step -> cached loads.
template <int R, int P>
void launch_down(const moe_ctx* c, const DownArgs& a, bool tiled, bool fp8, hipStream_t st) {
  const dim3 grid((c->s.d / 16 + R - 1) / R, a.routed_slots + c->s.n_shared, a.KS), block(64 * kWaves);
  const bool pk = a.T <= kPackedTokens;
  if (fp8) {  // tiled only (checked by the caller)
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, true, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, true, false>), grid, block, 0, st, a);
  } else if (tiled) {
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, false, false>), grid, block, 0, st, a);
  } else {
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, P, false, false, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, P, false, false, false, false>), grid, block, 0, st, a);
  }
}

// One layer-step after validation: router, gate/up, down, slab sum.  The expert-union step has no
// launch of its own: it is the liveness test at the top of the expert kernels.
// unique / n_unique / n_unique_extra: optional DEVICE outputs.
// out == NULL: the slabs are left for the caller (chained stack: chain_kernel sums them); *ks_used gets the
// split-K factor they were written with.
moe_status launch_layer(moe_ctx* c, const moe_layer_weights* w, const float* hidden, int T, float* out, int32_t* ids,
                        float* gates, int32_t* unique, int32_t* n_unique, int32_t* n_unique_extra, hipStream_t st,
                        int* ks_used = nullptr) {
  const moe_shape& s = c->s;
  const bool tiled = w->layout == MOE_LAYOUT_TILED, fp8 = w->dtype == MOE_WEIGHT_FP8_E4M3;
  if (fp8 && !tiled) return MOE_ERR_UNIMPLEMENTED;  // FP8 is streamed in the tiled layout only
  const Plan p = plan_for(c, T, tiled, fp8);
  mark(c, st);
  launch_route_and_group(c, hidden, w->router_w, T, ids, gates, unique, n_unique, n_unique_extra, st);
  mark(c, st);
  const int routed_slots = T * s.top_k < s.n_experts ? T * s.top_k : s.n_experts;  // largest union T tokens can form
  GateupArgs ga{w->w1, w->w3, w->sw1, w->sw3, w->w1_scale, w->w3_scale, w->sw1_scale, w->sw3_scale,
                c->xf_hi, c->xf_lo, c->n_unique, c->slot_expert, c->slot_gate,
                c->hf_hi, c->hf_lo, s.d, s.ffn, T, routed_slots, c->u_max};
  const bool pk = T <= kPackedTokens;  // must match what route_kernel wrote
  if (fp8) {
    // FP8 needs twice the fragment bytes per weight byte, and those come from L2: two tile pairs per wave
    // share each fragment load, and a shallow pipeline keeps four waves per SIMD (measured best of
    // {1, 2, 4} tile pairs x depths 2..10)
    const dim3 grid((s.ffn / 16 + 1) / 2, routed_slots + s.n_shared);
    if (pk) hipLaunchKernelGGL((gateup_kernel<2, 1, 3, true, true, true, true>), grid, dim3(64), 0, st, ga);
    else hipLaunchKernelGGL((gateup_kernel<2, 1, 3, true, true, true, false>), grid, dim3(64), 0, st, ga);
  } else if (tiled) {
    // one wave per 16-row tile pair over the whole of d (splitting d over 2 or 4 waves when the union
    // is small on a small expert was measured: no gain, the step is bound by launch latencies there)
    const dim3 grid(s.ffn / 16, routed_slots + s.n_shared);
    if (pk) hipLaunchKernelGGL((gateup_kernel<1, 1, 6, true, true, false, true>), grid, dim3(64), 0, st, ga);
    else hipLaunchKernelGGL((gateup_kernel<1, 1, 8, true, true, false, false>), grid, dim3(64), 0, st, ga);
  } else {
    switch (p.gu_R) {
      case 4: launch_gateup<4, 2>(c, ga, st); break;
      case 2: launch_gateup<2, 4>(c, ga, st); break;
      default: launch_gateup<1, 8>(c, ga, st); break;
    }
  }
  mark(c, st);
  DownArgs da{w->w2, w->sw2, w->w2_scale, w->sw2_scale, c->hf_hi, c->hf_lo, c->n_unique, c->slot_expert,
              c->slot_gate, c->partial, s.d, s.ffn, T, routed_slots, c->u_max, s.max_tokens, p.dn_KS};
  switch (p.dn_R) {
    case 4: launch_down<4, 4>(c, da, tiled, fp8, st); break;
    case 2: launch_down<2, 4>(c, da, tiled, fp8, st); break;
    default: launch_down<1, 8>(c, da, tiled, fp8, st); break;
  }
  mark(c, st);
  if (ks_used) *ks_used = p.dn_KS;
  if (out) {
    const int n4 = T * (s.d / 4);
    hipLaunchKernelGGL(combine_kernel, dim3((n4 + 255) / 256), dim3(256), 0, st, (const float*)c->partial,
                       (const int32_t*)c->tok_slot, out, s.d, T, s.top_k, c->u_max, s.n_shared, s.max_tokens, p.dn_KS);
  }
  mark(c, st);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// kernels use 128-bit loads: every tensor base must be 16-byte aligned (rows are, since d, ffn % 32 == 0)
bool weights_ok(const moe_ctx* c, const moe_layer_weights* w) {
  if (!w || !w->router_w || !w->w1 || !w->w3 || !w->w2) return false;
  if (w->layout != MOE_LAYOUT_ROW_MAJOR && w->layout != MOE_LAYOUT_TILED) return false;
  if (w->dtype != MOE_WEIGHT_BF16 && w->dtype != MOE_WEIGHT_FP8_E4M3) return false;
  if (w->dtype == MOE_WEIGHT_FP8_E4M3) {
    if (c->s.d % 64 || c->s.ffn % 64) return false;
    if (!w->w1_scale || !w->w3_scale || !w->w2_scale) return false;
    if (!aligned16(w->w1_scale) || !aligned16(w->w3_scale) || !aligned16(w->w2_scale)) return false;
    if (c->s.n_shared > 0) {
      if (!w->sw1_scale || !w->sw3_scale || !w->sw2_scale) return false;
      if (!aligned16(w->sw1_scale) || !aligned16(w->sw3_scale) || !aligned16(w->sw2_scale)) return false;
    }
  }
  if (!aligned16(w->router_w) || !aligned16(w->w1) || !aligned16(w->w3) || !aligned16(w->w2)) return false;
  if (c->s.n_shared > 0) {
    if (!w->sw1 || !w->sw3 || !w->sw2) return false;
    if (!aligned16(w->sw1) || !aligned16(w->sw3) || !aligned16(w->sw2)) return false;
  }
  return true;
}

}  // namespace

extern "C" {

const char* moe_strerror(moe_status s) {
  switch (s) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED_SHAPE: return "unsupported layer shape";
    case MOE_ERR_WORKSPACE: return "device workspace allocation failed";
    case MOE_ERR_HIP: return "HIP runtime error";
    case MOE_ERR_UNIMPLEMENTED: return "not implemented";
  }
  return "unknown status";
}

int moe_abi_version(void) { return 2; }

moe_status moe_ctx_create(const moe_shape* shape, moe_ctx** out) {
  if (out) *out = nullptr;
  if (!shape || !out) return MOE_ERR_INVALID_ARG;
  const moe_shape s = *shape;
  if (s.d < 32 || s.ffn < 32 || s.n_experts < 1 || s.top_k < 1 || s.n_shared < 0 || s.max_tokens < 1)
    return MOE_ERR_INVALID_ARG;
  if (s.top_k > s.n_experts) return MOE_ERR_INVALID_ARG;
  if (s.gate_mode != MOE_GATE_RENORM_TOPK && s.gate_mode != MOE_GATE_SOFTMAX_ALL) return MOE_ERR_INVALID_ARG;
  if (s.n_heads < 0 || s.n_kv_heads < 0 || s.head_dim < 0) return MOE_ERR_INVALID_ARG;
  if (s.n_heads == 0 && (s.n_kv_heads != 0 || s.head_dim != 0)) return MOE_ERR_INVALID_ARG;
  if (s.n_heads > 0) {
    if (s.n_kv_heads < 1 || s.n_heads % s.n_kv_heads) return MOE_ERR_INVALID_ARG;
    if (s.head_dim < 32 || s.head_dim > 128 || s.head_dim % 32 || s.n_heads > 1024) return MOE_ERR_UNSUPPORTED_SHAPE;
  }
  if (s.d % 32 || s.ffn % 32 || s.n_experts > kMaxExperts || s.top_k > kMaxTopK || s.n_shared > kMaxShared ||
      s.max_tokens > kMaxTokens || (int64_t)s.d * s.ffn > (int64_t)1 << 30)
    return MOE_ERR_UNSUPPORTED_SHAPE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
  moe_ctx* c = new (std::nothrow) moe_ctx();
  if (!c) return MOE_ERR_WORKSPACE;
  c->s = s;
  c->device = dev;
  c->profiling = false;
  c->u_max = s.max_tokens * s.top_k < s.n_experts ? s.max_tokens * s.top_k : s.n_experts;
  c->plan_override[0] = c->plan_override[1] = c->plan_override[2] = 0;
  if (const char* env = getenv("MOE_PLAN")) {  // tuning override: "guR,dnR,dnKS"
    int a = 0, b = 0, k = 0;
    if (sscanf(env, "%d,%d,%d", &a, &b, &k) == 3 && (a == 1 || a == 2 || a == 4) && (b == 1 || b == 2 || b == 4) &&
        k >= 1 && k <= kMaxKS) {
      c->plan_override[0] = a;
      c->plan_override[1] = b;
      c->plan_override[2] = k;
    }
  }
  // the slab buffer is sized for the largest split-K factor any T can ask for
  c->ks_alloc = 1;
  for (int T = 1; T <= s.max_tokens; ++T)
    for (bool tiled : {false, true})
      for (bool fp8 : {false, true}) {
        const int ks = plan_for(c, T, tiled, fp8).dn_KS;
        if (ks > c->ks_alloc) c->ks_alloc = ks;
      }

  const size_t A = (size_t)s.max_tokens * s.top_k;
  size_t off = 0;
  auto carve = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const size_t o_xh = carve((size_t)s.d * kGateCols * 2), o_xl = carve((size_t)s.d * kGateCols * 2);
  const size_t n_slots = (size_t)c->u_max + s.n_shared;
  const size_t o_hh = carve(n_slots * s.ffn * kGateCols * 2);
  const size_t o_hl = carve(n_slots * s.ffn * kGateCols * 2);
  const size_t o_ids = carve(A * 4), o_gates = carve(A * 4), o_nu = carve(4);
  const size_t o_se = carve((size_t)c->u_max * 4), o_sg = carve(n_slots * kGateCols * 4), o_ts = carve(A * 4);
  const size_t o_part = carve(n_slots * c->ks_alloc * s.max_tokens * s.d * 4);
  const size_t o_xn = carve((size_t)s.max_tokens * s.d * 4);
  const size_t o_r0 = carve((size_t)s.max_tokens * s.d * 4), o_r1 = carve((size_t)s.max_tokens * s.d * 4);
  const size_t nq = (size_t)s.n_heads * s.head_dim, nqkv = nq + 2 * (size_t)s.n_kv_heads * s.head_dim;
  const size_t o_hb = carve((size_t)s.max_tokens * s.d * 4), o_qkv = carve((size_t)s.max_tokens * nqkv * 4 + 16);
  const size_t o_ah = carve(nq * kGateCols * 2 + 16), o_al = carve(nq * kGateCols * 2 + 16);
  c->ws_bytes = off;
  if (c->ws_bytes > ((size_t)8 << 30) || hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return MOE_ERR_WORKSPACE;
  }
  c->xf_hi = reinterpret_cast<uint16_t*>(c->ws + o_xh);
  c->xf_lo = reinterpret_cast<uint16_t*>(c->ws + o_xl);
  c->hf_hi = reinterpret_cast<uint16_t*>(c->ws + o_hh);
  c->hf_lo = reinterpret_cast<uint16_t*>(c->ws + o_hl);
  c->ids = reinterpret_cast<int32_t*>(c->ws + o_ids);
  c->gates = reinterpret_cast<float*>(c->ws + o_gates);
  c->n_unique = reinterpret_cast<int32_t*>(c->ws + o_nu);
  c->slot_expert = reinterpret_cast<int32_t*>(c->ws + o_se);
  c->slot_gate = reinterpret_cast<float*>(c->ws + o_sg);
  c->tok_slot = reinterpret_cast<int32_t*>(c->ws + o_ts);
  c->partial = reinterpret_cast<float*>(c->ws + o_part);
  c->xn = reinterpret_cast<float*>(c->ws + o_xn);
  c->resid[0] = reinterpret_cast<float*>(c->ws + o_r0);
  c->resid[1] = reinterpret_cast<float*>(c->ws + o_r1);
  c->hbuf = reinterpret_cast<float*>(c->ws + o_hb);
  c->qkv = reinterpret_cast<float*>(c->ws + o_qkv);
  c->af_hi = reinterpret_cast<uint16_t*>(c->ws + o_ah);
  c->af_lo = reinterpret_cast<uint16_t*>(c->ws + o_al);
  if (hipMemset(c->ws, 0, c->ws_bytes) != hipSuccess) {  // padded token columns of the fragments are finite zeros
    (void)hipFree(c->ws);
    delete c;
    return MOE_ERR_HIP;
  }
  if (s.n_shared > 0) {  // shared-expert slots carry gate 1 for every token column
    float ones[kMaxShared * kGateCols];
    for (int i = 0; i < s.n_shared * kGateCols; ++i) ones[i] = 1.f;
    if (hipMemcpy(c->slot_gate + (size_t)c->u_max * kGateCols, ones, sizeof(float) * s.n_shared * kGateCols,
                  hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipFree(c->ws);
      delete c;
      return MOE_ERR_HIP;
    }
  }
  *out = c;
  return MOE_OK;
}

moe_status moe_ctx_destroy(moe_ctx* c) {
  if (!c) return MOE_OK;
  for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
  const hipError_t e = hipFree(c->ws);
  delete c;
  return e == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int64_t moe_ctx_workspace_bytes(const moe_ctx* c) { return c ? (int64_t)c->ws_bytes : 0; }

moe_status moe_route(moe_ctx* c, const float* hidden, const uint16_t* router_w, int32_t T, int32_t* ids, float* gates,
                     int32_t* unique_experts, int32_t* n_unique, void* stream) {
  if (!c || !hidden || !router_w || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(router_w)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  launch_route_and_group(c, hidden, router_w, T, ids, gates, unique_experts, n_unique, nullptr, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_group(moe_ctx* c, const int32_t* ids, int32_t T, int32_t* unique_experts, int32_t* n_unique,
                     int32_t* expert_count, int32_t* expert_offset, int32_t* assign, void* stream) {
  if (!c || !ids || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  GroupArgs ga{ids, nullptr, T, c->s.top_k, c->s.n_experts, unique_experts, n_unique, expert_count, expert_offset,
               assign, nullptr, nullptr, nullptr, nullptr, nullptr};
  hipLaunchKernelGGL(group_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, ga);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_verify_layer(moe_ctx* c, const moe_layer_weights* w, const float* hidden, int32_t T, float* out,
                            int32_t* ids_opt, float* gates_opt, int32_t* unique_opt, int32_t* n_unique_opt,
                            void* stream) {
  if (!c || !hidden || !out || T < 1 || T > c->s.max_tokens || !weights_ok(c, w)) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(out)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  hipStream_t st = (hipStream_t)stream;
  return launch_layer(c, w, hidden, T, out, ids_opt, gates_opt, unique_opt, n_unique_opt, nullptr, st);
}

moe_status moe_verify_stack(moe_ctx* c, const moe_layer_weights* layers, int32_t L, const float* hidden, int32_t T,
                            float* out, int32_t* n_unique_per_layer_opt, void* stream) {
  if (!c || !layers || L < 1 || !hidden || !out || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(out)) return MOE_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l) {
    if (!weights_ok(c, layers + l)) return MOE_ERR_INVALID_ARG;
    if (layers[l].dtype == MOE_WEIGHT_FP8_E4M3 && layers[l].layout != MOE_LAYOUT_TILED) return MOE_ERR_UNIMPLEMENTED;
  }
  if (moe_status st = check_stream_device(c)) return st;
  hipStream_t st = (hipStream_t)stream;
  const size_t per = (size_t)T * c->s.d;
  for (int l = 0; l < L; ++l) {
    if (moe_status rc = launch_layer(c, layers + l, hidden + l * per, T, out + l * per, nullptr, nullptr, nullptr,
                                     nullptr, n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st))
      return rc;
  }
  return MOE_OK;
}

moe_status moe_chained_stack(moe_ctx* c, const moe_layer_weights* layers, const uint16_t* const* gammas, int32_t L,
                             const float* x_in, int32_t T, float eps, float* x_out, float* trace_opt,
                             int32_t* n_unique_per_layer_opt, void* stream) {
  if (!c || !layers || !gammas || L < 1 || !x_in || !x_out || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!(eps >= 0.f) || !aligned16(x_in) || !aligned16(x_out) || (trace_opt && !aligned16(trace_opt)))
    return MOE_ERR_INVALID_ARG;
  if (c->s.d > 4 * kChainVecs * kChainThreads) return MOE_ERR_UNSUPPORTED_SHAPE;
  for (int l = 0; l < L; ++l) {
    if (!weights_ok(c, layers + l) || !gammas[l] || !aligned16(gammas[l])) return MOE_ERR_INVALID_ARG;
    if (layers[l].dtype == MOE_WEIGHT_FP8_E4M3 && layers[l].layout != MOE_LAYOUT_TILED) return MOE_ERR_UNIMPLEMENTED;
  }
  if (moe_status st = check_stream_device(c)) return st;
  hipStream_t st = (hipStream_t)stream;
  const moe_shape& s = c->s;
  const size_t per = (size_t)T * s.d;
  const float* cur = x_in;  // x_{l-1}: the stream the pending MoE term is added to
  int ks = 1;
  for (int l = 0; l <= L; ++l) {
    // finish block l-1 (if any) and, unless this is the end, normalise for block l
    ChainArgs a{};
    a.partial = l > 0 ? c->partial : nullptr;
    a.tok_slot = c->tok_slot;
    a.resid_in = cur;
    float* dst = l == L ? x_out : (trace_opt ? trace_opt + (size_t)l * per : (l > 0 ? c->resid[l & 1] : nullptr));
    a.resid_out = dst;  // l == 0 without a trace: x_0 stays where the caller has it
    a.gamma = l < L ? gammas[l] : nullptr;
    a.xn_out = c->xn;
    a.d = s.d, a.T = T, a.top_k = s.top_k, a.u_max = c->u_max, a.n_shared = s.n_shared, a.max_tokens = s.max_tokens;
    a.KS = ks, a.eps = eps;
    if (l > 0 || dst || a.gamma) hipLaunchKernelGGL(chain_kernel, dim3(T), dim3(kChainThreads), 0, st, a);
    if (dst) cur = dst;
    if (l == L) break;
    if (moe_status rc = launch_layer(c, layers + l, c->xn, T, nullptr, nullptr, nullptr, nullptr, nullptr,
                                     n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st, &ks))
      return rc;
  }
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_pack_matrix(moe_ctx* c, const void* src, void* dst, int64_t rows, int32_t K, int32_t dtype,
                           void* stream) {
  if (!c || !src || !dst || rows < 16 || rows % 16 || K < 32 || !aligned16(src) || !aligned16(dst)) return MOE_ERR_INVALID_ARG;
  if (dtype != MOE_WEIGHT_BF16 && dtype != MOE_WEIGHT_FP8_E4M3) return MOE_ERR_INVALID_ARG;
  const bool fp8 = dtype == MOE_WEIGHT_FP8_E4M3;
  if (K % (fp8 ? 64 : 32) || rows * (int64_t)K > (int64_t)1 << 34) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  const size_t units = (size_t)rows * (size_t)(K / (fp8 ? 16 : 8));
  const unsigned blocks = (unsigned)((units + 255) / 256 < 65536 ? (units + 255) / 256 : 65536);
  if (fp8)
    hipLaunchKernelGGL(pack_kernel_fp8, dim3(blocks), dim3(256), 0, (hipStream_t)stream, static_cast<const uint2*>(src),
                       static_cast<uint4*>(dst), (size_t)rows, K);
  else
    hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), (size_t)rows, K);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_decoder_stack(moe_ctx* c, const moe_layer_weights* layers, const moe_attn_weights* attn, int32_t L,
                             const float* x_in, int32_t T, float eps, float* x_out, float* trace_opt,
                             int32_t* n_unique_per_layer_opt, void* stream) {
  if (!c || !layers || !attn || L < 1 || !x_in || !x_out || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!(eps >= 0.f) || !aligned16(x_in) || !aligned16(x_out) || (trace_opt && !aligned16(trace_opt)))
    return MOE_ERR_INVALID_ARG;
  const moe_shape& s = c->s;
  if (s.n_heads < 1) return MOE_ERR_INVALID_ARG;  // the context was created without the attention geometry
  if (s.d > 4 * kChainVecs * kChainThreads) return MOE_ERR_UNSUPPORTED_SHAPE;
  for (int l = 0; l < L; ++l) {
    if (!weights_ok(c, layers + l)) return MOE_ERR_INVALID_ARG;
    if (layers[l].dtype == MOE_WEIGHT_FP8_E4M3 && layers[l].layout != MOE_LAYOUT_TILED) return MOE_ERR_UNIMPLEMENTED;
    const moe_attn_weights& a = attn[l];
    if (!a.wqkv || !a.wo || !a.gamma_attn || !a.gamma_moe) return MOE_ERR_INVALID_ARG;
    if (!aligned16(a.wqkv) || !aligned16(a.wo) || !aligned16(a.gamma_attn) || !aligned16(a.gamma_moe))
      return MOE_ERR_INVALID_ARG;
  }
  if (moe_status st = check_stream_device(c)) return st;
  hipStream_t st = (hipStream_t)stream;
  const size_t per = (size_t)T * s.d;
  const int nq = s.n_heads * s.head_dim, nqkv = nq + 2 * s.n_kv_heads * s.head_dim;
  const bool pk = T <= kPackedTokens;
  auto linear = [&](const LinearArgs& a) {
    if (pk) hipLaunchKernelGGL(linear_kernel<true>, dim3(a.rows / 16), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(linear_kernel<false>, dim3(a.rows / 16), dim3(256), 0, st, a);
  };
  ChainArgs base{};
  base.tok_slot = c->tok_slot;
  base.d = s.d, base.T = T, base.top_k = s.top_k, base.u_max = c->u_max, base.n_shared = s.n_shared;
  base.max_tokens = s.max_tokens, base.eps = eps;
  const float* cur = x_in;  // the stream the pending MoE term (if any) is added to
  int ks = 1;
  for (int l = 0; l <= L; ++l) {
    // x_l = (stream after the previous attention half) + (previous MoE term); normalise for this block's attention
    ChainArgs a = base;
    a.partial = l > 0 ? c->partial : nullptr;
    a.KS = ks;
    a.resid_in = cur;
    float* dst = l == L ? x_out : (trace_opt ? trace_opt + (size_t)l * per : (l > 0 ? c->resid[l & 1] : nullptr));
    a.resid_out = dst;
    if (l < L) {
      a.gamma = attn[l].gamma_attn;
      a.xf_hi = c->xf_hi, a.xf_lo = c->xf_lo;
    }
    if (l > 0 || dst || a.gamma) hipLaunchKernelGGL(chain_kernel, dim3(T), dim3(kChainThreads), 0, st, a);
    if (dst) cur = dst;
    if (l == L) break;
    // attention half: q|k|v projection, core, output projection + residual -> h
    linear(LinearArgs{attn[l].wqkv, c->xf_hi, c->xf_lo, nullptr, c->qkv, nqkv, s.d, T});
    hipLaunchKernelGGL(attn_core_kernel, dim3(s.n_heads), dim3(256), 0, st,
                       AttnArgs{c->qkv, c->af_hi, c->af_lo, T, s.n_heads, s.n_kv_heads, s.head_dim});
    linear(LinearArgs{attn[l].wo, c->af_hi, c->af_lo, cur, c->hbuf, s.d, nq, T});
    // MoE half on RMSNorm(h)
    ChainArgs m = base;
    m.KS = 1;
    m.resid_in = c->hbuf;
    m.gamma = attn[l].gamma_moe;
    m.xn_out = c->xn;
    hipLaunchKernelGGL(chain_kernel, dim3(T), dim3(kChainThreads), 0, st, m);
    cur = c->hbuf;
    if (moe_status rc = launch_layer(c, layers + l, c->xn, T, nullptr, nullptr, nullptr, nullptr, nullptr,
                                     n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st, &ks))
      return rc;
  }
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_pack_weights(moe_ctx* c, const moe_layer_weights* src, moe_layer_weights* dst, void* stream) {
  if (!c || !weights_ok(c, src) || src->layout != MOE_LAYOUT_ROW_MAJOR || !dst) return MOE_ERR_INVALID_ARG;
  moe_layer_weights chk = *dst;  // dst's buffers, seen with src's element type and scales
  chk.layout = MOE_LAYOUT_ROW_MAJOR;
  chk.dtype = src->dtype;
  chk.w1_scale = src->w1_scale, chk.w3_scale = src->w3_scale, chk.w2_scale = src->w2_scale;
  chk.sw1_scale = src->sw1_scale, chk.sw3_scale = src->sw3_scale, chk.sw2_scale = src->sw2_scale;
  if (!weights_ok(c, &chk)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  const moe_shape& s = c->s;
  hipStream_t st = (hipStream_t)stream;
  const bool fp8 = src->dtype == MOE_WEIGHT_FP8_E4M3;
  auto pack = [&](const void* a, const void* b, size_t rows, int K) {
    const size_t units = rows * (size_t)(K / (fp8 ? 16 : 8));  // 16-byte units written
    const unsigned blocks = (unsigned)((units + 255) / 256 < 65536 ? (units + 255) / 256 : 65536);
    if (fp8)
      hipLaunchKernelGGL(pack_kernel_fp8, dim3(blocks), dim3(256), 0, st, static_cast<const uint2*>(a),
                         static_cast<uint4*>(const_cast<void*>(b)), rows, K);
    else
      hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const uint4*>(a),
                         static_cast<uint4*>(const_cast<void*>(b)), rows, K);
  };
  if (dst->router_w != src->router_w &&
      hipMemcpyAsync(const_cast<uint16_t*>(dst->router_w), src->router_w, (size_t)s.n_experts * s.d * 2,
                     hipMemcpyDeviceToDevice, st) != hipSuccess)
    return MOE_ERR_HIP;
  pack(src->w1, dst->w1, (size_t)s.n_experts * s.ffn, s.d);
  pack(src->w3, dst->w3, (size_t)s.n_experts * s.ffn, s.d);
  pack(src->w2, dst->w2, (size_t)s.n_experts * s.d, s.ffn);
  if (s.n_shared > 0) {
    pack(src->sw1, dst->sw1, (size_t)s.n_shared * s.ffn, s.d);
    pack(src->sw3, dst->sw3, (size_t)s.n_shared * s.ffn, s.d);
    pack(src->sw2, dst->sw2, (size_t)s.n_shared * s.d, s.ffn);
  }
  dst->layout = MOE_LAYOUT_TILED;
  dst->dtype = src->dtype;
  dst->w1_scale = src->w1_scale, dst->w3_scale = src->w3_scale, dst->w2_scale = src->w2_scale;
  dst->sw1_scale = src->sw1_scale, dst->sw3_scale = src->sw3_scale, dst->sw2_scale = src->sw2_scale;
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_ctx_profile(moe_ctx* c, int32_t enable) {
  if (!c) return MOE_ERR_INVALID_ARG;
  c->profiling = enable != 0;
  return MOE_OK;
}

moe_status moe_ctx_profile_read(moe_ctx* c, double* ms_sum, int64_t* steps) {
  if (!c || !ms_sum || !steps) return MOE_ERR_INVALID_ARG;
  for (int i = 0; i < kProfMarks - 1; ++i) ms_sum[i] = 0.0;
  const size_t n = c->events.size() / kProfMarks;
  moe_status rc = MOE_OK;
  if (n > 0 && hipEventSynchronize(c->events[n * kProfMarks - 1]) != hipSuccess) rc = MOE_ERR_HIP;
  for (size_t i = 0; i < n && rc == MOE_OK; ++i)
    for (int k = 0; k < kProfMarks - 1; ++k) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, c->events[i * kProfMarks + k], c->events[i * kProfMarks + k + 1]) != hipSuccess)
        rc = MOE_ERR_HIP;
      ms_sum[k] += ms;
    }
  for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
  c->events.clear();
  *steps = (int64_t)n;
  return rc;
}

moe_status moe_stream_read_probe(const void* src, int64_t bytes, float* sink, void* stream) {
  if (!src || !sink || bytes < 16 || bytes % 16) return MOE_ERR_INVALID_ARG;
  const size_t n16 = (size_t)(bytes / 16);
  const unsigned blocks = 1024;  // 4096 waves, each streams n16 / 4096 units
  const size_t per_wave = ((n16 + blocks * 4 - 1) / (blocks * 4) + 63) / 64 * 64;
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const uint4*>(src), per_wave, n16, sink);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // extern "C"
