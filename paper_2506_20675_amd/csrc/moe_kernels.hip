// MoE verification path for MI355X (gfx950): hand-written HIP kernels + the device half of the C ABI.
//
// One decode iteration of speculative decoding pushes T = K+1 tokens through each MoE layer
// (paper: Section 2.2); every token picks top_k experts on its own, and the layer's cost is the
// HBM traffic for the UNION of the picked experts (Section 1, Section 2.4).  The path below touches
// every unique expert's weights exactly once per step:
//
//   route_kernel   router logits (fp64 accumulate), top-k, softmax gates; splits the fp32 activations
//                  into bf16 hi + lo fragments for the matrix cores; its last-finishing workgroup
//                  builds the union of experts, the per-expert token lists and the per-slot gate table
//   gateup_kernel  for each unique expert: G = w1 X, U = w3 X, H = gate * silu(G) * U      (2/3 of bytes)
//   down_kernel    split-K partial sums of w2 H over (expert, k-chunk)                     (1/3 of bytes);
//                  the last-finishing workgroup of each row block adds the slabs in a fixed order into
//                  out (gate-weighted combine, deterministic, no floating-point atomics)
//   (group_kernel  the grouping step alone, for callers that bring their own routing)
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

// Hand-off of a few words from one workgroup to another INSIDE a launch (the router's "last workgroup
// builds the expert union" tail).  The words are written and read with relaxed agent-scope atomics,
// which write through / read past the per-XCD caches, so no cache-wide writeback or invalidate is
// needed (a full agent-scope fence costs far more than the data it protects here); the producer only
// has to wait until its stores have been acknowledged before it takes its ticket.
// Producer side: all of this thread's earlier stores are acknowledged, and neither the compiler nor the
// hardware moves later accesses above this point.  Consumer side: the mirror image.
__device__ __forceinline__ void handoff_release() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
}
__device__ __forceinline__ void handoff_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); }

// Activation fragments.  The MFMA B operand of k-step s (32 k) wants, in lane (n = l%16, kg = l/16),
// the 8 values k = 32 s + 8 kg .. +7 of token column n.  Activations are therefore stored in that
// order — unit q = s*64 + kg*16 + n holds those 8 bf16 (16 bytes) — so a wave fetches the whole
// fragment of a k-step with ONE contiguous 1 KB load.  Token columns are padded to 16.
__device__ __forceinline__ size_t frag_unit(int k8, int n) {  // k8 = k / 8
  return (size_t)(k8 >> 2) * 64 + (size_t)(k8 & 3) * 16 + n;
}

__device__ __forceinline__ f32x4 mfma_bf16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                  0, 0);
}

// ------------------------------------------------------------------------------------------
// Step 2: union of activated experts + per-expert token lists.  One workgroup, thread e = expert e.
// ------------------------------------------------------------------------------------------
struct GroupOut {
  int32_t *unique, *n_unique, *count, *offset, *assign;
};
struct GroupArgs {
  const int32_t* ids;   // [T, top_k]
  const float* gates;   // [T, top_k] or NULL (then no gate table is built)
  int T, top_k, E;
  GroupOut ws, user;    // every pointer optional
  int32_t* n_unique_extra;
  int32_t* slot_expert;  // [u_max] expert of unique slot u
  float* slot_gate;      // [u_max, 16] gate of token column n for slot u, 0 = not routed
};

// Executed by one whole 256-thread workgroup.  ids/gates may have been written by other workgroups of
// the same launch: they are read with agent-scope atomic loads, which never hit a stale cache line.
__device__ void group_body(const GroupArgs& g) {
  __shared__ int s_ids[kMaxTokens * kMaxTopK];
  __shared__ int s_cnt[4], s_uni[4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int T = g.T, top_k = g.top_k, E = g.E;
  const GroupOut& ws = g.ws;
  const GroupOut& user = g.user;
  const float* gates = g.gates;
  int32_t* slot_expert = g.slot_expert;
  float* slot_gate = g.slot_gate;
  int32_t* n_unique_extra = g.n_unique_extra;
  const int A = T * top_k;
  if (tid < A) s_ids[tid] = __hip_atomic_load(g.ids + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  const int e = tid;
  int cnt = 0;
  if (e < E)
    for (int a = 0; a < A; ++a) cnt += (s_ids[a] == e);
  const int flag = cnt > 0;
  // inclusive scan of cnt inside the wave, ballot for the unique rank
  int incl = cnt;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  const unsigned long long bal = __ballot(flag);
  const int rank_in_wave = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 63) s_cnt[wave] = incl;
  if (lane == 0) s_uni[wave] = __popcll(bal);
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
  const int off = cbase + incl - cnt;
  const int rank = ubase + rank_in_wave;
  if (e < E) {
    if (ws.count) ws.count[e] = cnt;
    if (ws.offset) ws.offset[e] = off;
    if (user.count) user.count[e] = cnt;
    if (user.offset) user.offset[e] = off;
    if (flag) {
      if (ws.unique) ws.unique[rank] = e;
      if (user.unique) user.unique[rank] = e;
      if (slot_expert) slot_expert[rank] = e;
      float row[kGateCols];
#pragma unroll
      for (int n = 0; n < kGateCols; ++n) row[n] = 0.f;
      int j = 0;
      for (int a = 0; a < A; ++a)
        if (s_ids[a] == e) {
          if (ws.assign) ws.assign[off + j] = a;
          if (user.assign) user.assign[off + j] = a;
          ++j;
          if (gates) {
            const int tok = a / top_k;
            const float gv = __hip_atomic_load(gates + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int n = 0; n < kGateCols; ++n)
              if (n == tok) row[n] = gv;
          }
        }
      if (slot_gate && gates) {
#pragma unroll
        for (int n = 0; n < kGateCols; ++n) slot_gate[rank * kGateCols + n] = row[n];
      }
    }
    if (e >= n_unique) {
      if (ws.unique) ws.unique[e] = -1;
      if (user.unique) user.unique[e] = -1;
    }
  }
  if (tid == 0) {
    if (ws.offset) ws.offset[E] = total;
    if (user.offset) user.offset[E] = total;
    if (ws.n_unique) *ws.n_unique = n_unique;
    if (user.n_unique) *user.n_unique = n_unique;
    if (n_unique_extra) *n_unique_extra = n_unique;
  }
}

__global__ __launch_bounds__(256) void group_kernel(GroupArgs g) { group_body(g); }

// ------------------------------------------------------------------------------------------
// Step 1: router.  One workgroup (4 waves) per token.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ hidden,
                                                    const uint16_t* __restrict__ router_w, int d, int E, int top_k,
                                                    int32_t* __restrict__ ids_ws, float* __restrict__ gates_ws,
                                                    int32_t* __restrict__ ids_out, float* __restrict__ gates_out,
                                                    uint16_t* __restrict__ xs_hi, uint16_t* __restrict__ xs_lo,
                                                    int32_t* __restrict__ ticket, GroupArgs grp) {
  __shared__ double s_logit[kMaxExperts];
  __shared__ float s_sel[kMaxTopK];
  __shared__ int s_id[kMaxTopK];
  __shared__ int s_last;
  const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* x = hidden + (size_t)t * d;

  // activations -> bf16 hi/lo halves in fragment order, consumed by the expert kernels as the MFMA B operand
  for (int k8 = tid; k8 < (d >> 3); k8 += 256) {
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
    reinterpret_cast<uint4*>(xs_hi)[q] = uint4{h[0], h[1], h[2], h[3]};
    reinterpret_cast<uint4*>(xs_lo)[q] = uint4{l[0], l[1], l[2], l[3]};
  }

  // logits in fp64: fp32 x bf16 products are exact in double, so the top-k decision does not
  // depend on the order of summation (beyond ~1e-13 relative)
  for (int e = wave; e < E; e += 4) {
    const uint16_t* w = router_w + (size_t)e * d;
    double acc = 0.0;
    for (int j = lane * 8; j < d; j += 64 * 8) {
      const uint4 wv = *reinterpret_cast<const uint4*>(w + j);
      const float4 x0 = *reinterpret_cast<const float4*>(x + j);
      const float4 x1 = *reinterpret_cast<const float4*>(x + j + 4);
      acc = fma((double)x0.x, (double)bf16_to_f32(wv.x & 0xffffu), acc);
      acc = fma((double)x0.y, (double)bf16_to_f32(wv.x >> 16), acc);
      acc = fma((double)x0.z, (double)bf16_to_f32(wv.y & 0xffffu), acc);
      acc = fma((double)x0.w, (double)bf16_to_f32(wv.y >> 16), acc);
      acc = fma((double)x1.x, (double)bf16_to_f32(wv.z & 0xffffu), acc);
      acc = fma((double)x1.y, (double)bf16_to_f32(wv.z >> 16), acc);
      acc = fma((double)x1.z, (double)bf16_to_f32(wv.w & 0xffffu), acc);
      acc = fma((double)x1.w, (double)bf16_to_f32(wv.w >> 16), acc);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) s_logit[e] = acc;
  }
  __syncthreads();
  if (wave == 0) {
  // top-k by repeated wave-wide arg-max; ties go to the lower expert index
  double v[kMaxExperts / 64];
#pragma unroll
  for (int q = 0; q < kMaxExperts / 64; ++q) {
    const int e = lane + 64 * q;
    double lv = e < E ? s_logit[e] : 0.0;
    if (lv != lv) lv = -INFINITY;  // a NaN logit is never preferred
    v[q] = lv;
  }
  unsigned taken = 0;
  for (int i = 0; i < top_k; ++i) {
    double bv = -INFINITY;
    int be = INT_MAX;
#pragma unroll
    for (int q = 0; q < kMaxExperts / 64; ++q) {
      const int e = lane + 64 * q;
      if (e < E && !((taken >> q) & 1u) && (be == INT_MAX || v[q] > bv)) {
        bv = v[q];
        be = e;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const double ov = __shfl_xor(bv, o);
      const int oe = __shfl_xor(be, o);
      if (ov > bv || (ov == bv && oe < be)) {
        bv = ov;
        be = oe;
      }
    }
    if ((be & 63) == lane) taken |= 1u << (be >> 6);
    if (lane == 0) {
      s_id[i] = be;
      s_sel[i] = (float)bv;
    }
  }
  if (lane == 0) {
    // gates = softmax over the selected logits, summed in slot order
    float p[kMaxTopK];
    const float l0 = s_sel[0];
    float sum = 0.f;
    for (int i = 0; i < top_k; ++i) {
      p[i] = expf(s_sel[i] - l0);
      sum += p[i];
    }
    for (int i = 0; i < top_k; ++i) {
      const float g = p[i] / sum;
      const int a = t * top_k + i;
      __hip_atomic_store(ids_ws + a, s_id[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(gates_ws + a, g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ids_out) ids_out[a] = s_id[i];
      if (gates_out) gates_out[a] = g;
    }
    handoff_release();  // this token's routing is out before the ticket is taken
  }
  }  // wave 0

  // Step 2 rides in the same launch: the workgroup that finishes last sees every token's routing
  // and builds the expert union and the per-slot tables (fixed order -> deterministic).
  __syncthreads();
  if (tid == 0)
    s_last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1;
  __syncthreads();
  if (!s_last) return;
  handoff_acquire();
  group_body(grp);
  if (tid == 0) *ticket = 0;  // ready for the next launch on this stream
}

// ------------------------------------------------------------------------------------------
// Shared software pipeline of the two expert kernels.
//   NA  A tiles (16 rows x 32 k) consumed per k-step, each with its own wave-uniform base pointer
//   P   pipeline depth (k-steps of loads in flight per wave)
// A stage holds one 128-bit load per tile plus the hi and lo activation fragments.
// ------------------------------------------------------------------------------------------
template <int NA>
struct Stage {
  uint4 a[NA];
  uint4 bh, bl;
};

template <int NA, int P, class Load, class Compute>
__device__ __forceinline__ void pipeline(int nst, Load load, Compute compute) {
  Stage<NA> st[P];
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
// Weight addressing.  A k-step of a 16-row tile is 16 rows x 32 k = 1 KB of bf16.
//   row-major [rows, K]:  lane (r, kg) reads 16 B at row tile*16 + r, k = 32 s + 8 kg
//   tiled              :  the same 1 KB stored contiguously, block index tile*(K/32) + s, lane l at
//                         byte 16 l — what moe_pack_weights produces; one wave load = 1 KB contiguous
// ------------------------------------------------------------------------------------------
template <bool TILED>
struct WeightAddr {
  uint32_t lane_off, step_stride;
  size_t tile_stride;
  __device__ __forceinline__ WeightAddr(int K, int r, int kg, int lane) {
    if constexpr (TILED) {
      lane_off = lane * 16;
      step_stride = 1024;
      tile_stride = (size_t)(K >> 5) * 1024;
    } else {
      lane_off = ((uint32_t)r * K + kg * 8) * 2;
      step_stride = 64;
      tile_stride = (size_t)16 * K * 2;
    }
  }
};

// ------------------------------------------------------------------------------------------
// Step 3: gate/up projections + SiLU*mul for every unique expert (and shared expert).
// grid = (row blocks of 16*R rows of ffn, expert slots); block = W waves that split d.
// ------------------------------------------------------------------------------------------
struct GateupArgs {
  const uint16_t *w1, *w3, *sw1, *sw3;  // [E,ffn,d] / [n_shared,ffn,d]
  const uint16_t *xf_hi, *xf_lo;        // activation fragments, d*16 elements each
  const int32_t* n_unique;
  const int32_t* slot_expert;  // [u_max]
  const float* slot_gate;      // [u_tot,16]
  uint16_t *hf_hi, *hf_lo;     // [u_tot] fragments of gate*silu(G)*U, ffn*16 elements each
  int d, ffn, T, u_max;
};

template <int R, int W, int P, bool TILED, bool NT>
__global__ __launch_bounds__(64 * W) void gateup_kernel(GateupArgs g) {
  __shared__ float4 red[W > 1 ? W * 2 * R * 64 : 1];
  const int u = blockIdx.y;
  const char *W1, *W3;
  const size_t per = (size_t)g.ffn * g.d * 2;
  if (u < g.u_max) {
    if (u >= *g.n_unique) return;
    const int e = g.slot_expert[u];
    W1 = reinterpret_cast<const char*>(g.w1) + e * per;
    W3 = reinterpret_cast<const char*>(g.w3) + e * per;
  } else {
    W1 = reinterpret_cast<const char*>(g.sw1) + (u - g.u_max) * per;
    W3 = reinterpret_cast<const char*>(g.sw3) + (u - g.u_max) * per;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const int ntiles = g.ffn >> 4, tile0 = blockIdx.x * R;
  const int nsteps = g.d >> 5, chunk = (nsteps + W - 1) / W;
  const int nst = max(0, min(chunk, nsteps - wave * chunk));
  const int s_beg = min(wave * chunk, nsteps - 1);  // a wave without work still issues in-bounds loads

  const WeightAddr<TILED> wa(g.d, r, kg, lane);
  const char* base[2 * R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const size_t t = (size_t)min(tile0 + j, ntiles - 1);  // ragged last block: re-read a valid tile, result unused
    base[j] = W1 + t * wa.tile_stride + (size_t)s_beg * wa.step_stride;
    base[R + j] = W3 + t * wa.tile_stride + (size_t)s_beg * wa.step_stride;
  }
  const char* XH = reinterpret_cast<const char*>(g.xf_hi) + (size_t)s_beg * 1024;
  const char* XL = reinterpret_cast<const char*>(g.xf_lo) + (size_t)s_beg * 1024;
  const uint32_t b_off = lane * 16;

  f32x4 acc[2 * R];
#pragma unroll
  for (int j = 0; j < 2 * R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<2 * R, P>(
      nst,
      [&](Stage<2 * R>& st, int s) {
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) st.a[j] = ld128<NT>(base[j], wa.lane_off + (uint32_t)s * wa.step_stride);
#ifdef MOE_EXPERIMENT_NO_B
        st.bh = ld128<false>(XH, b_off);
        st.bl = ld128<false>(XL, b_off);
#else
        st.bh = ld128<false>(XH, b_off + (uint32_t)s * 1024);
        st.bl = ld128<false>(XL, b_off + (uint32_t)s * 1024);
#endif
      },
      [&](const Stage<2 * R>& st) {
#ifdef MOE_EXPERIMENT_NO_MFMA
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) {
          acc[j][0] += __uint_as_float((st.a[j].x ^ st.bh.x) & 0x3fffffffu);
          acc[j][1] += __uint_as_float((st.a[j].y ^ st.bl.y) & 0x3fffffffu);
          acc[j][2] += __uint_as_float((st.a[j].z ^ st.bh.z) & 0x3fffffffu);
          acc[j][3] += __uint_as_float((st.a[j].w ^ st.bl.w) & 0x3fffffffu);
        }
#else
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) acc[j] = mfma_bf16(st.a[j], st.bh, acc[j]);
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) acc[j] = mfma_bf16(st.a[j], st.bl, acc[j]);
#endif
      });

  // reduce the W k-slices through LDS, then wave w finishes tiles w, w+W, ...
  if constexpr (W > 1) {
#pragma unroll
    for (int j = 0; j < 2 * R; ++j)
      red[(wave * 2 * R + j) * 64 + lane] = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
    __syncthreads();
  }
  const float gate = g.slot_gate[u * kGateCols + r];
  uint16_t* HH = g.hf_hi + (size_t)u * g.ffn * 16;
  uint16_t* HL = g.hf_lo + (size_t)u * g.ffn * 16;
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
    if (r < g.T && gate != 0.f) {
      // lane holds rows 4*kg .. 4*kg+3 of the tile for token column r: four consecutive k of the
      // down projection, i.e. one half of a 16-byte fragment unit
      uint16_t hi[4], lo[4];
      split_bf16(gate * (G.x / (1.f + expf(-G.x))) * U.x, hi[0], lo[0]);
      split_bf16(gate * (G.y / (1.f + expf(-G.y))) * U.y, hi[1], lo[1]);
      split_bf16(gate * (G.z / (1.f + expf(-G.z))) * U.z, hi[2], lo[2]);
      split_bf16(gate * (G.w / (1.f + expf(-G.w))) * U.w, hi[3], lo[3]);
      const int k = (tile0 + j) * 16 + kg * 4;
      const size_t o = frag_unit(k >> 3, r) * 8 + (k & 4);
      *reinterpret_cast<uint2*>(HH + o) = uint2{(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
      *reinterpret_cast<uint2*>(HL + o) = uint2{(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 4: down projection, split-K over (expert slot, k-chunk).  The gate is already folded into H,
// so every slab is a plain partial sum of out.
// grid = (row blocks of 16*R rows of d, expert slots, KS k-chunks); block = W waves splitting the chunk.
// ------------------------------------------------------------------------------------------
struct DownArgs {
  const uint16_t *w2, *sw2;      // [E,d,ffn] / [n_shared,d,ffn]
  const uint16_t *hf_hi, *hf_lo; // [u_tot] fragments, ffn*16 elements each
  const int32_t* n_unique;
  const int32_t* slot_expert;
  const float* slot_gate;
  float* partial;                // [u_tot*KS, max_tokens, d]
  int d, ffn, T, u_max, max_tokens, KS;
};

template <int R, int W, int P, bool TILED, bool NT>
__global__ __launch_bounds__(64 * W) void down_kernel(DownArgs g) {
  __shared__ float4 red[W > 1 ? W * R * 64 : 1];
  const int u = blockIdx.y, ks = blockIdx.z;
  const char* W2;
  const size_t per = (size_t)g.ffn * g.d * 2;
  if (u < g.u_max) {
    if (u >= *g.n_unique) return;
    W2 = reinterpret_cast<const char*>(g.w2) + g.slot_expert[u] * per;
  } else {
    W2 = reinterpret_cast<const char*>(g.sw2) + (u - g.u_max) * per;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const int ntiles = g.d >> 4, tile0 = blockIdx.x * R;
  const int nsteps = g.ffn >> 5, parts = g.KS * W, chunk = (nsteps + parts - 1) / parts;
  const int nst = max(0, min(chunk, nsteps - (ks * W + wave) * chunk));
  const int s_beg = min((ks * W + wave) * chunk, nsteps - 1);  // a wave without work still issues in-bounds loads

  const WeightAddr<TILED> wa(g.ffn, r, kg, lane);
  const char* base[R];
#pragma unroll
  for (int j = 0; j < R; ++j)
    base[j] = W2 + (size_t)min(tile0 + j, ntiles - 1) * wa.tile_stride + (size_t)s_beg * wa.step_stride;
  // token column r contributes only if the token is routed to this expert (gate != 0)
  const bool live = r < g.T && g.slot_gate[u * kGateCols + r] != 0.f;
  const char* HH = reinterpret_cast<const char*>(g.hf_hi) + ((size_t)u * g.ffn * 16 + (size_t)s_beg * 512) * 2;
  const char* HL = reinterpret_cast<const char*>(g.hf_lo) + ((size_t)u * g.ffn * 16 + (size_t)s_beg * 512) * 2;
  const uint32_t b_off = lane * 16;

  f32x4 acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<R, P>(
      nst,
      [&](Stage<R>& st, int s) {
#pragma unroll
        for (int j = 0; j < R; ++j) st.a[j] = ld128<NT>(base[j], wa.lane_off + (uint32_t)s * wa.step_stride);
        st.bh = uint4{0u, 0u, 0u, 0u};
        st.bl = uint4{0u, 0u, 0u, 0u};
        if (live) {
          st.bh = ld128<false>(HH, b_off + (uint32_t)s * 1024);
          st.bl = ld128<false>(HL, b_off + (uint32_t)s * 1024);
        }
      },
      [&](const Stage<R>& st) {
#pragma unroll
        for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], st.bh, acc[j]);
#pragma unroll
        for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], st.bl, acc[j]);
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
    if (r < g.T) {
      const size_t o = (((size_t)u * g.KS + ks) * g.max_tokens + r) * g.d + (size_t)(tile0 + j) * 16 + kg * 4;
      *reinterpret_cast<float4*>(g.partial + o) = y;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 5 (after the split-K down kernel): out[t,c] = sum over live slabs, routed slots ascending then
// shared experts, k-chunks ascending — a fixed order, so reruns are bit-identical.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ partial,
                                                      const int32_t* __restrict__ n_unique_p, float* __restrict__ out,
                                                      int d, int T, int u_max, int n_shared, int max_tokens, int KS) {
  const int i = blockIdx.x * 256 + threadIdx.x;  // float4 index inside [T, d]
  const int per_tok = d >> 2;
  if (i >= T * per_tok) return;
  const int t = i / per_tok, c4 = i - t * per_tok;
  const int n_unique = *n_unique_p;
  float4 s = float4{0.f, 0.f, 0.f, 0.f};
  const size_t slab = (size_t)max_tokens * d;
  const float* p0 = partial + (size_t)t * d + (size_t)c4 * 4;
  for (int u = 0; u < n_unique; ++u)
    for (int k = 0; k < KS; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(p0 + ((size_t)u * KS + k) * slab);
      s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
    }
  for (int u = u_max; u < u_max + n_shared; ++u)
    for (int k = 0; k < KS; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(p0 + ((size_t)u * KS + k) * slab);
      s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
    }
  *reinterpret_cast<float4*>(out + (size_t)t * d + (size_t)c4 * 4) = s;
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

// ------------------------------------------------------------------------------------------
// Measurement aid: plain coalesced read stream.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          float* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], e = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ e.x ^ e.y ^ e.z ^ e.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if ((threadIdx.x & 63) == 0) atomicXor(reinterpret_cast<unsigned int*>(sink) + (blockIdx.x & 4095), acc);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

// ------------------------------------------------------------------------------------------
// Host side of the device ABI
// ------------------------------------------------------------------------------------------
struct moe_ctx {
  moe_shape s;
  int device;
  int u_max, u_tot;
  int ks_alloc;           // split-K slabs the partial buffer is sized for
  int plan_override[3];   // MOE_PLAN=guR,dnR,dnKS (tuning), zeros = automatic
  char* ws;
  size_t ws_bytes;
  uint16_t *xf_hi, *xf_lo, *hf_hi, *hf_lo;  // activation fragments (see frag_unit)
  int32_t *ids, *unique, *n_unique, *count, *offset, *assign, *slot_expert;
  float *gates, *slot_gate, *partial;
  int32_t* route_ticket;  // arrival counter of the router's fused grouping tail, zero between launches
  bool profiling;
  std::vector<hipEvent_t> events;  // kProfMarks per profiled layer-step
};

namespace {

constexpr int kProfMarks = 5;  // events per profiled layer-step: route+group, gate/up, down, combine
constexpr int kWaves = 4;    // waves per workgroup in the expert kernels (they split K)
constexpr int kMaxKS = 16;   // largest split-K factor of the down projection

// Launch plan of the two expert kernels for one (T, weight layout).
//   gu_R, dn_R  weight tiles (16 rows) per wave; the pipeline depth is tied to it (fewer tiles ->
//               deeper pipeline, same bytes in flight per wave)
//   dn_KS       split-K factor of the down projection across workgroups
// Chosen from measurements on Mixtral-shaped layers: tiled weights stream best with one tile per wave
// and 8 k-steps in flight; the down projection wants about 4-5 thousand waves in the grid.
struct Plan {
  int gu_R, dn_R, dn_KS;
};

int ks_cap_for(const moe_shape& s) {
  const int nsteps = s.ffn / 32;
  int cap = 1;
  while (cap < kMaxKS && nsteps / (kWaves * cap * 2) >= 4) cap *= 2;  // every wave keeps >= 4 k-steps
  return cap;
}

Plan plan_for(const moe_ctx* c, int T, bool tiled) {
  const moe_shape& s = c->s;
  // expected number of live expert slots for T tokens under uniform routing (balls into bins)
  double miss = 1.0;
  for (int t = 0; t < T; ++t) miss *= 1.0 - (double)s.top_k / s.n_experts;
  const double slots = s.n_experts * (1.0 - miss) + s.n_shared;
  Plan p;
  p.gu_R = tiled ? 1 : ((s.ffn / 16 / 2) * kWaves * slots >= 1536 ? 2 : 1);
  const int cap = ks_cap_for(s);
  p.dn_R = 1;
  p.dn_KS = cap;
  for (int R : {4, 2, 1}) {
    const double per_ks = (double)((s.d / 16 + R - 1) / R) * kWaves * slots;
    int ks = 1;
    while (ks < cap && per_ks * ks < 3584) ks *= 2;
    if (per_ks * ks >= 3072 || R == 1) {
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

moe_status launch_route_group(moe_ctx* c, const float* hidden, const uint16_t* router_w, int T, int32_t* ids,
                              float* gates, int32_t* unique, int32_t* n_unique, int32_t* n_unique_extra,
                              hipStream_t st) {
  const moe_shape& s = c->s;
  GroupArgs ga{c->ids, c->gates, T, s.top_k, s.n_experts,
               GroupOut{c->unique, c->n_unique, c->count, c->offset, c->assign},
               GroupOut{unique, n_unique, nullptr, nullptr, nullptr}, n_unique_extra, c->slot_expert, c->slot_gate};
  mark(c, st);
  hipLaunchKernelGGL(route_kernel, dim3(T), dim3(256), 0, st, hidden, router_w, s.d, s.n_experts, s.top_k, c->ids,
                     c->gates, ids, gates, c->xf_hi, c->xf_lo, c->route_ticket, ga);
  mark(c, st);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Tiled weights are read exactly once in contiguous 1 KB pieces -> streaming loads; row-major weights
// are read in 64-byte row segments whose cache lines are completed by the next k-step -> cached loads.
template <int R, int P>
void launch_gateup(const moe_ctx* c, const GateupArgs& a, bool tiled, hipStream_t st) {
  const dim3 grid((c->s.ffn / 16 + R - 1) / R, c->u_tot);
  if (tiled)
    hipLaunchKernelGGL((gateup_kernel<R, kWaves, P, true, true>), grid, dim3(64 * kWaves), 0, st, a);
  else
    hipLaunchKernelGGL((gateup_kernel<R, kWaves, P, false, false>), grid, dim3(64 * kWaves), 0, st, a);
}
template <int R, int P>
void launch_down(const moe_ctx* c, const DownArgs& a, bool tiled, hipStream_t st) {
  const dim3 grid((c->s.d / 16 + R - 1) / R, c->u_tot, a.KS);
  if (tiled)
    hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true>), grid, dim3(64 * kWaves), 0, st, a);
  else
    hipLaunchKernelGGL((down_kernel<R, kWaves, P, false, false>), grid, dim3(64 * kWaves), 0, st, a);
}

moe_status launch_experts(moe_ctx* c, const moe_layer_weights* w, int T, float* out, hipStream_t st) {
  const moe_shape& s = c->s;
  const bool tiled = w->layout == MOE_LAYOUT_TILED;
  const Plan p = plan_for(c, T, tiled);
  GateupArgs ga{w->w1, w->w3, w->sw1, w->sw3, c->xf_hi, c->xf_lo, c->n_unique, c->slot_expert, c->slot_gate,
                c->hf_hi, c->hf_lo, s.d, s.ffn, T, c->u_max};
  switch (p.gu_R) {
    case 4: launch_gateup<4, 2>(c, ga, tiled, st); break;
    case 2: launch_gateup<2, 4>(c, ga, tiled, st); break;
    default: launch_gateup<1, 8>(c, ga, tiled, st); break;
  }
  mark(c, st);
  DownArgs da{w->w2, w->sw2, c->hf_hi, c->hf_lo, c->n_unique, c->slot_expert, c->slot_gate, c->partial,
              s.d, s.ffn, T, c->u_max, s.max_tokens, p.dn_KS};
  switch (p.dn_R) {
    case 4: launch_down<4, 3>(c, da, tiled, st); break;
    case 2: launch_down<2, 4>(c, da, tiled, st); break;
    default: launch_down<1, 8>(c, da, tiled, st); break;
  }
  mark(c, st);
  const int n4 = T * (s.d / 4);
  hipLaunchKernelGGL(combine_kernel, dim3((n4 + 255) / 256), dim3(256), 0, st, (const float*)c->partial,
                     (const int32_t*)c->n_unique, out, s.d, T, c->u_max, s.n_shared, s.max_tokens, p.dn_KS);
  mark(c, st);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// kernels use 128-bit loads: every tensor base must be 16-byte aligned (rows are, since d, ffn % 32 == 0)
bool weights_ok(const moe_ctx* c, const moe_layer_weights* w) {
  if (!w || !w->router_w || !w->w1 || !w->w3 || !w->w2) return false;
  if (w->layout != MOE_LAYOUT_ROW_MAJOR && w->layout != MOE_LAYOUT_TILED) return false;
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

int moe_abi_version(void) { return 1; }

moe_status moe_ctx_create(const moe_shape* shape, moe_ctx** out) {
  if (out) *out = nullptr;
  if (!shape || !out) return MOE_ERR_INVALID_ARG;
  const moe_shape s = *shape;
  if (s.d < 32 || s.ffn < 32 || s.n_experts < 1 || s.top_k < 1 || s.n_shared < 0 || s.max_tokens < 1)
    return MOE_ERR_INVALID_ARG;
  if (s.top_k > s.n_experts) return MOE_ERR_INVALID_ARG;
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
  c->u_tot = c->u_max + s.n_shared;
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
  c->ks_alloc = ks_cap_for(s);

  const size_t A = (size_t)s.max_tokens * s.top_k;
  size_t off = 0;
  auto carve = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const size_t o_xh = carve((size_t)s.d * kGateCols * 2), o_xl = carve((size_t)s.d * kGateCols * 2);
  const size_t o_hh = carve((size_t)c->u_tot * s.ffn * kGateCols * 2);
  const size_t o_hl = carve((size_t)c->u_tot * s.ffn * kGateCols * 2);
  const size_t o_ids = carve(A * 4), o_gates = carve(A * 4), o_uni = carve((size_t)s.n_experts * 4);
  const size_t o_nu = carve(4), o_cnt = carve((size_t)s.n_experts * 4), o_off = carve((size_t)(s.n_experts + 1) * 4);
  const size_t o_asg = carve(A * 4), o_se = carve((size_t)c->u_max * 4);
  const size_t o_sg = carve((size_t)c->u_tot * kGateCols * 4);
  const size_t o_tk = carve(4);
  const size_t o_part = carve((size_t)c->u_tot * c->ks_alloc * s.max_tokens * s.d * 4);
  c->ws_bytes = off;
  if (hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes) != hipSuccess) {
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
  c->unique = reinterpret_cast<int32_t*>(c->ws + o_uni);
  c->n_unique = reinterpret_cast<int32_t*>(c->ws + o_nu);
  c->count = reinterpret_cast<int32_t*>(c->ws + o_cnt);
  c->offset = reinterpret_cast<int32_t*>(c->ws + o_off);
  c->assign = reinterpret_cast<int32_t*>(c->ws + o_asg);
  c->slot_expert = reinterpret_cast<int32_t*>(c->ws + o_se);
  c->slot_gate = reinterpret_cast<float*>(c->ws + o_sg);
  c->partial = reinterpret_cast<float*>(c->ws + o_part);
  c->route_ticket = reinterpret_cast<int32_t*>(c->ws + o_tk);
  // small tables start at zero; shared-expert slots carry gate 1 for every token column
  bool ok = hipMemset(c->ws, 0, c->ws_bytes) == hipSuccess;
  if (ok && s.n_shared > 0) {
    float ones[kMaxShared * kGateCols];
    for (int i = 0; i < s.n_shared * kGateCols; ++i) ones[i] = 1.f;
    ok = hipMemcpy(c->slot_gate + (size_t)c->u_max * kGateCols, ones, sizeof(float) * s.n_shared * kGateCols,
                   hipMemcpyHostToDevice) == hipSuccess;
  }
  if (!ok) {
    (void)hipFree(c->ws);
    delete c;
    return MOE_ERR_HIP;
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
  return launch_route_group(c, hidden, router_w, T, ids, gates, unique_experts, n_unique, nullptr,
                            (hipStream_t)stream);
}

moe_status moe_group(moe_ctx* c, const int32_t* ids, int32_t T, int32_t* unique_experts, int32_t* n_unique,
                     int32_t* expert_count, int32_t* expert_offset, int32_t* assign, void* stream) {
  if (!c || !ids || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  GroupArgs ga{ids, nullptr, T, c->s.top_k, c->s.n_experts, GroupOut{nullptr, nullptr, nullptr, nullptr, nullptr},
               GroupOut{unique_experts, n_unique, expert_count, expert_offset, assign}, nullptr, nullptr, nullptr};
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
  if (moe_status rc = launch_route_group(c, hidden, w->router_w, T, ids_opt, gates_opt, unique_opt, n_unique_opt,
                                         nullptr, st))
    return rc;
  return launch_experts(c, w, T, out, st);
}

moe_status moe_verify_stack(moe_ctx* c, const moe_layer_weights* layers, int32_t L, const float* hidden, int32_t T,
                            float* out, int32_t* n_unique_per_layer_opt, void* stream) {
  if (!c || !layers || L < 1 || !hidden || !out || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(out)) return MOE_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l)
    if (!weights_ok(c, layers + l)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  hipStream_t st = (hipStream_t)stream;
  const size_t per = (size_t)T * c->s.d;
  for (int l = 0; l < L; ++l) {
    if (moe_status rc = launch_route_group(c, hidden + l * per, layers[l].router_w, T, nullptr, nullptr, nullptr,
                                           nullptr, n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st))
      return rc;
    if (moe_status rc = launch_experts(c, layers + l, T, out + l * per, st)) return rc;
  }
  return MOE_OK;
}

moe_status moe_pack_weights(moe_ctx* c, const moe_layer_weights* src, moe_layer_weights* dst, void* stream) {
  if (!c || !weights_ok(c, src) || src->layout != MOE_LAYOUT_ROW_MAJOR || !dst) return MOE_ERR_INVALID_ARG;
  moe_layer_weights chk = *dst;
  chk.layout = MOE_LAYOUT_ROW_MAJOR;
  if (!weights_ok(c, &chk)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c)) return st;
  const moe_shape& s = c->s;
  hipStream_t st = (hipStream_t)stream;
  auto pack = [&](const uint16_t* a, uint16_t* b, size_t rows, int K) {
    const size_t units = rows * (size_t)(K / 8);
    const unsigned blocks = (unsigned)((units + 255) / 256 < 65536 ? (units + 255) / 256 : 65536);
    hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<const uint4*>(a),
                       reinterpret_cast<uint4*>(b), rows, K);
  };
  if (dst->router_w != src->router_w &&
      hipMemcpyAsync(const_cast<uint16_t*>(dst->router_w), src->router_w, (size_t)s.n_experts * s.d * 2,
                     hipMemcpyDeviceToDevice, st) != hipSuccess)
    return MOE_ERR_HIP;
  pack(src->w1, const_cast<uint16_t*>(dst->w1), (size_t)s.n_experts * s.ffn, s.d);
  pack(src->w3, const_cast<uint16_t*>(dst->w3), (size_t)s.n_experts * s.ffn, s.d);
  pack(src->w2, const_cast<uint16_t*>(dst->w2), (size_t)s.n_experts * s.d, s.ffn);
  if (s.n_shared > 0) {
    pack(src->sw1, const_cast<uint16_t*>(dst->sw1), (size_t)s.n_shared * s.ffn, s.d);
    pack(src->sw3, const_cast<uint16_t*>(dst->sw3), (size_t)s.n_shared * s.ffn, s.d);
    pack(src->sw2, const_cast<uint16_t*>(dst->sw2), (size_t)s.n_shared * s.d, s.ffn);
  }
  dst->layout = MOE_LAYOUT_TILED;
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
  hipLaunchKernelGGL(stream_read_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const uint4*>(src), (size_t)(bytes / 16), sink);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // extern "C"
