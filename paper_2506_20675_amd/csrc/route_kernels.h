// Steps 1 and 2 of the MoE verification path: router (logits, top-k, gates, activation fragments) and the
// expert-union grouping.  Part of the single translation unit moe_kernels.hip.
#pragma once
#include "moe_common.h"

namespace {

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
  int32_t* slot_mask;                                       // [u_max] bit t set: token t is routed to the slot
  float* slot_gate;                                         // [u_max, 16] its gate there (may be 0: see slot_mask)
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
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
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
      if (g.slot_mask) g.slot_mask[rank] = (int32_t)m;  // routed-ness is kept apart from the gate: a gate can underflow to 0
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

// The same tables for a SINGLE token (decoding without speculation, T = 1), where the union is the token's own picks:
// the slot of pick i is the number of picks with a smaller expert id.  No masks to merge, no scans, one barrier —
// this runs at the tail of the router's only workgroup, on the critical path of every non-speculative step.
// s_ids / s_gates: the top_k picks in LDS, written before the call (the call begins with a barrier).
__device__ __forceinline__ void group_single_token(const GroupArgs& g, const int* s_ids, const float* s_gates) {
  __syncthreads();
  const int tid = threadIdx.x, k = g.top_k;
  if (tid < k) {
    const int id = s_ids[tid];
    int slot = 0;
    for (int j = 0; j < k; ++j) slot += s_ids[j] < id ? 1 : 0;  // the picks of one token are distinct
    if (g.unique) g.unique[slot] = id;
    if (g.slot_expert) g.slot_expert[slot] = id;
    if (g.slot_mask) g.slot_mask[slot] = 1;  // token 0 is routed to every slot of the union
    if (g.tok_slot) g.tok_slot[tid] = slot;
    if (g.slot_gate && s_gates) g.slot_gate[slot * kGateCols] = s_gates[tid];
  }
  if (g.unique)
    for (int e = k + tid; e < g.E; e += blockDim.x) g.unique[e] = -1;
  if (tid == 0) {
    if (g.n_unique) *g.n_unique = k;
    if (g.n_unique_ws) *g.n_unique_ws = k;
    if (g.n_unique_extra) *g.n_unique_extra = k;
  }
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
                                           int E, int lane, int chunk, int e0, double* s_acc, int acc_base = 0) {
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
  if ((lane & 7) == 0 && e0 + idx < E) s_acc[e0 + idx - acc_base] += u1;  // s_acc[0] belongs to expert acc_base
}

// Ragged tail of d (a multiple of 32 elements past the last whole 512-element chunk) for experts e_lo .. e_hi-1:
// the wave's lanes walk it 8 elements at a time; one 6-step butterfly per expert.
__device__ __forceinline__ void route_tail(const float* __restrict__ x, const uint16_t* __restrict__ router_w, int d,
                                           int lane, int e_lo, int e_hi, double* s_acc) {
  for (int e = e_lo; e < e_hi; ++e) {
    double a = 0.0;
    for (int j = ((d >> 9) << 9) + lane * 8; j < d; j += 512) {
      const uint4 w = *reinterpret_cast<const uint4*>(router_w + (size_t)e * d + j);
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
    if (lane == 0) s_acc[e - e_lo] += a;
  }
}

// One workgroup (16 waves) per token.  The (chunk of d, batch of 8 experts) work items are dealt
// round-robin to the waves; partial logits meet in LDS and are summed in wave order.  Top-k by rank
// counting: thread e counts the logits that beat its own (larger, or equal with a lower index), the
// expert of rank i < top_k is pick i — no serial arg-max rounds.  Gates = softmax over the picked
// logits in fp32, summed in pick order.  With a single token in flight (T = 1, no speculation) this
// workgroup already sees the whole routing, so the expert-union step runs right here; with more
// tokens it needs the launch of its own that follows (group_kernel).
__device__ __forceinline__ void route_body(const RouteArgs& g, const GroupArgs& grp) {
  __shared__ double s_part[kRouteWaves][kMaxExperts];
  __shared__ double s_logit[kMaxExperts];
  __shared__ int s_ids[kMaxTopK];
  __shared__ float s_sel[kMaxTopK];
  __shared__ float s_gates[kMaxTopK];
  __shared__ float s_prob[kMaxExperts];
  const int t = blockIdx.x, tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int E = g.E, top_k = g.top_k;
  const float* x = g.hidden + (size_t)t * g.d;
  const int n_batches = (E + kRouteBatch - 1) / kRouteBatch;
  const int n_full = g.d >> 9;  // whole 512-element chunks
  const int n_items = n_full * n_batches;
  for (int e = lane; e < E; e += 64) s_part[wave][e] = 0.0;  // the wave's own row: no barrier needed
  for (int it = wave; it < n_items; it += kRouteWaves)
    route_item(x, g.router_w, g.d, E, lane, it / n_batches, (it % n_batches) * kRouteBatch, s_part[wave]);
  if ((g.d & 511) && wave == kRouteWaves - 1) route_tail(x, g.router_w, g.d, lane, 0, E, s_part[wave]);
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
#pragma unroll 8
    for (int j = 0; j < E; ++j) {  // unrolled: eight independent LDS reads in flight instead of one
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
  if (gridDim.x == 1) group_single_token(grp, s_ids, s_gates);  // one workgroup per token: a grid of one is T = 1
}

__global__ __launch_bounds__(64 * kRouteWaves) void route_kernel(RouteArgs g, GroupArgs grp) { route_body(g, grp); }

// ------------------------------------------------------------------------------------------
// Wide routers (many experts).  One workgroup per token cannot do E * d fp64 multiply-adds on the router weights
// fast enough (one compute unit: ~10 us at E = 64, d = 2048).  So the work is cut the other way:
//   logits_kernel      grid (T, E / 16): one workgroup per (token, 16 experts) -> fp64 logits in HBM, and the
//                      workgroups of the first expert block write the activation fragments;
//   topk_group_kernel  one workgroup: top-k by rank counting and gates for all T tokens, then the expert-union step.
// Same arithmetic, same orders of summation per logit as route_kernel up to the split of d over 8 instead of 16 waves.
// ------------------------------------------------------------------------------------------
constexpr int kLogitWaves = 8;
constexpr int kLogitExperts = 16;

// WAVES: wavefronts of the workgroup.  x_row != NULL: token t's input row is there (possibly in LDS) and not at
// g.hidden.
template <int WAVES>
__device__ __forceinline__ void logits_body(const RouteArgs& g, double* __restrict__ logits,
                                            const float* x_row = nullptr) {
  constexpr int kLogitWaves = WAVES;  // shadows the namespace constant inside this body
  __shared__ double s_part[kLogitWaves][kLogitExperts];
  const int t = blockIdx.x, e_lo = blockIdx.y * kLogitExperts, tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int nE = min(kLogitExperts, g.E - e_lo);
  const float* x = x_row ? x_row : g.hidden + (size_t)t * g.d;
  const int n_batches = (nE + kRouteBatch - 1) / kRouteBatch;
  const int n_items = (g.d >> 9) * n_batches;
  if (lane < kLogitExperts) s_part[wave][lane] = 0.0;
  for (int it = wave; it < n_items; it += kLogitWaves)
    route_item(x, g.router_w, g.d, g.E, lane, it / n_batches, e_lo + (it % n_batches) * kRouteBatch, s_part[wave], e_lo);
  if ((g.d & 511) && wave == kLogitWaves - 1) route_tail(x, g.router_w, g.d, lane, e_lo, e_lo + nE, s_part[wave]);
  if (blockIdx.y == 0) split_token(x, g.d, t, tid, 64 * kLogitWaves, g.xf_hi, g.xf_lo, g.T <= kPackedTokens);
  __syncthreads();
  if (tid < nE) {
    double l = 0.0;
#pragma unroll
    for (int w = 0; w < kLogitWaves; ++w) l += s_part[w][tid];
    if (l != l) l = -INFINITY;  // a NaN logit is never preferred
    logits[(size_t)t * g.E + e_lo + tid] = l;
  }
}

__global__ __launch_bounds__(64 * kLogitWaves) void logits_kernel(RouteArgs g, double* __restrict__ logits) {
  logits_body<kLogitWaves>(g, logits);
}

__device__ __forceinline__ void topk_group_body(const RouteArgs& g, const GroupArgs& grp,
                                                const double* __restrict__ logits) {
  __shared__ double s_logit[kMaxTokens * kMaxExperts];
  __shared__ int s_ids[kMaxTokens * kMaxTopK];
  __shared__ float s_sel[kMaxTokens * kMaxTopK];
  __shared__ float s_gates[kMaxTokens * kMaxTopK];
  const int tid = threadIdx.x, E = g.E, top_k = g.top_k, T = g.T;
  for (int i = tid; i < T * E; i += 1024) s_logit[i] = logits[i];
  __syncthreads();
  for (int i = tid; i < T * E; i += 1024) {  // pair (token, expert): the expert's rank among the token's logits
    const int t = i / E, e = i - t * E;
    const double* row = s_logit + t * E;
    const double mine = row[e];
    int rank = 0;
#pragma unroll 8
    for (int j = 0; j < E; ++j) {
      const double o = row[j];
      rank += (o > mine || (o == mine && j < e)) ? 1 : 0;
    }
    if (rank < top_k) {
      s_ids[t * top_k + rank] = e;
      s_sel[t * top_k + rank] = (float)mine;
    }
  }
  __syncthreads();
  if (tid < T * top_k) {  // pair (token, pick): its gate, by the same sums in the same order as route_kernel
    const int t = tid / top_k;
    const float l0 = s_sel[t * top_k];
    float sum = 0.f;
    if (g.gate_mode == MOE_GATE_SOFTMAX_ALL)
      for (int e = 0; e < E; ++e) sum += expf((float)s_logit[t * E + e] - l0);
    else
      for (int i = 0; i < top_k; ++i) sum += expf(s_sel[t * top_k + i] - l0);
    const float gate = expf(s_sel[tid] - l0) / sum;
    const int id = s_ids[tid];
    g.ids_ws[tid] = id;
    g.gates_ws[tid] = gate;
    if (g.ids_out) g.ids_out[tid] = id;
    if (g.gates_out) g.gates_out[tid] = gate;
    s_gates[tid] = gate;
  }
  if (T == 1)
    group_single_token(grp, s_ids, s_gates);
  else
    group_body(grp, s_ids, s_gates);  // begins with a barrier: the picks are in LDS by then
}

__global__ __launch_bounds__(1024) void topk_group_kernel(RouteArgs g, GroupArgs grp, const double* __restrict__ logits) {
  topk_group_body(g, grp, logits);
}

// ------------------------------------------------------------------------------------------
// Routing AHEAD for a batch of layers whose inputs are all known before the first of them runs — the stack of
// independent per-layer inputs (moe_verify_stack), never a decoder, where layer l + 1 reads what layer l wrote.
// The routing workspace (activation fragments, picks, gates, slot tables) exists in kRouteAhead copies one
// `set_stride` apart; layer b of the batch is routed by the workgroups with batch index b into copy b, with the
// same bodies as above, so every table and every fragment is bit-identical to what a launch per layer produces.
// Two launches per batch instead of one or two per layer.
// ------------------------------------------------------------------------------------------
constexpr int kRouteAhead = 16;
struct AheadArgs {
  const uint16_t* router_w[kRouteAhead];  // the batch's router matrices
  size_t hidden_stride;                   // floats between the inputs of consecutive layers
  size_t set_stride;                      // bytes between consecutive copies of the routing workspace
  size_t logits_stride;                   // doubles between the logits of consecutive layers
};

template <class P>
__device__ __forceinline__ void to_set(P*& p, size_t bytes) {
  if (p) p = reinterpret_cast<P*>(reinterpret_cast<char*>(p) + bytes);
}
// Arguments of batch layer b from those of batch layer 0.  The caller-visible outputs of single calls (picks, gates,
// union, lists) are not batched and must be NULL, except the per-layer union size n_unique_extra[b].
__device__ __forceinline__ void ahead_args(RouteArgs& g, GroupArgs& grp, const AheadArgs& a, int b) {
  const size_t off = (size_t)b * a.set_stride;
  g.hidden += (size_t)b * a.hidden_stride;
  g.router_w = a.router_w[b];
  to_set(g.ids_ws, off), to_set(g.gates_ws, off), to_set(g.xf_hi, off), to_set(g.xf_lo, off);
  grp.ids = g.ids_ws, grp.gates = g.gates_ws;
  to_set(grp.n_unique_ws, off), to_set(grp.slot_expert, off), to_set(grp.tok_slot, off);
  to_set(grp.slot_mask, off), to_set(grp.slot_gate, off);
  if (grp.n_unique_extra) grp.n_unique_extra += b;
}

__global__ __launch_bounds__(64 * kRouteWaves) void route_ahead_kernel(RouteArgs g, GroupArgs grp, AheadArgs a) {
  ahead_args(g, grp, a, blockIdx.y);  // grid (T, batch)
  route_body(g, grp);
}
__global__ __launch_bounds__(256) void group_ahead_kernel(RouteArgs g, GroupArgs grp, AheadArgs a) {
  ahead_args(g, grp, a, blockIdx.x);  // grid (batch)
  group_body(grp, nullptr, nullptr);
}
__global__ __launch_bounds__(64 * kLogitWaves) void logits_ahead_kernel(RouteArgs g, GroupArgs grp, AheadArgs a,
                                                                        double* __restrict__ logits) {
  ahead_args(g, grp, a, blockIdx.z);  // grid (T, expert blocks, batch)
  logits_body<kLogitWaves>(g, logits + (size_t)blockIdx.z * a.logits_stride);
}
__global__ __launch_bounds__(1024) void topk_group_ahead_kernel(RouteArgs g, GroupArgs grp, AheadArgs a,
                                                                const double* __restrict__ logits) {
  ahead_args(g, grp, a, blockIdx.x);  // grid (batch)
  topk_group_body(g, grp, logits + (size_t)blockIdx.x * a.logits_stride);
}

}  // namespace
