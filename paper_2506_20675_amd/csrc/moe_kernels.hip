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
//                  combine (for a single token, T = 1, route_kernel does this itself and the launch is skipped;
//                  with many experts and T > 1 the pair logits_kernel + topk_group_kernel replaces both)
//   gateup_kernel  for each slot of the union: G = w1 X, U = w3 X, H = gate * silu(G) * U   (2/3 of bytes)
//   down_kernel    split-K partial sums of w2 H over (slot, k-chunk)                        (1/3 of bytes)
//   combine_kernel out[t] = sum of the slabs of token t's own picks, in pick order (deterministic, no atomics)
//   down_fused_kernel   steps 4 + 5 in one launch for steps with few tokens in flight (compact H fragments)
//   *_ahead_kernel      steps 1 + 2 for a batch of layers at once, where all their inputs are known up front
//                       (moe_verify_stack); there the slab sum also rides in the next layer's gate/up launch
//
// Source layout (one translation unit): moe_common.h (conversions, fragment layout, MFMA wrapper, software
// pipeline, weight addressing), route_kernels.h (steps 1-2), expert_kernels.h (steps 3-5, weight re-layout),
// chain_kernels.h (chained stack: slab sum + residual + RMSNorm; attention stub), and this file: the
// stream-read probe, the launch plan and the device half of the C ABI.
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
#include "moe_common.h"
#include "route_kernels.h"
#include "expert_kernels.h"
#include "chain_kernels.h"

namespace {

// ------------------------------------------------------------------------------------------
// Measurement aid: plain coalesced read stream.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16_per_wave,
                                                          size_t n16, float* __restrict__ sink) {
  // Every wave owns one contiguous chunk and reads it in batches of eight non-temporal 1 KB loads.  The waves
  // start at different batches of their chunks (and wrap around): chunks are a power of two apart for the usual
  // sizes, and waves that walk them in lockstep keep meeting on the same memory channels — the staggered start
  // reads 3-5 % faster than the aligned one on this chip, and faster than any other pattern tried.
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + wave_index(threadIdx.x);
  const size_t beg = wave * n16_per_wave < n16 ? wave * n16_per_wave : n16;
  const size_t end = beg + n16_per_wave < n16 ? beg + n16_per_wave : n16;
  const size_t nb = (end - beg) / 512;  // whole batches of 8 x 64 units
  const size_t rot = nb ? (wave * 3) % nb : 0;
  uint32_t acc = 0;
  for (size_t b = 0; b < nb; ++b) {
    const size_t bb = b + rot < nb ? b + rot : b + rot - nb;
    const uint4* p = src + beg + bb * 512 + lane;
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld128<true>(reinterpret_cast<const char*>(p + 64 * u), 0);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (size_t i = beg + nb * 512 + lane; i < end; i += 64) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if (lane == 0) atomicXor(reinterpret_cast<unsigned int*>(sink) + (blockIdx.x & 4095), acc);
}

// ------------------------------------------------------------------------------------------
// Measurement aid: the weight loads of the tiled bf16 gate/up kernel and nothing else.  Same grid (one wave per
// 16-row tile of each of `slots` matrices pairs), same walk (the tile row of matrix a and the tile row of matrix
// b, `steps` contiguous 1 KB blocks each), same non-temporal 128-bit loads, same software pipeline of depth 6 —
// but no activation fragments, no matrix-core instructions and no epilogue: the loaded words are XOR-folded into
// `sink`.  Its duration is what ANY arithmetic formulation of the gate/up step (matrix cores, wavefront dot
// products, ...) has to pay for the bytes alone on this access pattern.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void weight_load_twin_kernel(const char* __restrict__ a, const char* __restrict__ b,
                                                             int steps, size_t slot_stride, float* __restrict__ sink) {
  const int lane = threadIdx.x;
  const char* pa = a + (size_t)blockIdx.y * slot_stride + (size_t)blockIdx.x * steps * 1024;
  const char* pb = b + (size_t)blockIdx.y * slot_stride + (size_t)blockIdx.x * steps * 1024;
  uint32_t acc = 0;
  pipeline<2, 1, true, 6>(
      steps,
      [&](Stage<2, 1, true>& st, int s) {
        st.a[0] = ld128<true>(pa, lane * 16 + (uint32_t)s * 1024);
        st.a[1] = ld128<true>(pb, lane * 16 + (uint32_t)s * 1024);
      },
      [&](const Stage<2, 1, true>& st) {
        acc ^= st.a[0].x ^ st.a[0].y ^ st.a[0].z ^ st.a[0].w ^ st.a[1].x ^ st.a[1].y ^ st.a[1].z ^ st.a[1].w;
      });
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if (lane == 0) atomicXor(reinterpret_cast<unsigned int*>(sink) + ((blockIdx.y * gridDim.x + blockIdx.x) & 4095), acc);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------------------------------
// Workspace of moe_verify_layer_noalloc: device memory that exists from the moment the code object is loaded, so
// that entry point never has to allocate.  Every GPU the library runs on holds its own copy of this array until
// the process ends.  In host code the NAME of the array is only a handle for hipGetSymbolAddress; the device
// address it yields (kept per device in g_noalloc) is what kernels, fills and copies are given.
// ------------------------------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Prepares the leading n16 16-byte units of the workspace (router-input fragments and slot tables): zeros, except
// the units [ones_beg, ones_end) — the constant gate rows of the shared experts — which get 1.0.  A kernel and not
// a memset, so that a caller may record it in a HIP graph like the rest of the call.
__global__ __launch_bounds__(256) void scratch_init_kernel(uint4* __restrict__ p, size_t n16, size_t ones_beg,
                                                           size_t ones_end) {
  const uint32_t one = 0x3f800000u;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
    p[i] = (i >= ones_beg && i < ones_end) ? uint4{one, one, one, one} : uint4{0u, 0u, 0u, 0u};
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Host side of the device ABI
// ------------------------------------------------------------------------------------------
struct moe_ctx {
  moe_shape s;
  int device;
  int u_max;              // largest possible union: min(E, max_tokens * top_k)
  int ks_alloc;           // split-K slabs the partial buffer is sized for
  int plan_override[3];   // moe_ctx_tune: gate/up tiles, down tiles, split-K factor; zero = automatic
  int fused_mode;         // moe_ctx_tune: -1 automatic, 0 never fuse down + combine, 1 always (tiled weights)
  int n_sets;             // copies of the routing workspace (moe_verify_stack routes that many layers ahead)
  size_t set_stride;      // bytes from one copy to the next; the pointers below name copy 0
  char* ws;
  size_t ws_bytes;
  uint16_t *xf_hi, *xf_lo, *hf_hi, *hf_lo;  // activation fragments (see frag_unit)
  int32_t *ids, *n_unique, *slot_expert, *tok_slot, *slot_mask;
  float *gates, *slot_gate, *partial;
  float *xn, *resid[2];  // chained stack: normalised router input and the residual stream (ping-pong), [max_tokens, d]
  double* logits;        // wide routers: fp64 logits [max_tokens, E] between logits_kernel and topk_group_kernel
  float *hbuf, *qkv;     // decoder stack: stream after the attention half [max_tokens, d]; q|k|v [max_tokens, (H+2Hkv) dh]
  uint16_t *af_hi, *af_lo;  // decoder stack: fragments of the attention output, H*dh*16 elements each
  bool profiling;
  std::vector<hipEvent_t> events;  // kProfMarks per profiled layer-step
};

namespace {

constexpr int kProfMarks = 5;  // events per profiled layer-step, bracketing route, gate/up, down, combine
constexpr int kWaves = 4;    // waves per workgroup in the expert kernels (they split K)
constexpr int kMaxKS = 16;   // largest split-K factor of the down projection
// The fused down + combine launch is chosen by the number of tokens in flight (see plan_for): with few tokens its
// compact H fragments make it stream as well as the split-K kernel, and it needs neither slabs nor a slab sum.
constexpr int kFusedMaxTokensBf16 = 5, kFusedMaxTokensFp8 = 4, kFusedMaxTokensRiding = 4;
constexpr double kFusedMaxSlots = 32.0;  // larger unions were not measured: they take the split-K plan
constexpr int kFusedHalvesBelow = 256;  // fused down + combine: fewer row tiles than this -> two workgroups per tile
constexpr int kWideRouterExperts = 32;  // from this many experts on, routing goes through logits_kernel + topk_group_kernel

// Launch plan of the two expert kernels for one (T, weight layout).
//   gu_R, dn_R  weight tiles (16 rows) per wave; the pipeline depth is tied to it (fewer tiles ->
//               deeper pipeline, same bytes in flight per wave)
//   dn_KS       split-K factor of the down projection across workgroups
// Chosen from measurements on Mixtral-shaped layers (see plan_for).
struct Plan {
  int gu_R, dn_R, dn_KS;
  int dn_fused_C;  // > 0: few tokens in flight: down projection and combine in one launch with this many k-chunks per slot
};

int ks_cap_for(const moe_shape& s, bool fp8) {
  const int nsteps = s.ffn / (fp8 ? 64 : 32);
  int cap = 1;
  while (cap < kMaxKS && nsteps / (kWaves * cap * 2) >= 4) cap *= 2;  // every wave keeps >= 4 k-steps
  return cap;
}

// expected number of live expert slots for T tokens under uniform routing (balls into bins), shared experts included
double expected_slots(const moe_shape& s, int T) {
  double miss = 1.0;
  for (int t = 0; t < T; ++t) miss *= 1.0 - (double)s.top_k / s.n_experts;
  return s.n_experts * (1.0 - miss) + s.n_shared;
}

// plan_override: three ints (gate/up tiles, down tiles, split-K factor), each zero = automatic (moe_ctx_tune)
Plan plan_for(const moe_shape& s, const int* plan_override, int fused_mode, int T, bool tiled, bool fp8,
              bool combine_rides = false) {
  const double slots = expected_slots(s, T);
  Plan p;
  p.gu_R = !tiled ? ((s.ffn / 16 / 2) * kWaves * slots >= 1536 ? 2 : 1)
           : fp8 ? ((s.ffn / 32) * slots >= 1024 || T > kPackedTokens ? 2 : 1) : 1;  // tiled: see launch_experts
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
  // Down projection and slab sum in ONE launch (down_fused_kernel, tiled weights, packed fragments): it fetches one
  // fragment byte per weight byte, but takes H in a compact layout of 2 T columns, so with few tokens in flight that
  // costs little, and it writes no slabs.  Measured against split-K + slab sum on all six shapes, each forced both
  // ways at every K: with bf16 weights it wins for T <= 5 (Mixtral-shaped layer 3-8 us at K = 0..3, Phi-3.5-like up
  // to 7 us, the 64-expert shapes 1-3 us), at T = 6 still by 2-4 us on the 4096-wide layers, and loses from T = 6 or
  // 7 on; with FP8 weights for T <= 4.  Where the slab
  // sum costs no launch anyway (moe_verify_stack, chained stacks) it still wins for T <= 4 with bf16 weights on
  // layers that give every compute unit a whole row tile (d / 16 >= 256: 3-5 us per layer); it loses on narrower
  // ones, whose half-tile workgroups fetch two fragment bytes per weight byte, and is level or worse with FP8 weights.  Items = live slots x k-chunks, dealt to 16 waves; every
  // item keeps >= 8 steps.
  p.dn_fused_C = 0;
  const int nsteps = s.ffn / (fp8 ? 64 : 32);
  bool fuse = false;
  if (tiled && T <= kPackedTokens && slots <= kFusedMaxSlots)
    fuse = combine_rides ? (!fp8 && s.d / 16 >= kFusedHalvesBelow && T <= kFusedMaxTokensRiding)
                         : T <= (fp8 ? kFusedMaxTokensFp8 : kFusedMaxTokensBf16 + (s.d / 16 >= kFusedHalvesBelow ? 1 : 0));
  if (fused_mode >= 0) fuse = fused_mode > 0 && tiled;
  if (fuse) {
    // the split that gives the 16 waves the fewest rounds of the shortest items for the expected union, an item
    // costing its steps plus about 6 steps' worth of pipeline restart
    int C = 1;
    double best = 1e30;
    for (int c = 1; c <= 8 && (c == 1 || nsteps / c >= 8); c *= 2) {
      const int rounds = ((int)(slots * c + 0.999) + kFusedWaves - 1) / kFusedWaves;
      const double cost = rounds * ((nsteps + c - 1) / c + 6.0);
      if (cost < best) best = cost, C = c;
    }
    p.dn_fused_C = C;
  }
  if (plan_override[0] > 0) p.gu_R = plan_override[0];
  if (plan_override[1] > 0) p.dn_R = plan_override[1];
  if (plan_override[2] > 0) p.dn_KS = plan_override[2] < cap ? plan_override[2] : cap;
  return p;
}
bool plan_override_free(const moe_ctx* c) { return c->plan_override[1] == 0; }  // moe_ctx_tune left the down tiles alone
Plan plan_for(const moe_ctx* c, int T, bool tiled, bool fp8, bool combine_rides = false) {
  return plan_for(c->s, c->plan_override, c->fused_mode, T, tiled, fp8, combine_rides);
}

// Geometry-dependent host fields of a context (automatic plan; slab buffer sized for the largest split-K factor
// any T can ask for).
void ctx_set_shape(moe_ctx* c, const moe_shape& s, int dev, int n_sets) {
  c->s = s;
  c->device = dev;
  c->n_sets = n_sets;
  c->profiling = false;
  c->u_max = s.max_tokens * s.top_k < s.n_experts ? s.max_tokens * s.top_k : s.n_experts;
  c->plan_override[0] = c->plan_override[1] = c->plan_override[2] = 0;
  c->fused_mode = -1;
  c->ks_alloc = 1;
  for (int T = 1; T <= s.max_tokens; ++T)
    for (bool tiled : {false, true})
      for (bool fp8 : {false, true}) {
        const int ks = plan_for(c, T, tiled, fp8).dn_KS;
        if (ks > c->ks_alloc) c->ks_alloc = ks;
      }
}

// Carves the workspace of a context out of `base` (256-byte aligned pieces) and returns its size; base == NULL
// only measures.  The pieces whose CONTENT a layer-step relies on before writing them come first — the
// activation fragments of the router input (their padded token columns are read by the matrix cores) and the
// per-slot tables (the shared experts' gate rows are constant 1) — and *init_bytes gets their total size.  That
// leading part, the routing workspace, is laid out c->n_sets times back to back (the pointers name copy 0).
size_t ctx_layout(moe_ctx* c, char* base, size_t* init_bytes = nullptr) {
  const moe_shape& s = c->s;
  const size_t A = (size_t)s.max_tokens * s.top_k;
  size_t off = 0;
  auto carve = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const size_t n_slots = (size_t)c->u_max + s.n_shared;
  const size_t o_xh = carve((size_t)s.d * kGateCols * 2), o_xl = carve((size_t)s.d * kGateCols * 2);
  const size_t o_ids = carve(A * 4), o_gates = carve(A * 4), o_nu = carve(4);
  const size_t o_se = carve((size_t)c->u_max * 4), o_sg = carve(n_slots * kGateCols * 4), o_ts = carve(A * 4);
  const size_t o_sm = carve((size_t)c->u_max * 4);
  if (init_bytes) *init_bytes = off;
  c->set_stride = off;
  off *= (size_t)c->n_sets;
  const size_t o_hh = carve(n_slots * s.ffn * kGateCols * 2);
  const size_t o_hl = carve(n_slots * s.ffn * kGateCols * 2);
  const size_t o_part = carve(n_slots * c->ks_alloc * s.max_tokens * s.d * 4);
  const size_t o_xn = carve((size_t)s.max_tokens * s.d * 4);
  const size_t o_r0 = carve((size_t)s.max_tokens * s.d * 4), o_r1 = carve((size_t)s.max_tokens * s.d * 4);
  const size_t nq = (size_t)s.n_heads * s.head_dim, nqkv = nq + 2 * (size_t)s.n_kv_heads * s.head_dim;
  const size_t o_hb = carve((size_t)s.max_tokens * s.d * 4), o_qkv = carve((size_t)s.max_tokens * nqkv * 4 + 16);
  const size_t o_ah = carve(nq * kGateCols * 2 + 16), o_al = carve(nq * kGateCols * 2 + 16);
  const size_t o_lg = carve((size_t)c->n_sets * s.max_tokens * s.n_experts * 8);
  if (!base) return off;
  c->ws = base;
  c->xf_hi = reinterpret_cast<uint16_t*>(base + o_xh);
  c->xf_lo = reinterpret_cast<uint16_t*>(base + o_xl);
  c->hf_hi = reinterpret_cast<uint16_t*>(base + o_hh);
  c->hf_lo = reinterpret_cast<uint16_t*>(base + o_hl);
  c->ids = reinterpret_cast<int32_t*>(base + o_ids);
  c->gates = reinterpret_cast<float*>(base + o_gates);
  c->n_unique = reinterpret_cast<int32_t*>(base + o_nu);
  c->slot_expert = reinterpret_cast<int32_t*>(base + o_se);
  c->slot_gate = reinterpret_cast<float*>(base + o_sg);
  c->tok_slot = reinterpret_cast<int32_t*>(base + o_ts);
  c->slot_mask = reinterpret_cast<int32_t*>(base + o_sm);
  c->partial = reinterpret_cast<float*>(base + o_part);
  c->xn = reinterpret_cast<float*>(base + o_xn);
  c->resid[0] = reinterpret_cast<float*>(base + o_r0);
  c->resid[1] = reinterpret_cast<float*>(base + o_r1);
  c->hbuf = reinterpret_cast<float*>(base + o_hb);
  c->qkv = reinterpret_cast<float*>(base + o_qkv);
  c->af_hi = reinterpret_cast<uint16_t*>(base + o_ah);
  c->af_lo = reinterpret_cast<uint16_t*>(base + o_al);
  c->logits = reinterpret_cast<double*>(base + o_lg);
  return off;
}

moe_status validate_shape(const moe_shape& s) {
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
  return MOE_OK;
}

// The context's workspace lives on one device: the current device must be that one, and so must the stream's
// (the NULL stream belongs to the current device; a stream HIP cannot place is taken as the caller's word).
moe_status check_stream_device(const moe_ctx* c, void* stream) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
  if (dev != c->device) return MOE_ERR_INVALID_ARG;
  if (stream) {
    hipDevice_t sdev = -1;
    if (hipStreamGetDevice((hipStream_t)stream, &sdev) != hipSuccess)
      (void)hipGetLastError();
    else if ((int)sdev != c->device)
      return MOE_ERR_INVALID_ARG;
  }
  return MOE_OK;
}

// profiling mode only: drop an event into the stream between kernels
void mark(moe_ctx* c, hipStream_t st) {
  if (!c->profiling) return;
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return;
  (void)hipEventRecord(e, st);
  c->events.push_back(e);
}

// One copy of the routing workspace: what steps 1 and 2 leave for the expert kernels and the slab sum.
struct RouteSet {
  uint16_t *xf_hi, *xf_lo;
  int32_t *n_unique, *slot_expert, *tok_slot, *slot_mask;
  float* slot_gate;
};
RouteSet route_set(const moe_ctx* c, int b) {
  const size_t off = (size_t)b * c->set_stride;
  auto at = [off](auto* p) { return reinterpret_cast<decltype(p)>(reinterpret_cast<char*>(p) + off); };
  return RouteSet{at(c->xf_hi), at(c->xf_lo), at(c->n_unique), at(c->slot_expert), at(c->tok_slot), at(c->slot_mask),
                  at(c->slot_gate)};
}

RouteArgs route_args(const moe_ctx* c, const float* hidden, const uint16_t* router_w, int T, int32_t* ids,
                     float* gates) {
  const moe_shape& s = c->s;
  return RouteArgs{hidden, router_w, s.d, s.n_experts, s.top_k, T, s.gate_mode, c->ids, ids, c->gates, gates,
                   c->xf_hi, c->xf_lo};
}
GroupArgs group_args(const moe_ctx* c, int T, int32_t* unique, int32_t* n_unique, int32_t* n_unique_extra) {
  const moe_shape& s = c->s;
  return GroupArgs{c->ids, c->gates, T, s.top_k, s.n_experts, unique, n_unique, nullptr, nullptr, nullptr,
                   c->n_unique, n_unique_extra, c->slot_expert, c->tok_slot, c->slot_mask, c->slot_gate};
}

// Steps 1 and 2 for B <= kRouteAhead layers at once (moe_verify_stack: every layer's input is known up front): layer
// l0 + b is routed into copy b of the routing workspace.  Two launches, whatever B is.
void launch_route_ahead(moe_ctx* c, const moe_layer_weights* layers, int B, const float* hidden, int T,
                        int32_t* n_unique_extra, hipStream_t st) {
  const moe_shape& s = c->s;
  const RouteArgs ra = route_args(c, hidden, nullptr, T, nullptr, nullptr);
  const GroupArgs ga = group_args(c, T, nullptr, nullptr, n_unique_extra);
  AheadArgs aa{};
  for (int b = 0; b < B; ++b) aa.router_w[b] = layers[b].router_w;
  aa.hidden_stride = (size_t)T * s.d;
  aa.set_stride = c->set_stride;
  aa.logits_stride = (size_t)s.max_tokens * s.n_experts;
  if (s.n_experts >= kWideRouterExperts) {
    const dim3 grid(T, (s.n_experts + kLogitExperts - 1) / kLogitExperts, B);
    hipLaunchKernelGGL(logits_ahead_kernel, grid, dim3(64 * kLogitWaves), 0, st, ra, ga, aa, c->logits);
    hipLaunchKernelGGL(topk_group_ahead_kernel, dim3(B), dim3(1024), 0, st, ra, ga, aa, (const double*)c->logits);
    return;
  }
  hipLaunchKernelGGL(route_ahead_kernel, dim3(T, B), dim3(64 * kRouteWaves), 0, st, ra, ga, aa);
  if (T > 1) hipLaunchKernelGGL(group_ahead_kernel, dim3(B), dim3(256), 0, st, ra, ga, aa);
}

// Steps 1 and 2.  ids / gates / unique / n_unique / n_unique_extra: optional DEVICE outputs.
// pre != NULL (chained stacks): the slab sum + residual + RMSNorm pass that produces `hidden` runs first — inside
// the router's launch when the router is the one-workgroup-per-token kernel.
void launch_route_and_group(moe_ctx* c, const float* hidden, const uint16_t* router_w, int T, int32_t* ids,
                            float* gates, int32_t* unique, int32_t* n_unique, int32_t* n_unique_extra, hipStream_t st,
                            const ChainArgs* pre = nullptr) {
  const moe_shape& s = c->s;
  const RouteArgs ra = route_args(c, hidden, router_w, T, ids, gates);
  const GroupArgs ga = group_args(c, T, unique, n_unique, n_unique_extra);
  if (s.n_experts >= kWideRouterExperts) {
    // many experts: logits over (token, 16 experts) workgroups, then one workgroup for top-k + union (measured
    // faster than the one-workgroup-per-token router even for a single token, where it costs a launch more)
    const dim3 grid(T, (s.n_experts + kLogitExperts - 1) / kLogitExperts);
    if (pre && pre->gamma && s.d <= kChainLogitsMaxD) {
      hipLaunchKernelGGL(chain_logits_kernel, grid, dim3(kChainThreads), 0, st, *pre, ra, c->logits);
    } else {
      if (pre) hipLaunchKernelGGL(chain_kernel, dim3(T), dim3(kChainThreads), 0, st, *pre);
      hipLaunchKernelGGL(logits_kernel, grid, dim3(64 * kLogitWaves), 0, st, ra, c->logits);
    }
    hipLaunchKernelGGL(topk_group_kernel, dim3(1), dim3(1024), 0, st, ra, ga, (const double*)c->logits);
    return;
  }
  if (pre)
    hipLaunchKernelGGL(chain_route_kernel, dim3(T), dim3(kChainThreads), 0, st, *pre, ra, ga);
  else
    hipLaunchKernelGGL(route_kernel, dim3(T), dim3(64 * kRouteWaves), 0, st, ra, ga);
  if (T > 1) hipLaunchKernelGGL(group_kernel, dim3(1), dim3(256), 0, st, ga);  // T = 1: done inside route_kernel
}

template <int R, int P>
void launch_gateup(const moe_ctx* c, const GateupArgs& a, hipStream_t st) {  // row-major bf16 weights
  const dim3 grid((c->s.ffn / 16 + R - 1) / R, a.routed_slots + c->s.n_shared + a.cmb_rows);
  if (a.T <= kPackedTokens)
    hipLaunchKernelGGL((gateup_kernel<R, kWaves, P, false, false, false, true>), grid, dim3(64 * kWaves), 0, st, a);
  else
    hipLaunchKernelGGL((gateup_kernel<R, kWaves, P, false, false, false, false>), grid, dim3(64 * kWaves), 0, st, a);
}
// Tiled weights are read exactly once in contiguous 1 KB pieces -> streaming loads; row-major weights
// are read in 64-byte row segments whose cache lines are completed by the next k-step -> cached loads.
template <int R, int P>
void launch_down(const moe_ctx* c, const DownArgs& a, bool tiled, bool fp8, hipStream_t st) {
  const dim3 grid((c->s.d / 16 + R - 1) / R, a.KS, a.routed_slots + c->s.n_shared), block(64 * kWaves);
  const bool pk = a.T <= kPackedTokens;
  constexpr int PF = P > 4 ? 4 : P;  // an FP8 stage carries the fragments of two k-steps: depth 4 at most
  if (fp8 && tiled) {
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, true, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, true, false>), grid, block, 0, st, a);
  } else if (fp8) {
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, PF, false, false, true, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, PF, false, false, true, false>), grid, block, 0, st, a);
  } else if (tiled) {
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, P, true, true, false, false>), grid, block, 0, st, a);
  } else {
    if (pk) hipLaunchKernelGGL((down_kernel<R, kWaves, P, false, false, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((down_kernel<R, kWaves, P, false, false, false, false>), grid, block, 0, st, a);
  }
}

void launch_combine(const CombineArgs& a, hipStream_t st) {
  const int n4 = a.T * (a.d / 4);
  hipLaunchKernelGGL(combine_kernel, dim3((n4 + 255) / 256), dim3(256), 0, st, a);
}
CombineArgs combine_args(const moe_ctx* c, const RouteSet& rs, int T, float* out, int ks) {
  const moe_shape& s = c->s;
  return CombineArgs{c->partial, rs.tok_slot, out, s.d, T, s.top_k, c->u_max, s.n_shared, s.max_tokens, ks};
}

// Steps 3 to 5 of one layer-step, on the routing tables and activation fragments in `rs`.  The expert-union step has
// no launch of its own: it is the liveness test at the top of the expert kernels.
// out == NULL: the slabs are left for the caller (chained stack: chain_kernel sums them); *ks_used gets the
// split-K factor they were written with.  defer_combine (with out != NULL): the same, unless the down projection
// is the fused one, which writes `out` itself (*ks_used = 0: nothing is pending).
// cmb != NULL: the gate/up launch also sums the slabs another layer-step left (see GateupArgs).
moe_status launch_experts(moe_ctx* c, const RouteSet& rs, const moe_layer_weights* w, int T, float* out,
                          hipStream_t st, int* ks_used, bool defer_combine, const CombineArgs* cmb) {
  const moe_shape& s = c->s;
  const bool tiled = w->layout == MOE_LAYOUT_TILED, fp8 = w->dtype == MOE_WEIGHT_FP8_E4M3;
  const Plan p = plan_for(c, T, tiled, fp8, defer_combine || !out);  // the slab sum rides in another launch
  const int routed_slots = T * s.top_k < s.n_experts ? T * s.top_k : s.n_experts;  // largest union T tokens can form
  const int cr = cmb ? 1 : 0;
  const bool pk = T <= kPackedTokens;  // must match what the router wrote
  // the fused down + combine kernel takes H in the compact packed layout: 2 T columns per k-group instead of 16
  const int h_cols = pk && p.dn_fused_C > 0 ? 2 * T : 0;
  GateupArgs ga{w->w1, w->w3, w->sw1, w->sw3, w->w1_scale, w->w3_scale, w->sw1_scale, w->sw3_scale,
                rs.xf_hi, rs.xf_lo, rs.n_unique, rs.slot_expert, rs.slot_mask, rs.slot_gate,
                c->hf_hi, c->hf_lo, s.d, s.ffn, T, routed_slots, c->u_max, cr, h_cols, cmb ? *cmb : CombineArgs{}};
  const unsigned rows = routed_slots + s.n_shared + cr;
  if (fp8 && !tiled) {
    // row-major FP8 (the layout checkpoints come in; the tiled one is the fast path): two tile pairs per wave,
    // four waves splitting d, whatever the plan says
    const dim3 grid((s.ffn / 16 + 1) / 2, rows), block(64 * kWaves);
    if (pk) hipLaunchKernelGGL((gateup_kernel<2, kWaves, 3, false, false, true, true>), grid, block, 0, st, ga);
    else hipLaunchKernelGGL((gateup_kernel<2, kWaves, 3, false, false, true, false>), grid, block, 0, st, ga);
  } else if (fp8) {
    // FP8 needs twice the fragment bytes per weight byte, and those come from L2: two tile pairs per wave
    // share each fragment load, and a shallow pipeline keeps four waves per SIMD (measured best of
    // {1, 2, 4} tile pairs x depths 2..10)
    // ... unless that leaves fewer than about a thousand waves in the grid (small unions of small experts): then one
    // pair per wave at depth 6, twice as many waves (OLMoE-like FP8 layer at K = 0: 29.2 -> 25.9 us)
    const dim3 grid((s.ffn / 16 + 1) / 2, rows), grid1(s.ffn / 16, rows);
    if (pk && p.gu_R == 1) hipLaunchKernelGGL((gateup_kernel<1, 1, 6, true, true, true, true>), grid1, dim3(64), 0, st, ga);
    else if (pk) hipLaunchKernelGGL((gateup_kernel<2, 1, 3, true, true, true, true>), grid, dim3(64), 0, st, ga);
    else hipLaunchKernelGGL((gateup_kernel<2, 1, 3, true, true, true, false>), grid, dim3(64), 0, st, ga);
  } else if (tiled) {
    // one wave per 16-row tile pair over the whole of d (splitting d over 2 or 4 waves when the union
    // is small on a small expert was measured: no gain, the step is bound by launch latencies there)
    const dim3 grid(s.ffn / 16, rows);
    if (pk) hipLaunchKernelGGL((gateup_kernel<1, 1, 6, true, true, false, true>), grid, dim3(64), 0, st, ga);
    else hipLaunchKernelGGL((gateup_kernel<1, 1, 6, true, true, false, false>), grid, dim3(64), 0, st, ga);
  } else {
    switch (p.gu_R) {
      case 4: launch_gateup<4, 2>(c, ga, st); break;
      case 2: launch_gateup<2, 4>(c, ga, st); break;
      default: launch_gateup<1, 8>(c, ga, st); break;
    }
  }
  mark(c, st);
  if (p.dn_fused_C > 0) {
    // down projection and combine in one launch; with no `out` (chained stack) the summed term goes to the slab
    // buffer as a plain [T, d] array and *ks_used = 0 tells the caller so
    DownFusedArgs fa{w->w2, w->sw2, w->w2_scale, w->sw2_scale, c->hf_hi, c->hf_lo, rs.n_unique, rs.slot_expert,
                     rs.slot_mask, out ? out : c->partial, s.d, s.ffn, T, s.n_shared, c->u_max, p.dn_fused_C,
                     s.d / 16 < kFusedHalvesBelow ? 2 : 1, h_cols};
    const dim3 grid(s.d / 16 * fa.halves), block(64 * kFusedWaves);
    if (fp8) {
      if (pk) hipLaunchKernelGGL((down_fused_kernel<4, true, true>), grid, block, 0, st, fa);
      else hipLaunchKernelGGL((down_fused_kernel<4, true, false>), grid, block, 0, st, fa);
    } else {
      if (pk) hipLaunchKernelGGL((down_fused_kernel<4, false, true>), grid, block, 0, st, fa);
      else hipLaunchKernelGGL((down_fused_kernel<4, false, false>), grid, block, 0, st, fa);
    }
    mark(c, st);
    if (ks_used) *ks_used = 0;
    mark(c, st);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
  }
  DownArgs da{w->w2, w->sw2, w->w2_scale, w->sw2_scale, c->hf_hi, c->hf_lo, rs.n_unique, rs.slot_expert,
              rs.slot_mask, c->partial, s.d, s.ffn, T, routed_slots, c->u_max, s.max_tokens, p.dn_KS};
  if (fp8 && tiled && !pk && p.dn_R == 4 && plan_override_free(c)) {
    // FP8 weights with split fragments (T > 8) need as many fragment bytes from L2 as weight bytes from HBM at 4
    // row tiles per wave; 8 tiles at depth 2 halve that (measured: 63 -> 60 us on the Mixtral-shaped layer at T = 9;
    // with packed fragments, and with bf16 weights, 4 tiles at depth 4 stay faster)
    const dim3 grid((s.d / 16 + 7) / 8, da.KS, routed_slots + s.n_shared), block(64 * kWaves);
    hipLaunchKernelGGL((down_kernel<8, kWaves, 2, true, true, true, false>), grid, block, 0, st, da);
  } else {
    switch (p.dn_R) {
      case 4: launch_down<4, 4>(c, da, tiled, fp8, st); break;
      case 2: launch_down<2, 4>(c, da, tiled, fp8, st); break;
      default: launch_down<1, 8>(c, da, tiled, fp8, st); break;
    }
  }
  mark(c, st);
  if (ks_used) *ks_used = p.dn_KS;
  if (out && !defer_combine) launch_combine(combine_args(c, rs, T, out, p.dn_KS), st);
  mark(c, st);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// One layer-step after validation: router, gate/up, down, slab sum.
// unique / n_unique / n_unique_extra: optional DEVICE outputs; ks_used / pre: see launch_experts and
// launch_route_and_group.
moe_status launch_layer(moe_ctx* c, const moe_layer_weights* w, const float* hidden, int T, float* out, int32_t* ids,
                        float* gates, int32_t* unique, int32_t* n_unique, int32_t* n_unique_extra, hipStream_t st,
                        int* ks_used = nullptr, const ChainArgs* pre = nullptr) {
  mark(c, st);
  launch_route_and_group(c, hidden, w->router_w, T, ids, gates, unique, n_unique, n_unique_extra, st, pre);
  mark(c, st);
  return launch_experts(c, route_set(c, 0), w, T, out, st, ks_used, false, nullptr);
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

// Per-device state of moe_verify_layer_noalloc: the device address of `scratch` on that device and a context that
// lives in host memory of this library and is laid out over it.
constexpr int kMaxDevices = 64;
struct NoAllocSlot {
  char* base = nullptr;     // device address of the scratch array on this device (hipGetSymbolAddress)
  bool have_shape = false;  // ctx below is set up for `shape`
  moe_shape shape;
  size_t init_bytes = 0;
  moe_ctx ctx;
};
NoAllocSlot g_noalloc[kMaxDevices];


}  // namespace

extern "C" {

const char* moe_strerror(moe_status s) {
  switch (s) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED_SHAPE: return "unsupported layer shape";
    case MOE_ERR_WORKSPACE: return "device workspace could not be allocated, or the geometry needs more than the fixed workspace";
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
  if (moe_status st = validate_shape(s)) return st;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
  moe_ctx* c = new (std::nothrow) moe_ctx();
  if (!c) return MOE_ERR_WORKSPACE;
  ctx_set_shape(c, s, dev, kRouteAhead);
  c->ws_bytes = ctx_layout(c, nullptr);
  if (c->ws_bytes > ((size_t)8 << 30) || hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return MOE_ERR_WORKSPACE;
  }
  (void)ctx_layout(c, c->ws);
  if (hipMemset(c->ws, 0, c->ws_bytes) != hipSuccess) {  // padded token columns of the fragments are finite zeros
    (void)hipFree(c->ws);
    delete c;
    return MOE_ERR_HIP;
  }
  if (s.n_shared > 0) {  // shared-expert slots carry gate 1 for every token column
    float ones[kMaxShared * kGateCols];
    for (int i = 0; i < s.n_shared * kGateCols; ++i) ones[i] = 1.f;
    for (int b = 0; b < c->n_sets; ++b)
      if (hipMemcpy(reinterpret_cast<char*>(c->slot_gate + (size_t)c->u_max * kGateCols) + b * c->set_stride, ones,
                    sizeof(float) * s.n_shared * kGateCols, hipMemcpyHostToDevice) != hipSuccess) {
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

moe_status moe_ctx_tune(moe_ctx* c, int32_t gu_tiles, int32_t dn_tiles, int32_t dn_split_k, int32_t fused_down) {
  auto tiles_ok = [](int v) { return v == 0 || v == 1 || v == 2 || v == 4; };
  if (!c || !tiles_ok(gu_tiles) || !tiles_ok(dn_tiles) || dn_split_k < 0 || dn_split_k > kMaxKS) return MOE_ERR_INVALID_ARG;
  if (dn_split_k & (dn_split_k - 1)) return MOE_ERR_INVALID_ARG;  // powers of two only
  if (fused_down < -1 || fused_down > 1) return MOE_ERR_INVALID_ARG;
  c->plan_override[0] = gu_tiles;
  c->plan_override[1] = dn_tiles;
  // the slab buffer was sized at creation for the automatic plan: a larger split does not fit
  c->plan_override[2] = dn_split_k < c->ks_alloc ? dn_split_k : c->ks_alloc;
  c->fused_mode = fused_down;
  return MOE_OK;
}

moe_status moe_plan_query(const moe_shape* shape, int32_t T, int32_t layout, int32_t dtype, moe_plan_info* out) {
  if (!shape || !out) return MOE_ERR_INVALID_ARG;
  const moe_shape s = *shape;
  if (moe_status st = validate_shape(s)) return st;
  if (T < 1 || T > s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (layout != MOE_LAYOUT_ROW_MAJOR && layout != MOE_LAYOUT_TILED) return MOE_ERR_INVALID_ARG;
  if (dtype != MOE_WEIGHT_BF16 && dtype != MOE_WEIGHT_FP8_E4M3) return MOE_ERR_INVALID_ARG;
  const bool tiled = layout == MOE_LAYOUT_TILED, fp8 = dtype == MOE_WEIGHT_FP8_E4M3;
  if (fp8 && (s.d % 64 || s.ffn % 64)) return MOE_ERR_UNSUPPORTED_SHAPE;
  const int automatic[3] = {0, 0, 0};
  const Plan p = plan_for(s, automatic, -1, T, tiled, fp8);
  out->routed_slots = T * s.top_k < s.n_experts ? T * s.top_k : s.n_experts;
  out->expected_slots = expected_slots(s, T);
  out->wide_router = s.n_experts >= kWideRouterExperts;
  out->packed_fragments = T <= kPackedTokens;
  out->gu_tiles = fp8 && !tiled ? 2 : p.gu_R;  // row-major FP8 has one fixed shape (see launch_experts)
  out->dn_tiles = p.dn_R;
  out->dn_split_k = p.dn_KS;
  out->dn_fused_chunks = p.dn_fused_C;
  const int route_launches = out->wide_router ? 2 : (T > 1 ? 2 : 1);
  out->launches = route_launches + 1 + (p.dn_fused_C > 0 ? 1 : 2);
  return MOE_OK;
}

moe_status moe_route(moe_ctx* c, const float* hidden, const uint16_t* router_w, int32_t T, int32_t* ids, float* gates,
                     int32_t* unique_experts, int32_t* n_unique, void* stream) {
  if (!c || !hidden || !router_w || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(router_w)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c, stream)) return st;
  launch_route_and_group(c, hidden, router_w, T, ids, gates, unique_experts, n_unique, nullptr, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_group(moe_ctx* c, const int32_t* ids, int32_t T, int32_t* unique_experts, int32_t* n_unique,
                     int32_t* expert_count, int32_t* expert_offset, int32_t* assign, void* stream) {
  if (!c || !ids || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c, stream)) return st;
  GroupArgs ga{ids, nullptr, T, c->s.top_k, c->s.n_experts, unique_experts, n_unique, expert_count, expert_offset,
               assign, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  hipLaunchKernelGGL(group_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, ga);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_verify_layer(moe_ctx* c, const moe_layer_weights* w, const float* hidden, int32_t T, float* out,
                            int32_t* ids_opt, float* gates_opt, int32_t* unique_opt, int32_t* n_unique_opt,
                            void* stream) {
  if (!c || !hidden || !out || T < 1 || T > c->s.max_tokens || !weights_ok(c, w)) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(out)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c, stream)) return st;
  hipStream_t st = (hipStream_t)stream;
  return launch_layer(c, w, hidden, T, out, ids_opt, gates_opt, unique_opt, n_unique_opt, nullptr, st);
}

moe_status moe_verify_layer_noalloc(const moe_shape* shape, const moe_layer_weights* w, const float* hidden, int32_t T,
                                    float* out, int32_t* ids_opt, float* gates_opt, int32_t* unique_opt,
                                    int32_t* n_unique_opt, void* stream) {
  if (!shape || !hidden || !out) return MOE_ERR_INVALID_ARG;
  const moe_shape s = *shape;
  if (moe_status st = validate_shape(s)) return st;
  if (T < 1 || T > s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(out)) return MOE_ERR_INVALID_ARG;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED_SHAPE;
  NoAllocSlot& slot = g_noalloc[dev];
  if (!slot.base) {
    // once per device, with that device current: every GPU has its own copy of the array at its own address
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return MOE_ERR_HIP;
    }
    slot.base = static_cast<char*>(ptr);
  }
  if (!slot.have_shape || memcmp(&slot.shape, &s, sizeof(s)) != 0) {
    slot.have_shape = false;
    ctx_set_shape(&slot.ctx, s, dev, 1);  // single layer-steps only: one copy of the routing workspace
    const size_t need = ctx_layout(&slot.ctx, nullptr, &slot.init_bytes);
    if (need > kScratchBytes) return MOE_ERR_WORKSPACE;  // this geometry needs more than the fixed workspace
    slot.ctx.ws_bytes = ctx_layout(&slot.ctx, slot.base);
    slot.shape = s;
    slot.have_shape = true;
  }
  moe_ctx* c = &slot.ctx;
  if (!weights_ok(c, w)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c, stream)) return st;
  hipStream_t st = (hipStream_t)stream;
  // the array keeps whatever the last call on this GPU left in it (possibly laid out for another geometry)
  const size_t n16 = slot.init_bytes / 16;
  const size_t ones_beg = (size_t)(reinterpret_cast<char*>(c->slot_gate + (size_t)c->u_max * kGateCols) - slot.base) / 16;
  const size_t ones_end = ones_beg + (size_t)s.n_shared * kGateCols * sizeof(float) / 16;
  const unsigned blocks = (unsigned)((n16 + 255) / 256 < 1024 ? (n16 + 255) / 256 : 1024);
  hipLaunchKernelGGL(scratch_init_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<uint4*>(slot.base), n16,
                     ones_beg, ones_end);
  return launch_layer(c, w, hidden, T, out, ids_opt, gates_opt, unique_opt, n_unique_opt, nullptr, st);
}

moe_status moe_verify_stack(moe_ctx* c, const moe_layer_weights* layers, int32_t L, const float* hidden, int32_t T,
                            float* out, int32_t* n_unique_per_layer_opt, void* stream) {
  if (!c || !layers || L < 1 || !hidden || !out || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!aligned16(hidden) || !aligned16(out)) return MOE_ERR_INVALID_ARG;
  for (int l = 0; l < L; ++l)
    if (!weights_ok(c, layers + l)) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c, stream)) return st;
  hipStream_t st = (hipStream_t)stream;
  const moe_shape& s = c->s;
  const size_t per = (size_t)T * s.d;
  if (c->profiling) {  // per-kernel timing wants the same marks per layer-step as a single call
    for (int l = 0; l < L; ++l)
      if (moe_status rc = launch_layer(c, layers + l, hidden + l * per, T, out + l * per, nullptr, nullptr, nullptr,
                                       nullptr, n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st))
        return rc;
    return MOE_OK;
  }
  // The inputs of all layers are here before the first layer runs (they do not depend on one another), so routing
  // is done ahead, for up to kRouteAhead layers per pair of launches, and the slab sum of layer l rides in the
  // gate/up launch of layer l + 1: two launches per layer-step instead of four or five.  Only this call can do that:
  // in a decoder the input of layer l + 1 is the output of layer l (moe_chained_stack, moe_decoder_stack).
  int ks = 0;  // > 0: the previous layer's slabs are waiting to be summed into its `out`
  for (int l0 = 0; l0 < L; l0 += c->n_sets) {
    const int B = L - l0 < c->n_sets ? L - l0 : c->n_sets;
    if (ks > 0) {  // its pick-to-slot table is in the last copy, which the routing below overwrites
      launch_combine(combine_args(c, route_set(c, c->n_sets - 1), T, out + (size_t)(l0 - 1) * per, ks), st);
      ks = 0;
    }
    launch_route_ahead(c, layers + l0, B, hidden + (size_t)l0 * per, T,
                       n_unique_per_layer_opt ? n_unique_per_layer_opt + l0 : nullptr, st);
    for (int b = 0; b < B; ++b) {
      const int l = l0 + b;
      CombineArgs cmb{};
      if (ks > 0) cmb = combine_args(c, route_set(c, b - 1), T, out + (size_t)(l - 1) * per, ks);
      if (moe_status rc = launch_experts(c, route_set(c, b), layers + l, T, out + (size_t)l * per, st, &ks, true,
                                         ks > 0 ? &cmb : nullptr))
        return rc;
    }
  }
  if (ks > 0) {
    const int last = (L - 1) % c->n_sets;
    launch_combine(combine_args(c, route_set(c, last), T, out + (size_t)(L - 1) * per, ks), st);
  }
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_chained_stack(moe_ctx* c, const moe_layer_weights* layers, const uint16_t* const* gammas, int32_t L,
                             const float* x_in, int32_t T, float eps, float* x_out, float* trace_opt,
                             int32_t* n_unique_per_layer_opt, void* stream) {
  if (!c || !layers || !gammas || L < 1 || !x_in || !x_out || T < 1 || T > c->s.max_tokens) return MOE_ERR_INVALID_ARG;
  if (!(eps >= 0.f) || !aligned16(x_in) || !aligned16(x_out) || (trace_opt && !aligned16(trace_opt)))
    return MOE_ERR_INVALID_ARG;
  if (c->s.d > 4 * kChainVecs * kChainThreads) return MOE_ERR_UNSUPPORTED_SHAPE;
  for (int l = 0; l < L; ++l)
    if (!weights_ok(c, layers + l) || !gammas[l] || !aligned16(gammas[l])) return MOE_ERR_INVALID_ARG;
  if (moe_status st = check_stream_device(c, stream)) return st;
  hipStream_t st = (hipStream_t)stream;
  const moe_shape& s = c->s;
  const size_t per = (size_t)T * s.d;
  const float* cur = x_in;  // x_{l-1}: the stream the pending MoE term is added to
  int ks = 1;
  for (int l = 0; l <= L; ++l) {
    // finish block l-1 (if any) and, unless this is the end, normalise for block l
    ChainArgs a{};
    a.partial = l > 0 && ks > 0 ? c->partial : nullptr;
    a.moe_out = l > 0 && ks == 0 ? c->partial : nullptr;  // ks == 0: the fused down projection already summed the term
    a.tok_slot = c->tok_slot;
    a.resid_in = cur;
    float* dst = l == L ? x_out : (trace_opt ? trace_opt + (size_t)l * per : (l > 0 ? c->resid[l & 1] : nullptr));
    a.resid_out = dst;  // l == 0 without a trace: x_0 stays where the caller has it
    a.gamma = l < L ? gammas[l] : nullptr;
    a.xn_out = c->xn;
    a.d = s.d, a.T = T, a.top_k = s.top_k, a.u_max = c->u_max, a.n_shared = s.n_shared, a.max_tokens = s.max_tokens;
    a.KS = ks, a.eps = eps;
    if (dst) cur = dst;
    if (l == L) {  // the last MoE term and nothing to normalise for
      hipLaunchKernelGGL(chain_kernel, dim3(T), dim3(kChainThreads), 0, st, a);
      break;
    }
    // this pass runs at the head of block l's router launch (or as a launch of its own in front of a wide router)
    if (moe_status rc = launch_layer(c, layers + l, c->xn, T, nullptr, nullptr, nullptr, nullptr, nullptr,
                                     n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st, &ks, &a))
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
  if (moe_status st = check_stream_device(c, stream)) return st;
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
    const moe_attn_weights& a = attn[l];
    if (!a.wqkv || !a.wo || !a.gamma_attn || !a.gamma_moe) return MOE_ERR_INVALID_ARG;
    if (!aligned16(a.wqkv) || !aligned16(a.wo) || !aligned16(a.gamma_attn) || !aligned16(a.gamma_moe))
      return MOE_ERR_INVALID_ARG;
  }
  if (moe_status st = check_stream_device(c, stream)) return st;
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
    a.partial = l > 0 && ks > 0 ? c->partial : nullptr;
    a.moe_out = l > 0 && ks == 0 ? c->partial : nullptr;  // ks == 0: the fused down projection already summed the term
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
    cur = c->hbuf;
    if (moe_status rc = launch_layer(c, layers + l, c->xn, T, nullptr, nullptr, nullptr, nullptr, nullptr,
                                     n_unique_per_layer_opt ? n_unique_per_layer_opt + l : nullptr, st, &ks, &m))
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
  if (moe_status st = check_stream_device(c, stream)) return st;
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
  const size_t per_wave = ((n16 + blocks * 4 - 1) / (blocks * 4) + 511) / 512 * 512;  // whole batches of 8 loads
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const uint4*>(src), per_wave, n16, sink);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_weight_load_twin(const void* a, const void* b, int32_t slots, int32_t tiles, int32_t steps,
                                int64_t slot_stride, float* sink, void* stream) {
  if (!a || !b || !sink || slots < 1 || slots > 65535 || tiles < 1 || steps < 1 || !aligned16(a) || !aligned16(b))
    return MOE_ERR_INVALID_ARG;
  if (slot_stride < (int64_t)tiles * steps * 1024 || slot_stride % 16) return MOE_ERR_INVALID_ARG;
  hipLaunchKernelGGL(weight_load_twin_kernel, dim3(tiles, slots), dim3(64), 0, (hipStream_t)stream,
                     static_cast<const char*>(a), static_cast<const char*>(b), steps, (size_t)slot_stride, sink);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // extern "C"
