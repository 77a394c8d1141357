// MoE verification path for MI355X (gfx950): hand-written HIP kernels + the device half of the C ABI.
//
// One decode iteration of speculative decoding pushes T = K+1 tokens through each MoE layer
// (paper: Section 2.2); every token picks top_k experts on its own, and the layer's cost is the
// HBM traffic for the UNION of the picked experts (Section 1, Section 2.4).  The path below touches
// every unique expert's weights exactly once per step:
//
//   route_kernel   router logits (fp64 accumulate), top-k, softmax gates; also splits the fp32
//                  activations into bf16 hi + lo halves for the matrix cores
//   group_kernel   union of experts, per-expert token lists, per-slot gate table
//   gateup_kernel  for each unique expert: G = w1 X, U = w3 X, H = gate * silu(G) * U      (2/3 of bytes)
//   down_kernel    split-K partial sums of w2 H over (expert, k-chunk)                     (1/3 of bytes)
//   combine_kernel out[t] = sum of the partial slabs in a fixed order (deterministic, no atomics)
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

__device__ __forceinline__ uint4 ld128(const char* base, uint32_t byte_off) {
  return *reinterpret_cast<const uint4*>(base + byte_off);
}

__device__ __forceinline__ f32x4 mfma_bf16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                  0, 0);
}

// ------------------------------------------------------------------------------------------
// Step 1: router.  One workgroup (4 waves) per token.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ hidden,
                                                    const uint16_t* __restrict__ router_w, int d, int E, int top_k,
                                                    int32_t* __restrict__ ids_ws, float* __restrict__ gates_ws,
                                                    int32_t* __restrict__ ids_out, float* __restrict__ gates_out,
                                                    uint16_t* __restrict__ xs_hi, uint16_t* __restrict__ xs_lo) {
  __shared__ double s_logit[kMaxExperts];
  __shared__ float s_sel[kMaxTopK];
  __shared__ int s_id[kMaxTopK];
  const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* x = hidden + (size_t)t * d;

  // activations -> bf16 hi/lo halves, consumed by the expert kernels as the MFMA B operand
  for (int j = tid * 4; j < d; j += 256 * 4) {
    const float4 v = *reinterpret_cast<const float4*>(x + j);
    ushort4 h, l;
    split_bf16(v.x, h.x, l.x);
    split_bf16(v.y, h.y, l.y);
    split_bf16(v.z, h.z, l.z);
    split_bf16(v.w, h.w, l.w);
    *reinterpret_cast<ushort4*>(xs_hi + (size_t)t * d + j) = h;
    *reinterpret_cast<ushort4*>(xs_lo + (size_t)t * d + j) = l;
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
  if (wave != 0) return;

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
      ids_ws[a] = s_id[i];
      gates_ws[a] = g;
      if (ids_out) ids_out[a] = s_id[i];
      if (gates_out) gates_out[a] = g;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 2: union of activated experts + per-expert token lists.  One workgroup, thread e = expert e.
// ------------------------------------------------------------------------------------------
struct GroupOut {
  int32_t *unique, *n_unique, *count, *offset, *assign;
};

__global__ __launch_bounds__(256) void group_kernel(const int32_t* __restrict__ ids, const float* __restrict__ gates,
                                                    int T, int top_k, int E, GroupOut ws, GroupOut user,
                                                    int32_t* __restrict__ n_unique_extra,
                                                    int32_t* __restrict__ slot_expert, float* __restrict__ slot_gate) {
  __shared__ int s_ids[kMaxTokens * kMaxTopK];
  __shared__ int s_cnt[4], s_uni[4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int A = T * top_k;
  if (tid < A) s_ids[tid] = ids[tid];
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
            const float g = gates[a];
#pragma unroll
            for (int n = 0; n < kGateCols; ++n)
              if (n == tok) row[n] = g;
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
// Step 3: gate/up projections + SiLU*mul for every unique expert (and shared expert).
// grid = (row blocks of 16*R rows of ffn, expert slots); block = W waves that split d.
// ------------------------------------------------------------------------------------------
struct GateupArgs {
  const uint16_t *w1, *w3, *sw1, *sw3;  // [E,ffn,d] / [n_shared,ffn,d]
  const uint16_t *xs_hi, *xs_lo;        // [max_tokens,d]
  const int32_t* n_unique;
  const int32_t* slot_expert;  // [u_max]
  const float* slot_gate;      // [u_tot,16]
  uint16_t *h_hi, *h_lo;       // [u_tot,max_tokens,ffn]
  int d, ffn, T, u_max, max_tokens;
};

template <int R, int W, int P>
__global__ __launch_bounds__(64 * W) void gateup_kernel(GateupArgs g) {
  __shared__ float4 red[W * 2 * R * 64];
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

  const char* base[2 * R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const size_t row0 = (size_t)min(tile0 + j, ntiles - 1) * 16;  // ragged last block: re-read a valid tile, result unused
    base[j] = W1 + row0 * g.d * 2;
    base[R + j] = W3 + row0 * g.d * 2;
  }
  const uint32_t a_off = ((uint32_t)r * g.d + s_beg * 32 + kg * 8) * 2;
  const int n = min(r, g.T - 1);  // columns >= T duplicate the last token; their results are dropped
  const uint32_t b_off = ((uint32_t)n * g.d + s_beg * 32 + kg * 8) * 2;
  const char* XH = reinterpret_cast<const char*>(g.xs_hi);
  const char* XL = reinterpret_cast<const char*>(g.xs_lo);

  f32x4 acc[2 * R];
#pragma unroll
  for (int j = 0; j < 2 * R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<2 * R, P>(
      nst,
      [&](Stage<2 * R>& st, int s) {
        const uint32_t ko = (uint32_t)s * 64;
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) st.a[j] = ld128(base[j], a_off + ko);
        st.bh = ld128(XH, b_off + ko);
        st.bl = ld128(XL, b_off + ko);
      },
      [&](const Stage<2 * R>& st) {
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) acc[j] = mfma_bf16(st.a[j], st.bh, acc[j]);
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) acc[j] = mfma_bf16(st.a[j], st.bl, acc[j]);
      });

  // reduce the W k-slices through LDS, then wave w finishes tiles w, w+W, ...
#pragma unroll
  for (int j = 0; j < 2 * R; ++j)
    red[(wave * 2 * R + j) * 64 + lane] = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
  __syncthreads();
  const float gate = g.slot_gate[u * kGateCols + r];
  for (int j = wave; j < R; j += W) {
    if (tile0 + j >= ntiles) break;
    float4 G = red[j * 64 + lane], U = red[(R + j) * 64 + lane];
    for (int w = 1; w < W; ++w) {
      const float4 g2 = red[(w * 2 * R + j) * 64 + lane], u2 = red[(w * 2 * R + R + j) * 64 + lane];
      G.x += g2.x, G.y += g2.y, G.z += g2.z, G.w += g2.w;
      U.x += u2.x, U.y += u2.y, U.z += u2.z, U.w += u2.w;
    }
    if (r < g.T && gate != 0.f) {
      // lane holds rows 4*kg .. 4*kg+3 of the tile for token column r
      const float hv[4] = {gate * (G.x / (1.f + expf(-G.x))) * U.x, gate * (G.y / (1.f + expf(-G.y))) * U.y,
                           gate * (G.z / (1.f + expf(-G.z))) * U.z, gate * (G.w / (1.f + expf(-G.w))) * U.w};
      ushort4 hi, lo;
      split_bf16(hv[0], hi.x, lo.x);
      split_bf16(hv[1], hi.y, lo.y);
      split_bf16(hv[2], hi.z, lo.z);
      split_bf16(hv[3], hi.w, lo.w);
      const size_t o = ((size_t)u * g.max_tokens + r) * g.ffn + (size_t)(tile0 + j) * 16 + kg * 4;
      *reinterpret_cast<ushort4*>(g.h_hi + o) = hi;
      *reinterpret_cast<ushort4*>(g.h_lo + o) = lo;
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
  const uint16_t *h_hi, *h_lo;   // [u_tot,max_tokens,ffn]
  const int32_t* n_unique;
  const int32_t* slot_expert;
  const float* slot_gate;
  float* partial;                // [u_tot*KS, max_tokens, d]
  int d, ffn, T, u_max, max_tokens, KS;
};

template <int R, int W, int P>
__global__ __launch_bounds__(64 * W) void down_kernel(DownArgs g) {
  __shared__ float4 red[W * R * 64];
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

  const char* base[R];
#pragma unroll
  for (int j = 0; j < R; ++j) base[j] = W2 + (size_t)min(tile0 + j, ntiles - 1) * 16 * g.ffn * 2;
  const uint32_t a_off = ((uint32_t)r * g.ffn + s_beg * 32 + kg * 8) * 2;
  // token column r contributes only if the token is routed to this expert (gate != 0)
  const bool live = r < g.T && g.slot_gate[u * kGateCols + r] != 0.f;
  const size_t hrow = ((size_t)u * g.max_tokens + min(r, g.T - 1)) * g.ffn;
  const char* HH = reinterpret_cast<const char*>(g.h_hi + hrow);
  const char* HL = reinterpret_cast<const char*>(g.h_lo + hrow);
  const uint32_t b_off = (uint32_t)(s_beg * 32 + kg * 8) * 2;

  f32x4 acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<R, P>(
      nst,
      [&](Stage<R>& st, int s) {
        const uint32_t ko = (uint32_t)s * 64;
#pragma unroll
        for (int j = 0; j < R; ++j) st.a[j] = ld128(base[j], a_off + ko);
        st.bh = uint4{0u, 0u, 0u, 0u};
        st.bl = uint4{0u, 0u, 0u, 0u};
        if (live) {
          st.bh = ld128(HH, b_off + ko);
          st.bl = ld128(HL, b_off + ko);
        }
      },
      [&](const Stage<R>& st) {
#pragma unroll
        for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], st.bh, acc[j]);
#pragma unroll
        for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], st.bl, acc[j]);
      });

#pragma unroll
  for (int j = 0; j < R; ++j) red[(wave * R + j) * 64 + lane] = float4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
  __syncthreads();
  for (int j = wave; j < R; j += W) {
    if (tile0 + j >= ntiles) break;
    float4 y = red[j * 64 + lane];
    for (int w = 1; w < W; ++w) {
      const float4 y2 = red[(w * R + j) * 64 + lane];
      y.x += y2.x, y.y += y2.y, y.z += y2.z, y.w += y2.w;
    }
    if (r < g.T) {
      const size_t o = (((size_t)u * g.KS + ks) * g.max_tokens + r) * g.d + (size_t)(tile0 + j) * 16 + kg * 4;
      *reinterpret_cast<float4*>(g.partial + o) = y;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 5: combine.  out[t,c] = sum over live slabs (routed slots ascending, then shared), fixed order.
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
  int gu_R, dn_R, dn_KS;  // launch plan
  char* ws;
  size_t ws_bytes;
  uint16_t *xs_hi, *xs_lo, *h_hi, *h_lo;
  int32_t *ids, *unique, *n_unique, *count, *offset, *assign, *slot_expert;
  float *gates, *slot_gate, *partial;
  bool profiling;
  std::vector<hipEvent_t> events;  // 6 per profiled layer-step
};

namespace {

constexpr int kWaves = 4;  // waves per workgroup in the expert kernels
constexpr int kDepth = 2;  // pipeline depth

long plan_waves(int ntiles, int R, int parts, int min_slots) {
  return (long)((ntiles + R - 1) / R) * parts * min_slots;
}

// The grid must put enough waves on 256 CUs even when the fewest experts are live (T = 1), while
// keeping R (weight tiles that share one activation fragment) as large as possible.
void make_plan(moe_ctx* c) {
  const moe_shape& s = c->s;
  const int min_slots = s.top_k + s.n_shared;
  c->gu_R = 1;
  for (int R : {4, 2})
    if (plan_waves(s.ffn / 16, R, kWaves, min_slots) >= 1536) {
      c->gu_R = R;
      break;
    }
  // down: split K over KS workgroups x kWaves waves, every wave keeping >= 4 k-steps
  const int nsteps = s.ffn / 32;
  int ks_cap = 1;
  while (ks_cap < 16 && nsteps / (kWaves * ks_cap * 2) >= 4) ks_cap *= 2;
  c->dn_R = 1;
  c->dn_KS = ks_cap;
  for (int R : {4, 2, 1}) {
    int ks = 1;
    while (ks < ks_cap && plan_waves(s.d / 16, R, kWaves * ks, min_slots) < 2048) ks *= 2;
    if (plan_waves(s.d / 16, R, kWaves * ks, min_slots) >= 1536 || R == 1) {
      c->dn_R = R;
      c->dn_KS = ks;
      break;
    }
  }
  if (const char* env = getenv("MOE_PLAN")) {  // tuning override: "guR,dnR,dnKS"
    int a = 0, b = 0, k = 0;
    if (sscanf(env, "%d,%d,%d", &a, &b, &k) == 3 && (a == 1 || a == 2 || a == 4) && (b == 1 || b == 2 || b == 4) &&
        k >= 1 && k <= 64) {
      c->gu_R = a;
      c->dn_R = b;
      c->dn_KS = k;
    }
  }
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
  mark(c, st);
  hipLaunchKernelGGL(route_kernel, dim3(T), dim3(256), 0, st, hidden, router_w, s.d, s.n_experts, s.top_k, c->ids,
                     c->gates, ids, gates, c->xs_hi, c->xs_lo);
  mark(c, st);
  GroupOut ws{c->unique, c->n_unique, c->count, c->offset, c->assign};
  GroupOut user{unique, n_unique, nullptr, nullptr, nullptr};
  hipLaunchKernelGGL(group_kernel, dim3(1), dim3(256), 0, st, (const int32_t*)c->ids, (const float*)c->gates, T,
                     s.top_k, s.n_experts, ws, user, n_unique_extra, c->slot_expert, c->slot_gate);
  mark(c, st);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

template <int R>
void launch_gateup(const moe_ctx* c, const GateupArgs& a, hipStream_t st) {
  const dim3 grid((c->s.ffn / 16 + R - 1) / R, c->u_tot);
  hipLaunchKernelGGL((gateup_kernel<R, kWaves, kDepth>), grid, dim3(64 * kWaves), 0, st, a);
}
template <int R>
void launch_down(const moe_ctx* c, const DownArgs& a, hipStream_t st) {
  const dim3 grid((c->s.d / 16 + R - 1) / R, c->u_tot, c->dn_KS);
  hipLaunchKernelGGL((down_kernel<R, kWaves, kDepth>), grid, dim3(64 * kWaves), 0, st, a);
}

moe_status launch_experts(moe_ctx* c, const moe_layer_weights* w, int T, float* out, hipStream_t st) {
  const moe_shape& s = c->s;
  GateupArgs ga{w->w1, w->w3, w->sw1, w->sw3, c->xs_hi, c->xs_lo, c->n_unique, c->slot_expert, c->slot_gate,
                c->h_hi, c->h_lo, s.d, s.ffn, T, c->u_max, s.max_tokens};
  switch (c->gu_R) {
    case 4: launch_gateup<4>(c, ga, st); break;
    case 2: launch_gateup<2>(c, ga, st); break;
    default: launch_gateup<1>(c, ga, st); break;
  }
  mark(c, st);
  DownArgs da{w->w2, w->sw2, c->h_hi, c->h_lo, c->n_unique, c->slot_expert, c->slot_gate, c->partial,
              s.d, s.ffn, T, c->u_max, s.max_tokens, c->dn_KS};
  switch (c->dn_R) {
    case 4: launch_down<4>(c, da, st); break;
    case 2: launch_down<2>(c, da, st); break;
    default: launch_down<1>(c, da, st); break;
  }
  mark(c, st);
  const int n4 = T * (s.d / 4);
  hipLaunchKernelGGL(combine_kernel, dim3((n4 + 255) / 256), dim3(256), 0, st, (const float*)c->partial,
                     (const int32_t*)c->n_unique, out, s.d, T, c->u_max, s.n_shared, s.max_tokens, c->dn_KS);
  mark(c, st);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// kernels use 128-bit loads: every tensor base must be 16-byte aligned (rows are, since d, ffn % 32 == 0)
bool weights_ok(const moe_ctx* c, const moe_layer_weights* w) {
  if (!w || !w->router_w || !w->w1 || !w->w3 || !w->w2) return false;
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
  make_plan(c);

  const size_t A = (size_t)s.max_tokens * s.top_k;
  size_t off = 0;
  auto carve = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const size_t o_xh = carve((size_t)s.max_tokens * s.d * 2), o_xl = carve((size_t)s.max_tokens * s.d * 2);
  const size_t o_hh = carve((size_t)c->u_tot * s.max_tokens * s.ffn * 2);
  const size_t o_hl = carve((size_t)c->u_tot * s.max_tokens * s.ffn * 2);
  const size_t o_ids = carve(A * 4), o_gates = carve(A * 4), o_uni = carve((size_t)s.n_experts * 4);
  const size_t o_nu = carve(4), o_cnt = carve((size_t)s.n_experts * 4), o_off = carve((size_t)(s.n_experts + 1) * 4);
  const size_t o_asg = carve(A * 4), o_se = carve((size_t)c->u_max * 4);
  const size_t o_sg = carve((size_t)c->u_tot * kGateCols * 4);
  const size_t o_part = carve((size_t)c->u_tot * c->dn_KS * s.max_tokens * s.d * 4);
  c->ws_bytes = off;
  if (hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return MOE_ERR_WORKSPACE;
  }
  c->xs_hi = reinterpret_cast<uint16_t*>(c->ws + o_xh);
  c->xs_lo = reinterpret_cast<uint16_t*>(c->ws + o_xl);
  c->h_hi = reinterpret_cast<uint16_t*>(c->ws + o_hh);
  c->h_lo = reinterpret_cast<uint16_t*>(c->ws + o_hl);
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
  // small tables start at zero; shared-expert slots carry gate 1 for every token column
  bool ok = hipMemset(c->ws + o_ids, 0, o_part - o_ids) == hipSuccess;
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
  GroupOut none{nullptr, nullptr, nullptr, nullptr, nullptr};
  GroupOut user{unique_experts, n_unique, expert_count, expert_offset, assign};
  hipLaunchKernelGGL(group_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, ids, (const float*)nullptr, T,
                     c->s.top_k, c->s.n_experts, none, user, (int32_t*)nullptr, (int32_t*)nullptr, (float*)nullptr);
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

moe_status moe_ctx_profile(moe_ctx* c, int32_t enable) {
  if (!c) return MOE_ERR_INVALID_ARG;
  c->profiling = enable != 0;
  return MOE_OK;
}

moe_status moe_ctx_profile_read(moe_ctx* c, double* ms_sum, int64_t* steps) {
  if (!c || !ms_sum || !steps) return MOE_ERR_INVALID_ARG;
  for (int i = 0; i < 5; ++i) ms_sum[i] = 0.0;
  const size_t n = c->events.size() / 6;
  moe_status rc = MOE_OK;
  if (n > 0 && hipEventSynchronize(c->events[n * 6 - 1]) != hipSuccess) rc = MOE_ERR_HIP;
  for (size_t i = 0; i < n && rc == MOE_OK; ++i)
    for (int k = 0; k < 5; ++k) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, c->events[i * 6 + k], c->events[i * 6 + k + 1]) != hipSuccess) rc = MOE_ERR_HIP;
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
