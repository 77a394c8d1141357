// Chained stack and decoder blocks: slab sum + residual + RMSNorm in one pass, the skinny projections and the
// per-head core of the attention stub.  Part of the single translation unit moe_kernels.hip.
#pragma once
#include "moe_common.h"
#include "route_kernels.h"

namespace {

// ------------------------------------------------------------------------------------------
// Chained stack: one workgroup per token finishes block l-1 and prepares block l in one pass over d:
//   x_l = x_{l-1} + (slabs of the token's picks, as in combine_kernel)      -> resid_out
//   n   = x_l / sqrt(mean(x_l^2) + eps) * gamma_l                           -> xn_out (the router's input)
// partial == NULL and moe_out == NULL: no MoE term (first block: x_0 is the caller's input); moe_out: the term is
// already summed.  gamma == NULL: no
// normalisation (after the last block only the residual stream is wanted).
// ------------------------------------------------------------------------------------------
struct ChainArgs {
  const float* moe_out;    // [T, d]: the MoE term already summed (fused down projection), or NULL
  const float* partial;
  const int32_t* tok_slot;
  const float* resid_in;   // [T, d] the stream the MoE term is added to
  float* resid_out;        // [T, d] or NULL
  const uint16_t* gamma;   // [d] bf16 or NULL
  float* xn_out;           // [T, d] fp32 normalised output, or NULL
  uint16_t *xf_hi, *xf_lo; // or: the normalised output as bf16 hi/lo fragments (MFMA B operand), or NULL
  int d, T, top_k, u_max, n_shared, max_tokens, KS;
  float eps;
};
constexpr int kChainThreads = 1024;
constexpr int kChainVecs = 4;  // float4 per thread: d <= 4 * 4 * 1024

// xs != NULL: the normalised row also goes there (LDS of the calling kernel, d floats).
__device__ __forceinline__ void chain_body(const ChainArgs& g, float* xs = nullptr) {
  __shared__ float s_ss[kChainThreads / 64];
  const int t = blockIdx.x, tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
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
      if (g.moe_out) m = *reinterpret_cast<const float4*>(g.moe_out + o);
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
      if (xs) *reinterpret_cast<float4*>(xs + (size_t)c4 * 4) = y;
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

__global__ __launch_bounds__(kChainThreads) void chain_kernel(ChainArgs g) { chain_body(g); }

// The same pass followed, in the same launch, by the router of the block it has just normalised for: both are one
// workgroup of 1024 threads per token, and the router reads exactly what this workgroup has written (c.xn_out ==
// r.hidden), so a workgroup barrier is all that lies between them.  Saves one launch per block in the chained stacks.
// Requires c.gamma != NULL.
static_assert(kChainThreads == 64 * kRouteWaves, "chain_route_kernel runs both bodies on one workgroup shape");
__global__ __launch_bounds__(kChainThreads) void chain_route_kernel(ChainArgs c, RouteArgs r, GroupArgs grp) {
  chain_body(c);
  __threadfence_block();
  __syncthreads();
  route_body(r, grp);
}

// In front of a wide router (logits_kernel: one workgroup per (token, 16 experts)) the same saving: every expert
// block of a token repeats the token's pass — a few KB of slabs and one row of the stream, L2 hits after the first
// block — keeps the normalised row in LDS and takes its logits from there; expert block 0 alone writes the pass's
// outputs.  Same arithmetic on the same values as chain_kernel followed by logits_kernel, so the same bits.
// Requires c.gamma != NULL and d <= kChainLogitsMaxD (the row must fit the LDS array).
constexpr int kChainLogitsMaxD = 8192;
__global__ __launch_bounds__(kChainThreads) void chain_logits_kernel(ChainArgs c, RouteArgs r, double* __restrict__ logits) {
  __shared__ __align__(16) float s_x[kChainLogitsMaxD];
  if (blockIdx.y != 0) c.resid_out = nullptr, c.xn_out = nullptr, c.xf_hi = nullptr, c.xf_lo = nullptr;
  chain_body(c, s_x);
  __syncthreads();
  logits_body<kChainThreads / 64>(r, logits, s_x);
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
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63, r = lane & 15, kg = lane >> 4;
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

}  // namespace
