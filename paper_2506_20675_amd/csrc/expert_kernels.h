// Steps 3 to 5: gate/up projection with SiLU*mul, split-K down projection, slab sum; and the one-off re-layout
// kernels of the tiled weight format.  Part of the single translation unit moe_kernels.hip.
#pragma once
#include "moe_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Step 5: out[t] = sum over the token's own picks i = 0 .. top_k-1 (the slot each landed in comes from
// the grouping step), then the shared experts; k-chunks ascending inside each.  A fixed order — the
// order of the defining sum — so reruns are bit-identical and no floating-point atomics are needed.
// ------------------------------------------------------------------------------------------
struct CombineArgs {
  const float* partial;      // [(u_max + n_shared) * KS, max_tokens, d] slabs of the down projection
  const int32_t* tok_slot;   // [T, top_k]
  float* out;                // [T, d]
  int d, T, top_k, u_max, n_shared, max_tokens, KS;
};

// float4 number i of out[T, d]
__device__ __forceinline__ void combine_one(const CombineArgs& g, int i) {
  const int per_tok = g.d >> 2;
  const int t = i / per_tok, c4 = i - t * per_tok;
  float4 s = float4{0.f, 0.f, 0.f, 0.f};
  const size_t slab = (size_t)g.max_tokens * g.d;
  const float* p0 = g.partial + (size_t)t * g.d + (size_t)c4 * 4;
  // flat walk over (pick, k-chunk): unrolled by 8 so that eight slab loads are in flight at a time
  const int n = (g.top_k + g.n_shared) * g.KS;
#pragma unroll 8
  for (int q = 0; q < n; ++q) {
    const int j = q / g.KS, k = q - j * g.KS;
    const int u = j < g.top_k ? g.tok_slot[t * g.top_k + j] : g.u_max + (j - g.top_k);
    const float4 v = *reinterpret_cast<const float4*>(p0 + ((size_t)u * g.KS + k) * slab);
    s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
  }
  *reinterpret_cast<float4*>(g.out + (size_t)t * g.d + (size_t)c4 * 4) = s;
}

__global__ __launch_bounds__(256) void combine_kernel(CombineArgs g) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < g.T * (g.d >> 2)) combine_one(g, i);
}

// ------------------------------------------------------------------------------------------
// Step 3: gate/up projections + SiLU*mul for every unique expert (and shared expert).
// grid = (row blocks of 16*R rows of ffn, min(E, T*top_k) + n_shared slots); block = W waves that split d.
// With cmb_rows = 1 the grid has one more row in front, y = 0, whose workgroups do not project anything: they sum
// the slabs another layer's down projection left (`cmb`) — independent work that then needs no launch of its
// own.  That row is dispatched first and is done within a couple of microseconds.
// ------------------------------------------------------------------------------------------
struct GateupArgs {
  const void *w1, *w3, *sw1, *sw3;      // [E,ffn,d] / [n_shared,ffn,d], bf16 or FP8 codes
  const float *s1, *s3, *ss1, *ss3;     // FP8 only: per-row scales [E,ffn] / [n_shared,ffn]
  const uint16_t *xf_hi, *xf_lo;        // activation fragments, d*16 elements each
  const int32_t* n_unique;              // [1]        size of the union                   } written by the
  const int32_t* slot_expert;           // [u_max]    expert of slot u (ascending)        } grouping step
  const int32_t* slot_mask;             // [u_max]    bit t set: token t is routed to slot u
  const float* slot_gate;               // [u_max+n_shared, 16] gate of token column n
  uint16_t *hf_hi, *hf_lo;              // [u_max + n_shared] fragments of gate*silu(G)*U, ffn*16 elements each
  int d, ffn, T, routed_slots, u_max;   // routed_slots = min(E, T*top_k) slots in this grid
  int cmb_rows;                         // 0, or 1: row y = 0 of the grid runs the slab sum `cmb`
  int h_cols;                           // 0: H in the regular fragment layout; 2 T: compact packed layout (see frag_unit_compact)
  CombineArgs cmb;
};

template <int R, int W, int P, bool TILED, bool NT, bool FP8, bool PK>
__global__ __launch_bounds__(64 * W) void gateup_kernel(GateupArgs g) {
  constexpr int NB = FP8 ? 2 : 1;
  __shared__ float4 red[W > 1 ? W * 2 * R * 64 : 1];
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const char *W1, *W3;
  const float *S1 = nullptr, *S3 = nullptr;  // FP8: scale rows of this expert
  const size_t per = (size_t)g.ffn * g.d * (FP8 ? 1 : 2);
  float gate;
  bool routed;  // token column r's token goes through this expert (its gate may still be 0 after underflow)
  const int col = PK ? (r & (kPackedTokens - 1)) : r;
  int slot = (int)blockIdx.y - g.cmb_rows;  // slot of the union, or routed_slots + s for shared expert s
  if (slot < 0) {  // the slab-sum row: uniform over the workgroup
    const int n4 = g.cmb.T * (g.cmb.d >> 2);
    for (int i = blockIdx.x * (64 * W) + tid; i < n4; i += gridDim.x * (64 * W)) combine_one(g.cmb, i);
    return;
  }
  if (slot < g.routed_slots) {
    // independent loads (one round trip); the tables are in bounds for every slot of the grid
    const int nu = *g.n_unique;
    const int e = g.slot_expert[slot];
    gate = g.slot_gate[slot * kGateCols + col];
    routed = (g.slot_mask[slot] >> col) & 1;
    if (slot >= nu) return;  // beyond the union of this step
    W1 = reinterpret_cast<const char*>(g.w1) + e * per;
    W3 = reinterpret_cast<const char*>(g.w3) + e * per;
    if constexpr (FP8) {
      S1 = g.s1 + (size_t)e * g.ffn;
      S3 = g.s3 + (size_t)e * g.ffn;
    }
  } else {
    gate = 1.f;  // shared expert: every token, gate 1
    routed = true;
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
  uint32_t b_off[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) b_off[b] = frag_lane_off<TILED, FP8>(r, kg, lane, b);

  f32x4 acc[2 * R];
#pragma unroll
  for (int j = 0; j < 2 * R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<2 * R, NB, PK, P>(
      nst,
      [&](Stage<2 * R, NB, PK>& st, int s) {
#pragma unroll
        for (int j = 0; j < 2 * R; ++j)
          st.a[j] = ld128<NT>(base[j], wa.lane_off + (uint32_t)s * wa.step_stride);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          st.bh[b] = ld128<false>(XH, b_off[b] + (uint32_t)s * (NB * 1024));
          if constexpr (!PK) st.bl[b] = ld128<false>(XL, b_off[b] + (uint32_t)s * (NB * 1024));
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
    if (r < g.T && (!PK || r < kPackedTokens) && routed) {
      // lane holds rows 4*kg .. 4*kg+3 of the tile for token column r: four consecutive k of the
      // down projection, i.e. one half of a 16-byte fragment unit
      uint16_t hi[4], lo[4];
      split_bf16(gate * (G.x / (1.f + expf(-G.x))) * U.x, hi[0], lo[0]);
      split_bf16(gate * (G.y / (1.f + expf(-G.y))) * U.y, hi[1], lo[1]);
      split_bf16(gate * (G.z / (1.f + expf(-G.z))) * U.z, hi[2], lo[2]);
      split_bf16(gate * (G.w / (1.f + expf(-G.w))) * U.w, hi[3], lo[3]);
      const int k = (tile0 + j) * 16 + kg * 4;
      size_t o = frag_unit(k >> 3, r) * 8 + (k & 4), o_lo = o + kPackedTokens * 8;
      if (PK && g.h_cols) {  // the fused down + combine kernel reads the compact layout
        o = frag_unit_compact(k >> 3, r, g.h_cols) * 8 + (k & 4);
        o_lo = o + (size_t)(g.h_cols >> 1) * 8;
      }
      *reinterpret_cast<uint2*>(HH + o) =
          uint2{(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
      *reinterpret_cast<uint2*>(PK ? HH + o_lo : HL + o) =
          uint2{(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
    }
  }
}

// ------------------------------------------------------------------------------------------
// Step 4: down projection, split-K over (expert, k-chunk).  The gate is already folded into H, so
// every slab is a plain partial sum of out.
// grid = (row blocks of 16*R rows of d, KS k-chunks, min(E, T*top_k) + n_shared slots); block = W waves
// splitting the chunk.
// ------------------------------------------------------------------------------------------
struct DownArgs {
  const void *w2, *sw2;           // [E,d,ffn] / [n_shared,d,ffn], bf16 or FP8 codes
  const float *s2, *ss2;          // FP8 only: per-row scales [E,d] / [n_shared,d]
  const uint16_t *hf_hi, *hf_lo;  // [u_max + n_shared] fragments, ffn*16 elements each
  const int32_t* n_unique;
  const int32_t* slot_expert;
  const int32_t* slot_mask;
  float* partial;                 // [(u_max + n_shared)*KS, max_tokens, d]
  int d, ffn, T, routed_slots, u_max, max_tokens, KS;
};

template <int R, int W, int P, bool TILED, bool NT, bool FP8, bool PK>
__global__ __launch_bounds__(64 * W) void down_kernel(DownArgs g) {
  constexpr int NB = FP8 ? 2 : 1;
  __shared__ float4 red[W > 1 ? W * R * 64 : 1];
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63, r = lane & 15, kg = lane >> 4;
  // the slot is the slowest grid index: workgroups are dispatched in index order, so those of slots beyond the
  // union (they read the union's size and exit) come after all the live ones instead of between them
  const int ks = blockIdx.y;
  int slot = blockIdx.z;
  const char* W2;
  const float* S2 = nullptr;
  const size_t per = (size_t)g.ffn * g.d * (FP8 ? 1 : 2);
  bool live;  // token column r contributes only if the token is routed to this expert
  if (slot < g.routed_slots) {
    const int nu = *g.n_unique;  // three independent loads, one round trip
    const int e = g.slot_expert[slot];
    // clear also for the padded columns r >= T; packed: column n + 8 belongs to token n
    live = (g.slot_mask[slot] >> (PK ? (r & (kPackedTokens - 1)) : r)) & 1;
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
  uint32_t b_off[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) b_off[b] = frag_lane_off<TILED, FP8>(r, kg, lane, b);

  f32x4 acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  pipeline<R, NB, PK, P>(
      nst,
      [&](Stage<R, NB, PK>& st, int s) {
#pragma unroll
        for (int j = 0; j < R; ++j)
          st.a[j] = ld128<NT>(base[j], wa.lane_off + (uint32_t)s * wa.step_stride);
        // The fragment loads are unconditional although H of a token that was not routed here was never written
        // (the address is inside the workspace, the value is whatever an earlier call left): a load under a
        // per-lane condition makes the compiler count on the smaller number of loads in flight and halves the
        // effective prefetch depth.  The unrouted columns are masked to zero where they are consumed.
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          st.bh[b] = ld128<false>(HH, b_off[b] + (uint32_t)s * (NB * 1024));
          if constexpr (!PK) st.bl[b] = ld128<false>(HL, b_off[b] + (uint32_t)s * (NB * 1024));
        }
      },
      [&](const Stage<R, NB, PK>& st) {
        uint4 bh[NB], bl[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          bh[b] = live ? st.bh[b] : uint4{0u, 0u, 0u, 0u};
          if constexpr (!PK) bl[b] = live ? st.bl[b] : uint4{0u, 0u, 0u, 0u};
        }
        if constexpr (FP8) {
#pragma unroll
          for (int j = 0; j < R; ++j) {
            uint4 k0, k1;
            fp8x16_to_bf16(st.a[j], k0, k1);
            acc[j] = mfma_bf16(k0, bh[0], acc[j]);
            if constexpr (!PK) acc[j] = mfma_bf16(k0, bl[0], acc[j]);
            acc[j] = mfma_bf16(k1, bh[1], acc[j]);
            if constexpr (!PK) acc[j] = mfma_bf16(k1, bl[1], acc[j]);
          }
        } else {
#pragma unroll
          for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], bh[0], acc[j]);
          if constexpr (!PK) {
#pragma unroll
            for (int j = 0; j < R; ++j) acc[j] = mfma_bf16(st.a[j], bl[0], acc[j]);
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
// Steps 4 + 5 in one launch, for steps with few tokens in flight: one workgroup of 16 waves per 16-row tile of d
// walks ALL live slots.  The waves take (slot, k-chunk)
// items round-robin; because the gate is already folded into H and the columns of unrouted tokens are masked to
// zero, every item simply adds into the wave's one accumulator tile, so the sum over a token's experts — the
// combine — happens in registers, the 16 waves meet in LDS in a fixed order, and out[t] is written directly:
// no slabs, no combine launch.  One row tile per wave means one H fragment byte per weight byte where the split-K
// kernel above shares each fragment among 4 row tiles; that is affordable because this kernel takes H in the compact
// packed layout (frag_unit_compact: 2 T columns instead of 16), and it is why the kernel is used up to T = 5 or 6
// only.   grid = d / 16.
// halves = 2 (when d / 16 alone would leave compute units without a workgroup): two workgroups per tile, each
// owning 8 of its 16 rows.  A lane whose row belongs to the other workgroup loads the address of its partner lane
// (row r ^ 8) instead — the same 16 bytes, so the pair costs one request and the workgroup fetches only its own 128-byte
// pieces of each 1 KB block — and the matrix core then computes that row twice; output row i depends on weight row
// i alone, so the rows a workgroup owns are exactly what the other variant computes, and only those are stored.
// grid = d / 16 * halves.
// ------------------------------------------------------------------------------------------
struct DownFusedArgs {
  const void *w2, *sw2;
  const float *s2, *ss2;
  const uint16_t *hf_hi, *hf_lo;
  const int32_t* n_unique;
  const int32_t* slot_expert;
  const int32_t* slot_mask;
  float* out;  // [T, d]
  int d, ffn, T, n_shared, u_max, C;  // C = k-chunks per slot
  int halves;                         // 1 or 2 workgroups per 16-row tile
  int h_cols;                         // 0: H in the regular fragment layout; 2 T: compact packed layout
};

constexpr int kFusedWaves = 16;

template <int P, bool FP8, bool PK>
__global__ __launch_bounds__(64 * kFusedWaves) void down_fused_kernel(DownFusedArgs g) {
  constexpr int NB = FP8 ? 2 : 1;
  __shared__ float4 red[kFusedWaves * 64];
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const int col = PK ? (r & (kPackedTokens - 1)) : r;
  const int tile = g.halves == 2 ? blockIdx.x >> 1 : blockIdx.x, half = blockIdx.x & 1;
  const int r_load = g.halves == 2 ? (r & 7) | (half << 3) : r;  // the row whose weights this lane loads
  const bool own = g.halves != 2 || (kg >> 1) == half;           // the lane's output rows 4 kg .. 4 kg + 3 are this workgroup's
  const size_t per = (size_t)g.ffn * g.d * (FP8 ? 1 : 2);
  const int nu = *g.n_unique, n_items = (nu + g.n_shared) * g.C;
  const int nsteps = g.ffn >> (FP8 ? 6 : 5), chunk = (nsteps + g.C - 1) / g.C;
  const WeightAddr<true, FP8> wa(g.ffn, r_load, kg, kg * 16 + r_load);
  // Fragment addressing: regular layout = 1 KB per k-step, lane l at byte 16 l.  Compact packed layout (PK only):
  // 2 T columns per k-group instead of 16 — this kernel fetches one fragment byte per weight byte, and at small T
  // most of a regular fragment is padding.  A lane of a padding column reads a live column's unit again (same
  // address, no extra request); its MFMA column is never stored.
  uint32_t b_off = lane * 16, kstep_bytes = 1024;
  if constexpr (PK) {
    if (g.h_cols) {
      const int Tn = g.h_cols >> 1, t = min(r & (kPackedTokens - 1), Tn - 1);
      b_off = (uint32_t)(kg * g.h_cols + (r < kPackedTokens ? t : Tn + t)) * 16;
      kstep_bytes = 64u * g.h_cols;
    }
  }
  f32x4 total = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int item = wave; item < n_items; item += kFusedWaves) {
    const int sl = item / g.C, c = item - sl * g.C;
    const char* W2;
    const float* S2 = nullptr;
    int hslot;
    bool live;
    if (sl < nu) {
      const int e = g.slot_expert[sl];
      live = (g.slot_mask[sl] >> col) & 1;
      W2 = reinterpret_cast<const char*>(g.w2) + e * per;
      if constexpr (FP8) S2 = g.s2 + (size_t)e * g.d;
      hslot = sl;
    } else {
      const int sh = sl - nu;
      live = col < g.T;
      W2 = reinterpret_cast<const char*>(g.sw2) + sh * per;
      if constexpr (FP8) S2 = g.ss2 + (size_t)sh * g.d;
      hslot = g.u_max + sh;
    }
    const int nst = max(0, min(chunk, nsteps - c * chunk));
    const int s_beg = min(c * chunk, nsteps - 1);
    const char* base = W2 + (size_t)tile * wa.tile_stride + (size_t)s_beg * wa.step_stride;
    const size_t h_off = (size_t)hslot * g.ffn * 32 + (size_t)s_beg * NB * (PK ? kstep_bytes : 1024u);
    const char* HH = reinterpret_cast<const char*>(g.hf_hi) + h_off;
    const char* HL = reinterpret_cast<const char*>(g.hf_lo) + h_off;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    pipeline<1, NB, PK, P>(
        nst,
        [&](Stage<1, NB, PK>& st, int s) {
          st.a[0] = ld128<true>(base, wa.lane_off + (uint32_t)s * wa.step_stride);
#pragma unroll
          for (int b = 0; b < NB; ++b) {  // unconditional loads, masked where consumed (as in down_kernel)
            if constexpr (PK) {
              st.bh[b] = ld128<false>(HH, b_off + (uint32_t)(s * NB + b) * kstep_bytes);
            } else {
              st.bh[b] = ld128<false>(HH, b_off + (uint32_t)(s * NB + b) * 1024);
              st.bl[b] = ld128<false>(HL, b_off + (uint32_t)(s * NB + b) * 1024);
            }
          }
        },
        [&](const Stage<1, NB, PK>& st) {
          uint4 bh[NB], bl[NB];
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            bh[b] = live ? st.bh[b] : uint4{0u, 0u, 0u, 0u};
            if constexpr (!PK) bl[b] = live ? st.bl[b] : uint4{0u, 0u, 0u, 0u};
          }
          if constexpr (FP8) {
            uint4 k0, k1;
            fp8x16_to_bf16(st.a[0], k0, k1);
            acc = mfma_bf16(k0, bh[0], acc);
            if constexpr (!PK) acc = mfma_bf16(k0, bl[0], acc);
            acc = mfma_bf16(k1, bh[1], acc);
            if constexpr (!PK) acc = mfma_bf16(k1, bl[1], acc);
          } else {
            acc = mfma_bf16(st.a[0], bh[0], acc);
            if constexpr (!PK) acc = mfma_bf16(st.a[0], bl[0], acc);
          }
        });
    if constexpr (FP8) {  // every slot has its own row scales: scale the item's sum before it joins the others
      const float4 c2 = *reinterpret_cast<const float4*>(S2 + tile * 16 + kg * 4);
      total[0] += acc[0] * c2.x, total[1] += acc[1] * c2.y, total[2] += acc[2] * c2.z, total[3] += acc[3] * c2.w;
    } else {
      total[0] += acc[0], total[1] += acc[1], total[2] += acc[2], total[3] += acc[3];
    }
  }
  red[wave * 64 + lane] = float4{total[0], total[1], total[2], total[3]};
  __syncthreads();
  if (wave != 0) return;
  float4 y = red[lane];
  for (int w = 1; w < kFusedWaves; ++w) {
    const float4 y2 = red[w * 64 + lane];
    y.x += y2.x, y.y += y2.y, y.z += y2.z, y.w += y2.w;
  }
  if constexpr (PK)
    y.x += __shfl_xor(y.x, 8), y.y += __shfl_xor(y.y, 8), y.z += __shfl_xor(y.z, 8), y.w += __shfl_xor(y.w, 8);
  if (own && r < g.T && (!PK || r < kPackedTokens))
    *reinterpret_cast<float4*>(g.out + (size_t)r * g.d + (size_t)tile * 16 + kg * 4) = y;
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

}  // namespace
