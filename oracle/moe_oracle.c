/* moe_oracle.c — TEST INFRASTRUCTURE, not a product path.
 *
 * Plain, slow, single-threaded CPU statement of what one MoE layer computes when
 * a speculative-decoding verification step pushes T = K+1 tokens through it
 * (paper: Section 1, the "2 of 8 experts per token, up to 6 for three drafts"
 * example; Section 2.1, router + experts; Section 2.2, verification of the K
 * drafts in one target step; Section 2.4, unique experts grow with K).
 *
 * Verification is iso-accuracy (Section 2.2): every token must get exactly what
 * decoding it alone would give.  So the oracle is simply the textbook definition
 * of a top-k softmax-gated SwiGLU mixture applied row by row — no grouping, no
 * blocking, no reuse across tokens.  The paper does not spell the operator out;
 * the benchmark definition does: bias-free linear router, top-k on the logits,
 * gates = softmax over the selected logits, expert = w2 . (silu(w1 x) * (w3 x)),
 * optional always-on shared experts with gate 1.
 *
 * Precision: the file is compiled twice, REAL=float (the "plain fp32" oracle the
 * parity bar is stated against) and REAL=double (accuracy reference).  In BOTH
 * builds the router logits are accumulated in double: a product of an fp32
 * activation and a bf16 weight is exact in double, so the logit, and with it the
 * integer top-k decision, does not depend on summation order beyond ~1e-13
 * relative — this is the precision the HIP router also decides in.
 *
 * Only tests/, the smoke check and the bench's cpu_baseline leg may call this.
 * Shares no code with the HIP library.  Parity pins: see tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif

static REAL real_exp(REAL v) { return sizeof(REAL) == sizeof(float) ? (REAL)expf((float)v) : (REAL)exp((double)v); }

/* bf16 is the upper half of an IEEE fp32: widening is exact. */
static float bf16_widen(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

int oracle_real_bytes(void) { return (int)sizeof(REAL); }

/* Router logits, top-k and gates for T tokens (Section 2.1: a small gating network
 * selects a few experts per token; each token selects independently, Section 1).
 *   logit[t,e] = sum_j hidden[t,j] * router_w[e,j]          (double, j ascending)
 *   ids[t,0..top_k) = repeated arg-max of logit[t,.]; equal values -> lower expert index
 *   gates[t,i] = exp(l_i - l_0) / sum_i exp(l_i - l_0),  l_i = (REAL)logit[t, ids[t,i]]
 * logits_out may be NULL; otherwise [T,E] doubles.  Returns 0, or -1 on bad sizes. */
int oracle_route(const float* hidden, const uint16_t* router_w, int T, int d, int E, int top_k,
                 int32_t* ids, float* gates, double* logits_out) {
  if (T < 1 || d < 1 || E < 1 || top_k < 1 || top_k > E) return -1;
  double* logit = (double*)malloc(sizeof(double) * (size_t)E);
  char* taken = (char*)malloc((size_t)E);
  REAL* p = (REAL*)malloc(sizeof(REAL) * (size_t)top_k);
  for (int t = 0; t < T; ++t) {
    for (int e = 0; e < E; ++e) {
      double s = 0.0;
      for (int j = 0; j < d; ++j) s += (double)hidden[(size_t)t * d + j] * (double)bf16_widen(router_w[(size_t)e * d + j]);
      logit[e] = s;
      if (logits_out) logits_out[(size_t)t * E + e] = s;
    }
    memset(taken, 0, (size_t)E);
    for (int i = 0; i < top_k; ++i) {
      int best = -1;
      for (int e = 0; e < E; ++e)
        if (!taken[e] && (best < 0 || logit[e] > logit[best])) best = e;
      taken[best] = 1;
      ids[(size_t)t * top_k + i] = best;
    }
    REAL l0 = (REAL)logit[ids[(size_t)t * top_k]];
    REAL sum = 0;
    for (int i = 0; i < top_k; ++i) {
      p[i] = real_exp((REAL)logit[ids[(size_t)t * top_k + i]] - l0);
      sum += p[i];
    }
    for (int i = 0; i < top_k; ++i) gates[(size_t)t * top_k + i] = (float)(p[i] / sum);
  }
  free(logit);
  free(taken);
  free(p);
  return 0;
}

/* Union of activated experts and the per-expert token lists (Section 1 and 2.2: the
 * in-flight tokens collectively activate a larger set; that set is what is fetched).
 *   unique[0..n_unique) ascending distinct ids; count[e]; offset[e] = sum_{e'<e} count[e'];
 *   assign[offset[e] ..) = flat assignment indices a = t*top_k + i with ids[a] == e, ascending. */
int oracle_union(const int32_t* ids, int T, int top_k, int E, int32_t* unique, int32_t* n_unique,
                 int32_t* count, int32_t* offset, int32_t* assign) {
  int A = T * top_k, n = 0, pos = 0;
  for (int e = 0; e < E; ++e) {
    int c = 0;
    offset[e] = pos;
    for (int a = 0; a < A; ++a)
      if (ids[a] == e) {
        assign[pos++] = a;
        ++c;
      }
    count[e] = c;
    if (c > 0) unique[n++] = e;
  }
  offset[E] = pos;
  for (int i = n; i < E; ++i) unique[i] = -1;
  *n_unique = n;
  return pos == A ? 0 : -1; /* an id outside [0,E) leaves assignments unplaced */
}

/* One SwiGLU expert on one token: y = w2 . ( silu(w1 x) * (w3 x) ), silu(z) = z / (1 + exp(-z)).
 * w1, w3: [ffn, d]; w2: [d, ffn]; all bf16 row-major.  h: scratch [ffn].  Index-ascending sums in REAL. */
void oracle_expert_ffn(const float* x, const uint16_t* w1, const uint16_t* w3, const uint16_t* w2, int d, int ffn,
                       REAL* h, REAL* y) {
  for (int r = 0; r < ffn; ++r) {
    REAL g = 0, u = 0;
    const uint16_t* a = w1 + (size_t)r * d;
    const uint16_t* b = w3 + (size_t)r * d;
    for (int j = 0; j < d; ++j) g += (REAL)bf16_widen(a[j]) * (REAL)x[j];
    for (int j = 0; j < d; ++j) u += (REAL)bf16_widen(b[j]) * (REAL)x[j];
    h[r] = (g / ((REAL)1 + real_exp(-g))) * u;
  }
  for (int c = 0; c < d; ++c) {
    REAL s = 0;
    const uint16_t* a = w2 + (size_t)c * ffn;
    for (int r = 0; r < ffn; ++r) s += (REAL)bf16_widen(a[r]) * h[r];
    y[c] = s;
  }
}

/* Gate-weighted combine given a routing (ids, gates):
 *   out[t] = sum_{i<top_k} gates[t,i] * FFN_{ids[t,i]}(x_t)   (slot order)
 *            + sum_{s<n_shared} FFN_shared_s(x_t)             (gate 1, index order)
 * Each (token, slot) pair is evaluated on its own: no sharing of work between tokens. */
int oracle_combine(const float* hidden, int T, int d, int ffn, int E, int top_k, int n_shared,
                   const uint16_t* w1, const uint16_t* w3, const uint16_t* w2,
                   const uint16_t* sw1, const uint16_t* sw3, const uint16_t* sw2,
                   const int32_t* ids, const float* gates, float* out) {
  REAL* h = (REAL*)malloc(sizeof(REAL) * (size_t)ffn);
  REAL* y = (REAL*)malloc(sizeof(REAL) * (size_t)d);
  REAL* acc = (REAL*)malloc(sizeof(REAL) * (size_t)d);
  const size_t per = (size_t)ffn * d;
  int rc = 0;
  for (int t = 0; t < T && rc == 0; ++t) {
    const float* x = hidden + (size_t)t * d;
    for (int c = 0; c < d; ++c) acc[c] = 0;
    for (int i = 0; i < top_k; ++i) {
      int e = ids[(size_t)t * top_k + i];
      if (e < 0 || e >= E) { rc = -1; break; }
      oracle_expert_ffn(x, w1 + e * per, w3 + e * per, w2 + e * per, d, ffn, h, y);
      REAL g = (REAL)gates[(size_t)t * top_k + i];
      for (int c = 0; c < d; ++c) acc[c] += g * y[c];
    }
    for (int s = 0; s < n_shared; ++s) {
      oracle_expert_ffn(x, sw1 + s * per, sw3 + s * per, sw2 + s * per, d, ffn, h, y);
      for (int c = 0; c < d; ++c) acc[c] += y[c];
    }
    for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = (float)acc[c];
  }
  free(h);
  free(y);
  free(acc);
  return rc;
}

/* The whole layer: route, then combine.  ids/gates are outputs. */
int oracle_layer(const float* hidden, int T, int d, int ffn, int E, int top_k, int n_shared,
                 const uint16_t* router_w, const uint16_t* w1, const uint16_t* w3, const uint16_t* w2,
                 const uint16_t* sw1, const uint16_t* sw3, const uint16_t* sw2,
                 int32_t* ids, float* gates, float* out) {
  int rc = oracle_route(hidden, router_w, T, d, E, top_k, ids, gates, NULL);
  if (rc) return rc;
  return oracle_combine(hidden, T, d, ffn, E, top_k, n_shared, w1, w3, w2, sw1, sw3, sw2, ids, gates, out);
}

/* Dense masked form of the same layer: EVERY expert is evaluated for every token and
 * multiplied by M[t,e] = gate if e was selected, else 0; summed in expert-index order.
 * Differs from oracle_combine only in summation order; used to cross-check it. */
int oracle_dense_masked(const float* hidden, int T, int d, int ffn, int E, int top_k, int n_shared,
                        const uint16_t* w1, const uint16_t* w3, const uint16_t* w2,
                        const uint16_t* sw1, const uint16_t* sw3, const uint16_t* sw2,
                        const int32_t* ids, const float* gates, float* out) {
  REAL* h = (REAL*)malloc(sizeof(REAL) * (size_t)ffn);
  REAL* y = (REAL*)malloc(sizeof(REAL) * (size_t)d);
  REAL* acc = (REAL*)malloc(sizeof(REAL) * (size_t)d);
  const size_t per = (size_t)ffn * d;
  for (int t = 0; t < T; ++t) {
    const float* x = hidden + (size_t)t * d;
    for (int c = 0; c < d; ++c) acc[c] = 0;
    for (int e = 0; e < E; ++e) {
      REAL m = 0;
      for (int i = 0; i < top_k; ++i)
        if (ids[(size_t)t * top_k + i] == e) m = (REAL)gates[(size_t)t * top_k + i];
      oracle_expert_ffn(x, w1 + e * per, w3 + e * per, w2 + e * per, d, ffn, h, y);
      for (int c = 0; c < d; ++c) acc[c] += m * y[c];
    }
    for (int s = 0; s < n_shared; ++s) {
      oracle_expert_ffn(x, sw1 + s * per, sw3 + s * per, sw2 + s * per, d, ffn, h, y);
      for (int c = 0; c < d; ++c) acc[c] += y[c];
    }
    for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = (float)acc[c];
  }
  free(h);
  free(y);
  free(acc);
  return 0;
}

/* ---------------------------------------------------------------------------------------------
 * FP8 expert weights (paper: Table 1 lists the Mixtral, Phi-3.5 and OLMoE checkpoints as FP8;
 * Section 6.1, quantised models).  The paper does not define the format or the scaling; the
 * reading taken here: weights are stored as 8-bit E4M3 codes with one fp32 scale per OUTPUT
 * channel (row of the matrix), the effective weight is W[r][j] = scale[r] * value(code[r][j]),
 * activations and arithmetic stay as in the bf16 layer, the router stays bf16.
 *
 * E4M3 as published for FP8 training/inference ("FP8 formats for deep learning", the OCP 8-bit
 * floating point specification): 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits;
 * exponent field 0 is subnormal (m/8 * 2^-6); there are no infinities; S.1111.111 is NaN; the
 * largest finite value is S.1111.110 = 1.75 * 2^8 = 448.
 * --------------------------------------------------------------------------------------------- */
double oracle_fp8_e4m3_value(uint8_t code) {
  const int sign = code >> 7, ex = (code >> 3) & 15, man = code & 7;
  double v;
  if (ex == 15 && man == 7) return NAN;
  if (ex == 0)
    v = ldexp((double)man / 8.0, -6);
  else
    v = ldexp(1.0 + (double)man / 8.0, ex - 7);
  return sign ? -v : v;
}

/* One SwiGLU expert with FP8 weights: as oracle_expert_ffn, with every weight replaced by
 * scale[row] * value(code).  q1, q3: [ffn, d] codes, s1, s3: [ffn]; q2: [d, ffn], s2: [d].
 * (The 256 code values are tabulated once per call only to keep the loops quick.) */
void oracle_expert_ffn_fp8(const float* x, const uint8_t* q1, const float* s1, const uint8_t* q3, const float* s3,
                           const uint8_t* q2, const float* s2, int d, int ffn, REAL* h, REAL* y) {
  REAL val[256];
  for (int c = 0; c < 256; ++c) val[c] = (REAL)oracle_fp8_e4m3_value((uint8_t)c);
  for (int r = 0; r < ffn; ++r) {
    REAL g = 0, u = 0;
    for (int j = 0; j < d; ++j) g += ((REAL)s1[r] * val[q1[(size_t)r * d + j]]) * (REAL)x[j];
    for (int j = 0; j < d; ++j) u += ((REAL)s3[r] * val[q3[(size_t)r * d + j]]) * (REAL)x[j];
    h[r] = (g / ((REAL)1 + real_exp(-g))) * u;
  }
  for (int c = 0; c < d; ++c) {
    REAL s = 0;
    for (int r = 0; r < ffn; ++r) s += ((REAL)s2[c] * val[q2[(size_t)c * ffn + r]]) * h[r];
    y[c] = s;
  }
}

/* Gate-weighted combine for a given routing, FP8 experts (same sum as oracle_combine).
 * q1, q3: [E, ffn, d]; q2: [E, d, ffn]; s1, s3: [E, ffn]; s2: [E, d]; shared experts likewise. */
int oracle_combine_fp8(const float* hidden, int T, int d, int ffn, int E, int top_k, int n_shared,
                       const uint8_t* q1, const uint8_t* q3, const uint8_t* q2,
                       const float* s1, const float* s3, const float* s2,
                       const uint8_t* sq1, const uint8_t* sq3, const uint8_t* sq2,
                       const float* ss1, const float* ss3, const float* ss2,
                       const int32_t* ids, const float* gates, float* out) {
  REAL* h = (REAL*)malloc(sizeof(REAL) * (size_t)ffn);
  REAL* y = (REAL*)malloc(sizeof(REAL) * (size_t)d);
  REAL* acc = (REAL*)malloc(sizeof(REAL) * (size_t)d);
  const size_t per = (size_t)ffn * d;
  int rc = 0;
  for (int t = 0; t < T && rc == 0; ++t) {
    const float* x = hidden + (size_t)t * d;
    for (int c = 0; c < d; ++c) acc[c] = 0;
    for (int i = 0; i < top_k; ++i) {
      int e = ids[(size_t)t * top_k + i];
      if (e < 0 || e >= E) { rc = -1; break; }
      oracle_expert_ffn_fp8(x, q1 + e * per, s1 + (size_t)e * ffn, q3 + e * per, s3 + (size_t)e * ffn,
                            q2 + e * per, s2 + (size_t)e * d, d, ffn, h, y);
      REAL g = (REAL)gates[(size_t)t * top_k + i];
      for (int c = 0; c < d; ++c) acc[c] += g * y[c];
    }
    for (int s = 0; s < n_shared; ++s) {
      oracle_expert_ffn_fp8(x, sq1 + s * per, ss1 + (size_t)s * ffn, sq3 + s * per, ss3 + (size_t)s * ffn,
                            sq2 + s * per, ss2 + (size_t)s * d, d, ffn, h, y);
      for (int c = 0; c < d; ++c) acc[c] += y[c];
    }
    for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = (float)acc[c];
  }
  free(h);
  free(y);
  free(acc);
  return rc;
}

/* The whole FP8 layer: the (bf16) router, then the FP8 combine. */
int oracle_layer_fp8(const float* hidden, int T, int d, int ffn, int E, int top_k, int n_shared,
                     const uint16_t* router_w,
                     const uint8_t* q1, const uint8_t* q3, const uint8_t* q2,
                     const float* s1, const float* s3, const float* s2,
                     const uint8_t* sq1, const uint8_t* sq3, const uint8_t* sq2,
                     const float* ss1, const float* ss3, const float* ss2,
                     int32_t* ids, float* gates, float* out) {
  int rc = oracle_route(hidden, router_w, T, d, E, top_k, ids, gates, NULL);
  if (rc) return rc;
  return oracle_combine_fp8(hidden, T, d, ffn, E, top_k, n_shared, q1, q3, q2, s1, s3, s2, sq1, sq3, sq2, ss1, ss3,
                            ss2, ids, gates, out);
}

/* ---------------------------------------------------------------------------------------------
 * Gate variant: softmax over ALL E logits, the selected probabilities used as they are (they sum
 * to less than 1).  Some of the Table 1 model families weight their picks this way instead of
 * renormalising over the picks; the paper does not say which, so both are offered.  Selection is
 * unchanged (same top-k, same tie rule):
 *   gates[t,i] = exp(l_{ids[t,i]} - m) / sum_{e<E} exp(l_e - m),   m = the largest logit of token t,
 * with l_e = (REAL)logit[t,e] and the sum taken in expert-index order.
 * --------------------------------------------------------------------------------------------- */
int oracle_route_softmax_all(const float* hidden, const uint16_t* router_w, int T, int d, int E, int top_k,
                             int32_t* ids, float* gates, double* logits_out) {
  if (T < 1 || d < 1 || E < 1 || top_k < 1 || top_k > E) return -1;
  double* logit = logits_out ? logits_out : (double*)malloc(sizeof(double) * (size_t)T * E);
  int rc = oracle_route(hidden, router_w, T, d, E, top_k, ids, gates, logit);
  for (int t = 0; t < T && rc == 0; ++t) {
    const double* l = logit + (size_t)t * E;
    const REAL m = (REAL)l[ids[(size_t)t * top_k]]; /* the first pick is the arg-max */
    REAL sum = 0;
    for (int e = 0; e < E; ++e) sum += real_exp((REAL)l[e] - m);
    for (int i = 0; i < top_k; ++i)
      gates[(size_t)t * top_k + i] = (float)(real_exp((REAL)l[ids[(size_t)t * top_k + i]] - m) / sum);
  }
  if (!logits_out) free(logit);
  return rc;
}

/* ---------------------------------------------------------------------------------------------
 * Chained decoder stack (the per-layer inputs are no longer independent: each MoE layer sits in a
 * pre-norm residual block, as in the Table 1 model families):
 *     n = RMSNorm(x) * gamma ;   x' = x + MoELayer(n)
 * RMSNorm of one token: n_j = x_j / sqrt( (1/d) sum_j x_j^2 + eps ) * gamma_j, gamma in bf16, the sum
 * taken in index order in REAL; n is rounded to fp32 because that is what the layer takes as hidden.
 * The paper's cost model needs no chaining (the expert-layer latency is what varies with K); the
 * chain is the alternative reading of how layer l+1 gets its input.
 * --------------------------------------------------------------------------------------------- */
void oracle_rmsnorm(const float* x, const uint16_t* gamma, int T, int d, double eps, float* y) {
  for (int t = 0; t < T; ++t) {
    const float* xt = x + (size_t)t * d;
    REAL ss = 0;
    for (int j = 0; j < d; ++j) ss += (REAL)xt[j] * (REAL)xt[j];
    const REAL mean = ss / (REAL)d;
    const REAL root = sizeof(REAL) == sizeof(float) ? (REAL)sqrtf((float)(mean + (REAL)eps)) : (REAL)sqrt((double)mean + eps);
    for (int j = 0; j < d; ++j) y[(size_t)t * d + j] = (float)(((REAL)xt[j] / root) * (REAL)bf16_widen(gamma[j]));
  }
}

/* x_out = x_in + delta, element by element in REAL, rounded to fp32 (the residual stream is fp32). */
void oracle_residual_add(const float* x_in, const float* delta, size_t n, float* x_out) {
  for (size_t i = 0; i < n; ++i) x_out[i] = (float)((REAL)x_in[i] + (REAL)delta[i]);
}

/* ---------------------------------------------------------------------------------------------
 * Attention stub of the chained decoder block.  The paper needs attention only as the part of an
 * iteration whose cost does NOT grow with K (Section 2.4: the expert layers are what grows; attention
 * is a small, constant share).  The stub is therefore the attention block's weight traffic with the
 * smallest arithmetic that is still attention: causal multi-head self-attention AMONG THE T IN-FLIGHT
 * TOKENS ONLY (no cache of earlier context, no positional rotation, no biases), grouped-query form:
 *   q_t = Wq n_t  [H heads x dh],   k_t = Wk n_t,  v_t = Wv n_t  [Hkv heads x dh]
 *   head h uses kv head h / (H / Hkv);  s_{t,u} = (q_t . k_u) / sqrt(dh) for u <= t
 *   p_{t,.} = softmax over u <= t;  o_t = sum_u p_{t,u} v_u;  a_t = Wo concat_h(o_t)
 * wqkv: [(H + 2 Hkv) dh, d] bf16, rows ordered q heads, then k heads, then v heads; wo: [d, H dh] bf16.
 * n: [T, d] fp32 (already normalised); out a: [T, d] fp32.  All sums in REAL, index order.
 * --------------------------------------------------------------------------------------------- */
int oracle_attention_stub(const float* n, const uint16_t* wqkv, const uint16_t* wo, int T, int d, int H, int Hkv,
                          int dh, float* a) {
  if (T < 1 || d < 1 || H < 1 || Hkv < 1 || dh < 1 || H % Hkv) return -1;
  const int nq = H * dh, nkv = Hkv * dh, nout = nq + 2 * nkv;
  REAL* qkv = (REAL*)malloc(sizeof(REAL) * (size_t)T * nout);
  REAL* o = (REAL*)malloc(sizeof(REAL) * (size_t)T * nq);
  REAL* p = (REAL*)malloc(sizeof(REAL) * (size_t)T);
  for (int t = 0; t < T; ++t)
    for (int r = 0; r < nout; ++r) {
      REAL s = 0;
      for (int j = 0; j < d; ++j) s += (REAL)bf16_widen(wqkv[(size_t)r * d + j]) * (REAL)n[(size_t)t * d + j];
      qkv[(size_t)t * nout + r] = s;
    }
  const REAL scale = (REAL)1 / (sizeof(REAL) == sizeof(float) ? (REAL)sqrtf((float)dh) : (REAL)sqrt((double)dh));
  for (int h = 0; h < H; ++h) {
    const int g = h / (H / Hkv);
    for (int t = 0; t < T; ++t) {
      const REAL* q = qkv + (size_t)t * nout + (size_t)h * dh;
      REAL m = 0;
      for (int u = 0; u <= t; ++u) {
        const REAL* k = qkv + (size_t)u * nout + nq + (size_t)g * dh;
        REAL s = 0;
        for (int j = 0; j < dh; ++j) s += q[j] * k[j];
        p[u] = s * scale;
        if (u == 0 || p[u] > m) m = p[u];
      }
      REAL sum = 0;
      for (int u = 0; u <= t; ++u) {
        p[u] = real_exp(p[u] - m);
        sum += p[u];
      }
      for (int j = 0; j < dh; ++j) {
        REAL acc = 0;
        for (int u = 0; u <= t; ++u) acc += (p[u] / sum) * qkv[(size_t)u * nout + nq + nkv + (size_t)g * dh + j];
        o[(size_t)t * nq + (size_t)h * dh + j] = acc;
      }
    }
  }
  for (int t = 0; t < T; ++t)
    for (int c = 0; c < d; ++c) {
      REAL s = 0;
      for (int j = 0; j < nq; ++j) s += (REAL)bf16_widen(wo[(size_t)c * nq + j]) * o[(size_t)t * nq + j];
      a[(size_t)t * d + c] = (float)s;
    }
  free(qkv);
  free(o);
  free(p);
  return 0;
}
