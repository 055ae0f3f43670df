/*
 * CPU oracle for the routed-expert MoE layer forward (FaaSMoE, Sec. 2.1 "Mixture-of-Experts
 * Models" and Sec. 3 "Architecture").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a slow, plain statement of what the layer computes,
 * used only to check the GPU library and to time a CPU baseline.  Nothing in the product path
 * links, loads or calls it, and it shares no code with the GPU library.
 *
 * What the paper fixes: each MoE layer is a gating network that picks the top-k experts per
 * token plus a set of experts (Sec. 2.1); after gating the orchestrator gathers the tokens that
 * go to one expert block into one batched request, the block runs its experts statelessly on
 * those tokens, and the orchestrator aggregates the results (Sec. 3; Sec. 4.1 "token-level
 * micro-batching"); the block size must not change the result (Sec. 3).  The model is
 * Qwen1.5-MoE-2.7B with 60 routed and 4 shared experts per layer (Sec. 5 "Model Selection").
 * The paper prints no formula; the arithmetic below is the usual definition of that layer:
 *
 *   logit[t,e] = <x[t,:], Wr[e,:]> (+ bias[e])                           fp32
 *   p[t,:]     = softmax_e(logit[t,:])                                    fp32
 *   ids[t,0..K-1] = experts with the K largest logits, descending, equal logits -> lower id
 *   w[t,j]     = p[t, ids[t,j]]   (divided by their sum over j when renorm != 0)
 *   FFN_e(v)   = Wd[e] . ( silu(Wg[e].v) * (Wu[e].v) ),   silu(a) = a / (1 + exp(-a))
 *   out[t,:]   = sum_j w[t,j] FFN_{ids[t,j]}(x[t,:])  +  sigmoid(<x[t,:], wgate>) FFN_shared(x[t,:])
 *
 * Precision.  The routing decision is taken in fp32 with a fixed summation order (below), so
 * that another implementation can reproduce the logits bit for bit.  Everything downstream of
 * the decision (FFNs, gate of the shared expert, combine) is evaluated in `real`, which is
 * double unless the file is compiled with -DREAL=float.  No intermediate value is rounded to a
 * narrower type.
 *
 * Fixed order of the router dot product.  H must be a multiple of 8.  Element h belongs to
 * partial sum j = (h / 8) mod 64.  Each of the 64 partial sums starts at +0 and takes its
 * elements in ascending h with one fused multiply-add each.  The 64 partials are then folded by
 * a butterfly: for s = 1, 2, 4, 8, 16, 32 every partial j becomes a[j] + a[j xor s].  Addition
 * is commutative, so after the last stage all 64 hold the same value, which is the dot product.
 * The bias, if any, is added after that.
 *
 * Both forms of the layer are here: the per-token definition (oracle_token_forward) and the
 * path form the paper describes (route -> group tokens by expert -> per-block expert calls ->
 * aggregate), whose integer arrays a GPU implementation is compared with bit for bit.
 *
 * Parity pins live in tests/ (brute force in numpy, torch CPU library routines, closed forms).
 * The paper prints no numeric value for this path, so absolute values are pinned only by those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

int oracle_real_bytes(void) { return (int)sizeof(real); }

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* ---------------------------------------------------------------- gating (Sec. 2.1) ------ */

/* Dot product in the fixed order described in the header. */
static float router_dot(const float* x, const float* w, int H) {
  float a[64], b[64];
  for (int j = 0; j < 64; ++j) a[j] = 0.0f;
  for (int h = 0; h < H; ++h) {
    int j = (h >> 3) & 63;
    a[j] = fmaf(x[h], w[h], a[j]);
  }
  for (int s = 1; s <= 32; s <<= 1) {
    for (int j = 0; j < 64; ++j) b[j] = a[j] + a[j ^ s];
    memcpy(a, b, sizeof a);
  }
  return a[0];
}

/* Gating for one token.  logits: scratch of E floats (kept for the caller if wanted). */
static void route_token(const float* xt, const float* Wr, const float* bias, int H, int E, int K,
                        int renorm, float* logits, int32_t* ids, float* w) {
  for (int e = 0; e < E; ++e) {
    float l = router_dot(xt, Wr + (size_t)e * H, H);
    if (bias) l = l + bias[e];
    logits[e] = l;
  }
  float m = logits[0];
  for (int e = 1; e < E; ++e)
    if (logits[e] > m) m = logits[e];
  float sum = 0.0f;
  for (int e = 0; e < E; ++e) sum += expf(logits[e] - m);

  /* K rounds of argmax over the experts not taken yet; a strict '>' keeps the lowest id
   * among equal logits (and treats -0 and +0 as equal). */
  for (int j = 0; j < K; ++j) {
    int best = -1;
    for (int e = 0; e < E; ++e) {
      int taken = 0;
      for (int i = 0; i < j; ++i)
        if (ids[i] == e) taken = 1;
      if (taken) continue;
      if (best < 0 || logits[e] > logits[best]) best = e;
    }
    ids[j] = best;
    w[j] = expf(logits[best] - m) / sum;
  }
  if (renorm) {
    float s = 0.0f;
    for (int j = 0; j < K; ++j) s += w[j];
    for (int j = 0; j < K; ++j) w[j] = w[j] / s;
  }
}

/* x [T,H], Wr [E,H], bias [E] or NULL -> ids [T,K], w [T,K], logits [T,E] (or NULL). */
void oracle_route(const float* x, const float* Wr, const float* bias, int T, int H, int E, int K,
                  int renorm, int32_t* ids, float* w, float* logits_out) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    float* l = (float*)malloc(sizeof(float) * (size_t)E);
    route_token(x + (size_t)t * H, Wr, bias, H, E, K, renorm, l, ids + (size_t)t * K,
                w + (size_t)t * K);
    if (logits_out) memcpy(logits_out + (size_t)t * E, l, sizeof(float) * (size_t)E);
    free(l);
  }
}

/* ------------------------------------- micro-batch construction (Sec. 3, Sec. 4.1) ------ */

/* Stable counting sort of the P = T*K (token, slot) pairs by expert id.
 * offsets [E+1]: rows of expert e are offsets[e] .. offsets[e+1]-1.
 * row_of_pair [P]: row that pair p = t*K + j lands on.  src_of_row [P]: its inverse.
 * Inside one expert the rows keep ascending pair order. */
void oracle_permute(const int32_t* ids, int T, int K, int E, int32_t* offsets,
                    int32_t* src_of_row, int32_t* row_of_pair) {
  int P = T * K;
  for (int e = 0; e <= E; ++e) offsets[e] = 0;
  for (int p = 0; p < P; ++p) offsets[ids[p] + 1] += 1;
  for (int e = 0; e < E; ++e) offsets[e + 1] += offsets[e];
  int32_t* next = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
  for (int e = 0; e < E; ++e) next[e] = offsets[e];
  for (int p = 0; p < P; ++p) {
    int r = next[ids[p]]++;
    row_of_pair[p] = r;
    src_of_row[r] = p;
  }
  free(next);
}

/* Xp[r,:] = x[src_of_row[r] / K, :] */
void oracle_gather(const float* x, const int32_t* src_of_row, int P, int K, int H, float* Xp) {
  for (int r = 0; r < P; ++r)
    memcpy(Xp + (size_t)r * H, x + (size_t)(src_of_row[r] / K) * H, sizeof(float) * (size_t)H);
}

/* ------------------------------------------------ expert FFN (SwiGLU MLP, Sec. 5) ------ */

static real silu(real a) { return a / ((real)1 + (real)exp(-(double)a)); }

/* y[0..H) = Wd . ( silu(Wg.v) * (Wu.v) );  Wg, Wu [I,H], Wd [H,I]; hbuf: I reals of scratch. */
static void ffn_row(const float* v, const float* Wg, const float* Wu, const float* Wd, int H,
                    int I, real* hbuf, real* y) {
  for (int n = 0; n < I; ++n) {
    const float* wg = Wg + (size_t)n * H;
    const float* wu = Wu + (size_t)n * H;
    real g = 0, u = 0;
    for (int k = 0; k < H; ++k) {
      g += (real)v[k] * (real)wg[k];
      u += (real)v[k] * (real)wu[k];
    }
    hbuf[n] = silu(g) * u;
  }
  for (int m = 0; m < H; ++m) {
    const float* wd = Wd + (size_t)m * I;
    real acc = 0;
    for (int n = 0; n < I; ++n) acc += hbuf[n] * (real)wd[n];
    y[m] = acc;
  }
}

/* One expert-block invocation (Sec. 3): experts [lo,hi) each run on their own rows of Xp.
 * Xp [P,H]; Wg,Wu [E,I,H]; Wd [E,H,I]; Yp [P,H]: only rows offsets[lo]..offsets[hi]-1 are
 * written.  The block sees tokens only: no gate weight is applied here. */
void oracle_expert_group_forward(int lo, int hi, const float* Xp, const int32_t* offsets,
                                 const float* Wg, const float* Wu, const float* Wd, int P, int H,
                                 int E, int I, real* Yp) {
  (void)P;
  (void)E;
  for (int e = lo; e < hi; ++e) {
    const float* wg = Wg + (size_t)e * I * H;
    const float* wu = Wu + (size_t)e * I * H;
    const float* wd = Wd + (size_t)e * H * I;
#pragma omp parallel
    {
      real* hbuf = (real*)malloc(sizeof(real) * (size_t)I);
#pragma omp for schedule(dynamic, 1)
      for (int r = offsets[e]; r < offsets[e + 1]; ++r)
        ffn_row(Xp + (size_t)r * H, wg, wu, wd, H, I, hbuf, Yp + (size_t)r * H);
      free(hbuf);
    }
  }
}

/* Shared expert on every token: S [T,H] = FFN_shared(x[t]); sg[t] = <x[t], wgate> (raw, the
 * sigmoid is applied where the outputs are combined). */
void oracle_shared_forward(const float* x, const float* Wsg, const float* Wsu, const float* Wsd,
                           const float* wgate, int T, int H, int Is, real* S, real* sg) {
#pragma omp parallel
  {
    real* hbuf = (real*)malloc(sizeof(real) * (size_t)(Is > 0 ? Is : 1));
#pragma omp for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
      const float* xt = x + (size_t)t * H;
      ffn_row(xt, Wsg, Wsu, Wsd, H, Is, hbuf, S + (size_t)t * H);
      real a = 0;
      if (wgate)
        for (int k = 0; k < H; ++k) a += (real)xt[k] * (real)wgate[k];
      sg[t] = a;
    }
    free(hbuf);
  }
}

/* ------------------------------------------------------ aggregation (Sec. 3, 4.2) ------ */

/* out[t,:] = sum_{j ascending} w[t,j] * Yp[row_of_pair[t*K+j],:]  + sigmoid(sg[t]) * S[t,:]
 * S and sg may be NULL (no shared expert). */
void oracle_combine(const real* Yp, const int32_t* row_of_pair, const float* w, const real* S,
                    const real* sg, int T, int H, int K, real* out) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    real* o = out + (size_t)t * H;
    for (int m = 0; m < H; ++m) o[m] = 0;
    for (int j = 0; j < K; ++j) {
      const real* y = Yp + (size_t)row_of_pair[(size_t)t * K + j] * H;
      real wj = (real)w[(size_t)t * K + j];
      for (int m = 0; m < H; ++m) o[m] += wj * y[m];
    }
    if (S && sg) {
      real gate = (real)1 / ((real)1 + (real)exp(-(double)sg[t]));
      const real* s = S + (size_t)t * H;
      for (int m = 0; m < H; ++m) o[m] += gate * s[m];
    }
  }
}

/* ------------------------------------------------------ chaining layers (no attention) ------ */

/* Round to bf16 (8 significant bits, round to nearest even) and return the value as a float. */
static float round_bf16(real v) {
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return f;
}

/* u = x[t,:] + y[t,:];  out[t,:] = bf16( u / sqrt(mean_h(u^2) + eps) ): the residual add and RMS
 * normalisation (no learned scale) placed between two MoE layers when a stack of them is run
 * without attention.  x [T,H] float (bf16 values), y [T,H] real, out [T,H] float (bf16 values). */
void oracle_residual_norm(const float* x, const real* y, int T, int H, double eps, float* out) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    real ss = 0;
    for (int h = 0; h < H; ++h) {
      real u = (real)x[(size_t)t * H + h] + y[(size_t)t * H + h];
      ss += u * u;
    }
    real scale = (real)1 / (real)sqrt((double)(ss / (real)H) + eps);
    for (int h = 0; h < H; ++h) {
      real u = (real)x[(size_t)t * H + h] + y[(size_t)t * H + h];
      out[(size_t)t * H + h] = round_bf16(u * scale);
    }
  }
}

/* ---------------------------------------------------------- per-token definition ------ */

/* The layer output for the listed tokens, straight from the definition in the header: no
 * grouping, no permutation.  tok [n] token indices; out [n,H]; ids_out [n,K], w_out [n,K] may
 * be NULL.  Shared expert is skipped when Is == 0. */
void oracle_token_forward(const int32_t* tok, int n, const float* x, const float* Wr,
                          const float* bias, const float* Wg, const float* Wu, const float* Wd,
                          const float* Wsg, const float* Wsu, const float* Wsd,
                          const float* wgate, int H, int E, int K, int I, int Is, int renorm,
                          real* out, int32_t* ids_out, float* w_out) {
#pragma omp parallel
  {
    int Imax = I > Is ? I : Is;
    real* hbuf = (real*)malloc(sizeof(real) * (size_t)(Imax > 0 ? Imax : 1));
    real* y = (real*)malloc(sizeof(real) * (size_t)H);
    float* logits = (float*)malloc(sizeof(float) * (size_t)E);
    int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
    float* w = (float*)malloc(sizeof(float) * (size_t)K);
#pragma omp for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
      const float* xt = x + (size_t)tok[i] * H;
      real* o = out + (size_t)i * H;
      route_token(xt, Wr, bias, H, E, K, renorm, logits, ids, w);
      for (int m = 0; m < H; ++m) o[m] = 0;
      for (int j = 0; j < K; ++j) {
        int e = ids[j];
        ffn_row(xt, Wg + (size_t)e * I * H, Wu + (size_t)e * I * H, Wd + (size_t)e * H * I, H,
                I, hbuf, y);
        for (int m = 0; m < H; ++m) o[m] += (real)w[j] * y[m];
      }
      if (Is > 0) {
        ffn_row(xt, Wsg, Wsu, Wsd, H, Is, hbuf, y);
        real a = 0;
        if (wgate)
          for (int k = 0; k < H; ++k) a += (real)xt[k] * (real)wgate[k];
        real gate = (real)1 / ((real)1 + (real)exp(-(double)a));
        for (int m = 0; m < H; ++m) o[m] += gate * y[m];
      }
      if (ids_out) memcpy(ids_out + (size_t)i * K, ids, sizeof(int32_t) * (size_t)K);
      if (w_out) memcpy(w_out + (size_t)i * K, w, sizeof(float) * (size_t)K);
    }
    free(hbuf);
    free(y);
    free(logits);
    free(ids);
    free(w);
  }
}
