/*
 * Driver for the sanitizer build of the CPU oracle (tests/test_oracle_sanitizers.py).
 *
 * Linked together with oracle/moe_oracle.c under -fsanitize=address,undefined, it runs every
 * exported oracle function on a few small layers (among them top-k = all experts, experts without
 * rows, a bias, a shared expert, no tokens at all) and writes every output to a file, which the test
 * compares bit for bit with what the ordinary build of the oracle returns for the same inputs.
 * Inputs come from a counter-based formula that the test repeats in numpy; none of the layer's
 * arithmetic lives here.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_route(const float* x, const float* Wr, const float* bias, int T, int H, int E, int K, int renorm,
                  int32_t* ids, float* w, float* logits_out);
void oracle_permute(const int32_t* ids, int T, int K, int E, int32_t* offsets, int32_t* src_of_row,
                    int32_t* row_of_pair);
void oracle_gather(const float* x, const int32_t* src_of_row, int P, int K, int H, float* Xp);
void oracle_expert_group_forward(int lo, int hi, const float* Xp, const int32_t* offsets, const float* Wg,
                                 const float* Wu, const float* Wd, int P, int H, int E, int I, double* Yp);
void oracle_shared_forward(const float* x, const float* Wsg, const float* Wsu, const float* Wsd, const float* wgate,
                           int T, int H, int Is, double* S, double* sg);
void oracle_combine(const double* Yp, const int32_t* row_of_pair, const float* w, const double* S, const double* sg,
                    int T, int H, int K, double* out);
void oracle_residual_norm(const float* x, const double* y, int T, int H, double eps, float* out);
void oracle_token_forward(const int32_t* tok, int n, const float* x, const float* Wr, const float* bias,
                          const float* Wg, const float* Wu, const float* Wd, const float* Wsg, const float* Wsu,
                          const float* Wsd, const float* wgate, int H, int E, int K, int I, int Is, int renorm,
                          double* out, int32_t* ids_out, float* w_out);
int oracle_real_bytes(void);

/* value i of stream s: a multiple of 1/256 in [-1, 1), scaled; exact in float */
static float draw(uint32_t s, uint32_t i, float scale) {
  uint32_t v = (i + 1u) * 2654435761u + s * 40503u;
  v ^= v >> 15;
  v *= 2246822519u;
  v ^= v >> 13;
  return ((float)(int)(v & 511u) - 256.0f) * (1.0f / 256.0f) * scale;
}

static float* fill(uint32_t s, size_t n, float scale) {
  float* p = (float*)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) p[i] = draw(s, (uint32_t)i, scale);
  return p;
}

struct layer_case { int T, H, E, K, I, Is, renorm, bias, cut; };

int main(int argc, char** argv) {
  if (argc != 2 || oracle_real_bytes() != 8) return 2;
  FILE* f = fopen(argv[1], "wb");
  if (!f) return 3;
  const struct layer_case cases[] = {
      {16, 64, 8, 2, 128, 0, 0, 0, 3},  {33, 128, 12, 4, 64, 192, 1, 1, 5}, {5, 8, 3, 3, 16, 8, 0, 1, 1},
      {40, 72, 20, 1, 24, 0, 1, 0, 19}, {0, 64, 4, 2, 64, 64, 0, 1, 2},
  };
  for (size_t c = 0; c < sizeof cases / sizeof cases[0]; ++c) {
    const struct layer_case k = cases[c];
    const int T = k.T, H = k.H, E = k.E, K = k.K, I = k.I, Is = k.Is, P = T * K;
    const uint32_t s = (uint32_t)c * 16u;
    float* x = fill(s + 0, (size_t)T * H, 1.0f);
    float* Wr = fill(s + 1, (size_t)E * H, 0.125f);
    float* bias = k.bias ? fill(s + 2, (size_t)E, 2.0f) : NULL;
    float* Wg = fill(s + 3, (size_t)E * I * H, 0.125f);
    float* Wu = fill(s + 4, (size_t)E * I * H, 0.125f);
    float* Wd = fill(s + 5, (size_t)E * H * I, 0.125f);
    float* Wsg = Is ? fill(s + 6, (size_t)Is * H, 0.125f) : NULL;
    float* Wsu = Is ? fill(s + 7, (size_t)Is * H, 0.125f) : NULL;
    float* Wsd = Is ? fill(s + 8, (size_t)H * Is, 0.125f) : NULL;
    float* wgate = Is ? fill(s + 9, (size_t)H, 0.125f) : NULL;

    int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P ? P : 1));
    float* w = (float*)malloc(sizeof(float) * (size_t)(P ? P : 1));
    float* logits = (float*)malloc(sizeof(float) * (size_t)(T * E ? T * E : 1));
    int32_t* off = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t* src = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P ? P : 1));
    int32_t* rowp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P ? P : 1));
    float* Xp = (float*)malloc(sizeof(float) * (size_t)(P * H ? P * H : 1));
    double* Yp = (double*)calloc((size_t)(P * H ? P * H : 1), sizeof(double));
    double* S = (double*)malloc(sizeof(double) * (size_t)(T * H ? T * H : 1));
    double* sg = (double*)malloc(sizeof(double) * (size_t)(T ? T : 1));
    double* out = (double*)malloc(sizeof(double) * (size_t)(T * H ? T * H : 1));
    double* tout = (double*)malloc(sizeof(double) * (size_t)(T * H ? T * H : 1));
    int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T ? T : 1));
    int32_t* tids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P ? P : 1));
    float* tw = (float*)malloc(sizeof(float) * (size_t)(P ? P : 1));
    float* xn = (float*)malloc(sizeof(float) * (size_t)(T * H ? T * H : 1));

    oracle_route(x, Wr, bias, T, H, E, K, k.renorm, ids, w, logits);
    oracle_permute(ids, T, K, E, off, src, rowp);
    oracle_gather(x, src, P, K, H, Xp);
    oracle_expert_group_forward(k.cut, E, Xp, off, Wg, Wu, Wd, P, H, E, I, Yp);   /* two blocks, the later one first */
    oracle_expert_group_forward(0, k.cut, Xp, off, Wg, Wu, Wd, P, H, E, I, Yp);
    if (Is) oracle_shared_forward(x, Wsg, Wsu, Wsd, wgate, T, H, Is, S, sg);
    oracle_combine(Yp, rowp, w, Is ? S : NULL, Is ? sg : NULL, T, H, K, out);
    for (int t = 0; t < T; ++t) tok[t] = T - 1 - t;
    oracle_token_forward(tok, T, x, Wr, bias, Wg, Wu, Wd, Wsg, Wsu, Wsd, wgate, H, E, K, I, Is, k.renorm, tout, tids, tw);
    oracle_residual_norm(x, out, T, H, 1e-6, xn);

    fwrite(ids, sizeof(int32_t), (size_t)P, f);
    fwrite(w, sizeof(float), (size_t)P, f);
    fwrite(logits, sizeof(float), (size_t)T * E, f);
    fwrite(off, sizeof(int32_t), (size_t)E + 1, f);
    fwrite(src, sizeof(int32_t), (size_t)P, f);
    fwrite(rowp, sizeof(int32_t), (size_t)P, f);
    fwrite(Xp, sizeof(float), (size_t)P * H, f);
    fwrite(Yp, sizeof(double), (size_t)P * H, f);
    if (Is) fwrite(S, sizeof(double), (size_t)T * H, f);
    if (Is) fwrite(sg, sizeof(double), (size_t)T, f);
    fwrite(out, sizeof(double), (size_t)T * H, f);
    fwrite(tout, sizeof(double), (size_t)T * H, f);
    fwrite(tids, sizeof(int32_t), (size_t)P, f);
    fwrite(tw, sizeof(float), (size_t)P, f);
    fwrite(xn, sizeof(float), (size_t)T * H, f);

    free(x); free(Wr); free(bias); free(Wg); free(Wu); free(Wd); free(Wsg); free(Wsu); free(Wsd); free(wgate);
    free(ids); free(w); free(logits); free(off); free(src); free(rowp); free(Xp); free(Yp); free(S); free(sg);
    free(out); free(tout); free(tok); free(tids); free(tw); free(xn);
  }
  if (fclose(f) != 0) return 4;
  printf("sanitize_driver: %zu cases done\n", sizeof cases / sizeof cases[0]);
  return 0;
}
