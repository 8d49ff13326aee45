/* Walks every entry point of the fp64 oracle on a small graph; built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py, which fails on any report.
 * The oracle's source is included, so that its static helpers are instrumented as well. */
#include "../../oracle/mggcn_ref.c"

#include <stdio.h>

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void) { /* xorshift: any deterministic numbers will do */
  state ^= state << 13; state ^= state >> 7; state ^= state << 17;
  return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}

#define CHECK(x) do { long long rc_ = (long long)(x); if (rc_ < 0) { printf("%s -> %lld\n", #x, rc_); return 1; } } while (0)

int main(void) {
  enum { n = 37, F = 9, C = 5, L = 3 };
  const int32_t dims[L + 1] = {F, 12, 7, C};
  /* ring + a hub + an isolated vertex, symmetric, sorted rows, no self-loops */
  int32_t rp[n + 1], ci[8 * n];
  int64_t nnz = 0;
  rp[0] = 0;
  for (int i = 0; i < n; ++i) {
    int32_t row[8]; int m = 0;
    if (i < n - 1) { /* vertex n-1 stays isolated */
      const int a = (i + n - 2) % (n - 1), b = (i + 1) % (n - 1);
      if (i != 0) row[m++] = 0;              /* hub 0 */
      if (a != i && a != 0) row[m++] = a;
      if (b != i && b != 0 && b != a) row[m++] = b;
      if (i == 0) { m = 0; for (int j = 1; j < n - 1 && m < 8; j += 5) row[m++] = j; }
    }
    for (int x = 0; x < m; ++x) for (int y = x + 1; y < m; ++y) if (row[y] < row[x]) { int32_t t = row[x]; row[x] = row[y]; row[y] = t; }
    for (int x = 0; x < m; ++x) ci[nnz++] = row[x];
    rp[i + 1] = (int32_t)nnz;
  }
  /* symmetrise by brute force so that the pattern is a valid undirected graph */
  static int adj[n][n];
  for (int i = 0; i < n; ++i) for (int k = rp[i]; k < rp[i + 1]; ++k) adj[i][ci[k]] = adj[ci[k]][i] = 1;
  nnz = 0;
  for (int i = 0; i < n; ++i) { for (int j = 0; j < n; ++j) if (adj[i][j] && i != j) ci[nnz++] = j; rp[i + 1] = (int32_t)nnz; }
  CHECK(mggcn_ref_csr_validate(n, n, rp, ci));

  int32_t rpo[n + 1], cio[9 * n], rpt[n + 1], cit[9 * n];
  double val[9 * n], valt[9 * n];
  for (int mode = 0; mode < 2; ++mode) {
    const int64_t m = mggcn_ref_csr_normalize(n, n, rp, ci, mode, NULL, NULL, rpo, cio, val);
    CHECK(m);
    CHECK(mggcn_ref_csr_transpose(n, n, rpo, cio, val, rpt, cit, valt));
  }
  CHECK(mggcn_ref_csr_normalize(n, n, rp, ci, REF_NORM_SYM, NULL, NULL, rpo, cio, val));

  double X[n * F], Y[n * F], Yt[n * F];
  for (int i = 0; i < n * F; ++i) { X[i] = rnd(); Y[i] = rnd(); Yt[i] = 0.0; }
  CHECK(mggcn_ref_spmm(REF_OP_N, n, n, rpo, cio, val, X, F, F, 1.0, Y, F));
  CHECK(mggcn_ref_spmm(REF_OP_T, n, n, rpo, cio, val, X, F, F - 2, 0.0, Yt, F));
  /* a rectangular block with given degrees */
  {
    enum { r = 5, c = 11 };
    const int32_t brp[r + 1] = {0, 2, 2, 5, 6, 8}, bci[8] = {1, 9, 0, 2, 10, 3, 4, 7};
    double dr[r], dc[c], bval[8 + r], bX[c * 3], bY[r * 3], bG[r * 3], bT[c * 3];
    int32_t orp[r + 1], oci[8 + r];
    for (int i = 0; i < r; ++i) dr[i] = 2 + i;
    for (int j = 0; j < c; ++j) dc[j] = 1 + j;
    for (int i = 0; i < c * 3; ++i) bX[i] = rnd();
    for (int i = 0; i < r * 3; ++i) bG[i] = rnd();
    CHECK(mggcn_ref_csr_normalize(r, c, brp, bci, REF_NORM_SYM, dr, dc, orp, oci, bval));
    CHECK(mggcn_ref_spmm(REF_OP_N, r, c, orp, oci, bval, bX, 3, 3, 0.0, bY, 3));
    CHECK(mggcn_ref_spmm(REF_OP_T, r, c, orp, oci, bval, bG, 3, 3, 0.0, bT, 3));
  }

  double A[7 * 5], B[5 * 4], Cm[7 * 4], Bt[4 * 5], At[5 * 7];
  for (int i = 0; i < 35; ++i) { A[i] = rnd(); At[i] = rnd(); }
  for (int i = 0; i < 20; ++i) { B[i] = rnd(); Bt[i] = rnd(); }
  for (int i = 0; i < 28; ++i) Cm[i] = rnd();
  CHECK(mggcn_ref_gemm(REF_OP_N, REF_OP_N, 7, 4, 5, A, 5, B, 4, 0.0, Cm, 4));
  CHECK(mggcn_ref_gemm(REF_OP_T, REF_OP_N, 7, 4, 5, At, 7, B, 4, 1.0, Cm, 4));
  CHECK(mggcn_ref_gemm(REF_OP_N, REF_OP_T, 7, 4, 5, A, 5, Bt, 5, 0.0, Cm, 4));
  mggcn_ref_relu(7, 4, Cm, 4);
  double Gm[28];
  for (int i = 0; i < 28; ++i) Gm[i] = rnd();
  mggcn_ref_relu_bwd(7, 4, Cm, 4, Gm, 4);
  uint8_t mask[28];
  for (int i = 0; i < 28; ++i) mask[i] = (uint8_t)(i & 1);
  mggcn_ref_apply_mask(7, 4, mask, Gm, 4);

  int32_t labels[n];
  for (int i = 0; i < n; ++i) labels[i] = i % C;
  double Z[n * C], dZ[n * C], loss;
  for (int i = 0; i < n * C; ++i) Z[i] = 4.0 * rnd();
  CHECK(mggcn_ref_softmax_ce(n, C, Z, C, labels, &loss, dZ, C));
  (void)mggcn_ref_order(3, 5);

  /* layers and epochs in both orders, with and without handed-in decisions / operands */
  double W0[F * 12], W1[12 * 7], W2[7 * C], G0[F * 12], G1[12 * 7], G2[7 * C];
  for (int i = 0; i < F * 12; ++i) W0[i] = rnd();
  for (int i = 0; i < 12 * 7; ++i) W1[i] = rnd();
  for (int i = 0; i < 7 * C; ++i) W2[i] = rnd();
  const double* W[L] = {W0, W1, W2};
  double* WG[L] = {G0, G1, G2};
  double H1[n * 12], HG[n * F], Gin[n * 12];
  for (int ord = 0; ord < 2; ++ord) {
    CHECK(mggcn_ref_layer_fwd(n, rpo, cio, val, F, 12, ord, 1, X, F, W0, 12, H1, 12));
    for (int i = 0; i < n * 12; ++i) Gin[i] = rnd();
    CHECK(mggcn_ref_layer_bwd(n, rpo, cio, val, F, 12, ord, 1, X, F, H1, 12, Gin, 12, W0, 12, G0, 12, HG, F));
    CHECK(mggcn_ref_layer_bwd(n, rpo, cio, val, F, 12, ord, 0, X, F, H1, 12, Gin, 12, W0, 12, G0, 12, NULL, F));
  }
  double logits[n * C];
  uint8_t m0[n * 12], m1[n * 7];
  for (int i = 0; i < n * 12; ++i) m0[i] = (uint8_t)((i * 7) % 3 != 0);
  for (int i = 0; i < n * 7; ++i) m1[i] = (uint8_t)((i * 5) % 4 != 0);
  const uint8_t* masks[L - 1] = {m0, m1};
  const int32_t ords_a[L] = {REF_GEMM_FIRST, REF_SPMM_FIRST, REF_GEMM_FIRST};
  const int32_t ords_b[L] = {REF_SPMM_FIRST, REF_GEMM_FIRST, REF_SPMM_FIRST};
  CHECK(mggcn_ref_epoch(n, rpo, cio, val, L, dims, NULL, X, F, labels, W, &loss, WG, logits, NULL));
  CHECK(mggcn_ref_epoch(n, rpo, cio, val, L, dims, ords_a, X, F, labels, W, &loss, WG, NULL, masks));
  CHECK(mggcn_ref_epoch(n, rpo, cio, val, L, dims, ords_b, X, F, labels, W, &loss, WG, NULL, NULL));

  /* bfloat16 gather epoch: own roundings out, then the same handed back in */
  uint16_t f0[n * 12], f1[n * 12], f2[n * 12], b0[n * 12], b1[n * 12], b2[n * 12];
  uint16_t* fo[L] = {f0, f1, f2};
  uint16_t* bo[L] = {b0, b1, b2};
  CHECK(mggcn_ref_epoch_bf16(n, rpo, cio, val, L, dims, ords_a, X, F, labels, W, &loss, WG, NULL, NULL, NULL, NULL, fo, bo));
  const uint16_t* fi[L] = {f0, f1, f2};
  const uint16_t* bi[L] = {b0, b1, b2};
  CHECK(mggcn_ref_epoch_bf16(n, rpo, cio, val, L, dims, ords_a, X, F, labels, W, &loss, WG, logits, masks, fi, bi, NULL, NULL));
  float xs[6] = {1.0f, -2.5f, 3.0e38f, 1.0e-40f, 0.0f, 65504.0f}, vs[6];
  uint16_t codes[6];
  mggcn_ref_bf16_round(6, xs, codes, vs);
  (void)mggcn_ref_bf16_value(mggcn_ref_bf16_code(1.00390625f));

  double m[F * 12], v[F * 12];
  for (int i = 0; i < F * 12; ++i) m[i] = v[i] = 0.0;
  for (int t = 1; t <= 3; ++t) CHECK(mggcn_ref_adam_step(F * 12, W0, G0, m, v, t, 1e-2, 0.9, 0.999, 1e-8));
  printf("oracle walk ok (loss %.6f)\n", loss);
  return 0;
}
