/* Runs every function of oracle/roast_oracle.c on small shapes chosen to touch the edges of its
 * arrays (ragged tiles, the last legal offset, a short last chunk, one-element blocks), so that a
 * build with -fsanitize=address,undefined reports any out-of-bounds access or undefined integer
 * operation.  Test infrastructure; linked with the oracle only.  Exit code 0 = all calls returned 0. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
  uint64_t P, a0, a1, a2, a3, s0, s1, s2, s3;
  uint32_t use_sign, align;
} oracle_hash_t;

int oracle_locate(const oracle_hash_t*, uint64_t, uint64_t, uint64_t, int64_t, int64_t, int64_t*, int32_t*);
int oracle_tile_index(const oracle_hash_t*, uint32_t, int64_t, int64_t, int32_t, int32_t, int64_t, int64_t*, int8_t*);
int oracle_materialize_w(const oracle_hash_t*, uint32_t, int64_t, int64_t, int32_t, int32_t, int64_t, double,
                         const float*, int32_t, double*);
void oracle_gemm_nn(int64_t, int64_t, int64_t, const double*, const double*, double*);
void oracle_gemm_nt(int64_t, int64_t, int64_t, const double*, const double*, double*);
void oracle_gemm_tn(int64_t, int64_t, int64_t, const double*, const double*, double*);
int oracle_scatter_dm(const oracle_hash_t*, uint32_t, int64_t, int64_t, int32_t, int32_t, int64_t, double,
                      const double*, double*);
int oracle_dm_window(const oracle_hash_t*, uint32_t, int64_t, int64_t, int64_t, int32_t, int32_t, int64_t, double,
                     const double*, const double*, int64_t, int64_t, double*);
int oracle_embed_fwd(const oracle_hash_t*, int64_t, int32_t, int64_t, double, int64_t, const int64_t*,
                     const uint32_t*, const float*, double*);
int oracle_embed_bwd(const oracle_hash_t*, int64_t, int32_t, int64_t, double, int64_t, const int64_t*,
                     const uint32_t*, const double*, double*);
int oracle_num_threads(void);

static double* dvec(int64_t n) {
  double* p = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  for (int64_t i = 0; i < n; ++i) p[i] = (double)((i * 37) % 11) - 5.0;
  return p;
}

int main(void) {
  const uint64_t primes[4] = {2, 65537, 2147483647ull, 4294967291ull};
  int bad = 0;
  for (int pi = 0; pi < 4; ++pi)
    for (uint32_t sign = 0; sign <= 2; ++sign)
      for (uint32_t align = 1; align <= 3; align += 2) {
        const uint64_t P = primes[pi];
        oracle_hash_t h = {P, 5 % P, 7 % P, 11 % P, 13 % P, 17 % P, 19 % P, 23 % P, 29 % P, sign, align};
        for (int Z1 = 1; Z1 <= 5; Z1 += 2)
          for (int Z2 = 1; Z2 <= 6; Z2 += 5) {
            const int64_t H = 7, O = 9, I = 5, L = (int64_t)Z1 * Z2;
            for (int64_t m = L; m <= L + 40; m += 20) {   /* m == L: the only legal offset is 0 */
              const int64_t ntx = (H + Z1 - 1) / Z1, nty = (O + Z2 - 1) / Z2;
              int64_t* off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(ntx * nty));
              int8_t* sg = (int8_t*)malloc((size_t)(ntx * nty));
              float* M = (float*)malloc(sizeof(float) * (size_t)m);
              for (int64_t i = 0; i < m; ++i) M[i] = (float)(i + 1);
              double *W = dvec(H * O), *X = dvec(I * H), *dY = dvec(I * O), *Y = dvec(I * O), *dX = dvec(I * H);
              double *dW = dvec(H * O), *dM = (double*)calloc((size_t)m, sizeof(double)), *win = (double*)calloc((size_t)m, sizeof(double));
              bad += oracle_tile_index(&h, 3u, H, O, Z1, Z2, m, off, sg);
              for (int64_t t = 0; t < ntx * nty; ++t) bad += (off[t] < 0 || off[t] > m - L);
              bad += oracle_materialize_w(&h, 3u, H, O, Z1, Z2, m, 0.5, M, (int32_t)(pi & 1), W);
              oracle_gemm_nn(I, H, O, X, W, Y);
              oracle_gemm_nt(I, H, O, dY, W, dX);
              oracle_gemm_tn(I, H, O, X, dY, dW);
              bad += oracle_scatter_dm(&h, 3u, H, O, Z1, Z2, m, 0.5, dW, dM);
              bad += oracle_dm_window(&h, 3u, I, H, O, Z1, Z2, m, 0.5, X, dY, 0, m, win);
              bad += oracle_dm_window(&h, 3u, I, H, O, Z1, Z2, m, 0.5, X, dY, m - 1, m, win);
              free(off); free(sg); free(M); free(W); free(X); free(dY); free(Y); free(dX); free(dW); free(dM); free(win);
            }
          }
        /* lookup: D not a multiple of Z (short last chunk), 40-bit row ids, |M| == Z */
        for (int Z = 1; Z <= 8; Z += 7)
          for (int64_t m = Z; m <= Z + 50; m += 50) {
            const int64_t D = 11, N = 6;
            int64_t rows[6] = {0, 1, (1ll << 40) + 3, 77, 77, (1ll << 62)};
            uint32_t tabs[6] = {0, 1, 2, 4294967295u, 4294967295u, 9};
            float* M = (float*)malloc(sizeof(float) * (size_t)m);
            for (int64_t i = 0; i < m; ++i) M[i] = (float)(i + 1);
            double *out = dvec(N * D), *dOut = dvec(N * D), *dM = (double*)calloc((size_t)m, sizeof(double));
            bad += oracle_embed_fwd(&h, D, Z, m, 2.0, N, rows, tabs, M, out);
            bad += oracle_embed_bwd(&h, D, Z, m, 2.0, N, rows, tabs, dOut, dM);
            free(M); free(out); free(dOut); free(dM);
          }
        int64_t o; int32_t s;
        bad += !oracle_locate(&h, 1, 2, 3, 3, 4, &o, &s);   /* block larger than M: must be refused */
      }
  printf("oracle sanitizer driver: %d failures, %d threads\n", bad, oracle_num_threads());
  return bad != 0;
}
