/* Runs the C oracle on a few small problems under AddressSanitizer / UndefinedBehaviorSanitizer (built by
 * tests/test_host_sanitize.py together with oracle/ss_oracle.c): every array is sized exactly, so an index error in
 * the oracle's loops shows up as a sanitizer report. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int ss_oracle_mask_check(const uint8_t *M, int64_t cout, int64_t K, int64_t *bad_row, int64_t *bad_group);
int ss_oracle_compress(const uint16_t *W, const uint8_t *M, int64_t cout, int64_t K, uint16_t *vals, uint8_t *meta);
void ss_oracle_decompress(const uint16_t *vals, const uint8_t *meta, int64_t cout, int64_t K, uint16_t *Wm);
int ss_oracle_conv2d(const uint16_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin, const uint16_t *W, const uint8_t *M,
                     int64_t cout, int64_t kh, int64_t kw, int korder, int dtype, const float *bias, const uint16_t *residual,
                     int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int act, double *y);
int ss_oracle_conv2d_points(const uint16_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin, const uint16_t *W, const uint8_t *M,
                            int64_t cout, int64_t kh, int64_t kw, int korder, int dtype, const float *bias,
                            const uint16_t *residual, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int act,
                            const int64_t *idx, int64_t n_idx, double *y);

int main(void)
{
    int fails = 0;
    for (int korder = 0; korder < 2; korder++)
        for (int stride = 1; stride <= 2; stride++)
            for (int pad = 0; pad <= 1; pad++) {
                const int N = 2, H = 5, Wd = 4, cin = 4, cout = 3, kh = 3, kw = 2;
                const int K = cin * kh * kw, Ho = (H + 2 * pad - kh) / stride + 1, Wo = (Wd + 2 * pad - kw) / stride + 1;
                if (Ho <= 0 || Wo <= 0) continue;
                uint16_t *x = malloc(sizeof(uint16_t) * N * H * Wd * cin), *W = malloc(sizeof(uint16_t) * cout * K);
                uint8_t *M = malloc((size_t)cout * K);
                float *bias = malloc(sizeof(float) * cout);
                double *y = malloc(sizeof(double) * N * Ho * Wo * cout);
                for (int i = 0; i < N * H * Wd * cin; i++) x[i] = (uint16_t)(0x3C00 + (i % 7) * 64);      /* binary16 around 1.0 */
                for (int i = 0; i < cout * K; i++) { W[i] = (uint16_t)(0x3800 + (i % 5) * 128); M[i] = (uint8_t)((i % 4) < 2); }
                for (int o = 0; o < cout; o++) bias[o] = 0.25f * (float)o;
                int64_t br = -1, bg = -1;
                if (ss_oracle_mask_check(M, cout, K, &br, &bg) != 0) { printf("mask rejected\n"); fails++; }
                uint16_t *vals = malloc(sizeof(uint16_t) * cout * K / 2), *back = malloc(sizeof(uint16_t) * cout * K);
                uint8_t *meta = malloc((size_t)cout * K / 4);
                if (ss_oracle_compress(W, M, cout, K, vals, meta) != 0) { printf("compress failed\n"); fails++; }
                ss_oracle_decompress(vals, meta, cout, K, back);
                for (int i = 0; i < cout * K; i++)
                    if (back[i] != (M[i] ? W[i] : 0)) { printf("round trip differs at %d\n", i); fails++; break; }
                if (ss_oracle_conv2d(x, N, H, Wd, cin, W, M, cout, kh, kw, korder, 0, bias, NULL, stride, stride, pad, pad, 1, y) != 0) {
                    printf("conv failed\n");
                    fails++;
                }
                /* the sampled form on the very first and the very last output must agree with the full tensor */
                int64_t idx[2] = {0, (int64_t)N * Ho * Wo * cout - 1};
                double yp[2];
                if (ss_oracle_conv2d_points(x, N, H, Wd, cin, W, M, cout, kh, kw, korder, 0, bias, NULL, stride, stride, pad, pad, 1,
                                            idx, 2, yp) != 0 || yp[0] != y[idx[0]] || yp[1] != y[idx[1]]) {
                    printf("sampled outputs differ\n");
                    fails++;
                }
                for (int i = 0; i < N * Ho * Wo * cout; i++)
                    if (!(y[i] >= 0.0)) { printf("negative or NaN after ReLU at %d\n", i); fails++; break; }
                free(x); free(W); free(M); free(bias); free(y); free(vals); free(back); free(meta);
            }
    if (!fails) printf("oracle checks passed\n");
    return fails ? 1 : 0;
}
