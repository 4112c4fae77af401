/* Runs the C oracle's entry points on small inputs; built with -fsanitize=address,undefined by the CPU test that
 * runs it, so that an out-of-bounds access or undefined arithmetic in the oracle fails loudly. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_vocab_row(const void* logits, int32_t dtype, int32_t V, double beta, double alpha, uint64_t seed, int32_t t, int32_t r,
                   int32_t forced, int32_t* out, double* res);
void orc_step(const void* logits, int32_t dtype, int64_t stride, int32_t R, int32_t V, double alpha_t, double alpha_prev,
              double beta, uint64_t seed, int32_t t, double* logW, double* cumlogp, int32_t* hist, int32_t T_max,
              int32_t* tokens, int32_t* second, double* gap, double* delta, int32_t eos_id, int32_t* done);
void orc_ess(const double* logW, int32_t B, int32_t N, double* ess, double* lognormw);
void orc_resample(double* logW, int32_t B, int32_t N, double kappa, uint64_t seed, int32_t t, int32_t* anc,
                  int32_t* resampled, double* ess_out, double* scratch_w, int32_t scheme, int32_t in_place);
void orc_gather_kv(const void* src, void* dst, const int32_t* anc, const int32_t* resampled, int32_t R, int32_t N,
                   int32_t H, int32_t S, int32_t D, int32_t elem, int32_t valid_len);
void orc_gather_state(const int32_t* hist_src, int32_t* hist_dst, int32_t T_max, int32_t t, const double* cum_src,
                      double* cum_dst, const int32_t* anc, const int32_t* resampled, int32_t R, int32_t N,
                      const int32_t* done_src, int32_t* done_dst);
void orc_final_draw(const double* logW, int32_t B, int32_t N, uint64_t seed, int32_t t, int32_t* choice);

int main(void)
{
    enum { B = 3, N = 5, R = B * N, V = 37, T = 6, H = 2, S = 4, D = 3 };
    float* logits = malloc(sizeof(float) * R * V);
    double logW[R], cum[R], gap[R], delta[R], ess[B], lnw[R], scratch[2 * N];
    int32_t hist2[R * T], done2[R]; double cum2[R];
    int32_t hist[R * T], tokens[R], second[R], done[R], anc[R], flag[B], choice[B];
    uint16_t* kv = malloc(sizeof(uint16_t) * R * H * S * D); uint16_t* kv2 = malloc(sizeof(uint16_t) * R * H * S * D);
    for (int i = 0; i < R; ++i) { logW[i] = 0; cum[i] = 0; done[i] = 0; }
    for (int i = 0; i < R * T; ++i) hist[i] = 0;
    for (int i = 0; i < R * H * S * D; ++i) kv[i] = (uint16_t)i;
    unsigned x = 1u;
    for (int t = 1; t <= T; ++t) {
        for (int i = 0; i < R * V; ++i) { x = x * 1664525u + 1013904223u; logits[i] = (float)(x >> 8) / 16777216.0f * 10.0f - 5.0f; }
        for (int scheme = 0; scheme < 4; ++scheme) {
            if (scheme > 0 && t != 3) continue;
            orc_step(logits, 1, V, R, V, 4.0, t == 1 ? 1.0 : 4.0, 4.0, 99u, t, logW, cum, hist, T, tokens, second, gap, delta, 5, done);
            orc_ess(logW, B, N, ess, lnw);
            orc_resample(logW, B, N, 0.9, 99u, t, anc, flag, ess, scratch, scheme, scheme & 1);
            orc_gather_kv(kv, kv2, anc, flag, R, N, H, S, D, 2, t < S ? t : S);
            orc_gather_state(hist, hist2, T, t, cum, cum2, anc, flag, R, N, done, done2);
            for (int i = 0; i < R; ++i) if (tokens[i] < 0 || tokens[i] >= V || anc[i] < 0 || anc[i] >= R) return 1;
        }
    }
    int32_t out[2]; double res[6];
    orc_vocab_row(logits, 1, V, 0.37, 2.5, 7u, 1, 0, 3, out, res);
    orc_vocab_row(logits, 1, 1, 4.0, 4.0, 7u, 1, 0, -1, out, res);
    orc_final_draw(logW, B, N, 99u, T, choice);
    for (int b = 0; b < B; ++b) if (choice[b] < b * N || choice[b] >= (b + 1) * N) return 2;
    free(logits); free(kv); free(kv2);
    printf("oracle_sanitized ok\n");
    return 0;
}
