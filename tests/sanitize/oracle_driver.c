/* Runs every entry point of the CPU oracle on small seeded inputs, with exactly-sized heap buffers, so
 * that a build with -fsanitize=address,undefined reports any access out of bounds or undefined
 * operation.  Built and run by tests/test_sanitizers.py together with oracle/fsd_oracle.c. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int fsd_oracle_verify_chain(const void*, const void*, const int32_t*, int, int, long, int, int, double, int, uint64_t,
                            uint64_t, int, int32_t*, int32_t*, double*, int32_t*, float*);
int fsd_oracle_verify_tree(const void*, const void*, const int32_t*, const int32_t*, int, int, int, long, int, int,
                           double, int, uint64_t, uint64_t, int, int32_t*, int32_t*, int32_t*, double*, int32_t*, float*);
int fsd_oracle_verify_tree_warped(const void*, const void*, const int32_t*, const int32_t*, int, int, int, long, int,
                                  int, double, int, uint64_t, uint64_t, int, float, int, double, int32_t*, int32_t*,
                                  int32_t*, double*, int32_t*, float*, float*, double*);
int sd_oracle_verify_chain(const void*, const void*, const int32_t*, int, int, long, int, int, uint64_t, uint64_t, int,
                           int32_t*, int32_t*, double*, double*, int32_t*, double*);
int sd_oracle_verify_tree(const void*, const void*, const int32_t*, const int32_t*, int, int, int, long, int, int,
                          uint64_t, uint64_t, int, int32_t*, int32_t*, int32_t*, double*, double*, int32_t*, double*);
int rfsd_oracle_verify_chain(const void*, const void*, const int32_t*, int, int, long, int, int, double, int, uint64_t,
                             uint64_t, int, int32_t*, int32_t*, double*, double*, double*, int32_t*, double*);
int fsd_oracle_verify_chain_warped(const void*, const void*, const int32_t*, int, int, long, int, int, double, int,
                                   uint64_t, uint64_t, int, float, int, double, int32_t*, int32_t*, double*, int32_t*,
                                   float*, float*, double*);

static uint64_t state = 88172645463325252ull;
static double unif(void) {   /* xorshift: inputs only */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0;
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(unif() + 1e-300)) * cos(6.283185307179586 * unif())); }
static uint16_t bf16(float x) { union { float f; uint32_t u; } v; v.f = x; return (uint16_t)((v.u + 0x7FFFu + ((v.u >> 16) & 1u)) >> 16); }

static void* rows(long n, int dt, float scale, int masks) {
    if (dt == 0) {
        float* p = malloc((size_t)n * sizeof(float));
        for (long i = 0; i < n; ++i) p[i] = (masks && unif() < 0.05) ? -INFINITY : gauss() * scale;
        return p;
    }
    uint16_t* p = malloc((size_t)n * sizeof(uint16_t));
    for (long i = 0; i < n; ++i) p[i] = (masks && unif() < 0.05) ? 0xFF80 : bf16(gauss() * scale);
    return p;
}

int main(void) {
    int fails = 0;
    const long Vs[] = {1, 7, 64, 1001};
    for (int dt = 0; dt < 2; ++dt)
        for (int vi = 0; vi < 4; ++vi)
            for (int masks = 0; masks < 2; ++masks) {
                const long V = Vs[vi];
                const int B = 3, K = 5, D = 4;
                void* t = rows((long)B * (K + 1) * V, dt, 2.0f, 0);
                void* d = rows((long)B * K * V, dt, 2.0f, masks);
                int32_t* tok = malloc(sizeof(int32_t) * B * K);
                int32_t* par = malloc(sizeof(int32_t) * B * K);
                for (int i = 0; i < B * K; ++i) { tok[i] = (int32_t)(unif() * V); par[i] = (i % K) ? (int32_t)(unif() * (i % K + 1)) - 1 : -1; }
                int32_t* len = malloc(sizeof(int32_t) * B);
                int32_t* out = malloc(sizeof(int32_t) * B * (K + 1));
                int32_t* pn = malloc(sizeof(int32_t) * B * D);
                int32_t* outt = malloc(sizeof(int32_t) * B * (D + 1));
                double* divs = malloc(sizeof(double) * B * K);
                double* lr = malloc(sizeof(double) * B * K);
                double* mg = malloc(sizeof(double) * B * K);
                int32_t* st = malloc(sizeof(int32_t) * B);
                float* gapf = malloc(sizeof(float) * B);
                double* gapd = malloc(sizeof(double) * B);
                float* thr = malloc(sizeof(float) * B);
                double* slack = malloc(sizeof(double) * B);
                for (int div = 0; div < 3; ++div)
                    for (int mode = 0; mode < 2; ++mode) {
                        fails += fsd_oracle_verify_chain(t, d, tok, B, K, V, dt, div, 0.1, mode, 3, 4, 0, len, out, divs, st, gapf) != 0;
                        fails += fsd_oracle_verify_tree(t, d, tok, par, B, K, D, V, dt, div, 0.1, mode, 3, 4, 0, len, pn, outt, divs, st, gapf) != 0;
                        fails += rfsd_oracle_verify_chain(t, d, tok, B, K, V, dt, div, 0.05, mode, 3, 4, 0, len, out, divs, lr, mg, st, gapd) != 0;
                        fails += fsd_oracle_verify_chain_warped(t, d, tok, B, K, V, dt, div, 0.1, mode, 3, 4, 0, 1.25f, 3, 0.8, len, out, divs, st, gapf, thr, slack) != 0;
                        fails += fsd_oracle_verify_tree_warped(t, d, tok, par, B, K, D, V, dt, div, 0.1, mode, 3, 4, 0, 0.7f, 0, 0.5, len, pn, outt, divs, st, gapf, thr, slack) != 0;
                    }
                for (int mode = 0; mode < 2; ++mode) {
                    fails += sd_oracle_verify_chain(t, d, tok, B, K, V, dt, mode, 3, 4, 0, len, out, lr, mg, st, gapd) != 0;
                    fails += sd_oracle_verify_tree(t, d, tok, par, B, K, D, V, dt, mode, 3, 4, 0, len, pn, outt, lr, mg, st, gapd) != 0;
                }
                free(t); free(d); free(tok); free(par); free(len); free(out); free(pn); free(outt); free(divs); free(lr);
                free(mg); free(st); free(gapf); free(gapd); free(thr); free(slack);
            }
    printf("oracle sanitizer driver: %d failing calls\n", fails);
    return fails ? 1 : 0;
}
