/* Drives every function of the CPU oracle on small inputs.  Built together with
 * oracle/fdd_oracle.c under -fsanitize=address,undefined by tests/test_sanitize.py;
 * any out-of-bounds access, leak or undefined operation makes the run fail. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int fddo_block_attn_ext(int N, int B, int L, int E, int Ecap, int Hq, int Hkv, int D, int dtype, double scale,
                        int causal_block, const void *q, const void *pk, const void *pv, const void *ek,
                        const void *ev, const void *bk, const void *bv, const int32_t *rows, int64_t n_rows, double *out);
int fddo_block_attn(int N, int B, int L, int Hq, int Hkv, int D, int dtype, double scale, const void *q, const void *pk,
                    const void *pv, const void *bk, const void *bv, const int32_t *rows, int64_t n_rows, double *out);
int fddo_unmask_step(int N, int B, int64_t V, int dtype, double tau, const void *logits, const uint8_t *scaffold,
                     uint8_t *mask, int32_t *tokens, double *conf, int32_t *cand, int32_t *n_unmasked, uint8_t *committed);
int fddo_verify_step_ex(int N, int B, int64_t V, int dtype, const void *ar_logits, const uint8_t *scaffold,
                        const int32_t *draft, uint8_t *mask, int32_t *tokens, int32_t *ar_tok, int32_t *n_accepted,
                        uint8_t *accepted, float temperature, uint64_t seed);
int fddo_block_commit(int N, int B, int E, int Ecap, int Hkv, int D, int dtype, const void *bk, const void *bv, void *ek,
                      void *ev);
int fddo_block_kv_update(int N, int B, int Hkv, int D, int T, int dtype, const int32_t *tokens, const uint8_t *committed,
                         const void *tk, const void *tv, void *bk, void *bv);
int fddo_fork_block(int N, size_t bytes, const void *src, void *dst);
int fddo_traj_mean(int N, int P, int dtype, const void *traj, double *out);

static uint32_t lcg = 12345u;
static double rnd(void) { lcg = lcg * 1664525u + 1013904223u; return ((lcg >> 8) / 16777216.0) * 4.0 - 2.0; }
static double *rand_f64(size_t n) { double *p = malloc(n * sizeof *p); for (size_t i = 0; i < n; ++i) p[i] = rnd(); return p; }
static float *rand_f32(size_t n) { float *p = malloc(n * sizeof *p); for (size_t i = 0; i < n; ++i) p[i] = (float)rnd(); return p; }
static uint16_t *rand_bf16(size_t n)
{
    uint16_t *p = malloc(n * sizeof *p);
    for (size_t i = 0; i < n; ++i) { float f = (float)rnd(); uint32_t u; memcpy(&u, &f, 4); p[i] = (uint16_t)(u >> 16); }
    return p;
}
#define CHECK(x) do { if ((x) != 0) { fprintf(stderr, "oracle call failed: %s\n", #x); return 1; } } while (0)

int main(void)
{
    /* attention, all three storage types, with an extension, causal and not, whole output and listed rows */
    const int N = 3, B = 5, L = 37, E = 4, Ecap = 6, Hq = 6, Hkv = 2, D = 8;
    for (int dtype = 0; dtype < 3; ++dtype) {
        void *(*mk)(size_t) = dtype == 0 ? (void *(*)(size_t))rand_f64 : dtype == 1 ? (void *(*)(size_t))rand_f32 : (void *(*)(size_t))rand_bf16;
        void *q = mk((size_t)N * B * Hq * D), *pk = mk((size_t)L * Hkv * D), *pv = mk((size_t)L * Hkv * D);
        void *bk = mk((size_t)N * B * Hkv * D), *bv = mk((size_t)N * B * Hkv * D);
        void *ek = mk((size_t)N * Ecap * Hkv * D), *ev = mk((size_t)N * Ecap * Hkv * D);
        double *out = malloc(sizeof(double) * N * B * Hq * D);
        for (int causal = 0; causal < 2; ++causal) {
            CHECK(fddo_block_attn_ext(N, B, L, E, Ecap, Hq, Hkv, D, dtype, 0.3, causal, q, pk, pv, ek, ev, bk, bv, NULL, 0, out));
            CHECK(fddo_block_attn_ext(N, B, 0, 0, 0, Hq, Hkv, D, dtype, 0.3, causal, q, NULL, NULL, NULL, NULL, bk, bv, NULL, 0, out));
        }
        const int32_t rows[] = {0, 0, 0, 2, 4, 5, 1, 3, 2};
        CHECK(fddo_block_attn(N, B, L, Hq, Hkv, D, dtype, 0.3, q, pk, pv, bk, bv, rows, 3, out));
        const int32_t bad_rows[] = {0, 0, 0, 3, 0, 0};           /* rollout 3 does not exist: reported, not read */
        if (fddo_block_attn(N, B, L, Hq, Hkv, D, dtype, 0.3, q, pk, pv, bk, bv, bad_rows, 2, out) == 0) return 2;
        for (int i = 0; i < N * B * Hq * D; ++i) if (!isfinite(out[i]) && i < 3 * D) return 3;
        free(q); free(pk); free(pv); free(bk); free(bv); free(ek); free(ev); free(out);
    }
    /* unmask and verify steps (greedy and sampled), odd vocabulary size */
    {
        const int n = 2, b = 7; const int64_t V = 101;
        for (int dtype = 0; dtype < 3; ++dtype) {
            void *lg = dtype == 0 ? (void *)rand_f64(n * b * V) : dtype == 1 ? (void *)rand_f32(n * b * V) : (void *)rand_bf16(n * b * V);
            uint8_t sc[14] = {0, 1, 0, 0, 1, 0, 0, 0, 0, 0, 1, 0, 0, 1}, mask[14], com[14];
            int32_t tok[14], cand[14], nun[2], draft[14];
            double conf[14];
            for (int i = 0; i < 14; ++i) { mask[i] = (uint8_t)(i % 5 != 3); tok[i] = -1; draft[i] = i % 3; }
            CHECK(fddo_unmask_step(n, b, V, dtype, 0.9, lg, sc, mask, tok, conf, cand, nun, com));
            CHECK(fddo_unmask_step(n, b, V, dtype, 0.0, lg, NULL, mask, tok, conf, NULL, NULL, NULL));
            for (int i = 0; i < 14; ++i) mask[i] = 1;
            CHECK(fddo_verify_step_ex(n, b, V, dtype, lg, sc, draft, mask, tok, cand, nun, com, 0.0f, 0));
            for (int i = 0; i < 14; ++i) mask[i] = 1;
            CHECK(fddo_verify_step_ex(n, b, V, dtype, lg, sc, draft, mask, tok, NULL, NULL, NULL, 0.7f, 0xfedcba9876543210ull));
            free(lg);
        }
    }
    /* bookkeeping */
    {
        const int n = 3, b = 4, hkv = 2, d = 8, T = 5, ecap = 9;
        uint16_t *bk = rand_bf16((size_t)n * b * hkv * d), *bv = rand_bf16((size_t)n * b * hkv * d);
        uint16_t *ek = rand_bf16((size_t)n * ecap * hkv * d), *ev = rand_bf16((size_t)n * ecap * hkv * d);
        uint16_t *tk = rand_bf16((size_t)T * hkv * d), *tv = rand_bf16((size_t)T * hkv * d);
        CHECK(fddo_block_commit(n, b, 5, ecap, hkv, d, 2, bk, bv, ek, ev));
        if (fddo_block_commit(n, b, 6, ecap, hkv, d, 2, bk, bv, ek, ev) == 0) return 4;     /* would overflow: refused */
        int32_t tok[12] = {0, -1, 7, 123456, -9, 4, 3, 2, 1, 0, 5, 6};
        uint8_t com[12] = {1, 1, 1, 1, 1, 0, 0, 1, 0, 0, 1, 1};
        CHECK(fddo_block_kv_update(n, b, hkv, d, T, 2, tok, com, tk, tv, bk, bv));
        uint16_t *forks = malloc((size_t)4 * b * hkv * d * 2);
        CHECK(fddo_fork_block(4, (size_t)b * hkv * d * 2, bk, forks));
        float *traj = rand_f32(6 * 40);
        double mean[40];
        CHECK(fddo_traj_mean(6, 40, 1, traj, mean));
        free(bk); free(bv); free(ek); free(ev); free(tk); free(tv); free(forks); free(traj);
    }
    puts("oracle sanitizer run: ok");
    return 0;
}
