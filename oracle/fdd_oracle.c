/*
 * fdd_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what one denoising step of a
 * section-aligned block computes.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the GPU library shares no code,
 * header, table or helper with this file.
 *
 * What each function follows:
 *
 *  fddo_block_attn      Block-causal attention (paper, Preliminaries,
 *                       "Block-Causal Diffusion"): a block attends
 *                       bidirectionally to itself and causally to the prompt
 *                       and all earlier blocks, never to later ones.  With N
 *                       rollouts forked from one KV cache (paper, "Shared
 *                       prefix" paragraph of the test-time-scaling section)
 *                       every rollout sees the same prefix rows and only its
 *                       own block.  Written as the definition: scores over
 *                       the L+B visible keys, max-subtracted two-pass softmax,
 *                       weighted sum of the value rows.  No tiling, no
 *                       streaming softmax, no reordering.
 *
 *                       With causal_block != 0 the in-block part is causal
 *                       instead: block position b sees block positions <= b.
 *                       That is the verify pass of Scaffold Speculative
 *                       Decoding (paper, "Scaffold Speculative Decoding (SS)",
 *                       step 3: "a causal forward pass over the entire block").
 *
 *  fddo_block_attn_ext  The same attention when a rollout has already finished
 *                       blocks of its own after the fork (paper, "Shared
 *                       prefix": the trajectory section is continued N times
 *                       from the forked cache, and that section spans several
 *                       blocks; "Block-Causal Diffusion": a block attends
 *                       causally to ALL earlier blocks).  The keys a row of
 *                       rollout n sees are then three runs: the shared prefix,
 *                       the E rows rollout n has committed since the fork
 *                       (its private extension), and its live block.
 *
 *  fddo_block_commit    A finished block joins its rollout's extension: rows
 *                       E .. E+B-1 of ext[n] become block[n] (a pure copy).
 *
 *  fddo_traj_mean       Trajectory averaging (paper, "Trajectory averaging",
 *                       the merge equation): the output trajectory is the
 *                       equal-weight mean of the N rollout trajectories,
 *                       tau_out = (1/N) sum_i tau^(i), waypoint by waypoint.
 *                       (The jerk-minimizing fit that turns a decoded rollout
 *                       into 20 waypoints is not specified in the paper and is
 *                       outside this file.)
 *
 *  fddo_verify_step     The accept rule of the same step 3: value positions
 *                       are visited left to right; a draft token equal to the
 *                       arg max of the AR distribution at its position is
 *                       accepted; at the first mismatch the AR token replaces
 *                       the draft (the one bonus token) and every later draft
 *                       is discarded.  Scaffold positions are auto-accepted
 *                       (step 1) and do not take part.
 *
 *  fddo_verify_step_ex  The same rule with a sampled verifier (paper,
 *                       "Trajectory-only stochasticity": the verifier samples
 *                       from the softmax in the trajectory section, which is
 *                       what makes forked rollouts differ).  The paper names
 *                       no sampling algorithm; the one used is the Gumbel-max
 *                       form of softmax sampling at temperature T, token =
 *                       arg max_v (x_v / T + g_v) with g_v standard Gumbel
 *                       noise, which is an exact sampler of softmax(x / T).
 *                       So that a sampled token is one well-defined integer,
 *                       the noise and the comparison are DEFINED in fp32
 *                       arithmetic (fddo_sample_key below: a counter-based
 *                       generator, Philox-4x32-10 of Salmon et al., SC'11,
 *                       keyed by the seed and counted by (row, vocabulary id),
 *                       and a polynomial log2 made of exactly rounded fp32
 *                       operations).  This is the one place where the oracle
 *                       does not work in fp64: the sampler's precision is part
 *                       of its definition.
 *
 *  fddo_unmask_step     One iteration of "iteratively unmasks value
 *                       positions" (paper, "Section Diffusion (SD)") under the
 *                       masked-diffusion rule that visible tokens stay fixed
 *                       (paper, "Masked Diffusion Language Models") and that
 *                       diffusion acts on the editable set only, scaffold
 *                       positions being frozen (paper, Eq. 2 and the scaffold
 *                       construction paragraph).  The paper does not print
 *                       the commit rule; the rule used is the task's:
 *                       confidence = largest softmax probability, commit when
 *                       it reaches tau, lowest index wins ties, and a block
 *                       that has an eligible position commits at least one.
 *
 *  fddo_block_kv_update Synthetic stand-in for recomputing the K/V rows of
 *                       positions that were just committed (no model is in
 *                       scope): row (token mod T) of a table.
 *
 *  fddo_fork_block      "fork the KV cache N times": the private block state
 *                       of one rollout replicated N times; the prefix is not
 *                       touched (it is shared by reference).
 *
 * Pins (tests/test_oracle_*.py): brute-force explicit-mask attention,
 * textbook causal attention for B=1, a library softmax-attention with an
 * explicit mask, closed forms, logsumexp from scipy, and the invariants of
 * the unmask rule.  fddo_block_kv_update and fddo_fork_block are pure copies
 * and are pinned by direct comparison with numpy indexing.  The sampler is
 * pinned by the published known-answer vectors of Philox-4x32-10, by the
 * accuracy of its log2 against the library's, and by the frequencies of its
 * samples against softmax(x / T) (tests/test_oracle_sample.py).
 *
 * Element types: 0 = double, 1 = float, 2 = bfloat16 stored as uint16.
 * Stored values are widened exactly to double before any arithmetic.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the parallel loops below will use (for reporting only) */
int fddo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double widen(const void *p, int dtype, size_t i)
{
    if (dtype == 0) return ((const double *)p)[i];
    if (dtype == 1) return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == 0 ? 8 : dtype == 1 ? 4 : 2; }

/*
 * out = softmax(scale * q K_n^T) V_n with K_n = [prefix_k ; block_k[n]] for
 * the KV head h / (Hq/Hkv).  rows == NULL: all (n,b,h), out is [N,B,Hq,D].
 * rows != NULL: n_rows triples (n,b,h); out is [n_rows,D].
 */
int fddo_block_attn_ext(int N, int B, int L, int E, int Ecap, int Hq, int Hkv, int D, int dtype, double scale,
                        int causal_block, const void *q, const void *prefix_k, const void *prefix_v,
                        const void *ext_k, const void *ext_v, const void *block_k, const void *block_v,
                        const int32_t *rows, int64_t n_rows, double *out);

int fddo_block_attn_ex(int N, int B, int L, int Hq, int Hkv, int D, int dtype, double scale, int causal_block,
                       const void *q, const void *prefix_k, const void *prefix_v,
                       const void *block_k, const void *block_v,
                       const int32_t *rows, int64_t n_rows, double *out)
{
    return fddo_block_attn_ext(N, B, L, 0, 0, Hq, Hkv, D, dtype, scale, causal_block, q, prefix_k, prefix_v, NULL, NULL,
                               block_k, block_v, rows, n_rows, out);
}

int fddo_block_attn(int N, int B, int L, int Hq, int Hkv, int D, int dtype, double scale,
                    const void *q, const void *prefix_k, const void *prefix_v,
                    const void *block_k, const void *block_v,
                    const int32_t *rows, int64_t n_rows, double *out)
{
    return fddo_block_attn_ex(N, B, L, Hq, Hkv, D, dtype, scale, 0, q, prefix_k, prefix_v, block_k, block_v,
                              rows, n_rows, out);
}

/*
 * Visible keys of a row of rollout n, in order: prefix rows 0..L-1 (shared),
 * extension rows ext[n, 0..E-1] (ext is [N, Ecap, Hkv, D]), block rows.
 * causal_block == 0: the whole own block is visible; != 0: block keys up to
 * the query's own position.
 */
int fddo_block_attn_ext(int N, int B, int L, int E, int Ecap, int Hq, int Hkv, int D, int dtype, double scale,
                        int causal_block, const void *q, const void *prefix_k, const void *prefix_v,
                        const void *ext_k, const void *ext_v, const void *block_k, const void *block_v,
                        const int32_t *rows, int64_t n_rows, double *out)
{
    if (N <= 0 || B <= 0 || L < 0 || E < 0 || E > Ecap || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv) return 1;
    const int G = Hq / Hkv;
    const int Sfull = L + E + B;
    const int64_t total = rows ? n_rows : (int64_t)N * B * Hq;
    int bad = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Sfull);
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < total; ++r) {
            int n, b, h;
            if (rows) { n = rows[3 * r]; b = rows[3 * r + 1]; h = rows[3 * r + 2]; }
            else { h = (int)(r % Hq); b = (int)((r / Hq) % B); n = (int)(r / ((int64_t)Hq * B)); }
            if (n < 0 || n >= N || b < 0 || b >= B || h < 0 || h >= Hq) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            const int kh = h / G;
            const int S = causal_block ? L + E + b + 1 : Sfull;   /* number of visible keys */
            const size_t qo = (((size_t)n * B + b) * Hq + h) * D;
            /* key j: which array it lives in and at which element offset */
            #define FDDO_KEY(j, PK, EK, BK, arr, off) do { \
                if ((j) < L) { arr = (PK); off = ((size_t)(j) * Hkv + kh) * D; } \
                else if ((j) < L + E) { arr = (EK); off = (((size_t)n * Ecap + ((j) - L)) * Hkv + kh) * D; } \
                else { arr = (BK); off = (((size_t)n * B + ((j) - L - E)) * Hkv + kh) * D; } } while (0)
            double smax = -INFINITY;
            for (int j = 0; j < S; ++j) {
                const void *arr; size_t ko;
                FDDO_KEY(j, prefix_k, ext_k, block_k, arr, ko);
                double acc = 0.0;
                for (int d = 0; d < D; ++d) acc += widen(q, dtype, qo + d) * widen(arr, dtype, ko + d);
                s[j] = scale * acc;
                if (s[j] > smax) smax = s[j];
            }
            double z = 0.0;
            for (int j = 0; j < S; ++j) { s[j] = exp(s[j] - smax); z += s[j]; }
            double *o = out + (size_t)r * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int j = 0; j < S; ++j) {
                const double p = s[j] / z;
                const void *arr; size_t vo;
                FDDO_KEY(j, prefix_v, ext_v, block_v, arr, vo);
                for (int d = 0; d < D; ++d) o[d] += p * widen(arr, dtype, vo + d);
            }
            #undef FDDO_KEY
        }
        free(s);
    }
    return bad;
}

/* ext[n, E .. E+B-1] = block[n] for K and V: the finished block joins the rollout's private extension. */
int fddo_block_commit(int N, int B, int E, int Ecap, int Hkv, int D, int dtype,
                      const void *block_k, const void *block_v, void *ext_k, void *ext_v)
{
    if (N <= 0 || B <= 0 || E < 0 || E + B > Ecap || Hkv <= 0 || D <= 0) return 1;
    const size_t row = (size_t)Hkv * D * elem_size(dtype);
    for (int n = 0; n < N; ++n) {
        memcpy((char *)ext_k + ((size_t)n * Ecap + E) * row, (const char *)block_k + (size_t)n * B * row, (size_t)B * row);
        memcpy((char *)ext_v + ((size_t)n * Ecap + E) * row, (const char *)block_v + (size_t)n * B * row, (size_t)B * row);
    }
    return 0;
}

/*
 * One unmask iteration over N blocks.  mask and tokens are updated in place.
 *   conf[n,b]      confidence of eligible positions, -inf elsewhere
 *   cand[n,b]      argmax token of eligible positions, -1 elsewhere (may be NULL)
 *   n_unmasked[n]  number of positions committed in block n (may be NULL)
 *   committed[n,b] 1 where this call committed the position (may be NULL)
 */
int fddo_unmask_step(int N, int B, int64_t V, int dtype, double tau, const void *logits,
                     const uint8_t *scaffold, uint8_t *mask, int32_t *tokens,
                     double *conf, int32_t *cand, int32_t *n_unmasked, uint8_t *committed)
{
    if (N <= 0 || B <= 0 || V <= 0) return 1;
    const int64_t NB = (int64_t)N * B;
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)NB);
    /* step 1-2: per eligible position, the arg max of the raw logits (lowest
       id on ties) and the largest softmax probability 1 / sum exp(x - max) */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < NB; ++i) {
        const int eligible = mask[i] == 1 && !(scaffold && scaffold[i]);
        conf[i] = -INFINITY;
        tok[i] = -1;
        if (!eligible) continue;
        const size_t base = (size_t)i * (size_t)V;
        double xmax = widen(logits, dtype, base);
        int64_t arg = 0;
        for (int64_t v = 1; v < V; ++v) {
            const double x = widen(logits, dtype, base + v);
            if (x > xmax) { xmax = x; arg = v; }
        }
        double z = 0.0;
        for (int64_t v = 0; v < V; ++v) z += exp(widen(logits, dtype, base + v) - xmax);
        conf[i] = 1.0 / z;
        tok[i] = (int32_t)arg;
    }
    /* step 3-6: per block, threshold test, forced single commit, write-back */
    for (int n = 0; n < N; ++n) {
        int count = 0, best = -1;
        for (int b = 0; b < B; ++b) {
            const int64_t i = (int64_t)n * B + b;
            if (committed) committed[i] = 0;
            if (tok[i] < 0) continue;                       /* not eligible */
            if (best < 0 || conf[i] > conf[(int64_t)n * B + best]) best = b;
            if (conf[i] >= tau) {
                tokens[i] = tok[i]; mask[i] = 0; ++count;
                if (committed) committed[i] = 1;
            }
        }
        if (count == 0 && best >= 0) {
            const int64_t i = (int64_t)n * B + best;
            tokens[i] = tok[i]; mask[i] = 0; count = 1;
            if (committed) committed[i] = 1;
        }
        if (n_unmasked) n_unmasked[n] = count;
    }
    if (cand) memcpy(cand, tok, sizeof(int32_t) * (size_t)NB);
    free(tok);
    return 0;
}

/* ---- the sampler's arithmetic (fp32 by definition) ------------------------- */

/* Philox-4x32 with 10 rounds: counter-based generator of Salmon, Moraes, Dror and
 * Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11). */
void fddo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* log2 of a positive normal float, made of exactly rounded fp32 operations:
 * x = m 2^e with m in [1/sqrt 2, sqrt 2), log2 x = e + f P(f), f = m - 1,
 * P of degree 8.  Absolute error below 1e-7 on the reduced range. */
float fddo_flog2(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, 4);
    int e = (int)((bits >> 23) & 255u) - 127;
    const uint32_t mb = (bits & 0x7fffffu) | 0x3f800000u;
    float m;
    memcpy(&m, &mb, 4);
    if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
    const float f = m - 1.0f;
    float p = 0.12614846229553223f;
    p = fmaf(p, f, -0.20742103457450867f);
    p = fmaf(p, f, 0.21566985547542572f);
    p = fmaf(p, f, -0.23892034590244293f);
    p = fmaf(p, f, 0.2879183292388916f);
    p = fmaf(p, f, -0.36070483922958374f);
    p = fmaf(p, f, 0.48091059923171997f);
    p = fmaf(p, f, -0.7213473320007324f);
    p = fmaf(p, f, 1.4426950216293335f);
    return fmaf(f, p, (float)e);
}

/* Gumbel-max key of vocabulary entry v of row `row` (= n B + b), in log2 units:
 *   r   = word (v mod 4) of Philox(counter = (v div 4, row, 0, 0), key = seed)
 *   u   = ((r >> 9) + 1/2) 2^-23          in (0, 1), exact in fp32
 *   key = x c - log2(-log2 u)             c = log2(e) / T rounded to fp32
 * arg max_v key samples softmax(x / T): -ln(-ln u) is standard Gumbel noise and
 * the change of logarithm base shifts every key by the same constant. */
float fddo_sample_key(float x, float c, uint64_t seed, uint32_t row, int64_t v)
{
    const uint32_t ctr[4] = {(uint32_t)(v >> 2), row, 0u, 0u};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t r[4];
    fddo_philox4x32_10(ctr, key, r);
    const float u = ((float)(r[v & 3] >> 9) + 0.5f) * 1.1920928955078125e-07f;
    const float a = -fddo_flog2(u);
    const float g = -fddo_flog2(a);
    return fmaf(x, c, g);
}

float fddo_sample_scale(float temperature) { return (float)(1.4426950408889634 / (double)temperature); }

/*
 * Verify pass of scaffold speculative decoding over N blocks.  A position is a
 * draft position when mask == 1 and it is not scaffold.  mask and tokens are
 * updated in place: accepted positions take their draft token, the rejection
 * point takes the AR token, both are unmasked; later draft positions stay masked
 * and keep their tokens entry.
 *   ar_tok[n,b]     arg max of the AR logits at draft positions (lowest id on
 *                   ties), -1 elsewhere (may be NULL)
 *   n_accepted[n]   positions unmasked in block n by this call
 *   accepted[n,b]   1 = draft accepted, 2 = replaced by the AR token, 0 otherwise (may be NULL)
 */
/* temperature == 0: greedy verifier (arg max of the logits); temperature > 0:
 * sampled verifier as defined above.  ar_tok receives the verifier's token. */
int fddo_verify_step_ex(int N, int B, int64_t V, int dtype, const void *ar_logits, const uint8_t *scaffold,
                        const int32_t *draft, uint8_t *mask, int32_t *tokens, int32_t *ar_tok,
                        int32_t *n_accepted, uint8_t *accepted, float temperature, uint64_t seed)
{
    if (N <= 0 || B <= 0 || V <= 0 || !(temperature >= 0.0f)) return 1;
    const float c = temperature > 0.0f ? fddo_sample_scale(temperature) : 0.0f;
    for (int n = 0; n < N; ++n) {
        int count = 0, rejected = 0;
        for (int b = 0; b < B; ++b) {
            const int64_t i = (int64_t)n * B + b;
            const int is_draft = mask[i] == 1 && !(scaffold && scaffold[i]);
            if (accepted) accepted[i] = 0;
            if (ar_tok) ar_tok[i] = -1;
            if (!is_draft) continue;
            const size_t base = (size_t)i * (size_t)V;
            int64_t arg = 0;
            if (temperature > 0.0f) {
                float kmax = fddo_sample_key((float)widen(ar_logits, dtype, base), c, seed, (uint32_t)i, 0);
                for (int64_t v = 1; v < V; ++v) {
                    const float k = fddo_sample_key((float)widen(ar_logits, dtype, base + v), c, seed, (uint32_t)i, v);
                    if (k > kmax) { kmax = k; arg = v; }
                }
            } else {
                double xmax = widen(ar_logits, dtype, base);
                for (int64_t v = 1; v < V; ++v) {
                    const double x = widen(ar_logits, dtype, base + v);
                    if (x > xmax) { xmax = x; arg = v; }
                }
            }
            if (ar_tok) ar_tok[i] = (int32_t)arg;
            if (rejected) continue;                 /* discarded: stays masked */
            if ((int32_t)arg == draft[i]) {
                tokens[i] = draft[i]; mask[i] = 0; ++count;
                if (accepted) accepted[i] = 1;
            } else {
                tokens[i] = (int32_t)arg; mask[i] = 0; ++count; rejected = 1;
                if (accepted) accepted[i] = 2;
            }
        }
        if (n_accepted) n_accepted[n] = count;
    }
    return 0;
}

int fddo_verify_step(int N, int B, int64_t V, int dtype, const void *ar_logits, const uint8_t *scaffold,
                     const int32_t *draft, uint8_t *mask, int32_t *tokens, int32_t *ar_tok,
                     int32_t *n_accepted, uint8_t *accepted)
{
    return fddo_verify_step_ex(N, B, V, dtype, ar_logits, scaffold, draft, mask, tokens, ar_tok, n_accepted, accepted,
                               0.0f, 0u);
}

/* out[p] = (1/N) sum_n traj[n, p]; traj is [N, P] (P = waypoints x coordinates), dtype 0 or 1. */
int fddo_traj_mean(int N, int P, int dtype, const void *traj, double *out)
{
    if (N <= 0 || P <= 0 || (dtype != 0 && dtype != 1)) return 1;
    for (int p = 0; p < P; ++p) {
        double acc = 0.0;
        for (int n = 0; n < N; ++n) acc += widen(traj, dtype, (size_t)n * P + p);
        out[p] = acc / (double)N;
    }
    return 0;
}

/* K/V rows of just-committed positions <- table row (token mod T). */
int fddo_block_kv_update(int N, int B, int Hkv, int D, int T, int dtype,
                         const int32_t *tokens, const uint8_t *committed,
                         const void *table_k, const void *table_v,
                         void *block_k, void *block_v)
{
    if (N <= 0 || B <= 0 || Hkv <= 0 || D <= 0 || T <= 0) return 1;
    const size_t row = (size_t)Hkv * D * elem_size(dtype);
    for (int64_t i = 0; i < (int64_t)N * B; ++i) {
        if (!committed[i]) continue;
        int64_t t = tokens[i] % T;
        if (t < 0) t += T;
        memcpy((char *)block_k + (size_t)i * row, (const char *)table_k + (size_t)t * row, row);
        memcpy((char *)block_v + (size_t)i * row, (const char *)table_v + (size_t)t * row, row);
    }
    return 0;
}

/* dst[n] = src for n in [0,N): the private per-rollout state after a fork. */
int fddo_fork_block(int N, size_t bytes, const void *src, void *dst)
{
    if (N <= 0) return 1;
    for (int n = 0; n < N; ++n) memcpy((char *)dst + (size_t)n * bytes, src, bytes);
    return 0;
}
