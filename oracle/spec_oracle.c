/*
 * CPU oracle for the target-side verification step of hybrid ordinary-parallel
 * speculative serving (paper: Method, "Target-Side Adaptive Hybrid Policy";
 * Appendix "Implementation Details", subsection "Target side").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 restatement of what
 * the four calls of the verification step compute.  It shares no code, header,
 * table or helper with the GPU library, is never linked into it, and must only
 * be called from tests, the smoke check and the cpu_baseline leg of the
 * benchmark.  No blocking, no fusion, no online softmax: every function is the
 * textbook definition (attention, matmul, argmax, prefix match, page-table
 * truncation) or the canonical speculative rejection-sampling procedure the
 * paper names (Fig. "Illustration of SPECTRE decoding": the target verifies
 * drafts via rejection sampling; Related Work: canonical rejection sampling
 * preserves the target distribution), taken step by step.
 *
 * Notation (paper, Appendix "Target side"): request i has a committed prefix
 * of c_i tokens, gamma_i draft tokens d_1..d_gamma, and the verification
 * candidate y = [b, d_1, ..., d_gamma] with b the last committed (bonus)
 * token, so n_i = gamma_i + 1 rows are scored; qo_indptr[i] is the first row
 * of request i in the merged batch Y_n.  gamma_i = 0 is the padded
 * parallel-mode / one-token-decode candidate (eq. parallel_rollback_pad and
 * the "Fallback" paragraph): a single row, ordinary decoding.
 *
 * All pointers are host pointers.  bf16 values are passed as uint16_t bit
 * patterns.  Return value 0 = ok, negative = bad argument.
 *
 * Pinned by tests/test_oracle_*.py (prefix-match, q == p, gamma = 0 decode,
 * tiny-vocabulary exact distribution, Philox known answers, page
 * conservation, textbook matmul/softmax special cases).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)

static float bf16_bits_to_float(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* ------------------------------------------------------------------------- *
 * Attention over the paged KV cache for every candidate position.
 * Row j of request i attends to key positions 0 .. c_i + j (its committed
 * prefix plus the candidate tokens up to and including itself: causal inside
 * the draft block).  Position t lives in physical page
 * page_table[i][t / P] at slot t % P; cache layout [page][kv_head][slot][D].
 * Query head h reads kv head h / (Hq / Hkv).
 *   s_t = scale * <q, k_t>;  w_t = exp(s_t - max s);  O = sum w_t v_t / sum w_t
 * out is fp32 [M, Hq, D]; lse (optional) = max s + log(sum w) per (row, head).
 * ------------------------------------------------------------------------- */
int oracle_verify_attn(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                       const int32_t* page_table, int max_pages_per_seq,
                       const int32_t* seq_lens, const int32_t* qo_indptr,
                       float* out, float* lse,
                       int B, int M, int Hq, int Hkv, int D, int page_size, float scale)
{
    if (!q || !k_cache || !v_cache || !page_table || !seq_lens || !qo_indptr || !out) return ORACLE_EINVAL;
    if (B < 0 || M < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || page_size <= 0 || Hq % Hkv) return ORACLE_EINVAL;
    const int G = Hq / Hkv;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int i = 0; i < B; ++i) {
        for (int h = 0; h < Hq; ++h) {
            const int r0 = qo_indptr[i], n = qo_indptr[i + 1] - qo_indptr[i];
            const int c = seq_lens[i];
            const int kvh = h / G;
            double* s = (double*)malloc(sizeof(double) * (size_t)(c + n > 0 ? c + n : 1));
            double* acc = (double*)malloc(sizeof(double) * (size_t)D);
            for (int j = 0; j < n; ++j) {
                const int row = r0 + j;
                const int nk = c + j + 1;
                const uint16_t* qv = q + ((size_t)row * Hq + h) * D;
                double m = -INFINITY;
                for (int t = 0; t < nk; ++t) {
                    const int page = page_table[(size_t)i * max_pages_per_seq + t / page_size];
                    if (page < 0) { status = ORACLE_EINVAL; s[t] = -INFINITY; continue; }
                    const uint16_t* kv = k_cache + (((size_t)page * Hkv + kvh) * page_size + t % page_size) * D;
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += (double)bf16_bits_to_float(qv[d]) * (double)bf16_bits_to_float(kv[d]);
                    s[t] = (double)scale * dot;
                    if (s[t] > m) m = s[t];
                }
                for (int d = 0; d < D; ++d) acc[d] = 0.0;
                double denom = 0.0;
                for (int t = 0; t < nk; ++t) {
                    const int page = page_table[(size_t)i * max_pages_per_seq + t / page_size];
                    if (page < 0) continue;
                    const double w = exp(s[t] - m);
                    denom += w;
                    const uint16_t* vv = v_cache + (((size_t)page * Hkv + kvh) * page_size + t % page_size) * D;
                    for (int d = 0; d < D; ++d) acc[d] += w * (double)bf16_bits_to_float(vv[d]);
                }
                float* o = out + ((size_t)row * Hq + h) * D;
                for (int d = 0; d < D; ++d) o[d] = (float)(acc[d] / denom);
                if (lse) lse[(size_t)row * Hq + h] = (float)(m + log(denom));
            }
            free(s);
            free(acc);
        }
    }
    return status;
}

/* ------------------------------------------------------------------------- *
 * LM head: one logits row per candidate position (every position of Y_n must
 * be scored).  logits[r][v] = sum_k hidden[r][k] * W[v][k], fp64 sum, fp32 out.
 * ------------------------------------------------------------------------- */
int oracle_lm_head(const uint16_t* hidden, const uint16_t* W, float* logits, int M, int H, int V)
{
    if (!hidden || !W || !logits || M < 0 || H <= 0 || V < 0) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (long v = 0; v < V; ++v) {
        const uint16_t* w = W + (size_t)v * H;
        for (int r = 0; r < M; ++r) {
            const uint16_t* x = hidden + (size_t)r * H;
            double dot = 0.0;
            for (int k = 0; k < H; ++k)
                dot += (double)bf16_bits_to_float(x[k]) * (double)bf16_bits_to_float(w[k]);
            logits[(size_t)r * V + v] = (float)dot;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplies with the key
 * bumped by the Weyl constants between rounds.
 * ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
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

/* The uniform the acceptance rule draws: counter (0, j, tag, round), key =
 * the two halves of the per-request seed, first output word, top 24 bits.
 * tag 0 = accept test of draft j, tag 1 = the bonus/residual draw at row j. */
float oracle_uniform(uint64_t seed, uint32_t round, uint32_t j, uint32_t tag)
{
    const uint32_t ctr[4] = {0u, j, tag, round};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    oracle_philox4x32_10(ctr, key, x);
    return (float)(x[0] >> 8) * (1.0f / 16777216.0f);
}

/* Target distribution of one logits row at temperature T (> 0):
 * p(v) = float( exp((l_v - max l) / T) / sum_w exp((l_w - max l) / T) ), fp64
 * inside.  Returns 0 if the row is unusable (NaN present or max not finite). */
static int row_is_valid(const float* l, int V)
{
    float m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        if (l[v] != l[v]) return 0;
        if (l[v] > m) m = l[v];
    }
    return isfinite(m);
}

int oracle_target_probs(const float* l, int V, float T, float* p)
{
    if (!l || !p || V <= 0 || !(T > 0.0f)) return ORACLE_EINVAL;
    if (!row_is_valid(l, V)) return ORACLE_EINVAL;
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) if ((double)l[v] > m) m = (double)l[v];
    double Z = 0.0;
    for (int v = 0; v < V; ++v) Z += exp(((double)l[v] - m) / (double)T);
    for (int v = 0; v < V; ++v) p[v] = (float)(exp(((double)l[v] - m) / (double)T) / Z);
    return ORACLE_OK;
}

static int row_argmax(const float* l, int V)
{
    int best = 0;
    for (int v = 1; v < V; ++v) if (l[v] > l[best]) best = v;   /* ties: lowest index */
    return best;
}

/* Inverse-CDF draw from weights rho (>= 0) with uniform u in [0,1): smallest v
 * whose running fp64 sum exceeds u * total; if rounding lets the loop run out,
 * the last v with positive weight. */
static int sample_from_weights(const float* rho, int V, double total, float u)
{
    const double t = (double)u * total;
    double run = 0.0;
    int last = -1;
    for (int v = 0; v < V; ++v) {
        run += (double)rho[v];
        if (rho[v] > 0.0f) last = v;
        if (run > t) return v;
    }
    return last;
}

/* ------------------------------------------------------------------------- *
 * Acceptance.  Per request i with rows r_j = qo_indptr[i] + j, j = 0..gamma_i:
 *  T_i == 0  greedy: g_j = argmax of row j; accept d_j while d_j == g_{j-1};
 *            the emitted bonus is g_a at the first mismatch (or g_gamma).
 *  T_i  > 0  rejection sampling: p_j = softmax(row j / T).  For j = 1..gamma:
 *            accept d_j iff u_j * q_j(d_j) < p_{j-1}(d_j); at the first
 *            rejection j* draw the bonus from norm(max(0, p_{j*-1} - q_{j*}));
 *            if nothing is rejected draw it from p_gamma.
 *            draft_probs == NULL means the drafter is deterministic: q_j is
 *            one-hot at d_j.
 * Outputs: accept_len[i] = a; out_tokens[i] = [d_1..d_a, bonus, -1, ...]
 * (row stride gamma_max + 1); rollback[i] = (a < gamma_i).
 * A request any of whose rows holds a NaN or has a non-finite maximum yields
 * a = 0 and bonus -1 and ORs bit 0 into *status_flags.
 * ------------------------------------------------------------------------- */
int oracle_accept(const float* logits, const int32_t* tokens, const float* draft_probs,
                  const float* temperature, const uint64_t* seeds, uint32_t round,
                  const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens,
                  uint8_t* rollback, int32_t* status_flags, int B, int M, int V, int gamma_max)
{
    if (!logits || !tokens || !temperature || !qo_indptr || !accept_len || !out_tokens) return ORACLE_EINVAL;
    if (B < 0 || M < 0 || V <= 0 || gamma_max < 0) return ORACLE_EINVAL;
    int flags = 0, bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(|:flags) reduction(|:bad)
    for (int i = 0; i < B; ++i) {
        const int r0 = qo_indptr[i];
        const int gamma = qo_indptr[i + 1] - r0 - 1;
        int32_t* emit = out_tokens + (size_t)i * (gamma_max + 1);
        for (int j = 0; j <= gamma_max; ++j) emit[j] = -1;
        accept_len[i] = 0;
        if (rollback) rollback[i] = 0;
        if (gamma < 0 || gamma > gamma_max) { bad = 1; continue; }
        const float T = temperature[i];
        if (T > 0.0f && !seeds) { bad = 1; continue; }
        int valid = 1;
        for (int j = 0; j <= gamma; ++j) valid &= row_is_valid(logits + (size_t)(r0 + j) * V, V);
        for (int j = 1; j <= gamma; ++j) valid &= (tokens[r0 + j] >= 0 && tokens[r0 + j] < V);
        if (!valid || !(T >= 0.0f)) {
            flags |= 1;
            if (rollback) rollback[i] = (uint8_t)(gamma > 0);
            continue;
        }
        int a = 0, bonus = -1;
        if (T == 0.0f) {
            while (a < gamma && tokens[r0 + a + 1] == row_argmax(logits + (size_t)(r0 + a) * V, V)) ++a;
            bonus = row_argmax(logits + (size_t)(r0 + a) * V, V);
        } else {
            float* p = (float*)malloc(sizeof(float) * (size_t)V);
            float* rho = (float*)malloc(sizeof(float) * (size_t)V);
            int rejected_at = 0;                       /* j* (1-based), 0 = none */
            for (int j = 1; j <= gamma; ++j) {
                oracle_target_probs(logits + (size_t)(r0 + j - 1) * V, V, T, p);
                const int d = tokens[r0 + j];
                const float qd = draft_probs ? draft_probs[(size_t)(r0 - i + j - 1) * V + d] : 1.0f;
                const float u = oracle_uniform(seeds[i], round, (uint32_t)j, 0u);
                if ((float)((double)u * (double)qd) < p[d]) { ++a; }
                else { rejected_at = j; break; }
            }
            if (rejected_at) {
                /* p still holds p_{j*-1} */
                const int d = tokens[r0 + rejected_at];
                const float* qrow = draft_probs ? draft_probs + (size_t)(r0 - i + rejected_at - 1) * V : NULL;
                double total = 0.0;
                for (int v = 0; v < V; ++v) {
                    const float qv = qrow ? qrow[v] : (v == d ? 1.0f : 0.0f);
                    const float diff = p[v] - qv;
                    rho[v] = diff > 0.0f ? diff : 0.0f;
                    total += (double)rho[v];
                }
                if (!(total > 0.0)) {              /* p == q numerically: fall back to p */
                    total = 0.0;
                    for (int v = 0; v < V; ++v) { rho[v] = p[v]; total += (double)p[v]; }
                }
                bonus = sample_from_weights(rho, V, total, oracle_uniform(seeds[i], round, (uint32_t)rejected_at, 1u));
            } else {
                oracle_target_probs(logits + (size_t)(r0 + gamma) * V, V, T, p);
                double total = 0.0;
                for (int v = 0; v < V; ++v) total += (double)p[v];
                bonus = sample_from_weights(p, V, total, oracle_uniform(seeds[i], round, (uint32_t)(gamma + 1), 1u));
            }
            free(p);
            free(rho);
        }
        accept_len[i] = a;
        for (int j = 0; j < a; ++j) emit[j] = tokens[r0 + j + 1];
        emit[a] = bonus;
        if (rollback) rollback[i] = (uint8_t)(a < gamma);
    }
    if (status_flags) *status_flags |= flags;
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Commit (Appendix "Target side": p_{n+1} = Commit(p_n, y_n, L_n); only
 * verified tokens enter the committed prefix) on the KV side.  Before the
 * step request i owns ceil((c_i + n_i) / P) pages (the candidate's K/V were
 * written at positions c_i .. c_i + gamma_i).  Afterwards its length is
 * c_i + a_i + 1 (accepted drafts plus the row that produced the bonus; the
 * bonus token's own K/V is written by the next step) and every page beyond
 * ceil(new_len / P) is unmapped (-1) and pushed on the free list, requests in
 * ascending order, logical pages in ascending order.
 * ------------------------------------------------------------------------- */
int oracle_kv_commit(int32_t* page_table, int max_pages_per_seq, int32_t* seq_lens,
                     const int32_t* qo_indptr, const int32_t* accept_len,
                     int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                     int B, int page_size)
{
    if (!page_table || !seq_lens || !qo_indptr || !accept_len || !free_list || !free_count) return ORACLE_EINVAL;
    if (B < 0 || page_size <= 0 || max_pages_per_seq < 0) return ORACLE_EINVAL;
    int status = ORACLE_OK;
    for (int i = 0; i < B; ++i) {
        const int n = qo_indptr[i + 1] - qo_indptr[i];
        const int c = seq_lens[i];
        int a = accept_len[i];
        if (a < 0) a = 0;
        if (a > n - 1) a = n - 1;
        const int new_len = c + a + 1;
        const int had = (c + n + page_size - 1) / page_size;
        const int keep = (new_len + page_size - 1) / page_size;
        for (int pg = keep; pg < had && pg < max_pages_per_seq; ++pg) {
            int32_t* slot = page_table + (size_t)i * max_pages_per_seq + pg;
            if (*slot >= 0) {
                if (*free_count < free_capacity) free_list[(*free_count)++] = *slot;
                else status = ORACLE_EINVAL;
                *slot = -1;
            }
        }
        seq_lens[i] = new_len;
    }
    return status;
}

/* ------------------------------------------------------------------------- *
 * Rollback ratio and the mode threshold (Section "Throughput-Guided Hybrid
 * Coordination", eq. r_threshold; Method, eq. mode_switch_batch).
 * ------------------------------------------------------------------------- */
double oracle_thr_ordinary(double B, double L, double gamma, double T_D, double T_T)
{
    return B * L / (T_T + (gamma - 1.0) * T_D);
}

double oracle_thr_parallel(double B, double L, double r, double T_T)
{
    return B * (r + (1.0 - r) * L) / T_T;
}

double oracle_r_star(double L, double gamma, double T_D, double T_T)
{
    return (gamma - 1.0) * L * T_D / ((T_T + (gamma - 1.0) * T_D) * (L - 1.0));
}

/* Mode of round n+1 (Method, eq. mode_switch_batch): 1 = PARALLEL iff r_hat = |R_n| / B <= r*, else
 * 0 = ORDINARY.  L is the mean number of tokens a request emitted in round n.  With L <= 1 the
 * derivation's assumption L > 1 fails: speculation then yields one token per request either way, the
 * ordinary round is longer by (gamma-1) T_D, so PARALLEL is never worse and is returned. */
int oracle_next_mode(int rollback_count, int emitted, int B, double gamma, double T_D, double T_T,
                     double* r_hat_out, double* r_star_out)
{
    double r_hat = (double)rollback_count / (double)B;
    double L = (double)emitted / (double)B;
    double rs = L > 1.0 ? oracle_r_star(L, gamma, T_D, T_T) : INFINITY;
    if (r_hat_out) *r_hat_out = r_hat;
    if (r_star_out) *r_star_out = rs;
    return r_hat <= rs ? 1 : 0;
}

/* ------------------------------------------------------------------------- *
 * Candidates of round n+1 (Method, "Execution in ordinary mode" / "Execution in
 * parallel mode", eqs. ordinary_rollback_seq, ordinary_stable_seq,
 * parallel_stable_seq, parallel_rollback_pad; Appendix "Target side",
 * eq. target_suffix_reuse).  Per request, after round n: a = accepted drafts,
 * b = bonus token (out_tokens[i][a]), gamma_i = drafts that were verified.
 *   cont[i][0 .. cont_len[i])   the continuation the drafter prepared while round n
 *                               was verified: what it expects AFTER the verified
 *                               drafts; its first token is its guess of b.
 *   repair[i][0 .. repair_len[i])  ordinary mode only: the continuation regenerated
 *                               from b for a rollback request.
 * A request is stable iff all its drafts were accepted and the prepared
 * continuation agrees with what the target committed, i.e. cont_len >= 1 and
 * cont[0] == b (the reading taken for Consistent()); otherwise it is in the
 * rollback set (Method, "Rollback-Based Mode Selection": membership means that
 * some verified draft was not accepted, or that the continuation prepared in the
 * meantime no longer fits what verification produced).
 *   stable:              y = [b, cont[1 .. 1+g)]           g = min(cont_len-1, gamma_next)
 *   rollback, ORDINARY:  y = [b, repair[0 .. g)]           g = min(repair_len, gamma_next)
 *   rollback, PARALLEL:  y = [b]                           (the padded candidate, ragged)
 * A request whose acceptance failed (bonus < 0) gets the single row [-1].
 * Writes next_tokens (rows of all requests, request order), next_qo_indptr [B+1],
 * rollback [B], stats = {|R_n|, sum (a+1), B, rows of round n+1}.
 * mode: 0 = ORDINARY, 1 = PARALLEL.  Returns the number of rows, or < 0.
 * ------------------------------------------------------------------------- */
int oracle_assemble_next(const int32_t* accept_len, const int32_t* out_tokens, int gamma_max,
                         const int32_t* qo_indptr, int B,
                         const int32_t* cont, int cont_stride, const int32_t* cont_len,
                         const int32_t* repair, int repair_stride, const int32_t* repair_len,
                         int mode, int gamma_next,
                         int32_t* next_tokens, int32_t* next_qo_indptr, uint8_t* rollback, int32_t* stats)
{
    if (!accept_len || !out_tokens || !qo_indptr || !next_tokens || !next_qo_indptr) return ORACLE_EINVAL;
    if (B < 0 || gamma_max < 0 || gamma_next < 0 || (mode != 0 && mode != 1)) return ORACLE_EINVAL;
    int rows = 0, rolled = 0, emitted = 0;
    next_qo_indptr[0] = 0;
    for (int i = 0; i < B; ++i) {
        const int gamma = qo_indptr[i + 1] - qo_indptr[i] - 1;
        const int a = accept_len[i];
        const int ok = gamma >= 0 && gamma <= gamma_max && a >= 0 && a <= gamma;
        const int b = ok ? out_tokens[(size_t)i * (gamma_max + 1) + a] : -1;
        int is_rollback = 1, g = 0;
        const int32_t* from = NULL;
        if (b >= 0) {
            const int cl = (cont && cont_len) ? cont_len[i] : 0;
            if (a == gamma && cl >= 1 && cont[(size_t)i * cont_stride] == b) {
                is_rollback = 0;
                g = cl - 1 < gamma_next ? cl - 1 : gamma_next;
                from = cont + (size_t)i * cont_stride + 1;
            } else if (mode == 0 && repair && repair_len) {
                g = repair_len[i] < gamma_next ? repair_len[i] : gamma_next;
                if (g < 0) g = 0;
                from = repair + (size_t)i * repair_stride;
            }
            emitted += a + 1;
        } else {
            is_rollback = gamma > 0;          /* what spec_accept reports for a request it could not decide */
        }
        next_tokens[rows++] = b;
        for (int j = 0; j < g; ++j) next_tokens[rows++] = from[j];
        next_qo_indptr[i + 1] = rows;
        if (rollback) rollback[i] = (uint8_t)is_rollback;
        rolled += is_rollback;
    }
    if (stats) { stats[0] = rolled; stats[1] = emitted; stats[2] = B; stats[3] = rows; }
    return rows;
}

/* ------------------------------------------------------------------------- *
 * Draft-side reconciliation (Appendix "Draft side", "Message handling and
 * update"): delta_i = min{ t : p_i[t] != h_i[t] }, the first position at which
 * the verified prefix p_i and the draft's own decoded tokens h_i differ
 * (0-based over the ragged rows p_indptr / h_indptr).  When one is a prefix of
 * the other there is no such t and delta_i is the shorter length: everything
 * the two share is kept.
 * ------------------------------------------------------------------------- */
int oracle_divergence(const int32_t* p_tokens, const int32_t* p_indptr, const int32_t* h_tokens,
                      const int32_t* h_indptr, int32_t* delta, int B)
{
    if (!p_indptr || !h_indptr || !delta || B < 0) return ORACLE_EINVAL;
    for (int i = 0; i < B; ++i) {
        const int lp = p_indptr[i + 1] - p_indptr[i], lh = h_indptr[i + 1] - h_indptr[i];
        const int n = lp < lh ? lp : lh;
        int t = 0;
        while (t < n && p_tokens[p_indptr[i] + t] == h_tokens[h_indptr[i] + t]) ++t;
        delta[i] = t;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- *
 * Rollback(S, delta) on the paged KV cache (Appendix "Draft side", "State
 * recovery": rollback truncates the speculative suffix and frees the
 * corresponding KV cache).  Request i keeps min(len_i, max(keep_len[i], 0))
 * tokens; the pages beyond ceil(new_len / P), up to ceil(len_i / P), are unmapped
 * and pushed on the free list, requests ascending, logical pages ascending.
 * ------------------------------------------------------------------------- */
int oracle_kv_truncate(int32_t* page_table, int max_pages_per_seq, int32_t* seq_lens, const int32_t* keep_len,
                       int32_t* free_list, int32_t free_capacity, int32_t* free_count, int B, int page_size)
{
    if (!page_table || !seq_lens || !keep_len || !free_list || !free_count) return ORACLE_EINVAL;
    if (B < 0 || page_size <= 0 || max_pages_per_seq < 0) return ORACLE_EINVAL;
    int status = ORACLE_OK;
    for (int i = 0; i < B; ++i) {
        const int c = seq_lens[i];
        int k = keep_len[i];
        if (k < 0) k = 0;
        if (k > c) k = c;
        const int had = (c + page_size - 1) / page_size;
        const int keep = (k + page_size - 1) / page_size;
        for (int pg = keep; pg < had && pg < max_pages_per_seq; ++pg) {
            int32_t* slot = page_table + (size_t)i * max_pages_per_seq + pg;
            if (*slot >= 0) {
                if (*free_count < free_capacity) free_list[(*free_count)++] = *slot;
                else status = ORACLE_EINVAL;
                *slot = -1;
            }
        }
        seq_lens[i] = k;
    }
    return status;
}

/* ------------------------------------------------------------------------- *
 * Draft-side context compression (Method, "Draft-side context compression",
 * eq. token_eviction): E(x_{1:S}) = [x_{:k}, x_{S-k+1:}], k = floor(p S / 2),
 * the first k and the last k tokens of a prompt, 2k <= p S of them, with the
 * retained ratio p = p_num / p_den given as a fraction so that k is an exact
 * integer: k = (p_num * S) / (2 * p_den).  A prompt with 2k >= S is kept whole.
 * Ragged in (tokens, indptr [B+1]) and out; kept_index (optional) receives the
 * position inside its prompt of every kept token.  Returns the number of
 * tokens kept, or < 0.
 * ------------------------------------------------------------------------- */
long oracle_compress_prompts(const int32_t* tokens, const int32_t* indptr, int B, int p_num, int p_den,
                             int32_t* out_tokens, int32_t* out_indptr, int32_t* kept_index)
{
    if (!indptr || !out_indptr || B < 0 || p_num < 0 || p_den <= 0) return ORACLE_EINVAL;
    long n = 0;
    out_indptr[0] = 0;
    for (int i = 0; i < B; ++i) {
        const long S = indptr[i + 1] - indptr[i];
        const long k = (long)p_num * S / (2L * p_den);
        const int32_t* x = tokens + indptr[i];
        if (2 * k >= S) {
            for (long t = 0; t < S; ++t) { out_tokens[n] = x[t]; if (kept_index) kept_index[n] = (int32_t)t; ++n; }
        } else {
            for (long t = 0; t < k; ++t) { out_tokens[n] = x[t]; if (kept_index) kept_index[n] = (int32_t)t; ++n; }
            for (long t = S - k; t < S; ++t) { out_tokens[n] = x[t]; if (kept_index) kept_index[n] = (int32_t)t; ++n; }
        }
        out_indptr[i + 1] = (int32_t)n;
    }
    return n;
}

/* ------------------------------------------------------------------------- *
 * Tree-structured verification (Appendix "Target side", "Unified verification
 * interface": the remote tokens are turned into a verification tree T_n^(i);
 * a single remote sequence is the chain handled above).  The candidate rows of
 * a request form a tree: row 0 is the root (the last committed / bonus token),
 * parent[r0 + j] is the row-local index of the parent of row j (parent < j,
 * -1 for the root).  The K/V of row j sits at cache position c_i + j.
 *
 * Attention: row j attends to the committed prefix 0 .. c_i - 1 and to the
 * candidate rows on its own path to the root, itself included.
 * ------------------------------------------------------------------------- */
static int tree_ok(const int32_t* parent, int n)
{
    if (n < 1 || parent[0] != -1) return 0;
    for (int j = 1; j < n; ++j) if (parent[j] < 0 || parent[j] >= j) return 0;
    return 1;
}

int oracle_verify_attn_tree(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                            const int32_t* page_table, int max_pages_per_seq,
                            const int32_t* seq_lens, const int32_t* qo_indptr, const int32_t* parent,
                            float* out, float* lse,
                            int B, int M, int Hq, int Hkv, int D, int page_size, float scale)
{
    if (!q || !k_cache || !v_cache || !page_table || !seq_lens || !qo_indptr || !parent || !out) return ORACLE_EINVAL;
    if (B < 0 || M < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || page_size <= 0 || Hq % Hkv) return ORACLE_EINVAL;
    const int G = Hq / Hkv;
    int status = ORACLE_OK;
    for (int i = 0; i < B; ++i) {
        const int r0 = qo_indptr[i], n = qo_indptr[i + 1] - qo_indptr[i], c = seq_lens[i];
        if (!tree_ok(parent + r0, n)) { status = ORACLE_EINVAL; continue; }
        char* visible = (char*)malloc((size_t)(c + n));
        double* s = (double*)malloc(sizeof(double) * (size_t)(c + n));
        double* acc = (double*)malloc(sizeof(double) * (size_t)D);
        for (int j = 0; j < n; ++j) {
            for (int t = 0; t < c + n; ++t) visible[t] = t < c;
            for (int a = j; a >= 0; a = parent[r0 + a]) visible[c + a] = 1;
            for (int h = 0; h < Hq; ++h) {
                const int kvh = h / G, row = r0 + j;
                const uint16_t* qv = q + ((size_t)row * Hq + h) * D;
                double m = -INFINITY;
                for (int t = 0; t < c + n; ++t) {
                    if (!visible[t]) continue;
                    const int page = page_table[(size_t)i * max_pages_per_seq + t / page_size];
                    if (page < 0) { status = ORACLE_EINVAL; visible[t] = 0; continue; }
                    const uint16_t* kv = k_cache + (((size_t)page * Hkv + kvh) * page_size + t % page_size) * D;
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d) dot += (double)bf16_bits_to_float(qv[d]) * (double)bf16_bits_to_float(kv[d]);
                    s[t] = (double)scale * dot;
                    if (s[t] > m) m = s[t];
                }
                for (int d = 0; d < D; ++d) acc[d] = 0.0;
                double denom = 0.0;
                for (int t = 0; t < c + n; ++t) {
                    if (!visible[t]) continue;
                    const int page = page_table[(size_t)i * max_pages_per_seq + t / page_size];
                    const double w = exp(s[t] - m);
                    denom += w;
                    const uint16_t* vv = v_cache + (((size_t)page * Hkv + kvh) * page_size + t % page_size) * D;
                    for (int d = 0; d < D; ++d) acc[d] += w * (double)bf16_bits_to_float(vv[d]);
                }
                float* o = out + ((size_t)row * Hq + h) * D;
                for (int d = 0; d < D; ++d) o[d] = (float)(acc[d] / denom);
                if (lse) lse[(size_t)row * Hq + h] = (float)(m + log(denom));
            }
        }
        free(visible); free(s); free(acc);
    }
    return status;
}

/* Greedy acceptance on a tree: from the root, follow the child whose token is the argmax of the current
 * node's logits row (lowest index wins ties; the lowest row among equal children) as long as there is one.
 * accept_len = drafts accepted, out_tokens = their tokens then the bonus (the argmax at the last node), path =
 * row-local indices of the visited nodes (path[0] = 0), -1 padded.  rollback = the last node still had children
 * (the drafter went on from it, but not with the token the target produced).  A NaN row, a row maximum that is
 * not finite, a token outside [0, V) or a malformed tree: a = 0, tokens -1, path = {0}, a status bit. */
int oracle_accept_tree(const float* logits, const int32_t* tokens, const int32_t* parent, const int32_t* qo_indptr,
                       int32_t* accept_len, int32_t* out_tokens, int32_t* path, uint8_t* rollback, int32_t* status_flags,
                       int B, int M, int V, int gamma_max)
{
    if (!logits || !tokens || !parent || !qo_indptr || !accept_len || !out_tokens || !path) return ORACLE_EINVAL;
    if (B < 0 || M < 0 || V <= 0 || gamma_max < 0) return ORACLE_EINVAL;
    for (int i = 0; i < B; ++i) {
        const int r0 = qo_indptr[i], n = qo_indptr[i + 1] - qo_indptr[i];
        int32_t* emit = out_tokens + (size_t)i * (gamma_max + 1);
        int32_t* pth = path + (size_t)i * (gamma_max + 1);
        for (int k = 0; k <= gamma_max; ++k) { emit[k] = -1; pth[k] = -1; }
        pth[0] = 0;
        accept_len[i] = 0;
        if (rollback) rollback[i] = 0;
        int flags = 0;
        if (n < 1 || n - 1 > gamma_max || !tree_ok(parent + r0, n)) flags |= 2;
        int* arg = (int*)malloc(sizeof(int) * (size_t)(n > 0 ? n : 1));
        if (!flags) {
            for (int j = 0; j < n; ++j) {
                const float* l = logits + (size_t)(r0 + j) * V;
                int best = 0, bad = 0;
                for (int v = 0; v < V; ++v) { if (l[v] != l[v]) bad = 1; if (l[v] > l[best]) best = v; }
                if (bad || !(l[best] > -INFINITY && l[best] < INFINITY)) flags |= 4;
                arg[j] = best;
                if (j > 0 && (tokens[r0 + j] < 0 || tokens[r0 + j] >= V)) flags |= 8;
            }
        }
        if (flags) {
            if (status_flags) *status_flags |= flags;
            if (rollback) rollback[i] = (uint8_t)(n > 1);
            free(arg);
            continue;
        }
        int u = 0, a = 0;
        for (;;) {
            int next = -1;
            for (int v = u + 1; v < n; ++v)
                if (parent[r0 + v] == u && tokens[r0 + v] == arg[u]) { next = v; break; }
            if (next < 0) break;
            emit[a] = tokens[r0 + next];
            ++a;
            pth[a] = next;
            u = next;
        }
        emit[a] = arg[u];
        accept_len[i] = a;
        int has_child = 0;
        for (int v = u + 1; v < n; ++v) if (parent[r0 + v] == u) has_child = 1;
        if (rollback) rollback[i] = (uint8_t)has_child;
        free(arg);
    }
    return ORACLE_OK;
}

/* Commit of an accepted tree path: the K/V of the accepted nodes (cache positions c + path[k], k = 1 .. a) are
 * moved to positions c + 1 .. c + a, so that the committed prefix is contiguous again; then lengths, page table
 * and free list are updated exactly as by oracle_kv_commit (new length c + a + 1). */
int oracle_kv_commit_tree(uint16_t* k_cache, uint16_t* v_cache, int32_t* page_table, int max_pages_per_seq,
                          int32_t* seq_lens, const int32_t* qo_indptr, const int32_t* accept_len,
                          const int32_t* path, int gamma_max,
                          int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                          int B, int Hkv, int D, int page_size)
{
    if (!k_cache || !v_cache || !page_table || !seq_lens || !qo_indptr || !accept_len || !path) return ORACLE_EINVAL;
    for (int i = 0; i < B; ++i) {
        const int n = qo_indptr[i + 1] - qo_indptr[i], c = seq_lens[i];
        int a = accept_len[i];
        if (a < 0) a = 0;
        if (a > n - 1) a = n - 1;
        for (int k = 1; k <= a; ++k) {
            const int src = c + path[(size_t)i * (gamma_max + 1) + k], dst = c + k;
            if (src == dst) continue;
            if (src < dst || src >= c + n) return ORACLE_EINVAL;
            const int ps = page_table[(size_t)i * max_pages_per_seq + src / page_size];
            const int pd = page_table[(size_t)i * max_pages_per_seq + dst / page_size];
            if (ps < 0 || pd < 0) return ORACLE_EINVAL;
            for (int h = 0; h < Hkv; ++h) {
                const size_t so = (((size_t)ps * Hkv + h) * page_size + src % page_size) * D;
                const size_t dn = (((size_t)pd * Hkv + h) * page_size + dst % page_size) * D;
                memcpy(k_cache + dn, k_cache + so, sizeof(uint16_t) * (size_t)D);
                memcpy(v_cache + dn, v_cache + so, sizeof(uint16_t) * (size_t)D);
            }
        }
    }
    return oracle_kv_commit(page_table, max_pages_per_seq, seq_lens, qo_indptr, accept_len, free_list, free_capacity,
                            free_count, B, page_size);
}

