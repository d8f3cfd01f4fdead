/*
 * CPU checker for the Sequoia verification walk.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product path may call this.
 *
 * What is computed.  Algorithm 2 ("Sequoia Sampling and Verification", Sec. 3.2.1) applied
 * recursively from the root of the token tree (Sec. 2.2: every such method starts at the
 * root and goes on at the child it accepts).  It is a randomized procedure, so the
 * checker is the procedure itself, run on uniforms handed in by the caller, step by step in
 * the algorithm's own notation:
 *
 *   at node v:   R <- P(.|v)   D <- Q(.|v)   S <- {}                       (initialisation)
 *   for every child c of v, in ascending node id (= the order the drafter sampled them):
 *       s <- tree_tokens[c]   r <- uniforms[c]
 *       if r < R[s] / D[s]:  accept c, continue the walk at c              (accept test)
 *       else  R <- norm(max(R - D, 0))                                    (residual update)
 *             D[s] <- 0 ; S.add(s)                                        (no second mistake)
 *             if sum(D) = 0:  D[t] <- 0 if t in S else 1                  (uniform fallback)
 *             D <- norm(D)
 *   no child accepted (or v is a leaf):  return x ~ R                     (bonus token)
 *
 * P and Q are softmax(logits / T) of row v of the target and draft logits.  T = 0 means
 * greedy decoding: one-hot at the arg-max, lowest index on ties.
 *
 * Readings where the paper is silent:
 *   - the same temperature tempers both models (every table row has one T);
 *   - uniforms[c] decides node c, uniforms[0] draws the bonus token;
 *   - "x ~ R" is the inverse CDF in ascending token id: the first x whose inclusive
 *     cumulative mass exceeds u * sum(R); if rounding leaves none, the last x with R[x] > 0;
 *   - D[s] = 0 for a supplied token (impossible for a tree really drawn from D): the ratio is
 *     +infinity when R[s] > 0 and 0 when R[s] = 0;
 *   - sum(max(R - D, 0)) = 0 on a rejection (impossible in exact arithmetic, see the Lemma in
 *     App. "Proof of correctness"): R is left unchanged and the event is counted.
 *
 * Arithmetic is fp64.  Logits and uniforms arrive as float (an exact container for bf16 and
 * fp32 inputs).  One thread; every vocabulary-wide step is a plain loop.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_DECISION_DOUBLES 8 /* node, token, u, R[s], D[s], ratio, accepted, parent */
#define ORACLE_BONUS_DOUBLES 8    /* stop node, u0, sum(R), cdf_lo, cdf_hi, margin, token, 0 */

static void tempered_softmax(const float* logits, int32_t V, double T, double* out)
{
    if (T == 0.0) {
        int32_t best = 0;
        for (int32_t x = 1; x < V; ++x)
            if ((double)logits[x] > (double)logits[best]) best = x;
        for (int32_t x = 0; x < V; ++x) out[x] = 0.0;
        out[best] = 1.0;
        return;
    }
    double m = -INFINITY;
    for (int32_t x = 0; x < V; ++x)
        if ((double)logits[x] > m) m = (double)logits[x];
    double z = 0.0;
    for (int32_t x = 0; x < V; ++x) {
        out[x] = exp(((double)logits[x] - m) / T);
        z += out[x];
    }
    for (int32_t x = 0; x < V; ++x) out[x] /= z;
}

/*
 * target_logits, draft_logits [n][V]; tree_tokens [n]; parent [n]; uniforms [n].
 * accepted_path [n]: accepted node ids root-to-leaf, then -1.  bonus_token [1].
 * Optional outputs (NULL to skip):
 *   decisions [ (n-1) * 8 ] one record per accept test, in order; *n_decisions their number;
 *   bonus_info [8]; final_R [V], final_D [V]: R and D at the moment the bonus token is drawn;
 *   counters [2]: number of degenerate residual updates, number of uniform fallbacks.
 */
int oracle_verify(const float* target_logits, const float* draft_logits,
                  const int32_t* tree_tokens, const int32_t* parent, double temperature,
                  const float* uniforms, int32_t n, int32_t V,
                  int32_t* accepted_path, int32_t* bonus_token,
                  double* decisions, int32_t* n_decisions, double* bonus_info,
                  double* final_R, double* final_D, int32_t* counters)
{
    if (n < 1 || V < 1 || !(temperature >= 0.0) || parent[0] != -1) return -1;
    for (int32_t i = 1; i < n; ++i) {
        if (parent[i] < 0 || parent[i] >= i) return -1;
        if (tree_tokens[i] < 0 || tree_tokens[i] >= V) return -1;
    }
    double* R = (double*)malloc(sizeof(double) * (size_t)V);
    double* D = (double*)malloc(sizeof(double) * (size_t)V);
    double* tmp = (double*)malloc(sizeof(double) * (size_t)V);
    unsigned char* inS = (unsigned char*)malloc((size_t)V);
    if (!R || !D || !tmp || !inS) { free(R); free(D); free(tmp); free(inS); return -2; }

    int32_t n_dec = 0, path_len = 0, degenerate = 0, fallbacks = 0;
    for (int32_t i = 0; i < n; ++i) accepted_path[i] = -1;

    int32_t v = 0;
    for (;;) {
        tempered_softmax(target_logits + (size_t)v * V, V, temperature, R);
        tempered_softmax(draft_logits + (size_t)v * V, V, temperature, D);
        memset(inS, 0, (size_t)V);

        int32_t next = -1;
        for (int32_t c = v + 1; c < n && next < 0; ++c) {
            if (parent[c] != v) continue;
            const int32_t s = tree_tokens[c];
            const double r = (double)uniforms[c];
            double ratio;
            if (D[s] > 0.0) ratio = R[s] / D[s];
            else ratio = (R[s] > 0.0) ? INFINITY : 0.0;
            const int accept = (r < ratio);
            if (decisions) {
                double* rec = decisions + (size_t)n_dec * ORACLE_DECISION_DOUBLES;
                rec[0] = c; rec[1] = s; rec[2] = r; rec[3] = R[s]; rec[4] = D[s];
                rec[5] = ratio; rec[6] = accept; rec[7] = v;
            }
            ++n_dec;
            if (accept) { next = c; break; }

            /* R <- norm(max(R - D, 0)) */
            double sum = 0.0;
            for (int32_t x = 0; x < V; ++x) {
                const double diff = R[x] - D[x];
                tmp[x] = diff > 0.0 ? diff : 0.0;
                sum += tmp[x];
            }
            if (sum > 0.0) { for (int32_t x = 0; x < V; ++x) R[x] = tmp[x] / sum; }
            else ++degenerate;
            /* D[s] <- 0, S.add(s) */
            D[s] = 0.0;
            inS[s] = 1;
            double sumD = 0.0;
            for (int32_t x = 0; x < V; ++x) sumD += D[x];
            if (sumD == 0.0) {
                ++fallbacks;
                for (int32_t x = 0; x < V; ++x) { D[x] = inS[x] ? 0.0 : 1.0; sumD += D[x]; }
            }
            if (sumD > 0.0) for (int32_t x = 0; x < V; ++x) D[x] /= sumD;
        }
        if (next >= 0) { accepted_path[path_len++] = next; v = next; continue; }

        /* x ~ R by inverse CDF with uniforms[0] */
        double total = 0.0;
        for (int32_t x = 0; x < V; ++x) total += R[x];
        const double u0 = (double)uniforms[0];
        const double target = u0 * total;
        double cum = 0.0, lo = 0.0, hi = 0.0;
        int32_t pick = -1, last_pos = -1;
        for (int32_t x = 0; x < V; ++x) {
            if (R[x] > 0.0) last_pos = x;
            const double before = cum;
            cum += R[x];
            if (pick < 0 && cum > target) { pick = x; lo = before; hi = cum; }
        }
        if (pick < 0) { pick = last_pos < 0 ? V - 1 : last_pos; lo = cum; hi = cum; }
        *bonus_token = pick;
        if (bonus_info) {
            double m1 = target - lo, m2 = hi - target;
            bonus_info[0] = v; bonus_info[1] = u0; bonus_info[2] = total;
            bonus_info[3] = lo; bonus_info[4] = hi;
            bonus_info[5] = (m1 < m2 ? m1 : m2) / (total > 0.0 ? total : 1.0);
            bonus_info[6] = pick; bonus_info[7] = 0.0;
        }
        if (final_R) memcpy(final_R, R, sizeof(double) * (size_t)V);
        if (final_D) memcpy(final_D, D, sizeof(double) * (size_t)V);
        break;
    }
    if (n_decisions) *n_decisions = n_dec;
    if (counters) { counters[0] = degenerate; counters[1] = fallbacks; }
    free(R); free(D); free(tmp); free(inS);
    return 0;
}

/*
 * Many independent walks over trees of one shape (statistical tests).  Arrays carry a leading
 * trial dimension; the logits are shared by all trials when shared_logits != 0.
 * first_token[t] = token of the first accepted node, or the bonus token if none was accepted.
 */
int oracle_verify_trials(int64_t trials, int32_t shared_logits,
                         const float* target_logits, const float* draft_logits,
                         const int32_t* tree_tokens, const int32_t* parent, double temperature,
                         const float* uniforms, int32_t n, int32_t V,
                         int32_t* path_len_out, int32_t* first_token, int32_t* bonus_out)
{
    int32_t* path = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    if (!path) return -2;
    for (int64_t t = 0; t < trials; ++t) {
        const size_t lo = shared_logits ? 0 : (size_t)t * n * V;
        const int32_t* tok = tree_tokens + (size_t)t * n;
        int32_t bonus = -1;
        int rc = oracle_verify(target_logits + lo, draft_logits + lo, tok, parent, temperature,
                               uniforms + (size_t)t * n, n, V, path, &bonus,
                               NULL, NULL, NULL, NULL, NULL, NULL);
        if (rc) { free(path); return rc; }
        int32_t len = 0;
        while (len < n && path[len] >= 0) ++len;
        if (path_len_out) path_len_out[t] = len;
        if (bonus_out) bonus_out[t] = bonus;
        first_token[t] = len > 0 ? tok[path[0]] : bonus;
    }
    free(path);
    return 0;
}
