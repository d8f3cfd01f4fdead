/*
 * CPU checker for the two baseline verification algorithms the paper holds Sequoia's against
 * (Sec. 2.2).  TEST INFRASTRUCTURE ONLY: nothing in the product path may call this.
 *
 * Both verify a token tree recursively from the root, like Algorithm 2, and differ only in
 * what happens at a node v with P = softmax(target_logits[v] / T), Q = softmax(draft_logits[v] / T):
 *
 *   SpecInfer (algorithm 1): Algorithm 2 of Sec. 3.2.1 without its blue lines -- the children
 *   were drawn from Q independently (with replacement), so D stays Q for every child:
 *       R <- P
 *       for every child c of v in ascending node id:  s <- tree_tokens[c], r <- uniforms[c]
 *           if r < R[s] / Q[s]: accept c, continue the walk at c
 *           else R <- norm(max(R - Q, 0))
 *       no child accepted: return x ~ R                      (inverse CDF with uniforms[0])
 *
 *   Naive / top-k sampling (algorithm 2): draw x ~ P and accept x if it is the token of one of
 *   v's children (the first such child in sibling order), continue the walk there; otherwise x
 *   itself is the token the step emits.  The draw at node v uses uniforms[v] (the root's is
 *   uniforms[0]): every node has one uniform, and this algorithm needs one per visited node.
 *
 * Readings shared with the checker of Algorithm 2: T = 0 means one-hot at the arg-max (lowest
 * index on ties); "x ~ R" is the inverse CDF in ascending token id, the first x whose inclusive
 * cumulative mass exceeds u * sum(R), else the last x with R[x] > 0; Q[s] = 0 gives ratio +inf if
 * R[s] > 0 else 0; a residual update whose mass is 0 leaves R unchanged.
 *
 * Arithmetic is fp64; logits and uniforms arrive as float.  One thread, plain loops.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define BASELINE_RECORD_DOUBLES 8

static void tempered(const float* logits, int32_t V, double T, double* out)
{
    if (T == 0.0) {
        int32_t best = 0;
        for (int32_t x = 1; x < V; ++x)
            if ((double)logits[x] > (double)logits[best]) best = x;
        for (int32_t x = 0; x < V; ++x) out[x] = 0.0;
        out[best] = 1.0;
        return;
    }
    double m = -INFINITY, z = 0.0;
    for (int32_t x = 0; x < V; ++x)
        if ((double)logits[x] > m) m = (double)logits[x];
    for (int32_t x = 0; x < V; ++x) { out[x] = exp(((double)logits[x] - m) / T); z += out[x]; }
    for (int32_t x = 0; x < V; ++x) out[x] /= z;
}

/* x ~ R by inverse CDF; info[0..3] = total, cdf below x, cdf including x, margin relative to total */
static int32_t inverse_cdf(const double* R, int32_t V, double u, double* info)
{
    double total = 0.0;
    for (int32_t x = 0; x < V; ++x) total += R[x];
    const double goal = u * total;
    double cum = 0.0, lo = 0.0, hi = 0.0;
    int32_t pick = -1, last_pos = -1;
    for (int32_t x = 0; x < V; ++x) {
        if (R[x] > 0.0) last_pos = x;
        const double before = cum;
        cum += R[x];
        if (pick < 0 && cum > goal) { pick = x; lo = before; hi = cum; }
    }
    if (pick < 0) { pick = last_pos < 0 ? V - 1 : last_pos; lo = cum; hi = cum; }
    if (info) {
        const double m1 = goal - lo, m2 = hi - goal;
        info[0] = total; info[1] = lo; info[2] = hi;
        info[3] = (m1 < m2 ? m1 : m2) / (total > 0.0 ? total : 1.0);
    }
    return pick;
}

/*
 * algorithm: 1 SpecInfer, 2 naive / top-k.
 * records [(n) * 8], *n_records: one per accept test (SpecInfer: node, token, u, R[s], Q[s], ratio,
 * accepted, parent) or per visited node (top-k: node, drawn token, u, cdf below, cdf including,
 * margin, matched child or -1, 0).  bonus_info [8]: stop node, u, total, cdf below, cdf including,
 * margin, token, 0.
 */
int oracle_verify_baseline(int32_t algorithm, const float* target_logits, const float* draft_logits,
                           const int32_t* tree_tokens, const int32_t* parent, double temperature,
                           const float* uniforms, int32_t n, int32_t V, int32_t* accepted_path,
                           int32_t* bonus_token, double* records, int32_t* n_records, double* bonus_info)
{
    if ((algorithm != 1 && algorithm != 2) || n < 1 || V < 1 || !(temperature >= 0.0) || parent[0] != -1) return -1;
    for (int32_t i = 1; i < n; ++i) {
        if (parent[i] < 0 || parent[i] >= i) return -1;
        if (tree_tokens[i] < 0 || tree_tokens[i] >= V) return -1;
    }
    double* R = (double*)malloc(sizeof(double) * (size_t)V);
    double* Q = (double*)malloc(sizeof(double) * (size_t)V);
    double* tmp = (double*)malloc(sizeof(double) * (size_t)V);
    if (!R || !Q || !tmp) { free(R); free(Q); free(tmp); return -2; }
    for (int32_t i = 0; i < n; ++i) accepted_path[i] = -1;
    int32_t n_rec = 0, path_len = 0, v = 0;
    double info[4];
    for (;;) {
        tempered(target_logits + (size_t)v * V, V, temperature, R);
        int32_t next = -1;
        if (algorithm == 2) {
            const double u = (double)uniforms[v];
            const int32_t x = inverse_cdf(R, V, u, info);
            for (int32_t c = v + 1; c < n && next < 0; ++c)
                if (parent[c] == v && tree_tokens[c] == x) next = c;
            if (records) {
                double* rec = records + (size_t)n_rec * BASELINE_RECORD_DOUBLES;
                rec[0] = v; rec[1] = x; rec[2] = u; rec[3] = info[1]; rec[4] = info[2]; rec[5] = info[3];
                rec[6] = next; rec[7] = 0.0;
            }
            ++n_rec;
            if (next < 0) {
                *bonus_token = x;
                if (bonus_info) {
                    bonus_info[0] = v; bonus_info[1] = u; bonus_info[2] = info[0]; bonus_info[3] = info[1];
                    bonus_info[4] = info[2]; bonus_info[5] = info[3]; bonus_info[6] = x; bonus_info[7] = 0.0;
                }
                break;
            }
            accepted_path[path_len++] = next;
            v = next;
            continue;
        }
        tempered(draft_logits + (size_t)v * V, V, temperature, Q);
        for (int32_t c = v + 1; c < n && next < 0; ++c) {
            if (parent[c] != v) continue;
            const int32_t s = tree_tokens[c];
            const double r = (double)uniforms[c];
            double ratio;
            if (Q[s] > 0.0) ratio = R[s] / Q[s];
            else ratio = (R[s] > 0.0) ? INFINITY : 0.0;
            const int accept = (r < ratio);
            if (records) {
                double* rec = records + (size_t)n_rec * BASELINE_RECORD_DOUBLES;
                rec[0] = c; rec[1] = s; rec[2] = r; rec[3] = R[s]; rec[4] = Q[s];
                rec[5] = ratio; rec[6] = accept; rec[7] = v;
            }
            ++n_rec;
            if (accept) { next = c; break; }
            double sum = 0.0;
            for (int32_t x = 0; x < V; ++x) {
                const double diff = R[x] - Q[x];
                tmp[x] = diff > 0.0 ? diff : 0.0;
                sum += tmp[x];
            }
            if (sum > 0.0) for (int32_t x = 0; x < V; ++x) R[x] = tmp[x] / sum;
        }
        if (next >= 0) { accepted_path[path_len++] = next; v = next; continue; }
        const double u0 = (double)uniforms[0];
        const int32_t x = inverse_cdf(R, V, u0, info);
        *bonus_token = x;
        if (bonus_info) {
            bonus_info[0] = v; bonus_info[1] = u0; bonus_info[2] = info[0]; bonus_info[3] = info[1];
            bonus_info[4] = info[2]; bonus_info[5] = info[3]; bonus_info[6] = x; bonus_info[7] = 0.0;
        }
        break;
    }
    if (n_records) *n_records = n_rec;
    free(R); free(Q); free(tmp);
    return 0;
}
