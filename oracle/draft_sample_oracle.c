/*
 * CPU checker for the drafter's ordered draw of child tokens.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call this.
 *
 * What is computed.  Algorithm 2 ("Sequoia Sampling and Verification", Sec. 3.2.1) assumes
 * that the children of a node were drawn from the draft distribution Q = softmax(logits / T)
 * one after the other WITHOUT replacement, and, once every token of non-zero probability has
 * been drawn, uniformly among the tokens not drawn yet.  The implementation details of Sec. 4.1
 * name the exponential-sort method for it: give every token x an independent Exp(1) variate
 * E[x] and order the tokens by Q[x] / E[x], largest first; the first k tokens of that order are
 * an ordered draw of k tokens without replacement.  In logarithms, with g = -ln E (a standard
 * Gumbel variate):
 *
 *     key[x] = logits[x] / T + g[x]                      order: key descending
 *
 * Tokens of zero probability (logit -inf; NaN is read the same way) come after all others, in
 * the order of g alone: equal weights, hence a uniformly random order, which is the uniform
 * continuation the algorithm prescribes.  Equal keys (possible only through rounding) go to the
 * lower token id.
 *
 * T = 0 is read as the limit T -> 0+: the k largest logits in descending order, lower id first
 * among equals (the top-k drafting of Sec. 2.2); zero-probability tokens follow in ascending id.
 *
 * Randomness is a counter-based generator so that the checker and the library can each draw
 * the same numbers on their own: Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11) with key (seed low, seed high) and counter
 * (x / 4, row, step low, step high); token x takes output word x % 4, and
 *
 *     w = ((word >> 9) + 0.5) * 2^-23   in (0, 1), exact in fp32 and fp64
 *     E = -ln w,   g = -ln E
 *
 * Arithmetic is fp64; logits arrive as float (an exact container for bf16 and fp32).  One
 * thread, one plain sort per row.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

void oracle_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t prod_a = (uint64_t)0xD2511F53u * c0;
        const uint64_t prod_b = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)prod_b;
        const uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)prod_a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;   /* the key schedule: golden-ratio and sqrt(3)-1 Weyl steps */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform w in (0,1) that token x of a row gets at a given step. */
double oracle_draft_uniform(uint64_t seed, uint64_t step, int32_t row, int32_t x)
{
    const uint32_t counter[4] = {(uint32_t)x / 4u, (uint32_t)row, (uint32_t)step, (uint32_t)(step >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    oracle_philox4x32_10(counter, key, out);
    const uint32_t word = out[(uint32_t)x % 4u];
    return ((double)(word >> 9) + 0.5) * 0x1p-23;
}

typedef struct {
    int zero_probability; /* 1: comes after every token of non-zero probability */
    double key;
    int32_t token;
} Entry;

static int before(const void* pa, const void* pb)
{
    const Entry* a = (const Entry*)pa;
    const Entry* b = (const Entry*)pb;
    if (a->zero_probability != b->zero_probability) return a->zero_probability - b->zero_probability;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    return a->token < b->token ? -1 : (a->token > b->token ? 1 : 0);
}

/*
 * logits      [n_rows][V]
 * row_ids     optional [n_rows]: the row number each row draws its random numbers with (so that
 *             a test can check single rows of a large call); NULL = 0, 1, 2, ...
 * n_children  [n_rows], each in [0, k_stride]; row r receives its first n_children[r] tokens of
 *             the order, then -1 up to k_stride
 * order_keys  optional [n_rows][k_stride + 1]: the keys of the first k+1 tokens of the order
 *             (k = n_children[r]; NaN beyond), so that a test can see how close a decision was;
 *             zero-probability tokens report their g
 * order_class optional [n_rows][k_stride + 1]: 1 where that token had zero probability
 * Returns 0, or -1 on bad arguments.
 */
int oracle_draft_sample(const float* logits, const int32_t* row_ids, int32_t n_rows, int32_t V,
                        const int32_t* n_children, double T, uint64_t seed, uint64_t step, int32_t k_stride, int32_t* tokens,
                        double* order_keys, int32_t* order_class)
{
    if (!logits || !n_children || !tokens || n_rows < 1 || V < 1 || k_stride < 1 || !(T >= 0.0)) return -1;
    Entry* e = (Entry*)malloc(sizeof(Entry) * (size_t)V);
    if (!e) return -1;
    for (int32_t r = 0; r < n_rows; ++r) {
        const int32_t k = n_children[r];
        if (k < 0 || k > k_stride || k > V) { free(e); return -1; }
        const float* row = logits + (size_t)r * V;
        for (int32_t x = 0; x < V; ++x) {
            const double l = (double)row[x];
            const int zero = isnan(l) || (isinf(l) && l < 0);
            e[x].zero_probability = zero;
            e[x].token = x;
            if (T == 0.0) {
                e[x].key = zero ? 0.0 : l;
            } else {
                const double w = oracle_draft_uniform(seed, step, row_ids ? row_ids[r] : r, x);
                const double g = -log(-log(w));
                e[x].key = zero ? g : l / T + g;
            }
        }
        qsort(e, (size_t)V, sizeof(Entry), before);
        for (int32_t j = 0; j < k_stride; ++j) tokens[(size_t)r * k_stride + j] = j < k ? e[j].token : -1;
        for (int32_t j = 0; j <= k_stride; ++j) {
            const int have = j <= k && j < V;
            if (order_keys) order_keys[(size_t)r * (k_stride + 1) + j] = have ? e[j].key : NAN;
            if (order_class) order_class[(size_t)r * (k_stride + 1) + j] = have ? e[j].zero_probability : 0;
        }
    }
    free(e);
    return 0;
}
