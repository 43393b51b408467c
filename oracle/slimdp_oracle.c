/*
 * CPU oracle for the Slim-DP communication-set path (Sun et al., AAAI-18,
 * "Slim-DP: A Light Communication Data Parallelism for DNN").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-threaded statement of what each step computes, written so that it
 * can be checked against the paper by eye.  It shares no code, header,
 * table or helper with the HIP library and neither includes the other.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.
 *
 * Every function is pinned by tests that do not go through this file:
 * published Philox known-answer vectors, closed forms, brute-force stable
 * argsort on tiny inputs, the dense (Plump-DP) special case, conservation,
 * hand-built collision cases, exact rationals and (for the quantiser) grid
 * points, the random draw fed through a known answer, and unbiasedness.
 * No function here is "parity unpinned".
 *
 * Conventions: indices are 0-based uint32 (the paper counts from 1), values
 * are IEEE binary32, all arithmetic is round-to-nearest-even with no
 * contraction other than the explicit fmaf calls below.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Counter-based random numbers: Philox4x32 with 10 rounds            */
/* (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as  */
/* 1, 2, 3", SC'11, section 3.3 and table 2 constants).               */
/* The paper's Exploration operator (section 3.1 item 2, section 3.3  */
/* step 2) only says "randomly"; this generator is the reading taken  */
/* so that the draw is reproducible and independent of any schedule.  */
/* ------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The random word attached to parameter index i for (seed, iteration,
 * worker): word (i mod 4) of the block whose counter is
 * (i div 4, worker, iteration low, iteration high) under the key
 * (seed low, seed high). */
uint32_t oracle_explore_word(uint64_t seed, uint64_t iteration, uint32_t worker, uint32_t i)
{
    uint32_t ctr[4] = { i >> 2, worker, (uint32_t)iteration, (uint32_t)(iteration >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return out[i & 3u];
}

void oracle_explore_words(uint64_t seed, uint64_t iteration, uint32_t worker,
                          uint32_t i0, uint64_t count, uint32_t* out)
{
    for (uint64_t j = 0; j < count; ++j)
        out[j] = oracle_explore_word(seed, iteration, worker, (uint32_t)(i0 + j));
}

/* ------------------------------------------------------------------ */
/* Significance, equation (1) of section 3.2:  S_i = |w_i| + c |g_i|. */
/* g is the sum of the W workers' updates in worker order (what the   */
/* server holds after a full push, section 3.3 steps 3 and 6).        */
/* Rounding: one fused multiply-add.  A NaN result is replaced by the */
/* one canonical quiet NaN so that its bit pattern is defined.        */
/* ------------------------------------------------------------------ */
void oracle_score(uint64_t n, uint32_t W, const float* w, const float* const* g,
                  float c, float* S)
{
    for (uint64_t i = 0; i < n; ++i) {
        float gi = g[0][i];
        for (uint32_t k = 1; k < W; ++k)
            gi = gi + g[k][i];
        float s = fmaf(c, fabsf(gi), fabsf(w[i]));
        if (s != s) {
            uint32_t qnan = 0x7FC00000u;
            memcpy(&s, &qnan, 4);
        }
        S[i] = s;
    }
}

/* ------------------------------------------------------------------ */
/* Ranking helpers: (key, index) pairs and a full comparison sort.    */
/* ------------------------------------------------------------------ */
typedef struct { uint32_t key; uint32_t idx; } pair_t;

static int cmp_key_desc_idx_asc(const void* a, const void* b)
{
    const pair_t* x = (const pair_t*)a; const pair_t* y = (const pair_t*)b;
    if (x->key != y->key) return (x->key > y->key) ? -1 : 1;
    if (x->idx != y->idx) return (x->idx < y->idx) ? -1 : 1;
    return 0;
}
static int cmp_key_asc_idx_asc(const void* a, const void* b)
{
    const pair_t* x = (const pair_t*)a; const pair_t* y = (const pair_t*)b;
    if (x->key != y->key) return (x->key < y->key) ? -1 : 1;
    if (x->idx != y->idx) return (x->idx < y->idx) ? -1 : 1;
    return 0;
}
static int cmp_u32_asc(const void* a, const void* b)
{
    uint32_t x = *(const uint32_t*)a, y = *(const uint32_t*)b;
    return (x > y) - (x < y);
}

/* ------------------------------------------------------------------ */
/* Core-Selection (section 3.1 item 1, section 3.2 last sentence,     */
/* section 3.3 step 6): rank the parameters of one segment            */
/* [base, base+len) by significance and keep the top k.  The rank     */
/* order is (score bit pattern as uint32, descending; index           */
/* ascending), which for non-negative scores is the numeric order.    */
/* Output: the k chosen GLOBAL indices in ascending order.            */
/* Returns 0, or -1 on bad arguments / allocation failure.            */
/* ------------------------------------------------------------------ */
int oracle_select_core(const float* S, uint32_t base, uint32_t len, uint32_t k, uint32_t* core_idx)
{
    if (k > len) return -1;
    if (len == 0) return 0;
    pair_t* p = (pair_t*)malloc((size_t)len * sizeof(pair_t));
    if (!p) return -1;
    for (uint32_t j = 0; j < len; ++j) {
        uint32_t bits;
        memcpy(&bits, &S[base + j], 4);
        p[j].key = bits;
        p[j].idx = base + j;
    }
    qsort(p, len, sizeof(pair_t), cmp_key_desc_idx_asc);
    for (uint32_t j = 0; j < k; ++j) core_idx[j] = p[j].idx;
    qsort(core_idx, k, sizeof(uint32_t), cmp_u32_asc);
    free(p);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Exploration (section 3.1 item 2, section 3.3 step 2): worker k     */
/* draws m parameters uniformly without replacement from those of the */
/* segment [base, base+len) that are NOT in the core.  Realised as    */
/* random-key selection: every non-core index gets its random word,   */
/* and the m indices with the smallest (word, index) are taken.       */
/* in_core: one byte per GLOBAL index, non-zero = in the core.        */
/* Output: the m chosen GLOBAL indices in ascending order.            */
/* ------------------------------------------------------------------ */
int oracle_sample_explore(const uint8_t* in_core, uint32_t base, uint32_t len,
                          uint64_t seed, uint64_t iteration, uint32_t worker,
                          uint32_t m, uint32_t* expl_idx)
{
    if (len == 0) return (m == 0) ? 0 : -1;
    pair_t* p = (pair_t*)malloc((size_t)len * sizeof(pair_t));
    if (!p) return -1;
    uint32_t cnt = 0;
    for (uint32_t j = 0; j < len; ++j) {
        uint32_t i = base + j;
        if (in_core[i]) continue;
        p[cnt].key = oracle_explore_word(seed, iteration, worker, i);
        p[cnt].idx = i;
        ++cnt;
    }
    if (m > cnt) { free(p); return -1; }
    qsort(p, cnt, sizeof(pair_t), cmp_key_asc_idx_asc);
    for (uint32_t j = 0; j < m; ++j) expl_idx[j] = p[j].idx;
    qsort(expl_idx, m, sizeof(uint32_t), cmp_u32_asc);
    free(p);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Push, worker side (section 3.3 step 3; wire format of section 3.5):*/
/* extract the worker's updates at the core (values only, the keys    */
/* are cached on both ends) and at its explorer (<key, value> pairs;  */
/* the keys are expl_idx itself).  Bit copies.                        */
/* ------------------------------------------------------------------ */
void oracle_pack(const float* g_k, const uint32_t* core_idx, uint64_t k,
                 const uint32_t* expl_idx, uint64_t m, float* core_val, float* expl_val)
{
    for (uint64_t j = 0; j < k; ++j) core_val[j] = g_k[core_idx[j]];
    for (uint64_t j = 0; j < m; ++j) expl_val[j] = g_k[expl_idx[j]];
}

/* ------------------------------------------------------------------ */
/* Update, server side (section 3.3 step 3):                          */
/*   w_i <- w_i - lr * sum_k T_C(delta_k)_i                           */
/* The sum runs over the workers whose communication set contains i,  */
/* in ascending worker order, starting from +0; one fused             */
/* multiply-add applies it.  Indices no worker sent are not written.  */
/* scratch_acc (n floats) and scratch_hit (n bytes) are caller-owned  */
/* work arrays; their contents on entry do not matter.                */
/* ------------------------------------------------------------------ */
void oracle_merge(uint64_t n, float* w, float lr, uint32_t W,
                  const uint32_t* core_idx, uint64_t k, const float* const* core_val,
                  const uint32_t* const* expl_idx, const float* const* expl_val,
                  const uint64_t* m_w, float* scratch_acc, uint8_t* scratch_hit)
{
    for (uint64_t i = 0; i < n; ++i) { scratch_acc[i] = 0.0f; scratch_hit[i] = 0; }
    for (uint32_t wk = 0; wk < W; ++wk) {
        for (uint64_t j = 0; j < k; ++j) {
            uint32_t i = core_idx[j];
            scratch_acc[i] = scratch_acc[i] + core_val[wk][j];
            scratch_hit[i] = 1;
        }
        for (uint64_t j = 0; j < m_w[wk]; ++j) {
            uint32_t i = expl_idx[wk][j];
            scratch_acc[i] = scratch_acc[i] + expl_val[wk][j];
            scratch_hit[i] = 1;
        }
    }
    for (uint64_t i = 0; i < n; ++i)
        if (scratch_hit[i]) w[i] = fmaf(-lr, scratch_acc[i], w[i]);
}

/* ------------------------------------------------------------------ */
/* The last iteration before a reselection (algorithm 1: the branch    */
/* (t+1) % q == 0; section 3.3 steps 3 and 6): every worker pushes its */
/* whole update, the server applies all of them,                       */
/*     w_new_i = w_i - lr * sum_k g_k[i],                              */
/* and the new core is ranked with the NEW model and these updates,    */
/*     S_i = |w_new_i| + c * |sum_k g_k[i]|        (equation (1)).     */
/* The sum is the server's: from +0, one worker after the other, as in */
/* oracle_merge with every index sent by every worker; one fmaf for    */
/* the model, one for the significance.                                */
/* ------------------------------------------------------------------ */
void oracle_dense_update_score(uint64_t n, uint32_t W, float* w, const float* const* g,
                               float lr, float c, float* S)
{
    for (uint64_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (uint32_t k = 0; k < W; ++k)
            acc = acc + g[k][i];
        w[i] = fmaf(-lr, acc, w[i]);
        float s = fmaf(c, fabsf(acc), fabsf(w[i]));
        if (s != s) {
            uint32_t qnan = 0x7FC00000u;
            memcpy(&s, &qnan, 4);
        }
        S[i] = s;
    }
}

/* The update of oracle_merge in binary64 with no intermediate rounding to
 * binary32: the reference against which the binary32 tolerance is stated. */
void oracle_merge_f64(uint64_t n, const float* w_in, double* w_out, double lr, uint32_t W,
                      const uint32_t* core_idx, uint64_t k, const float* const* core_val,
                      const uint32_t* const* expl_idx, const float* const* expl_val,
                      const uint64_t* m_w)
{
    for (uint64_t i = 0; i < n; ++i) w_out[i] = 0.0;
    for (uint32_t wk = 0; wk < W; ++wk) {
        for (uint64_t j = 0; j < k; ++j) w_out[core_idx[j]] += (double)core_val[wk][j];
        for (uint64_t j = 0; j < m_w[wk]; ++j) w_out[expl_idx[wk][j]] += (double)expl_val[wk][j];
    }
    for (uint64_t i = 0; i < n; ++i) w_out[i] = (double)w_in[i] - lr * w_out[i];
}

/* ------------------------------------------------------------------ */
/* Signature of the cached keys (section 3.5: for the core only the    */
/* values travel, with a signature of the cached keys).  The paper does  */
/* not say which; the reading taken: the 64-bit sum, modulo 2^64, over the  */
/* list positions j of mix(core_idx[j] + 2^32 * j), mix being the       */
/* output function of SplitMix64 (Steele, Lea, Flood, OOPSLA 2014).     */
/* Order-sensitive, and a plain sum so that any schedule gives it.      */
/* ------------------------------------------------------------------ */
uint64_t oracle_splitmix64_mix(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t oracle_core_signature(const uint32_t* core_idx, uint64_t k)
{
    uint64_t sig = 0;
    for (uint64_t j = 0; j < k; ++j)
        sig += oracle_splitmix64_mix((uint64_t)core_idx[j] + (j << 32));
    return sig;
}

/* ------------------------------------------------------------------ */
/* Pull and local Merge (section 3.3 steps 4 and 5): read the global  */
/* model at the worker's communication set; if w_local is given,      */
/* overwrite the local model at those indices and leave the rest.     */
/* ------------------------------------------------------------------ */
void oracle_pull(const float* w, const uint32_t* core_idx, uint64_t k,
                 const uint32_t* expl_idx, uint64_t m,
                 float* core_out, float* expl_out, float* w_local)
{
    for (uint64_t j = 0; j < k; ++j) {
        core_out[j] = w[core_idx[j]];
        if (w_local) w_local[core_idx[j]] = core_out[j];
    }
    for (uint64_t j = 0; j < m; ++j) {
        expl_out[j] = w[expl_idx[j]];
        if (w_local) w_local[expl_idx[j]] = expl_out[j];
    }
}


/* ------------------------------------------------------------------ */
/* LocalTrain (section 3.3 step 1; algorithm 1, first line of the      */
/* worker loop): one mini-batch step of worker k on its LOCAL model,   */
/*     w_k <- w_k - eta * grad,                                        */
/* and the accumulation of the update over the p mini-batches between  */
/* two communications, delta_k = grad_1 + grad_2 + ... in binary32 in  */
/* mini-batch order (first != 0 starts a new accumulation).  The       */
/* gradient itself is an input: there is no network here to           */
/* differentiate.  One fmaf for the model.                             */
/* ------------------------------------------------------------------ */
void oracle_local_step(uint64_t n, float* w_local, float* delta, const float* grad, float eta, int first)
{
    for (uint64_t i = 0; i < n; ++i) {
        w_local[i] = fmaf(-eta, grad[i], w_local[i]);
        delta[i] = first ? grad[i] : delta[i] + grad[i];
    }
}

/* ------------------------------------------------------------------ */
/* Quantisation of the packed values (section 2.2, last sentences:     */
/* the method composes with gradient quantisation; section 4.2: the    */
/* comparison uses random quantisation, 8 bits, buckets of 512).       */
/* Random quantisation after Alistarh et al. (QSGD): per bucket a      */
/* scale, per value a sign and a level l in 0..127 on the grid         */
/* scale * l / 127, rounded up with probability equal to the fraction  */
/* so that the expectation is the value.  Readings (the paper fixes    */
/* none): the scale is the bucket's largest magnitude (exact, order-   */
/* free); 8 bits = sign + 7 level bits; arithmetic in binary32:        */
/*   y = (|v| / scale) * 127, l = floor(y), up = u < y - l,            */
/*   u = (random word >> 8) * 2^-24.                                   */
/* The random word of element j of list `kind` (0 core values, 1       */
/* explorer values) of a worker: word (j mod 4) of Philox4x32-10 with  */
/* counter (j div 4, worker, iteration low, iteration high) and key    */
/* (seed low ^ 0x51534744, seed high ^ kind): another key than the     */
/* explorer's.  A bucket of zeros has scale 0 and levels 0.  Values    */
/* must be finite.                                                     */
/* ------------------------------------------------------------------ */
#define ORACLE_QUANT_BUCKET 512u
#define ORACLE_QUANT_LEVELS 127.0f

uint32_t oracle_quant_word(uint64_t seed, uint64_t iteration, uint32_t worker, uint32_t kind, uint64_t j)
{
    uint32_t ctr[4] = { (uint32_t)(j >> 2), worker, (uint32_t)iteration, (uint32_t)(iteration >> 32) };
    uint32_t key[2] = { (uint32_t)seed ^ 0x51534744u, (uint32_t)(seed >> 32) ^ kind };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return out[j & 3u];
}

void oracle_quantize(const float* v, uint64_t count, uint64_t seed, uint64_t iteration, uint32_t worker,
                     uint32_t kind, uint8_t* code, float* scale)
{
    for (uint64_t b0 = 0; b0 < count; b0 += ORACLE_QUANT_BUCKET) {
        uint64_t b1 = b0 + ORACLE_QUANT_BUCKET < count ? b0 + ORACLE_QUANT_BUCKET : count;
        float s = 0.0f;
        for (uint64_t j = b0; j < b1; ++j)
            if (fabsf(v[j]) > s) s = fabsf(v[j]);
        scale[b0 / ORACLE_QUANT_BUCKET] = s;
        for (uint64_t j = b0; j < b1; ++j) {
            uint32_t level = 0;
            if (s > 0.0f) {
                float y = (fabsf(v[j]) / s) * ORACLE_QUANT_LEVELS;
                float l = floorf(y);
                float frac = y - l;
                float u = (float)(oracle_quant_word(seed, iteration, worker, kind, j) >> 8) * 0x1p-24f;
                level = (uint32_t)l + (u < frac ? 1u : 0u);
            }
            code[j] = (uint8_t)((signbit(v[j]) ? 0x80u : 0u) | level);
        }
    }
}

/* value = sign * (scale * level / 127), two binary32 roundings: the product, then the quotient */
void oracle_dequantize(const uint8_t* code, const float* scale, uint64_t count, float* out)
{
    for (uint64_t j = 0; j < count; ++j) {
        float s = scale[j / ORACLE_QUANT_BUCKET];
        float mag = (s * (float)(code[j] & 0x7Fu)) / ORACLE_QUANT_LEVELS;
        out[j] = (code[j] & 0x80u) ? -mag : mag;
    }
}
