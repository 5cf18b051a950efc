/*
 * sgns_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded CPU statement of what the skip-gram
 * negative-sampling (SGNS) training path computes.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may build or call it; the GPU
 * library shares no code, header, table or constant with this file.
 *
 * Source of each piece (FULL-W2V paper, by section):
 *   - problem statement, sliding window of 2W words, N negatives drawn from
 *     a weighted distribution ...................... Section 2.1
 *   - the N negatives are drawn once per context window and shared by all of
 *     its context words; the window pairs every context word with the N+1
 *     "samples" (target + negatives) .............. Section 3.1, Figure 3,
 *                                                    Figure 4 caption
 *   - the update of a window is the sum over all pairings, order-free
 *                                                    Section 3.1 (independence
 *                                                    of negative samples)
 *   - windows of one sentence are processed strictly in order
 *                                                    Section 3.1 (last par.)
 *   - traditional window width: random in [1, W]    Section 3.2
 *   - the paper's own variant: fixed width ceil(W/2) Section 3.2
 *   - sentences are independent units (Hogwild)     Section 2.2 / 2.3
 *   - optional extension named as future work: one set of negatives for the
 *     windows of several consecutive tokens .......... Section 3.1 (temporal
 *                                                    locality and reuse),
 *                                                    Section 7 (future work)
 *   - words with >= 5 occurrences, <= 1000 words per sentence: corpus
 *     preparation, done by the caller ............... Table 3 caption
 *   - extension, not in the paper (which computes and stores in fp32,
 *     Section 5.1): tables STORED as bfloat16, arithmetic in fp32 on the
 *     on-chip copies the paper keeps (context rows for as long as the
 *     window span holds them, Section 3.2; target and negative rows for
 *     one window, Section 3.1), stochastic rounding when a copy goes back
 * Where the paper is silent (sampling distribution exponent, subsampling
 * rule, learning-rate schedule, random numbers, weight initialisation) the
 * conventions of the word2vec papers it cites are used; each such choice is
 * spelled out next to the function that implements it.
 *
 * Build:  gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC \
 *             -DREAL=float  sgns_oracle.c -o liboracle_f32.so -lm
 *         (and -DREAL=double for the gradient-check build)
 *
 * Parity pins (tests/test_oracle_*.py): published SplitMix64 outputs for the
 * mixer, closed forms for table / thresholds / width, hand-computed windows,
 * central finite differences of the window loss, brute-force enumeration on
 * an 8-word vocabulary, untouched-row invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif
typedef REAL real_t;

#define ORC_MAX_NEG 64
#define ORC_MAX_CTX 64

/* ------------------------------------------------------------------ */
/* Random numbers: counter-based, keyed by (seed, epoch, position, j). */
/* The mixer is the finaliser of the public-domain SplitMix64          */
/* generator (Steele, Lea, Flood 2014): mix64(k*G), k=1,2,.. with      */
/* seed 0 reproduces that generator's published output stream.         */
/* ------------------------------------------------------------------ */
static const uint64_t ORC_G = 0x9E3779B97F4A7C15ull;

uint64_t orc_mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

/* draw j of global (pre-subsampling) token position pos in epoch `epoch`:
 *   j = 0  subsampling decision, j = 1 window width, j = 2+k negative k. */
uint64_t orc_draw(uint64_t seed, uint32_t epoch, uint64_t pos, uint32_t j)
{
    uint64_t key  = orc_mix64(seed + ORC_G * ((uint64_t)epoch + 1u));
    uint64_t base = orc_mix64(key ^ orc_mix64(pos));
    return orc_mix64(base + ORC_G * ((uint64_t)j + 1u));
}

static uint32_t u32_of(uint64_t draw) { return (uint32_t)(draw >> 32); }
static uint32_t mulhi32(uint32_t a, uint32_t n) { return (uint32_t)(((uint64_t)a * (uint64_t)n) >> 32); }

/* ------------------------------------------------------------------ */
/* Negative-sampling distribution ("weighted distribution", Sec. 2.1). */
/* weight_i = count_i^0.75 (Mikolov et al.), written as                */
/* sqrt(c)*sqrt(sqrt(c)) so that only correctly rounded IEEE           */
/* operations are involved.  The distribution is quantised onto        */
/* `tsz` equal slots: word i owns slots [end[i-1], end[i]).            */
/* ------------------------------------------------------------------ */
int orc_table_ends(const uint64_t *counts, uint32_t V, uint64_t tsz, uint64_t *end)
{
    double total = 0.0;
    for (uint32_t i = 0; i < V; ++i) {
        double c = (double)counts[i];
        total += sqrt(c) * sqrt(sqrt(c));
    }
    if (!(total > 0.0)) return -1;
    double cum = 0.0;
    for (uint32_t i = 0; i < V; ++i) {
        double c = (double)counts[i];
        cum += sqrt(c) * sqrt(sqrt(c));
        double e = floor((cum / total) * (double)tsz);
        uint64_t ei = (uint64_t)e;
        if (ei > tsz) ei = tsz;
        end[i] = ei;
    }
    end[V - 1] = tsz;
    return 0;
}

/* word that owns slot `slot`: the smallest i with end[i] > slot. */
int32_t orc_word_of_slot(const uint64_t *end, uint32_t V, uint64_t slot)
{
    uint32_t lo = 0, hi = V - 1;
    while (lo < hi) {
        uint32_t mid = lo + (hi - lo) / 2;
        if (end[mid] > slot) hi = mid; else lo = mid + 1;
    }
    return (int32_t)lo;
}

int32_t orc_negative(const uint64_t *end, uint32_t V, uint64_t tsz,
                     uint64_t seed, uint32_t epoch, uint64_t pos, uint32_t k)
{
    uint32_t u = u32_of(orc_draw(seed, epoch, pos, 2u + k));
    return orc_word_of_slot(end, V, (uint64_t)mulhi32(u, (uint32_t)tsz));
}

/* ------------------------------------------------------------------ */
/* Frequent-word subsampling (Mikolov et al. 2013, the "conventional   */
/* hyperparameters" the paper's evaluation refers to):                 */
/*   P_keep(w) = min(1, sqrt(t / f_w)),  f_w = count_w / sum(counts).  */
/* Quantised to 32 bits; 0xFFFFFFFF means "always keep".               */
/* ------------------------------------------------------------------ */
void orc_thresholds(const uint64_t *counts, uint32_t V, double t, uint32_t *thr)
{
    double total = 0.0;
    for (uint32_t i = 0; i < V; ++i) total += (double)counts[i];
    for (uint32_t i = 0; i < V; ++i) {
        if (!(t > 0.0) || counts[i] == 0) { thr[i] = 0xFFFFFFFFu; continue; }
        double f = (double)counts[i] / total;
        double p = sqrt(t / f);
        if (p >= 1.0) { thr[i] = 0xFFFFFFFFu; continue; }
        double q = floor(p * 4294967296.0);
        thr[i] = (q >= 4294967295.0) ? 0xFFFFFFFFu : (uint32_t)q;
    }
}

int orc_keep(const uint32_t *thr, int32_t w, uint64_t seed, uint32_t epoch, uint64_t pos)
{
    uint32_t t = thr[w];
    if (t == 0xFFFFFFFFu) return 1;
    return u32_of(orc_draw(seed, epoch, pos, 0)) < t;
}

/* window width: uniform on {1..W} (mode 0, Sec. 3.2 "traditional") or
 * the fixed ceil(W/2) of the paper's own variant (mode 1). */
uint32_t orc_width(uint32_t W, uint32_t mode, uint64_t seed, uint32_t epoch, uint64_t pos)
{
    if (mode == 1) return (W + 1u) / 2u;
    return 1u + mulhi32(u32_of(orc_draw(seed, epoch, pos, 1)), W);
}

/* ------------------------------------------------------------------ */
/* Learning rate of a sentence: linear decay over all epochs, from the */
/* global offset of the sentence's first token (schedule-independent). */
/* ------------------------------------------------------------------ */
float orc_lr(double lr0, double lr_min_frac, uint32_t epoch, uint32_t total_epochs,
             uint64_t tokens_per_epoch, uint64_t sentence_start)
{
    double done = (double)((uint64_t)epoch * tokens_per_epoch + sentence_start);
    double all  = (double)((uint64_t)total_epochs * tokens_per_epoch);
    double frac = 1.0 - done / all;
    if (frac < lr_min_frac) frac = lr_min_frac;
    return (float)(lr0 * frac);
}

/* ------------------------------------------------------------------ */
/* Initial weights: syn0 ~ U(-0.5/d, 0.5/d) from the seed, syn1neg = 0 */
/* ------------------------------------------------------------------ */
void orc_init_weights(uint64_t seed, uint32_t V, uint32_t d, real_t *syn0, real_t *syn1neg)
{
    uint64_t k = orc_mix64(seed ^ 0x696E6974ull);
    for (uint64_t i = 0; i < (uint64_t)V; ++i)
        for (uint64_t j = 0; j < d; ++j) {
            uint32_t u = u32_of(orc_mix64(k + (i * d + j)));
            double r = ((double)(u >> 8) * (1.0 / 16777216.0) - 0.5) / (double)d;
            syn0[i * d + j] = (real_t)(float)r;
        }
    memset(syn1neg, 0, sizeof(real_t) * (size_t)V * d);
}

/* ------------------------------------------------------------------ */
/* One context window = one minibatch SGD step on                      */
/*   L_win = sum_c [ softplus(-<I_c,O_0>) + sum_{k>=1} m_k softplus(<I_c,O_k>) ] */
/* I_c = syn0[ctx[c]] (context words), O_0 = syn1neg[target],          */
/* O_k = syn1neg[negative k]; m_k = 0 when negative k is the target.   */
/* All dot products use the values the rows had when the window began; */
/* the summed update is applied at the end (Sec. 3.1).  A row that     */
/* occurs several times receives the sum of its deltas.                */
/* ------------------------------------------------------------------ */
static real_t sigmoid_r(real_t x) { return (real_t)1 / ((real_t)1 + (real_t)exp(-(double)x)); }
static double softplus_d(double x) { return (x > 0 ? x : 0) + log1p(exp(-fabs(x))); }

void orc_window_step(real_t *syn0, real_t *syn1neg, uint32_t d,
                     const int32_t *ctx, uint32_t nctx,
                     const int32_t *out, uint32_t nout,   /* out[0] = target */
                     real_t alpha, double *loss_sum)
{
    real_t g[ORC_MAX_CTX][ORC_MAX_NEG + 1];
    real_t *dI = (real_t *)calloc((size_t)nctx * d, sizeof(real_t));
    real_t *dO = (real_t *)calloc((size_t)nout * d, sizeof(real_t));
    for (uint32_t c = 0; c < nctx; ++c) {
        const real_t *I = syn0 + (size_t)ctx[c] * d;
        for (uint32_t k = 0; k < nout; ++k) {
            const real_t *O = syn1neg + (size_t)out[k] * d;
            int masked = (k >= 1 && out[k] == out[0]);
            real_t x = 0;
            for (uint32_t j = 0; j < d; ++j) x += I[j] * O[j];
            real_t label = (k == 0) ? (real_t)1 : (real_t)0;
            g[c][k] = masked ? (real_t)0 : alpha * (label - sigmoid_r(x));
            if (!masked && loss_sum) *loss_sum += softplus_d(k == 0 ? -(double)x : (double)x);
        }
    }
    for (uint32_t c = 0; c < nctx; ++c)
        for (uint32_t k = 0; k < nout; ++k) {
            const real_t *I = syn0 + (size_t)ctx[c] * d;
            const real_t *O = syn1neg + (size_t)out[k] * d;
            for (uint32_t j = 0; j < d; ++j) {
                dI[(size_t)c * d + j] += g[c][k] * O[j];
                dO[(size_t)k * d + j] += g[c][k] * I[j];
            }
        }
    for (uint32_t c = 0; c < nctx; ++c) {
        real_t *I = syn0 + (size_t)ctx[c] * d;
        for (uint32_t j = 0; j < d; ++j) I[j] += dI[(size_t)c * d + j];
    }
    for (uint32_t k = 0; k < nout; ++k) {
        real_t *O = syn1neg + (size_t)out[k] * d;
        for (uint32_t j = 0; j < d; ++j) O[j] += dO[(size_t)k * d + j];
    }
    free(dI);
    free(dO);
}

/* The other reading of Sec. 4.2 ("pair one sample with all the context
 * words, then iterate over the samples") with every pairing applied at
 * once.  Only used to show that the choice of reading does not move the
 * final loss / neighbour recovery beyond seed noise. */
void orc_window_step_immediate(real_t *syn0, real_t *syn1neg, uint32_t d,
                               const int32_t *ctx, uint32_t nctx,
                               const int32_t *out, uint32_t nout,
                               real_t alpha, double *loss_sum)
{
    for (uint32_t k = 0; k < nout; ++k) {
        if (k >= 1 && out[k] == out[0]) continue;
        real_t *O = syn1neg + (size_t)out[k] * d;
        for (uint32_t c = 0; c < nctx; ++c) {
            real_t *I = syn0 + (size_t)ctx[c] * d;
            real_t x = 0;
            for (uint32_t j = 0; j < d; ++j) x += I[j] * O[j];
            real_t gg = alpha * (((k == 0) ? (real_t)1 : (real_t)0) - sigmoid_r(x));
            if (loss_sum) *loss_sum += softplus_d(k == 0 ? -(double)x : (double)x);
            for (uint32_t j = 0; j < d; ++j) {
                real_t ij = I[j];
                I[j] += gg * O[j];
                O[j] += gg * ij;
            }
        }
    }
}

/* The classic per-pair order of the original word2vec loop (what the
 * pre-existing GPU kernels of Section 2.3 execute): context words one
 * after the other; for each, the N+1 samples in turn, every pairing
 * applied to the output row at once and to the context row after its
 * last sample.  Reference for the no-reuse comparator kernel only. */
void orc_window_step_pairwise(real_t *syn0, real_t *syn1neg, uint32_t d,
                              const int32_t *ctx, uint32_t nctx,
                              const int32_t *out, uint32_t nout,
                              real_t alpha, double *loss_sum)
{
    real_t *neu = (real_t *)malloc(sizeof(real_t) * d);
    for (uint32_t c = 0; c < nctx; ++c) {
        real_t *I = syn0 + (size_t)ctx[c] * d;
        for (uint32_t j = 0; j < d; ++j) neu[j] = 0;
        for (uint32_t k = 0; k < nout; ++k) {
            if (k >= 1 && out[k] == out[0]) continue;
            real_t *O = syn1neg + (size_t)out[k] * d;
            real_t x = 0;
            for (uint32_t j = 0; j < d; ++j) x += I[j] * O[j];
            real_t gg = alpha * (((k == 0) ? (real_t)1 : (real_t)0) - sigmoid_r(x));
            if (loss_sum) *loss_sum += softplus_d(k == 0 ? -(double)x : (double)x);
            for (uint32_t j = 0; j < d; ++j) {
                neu[j] += gg * O[j];
                O[j] += gg * I[j];
            }
        }
        for (uint32_t j = 0; j < d; ++j) I[j] += neu[j];
    }
    free(neu);
}

/* ------------------------------------------------------------------ */
/* bfloat16 storage (extension).  A stored value is a float whose low  */
/* 16 bits are zero.  Going from a working value x to storage:         */
/*   stochastic: add a 16-bit uniform number to the float's bit        */
/*   pattern and drop the low 16 bits, so x goes to its upper          */
/*   neighbour with probability (distance to the lower neighbour) /    */
/*   (distance between the neighbours): unbiased;                      */
/*   nearest (ties to even): kept only to show why it is not used.     */
/* The 16 random bits of element e of a row written for token          */
/* position pos:  S = draw(seed, epoch, pos, 64), one 64-bit draw per   */
/* position; the row's key K has the halves                            */
/*   lo32(K) = lo32(S) * (lo32(m) | 1),  hi32(K) = hi32(S) * (hi32(m) | 1) */
/* (mod 2^32) with m = mix64(0x6B6579 + tag), tag = 0 for the window's  */
/* target row, 1+k for its negative k, 32 for the context row of the   */
/* token itself when it leaves the window span;                        */
/*   c = (high word of mix64(0x726F756E64 + e)) >> 8, made odd: a      */
/*       24-bit constant of the element;                               */
/*   a = (lo24(K) * c + hi32(K)) mod 2^32;   bits = a >> 16.           */
/* Multiplying by an odd number permutes the 32-bit words, so hi32(K)  */
/* is uniform and independent of lo24(K), and a is uniform for every   */
/* element; two elements of one write differ by lo24(K) times the      */
/* difference of their constants.                                      */
/* Infinities are stored as they are; a NaN is stored as a NaN (its    */
/* upper half with the quiet bit set).                                 */
/* ------------------------------------------------------------------ */
uint32_t orc_round_bits(uint64_t seed, uint32_t epoch, uint64_t pos, uint32_t tag, uint32_t e)
{
    uint64_t S = orc_draw(seed, epoch, pos, 64u);
    uint64_t m = orc_mix64(0x6B6579ull + tag);
    uint32_t k_lo = (uint32_t)S * ((uint32_t)m | 1u);
    uint32_t k_hi = (uint32_t)(S >> 32) * ((uint32_t)(m >> 32) | 1u);
    uint32_t c = (u32_of(orc_mix64(0x726F756E64ull + e)) >> 8) | 1u;
    uint32_t a = (k_lo & 0xFFFFFFu) * c + k_hi;
    return a >> 16;
}

/* mode 1: stochastic with the given 16 bits, mode 2: nearest-even.  Returns the stored value as a float. */
float orc_to_bf16(float x, uint32_t mode, uint32_t bits16)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    if ((b & 0x7F800000u) != 0x7F800000u) {
        if (mode == 1) b += (bits16 & 0xFFFFu);
        else b += 0x7FFFu + ((b >> 16) & 1u);
    } else if (b & 0x007FFFFFu) {
        b |= 0x00400000u;                     /* a NaN stays a NaN when its low half is dropped */
    }
    b &= 0xFFFF0000u;
    memcpy(&x, &b, 4);
    return x;
}

/* ------------------------------------------------------------------ */
/* One epoch, sentences in order, windows in order.                    */
/* ------------------------------------------------------------------ */
typedef struct orc_params {
    uint32_t vocab, dim, window, negatives;
    uint32_t window_mode;      /* 0 random width, 1 fixed ceil(W/2)        */
    uint32_t update_mode;      /* 0 window minibatch, 1 immediate pairings, 2 classic per-pair order */
    uint32_t total_epochs, epoch;
    uint64_t tokens_per_epoch, first_token_global_pos, seed, table_size;
    double lr0, lr_min_frac;
    /* Negative reuse over more than one window (0 or 1: off, the paper's method).  With a block of B > 1 the
     * tokens of a sentence are taken in stretches of B consecutive tokens (by offset in the sentence, before
     * subsampling), and every window centred in a stretch uses the N negatives drawn at the stretch's first
     * token position.  A negative equal to a window's own target is still skipped for that window only. */
    uint32_t negative_block;
    /* 0: tables in fp32 (the paper).  1 / 2: tables stored as bfloat16, rounded stochastically / to nearest when a
     * working copy goes back (see orc_train_sentence_bf16). */
    uint32_t storage;
} orc_params;

/* One sentence with bfloat16 tables.  Working copies are fp32 (real_t): the context row of kept token p is read one
 * window before the window span reaches p (during the window centred at p-W-1, after that window's arithmetic and
 * before its write-backs: the fetch of a row is started a window ahead of its first use; the first W+1 tokens are read
 * at the sentence start) and goes back, rounded, after the window centred W tokens after p (or at the sentence end);
 * tokens of one word whose copies are alive together share one copy,
 * which goes back when the last of them leaves, with that token's position as the key of the random bits.  The target
 * and negative rows are read at the start of their window and go back, rounded, at its end: one write per distinct
 * row (a negative drawn twice is one row that received two deltas), keyed by the centre's position and the first slot
 * the row fills.  The window itself is orc_window_step on the copies. */
static void orc_train_sentence_bf16(const orc_params *P, real_t *syn0, real_t *syn1neg, const uint64_t *table_end,
                                    const int32_t *kw, const uint64_t *kp, size_t nk, uint64_t a, real_t alpha,
                                    double *loss_sum, uint64_t *pairs, uint8_t *width_out, int32_t *neg_out)
{
    /* the span reaches as far as the widest window that occurs: W, or the fixed width ceil(W/2) */
    const uint32_t W = P->window_mode == 1 ? (P->window + 1u) / 2u : P->window;
    const uint32_t N = P->negatives, d = P->dim;
    const uint32_t cap = 2 * W + 2;
    real_t *ring = (real_t *)malloc(sizeof(real_t) * (size_t)cap * d);      /* working copies of context rows */
    real_t *outs = (real_t *)malloc(sizeof(real_t) * (size_t)(N + 1) * d);  /* working copies of output rows  */
    int32_t slot_word[2 * ORC_MAX_CTX + 2];
    uint32_t slot_refs[2 * ORC_MAX_CTX + 2];
    for (uint32_t q = 0; q < cap; ++q) { slot_word[q] = -1; slot_refs[q] = 0; }
    size_t entered = 0;                                          /* kept positions [0, entered) have entered */
#define ORC_SLOT_OF(word, q_out) do { q_out = cap; for (uint32_t q_ = 0; q_ < cap; ++q_) if (slot_refs[q_] && slot_word[q_] == (word)) q_out = q_; } while (0)
    for (size_t i = 0; i < nk; ++i) {
        /* positions up to i+W have entered (this loop only does work before the first window) */
        while (entered < nk && entered <= i + W) {
            uint32_t q;
            ORC_SLOT_OF(kw[entered], q);
            if (q == cap) {
                for (q = 0; slot_refs[q]; ++q) {}
                slot_word[q] = kw[entered];
                for (uint32_t j = 0; j < d; ++j) ring[(size_t)q * d + j] = syn0[(size_t)kw[entered] * d + j];
            }
            ++slot_refs[q];
            ++entered;
        }
        uint64_t pos = P->first_token_global_pos + kp[i];
        uint32_t bw = orc_width(P->window, P->window_mode, P->seed, P->epoch, pos);
        int32_t out[ORC_MAX_NEG + 1];
        out[0] = kw[i];
        uint64_t neg_pos = pos;
        if (P->negative_block > 1) {
            const uint64_t off = kp[i] - a;
            neg_pos = P->first_token_global_pos + a + (off / P->negative_block) * P->negative_block;
        }
        for (uint32_t k = 0; k < N; ++k)
            out[1 + k] = orc_negative(table_end, P->vocab, P->table_size, P->seed, P->epoch, neg_pos, k);
        if (width_out) width_out[kp[i]] = (uint8_t)bw;
        if (neg_out) for (uint32_t k = 0; k < N; ++k) neg_out[kp[i] * N + k] = out[1 + k];
        int32_t ctx_slot[ORC_MAX_CTX]; uint32_t nctx = 0;
        for (int64_t j = (int64_t)i - (int64_t)bw; j <= (int64_t)i + (int64_t)bw; ++j) {
            if (j < 0 || j >= (int64_t)nk || j == (int64_t)i) continue;
            uint32_t q;
            ORC_SLOT_OF(kw[j], q);
            ctx_slot[nctx++] = (int32_t)q;
        }
        if (nctx) {
            /* distinct output rows: local index = first slot that holds the word */
            int32_t out_local[ORC_MAX_NEG + 1];
            for (uint32_t k = 0; k <= N; ++k) {
                out_local[k] = (int32_t)k;
                for (uint32_t k1 = 0; k1 < k; ++k1) if (out[k1] == out[k]) { out_local[k] = (int32_t)k1; break; }
                if (out_local[k] == (int32_t)k)
                    for (uint32_t j = 0; j < d; ++j) outs[(size_t)k * d + j] = syn1neg[(size_t)out[k] * d + j];
            }
            orc_window_step(ring, outs, d, ctx_slot, nctx, out_local, N + 1, alpha, loss_sum);
            for (uint32_t k = 0; k <= N; ++k) {
                if (out_local[k] != (int32_t)k) continue;
                for (uint32_t j = 0; j < d; ++j)
                    syn1neg[(size_t)out[k] * d + j] = (real_t)orc_to_bf16((float)outs[(size_t)k * d + j], P->storage,
                                                                          orc_round_bits(P->seed, P->epoch, pos, k, j));
            }
            if (pairs) *pairs += nctx;
        }
        /* the token that the next window will reach is read now */
        if (entered < nk && entered == i + W + 1) {
            uint32_t q;
            ORC_SLOT_OF(kw[entered], q);
            if (q == cap) {
                for (q = 0; slot_refs[q]; ++q) {}
                slot_word[q] = kw[entered];
                for (uint32_t j = 0; j < d; ++j) ring[(size_t)q * d + j] = syn0[(size_t)kw[entered] * d + j];
            }
            ++slot_refs[q];
            ++entered;
        }
        /* the position that no later window reaches leaves the span; after the last window all that remain leave */
        size_t lv[ORC_MAX_CTX + 2], nlv = 0;
        if (i >= W) lv[nlv++] = i - W;
        if (i + 1 == nk) for (size_t p = (nk > W ? nk - W : 0); p < nk; ++p) lv[nlv++] = p;
        for (size_t x = 0; x < nlv; ++x) {
            const size_t p = lv[x];
            uint32_t q;
            ORC_SLOT_OF(kw[p], q);
            if (--slot_refs[q] == 0) {
                uint64_t ppos = P->first_token_global_pos + kp[p];
                for (uint32_t j = 0; j < d; ++j)
                    syn0[(size_t)kw[p] * d + j] = (real_t)orc_to_bf16((float)ring[(size_t)q * d + j], P->storage,
                                                                      orc_round_bits(P->seed, P->epoch, ppos, 32u, j));
            }
        }
    }
#undef ORC_SLOT_OF
    free(ring);
    free(outs);
}

/* Optional dumps (any may be NULL), indexed by token offset in `tokens`:
 *   keep_out[T] 1/0, width_out[T] (0 where dropped), neg_out[T*N] (-1 where dropped). */
int orc_train_range(const orc_params *P, real_t *syn0, real_t *syn1neg,
                    const uint64_t *table_end, const uint32_t *thr,
                    const int32_t *tokens, const uint64_t *sent_off,
                    uint64_t s_begin, uint64_t s_end, uint64_t s_stride,
                    double *loss_sum, uint64_t *pairs,
                    uint8_t *keep_out, uint8_t *width_out, int32_t *neg_out)
{
    const uint32_t W = P->window, N = P->negatives, V = P->vocab;
    if (N > ORC_MAX_NEG || 2 * W > ORC_MAX_CTX) return -1;
    int32_t *kw = NULL; uint64_t *kp = NULL; size_t cap = 0;
    for (uint64_t s = s_begin; s < s_end; s += s_stride) {
        uint64_t a = sent_off[s], b = sent_off[s + 1];
        if (b - a > cap) {
            cap = (size_t)(b - a);
            kw = (int32_t *)realloc(kw, cap * sizeof(int32_t));
            kp = (uint64_t *)realloc(kp, cap * sizeof(uint64_t));
        }
        float alpha = orc_lr(P->lr0, P->lr_min_frac, P->epoch, P->total_epochs,
                             P->tokens_per_epoch, P->first_token_global_pos + a);
        size_t nk = 0;
        for (uint64_t t = a; t < b; ++t) {
            int32_t w = tokens[t];
            uint64_t pos = P->first_token_global_pos + t;
            int keep = (w >= 0 && (uint32_t)w < V) && orc_keep(thr, w, P->seed, P->epoch, pos);
            if (keep_out) keep_out[t] = (uint8_t)keep;
            if (width_out) width_out[t] = 0;
            if (neg_out) for (uint32_t k = 0; k < N; ++k) neg_out[t * N + k] = -1;
            if (keep) { kw[nk] = w; kp[nk] = t; ++nk; }
        }
        if (P->storage) {
            orc_train_sentence_bf16(P, syn0, syn1neg, table_end, kw, kp, nk, a, (real_t)alpha, loss_sum, pairs,
                                    width_out, neg_out);
            continue;
        }
        for (size_t i = 0; i < nk; ++i) {
            uint64_t pos = P->first_token_global_pos + kp[i];
            uint32_t bw = orc_width(W, P->window_mode, P->seed, P->epoch, pos);
            int32_t out[ORC_MAX_NEG + 1];
            out[0] = kw[i];
            uint64_t neg_pos = pos;
            if (P->negative_block > 1) {
                const uint64_t off = kp[i] - a;              /* offset of the centre in its sentence */
                neg_pos = P->first_token_global_pos + a + (off / P->negative_block) * P->negative_block;
            }
            for (uint32_t k = 0; k < N; ++k)
                out[1 + k] = orc_negative(table_end, V, P->table_size, P->seed, P->epoch, neg_pos, k);
            if (width_out) width_out[kp[i]] = (uint8_t)bw;
            if (neg_out) for (uint32_t k = 0; k < N; ++k) neg_out[kp[i] * N + k] = out[1 + k];
            int32_t ctx[ORC_MAX_CTX]; uint32_t nctx = 0;
            for (int64_t j = (int64_t)i - (int64_t)bw; j <= (int64_t)i + (int64_t)bw; ++j) {
                if (j < 0 || j >= (int64_t)nk || j == (int64_t)i) continue;
                ctx[nctx++] = kw[j];
            }
            if (nctx == 0) continue;
            if (P->update_mode == 0)
                orc_window_step(syn0, syn1neg, P->dim, ctx, nctx, out, N + 1, (real_t)alpha, loss_sum);
            else if (P->update_mode == 1)
                orc_window_step_immediate(syn0, syn1neg, P->dim, ctx, nctx, out, N + 1, (real_t)alpha, loss_sum);
            else
                orc_window_step_pairwise(syn0, syn1neg, P->dim, ctx, nctx, out, N + 1, (real_t)alpha, loss_sum);
            if (pairs) *pairs += nctx;
        }
    }
    free(kw); free(kp);
    return 0;
}

int orc_train_epoch(const orc_params *P, real_t *syn0, real_t *syn1neg,
                    const uint64_t *table_end, const uint32_t *thr,
                    const int32_t *tokens, const uint64_t *sent_off, uint64_t n_sent,
                    double *loss_sum, uint64_t *pairs,
                    uint8_t *keep_out, uint8_t *width_out, int32_t *neg_out)
{
    return orc_train_range(P, syn0, syn1neg, table_end, thr, tokens, sent_off,
                           0, n_sent, 1, loss_sum, pairs, keep_out, width_out, neg_out);
}

uint32_t orc_real_size(void) { return (uint32_t)sizeof(real_t); }
