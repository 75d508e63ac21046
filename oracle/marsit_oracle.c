/*
 * marsit_oracle.c -- plain CPU oracle for the one-bit synchronisation pass of Marsit
 * ("Sign Bit is Enough", arXiv 2204.06787).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, by-eye-checkable statement of what the
 * hot path computes.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or constant generator with the HIP library; the
 * product never routes through it.
 *
 * What it follows
 *   - Algorithm 1, the branch mod(t,K) != 0, step by step in its order: compensated gradient,
 *     split into M parts, per-part chain of "sign, merge, send", decode, global compensation.
 *   - Eq. 2 of Section 4.1.1: the transient Bernoulli vector v.
 *   - The operator  v_i (.) v_i* = (v_i AND v_i*) OR ((v_i XOR v_i*) AND v)  of Section 4.1.1.
 *   - Algorithm 1, the branch mod(t,K) == 0: full-precision mean, c <- 0.
 *   - Algorithm 2, the model update: x <- x - g_t.
 *
 * Readings taken where the paper is silent (each is listed in the design notes of the build):
 *   - "m" in Eq. 2 is the fold count: how many workers' signs the outgoing vector will stand
 *     for, the local one included.  Hop h of a chain (h = 1..M-1) has m = h + 1.
 *   - bit 1 means +1.  sgn() is the complement of the IEEE-754 sign bit (+0 -> +1, -0 -> -1).
 *   - Bernoulli draws: one 32-bit word u per (seed, hop, packed word, bit);
 *       keep-local indicator t = (u < floor(2^32 / m)),  v = XNOR(v*, t)   (that is Eq. 2).
 *     u is the j-th 32-bit output of the Philox4x32-10 stream with key = the 64-bit seed and
 *     counter = (j / 4, hop id, word index low, word index high); j = bit position 0..63.
 *   - Packing: element e sits in 64-bit word e / 64 at bit e % 64 (least significant first);
 *     bits at positions >= d are zero.
 *   - Split into parts: word-aligned, part i = words [floor(i*W/P), floor((i+1)*W/P)).
 *   - Ring: part i starts at worker i; hop h folds in worker (i + h) mod M.
 *   - 2D torus, X columns by Y rows, worker (y, x) = y*X + x: rows first (ring over the X
 *     columns inside every row, parts = X row-parts of the W words), then columns (ring over
 *     the Y row results, every row-part split again in Y sub-parts).
 *   - A torus whose last row is short (M not a multiple of X): rows as above with their own
 *     length, the column merges weighted by the workers each side stands for.
 *   - Arithmetic type: the gradients and the compensation are fp32 vectors (Section 1 speaks
 *     of 32-bit single precision), so the compensated sum and the compensation update are one fp32 round-to-nearest-even
 *     operation each.  Build with -ffp-contract=off and without fast-math.
 *
 * Parity status: the building blocks are pinned by tests (exact enumeration of the
 * unbiasedness property, binomial frequency tests, identity cases, an independently written
 * second formulation, numpy reductions, Philox known answers).  The specific merged bitmaps
 * for a given seed have no published worked example: "parity unpinned" beyond those pins.
 */

#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ORACLE_MAX_WORKERS 64

/* ------------------------------------------------------------------------------------------
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11).  Four 32-bit counter words, two 32-bit key words, ten rounds.  The key is bumped by
 * the two Weyl constants before every round but the first.
 * ---------------------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t mult_a = 0xD2511F53u;   /* multiplies counter word 0 */
    const uint32_t mult_b = 0xCD9E8D57u;   /* multiplies counter word 2 */
    const uint32_t weyl_a = 0x9E3779B9u;   /* golden ratio               */
    const uint32_t weyl_b = 0xBB67AE85u;   /* sqrt(3) - 1                */

    uint32_t x0 = ctr[0], x1 = ctr[1], x2 = ctr[2], x3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];

    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += weyl_a;
            k1 += weyl_b;
        }
        uint64_t prod_a = (uint64_t)mult_a * (uint64_t)x0;
        uint64_t prod_b = (uint64_t)mult_b * (uint64_t)x2;
        uint32_t hi_a = (uint32_t)(prod_a >> 32), lo_a = (uint32_t)prod_a;
        uint32_t hi_b = (uint32_t)(prod_b >> 32), lo_b = (uint32_t)prod_b;
        uint32_t y0 = hi_b ^ x1 ^ k0;
        uint32_t y1 = lo_b;
        uint32_t y2 = hi_a ^ x3 ^ k1;
        uint32_t y3 = lo_a;
        x0 = y0; x1 = y1; x2 = y2; x3 = y3;
    }
    out[0] = x0; out[1] = x1; out[2] = x2; out[3] = x3;
}

/* The j-th 32-bit word (j = 0..63) of the stream that belongs to (seed, hop id, word index). */
uint32_t oracle_stream_u32(uint64_t seed, uint32_t hop_id, uint64_t word_index, uint32_t j)
{
    uint32_t ctr[4], key[2], out[4];
    ctr[0] = j / 4u;
    ctr[1] = hop_id;
    ctr[2] = (uint32_t)(word_index & 0xFFFFFFFFu);
    ctr[3] = (uint32_t)(word_index >> 32);
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    oracle_philox4x32_10(ctr, key, out);
    return out[j % 4u];
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1, compensated gradient:  g <- g + c   (elementwise, fp32).
 * ---------------------------------------------------------------------------------------- */
void oracle_add_compensation(const float *g, const float *c, float *s, uint64_t d)
{
    for (uint64_t e = 0; e < d; ++e) {
        float ce = (c != NULL) ? c[e] : 0.0f;
        s[e] = g[e] + ce;                        /* one rounding to fp32 */
    }
}

/* sgn() of one fp32 value as a bit: 1 for +, 0 for -, decided by the IEEE-754 sign bit. */
static unsigned sign_bit_plus(float x)
{
    uint32_t raw;
    memcpy(&raw, &x, sizeof raw);
    return (raw >> 31) ? 0u : 1u;
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1, sign step:  v* <- sgn(g_part), stored one bit per element.
 * bits has ceil(d/64) words; positions >= d stay 0.
 * ---------------------------------------------------------------------------------------- */
void oracle_sign_pack(const float *s, uint64_t *bits, uint64_t d)
{
    uint64_t n_words = (d + 63u) / 64u;
    for (uint64_t w = 0; w < n_words; ++w)
        bits[w] = 0;
    for (uint64_t e = 0; e < d; ++e) {
        if (sign_bit_plus(s[e]))
            bits[e / 64u] |= (uint64_t)1 << (e % 64u);
    }
}

/* Inverse of the packing: out[e] = +1.0f or -1.0f. */
void oracle_sign_unpack(const uint64_t *bits, float *out, uint64_t d)
{
    for (uint64_t e = 0; e < d; ++e)
        out[e] = ((bits[e / 64u] >> (e % 64u)) & 1u) ? 1.0f : -1.0f;
}

/* ------------------------------------------------------------------------------------------
 * Eq. 2: the transient vector for one packed word, given the local sign word v*, the fold
 * count m and the 64 "keep local" outcomes t (bit j of keep: the Bernoulli(1/m) draw of bit j
 * came up).   b_j = (m-1)/m if v*_j = 0,  1/m if v*_j = 1   <=>   v_j = NOT (v*_j XOR t_j).
 * ---------------------------------------------------------------------------------------- */
uint64_t oracle_transient_from_keep(uint64_t local, uint64_t keep)
{
    uint64_t v = 0;
    for (unsigned j = 0; j < 64; ++j) {
        unsigned l = (unsigned)((local >> j) & 1u);
        unsigned t = (unsigned)((keep >> j) & 1u);
        unsigned vj = (l == 1u) ? t : (1u - t);     /* P(v=1) = 1/m when v*=1, (m-1)/m when v*=0 */
        v |= (uint64_t)vj << j;
    }
    return v;
}

/* The 64 Bernoulli(1/m) outcomes of (seed, hop id, word): t_j = (u_j < floor(2^32/m)). */
uint64_t oracle_keep_mask(uint32_t fold, uint32_t hop_id, uint64_t seed, uint64_t word_index)
{
    uint64_t threshold = ((uint64_t)1 << 32) / (uint64_t)fold;   /* 2^32 when fold == 1 */
    uint64_t keep = 0;
    for (unsigned j = 0; j < 64; ++j) {
        uint64_t u = oracle_stream_u32(seed, hop_id, word_index, j);
        if (u < threshold)
            keep |= (uint64_t)1 << j;
    }
    return keep;
}

/* The operator of Section 4.1.1:  (recv AND local) OR ((recv XOR local) AND v). */
uint64_t oracle_odot(uint64_t recv, uint64_t local, uint64_t v)
{
    return (recv & local) | ((recv ^ local) & v);
}

/* One hop for one packed word: draw v by Eq. 2, then apply the operator. */
uint64_t oracle_merge_word(uint64_t recv, uint64_t local, uint32_t fold, uint32_t hop_id,
                           uint64_t seed, uint64_t word_index)
{
    uint64_t keep = oracle_keep_mask(fold, hop_id, seed, word_index);
    uint64_t v = oracle_transient_from_keep(local, keep);
    return oracle_odot(recv, local, v);
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1, merge step, for a run of words: out = recv (.) local.
 * word_begin is the global index of the first word (it keys the random stream).
 * Returns 0, or -1 on a bad argument.
 * ---------------------------------------------------------------------------------------- */
int oracle_hop_merge(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                     uint64_t word_begin, uint64_t n_words, uint32_t fold, uint32_t hop_id,
                     uint64_t seed)
{
    if (fold == 0)
        return -1;
    for (uint64_t i = 0; i < n_words; ++i)
        out[i] = oracle_merge_word(recv[i], local[i], fold, hop_id, seed, word_begin + i);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1, aggregation of the global update:  g_t <- eta_s * (union of the final sign parts): +scale or -scale.
 * ---------------------------------------------------------------------------------------- */
void oracle_decode(const uint64_t *bits, float scale, float *update, uint64_t d)
{
    for (uint64_t e = 0; e < d; ++e) {
        unsigned bit = (unsigned)((bits[e / 64u] >> (e % 64u)) & 1u);
        update[e] = bit ? scale : -scale;
    }
}

/* Algorithm 1, compensation update:  c_{t+1} <- g (the compensated gradient) - g_t. */
void oracle_compensate(const float *s, const float *update, float *c_next, uint64_t d)
{
    for (uint64_t e = 0; e < d; ++e) {
        c_next[e] = s[e] - update[e];            /* one rounding to fp32 */
    }
}

/* Algorithm 1, split step: bounds[i] = floor(i * n / parts) + begin, i = 0..parts. */
void oracle_split_bounds(uint64_t begin, uint64_t n, uint32_t parts, uint64_t *bounds)
{
    for (uint32_t i = 0; i <= parts; ++i)
        bounds[i] = begin + (uint64_t)(((unsigned __int128)i * n) / parts);
}

static uint32_t part_of(uint64_t w, const uint64_t *bounds, uint32_t parts)
{
    for (uint32_t i = 0; i < parts; ++i)
        if (bounds[i] <= w && w < bounds[i + 1])
            return i;
    return parts - 1;   /* not reached for w inside [bounds[0], bounds[parts]) */
}

/* hop ids: row phase (phase 0) carries the row y and the hop h; column phase (phase 1) the hop. */
uint32_t oracle_hop_id(uint32_t phase, uint32_t row, uint32_t hop)
{
    return (phase << 16) | (row << 8) | hop;
}

/* ------------------------------------------------------------------------------------------
 * The whole one-bit pass for M simulated workers (Algorithm 1, the branch mod(t,K) != 0).
 *
 *   g          [M][ld]  gradients (already scaled by the local step, as Algorithm 2 passes them)
 *   c          [M][ld]  compensation, read as c_t and overwritten with c_{t+1}
 *   update     [d]      g_t
 *   bits_final [W]      the final merged bitmap every worker ends up with (may be NULL)
 *   sign_maps  [M][W]   every worker's own v* (may be NULL)
 *   grid_x     0 or M: ring.  Otherwise X columns, Y = M / X rows, rows first.
 *   threads    > 1: the loop over packed words is run by that many OpenMP threads (the words
 *              are independent because the stream is counter based); results do not change.
 * Returns 0, -1 for bad arguments, -2 if memory ran out.
 * ---------------------------------------------------------------------------------------- */
int oracle_sync_step(const float *g, float *c, float *update, uint64_t *bits_final,
                     uint64_t *sign_maps, uint32_t M, uint64_t d, uint64_t ld, float scale,
                     uint64_t seed, uint32_t grid_x, int threads)
{
    if (M == 0 || M > ORACLE_MAX_WORKERS || ld < d || g == NULL || c == NULL || update == NULL)
        return -1;
    uint32_t X = (grid_x == 0) ? M : grid_x;
    if (X == 0 || M % X != 0)
        return -1;
    uint32_t Y = M / X;
    if (d == 0)
        return 0;
    if (threads < 1)
        threads = 1;

    uint64_t W = (d + 63u) / 64u;
    float *s = (float *)malloc((size_t)M * d * sizeof(float));
    uint64_t *L = (uint64_t *)malloc((size_t)M * W * sizeof(uint64_t));
    uint64_t *B = (uint64_t *)malloc((size_t)W * sizeof(uint64_t));
    if (s == NULL || L == NULL || B == NULL) {
        free(s); free(L); free(B);
        return -2;
    }

    /* compensated gradient and its signs, for every worker */
    for (uint32_t m = 0; m < M; ++m) {
        oracle_add_compensation(g + (size_t)m * ld, c + (size_t)m * ld, s + (size_t)m * d, d);
        oracle_sign_pack(s + (size_t)m * d, L + (size_t)m * W, d);
    }

    /* split step: the W packed words are split in X row-parts */
    uint64_t row_bounds[ORACLE_MAX_WORKERS + 1];
    oracle_split_bounds(0, W, X, row_bounds);

    /* the loop over the parts (sign, merge, send), one packed word at a time */
    #pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
    for (uint64_t w = 0; w < W; ++w) {
        uint32_t a = part_of(w, row_bounds, X);

        /* row phase: in every row y the chain of part a starts at column a */
        uint64_t R[ORACLE_MAX_WORKERS];
        for (uint32_t y = 0; y < Y; ++y) {
            uint64_t r = L[(size_t)(y * X + a) * W + w];          /* first holder sends its own signs */
            for (uint32_t h = 1; h < X; ++h) {
                uint32_t col = (a + h) % X;
                uint64_t local = L[(size_t)(y * X + col) * W + w];
                r = oracle_merge_word(r, local, h + 1u, oracle_hop_id(0, y, h), seed, w);
            }
            R[y] = r;
        }

        /* column phase: row-part a is split again in Y sub-parts; chain of sub-part b starts at row b */
        uint64_t col_bounds[ORACLE_MAX_WORKERS + 1];
        oracle_split_bounds(row_bounds[a], row_bounds[a + 1] - row_bounds[a], Y, col_bounds);
        uint32_t b = part_of(w, col_bounds, Y);
        uint64_t r = R[b];
        for (uint32_t k = 1; k < Y; ++k) {
            uint64_t local = R[(b + k) % Y];
            r = oracle_merge_word(r, local, k + 1u, oracle_hop_id(1, 0, k), seed, w);
        }
        B[w] = r;
    }

    /* global update, then compensation update */
    oracle_decode(B, scale, update, d);
    for (uint32_t m = 0; m < M; ++m)
        oracle_compensate(s + (size_t)m * d, update, c + (size_t)m * ld, d);

    if (bits_final != NULL)
        memcpy(bits_final, B, (size_t)W * sizeof(uint64_t));
    if (sign_maps != NULL)
        memcpy(sign_maps, L, (size_t)M * W * sizeof(uint64_t));
    free(s); free(L); free(B);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1, the branch mod(t,K) == 0 (full-precision round):  g_t <- (1/M) sum_m (g^(m) + c^(m)),  c <- 0.
 * The sum is taken in double and rounded once to fp32.
 * ---------------------------------------------------------------------------------------- */
int oracle_full_sync(const float *g, float *c, float *update, uint32_t M, uint64_t d, uint64_t ld)
{
    if (M == 0 || ld < d || g == NULL || c == NULL || update == NULL)
        return -1;
    for (uint64_t e = 0; e < d; ++e) {
        double acc = 0.0;
        for (uint32_t m = 0; m < M; ++m) {
            float sm = g[(size_t)m * ld + e] + c[(size_t)m * ld + e];   /* compensated gradient, fp32 */
            acc += (double)sm;
        }
        update[e] = (float)(acc / (double)M);
    }
    for (uint32_t m = 0; m < M; ++m)
        for (uint64_t e = 0; e < d; ++e)
            c[(size_t)m * ld + e] = 0.0f;
    return 0;
}

/* Algorithm 2, model update:  x <- x - g_t. */
void oracle_apply_update(float *x, const float *update, uint64_t d)
{
    for (uint64_t e = 0; e < d; ++e) {
        x[e] = x[e] - update[e];
    }
}

/*
 * Local momentum of a worker (Section 5, "Optimizers and hyper-parameters": the image runs use the
 * Momentum optimizer; the paper prints no formula, so the common heavy-ball form is taken):
 *     buf <- beta * buf + grad;     g <- eta_l * buf,
 * one fp32 rounding per operation (product, sum, product), for every worker m and element e < d.
 * g is what Algorithm 2 hands to Marsit as its (already scaled) gradient.
 */
int oracle_local_momentum(float *buf, const float *grad, float *g_out, uint32_t M, uint64_t d,
                          uint64_t ld, float beta, float eta_l)
{
    if (ld < d)
        return -1;
    for (uint32_t m = 0; m < M; ++m) {
        for (uint64_t e = 0; e < d; ++e) {
            const size_t i = (size_t)m * ld + e;
            const float carried = beta * buf[i];
            const float v = carried + grad[i];
            buf[i] = v;
            g_out[i] = eta_l * v;
        }
    }
    return 0;
}

/*
 * Local Adam of a worker (Section 5, "Optimizers and hyper-parameters": the sentiment-analysis runs
 * use Adam; the paper prints no formula, so the optimizer's published form with bias correction is
 * taken).  Per worker m and element e < d, with first moment p, second moment q and gradient a:
 *     p <- beta1 * p + (1 - beta1) * a
 *     q <- beta2 * q + (1 - beta2) * (a * a)
 *     g <- eta_l * ( (p / bias1) / (sqrt(q / bias2) + eps) )
 * bias1 = 1 - beta1^t and bias2 = 1 - beta2^t are the caller's (they depend on the round only).
 * Every operation is one fp32 rounding, in the order written: 1 - beta is rounded once; each
 * moment is product, product, sum; the step is quotient, quotient, root, sum, quotient, product.
 * g is what Algorithm 2 hands to Marsit as its (already scaled) gradient.
 */
int oracle_local_adam(float *mom1, float *mom2, const float *grad, float *g_out, uint32_t M,
                      uint64_t d, uint64_t ld, float beta1, float beta2, float eps, float eta_l,
                      float bias1, float bias2)
{
    if (ld < d)
        return -1;
    const float rest1 = 1.0f - beta1;
    const float rest2 = 1.0f - beta2;
    for (uint32_t m = 0; m < M; ++m) {
        for (uint64_t e = 0; e < d; ++e) {
            const size_t i = (size_t)m * ld + e;
            const float a = grad[i];
            const float p_old = beta1 * mom1[i];
            const float p_new = rest1 * a;
            const float p = p_old + p_new;
            const float a2 = a * a;
            const float q_old = beta2 * mom2[i];
            const float q_new = rest2 * a2;
            const float q = q_old + q_new;
            mom1[i] = p;
            mom2[i] = q;
            const float p_hat = p / bias1;
            const float q_hat = q / bias2;
            const float root = sqrtf(q_hat);
            const float denom = root + eps;
            const float dir = p_hat / denom;
            g_out[i] = eta_l * dir;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Diagnostics of Section 3.2.2 / Fig. 2(b): the "matching rate" of a sign vector is the share of
 * elements whose sign equals the sign of the non-compressed aggregate sum_m (g^(m) + c^(m)).
 * The aggregate is summed in double, in worker order.
 * ---------------------------------------------------------------------------------------- */
void oracle_aggregate_sign(const float *g, const float *c, uint64_t *bits, uint32_t M, uint64_t d,
                           uint64_t ld)
{
    uint64_t n_words = (d + 63u) / 64u;
    for (uint64_t w = 0; w < n_words; ++w)
        bits[w] = 0;
    for (uint64_t e = 0; e < d; ++e) {
        double acc = 0.0;
        for (uint32_t m = 0; m < M; ++m) {
            float sm = g[(size_t)m * ld + e] + c[(size_t)m * ld + e];     /* compensated gradient of Algorithm 1, fp32 */
            acc += (double)sm;
        }
        uint64_t raw;
        memcpy(&raw, &acc, sizeof raw);
        if ((raw >> 63) == 0)
            bits[e / 64u] |= (uint64_t)1 << (e % 64u);
    }
}

/* signSGD with majority vote (one of the paper's comparison points): +1 where at least as many
 * workers have a + sign as a - sign (a tie counts as +). */
void oracle_majority_vote(const float *g, const float *c, uint64_t *bits, uint32_t M, uint64_t d,
                          uint64_t ld)
{
    uint64_t n_words = (d + 63u) / 64u;
    for (uint64_t w = 0; w < n_words; ++w)
        bits[w] = 0;
    for (uint64_t e = 0; e < d; ++e) {
        uint32_t plus = 0;
        for (uint32_t m = 0; m < M; ++m) {
            float sm = g[(size_t)m * ld + e] + c[(size_t)m * ld + e];
            plus += sign_bit_plus(sm);
        }
        if (2u * plus >= M)
            bits[e / 64u] |= (uint64_t)1 << (e % 64u);
    }
}

/* Number of positions e < d at which two sign bitmaps agree. */
uint64_t oracle_count_matching(const uint64_t *a, const uint64_t *b, uint64_t d)
{
    uint64_t count = 0;
    for (uint64_t e = 0; e < d; ++e) {
        unsigned ba = (unsigned)((a[e / 64u] >> (e % 64u)) & 1u);
        unsigned bb = (unsigned)((b[e / 64u] >> (e % 64u)) & 1u);
        if (ba == bb)
            ++count;
    }
    return count;
}

/* ------------------------------------------------------------------------------------------
 * Other multi-hop schedules (Section 5 says the method extends to tree all-reduce and others, with
 * no detail).  Reading taken: when the two operands of a merge stand for different numbers of
 * workers, Eq. 2 is used with the local share in place of 1/m:
 *     b_j = w_recv / (w_recv + w_local)  if v*_j = 0,   w_local / (w_recv + w_local)  if v*_j = 1,
 * i.e. the local sign is kept with probability w_local / (w_recv + w_local), decided by
 * u < floor(2^32 * w_local / (w_recv + w_local)).  w_local = 1, w_recv = m - 1 is Eq. 2 itself.
 * ---------------------------------------------------------------------------------------- */
uint64_t oracle_weighted_threshold(uint32_t w_recv, uint32_t w_local)
{
    return (((uint64_t)w_local) << 32) / ((uint64_t)w_recv + (uint64_t)w_local);   /* 2^32 if w_recv == 0 */
}

uint64_t oracle_merge_word_weighted(uint64_t recv, uint64_t local, uint32_t w_recv, uint32_t w_local,
                                    uint32_t hop_id, uint64_t seed, uint64_t word_index)
{
    uint64_t threshold = oracle_weighted_threshold(w_recv, w_local);
    uint64_t keep = 0;
    for (unsigned j = 0; j < 64; ++j) {
        uint64_t u = oracle_stream_u32(seed, hop_id, word_index, j);
        if (u < threshold)
            keep |= (uint64_t)1 << j;
    }
    uint64_t v = oracle_transient_from_keep(local, keep);
    return oracle_odot(recv, local, v);
}

int oracle_hop_merge_weighted(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                              uint64_t word_begin, uint64_t n_words, uint32_t w_recv, uint32_t w_local,
                              uint32_t hop_id, uint64_t seed)
{
    if (w_local == 0)
        return -1;
    for (uint64_t i = 0; i < n_words; ++i)
        out[i] = oracle_merge_word_weighted(recv[i], local[i], w_recv, w_local, hop_id, seed,
                                            word_begin + i);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * The one-bit pass over a torus whose last row is short (M need not be a multiple of the number
 * of columns; Section 5 names further all-reduce layouts without detail):
 *   X columns, Y = ceil(M / X) rows, worker (y, x) = y*X + x for y*X + x < M; row y has
 *   X_y = X workers, except the last one with M - (Y-1)*X.
 *   Row phase: the W words are split in X row-parts; in row y the chain of row-part a starts at
 *   column a mod X_y and folds columns (start + h) mod X_y, h = 1..X_y-1, fold count h + 1,
 *   hop id (y << 8) | h.  The row result stands for X_y workers.
 *   Column phase: row-part a is split again in Y sub-parts; the chain of sub-part b starts at
 *   row b and folds rows (b + k) mod Y, k = 1..Y-1, each side weighted by the workers it stands
 *   for (the weighted merge), hop id (1 << 16) | k.
 * With X dividing M every weight ratio is 1/(k+1) and this is oracle_sync_step bit for bit.
 * ---------------------------------------------------------------------------------------- */
int oracle_ragged_torus_step(const float *g, float *c, float *update, uint64_t *bits_final,
                             uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                             uint32_t grid_x, int threads)
{
    if (M == 0 || M > ORACLE_MAX_WORKERS || ld < d || g == NULL || c == NULL || update == NULL ||
        grid_x == 0 || grid_x > M)
        return -1;
    const uint32_t X = grid_x;
    const uint32_t Y = (M + X - 1) / X;
    const uint32_t X_last = M - (Y - 1) * X;
    if (d == 0)
        return 0;
    if (threads < 1)
        threads = 1;

    uint64_t W = (d + 63u) / 64u;
    float *s = (float *)malloc((size_t)M * d * sizeof(float));
    uint64_t *L = (uint64_t *)malloc((size_t)M * W * sizeof(uint64_t));
    uint64_t *B = (uint64_t *)malloc((size_t)W * sizeof(uint64_t));
    if (s == NULL || L == NULL || B == NULL) {
        free(s); free(L); free(B);
        return -2;
    }
    for (uint32_t m = 0; m < M; ++m) {
        oracle_add_compensation(g + (size_t)m * ld, c + (size_t)m * ld, s + (size_t)m * d, d);
        oracle_sign_pack(s + (size_t)m * d, L + (size_t)m * W, d);
    }
    uint64_t row_bounds[ORACLE_MAX_WORKERS + 1];
    oracle_split_bounds(0, W, X, row_bounds);

    #pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
    for (uint64_t w = 0; w < W; ++w) {
        uint32_t a = part_of(w, row_bounds, X);

        uint64_t R[ORACLE_MAX_WORKERS];
        uint32_t weight[ORACLE_MAX_WORKERS];
        for (uint32_t y = 0; y < Y; ++y) {
            uint32_t Xy = (y + 1 < Y) ? X : X_last;
            uint32_t start = a % Xy;
            uint64_t r = L[(size_t)(y * X + start) * W + w];
            for (uint32_t h = 1; h < Xy; ++h) {
                uint32_t col = (start + h) % Xy;
                uint64_t local = L[(size_t)(y * X + col) * W + w];
                r = oracle_merge_word(r, local, h + 1u, oracle_hop_id(0, y, h), seed, w);
            }
            R[y] = r;
            weight[y] = Xy;
        }

        uint64_t col_bounds[ORACLE_MAX_WORKERS + 1];
        oracle_split_bounds(row_bounds[a], row_bounds[a + 1] - row_bounds[a], Y, col_bounds);
        uint32_t b = part_of(w, col_bounds, Y);
        uint64_t r = R[b];
        uint32_t gathered = weight[b];                 /* workers the running result stands for */
        for (uint32_t k = 1; k < Y; ++k) {
            uint32_t row = (b + k) % Y;
            r = oracle_merge_word_weighted(r, R[row], gathered, weight[row], oracle_hop_id(1, 0, k),
                                           seed, w);
            gathered += weight[row];
        }
        B[w] = r;
    }

    oracle_decode(B, scale, update, d);
    for (uint32_t m = 0; m < M; ++m)
        oracle_compensate(s + (size_t)m * d, update, c + (size_t)m * ld, d);
    if (bits_final != NULL)
        memcpy(bits_final, B, (size_t)W * sizeof(uint64_t));
    free(s); free(L); free(B);
    return 0;
}

/* hop id of a tree merge: phase 2, the level and the receiving worker. */
uint32_t oracle_tree_hop_id(uint32_t level, uint32_t receiver)
{
    return (2u << 16) | (level << 8) | receiver;
}

/* ------------------------------------------------------------------------------------------
 * The one-bit pass over a binary reduction tree (whole vectors, no split in parts): at level l
 * (stride 2^l) worker k = 0, 2*2^l, 4*2^l, ... receives the sign vector of worker k + 2^l and
 * folds it into its own; each side stands for the workers of its subtree.  After ceil(log2 M)
 * levels worker 0 holds the final vector (then broadcast).  Same arguments as oracle_sync_step.
 * ---------------------------------------------------------------------------------------- */
int oracle_tree_step(const float *g, float *c, float *update, uint64_t *bits_final, uint32_t M,
                     uint64_t d, uint64_t ld, float scale, uint64_t seed)
{
    if (M == 0 || M > ORACLE_MAX_WORKERS || ld < d || g == NULL || c == NULL || update == NULL)
        return -1;
    if (d == 0)
        return 0;
    uint64_t W = (d + 63u) / 64u;
    float *s = (float *)malloc((size_t)M * d * sizeof(float));
    uint64_t *B = (uint64_t *)malloc((size_t)M * W * sizeof(uint64_t));
    if (s == NULL || B == NULL) {
        free(s); free(B);
        return -2;
    }
    for (uint32_t m = 0; m < M; ++m) {
        oracle_add_compensation(g + (size_t)m * ld, c + (size_t)m * ld, s + (size_t)m * d, d);
        oracle_sign_pack(s + (size_t)m * d, B + (size_t)m * W, d);
    }
    uint32_t level = 0;
    for (uint32_t stride = 1; stride < M; stride *= 2, ++level) {
        for (uint32_t k = 0; k + stride < M; k += 2 * stride) {
            uint32_t src = k + stride;
            uint32_t w_local = (M - k < stride) ? (M - k) : stride;       /* workers under k so far   */
            uint32_t w_recv = (M - src < stride) ? (M - src) : stride;    /* workers under the sender */
            oracle_hop_merge_weighted(B + (size_t)src * W, B + (size_t)k * W, B + (size_t)k * W, 0, W,
                                      w_recv, w_local, oracle_tree_hop_id(level, k), seed);
        }
    }
    oracle_decode(B, scale, update, d);
    for (uint32_t m = 0; m < M; ++m)
        oracle_compensate(s + (size_t)m * d, update, c + (size_t)m * ld, d);
    if (bits_final != NULL)
        memcpy(bits_final, B, (size_t)W * sizeof(uint64_t));
    free(s); free(B);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * The strawman of Section 3.2: SSDM's stochastic sign Q(.) and cascading compression.
 *
 * Appendix A: an element v_j is compressed to +1 with probability 1/2 + v_j / (2 ||v||), to -1
 * otherwise; Q(v) = ||v|| * sign~(v), an unbiased estimate of v.  (Section 3.2 prints the
 * probability as 1/2 + |g_i| / ||g||; the appendix form is the one whose expectation the proof
 * uses, and the one taken here.)
 *
 * Arithmetic, fixed so that the stochastic decision is the same integer on every machine:
 *   norm   = sqrtf( (float) sum_j (double)t_j * (double)t_j )        (sum in double)
 *   p_j    = 0.5f + t_j / (2.0f * norm)     in fp32, one rounding per operation; 0.5f if norm == 0
 *   bit_j  = 1  iff  (double)u_j < (double)p_j * 2^32,
 * u_j being the j-th 32-bit word of the Philox stream of (seed, hop id, packed word).
 * ---------------------------------------------------------------------------------------- */
float oracle_l2_norm(const float *t, uint64_t n)
{
    double acc = 0.0;
    for (uint64_t e = 0; e < n; ++e)
        acc += (double)t[e] * (double)t[e];
    return sqrtf((float)acc);
}

/* bits[] covers the n elements starting at bit 0 of word 0; word_begin keys the stream. */
void oracle_ssdm_sign(const float *t, float norm, uint64_t *bits, uint64_t n, uint64_t word_begin,
                      uint32_t hop_id, uint64_t seed)
{
    uint64_t n_words = (n + 63u) / 64u;
    for (uint64_t w = 0; w < n_words; ++w)
        bits[w] = 0;
    for (uint64_t e = 0; e < n; ++e) {
        float p = 0.5f;
        if (norm != 0.0f) {
            float twice = 2.0f * norm;
            float q = t[e] / twice;
            p = 0.5f + q;
        }
        uint32_t u = oracle_stream_u32(seed, hop_id, word_begin + e / 64u, (uint32_t)(e % 64u));
        if ((double)u < (double)p * 4294967296.0)
            bits[e / 64u] |= (uint64_t)1 << (e % 64u);
    }
}

/* hop ids of the cascading chain: phase 3, hop h (h = 0 is the first holder's own compression). */
uint32_t oracle_cascade_hop_id(uint32_t hop)
{
    return (3u << 16) | hop;
}

/* ------------------------------------------------------------------------------------------
 * Cascading compression over the ring (Section 3.2's five steps), per part i of the word-aligned
 * split: the first holder sends Q(s^(i)); at hop h worker (i+h) mod M receives (norm, signs),
 * recovers w = norm * signs, aggregates t = w + s^(local), compresses Q(t) and sends it on.
 * After M-1 hops the part's result is (1/M) * norm * signs.
 *   g, c        [M][ld]; s = g + c as in Algorithm 1 (c is NOT updated: the strawman has no
 *               compensation step)
 *   bits_final  [W] final signs;  norms_final [M] final norm of every part
 *   update      [d]  (1/M) * norm_part * (+-1)
 * Returns 0, -1 for bad arguments, -2 if memory ran out.
 * ---------------------------------------------------------------------------------------- */
int oracle_cascade_ring_step(const float *g, const float *c, float *update, uint64_t *bits_final,
                             float *norms_final, uint32_t M, uint64_t d, uint64_t ld, uint64_t seed)
{
    if (M == 0 || M > ORACLE_MAX_WORKERS || ld < d || g == NULL || c == NULL || update == NULL ||
        bits_final == NULL || norms_final == NULL)
        return -1;
    if (d == 0)
        return 0;
    uint64_t W = (d + 63u) / 64u;
    uint64_t bounds[ORACLE_MAX_WORKERS + 1];
    oracle_split_bounds(0, W, M, bounds);
    uint64_t max_elems = (W / M + 1u) * 64u;
    float *t = (float *)malloc((size_t)max_elems * sizeof(float));
    uint64_t *bits = (uint64_t *)malloc((size_t)(W / M + 1u) * sizeof(uint64_t));
    if (t == NULL || bits == NULL) {
        free(t); free(bits);
        return -2;
    }
    for (uint32_t i = 0; i < M; ++i) {
        uint64_t lo = bounds[i], hi = bounds[i + 1];
        norms_final[i] = 0.0f;
        if (hi == lo)
            continue;
        uint64_t e0 = lo * 64u, e1 = (hi * 64u < d) ? hi * 64u : d, n = e1 - e0;
        float norm = 0.0f;
        for (uint32_t h = 0; h < M; ++h) {
            uint32_t worker = (i + h) % M;
            for (uint64_t e = 0; e < n; ++e) {
                float local = g[(size_t)worker * ld + e0 + e] + c[(size_t)worker * ld + e0 + e];
                if (h == 0) {
                    t[e] = local;                                   /* first holder: its own vector */
                } else {
                    float recovered = ((bits[e / 64u] >> (e % 64u)) & 1u) ? norm : -norm;   /* recover */
                    t[e] = recovered + local;                        /* aggregate */
                }
            }
            norm = oracle_l2_norm(t, n);                             /* compress ... */
            oracle_ssdm_sign(t, norm, bits, n, lo, oracle_cascade_hop_id(h), seed);
        }                                                            /* ... and send */
        norms_final[i] = norm;
        for (uint64_t w = lo; w < hi; ++w)
            bits_final[w] = bits[w - lo];
        for (uint64_t e = 0; e < n; ++e) {
            float v = ((bits[e / 64u] >> (e % 64u)) & 1u) ? norm : -norm;
            update[e0 + e] = v / (float)M;
        }
    }
    free(t); free(bits);
    return 0;
}
