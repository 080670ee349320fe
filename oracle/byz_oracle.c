/*
 * CPU oracle for the ByzShield aggregation path (arXiv 2010.04902), plain C.
 *
 * TEST INFRASTRUCTURE ONLY.  Same definitions as byz_oracle.py, written so
 * that full-size inputs finish in seconds: nothing here is blocked, fused or
 * reordered beyond "loop over files" and "loop over coordinates".  It shares
 * no code with the HIP path or its host library.
 *
 *   oracle_vote    Eq. 3 + the implementation note of Sec. 2: exact-match
 *                  counting of whole d-vectors, most frequent copy wins,
 *                  lowest replica index on ties (paper silent on ties).
 *   oracle_vote_tolerant  the same vote with "close" instead of "identical" copies (fp32 test).
 *   oracle_median  Sec. 2 / Sec. 6.1: coordinate-wise median of f vectors
 *                  (f odd): sort the f values of a coordinate, take the middle.
 *                  Order: total order on bit patterns (-NaN < -inf < .. < -0 <
 *                  +0 < .. < +inf < +NaN); the paper is silent on +-0 / NaN.
 *   oracle_trimmed_mean  coordinate-wise trimmed mean in fp64 (Sec. 1's other robust
 *                  aggregator): sort, drop b at each end, mean of the rest.
 *   oracle_bulyan  Bulyan on f vectors (repeated Krum, then mean around the median), fp64.
 *   oracle_worst_case  Sec. 5.3.2: exhaustive search over all q-subsets.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (see build_oracle.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* pair p <-> (a, b), a < b, lexicographic: (0,1),(0,2),..,(1,2),.. */
static int pair_bit(int r, int a, int b) {
    int p = 0;
    for (int x = 0; x < r; ++x)
        for (int y = x + 1; y < r; ++y) {
            if (x == a && y == b) return p;
            ++p;
        }
    return -1;
}

/* Eq. 3 for one file j: the files are independent of each other. */
static void vote_one_file(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int j, int r,
                          int32_t *winner_replica, int32_t *winner_row, uint32_t *pair_neq) {
    int eq[8][8];
    for (int a = 0; a < r; ++a)
        for (int b = 0; b < r; ++b) {
            const uint32_t *pa = X + (int64_t)rows[j * r + a] * ld;
            const uint32_t *pb = X + (int64_t)rows[j * r + b] * ld;
            eq[a][b] = (memcmp(pa, pb, (size_t)d * 4) == 0);
        }
    int best = -1, a_star = 0;
    for (int a = 0; a < r; ++a) {
        int count = 0;
        for (int b = 0; b < r; ++b) count += eq[a][b];
        if (count > best) { best = count; a_star = a; }
    }
    winner_replica[j] = a_star;
    winner_row[j] = rows[j * r + a_star];
    uint32_t bits = 0;
    for (int a = 0; a < r; ++a)
        for (int b = a + 1; b < r; ++b)
            if (!eq[a][b]) bits |= 1u << pair_bit(r, a, b);
    pair_neq[j] = bits;
}

int oracle_vote(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f, int r,
                int32_t *winner_replica, int32_t *winner_row, uint32_t *pair_neq) {
    if (r < 1 || r > 7 || f < 1) return -1;
    for (int j = 0; j < f; ++j)
        vote_one_file(X, d, ld, rows, j, r, winner_replica, winner_row, pair_neq);
    return 0;
}

/* The same vote with the loop over files spread over `threads` host threads (each file is
 * decided by one thread exactly as above).  Returns the number of threads used, or <0. */
int oracle_vote_threads(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f, int r,
                        int32_t *winner_replica, int32_t *winner_row, uint32_t *pair_neq,
                        int threads) {
    if (r < 1 || r > 7 || f < 1) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    if (threads > f) threads = f;
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int j = 0; j < f; ++j)
        vote_one_file(X, d, ld, rows, j, r, winner_replica, winner_row, pair_neq);
    return used;
}

/*
 * Tolerant vote (Sec. 2 suggests voting over clusters of nearby vectors when honest copies
 * differ by rounding; the paper gives no rule).  Two words are close iff their bit patterns are identical or
 * |a - b| <= atol + rtol * max(|a|, |b|), every operation rounded to fp32; two copies are close
 * iff all d words are; count[a] = copies close to a (itself included); smallest a with the
 * largest count wins.  pair_far: bit p set iff pair p is not close.
 */
int oracle_vote_tolerant(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f,
                         int r, float atol, float rtol, int32_t *winner_replica,
                         int32_t *winner_row, uint32_t *pair_far) {
    if (r < 1 || r > 7 || f < 1) return -1;
    for (int j = 0; j < f; ++j) {
        int close[8][8];
        for (int a = 0; a < r; ++a)
            for (int b = a; b < r; ++b) {
                const uint32_t *pa = X + (int64_t)rows[j * r + a] * ld;
                const uint32_t *pb = X + (int64_t)rows[j * r + b] * ld;
                int ok = 1;
                for (int64_t t = 0; t < d && ok; ++t) {
                    if (pa[t] == pb[t]) continue;
                    float x, y;
                    memcpy(&x, pa + t, 4);
                    memcpy(&y, pb + t, 4);
                    const float diff = fabsf(x - y);
                    const float ax = fabsf(x), ay = fabsf(y);
                    const float big = ax > ay ? ax : ay;  /* a NaN makes diff NaN: not close either way */
                    const float prod = rtol * big;
                    const float bound = atol + prod;
                    if (!(diff <= bound)) ok = 0;
                }
                close[a][b] = close[b][a] = ok;
            }
        int best = -1, a_star = 0;
        for (int a = 0; a < r; ++a) {
            int count = 0;
            for (int b = 0; b < r; ++b) count += close[a][b];
            if (count > best) { best = count; a_star = a; }
        }
        winner_replica[j] = a_star;
        winner_row[j] = rows[j * r + a_star];
        uint32_t bits = 0;
        for (int a = 0; a < r; ++a)
            for (int b = a + 1; b < r; ++b)
                if (!close[a][b]) bits |= 1u << pair_bit(r, a, b);
        pair_far[j] = bits;
    }
    return 0;
}

static uint32_t order_key(uint32_t u) {
    return (u >> 31) ? (u ^ 0xFFFFFFFFu) : (u ^ 0x80000000u);
}

static uint32_t key_to_bits(uint32_t k) {
    /* inverse of order_key: keys of negative-sign patterns have the top bit clear */
    return (k >> 31) ? (k ^ 0x80000000u) : (k ^ 0xFFFFFFFFu);
}

/* returns the number of threads used, or <0 on error */
int oracle_median(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                  uint32_t *out, int threads) {
    if (f < 1 || f > 1024 || (f % 2) == 0) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t c = 0; c < d; ++c) {
        uint32_t key[1024];
        for (int j = 0; j < f; ++j) key[j] = order_key(X[(int64_t)row_index[j] * ld + c]);
        /* insertion sort, ascending */
        for (int i = 1; i < f; ++i) {
            uint32_t x = key[i];
            int t = i - 1;
            while (t >= 0 && key[t] > x) { key[t + 1] = key[t]; --t; }
            key[t + 1] = x;
        }
        out[c] = key_to_bits(key[(f - 1) / 2]);
    }
    return used;
}

/*
 * Coordinate-wise trimmed mean: sort the f values of a coordinate (same total order), drop
 * the b smallest and the b largest, fp64 mean of the rest summed in ascending order.
 * Returns the number of threads used, or <0 on error.
 */
int oracle_trimmed_mean(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                        int b, double *out, int threads) {
    if (f < 1 || f > 1024 || b < 0 || 2 * b >= f) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t c = 0; c < d; ++c) {
        uint32_t key[1024];
        for (int j = 0; j < f; ++j) key[j] = order_key(X[(int64_t)row_index[j] * ld + c]);
        for (int i = 1; i < f; ++i) {
            uint32_t x = key[i];
            int t = i - 1;
            while (t >= 0 && key[t] > x) { key[t + 1] = key[t]; --t; }
            key[t + 1] = x;
        }
        double acc = 0.0;
        for (int i = b; i < f - b; ++i) {
            uint32_t bits = key_to_bits(key[i]);
            float v;
            memcpy(&v, &bits, 4);
            acc += (double)v;
        }
        out[c] = acc / (double)(f - 2 * b);
    }
    return used;
}

/*
 * Second phase of Bulyan on its own: for every coordinate the mean (fp64) of the beta values
 * closest to the median among the theta rows row_index[chosen[0..theta-1]] (theta odd).
 * The window rule is the one described at oracle_bulyan.  Returns threads used, <0 on error.
 */
int oracle_mean_around_median(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index,
                              const int32_t *chosen, int theta, int beta, double *out,
                              int threads) {
    if (theta < 1 || theta > 1024 || (theta % 2) == 0 || beta < 1 || beta > theta) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#endif
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t t = 0; t < d; ++t) {
        uint32_t key[1024];
        float s[1024];
        for (int j = 0; j < theta; ++j)
            key[j] = order_key(X[(int64_t)row_index[chosen[j]] * ld + t]);
        for (int i = 1; i < theta; ++i) {
            uint32_t x = key[i];
            int u = i - 1;
            while (u >= 0 && key[u] > x) { key[u + 1] = key[u]; --u; }
            key[u + 1] = x;
        }
        for (int j = 0; j < theta; ++j) {
            uint32_t bits = key_to_bits(key[j]);
            memcpy(&s[j], &bits, 4);
        }
        const int h = (theta - 1) / 2;
        const float med = s[h];
        int lo = h, hi = h;
        for (int step = 1; step < beta; ++step) {
            const int can_l = lo > 0, can_r = hi < theta - 1;
            int take_left = 0;
            if (can_l && !can_r) {
                take_left = 1;
            } else if (can_l && can_r) {
                const float dl = med - s[lo - 1];
                const float dr = s[hi + 1] - med;
                take_left = dl <= dr;
            }
            if (take_left) --lo; else ++hi;
        }
        double acc = 0.0;
        for (int j = lo; j <= hi; ++j) acc += (double)s[j];
        out[t] = acc / (double)beta;
    }
    return used;
}

/*
 * Bulyan (El Mhamdi, Guerraoui, Rouault 2018), which Sec. 7 names as an aggregator that can
 * replace the median on the vote winners: theta = f - 2c vectors are chosen by applying Krum
 * again and again to the vectors not yet chosen, then every coordinate is the mean of the
 * beta = theta - 2c chosen values closest to their median.
 *   Krum round on the remaining set (size n'): score(i) = sum, in ascending order, of the
 *   n' - c - 2 smallest squared distances to the other remaining vectors (no terms if that is
 *   <= 0); lowest score wins, lowest index on ties.
 *   Closest to the median: the chosen values in the total order of oracle_median; the window
 *   starts at the middle one and grows by one neighbour at a time, the lower one when
 *   (float)(median - lower) <= (float)(upper - median) or no upper one is left.
 * Squared distances and the mean in fp64.  chosen_out[theta]: indices into row_index in the
 * order chosen.  dist_out[f*f] may be NULL.  Returns threads used, <0 on error.
 */
int oracle_bulyan(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f, int c,
                  double *out, int32_t *chosen_out, double *dist_out, int threads) {
    if (f < 1 || f > 1024 || c < 0 || f < 4 * c + 3) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#endif
    const int theta = f - 2 * c, beta = theta - 2 * c;
    double *dist = (double *)malloc(sizeof(double) * (size_t)f * f);
    if (!dist) return -2;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic) num_threads(threads)
#endif
    for (int p = 0; p < f * f; ++p) {
        const int i = p / f, j = p % f;
        const uint32_t *a = X + (int64_t)row_index[i] * ld, *b = X + (int64_t)row_index[j] * ld;
        double acc = 0.0;
        for (int64_t t = 0; t < d; ++t) {
            float x, y;
            memcpy(&x, a + t, 4);
            memcpy(&y, b + t, 4);
            const double diff = (double)x - (double)y;
            acc += diff * diff;
        }
        dist[p] = acc;
    }
    if (dist_out) memcpy(dist_out, dist, sizeof(double) * (size_t)f * f);
    /* phase 1: repeated Krum */
    int remaining[1024];
    double others[1024];
    for (int i = 0; i < f; ++i) remaining[i] = 1;
    for (int round = 0; round < theta; ++round) {
        int k = (f - round) - c - 2;
        if (k < 0) k = 0;
        int best = -1;
        double best_score = 0.0;
        for (int i = 0; i < f; ++i) {
            if (!remaining[i]) continue;
            int n = 0;
            for (int j = 0; j < f; ++j) {
                if (!remaining[j] || j == i) continue;
                double v = dist[i * f + j];
                int t = n - 1;
                while (t >= 0 && others[t] > v) { others[t + 1] = others[t]; --t; }
                others[t + 1] = v;
                ++n;
            }
            double score = 0.0;
            for (int t = 0; t < k; ++t) score += others[t];
            if (best < 0 || score < best_score) { best = i; best_score = score; }
        }
        chosen_out[round] = best;
        remaining[best] = 0;
    }
    free(dist);
    {
        int rc2 = oracle_mean_around_median(X, d, ld, row_index, chosen_out, theta, beta, out, threads);
        if (rc2 < 0) return rc2;
    }
    return used;
}

/* vote then median over the winners; returns threads used by the median, <0 on error */
int oracle_aggregate(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f, int r,
                     uint32_t *out, int32_t *winner_replica, int threads) {
    int32_t *wrow = (int32_t *)malloc(sizeof(int32_t) * (size_t)f);
    uint32_t *neq = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)f);
    if (!wrow || !neq) { free(wrow); free(neq); return -2; }
    int rc = oracle_vote_threads(X, d, ld, rows, f, r, winner_replica, wrow, neq, threads);
    if (rc >= 0) rc = oracle_median(X, d, ld, wrow, f, out, threads);
    free(wrow);
    free(neq);
    return rc;
}

/*
 * H: K x f, row-major 0/1 bytes.  Visits the q-subsets in lexicographic order
 * and keeps the first one with the largest number of files that have at least
 * r' = (r+1)/2 copies inside the subset.
 */
int oracle_worst_case(const uint8_t *H, int K, int f, int r, int q, int32_t *S_out,
                      int32_t *cmax_out) {
    if (q < 0 || q > K || K > 64 || f > 4096) return -1;
    int rp = (r + 1) / 2;
    int S[64];
    for (int i = 0; i < q; ++i) S[i] = i;
    int best = -1;
    for (;;) {
        int c = 0;
        for (int j = 0; j < f; ++j) {
            int cnt = 0;
            for (int i = 0; i < q; ++i) cnt += H[S[i] * f + j];
            if (cnt >= rp) ++c;
        }
        if (c > best) {
            best = c;
            for (int i = 0; i < q; ++i) S_out[i] = S[i];
        }
        /* next combination in lexicographic order */
        int i = q - 1;
        while (i >= 0 && S[i] == K - q + i) --i;
        if (i < 0) break;
        ++S[i];
        for (int t = i + 1; t < q; ++t) S[t] = S[t - 1] + 1;
    }
    *cmax_out = best;
    return 0;
}
