/*
 * byzshield.h -- C-ABI of libbyzshield: the parameter-server aggregation path of
 * ByzShield (Konstantinidis & Ramamoorthy, arXiv 2010.04902) on one AMD MI355X.
 *
 * The path: K workers return R = r*f gradient vectors of d fp32 coordinates (f files,
 * each replicated on r workers by a MOLS or Ramanujan-bigraph assignment).  The
 * parameter server takes, per file, the copy that appears most often among its r copies
 * (majority vote, Eq. 3) and then the coordinate-wise median over the f winners (Sec. 2,
 * Sec. 6.1).  Host entry points build the assignment (Sec. 4) and search the worst-case
 * Byzantine set (Sec. 5.3.2); device entry points run vote, median and the fused
 * vote+median on HIP streams.
 *
 * Conventions
 *   - Every function returns BYZ_OK (0) or a negative byz_status; nothing throws, aborts
 *     or prints.  byz_strerror() names a code.
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device
 *     memory of the current device, both owned by the caller.  Inputs are never modified.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device entry
 *     points only enqueue work: no allocation, no host synchronisation.
 *   - Stacked returns `copies`: R rows of `ld` 32-bit words, row-major, ld >= d; only the
 *     first d words of a row are read.  Worker w's t-th file (ascending file index, the
 *     order in which a worker returns its l gradients in Algorithm 1) is row w*l + t.
 *     Any base alignment and any ld work; a 16-byte aligned base with ld % 4 == 0 is a few
 *     per cent faster than rows that are only dword aligned.  d <= 2^30.
 *   - Equality of two copies is equality of all d 32-bit patterns (+0 != -0; a NaN equals
 *     a NaN of the same payload).  The median orders values by the total order
 *     -NaN < -inf < ... < -0 < +0 < ... < +inf < +NaN and returns one of its inputs
 *     bit for bit; f must be odd.
 */
#ifndef BYZSHIELD_H
#define BYZSHIELD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum byz_status {
    BYZ_OK = 0,
    BYZ_EINVAL = -1,       /* null pointer, size out of range, even r, q outside [0,K], ...      */
    BYZ_EUNSUPPORTED = -2, /* valid in the paper but not built: even f, l > 255, s not prime ...     */
    BYZ_ENOMEM = -3,       /* host allocation failed, or the workspace is too small               */
    BYZ_EDEVICE = -4,      /* a HIP call failed; see byz_last_hip_error()                          */
    BYZ_EINTERNAL = -5     /* an assignment invariant did not hold (a bug)                         */
} byz_status;

typedef enum byz_scheme {
    BYZ_SCHEME_MOLS = 0,     /* Algorithm 2: a = l (prime power), b = r <= l-1; K = r*l, f = l*l      */
    BYZ_SCHEME_RAMANUJAN = 1, /* Sec. 4.2.1: a = s (prime), b = m >= 2; Case 1 (m < s) or 2 (m >= s) */
    BYZ_SCHEME_FRC = 2       /* Sec. 5.3.1 (DETOX / DRACO): a = K, b = r | K; f = K/r, l = 1           */
} byz_scheme;

#define BYZ_MAX_F 64       /* largest f of the kernels that keep a column in a per-thread array (d < 4)  */
#define BYZ_MAX_F_KRUM 128 /* largest f of Multi-Krum and Bulyan                                         */
#define BYZ_MAX_F_WIDE 256 /* largest f of byz_vote, byz_median, byz_aggregate and the search            */
#define BYZ_MAX_R 7  /* largest replication factor                                           */

/* Opaque worker-file assignment graph G (Sec. 2): host memory owned by the library. */
typedef struct byz_assignment byz_assignment;

/* ---------------------------------------------------------------- host: assignment (Sec. 4) */

/*
 * Builds the biregular worker-file graph.
 *   BYZ_SCHEME_MOLS (Sec. 4.1, Algorithm 2): file i*l+j goes, for k = 0..r-1, to worker
 *     U_{k*l+s} with s = L_{k+1}(i,j) = (k+1)*i + j in F_l.  Needs l a prime power <= 255,
 *     1 <= r <= l-1.  For l = p^k with k > 1 (the paper does not number the field's elements)
 *     integer n stands for the polynomial over F_p whose coefficients are the base-p digits
 *     of n, lowest digit = constant term, and products are taken modulo the monic irreducible
 *     polynomial of degree k with the smallest number (GF(4): x^2+x+1, GF(8): x^3+x+1,
 *     GF(9): x^2+1); for prime l this is arithmetic modulo l.
 *   BYZ_SCHEME_RAMANUJAN (Sec. 4.2.1, Eq. 6): H = B (m >= s) or B^T (m < s), B the s x m
 *     block matrix of powers P^(a*b) of the cyclic shift P.  Needs s prime, m >= 2.
 *   BYZ_SCHEME_FRC (Sec. 5.3.1, the Fractional Repetition Code the paper compares with):
 *     K/r groups of r workers, all workers of a group hold the group's one file; replica k of
 *     file j sits on worker k*(K/r) + j.  Needs r | K.
 * After building, the library checks the structure the paper proves (every worker holds l
 * files, every file sits on r workers, each parallel class holds each file once, two workers
 * share at most one file ...) and returns BYZ_EINTERNAL if any fails.
 * *out receives the graph (free with byz_free_assignment).  Errors: BYZ_EINVAL (null out,
 * a < 2 or > 255, r outside its range, unknown scheme), BYZ_EUNSUPPORTED (l not a prime power,
 * s not prime), BYZ_ENOMEM.
 */
int byz_build_assignment(int scheme, int a, int b, byz_assignment **out);

/* Releases a graph; NULL is allowed. */
void byz_free_assignment(byz_assignment *g);

/* (K, f, l, r) of Sec. 2: workers, files, files per worker, copies per file.  Any out
 * pointer may be NULL.  BYZ_EINVAL if g is NULL. */
int byz_assignment_dims(const byz_assignment *g, int *K, int *f, int *l, int *r);

/* host out[K*l]: the files of worker w, ascending, at out[w*l .. w*l+l-1]  (N(U_w)). */
int byz_assignment_worker_files(const byz_assignment *g, int32_t *out);

/* host out[f*r]: the workers of file j, ascending (= parallel-class order), at out[j*r ..]  (N(B_j)). */
int byz_assignment_file_workers(const byz_assignment *g, int32_t *out);

/* host out[f*r]: row of `copies` holding replica k of file j: w*l + t with w the k-th worker of
 * the file and t the rank of j among w's files. */
int byz_assignment_file_rows(const byz_assignment *g, int32_t *out);

/* ------------------------------------------------- host: worst-case adversary (Sec. 5.3.2) */

/*
 * Exhaustive search over all q-subsets S of the K workers for the largest number of files
 * with at least r' = (r+1)/2 copies on workers of S (c_max^(q) of Claim 1 and Tables 3-6).
 * Among maximisers the lexicographically first ascending tuple is returned.
 *   byz_workers_out   host [q], ascending (may be NULL)
 *   cmax_out          host, c_max^(q) (may be NULL)
 *   distorted_mask_out host [ceil(f/64)] words, bit j%64 of word j/64 set iff file j is
 *                     distorted by the returned set (may be NULL)
 * Errors: BYZ_EINVAL (null g, q < 0, q > K), BYZ_EUNSUPPORTED (f > BYZ_MAX_F_WIDE), BYZ_ENOMEM.
 * Cost grows as C(K, q) (about 2*10^8 subsets per second and core); searches above 2*10^7
 * subsets use up to 16 host threads.  Not interruptible.
 *
 * Above 2*10^6 subsets the search first finds the value c_max over one representative per orbit
 * of the assignment's symmetries -- translations of the file grid, which permute the workers of
 * every parallel class among themselves: a set can be moved so that it contains the first
 * worker of the lowest class it touches and, for MOLS and Ramanujan with m <= s, also the first
 * worker of the next class (about K/q resp. l times fewer subsets) -- and then walks the
 * subsets in lexicographic order only until the first one that reaches c_max.  Every symmetry
 * is checked on the graph before it is used; the result is the same as the plain search's.
 */
int byz_worst_case(const byz_assignment *g, int q, int32_t *byz_workers_out, int32_t *cmax_out,
                   uint64_t *distorted_mask_out);

/* byz_worst_case with the strategy fixed: flags = 0 chooses as described above. */
#define BYZ_SEARCH_EXHAUSTIVE 1u /* plain search over all C(K, q) subsets             */
#define BYZ_SEARCH_SYMMETRY 2u   /* symmetry-reduced search whatever the size        */
int byz_worst_case_opts(const byz_assignment *g, int q, unsigned flags, int32_t *byz_workers_out,
                        int32_t *cmax_out, uint64_t *distorted_mask_out);

/* Upper bound gamma on c_max^(q): Eq. 5 with mu_1 = 1/r (Lemma 2) put into Claim 1.
 * Returns NaN if g is NULL or q is outside [0, K]. */
double byz_gamma_bound(const byz_assignment *g, int q);

/* --------------------------------------------------------------- device: vote (Eq. 3) */

/*
 * Majority vote per file.
 *   copies        device [R][ld] fp32 (R = f*r rows are addressed through file_rows_dev)
 *   file_rows_dev device [f*r] int32, as written by byz_assignment_file_rows
 *   winner_replica device [f] int32 out: smallest replica index among the copies that
 *                 appear most often (ties between equally frequent values go to the value
 *                 held by the lowest replica index; the paper leaves ties open)
 *   winner_row    device [f] int32 out: file_rows[j][winner_replica[j]]
 *   pair_neq      device [f] uint32 out: bit p set iff the two copies of pair p differ,
 *                 pairs (a,b), a < b, numbered lexicographically (0,1),(0,2),..,(1,2),..
 * Errors: BYZ_EINVAL (null pointers, d < 0, ld < d, f outside [1,BYZ_MAX_F_WIDE], r even or
 * outside [3,7]), BYZ_EDEVICE.  Row indices are trusted (not range-checked on the device).
 * d == 0: every copy is equal (winner 0, pair_neq 0).
 */
int byz_vote(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev, int f,
             int r, int32_t *winner_replica, int32_t *winner_row, uint32_t *pair_neq,
             void *stream);

/*
 * Majority vote for honest copies that agree only up to rounding.  Sec. 2 remarks that such
 * precision differences between honest workers could be dealt with by voting over clusters of
 * nearby vectors and gives no rule; the rule here: two words are close iff their bit
 * patterns are identical or |a - b| <= atol + rtol * max(|a|, |b|), the subtraction, the
 * product and the sum each rounded to fp32 (a NaN is close only to an identical NaN); two
 * copies are close iff all d words are; the winner of a file is the copy with the most close
 * copies (itself included), the lowest replica index among equals.  Closeness is not
 * transitive: this counts neighbours, it does not partition.  atol = rtol = 0 is byz_vote
 * except that +0 and -0 count as close.
 *   pair_far      device [f] uint32 out: bit p set iff the copies of pair p are not close
 *   other arguments and errors as byz_vote; BYZ_EINVAL also for negative or NaN atol / rtol.
 * Feed winner_row to byz_median (or another aggregator) as after byz_vote.
 */
int byz_vote_tolerant(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev,
                      int f, int r, float atol, float rtol, int32_t *winner_replica,
                      int32_t *winner_row, uint32_t *pair_far, void *stream);

/* --------------------------------------------- device: coordinate-wise median (Sec. 2, 6.1) */

/*
 * out[c] = element of rank (f-1)/2 of { rows_base[row_index[j]*ld + c] : j < f }.
 *   rows_base     device [*][ld] fp32;  row_index_dev device [f] int32;  out device [d] fp32,
 *                 must not overlap the input rows (may be NULL when d == 0).
 * f odd, 1 <= f <= 255.  A register selection network does the work for every f: generated for
 * f in {3,5,7,9,15,21,25,35,49,63,65,81,121,169} (the paper's file and worker counts and MOLS
 * over F_9, F_11, F_13), any other f <= 169 on the next of those sizes with the spare wires tied
 * half to the smallest and half to the largest key; past 169 the rows are split over two
 * wavefronts that sort a half each (11.2 M coordinates: f = 27 0.23 ms, f = 63 0.44 ms,
 * f = 255 3.0 ms).  Errors: BYZ_EINVAL, BYZ_EUNSUPPORTED (even f), BYZ_EDEVICE.
 */
int byz_median(const float *rows_base, int64_t d, int64_t ld, const int32_t *row_index_dev,
               int f, float *out, void *stream);

/* ------------------------------- device: another aggregator for the winners (Sec. 1, Sec. 7) */

/*
 * Coordinate-wise trimmed mean, the robust aggregator the paper lists beside the median
 * (Sec. 1) and a candidate for "other aggregation schemes on the vote winners" (Sec. 7):
 * out[c] = mean of the f - 2b values of { rows_base[row_index[j]*ld + c] } left after
 * dropping the b smallest and the b largest (total order of byz_median, so NaNs and
 * infinities go first).  b = 0 is the plain mean.  Not pure selection; the rounding contract
 * is: fp32, kept values added one by one in ascending order starting from +0, then one IEEE
 * division by float(f - 2b).
 *   f in {9,15,21,25,35,49,63,65,81,121,169} runs a generated register sorting network, any
 *   other f <= 169 the next of those sizes with the spare wires tied to the largest key, and
 *   169 < f <= BYZ_MAX_F_WIDE two wavefronts that sort half of the rows each and merge
 *   (11.2 M coordinates: f = 25 0.19 ms, f = 81 0.80 ms, f = 255 4.0 ms).
 * Errors: BYZ_EINVAL (null pointers, sizes, b < 0 or 2b >= f), BYZ_EDEVICE.
 */
int byz_trimmed_mean(const float *rows_base, int64_t d, int64_t ld, const int32_t *row_index_dev,
                     int f, int b, float *out, void *stream);

/*
 * Multi-Krum over f vectors (the aggregator Sec. 6.1 and Sec. 7 name as an alternative to the
 * median on the vote winners; the rule itself is the published one): with c of the f vectors
 * possibly Byzantine, 2c + 3 <= f <= BYZ_MAX_F_KRUM (the lower bound is the requirement Sec. 6.1
 * quotes),
 *   score(i) = sum of the f - c - 2 smallest squared Euclidean distances from vector i to the
 *              other vectors,
 *   the m vectors of lowest score are selected (equal scores: lower index first), 1 <= m <= f - c
 *   (m = 1 is Krum, m = f - c the usual Multi-Krum), and out = their coordinate-wise mean.
 * Arithmetic: the Gram matrix of the f rows is accumulated by fp32 matrix instructions over
 * 512 fixed coordinate slices and the slices are added in fp64 in a fixed order (results are
 * reproducible); distances d(i,j) = G_ii + G_jj - 2 G_ij, scores and ranking in fp64; the mean
 * is fp32, selected rows added one by one in ascending index from +0, one IEEE division by m.
 *   rows_base / row_index_dev  as byz_median (f rows gathered through the index table)
 *   out           device [d] fp32
 *   selected_out  device [f] int32 out: 1 for the selected rows, else 0
 *   scores_out    device [f] double out, may be NULL
 *   dist_out      device [f*f] double out, may be NULL
 *   workspace     device, >= byz_multi_krum_workspace_bytes(f) bytes, 256-byte aligned
 * Errors: BYZ_EINVAL (null pointers, f < 2c + 3, f > BYZ_MAX_F_KRUM, m outside [1, f - c],
 * sizes), BYZ_ENOMEM (workspace too small), BYZ_EDEVICE.
 */
size_t byz_multi_krum_workspace_bytes(int f);
int byz_multi_krum(const float *rows_base, int64_t d, int64_t ld, const int32_t *row_index_dev,
                   int f, int c, int m, float *out, int32_t *selected_out, double *scores_out,
                   double *dist_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Bulyan over f vectors (named with Multi-Krum in Sec. 6.1 and Sec. 7 as an aggregator for the
 * vote winners; the rule is the published one): with c of the f vectors possibly Byzantine,
 * 4c + 3 <= f <= BYZ_MAX_F_KRUM (the lower bound is the requirement Sec. 6.1 quotes),
 *   phase 1: theta = f - 2c vectors are chosen by applying Krum again and again to the vectors
 *            not yet chosen: with n' vectors left, score(i) = sum of the n' - c - 2 smallest
 *            squared distances from i to the other vectors left (no terms when n' - c - 2 <= 0,
 *            as in the last rounds); lowest score wins, lowest index among equal scores;
 *   phase 2: out[t] = mean of the beta = theta - 2c chosen values of coordinate t closest to
 *            their median: in the total order of byz_median, starting from the middle value
 *            the window grows one neighbour at a time, the lower one when
 *            (median - lower) <= (upper - median), both differences in fp32, or when no upper
 *            neighbour is left.
 * Arithmetic: distances as in byz_multi_krum (fp32 matrix instructions, fp64 reduction in a
 * fixed order), scores in fp64 added in ascending order; the mean is fp32, window values added
 * one by one in ascending order from +0, one IEEE division by float(beta).  Inputs with
 * non-finite values give NaN distances, for which phase 1 is not specified.
 *   selected_out  device [f] int32 out: 1 for the theta chosen rows, else 0
 *   order_out     device [theta] int32 out, may be NULL: indices (into row_index_dev) in the
 *                 order chosen
 *   dist_out      device [f*f] double out, may be NULL
 *   workspace     device, >= byz_bulyan_workspace_bytes(f) bytes, 256-byte aligned
 * Errors: BYZ_EINVAL (null pointers, f < 4c + 3, f > BYZ_MAX_F_KRUM, sizes), BYZ_EUNSUPPORTED (even
 * f: the median of the chosen values would not be one of them), BYZ_ENOMEM (workspace too
 * small), BYZ_EDEVICE.
 */
size_t byz_bulyan_workspace_bytes(int f);
int byz_bulyan(const float *rows_base, int64_t d, int64_t ld, const int32_t *row_index_dev, int f,
               int c, float *out, int32_t *selected_out, int32_t *order_out, double *dist_out,
               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Mean around the median, the coordinate-wise aggregator Sec. 1 names beside the median (the
 * average of the values of a coordinate that lie closest to its median) and the second phase
 * of byz_bulyan, on its own: out[t] = mean of the beta values of
 * { rows_base[row_index[j]*ld + t] : j < f } closest to their median, window and arithmetic
 * exactly as in phase 2 of byz_bulyan (beta = 1 is byz_median, beta = f the plain mean in
 * ascending order).  f odd, 1 <= f <= BYZ_MAX_F_KRUM, 1 <= beta <= f.
 * Errors: BYZ_EINVAL (null pointers, sizes, beta), BYZ_EUNSUPPORTED (even f), BYZ_EDEVICE.
 */
int byz_mean_around_median(const float *rows_base, int64_t d, int64_t ld,
                           const int32_t *row_index_dev, int f, int beta, float *out,
                           void *stream);

/* --------------------------------------------------- device: fused vote + median (whole path) */

/* Bytes of device scratch byz_aggregate needs for (f, r); 0 if (f, r) is invalid. */
size_t byz_aggregate_workspace_bytes(int f, int r);

/*
 * Whole path in one pass over the R*d inputs: out = median over files of the vote winners,
 * exactly the result of byz_vote followed by byz_median on winner_row.
 *   out            device [d] fp32
 *   winner_replica device [f] int32 out, may be NULL
 *   workspace      device, >= byz_aggregate_workspace_bytes(f, r) bytes, 256-byte aligned,
 *                  contents irrelevant on entry; calls sharing a workspace must not overlap.
 * The streaming pass compares every pair of copies of every file over all d coordinates -- the
 * whole of Eq. 3's comparison, so the true winners are known when the pass ends -- and, as it
 * goes, every wavefront feeds the median network from the first copy of the class of copies
 * that is largest on the 64..256 coordinates it has just compared.  A class that
 * holds a strict majority of a file's copies over all of d lies inside the largest class on
 * every such stretch, so for a file with a majority the values fed are the winner's
 * everywhere, whichever copies were tampered with and where: the output stands, one pass,
 * 4(rf+1) bytes per coordinate.  Only a file without a majority (copies that agree on most
 * coordinates and are told apart by a few words, so that Eq. 3's tie rule picks a winner that
 * most stretches saw outnumbered) can make the pass feed a loser's values; the decision behind
 * the pass sees that, and the median is redone from the true winners, 4(f+1) more bytes; the
 * copies are never compared a second time.  Workers that do this give up the vote in those
 * files.  The result is the same either way; byz_aggregate_path tells which it was.
 * The single pass is compiled for (f, r) = (9,3), (15,3), (21,3), (25,3), (25,5), (35,5),
 * (49,3), (49,5), (49,7), (63,7), (65,5), (81,3), (121,3), (169,3)
 * (byz_aggregate_has_single_pass; with and without BYZ_AGG_TRIM); for
 * every other valid (f, r), and for d < 4, the call runs byz_vote's kernels and then
 * byz_median's (or byz_trimmed_mean's), reading the winners a second time.
 * Errors: as byz_vote / byz_median, plus BYZ_ENOMEM (workspace too small).
 */
int byz_aggregate(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev,
                  int f, int r, float *out, int32_t *winner_replica, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * byz_aggregate with options.  flags = 0 is byz_aggregate.
 *   BYZ_AGG_EARLY_MAJORITY  r' = (r+1)/2 copies that are identical on all d coordinates are the
 *     majority whatever the other r - r' copies hold (Sec. 2: a file is distorted only if at
 *     least r' of its copies are).  A probe compares the copies on a sample of coordinates, and
 *     for every file whose probable winner's class has at least r' members only r' copies of
 *     that class are read and compared.  Same output as flags = 0 for every input; HBM traffic
 *     drops from 4(rf+1) towards 4(r'f+1) bytes per coordinate.  If the r' copies read of some
 *     file turn out to differ (off the probe's sample), nothing is known about the copies that
 *     were skipped: all copies of those files are then compared (BYZ_PATH_REVOTED; 4rd more
 *     bytes per such file) and, unless what the pass fed there was the winner's all along, the
 *     median is redone.  Every Byzantine worker can do that to the l files it holds, so in the
 *     worst case the mode costs more than flags = 0; it suits settings where timing is not
 *     attacked.  Ignored where the single pass does not run.
 * Errors: as byz_aggregate; BYZ_EINVAL for unknown flag bits.
 */
#define BYZ_AGG_EARLY_MAJORITY 1u
/*   BYZ_AGG_TRIM(b)  aggregate the winners by the trimmed mean of byz_trimmed_mean (b values
 *     dropped at each end, 0 <= 2b < f, b <= 255) instead of the median, in the same single
 *     pass; result = byz_vote followed by byz_trimmed_mean on winner_row, to its rounding
 *     contract.  May be combined with BYZ_AGG_EARLY_MAJORITY. */
#define BYZ_AGG_TRIMMED_MEAN 2u
#define BYZ_AGG_TRIM(b) (BYZ_AGG_TRIMMED_MEAN | ((unsigned)(b) << 8))
/*   BYZ_AGG_PROBE_SHIFT(s)  with BYZ_AGG_EARLY_MAJORITY only (ignored otherwise): moves the
 *     <= 256 coordinates on which that mode's probe compares the copies of a file to decide
 *     which r' of them to read (16 runs of 16 words, evenly spaced from a start that s,
 *     0..65535, picks).  The output never depends on it.  It is no defence: a worker that
 *     changes a single word of its vector misses any sample of 256 coordinates with
 *     probability 1 - 256/d wherever the sample lies. */
#define BYZ_AGG_PROBE_SHIFT(s) (((unsigned)(s) & 0xFFFFu) << 16)
int byz_aggregate_opts(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev,
                       int f, int r, float *out, int32_t *winner_replica, void *workspace,
                       size_t workspace_bytes, unsigned flags, void *stream);

/*
 * byz_aggregate_opts for callers that cannot allocate device memory and so have no workspace
 * to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and errors, minus the workspace: the scratch is a fixed
 * 24 KiB array in the library's device image (every GPU the library runs on holds its own copy
 * until the process ends), large enough for every (f, r) the library accepts, i.e. f <=
 * BYZ_MAX_F_WIDE and r <= BYZ_MAX_R; anything beyond that is refused with BYZ_ENOMEM.  The call
 * allocates nothing and frees nothing; on its first use on a device it looks the array's
 * address up (BYZ_EDEVICE if that fails, BYZ_EUNSUPPORTED for a device ordinal above 63), so
 * make that first call outside a graph capture; every later call only enqueues kernels.
 * All calls on one GPU share that array, which keeps whatever the last call left in it (each
 * call clears what it needs): calls that overlap in time on one GPU -- different streams,
 * different threads -- race and give undefined results; calls on one stream are fine.
 */
int byz_aggregate_static(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev,
                         int f, int r, float *out, int32_t *winner_replica, unsigned flags,
                         void *stream);

/* 1 if byz_aggregate runs (f, r) as the single pass described above, 0 if it runs byz_vote's and
 * byz_median's kernels one after the other (shapes without a compiled single-pass kernel, or
 * invalid (f, r)). */
int byz_aggregate_has_single_pass(int f, int r);

/*
 * What the last byz_aggregate / byz_aggregate_opts call on this workspace did, once its work on
 * `stream` has completed: copies a byz_path value from the workspace (device) into *path
 * (host).  Synchronises the stream.  Diagnostic only.
 */
typedef enum byz_path {
    BYZ_PATH_SINGLE_PASS = 0,   /* the single pass's output stood                                 */
    BYZ_PATH_MEDIAN_REDONE = 1, /* somewhere the pass fed the median a value that was not the
                                   file's winner's (a file without a majority): the median was
                                   redone from the true winners (bit 0)                          */
    BYZ_PATH_REVOTED = 2,       /* early-majority mode only: the r' copies read of some files
                                   differed and all copies of those files were compared (bit 1;
                                   with bit 0 if the median was redone as well: 3)               */
    BYZ_PATH_TWO_STEP = 4       /* no single pass for this (f, r) or d < 4: byz_vote's and
                                   byz_median's kernels one after the other                      */
} byz_path;
int byz_aggregate_path(const void *workspace, int *path, void *stream);

/* ------------------------------------------------------------------------------ misc */

const char *byz_strerror(int code);

/* hipError_t of the last failing HIP call on this thread (0 if none), for BYZ_EDEVICE. */
int byz_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BYZSHIELD_H */
