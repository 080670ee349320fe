// Shared between the translation units of libbyzshield (not part of the C-ABI).
#ifndef BYZ_INTERNAL_H
#define BYZ_INTERNAL_H

// Records the hipError_t that byz_last_hip_error() reports for the calling thread.
void byz_internal_set_hip_error(int code);

// Second phase of Bulyan (kernels.hip): out[c] = mean of the beta values closest to the median
// among the rows selected_rows_dev[0..theta-1].  Returns a byz_status.
int byz_internal_launch_bulyan_mean(const float *rows_base, long long d, long long ld,
                                    const int *selected_rows_dev, int f, int theta, int beta,
                                    float *out, void *stream);
// The same on the 81- and the 121-wire network (kernels.hip, build parts 12 and 13), d >= 4.
int byz_internal_launch_bulyan_mean_81(const void *X, long long d, long long ld,
                                       const int *selected_rows, int theta, int beta, void *out,
                                       void *stream);
int byz_internal_launch_bulyan_mean_121(const void *X, long long d, long long ld,
                                        const int *selected_rows, int theta, int beta, void *out,
                                        void *stream);

// Probe + single-pass kernel for the (f, r) of group n (kernels.hip, part n); the arguments are
// byz_aggregate_opts' after validation, ws its workspace; probe_opts: bit 0 early-majority mode,
// bits 16..31 the shift of the probe's sample.  Returns a byz_status.
#define BYZ_DECLARE_SINGLE_PASS(n)                                                              \
    int byz_internal_launch_single_pass_##n(int f, int r, const void *X, long long d,           \
                                            long long ld, const int *rows, void *ws, void *out, \
                                            int probe_opts, int trim_b, void *stream)
BYZ_DECLARE_SINGLE_PASS(1);
BYZ_DECLARE_SINGLE_PASS(2);
BYZ_DECLARE_SINGLE_PASS(3);
BYZ_DECLARE_SINGLE_PASS(4);
BYZ_DECLARE_SINGLE_PASS(5);
BYZ_DECLARE_SINGLE_PASS(6);
BYZ_DECLARE_SINGLE_PASS(7);
BYZ_DECLARE_SINGLE_PASS(8);  // (169, 3) with the trimmed mean only

// Coordinate-wise median / trimmed mean of the rows row_index[0..f-1] (kernels.hip, parts 5 and
// 6): picks the network kernel for f; gate != NULL makes the kernels return at once unless one
// of gate[0..gate_n-1] is nonzero.  Device pointers.  Returns a byz_status.
int byz_internal_launch_median(const void *X, long long d, long long ld, const int *row_index,
                               int f, void *out, const void *gate, int gate_n, void *stream);
int byz_internal_launch_trimmed_mean(const void *X, long long d, long long ld,
                                     const int *row_index, int f, int b, void *out,
                                     const void *gate, int gate_n, void *stream);

// Trimmed mean of 49 < f <= 63 and 63 < f <= 65 rows on the 63- and 65-wire sorting networks
// (kernels.hip, build parts 14 and 15).
int byz_internal_launch_trimmed_mean_63(const void *X, long long d, long long ld,
                                        const int *row_index, int f, int b, void *out,
                                        const void *gate, int gate_n, void *stream);
int byz_internal_launch_trimmed_mean_65(const void *X, long long d, long long ld,
                                        const int *row_index, int f, int b, void *out,
                                        const void *gate, int gate_n, void *stream);

// Median / trimmed mean on the 169-wire network, exactly 169 rows or fewer with spare wires
// (kernels.hip, build parts 8..11).
int byz_internal_launch_trimmed_mean_169(const void *X, long long d, long long ld,
                                         const int *row_index, int f, int b, void *out,
                                         const void *gate, int gate_n, void *stream);
int byz_internal_launch_trimmed_mean_169_padded(const void *X, long long d, long long ld,
                                                const int *row_index, int f, int b, void *out,
                                                const void *gate, int gate_n, void *stream);
int byz_internal_launch_median_169(const void *X, long long d, long long ld, const int *row_index,
                                   int f, void *out, const void *gate, int gate_n, void *stream);
int byz_internal_launch_median_169_padded(const void *X, long long d, long long ld,
                                          const int *row_index, int f, void *out, const void *gate,
                                          int gate_n, void *stream);

// ... and past 169 rows, with the rows split over two waves that sort a half each: median
// 169 < f <= 255, trimmed mean 169 < f <= 256 (build parts 16 and 17).
int byz_internal_launch_median_255_padded(const void *X, long long d, long long ld,
                                          const int *row_index, int f, void *out, const void *gate,
                                          int gate_n, void *stream);
int byz_internal_launch_trimmed_mean_256_padded(const void *X, long long d, long long ld,
                                                const int *row_index, int f, int b, void *out,
                                                const void *gate, int gate_n, void *stream);

// Records the event before (which = 0) or after (1) the dominant kernel of an aggregation, if
// byz_profile_enable has armed any.  Returns a byz_status.
int byz_internal_profile_mark(int which, void *stream);

#endif
