// Device side of libbyzshield (gfx950): majority vote over the r copies of each file (Eq. 3 of
// the ByzShield paper), coordinate-wise median over the f winners (Sec. 2, Sec. 6.1) and the
// fused single-pass vote+median, plus the C-ABI entry points that launch them.
//
// Work decomposition shared by all streaming kernels: one thread owns V consecutive
// coordinates (V = 4, 2 or 1 dwords, chosen from the alignment of the rows) and walks over
// all files, so every global load of a wave is one contiguous 64*V*4-byte segment of one row.
// Per-file "copies differ" bits are reduced inside a wave with ballots (scalar registers),
// parked in lane j for file j, and merged across waves with one atomicOr per file and wave
// that is skipped when the bits are already set.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <new>

#include "byzshield.h"

namespace {

thread_local int g_last_hip_error = 0;

#define BYZ_HIP(call)                         \
    do {                                      \
        hipError_t e_ = (call);               \
        if (e_ != hipSuccess) {               \
            g_last_hip_error = (int)e_;       \
            return BYZ_EDEVICE;               \
        }                                     \
    } while (0)

// Optional timing of the streaming kernel: event pairs recorded around it by byz_aggregate.
struct ProfileState {
    int capacity = 0;
    int count = 0;
    hipEvent_t *start = nullptr;
    hipEvent_t *stop = nullptr;
};
thread_local ProfileState g_prof;

constexpr int kBlock = 256;
constexpr int kRowStride = 8;  // slots per file in the permuted row table (>= BYZ_MAX_R)

// ----------------------------------------------------------------------------- helpers

template <int V> struct VecT;
template <> struct VecT<1> { typedef uint32_t type; };
template <> struct VecT<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct VecT<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

template <int V>
__device__ __forceinline__ void load_vec(const uint32_t *p, uint32_t (&x)[V]) {
    if constexpr (V == 1) {
        x[0] = *p;
    } else {
        typename VecT<V>::type t = *reinterpret_cast<const typename VecT<V>::type *>(p);
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = t[v];
    }
}

template <int V>
__device__ __forceinline__ void store_vec(uint32_t *p, const uint32_t (&x)[V]) {
    if constexpr (V == 1) {
        *p = x[0];
    } else {
        typename VecT<V>::type t;
#pragma unroll
        for (int v = 0; v < V; ++v) t[v] = x[v];
        *reinterpret_cast<typename VecT<V>::type *>(p) = t;
    }
}

// OR over the V words of (a xor b): nonzero iff the two copies differ somewhere in the chunk
template <int V>
__device__ __forceinline__ uint32_t differ(const uint32_t (&a)[V], const uint32_t (&b)[V]) {
    uint32_t acc = 0;
#pragma unroll
    for (int v = 0; v < V; ++v) acc |= a[v] ^ b[v];
    return acc;
}

// 1 iff any lane of the wave has a nonzero x (wave-uniform result)
__device__ __forceinline__ uint32_t wave_any(uint32_t x) {
    return __builtin_amdgcn_ballot_w64(x != 0) != 0 ? 1u : 0u;
}

// Total order on fp32 bit patterns as unsigned keys:
//   -NaN < -inf < ... < -0 < +0 < ... < +inf < +NaN
__device__ __forceinline__ uint32_t to_key(uint32_t u) {
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ uint32_t from_key(uint32_t k) {
    return k ^ ((uint32_t)((int32_t)(~k) >> 31) | 0x80000000u);
}

// Bit of pair (a, b), a < b, in lexicographic numbering (0,1),(0,2),..,(1,2),..
__device__ __host__ __forceinline__ int pair_bit(int r, int a, int b) {
    return a * r - a * (a + 1) / 2 + (b - a - 1);
}

__device__ __forceinline__ bool copies_equal(uint32_t neq, int r, int a, int b) {
    if (a == b) return true;
    const int lo = a < b ? a : b, hi = a < b ? b : a;
    return ((neq >> pair_bit(r, lo, hi)) & 1u) == 0;
}

// Eq. 3 with the implementation note of Sec. 2: the copy that appears most often; among
// equally frequent values the one held by the lowest replica index.
__device__ __forceinline__ int decide_winner(uint32_t neq, int r) {
    int best = -1, arg = 0;
    for (int a = 0; a < r; ++a) {
        int cnt = 0;
        for (int b = 0; b < r; ++b) cnt += copies_equal(neq, r, a, b) ? 1 : 0;
        if (cnt > best) { best = cnt; arg = a; }
    }
    return arg;
}

// Merge a wave's per-file bits (lane j = file j) into global words, skipping the atomic when
// nothing new would be set.  A stale read only costs a redundant atomic.
__device__ __forceinline__ void merge_flags(uint32_t *words, int f, int lane, uint32_t flags) {
    if (lane < f && flags != 0) {
        const uint32_t cur = __atomic_load_n(&words[lane], __ATOMIC_RELAXED);
        if ((cur & flags) != flags) atomicOr(&words[lane], flags);
    }
}

// ------------------------------------------------------------------- selection networks

#define BYZ_CE(i, j)                                   \
    {                                                  \
        const uint32_t a_ = k[i], b_ = k[j];           \
        k[i] = a_ < b_ ? a_ : b_;                      \
        k[j] = a_ < b_ ? b_ : a_;                      \
    }
#define BYZ_CE_LO(i, j) { k[i] = k[i] < k[j] ? k[i] : k[j]; }
#define BYZ_CE_HI(i, j) { k[j] = k[i] < k[j] ? k[j] : k[i]; }
#define BYZ_MEDIAN_WIRE(w) result = k[w];

template <int F> struct SelNet;
template <> struct SelNet<1> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[1]) { return k[0]; }
};
template <> struct SelNet<3> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[3]) {
        uint32_t result;
#include "generated/selnet_3.inc"
        return result;
    }
};
template <> struct SelNet<5> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[5]) {
        uint32_t result;
#include "generated/selnet_5.inc"
        return result;
    }
};
template <> struct SelNet<7> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[7]) {
        uint32_t result;
#include "generated/selnet_7.inc"
        return result;
    }
};
template <> struct SelNet<9> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[9]) {
        uint32_t result;
#include "generated/selnet_9.inc"
        return result;
    }
};
template <> struct SelNet<25> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[25]) {
        uint32_t result;
#include "generated/selnet_25.inc"
        return result;
    }
};
template <> struct SelNet<49> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[49]) {
        uint32_t result;
#include "generated/selnet_49.inc"
        return result;
    }
};

// --------------------------------------------------------------------- device workspace

struct AggWorkspace {
    uint32_t viol[BYZ_MAX_F];        // fused pass: assumed-equal neighbours that differ
    uint32_t pair_neq[BYZ_MAX_F];    // exact path: all pair bits
    int32_t perm_rows[BYZ_MAX_F * kRowStride];  // rows of a file, probable winner's class first
    uint32_t chain_mask[BYZ_MAX_F];  // bit k-1: permuted copies k-1 and k were equal on the sample
    int32_t prov_winner[BYZ_MAX_F];  // probable winner (original replica index)
    int32_t winner_row[BYZ_MAX_F];   // exact path result
    int32_t winner_replica[BYZ_MAX_F];
    uint32_t need_exact;             // 1 iff some assumed equality failed
    uint32_t pad[63];
};

// ------------------------------------------------------------------------------ kernels

__global__ void fill_u32_kernel(uint32_t *p, int n, uint32_t value) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

// Step a1: for every file, which pairs of copies differ anywhere in [c_begin, c_end).
// (c_end - c_begin) % V == 0 and every row start + c_begin is 4*V-byte aligned.
template <int R, int V>
__global__ __launch_bounds__(kBlock) void vote_pairs_kernel(
    const uint32_t *__restrict__ X, int64_t c_begin, int64_t c_end, int64_t ld,
    const int32_t *__restrict__ file_rows, int f, uint32_t *pair_neq,
    const uint32_t *__restrict__ enable) {
    if (enable != nullptr && *enable == 0) return;
    const int lane = threadIdx.x & 63;
    const int64_t c0 = c_begin + ((int64_t)blockIdx.x * kBlock + threadIdx.x) * V;
    const bool active = c0 < c_end;
    uint32_t flags = 0;
    for (int j = 0; j < f; ++j) {
        uint32_t x[R][V];
#pragma unroll
        for (int k = 0; k < R; ++k) {
#pragma unroll
            for (int v = 0; v < V; ++v) x[k][v] = 0;
            if (active) load_vec<V>(X + (int64_t)file_rows[j * R + k] * ld + c0, x[k]);
        }
        uint32_t wb = 0;
#pragma unroll
        for (int a = 0; a < R; ++a)
#pragma unroll
            for (int b = a + 1; b < R; ++b)
                wb |= wave_any(differ<V>(x[a], x[b])) << pair_bit(R, a, b);
        if (lane == j) flags |= wb;
    }
    merge_flags(pair_neq, f, lane, flags);
}

// Step a2: winners from the pair bits.
__global__ void vote_decide_kernel(const uint32_t *__restrict__ pair_neq,
                                   const int32_t *__restrict__ file_rows, int f, int r,
                                   int32_t *winner_replica, int32_t *winner_row,
                                   const uint32_t *__restrict__ enable) {
    if (enable != nullptr && *enable == 0) return;
    const int j = threadIdx.x;
    if (j >= f) return;
    const int a = decide_winner(pair_neq[j], r);
    if (winner_replica != nullptr) winner_replica[j] = a;
    if (winner_row != nullptr) winner_row[j] = file_rows[j * r + a];
}

// Step a3: coordinate-wise median of F rows by a register selection network.
template <int F, int V>
__global__ __launch_bounds__(kBlock) void median_kernel(
    const uint32_t *__restrict__ X, int64_t c_begin, int64_t c_end, int64_t ld,
    const int32_t *__restrict__ row_index, uint32_t *__restrict__ out,
    const uint32_t *__restrict__ enable) {
    if (enable != nullptr && *enable == 0) return;
    const int64_t c0 = c_begin + ((int64_t)blockIdx.x * kBlock + threadIdx.x) * V;
    if (c0 >= c_end) return;
    uint32_t key[V][F];
#pragma unroll
    for (int j = 0; j < F; ++j) {
        uint32_t x[V];
        load_vec<V>(X + (int64_t)row_index[j] * ld + c0, x);
#pragma unroll
        for (int v = 0; v < V; ++v) key[v][j] = to_key(x[v]);
    }
    uint32_t o[V];
#pragma unroll
    for (int v = 0; v < V; ++v) o[v] = from_key(SelNet<F>::median(key[v]));
    store_vec<V>(out + c0, o);
}

// Step a3 for any odd f <= 64 (no generated network): rank counting, one coordinate a thread.
__global__ __launch_bounds__(kBlock) void median_generic_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, uint32_t *__restrict__ out, const uint32_t *__restrict__ enable) {
    if (enable != nullptr && *enable == 0) return;
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= d) return;
    uint32_t key[BYZ_MAX_F];
    for (int j = 0; j < f; ++j) key[j] = to_key(X[(int64_t)row_index[j] * ld + c]);
    const int mid = (f - 1) / 2;
    uint32_t result = key[0];
    for (int i = 0; i < f; ++i) {
        int rank = 0;
        for (int t = 0; t < f; ++t) rank += (key[t] < key[i] || (key[t] == key[i] && t < i)) ? 1 : 0;
        if (rank == mid) result = key[i];
    }
    out[c] = from_key(result);
}

// Probe: compares the copies of every file on a sample of <= 512 coordinates (32 runs of 16
// consecutive words spread over [0, d)), derives the probable equality classes, and lays out
// the rows of each file with the probable winner first and equal-looking copies adjacent.
// Also clears the state the later kernels accumulate into.  One block of 512 threads.
template <int R>
__global__ __launch_bounds__(512) void probe_kernel(const uint32_t *__restrict__ X, int64_t d,
                                                    int64_t ld,
                                                    const int32_t *__restrict__ file_rows, int f,
                                                    AggWorkspace *ws) {
    __shared__ uint32_t s_neq[BYZ_MAX_F];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    if (tid < BYZ_MAX_F) {
        s_neq[tid] = 0;
        ws->viol[tid] = 0;
        ws->pair_neq[tid] = 0;
    }
    if (tid == 0) ws->need_exact = 0;
    __syncthreads();

    int64_t c = -1;
    if (d <= 512) {
        if (tid < d) c = tid;
    } else {
        const int64_t run = tid >> 4, off = tid & 15;
        c = run * ((d - 16) / 31) + off;
    }
    const bool active = c >= 0;
    uint32_t flags = 0;
    for (int j = 0; j < f; ++j) {
        uint32_t x[R];
#pragma unroll
        for (int k = 0; k < R; ++k)
            x[k] = active ? X[(int64_t)file_rows[j * R + k] * ld + c] : 0u;
        uint32_t wb = 0;
#pragma unroll
        for (int a = 0; a < R; ++a)
#pragma unroll
            for (int b = a + 1; b < R; ++b) wb |= wave_any(x[a] ^ x[b]) << pair_bit(R, a, b);
        if (lane == j) flags |= wb;
    }
    if (lane < f && flags != 0) atomicOr(&s_neq[lane], flags);
    __syncthreads();

    if (tid < f) {
        const int j = tid;
        const uint32_t neq = s_neq[j];
        const int w = decide_winner(neq, R);
        // label[k] = lowest replica that looked equal to k on the sample
        int label[R];
        for (int k = 0; k < R; ++k) {
            label[k] = k;
            for (int a = 0; a < k; ++a)
                if (copies_equal(neq, R, a, k)) { label[k] = a; break; }
        }
        // order: the winner's class, then the other classes by lowest member; members ascending
        int perm[R];
        int n = 0;
        for (int k = 0; k < R; ++k)
            if (label[k] == label[w]) perm[n++] = k;
        for (int c0 = 0; c0 < R; ++c0) {
            if (label[c0] != c0 || c0 == label[w]) continue;
            for (int k = 0; k < R; ++k)
                if (label[k] == c0) perm[n++] = k;
        }
        uint32_t chain = 0;
        for (int p = 0; p < R; ++p) {
            ws->perm_rows[j * kRowStride + p] = file_rows[j * R + perm[p]];
            if (p > 0 && label[perm[p]] == label[perm[p - 1]]) chain |= 1u << (p - 1);
        }
        ws->chain_mask[j] = chain;
        ws->prov_winner[j] = w;
    }
}

// Fused a1+a2+a3: streams all R*F rows once.  The probable winner of each file (slot 0 of
// its permuted row list) feeds the median network; every equality the probe assumed between
// neighbouring slots is checked over all coordinates and violations are recorded per file.
template <int F, int R, int V>
__global__ __launch_bounds__(kBlock) void fused_kernel(const uint32_t *__restrict__ X,
                                                       int64_t c_begin, int64_t c_end, int64_t ld,
                                                       const AggWorkspace *__restrict__ ws,
                                                       uint32_t *viol, uint32_t *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t c0 = c_begin + ((int64_t)blockIdx.x * kBlock + threadIdx.x) * V;
    const bool active = c0 < c_end;
    uint32_t key[V][F];
    uint32_t flags = 0;
#pragma unroll
    for (int j = 0; j < F; ++j) {
        uint32_t x[R][V];
#pragma unroll
        for (int k = 0; k < R; ++k) {
#pragma unroll
            for (int v = 0; v < V; ++v) x[k][v] = 0;
            if (active) load_vec<V>(X + (int64_t)ws->perm_rows[j * kRowStride + k] * ld + c0, x[k]);
        }
        uint32_t wb = 0;
#pragma unroll
        for (int k = 1; k < R; ++k) wb |= wave_any(differ<V>(x[k - 1], x[k])) << (k - 1);
        wb &= ws->chain_mask[j];
        if (lane == j) flags |= wb;
#pragma unroll
        for (int v = 0; v < V; ++v) key[v][j] = to_key(x[0][v]);
    }
    uint32_t o[V];
#pragma unroll
    for (int v = 0; v < V; ++v) o[v] = from_key(SelNet<F>::median(key[v]));
    if (active) store_vec<V>(out + c0, o);
    merge_flags(viol, F, lane, flags);
}

// After the fused pass: if no assumed equality failed, the probable classes are the true
// ones and the probable winners are final; otherwise request the exact path.
__global__ void fused_finalize_kernel(AggWorkspace *ws, int f, int32_t *winner_replica) {
    const int j = threadIdx.x;  // one wave
    const uint32_t v = j < f ? ws->viol[j] : 0u;
    const bool bad = __builtin_amdgcn_ballot_w64(v != 0) != 0;
    if (bad) {
        if (j == 0) ws->need_exact = 1;
    } else if (j < f && winner_replica != nullptr) {
        winner_replica[j] = ws->prov_winner[j];
    }
}

// ---------------------------------------------------------------------------- launchers

int vec_width(const void *base, int64_t ld, const void *out) {
    const uintptr_t a = (uintptr_t)base | (uintptr_t)out;
    if ((a & 15u) == 0 && (ld & 3) == 0) return 4;
    if ((a & 7u) == 0 && (ld & 1) == 0) return 2;
    return 1;
}

inline unsigned blocks_for(int64_t n_items) { return (unsigned)((n_items + kBlock - 1) / kBlock); }

constexpr int64_t kMaxCoords = (int64_t)1 << 38;  // keeps every grid below 2^31 blocks

template <int R>
int launch_vote_pairs(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f,
                      uint32_t *neq, const uint32_t *enable, hipStream_t s) {
    const int V = vec_width(X, ld, nullptr);
    const int64_t d_main = d - d % V;
    if (d_main > 0) {
        const unsigned g = blocks_for(d_main / V);
        if (V == 4)
            vote_pairs_kernel<R, 4><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, rows, f, neq, enable);
        else if (V == 2)
            vote_pairs_kernel<R, 2><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, rows, f, neq, enable);
        else
            vote_pairs_kernel<R, 1><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, rows, f, neq, enable);
        BYZ_HIP(hipGetLastError());
    }
    if (d_main < d) {
        vote_pairs_kernel<R, 1><<<1, kBlock, 0, s>>>(X, d_main, d, ld, rows, f, neq, enable);
        BYZ_HIP(hipGetLastError());
    }
    return BYZ_OK;
}

int launch_vote_pairs_r(int r, const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows,
                        int f, uint32_t *neq, const uint32_t *enable, hipStream_t s) {
    switch (r) {
        case 3: return launch_vote_pairs<3>(X, d, ld, rows, f, neq, enable, s);
        case 5: return launch_vote_pairs<5>(X, d, ld, rows, f, neq, enable, s);
        case 7: return launch_vote_pairs<7>(X, d, ld, rows, f, neq, enable, s);
        default: return BYZ_EINVAL;
    }
}

template <int F>
int launch_median_net(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index,
                      uint32_t *out, const uint32_t *enable, hipStream_t s) {
    const int V = vec_width(X, ld, out);
    const int64_t d_main = d - d % V;
    if (d_main > 0) {
        const unsigned g = blocks_for(d_main / V);
        if (V == 4)
            median_kernel<F, 4><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, row_index, out, enable);
        else if (V == 2)
            median_kernel<F, 2><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, row_index, out, enable);
        else
            median_kernel<F, 1><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, row_index, out, enable);
        BYZ_HIP(hipGetLastError());
    }
    if (d_main < d) {
        median_kernel<F, 1><<<1, kBlock, 0, s>>>(X, d_main, d, ld, row_index, out, enable);
        BYZ_HIP(hipGetLastError());
    }
    return BYZ_OK;
}

int launch_median(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                  uint32_t *out, const uint32_t *enable, hipStream_t s) {
    if (d == 0) return BYZ_OK;
    switch (f) {
        case 1: return launch_median_net<1>(X, d, ld, row_index, out, enable, s);
        case 3: return launch_median_net<3>(X, d, ld, row_index, out, enable, s);
        case 5: return launch_median_net<5>(X, d, ld, row_index, out, enable, s);
        case 7: return launch_median_net<7>(X, d, ld, row_index, out, enable, s);
        case 9: return launch_median_net<9>(X, d, ld, row_index, out, enable, s);
        case 25: return launch_median_net<25>(X, d, ld, row_index, out, enable, s);
        case 49: return launch_median_net<49>(X, d, ld, row_index, out, enable, s);
        default:
            median_generic_kernel<<<blocks_for(d), kBlock, 0, s>>>(X, d, ld, row_index, f, out,
                                                                   enable);
            BYZ_HIP(hipGetLastError());
            return BYZ_OK;
    }
}

template <int F, int R>
int launch_fused(const uint32_t *X, int64_t d, int64_t ld, AggWorkspace *ws, uint32_t *out,
                 hipStream_t s) {
    const int V = vec_width(X, ld, out);
    const int64_t d_main = d - d % V;
    if (d_main > 0) {
        const unsigned g = blocks_for(d_main / V);
        const bool timed = g_prof.count < g_prof.capacity;
        if (timed) BYZ_HIP(hipEventRecord(g_prof.start[g_prof.count], s));
        if (V == 4)
            fused_kernel<F, R, 4><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, ws, ws->viol, out);
        else if (V == 2)
            fused_kernel<F, R, 2><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, ws, ws->viol, out);
        else
            fused_kernel<F, R, 1><<<g, kBlock, 0, s>>>(X, 0, d_main, ld, ws, ws->viol, out);
        BYZ_HIP(hipGetLastError());
        if (timed) {
            BYZ_HIP(hipEventRecord(g_prof.stop[g_prof.count], s));
            ++g_prof.count;
        }
    }
    if (d_main < d) {
        fused_kernel<F, R, 1><<<1, kBlock, 0, s>>>(X, d_main, d, ld, ws, ws->viol, out);
        BYZ_HIP(hipGetLastError());
    }
    return BYZ_OK;
}

template <int R>
int launch_probe(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f,
                 AggWorkspace *ws, hipStream_t s) {
    probe_kernel<R><<<1, 512, 0, s>>>(X, d, ld, rows, f, ws);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

bool has_fused(int f, int r) {
    return (f == 9 && r == 3) || ((f == 25 || f == 49) && (r == 3 || r == 5));
}

int check_common(const void *copies, int64_t d, int64_t ld, const void *rows, int f, int r) {
    if (copies == nullptr || rows == nullptr) return BYZ_EINVAL;
    if (d < 0 || ld < d || d > kMaxCoords) return BYZ_EINVAL;
    if (f < 1 || f > BYZ_MAX_F) return BYZ_EINVAL;
    if (r < 3 || r > BYZ_MAX_R || (r % 2) == 0) return BYZ_EINVAL;
    return BYZ_OK;
}

}  // namespace

// ---------------------------------------------------------------------------- C-ABI

extern "C" int byz_last_hip_error(void) { return g_last_hip_error; }

extern "C" int byz_vote(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev,
                        int f, int r, int32_t *winner_replica, int32_t *winner_row,
                        uint32_t *pair_neq, void *stream) {
    int rc = check_common(copies, d, ld, file_rows_dev, f, r);
    if (rc != BYZ_OK) return rc;
    if (winner_replica == nullptr || winner_row == nullptr || pair_neq == nullptr)
        return BYZ_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t *X = reinterpret_cast<const uint32_t *>(copies);
    fill_u32_kernel<<<1, BYZ_MAX_F, 0, s>>>(pair_neq, f, 0u);
    BYZ_HIP(hipGetLastError());
    if (d > 0) {
        rc = launch_vote_pairs_r(r, X, d, ld, file_rows_dev, f, pair_neq, nullptr, s);
        if (rc != BYZ_OK) return rc;
    }
    vote_decide_kernel<<<1, BYZ_MAX_F, 0, s>>>(pair_neq, file_rows_dev, f, r, winner_replica,
                                               winner_row, nullptr);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

extern "C" int byz_median(const float *rows_base, int64_t d, int64_t ld,
                          const int32_t *row_index_dev, int f, float *out, void *stream) {
    if (rows_base == nullptr || row_index_dev == nullptr || (out == nullptr && d > 0))
        return BYZ_EINVAL;
    if (d < 0 || ld < d || d > kMaxCoords) return BYZ_EINVAL;
    if (f < 1 || f > BYZ_MAX_F) return BYZ_EINVAL;
    if ((f % 2) == 0) return BYZ_EUNSUPPORTED;
    return launch_median(reinterpret_cast<const uint32_t *>(rows_base), d, ld, row_index_dev, f,
                         reinterpret_cast<uint32_t *>(out), nullptr, (hipStream_t)stream);
}

extern "C" size_t byz_aggregate_workspace_bytes(int f, int r) {
    if (f < 1 || f > BYZ_MAX_F || r < 3 || r > BYZ_MAX_R || (r % 2) == 0) return 0;
    return sizeof(AggWorkspace);
}

extern "C" int byz_aggregate(const float *copies, int64_t d, int64_t ld,
                             const int32_t *file_rows_dev, int f, int r, float *out,
                             int32_t *winner_replica, void *workspace, size_t workspace_bytes,
                             void *stream) {
    int rc = check_common(copies, d, ld, file_rows_dev, f, r);
    if (rc != BYZ_OK) return rc;
    if ((out == nullptr && d > 0) || workspace == nullptr) return BYZ_EINVAL;
    if ((f % 2) == 0) return BYZ_EUNSUPPORTED;
    if (((uintptr_t)workspace & 255u) != 0) return BYZ_EINVAL;
    if (workspace_bytes < sizeof(AggWorkspace)) return BYZ_ENOMEM;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t *X = reinterpret_cast<const uint32_t *>(copies);
    uint32_t *O = reinterpret_cast<uint32_t *>(out);
    AggWorkspace *ws = reinterpret_cast<AggWorkspace *>(workspace);

    if (!has_fused(f, r) || d == 0) {
        // two-step path, unconditionally: vote (a1, a2), then median (a3) over the winners
        fill_u32_kernel<<<1, BYZ_MAX_F, 0, s>>>(ws->pair_neq, BYZ_MAX_F, 0u);
        BYZ_HIP(hipGetLastError());
        fill_u32_kernel<<<1, 1, 0, s>>>(&ws->need_exact, 1, 1u);
        BYZ_HIP(hipGetLastError());
        if (d > 0) {
            rc = launch_vote_pairs_r(r, X, d, ld, file_rows_dev, f, ws->pair_neq, nullptr, s);
            if (rc != BYZ_OK) return rc;
        }
        vote_decide_kernel<<<1, BYZ_MAX_F, 0, s>>>(ws->pair_neq, file_rows_dev, f, r,
                                                   winner_replica, ws->winner_row, nullptr);
        BYZ_HIP(hipGetLastError());
        return launch_median(X, d, ld, ws->winner_row, f, O, nullptr, s);
    }

    // probe -> fused pass -> finalize -> (only if an assumed equality failed) exact path
    rc = (r == 3) ? launch_probe<3>(X, d, ld, file_rows_dev, f, ws, s)
                  : launch_probe<5>(X, d, ld, file_rows_dev, f, ws, s);
    if (rc != BYZ_OK) return rc;
    if (f == 9) rc = launch_fused<9, 3>(X, d, ld, ws, O, s);
    else if (f == 25 && r == 3) rc = launch_fused<25, 3>(X, d, ld, ws, O, s);
    else if (f == 25 && r == 5) rc = launch_fused<25, 5>(X, d, ld, ws, O, s);
    else if (f == 49 && r == 3) rc = launch_fused<49, 3>(X, d, ld, ws, O, s);
    else rc = launch_fused<49, 5>(X, d, ld, ws, O, s);
    if (rc != BYZ_OK) return rc;
    fused_finalize_kernel<<<1, 64, 0, s>>>(ws, f, winner_replica);
    BYZ_HIP(hipGetLastError());
    rc = launch_vote_pairs_r(r, X, d, ld, file_rows_dev, f, ws->pair_neq, &ws->need_exact, s);
    if (rc != BYZ_OK) return rc;
    vote_decide_kernel<<<1, BYZ_MAX_F, 0, s>>>(ws->pair_neq, file_rows_dev, f, r, winner_replica,
                                               ws->winner_row, &ws->need_exact);
    BYZ_HIP(hipGetLastError());
    return launch_median(X, d, ld, ws->winner_row, f, O, &ws->need_exact, s);
}

extern "C" int byz_profile_enable(int max_calls) {
    for (int i = 0; i < g_prof.capacity; ++i) {
        (void)hipEventDestroy(g_prof.start[i]);
        (void)hipEventDestroy(g_prof.stop[i]);
    }
    delete[] g_prof.start;
    delete[] g_prof.stop;
    g_prof = ProfileState();
    if (max_calls < 0 || max_calls > 100000) return BYZ_EINVAL;
    if (max_calls == 0) return BYZ_OK;
    g_prof.start = new (std::nothrow) hipEvent_t[max_calls];
    g_prof.stop = new (std::nothrow) hipEvent_t[max_calls];
    if (g_prof.start == nullptr || g_prof.stop == nullptr) {
        delete[] g_prof.start;
        delete[] g_prof.stop;
        g_prof = ProfileState();
        return BYZ_ENOMEM;
    }
    for (int i = 0; i < max_calls; ++i) {
        hipError_t e = hipEventCreate(&g_prof.start[i]);
        if (e == hipSuccess) {
            e = hipEventCreate(&g_prof.stop[i]);
            if (e != hipSuccess) (void)hipEventDestroy(g_prof.start[i]);
        }
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            g_prof.capacity = i;
            (void)byz_profile_enable(0);
            return BYZ_EDEVICE;
        }
        g_prof.capacity = i + 1;
    }
    return BYZ_OK;
}

extern "C" int byz_profile_collect(float *ms_out, int capacity, int *n_out) {
    if (n_out == nullptr || capacity < 0 || (ms_out == nullptr && capacity > 0)) return BYZ_EINVAL;
    const int n = g_prof.count < capacity ? g_prof.count : capacity;
    for (int i = 0; i < n; ++i) {
        BYZ_HIP(hipEventSynchronize(g_prof.stop[i]));
        BYZ_HIP(hipEventElapsedTime(&ms_out[i], g_prof.start[i], g_prof.stop[i]));
    }
    *n_out = n;
    g_prof.count = 0;
    return BYZ_OK;
}

extern "C" int byz_aggregate_took_exact_path(const void *workspace, int *took_exact_path,
                                             void *stream) {
    if (workspace == nullptr || took_exact_path == nullptr) return BYZ_EINVAL;
    const AggWorkspace *ws = reinterpret_cast<const AggWorkspace *>(workspace);
    uint32_t v = 0;
    hipStream_t s = (hipStream_t)stream;
    BYZ_HIP(hipMemcpyAsync(&v, &ws->need_exact, sizeof(v), hipMemcpyDeviceToHost, s));
    BYZ_HIP(hipStreamSynchronize(s));
    *took_exact_path = (int)v;
    return BYZ_OK;
}
