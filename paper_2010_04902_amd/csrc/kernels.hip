// Device side of libbyzshield (gfx950): majority vote over the r copies of each file (Eq. 3 of
// the ByzShield paper; exact and tolerant), coordinate-wise median over the f winners (Sec. 2,
// Sec. 6.1), the fused single-pass vote+median, the trimmed mean and the second phase of
// Bulyan, plus the C-ABI entry points that launch them.
//
// Work decomposition shared by all streaming kernels: one thread owns V consecutive
// coordinates (4; 2 or 1 for the largest networks) and walks over all files, so every global
// load of a wave is one contiguous segment of one row (1 KiB with 16-byte loads; gfx950 global
// loads only need dword alignment).  Threads past the end of the grid redo the last vector, so
// loads and wave ballots sit in straight-line code; trailing words are done by a few threads
// of the last block or by letting the last vector overlap its neighbour.
// Per-file "copies differ" bits are reduced inside a wave with ballots (scalar registers),
// parked in lane j mod 64 for file j (one word per 64 files), and merged across waves with one
// atomicOr per file and wave that is skipped when the bits are already set.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <new>

#include "byz_internal.h"
#include "byzshield.h"
#include "byzshield_bench.h"

// The build compiles this file once per BYZ_PART, in parallel, because the single-pass kernels
// are large: part 0 holds every entry point, the vote and the Bulyan kernels, parts 1..4 one
// group of single-pass instantiations each (byz_internal_launch_single_pass_<n>; the fifth
// group is part 7, the sixth and seventh parts 14 and 15, which also hold the 63- and 65-wire
// trimmed-mean kernels, the eighth part 18), part 5 the median kernels, part 6 the
// trimmed-mean kernels, parts 8..11 one 169-wire network kernel each, parts 12 and 13 the 81- and
// 121-wire second phase of Bulyan, parts 16 and 17 the two-wave median and trimmed-mean kernels for f > 169.
// Without BYZ_PART the whole library is
// this one translation unit.
#ifndef BYZ_PART
#define BYZ_PART -1
#endif
#define BYZ_IN_PART(p) (BYZ_PART == -1 || BYZ_PART == (p))

namespace {

#define BYZ_HIP(call)                                \
    do {                                             \
        hipError_t e_ = (call);                      \
        if (e_ != hipSuccess) {                      \
            byz_internal_set_hip_error((int)e_);     \
            return BYZ_EDEVICE;                      \
        }                                            \
    } while (0)

#if BYZ_IN_PART(0)
thread_local int g_last_hip_error = 0;

// Optional timing of the dominant kernel: event pairs recorded around it by byz_aggregate.
struct ProfileState {
    int capacity = 0;
    int count = 0;
    hipEvent_t *start = nullptr;
    hipEvent_t *stop = nullptr;
};
thread_local ProfileState g_prof;
#endif

// Files the single-pass kernel prefetches ahead of the one it consumes, from the number of
// 16-byte loads per thread it should keep in flight.  Measured on MI355X: about 6 for f = 25
// (3-4 waves per SIMD), about 12 for f = 49 (2 waves per SIMD); more is slower.  f = 121 runs
// one word per thread (4-byte loads) and, with one slot per file, gains up to 20 files ahead;
// f = 81 (two words per thread, 253 registers) has no room for more than 5.
constexpr int prefetch_depth(int f, int slots) {
    if (f > 81) return slots == 1 ? 20 : 5;
    const int target = f >= 49 ? 12 : 6;
    const int a = (target + slots - 1) / slots - 1;
    return a < 1 ? 1 : (a > 5 ? 5 : a);
}
// f with a generated streamed network (gen_selnet.py STREAMED_SIZES): the paper's file counts
// l^2 (MOLS, Ramanujan Case 1; 81, 121, 169 for l = 9, 11, 13) and m*s (Ramanujan Case 2)
constexpr bool has_streamed_network(int f) {
    return f == 9 || f == 15 || f == 21 || f == 25 || f == 35 || f == 49 || f == 63 || f == 65 ||
           f == 81 || f == 121 || f == 169;
}
// words per thread: fewer for the large networks, whose keys fill the register file
constexpr int vec_for(int f) { return f <= 49 ? 4 : (f <= 81 ? 2 : 1); }
// ... of the median kernels: above 49 wires they are bound by min/max issue, and one word per
// thread (fewer registers, more waves per SIMD) measured 4-8 % faster than two at f = 63, 81
constexpr int vec_for_median(int f) { return f <= 49 ? 4 : 1; }
// ... of the trimmed-mean kernels: the same above 49 wires (f = 81: 5 % faster, fewer files on
// the 81-wire network: 15 %); at f = 49 the kernel runs at the vector ALU's practical limit
// whatever the width (0.43 ms for 11.2 M coordinates with four, two or one word per thread)
constexpr int vec_for_trimmed(int f) { return f <= 49 ? 4 : 1; }
// ... and of the second phase of Bulyan, where narrower threads measured slightly slower
constexpr int vec_for_sort(int f) { return vec_for(f); }
// ... and of the single pass: with five or seven copies of a file in flight two words per thread
// (more waves per SIMD, 8-byte loads) measured 1-2 % faster than four (r = 7 would not fit
// the registers with four); with three copies four words are faster
constexpr int vec_for_pass(int f, int r) { return (r >= 5 && f <= 49) ? 2 : vec_for(f); }
constexpr int kProbe = 256;  // sampled coordinates of the probe (512: 2x slower)
constexpr int kProbeSplit = 4;  // the files are dealt out to this many groups of kProbe threads
constexpr int kProbeThreads = kProbe * kProbeSplit;
constexpr int kBlock = 256;  // threads per block of the streaming kernels (128/512/1024: slower)
constexpr int kWide = BYZ_MAX_F_WIDE;  // largest f of the vote, the median (255) and the trimmed mean
static_assert(kWide <= kBlock, "one thread per file in the deciding block");
constexpr int kPinFrom = 169;  // network sizes from which the trimmed-mean kernel pins its schedule
constexpr int kRowStride = 8;  // slots per file in the permuted row table (>= BYZ_MAX_R)

// ----------------------------------------------------------------------------- helpers

template <int V> struct VecT;
template <> struct VecT<1> { typedef uint32_t type; };
// Vector types that only promise dword alignment: global memory accesses of gfx950 need no
// more, so rows whose pitch is not a multiple of four words still get 16-byte loads.
template <> struct VecT<2> {
    typedef uint32_t type __attribute__((ext_vector_type(2), aligned(4)));
};
template <> struct VecT<4> {
    typedef uint32_t type __attribute__((ext_vector_type(4), aligned(4)));
};

// Streaming load of V words (each input word is used exactly once: non-temporal hint).
template <int V>
__device__ __forceinline__ void load_vec(const uint32_t *p, uint32_t (&x)[V]) {
    typedef typename VecT<V>::type T;
    const T t = __builtin_nontemporal_load(reinterpret_cast<const T *>(p));
    if constexpr (V == 1) {
        x[0] = t;
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = t[v];
    }
}

template <int V>
__device__ __forceinline__ void store_vec(uint32_t *p, const uint32_t (&x)[V]) {
    typedef typename VecT<V>::type T;
    T t;
    if constexpr (V == 1) {
        t = x[0];
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) t[v] = x[v];
    }
    __builtin_nontemporal_store(t, reinterpret_cast<T *>(p));
}

// OR over the V words of (a xor b): nonzero iff the two copies differ somewhere in the chunk
template <int V>
__device__ __forceinline__ uint32_t differ(const uint32_t (&a)[V], const uint32_t (&b)[V]) {
    uint32_t acc = 0;
#pragma unroll
    for (int v = 0; v < V; ++v) acc |= a[v] ^ b[v];
    return acc;
}

// 1 iff the two chunks differ in any active lane of the wave (wave-uniform result).  One ballot
// per word, merged as scalars: each is a single vector compare that writes its lane mask.
template <int V>
__device__ __forceinline__ uint32_t wave_differ(const uint32_t (&a)[V], const uint32_t (&b)[V]) {
    uint64_t m = 0;
#pragma unroll
    for (int v = 0; v < V; ++v) m |= __builtin_amdgcn_ballot_w64(a[v] != b[v]);
    return m != 0 ? 1u : 0u;
}

// 1 iff any active lane of the wave has a nonzero x (wave-uniform result)
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
__device__ __host__ __forceinline__ constexpr int pair_bit(int r, int a, int b) {
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

// All pair bits that involve slot a, of n slots.
__device__ __host__ __forceinline__ constexpr uint32_t pairs_of_slot(int n, int a) {
    uint32_t m = 0;
    for (int b = 0; b < n; ++b)
        if (b != a) m |= 1u << pair_bit(n, a < b ? a : b, a < b ? b : a);
    return m;
}

// Which of a file's NS slots feeds the median network on one wave's coordinates, from the pair
// bits wb the wave found there (all wave-uniform): the first slot of the largest class of slots
// that are identical on these coordinates.  Being identical on a fixed set of coordinates is an
// equivalence, so a class that holds a strict majority of the copies over all of d is inside the
// largest class here, and the chosen slot then carries the majority's values on this wave's
// coordinates whether or not it belongs to the majority elsewhere.  differs gets bit b set iff
// slot b differs from the chosen one here.
// Packed as pick | differs << 3.
__device__ __host__ __forceinline__ constexpr uint32_t local_choice_packed(int ns, uint32_t wb) {
    int pick = 0, fewest = ns;
    for (int a = 0; a < ns; ++a) {
        int n = 0;
        for (int b = 0; b < ns; ++b)
            if (b != a) n += (int)((wb >> pair_bit(ns, a < b ? a : b, a < b ? b : a)) & 1u);
        if (n < fewest) { fewest = n; pick = a; }
    }
    uint32_t differs = 0;
    for (int b = 0; b < ns; ++b)
        if (b != pick)
            differs |= ((wb >> pair_bit(ns, pick < b ? pick : b, pick < b ? b : pick)) & 1u) << b;
    return (uint32_t)pick | differs << 3;
}
static_assert(local_choice_packed(3, 0b110u) == (0u | 0b100u << 3), "{0,1},{2}: slot 0 feeds, 2 differs");
static_assert(local_choice_packed(3, 0b011u) == (1u | 0b001u << 3), "{0},{1,2}: slot 1 feeds, 0 differs");
static_assert(local_choice_packed(3, 0b111u) == (0u | 0b110u << 3), "three singletons: slot 0 feeds");
static_assert(local_choice_packed(5, 0u) == 0u, "all alike");
// The eight cases of three slots as one constant, a byte each: pick in bits 0..1, above it what
// the wave adds to the file's word in the workspace (its pair bits, then the differs bits).
__device__ __host__ __forceinline__ constexpr uint64_t local_choice_table3() {
    uint64_t t = 0;
    for (uint32_t wb = 0; wb < 8; ++wb) {
        const uint32_t p = local_choice_packed(3, wb);
        t |= (uint64_t)((p & 3u) | (wb | (p >> 3) << 3) << 2) << (8 * wb);
    }
    return t;
}
// -> the slot that feeds; word = what the wave adds to the file's word in the workspace.
template <int NS>
__device__ __forceinline__ int local_choice(uint32_t wb, uint32_t &word) {
    if constexpr (NS == 2) {
        word = wb | wb << 2;  // two unequal slots: the first feeds, the second differs from it
        return 0;
    } else if constexpr (NS == 3) {
        constexpr uint64_t kTable = local_choice_table3();
        const uint32_t e = (uint32_t)(kTable >> (8 * wb)) & 255u;
        word = e >> 2;
        return (int)(e & 3u);
    } else {
        word = wb;
        if (wb == 0) return 0;
        int pick = 0, fewest = NS;
#pragma unroll
        for (int a = 0; a < NS; ++a) {
            const int n = __builtin_popcount(wb & pairs_of_slot(NS, a));
            if (n < fewest) { fewest = n; pick = a; }
        }
        uint32_t differs = 0;
#pragma unroll
        for (int a = 0; a < NS; ++a)
            if (pick == a) {
#pragma unroll
                for (int b = 0; b < NS; ++b)
                    if (b != a) differs |= ((wb >> pair_bit(NS, a < b ? a : b, a < b ? b : a)) & 1u) << b;
            }
        word |= differs << (NS * (NS - 1) / 2);
        return pick;
    }
}

__device__ __forceinline__ uint32_t load_shared_word(const uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wave-uniform: is any of words[0..n-1] nonzero?  Used by the gated kernels behind the single
// pass to return at once when the decision kernel did not ask for them.
__device__ __forceinline__ bool any_word_set(const uint32_t *__restrict__ words, int n) {
    const int lane = threadIdx.x & 63;
    bool any = false;
    for (int n0 = 0; n0 < n; n0 += 64) {
        const uint32_t v = n0 + lane < n ? words[n0 + lane] : 0u;
        any = any || __builtin_amdgcn_ballot_w64(v != 0) != 0;
    }
    return any;
}

// Merge a wave's per-file bits (lane j = file j) into global words, skipping the atomic when
// nothing new would be set.  A stale read only costs a redundant atomic.
__device__ __forceinline__ void merge_flags(uint32_t *words, int f, int lane, uint32_t flags) {
    if (lane < f && flags != 0) {
        const uint32_t cur = load_shared_word(&words[lane]);
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
template <> struct SelNet<15> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[15]) {
        uint32_t result;
#include "generated/selnet_15.inc"
        return result;
    }
};
template <> struct SelNet<21> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[21]) {
        uint32_t result;
#include "generated/selnet_21.inc"
        return result;
    }
};
template <> struct SelNet<35> {
    static __device__ __forceinline__ uint32_t median(uint32_t (&k)[35]) {
        uint32_t result;
#include "generated/selnet_35.inc"
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
    // single pass: bit pair_bit(NS, p, q) set iff the copies in slots p < q of the file's
    // permuted row list differ anywhere in [0, d) (NS = slots the pass read: r, or r' when every
    // file ran in early-majority mode); above them, bit NS(NS-1)/2 + p set iff some wave fed the
    // network from a slot that differed from slot p on that wave's coordinates
    uint32_t pneq[kWide];
    uint32_t pair_neq[kWide];        // two-step path and re-vote: all pair bits, replica numbering
    // byte offsets row*ld*4 of a file's rows, probable winner's class first
    uint64_t perm_off[kWide * kRowStride];
    // bits 3p..3p+2: replica in slot p; bits 24..27: slots of the file that hold a copy of their
    // own (r, or r' for a file read in early-majority mode; the other slots repeat slot 0)
    uint32_t perm[kWide];
    int32_t winner_row[kWide];       // rows of the true winners (decided after the pass)
    uint32_t revote_file[kWide];     // early-majority mode: 1 for the files whose r' copies differed
    uint32_t need_median;            // 1: some file's slot 0 was not its winner -> median redone
    uint32_t need_revote;            // 1: early-majority mode met a file whose r' copies differ
    uint32_t path;                   // byz_path of the call, for byz_aggregate_path
    uint32_t slots_per_file;         // slots of every file the single pass reads: r or r'
    uint32_t pad[60];
};
static_assert(sizeof(AggWorkspace) % 256 == 0, "whole 256-byte lines");

// ------------------------------------------------------------------------------ kernels

// Clears the accumulators of one two-step aggregation (no hipMemset: callers may capture).
__global__ void reset_workspace_kernel(AggWorkspace *ws, uint32_t path) {
    const int i = threadIdx.x;
    if (i < kWide) {
        ws->pneq[i] = 0;
        ws->pair_neq[i] = 0;
    }
    if (i == 0) {
        ws->need_median = 0;
        ws->need_revote = 0;
        ws->path = path;
    }
}

// Plain copy with the same load/store flavour as the streaming kernels (16-byte non-temporal):
// a reference of known traffic for reading hardware HBM counters.
__global__ __launch_bounds__(kBlock) void calibration_copy_kernel(const uint32_t *__restrict__ src,
                                                                  uint32_t *__restrict__ dst,
                                                                  int64_t n_vec) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_vec) return;
    uint32_t x[4];
    load_vec<4>(src + i * 4, x);
    store_vec<4>(dst + i * 4, x);
}

// The single pass's memory access pattern and nothing else: every thread reads 16 bytes of
// each of n_rows rows (non-temporal loads, six in flight), XORs them, and -- if do_store --
// writes its 16 bytes (non-temporal).  Timed with and without the store it tells what a kernel
// of this shape can reach and what the output costs.
__global__ __launch_bounds__(kBlock) void calibration_read_rows_kernel(
    const uint32_t *__restrict__ X, int64_t n_vec, int64_t ld, int n_rows,
    uint32_t *__restrict__ out, int do_store) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_vec) return;
    constexpr int kRing = 6;
    const uint32_t *p = X + i * 4;
    uint32_t st[kRing][4];
#pragma unroll
    for (int u = 0; u < kRing; ++u) load_vec<4>(p + (int64_t)(u < n_rows ? u : 0) * ld, st[u]);
    uint32_t acc[4] = {0, 0, 0, 0};
    for (int k0 = 0; k0 < n_rows; k0 += kRing) {
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
            const int k = k0 + u;  // the same for every thread
            if (k < n_rows) {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] ^= st[u][e];
                if (k + kRing < n_rows) load_vec<4>(p + (int64_t)(k + kRing) * ld, st[u]);
            }
        }
    }
    if (do_store != 0) {
        store_vec<4>(out + i * 4, acc);
    } else if (acc[0] == 0x5EEDu && acc[1] == 0xC0FFEEu && acc[2] == 0x12345u) {
        out[0] = acc[3];  // practically never: keeps the loads alive without a store
    }
}

__global__ void fill_u32_kernel(uint32_t *p, int n, uint32_t value) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

// Vote, decision: winners from the pair bits (thread j = file j).
__device__ __forceinline__ void decide_files(const uint32_t *pair_neq,
                                             const int32_t *__restrict__ file_rows, int f, int r,
                                             int32_t *winner_replica, int32_t *winner_row) {
    const int j = threadIdx.x;
    if (j >= f) return;
    const int a = decide_winner(load_shared_word(&pair_neq[j]), r);
    if (winner_replica != nullptr) winner_replica[j] = a;
    if (winner_row != nullptr) winner_row[j] = file_rows[j * r + a];
}

__global__ void vote_decide_kernel(const uint32_t *pair_neq, const int32_t *__restrict__ file_rows,
                                   int f, int r, int32_t *winner_replica, int32_t *winner_row) {
    decide_files(pair_neq, file_rows, f, r, winner_replica, winner_row);
}

// Replica held by slot p of a file's permuted row list (AggWorkspace::perm).
__device__ __forceinline__ int perm_slot(uint32_t packed, int p) { return (int)((packed >> (3 * p)) & 7u); }

// Bit of a file's word in AggWorkspace::pneq that says: on some wave's coordinates, the slot that
// fed the network there differed from slot p (ns = slots the pass numbered its bits by).
__device__ __forceinline__ uint32_t fed_differs_bit(int ns, int p) { return 1u << (ns * (ns - 1) / 2 + p); }

// The decision behind the single pass (one block, thread j = file j).  The pass compared every
// pair of the slots it read over all d coordinates, so its bits are the vote's pair bits up to
// the slot numbering: the true winner of every file follows by Eq. 3, whatever order the
// slots are in.  The pass's output stands iff, for every file, no wave fed the network from a slot
// that differed from the winner's on that wave's coordinates; otherwise need_median makes the
// gated median kernel redo the output from the true winners (the inputs are not compared again).
// A file read in early-majority mode has only r' slots of its own: if they are identical they
// are the majority (Sec. 2) and any of them is the winner; if not, nothing is known about the
// copies that were skipped and need_revote sends the call through the gated vote kernel.
__global__ void single_pass_decide_kernel(AggWorkspace *ws, const int32_t *__restrict__ file_rows,
                                          int f, int r, int32_t *winner_replica) {
    __shared__ uint32_t s_median, s_revote;
    if (threadIdx.x == 0) { s_median = 0; s_revote = 0; }
    __syncthreads();
    const int j = threadIdx.x;
    if (j < f) {
        const uint32_t pn = load_shared_word(&ws->pneq[j]);
        const uint32_t packed = ws->perm[j];
        const int own = (int)(packed >> 24);       // slots with a copy of their own
        const int ns = (int)ws->slots_per_file;    // slots the pass read and numbered its bits by
        if (own == r) {
            uint32_t neq = 0;
            for (int p = 0; p < r; ++p)
                for (int q = p + 1; q < r; ++q)
                    if ((pn >> pair_bit(ns, p, q)) & 1u) {
                        const int a = perm_slot(packed, p), b = perm_slot(packed, q);
                        neq |= 1u << pair_bit(r, a < b ? a : b, a < b ? b : a);
                    }
            const int w = decide_winner(neq, r);
            if (winner_replica != nullptr) winner_replica[j] = w;
            ws->winner_row[j] = file_rows[j * r + w];
            for (int p = 0; p < r; ++p)
                if (perm_slot(packed, p) == w && (pn & fed_differs_bit(ns, p)) != 0) s_median = 1;
        } else {
            uint32_t differ_bits = 0;
            for (int p = 0; p < own; ++p)
                for (int q = p + 1; q < own; ++q) differ_bits |= (pn >> pair_bit(ns, p, q)) & 1u;
            const int w = perm_slot(packed, 0);
            if (winner_replica != nullptr) winner_replica[j] = w;
            ws->winner_row[j] = file_rows[j * r + w];
            if (differ_bits != 0) s_revote = 1;
            ws->revote_file[j] = differ_bits;
        }
        if (own == r) ws->revote_file[j] = 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        ws->need_median = s_median;
        ws->need_revote = s_revote;
        ws->path = (s_median != 0 ? (uint32_t)BYZ_PATH_MEDIAN_REDONE : 0u) |
                   (s_revote != 0 ? (uint32_t)BYZ_PATH_REVOTED : 0u);
    }
}

// Early-majority mode only, after the gated vote kernel: if the decision above asked for a
// re-vote, the winners of the files it named come from the pair bits that kernel collected
// for them, and the median is redone unless, for each of those files, the winner's copy was
// among the slots the pass read and no wave fed the network from a slot that differed from it.
__global__ void revote_decide_kernel(AggWorkspace *ws, const int32_t *__restrict__ file_rows, int f,
                                     int r, int32_t *winner_replica) {
    if (ws->need_revote == 0) return;
    __shared__ uint32_t s_median;
    if (threadIdx.x == 0) s_median = 0;
    __syncthreads();
    const int j = threadIdx.x;
    if (j < f && ws->revote_file[j] != 0) {  // the other files keep the winners decided above
        const uint32_t neq = load_shared_word(&ws->pair_neq[j]);
        const int a = decide_winner(neq, r);
        if (winner_replica != nullptr) winner_replica[j] = a;
        ws->winner_row[j] = file_rows[j * r + a];
        const uint32_t pn = load_shared_word(&ws->pneq[j]);
        const uint32_t packed = ws->perm[j];
        const int own = (int)(packed >> 24), ns = (int)ws->slots_per_file;
        bool stands = false;
        for (int p = 0; p < own; ++p)
            if (perm_slot(packed, p) == a && (pn & fed_differs_bit(ns, p)) == 0) stands = true;
        if (!stands) s_median = 1;
    }
    __syncthreads();
    if (threadIdx.x == 0 && s_median != 0) {
        ws->need_median = 1;
        ws->path = (uint32_t)BYZ_PATH_REVOTED | (uint32_t)BYZ_PATH_MEDIAN_REDONE;
    }
}

// Vote, comparison: for every file, which pairs of copies differ anywhere in [0, d).  Threads own
// vectors of V words; the d % V trailing words go to the first threads of the last block.
// If `gate` is given, the kernel only runs when one of gate[0..gate_n-1] is nonzero; if
// `only_files` is given, only the files j with only_files[j] != 0 are read and compared.
template <int R, int V>
__global__ __launch_bounds__(kBlock) void vote_pairs_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ file_rows,
    int f, uint32_t *pair_neq, const uint32_t *__restrict__ gate, int gate_n,
    const uint32_t *__restrict__ only_files) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    const int lane = threadIdx.x & 63;
    const int64_t n_vec = d / V;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n_vec > 0) {
        // threads past the end redo the last vector: no branches around loads and ballots
        const uint32_t *base = X + (gt < n_vec ? gt : n_vec - 1) * V;
        // files in groups of 64: lane j - j0 collects the bits of file j
        for (int j0 = 0; j0 < f; j0 += 64) {
            const int j1 = j0 + 64 < f ? j0 + 64 : f;
            uint32_t flags = 0;
            for (int j = j0; j < j1; ++j) {
                if (only_files != nullptr && only_files[j] == 0) continue;  // the same for every thread
                uint32_t x[R][V];
#pragma unroll
                for (int k = 0; k < R; ++k)
                    load_vec<V>(base + (int64_t)file_rows[j * R + k] * ld, x[k]);
                uint32_t wb = 0;
#pragma unroll
                for (int a = 0; a < R; ++a)
#pragma unroll
                    for (int b = a + 1; b < R; ++b)
                        wb |= wave_any(differ<V>(x[a], x[b])) << pair_bit(R, a, b);
                if (lane == j - j0) flags |= wb;
            }
            merge_flags(pair_neq + j0, j1 - j0, lane, flags);
        }
    }
    const int tail = (int)(d - n_vec * V);
    if (blockIdx.x == gridDim.x - 1 && (int)threadIdx.x < tail) {
        const int64_t c = n_vec * V + threadIdx.x;
        for (int j = 0; j < f; ++j) {
            if (only_files != nullptr && only_files[j] == 0) continue;
            uint32_t x[R];
#pragma unroll
            for (int k = 0; k < R; ++k) x[k] = X[(int64_t)file_rows[j * R + k] * ld + c];
            uint32_t bits = 0;
#pragma unroll
            for (int a = 0; a < R; ++a)
#pragma unroll
                for (int b = a + 1; b < R; ++b)
                    bits |= (x[a] != x[b] ? 1u : 0u) << pair_bit(R, a, b);
            if (bits != 0) atomicOr(&pair_neq[j], bits);
        }
    }
}

// Nonzero iff some word of the two chunks is not close: bit patterns differ and
// |a - b| > atol + rtol * max(|a|, |b|) (or the test involves a NaN).  Every operation is
// rounded to fp32 on its own (no fused multiply-add), as the CPU reference does.
template <int V>
__device__ __forceinline__ uint32_t far_apart(const uint32_t (&a)[V], const uint32_t (&b)[V],
                                              float atol, float rtol) {
    uint32_t acc = 0;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float x = __uint_as_float(a[v]), y = __uint_as_float(b[v]);
        const float diff = fabsf(__fsub_rn(x, y));
        const float bound = __fadd_rn(atol, __fmul_rn(rtol, fmaxf(fabsf(x), fabsf(y))));
        acc |= (a[v] != b[v] && !(diff <= bound)) ? 1u : 0u;
    }
    return acc;
}

// Tolerant variant of the vote's comparison (Sec. 2: rounding differences between honest copies can be
// handled by clustering the copies): for every file, which pairs of copies are not close
// somewhere in [0, d).  Same decomposition as vote_pairs_kernel.
template <int R, int V>
__global__ __launch_bounds__(kBlock) void vote_pairs_tolerant_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ file_rows,
    int f, float atol, float rtol, uint32_t *pair_far) {
    const int lane = threadIdx.x & 63;
    const int64_t n_vec = d / V;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n_vec > 0) {
        const uint32_t *base = X + (gt < n_vec ? gt : n_vec - 1) * V;
        for (int j0 = 0; j0 < f; j0 += 64) {
            const int j1 = j0 + 64 < f ? j0 + 64 : f;
            uint32_t flags = 0;
            for (int j = j0; j < j1; ++j) {
                uint32_t x[R][V];
#pragma unroll
                for (int k = 0; k < R; ++k)
                    load_vec<V>(base + (int64_t)file_rows[j * R + k] * ld, x[k]);
                uint32_t wb = 0;
#pragma unroll
                for (int a = 0; a < R; ++a)
#pragma unroll
                    for (int b = a + 1; b < R; ++b)
                        wb |= wave_any(far_apart<V>(x[a], x[b], atol, rtol)) << pair_bit(R, a, b);
                if (lane == j - j0) flags |= wb;
            }
            merge_flags(pair_far + j0, j1 - j0, lane, flags);
        }
    }
    const int tail = (int)(d - n_vec * V);
    if (blockIdx.x == gridDim.x - 1 && (int)threadIdx.x < tail) {
        const int64_t c = n_vec * V + threadIdx.x;
        for (int j = 0; j < f; ++j) {
            uint32_t x[R][1];
#pragma unroll
            for (int k = 0; k < R; ++k) x[k][0] = X[(int64_t)file_rows[j * R + k] * ld + c];
            uint32_t bits = 0;
#pragma unroll
            for (int a = 0; a < R; ++a)
#pragma unroll
                for (int b = a + 1; b < R; ++b)
                    bits |= far_apart<1>(x[a], x[b], atol, rtol) << pair_bit(R, a, b);
            if (bits != 0) atomicOr(&pair_far[j], bits);
        }
    }
}

// Steps of the generated streamed programs (selnet_stream_<f>.inc), written against local names
// of the kernel that includes them: NS slots per file, V words per thread, kAhead, stage, key,
// o, lane, flags (one word per 64 files), and BYZ_S_ROW_ADDR(j, k) = address of this thread's vector in
// slot k of file j.
// Hook a kernel may redefine around the include: BYZ_S_KEY(j, x) = key of word x of file j.
// BYZ_S_STEP(j) opens file j's share of the program and BYZ_S_PIN(w) follows the comparators of
// a share for every wire they changed; both do nothing unless a kernel redefines them.
#define BYZ_S_KEY(j, x) to_key(x)
#define BYZ_S_STEP(j)
#define BYZ_S_PIN(w)
// An empty statement the compiler may not execute speculatively: keeps the one-lane update of a
// file's pair bits a real branch, and with it the file boundaries of the program (left as one
// straight-line block, the compiler keeps every ballot alive to the end and runs out of
// registers).
#define BYZ_S_KEEP_BRANCH asm volatile("" ::: "memory");
#define BYZ_S_LOAD_(j)                                                                        \
    _Pragma("unroll") for (int k_ = 0; k_ < NS; ++k_)                                         \
        load_vec<V>(reinterpret_cast<const uint32_t *>(BYZ_S_ROW_ADDR(j, k_)),                \
                    stage[(j) % (kAhead + 1)][k_]);
#define BYZ_S_LOAD1(j) if constexpr (kAhead == 1) { BYZ_S_LOAD_(j) }
#define BYZ_S_LOAD2(j) if constexpr (kAhead == 2) { BYZ_S_LOAD_(j) }
#define BYZ_S_LOAD3(j) if constexpr (kAhead == 3) { BYZ_S_LOAD_(j) }
#define BYZ_S_LOAD4(j) if constexpr (kAhead == 4) { BYZ_S_LOAD_(j) }
#define BYZ_S_LOAD5(j) if constexpr (kAhead == 5) { BYZ_S_LOAD_(j) }
#define BYZ_S_LOAD20(j) if constexpr (kAhead == 20) { BYZ_S_LOAD_(j) }
#define BYZ_S_USE(j)                                                                          \
    {                                                                                         \
        [[maybe_unused]] int pick_ = 0;                                                       \
        if constexpr (NS > 1) {                                                               \
        uint32_t wb_ = 0, word_ = 0;                                                          \
        _Pragma("unroll") for (int a_ = 0; a_ < NS; ++a_)                                     \
        _Pragma("unroll") for (int b_ = a_ + 1; b_ < NS; ++b_)                                \
            wb_ |= wave_differ<V>(stage[(j) % (kAhead + 1)][a_],                              \
                                  stage[(j) % (kAhead + 1)][b_]) << pair_bit(NS, a_, b_);     \
        pick_ = local_choice<NS>(wb_, word_);                                                 \
        if (lane == ((j) & 63)) {                                                             \
            flags[(j) >> 6] |= word_;                                                         \
            BYZ_S_KEEP_BRANCH                                                                 \
        }                                                                                     \
        }                                                                                     \
        _Pragma("unroll") for (int v_ = 0; v_ < V; ++v_)                                      \
            key[v_][j] = BYZ_S_KEY(j, stage[(j) % (kAhead + 1)][0][v_]);                      \
        if constexpr (NS > 1) {                                                               \
        /* wave-uniform and rare: slot 0 is outside the largest class of this wave */         \
        if (__builtin_expect(pick_ != 0, 0)) {                                                \
            _Pragma("unroll") for (int v_ = 0; v_ < V; ++v_) {                                \
                uint32_t x_ = stage[(j) % (kAhead + 1)][1][v_];                               \
                _Pragma("unroll") for (int k_ = 2; k_ < NS; ++k_)                             \
                    x_ = pick_ == k_ ? stage[(j) % (kAhead + 1)][k_][v_] : x_;                \
                key[v_][j] = BYZ_S_KEY(j, x_);                                                \
            }                                                                                 \
            BYZ_S_KEEP_BRANCH                                                                 \
        }                                                                                     \
        }                                                                                     \
    }
#define BYZ_S_CE(i, j)                                                                        \
    _Pragma("unroll") for (int v_ = 0; v_ < V; ++v_) {                                        \
        const uint32_t a_ = key[v_][i], b_ = key[v_][j];                                      \
        key[v_][i] = a_ < b_ ? a_ : b_;                                                       \
        key[v_][j] = a_ < b_ ? b_ : a_;                                                       \
    }
#define BYZ_S_CE_LO(i, j)                                                                     \
    _Pragma("unroll") for (int v_ = 0; v_ < V; ++v_)                                          \
        key[v_][i] = key[v_][i] < key[v_][j] ? key[v_][i] : key[v_][j];
#define BYZ_S_CE_HI(i, j)                                                                     \
    _Pragma("unroll") for (int v_ = 0; v_ < V; ++v_)                                          \
        key[v_][j] = key[v_][i] < key[v_][j] ? key[v_][j] : key[v_][i];
#define BYZ_S_SORTED(n)  // wires 0..n-1 now hold the keys in ascending order
#define BYZ_S_MEDIAN(w)                                                                       \
    _Pragma("unroll") for (int v_ = 0; v_ < V; ++v_) o[v_] = from_key(key[v_][w]);

// Coordinate-wise median of F rows by a register selection network.
template <int F, int V>
__global__ __launch_bounds__(kBlock) void median_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    const int64_t n_vec = d / V;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gt < n_vec) {
        uint32_t key[V][F];
        uint32_t o[V];
        if constexpr (has_streamed_network(F)) {
            // same streamed program as the single-pass kernel, one slot per file, no compares
            constexpr int NS = 1;
            constexpr int kAhead = prefetch_depth(F, NS);
            const uint32_t voff = (uint32_t)(gt * (V * 4));
            const char *Xb = reinterpret_cast<const char *>(X);
            uint32_t stage[kAhead + 1][NS][V];
            const int lane = 0;
            uint32_t flags[(F + 63) / 64] = {};
            (void)lane; (void)flags;
#define BYZ_S_ROW_ADDR(j, k) (Xb + (uint64_t)(uint32_t)row_index[j] * (uint64_t)ld * 4u + voff)
#include "generated/selnet_stream_dispatch.inc"
#undef BYZ_S_ROW_ADDR
        } else {
            const uint32_t *base = X + gt * V;
#pragma unroll
            for (int j = 0; j < F; ++j) {
                uint32_t x[V];
                load_vec<V>(base + (int64_t)row_index[j] * ld, x);
#pragma unroll
                for (int v = 0; v < V; ++v) key[v][j] = to_key(x[v]);
            }
#pragma unroll
            for (int v = 0; v < V; ++v) o[v] = from_key(SelNet<F>::median(key[v]));
        }
        store_vec<V>(out + gt * V, o);
    }
    const int tail = (int)(d - n_vec * V);
    if (blockIdx.x == gridDim.x - 1 && (int)threadIdx.x < tail) {
        const int64_t c = n_vec * V + threadIdx.x;
        uint32_t key[F];
#pragma unroll
        for (int j = 0; j < F; ++j) key[j] = to_key(X[(int64_t)row_index[j] * ld + c]);
        out[c] = from_key(SelNet<F>::median(key));
    }
}

// Coordinate-wise median by the streamed program of the generated network on F wires with V = vec_for_median(F)
// words per thread: the large networks (F = 81, 121: MOLS over F_9 and F_11) and, with PAD,
// any odd f < F on the next generated size -- the F - f spare wires reload row_index[0] and
// are tied half to the smallest and half to the largest key, which leaves the median where
// it was.  Thread t owns the words starting at min(V*t, d - V): the last vector overlaps its
// neighbour (both write the same values).  Needs d >= V.
template <int F, int V, bool PAD>
__global__ __launch_bounds__(kBlock) void median_large_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    const int pad_low_end = f + (F - f) / 2;  // wires [f, pad_low_end) smallest key, rest largest
    (void)pad_low_end;
    const int64_t n_thr = (d + V - 1) / V;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gt >= n_thr) return;
    const int64_t c0 = gt * V < d - V ? gt * V : d - V;
    uint32_t key[V][F];
    uint32_t o[V];
    constexpr int NS = 1;
    // one word per thread: 4-byte loads, twenty files ahead (as measured best at F = 121)
    constexpr int kAhead = V == 1 ? 20 : prefetch_depth(F, NS);
    const uint32_t voff = (uint32_t)(c0 * 4);
    const char *Xb = reinterpret_cast<const char *>(X);
    uint32_t stage[kAhead + 1][NS][V];
    const int lane = 0;
    uint32_t flags[(F + 63) / 64] = {};
    (void)lane; (void)flags;
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) \
    (!PAD || (j) < f ? to_key(x) : ((j) < pad_low_end ? 0u : 0xFFFFFFFFu))
#define BYZ_S_ROW_ADDR(j, k) \
    (Xb + (uint64_t)(uint32_t)row_index[!PAD || (j) < f ? (j) : 0] * (uint64_t)ld * 4u + voff)
#include "generated/selnet_stream_dispatch.inc"
#undef BYZ_S_ROW_ADDR
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) to_key(x)
    store_vec<V>(out + c0, o);
}

// Coordinate-wise median of H < f <= 2H - 1 rows (H = 96, 112, 128: up to 255 rows), two waves per
// 64 coordinates: wave h of a block sorts wires [hH, hH + H) of its coordinates in registers
// (H-wire sorting network, one word per thread), wave 1 hands its sorted keys over through LDS,
// and wave 0 takes rank H - 1 of the union of the two sorted halves A and B as
//     min( B[H-1], A[H-1], min over m = 0..H-2 of max(A[m], B[H-2-m]) )
// (the H smallest of the union are the i smallest of A and the H - i smallest of B for some i;
// the largest of those is max(A[i-1], B[H-1-i]), and the right i minimises it).  The 2H - f
// spare wires sit at the end of half B, H - 1 - (f-1)/2 of them with the smallest key and the
// rest with the largest, which puts the median of the f values at rank H - 1.  Half the
// registers of one network over all rows, so two or three waves per SIMD instead of one and no
// spills; the schedule is not pinned (pinned as in the single pass it was 14 % slower).
// The waves-per-SIMD attribute states what the registers allow anyway; without it the compiler
// schedules the H = 128 kernel half as fast (4.7 instead of 3.0 ms on 11.2 M coordinates).
template <int F>  // = H
__global__ __launch_bounds__(128)
__attribute__((amdgpu_waves_per_eu(F <= 96 ? 3 : 2, F <= 96 ? 3 : 2)))
void median_halves_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    __shared__ uint32_t s_half[F * 64];
    const int ln = threadIdx.x & 63;
    const int first = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) * F;  // first wire of this wave
    const int64_t c = (int64_t)blockIdx.x * 64 + ln;
    const int64_t cc = c < d ? c : d - 1;  // lanes past the end redo the last coordinate
    const int pad_low_end = f + (F - 1 - (f - 1) / 2);
    constexpr int V = 1, NS = 1, kAhead = 20;
    uint32_t key[V][F];
    const uint32_t voff = (uint32_t)(cc * 4);
    const char *Xb = reinterpret_cast<const char *>(X);
    uint32_t stage[kAhead + 1][NS][V];
    const int lane = 0;
    uint32_t flags[(F + 63) / 64] = {};
    (void)lane; (void)flags;
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) \
    (first + (j) < f ? to_key(x) : (first + (j) < pad_low_end ? 0u : 0xFFFFFFFFu))
#define BYZ_S_ROW_ADDR(j, k) \
    (Xb + (uint64_t)(uint32_t)row_index[first + (j) < f ? first + (j) : 0] * (uint64_t)ld * 4u + voff)
#include "generated/selnet_sort_stream_dispatch.inc"
#undef BYZ_S_ROW_ADDR
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) to_key(x)
    if (first != 0) {
#pragma unroll
        for (int m = 0; m < F; ++m) s_half[m * 64 + ln] = key[0][m];
    }
    __syncthreads();
    if (first == 0) {
        uint32_t best = key[0][F - 1] < s_half[(F - 1) * 64 + ln] ? key[0][F - 1] : s_half[(F - 1) * 64 + ln];
#pragma unroll
        for (int m = 0; m < F - 1; ++m) {
            const uint32_t b = s_half[(F - 2 - m) * 64 + ln];
            const uint32_t t = key[0][m] > b ? key[0][m] : b;
            best = best < t ? best : t;
        }
        if (c < d) out[c] = from_key(best);
    }
}

// Coordinate-wise median for d below the vector width of the network kernels (f <= 64): rank
// counting, one coordinate a thread.
__global__ __launch_bounds__(kBlock) void median_generic_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
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

// Rounding contract of the trimmed mean: fp32, the kept values (ranks b .. F-b-1 of the sorted
// keys) are added one by one in ascending order starting from +0, then one IEEE division.
template <int F, int V, bool RUNS = false>
__device__ __forceinline__ void trimmed_mean_of_sorted(const uint32_t (&key)[V][F], int f, int b,
                                                       uint32_t (&o)[V]) {
    // wires 0..f-1 hold the f values in ascending order (f = F unless the network is padded)
    const float denom = (float)(f - 2 * b);
    if constexpr (RUNS) {
        // b and f are wave-uniform: runs of eight ranks that lie wholly inside [b, f - b) are
        // added without a test, runs wholly outside are skipped (for the kernels whose
        // schedule is pinned; the others lose registers to it)
        float acc[V];
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int i0 = 0; i0 < F; i0 += 8) {
            const int lo = i0, hi = (i0 + 8 < F ? i0 + 8 : F) - 1;
            if (lo >= b && hi < f - b) {
#pragma unroll
                for (int i = i0; i < i0 + 8; ++i)
                    if (i < F) {
#pragma unroll
                        for (int v = 0; v < V; ++v)
                            acc[v] += __uint_as_float(from_key(key[v][i < F ? i : 0]));
                    }
            } else if (hi >= b && lo < f - b) {
#pragma unroll
                for (int i = i0; i < i0 + 8; ++i)
                    if (i < F && i >= b && i < f - b) {
#pragma unroll
                        for (int v = 0; v < V; ++v)
                            acc[v] += __uint_as_float(from_key(key[v][i < F ? i : 0]));
                    }
            }
        }
#pragma unroll
        for (int v = 0; v < V; ++v) o[v] = __float_as_uint(acc[v] / denom);
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float acc = 0.0f;
#pragma unroll
            for (int i = 0; i < F; ++i)
                if (i >= b && i < f - b) acc += __uint_as_float(from_key(key[v][i]));
            o[v] = __float_as_uint(acc / denom);
        }
    }
}

// Coordinate-wise trimmed mean of F rows: the F values of a coordinate are sorted (total order
// of the keys), the b smallest and the b largest are dropped and the remaining F - 2b are
// averaged.  Rounding contract: fp32, the kept values are added one by one in ascending order
// starting from +0, then divided by float(F - 2b) (IEEE division).  Thread t owns the four
// words starting at min(4t, d - 4): the last vector overlaps its neighbour instead of a scalar
// tail (both write the same values).  Needs d >= 4.
template <int F, int V, bool PAD>
__global__ __launch_bounds__(kBlock) void trimmed_mean_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, int b, uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    const int64_t n_thr = (d + V - 1) / V;
    const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gt >= n_thr) return;
    const int64_t c0 = gt * V + V <= d ? gt * V : d - V;
    uint32_t key[V][F];
    constexpr int NS = 1;
    constexpr int kAhead = V == 1 ? 20 : prefetch_depth(F, NS);  // as the one-word median kernels
    const uint32_t voff = (uint32_t)(c0 * 4);
    const char *Xb = reinterpret_cast<const char *>(X);
    uint32_t stage[kAhead + 1][NS][V];
    const int lane = 0;
    uint32_t flags[(F + 63) / 64] = {};
    (void)lane; (void)flags;
    // PAD: f < F rows on the next generated size; the spare wires reload row_index[0] and carry
    // the largest key, so wires 0..f-1 end up holding the f values in ascending order
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) (!PAD || (j) < f ? to_key(x) : 0xFFFFFFFFu)
#define BYZ_S_ROW_ADDR(j, k) \
    (Xb + (uint64_t)(uint32_t)row_index[!PAD || (j) < f ? (j) : 0] * (uint64_t)ld * 4u + voff)
    // the widest sorting networks run with their schedule pinned (F = 169: 2.2 instead of 2.8 ms
    // for 11.2 M coordinates; the smaller ones and the median networks are faster left alone)
    if constexpr (F >= kPinFrom) {
#include "selnet_pin_on.inc"
#include "generated/selnet_sort_stream_dispatch.inc"
#include "selnet_pin_off.inc"
    } else {
#include "generated/selnet_sort_stream_dispatch.inc"
    }
#undef BYZ_S_ROW_ADDR
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) to_key(x)
    uint32_t o[V];
    trimmed_mean_of_sorted<F, V, (F >= kPinFrom)>(key, PAD ? f : F, b, o);
    store_vec<V>(out + c0, o);
}

// Sorts a bitonic sequence of F keys ascending with the log2(P) rounds of comparators P/2, P/4,
// ..., 1 apart of the P-wire bitonic merger, P the power of two at or above F.  The P - F spare
// wires carry the smallest key in front of a sequence that rises and then falls (LOW), the
// largest key behind one that falls and then rises (!LOW), which keeps either bitonic;
// comparators that only see spare wires fold away at compile time.
template <int F, int P, bool LOW>
__device__ __forceinline__ void sort_bitonic(uint32_t (&keys)[F]) {
    static_assert((P & (P - 1)) == 0 && P >= F && P < 2 * F, "P = power of two at or above F");
    if constexpr (P == F) {
        uint32_t(&k)[F] = keys;
#pragma unroll
        for (int apart = P / 2; apart >= 1; apart /= 2)
#pragma unroll
            for (int i = 0; i < P; ++i)
                if ((i & apart) == 0) BYZ_CE(i, i + apart)
    } else {
        uint32_t k[P];
#pragma unroll
        for (int i = 0; i < P; ++i)
            k[i] = LOW ? (i < P - F ? 0u : keys[i - (P - F) < 0 ? 0 : i - (P - F)])
                       : (i < F ? keys[i < F ? i : 0] : 0xFFFFFFFFu);
#pragma unroll
        for (int apart = P / 2; apart >= 1; apart /= 2)
#pragma unroll
            for (int i = 0; i < P; ++i)
                if ((i & apart) == 0) BYZ_CE(i, i + apart)
#pragma unroll
        for (int i = 0; i < F; ++i) keys[i] = k[LOW ? P - F + i : i];
    }
}

// acc += the keys' values whose ranks rank0 + i lie in [b, f - b), in ascending order.  b and f are
// wave-uniform: runs of eight ranks that lie wholly inside are added without a test, runs
// wholly outside are skipped.
template <int F>
__device__ __forceinline__ float add_kept_ranks(const uint32_t (&k)[F], int rank0, int b, int f,
                                                float acc) {
    static_assert(F % 8 == 0, "runs of eight");
#pragma unroll
    for (int i0 = 0; i0 < F; i0 += 8) {
        const int lo = rank0 + i0, hi = lo + 7;
        if (lo >= b && hi < f - b) {
#pragma unroll
            for (int i = i0; i < i0 + 8; ++i) acc += __uint_as_float(from_key(k[i]));
        } else if (hi >= b && lo < f - b) {
#pragma unroll
            for (int i = i0; i < i0 + 8; ++i)
                if (rank0 + i >= b && rank0 + i < f - b) acc += __uint_as_float(from_key(k[i]));
        }
    }
    return acc;
}

// Coordinate-wise trimmed mean of F < f <= 2F rows (F = 96, 112, 128), two waves per 64 coordinates, same
// rounding contract as trimmed_mean_kernel.  Wave h sorts wires [hF, hF + F) of its coordinates
// in registers (the 2F - f spare wires at the end carry the largest key).  With A and B the two
// sorted halves, min(A[m], B[F-1-m]) over m holds the F smallest of the union and max(...) the
// F largest, each as a bitonic sequence: wave 1 passes B through LDS, wave 0 keeps the minima
// and passes the maxima back through the same words, and each wave sorts its bitonic half
// (sort_bitonic).  Wave 0 then holds ranks 0..F-1 and
// wave 1 ranks F..2F-1; the kept ranks are added in ascending order, wave 0's partial sum
// going to wave 1 through LDS.  Half the registers of one 256-wire network per thread.
template <int F>
__global__ __launch_bounds__(128)
__attribute__((amdgpu_waves_per_eu(2, 2)))
void trimmed_halves_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, int b, uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    __shared__ uint32_t s_half[F * 64];
    __shared__ float s_sum[64];
    const int ln = threadIdx.x & 63;
    const int first = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) * F;  // first wire of this wave
    const int64_t c = (int64_t)blockIdx.x * 64 + ln;
    const int64_t cc = c < d ? c : d - 1;  // lanes past the end redo the last coordinate
    constexpr int V = 1, NS = 1, kAhead = 20;
    uint32_t key[V][F];
    const uint32_t voff = (uint32_t)(cc * 4);
    const char *Xb = reinterpret_cast<const char *>(X);
    uint32_t stage[kAhead + 1][NS][V];
    const int lane = 0;
    uint32_t flags[(F + 63) / 64] = {};
    (void)lane; (void)flags;
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) (first + (j) < f ? to_key(x) : 0xFFFFFFFFu)
#define BYZ_S_ROW_ADDR(j, k) \
    (Xb + (uint64_t)(uint32_t)row_index[first + (j) < f ? first + (j) : 0] * (uint64_t)ld * 4u + voff)
#include "generated/selnet_sort_stream_dispatch.inc"
#undef BYZ_S_ROW_ADDR
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) to_key(x)
    uint32_t(&k)[F] = key[0];
    if (first != 0) {
#pragma unroll
        for (int m = 0; m < F; ++m) s_half[m * 64 + ln] = k[m];
    }
    __syncthreads();
    if (first == 0) {
#pragma unroll
        for (int m = 0; m < F; ++m) {
            const uint32_t a_ = k[m], b_ = s_half[(F - 1 - m) * 64 + ln];
            k[m] = a_ < b_ ? a_ : b_;
            s_half[(F - 1 - m) * 64 + ln] = a_ < b_ ? b_ : a_;
        }
    }
    __syncthreads();
    // ranks first .. first + F - 1, ascending; wave 0 adds its kept ranks first
    float acc = 0.0f;
    constexpr int P = 128;  // wires of the bitonic merger
    if constexpr (F == P) {
        if (first != 0) {
#pragma unroll
            for (int m = 0; m < F; ++m) k[m] = s_half[m * 64 + ln];
        }
        sort_bitonic<F, P, true>(k);  // no spare wires: one code path for both waves
    }
    if (first == 0) {
        if constexpr (F != P) sort_bitonic<F, P, true>(k);
        acc = add_kept_ranks<F>(k, 0, b, f, acc);
        s_sum[ln] = acc;
    }
    __syncthreads();
    if (first != 0) {
        if constexpr (F != P) {
#pragma unroll
            for (int m = 0; m < F; ++m) k[m] = s_half[m * 64 + ln];
            sort_bitonic<F, P, false>(k);
        }
        acc = add_kept_ranks<F>(k, F, b, f, s_sum[ln]);
        if (c < d) out[c] = __float_as_uint(acc / (float)(f - 2 * b));
    }
}

// Trimmed mean for d below the vector width of the network kernels (f <= 64): insertion sort
// in per-thread memory, one coordinate a thread; same rounding contract as trimmed_mean_kernel.
__global__ __launch_bounds__(kBlock) void trimmed_mean_generic_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const int32_t *__restrict__ row_index,
    int f, int b, uint32_t *__restrict__ out, const uint32_t *__restrict__ gate, int gate_n) {
    if (gate != nullptr && !any_word_set(gate, gate_n)) return;
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= d) return;
    uint32_t key[BYZ_MAX_F];
    for (int j = 0; j < f; ++j) {
        const uint32_t x = to_key(X[(int64_t)row_index[j] * ld + c]);
        int t = j - 1;
        while (t >= 0 && key[t] > x) { key[t + 1] = key[t]; --t; }
        key[t + 1] = x;
    }
    float acc = 0.0f;
    for (int i = b; i < f - b; ++i) acc += __uint_as_float(from_key(key[i]));
    out[c] = __float_as_uint(acc / (float)(f - 2 * b));
}

// Mean around the median (second phase of Bulyan) for one coordinate whose theta values sit
// in ascending order in col[0], col[stride], ..: the beta values closest to the middle one
// (the median), added in ascending order from +0 in fp32 and divided by float(beta).
// Growing the window from the median one neighbour at a time -- the lower one when
// (median - lower) <= (upper - median) in fp32, or when no upper one is left -- ends, for
// finite values, at the window that starts at the first position s (from max(0, h-beta+1) to
// h, h the median's position) whose value is taken before the one beta places above it:
// s + beta beyond the end, or (median - col[s]) <= (col[s+beta] - median).  That test is
// false up to s and true from s on (rounded differences stay monotone), so the start is the
// lowest candidate plus the number of failed tests: independent LDS reads, no chain.
__device__ __forceinline__ float mean_around_median(const float *col, int stride, int theta,
                                                    int beta) {
    const int h = (theta - 1) / 2;
    const float med = col[h * stride];
    const int s_min = h - beta + 1 > 0 ? h - beta + 1 : 0;
    // eight candidates at a time: all their LDS reads first (indices clamped into the column,
    // results of positions past the last candidate discarded), then the tests
    int fails = 0;
    for (int s0 = s_min; s0 < h; s0 += 8) {
        float xl[8], xr[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int s = s0 + u < h ? s0 + u : h;
            const int up = s + beta <= theta - 1 ? s + beta : theta - 1;
            xl[u] = col[s * stride];
            xr[u] = col[up * stride];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int s = s0 + u;
            const bool taken = s + beta > theta - 1 || (med - xl[u]) <= (xr[u] - med);
            fails += (s < h && !taken) ? 1 : 0;
        }
    }
    const int lo = s_min + fails;
    float acc = 0.0f;
    for (int t0 = 0; t0 < beta; t0 += 8) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = col[(lo + (t0 + u < beta ? t0 + u : beta - 1)) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = t0 + u < beta ? acc + x[u] : acc;
    }
    return acc / (float)beta;
}

// Second phase of Bulyan: the theta rows selected_rows[0..theta-1] are sorted per coordinate
// by the streamed full-sort network on N >= theta wires (N the next generated size); the
// N - theta spare wires reload the first row and are tied to the largest
// key, so wires 0..theta-1
// end up holding the chosen values in ascending order.  They go to an LDS column of the thread
// (word i*BLOCK + thread: conflict-free), where the window around the median is found with
// run-time indices.  Thread t owns the words from min(V*t, d - V); needs d >= V.
// Dynamic LDS: N*BLOCK*4 bytes; the widest networks run one wave a block, so that several
// blocks' columns fit a CU and the number of waves is again what the registers allow.
template <int F, int V, int BLOCK>
__global__ __launch_bounds__(BLOCK) void bulyan_mean_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld,
    const int32_t *__restrict__ selected_rows, int theta, int beta, uint32_t *__restrict__ out) {
    extern __shared__ float s_bulyan_col[];
    const int64_t n_thr = (d + V - 1) / V;
    const int64_t gt = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (gt >= n_thr) return;
    const int64_t c0 = gt * V + V <= d ? gt * V : d - V;
    uint32_t key[V][F];
    constexpr int NS = 1;
    constexpr int kAhead = prefetch_depth(F, NS);
    const uint32_t voff = (uint32_t)(c0 * 4);
    const char *Xb = reinterpret_cast<const char *>(X);
    uint32_t stage[kAhead + 1][NS][V];
    const int lane = 0;
    uint32_t flags[(F + 63) / 64] = {};
    (void)lane; (void)flags;
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) ((j) < theta ? to_key(x) : 0xFFFFFFFFu)
#define BYZ_S_ROW_ADDR(j, k) \
    (Xb + (uint64_t)(uint32_t)selected_rows[(j) < theta ? (j) : 0] * (uint64_t)ld * 4u + voff)
#include "generated/selnet_sort_stream_dispatch.inc"
#undef BYZ_S_ROW_ADDR
#undef BYZ_S_KEY
#define BYZ_S_KEY(j, x) to_key(x)
    float *col = s_bulyan_col + threadIdx.x;
    uint32_t o[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
#pragma unroll
        for (int i = 0; i < F; ++i) col[i * BLOCK] = __uint_as_float(from_key(key[v][i]));
        o[v] = __float_as_uint(mean_around_median(col, BLOCK, theta, beta));
    }
    store_vec<V>(out + c0, o);
}

// Second phase of Bulyan for theta > 121 and for d < 4: one coordinate a thread, the chosen
// values insertion-sorted in the thread's LDS column.  Dynamic LDS: theta*kBlock*4 bytes.
__global__ __launch_bounds__(kBlock) void bulyan_mean_generic_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld,
    const int32_t *__restrict__ selected_rows, int theta, int beta, uint32_t *__restrict__ out) {
    extern __shared__ float s_bulyan_col[];
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= d) return;
    uint32_t *kcol = reinterpret_cast<uint32_t *>(s_bulyan_col) + threadIdx.x;
    for (int j = 0; j < theta; ++j) {
        const uint32_t x = to_key(X[(int64_t)selected_rows[j] * ld + c]);
        int t = j - 1;
        while (t >= 0 && kcol[t * kBlock] > x) {
            kcol[(t + 1) * kBlock] = kcol[t * kBlock];
            --t;
        }
        kcol[(t + 1) * kBlock] = x;
    }
    for (int j = 0; j < theta; ++j) kcol[j * kBlock] = from_key(kcol[j * kBlock]);
    out[c] = __float_as_uint(mean_around_median(s_bulyan_col + threadIdx.x, kBlock, theta, beta));
}

// First kernel of a single-pass call: clears the state the later kernels accumulate into and
// lays out the rows of each file for the pass.  When every copy is read, that is the replica
// order as it stands: each wave chooses for itself which copy feeds the median.
// In early-majority mode the kernel is a probe: it compares the copies of every file on a
// sample of <= kProbe coordinates (kProbe/16 runs of 16 consecutive words spread over [0, d); all
// of [0, d) when d <= kProbe), derives the probable equality classes, and puts the probable
// winner's class first (the copies that mode reads) and equal-looking copies adjacent.  Only
// the speed of the call depends on this guess.
// One block of kProbeThreads threads: thread group q = tid / kProbe takes the files
// q, q + kProbeSplit, ..., every group on the same kProbe sample coordinates, so a thread waits
// for F*R / kProbeSplit loads.
template <int F, int R>
__global__ __launch_bounds__(kProbeThreads) void probe_kernel(const uint32_t *__restrict__ X,
                                                           int64_t d, int64_t ld,
                                                           const int32_t *__restrict__ file_rows,
                                                           AggWorkspace *ws, int probe_opts) {
    const int early_majority = probe_opts & 1;        // bit 0: early-majority mode
    const uint32_t shift = (uint32_t)probe_opts >> 16;  // bits 16..31: moves the sample
    __shared__ uint32_t s_neq[kWide];
    __shared__ uint32_t s_all_majority;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    static_assert(kProbe >= kWide, "one probe thread per file");
    if (tid < kWide) {
        s_neq[tid] = 0;
        ws->pneq[tid] = 0;
        ws->pair_neq[tid] = 0;
    }
    if (tid == 0) {
        s_all_majority = 1;
        ws->need_median = 0;
        ws->need_revote = 0;
        ws->path = 0;
    }
    __syncthreads();
    if (early_majority == 0) {
        if (tid < F) {
            uint32_t packed = (uint32_t)R << 24;
            for (int p = 0; p < R; ++p) {
                ws->perm_off[tid * kRowStride + p] = (uint64_t)file_rows[tid * R + p] * (uint64_t)ld * 4u;
                packed |= (uint32_t)p << (3 * p);
            }
            ws->perm[tid] = packed;
        }
        if (tid == 0) ws->slots_per_file = R;
        return;
    }

    // threads without a sample coordinate of their own redo coordinate 0
    const int ct = tid % kProbe;  // which sample coordinate
    const int q = tid / kProbe;   // which share of the files (wave-uniform: kProbe % 64 == 0)
    int64_t c = 0;
    if (d <= kProbe) {
        if (ct < d) c = ct;
    } else {
        // runs start (d - 16) / 15 apart from a point the caller's shift picks, wrapping
        // around so that a run stays inside [0, d)
        const int64_t run = ct >> 4, off = ct & 15;
        const uint64_t start = ((uint64_t)shift * 2654435761ull) % (uint64_t)(d - 15);
        c = (int64_t)(((uint64_t)(run * ((d - 16) / (kProbe / 16 - 1))) + start) % (uint64_t)(d - 15)) + off;
    }
    // this group's files in batches of G: all loads of a batch are issued before the first
    // ballot waits; the bits of file j are parked in lane j % 64, word j / 64
    constexpr int kMine = (F + kProbeSplit - 1) / kProbeSplit;  // files per group, at most
    constexpr int G = (kMine * R <= 96) ? kMine : 96 / R;
    uint32_t flags[(F + 63) / 64] = {};
#pragma unroll
    for (int t0 = 0; t0 < kMine; t0 += G) {
        uint32_t x[G][R];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int j = q + kProbeSplit * (t0 + g);
#pragma unroll
            for (int k = 0; k < R; ++k)
                if (t0 + g < kMine && j < F) x[g][k] = X[(int64_t)file_rows[j * R + k] * ld + c];
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int j = q + kProbeSplit * (t0 + g);
            if (t0 + g >= kMine || j >= F) continue;
            uint32_t wb = 0;
#pragma unroll
            for (int a = 0; a < R; ++a)
#pragma unroll
                for (int b = a + 1; b < R; ++b)
                    wb |= wave_any(x[g][a] ^ x[g][b]) << pair_bit(R, a, b);
#pragma unroll
            for (int w = 0; w < (F + 63) / 64; ++w)
                if (lane == (j & 63) && (j >> 6) == w) flags[w] |= wb;
        }
    }
#pragma unroll
    for (int w = 0; w < (F + 63) / 64; ++w)
        if (64 * w + lane < F && flags[w] != 0) atomicOr(&s_neq[64 * w + lane], flags[w]);
    __syncthreads();

    if (tid < F) {
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
        // Early-majority mode: once r' = (R+1)/2 copies are known to be identical they are the
        // majority whatever the other copies hold (Sec. 2), so when the probable winner's class
        // has at least r' members only its first r' are read and verified; the remaining slots
        // repeat slot 0 (served from cache) and carry no assumption.
        int members = 0;
        for (int k = 0; k < R; ++k) members += label[k] == label[w] ? 1 : 0;
        const int need = (R + 1) / 2;
        const int slots = (early_majority != 0 && members >= need) ? need : R;
        uint32_t packed = (uint32_t)slots << 24;
        for (int p = 0; p < R; ++p) {
            const int k = perm[p < slots ? p : 0];
            ws->perm_off[j * kRowStride + p] = (uint64_t)file_rows[j * R + k] * (uint64_t)ld * 4u;
            packed |= (uint32_t)k << (3 * p);
        }
        ws->perm[j] = packed;
        if (slots != need) s_all_majority = 0;
    }
    __syncthreads();
    // if every file gets by with r' slots, the single pass loads only those
    if (tid == 0) ws->slots_per_file = (early_majority != 0 && s_all_majority != 0) ? (R + 1) / 2 : R;
}

// Which tile of kBlock threads a block works on.  Blocks go to the eight XCDs round-robin
// (block b runs on XCD b mod 8).  A launch that is over after a round or two of resident blocks
// is dominated by its start: there every XCD gets one contiguous eighth of the tiles, so that
// its L2 and address translation see one range of every row instead of all of it (d = 2^20,
// 75 rows: 56 -> 52.5 us).  Long launches keep the plain order, which measured 1-3 % faster there.
constexpr unsigned kShortLaunchBlocks = 2048;
__device__ __forceinline__ unsigned tile_of_block(unsigned b, unsigned n_blocks) {
    if (n_blocks > kShortLaunchBlocks) return b;
    const unsigned q = n_blocks / 8, rem = n_blocks % 8, x = b % 8, i = b / 8;
    return x * q + (x < rem ? x : rem) + i;  // XCD x owns q tiles, one more if x < rem
}

// Vote and median in one pass: streams the first NS slots of every file's permuted row list once (NS = R:
// every copy; NS = r' = (R+1)/2 in early-majority mode when every file has a probable
// majority).  Every pair of slots is compared over all coordinates (ws->pneq), which is the whole
// of the vote's comparison, and each wave feeds the median network from the slot that
// local_choice picks by what it has just compared: where a file has a strict majority over all
// of d, that slot holds the majority's values on the wave's coordinates, so a copy that was
// tampered with somewhere else costs nothing.  The decision kernel behind this one knows the
// true winners and, from the bits that say which slots the fed ones differed from, whether
// every wave fed the winner's values.
template <int F, int R, int NS, bool TRIM, int V>
__device__ __forceinline__ void fused_body(const uint32_t *__restrict__ X, int64_t d, int64_t ld,
                                           const uint64_t *__restrict__ perm_off,
                                           AggWorkspace *ws, int trim_b,
                                           uint32_t *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    // Thread t owns the V words starting at min(V*t, d - V): the last vector of a row overlaps
    // its neighbour instead of a scalar tail, and threads past the end redo it, so there are
    // no branches around loads and ballots (d >= V is the launcher's business).
    const int64_t n_thr = (d + V - 1) / V;
    const int64_t gt = (int64_t)tile_of_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
    const int64_t c0 = (gt + 1) * V <= d ? gt * V : d - V;
    uint32_t flags[(F + 63) / 64] = {};  // lane j%64 collects the pair bits of file j
    // What other waves have published so far, read now so that the wait is over long before the
    // end: a wave whose bits were all there when it started (all but the first waves of a
    // launch) ends without touching the shared words at all.
    uint32_t seen[(F + 63) / 64];
#pragma unroll
    for (int w = 0; w < (F + 63) / 64; ++w)
        seen[w] = 64 * w + lane < F ? load_shared_word(&ws->pneq[64 * w + lane]) : 0u;
    const uint32_t voff = (uint32_t)(c0 * 4);
    const char *Xb = reinterpret_cast<const char *>(X);
    uint32_t key[V][F];       // wire j of the network = file j
    // files prefetched ahead of the one being consumed
    constexpr int kAhead = prefetch_depth(F, NS);
    uint32_t stage[kAhead + 1][NS][V];  // copies of the file in use and of those in flight
    uint32_t o[V];
    // The generated program walks the files in order: the loads of file j+kAhead are issued
    // before file j is consumed (compares, key), followed by every comparator of the median
    // (or, for the trimmed mean, sorting) network whose inputs are complete by then.
#define BYZ_S_ROW_ADDR(j, k) (Xb + perm_off[(j) * kRowStride + (k)] + voff)
    if constexpr (!TRIM) {
        // median: every comparator is made to run in the share of the file that completes its
        // inputs, so that a wave has loads in flight while it works through the network instead
        // of running the whole network at the end
#include "selnet_pin_on.inc"
#include "generated/selnet_stream_dispatch.inc"
#include "selnet_pin_off.inc"
    } else {
#include "selnet_pin_on.inc"
#include "generated/selnet_sort_stream_dispatch.inc"
#include "selnet_pin_off.inc"
        trimmed_mean_of_sorted<F, V, true>(key, F, trim_b, o);
    }
#undef BYZ_S_ROW_ADDR
    if (gt < n_thr) store_vec<V>(out + c0, o);
#pragma unroll
    for (int w = 0; w < (F + 63) / 64; ++w)
        merge_flags(ws->pneq + 64 * w, F - 64 * w < 64 ? F - 64 * w : 64, lane,
                    flags[w] & ~seen[w]);
}

template <int F, int R, bool TRIM, int V>
__global__ __launch_bounds__(kBlock) void fused_kernel(
    const uint32_t *__restrict__ X, int64_t d, int64_t ld, const uint64_t *__restrict__ perm_off,
    const uint32_t *__restrict__ slots_per_file, AggWorkspace *ws, int trim_b,
    uint32_t *__restrict__ out) {
    // wave-uniform choice written by the probe
    if (*slots_per_file == (R + 1) / 2)
        fused_body<F, R, (R + 1) / 2, TRIM, V>(X, d, ld, perm_off, ws, trim_b, out);
    else
        fused_body<F, R, R, TRIM, V>(X, d, ld, perm_off, ws, trim_b, out);
}

// ---------------------------------------------------------------------------- launchers

[[maybe_unused]] constexpr int kVec = 4;  // words per thread and load; rows only need dword alignment

// blocks for n_vec vector-owning threads; at least one so the trailing words get a block
inline unsigned blocks_for(int64_t n_vec) {
    const int64_t b = (n_vec + kBlock - 1) / kBlock;
    return (unsigned)(b > 0 ? b : 1);
}

[[maybe_unused]] constexpr int64_t kMaxCoords = (int64_t)1 << 30;  // byte offsets inside a row fit 32 bits

#if BYZ_IN_PART(0)
template <int R>
int launch_vote_pairs(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, int f,
                      uint32_t *neq, const uint32_t *gate, int gate_n, const uint32_t *only_files,
                      hipStream_t s) {
    vote_pairs_kernel<R, kVec><<<blocks_for(d / kVec), kBlock, 0, s>>>(X, d, ld, rows, f, neq, gate,
                                                                      gate_n, only_files);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

int launch_vote_pairs_r(int r, const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows,
                        int f, uint32_t *neq, const uint32_t *gate, int gate_n,
                        const uint32_t *only_files, hipStream_t s) {
    switch (r) {
        case 3: return launch_vote_pairs<3>(X, d, ld, rows, f, neq, gate, gate_n, only_files, s);
        case 5: return launch_vote_pairs<5>(X, d, ld, rows, f, neq, gate, gate_n, only_files, s);
        case 7: return launch_vote_pairs<7>(X, d, ld, rows, f, neq, gate, gate_n, only_files, s);
        default: return BYZ_EINVAL;
    }
}

int launch_vote_pairs_tolerant(int r, const uint32_t *X, int64_t d, int64_t ld,
                               const int32_t *rows, int f, float atol, float rtol, uint32_t *far,
                               hipStream_t s) {
    const unsigned g = blocks_for(d / kVec);
    switch (r) {
        case 3:
            vote_pairs_tolerant_kernel<3, kVec><<<g, kBlock, 0, s>>>(X, d, ld, rows, f, atol, rtol, far);
            break;
        case 5:
            vote_pairs_tolerant_kernel<5, kVec><<<g, kBlock, 0, s>>>(X, d, ld, rows, f, atol, rtol, far);
            break;
        case 7:
            vote_pairs_tolerant_kernel<7, kVec><<<g, kBlock, 0, s>>>(X, d, ld, rows, f, atol, rtol, far);
            break;
        default: return BYZ_EINVAL;
    }
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

#endif  // part 0

#if BYZ_IN_PART(5)
template <int F>
int launch_median_net(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index,
                      uint32_t *out, const uint32_t *gate, int gate_n, hipStream_t s) {
    median_kernel<F, kVec><<<blocks_for(d / kVec), kBlock, 0, s>>>(X, d, ld, row_index, out, gate,
                                                                  gate_n);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

#endif  // part 5

#if BYZ_IN_PART(5) || BYZ_IN_PART(9) || BYZ_IN_PART(11) || BYZ_IN_PART(16)
template <int F, bool PAD>
int launch_median_large(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                        uint32_t *out, const uint32_t *gate, int gate_n, hipStream_t s) {
    constexpr int V = vec_for_median(F);
    median_large_kernel<F, V, PAD><<<blocks_for((d + V - 1) / V), kBlock, 0, s>>>(
        X, d, ld, row_index, f, out, gate, gate_n);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

#endif  // parts 5, 9, 11, 16

#if BYZ_IN_PART(5)
int launch_median(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                  uint32_t *out, const uint32_t *gate, int gate_n, hipStream_t s) {
    if (d == 0) return BYZ_OK;
    switch (f) {
        case 1: return launch_median_net<1>(X, d, ld, row_index, out, gate, gate_n, s);
        case 3: return launch_median_net<3>(X, d, ld, row_index, out, gate, gate_n, s);
        case 5: return launch_median_net<5>(X, d, ld, row_index, out, gate, gate_n, s);
        case 7: return launch_median_net<7>(X, d, ld, row_index, out, gate, gate_n, s);
        case 9: return launch_median_net<9>(X, d, ld, row_index, out, gate, gate_n, s);
        case 15: return launch_median_net<15>(X, d, ld, row_index, out, gate, gate_n, s);
        case 21: return launch_median_net<21>(X, d, ld, row_index, out, gate, gate_n, s);
        case 25: return launch_median_net<25>(X, d, ld, row_index, out, gate, gate_n, s);
        case 35: return launch_median_net<35>(X, d, ld, row_index, out, gate, gate_n, s);
        case 49: return launch_median_net<49>(X, d, ld, row_index, out, gate, gate_n, s);
        default: break;
    }
    if (d < kVec && f <= BYZ_MAX_F) {  // too short for the vector kernels: cost is irrelevant
        median_generic_kernel<<<blocks_for(d), kBlock, 0, s>>>(X, d, ld, row_index, f, out, gate,
                                                               gate_n);
        BYZ_HIP(hipGetLastError());
        return BYZ_OK;
    }
    // any other odd f: the next generated size with spare wires, if d allows its vector width
    if (f <= 15) return launch_median_large<15, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 21) return launch_median_large<21, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 25) return launch_median_large<25, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 35) return launch_median_large<35, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 49) return launch_median_large<49, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if ((f == 63 || f == 65) && d >= vec_for_median(81))  // Ramanujan Case 2 shapes (63,7), (65,5)
        return f == 63 ? launch_median_large<63, false>(X, d, ld, row_index, f, out, gate, gate_n, s)
                       : launch_median_large<65, false>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f == 81 && d >= vec_for_median(81))
        return launch_median_large<81, false>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 81 && d >= vec_for_median(81))
        return launch_median_large<81, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f == 121) return launch_median_large<121, false>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 121) return launch_median_large<121, true>(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f == 169) return byz_internal_launch_median_169(X, d, ld, row_index, f, out, gate, gate_n, s);
    if (f <= 169) return byz_internal_launch_median_169_padded(X, d, ld, row_index, f, out, gate, gate_n, s);
    return byz_internal_launch_median_255_padded(X, d, ld, row_index, f, out, gate, gate_n, s);
}

#endif  // part 5

// WITH_TRIM = false / WITH_MEDIAN = false leave that variant of the kernel out (a shape whose two
// variants are compiled in different build parts)
template <int F, int R, bool WITH_TRIM = true, bool WITH_MEDIAN = true>
int launch_fused(const uint32_t *X, int64_t d, int64_t ld, const int32_t *rows, AggWorkspace *ws,
                 uint32_t *out, int probe_opts, int trim_b, hipStream_t s) {
    if ((!WITH_TRIM && trim_b >= 0) || (!WITH_MEDIAN && trim_b < 0)) return BYZ_EINTERNAL;
    probe_kernel<F, R><<<1, kProbeThreads, 0, s>>>(X, d, ld, rows, ws, probe_opts);
    BYZ_HIP(hipGetLastError());
    int rc = byz_internal_profile_mark(0, s);
    if (rc != BYZ_OK) return rc;
    constexpr int V = vec_for_pass(F, R);
    const unsigned g = blocks_for((d + V - 1) / V);
    if (trim_b < 0) {
        if constexpr (WITH_MEDIAN)
            fused_kernel<F, R, false, V><<<g, kBlock, 0, s>>>(
                X, d, ld, ws->perm_off, &ws->slots_per_file, ws, 0, out);
    } else if constexpr (WITH_TRIM) {
        fused_kernel<F, R, true, V><<<g, kBlock, 0, s>>>(
            X, d, ld, ws->perm_off, &ws->slots_per_file, ws, trim_b, out);
    }
    BYZ_HIP(hipGetLastError());
    return byz_internal_profile_mark(1, s);
}

#if BYZ_IN_PART(6) || BYZ_IN_PART(8) || BYZ_IN_PART(10) || BYZ_IN_PART(14) || BYZ_IN_PART(15) || BYZ_IN_PART(17)
template <int F, bool PAD>
int launch_trimmed_net(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                       int b, uint32_t *O, const uint32_t *gate, int gate_n, hipStream_t s) {
    constexpr int V = vec_for_trimmed(F);
    trimmed_mean_kernel<F, V, PAD><<<blocks_for((d + V - 1) / V), kBlock, 0, s>>>(
        X, d, ld, row_index, f, b, O, gate, gate_n);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

#endif  // parts 6, 8, 10, 14, 15, 17

#if BYZ_IN_PART(6)
int launch_trimmed_mean(const uint32_t *X, int64_t d, int64_t ld, const int32_t *row_index, int f,
                        int b, uint32_t *O, const uint32_t *gate, int gate_n, hipStream_t s) {
    if (d == 0) return BYZ_OK;
    if (d < kVec && f <= BYZ_MAX_F) {  // too short for the vector kernels: cost is irrelevant
        trimmed_mean_generic_kernel<<<blocks_for(d), kBlock, 0, s>>>(X, d, ld, row_index, f, b, O,
                                                                     gate, gate_n);
        BYZ_HIP(hipGetLastError());
        return BYZ_OK;
    }
    // the generated full-sort network of size f, else the next size with spare wires
    switch (f) {
        case 9: return launch_trimmed_net<9, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        case 15: return launch_trimmed_net<15, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        case 21: return launch_trimmed_net<21, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        case 25: return launch_trimmed_net<25, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        case 35: return launch_trimmed_net<35, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        case 49: return launch_trimmed_net<49, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        default: break;
    }
    if (d >= kVec) {
        if (f <= 9) return launch_trimmed_net<9, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        if (f <= 15) return launch_trimmed_net<15, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        if (f <= 21) return launch_trimmed_net<21, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        if (f <= 25) return launch_trimmed_net<25, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        if (f <= 35) return launch_trimmed_net<35, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
        if (f <= 49) return launch_trimmed_net<49, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    }
    if (f <= 63) return byz_internal_launch_trimmed_mean_63(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f <= 65) return byz_internal_launch_trimmed_mean_65(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f == 81 && d >= vec_for_trimmed(81))
        return launch_trimmed_net<81, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f <= 81 && d >= vec_for_trimmed(81))
        return launch_trimmed_net<81, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f == 121) return launch_trimmed_net<121, false>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f <= 121) return launch_trimmed_net<121, true>(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f == 169) return byz_internal_launch_trimmed_mean_169(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    if (f <= 169)
        return byz_internal_launch_trimmed_mean_169_padded(X, d, ld, row_index, f, b, O, gate, gate_n, s);
    return byz_internal_launch_trimmed_mean_256_padded(X, d, ld, row_index, f, b, O, gate, gate_n, s);
}

#endif  // part 6

#if BYZ_IN_PART(0) || BYZ_IN_PART(12) || BYZ_IN_PART(13)
template <int F>
int launch_bulyan_net(const uint32_t *X, int64_t d, int64_t ld, const int32_t *selected_rows,
                      int theta, int beta, uint32_t *O, hipStream_t s) {
    constexpr int V = vec_for_sort(F);
    constexpr int BLOCK = F > 49 ? 64 : kBlock;
    constexpr size_t lds = (size_t)F * BLOCK * 4;
    static_assert(lds <= 64 * 1024, "more than a kernel may use without asking");
    const int64_t n_thr = (d + V - 1) / V;
    bulyan_mean_kernel<F, V, BLOCK><<<(unsigned)((n_thr + BLOCK - 1) / BLOCK), BLOCK, lds, s>>>(
        X, d, ld, selected_rows, theta, beta, O);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}
#endif

#if BYZ_IN_PART(0)

// (f, r) with a compiled single-pass kernel: MOLS / Ramanujan Case 1 (f = l^2: 9, 25, 49) with
// r = 3, 5 (and 7 for f = 49, which is also Ramanujan Case 2 with m = s = 7), the Ramanujan Case 2
// shapes f = m*s with r = s: (15,3), (21,3), (35,5), (65,5), (63,7), and MOLS over F_9, F_11 and
// F_13 with r = 3: (81,3), (121,3), (169,3)
bool has_fused(int f, int r) {
    return (f == 9 && r == 3) || (f == 25 && (r == 3 || r == 5)) ||
           (f == 49 && (r == 3 || r == 5 || r == 7)) || ((f == 15 || f == 21) && r == 3) ||
           (f == 35 && r == 5) || (f == 65 && r == 5) || (f == 63 && r == 7) ||
           ((f == 81 || f == 121 || f == 169) && r == 3);
}
// ... whose trimmed-mean variant is compiled as well: all of them
bool has_fused_trim(int f, int r) { return has_fused(f, r); }

int check_common(const void *copies, int64_t d, int64_t ld, const void *rows, int f, int r) {
    if (copies == nullptr || rows == nullptr) return BYZ_EINVAL;
    if (d < 0 || ld < d || d > kMaxCoords) return BYZ_EINVAL;
    if (f < 1 || f > kWide) return BYZ_EINVAL;
    if (r < 3 || r > BYZ_MAX_R || (r % 2) == 0) return BYZ_EINVAL;
    return BYZ_OK;
}

#endif  // part 0

}  // namespace

// --------------------------------------- median and trimmed-mean launchers, a part each

#if BYZ_IN_PART(5)
int byz_internal_launch_median(const void *X, long long d, long long ld, const int *row_index,
                               int f, void *out, const void *gate, int gate_n, void *stream) {
    return launch_median(static_cast<const uint32_t *>(X), d, ld, row_index, f,
                         static_cast<uint32_t *>(out), static_cast<const uint32_t *>(gate), gate_n,
                         (hipStream_t)stream);
}
#endif

// second phase of Bulyan on the 81- and 121-wire networks, a build part each
#if BYZ_IN_PART(12)
int byz_internal_launch_bulyan_mean_81(const void *X, long long d, long long ld,
                                       const int *selected_rows, int theta, int beta, void *out,
                                       void *stream) {
    return launch_bulyan_net<81>(static_cast<const uint32_t *>(X), d, ld, selected_rows, theta, beta,
                                 static_cast<uint32_t *>(out), (hipStream_t)stream);
}
#endif
#if BYZ_IN_PART(13)
int byz_internal_launch_bulyan_mean_121(const void *X, long long d, long long ld,
                                        const int *selected_rows, int theta, int beta, void *out,
                                        void *stream) {
    return launch_bulyan_net<121>(static_cast<const uint32_t *>(X), d, ld, selected_rows, theta, beta,
                                  static_cast<uint32_t *>(out), (hipStream_t)stream);
}
#endif

// the 63- and 65-wire sorting networks (Ramanujan Case 2 with (m, s) = (9, 7) and (13, 5), and
// padded the f between 49 and 65), in the build parts of those shapes' single-pass kernels
#if BYZ_IN_PART(14)
int byz_internal_launch_trimmed_mean_63(const void *X, long long d, long long ld,
                                        const int *row_index, int f, int b, void *out,
                                        const void *gate, int gate_n, void *stream) {
    const uint32_t *x = static_cast<const uint32_t *>(X), *g = static_cast<const uint32_t *>(gate);
    if (f == 63)
        return launch_trimmed_net<63, false>(x, d, ld, row_index, f, b, static_cast<uint32_t *>(out),
                                             g, gate_n, (hipStream_t)stream);
    return launch_trimmed_net<63, true>(x, d, ld, row_index, f, b, static_cast<uint32_t *>(out), g,
                                        gate_n, (hipStream_t)stream);
}
#endif
#if BYZ_IN_PART(15)
int byz_internal_launch_trimmed_mean_65(const void *X, long long d, long long ld,
                                        const int *row_index, int f, int b, void *out,
                                        const void *gate, int gate_n, void *stream) {
    const uint32_t *x = static_cast<const uint32_t *>(X), *g = static_cast<const uint32_t *>(gate);
    if (f == 65)
        return launch_trimmed_net<65, false>(x, d, ld, row_index, f, b, static_cast<uint32_t *>(out),
                                             g, gate_n, (hipStream_t)stream);
    return launch_trimmed_net<65, true>(x, d, ld, row_index, f, b, static_cast<uint32_t *>(out), g,
                                        gate_n, (hipStream_t)stream);
}
#endif

// the 169-wire networks (MOLS over F_13 and, padded, 121 < f < 169), a build part each
#if BYZ_IN_PART(8)
int byz_internal_launch_trimmed_mean_169(const void *X, long long d, long long ld,
                                         const int *row_index, int f, int b, void *out,
                                         const void *gate, int gate_n, void *stream) {
    return launch_trimmed_net<169, false>(static_cast<const uint32_t *>(X), d, ld, row_index, f, b,
                                          static_cast<uint32_t *>(out),
                                          static_cast<const uint32_t *>(gate), gate_n,
                                          (hipStream_t)stream);
}
#endif
#if BYZ_IN_PART(10)
int byz_internal_launch_trimmed_mean_169_padded(const void *X, long long d, long long ld,
                                                const int *row_index, int f, int b, void *out,
                                                const void *gate, int gate_n, void *stream) {
    return launch_trimmed_net<169, true>(static_cast<const uint32_t *>(X), d, ld, row_index, f, b,
                                         static_cast<uint32_t *>(out),
                                         static_cast<const uint32_t *>(gate), gate_n,
                                         (hipStream_t)stream);
}
#endif
#if BYZ_IN_PART(9)
int byz_internal_launch_median_169(const void *X, long long d, long long ld, const int *row_index,
                                   int f, void *out, const void *gate, int gate_n, void *stream) {
    return launch_median_large<169, false>(static_cast<const uint32_t *>(X), d, ld, row_index, f,
                                           static_cast<uint32_t *>(out),
                                           static_cast<const uint32_t *>(gate), gate_n,
                                           (hipStream_t)stream);
}
#endif
#if BYZ_IN_PART(11)
int byz_internal_launch_median_169_padded(const void *X, long long d, long long ld,
                                          const int *row_index, int f, void *out, const void *gate,
                                          int gate_n, void *stream) {
    return launch_median_large<169, true>(static_cast<const uint32_t *>(X), d, ld, row_index, f,
                                          static_cast<uint32_t *>(out),
                                          static_cast<const uint32_t *>(gate), gate_n,
                                          (hipStream_t)stream);
}
#endif

// more than 169 rows: the two-wave kernels, median for 169 < f <= 255, trimmed mean for
// 169 < f <= 256 (it also takes even f); a build part each
#if BYZ_IN_PART(16)
int byz_internal_launch_median_255_padded(const void *X, long long d, long long ld,
                                          const int *row_index, int f, void *out, const void *gate,
                                          int gate_n, void *stream) {
    if (d <= 0) return BYZ_OK;
    if (f <= 128 || f > 255) return BYZ_EINTERNAL;
    const unsigned g = (unsigned)((d + 63) / 64);
    const uint32_t *x = static_cast<const uint32_t *>(X), *gt = static_cast<const uint32_t *>(gate);
    uint32_t *o = static_cast<uint32_t *>(out);
    hipStream_t s = (hipStream_t)stream;
    // the smallest pair of halves that holds f rows
    if (f <= 2 * 96 - 1)
        median_halves_kernel<96><<<g, 128, 0, s>>>(x, d, ld, row_index, f, o, gt, gate_n);
    else if (f <= 2 * 112 - 1)
        median_halves_kernel<112><<<g, 128, 0, s>>>(x, d, ld, row_index, f, o, gt, gate_n);
    else
        median_halves_kernel<128><<<g, 128, 0, s>>>(x, d, ld, row_index, f, o, gt, gate_n);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}
#endif
#if BYZ_IN_PART(17)
int byz_internal_launch_trimmed_mean_256_padded(const void *X, long long d, long long ld,
                                                const int *row_index, int f, int b, void *out,
                                                const void *gate, int gate_n, void *stream) {
    if (d <= 0) return BYZ_OK;
    if (f <= 128 || f > 256) return BYZ_EINTERNAL;
    const unsigned g = (unsigned)((d + 63) / 64);
    const uint32_t *x = static_cast<const uint32_t *>(X), *gt = static_cast<const uint32_t *>(gate);
    uint32_t *o = static_cast<uint32_t *>(out);
    hipStream_t s = (hipStream_t)stream;
    // the smallest pair of halves that holds f rows
    if (f <= 2 * 96)
        trimmed_halves_kernel<96><<<g, 128, 0, s>>>(x, d, ld, row_index, f, b, o, gt, gate_n);
    else if (f <= 2 * 112)
        trimmed_halves_kernel<112><<<g, 128, 0, s>>>(x, d, ld, row_index, f, b, o, gt, gate_n);
    else
        trimmed_halves_kernel<128><<<g, 128, 0, s>>>(x, d, ld, row_index, f, b, o, gt, gate_n);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}
#endif

#if BYZ_IN_PART(6)
int byz_internal_launch_trimmed_mean(const void *X, long long d, long long ld,
                                     const int *row_index, int f, int b, void *out,
                                     const void *gate, int gate_n, void *stream) {
    return launch_trimmed_mean(static_cast<const uint32_t *>(X), d, ld, row_index, f, b,
                               static_cast<uint32_t *>(out), static_cast<const uint32_t *>(gate),
                               gate_n, (hipStream_t)stream);
}
#endif

// ------------------------------------------------- single-pass launchers, one group per part

#if BYZ_IN_PART(1)
int byz_internal_launch_single_pass_1(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    const uint32_t *x = static_cast<const uint32_t *>(X);
    AggWorkspace *w = static_cast<AggWorkspace *>(ws);
    uint32_t *o = static_cast<uint32_t *>(out);
    hipStream_t s = (hipStream_t)stream;
    if (f == 9 && r == 3) return launch_fused<9, 3>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 15 && r == 3) return launch_fused<15, 3>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 21 && r == 3) return launch_fused<21, 3>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 25 && r == 3) return launch_fused<25, 3>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 25 && r == 5) return launch_fused<25, 5>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 35 && r == 5) return launch_fused<35, 5>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(2)
int byz_internal_launch_single_pass_2(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    const uint32_t *x = static_cast<const uint32_t *>(X);
    AggWorkspace *w = static_cast<AggWorkspace *>(ws);
    uint32_t *o = static_cast<uint32_t *>(out);
    hipStream_t s = (hipStream_t)stream;
    if (f == 49 && r == 3) return launch_fused<49, 3>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 49 && r == 5) return launch_fused<49, 5>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    if (f == 49 && r == 7) return launch_fused<49, 7>(x, d, ld, rows, w, o, probe_opts, trim_b, s);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(3)
int byz_internal_launch_single_pass_3(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    if (f == 81 && r == 3)
        return launch_fused<81, 3>(static_cast<const uint32_t *>(X), d, ld, rows,
                                   static_cast<AggWorkspace *>(ws), static_cast<uint32_t *>(out),
                                   probe_opts, trim_b, (hipStream_t)stream);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(4)
int byz_internal_launch_single_pass_4(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    if (f == 121 && r == 3)
        return launch_fused<121, 3>(static_cast<const uint32_t *>(X), d, ld, rows,
                                    static_cast<AggWorkspace *>(ws), static_cast<uint32_t *>(out),
                                    probe_opts, trim_b, (hipStream_t)stream);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(7)
int byz_internal_launch_single_pass_5(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    if (f == 169 && r == 3)
        return launch_fused<169, 3, false>(static_cast<const uint32_t *>(X), d, ld, rows,
                                    static_cast<AggWorkspace *>(ws), static_cast<uint32_t *>(out),
                                    probe_opts, trim_b, (hipStream_t)stream);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(18)
// (169, 3) with the trimmed mean: the widest sorting network in the single pass, a part of its own
int byz_internal_launch_single_pass_8(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    if (f == 169 && r == 3)
        return launch_fused<169, 3, true, false>(static_cast<const uint32_t *>(X), d, ld, rows,
                                    static_cast<AggWorkspace *>(ws), static_cast<uint32_t *>(out),
                                    probe_opts, trim_b, (hipStream_t)stream);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(14)
int byz_internal_launch_single_pass_6(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    if (f == 63 && r == 7)
        return launch_fused<63, 7>(static_cast<const uint32_t *>(X), d, ld, rows,
                                    static_cast<AggWorkspace *>(ws), static_cast<uint32_t *>(out),
                                    probe_opts, trim_b, (hipStream_t)stream);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(15)
int byz_internal_launch_single_pass_7(int f, int r, const void *X, long long d, long long ld,
                                      const int *rows, void *ws, void *out, int probe_opts, int trim_b,
                                      void *stream) {
    if (f == 65 && r == 5)
        return launch_fused<65, 5>(static_cast<const uint32_t *>(X), d, ld, rows,
                                    static_cast<AggWorkspace *>(ws), static_cast<uint32_t *>(out),
                                    probe_opts, trim_b, (hipStream_t)stream);
    return BYZ_EINTERNAL;
}
#endif

#if BYZ_IN_PART(0)

// ---------------------------------------------------------------------------- C-ABI

// which: 0 = before, 1 = after the dominant kernel of an aggregation on `stream`
int byz_internal_profile_mark(int which, void *stream) {
    if (g_prof.count >= g_prof.capacity) return BYZ_OK;
    if (which == 0) {
        BYZ_HIP(hipEventRecord(g_prof.start[g_prof.count], (hipStream_t)stream));
    } else {
        BYZ_HIP(hipEventRecord(g_prof.stop[g_prof.count], (hipStream_t)stream));
        ++g_prof.count;
    }
    return BYZ_OK;
}

int byz_internal_launch_bulyan_mean(const float *rows_base, long long d, long long ld,
                                    const int *selected_rows_dev, int f, int theta, int beta,
                                    float *out, void *stream) {
    if (d == 0) return BYZ_OK;
    if (f < 1 || f > BYZ_MAX_F_KRUM || theta < 1 || theta > f || (theta % 2) == 0 || beta < 1 ||
        beta > theta)
        return BYZ_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t *X = reinterpret_cast<const uint32_t *>(rows_base);
    uint32_t *O = reinterpret_cast<uint32_t *>(out);
    if (d >= kVec) {
        // the smallest generated network that holds the theta chosen rows
        if (theta <= 9) return launch_bulyan_net<9>(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 15) return launch_bulyan_net<15>(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 21) return launch_bulyan_net<21>(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 25) return launch_bulyan_net<25>(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 35) return launch_bulyan_net<35>(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 49) return launch_bulyan_net<49>(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 81)
            return byz_internal_launch_bulyan_mean_81(X, d, ld, selected_rows_dev, theta, beta, O, s);
        if (theta <= 121)
            return byz_internal_launch_bulyan_mean_121(X, d, ld, selected_rows_dev, theta, beta, O, s);
    }
    const size_t lds = (size_t)theta * kBlock * 4;
    if (lds > 64 * 1024)
        BYZ_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&bulyan_mean_generic_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    bulyan_mean_generic_kernel<<<blocks_for(d), kBlock, lds, s>>>(
        X, d, ld, selected_rows_dev, theta, beta, O);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

extern "C" int byz_last_hip_error(void) { return g_last_hip_error; }

void byz_internal_set_hip_error(int code) { g_last_hip_error = code; }

extern "C" int byz_vote(const float *copies, int64_t d, int64_t ld, const int32_t *file_rows_dev,
                        int f, int r, int32_t *winner_replica, int32_t *winner_row,
                        uint32_t *pair_neq, void *stream) {
    int rc = check_common(copies, d, ld, file_rows_dev, f, r);
    if (rc != BYZ_OK) return rc;
    if (winner_replica == nullptr || winner_row == nullptr || pair_neq == nullptr)
        return BYZ_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t *X = reinterpret_cast<const uint32_t *>(copies);
    fill_u32_kernel<<<1, kWide, 0, s>>>(pair_neq, f, 0u);
    BYZ_HIP(hipGetLastError());
    if (d > 0) {
        rc = launch_vote_pairs_r(r, X, d, ld, file_rows_dev, f, pair_neq, nullptr, 0, nullptr, s);
        if (rc != BYZ_OK) return rc;
    }
    vote_decide_kernel<<<1, kWide, 0, s>>>(pair_neq, file_rows_dev, f, r, winner_replica,
                                               winner_row);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

extern "C" int byz_vote_tolerant(const float *copies, int64_t d, int64_t ld,
                                 const int32_t *file_rows_dev, int f, int r, float atol, float rtol,
                                 int32_t *winner_replica, int32_t *winner_row, uint32_t *pair_far,
                                 void *stream) {
    int rc = check_common(copies, d, ld, file_rows_dev, f, r);
    if (rc != BYZ_OK) return rc;
    if (winner_replica == nullptr || winner_row == nullptr || pair_far == nullptr)
        return BYZ_EINVAL;
    if (!(atol >= 0.0f) || !(rtol >= 0.0f)) return BYZ_EINVAL;  // also rejects NaN
    hipStream_t s = (hipStream_t)stream;
    const uint32_t *X = reinterpret_cast<const uint32_t *>(copies);
    fill_u32_kernel<<<1, kWide, 0, s>>>(pair_far, f, 0u);
    BYZ_HIP(hipGetLastError());
    if (d > 0) {
        rc = launch_vote_pairs_tolerant(r, X, d, ld, file_rows_dev, f, atol, rtol, pair_far, s);
        if (rc != BYZ_OK) return rc;
    }
    vote_decide_kernel<<<1, kWide, 0, s>>>(pair_far, file_rows_dev, f, r, winner_replica,
                                           winner_row);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

extern "C" int byz_median(const float *rows_base, int64_t d, int64_t ld,
                          const int32_t *row_index_dev, int f, float *out, void *stream) {
    if (rows_base == nullptr || row_index_dev == nullptr || (out == nullptr && d > 0))
        return BYZ_EINVAL;
    if (d < 0 || ld < d || d > kMaxCoords) return BYZ_EINVAL;
    if (f < 1 || f > kWide) return BYZ_EINVAL;
    if ((f % 2) == 0) return BYZ_EUNSUPPORTED;
    return byz_internal_launch_median(rows_base, d, ld, row_index_dev, f, out, nullptr, 0, stream);
}

extern "C" int byz_trimmed_mean(const float *rows_base, int64_t d, int64_t ld,
                                const int32_t *row_index_dev, int f, int b, float *out,
                                void *stream) {
    if (rows_base == nullptr || row_index_dev == nullptr || (out == nullptr && d > 0))
        return BYZ_EINVAL;
    if (d < 0 || ld < d || d > kMaxCoords) return BYZ_EINVAL;
    if (f < 1 || f > kWide || b < 0 || 2 * b >= f) return BYZ_EINVAL;
    if (d == 0) return BYZ_OK;
    return byz_internal_launch_trimmed_mean(rows_base, d, ld, row_index_dev, f, b, out, nullptr, 0,
                                            stream);
}

extern "C" size_t byz_aggregate_workspace_bytes(int f, int r) {
    if (f < 1 || f > kWide || r < 3 || r > BYZ_MAX_R || (r % 2) == 0) return 0;
    return sizeof(AggWorkspace);
}

extern "C" int byz_aggregate_has_single_pass(int f, int r) { return has_fused(f, r) ? 1 : 0; }

// byz_aggregate_opts after its workspace has been settled: validates the rest and enqueues
// the launches.  ws is device memory of sizeof(AggWorkspace) bytes, 256-byte aligned.
static int aggregate_on_workspace(const float *copies, int64_t d, int64_t ld,
                                  const int32_t *file_rows_dev, int f, int r, float *out,
                                  int32_t *winner_replica, AggWorkspace *ws, unsigned flags,
                                  void *stream) {
    if ((flags & ~(unsigned)(BYZ_AGG_EARLY_MAJORITY | BYZ_AGG_TRIMMED_MEAN | 0xFFFFFF00u)) != 0)
        return BYZ_EINVAL;
    // what the probe needs to know: bit 0 early-majority mode, bits 16..31 the sample shift
    const int probe_opts = (int)((flags & BYZ_AGG_EARLY_MAJORITY) | (flags & 0xFFFF0000u));
    // trim_b < 0: median; otherwise trimmed mean dropping trim_b values at each end
    const int trim_b = (flags & BYZ_AGG_TRIMMED_MEAN) != 0 ? (int)((flags >> 8) & 0xFFu) : -1;
    if (trim_b < 0 && (flags & 0xFF00u) != 0) return BYZ_EINVAL;
    if (trim_b >= 0 && 2 * trim_b >= f) return BYZ_EINVAL;
    int rc = check_common(copies, d, ld, file_rows_dev, f, r);
    if (rc != BYZ_OK) return rc;
    if ((out == nullptr && d > 0) || ws == nullptr) return BYZ_EINVAL;
    if ((f % 2) == 0) return BYZ_EUNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t *X = reinterpret_cast<const uint32_t *>(copies);
    uint32_t *O = reinterpret_cast<uint32_t *>(out);

    if (!has_fused(f, r) || d < kVec || (trim_b >= 0 && !has_fused_trim(f, r))) {
        // two-step path, unconditionally: vote, then median over the winners
        reset_workspace_kernel<<<1, kWide, 0, s>>>(ws, (uint32_t)BYZ_PATH_TWO_STEP);
        BYZ_HIP(hipGetLastError());
        if (d > 0) {
            rc = byz_internal_profile_mark(0, s);
            if (rc != BYZ_OK) return rc;
            rc = launch_vote_pairs_r(r, X, d, ld, file_rows_dev, f, ws->pair_neq, nullptr, 0, nullptr, s);
            if (rc != BYZ_OK) return rc;
            rc = byz_internal_profile_mark(1, s);
            if (rc != BYZ_OK) return rc;
        }
        vote_decide_kernel<<<1, kWide, 0, s>>>(ws->pair_neq, file_rows_dev, f, r, winner_replica,
                                               ws->winner_row);
        BYZ_HIP(hipGetLastError());
        if (trim_b >= 0)
            return byz_internal_launch_trimmed_mean(X, d, ld, ws->winner_row, f, trim_b, O, nullptr,
                                                    0, s);
        return byz_internal_launch_median(X, d, ld, ws->winner_row, f, O, nullptr, 0, s);
    }

    // probe -> single pass -> decision (one block) -> median, which returns at once unless the
    // decision found a file whose slot 0 did not hold its winner.  Early-majority mode adds the
    // gated vote kernel and its decision between the two, for the files whose r' copies differ.
    if (f == 169 && trim_b >= 0)
        rc = byz_internal_launch_single_pass_8(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else if (f == 169)
        rc = byz_internal_launch_single_pass_5(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else if (f == 121)
        rc = byz_internal_launch_single_pass_4(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else if (f == 81)
        rc = byz_internal_launch_single_pass_3(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else if (f == 63)
        rc = byz_internal_launch_single_pass_6(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else if (f == 65)
        rc = byz_internal_launch_single_pass_7(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else if (f == 49)
        rc = byz_internal_launch_single_pass_2(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    else
        rc = byz_internal_launch_single_pass_1(f, r, X, d, ld, file_rows_dev, ws, O, probe_opts, trim_b, s);
    if (rc != BYZ_OK) return rc;
    single_pass_decide_kernel<<<1, kWide, 0, s>>>(ws, file_rows_dev, f, r, winner_replica);
    BYZ_HIP(hipGetLastError());
    if ((flags & BYZ_AGG_EARLY_MAJORITY) != 0) {
        rc = launch_vote_pairs_r(r, X, d, ld, file_rows_dev, f, ws->pair_neq, &ws->need_revote, 1,
                                 ws->revote_file, s);
        if (rc != BYZ_OK) return rc;
        revote_decide_kernel<<<1, kWide, 0, s>>>(ws, file_rows_dev, f, r, winner_replica);
        BYZ_HIP(hipGetLastError());
    }
    if (trim_b >= 0)
        return byz_internal_launch_trimmed_mean(X, d, ld, ws->winner_row, f, trim_b, O,
                                                &ws->need_median, 1, s);
    return byz_internal_launch_median(X, d, ld, ws->winner_row, f, O, &ws->need_median, 1, s);
}

extern "C" int byz_aggregate_opts(const float *copies, int64_t d, int64_t ld,
                                  const int32_t *file_rows_dev, int f, int r, float *out,
                                  int32_t *winner_replica, void *workspace, size_t workspace_bytes,
                                  unsigned flags, void *stream) {
    if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0) return BYZ_EINVAL;
    // the reasons that come before "workspace too small" keep their codes
    const int rc = check_common(copies, d, ld, file_rows_dev, f, r);
    if (rc != BYZ_OK) return rc;
    if (workspace_bytes < sizeof(AggWorkspace)) return BYZ_ENOMEM;
    return aggregate_on_workspace(copies, d, ld, file_rows_dev, f, r, out, winner_replica,
                                  reinterpret_cast<AggWorkspace *>(workspace), flags, stream);
}

extern "C" int byz_aggregate(const float *copies, int64_t d, int64_t ld,
                             const int32_t *file_rows_dev, int f, int r, float *out,
                             int32_t *winner_replica, void *workspace, size_t workspace_bytes,
                             void *stream) {
    return byz_aggregate_opts(copies, d, ld, file_rows_dev, f, r, out, winner_replica, workspace,
                              workspace_bytes, 0u, stream);
}

// Scratch of byz_aggregate_static: one AggWorkspace per GPU, part of the loaded code object
// (so it is there without any allocation) and held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; what the kernels get is the device
// address that call returns, looked up once per device.
constexpr size_t kStaticScratchBytes = 24 * 1024;
static_assert(sizeof(AggWorkspace) <= kStaticScratchBytes, "byz_aggregate_static's scratch");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

extern "C" int byz_aggregate_static(const float *copies, int64_t d, int64_t ld,
                                    const int32_t *file_rows_dev, int f, int r, float *out,
                                    int32_t *winner_replica, unsigned flags, void *stream) {
    // sizes first: what the fixed scratch cannot hold is refused before anything else happens
    if (f > kWide || r > BYZ_MAX_R) return BYZ_ENOMEM;
    int dev = -1;
    BYZ_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return BYZ_EUNSUPPORTED;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        // first call on this device (which is current): every GPU has its own copy of the array
        BYZ_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr || ((uintptr_t)ptr & 255u) != 0) return BYZ_EINTERNAL;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    return aggregate_on_workspace(copies, d, ld, file_rows_dev, f, r, out, winner_replica,
                                  static_cast<AggWorkspace *>(ptr), flags, stream);
}

extern "C" int byz_calibration_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (src == nullptr || dst == nullptr || bytes == 0 || (bytes % 16) != 0) return BYZ_EINVAL;
    if ((((uintptr_t)src | (uintptr_t)dst) & 3u) != 0 || bytes > ((size_t)1 << 40)) return BYZ_EINVAL;
    const int64_t n_vec = (int64_t)(bytes / 16);
    calibration_copy_kernel<<<blocks_for(n_vec), kBlock, 0, (hipStream_t)stream>>>(
        reinterpret_cast<const uint32_t *>(src), reinterpret_cast<uint32_t *>(dst), n_vec);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

extern "C" int byz_calibration_read_rows(const void *rows_base, int64_t d, int64_t ld, int n_rows,
                                         void *out, int store, void *stream) {
    if (rows_base == nullptr || out == nullptr || d < 4 || ld < d || d > kMaxCoords) return BYZ_EINVAL;
    if (n_rows < 1 || n_rows > kWide * BYZ_MAX_R) return BYZ_EINVAL;
    if ((((uintptr_t)rows_base | (uintptr_t)out) & 3u) != 0) return BYZ_EINVAL;
    const int64_t n_vec = d / 4;
    calibration_read_rows_kernel<<<blocks_for(n_vec), kBlock, 0, (hipStream_t)stream>>>(
        reinterpret_cast<const uint32_t *>(rows_base), n_vec, ld, n_rows,
        reinterpret_cast<uint32_t *>(out), store);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
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

extern "C" int byz_aggregate_path(const void *workspace, int *path, void *stream) {
    if (workspace == nullptr || path == nullptr) return BYZ_EINVAL;
    const AggWorkspace *ws = reinterpret_cast<const AggWorkspace *>(workspace);
    uint32_t v = 0;
    hipStream_t s = (hipStream_t)stream;
    BYZ_HIP(hipMemcpyAsync(&v, &ws->path, sizeof(v), hipMemcpyDeviceToHost, s));
    BYZ_HIP(hipStreamSynchronize(s));
    *path = (int)v;
    return BYZ_OK;
}

#endif  // part 0
