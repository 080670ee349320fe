// Multi-Krum on the vote winners (gfx950).  The ByzShield paper pairs its vote with the
// coordinate-wise median and names Multi-Krum and Bulyan as aggregators that can take the
// median's place (Sec. 6.1, Sec. 7); it defines neither, so this file follows the published
// rule: with f vectors of which c may be Byzantine (f >= 2c + 3, the requirement quoted in
// Sec. 6.1), the score of vector i is the sum of its f - c - 2 smallest squared distances to
// other vectors; the m vectors of lowest score are averaged.
//
// The pairwise squared distances come from the Gram matrix G = W W^T of the f x d matrix of
// winners: the one dense contraction of the whole path, done with fp32 MFMA tiles
// (v_mfma_f32_16x16x4f32; only the tiles on and above the diagonal of the symmetric matrix,
// so f = 25 costs 3 tiles of 16x16 instead of one padded 32x32).  A block stages a
// 256-coordinate chunk of all f rows in LDS (global loads stay 1 KiB-contiguous per wave), each
// of its four waves multiplies 64 of those coordinates, and the blocks walk the chunks
// grid-stride.  Per-block partial tiles are added in fp64 in block order, so the result does
// not depend on scheduling.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "byz_internal.h"
#include "byzshield.h"

namespace {

#define BYZ_HIP(call)                              \
    do {                                           \
        hipError_t e_ = (call);                    \
        if (e_ != hipSuccess) {                    \
            byz_internal_set_hip_error((int)e_);   \
            return BYZ_EDEVICE;                    \
        }                                          \
    } while (0)

constexpr int kBlock = 256;            // 4 waves
constexpr int kChunk = 256;            // coordinates staged per block and step
constexpr int kStride = kChunk + 4;    // row pitch in LDS: rows stay 16-byte aligned (one 16-byte
                                       // staging write per lane); see the column swizzle below
constexpr int kGramBlocks = 512;       // partial Gram tiles (2 blocks per CU; 1024: 4 % faster, reduction 3 us slower)
constexpr int kTile = 16 * 16;         // outputs of one MFMA tile
constexpr int kMaxKrum = BYZ_MAX_F_KRUM;  // most vectors Multi-Krum takes (Bulyan: BYZ_MAX_F)
constexpr int kMaxNT = kMaxKrum / 16;  // row tiles of the largest matrix
constexpr int kMaxPairs = kMaxNT * (kMaxNT + 1) / 2;  // tiles on and above the diagonal

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Row tiles of 16 the Gram matrix of f vectors is computed with (the compiled kernels have
// 1, 2, 3, 4, 6 or 8); the tiles on and above the diagonal are stored.
__host__ __device__ constexpr int row_tiles(int f) {
    return f <= 64 ? (f + 15) / 16 : (f <= 96 ? 6 : 8);
}

// Tile (ti, tj), ti <= tj < nt, of the upper triangle, numbered row by row.
__host__ __device__ constexpr int tile_pair(int nt, int ti, int tj) {
    return ti * nt - ti * (ti - 1) / 2 + (tj - ti);
}

// The 16x16 MFMA result: accumulator register v of lane l holds row 4*(l/16) + v, column l%16
// (gram_at below inverts this).

// Partial Gram tiles of the rows row_index[0..f-1] over this block's chunks.
// NT = ceil(f / 16) row tiles; RW = rows a wave stages per chunk (rows wave, wave+4, ...):
// ceil(f / 4) rounded up to a compiled value.  partial: [gridDim.x][pairs][256] floats,
// position v*64 + lane, pairs = NT(NT+1)/2.
// Per chunk: the rows' 16-byte loads for the NEXT chunk are issued, then the current chunk
// (already in registers) goes to LDS, is multiplied, and the loop turns: global latency hides
// behind the matrix instructions.
template <int NT, int RW>
__global__ __launch_bounds__(kBlock) void gram_partial_kernel(const float *__restrict__ X, int64_t d,
                                                              int64_t ld,
                                                              const int32_t *__restrict__ row_index,
                                                              int f, float *__restrict__ partial) {
    extern __shared__ float T[];  // [16*NT][kStride]; rows >= f stay zero
    constexpr int NP = NT * (NT + 1) / 2;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int i = tid; i < (16 * NT - f) * kStride; i += kBlock) T[f * kStride + i] = 0.0f;
    f32x4 acc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    const int64_t n_chunks = (d + kChunk - 1) / kChunk;

    // this wave's rows; slots past f repeat the last row (loaded, never stored).  The widest
    // shapes keep row numbers instead of pointers: half the registers, one multiply per load.
    constexpr bool kRowNumbers = RW > 24;
    const float *rowp[kRowNumbers ? 1 : RW];
    int32_t rown[kRowNumbers ? RW : 1];
#pragma unroll
    for (int t = 0; t < RW; ++t) {
        const int j = wave + 4 * t;
        const int32_t row = row_index[j < f ? j : f - 1];
        if constexpr (kRowNumbers)
            rown[t] = row;
        else
            rowp[t] = X + (int64_t)row * ld + 4 * lane;
    }
    auto row_ptr = [&](int t) -> const float * {
        if constexpr (kRowNumbers)
            return X + (int64_t)rown[t] * ld + 4 * lane;
        else
            return rowp[t];
    };
    float reg[RW][4];
    auto fetch = [&](int64_t chunk) {
        const int64_t c0 = chunk * kChunk + 4 * lane;
        if ((chunk + 1) * kChunk <= d) {  // whole chunk inside the row: branch-free loads
#pragma unroll
            for (int t = 0; t < RW; ++t) {
                const f32x4u v = __builtin_nontemporal_load(
                    reinterpret_cast<const f32x4u *>(row_ptr(t) + chunk * kChunk));
                reg[t][0] = v[0]; reg[t][1] = v[1]; reg[t][2] = v[2]; reg[t][3] = v[3];
            }
        } else {  // the ragged last chunk: missing coordinates count as zero
#pragma unroll
            for (int t = 0; t < RW; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    reg[t][e] = c0 + e < d ? row_ptr(t)[chunk * kChunk + e] : 0.0f;
        }
    };

    int64_t chunk = blockIdx.x;
    if (chunk < n_chunks) fetch(chunk);
    for (; chunk < n_chunks; chunk += gridDim.x) {
#pragma unroll
        for (int t = 0; t < RW; ++t) {
            const int j = wave + 4 * t;
            if (j < f) {
                // column c of row j lives at c ^ 2 if bit 3 of j is set: with pitch 260 the 32
                // lanes an operand read serves per cycle (rows 0..15, k = 0,1 or 2,3) then hit
                // bank 4*(row % 8) + (k ^ 2*(row / 8)), all different
                f32x4 *dst = reinterpret_cast<f32x4 *>(T + j * kStride + 4 * lane);
                const bool swz = (j & 8) != 0;
                f32x4 v;
                v[0] = swz ? reg[t][2] : reg[t][0];
                v[1] = swz ? reg[t][3] : reg[t][1];
                v[2] = swz ? reg[t][0] : reg[t][2];
                v[3] = swz ? reg[t][1] : reg[t][3];
                *dst = v;
            }
        }
        __syncthreads();
        if (chunk + gridDim.x < n_chunks) fetch(chunk + gridDim.x);
        // wave w multiplies coordinates [64w, 64w+64) of the chunk, four per MFMA: lane l holds
        // A[row = l%16][k = l/16], which is also B[k][col = l%16] of the transposed operand
        const float *t0 = T + (lane & 15) * kStride + wave * 64 + ((lane >> 4) ^ ((lane & 8) >> 2));
        constexpr int SB = NT > 6 ? 2 : (NT > 4 ? 4 : 8);  // steps whose operands are read ahead of their MFMAs
#pragma unroll
        for (int s0 = 0; s0 < 16; s0 += SB) {
            float x[NT][SB];
#pragma unroll
            for (int s = 0; s < SB; ++s)
#pragma unroll
                for (int t = 0; t < NT; ++t) x[t][s] = t0[16 * t * kStride + 4 * (s0 + s)];
#pragma unroll
            for (int s = 0; s < SB; ++s)
#pragma unroll
                for (int ti = 0; ti < NT; ++ti)
#pragma unroll
                    for (int tj = ti; tj < NT; ++tj)
                        acc[tile_pair(NT, ti, tj)] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                            x[ti][s], x[tj][s], acc[tile_pair(NT, ti, tj)], 0, 0, 0);
        }
        __syncthreads();
    }
    // add the four waves' tiles through LDS (the staging tile is free now), then store:
    // ((wave 0 + wave 1) + wave 2) + wave 3 either way
    float *red = T;
    float *dst = partial + (int64_t)blockIdx.x * NP * kTile;
    if constexpr (4 * NP * kTile <= 16 * NT * kStride) {  // [4][NP][256] floats fit the tile
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[(wave * NP + p) * kTile + v * 64 + lane] = acc[p][v];
        __syncthreads();
        for (int i = tid; i < NP * kTile; i += kBlock)
            dst[i] = ((red[i] + red[NP * kTile + i]) + red[2 * NP * kTile + i]) + red[3 * NP * kTile + i];
    } else {  // one [NP][256] array, the waves add their tiles in turn
        for (int w = 0; w < 4; ++w) {
            if (wave == w) {
#pragma unroll
                for (int p = 0; p < NP; ++p)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float *cell = red + p * kTile + v * 64 + lane;
                        *cell = w == 0 ? acc[p][v] : *cell + acc[p][v];
                    }
            }
            __syncthreads();
        }
        for (int i = tid; i < NP * kTile; i += kBlock) dst[i] = red[i];
    }
}

// gram[t][pos] = sum over blocks of partial[block][t][pos] in fp64, in a fixed order: thread
// (pos, g) adds the blocks g, g+8, g+16, ... one by one, then the eight group sums are added
// in order.  Block = 32 positions x 8 groups.
__global__ __launch_bounds__(kBlock) void gram_reduce_kernel(const float *__restrict__ partial,
                                                             int n_partial, int ntiles,
                                                             double *__restrict__ gram) {
    __shared__ double s_sum[8][32];
    const int lp = threadIdx.x & 31, g = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + lp;  // ntiles * 256 is a multiple of 32
    double acc = 0.0;
#pragma unroll 8
    for (int p = g; p < n_partial; p += 8) acc += (double)partial[(int64_t)p * ntiles * kTile + i];
    s_sum[g][lp] = acc;
    __syncthreads();
    if (g == 0) {
        double total = s_sum[0][lp];
        for (int k = 1; k < 8; ++k) total += s_sum[k][lp];
        gram[i] = total;
    }
}

__device__ inline double gram_at(const double *gram, int f, int i, int j) {
    // entry (i, j) of the symmetric matrix from the stored upper-triangle tiles
    if (i > j) { const int t = i; i = j; j = t; }
    const int nt = row_tiles(f);
    const int r = i % 16, c = j % 16;
    // row r = 4*(l/16) + v, column c = l%16  =>
    const int v = r % 4, l = c + 16 * (r / 4);
    return gram[tile_pair(nt, i / 16, j / 16) * kTile + v * 64 + l];
}

// The value lane `from` (the same for the whole wave) holds.
__device__ __forceinline__ double lane_value(double v, int from) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), from);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), from);
    return __hiloint2double(hi, lo);
}

// (key, tag) pairs of the row sort: spare keys (tag >= 256) last, else by value, then by tag.
__device__ __forceinline__ bool key_before(double a_v, int a_t, double b_v, int b_t) {
    const bool a_spare = a_t >= 256, b_spare = b_t >= 256;
    return a_spare != b_spare ? b_spare : (a_v < b_v || (a_v == b_v && a_t < b_t));
}

// Set-up of the selections, one wave per vector i (4 per block), for f <= 64*PER: the lane
// computes the squared distances d(i,j) = G_ii + G_jj - 2 G_ij (clamped at 0, exactly 0 on the
// diagonal) for j = lane and, with PER = 2, j = lane + 64, and writes them to dist_out; a
// bitonic network over the 64*PER keys of the wave then sorts the distances to the other
// vectors in ascending order (value, then index), the keys of j = i and j >= f sorting behind
// every distance.  The t-th nearest of vector i goes to sorted_dist[t*kRowStride + i] and
// sorted_nbr[t*kRowStride + i] (t < f-1; the other entries are not written).  With
// n_terms >= 0 the wave also adds the n_terms smallest distances one by one in ascending
// order from +0: the Krum score, into scores and scores_out.
constexpr int kRowStride = kMaxKrum;

template <int PER>
__global__ __launch_bounds__(kBlock) void distance_rows_kernel(const double *__restrict__ gram, int f,
                                                               int n_terms, double *dist_out,
                                                               double *__restrict__ sorted_dist,
                                                               uint8_t *__restrict__ sorted_nbr,
                                                               double *__restrict__ scores,
                                                               double *scores_out) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (i >= f) return;  // whole wave
    double v[PER];
    int tag[PER];
    const double g_ii = gram_at(gram, f, i, i);
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int j = lane + 64 * e;
        v[e] = 0.0;
        if (j < f) {
            const double dij = g_ii + gram_at(gram, f, j, j) - 2.0 * gram_at(gram, f, i, j);
            if (!(dij < 0.0) && j != i) v[e] = dij;
            if (dist_out != nullptr) dist_out[i * f + j] = v[e];
        }
        tag[e] = j | ((j >= f || j == i) ? 256 : 0);  // every key distinct
    }
#pragma unroll
    for (int k = 2; k <= 64 * PER; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j == 64) {
                // partner in the same lane; k = 128 here, so the order is ascending
                if constexpr (PER == 2) {
                    if (!key_before(v[0], tag[0], v[1], tag[1])) {
                        const double tv = v[0];
                        const int tt = tag[0];
                        v[0] = v[1];
                        tag[0] = tag[1];
                        v[1] = tv;
                        tag[1] = tt;
                    }
                }
            } else {
                const bool lower = (lane & j) == 0;
#pragma unroll
                for (int e = 0; e < PER; ++e) {
                    const double ov = __shfl_xor(v[e], j, 64);
                    const int otag = __shfl_xor(tag[e], j, 64);
                    // both lanes of a pair evaluate the same comparison (lower lane's key
                    // first), so the exchange is a permutation whatever the values are
                    const bool lo_first = lower ? key_before(v[e], tag[e], ov, otag)
                                                : key_before(ov, otag, v[e], tag[e]);
                    const bool ascending = ((lane + 64 * e) & k) == 0;
                    if (lo_first != ascending) {
                        v[e] = ov;
                        tag[e] = otag;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int t = lane + 64 * e;
        if (t < f - 1) {
            sorted_dist[t * kRowStride + i] = v[e];
            sorted_nbr[t * kRowStride + i] = (uint8_t)tag[e];
        }
    }
    if (n_terms >= 0) {
        double score = 0.0;
        for (int t = 0; t < n_terms && t < 64; ++t) score += lane_value(v[0], t);
        if constexpr (PER == 2)
            for (int t = 64; t < n_terms; ++t) score += lane_value(v[1], t - 64);
        if (lane == 0) {
            scores[i] = score;
            if (scores_out != nullptr) scores_out[i] = score;
        }
    }
}

// Multi-Krum's choice, thread i = vector i (one block of kMaxKrum threads): the m lowest
// scores, the lower index first among equal scores.
__global__ __launch_bounds__(kMaxKrum) void krum_select_kernel(const double *__restrict__ scores, int f,
                                                               int m, int32_t *selected_out,
                                                               int32_t *selected_list,
                                                               int32_t *n_selected) {
    __shared__ double s_score[kMaxKrum];
    __shared__ uint64_t s_chosen[kMaxKrum / 64];
    const int i = threadIdx.x;
    const double mine = i < f ? scores[i] : 0.0;
    s_score[i] = mine;
    __syncthreads();
    int rank = 0;
#pragma unroll 8
    for (int k = 0; k < f; ++k) {
        const double other = s_score[k];
        rank += (other < mine || (other == mine && k < i)) ? 1 : 0;
    }
    const bool chosen = i < f && rank < m;
    const uint64_t mask = __builtin_amdgcn_ballot_w64(chosen);
    if ((i & 63) == 0) s_chosen[i >> 6] = mask;
    __syncthreads();
    int before = __builtin_popcountll(mask & ((1ull << (i & 63)) - 1ull));
    int total = 0;
#pragma unroll
    for (int w = 0; w < kMaxKrum / 64; ++w) {
        const int n = __builtin_popcountll(s_chosen[w]);
        if (w < (i >> 6)) before += n;
        total += n;
    }
    if (i < f) selected_out[i] = chosen ? 1 : 0;
    if (chosen) selected_list[before] = i;
    if (i == 0) *n_selected = total;
}

// One exchange of a wave-wide search for the lowest (score, index): every lane looks at the
// lane the data-parallel-primitive pattern CTRL pairs it with (a pairing inside a row of 16
// lanes that is its own inverse) and keeps the lower of the two keys.
template <int CTRL>
__device__ __forceinline__ void argmin_exchange(double &score, int &best) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(score), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(score), CTRL, 0xF, 0xF, false);
    const int o_best = __builtin_amdgcn_update_dpp(0, best, CTRL, 0xF, 0xF, false);
    const double o_score = __hiloint2double(hi, lo);
    if (o_score < score || (o_score == score && o_best < best)) {
        score = o_score;
        best = o_best;
    }
}

// First phase of Bulyan: Krum applied again and again to the vectors not yet chosen, until
// theta = f - 2c are chosen.  Round with n' vectors left: score(i) = the n' - c - 2 smallest
// distances from i to the other vectors left, added one by one in ascending order (no terms
// when that count is <= 0); lowest score wins, lowest index among equal scores.
// One wave with lane i = vector i, on the sorted rows distance_rows_kernel left.  The lane keeps
// its sorted row in registers and, as a 64-bit mask over the positions of that row, the terms
// of its next score.  A vector left has n' - 1 others left and takes n' - c - 2 of them, so the
// terms are the others left without the c + 1 farthest; choosing a vector removes it from
// every row: where it was a term the mask just loses it, elsewhere it was one of the c + 1
// farthest and the farthest term takes its place there.  A score is then one walk over the
// mask, and the winner is the lowest (score, index) of the wave.
__global__ __launch_bounds__(64) void bulyan_select_kernel(const double *__restrict__ sorted_dist,
                                                           const uint8_t *__restrict__ sorted_nbr,
                                                           int f, int c, int32_t *selected_out,
                                                           int32_t *order_out,
                                                           int32_t *selected_list,
                                                           int32_t *n_selected,
                                                           const int32_t *__restrict__ row_index,
                                                           int32_t *selected_rows) {
    __shared__ uint8_t s_pos[BYZ_MAX_F * 64];  // [j*64 + i]: where vector j stands in i's row
    const int i = threadIdx.x;
    if (i < f) selected_out[i] = 0;
    const int theta = f - 2 * c;
    const int32_t my_row = row_index[i < f ? i : 0];  // a round then needs no load from memory
    int32_t first_row = my_row;
    // entries the set-up did not write are loaded and set aside
    constexpr int kMaxOthers = BYZ_MAX_F - 1;
    double rdist[kMaxOthers];
#pragma unroll
    for (int t = 0; t < kMaxOthers; ++t) {
        const bool have = i < f && t < f - 1;
        const double dv = sorted_dist[t * kRowStride + i];
        const uint32_t nv = sorted_nbr[t * kRowStride + i];
        rdist[t] = have ? dv : 0.0;
        if (have) s_pos[nv * 64 + i] = (uint8_t)t;
    }
    __syncthreads();
    bool left = i < f;  // not chosen yet
    uint64_t terms = left ? ((1ull << (f - c - 2)) - 1ull) : 0ull;  // f - c - 2 <= 62
    for (int round = 0; round < theta; ++round) {
        double score = left ? 0.0 : __builtin_huge_val();
        bool done = __builtin_amdgcn_ballot_w64(terms != 0) == 0;
#pragma unroll
        for (int t0 = 0; t0 < kMaxOthers; t0 += 8) {
            if (!done && t0 < f - 1) {
#pragma unroll
                for (int t = t0; t < t0 + 8 && t < kMaxOthers; ++t)
                    score += ((terms >> t) & 1ull) != 0 ? rdist[t] : 0.0;
                if (t0 + 8 < 64) done = __builtin_amdgcn_ballot_w64((terms >> (t0 + 8)) != 0) == 0;
            }
        }
        // lowest (score, index) of the wave: four exchanges inside each row of 16 lanes, then
        // the four rows are compared from their first lanes
        int best = i;
        argmin_exchange<0xB1>(score, best);   // quad_perm [1,0,3,2]: lane ^ 1
        argmin_exchange<0x4E>(score, best);   // quad_perm [2,3,0,1]: lane ^ 2
        argmin_exchange<0x141>(score, best);  // row_half_mirror: the other quad of the 8
        argmin_exchange<0x140>(score, best);  // row_mirror: the other half of the 16
        {
            double w_score = lane_value(score, 0);
            int w_best = __builtin_amdgcn_readlane(best, 0);
#pragma unroll
            for (int row = 1; row < 4; ++row) {
                const double r_score = lane_value(score, 16 * row);
                const int r_best = __builtin_amdgcn_readlane(best, 16 * row);
                if (r_score < w_score || (r_score == w_score && r_best < w_best)) {
                    w_score = r_score;
                    w_best = r_best;
                }
            }
            best = w_best;
        }
        const int32_t best_row = __shfl(my_row, best, 64);
        if (round == 0) first_row = best_row;
        if (i == 0) {
            selected_list[round] = best;
            selected_rows[round] = best_row;
            selected_out[best] = 1;
            if (order_out != nullptr) order_out[round] = best;
        }
        if (i == best) {
            left = false;
            terms = 0;
        } else if (left) {
            const uint64_t bit = 1ull << s_pos[best * 64 + i];
            if ((terms & bit) != 0)
                terms &= ~bit;
            else if (terms != 0)
                terms &= ~(1ull << (63 - __builtin_clzll(terms)));
        }
    }
    // rows of the chosen vectors for the second phase; the spare entries of the whole table
    // (the second phase's network may have more wires than this kernel has lanes) repeat the
    // first one
    for (int e = i; e < kMaxKrum; e += 64)
        if (e >= theta) selected_rows[e] = first_row;
    if (i == 0) *n_selected = theta;
}

// The same rounds for 64 < f <= kMaxKrum: one block of kMaxKrum threads, thread i = vector i.
// The sorted rows do not fit registers and stay in LDS ([t*kRowStride + i], read once per
// position of a walk), a vector's terms are a 128-bit mask, and the winner is the lower of the
// two waves' winners.  Dynamic LDS: (f-1)*kRowStride doubles, then kMaxKrum*kRowStride bytes.
__global__ __launch_bounds__(kMaxKrum) void bulyan_select_wide_kernel(
    const double *__restrict__ sorted_dist, const uint8_t *__restrict__ sorted_nbr, int f, int c,
    int32_t *selected_out, int32_t *order_out, int32_t *selected_list, int32_t *n_selected,
    const int32_t *__restrict__ row_index, int32_t *selected_rows) {
    extern __shared__ double s_rows[];
    uint8_t *s_pos = reinterpret_cast<uint8_t *>(s_rows + (f - 1) * kRowStride);  // [j*kRowStride + i]
    __shared__ double s_wave_score[kMaxKrum / 64];
    __shared__ int s_wave_best[kMaxKrum / 64];
    __shared__ int32_t s_row_of[kMaxKrum];
    const int i = threadIdx.x;
    const int theta = f - 2 * c;
    if (i < f) selected_out[i] = 0;
    s_row_of[i] = row_index[i < f ? i : 0];
    for (int t = 0; t < f - 1; ++t) {
        if (i < f) {
            s_rows[t * kRowStride + i] = sorted_dist[t * kRowStride + i];
            s_pos[sorted_nbr[t * kRowStride + i] * kRowStride + i] = (uint8_t)t;
        }
    }
    __syncthreads();
    bool left = i < f;  // not chosen yet
    // the f - c - 2 <= 125 nearest: bits 0..63 in lo, 64.. in hi
    const int k0 = f - c - 2;
    uint64_t lo = !left ? 0ull : (k0 >= 64 ? ~0ull : ((1ull << k0) - 1ull));
    uint64_t hi = !left || k0 <= 64 ? 0ull : ((1ull << (k0 - 64)) - 1ull);
    int32_t first_row = 0;
    for (int round = 0; round < theta; ++round) {
        double score = left ? 0.0 : __builtin_huge_val();
        for (int t0 = 0; t0 < f - 1; t0 += 8) {
            const uint64_t rest = t0 < 64 ? ((lo >> t0) | hi) : (hi >> (t0 - 64));
            if (__builtin_amdgcn_ballot_w64(rest != 0) == 0) break;  // this wave has its terms
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = t0 + u;  // the same for the whole block
                if (t < f - 1) {
                    const uint64_t word = t < 64 ? lo : hi;
                    const double x = s_rows[t * kRowStride + i];
                    score += ((word >> (t & 63)) & 1ull) != 0 ? x : 0.0;
                }
            }
        }
        int best = i;
        argmin_exchange<0xB1>(score, best);   // quad_perm [1,0,3,2]: lane ^ 1
        argmin_exchange<0x4E>(score, best);   // quad_perm [2,3,0,1]: lane ^ 2
        argmin_exchange<0x141>(score, best);  // row_half_mirror: the other quad of the 8
        argmin_exchange<0x140>(score, best);  // row_mirror: the other half of the 16
        double w_score = lane_value(score, 0);
        int w_best = __builtin_amdgcn_readlane(best, 0);
#pragma unroll
        for (int row = 1; row < 4; ++row) {
            const double r_score = lane_value(score, 16 * row);
            const int r_best = __builtin_amdgcn_readlane(best, 16 * row);
            if (r_score < w_score || (r_score == w_score && r_best < w_best)) {
                w_score = r_score;
                w_best = r_best;
            }
        }
        if ((i & 63) == 0) {
            s_wave_score[i >> 6] = w_score;
            s_wave_best[i >> 6] = w_best;
        }
        __syncthreads();
        best = s_wave_best[0];
        {
            double b_score = s_wave_score[0];
#pragma unroll
            for (int w = 1; w < kMaxKrum / 64; ++w) {
                const double o_score = s_wave_score[w];
                const int o_best = s_wave_best[w];
                if (o_score < b_score || (o_score == b_score && o_best < best)) {
                    b_score = o_score;
                    best = o_best;
                }
            }
        }
        const int32_t best_row = s_row_of[best];
        __syncthreads();  // the waves' winners are read before the next round replaces them
        if (round == 0) first_row = best_row;
        if (i == 0) {
            selected_list[round] = best;
            selected_rows[round] = best_row;
            selected_out[best] = 1;
            if (order_out != nullptr) order_out[round] = best;
        }
        if (i == best) {
            left = false;
            lo = 0;
            hi = 0;
        } else if (left) {
            const int p = s_pos[best * kRowStride + i];
            const uint64_t bit = 1ull << (p & 63);
            uint64_t &word = p < 64 ? lo : hi;
            if ((word & bit) != 0)
                word &= ~bit;
            else if (hi != 0)
                hi &= ~(1ull << (63 - __builtin_clzll(hi)));
            else if (lo != 0)
                lo &= ~(1ull << (63 - __builtin_clzll(lo)));
        }
    }
    // rows of the chosen vectors for the second phase; the spare entries repeat the first one
    if (i >= theta) selected_rows[i] = first_row;
    if (i == 0) *n_selected = theta;
}

// out[c] = mean of the selected rows: fp32, added one by one in ascending file index starting
// from +0, one IEEE division by the count.  Thread t owns the words from min(4t, d-4) (d >= 4).
__global__ __launch_bounds__(kBlock) void selected_mean_kernel(const float *__restrict__ X, int64_t d,
                                                               int64_t ld,
                                                               const int32_t *__restrict__ row_index,
                                                               const int32_t *__restrict__ selected_list,
                                                               const int32_t *__restrict__ n_selected,
                                                               float *__restrict__ out) {
    const int n = *n_selected;
    if (d >= 4) {
        const int64_t n_thr = (d + 3) / 4;
        const int64_t gt = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        if (gt >= n_thr) return;
        const int64_t c0 = (gt + 1) * 4 <= d ? gt * 4 : d - 4;
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
#pragma unroll 4
        for (int t = 0; t < n; ++t) {
            const float *p = X + (int64_t)row_index[selected_list[t]] * ld + c0;
            const f32x4u v = __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(p));
            a0 += v[0]; a1 += v[1]; a2 += v[2]; a3 += v[3];
        }
        const float dn = (float)n;
        f32x4u o;
        o[0] = a0 / dn; o[1] = a1 / dn; o[2] = a2 / dn; o[3] = a3 / dn;
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4u *>(out + c0));
    } else {
        const int64_t cc = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        if (cc >= d) return;
        float a = 0.0f;
        for (int t = 0; t < n; ++t) a += X[(int64_t)row_index[selected_list[t]] * ld + cc];
        out[cc] = a / (float)n;
    }
}

struct KrumWorkspace {
    double gram[kMaxPairs * kTile];
    double sorted_dist[kMaxKrum * kRowStride];  // [t*kRowStride + i]: i's t-th smallest distance
    double scores[kMaxKrum];
    uint8_t sorted_nbr[kMaxKrum * kRowStride];  // and the vector it leads to
    int32_t selected_list[kMaxKrum];
    int32_t selected_rows[kMaxKrum];  // Bulyan: rows of the chosen vectors, spare entries valid
    int32_t n_selected;
    int32_t pad[63];
    float partial[1];  // [kGramBlocks][tiles of f][256], sized by krum_workspace_bytes
};

inline int stored_tiles(int f) { return row_tiles(f) * (row_tiles(f) + 1) / 2; }

inline size_t krum_workspace_bytes(int f) {
    return offsetof(KrumWorkspace, partial) +
           sizeof(float) * (size_t)kGramBlocks * stored_tiles(f) * kTile;
}

// Gram matrix of the f rows into ws->gram (partial tiles, then the fp64 reduction).
template <int NT, int RW>
int launch_gram_shape(int grid, const float *rows_base, int64_t d, int64_t ld,
                      const int32_t *row_index_dev, int f, float *partial, hipStream_t s) {
    const size_t lds = (size_t)16 * NT * kStride * sizeof(float);
    if (lds > 64 * 1024)  // more than a kernel may use without asking
        BYZ_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&gram_partial_kernel<NT, RW>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    gram_partial_kernel<NT, RW><<<grid, kBlock, lds, s>>>(rows_base, d, ld, row_index_dev, f, partial);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

int launch_gram(const float *rows_base, int64_t d, int64_t ld, const int32_t *row_index_dev, int f,
                KrumWorkspace *ws, hipStream_t s) {
    int64_t n_chunks = (d + kChunk - 1) / kChunk;
    if (n_chunks < 1) n_chunks = 1;  // d == 0: one block writes zero tiles
    const int grid = n_chunks < kGramBlocks ? (int)n_chunks : kGramBlocks;
    // (row tiles, rows a wave stages per chunk = ceil(f / 4) rounded up to a compiled value)
    int rc;
    if (f <= 16) rc = launch_gram_shape<1, 4>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 28) rc = launch_gram_shape<2, 7>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 32) rc = launch_gram_shape<2, 8>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 36) rc = launch_gram_shape<3, 9>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 48) rc = launch_gram_shape<3, 12>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 52) rc = launch_gram_shape<4, 13>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 64) rc = launch_gram_shape<4, 16>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 84) rc = launch_gram_shape<6, 21>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else if (f <= 96) rc = launch_gram_shape<6, 24>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    else rc = launch_gram_shape<8, 32>(grid, rows_base, d, ld, row_index_dev, f, ws->partial, s);
    if (rc != BYZ_OK) return rc;
    const int ntiles = stored_tiles(f);
    gram_reduce_kernel<<<ntiles * kTile / 32, kBlock, 0, s>>>(ws->partial, grid, ntiles, ws->gram);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

// Sorted distance rows (and Krum scores when n_terms >= 0) from ws->gram.
int launch_distance_rows(int f, int n_terms, double *dist_out, double *scores_out, KrumWorkspace *ws,
                         hipStream_t s) {
    const int row_blocks = (f + kBlock / 64 - 1) / (kBlock / 64);
    if (f <= 64)
        distance_rows_kernel<1><<<row_blocks, kBlock, 0, s>>>(ws->gram, f, n_terms, dist_out,
                                                              ws->sorted_dist, ws->sorted_nbr,
                                                              ws->scores, scores_out);
    else
        distance_rows_kernel<2><<<row_blocks, kBlock, 0, s>>>(ws->gram, f, n_terms, dist_out,
                                                              ws->sorted_dist, ws->sorted_nbr,
                                                              ws->scores, scores_out);
    BYZ_HIP(hipGetLastError());
    return BYZ_OK;
}

}  // namespace

extern "C" size_t byz_multi_krum_workspace_bytes(int f) {
    if (f < 1 || f > kMaxKrum) return 0;
    return krum_workspace_bytes(f);
}

extern "C" int byz_multi_krum(const float *rows_base, int64_t d, int64_t ld,
                              const int32_t *row_index_dev, int f, int c, int m, float *out,
                              int32_t *selected_out, double *scores_out, double *dist_out,
                              void *workspace, size_t workspace_bytes, void *stream) {
    if (rows_base == nullptr || row_index_dev == nullptr || selected_out == nullptr ||
        workspace == nullptr || (out == nullptr && d > 0))
        return BYZ_EINVAL;
    if (d < 0 || ld < d || d > ((int64_t)1 << 30)) return BYZ_EINVAL;
    if (f < 3 || f > kMaxKrum || c < 0 || f < 2 * c + 3) return BYZ_EINVAL;  // Sec. 6.1
    if (m < 1 || m > f - c) return BYZ_EINVAL;
    if (((uintptr_t)workspace & 255u) != 0) return BYZ_EINVAL;
    if (workspace_bytes < krum_workspace_bytes(f)) return BYZ_ENOMEM;
    hipStream_t s = (hipStream_t)stream;
    KrumWorkspace *ws = reinterpret_cast<KrumWorkspace *>(workspace);
    int rc = launch_gram(rows_base, d, ld, row_index_dev, f, ws, s);
    if (rc != BYZ_OK) return rc;
    rc = launch_distance_rows(f, f - c - 2, dist_out, scores_out, ws, s);
    if (rc != BYZ_OK) return rc;
    krum_select_kernel<<<1, kMaxKrum, 0, s>>>(ws->scores, f, m, selected_out, ws->selected_list,
                                              &ws->n_selected);
    BYZ_HIP(hipGetLastError());
    if (d > 0) {
        const int64_t n_thr = d >= 4 ? (d + 3) / 4 : d;
        selected_mean_kernel<<<(unsigned)((n_thr + kBlock - 1) / kBlock), kBlock, 0, s>>>(
            rows_base, d, ld, row_index_dev, ws->selected_list, &ws->n_selected, out);
        BYZ_HIP(hipGetLastError());
    }
    return BYZ_OK;
}

extern "C" size_t byz_bulyan_workspace_bytes(int f) { return byz_multi_krum_workspace_bytes(f); }

extern "C" int byz_bulyan(const float *rows_base, int64_t d, int64_t ld,
                          const int32_t *row_index_dev, int f, int c, float *out,
                          int32_t *selected_out, int32_t *order_out, double *dist_out,
                          void *workspace, size_t workspace_bytes, void *stream) {
    if (rows_base == nullptr || row_index_dev == nullptr || selected_out == nullptr ||
        workspace == nullptr || (out == nullptr && d > 0))
        return BYZ_EINVAL;
    if (d < 0 || ld < d || d > ((int64_t)1 << 30)) return BYZ_EINVAL;
    if (f < 3 || f > kMaxKrum || c < 0 || f < 4 * c + 3) return BYZ_EINVAL;  // Sec. 6.1
    if ((f % 2) == 0) return BYZ_EUNSUPPORTED;  // the median of the f - 2c chosen values must be one of them
    if (((uintptr_t)workspace & 255u) != 0) return BYZ_EINVAL;
    if (workspace_bytes < krum_workspace_bytes(f)) return BYZ_ENOMEM;
    hipStream_t s = (hipStream_t)stream;
    KrumWorkspace *ws = reinterpret_cast<KrumWorkspace *>(workspace);
    int rc = launch_gram(rows_base, d, ld, row_index_dev, f, ws, s);
    if (rc != BYZ_OK) return rc;
    rc = launch_distance_rows(f, -1, dist_out, nullptr, ws, s);
    if (rc != BYZ_OK) return rc;
    if (f <= BYZ_MAX_F) {
        bulyan_select_kernel<<<1, 64, 0, s>>>(ws->sorted_dist, ws->sorted_nbr, f, c, selected_out,
                                              order_out, ws->selected_list, &ws->n_selected,
                                              row_index_dev, ws->selected_rows);
    } else {
        const size_t lds = (size_t)(f - 1) * kRowStride * sizeof(double) + (size_t)kMaxKrum * kRowStride;
        BYZ_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&bulyan_select_wide_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        bulyan_select_wide_kernel<<<1, kMaxKrum, lds, s>>>(
            ws->sorted_dist, ws->sorted_nbr, f, c, selected_out, order_out, ws->selected_list,
            &ws->n_selected, row_index_dev, ws->selected_rows);
    }
    BYZ_HIP(hipGetLastError());
    const int theta = f - 2 * c;
    return byz_internal_launch_bulyan_mean(rows_base, d, ld, ws->selected_rows, f, theta,
                                           theta - 2 * c, out, stream);
}

extern "C" int byz_mean_around_median(const float *rows_base, int64_t d, int64_t ld,
                                      const int32_t *row_index_dev, int f, int beta, float *out,
                                      void *stream) {
    if (rows_base == nullptr || row_index_dev == nullptr || (out == nullptr && d > 0))
        return BYZ_EINVAL;
    if (d < 0 || ld < d || d > ((int64_t)1 << 30)) return BYZ_EINVAL;
    if (f < 1 || f > kMaxKrum || beta < 1 || beta > f) return BYZ_EINVAL;
    if ((f % 2) == 0) return BYZ_EUNSUPPORTED;  // the median must be one of the values
    return byz_internal_launch_bulyan_mean(rows_base, d, ld, row_index_dev, f, f, beta, out, stream);
}
