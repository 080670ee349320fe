// Host side of libbyzshield: worker-file assignment graphs (Sec. 4 of the ByzShield paper)
// and the exhaustive worst-case adversary search (Sec. 5.3.2).  No GPU is touched here.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <algorithm>
#include <atomic>
#include <map>
#include <new>
#include <system_error>
#include <thread>
#include <vector>

#include "byzshield.h"
#include "byzshield_bench.h"

struct byz_assignment {
    int scheme = 0;
    int K = 0, f = 0, l = 0, r = 0;
    int class_size = 0;    // workers per parallel class (one replica of every file per class)
    int shared_lo = 0;     // two workers of different classes share between shared_lo and
    int shared_hi = 0;     // shared_hi files
    std::vector<int32_t> worker_files;  // [K][l] ascending
    std::vector<int32_t> file_workers;  // [f][r] ascending = class order
    std::vector<int32_t> file_rows;     // [f][r]
    // the files as a gx x gy grid (index x*gy + y) and the addition used on its coordinates
    // (empty: modulo gx resp. gy; else the table of F_l, gx == gy == l): what the search's
    // symmetry reduction translates the grid with
    int gx = 1, gy = 1;
    std::vector<uint8_t> add_tab;
};

namespace {

bool is_prime(int n) {
    if (n < 2) return false;
    for (int p = 2; (int64_t)p * p <= n; ++p)
        if (n % p == 0) return false;
    return true;
}

inline int mod(int64_t x, int m) {
    int64_t t = x % m;
    return (int)(t < 0 ? t + m : t);
}

// F_q for a prime power q = p^k <= 255 (Sec. 4.1.1 takes row, column and symbol sets to be
// F_l).  Element n is the polynomial whose coefficients are the base-p digits of n, lowest
// digit = constant term; products are reduced modulo the monic irreducible polynomial of degree
// k with the smallest number.  For k = 1 this is arithmetic modulo p.
struct Field {
    int q = 0, p = 0, k = 0;
    std::vector<uint8_t> add_tab, mul_tab;  // [q][q]
    int add(int a, int b) const { return add_tab[(size_t)a * q + b]; }
    int mul(int a, int b) const { return mul_tab[(size_t)a * q + b]; }
};

// Remainder of polynomial num (degree < n_num) by monic polynomial den of degree deg, over F_p.
// Coefficient vectors, lowest degree first; den has deg + 1 entries with den[deg] == 1.
void poly_rem(std::vector<int> &num, const std::vector<int> &den, int deg, int p) {
    for (int t = (int)num.size() - 1; t >= deg; --t) {
        const int c = num[t];
        if (c == 0) continue;
        for (int j = 0; j <= deg; ++j) num[t - deg + j] = mod((int64_t)num[t - deg + j] - (int64_t)c * den[j], p);
    }
    num.resize((size_t)deg);
}

bool make_field(int q, Field &F) {
    int p = 0;
    for (int c = 2; c <= q; ++c)
        if (q % c == 0) { p = c; break; }  // smallest divisor > 1 is prime
    if (p == 0) return false;
    int k = 0, t = q;
    while (t % p == 0) { t /= p; ++k; }
    if (t != 1) return false;
    F.q = q; F.p = p; F.k = k;
    auto digits = [&](int n, int len) {
        std::vector<int> c((size_t)len, 0);
        for (int i = 0; i < len && n > 0; ++i) { c[i] = n % p; n /= p; }
        return c;
    };
    auto number = [&](const std::vector<int> &c) {
        int n = 0;
        for (int i = (int)c.size() - 1; i >= 0; --i) n = n * p + c[i];
        return n;
    };
    // modulus x^k + (digits of low): the first one with no monic divisor of degree 1..k/2
    std::vector<int> modulus;
    for (int low = 0; low < q && modulus.empty(); ++low) {
        std::vector<int> cand = digits(low, k);
        cand.push_back(1);
        bool irreducible = true;
        int count = p;  // monic polynomials of degree deg: p^deg
        for (int deg = 1; deg <= k / 2 && irreducible; ++deg, count *= p)
            for (int n = 0; n < count && irreducible; ++n) {
                std::vector<int> den = digits(n, deg);
                den.push_back(1);
                std::vector<int> rem = cand;
                poly_rem(rem, den, deg, p);
                bool zero = true;
                for (int c : rem) zero = zero && c == 0;
                if (zero) irreducible = false;
            }
        if (irreducible) modulus = cand;
    }
    if (modulus.empty()) return false;
    F.add_tab.assign((size_t)q * q, 0);
    F.mul_tab.assign((size_t)q * q, 0);
    for (int a = 0; a < q; ++a) {
        const std::vector<int> ca = digits(a, k);
        for (int b = 0; b < q; ++b) {
            const std::vector<int> cb = digits(b, k);
            std::vector<int> sum((size_t)k), prod((size_t)(2 * k - 1), 0);
            for (int i = 0; i < k; ++i) sum[i] = (ca[i] + cb[i]) % p;
            for (int i = 0; i < k; ++i)
                for (int j = 0; j < k; ++j) prod[i + j] = (prod[i + j] + ca[i] * cb[j]) % p;
            poly_rem(prod, modulus, k, p);
            F.add_tab[(size_t)a * q + b] = (uint8_t)number(sum);
            F.mul_tab[(size_t)a * q + b] = (uint8_t)number(prod);
        }
    }
    return true;
}

// Fills per-class "which worker of class k holds file j".  All three constructions are lines
// of the affine plane over F_p (F_l for MOLS): file (x, y) belongs to the class-k worker whose
// index inside the class is the value of a linear form in (x, y).
//   MOLS, Algorithm 2: file i*l+j, class k (square L_{k+1}) -> symbol (k+1)*i + j in F_l.
//   Ramanujan Case 2 (H = B): worker a*s+u holds file b*s+v iff v = u - a*b, so file (b, v)
//     is held in class a by u = v + a*b.
//   Ramanujan Case 1 (H = B^T): worker b*s+v holds file a*s+u iff u = v + a*b, so file
//     (a, u) is held in class b by v = u - a*b.
//   FRC (the comparison assignment of Sec. 5.3.1) has no grid: class k is the k-th member of
//     every group and holds file y on its y-th worker.
int holder_in_class(int scheme, bool case2, int p, const Field &F, int k, int x, int y) {
    if (scheme == BYZ_SCHEME_FRC) return y;  // replica k of file y sits on worker k*f + y
    if (scheme == BYZ_SCHEME_MOLS) return F.add(F.mul(k + 1, x), y);
    if (case2) return mod((int64_t)y + (int64_t)k * x, p);
    return mod((int64_t)y - (int64_t)k * x, p);
}

int check_invariants(const byz_assignment &g) {
    const int K = g.K, f = g.f, l = g.l, r = g.r;
    if ((int64_t)K * l != (int64_t)f * r) return BYZ_EINTERNAL;
    std::vector<uint8_t> H((size_t)K * f, 0);
    for (int w = 0; w < K; ++w) {
        for (int t = 0; t < l; ++t) {
            int j = g.worker_files[(size_t)w * l + t];
            if (j < 0 || j >= f) return BYZ_EINTERNAL;
            if (t > 0 && g.worker_files[(size_t)w * l + t - 1] >= j) return BYZ_EINTERNAL;
            H[(size_t)w * f + j] = 1;
        }
    }
    // every file on exactly r workers, one per parallel class, listed in class order
    for (int j = 0; j < f; ++j) {
        int cnt = 0;
        for (int w = 0; w < K; ++w) cnt += H[(size_t)w * f + j];
        if (cnt != r) return BYZ_EINTERNAL;
        for (int k = 0; k < r; ++k) {
            int w = g.file_workers[(size_t)j * r + k];
            if (w < 0 || w >= K || !H[(size_t)w * f + j]) return BYZ_EINTERNAL;
            if (w / g.class_size != k) return BYZ_EINTERNAL;
            int row = g.file_rows[(size_t)j * r + k];
            if (row / l != w || g.worker_files[row] != j) return BYZ_EINTERNAL;
        }
    }
    // Latin-square / orthogonality consequences (Sec. 4.1.2): same class -> no common file,
    // different classes -> exactly one (more only for Ramanujan Case 2 with m > s)
    if ((double)K * K * f > 2e9) return BYZ_OK;  // pairwise check only where it is cheap
    for (int u = 0; u < K; ++u)
        for (int v = u + 1; v < K; ++v) {
            int common = 0;
            for (int j = 0; j < f; ++j) common += H[(size_t)u * f + j] & H[(size_t)v * f + j];
            if (u / g.class_size == v / g.class_size) {
                if (common != 0) return BYZ_EINTERNAL;
            } else if (common < g.shared_lo || common > g.shared_hi) {
                return BYZ_EINTERNAL;
            }
        }
    return BYZ_OK;
}

}  // namespace

extern "C" int byz_build_assignment(int scheme, int a, int b, byz_assignment **out) {
    if (!out) return BYZ_EINVAL;
    *out = nullptr;
    if (scheme != BYZ_SCHEME_MOLS && scheme != BYZ_SCHEME_RAMANUJAN && scheme != BYZ_SCHEME_FRC)
        return BYZ_EINVAL;
    if (a < 2 || a > 255) return BYZ_EINVAL;
    int K, f, l, r, classes, class_size, gx, gy;  // files form a gx x gy grid, index x*gy + y
    bool case2 = false;
    int shared_lo = 1, shared_hi = 1;
    Field field;
    if (scheme == BYZ_SCHEME_FRC) {
        // Sec. 5.3.1: K/r groups of r workers, every worker of a group holds the group's file
        if (b < 1 || b > a || a % b != 0) return BYZ_EINVAL;
        K = a; r = b; f = K / r; l = 1; classes = r; class_size = f; gx = 1; gy = f;
        shared_lo = 0;  // two workers share their file iff they are in the same group
    } else if (scheme == BYZ_SCHEME_MOLS) {
        if (b < 1 || b > a - 1) return BYZ_EINVAL;  // Algorithm 2 needs r <= l-1
        if (!make_field(a, field)) return BYZ_EUNSUPPORTED;  // l must be a prime power
        l = a; r = b; K = r * l; f = l * l; classes = r; class_size = l; gx = l; gy = l;
    } else {
        const int s = a, m = b;
        if (m < 2 || m > 255) return BYZ_EINVAL;
        if (!is_prime(s)) return BYZ_EUNSUPPORTED;
        if (m >= s) {  // Eq. 6, Case 2
            case2 = true;
            K = s * s; f = m * s; l = m; r = s; classes = s; class_size = s; gx = m; gy = s;
        } else {  // Eq. 6, Case 1
            K = m * s; f = s * s; l = s; r = m; classes = m; class_size = s; gx = s; gy = s;
        }
    }
    byz_assignment *g = new (std::nothrow) byz_assignment();
    if (!g) return BYZ_ENOMEM;
    try {
        g->scheme = scheme; g->K = K; g->f = f; g->l = l; g->r = r; g->class_size = class_size;
        g->gx = gx; g->gy = gy;
        if (scheme == BYZ_SCHEME_MOLS && field.k > 1) g->add_tab = field.add_tab;
        if (case2 && l > class_size) {
            g->shared_lo = l / class_size;
            g->shared_hi = (l + class_size - 1) / class_size;
        } else {
            g->shared_lo = shared_lo;
            g->shared_hi = shared_hi;
        }
        g->worker_files.assign((size_t)K * l, -1);
        g->file_workers.assign((size_t)f * r, -1);
        g->file_rows.assign((size_t)f * r, -1);
        std::vector<int> fill((size_t)K, 0);
        // files in ascending order, so each worker's list comes out ascending
        for (int x = 0; x < gx; ++x)
            for (int y = 0; y < gy; ++y) {
                const int j = x * gy + y;
                for (int k = 0; k < classes; ++k) {
                    const int w = k * class_size + holder_in_class(scheme, case2, a, field, k, x, y);
                    if (fill[w] >= l) { delete g; return BYZ_EINTERNAL; }
                    g->worker_files[(size_t)w * l + fill[w]] = j;
                    g->file_workers[(size_t)j * r + k] = w;
                    g->file_rows[(size_t)j * r + k] = w * l + fill[w];
                    ++fill[w];
                }
            }
        for (int w = 0; w < K; ++w)
            if (fill[w] != l) { delete g; return BYZ_EINTERNAL; }
        int rc = check_invariants(*g);
        if (rc != BYZ_OK) { delete g; return rc; }
    } catch (const std::bad_alloc &) {
        delete g;
        return BYZ_ENOMEM;
    }
    *out = g;
    return BYZ_OK;
}

extern "C" void byz_free_assignment(byz_assignment *g) { delete g; }

extern "C" int byz_assignment_dims(const byz_assignment *g, int *K, int *f, int *l, int *r) {
    if (!g) return BYZ_EINVAL;
    if (K) *K = g->K;
    if (f) *f = g->f;
    if (l) *l = g->l;
    if (r) *r = g->r;
    return BYZ_OK;
}

extern "C" int byz_assignment_worker_files(const byz_assignment *g, int32_t *out) {
    if (!g || !out) return BYZ_EINVAL;
    std::memcpy(out, g->worker_files.data(), g->worker_files.size() * sizeof(int32_t));
    return BYZ_OK;
}

extern "C" int byz_assignment_file_workers(const byz_assignment *g, int32_t *out) {
    if (!g || !out) return BYZ_EINVAL;
    std::memcpy(out, g->file_workers.data(), g->file_workers.size() * sizeof(int32_t));
    return BYZ_OK;
}

extern "C" int byz_assignment_file_rows(const byz_assignment *g, int32_t *out) {
    if (!g || !out) return BYZ_EINVAL;
    std::memcpy(out, g->file_rows.data(), g->file_rows.size() * sizeof(int32_t));
    return BYZ_OK;
}

// ------------------------------------------------------------------ worst-case search

namespace {

// Per-file copy counters for up to 64*W files, one bit plane per binary digit (counts <= 7).
template <int W> struct FileSet {
    uint64_t w[W];
};

template <int W> struct Planes {
    FileSet<W> c0, c1, c2;
};

template <int W> inline Planes<W> add_mask(Planes<W> p, const FileSet<W> &m) {
    for (int i = 0; i < W; ++i) {
        const uint64_t carry = p.c0.w[i] & m.w[i];
        p.c0.w[i] ^= m.w[i];
        const uint64_t carry2 = p.c1.w[i] & carry;
        p.c1.w[i] ^= carry;
        p.c2.w[i] ^= carry2;
    }
    return p;
}

// bit j set iff count_j >= need, need in 1..4
template <int W> inline FileSet<W> at_least(const Planes<W> &p, int need) {
    FileSet<W> out;
    for (int i = 0; i < W; ++i) {
        const uint64_t c0 = p.c0.w[i], c1 = p.c1.w[i], c2 = p.c2.w[i];
        switch (need) {
            case 1: out.w[i] = c0 | c1 | c2; break;
            case 2: out.w[i] = c1 | c2; break;
            case 3: out.w[i] = c2 | (c1 & c0); break;
            default: out.w[i] = c2; break;
        }
    }
    return out;
}

template <int W> inline int count(const FileSet<W> &s) {
    int c = 0;
    for (int i = 0; i < W; ++i) c += __builtin_popcountll(s.w[i]);
    return c;
}

template <int W> struct SearchResult {
    int best = -1;
    FileSet<W> files = {};
    std::vector<int> set;
    uint64_t visited = 0;  // subsets evaluated
};

// All q-subsets that start with the ascending workers prefix[0..p-1] (1 <= p <= q), in
// lexicographic order; keeps the first one with the largest number of files that have at least
// `need` copies inside the subset.  With target >= 0 the walk ends at the first subset that
// reaches target files, and gives up (best stays below target) as soon as *stop_below holds a
// task number smaller than my_task (an earlier task has already found one).
template <int W>
SearchResult<W> search_with_prefix(const std::vector<FileSet<W>> &mask, int K, int q, int need,
                                   const int *prefix, int p, int target = -1,
                                   const std::atomic<int> *stop_below = nullptr, int my_task = 0) {
    SearchResult<W> res;
    res.set.assign((size_t)q, 0);
    std::vector<int> cur((size_t)q + 1, 0);
    // planes[t] = per-file counters of the first t chosen workers
    std::vector<Planes<W>> planes((size_t)q + 1, Planes<W>{});
    for (int i = 0; i < p; ++i) {
        cur[i] = prefix[i];
        planes[i + 1] = add_mask(planes[i], mask[prefix[i]]);
    }
    if (p == q) {
        const FileSet<W> hit = at_least(planes[p], need);
        res.best = count(hit);
        res.files = hit;
        res.visited = 1;
        for (int i = 0; i < q; ++i) res.set[i] = prefix[i];
        return res;
    }
    int t = p;
    cur[p] = prefix[p - 1];
    for (;;) {
        ++cur[t];
        if (cur[t] > K - (q - t)) {  // exhausted this position
            if (t == p) break;
            --t;
            continue;
        }
        if (t < q - 1) {
            planes[t + 1] = add_mask(planes[t], mask[cur[t]]);
            cur[t + 1] = cur[t];
            ++t;
            continue;
        }
        // last position: sweep all remaining workers in a tight loop
        const Planes<W> base = planes[t];
        res.visited += (uint64_t)(K - cur[t]);
        for (int w = cur[t]; w < K; ++w) {
            const FileSet<W> hit = at_least(add_mask(base, mask[w]), need);
            const int c = count(hit);
            if (c > res.best) {
                res.best = c;
                res.files = hit;
                for (int i = 0; i < t; ++i) res.set[i] = cur[i];
                res.set[t] = w;
                if (target >= 0 && c >= target) return res;
            }
        }
        if (stop_below != nullptr && stop_below->load(std::memory_order_relaxed) < my_task)
            return res;
        if (t == p) break;
        --t;
    }
    return res;
}

// Runs tasks (prefixes) over up to 16 host threads; on_result(task, result) is called for
// every finished task, from the worker threads, under no lock.
template <int W, class F>
int run_tasks(const std::vector<FileSet<W>> &mask, int K, int q, int need,
              const std::vector<std::vector<int>> &tasks, double work, int target,
              std::atomic<int> *stop_below, F on_result) {
    const int n_tasks = (int)tasks.size();
    unsigned n_threads = 1;
    if (work > 2e7) {
        n_threads = std::thread::hardware_concurrency();
        if (n_threads < 1) n_threads = 1;
        if (n_threads > 16) n_threads = 16;
        if (n_threads > (unsigned)n_tasks) n_threads = (unsigned)n_tasks;
    }
    std::atomic<int> next_task(0);
    auto worker = [&]() {
        for (;;) {
            const int i = next_task.fetch_add(1);
            if (i >= n_tasks) break;
            if (stop_below != nullptr && stop_below->load(std::memory_order_relaxed) < i) continue;
            on_result(i, search_with_prefix<W>(mask, K, q, need, tasks[(size_t)i].data(),
                                               (int)tasks[(size_t)i].size(), target, stop_below, i));
        }
    };
    if (n_threads <= 1) {
        worker();
        return BYZ_OK;
    }
    try {
        std::vector<std::thread> pool;
        for (unsigned i = 0; i < n_threads; ++i) pool.emplace_back(worker);
        for (auto &th : pool) th.join();
    } catch (const std::system_error &) {
        return BYZ_ENOMEM;  // threads could not be started
    }
    return BYZ_OK;
}

// Symmetries of the assignment that the search may use: translations of the file grid that
// map every worker's file set onto another worker's of the same parallel class.  All three
// constructions are lines of an affine plane, so translating the files permutes the lines of
// every direction (class) among themselves; each candidate is nevertheless checked on the graph
// itself, and what does not check out is not used.
struct Symmetry {
    std::vector<std::vector<int>> worker_perm;  // verified automorphisms, as worker maps
    bool level1 = false;  // every class is one orbit
    bool level2 = false;  // ... and the maps fixing a class pointwise act transitively on every other
};

Symmetry find_symmetry(const byz_assignment &g) {
    Symmetry sym;
    const int K = g.K, f = g.f, l = g.l, cs = g.class_size, classes = K / cs;
    if (g.gx * g.gy != f || cs < 1 || K % cs != 0) return sym;
    // worker by (class, files): with FRC several workers, one per class, hold the same files
    std::map<std::vector<int>, int> by_files;
    for (int w = 0; w < K; ++w) {
        std::vector<int> key(g.worker_files.begin() + (size_t)w * l,
                             g.worker_files.begin() + (size_t)(w + 1) * l);
        key.push_back(w / cs);
        by_files[key] = w;
    }
    auto shift = [&](int a, int by, int n) {
        return g.add_tab.empty() ? (a + by) % n : (int)g.add_tab[(size_t)a * n + by];
    };
    for (int u = 0; u < g.gx; ++u)
        for (int v = 0; v < g.gy; ++v) {
            if (u == 0 && v == 0) continue;
            std::vector<int> perm((size_t)K, -1);
            bool ok = true;
            for (int w = 0; w < K && ok; ++w) {
                std::vector<int> img((size_t)l);
                for (int t = 0; t < l; ++t) {
                    const int j = g.worker_files[(size_t)w * l + t];
                    img[(size_t)t] = shift(j / g.gy, u, g.gx) * g.gy + shift(j % g.gy, v, g.gy);
                }
                std::sort(img.begin(), img.end());
                img.push_back(w / cs);
                auto it = by_files.find(img);
                if (it == by_files.end()) ok = false;
                else perm[(size_t)w] = it->second;
            }
            if (ok) sym.worker_perm.push_back(perm);
        }
    // level 1: the first worker of every class reaches the whole class
    auto orbit_covers = [&](const std::vector<const std::vector<int> *> &maps, int cls) {
        std::vector<char> seen((size_t)K, 0);
        std::vector<int> todo(1, cls * cs);
        seen[(size_t)(cls * cs)] = 1;
        int n = 1;
        while (!todo.empty()) {
            const int w = todo.back();
            todo.pop_back();
            for (const auto *m : maps) {
                const int x = (*m)[(size_t)w];
                if (!seen[(size_t)x]) { seen[(size_t)x] = 1; ++n; todo.push_back(x); }
            }
        }
        return n == cs;
    };
    std::vector<const std::vector<int> *> all;
    for (const auto &m : sym.worker_perm) all.push_back(&m);
    sym.level1 = true;
    for (int c = 0; c < classes; ++c) sym.level1 = sym.level1 && orbit_covers(all, c);
    if (!sym.level1) return sym;
    sym.level2 = classes >= 2 && cs <= 20;  // the step-1 tasks enumerate 2^(cs-1) partial classes
    for (int c0 = 0; c0 < classes && sym.level2; ++c0) {
        std::vector<const std::vector<int> *> fixing;
        for (const auto &m : sym.worker_perm) {
            bool fixes = true;
            for (int i = 0; i < cs; ++i) fixes = fixes && m[(size_t)(c0 * cs + i)] == c0 * cs + i;
            if (fixes) fixing.push_back(&m);
        }
        for (int c1 = c0 + 1; c1 < classes; ++c1)
            sym.level2 = sym.level2 && orbit_covers(fixing, c1);
    }
    return sym;
}

thread_local uint64_t g_last_visited = 0;

template <int W>
int worst_case_impl(const byz_assignment *g, int q, unsigned flags, int32_t *byz_workers_out,
                    int32_t *cmax_out, uint64_t *distorted_mask_out) {
    const int K = g->K, l = g->l;
    const int need = (g->r + 1) / 2;  // r' of Sec. 2
    std::vector<FileSet<W>> mask((size_t)K, FileSet<W>{});
    for (int w = 0; w < K; ++w)
        for (int t = 0; t < l; ++t) {
            const int j = g->worker_files[(size_t)w * l + t];
            mask[w].w[j >> 6] |= 1ull << (j & 63);
        }
    g_last_visited = 0;
    int best = -1;
    FileSet<W> best_files = {};
    std::vector<int> best_set((size_t)q, 0);
    if (q == 0) {
        best = 0;
    } else {
        double subsets = 1.0;
        for (int i = 0; i < q; ++i) subsets = subsets * (K - i) / (i + 1);
        std::atomic<uint64_t> visited(0);
        // Lexicographic tasks: one per choice of the first one or two (smallest) workers of
        // the set.  Inside a task the tuples are visited depth-first in ascending =
        // lexicographic order, so a task's result is its first maximiser; merging the tasks in
        // order and keeping a result only when it is strictly better keeps the overall first
        // maximiser.
        const int p = q >= 3 ? 2 : 1;
        std::vector<std::vector<int>> lex_tasks;
        for (int a0 = 0; a0 <= K - q; ++a0) {
            if (p == 1) {
                lex_tasks.push_back({a0});
            } else {
                for (int a1 = a0 + 1; a1 <= K - q + 1; ++a1) lex_tasks.push_back({a0, a1});
            }
        }
        Symmetry sym;
        const bool want_sym = (flags & BYZ_SEARCH_EXHAUSTIVE) == 0 && q >= 2 &&
                              ((flags & BYZ_SEARCH_SYMMETRY) != 0 || subsets > 2e6);
        if (want_sym) sym = find_symmetry(*g);
        if (!sym.level1) {
            // plain exhaustive search
            std::vector<SearchResult<W>> results(lex_tasks.size());
            int rc = run_tasks<W>(mask, K, q, need, lex_tasks, subsets, -1, nullptr,
                                  [&](int i, SearchResult<W> r) {
                                      visited += r.visited;
                                      results[(size_t)i] = std::move(r);
                                  });
            if (rc != BYZ_OK) return rc;
            for (const auto &res : results)
                if (res.best > best) {
                    best = res.best;
                    best_files = res.files;
                    best_set = res.set;
                }
        } else {
            // Step 1, the value c_max alone, over one representative per orbit: every set can
            // be translated so that, of the lowest class c0 it touches, it contains the first
            // worker w0; with level 2, keeping class c0 in place, also so that of the next
            // class c1 it touches it contains the first worker w1.  Workers of one class share
            // no file, so the members of c0 beside w0 are free, nothing lies between the
            // classes, and the rest of the set comes after w1.
            const int cs = g->class_size, classes = K / cs;
            std::vector<std::vector<int>> tasks;
            for (int c0 = 0; c0 < classes; ++c0) {
                const int w0 = c0 * cs;
                if (q <= cs) {  // all inside class c0: equivalent sets, one stands for all
                    std::vector<int> inside;
                    for (int i = 0; i < q; ++i) inside.push_back(w0 + i);
                    tasks.push_back(inside);
                }
                if (!sym.level2) {
                    // second member anywhere after w0 (sets inside the class are visited again:
                    // harmless)
                    for (int a1 = w0 + 1; a1 <= K - q + 1; ++a1) tasks.push_back({w0, a1});
                    continue;
                }
                for (int c1 = c0 + 1; c1 < classes; ++c1) {
                    const int w1 = c1 * cs;
                    // subsets A of the other cs - 1 workers of class c0, by bit mask
                    for (uint32_t bits = 0; bits < (1u << (cs - 1)); ++bits) {
                        const int a = __builtin_popcount(bits);
                        if (a > q - 2 || K - w1 - 1 < q - 2 - a) continue;
                        std::vector<int> prefix(1, w0);
                        for (int i = 0; i < cs - 1; ++i)
                            if ((bits >> i) & 1u) prefix.push_back(w0 + 1 + i);
                        prefix.push_back(w1);
                        tasks.push_back(prefix);
                    }
                }
            }
            std::atomic<int> best_value(-1);
            int rc = run_tasks<W>(mask, K, q, need, tasks, subsets / cs, -1, nullptr,
                                  [&](int, SearchResult<W> r) {
                                      visited += r.visited;
                                      int seen = best_value.load();
                                      while (r.best > seen &&
                                             !best_value.compare_exchange_weak(seen, r.best)) {
                                      }
                                  });
            if (rc != BYZ_OK) return rc;
            const int cmax = best_value.load();
            // Step 2, the lexicographically first set that reaches c_max: lexicographic
            // tasks again, each ending at its first hit, later tasks dropped once an earlier
            // one has hit.
            std::vector<SearchResult<W>> results(lex_tasks.size());
            std::atomic<int> first_hit((int)lex_tasks.size());
            rc = run_tasks<W>(mask, K, q, need, lex_tasks, subsets, cmax, &first_hit,
                              [&](int i, SearchResult<W> r) {
                                  visited += r.visited;
                                  if (r.best >= cmax) {
                                      int seen = first_hit.load();
                                      while (i < seen && !first_hit.compare_exchange_weak(seen, i)) {
                                      }
                                  }
                                  results[(size_t)i] = std::move(r);
                              });
            if (rc != BYZ_OK) return rc;
            const int hit = first_hit.load();
            if (hit >= (int)lex_tasks.size() || results[(size_t)hit].best != cmax)
                return BYZ_EINTERNAL;  // the symmetric step found a value no set attains
            best = cmax;
            best_files = results[(size_t)hit].files;
            best_set = results[(size_t)hit].set;
        }
        g_last_visited = visited.load();
    }
    if (byz_workers_out)
        for (int i = 0; i < q; ++i) byz_workers_out[i] = best_set[i];
    if (cmax_out) *cmax_out = best;
    if (distorted_mask_out)
        for (int i = 0; i < (g->f + 63) / 64; ++i) distorted_mask_out[i] = best_files.w[i];
    return BYZ_OK;
}

}  // namespace

extern "C" int byz_worst_case_opts(const byz_assignment *g, int q, unsigned flags,
                                   int32_t *byz_workers_out, int32_t *cmax_out,
                                   uint64_t *distorted_mask_out) {
    if (!g || q < 0 || q > g->K) return BYZ_EINVAL;
    if ((flags & ~(unsigned)(BYZ_SEARCH_EXHAUSTIVE | BYZ_SEARCH_SYMMETRY)) != 0 ||
        flags == (BYZ_SEARCH_EXHAUSTIVE | BYZ_SEARCH_SYMMETRY))
        return BYZ_EINVAL;
    if (g->f > BYZ_MAX_F_WIDE || g->r > BYZ_MAX_R) return BYZ_EUNSUPPORTED;
    try {
        if (g->f <= 64)
            return worst_case_impl<1>(g, q, flags, byz_workers_out, cmax_out, distorted_mask_out);
        if (g->f <= 128)
            return worst_case_impl<2>(g, q, flags, byz_workers_out, cmax_out, distorted_mask_out);
        return worst_case_impl<4>(g, q, flags, byz_workers_out, cmax_out, distorted_mask_out);
    } catch (const std::bad_alloc &) {
        return BYZ_ENOMEM;
    }
}

extern "C" int byz_worst_case(const byz_assignment *g, int q, int32_t *byz_workers_out,
                              int32_t *cmax_out, uint64_t *distorted_mask_out) {
    return byz_worst_case_opts(g, q, 0u, byz_workers_out, cmax_out, distorted_mask_out);
}

extern "C" uint64_t byz_worst_case_last_visited(void) { return g_last_visited; }

extern "C" double byz_gamma_bound(const byz_assignment *g, int q) {
    if (!g || q < 0 || q > g->K) return std::nan("");
    const double K = g->K, l = g->l, r = g->r;
    const double mu1 = 1.0 / r;                                      // Lemma 2
    const double beta = (q * l / r) / (mu1 + (1.0 - mu1) * q / K);   // Eq. 5
    return (q * l - beta) / ((r - 1.0) / 2.0);                       // Claim 1
}

extern "C" const char *byz_strerror(int code) {
    switch (code) {
        case BYZ_OK: return "ok";
        case BYZ_EINVAL: return "invalid argument";
        case BYZ_EUNSUPPORTED: return "valid but not supported by this build";
        case BYZ_ENOMEM: return "out of memory or workspace too small";
        case BYZ_EDEVICE: return "HIP call failed";
        case BYZ_EINTERNAL: return "internal invariant violated";
        default: return "unknown byz_status";
    }
}
