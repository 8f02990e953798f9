// topology_build / topology_build_ex / topology_metropolis: neighbour lists and weights (host only).
//
// Appendix "Network topologies": ring, mesh, (symmetric) exponential graph with hops
// 2^0 .. 2^floor(log2(n-1)), bipartite random match; Introduction: the one-peer exponential
// graph uses a single hop per iteration, cycling through them.  Weights follow the
// Metropolis-Hastings rule the paper cites, w_ij = 1 / (1 + max(deg_i, deg_j)) for j != i and
// w_ii = 1 - sum_j w_ij (deg = number of neighbours other than i); on a regular graph this is
// the uniform 1 / |N_i|, which is evaluated directly so that the common cases carry exactly
// (float)1 / (float)|N_i|.
//
// A phase is first built as plain adjacency (self first, then neighbours in the documented
// order, duplicates dropped keeping the first occurrence); weights and the reported
// properties are then computed from the adjacency alone.
#include <algorithm>
#include <cmath>
#include <vector>

#include "internal.hpp"

namespace {

using Rows = std::vector<std::vector<int32_t>>;  // Rows[i] = N_i, i itself first

int32_t exponent_count(int32_t n) {  // number of t with 2^t <= n-1
    int32_t tau = 0;
    for (int64_t h = 1; h <= static_cast<int64_t>(n) - 1; h <<= 1) ++tau;
    return tau;
}

void add_unique(std::vector<int32_t>& row, int64_t j, int32_t n) {
    j %= n;
    if (j < 0) j += n;
    if (std::find(row.begin(), row.end(), static_cast<int32_t>(j)) == row.end())
        row.push_back(static_cast<int32_t>(j));
}

Rows circulant(int32_t n, const std::vector<int64_t>& offsets) {
    Rows rows(n);
    for (int32_t i = 0; i < n; ++i) {
        rows[i].push_back(i);
        for (int64_t o : offsets) add_unique(rows[i], static_cast<int64_t>(i) + o, n);
    }
    return rows;
}

// 2-D grid, R x C with R the largest divisor of n not above sqrt(n), node i at (i / C, i % C),
// 4-neighbourhood without wrap-around; order: up, down, left, right.
Rows mesh(int32_t n) {
    int32_t R = 1;
    for (int32_t r = 1; static_cast<int64_t>(r) * r <= n; ++r)
        if (n % r == 0) R = r;
    const int32_t C = n / R;
    Rows rows(n);
    for (int32_t i = 0; i < n; ++i) {
        const int32_t a = i / C, b = i % C;
        rows[i].push_back(i);
        if (a > 0) rows[i].push_back(i - C);
        if (a + 1 < R) rows[i].push_back(i + C);
        if (b > 0) rows[i].push_back(i - 1);
        if (b + 1 < C) rows[i].push_back(i + 1);
    }
    return rows;
}

// splitmix64 (Steele, Lea, Flood 2014): the counter-based generator behind the random matching.
struct SplitMix64 {
    uint64_t state;
    uint64_t next() {
        uint64_t z = (state += 0x9E3779B97F4A7C15ULL);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
        return z ^ (z >> 31);
    }
};

// Bipartite random match of one phase: shuffle 0..n-1 (Fisher-Yates from the top, index drawn
// as next() % (t + 1)), the first half of the shuffled order is one group, the second half the
// other, and position q pairs with position q + n/2.  Odd n leaves the last position alone.
Rows random_match(int32_t n, uint64_t seed, int32_t phase) {
    std::vector<int32_t> perm(n);
    for (int32_t i = 0; i < n; ++i) perm[i] = i;
    SplitMix64 rng{seed ^ (0xD1B54A32D192ED03ULL * (static_cast<uint64_t>(phase) + 1))};
    for (int32_t t = n - 1; t > 0; --t) {
        const int32_t q = static_cast<int32_t>(rng.next() % static_cast<uint64_t>(t + 1));
        std::swap(perm[t], perm[q]);
    }
    Rows rows(n);
    for (int32_t i = 0; i < n; ++i) rows[i].push_back(i);
    const int32_t half = n / 2;
    for (int32_t q = 0; q < half; ++q) {
        rows[perm[q]].push_back(perm[q + half]);
        rows[perm[q + half]].push_back(perm[q]);
    }
    return rows;
}

bool build_phase(int kind, int32_t n, uint64_t seed, int32_t phase, Rows* out) {
    const int32_t tau = exponent_count(n);
    switch (kind) {
        case DL_TOPO_RING:
            *out = circulant(n, {-1, +1});
            return true;
        case DL_TOPO_EXP_STATIC: {
            std::vector<int64_t> o;
            for (int32_t t = 0; t < tau; ++t) o.push_back(int64_t{1} << t);
            *out = circulant(n, o);
            return true;
        }
        case DL_TOPO_EXP_ONEPEER:
            *out = tau == 0 ? circulant(n, {}) : circulant(n, {int64_t{1} << phase});
            return true;
        case DL_TOPO_EXP_SYM: {
            std::vector<int64_t> o;
            for (int32_t t = 0; t < tau; ++t) {
                o.push_back(int64_t{1} << t);
                o.push_back(-(int64_t{1} << t));
            }
            *out = circulant(n, o);
            return true;
        }
        case DL_TOPO_MESH:
            *out = mesh(n);
            return true;
        case DL_TOPO_BIPARTITE_MATCH:
            *out = random_match(n, seed, phase);
            return true;
        default:
            return false;
    }
}

// Metropolis-Hastings weights of an undirected adjacency given as rows with self first.
// A directed row set (static / one-peer exponential) has no Metropolis rule; it gets the
// uniform 1 / |N_i| the workloads define.
void weights_for(const Rows& rows, bool metropolis, std::vector<std::vector<float>>* w) {
    const size_t n = rows.size();
    w->assign(n, {});
    for (size_t i = 0; i < n; ++i) {
        const size_t deg_i = rows[i].size() - 1;
        bool regular = true;
        if (metropolis)
            for (size_t t = 1; t < rows[i].size(); ++t) regular &= (rows[rows[i][t]].size() - 1 == deg_i);
        std::vector<float>& wi = (*w)[i];
        wi.resize(rows[i].size());
        if (!metropolis || regular) {
            const float u = 1.0f / static_cast<float>(rows[i].size());
            std::fill(wi.begin(), wi.end(), u);
            continue;
        }
        double others = 0.0;
        for (size_t t = 1; t < rows[i].size(); ++t) {
            const size_t deg_j = rows[rows[i][t]].size() - 1;
            wi[t] = 1.0f / static_cast<float>(1 + std::max(deg_i, deg_j));
            others += static_cast<double>(wi[t]);
        }
        wi[0] = static_cast<float>(1.0 - others);
    }
}

struct Entry {
    int32_t j;
    float w;
};

// Row / column stochasticity and symmetry of one phase.
uint32_t flags_of(const Rows& rows, const std::vector<std::vector<float>>& w) {
    const size_t n = rows.size();
    std::vector<double> col(n, 0.0);
    bool row_ok = true, sym = true;
    std::vector<std::vector<Entry>> sorted(n);
    for (size_t i = 0; i < n; ++i) {
        double sum = 0.0;
        for (size_t t = 0; t < rows[i].size(); ++t) {
            sum += static_cast<double>(w[i][t]);
            col[rows[i][t]] += static_cast<double>(w[i][t]);
            sorted[i].push_back({rows[i][t], w[i][t]});
        }
        row_ok &= std::fabs(sum - 1.0) <= 1e-6;
        std::sort(sorted[i].begin(), sorted[i].end(), [](const Entry& a, const Entry& b) { return a.j < b.j; });
    }
    bool col_ok = true;
    for (size_t j = 0; j < n; ++j) col_ok &= std::fabs(col[j] - 1.0) <= 1e-6;
    for (size_t i = 0; i < n && sym; ++i)
        for (const Entry& e : sorted[i]) {
            const auto& other = sorted[e.j];
            auto it = std::lower_bound(other.begin(), other.end(), static_cast<int32_t>(i),
                                       [](const Entry& a, int32_t key) { return a.j < key; });
            if (it == other.end() || it->j != static_cast<int32_t>(i) || it->w != e.w) {
                sym = false;
                break;
            }
        }
    return (row_ok ? DL_FLAG_ROW_STOCHASTIC : 0u) | (col_ok ? DL_FLAG_COL_STOCHASTIC : 0u) |
           (sym ? DL_FLAG_SYMMETRIC : 0u);
}

}  // namespace

extern "C" int topology_build_ex(int kind, int32_t n, uint64_t seed, int32_t phases, int32_t* row_ptr,
                                 int64_t row_ptr_cap, int32_t* col_idx, float* w, int64_t nnz_cap,
                                 int32_t* period_out, int64_t* nnz_out, uint32_t* flags_out) {
    dl::clear_error();
    if (n < 1) return dl::set_error(DL_EINVAL, "topology_build: n = %d, need n >= 1", n);
    if (kind < DL_TOPO_RING || kind > DL_TOPO_BIPARTITE_MATCH)
        return dl::set_error(DL_EINVAL, "topology_build: unknown kind %d", kind);
    if (!period_out || !nnz_out)
        return dl::set_error(DL_EINVAL, "topology_build: period_out and nnz_out must not be NULL");
    const bool query = (row_ptr == nullptr);
    if (!query && (!col_idx || !w))
        return dl::set_error(DL_EINVAL, "topology_build: col_idx and w must accompany row_ptr");

    int32_t period = 1;
    if (kind == DL_TOPO_EXP_ONEPEER && n > 1) period = exponent_count(n);
    if (kind == DL_TOPO_BIPARTITE_MATCH) {
        if (phases < 1)
            return dl::set_error(DL_EINVAL, "topology_build: bipartite random match needs phases >= 1, got %d", phases);
        period = phases;
    }
    const bool metropolis = kind != DL_TOPO_EXP_STATIC && kind != DL_TOPO_EXP_ONEPEER;

    std::vector<Rows> all(period);
    std::vector<std::vector<std::vector<float>>> weights(period);
    int64_t nnz = 0;
    uint32_t flags = DL_FLAG_ROW_STOCHASTIC | DL_FLAG_COL_STOCHASTIC | DL_FLAG_SYMMETRIC;
    for (int32_t p = 0; p < period; ++p) {
        build_phase(kind, n, seed, p, &all[p]);
        weights_for(all[p], metropolis, &weights[p]);
        flags &= flags_of(all[p], weights[p]);
        for (const auto& r : all[p]) nnz += static_cast<int64_t>(r.size());
    }
    *period_out = period;
    *nnz_out = nnz;
    if (flags_out) *flags_out = flags;
    if (query) return DL_OK;

    const int64_t need_rows = static_cast<int64_t>(period) * (static_cast<int64_t>(n) + 1);
    if (row_ptr_cap < need_rows || nnz_cap < nnz)
        return dl::set_error(DL_ECAP, "topology_build: need row_ptr_cap >= %lld and nnz_cap >= %lld",
                             static_cast<long long>(need_rows), static_cast<long long>(nnz));
    if (nnz > INT32_MAX)
        return dl::set_error(DL_ECAP, "topology_build: %lld entries exceed int32 offsets",
                             static_cast<long long>(nnz));
    int64_t at = 0;
    for (int32_t p = 0; p < period; ++p) {
        int32_t* rp = row_ptr + static_cast<int64_t>(p) * (n + 1);
        for (int32_t i = 0; i < n; ++i) {
            rp[i] = static_cast<int32_t>(at);
            for (size_t t = 0; t < all[p][i].size(); ++t) {
                col_idx[at] = all[p][i][t];
                w[at] = weights[p][i][t];
                ++at;
            }
        }
        rp[n] = static_cast<int32_t>(at);
    }
    return DL_OK;
}

extern "C" int topology_build(int kind, int32_t n, int32_t* row_ptr, int64_t row_ptr_cap, int32_t* col_idx,
                              float* w, int64_t nnz_cap, int32_t* period_out, int64_t* nnz_out,
                              uint32_t* flags_out) {
    if (kind == DL_TOPO_BIPARTITE_MATCH) {
        dl::clear_error();
        return dl::set_error(DL_EINVAL, "topology_build: the bipartite random match takes a seed and a "
                                        "phase count; use topology_build_ex");
    }
    return topology_build_ex(kind, n, 0, 1, row_ptr, row_ptr_cap, col_idx, w, nnz_cap, period_out, nnz_out,
                             flags_out);
}

extern "C" int topology_metropolis(int32_t n, const int32_t* row_ptr, const int32_t* col_idx, float* w,
                                   uint32_t* flags_out) {
    dl::clear_error();
    if (n < 1) return dl::set_error(DL_EINVAL, "topology_metropolis: n = %d, need n >= 1", n);
    if (!row_ptr || !col_idx || !w)
        return dl::set_error(DL_EINVAL, "topology_metropolis: row_ptr, col_idx and w must not be NULL");
    Rows rows(n);
    for (int32_t i = 0; i < n; ++i) {
        if (row_ptr[i + 1] <= row_ptr[i])
            return dl::set_error(DL_ETOPO, "topology_metropolis: row %d is empty or row_ptr decreases", i);
        bool has_self = false;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int32_t j = col_idx[q];
            if (j < 0 || j >= n)
                return dl::set_error(DL_ETOPO, "topology_metropolis: row %d: neighbour index %d outside [0, %d)", i, j, n);
            if (std::find(rows[i].begin(), rows[i].end(), j) != rows[i].end())
                return dl::set_error(DL_ETOPO, "topology_metropolis: row %d lists neighbour %d twice", i, j);
            has_self |= (j == i);
            rows[i].push_back(j);
        }
        if (!has_self)
            return dl::set_error(DL_ETOPO, "topology_metropolis: row %d does not contain %d itself", i, i);
    }
    // the rule needs an undirected graph: j in N_i  <=>  i in N_j
    for (int32_t i = 0; i < n; ++i)
        for (int32_t j : rows[i])
            if (std::find(rows[j].begin(), rows[j].end(), i) == rows[j].end())
                return dl::set_error(DL_ETOPO, "topology_metropolis: %d lists %d but not the reverse", i, j);
    // weights_for expects self first; compute in that order, then scatter back to the caller's order
    Rows self_first(n);
    for (int32_t i = 0; i < n; ++i) {
        self_first[i].push_back(i);
        for (int32_t j : rows[i])
            if (j != i) self_first[i].push_back(j);
    }
    std::vector<std::vector<float>> ws;
    weights_for(self_first, true, &ws);
    for (int32_t i = 0; i < n; ++i) {
        size_t t = 1;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) w[q] = (col_idx[q] == i) ? ws[i][0] : ws[i][t++];
    }
    if (flags_out) *flags_out = flags_of(self_first, ws);
    return DL_OK;
}
