// topology_build: neighbour lists of the paper's circulant topologies (host only).
//
// Appendix "Network topologies": ring (two direct neighbours) and the exponential
// graph with hops 2^0 .. 2^floor(log2(n-1)); Introduction: the one-peer variant
// uses a single hop per iteration, cycling through them.  Every graph here is
// circulant, so a phase is described by a short list of signed offsets.
#include <cmath>
#include <vector>

#include "internal.hpp"

namespace {

struct Shape {
    int32_t period = 1;
    std::vector<std::vector<int64_t>> offsets;  // per phase, self (0) first
};

int32_t exponent_count(int32_t n) {
    // number of t with 2^t <= n-1
    int32_t tau = 0;
    for (int64_t h = 1; h <= static_cast<int64_t>(n) - 1; h <<= 1) ++tau;
    return tau;
}

Shape shape_of(int kind, int32_t n) {
    Shape s;
    const int32_t tau = exponent_count(n);
    switch (kind) {
        case DL_TOPO_RING:
            s.offsets.push_back({0, -1, +1});
            break;
        case DL_TOPO_EXP_STATIC: {
            std::vector<int64_t> o{0};
            for (int32_t t = 0; t < tau; ++t) o.push_back(int64_t{1} << t);
            s.offsets.push_back(o);
            break;
        }
        case DL_TOPO_EXP_ONEPEER:
            if (tau == 0) {
                s.offsets.push_back({0});
            } else {
                s.period = tau;
                for (int32_t t = 0; t < tau; ++t) s.offsets.push_back({0, int64_t{1} << t});
            }
            break;
    }
    return s;
}

// Distinct residues of i + offsets (mod n), first occurrence kept.
void row_members(int32_t i, int32_t n, const std::vector<int64_t>& off, std::vector<int32_t>& out) {
    out.clear();
    for (int64_t o : off) {
        int64_t j = (static_cast<int64_t>(i) + o) % n;
        if (j < 0) j += n;
        bool seen = false;
        for (int32_t q : out) seen |= (q == j);
        if (!seen) out.push_back(static_cast<int32_t>(j));
    }
}

}  // namespace

extern "C" int topology_build(int kind, int32_t n, int32_t* row_ptr, int64_t row_ptr_cap,
                              int32_t* col_idx, float* w, int64_t nnz_cap, int32_t* period_out,
                              int64_t* nnz_out, uint32_t* flags_out) {
    dl::clear_error();
    if (n < 1) return dl::set_error(DL_EINVAL, "topology_build: n = %d, need n >= 1", n);
    if (kind != DL_TOPO_RING && kind != DL_TOPO_EXP_STATIC && kind != DL_TOPO_EXP_ONEPEER)
        return dl::set_error(DL_EINVAL, "topology_build: unknown kind %d", kind);
    if (!period_out || !nnz_out)
        return dl::set_error(DL_EINVAL, "topology_build: period_out and nnz_out must not be NULL");
    const bool query = (row_ptr == nullptr);
    if (!query && (!col_idx || !w))
        return dl::set_error(DL_EINVAL, "topology_build: col_idx and w must accompany row_ptr");

    const Shape s = shape_of(kind, n);
    std::vector<int32_t> members;

    // sizes and properties first: they are reported even when the capacity is short
    int64_t nnz = 0;
    bool symmetric = true;
    for (int32_t p = 0; p < s.period; ++p) {
        row_members(0, n, s.offsets[p], members);
        nnz += static_cast<int64_t>(members.size()) * n;
        // circulant with uniform weights: symmetric iff the offset set is closed under negation
        for (int32_t j : members) {
            bool has_neg = false;
            for (int32_t q : members) has_neg |= (q == (n - j) % n);
            symmetric &= has_neg;
        }
    }
    *period_out = s.period;
    *nnz_out = nnz;
    if (flags_out) {
        // uniform 1/deg on a circulant graph: every row and every column holds deg entries of
        // fl32(1/deg); deg * fl32(1/deg) differs from 1 by at most deg * 2^-25 / deg < 1e-6
        *flags_out = DL_FLAG_ROW_STOCHASTIC | DL_FLAG_COL_STOCHASTIC | (symmetric ? DL_FLAG_SYMMETRIC : 0u);
    }
    if (query) return DL_OK;

    const int64_t need_rows = static_cast<int64_t>(s.period) * (static_cast<int64_t>(n) + 1);
    if (row_ptr_cap < need_rows || nnz_cap < nnz)
        return dl::set_error(DL_ECAP, "topology_build: need row_ptr_cap >= %lld and nnz_cap >= %lld",
                             static_cast<long long>(need_rows), static_cast<long long>(nnz));
    if (nnz > INT32_MAX)
        return dl::set_error(DL_ECAP, "topology_build: %lld entries exceed int32 offsets",
                             static_cast<long long>(nnz));

    int64_t at = 0;
    for (int32_t p = 0; p < s.period; ++p) {
        int32_t* rp = row_ptr + static_cast<int64_t>(p) * (n + 1);
        for (int32_t i = 0; i < n; ++i) {
            rp[i] = static_cast<int32_t>(at);
            row_members(i, n, s.offsets[p], members);
            const float weight = 1.0f / static_cast<float>(members.size());
            for (int32_t j : members) {
                col_idx[at] = j;
                w[at] = weight;
                ++at;
            }
        }
        rp[n] = static_cast<int32_t>(at);
    }
    return DL_OK;
}
