// Host boundary: argument validation, error reporting, packing of one phase of W
// into kernel arguments.  Every exported function returns a dl_status.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "internal.hpp"

namespace dl {

namespace {
thread_local char g_error[512] = "";
}

void clear_error() { g_error[0] = '\0'; }

int set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

int check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return DL_OK;
    return set_error(DL_EHIP, "%s: %s", what, hipGetErrorString(e));
}

namespace {

// Byte range [lo, hi) touched by an n x d array with row stride ld.
struct Span {
    uintptr_t lo, hi;
};
Span span_of(const void* p, int64_t rows, int64_t cols, int64_t ld, int64_t elem_bytes = 4) {
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    if (rows <= 0 || cols <= 0) return {lo, lo};
    return {lo, lo + static_cast<uintptr_t>(((rows - 1) * ld + cols) * elem_bytes)};
}
bool overlap(Span a, Span b) { return a.lo < b.hi && b.lo < a.hi; }

// Validate phase `p` of the caller's CSR (the rules of the header: rows non-empty, indices in range, no duplicate
// in a row, weights finite and positive, row sums 1 within 1e-6) for up to `max_n` nodes.
int validate_phase(const char* fn, int32_t n, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                   int32_t p, int32_t max_n, int64_t* nnz_out) {
    if (n > max_n) return set_error(DL_ETOPO, "%s: n = %d exceeds the limit of %d nodes", fn, n, max_n);
    const int32_t* rp = row_ptr + static_cast<int64_t>(p) * (n + 1);
    const int64_t base = rp[0];
    const int64_t nnz = static_cast<int64_t>(rp[n]) - base;
    if (base < 0 || nnz < n) return set_error(DL_ETOPO, "%s: phase %d: row_ptr not monotone or a row is empty", fn, p);
    std::vector<int32_t> last_seen(static_cast<size_t>(n), -1);
    for (int32_t i = 0; i < n; ++i) {
        const int64_t b = rp[i], e = rp[i + 1];
        if (e <= b) return set_error(DL_ETOPO, "%s: phase %d row %d is empty or row_ptr decreases", fn, p, i);
        double sum = 0.0;
        for (int64_t q = b; q < e; ++q) {
            const int32_t j = col_idx[q];
            const float wij = w[q];
            if (j < 0 || j >= n)
                return set_error(DL_ETOPO, "%s: phase %d row %d: neighbour index %d outside [0, %d)", fn, p, i, j, n);
            if (last_seen[j] == i) return set_error(DL_ETOPO, "%s: phase %d row %d lists neighbour %d twice", fn, p, i, j);
            last_seen[j] = i;
            if (!std::isfinite(wij) || !(wij > 0.0f))
                return set_error(DL_ETOPO, "%s: phase %d: w[%d,%d] = %g must be finite and > 0", fn, p, i, j,
                                 static_cast<double>(wij));
            sum += static_cast<double>(wij);
        }
        if (std::fabs(sum - 1.0) > 1e-6)
            return set_error(DL_ETOPO, "%s: phase %d row %d sums to %.9g, not 1", fn, p, i, sum);
    }
    *nnz_out = nnz;
    return DL_OK;
}

// Validate phase `p` of the caller's CSR and copy it into kernel-argument form.
int pack_phase(const char* fn, int32_t n, const int32_t* row_ptr, const int32_t* col_idx,
               const float* w, int32_t p, PhaseArgs* out) {
    if (n > DL_MAX_NODES)
        return set_error(DL_ETOPO, "%s: n = %d exceeds DL_MAX_NODES = %d", fn, n, DL_MAX_NODES);
    const int32_t* rp = row_ptr + static_cast<int64_t>(p) * (n + 1);
    const int64_t base = rp[0];
    const int64_t nnz = static_cast<int64_t>(rp[n]) - base;
    if (base < 0 || nnz < n)
        return set_error(DL_ETOPO, "%s: phase %d: row_ptr not monotone or a row is empty", fn, p);
    if (nnz > kMaxNnzRowWeights)
        return set_error(DL_ETOPO, "%s: phase %d has %lld entries, limit DL_MAX_NNZ_ROW_WEIGHTS = %d", fn, p,
                         static_cast<long long>(nnz), kMaxNnzRowWeights);
    out->n = n;
    // first pass: validate, and collect the distinct weight values while there are few of them
    float values[kMaxWeightValues];
    int n_values = 0;
    bool few_values = true;
    bool one_value_per_row = true;
    int32_t last_seen[DL_MAX_NODES];
    for (int32_t j = 0; j < n; ++j) last_seen[j] = -1;
    for (int32_t i = 0; i < n; ++i) {
        const int64_t b = rp[i], e = rp[i + 1];
        if (e <= b)
            return set_error(DL_ETOPO, "%s: phase %d row %d is empty or row_ptr decreases", fn, p, i);
        out->row_ptr[i] = static_cast<uint16_t>(b - base);
        double sum = 0.0;
        for (int64_t q = b; q < e; ++q) {
            const int32_t j = col_idx[q];
            const float wij = w[q];
            if (j < 0 || j >= n)
                return set_error(DL_ETOPO, "%s: phase %d row %d: neighbour index %d outside [0, %d)",
                                 fn, p, i, j, n);
            if (last_seen[j] == i)
                return set_error(DL_ETOPO, "%s: phase %d row %d lists neighbour %d twice", fn, p, i, j);
            last_seen[j] = i;
            if (!std::isfinite(wij) || !(wij > 0.0f))
                return set_error(DL_ETOPO, "%s: phase %d: w[%d,%d] = %g must be finite and > 0", fn,
                                 p, i, j, static_cast<double>(wij));
            sum += static_cast<double>(wij);
            if (wij != w[b]) one_value_per_row = false;
            if (few_values) {
                int v = 0;
                while (v < n_values && values[v] != wij) ++v;
                if (v == n_values) {
                    if (n_values < kMaxWeightValues) values[n_values++] = wij;
                    else few_values = false;
                }
            }
        }
        if (std::fabs(sum - 1.0) > 1e-6)
            return set_error(DL_ETOPO, "%s: phase %d row %d sums to %.9g, not 1", fn, p, i, sum);
    }
    out->row_ptr[n] = static_cast<uint16_t>(nnz);
    // second pass: encode; the direct form while it fits (one load per entry in the kernel, where the
    // palette needs a second, dependent one)
    if (nnz <= DL_MAX_NNZ) {
        out->palette = 0;
        for (int64_t q = 0; q < nnz; ++q) {
            out->direct.col[q] = static_cast<uint8_t>(col_idx[base + q]);
            out->direct.w[q] = w[base + q];
        }
        return DL_OK;
    }
    if (!few_values)
        return set_error(DL_ETOPO, "%s: phase %d has %lld entries with more than %d distinct weights, "
                         "limit DL_MAX_NNZ = %d", fn, p, static_cast<long long>(nnz), kMaxWeightValues, DL_MAX_NNZ);
    if (nnz > kMaxNnzPalette) {
        if (!one_value_per_row)
            return set_error(DL_ETOPO, "%s: phase %d has %lld entries and rows of mixed weights, limit "
                             "DL_MAX_NNZ_PALETTE = %d", fn, p, static_cast<long long>(nnz), kMaxNnzPalette);
        out->palette = 2;
        for (int v = 0; v < n_values; ++v) out->rows.value[v] = values[v];
        for (int64_t q = 0; q < nnz; ++q) out->rows.col[q] = static_cast<uint8_t>(col_idx[base + q]);
        for (int32_t i = 0; i < n; ++i) {
            int v = 0;
            while (values[v] != w[rp[i]]) ++v;
            out->rows.widx[i] = static_cast<uint8_t>(v);
        }
        return DL_OK;
    }
    out->palette = 1;
    for (int v = 0; v < n_values; ++v) out->pal.value[v] = values[v];
    for (int64_t q = 0; q < nnz; ++q) {
        out->pal.col[q] = static_cast<uint8_t>(col_idx[base + q]);
        int v = 0;
        while (values[v] != w[base + q]) ++v;
        out->pal.widx[q] = static_cast<uint8_t>(v);
    }
    return DL_OK;
}

// Optional extras of a step call: a gradient format other than fp32 with its own row stride, and
// the tensor table with its outputs.
struct StepExtras {
    int g_format = DL_GRAD_F32;
    int64_t ldg = -1;               // -1: same as ld
    bool multi = false;
    int32_t num_tensors = 0;
    const int64_t* offsets = nullptr;   // host
    double* norms = nullptr;            // device or NULL
    void* workspace = nullptr;
    size_t workspace_bytes = 0;
};

size_t multi_workspace_bytes(int32_t n, int64_t d) {
    return static_cast<size_t>(norm_tiles_bound(d)) * static_cast<size_t>(n) * 3 * sizeof(double);
}

// Checks shared by every step entry point: scalar arguments and the presence of W.
int check_step_scalars(const char* fn, Algo algo, int32_t n, int g_format, float gamma, float gamma_prev, float beta,
                       int64_t k, int32_t period, const int32_t* row_ptr, const int32_t* col_idx, const float* w) {
    if (algo == ALGO_DECENTLAM_XPREV && (!std::isfinite(gamma_prev) || !(gamma_prev > 0.0f)))
        return set_error(DL_EINVAL, "%s: gamma_prev = %g must be finite and > 0", fn, static_cast<double>(gamma_prev));
    if (n < 1) return set_error(DL_EINVAL, "%s: n = %d, need n >= 1", fn, n);
    if (g_format != DL_GRAD_F32 && g_format != DL_GRAD_BF16 && g_format != DL_GRAD_F16)
        return set_error(DL_EINVAL, "%s: g_format = %d is not a dl_grad_format", fn, g_format);
    if (!std::isfinite(gamma) || !(gamma > 0.0f))
        return set_error(DL_EINVAL, "%s: gamma = %g must be finite and > 0", fn, static_cast<double>(gamma));
    if (!(beta >= 0.0f && beta < 1.0f))
        return set_error(DL_EINVAL, "%s: beta = %g must lie in [0, 1)", fn, static_cast<double>(beta));
    if (k < 0) return set_error(DL_EINVAL, "%s: k = %lld, need k >= 0", fn, static_cast<long long>(k));
    if (period < 1) return set_error(DL_EINVAL, "%s: period = %d, need period >= 1", fn, period);
    if (!row_ptr || !col_idx || !w)
        return set_error(DL_EINVAL, "%s: row_ptr, col_idx and w must not be NULL", fn);
    return DL_OK;
}

// A packed topology (topology_pack): a header, then `period` phases in kernel-argument form.  Caller-owned
// host memory; the library keeps no reference to it.
constexpr uint32_t kPackedMagic = 0x444C5450u;   // "DLTP"
struct PackedHeader {
    uint32_t magic;
    int32_t n;
    int32_t period;
    uint32_t phase_bytes;   // sizeof(PhaseArgs) of the library that packed it
};
static_assert(sizeof(PackedHeader) == 16 && sizeof(PhaseArgs) % 4 == 0, "phases follow the header, 4-byte aligned");

// The phase of a packed topology that iteration k uses.
int packed_phase(const char* fn, const void* packed, int32_t n, int64_t k, const PhaseArgs** out) {
    if (!packed) return set_error(DL_EINVAL, "%s: packed must not be NULL", fn);
    if (reinterpret_cast<uintptr_t>(packed) & 3u) return set_error(DL_EINVAL, "%s: packed must be 4-byte aligned", fn);
    const PackedHeader* h = static_cast<const PackedHeader*>(packed);
    if (h->magic != kPackedMagic || h->phase_bytes != sizeof(PhaseArgs) || h->period < 1 || h->n < 1)
        return set_error(DL_ETOPO, "%s: packed was not written by this library's topology_pack", fn);
    if (h->n != n)
        return set_error(DL_ETOPO, "%s: packed topology has %d nodes, the arrays have %d rows", fn, h->n, n);
    if (k < 0) return set_error(DL_EINVAL, "%s: k = %lld, need k >= 0", fn, static_cast<long long>(k));
    const char* phases = static_cast<const char*>(packed) + sizeof(PackedHeader);
    *out = reinterpret_cast<const PhaseArgs*>(phases + static_cast<size_t>(k % h->period) * sizeof(PhaseArgs));
    return DL_OK;
}

// The tensor table of a multi-tensor call: at least one tensor, offsets that do not decrease.
int check_offsets(const char* fn, int32_t num_tensors, const int64_t* offsets) {
    if (num_tensors < 1) return set_error(DL_EINVAL, "%s: num_tensors = %d, need >= 1", fn, num_tensors);
    if (!offsets) return set_error(DL_EINVAL, "%s: offsets must not be NULL", fn);
    if (offsets[0] < 0)
        return set_error(DL_EINVAL, "%s: offsets[0] = %lld < 0", fn, static_cast<long long>(offsets[0]));
    for (int32_t t = 0; t < num_tensors; ++t)
        if (offsets[t + 1] < offsets[t]) return set_error(DL_EINVAL, "%s: offsets decrease at tensor %d", fn, t);
    return DL_OK;
}

// Workspace and output of the per-tensor sums: present, large enough, 8-byte aligned.
int check_norms_buffers(const char* fn, int32_t n, int64_t d, const void* workspace, size_t workspace_bytes,
                        const double* norms) {
    const size_t need = multi_workspace_bytes(n, d);
    if (!workspace || workspace_bytes < need)
        return set_error(DL_ECAP, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                         workspace ? workspace_bytes : size_t{0});
    if ((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(norms)) & 7u)
        return set_error(DL_EINVAL, "%s: workspace and norms must be 8-byte aligned", fn);
    return DL_OK;
}

int step_entry(const char* fn, Algo algo, float* x, float* m, const void* g, int32_t n, int64_t d,
               int64_t ld, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
               int32_t period, float gamma, float beta, int64_t k, void* stream, float gamma_prev = 0.0f,
               const StepExtras& ex = StepExtras(), const void* packed = nullptr, bool use_packed = false,
               const dl_device_topology* device_topo = nullptr, bool use_device = false) {
    clear_error();
    static const int32_t kNoRows[2] = {0, 0};
    static const float kNoWeight[1] = {0.f};
    if (use_packed || use_device) {   // W comes validated and encoded: only its presence is checked below
        row_ptr = col_idx = kNoRows;
        w = kNoWeight;
        period = 1;
    }
    if (int rc = check_step_scalars(fn, algo, n, ex.g_format, gamma, gamma_prev, beta, k, period, row_ptr, col_idx, w))
        return rc;
    int64_t col0 = 0;
    if (ex.multi) {   // the tensor table fixes the column range
        if (int rc = check_offsets(fn, ex.num_tensors, ex.offsets)) return rc;
        col0 = ex.offsets[0];
        d = ex.offsets[ex.num_tensors] - col0;
        if (ex.offsets[ex.num_tensors] > ld)
            return set_error(DL_EINVAL, "%s: offsets end at %lld > ld = %lld", fn,
                             static_cast<long long>(ex.offsets[ex.num_tensors]), static_cast<long long>(ld));
    }
    if (d < 0) return set_error(DL_EINVAL, "%s: d = %lld, need d >= 0", fn, static_cast<long long>(d));
    if (ld < d)
        return set_error(DL_EINVAL, "%s: ld = %lld < d = %lld", fn, static_cast<long long>(ld),
                         static_cast<long long>(d));
    const int64_t ldg = ex.ldg < 0 ? ld : ex.ldg;
    if (ldg < col0 + d)
        return set_error(DL_EINVAL, "%s: ldg = %lld does not cover the columns", fn, static_cast<long long>(ldg));

    PhaseArgs packed_now;
    const PhaseArgs* phase = nullptr;
    if (use_device) {
        if (!device_topo) return set_error(DL_EINVAL, "%s: W must not be NULL", fn);
        if (device_topo->magic != kDeviceTopoMagic || !device_topo->device || device_topo->period < 1)
            return set_error(DL_ETOPO, "%s: W was not written by topology_pack_device", fn);
        if (device_topo->n != n)
            return set_error(DL_ETOPO, "%s: W has %d nodes, the arrays have %d rows", fn, device_topo->n, n);
        std::memset(&packed_now, 0, sizeof(packed_now));   // not used by this path
        phase = &packed_now;
    } else if (use_packed) {
        if (int rc = packed_phase(fn, packed, n, k, &phase)) return rc;
    } else {
        std::memset(&packed_now, 0, sizeof(packed_now));
        if (int rc = pack_phase(fn, n, row_ptr, col_idx, w, static_cast<int32_t>(k % period), &packed_now)) return rc;
        phase = &packed_now;
    }
    const PhaseArgs& topo = *phase;

    const bool want_norms = ex.multi && ex.norms != nullptr;
    if (want_norms) {
        if (int rc = check_norms_buffers(fn, n, d, ex.workspace, ex.workspace_bytes, ex.norms)) return rc;
    }
    if (d == 0 && !want_norms) return DL_OK;
    const bool uses_m = algo != ALGO_DSGD;
    if (!x || !g || (uses_m && !m)) return set_error(DL_EINVAL, "%s: x, m and g must not be NULL", fn);
    const uintptr_t gbytes = grad_elem_bytes(ex.g_format);
    if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m)) & 3u) ||
        (reinterpret_cast<uintptr_t>(g) & (gbytes - 1)))
        return set_error(DL_EINVAL, "%s: x, m and g must be aligned to their element size", fn);
    x += col0;
    if (m) m += col0;
    g = static_cast<const char*>(g) + static_cast<size_t>(col0) * gbytes;
    const Span sx = span_of(x, n, d, ld), sm = span_of(m, n, d, ld), sg = span_of(g, n, d, ldg, gbytes);
    // Rows of different arrays may interleave when ld > d (views of one padded buffer); what
    // must not happen is that the arrays share elements.  Whole-span overlap is only an error
    // if the arrays are not column-disjoint views with the same stride.
    auto shares = [&](const void* a, Span sa, const void* b2, Span sb) {
        if (!overlap(sa, sb)) return false;
        const intptr_t delta = (reinterpret_cast<intptr_t>(a) - reinterpret_cast<intptr_t>(b2)) / 4;
        const int64_t off = ((delta % ld) + ld) % ld;  // column offset between the two views
        return !(off >= d && ld - off >= d);
    };
    const bool g_like_x = ex.g_format == DL_GRAD_F32 && ldg == ld;
    auto g_shares = [&](const void* a, Span sa) { return g_like_x ? shares(a, sa, g, sg) : overlap(sa, sg); };
    if ((uses_m && (shares(x, sx, m, sm) || g_shares(m, sm))) || g_shares(x, sx))
        return set_error(DL_EALIAS, "%s: x, m and g must not overlap", fn);

    double beta_eff = static_cast<double>(beta);
    if (algo == ALGO_DECENTLAM_XPREV)
        beta_eff = beta_eff * static_cast<double>(gamma) / static_cast<double>(gamma_prev);
    const GradArg ga{g, ex.g_format, ldg};
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (use_device) {
        const Span st = {reinterpret_cast<uintptr_t>(device_topo->device),
                         reinterpret_cast<uintptr_t>(device_topo->device) + static_cast<uintptr_t>(device_topo->device_bytes)};
        if (overlap(st, sx) || (uses_m && overlap(st, sm)))
            return set_error(DL_EALIAS, "%s: W's device buffer overlaps x or m", fn);
        return launch_step_wide(algo, x, m, static_cast<const float*>(g), n, d, ld, gamma, beta_eff, device_topo->device,
                                static_cast<int32_t>(k % device_topo->period), s);
    }
    if (!want_norms) return launch_step(algo, x, m, ga, n, d, ld, topo, gamma, beta_eff, s);

    const size_t need = multi_workspace_bytes(n, d);
    const Span sw = {reinterpret_cast<uintptr_t>(ex.workspace), reinterpret_cast<uintptr_t>(ex.workspace) + need};
    const Span sn = span_of(ex.norms, 1, static_cast<int64_t>(ex.num_tensors) * n * 3,
                            static_cast<int64_t>(ex.num_tensors) * n * 3, 8);
    if (overlap(sw, sn) || overlap(sw, sx) || overlap(sw, sm) || overlap(sw, sg) || overlap(sn, sx) ||
        overlap(sn, sm) || overlap(sn, sg))
        return set_error(DL_EALIAS, "%s: norms / workspace overlap another array", fn);
    NormPlan plan;
    std::memset(&plan, 0, sizeof(plan));
    plan.offsets = ex.offsets;
    plan.num_tensors = ex.num_tensors;
    plan.partial = static_cast<double*>(ex.workspace);
    plan.capacity = norm_tiles_bound(d);
    plan.norms = ex.norms;
    if (int rc = launch_step(algo, x, m, ga, n, d, ld, topo, gamma, beta_eff, s, &plan)) return rc;
    return launch_norms_finish(plan, x, m, ga, ld, n, s);
}

// Blocked layout: the n x d problem is stored as ceil(d / bw) blocks of bw columns, each block a
// row-major n x bw matrix (row stride bw), blocks back to back: element (i, c) lives at
// ((c / bw) * n + i) * bw + c % bw.  The full blocks are one batched launch, a narrower last block
// is an ordinary row-major problem with ld = bw.
int blocked_entry(const char* fn, Algo algo, float* x, float* m, const void* g, int32_t n, int64_t d,
                  int64_t bw, const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  float gamma, float beta, int64_t k, void* stream, int g_format = DL_GRAD_F32,
                  float gamma_prev = 0.0f, const StepExtras* multi = nullptr) {
    clear_error();
    if (multi) {   // the tensor table fixes d
        if (int rc = check_offsets(fn, multi->num_tensors, multi->offsets)) return rc;
        if (multi->offsets[0] != 0)
            return set_error(DL_EINVAL, "%s: offsets[0] = %lld; in the blocked layout the table starts at column 0",
                             fn, static_cast<long long>(multi->offsets[0]));
        d = multi->offsets[multi->num_tensors];
    }
    if (int rc = check_step_scalars(fn, algo, n, g_format, gamma, gamma_prev, beta, k, period, row_ptr, col_idx, w))
        return rc;
    if (d < 0) return set_error(DL_EINVAL, "%s: d = %lld, need d >= 0", fn, static_cast<long long>(d));
    if (bw < 1) return set_error(DL_EINVAL, "%s: bw = %lld, need bw >= 1", fn, static_cast<long long>(bw));
    PhaseArgs topo;
    std::memset(&topo, 0, sizeof(topo));
    if (int rc = pack_phase(fn, n, row_ptr, col_idx, w, static_cast<int32_t>(k % period), &topo)) return rc;
    const bool want_norms = multi && multi->norms != nullptr;
    if (want_norms) {
        if (int rc = check_norms_buffers(fn, n, d, multi->workspace, multi->workspace_bytes, multi->norms)) return rc;
        // whole tiles per block and no peeled columns: the tile records then line up with the columns
        if (bw % 256 != 0 || ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m)) & 15u) ||
            (reinterpret_cast<uintptr_t>(g) & (4 * grad_elem_bytes(g_format) - 1)))
            return set_error(DL_EINVAL, "%s: per-tensor sums in the blocked layout need bw %% 256 == 0 and "
                             "16-byte aligned x, m (g: 4 elements)", fn);
    }
    if (d == 0 && !want_norms) return DL_OK;
    if (!x || !m || !g) return set_error(DL_EINVAL, "%s: x, m and g must not be NULL", fn);
    const uintptr_t gbytes = grad_elem_bytes(g_format);
    if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m)) & 3u) ||
        (reinterpret_cast<uintptr_t>(g) & (gbytes - 1)))
        return set_error(DL_EINVAL, "%s: x, m and g must be aligned to their element size", fn);
    const int64_t full = d / bw, rest = d % bw;
    const int64_t block = static_cast<int64_t>(n) * bw;
    const int64_t elements = full * block + (rest ? (static_cast<int64_t>(n) - 1) * bw + rest : 0);
    const Span sx = span_of(x, 1, elements, elements), sm = span_of(m, 1, elements, elements),
               sg = span_of(g, 1, elements, elements, static_cast<int64_t>(gbytes));
    if (overlap(sx, sm) || overlap(sx, sg) || overlap(sm, sg))
        return set_error(DL_EALIAS, "%s: x, m and g must not overlap", fn);
    double beta_eff = static_cast<double>(beta);
    if (algo == ALGO_DECENTLAM_XPREV)
        beta_eff = beta_eff * static_cast<double>(gamma) / static_cast<double>(gamma_prev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    NormPlan plan;
    std::memset(&plan, 0, sizeof(plan));
    NormPlan* np = nullptr;
    if (want_norms) {
        const size_t need = multi_workspace_bytes(n, d);
        const Span sw = {reinterpret_cast<uintptr_t>(multi->workspace),
                         reinterpret_cast<uintptr_t>(multi->workspace) + need};
        const int64_t count = static_cast<int64_t>(multi->num_tensors) * n * 3;
        const Span sn = span_of(multi->norms, 1, count, count, 8);
        if (overlap(sw, sn) || overlap(sw, sx) || overlap(sw, sm) || overlap(sw, sg) || overlap(sn, sx) ||
            overlap(sn, sm) || overlap(sn, sg))
            return set_error(DL_EALIAS, "%s: norms / workspace overlap another array", fn);
        plan.offsets = multi->offsets;
        plan.num_tensors = multi->num_tensors;
        plan.partial = static_cast<double*>(multi->workspace);
        plan.capacity = norm_tiles_bound(d);
        plan.norms = multi->norms;
        plan.bw = bw;
        np = &plan;
    }
    if (full > 0) {
        if (int rc = launch_step(algo, x, m, GradArg{g, g_format, bw}, n, bw, bw, topo, gamma, beta_eff, s, np,
                                 full, block, block))
            return rc;
    }
    if (rest > 0) {
        const int64_t at = full * block;
        const void* g_rest = static_cast<const char*>(g) + static_cast<size_t>(at) * gbytes;
        plan.col_base = full * bw;
        if (int rc = launch_step(algo, x + at, m + at, GradArg{g_rest, g_format, bw}, n, rest, bw, topo, gamma,
                                 beta_eff, s, np))
            return rc;
    }
    if (np) return launch_norms_finish(plan, x, m, GradArg{g, g_format, bw}, bw, n, s);
    return DL_OK;
}

}  // namespace
}  // namespace dl

extern "C" {

int decentlam_step(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                   const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                   float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("decentlam_step", dl::ALGO_DECENTLAM, x, m, g, n, d, ld, row_ptr, col_idx, w,
                          period, gamma, beta, k, stream);
}

int dmsgd_step(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
               const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
               float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("dmsgd_step", dl::ALGO_DMSGD, x, m, g, n, d, ld, row_ptr, col_idx, w, period,
                          gamma, beta, k, stream);
}

size_t topology_pack_bytes(int32_t n, int32_t period) {
    if (n < 1 || n > DL_MAX_NODES || period < 1) return 0;
    return sizeof(dl::PackedHeader) + static_cast<size_t>(period) * sizeof(dl::PhaseArgs);
}

int topology_pack(int32_t n, const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  void* packed, size_t packed_bytes) {
    using namespace dl;
    const char* fn = "topology_pack";
    clear_error();
    if (n < 1) return set_error(DL_EINVAL, "%s: n = %d, need n >= 1", fn, n);
    if (period < 1) return set_error(DL_EINVAL, "%s: period = %d, need period >= 1", fn, period);
    if (!row_ptr || !col_idx || !w || !packed)
        return set_error(DL_EINVAL, "%s: row_ptr, col_idx, w and packed must not be NULL", fn);
    if (n > DL_MAX_NODES) return set_error(DL_ETOPO, "%s: n = %d exceeds DL_MAX_NODES = %d", fn, n, DL_MAX_NODES);
    if (reinterpret_cast<uintptr_t>(packed) & 3u) return set_error(DL_EINVAL, "%s: packed must be 4-byte aligned", fn);
    const size_t need = topology_pack_bytes(n, period);
    if (packed_bytes < need)
        return set_error(DL_ECAP, "%s: packed needs %zu bytes (topology_pack_bytes), %zu given", fn, need, packed_bytes);
    // every phase is validated and encoded before the header is written: a failed call leaves no valid buffer
    PackedHeader* h = static_cast<PackedHeader*>(packed);
    h->magic = 0;
    char* phases = static_cast<char*>(packed) + sizeof(PackedHeader);
    for (int32_t p = 0; p < period; ++p) {
        PhaseArgs* out = reinterpret_cast<PhaseArgs*>(phases + static_cast<size_t>(p) * sizeof(PhaseArgs));
        std::memset(out, 0, sizeof(PhaseArgs));
        if (int rc = pack_phase(fn, n, row_ptr, col_idx, w, p, out)) return rc;
    }
    h->n = n;
    h->period = period;
    h->phase_bytes = static_cast<uint32_t>(sizeof(PhaseArgs));
    h->magic = kPackedMagic;
    return DL_OK;
}

int decentlam_step_packed(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, const void* packed,
                          float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("decentlam_step_packed", dl::ALGO_DECENTLAM, x, m, g, n, d, ld, nullptr, nullptr, nullptr, 1,
                          gamma, beta, k, stream, 0.0f, dl::StepExtras(), packed, true);
}

int dmsgd_step_packed(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, const void* packed,
                      float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("dmsgd_step_packed", dl::ALGO_DMSGD, x, m, g, n, d, ld, nullptr, nullptr, nullptr, 1, gamma,
                          beta, k, stream, 0.0f, dl::StepExtras(), packed, true);
}

int dsgd_step_packed(float* x, const float* g, int32_t n, int64_t d, int64_t ld, const void* packed, float gamma,
                     int64_t k, void* stream) {
    return dl::step_entry("dsgd_step_packed", dl::ALGO_DSGD, x, nullptr, g, n, d, ld, nullptr, nullptr, nullptr, 1, gamma,
                          0.0f, k, stream, 0.0f, dl::StepExtras(), packed, true);
}

size_t topology_device_bytes(int32_t n, int32_t period, int64_t nnz_total) {
    if (n < 1 || n > DL_MAX_NODES_DEVICE || period < 1 || nnz_total < 0) return 0;
    const size_t words = static_cast<size_t>(dl::kDeviceTopoHeaderWords) + ((static_cast<size_t>(period) + 1) & ~size_t{1}) +
                         static_cast<size_t>(period) * dl::device_topo_row_ptr_words(n) + 2 * static_cast<size_t>(nnz_total);
    return words * 4;
}

int topology_pack_device(int32_t n, const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                         void* device_buffer, size_t device_bytes, dl_device_topology* out) {
    using namespace dl;
    const char* fn = "topology_pack_device";
    clear_error();
    if (n < 1) return set_error(DL_EINVAL, "%s: n = %d, need n >= 1", fn, n);
    if (period < 1) return set_error(DL_EINVAL, "%s: period = %d, need period >= 1", fn, period);
    if (!row_ptr || !col_idx || !w || !device_buffer || !out)
        return set_error(DL_EINVAL, "%s: row_ptr, col_idx, w, device_buffer and out must not be NULL", fn);
    if (reinterpret_cast<uintptr_t>(device_buffer) & 7u) return set_error(DL_EINVAL, "%s: device_buffer must be 8-byte aligned", fn);
    out->magic = 0;
    int64_t total = 0;
    for (int32_t p = 0; p < period; ++p) {
        int64_t nnz = 0;
        if (int rc = validate_phase(fn, n, row_ptr, col_idx, w, p, DL_MAX_NODES_DEVICE, &nnz)) return rc;
        total += nnz;
    }
    const size_t need = topology_device_bytes(n, period, total);
    if (device_bytes < need)
        return set_error(DL_ECAP, "%s: device_buffer needs %zu bytes (topology_device_bytes), %zu given", fn, need, device_bytes);
    std::vector<uint32_t> img(need / 4, 0u);
    img[0] = kDeviceTopoMagic;
    img[1] = static_cast<uint32_t>(n);
    img[2] = static_cast<uint32_t>(period);
    size_t at = static_cast<size_t>(kDeviceTopoHeaderWords) + ((static_cast<size_t>(period) + 1) & ~size_t{1});
    for (int32_t p = 0; p < period; ++p) {
        const int32_t* rp = row_ptr + static_cast<int64_t>(p) * (n + 1);
        img[kDeviceTopoHeaderWords + p] = static_cast<uint32_t>(at);
        for (int32_t i = 0; i <= n; ++i) img[at + i] = static_cast<uint32_t>(rp[i] - rp[0]);
        at += device_topo_row_ptr_words(n);
        for (int64_t q = rp[0]; q < rp[n]; ++q) {
            img[at++] = static_cast<uint32_t>(col_idx[q]);
            uint32_t bits;
            std::memcpy(&bits, &w[q], 4);
            img[at++] = bits;
        }
    }
    // a set-up call: the copy is synchronous, so the host image may go when the call returns
    if (int rc = check_hip(hipMemcpy(device_buffer, img.data(), need, hipMemcpyHostToDevice), "hipMemcpy(topology)")) return rc;
    out->n = n;
    out->period = period;
    out->device = device_buffer;
    out->device_bytes = need;
    out->magic = kDeviceTopoMagic;
    return DL_OK;
}

int decentlam_step_dev(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, const dl_device_topology* W,
                       float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("decentlam_step_dev", dl::ALGO_DECENTLAM, x, m, g, n, d, ld, nullptr, nullptr, nullptr, 1, gamma,
                          beta, k, stream, 0.0f, dl::StepExtras(), nullptr, false, W, true);
}

int dmsgd_step_dev(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, const dl_device_topology* W,
                   float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("dmsgd_step_dev", dl::ALGO_DMSGD, x, m, g, n, d, ld, nullptr, nullptr, nullptr, 1, gamma, beta, k,
                          stream, 0.0f, dl::StepExtras(), nullptr, false, W, true);
}

int dsgd_step_dev(float* x, const float* g, int32_t n, int64_t d, int64_t ld, const dl_device_topology* W, float gamma,
                  int64_t k, void* stream) {
    return dl::step_entry("dsgd_step_dev", dl::ALGO_DSGD, x, nullptr, g, n, d, ld, nullptr, nullptr, nullptr, 1, gamma, 0.0f,
                          k, stream, 0.0f, dl::StepExtras(), nullptr, false, W, true);
}

int decentlam_step_blocked(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t bw,
                           const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                           float gamma, float beta, int64_t k, void* stream) {
    return dl::blocked_entry("decentlam_step_blocked", dl::ALGO_DECENTLAM, x, m, g, n, d, bw, row_ptr, col_idx, w,
                             period, gamma, beta, k, stream);
}

int dmsgd_step_blocked(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t bw,
                       const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                       float gamma, float beta, int64_t k, void* stream) {
    return dl::blocked_entry("dmsgd_step_blocked", dl::ALGO_DMSGD, x, m, g, n, d, bw, row_ptr, col_idx, w, period,
                             gamma, beta, k, stream);
}

namespace dl {
namespace {
// The general form: layout and gradient format from a dl_layout.
int ex_entry(const char* fn, Algo algo, float* x, float* m, const void* g, int32_t n, int64_t d,
             const dl_layout* layout, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
             int32_t period, float gamma, float gamma_prev, float beta, int64_t k, void* stream) {
    if (!layout) {
        clear_error();
        return set_error(DL_EINVAL, "%s: layout must not be NULL", fn);
    }
    if (layout->bw > 0)
        return blocked_entry(fn, algo, x, m, g, n, d, layout->bw, row_ptr, col_idx, w, period, gamma, beta, k,
                             stream, layout->g_format, gamma_prev);
    if (layout->bw < 0) {
        clear_error();
        return set_error(DL_EINVAL, "%s: layout.bw = %lld, need >= 0", fn, static_cast<long long>(layout->bw));
    }
    StepExtras ex;
    ex.g_format = layout->g_format;
    ex.ldg = layout->ldg;
    return step_entry(fn, algo, x, m, g, n, d, layout->ld, row_ptr, col_idx, w, period, gamma, beta, k, stream,
                      gamma_prev, ex);
}
}  // namespace
}  // namespace dl

int decentlam_step_ex(float* x, float* m, const void* g, int32_t n, int64_t d, const dl_layout* layout,
                      const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                      float gamma, float beta, int64_t k, void* stream) {
    return dl::ex_entry("decentlam_step_ex", dl::ALGO_DECENTLAM, x, m, g, n, d, layout, row_ptr, col_idx, w, period,
                        gamma, 0.0f, beta, k, stream);
}

int dmsgd_step_ex(float* x, float* m, const void* g, int32_t n, int64_t d, const dl_layout* layout,
                  const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  float gamma, float beta, int64_t k, void* stream) {
    return dl::ex_entry("dmsgd_step_ex", dl::ALGO_DMSGD, x, m, g, n, d, layout, row_ptr, col_idx, w, period, gamma,
                        0.0f, beta, k, stream);
}

int awc_dmsgd_step_ex(float* x, float* m, const void* g, int32_t n, int64_t d, const dl_layout* layout,
                      const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                      float gamma, float beta, int64_t k, void* stream) {
    return dl::ex_entry("awc_dmsgd_step_ex", dl::ALGO_AWC_DMSGD, x, m, g, n, d, layout, row_ptr, col_idx, w, period, gamma,
                        0.0f, beta, k, stream);
}

int da_dmsgd_step_ex(float* x, float* m, const void* g, int32_t n, int64_t d, const dl_layout* layout,
                     const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                     float gamma, float beta, int64_t k, void* stream) {
    return dl::ex_entry("da_dmsgd_step_ex", dl::ALGO_DA_DMSGD, x, m, g, n, d, layout, row_ptr, col_idx, w, period, gamma,
                        0.0f, beta, k, stream);
}

int decentlam_step_xprev_ex(const float* x, float* x_prev, const void* g, int32_t n, int64_t d,
                            const dl_layout* layout, const int32_t* row_ptr, const int32_t* col_idx,
                            const float* w, int32_t period, float gamma, float gamma_prev, float beta, int64_t k,
                            void* stream) {
    return dl::ex_entry("decentlam_step_xprev_ex", dl::ALGO_DECENTLAM_XPREV, const_cast<float*>(x), x_prev, g, n, d,
                        layout, row_ptr, col_idx, w, period, gamma, gamma_prev, beta, k, stream);
}

namespace dl {
namespace {
int multi_ex_entry(const char* fn, Algo algo, float* x, float* m, const void* g, int32_t n,
                   const dl_layout* layout, int32_t num_tensors, const int64_t* offsets, double* norms,
                   void* workspace, size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx,
                   const float* w, int32_t period, float gamma, float beta, int64_t k, void* stream) {
    if (!layout) {
        clear_error();
        return set_error(DL_EINVAL, "%s: layout must not be NULL", fn);
    }
    if (layout->bw < 0) {
        clear_error();
        return set_error(DL_EINVAL, "%s: layout.bw = %lld, need >= 0", fn, static_cast<long long>(layout->bw));
    }
    StepExtras ex;
    ex.g_format = layout->g_format;
    ex.ldg = layout->ldg;
    ex.multi = true;
    ex.num_tensors = num_tensors;
    ex.offsets = offsets;
    ex.norms = norms;
    ex.workspace = workspace;
    ex.workspace_bytes = workspace_bytes;
    if (layout->bw > 0)
        return blocked_entry(fn, algo, x, m, g, n, 0, layout->bw, row_ptr, col_idx, w, period, gamma, beta, k, stream,
                             layout->g_format, 0.0f, &ex);
    return step_entry(fn, algo, x, m, g, n, 0, layout->ld, row_ptr, col_idx, w, period, gamma, beta, k, stream, 0.0f,
                      ex);
}
}  // namespace
}  // namespace dl

int decentlam_step_multi_ex(float* x, float* m, const void* g, int32_t n, const dl_layout* layout,
                            int32_t num_tensors, const int64_t* offsets, double* norms, void* workspace,
                            size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                            int32_t period, float gamma, float beta, int64_t k, void* stream) {
    return dl::multi_ex_entry("decentlam_step_multi_ex", dl::ALGO_DECENTLAM, x, m, g, n, layout, num_tensors, offsets,
                              norms, workspace, workspace_bytes, row_ptr, col_idx, w, period, gamma, beta, k, stream);
}

int dmsgd_step_multi_ex(float* x, float* m, const void* g, int32_t n, const dl_layout* layout,
                        int32_t num_tensors, const int64_t* offsets, double* norms, void* workspace,
                        size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                        int32_t period, float gamma, float beta, int64_t k, void* stream) {
    return dl::multi_ex_entry("dmsgd_step_multi_ex", dl::ALGO_DMSGD, x, m, g, n, layout, num_tensors, offsets, norms,
                              workspace, workspace_bytes, row_ptr, col_idx, w, period, gamma, beta, k, stream);
}

int awc_dmsgd_step_multi_ex(float* x, float* m, const void* g, int32_t n, const dl_layout* layout,
                            int32_t num_tensors, const int64_t* offsets, double* norms, void* workspace,
                            size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                            int32_t period, float gamma, float beta, int64_t k, void* stream) {
    return dl::multi_ex_entry("awc_dmsgd_step_multi_ex", dl::ALGO_AWC_DMSGD, x, m, g, n, layout, num_tensors, offsets, norms,
                              workspace, workspace_bytes, row_ptr, col_idx, w, period, gamma, beta, k, stream);
}

int da_dmsgd_step_multi_ex(float* x, float* m, const void* g, int32_t n, const dl_layout* layout,
                           int32_t num_tensors, const int64_t* offsets, double* norms, void* workspace,
                           size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                           int32_t period, float gamma, float beta, int64_t k, void* stream) {
    return dl::multi_ex_entry("da_dmsgd_step_multi_ex", dl::ALGO_DA_DMSGD, x, m, g, n, layout, num_tensors, offsets, norms,
                              workspace, workspace_bytes, row_ptr, col_idx, w, period, gamma, beta, k, stream);
}

int awc_dmsgd_step(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                   const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                   float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("awc_dmsgd_step", dl::ALGO_AWC_DMSGD, x, m, g, n, d, ld, row_ptr, col_idx, w, period,
                          gamma, beta, k, stream);
}

int da_dmsgd_step(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                  const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  float gamma, float beta, int64_t k, void* stream) {
    return dl::step_entry("da_dmsgd_step", dl::ALGO_DA_DMSGD, x, m, g, n, d, ld, row_ptr, col_idx, w, period,
                          gamma, beta, k, stream);
}

int decentlam_step_g16(float* x, float* m, const void* g, int32_t g_format, int32_t n, int64_t d, int64_t ld,
                       int64_t ldg, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                       int32_t period, float gamma, float beta, int64_t k, void* stream) {
    dl::StepExtras ex;
    ex.g_format = g_format;
    ex.ldg = ldg;
    return dl::step_entry("decentlam_step_g16", dl::ALGO_DECENTLAM, x, m, g, n, d, ld, row_ptr, col_idx, w,
                          period, gamma, beta, k, stream, 0.0f, ex);
}

int dmsgd_step_g16(float* x, float* m, const void* g, int32_t g_format, int32_t n, int64_t d, int64_t ld,
                   int64_t ldg, const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                   float gamma, float beta, int64_t k, void* stream) {
    dl::StepExtras ex;
    ex.g_format = g_format;
    ex.ldg = ldg;
    return dl::step_entry("dmsgd_step_g16", dl::ALGO_DMSGD, x, m, g, n, d, ld, row_ptr, col_idx, w, period,
                          gamma, beta, k, stream, 0.0f, ex);
}

size_t decentlam_step_multi_workspace(int32_t n, int64_t d, int32_t num_tensors) {
    if (n < 1 || d < 0 || num_tensors < 1) return 0;
    return dl::multi_workspace_bytes(n, d);
}

namespace dl {
namespace {
int multi_entry(const char* fn, Algo algo, float* x, float* m, const void* g, int32_t g_format, int32_t n,
                int64_t ld, int64_t ldg, int32_t num_tensors, const int64_t* offsets, double* norms,
                void* workspace, size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx,
                const float* w, int32_t period, float gamma, float beta, int64_t k, void* stream) {
    StepExtras ex;
    ex.g_format = g_format;
    ex.ldg = ldg;
    ex.multi = true;
    ex.num_tensors = num_tensors;
    ex.offsets = offsets;
    ex.norms = norms;
    ex.workspace = workspace;
    ex.workspace_bytes = workspace_bytes;
    return step_entry(fn, algo, x, m, g, n, 0, ld, row_ptr, col_idx, w, period, gamma, beta, k, stream, 0.0f, ex);
}
}  // namespace
}  // namespace dl

int decentlam_step_multi(float* x, float* m, const void* g, int32_t g_format, int32_t n, int64_t ld, int64_t ldg,
                         int32_t num_tensors, const int64_t* offsets, double* norms, void* workspace,
                         size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                         int32_t period, float gamma, float beta, int64_t k, void* stream) {
    return dl::multi_entry("decentlam_step_multi", dl::ALGO_DECENTLAM, x, m, g, g_format, n, ld, ldg, num_tensors,
                           offsets, norms, workspace, workspace_bytes, row_ptr, col_idx, w, period, gamma, beta,
                           k, stream);
}

int dmsgd_step_multi(float* x, float* m, const void* g, int32_t g_format, int32_t n, int64_t ld, int64_t ldg,
                     int32_t num_tensors, const int64_t* offsets, double* norms, void* workspace,
                     size_t workspace_bytes, const int32_t* row_ptr, const int32_t* col_idx, const float* w,
                     int32_t period, float gamma, float beta, int64_t k, void* stream) {
    return dl::multi_entry("dmsgd_step_multi", dl::ALGO_DMSGD, x, m, g, g_format, n, ld, ldg, num_tensors, offsets,
                           norms, workspace, workspace_bytes, row_ptr, col_idx, w, period, gamma, beta, k, stream);
}

int decentlam_step_xprev(const float* x, float* x_prev, const float* g, int32_t n, int64_t d, int64_t ld,
                         const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                         float gamma, float gamma_prev, float beta, int64_t k, void* stream) {
    return dl::step_entry("decentlam_step_xprev", dl::ALGO_DECENTLAM_XPREV, const_cast<float*>(x), x_prev, g, n,
                          d, ld, row_ptr, col_idx, w, period, gamma, beta, k, stream, gamma_prev);
}

int dsgd_step(float* x, const float* g, int32_t n, int64_t d, int64_t ld, const int32_t* row_ptr,
              const int32_t* col_idx, const float* w, int32_t period, float gamma, int64_t k, void* stream) {
    return dl::step_entry("dsgd_step", dl::ALGO_DSGD, x, nullptr, g, n, d, ld, row_ptr, col_idx, w, period,
                          gamma, 0.0f, k, stream);
}

size_t local_grad_lsq_workspace(int32_t n, int32_t b, int64_t d) {
    if (n < 1 || b < 1 || d < 0) return 0;
    return dl::lsq_workspace_bytes(n, b, d);
}

}  // extern "C"

namespace dl {
int lsq_entry(const char* fn, const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
              int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs, bool sampled,
              float scale, void* workspace, size_t workspace_bytes, void* stream, bool exact_need) {
    clear_error();
    if (n < 1) return set_error(DL_EINVAL, "%s: n = %d, need n >= 1", fn, n);
    if (b < 1) return set_error(DL_EINVAL, "%s: b = %d, need b >= 1", fn, b);
    if (d < 0) return set_error(DL_EINVAL, "%s: d = %lld, need d >= 0", fn, static_cast<long long>(d));
    if (ldA < d || ld < d)
        return set_error(DL_EINVAL, "%s: ldA = %lld and ld = %lld must be >= d = %lld", fn,
                         static_cast<long long>(ldA), static_cast<long long>(ld), static_cast<long long>(d));
    if (!std::isfinite(scale)) return set_error(DL_EINVAL, "%s: scale must be finite", fn);
    if (!A || !y || !x || !g) return set_error(DL_EINVAL, "%s: A, y, x and g must not be NULL", fn);
    if (sampled) {
        if (!rows) return set_error(DL_EINVAL, "%s: rows must not be NULL", fn);
        if (bs < 1) return set_error(DL_EINVAL, "%s: bs = %d, need bs >= 1", fn, bs);
    } else {
        bs = b;
    }
    if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(x) |
         reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(loss) | reinterpret_cast<uintptr_t>(rows)) & 3u)
        return set_error(DL_EINVAL, "%s: arrays must be 4-byte aligned", fn);
    // the documented size covers every path; the library's own array is checked against the path taken
    const size_t need = exact_need ? lsq_workspace_bytes_path(n, bs, d, lsq_path(bs, d, lsq_wide_accesses(A, x, d, ldA, ld)))
                                   : lsq_workspace_bytes(n, bs, d);
    if (!workspace || workspace_bytes < need)
        return set_error(DL_ECAP, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                         workspace ? workspace_bytes : size_t{0});
    if (reinterpret_cast<uintptr_t>(workspace) & 15u)
        return set_error(DL_EINVAL, "%s: workspace must be 16-byte aligned", fn);
    const Span sg = span_of(g, n, d, ld);
    const Span sA = span_of(A, static_cast<int64_t>(n) * b, d, ldA);
    const Span sy = span_of(y, 1, static_cast<int64_t>(n) * b, static_cast<int64_t>(n) * b);
    const Span sx = span_of(x, n, d, ld);
    const Span sw = {reinterpret_cast<uintptr_t>(workspace), reinterpret_cast<uintptr_t>(workspace) + need};
    if (overlap(sg, sA) || overlap(sg, sy) || overlap(sg, sw) || overlap(sw, sA) || overlap(sw, sy) ||
        overlap(sw, sx))
        return set_error(DL_EALIAS, "%s: g / workspace overlap an input", fn);
    if (d > 0 && overlap(sg, sx)) {
        const intptr_t delta = (reinterpret_cast<intptr_t>(g) - reinterpret_cast<intptr_t>(x)) / 4;
        const int64_t off = ((delta % ld) + ld) % ld;
        if (!(off >= d && ld - off >= d)) return set_error(DL_EALIAS, "%s: g overlaps x", fn);
    }
    if (loss) {
        const Span sl = span_of(loss, 1, n, n);
        if (overlap(sl, sA) || overlap(sl, sy) || overlap(sl, sx) || overlap(sl, sg) || overlap(sl, sw))
            return set_error(DL_EALIAS, "%s: loss overlaps another array", fn);
    }
    if (sampled) {
        const Span sr = span_of(rows, 1, static_cast<int64_t>(n) * bs, static_cast<int64_t>(n) * bs);
        if (overlap(sr, sg) || overlap(sr, sw) || (loss && overlap(sr, span_of(loss, 1, n, n))))
            return set_error(DL_EALIAS, "%s: rows overlaps an output", fn);
    }
    return launch_lsq(A, y, x, g, loss, n, b, d, ldA, ld, sampled ? rows : nullptr, bs, scale, workspace,
                      static_cast<hipStream_t>(stream));
}
}  // namespace dl

extern "C" {

int local_grad_lsq_poll_limit(int polls) { return dl::lsq_poll_limit(polls); }

int local_grad_lsq(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
                   int32_t b, int64_t d, int64_t ldA, int64_t ld, float scale, void* workspace,
                   size_t workspace_bytes, void* stream) {
    return dl::lsq_entry("local_grad_lsq", A, y, x, g, loss, n, b, d, ldA, ld, nullptr, b, false, scale,
                         workspace, workspace_bytes, stream);
}

int local_grad_lsq_rows(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
                        int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs,
                        float scale, void* workspace, size_t workspace_bytes, void* stream) {
    return dl::lsq_entry("local_grad_lsq_rows", A, y, x, g, loss, n, b, d, ldA, ld, rows, bs, true, scale,
                         workspace, workspace_bytes, stream);
}

size_t decentlam_stats_workspace(int32_t n, int64_t d) {
    if (n < 1 || d < 0) return 0;
    return dl::stats_workspace_bytes(d);
}

int decentlam_stats(const float* x, const float* m, const float* ref, int32_t n, int64_t d, int64_t ld,
                    double* out, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace dl;
    const char* fn = "decentlam_stats";
    clear_error();
    if (n < 1) return set_error(DL_EINVAL, "%s: n = %d, need n >= 1", fn, n);
    if (d < 0) return set_error(DL_EINVAL, "%s: d = %lld, need d >= 0", fn, static_cast<long long>(d));
    if (ld < d)
        return set_error(DL_EINVAL, "%s: ld = %lld < d = %lld", fn, static_cast<long long>(ld),
                         static_cast<long long>(d));
    if (!out) return set_error(DL_EINVAL, "%s: out must not be NULL", fn);
    if (d > 0 && !x) return set_error(DL_EINVAL, "%s: x must not be NULL", fn);
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(ref)) & 3u)
        return set_error(DL_EINVAL, "%s: x, m and ref must be 4-byte aligned", fn);
    if (reinterpret_cast<uintptr_t>(out) & 7u) return set_error(DL_EINVAL, "%s: out must be 8-byte aligned", fn);
    const size_t need = stats_workspace_bytes(d);
    if (!workspace || workspace_bytes < need)
        return set_error(DL_ECAP, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                         workspace ? workspace_bytes : size_t{0});
    if (reinterpret_cast<uintptr_t>(workspace) & 7u)
        return set_error(DL_EINVAL, "%s: workspace must be 8-byte aligned", fn);
    return launch_stats(x, m, ref, n, d, ld, out, workspace, static_cast<hipStream_t>(stream));
}

const char* dl_last_error(void) { return dl::g_error; }

}  // extern "C"
