// Host side of libsbn: block importance, magnitude pruning, whole-network
// rearrangement and the canonical group-sparse packer (offline steps of the
// method: Section 3.2, Section 3.4, and the "sparse info" of Algorithm 1).
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <numeric>

#include "sbn_internal.h"

namespace sbn {

static thread_local std::string g_err;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

void clear_error() { g_err.clear(); }

// kernel form forced by sbn_force_kernel_form, per layer kind; 0 = chosen per launch
static std::atomic<int> g_form1x1{0}, g_form3x3{0};
int forced_kernel_form(int kind) { return (kind == SBN_CONV3X3 ? g_form3x3 : g_form1x1).load(std::memory_order_relaxed); }

bool is_permutation(const int32_t* p, int n)
{
    std::vector<char> seen((size_t)n, 0);
    for (int i = 0; i < n; ++i) {
        if (p[i] < 0 || p[i] >= n || seen[(size_t)p[i]]) return false;
        seen[(size_t)p[i]] = 1;
    }
    return true;
}

// Section 3.2 / Eq. 2: importance of block (i, j) = l1 norm of the go x gi
// (x kh x kw) weights it covers.  fp64, summed filter -> ky -> kx -> channel.
void block_norms(const float* w, int c_out, int kh, int kw, int c_in, int go, int gi, std::vector<double>& out)
{
    const int rows = c_out / go, cols = c_in / gi;
    out.assign((size_t)rows * cols, 0.0);
    for (int i = 0; i < rows; ++i)
        for (int j = 0; j < cols; ++j) {
            double s = 0.0;
            for (int o = 0; o < go; ++o)
                for (int ky = 0; ky < kh; ++ky)
                    for (int kx = 0; kx < kw; ++kx) {
                        const float* q = w + ((((size_t)(i * go + o)) * kh + ky) * kw + kx) * c_in + (size_t)j * gi;
                        for (int c = 0; c < gi; ++c) s += std::fabs((double)q[c]);
                    }
            out[(size_t)i * cols + j] = s;
        }
}

static int check_geometry(int kind, int c_in, int c_out, int go, int gi)
{
    if (kind != SBN_CONV1X1 && kind != SBN_CONV3X3)
        return fail(SBN_EINVAL, "kind must be SBN_CONV1X1 or SBN_CONV3X3 (got %d)", kind);
    if (c_in <= 0 || c_out <= 0)
        return fail(SBN_EINVAL, "c_in and c_out must be positive (got %d, %d)", c_in, c_out);
    if (c_in > 65528) return fail(SBN_EINVAL, "c_in %d does not fit the 16-bit channel index", c_in);
    if (go != 4 && go != 8) return fail(SBN_EINVAL, "go must be 4 or 8 (got %d)", go);
    if (gi != 1 && gi != 2 && gi != 4 && gi != 8) return fail(SBN_EINVAL, "gi must be 1, 2, 4 or 8 (got %d)", gi);
    if (c_out % go) return fail(SBN_ESHAPE, "c_out %d is not a multiple of go %d", c_out, go);
    if (c_in % gi) return fail(SBN_ESHAPE, "c_in %d is not a multiple of gi %d", c_in, gi);
    return SBN_OK;
}

static size_t removed_count(size_t n_blocks, int pct) { return n_blocks * (size_t)pct / 100; }

// Sorting by importance needs a strict weak order: NaN norms have none, so they are refused.
static bool all_finite(const std::vector<double>& v)
{
    for (double x : v)
        if (!std::isfinite(x)) return false;
    return true;
}

// Permuted copy: wp[r][ky][kx][c] = w[perm_out[r]][ky][kx][perm_in[c]].
static void permute_ohwi(const float* w, int c_out, int taps, int c_in, const int32_t* perm_out,
                         const int32_t* perm_in, std::vector<float>& wp)
{
    wp.resize((size_t)c_out * taps * c_in);
    for (int r = 0; r < c_out; ++r) {
        const int ro = perm_out ? perm_out[r] : r;
        for (int t = 0; t < taps; ++t) {
            const float* src = w + ((size_t)ro * taps + t) * c_in;
            float* dst = wp.data() + ((size_t)r * taps + t) * c_in;
            if (perm_in)
                for (int c = 0; c < c_in; ++c) dst[c] = src[perm_in[c]];
            else
                std::memcpy(dst, src, sizeof(float) * (size_t)c_in);
        }
    }
}

// ---------------------------------------------------------------------------
// Rearrangement search (Section 3.4).  A tensor's channel order is the filter
// order of every layer that produces it, so the search runs over one
// permutation shared by all of them (PARTS): part k works on per-filter
// column-group norms a_k[f][j] = l1 norm of filter f of layer k over its channel
// group j (all taps); the norm of a block is the sum of a_k[f][j] over the go
// filters of its row group; the objective is the sum over the parts of the
// importance that survives pruning.
// ---------------------------------------------------------------------------
struct RowSearch {
    struct Part {
        int cols = 0;
        size_t keep = 0;                   // number of blocks that survive pruning
        std::vector<double> a;             // [n][cols]
        std::vector<double> s;             // block norms of the current order [rows][cols]
    };
    int n = 0, go = 0, rows = 0;
    std::vector<Part> parts;
    std::vector<int32_t> perm;             // current order, rows*go
    std::vector<double> tmp;

    static void row_norms(const Part& p, int go, const int32_t* members, double* out)
    {
        for (int j = 0; j < p.cols; ++j) {
            double v = 0.0;
            for (int o = 0; o < go; ++o) v += p.a[(size_t)members[o] * p.cols + j];
            out[j] = v;
        }
    }
    void rebuild()
    {
        for (Part& p : parts) {
            p.s.resize((size_t)rows * p.cols);
            for (int i = 0; i < rows; ++i) row_norms(p, go, &perm[(size_t)i * go], &p.s[(size_t)i * p.cols]);
        }
    }
    // sum of the `keep` largest entries of v (v is reordered)
    static double top_sum(std::vector<double>& v, size_t keep)
    {
        if (keep == 0) return 0.0;
        if (keep < v.size()) std::nth_element(v.begin(), v.begin() + (v.size() - keep), v.end());
        double t = 0.0;
        for (size_t i = v.size() - keep; i < v.size(); ++i) t += v[i];
        return t;
    }
    double objective()
    {
        double t = 0.0;
        for (Part& p : parts) {
            tmp = p.s;
            t += top_sum(tmp, p.keep);
        }
        return t;
    }
    // objective with rows ga and gb replaced by the norms of the current perm's members
    double objective_with(int ga, int gb, std::vector<std::vector<double>>& ra, std::vector<std::vector<double>>& rb)
    {
        double t = 0.0;
        for (size_t k = 0; k < parts.size(); ++k) {
            Part& p = parts[k];
            ra[k].resize((size_t)p.cols);
            rb[k].resize((size_t)p.cols);
            row_norms(p, go, &perm[(size_t)ga * go], ra[k].data());
            row_norms(p, go, &perm[(size_t)gb * go], rb[k].data());
            tmp = p.s;
            std::copy(ra[k].begin(), ra[k].end(), tmp.begin() + (size_t)ga * p.cols);
            std::copy(rb[k].begin(), rb[k].end(), tmp.begin() + (size_t)gb * p.cols);
            t += top_sum(tmp, p.keep);
        }
        return t;
    }
    void commit(int ga, int gb, const std::vector<std::vector<double>>& ra, const std::vector<std::vector<double>>& rb)
    {
        for (size_t k = 0; k < parts.size(); ++k) {
            std::copy(ra[k].begin(), ra[k].end(), parts[k].s.begin() + (size_t)ga * parts[k].cols);
            std::copy(rb[k].begin(), rb[k].end(), parts[k].s.begin() + (size_t)gb * parts[k].cols);
        }
    }
};

static inline uint64_t splitmix64(uint64_t& state)
{
    uint64_t z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static void canonicalize(std::vector<int32_t>& perm, int go)
{
    const int rows = (int)perm.size() / go;
    std::vector<std::vector<int32_t>> g((size_t)rows);
    for (int i = 0; i < rows; ++i) {
        g[(size_t)i].assign(perm.begin() + (size_t)i * go, perm.begin() + (size_t)(i + 1) * go);
        std::sort(g[(size_t)i].begin(), g[(size_t)i].end());
    }
    std::sort(g.begin(), g.end(), [](const std::vector<int32_t>& x, const std::vector<int32_t>& y) { return x[0] < y[0]; });
    for (int i = 0; i < rows; ++i) std::copy(g[(size_t)i].begin(), g[(size_t)i].end(), perm.begin() + (size_t)i * go);
}

// Number of canonical groupings of n filters into groups of go, n! / ((go!)^(n/go) (n/go)!)
// (Section 3.4's canonical form), saturating at `cap`.
static double canonical_count(int n, int go, double cap)
{
    double c = 1.0;
    for (int left = n; left > 0; left -= go) {          // the first free filter opens a group: C(left-1, go-1) ways
        double ways = 1.0;
        for (int i = 1; i < go; ++i) ways = ways * (double)(left - i) / (double)i;
        c *= ways;
        if (c > cap) return cap;
    }
    return c;
}

// Enumerates every canonical grouping (first free filter opens a group, the
// rest of the group is chosen in ascending combinations) and keeps the first
// one with the largest objective.
static void exhaustive(RowSearch& rs, std::vector<int32_t>& cur, std::vector<char>& used, int filled,
                       double& best_obj, std::vector<int32_t>& best)
{
    const int n = rs.n, go = rs.go;
    if (filled == n) {
        rs.perm = cur;
        rs.rebuild();
        const double obj = rs.objective();
        if (obj > best_obj) {
            best_obj = obj;
            best = cur;
        }
        return;
    }
    int first = 0;
    while (used[(size_t)first]) ++first;
    used[(size_t)first] = 1;
    cur[(size_t)filled] = first;
    // choose go-1 more members > first, ascending
    std::vector<int> cand;
    for (int f = first + 1; f < n; ++f)
        if (!used[(size_t)f]) cand.push_back(f);
    const int m = (int)cand.size(), k = go - 1;
    if (k == 0) {
        exhaustive(rs, cur, used, filled + 1, best_obj, best);
    } else if (m >= k) {
        std::vector<int> idx((size_t)k);
        std::iota(idx.begin(), idx.end(), 0);
        while (true) {
            for (int t = 0; t < k; ++t) {
                cur[(size_t)filled + 1 + t] = cand[(size_t)idx[(size_t)t]];
                used[(size_t)cand[(size_t)idx[(size_t)t]]] = 1;
            }
            exhaustive(rs, cur, used, filled + go, best_obj, best);
            for (int t = 0; t < k; ++t) used[(size_t)cand[(size_t)idx[(size_t)t]]] = 0;
            int t = k - 1;
            while (t >= 0 && idx[(size_t)t] == m - k + t) --t;
            if (t < 0) break;
            ++idx[(size_t)t];
            for (int u = t + 1; u < k; ++u) idx[(size_t)u] = idx[(size_t)u - 1] + 1;
        }
    }
    used[(size_t)first] = 0;
}

// Layers at most this many canonical groupings large are searched exhaustively (12 filters in
// groups of 4: 5 775; 16 in groups of 8: 6 435; 8 in groups of 4: 35).
#ifndef SBN_EXHAUSTIVE_LIMIT
#define SBN_EXHAUSTIVE_LIMIT 20000.0       // (a build with 0 runs the bounded search everywhere: used to compare the two)
#endif
constexpr double kExhaustiveLimit = SBN_EXHAUSTIVE_LIMIT;

struct SearchPart {
    const float* wc;                       // OHWI weights, channels already in their final order
    int taps, c_in, gi;
};

// One tensor's filter order from the layers that produce it.  Small cases: every canonical
// grouping.  Otherwise a seeded, bounded local search over swaps of two filters of different
// groups ("bounded regression" in the paper's words; its algorithm is not given): a swap is kept
// if the objective strictly increases; after a run of rejected candidates as long as the number
// of filters the search restarts from the best order so far with two random swaps applied, and
// the best order ever seen is returned -- never worse than the identity it starts from.
static void search_rows(const std::vector<SearchPart>& parts, int c_out, int go, int pct, uint64_t seed, int max_iters,
                        std::vector<int32_t>& perm_out)
{
    RowSearch rs;
    rs.n = c_out;
    rs.go = go;
    rs.rows = c_out / go;
    for (const SearchPart& sp : parts) {
        RowSearch::Part p;
        p.cols = sp.c_in / sp.gi;
        const size_t nb = (size_t)rs.rows * p.cols;
        p.keep = nb - removed_count(nb, pct);
        p.a.assign((size_t)c_out * p.cols, 0.0);
        for (int f = 0; f < c_out; ++f)
            for (int t = 0; t < sp.taps; ++t) {
                const float* q = sp.wc + ((size_t)f * sp.taps + t) * sp.c_in;
                for (int c = 0; c < sp.c_in; ++c) p.a[(size_t)f * p.cols + c / sp.gi] += std::fabs((double)q[c]);
            }
        rs.parts.push_back(std::move(p));
    }
    perm_out.resize((size_t)c_out);
    std::iota(perm_out.begin(), perm_out.end(), 0);
    if (rs.rows < 2 || rs.parts.empty()) return;

    if (canonical_count(c_out, go, kExhaustiveLimit + 1) <= kExhaustiveLimit) {
        std::vector<int32_t> cur((size_t)c_out), best = perm_out;
        std::vector<char> used((size_t)c_out, 0);
        double best_obj = -1.0;
        exhaustive(rs, cur, used, 0, best_obj, best);
        perm_out = best;
        return;
    }

    rs.perm = perm_out;
    rs.rebuild();
    double cur_obj = rs.objective(), best_obj = cur_obj;
    std::vector<int32_t> best = rs.perm;
    uint64_t st = seed;
    std::vector<std::vector<double>> ra(rs.parts.size()), rb(rs.parts.size());
    int rejected = 0;
    auto random_pair = [&](int& pa, int& pb) {
        const uint64_t r0 = splitmix64(st), r1 = splitmix64(st);
        pa = (int)(r0 % (uint64_t)c_out);
        pb = (int)(r1 % (uint64_t)c_out);
        if (pa / go == pb / go) {                             // force a different group, deterministically
            const int gb = (pb / go + 1 + (int)((r1 >> 32) % (uint64_t)(rs.rows - 1))) % rs.rows;
            pb = gb * go + pb % go;
        }
    };
    for (int it = 0; it < max_iters; ++it) {
        if (rejected >= c_out) {                              // stuck: restart near the best order so far
            rs.perm = best;
            for (int k = 0; k < 2; ++k) {
                int pa, pb;
                random_pair(pa, pb);
                std::swap(rs.perm[(size_t)pa], rs.perm[(size_t)pb]);
            }
            rs.rebuild();
            cur_obj = rs.objective();
            rejected = 0;
            if (cur_obj > best_obj) best_obj = cur_obj, best = rs.perm;
            continue;
        }
        int pa, pb;
        random_pair(pa, pb);
        const int ga = pa / go, gb = pb / go;
        std::swap(rs.perm[(size_t)pa], rs.perm[(size_t)pb]);
        const double obj = rs.objective_with(ga, gb, ra, rb);
        if (obj > cur_obj) {
            cur_obj = obj;
            rs.commit(ga, gb, ra, rb);
            rejected = 0;
            if (cur_obj > best_obj) best_obj = cur_obj, best = rs.perm;
        } else {
            std::swap(rs.perm[(size_t)pa], rs.perm[(size_t)pb]);
            ++rejected;
        }
    }
    perm_out = best;
    canonicalize(perm_out, go);
}

}  // namespace sbn

using namespace sbn;

extern "C" {

const char* sbn_last_error(void) { return sbn::g_err.c_str(); }

int sbn_force_kernel_form(int kind, int form)
{
    clear_error();
    static const int forms1x1[] = {0, 1, 11, 12, 14, 21, 22, 112, 121, 504, 508, 516, 1012, 1021, 1112, 1121}, forms3x3[] = {0, 1, 2, 3, 32};
    bool ok = false;
    if (kind == SBN_CONV1X1)
        for (int f : forms1x1) ok |= f == form;
    else if (kind == SBN_CONV3X3)
        for (int f : forms3x3) ok |= f == form;
    else
        return fail(SBN_EINVAL, "sbn_force_kernel_form: kind must be SBN_CONV1X1 or SBN_CONV3X3 (got %d)", kind);
    if (!ok) return fail(SBN_EINVAL, "sbn_force_kernel_form: %d is not a kernel form of this kind", form);
    (kind == SBN_CONV3X3 ? sbn::g_form3x3 : sbn::g_form1x1).store(form, std::memory_order_relaxed);
    return SBN_OK;
}

int sbn_prune_magnitude(const float* w, int kind, int c_in, int c_out, int go, int gi, int pct, uint8_t* mask_out)
{
    clear_error();
    if (!w || !mask_out) return fail(SBN_EINVAL, "sbn_prune_magnitude: NULL pointer");
    if (pct < 0 || pct > 100) return fail(SBN_EINVAL, "sparsity_percent must be in [0,100] (got %d)", pct);
    if (int rc = check_geometry(kind, c_in, c_out, go, gi)) return rc;
    return guarded("sbn_prune_magnitude", [&]() -> int {
        const int k = kind == SBN_CONV3X3 ? 3 : 1;
        std::vector<double> s;
        block_norms(w, c_out, k, k, c_in, go, gi, s);
        if (!all_finite(s)) return fail(SBN_EINVAL, "sbn_prune_magnitude: the weights contain NaN or infinity");
        std::vector<uint32_t> order(s.size());
        std::iota(order.begin(), order.end(), 0u);
        std::sort(order.begin(), order.end(),
                  [&](uint32_t a, uint32_t b) { return s[a] < s[b] || (s[a] == s[b] && a < b); });
        const size_t r = removed_count(s.size(), pct);
        std::fill(mask_out, mask_out + s.size(), (uint8_t)1);
        for (size_t i = 0; i < r; ++i) mask_out[order[i]] = 0;
        return SBN_OK;
    });
}

int sbn_retained_l1(const float* w, int kind, int c_in, int c_out, int go, int gi, int pct, double* out)
{
    clear_error();
    if (!w || !out) return fail(SBN_EINVAL, "sbn_retained_l1: NULL pointer");
    if (pct < 0 || pct > 100) return fail(SBN_EINVAL, "sparsity_percent must be in [0,100] (got %d)", pct);
    if (int rc = check_geometry(kind, c_in, c_out, go, gi)) return rc;
    return guarded("sbn_retained_l1", [&]() -> int {
        const int k = kind == SBN_CONV3X3 ? 3 : 1;
        std::vector<double> s;
        block_norms(w, c_out, k, k, c_in, go, gi, s);
        if (!all_finite(s)) return fail(SBN_EINVAL, "sbn_retained_l1: the weights contain NaN or infinity");
        std::sort(s.begin(), s.end());
        double t = 0.0;
        for (size_t i = removed_count(s.size(), pct); i < s.size(); ++i) t += s[i];
        *out = t;
        return SBN_OK;
    });
}

// ---- 3:9 pattern group pruning of depthwise kernels (Section 3.2, DwConv3x3)

extern "C++" {
namespace sbn {
int dw_group_starts(int c, int go, std::vector<int>& start)
{
    if (c <= 0 || c % 4) return fail(SBN_ESHAPE, "depthwise pattern pruning needs a positive multiple of 4 channels (got %d)", c);
    if (go != 4 && go != 8 && go != 16) return fail(SBN_EINVAL, "depthwise pattern group size must be 4, 8 or 16 (got %d)", go);
    start.clear();
    int pos = 0;
    for (; c - pos >= go; pos += go) start.push_back(pos);
    for (int g = 8; g >= 4; g /= 2)
        for (; g < go && c - pos >= g; pos += g) start.push_back(pos);
    start.push_back(c);
    return SBN_OK;
}
}  // namespace sbn
}  // extern "C++"

int sbn_dw_pattern_groups(int c, int go, int* n_groups_out, int* group_start)
{
    clear_error();
    if (!n_groups_out) return fail(SBN_EINVAL, "sbn_dw_pattern_groups: NULL pointer");
    return guarded("sbn_dw_pattern_groups", [&]() -> int {
        std::vector<int> st;
        if (int rc = sbn::dw_group_starts(c, go, st)) return rc;
        *n_groups_out = (int)st.size() - 1;
        if (group_start) std::copy(st.begin(), st.end(), group_start);
        return SBN_OK;
    });
}

static int sbn_dw_pattern_select_impl(const float* w, int c, int go, const uint8_t* keep_dense, uint8_t* pattern_out)
{
    clear_error();
    if (!w || !pattern_out) return fail(SBN_EINVAL, "sbn_dw_pattern_select: NULL pointer");
    std::vector<int> st;
    if (int rc = sbn::dw_group_starts(c, go, st)) return rc;
    for (size_t g = 0; g + 1 < st.size(); ++g) {
        if (keep_dense && keep_dense[g]) {
            pattern_out[g] = SBN_DW_PATTERN_DENSE;
            continue;
        }
        double best = -1.0;
        int best_id = 0;
        for (int pid = 0; pid < 8; ++pid) {
            double tot = 0.0;
            for (int ch = st[g]; ch < st[g + 1]; ++ch)
                for (int r = 0; r < 3; ++r) {
                    const int gone = (pid >> r) & 1 ? 2 : 0;
                    for (int col = 0; col < 3; ++col)
                        if (col != gone) tot += std::fabs((double)w[(size_t)ch * 9 + r * 3 + col]);
                }
            if (tot > best) best = tot, best_id = pid;
        }
        pattern_out[g] = (uint8_t)best_id;
    }
    return SBN_OK;
}

static int sbn_dw_pattern_apply_impl(const float* w, int c, int go, const uint8_t* pattern, float* w_out)
{
    clear_error();
    if (!w || !pattern || !w_out) return fail(SBN_EINVAL, "sbn_dw_pattern_apply: NULL pointer");
    std::vector<int> st;
    if (int rc = sbn::dw_group_starts(c, go, st)) return rc;
    for (size_t g = 0; g + 1 < st.size(); ++g)
        if (pattern[g] > SBN_DW_PATTERN_DENSE) return fail(SBN_EINVAL, "pattern id %d of group %zu is not in 0..8", pattern[g], g);
    for (size_t g = 0; g + 1 < st.size(); ++g)
        for (int ch = st[g]; ch < st[g + 1]; ++ch)
            for (int r = 0; r < 3; ++r) {
                const int gone = pattern[g] == SBN_DW_PATTERN_DENSE ? -1 : (pattern[g] >> r) & 1 ? 2 : 0;
                for (int col = 0; col < 3; ++col) {
                    const size_t i = (size_t)ch * 9 + r * 3 + col;
                    w_out[i] = col == gone ? 0.0f : w[i];
                }
            }
    return SBN_OK;
}

// ---- 4-of-9 pattern pruning inside kept 3x3 kernels (Section 3.2, Conv3x3)

// kept taps of a pattern id; the ids enumerate the 3-subsets of the non-centre taps in
// lexicographic order
static uint32_t k3_pattern_taps(int pattern)
{
    if (pattern == SBN_K3_PATTERN_DENSE) return 0x1FFu;
    static const int other[8] = {0, 1, 2, 3, 5, 6, 7, 8};
    int id = 0;
    for (int a = 0; a < 8; ++a)
        for (int b = a + 1; b < 8; ++b)
            for (int c = b + 1; c < 8; ++c, ++id)
                if (id == pattern) return (1u << other[a]) | (1u << other[b]) | (1u << other[c]) | (1u << 4);
    return 0;
}

static int k3_pattern_args(const char* who, int c_out, int c_in, int share)
{
    if (share != 1 && share != 2 && share != 4)
        return fail(SBN_EINVAL, "%s: a pattern is shared by 4, 2 or 1 filters (got %d)", who, share);
    if (c_out <= 0 || c_in <= 0 || c_out % share)
        return fail(SBN_ESHAPE, "%s: %d filters do not split into groups of %d", who, c_out, share);
    return SBN_OK;
}

int sbn_conv3x3_pattern_taps(int pattern, uint32_t* tap_mask_out)
{
    clear_error();
    if (!tap_mask_out) return fail(SBN_EINVAL, "sbn_conv3x3_pattern_taps: NULL pointer");
    if (pattern < 0 || pattern > SBN_K3_PATTERN_DENSE)
        return fail(SBN_EINVAL, "pattern id %d is not in 0..%d", pattern, SBN_K3_PATTERN_DENSE);
    *tap_mask_out = k3_pattern_taps(pattern);
    return SBN_OK;
}

int sbn_conv3x3_pattern_select(const float* w, int c_out, int c_in, int share, uint8_t* pattern_out)
{
    clear_error();
    if (!w || !pattern_out) return fail(SBN_EINVAL, "sbn_conv3x3_pattern_select: NULL pointer");
    if (int rc = k3_pattern_args("sbn_conv3x3_pattern_select", c_out, c_in, share)) return rc;
    uint32_t taps[SBN_K3_PATTERNS];
    for (int p = 0; p < SBN_K3_PATTERNS; ++p) taps[p] = k3_pattern_taps(p);
    for (int f = 0; f < c_out / share; ++f)
        for (int c = 0; c < c_in; ++c) {
            double s[9];
            for (int t = 0; t < 9; ++t) {
                s[t] = 0.0;
                for (int i = 0; i < share; ++i)
                    s[t] += std::fabs((double)w[((size_t)(f * share + i) * 9 + t) * c_in + c]);
            }
            double best = -1.0;
            int best_id = 0;
            for (int p = 0; p < SBN_K3_PATTERNS; ++p) {
                double tot = 0.0;
                for (int t = 0; t < 9; ++t)
                    if (t != 4 && ((taps[p] >> t) & 1u)) tot += s[t];
                if (tot > best) best = tot, best_id = p;
            }
            pattern_out[(size_t)f * c_in + c] = (uint8_t)best_id;
        }
    return SBN_OK;
}

int sbn_conv3x3_pattern_apply(const float* w, int c_out, int c_in, int share, const uint8_t* pattern, float* w_out)
{
    clear_error();
    if (!w || !pattern || !w_out) return fail(SBN_EINVAL, "sbn_conv3x3_pattern_apply: NULL pointer");
    if (int rc = k3_pattern_args("sbn_conv3x3_pattern_apply", c_out, c_in, share)) return rc;
    const size_t n_ids = (size_t)(c_out / share) * c_in;
    for (size_t i = 0; i < n_ids; ++i)
        if (pattern[i] > SBN_K3_PATTERN_DENSE)
            return fail(SBN_EINVAL, "pattern id %d at position %zu is not in 0..%d", pattern[i], i, SBN_K3_PATTERN_DENSE);
    uint32_t taps[SBN_K3_PATTERN_DENSE + 1];
    for (int p = 0; p <= SBN_K3_PATTERN_DENSE; ++p) taps[p] = k3_pattern_taps(p);
    for (int n = 0; n < c_out; ++n)
        for (int t = 0; t < 9; ++t)
            for (int c = 0; c < c_in; ++c) {
                const size_t i = ((size_t)n * 9 + t) * c_in + c;
                const uint32_t keep = taps[pattern[(size_t)(n / share) * c_in + c]];
                w_out[i] = (keep >> t) & 1u ? w[i] : 0.0f;
            }
    return SBN_OK;
}

// Tensors in increasing number; a tensor's order is searched over all layers that write it, each
// with its channels in the order of its input tensor if that is already decided (lower number),
// else in original order.
static int sbn_rearrange_graph_impl(const sbn_layer_desc_t* layers, int n_layers, const int* in_tensor,
                                    const int* out_tensor, int n_tensors, const int* tensor_fixed, int pct,
                                    uint64_t seed, int max_iters, int32_t* const* perm_out)
{
    clear_error();
    if (!layers || !in_tensor || !out_tensor || !perm_out || n_layers < 0 || n_tensors <= 0)
        return fail(SBN_EINVAL, "sbn_rearrange_graph: NULL pointer or empty graph");
    if (pct < 0 || pct > 100) return fail(SBN_EINVAL, "sparsity_percent must be in [0,100] (got %d)", pct);
    if (max_iters < 0) return fail(SBN_EINVAL, "max_iters must be >= 0");
    std::vector<int> channels((size_t)n_tensors, 0);          // channel count of every tensor, 0 = not seen yet
    auto see = [&](int t, int c, int l, const char* side) -> int {
        if (t < 0 || t >= n_tensors) return fail(SBN_EINVAL, "layer %d: %s tensor %d is not in 0..%d", l, side, t, n_tensors - 1);
        if (channels[(size_t)t] && channels[(size_t)t] != c)
            return fail(SBN_ESHAPE, "tensor %d has %d channels but layer %d %s %d", t, channels[(size_t)t], l,
                        side[0] == 'i' ? "reads" : "writes", c);
        channels[(size_t)t] = c;
        return SBN_OK;
    };
    for (int l = 0; l < n_layers; ++l) {
        const sbn_layer_desc_t& d = layers[l];
        if (!d.w) return fail(SBN_EINVAL, "sbn_rearrange_graph: layer %d has no weights", l);
        if (int rc = check_geometry(d.kind, d.c_in, d.c_out, d.go, d.gi)) return rc;
        if (int rc = see(in_tensor[l], d.c_in, l, "input")) return rc;
        if (int rc = see(out_tensor[l], d.c_out, l, "output")) return rc;
    }
    for (int t = 0; t < n_tensors; ++t) {
        if (!channels[(size_t)t]) return fail(SBN_EINVAL, "tensor %d is used by no layer", t);
        if (!perm_out[t]) return fail(SBN_EINVAL, "sbn_rearrange_graph: no room for the order of tensor %d", t);
    }
    std::vector<char> decided((size_t)n_tensors, 0);
    std::vector<std::vector<float>> wc;
    std::vector<int32_t> perm;
    for (int t = 0; t < n_tensors; ++t) {
        const int c = channels[(size_t)t];
        std::vector<SearchPart> parts;
        wc.clear();
        int go = 0;
        if (!(tensor_fixed && tensor_fixed[t])) {
            for (int l = 0; l < n_layers; ++l) {
                if (out_tensor[l] != t) continue;
                const sbn_layer_desc_t& d = layers[l];
                if (go && d.go != go)
                    return fail(SBN_ESHAPE, "the layers that write tensor %d group their filters by %d and by %d", t, go, d.go);
                go = d.go;
                const int taps = d.kind == SBN_CONV3X3 ? 9 : 1;
                const int32_t* pin = decided[(size_t)in_tensor[l]] ? perm_out[in_tensor[l]] : nullptr;
                wc.emplace_back();
                permute_ohwi(d.w, d.c_out, taps, d.c_in, nullptr, pin, wc.back());
                for (float v : wc.back())
                    if (!std::isfinite(v)) return fail(SBN_EINVAL, "sbn_rearrange_graph: the weights of layer %d contain NaN or infinity", l);
                parts.push_back(SearchPart{nullptr, taps, d.c_in, d.gi});
            }
            for (size_t k = 0; k < parts.size(); ++k) parts[k].wc = wc[k].data();
        }
        if (parts.empty()) {                                 // a network input, or kept in place: identity
            for (int i = 0; i < c; ++i) perm_out[t][i] = i;
        } else {
            const uint64_t s = seed ^ (0xD1B54A32D192ED03ull * (uint64_t)(t + 1));
            search_rows(parts, c, go, pct, s, max_iters, perm);
            std::copy(perm.begin(), perm.end(), perm_out[t]);
        }
        decided[(size_t)t] = 1;
    }
    return SBN_OK;
}

// The chain / tree form: tensor 0 is the network input, tensor l + 1 the output of layer l.
static int sbn_rearrange_impl(const sbn_layer_desc_t* layers, int n_layers, const int* parent, const int* keep_output_order,
                              int pct, uint64_t seed, int max_iters, int32_t* const* perm_out)
{
    clear_error();
    if (!layers || !parent || !perm_out || n_layers < 0) return fail(SBN_EINVAL, "sbn_rearrange: NULL pointer");
    for (int l = 0; l < n_layers; ++l) {
        if (!perm_out[l]) return fail(SBN_EINVAL, "sbn_rearrange: layer %d has a NULL pointer", l);
        if (parent[l] >= l || parent[l] < -1)
            return fail(SBN_ESHAPE, "parent[%d] = %d: parents must come first", l, parent[l]);
        if (parent[l] >= 0 && layers[parent[l]].c_out != layers[l].c_in)
            return fail(SBN_ESHAPE, "layer %d reads %d channels but its parent %d writes %d", l, layers[l].c_in, parent[l],
                        layers[parent[l]].c_out);
    }
    // Layers that read the network input directly may differ in c_in: each gets an input tensor of its own.
    std::vector<int> in_t((size_t)n_layers), out_t((size_t)n_layers), fixed;
    int n_tensors = n_layers;
    for (int l = 0; l < n_layers; ++l) {
        out_t[(size_t)l] = l;
        in_t[(size_t)l] = parent[l] >= 0 ? parent[l] : n_tensors++;
    }
    fixed.assign((size_t)n_tensors, 0);
    for (int l = 0; l < n_layers; ++l) fixed[(size_t)l] = keep_output_order && keep_output_order[l] ? 1 : 0;
    for (int t = n_layers; t < n_tensors; ++t) fixed[(size_t)t] = 1;
    // The graph call decides tensors in increasing number and looks an input's order up only if
    // it is decided: network inputs (numbered last) count as identity either way.
    std::vector<std::vector<int32_t>> extra((size_t)(n_tensors - n_layers));
    std::vector<int32_t*> ptrs((size_t)n_tensors);
    for (int l = 0; l < n_layers; ++l) ptrs[(size_t)l] = perm_out[l];
    for (int t = n_layers; t < n_tensors; ++t) {
        extra[(size_t)(t - n_layers)].resize((size_t)layers[std::find(in_t.begin(), in_t.end(), t) - in_t.begin()].c_in);
        ptrs[(size_t)t] = extra[(size_t)(t - n_layers)].data();
    }
    return sbn_rearrange_graph_impl(layers, n_layers, in_t.data(), out_t.data(), n_tensors, fixed.data(), pct, seed, max_iters,
                                    ptrs.data());
}

// Order of the filter groups of every tensor (the grouping itself stays as it is).  The kernels
// walk 16 consecutive filters (a bundle) together over the union of the 4-channel input pieces
// that any of them keeps, so the groups that keep the same pieces belong next to each other.
// Greedy: a bundle is opened by the unit with the most kept pieces and filled with the units
// that add the fewest new pieces (ties: the most shared pieces, then the lower position); then
// two units of different bundles are exchanged wherever that shrinks the two unions.  A unit
// is max(go of the writers, gi of the readers) filters, so that every reader's blocks stay whole.
static int sbn_order_groups_graph_impl(const sbn_layer_desc_t* layers, int n_layers, const int* in_tensor,
                                       const int* out_tensor, int n_tensors, const int* tensor_fixed, int pct,
                                       int32_t* const* perm)
{
    clear_error();
    if (!layers || !in_tensor || !out_tensor || !perm || n_layers < 0 || n_tensors <= 0)
        return fail(SBN_EINVAL, "sbn_order_groups_graph: NULL pointer or empty graph");
    if (pct < 0 || pct > 100) return fail(SBN_EINVAL, "sparsity_percent must be in [0,100] (got %d)", pct);
    std::vector<int> channels((size_t)n_tensors, 0);
    for (int l = 0; l < n_layers; ++l) {
        const sbn_layer_desc_t& d = layers[l];
        if (!d.w) return fail(SBN_EINVAL, "sbn_order_groups_graph: layer %d has no weights", l);
        if (int rc = check_geometry(d.kind, d.c_in, d.c_out, d.go, d.gi)) return rc;
        const int ts[2] = {in_tensor[l], out_tensor[l]}, cs[2] = {d.c_in, d.c_out};
        for (int k = 0; k < 2; ++k) {
            if (ts[k] < 0 || ts[k] >= n_tensors) return fail(SBN_EINVAL, "layer %d: tensor %d is not in 0..%d", l, ts[k], n_tensors - 1);
            if (channels[(size_t)ts[k]] && channels[(size_t)ts[k]] != cs[k])
                return fail(SBN_ESHAPE, "tensor %d has %d channels but layer %d uses %d", ts[k], channels[(size_t)ts[k]], l, cs[k]);
            channels[(size_t)ts[k]] = cs[k];
        }
    }
    for (int t = 0; t < n_tensors; ++t) {
        if (!channels[(size_t)t]) return fail(SBN_EINVAL, "tensor %d is used by no layer", t);
        if (!perm[t]) return fail(SBN_EINVAL, "sbn_order_groups_graph: no order given for tensor %d", t);
        if (!is_permutation(perm[t], channels[(size_t)t]))
            return fail(SBN_EPERM, "the order given for tensor %d is not a permutation of 0..%d", t, channels[(size_t)t] - 1);
    }
    for (int t = 0; t < n_tensors; ++t) {
        if (tensor_fixed && tensor_fixed[t]) continue;
        const int c = channels[(size_t)t];
        int unit = 0, go = 0;
        for (int l = 0; l < n_layers; ++l) {
            if (out_tensor[l] == t) {
                if (go && layers[l].go != go)
                    return fail(SBN_ESHAPE, "the layers that write tensor %d group their filters by %d and by %d", t, go, layers[l].go);
                go = layers[l].go;
            }
        }
        if (!go) continue;                                    // a network input
        unit = go;
        for (int l = 0; l < n_layers; ++l)
            if (in_tensor[l] == t) unit = std::max(unit, layers[l].gi);
        if (c % unit) continue;                               // (cannot happen: both divide c and are powers of two)
        const int n_units = c / unit, per_bundle = 16 / unit;
        if (n_units <= per_bundle) continue;
        // kept 4-channel pieces of every unit, over all writers
        std::vector<std::vector<uint64_t>> pieces((size_t)n_units);
        size_t words = 0;
        std::vector<float> wp;
        std::vector<double> norms;
        for (int l = 0; l < n_layers; ++l) {
            if (out_tensor[l] != t) continue;
            const sbn_layer_desc_t& d = layers[l];
            const int k = d.kind == SBN_CONV3X3 ? 3 : 1, cols = d.c_in / d.gi, n_pieces = (d.c_in + 3) / 4;
            permute_ohwi(d.w, d.c_out, k * k, d.c_in, perm[t], perm[in_tensor[l]], wp);
            block_norms(wp.data(), d.c_out, k, k, d.c_in, d.go, d.gi, norms);
            if (!all_finite(norms)) return fail(SBN_EINVAL, "sbn_order_groups_graph: the weights of layer %d contain NaN or infinity", l);
            std::vector<uint32_t> order(norms.size());
            std::iota(order.begin(), order.end(), 0u);
            std::sort(order.begin(), order.end(),
                      [&](uint32_t a, uint32_t b) { return norms[a] < norms[b] || (norms[a] == norms[b] && a < b); });
            const size_t removed = removed_count(norms.size(), pct);
            const size_t base = words, add = ((size_t)n_pieces + 63) / 64;
            words += add;
            for (auto& v : pieces) v.resize(words, 0);
            for (size_t i = removed; i < order.size(); ++i) {
                const int row = (int)(order[i] / (uint32_t)cols), col = (int)(order[i] % (uint32_t)cols);
                std::vector<uint64_t>& v = pieces[(size_t)(row * d.go / unit)];
                for (int ch = col * d.gi; ch < (col + 1) * d.gi; ch += 4 - ch % 4) v[base + (size_t)(ch / 4) / 64] |= 1ull << ((ch / 4) % 64);
            }
        }
        auto count = [&](const std::vector<uint64_t>& a, const std::vector<uint64_t>* mask, bool in_mask) {
            int nbits = 0;
            for (size_t i = 0; i < words; ++i) {
                uint64_t v = a[i];
                if (mask) v &= in_mask ? (*mask)[i] : ~(*mask)[i];
                nbits += __builtin_popcountll(v);
            }
            return nbits;
        };
        std::vector<char> used((size_t)n_units, 0);
        std::vector<int> sequence;
        std::vector<uint64_t> uni(words);
        while ((int)sequence.size() < n_units) {
            int seed_unit = -1, seed_count = -1;
            for (int i = 0; i < n_units; ++i)
                if (!used[(size_t)i]) {
                    const int k = count(pieces[(size_t)i], nullptr, false);
                    if (k > seed_count) seed_count = k, seed_unit = i;
                }
            used[(size_t)seed_unit] = 1;
            sequence.push_back(seed_unit);
            uni = pieces[(size_t)seed_unit];
            for (int m = 1; m < per_bundle && (int)sequence.size() < n_units; ++m) {
                int best = -1, best_new = 0, best_shared = 0;
                for (int i = 0; i < n_units; ++i) {
                    if (used[(size_t)i]) continue;
                    const int fresh = count(pieces[(size_t)i], &uni, false), shared = count(pieces[(size_t)i], &uni, true);
                    if (best < 0 || fresh < best_new || (fresh == best_new && shared > best_shared))
                        best = i, best_new = fresh, best_shared = shared;
                }
                used[(size_t)best] = 1;
                sequence.push_back(best);
                for (size_t i = 0; i < words; ++i) uni[i] |= pieces[(size_t)best][i];
            }
        }
        // then exchanges of two units of different bundles while the total shrinks (a few sweeps)
        auto bundle_size = [&](int b) {
            int nbits = 0;
            for (size_t i = 0; i < words; ++i) {
                uint64_t v = 0;
                for (int m = b * per_bundle; m < std::min((b + 1) * per_bundle, n_units); ++m) v |= pieces[(size_t)sequence[(size_t)m]][i];
                nbits += __builtin_popcountll(v);
            }
            return nbits;
        };
        const int n_bundles = (n_units + per_bundle - 1) / per_bundle;
        std::vector<int> size_of((size_t)n_bundles);
        for (int b = 0; b < n_bundles; ++b) size_of[(size_t)b] = bundle_size(b);
        for (int sweep = 0, improved = 1; sweep < 8 && improved; ++sweep) {
            improved = 0;
            for (int i = 0; i < n_units; ++i)
                for (int j = (i / per_bundle + 1) * per_bundle; j < n_units; ++j) {
                    const int bi = i / per_bundle, bj = j / per_bundle;
                    std::swap(sequence[(size_t)i], sequence[(size_t)j]);
                    const int si = bundle_size(bi), sj = bundle_size(bj);
                    if (si + sj < size_of[(size_t)bi] + size_of[(size_t)bj]) {
                        size_of[(size_t)bi] = si;
                        size_of[(size_t)bj] = sj;
                        improved = 1;
                    } else {
                        std::swap(sequence[(size_t)i], sequence[(size_t)j]);
                    }
                }
        }
        std::vector<int32_t> old(perm[t], perm[t] + c);
        for (int i = 0; i < n_units; ++i)
            std::copy(old.begin() + (size_t)sequence[(size_t)i] * unit, old.begin() + (size_t)(sequence[(size_t)i] + 1) * unit,
                      perm[t] + (size_t)i * unit);
    }
    return SBN_OK;
}

// The chain / tree form, tensors numbered as in sbn_rearrange_impl.
static int sbn_order_groups_impl(const sbn_layer_desc_t* layers, int n_layers, const int* parent, const int* keep_output_order,
                                 int pct, int32_t* const* perm)
{
    clear_error();
    if (!layers || !parent || !perm || n_layers < 0) return fail(SBN_EINVAL, "sbn_order_groups: NULL pointer");
    for (int l = 0; l < n_layers; ++l) {
        if (!perm[l]) return fail(SBN_EINVAL, "sbn_order_groups: layer %d has a NULL pointer", l);
        if (parent[l] >= l || parent[l] < -1) return fail(SBN_ESHAPE, "parent[%d] = %d: parents must come first", l, parent[l]);
        if (parent[l] >= 0 && layers[parent[l]].c_out != layers[l].c_in)
            return fail(SBN_ESHAPE, "layer %d reads %d channels but its parent %d writes %d", l, layers[l].c_in, parent[l],
                        layers[parent[l]].c_out);
        if (layers[l].c_in <= 0) return fail(SBN_EINVAL, "c_in and c_out must be positive");
    }
    std::vector<int> in_t((size_t)n_layers), out_t((size_t)n_layers), fixed;
    int n_tensors = n_layers;
    for (int l = 0; l < n_layers; ++l) {
        out_t[(size_t)l] = l;
        in_t[(size_t)l] = parent[l] >= 0 ? parent[l] : n_tensors++;
    }
    fixed.assign((size_t)n_tensors, 0);
    for (int l = 0; l < n_layers; ++l) fixed[(size_t)l] = keep_output_order && keep_output_order[l] ? 1 : 0;
    std::vector<std::vector<int32_t>> extra((size_t)(n_tensors - n_layers));
    std::vector<int32_t*> ptrs((size_t)n_tensors);
    for (int l = 0; l < n_layers; ++l) ptrs[(size_t)l] = perm[l];
    for (int t = n_layers; t < n_tensors; ++t) {
        std::vector<int32_t>& e = extra[(size_t)(t - n_layers)];
        e.resize((size_t)layers[std::find(in_t.begin(), in_t.end(), t) - in_t.begin()].c_in);
        std::iota(e.begin(), e.end(), 0);
        ptrs[(size_t)t] = e.data();
        fixed[(size_t)t] = 1;
    }
    return sbn_order_groups_graph_impl(layers, n_layers, in_t.data(), out_t.data(), n_tensors, fixed.data(), pct, ptrs.data());
}

static int sbn_pack_impl(const sbn_layer_desc_t* d, int device, sbn_packed_t** out)
{
    clear_error();
    if (!d || !out) return fail(SBN_EINVAL, "sbn_pack: NULL pointer");
    *out = nullptr;
    if (!d->w) return fail(SBN_EINVAL, "sbn_pack: weights pointer is NULL");
    if (int rc = check_geometry(d->kind, d->c_in, d->c_out, d->go, d->gi)) return rc;
    if (d->act != SBN_ACT_NONE && d->act != SBN_ACT_RELU) return fail(SBN_EINVAL, "unknown activation %d", d->act);
    if (d->kind == SBN_CONV1X1 && (d->stride != 1 || d->pad != 0))
        return fail(SBN_EINVAL, "1x1 layers need stride 1, pad 0 (got %d, %d)", d->stride, d->pad);
    if (d->kind == SBN_CONV3X3 && ((d->stride != 1 && d->stride != 2) || d->pad != 1))
        return fail(SBN_EINVAL, "3x3 layers need stride 1 or 2 and pad 1 (got %d, %d)", d->stride, d->pad);
    if (device < -1) return fail(SBN_EINVAL, "device must be >= -1");
    if (d->perm_out && !is_permutation(d->perm_out, d->c_out)) return fail(SBN_EPERM, "perm_out is not a permutation of 0..%d", d->c_out - 1);
    if (d->perm_in && !is_permutation(d->perm_in, d->c_in)) return fail(SBN_EPERM, "perm_in is not a permutation of 0..%d", d->c_in - 1);

    if (d->kind == SBN_CONV3X3 && device >= 0 && d->c_in % 4)
        return fail(SBN_ESHAPE, "a 3x3 layer that runs on a device needs c_in to be a multiple of 4 (got %d)", d->c_in);

    std::unique_ptr<sbn_packed> holder(new (std::nothrow) sbn_packed);     // freed on every early return
    sbn_packed* p = holder.get();
    if (!p) return fail(SBN_ENOMEM, "out of host memory");
    {
        p->kind = d->kind;
        p->c_in = d->c_in;
        p->c_out = d->c_out;
        p->go = d->go;
        p->gi = d->gi;
        p->stride = d->stride;
        p->pad = d->pad;
        p->act = d->act;
        p->kh = p->kw = d->kind == SBN_CONV3X3 ? 3 : 1;
        p->device = device;
        const int taps = p->kh * p->kw, go = d->go, gi = d->gi;
        const int rows = d->c_out / go, cols = d->c_in / gi;

        p->perm_out.resize((size_t)d->c_out);
        p->perm_in.resize((size_t)d->c_in);
        for (int i = 0; i < d->c_out; ++i) p->perm_out[(size_t)i] = d->perm_out ? d->perm_out[i] : i;
        for (int i = 0; i < d->c_in; ++i) p->perm_in[(size_t)i] = d->perm_in ? d->perm_in[i] : i;
        p->has_bias = d->bias != nullptr;
        p->bias.assign((size_t)d->c_out, 0.0f);
        if (d->bias)
            for (int i = 0; i < d->c_out; ++i) p->bias[(size_t)i] = d->bias[p->perm_out[(size_t)i]];

        std::vector<float> wp;
        permute_ohwi(d->w, d->c_out, taps, d->c_in, d->perm_out, d->perm_in, wp);

        // Gather kept blocks row by row, ascending channel inside a row.
        p->row_ptr.assign((size_t)rows + 1, 0u);
        const size_t blk = (size_t)taps * gi * go;
        for (int i = 0; i < rows; ++i) {
            for (int j = 0; j < cols; ++j) {
                bool kept;
                if (d->mask) {
                    kept = d->mask[(size_t)i * cols + j] != 0;
                } else {
                    kept = false;
                    for (int o = 0; o < go && !kept; ++o)
                        for (int t = 0; t < taps && !kept; ++t) {
                            const float* q = wp.data() + ((size_t)(i * go + o) * taps + t) * d->c_in + (size_t)j * gi;
                            for (int c = 0; c < gi; ++c) {
                                uint32_t bits;
                                std::memcpy(&bits, q + c, 4);
                                if (bits & 0x7FFFFFFFu) {
                                    kept = true;
                                    break;
                                }
                            }
                        }
                }
                if (!kept) continue;
                p->kidx.push_back((uint16_t)(j * gi));
                const size_t base = p->vals.size();
                p->vals.resize(base + blk);
                for (int t = 0; t < taps; ++t)
                    for (int c = 0; c < gi; ++c)
                        for (int o = 0; o < go; ++o)
                            p->vals[base + ((size_t)t * gi + c) * go + o] =
                                wp[((size_t)(i * go + o) * taps + t) * d->c_in + (size_t)j * gi + c];
            }
            p->row_ptr[(size_t)i + 1] = (uint32_t)p->kidx.size();
        }
        build_device_layout(p);
    }
    if (const char* what = check_device_layout(p))
        return fail(SBN_EINVAL, "internal error: device layout is inconsistent (%s)", what);
    if (device >= 0)
        if (int rc = upload_device_layout(p)) return rc;
    *out = holder.release();
    return SBN_OK;
}

int sbn_unpack(const sbn_packed_t* p, float* w_out, uint8_t* mask_out)
{
    clear_error();
    if (!p || !w_out) return fail(SBN_EINVAL, "sbn_unpack: NULL pointer");
    const int taps = p->kh * p->kw, go = p->go, gi = p->gi;
    const int rows = p->c_out / go, cols = p->c_in / gi;
    std::fill(w_out, w_out + (size_t)p->c_out * taps * p->c_in, 0.0f);
    if (mask_out) std::fill(mask_out, mask_out + (size_t)rows * cols, (uint8_t)0);
    const size_t blk = (size_t)taps * gi * go;
    for (int i = 0; i < rows; ++i)
        for (uint32_t e = p->row_ptr[(size_t)i]; e < p->row_ptr[(size_t)i + 1]; ++e) {
            const int k0 = p->kidx[e];
            if (mask_out) mask_out[(size_t)i * cols + k0 / gi] = 1;
            for (int t = 0; t < taps; ++t)
                for (int c = 0; c < gi; ++c)
                    for (int o = 0; o < go; ++o) {
                        const int fo = p->perm_out[(size_t)(i * go + o)];
                        const int co = p->perm_in[(size_t)(k0 + c)];
                        w_out[((size_t)fo * taps + t) * p->c_in + co] = p->vals[e * blk + ((size_t)t * gi + c) * go + o];
                    }
        }
    return SBN_OK;
}

int sbn_export(const sbn_packed_t* p, uint32_t* row_ptr, uint16_t* kidx, float* vals, int32_t* perm_out,
               int32_t* perm_in, float* bias, size_t* nnz_out)
{
    clear_error();
    if (!p) return fail(SBN_EINVAL, "sbn_export: NULL pointer");
    if (row_ptr) std::copy(p->row_ptr.begin(), p->row_ptr.end(), row_ptr);
    if (kidx) std::copy(p->kidx.begin(), p->kidx.end(), kidx);
    if (vals) std::copy(p->vals.begin(), p->vals.end(), vals);
    if (perm_out) std::copy(p->perm_out.begin(), p->perm_out.end(), perm_out);
    if (perm_in) std::copy(p->perm_in.begin(), p->perm_in.end(), perm_in);
    if (bias) std::copy(p->bias.begin(), p->bias.end(), bias);
    if (nnz_out) *nnz_out = p->kidx.size();
    return SBN_OK;
}

int sbn_packed_info(const sbn_packed_t* p, int* kind, int* c_in, int* c_out, int* go, int* gi, int* stride, int* act,
                    int* device)
{
    clear_error();
    if (!p) return fail(SBN_EINVAL, "sbn_packed_info: NULL pointer");
    if (kind) *kind = p->kind;
    if (c_in) *c_in = p->c_in;
    if (c_out) *c_out = p->c_out;
    if (go) *go = p->go;
    if (gi) *gi = p->gi;
    if (stride) *stride = p->stride;
    if (act) *act = p->act;
    if (device) *device = p->device;
    return SBN_OK;
}

int sbn_packed_work(const sbn_packed_t* p, size_t* nnz, size_t* macs)
{
    clear_error();
    if (!p) return fail(SBN_EINVAL, "sbn_packed_work: NULL pointer");
    if (nnz) *nnz = p->kidx.size();
    if (macs) *macs = p->kidx.size() * (size_t)p->go * p->gi * p->kh * p->kw;
    return SBN_OK;
}

int sbn_packed_layout(const sbn_packed_t* p, size_t* entries, size_t* table_bytes, int* every_piece)
{
    clear_error();
    if (!p) return fail(SBN_EINVAL, "sbn_packed_layout: NULL pointer");
    const DeviceLayout& L = p->dev;
    if (entries) *entries = L.n_entries;
    if (table_bytes)
        *table_bytes = (L.records.size() + L.woff.size() + L.records32.size() + L.woff32.size() + L.desc_s.size()) * sizeof(uint32_t) +
                       (L.wts.size() + L.wts_s.size() + L.bias_padded.size()) * sizeof(float);
    if (every_piece) *every_piece = L.desc_s.empty() ? 0 : 1;
    return SBN_OK;
}

void sbn_free(sbn_packed_t* p)
{
    if (!p) return;
    release_device_layout(p);
    delete p;
}

// ---- entry points whose bodies allocate: no exception leaves the library

int sbn_dw_pattern_select(const float* w, int c, int go, const uint8_t* keep_dense, uint8_t* pattern_out)
{
    return guarded("sbn_dw_pattern_select", [&]() -> int { return sbn_dw_pattern_select_impl(w, c, go, keep_dense, pattern_out); });
}

int sbn_dw_pattern_apply(const float* w, int c, int go, const uint8_t* pattern, float* w_out)
{
    return guarded("sbn_dw_pattern_apply", [&]() -> int { return sbn_dw_pattern_apply_impl(w, c, go, pattern, w_out); });
}

int sbn_rearrange(const sbn_layer_desc_t* layers, int n_layers, const int* parent, const int* keep_output_order,
                  int pct, uint64_t seed, int max_iters, int32_t* const* perm_out)
{
    return guarded("sbn_rearrange", [&]() -> int { return sbn_rearrange_impl(layers, n_layers, parent, keep_output_order, pct, seed, max_iters, perm_out); });
}

int sbn_pack(const sbn_layer_desc_t* d, int device, sbn_packed_t** out)
{
    return guarded("sbn_pack", [&]() -> int { return sbn_pack_impl(d, device, out); });
}

int sbn_rearrange_graph(const sbn_layer_desc_t* layers, int n_layers, const int* in_tensor, const int* out_tensor,
                        int n_tensors, const int* tensor_fixed, int pct, uint64_t seed, int max_iters,
                        int32_t* const* perm_per_tensor_out)
{
    return guarded("sbn_rearrange_graph", [&]() -> int {
        return sbn_rearrange_graph_impl(layers, n_layers, in_tensor, out_tensor, n_tensors, tensor_fixed, pct, seed,
                                        max_iters, perm_per_tensor_out);
    });
}

int sbn_order_groups(const sbn_layer_desc_t* layers, int n_layers, const int* parent, const int* keep_output_order,
                     int pct, int32_t* const* perm_per_layer_inout)
{
    return guarded("sbn_order_groups", [&]() -> int { return sbn_order_groups_impl(layers, n_layers, parent, keep_output_order, pct, perm_per_layer_inout); });
}

int sbn_order_groups_graph(const sbn_layer_desc_t* layers, int n_layers, const int* in_tensor, const int* out_tensor,
                           int n_tensors, const int* tensor_fixed, int pct, int32_t* const* perm_per_tensor_inout)
{
    return guarded("sbn_order_groups_graph", [&]() -> int {
        return sbn_order_groups_graph_impl(layers, n_layers, in_tensor, out_tensor, n_tensors, tensor_fixed, pct,
                                           perm_per_tensor_inout);
    });
}

}  // extern "C"
