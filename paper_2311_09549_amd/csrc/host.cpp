// Host side of libsparsecontract: status text, COO -> CSF conversion, expression parsing,
// validation, derivation of the temporaries (Section 4.2), equal-work tile tables, the
// flop / byte model and the C entry points.  All device work is in kernels.hip.
#include <algorithm>
#include <cctype>
#include <cstdarg>
#include <climits>
#include <cstdio>
#include <cstring>
#include <new>
#include <stdexcept>
#include <set>
#include <string>
#include <vector>

#include "plan.h"

using namespace sck;

// ------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------
namespace {

const char *kStatusText[] = {
    "ok",
    "a required pointer argument is NULL",
    "sparse order must be 2, 3 or 4 and agree with the expression",
    "unknown dtype or operands of different dtypes",
    "a dimension, nnz or node count is negative, inconsistent or exceeds int32",
    "a pos array is not strictly increasing from 0 to the child count",
    "a coordinate is outside its dimension",
    "coordinates are not in lexicographic order",
    "a coordinate is stored twice",
    "the expression is not well-formed index notation",
    "the expression is not in the supported family",
    "the schedule (kind, fuse depth, intermediate name, determinism or rank) is not available",
    "operand shapes or alignment disagree with the expression or the plan",
    "the workspace is smaller than sc_plan_workspace_bytes()",
    "no usable GPU, a HIP call failed, or a host view was given where a device view is required",
    "host allocation failed",
};

size_t esize(sc_dtype d) { return d == SC_F64 ? 8 : 4; }
bool dtype_ok(sc_dtype d) { return d == SC_F32 || d == SC_F64; }

struct Term {
    std::string name;
    std::vector<std::string> idx;
};

// term := ident '(' ident (',' ident)* ')'
bool parse_term(const char *&p, Term &t)
{
    auto skip = [&]() { while (*p && isspace((unsigned char)*p)) ++p; };
    auto ident = [&](std::string &s) {
        skip();
        if (!(isalpha((unsigned char)*p) || *p == '_')) return false;
        const char *b = p;
        while (isalnum((unsigned char)*p) || *p == '_' || *p == '\'') ++p;
        s.assign(b, p);
        return true;
    };
    t.idx.clear();
    if (!ident(t.name)) return false;
    skip();
    if (*p != '(') return false;
    ++p;
    for (;;) {
        std::string s;
        if (!ident(s)) return false;
        t.idx.push_back(s);
        skip();
        if (*p == ',') { ++p; continue; }
        if (*p == ')') { ++p; break; }
        return false;
    }
    return true;
}

// expr := term ('=' | '+=') term ('*' term)*
bool parse_expr(const char *s, Term &lhs, std::vector<Term> &rhs)
{
    const char *p = s;
    auto skip = [&]() { while (*p && isspace((unsigned char)*p)) ++p; };
    if (!parse_term(p, lhs)) return false;
    skip();
    if (*p == '+') ++p;
    if (*p != '=') return false;
    ++p;
    rhs.clear();
    for (;;) {
        Term t;
        if (!parse_term(p, t)) return false;
        rhs.push_back(t);
        skip();
        if (*p == '*') { ++p; continue; }
        if (*p == '\0') break;
        return false;
    }
    return true;
}

bool contains(const std::vector<std::string> &v, const std::string &s)
{
    return std::find(v.begin(), v.end(), s) != v.end();
}

std::string join(const std::string &name, const std::vector<std::string> &idx)
{
    std::string r = name + "(";
    for (size_t i = 0; i < idx.size(); ++i) r += (i ? "," : "") + idx[i];
    return r + ")";
}

struct Family {
    Kind kind;
    int slot_of_factor[4];  // canonical slot -> position among the dense factors (0-based after the sparse operand)
    std::vector<std::vector<std::string>> temp_idx;  // derived temporaries, deepest producer first
    std::vector<std::string> temp_name;
};

// Classify a parsed expression into the supported family and derive the index sets of the
// temporaries: indices of the producer that also occur in the consumer or in the output
// (worked example of Section 4.2).  The producer always starts at the sparse operand and
// absorbs the factors from the LAST sparse mode backwards, so that each temporary is
// attached to a prefix of the CSF tree.
sc_status classify(const Term &lhs, const std::vector<Term> &rhs, Family &fam)
{
    if (rhs.size() < 2) return SC_ERR_EXPR_UNSUPPORTED;
    const Term &sp = rhs[0];
    const size_t d = sp.idx.size();
    if (d < 2 || d > 4) return SC_ERR_EXPR_UNSUPPORTED;
    {
        std::set<std::string> u(sp.idx.begin(), sp.idx.end());
        if (u.size() != d) return SC_ERR_EXPR_UNSUPPORTED;
    }
    const size_t nf = rhs.size() - 1;
    for (size_t f = 1; f <= nf; ++f)
        if (rhs[f].idx.size() != 2 || rhs[f].idx[0] == rhs[f].idx[1]) return SC_ERR_EXPR_UNSUPPORTED;
    if (d == 3 && nf == 3 && lhs.idx.size() == 3 && !contains(sp.idx, lhs.idx[0])) {
        // B(i,j,k) * C(i,l) * D(j,m) * E(k,n) -> A(l,m,n): a factor on every mode, no sparse index in the output
        // (kernel 5 of Table 2).  Temporaries of its second schedule: the producer B*E keeps {i,j,n}, B*E*D keeps {i,m,n}.
        int on[3];
        for (size_t m = 0; m < 3; ++m) {
            on[m] = -1;
            for (size_t f = 1; f <= nf; ++f)
                if (rhs[f].idx[0] == sp.idx[m]) {
                    if (on[m] >= 0) return SC_ERR_EXPR_UNSUPPORTED;
                    on[m] = (int)f;
                }
            if (on[m] < 0) return SC_ERR_EXPR_UNSUPPORTED;
        }
        std::set<std::string> ux;
        for (size_t m = 0; m < 3; ++m) {
            const std::string &xi = rhs[on[m]].idx[1];
            if (contains(sp.idx, xi) || lhs.idx[m] != xi) return SC_ERR_EXPR_UNSUPPORTED;
            ux.insert(xi);
            fam.slot_of_factor[m] = on[m] - 1;
        }
        if (ux.size() != 3) return SC_ERR_EXPR_UNSUPPORTED;
        fam.kind = K_TTMC_ALL;
        fam.temp_idx = {{sp.idx[0], sp.idx[1], lhs.idx[2]}, {sp.idx[0], lhs.idx[1], lhs.idx[2]}};
        fam.temp_name = {"T1", "T2"};
        return SC_OK;
    }
    if (lhs.idx.empty() || lhs.idx[0] != sp.idx[0]) return SC_ERR_EXPR_UNSUPPORTED;

    auto find_on = [&](const std::string &first, int skip_pos) -> int {
        for (size_t f = 1; f <= nf; ++f)
            if ((int)f != skip_pos && rhs[f].idx[0] == first) return (int)f;
        return -1;
    };

    if (d == 3 && nf == 3 && lhs.idx.size() == 2) {
        // B(i,j,k) * C(j,r) * D(k,r) * E(r,m) -> A(i,m): the MTTKRP followed by a dense product (kernel 8 of Table 2)
        const int c = find_on(sp.idx[1], -1), dd = find_on(sp.idx[2], -1);
        if (c < 0 || dd < 0 || c == dd) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &r = rhs[c].idx[1];
        if (rhs[dd].idx[1] != r || contains(sp.idx, r)) return SC_ERR_EXPR_UNSUPPORTED;
        int e = -1;
        for (size_t f = 1; f <= nf; ++f)
            if ((int)f != c && (int)f != dd) e = (int)f;
        if (e < 0 || rhs[e].idx[0] != r) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &m = rhs[e].idx[1];
        if (contains(sp.idx, m) || m == r || lhs.idx[1] != m) return SC_ERR_EXPR_UNSUPPORTED;
        fam.kind = K_MTTKRP_GEMM;
        fam.slot_of_factor[0] = c - 1; fam.slot_of_factor[1] = dd - 1; fam.slot_of_factor[2] = e - 1;
        fam.temp_idx = {{sp.idx[0], sp.idx[1], r}, {sp.idx[0], r}};
        fam.temp_name = {"T1", "T2"};
        return SC_OK;
    }
    if (d == 2 && nf == 4) {
        // S(i,j) * X(i,k) * Y(j,k) * Z(j,l) * F(l,m) -> A(i,m): kernel 1 followed by a dense product (kernel 2 of Table 2)
        if (lhs.idx.size() != 2) return SC_ERR_EXPR_UNSUPPORTED;
        const int x = find_on(sp.idx[0], -1);
        if (x < 0) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &k = rhs[x].idx[1];
        int y = -1, z = -1, ff = -1;
        for (size_t f = 1; f <= nf; ++f) {
            if ((int)f == x) continue;
            if (rhs[f].idx[0] == sp.idx[1]) {
                if (rhs[f].idx[1] == k) { if (y >= 0) return SC_ERR_EXPR_UNSUPPORTED; y = (int)f; }
                else { if (z >= 0) return SC_ERR_EXPR_UNSUPPORTED; z = (int)f; }
            } else {
                if (ff >= 0) return SC_ERR_EXPR_UNSUPPORTED;
                ff = (int)f;
            }
        }
        if (y < 0 || z < 0 || ff < 0) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &l = rhs[z].idx[1];
        if (rhs[ff].idx[0] != l) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &m = rhs[ff].idx[1];
        if (contains(sp.idx, k) || contains(sp.idx, l) || contains(sp.idx, m) || m == l || m == k || l == k) return SC_ERR_EXPR_UNSUPPORTED;
        if (lhs.idx[1] != m) return SC_ERR_EXPR_UNSUPPORTED;
        fam.kind = K_SDDMM_SPMM_GEMM;
        fam.slot_of_factor[0] = x - 1; fam.slot_of_factor[1] = y - 1; fam.slot_of_factor[2] = z - 1; fam.slot_of_factor[3] = ff - 1;
        fam.temp_idx = {{sp.idx[0], sp.idx[1]}, {sp.idx[0], l}};
        fam.temp_name = {"T1", "T2"};
        return SC_OK;
    }
    if (d == 2 && nf == 3) {
        // S(i,j) * X(i,k) * Y(j,k) * Z(j,l) -> A(i,l)
        int x = find_on(sp.idx[0], -1);
        if (x < 0) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &k = rhs[x].idx[1];
        int y = -1, z = -1;
        for (size_t f = 1; f <= nf; ++f) {
            if ((int)f == x) continue;
            if (rhs[f].idx[0] != sp.idx[1]) return SC_ERR_EXPR_UNSUPPORTED;
            if (rhs[f].idx[1] == k) y = (int)f; else z = (int)f;
        }
        if (y < 0 || z < 0) return SC_ERR_EXPR_UNSUPPORTED;
        const std::string &l = rhs[z].idx[1];
        if (contains(sp.idx, k) || contains(sp.idx, l)) return SC_ERR_EXPR_UNSUPPORTED;
        if (lhs.idx.size() != 2 || lhs.idx[1] != l) return SC_ERR_EXPR_UNSUPPORTED;
        fam.kind = K_SDDMM_SPMM;
        fam.slot_of_factor[0] = x - 1; fam.slot_of_factor[1] = y - 1; fam.slot_of_factor[2] = z - 1;
        fam.temp_idx = {{sp.idx[0], sp.idx[1]}};
        fam.temp_name = {"T"};
        return SC_OK;
    }
    if ((d == 3 && nf == 2) || (d == 4 && nf == 3)) {
        int on[4] = {-1, -1, -1, -1};
        for (size_t m = 1; m < d; ++m) {
            on[m] = find_on(sp.idx[m], -1);
            if (on[m] < 0) return SC_ERR_EXPR_UNSUPPORTED;
            for (size_t q = 1; q < m; ++q) if (on[q] == on[m]) return SC_ERR_EXPR_UNSUPPORTED;
        }
        std::vector<std::string> x;
        for (size_t m = 1; m < d; ++m) {
            const std::string &xi = rhs[on[m]].idx[1];
            if (contains(sp.idx, xi)) return SC_ERR_EXPR_UNSUPPORTED;
            x.push_back(xi);
        }
        for (size_t m = 1; m < d; ++m) fam.slot_of_factor[m - 1] = on[m] - 1;
        const bool all_same = (x[0] == x[1]) && (d == 3);
        std::set<std::string> ux(x.begin(), x.end());
        if (d == 3 && all_same) {
            if (lhs.idx.size() != 2 || lhs.idx[1] != x[0]) return SC_ERR_EXPR_UNSUPPORTED;
            fam.kind = K_MTTKRP3;
            fam.temp_idx = {{sp.idx[0], sp.idx[1], x[0]}};
            fam.temp_name = {"T"};
            return SC_OK;
        }
        if (ux.size() != x.size()) return SC_ERR_EXPR_UNSUPPORTED;
        if (lhs.idx.size() != d) return SC_ERR_EXPR_UNSUPPORTED;
        for (size_t m = 1; m < d; ++m) if (lhs.idx[m] != x[m - 1]) return SC_ERR_EXPR_UNSUPPORTED;
        if (d == 3) {
            fam.kind = K_TTMC3;
            fam.temp_idx = {{sp.idx[0], sp.idx[1], x[1]}};
            fam.temp_name = {"T"};
        } else {
            fam.kind = K_TTMC4;
            fam.temp_idx = {{sp.idx[0], sp.idx[1], sp.idx[2], x[2]}, {sp.idx[0], sp.idx[1], x[1], x[2]}};
            fam.temp_name = {"T1", "T2"};
        }
        return SC_OK;
    }
    return SC_ERR_EXPR_UNSUPPORTED;
}

// ------------------------------------------------------------------------------------------
// structure validation
// ------------------------------------------------------------------------------------------
sc_status check_header(int32_t order, const int64_t *dims, int64_t nnz, sc_dtype dtype)
{
    if (order < 2 || order > 4) return SC_ERR_BAD_ORDER;
    if (!dtype_ok(dtype)) return SC_ERR_BAD_DTYPE;
    for (int m = 0; m < order; ++m)
        if (dims[m] <= 0 || dims[m] > INT32_MAX) return SC_ERR_BAD_DIMS;
    if (nnz < 0 || nnz > INT32_MAX - 4096) return SC_ERR_BAD_DIMS;
    return SC_OK;
}

// Node counts of a CSF view: non-negative, non-decreasing from the root to the leaves, the leaf
// count equal to nnz, no more slices than the first dimension, all zero exactly when nothing is stored.
sc_status check_node_counts(const sc_csf_view *v)
{
    const int d = v->order;
    if (v->nfib[d - 1] != v->nnz) return SC_ERR_BAD_DIMS;
    for (int m = 0; m < d; ++m) {
        if (v->nfib[m] < 0 || v->nfib[m] > v->nnz) return SC_ERR_BAD_DIMS;
        if (m && v->nfib[m] < v->nfib[m - 1]) return SC_ERR_BAD_DIMS;
        if ((v->nfib[m] == 0) != (v->nnz == 0)) return SC_ERR_BAD_DIMS;
    }
    if (v->nfib[0] > v->dims[0]) return SC_ERR_BAD_DIMS;
    return SC_OK;
}

// Host arrays of a CSF view (copied from the device when needed).
struct HostCsf {
    std::vector<int32_t> pos_store[4], crd_store[4];
    const int32_t *pos[4] = {nullptr, nullptr, nullptr, nullptr};
    const int32_t *crd[4] = {nullptr, nullptr, nullptr, nullptr};
    bool have_crd = false;
};

sc_status fetch_csf(const sc_csf_view *v, HostCsf &h, bool want_crd)
{
    for (int m = 0; m < v->order; ++m) {
        const int64_t npos = m ? v->nfib[m - 1] + 1 : 0;
        const int64_t ncrd = v->nfib[m];
        if (m && !v->pos[m]) return SC_ERR_NULL;
        if (ncrd > 0 && !v->crd[m]) return SC_ERR_NULL;
        if (!v->on_device) {
            h.pos[m] = v->pos[m];
            h.crd[m] = v->crd[m];
            continue;
        }
        try {
            if (m) h.pos_store[m].resize((size_t)npos);
            if (want_crd) h.crd_store[m].resize((size_t)ncrd);
        } catch (const std::bad_alloc &) { return SC_ERR_ALLOC; }
        if (m && hipMemcpy(h.pos_store[m].data(), v->pos[m], sizeof(int32_t) * (size_t)npos, hipMemcpyDeviceToHost) != hipSuccess)
            return SC_ERR_DEVICE;
        if (want_crd && ncrd &&
            hipMemcpy(h.crd_store[m].data(), v->crd[m], sizeof(int32_t) * (size_t)ncrd, hipMemcpyDeviceToHost) != hipSuccess)
            return SC_ERR_DEVICE;
        h.pos[m] = m ? h.pos_store[m].data() : nullptr;
        h.crd[m] = want_crd ? h.crd_store[m].data() : nullptr;
    }
    h.have_crd = want_crd || !v->on_device;
    return SC_OK;
}

sc_status validate_csf(const sc_csf_view *v, const HostCsf &h)
{
    sc_status st = check_header(v->order, v->dims, v->nnz, v->dtype);
    if (st != SC_OK) return st;
    const int d = v->order;
    st = check_node_counts(v);
    if (st != SC_OK) return st;
    if (v->nnz > 0 && !v->vals) return SC_ERR_NULL;
    for (int m = 1; m < d; ++m) {
        const int32_t *pos = h.pos[m];
        const int64_t np = v->nfib[m - 1];
        if (pos[0] != 0 || pos[np] != v->nfib[m]) return SC_ERR_BAD_POS;
        for (int64_t p = 0; p < np; ++p)
            if (pos[p + 1] <= pos[p]) return SC_ERR_BAD_POS;
    }
    if (!h.have_crd) return SC_OK;
    for (int m = 0; m < d; ++m) {
        const int32_t *crd = h.crd[m];
        const int64_t n = v->nfib[m];
        for (int64_t c = 0; c < n; ++c)
            if (crd[c] < 0 || crd[c] >= v->dims[m]) return SC_ERR_CRD_RANGE;
        if (m == 0) {
            for (int64_t c = 1; c < n; ++c) {
                if (crd[c] == crd[c - 1]) return SC_ERR_DUPLICATE;
                if (crd[c] < crd[c - 1]) return SC_ERR_UNSORTED;
            }
        } else {
            const int32_t *pos = h.pos[m];
            for (int64_t p = 0; p < v->nfib[m - 1]; ++p)
                for (int64_t c = pos[p] + 1; c < pos[p + 1]; ++c) {
                    if (crd[c] == crd[c - 1]) return SC_ERR_DUPLICATE;
                    if (crd[c] < crd[c - 1]) return SC_ERR_UNSORTED;
                }
        }
    }
    return SC_OK;
}

sc_status validate_coo(const sc_coo_view *c)
{
    if (!c) return SC_ERR_NULL;
    sc_status st = check_header(c->order, c->dims, c->nnz, c->dtype);
    if (st != SC_OK) return st;
    if (c->on_device) return SC_ERR_DEVICE;
    if (c->nnz == 0) return SC_OK;
    for (int m = 0; m < c->order; ++m)
        if (!c->crd[m]) return SC_ERR_NULL;
    for (int64_t z = 0; z < c->nnz; ++z) {
        for (int m = 0; m < c->order; ++m)
            if (c->crd[m][z] < 0 || c->crd[m][z] >= c->dims[m]) return SC_ERR_CRD_RANGE;
        if (z) {
            int cmp = 0;
            for (int m = 0; m < c->order && cmp == 0; ++m)
                cmp = (c->crd[m][z] > c->crd[m][z - 1]) - (c->crd[m][z] < c->crd[m][z - 1]);
            if (cmp == 0) return SC_ERR_DUPLICATE;
            if (cmp < 0) return SC_ERR_UNSORTED;
        }
    }
    return SC_OK;
}

// ------------------------------------------------------------------------------------------
// tiles
// ------------------------------------------------------------------------------------------

// Node of level `lvl` that contains node `x` of level `lvl + 1` (pos = pos[lvl + 1]).
inline int32_t parent_of(const int32_t *pos, int64_t nparent, int32_t x)
{
    return (int32_t)(std::upper_bound(pos, pos + nparent + 1, x) - pos) - 1;
}

// Builds the tile table: leaves are cut into runs of at most caps.tn, shortened so that no
// tile touches more than caps.ta level-a nodes (and caps.tb level-b nodes for order 4).
void build_tiles(const sc_csf_view *v, const HostCsf &h, const TileCaps &caps, std::vector<TileRec> &tiles)
{
    const int d = v->order;
    const int64_t nnz = v->nnz;
    tiles.clear();
    // level indices: leaves = d-1, a = d-2, b = d-3, c = d-4
    const int la = d - 2, lb = d - 3, lc = d - 4;
    int64_t n0 = 0;
    while (n0 < nnz) {
        TileRec t;
        memset(&t, 0, sizeof(t));
        int64_t n1 = std::min<int64_t>(n0 + caps.tn, nnz);
        const int32_t a0 = parent_of(h.pos[la + 1], v->nfib[la], (int32_t)n0);
        if ((int64_t)a0 + caps.ta < v->nfib[la]) n1 = std::min<int64_t>(n1, h.pos[la + 1][a0 + caps.ta]);
        int32_t b0 = 0, c0 = 0;
        if (lb >= 0) {
            b0 = parent_of(h.pos[lb + 1], v->nfib[lb], a0);
            if (caps.tb > 0 && (int64_t)b0 + caps.tb < v->nfib[lb])
                n1 = std::min<int64_t>(n1, h.pos[la + 1][h.pos[lb + 1][b0 + caps.tb]]);
        }
        if (lc >= 0) c0 = parent_of(h.pos[lc + 1], v->nfib[lc], b0);
        const int32_t a1 = parent_of(h.pos[la + 1], v->nfib[la], (int32_t)(n1 - 1));
        t.n0 = (int32_t)n0; t.n1 = (int32_t)n1;
        t.a0 = a0; t.na = a1 - a0 + 1;
        int32_t flags = 0;
        if (h.pos[la + 1][a0] < n0) flags |= 1;
        if (h.pos[la + 1][a1 + 1] > n1) flags |= 2;
        if (lb >= 0) {
            const int32_t b1 = parent_of(h.pos[lb + 1], v->nfib[lb], a1);
            t.b0 = b0; t.nb = b1 - b0 + 1;
            if (h.pos[la + 1][h.pos[lb + 1][b0]] < n0) flags |= 4;
            if (h.pos[la + 1][h.pos[lb + 1][b1 + 1]] > n1) flags |= 8;
            if (lc >= 0) {
                const int32_t c1 = parent_of(h.pos[lc + 1], v->nfib[lc], b1);
                t.c0 = c0; t.nc = c1 - c0 + 1;
                if (h.pos[la + 1][h.pos[lb + 1][h.pos[lc + 1][c0]]] < n0) flags |= 16;
                if (h.pos[la + 1][h.pos[lb + 1][h.pos[lc + 1][c1 + 1]]] > n1) flags |= 32;
            }
        }
        t.flags = flags;
        tiles.push_back(t);
        n0 = n1;
    }
}

void appendf(std::string &s, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// Walk tables of a plan (see WalkTables): the coordinate arrays of the two lowest levels with the
// end-of-node bits folded in, and per tile the node at the head of every lane group's chunk.  `order`
// is the device tile table.
sc_status build_walk_tables(sc_plan *p, const sc_csf_view *v, const HostCsf &h, const std::vector<TileRec> &order)
{
    WalkTables &w = p->walk;
    const int d = v->order;
    if (w.shape.levels <= 0 || !h.have_crd || order.empty()) return SC_OK;
    if (p->caps.ta > 0x7fff || p->caps.tb > 0x7fff) return SC_ERR_SCHED_UNSUPPORTED;   // a chunk head holds a tile-local node number in 15 bits
    size_t table_bytes = 0;
    try {
        for (int lv = 0; lv < w.shape.levels; ++lv) {
            const int m = d - 1 - lv;                 // CSF level of the children
            const int64_t n = v->nfib[m], nparent = v->nfib[m - 1];
            std::vector<uint32_t> rec((size_t)n);
            for (int64_t c = 0; c < n; ++c) rec[(size_t)c] = (uint32_t)h.crd[m][c];
            for (int64_t f = 0; f < nparent; ++f) rec[(size_t)h.pos[m][f + 1] - 1] |= 0x80000000u;
            if (hipMalloc((void **)&w.d_rec[lv], sizeof(uint32_t) * (size_t)n) != hipSuccess) return SC_ERR_DEVICE;
            if (hipMemcpy(w.d_rec[lv], rec.data(), sizeof(uint32_t) * (size_t)n, hipMemcpyHostToDevice) != hipSuccess) return SC_ERR_DEVICE;
            table_bytes += sizeof(uint32_t) * (size_t)n;
        }
        const int g0 = w.shape.groups[0], g1 = w.shape.levels > 1 ? w.shape.groups[1] : 0;
        w.heads_per_tile = (g0 + g1 + 1) / 2 * 2;
        std::vector<uint16_t> heads(order.size() * (size_t)w.heads_per_tile, 0);
        for (size_t t = 0; t < order.size(); ++t) {
            const TileRec &tr = order[t];
            uint16_t *hd = heads.data() + t * (size_t)w.heads_per_tile;
            // leaf walk: children n0 .. n1 of the nodes a0 .. of level d - 2
            {
                const int32_t *pos = h.pos[d - 1];
                const int n = tr.n1 - tr.n0, q = walk_chunk(n, g0, w.shape.batch[0]);
                int32_t node = tr.a0;
                for (int g = 0; g < g0 && (int64_t)g * q < n; ++g) {
                    const int32_t x = tr.n0 + g * q;
                    while (pos[node + 1] <= x) ++node;
                    const bool head = g > 0 && pos[node] != x;
                    hd[g] = (uint16_t)((node - tr.a0) | (head ? 0x8000 : 0));
                }
            }
            if (w.shape.levels > 1) {   // the walk one level up: children a0 .. a0 + na of the nodes b0 ..
                const int32_t *pos = h.pos[d - 2];
                const int n = tr.na, q = walk_chunk(n, g1, w.shape.batch[1]);
                int32_t node = tr.b0;
                for (int g = 0; g < g1 && (int64_t)g * q < n; ++g) {
                    const int32_t x = tr.a0 + g * q;
                    while (pos[node + 1] <= x) ++node;
                    const bool head = g > 0 && pos[node] != x;
                    hd[g0 + g] = (uint16_t)((node - tr.b0) | (head ? 0x8000 : 0));
                }
            }
        }
        if (hipMalloc((void **)&w.d_heads, sizeof(uint16_t) * heads.size()) != hipSuccess) return SC_ERR_DEVICE;
        if (hipMemcpy(w.d_heads, heads.data(), sizeof(uint16_t) * heads.size(), hipMemcpyHostToDevice) != hipSuccess) return SC_ERR_DEVICE;
        table_bytes += sizeof(uint16_t) * heads.size();
        appendf(p->text, "walk tables: %zu bytes of plan-owned device memory (coordinates of the walked levels with the end-of-node bits, chunk heads per tile)\n",
                table_bytes);
    } catch (const std::bad_alloc &) { return SC_ERR_ALLOC; }
    return SC_OK;
}

// Top level of a tile record ("a" for order 2, "b" for order 3, "c" for order 4): whether its
// first / last slice continues from the previous / into the next tile, first slice, slice count.
struct TopLevel {
    bool in, out;
    int32_t top0, ntop;
};
TopLevel top_level(int order, const TileRec &t)
{
    const bool o4 = order == 4, o2 = order == 2;
    const int32_t in_bit = o4 ? 16 : o2 ? 1 : 4, out_bit = o4 ? 32 : o2 ? 2 : 8;
    return {(t.flags & in_bit) != 0, (t.flags & out_bit) != 0, o4 ? t.c0 : o2 ? t.a0 : t.b0, o4 ? t.nc : o2 ? t.na : t.nb};
}

// Lists the output rows that the kernels do not overwrite completely and that therefore have
// to be zero before they run: rows of empty slices and, unless the schedule is deterministic
// (then a last kernel writes them), rows whose slice spans several tiles and is accumulated
// atomically.  Every other row is stored whole by the one tile that holds its slice.
void list_rows_to_zero(sc_plan *p, const HostCsf &h)
{
    p->zero_rows.clear();
    p->zero_selective = false;
    if (p->sched == SC_SCHED_LINEAR) return;   // every row is accumulated atomically: the whole output starts at zero
    const int64_t rows = p->dims[0];
    std::vector<char> stored((size_t)rows, 0);
    for (int64_t s = 0; s < p->nfib[0]; ++s) stored[(size_t)h.crd[0][s]] = 1;
    p->zero_rows.clear();
    for (int64_t r = 0; r < rows; ++r)
        if (!stored[(size_t)r]) p->zero_rows.push_back((int32_t)r);
    if (!p->deterministic) {
        // Kernels that take one tile per workgroup add every piece of a spanning slice atomically.  The persistent
        // kernels keep such a slice in registers from tile to tile of a run and add only what crosses a run's end.
        const int run = plan_output_run(p);
        int32_t last_listed = -1;
        for (size_t n = 0; n < p->tiles.size(); ++n) {
            const TileRec &t = p->tiles[n];
            const TopLevel tl = top_level(p->order, t);
            if (!tl.out) continue;
            const int32_t row = h.crd[0][tl.top0 + tl.ntop - 1];
            if (run > 0) {
                if ((n + 1) % (size_t)run != 0) continue;        // continues inside the run
                if (row == last_listed) continue;                // a slice crossing several runs' ends is listed once
            } else if (tl.in && tl.ntop == 1) {
                continue;                                        // listed where the slice starts
            }
            p->zero_rows.push_back(row);
            last_listed = row;
        }
    }
    p->zero_selective = (int64_t)p->zero_rows.size() * 2 <= rows;
    if (!p->zero_selective) {
        p->zero_rows.clear();
        p->zero_rows.shrink_to_fit();
    }
}

// Deterministic schedules: numbers the pieces of every output row that spans several tiles
// (consecutive slots in tile order) and lists those rows.  The top level is "a" for order 2, "b"
// for order 3 and "c" for order 4; its flag bits say whether the tile's first / last slice continues
// from the previous / into the next tile.  A tile whose only slice does both holds one piece.
// Cuts the pieces of every spanning row into the segments of the first fix-up pass; a row's
// segments are consecutive.  On entry a record holds {row, first slot, pieces}.
void make_segments(FixLevel &lv)
{
    lv.segs.clear();
    for (FixRec &f : lv.fix) {
        const int32_t slot0 = f.first, pieces = f.count;
        f.first = (int32_t)lv.segs.size();
        f.count = (pieces + kFixSegment - 1) / kFixSegment;
        for (int32_t s0 = 0; s0 < pieces; s0 += kFixSegment) {
            FixRec g;
            g.row = (int32_t)lv.segs.size();
            g.first = slot0 + s0;
            g.count = std::min<int32_t>(kFixSegment, pieces - s0);
            g.pad = 0;
            lv.segs.push_back(g);
        }
    }
}

void assign_piece_slots(sc_plan *p, const HostCsf &h)
{
    // output rows
    FixLevel &top = p->det_top;
    top.rowlen = p->out_row_elems;
    int32_t next = 0;
    top.fix.clear();
    for (TileRec &t : p->tiles) {
        const TopLevel tl = top_level(p->order, t);
        t.pad[0] = t.pad[1] = t.pad[2] = -1;
        if (tl.in) {   // a piece of the row that the previous tile left open
            t.pad[0] = next++;
            top.fix.back().count++;
        }
        if (tl.out && !(tl.in && tl.ntop == 1)) {   // the tile's last slice starts here and goes on
            FixRec f;
            f.row = h.crd[0][tl.top0 + tl.ntop - 1];
            f.first = next;
            f.count = 1;
            f.pad = 0;
            top.fix.push_back(f);
            t.pad[1] = next++;
        }
    }
    top.n_slots = next;
    make_segments(top);

    // FISSIONED, order >= 3: rows of the first temporary, one per leaf fiber (level "a", flag bits 1 / 2)
    FixLevel &la = p->det_a;
    la.fix.clear();
    la.n_slots = 0;
    if (p->sched == SC_SCHED_FISSIONED && p->order >= 3) {
        la.rowlen = p->kind == K_TTMC4 ? p->fcols[2] : p->kind == K_TTMC3 ? p->fcols[1] : p->fcols[0];   // width of the temporary's rows
        next = 0;
        for (TileRec &t : p->tiles) {
            const bool in = (t.flags & 1) != 0, out = (t.flags & 2) != 0;
            t.pad[2] = next;
            if (in) {
                ++next;
                la.fix.back().count++;
            }
            if (out && !(in && t.na == 1)) {
                FixRec f;
                f.row = t.a0 + t.na - 1;   // position of the fiber = row of the temporary
                f.first = next++;
                f.count = 1;
                f.pad = 0;
                la.fix.push_back(f);
            }
        }
        la.n_slots = next;
        make_segments(la);
    }

    // FISSIONED, order 4: rows of the second temporary, one per level-b node (flag bits 4 / 8)
    FixLevel &lb = p->det_b;
    lb.fix.clear();
    lb.n_slots = 0;
    p->slot_b.clear();
    if (p->sched == SC_SCHED_FISSIONED && p->order == 4) {
        lb.rowlen = p->fcols[1] * p->fcols[2];
        next = 0;
        for (const TileRec &t : p->tiles) {
            const bool in = (t.flags & 4) != 0, out = (t.flags & 8) != 0;
            p->slot_b.push_back(next);
            if (in) {
                ++next;
                lb.fix.back().count++;
            }
            if (out && !(in && t.nb == 1)) {
                FixRec f;
                f.row = t.b0 + t.nb - 1;   // position of the node = row of the temporary
                f.first = next++;
                f.count = 1;
                f.pad = 0;
                lb.fix.push_back(f);
            }
        }
        lb.n_slots = next;
        make_segments(lb);
    }
}

void appendf(std::string &s, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void appendf(std::string &s, const char *fmt, ...)
{
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    s += buf;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// tuning knobs
// ------------------------------------------------------------------------------------------
sck::Tuning &sck::tuning()
{
    static Tuning t;
    return t;
}

extern "C" sc_status sc_tuning_set(const char *name, int64_t value)
{
    if (!name) return SC_ERR_NULL;
    if (value < 0 || value > (1 << 20)) return SC_ERR_BAD_DIMS;
    Tuning &t = tuning();
    if (!strcmp(name, "tile_leaves")) t.tn = (int32_t)value;
    else if (!strcmp(name, "tile_nodes_a")) t.ta = (int32_t)value;
    else if (!strcmp(name, "tile_nodes_b")) t.tb = (int32_t)value;
    else if (!strcmp(name, "tile_interleave")) t.interleave = (int32_t)value;
    else if (!strcmp(name, "persistent_per_cu")) t.per_cu = (int32_t)value;
    else return SC_ERR_EXPR_PARSE;
    return SC_OK;
}

// ------------------------------------------------------------------------------------------
// C entry points
// ------------------------------------------------------------------------------------------
extern "C" sc_status sc_version(int *major, int *minor)
{
    if (!major || !minor) return SC_ERR_NULL;
    *major = 0;
    *minor = 1;
    return SC_OK;
}

extern "C" const char *sc_status_string(sc_status s)
{
    const int n = (int)(sizeof(kStatusText) / sizeof(kStatusText[0]));
    if ((int)s < 0 || (int)s >= n) return "unknown status";
    return kStatusText[(int)s];
}

// Runs `body` and turns any C++ exception into a status: nothing may cross the C boundary.
template <typename Body>
static sc_status guarded(Body body)
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return SC_ERR_ALLOC;
    } catch (const std::length_error &) {
        return SC_ERR_BAD_DIMS;
    } catch (...) {
        return SC_ERR_BAD_DIMS;
    }
}

static sc_status coo_to_csf_sizes_impl(const sc_coo_view *coo, int64_t nfib_out[4])
{
    if (!coo || !nfib_out) return SC_ERR_NULL;
    sc_status st = validate_coo(coo);
    if (st != SC_OK) return st;
    for (int m = 0; m < 4; ++m) nfib_out[m] = 0;
    const int d = coo->order;
    for (int64_t z = 0; z < coo->nnz; ++z) {
        // first level at which entry z differs from entry z-1: a new node starts there and below
        int first = 0;
        if (z) {
            while (first < d && coo->crd[first][z] == coo->crd[first][z - 1]) ++first;
        }
        for (int m = first; m < d; ++m) nfib_out[m]++;
    }
    return SC_OK;
}

extern "C" sc_status sc_coo_to_csf_sizes(const sc_coo_view *coo, int64_t nfib_out[4])
{
    return guarded([&] { return coo_to_csf_sizes_impl(coo, nfib_out); });
}

static sc_status coo_to_csf_impl(const sc_coo_view *coo, sc_csf_view *out)
{
    if (!coo || !out) return SC_ERR_NULL;
    int64_t nfib[4];
    sc_status st = coo_to_csf_sizes_impl(coo, nfib);
    if (st != SC_OK) return st;
    const int d = coo->order;
    for (int m = 0; m < d; ++m) {
        if (m && !out->pos[m]) return SC_ERR_NULL;
        if (nfib[m] && !out->crd[m]) return SC_ERR_NULL;
    }
    int32_t *pos[4], *crd[4];
    for (int m = 0; m < d; ++m) {
        pos[m] = const_cast<int32_t *>(out->pos[m]);
        crd[m] = const_cast<int32_t *>(out->crd[m]);
    }
    int64_t cnt[4] = {0, 0, 0, 0};
    for (int64_t z = 0; z < coo->nnz; ++z) {
        int first = 0;
        if (z) {
            while (first < d && coo->crd[first][z] == coo->crd[first][z - 1]) ++first;
        }
        for (int m = first; m < d; ++m) {
            // a new node of level m; if its parent (level m-1) is new too, the parent's
            // child range starts here
            if (m > 0 && m - 1 >= first) pos[m][cnt[m - 1] - 1] = (int32_t)cnt[m];
            crd[m][cnt[m]] = coo->crd[m][z];
            cnt[m]++;
        }
    }
    for (int m = 1; m < d; ++m) pos[m][nfib[m - 1]] = (int32_t)nfib[m];
    if (out->vals && coo->nnz) {
        if (!coo->vals) return SC_ERR_NULL;
        memcpy(const_cast<void *>(out->vals), coo->vals, esize(coo->dtype) * (size_t)coo->nnz);
    }
    out->order = coo->order;
    out->nnz = coo->nnz;
    out->dtype = coo->dtype;
    out->on_device = 0;
    for (int m = 0; m < 4; ++m) {
        out->dims[m] = m < d ? coo->dims[m] : 0;
        out->nfib[m] = m < d ? nfib[m] : 0;
    }
    return SC_OK;
}

extern "C" sc_status sc_coo_to_csf(const sc_coo_view *coo, sc_csf_view *out)
{
    return guarded([&] { return coo_to_csf_impl(coo, out); });
}

// Iteration count (multiply = 1, add = 1) and compulsory HBM bytes of one schedule class of an expression,
// from the concrete node counts and ranks (the cost expressions of Section 3, evaluated as in the run-time
// stage of Section 5).  `extra` = bytes a FISSIONED schedule adds by writing and reading its temporaries.
static void schedule_model(const sc_plan *p, sc_sched_kind sched, double *flops_out, double *bytes_out)
{
    const double e = (double)esize(p->dtype), nnz = (double)p->nnz, S = (double)p->nfib[0];
    double fac_bytes = 0;
    for (int s = 0; s < p->nfactors; ++s) fac_bytes += (double)p->frows[s] * (double)p->fcols[s] * e;
    double flops = 0, bytes = 0, extra = 0;
    switch (p->kind) {
    case K_TTMC3: {
        const double F = (double)p->nfib[1], L = (double)p->fcols[0], M = (double)p->fcols[1];
        flops = 2 * M * nnz + 2 * L * M * F;
        bytes = nnz * (4 + e) + F * 8 + S * 8 + fac_bytes + (double)p->out_elems * e;
        extra = 2 * F * M * e;
        break;
    }
    case K_MTTKRP3: {
        const double F = (double)p->nfib[1], R = (double)p->fcols[0];
        flops = 2 * R * (nnz + F);
        bytes = nnz * (4 + e) + F * 8 + S * 8 + fac_bytes + (double)p->out_elems * e;
        extra = 2 * F * R * e;
        break;
    }
    case K_SDDMM_SPMM: {
        const double K = (double)p->fcols[0], L = (double)p->fcols[2];
        flops = nnz * (2 * K + 1 + 2 * L);
        // every array touched once (perfect reuse of the gathered rows)
        bytes = nnz * (4 + e) + S * 8 + S * K * e + (double)p->frows[1] * (K + L) * e + (double)p->out_elems * e;
        extra = 2 * nnz * e;
        break;
    }
    case K_TTMC4: {
        const double F2 = (double)p->nfib[1], F3 = (double)p->nfib[2];
        const double L = (double)p->fcols[0], M = (double)p->fcols[1], N = (double)p->fcols[2];
        flops = 2 * N * nnz + 2 * M * N * F3 + 2 * L * M * N * F2;
        bytes = nnz * (4 + e) + F3 * 8 + F2 * 8 + S * 8 + fac_bytes + (double)p->out_elems * e;
        extra = 2 * F3 * N * e + 2 * F2 * M * N * e;
        break;
    }
    case K_TTMC_ALL:
    case K_MTTKRP_GEMM:
    case K_SDDMM_SPMM_GEMM: break;   // see plan_ttmc_all / plan_trailing_gemm
    }
    if (sched == SC_SCHED_LINEAR) {   // every stored entry times every combination of the dense output indices (and of k for the SDDMM)
        const double per = p->kind == K_SDDMM_SPMM ? 4.0 * (double)p->fcols[0] : (double)(p->nfactors + 1);
        flops = per * (double)p->out_row_elems * nnz;
    }
    if (sched == SC_SCHED_FISSIONED) bytes += extra;
    *flops_out = flops;
    *bytes_out = bytes;
}

// Run-time stage of the scheduler (Section 5, "Time-Complexity-Based Pruning"), for the schedule classes this
// library has kernels for.  The paper keeps the schedules of least iteration count whose auxiliary memory is
// below half of the last-level cache; on this machine the temporary of a fused nest lives in LDS, so a class is
// admissible when kernels exist for the ranks and a workgroup's on-chip buffers leave room for a second
// workgroup on the compute unit.  Among the admissible classes the least predicted time wins, time being
// the larger of iteration count / vector peak and compulsory bytes / HBM peak (ties: fewer bytes first).
struct Candidate {
    sc_sched_kind kind;
    int variant;          // kernel 5 only: schedule of Table 2
    double flops, bytes, seconds;
    size_t lds;
    int wg_per_cu;
    bool available, admissible;
};

static double predicted_seconds(const sc_plan *p, double flops, double bytes)
{
    const double peak_flops = (double)p->n_cu * 64.0 * 2.0 * 2.4e9;   // one fused multiply-add per lane and clock
    const double peak_bytes = 8.0e12 * (double)p->n_cu / 256.0;
    return std::max(flops / peak_flops, bytes / peak_bytes);
}

static const char *sched_name(sc_sched_kind k)
{
    return k == SC_SCHED_LINEAR ? "LINEAR" : k == SC_SCHED_FUSED ? "FUSED" : k == SC_SCHED_FISSIONED ? "FISSIONED" : "AUTO";
}

// Availability and on-chip footprint of one schedule class of an order-2/3/4 contraction.
static void probe_class(const sc_plan *p, sc_sched_kind kind, bool deterministic, Candidate &c)
{
    sc_plan q;
    q.kind = p->kind; q.dtype = p->dtype; q.order = p->order; q.nnz = p->nnz; q.nfactors = p->nfactors;
    for (int m = 0; m < 4; ++m) { q.dims[m] = p->dims[m]; q.nfib[m] = p->nfib[m]; }
    for (int s = 0; s < 3; ++s) { q.frows[s] = p->frows[s]; q.fcols[s] = p->fcols[s]; }
    q.out_elems = p->out_elems; q.out_row_elems = p->out_row_elems;
    q.sched = kind;
    q.deterministic = deterministic;
    q.caps = kind == SC_SCHED_LINEAR ? TileCaps{1024, 1024, 1024} : default_caps(q.kind, q.dtype, kind, q.fcols);
    c.kind = kind;
    c.variant = 0;
    c.available = q.caps.tn > 0 && !(deterministic && (kind == SC_SCHED_LINEAR || !plan_supports_deterministic(&q)));
    c.lds = c.available ? lds_bytes_needed(&q) : 0;
    if (c.lds > 64 * 1024) c.available = false;
    c.wg_per_cu = c.available ? lds_workgroups_per_cu(c.lds, p->lds_per_cu) : 0;
    c.admissible = c.available && c.wg_per_cu >= 2;
}

static void describe_candidates(std::string &tx, const std::vector<Candidate> &cands, size_t best)
{
    appendf(tx, "cost evaluator (run-time stage of Section 5): predicted time = max(iterations / vector peak, compulsory bytes / HBM peak); "
                "admissible = kernels exist and a workgroup's on-chip buffers leave room for a second one per compute unit\n");
    for (size_t n = 0; n < cands.size(); ++n) {
        const Candidate &c = cands[n];
        if (c.variant) appendf(tx, "  candidate Table 2 schedule %d, %s:", c.variant, sched_name(c.kind));
        else appendf(tx, "  candidate %s:", sched_name(c.kind));
        if (!c.available) {
            appendf(tx, " no kernel for these ranks / options\n");
            continue;
        }
        appendf(tx, " %.4g flops, %.4g bytes, %zu bytes of LDS per workgroup (%d per compute unit), predicted %.1f us%s%s\n", c.flops, c.bytes,
                c.lds, c.wg_per_cu, c.seconds * 1e6, c.admissible ? "" : ", not admissible", n == best ? "  <- chosen" : "");
    }
}

static size_t pick_candidate(const std::vector<Candidate> &cands)
{
    size_t best = cands.size();
    for (size_t n = 0; n < cands.size(); ++n) {
        if (!cands[n].admissible) continue;
        if (best == cands.size() || cands[n].seconds < cands[best].seconds ||
            (cands[n].seconds == cands[best].seconds && cands[n].bytes < cands[best].bytes))
            best = n;
    }
    if (best == cands.size())   // nothing admissible: fall back to whatever has a kernel
        for (size_t n = 0; n < cands.size() && best == cands.size(); ++n)
            if (cands[n].available) best = n;
    return best;
}

static sc_status plan_create_impl(sc_plan **out, const char *expr, const sc_csf_view *sparse, const sc_dense_view *factors,
                                  int32_t nfactors, const sc_schedule *sched);

// Kernel 5 of Table 2 (all-mode TTMC).  The caller picks one of the three schedules Table 2 lists by naming
// its temporaries: {T(i,j,n)} = schedule 1, {T1(i,j,n), T2(i,m,n)} or nothing = schedule 2, {T(i,m,n)} = schedule 3.
// The sparse part is planned as an inner order-3 chain over the same tensor with the factors on modes 1 and 2.
static sc_status plan_ttmc_all(sc_plan *p, const char *expr, const Term &lhs, const std::vector<Term> &rhs, const Family &fam,
                               const sc_csf_view *sparse, const sc_dense_view *factors, const sc_schedule *sched)
{
    if (sched->deterministic != 0 && sched->deterministic != 1) return SC_ERR_SCHED_UNSUPPORTED;
    sc_schedule picked = {};
    std::string choice_text;
    int auto_variant = 0;
    if (sched->kind == SC_SCHED_AUTO) {
        // candidates: the three schedules of Table 2 in the classes the library runs them in.  Their iteration counts
        // differ (N nnz + L M N F, N nnz + M N F + L M N S, M N nnz + L M N S); so do the bytes the sparse part moves.
        if (sched->n_intermediates != 0) return SC_ERR_SCHED_UNSUPPORTED;
        const double e = (double)esize(p->dtype), nnz = (double)p->nnz, S = (double)p->nfib[0], F = (double)p->nfib[1];
        const double L = (double)p->fcols[0], M = (double)p->fcols[1], N = (double)p->fcols[2];
        double fb = 0;
        for (int s = 0; s < 3; ++s) fb += (double)p->frows[s] * (double)p->fcols[s] * e;
        const double base = nnz * (4 + e) + F * 8 + S * 8 + fb + (double)p->out_elems * e;
        const double tiles = 2 * (double)p->dims[0] * M * N * e, trows = 2 * F * N * e;
        sc_plan inner;   // the order-3 chain over modes 1 and 2, for availability and LDS footprint
        inner.kind = K_TTMC3; inner.dtype = p->dtype; inner.order = 3; inner.nnz = p->nnz; inner.nfactors = 2;
        for (int m = 0; m < 4; ++m) { inner.dims[m] = p->dims[m]; inner.nfib[m] = p->nfib[m]; }
        inner.frows[0] = p->frows[1]; inner.frows[1] = p->frows[2]; inner.fcols[0] = p->fcols[1]; inner.fcols[1] = p->fcols[2];
        inner.out_row_elems = p->fcols[1] * p->fcols[2];
        inner.out_elems = p->dims[0] * inner.out_row_elems;
        inner.n_cu = p->n_cu; inner.lds_per_cu = p->lds_per_cu;
        struct { int variant; sc_sched_kind outer, inner; double flops, bytes; } opt[4] = {
            {2, SC_SCHED_FUSED, SC_SCHED_FUSED, 2 * N * nnz + 2 * M * N * F + 2 * L * M * N * S, base + tiles},
            {2, SC_SCHED_FISSIONED, SC_SCHED_FISSIONED, 2 * N * nnz + 2 * M * N * F + 2 * L * M * N * S, base + tiles + trows},
            {1, SC_SCHED_FISSIONED, SC_SCHED_FISSIONED, 2 * N * nnz + 3 * L * M * N * F, base + trows},
            {3, SC_SCHED_FUSED, SC_SCHED_LINEAR, 3 * M * N * nnz + 2 * L * M * N * S, base + tiles}};
        std::vector<Candidate> cands(4);
        for (int n = 0; n < 4; ++n) {
            probe_class(&inner, opt[n].inner, sched->deterministic == 1 && opt[n].variant != 3, cands[n]);
            if (opt[n].variant == 3 && sched->deterministic == 1) cands[n].available = cands[n].admissible = false;
            cands[n].kind = opt[n].outer;
            cands[n].variant = opt[n].variant;
            cands[n].flops = opt[n].flops;
            cands[n].bytes = opt[n].bytes;
            cands[n].seconds = predicted_seconds(p, opt[n].flops, opt[n].bytes);
        }
        const size_t best = pick_candidate(cands);
        if (best == cands.size()) return SC_ERR_SCHED_UNSUPPORTED;
        describe_candidates(choice_text, cands, best);
        picked.kind = cands[best].kind;
        picked.deterministic = sched->deterministic;
        auto_variant = cands[best].variant;
        sched = &picked;
    }
    if (sched->kind != SC_SCHED_FUSED && sched->kind != SC_SCHED_FISSIONED && sched->kind != SC_SCHED_LINEAR) return SC_ERR_SCHED_UNSUPPORTED;
    p->sched = sched->kind;
    p->deterministic = sched->deterministic == 1;
    // which schedule: match the named temporaries against the derived index sets
    int variant = auto_variant ? auto_variant : 2;
    if (sched->kind == SC_SCHED_LINEAR) {   // Figure 2a: no temporary (the reduction over the grid is ordered, so the result is reproducible either way)
        if (sched->n_intermediates != 0) return SC_ERR_SCHED_UNSUPPORTED;
        variant = 0;
    }
    if (sched->n_intermediates < 0 || sched->n_intermediates > 2) return SC_ERR_SCHED_UNSUPPORTED;
    if (sched->n_intermediates) {
        bool has[2] = {false, false};
        for (int t = 0; t < sched->n_intermediates; ++t) {
            if (!sched->intermediate[t]) return SC_ERR_SCHED_UNSUPPORTED;
            Term tt;
            const char *q = sched->intermediate[t];
            if (!parse_term(q, tt)) return SC_ERR_SCHED_UNSUPPORTED;
            while (*q && isspace((unsigned char)*q)) ++q;
            if (*q) return SC_ERR_SCHED_UNSUPPORTED;
            std::set<std::string> got(tt.idx.begin(), tt.idx.end());
            if (got.size() != tt.idx.size()) return SC_ERR_SCHED_UNSUPPORTED;
            int match = -1;
            for (int u = 0; u < 2; ++u) {
                std::set<std::string> want(fam.temp_idx[u].begin(), fam.temp_idx[u].end());
                if (!has[u] && want == got) match = u;
            }
            if (match < 0) return SC_ERR_SCHED_UNSUPPORTED;
            has[match] = true;
            if (sched->fuse_depth[t] != 0) return SC_ERR_SCHED_UNSUPPORTED;   // the on-chip granularity is the library's choice here
        }
        variant = has[0] && has[1] ? 2 : has[0] ? 1 : 3;
    }
    p->k5_variant = variant;
    // schedule 1 keeps t(i,j,n) in the workspace and schedule 3 keeps its scalar per (i,m,n) in registers of the
    // unfactored inner nest: one class each
    if (variant == 1 && sched->kind != SC_SCHED_FISSIONED) return SC_ERR_SCHED_UNSUPPORTED;
    if (variant == 3 && (sched->kind != SC_SCHED_FUSED || p->deterministic)) return SC_ERR_SCHED_UNSUPPORTED;

    // inner plan: S(i,m,n) = B(i,j,k) * D(j,m) * E(k,n)
    const std::vector<std::string> &si = rhs[0].idx;
    const std::string inner_expr = "S(" + si[0] + "," + lhs.idx[1] + "," + lhs.idx[2] + ")=" + join(rhs[0].name, si) + "*D_(" + si[1] + "," +
                                   lhs.idx[1] + ")*E_(" + si[2] + "," + lhs.idx[2] + ")";
    const sc_dense_view inner_fac[2] = {factors[fam.slot_of_factor[1]], factors[fam.slot_of_factor[2]]};
    sc_schedule is = {};
    is.kind = (variant == 3 || variant == 0) ? SC_SCHED_LINEAR : variant == 1 ? SC_SCHED_FISSIONED : sched->kind;
    is.deterministic = (variant == 3 || variant == 0) ? 0 : sched->deterministic;
    sc_status st = plan_create_impl(&p->inner, inner_expr.c_str(), sparse, inner_fac, 2, &is);
    if (st != SC_OK) return st;
    const sc_plan *in = p->inner;
    p->has_device = in->has_device;
    p->tune = in->tune;
    p->n_cu = in->n_cu;
    p->lds_per_cu = in->lds_per_cu;
    p->caps = in->caps;

    const double e = (double)esize(p->dtype), nnz = (double)p->nnz;
    const double S = (double)p->nfib[0], F = (double)p->nfib[1];
    const double L = (double)p->fcols[0], M = (double)p->fcols[1], N = (double)p->fcols[2];
    // reduction over slices (fibers for schedule 1): contiguous chunks, one slot each
    const int64_t units = variant <= 1 ? p->nfib[1] : p->dims[0];
    const int64_t per = variant == 1 ? 1024 : variant == 0 ? 256 : 64;
    p->k5_nchunks = std::max<int64_t>(1, std::min<int64_t>((units + per - 1) / per, (int64_t)p->n_cu * 2));
    // In fp32 at L = 16, 32, 64, 128 the contraction over the first mode runs on the matrix cores (a workgroup takes all of L for
    // 64 columns of (m,n), so S is read once); its grid has M N / 64 workgroups per chunk of slices, and fewer chunks
    // keep the slots small when the output is large.
    const int64_t mn = p->fcols[1] * p->fcols[2];
    p->k5_mfma_reduce = variant >= 2 && p->dtype == SC_F32 && (p->fcols[0] == 16 || p->fcols[0] == 32 || p->fcols[0] == 64 || p->fcols[0] == 128) && mn % 64 == 0;
    if (p->k5_mfma_reduce) {
        const int64_t per_chunk = mn / 64, want = (int64_t)p->n_cu * 8;
        p->k5_nchunks = std::max<int64_t>(1, std::min<int64_t>(p->k5_nchunks, (want + per_chunk - 1) / per_chunk));
    }
    p->k5_chunk = std::max<int64_t>(1, (units + p->k5_nchunks - 1) / p->k5_nchunks);
    p->k5_nchunks = std::max<int64_t>(1, (units + p->k5_chunk - 1) / p->k5_chunk);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) & ~(size_t)255;
        return at;
    };
    p->k5_s_offset = variant <= 1 ? 0 : take((size_t)p->dims[0] * (size_t)(p->fcols[1] * p->fcols[2]) * esize(p->dtype));
    p->k5_inner_ws_offset = take(variant == 0 ? 0 : in->ws_bytes);
    p->k5_partials_offset = take((size_t)p->k5_nchunks * (size_t)p->out_elems * esize(p->dtype));
    p->ws_bytes = off;

    // temporaries as the caller can read them back after a FISSIONED execution: t rows (one per fiber) and
    // the per-slice tiles (one row per coordinate of the first mode, empty slices included)
    p->n_inter = variant == 2 ? 2 : variant == 0 ? 0 : 1;
    const int t2 = variant == 2 ? 1 : 0;
    if (variant == 1 || variant == 2) {
        p->inter[0].name = join(fam.temp_name[0], fam.temp_idx[0]);
        p->inter[0].rows = p->nfib[1];
        p->inter[0].cols = p->fcols[2];
        p->inter[0].offset = p->k5_inner_ws_offset + (in->sched == SC_SCHED_FISSIONED ? in->inter[0].offset : 0);
    }
    if (variant >= 2) {
        p->inter[t2].name = join(fam.temp_name[1], fam.temp_idx[1]);
        p->inter[t2].rows = p->dims[0];
        p->inter[t2].cols = p->fcols[1] * p->fcols[2];
        p->inter[t2].offset = p->k5_s_offset;
    }

    // iteration counts of the nests as Table 2 writes them (multiply = 1, add = 1)
    double flops = 0;
    if (variant == 0) flops = 4 * L * M * N * nnz;
    else if (variant == 1) flops = 2 * N * nnz + 3 * L * M * N * F;
    else if (variant == 2) flops = 2 * N * nnz + 2 * M * N * F + 2 * L * M * N * S;
    else flops = 3 * M * N * nnz + 2 * L * M * N * S;
    double fac_bytes = 0;
    for (int s = 0; s < 3; ++s) fac_bytes += (double)p->frows[s] * (double)p->fcols[s] * e;
    double bytes = nnz * (4 + e) + F * 8 + S * 8 + fac_bytes + (double)p->out_elems * e;
    if (variant == 1 || (variant == 2 && p->sched == SC_SCHED_FISSIONED)) bytes += 2 * F * N * e;   // t(i,j,n) written and read
    p->model_flops = flops;
    p->model_bytes = bytes;

    std::string &tx = p->text;
    appendf(tx, "expression: %s\n", expr);
    const char *Cn = rhs[fam.slot_of_factor[0] + 1].name.c_str(), *Dn = rhs[fam.slot_of_factor[1] + 1].name.c_str(),
               *En = rhs[fam.slot_of_factor[2] + 1].name.c_str();
    const char *i_ = si[0].c_str(), *j_ = si[1].c_str(), *k_ = si[2].c_str();
    const char *l_ = lhs.idx[0].c_str(), *m_ = lhs.idx[1].c_str(), *n_ = lhs.idx[2].c_str();
    if (variant == 0)
        appendf(tx, "schedule: LINEAR (Figure 2a: the perfectly nested loop, no temporary)\n");
    else
        appendf(tx, "schedule: Table 2, kernel 5, schedule %d (%s)\n", variant,
                p->sched == SC_SCHED_FUSED ? "FUSED: the temporaries of the sparse part stay on chip" : "FISSIONED: t in the workspace");
    tx += choice_text;
    if (variant == 0)
        appendf(tx, "nest: forall(%s,%s,%s,%s,%s',%s', A += %s * %s * %s * %s)\n", l_, m_, n_, i_, j_, k_, rhs[0].name.c_str(), Cn, Dn, En);
    else if (variant == 1)
        appendf(tx, "nest: forall(%s,%s',%s, where(forall(%s,%s, A += t * %s * %s), forall(%s', t += %s * %s)))\n", i_, j_, n_, m_, l_, Cn, Dn, k_,
                rhs[0].name.c_str(), En);
    else if (variant == 2)
        appendf(tx, "nest: forall(%s,%s, where(forall(%s,%s, A += T(%s) * %s), forall(%s', where(forall(%s, T(%s) += t * %s), forall(%s', t += %s * %s)))))\n",
                i_, n_, m_, l_, m_, Cn, j_, m_, m_, Dn, k_, rhs[0].name.c_str(), En);
    else
        appendf(tx, "nest: forall(%s,%s,%s, where(forall(%s, A += t * %s), forall(%s',%s', t += %s * %s * %s)))\n", i_, m_, n_, l_, Cn, j_, k_,
                rhs[0].name.c_str(), Dn, En);
    if (variant == 0)
        appendf(tx, "the output has no sparse index: %lld workgroups sum contiguous chunks of fibers, their partial tiles are added in chunk order\n",
                (long long)p->k5_nchunks);
    else if (variant == 1)
        appendf(tx, "the output has no sparse index: the rows t(%s,%s,:) pass through the workspace once and are reduced over all fibers by %lld workgroups, "
                    "whose partial tiles are added in chunk order (always reproducible)\n", i_, j_, (long long)p->k5_nchunks);
    else
        appendf(tx, "the output has no sparse index: per-slice tiles S(%s,%s,%s) pass through the workspace once and are reduced over %s by %lld workgroups, "
                    "whose partial tiles are added in chunk order (always reproducible)\n", i_, m_, n_, i_, (long long)p->k5_nchunks);
    for (int t = 0; t < p->n_inter; ++t)
        appendf(tx, "temporary %d: %s, %lld x %lld\n", t, p->inter[t].name.c_str(), (long long)p->inter[t].rows, (long long)p->inter[t].cols);
    appendf(tx, "structure: nnz=%lld nodes[0]=%lld nodes[1]=%lld\n", (long long)p->nnz, (long long)p->nfib[0], (long long)p->nfib[1]);
    appendf(tx, "model: %.6g flops, %.6g compulsory HBM bytes, workspace %zu bytes\n", flops, bytes, p->ws_bytes);
    appendf(tx, "inner plan:\n%s", in->text.c_str());
    return SC_OK;
}

// Kernels 8 <MTTKRP,GEMM> and 2 <SDDMM,SpMM,GEMM> of Table 2: a two-level nest whose inner level is an expression the
// library already runs (the MTTKRP, or kernel 1) and whose outer level multiplies the row it leaves per slice with the
// last factor.  The sparse part is planned as an inner plan under the caller's schedule class (AUTO included); its
// rows pass through the workspace once and the dense product runs on the matrix cores.
static sc_status plan_trailing_gemm(sc_plan *p, const char *expr, const Term &lhs, const std::vector<Term> &rhs, const Family &fam,
                                    const sc_csf_view *sparse, const sc_dense_view *factors, const sc_schedule *sched)
{
    if (sched->deterministic != 0 && sched->deterministic != 1) return SC_ERR_SCHED_UNSUPPORTED;
    const int nin = p->nfactors - 1;   // factors of the sparse part
    const std::vector<std::string> &si = rhs[0].idx;
    const std::string &r = fam.temp_idx[1][1];   // index contracted by the dense product
    // named temporaries: the sparse part's own one and / or the row temporary; anything else is refused
    if (sched->n_intermediates < 0 || sched->n_intermediates > 2) return SC_ERR_SCHED_UNSUPPORTED;
    bool has[2] = {false, false};
    for (int t = 0; t < sched->n_intermediates; ++t) {
        if (!sched->intermediate[t]) return SC_ERR_SCHED_UNSUPPORTED;
        Term tt;
        const char *q = sched->intermediate[t];
        if (!parse_term(q, tt)) return SC_ERR_SCHED_UNSUPPORTED;
        while (*q && isspace((unsigned char)*q)) ++q;
        if (*q) return SC_ERR_SCHED_UNSUPPORTED;
        std::set<std::string> got(tt.idx.begin(), tt.idx.end());
        if (got.size() != tt.idx.size()) return SC_ERR_SCHED_UNSUPPORTED;
        int match = -1;
        for (int u = 0; u < 2; ++u) {
            std::set<std::string> want(fam.temp_idx[u].begin(), fam.temp_idx[u].end());
            if (!has[u] && want == got) match = u;
        }
        if (match < 0 || sched->fuse_depth[t] != 0) return SC_ERR_SCHED_UNSUPPORTED;
        has[match] = true;
    }
    std::string inner_expr = "P(" + si[0] + "," + r + ")=" + join(rhs[0].name, si);
    sc_dense_view inner_fac[3];
    for (int s = 0; s < nin; ++s) {
        const Term &t = rhs[fam.slot_of_factor[s] + 1];
        inner_expr += "*F" + std::to_string(s) + "_(" + t.idx[0] + "," + t.idx[1] + ")";
        inner_fac[s] = factors[fam.slot_of_factor[s]];
    }
    sc_schedule is = {};
    is.kind = sched->kind;
    is.deterministic = sched->deterministic;
    sc_status st = plan_create_impl(&p->inner, inner_expr.c_str(), sparse, inner_fac, nin, &is);
    if (st != SC_OK) return st;
    const sc_plan *in = p->inner;
    p->sched = in->sched;
    p->deterministic = in->deterministic;
    p->has_device = in->has_device;
    p->tune = in->tune;
    p->n_cu = in->n_cu;
    p->lds_per_cu = in->lds_per_cu;
    p->caps = in->caps;

    const int64_t R = p->fcols[nin - 1], M = p->fcols[nin];
    const double e = (double)esize(p->dtype);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) & ~(size_t)255;
        return at;
    };
    p->tg_rows_offset = take((size_t)p->dims[0] * (size_t)R * esize(p->dtype));
    p->tg_inner_ws_offset = take(in->ws_bytes);
    p->ws_bytes = off;
    p->n_inter = in->sched == SC_SCHED_LINEAR ? 1 : 2;
    int t2 = 0;
    if (p->n_inter == 2) {
        p->inter[0].name = join(fam.temp_name[0], fam.temp_idx[0]);
        p->inter[0].rows = in->inter[0].rows;
        p->inter[0].cols = in->inter[0].cols;
        p->inter[0].offset = p->tg_inner_ws_offset + in->inter[0].offset;
        t2 = 1;
    }
    p->inter[t2].name = join(fam.temp_name[1], fam.temp_idx[1]);
    p->inter[t2].rows = p->dims[0];
    p->inter[t2].cols = R;
    p->inter[t2].offset = p->tg_rows_offset;

    // the sparse part's iteration count, then one multiply-add per (non-empty slice, r, m); bytes: every input and
    // the output once (the rows in between are the price of the split, not counted)
    p->model_flops = in->model_flops + 2.0 * (double)R * (double)M * (double)p->nfib[0];
    p->model_bytes = in->model_bytes - (double)in->out_elems * e + (double)p->frows[nin] * (double)M * e + (double)p->out_elems * e;

    std::string &tx = p->text;
    appendf(tx, "expression: %s\n", expr);
    appendf(tx, "schedule: Table 2, kernel %d: the rows %s of the sparse part (%s) pass through the workspace and are multiplied with %s on the matrix cores "
                "(fp32, %s in {16, 32, 64, 128} and %s a multiple of 16; the vector ALUs otherwise)\n",
            p->kind == K_MTTKRP_GEMM ? 8 : 2, p->inter[t2].name.c_str(), sched_name(in->sched), rhs[fam.slot_of_factor[nin] + 1].name.c_str(),
            r.c_str(), lhs.idx[1].c_str());
    appendf(tx, "nest: forall(%s, where(forall(%s,%s, %s += %s * %s), <sparse part>))\n", si[0].c_str(), lhs.idx[1].c_str(), r.c_str(),
            join(lhs.name, lhs.idx).c_str(), p->inter[t2].name.c_str(), rhs[fam.slot_of_factor[nin] + 1].name.c_str());
    for (int t = 0; t < p->n_inter; ++t)
        appendf(tx, "temporary %d: %s, %lld x %lld\n", t, p->inter[t].name.c_str(), (long long)p->inter[t].rows, (long long)p->inter[t].cols);
    appendf(tx, "model: %.6g flops, %.6g compulsory HBM bytes, workspace %zu bytes\n", p->model_flops, p->model_bytes, p->ws_bytes);
    appendf(tx, "inner plan:\n%s", in->text.c_str());
    return SC_OK;
}

static sc_status plan_create_impl(sc_plan **out, const char *expr, const sc_csf_view *sparse,
                                  const sc_dense_view *factors, int32_t nfactors, const sc_schedule *sched)
{
    if (!out) return SC_ERR_NULL;
    *out = nullptr;
    if (!expr || !sparse || !factors || !sched) return SC_ERR_NULL;

    Term lhs;
    std::vector<Term> rhs;
    if (!parse_expr(expr, lhs, rhs)) return SC_ERR_EXPR_PARSE;
    Family fam;
    sc_status st = classify(lhs, rhs, fam);
    if (st != SC_OK) return st;
    if ((int)rhs[0].idx.size() != sparse->order) return SC_ERR_BAD_ORDER;
    if (nfactors != (int32_t)rhs.size() - 1) return SC_ERR_SHAPE_MISMATCH;

    st = check_header(sparse->order, sparse->dims, sparse->nnz, sparse->dtype);
    if (st != SC_OK) return st;
    st = check_node_counts(sparse);   // before any array is sized from them
    if (st != SC_OK) return st;
    HostCsf h;
    st = fetch_csf(sparse, h, /*want_crd=*/true);
    if (st != SC_OK) return st;
    st = validate_csf(sparse, h);
    if (st != SC_OK) return st;

    sc_plan *p = new (std::nothrow) sc_plan();
    if (!p) return SC_ERR_ALLOC;
    struct Guard {
        sc_plan *p;
        ~Guard() { if (p) sc_plan_destroy(p); }
    } guard{p};

    p->kind = fam.kind;
    p->dtype = sparse->dtype;
    p->order = sparse->order;
    p->nnz = sparse->nnz;
    for (int m = 0; m < 4; ++m) { p->dims[m] = sparse->dims[m]; p->nfib[m] = sparse->nfib[m]; }
    p->nfactors = nfactors;
    for (int s = 0; s < nfactors; ++s) {
        p->slot_of_factor[s] = fam.slot_of_factor[s];
        const sc_dense_view &f = factors[fam.slot_of_factor[s]];
        if (f.dtype != p->dtype) return dtype_ok(f.dtype) ? SC_ERR_BAD_DTYPE : SC_ERR_BAD_DTYPE;
        if (f.rows <= 0 || f.cols <= 0 || f.cols > 4096) return SC_ERR_SHAPE_MISMATCH;
        // rows are addressed with byte offsets of 31 bits (the walks use bit 31 as the end-of-node mark)
        if ((uint64_t)f.rows * (uint64_t)f.cols * esize(p->dtype) >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
        p->frows[s] = f.rows;
        p->fcols[s] = f.cols;
    }
    // factor rows must equal the sparse dimension they index
    switch (p->kind) {
    case K_TTMC3:
        if (p->frows[0] != p->dims[1] || p->frows[1] != p->dims[2]) return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[0] * p->fcols[1];
        break;
    case K_MTTKRP3:
        if (p->frows[0] != p->dims[1] || p->frows[1] != p->dims[2] || p->fcols[0] != p->fcols[1]) return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[0];
        break;
    case K_SDDMM_SPMM:
        if (p->frows[0] != p->dims[0] || p->frows[1] != p->dims[1] || p->frows[2] != p->dims[1] || p->fcols[0] != p->fcols[1])
            return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[2];
        break;
    case K_TTMC4:
        if (p->frows[0] != p->dims[1] || p->frows[1] != p->dims[2] || p->frows[2] != p->dims[3]) return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[0] * p->fcols[1] * p->fcols[2];
        break;
    case K_TTMC_ALL:
        if (p->frows[0] != p->dims[0] || p->frows[1] != p->dims[1] || p->frows[2] != p->dims[2]) return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[0] * p->fcols[1] * p->fcols[2];
        break;
    case K_MTTKRP_GEMM:
        if (p->frows[0] != p->dims[1] || p->frows[1] != p->dims[2] || p->fcols[0] != p->fcols[1] || p->frows[2] != p->fcols[0])
            return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[2];
        break;
    case K_SDDMM_SPMM_GEMM:
        if (p->frows[0] != p->dims[0] || p->frows[1] != p->dims[1] || p->frows[2] != p->dims[1] || p->fcols[0] != p->fcols[1] ||
            p->frows[3] != p->fcols[2])
            return SC_ERR_SHAPE_MISMATCH;
        p->out_row_elems = p->fcols[3];
        break;
    }
    p->tune = tuning();   // read once; executions use the plan's copy
    {
        int ndev0 = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDeviceCount(&ndev0) == hipSuccess && ndev0 > 0 && hipGetDevice(&dev) == hipSuccess &&
            hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            if (prop.multiProcessorCount > 0) p->n_cu = prop.multiProcessorCount;
            if (prop.maxSharedMemoryPerMultiProcessor >= 64 * 1024) p->lds_per_cu = (int64_t)prop.maxSharedMemoryPerMultiProcessor;
        } else {
            (void)hipGetLastError();
        }
    }
    p->out_elems = p->kind == K_TTMC_ALL ? p->out_row_elems : p->dims[0] * p->out_row_elems;
    if (p->kind == K_TTMC_ALL || p->kind == K_MTTKRP_GEMM || p->kind == K_SDDMM_SPMM_GEMM) {
        st = p->kind == K_TTMC_ALL ? plan_ttmc_all(p, expr, lhs, rhs, fam, sparse, factors, sched)
                                   : plan_trailing_gemm(p, expr, lhs, rhs, fam, sparse, factors, sched);
        if (st != SC_OK) return st;
        guard.p = nullptr;
        *out = p;
        return SC_OK;
    }

    // ---- schedule ----
    if (sched->deterministic != 0 && sched->deterministic != 1) return SC_ERR_SCHED_UNSUPPORTED;
    sc_schedule picked = {};
    std::string choice_text;
    if (sched->kind == SC_SCHED_AUTO) {
        if (sched->n_intermediates != 0) return SC_ERR_SCHED_UNSUPPORTED;   // AUTO derives the temporaries itself
        std::vector<Candidate> cands(3);
        const sc_sched_kind classes[3] = {SC_SCHED_FUSED, SC_SCHED_FISSIONED, SC_SCHED_LINEAR};
        for (int n = 0; n < 3; ++n) {
            probe_class(p, classes[n], sched->deterministic == 1, cands[n]);
            schedule_model(p, classes[n], &cands[n].flops, &cands[n].bytes);
            cands[n].seconds = predicted_seconds(p, cands[n].flops, cands[n].bytes);
        }
        const size_t best = pick_candidate(cands);
        if (best == cands.size()) return SC_ERR_SCHED_UNSUPPORTED;
        describe_candidates(choice_text, cands, best);
        picked.kind = cands[best].kind;
        picked.deterministic = sched->deterministic;
        sched = &picked;
    }
    if (sched->kind != SC_SCHED_LINEAR && sched->kind != SC_SCHED_FUSED && sched->kind != SC_SCHED_FISSIONED) return SC_ERR_SCHED_UNSUPPORTED;
    p->deterministic = sched->deterministic == 1;
    p->sched = sched->kind;
    const bool linear = sched->kind == SC_SCHED_LINEAR;
    // LINEAR: the unfactored nest has no temporary, and its row sums are combined with atomics only
    if (linear && (sched->n_intermediates != 0 || p->deterministic)) return SC_ERR_SCHED_UNSUPPORTED;
    p->n_inter = linear ? 0 : (int32_t)fam.temp_idx.size();
    if (sched->n_intermediates != 0 && sched->n_intermediates != p->n_inter) return SC_ERR_SCHED_UNSUPPORTED;
    for (int t = 0; t < p->n_inter; ++t) {
        p->inter[t].name = join(fam.temp_name[t], fam.temp_idx[t]);
        const int fd = sched->n_intermediates ? sched->fuse_depth[t] : 0;
        if (sched->kind == SC_SCHED_FISSIONED && fd != 0) return SC_ERR_SCHED_UNSUPPORTED;
        // the depth the FUSED kernel of this expression is built at (0 = that depth); nothing else is offered
        const int built = (p->kind == K_MTTKRP3 || p->kind == K_SDDMM_SPMM) ? 2 : 1;
        if (sched->kind == SC_SCHED_FUSED && fd != 0 && fd != built) return SC_ERR_SCHED_UNSUPPORTED;
        p->fuse_depth[t] = fd;
    }
    if (sched->n_intermediates) {
        // each named temporary must match one of the derived index sets, each derived set at most once
        bool used[2] = {false, false};
        for (int t = 0; t < sched->n_intermediates; ++t) {
            if (!sched->intermediate[t]) continue;
            Term tt;
            const char *q = sched->intermediate[t];
            if (!parse_term(q, tt)) return SC_ERR_SCHED_UNSUPPORTED;
            while (*q && isspace((unsigned char)*q)) ++q;
            if (*q) return SC_ERR_SCHED_UNSUPPORTED;
            std::set<std::string> got(tt.idx.begin(), tt.idx.end());
            if (got.size() != tt.idx.size()) return SC_ERR_SCHED_UNSUPPORTED;
            int match = -1;
            for (int u = 0; u < p->n_inter; ++u) {
                std::set<std::string> want(fam.temp_idx[u].begin(), fam.temp_idx[u].end());
                if (!used[u] && want == got) { match = u; break; }
            }
            if (match < 0) return SC_ERR_SCHED_UNSUPPORTED;
            used[match] = true;
        }
    }

    // ---- tiles ----
    p->caps = linear ? TileCaps{1024, 1024, 1024}   // node caps that never bind: the kernel keeps no per-node state
                     : default_caps(p->kind, p->dtype, p->sched, p->fcols);
    if (p->caps.tn <= 0) return SC_ERR_SCHED_UNSUPPORTED;  // no kernel instantiated for these ranks
    const Tuning &tu = p->tune;
    if (tu.tn) p->caps.tn = tu.tn;
    if (tu.ta) p->caps.ta = tu.ta;
    if (tu.tb) p->caps.tb = tu.tb;
    if (lds_bytes_needed(p) > 64 * 1024) return SC_ERR_SCHED_UNSUPPORTED;
    try {
        build_tiles(sparse, h, p->caps, p->tiles);
        if (p->deterministic) {
            if (!plan_supports_deterministic(p)) return SC_ERR_SCHED_UNSUPPORTED;
            assign_piece_slots(p, h);
        }
        list_rows_to_zero(p, h);
    } catch (const std::bad_alloc &) { return SC_ERR_ALLOC; }

    // ---- workspace, model, text ----
    const int d = p->order;
    double flops = 0, bytes = 0;
    schedule_model(p, p->sched, &flops, &bytes);
    size_t off = 0;
    auto place = [&](int t, int64_t rows, int64_t cols) {
        p->inter[t].rows = rows;
        p->inter[t].cols = cols;
        p->inter[t].offset = off;
        off += ((size_t)rows * (size_t)cols * esize(p->dtype) + 255) & ~(size_t)255;
    };
    switch (p->kind) {
    case K_TTMC3: place(0, p->nfib[1], p->fcols[1]); break;
    case K_MTTKRP3: place(0, p->nfib[1], p->fcols[0]); break;
    case K_SDDMM_SPMM: place(0, p->nnz, 1); break;
    case K_TTMC4:
        place(0, p->nfib[2], p->fcols[2]);
        place(1, p->nfib[1], p->fcols[1] * p->fcols[2]);
        break;
    case K_TTMC_ALL:
    case K_MTTKRP_GEMM:
    case K_SDDMM_SPMM_GEMM: break;   // planned by plan_ttmc_all / plan_trailing_gemm
    }
    if (p->sched == SC_SCHED_FISSIONED) {
        p->ws_bytes = off;
    } else {
        p->ws_bytes = 0;
        for (int t = 0; t < p->n_inter; ++t) p->inter[t].offset = 0;
    }
    if (p->deterministic) {
        for (FixLevel *lv : {&p->det_top, &p->det_a, &p->det_b}) {
            if (!lv->n_slots) continue;
            const size_t row_bytes = (size_t)lv->rowlen * esize(p->dtype);
            lv->slot_offset = (p->ws_bytes + 255) & ~(size_t)255;
            lv->seg_offset = (lv->slot_offset + (size_t)lv->n_slots * row_bytes + 255) & ~(size_t)255;
            p->ws_bytes = lv->seg_offset + lv->segs.size() * row_bytes;
        }
    }
    p->model_flops = flops;
    p->model_bytes = bytes;

    std::string &tx = p->text;
    appendf(tx, "expression: %s\n", expr);
    appendf(tx, "schedule: %s\n", linear ? "LINEAR (the unfactored nest, no temporary)"
                                  : p->sched == SC_SCHED_FUSED ? "FUSED (temporaries on chip)" : "FISSIONED (temporaries in the workspace)");
    tx += choice_text;
    const std::vector<std::string> &si = rhs[0].idx;
    if (linear)
        appendf(tx, "nest: forall(entries of %s, forall(dense indices, %s += product of one element of every operand))\n", rhs[0].name.c_str(),
                join(lhs.name, lhs.idx).c_str());
    else switch (p->kind) {
    case K_TTMC3:
    case K_MTTKRP3: {
        const std::string x = fam.temp_idx[0][2];
        const std::string l = lhs.idx[1];
        if (p->sched == SC_SCHED_FUSED)
            appendf(tx, "nest: forall(tile of %s,%s', where(forall(%s', forall(%s, %s += T(%s',%s) * %s)), forall(%s',%s', forall(%s, T(%s',%s) += %s * %s))))\n",
                    si[0].c_str(), si[1].c_str(), si[1].c_str(), l.c_str(), join(lhs.name, lhs.idx).c_str(), si[1].c_str(), x.c_str(),
                    rhs[p->slot_of_factor[0] + 1].name.c_str(), si[1].c_str(), si[2].c_str(), x.c_str(), si[1].c_str(), x.c_str(),
                    rhs[0].name.c_str(), rhs[p->slot_of_factor[1] + 1].name.c_str());
        else
            appendf(tx, "nest: where(forall(%s,%s', forall(%s.., %s += %s * %s)), forall(%s,%s',%s', forall(%s, %s += %s * %s)))\n",
                    si[0].c_str(), si[1].c_str(), l.c_str(), join(lhs.name, lhs.idx).c_str(), p->inter[0].name.c_str(),
                    rhs[p->slot_of_factor[0] + 1].name.c_str(), si[0].c_str(), si[1].c_str(), si[2].c_str(), x.c_str(),
                    p->inter[0].name.c_str(), rhs[0].name.c_str(), rhs[p->slot_of_factor[1] + 1].name.c_str());
        break;
    }
    case K_SDDMM_SPMM:
        appendf(tx, "nest: forall(%s, forall(%s', where(forall(l, A += t * Z), forall(k, t += S * X * Y))))%s\n", si[0].c_str(), si[1].c_str(),
                p->sched == SC_SCHED_FUSED ? " with scalar t in registers" : " split into SDDMM and SpMM over the sampled values");
        break;
    case K_TTMC4:
        appendf(tx, "nest: two-level where: %s from leaves, %s from %s, output from %s (%s)\n", p->inter[0].name.c_str(),
                p->inter[1].name.c_str(), p->inter[0].name.c_str(), p->inter[1].name.c_str(),
                p->sched == SC_SCHED_FUSED ? "both per tile in LDS" : "both in the workspace");
        break;
    case K_TTMC_ALL:
    case K_MTTKRP_GEMM:
    case K_SDDMM_SPMM_GEMM: break;
    }
    for (int t = 0; t < p->n_inter; ++t)
        appendf(tx, "temporary %d: %s, %lld x %lld, position-compressed along the sparse prefix%s\n", t, p->inter[t].name.c_str(),
                (long long)p->inter[t].rows, (long long)p->inter[t].cols,
                p->sched == SC_SCHED_FUSED ? ", live per tile only" : "");
    appendf(tx, "structure: nnz=%lld", (long long)p->nnz);
    for (int m = 0; m < d - 1; ++m) appendf(tx, " nodes[%d]=%lld", m, (long long)p->nfib[m]);
    appendf(tx, "\ntiles: %zu (<= %d leaves, <= %d level-a nodes", p->tiles.size(), p->caps.tn, p->caps.ta);
    if (d == 4) appendf(tx, ", <= %d level-b nodes", p->caps.tb);
    appendf(tx, ")\nmodel: %.6g flops, %.6g compulsory HBM bytes, workspace %zu bytes\n", flops, bytes, p->ws_bytes);
    if (p->deterministic) {
        appendf(tx, "deterministic: %zu output rows span several tiles; their %lld pieces are stored in the workspace and added in tile order (%zu segments of at most %d)\n",
                p->det_top.fix.size(), (long long)p->det_top.n_slots, p->det_top.segs.size(), kFixSegment);
        if (p->det_a.n_slots)
            appendf(tx, "deterministic: %zu rows of %s span several tiles; %lld pieces (%zu segments)\n", p->det_a.fix.size(),
                    p->inter[0].name.c_str(), (long long)p->det_a.n_slots, p->det_a.segs.size());
        if (p->det_b.n_slots)
            appendf(tx, "deterministic: %zu rows of %s span several tiles; %lld pieces (%zu segments)\n", p->det_b.fix.size(),
                    p->inter[1].name.c_str(), (long long)p->det_b.n_slots, p->det_b.segs.size());
    }

    // ---- device tables ----
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0) {
        if (!p->tiles.empty()) {
            if (hipMalloc((void **)&p->d_tiles, sizeof(TileRec) * p->tiles.size()) != hipSuccess) return SC_ERR_DEVICE;
            // Upload in an interleaved order: workgroups that run at the same time then work on
            // tiles far apart in the tensor, so the atomic updates of one heavy output row are
            // spread over the kernel's duration instead of queueing on one address.
            const size_t nt = p->tiles.size();
            const size_t stride =
                plan_wants_tensor_order(p) ? 1 : (size_t)std::max<int32_t>(1, p->tune.interleave ? p->tune.interleave : 64);
            std::vector<TileRec> order;
            try {
                order.reserve(nt);
            } catch (const std::bad_alloc &) { return SC_ERR_ALLOC; }
            for (size_t r = 0; r < stride; ++r)
                for (size_t t = r; t < nt; t += stride) order.push_back(p->tiles[t]);
            if (hipMemcpy(p->d_tiles, order.data(), sizeof(TileRec) * nt, hipMemcpyHostToDevice) != hipSuccess)
                return SC_ERR_DEVICE;
            if (p->deterministic && p->slot_b.size() == nt) {   // same order as the tile table
                std::vector<int32_t> sb;
                try {
                    sb.reserve(nt);
                } catch (const std::bad_alloc &) { return SC_ERR_ALLOC; }
                for (size_t r = 0; r < stride; ++r)
                    for (size_t t = r; t < nt; t += stride) sb.push_back(p->slot_b[t]);
                if (hipMalloc((void **)&p->d_slot_b, sizeof(int32_t) * nt) != hipSuccess) return SC_ERR_DEVICE;
                if (hipMemcpy(p->d_slot_b, sb.data(), sizeof(int32_t) * nt, hipMemcpyHostToDevice) != hipSuccess) return SC_ERR_DEVICE;
            }
            p->walk.shape = plan_walk_shape(p);
            const sc_status ws = build_walk_tables(p, sparse, h, order);
            if (ws != SC_OK) return ws;
        }
        if (p->zero_selective && !p->zero_rows.empty()) {
            if (hipMalloc((void **)&p->d_zero_rows, sizeof(int32_t) * p->zero_rows.size()) != hipSuccess) return SC_ERR_DEVICE;
            if (hipMemcpy(p->d_zero_rows, p->zero_rows.data(), sizeof(int32_t) * p->zero_rows.size(), hipMemcpyHostToDevice) != hipSuccess)
                return SC_ERR_DEVICE;
        }
        for (FixLevel *lv : {&p->det_top, &p->det_a, &p->det_b}) {
            if (lv->fix.empty()) continue;
            if (hipMalloc((void **)&lv->d_fix, sizeof(FixRec) * lv->fix.size()) != hipSuccess) return SC_ERR_DEVICE;
            if (hipMemcpy(lv->d_fix, lv->fix.data(), sizeof(FixRec) * lv->fix.size(), hipMemcpyHostToDevice) != hipSuccess)
                return SC_ERR_DEVICE;
            if (hipMalloc((void **)&lv->d_segs, sizeof(FixRec) * lv->segs.size()) != hipSuccess) return SC_ERR_DEVICE;
            if (hipMemcpy(lv->d_segs, lv->segs.data(), sizeof(FixRec) * lv->segs.size(), hipMemcpyHostToDevice) != hipSuccess)
                return SC_ERR_DEVICE;
        }
        p->has_device = true;
        // set-up step of sc_execute_static: look the fixed scratch array up on this device now, so that the
        // entry point itself has nothing left to resolve (a failure here only matters to that entry point)
        sc_status ignored = SC_OK;
        (void)static_scratch(&ignored);
    } else {
        (void)hipGetLastError();
    }
    guard.p = nullptr;
    *out = p;
    return SC_OK;
}

extern "C" sc_status sc_plan_create(sc_plan **out, const char *expr, const sc_csf_view *sparse,
                                    const sc_dense_view *factors, int32_t nfactors, const sc_schedule *sched)
{
    return guarded([&] { return plan_create_impl(out, expr, sparse, factors, nfactors, sched); });
}

extern "C" sc_status sc_plan_workspace_bytes(const sc_plan *plan, size_t *bytes)
{
    if (!plan || !bytes) return SC_ERR_NULL;
    *bytes = plan->ws_bytes;
    return SC_OK;
}

extern "C" sc_status sc_plan_describe(const sc_plan *plan, char *buf, size_t n)
{
    if (!plan || !buf) return SC_ERR_NULL;
    if (n == 0) return SC_ERR_BAD_DIMS;
    const size_t k = std::min(n - 1, plan->text.size());
    memcpy(buf, plan->text.data(), k);
    buf[k] = '\0';
    return SC_OK;
}

extern "C" sc_status sc_plan_chosen(const sc_plan *plan, sc_sched_kind *kind, int32_t *table2_schedule)
{
    if (!plan) return SC_ERR_NULL;
    if (kind) *kind = plan->sched;
    if (table2_schedule) *table2_schedule = plan->kind == sck::K_TTMC_ALL ? plan->k5_variant : 0;
    return SC_OK;
}

extern "C" sc_status sc_plan_model(const sc_plan *plan, double *flops, double *bytes)
{
    if (!plan) return SC_ERR_NULL;
    if (flops) *flops = plan->model_flops;
    if (bytes) *bytes = plan->model_bytes;
    return SC_OK;
}

extern "C" sc_status sc_plan_intermediate(const sc_plan *plan, int32_t index, size_t *offset_bytes, int64_t *rows, int64_t *cols)
{
    if (!plan) return SC_ERR_NULL;
    if (plan->kind == sck::K_TTMC_ALL) {
        // the per-slice tiles always pass through the workspace; t(i,j,n) only when the sparse part is FISSIONED
        if (index < 0 || index >= plan->n_inter) return SC_ERR_BAD_DIMS;
        const bool is_t = plan->k5_variant != 3 && index == 0;
        if (is_t && plan->inner->sched != SC_SCHED_FISSIONED) return SC_ERR_SCHED_UNSUPPORTED;
    } else if (plan->kind == sck::K_MTTKRP_GEMM || plan->kind == sck::K_SDDMM_SPMM_GEMM) {
        // the rows of the sparse part always pass through the workspace; its own temporary only when it runs FISSIONED
        if (index < 0 || index >= plan->n_inter) return SC_ERR_BAD_DIMS;
        if (index < plan->n_inter - 1 && plan->inner->sched != SC_SCHED_FISSIONED) return SC_ERR_SCHED_UNSUPPORTED;
    } else if (plan->sched != SC_SCHED_FISSIONED) return SC_ERR_SCHED_UNSUPPORTED;
    if (index < 0 || index >= plan->n_inter) return SC_ERR_BAD_DIMS;
    if (offset_bytes) *offset_bytes = plan->inter[index].offset;
    if (rows) *rows = plan->inter[index].rows;
    if (cols) *cols = plan->inter[index].cols;
    return SC_OK;
}

extern "C" sc_status sc_plan_tile_count(const sc_plan *plan, int64_t *count)
{
    if (!plan || !count) return SC_ERR_NULL;
    if (plan->inner) plan = plan->inner;
    *count = (int64_t)plan->tiles.size();
    return SC_OK;
}

extern "C" sc_status sc_plan_tile(const sc_plan *plan, int64_t index, int32_t rec[9])
{
    if (!plan || !rec) return SC_ERR_NULL;
    if (plan->inner) plan = plan->inner;
    if (index < 0 || index >= (int64_t)plan->tiles.size()) return SC_ERR_BAD_DIMS;
    memcpy(rec, &plan->tiles[(size_t)index], 9 * sizeof(int32_t));
    return SC_OK;
}

// Argument checks and launches shared by every execute entry point.
sc_status sck::execute_checked(const sc_plan *plan, const sc_csf_view *sparse, const sc_dense_view *factors, int32_t nfactors,
                               void *out, void *workspace, size_t workspace_bytes, hipStream_t hip_stream)
{
    if (!plan || !sparse || !factors || !out) return SC_ERR_NULL;
    if (!plan->has_device) return SC_ERR_DEVICE;
    if (!sparse->on_device) return SC_ERR_DEVICE;
    if (nfactors != plan->nfactors) return SC_ERR_SHAPE_MISMATCH;
    if (sparse->order != plan->order) return SC_ERR_BAD_ORDER;
    if (sparse->dtype != plan->dtype) return SC_ERR_BAD_DTYPE;
    if (sparse->nnz != plan->nnz) return SC_ERR_SHAPE_MISMATCH;
    for (int m = 0; m < plan->order; ++m) {
        if (sparse->dims[m] != plan->dims[m] || sparse->nfib[m] != plan->nfib[m]) return SC_ERR_SHAPE_MISMATCH;
        if (plan->nnz > 0 && (!sparse->crd[m] || (m && !sparse->pos[m]))) return SC_ERR_NULL;
    }
    if (plan->nnz > 0 && !sparse->vals) return SC_ERR_NULL;
    if ((uintptr_t)out % 16) return SC_ERR_SHAPE_MISMATCH;
    sc_dense_view canon[4];
    for (int s = 0; s < plan->nfactors; ++s) {
        const sc_dense_view &f = factors[plan->slot_of_factor[s]];
        if (!f.data) return SC_ERR_NULL;
        if (f.dtype != plan->dtype) return SC_ERR_BAD_DTYPE;
        if (f.rows != plan->frows[s] || f.cols != plan->fcols[s] || f.ld < f.cols) return SC_ERR_SHAPE_MISMATCH;
        // rows are read with 16-byte vector loads
        if ((uintptr_t)f.data % 16 || (f.ld * (int64_t)esize(f.dtype)) % 16) return SC_ERR_SHAPE_MISMATCH;
        // ... and addressed with 31-bit byte offsets: checked here, before anything is launched
        if ((uint64_t)f.rows * (uint64_t)f.ld * esize(f.dtype) >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
        canon[s] = f;
    }
    if (workspace_bytes < plan->ws_bytes) return SC_ERR_WORKSPACE_SMALL;
    if (plan->ws_bytes && (!workspace || (uintptr_t)workspace % 256)) return plan->ws_bytes && !workspace ? SC_ERR_NULL : SC_ERR_SHAPE_MISMATCH;
    return launch_plan(plan, sparse, canon, out, workspace, hip_stream);
}

extern "C" sc_status sc_execute(const sc_plan *plan, const sc_csf_view *sparse, const sc_dense_view *factors, int32_t nfactors,
                                void *out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return guarded([&] { return execute_checked(plan, sparse, factors, nfactors, out, workspace, workspace_bytes, (hipStream_t)hip_stream); });
}

extern "C" sc_status sc_plan_set_profiling(sc_plan *plan, int32_t on)
{
    if (!plan) return SC_ERR_NULL;
    if (on && !plan->prof) {
        if (!plan->has_device) return SC_ERR_DEVICE;
        ProfileState *pr = new (std::nothrow) ProfileState();
        if (!pr) return SC_ERR_ALLOC;
        int made = 0;
        bool ok = true;
        for (; made < kMaxLaunches && ok; ++made) {
            ok = hipEventCreate(&pr->ev_begin[made]) == hipSuccess;
            if (ok && hipEventCreate(&pr->ev_end[made]) != hipSuccess) {
                (void)hipEventDestroy(pr->ev_begin[made]);
                ok = false;
            }
            if (!ok) break;
        }
        if (!ok) {
            for (int i = 0; i < made; ++i) {
                (void)hipEventDestroy(pr->ev_begin[i]);
                (void)hipEventDestroy(pr->ev_end[i]);
            }
            delete pr;
            return SC_ERR_DEVICE;
        }
        plan->prof = pr;
    }
    if (plan->prof) {
        plan->prof->on = on != 0;
        plan->prof->n_launch = 0;
    }
    if (plan->inner) plan->inner->prof = plan->prof;   // the inner plan's launches are timed into the same record
    return SC_OK;
}

extern "C" sc_status sc_plan_kernel_count(const sc_plan *plan, int32_t *count)
{
    if (!plan || !count) return SC_ERR_NULL;
    *count = plan->prof ? plan->prof->n_launch : 0;
    return SC_OK;
}

extern "C" sc_status sc_plan_kernel_time(const sc_plan *plan, int32_t index, char *name, size_t name_len, float *ms)
{
    if (!plan || !ms) return SC_ERR_NULL;
    if (!plan->prof || !plan->prof->on) return SC_ERR_SCHED_UNSUPPORTED;
    const ProfileState &pr = *plan->prof;
    if (index < 0 || index >= pr.n_launch) return SC_ERR_BAD_DIMS;
    if (hipEventElapsedTime(ms, pr.ev_begin[index], pr.ev_end[index]) != hipSuccess) return SC_ERR_DEVICE;
    if (name && name_len) {
        snprintf(name, name_len, "%s", pr.launch_name[index]);
    }
    return SC_OK;
}

extern "C" sc_status sc_plan_destroy(sc_plan *plan)
{
    if (!plan) return SC_OK;
    if (plan->inner) {
        plan->inner->prof = nullptr;   // shared with this plan, freed below
        (void)sc_plan_destroy(plan->inner);
    }
    if (plan->d_tiles) (void)hipFree(plan->d_tiles);
    if (plan->d_slot_b) (void)hipFree(plan->d_slot_b);
    for (uint32_t *r : plan->walk.d_rec)
        if (r) (void)hipFree(r);
    if (plan->walk.d_heads) (void)hipFree(plan->walk.d_heads);
    for (sck::FixLevel *lv : {&plan->det_top, &plan->det_a, &plan->det_b}) {
        if (lv->d_fix) (void)hipFree(lv->d_fix);
        if (lv->d_segs) (void)hipFree(lv->d_segs);
    }
    if (plan->d_zero_rows) (void)hipFree(plan->d_zero_rows);
    if (plan->prof) {
        for (int i = 0; i < kMaxLaunches; ++i) {
            (void)hipEventDestroy(plan->prof->ev_begin[i]);
            (void)hipEventDestroy(plan->prof->ev_end[i]);
        }
        delete plan->prof;
    }
    delete plan;
    return SC_OK;
}
