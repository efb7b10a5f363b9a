// Host-side planning (see p2_plan.h).  Sections cited are those of arXiv 2110.10548.
#include "p2_plan.h"
#include "p2_device_pack.h"

#include <algorithm>
#include <map>

namespace p2 {

// ---------------------------------------------------------------------------------------------
// Sec. 3.1.  A row of the matrix is a factorisation of its axis over the levels with each factor
// dividing the level's cardinality; rows are generated in lexicographic order and combined row by
// row under the column constraint, which yields the lexicographic order of the flattening.
// ---------------------------------------------------------------------------------------------
namespace {

void row_factorisations(const int32_t* card, int n, int j, int64_t left, std::vector<int32_t>& cur,
                        std::vector<std::vector<int32_t>>& out) {
    if (j == n) {
        if (left == 1) out.push_back(cur);
        return;
    }
    for (int32_t v = 1; v <= card[j]; ++v) {
        if (card[j] % v != 0 || left % v != 0) continue;
        cur[j] = v;
        row_factorisations(card, n, j + 1, left / v, cur, out);
    }
}

struct PlaceCtx {
    int n, m;
    std::vector<std::vector<std::vector<int32_t>>> rows;   // per axis, its factorisations
    std::vector<int64_t> col_left;
    std::vector<const std::vector<int32_t>*> chosen;
    int32_t* out;
    int64_t cap, count;
};

void place_rows(PlaceCtx& c, int i) {
    if (i == c.m) {
        for (int j = 0; j < c.n; ++j)
            if (c.col_left[j] != 1) return;
        if (c.count < c.cap)
            for (int a = 0; a < c.m; ++a)
                for (int j = 0; j < c.n; ++j) c.out[(c.count * c.m + a) * c.n + j] = (*c.chosen[a])[j];
        ++c.count;
        return;
    }
    for (const auto& row : c.rows[i]) {
        bool ok = true;
        for (int j = 0; j < c.n && ok; ++j) ok = (c.col_left[j] % row[j] == 0);
        if (!ok) continue;
        for (int j = 0; j < c.n; ++j) c.col_left[j] /= row[j];
        c.chosen[i] = &row;
        place_rows(c, i + 1);
        for (int j = 0; j < c.n; ++j) c.col_left[j] *= row[j];
    }
}

int32_t check_hierarchy(const p2_hierarchy* h, bool need_links, int64_t& devices, std::string& err) {
    if (!h || !h->card) { err = "null hierarchy"; return P2_EINVAL; }
    if (h->n_levels < 1) { err = "n_levels < 1"; return P2_EINVAL; }
    if (h->n_levels > P2_MAX_LEVELS) { err = "more than 8 hardware levels"; return P2_EUNSUPPORTED; }
    devices = 1;
    for (int j = 0; j < h->n_levels; ++j) {
        if (h->card[j] < 1) { err = "level cardinality < 1"; return P2_EINVAL; }
        devices *= h->card[j];
        if (devices > (int64_t)1 << 40) { err = "too many devices"; return P2_EUNSUPPORTED; }
    }
    if (need_links) {
        if (!h->bw_bytes_per_s || !h->alpha_s) { err = "bandwidth/latency arrays are required for costs"; return P2_EINVAL; }
        for (int j = 0; j < h->n_levels; ++j) {
            if (!(h->bw_bytes_per_s[j] > 0.0)) { err = "bandwidth must be > 0"; return P2_EINVAL; }
            if (!(h->alpha_s[j] >= 0.0)) { err = "latency must be >= 0"; return P2_EINVAL; }
        }
    }
    return P2_OK;
}

}  // namespace

int32_t enumerate_placements(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, int32_t* out, int64_t cap,
                             int64_t* out_count, std::string& err) {
    int64_t devices = 0;
    int32_t st = check_hierarchy(h, false, devices, err);
    if (st != P2_OK) return st;
    if (!axes || !out_count) { err = "null argument"; return P2_EINVAL; }
    if (n_axes < 1) { err = "n_axes < 1"; return P2_EINVAL; }
    if (n_axes > P2_MAX_AXES) { err = "more than 8 axes"; return P2_EUNSUPPORTED; }
    if (cap < 0 || (cap > 0 && !out)) { err = "bad output buffer"; return P2_EINVAL; }
    int64_t prod = 1;
    for (int i = 0; i < n_axes; ++i) {
        if (axes[i] < 1) { err = "axis size < 1"; return P2_EINVAL; }
        prod *= axes[i];
        if (prod > (int64_t)1 << 40) break;
    }
    if (prod != devices) { err = "product of axes differs from the number of devices"; return P2_EINVAL; }
    PlaceCtx c;
    c.n = h->n_levels; c.m = n_axes; c.out = out; c.cap = cap; c.count = 0;
    c.rows.resize(n_axes);
    c.chosen.resize(n_axes);
    std::vector<int32_t> cur(c.n);
    for (int i = 0; i < n_axes; ++i) row_factorisations(h->card, c.n, 0, axes[i], cur, c.rows[i]);
    c.col_left.assign(h->card, h->card + c.n);
    place_rows(c, 0);
    *out_count = c.count;
    if (c.count > cap && cap > 0) { err = "placement buffer too small"; return P2_ENOSPC; }
    return P2_OK;
}

// ---------------------------------------------------------------------------------------------
// Bandwidth rows of one pattern.  A group whose members first differ at hardware level `span`
// crosses the uplink of every level-j unit (j >= span) that holds one of its members; the load of
// a unit is the sum of the bytes of those groups (they all belong to this pattern).  Groups of
// different copies with the same local group id carry the same bytes, so a unit is described by
// how many groups of each local id touch it.  Units with equal descriptions are merged, and a
// unit is dropped when another unit of the same level is at least as loaded whatever the bytes.
// ---------------------------------------------------------------------------------------------
namespace {

inline bool takes_part(const Pattern& p, int local) { return !p.master || (local % p.s) == 0; }
inline int local_group(const Pattern& p, int local) {
    int hi = local / (p.g * p.s), lo = local % p.s;
    return p.master ? hi : hi * p.s + lo;
}
inline int group_base(const Pattern& p, int group) {       // local id of the group's first device
    return p.master ? group * p.g * p.s : (group / p.s) * p.g * p.s + group % p.s;
}

void build_cost_rows(const Plan& pl, Pattern& p) {
    // scratch kept between calls: this runs for every pattern of every query of every call
    thread_local std::vector<int32_t> stamp, cnt, touched, row_begin, group_of, key_of, table, by_group_at, by_group, fill_at;
    thread_local std::vector<uint32_t> flat;
    thread_local std::vector<char> dead;
    p.row_ptr.assign(1, 0);
    p.row_level.clear();
    p.entries.clear();
    const int n_rep = pl.D / pl.R;
    stamp.assign((size_t)n_rep * p.n_groups, -1);
    cnt.assign(p.n_groups, 0);
    int stamp_id = 0;
    int below = pl.D;
    // a device's group in this pattern (-1: takes no part) and its (replica, group) key: the same at every level
    group_of.assign(pl.D, -1);
    key_of.assign(pl.D, 0);
    for (int d = 0; d < pl.D; ++d) {
        const int loc = pl.local_of[d];
        if (!takes_part(p, loc)) continue;
        group_of[d] = local_group(p, loc);
        key_of[d] = pl.replica_of[d] * p.n_groups + group_of[d];
    }
    for (int j = 0; j < pl.n; ++j) {
        below /= pl.h[j];
        if (j < p.span) continue;
        // rows of this level, one after the other in `flat`; row r is flat[row_begin[r] .. row_begin[r + 1])
        flat.clear();
        row_begin.assign(1, 0);
        size_t table_size = 16;                          // open addressing: row indices, -1 = free; at most half full
        while (table_size < 2 * (size_t)(pl.D / below)) table_size *= 2;
        table.assign(table_size, -1);
        const size_t table_mask = table_size - 1;
        for (int u = 0; u < pl.D / below; ++u) {
            ++stamp_id;
            touched.clear();
            for (int d = u * below; d < (u + 1) * below; ++d) {
                const int lg = group_of[d];
                if (lg < 0) continue;
                const size_t key = (size_t)key_of[d];
                if (stamp[key] == stamp_id) continue;
                stamp[key] = stamp_id;
                if (cnt[lg]++ == 0) touched.push_back(lg);
            }
            if (touched.empty()) continue;
            std::sort(touched.begin(), touched.end());
            const size_t first = flat.size();
            for (int lg : touched) { flat.push_back(entry_pack((uint32_t)lg, (uint32_t)group_base(p, lg), (uint32_t)cnt[lg])); cnt[lg] = 0; }
            // units with equal descriptions are one row: looked up by a hash of the description (the innermost level
            // has a unit per device, and comparing each with every row before it was most of this function's time)
            const size_t len = flat.size() - first;
            uint64_t hsh = 0x9e3779b97f4a7c15ull ^ len;
            for (size_t x = first; x < flat.size(); ++x) { hsh ^= flat[x]; hsh *= 0x100000001b3ull; hsh ^= hsh >> 29; }
            bool dup = false;
            size_t slot = (size_t)hsh & table_mask;
            for (;; slot = (slot + 1) & table_mask) {
                const int32_t r = table[slot];
                if (r < 0) break;
                if ((size_t)(row_begin[r + 1] - row_begin[r]) == len &&
                    std::equal(flat.begin() + first, flat.end(), flat.begin() + row_begin[r])) { dup = true; break; }
            }
            if (dup) flat.resize(first);
            else { table[slot] = (int32_t)row_begin.size() - 1; row_begin.push_back((int32_t)flat.size()); }
        }
        // drop rows dominated by another row of the same level
        const size_t n_rows = row_begin.size() - 1;
        dead.assign(n_rows, 0);
        // (a row that dominates row a holds every group of a, its first among them: the rows are listed by group, in
        //  ascending order, and only those of a's first group are asked)
        by_group_at.assign((size_t)p.n_groups + 1, 0);
        for (size_t x = 0; x < flat.size(); ++x) ++by_group_at[entry_group(flat[x]) + 1];
        for (int g2 = 0; g2 < p.n_groups; ++g2) by_group_at[g2 + 1] += by_group_at[g2];
        by_group.resize(flat.size());
        fill_at.assign(by_group_at.begin(), by_group_at.end() - 1);
        for (size_t r = 0; r < n_rows; ++r)
            for (int x = row_begin[r]; x < row_begin[r + 1]; ++x) by_group[fill_at[entry_group(flat[x])]++] = (int32_t)r;
        for (size_t a = 0; a < n_rows; ++a) {
            const uint32_t* ra = flat.data() + row_begin[a];
            const size_t na = (size_t)(row_begin[a + 1] - row_begin[a]);
            const uint32_t g0 = entry_group(ra[0]);
            for (int32_t at = by_group_at[g0]; at < by_group_at[g0 + 1] && !dead[a]; ++at) {
                const size_t b = (size_t)by_group[at];
                const uint32_t* rb = flat.data() + row_begin[b];
                const size_t nb = (size_t)(row_begin[b + 1] - row_begin[b]);
                if (a == b || dead[b] || nb < na) continue;
                size_t ib = 0;
                bool dom = true;
                for (size_t ia = 0; ia < na && dom; ++ia) {
                    uint32_t lg = entry_group(ra[ia]), c = entry_cnt(ra[ia]);
                    while (ib < nb && entry_group(rb[ib]) < lg) ++ib;
                    dom = ib < nb && entry_group(rb[ib]) == lg && entry_cnt(rb[ib]) >= c;
                }
                if (dom) dead[a] = 1;
            }
        }
        for (size_t a = 0; a < n_rows; ++a) {
            if (dead[a]) continue;
            p.entries.insert(p.entries.end(), flat.begin() + row_begin[a], flat.begin() + row_begin[a + 1]);
            p.row_ptr.push_back((int32_t)p.entries.size());
            p.row_level.push_back(j);
        }
    }
}

}  // namespace


// ---------------------------------------------------------------------------------------------
// Sec. 3.4: the hierarchies other than (d).  A level is a list of factors (axis i, hardware level
// j) of the matrix; the local id of a device is the mixed-radix number of its digits a_{i,j} taken
// level by level (first level and, inside a level, first factor most significant); the digits of
// the factors that belong to no level number the copy.  Devices: id = mixed radix of hardware
// coordinates, the coordinate at level j = mixed radix of the a_{i,j}, axis 0 most significant.
// ---------------------------------------------------------------------------------------------
namespace {

int32_t number_by_levels(Plan& pl, std::vector<int>& lf, std::vector<int>& lspan, std::string& err) {
    struct Cell { int i, j; };
    std::vector<std::vector<Cell>> levels;
    const int m = pl.m, n = pl.n;
    switch (pl.hierarchy) {
    case P2_HIERARCHY_SYSTEM:
        for (int j = 0; j < n; ++j) { levels.emplace_back(); for (int i = 0; i < m; ++i) levels.back().push_back({i, j}); }
        break;
    case P2_HIERARCHY_COLUMN:
        for (int j = 0; j < n; ++j) for (int i = 0; i < m; ++i) levels.push_back({{i, j}});
        break;
    case P2_HIERARCHY_ROW:
        for (int i = 0; i < m; ++i) for (int j = 0; j < n; ++j) levels.push_back({{i, j}});
        break;
    default:   // P2_HIERARCHY_REDUCTION
        for (int i = 0; i < m; ++i) if (pl.is_reduce[i]) for (int j = 0; j < n; ++j) levels.push_back({{i, j}});
        break;
    }
    int owner[P2_MAX_AXES][P2_MAX_LEVELS];
    for (int i = 0; i < m; ++i) for (int j = 0; j < n; ++j) owner[i][j] = -1;
    pl.R = 1;
    bool over_other_axes = false;
    for (size_t l = 0; l < levels.size(); ++l) {
        int f = 1, span = n;
        for (const Cell& c : levels[l]) {
            owner[c.i][c.j] = (int)l;
            f *= pl.x[c.i][c.j];
            if (pl.x[c.i][c.j] > 1) { span = std::min(span, c.j); over_other_axes = over_other_axes || !pl.is_reduce[c.i]; }
        }
        lf.push_back(f); lspan.push_back(span);
        pl.R *= f;
    }
    pl.level_f = lf;
    (void)err;

    pl.local_of.resize(pl.D);
    pl.replica_of.resize(pl.D);
    std::vector<int> other(pl.D);                              // number made of the non-reduction digits
    for (int d = 0; d < pl.D; ++d) {
        int a[P2_MAX_AXES][P2_MAX_LEVELS], rest = d;
        for (int j = n - 1; j >= 0; --j) {
            int c = rest % pl.h[j];
            rest /= pl.h[j];
            for (int i = m - 1; i >= 0; --i) { a[i][j] = c % pl.x[i][j]; c /= pl.x[i][j]; }
        }
        int local = 0, rep = 0, oth = 0;
        for (const auto& lv : levels)
            for (const Cell& c : lv) local = local * pl.x[c.i][c.j] + a[c.i][c.j];
        for (int j = 0; j < n; ++j)
            for (int i = 0; i < m; ++i) {
                if (owner[i][j] < 0) rep = rep * pl.x[i][j] + a[i][j];
                if (!pl.is_reduce[i]) oth = oth * pl.x[i][j] + a[i][j];
            }
        pl.local_of[d] = local; pl.replica_of[d] = rep; other[d] = oth;
    }
    // Sec. 3.2, goal: every device holds the sum over its reduction group.  With levels over other axes
    // the copy holds several reduction groups (the devices with equal digits on the other axes).
    if (over_other_axes) {
        const int mw = (pl.R + 31) / 32;
        pl.goal.assign((size_t)pl.R * mw, 0u);
        for (int d = 0; d < pl.D; ++d) {
            if (pl.replica_of[d] != 0) continue;
            for (int e = 0; e < pl.D; ++e)
                if (pl.replica_of[e] == 0 && other[e] == other[d])
                    pl.goal[(size_t)pl.local_of[d] * mw + (pl.local_of[e] >> 5)] |= 1u << (pl.local_of[e] & 31);
        }
    }
    return P2_OK;
}

// Ranks inside a group (ascending device id) of the members taken in ascending local id; the same for
// every group of a pattern, because the order of two members depends on the varied digits only.
void member_ranks(Plan& pl) {
    std::vector<int> dev_of(pl.R, 0);                          // device of copy 0 with a given local id
    for (int d = 0; d < pl.D; ++d)
        if (pl.replica_of[d] == 0) dev_of[pl.local_of[d]] = d;
    for (Pattern& p : pl.patterns) {
        p.rank.assign(p.g, 0);
        bool identity = true;
        for (int t = 0; t < p.g; ++t) {
            int r = 0;
            for (int u = 0; u < p.g; ++u) r += dev_of[u * p.s] < dev_of[t * p.s];
            p.rank[t] = r;
            identity = identity && r == t;
        }
        if (identity) p.rank.clear();
    }
}

}  // namespace

int32_t make_plan(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* placement,
                  const int32_t* reduce_axes, int32_t n_reduce, int32_t max_len, const p2_options* opt, bool with_cost,
                  Plan& pl, std::string& err, bool build_rows) {
    int64_t devices = 0;
    int32_t st = check_hierarchy(h, with_cost, devices, err);
    if (st != P2_OK) return st;
    if (!axes || !placement || !reduce_axes) { err = "null argument"; return P2_EINVAL; }
    if (n_axes < 1) { err = "n_axes < 1"; return P2_EINVAL; }
    if (n_axes > P2_MAX_AXES) { err = "more than 8 axes"; return P2_EUNSUPPORTED; }
    if (devices > P2_MAX_DEVICES) { err = "more than 512 devices"; return P2_EUNSUPPORTED; }
    if (n_reduce < 1) { err = "empty set of reduce axes"; return P2_EINVAL; }
    if (max_len < 1) { err = "max_len < 1"; return P2_EINVAL; }
    if (max_len > P2_MAX_LEN) { err = "max_len > 7"; return P2_EUNSUPPORTED; }
    if (opt && opt->algo != 0 && opt->algo != 1) { err = "unknown cost model (algo is 0 = ring or 1 = tree)"; return P2_EUNSUPPORTED; }
    if (opt && (opt->hierarchy < 0 || opt->hierarchy > P2_HIERARCHY_REDUCTION)) { err = "unknown synthesis hierarchy"; return P2_EUNSUPPORTED; }
    if (opt && (opt->max_row_classes < 0 || opt->max_row_classes > 64)) { err = "max_row_classes outside 0..64"; return P2_EINVAL; }
    if (opt && (opt->frontier_pairs < 0 || opt->frontier_pairs > P2_FRONTIER_PAIRS_NONE)) { err = "unknown frontier_pairs"; return P2_EINVAL; }
    if (opt && (opt->flags & ~(P2_FLAG_EVALUATE_EVERY_QUERY | P2_FLAG_ONE_ENUMERATION_AT_A_TIME)) != 0) { err = "unknown option flag"; return P2_EINVAL; }

    pl = Plan();
    pl.n = h->n_levels; pl.m = n_axes; pl.D = (int)devices; pl.max_len = max_len;
    pl.algo = opt ? opt->algo : 0;
    pl.hierarchy = opt ? opt->hierarchy : P2_HIERARCHY_COLLAPSED;
    pl.max_row_classes = (opt && opt->max_row_classes > 0) ? opt->max_row_classes : 64;
    pl.frontier_pairs = opt ? opt->frontier_pairs : P2_FRONTIER_PAIRS_AUTO;
    for (int j = 0; j < pl.n; ++j) {
        pl.h[j] = h->card[j];
        pl.bw[j] = h->bw_bytes_per_s ? h->bw_bytes_per_s[j] : 1.0;
        pl.alpha[j] = h->alpha_s ? h->alpha_s[j] : 0.0;
    }
    int64_t prod_axes = 1;
    for (int i = 0; i < n_axes; ++i) {
        if (axes[i] < 1) { err = "axis size < 1"; return P2_EINVAL; }
        prod_axes *= axes[i];
        if (prod_axes > devices) break;
    }
    if (prod_axes != devices) { err = "product of axes differs from the number of devices"; return P2_EINVAL; }
    for (int i = 0; i < n_axes; ++i) {
        int64_t pr = 1;
        for (int j = 0; j < pl.n; ++j) {
            int v = placement[i * pl.n + j];
            if (v < 1) { err = "placement factor < 1"; return P2_EINVAL; }
            pl.x[i][j] = v;
            pr *= v;
        }
        if (pr != axes[i]) { err = "placement row product differs from the axis size (Eq. 2)"; return P2_EINVAL; }
    }
    for (int j = 0; j < pl.n; ++j) {
        int64_t pr = 1;
        for (int i = 0; i < n_axes; ++i) pr *= pl.x[i][j];
        if (pr != pl.h[j]) { err = "placement column product differs from the level cardinality (Eq. 1)"; return P2_EINVAL; }
    }
    for (int r = 0; r < n_reduce; ++r) {
        int a = reduce_axes[r];
        if (a < 0 || a >= n_axes) { err = "reduce axis out of range"; return P2_EINVAL; }
        if (pl.is_reduce[a]) { err = "duplicate reduce axis"; return P2_EINVAL; }
        pl.is_reduce[a] = true;
    }
    pl.form_mask = (opt && opt->form_mask) ? (opt->form_mask & 7u) : 7u;
    pl.op_mask = (opt && opt->op_mask) ? (opt->op_mask & 31u) : 31u;
    if (pl.form_mask == 0 || pl.op_mask == 0) { err = "empty form or op mask"; return P2_EINVAL; }
    for (int o = 0; o < 5; ++o)
        if (pl.op_mask & (1u << o)) pl.ops[pl.n_ops++] = o;
    int k = (opt && opt->n_chunks != 0) ? opt->n_chunks : pl.D;
    if (k < 1) { err = "n_chunks < 0"; return P2_EINVAL; }
    if (k > 512) { err = "more than 512 chunks"; return P2_EUNSUPPORTED; }
    pl.k = k;

    std::vector<int> lf;                                        // factor of every synthesis level
    std::vector<int> lspan;                                     // outermost hardware level of its factors > 1
    if (pl.hierarchy == P2_HIERARCHY_COLLAPSED) {
        // Sec. 3.4, hierarchy (d): per hardware level the product of the reduce axes' factors.
        pl.R = 1;
        for (int j = 0; j < pl.n; ++j) {
            pl.f[j] = 1;
            for (int i = 0; i < n_axes; ++i)
                if (pl.is_reduce[i]) pl.f[j] *= pl.x[i][j];
            pl.R *= pl.f[j];
        }
        // Devices: id = mixed radix of hardware coordinates; inside a level the coordinate is a mixed
        // radix of the axis digits, axis 0 most significant.  Split every coordinate into its
        // reduce-axis part (-> local id) and the rest (-> replica).
        pl.local_of.resize(pl.D);
        pl.replica_of.resize(pl.D);
        for (int d = 0; d < pl.D; ++d) {
            int coord[P2_MAX_LEVELS], rest = d;
            for (int j = pl.n - 1; j >= 0; --j) { coord[j] = rest % pl.h[j]; rest /= pl.h[j]; }
            int local = 0, rep = 0;
            for (int j = 0; j < pl.n; ++j) {
                int c = coord[j], gdig = 0, rdig = 0, gmul = 1, rmul = 1;
                for (int i = n_axes - 1; i >= 0; --i) {          // least significant axis first
                    int a = c % pl.x[i][j];
                    c /= pl.x[i][j];
                    if (pl.is_reduce[i]) { gdig += a * gmul; gmul *= pl.x[i][j]; }
                    else { rdig += a * rmul; rmul *= pl.x[i][j]; }
                }
                local = local * pl.f[j] + gdig;
                rep = rep * (pl.h[j] / pl.f[j]) + rdig;
            }
            pl.local_of[d] = local;
            pl.replica_of[d] = rep;
        }
        for (int j = 0; j < pl.n; ++j) { lf.push_back(pl.f[j]); lspan.push_back(j); }
    } else {
        st = number_by_levels(pl, lf, lspan, err);
        if (st != P2_OK) return st;
    }
    const int sl = (int)lf.size();

    // Sec. 3.3 patterns in the order: for every slice e_i (e_0 = root): InsideGroup,
    // Parallel(e_0..e_{i-1}), Master(e_0..e_{i-1}).  Level e_l (l >= 1) is hardware level l-1.
    // A pattern is identified by the levels with factor > 1 that vary inside a group plus whether
    // the Master restriction removes anything; equal identities give equal group sets, and the
    // first occurrence keeps the id.
    std::vector<int> suffix(sl + 1, 1);                         // suffix[j] = prod lf[j..sl-1]
    for (int j = sl - 1; j >= 0; --j) suffix[j] = suffix[j + 1] * lf[j];
    auto add = [&](int slice, int form, int form_level, int a, int b) {   // synthesis levels a..b vary
        int lo = -1, hi = -1, span = pl.n;
        for (int j = a; j <= b; ++j)
            if (lf[j] > 1) { if (lo < 0) lo = j; hi = j; span = std::min(span, lspan[j]); }
        if (lo < 0) return;                                     // only groups of one device
        Pattern p;
        p.slice = slice; p.form = form; p.form_level = form_level; p.lo = lo; p.hi = hi; p.span = span;
        p.s = suffix[hi + 1];
        p.g = suffix[lo] / p.s;
        p.master = (form == 2 && p.s > 1) ? 1 : 0;
        p.n_groups = p.master ? pl.R / (p.g * p.s) : pl.R / p.g;
        for (const Pattern& q : pl.patterns)
            if (q.lo == p.lo && q.hi == p.hi && q.master == p.master) return;
        pl.patterns.push_back(p);
    };
    for (int i = 0; i <= sl; ++i) {
        if (pl.form_mask & 1u) add(i, 0, -1, i, sl - 1);
        if (pl.form_mask & 2u)
            for (int j = 0; j < i; ++j) add(i, 1, j, j, i - 1);
        if (pl.form_mask & 4u)
            for (int j = 0; j < i; ++j) add(i, 2, j, j, i - 1);
    }
    if (pl.hierarchy != P2_HIERARCHY_COLLAPSED) member_ranks(pl);
    pl.alphabet = (int)pl.patterns.size() * pl.n_ops;

    // Candidate numbering: by length, then lexicographic.
    uint64_t pw = 1, total = 0;
    pl.base[1] = 0;
    for (int l = 1; l <= max_len; ++l) {
        if (pl.alphabet != 0 && pw > UINT64_MAX / (uint64_t)pl.alphabet) { err = "candidate count overflows 64 bits"; return P2_EINVAL; }
        pw *= (uint64_t)pl.alphabet;
        if (total > UINT64_MAX - pw) { err = "candidate count overflows 64 bits"; return P2_EINVAL; }
        total += pw;
        pl.base[l + 1] = total;
    }
    pl.n_candidates = total;
    if (with_cost && build_rows)
        for (Pattern& p : pl.patterns) build_cost_rows(pl, p);
    return P2_OK;
}

void build_cost_tables(Plan& pl) {
    for (Pattern& p : pl.patterns) build_cost_rows(pl, p);
}

void describe_pattern(const Plan& pl, int pattern_id, int32_t* group_of_device, int32_t* rank_in_group) {
    const Pattern& p = pl.patterns[pattern_id];
    std::map<std::pair<int, int>, int> ids;
    for (int d = 0; d < pl.D; ++d) {
        int loc = pl.local_of[d];
        if (!takes_part(p, loc)) { group_of_device[d] = -1; rank_in_group[d] = -1; continue; }
        auto key = std::make_pair(pl.replica_of[d], local_group(p, loc));
        auto it = ids.find(key);
        if (it == ids.end()) it = ids.emplace(key, (int)ids.size()).first;
        group_of_device[d] = it->second;
        const int t = (loc / p.s) % p.g;
        rank_in_group[d] = p.rank.empty() ? t : p.rank[t];
    }
}

}  // namespace p2
