/*
 * p2_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-file CPU statement of what the P^2 reduction-program
 * synthesizer (arXiv 2110.10548) computes: parallelism placements (Sec. 3.1,
 * Eq. 1-2), the device-state semantics of the five collectives (Sec. 3.2 and
 * the figure "Semantics of collective operations"), the reduction DSL and its
 * device groups (Sec. 3.3 and the table "Hierarchical communication
 * patterns"), the reduction-axis synthesis hierarchy with its root level
 * (Sec. 3.4, Appendix B), the init/goal states and enumeration by program
 * size (Sec. 3.5), a ring alpha-beta cost (Sec. 5 names only the bandwidth
 * inputs; the formula below is a stated reading) and a sort-based top-k.
 *
 * Everything here works on the literal objects of the paper: the FULL system
 * of D devices, one k x D boolean state matrix per device (stored as k rows
 * of D-bit masks), and explicit lists of member devices per group.  Nothing
 * is blocked, fused, compressed or replicated.  It shares no code with the
 * GPU library and must only be used by tests, the smoke check and the
 * CPU-baseline leg of the benchmark.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * into this file.
 *
 * What pins it (tests/test_oracle_pins.py): the paper's placement lists and
 * program totals, its worked examples of the five collectives, its tables of
 * device groups and synthesis hierarchies, its named programs, its lemmas and
 * its expressiveness theorem.  Parity unpinned by any value the paper prints,
 * and held only by closed forms, invariants and hand-worked cases: the
 * semantics of the Master form, the program sets of three and more levels,
 * and every cost (ring and tree models are stated readings).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <stdio.h>

#define MAXLV 8            /* hardware levels                      */
#define MAXAX 8            /* parallelism axes                     */
#define MAXD 512           /* devices                              */
#define MAXW (MAXD / 64)   /* 64-bit words per D-bit column mask   */
#define MAXSL (MAXAX * MAXLV) /* levels of a synthesis hierarchy (one per matrix cell at most) */
#define MAXPAT ((MAXLV + 1) * (MAXLV + 1))
#define MAXLEN 8           /* program size limit supported         */

enum { OP_ALLREDUCE = 0, OP_REDUCESCATTER = 1, OP_ALLGATHER = 2, OP_REDUCE = 3, OP_BROADCAST = 4 };
enum { FORM_INSIDEGROUP = 0, FORM_PARALLEL = 1, FORM_MASTER = 2 };

/* ------------------------------------------------------------------ */
/* Sec. 3.1: parallelism matrices.  x[i][j] >= 1 integer,              */
/*   Eq. (1): prod_i x[i][j] = h_j,   Eq. (2): prod_j x[i][j] = p_i.   */
/* Enumerated in lexicographic order of the row-major flattening.      */
/* ------------------------------------------------------------------ */
typedef struct {
    int n, m;
    const int32_t *h, *p;
    int x[MAXAX][MAXLV];
    int32_t *out;
    int64_t cap, count;
} place_ctx;

static void place_rec(place_ctx *c, int pos)
{
    int n = c->n, m = c->m;
    if (pos == n * m) {
        /* every cell chosen: check Eq. (1) and Eq. (2) literally */
        for (int j = 0; j < n; j++) {
            long long pr = 1;
            for (int i = 0; i < m; i++) pr *= c->x[i][j];
            if (pr != c->h[j]) return;
        }
        for (int i = 0; i < m; i++) {
            long long pr = 1;
            for (int j = 0; j < n; j++) pr *= c->x[i][j];
            if (pr != c->p[i]) return;
        }
        if (c->count < c->cap)
            for (int i = 0; i < m; i++)
                for (int j = 0; j < n; j++)
                    c->out[(c->count * m + i) * n + j] = c->x[i][j];
        c->count++;
        return;
    }
    int i = pos / n, j = pos % n;
    /* a cell can only be a divisor of what is left of its row and column */
    long long rowleft = c->p[i], colleft = c->h[j];
    for (int jj = 0; jj < j; jj++) rowleft /= c->x[i][jj];
    for (int ii = 0; ii < i; ii++) colleft /= c->x[ii][j];
    for (int v = 1; v <= rowleft && v <= colleft; v++) {
        if (rowleft % v || colleft % v) continue;
        c->x[i][j] = v;
        place_rec(c, pos + 1);
    }
}

int64_t p2o_enumerate_placements(int n_levels, const int32_t *card, int n_axes, const int32_t *axes,
                                 int32_t *out, int64_t cap)
{
    if (n_levels < 1 || n_levels > MAXLV || n_axes < 1 || n_axes > MAXAX) return -1;
    place_ctx c;
    memset(&c, 0, sizeof c);
    c.n = n_levels; c.m = n_axes; c.h = card; c.p = axes; c.out = out; c.cap = cap;
    place_rec(&c, 0);
    return c.count;
}

int p2o_hierarchy_of_matrix(int m, int n, const int32_t *x, const int32_t *is_reduce, int kind, int64_t *out);

/* ------------------------------------------------------------------ */
/* A query: system + placement + reduction axes, and everything        */
/* derived from them.                                                  */
/* ------------------------------------------------------------------ */
typedef struct {
    int slice, form, form_level;  /* (slice e_i, form, form's level e_j or -1) */
    int n_groups;
    int *group_of;                /* [D]  group id or -1                        */
    int *rank_of;                 /* [D]  position inside the group             */
    int *gsize;                   /* [n_groups]                                 */
    int *gstart;                  /* [n_groups] offset into members             */
    int *members;                 /* concatenated member device ids, ascending  */
} p2o_pattern;

typedef struct {
    int n, m;                     /* hardware levels, axes                      */
    int h[MAXLV];
    double bw[MAXLV], alpha[MAXLV];
    int p[MAXAX];
    int x[MAXAX][MAXLV];
    int is_reduce[MAXAX];
    int D, k, W;
    int (*coord)[MAXLV];          /* [D][n]   hardware coordinate c_j of a device          */
    int (*digit)[MAXAX][MAXLV];   /* [D][m][n] axis digit a_{i,j} of a device              */
    int kind;                     /* synthesis hierarchy (Sec. 3.4): 3 = (d), the tool's choice;
                                     4 = (a) system, 0 = (b) column-based, 1 = (c) row-based,
                                     2 = reduction-axis factors before they are collapsed  */
    int sl;                       /* its levels e_1..e_sl; e_0 = root (1) is put in front  */
    int f[MAXSL + 1];             /* their factors, f[0] = 1                               */
    int cell_level[MAXAX][MAXLV]; /* level that the factor x[i][j] belongs to; 0 = none:
                                     the pattern is repeated over that digit (lowering)    */
    uint64_t *goal;               /* [D][W]   mask of the device's reduction group         */
    int n_patterns;
    p2o_pattern pat[MAXPAT];
    uint32_t form_mask, op_mask;
    int n_ops, ops[5];            /* enabled collectives in the paper's order              */
    int algo;                     /* cost model of AllReduce: 0 ring, 1 tree (Sec. 4)      */
    char err[256];
} p2o_query;

static void pattern_free(p2o_pattern *pt)
{
    free(pt->group_of); free(pt->rank_of); free(pt->gsize); free(pt->gstart); free(pt->members);
    memset(pt, 0, sizeof *pt);
}

void p2o_query_free(p2o_query *q)
{
    if (!q) return;
    for (int i = 0; i < q->n_patterns; i++) pattern_free(&q->pat[i]);
    free(q->coord); free(q->digit); free(q->goal);
    free(q);
}

/*
 * Device groups of one (slice e_i, form) pair on the full system (Sec. 3.3).
 * A level of the synthesis hierarchy owns some factors x[i][j] of the matrix
 * (cell_level); a device's digit at the level is made of its digits a_{i,j}
 * at those factors.
 *   InsideGroup : devices that agree on everything except the digits of
 *                 levels e_{i+1}..e_last form one group.
 *   Parallel(e_j), j < i : devices that agree on everything except the digits
 *                 of levels e_{j+1}..e_i ("the first device of each e_i-group,
 *                 the second, ..., as far as they connect to the same e_j").
 *   Master(e_j): the Parallel(e_j) groups, but only those made of the first
 *                 device of each e_i-group, i.e. digits of e_{i+1}..e_n all 0.
 *                 Reading: "first" is taken per e_j instance and per replica
 *                 over the non-reduction axes, because lowering applies the
 *                 pattern to the non-reduction axes (Sec. 3.4).
 * "Everything" includes every digit of every factor outside the hierarchy:
 * for (d), every digit of every non-reduction axis (lowering).
 * Groups of one device are not reductions and are dropped (Appendix B).
 */
static int build_pattern(const p2o_query *q, int slice, int form, int form_level, p2o_pattern *pt)
{
    int D = q->D, n = q->n;
    int vlo, vhi;                         /* levels whose digit varies inside a group */
    if (form == FORM_INSIDEGROUP) { vlo = slice + 1; vhi = q->sl; }
    else                          { vlo = form_level + 1; vhi = slice; }
    memset(pt, 0, sizeof *pt);
    pt->slice = slice; pt->form = form; pt->form_level = form_level;
    pt->group_of = malloc(sizeof(int) * D);
    pt->rank_of = malloc(sizeof(int) * D);
    pt->gsize = malloc(sizeof(int) * D);
    pt->gstart = malloc(sizeof(int) * D);
    pt->members = malloc(sizeof(int) * D);
    int *leader = malloc(sizeof(int) * D);   /* smallest device of each tentative group */
    int *tsize = malloc(sizeof(int) * D);
    int *tgroup = malloc(sizeof(int) * D);
    int nt = 0;
    for (int d = 0; d < D; d++) {
        tgroup[d] = -1;
        if (form == FORM_MASTER) {
            int first = 1;
            for (int i = 0; i < q->m; i++)
                for (int j = 0; j < n; j++) if (q->cell_level[i][j] > slice && q->digit[d][i][j] != 0) first = 0;
            if (!first) continue;
        }
        /* look for an earlier group whose leader agrees with d outside the varying levels */
        int g = -1;
        for (int t = 0; t < nt && g < 0; t++) {
            int e = leader[t], same = 1;
            for (int i = 0; i < q->m && same; i++)
                for (int j = 0; j < n; j++) {
                    int l = q->cell_level[i][j];      /* 0: a digit outside the hierarchy never varies */
                    if (l >= vlo && l <= vhi && l > 0) continue;
                    if (q->digit[d][i][j] != q->digit[e][i][j]) { same = 0; break; }
                }
            if (same) g = t;
        }
        if (g < 0) { g = nt++; leader[g] = d; tsize[g] = 0; }
        tgroup[d] = g;
        tsize[g]++;
    }
    /* keep groups with more than one device; number them by smallest member */
    int *newid = malloc(sizeof(int) * (nt > 0 ? nt : 1));
    int ng = 0, off = 0;
    for (int t = 0; t < nt; t++) {
        if (tsize[t] > 1) { newid[t] = ng; pt->gsize[ng] = tsize[t]; pt->gstart[ng] = off; off += tsize[t]; ng++; }
        else newid[t] = -1;
    }
    int *fill = calloc(ng > 0 ? ng : 1, sizeof(int));
    for (int d = 0; d < D; d++) {
        pt->group_of[d] = -1; pt->rank_of[d] = -1;
        if (tgroup[d] < 0 || newid[tgroup[d]] < 0) continue;
        int g = newid[tgroup[d]];
        pt->group_of[d] = g;
        pt->rank_of[d] = fill[g];
        pt->members[pt->gstart[g] + fill[g]] = d;   /* ascending device id: d runs upward */
        fill[g]++;
    }
    pt->n_groups = ng;
    free(leader); free(tsize); free(tgroup); free(newid); free(fill);
    return ng;
}

static int same_groups(const p2o_pattern *a, const p2o_pattern *b, int D)
{
    /* two patterns are the same iff they induce the same set of device groups */
    if (a->n_groups != b->n_groups) return 0;
    for (int d = 0; d < D; d++) {
        if ((a->group_of[d] < 0) != (b->group_of[d] < 0)) return 0;
        if (a->group_of[d] < 0) continue;
        /* groups are numbered by smallest member in both, so ids must agree */
        if (a->group_of[d] != b->group_of[d]) return 0;
    }
    return 1;
}

p2o_query *p2o_query_create_kind(int n_levels, const int32_t *card, const double *bw, const double *alpha,
                                 int n_axes, const int32_t *axes, const int32_t *placement,
                                 int n_reduce, const int32_t *reduce_axes,
                                 int n_chunks, uint32_t form_mask, uint32_t op_mask, int kind);

p2o_query *p2o_query_create(int n_levels, const int32_t *card, const double *bw, const double *alpha,
                            int n_axes, const int32_t *axes, const int32_t *placement,
                            int n_reduce, const int32_t *reduce_axes,
                            int n_chunks, uint32_t form_mask, uint32_t op_mask)
{
    /* the tool synthesizes on hierarchy (d) */
    return p2o_query_create_kind(n_levels, card, bw, alpha, n_axes, axes, placement, n_reduce, reduce_axes,
                                 n_chunks, form_mask, op_mask, 3);
}

/* kind: the synthesis hierarchy (Sec. 3.4, Appendix A): 4 = (a) the system's own levels, 0 = (b) the
 * matrix's factors column by column, 1 = (c) row by row, 2 = the reduction axes' rows only,
 * 3 = (d) those rows collapsed per hardware level.  Every kind gets a root level in front. */
p2o_query *p2o_query_create_kind(int n_levels, const int32_t *card, const double *bw, const double *alpha,
                                 int n_axes, const int32_t *axes, const int32_t *placement,
                                 int n_reduce, const int32_t *reduce_axes,
                                 int n_chunks, uint32_t form_mask, uint32_t op_mask, int kind)
{
    if (kind < 0 || kind > 4) return NULL;
    if (n_levels < 1 || n_levels > MAXLV || n_axes < 1 || n_axes > MAXAX) return NULL;
    if (n_reduce < 1 || n_reduce > n_axes) return NULL;
    p2o_query *q = calloc(1, sizeof *q);
    q->n = n_levels; q->m = n_axes;
    long long D = 1;
    for (int j = 0; j < n_levels; j++) {
        if (card[j] < 1) { free(q); return NULL; }
        q->h[j] = card[j]; q->bw[j] = bw ? bw[j] : 1.0; q->alpha[j] = alpha ? alpha[j] : 0.0;
        D *= card[j];
        if (D > MAXD) { free(q); return NULL; }
    }
    for (int i = 0; i < n_axes; i++) {
        q->p[i] = axes[i];
        for (int j = 0; j < n_levels; j++) q->x[i][j] = placement[i * n_levels + j];
    }
    /* the placement must satisfy Eq. (1) and Eq. (2) */
    for (int j = 0; j < n_levels; j++) {
        long long pr = 1;
        for (int i = 0; i < n_axes; i++) { if (q->x[i][j] < 1) { free(q); return NULL; } pr *= q->x[i][j]; }
        if (pr != q->h[j]) { free(q); return NULL; }
    }
    for (int i = 0; i < n_axes; i++) {
        long long pr = 1;
        for (int j = 0; j < n_levels; j++) pr *= q->x[i][j];
        if (pr != q->p[i]) { free(q); return NULL; }
    }
    for (int r = 0; r < n_reduce; r++) {
        int a = reduce_axes[r];
        if (a < 0 || a >= n_axes || q->is_reduce[a]) { free(q); return NULL; }
        q->is_reduce[a] = 1;
    }
    q->D = (int)D;
    q->k = n_chunks > 0 ? n_chunks : q->D;        /* Sec. 3.2: data is split in k chunks, k = #devices */
    q->W = (q->D + 63) / 64;
    q->form_mask = form_mask; q->op_mask = op_mask;
    for (int o = 0; o < 5; o++) if (op_mask & (1u << o)) q->ops[q->n_ops++] = o;

    int n = q->n, m = q->m;
    q->coord = calloc(q->D, sizeof *q->coord);
    q->digit = calloc(q->D, sizeof *q->digit);
    q->goal = calloc((size_t)q->D * q->W, sizeof(uint64_t));

    /* Device id = mixed radix of the hardware coordinates, outermost level most
     * significant (devices A0..D3 of the running example).  Inside one hardware
     * level the coordinate is a mixed radix of the axis digits with radices
     * x[0][j], x[1][j], ..., axis 0 most significant (the column-based hierarchy
     * lists x_{0j} before x_{1j}). */
    for (int d = 0; d < q->D; d++) {
        int rest = d;
        for (int j = n - 1; j >= 0; j--) { q->coord[d][j] = rest % q->h[j]; rest /= q->h[j]; }
        for (int j = 0; j < n; j++) {
            int c = q->coord[d][j];
            for (int i = m - 1; i >= 0; i--) { q->digit[d][i][j] = c % q->x[i][j]; c /= q->x[i][j]; }
        }
    }
    /* Synthesis hierarchy: which factor of the matrix belongs to which level.
     * (d): reduction-axis factors only, factors of the same hardware level
     * collapsed (multiplied); (root,1) is put in front of every kind. */
    q->kind = kind;
    q->f[0] = 1;
    {
        int32_t flat[MAXAX * MAXLV], red[MAXAX];
        int64_t col[MAXSL];
        for (int i = 0; i < m; i++) { red[i] = q->is_reduce[i]; for (int j = 0; j < n; j++) flat[i * n + j] = q->x[i][j]; }
        if (kind == 4) {                                   /* (a): one level per hardware level */
            q->sl = n;
            for (int j = 0; j < n; j++) { q->f[j + 1] = q->h[j]; for (int i = 0; i < m; i++) q->cell_level[i][j] = j + 1; }
        } else {
            q->sl = p2o_hierarchy_of_matrix(m, n, flat, red, kind, col);
            for (int l = 0; l < q->sl; l++) q->f[l + 1] = (int)col[l];
            int l = 0;
            if (kind == 0) { for (int j = 0; j < n; j++) for (int i = 0; i < m; i++) q->cell_level[i][j] = ++l; }
            else if (kind == 1) { for (int i = 0; i < m; i++) for (int j = 0; j < n; j++) q->cell_level[i][j] = ++l; }
            else if (kind == 2) { for (int i = 0; i < m; i++) if (red[i]) for (int j = 0; j < n; j++) q->cell_level[i][j] = ++l; }
            else { for (int j = 0; j < n; j++) for (int i = 0; i < m; i++) q->cell_level[i][j] = red[i] ? j + 1 : 0; }
        }
    }
    /* Goal (Sec. 3.5): a device ends with the columns of every device it reduces
     * with: those that agree with it on all digits of all non-reduction axes. */
    for (int d = 0; d < q->D; d++)
        for (int e = 0; e < q->D; e++) {
            int same = 1;
            for (int i = 0; i < m && same; i++) {
                if (q->is_reduce[i]) continue;
                for (int j = 0; j < n; j++) if (q->digit[d][i][j] != q->digit[e][i][j]) { same = 0; break; }
            }
            if (same) q->goal[(size_t)d * q->W + e / 64] |= 1ull << (e % 64);
        }
    /* Patterns: for every slice e_i: InsideGroup, Parallel(e_0..e_{i-1}),
     * Master(e_0..e_{i-1}); the form's level is a strict ancestor of the slice.
     * A pattern with no group left is dropped; a pattern whose groups equal an
     * earlier pattern's is the same instruction and is dropped too. */
    for (int i = 0; i <= q->sl; i++) {
        for (int form = 0; form < 3; form++) {
            if (!(form_mask & (1u << form))) continue;
            int jlo = (form == FORM_INSIDEGROUP) ? -1 : 0;
            int jhi = (form == FORM_INSIDEGROUP) ? -1 : i - 1;
            for (int j = jlo; j <= jhi; j++) {
                p2o_pattern pt;
                int ng = build_pattern(q, i, form, j, &pt);
                int dup = 0;
                for (int t = 0; t < q->n_patterns && !dup; t++) dup = same_groups(&q->pat[t], &pt, q->D);
                if (ng == 0 || dup) { pattern_free(&pt); continue; }
                if (q->n_patterns == MAXPAT) { pattern_free(&pt); p2o_query_free(q); return NULL; }
                q->pat[q->n_patterns++] = pt;
            }
        }
    }
    return q;
}

/* Device groups of a single (slice, form) pair before empty patterns are dropped
 * and duplicates removed -- the rows of the table "Hierarchical communication
 * patterns".  form_level is ignored for InsideGroup.  Returns the group count. */
int p2o_groups_raw(const p2o_query *q, int slice, int form, int form_level,
                   int32_t *group_of_device, int32_t *rank_in_group)
{
    if (slice < 0 || slice > q->sl || form < 0 || form > 2) return -1;
    if (form != FORM_INSIDEGROUP && (form_level < 0 || form_level >= slice)) return -1;
    p2o_pattern pt;
    int ng = build_pattern(q, slice, form, form == FORM_INSIDEGROUP ? -1 : form_level, &pt);
    for (int d = 0; d < q->D; d++) { group_of_device[d] = pt.group_of[d]; rank_in_group[d] = pt.rank_of[d]; }
    pattern_free(&pt);
    return ng;
}

/* Synthesis hierarchies of Sec. 2.4 / Sec. 3.4 for a parallelism matrix
 * x[m][n] (row = axis, column = hardware level):
 *   kind 0: column-based factors   (b)   x00 x10 .. x01 x11 ..
 *   kind 1: row-based factors      (c)   x00 x01 .. x10 x11 ..
 *   kind 2: reduction-axis factors       rows of the reduced axes, row-wise
 *   kind 3: collapsed (d)                product of the reduced rows per column
 * Returns the number of entries written (no root level is added here). */
int p2o_hierarchy_of_matrix(int m, int n, const int32_t *x, const int32_t *is_reduce, int kind, int64_t *out)
{
    int c = 0;
    if (kind == 0) { for (int j = 0; j < n; j++) for (int i = 0; i < m; i++) out[c++] = x[i * n + j]; }
    else if (kind == 1) { for (int i = 0; i < m; i++) for (int j = 0; j < n; j++) out[c++] = x[i * n + j]; }
    else if (kind == 2) { for (int i = 0; i < m; i++) if (is_reduce[i]) for (int j = 0; j < n; j++) out[c++] = x[i * n + j]; }
    else if (kind == 3) {
        for (int j = 0; j < n; j++) { int64_t pr = 1; for (int i = 0; i < m; i++) if (is_reduce[i]) pr *= x[i * n + j]; out[c++] = pr; }
    } else return -1;
    return c;
}

int p2o_set_algo(p2o_query *q, int algo)
{
    if (algo != 0 && algo != 1) return -1;
    q->algo = algo;
    return 0;
}
int p2o_num_devices(const p2o_query *q) { return q->D; }
int p2o_num_chunks(const p2o_query *q) { return q->k; }
int p2o_num_patterns(const p2o_query *q) { return q->n_patterns; }
int p2o_alphabet_size(const p2o_query *q) { return q->n_patterns * q->n_ops; }
int p2o_synthesis_levels(const p2o_query *q) { return q->sl; }
void p2o_synthesis_hierarchy(const p2o_query *q, int32_t *out) { for (int l = 0; l <= q->sl; l++) out[l] = q->f[l]; }

int p2o_pattern_info(const p2o_query *q, int pid, int32_t *slice, int32_t *form, int32_t *form_level,
                     int32_t *group_of_device, int32_t *rank_in_group)
{
    if (pid < 0 || pid >= q->n_patterns) return -1;
    const p2o_pattern *pt = &q->pat[pid];
    *slice = pt->slice; *form = pt->form; *form_level = pt->form_level;
    for (int d = 0; d < q->D; d++) { group_of_device[d] = pt->group_of[d]; rank_in_group[d] = pt->rank_of[d]; }
    return pt->n_groups;
}

/* ------------------------------------------------------------------ */
/* Candidate numbering: programs ordered by length, then               */
/* lexicographically with the first instruction most significant.      */
/* An instruction digit is pattern_index * n_ops + op_index; the       */
/* stored instruction code is pattern_id * 5 + op.                     */
/* ------------------------------------------------------------------ */
uint64_t p2o_num_candidates(const p2o_query *q, int max_len)
{
    uint64_t I = (uint64_t)p2o_alphabet_size(q), total = 0, pw = 1;
    for (int l = 1; l <= max_len; l++) {
        if (I != 0 && pw > UINT64_MAX / I) return UINT64_MAX;
        pw *= I;
        if (total > UINT64_MAX - pw) return UINT64_MAX;
        total += pw;
    }
    return total;
}

int p2o_unrank(const p2o_query *q, int max_len, uint64_t index, uint8_t *instr)
{
    uint64_t I = (uint64_t)p2o_alphabet_size(q), pw = 1;
    for (int l = 1; l <= max_len; l++) {
        pw *= I;
        if (index < pw) {
            for (int t = l - 1; t >= 0; t--) {
                int dg = (int)(index % I);
                index /= I;
                instr[t] = (uint8_t)((dg / q->n_ops) * 5 + q->ops[dg % q->n_ops]);
            }
            return l;
        }
        index -= pw;
    }
    return -1;
}

static uint64_t rank_program(const p2o_query *q, const uint8_t *instr, int len)
{
    uint64_t I = (uint64_t)p2o_alphabet_size(q), pw = 1, base = 0, v = 0;
    for (int l = 1; l < len; l++) { pw *= I; base += pw; }
    for (int t = 0; t < len; t++) {
        int pid = instr[t] / 5, op = instr[t] % 5, oi = -1;
        for (int o = 0; o < q->n_ops; o++) if (q->ops[o] == op) oi = o;
        v = v * I + (uint64_t)(pid * q->n_ops + oi);
    }
    return base + v;
}

/* ------------------------------------------------------------------ */
/* Sec. 3.2: device states and the five rules.                         */
/* state[d][r] = D-bit mask: bit j set <=> device j contributed its    */
/* original r-th chunk to what device d holds as chunk r.              */
/* ------------------------------------------------------------------ */
static inline uint64_t *cell(const p2o_query *q, uint64_t *s, int d, int r) { return s + ((size_t)d * q->k + r) * q->W; }
static inline const uint64_t *ccell(const p2o_query *q, const uint64_t *s, int d, int r) { return s + ((size_t)d * q->k + r) * q->W; }
static size_t state_words(const p2o_query *q) { return (size_t)q->D * q->k * q->W; }

static int row_nonempty(const p2o_query *q, const uint64_t *s, int d, int r)
{
    const uint64_t *c = ccell(q, s, d, r);
    for (int w = 0; w < q->W; w++) if (c[w]) return 1;
    return 0;
}
static int count_rows(const p2o_query *q, const uint64_t *s, int d)
{
    int c = 0;
    for (int r = 0; r < q->k; r++) c += row_nonempty(q, s, d, r);
    return c;
}

/* what one group adds to the cost of the step */
typedef struct { int g; int rows; int op; int active; } group_cost;

/*
 * Apply collective `op` to ONE device group (members ascending, first = root).
 * Reads `in`, writes the members' rows of `out` (out starts as a copy of in).
 * Returns 1 if the rule's premises hold, 0 otherwise.
 */
static int apply_group(const p2o_query *q, int op, const int *mem, int g,
                       const uint64_t *in, uint64_t *out, group_cost *gc)
{
    int k = q->k, W = q->W;
    gc->g = g; gc->op = op; gc->rows = 0; gc->active = 0;
    for (int p = 0; p < g; p++) if (count_rows(q, in, mem[p]) > 0) gc->active = 1;

    if (op == OP_ALLREDUCE || op == OP_REDUCESCATTER || op == OP_REDUCE) {
        /* premise: every member holds the same set of non-empty rows */
        for (int p = 1; p < g; p++)
            for (int r = 0; r < k; r++)
                if (row_nonempty(q, in, mem[p], r) != row_nonempty(q, in, mem[0], r)) return 0;
        /* premise: in every row the members' columns are pairwise disjoint */
        for (int r = 0; r < k; r++)
            for (int p = 0; p < g; p++)
                for (int p2 = p + 1; p2 < g; p2++)
                    for (int w = 0; w < W; w++)
                        if (ccell(q, in, mem[p], r)[w] & ccell(q, in, mem[p2], r)[w]) return 0;
        /* the sum of all member matrices */
        uint64_t *t = calloc((size_t)k * W, sizeof(uint64_t));
        for (int r = 0; r < k; r++)
            for (int p = 0; p < g; p++)
                for (int w = 0; w < W; w++) t[(size_t)r * W + w] |= ccell(q, in, mem[p], r)[w];
        int nrows = 0;
        for (int r = 0; r < k; r++) { int ne = 0; for (int w = 0; w < W; w++) if (t[(size_t)r * W + w]) ne = 1; nrows += ne; }
        gc->rows = nrows;
        if (op == OP_ALLREDUCE) {
            for (int p = 0; p < g; p++)
                for (int r = 0; r < k; r++) memcpy(cell(q, out, mem[p], r), t + (size_t)r * W, sizeof(uint64_t) * W);
        } else if (op == OP_REDUCE) {
            for (int p = 0; p < g; p++)
                for (int r = 0; r < k; r++) {
                    if (p == 0) memcpy(cell(q, out, mem[p], r), t + (size_t)r * W, sizeof(uint64_t) * W);
                    else memset(cell(q, out, mem[p], r), 0, sizeof(uint64_t) * W);
                }
        } else {
            /* scatter: error unless the number of chunks divides evenly; the
             * member of rank p keeps the p-th contiguous block of the non-empty
             * rows taken in ascending order */
            if (nrows % g != 0) { free(t); return 0; }
            int per = nrows / g, seen = 0;
            for (int r = 0; r < k; r++) {
                int ne = 0; for (int w = 0; w < W; w++) if (t[(size_t)r * W + w]) ne = 1;
                int owner = ne ? seen / per : -1;
                for (int p = 0; p < g; p++) {
                    if (p == owner) memcpy(cell(q, out, mem[p], r), t + (size_t)r * W, sizeof(uint64_t) * W);
                    else memset(cell(q, out, mem[p], r), 0, sizeof(uint64_t) * W);
                }
                seen += ne;
            }
        }
        free(t);
        return 1;
    }
    if (op == OP_ALLGATHER) {
        /* premise (reading): no member is empty */
        for (int p = 0; p < g; p++) if (count_rows(q, in, mem[p]) == 0) return 0;
        /* premise: the members' rows are pairwise disjoint */
        for (int r = 0; r < k; r++) {
            int holders = 0;
            for (int p = 0; p < g; p++) holders += row_nonempty(q, in, mem[p], r);
            if (holders > 1) return 0;
        }
        int total = 0;
        for (int r = 0; r < k; r++) {
            uint64_t u[MAXW];
            memset(u, 0, sizeof u);
            for (int p = 0; p < g; p++) for (int w = 0; w < W; w++) u[w] |= ccell(q, in, mem[p], r)[w];
            int ne = 0; for (int w = 0; w < W; w++) if (u[w]) ne = 1;
            total += ne;
            for (int p = 0; p < g; p++) memcpy(cell(q, out, mem[p], r), u, sizeof(uint64_t) * W);
        }
        gc->rows = total;            /* rows held after the gather */
        return 1;
    }
    if (op == OP_BROADCAST) {
        /* premise: the root's data is at least as informative as every member's ... */
        int strictly = 0;
        for (int p = 1; p < g; p++)
            for (int r = 0; r < k; r++)
                for (int w = 0; w < W; w++) {
                    uint64_t a = ccell(q, in, mem[0], r)[w], b = ccell(q, in, mem[p], r)[w];
                    if (b & ~a) return 0;
                    if (a != b) strictly = 1;
                }
        /* ... and more informative than at least one */
        if (!strictly) return 0;
        gc->rows = count_rows(q, in, mem[0]);
        for (int p = 1; p < g; p++)
            for (int r = 0; r < k; r++) memcpy(cell(q, out, mem[p], r), ccell(q, in, mem[0], r), sizeof(uint64_t) * W);
        return 1;
    }
    return 0;
}

/*
 * Cost of one step (ring algorithm, alpha-beta; a stated reading, the paper
 * gives only the simulator's bandwidth inputs in Sec. 5):
 *   a group of g devices, each holding n bytes = msg * rows / k, needs
 *     AllReduce      2(g-1) ring steps, 2(g-1)/g * n bytes through each member link
 *     ReduceScatter   (g-1) steps,       (g-1)/g * n
 *     AllGather       (g-1) steps,       (g-1)/g * n_out   (n_out: bytes held afterwards)
 *     Reduce          (g-1) steps,        n                (pipelined chain)
 *     Broadcast       (g-1) steps,        n
 *   latency  : T_alpha = max over groups of steps * alpha[level at which the group's
 *              members first differ, outermost first]
 *   bandwidth: every hardware unit (a prefix c_0..c_j of coordinates) owns one uplink
 *              of bw[j]; a group that has members inside and outside the unit sends
 *              its bytes through that uplink once; T_beta = max over units of
 *              (sum of such bytes) / bw[j]
 *   step time = T_alpha + T_beta.  Groups whose members are all empty cost nothing.
 *
 * Tree model (algo 1; Sec. 4 runs the library's ring and tree algorithms, the tree being the
 * two-tree scheme of its reference, which that library uses for AllReduce only; again a stated
 * reading, the paper prints no formula): an AllReduce goes up a binary tree and down again,
 *     AllReduce      2 * ceil(log2 g) steps, 2 * n bytes through each member link
 * (every device is an inner node of one of the two trees and a leaf of the other, so it forwards
 * the whole message once per phase); the other collectives keep their ring figures.
 */
static int ceil_log2(int g)
{
    int l = 0;
    while ((1 << l) < g) l++;
    return l;
}

static double step_cost(const p2o_query *q, const p2o_pattern *pt, const group_cost *gcs, double msg)
{
    int n = q->n, D = q->D;
    double t_alpha = 0.0, t_beta = 0.0;
    double *load = calloc((size_t)n * D, sizeof(double));
    for (int G = 0; G < pt->n_groups; G++) {
        const group_cost *gc = &gcs[G];
        if (!gc->active) continue;
        const int *mem = pt->members + pt->gstart[G];
        int g = gc->g;
        double nbytes = msg * (double)gc->rows / (double)q->k;
        double steps, bytes;
        switch (gc->op) {
        case OP_ALLREDUCE:
            if (q->algo == 1) { steps = 2.0 * ceil_log2(g); bytes = 2.0 * nbytes; }
            else              { steps = 2.0 * (g - 1);      bytes = 2.0 * (g - 1) / g * nbytes; }
            break;
        case OP_REDUCESCATTER: steps = (g - 1);       bytes = (double)(g - 1) / g * nbytes; break;
        case OP_ALLGATHER:     steps = (g - 1);       bytes = (double)(g - 1) / g * nbytes; break;
        default:               steps = (g - 1);       bytes = nbytes; break;
        }
        int span = n;                       /* outermost level at which two members differ */
        for (int p = 1; p < g; p++)
            for (int j = 0; j < n; j++)
                if (q->coord[mem[p]][j] != q->coord[mem[0]][j]) { if (j < span) span = j; break; }
        if (span < n && steps * q->alpha[span] > t_alpha) t_alpha = steps * q->alpha[span];
        /* units the group straddles */
        int below = D;                      /* devices per unit at level j */
        for (int j = 0; j < n; j++) {
            below /= q->h[j];
            int nunits = D / below;
            for (int u = 0; u < nunits; u++) {
                int inside = 0;
                for (int p = 0; p < g; p++) if (mem[p] / below == u) inside++;
                if (inside > 0 && inside < g) load[(size_t)j * D + u] += bytes;
            }
        }
    }
    int below = D;
    for (int j = 0; j < n; j++) {
        below /= q->h[j];
        for (int u = 0; u < D / below; u++) {
            double tt = load[(size_t)j * D + u] / q->bw[j];
            if (tt > t_beta) t_beta = tt;
        }
    }
    free(load);
    return t_alpha + t_beta;
}

/*
 * One instruction (Sec. 3.3): apply the collective to every group of the
 * pattern; devices outside every group keep their state.  The instruction is
 * rejected if any group's rule fails, or if it leaves the whole state context
 * unchanged (every operation must increase information, Sec. 4.2 Result 2).
 * step_costs[i] (if not NULL) gets the step time for message size msg[i].
 */
static int apply_instruction(const p2o_query *q, int pid, int op, const uint64_t *in, uint64_t *out,
                             int n_msg, const double *msg, double *step_costs)
{
    const p2o_pattern *pt = &q->pat[pid];
    size_t words = state_words(q);
    memcpy(out, in, words * sizeof(uint64_t));
    group_cost *gcs = malloc(sizeof(group_cost) * (pt->n_groups > 0 ? pt->n_groups : 1));
    for (int G = 0; G < pt->n_groups; G++) {
        if (!apply_group(q, op, pt->members + pt->gstart[G], pt->gsize[G], in, out, &gcs[G])) { free(gcs); return 0; }
    }
    if (memcmp(in, out, words * sizeof(uint64_t)) == 0) { free(gcs); return 0; }
    if (step_costs) for (int i = 0; i < n_msg; i++) step_costs[i] = step_cost(q, pt, gcs, msg[i]);
    free(gcs);
    return 1;
}

static void init_state(const p2o_query *q, uint64_t *s)
{
    /* Sec. 3.5: device i has 1 in column i of every row */
    memset(s, 0, state_words(q) * sizeof(uint64_t));
    for (int d = 0; d < q->D; d++)
        for (int r = 0; r < q->k; r++) cell(q, s, d, r)[d / 64] |= 1ull << (d % 64);
}

static int is_goal(const p2o_query *q, const uint64_t *s)
{
    for (int d = 0; d < q->D; d++)
        for (int r = 0; r < q->k; r++)
            if (memcmp(ccell(q, s, d, r), q->goal + (size_t)d * q->W, sizeof(uint64_t) * q->W)) return 0;
    return 1;
}

/*
 * Evaluate one program from the init state.  Returns 1 if every step is valid
 * and the final state is the goal, else 0; *steps_run gets the number of
 * instructions applied (including a failing one).  cost[i] = sum of step times
 * for msg[i], added left to right (only meaningful when the result is 1).
 */
int p2o_eval_program(const p2o_query *q, const uint8_t *instr, int len, int n_msg, const double *msg,
                     double *cost, int32_t *steps_run)
{
    size_t words = state_words(q);
    uint64_t *a = malloc(words * sizeof(uint64_t)), *b = malloc(words * sizeof(uint64_t));
    double sc[64];
    if (n_msg > 64) n_msg = 64;
    for (int i = 0; i < n_msg; i++) cost[i] = 0.0;
    init_state(q, a);
    int ok = 1, ran = 0;
    for (int t = 0; t < len && ok; t++) {
        int pid = instr[t] / 5, op = instr[t] % 5;
        ran++;
        if (pid >= q->n_patterns || !(q->op_mask & (1u << op))) { ok = 0; break; }
        ok = apply_instruction(q, pid, op, a, b, n_msg, msg, n_msg > 0 ? sc : NULL);
        if (ok) { for (int i = 0; i < n_msg; i++) cost[i] += sc[i]; uint64_t *tmp = a; a = b; b = tmp; }
    }
    if (ok) ok = is_goal(q, a);
    if (steps_run) *steps_run = ran;
    free(a); free(b);
    return ok;
}

/* Flat, unpruned evaluation of candidate indices (every candidate from the init
 * state).  indices == NULL means start, start+1, ...  Returns the number valid;
 * valid[i] (if not NULL) gets 0/1, *total_steps the instructions applied. */
int64_t p2o_eval_indices(const p2o_query *q, int max_len, const uint64_t *indices, uint64_t start, int64_t count,
                         uint8_t *valid, int64_t *total_steps, int n_threads)
{
    int64_t nvalid = 0, steps = 0;
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : nvalid, steps) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int64_t i = 0; i < count; i++) {
        uint8_t instr[MAXLEN];
        uint64_t idx = indices ? indices[i] : start + (uint64_t)i;
        int len = p2o_unrank(q, max_len, idx, instr);
        int32_t ran = 0;
        int ok = len > 0 ? p2o_eval_program(q, instr, len, 0, NULL, NULL, &ran) : 0;
        if (valid) valid[i] = (uint8_t)ok;
        nvalid += ok;
        steps += ran;
    }
    if (total_steps) *total_steps = steps;
    return nvalid;
}

/* ------------------------------------------------------------------ */
/* Sec. 3.5: enumerate programs by increasing size; a prefix whose     */
/* step violates a rule is not extended (its extensions are invalid by */
/* definition).  Programs that end in the goal state are the result.   */
/* ------------------------------------------------------------------ */
typedef struct {
    const p2o_query *q;
    int max_len, n_msg;
    const double *msg;
    uint64_t **st;        /* state after t instructions */
    uint8_t instr[MAXLEN];
    double cost[MAXLEN + 1][64];
    uint64_t *out_index; uint8_t *out_len; uint8_t *out_instr; double *out_cost;
    int64_t cap, count;
    int64_t steps_tried;
} synth_ctx;

static void synth_rec(synth_ctx *c, int depth)
{
    const p2o_query *q = c->q;
    if (depth > 0 && is_goal(q, c->st[depth])) {
        if (c->count < c->cap) {
            c->out_index[c->count] = rank_program(q, c->instr, depth);
            c->out_len[c->count] = (uint8_t)depth;
            memset(c->out_instr + c->count * MAXLEN, 0, MAXLEN);
            memcpy(c->out_instr + c->count * MAXLEN, c->instr, depth);
            for (int i = 0; i < c->n_msg; i++) c->out_cost[c->count * c->n_msg + i] = c->cost[depth][i];
        }
        c->count++;
    }
    if (depth == c->max_len) return;
    for (int pid = 0; pid < q->n_patterns; pid++)
        for (int oi = 0; oi < q->n_ops; oi++) {
            double sc[64];
            c->steps_tried++;
            if (!apply_instruction(q, pid, q->ops[oi], c->st[depth], c->st[depth + 1], c->n_msg, c->msg, sc)) continue;
            c->instr[depth] = (uint8_t)(pid * 5 + q->ops[oi]);
            for (int i = 0; i < c->n_msg; i++) c->cost[depth + 1][i] = c->cost[depth][i] + sc[i];
            synth_rec(c, depth + 1);
        }
}

typedef struct { uint64_t index; int64_t pos; } idx_pos;
static int cmp_idx(const void *a, const void *b)
{
    uint64_t x = ((const idx_pos *)a)->index, y = ((const idx_pos *)b)->index;
    return x < y ? -1 : x > y;
}

/* Returns the number of valid programs (may exceed cap; then only the first cap
 * found are stored, unsorted).  Output sorted by ascending candidate index. */
int64_t p2o_synthesize(const p2o_query *q, int max_len, int n_msg, const double *msg,
                       uint64_t *out_index, uint8_t *out_len, uint8_t *out_instr /* [cap][8] */,
                       double *out_cost /* [cap][n_msg] */, int64_t cap, int64_t *steps_tried)
{
    if (max_len < 1 || max_len > MAXLEN || n_msg > 64) return -1;
    synth_ctx c;
    memset(&c, 0, sizeof c);
    c.q = q; c.max_len = max_len; c.n_msg = n_msg; c.msg = msg;
    c.out_index = out_index; c.out_len = out_len; c.out_instr = out_instr; c.out_cost = out_cost; c.cap = cap;
    c.st = malloc(sizeof(uint64_t *) * (max_len + 1));
    for (int t = 0; t <= max_len; t++) c.st[t] = malloc(state_words(q) * sizeof(uint64_t));
    init_state(q, c.st[0]);
    synth_rec(&c, 0);
    for (int t = 0; t <= max_len; t++) free(c.st[t]);
    free(c.st);
    if (steps_tried) *steps_tried = c.steps_tried;
    int64_t n = c.count < cap ? c.count : cap;
    if (c.count <= cap && n > 1) {
        /* sort the records by candidate index */
        idx_pos *ord = malloc(sizeof(idx_pos) * n);
        for (int64_t i = 0; i < n; i++) { ord[i].index = out_index[i]; ord[i].pos = i; }
        qsort(ord, n, sizeof(idx_pos), cmp_idx);
        uint64_t *ti = malloc(sizeof(uint64_t) * n); uint8_t *tl = malloc(n); uint8_t *tp = malloc(n * MAXLEN);
        double *tc = malloc(sizeof(double) * n * (n_msg > 0 ? n_msg : 1));
        for (int64_t i = 0; i < n; i++) {
            int64_t s = ord[i].pos;
            ti[i] = out_index[s]; tl[i] = out_len[s]; memcpy(tp + i * MAXLEN, out_instr + s * MAXLEN, MAXLEN);
            for (int j = 0; j < n_msg; j++) tc[i * n_msg + j] = out_cost[s * n_msg + j];
        }
        memcpy(out_index, ti, sizeof(uint64_t) * n); memcpy(out_len, tl, n); memcpy(out_instr, tp, n * MAXLEN);
        if (n_msg > 0) memcpy(out_cost, tc, sizeof(double) * n * n_msg);
        free(ord); free(ti); free(tl); free(tp); free(tc);
    }
    return c.count;
}

/* ------------------------------------------------------------------ */
/* Raw access to the rules for hand-worked examples: apply one         */
/* collective to an explicit group of a D-device, k-row system whose   */
/* state is given as booleans state[d][r][j].  Returns 1/0; on 1 the   */
/* state is updated in place.                                          */
/* ------------------------------------------------------------------ */
int p2o_apply_collective_raw(int D, int k, uint8_t *state, int op, const int32_t *members, int g)
{
    if (D < 1 || D > MAXD || k < 1 || g < 1) return -1;
    p2o_query q;
    memset(&q, 0, sizeof q);
    q.D = D; q.k = k; q.W = (D + 63) / 64;
    size_t words = state_words(&q);
    uint64_t *in = calloc(words, sizeof(uint64_t)), *out = malloc(words * sizeof(uint64_t));
    for (int d = 0; d < D; d++)
        for (int r = 0; r < k; r++)
            for (int j = 0; j < D; j++)
                if (state[((size_t)d * k + r) * D + j]) cell(&q, in, d, r)[j / 64] |= 1ull << (j % 64);
    memcpy(out, in, words * sizeof(uint64_t));
    int mem[MAXD];
    for (int p = 0; p < g; p++) mem[p] = members[p];
    group_cost gc;
    int ok = apply_group(&q, op, mem, g, in, out, &gc);
    if (ok)
        for (int d = 0; d < D; d++)
            for (int r = 0; r < k; r++)
                for (int j = 0; j < D; j++)
                    state[((size_t)d * k + r) * D + j] = (uint8_t)((ccell(&q, out, d, r)[j / 64] >> (j % 64)) & 1);
    free(in); free(out);
    return ok;
}

/* Run a program and hand back the final state as booleans [D][k][D] (for
 * invariants such as "RS;AG leaves the same state as AR").  Returns the number
 * of instructions that were valid (== len if all were). */
int p2o_run_program_state(const p2o_query *q, const uint8_t *instr, int len, uint8_t *state_out, int32_t *reached_goal)
{
    size_t words = state_words(q);
    uint64_t *a = malloc(words * sizeof(uint64_t)), *b = malloc(words * sizeof(uint64_t));
    init_state(q, a);
    int t = 0;
    for (; t < len; t++) {
        int pid = instr[t] / 5, op = instr[t] % 5;
        if (pid >= q->n_patterns) break;
        if (!apply_instruction(q, pid, op, a, b, 0, NULL, NULL)) break;
        uint64_t *tmp = a; a = b; b = tmp;
    }
    if (reached_goal) *reached_goal = is_goal(q, a);
    if (state_out)
        for (int d = 0; d < q->D; d++)
            for (int r = 0; r < q->k; r++)
                for (int j = 0; j < q->D; j++)
                    state_out[((size_t)d * q->k + r) * q->D + j] = (uint8_t)((ccell(q, a, d, r)[j / 64] >> (j % 64)) & 1);
    free(a); free(b);
    return t;
}

/* ------------------------------------------------------------------ */
/* Top-k: positions of the k smallest (cost, index) pairs, ascending   */
/* cost, ties by ascending index.  Full sort.                          */
/* ------------------------------------------------------------------ */
typedef struct { double cost; uint64_t index; int64_t pos; } ck;
static int cmp_ck(const void *a, const void *b)
{
    const ck *x = a, *y = b;
    if (x->cost < y->cost) return -1;
    if (x->cost > y->cost) return 1;
    if (x->index < y->index) return -1;
    if (x->index > y->index) return 1;
    return x->pos < y->pos ? -1 : x->pos > y->pos;
}
int64_t p2o_topk(const double *cost, const uint64_t *index, int64_t n, int k, int64_t *out_pos)
{
    if (n < 0 || k < 0) return -1;
    for (int64_t i = 0; i < n; i++) if (cost[i] != cost[i]) return -1;   /* NaN */
    ck *a = malloc(sizeof(ck) * (n > 0 ? n : 1));
    for (int64_t i = 0; i < n; i++) { a[i].cost = cost[i]; a[i].index = index[i]; a[i].pos = i; }
    qsort(a, n, sizeof(ck), cmp_ck);
    int64_t kk = k < n ? k : n;
    for (int64_t i = 0; i < kk; i++) out_pos[i] = a[i].pos;
    free(a);
    return kk;
}
