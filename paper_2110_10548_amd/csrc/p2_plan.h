// Host-side planning of one query: from (hierarchy, axes, placement, reduce axes) to the
// tables the kernels read.  Plain C++, no device code.
//
// The kernels never see the full system.  Lowering applies a pattern of the reduction-axis
// hierarchy to every combination of non-reduction coordinates (Sec. 3.4), so the system is
// D/R identical copies ("replicas") of one reduction group of R devices, and a program is
// valid on the system iff it is valid on one copy.  Devices of a copy are numbered by their
// "local id": the mixed-radix number of their reduction-axis digits, outermost hardware level
// first; inside a copy that order equals the order of device ids.  A pattern then is
// (g, s, master): its groups are the arithmetic progressions {base + t*s : t < g}, and with
// `master` only those whose base has zero digits below the varied levels take part.
// Only the cost needs the full system: how many groups share the uplink of a hardware unit.
//
// The other synthesis hierarchies of Sec. 3.4 (the system's own levels, the column-based and the
// row-based factors, the reduction axes' factors before they are collapsed) fit the same tables: a
// level owns some factors x[i][j] of the matrix, the local id is the mixed-radix number of a device's
// digits level by level, and the factors that belong to no level number the copies.  Two things are
// then no longer implied: the members of a group in ascending local id need not be in ascending
// device id (a ReduceScatter hands block p to the member of *rank* p, so a pattern carries its
// ranks), and where a hierarchy has levels over non-reduction axes a copy is the whole system and a
// device's goal is the set of local ids of its own reduction group.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/p2.h"

namespace p2 {

struct Pattern {
    int slice, form, form_level;   // first (slice, form) pair that produced this group set
    int lo, hi;                    // varied synthesis levels lo..hi (both with factor > 1); for
                                   // hierarchy (d) these are the hardware levels
    int span;                      // outermost hardware level at which members of a group differ
    int g, s;                      // group size, stride of local ids inside a group
    int master;                    // 1: only groups with (local id % s) == 0 take part
    int n_groups;                  // participating groups inside one reduction group
    std::vector<int32_t> rank;     // [g] rank by device id of the member with the t-th local id; empty: t
    // sparse rows for the bandwidth term: for hardware unit classes that can carry the
    // maximum load, (local group, number of system groups touching the unit) pairs
    std::vector<int32_t> row_ptr;      // [n_rows + 1]
    std::vector<int32_t> row_level;    // [n_rows] hardware level of the unit
    std::vector<uint32_t> entries;     // entry_pack(local group, its first device, count)
};

struct Plan {
    int n = 0, m = 0;
    int h[P2_MAX_LEVELS] = {0};
    double bw[P2_MAX_LEVELS] = {0}, alpha[P2_MAX_LEVELS] = {0};
    int x[P2_MAX_AXES][P2_MAX_LEVELS] = {{0}};
    bool is_reduce[P2_MAX_AXES] = {false};
    int D = 0, R = 0, k = 0;
    int f[P2_MAX_LEVELS] = {0};        // reduction-axis factor of each hardware level (collapsed)
    int hierarchy = 0;                 // P2_HIERARCHY_*
    std::vector<int> level_f;          // hierarchy != collapsed: factor of each synthesis level
    std::vector<uint32_t> goal;        // [R][ceil(R/32)] goal mask of each local id; empty: all of the copy
    uint32_t form_mask = 7, op_mask = 31;
    int algo = 0;                  // cost model of AllReduce: 0 ring, 1 tree
    int frontier_pairs = 0;        // P2_FRONTIER_PAIRS_*
    int max_row_classes = 64;      // limit of the literal kernels' state by classes of equal rows (1..64)
    int n_ops = 0, ops[5] = {0};
    std::vector<Pattern> patterns;
    int alphabet = 0;
    int max_len = 0;
    uint64_t n_candidates = 0;
    uint64_t base[P2_MAX_LEN + 2] = {0};   // base[l] = index of the first program of length l
    std::vector<int32_t> local_of;         // [D] local id of a device inside its reduction group
    std::vector<int32_t> replica_of;       // [D] which copy the device belongs to
};

// Returns P2_OK or an error code; `err` gets the reason.  with_cost: the links must be given, and the
// bandwidth rows are built (unless build_rows is false: build_cost_tables does that later).
int32_t enumerate_placements(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, int32_t* out, int64_t cap,
                             int64_t* out_count, std::string& err);
int32_t make_plan(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* placement,
                  const int32_t* reduce_axes, int32_t n_reduce, int32_t max_len, const p2_options* opt, bool with_cost,
                  Plan& plan, std::string& err, bool build_rows = true);
// The bandwidth rows of every pattern of a plan made without them (make_plan with with_cost = false).
void build_cost_tables(Plan& plan);
// Group id / rank of every device of the full system for one canonical pattern.
void describe_pattern(const Plan& plan, int pattern_id, int32_t* group_of_device, int32_t* rank_in_group);

}  // namespace p2
