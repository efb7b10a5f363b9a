// Structures shared by the host API and the kernels, and the launch entry points.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/p2.h"
#include "p2_device_pack.h"

namespace p2 {

constexpr int kMaxPatterns = 64;
constexpr int kMaxMsg = 64;        // message sizes per call (one wavefront lane each)
constexpr int kMaxTopK = 1024;

enum : int { OP_AR = 0, OP_RS = 1, OP_AG = 2, OP_RD = 3, OP_BC = 4 };

// Words per device mask in the literal state's kernels (their MW template argument): ceil(R/32) rounded up
// to a power of two.
inline int literal_mask_words(int R) { return R <= 32 ? 1 : R <= 64 ? 2 : R <= 128 ? 4 : R <= 256 ? 8 : 16; }

// One canonical pattern inside a reduction group of R devices numbered by local id: group G is
// {base(G) + t*s : t < g}; with master only bases whose (id % s) == 0 exist.
struct DevPattern {
    int32_t g, s, master, n_groups;
    int32_t span_level;            // outermost hardware level at which members differ
    int32_t rank_off;              // 0: the member with the t-th local id has rank t; else its rank is
                                   // DevQuery::rank_tbl[rank_off - 1 + t] (literal engine only)
    int32_t pad1;
    int32_t reg_shape;             // shape number of the register engine (p2_regs.hip), -1 if it has none
};

// A run of equally long candidates of one query: blocks [first_block, next segment's first_block)
// take `iters` x 64 consecutive candidates each, starting at candidate index first_index.
struct DevSegment {
    uint32_t first_block;
    int32_t query;
    int32_t len;
    int32_t iters;
    unsigned long long first_index;
    unsigned long long count;
};

// Shared-prefix kernel: the grid blocks [first_block, first_block + n_blocks) serve the work items
// [first_item, first_item + n_items) of one query (item numbers are the first_block numbers of its segments).
struct DevShare {
    uint32_t first_block, n_blocks;
    uint32_t first_item, n_items;
    int32_t query;                 // the query, and its segments [first_seg, first_seg + n_segs) of the launch's table
    int32_t first_seg, n_segs;
    int32_t cut_log;               // a stem of a segment with len >= 2 is 2^cut_log items of seg.iters groups each
};

// Work of the kernels that run after the evaluation (ordering, costing, literal re-runs), which
// serve all queries of a batch in one launch: blocks [first_block, next first_block) handle
// `count` list entries of one query, `per_block` each, read at in_off and written at out_off
// (element offsets into the batch-wide buffers).
struct DevPostSeg {
    uint32_t first_block;
    int32_t query;
    uint32_t count;
    uint32_t per_block;
    unsigned long long in_off;
    unsigned long long out_off;
};
__device__ inline DevPostSeg find_post_seg(const DevPostSeg* __restrict__ segs, int n_segs, uint32_t block) {
    int a = 0, b = n_segs - 1;
    while (a < b) {
        const int mid = (a + b + 1) >> 1;
        if (segs[mid].first_block <= block) a = mid; else b = mid - 1;
    }
    return segs[a];
}

// Entries of rerun_idx written by the shared-prefix engine: the index of a group's first candidate, or,
// with kStemEntry set, of the first candidate of the first of `count` consecutive groups under one
// stem whose own state left the compact form (count in bits 52..62; candidate indices stay below 2^52).
constexpr unsigned long long kStemEntry = 1ull << 63;
constexpr int kStemCountShift = 52;
constexpr unsigned long long kEntryIndexMask = (1ull << kStemCountShift) - 1ull;

// Counters a query's kernels add to.
constexpr int kCounterStripes = 64;   // blocks add to stripe (blockIdx % 64): same-address atomics serialise
struct DevCounters {
    uint32_t n_valid;              // entries appended to valid_idx (may exceed valid_cap)
    uint32_t n_rerun;              // entries appended to rerun_idx (compact engine gave up)
    uint32_t nan_seen;
    uint32_t next_unit;            // work counter of the device-driven literal launch whose first query this is
    uint32_t n_rerun_groups;       // shared-prefix engine: groups behind the rerun_idx entries (a stem entry stands for several)
    uint32_t pad[3];
    unsigned long long steps[kCounterStripes];     // instructions applied
    unsigned long long members[kCounterStripes];   // devices taking part in those instructions, summed
    unsigned long long evaluated[kCounterStripes];           // instruction applications carried out, where they differ from `steps`
    unsigned long long evaluated_members[kCounterStripes];   // devices taking part in those, summed
};

// Latency steps and bytes through each member's link (as a multiple of the bytes a member holds) of one
// collective on a group of g devices.  Ring figures; with algo = 1 an AllReduce instead goes up and down a
// binary tree (2 ceil(log2 g) steps) and every device forwards the whole message once per phase (2 n).
__host__ __device__ inline void step_factors(int op, int g, int algo, double& steps, double& mult) {
    const double gm1 = (double)(g - 1);
    if (op == OP_AR) {
        if (algo == 1) {
            int l = 0;
            while ((1 << l) < g) ++l;
            steps = 2.0 * (double)l; mult = 2.0;
        } else {
            steps = 2.0 * gm1; mult = 2.0 * gm1 / (double)g;
        }
    } else {
        steps = gm1;
        mult = (op == OP_RS || op == OP_AG) ? gm1 / (double)g : 1.0;
    }
}

// Bandwidth rows of one query (cost model): CSR of packed (local group, first device, multiplicity)
// entries; pattern p owns the rows [pat_begin[p], pat_begin[p + 1]).  Uploaded apart from the query
// descriptors (the host builds the rows while the evaluation kernels run); only the cost kernels read it.
struct DevRows {
    const int32_t* row_ptr;
    const int32_t* row_level;      // hardware level of the row's unit
    const uint32_t* entries;       // entry_pack(local group, its first device, groups touching the unit)
    int32_t pat_begin[kMaxPatterns + 1];
    int32_t pad;
    // per pattern and hardware level the largest sum of multiplicities over the level's rows: where every group
    // of the pattern holds the same number of rows c, the busiest unit of a level carries c times this
    uint32_t level_max[kMaxPatterns][P2_MAX_LEVELS];
};

struct DevQuery {
    int32_t R, k;                  // devices of one reduction group, chunks
    int32_t MW, KW;                // 32-bit words per contribution mask / per chunk set
    int32_t n_patterns, n_ops, alphabet, max_len;
    int32_t n_levels, n_msg;
    int32_t algo, pad0;            // cost model of AllReduce: 0 ring, 1 tree
    unsigned long long n_candidates;
    unsigned long long base[P2_MAX_LEN + 2];   // base[l]: index of the first program of length l
    uint8_t ops[8];
    uint32_t magic_alphabet;       // ceil(2^32 / alphabet): v / alphabet == umulhi(v, magic) for v < 2^23
    uint16_t instr_of_digit[kMaxPatterns * 5];   // digit -> (pattern id << 3) | op
    DevPattern pat[kMaxPatterns];
    // small-group engines: per pattern, shape (log2 g | log2 s << 4 | master << 8) | participating devices << 16,
    // the bit set of participating devices, and the participating devices summed over the alphabet
    uint32_t reg_shape[kMaxPatterns];
    unsigned long long reg_part[kMaxPatterns];
    uint32_t reg_sum_part;
    double alpha[P2_MAX_LEVELS], inv_bw[P2_MAX_LEVELS];
    const DevRows* rows;           // bandwidth rows (valid by the time a cost kernel runs)
    const double* msg_bytes;       // [n_msg]
    // synthesis hierarchies other than the collapsed one (literal engine only)
    const uint32_t* goal_mask;     // [R][literal_mask_words(R)] goal of each device; nullptr: every device of the group
    const int32_t* rank_tbl;       // ranks of the patterns with rank_off != 0
    // outputs of the evaluation kernels
    unsigned long long* valid_idx;
    unsigned long long* rerun_idx;
    uint32_t valid_cap, rerun_cap;
    DevCounters* counters;
};

// LDS bytes one wavefront of the literal engine needs for a query (0 = does not fit; the state
// then lives in a global buffer of literal_scratch_bytes, split over *blocks blocks).
size_t literal_lds_bytes(int R, int k);
size_t literal_scratch_bytes(int R, int k, unsigned* blocks);
// Same for the literal frontier kernel, which keeps row-class tables beside the state.
size_t front_literal_lds_bytes(int R, int k);

// Evaluate candidates [start, start + count) of query *q (device pointer), or, if list != nullptr,
// the `count` candidate indices stored at list (device pointer; count may also be read from
// *list_count when list_count != nullptr).  Valid ones are appended to q->valid_idx.
hipError_t launch_eval_literal(const DevQuery* q, int R, int k, unsigned long long start, unsigned long long count,
                               const unsigned long long* list, const uint32_t* list_count, void* gscratch,
                               hipStream_t stream);
// Compact engine: one launch over the segments of many queries (all with R <= max_R, k <= max_k).
hipError_t launch_eval_compact(const DevQuery* queries, const DevSegment* segs, int n_segs, unsigned total_blocks,
                               int max_R, int max_k, hipStream_t stream);
// Engines for patterns with power-of-two group size and stride: shape word of a pattern
// (log2 g | log2 s << 4 | master << 8) or -1 if its group bits do not fit in max_bits (5: the
// per-candidate engine for R <= 32, k <= 32; 6: the shared-prefix engine for R <= 64), and the launch
// of the per-candidate engine over the segments of many queries (64 candidates per wavefront).
int reg_shape_of(int g, int s, int master, int max_bits);
hipError_t launch_eval_regs(const DevQuery* queries, const DevSegment* segs, int n_segs, unsigned total_blocks,
                            hipStream_t stream);
// Shared-prefix engine: `grid` blocks, divided among the queries by the share table.
hipError_t launch_eval_shared(const DevQuery* queries, const DevSegment* segs, int n_segs, const DevShare* shares,
                              int n_shares, unsigned grid, int max_R, int max_k, hipStream_t stream);
// Ordering, program records and costs of the valid candidates of shared-prefix-capable queries, one block per
// entry of the unordered lists (in_off of a segment: where its list starts in valid, or, with bit 63 set, in
// valid2): the block finds its entry's rank and writes sorted, progs and costs at out_off + rank.
hipError_t launch_cost_shared(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks, int max_R,
                              int max_k, const unsigned long long* valid, const unsigned long long* valid2,
                              unsigned long long* sorted, p2_program* progs, double* costs, hipStream_t stream);
// Best rate, in lane-operations per second, of a stream of independent 32-bit vector ALU instructions.
hipError_t measure_alu_peak(int reps, double* lane_ops_per_s, hipStream_t stream);
hipError_t measure_lds_peak(int reps, double* bytes_per_s, hipStream_t stream);
// Candidates per wavefront the compact engine can keep in LDS for this state size (0 = none).
int compact_lanes(int R, int k);
// Per segment: sorted[out_off + i] = i-th smallest of valid[in_off .. in_off + count)  (distinct keys).
// per_block must be 256.
// A segment whose in_off has bit 63 set reads from valid2 (the frontier engine's lists) instead.
hipError_t launch_rank_sort(const unsigned long long* valid, const unsigned long long* valid2, unsigned long long* sorted,
                            const DevPostSeg* segs, int n_segs, unsigned blocks, hipStream_t stream);
// Literal evaluation of listed candidates (one per block): list[in_off + i], i < count, of each segment's query.
// The queries of a launch have the mask width of max_R; lds_bytes = the largest literal_lds_bytes(R, k) among
// them (each fits on its own; the largest R and the largest k together need not).
hipError_t launch_eval_literal_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                    int max_R, size_t lds_bytes, const unsigned long long* list, hipStream_t stream);
// Groups handed over by the shared-prefix engine (list entries = index of a group's first candidate), for
// the queries qlist[0 .. n_q) (device array of query numbers): counts and lists are read on the device from
// each query's counters, so the launch can be queued right behind the evaluation kernel.  States that fit
// in LDS (front_literal_lds_bytes of max_R, max_k) use 4096 blocks; otherwise the blocks of
// literal_group_scratch_bytes, each with a slice of gscratch.
size_t literal_group_scratch_bytes(int max_R, int max_k, unsigned* blocks);
// gscratch (literal_group_scratch_bytes) is needed in both cases: a stem entry keeps a copy of the stem's state there.
// class_cap as for launch_front_classify_literal.
hipError_t launch_eval_literal_groups_auto(const DevQuery* queries, const int32_t* qlist, int n_q, int max_R, int max_k,
                                           void* gscratch, int class_cap, hipStream_t stream);
// Program records and costs of the sorted valid candidates at out_off + i of each segment.
// The same for states of which only a few fit in LDS (cost_wide_applies): one wavefront per program.
bool cost_wide_applies(int max_R, int max_k);
hipError_t launch_cost_wide_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                 int max_R, int max_k, const unsigned long long* sorted, p2_program* progs,
                                 double* costs, hipStream_t stream);
hipError_t launch_cost_compact_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                    int max_R, int max_k, const unsigned long long* sorted, p2_program* progs,
                                    double* costs, hipStream_t stream);
hipError_t launch_cost_literal_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                    int max_R, size_t lds_bytes, const unsigned long long* sorted, p2_program* progs,
                                    double* costs, int only_missing, hipStream_t stream);
// For each of the n sorted valid candidates: its program record and its cost for every message size.
hipError_t launch_cost(const DevQuery* q, int R, int k, int engine, const unsigned long long* sorted, uint32_t n,
                       p2_program* out_prog, double* out_cost, hipStream_t stream);
// ---- frontier evaluation (p2_frontier.hip, p2_literal.hip) -------------------------------------
// A prefix of the frontier: instruction digit t at bits [9t, 9t + 9) of `digits`.
struct FrontEntry {
    uint32_t query;
    uint32_t len;
    unsigned long long digits;
};
// A valid extension of a prefix: code 1 = prefix whose devices hold one (chunk set, mask) pair each, 4 = prefix
// with a device that holds two, 2 = goal, 3 = prefix whose state only the literal engine can hold; bit 8 set:
// `entry` counts in the two-pair list.
struct FrontSurvivor {
    uint32_t entry;
    uint16_t digit;
    uint16_t code;
    uint32_t slot;                 // pair kernels: the child's place in the next frontier list of its kind, or the
                                   // goal's place among this level's goals
};
struct FrontCounters {
    // reset before every level
    unsigned long long surv_goal;  // low half: survivors the pair kernels appended; high half: goals among them
    unsigned long long pref_pref2; // low half: one-pair children; high half: two-pair children
    uint32_t n_surv_literal;       // survivors appended by the literal classify kernels
    uint32_t n_goal;               // goals among those
    uint32_t n_prefix_literal;     // literal children (of any kernel)
    uint32_t next_literal;         // entries written to the next literal list
    uint32_t next_unit;            // work counter of the device-driven literal launch whose first query this is
    uint32_t n_overflow;           // literal prefixes left to the full-state kernel
    uint32_t n_unknown;            // two-pair prefixes handed to the literal kernels
    uint32_t next_goal_literal;    // goals of literal prefixes written so far
    uint32_t t_count[3];           // children of the judged states, by kind: one-pair states, two-pair states, goals
    uint32_t t_next[3];            // ... places handed out so far
    uint32_t n_ssurv;              // ... entries of their list
    uint32_t n_walked_planes;      // planes of the states whose patterns the classification walked (the last level skips
                                   // the states from which no instruction can end at the goal)
    uint32_t n_walk[2];            // the last level: states of the one-pair / two-pair list left to the classification
    // running totals of the enumeration
    unsigned long long steps, members;
    // distinct states found among the entries of the one-pair / two-pair list (cleared before each level's search)
    uint32_t n_reps[2];
};
// One level of one enumeration.  A level has two lists of states (devices with one (chunk set, mask) pair each;
// devices with up to two) and two lists of prefixes, one per state list; a prefix is its instructions, its running
// cost sums for every query of the enumeration, and the index of its state (many prefixes share a state).
// For the kernel that builds the children of the judged states:
struct FrontLevel {
    uint32_t query;                // the enumerating query (its DevQuery describes the patterns)
    const int32_t* share;          // [n_share] the queries of the enumeration (indices into the DevQuery array)
    int32_t n_share, n_msg;
    const uint32_t* states1; const uint32_t* states2;      // the level's state lists
    const FrontSurvivor* surv; uint32_t n_surv;            // (state, instruction) pairs: entry = state, slot = the child's
                                                           // place in the next state list of its kind / among the goals
    int32_t lds_planes;            // 2 if a parent or a child of this level has two pairs, else 1
    FrontCounters* ctr;            // the level's counters: those of its first half (which the host has read) are cleared
                                   // by the kernel for the next level; null: left alone
    uint32_t* n_reps;              // [2] cleared by the kernel (the counts of distinct children, which the search that
                                   // follows adds up); null: left alone
    uint32_t* next_states1; uint32_t* next_states2;
    unsigned long long* next_hash1; unsigned long long* next_hash2;      // hash of every child's state (zero on entry)
    double* delta1; double* delta2; double* delta_goal;   // [child][n_share][2]: what the step adds to the cost sums
};
// For the kernel that writes the prefixes of the next level (and the goals) from the survivors of this level's prefixes:
struct FrontPrefixes {
    uint32_t query;
    int32_t n_share, n_msg;
    const FrontSurvivor* surv; uint32_t n_surv;            // entry = prefix (in the list the code names), slot = its place
    int32_t parent_len, keep_prefixes;
    const FrontEntry* entries1; const uint32_t* sid1; const double* sums1;        // the level's prefix lists
    const FrontEntry* entries2; const uint32_t* sid2; const double* sums2;
    const uint32_t* child_of1; const uint32_t* child_of2;  // [state][instruction] -> child (place of its kind)
    const uint32_t* rep1; const uint32_t* rep2;            // next state lists: child -> the state that stands for it (null: itself)
    const double* delta1; const double* delta2; const double* delta_goal;
    FrontEntry* next_entries1; uint32_t* next_sid1; double* next_sums1;
    FrontEntry* next_entries2; uint32_t* next_sid2; double* next_sums2;
    FrontEntry* next_literal;
    unsigned long long* valid_out; double* goal_sums;      // goals: candidate index and [n_share][2] sums
    FrontCounters* ctr;
};
// The valid programs of an enumeration written out for one of its queries.
struct FrontFinish {
    uint32_t query;                // whose rows are written (its links set the costs)
    int32_t n_share, share_pos;    // its place among the enumeration's queries
    uint32_t n_valid;
    const unsigned long long* valid; const uint32_t* rank; const double* goal_sums;
    unsigned long long out_first;  // first row of the query in the batch-wide buffers
    unsigned long long* sorted; p2_program* progs; double* costs;
};
// Bytes from one state's row of codes to the next: the alphabet rounded up to whole words, so that the kernels that
// list survivors and children read four codes at a time (the bytes past the alphabet are never looked at).
__host__ __device__ inline uint32_t front_code_stride(int alphabet) { return ((uint32_t)alphabet + 3u) & ~3u; }
size_t frontier_state_words(int R, int k);
// 2 where two planes of the state fit in LDS, else 1.
int frontier_max_pairs(int R, int k);
hipError_t launch_front_init(const DevQuery* q, uint32_t query, int R, int k, FrontEntry* entries, uint32_t* states,
                             double* sums, uint32_t* sid, int n_share, hipStream_t stream);
// Many prefixes of a frontier list have the same state (instructions that commute, detours that end alike), and
// what the rules say about the next instruction depends on the state alone.  The entries of a list are therefore
// grouped by state first: rep[p] = an entry with the same state as p (itself for one entry per distinct state,
// which are also listed in reps_list / counted in *n_reps).  Equal hashes only propose a pair; it is the
// comparison of the two states, word by word, that decides.  table: table_size (a power of two, at least 2 n)
// words, all ones on entry.  n < 2^24.
hipError_t launch_front_dedup(const uint32_t* states, size_t state_words, const unsigned long long* hash, uint32_t n,
                              unsigned long long* table, uint32_t table_size, uint32_t* rep, uint32_t* reps_list,
                              uint32_t* n_reps, hipStream_t stream);
// Judges the entries list[0 .. *n_list) of a frontier list (every entry 0 .. n - 1 if list is null) against the
// alphabet: codes[e * alphabet + digit] = CODE_* of that extension of entry e, unknown[e] = 1 where the pair form
// cannot judge the entry.  np: planes per entry (1: the one-pair list, 2: the two-pair list).  max_pairs = 1 sends
// children that need two pairs to the literal list.  row_counts[e]: how many of the row's codes are survivors, goals
// (low word, 16 bits each), one-pair and two-pair children (high word).  count_children != 0 adds the children of the
// entries it could judge to ctr->t_count (by kind).
hipError_t launch_front_classify(const DevQuery* q, int R, int k, const uint32_t* states, uint32_t n, const uint32_t* list,
                                 const uint32_t* n_list, int np, int max_pairs, int goals_only, int count_children, uint8_t* codes,
                                 unsigned long long* row_counts, uint8_t* unknown, FrontCounters* ctr, hipStream_t stream);
// The last level, before the classification (which then runs with goals_only on the list this leaves): the entries
// from which no instruction can end at the goal get a row of invalid codes; the others are listed in
// walk[0 .. *n_walk) (*n_walk zero on entry; any order).
hipError_t launch_front_goal_filter(const DevQuery* q, int R, int k, const uint32_t* states, uint32_t n, const uint32_t* list,
                                    const uint32_t* n_list, int np, uint8_t* codes, unsigned long long* row_counts, uint8_t* unknown,
                                    uint32_t* walk, uint32_t* n_walk, hipStream_t stream);
// The survivors of every entry of a list from the codes of the entry that stands for its state (rep null: its own):
// appended to surv with their places in the next frontier; entries that cannot be judged go to unknown_out
// (counted in n_unknown); handover != 0 treats every entry so (the hand-over path, for tests).
// row_counts: what the classification (or the last level's filter) left beside each row of codes: the numbers of
// survivors, goals, one-pair and two-pair children among its codes, 16 bits each.
hipError_t launch_front_expand(const DevQuery* q, const FrontEntry* entries, uint32_t n, const uint32_t* rep,
                               const uint8_t* codes, const unsigned long long* row_counts, const uint8_t* unknown, int np, int handover,
                               FrontSurvivor* surv, uint32_t surv_cap, FrontEntry* unknown_out, FrontCounters* ctr, hipStream_t stream);
// Bytes of the scratch buffer launch_front_classify_literal needs for n literal prefixes (always passed).
size_t front_literal_scratch_bytes(int R, int k, uint32_t n);
// class_cap: most classes of equal rows the class-state kernel may hold (1..64) before a prefix goes to the
// full-state kernel.  goals_only != 0 (the level at the size limit): only the instructions that can reach the
// goal from the prefix's state are judged, and only goals are reported.
hipError_t launch_front_classify_literal(const DevQuery* q, int R, int k, const FrontEntry* entries, uint32_t n,
                                         int parent_len, int goals_only, FrontSurvivor* surv, uint32_t surv_cap,
                                         FrontCounters* ctr, void* gscratch, int class_cap, hipStream_t stream);
// The children of the judged states of a list (every state 0 .. n - 1 if list is null), from their codes: counted by
// kind (write = 0: t_count), or given their places (write = 1: child_of[state * alphabet + digit], t_next) and
// listed in ssurv (n_ssurv).  keep = 0: goals only.
hipError_t launch_front_children(const DevQuery* q, uint32_t n, const uint32_t* list, const uint32_t* n_list, const uint8_t* codes,
                                 const uint8_t* unknown, int np, int keep, int write, uint32_t* child_of, FrontSurvivor* ssurv,
                                 FrontCounters* ctr, hipStream_t stream);
hipError_t launch_front_materialize(const DevQuery* queries, int R, int k, const FrontLevel& level, hipStream_t stream);
hipError_t launch_front_prefixes(const DevQuery* queries, const FrontPrefixes& P, hipStream_t stream);
hipError_t launch_front_emit(const DevQuery* q, uint32_t query, const FrontEntry* entries, const FrontSurvivor* surv,
                             uint32_t n_surv, int parent_len, int keep_prefixes, FrontEntry* next_literal,
                             unsigned long long* valid_out, double* goal_sums, int n_share, FrontCounters* ctr,
                             hipStream_t stream);
// The counters to pinned host memory; clears those that the second half of a level counts with.
hipError_t launch_front_counters_out(FrontCounters* host_dst, FrontCounters* ctr, hipStream_t stream);
hipError_t launch_front_rank(const unsigned long long* valid, uint32_t n, uint32_t* rank, hipStream_t stream);
// The rows of n_jobs queries in one launch (jobs in device memory; max_valid = the largest n_valid among them).
hipError_t launch_front_finish(const DevQuery* queries, const FrontFinish* jobs, uint32_t n_jobs, uint32_t max_valid, hipStream_t stream);

// One selection of launch_topk_jobs: the k best of (cost[i * stride], index[i]), i < n, ties by index;
// positions go to out_pos[min(k, n)], nan_flag is set to 1 when a cost is NaN.  All device pointers.
struct DevTopkJob {
    const double* cost;
    const unsigned long long* index;
    long long* out_pos;
    uint32_t* nan_flag;
    long long n;
    long long stride;
    int k;
    int pad;
};
// Block b of the launch does jobs[b] alone: meant for many selections of a few thousand entries each.
hipError_t launch_topk_jobs(const DevTopkJob* jobs, unsigned n_jobs, int max_k, hipStream_t stream);
// The rows that the selections of a batch picked, gathered so that only they go back to the host: segment s (one
// per query) has `rows` positions from pos[pos_first] on, relative to row out_first of the batch-wide program and
// cost arrays; selected row pos_first + t gets program and costs of row out_first + pos[pos_first + t].
struct DevGatherSeg {
    unsigned long long out_first, pos_first;
    uint32_t rows, pad;
};
hipError_t launch_gather_rows(const DevGatherSeg* segs, unsigned n_segs, const p2_program* progs, const double* costs, int n_cost,
                              const long long* pos, p2_program* sel_progs, double* sel_costs, hipStream_t stream);
// Many selections of many entries each: two launches for all of them (every job cut into strided shares, then a
// merge per job).  scratch: topk_big_scratch_bytes(n_jobs, max_k) bytes.  Grid limit: n_jobs <= 65535.
size_t topk_big_scratch_bytes(unsigned n_jobs, int max_k);
hipError_t launch_topk_big(const DevTopkJob* jobs, unsigned n_jobs, int max_k, void* scratch, hipStream_t stream);

// Results to the host: a kernel copies `bytes` (rounded up to 16; both buffers must hold that) from device
// memory to pinned, device-accessible host memory.  Used instead of hipMemcpyAsync, whose queueing of a
// device-to-host copy was seen to take 0.1 ms longer in some processes (never in others).
hipError_t launch_copy_out(void* dst_host, const void* src_dev, size_t bytes, hipStream_t stream);
// Up to three of them in one launch (bytes may be 0).
hipError_t launch_copy_out3(void* dst0, const void* src0, size_t bytes0, void* dst1, const void* src1, size_t bytes1,
                            void* dst2, const void* src2, size_t bytes2, hipStream_t stream);

// Top-k of (cost[i * stride], index[i]) over i < n: positions into out_pos[min(k, n)].
// scratch: device buffer of topk_scratch_bytes(n, k) bytes.  nan_flag: device uint32 set to 1 on NaN.
size_t topk_scratch_bytes(long long n, int k);
hipError_t launch_topk(const double* cost, long long stride, const unsigned long long* index, long long n, int k,
                       long long* out_pos, void* scratch, uint32_t* nan_flag, hipStream_t stream);

// The same selection with the stage-1 lists in a fixed array of the device image (no allocation): k at most
// topk_fixed_max_k(); nan_flag (device, may be null) is cleared and then set to 1 when a cost is NaN.
// Only queues kernels.  hipErrorInvalidValue when k is too large.
int topk_fixed_max_k();
hipError_t launch_topk_fixed(const double* cost, long long stride, const unsigned long long* index, long long n, int k,
                             long long* out_pos, uint32_t* nan_flag, hipStream_t stream);

}  // namespace p2
