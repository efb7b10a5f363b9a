/*
 * p2.h -- C ABI of the MI355X batch evaluator for reduction programs.
 *
 * The library evaluates, on one GPU, candidate reduction programs of the P^2
 * synthesizer (arXiv 2110.10548): a candidate is a sequence of collectives
 * (AllReduce, ReduceScatter, AllGather, Reduce, Broadcast) in the
 * InsideGroup / Parallel / Master forms (Sec. 3.3), applied to levels of the
 * reduction-axis synthesis hierarchy of a parallelism placement (Sec. 3.4).
 * Every candidate is derived from an integer index, checked against the
 * device-state semantics of Sec. 3.2 from the init state to the goal state
 * of Sec. 3.5, costed with a hierarchical alpha-beta model in fp64 (ring, or
 * tree for AllReduce; Sec. 5 gives the simulator's inputs) and ranked.
 *
 * Conventions
 *  - Every function returns an int32 status: P2_OK or a negative error.  The
 *    library never throws and never aborts; p2_last_error() returns the text
 *    of the calling thread's last error.
 *  - Unless a parameter says "device", every pointer is a HOST pointer.  All
 *    buffers are caller-owned; the library keeps no caller pointer after a
 *    call returns.  Device scratch is owned by the library, cached per host
 *    thread and reused between calls; calls from different host threads do
 *    not share it.
 *  - Two-call sizing: a call with cap = 0 (and NULL outputs) only writes the
 *    required count.  If cap is too small the call returns P2_ENOSPC, the
 *    required count is still written and the output contents are unspecified.
 *    Such a call evaluates the candidates (the counts and the stats come from
 *    that) but does not order, cost or select anything.
 *  - Arrays over hardware levels are outermost level first.
 */
#ifndef P2_H
#define P2_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define P2_OK 0
#define P2_EINVAL (-1)        /* bad pointer, factor does not divide, empty/duplicate reduce axes,
                                 prod(axes) != prod(card), placement violating Eq. (1)-(2),
                                 max_len < 1, candidate count overflowing 64 bits, NaN cost       */
#define P2_ENOSPC (-2)        /* caller buffer too small                                          */
#define P2_EUNSUPPORTED (-3)  /* more than 512 devices, 8 levels, 8 axes, max_len > 7, top-k > 1024,
                                 or a state too large for the selected engine                     */
#define P2_EDEVICE (-4)       /* a HIP call failed; see p2_last_error()                            */

#define P2_MAX_LEVELS 8
#define P2_MAX_AXES 8
#define P2_MAX_DEVICES 512
#define P2_MAX_LEN 7

/* A hierarchical system (Sec. 2): level j has card[j] children per parent; two devices that
 * first differ at level j talk through the uplinks of their level-j units, each of bandwidth
 * bw_bytes_per_s[j] and latency alpha_s[j].  bw and alpha may be NULL where no cost is asked. */
typedef struct {
    int32_t n_levels;
    const int32_t* card;            /* [n_levels], >= 1                       */
    const double* bw_bytes_per_s;   /* [n_levels], > 0                        */
    const double* alpha_s;          /* [n_levels], >= 0                       */
} p2_hierarchy;

/* Sec. 3.1: all parallelism matrices x[n_axes][n_levels] of positive integers whose column
 * products are card[j] (Eq. 1) and row products are axes[i] (Eq. 2), written row-major into
 * out[cap][n_axes][n_levels] in lexicographic order of the flattening.  *out_count = number of
 * matrices.  Host-only; no device work. */
int32_t p2_enumerate_placements(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes,
                                int32_t* out, int64_t cap, int64_t* out_count);

/* Evaluation engines.  All give identical results; they differ in the state they keep. */
#define P2_ENGINE_AUTO 0      /* shared-prefix engine where it applies, else the compact engine; the
                                 literal engine for the candidates they cannot hold; the frontier
                                 engine above 2^30 candidates                                     */
#define P2_ENGINE_LITERAL 1   /* R x k masks of R bits per candidate in LDS, one wavefront each   */
#define P2_ENGINE_COMPACT 2   /* per device one chunk set and one contribution mask, in LDS; one
                                 candidate per lane                                               */
#define P2_ENGINE_FRONTIER 3  /* enumeration by program size with pruning (Sec. 3.5): only valid
                                 prefixes are extended; AUTO picks it above 2^30 candidates.
                                 Queries of one batch with the same reduction-group size, chunk
                                 count, patterns, alphabet and size limit are enumerated once (the
                                 later ones report the first one's counts in their stats)        */
#define P2_ENGINE_SMALL 4     /* compact form for reduction groups of at most 32 devices, at most
                                 32 chunks and patterns whose group size and stride are powers of
                                 two: one candidate per lane, every step computed in registers;
                                 P2_EUNSUPPORTED where it does not apply                          */
#define P2_ENGINE_SHARED 5    /* reduction groups of at most 64 devices, patterns whose group size
                                 and stride are powers of two: the instructions that consecutive
                                 candidates have in common are applied once per wavefront (lanes
                                 play the devices), each candidate then applies its own last
                                 instruction where that can reach the goal; P2_EUNSUPPORTED where
                                 it does not apply                                                */

/* Synthesis hierarchies (Sec. 3.4, Appendix A).  The tool synthesizes on (d); the others are there so
 * that the section's claim (each hierarchy of the list expresses every program of the one before)
 * can be checked on this evaluator.  A level of the hierarchy owns factors x[i][j] of the matrix:
 *   COLLAPSED  (d)  per hardware level j the product of the reduction axes' factors
 *   SYSTEM     (a)  per hardware level j all its factors (every axis): the system's own levels
 *   COLUMN     (b)  one level per factor, x00 x10 .. x01 x11 .. (hardware level by hardware level)
 *   ROW        (c)  one level per factor, x00 x01 .. x10 x11 .. (axis by axis)
 *   REDUCTION       one level per factor of the reduction axes only, axis by axis ((d) before the
 *                   factors of one hardware level are multiplied)
 * Under COLLAPSED and REDUCTION a program runs on one reduction group and is repeated over the
 * other axes; under the other three it runs on the whole system (group_size in the stats is then
 * the number of devices, and the goal is per device).  Everything but COLLAPSED is evaluated by the
 * literal engine (engine AUTO or LITERAL; another engine => P2_EUNSUPPORTED). */
#define P2_HIERARCHY_COLLAPSED 0
#define P2_HIERARCHY_SYSTEM 1
#define P2_HIERARCHY_COLUMN 2
#define P2_HIERARCHY_ROW 3
#define P2_HIERARCHY_REDUCTION 4

typedef struct {
    int32_t n_chunks;    /* k of Sec. 3.2; 0 => number of devices (the paper's choice)           */
    uint32_t form_mask;  /* bit 0 InsideGroup, bit 1 Parallel, bit 2 Master; 0 => all            */
    uint32_t op_mask;    /* bits 0..4 = AllReduce, ReduceScatter, AllGather, Reduce, Broadcast;
                            0 => all                                                             */
    int32_t algo;        /* cost model of an AllReduce step (Sec. 4 runs both): 0 = ring, 2(g-1)
                            steps and 2(g-1)/g n bytes per member link; 1 = two-tree, 2 ceil(log2 g)
                            steps and 2 n bytes.  The other collectives always use the ring figures.
                            Anything else => P2_EUNSUPPORTED                                     */
    int32_t topk;        /* 0 => return every valid program; else see p2_synthesize              */
    int32_t engine;      /* P2_ENGINE_*                                                          */
    int32_t hierarchy;   /* P2_HIERARCHY_*; 0 => (d), the tool's own                             */
    uint32_t flags;      /* P2_FLAG_* bits; 0 => none                                            */
    int32_t max_row_classes; /* 0 => 64.  The literal kernels that serve the shared-prefix and the
                            frontier engine keep a state by classes of equal rows, up to this
                            many (1..64), and fall back to the full literal state beyond it;
                            results do not depend on it (a lower limit sends more work down
                            the fall-back path, which is what tests of that path set it for).
                            Kernels that serve several queries use the smallest limit among
                            them.  Outside 0..64 => P2_EINVAL                                    */
    int32_t frontier_pairs; /* P2_FRONTIER_PAIRS_*: state form of the frontier engine; 0 => the default  */
    void* hip_stream;    /* hipStream_t to run on; NULL => the default stream                    */
} p2_options;

/* p2_options.frontier_pairs.  The frontier engine keeps a prefix's state as up to two (chunk set, mask)
 * pairs per device and hands what that form cannot hold to kernels that rebuild the literal state from the
 * prefix's instructions.  Results do not depend on the choice; the other values exist so that every path
 * can be run on purpose. */
#define P2_FRONTIER_PAIRS_AUTO 0          /* two pairs where two planes of the state fit in LDS, else one    */
#define P2_FRONTIER_PAIRS_ONE 1           /* one pair per device; a prefix that needs two goes to the literal kernels */
#define P2_FRONTIER_PAIRS_TWO 2           /* as AUTO                                                          */
#define P2_FRONTIER_PAIRS_TWO_HANDOVER 3  /* two pairs are kept, but every two-pair prefix is classified by the
                                             literal kernels (the path of prefixes whose groups split their rows
                                             differently)                                                    */
#define P2_FRONTIER_PAIRS_NONE 4          /* no pair states: every prefix is a literal prefix, and valid programs
                                             are costed by re-running them                                   */

/* p2_options.flags */
#define P2_FLAG_EVALUATE_EVERY_QUERY 1u   /* p2_synthesize_batch: do not share the evaluation of queries
                                             that are equal in everything validity depends on (see
                                             there); set on any query of the batch, it holds for all  */
#define P2_FLAG_ONE_ENUMERATION_AT_A_TIME 2u /* frontier engine: run the enumerations of the batch one after
                                             the other on one stream instead of several side by side
                                             (results are the same; the per-kernel times of p2_profile are
                                             then those of kernels that have the chip to themselves); set
                                             on any query of the batch, it holds for all                */

/* One program.  instr[t] = pattern_id * 5 + op, op in the order AllReduce, ReduceScatter,
 * AllGather, Reduce, Broadcast; pattern ids are those of p2_describe_pattern.  index is the
 * candidate's rank: programs ordered by length, then lexicographically with instr[0] most
 * significant, the digit of an instruction being pattern_id * (enabled ops) + (rank of op
 * among the enabled ops). */
typedef struct {
    uint64_t index;
    uint8_t len;
    uint8_t instr[7];
} p2_program;

/* Counters of one query (all optional outputs). */
typedef struct {
    uint64_t candidates;       /* programs of length <= max_len over the alphabet: the candidate
                                  space this query's results cover.  A query that shares another
                                  query's evaluation (p2_synthesize_batch) reports the same number
                                  although nothing was evaluated for it                           */
    uint64_t steps_executed;   /* instructions applied, counted per candidate (a candidate stops at
                                  its first bad step): what evaluating every candidate on its own
                                  executes, whichever engine ran                                  */
    uint64_t literal_reruns;   /* candidates the compact engine handed to the literal engine      */
    uint64_t member_visits;    /* sum over applied instructions of the devices taking part in them */
    int64_t valid;             /* valid programs found                                            */
    int32_t group_size;        /* R: devices in one reduction group                               */
    int32_t n_patterns;        /* canonical (slice, form) patterns                                */
    int32_t alphabet;          /* instructions = patterns x enabled ops                           */
    int32_t engine;            /* engine that evaluated the bulk of the candidates                */
    uint64_t steps_evaluated;  /* instruction applications the engine carried out; an application
                                  shared by several candidates counts once (P2_ENGINE_SHARED: the
                                  candidates handed to the literal engine not included), so it is
                                  at most steps_executed                                          */
    uint64_t members_evaluated;/* devices taking part in those applications, summed               */
    int32_t evaluated_with;    /* p2_synthesize_batch: index of the earlier query of the batch whose
                                  evaluation this one shares (its validity results are that
                                  query's, its costs its own; steps_* and members_* repeat that
                                  query's figures), or -1: evaluated for itself                   */
    int32_t reserved0;
} p2_stats;

/* Sec. 3.5 on one placement: evaluate every program of length <= max_len.  A program is valid
 * iff each instruction satisfies its rule (Sec. 3.2) on every device group of its pattern,
 * changes the state, and the final state is the goal.  Valid programs are written in ascending
 * candidate index with cost[i][m] = simulated seconds for msg_bytes[m] (bytes held per device).
 *
 * With opt->topk = K > 0 the output is instead n_msg consecutive blocks of kk = min(K, valid)
 * programs: block m holds the kk cheapest programs for msg_bytes[m] in ascending (cost, index);
 * out_cost keeps all n_msg costs of each listed program; *out_count = n_msg * kk.
 *
 * placement [n_axes][n_levels] row-major; reduce_axes: distinct axis numbers.  n_msg may be 0
 * (then out_cost is unused and topk must be 0).  stats may be NULL. */
int32_t p2_synthesize(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* placement,
                      const int32_t* reduce_axes, int32_t n_reduce, int32_t max_len,
                      const double* msg_bytes, int32_t n_msg, const p2_options* opt,
                      p2_program* out_prog, double* out_cost /* [cap][n_msg] */, int64_t cap,
                      int64_t* out_count, uint64_t* out_candidates_evaluated, p2_stats* stats);

/* One query of a batch (same meaning as the arguments of p2_synthesize). */
typedef struct {
    const p2_hierarchy* h;
    const int32_t* axes;
    int32_t n_axes;
    const int32_t* placement;
    const int32_t* reduce_axes;
    int32_t n_reduce;
    int32_t max_len;
    const p2_options* opt;     /* NULL => defaults; hip_stream of the first query is used for all */
} p2_query;

/* Many placements / reduce sets at once (the synthesizer's outer loop, Sec. 4: every matrix of
 * every requested reduction).  All queries share msg_bytes.  Results of query i occupy
 * out_prog[out_offset[i] .. out_offset[i+1]) and the matching rows of out_cost;
 * out_offset has n_queries + 1 entries; stats (optional) has n_queries entries.
 * Whether a program is valid depends on the reduction group, the chunks, the patterns, the alphabet
 * and the size limit only, not on the links nor on where the placement puts the group: queries of
 * the batch that agree in these are evaluated once and then costed each with its own links (the
 * later ones report the first one's per-candidate counts in their stats, and steps_evaluated = 0
 * under the shared-prefix engine).  P2_FLAG_EVALUATE_EVERY_QUERY in the options of any query of the
 * batch switches this off for the whole batch, on every engine.
 * The kernels of all queries share their launches; the call waits for the device twice: after
 * the evaluation (to size the result lists) and for the results.  Queries on the frontier engine
 * run on streams of the library's own, up to four enumerations side by side, and the call waits
 * for them; the first such call of a host thread also waits for the caller's stream and spends a
 * few milliseconds timing short kernels on a handful of new streams, to pick four that do not
 * share a hardware queue. */
int32_t p2_synthesize_batch(const p2_query* queries, int32_t n_queries, const double* msg_bytes, int32_t n_msg,
                            p2_program* out_prog, double* out_cost, int64_t cap, int64_t* out_offset,
                            p2_stats* stats);

/* One (placement, reduction) pair of p2_search_placements. */
typedef struct {
    p2_program best;         /* the valid program with the smallest (cost, index); len = 0 when there
                                is none, or when the reduction group is a single device            */
    double best_cost;        /* its simulated seconds; 0 for a single device; +inf when no program
                                of length <= max_len is valid                                      */
    double allreduce_cost;   /* the one-instruction program AllReduce over the whole reduction group
                                (InsideGroup on the root level; always valid): the baseline that the
                                evaluation compares synthesized programs with (Sec. 4.2)           */
    uint64_t valid;          /* valid programs of length <= max_len                                */
    uint64_t candidates;     /* programs evaluated                                                 */
} p2_search_row;

/* The synthesizer's outer loop with its ranking (Sec. 2.2 and 4.1): every parallelism matrix of the
 * system (in the order of p2_enumerate_placements) x every requested reduction, all in one batch on
 * the GPU.  reduce_sets holds the axis numbers of the n_sets reductions one after another,
 * reduce_set_len[s] of them for reduction s.  One message size (bytes held per device).
 * out_rows[p * n_sets + s] describes placement p under reduction s; out_total[p] =
 * sum_s weights[s] * best_cost (weights NULL => all 1: a mapping is chosen with all of a model's
 * reductions in view, Sec. 4.1); out_order lists the placements by ascending (total, p).
 * opt->topk is ignored; opt->hierarchy must be P2_HIERARCHY_COLLAPSED (else P2_EUNSUPPORTED).
 * *out_count = number of placements; with cap = 0 only that is written; cap < *out_count =>
 * P2_ENOSPC. */
int32_t p2_search_placements(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* reduce_sets,
                             const int32_t* reduce_set_len, int32_t n_sets, const double* weights, int32_t max_len,
                             double msg_bytes, const p2_options* opt, int32_t* out_placements /* [cap][n_axes][n_levels] */,
                             p2_search_row* out_rows /* [cap][n_sets] */, double* out_total /* [cap] */,
                             int32_t* out_order /* [cap] */, int64_t cap, int64_t* out_count);

/* The device groups of canonical pattern `pattern_id` on the full system (Sec. 3.3 and the
 * table of hierarchical communication patterns): slice level and form level are indices into
 * the synthesis hierarchy e_0 = root, e_1..e_n (form_level = -1 for InsideGroup); form is
 * 0 InsideGroup, 1 Parallel, 2 Master.  group_of_device[d] = group id (groups numbered by their
 * smallest device) or -1; rank_in_group[d] = position in ascending device order (rank 0 is the
 * root of Reduce and Broadcast).  *out_n_patterns (optional) = number of canonical patterns.
 * Host-only. */
int32_t p2_describe_pattern(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* placement,
                            const int32_t* reduce_axes, int32_t n_reduce, const p2_options* opt,
                            int32_t pattern_id, int32_t* slice_level, int32_t* form, int32_t* form_level,
                            int32_t* group_of_device /* [D] */, int32_t* rank_in_group /* [D] */,
                            int32_t* out_n_patterns);

/* Positions of the min(k, n) smallest (cost, index) pairs in ascending cost, ties by ascending
 * index (the simulator's shortlist, Sec. 5).  NaN in cost => P2_EINVAL.  Host arrays; the data
 * is copied to the GPU and selected there. */
int32_t p2_topk(const double* cost, const uint64_t* index, int64_t n, int32_t k, int64_t* out_pos);

/* Same on DEVICE arrays: cost, index (n entries each; cost read with stride cost_stride doubles)
 * and out_pos (min(k, n) entries) are device pointers; stream is a hipStream_t or NULL.
 * Returns after the result is in out_pos. */
int32_t p2_topk_device(const double* cost, int64_t cost_stride, const uint64_t* index, int64_t n, int32_t k,
                       int64_t* out_pos, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): p2_topk_device with its intermediate lists in a fixed 3 MiB array of the
 * library's device image instead of library-allocated scratch.  Calls no hipMalloc / hipFree / pinned-memory
 * routine, only queues kernels on `stream` and returns without waiting: out_pos (device, min(k, n)
 * entries) is complete once the stream has passed this point.  out_nan (device uint32, may be NULL) is
 * set to 0 by the call and to 1 by its kernels when a cost is NaN (NaN entries are then left out and
 * trailing positions are -1); nothing is reported to the host.  k > 64 => P2_EUNSUPPORTED.
 * Every GPU holds one copy of the array until the process ends and all calls on a GPU share it: calls that
 * overlap on one GPU (different streams or host threads) race; calls on one stream are safe. */
int32_t p2_topk_device_noalloc(const double* cost, int64_t cost_stride, const uint64_t* index, int64_t n, int32_t k,
                               int64_t* out_pos, uint32_t* out_nan, void* stream);

/* Timing of the calling thread's last p2_synthesize / p2_synthesize_batch call, taken with HIP
 * events on the call's stream.  Off by default; p2_set_profiling(1) turns the events on.
 * p2_set_profiling(2) does the same but, of the frontier engine's launches, times only the classification
 * and the building of the children (front_classify_*, front_materialize_*): front_literal_ms and
 * front_group_ms then stay zero.  An event pair per group of small launches costs host time (some 2 000 pairs
 * in a call on a large batch, several per cent of the call), which a measurement of the whole call can do without. */
typedef struct {
    float eval_ms;             /* all evaluation-kernel launches of the call                       */
    float post_ms;             /* ordering, cost and top-k kernels                                 */
    int32_t eval_launches;     /* evaluation kernels launched                                      */
    int32_t post_launches;
    float host_plan_ms;        /* host: planning of all queries before the first launch (patterns,
                                  alphabet; the cost model's tables are built while the GPU runs)  */
    float host_total_ms;       /* host: whole call, wall clock                                     */
    /* Enumeration by program size (Sec. 3.5; the frontier engine): device time of the whole
     * enumeration (not part of eval_ms / post_ms) and, from an event pair around every launch,
     * of its three kernel families, with what those launches worked on.                            */
    float front_ms;
    float front_classify_ms;          /* prefixes held as (chunk set, mask) pairs judged against the
                                         alphabet (Sec. 3.2's rules on every instruction)          */
    float front_literal_ms;           /* prefixes held literally, judged from their instructions    */
    float front_materialize_ms;       /* children of the judged states: state and step costs        */
    int32_t front_classify_launches, front_literal_launches, front_materialize_launches;
    float front_group_ms;             /* the search for entries with equal states, and the listing of
                                         every entry's survivors from the codes of its state       */
    double front_prefixes;            /* prefixes the pair classification judged: one per distinct
                                         state of a frontier list                                   */
    double front_classify_state_bytes;/* bytes of their states, R * (ceil(k/32) + ceil(R/32)) words
                                         per pair plane: what the classification must read from
                                         device memory                                              */
    double front_classify_lane_ops;   /* 4 lane-operations (read, union, intersection / seen-twice,
                                         compare) per state word of every device that a pattern of
                                         the alphabet visits, per judged prefix and plane           */
    double front_survivors;           /* children built: one per (judged state, valid instruction)  */
    double front_materialize_bytes;   /* bytes that must move for them: a parent plane read per child,
                                         the planes of every kept child written, what the step adds
                                         to the cost sums                                           */
    double front_entries;             /* prefixes of the pair lists, all levels (they end in
                                         front_prefixes distinct states, which were judged)         */
} p2_profile;
int32_t p2_set_profiling(int32_t on);
int32_t p2_get_profile(p2_profile* out);

/* Measurement aid: the best rate, in lane-operations per second, that `reps` (1..100) timed runs of a
 * stream of independent 32-bit integer vector instructions reach on the current device; the
 * evaluators' lane-operation rates (Sec. 3.2's rules are bit operations on the device masks) are set
 * against the ceiling derived from the unit counts and the clock, and this shows how close the
 * device comes to it.  hip_stream: hipStream_t or NULL.  P2_EINVAL on bad arguments. */
int32_t p2_measure_alu_peak(int32_t reps, double* out_lane_ops_per_s, void* hip_stream);

/* Measurement aid: the best rate, in bytes per second, that `reps` (1..100) timed runs of a stream of
 * 128-bit reads from the local data share reach on the current device (every lane 16 bytes per
 * instruction, all banks, many reads in flight): the frontier engine's classification (Sec. 3.5: every
 * valid prefix is judged against every instruction of the alphabet) reads the prefix's state from LDS
 * once per pattern, and its LDS byte rate is set against 256 compute units x 256 bytes per clock x
 * 2.4 GHz; this shows how close the device comes to that.  hip_stream: hipStream_t or NULL.
 * P2_EINVAL on bad arguments. */
int32_t p2_measure_lds_peak(int32_t reps, double* out_bytes_per_s, void* hip_stream);

/* Gives back what the calling host thread's calls have cached: device buffers, pinned host buffers,
 * the upload stream and the profiling events (profiling is switched off).  The next call of the thread
 * allocates afresh.  A host thread that ends gives its cache back by itself; the thread that loaded the
 * library keeps it until the process ends unless it calls this. */
int32_t p2_release_thread(void);

const char* p2_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* P2_H */
