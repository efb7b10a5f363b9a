// Shared-prefix engine: reduction groups of at most 64 devices, patterns whose group size g and
// stride s are powers of two (every pattern of a hierarchy with power-of-two levels).
//
// Same state form as p2_compact.hip -- per device one chunk set and one contribution mask -- but
// held by the wavefront as a whole: lane d plays device d (with at most 32 devices, lane d + 32
// mirrors lane d) and keeps that device's pair in registers.  The members of a group differ exactly
// in bits [log2 s, log2 s + log2 g) of the device number, so a rule is a sequence of stages, one
// per such bit J, each a lane exchange with lane d ^ 2^J:
//   AllReduce-like : union of the masks along each bit; the two sides of every pair must hold the
//                    same chunks and disjoint masks (the sides' running unions are disjoint at
//                    every stage iff all members are pairwise disjoint).
//   ReduceScatter  : then the member of rank p keeps the p-th block of the chunks.
//   Reduce         : then every member that has one of the bits set is cleared.
//   AllGather      : union of the chunk sets along each bit, sides disjoint; nobody empty.
//   Broadcast      : binomial tree from the member with all bits clear; a member is compared with
//                    the root's pair right before it takes it.
//
// Candidates of one length are numbered prefix * alphabet + last instruction, so the `alphabet`
// candidates of a group (same first len-1 instructions) are consecutive, and so are the groups of
// a stem (same first len-2 instructions).  The state after a prefix is the same for the whole
// group, so it is computed once per group, the stem's part of it once per work item; a group whose
// stem or prefix is invalid is settled for all its candidates at once.  A candidate is still
// resolved individually: under a valid prefix it applies its own last instruction where that can
// reach the goal.
#include "p2_compact_dev.h"

#include <type_traits>

namespace p2 {

namespace {

enum : int { WSTEP_INVALID = 0, WSTEP_OK = 1, WSTEP_GIVE_UP = 2 };

// Groups per hand-over entry of a stem whose own state leaves the compact form: the literal engine rebuilds
// the stem once per entry, so more groups save work, fewer keep its units of work short.
constexpr uint32_t kStemGroups = 4;

template <int N>
__device__ __forceinline__ Words<N> exchange(const Words<N>& a, int lane_xor) {
    Words<N> o;
#pragma unroll
    for (int i = 0; i < N; ++i) o.w[i] = (uint32_t)__shfl_xor((int)a.w[i], lane_xor, kWave);
    return o;
}
template <int N>
__device__ __forceinline__ void unite(Words<N>& a, const Words<N>& b) {
#pragma unroll
    for (int i = 0; i < N; ++i) a.w[i] |= b.w[i];
}
template <int N>
__device__ __forceinline__ void clear(Words<N>& a) {
#pragma unroll
    for (int i = 0; i < N; ++i) a.w[i] = 0u;
}

// One instruction on the wavefront-held state (rv, mv: pair of device `dev` = lane modulo 32 or 64).
// All lanes are active and all arguments but rv, mv, dev are wave-uniform.  lg, ls: log2 of group
// size and stride; part: bit d set iff device d takes part; devs: 32 or 64.
template <int KW, int MW>
__device__ __forceinline__ int wave_step(Words<KW>& rv, Words<MW>& mv, int dev, int op, int lg, int ls,
                                         unsigned long long part, int devs) {
    const int gm1 = (1 << lg) - 1;
    const uint32_t gmask = (uint32_t)gm1 << ls;
    const bool in = ((part >> dev) & 1ull) != 0ull;
    bool bad = false;
    if (op == OP_AR || op == OP_RS || op == OP_RD) {
        // same chunks on every member, no contribution reduced twice: union of the masks along each bit
        for (int J = ls; J < ls + lg; ++J) {
            const Words<KW> pr = exchange(rv, 1 << J);
            const Words<MW> pm = exchange(mv, 1 << J);
            bad |= in && ((fold_xor(rv, pr) | fold_and(mv, pm)) != 0u);
            if (in) unite(mv, pm);
        }
        if (__any(bad)) return WSTEP_INVALID;
        if (!__any(in && fold_or(rv) != 0u)) return WSTEP_INVALID;      // only groups of empty devices: nothing changes
        if (op == OP_RS) {
            // the member of rank p keeps the p-th block of the chunks in ascending order
            const int c = popcount(rv);
            const int per = c >> lg, p = (dev >> ls) & gm1;
            bad = in && (c & gm1) != 0;
            const Words<KW> upto = lowest_n(rv, (p + 1) * per), below = lowest_n(rv, p * per);
            if (in) {
#pragma unroll
                for (int i = 0; i < KW; ++i) rv.w[i] = upto.w[i] & ~below.w[i];
            }
            if (__any(bad)) return WSTEP_INVALID;
        } else if (op == OP_RD) {
            if (in && ((uint32_t)dev & gmask) != 0u) { clear(rv); clear(mv); }
        }
        return WSTEP_OK;
    }
    if (op == OP_AG) {
        // nobody empty, every chunk held once: union of the chunk sets along each bit
        if (__any(in && fold_or(rv) == 0u)) return WSTEP_INVALID;
        bool differs = false;
        for (int J = ls; J < ls + lg; ++J) {
            const Words<KW> pr = exchange(rv, 1 << J);
            const Words<MW> pm = exchange(mv, 1 << J);
            bad |= in && fold_and(rv, pr) != 0u;
            differs |= in && fold_xor(mv, pm) != 0u;
            if (in) unite(rv, pr);
        }
        if (__any(bad)) return WSTEP_INVALID;
        return __any(differs) ? WSTEP_GIVE_UP : WSTEP_OK;      // rows with different column sets leave this form
    }
    // Broadcast as a binomial tree from the member with all group bits clear: a member is compared
    // with the root's pair right before it takes it
    bool neq = false;
    for (int J = ls; J < ls + lg; ++J) {
        const Words<KW> pr = exchange(rv, 1 << J);
        const Words<MW> pm = exchange(mv, 1 << J);
        const bool takes = in && ((dev >> J) & 1) != 0 && ((uint32_t)dev & gmask & (~0u << (J + 1))) == 0u;
        if (takes) {
            bad |= (fold_andn(rv, pr) | fold_andn(mv, pm)) != 0u;
            neq |= (fold_xor(rv, pr) | fold_xor(mv, pm)) != 0u;
            rv = pr;
            mv = pm;
        }
    }
    if (__any(bad)) return WSTEP_INVALID;
    // in every group some member must have differed from the root: fold the flags onto the roots' bits
    const unsigned long long low = devs >= 64 ? ~0ull : ((1ull << devs) - 1ull);
    unsigned long long flags = __ballot(neq) & low;
    const unsigned long long roots = __ballot(in && ((uint32_t)dev & gmask) == 0u) & low;
    for (int J = ls; J < ls + lg; ++J) flags |= flags >> (1u << J);
    return (~flags & roots) != 0ull ? WSTEP_INVALID : WSTEP_OK;
}

// The last instruction of a candidate matters only through the goal, and only three kinds of last
// instruction can reach it; each is judged by what is left of its rule on the states that allow it.
//
// AllReduce on a state whose devices all hold every chunk: the goal is reached iff in every group the masks
// are pairwise disjoint and unite to all columns, and the devices outside the pattern are complete already
// (the members hold the same chunks, so only masks travel).
template <int MW>
__device__ __forceinline__ bool judge_allreduce(Words<MW> mv, int dev, int lg, int ls, unsigned long long part, int R,
                                                const Words<MW>& all_cols) {
    const bool in = ((part >> dev) & 1ull) != 0ull;
    bool bad = false;
    for (int J = ls; J < ls + lg; ++J) {
        const Words<MW> pm = exchange(mv, 1 << J);
        bad |= in && fold_and(mv, pm) != 0u;
        if (in) unite(mv, pm);
    }
    bad |= dev < R && fold_xor(mv, all_cols) != 0u;
    return !__any(bad);
}
// AllGather on a state whose devices all carry every column: the goal is reached iff no member is empty, in
// every group the chunk sets are pairwise disjoint and unite to all chunks, and the devices outside the
// pattern hold every chunk already (the masks are equal, so only chunk sets travel).
template <int KW>
__device__ __forceinline__ bool judge_allgather(Words<KW> rv, int dev, int lg, int ls, unsigned long long part, int R,
                                                const Words<KW>& all_rows) {
    const bool in = ((part >> dev) & 1ull) != 0ull;
    bool bad = in && fold_or(rv) == 0u;
    for (int J = ls; J < ls + lg; ++J) {
        const Words<KW> pr = exchange(rv, 1 << J);
        bad |= in && fold_and(rv, pr) != 0u;
        if (in) unite(rv, pr);
    }
    bad |= dev < R && fold_xor(rv, all_rows) != 0u;
    return !__any(bad);
}
// Broadcast: every member ends with its root's pair, so the goal is reached iff every root is complete, every
// group has a member that is not (the information increase the rule asks for; a complete root knows what any
// member knows), and the devices outside the pattern are complete.  complete: bit d set iff device d < R holds
// every chunk with every column.
__device__ __forceinline__ bool judge_broadcast(unsigned long long complete, int lg, int ls, unsigned long long part, int R) {
    const unsigned long long devices = R >= 64 ? ~0ull : ((1ull << R) - 1ull);
    // the roots: participating devices whose number has all group bits clear
    unsigned long long roots = part & devices;
    for (int J = ls; J < ls + lg; ++J) {
        const unsigned long long bit_clear = J == 0 ? 0x5555555555555555ull : J == 1 ? 0x3333333333333333ull
                                           : J == 2 ? 0x0f0f0f0f0f0f0f0full : J == 3 ? 0x00ff00ff00ff00ffull
                                           : J == 4 ? 0x0000ffff0000ffffull : 0x00000000ffffffffull;
        roots &= bit_clear;
    }
    if ((roots & ~complete) != 0ull || (devices & ~part & ~complete) != 0ull) return false;
    unsigned long long flags = part & devices & ~complete;  // members that are not complete, folded onto their roots
    for (int J = ls; J < ls + lg; ++J) flags |= flags >> (1u << J);
    return (roots & ~flags) == 0ull;
}

// The first instruction of a program, on the init state of Sec. 3.5 (every device holds every chunk,
// device i column i): what the rules give there is known without an exchange.  Members of a group hold
// the same chunks and disjoint columns, so the AllReduce-like rules apply (ReduceScatter if the group
// size divides k) and every member ends with the columns of its group, the devices that agree with it
// outside bits [ls, ls + lg); AllGather and Broadcast never apply.  rv, mv hold the init state on entry.
template <int KW, int MW>
__device__ __forceinline__ int first_wave_step(Words<KW>& rv, Words<MW>& mv, int dev, int op, int lg, int ls,
                                               unsigned long long part, int k) {
    if (op == OP_AG || op == OP_BC) return WSTEP_INVALID;
    const int gm1 = (1 << lg) - 1;
    if (op == OP_RS && (k & gm1) != 0) return WSTEP_INVALID;
    const bool in = ((part >> dev) & 1ull) != 0ull;
    if (!in) return WSTEP_OK;                         // (wave-uniform result; this lane's device keeps its state)
    const uint32_t gmask = (uint32_t)gm1 << ls;
    unsigned long long cols = 1ull << ((uint32_t)dev & ~gmask);
    for (int J = ls; J < ls + lg; ++J) cols |= cols << (1u << J);
    mv.w[0] = (uint32_t)cols;
    if (MW > 1) mv.w[MW > 1 ? 1 : 0] = (uint32_t)(cols >> 32);
    if (op == OP_RS) {
        const int per = k >> lg, p = (dev >> ls) & gm1;
        const Words<KW> upto = lowest_n(rv, (p + 1) * per), below = lowest_n(rv, p * per);
#pragma unroll
        for (int i = 0; i < KW; ++i) rv.w[i] = upto.w[i] & ~below.w[i];
    } else if (op == OP_RD && ((uint32_t)dev & gmask) != 0u) {
        clear(rv); clear(mv);
    }
    return WSTEP_OK;
}

// A work item is seg.iters consecutive groups of one stem (a length-1 segment is a single item).
// Every query has a share of the grid's blocks in proportion to its items; block j of n walks the
// query's items j, j + n, ..., so the items of a valid stem, which are the expensive ones, go to
// different blocks.  Lane a holds the candidate of a group whose last instruction has digit a
// (a + 64 in a second pass for alphabets above 64).
template <int KW, int MW>
__global__ __launch_bounds__(kWave) void k_eval_shared(const DevQuery* __restrict__ queries,
                                                       const DevSegment* __restrict__ segs, int n_segs,
                                                       const DevShare* __restrict__ shares, int n_shares) {
    __shared__ uint16_t sdig[kMaxPatterns * 5];              // digit -> (pattern id << 3) | op
    __shared__ uint32_t sshape[kMaxPatterns];                // pattern id -> lg | ls << 4 | master << 8 | participating devices << 16
    __shared__ unsigned long long spart[kMaxPatterns];       // pattern id -> bit d set iff device d takes part
    __shared__ DevSegment sseg[P2_MAX_LEN + 1];              // the segments of this block's query (one per program length)
    const int lane = threadIdx.x;
    // The share (hence the query) this block works for: the last one whose first_block <= blockIdx.x.
    // The lanes read 64 table entries at a time, so the search costs one memory round trip per 64 shares.
    DevShare sh;
    {
        static_assert(sizeof(DevShare) == 32, "a share is read as two 16-byte words");
        sh.first_block = 0; sh.n_blocks = 1; sh.first_item = 0; sh.n_items = 0; sh.query = 0; sh.first_seg = 0; sh.n_segs = 0; sh.cut_log = 0;
        for (int base = 0; base < n_shares; base += kWave) {
            const int i = base + lane;
            uint4 lo = make_uint4(0u, 0u, 0u, 0u), hi = lo;
            if (i < n_shares) {
                const uint4* sp = reinterpret_cast<const uint4*>(shares + i);
                lo = sp[0]; hi = sp[1];
            }
            const int n_le = __popcll(__ballot(i < n_shares && lo.x <= blockIdx.x));
            if (n_le > 0) {
                const int src = n_le - 1;
                sh.first_block = (uint32_t)__builtin_amdgcn_readlane((int)lo.x, src);
                sh.n_blocks = (uint32_t)__builtin_amdgcn_readlane((int)lo.y, src);
                sh.first_item = (uint32_t)__builtin_amdgcn_readlane((int)lo.z, src);
                sh.n_items = (uint32_t)__builtin_amdgcn_readlane((int)lo.w, src);
                sh.query = __builtin_amdgcn_readlane((int)hi.x, src);
                sh.first_seg = __builtin_amdgcn_readlane((int)hi.y, src);
                sh.n_segs = __builtin_amdgcn_readlane((int)hi.z, src);
                sh.cut_log = __builtin_amdgcn_readlane((int)hi.w, src);
            }
            if (n_le < kWave) break;
        }
    }
    // everything else the block needs from memory is asked for at once: the query's tables, its segments
    // and a few scalars
    const DevQuery* const qp = queries + sh.query;
    const DevQuery& q = *qp;
    for (int i = lane; i < q.n_patterns; i += kWave) { sshape[i] = q.reg_shape[i]; spart[i] = q.reg_part[i]; }
    for (int i = lane; i < q.alphabet; i += kWave) sdig[i] = q.instr_of_digit[i];
    if (lane < sh.n_segs) sseg[lane] = segs[sh.first_seg + lane];
    const int R = q.R;
    const int devs = R > 32 ? 64 : 32;
    const int dev = lane & (devs - 1);
    const uint32_t I = (uint32_t)q.alphabet;
    const uint32_t magic = q.magic_alphabet;            // ceil(2^32 / I): v / I == umulhi(v, magic) for v < 2^23
    const Words<KW> all_rows = full_mask<KW>(q.k);
    const Words<MW> all_cols = full_mask<MW>(R);
    const uint32_t sum_part = q.reg_sum_part;           // participating devices summed over the alphabet
    __syncthreads();
    DevSegment seg;
    int len = 1;
    uint32_t items_log = 0;                             // a stem is cut into 2^items_log items of seg.iters groups
    unsigned long long steps = 0, members = 0, evaluated = 0, evaluated_members = 0;   // wave-uniform totals of this block
    const uint32_t end_item = sh.first_item + sh.n_items;
    const uint32_t blk = blockIdx.x - sh.first_block;
    uint32_t turn = 0;                                  // units of the earlier segments, modulo the share's blocks
    // The blocks of a share take the units of its segments in turn.  A unit is one item, or, where an item is
    // a whole stem of at least three instructions, the `alphabet` stems that differ in their last instruction
    // only: their common part is worked out once per unit, and a unit whose common part is invalid is
    // settled as a whole.
    for (int sgi = 0; sgi < sh.n_segs; ++sgi) {
    seg = sseg[sgi];
    const uint32_t seg_end = sgi + 1 < sh.n_segs ? sseg[sgi + 1].first_block : end_item;
    len = seg.len;
    items_log = len >= 2 ? (uint32_t)sh.cut_log : 0u;
    const bool runs = items_log == 0u && len >= 5;
    // (a run of `alphabet` stems is cut into parts where the share would otherwise have fewer than about 32
    // units per block: long units balance badly)
    const uint32_t seg_items = seg_end - seg.first_block;
    uint32_t parts = 1;
    if (runs) {
        const uint32_t n_runs = seg_items / I;
        while (parts < I && n_runs * parts < 32u * sh.n_blocks) parts *= 2u;
        if (parts > I) parts = I;
    }
    const uint32_t ulen = runs ? (I + parts - 1u) / parts : 1u;             // stems of a unit
    const uint32_t n_units = runs ? (seg_items / I) * parts : seg_items;
    const uint32_t u0 = (blk + sh.n_blocks - turn) % sh.n_blocks;
    turn = (turn + n_units % sh.n_blocks) % sh.n_blocks;
    // one unit; kRuns: its stems share all but their last instruction
    auto do_unit = [&](auto runs_c, const uint32_t u) {
    constexpr bool kRuns = decltype(runs_c)::value;
    // the state after the unit's common instructions (the first len-3 of the stem), once it is known
    bool have_common = false;
    Words<KW> p_rv = all_rows;
    Words<MW> p_mv = all_cols;
    uint32_t p_ran = 0, p_visited = 0;
    int p_rc = WSTEP_OK;
    uint32_t item0 = seg.first_block + u, unit = 1u;
    if (kRuns) {
        const uint32_t run = u / parts, piece = u - run * parts;
        const uint32_t lo = piece * ulen, hi = lo + ulen < I ? lo + ulen : I;
        item0 = seg.first_block + run * I + lo;
        unit = hi > lo ? hi - lo : 0u;
    }
    for (uint32_t ju = 0; ju < unit; ++ju) {
        const uint32_t item = item0 + ju;
        // the item's stem (number S, instruction t at digit dg[t], t < len-2) and its groups: the prefix's
        // last instruction runs over the digits dlast0 .. dlast0 + n_here - 1
        const uint32_t rel = item - seg.first_block;
        const uint32_t S = rel >> items_log;
        const uint32_t dlast0 = (rel - (S << items_log)) * (uint32_t)seg.iters;
        if (len >= 2 && dlast0 >= I) continue;           // the stem has fewer groups than items: nothing here
        const uint32_t n_here = len >= 2 ? (I - dlast0 < (uint32_t)seg.iters ? I - dlast0 : (uint32_t)seg.iters) : 1u;
        if (kRuns && have_common && p_rc == WSTEP_INVALID) {
            // the common part is invalid: every candidate of the unit's remaining stems stops inside it
            const unsigned long long rest = (unsigned long long)(unit - ju) * (unsigned long long)(n_here * I);
            steps += rest * p_ran;
            members += rest * p_visited;
            break;
        }
        uint32_t dg[P2_MAX_LEN];
        {
            uint32_t rem = S;
            const bool small = S < (1u << 23);           // then a multiplication divides by the alphabet
#pragma unroll
            for (int t = P2_MAX_LEN - 3; t >= 0; --t) {
                if (t < len - 2) {
                    const uint32_t nx = small ? __umulhi(rem, magic) : rem / I;
                    dg[t] = rem - nx * I; rem = nx;
                } else dg[t] = 0;
            }
        }
        // offset in the segment of the first candidate of the item's first group
        unsigned long long first_off = len >= 2 ? ((unsigned long long)S * I + dlast0) * I : 0ull;
        // the stem's state; Sec. 3.5: device i holds column i in every row
        Words<KW> c_rv = all_rows;
        Words<MW> c_mv;
#pragma unroll
        for (int i = 0; i < MW; ++i) c_mv.w[i] = (i == (dev >> 5)) ? (1u << (dev & 31)) : 0u;
        uint32_t c_ran = 0, c_visited = 0;
        int c_rc = WSTEP_OK;
        if (kRuns && have_common) { c_rv = p_rv; c_mv = p_mv; c_ran = p_ran; c_visited = p_visited; c_rc = p_rc; }
#pragma unroll
        for (int t = 0; t < P2_MAX_LEN - 2; ++t) {
            if (t < len - 2 && c_rc == WSTEP_OK && !(kRuns && have_common && t < len - 3)) {
                const uint32_t ins0 = sdig[dg[t]];
                const uint32_t shape = sshape[ins0 >> 3];
                ++c_ran;
                c_visited += shape >> 16;
                ++evaluated; evaluated_members += shape >> 16;
                const int op0 = (int)(ins0 & 7u);
                if (t == 0) c_rc = first_wave_step<KW, MW>(c_rv, c_mv, dev, op0, (int)(shape & 15u), (int)((shape >> 4) & 15u), spart[ins0 >> 3], q.k);
                else c_rc = wave_step<KW, MW>(c_rv, c_mv, dev, op0, (int)(shape & 15u), (int)((shape >> 4) & 15u), spart[ins0 >> 3], devs);
            }
            if (kRuns && !have_common && t == len - 4) {
                // (the common part of the unit's stems ends here)
                p_rv = c_rv; p_mv = c_mv; p_ran = c_ran; p_visited = c_visited; p_rc = c_rc;
            }
        }
        if (kRuns) have_common = true;
        if (c_rc == WSTEP_INVALID) {
            // every candidate of the item stops inside the stem
            steps += (unsigned long long)(n_here * I) * c_ran;
            members += (unsigned long long)(n_here * I) * c_visited;
            continue;
        }
        if (c_rc == WSTEP_GIVE_UP) {
            // the stem's own state leaves the compact form: the literal engine gets the item's groups in
            // entries of up to kStemGroups groups, rebuilds the stem once per entry and evaluates (and counts)
            // every group from there
            if (lane == 0) {
                const uint32_t n_entries = (n_here + kStemGroups - 1u) / kStemGroups;
                const uint32_t pos = atomicAdd(&q.counters->n_rerun, n_entries);
                for (uint32_t j = 0; j < n_entries; ++j) {
                    const uint32_t cnt = n_here - kStemGroups * j < kStemGroups ? n_here - kStemGroups * j : kStemGroups;
                    if (pos + j < q.rerun_cap)
                        q.rerun_idx[pos + j] = kStemEntry | ((unsigned long long)cnt << kStemCountShift) |
                                               (seg.first_index + first_off + (unsigned long long)(kStemGroups * j) * I);
                }
                atomicAdd(&q.counters->n_rerun_groups, n_here);
            }
            continue;
        }
        uint32_t item_steps = 0, item_members = 0;   // an item is at most alphabet / 4 groups: these stay below 2^32
        for (uint32_t gi = 0; gi < n_here; ++gi, first_off += I) {
            Words<KW> rv = c_rv;
            Words<MW> mv = c_mv;
            int rc = c_rc;
            uint32_t g_ran = c_ran, g_visited = c_visited;
            if (rc == WSTEP_OK && len >= 2) {
                const uint32_t ins0 = sdig[dlast0 + gi];
                const uint32_t shape = sshape[ins0 >> 3];
                ++g_ran;
                g_visited += shape >> 16;
                ++evaluated; evaluated_members += shape >> 16;
                rc = wave_step<KW, MW>(rv, mv, dev, (int)(ins0 & 7u), (int)(shape & 15u), (int)((shape >> 4) & 15u), spart[ins0 >> 3], devs);
            }
            if (rc == WSTEP_GIVE_UP) {
                // the literal engine evaluates (and counts) the group from its first instruction: it gets the
                // index of the group's first candidate
                if (lane == 0) {
                    const uint32_t pos = atomicAdd(&q.counters->n_rerun, 1u);
                    if (pos < q.rerun_cap) q.rerun_idx[pos] = seg.first_index + first_off;
                    atomicAdd(&q.counters->n_rerun_groups, 1u);
                }
            } else if (rc == WSTEP_INVALID) {
                item_steps += I * g_ran;
                item_members += I * g_visited;
            } else {
                // every candidate applies its last instruction
                item_steps += I * (g_ran + 1u);
                item_members += I * g_visited + sum_part;
                // The last instruction matters only through the goal test.  The goal can only come from an
                // AllReduce on devices that all hold every chunk, from an AllGather on devices whose chunks
                // all carry every column, or from a Broadcast whose roots (device 0 is one in every pattern)
                // are at the goal already; ReduceScatter and Reduce leave members short of chunks.
                // Candidates that pass this test apply their last instruction to a copy of the group's
                // state, one after the other, again with the wavefront's lanes as devices.
                const uint32_t rows_off = fold_xor(rv, all_rows), cols_off = fold_xor(mv, all_cols);
                const bool rows_full = !__any(dev < R && rows_off != 0u);
                const bool cols_full = !__any(dev < R && cols_off != 0u);
                const unsigned long long complete = __ballot(dev < R && (rows_off | cols_off) == 0u) & (R >= 64 ? ~0ull : ((1ull << R) - 1ull));
                const bool root_done = (complete & 1ull) != 0ull;                                 // lane 0 is device 0
                if (rows_full || cols_full || root_done) {
                    for (uint32_t a0 = 0; a0 < I; a0 += kWave) {
                        const uint32_t a = a0 + (uint32_t)lane;
                        const uint32_t my_ins = a < I ? sdig[a] : 0u;
                        const int my_op = (int)(my_ins & 7u);
                        const bool may = a < I && ((my_op == OP_AR && rows_full) || (my_op == OP_AG && cols_full) || (my_op == OP_BC && root_done));
                        bool goal = false;
                        for (unsigned long long left = __ballot(may); left != 0ull; left &= left - 1ull) {
                            const int l = __ffsll((long long)left) - 1;
                            const uint32_t ins0 = sdig[a0 + (uint32_t)l];
                            const uint32_t shape = sshape[ins0 >> 3];
                            const int op2 = (int)(ins0 & 7u), lg2 = (int)(shape & 15u), ls2 = (int)((shape >> 4) & 15u);
                            ++evaluated; evaluated_members += shape >> 16;
                            // goal: every device holds every chunk with the columns of the whole group
                            bool reached;
                            if (op2 == OP_AR) reached = judge_allreduce<MW>(mv, dev, lg2, ls2, spart[ins0 >> 3], R, all_cols);
                            else if (op2 == OP_AG) reached = judge_allgather<KW>(rv, dev, lg2, ls2, spart[ins0 >> 3], R, all_rows);
                            else reached = judge_broadcast(complete, lg2, ls2, spart[ins0 >> 3], R);
                            if (lane == l) goal = reached;
                        }
                        if (goal) {
                            const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
                            if (pos < q.valid_cap) q.valid_idx[pos] = seg.first_index + first_off + a;
                        }
                    }
                }
            }
        }
        steps += item_steps;
        members += item_members;
    }
    };
    for (uint32_t u = u0; u < n_units; u += sh.n_blocks) {
        if (runs) do_unit(std::true_type{}, u);
        else do_unit(std::false_type{}, u);
    }
    }
    if (lane == 0 && (steps | evaluated) != 0ull) {
        atomicAdd(&qp->counters->steps[blockIdx.x % kCounterStripes], steps);
        atomicAdd(&qp->counters->members[blockIdx.x % kCounterStripes], members);
        atomicAdd(&qp->counters->evaluated[blockIdx.x % kCounterStripes], evaluated);
        atomicAdd(&qp->counters->evaluated_members[blockIdx.x % kCounterStripes], evaluated_members);
    }
}

// Cost of valid programs: one wavefront per program re-runs it with the lanes as devices and adds up
// the ring alpha-beta step times (hierarchical cost model, see p2.h).  The chunk set that sets a
// group's bytes is the members' common one before an AllReduce-like step, the root's before a
// Broadcast, the gathered one after an AllGather.  A program whose state leaves the compact form
// gets NaN costs; the literal cost kernel fills those rows.
template <int KW, int MW>
__global__ __launch_bounds__(kWave) void k_cost_shared(const DevQuery* __restrict__ queries,
                                                       const DevPostSeg* __restrict__ segs, int n_segs,
                                                       const unsigned long long* __restrict__ valid,
                                                       const unsigned long long* __restrict__ valid2,
                                                       unsigned long long* __restrict__ sorted,
                                                       p2_program* __restrict__ out_prog, double* __restrict__ out_cost) {
    __shared__ uint32_t srows[kWave];                // chunks that set the bytes of the group whose first device is d
    const DevPostSeg seg = find_post_seg(segs, n_segs, blockIdx.x);
    const DevQuery& q = queries[seg.query];
    const int lane = threadIdx.x;
    const int devs = q.R > 32 ? 64 : 32;
    const int dev = lane & (devs - 1);
    // The block's program is entry j of the query's unordered list of valid indices; its place in the
    // ascending order is the number of smaller entries (distinct keys), counted here by the wavefront, so
    // no separate sort runs for these queries.  A list whose in_off has bit 63 set is in valid2.
    const unsigned long long* in = (seg.in_off >> 63) ? valid2 + (seg.in_off & ~(1ull << 63)) : valid + seg.in_off;
    const unsigned long long idx = in[blockIdx.x - seg.first_block];
    uint32_t rank = 0;
    for (uint32_t t = (uint32_t)lane; t < seg.count; t += kWave) rank += in[t] < idx ? 1u : 0u;
    for (int off = 32; off > 0; off >>= 1) rank += __shfl_xor(rank, off, kWave);
    const size_t i = seg.out_off + rank;
    if (lane == 0) sorted[i] = idx;
    int len = 1;
    while (len < q.max_len && idx >= q.base[len + 1]) ++len;
    uint32_t digit[P2_MAX_LEN];
    {
        unsigned long long rem = idx - q.base[len];
        const unsigned long long I = (unsigned long long)q.alphabet;
#pragma unroll
        for (int t = P2_MAX_LEN - 1; t >= 0; --t) {
            if (t < len) { const unsigned long long nx = rem / I; digit[t] = (uint32_t)(rem - nx * I); rem = nx; }
            else digit[t] = 0;
        }
    }
    // Sec. 3.5: device i holds column i in every row
    Words<KW> rv = full_mask<KW>(q.k);
    Words<MW> mv;
#pragma unroll
    for (int w = 0; w < MW; ++w) mv.w[w] = (w == (dev >> 5)) ? (1u << (dev & 31)) : 0u;
    double sum_alpha = 0.0, sum_beta = 0.0;
    bool ok = true;
    p2_program pr;
    pr.index = idx;
    pr.len = (uint8_t)len;
#pragma unroll
    for (int t = 0; t < P2_MAX_LEN; ++t) {
        pr.instr[t] = 0;
        if (t < len) {
            const uint32_t ins = q.instr_of_digit[digit[t]];
            const int pid = (int)(ins >> 3), op = (int)(ins & 7u);
            pr.instr[t] = (uint8_t)(pid * 5 + op);
            if (ok) {
                const uint32_t shape = q.reg_shape[pid];
                const int before = popcount(rv);
                ok = wave_step<KW, MW>(rv, mv, dev, op, (int)(shape & 15u), (int)((shape >> 4) & 15u), q.reg_part[pid], devs) == WSTEP_OK;
                if (ok) {
                    __syncthreads();
                    if (lane < devs) srows[lane] = (uint32_t)(op == OP_AG ? popcount(rv) : before);
                    __syncthreads();
                    // bandwidth term: the most loaded uplink
                    const DevPattern& P = q.pat[pid];
                    const DevRows& rw = *q.rows;
                    double best = 0.0;
                    for (int row = rw.pat_begin[pid] + lane; row < rw.pat_begin[pid + 1]; row += kWave) {
                        long long dot = 0;
                        for (int e = rw.row_ptr[row]; e < rw.row_ptr[row + 1]; ++e) {
                            const uint32_t ent = rw.entries[e];
                            dot += (long long)entry_cnt(ent) * (long long)srows[entry_base(ent)];
                        }
                        best = fmax(best, (double)dot * q.inv_bw[rw.row_level[row]]);
                    }
                    for (int off = 32; off > 0; off >>= 1) best = fmax(best, __shfl_xor(best, off, kWave));
                    double ring_steps, mult;
                    step_factors(op, P.g, q.algo, ring_steps, mult);
                    sum_alpha += ring_steps * q.alpha[P.span_level];
                    sum_beta += (mult / (double)q.k) * best;
                }
            }
        }
    }
    if (lane == 0) out_prog[i] = pr;
    if (lane < q.n_msg)
        out_cost[i * q.n_msg + lane] = ok ? sum_alpha + q.msg_bytes[lane] * sum_beta : __longlong_as_double(0x7ff8000000000000ll);
}

inline int word_class_s(int bits) {
    const int w = (bits + 31) / 32;
    return w <= 1 ? 1 : w <= 2 ? 2 : w <= 4 ? 4 : w <= 8 ? 8 : 16;
}

}  // namespace

#define P2_SHARED_DISPATCH(KW, MW, GO)                  \
    switch (KW * 10 + MW) {                             \
    case 11: GO(1, 1) break;                            \
    case 12: GO(1, 2) break;                            \
    case 21: GO(2, 1) break;                            \
    case 22: GO(2, 2) break;                            \
    case 41: GO(4, 1) break;                            \
    case 42: GO(4, 2) break;                            \
    case 81: GO(8, 1) break;                            \
    case 82: GO(8, 2) break;                            \
    case 161: GO(16, 1) break;                          \
    case 162: GO(16, 2) break;                          \
    default: return hipErrorInvalidValue;               \
    }

hipError_t launch_eval_shared(const DevQuery* queries, const DevSegment* segs, int n_segs, const DevShare* shares,
                              int n_shares, unsigned grid, int max_R, int max_k, hipStream_t stream) {
    if (n_segs == 0 || n_shares == 0 || grid == 0) return hipSuccess;
    const int KW = word_class_s(max_k), MW = word_class_s(max_R);
#define P2_GO(KWV, MWV) \
    hipLaunchKernelGGL((k_eval_shared<KWV, MWV>), dim3(grid), dim3(kWave), 0, stream, queries, segs, n_segs, shares, n_shares);
    P2_SHARED_DISPATCH(KW, MW, P2_GO)
#undef P2_GO
    return hipGetLastError();
}

hipError_t launch_cost_shared(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks, int max_R,
                              int max_k, const unsigned long long* valid, const unsigned long long* valid2,
                              unsigned long long* sorted, p2_program* progs, double* costs, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const int KW = word_class_s(max_k), MW = word_class_s(max_R);
#define P2_GO(KWV, MWV) \
    hipLaunchKernelGGL((k_cost_shared<KWV, MWV>), dim3(blocks), dim3(kWave), 0, stream, queries, segs, n_segs, valid, valid2, sorted, progs, costs);
    P2_SHARED_DISPATCH(KW, MW, P2_GO)
#undef P2_GO
    return hipGetLastError();
}

}  // namespace p2
