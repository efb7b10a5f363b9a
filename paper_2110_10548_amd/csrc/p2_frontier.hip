// Frontier evaluation: the enumeration by program size of Sec. 3.5 with its pruning -- a prefix
// whose step violates a rule is never extended -- for candidate spaces too large to walk index by
// index (10^11 programs per query at four hierarchy levels and size limit 6).
//
// A frontier holds the valid, non-goal prefixes of one length of one *enumeration*: the queries of
// a batch that agree in everything validity depends on (reduction group, chunks, patterns, alphabet,
// size limit) are enumerated together, and every prefix carries, for each of them, the simulated time
// of its instructions so far (one latency sum and one per-byte sum in fp64), because the time of a
// step depends on the state before it and on the query's links only.  A program's cost is therefore
// complete the moment it reaches the goal, and no valid program is ever simulated a second time.
//
// States and prefixes are kept apart.  What the rules say about the next instruction depends on the
// state alone, and many prefixes end in the same state, so a level holds its distinct states once
// (two lists, see below) and its prefixes as records: instructions, sums, index of the state.
//
// State.  From the init state every rule of Sec. 3.2 keeps the non-empty rows of a device equal to
// each other unless an AllGather joins members whose rows carry different column sets
// (p2_compact.hip).  Here a device holds up to TWO (chunk set, contribution mask) pairs: the rows of
// pair 0 all carry mask 0, the rows of pair 1 mask 1; the chunk sets are disjoint, pair 0 owns the
// lowest row, an empty pair has an empty mask, and two pairs never carry the same mask.  States
// whose devices all have one pair are one plane of R x WQ 16-byte quads in HBM ("one-pair list"),
// the others two planes ("two-pair list").  The rules on two-pair states:
//   AllReduce-like : members must hold the same rows.  Their pairs must be *aligned*: every member
//                    with two pairs splits the rows the same way (members with one pair fit any
//                    split).  Then the rule is checked and carried out plane by plane.  A group
//                    that is not aligned cannot be judged in this form: the prefixes of the state
//                    are handed to the literal kernels, which rebuild the literal state from the
//                    instructions.
//   AllGather      : rows pairwise disjoint, nobody empty; the result has one pair per distinct
//                    mask among the members' pairs.  More than two: the child is a "literal"
//                    prefix (it keeps only its instructions; p2_literal.hip takes it from there).
//   Broadcast      : compared pair against pair (a row's mask is its pair's mask).
// One level, in launch order (the host waits once, after `expand`, and sizes the next level's
// buffers exactly from the counts, so nothing overflows):
//   goal filter      : the last level only, where nothing but goals counts: the states from which no
//                      instruction can end at the goal get a row of invalid codes, the others are listed.
//   classify         : block = one distinct state, its planes in LDS, wavefronts over patterns,
//                      lanes = (device slot, 16-byte quad); writes a code per instruction, how many of
//                      them are survivors by kind, and adds up the children of the states it judged.
//   expand           : for every prefix, the survivors among its extensions (from its state's counts
//                      and codes) with their places in the next prefix lists / among the goals.
//   children         : for every (state, valid instruction), the child's place in the next state lists.
//   materialize      : block = one child: parent planes into LDS, the instruction applied in place,
//                      the child streamed out with its hash; what the step adds to every query's sums.
//   dedup + verify   : children with equal hashes are compared word by word; one of every group of
//                      equal states stands for the others.
//   prefixes         : the next level's prefix records (sums = parent's + step's) and the goals.
#include "p2_compact_dev.h"

namespace p2 {

namespace {


enum : int { CODE_INVALID = 0, CODE_PREFIX = 1, CODE_GOAL = 2, CODE_PREFIX_LITERAL = 3, CODE_PREFIX2 = 4, CODE_UNKNOWN = 5 };
constexpr int kFromTwoPair = 0x100;       // survivor code bit: the parent is an entry of the two-pair list

template <int N>
__device__ inline Words<N> zero_words() {
    Words<N> z;
#pragma unroll
    for (int i = 0; i < N; ++i) z.w[i] = 0u;
    return z;
}
template <int N>
__device__ inline Words<N> or_words(const Words<N>& a, const Words<N>& b) {
    Words<N> o;
#pragma unroll
    for (int i = 0; i < N; ++i) o.w[i] = a.w[i] | b.w[i];
    return o;
}
template <int N>
__device__ inline Words<N> and_words(const Words<N>& a, const Words<N>& b) {
    Words<N> o;
#pragma unroll
    for (int i = 0; i < N; ++i) o.w[i] = a.w[i] & b.w[i];
    return o;
}
template <int N>
__device__ inline Words<N> andn_words(const Words<N>& a, const Words<N>& b) {      // a without b
    Words<N> o;
#pragma unroll
    for (int i = 0; i < N; ++i) o.w[i] = a.w[i] & ~b.w[i];
    return o;
}
// Layout of a state plane, in HBM and in LDS: per device the chunk set padded to whole 16-byte quads, then the
// contribution mask padded likewise (the padding stays zero), so that a device is WQ quads and the
// wavefront-wide kernels read it with 128-bit accesses.
template <int KW, int MW>
struct FL {
    static constexpr int QK = (KW + 3) / 4, QM = (MW + 3) / 4, WQ = QK + QM;   // quads: rows, mask, device
    static constexpr int WS = WQ * 4, MO = QK * 4;                             // words per device, offset of the mask
};
template <int KW, int MW>
__device__ inline Slot<KW, MW> fload(const uint32_t* plane, int dev) {
    const uint32_t* p = plane + dev * FL<KW, MW>::WS;
    Slot<KW, MW> s;
#pragma unroll
    for (int i = 0; i < KW; ++i) s.r.w[i] = p[i];
#pragma unroll
    for (int i = 0; i < MW; ++i) s.m.w[i] = p[FL<KW, MW>::MO + i];
    return s;
}
template <int KW, int MW>
__device__ inline void fstore(uint32_t* plane, int dev, const Words<KW>& r, const Words<MW>& m) {
    uint32_t* p = plane + dev * FL<KW, MW>::WS;
#pragma unroll
    for (int i = 0; i < KW; ++i) p[i] = r.w[i];
#pragma unroll
    for (int i = 0; i < MW; ++i) p[FL<KW, MW>::MO + i] = m.w[i];
}

// ---- classification, a wavefront per pattern ----------------------------------------------------------
// Block = one prefix (its planes in LDS), wavefront = one pattern at a time, all rules of that pattern at
// once.  A lane is (slot, quad): the 8 lanes of a slot read one device with one 128-bit access each, so a
// wavefront has 8 devices in flight; the slots of a wavefront walk 8 groups of the pattern side by side,
// member after member (patterns with fewer than 8 groups give every group several slots, which share
// its members).  Per 32-bit word of the state a lane keeps, over the members of its group: the union,
// the intersection, the bits seen in two members, and the first member's word.  Every premise of Sec. 3.2
// on one-pair states is a statement about those:
//   same rows on every member        union == intersection (chunk-set words)
//   no contribution reduced twice    no mask bit seen twice
//   AllGather: rows held once        no chunk-set bit seen twice;  nobody empty: a flag per device
//   Broadcast: root knows more       union == the first member's words, and union != intersection somewhere
//   results: AllReduce leaves (rows, united mask), AllGather (united rows, mask), Broadcast the root's pair
// On two-pair states the AllReduce-like rules are the same statements plane by plane (plane B of a member
// with one pair is its only pair), plus: the members that have two pairs split their rows alike.  What
// these word-wise accumulators cannot decide goes to routines of its own, each a second walk of the pattern by
// one wavefront: an AllGather of members with different masks (how many masks?), a ReduceScatter of a split
// group (does a block straddle the split?), a Broadcast among two-pair devices that passes the
// necessary conditions checked here.
// The kernel writes a code per instruction of the alphabet for every entry it judges; the survivors are listed
// afterwards (k_front_expand), for every entry of the list from the codes of the entry that stands for its state.
constexpr int kClsThreads = 512, kClsWaves = kClsThreads / 64;

__device__ inline uint4 q_or(uint4 a, uint4 b) { return make_uint4(a.x | b.x, a.y | b.y, a.z | b.z, a.w | b.w); }
__device__ inline uint4 q_and(uint4 a, uint4 b) { return make_uint4(a.x & b.x, a.y & b.y, a.z & b.z, a.w & b.w); }
__device__ inline uint4 q_andn(uint4 a, uint4 b) { return make_uint4(a.x & ~b.x, a.y & ~b.y, a.z & ~b.z, a.w & ~b.w); }
__device__ inline uint4 q_xor(uint4 a, uint4 b) { return make_uint4(a.x ^ b.x, a.y ^ b.y, a.z ^ b.z, a.w ^ b.w); }
__device__ inline bool q_any(uint4 a) { return (a.x | a.y | a.z | a.w) != 0u; }
__device__ inline int q_popc(uint4 a) { return __popc(a.x) + __popc(a.y) + __popc(a.z) + __popc(a.w); }
__device__ inline uint4 q_zero() { return make_uint4(0u, 0u, 0u, 0u); }
__device__ inline uint4 q_ones() { return make_uint4(~0u, ~0u, ~0u, ~0u); }
__device__ inline uint4 q_shfl_xor(uint4 a, int m) {
    return make_uint4(__shfl_xor(a.x, m, 64), __shfl_xor(a.y, m, 64), __shfl_xor(a.z, m, 64), __shfl_xor(a.w, m, 64));
}
__device__ inline uint4 q_shfl(uint4 a, int src) {
    return make_uint4(__shfl(a.x, src, 64), __shfl(a.y, src, 64), __shfl(a.z, src, 64), __shfl(a.w, src, 64));
}
// union / intersection / seen-twice of a run of members; two runs put together
struct QAcc {
    uint4 o, a, t;
    __device__ inline void init() { o = q_zero(); a = q_ones(); t = q_zero(); }
    __device__ inline void add(uint4 v) { t = q_or(t, q_and(v, o)); o = q_or(o, v); a = q_and(a, v); }
    // the same, or nothing at all (v must be zero where `on` is false)
    __device__ inline void add_if(uint4 v, bool on) {
        t = q_or(t, q_and(v, o)); o = q_or(o, v);
        a = make_uint4(a.x & (on ? v.x : ~0u), a.y & (on ? v.y : ~0u), a.z & (on ? v.z : ~0u), a.w & (on ? v.w : ~0u));
    }
    __device__ inline void merge_xor(int m) {
        const uint4 oo = q_shfl_xor(o, m), oa = q_shfl_xor(a, m), ot = q_shfl_xor(t, m);
        t = q_or(q_or(t, ot), q_and(o, oo)); o = q_or(o, oo); a = q_and(a, oa);
    }
    __device__ inline bool differ() const { return q_any(q_xor(o, a)); }
};

constexpr uint32_t kFlagEmpty = 1u, kFlagGoal = 2u, kFlagTwo = 4u;
// what the groups of a pattern have shown so far (one word per pattern)
constexpr uint32_t kPfBadRed = 1u, kPfBadB = 2u, kPfUnal = 4u, kPfBadRs = 8u, kPfBadAg = 16u, kPfChanged = 32u, kPfAgUneq = 64u,
                   kPfBadBc1 = 128u, kPfBcFail = 256u, kPfAnyTwo = 512u, kPfNgAr = 1024u, kPfNgAg = 2048u, kPfNgBc = 4096u,
                   kPfPatTwo = 8192u;
constexpr int kClsChunks = 8;          // a pattern's groups go to the wavefronts in at most this many runs
struct ClsItem { uint16_t pid, first_batch, n_batches; };

// Sum over the 8 lanes of a slot, in every lane of the slot, with data-parallel-primitive moves (all lanes active):
// swap neighbours, swap pairs, mirror the half row.
__device__ inline int sum_slot(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);      // quad_perm [1, 0, 3, 2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);      // quad_perm [2, 3, 0, 1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);     // row_half_mirror
    return v;
}

// The lowest n set bits of w (none for n <= 0, all for n >= popcount).
__device__ inline uint32_t low_bits(uint32_t w, int n) {
    if (n <= 0) return 0u;
    if (n >= __popc(w)) return w;
    int pos = 0;                                   // position of the n-th set bit: binary search on prefix counts
#pragma unroll
    for (int step = 16; step > 0; step >>= 1)
        if (__popc(w & ((1u << (pos + step)) - 1u)) < n) pos += step;
    return w & ((2u << pos) - 1u);
}

// ---- pieces of the classification kernel ------------------------------------------------------------------
// What a lane knows about its place in the wavefront and about the prefix whose planes lie in LDS.
template <int KW, int MW, int NP>
struct ClsLane {
    const uint4* ldsq;             // NP planes of [R][WQ] quads
    const uint8_t* flags;          // per device: kFlag* bits
    int R, plane_q;
    int lane, slot, qd;
    bool is_row, is_mask, has_quad;
    uint4 goal_quad;               // this lane's quad of a device at the goal
};
// what a run of a pattern's groups has shown (the same in every lane)
struct ClsFound { uint32_t bits; int goal_part, two_part; };

// Per device: is it empty, is it at the goal, does it hold two pairs.  The wavefront takes the devices
// first + slot, first + stride + slot, ...; at_goal and with_two come back summed over the wavefront.
// With `shortfalls`, also (for the filter of the last level): rows_short = devices that lack a row, cols_short =
// devices that hold rows whose columns are not all there.
template <int KW, int MW, int NP>
__device__ inline void cls_flags(const ClsLane<KW, MW, NP>& c, uint8_t* flags, int first, int stride, int& at_goal, int& with_two,
                                 bool shortfalls, int& rows_short, int& cols_short) {
    using L = FL<KW, MW>;
    at_goal = 0; with_two = 0; rows_short = 0; cols_short = 0;
    for (int d0 = first; d0 < c.R; d0 += stride) {
        const int d = d0 + c.slot;
        const bool act = d < c.R && c.has_quad;
        const uint4 v = act ? c.ldsq[d * L::WQ + c.qd] : q_zero();
        const uint4 v1 = (NP == 2 && act) ? c.ldsq[c.plane_q + d * L::WQ + c.qd] : q_zero();
        const unsigned long long nz = __ballot(act && c.is_row && q_any(v));
        const unsigned long long ng = __ballot(act && q_any(q_xor(v, c.goal_quad)));
        const unsigned long long n2 = NP == 2 ? __ballot(act && c.is_row && q_any(v1)) : 0ull;
        unsigned long long rs = 0ull, m0 = 0ull, m1 = 0ull;
        if (shortfalls) {
            rs = __ballot(act && c.is_row && q_any(q_xor(q_or(v, v1), c.goal_quad)));
            m0 = __ballot(act && c.is_mask && q_any(q_xor(v, c.goal_quad)));
            m1 = NP == 2 ? __ballot(act && c.is_mask && q_any(q_xor(v1, c.goal_quad))) : 0ull;
        }
        if (c.qd == 0 && d < c.R) {
            const int sh = c.slot * 8;
            const bool empty = ((nz >> sh) & 0xffull) == 0ull, two = ((n2 >> sh) & 0xffull) != 0ull;
            const bool goal = ((ng >> sh) & 0xffull) == 0ull && !two;
            flags[d] = (uint8_t)((empty ? kFlagEmpty : 0u) | (goal ? kFlagGoal : 0u) | (two ? kFlagTwo : 0u));
            at_goal += goal ? 1 : 0;
            with_two += two ? 1 : 0;
            rows_short += ((rs >> sh) & 0xffull) != 0ull ? 1 : 0;
            cols_short += ((!empty && ((m0 >> sh) & 0xffull) != 0ull) || (two && ((m1 >> sh) & 0xffull) != 0ull)) ? 1 : 0;
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        at_goal += __shfl_xor(at_goal, o, 64); with_two += __shfl_xor(with_two, o, 64);
        rows_short += __shfl_xor(rows_short, o, 64); cols_short += __shfl_xor(cols_short, o, 64);
    }
}

// The batches [first_batch, first_batch + n_batches) of a pattern's groups (8 slots side by side: a batch is
// 8 groups, or fewer groups with several slots each), every rule at once.  Stops early once every rule of the
// pattern has failed; with goal_ops >= 0 (the last level: bit 0 / 1 / 2 = an AllReduce / AllGather / Broadcast may
// still end at the goal) also once every rule has failed or has left some device short of the goal.
template <int KW, int MW, int NP>
__device__ inline ClsFound cls_walk(const ClsLane<KW, MW, NP>& c, const PatLds P, int first_batch, int n_batches, int goal_ops) {
    using L = FL<KW, MW>;
    const uint4* const ldsq = c.ldsq;
    const int plane_q = c.plane_q, slot = c.slot, qd = c.qd;
    const bool is_row = c.is_row, is_mask = c.is_mask;
    const uint4 goal_quad = c.goal_quad;
    const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    int spg = 1;                                         // slots that share a group
    while (spg * 2 * ng <= 8) spg *= 2;
    const int gpb = 8 / spg;                             // groups side by side
    const int my_g = slot / spg, part = slot - my_g * spg;
    const int trips = (g + spg - 1) / spg;
    bool bad_red = false, bad_b = false, unal = false, bad_rs = false, bad_ag = false, changed = false, ag_uneq = false;
    bool bad_bc1 = false, bc_fail = false, any_two = false;
    bool ng_ar = false, ng_ag = false, ng_bc = false;    // some device is not at the goal afterwards
    uint32_t fl_pat = 0;
    int goal_part = 0, two_part = 0;
    const int G_end = min(ng, (first_batch + n_batches) * gpb);
    for (int G0 = first_batch * gpb; G0 < G_end; G0 += gpb) {
        const int G = G0 + my_g;
        const bool act = G < ng && c.has_quad;
        int base = 0;
        if (P.master) base = G * gs;
        else { const int hi = div_small(G, s); base = hi * gs + (G - hi * s); }
        // row lanes: p = rows (both pairs), al = pair-0 rows of the members with two pairs
        // mask lanes: p = plane A (pair 0), sB = plane B, al = every pair's mask
        QAcc p, sB, al, i0, i1;
        p.init(); sB.init(); al.init(); i0.init(); i1.init();
        uint4 first0 = q_zero(), first1 = q_zero();
        uint32_t fl_or = 0;
        // (members in flight: four, or two where a member is two quads and five accumulators, which leave no registers for more)
        constexpr int kFlight = 2;
        for (int it0 = 0; it0 < trips; it0 += kFlight) {
            uint4 a0[kFlight], a1[kFlight];
            uint32_t ff[kFlight];
            bool on[kFlight];
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const int t = (it0 + u) * spg + part;
                on[u] = act && t < g;
                const int d = base + t * s;
                a0[u] = on[u] ? ldsq[d * L::WQ + qd] : q_zero();
                a1[u] = (NP == 2 && on[u]) ? ldsq[plane_q + d * L::WQ + qd] : q_zero();
                ff[u] = on[u] ? (uint32_t)c.flags[d] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const uint4 v0 = a0[u];
                const uint32_t f = ff[u];
                fl_or |= f;
                goal_part += (qd == 0 && (f & kFlagGoal)) ? 1 : 0;
                if constexpr (NP == 2) {
                    const uint4 v1 = a1[u];
                    const bool two = (f & kFlagTwo) != 0u;
                    two_part += (qd == 0 && two) ? 1 : 0;
                    i0.add_if(v0, on[u]); i1.add_if(v1, on[u]);
                    if (is_row) {
                        p.add_if(q_or(v0, v1), on[u]);
                        al.add_if(two ? v0 : q_zero(), two);
                    } else {
                        p.add_if(v0, on[u]);
                        sB.add_if(two ? v1 : v0, on[u]);
                        al.add_if(v0, on[u]);
                        al.add_if(two ? v1 : q_zero(), two);
                    }
                    if (it0 + u == 0 && part == 0) { first0 = v0; first1 = v1; }
                } else {
                    p.add_if(v0, on[u]);
                    if (it0 + u == 0 && part == 0) first0 = v0;
                }
            }
        }
        for (int m = 8; m < 8 * spg; m <<= 1) {          // the slots of one group put their members together
            p.merge_xor(m);
            if constexpr (NP == 2) { sB.merge_xor(m); al.merge_xor(m); i0.merge_xor(m); i1.merge_xor(m); }
            fl_or |= (uint32_t)__shfl_xor((int)fl_or, m, 64);
        }
        if (spg > 1) {
            first0 = q_shfl(first0, (slot - part) * 8 + qd);
            if constexpr (NP == 2) first1 = q_shfl(first1, (slot - part) * 8 + qd);
        }
        fl_pat |= act ? fl_or : 0u;
        const int rows = sum_slot((act && is_row) ? q_popc(p.o) : 0);
        const int sh = slot * 8;
        if constexpr (NP == 1) {
            const unsigned long long dif_slots = __ballot(act && p.differ());
            if (act) {
                const bool twice = q_any(p.t), differ = p.differ();
                if (is_row) { bad_red |= differ; bad_ag |= twice; changed |= q_any(p.o); }
                else { bad_red |= twice; ag_uneq |= differ; }
                bad_rs |= div_small(rows, g) * g != rows;
                bad_ag |= (fl_or & kFlagEmpty) != 0u;
                bad_bc1 |= q_any(q_xor(p.o, first0)) || ((dif_slots >> sh) & 0xffull) == 0ull;
                ng_ar |= q_any(q_xor(p.o, goal_quad));
                ng_ag |= q_any(q_xor(is_row ? p.o : first0, goal_quad));
                ng_bc |= q_any(q_xor(first0, goal_quad));
            }
        } else {
            const bool g_two = (fl_or & kFlagTwo) != 0u;
            const unsigned long long unal_slots = __ballot(act && is_row && g_two && al.differ());
            const unsigned long long split_slots = __ballot(act && is_mask && g_two && q_any(q_xor(p.o, sB.o)));
            const unsigned long long dif_slots = __ballot(act && (i0.differ() || i1.differ()));
            if (act) {
                const bool unal_g = ((unal_slots >> sh) & 0xffull) != 0ull, split_g = ((split_slots >> sh) & 0xffull) != 0ull;
                const bool differs_g = ((dif_slots >> sh) & 0xffull) != 0ull;
                if (is_row) { bad_red |= p.differ(); bad_ag |= q_any(p.t); changed |= q_any(p.o); }
                else { bad_red |= q_any(p.t); bad_b |= !unal_g && q_any(sB.t); ag_uneq |= al.differ(); }
                unal |= unal_g;
                any_two |= split_g;
                bad_rs |= div_small(rows, g) * g != rows;
                bad_ag |= (fl_or & kFlagEmpty) != 0u;
                // Broadcast, exact where no member of the pattern holds two pairs ...
                bad_bc1 |= q_any(q_xor(p.o, first0)) || !differs_g;
                // ... and otherwise what must hold at least: rows and masks inside the root's, someone differs
                if (is_row) bc_fail |= q_any(q_xor(p.o, q_or(first0, first1)));
                else bc_fail |= q_any(q_andn(al.o, q_or(first0, first1)));
                bc_fail |= !differs_g;
                // (what the masks of a group that is not aligned come to is not known here: cls_codes asks for this bit
                //  only where every group is aligned, and the last level's early exit must not go by a guess)
                ng_ar |= (is_row && q_any(q_xor(p.o, goal_quad))) || (!unal_g && (q_any(q_xor(p.o, goal_quad)) || split_g));
                ng_ag |= q_any(q_xor(is_row ? p.o : al.o, goal_quad));
                ng_bc |= q_any(q_xor(first0, goal_quad)) || q_any(first1);
            }
        }
        // every rule of the pattern has failed already: the other groups cannot change that
        const bool dead_red = __any(bad_red), dead_ag = __any(bad_ag), dead_bc = __any(bad_bc1 && (NP == 1 || bc_fail));
        if (dead_red && dead_ag && dead_bc) break;
        if (goal_ops >= 0 && (!(goal_ops & 1) || dead_red || __any(ng_ar)) && (!(goal_ops & 2) || dead_ag || __any(ag_uneq) || __any(ng_ag)) &&
            (!(goal_ops & 4) || dead_bc || __any(ng_bc)))
            break;
    }
    ClsFound f;
    uint32_t bits = 0;
    bits |= __any(bad_red) ? kPfBadRed : 0u; bits |= __any(bad_b) ? kPfBadB : 0u; bits |= __any(unal) ? kPfUnal : 0u;
    bits |= __any(bad_rs) ? kPfBadRs : 0u; bits |= __any(bad_ag) ? kPfBadAg : 0u; bits |= __any(changed) ? kPfChanged : 0u;
    bits |= __any(ag_uneq) ? kPfAgUneq : 0u; bits |= __any(bad_bc1) ? kPfBadBc1 : 0u; bits |= __any(bc_fail) ? kPfBcFail : 0u;
    bits |= __any(any_two) ? kPfAnyTwo : 0u; bits |= __any(ng_ar) ? kPfNgAr : 0u; bits |= __any(ng_ag) ? kPfNgAg : 0u;
    bits |= __any(ng_bc) ? kPfNgBc : 0u; bits |= __any((fl_pat & kFlagTwo) != 0u) ? kPfPatTwo : 0u;
    for (int o = 32; o > 0; o >>= 1) { goal_part += __shfl_xor(goal_part, o, 64); two_part += __shfl_xor(two_part, o, 64); }
    f.bits = bits; f.goal_part = goal_part; f.two_part = two_part;
    return f;
}

// A valid AllGather of members with different masks: does some device hold more than two masks afterwards?
// Second walk, the wavefront together: per group the first pair's mask, the first mask that differs from it,
// and whether a third one shows up (the child then needs the literal state).
template <int KW, int MW, int NP>
__device__ inline bool cls_many_masks(const ClsLane<KW, MW, NP>& c, const PatLds P) {
    using L = FL<KW, MW>;
    const uint4* const ldsq = c.ldsq;
    const int plane_q = c.plane_q, slot = c.slot, qd = c.qd;
    const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    int spg = 1;
    while (spg * 2 * ng <= 8) spg *= 2;
    const int gpb = 8 / spg;
    const int my_g = slot / spg, part = slot - my_g * spg;
    const int trips = (g + spg - 1) / spg;
    bool many = false;
    for (int G0 = 0; G0 < ng; G0 += gpb) {
        const int G = G0 + my_g;
        const bool act = G < ng && c.is_mask;
        int base = 0;
        if (P.master) base = G * gs;
        else { const int hi = div_small(G, s); base = hi * gs + (G - hi * s); }
        const uint4 d0 = act ? ldsq[base * L::WQ + qd] : q_zero();
        uint4 d1 = q_zero();
        bool have1 = false;
        const int sh = slot * 8;
        for (int it = 0; it < trips; ++it) {
            const int t = it * spg + part;
            const bool on = act && t < g;
            const int d = base + t * s;
#pragma unroll
            for (int pl = 0; pl < NP; ++pl) {
                const uint4 m = on ? ldsq[pl * plane_q + d * L::WQ + qd] : q_zero();
                // (an empty second pair has an empty mask; the first pair of a member is never empty here)
                const bool there = on && (pl == 0 || (c.flags[d] & kFlagTwo) != 0u);
                const unsigned long long ne0 = __ballot(there && q_any(q_xor(m, d0)));
                const unsigned long long ne1 = __ballot(there && q_any(q_xor(m, d1)));
                if (there && ((ne0 >> sh) & 0xffull) != 0ull) {
                    if (!have1) { d1 = m; have1 = true; }
                    else if (((ne1 >> sh) & 0xffull) != 0ull) many = true;
                }
            }
        }
        for (int m = 8; m < 8 * spg; m <<= 1) {      // the slots of one group compare what they found
            const uint4 o1 = q_shfl_xor(d1, m);
            const bool o_have = __shfl_xor((int)have1, m, 64) != 0;
            const unsigned long long ne = __ballot(act && have1 && o_have && q_any(q_xor(d1, o1)));
            if (act && o_have) {
                if (!have1) { d1 = o1; have1 = true; }
                else if (((ne >> sh) & 0xffull) != 0ull) many = true;
            }
        }
    }
    return __any(many) != 0;
}

// Broadcast on a pattern with two-pair members that has passed the necessary conditions of the walk above, the
// wavefront together (the rule of bcast_compare): every member's rows lie inside the root's; where a pair of the
// member shares rows with a pair of the root, the member's mask lies inside the root's; and in every group some
// member differs from its root.  Returns 0 (invalid), else 1 | 2 (some root holds two pairs) | 4 (every root is
// at the goal).
template <int KW, int MW, int NP>
__device__ inline int cls_bcast_pairs(const ClsLane<KW, MW, NP>& c, const PatLds P) {
    using L = FL<KW, MW>;
    const uint4* const ldsq = c.ldsq;
    const int plane_q = c.plane_q, slot = c.slot, qd = c.qd, sh = slot * 8;
    const bool is_row = c.is_row, is_mask = c.is_mask;
    const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    int spg = 1;
    while (spg * 2 * ng <= 8) spg *= 2;
    const int gpb = 8 / spg;
    const int my_g = slot / spg, part = slot - my_g * spg;
    const int trips = (g + spg - 1) / spg;
    bool bad = false, any_two = false, not_goal = false;
    for (int G0 = 0; G0 < ng; G0 += gpb) {
        const int G = G0 + my_g;
        const bool act = G < ng && c.has_quad;
        int base = 0;
        if (P.master) base = G * gs;
        else { const int hi = div_small(G, s); base = hi * gs + (G - hi * s); }
        const uint4 r0 = act ? ldsq[base * L::WQ + qd] : q_zero();
        const uint4 r1 = (NP == 2 && act) ? ldsq[plane_q + base * L::WQ + qd] : q_zero();
        bool not_sub = false, dif = false;
        for (int it = 0; it < trips; ++it) {
            const int t = it * spg + part;
            const bool on = act && t < g && t > 0;
            const int d = base + t * s;
            const uint4 v0 = on ? ldsq[d * L::WQ + qd] : q_zero();
            const uint4 v1 = (NP == 2 && on) ? ldsq[plane_q + d * L::WQ + qd] : q_zero();
            // which pairs of the member share rows with which pairs of the root (row lanes tell the slot)
            const bool o00 = ((__ballot(on && is_row && q_any(q_and(r0, v0))) >> sh) & 0xffull) != 0ull;
            const bool o01 = ((__ballot(on && is_row && q_any(q_and(r0, v1))) >> sh) & 0xffull) != 0ull;
            const bool o10 = ((__ballot(on && is_row && q_any(q_and(r1, v0))) >> sh) & 0xffull) != 0ull;
            const bool o11 = ((__ballot(on && is_row && q_any(q_and(r1, v1))) >> sh) & 0xffull) != 0ull;
            if (on) {
                if (is_row) {
                    const uint4 um = q_or(v0, v1), ur = q_or(r0, r1);
                    not_sub |= q_any(q_andn(um, ur));
                    dif |= q_any(q_xor(um, ur));
                } else if (is_mask) {
                    if (o00) { not_sub |= q_any(q_andn(v0, r0)); dif |= q_any(q_xor(v0, r0)); }
                    if (o01) { not_sub |= q_any(q_andn(v1, r0)); dif |= q_any(q_xor(v1, r0)); }
                    if (o10) { not_sub |= q_any(q_andn(v0, r1)); dif |= q_any(q_xor(v0, r1)); }
                    if (o11) { not_sub |= q_any(q_andn(v1, r1)); dif |= q_any(q_xor(v1, r1)); }
                }
            }
        }
        // a group's verdict: nothing outside the root's, and a difference in some slot of the group
        const unsigned long long dif_slots = __ballot(dif);
        const unsigned long long group_bits = (spg == 8 ? ~0ull : ((1ull << (8 * spg)) - 1ull) << ((slot - part) * 8));
        const bool root_two = ((__ballot(act && is_row && q_any(r1)) >> sh) & 0xffull) != 0ull;
        if (act) {
            bad |= not_sub || (dif_slots & group_bits) == 0ull;
            any_two |= root_two;
            not_goal |= root_two || q_any(q_xor(r0, c.goal_quad));
        }
    }
    if (__any(bad)) return 0;
    return 1 | (__any(any_two) ? 2 : 0) | (__any(not_goal) ? 0 : 4);
}

// A ReduceScatter on a pattern whose groups are valid, aligned and split (some member holds two pairs), the
// wavefront together: rank t keeps the t-th block of the group's rows in ascending order; does a block fall on both
// sides of a split whose sides carry different masks?  (Then that member holds two pairs afterwards.)  Per group the
// slots put together the rows (the same on every member), the pair-0 rows of the members with two pairs, and the
// united masks of either side, as the kernel that builds the child does; then every rank's block is cut out of the
// rows and looked at from both sides.
template <int KW, int MW, int NP>
__device__ inline bool cls_rs_straddles(const ClsLane<KW, MW, NP>& c, const PatLds P) {
    using L = FL<KW, MW>;
    const uint4* const ldsq = c.ldsq;
    const int plane_q = c.plane_q, slot = c.slot, qd = c.qd, sh = slot * 8;
    const bool is_row = c.is_row, is_mask = c.is_mask;
    const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    int spg = 1;
    while (spg * 2 * ng <= 8) spg *= 2;
    const int gpb = 8 / spg;
    const int my_g = slot / spg, part = slot - my_g * spg;
    const int trips = (g + spg - 1) / spg;
    bool straddles = false;
    for (int G0 = 0; G0 < ng; G0 += gpb) {
        const int G = G0 + my_g;
        const bool act = G < ng && c.has_quad;
        int base = 0;
        if (P.master) base = G * gs;
        else { const int hi = div_small(G, s); base = hi * gs + (G - hi * s); }
        // row lanes: u = the rows, xa = pair-0 rows of the members with two pairs; mask lanes: u = united first
        // masks, mb = united masks of the other side (a member with one pair has its only mask on both sides)
        uint4 u = q_zero(), xa = q_zero(), mb = q_zero();
        bool split = false;
        for (int it = 0; it < trips; ++it) {
            const int t = it * spg + part;
            const bool on = act && t < g;
            const int d = base + t * s;
            const uint4 v0 = on ? ldsq[d * L::WQ + qd] : q_zero();
            const uint4 v1 = (NP == 2 && on) ? ldsq[plane_q + d * L::WQ + qd] : q_zero();
            const bool two = ((__ballot(is_row && q_any(v1)) >> sh) & 0xffull) != 0ull;
            split |= two;
            if (is_row) { u = q_or(u, q_or(v0, v1)); if (two) xa = q_or(xa, v0); }
            else { u = q_or(u, v0); mb = q_or(mb, two ? v1 : v0); }
        }
        for (int m = 8; m < 8 * spg; m <<= 1) {
            u = q_or(u, q_shfl_xor(u, m)); xa = q_or(xa, q_shfl_xor(xa, m)); mb = q_or(mb, q_shfl_xor(mb, m));
            split |= __shfl_xor((int)split, m, 64) != 0;
        }
        const bool sides_differ = ((__ballot(act && is_mask && q_any(q_xor(u, mb))) >> sh) & 0xffull) != 0ull;
        const int mine = (act && is_row) ? q_popc(u) : 0;
        const int rows = sum_slot(mine);
        const int per = div_small(rows, g);
        int before = 0;                                  // rows in the quads below this lane's
#pragma unroll
        for (int j = 0; j < L::QK; ++j) { const int cnt = __shfl(mine, sh + j, 64); if (j < qd) before += cnt; }
        const uint4 xb = q_andn(u, xa);
        const bool look = act && split && sides_differ && rows > 0;
        for (int it = 0; it < trips; ++it) {
            const int t = it * spg + part;
            const int lo = t * per, hi = lo + per;
            uint4 blk = q_zero();
            if (is_row) {
                int p0 = before;
                blk.x = low_bits(u.x, hi - p0) & ~low_bits(u.x, lo - p0); p0 += __popc(u.x);
                blk.y = low_bits(u.y, hi - p0) & ~low_bits(u.y, lo - p0); p0 += __popc(u.y);
                blk.z = low_bits(u.z, hi - p0) & ~low_bits(u.z, lo - p0); p0 += __popc(u.z);
                blk.w = low_bits(u.w, hi - p0) & ~low_bits(u.w, lo - p0);
            }
            const unsigned long long on_a = __ballot(is_row && q_any(q_and(blk, xa))), on_b = __ballot(is_row && q_any(q_and(blk, xb)));
            if (look && t < g && ((on_a >> sh) & 0xffull) != 0ull && ((on_b >> sh) & 0xffull) != 0ull) straddles = true;
        }
    }
    return __any(straddles) != 0;
}

// One lane: the codes of a pattern's instructions from what its groups have shown.  goal_ops < 0: every code;
// else (the last level, where only goals count) bit 0 / 1 / 2: an AllReduce / AllGather / Broadcast may still end
// at the goal, and everything that does not (or that this form cannot judge) is written as invalid.
template <int KW, int MW, int NP>
__device__ inline void cls_codes(const ClsLane<KW, MW, NP>& c, const PatLds P, int pid, uint32_t pf, int goal_part, int two_part,
                                 int n_goal, int n_two, bool MANY_MASKS, int bc_pairs, bool RS_STRADDLES, const int (&ops_r)[5], int n_ops, int max_pairs,
                                 const Words<KW>& all_rows, const Words<MW>& all_cols, int goal_ops, uint8_t* __restrict__ codes,
                                 uint8_t* __restrict__ unknown) {
    const int R = c.R;
    const bool BAD_RED = pf & kPfBadRed, BAD_B = pf & kPfBadB, UNAL = pf & kPfUnal, BAD_RS = pf & kPfBadRs;
    const bool BAD_AG = pf & kPfBadAg, CHANGED = pf & kPfChanged, AG_UNEQ = pf & kPfAgUneq;
    const bool BAD_BC1 = pf & kPfBadBc1, BC_FAIL = pf & kPfBcFail, ANY_TWO = pf & kPfAnyTwo;
    const bool NG_AR = pf & kPfNgAr, NG_AG = pf & kPfNgAg, NG_BC = pf & kPfNgBc, PAT_TWO = pf & kPfPatTwo;
    const bool rest_done = (n_goal - goal_part) == (R - P.n_groups * P.g);      // the devices left untouched are at the goal
    const bool rest_two = n_two - two_part > 0;                                 // ... or one of them holds two pairs
#pragma unroll
    for (int oi = 0; oi < 5; ++oi) {
        const int op = ops_r[oi];
        if (op < 0) continue;
        int code;
        if (goal_ops >= 0 && !((op == OP_AR && (goal_ops & 1)) || (op == OP_AG && (goal_ops & 2)) || (op == OP_BC && (goal_ops & 4)))) {
            code = CODE_INVALID;                         // (last level: this instruction cannot end at the goal)
        } else if (op == OP_AR || op == OP_RS || op == OP_RD) {
            if (BAD_RED || !CHANGED || (op == OP_RS && BAD_RS)) code = CODE_INVALID;
            else if (goal_ops >= 0 && NG_AR) code = CODE_INVALID;       // (last level: some device is left short of the goal)
            else if (UNAL) code = CODE_UNKNOWN;
            else if (BAD_B) code = CODE_INVALID;
            else if (op == OP_RS) {
                code = ((ANY_TWO && RS_STRADDLES) || rest_two) ? CODE_PREFIX2 : CODE_PREFIX;
            } else if (ANY_TWO || rest_two) code = CODE_PREFIX2;
            else code = (op == OP_AR && !NG_AR && rest_done) ? CODE_GOAL : CODE_PREFIX;
        } else if (op == OP_AG) {
            if (BAD_AG) code = CODE_INVALID;
            else if (AG_UNEQ) code = MANY_MASKS ? CODE_PREFIX_LITERAL : CODE_PREFIX2;   // members with different masks
            else if (rest_two) code = CODE_PREFIX2;
            else code = (!NG_AG && rest_done) ? CODE_GOAL : CODE_PREFIX;
        } else {
            if (!PAT_TWO) code = BAD_BC1 ? CODE_INVALID : rest_two ? CODE_PREFIX2 : (!NG_BC && rest_done) ? CODE_GOAL : CODE_PREFIX;
            else if (BC_FAIL || bc_pairs == 0) code = CODE_INVALID;
            else code = ((bc_pairs & 2) || rest_two) ? CODE_PREFIX2 : ((bc_pairs & 4) && rest_done) ? CODE_GOAL : CODE_PREFIX;
        }
        if (code == CODE_PREFIX2 && max_pairs < 2) code = CODE_PREFIX_LITERAL;
        if (goal_ops >= 0 && code != CODE_GOAL && code != CODE_UNKNOWN) code = CODE_INVALID;    // (last level: goals only)
        if (code == CODE_UNKNOWN) *unknown = 1;          // (after the block's barriers that follow the clearing)
        codes[pid * n_ops + oi] = (uint8_t)code;
    }
}

// ---- survivors of every entry from the codes of its state ------------------------------------------------
// The classification leaves, beside a state's row of codes, how many of them are survivors, goals, one-pair and
// two-pair children (row_counts: 16 bits each).  A lane per entry (the first `epw` lanes of a wavefront: 8 to 64,
// fewer where the list is short, so that its second pass is spread over more wavefronts) adds those up; the block's wavefronts reserve
// list positions and the children's places in the next frontier together (two additions to the level's counters per
// block and round: returning additions to one address are served one after the other); then the wavefront goes
// through its entries that have survivors, eight at a time, their rows loaded before any is looked at (four codes
// a word; an alphabet has at most 512 instructions: 128 words, two per lane), and writes.
constexpr int kExpThreads = 1024, kExpWaves = kExpThreads / 64, kExpBatch = 8;
template <int NP>
__global__ __launch_bounds__(kExpThreads) void k_front_expand(const DevQuery* __restrict__ qp, const FrontEntry* __restrict__ entries,
                                                             uint32_t n, const uint32_t* __restrict__ rep,
                                                             const uint8_t* __restrict__ codes, const uint2* __restrict__ row_counts,
                                                             const uint8_t* __restrict__ unknown,
                                                             int handover, int epw, FrontSurvivor* __restrict__ surv, uint32_t surv_cap,
                                                             FrontEntry* __restrict__ unknown_out, FrontCounters* __restrict__ ctr) {
    __shared__ uint32_t s_tot[kExpWaves][4];             // per wavefront: survivors, goals, one-pair children, two-pair children
    __shared__ uint32_t s_at[kExpWaves][4];              // ... where each kind starts for the wavefront
    __shared__ unsigned long long s_judged;              // entries judged by the block
    if (threadIdx.x == 0) s_judged = 0ull;
    __syncthreads();
    const DevQuery& q = *qp;
    const int I = q.alphabet;
    const uint32_t CS = front_code_stride(I);
    const int CW = (int)(CS / 4u);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    uint32_t in_alphabet[2];                             // the bytes of a lane's two words that are instructions (invalid = 0 elsewhere)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int left = I - (lane + 64 * h) * 4;
        in_alphabet[h] = left >= 4 ? 0xffffffffu : left > 0 ? ((1u << (8 * left)) - 1u) : 0u;
    }
    unsigned long long judged = 0;                       // entries judged from their states' codes (lane 0 counts)
    const uint32_t per_block = (uint32_t)(kExpWaves * epw);
    for (uint32_t base = blockIdx.x * per_block; base < n; base += gridDim.x * per_block) {
        const uint32_t p = base + (uint32_t)(wv * epw + lane);
        const bool valid = lane < epw && p < n;
        const uint32_t row = valid ? (rep ? rep[p] : p) : 0u;
        const bool unk = valid && (handover != 0 || unknown[row] != 0);
        const uint2 cnt = (valid && !unk) ? row_counts[row] : make_uint2(0u, 0u);
        const uint32_t c_surv = cnt.x & 0xffffu, c_goal = cnt.x >> 16, c_p1 = cnt.y & 0xffffu, c_p2 = cnt.y >> 16;
        uint32_t x_surv = c_surv, x_goal = c_goal, x_p1 = c_p1, x_p2 = c_p2;          // inclusive sums over the lanes
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t a0 = __shfl_up(x_surv, o, 64), a1 = __shfl_up(x_goal, o, 64), a2 = __shfl_up(x_p1, o, 64), a3 = __shfl_up(x_p2, o, 64);
            if (lane >= o) { x_surv += a0; x_goal += a1; x_p1 += a2; x_p2 += a3; }
        }
        if (lane == 63) { s_tot[wv][0] = x_surv; s_tot[wv][1] = x_goal; s_tot[wv][2] = x_p1; s_tot[wv][3] = x_p2; }
        __syncthreads();
        if (wv == 0) {
            // lane w < kExpWaves: the totals of wavefront w; sums over the wavefronts before it; one lane reserves
            uint32_t t[4], x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { t[j] = lane < kExpWaves ? s_tot[lane][j] : 0u; x[j] = t[j]; }
            for (int o = 1; o < kExpWaves; o <<= 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) { const uint32_t up = __shfl_up(x[j], o, 64); if (lane >= o) x[j] += up; }
            }
            uint32_t all[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) all[j] = __shfl(x[j], kExpWaves - 1, 64);
            unsigned long long b0 = 0, b1 = 0;
            if (lane == 0) {
                if (all[0]) b0 = atomicAdd(&ctr->surv_goal, (unsigned long long)all[0] | ((unsigned long long)all[1] << 32));
                if (all[2] | all[3]) b1 = atomicAdd(&ctr->pref_pref2, (unsigned long long)all[2] | ((unsigned long long)all[3] << 32));
            }
            b0 = __shfl(b0, 0, 64); b1 = __shfl(b1, 0, 64);
            if (lane < kExpWaves) {
                s_at[lane][0] = (uint32_t)b0 + x[0] - t[0]; s_at[lane][1] = (uint32_t)(b0 >> 32) + x[1] - t[1];
                s_at[lane][2] = (uint32_t)b1 + x[2] - t[2]; s_at[lane][3] = (uint32_t)(b1 >> 32) + x[3] - t[3];
            }
        }
        __syncthreads();
        if (unk) unknown_out[atomicAdd(&ctr->n_unknown, 1u)] = entries[p];
        {
            const unsigned long long took = __ballot(valid && !unk);
            if (lane == 0) judged += (unsigned long long)__popcll(took);
        }
        // this entry's first places
        const uint32_t e_surv = s_at[wv][0] + x_surv - c_surv, e_goal = s_at[wv][1] + x_goal - c_goal;
        const uint32_t e_p1 = s_at[wv][2] + x_p1 - c_p1, e_p2 = s_at[wv][3] + x_p2 - c_p2;
        unsigned long long todo = __ballot(c_surv > 0u);
        while (todo != 0ull) {
            int src[kExpBatch];
            uint32_t four[kExpBatch][2];
#pragma unroll
            for (int b = 0; b < kExpBatch; ++b) {
                src[b] = -1;
                if (todo != 0ull) { src[b] = __ffsll((long long)todo) - 1; todo &= todo - 1ull; }
            }
#pragma unroll
            for (int b = 0; b < kExpBatch; ++b) {
                // (every load is made, from a word that exists, and what was not asked for is dropped afterwards: loads
                //  under a condition are waited for one by one, these sixteen are in flight together)
                const uint32_t r = (uint32_t)__shfl((int)row, src[b] < 0 ? 0 : src[b], 64);
                const uint32_t* const words = reinterpret_cast<const uint32_t*>(codes + (size_t)r * CS);
#pragma unroll
                for (int h = 0; h < 2; ++h) four[b][h] = words[lane + 64 * h < CW ? lane + 64 * h : 0];
            }
#pragma unroll
            for (int b = 0; b < kExpBatch; ++b) {
#pragma unroll
                for (int h = 0; h < 2; ++h) four[b][h] = (src[b] >= 0 && lane + 64 * h < CW) ? (four[b][h] & in_alphabet[h]) : 0u;
            }
#pragma unroll
            for (int b = 0; b < kExpBatch; ++b) {
                if (src[b] < 0) continue;
                // this lane's survivors of the entry by kind, and those of the lanes before it
                uint32_t k_surv = 0, k_goal = 0, k_p1 = 0, k_p2 = 0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int code = (int)((four[b][h] >> (8 * j)) & 0xffu);
                        k_surv += code != CODE_INVALID; k_goal += code == CODE_GOAL; k_p1 += code == CODE_PREFIX; k_p2 += code == CODE_PREFIX2;
                    }
                }
                uint32_t y_surv = k_surv, y_goal = k_goal, y_p1 = k_p1, y_p2 = k_p2;
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t a0 = __shfl_up(y_surv, o, 64), a1 = __shfl_up(y_goal, o, 64), a2 = __shfl_up(y_p1, o, 64), a3 = __shfl_up(y_p2, o, 64);
                    if (lane >= o) { y_surv += a0; y_goal += a1; y_p1 += a2; y_p2 += a3; }
                }
                uint32_t at_surv = (uint32_t)__shfl((int)e_surv, src[b], 64) + y_surv - k_surv;
                uint32_t at_goal = (uint32_t)__shfl((int)e_goal, src[b], 64) + y_goal - k_goal;
                uint32_t at_p1 = (uint32_t)__shfl((int)e_p1, src[b], 64) + y_p1 - k_p1;
                uint32_t at_p2 = (uint32_t)__shfl((int)e_p2, src[b], 64) + y_p2 - k_p2;
                const uint32_t entry = base + (uint32_t)(wv * epw + src[b]);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (four[b][h] == 0u) continue;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int a = (lane + 64 * h) * 4 + j;
                        const int code = (int)((four[b][h] >> (8 * j)) & 0xffu);
                        if (code == CODE_INVALID) continue;
                        FrontSurvivor sv;
                        sv.entry = entry; sv.digit = (uint16_t)a; sv.code = (uint16_t)(code | (NP == 2 ? kFromTwoPair : 0));
                        sv.slot = code == CODE_GOAL ? at_goal++ : code == CODE_PREFIX ? at_p1++ : code == CODE_PREFIX2 ? at_p2++ : 0u;
                        if (code == CODE_PREFIX_LITERAL) atomicAdd(&ctr->n_prefix_literal, 1u);
                        if (at_surv < surv_cap) surv[at_surv] = sv;
                        ++at_surv;
                    }
                }
            }
        }
    }
    // (one addition per block: additions to one address are served one after the other, some 10⁸ a second, and a
    //  launch of four thousand wavefronts that each add twice lasts a tenth of a millisecond for that alone)
    if (lane == 0 && judged) atomicAdd(&s_judged, judged);
    __syncthreads();
    if (threadIdx.x == 0 && s_judged) {
        atomicAdd(&ctr->steps, s_judged * (unsigned long long)I);
        atomicAdd(&ctr->members, s_judged * (unsigned long long)q.reg_sum_part);
    }
}

// ---- entries with equal states ---------------------------------------------------------------------------
// 64 bits of a state: a sum over its 16-byte quads, so that the lanes that stream a state can each hash their own
// quads.  (It only proposes which entries to compare.)
__device__ inline unsigned long long hash_quad(uint4 v, uint32_t idx) {
    uint32_t a = v.x * 0x9e3779b1u + v.y * 0x85ebca77u + v.z * 0xc2b2ae3du + v.w * 0x27d4eb2fu + idx * 0x165667b1u;
    uint32_t b = v.x * 0x7feb352du + v.y * 0x846ca68bu + v.z * 0x9e3779b9u + v.w * 0x85ebca6bu + idx * 0xc2b2ae35u;
    a ^= a >> 15; a *= 0x2c1b3c6du; a ^= a >> 12; a *= 0x297a2d39u; a ^= a >> 15;
    b ^= b >> 16; b *= 0x7feb352du; b ^= b >> 15; b *= 0x846ca68bu; b ^= b >> 16;
    return ((unsigned long long)a << 32) | b;
}
constexpr unsigned long long kTableEmpty = ~0ull;
// Open addressing on the upper 40 bits of the hash; a table word is (those bits << 24) | entry.  The first entry
// to claim a word stands for the hash; the others take it as their candidate.
__global__ __launch_bounds__(256) void k_front_dedup(const unsigned long long* __restrict__ hash, uint32_t n,
                                                     unsigned long long* __restrict__ table, uint32_t mask, uint32_t* __restrict__ rep,
                                                     uint32_t* __restrict__ reps_list, uint32_t* __restrict__ n_reps) {
    const uint32_t p = blockIdx.x * 256u + threadIdx.x;
    if (p >= n) return;
    const unsigned long long h = hash[p];
    const unsigned long long key = h >> 24;
    uint32_t at = (uint32_t)((h * 0x9e3779b97f4a7c15ull) >> 32) & mask;
    for (uint32_t probe = 0; probe <= mask; ++probe) {        // (the table has room for every entry: an empty word turns up)
        const unsigned long long old = atomicCAS(&table[at], kTableEmpty, (key << 24) | p);
        if (old == kTableEmpty) { rep[p] = p; reps_list[atomicAdd(n_reps, 1u)] = p; return; }
        if ((old >> 24) == key) { rep[p] = (uint32_t)(old & 0xffffffull); return; }
        at = (at + 1u) & mask;
    }
    rep[p] = p; reps_list[atomicAdd(n_reps, 1u)] = p;         // never reached with a table of 2 n words
}
// A wavefront per entry that took a candidate: the two states word by word; an entry that differs stands for itself.
__global__ __launch_bounds__(256) void k_front_verify(const uint4* __restrict__ states, uint32_t quads, uint32_t n,
                                                      uint32_t* __restrict__ rep, uint32_t* __restrict__ reps_list,
                                                      uint32_t* __restrict__ n_reps) {
    const int lane = threadIdx.x & 63;
    const uint32_t wave = (blockIdx.x * 256u + threadIdx.x) >> 6, n_waves = gridDim.x * 4u;
    for (uint32_t p = wave; p < n; p += n_waves) {
        const uint32_t r = rep[p];
        if (r == p) continue;
        const uint4* a = states + (size_t)p * quads;
        const uint4* b = states + (size_t)r * quads;
        bool differ = false;
        for (uint32_t i0 = (uint32_t)lane; i0 < quads; i0 += 256u) {
            // (all eight loads are made, past the end from the last quad again, which changes nothing: loads under a
            //  condition are waited for pair by pair)
            uint4 x[4], y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t i = min(i0 + 64u * u, quads - 1u);
                x[u] = a[i]; y[u] = b[i];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) differ |= q_any(q_xor(x[u], y[u]));
        }
        if (__any(differ) && lane == 0) { rep[p] = p; reps_list[atomicAdd(n_reps, 1u)] = p; }
    }
}

// this lane's quad of a device at the goal: every row, every column of the reduction group
template <int KW, int MW>
__device__ inline uint4 goal_quad_of(const Words<KW>& all_rows, const Words<MW>& all_cols, int qd, bool is_row, bool is_mask) {
    using L = FL<KW, MW>;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < KW; ++i) if (is_row && i == qd * 4 + j) w[j] = all_rows.w[i];
#pragma unroll
        for (int i = 0; i < MW; ++i) if (is_mask && i == (qd - L::QK) * 4 + j) w[j] = all_cols.w[i];
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// ---- the last level: which states are worth a walk ---------------------------------------------------
// At the size limit only goals count, and one instruction ends at the goal only from a state that is nearly there:
// an AllReduce leaves the rows of its members as they are and touches no other device, so every device must hold
// every row already; an AllGather leaves the columns of the rows it moves as they are, so every row that a device
// holds must carry every column; a Broadcast makes its members equal to their roots, and device 0 is a root of
// every pattern, so device 0 must be at the goal.  A wavefront per state reads the devices straight from device
// memory (8 at a time, a lane per quad) until all three have failed, in which case the state's row of codes is
// written as invalid; the other states go on the list walk[0 .. *n_walk) for the classification kernel.
template <int KW, int MW, int NP>
__global__ __launch_bounds__(256) void k_front_goal_filter(const DevQuery* __restrict__ qp, const uint32_t* __restrict__ states,
                                                           uint32_t n_entries, const uint32_t* __restrict__ list,
                                                           const uint32_t* __restrict__ n_list, uint8_t* __restrict__ codes,
                                                           uint2* __restrict__ row_counts, uint8_t* __restrict__ unknown,
                                                           uint32_t* __restrict__ walk, uint32_t* __restrict__ n_walk) {
    using L = FL<KW, MW>;
    const DevQuery& q = *qp;
    const int R = q.R, I = q.alphabet;
    const int plane_q = R * L::WQ;
    const int lane = threadIdx.x & 63, slot = lane >> 3, qd = lane & 7, sh = slot * 8;
    const bool is_row = qd < L::QK, is_mask = qd >= L::QK && qd < L::WQ, has_quad = qd < L::WQ;
    const uint4 goal_quad = goal_quad_of<KW, MW>(full_mask<KW>(q.k), full_mask<MW>(R), qd, is_row, is_mask);
    const uint32_t wave = (blockIdx.x * 256u + threadIdx.x) >> 6, n_waves = gridDim.x * 4u;
    const uint32_t n_work = list ? *n_list : n_entries;
    for (uint32_t at = wave; at < n_work; at += n_waves) {
        const uint32_t e = list ? list[at] : at;
        const uint4* src = reinterpret_cast<const uint4*>(states) + (size_t)e * NP * plane_q;
        bool rows_short = false, cols_short = false, root_short = false;
        for (int d0 = 0; d0 < R; d0 += 8) {
            const int d = d0 + slot;
            const bool act = d < R && has_quad;
            const uint4 v = act ? src[d * L::WQ + qd] : q_zero();
            const uint4 v1 = (NP == 2 && act) ? src[plane_q + d * L::WQ + qd] : q_zero();
            const unsigned long long nz = __ballot(act && is_row && q_any(v));
            const unsigned long long ng = __ballot(act && q_any(q_xor(v, goal_quad)));
            const unsigned long long n2 = NP == 2 ? __ballot(act && is_row && q_any(v1)) : 0ull;
            const unsigned long long rs = __ballot(act && is_row && q_any(q_xor(q_or(v, v1), goal_quad)));
            const unsigned long long m0 = __ballot(act && is_mask && q_any(q_xor(v, goal_quad)));
            const unsigned long long m1 = NP == 2 ? __ballot(act && is_mask && q_any(q_xor(v1, goal_quad))) : 0ull;
            if (d < R) {
                const bool empty = ((nz >> sh) & 0xffull) == 0ull, two = ((n2 >> sh) & 0xffull) != 0ull;
                rows_short |= ((rs >> sh) & 0xffull) != 0ull;
                cols_short |= (!empty && ((m0 >> sh) & 0xffull) != 0ull) || (two && ((m1 >> sh) & 0xffull) != 0ull);
                if (d == 0) root_short = ((ng >> sh) & 0xffull) != 0ull || two;
            }
            if (__any(rows_short) && __any(cols_short) && __any(root_short)) break;
        }
        if (__any(rows_short) && __any(cols_short) && __any(root_short)) {
            uint32_t* const words = reinterpret_cast<uint32_t*>(codes + (size_t)e * front_code_stride(I));
            for (int w = lane; w * 4 < I; w += 64) words[w] = 0u;          // (CODE_INVALID is zero)
            if (lane == 0) { unknown[e] = 0; row_counts[e] = make_uint2(0u, 0u); }
        } else if (lane == 0) {
            walk[atomicAdd(n_walk, 1u)] = e;
        }
    }
}

// ---- a block per prefix ---------------------------------------------------------------------------------
template <int KW, int MW, int NP>
// (second bound: wavefronts per SIMD, so that two blocks of one-plane states share a compute unit)
__global__ __launch_bounds__(kClsThreads, NP == 1 ? 4 : 2) void k_front_classify(const DevQuery* __restrict__ qp,
                                                                const uint32_t* __restrict__ states, uint32_t n_entries,
                                                                const uint32_t* __restrict__ list, const uint32_t* __restrict__ n_list,
                                                                int max_pairs, int goals_only, int count_children,
                                                                uint8_t* __restrict__ codes, uint2* __restrict__ row_counts,
                                                                uint8_t* __restrict__ unknown, FrontCounters* __restrict__ ctr) {
    extern __shared__ uint4 ldsq[];                      // NP planes of [R][WQ] quads, then R flag bytes
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ int s_goal, s_two, s_next, s_n_items, s_rows_short, s_cols_short;
    __shared__ uint32_t s_pflags[kMaxPatterns];
    __shared__ int s_pgoal[kMaxPatterns], s_ptwo[kMaxPatterns];
    __shared__ ClsItem s_items[kMaxPatterns * kClsChunks];
    __shared__ __align__(16) uint8_t s_codes[512];        // the row of codes of the state at hand (an alphabet has at most 512 instructions)
    using L = FL<KW, MW>;
    const DevQuery& q = *qp;
    const int R = q.R, I = q.alphabet, n_ops = q.n_ops, n_pat = q.n_patterns;
    const int plane_q = R * L::WQ;                       // quads per plane
    uint8_t* const flags = reinterpret_cast<uint8_t*>(ldsq + (size_t)NP * plane_q);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < n_pat; i += kClsThreads) {
        PatLds p;
        p.g = q.pat[i].g; p.s = q.pat[i].s; p.master = q.pat[i].master; p.n_groups = q.pat[i].n_groups;
        spat[i] = p;
    }
    __syncthreads();
    // work items: a pattern's batches of groups in up to kClsChunks runs; the long items (whole patterns) first, then
    // the other patterns' runs, pattern after pattern.  A thread per pattern works out its runs and where they go (a
    // block judges a state or two, so what it sets up first is not paid once and forgotten).
    {
        int* const s_runs = s_pgoal;                     // (not in use yet) runs of pattern i, negated for a whole pattern
        for (int i = tid; i < n_pat; i += kClsThreads) {
            const int ng = spat[i].n_groups;
            int spg = 1;
            while (spg * 2 * ng <= 8) spg *= 2;
            const int batches = (ng + 8 / spg - 1) / (8 / spg);
            const int per = batches >= 2 * kClsChunks ? (batches + kClsChunks - 1) / kClsChunks : batches >= 4 ? 2 : batches;
            s_runs[i] = per == batches ? -1 : (batches + per - 1) / per;
        }
        __syncthreads();
        for (int i = tid; i < n_pat; i += kClsThreads) {
            const int ng = spat[i].n_groups;
            int spg = 1;
            while (spg * 2 * ng <= 8) spg *= 2;
            const int batches = (ng + 8 / spg - 1) / (8 / spg);
            const int per = batches >= 2 * kClsChunks ? (batches + kClsChunks - 1) / kClsChunks : batches >= 4 ? 2 : batches;
            const bool whole = s_runs[i] < 0;
            int at = 0, n_whole = 0, total = 0;
            for (int j = 0; j < n_pat; ++j) {
                const int rj = s_runs[j];
                n_whole += rj < 0 ? 1 : 0;
                total += rj < 0 ? 1 : rj;
                if (j < i && (rj < 0) == whole) at += rj < 0 ? 1 : rj;
            }
            if (!whole) at += n_whole;
            for (int b = 0; b < batches; b += per) {
                ClsItem w; w.pid = (uint16_t)i; w.first_batch = (uint16_t)b; w.n_batches = (uint16_t)min(per, batches - b);
                s_items[at++] = w;
            }
            if (i == 0) s_n_items = total;
        }
    }
    const Words<KW> all_rows = full_mask<KW>(q.k);
    const Words<MW> all_cols = full_mask<MW>(R);
    ClsLane<KW, MW, NP> c;
    c.ldsq = ldsq; c.flags = flags; c.R = R; c.plane_q = plane_q;
    c.lane = lane; c.slot = lane >> 3; c.qd = lane & 7;
    c.is_row = c.qd < L::QK; c.is_mask = c.qd >= L::QK && c.qd < L::WQ; c.has_quad = c.qd < L::WQ;
    c.goal_quad = goal_quad_of<KW, MW>(all_rows, all_cols, c.qd, c.is_row, c.is_mask);
    int ops_r[5];
    bool has_bcast = false, has_scatter = false;
#pragma unroll
    for (int i = 0; i < 5; ++i) { ops_r[i] = i < n_ops ? q.ops[i] : -1; has_bcast |= ops_r[i] == OP_BC; has_scatter |= ops_r[i] == OP_RS; }
    const uint32_t n_work = list ? *n_list : n_entries;
    uint32_t walked = 0;                                 // states whose patterns were walked (thread 0 counts)
    uint32_t kids[3] = {0u, 0u, 0u};                     // one-pair children, two-pair children, goals of this block's states
    for (uint32_t at = blockIdx.x; at < n_work; at += gridDim.x) {
        const uint32_t e = list ? list[at] : at;
        __syncthreads();
        const uint4* src = reinterpret_cast<const uint4*>(states) + (size_t)e * NP * plane_q;
        // (all of a thread's loads are issued before the first store: one trip to HBM, not one per quad)
        for (int i0 = tid; i0 < NP * plane_q; i0 += 8 * kClsThreads) {
            uint4 tmp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { const int i = i0 + u * kClsThreads; tmp[u] = i < NP * plane_q ? src[i] : q_zero(); }
#pragma unroll
            for (int u = 0; u < 8; ++u) { const int i = i0 + u * kClsThreads; if (i < NP * plane_q) ldsq[i] = tmp[u]; }
        }
        if (tid == 0) { s_goal = 0; s_two = 0; s_next = 0; s_rows_short = 0; s_cols_short = 0; unknown[e] = 0; }
        for (int i = tid; i < n_pat; i += kClsThreads) { s_pflags[i] = 0u; s_pgoal[i] = 0; s_ptwo[i] = 0; }
        __syncthreads();
        {
            int at_goal, with_two, rows_short, cols_short;
            cls_flags<KW, MW, NP>(c, flags, wave * 8, kClsWaves * 8, at_goal, with_two, goals_only != 0, rows_short, cols_short);
            if (lane == 0 && at_goal) atomicAdd(&s_goal, at_goal);
            if (lane == 0 && with_two) atomicAdd(&s_two, with_two);
            if (lane == 0 && rows_short) atomicAdd(&s_rows_short, rows_short);
            if (lane == 0 && cols_short) atomicAdd(&s_cols_short, cols_short);
        }
        __syncthreads();
        const int n_goal = s_goal, n_two = s_two, n_items = s_n_items;
        // At the size limit only goals count, and one instruction ends at the goal only from a state that is nearly
        // there: an AllReduce leaves the rows of its members as they are and touches no other device, so every device
        // must hold every row already; an AllGather leaves the columns of the rows it moves as they are, so every row
        // that a device holds must carry every column; a Broadcast makes its members equal to their roots, and device 0
        // is a root of every pattern, so device 0 must be at the goal.  A state that fails all three has no goal among
        // its extensions and is not walked.
        int goal_ops = -1;
        if (goals_only) {
            goal_ops = (s_rows_short == 0 ? 1 : 0) | (s_cols_short == 0 ? 2 : 0) | ((flags[0] & kFlagGoal) ? 4 : 0);
            if (goal_ops == 0) {
                uint32_t* const words = reinterpret_cast<uint32_t*>(codes + (size_t)e * front_code_stride(I));
                for (int w = tid; w * 4 < I; w += kClsThreads) words[w] = 0u;      // (CODE_INVALID is zero)
                if (tid == 0) row_counts[e] = make_uint2(0u, 0u);
                continue;
            }
        }
        if (tid == 0) ++walked;
        // ---- stage A: the patterns' groups, cut into work items that the wavefronts take as they come (patterns
        //      differ widely in cost, and a pattern whose rules have all failed is dropped at once); what an item
        //      finds goes into its pattern's flag word
        for (;;) {
            // (all 64 lanes add one, so the counter runs in steps of 64: a fetch under `if (lane == 0)` followed by
            //  a cross-lane read is a lane-dependent branch inside the loop, and the compiler has been seen to split
            //  the loop on it, so that the other lanes read lane 0 while it is away and get item 0 for ever)
            const int item = __builtin_amdgcn_readfirstlane(atomicAdd(&s_next, 1)) >> 6;
            if (item >= n_items) break;
            const ClsItem W = s_items[item];
            const int pid = W.pid;
            {
                const uint32_t pf = s_pflags[pid];
                const bool dead_red = pf & kPfBadRed, dead_ag = pf & kPfBadAg, dead_bc = (pf & kPfBadBc1) && (NP == 1 || (pf & kPfBcFail));
                if (dead_red && dead_ag && dead_bc) continue;
                if (goal_ops >= 0 && (!(goal_ops & 1) || dead_red || (pf & kPfNgAr)) && (!(goal_ops & 2) || dead_ag || (pf & (kPfAgUneq | kPfNgAg))) &&
                    (!(goal_ops & 4) || dead_bc || (pf & kPfNgBc)))
                    continue;
            }
            const ClsFound f = cls_walk<KW, MW, NP>(c, spat[pid], W.first_batch, W.n_batches, goal_ops);
            if (lane == 0) {
                if (f.bits) atomicOr(&s_pflags[pid], f.bits);
                if (f.goal_part) atomicAdd(&s_pgoal[pid], f.goal_part);
                if (f.two_part) atomicAdd(&s_ptwo[pid], f.two_part);
            }
        }
        __syncthreads();
        // ---- stage B: a pattern's flag word gives the codes of its instructions
        for (int pid = wave; pid < n_pat; pid += kClsWaves) {
            const PatLds P = spat[pid];
            const uint32_t pf = s_pflags[pid];
            // (an AllGather of members with different masks is no goal: how many masks it leaves is not asked at the last level)
            const bool many = (goal_ops < 0 && !(pf & kPfBadAg) && (pf & kPfAgUneq)) ? cls_many_masks<KW, MW, NP>(c, P) : false;
            int bc_pairs = 0;                            // (Broadcast among two-pair devices: the pairs compared)
            if (NP == 2 && has_bcast && (goal_ops & 4) && (pf & kPfPatTwo) && !(pf & kPfBcFail)) bc_pairs = cls_bcast_pairs<KW, MW, NP>(c, P);
            // (ReduceScatter of a split group: asked where cls_codes gets as far as the question, and not at the last level)
            bool rs_straddles = false;
            if (NP == 2 && has_scatter && goal_ops < 0 && (pf & kPfAnyTwo) && !(pf & (kPfBadRed | kPfBadRs | kPfUnal | kPfBadB)) && (pf & kPfChanged))
                rs_straddles = cls_rs_straddles<KW, MW, NP>(c, P);
            if (lane == 0)
                cls_codes<KW, MW, NP>(c, P, pid, pf, s_pgoal[pid], s_ptwo[pid], n_goal, n_two, many, bc_pairs, rs_straddles, ops_r, n_ops, max_pairs,
                                      all_rows, all_cols, goal_ops, s_codes, unknown + e);
        }
        // ---- how many of the row's codes are survivors, goals, one-pair and two-pair children (16 bits each), for the
        //      kernel that lists the survivors of the prefixes: it then reads the rows of the prefixes that have any
        //      (the codes were put together in LDS, a byte per instruction from the lane that judged its pattern; they go
        //      out as whole words, the bytes past the alphabet as invalid)
        __syncthreads();
        if (wave == 0) {
            uint32_t* const words = reinterpret_cast<uint32_t*>(codes + (size_t)e * front_code_stride(I));
            uint32_t k_surv = 0, k_goal = 0, k_p1 = 0, k_p2 = 0;
            for (int w = lane; w * 4 < I; w += 64) {
                const int left = I - w * 4;
                const uint32_t four = reinterpret_cast<const uint32_t*>(s_codes)[w] & (left >= 4 ? 0xffffffffu : ((1u << (8 * left)) - 1u));
                words[w] = four;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int code = (int)((four >> (8 * j)) & 0xffu);
                    k_surv += code != CODE_INVALID; k_goal += code == CODE_GOAL; k_p1 += code == CODE_PREFIX; k_p2 += code == CODE_PREFIX2;
                }
            }
            uint32_t lo = k_surv | (k_goal << 16), hi = k_p1 | (k_p2 << 16);      // (at most 512 each: no carry between the halves)
            for (int o = 32; o > 0; o >>= 1) { lo += (uint32_t)__shfl_xor((int)lo, o, 64); hi += (uint32_t)__shfl_xor((int)hi, o, 64); }
            if (lane == 0) {
                row_counts[e] = make_uint2(lo, hi);
                // the children of the judged states by kind (a state that this form cannot judge has none: its prefixes
                // go to the literal kernels)
                if (count_children && unknown[e] == 0) { kids[0] += hi & 0xffffu; kids[1] += hi >> 16; kids[2] += lo >> 16; }
            }
        }
    }
    if (tid == 0) {
#pragma unroll
        for (int kd = 0; kd < 3; ++kd)
            if (kids[kd]) atomicAdd(&ctr->t_count[kd], kids[kd]);
    }
    if (tid == 0 && walked) atomicAdd(&ctr->n_walked_planes, walked * (uint32_t)NP);
}

__device__ inline unsigned long long rank_of(const DevQuery& q, unsigned long long digits, int len) {
    unsigned long long v = 0;
    for (int t = 0; t < len; ++t) v = v * (unsigned long long)q.alphabet + ((digits >> (9 * t)) & 511ull);
    return q.base[len] + v;
}

// ---- children of the survivors -----------------------------------------------------------------------
// Threads of a block: 256, or 1024 where the planes in LDS leave room for one or two blocks on a compute unit only
// (large reduction groups), so that the loads and stores of a child are still the work of many wavefronts.
constexpr int kMatThreads = 256, kMatThreadsBig = 1024;
constexpr size_t kMatBigLds = 60 * 1024;

// Smallest over the 8 lanes of a slot, in every lane of the slot (all lanes active).
__device__ inline int min_slot(int v) {
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false));
    return v;
}
// A device's two pairs, a lane per quad (a: first pair, b: second), brought into the stored form by the 8 lanes
// of its slot together: an empty pair has an empty mask, pairs with equal masks are one pair, the pair that
// holds the lowest row comes first.  Every lane of the wavefront calls it.
__device__ inline void canonical_slot(uint4& a, uint4& b, bool is_row, bool is_mask, int qd, int sh) {
    const unsigned long long nz0 = __ballot(is_row && q_any(a)), nz1 = __ballot(is_row && q_any(b));
    const bool e0 = ((nz0 >> sh) & 0xffull) == 0ull, e1 = ((nz1 >> sh) & 0xffull) == 0ull;
    if (is_mask) { if (e0) a = q_zero(); if (e1) b = q_zero(); }
    const unsigned long long md = __ballot(is_mask && q_any(q_xor(a, b)));
    if (!e1 && ((md >> sh) & 0xffull) == 0ull) {
        if (is_row) a = q_or(a, b);
        b = q_zero();
    }
    int l0 = 1 << 20, l1 = 1 << 20;
    if (is_row) {
        if (q_any(a)) l0 = qd * 128 + (a.x ? __ffs((int)a.x) - 1 : a.y ? 31 + __ffs((int)a.y) : a.z ? 63 + __ffs((int)a.z) : 95 + __ffs((int)a.w));
        if (q_any(b)) l1 = qd * 128 + (b.x ? __ffs((int)b.x) - 1 : b.y ? 31 + __ffs((int)b.y) : b.z ? 63 + __ffs((int)b.z) : 95 + __ffs((int)b.w));
    }
    l0 = min_slot(l0); l1 = min_slot(l1);
    if (l1 < l0) { const uint4 t = a; a = b; b = t; }
}

// A block per survivor of the one-pair and two-pair frontiers at a time: the parent's planes come into LDS with
// 128-bit loads, the instruction is applied there in place (a lane is (slot, quad) as in the classification; the
// slots of a wavefront take 8 groups side by side, or share the members of a group where the pattern has fewer
// groups: first the members are put together, then every member's new pairs are written), and the child's planes
// go out with 128-bit stores.  Groups are disjoint sets of devices, so the wavefronts do not meet.  The rows that
// a group's members hold set the bytes of the step (s_count), from which the wavefronts then work out the step's
// time for every query of the enumeration.
template <int KW, int MW, int NT>
__global__ __launch_bounds__(NT) void k_front_materialize(const DevQuery* __restrict__ queries, FrontLevel A) {
    extern __shared__ uint4 ldsq[];                      // A.lds_planes planes of [R][WQ] quads
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ uint32_t s_count[P2_MAX_DEVICES / 2];     // rows that set a group's bytes
    __shared__ unsigned long long s_hash[NT / 64];       // the wavefronts' shares of the child's hash
    using L = FL<KW, MW>;
    const DevQuery& q = queries[A.query];
    const int R = q.R;
    const int plane_q = R * L::WQ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane >> 3, qd = lane & 7, sh = slot * 8;
    const bool is_row = qd < L::QK, is_mask = qd >= L::QK && qd < L::WQ, has_quad = qd < L::WQ;
    for (int i = tid; i < q.n_patterns; i += NT) {
        PatLds p;
        p.g = q.pat[i].g; p.s = q.pat[i].s; p.master = q.pat[i].master; p.n_groups = q.pat[i].n_groups;
        spat[i] = p;
    }
    // (the search for equal states among the children, which follows this kernel, counts the distinct ones from zero;
    //  nothing reads the counts of the level's own lists any more)
    if (A.n_reps && blockIdx.x == 0 && tid < 2) A.n_reps[tid] = 0u;
    // (likewise the counters of the level's first half, which the host has read by now: the next level counts from zero)
    if (A.ctr && blockIdx.x == 0 && tid == 0) {
        FrontCounters* const c = A.ctr;
        c->surv_goal = 0ull; c->pref_pref2 = 0ull; c->n_surv_literal = 0u; c->n_goal = 0u; c->n_prefix_literal = 0u;
        c->n_overflow = 0u; c->n_unknown = 0u; c->t_count[0] = 0u; c->t_count[1] = 0u; c->t_count[2] = 0u;
        c->n_walked_planes = 0u; c->n_walk[0] = 0u; c->n_walk[1] = 0u;
    }
    __syncthreads();
    for (uint32_t i = blockIdx.x; i < A.n_surv; i += gridDim.x) {
        const FrontSurvivor sv = A.surv[i];
        const int code = sv.code & 0xff;
        const int np = (sv.code & kFromTwoPair) ? 2 : 1;
        const size_t plane_w = (size_t)plane_q * 4;
        const uint4* parent = reinterpret_cast<const uint4*>(np == 2 ? A.states2 + (size_t)sv.entry * 2 * plane_w
                                                                      : A.states1 + (size_t)sv.entry * plane_w);
        const int cnp = code == CODE_PREFIX2 ? 2 : 1;
        const uint32_t place = sv.slot;                  // the child's place in the next state list of its kind
        __syncthreads();                                 // (the block is done with the planes and counts of its last survivor)
        for (int i0 = tid; i0 < np * plane_q; i0 += 8 * NT) {
            uint4 tmp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { const int w = i0 + u * NT; tmp[u] = w < np * plane_q ? parent[w] : q_zero(); }
#pragma unroll
            for (int u = 0; u < 8; ++u) { const int w = i0 + u * NT; if (w < np * plane_q) ldsq[w] = tmp[u]; }
        }
        if (np == 1 && cnp == 2)                         // the devices that take no part have no second pair
            for (int w = tid; w < plane_q; w += NT) ldsq[plane_q + w] = q_zero();
        __syncthreads();
        // ---- apply the instruction in LDS
        const uint32_t ins = q.instr_of_digit[sv.digit];
        const int pid = (int)(ins >> 3);
        const PatLds P = spat[pid];
        const int op = (int)(ins & 7u);
        const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
        int spg = 1;                                     // slots that share a group
        while (spg * 2 * ng <= 8) spg *= 2;
        const int gpb = 8 / spg;                         // groups side by side
        const int my_g = slot / spg, part = slot - my_g * spg;
        const int trips = (g + spg - 1) / spg;
        const bool both = np == 2;                       // the parent has a second plane
        for (int G0 = wave * gpb; G0 < ng; G0 += (NT / 64) * gpb) {
            const int G = G0 + my_g;
            const bool act = G < ng && has_quad;
            int base = 0;
            if (P.master) base = G * gs;
            else { const int hi = div_small(G, s); base = hi * gs + (G - hi * s); }
            int rows_held = 0;
            if (op == OP_AR || op == OP_RS || op == OP_RD) {
                // row lanes: u = the rows (every member holds the same), xa = first-pair rows of the members with two pairs;
                // mask lanes: u = united first masks, mb = united masks of the other side of the split
                uint4 u = q_zero(), xa = q_zero(), mb = q_zero();
                bool split = false;
                for (int it = 0; it < trips; ++it) {
                    const int t = it * spg + part;
                    const bool on = act && t < g;
                    const int d = base + t * s;
                    const uint4 v0 = on ? ldsq[d * L::WQ + qd] : q_zero();
                    const uint4 v1 = (both && on) ? ldsq[plane_q + d * L::WQ + qd] : q_zero();
                    const bool two = ((__ballot(is_row && q_any(v1)) >> sh) & 0xffull) != 0ull;
                    split |= two;
                    if (is_row) { u = q_or(u, q_or(v0, v1)); if (two) xa = q_or(xa, v0); }
                    else { u = q_or(u, v0); mb = q_or(mb, two ? v1 : v0); }
                }
                for (int m = 8; m < 8 * spg; m <<= 1) {
                    u = q_or(u, q_shfl_xor(u, m)); xa = q_or(xa, q_shfl_xor(xa, m)); mb = q_or(mb, q_shfl_xor(mb, m));
                    split |= __shfl_xor((int)split, m, 64) != 0;
                }
                rows_held = sum_slot((act && is_row) ? q_popc(u) : 0);
                // the group's result: rows xa (or all of them) with the united first masks, the other rows with mb
                const uint4 ra = is_row ? (split ? xa : u) : u;
                const uint4 rb = is_row ? (split ? q_andn(u, xa) : q_zero()) : mb;
                if (op == OP_RS) {
                    // rank t keeps the t-th block of the rows in ascending order, on both sides of the split
                    const int per = div_small(rows_held, g);
                    const int mine = (act && is_row) ? q_popc(u) : 0;
                    int before = 0;                      // rows in the quads below this lane's
#pragma unroll
                    for (int j = 0; j < L::QK; ++j) { const int c = __shfl(mine, sh + j, 64); if (j < qd) before += c; }
                    for (int it = 0; it < trips; ++it) {
                        const int t = it * spg + part;
                        const bool on = act && t < g;
                        const int d = base + t * s;
                        const int lo = t * per, hi = lo + per;
                        uint4 blk = q_zero();
                        if (is_row) {
                            int p0 = before;
                            blk.x = low_bits(u.x, hi - p0) & ~low_bits(u.x, lo - p0); p0 += __popc(u.x);
                            blk.y = low_bits(u.y, hi - p0) & ~low_bits(u.y, lo - p0); p0 += __popc(u.y);
                            blk.z = low_bits(u.z, hi - p0) & ~low_bits(u.z, lo - p0); p0 += __popc(u.z);
                            blk.w = low_bits(u.w, hi - p0) & ~low_bits(u.w, lo - p0);
                        }
                        uint4 a = is_row ? q_and(blk, ra) : ra, b = is_row ? q_and(blk, rb) : rb;
                        canonical_slot(a, b, is_row, is_mask, qd, sh);
                        if (on) { ldsq[d * L::WQ + qd] = a; if (cnp == 2) ldsq[plane_q + d * L::WQ + qd] = b; }
                    }
                } else {
                    uint4 a = ra, b = rb;
                    canonical_slot(a, b, is_row, is_mask, qd, sh);
                    for (int it = 0; it < trips; ++it) {
                        const int t = it * spg + part;
                        const bool on = act && t < g;
                        const int d = base + t * s;
                        const bool keeps = op == OP_AR || t == 0;        // Reduce: the root alone keeps the result
                        if (on) { ldsq[d * L::WQ + qd] = keeps ? a : q_zero(); if (cnp == 2) ldsq[plane_q + d * L::WQ + qd] = keeps ? b : q_zero(); }
                    }
                }
            } else if (op == OP_AG) {
                // the first member's first mask, and whatever differs from it (at most one other mask: the
                // classification has counted); row lanes collect the rows that carry each
                const uint4 d0 = (act && is_mask) ? ldsq[base * L::WQ + qd] : q_zero();
                uint4 x0 = q_zero(), x1 = q_zero(), d1 = q_zero();
                for (int it = 0; it < trips; ++it) {
                    const int t = it * spg + part;
                    const bool on = act && t < g;
                    const int d = base + t * s;
#pragma unroll
                    for (int pl = 0; pl < 2; ++pl) {
                        const uint4 v = (on && (pl == 0 || both)) ? ldsq[pl * plane_q + d * L::WQ + qd] : q_zero();
                        const bool there = ((__ballot(is_row && q_any(v)) >> sh) & 0xffull) != 0ull;
                        const bool other = ((__ballot(is_mask && q_any(q_xor(v, d0))) >> sh) & 0xffull) != 0ull;
                        if (there) {
                            if (is_row) { if (other) x1 = q_or(x1, v); else x0 = q_or(x0, v); }
                            else if (other) d1 = q_or(d1, v);
                        }
                    }
                }
                for (int m = 8; m < 8 * spg; m <<= 1) {
                    x0 = q_or(x0, q_shfl_xor(x0, m)); x1 = q_or(x1, q_shfl_xor(x1, m)); d1 = q_or(d1, q_shfl_xor(d1, m));
                }
                rows_held = sum_slot((act && is_row) ? q_popc(q_or(x0, x1)) : 0);
                uint4 a = is_row ? x0 : d0, b = is_row ? x1 : d1;
                canonical_slot(a, b, is_row, is_mask, qd, sh);
                for (int it = 0; it < trips; ++it) {
                    const int t = it * spg + part;
                    const bool on = act && t < g;
                    const int d = base + t * s;
                    if (on) { ldsq[d * L::WQ + qd] = a; if (cnp == 2) ldsq[plane_q + d * L::WQ + qd] = b; }
                }
            } else {
                // Broadcast: the root's pairs, as they are
                const uint4 a = act ? ldsq[base * L::WQ + qd] : q_zero();
                const uint4 b = (act && both) ? ldsq[plane_q + base * L::WQ + qd] : q_zero();
                rows_held = sum_slot((act && is_row) ? q_popc(q_or(a, b)) : 0);
                for (int it = 0; it < trips; ++it) {
                    const int t = it * spg + part;
                    const bool on = act && t < g && t > 0;
                    const int d = base + t * s;
                    if (on) { ldsq[d * L::WQ + qd] = a; if (cnp == 2) ldsq[plane_q + d * L::WQ + qd] = b; }
                }
            }
            if (qd == 0 && part == 0 && G < ng) s_count[G] = (uint32_t)rows_held;
        }
        __syncthreads();
        if (code != CODE_GOAL) {
            uint4* child = reinterpret_cast<uint4*>(cnp == 2 ? A.next_states2 + (size_t)place * 2 * plane_w
                                                             : A.next_states1 + (size_t)place * plane_w);
            unsigned long long h = 0;                    // (what the search for equal states goes by)
            for (int w = tid; w < cnp * plane_q; w += NT) {
                const uint4 v = ldsq[w];
                child[w] = v;
                if (q_any(v)) h += hash_quad(v, (uint32_t)w);
            }
            uint32_t hl = (uint32_t)h, hh = (uint32_t)(h >> 32);
            for (int o = 32; o > 0; o >>= 1) {
                const unsigned long long other = ((unsigned long long)(uint32_t)__shfl_xor((int)hh, o, 64) << 32) | (uint32_t)__shfl_xor((int)hl, o, 64);
                h += other;
                hl = (uint32_t)h; hh = (uint32_t)(h >> 32);
            }
            if (lane == 0) s_hash[wave] = h;
        }
        __syncthreads();
        if (code != CODE_GOAL && tid == 0) {             // (written, not added up: the list needs no clearing)
            unsigned long long h = 0;
            for (int w = 0; w < NT / 64; ++w) h += s_hash[w];
            (cnp == 2 ? A.next_hash2 : A.next_hash1)[place] = h;
        }
        // ---- the step's time for every query of the enumeration (alpha-beta model: latency steps of the
        //      slowest group's link; bytes through the busiest uplink, from the query's bandwidth rows)
        double* out = (code == CODE_GOAL ? A.delta_goal : code == CODE_PREFIX2 ? A.delta2 : A.delta1) + (size_t)place * 2 * A.n_share;
        // Where every group holds the same number of rows c (the usual case), the busiest unit of a hardware level
        // carries c times the largest multiplicity sum of that level's rows, which the row tables carry per pattern:
        // the same maximum, term by term, without walking the rows; a lane per query then.
        const uint32_t c0 = s_count[0];
        bool same = true;
        for (int G = lane; G < ng; G += 64) same &= s_count[G] == c0;
        const bool uniform = __all(same) != 0;
        if (A.n_msg > 0 && uniform) {
            for (int j = tid; j < A.n_share; j += NT) {
                const DevQuery& cq = queries[A.share[j]];
                const DevRows& rw = *cq.rows;
                double best = 0.0;
                for (int l = 0; l < cq.n_levels; ++l)
                    best = fmax(best, (double)((long long)c0 * (long long)rw.level_max[pid][l]) * cq.inv_bw[l]);
                double ring_steps, mult;
                step_factors(op, P.g, cq.algo, ring_steps, mult);
                out[2 * j] = ring_steps * cq.alpha[cq.pat[pid].span_level];
                out[2 * j + 1] = (mult / (double)cq.k) * best;
            }
        } else if (A.n_msg > 0) {
            for (int j = wave; j < A.n_share; j += (NT / 64)) {
                const DevQuery& cq = queries[A.share[j]];
                const DevRows& rw = *cq.rows;
                double best = 0.0;
                for (int row = rw.pat_begin[pid] + lane; row < rw.pat_begin[pid + 1]; row += 64) {
                    long long dot = 0;
                    int e = rw.row_ptr[row];
                    const int e_end = rw.row_ptr[row + 1];
                    // (eight entries in flight: a row of the outer levels has an entry per group, and one load after the
                    //  other made this loop the longest part of the kernel)
                    for (; e + 8 <= e_end; e += 8) {
                        uint32_t ent[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) ent[u] = rw.entries[e + u];
#pragma unroll
                        for (int u = 0; u < 8; ++u) dot += (long long)entry_cnt(ent[u]) * (long long)s_count[entry_group(ent[u])];
                    }
                    for (; e < e_end; ++e) {
                        const uint32_t ent = rw.entries[e];
                        dot += (long long)entry_cnt(ent) * (long long)s_count[entry_group(ent)];
                    }
                    best = fmax(best, (double)dot * cq.inv_bw[rw.row_level[row]]);
                }
                for (int off = 32; off > 0; off >>= 1) best = fmax(best, __shfl_xor(best, off, 64));
                if (lane == 0) {
                    double ring_steps, mult;
                    step_factors(op, P.g, cq.algo, ring_steps, mult);
                    out[2 * j] = ring_steps * cq.alpha[cq.pat[pid].span_level];
                    out[2 * j + 1] = (mult / (double)cq.k) * best;
                }
            }
        }
    }
}

// ---- the children of the judged states, from their codes ----------------------------------------------
constexpr int kChildChunk = 8;
__global__ __launch_bounds__(256) void k_front_children(const DevQuery* __restrict__ qp, uint32_t n_states,
                                                        const uint32_t* __restrict__ list, const uint32_t* __restrict__ n_list,
                                                        const uint8_t* __restrict__ codes, const uint8_t* __restrict__ unknown, int np,
                                                        int keep, int write, uint32_t* __restrict__ child_of,
                                                        FrontSurvivor* __restrict__ ssurv, FrontCounters* __restrict__ ctr) {
    const uint32_t I = (uint32_t)qp->alphabet;
    const uint32_t CS = front_code_stride((int)I);
    const uint32_t n_work = list ? *n_list : n_states;
    // A wavefront takes kChildChunk states at a time, a lane per instruction: it counts the chunk's children by kind,
    // reserves their places once (the counters are few, and every reservation of the same word waits for the one
    // before it), and hands them out in a second pass over the chunk.
    const int lane = threadIdx.x & 63;
    uint32_t in_alphabet[2];                             // the bytes of a lane's two words that are instructions (invalid = 0 elsewhere)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int left = (int)I - (lane + 64 * h) * 4;
        in_alphabet[h] = left >= 4 ? 0xffffffffu : left > 0 ? ((1u << (8 * left)) - 1u) : 0u;
    }
    const uint32_t wave = (blockIdx.x * 256u + threadIdx.x) >> 6, n_waves = gridDim.x * 4u;
    for (uint32_t c0 = wave * kChildChunk; c0 < n_work; c0 += n_waves * kChildChunk) {
        const uint32_t c1 = min(c0 + (uint32_t)kChildChunk, n_work);
        // the rows of the chunk: four codes a word, a lane's two words of every row loaded before any is looked at
        // (an alphabet has at most 512 instructions: 128 words)
        uint32_t st_of[kChildChunk], four[kChildChunk][2];
#pragma unroll
        for (int b = 0; b < kChildChunk; ++b) {
            const uint32_t i = c0 + (uint32_t)b;
            st_of[b] = i < c1 ? (list ? list[i] : i) : 0u;
        }
        // (every load is made, from a state and a word that exist, and what was not asked for is dropped afterwards:
        //  loads under a condition are waited for one by one, these are in flight together)
        uint8_t unk[kChildChunk];
#pragma unroll
        for (int b = 0; b < kChildChunk; ++b) {
            unk[b] = unknown[st_of[b]];
            const uint32_t* const row = reinterpret_cast<const uint32_t*>(codes + (size_t)st_of[b] * CS);
#pragma unroll
            for (int h = 0; h < 2; ++h) four[b][h] = row[(uint32_t)(lane + 64 * h) < CS / 4u ? lane + 64 * h : 0];
        }
#pragma unroll
        for (int b = 0; b < kChildChunk; ++b) {
            const bool on = c0 + (uint32_t)b < c1 && !unk[b];                  // (an unknown state's prefixes go to the literal kernels)
#pragma unroll
            for (int h = 0; h < 2; ++h) four[b][h] = (on && (uint32_t)(lane + 64 * h) < CS / 4u) ? (four[b][h] & in_alphabet[h]) : 0u;
        }
        uint32_t mine[3] = {0u, 0u, 0u};
#pragma unroll
        for (int b = 0; b < kChildChunk; ++b) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (uint32_t j = 0; j < 4u; ++j) {
                    const int code = (int)((four[b][h] >> (8u * j)) & 0xffu);
                    mine[0] += (code == CODE_PREFIX && keep) ? 1u : 0u;
                    mine[1] += (code == CODE_PREFIX2 && keep) ? 1u : 0u;
                    mine[2] += code == CODE_GOAL ? 1u : 0u;
                }
            }
        }
        uint32_t before[3], total[3];                // over the lanes: exclusive sums, totals
#pragma unroll
        for (int kd = 0; kd < 3; ++kd) {
            uint32_t x = mine[kd];
            for (int o = 1; o < 64; o <<= 1) { const uint32_t y = __shfl_up(x, o, 64); if (lane >= o) x += y; }
            before[kd] = x - mine[kd];
            total[kd] = __shfl(x, 63, 64);
        }
        // One trip to the counters for the three kinds and the list: lanes 0-2 add a kind's total each, lane 3 the
        // length of the list (returning additions take a microsecond or two each, one after the other).
        uint32_t* const counts = write ? ctr->t_next : ctr->t_count;
        const uint32_t all = total[0] + total[1] + total[2];
        const uint32_t add = lane == 0 ? total[0] : lane == 1 ? total[1] : lane == 2 ? total[2] : (lane == 3 && write) ? all : 0u;
        uint32_t got = 0u;
        if (lane < 4 && add != 0u) got = atomicAdd(lane < 3 ? &counts[lane] : &ctr->n_ssurv, add);
        const uint32_t base[3] = {__shfl(got, 0, 64), __shfl(got, 1, 64), __shfl(got, 2, 64)};
        const uint32_t list_at = __shfl(got, 3, 64);
        if (!write) continue;
        if (all == 0) continue;
        uint32_t at_list = list_at + before[0] + before[1] + before[2];
        uint32_t next[3] = {base[0] + before[0], base[1] + before[1], base[2] + before[2]};
#pragma unroll
        for (int b = 0; b < kChildChunk; ++b) {
            const uint32_t st = st_of[b];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (four[b][h] == 0u) continue;
#pragma unroll
                for (uint32_t j = 0; j < 4u; ++j) {
                    const uint32_t a = (uint32_t)(lane + 64 * h) * 4u + j;
                    const int code = (int)((four[b][h] >> (8u * j)) & 0xffu);
                    const int kind = (code == CODE_PREFIX && keep) ? 0 : (code == CODE_PREFIX2 && keep) ? 1 : code == CODE_GOAL ? 2 : -1;
                    if (kind < 0) continue;
                    const uint32_t t = kind == 0 ? next[0]++ : kind == 1 ? next[1]++ : next[2]++;
                    child_of[(size_t)st * I + a] = t;
                    FrontSurvivor sv;
                    sv.entry = st; sv.digit = (uint16_t)a; sv.code = (uint16_t)(code | (np == 2 ? kFromTwoPair : 0)); sv.slot = t;
                    ssurv[at_list++] = sv;
                }
            }
        }
    }
}

// ---- the prefixes of the next level and the goals, from the survivors of this level's prefixes ------------
// A thread per (survivor, cost sum): the child's sums are the parent's plus what the step adds, which the kernel
// above worked out once per (state, instruction); the thread of the first sum also writes the record.
__global__ __launch_bounds__(256) void k_front_prefixes(const DevQuery* __restrict__ queries, FrontPrefixes A) {
    __shared__ unsigned long long s_made[2];
    if (threadIdx.x < 2) s_made[threadIdx.x] = 0ull;
    __syncthreads();
    const DevQuery& q = queries[A.query];
    const uint32_t I = (uint32_t)q.alphabet;
    const uint32_t per = A.n_msg > 0 ? 2u * (uint32_t)A.n_share : 1u;
    const unsigned long long total = (unsigned long long)A.n_surv * per;
    for (unsigned long long at = (unsigned long long)blockIdx.x * 256u + threadIdx.x; at < total; at += (unsigned long long)gridDim.x * 256u) {
        const uint32_t i = (uint32_t)(at / per), j = (uint32_t)(at - (unsigned long long)i * per);
        const FrontSurvivor sv = A.surv[i];
        const int code = sv.code & 0xff;
        const bool two = (sv.code & kFromTwoPair) != 0;
        const uint32_t place = sv.slot;
        if (code == CODE_PREFIX_LITERAL) {
            if (j == 0 && A.keep_prefixes) {
                const FrontEntry pe = (two ? A.entries2 : A.entries1)[sv.entry];
                FrontEntry ce;
                ce.query = A.query; ce.len = (uint32_t)(A.parent_len + 1);
                ce.digits = pe.digits | ((unsigned long long)sv.digit << (9 * A.parent_len));
                A.next_literal[atomicAdd(&A.ctr->next_literal, 1u)] = ce;
            }
            continue;
        }
        if (code != CODE_GOAL && !A.keep_prefixes) continue;     // the size limit is reached: nothing extends this prefix
        const uint32_t st = (two ? A.sid2 : A.sid1)[sv.entry];
        const uint32_t t = (two ? A.child_of2 : A.child_of1)[(size_t)st * I + sv.digit];
        if (A.n_msg > 0) {
            const double parent = (two ? A.sums2 : A.sums1)[(size_t)sv.entry * per + j];
            const double step = (code == CODE_GOAL ? A.delta_goal : code == CODE_PREFIX2 ? A.delta2 : A.delta1)[(size_t)t * per + j];
            double* out = code == CODE_GOAL ? A.goal_sums : code == CODE_PREFIX2 ? A.next_sums2 : A.next_sums1;
            out[(size_t)place * per + j] = parent + step;
        }
        if (j != 0) continue;
        const FrontEntry pe = (two ? A.entries2 : A.entries1)[sv.entry];
        const unsigned long long digits = pe.digits | ((unsigned long long)sv.digit << (9 * A.parent_len));
        if (code == CODE_GOAL) {
            A.valid_out[place] = rank_of(q, digits, A.parent_len + 1);
            continue;
        }
        FrontEntry ce;
        ce.query = A.query; ce.len = (uint32_t)(A.parent_len + 1); ce.digits = digits;
        if (code == CODE_PREFIX2) { A.next_entries2[place] = ce; A.next_sid2[place] = A.rep2 ? A.rep2[t] : t; }
        else { A.next_entries1[place] = ce; A.next_sid1[place] = A.rep1 ? A.rep1[t] : t; }
        // (an instruction application per child built, as if every prefix had its own state)
        const uint32_t ins = q.instr_of_digit[sv.digit];
        atomicAdd(&s_made[0], 1ull);
        atomicAdd(&s_made[1], (unsigned long long)(q.pat[ins >> 3].n_groups * q.pat[ins >> 3].g));
    }
    __syncthreads();
    if (threadIdx.x == 0 && s_made[0]) { atomicAdd(&A.ctr->steps, s_made[0]); atomicAdd(&A.ctr->members, s_made[1]); }
}

// Survivors of the literal frontier carry no state: a goal becomes a valid program, the rest
// prefixes of the next literal frontier.  Such a goal has no sums (NaN: its cost is worked out by
// the cost kernels that re-run a program).
__global__ __launch_bounds__(256) void k_front_emit(const DevQuery* __restrict__ qp, uint32_t query,
                                                    const FrontEntry* __restrict__ entries,
                                                    const FrontSurvivor* __restrict__ surv, uint32_t n_surv, int parent_len,
                                                    int keep_prefixes, FrontEntry* __restrict__ next_literal,
                                                    unsigned long long* __restrict__ valid_out, double* __restrict__ goal_sums,
                                                    int n_share, FrontCounters* __restrict__ ctr) {
    // (valid_out / goal_sums start behind the goals of this level that the pair kernels found)
    const DevQuery& q = *qp;
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n_surv) return;
    const FrontSurvivor sv = surv[i];
    const unsigned long long digits = entries[sv.entry].digits | ((unsigned long long)sv.digit << (9 * parent_len));
    if (sv.code == CODE_GOAL) {
        const uint32_t slot = atomicAdd(&ctr->next_goal_literal, 1u);
        valid_out[slot] = rank_of(q, digits, parent_len + 1);
        for (int j = 0; j < 2 * n_share; ++j) goal_sums[(size_t)slot * 2 * n_share + j] = __longlong_as_double(0x7ff8000000000000ll);
    } else if (keep_prefixes) {
        FrontEntry ce;
        ce.query = query; ce.len = (uint32_t)(parent_len + 1); ce.digits = digits;
        next_literal[atomicAdd(&ctr->next_literal, 1u)] = ce;
    }
}

template <int KW, int MW>
__global__ __launch_bounds__(64) void k_front_init(const DevQuery* __restrict__ qp, uint32_t query, FrontEntry* entries,
                                                   uint32_t* states, double* sums, uint32_t* sid, int n_share) {
    // Sec. 3.5: the empty program; device i holds column i in every row
    const DevQuery& q = *qp;
    constexpr int WPD = FL<KW, MW>::WS;
    const Words<KW> all_rows = full_mask<KW>(q.k);
    for (int i = threadIdx.x; i < q.R * WPD; i += 64) states[i] = 0u;         // (the padding stays zero for good)
    __syncthreads();
    for (int d = threadIdx.x; d < q.R; d += 64) {
        Words<MW> m;
#pragma unroll
        for (int i = 0; i < MW; ++i) m.w[i] = (i == (d >> 5)) ? (1u << (d & 31)) : 0u;
        fstore<KW, MW>(states, d, all_rows, m);
    }
    for (int j = threadIdx.x; j < 2 * n_share; j += 64) sums[j] = 0.0;
    if (threadIdx.x == 0) { FrontEntry e; e.query = query; e.len = 0; e.digits = 0ull; entries[0] = e; sid[0] = 0u; }
}

// Programs and costs of an enumeration's valid programs for one of its queries: entry i of the unordered
// list, whose place in ascending index order is rank[i], becomes row out_first + rank[i] (row out_first + i where
// no order is asked for: rank null).
__global__ __launch_bounds__(256) void k_front_finish(const DevQuery* __restrict__ queries, const FrontFinish* __restrict__ jobs) {
    const FrontFinish F = jobs[blockIdx.y];              // (a query per grid row)
    const DevQuery& q = queries[F.query];
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < F.n_valid; i += gridDim.x * 256u) {
    const unsigned long long idx = F.valid[i];
    const size_t row = F.out_first + (F.rank ? F.rank[i] : i);
    int len = 1;
    while (len < q.max_len && idx >= q.base[len + 1]) ++len;
    p2_program pr;
    pr.index = idx;
    pr.len = (uint8_t)len;
    for (int t = 0; t < P2_MAX_LEN; ++t) pr.instr[t] = 0;
    unsigned long long rem = idx - q.base[len];
    const unsigned long long I = (unsigned long long)q.alphabet;
    for (int t = len - 1; t >= 0; --t) {
        const unsigned long long nx = rem / I;
        const uint32_t ins = q.instr_of_digit[(uint32_t)(rem - nx * I)];
        pr.instr[t] = (uint8_t)((ins >> 3) * 5u + (ins & 7u));
        rem = nx;
    }
    F.sorted[row] = idx;
    F.progs[row] = pr;
    const double sa = F.goal_sums[((size_t)i * F.n_share + F.share_pos) * 2], sb = F.goal_sums[((size_t)i * F.n_share + F.share_pos) * 2 + 1];
    for (int m = 0; m < q.n_msg; ++m) F.costs[row * q.n_msg + m] = sa + q.msg_bytes[m] * sb;
    }
}

// The level's counters to the host (dst: pinned host memory the device can write), before the host's one wait of the
// level; the counters that only the second half of the level uses (places handed out while the children and the next
// lists are written) start from zero there, so they are cleared here rather than by a fill of their own.
__global__ __launch_bounds__(64) void k_front_counters_out(FrontCounters* __restrict__ dst, FrontCounters* __restrict__ ctr) {
    static_assert(sizeof(FrontCounters) % 4 == 0, "copied word by word");
    const uint32_t* const src = reinterpret_cast<const uint32_t*>(ctr);
    uint32_t* const out = reinterpret_cast<uint32_t*>(dst);
    for (uint32_t i = threadIdx.x; i < sizeof(FrontCounters) / 4; i += 64u) out[i] = src[i];
    __syncthreads();
    if (threadIdx.x == 0) {
        ctr->next_literal = 0u; ctr->next_goal_literal = 0u; ctr->n_ssurv = 0u;
        ctr->t_next[0] = 0u; ctr->t_next[1] = 0u; ctr->t_next[2] = 0u;
    }
}

// rank[i] = number of entries of the list smaller than entry i (distinct keys).
__global__ __launch_bounds__(256) void k_front_rank(const unsigned long long* __restrict__ in, uint32_t n, uint32_t* __restrict__ rank) {
    __shared__ unsigned long long tile[256];
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    const unsigned long long key = i < n ? in[i] : 0ull;
    uint32_t r = 0;
    for (uint32_t t0 = 0; t0 < n; t0 += 256u) {
        const uint32_t j = t0 + threadIdx.x;
        tile[threadIdx.x] = j < n ? in[j] : ~0ull;
        __syncthreads();
        const uint32_t lim = n - t0 < 256u ? n - t0 : 256u;
        for (uint32_t u = 0; u < lim; ++u) r += tile[u] < key;
        __syncthreads();
    }
    if (i < n) rank[i] = r;
}

inline int round_words_f(int bits) {
    const int w = (bits + 31) / 32;
    return w <= 1 ? 1 : w <= 2 ? 2 : w <= 4 ? 4 : w <= 8 ? 8 : 16;
}

template <typename F>
hipError_t allow_lds_f(F func, size_t bytes) {
    if (bytes <= 32 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(func), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

struct FrontArgs {
    const DevQuery* q; uint32_t query;
    const FrontEntry* entries; const uint32_t* states; uint32_t n;
    int np, max_pairs;
    const uint32_t* list; const uint32_t* n_list;
    uint8_t* codes; uint8_t* unknown; int goals_only, count_children; FrontCounters* ctr;
    uint32_t* walk; uint32_t* n_walk; uint2* row_counts;
    double* sums; uint32_t* sid; int n_share;
    const DevQuery* queries; const FrontLevel* level;
    int R;
};

template <int KW, int MW>
hipError_t front_go(int what, const FrontArgs& A, hipStream_t stream) {
    if (what == 0) {
        hipLaunchKernelGGL((k_front_init<KW, MW>), dim3(1), dim3(64), 0, stream, A.q, A.query, const_cast<FrontEntry*>(A.entries),
                           const_cast<uint32_t*>(A.states), A.sums, A.sid, A.n_share);
    } else if (what == 1) {
        const size_t lds = (size_t)A.np * A.R * FL<KW, MW>::WS * 4 + (((size_t)A.R + 15) & ~(size_t)15);
        // (a block keeps going over entries: what it sets up at its start is paid once; with a list of distinct
        //  states the number of entries is only known on the device, at most n)
        const unsigned want = A.list ? (A.n + 1u) / 2u : A.n;
        const unsigned blocks = want < 2048u ? want : 2048u;
        hipError_t e = A.np == 2 ? allow_lds_f(k_front_classify<KW, MW, 2>, lds) : allow_lds_f(k_front_classify<KW, MW, 1>, lds);
        if (e != hipSuccess) return e;
        if (A.np == 2)
            hipLaunchKernelGGL((k_front_classify<KW, MW, 2>), dim3(blocks), dim3(kClsThreads), lds, stream, A.q, A.states, A.n, A.list,
                               A.n_list, A.max_pairs, A.goals_only, A.count_children, A.codes, A.row_counts, A.unknown, A.ctr);
        else
            hipLaunchKernelGGL((k_front_classify<KW, MW, 1>), dim3(blocks), dim3(kClsThreads), lds, stream, A.q, A.states, A.n, A.list,
                               A.n_list, A.max_pairs, A.goals_only, A.count_children, A.codes, A.row_counts, A.unknown, A.ctr);
    } else if (what == 3) {
        // a wavefront per state, four to a block
        const unsigned want = (A.n + 3u) / 4u;
        const unsigned blocks = want < 16384u ? want : 16384u;
        if (A.np == 2)
            hipLaunchKernelGGL((k_front_goal_filter<KW, MW, 2>), dim3(blocks), dim3(256), 0, stream, A.q, A.states, A.n, A.list, A.n_list,
                               A.codes, A.row_counts, A.unknown, A.walk, A.n_walk);
        else
            hipLaunchKernelGGL((k_front_goal_filter<KW, MW, 1>), dim3(blocks), dim3(256), 0, stream, A.q, A.states, A.n, A.list, A.n_list,
                               A.codes, A.row_counts, A.unknown, A.walk, A.n_walk);
    } else {
        const size_t lds = (size_t)A.level->lds_planes * A.R * FL<KW, MW>::WS * 4;
        const unsigned blocks = A.level->n_surv < 8192u ? A.level->n_surv : 8192u;
        if (lds > kMatBigLds) {
            const hipError_t e = allow_lds_f(k_front_materialize<KW, MW, kMatThreadsBig>, lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((k_front_materialize<KW, MW, kMatThreadsBig>), dim3(blocks), dim3(kMatThreadsBig), lds, stream, A.queries, *A.level);
        } else {
            const hipError_t e = allow_lds_f(k_front_materialize<KW, MW, kMatThreads>, lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((k_front_materialize<KW, MW, kMatThreads>), dim3(blocks), dim3(kMatThreads), lds, stream, A.queries, *A.level);
        }
    }
    return hipGetLastError();
}

template <int KW>
hipError_t front_mw(int MW, int what, const FrontArgs& A, hipStream_t stream) {
    switch (MW) {
    case 1: return front_go<KW, 1>(what, A, stream);
    case 2: return front_go<KW, 2>(what, A, stream);
    case 4: return front_go<KW, 4>(what, A, stream);
    case 8: return front_go<KW, 8>(what, A, stream);
    default: return front_go<KW, 16>(what, A, stream);
    }
}

hipError_t front_dispatch(int R, int k, int what, const FrontArgs& A, hipStream_t stream) {
    const int MW = round_words_f(R);
    switch (round_words_f(k)) {
    case 1: return front_mw<1>(MW, what, A, stream);
    case 2: return front_mw<2>(MW, what, A, stream);
    case 4: return front_mw<4>(MW, what, A, stream);
    case 8: return front_mw<8>(MW, what, A, stream);
    default: return front_mw<16>(MW, what, A, stream);
    }
}

}  // namespace

size_t frontier_state_words(int R, int k) {
    return (size_t)R * 4 * (size_t)((round_words_f(k) + 3) / 4 + (round_words_f(R) + 3) / 4);      // FL<KW, MW>::WS per device
}

// Two planes must fit in LDS for the two-pair list to be used.
int frontier_max_pairs(int R, int k) { return frontier_state_words(R, k) * 2 * 4 + 2048 <= kLdsBudget ? 2 : 1; }

hipError_t launch_front_init(const DevQuery* q, uint32_t query, int R, int k, FrontEntry* entries, uint32_t* states,
                             double* sums, uint32_t* sid, int n_share, hipStream_t stream) {
    FrontArgs A{};
    A.q = q; A.query = query; A.entries = entries; A.states = states; A.R = R; A.sums = sums; A.sid = sid; A.n_share = n_share;
    return front_dispatch(R, k, 0, A, stream);
}

hipError_t launch_front_children(const DevQuery* q, uint32_t n, const uint32_t* list, const uint32_t* n_list, const uint8_t* codes,
                                 const uint8_t* unknown, int np, int keep, int write, uint32_t* child_of, FrontSurvivor* ssurv,
                                 FrontCounters* ctr, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const unsigned want = (n + 4u * kChildChunk - 1u) / (4u * kChildChunk);      // (a wavefront per chunk of states)
    hipLaunchKernelGGL(k_front_children, dim3(want < 4096u ? want : 4096u), dim3(256), 0, stream, q, n, list, n_list, codes, unknown, np,
                       keep, write, child_of, ssurv, ctr);
    return hipGetLastError();
}

hipError_t launch_front_prefixes(const DevQuery* queries, const FrontPrefixes& P, hipStream_t stream) {
    if (P.n_surv == 0) return hipSuccess;
    const unsigned long long total = (unsigned long long)P.n_surv * (P.n_msg > 0 ? 2ull * (unsigned long long)P.n_share : 1ull);
    // (every block ends with two additions to the level's counters, and additions to one address are served one after
    //  the other, some 10⁸ a second: with 16 384 blocks they were the whole time of the kernel, 0.4 ms)
    const unsigned long long want = (total + 255ull) / 256ull;
    hipLaunchKernelGGL(k_front_prefixes, dim3((unsigned)(want < 2048ull ? want : 2048ull)), dim3(256), 0, stream, queries, P);
    return hipGetLastError();
}

hipError_t launch_front_goal_filter(const DevQuery* q, int R, int k, const uint32_t* states, uint32_t n, const uint32_t* list,
                                    const uint32_t* n_list, int np, uint8_t* codes, unsigned long long* row_counts, uint8_t* unknown,
                                    uint32_t* walk, uint32_t* n_walk, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    FrontArgs A{};
    A.q = q; A.states = states; A.n = n; A.np = np; A.list = list; A.n_list = n_list;
    A.codes = codes; A.unknown = unknown; A.R = R; A.walk = walk; A.n_walk = n_walk; A.row_counts = reinterpret_cast<uint2*>(row_counts);
    return front_dispatch(R, k, 3, A, stream);
}

hipError_t launch_front_classify(const DevQuery* q, int R, int k, const uint32_t* states, uint32_t n, const uint32_t* list,
                                 const uint32_t* n_list, int np, int max_pairs, int goals_only, int count_children, uint8_t* codes,
                                 unsigned long long* row_counts, uint8_t* unknown, FrontCounters* ctr, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    FrontArgs A{};
    A.q = q; A.states = states; A.n = n; A.np = np; A.max_pairs = max_pairs; A.list = list; A.n_list = n_list;
    A.codes = codes; A.unknown = unknown; A.R = R; A.goals_only = goals_only; A.count_children = count_children; A.ctr = ctr; A.row_counts = reinterpret_cast<uint2*>(row_counts);
    return front_dispatch(R, k, 1, A, stream);
}

hipError_t launch_front_dedup(const uint32_t* states, size_t state_words, const unsigned long long* hash, uint32_t n,
                              unsigned long long* table, uint32_t table_size, uint32_t* rep, uint32_t* reps_list,
                              uint32_t* n_reps, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_front_dedup, dim3((n + 255u) / 256u), dim3(256), 0, stream, hash, n, table, table_size - 1u, rep, reps_list, n_reps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const unsigned waves = n, blocks = (waves + 3u) / 4u;
    hipLaunchKernelGGL(k_front_verify, dim3(blocks < 8192u ? blocks : 8192u), dim3(256), 0, stream,
                       reinterpret_cast<const uint4*>(states), (uint32_t)(state_words / 4), n, rep, reps_list, n_reps);
    return hipGetLastError();
}

hipError_t launch_front_expand(const DevQuery* q, const FrontEntry* entries, uint32_t n, const uint32_t* rep,
                               const uint8_t* codes, const unsigned long long* row_counts, const uint8_t* unknown, int np, int handover,
                               FrontSurvivor* surv, uint32_t surv_cap, FrontEntry* unknown_out, FrontCounters* ctr, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    // entries per wavefront: as many as leave some 4096 wavefronts to share the second pass
    int epw = 8;
    while (epw < 64 && n / (unsigned)epw > 4096u) epw *= 2;
    const unsigned per_block = (unsigned)(kExpWaves * epw), want = (n + per_block - 1) / per_block;
    const unsigned blocks = want < 2048u ? want : 2048u;
    const uint2* const rc = reinterpret_cast<const uint2*>(row_counts);
    if (np == 2)
        hipLaunchKernelGGL(k_front_expand<2>, dim3(blocks), dim3(kExpThreads), 0, stream, q, entries, n, rep, codes, rc, unknown, handover, epw, surv,
                           surv_cap, unknown_out, ctr);
    else
        hipLaunchKernelGGL(k_front_expand<1>, dim3(blocks), dim3(kExpThreads), 0, stream, q, entries, n, rep, codes, rc, unknown, handover, epw, surv,
                           surv_cap, unknown_out, ctr);
    return hipGetLastError();
}

hipError_t launch_front_counters_out(FrontCounters* host_dst, FrontCounters* ctr, hipStream_t stream) {
    hipLaunchKernelGGL(k_front_counters_out, dim3(1), dim3(64), 0, stream, host_dst, ctr);
    return hipGetLastError();
}

hipError_t launch_front_materialize(const DevQuery* queries, int R, int k, const FrontLevel& level, hipStream_t stream) {
    if (level.n_surv == 0) return hipSuccess;
    FrontArgs A{};
    A.queries = queries; A.level = &level; A.R = R;
    return front_dispatch(R, k, 2, A, stream);
}

hipError_t launch_front_emit(const DevQuery* q, uint32_t query, const FrontEntry* entries, const FrontSurvivor* surv,
                             uint32_t n_surv, int parent_len, int keep_prefixes, FrontEntry* next_literal,
                             unsigned long long* valid_out, double* goal_sums, int n_share, FrontCounters* ctr,
                             hipStream_t stream) {
    if (n_surv == 0) return hipSuccess;
    hipLaunchKernelGGL(k_front_emit, dim3((n_surv + 255u) / 256u), dim3(256), 0, stream, q, query, entries, surv, n_surv, parent_len,
                       keep_prefixes, next_literal, valid_out, goal_sums, n_share, ctr);
    return hipGetLastError();
}

hipError_t launch_front_rank(const unsigned long long* valid, uint32_t n, uint32_t* rank, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_front_rank, dim3((n + 255u) / 256u), dim3(256), 0, stream, valid, n, rank);
    return hipGetLastError();
}

hipError_t launch_front_finish(const DevQuery* queries, const FrontFinish* jobs, uint32_t n_jobs, uint32_t max_valid, hipStream_t stream) {
    if (n_jobs == 0 || max_valid == 0) return hipSuccess;
    const uint32_t want = (max_valid + 255u) / 256u;
    for (uint32_t j0 = 0; j0 < n_jobs; j0 += 65535u) {
        const uint32_t nj = n_jobs - j0 < 65535u ? n_jobs - j0 : 65535u;
        hipLaunchKernelGGL(k_front_finish, dim3(want < 1024u ? want : 1024u, nj), dim3(256), 0, stream, queries, jobs + j0);
    }
    return hipGetLastError();
}

}  // namespace p2
