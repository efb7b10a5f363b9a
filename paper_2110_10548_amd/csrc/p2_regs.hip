// Per-candidate engine for small reduction groups: one candidate per lane, every step computed in
// registers.
//
// Same state form as p2_compact.hip -- per device one chunk set and one contribution mask -- for
// R <= 32 devices and k <= 32 chunks, so a pair is two 32-bit words and a candidate's state is 64
// words.  Between steps the state rests in LDS (pair of device d of lane l at byte l*8 + d*512, so
// every access of the wavefront is conflict-free and addressed with a constant offset).  A step
// loads all 32 pairs back to back (one LDS round trip), applies the rule in registers as straight
// vector code without address arithmetic, and writes the pairs back only if the step is valid and
// is not the last; the first step uses the closed form of the rules on the init state.
//
// Registers cannot be indexed by a run-time device number.  For patterns whose group size g and
// stride s are powers of two (every pattern of a hierarchy with power-of-two levels), the members
// of a group differ exactly in bits [log2 s, log2 s + log2 g) of the device number, so a rule is
// applied as a sequence of stages, one per such bit J: stage J combines every device d whose bit J
// is clear with d + 2^J.  The 16 pairs of a stage are compile-time constants; only J (five values)
// selects code.
//   AllReduce-like : union of the masks along each bit; the two sides of every pair must hold the
//                    same chunks and disjoint masks (the sides' running unions are disjoint at
//                    every stage iff all members are pairwise disjoint).
//   ReduceScatter  : then the member of rank p keeps the p-th block of the chunks.
//   Reduce         : then every member that has one of the bits set is cleared.
//   AllGather      : union of the chunk sets along each bit, sides disjoint; nobody empty.
//   Broadcast      : binomial tree from the device with all bits clear; a member is compared with
//                    the root's pair right before it is overwritten.
// Devices outside the pattern (Master forms, or R < 32) are neutralised by a scalar all-zero mask
// per pair, so a stage has no control flow.
//
// The 64 lanes of a wavefront hold consecutive candidates.  At a step the lanes that share the
// first pending lane's instruction run it together under their execution mask; the others wait
// for the next round.  Prefix instructions are the same in all lanes, so they take one round.  The
// last instruction, different in every lane, is judged per lane without writing the state.
#include "p2_device.h"

namespace p2 {

namespace {

constexpr int kWaveR = 64;
constexpr int kRegDevices = 32;

enum : int { RSTEP_INVALID = 0, RSTEP_OK = 1, RSTEP_GIVE_UP = 2, RSTEP_GOAL = 3 };

struct RegState {
    uint32_t r[kRegDevices];   // chunk set of device d
    uint32_t m[kRegDevices];   // contribution mask of its non-empty rows
};

// the n lowest set bits of v, n <= popc(v)
__device__ inline uint32_t lowest_bits(uint32_t v, int n) {
    if (n >= __popc(v)) return v;
    uint32_t pos = 0;
#pragma unroll
    for (uint32_t b = 16; b > 0; b >>= 1) {
        const int t = __popc(v & ((1u << (pos + b)) - 1u));
        if (t <= n) pos += b;
    }
    return v & ((1u << pos) - 1u);
}

// All ones if device d takes part in the instruction, else zero (part is wave-uniform, d a constant).
// Without PRED every device takes part and the masks fold away.
template <bool PRED>
__device__ __forceinline__ uint32_t lane_mask_of(uint32_t part, int d) {
    return (!PRED || ((part >> d) & 1u)) ? 0xffffffffu : 0u;
}

// AllReduce-like stage along bit J: same chunks, disjoint masks, union of the masks on both sides.
// Pairs outside the pattern are neutralised by their all-zero mask pm instead of being branched around.
template <int J, bool PRED>
__device__ __forceinline__ void stage_red(RegState& st, uint32_t part, uint32_t& badx) {
#pragma unroll
    for (int d = 0; d < kRegDevices; ++d) {
        if (d & (1 << J)) continue;
        const int e = d | (1 << J);
        const uint32_t pm = lane_mask_of<PRED>(part, d);
        badx |= ((st.r[d] ^ st.r[e]) | (st.m[d] & st.m[e])) & pm;
        const uint32_t md = st.m[d];
        st.m[d] |= st.m[e] & pm;
        st.m[e] |= md & pm;
    }
}
// AllGather stage along bit J: disjoint chunk sets, union on both sides; smx collects mask differences.
template <int J, bool PRED>
__device__ __forceinline__ void stage_gather(RegState& st, uint32_t part, uint32_t& badx, uint32_t& smx) {
#pragma unroll
    for (int d = 0; d < kRegDevices; ++d) {
        if (d & (1 << J)) continue;
        const int e = d | (1 << J);
        const uint32_t pm = lane_mask_of<PRED>(part, d);
        badx |= (st.r[d] & st.r[e]) & pm;
        smx |= (st.m[d] ^ st.m[e]) & pm;
        const uint32_t rd = st.r[d];
        st.r[d] |= st.r[e] & pm;
        st.r[e] |= rd & pm;
    }
}
// Broadcast stage along bit J: devices that already hold the root's pair (their group bits from J
// up are clear) overwrite their partner; neq gets bit e where the partner differed.
template <int J>
__device__ __forceinline__ void stage_bcast(RegState& st, uint32_t part, uint32_t gmask, uint32_t& badx, uint32_t& neq) {
    const uint32_t high = gmask & (~0u << J);
#pragma unroll
    for (int d = 0; d < kRegDevices; ++d) {
        if (d & (1 << J)) continue;
        const int e = d | (1 << J);
        const uint32_t pm = (((part >> d) & 1u) && ((uint32_t)d & high) == 0u) ? 0xffffffffu : 0u;
        badx |= ((st.r[e] & ~st.r[d]) | (st.m[e] & ~st.m[d])) & pm;
        const uint32_t dif = ((st.r[e] ^ st.r[d]) | (st.m[e] ^ st.m[d])) & pm;
        neq |= dif != 0u ? (1u << e) : 0u;
        st.r[e] = (st.r[d] & pm) | (st.r[e] & ~pm);
        st.m[e] = (st.m[d] & pm) | (st.m[e] & ~pm);
    }
}
// ReduceScatter: the member of rank p (bits [ls, ls + lg) of its number) keeps the p-th block of
// the chunks in ascending order.
template <bool PRED>
__device__ __forceinline__ void scatter_rows(RegState& st, uint32_t part, int lg, int ls, uint32_t& badx) {
    const int gm1 = (1 << lg) - 1;
#pragma unroll
    for (int d = 0; d < kRegDevices; ++d) {
        const uint32_t pm = lane_mask_of<PRED>(part, d);
        const int p = (d >> ls) & gm1;
        const uint32_t v = st.r[d];
        const int c = __popc(v);
        const int per = c >> lg;
        badx |= (uint32_t)(c & gm1) & pm;            // the chunks must divide evenly
        const uint32_t lowbit = v & (0u - v);
        uint32_t nv;
        if (((v + lowbit) & v) == 0u) {
            // one run of ones: the block is a run of `per` ones, p blocks further up
            nv = (((lowbit << per) - lowbit) << (p * per)) & v;
        } else {
            nv = lowest_bits(v, (p + 1) * per) ^ lowest_bits(v, p * per);
        }
        st.r[d] = PRED ? ((nv & pm) | (v & ~pm)) : nv;
    }
}

// One instruction on the register state; all arguments but the state are wave-uniform.
// lg, ls: log2 of group size and stride; part: bit d set iff device d takes part (all do without PRED).
template <bool PRED>
__device__ __forceinline__ int reg_step(RegState& st, int op, int lg, int ls, uint32_t part) {
    const uint32_t gmask = ((1u << lg) - 1u) << ls;
    uint32_t badx = 0;          // any bit set: a premise failed
    uint32_t chgx = 1;          // zero: the instruction leaves the state as it is
    uint32_t smx = 0;           // AllGather of members with different masks: this form cannot hold the result
#define P2_STAGES(CALL)                                                                  \
    if (ls <= 0 && 0 < ls + lg) { CALL(0) if (__all(badx != 0u)) return RSTEP_INVALID; } \
    if (ls <= 1 && 1 < ls + lg) { CALL(1) if (__all(badx != 0u)) return RSTEP_INVALID; } \
    if (ls <= 2 && 2 < ls + lg) { CALL(2) if (__all(badx != 0u)) return RSTEP_INVALID; } \
    if (ls <= 3 && 3 < ls + lg) { CALL(3) if (__all(badx != 0u)) return RSTEP_INVALID; } \
    if (ls <= 4 && 4 < ls + lg) { CALL(4) if (__all(badx != 0u)) return RSTEP_INVALID; }
    if (op == OP_AR || op == OP_RS || op == OP_RD) {
#define P2_CALL(JV) stage_red<JV, PRED>(st, part, badx);
        P2_STAGES(P2_CALL)
#undef P2_CALL
        // a group of empty devices is a no-op; the chunk sets of a group are equal, so any device tells
        chgx = 0;
#pragma unroll
        for (int d = 0; d < kRegDevices; ++d) chgx |= st.r[d] & lane_mask_of<PRED>(part, d);
        if (op == OP_RS) {
            scatter_rows<PRED>(st, part, lg, ls, badx);
        } else if (op == OP_RD) {
#pragma unroll
            for (int d = 0; d < kRegDevices; ++d) {
                const uint32_t keep = (((part >> d) & 1u) && ((uint32_t)d & gmask) != 0u) ? 0u : 0xffffffffu;
                st.r[d] &= keep;
                st.m[d] &= keep;
            }
        }
    } else if (op == OP_AG) {
        // nobody empty
        uint32_t least = 0xffffffffu;
#pragma unroll
        for (int d = 0; d < kRegDevices; ++d) least = min(least, st.r[d] | ~lane_mask_of<PRED>(part, d));
        badx |= (uint32_t)(least == 0u);
        if (__all(badx != 0u)) return RSTEP_INVALID;
#define P2_CALL(JV) stage_gather<JV, PRED>(st, part, badx, smx);
        P2_STAGES(P2_CALL)
#undef P2_CALL
    } else {
        // the root holds what every member holds, and in every group more than at least one of them
        uint32_t neq = 0;
#define P2_CALL(JV) stage_bcast<JV>(st, part, gmask, badx, neq);
        P2_STAGES(P2_CALL)
#undef P2_CALL
        // fold the difference flags of a group onto its root's bit
        uint32_t roots = 0;
#pragma unroll
        for (int d = 0; d < kRegDevices; ++d)
            if (((part >> d) & 1u) && ((uint32_t)d & gmask) == 0u) roots |= 1u << d;
        for (int J = ls; J < ls + lg; ++J) neq |= neq >> (1u << J);
        badx |= ~neq & roots;
    }
#undef P2_STAGES
    if (badx != 0u || chgx == 0u) return RSTEP_INVALID;
    return smx != 0u ? RSTEP_GIVE_UP : RSTEP_OK;     // rows with different column sets leave this form
}

// The first instruction, on the init state of Sec. 3.5 (device i holds column i in every chunk):
// what the rules give there is known in closed form.  The members of a group hold the same chunks
// and disjoint columns, so the AllReduce-like rules always apply (ReduceScatter if g divides k):
// every member ends with the group's columns; AllGather and Broadcast never apply (every member
// holds every chunk; no member's columns lie inside the root's).  All values are wave-uniform;
// the new state goes straight to LDS.  Returns false if the step is invalid.
__device__ __forceinline__ bool first_step(uint2* my, int op, int lg, int ls, uint32_t part, int k, uint32_t all_rows) {
    if (op == OP_AG || op == OP_BC) return false;
    const int gm1 = (1 << lg) - 1;
    if (op == OP_RS && (k & gm1) != 0) return false;
    const uint32_t gmask = (uint32_t)gm1 << ls;
    uint32_t gcols = 1u;                              // columns of the group of device 0
    for (int j = ls; j < ls + lg; ++j) gcols |= gcols << (1u << j);
    const int per = k >> lg;
    const uint32_t block = per >= 32 ? 0xffffffffu : ((1u << per) - 1u);
    if (__ballot(1) == ~0ull) {
        // the whole wavefront is here: lane d works out the pair of device d (mod 32) once, and every
        // lane then stores the 32 pairs, read from those lanes, into its own candidate's state
        const int d = (int)(threadIdx.x & (kRegDevices - 1));
        uint32_t r = all_rows, m = 1u << d;
        if ((part >> d) & 1u) {
            const int p = (d >> ls) & gm1;
            m = gcols << ((uint32_t)d & ~gmask);
            if (op == OP_RS) r = block << (p * per);
            else if (op == OP_RD && p != 0) { r = 0u; m = 0u; }
        }
#pragma unroll
        for (int dd = 0; dd < kRegDevices; ++dd)
            my[dd * kWaveR] = make_uint2((uint32_t)__builtin_amdgcn_readlane((int)r, dd), (uint32_t)__builtin_amdgcn_readlane((int)m, dd));
        return true;
    }
#pragma unroll
    for (int d = 0; d < kRegDevices; ++d) {
        uint32_t r = all_rows, m = 1u << d;
        if ((part >> d) & 1u) {
            const int p = (d >> ls) & gm1;
            m = gcols << ((uint32_t)d & ~gmask);
            if (op == OP_RS) r = block << (p * per);
            else if (op == OP_RD && p != 0) { r = 0u; m = 0u; }
        }
        my[d * kWaveR] = make_uint2(r, m);
    }
    return true;
}

// The last instruction of a candidate, a different one in every lane: decides from the state in LDS
// (pair of device d at my[d * STRIDE]),
// without writing it, whether the step is valid and its result the goal.  All arguments are per lane.
// Members are visited in group-major order, eight loads at a time.
template <int STRIDE>
__device__ __forceinline__ int judge_last(const uint2* my, uint32_t shape, int op, int R, uint32_t all_rows, uint32_t all_cols) {
    const int lg = (int)(shape & 15u), ls = (int)((shape >> 4) & 15u);
    const bool master = ((shape >> 8) & 1u) != 0u;
    const int n_part = (int)(shape >> 16);
    const int gm1 = (1 << lg) - 1, sm1 = (1 << ls) - 1;
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    uint32_t badx = 0;
    bool changed = false, all_goal = true;
    uint32_t fr = 0, fm = 0, ar = 0, am = 0, eqx = 0, dmx = 0, drx = 0, smx = 0, subx = 0;
    bool anyzero = false;
    constexpr int NB = 8;
    for (int j0 = 0; j0 < n_part && badx == 0u; j0 += NB) {
        uint2 L[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int j = j0 + b;
            if (j < n_part) {
                const int G = j >> lg, p = j & gm1;
                const int base = master ? (G << (lg + ls)) : (((G >> ls) << (lg + ls)) + (G & sm1));
                L[b] = my[(base + (p << ls)) * STRIDE];
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int j = j0 + b;
            if (j >= n_part) continue;
            const int p = j & gm1;
            const uint32_t r = L[b].x, m = L[b].y;
            if (p == 0) {
                fr = r; fm = m; ar = r; am = m;
                eqx = 0; dmx = 0; drx = 0; smx = 0; subx = 0;
                anyzero = r == 0u;
            } else {
                eqx |= r ^ fr;                 // same chunks on every member
                dmx |= m & am;                 // no contribution reduced twice
                drx |= r & ar;                 // AllGather: chunks held once
                smx |= m ^ fm;
                subx |= (r & ~fr) | (m & ~fm); // Broadcast: the root knows more
                anyzero |= r == 0u;            // AllGather: nobody empty
                ar |= r;
                am |= m;
            }
            if (p == gm1) {
                if (red) {
                    badx |= eqx | dmx;
                    changed |= fr != 0u;       // a group of empty devices is a no-op
                    if (op == OP_RS) badx |= (uint32_t)(__popc(fr) & gm1);   // chunks must divide evenly
                    // AllReduce leaves (same chunks, union of masks) on every member; ReduceScatter and
                    // Reduce leave members with fewer chunks than the goal has
                    all_goal &= op == OP_AR && ((fr ^ all_rows) | (am ^ all_cols)) == 0u;
                } else if (op == OP_AG) {
                    badx |= drx | (uint32_t)anyzero;
                    changed = true;
                    // members with different masks leave rows with different column sets: never the goal
                    all_goal &= (smx | (ar ^ all_rows) | (fm ^ all_cols)) == 0u;
                } else {
                    badx |= subx | (uint32_t)((eqx | smx) == 0u);   // information increase
                    changed = true;
                    all_goal &= ((fr ^ all_rows) | (fm ^ all_cols)) == 0u;
                }
            }
        }
    }
    if (badx != 0u || !changed) return RSTEP_INVALID;
    if (!all_goal) return RSTEP_OK;
    if (master) {
        // devices outside the pattern must be at the goal already
        uint32_t dif = 0;
        for (int d = 0; d < R; ++d) {
            if ((d & sm1) == 0) continue;
            const uint2 v = my[d * STRIDE];
            dif |= (v.x ^ all_rows) | (v.y ^ all_cols);
        }
        if (dif != 0u) return RSTEP_OK;
    }
    return RSTEP_GOAL;
}

// Flat evaluation, one candidate per lane, as k_eval_compact.
__global__ __launch_bounds__(kWaveR) void k_eval_regs(const DevQuery* __restrict__ queries,
                                                      const DevSegment* __restrict__ segs, int n_segs) {
    __shared__ uint2 sstate[kRegDevices * kWaveR];   // pair of device d of lane l at [d * 64 + l]
    __shared__ uint16_t sdig[kMaxPatterns * 5];      // digit -> (pattern id << 3) | op
    __shared__ uint32_t sshape[kMaxPatterns];        // pattern id -> lg | ls << 4 | master << 8 | participating devices << 16
    int a = 0, b = n_segs - 1;                       // last segment whose first_block <= blockIdx.x
    while (a < b) {
        const int mid = (a + b + 1) >> 1;
        if (segs[mid].first_block <= blockIdx.x) a = mid; else b = mid - 1;
    }
    const DevSegment seg = segs[a];
    const DevQuery& q = queries[seg.query];
    const int lane = threadIdx.x;
    for (int i = lane; i < q.n_patterns; i += kWaveR)
        sshape[i] = (uint32_t)q.pat[i].reg_shape | ((uint32_t)(q.pat[i].n_groups * q.pat[i].g) << 16);
    for (int i = lane; i < q.alphabet; i += kWaveR) sdig[i] = q.instr_of_digit[i];
    __syncthreads();
    uint2* my = sstate + lane;
    const int len = seg.len;
    const int R = q.R;
    const uint32_t I = (uint32_t)q.alphabet;
    const uint32_t magic = q.magic_alphabet;
    const uint32_t all_rows = q.k >= 32 ? 0xffffffffu : ((1u << q.k) - 1u);
    const uint32_t all_cols = R >= 32 ? 0xffffffffu : ((1u << R) - 1u);
    const unsigned long long off0 = (unsigned long long)(blockIdx.x - seg.first_block) * (unsigned long long)(seg.iters * kWaveR);
    // digits of the block's first candidate (most significant first)
    uint32_t d0[P2_MAX_LEN];
    {
        unsigned long long rem = off0;
#pragma unroll
        for (int t = P2_MAX_LEN - 1; t >= 0; --t) {
            if (t < len) { const unsigned long long nx = rem / I; d0[t] = (uint32_t)(rem - nx * I); rem = nx; }
            else d0[t] = 0;
        }
    }
    unsigned long long steps = 0, members = 0;
    for (int it = 0; it < seg.iters; ++it) {
        const uint32_t add = (uint32_t)(it * kWaveR + lane);
        const unsigned long long off = off0 + add;
        bool alive = off < seg.count;
        if (!__any(alive)) break;
        // this lane's instructions: digits of d0 + add carried through base I, 9 bits per instruction
        unsigned long long prog = 0;
        uint32_t carry = add;
#pragma unroll
        for (int t = P2_MAX_LEN - 1; t >= 0; --t) {
            if (t < len) {
                const uint32_t v = d0[t] + carry;
                carry = __umulhi(v, magic);
                prog = (prog << 9) | sdig[v - carry * I];
            }
        }
        bool give_up = false, goal = false;
        uint32_t ran = 0, visited = 0;
        for (int t = 0; t < len; ++t) {
            if (!__any(alive)) break;
            if (alive) {
                const uint32_t ins = (uint32_t)(prog >> (9 * t)) & 511u;
                const bool last = t == len - 1;
                ++ran;
                visited += sshape[ins >> 3] >> 16;
                int rc = RSTEP_INVALID;
                bool done = false;
                if (last) {
                    if (t == 0) {
                        // Sec. 3.5: device i holds column i in every row
#pragma unroll
                        for (int d = 0; d < kRegDevices; ++d) my[d * kWaveR] = make_uint2(all_rows, 1u << d);
                    }
                    rc = judge_last<kWaveR>(my, sshape[ins >> 3], (int)(ins & 7u), R, all_rows, all_cols);
                    done = true;
                }
                while (__any(!done)) {
                    if (!done) {
                        const uint32_t ins0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)ins);
                        if (ins == ins0) {
                            const int op0 = (int)(ins0 & 7u);
                            const uint32_t shape = (uint32_t)__builtin_amdgcn_readfirstlane((int)sshape[ins0 >> 3]);
                            const int lg = (int)(shape & 15u), ls = (int)((shape >> 4) & 15u);
                            // devices taking part: below R and, in a Master form, those whose bits below the stride are clear
                            uint32_t part = all_cols;
                            if ((shape >> 8) & 1u) {
                                uint32_t every = 1u;                          // bit d set iff d % 2^ls == 0
                                for (int j = ls; j < 5; ++j) every |= every << (1u << j);
                                part &= every;
                            }
                            if (t == 0) {
                                rc = first_step(my, op0, lg, ls, part, q.k, all_rows) ? RSTEP_OK : RSTEP_INVALID;
                            } else {
                                RegState st;
#pragma unroll
                                for (int d = 0; d < kRegDevices; ++d) {
                                    const uint2 v = my[d * kWaveR];
                                    st.r[d] = v.x; st.m[d] = v.y;
                                }
                                rc = part == 0xffffffffu ? reg_step<false>(st, op0, lg, ls, part) : reg_step<true>(st, op0, lg, ls, part);
                                if (rc == RSTEP_OK) {
#pragma unroll
                                    for (int d = 0; d < kRegDevices; ++d) my[d * kWaveR] = make_uint2(st.r[d], st.m[d]);
                                }
                            }
                            done = true;
                        }
                    }
                }
                alive = rc == RSTEP_OK && !last;
                give_up = rc == RSTEP_GIVE_UP;
                goal = rc == RSTEP_GOAL;
            }
        }
        if (goal) {
            const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
            if (pos < q.valid_cap) q.valid_idx[pos] = seg.first_index + off;
        }
        if (give_up) {
            // the literal engine evaluates (and counts) this candidate from its first instruction
            const uint32_t pos = atomicAdd(&q.counters->n_rerun, 1u);
            if (pos < q.rerun_cap) q.rerun_idx[pos] = seg.first_index + off;
        } else {
            steps += ran;
            members += visited;
        }
    }
    for (int o = 32; o > 0; o >>= 1) { steps += __shfl_xor(steps, o, kWaveR); members += __shfl_xor(members, o, kWaveR); }
    if (lane == 0 && steps) {
        atomicAdd(&q.counters->steps[blockIdx.x % kCounterStripes], steps);
        atomicAdd(&q.counters->members[blockIdx.x % kCounterStripes], members);
    }
}

inline int exact_log2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return (1 << l) == v ? l : -1;
}

}  // namespace

int reg_shape_of(int g, int s, int master, int max_bits) {
    const int lg = exact_log2(g), ls = exact_log2(s);
    if (lg < 1 || ls < 0 || lg + ls > max_bits) return -1;
    return lg | (ls << 4) | ((master ? 1 : 0) << 8);
}

hipError_t launch_eval_regs(const DevQuery* queries, const DevSegment* segs, int n_segs, unsigned total_blocks,
                            hipStream_t stream) {
    if (n_segs == 0 || total_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_eval_regs, dim3(total_blocks), dim3(kWaveR), 0, stream, queries, segs, n_segs);
    return hipGetLastError();
}

}  // namespace p2
