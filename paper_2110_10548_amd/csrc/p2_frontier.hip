// Frontier evaluation: the enumeration by program size of Sec. 3.5 with its pruning -- a prefix
// whose step violates a rule is never extended -- for candidate spaces too large to walk index by
// index (10^11 programs per query at four hierarchy levels and size limit 6).
//
// A frontier holds the valid, non-goal prefixes of one length.  Prefixes whose state has the
// compact form (one chunk set + one mask per device, see p2_compact.hip) keep that state in HBM,
// R * (KW + MW) words each; the others ("literal" prefixes, reached through an AllGather of
// members with different masks) keep only their instructions and are re-run by the literal engine.
// One level is two kernels:
//   classify    : block = one prefix, its state copied to LDS; thread = one instruction, which
//                 decides read-only whether the step is valid and whether its result is the goal.
//                 Survivors (valid steps) are appended to a list and counted by kind.
//   materialize : one wavefront per survivor: a goal becomes a valid program (its candidate index
//                 is appended), anything else a prefix of the next frontier; for compact results
//                 the new state is built from the parent's and written to HBM.
// The host sizes the next level's buffers from the counts between the two, so nothing overflows.
#include "p2_compact_dev.h"

namespace p2 {

namespace {

constexpr int kClassifyThreads = 128;

enum : int { CODE_INVALID = 0, CODE_PREFIX = 1, CODE_GOAL = 2, CODE_PREFIX_LITERAL = 3 };

// Is the step valid, and what does it lead to?  Reads the state only.  n_goal: devices of the
// state that are already at the goal.
template <int KW, int MW>
__device__ inline int classify_step(const uint32_t* st, const PatLds P, int op, int R, const Words<KW>& all_rows,
                                    const Words<MW>& all_cols, int n_goal) {
    constexpr int WPD = KW + MW;
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    uint32_t badx = 0;
    bool changed = false, give_up = false, all_goal = true;
    int goal_part = 0;                      // participants that are at the goal before the step
    GroupWalk wk;
    wk.start();
    Slot<KW, MW> first, acc;
    uint32_t eqx = 0, dmx = 0, drx = 0, smx = 0, subx = 0;
    bool anyzero = false;
    const int n_part = P.n_groups * P.g;
    for (int j = 0; j < n_part; ++j) {
        const Slot<KW, MW> cur = load_slot<KW, MW>(st, WPD, wk.dev);
        goal_part += (fold_xor(cur.r, all_rows) | fold_xor(cur.m, all_cols)) == 0 ? 1 : 0;
        if (wk.p == 0) {
            first = cur; acc = cur;
            eqx = 0; dmx = 0; drx = 0; smx = 0; subx = 0;
            anyzero = fold_or(cur.r) == 0;
        } else {
            eqx |= fold_xor(cur.r, first.r);
            dmx |= fold_and(cur.m, acc.m);
            drx |= fold_and(cur.r, acc.r);
            smx |= fold_xor(cur.m, first.m);
            subx |= fold_andn(cur.r, first.r) | fold_andn(cur.m, first.m);
            anyzero |= fold_or(cur.r) == 0;
#pragma unroll
            for (int i = 0; i < KW; ++i) acc.r.w[i] |= cur.r.w[i];
#pragma unroll
            for (int i = 0; i < MW; ++i) acc.m.w[i] |= cur.m.w[i];
        }
        if (wk.next(P)) {
            if (red) {
                badx |= eqx | dmx;
                changed |= fold_or(first.r) != 0;
                if (op == OP_RS) {
                    const int rows = popcount(first.r);
                    badx |= (uint32_t)(div_small(rows, P.g) * P.g != rows);
                }
                // AllReduce leaves (same chunks, union) on every member; ReduceScatter and Reduce leave
                // members with fewer chunks than the goal has
                all_goal &= op == OP_AR && (fold_xor(first.r, all_rows) | fold_xor(acc.m, all_cols)) == 0;
            } else if (op == OP_AG) {
                badx |= drx | (uint32_t)anyzero;
                give_up |= smx != 0;
                changed = true;
                all_goal &= (fold_xor(acc.r, all_rows) | fold_xor(first.m, all_cols)) == 0;
            } else {
                badx |= subx | (uint32_t)((eqx | smx) == 0);
                changed = true;
                all_goal &= (fold_xor(first.r, all_rows) | fold_xor(first.m, all_cols)) == 0;
            }
            wk.next_group(P);
        }
    }
    if (badx != 0 || !changed) return CODE_INVALID;
    if (give_up) return CODE_PREFIX_LITERAL;        // rows with different column sets: never the goal
    const bool rest_done = (n_goal - goal_part) == (R - n_part);     // devices left untouched
    return (all_goal && rest_done) ? CODE_GOAL : CODE_PREFIX;
}

template <int KW, int MW>
__global__ __launch_bounds__(kClassifyThreads) void k_front_classify(const DevQuery* __restrict__ qp,
                                                                     const FrontEntry* __restrict__ entries,
                                                                     const uint32_t* __restrict__ states, uint32_t n_entries,
                                                                     FrontSurvivor* __restrict__ surv, uint32_t surv_cap,
                                                                     FrontCounters* __restrict__ ctr) {
    extern __shared__ uint32_t lds[];
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ uint16_t sdig[kMaxPatterns * 5];
    __shared__ int s_goal;
    const DevQuery& q = *qp;
    constexpr int WPD = KW + MW;
    const int R = q.R, I = q.alphabet;
    const int words = R * WPD;
    for (int i = threadIdx.x; i < q.n_patterns; i += kClassifyThreads) {
        PatLds p;
        p.g = q.pat[i].g; p.s = q.pat[i].s; p.master = q.pat[i].master; p.n_groups = q.pat[i].n_groups;
        spat[i] = p;
    }
    for (int i = threadIdx.x; i < I; i += kClassifyThreads) sdig[i] = q.instr_of_digit[i];
    const Words<KW> all_rows = full_mask<KW>(q.k);
    const Words<MW> all_cols = full_mask<MW>(R);
    unsigned long long steps = 0, members = 0;
    for (uint32_t e = blockIdx.x; e < n_entries; e += gridDim.x) {
        __syncthreads();
        const uint32_t* src = states + (size_t)e * words;
        for (int i = threadIdx.x; i < words; i += kClassifyThreads) lds[i] = src[i];
        if (threadIdx.x == 0) s_goal = 0;
        __syncthreads();
        int mine = 0;
        for (int d = threadIdx.x; d < R; d += kClassifyThreads) {
            const Slot<KW, MW> sl = load_slot<KW, MW>(lds, WPD, d);
            mine += (fold_xor(sl.r, all_rows) | fold_xor(sl.m, all_cols)) == 0 ? 1 : 0;
        }
        if (mine) atomicAdd(&s_goal, mine);
        __syncthreads();
        const int n_goal = s_goal;
        for (int a = threadIdx.x; a < I; a += kClassifyThreads) {
            const uint32_t ins = sdig[a];
            const PatLds P = spat[ins >> 3];
            const int code = classify_step<KW, MW>(lds, P, (int)(ins & 7u), R, all_rows, all_cols, n_goal);
            ++steps;
            members += (unsigned long long)(P.n_groups * P.g);
            if (code != CODE_INVALID) {
                const uint32_t pos = atomicAdd(&ctr->n_surv, 1u);
                if (pos < surv_cap) { FrontSurvivor sv; sv.entry = e; sv.digit = (uint16_t)a; sv.code = (uint16_t)code; surv[pos] = sv; }
                atomicAdd(code == CODE_GOAL ? &ctr->n_goal : code == CODE_PREFIX ? &ctr->n_prefix : &ctr->n_prefix_literal, 1u);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) { steps += __shfl_xor(steps, o, 64); members += __shfl_xor(members, o, 64); }
    if ((threadIdx.x & 63) == 0 && steps) { atomicAdd(&ctr->steps, steps); atomicAdd(&ctr->members, members); }
}

__device__ inline unsigned long long rank_of(const DevQuery& q, unsigned long long digits, int len) {
    unsigned long long v = 0;
    for (int t = 0; t < len; ++t) v = v * (unsigned long long)q.alphabet + ((digits >> (9 * t)) & 511ull);
    return q.base[len] + v;
}

// One wavefront per survivor of the compact frontier.
template <int KW, int MW>
__global__ __launch_bounds__(64) void k_front_materialize(const DevQuery* __restrict__ qp, uint32_t query,
                                                          const FrontEntry* __restrict__ entries,
                                                          const uint32_t* __restrict__ states,
                                                          const FrontSurvivor* __restrict__ surv, uint32_t n_surv,
                                                          int parent_len, int keep_prefixes,
                                                          FrontEntry* __restrict__ next_entries, uint32_t* __restrict__ next_states,
                                                          FrontEntry* __restrict__ next_literal,
                                                          unsigned long long* __restrict__ valid_out,
                                                          FrontCounters* __restrict__ ctr) {
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ uint32_t s_slot;
    const DevQuery& q = *qp;
    constexpr int WPD = KW + MW;
    const int lane = threadIdx.x;
    const int R = q.R;
    const int words = R * WPD;
    for (int i = lane; i < q.n_patterns; i += 64) {
        PatLds p;
        p.g = q.pat[i].g; p.s = q.pat[i].s; p.master = q.pat[i].master; p.n_groups = q.pat[i].n_groups;
        spat[i] = p;
    }
    __syncthreads();
    for (uint32_t i = blockIdx.x; i < n_surv; i += gridDim.x) {
        const FrontSurvivor sv = surv[i];
        const FrontEntry pe = entries[sv.entry];
        const unsigned long long digits = pe.digits | ((unsigned long long)sv.digit << (9 * parent_len));
        if (sv.code == CODE_GOAL) {
            if (lane == 0) valid_out[atomicAdd(&ctr->valid_written, 1u)] = rank_of(q, digits, parent_len + 1);
            continue;
        }
        if (!keep_prefixes) continue;                 // the size limit is reached: nothing extends this prefix
        FrontEntry ce;
        ce.query = query; ce.len = (uint32_t)(parent_len + 1); ce.digits = digits;
        if (sv.code == CODE_PREFIX_LITERAL) {
            if (lane == 0) next_literal[atomicAdd(&ctr->next_literal, 1u)] = ce;
            continue;
        }
        __syncthreads();
        if (lane == 0) { s_slot = atomicAdd(&ctr->next_compact, 1u); next_entries[s_slot] = ce; }
        __syncthreads();
        const uint32_t* parent = states + (size_t)sv.entry * words;
        uint32_t* child = next_states + (size_t)s_slot * words;
        for (int w = lane; w < words; w += 64) child[w] = parent[w];
        __syncthreads();
        // apply the instruction: lanes over groups, members in order; reads the parent, writes the child
        const uint32_t ins = q.instr_of_digit[sv.digit];
        const PatLds P = spat[ins >> 3];
        const int op = (int)(ins & 7u);
        const int gs = P.g * P.s;
        for (int G = lane; G < P.n_groups; G += 64) {
            const int base = P.master ? G * gs : (G / P.s) * gs + (G % P.s);
            const Slot<KW, MW> first = load_slot<KW, MW>(parent, WPD, base);
            Slot<KW, MW> acc = first;
            for (int p = 1; p < P.g; ++p) {
                const Slot<KW, MW> cur = load_slot<KW, MW>(parent, WPD, base + p * P.s);
#pragma unroll
                for (int w = 0; w < KW; ++w) acc.r.w[w] |= cur.r.w[w];
#pragma unroll
                for (int w = 0; w < MW; ++w) acc.m.w[w] |= cur.m.w[w];
            }
            Words<KW> prev;
#pragma unroll
            for (int w = 0; w < KW; ++w) prev.w[w] = 0;
            const int per = op == OP_RS ? div_small(popcount(first.r), P.g) : 0;
            for (int p = 0; p < P.g; ++p) {
                Words<KW> nr = first.r;
                Words<MW> nm = acc.m;
                if (op == OP_RS) {
                    const Words<KW> upto = lowest_n(first.r, (p + 1) * per);
#pragma unroll
                    for (int w = 0; w < KW; ++w) { nr.w[w] = upto.w[w] & ~prev.w[w]; prev.w[w] = upto.w[w]; }
                } else if (op == OP_RD) {
                    if (p != 0) {
#pragma unroll
                        for (int w = 0; w < KW; ++w) nr.w[w] = 0;
#pragma unroll
                        for (int w = 0; w < MW; ++w) nm.w[w] = 0;
                    }
                } else if (op == OP_AG) {
                    nr = acc.r; nm = first.m;
                } else if (op == OP_BC) {
                    nm = first.m;
                }
                store_slot<KW, MW>(child, WPD, base + p * P.s, nr, nm);
            }
        }
        if (lane == 0) { atomicAdd(&ctr->steps, 1ull); atomicAdd(&ctr->members, (unsigned long long)(P.n_groups * P.g)); }
    }
}

// Survivors of the literal frontier carry no state: a goal becomes a valid program, the rest
// prefixes of the next literal frontier.
__global__ __launch_bounds__(256) void k_front_emit(const DevQuery* __restrict__ qp, uint32_t query,
                                                    const FrontEntry* __restrict__ entries,
                                                    const FrontSurvivor* __restrict__ surv, uint32_t n_surv, int parent_len,
                                                    int keep_prefixes, FrontEntry* __restrict__ next_literal,
                                                    unsigned long long* __restrict__ valid_out, FrontCounters* __restrict__ ctr) {
    const DevQuery& q = *qp;
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n_surv) return;
    const FrontSurvivor sv = surv[i];
    const unsigned long long digits = entries[sv.entry].digits | ((unsigned long long)sv.digit << (9 * parent_len));
    if (sv.code == CODE_GOAL) {
        valid_out[atomicAdd(&ctr->valid_written, 1u)] = rank_of(q, digits, parent_len + 1);
    } else if (keep_prefixes) {
        FrontEntry ce;
        ce.query = query; ce.len = (uint32_t)(parent_len + 1); ce.digits = digits;
        next_literal[atomicAdd(&ctr->next_literal, 1u)] = ce;
    }
}

template <int KW, int MW>
__global__ __launch_bounds__(64) void k_front_init(const DevQuery* __restrict__ qp, uint32_t query, FrontEntry* entries,
                                                   uint32_t* states) {
    // Sec. 3.5: the empty program; device i holds column i in every row
    const DevQuery& q = *qp;
    constexpr int WPD = KW + MW;
    const Words<KW> all_rows = full_mask<KW>(q.k);
    for (int d = threadIdx.x; d < q.R; d += 64) {
        Words<MW> m;
#pragma unroll
        for (int i = 0; i < MW; ++i) m.w[i] = (i == (d >> 5)) ? (1u << (d & 31)) : 0u;
        store_slot<KW, MW>(states, WPD, d, all_rows, m);
    }
    if (threadIdx.x == 0) { FrontEntry e; e.query = query; e.len = 0; e.digits = 0ull; entries[0] = e; }
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
    FrontSurvivor* surv; uint32_t surv_cap; uint32_t n_surv;
    int parent_len, keep_prefixes;
    FrontEntry* next_entries; uint32_t* next_states; FrontEntry* next_literal;
    unsigned long long* valid_out; FrontCounters* ctr;
    int R;
};

template <int KW, int MW>
hipError_t front_go(int what, const FrontArgs& A, hipStream_t stream) {
    if (what == 0) {
        hipLaunchKernelGGL((k_front_init<KW, MW>), dim3(1), dim3(64), 0, stream, A.q, A.query, const_cast<FrontEntry*>(A.entries),
                           const_cast<uint32_t*>(A.states));
    } else if (what == 1) {
        const size_t lds = (size_t)A.R * (KW + MW) * 4;
        hipError_t e = allow_lds_f(k_front_classify<KW, MW>, lds);
        if (e != hipSuccess) return e;
        const unsigned blocks = A.n < 65536u ? A.n : 65536u;
        hipLaunchKernelGGL((k_front_classify<KW, MW>), dim3(blocks), dim3(kClassifyThreads), lds, stream, A.q, A.entries, A.states,
                           A.n, A.surv, A.surv_cap, A.ctr);
    } else {
        const unsigned blocks = A.n_surv < 65536u ? A.n_surv : 65536u;
        hipLaunchKernelGGL((k_front_materialize<KW, MW>), dim3(blocks), dim3(64), 0, stream, A.q, A.query, A.entries, A.states,
                           A.surv, A.n_surv, A.parent_len, A.keep_prefixes, A.next_entries, A.next_states, A.next_literal,
                           A.valid_out, A.ctr);
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

size_t frontier_state_words(int R, int k) { return (size_t)R * (size_t)(round_words_f(k) + round_words_f(R)); }

hipError_t launch_front_init(const DevQuery* q, uint32_t query, int R, int k, FrontEntry* entries, uint32_t* states,
                             hipStream_t stream) {
    FrontArgs A{};
    A.q = q; A.query = query; A.entries = entries; A.states = states; A.R = R;
    return front_dispatch(R, k, 0, A, stream);
}

hipError_t launch_front_classify(const DevQuery* q, int R, int k, const FrontEntry* entries, const uint32_t* states,
                                 uint32_t n, FrontSurvivor* surv, uint32_t surv_cap, FrontCounters* ctr, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    FrontArgs A{};
    A.q = q; A.entries = entries; A.states = states; A.n = n; A.surv = surv; A.surv_cap = surv_cap; A.ctr = ctr; A.R = R;
    return front_dispatch(R, k, 1, A, stream);
}

hipError_t launch_front_materialize(const DevQuery* q, uint32_t query, int R, int k, const FrontEntry* entries,
                                    const uint32_t* states, const FrontSurvivor* surv, uint32_t n_surv, int parent_len,
                                    int keep_prefixes, FrontEntry* next_entries, uint32_t* next_states,
                                    FrontEntry* next_literal, unsigned long long* valid_out, FrontCounters* ctr,
                                    hipStream_t stream) {
    if (n_surv == 0) return hipSuccess;
    FrontArgs A{};
    A.q = q; A.query = query; A.entries = entries; A.states = states; A.surv = const_cast<FrontSurvivor*>(surv); A.n_surv = n_surv;
    A.parent_len = parent_len; A.keep_prefixes = keep_prefixes; A.next_entries = next_entries; A.next_states = next_states;
    A.next_literal = next_literal; A.valid_out = valid_out; A.ctr = ctr; A.R = R;
    return front_dispatch(R, k, 2, A, stream);
}

hipError_t launch_front_emit(const DevQuery* q, uint32_t query, const FrontEntry* entries, const FrontSurvivor* surv,
                             uint32_t n_surv, int parent_len, int keep_prefixes, FrontEntry* next_literal,
                             unsigned long long* valid_out, FrontCounters* ctr, hipStream_t stream) {
    if (n_surv == 0) return hipSuccess;
    hipLaunchKernelGGL(k_front_emit, dim3((n_surv + 255u) / 256u), dim3(256), 0, stream, q, query, entries, surv, n_surv, parent_len,
                       keep_prefixes, next_literal, valid_out, ctr);
    return hipGetLastError();
}

}  // namespace p2
