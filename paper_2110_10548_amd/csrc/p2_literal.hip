// Literal engine: the device-state semantics of Sec. 3.2 on the literal state of one reduction
// group -- R devices x k chunk rows, each row a mask of R contribution bits -- kept in LDS by
// one wavefront per candidate.  A step works on (group, row) items: an item reads the row of
// every member of its group, checks the rule's premises, and writes the members' new rows.
// The same code, with kCost set, recomputes a valid program and adds up its ring alpha-beta
// step times (hierarchical cost model, see p2.h).
#include "p2_device.h"

#include <cstdlib>

namespace p2 {

namespace {

constexpr int kWave = 64;

// v / d for 0 <= v < 2^22 and 1 <= d <= 2^15: a float quotient (off by one at most), then one correction.
__device__ __forceinline__ int div_fast(int v, int d) {
    int q = (int)__fdividef((float)v + 0.5f, (float)d);
    const int r = v - q * d;
    q += r >= d ? 1 : r < 0 ? -1 : 0;
    return q;
}
// First device of group G of a pattern with stride s and gs = g * s.
__device__ __forceinline__ int group_base(int master, int G, int s, int gs) {
    if (master) return G * gs;
    const int hi = div_fast(G, s);
    return hi * gs + (G - hi * s);
}
constexpr size_t kLdsLimit = 160 * 1024 - 512;

struct LitLayout {
    int s_words, t_words, ngmax, kw;
    __host__ __device__ LitLayout(int R, int k, int MW) {
        ngmax = R / 2 > 0 ? R / 2 : 1;
        kw = (k + 31) / 32;
        s_words = R * k * MW;
        t_words = ngmax * k * MW;
    }
    __host__ __device__ int total_words() const { return s_words + t_words + ngmax * (2 + kw) + 512 + 4; }
};

struct LitLds {
    uint32_t* S;       // [R][k][MW]   state
    uint32_t* T;       // [ng][k][MW]  combined rows of each group
    uint32_t* gcount;  // [ng]         non-empty rows of the group's result / root
    uint32_t* gflag;   // [ng]         Broadcast: some member differs from the root
    uint32_t* gbits;   // [ng][kw]     which rows of the group's result are non-empty
    uint32_t* devne;   // [R] (<=512)  AllGather: device holds something
    uint32_t* flags;   // [4]          0: premise failed, 1: state changed
};

__device__ inline LitLds carve(uint32_t* lds, int R, int k, int MW) {
    LitLayout lay(R, k, MW);
    LitLds L;
    L.S = lds;
    L.T = L.S + lay.s_words;
    L.gcount = L.T + lay.t_words;
    L.gflag = L.gcount + lay.ngmax;
    L.gbits = L.gflag + lay.ngmax;
    L.devne = L.gbits + lay.ngmax * lay.kw;
    L.flags = L.devne + 512;
    return L;
}

__device__ inline int unrank(const DevQuery& q, unsigned long long idx, uint16_t* digit) {
    int len = 1;
    while (len < q.max_len && idx >= q.base[len + 1]) ++len;
    unsigned long long rem = idx - q.base[len];
    const unsigned long long I = (unsigned long long)q.alphabet;
    for (int t = len - 1; t >= 0; --t) {
        unsigned long long nx = rem / I;
        digit[t] = (uint16_t)(rem - nx * I);
        rem = nx;
    }
    return len;
}

__device__ inline double wave_max(double v) {
    for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, kWave));
    return v;
}

// One instruction on the literal state.  All nt threads of the block call it with identical arguments
// (lane = thread number; nt = 64, one wavefront, unless stated; kCost needs nt = 64).
// Returns false if a premise fails or nothing changes.  With kCost, *cost_lane (lane m = message
// size m) gets the step time added.
template <int MW, bool kCost>
__device__ bool lit_step(const DevQuery& q, const DevPattern& P, int op, const LitLds& L, int lane, double* cost_lane,
                         const int nt = kWave) {
    const int k = q.k, g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    const int kw = (k + 31) / 32;
    for (int i = lane; i < ng; i += nt) { L.gcount[i] = 0; L.gflag[i] = 0; }
    for (int i = lane; i < ng * kw; i += nt) L.gbits[i] = 0;
    if (op == OP_AG)
        for (int i = lane; i < q.R; i += nt) L.devne[i] = 0;
    if (lane == 0) { L.flags[0] = 0; L.flags[1] = 0; }
    __syncthreads();

    const int items = ng * k;
    bool bad = false;
    for (int it = lane; it < items; it += nt) {
        const int G = div_fast(it, k), r = it - G * k;
        const int base = group_base(P.master, G, s, gs);
        uint32_t acc[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) acc[w] = 0;
        if (op == OP_AR || op == OP_RS || op == OP_RD) {
            // premises: same non-empty rows on every member; columns of a row pairwise disjoint
            bool ne0 = false;
            for (int p = 0; p < g; ++p) {
                const uint32_t* x = L.S + ((base + p * s) * k + r) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    uint32_t v = x[w];
                    any |= v;
                    bad |= (acc[w] & v) != 0;
                    acc[w] |= v;
                }
                if (p == 0) ne0 = any != 0;
                else bad |= (any != 0) != ne0;
            }
            if (ne0) {
                atomicAdd(&L.gcount[G], 1u);
                atomicOr(&L.gbits[G * kw + (r >> 5)], 1u << (r & 31));
            }
        } else if (op == OP_AG) {
            // premises: every member holds something; a row is held by at most one member
            int holders = 0;
            for (int p = 0; p < g; ++p) {
                const int dev = base + p * s;
                const uint32_t* x = L.S + (dev * k + r) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) { uint32_t v = x[w]; any |= v; acc[w] |= v; }
                if (any) { ++holders; L.devne[dev] = 1; }
            }
            bad |= holders > 1;
            if (holders) atomicAdd(&L.gcount[G], 1u);
        } else {
            // Broadcast: the root's row contains every member's row; some member differs somewhere
            const uint32_t* root = L.S + (base * k + r) * MW;
            uint32_t any = 0;
#pragma unroll
            for (int w = 0; w < MW; ++w) { acc[w] = root[w]; any |= acc[w]; }
            bool differs = false;
            for (int p = 1; p < g; ++p) {
                const uint32_t* x = L.S + ((base + p * s) * k + r) * MW;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    uint32_t v = x[w];
                    bad |= (v & ~acc[w]) != 0;
                    differs |= v != acc[w];
                }
            }
            if (differs) L.gflag[G] = 1;
            if (any) atomicAdd(&L.gcount[G], 1u);
        }
        uint32_t* t = L.T + (G * k + r) * MW;
#pragma unroll
        for (int w = 0; w < MW; ++w) t[w] = acc[w];
    }
    if (bad) L.flags[0] = 1;
    __syncthreads();

    // per-group premises
    for (int G = lane; G < ng; G += nt) {
        const uint32_t cnt = L.gcount[G];
        if (op == OP_AR || op == OP_RS || op == OP_RD) {
            if (op == OP_RS && cnt % (uint32_t)g != 0) L.flags[0] = 1;   // scatter: chunks must divide evenly
            if (cnt) L.flags[1] = 1;                                    // a group of empty devices is a no-op
        } else if (op == OP_AG) {
            const int base = group_base(P.master, G, s, gs);
            for (int p = 0; p < g; ++p)
                if (!L.devne[base + p * s]) L.flags[0] = 1;
            L.flags[1] = 1;
        } else {
            if (!L.gflag[G]) L.flags[0] = 1;                            // no information increase
            L.flags[1] = 1;
        }
    }
    __syncthreads();
    if (L.flags[0] || !L.flags[1]) return false;

    if (kCost) {
        // bandwidth term: the most loaded uplink; gcount holds the rows that set a group's bytes
        double best = 0.0;
        const DevRows& rw = *q.rows;
        const int pid = (int)(&P - q.pat);
        for (int row = rw.pat_begin[pid] + lane; row < rw.pat_begin[pid + 1]; row += kWave) {
            long long dot = 0;
            for (int e = rw.row_ptr[row]; e < rw.row_ptr[row + 1]; ++e) {
                const uint32_t ent = rw.entries[e];
                dot += (long long)entry_cnt(ent) * (long long)L.gcount[entry_group(ent)];
            }
            best = fmax(best, (double)dot * q.inv_bw[rw.row_level[row]]);
        }
        best = wave_max(best);
        double ring_steps, mult;
        step_factors(op, g, q.algo, ring_steps, mult);
        if (lane < q.n_msg) *cost_lane += ring_steps * q.alpha[P.span_level] + q.msg_bytes[lane] * (mult / (double)k) * best;
    }

    // write the members' new rows (block p of a ReduceScatter goes to the member of rank p)
    const int32_t* rank = P.rank_off ? q.rank_tbl + (P.rank_off - 1) : nullptr;
    for (int it = lane; it < items; it += nt) {
        const int G = div_fast(it, k), r = it - G * k;
        const int base = group_base(P.master, G, s, gs);
        uint32_t t[MW];
        uint32_t any = 0;
#pragma unroll
        for (int w = 0; w < MW; ++w) { t[w] = L.T[(G * k + r) * MW + w]; any |= t[w]; }
        int owner = -2;                                   // -2: everyone, else the only member keeping the row
        if (op == OP_RD) owner = 0;
        else if (op == OP_RS) {
            owner = -1;
            if (any) {
                // position of row r among the group's non-empty rows, ascending
                int before = 0;
                for (int w = 0; w < (r >> 5); ++w) before += __popc(L.gbits[G * kw + w]);
                before += __popc(L.gbits[G * kw + (r >> 5)] & ((1u << (r & 31)) - 1u));
                owner = before / (int)(L.gcount[G] / (uint32_t)g);
            }
        }
        for (int p = (op == OP_BC ? 1 : 0); p < g; ++p) {
            uint32_t* x = L.S + ((base + p * s) * k + r) * MW;
            const bool keep = owner == -2 || owner == (rank ? rank[p] : p);
#pragma unroll
            for (int w = 0; w < MW; ++w) x[w] = keep ? t[w] : 0u;
        }
    }
    __syncthreads();
    return true;
}

template <int MW>
__device__ inline void lit_init(const DevQuery& q, const LitLds& L, int lane, const int nt = kWave) {
    // Sec. 3.5: device i holds column i in every row
    const int cells = q.R * q.k;
    for (int c = lane; c < cells; c += nt) {
        const int d = c / q.k;
#pragma unroll
        for (int w = 0; w < MW; ++w) L.S[c * MW + w] = (w == (d >> 5)) ? (1u << (d & 31)) : 0u;
    }
    __syncthreads();
}

// The state after a program's first instruction, written directly (reduction groups of at most 64
// devices whose patterns have power-of-two group sizes and strides: the queries of the shared-prefix
// engine).  On the init state the AllReduce-like rules always apply (ReduceScatter if the group size divides
// k): every member ends with the columns of its group, the devices that agree with it outside bits
// [ls, ls + lg) of the device number, on all rows (AllReduce), on its block of rows (ReduceScatter), or on
// all rows of the root only (Reduce); AllGather and Broadcast never apply.  Returns false where the
// instruction is invalid (the state is then not written).
template <int MW>
__device__ inline bool lit_init_first(const DevQuery& q, const DevPattern& P, int op, const LitLds& L, int lane) {
    static_assert(MW <= 2, "groups of at most 64 devices");
    if (op == OP_AG || op == OP_BC) return false;
    if (op == OP_RS && q.k % P.g != 0) return false;
    const int per = q.k / P.g;
    const uint32_t gmask = (uint32_t)(P.g - 1) * (uint32_t)P.s;          // g and s are powers of two
    const int cells = q.R * q.k;
    for (int c = lane; c < cells; c += kWave) {
        const int d = c / q.k, r = c - d * q.k;
        const bool in = !P.master || (d % P.s) == 0;
        unsigned long long cols = 1ull << d;
        if (in) {
            cols = 1ull << ((uint32_t)d & ~gmask);
            for (uint32_t b = (uint32_t)P.s; b < (uint32_t)(P.g * P.s); b <<= 1) cols |= cols << b;
            const int p = (int)(((uint32_t)d & gmask) / (uint32_t)P.s);
            if (op == OP_RS && (r < p * per || r >= (p + 1) * per)) cols = 0ull;
            if (op == OP_RD && p != 0) cols = 0ull;
        }
        L.S[c * MW] = (uint32_t)cols;
        if (MW > 1) L.S[c * MW + (MW > 1 ? 1 : 0)] = (uint32_t)(cols >> 32);
    }
    __syncthreads();
    return true;
}

template <int MW>
__device__ inline bool lit_is_goal(const DevQuery& q, const LitLds& L, int lane) {
    // every device holds, in every row, the columns of its whole reduction group
    const int cells = q.R * q.k;
    bool ok = true;
    for (int c = lane; c < cells; c += kWave) {
        const uint32_t* goal = q.goal_mask ? q.goal_mask + (size_t)(c / q.k) * MW : nullptr;
#pragma unroll
        for (int w = 0; w < MW; ++w) {
            const int bits = q.R - 32 * w;
            const uint32_t full = goal ? goal[w] : bits >= 32 ? 0xffffffffu : bits > 0 ? ((1u << bits) - 1u) : 0u;
            ok &= L.S[c * MW + w] == full;
        }
    }
    return __all(ok);
}

// One wavefront per candidate; a block takes `per_block` consecutive candidates.
template <int MW>
__global__ __launch_bounds__(kWave) void k_eval_literal(const DevQuery* __restrict__ qp, unsigned long long start,
                                                        unsigned long long count, uint32_t per_block,
                                                        const unsigned long long* __restrict__ list,
                                                        const uint32_t* __restrict__ list_count,
                                                        uint32_t* __restrict__ gscratch, unsigned long long gwords) {
    extern __shared__ uint32_t lds[];
    const DevQuery& q = *qp;
    const int lane = threadIdx.x;
    // the state lives in LDS, or, when it does not fit, in this block's slice of a global buffer
    const LitLds L = carve(gscratch ? gscratch + (size_t)blockIdx.x * gwords : lds, q.R, q.k, MW);
    if (list_count) {
        unsigned long long n = *list_count;
        if (n < count) count = n;
    }
    unsigned long long first = (unsigned long long)blockIdx.x * per_block;
    unsigned long long steps = 0, members = 0;
    for (uint32_t i = 0; i < per_block && first + i < count; ++i) {
        const unsigned long long idx = list ? list[first + i] : start + first + i;
        uint16_t digit[P2_MAX_LEN + 1];
        const int len = unrank(q, idx, digit);
        lit_init<MW>(q, L, lane);
        bool ok = true;
        for (int t = 0; t < len && ok; ++t) {
            const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
            ++steps;
            members += (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
            ok = lit_step<MW, false>(q, q.pat[pid], op, L, lane, nullptr);
        }
        if (ok && lit_is_goal<MW>(q, L, lane) && lane == 0) {
            const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
            if (pos < q.valid_cap) q.valid_idx[pos] = idx;
        }
        __syncthreads();
    }
    if (lane == 0 && steps) {
        atomicAdd(&q.counters->steps[blockIdx.x % kCounterStripes], steps);
        atomicAdd(&q.counters->members[blockIdx.x % kCounterStripes], members);
    }
}

// Cost of valid programs: block i re-runs sorted[i] with the cost terms switched on and writes
// the program record and cost[i][0..n_msg).
template <int MW>
__global__ __launch_bounds__(kWave) void k_cost_literal(const DevQuery* __restrict__ qp,
                                                        const unsigned long long* __restrict__ sorted, uint32_t n,
                                                        p2_program* __restrict__ out_prog, double* __restrict__ out_cost,
                                                        int only_missing, uint32_t* __restrict__ gscratch,
                                                        unsigned long long gwords) {
    extern __shared__ uint32_t lds[];
    const DevQuery& q = *qp;
    const int lane = threadIdx.x;
    const LitLds L = carve(gscratch ? gscratch + (size_t)blockIdx.x * gwords : lds, q.R, q.k, MW);
    for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
        // only_missing: another engine has filled every row but those it marked with NaN
        if (only_missing) {
            const double have = out_cost[(size_t)i * q.n_msg];
            if (have == have) continue;
        }
        const unsigned long long idx = sorted[i];
        uint16_t digit[P2_MAX_LEN + 1];
        const int len = unrank(q, idx, digit);
        lit_init<MW>(q, L, lane);
        double cost = 0.0;
        bool ok = true;
        for (int t = 0; t < len && ok; ++t) {
            const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
            ok = lit_step<MW, true>(q, q.pat[pid], op, L, lane, &cost);
        }
        if (lane == 0) {
            p2_program pr;
            pr.index = idx;
            pr.len = (uint8_t)len;
            for (int t = 0; t < 7; ++t) {
                int code = 0;
                if (t < len) { const int pid = digit[t] / q.n_ops; code = pid * 5 + q.ops[digit[t] - pid * q.n_ops]; }
                pr.instr[t] = (uint8_t)code;
            }
            out_prog[i] = pr;
        }
        if (lane < q.n_msg) out_cost[(size_t)i * q.n_msg + lane] = ok ? cost : __longlong_as_double(0x7ff8000000000000ll);
        __syncthreads();
    }
}

// The two kernels above for lists spread over many queries: block b serves one entry of its segment.
template <int MW>
__global__ __launch_bounds__(kWave) void k_eval_literal_list(const DevQuery* __restrict__ queries,
                                                             const DevPostSeg* __restrict__ segs, int n_segs,
                                                             const unsigned long long* __restrict__ list) {
    extern __shared__ uint32_t lds[];
    const DevPostSeg seg = find_post_seg(segs, n_segs, blockIdx.x);
    const DevQuery& q = queries[seg.query];
    const int lane = threadIdx.x;
    const LitLds L = carve(lds, q.R, q.k, MW);
    const unsigned long long idx = list[seg.in_off + (blockIdx.x - seg.first_block)];
    uint16_t digit[P2_MAX_LEN + 1];
    const int len = unrank(q, idx, digit);
    lit_init<MW>(q, L, lane);
    unsigned long long steps = 0, members = 0;
    bool ok = true;
    for (int t = 0; t < len && ok; ++t) {
        const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
        ++steps;
        members += (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        ok = lit_step<MW, false>(q, q.pat[pid], op, L, lane, nullptr);
    }
    if (ok && lit_is_goal<MW>(q, L, lane) && lane == 0) {
        const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
        if (pos < q.valid_cap) q.valid_idx[pos] = idx;
    }
    if (lane == 0) {
        atomicAdd(&q.counters->steps[blockIdx.x % kCounterStripes], steps);
        atomicAdd(&q.counters->members[blockIdx.x % kCounterStripes], members);
    }
}

template <int MW>
__global__ __launch_bounds__(kWave) void k_cost_literal_list(const DevQuery* __restrict__ queries,
                                                             const DevPostSeg* __restrict__ segs, int n_segs,
                                                             const unsigned long long* __restrict__ sorted,
                                                             p2_program* __restrict__ out_prog, double* __restrict__ out_cost,
                                                             int only_missing) {
    extern __shared__ uint32_t lds[];
    const DevPostSeg seg = find_post_seg(segs, n_segs, blockIdx.x);
    const DevQuery& q = queries[seg.query];
    const int lane = threadIdx.x;
    const size_t i = seg.out_off + (blockIdx.x - seg.first_block);
    // only_missing: another engine has filled every row but those it marked with NaN
    if (only_missing) {
        const double have = out_cost[i * q.n_msg];
        if (have == have) return;
    }
    const LitLds L = carve(lds, q.R, q.k, MW);
    const unsigned long long idx = sorted[i];
    uint16_t digit[P2_MAX_LEN + 1];
    const int len = unrank(q, idx, digit);
    lit_init<MW>(q, L, lane);
    double cost = 0.0;
    bool ok = true;
    for (int t = 0; t < len && ok; ++t) {
        const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
        ok = lit_step<MW, true>(q, q.pat[pid], op, L, lane, &cost);
    }
    if (lane == 0) {
        p2_program pr;
        pr.index = idx;
        pr.len = (uint8_t)len;
        for (int t = 0; t < 7; ++t) {
            int code = 0;
            if (t < len) { const int pid = digit[t] / q.n_ops; code = pid * 5 + q.ops[digit[t] - pid * q.n_ops]; }
            pr.instr[t] = (uint8_t)code;
        }
        out_prog[i] = pr;
    }
    if (lane < q.n_msg) out_cost[i * q.n_msg + lane] = ok ? cost : __longlong_as_double(0x7ff8000000000000ll);
}

// ---- frontier level for prefixes only the literal engine can hold ---------------------------------
// A block rebuilds the literal state of one prefix, then classifies every instruction against it
// without writing the state.  All rules act row by row, and rows that are equal on every device
// behave alike, so the classification looks at one representative row per class of equal rows
// (with the class size where the rule counts rows).
struct FrontLit {
    uint32_t* h1;       // [k]   two hashes of a row over all devices
    uint32_t* h2;       // [k]
    uint32_t* rep;      // [k]   smallest equal row
    uint32_t* reps;     // [k]   the representatives, ascending
    uint32_t* multr;    // [k]   rows in the class of a representative
    uint32_t* devany;   // [512] device holds something
    uint32_t* devfull;  // [512] device is at the goal
};
__host__ __device__ inline int front_lit_words(int k) { return 5 * k + 1024; }
__device__ inline FrontLit carve_front(uint32_t* p, int k) {
    FrontLit X;
    X.h1 = p; X.h2 = X.h1 + k; X.rep = X.h2 + k; X.reps = X.rep + k; X.multr = X.reps + k;
    X.devany = X.multr + k; X.devfull = X.devany + 512;
    return X;
}

// One instruction against the state, read-only: 0 = invalid step, 2 = valid and the result is the
// goal, 3 = valid prefix.  C = number of row classes.  All nt threads of the block call it with the same arguments.
template <int MW>
__device__ int lit_classify(const DevQuery& q, const DevPattern& P, int op, const LitLds& L, const FrontLit& X, int C,
                            const uint32_t* full, int lane, const int nt = kWave) {
    const int k = q.k, g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    for (int i = lane; i < ng; i += nt) { L.gcount[i] = 0; L.gflag[i] = 0; }
    if (lane == 0) { L.flags[0] = 0; L.flags[1] = 0; L.flags[2] = 0; }
    __syncthreads();
    const int items = ng * C;
    bool bad = false, notfull = false;
    for (int it = lane; it < items; it += nt) {
        const int G = div_fast(it, C), c = it - G * C;
        const int r = (int)X.reps[c];
        const int base = group_base(P.master, G, s, gs);
        uint32_t acc[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) acc[w] = 0;
        if (red) {
            bool ne0 = false;
            for (int p = 0; p < g; ++p) {
                const uint32_t* x = L.S + ((base + p * s) * k + r) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    uint32_t v = x[w];
                    any |= v;
                    bad |= (acc[w] & v) != 0;
                    acc[w] |= v;
                }
                if (p == 0) ne0 = any != 0;
                else bad |= (any != 0) != ne0;
            }
            if (ne0) atomicAdd(&L.gcount[G], X.multr[r]);
        } else if (op == OP_AG) {
            int holders = 0;
            for (int p = 0; p < g; ++p) {
                const int dev = base + p * s;
                const uint32_t* x = L.S + (dev * k + r) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) { uint32_t v = x[w]; any |= v; acc[w] |= v; }
                holders += any != 0;
                if (c == 0) bad |= X.devany[dev] == 0;
            }
            bad |= holders > 1;
        } else {
            const uint32_t* root = L.S + (base * k + r) * MW;
#pragma unroll
            for (int w = 0; w < MW; ++w) acc[w] = root[w];
            bool differs = false;
            for (int p = 1; p < g; ++p) {
                const uint32_t* x = L.S + ((base + p * s) * k + r) * MW;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    uint32_t v = x[w];
                    bad |= (v & ~acc[w]) != 0;
                    differs |= v != acc[w];
                }
            }
            if (differs) L.gflag[G] = 1;
        }
        // AllReduce, AllGather and Broadcast leave acc on every member
#pragma unroll
        for (int w = 0; w < MW; ++w) notfull |= acc[w] != full[w];
    }
    if (bad) L.flags[0] = 1;
    if (notfull) L.flags[2] = 1;
    // devices the pattern does not touch must already be at the goal
    if (P.master)
        for (int d = lane; d < q.R; d += nt) {
            const bool part = d % s == 0 && d / gs < ng;
            if (!part && !X.devfull[d]) L.flags[2] = 1;
        }
    __syncthreads();
    for (int G = lane; G < ng; G += nt) {
        const uint32_t cnt = L.gcount[G];
        if (red) {
            if (op == OP_RS && cnt % (uint32_t)g != 0) L.flags[0] = 1;
            if (cnt) L.flags[1] = 1;
        } else if (op == OP_BC) {
            if (!L.gflag[G]) L.flags[0] = 1;
        }
    }
    __syncthreads();
    const bool invalid = L.flags[0] != 0 || (red && L.flags[1] == 0);
    const bool goal = (op == OP_AR || op == OP_AG || op == OP_BC) && L.flags[2] == 0;
    __syncthreads();
    return invalid ? 0 : goal ? 2 : 3;
}

// Classes of equal rows of the state in L.S, and per device whether it holds anything and whether it
// is at the goal.  Hash every row over all devices, point each row at the first row with its hash,
// and keep the pointer only if the two rows really are equal.  Returns the number of classes.  All nt
// threads of the block call it (nt a multiple of 64).
template <int MW>
__device__ inline int row_classes(const DevQuery& q, const LitLds& L, const FrontLit& X, const uint32_t* full, int lane,
                                  const int nt = kWave) {
    const int R = q.R, k = q.k;
    for (int r = lane; r < k; r += nt) {
        uint32_t a = 0x811c9dc5u, b = 0x9e3779b9u;
        for (int d = 0; d < R; ++d) {
            const uint32_t* x = L.S + (d * k + r) * MW;
#pragma unroll
            for (int w = 0; w < MW; ++w) {
                const uint32_t v = x[w];
                a = (a ^ v) * 0x01000193u;
                b = (b + v) * 0x85ebca6bu + (b >> 13);
            }
        }
        X.h1[r] = a; X.h2[r] = b;
        X.multr[r] = 0;
    }
    __syncthreads();
    for (int r = lane; r < k; r += nt) {
        const uint32_t a = X.h1[r], b = X.h2[r];
        int r0 = 0;
        while (r0 < r && (X.h1[r0] != a || X.h2[r0] != b)) ++r0;
        if (r0 != r) {
            bool same = true;
            for (int d = 0; d < R; ++d) {
                const uint32_t* x = L.S + (d * k + r) * MW;
                const uint32_t* y = L.S + (d * k + r0) * MW;
#pragma unroll
                for (int w = 0; w < MW; ++w) same &= x[w] == y[w];
            }
            if (!same) r0 = r;
        }
        X.rep[r] = (uint32_t)r0;
    }
    __syncthreads();
    // the representatives in ascending order: the block's first wavefront lists them
    int C = 0;
    if (lane < kWave) {
        for (int r0 = 0; r0 < k; r0 += kWave) {
            const int r = r0 + lane;
            const bool is = r < k && X.rep[r] == (uint32_t)r;
            const unsigned long long bal = __ballot(is);
            if (is) X.reps[C + __popcll(bal & ((1ull << lane) - 1ull))] = (uint32_t)r;
            C += __popcll(bal);
            if (r < k) atomicAdd(&X.multr[X.rep[r]], 1u);
        }
        // the hashes are no longer needed: their first words become the two flags below
        if (lane == 0) { L.flags[3] = (uint32_t)C; X.h1[0] = 0; X.h1[1] = 0; }
    }
    __syncthreads();
    C = (int)L.flags[3];
    bool hole = false, partial = false;
    for (int d = lane; d < R; d += nt) {
        bool any = false, all = true;
        for (int c = 0; c < C; ++c) {
            const uint32_t* x = L.S + (d * k + (int)X.reps[c]) * MW;
            bool ne = false, fl = true;
#pragma unroll
            for (int w = 0; w < MW; ++w) { ne |= x[w] != 0; fl &= x[w] == full[w]; }
            any |= ne; all &= fl;
            hole |= !ne; partial |= ne && !fl;
        }
        X.devany[d] = any; X.devfull[d] = all;
    }
    if (hole) X.h1[0] = 1;
    if (partial) X.h1[1] = 1;
    __syncthreads();
    return C;
}
// After row_classes (rows of a class are equal on every device, so its representative speaks for them): does
// every device hold every row; does every row that a device holds carry every column.
__device__ inline bool rows_all_held(const FrontLit& X) { return X.h1[0] == 0u; }
__device__ inline bool held_rows_complete(const FrontLit& X) { return X.h1[1] == 0u; }

// ---- groups handed over by the shared-prefix engine ------------------------------------------------
// A list entry is the index of a group's first candidate: `alphabet` consecutive candidates with the
// same first len-1 instructions, whose common state the compact form could not hold.  The literal
// state of that prefix is rebuilt once, every step checked, and all last instructions are judged
// against it (one representative per class of equal rows, as in the frontier kernel above).
// part / parts: this block judges the last instructions a = part, part + parts, ... and part 0 does the counting.
template <int MW>
__device__ inline void literal_group(const DevQuery& q, unsigned long long idx0, const LitLds& L, const FrontLit& X,
                                     const uint32_t* full, int lane, int part, int parts, unsigned long long& steps,
                                     unsigned long long& members) {
    uint16_t digit[P2_MAX_LEN + 1];
    const int len = unrank(q, idx0, digit);
    const unsigned long long I = (unsigned long long)q.alphabet;
    bool ok = true;
    unsigned long long ran = 0, visited = 0;
    int t0 = 0;
    if (len - 1 >= 1) {                              // the first instruction: its result is known without a pass
        const int pid = digit[0] / q.n_ops, op = q.ops[digit[0] - pid * q.n_ops];
        ran = 1;
        visited = (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        ok = lit_init_first<MW>(q, q.pat[pid], op, L, lane);
        t0 = 1;
    } else {
        lit_init<MW>(q, L, lane);
    }
    for (int t = t0; t < len - 1 && ok; ++t) {
        const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
        ++ran;
        visited += (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        ok = lit_step<MW, false>(q, q.pat[pid], op, L, lane, nullptr);
    }
    if (!ok) {                       // every candidate of the group stops inside the prefix
        if (part == 0) { steps += I * ran; members += I * visited; }
        return;
    }
    const int C = row_classes<MW>(q, L, X, full, lane);
    for (int a = part; a < q.alphabet; a += parts) {
        const uint32_t ins = q.instr_of_digit[a];
        if (lit_classify<MW>(q, q.pat[ins >> 3], (int)(ins & 7u), L, X, C, full, lane) == 2 && lane == 0) {
            const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
            if (pos < q.valid_cap) q.valid_idx[pos] = idx0 + (unsigned long long)a;
        }
    }
    if (part == 0) {
        steps += I * (ran + 1ull);
        members += I * visited + (unsigned long long)q.reg_sum_part;
    }
}

// `count` consecutive groups under one stem whose state left the compact form (kStemEntry): the stem's
// literal state is rebuilt once and kept in `backup`; every group then adds its own instruction to it
// (an invalid instruction leaves the state as it was, a valid one is undone from the copy) and judges all
// last instructions as literal_group does.  Part `part` of `parts` takes the groups part, part + parts, ...
// and counts the steps of their candidates.
template <int MW>
__device__ inline void literal_stem(const DevQuery& q, unsigned long long idx0, int count, const LitLds& L, const FrontLit& X,
                                    const uint32_t* full, int lane, int part, int parts, uint32_t* __restrict__ backup,
                                    unsigned long long& steps, unsigned long long& members) {
    uint16_t digit[P2_MAX_LEN + 1];
    const int len = unrank(q, idx0, digit);         // len >= 3: digit[len-2] is the first group's instruction
    const unsigned long long I = (unsigned long long)q.alphabet;
    bool ok = true;
    unsigned long long ran = 0, visited = 0;
    int t0 = 0;
    if (len - 2 >= 1) {                              // the first instruction: its result is known without a pass
        const int pid = digit[0] / q.n_ops, op = q.ops[digit[0] - pid * q.n_ops];
        ran = 1;
        visited = (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        ok = lit_init_first<MW>(q, q.pat[pid], op, L, lane);
        t0 = 1;
    } else {
        lit_init<MW>(q, L, lane);
    }
    for (int t = t0; t < len - 2 && ok; ++t) {
        const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
        ++ran;
        visited += (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        ok = lit_step<MW, false>(q, q.pat[pid], op, L, lane, nullptr);
    }
    const int mine = part < count ? (count - part + parts - 1) / parts : 0;      // groups of this part
    if (!ok) {                                      // every candidate under the stem stops inside it
        steps += (unsigned long long)mine * I * ran;
        members += (unsigned long long)mine * I * visited;
        return;
    }
    const int s_words = q.R * q.k * MW;
    __syncthreads();
    for (int i = lane; i < s_words; i += kWave) backup[i] = L.S[i];
    bool dirty = false;
    for (int gi = part; gi < count; gi += parts) {
        if (dirty) {
            __syncthreads();
            for (int i = lane; i < s_words; i += kWave) L.S[i] = backup[i];
            __syncthreads();
            dirty = false;
        }
        const int dgt = (int)digit[len - 2] + gi;
        const int pid = dgt / q.n_ops, op = q.ops[dgt - pid * q.n_ops];
        const unsigned long long g_ran = ran + 1ull;
        const unsigned long long g_vis = visited + (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        if (!lit_step<MW, false>(q, q.pat[pid], op, L, lane, nullptr)) {
            steps += I * g_ran;
            members += I * g_vis;
            continue;
        }
        dirty = true;
        const int C = row_classes<MW>(q, L, X, full, lane);
        const unsigned long long first = idx0 + (unsigned long long)gi * I;
        for (int a = 0; a < q.alphabet; ++a) {
            const uint32_t ins = q.instr_of_digit[a];
            if (lit_classify<MW>(q, q.pat[ins >> 3], (int)(ins & 7u), L, X, C, full, lane) == 2 && lane == 0) {
                const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
                if (pos < q.valid_cap) q.valid_idx[pos] = first + (unsigned long long)a;
            }
        }
        steps += I * (g_ran + 1ull);
        members += I * g_vis + (unsigned long long)q.reg_sum_part;
    }
}

// ---- the literal state by classes of equal rows ----------------------------------------------------
// Rows that are equal on every device stay equal under AllReduce, Reduce, AllGather and Broadcast (the
// rules act row by row), and a ReduceScatter splits a class only where a block boundary of some group
// falls between two of its rows.  So a literal state can be kept as one row per class: [R][C] masks plus
// the class of every row and the class sizes; a step then costs C instead of k rows.  C is at most 64
// here; a ReduceScatter that would need more classes reports an overflow and the caller evaluates that
// entry on the full literal state instead.
struct ClsLds {
    uint32_t* S;        // [R][cs][MW]  mask of class c on device d
    uint32_t* T;        // [ng][cm][MW] combined rows of each group
    uint32_t* csize;    // [cm]  rows in the class
    uint32_t* ncsize;   // [cm]  (ReduceScatter) sizes of the new classes
    uint32_t* crow;     // [cm]  (ReduceScatter) first row of a new class
    uint32_t* gcount;   // [ng]  non-empty rows of the group's result
    uint32_t* gflag;    // [ng]  Broadcast: some member differs from the root
    uint32_t* gne;      // [ng][2] which classes of the group's result are non-empty
    uint32_t* devne;    // [R]   AllGather: device holds something
    uint32_t* devany;   // [R]   device holds something       (for instructions judged read-only)
    uint32_t* devfull;  // [R]   device is at the goal
    uint32_t* flags;    // [4]
    uint32_t* start;    // [16]  (ReduceScatter) bit r: row r is the first of a new class
    uint16_t* cls;      // [k]   class of a row
    uint16_t* ncls;     // [k]
    uint32_t* rows;     // [cm][kw] (ReduceScatter) bit r of class c: row r belongs to it
    uint32_t* bnd;      // [cm][kw] (ReduceScatter) bit r of class c: some group in which the class is not empty
                        //          starts a new block at row r
    uint8_t* own;       // [cm][ngs] (ReduceScatter) rank that keeps the new class in each group, 0xff: empty there
    int cm, cs, ngs;    // most classes held; words between the rows of two devices in S (odd: lanes that
                        // read the same class of different devices hit different banks); bytes per class in own
};
__host__ __device__ inline int cls_cmax(int k) { return k < 64 ? k : 64; }
// Words of the masks (S and T) and of the tables beside them.
__host__ __device__ inline int cls_mask_words(int R, int k, int MW) {
    const int cm = cls_cmax(k), ng = R / 2 > 0 ? R / 2 : 1;
    return R * (cm | 1) * MW + ng * cm * MW;
}
__host__ __device__ inline int cls_table_words(int R, int k) {
    const int cm = cls_cmax(k), ng = R / 2 > 0 ? R / 2 : 1, ngs = (ng + 3) & ~3, kh = (k + 1) / 2, kw = (k + 31) / 32;
    return 3 * cm + 4 * ng + 3 * R + 4 + 16 + 2 * kh + 2 * cm * kw + (cm * ngs) / 4 + 8;
}
__host__ __device__ inline int cls_words(int R, int k, int MW) { return cls_mask_words(R, k, MW) + cls_table_words(R, k); }
// Words of a stem's saved class state: S, the classes of the rows, the class sizes.
__host__ __device__ inline int cls_backup_words(int R, int k, int MW) { return R * cls_cmax(k) * MW + (k + 1) / 2 + cls_cmax(k) + 8; }
// masks: cls_mask_words words for S and T; p: cls_table_words words for the rest (may follow the masks).
__device__ inline ClsLds carve_cls(uint32_t* masks, uint32_t* p, int R, int k, int MW) {
    ClsLds X;
    X.cm = cls_cmax(k);
    const int ng = R / 2 > 0 ? R / 2 : 1, kh = (k + 1) / 2, kw = (k + 31) / 32;
    X.ngs = (ng + 3) & ~3;
    X.cs = X.cm | 1;
    X.S = masks;
    X.T = masks + R * X.cs * MW;
    X.csize = p; p += X.cm;
    X.ncsize = p; p += X.cm;
    X.crow = p; p += X.cm;
    X.gcount = p; p += ng;
    X.gflag = p; p += ng;
    X.gne = p; p += 2 * ng;
    X.devne = p; p += R;
    X.devany = p; p += R;
    X.devfull = p; p += R;
    X.flags = p; p += 4;
    X.start = p; p += 16;
    X.cls = reinterpret_cast<uint16_t*>(p); p += kh;
    X.ncls = reinterpret_cast<uint16_t*>(p); p += kh;
    X.rows = p; p += X.cm * kw;
    X.bnd = p; p += X.cm * kw;
    X.own = reinterpret_cast<uint8_t*>(p);
    return X;
}

enum : int { CSTEP_INVALID = 0, CSTEP_OK = 1, CSTEP_OVERFLOW = 2 };

// Sec. 3.5: device i holds column i in every row -- one class.
template <int MW>
__device__ inline void cls_init(const DevQuery& q, const ClsLds& X, int& C, int lane, const int nt = kWave) {
    for (int d = lane; d < q.R; d += nt) {
#pragma unroll
        for (int w = 0; w < MW; ++w) X.S[d * X.cs * MW + w] = (w == (d >> 5)) ? (1u << (d & 31)) : 0u;
    }
    for (int r = lane; r < q.k; r += nt) X.cls[r] = 0;
    if (lane == 0) X.csize[0] = (uint32_t)q.k;
    C = 1;
    __syncthreads();
}

// The class state after a program's first instruction, written directly (see lit_init_first): one class
// after an AllReduce or a Reduce, one class per block of rows after a ReduceScatter.
template <int MW>
__device__ inline int cls_init_first(const DevQuery& q, const DevPattern& P, int op, const ClsLds& X, int& C, int lane) {
    static_assert(MW <= 2, "groups of at most 64 devices");
    if (op == OP_AG || op == OP_BC) return CSTEP_INVALID;
    if (op == OP_RS && q.k % P.g != 0) return CSTEP_INVALID;
    const int nc = op == OP_RS ? P.g : 1;
    if (nc > X.cm) return CSTEP_OVERFLOW;
    const int per = q.k / nc;
    const uint32_t gmask = (uint32_t)(P.g - 1) * (uint32_t)P.s;          // g and s are powers of two
    for (int it = lane; it < q.R * nc; it += kWave) {
        const int d = it / nc, c = it - d * nc;
        const bool in = !P.master || (d % P.s) == 0;
        unsigned long long cols = 1ull << d;
        if (in) {
            cols = 1ull << ((uint32_t)d & ~gmask);
            for (uint32_t b = (uint32_t)P.s; b < (uint32_t)(P.g * P.s); b <<= 1) cols |= cols << b;
            const int p = (int)(((uint32_t)d & gmask) / (uint32_t)P.s);
            if (op == OP_RS && c != p) cols = 0ull;
            if (op == OP_RD && p != 0) cols = 0ull;
        }
        X.S[(d * X.cs + c) * MW] = (uint32_t)cols;
        if (MW > 1) X.S[(d * X.cs + c) * MW + (MW > 1 ? 1 : 0)] = (uint32_t)(cols >> 32);
    }
    for (int r = lane; r < q.k; r += kWave) X.cls[r] = (uint16_t)(r / per);
    for (int c = lane; c < nc; c += kWave) X.csize[c] = (uint32_t)per;
    C = nc;
    __syncthreads();
    return CSTEP_OK;
}

// b / per for b < 512 and 0 < per <= 512: the quotient of (b + 1/2) / per is at least 1/1024 away from an
// integer, far more than the error of the fast division.
__device__ __forceinline__ uint32_t small_div(uint32_t b, uint32_t per) {
    return (uint32_t)__fdividef((float)b + 0.5f, (float)per);
}

// ReduceScatter on the class state, after cls_step has checked the premises and left the groups' combined
// rows in T, their non-empty classes in gne and their non-empty row counts in gcount.  Row r, the b-th
// non-empty row of group G, stays with the member of rank b / (gcount[G] / g).  Two rows of a class remain
// in one class iff they stay with the same rank in every group in which the class is not empty; the ranks
// grow with the row number, so the new classes are runs of consecutive rows of an old class, and a row
// starts a run iff some such group starts a new block after the previous row of the class, up to the row.
template <int MW>
__device__ int cls_scatter(const DevQuery& q, const DevPattern& P, const ClsLds& X, int& C, int lane, const int nt = kWave) {
    const int k = q.k, g = P.g, s = P.s, ng = P.n_groups, gs = g * s, cm = X.cm, cs = X.cs, ngs = X.ngs;
    const int kw = (k + 31) / 32;
    // (lane = thread of the block's nt; the passes that go by ballots over 64 consecutive rows are dealt out to
    //  the block's wavefronts by group or by run of rows)
    const int ln = lane & (kWave - 1), wv = lane / kWave, nw = nt / kWave;
    const unsigned long long below = (1ull << ln) - 1ull;
    for (int i = lane; i < C * kw; i += nt) { X.rows[i] = 0; X.bnd[i] = 0; }
    if (lane == 0) X.flags[3] = 0;                       // (the number of new classes is added up here)
    __syncthreads();
    for (int r = lane; r < k; r += nt) atomicOr(&X.rows[(int)X.cls[r] * kw + (r >> 5)], 1u << (r & 31));
    // block starts of every group, united per class (lane c keeps the words of class c)
    for (int G = wv; G < ng; G += nw) {
        const uint32_t per = X.gcount[G] / (uint32_t)g;
        if (per == 0u) continue;                          // a group of empty devices
        const unsigned long long gne = (unsigned long long)X.gne[2 * G] | ((unsigned long long)X.gne[2 * G + 1] << 32);
        const bool mine = ln < C && ((gne >> ln) & 1ull) != 0ull;
        uint32_t carry = 0;                               // non-empty rows of the group below the chunk
        for (int r0 = 0; r0 < k; r0 += kWave) {
            const int r = r0 + ln;
            const bool ne = r < k && ((gne >> X.cls[r < k ? r : 0]) & 1ull) != 0ull;
            const unsigned long long bal = __ballot(ne);
            const uint32_t before = carry + (uint32_t)__popcll(bal & below);
            const unsigned long long starts = __ballot(ne && before != 0u && small_div(before, per) * per == before);
            if (mine) {                                   // (several wavefronts, each with a group of its own, may meet in a word)
                if ((uint32_t)starts) atomicOr(&X.bnd[ln * kw + (r0 >> 5)], (uint32_t)starts);
                if ((r0 >> 5) + 1 < kw && (uint32_t)(starts >> 32)) atomicOr(&X.bnd[ln * kw + (r0 >> 5) + 1], (uint32_t)(starts >> 32));
            }
            carry += (uint32_t)__popcll(bal);
        }
    }
    __syncthreads();
    // run starts
    int newC = 0;
    for (int r0 = wv * kWave; r0 < k; r0 += nt) {
        const int r = r0 + ln;
        bool st = false;
        if (r < k) {
            const int c = (int)X.cls[r];
            const uint32_t* const mine = X.rows + c * kw;
            int w = r >> 5;
            uint32_t m = mine[w] & ((1u << (r & 31)) - 1u);
            while (m == 0u && w > 0) { --w; m = mine[w]; }
            st = m == 0u;                                  // no earlier row in the class
            if (!st) {
                const int p = w * 32 + 31 - __clz((int)m);  // the previous row of the class: a block start in (p, r]?
                const uint32_t* const b = X.bnd + c * kw;
                for (int v = p >> 5; v <= (r >> 5); ++v) {
                    uint32_t x = b[v];
                    if (v == (p >> 5)) x &= ~(((1u << (p & 31)) << 1) - 1u);
                    if (v == (r >> 5)) x &= ((1u << (r & 31)) << 1) - 1u;
                    st |= x != 0u;
                }
            }
        }
        const unsigned long long bal = __ballot(st);
        if (ln == 0) { X.start[r0 >> 5] = (uint32_t)bal; X.start[(r0 >> 5) + 1] = (uint32_t)(bal >> 32); }
        newC += __popcll(bal);
    }
    if (ln == 0 && newC) atomicAdd(&X.flags[3], (uint32_t)newC);
    __syncthreads();
    newC = (int)X.flags[3];
    if (newC > cm) return CSTEP_OVERFLOW;                 // (nothing of the state has been written yet)
    for (int i = lane; i < newC; i += nt) X.ncsize[i] = 0;
    __syncthreads();
    // the new class of a row: the number of run starts below the start of its own run
    for (int r = lane; r < k; r += nt) {
        const uint32_t* const mine = X.rows + (int)X.cls[r] * kw;
        int w = r >> 5;
        uint32_t m = mine[w] & X.start[w] & (((1u << (r & 31)) << 1) - 1u);
        while (m == 0u) { --w; m = mine[w] & X.start[w]; }           // (the first row of a class starts a run)
        const int sr = w * 32 + 31 - __clz((int)m);
        int id = 0;
        for (int v = 0; v < (sr >> 5); ++v) id += __popc(X.start[v]);
        id += __popc(X.start[sr >> 5] & ((1u << (sr & 31)) - 1u));
        X.ncls[r] = (uint16_t)id;
        atomicAdd(&X.ncsize[id], 1u);
        if (sr == r) X.crow[id] = (uint32_t)r;
    }
    __syncthreads();
    // the rank that keeps each new class in each group: that of the class's first row
    for (int G = wv; G < ng; G += nw) {
        const uint32_t per = X.gcount[G] / (uint32_t)g;
        if (per == 0u) {
            for (int c2 = ln; c2 < newC; c2 += kWave) X.own[c2 * ngs + G] = (uint8_t)0xff;
            continue;
        }
        const unsigned long long gne = (unsigned long long)X.gne[2 * G] | ((unsigned long long)X.gne[2 * G + 1] << 32);
        uint32_t carry = 0;
        for (int r0 = 0; r0 < k; r0 += kWave) {
            const int r = r0 + ln;
            const bool ne = r < k && ((gne >> X.cls[r < k ? r : 0]) & 1ull) != 0ull;
            const unsigned long long bal = __ballot(ne);
            const uint32_t before = carry + (uint32_t)__popcll(bal & below);
            if (r < k && ((X.start[r >> 5] >> (r & 31)) & 1u) != 0u)
                X.own[(int)X.ncls[r] * ngs + G] = ne ? (uint8_t)small_div(before, per) : (uint8_t)0xff;
            carry += (uint32_t)__popcll(bal);
        }
    }
    __syncthreads();
    // members: the rank that keeps the class takes the group's combined row, the others are left empty
    for (int it = lane; it < q.R * newC; it += nt) {
        const int d = it / newC, c2 = it - d * newC;
        if (P.master && (d % s) != 0) continue;
        const int G = P.master ? d / gs : (d / gs) * s + d % s;
        const int p = (d / s) % g;
        const int oc = (int)X.cls[X.crow[c2]];
        const bool keep = (int)X.own[c2 * ngs + G] == p;
#pragma unroll
        for (int w = 0; w < MW; ++w) X.S[(d * cs + c2) * MW + w] = keep ? X.T[(G * cm + oc) * MW + w] : 0u;
    }
    // devices outside the pattern keep their rows: move them to the new classes, one device at a time
    // (a lane per new class reads its old class, then all write)
    if (P.master) {
        for (int d = 0; d < q.R; ++d) {
            if ((d % s) == 0) continue;
            uint32_t v[MW];
            if (lane < newC) {
                const int oc = (int)X.cls[X.crow[lane]];
#pragma unroll
                for (int w = 0; w < MW; ++w) v[w] = X.S[(d * cs + oc) * MW + w];
            }
            __syncthreads();
            if (lane < newC) {
#pragma unroll
                for (int w = 0; w < MW; ++w) X.S[(d * cs + lane) * MW + w] = v[w];
            }
            __syncthreads();
        }
    }
    __syncthreads();
    for (int r = lane; r < k; r += nt) X.cls[r] = X.ncls[r];
    for (int i = lane; i < newC; i += nt) X.csize[i] = X.ncsize[i];
    C = newC;
    __syncthreads();
    return CSTEP_OK;
}

// One instruction on the class state (the rules of lit_step, a class standing for its rows).  All nt threads
// of the block call it with the same arguments (lane = thread number; nt a multiple of 64).  An invalid step and an overflow leave the state as it was.
template <int MW>
__device__ int cls_step(const DevQuery& q, const DevPattern& P, int op, const ClsLds& X, int& C, int lane, const int nt = kWave) {
    const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s, cm = X.cm, cs = X.cs;
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    for (int i = lane; i < ng; i += nt) { X.gcount[i] = 0; X.gflag[i] = 0; X.gne[2 * i] = 0; X.gne[2 * i + 1] = 0; }
    if (op == OP_AG)
        for (int i = lane; i < q.R; i += nt) X.devne[i] = 0;
    if (lane == 0) { X.flags[0] = 0; X.flags[1] = 0; }
    __syncthreads();
    const int items = ng * C;
    bool bad = false;
    for (int it = lane; it < items; it += nt) {
        const int G = div_fast(it, C), c = it - G * C;
        const int base = group_base(P.master, G, s, gs);
        uint32_t acc[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) acc[w] = 0;
        if (red) {
            bool ne0 = false;
            for (int p = 0; p < g; ++p) {
                const uint32_t* x = X.S + ((base + p * s) * cs + c) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    const uint32_t v = x[w];
                    any |= v;
                    bad |= (acc[w] & v) != 0;
                    acc[w] |= v;
                }
                if (p == 0) ne0 = any != 0;
                else bad |= (any != 0) != ne0;
            }
            if (ne0) {
                atomicAdd(&X.gcount[G], X.csize[c]);
                atomicOr(&X.gne[2 * G + (c >> 5)], 1u << (c & 31));
            }
        } else if (op == OP_AG) {
            int holders = 0;
            for (int p = 0; p < g; ++p) {
                const int dev = base + p * s;
                const uint32_t* x = X.S + (dev * cs + c) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) { const uint32_t v = x[w]; any |= v; acc[w] |= v; }
                if (any) { ++holders; X.devne[dev] = 1; }
            }
            bad |= holders > 1;
        } else {
            const uint32_t* root = X.S + (base * cs + c) * MW;
#pragma unroll
            for (int w = 0; w < MW; ++w) acc[w] = root[w];
            bool differs = false;
            for (int p = 1; p < g; ++p) {
                const uint32_t* x = X.S + ((base + p * s) * cs + c) * MW;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    const uint32_t v = x[w];
                    bad |= (v & ~acc[w]) != 0;
                    differs |= v != acc[w];
                }
            }
            if (differs) X.gflag[G] = 1;
        }
#pragma unroll
        for (int w = 0; w < MW; ++w) X.T[(G * cm + c) * MW + w] = acc[w];
    }
    if (bad) X.flags[0] = 1;
    __syncthreads();
    for (int G = lane; G < ng; G += nt) {
        const uint32_t cnt = X.gcount[G];
        if (red) {
            if (op == OP_RS && cnt % (uint32_t)g != 0) X.flags[0] = 1;   // scatter: chunks must divide evenly
            if (cnt) X.flags[1] = 1;                                    // a group of empty devices is a no-op
        } else if (op == OP_AG) {
            const int base = group_base(P.master, G, s, gs);
            for (int p = 0; p < g; ++p)
                if (!X.devne[base + p * s]) X.flags[0] = 1;
            X.flags[1] = 1;
        } else {
            if (!X.gflag[G]) X.flags[0] = 1;                            // no information increase
            X.flags[1] = 1;
        }
    }
    __syncthreads();
    if (X.flags[0] || !X.flags[1]) return CSTEP_INVALID;
    if (op == OP_RS) return cls_scatter<MW>(q, P, X, C, lane, nt);
    for (int it = lane; it < items; it += nt) {
        const int G = div_fast(it, C), c = it - G * C;
        const int base = group_base(P.master, G, s, gs);
        uint32_t t[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) t[w] = X.T[(G * cm + c) * MW + w];
        for (int p = (op == OP_BC ? 1 : 0); p < g; ++p) {
            uint32_t* x = X.S + ((base + p * s) * cs + c) * MW;
            const bool keep = op != OP_RD || p == 0;
#pragma unroll
            for (int w = 0; w < MW; ++w) x[w] = keep ? t[w] : 0u;
        }
    }
    __syncthreads();
    return CSTEP_OK;
}

// One instruction against the class state, read-only (lit_classify on classes): 0 = invalid step,
// 2 = valid and the result is the goal, 3 = valid.  Needs devany and devfull.
template <int MW>
__device__ int cls_classify(const DevQuery& q, const DevPattern& P, int op, const ClsLds& X, int C, const uint32_t* full,
                            int lane, const int nt = kWave) {
    const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s, cs = X.cs;
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    for (int i = lane; i < ng; i += nt) { X.gcount[i] = 0; X.gflag[i] = 0; }
    if (lane == 0) { X.flags[0] = 0; X.flags[1] = 0; X.flags[2] = 0; }
    __syncthreads();
    const int items = ng * C;
    bool bad = false, notfull = false;
    for (int it = lane; it < items; it += nt) {
        const int G = div_fast(it, C), c = it - G * C;
        const int base = group_base(P.master, G, s, gs);
        uint32_t acc[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) acc[w] = 0;
        if (red) {
            bool ne0 = false;
            for (int p = 0; p < g; ++p) {
                const uint32_t* x = X.S + ((base + p * s) * cs + c) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    const uint32_t v = x[w];
                    any |= v;
                    bad |= (acc[w] & v) != 0;
                    acc[w] |= v;
                }
                if (p == 0) ne0 = any != 0;
                else bad |= (any != 0) != ne0;
            }
            if (ne0) atomicAdd(&X.gcount[G], X.csize[c]);
        } else if (op == OP_AG) {
            int holders = 0;
            for (int p = 0; p < g; ++p) {
                const int dev = base + p * s;
                const uint32_t* x = X.S + (dev * cs + c) * MW;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < MW; ++w) { const uint32_t v = x[w]; any |= v; acc[w] |= v; }
                holders += any != 0;
                if (c == 0) bad |= X.devany[dev] == 0;
            }
            bad |= holders > 1;
        } else {
            const uint32_t* root = X.S + (base * cs + c) * MW;
#pragma unroll
            for (int w = 0; w < MW; ++w) acc[w] = root[w];
            bool differs = false;
            for (int p = 1; p < g; ++p) {
                const uint32_t* x = X.S + ((base + p * s) * cs + c) * MW;
#pragma unroll
                for (int w = 0; w < MW; ++w) {
                    const uint32_t v = x[w];
                    bad |= (v & ~acc[w]) != 0;
                    differs |= v != acc[w];
                }
            }
            if (differs) X.gflag[G] = 1;
        }
#pragma unroll
        for (int w = 0; w < MW; ++w) notfull |= acc[w] != full[w];
    }
    if (bad) X.flags[0] = 1;
    if (notfull) X.flags[2] = 1;
    // devices the pattern does not touch must already be at the goal
    if (P.master)
        for (int d = lane; d < q.R; d += nt) {
            const bool part = d % s == 0 && d / gs < ng;
            if (!part && !X.devfull[d]) X.flags[2] = 1;
        }
    __syncthreads();
    for (int G = lane; G < ng; G += nt) {
        const uint32_t cnt = X.gcount[G];
        if (red) {
            if (op == OP_RS && cnt % (uint32_t)g != 0) X.flags[0] = 1;
            if (cnt) X.flags[1] = 1;
        } else if (op == OP_BC) {
            if (!X.gflag[G]) X.flags[0] = 1;
        }
    }
    __syncthreads();
    const bool invalid = X.flags[0] != 0 || (red && X.flags[1] == 0);
    const bool goal = (op == OP_AR || op == OP_AG || op == OP_BC) && X.flags[2] == 0;
    __syncthreads();
    return invalid ? 0 : goal ? 2 : 3;
}

// Per device: holds anything (devany), is at the goal (devfull); and over all devices: every row is held
// everywhere, every held row is complete, device 0 is at the goal.
template <int MW>
__device__ inline void cls_device_flags(const DevQuery& q, const ClsLds& X, int C, const uint32_t* full, int lane,
                                        bool& rows_full, bool& cols_full, bool& root_done, const int nt = kWave) {
    bool rows_bad = false, cols_bad = false;
    if (lane == 0) { X.flags[0] = 0; X.flags[1] = 0; }
    __syncthreads();
    for (int d = lane; d < q.R; d += nt) {
        bool any = false, all = true;
        for (int c = 0; c < C; ++c) {
            const uint32_t* x = X.S + (d * X.cs + c) * MW;
            bool ne = false, fl = true;
#pragma unroll
            for (int w = 0; w < MW; ++w) { ne |= x[w] != 0u; fl &= x[w] == full[w]; }
            rows_bad |= !ne; cols_bad |= ne && !fl; all &= fl; any |= ne;
        }
        X.devany[d] = any; X.devfull[d] = all;
    }
    if (rows_bad) X.flags[0] = 1;
    if (cols_bad) X.flags[1] = 1;
    __syncthreads();
    rows_full = X.flags[0] == 0u;
    cols_full = X.flags[1] == 0u;
    root_done = X.devfull[0] != 0u;
    __syncthreads();                                     // (the flags are used again by what follows)
}

// The last instructions a = part, part + parts, ... of a group against the class state; those that are valid
// and reach the goal are reported.  Only the goal matters here (the candidates' steps are counted by the
// caller), and the goal can only come from an AllReduce on devices that all hold every row, from an AllGather
// on devices whose rows all carry every column, or from a Broadcast whose roots (device 0 is one in every
// pattern) are at the goal already: ReduceScatter and Reduce leave members short of rows, an AllReduce gives
// nobody a new row, an AllGather leaves every row with its holder's columns, a Broadcast with its root's.
// So most states need no instruction looked at.
template <int MW>
__device__ inline void cls_judge_all(const DevQuery& q, unsigned long long first, const ClsLds& X, int C, const uint32_t* full,
                                     int lane, int part, int parts) {
    bool rows_full, cols_full, root_done;
    cls_device_flags<MW>(q, X, C, full, lane, rows_full, cols_full, root_done);
    if (!(rows_full || cols_full || root_done)) return;
    for (int a = part; a < q.alphabet; a += parts) {
        const uint32_t ins = q.instr_of_digit[a];
        const int op = (int)(ins & 7u);
        if (!((op == OP_AR && rows_full) || (op == OP_AG && cols_full) || (op == OP_BC && root_done))) continue;
        if (cls_classify<MW>(q, q.pat[ins >> 3], op, X, C, full, lane) == 2 && lane == 0) {
            const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
            if (pos < q.valid_cap) q.valid_idx[pos] = first + (unsigned long long)a;
        }
    }
}

// Frontier level for literal prefixes, on the full literal state: a block rebuilds the state of one
// prefix and classifies every instruction against it.  With elist, only the entries elist[0 .. *elist_n).
// NT threads per block: one wavefront where the state is in LDS; eight where it lies in the block's slice of
// global memory (R * k * MW words: 16 MiB for 512 devices and chunks), so that a pass over it is the work of
// eight wavefronts' loads in flight instead of one's.
template <int MW, int NT>
__global__ __launch_bounds__(NT) void k_front_classify_literal(const DevQuery* __restrict__ qp,
                                                                  const FrontEntry* __restrict__ entries, uint32_t n_entries,
                                                                  const uint32_t* __restrict__ elist,
                                                                  const uint32_t* __restrict__ elist_n,
                                                                  int parent_len, int goals_only, FrontSurvivor* __restrict__ surv,
                                                                  uint32_t surv_cap, FrontCounters* __restrict__ ctr,
                                                                  uint32_t* __restrict__ gscratch, unsigned long long gwords) {
    extern __shared__ uint32_t lds[];
    const DevQuery& q = *qp;
    const int lane = threadIdx.x;
    const LitLds L = carve(gscratch ? gscratch + (size_t)blockIdx.x * gwords : lds, q.R, q.k, MW);
    const FrontLit X = carve_front(L.flags + 4, q.k);
    const int R = q.R, I = q.alphabet;
    uint32_t full[MW];
#pragma unroll
    for (int w = 0; w < MW; ++w) {
        const int bits = R - 32 * w;
        full[w] = bits >= 32 ? 0xffffffffu : bits > 0 ? ((1u << bits) - 1u) : 0u;
    }
    unsigned long long steps = 0, members = 0;
    const uint32_t n = elist ? *elist_n : n_entries;
    for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
        const uint32_t e = elist ? elist[i] : i;
        const unsigned long long digits = entries[e].digits;
        lit_init<MW>(q, L, lane, NT);
        for (int t = 0; t < parent_len; ++t) {
            const uint32_t ins = q.instr_of_digit[(int)((digits >> (9 * t)) & 511ull)];
            lit_step<MW, false>(q, q.pat[ins >> 3], (int)(ins & 7u), L, lane, nullptr, NT);
        }
        const int C = row_classes<MW>(q, L, X, full, lane, NT);
        // At the size limit only goals count, and few instructions can reach the goal from a given state (see
        // cls_judge_all): the others are not looked at.
        const bool rows_full = rows_all_held(X), cols_full = held_rows_complete(X), root_done = X.devfull[0] != 0u;
        for (int a = 0; a < I; ++a) {
            const uint32_t ins = q.instr_of_digit[a];
            const DevPattern& P = q.pat[ins >> 3];
            ++steps;
            members += (unsigned long long)(P.n_groups * P.g);
            if (goals_only) {
                const int op = (int)(ins & 7u);
                if (!((op == OP_AR && rows_full) || (op == OP_AG && cols_full) || (op == OP_BC && root_done))) continue;
            }
            const int code = lit_classify<MW>(q, P, (int)(ins & 7u), L, X, C, full, lane, NT);
            if (code != 0 && lane == 0) {
                const uint32_t pos = atomicAdd(&ctr->n_surv_literal, 1u);
                if (pos < surv_cap) { FrontSurvivor sv; sv.entry = e; sv.digit = (uint16_t)a; sv.code = (uint16_t)code; surv[pos] = sv; }
                atomicAdd(code == 2 ? &ctr->n_goal : &ctr->n_prefix_literal, 1u);
            }
        }
        __syncthreads();
    }
    if (lane == 0 && steps) { atomicAdd(&ctr->steps, steps); atomicAdd(&ctr->members, members); }
}

// The same on the class state (in LDS, or in the block's slice of a global buffer where it does not fit): a
// prefix is rebuilt at the cost of its classes instead of its k rows.  A prefix that needs more classes than
// the state holds is put on the list `over` (ctr->n_overflow entries) for the kernel above.  NT threads per block:
// one wavefront where the masks are in LDS, several where they lie in global memory (as in the kernel above).
template <int MW, int NT>
__global__ __launch_bounds__(NT) void k_front_classify_classes(const DevQuery* __restrict__ qp,
                                                                  const FrontEntry* __restrict__ entries, uint32_t n_entries,
                                                                  int parent_len, int goals_only, FrontSurvivor* __restrict__ surv,
                                                                  uint32_t surv_cap, FrontCounters* __restrict__ ctr,
                                                                  uint32_t* __restrict__ over, uint32_t* __restrict__ gscratch,
                                                                  unsigned long long gwords, int class_cap) {
    extern __shared__ uint32_t lds[];
    const DevQuery& q = *qp;
    const int lane = threadIdx.x;
    // the tables are always in LDS; the masks follow them there, or are in the block's global slice
    ClsLds X = carve_cls(gscratch ? gscratch + (size_t)blockIdx.x * gwords : lds + cls_table_words(q.R, q.k), lds, q.R, q.k, MW);
    X.cm = X.cm < class_cap ? X.cm : class_cap;
    const int R = q.R, I = q.alphabet;
    uint32_t full[MW];
#pragma unroll
    for (int w = 0; w < MW; ++w) {
        const int bits = R - 32 * w;
        full[w] = bits >= 32 ? 0xffffffffu : bits > 0 ? ((1u << bits) - 1u) : 0u;
    }
    unsigned long long steps = 0, members = 0;
    for (uint32_t e = blockIdx.x; e < n_entries; e += gridDim.x) {
        const unsigned long long digits = entries[e].digits;
        int C = 1, rc = CSTEP_OK;
        cls_init<MW>(q, X, C, lane, NT);
        for (int t = 0; t < parent_len && rc == CSTEP_OK; ++t) {
            const uint32_t ins = q.instr_of_digit[(int)((digits >> (9 * t)) & 511ull)];
            rc = cls_step<MW>(q, q.pat[ins >> 3], (int)(ins & 7u), X, C, lane, NT);
        }
        if (rc != CSTEP_OK) {                    // too many classes: the full literal state decides
            if (lane == 0) over[atomicAdd(&ctr->n_overflow, 1u)] = e;
            continue;
        }
        bool rows_full, cols_full, root_done;
        cls_device_flags<MW>(q, X, C, full, lane, rows_full, cols_full, root_done, NT);
        for (int a = 0; a < I; ++a) {
            const uint32_t ins = q.instr_of_digit[a];
            const DevPattern& P = q.pat[ins >> 3];
            ++steps;
            members += (unsigned long long)(P.n_groups * P.g);
            if (goals_only) {        // (at the size limit only goals count: see cls_judge_all)
                const int op = (int)(ins & 7u);
                if (!((op == OP_AR && rows_full) || (op == OP_AG && cols_full) || (op == OP_BC && root_done))) continue;
            }
            const int code = cls_classify<MW>(q, P, (int)(ins & 7u), X, C, full, lane, NT);
            if (code != 0 && lane == 0) {
                const uint32_t pos = atomicAdd(&ctr->n_surv_literal, 1u);
                if (pos < surv_cap) { FrontSurvivor sv; sv.entry = e; sv.digit = (uint16_t)a; sv.code = (uint16_t)code; surv[pos] = sv; }
                atomicAdd(code == 2 ? &ctr->n_goal : &ctr->n_prefix_literal, 1u);
            }
        }
        __syncthreads();
    }
    if (lane == 0 && steps) { atomicAdd(&ctr->steps, steps); atomicAdd(&ctr->members, members); }
}

// literal_group on the class state.  Returns false, with nothing counted or reported, when a step needs more
// classes than the state holds.
template <int MW>
__device__ inline bool cls_group(const DevQuery& q, unsigned long long idx0, const ClsLds& X, const uint32_t* full, int lane,
                                 int part, int parts, unsigned long long& steps, unsigned long long& members) {
    uint16_t digit[P2_MAX_LEN + 1];
    const int len = unrank(q, idx0, digit);
    const unsigned long long I = (unsigned long long)q.alphabet;
    int rc = CSTEP_OK, C = 1;
    unsigned long long ran = 0, visited = 0;
    int t0 = 0;
    if (len - 1 >= 1) {
        const int pid = digit[0] / q.n_ops, op = q.ops[digit[0] - pid * q.n_ops];
        ran = 1;
        visited = (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        rc = cls_init_first<MW>(q, q.pat[pid], op, X, C, lane);
        t0 = 1;
    } else {
        cls_init<MW>(q, X, C, lane);
    }
    for (int t = t0; t < len - 1 && rc == CSTEP_OK; ++t) {
        const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
        ++ran;
        visited += (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        rc = cls_step<MW>(q, q.pat[pid], op, X, C, lane);
    }
    if (rc == CSTEP_OVERFLOW) return false;
    if (rc == CSTEP_INVALID) {
        if (part == 0) { steps += I * ran; members += I * visited; }
        return true;
    }
    cls_judge_all<MW>(q, idx0, X, C, full, lane, part, parts);
    if (part == 0) {
        steps += I * (ran + 1ull);
        members += I * visited + (unsigned long long)q.reg_sum_part;
    }
    return true;
}

// literal_stem on the class state; the stem's class state is kept in `backup` (global).  Returns false, with
// nothing counted or reported, when the stem itself needs more classes than the state holds; a group whose
// own instruction does is evaluated by literal_group on the full state (L, F).
template <int MW>
__device__ inline bool cls_stem(const DevQuery& q, unsigned long long idx0, int count, const ClsLds& X, const uint32_t* full,
                                int lane, int part, int parts, uint32_t* __restrict__ backup, const LitLds& L, const FrontLit& F,
                                unsigned long long& steps, unsigned long long& members) {
    uint16_t digit[P2_MAX_LEN + 1];
    const int len = unrank(q, idx0, digit);         // len >= 3: digit[len-2] is the first group's instruction
    const unsigned long long I = (unsigned long long)q.alphabet;
    int rc = CSTEP_OK, C = 1;
    unsigned long long ran = 0, visited = 0;
    int t0 = 0;
    if (len - 2 >= 1) {
        const int pid = digit[0] / q.n_ops, op = q.ops[digit[0] - pid * q.n_ops];
        ran = 1;
        visited = (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        rc = cls_init_first<MW>(q, q.pat[pid], op, X, C, lane);
        t0 = 1;
    } else {
        cls_init<MW>(q, X, C, lane);
    }
    for (int t = t0; t < len - 2 && rc == CSTEP_OK; ++t) {
        const int pid = digit[t] / q.n_ops, op = q.ops[digit[t] - pid * q.n_ops];
        ++ran;
        visited += (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        rc = cls_step<MW>(q, q.pat[pid], op, X, C, lane);
    }
    if (rc == CSTEP_OVERFLOW) return false;
    const int mine = part < count ? (count - part + parts - 1) / parts : 0;      // groups of this part
    if (rc == CSTEP_INVALID) {                      // every candidate under the stem stops inside it
        steps += (unsigned long long)mine * I * ran;
        members += (unsigned long long)mine * I * visited;
        return true;
    }
    const int cm = X.cm, cs = X.cs, kh = (q.k + 1) / 2, C0 = C;
    uint32_t* const b_cls = backup + q.R * cm * MW;
    uint32_t* const b_size = b_cls + kh;
    const uint32_t* const cls_w = reinterpret_cast<const uint32_t*>(X.cls);
    uint32_t* const cls_ww = reinterpret_cast<uint32_t*>(X.cls);
    for (int it = lane; it < q.R * C0; it += kWave) {
        const int d = it / C0, c = it - d * C0;
#pragma unroll
        for (int w = 0; w < MW; ++w) backup[(d * cm + c) * MW + w] = X.S[(d * cs + c) * MW + w];
    }
    for (int i = lane; i < kh; i += kWave) b_cls[i] = cls_w[i];
    for (int i = lane; i < C0; i += kWave) b_size[i] = X.csize[i];
    bool dirty = false;
    for (int gi = part; gi < count; gi += parts) {
        if (dirty) {
            __syncthreads();
            for (int it = lane; it < q.R * C0; it += kWave) {
                const int d = it / C0, c = it - d * C0;
#pragma unroll
                for (int w = 0; w < MW; ++w) X.S[(d * cs + c) * MW + w] = backup[(d * cm + c) * MW + w];
            }
            for (int i = lane; i < kh; i += kWave) cls_ww[i] = b_cls[i];
            for (int i = lane; i < C0; i += kWave) X.csize[i] = b_size[i];
            C = C0;
            __syncthreads();
            dirty = false;
        }
        const int dgt = (int)digit[len - 2] + gi;
        const int pid = dgt / q.n_ops, op = q.ops[dgt - pid * q.n_ops];
        const unsigned long long g_ran = ran + 1ull;
        const unsigned long long g_vis = visited + (unsigned long long)(q.pat[pid].n_groups * q.pat[pid].g);
        const unsigned long long first = idx0 + (unsigned long long)gi * I;
        const int rg = cls_step<MW>(q, q.pat[pid], op, X, C, lane);
        if (rg == CSTEP_INVALID) {
            steps += I * g_ran;
            members += I * g_vis;
            continue;
        }
        if (rg == CSTEP_OVERFLOW) {                 // (the class state is untouched)
            literal_group<MW>(q, first, L, F, full, lane, 0, 1, steps, members);
            continue;
        }
        dirty = true;
        cls_judge_all<MW>(q, first, X, C, full, lane, 0, 1);
        steps += I * (g_ran + 1ull);
        members += I * g_vis + (unsigned long long)q.reg_sum_part;
    }
    return true;
}

// The groups that the shared-prefix kernel has just handed over, found on the device: those of the queries
// qlist[0 .. n_q), read from their counters and lists.  A unit of work is one (group, part) pair; blocks
// stride over the units.  This lets the host queue the kernel
// right behind the evaluation, without waiting for the counts.  A query whose list overflowed is left
// out (the host grows the list and runs the query again).  Few groups: up to 8 blocks share one.
template <int MW>
__global__ __launch_bounds__(kWave) void k_eval_literal_groups_auto(const DevQuery* __restrict__ queries,
                                                                    const int32_t* __restrict__ qlist, int n_q,
                                                                    uint32_t* __restrict__ gscratch,
                                                                    unsigned long long gwords, int cls_backup,
                                                                    int class_cap) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    // LDS holds the class state.  The block's slice of the global buffer: the copy of a stem's class state,
    // and for the entries that need more classes than the state holds the full literal state with its tables
    // and the copy of a stem's full state.
    uint32_t* const cls_copy = gscratch + (size_t)blockIdx.x * gwords;
    uint32_t* const mem = cls_copy + cls_backup;
    auto count_of = [&](int i) -> uint32_t {
        if (i >= n_q) return 0u;
        const DevQuery& q = queries[qlist[i]];
        const uint32_t n = q.counters->n_rerun;
        return n <= q.rerun_cap ? n : 0u;
    };
    uint32_t total = 0;
    for (int i0 = 0; i0 < n_q; i0 += kWave) {
        uint32_t c = count_of(i0 + lane);
        for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, kWave);
        total += c;
    }
    if (total == 0) return;
    uint32_t parts = gridDim.x / total;
    parts = parts < 1u ? 1u : parts > 8u ? 8u : parts;
    const unsigned long long n_units = (unsigned long long)total * parts;
    // units differ widely in length (a group whose prefix is invalid ends at once): blocks draw them from a
    // counter (kept with the first query's counters, zero at launch); total * parts < 2^32
    uint32_t* const next_unit = &queries[qlist[0]].counters->next_unit;
    // (a block's first unit is its own number, so a launch with fewer units than blocks draws nothing;
    // later draws take four units at a time)
    constexpr uint32_t kDraw = 4;
    uint32_t own_lo = 0, own_hi = 0;                    // entries [own_lo, own_hi) belong to query `owner`
    int owner = -1;
    unsigned long long unit = blockIdx.x, unit_end = unit + 1;
    while (unit < n_units) {
        const uint32_t e = (uint32_t)(unit / parts);
        const int part = (int)(unit - (unsigned long long)e * parts);
        if (owner < 0 || e < own_lo || e >= own_hi) {
            // the query that owns entry e: running sums of the counts, 64 queries at a time
            uint32_t base = 0;
            owner = -1;
            for (int i0 = 0; i0 < n_q && owner < 0; i0 += kWave) {
                const uint32_t c = count_of(i0 + lane);
                uint32_t incl = c;
                for (int off = 1; off < kWave; off <<= 1) {
                    const uint32_t up = __shfl_up(incl, off, kWave);
                    if (lane >= off) incl += up;
                }
                const bool mine = c != 0u && e >= base + incl - c && e < base + incl;
                const unsigned long long hit = __ballot(mine);
                if (hit != 0ull) {
                    const int src = __ffsll((long long)hit) - 1;
                    owner = i0 + src;
                    own_hi = base + __shfl(incl, src, kWave);
                    own_lo = base + __shfl(incl - c, src, kWave);
                } else {
                    base += __shfl(incl, kWave - 1, kWave);
                }
            }
            if (owner < 0) break;                       // cannot happen: e < total
        }
        const DevQuery& q = queries[qlist[owner]];
        const LitLds L = carve(mem, q.R, q.k, MW);
        const FrontLit X = carve_front(L.flags + 4, q.k);
        ClsLds Y = carve_cls(lds, lds + cls_mask_words(q.R, q.k, MW), q.R, q.k, MW);
        Y.cm = Y.cm < class_cap ? Y.cm : class_cap;
        uint32_t full[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) {
            const int bits = q.R - 32 * w;
            full[w] = bits >= 32 ? 0xffffffffu : bits > 0 ? ((1u << bits) - 1u) : 0u;
        }
        unsigned long long steps = 0, members = 0;
        const unsigned long long entry = q.rerun_idx[e - own_lo];
        // on the class state; on the full literal state where that needs more classes than it holds
        if (entry & kStemEntry) {
            const unsigned long long idx0 = entry & kEntryIndexMask;
            const int count = (int)((entry >> kStemCountShift) & 0x7ffull);
            if (!cls_stem<MW>(q, idx0, count, Y, full, lane, part, (int)parts, cls_copy, L, X, steps, members)) {
                LitLayout lay(q.R, q.k, MW);
                uint32_t* const backup = mem + lay.total_words() + front_lit_words(q.k);
                literal_stem<MW>(q, idx0, count, L, X, full, lane, part, (int)parts, backup, steps, members);
            }
        } else if (!cls_group<MW>(q, entry, Y, full, lane, part, (int)parts, steps, members)) {
            literal_group<MW>(q, entry, L, X, full, lane, part, (int)parts, steps, members);
        }
        if (lane == 0 && steps) {
            atomicAdd(&q.counters->steps[unit % kCounterStripes], steps);
            atomicAdd(&q.counters->members[unit % kCounterStripes], members);
        }
        __syncthreads();
        if (++unit == unit_end) {
            if (n_units <= gridDim.x) break;            // every unit was some block's first: nothing to draw
            uint32_t drawn = 0;
            if (lane == 0) drawn = atomicAdd(next_unit, kDraw);
            unit = (unsigned long long)gridDim.x + (uint32_t)__builtin_amdgcn_readfirstlane((int)drawn);
            unit_end = unit + kDraw;
        }
    }
}

template <typename F>
hipError_t allow_big_lds(F func, size_t bytes) {
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(func), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

inline int mask_words(int R) { return literal_mask_words(R); }

}  // namespace

size_t literal_lds_bytes(int R, int k) {
    LitLayout lay(R, k, mask_words(R));
    size_t bytes = (size_t)lay.total_words() * 4;
    return bytes <= kLdsLimit ? bytes : 0;
}
size_t literal_scratch_bytes(int R, int k, unsigned* blocks) {
    // states that do not fit in LDS: a fixed number of blocks, each with its own global slice
    LitLayout lay(R, k, mask_words(R));
    const size_t per = ((size_t)(lay.total_words() + front_lit_words(k)) * 4 + 255) / 256 * 256;
    unsigned b = 512;
    while (b > 1 && per * b > ((size_t)8 << 30)) b >>= 1;
    *blocks = b;
    return per * b;
}
size_t front_literal_lds_bytes(int R, int k) {
    LitLayout lay(R, k, mask_words(R));
    size_t bytes = (size_t)(lay.total_words() + front_lit_words(k)) * 4;
    return bytes <= kLdsLimit ? bytes : 0;
}

hipError_t launch_eval_literal(const DevQuery* q, int R, int k, unsigned long long start, unsigned long long count,
                               const unsigned long long* list, const uint32_t* list_count, void* gscratch,
                               hipStream_t stream) {
    if (count == 0) return hipSuccess;
    size_t lds = literal_lds_bytes(R, k);
    const int MW = mask_words(R);
    uint32_t per_block = 64;
    unsigned long long blocks;
    unsigned long long gwords = 0;
    if (lds == 0) {
        if (!gscratch) return hipErrorInvalidValue;
        unsigned nb = 0;
        gwords = literal_scratch_bytes(R, k, &nb) / nb / 4;
        blocks = nb < count ? nb : count;
        const unsigned long long pb = (count + blocks - 1) / blocks;
        if (pb > 0xffffffffull) return hipErrorInvalidValue;
        per_block = (uint32_t)pb;
        blocks = (count + per_block - 1) / per_block;
    } else {
        gscratch = nullptr;
        // enough blocks to fill 256 CUs several times over, at most 64 candidates per block
        while (per_block > 1 && (count + per_block - 1) / per_block < 8192) per_block >>= 1;
        blocks = (count + per_block - 1) / per_block;
    }
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_eval_literal<MWV>, lds);                                                               \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_eval_literal<MWV>, dim3((unsigned)blocks), dim3(kWave), lds, stream, q, start,    \
                           count, per_block, list, list_count, static_cast<uint32_t*>(gscratch), gwords);
    switch (MW) {
    case 1: P2_LAUNCH(1) break;
    case 2: P2_LAUNCH(2) break;
    case 4: P2_LAUNCH(4) break;
    case 8: P2_LAUNCH(8) break;
    default: P2_LAUNCH(16) break;
    }
#undef P2_LAUNCH
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

hipError_t launch_cost_literal(const DevQuery* q, int R, int k, const unsigned long long* sorted, uint32_t n,
                               p2_program* out_prog, double* out_cost, int only_missing, void* gscratch,
                               hipStream_t stream) {
    if (n == 0) return hipSuccess;
    size_t lds = literal_lds_bytes(R, k);
    const int MW = mask_words(R);
    unsigned blocks = n < 65536u ? n : 65536u;
    unsigned long long gwords = 0;
    if (lds == 0) {
        if (!gscratch) return hipErrorInvalidValue;
        unsigned nb = 0;
        gwords = literal_scratch_bytes(R, k, &nb) / nb / 4;
        blocks = nb < n ? nb : n;
    } else gscratch = nullptr;
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_cost_literal<MWV>, lds);                                                               \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_cost_literal<MWV>, dim3(blocks), dim3(kWave), lds, stream, q, sorted, n, out_prog, \
                           out_cost, only_missing, static_cast<uint32_t*>(gscratch), gwords);
    switch (MW) {
    case 1: P2_LAUNCH(1) break;
    case 2: P2_LAUNCH(2) break;
    case 4: P2_LAUNCH(4) break;
    case 8: P2_LAUNCH(8) break;
    default: P2_LAUNCH(16) break;
    }
#undef P2_LAUNCH
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

hipError_t launch_eval_literal_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                    int max_R, size_t lds_bytes, const unsigned long long* list, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const size_t lds = lds_bytes;
    if (lds == 0 || lds > kLdsLimit) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_eval_literal_list<MWV>, lds);                                                          \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_eval_literal_list<MWV>, dim3(blocks), dim3(kWave), lds, stream, queries, segs, n_segs, list);
    switch (mask_words(max_R)) {
    case 1: P2_LAUNCH(1) break;
    case 2: P2_LAUNCH(2) break;
    case 4: P2_LAUNCH(4) break;
    case 8: P2_LAUNCH(8) break;
    default: P2_LAUNCH(16) break;
    }
#undef P2_LAUNCH
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

hipError_t launch_cost_literal_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                    int max_R, size_t lds_bytes, const unsigned long long* sorted, p2_program* progs,
                                    double* costs, int only_missing, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const size_t lds = lds_bytes;
    if (lds == 0 || lds > kLdsLimit) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_cost_literal_list<MWV>, lds);                                                          \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_cost_literal_list<MWV>, dim3(blocks), dim3(kWave), lds, stream, queries, segs, n_segs, \
                           sorted, progs, costs, only_missing);
    switch (mask_words(max_R)) {
    case 1: P2_LAUNCH(1) break;
    case 2: P2_LAUNCH(2) break;
    case 4: P2_LAUNCH(4) break;
    case 8: P2_LAUNCH(8) break;
    default: P2_LAUNCH(16) break;
    }
#undef P2_LAUNCH
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

// The state of the class kernels holds up to 64 classes of rows; entries that would need more are evaluated
// on the full literal state.  A caller may lower the limit (p2_options.max_row_classes), which sends entries
// down that path.
// threads of a block of the full-state kernel where the state lies in global memory
constexpr int kFullThreads = 512;
// ... and of the class-state kernel where its masks do
constexpr int kClassThreads = 256;
static int row_class_cap(int asked) { return asked >= 1 && asked < 64 ? asked : 64; }

// Scratch of launch_front_classify_literal: the slices of the full-state kernel (where that state does not
// fit in LDS), the slices of the class kernel (likewise), the list of the entries left to the former.
namespace {
struct FrontLiteralScratch {
    size_t full_lds = 0, full_bytes = 0, cls_lds = 0, cls_bytes = 0, cls_per = 0, total = 0;
    unsigned full_blocks = 16384, cls_blocks = 16384;
};
FrontLiteralScratch front_literal_scratch(int R, int k, uint32_t n) {
    FrontLiteralScratch p;
    p.full_lds = front_literal_lds_bytes(R, k);
    if (p.full_lds == 0) p.full_bytes = literal_scratch_bytes(R, k, &p.full_blocks);
    const size_t cw = (size_t)cls_words(R, k, mask_words(R)) * 4;
    if (cw <= kLdsLimit) p.cls_lds = cw;
    else {
        // the tables stay in LDS, the masks go to global slices
        p.cls_lds = (size_t)cls_table_words(R, k) * 4;
        p.cls_per = ((size_t)cls_mask_words(R, k, mask_words(R)) * 4 + 255) / 256 * 256;
        p.cls_blocks = 2048;
        while (p.cls_blocks > 1 && p.cls_per * p.cls_blocks > ((size_t)8 << 30)) p.cls_blocks >>= 1;
        p.cls_bytes = p.cls_per * p.cls_blocks;
    }
    p.total = p.full_bytes + p.cls_bytes + ((size_t)n * 4 + 255) / 256 * 256;
    return p;
}
}  // namespace

size_t front_literal_scratch_bytes(int R, int k, uint32_t n) { return front_literal_scratch(R, k, n).total; }

hipError_t launch_front_classify_literal(const DevQuery* q, int R, int k, const FrontEntry* entries, uint32_t n,
                                         int parent_len, int goals_only, FrontSurvivor* surv, uint32_t surv_cap, FrontCounters* ctr,
                                         void* gscratch, int class_cap_asked, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (!gscratch) return hipErrorInvalidValue;
    const FrontLiteralScratch sc = front_literal_scratch(R, k, n);
    char* const base = static_cast<char*>(gscratch);
    uint32_t* const full_mem = sc.full_lds ? nullptr : reinterpret_cast<uint32_t*>(base);
    uint32_t* const cls_mem = sc.cls_bytes ? reinterpret_cast<uint32_t*>(base + sc.full_bytes) : nullptr;
    uint32_t* const over = reinterpret_cast<uint32_t*>(base + sc.full_bytes + sc.cls_bytes);
    const unsigned cls_blocks = sc.cls_blocks < n ? sc.cls_blocks : n, full_blocks = sc.full_blocks < n ? sc.full_blocks : n;
    const unsigned long long cls_words_per = sc.cls_per / 4;
    const unsigned long long full_words_per = sc.full_lds ? 0ull : sc.full_bytes / sc.full_blocks / 4;
    const int class_cap = row_class_cap(class_cap_asked);
    hipError_t e = hipSuccess;
    // first on the class state; what needs more classes than that holds, on the full literal state
#define P2_LAUNCH(MWV)                                                                                         \
    if (cls_mem) {                                                                                             \
        e = allow_big_lds(k_front_classify_classes<MWV, kClassThreads>, sc.cls_lds);                           \
        if (e == hipSuccess)                                                                                   \
            hipLaunchKernelGGL((k_front_classify_classes<MWV, kClassThreads>), dim3(cls_blocks), dim3(kClassThreads), sc.cls_lds, stream, q, entries, n, \
                               parent_len, goals_only, surv, surv_cap, ctr, over, cls_mem, cls_words_per, class_cap); \
    } else {                                                                                                   \
        e = allow_big_lds(k_front_classify_classes<MWV, kWave>, sc.cls_lds);                                   \
        if (e == hipSuccess)                                                                                   \
            hipLaunchKernelGGL((k_front_classify_classes<MWV, kWave>), dim3(cls_blocks), dim3(kWave), sc.cls_lds, stream, q, entries, n, \
                               parent_len, goals_only, surv, surv_cap, ctr, over, cls_mem, cls_words_per, class_cap); \
    }                                                                                                          \
    if (e == hipSuccess && sc.full_lds) {                                                                      \
        e = allow_big_lds(k_front_classify_literal<MWV, kWave>, sc.full_lds);                                  \
        if (e == hipSuccess)                                                                                   \
            hipLaunchKernelGGL((k_front_classify_literal<MWV, kWave>), dim3(full_blocks), dim3(kWave), sc.full_lds, stream, q, entries, n, \
                               over, &ctr->n_overflow, parent_len, goals_only, surv, surv_cap, ctr, full_mem, full_words_per); \
    } else if (e == hipSuccess) {                                                                              \
        hipLaunchKernelGGL((k_front_classify_literal<MWV, kFullThreads>), dim3(full_blocks), dim3(kFullThreads), 0, stream, q, entries, n, \
                           over, &ctr->n_overflow, parent_len, goals_only, surv, surv_cap, ctr, full_mem, full_words_per); \
    }
    switch (mask_words(R)) {
    case 1: P2_LAUNCH(1) break;
    case 2: P2_LAUNCH(2) break;
    case 4: P2_LAUNCH(4) break;
    case 8: P2_LAUNCH(8) break;
    default: P2_LAUNCH(16) break;
    }
#undef P2_LAUNCH
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

size_t literal_group_scratch_bytes(int max_R, int max_k, unsigned* blocks) {
    // up to 4096 blocks, each with its own global slice: the copy of a stem's class state, the full literal
    // state with its tables, the copy of a stem's full state (LDS holds the class state only: with the full
    // state beside it fewer blocks fit on a compute unit, and hardly any entry needs it)
    LitLayout lay(max_R, max_k, mask_words(max_R));
    const size_t state = (size_t)(lay.total_words() + front_lit_words(max_k));
    const size_t per = (((size_t)cls_backup_words(max_R, max_k, mask_words(max_R)) + state + (size_t)lay.s_words) * 4 + 255) / 256 * 256;
    unsigned b = 4096;
    while (b > 1 && per * b > ((size_t)8 << 30)) b >>= 1;
    *blocks = b;
    return per * b;
}

hipError_t launch_eval_literal_groups_auto(const DevQuery* queries, const int32_t* qlist, int n_q, int max_R, int max_k,
                                           void* gscratch, int class_cap_asked, hipStream_t stream) {
    if (n_q == 0) return hipSuccess;
    if (!gscratch || max_R > 64) return hipErrorInvalidValue;
    const size_t lds = (size_t)cls_words(max_R, max_k, mask_words(max_R)) * 4;
    unsigned blocks = 0;
    const unsigned long long gwords = literal_group_scratch_bytes(max_R, max_k, &blocks) / blocks / 4;
    const int cls_backup = cls_backup_words(max_R, max_k, mask_words(max_R));
    // (64 classes are all that power-of-two groups can produce)
    const int class_cap = row_class_cap(class_cap_asked);
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_eval_literal_groups_auto<MWV>, lds);                                                   \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_eval_literal_groups_auto<MWV>, dim3(blocks), dim3(kWave), lds, stream, queries, qlist, n_q, \
                           static_cast<uint32_t*>(gscratch), gwords, cls_backup, class_cap);
    switch (mask_words(max_R)) {              // reduction groups of at most 64 devices
    case 1: P2_LAUNCH(1) break;
    case 2: P2_LAUNCH(2) break;
    default: return hipErrorInvalidValue;
    }
#undef P2_LAUNCH
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace p2
