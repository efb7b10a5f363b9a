// Literal engine: the device-state semantics of Sec. 3.2 on the literal state of one reduction
// group -- R devices x k chunk rows, each row a mask of R contribution bits -- kept in LDS by
// one wavefront per candidate.  A step works on (group, row) items: an item reads the row of
// every member of its group, checks the rule's premises, and writes the members' new rows.
// The same code, with kCost set, recomputes a valid program and adds up its ring alpha-beta
// step times (hierarchical cost model, see p2.h).
#include "p2_device.h"

namespace p2 {

namespace {

constexpr int kWave = 64;
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

// One instruction on the literal state.  All 64 lanes call it with identical arguments.
// Returns false if a premise fails or nothing changes.  With kCost, *cost_lane (lane m = message
// size m) gets the step time added.
template <int MW, bool kCost>
__device__ bool lit_step(const DevQuery& q, const DevPattern& P, int op, const LitLds& L, int lane, double* cost_lane) {
    const int k = q.k, g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    const int kw = (k + 31) / 32;
    for (int i = lane; i < ng; i += kWave) { L.gcount[i] = 0; L.gflag[i] = 0; }
    for (int i = lane; i < ng * kw; i += kWave) L.gbits[i] = 0;
    if (op == OP_AG)
        for (int i = lane; i < q.R; i += kWave) L.devne[i] = 0;
    if (lane == 0) { L.flags[0] = 0; L.flags[1] = 0; }
    __syncthreads();

    const int items = ng * k;
    bool bad = false;
    for (int it = lane; it < items; it += kWave) {
        const int G = it / k, r = it - G * k;
        const int base = P.master ? G * gs : (G / s) * gs + (G % s);
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
    for (int G = lane; G < ng; G += kWave) {
        const uint32_t cnt = L.gcount[G];
        if (op == OP_AR || op == OP_RS || op == OP_RD) {
            if (op == OP_RS && cnt % (uint32_t)g != 0) L.flags[0] = 1;   // scatter: chunks must divide evenly
            if (cnt) L.flags[1] = 1;                                    // a group of empty devices is a no-op
        } else if (op == OP_AG) {
            const int base = P.master ? G * gs : (G / s) * gs + (G % s);
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
    for (int it = lane; it < items; it += kWave) {
        const int G = it / k, r = it - G * k;
        const int base = P.master ? G * gs : (G / s) * gs + (G % s);
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
__device__ inline void lit_init(const DevQuery& q, const LitLds& L, int lane) {
    // Sec. 3.5: device i holds column i in every row
    const int cells = q.R * q.k;
    for (int c = lane; c < cells; c += kWave) {
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
// goal, 3 = valid prefix.  C = number of row classes.  All 64 lanes call it with the same arguments.
template <int MW>
__device__ int lit_classify(const DevQuery& q, const DevPattern& P, int op, const LitLds& L, const FrontLit& X, int C,
                            const uint32_t* full, int lane) {
    const int k = q.k, g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    for (int i = lane; i < ng; i += kWave) { L.gcount[i] = 0; L.gflag[i] = 0; }
    if (lane == 0) { L.flags[0] = 0; L.flags[1] = 0; L.flags[2] = 0; }
    __syncthreads();
    const int items = ng * C;
    bool bad = false, notfull = false;
    for (int it = lane; it < items; it += kWave) {
        const int G = it / C, c = it - G * C;
        const int r = (int)X.reps[c];
        const int base = P.master ? G * gs : (G / s) * gs + (G % s);
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
        for (int d = lane; d < q.R; d += kWave) {
            const bool part = d % s == 0 && d / gs < ng;
            if (!part && !X.devfull[d]) L.flags[2] = 1;
        }
    __syncthreads();
    for (int G = lane; G < ng; G += kWave) {
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
// and keep the pointer only if the two rows really are equal.  Returns the number of classes.
template <int MW>
__device__ inline int row_classes(const DevQuery& q, const LitLds& L, const FrontLit& X, const uint32_t* full, int lane) {
    const int R = q.R, k = q.k;
    for (int r = lane; r < k; r += kWave) {
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
    for (int r = lane; r < k; r += kWave) {
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
    int C = 0;
    for (int r0 = 0; r0 < k; r0 += kWave) {
        const int r = r0 + lane;
        const bool is = r < k && X.rep[r] == (uint32_t)r;
        const unsigned long long bal = __ballot(is);
        if (is) X.reps[C + __popcll(bal & ((1ull << lane) - 1ull))] = (uint32_t)r;
        C += __popcll(bal);
        if (r < k) atomicAdd(&X.multr[X.rep[r]], 1u);
    }
    __syncthreads();
    for (int d = lane; d < R; d += kWave) {
        bool any = false, all = true;
        for (int c = 0; c < C; ++c) {
            const uint32_t* x = L.S + (d * k + (int)X.reps[c]) * MW;
#pragma unroll
            for (int w = 0; w < MW; ++w) { any |= x[w] != 0; all &= x[w] == full[w]; }
        }
        X.devany[d] = any; X.devfull[d] = all;
    }
    __syncthreads();
    return C;
}

template <int MW>
__global__ __launch_bounds__(kWave) void k_front_classify_literal(const DevQuery* __restrict__ qp,
                                                                  const FrontEntry* __restrict__ entries, uint32_t n_entries,
                                                                  int parent_len, FrontSurvivor* __restrict__ surv,
                                                                  uint32_t surv_cap, FrontCounters* __restrict__ ctr,
                                                                  uint32_t* __restrict__ gscratch, unsigned long long gwords) {
    extern __shared__ uint32_t lds[];
    const DevQuery& q = *qp;
    const int lane = threadIdx.x;
    const LitLds L = carve(gscratch ? gscratch + (size_t)blockIdx.x * gwords : lds, q.R, q.k, MW);
    const FrontLit X = carve_front(L.flags + 4, q.k);
    const int R = q.R, k = q.k, I = q.alphabet;
    uint32_t full[MW];
#pragma unroll
    for (int w = 0; w < MW; ++w) {
        const int bits = R - 32 * w;
        full[w] = bits >= 32 ? 0xffffffffu : bits > 0 ? ((1u << bits) - 1u) : 0u;
    }
    unsigned long long steps = 0, members = 0;
    for (uint32_t e = blockIdx.x; e < n_entries; e += gridDim.x) {
        const unsigned long long digits = entries[e].digits;
        lit_init<MW>(q, L, lane);
        for (int t = 0; t < parent_len; ++t) {
            const uint32_t ins = q.instr_of_digit[(int)((digits >> (9 * t)) & 511ull)];
            lit_step<MW, false>(q, q.pat[ins >> 3], (int)(ins & 7u), L, lane, nullptr);
        }
        const int C = row_classes<MW>(q, L, X, full, lane);
        for (int a = 0; a < I; ++a) {
            const uint32_t ins = q.instr_of_digit[a];
            const DevPattern& P = q.pat[ins >> 3];
            const int code = lit_classify<MW>(q, P, (int)(ins & 7u), L, X, C, full, lane);
            ++steps;
            members += (unsigned long long)(P.n_groups * P.g);
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

// The groups that the shared-prefix kernel has just handed over, found on the device: those of the queries
// qlist[0 .. n_q), read from their counters and lists.  A unit of work is one (group, part) pair; blocks
// stride over the units.  States that fit in LDS live there; larger ones in the block's slice of a global buffer.  This lets the host queue the kernel
// right behind the evaluation, without waiting for the counts.  A query whose list overflowed is left
// out (the host grows the list and runs the query again).  Few groups: up to 8 blocks share one.
template <int MW>
__global__ __launch_bounds__(kWave) void k_eval_literal_groups_auto(const DevQuery* __restrict__ queries,
                                                                    const int32_t* __restrict__ qlist, int n_q,
                                                                    uint32_t* __restrict__ gscratch,
                                                                    unsigned long long gwords, int state_in_lds) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x;
    // the block's slice of the global buffer: the state itself where it does not fit in LDS, then the stem copy
    uint32_t* const slice = gscratch + (size_t)blockIdx.x * gwords;
    uint32_t* const mem = state_in_lds ? lds : slice;
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
        uint32_t full[MW];
#pragma unroll
        for (int w = 0; w < MW; ++w) {
            const int bits = q.R - 32 * w;
            full[w] = bits >= 32 ? 0xffffffffu : bits > 0 ? ((1u << bits) - 1u) : 0u;
        }
        unsigned long long steps = 0, members = 0;
        const unsigned long long entry = q.rerun_idx[e - own_lo];
        if (entry & kStemEntry) {
            LitLayout lay(q.R, q.k, MW);
            uint32_t* const backup = state_in_lds ? slice : slice + lay.total_words() + front_lit_words(q.k);
            literal_stem<MW>(q, entry & kEntryIndexMask, (int)((entry >> kStemCountShift) & 0x7ffull), L, X, full, lane, part,
                             (int)parts, backup, steps, members);
        } else {
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

inline int mask_words(int R) { return R <= 32 ? 1 : R <= 64 ? 2 : R <= 128 ? 4 : R <= 256 ? 8 : 16; }

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
                                    int max_R, int max_k, const unsigned long long* list, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const size_t lds = literal_lds_bytes(max_R, max_k);
    if (lds == 0) return hipErrorInvalidValue;
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
                                    int max_R, int max_k, const unsigned long long* sorted, p2_program* progs,
                                    double* costs, int only_missing, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const size_t lds = literal_lds_bytes(max_R, max_k);
    if (lds == 0) return hipErrorInvalidValue;
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

hipError_t launch_front_classify_literal(const DevQuery* q, int R, int k, const FrontEntry* entries, uint32_t n,
                                         int parent_len, FrontSurvivor* surv, uint32_t surv_cap, FrontCounters* ctr,
                                         void* gscratch, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    size_t lds = front_literal_lds_bytes(R, k);
    unsigned blocks = n < 16384u ? n : 16384u;
    unsigned long long gwords = 0;
    if (lds == 0) {
        if (!gscratch) return hipErrorInvalidValue;
        unsigned nb = 0;
        gwords = literal_scratch_bytes(R, k, &nb) / nb / 4;
        blocks = nb < n ? nb : n;
    } else gscratch = nullptr;
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_front_classify_literal<MWV>, lds);                                                     \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_front_classify_literal<MWV>, dim3(blocks), dim3(kWave), lds, stream, q, entries, n, \
                           parent_len, surv, surv_cap, ctr, static_cast<uint32_t*>(gscratch), gwords);
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
    // up to 4096 blocks, each with its own global slice: the copy of a stem's state, and in front of it
    // the state itself with its tables where that does not fit in LDS
    LitLayout lay(max_R, max_k, mask_words(max_R));
    const size_t state = front_literal_lds_bytes(max_R, max_k) != 0 ? 0 : (size_t)(lay.total_words() + front_lit_words(max_k));
    const size_t per = ((state + (size_t)lay.s_words) * 4 + 255) / 256 * 256;
    unsigned b = 4096;
    while (b > 1 && per * b > ((size_t)8 << 30)) b >>= 1;
    *blocks = b;
    return per * b;
}

hipError_t launch_eval_literal_groups_auto(const DevQuery* queries, const int32_t* qlist, int n_q, int max_R, int max_k,
                                           void* gscratch, hipStream_t stream) {
    if (n_q == 0) return hipSuccess;
    const size_t lds = front_literal_lds_bytes(max_R, max_k);
    if (!gscratch) return hipErrorInvalidValue;
    unsigned blocks = 0;
    const unsigned long long gwords = literal_group_scratch_bytes(max_R, max_k, &blocks) / blocks / 4;
    const int state_in_lds = lds != 0 ? 1 : 0;
    hipError_t e = hipSuccess;
#define P2_LAUNCH(MWV)                                                                                         \
    e = allow_big_lds(k_eval_literal_groups_auto<MWV>, lds);                                                   \
    if (e == hipSuccess)                                                                                       \
        hipLaunchKernelGGL(k_eval_literal_groups_auto<MWV>, dim3(blocks), dim3(kWave), lds, stream, queries, qlist, n_q, \
                           static_cast<uint32_t*>(gscratch), gwords, state_in_lds);
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
