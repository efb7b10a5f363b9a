// Compact engine: one candidate per lane.
//
// From the init state of Sec. 3.5 every rule of Sec. 3.2 keeps a device's non-empty rows equal to
// each other as long as no AllGather joins members whose rows carry different column sets: the
// sum of AllReduce / ReduceScatter / Reduce is the same in every row, scatter and Reduce only
// drop rows, Broadcast copies the root.  So a device state is held as ONE chunk set (k bits: which
// rows are non-empty) plus ONE contribution mask (R bits: the columns of each of those rows).
// An AllGather of members with different masks leaves that form; the lane then reports the
// candidate for re-evaluation by the literal engine, so results stay exact.
//
// A lane keeps the R (chunk set, mask) pairs of its candidate in LDS, word-interleaved across
// lanes (word w of lane l at w * LS + l: every lane its own bank).  No lane ever reads another
// lane's state, so the kernel needs no barrier.  A step is two flat loops over the participating
// devices of the instruction's pattern in group-major order: pass A folds the members of a
// group and checks the rule's premises, leaving the group's result in its first member's slot;
// pass B writes every member's new pair from that slot.  The rule-specific parts are selects,
// not branches, because the 64 lanes of a wavefront hold consecutive candidates whose last
// instructions all differ.
#include "p2_device.h"

namespace p2 {

hipError_t launch_cost_compact(const DevQuery* q, int R, int k, const unsigned long long* sorted, uint32_t n,
                               p2_program* out_prog, double* out_cost, hipStream_t stream);

namespace {

constexpr int kWave = 64;
constexpr size_t kLdsBudget = 160 * 1024 - 4096;

template <int N>
struct Words {
    uint32_t w[N];
};
template <int N>
__device__ inline bool is_zero(const Words<N>& a) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i];
    return o == 0;
}
template <int N>
__device__ inline bool differs(const Words<N>& a, const Words<N>& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i] ^ b.w[i];
    return o != 0;
}
template <int N>
__device__ inline bool intersects(const Words<N>& a, const Words<N>& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i] & b.w[i];
    return o != 0;
}
template <int N>
__device__ inline bool not_subset(const Words<N>& a, const Words<N>& b) {   // a has a bit outside b
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i] & ~b.w[i];
    return o != 0;
}
template <int N>
__device__ inline int popcount(const Words<N>& a) {
    int c = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) c += __popc(a.w[i]);
    return c;
}
template <int N>
__device__ inline Words<N> full_mask(int bits) {
    Words<N> f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int b = bits - 32 * i;
        f.w[i] = b >= 32 ? 0xffffffffu : b > 0 ? ((1u << b) - 1u) : 0u;
    }
    return f;
}

// mask of the n lowest set bits of v, for n < popc(v)
__device__ inline uint32_t lowest_in_word(uint32_t v, int n) {
    uint32_t pos = 0;
#pragma unroll
    for (uint32_t b = 16; b > 0; b >>= 1) {
        const int t = __popc(v & ((1u << (pos + b)) - 1u));
        if (t <= n) pos += b;
    }
    return v & ((1u << pos) - 1u);
}
// the n lowest set bits of x (all of x if it has no more than n)
template <int N>
__device__ inline Words<N> lowest_n(const Words<N>& x, int n) {
    Words<N> o;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = __popc(x.w[i]);
        if (n >= c) { o.w[i] = x.w[i]; n -= c; }
        else { o.w[i] = lowest_in_word(x.w[i], n); n = 0; }
    }
    return o;
}

template <int KW, int MW>
struct Slot {
    Words<KW> r;   // chunk set
    Words<MW> m;   // contribution mask of every non-empty row
};
template <int KW, int MW>
__device__ inline Slot<KW, MW> load_slot(const uint32_t* my, int LS, int dev) {
    const uint32_t* p = my + dev * (KW + MW) * LS;
    Slot<KW, MW> s;
#pragma unroll
    for (int i = 0; i < KW; ++i) s.r.w[i] = p[i * LS];
#pragma unroll
    for (int i = 0; i < MW; ++i) s.m.w[i] = p[(KW + i) * LS];
    return s;
}
template <int KW, int MW>
__device__ inline void store_slot(uint32_t* my, int LS, int dev, const Words<KW>& r, const Words<MW>& m) {
    uint32_t* p = my + dev * (KW + MW) * LS;
#pragma unroll
    for (int i = 0; i < KW; ++i) p[i * LS] = r.w[i];
#pragma unroll
    for (int i = 0; i < MW; ++i) p[(KW + i) * LS] = m.w[i];
}

struct PatLds {
    int g, s, master, n_part;     // n_part = participating devices = groups * g
};

struct GroupWalk {                // group-major walk over the participating devices of a pattern
    int p, lo, hib, dev;
    __device__ inline void start() { p = 0; lo = 0; hib = 0; dev = 0; }
    __device__ inline int root() const { return hib + lo; }
    __device__ inline bool next(const PatLds& P) {      // returns true when the group is complete
        ++p;
        dev += P.s;
        return p == P.g;
    }
    __device__ inline void next_group(const PatLds& P) {
        p = 0;
        const int gs = P.g * P.s;
        if (P.master) hib += gs;
        else if (++lo == P.s) { lo = 0; hib += gs; }
        dev = hib + lo;
    }
};

enum : int { STEP_INVALID = 0, STEP_OK = 1, STEP_GIVE_UP = 2 };

// One instruction for this lane's candidate.  cost_* only with kCost.
template <int KW, int MW, bool kCost>
__device__ inline int compact_step(uint32_t* my, int LS, const PatLds P, int op, const DevQuery& q, const DevPattern* dp,
                                   double* sum_alpha, double* sum_beta) {
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    bool bad = false, changed = false, give_up = false;
    GroupWalk wk;
    wk.start();
    Slot<KW, MW> first, acc;
    bool eq = true, disj_m = true, disj_r = true, all_ne = true, same_m = true, sub = true, strict = false;
    // ---- pass A: fold each group, check the premises, leave the result in the first member's slot
    for (int j = 0; j < P.n_part; ++j) {
        const Slot<KW, MW> cur = load_slot<KW, MW>(my, LS, wk.dev);
        if (wk.p == 0) {
            first = cur; acc = cur;
            eq = true; disj_m = true; disj_r = true; same_m = true; sub = true; strict = false;
            all_ne = !is_zero(cur.r);
        } else {
            eq &= !differs(cur.r, first.r);               // same chunks on every member
            disj_m &= !intersects(cur.m, acc.m);          // no contribution reduced twice
            disj_r &= !intersects(cur.r, acc.r);          // AllGather: chunks held once
            all_ne &= !is_zero(cur.r);                    // AllGather: nobody empty
            same_m &= !differs(cur.m, first.m);
            sub &= !not_subset(cur.r, first.r) && !not_subset(cur.m, first.m);   // Broadcast: root knows more
            strict |= differs(cur.r, first.r) || differs(cur.m, first.m);
#pragma unroll
            for (int i = 0; i < KW; ++i) acc.r.w[i] |= cur.r.w[i];
#pragma unroll
            for (int i = 0; i < MW; ++i) acc.m.w[i] |= cur.m.w[i];
        }
        if (wk.next(P)) {
            const int root = wk.root();
            if (red) {
                bad |= !eq || !disj_m;
                const bool ne = !is_zero(first.r);
                changed |= ne;                            // a group of empty devices is a no-op
                if (op == OP_RS) {
                    const int rows = popcount(first.r);
                    bad |= (rows / P.g) * P.g != rows;    // scatter needs the chunks to divide evenly
                }
                store_slot<KW, MW>(my, LS, root, first.r, acc.m);
            } else if (op == OP_AG) {
                bad |= !all_ne || !disj_r;
                give_up |= !same_m;                       // rows with different column sets: not this form
                changed = true;
                store_slot<KW, MW>(my, LS, root, acc.r, first.m);
            } else {
                bad |= !sub || !strict;                   // information increase
                changed = true;
            }
            wk.next_group(P);
        }
    }
    if (bad || !changed) return STEP_INVALID;
    if (give_up) return STEP_GIVE_UP;

    if (kCost) {
        // ring alpha-beta time of the step: the first slot of a group now holds the chunk set that
        // sets its bytes (common rows / rows after the gather / the root's rows)
        double best = 0.0;
        for (int row = dp->row_begin; row < dp->row_end; ++row) {
            long long dot = 0;
            for (int e = q.row_ptr[row]; e < q.row_ptr[row + 1]; ++e) {
                const uint32_t ent = q.entries[e];
                const Slot<KW, MW> s = load_slot<KW, MW>(my, LS, (int)entry_base(ent));
                dot += (long long)entry_cnt(ent) * (long long)popcount(s.r);
            }
            best = fmax(best, (double)dot * q.inv_bw[q.row_level[row]]);
        }
        const double gm1 = (double)(P.g - 1);
        const double ring_steps = (op == OP_AR) ? 2.0 * gm1 : gm1;
        const double mult = (op == OP_AR) ? 2.0 * gm1 / (double)P.g : (op == OP_RS || op == OP_AG) ? gm1 / (double)P.g : 1.0;
        *sum_alpha += ring_steps * q.alpha[dp->span_level];
        *sum_beta += (mult / (double)q.k) * best;
    }

    // ---- pass B: every member's new pair from the group's slot
    wk.start();
    Slot<KW, MW> grp;
    Words<KW> prev;
    int per = 0;
    for (int j = 0; j < P.n_part; ++j) {
        if (wk.p == 0) {
            grp = load_slot<KW, MW>(my, LS, wk.dev);
            if (op == OP_RS) {
                per = popcount(grp.r) / P.g;
#pragma unroll
                for (int i = 0; i < KW; ++i) prev.w[i] = 0;
            }
        }
        Words<KW> nr = grp.r;
        Words<MW> nm = grp.m;
        if (op == OP_RS) {
            // rank p keeps the p-th block of `per` chunks in ascending order
            const Words<KW> upto = lowest_n(grp.r, (wk.p + 1) * per);
#pragma unroll
            for (int i = 0; i < KW; ++i) { nr.w[i] = upto.w[i] & ~prev.w[i]; prev.w[i] = upto.w[i]; }
        } else if (op == OP_RD && wk.p != 0) {
#pragma unroll
            for (int i = 0; i < KW; ++i) nr.w[i] = 0;
#pragma unroll
            for (int i = 0; i < MW; ++i) nm.w[i] = 0;
        }
        store_slot<KW, MW>(my, LS, wk.dev, nr, nm);
        if (wk.next(P)) wk.next_group(P);
    }
    return STEP_OK;
}

template <int KW, int MW>
__device__ inline void compact_init(uint32_t* my, int LS, int R, int k) {
    const Words<KW> all_rows = full_mask<KW>(k);
    for (int d = 0; d < R; ++d) {
        Words<MW> m;
#pragma unroll
        for (int i = 0; i < MW; ++i) m.w[i] = (i == (d >> 5)) ? (1u << (d & 31)) : 0u;
        store_slot<KW, MW>(my, LS, d, all_rows, m);
    }
}
template <int KW, int MW>
__device__ inline bool compact_is_goal(const uint32_t* my, int LS, int R, int k) {
    const Words<KW> all_rows = full_mask<KW>(k);
    const Words<MW> all_cols = full_mask<MW>(R);
    bool ok = true;
    for (int d = 0; d < R; ++d) {
        const Slot<KW, MW> s = load_slot<KW, MW>(my, LS, d);
        ok &= !differs(s.r, all_rows) && !differs(s.m, all_cols);
    }
    return ok;
}

__device__ inline void load_patterns(const DevQuery& q, PatLds* spat, uint16_t* sdig) {
    for (int i = threadIdx.x; i < q.n_patterns; i += kWave) {
        PatLds p;
        p.g = q.pat[i].g; p.s = q.pat[i].s; p.master = q.pat[i].master; p.n_part = q.pat[i].n_groups * q.pat[i].g;
        spat[i] = p;
    }
    for (int i = threadIdx.x; i < q.alphabet; i += kWave) sdig[i] = q.instr_of_digit[i];
    __syncthreads();
}

// Flat evaluation: block b finds its segment (query, length), unranks the digits of its first
// candidate once, and walks `iters` x LS consecutive candidates, one per lane.
template <int KW, int MW>
__global__ __launch_bounds__(kWave) void k_eval_compact(const DevQuery* __restrict__ queries,
                                                        const DevSegment* __restrict__ segs, int n_segs, int LS) {
    extern __shared__ uint32_t lds[];
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ uint16_t sdig[kMaxPatterns * 5];
    int a = 0, b = n_segs - 1;                  // last segment whose first_block <= blockIdx.x
    while (a < b) {
        const int mid = (a + b + 1) >> 1;
        if (segs[mid].first_block <= blockIdx.x) a = mid; else b = mid - 1;
    }
    const DevSegment seg = segs[a];
    const DevQuery& q = queries[seg.query];
    load_patterns(q, spat, sdig);
    const int lane = threadIdx.x;
    uint32_t* my = lds + lane;
    const int len = seg.len;
    const uint32_t I = (uint32_t)q.alphabet;
    const unsigned long long off0 = (unsigned long long)(blockIdx.x - seg.first_block) * (unsigned long long)(seg.iters * LS);
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
    unsigned long long steps = 0;
    for (int it = 0; it < seg.iters; ++it) {
        const uint32_t add = (uint32_t)(it * LS + lane);
        const unsigned long long off = off0 + add;
        bool alive = lane < LS && off < seg.count;
        if (!__any(alive)) break;
        // this lane's instructions: digits of d0 + add carried through base I, 9 bits per instruction
        unsigned long long prog = 0;
        uint32_t carry = add;
#pragma unroll
        for (int t = P2_MAX_LEN - 1; t >= 0; --t) {
            if (t < len) {
                const uint32_t v = d0[t] + carry;
                carry = __umulhi(v, q.magic_alphabet);
                prog = (prog << 9) | sdig[v - carry * I];
            }
        }
        if (alive) compact_init<KW, MW>(my, LS, q.R, q.k);
        bool give_up = false;
        uint32_t ran = 0;
        for (int t = 0; t < len; ++t) {
            if (!__any(alive)) break;
            if (alive) {
                const uint32_t ins = (uint32_t)(prog >> (9 * t)) & 511u;
                ++ran;
                const int rc = compact_step<KW, MW, false>(my, LS, spat[ins >> 3], (int)(ins & 7u), q, nullptr, nullptr, nullptr);
                alive = rc == STEP_OK;
                give_up = rc == STEP_GIVE_UP;
            }
        }
        if (alive && compact_is_goal<KW, MW>(my, LS, q.R, q.k)) {
            const uint32_t pos = atomicAdd(&q.counters->n_valid, 1u);
            if (pos < q.valid_cap) q.valid_idx[pos] = seg.first_index + off;
        }
        if (give_up) {
            // the literal engine evaluates (and counts) this candidate from its first instruction
            const uint32_t pos = atomicAdd(&q.counters->n_rerun, 1u);
            if (pos < q.rerun_cap) q.rerun_idx[pos] = seg.first_index + off;
        } else {
            steps += ran;
        }
    }
    for (int o = 32; o > 0; o >>= 1) steps += __shfl_xor(steps, o, kWave);
    if (lane == 0 && steps) atomicAdd(&q.counters->steps, steps);
}

// Cost of the valid programs of one query: lane i re-runs sorted[i] with the cost terms on.
template <int KW, int MW>
__global__ __launch_bounds__(kWave) void k_cost_compact(const DevQuery* __restrict__ qp,
                                                        const unsigned long long* __restrict__ sorted, uint32_t n,
                                                        p2_program* __restrict__ out_prog, double* __restrict__ out_cost,
                                                        int LS) {
    extern __shared__ uint32_t lds[];
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ uint16_t sdig[kMaxPatterns * 5];
    const DevQuery& q = *qp;
    load_patterns(q, spat, sdig);
    const int lane = threadIdx.x;
    uint32_t* my = lds + lane;
    const uint32_t i = blockIdx.x * (uint32_t)LS + (uint32_t)lane;
    if (lane >= LS || i >= n) return;
    const unsigned long long idx = sorted[i];
    int len = 1;
    while (len < q.max_len && idx >= q.base[len + 1]) ++len;
    unsigned long long prog = 0;
    {
        unsigned long long rem = idx - q.base[len];
        const unsigned long long I = (unsigned long long)q.alphabet;
        for (int t = len - 1; t >= 0; --t) {
            const unsigned long long nx = rem / I;
            prog = (prog << 9) | sdig[(uint32_t)(rem - nx * I)];
            rem = nx;
        }
    }
    compact_init<KW, MW>(my, LS, q.R, q.k);
    double sum_alpha = 0.0, sum_beta = 0.0;
    bool ok = true;
    p2_program pr;
    pr.index = idx;
    pr.len = (uint8_t)len;
    for (int t = 0; t < 7; ++t) pr.instr[t] = 0;
    for (int t = 0; t < len; ++t) {
        const uint32_t ins = (uint32_t)(prog >> (9 * t)) & 511u;
        pr.instr[t] = (uint8_t)((ins >> 3) * 5u + (ins & 7u));
        if (ok) ok = compact_step<KW, MW, true>(my, LS, spat[ins >> 3], (int)(ins & 7u), q, &q.pat[ins >> 3],
                                                &sum_alpha, &sum_beta) == STEP_OK;
    }
    out_prog[i] = pr;
    for (int m = 0; m < q.n_msg; ++m)
        out_cost[(size_t)i * q.n_msg + m] = ok ? sum_alpha + q.msg_bytes[m] * sum_beta : __longlong_as_double(0x7ff8000000000000ll);
}

inline int round_words(int bits) {
    const int w = (bits + 31) / 32;
    return w <= 1 ? 1 : w <= 2 ? 2 : w <= 4 ? 4 : w <= 8 ? 8 : 16;
}

template <typename F>
hipError_t allow_lds(F func, size_t bytes) {
    if (bytes <= 32 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(func), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int KW>
hipError_t eval_mw(int MW, const DevQuery* queries, const DevSegment* segs, int n_segs, unsigned blocks, int LS, size_t lds,
                   hipStream_t stream) {
    hipError_t e = hipSuccess;
#define P2_GO(MWV)                                                                                                        \
    e = allow_lds(k_eval_compact<KW, MWV>, lds);                                                                          \
    if (e == hipSuccess) hipLaunchKernelGGL((k_eval_compact<KW, MWV>), dim3(blocks), dim3(kWave), lds, stream, queries, segs, n_segs, LS);
    switch (MW) {
    case 1: P2_GO(1) break;
    case 2: P2_GO(2) break;
    case 4: P2_GO(4) break;
    case 8: P2_GO(8) break;
    default: P2_GO(16) break;
    }
#undef P2_GO
    return e != hipSuccess ? e : hipGetLastError();
}
template <int KW>
hipError_t cost_mw(int MW, const DevQuery* q, const unsigned long long* sorted, uint32_t n, p2_program* out_prog,
                   double* out_cost, unsigned blocks, int LS, size_t lds, hipStream_t stream) {
    hipError_t e = hipSuccess;
#define P2_GO(MWV)                                                                                                        \
    e = allow_lds(k_cost_compact<KW, MWV>, lds);                                                                          \
    if (e == hipSuccess) hipLaunchKernelGGL((k_cost_compact<KW, MWV>), dim3(blocks), dim3(kWave), lds, stream, q, sorted, n, out_prog, out_cost, LS);
    switch (MW) {
    case 1: P2_GO(1) break;
    case 2: P2_GO(2) break;
    case 4: P2_GO(4) break;
    case 8: P2_GO(8) break;
    default: P2_GO(16) break;
    }
#undef P2_GO
    return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace

int compact_lanes(int R, int k) {
    const size_t per_lane = (size_t)R * (size_t)(round_words(k) + round_words(R)) * 4;
    int lanes = 64;
    while (lanes >= 1 && per_lane * (size_t)lanes > kLdsBudget) lanes >>= 1;
    return lanes;       // 0 if even one candidate does not fit
}

hipError_t launch_eval_compact(const DevQuery* queries, const DevSegment* segs, int n_segs, unsigned total_blocks,
                               int max_R, int max_k, hipStream_t stream) {
    if (n_segs == 0 || total_blocks == 0) return hipSuccess;
    const int LS = compact_lanes(max_R, max_k);
    if (LS == 0) return hipErrorInvalidValue;
    const int KW = round_words(max_k), MW = round_words(max_R);
    const size_t lds = (size_t)max_R * (size_t)(KW + MW) * 4 * (size_t)LS;
    switch (KW) {
    case 1: return eval_mw<1>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    case 2: return eval_mw<2>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    case 4: return eval_mw<4>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    case 8: return eval_mw<8>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    default: return eval_mw<16>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    }
}

hipError_t launch_cost_compact(const DevQuery* q, int R, int k, const unsigned long long* sorted, uint32_t n,
                               p2_program* out_prog, double* out_cost, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const int LS = compact_lanes(R, k);
    if (LS == 0) return hipErrorInvalidValue;
    const int KW = round_words(k), MW = round_words(R);
    const size_t lds = (size_t)R * (size_t)(KW + MW) * 4 * (size_t)LS;
    const unsigned blocks = (n + (unsigned)LS - 1) / (unsigned)LS;
    switch (KW) {
    case 1: return cost_mw<1>(MW, q, sorted, n, out_prog, out_cost, blocks, LS, lds, stream);
    case 2: return cost_mw<2>(MW, q, sorted, n, out_prog, out_cost, blocks, LS, lds, stream);
    case 4: return cost_mw<4>(MW, q, sorted, n, out_prog, out_cost, blocks, LS, lds, stream);
    case 8: return cost_mw<8>(MW, q, sorted, n, out_prog, out_cost, blocks, LS, lds, stream);
    default: return cost_mw<16>(MW, q, sorted, n, out_prog, out_cost, blocks, LS, lds, stream);
    }
}

}  // namespace p2
