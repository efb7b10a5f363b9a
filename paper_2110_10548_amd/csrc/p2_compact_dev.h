// Device code of the compact state form, shared by the flat evaluator (p2_compact.hip) and the
// frontier evaluator (p2_frontier.hip).  See p2_compact.hip for the description of the form.
#pragma once
#include "p2_device.h"

namespace p2 {
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
struct Lay {
    static constexpr int WPD = KW + MW;
    static constexpr int WS = (WPD == 2 || WPD == 4) ? WPD : (WPD | 1);   // words between lanes
};
// `my` points at this lane's pair of device 0; device d is at my + d * dstride (dstride = LS * WS).
template <int KW, int MW>
__device__ inline Slot<KW, MW> load_slot(const uint32_t* my, int dstride, int dev) {
    const uint32_t* p = my + dev * dstride;
    Slot<KW, MW> s;
    if constexpr (KW == 1 && MW == 1) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        s.r.w[0] = v.x; s.m.w[0] = v.y;
    } else if constexpr (KW + MW == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t t[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < KW; ++i) s.r.w[i] = t[i];
#pragma unroll
        for (int i = 0; i < MW; ++i) s.m.w[i] = t[KW + i];
    } else {
#pragma unroll
        for (int i = 0; i < KW; ++i) s.r.w[i] = p[i];
#pragma unroll
        for (int i = 0; i < MW; ++i) s.m.w[i] = p[KW + i];
    }
    return s;
}
template <int KW, int MW>
__device__ inline void store_slot(uint32_t* my, int dstride, int dev, const Words<KW>& r, const Words<MW>& m) {
    uint32_t* p = my + dev * dstride;
    if constexpr (KW == 1 && MW == 1) {
        *reinterpret_cast<uint2*>(p) = make_uint2(r.w[0], m.w[0]);
    } else if constexpr (KW + MW == 4) {
        uint32_t t[4];
#pragma unroll
        for (int i = 0; i < KW; ++i) t[i] = r.w[i];
#pragma unroll
        for (int i = 0; i < MW; ++i) t[KW + i] = m.w[i];
        *reinterpret_cast<uint4*>(p) = make_uint4(t[0], t[1], t[2], t[3]);
    } else {
#pragma unroll
        for (int i = 0; i < KW; ++i) p[i] = r.w[i];
#pragma unroll
        for (int i = 0; i < MW; ++i) p[KW + i] = m.w[i];
    }
}
template <int KW, int MW>
__device__ inline void store_mask(uint32_t* my, int dstride, int dev, const Words<MW>& m) {
    uint32_t* p = my + dev * dstride + KW;
#pragma unroll
    for (int i = 0; i < MW; ++i) p[i] = m.w[i];
}
template <int KW, int MW>
__device__ inline void store_rows(uint32_t* my, int dstride, int dev, const Words<KW>& r) {
    uint32_t* p = my + dev * dstride;
#pragma unroll
    for (int i = 0; i < KW; ++i) p[i] = r.w[i];
}
template <int N>
__device__ inline uint32_t fold_xor(const Words<N>& a, const Words<N>& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i] ^ b.w[i];
    return o;
}
template <int N>
__device__ inline uint32_t fold_and(const Words<N>& a, const Words<N>& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i] & b.w[i];
    return o;
}
template <int N>
__device__ inline uint32_t fold_andn(const Words<N>& a, const Words<N>& b) {   // bits of a outside b
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i] & ~b.w[i];
    return o;
}
template <int N>
__device__ inline uint32_t fold_or(const Words<N>& a) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) o |= a.w[i];
    return o;
}

struct PatLds {
    int g, s, master, n_groups;   // participating devices = n_groups * g
};
__device__ inline int div_small(int v, int d) {      // v / d for 0 <= v <= 512, 1 <= d <= 512, exact
    return (int)__fdividef((float)v + 0.5f, (float)d);
}

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

// One instruction, the same (pattern, rule) in every live lane: g, s, master, n_groups are scalars.
template <int KW, int MW>
__device__ inline int step_uniform(uint32_t* my, int dstride, int g, int s, int master, int n_groups, int op) {
    const int gs = g * s;
    uint32_t badx = 0;          // any bit set: a premise failed
    bool changed = false, give_up = false;
    int lo = 0, hib = 0;
    for (int G = 0; G < n_groups; ++G) {
        const int base = hib + lo;
        const Slot<KW, MW> first = load_slot<KW, MW>(my, dstride, base);
        if (op == OP_AR || op == OP_RS || op == OP_RD) {
            // premises: same chunks on every member, no contribution reduced twice
            Words<MW> accm = first.m;
            for (int p = 1; p < g; ++p) {
                const Slot<KW, MW> cur = load_slot<KW, MW>(my, dstride, base + p * s);
                badx |= fold_xor(cur.r, first.r) | fold_and(cur.m, accm);
#pragma unroll
                for (int i = 0; i < MW; ++i) accm.w[i] |= cur.m.w[i];
            }
            changed |= fold_or(first.r) != 0;               // a group of empty devices is a no-op
            if (op == OP_AR) {
                for (int p = 0; p < g; ++p) store_mask<KW, MW>(my, dstride, base + p * s, accm);
            } else if (op == OP_RD) {
                store_mask<KW, MW>(my, dstride, base, accm);
                Words<KW> zr; Words<MW> zm;
#pragma unroll
                for (int i = 0; i < KW; ++i) zr.w[i] = 0;
#pragma unroll
                for (int i = 0; i < MW; ++i) zm.w[i] = 0;
                for (int p = 1; p < g; ++p) store_slot<KW, MW>(my, dstride, base + p * s, zr, zm);
            } else {
                // scatter: the chunks must divide evenly; rank p keeps the p-th block in ascending order
                const int rows = popcount(first.r);
                const int per = div_small(rows, g);
                badx |= (uint32_t)(per * g != rows);
                Words<KW> prev;
#pragma unroll
                for (int i = 0; i < KW; ++i) prev.w[i] = 0;
                for (int p = 0; p < g; ++p) {
                    const Words<KW> upto = lowest_n(first.r, (p + 1) * per);
                    Words<KW> nr;
#pragma unroll
                    for (int i = 0; i < KW; ++i) { nr.w[i] = upto.w[i] & ~prev.w[i]; prev.w[i] = upto.w[i]; }
                    store_slot<KW, MW>(my, dstride, base + p * s, nr, accm);
                }
            }
        } else if (op == OP_AG) {
            // premises: nobody empty, every chunk held once; members with different masks leave this form
            Words<KW> accr = first.r;
            uint32_t smx = 0;
            bool anyzero = fold_or(first.r) == 0;
            for (int p = 1; p < g; ++p) {
                const Slot<KW, MW> cur = load_slot<KW, MW>(my, dstride, base + p * s);
                badx |= fold_and(cur.r, accr);
                smx |= fold_xor(cur.m, first.m);
                anyzero |= fold_or(cur.r) == 0;
#pragma unroll
                for (int i = 0; i < KW; ++i) accr.w[i] |= cur.r.w[i];
            }
            badx |= (uint32_t)anyzero;
            give_up |= smx != 0;
            changed = true;
            for (int p = 0; p < g; ++p) store_rows<KW, MW>(my, dstride, base + p * s, accr);
        } else {
            // Broadcast: the root holds what every member holds, and more than at least one of them
            uint32_t subx = 0, difx = 0;
            for (int p = 1; p < g; ++p) {
                const Slot<KW, MW> cur = load_slot<KW, MW>(my, dstride, base + p * s);
                subx |= fold_andn(cur.r, first.r) | fold_andn(cur.m, first.m);
                difx |= fold_xor(cur.r, first.r) | fold_xor(cur.m, first.m);
            }
            badx |= subx | (uint32_t)(difx == 0);
            changed = true;
            for (int p = 1; p < g; ++p) store_slot<KW, MW>(my, dstride, base + p * s, first.r, first.m);
        }
        if (master) hib += gs;
        else if (++lo == s) { lo = 0; hib += gs; }
    }
    if (badx != 0 || !changed) return STEP_INVALID;
    return give_up ? STEP_GIVE_UP : STEP_OK;
}

// The same for groups of GT = 2, 4, 8 or 16 devices: 16 members (16 / GT whole groups) are loaded
// back to back before any of them is used, so a step waits for LDS once per 16 devices instead of
// once per device.
template <int KW, int MW, int GT>
__device__ inline int step_batched(uint32_t* my, int dstride, int s, int master, int n_groups, int op) {
    constexpr int WPD = KW + MW;
    constexpr int NB_MAX = WPD <= 4 ? 16 : WPD <= 8 ? 8 : WPD <= 16 ? 4 : 2;   // keep a batch within ~64 registers
    if constexpr (GT > NB_MAX) {
        return step_uniform<KW, MW>(my, dstride, GT, s, master, n_groups, op);
    } else {
    constexpr int NB = NB_MAX, GPB = NB / GT;
    const int gs = GT * s;
    uint32_t badx = 0;
    bool changed = false, give_up = false;
    int lo = 0, hib = 0;
    for (int G0 = 0; G0 < n_groups; G0 += GPB) {
        int base[GPB];
#pragma unroll
        for (int i = 0; i < GPB; ++i) {
            base[i] = hib + lo;
            if (master) hib += gs;
            else if (++lo == s) { lo = 0; hib += gs; }
        }
        Slot<KW, MW> L[NB];
#pragma unroll
        for (int i = 0; i < GPB; ++i) {
            if (G0 + i < n_groups) {
#pragma unroll
                for (int p = 0; p < GT; ++p) L[i * GT + p] = load_slot<KW, MW>(my, dstride, base[i] + p * s);
            }
        }
#pragma unroll
        for (int i = 0; i < GPB; ++i) {
            if (G0 + i >= n_groups) continue;
            const Slot<KW, MW> first = L[i * GT];
            const int b0 = base[i];
            if (op == OP_AR || op == OP_RS || op == OP_RD) {
                Words<MW> accm = first.m;
#pragma unroll
                for (int p = 1; p < GT; ++p) {
                    const Slot<KW, MW>& cur = L[i * GT + p];
                    badx |= fold_xor(cur.r, first.r) | fold_and(cur.m, accm);
#pragma unroll
                    for (int w = 0; w < MW; ++w) accm.w[w] |= cur.m.w[w];
                }
                changed |= fold_or(first.r) != 0;
                if (op == OP_AR) {
#pragma unroll
                    for (int p = 0; p < GT; ++p) store_mask<KW, MW>(my, dstride, b0 + p * s, accm);
                } else if (op == OP_RD) {
                    store_mask<KW, MW>(my, dstride, b0, accm);
                    Words<KW> zr; Words<MW> zm;
#pragma unroll
                    for (int w = 0; w < KW; ++w) zr.w[w] = 0;
#pragma unroll
                    for (int w = 0; w < MW; ++w) zm.w[w] = 0;
#pragma unroll
                    for (int p = 1; p < GT; ++p) store_slot<KW, MW>(my, dstride, b0 + p * s, zr, zm);
                } else {
                    const int rows = popcount(first.r);
                    const int per = rows / GT;
                    badx |= (uint32_t)(per * GT != rows);
                    Words<KW> prev;
#pragma unroll
                    for (int w = 0; w < KW; ++w) prev.w[w] = 0;
#pragma unroll
                    for (int p = 0; p < GT; ++p) {
                        const Words<KW> upto = lowest_n(first.r, (p + 1) * per);
                        Words<KW> nr;
#pragma unroll
                        for (int w = 0; w < KW; ++w) { nr.w[w] = upto.w[w] & ~prev.w[w]; prev.w[w] = upto.w[w]; }
                        store_slot<KW, MW>(my, dstride, b0 + p * s, nr, accm);
                    }
                }
            } else if (op == OP_AG) {
                Words<KW> accr = first.r;
                uint32_t smx = 0;
                bool anyzero = fold_or(first.r) == 0;
#pragma unroll
                for (int p = 1; p < GT; ++p) {
                    const Slot<KW, MW>& cur = L[i * GT + p];
                    badx |= fold_and(cur.r, accr);
                    smx |= fold_xor(cur.m, first.m);
                    anyzero |= fold_or(cur.r) == 0;
#pragma unroll
                    for (int w = 0; w < KW; ++w) accr.w[w] |= cur.r.w[w];
                }
                badx |= (uint32_t)anyzero;
                give_up |= smx != 0;
                changed = true;
#pragma unroll
                for (int p = 0; p < GT; ++p) store_rows<KW, MW>(my, dstride, b0 + p * s, accr);
            } else {
                uint32_t subx = 0, difx = 0;
#pragma unroll
                for (int p = 1; p < GT; ++p) {
                    const Slot<KW, MW>& cur = L[i * GT + p];
                    subx |= fold_andn(cur.r, first.r) | fold_andn(cur.m, first.m);
                    difx |= fold_xor(cur.r, first.r) | fold_xor(cur.m, first.m);
                }
                badx |= subx | (uint32_t)(difx == 0);
                changed = true;
#pragma unroll
                for (int p = 1; p < GT; ++p) store_slot<KW, MW>(my, dstride, b0 + p * s, first.r, first.m);
            }
        }
    }
    if (badx != 0 || !changed) return STEP_INVALID;
    return give_up ? STEP_GIVE_UP : STEP_OK;
    }
}

// One instruction, lanes may differ in pattern and rule.  cost_* only with kCost.
template <int KW, int MW, bool kCost>
__device__ inline int step_mixed(uint32_t* my, int dstride, const PatLds P, int op, const DevQuery& q, const DevPattern* dp,
                                 double* sum_alpha, double* sum_beta) {
    const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
    uint32_t badx = 0;
    bool changed = false, give_up = false;
    GroupWalk wk;
    wk.start();
    Slot<KW, MW> first, acc;
    uint32_t eqx = 0, dmx = 0, drx = 0, smx = 0, subx = 0;
    bool anyzero = false;
    // ---- pass A: fold each group, check the premises, leave the result in the first member's slot
    for (int j = 0, n_part = P.n_groups * P.g; j < n_part; ++j) {
        const Slot<KW, MW> cur = load_slot<KW, MW>(my, dstride, wk.dev);
        if (wk.p == 0) {
            first = cur; acc = cur;
            eqx = 0; dmx = 0; drx = 0; smx = 0; subx = 0;
            anyzero = fold_or(cur.r) == 0;
        } else {
            eqx |= fold_xor(cur.r, first.r);              // same chunks on every member
            dmx |= fold_and(cur.m, acc.m);                // no contribution reduced twice
            drx |= fold_and(cur.r, acc.r);                // AllGather: chunks held once
            smx |= fold_xor(cur.m, first.m);
            subx |= fold_andn(cur.r, first.r) | fold_andn(cur.m, first.m);   // Broadcast: root knows more
            anyzero |= fold_or(cur.r) == 0;               // AllGather: nobody empty
#pragma unroll
            for (int i = 0; i < KW; ++i) acc.r.w[i] |= cur.r.w[i];
#pragma unroll
            for (int i = 0; i < MW; ++i) acc.m.w[i] |= cur.m.w[i];
        }
        if (wk.next(P)) {
            const int root = wk.root();
            if (red) {
                badx |= eqx | dmx;
                changed |= fold_or(first.r) != 0;         // a group of empty devices is a no-op
                if (op == OP_RS) {
                    const int rows = popcount(first.r);
                    badx |= (uint32_t)(div_small(rows, P.g) * P.g != rows);   // chunks must divide evenly
                }
                store_mask<KW, MW>(my, dstride, root, acc.m);
            } else if (op == OP_AG) {
                badx |= drx | (uint32_t)anyzero;
                give_up |= smx != 0;                      // rows with different column sets: not this form
                changed = true;
                store_rows<KW, MW>(my, dstride, root, acc.r);
            } else {
                badx |= subx | (uint32_t)((eqx | smx) == 0);   // information increase
                changed = true;
            }
            wk.next_group(P);
        }
    }
    if (badx != 0 || !changed) return STEP_INVALID;
    if (give_up) return STEP_GIVE_UP;

    if (kCost) {
        // ring alpha-beta time of the step: the first slot of a group now holds the chunk set that
        // sets its bytes (common rows / rows after the gather / the root's rows)
        double best = 0.0;
        const DevRows& rw = *q.rows;
        const int pid = (int)(dp - q.pat);
        for (int row = rw.pat_begin[pid]; row < rw.pat_begin[pid + 1]; ++row) {
            long long dot = 0;
            for (int e = rw.row_ptr[row]; e < rw.row_ptr[row + 1]; ++e) {
                const uint32_t ent = rw.entries[e];
                const Slot<KW, MW> sl = load_slot<KW, MW>(my, dstride, (int)entry_base(ent));
                dot += (long long)entry_cnt(ent) * (long long)popcount(sl.r);
            }
            best = fmax(best, (double)dot * q.inv_bw[rw.row_level[row]]);
        }
        double ring_steps, mult;
        step_factors(op, P.g, q.algo, ring_steps, mult);
        *sum_alpha += ring_steps * q.alpha[dp->span_level];
        *sum_beta += (mult / (double)q.k) * best;
    }

    // ---- pass B: every member's new pair from the group's slot
    wk.start();
    Slot<KW, MW> grp;
    Words<KW> prev;
    int per = 0;
    for (int j = 0, n_part = P.n_groups * P.g; j < n_part; ++j) {
        if (wk.p == 0) {
            grp = load_slot<KW, MW>(my, dstride, wk.dev);
            if (op == OP_RS) {
                per = div_small(popcount(grp.r), P.g);
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
        store_slot<KW, MW>(my, dstride, wk.dev, nr, nm);
        if (wk.next(P)) wk.next_group(P);
    }
    return STEP_OK;
}

template <int KW, int MW>
__device__ inline void compact_init(uint32_t* my, int dstride, int R, int k) {
    // Sec. 3.5: device i holds column i in every row
    const Words<KW> all_rows = full_mask<KW>(k);
    for (int d = 0; d < R; ++d) {
        Words<MW> m;
#pragma unroll
        for (int i = 0; i < MW; ++i) m.w[i] = (i == (d >> 5)) ? (1u << (d & 31)) : 0u;
        store_slot<KW, MW>(my, dstride, d, all_rows, m);
    }
}
template <int KW, int MW>
__device__ inline bool compact_is_goal(const uint32_t* my, int dstride, int R, int k) {
    // every device holds every row, each with the columns of the whole reduction group
    const Words<KW> all_rows = full_mask<KW>(k);
    const Words<MW> all_cols = full_mask<MW>(R);
    uint32_t dif = 0;
    for (int d = 0; d < R; ++d) {
        const Slot<KW, MW> sl = load_slot<KW, MW>(my, dstride, d);
        dif |= fold_xor(sl.r, all_rows) | fold_xor(sl.m, all_cols);
    }
    return dif == 0;
}

__device__ inline void load_patterns(const DevQuery& q, PatLds* spat, uint16_t* sdig) {
    for (int i = threadIdx.x; i < q.n_patterns; i += kWave) {
        PatLds p;
        p.g = q.pat[i].g; p.s = q.pat[i].s; p.master = q.pat[i].master; p.n_groups = q.pat[i].n_groups;
        spat[i] = p;
    }
    for (int i = threadIdx.x; i < q.alphabet; i += kWave) sdig[i] = q.instr_of_digit[i];
    __syncthreads();
}

}  // namespace
}  // namespace p2
