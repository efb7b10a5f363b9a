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
// A lane keeps the R (chunk set, mask) pairs of its candidate in LDS: the pair of device d of
// lane l sits at word (d * LS + l) * WS, WS = words per pair (padded to an odd count unless it is
// 2 or 4, which are read with one 64/128-bit access), so the 64 lanes of one access fall into
// distinct banks.  No lane ever reads another lane's state, so the kernel needs no barrier.
//
// The 64 lanes of a wavefront hold consecutive candidates, which share every instruction but the
// last.  A step whose instruction is the same in all live lanes takes the uniform path: scalar
// loops over groups and members, one specialised body per rule.  Otherwise (the last instruction,
// or a wavefront that straddles two prefixes) the mixed path runs two flat loops over the
// participating devices in group-major order -- pass A folds a group and leaves its result in
// the first member's slot, pass B writes every member's new pair from that slot -- with the
// rule-specific parts as selects, so lanes with different rules and group shapes stay together.
#include "p2_compact_dev.h"

#include <type_traits>

namespace p2 {

namespace {

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
    constexpr int WS = Lay<KW, MW>::WS;
    uint32_t* my = lds + lane * WS;
    const int dstride = LS * WS;
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
    unsigned long long steps = 0, members = 0;
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
        if (alive) compact_init<KW, MW>(my, dstride, q.R, q.k);
        bool give_up = false;
        uint32_t ran = 0, visited = 0;
        for (int t = 0; t < len; ++t) {
            if (!__any(alive)) break;
            if (alive) {
                const uint32_t ins = (uint32_t)(prog >> (9 * t)) & 511u;
                ++ran;
                visited += (uint32_t)(spat[ins >> 3].n_groups * spat[ins >> 3].g);
                // the live lanes of a wavefront usually hold the same instruction here
                const uint32_t ins0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)ins);
                int rc;
                if (__all(ins == ins0)) {
                    const PatLds P0 = spat[ins0 >> 3];
                    const int g0 = __builtin_amdgcn_readfirstlane(P0.g), s0 = __builtin_amdgcn_readfirstlane(P0.s);
                    const int ma0 = __builtin_amdgcn_readfirstlane(P0.master), ng0 = __builtin_amdgcn_readfirstlane(P0.n_groups);
                    const int op0 = (int)(ins0 & 7u);
                    switch (g0) {
                    case 2: rc = step_batched<KW, MW, 2>(my, dstride, s0, ma0, ng0, op0); break;
                    case 4: rc = step_batched<KW, MW, 4>(my, dstride, s0, ma0, ng0, op0); break;
                    case 8: rc = step_batched<KW, MW, 8>(my, dstride, s0, ma0, ng0, op0); break;
                    case 16: rc = step_batched<KW, MW, 16>(my, dstride, s0, ma0, ng0, op0); break;
                    default: rc = step_uniform<KW, MW>(my, dstride, g0, s0, ma0, ng0, op0); break;
                    }
                } else {
                    rc = step_mixed<KW, MW, false>(my, dstride, spat[ins >> 3], (int)(ins & 7u), q, nullptr, nullptr, nullptr);
                }
                alive = rc == STEP_OK;
                give_up = rc == STEP_GIVE_UP;
            }
        }
        if (alive && compact_is_goal<KW, MW>(my, dstride, q.R, q.k)) {
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
    for (int o = 32; o > 0; o >>= 1) { steps += __shfl_xor(steps, o, kWave); members += __shfl_xor(members, o, kWave); }
    if (lane == 0 && steps) {
        atomicAdd(&q.counters->steps[blockIdx.x % kCounterStripes], steps);
        atomicAdd(&q.counters->members[blockIdx.x % kCounterStripes], members);
    }
}

// Cost of valid programs: lane i of a segment's block re-runs sorted[out_off + i] with the cost terms on.
template <int KW, int MW>
__global__ __launch_bounds__(kWave) void k_cost_compact(const DevQuery* __restrict__ queries,
                                                        const DevPostSeg* __restrict__ segs, int n_segs,
                                                        const unsigned long long* __restrict__ sorted,
                                                        p2_program* __restrict__ out_prog, double* __restrict__ out_cost,
                                                        int LS) {
    extern __shared__ uint32_t lds[];
    __shared__ PatLds spat[kMaxPatterns];
    __shared__ uint16_t sdig[kMaxPatterns * 5];
    const DevPostSeg seg = find_post_seg(segs, n_segs, blockIdx.x);
    const DevQuery& q = queries[seg.query];
    load_patterns(q, spat, sdig);
    const int lane = threadIdx.x;
    constexpr int WS = Lay<KW, MW>::WS;
    uint32_t* my = lds + lane * WS;
    const int dstride = LS * WS;
    const uint32_t li = (blockIdx.x - seg.first_block) * (uint32_t)LS + (uint32_t)lane;
    if (lane >= LS || li >= seg.count) return;
    const size_t i = seg.out_off + li;
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
    compact_init<KW, MW>(my, dstride, q.R, q.k);
    double sum_alpha = 0.0, sum_beta = 0.0;
    bool ok = true;
    p2_program pr;
    pr.index = idx;
    pr.len = (uint8_t)len;
    for (int t = 0; t < 7; ++t) pr.instr[t] = 0;
    for (int t = 0; t < len; ++t) {
        const uint32_t ins = (uint32_t)(prog >> (9 * t)) & 511u;
        pr.instr[t] = (uint8_t)((ins >> 3) * 5u + (ins & 7u));
        if (ok) ok = step_mixed<KW, MW, true>(my, dstride, spat[ins >> 3], (int)(ins & 7u), q, &q.pat[ins >> 3],
                                                &sum_alpha, &sum_beta) == STEP_OK;
    }
    out_prog[i] = pr;
    for (int m = 0; m < q.n_msg; ++m)
        out_cost[i * q.n_msg + m] = ok ? sum_alpha + q.msg_bytes[m] * sum_beta : __longlong_as_double(0x7ff8000000000000ll);
}

// Cost of valid programs whose state is too large for more than a few candidates per wavefront in LDS
// (hundreds of devices): one wavefront per program, the 64 lanes share every step.  State: [R][KW + MW]
// words in LDS (chunk set, contribution mask of each device).  A step is two passes.  Pass 1, one item per
// (group, word): fold the word over the members, check the premises that can be seen in one word, leave the
// result in the first member's slot (the united mask of an AllReduce-like step, the united chunk set of an
// AllGather) and add the word's share to the number of chunks that sets the group's bytes.  Pass 2, one
// item per (member, word), or per member for ReduceScatter: take the result from the first member.  The
// rules and the cost terms are those of step_mixed; a program whose state leaves this form gets NaN costs
// (the literal cost kernel fills those rows).
template <int KW, int MW>
__global__ __launch_bounds__(kWave) void k_cost_wide(const DevQuery* __restrict__ queries,
                                                     const DevPostSeg* __restrict__ segs, int n_segs,
                                                     const unsigned long long* __restrict__ sorted,
                                                     p2_program* __restrict__ out_prog, double* __restrict__ out_cost) {
    extern __shared__ uint32_t lds[];
    constexpr int WPD = KW + MW;
    const DevPostSeg seg = find_post_seg(segs, n_segs, blockIdx.x);
    const DevQuery& q = queries[seg.query];
    const int lane = threadIdx.x, R = q.R;
    uint32_t* const S = lds;                       // [R][WPD]
    uint32_t* const gcount = S + R * WPD;          // [R / 2] chunks that set a group's bytes
    uint32_t* const gflag = gcount + (R / 2 > 0 ? R / 2 : 1);   // [R / 2] Broadcast: some member differs from the root
    uint32_t* const flags = gflag + (R / 2 > 0 ? R / 2 : 1);    // 0: premise failed, 1: something changes, 2: leaves the form
    const size_t i = seg.out_off + (blockIdx.x - seg.first_block);
    const unsigned long long idx = sorted[i];
    int len = 1;
    while (len < q.max_len && idx >= q.base[len + 1]) ++len;
    uint32_t digit[P2_MAX_LEN];
    {
        unsigned long long rem = idx - q.base[len];
        const unsigned long long I = (unsigned long long)q.alphabet;
        for (int t = P2_MAX_LEN - 1; t >= 0; --t) {
            if (t < len) { const unsigned long long nx = rem / I; digit[t] = (uint32_t)(rem - nx * I); rem = nx; }
            else digit[t] = 0;
        }
    }
    // Sec. 3.5: device i holds column i in every row
    const Words<KW> all_rows = full_mask<KW>(q.k);
    for (int it = lane; it < R * WPD; it += kWave) {
        const int d = it / WPD, w = it - d * WPD;
        S[it] = w < KW ? all_rows.w[w] : ((w - KW) == (d >> 5) ? (1u << (d & 31)) : 0u);
    }
    __syncthreads();
    double sum_alpha = 0.0, sum_beta = 0.0;
    bool ok = true;
    p2_program pr;
    pr.index = idx;
    pr.len = (uint8_t)len;
    for (int t = 0; t < P2_MAX_LEN; ++t) pr.instr[t] = 0;
    for (int t = 0; t < len; ++t) {
        const uint32_t ins = q.instr_of_digit[digit[t]];
        const int pid = (int)(ins >> 3), op = (int)(ins & 7u);
        pr.instr[t] = (uint8_t)(pid * 5 + op);
        if (!ok) continue;
        const DevPattern& P = q.pat[pid];
        const int g = P.g, s = P.s, ng = P.n_groups, gs = g * s;
        const bool red = op == OP_AR || op == OP_RS || op == OP_RD;
        auto first_of = [&](int G) -> int {               // first device of group G
            if (P.master) return G * gs;
            const int hi = div_small(G, s);
            return hi * gs + (G - hi * s);
        };
        for (int G = lane; G < ng; G += kWave) { gcount[G] = 0; gflag[G] = 0; }
        if (lane == 0) { flags[0] = 0; flags[1] = 0; flags[2] = 0; }
        __syncthreads();
        bool bad = false, leaves = false;
        if (op == OP_AG) {
            // nobody empty
            for (int j = lane; j < ng * g; j += kWave) {
                const int G = div_small(j, g), p = j - G * g;
                const int d = first_of(G) + p * s;
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < KW; ++w) any |= S[d * WPD + w];
                bad |= any == 0u;
            }
        }
        // ---- pass 1
        for (int it = lane; it < ng * WPD; it += kWave) {
            const int G = it / WPD, w = it - G * WPD;
            const int base = first_of(G);
            const uint32_t first = S[base * WPD + w];
            uint32_t acc = first, dif = 0, over = 0, sub = 0;
            for (int p = 1; p < g; ++p) {
                const uint32_t v = S[(base + p * s) * WPD + w];
                dif |= v ^ first; over |= v & acc; sub |= v & ~first;
                acc |= v;
            }
            if (red) {
                if (w < KW) { bad |= dif != 0u; atomicAdd(&gcount[G], (uint32_t)__popc(first)); }   // same chunks on every member
                else { bad |= over != 0u; S[base * WPD + w] = acc; }                                // no contribution reduced twice
            } else if (op == OP_AG) {
                if (w < KW) { bad |= over != 0u; S[base * WPD + w] = acc; atomicAdd(&gcount[G], (uint32_t)__popc(acc)); }   // chunks held once
                else leaves |= dif != 0u;                  // rows with different column sets: not this form
            } else {
                bad |= sub != 0u;                          // the root knows what every member knows
                if (dif != 0u) gflag[G] = 1;
                if (w < KW) atomicAdd(&gcount[G], (uint32_t)__popc(first));
            }
        }
        if (bad) flags[0] = 1;
        if (leaves) flags[2] = 1;
        __syncthreads();
        for (int G = lane; G < ng; G += kWave) {
            const uint32_t cnt = gcount[G];
            if (red) {
                if (op == OP_RS && cnt % (uint32_t)g != 0u) flags[0] = 1;   // chunks must divide evenly
                if (cnt) flags[1] = 1;                                     // a group of empty devices is a no-op
            } else {
                if (op == OP_BC && !gflag[G]) flags[0] = 1;                // information increase
                flags[1] = 1;
            }
        }
        __syncthreads();
        if (flags[0] || !flags[1] || flags[2]) { ok = false; continue; }   // (valid programs only fail by leaving the form)
        // ---- ring alpha-beta time of the step
        {
            double best = 0.0;
            const DevRows& rw = *q.rows;
            for (int row = rw.pat_begin[pid] + lane; row < rw.pat_begin[pid + 1]; row += kWave) {
                long long dot = 0;
                for (int e = rw.row_ptr[row]; e < rw.row_ptr[row + 1]; ++e) {
                    const uint32_t ent = rw.entries[e];
                    dot += (long long)entry_cnt(ent) * (long long)gcount[entry_group(ent)];
                }
                best = fmax(best, (double)dot * q.inv_bw[rw.row_level[row]]);
            }
            for (int off = 32; off > 0; off >>= 1) best = fmax(best, __shfl_xor(best, off, kWave));
            double ring_steps, mult;
            step_factors(op, g, q.algo, ring_steps, mult);
            sum_alpha += ring_steps * q.alpha[P.span_level];
            sum_beta += (mult / (double)q.k) * best;
        }
        // ---- pass 2
        if (op == OP_RS) {
            // the member of rank p keeps the p-th block of its chunks in ascending order (all members hold the same)
            for (int j = lane; j < ng * g; j += kWave) {
                const int G = div_small(j, g), p = j - G * g;
                const int base = first_of(G);
                const int d = base + p * s;
                Words<KW> r;
#pragma unroll
                for (int w = 0; w < KW; ++w) r.w[w] = S[d * WPD + w];
                const int per = div_small((int)gcount[G], g);
                const Words<KW> upto = lowest_n(r, (p + 1) * per), below = lowest_n(r, p * per);
#pragma unroll
                for (int w = 0; w < KW; ++w) S[d * WPD + w] = upto.w[w] & ~below.w[w];
                if (p != 0) {
#pragma unroll
                    for (int w = 0; w < MW; ++w) S[d * WPD + KW + w] = S[base * WPD + KW + w];
                }
            }
        } else {
            // (a division by a constant is a multiplication; group and member numbers stay below 512, where
            // div_small is exact)
            auto copy_words = [&](auto w0_c, auto nw_c) {
                constexpr int w0 = decltype(w0_c)::value, nw = decltype(nw_c)::value;
                for (int it = lane; it < ng * (g - 1) * nw; it += kWave) {
                    const int j = it / nw, w = w0 + (it - j * nw);
                    const int G = div_small(j, g - 1), p = 1 + (j - G * (g - 1));
                    const int base = first_of(G);
                    S[(base + p * s) * WPD + w] = op == OP_RD ? 0u : S[base * WPD + w];
                }
            };
            if (op == OP_AR) copy_words(std::integral_constant<int, KW>{}, std::integral_constant<int, MW>{});
            else if (op == OP_AG) copy_words(std::integral_constant<int, 0>{}, std::integral_constant<int, KW>{});
            else copy_words(std::integral_constant<int, 0>{}, std::integral_constant<int, WPD>{});
        }
        __syncthreads();
    }
    if (lane == 0) out_prog[i] = pr;
    if (lane < q.n_msg)
        out_cost[i * q.n_msg + lane] = ok ? sum_alpha + q.msg_bytes[lane] * sum_beta : __longlong_as_double(0x7ff8000000000000ll);
}

inline int round_words(int bits) {
    const int w = (bits + 31) / 32;
    return w <= 1 ? 1 : w <= 2 ? 2 : w <= 4 ? 4 : w <= 8 ? 8 : 16;
}
inline int lane_words(int kw, int mw) {          // Lay<kw, mw>::WS
    const int wpd = kw + mw;
    return (wpd == 2 || wpd == 4) ? wpd : (wpd | 1);
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
hipError_t cost_mw(int MW, const DevQuery* queries, const DevPostSeg* segs, int n_segs, const unsigned long long* sorted,
                   p2_program* out_prog, double* out_cost, unsigned blocks, int LS, size_t lds, hipStream_t stream) {
    hipError_t e = hipSuccess;
#define P2_GO(MWV)                                                                                                        \
    e = allow_lds(k_cost_compact<KW, MWV>, lds);                                                                          \
    if (e == hipSuccess) hipLaunchKernelGGL((k_cost_compact<KW, MWV>), dim3(blocks), dim3(kWave), lds, stream, queries, segs, n_segs, sorted, out_prog, out_cost, LS);
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
    const size_t per_lane = (size_t)R * (size_t)lane_words(round_words(k), round_words(R)) * 4;
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
    const size_t lds = (size_t)max_R * (size_t)lane_words(KW, MW) * 4 * (size_t)LS;
    switch (KW) {
    case 1: return eval_mw<1>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    case 2: return eval_mw<2>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    case 4: return eval_mw<4>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    case 8: return eval_mw<8>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    default: return eval_mw<16>(MW, queries, segs, n_segs, total_blocks, LS, lds, stream);
    }
}

hipError_t launch_cost_compact_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                    int max_R, int max_k, const unsigned long long* sorted, p2_program* progs,
                                    double* costs, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const int LS = compact_lanes(max_R, max_k);       // the segments' per_block
    if (LS == 0) return hipErrorInvalidValue;
    const int KW = round_words(max_k), MW = round_words(max_R);
    const size_t lds = (size_t)max_R * (size_t)lane_words(KW, MW) * 4 * (size_t)LS;
    switch (KW) {
    case 1: return cost_mw<1>(MW, queries, segs, n_segs, sorted, progs, costs, blocks, LS, lds, stream);
    case 2: return cost_mw<2>(MW, queries, segs, n_segs, sorted, progs, costs, blocks, LS, lds, stream);
    case 4: return cost_mw<4>(MW, queries, segs, n_segs, sorted, progs, costs, blocks, LS, lds, stream);
    case 8: return cost_mw<8>(MW, queries, segs, n_segs, sorted, progs, costs, blocks, LS, lds, stream);
    default: return cost_mw<16>(MW, queries, segs, n_segs, sorted, progs, costs, blocks, LS, lds, stream);
    }
}

bool cost_wide_applies(int max_R, int max_k) { return max_R > 64 && compact_lanes(max_R, max_k) <= 8; }

hipError_t launch_cost_wide_list(const DevQuery* queries, const DevPostSeg* segs, int n_segs, unsigned blocks,
                                 int max_R, int max_k, const unsigned long long* sorted, p2_program* progs,
                                 double* costs, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    const int KW = round_words(max_k), MW = round_words(max_R);
    const size_t lds = ((size_t)max_R * (size_t)(KW + MW) + (size_t)max_R + 8) * 4;
    hipError_t e = hipSuccess;
#define P2_GO(KWV, MWV)                                                                                                   \
    e = allow_lds(k_cost_wide<KWV, MWV>, lds);                                                                            \
    if (e == hipSuccess) hipLaunchKernelGGL((k_cost_wide<KWV, MWV>), dim3(blocks), dim3(kWave), lds, stream, queries, segs, n_segs, sorted, progs, costs);
    // (more than 64 devices)
    switch (KW * 100 + MW) {
    case 104: P2_GO(1, 4) break;
    case 204: P2_GO(2, 4) break;
    case 404: P2_GO(4, 4) break;
    case 804: P2_GO(8, 4) break;
    case 1604: P2_GO(16, 4) break;
    case 108: P2_GO(1, 8) break;
    case 208: P2_GO(2, 8) break;
    case 408: P2_GO(4, 8) break;
    case 808: P2_GO(8, 8) break;
    case 1608: P2_GO(16, 8) break;
    case 116: P2_GO(1, 16) break;
    case 216: P2_GO(2, 16) break;
    case 416: P2_GO(4, 16) break;
    case 816: P2_GO(8, 16) break;
    case 1616: P2_GO(16, 16) break;
    default: return hipErrorInvalidValue;
    }
#undef P2_GO
    return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace p2
