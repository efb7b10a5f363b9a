// Ordering kernels: rank-sort of the (few) valid candidate indices, and top-k selection of
// (cost, index) pairs by wavefront-level filtered insertion (the simulator's shortlist, Sec. 5).
#include "p2_device.h"

#include <mutex>

namespace p2 {

namespace {

constexpr int kWave = 64;

// sorted[rank(in[i])] = in[i], rank = number of smaller keys, per segment.  Keys are distinct
// candidate indices and a query has few valid ones next to its candidate space, so the quadratic
// count is the cheap way to a deterministic ascending order after an unordered atomic append.
__global__ __launch_bounds__(256) void k_rank_sort(const unsigned long long* __restrict__ valid,
                                                   const unsigned long long* __restrict__ valid2,
                                                   unsigned long long* __restrict__ sorted,
                                                   const DevPostSeg* __restrict__ segs, int n_segs) {
    __shared__ unsigned long long tile[256];
    const DevPostSeg seg = find_post_seg(segs, n_segs, blockIdx.x);
    const unsigned long long* in = (seg.in_off >> 63) ? valid2 + (seg.in_off & ~(1ull << 63)) : valid + seg.in_off;
    const uint32_t n = seg.count;
    const uint32_t i = (blockIdx.x - seg.first_block) * 256u + threadIdx.x;
    const unsigned long long key = i < n ? in[i] : 0ull;
    uint32_t rank = 0;
    for (uint32_t t0 = 0; t0 < n; t0 += 256u) {
        const uint32_t j = t0 + threadIdx.x;
        tile[threadIdx.x] = j < n ? in[j] : ~0ull;
        __syncthreads();
        const uint32_t lim = n - t0 < 256u ? n - t0 : 256u;
        for (uint32_t u = 0; u < lim; ++u) rank += tile[u] < key;
        __syncthreads();
    }
    if (i < n) sorted[seg.out_off + rank] = key;
}

struct Item {
    double c;
    unsigned long long idx;
    long long pos;
};

__device__ inline bool item_less(const Item& a, const Item& b) {
    if (a.c < b.c) return true;
    if (a.c > b.c) return false;
    if (a.idx != b.idx) return a.idx < b.idx;
    return a.pos < b.pos;
}

struct TopList {
    double* c;
    unsigned long long* idx;
    long long* pos;
};

// Insert `it` (same value in all lanes) into the wavefront's sorted list of at most K entries.
__device__ inline void list_insert(const TopList& L, int& cnt, int K, const Item& it, int lane) {
    int below = 0;
    for (int j = lane; j < cnt; j += kWave) {
        Item e{L.c[j], L.idx[j], L.pos[j]};
        below += item_less(e, it) ? 1 : 0;
    }
    for (int off = 32; off > 0; off >>= 1) below += __shfl_xor(below, off, kWave);
    const int p = below;
    if (p >= K) return;
    const int newcnt = cnt < K ? cnt + 1 : K;
    // shift entries p .. newcnt-2 one place up, highest chunk first
    for (int hi = newcnt - 1; hi > p; hi -= kWave) {
        const int j = hi - lane;                // destination
        Item e{0.0, 0ull, 0ll};
        const bool act = j > p;
        if (act) e = Item{L.c[j - 1], L.idx[j - 1], L.pos[j - 1]};
        __syncthreads();
        if (act) { L.c[j] = e.c; L.idx[j] = e.idx; L.pos[j] = e.pos; }
        __syncthreads();
    }
    if (lane == 0) { L.c[p] = it.c; L.idx[p] = it.idx; L.pos[p] = it.pos; }
    __syncthreads();
    cnt = newcnt;
}

// Feed one item per lane (valid = lane has one) through the list.
__device__ inline void list_offer(const TopList& L, int& cnt, int K, Item mine, bool valid, int lane) {
    for (;;) {
        bool want = valid;
        if (want && cnt == K) {
            Item last{L.c[K - 1], L.idx[K - 1], L.pos[K - 1]};
            want = item_less(mine, last);
        }
        const unsigned long long m = __ballot(want);
        if (m == 0ull) break;
        const int src = __ffsll((long long)m) - 1;
        Item it;
        it.c = __shfl(mine.c, src, kWave);
        it.idx = __shfl(mine.idx, src, kWave);
        it.pos = __shfl(mine.pos, src, kWave);
        list_insert(L, cnt, K, it, lane);
        if (lane == src) valid = false;
    }
}

// Stage 1: block b keeps the K best of its strided share of the input; stage 2 (one block) merges
// the block lists.  part_* hold gridDim.x lists of K entries (pos = -1 marks an unused slot).
__global__ __launch_bounds__(kWave) void k_topk_partial(const double* __restrict__ cost, long long stride,
                                                        const unsigned long long* __restrict__ index, long long n, int K,
                                                        double* __restrict__ part_c, unsigned long long* __restrict__ part_i,
                                                        long long* __restrict__ part_p, uint32_t* __restrict__ nan_flag) {
    extern __shared__ unsigned char raw[];
    TopList L;
    L.c = reinterpret_cast<double*>(raw);
    L.idx = reinterpret_cast<unsigned long long*>(L.c + K);
    L.pos = reinterpret_cast<long long*>(L.idx + K);
    const int lane = threadIdx.x;
    int cnt = 0;
    bool nan = false;
    for (long long t0 = (long long)blockIdx.x * kWave; t0 < n; t0 += (long long)gridDim.x * kWave) {
        const long long i = t0 + lane;
        Item mine{0.0, 0ull, i};
        const bool valid = i < n;
        if (valid) { mine.c = cost[i * stride]; mine.idx = index[i]; nan |= mine.c != mine.c; }
        list_offer(L, cnt, K, mine, valid && !(mine.c != mine.c), lane);
    }
    if (nan) atomicOr(nan_flag, 1u);
    __syncthreads();
    for (int j = lane; j < K; j += kWave) {
        const size_t o = (size_t)blockIdx.x * K + j;
        part_c[o] = j < cnt ? L.c[j] : 0.0;
        part_i[o] = j < cnt ? L.idx[j] : 0ull;
        part_p[o] = j < cnt ? L.pos[j] : -1ll;
    }
}

__global__ __launch_bounds__(kWave) void k_topk_merge(const double* __restrict__ part_c,
                                                      const unsigned long long* __restrict__ part_i,
                                                      const long long* __restrict__ part_p, long long total, int K,
                                                      long long* __restrict__ out_pos, long long n_out) {
    extern __shared__ unsigned char raw[];
    TopList L;
    L.c = reinterpret_cast<double*>(raw);
    L.idx = reinterpret_cast<unsigned long long*>(L.c + K);
    L.pos = reinterpret_cast<long long*>(L.idx + K);
    const int lane = threadIdx.x;
    int cnt = 0;
    for (long long t0 = 0; t0 < total; t0 += kWave) {
        const long long i = t0 + lane;
        Item mine{0.0, 0ull, -1ll};
        if (i < total) mine = Item{part_c[i], part_i[i], part_p[i]};
        list_offer(L, cnt, K, mine, i < total && mine.pos >= 0, lane);
    }
    __syncthreads();
    for (int j = lane; j < n_out; j += kWave) out_pos[j] = j < cnt ? L.pos[j] : -1ll;
}

// Many small selections in one launch: block b does job b from start to end (the list of K best of
// jobs[b].n entries) and writes the positions itself.
__global__ __launch_bounds__(kWave) void k_topk_jobs(const DevTopkJob* __restrict__ jobs) {
    extern __shared__ unsigned char raw[];
    const DevTopkJob J = jobs[blockIdx.x];
    const int K = J.k;
    TopList L;
    L.c = reinterpret_cast<double*>(raw);
    L.idx = reinterpret_cast<unsigned long long*>(L.c + K);
    L.pos = reinterpret_cast<long long*>(L.idx + K);
    const int lane = threadIdx.x;
    int cnt = 0;
    bool nan = false;
    for (long long t0 = 0; t0 < J.n; t0 += kWave) {
        const long long i = t0 + lane;
        Item mine{0.0, 0ull, i};
        const bool valid = i < J.n;
        if (valid) { mine.c = J.cost[i * J.stride]; mine.idx = J.index[i]; nan |= mine.c != mine.c; }
        list_offer(L, cnt, K, mine, valid && !(mine.c != mine.c), lane);
    }
    if (nan) atomicOr(J.nan_flag, 1u);
    __syncthreads();
    const long long n_out = K < J.n ? K : J.n;
    for (int j = lane; j < n_out; j += kWave) J.out_pos[j] = j < cnt ? L.pos[j] : -1ll;
}

// Many large selections in two launches: job j is cut into kBigParts strided shares, block (part, j) keeps the K best
// of its share in the job's piece of the scratch buffer (kBigParts lists of max_k entries), then block j of the
// second launch merges the job's lists.
constexpr int kBigParts = 64;
__global__ __launch_bounds__(kWave) void k_topk_big_partial(const DevTopkJob* __restrict__ jobs, int max_k, double* __restrict__ part_c,
                                                            unsigned long long* __restrict__ part_i, long long* __restrict__ part_p) {
    extern __shared__ unsigned char raw[];
    const DevTopkJob J = jobs[blockIdx.y];
    const int K = J.k;
    TopList L;
    L.c = reinterpret_cast<double*>(raw);
    L.idx = reinterpret_cast<unsigned long long*>(L.c + K);
    L.pos = reinterpret_cast<long long*>(L.idx + K);
    const int lane = threadIdx.x;
    int cnt = 0;
    bool nan = false;
    for (long long t0 = (long long)blockIdx.x * kWave; t0 < J.n; t0 += (long long)kBigParts * kWave) {
        const long long i = t0 + lane;
        Item mine{0.0, 0ull, i};
        const bool valid = i < J.n;
        if (valid) { mine.c = J.cost[i * J.stride]; mine.idx = J.index[i]; nan |= mine.c != mine.c; }
        list_offer(L, cnt, K, mine, valid && !(mine.c != mine.c), lane);
    }
    if (nan) atomicOr(J.nan_flag, 1u);
    __syncthreads();
    const size_t o0 = ((size_t)blockIdx.y * kBigParts + blockIdx.x) * (size_t)max_k;
    for (int j = lane; j < K; j += kWave) {
        part_c[o0 + j] = j < cnt ? L.c[j] : 0.0;
        part_i[o0 + j] = j < cnt ? L.idx[j] : 0ull;
        part_p[o0 + j] = j < cnt ? L.pos[j] : -1ll;
    }
}
__global__ __launch_bounds__(kWave) void k_topk_big_merge(const DevTopkJob* __restrict__ jobs, int max_k, const double* __restrict__ part_c,
                                                          const unsigned long long* __restrict__ part_i,
                                                          const long long* __restrict__ part_p) {
    extern __shared__ unsigned char raw[];
    const DevTopkJob J = jobs[blockIdx.x];
    const int K = J.k;
    TopList L;
    L.c = reinterpret_cast<double*>(raw);
    L.idx = reinterpret_cast<unsigned long long*>(L.c + K);
    L.pos = reinterpret_cast<long long*>(L.idx + K);
    const int lane = threadIdx.x;
    int cnt = 0;
    const size_t o0 = (size_t)blockIdx.x * kBigParts * (size_t)max_k;
    for (int part = 0; part < kBigParts; ++part)
        for (int t0 = 0; t0 < K; t0 += kWave) {
            const int j = t0 + lane;
            Item mine{0.0, 0ull, -1ll};
            if (j < K) { const size_t o = o0 + (size_t)part * max_k + j; mine = Item{part_c[o], part_i[o], part_p[o]}; }
            list_offer(L, cnt, K, mine, j < K && mine.pos >= 0, lane);
        }
    __syncthreads();
    const long long n_out = K < J.n ? K : J.n;
    for (int j = lane; j < n_out; j += kWave) J.out_pos[j] = j < cnt ? L.pos[j] : -1ll;
}

// Device memory -> pinned host memory, written by the GPU itself in 16-byte words.
__global__ __launch_bounds__(256) void k_copy_out(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Up to three such copies in one launch (a call's programs, costs and shortlist positions).
struct CopyOut { uint4* dst; const uint4* src; size_t n16; };
__global__ __launch_bounds__(256) void k_copy_out3(CopyOut a, CopyOut b, CopyOut c) {
    const size_t ab = a.n16 + b.n16, total = ab + c.n16;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        if (i < a.n16) a.dst[i] = a.src[i];
        else if (i < ab) b.dst[i - a.n16] = b.src[i - a.n16];
        else c.dst[i - ab] = c.src[i - ab];
    }
}

inline unsigned topk_blocks(long long n) {
    long long b = (n + 64 * 16 - 1) / (64 * 16);      // at least 16 tiles per block
    if (b < 1) b = 1;
    if (b > 2048) b = 2048;
    return (unsigned)b;
}

}  // namespace

hipError_t launch_copy_out(void* dst_host, const void* src_dev, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return hipSuccess;
    const size_t n16 = (bytes + 15) / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(k_copy_out, dim3(blocks), dim3(256), 0, stream, static_cast<uint4*>(dst_host),
                       static_cast<const uint4*>(src_dev), n16);
    return hipGetLastError();
}

hipError_t launch_copy_out3(void* dst0, const void* src0, size_t bytes0, void* dst1, const void* src1, size_t bytes1,
                            void* dst2, const void* src2, size_t bytes2, hipStream_t stream) {
    const CopyOut a{static_cast<uint4*>(dst0), static_cast<const uint4*>(src0), (bytes0 + 15) / 16};
    const CopyOut b{static_cast<uint4*>(dst1), static_cast<const uint4*>(src1), (bytes1 + 15) / 16};
    const CopyOut c{static_cast<uint4*>(dst2), static_cast<const uint4*>(src2), (bytes2 + 15) / 16};
    const size_t n16 = a.n16 + b.n16 + c.n16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(k_copy_out3, dim3(blocks), dim3(256), 0, stream, a, b, c);
    return hipGetLastError();
}

hipError_t launch_rank_sort(const unsigned long long* valid, const unsigned long long* valid2, unsigned long long* sorted,
                            const DevPostSeg* segs, int n_segs, unsigned blocks, hipStream_t stream) {
    if (n_segs == 0 || blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_rank_sort, dim3(blocks), dim3(256), 0, stream, valid, valid2, sorted, segs, n_segs);
    return hipGetLastError();
}

size_t topk_scratch_bytes(long long n, int k) { return (size_t)topk_blocks(n) * (size_t)k * 24; }

hipError_t launch_topk_jobs(const DevTopkJob* jobs, unsigned n_jobs, int max_k, hipStream_t stream) {
    if (n_jobs == 0) return hipSuccess;
    hipLaunchKernelGGL(k_topk_jobs, dim3(n_jobs), dim3(kWave), (size_t)max_k * 24, stream, jobs);
    return hipGetLastError();
}

__global__ __launch_bounds__(kWave) void k_gather_rows(const DevGatherSeg* __restrict__ segs, const p2_program* __restrict__ progs,
                                                       const double* __restrict__ costs, int n_cost, const long long* __restrict__ pos,
                                                       p2_program* __restrict__ sel_progs, double* __restrict__ sel_costs) {
    const DevGatherSeg S = segs[blockIdx.x];
    for (uint32_t t = threadIdx.x; t < S.rows; t += kWave) {
        const long long p = pos[S.pos_first + t];
        if (p < 0) continue;                         // (the host reports a selection that came back short)
        const size_t src = (size_t)(S.out_first + (unsigned long long)p), dst = (size_t)(S.pos_first + t);
        sel_progs[dst] = progs[src];
        for (int c = 0; c < n_cost; ++c) sel_costs[dst * n_cost + c] = costs[src * n_cost + c];
    }
}

hipError_t launch_gather_rows(const DevGatherSeg* segs, unsigned n_segs, const p2_program* progs, const double* costs, int n_cost,
                              const long long* pos, p2_program* sel_progs, double* sel_costs, hipStream_t stream) {
    if (n_segs == 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_rows, dim3(n_segs), dim3(kWave), 0, stream, segs, progs, costs, n_cost, pos, sel_progs, sel_costs);
    return hipGetLastError();
}

size_t topk_big_scratch_bytes(unsigned n_jobs, int max_k) { return (size_t)n_jobs * kBigParts * (size_t)max_k * 24; }

hipError_t launch_topk_big(const DevTopkJob* jobs, unsigned n_jobs, int max_k, void* scratch, hipStream_t stream) {
    if (n_jobs == 0) return hipSuccess;
    const size_t per = (size_t)n_jobs * kBigParts * (size_t)max_k;
    double* pc = reinterpret_cast<double*>(scratch);
    unsigned long long* pi = reinterpret_cast<unsigned long long*>(pc + per);
    long long* pp = reinterpret_cast<long long*>(pi + per);
    const size_t lds = (size_t)max_k * 24;
    hipLaunchKernelGGL(k_topk_big_partial, dim3(kBigParts, n_jobs), dim3(kWave), lds, stream, jobs, max_k, pc, pi, pp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_topk_big_merge, dim3(n_jobs), dim3(kWave), lds, stream, jobs, max_k, pc, pi, pp);
    return hipGetLastError();
}

hipError_t launch_topk(const double* cost, long long stride, const unsigned long long* index, long long n, int k,
                       long long* out_pos, void* scratch, uint32_t* nan_flag, hipStream_t stream) {
    if (n <= 0 || k <= 0) return hipSuccess;
    const unsigned blocks = topk_blocks(n);
    double* pc = reinterpret_cast<double*>(scratch);
    unsigned long long* pi = reinterpret_cast<unsigned long long*>(pc + (size_t)blocks * k);
    long long* pp = reinterpret_cast<long long*>(pi + (size_t)blocks * k);
    const size_t lds = (size_t)k * 24;
    hipLaunchKernelGGL(k_topk_partial, dim3(blocks), dim3(kWave), lds, stream, cost, stride, index, n, k, pc, pi, pp, nan_flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long n_out = k < n ? k : n;
    hipLaunchKernelGGL(k_topk_merge, dim3(1), dim3(kWave), lds, stream, pc, pi, pp, (long long)blocks * k, k, out_pos, n_out);
    return hipGetLastError();
}

// ---- selection without any allocation ------------------------------------------------------------
// The two-stage selection keeps its stage-1 lists (blocks x k entries of 24 bytes) in device memory.  For
// callers that may not allocate, that memory is a fixed array in the library's device image: every GPU the
// library runs on holds its own copy at its own address for the life of the process, and all calls on one
// GPU share it.  Host code never uses the array's name as an address: the device address is asked for once
// per device and kept.
constexpr int kFixedTopkMaxK = 64;
constexpr size_t kFixedTopkListBytes = (size_t)2048 * kFixedTopkMaxK * 24;     // topk_blocks() <= 2048
static __device__ __align__(256) unsigned char scratch[kFixedTopkListBytes + 256];   // lists, then a flag word

namespace {
constexpr int kMaxGpus = 64;
std::mutex g_fixed_mutex;
void* g_fixed_ptr[kMaxGpus] = {nullptr};

__global__ void k_clear_word(uint32_t* w) { *w = 0u; }

// Device address of `scratch` on the current device.
hipError_t fixed_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxGpus) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_fixed_mutex);
    if (!g_fixed_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_fixed_ptr[dev] = p;
    }
    *out = g_fixed_ptr[dev];
    return hipSuccess;
}
}  // namespace

int topk_fixed_max_k() { return kFixedTopkMaxK; }

hipError_t launch_topk_fixed(const double* cost, long long stride, const unsigned long long* index, long long n, int k,
                             long long* out_pos, uint32_t* nan_flag, hipStream_t stream) {
    if (n <= 0 || k <= 0) return hipSuccess;
    if (k > kFixedTopkMaxK || topk_scratch_bytes(n, k) > kFixedTopkListBytes) return hipErrorInvalidValue;
    void* base = nullptr;
    hipError_t e = fixed_scratch(&base);
    if (e != hipSuccess) return e;
    // the flag starts at zero for this call (a fill kernel, so that the call can be recorded into a graph)
    uint32_t* flag = nan_flag ? nan_flag : reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(base) + kFixedTopkListBytes);
    hipLaunchKernelGGL(k_clear_word, dim3(1), dim3(1), 0, stream, flag);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // (stage 1 writes every slot of the lists it hands to stage 2, so the lists need no clearing)
    return launch_topk(cost, stride, index, n, k, out_pos, base, flag, stream);
}

}  // namespace p2
