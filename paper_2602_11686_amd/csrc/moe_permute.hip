// Token rearrangement by expert and its inverse: moe_permute,
// moe_unpermute_combine, moe_combine_bwd.
//
// The paper's implementation section replaces a host-blocking masked select by
// a device kernel for "token rearrangement"; the combine is the weighted sum of
// the mixture formula (Preliminary section).  Everything here is HBM-bound
// copy work plus a small integer sort, so the kernels move rows as 16-byte
// vectors, read each token row once, and keep all counts on the device.
//
// Stable counting sort of the R = T*k pairs:
//   1. per-chunk histograms (one wavefront owns CHUNK consecutive pairs),
//   2. per-chunk starting rows (exclusive scan down the chunks for every expert,
//      then across experts),
//   3. each wavefront walks its chunk in order, 64 pairs at a time: lanes with
//      the same expert are found with 8 ballots over the bits of the expert id,
//      the lane's rank is the running count of its expert plus the number of
//      lower lanes in its group.
// moe_permute runs 1 as one kernel and 2 + 3 as a second one, in which every
// workgroup redoes the scan for its own chunks; moe_permute_lite keeps 2 as a
// one-workgroup kernel of its own, because it also checks and expands the
// replica table there.  A last kernel copies the rows: one pass over x, k row
// writes per token.
#include <mutex>

#include "moe_internal.h"

namespace moe {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// pairs per wavefront in the sort: 128, doubled until there are at most 256 chunks (the scan walks the
// chunks of an expert one after the other; short chunks keep the histogram and rank kernels parallel)
static inline int chunk_pairs(int64_t R) {
    int c = 128;
    while ((R + c - 1) / c > 256 && c < 8192) c *= 2;
    return c;
}
constexpr int kWavesPerBlock = 4;  // 256 threads

constexpr size_t kLiteTableBytes = (4 * MOE_MAX_EXPERTS + 64) * sizeof(int32_t);

static inline int num_chunks(int64_t R) { const int c = chunk_pairs(R); return (int)((R + c - 1) / c); }

size_t permute_workspace_bytes(const moe_shape* s) {
    const int64_t R = (int64_t)s->T * s->k;
    // chunk histograms + chunk bases + (lite routing) four per-expert tables and a flag
    return 2 * align_up((size_t)num_chunks(R) * s->E * sizeof(int32_t), 256) + kLiteTableBytes;
}

// ---- 1. per-chunk histogram ---------------------------------------------------
__global__ __launch_bounds__(256) void permute_hist_kernel(const int32_t* __restrict__ ids, int R, int E, int kChunk,
                                                           int32_t* __restrict__ chunk_hist) {
    extern __shared__ int32_t lds_hist[];  // [kWavesPerBlock][E]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int32_t* h = lds_hist + wave * E;
    for (int e = lane; e < E; e += 64) h[e] = 0;
    __syncthreads();
    const int chunk = blockIdx.x * kWavesPerBlock + wave;
    const int p0 = chunk * kChunk;
    for (int i = lane; i < kChunk; i += 64) {
        const int p = p0 + i;
        if (p < R) atomicAdd(&h[ids[p]], 1);
    }
    __syncthreads();
    if (p0 < R)
        for (int e = lane; e < E; e += 64) chunk_hist[(size_t)chunk * E + e] = h[e];
}

// ---- 2. scan helpers (lite routing): chunk_base[c][e] = rank of the first pair of chunk c inside expert e ----
// 256 threads = P parts x E experts (P = 256 / E): part p of expert e owns a contiguous range of
// chunks, sums it, and after the parts' sums and the experts' offsets are known writes the running
// base of every chunk of its range.  Input and output are different arrays, so the loads of the
// two passes do not wait for the stores.
struct ScanParts {
    int e, part, c_begin, c_end;  // this thread's expert and chunk range (empty for surplus threads)
    int P;
};
__device__ __forceinline__ ScanParts scan_parts(int nchunks, int E) {
    ScanParts sp;
    sp.P = 256 / E;  // E <= 256
    sp.e = threadIdx.x % E;
    sp.part = threadIdx.x / E;
    const int len = (nchunks + sp.P - 1) / sp.P;
    sp.c_begin = sp.part < sp.P ? min(sp.part * len, nchunks) : 0;
    sp.c_end = sp.part < sp.P ? min(sp.c_begin + len, nchunks) : 0;
    return sp;
}
__device__ __forceinline__ int32_t scan_range_sum(const int32_t* __restrict__ chunk_hist, int E, const ScanParts& sp) {
    // (the histograms were written by workgroups on other XCDs: every batch of loads pays a trip beyond
    // this XCD's L2, so the batches are made long)
    int32_t run = 0;
    int c = sp.c_begin;
    for (; c + 32 <= sp.c_end; c += 32) {
        int32_t v[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) v[u] = chunk_hist[(size_t)(c + u) * E + sp.e];
#pragma unroll
        for (int u = 0; u < 32; ++u) run += v[u];
    }
    for (; c + 8 <= sp.c_end; c += 8) {
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = chunk_hist[(size_t)(c + u) * E + sp.e];
#pragma unroll
        for (int u = 0; u < 8; ++u) run += v[u];
    }
    for (; c < sp.c_end; ++c) run += chunk_hist[(size_t)c * E + sp.e];
    return run;
}
__device__ __forceinline__ void scan_range_write(const int32_t* __restrict__ chunk_hist, int32_t* __restrict__ chunk_base,
                                                 int E, const ScanParts& sp, int32_t run) {
    int c = sp.c_begin;
    for (; c + 32 <= sp.c_end; c += 32) {
        int32_t v[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) v[u] = chunk_hist[(size_t)(c + u) * E + sp.e];
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            chunk_base[(size_t)(c + u) * E + sp.e] = run;
            run += v[u];
        }
    }
    for (; c + 8 <= sp.c_end; c += 8) {
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = chunk_hist[(size_t)(c + u) * E + sp.e];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            chunk_base[(size_t)(c + u) * E + sp.e] = run;
            run += v[u];
        }
    }
    for (; c < sp.c_end; ++c) {
        chunk_base[(size_t)c * E + sp.e] = run;
        run += chunk_hist[(size_t)c * E + sp.e];
    }
}

// ---- 2 + 3 in one launch --------------------------------------------------------------------
// Every workgroup redoes the part of the scan it needs instead of waiting for a one-workgroup scan kernel:
// 1024 threads = P parts x E experts sum the chunk histograms (all chunks: the experts' totals; the chunks
// before this workgroup's: the rows already taken), one wavefront scans the totals across the experts, and
// the first four wavefronts then rank one chunk each as in step 3.  The histograms are read by every
// workgroup (nchunks * E * 4 bytes, from L2), which is cheaper than a launch that all of them wait for.
constexpr int kRankScanThreads = 1024;
__global__ __launch_bounds__(kRankScanThreads) void permute_rank_scan_kernel(
    const int32_t* __restrict__ ids, int R, int E, int kChunk, const int32_t* __restrict__ chunk_hist, int nchunks,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ row_of_pair,
    int32_t* __restrict__ pair_of_row) {
    __shared__ int32_t ps_all[kRankScanThreads], ps_before[kRankScanThreads];  // [part][expert]
    __shared__ int32_t e_total[MOE_MAX_EXPERTS], e_before[MOE_MAX_EXPERTS], e_off[MOE_MAX_EXPERTS + 1];
    __shared__ int32_t lds_next[kWavesPerBlock * MOE_MAX_EXPERTS];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c_first = blockIdx.x * kWavesPerBlock;
    int P = kRankScanThreads / E;  // E <= 256: at least 4 parts
    if (P > 32) P = 32;
    {
        const int e = tid % E, part = tid / E;
        int32_t all = 0, before = 0;
        if (part < P) {
            const int len = (nchunks + P - 1) / P;
            const int cb = min(part * len, nchunks), ce = min(cb + len, nchunks);
            int c = cb;
            for (; c + 16 <= ce; c += 16) {
                int32_t v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = chunk_hist[(size_t)(c + u) * E + e];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    all += v[u];
                    before += (c + u < c_first) ? v[u] : 0;
                }
            }
            for (; c < ce; ++c) {
                const int32_t v = chunk_hist[(size_t)c * E + e];
                all += v;
                before += (c < c_first) ? v : 0;
            }
            ps_all[part * E + e] = all;
            ps_before[part * E + e] = before;
        }
    }
    __syncthreads();
    if (tid < E) {
        int32_t all = 0, before = 0;
        for (int p = 0; p < P; ++p) {
            all += ps_all[p * E + tid];
            before += ps_before[p * E + tid];
        }
        e_total[tid] = all;
        e_before[tid] = before;
    }
    __syncthreads();
    if (wave == 0) {  // exclusive scan of the totals: 4 experts per lane, then across the lanes
        int32_t c[4], sum = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = lane * 4 + u;
            c[u] = e < E ? e_total[e] : 0;
            sum += c[u];
        }
        int32_t incl = sum;
#pragma unroll
        for (int dlt = 1; dlt < 64; dlt <<= 1) {
            const int32_t o = __shfl_up(incl, dlt, 64);
            if (lane >= dlt) incl += o;
        }
        int32_t run = incl - sum;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = lane * 4 + u;
            if (e <= E) e_off[e] = run;
            run += c[u];
        }
        if (lane == 63 && E == MOE_MAX_EXPERTS) e_off[MOE_MAX_EXPERTS] = run;
    }
    __syncthreads();
    if (blockIdx.x == 0) {
        if (tid < E) {
            counts[tid] = e_total[tid];
            offsets[tid] = e_off[tid];
        }
        if (tid == 0) offsets[E] = e_off[E];
    }
    if (wave >= kWavesPerBlock) return;  // whole wavefronts leave; no workgroup barrier below
    const int chunk = c_first + wave;
    const int p0 = chunk * kChunk;
    if (p0 >= R) return;
    int32_t* next = lds_next + wave * E;
    for (int e = lane; e < E; e += 64) {
        int32_t b = e_off[e] + e_before[e];
        for (int j = 0; j < wave; ++j) b += chunk_hist[(size_t)(c_first + j) * E + e];
        next[e] = b;
    }
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int i = 0; i < kChunk; i += 64) {
        const int p = p0 + i + lane;
        const bool live = p < R;
        const int e = live ? ids[p] : -1;
        uint64_t same = __ballot(live);
        if (!live) same = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t bal = __ballot((e >> b) & 1);
            same &= ((e >> b) & 1) ? bal : ~bal;
        }
        if (live) {
            const int before = __popcll(same & lt_mask);
            const int row = next[e] + before;
            row_of_pair[p] = row;
            pair_of_row[row] = p;
        }
        __builtin_amdgcn_wave_barrier();
        if (live && (same >> lane) == 1ull) next[e] += __popcll(same);
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- 2L / 3L. the same sort with the lite routing of the paper's appendix folded in ---------------
// Every expert e has a list of replica groups rep_group[rep_begin[e] .. rep_begin[e+1]) (the replicas the
// sending device may use: those in its node, else all).  The n_e pairs of the expert, in stable order, are
// cut into len consecutive blocks whose sizes differ by at most one (larger blocks first); block r goes to
// group rep_group[rep_begin[e] + r].  Rows are ordered by group.
//
// The table comes from outside and is checked here: list bounds, a list for every expert that has pairs,
// group ids inside [0, G), no group listed twice.  If a check fails, *table_errors is set and the rows fall
// back to plain expert order with all of them counted in group 0, so that every index written stays inside
// [0, R) whatever the table holds.
struct LiteTables {          // in the workspace, written by the scan, read by the rank kernel
    int32_t* lo;             // [E] first list entry of the expert        (fallback: first row of the expert)
    int32_t* base;           // [E] n_e / len
    int32_t* rem;            // [E] n_e % len
    int32_t* ok;             // [1]
};

// exclusive prefix sum of v[0..255] over the 256 threads of the workgroup (every thread calls it)
__device__ __forceinline__ int32_t block_exclusive_scan_256(int32_t mine, int32_t* tmp) {
    const int t = threadIdx.x;
    tmp[t] = mine;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {
        const int32_t add = t >= d ? tmp[t - d] : 0;
        __syncthreads();
        tmp[t] += add;
        __syncthreads();
    }
    return tmp[t] - mine;
}

__global__ __launch_bounds__(256) void permute_scan_lite_kernel(const int32_t* __restrict__ chunk_hist,
                                                                int32_t* __restrict__ chunk_base, int nchunks, int E,
                                                                int G, int n_rep, int R,
                                                                const int32_t* __restrict__ rep_begin,
                                                                const int32_t* __restrict__ rep_group,
                                                                int32_t* __restrict__ expert_counts,
                                                                int32_t* __restrict__ group_counts,
                                                                int32_t* __restrict__ group_offsets, LiteTables tb,
                                                                int32_t* __restrict__ table_errors) {
    __shared__ int32_t tmp[256];
    __shared__ int32_t listed[MOE_MAX_EXPERTS];
    __shared__ int32_t gcnt[MOE_MAX_EXPERTS];
    __shared__ int32_t bad;
    const int e = threadIdx.x;
    const ScanParts sp = scan_parts(nchunks, E);
    __shared__ int32_t psum[256];
    __shared__ int32_t nexp[MOE_MAX_EXPERTS];
    psum[threadIdx.x] = sp.part < sp.P ? scan_range_sum(chunk_hist, E, sp) : 0;
    __syncthreads();
    int32_t part_before = 0;
    if (sp.part < sp.P) {
        int32_t total = 0;
        for (int p = 0; p < sp.P; ++p) {
            const int32_t v = psum[p * E + sp.e];
            if (p < sp.part) part_before += v;
            total += v;
        }
        if (sp.part == 0) nexp[sp.e] = total;
    }
    __syncthreads();
    int32_t n = 0;
    if (e < E) {
        n = nexp[e];
        expert_counts[e] = n;
    }
    listed[e] = 0;
    gcnt[e] = 0;
    if (e == 0) bad = 0;
    __syncthreads();
    int lo = 0, hi = 0;
    if (e < E) {
        lo = rep_begin[e];
        hi = rep_begin[e + 1];
        if (lo < 0 || hi < lo || hi > n_rep) {
            atomicOr(&bad, 1);
            lo = hi = 0;
        } else {
            if (n > 0 && hi == lo) atomicOr(&bad, 2);
            for (int r = lo; r < hi; ++r) {
                const int g = rep_group[r];
                if ((unsigned)g >= (unsigned)G) atomicOr(&bad, 4);
                else if (atomicAdd(&listed[g], 1) > 0) atomicOr(&bad, 8);
            }
        }
    }
    __syncthreads();
    const bool ok = bad == 0;
    const int32_t expert_off = block_exclusive_scan_256(e < E ? n : 0, tmp);  // the fallback order
    if (e == 0) {
        tb.ok[0] = ok ? 1 : 0;
        if (table_errors) table_errors[0] = bad;
        if (!ok) gcnt[0] = R;
    }
    if (e < E) {
        if (ok) {
            const int len = hi - lo;
            const int b = len ? n / len : 0, rm = len ? n % len : 0;
            for (int r = 0; r < len; ++r) gcnt[rep_group[lo + r]] = b + (r < rm ? 1 : 0);
            tb.lo[e] = lo;
            tb.base[e] = b;
            tb.rem[e] = rm;
        } else {
            tb.lo[e] = expert_off;
            tb.base[e] = 0;
            tb.rem[e] = 0;
        }
    }
    __syncthreads();
    const int32_t mine = e < G ? gcnt[e] : 0;
    const int32_t goff = block_exclusive_scan_256(mine, tmp);
    if (e < G) {
        group_counts[e] = mine;
        group_offsets[e] = goff;
    }
    if (e == G - 1) group_offsets[G] = goff + mine;
    // rank of the first pair of every chunk inside its expert
    if (sp.part < sp.P) scan_range_write(chunk_hist, chunk_base, E, sp, part_before);
}

__global__ __launch_bounds__(256) void permute_rank_lite_kernel(const int32_t* __restrict__ ids, int R, int E, int kChunk,
                                                                const int32_t* __restrict__ chunk_base,
                                                                const int32_t* __restrict__ rep_group,
                                                                const int32_t* __restrict__ group_offsets,
                                                                LiteTables tb, int32_t* __restrict__ row_of_pair,
                                                                int32_t* __restrict__ pair_of_row) {
    extern __shared__ int32_t lds_next[];  // [kWavesPerBlock][4][E]: next rank, list start, base, rem
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * kWavesPerBlock + wave;
    const int p0 = chunk * kChunk;
    if (p0 >= R) return;  // whole wavefront leaves together; no barrier below
    int32_t* next = lds_next + wave * 4 * E;
    int32_t* lo = next + E;
    int32_t* base = lo + E;
    int32_t* rem = base + E;
    for (int e = lane; e < E; e += 64) {
        next[e] = chunk_base[(size_t)chunk * E + e];
        lo[e] = tb.lo[e];
        base[e] = tb.base[e];
        rem[e] = tb.rem[e];
    }
    const bool ok = tb.ok[0] != 0;
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int i = 0; i < kChunk; i += 64) {
        const int p = p0 + i + lane;
        const bool live = p < R;
        const int e = live ? ids[p] : -1;
        uint64_t same = __ballot(live);
        if (!live) same = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t bal = __ballot((e >> b) & 1);
            same &= ((e >> b) & 1) ? bal : ~bal;
        }
        if (live) {
            const int q = next[e] + __popcll(same & lt_mask);  // stable rank inside the expert
            int row;
            if (ok) {
                const int b = base[e], rm = rem[e], big = rm * (b + 1);
                int r, start;
                if (q < big) {
                    r = q / (b + 1);
                    start = r * (b + 1);
                } else {  // b >= 1 here: q >= big = rm*(b+1) with b == 0 would mean q >= n_e
                    r = rm + (q - big) / b;
                    start = big + (r - rm) * b;
                }
                row = group_offsets[rep_group[lo[e] + r]] + (q - start);
            } else {
                row = lo[e] + q;
            }
            row_of_pair[p] = row;
            pair_of_row[row] = p;
        }
        __builtin_amdgcn_wave_barrier();
        if (live && (same >> lane) == 1ull) next[e] += __popcll(same);
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- 4. row scatter: x[t] -> x_perm[row_of_pair[t*k+s]] for s < k ----------------------

template <int KT>  // KT > 0: k at compile time (the k row indices are requested together); 0: any k
__global__ __launch_bounds__(256) void permute_scatter_rows_kernel(const u32x4* __restrict__ x,
                                                                   const int32_t* __restrict__ row_of_pair,
                                                                   u32x4* __restrict__ x_perm, int T, int k,
                                                                   int vecs_per_row) {
    const int64_t total = (int64_t)T * vecs_per_row;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int t = (int)(i / vecs_per_row);
        const int v = (int)(i - (int64_t)t * vecs_per_row);
        const u32x4 val = __builtin_nontemporal_load(&x[i]);
        if constexpr (KT > 0) {
            int rows[KT];
#pragma unroll
            for (int s = 0; s < KT; ++s) rows[s] = row_of_pair[(size_t)t * KT + s];
#pragma unroll
            for (int s = 0; s < KT; ++s) __builtin_nontemporal_store(val, &x_perm[(size_t)rows[s] * vecs_per_row + v]);
        } else {
            for (int s = 0; s < k; ++s) {
                const int row = row_of_pair[(size_t)t * k + s];
                __builtin_nontemporal_store(val, &x_perm[(size_t)row * vecs_per_row + v]);
            }
        }
    }
}

// ---- combine: y[t] = sum_s w[t,s] * y_perm[row_of_pair[t*k+s]] ------------------------
template <class T, int VEC>
struct VecIO;
template <>
struct VecIO<bf16_t, 8> {
    template <bool NT = false>
    static __device__ __forceinline__ void load(const void* p, float (&v)[8]) {
        u32x4 u;
        if constexpr (NT) u = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        else u = *reinterpret_cast<const u32x4*>(p);
        const uint32_t w[4] = {u[0], u[1], u[2], u[3]};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    template <bool NT = false>
    static __device__ __forceinline__ void store(void* p, const float (&v)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        u32x4 o;
        o[0] = w[0]; o[1] = w[1]; o[2] = w[2]; o[3] = w[3];
        if constexpr (NT) __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(p));
        else *reinterpret_cast<u32x4*>(p) = o;
    }
};
template <>
struct VecIO<float, 4> {
    template <bool NT = false>
    static __device__ __forceinline__ void load(const void* p, float (&v)[4]) {
        f32x4 u;
        if constexpr (NT) u = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        else u = *reinterpret_cast<const f32x4*>(p);
        v[0] = u[0]; v[1] = u[1]; v[2] = u[2]; v[3] = u[3];
    }
    template <bool NT = false>
    static __device__ __forceinline__ void store(void* p, const float (&v)[4]) {
        f32x4 u;
        u[0] = v[0]; u[1] = v[1]; u[2] = v[2]; u[3] = v[3];
        if constexpr (NT) __builtin_nontemporal_store(u, reinterpret_cast<f32x4*>(p));
        else *reinterpret_cast<f32x4*>(p) = u;
    }
};

// KT > 0: k is known at compile time, so the k row indices, then the k row pieces, are all requested before
// the first of them is used (a gather is bound by how many loads are in flight, not by arithmetic).
// KT == 0: any k, one row after the other.  The sum runs over s = 0 .. k-1 in this order either way.
// The rows of y_perm are read once and are loaded non-temporally, so that they do not push the output (which
// the next kernel reads) out of the caches; the same holds for y_perm in the backward kernel below.  Measured:
// non-temporal stores of the outputs make the kernels that follow slower.
template <class T, int VEC, int KT>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ y_perm,
                                                      const int32_t* __restrict__ row_of_pair,
                                                      const float* __restrict__ w, T* __restrict__ y, int Tn,
                                                      int d, int k) {
    const int vecs_per_row = d / VEC;
    const int64_t total = (int64_t)Tn * vecs_per_row;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int t = (int)(i / vecs_per_row);
        const int v = (int)(i - (int64_t)t * vecs_per_row);
        float acc[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
        if constexpr (KT > 0) {
            int rows[KT];
            float ws[KT];
#pragma unroll
            for (int s = 0; s < KT; ++s) {
                rows[s] = row_of_pair[(size_t)t * KT + s];
                ws[s] = w ? w[(size_t)t * KT + s] : 1.0f;
            }
            float val[KT][VEC];
#pragma unroll
            for (int s = 0; s < KT; ++s) VecIO<T, VEC>::template load<true>(y_perm + (size_t)rows[s] * d + (size_t)v * VEC, val[s]);
#pragma unroll
            for (int s = 0; s < KT; ++s)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] += ws[s] * val[s][j];
        } else {
            for (int s = 0; s < k; ++s) {
                const int row = row_of_pair[(size_t)t * k + s];
                const float ws = w ? w[(size_t)t * k + s] : 1.0f;
                float val[VEC];
                VecIO<T, VEC>::template load<true>(y_perm + (size_t)row * d + (size_t)v * VEC, val);
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] += ws * val[j];
            }
        }
        VecIO<T, VEC>::store(y + (size_t)t * d + (size_t)v * VEC, acc);
    }
}

// ---- combine backward: one wavefront per token -----------------------------------
// dy_perm[row(t,s)] = w[t,s] * dy[t],  dw[t,s] = <dy[t], y_perm[row(t,s)]>.
// KT > 0: the wavefront walks the row in pieces of 64 lanes x VEC columns; a piece of dy[t] is read once
// and meets the same piece of all k rows, whose loads are in flight together.  Per (t,s) the products are
// added in the same order as in the KT == 0 form: ascending columns inside a lane, then across the lanes.
template <class T, int VEC, int KT>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ y_perm,
                                                          const int32_t* __restrict__ row_of_pair,
                                                          const float* __restrict__ w, T* __restrict__ dy_perm,
                                                          float* __restrict__ dw, int Tn, int d, int k) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const int vecs_per_row = d / VEC;
    if constexpr (KT > 0) {
        int rows[KT];
        float ws[KT], dot[KT];
#pragma unroll
        for (int s = 0; s < KT; ++s) {
            rows[s] = row_of_pair[(size_t)t * KT + s];
            ws[s] = w[(size_t)t * KT + s];
            dot[s] = 0.f;
        }
        for (int v = lane; v < vecs_per_row; v += 64) {
            float g[VEC], yv[KT][VEC];
            VecIO<T, VEC>::load(dy + (size_t)t * d + (size_t)v * VEC, g);
#pragma unroll
            for (int s = 0; s < KT; ++s) VecIO<T, VEC>::template load<true>(y_perm + (size_t)rows[s] * d + (size_t)v * VEC, yv[s]);
#pragma unroll
            for (int s = 0; s < KT; ++s) {
                float o[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    dot[s] += g[j] * yv[s][j];
                    o[j] = ws[s] * g[j];
                }
                VecIO<T, VEC>::store(dy_perm + (size_t)rows[s] * d + (size_t)v * VEC, o);
            }
        }
#pragma unroll
        for (int s = 0; s < KT; ++s) {
            float ds = dot[s];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) ds += __shfl_xor(ds, m, 64);
            if (lane == 0) dw[(size_t)t * KT + s] = ds;
        }
    } else {
        for (int s = 0; s < k; ++s) {
            const int row = row_of_pair[(size_t)t * k + s];
            const float ws = w[(size_t)t * k + s];
            float dot = 0.f;
            for (int v = lane; v < vecs_per_row; v += 64) {
                float g[VEC], yv[VEC], o[VEC];
                VecIO<T, VEC>::load(dy + (size_t)t * d + (size_t)v * VEC, g);
                VecIO<T, VEC>::template load<true>(y_perm + (size_t)row * d + (size_t)v * VEC, yv);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    dot += g[j] * yv[j];
                    o[j] = ws * g[j];
                }
                VecIO<T, VEC>::store(dy_perm + (size_t)row * d + (size_t)v * VEC, o);
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
            if (lane == 0) dw[(size_t)t * k + s] = dot;
        }
    }
}

static inline int grid_for(int64_t work_items, int block, int max_blocks) {
    int64_t g = (work_items + block - 1) / block;
    if (g > max_blocks) g = max_blocks;
    if (g < 1) g = 1;
    return (int)g;
}

}  // namespace moe

using namespace moe;

// launch with k as a template argument where a specialisation exists (k = 1, 2, 4, 6, 8), else the runtime-k form
#define MOE_DISPATCH_K(kval, CALL)      \
    switch (kval) {                     \
        case 1: { CALL(1); break; }     \
        case 2: { CALL(2); break; }     \
        case 4: { CALL(4); break; }     \
        case 6: { CALL(6); break; }     \
        case 8: { CALL(8); break; }     \
        default: { CALL(0); break; }    \
    }


// The kernels of moe_permute; chunk_hist: nchunks * E int32 of device memory that needs no initialisation
// (every entry that is read is written by the histogram kernel first).
static moe_status permute_launch(const char* who, const moe_shape* s, const void* x, const int32_t* topk_ids,
                                 int32_t* counts, int32_t* offsets, int32_t* row_of_pair, int32_t* pair_of_row,
                                 void* x_perm, int32_t* chunk_hist, hipStream_t st) {
    const int R = s->T * s->k, E = s->E;
    const int nchunks = num_chunks(R);
    const int nblocks = (nchunks + kWavesPerBlock - 1) / kWavesPerBlock;
    const size_t lds = (size_t)kWavesPerBlock * E * sizeof(int32_t);
    permute_hist_kernel<<<nblocks, 256, lds, st>>>(topk_ids, R, E, chunk_pairs(R), chunk_hist);
    permute_rank_scan_kernel<<<nblocks, kRankScanThreads, 0, st>>>(topk_ids, R, E, chunk_pairs(R), chunk_hist, nchunks,
                                                                   counts, offsets, row_of_pair, pair_of_row);
    if (x_perm) {
        const int vecs_per_row = (int)((size_t)s->d * el_size(s) / 16);
        const int grid = grid_for((int64_t)s->T * vecs_per_row, 256, 256 * 16);
#define MOE_CALL(KT)                                                                                       \
    permute_scatter_rows_kernel<KT><<<grid, 256, 0, st>>>(static_cast<const u32x4*>(x), row_of_pair,        \
                                                          static_cast<u32x4*>(x_perm), s->T, s->k, vecs_per_row)
        MOE_DISPATCH_K(s->k, MOE_CALL)
#undef MOE_CALL
    }
    return launch_status(who);
}

static moe_status permute_check_args(const char* who, const moe_shape* s, const void* x, const int32_t* topk_ids,
                                     int32_t* counts, int32_t* offsets, int32_t* row_of_pair, int32_t* pair_of_row,
                                     void* x_perm) {
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(topk_ids, "topk_ids", who));
    MOE_RETURN_IF(check_ptr(counts, "counts", who));
    MOE_RETURN_IF(check_ptr(offsets, "offsets", who));
    MOE_RETURN_IF(check_ptr(row_of_pair, "row_of_pair", who));
    MOE_RETURN_IF(check_ptr(pair_of_row, "pair_of_row", who));
    MOE_RETURN_IF(check_ptr(x_perm, "x_perm", who, true));
    if (x_perm) MOE_RETURN_IF(check_ptr(x, "x", who));
    return MOE_OK;
}

extern "C" moe_status moe_permute(const moe_shape* s, const void* x, const int32_t* topk_ids, int32_t* counts,
                                  int32_t* offsets, int32_t* row_of_pair, int32_t* pair_of_row, void* x_perm,
                                  void* ws, size_t ws_bytes, void* stream) {
    const char* who = "moe_permute";
    MOE_RETURN_IF(permute_check_args(who, s, x, topk_ids, counts, offsets, row_of_pair, pair_of_row, x_perm));
    MOE_RETURN_IF(check_ptr(ws, "ws", who));
    if (ws_bytes < permute_workspace_bytes(s)) {
        set_error("%s: workspace %zu < %zu bytes", who, ws_bytes, permute_workspace_bytes(s));
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    return permute_launch(who, s, x, topk_ids, counts, offsets, row_of_pair, pair_of_row, x_perm,
                          static_cast<int32_t*>(ws), static_cast<hipStream_t>(stream));
}

// ---- moe_permute for callers that cannot allocate ------------------------------------------------------
// The per-chunk histograms live in a file-scope device array instead of a caller's workspace.  Every GPU
// that loads the library holds its own copy of the array at its own address; in host code the array's name
// is only a handle for hipGetSymbolAddress, never a device address.  The address is looked up once per
// device (with that device current) and kept; the kernels receive it as an ordinary pointer argument.
namespace moe {
constexpr int kStaticHistInts = 65536;                                       // 256 KiB per GPU
static __device__ __align__(256) int32_t scratch[kStaticHistInts];
constexpr int kMaxDevices = 64;
static int32_t* g_scratch_ptr[kMaxDevices];                                  // per device; null until looked up
static std::mutex g_scratch_mutex;

static moe_status static_scratch_ptr(const char* who, int32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_error("%s: hipGetDevice failed or device index %d is outside [0, %d): %s", who, dev, kMaxDevices,
                  hipGetErrorString(e));
        return MOE_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("%s: hipGetSymbolAddress(scratch) failed on device %d: %s", who, dev, hipGetErrorString(e));
            return MOE_ERR_DEVICE;
        }
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace moe

extern "C" size_t moe_permute_static_max_hist_entries(void) { return (size_t)kStaticHistInts; }

extern "C" moe_status moe_permute_static(const moe_shape* s, const void* x, const int32_t* topk_ids, int32_t* counts,
                                         int32_t* offsets, int32_t* row_of_pair, int32_t* pair_of_row, void* x_perm,
                                         void* stream) {
    const char* who = "moe_permute_static";
    MOE_RETURN_IF(permute_check_args(who, s, x, topk_ids, counts, offsets, row_of_pair, pair_of_row, x_perm));
    const int64_t need = (int64_t)num_chunks((int64_t)s->T * s->k) * s->E;
    if (need > kStaticHistInts) {
        set_error("%s: %lld histogram entries (chunks of the T*k pairs x E) exceed the static scratch of %d entries; "
                  "use moe_permute with a workspace", who, (long long)need, kStaticHistInts);
        return MOE_ERR_UNSUPPORTED;
    }
    int32_t* hist = nullptr;
    MOE_RETURN_IF(static_scratch_ptr(who, &hist));
    return permute_launch(who, s, x, topk_ids, counts, offsets, row_of_pair, pair_of_row, x_perm, hist,
                          static_cast<hipStream_t>(stream));
}

extern "C" moe_status moe_permute_lite(const moe_shape* s, int32_t G, int32_t n_rep, const void* x,
                                       const int32_t* topk_ids, const int32_t* rep_begin, const int32_t* rep_group,
                                       int32_t* expert_counts, int32_t* group_counts, int32_t* group_offsets,
                                       int32_t* row_of_pair, int32_t* pair_of_row, void* x_perm,
                                       int32_t* table_errors, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "moe_permute_lite";
    MOE_RETURN_IF(check_shape(s, who));
    if (G < 1 || G > MOE_MAX_EXPERTS || n_rep < 0) {
        set_error("%s: G=%d must be in [1, %d] and n_rep=%d >= 0", who, G, MOE_MAX_EXPERTS, n_rep);
        return MOE_ERR_INVALID_ARG;
    }
    MOE_RETURN_IF(check_ptr(topk_ids, "topk_ids", who));
    MOE_RETURN_IF(check_ptr(rep_begin, "rep_begin", who));
    if (n_rep > 0) MOE_RETURN_IF(check_ptr(rep_group, "rep_group", who));
    MOE_RETURN_IF(check_ptr(expert_counts, "expert_counts", who));
    MOE_RETURN_IF(check_ptr(group_counts, "group_counts", who));
    MOE_RETURN_IF(check_ptr(group_offsets, "group_offsets", who));
    MOE_RETURN_IF(check_ptr(row_of_pair, "row_of_pair", who));
    MOE_RETURN_IF(check_ptr(pair_of_row, "pair_of_row", who));
    MOE_RETURN_IF(check_ptr(x_perm, "x_perm", who, true));
    if (x_perm) MOE_RETURN_IF(check_ptr(x, "x", who));
    MOE_RETURN_IF(check_ptr(table_errors, "table_errors", who, true));
    MOE_RETURN_IF(check_ptr(ws, "ws", who));
    if (ws_bytes < permute_workspace_bytes(s)) {
        set_error("%s: workspace %zu < %zu bytes", who, ws_bytes, permute_workspace_bytes(s));
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int R = s->T * s->k, E = s->E;
    const int nchunks = num_chunks(R);
    const int nblocks = (nchunks + kWavesPerBlock - 1) / kWavesPerBlock;
    const size_t hist_ints = align_up((size_t)nchunks * E * sizeof(int32_t), 256) / sizeof(int32_t);
    int32_t* chunk_hist = static_cast<int32_t*>(ws);
    int32_t* chunk_base = chunk_hist + hist_ints;
    int32_t* tables = chunk_base + hist_ints;
    LiteTables tb{tables, tables + MOE_MAX_EXPERTS, tables + 2 * MOE_MAX_EXPERTS, tables + 4 * MOE_MAX_EXPERTS};
    permute_hist_kernel<<<nblocks, 256, (size_t)kWavesPerBlock * E * sizeof(int32_t), st>>>(topk_ids, R, E, chunk_pairs(R), chunk_hist);
    permute_scan_lite_kernel<<<1, 256, 0, st>>>(chunk_hist, chunk_base, nchunks, E, G, n_rep, R, rep_begin, rep_group,
                                                expert_counts, group_counts, group_offsets, tb, table_errors);
    permute_rank_lite_kernel<<<nblocks, 256, (size_t)kWavesPerBlock * 4 * E * sizeof(int32_t), st>>>(
        topk_ids, R, E, chunk_pairs(R), chunk_base, rep_group, group_offsets, tb, row_of_pair, pair_of_row);
    if (x_perm) {
        const int vecs_per_row = (int)((size_t)s->d * el_size(s) / 16);
        const int grid = grid_for((int64_t)s->T * vecs_per_row, 256, 256 * 16);
#define MOE_CALL(KT)                                                                                       \
    permute_scatter_rows_kernel<KT><<<grid, 256, 0, st>>>(static_cast<const u32x4*>(x), row_of_pair,        \
                                                          static_cast<u32x4*>(x_perm), s->T, s->k, vecs_per_row)
        MOE_DISPATCH_K(s->k, MOE_CALL)
#undef MOE_CALL
    }
    return launch_status(who);
}

extern "C" moe_status moe_unpermute_combine(const moe_shape* s, const void* y_perm, const int32_t* row_of_pair,
                                            const float* topk_w, void* y, void* stream) {
    const char* who = "moe_unpermute_combine";
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(y_perm, "y_perm", who));
    MOE_RETURN_IF(check_ptr(row_of_pair, "row_of_pair", who));
    MOE_RETURN_IF(check_ptr(topk_w, "topk_w", who, true));
    MOE_RETURN_IF(check_ptr(y, "y", who));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (s->dtype == MOE_BF16) {
        const int grid = grid_for((int64_t)s->T * (s->d / 8), 256, 256 * 16);
#define MOE_CALL(KT)                                                                                                  \
    combine_kernel<bf16_t, 8, KT><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(y_perm), row_of_pair, topk_w,     \
                                                        static_cast<bf16_t*>(y), s->T, s->d, s->k)
        MOE_DISPATCH_K(s->k, MOE_CALL)
#undef MOE_CALL
    } else {
        const int grid = grid_for((int64_t)s->T * (s->d / 4), 256, 256 * 16);
#define MOE_CALL(KT)                                                                                                  \
    combine_kernel<float, 4, KT><<<grid, 256, 0, st>>>(static_cast<const float*>(y_perm), row_of_pair, topk_w,       \
                                                       static_cast<float*>(y), s->T, s->d, s->k)
        MOE_DISPATCH_K(s->k, MOE_CALL)
#undef MOE_CALL
    }
    return launch_status(who);
}

extern "C" moe_status moe_combine_bwd(const moe_shape* s, const void* dy, const void* y_perm,
                                      const int32_t* row_of_pair, const float* topk_w, void* dy_perm,
                                      float* dtopk_w, void* stream) {
    const char* who = "moe_combine_bwd";
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(dy, "dy", who));
    MOE_RETURN_IF(check_ptr(y_perm, "y_perm", who));
    MOE_RETURN_IF(check_ptr(row_of_pair, "row_of_pair", who));
    MOE_RETURN_IF(check_ptr(topk_w, "topk_w", who));
    MOE_RETURN_IF(check_ptr(dy_perm, "dy_perm", who));
    MOE_RETURN_IF(check_ptr(dtopk_w, "dtopk_w", who));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int grid = (s->T + 3) / 4;
    if (s->dtype == MOE_BF16) {
#define MOE_CALL(KT)                                                                                                  \
    combine_bwd_kernel<bf16_t, 8, KT><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(dy),                          \
                                                            static_cast<const bf16_t*>(y_perm), row_of_pair, topk_w, \
                                                            static_cast<bf16_t*>(dy_perm), dtopk_w, s->T, s->d, s->k)
        MOE_DISPATCH_K(s->k, MOE_CALL)
#undef MOE_CALL
    } else {
#define MOE_CALL(KT)                                                                                                  \
    combine_bwd_kernel<float, 4, KT><<<grid, 256, 0, st>>>(static_cast<const float*>(dy),                            \
                                                           static_cast<const float*>(y_perm), row_of_pair, topk_w,   \
                                                           static_cast<float*>(dy_perm), dtopk_w, s->T, s->d, s->k)
        MOE_DISPATCH_K(s->k, MOE_CALL)
#undef MOE_CALL
    }
    return launch_status(who);
}
