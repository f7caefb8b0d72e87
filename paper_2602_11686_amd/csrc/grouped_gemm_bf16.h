// Grouped bf16 GEMM for CDNA4 (gfx950): 256x256x64 workgroup tiles, 8 wavefronts,
// MFMA 32x32x16 bf16 with fp32 accumulators, operands streamed HBM -> LDS by the
// DMA path of the global loads (no register staging) into two LDS stages of 64 KB.
//
// One template covers the six products of the expert FFN (paper section 3.1;
// 6*H*H' FLOPs per routed token forward, backward twice that):
//
//   RAGK == false: the ragged dimension is M (the rows of one expert)
//       A  [rows][K]  K contiguous                 (Xp, H, dYp, dA, dB)
//       B  BT == 0: [K][N]  N contiguous           (forward: W1, W3 [d][f], W2 [f][d])
//          BT == 1: [N][K]  K contiguous           (dgrad:   W2 as [f][d], W1/W3 as [d][f])
//   RAGK == true: the ragged dimension is the contraction (wgrad), AT == 1, BT == 0
//       A  [rows][M]  M contiguous                 (Xp, H)
//       B  [rows][N]  N contiguous                 (dA|dB, dYp)
//       C_e [M][N] = sum over the rows of expert e;  an expert without rows gets zeros.
//
// A k-stage is 64 wide.  What the vector memory path charges for is the cache line it touches, not the
// bytes it delivers (measured per CU for a 32 KB stage from L2: 1300 clocks when every request takes 64 bytes
// of a line, 770 with whole 128-byte lines, 620 with 512 contiguous bytes - against 1024 clocks of MFMAs
// for the same stage), so every DMA instruction here asks for whole lines.
//
// An operand tile whose contraction index is contiguous in memory ("row form") is kept in LDS as
// 256 rows x 128 B and read with ds_read_b128; the 16-byte piece p of row r sits in slot
// p ^ ((r >> 1) & 7).  An operand tile whose other index is contiguous ("k-row form") is kept as
// 64 k-rows x 512 B and read with the transposing LDS read (ds_read_b64_tr_b16: lane i of a 16-lane
// group receives column i of a 4(k) x 16 block); piece p of k-row q sits in slot
// p ^ (2*(q&3) + 8*(q&1)).  Both swizzles make every LDS read instruction of the main loop
// conflict-free on the 64 banks.  A DMA load writes 64 lanes x 16 B to consecutive LDS addresses, so
// the swizzle is applied on the global side: lane l fetches the piece that belongs in slot l.
//
// DUAL: two B matrices share the A tile (W1|W3 forward, dA|dB wgrad): the B tile holds 128 columns of the
// first as 64 k-rows x 256 B, then the same 128 columns of the second (same swizzle inside the 16 pieces of
// a k-row), so that one DMA instruction (4 k-rows x 256 B) reads from one matrix only.  Each wavefront
// accumulates both products for the same outputs (forward: the epilogue writes silu(a)*b).
#pragma once

namespace moe {

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int kStages = 2;
constexpr int kStageBytes = 65536;  // 32 KB A + 32 KB B
constexpr int kBOff = 32768;        // B tile inside a stage
constexpr int kWaves = 8;           // wave tile 128 x 64, two wavefronts per SIMD
constexpr int kThreads = kWaves * 64;
constexpr int kWN = kWaves / 2;            // wavefronts along N (two along M)
constexpr int NJ = 8 / kWN;                // 32-column MFMA blocks per wavefront
constexpr int CPW = 32 / kWaves;           // 1 KB DMA chunks per wavefront per operand tile
constexpr int kSteps = TK / 16;            // MFMA k-steps per stage
// LDS map (160 KB): the two stage buffers, then the epilogue's staging area, then the expert table and the
// two draw slots.  The staging area (32 KB) does not fit behind the stage buffers: it starts inside the last
// kDeferChunks 1 KB chunks of the second buffer's B half.  Those chunks (the last ones wavefront 7 loads)
// are requested after the epilogue when a tile's first two stages are requested in front of it.
constexpr int kLdsBytes = 160 * 1024;
constexpr int kTableBytes = 2 * (MOE_MAX_EXPERTS + 1) * 4 + 16;            // expert table + 2 draw slots
constexpr int kTableOff = (kLdsBytes - kTableBytes) & ~15;
constexpr int kStagingBytes = 32768;
constexpr int kStagingOff = kTableOff - kStagingBytes;
constexpr int kDeferChunks = (kStages * kStageBytes - kStagingOff + 1023) / 1024;
static_assert(kStagingOff >= kStages * kStageBytes - CPW * 1024 + 1024 && kDeferChunks >= 1 && kDeferChunks < CPW,
              "the staging area may only reach into chunks that one wavefront loads last");
constexpr int kGemmLds = kLdsBytes;
// Tile queues (GArgs::sched): one counter per XCD, kSchedStride words apart, all zero when the kernel starts.
constexpr int kSchedStride = 32;
constexpr int kSchedWords = 8 * kSchedStride;

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4v __attribute__((ext_vector_type(4)));
typedef float f32x2v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#define LDS_AS __attribute__((address_space(3)))


// Scheduling pattern for one k-step: MFMA, LDS read, MFMA, LDS read, ... (as many pairs as there are
// MFMAs or reads, whichever is more), then a fence.
template <int kMfma, int kReads>
__device__ __forceinline__ void interleave_mfma_dsread() {
#pragma unroll
    for (int i = 0; i < (kMfma > kReads ? kMfma : kReads); ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
    }
    __builtin_amdgcn_sched_barrier(0);
}

// slot = piece ^ swz: chosen so that the rows one LDS read instruction touches fall into different banks
__device__ __forceinline__ int swz_rows(int row) { return (row >> 1) & 7; }              // 128-byte rows, b128 reads
__device__ __forceinline__ int swz_krow(int q) { return 2 * (q & 3) + 8 * (q & 1); }      // 512-byte k-rows, tr reads

// 16 bytes per lane, global -> LDS, without passing through registers: lane l lands at
// lds_addr + 16*l (lds_addr is wave-uniform and travels in M0).  Written as inline assembly so
// that the compiler does not serialise later LDS reads of the *other* stage behind it; the
// kernel waits for these loads itself (s_waitcnt vmcnt) before the barrier that publishes a stage.
__device__ __forceinline__ void dma16(const void* gsrc, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gsrc)
                 : "memory", "m0");
}

// The same with the address split into a wave-uniform 64-bit base (SGPR pair) and a per-lane 32-bit byte
// offset (kept below 2^31): nothing but a scalar add is needed to move the base from one k-stage to the next.
__device__ __forceinline__ void dma16_s(const void* sbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// Walk of the n-tiles x m-tiles grid of one expert: n-tiles in super-columns of kSuperN,
// m-tiles next, the n-tiles of the super-column fastest.  32 consecutive tiles (what one
// XCD runs at a time) then form a block of 8 m-tiles x 4 n-tiles (or all m-tiles x more
// n-tiles for a short expert), which bounds the operand traffic from beyond the XCD's L2.
constexpr int kSuperN = 4;
__device__ __forceinline__ void walk_tile(int local, int nm, int n_tiles, int& m, int& nt) {
    const int full = (n_tiles / kSuperN) * kSuperN * nm;
    int width = kSuperN, nbase = 0;
    if (local >= full) {
        local -= full;
        nbase = (n_tiles / kSuperN) * kSuperN;
        width = n_tiles - nbase;
    } else {
        const int sc = local / (kSuperN * nm);
        local -= sc * kSuperN * nm;
        nbase = sc * kSuperN;
    }
    m = local / width;
    nt = nbase + (local - m * width);
}

// Workgroups are dealt round-robin to the 8 XCDs.  Hand out the logical tile order in
// blocks of 32 (one block = what the 32 CUs of one XCD run together); consecutive blocks go
// to different XCDs, so the XCDs work on neighbouring blocks and share panels in the
// memory-side cache.  The grid is a multiple of 256 workgroups.
__device__ __forceinline__ int logical_tile(int wg) {
    const int xcd = wg & 7, idx = wg >> 3;
    return (((idx >> 5) * 8 + xcd) << 5) + (idx & 31);
}

template <int N>
struct IntTag {
    static constexpr int value = N;
};

struct TileDesc {
    int e, m0, m_lim, n0, kbeg, kend, nk;  // nk = k-stages per K segment
    bool valid;
    bool half;  // ragged M: at most TM/2 live rows (the tail of an expert): computed as a 128 x 256 tile
};

// The kernel is persistent: one workgroup per CU.  Inside a tile the DMA loads run one k-stage ahead of
// the MFMAs (two stage buffers); the first two stages of the next tile are requested before the current
// tile's epilogue, so they arrive while the epilogue runs (no workgroup relaunch, no cold prologue per tile).
//
// Which tiles a workgroup runs.  Without GArgs::sched: logical_tile(blockIdx.x + r * gridDim.x), r = 0, 1, ...
// With it: the logical tile order is cut into blocks of 32, block b belongs to the queue of XCD b % 8, and
// the 32 workgroups of an XCD draw from their queue with an atomic counter (draw c of queue x is tile
// ((c / 32) * 8 + x) * 32 + c % 32), then from the queues of the other XCDs once theirs is empty.  Tiles
// differ in cost (128-row tails, experts of different row counts in wgrad), so drawing evens out the
// finish times, while an XCD still works on one block of neighbouring tiles at a time.  The draw for the
// next tile is made when a tile starts (one lane; its latency hides behind the main loop), reaches LDS
// before the last barrier of the main loop and is read by all wavefronts after it.
template <int AT, int BT, bool DUAL, int EPI, bool RAGK>
__global__ __launch_bounds__(kThreads) void gg256_kernel(const GArgs g) {
    static_assert(RAGK ? (AT == 1 && BT == 0) : (AT == 0), "operand forms");
    static_assert(!(DUAL && BT == 1), "two B matrices are taken in k-row form only");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    int32_t* t_off = reinterpret_cast<int32_t*>(smem + kTableOff);  // [E+1] rows of each expert
    int32_t* t_pref = t_off + MOE_MAX_EXPERTS + 1;                              // [E+1] tiles before expert e
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / kWN, wn = wave % kWN;  // 2 x kWN wavefronts, 128 rows x 32*NJ columns each
    const int n_out = DUAL ? TN / 2 : TN;     // output columns per tile
    const int n_tiles = (g.N + n_out - 1) / n_out;
    const int m_tiles_k = (g.M + TM - 1) / TM;  // ragged K only

    // ---- expert table in LDS: rows of each expert and the number of tiles before it ----
    for (int i = threadIdx.x; i <= g.E; i += kThreads) t_off[i] = g.offsets[i];
    __syncthreads();
    if (wave == 0) {  // exclusive scan of the per-expert tile counts: 4 experts per lane, then across lanes
        int c[4], sum = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = lane * 4 + u;
            c[u] = 0;
            if (e < g.E) c[u] = RAGK ? m_tiles_k * n_tiles : ((t_off[e + 1] - t_off[e] + TM - 1) / TM) * n_tiles;
            sum += c[u];
        }
        int incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        int run = incl - sum;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = lane * 4 + u;
            if (e <= g.E) t_pref[e] = run;
            run += c[u];
        }
        // E == MOE_MAX_EXPERTS: the total belongs to "lane 64"; the last lane holds it after its four experts
        if (lane == 63) t_pref[MOE_MAX_EXPERTS] = run;
    }
    __syncthreads();
    // Ragged M in the fixed tile order: when the last round of tiles fills at most half of the workgroups, its
    // tiles are cut into their upper and lower 128 rows (logical tiles split_from + 2i and + 2i + 1), so that
    // the round costs a 128-row tile's time instead of a full one's.
    int total_tiles = t_pref[g.E], split_from = total_tiles;
    if constexpr (!RAGK) {
        const int left = total_tiles % (int)gridDim.x;
        if (g.sched == nullptr && left > 0 && 2 * left <= (int)gridDim.x) {
            split_from = total_tiles - left;
            total_tiles += left;
        }
    }
    // ---- tile queues ----
    int* s_draw = reinterpret_cast<int*>(t_pref + MOE_MAX_EXPERTS + 1);  // [0]: synchronous draws, [1]: the draw made ahead
    const bool dyn = g.sched != nullptr;
    const int xcd = blockIdx.x & 7;
    int qx = 0;  // queues exhausted so far; the current one is that of XCD (xcd + qx) % 8
    auto queue_counter = [&]() { return g.sched + ((xcd + qx) & 7) * kSchedStride; };
    auto tile_of_draw = [&](int c) { return (((c >> 5) * 8 + ((xcd + qx) & 7)) << 5) + (c & 31); };
    // A draw that every wavefront waits for (the first tile, and the end phase when a queue has run dry);
    // returns a tile index < total_tiles, or total_tiles when all eight queues are empty.  With `probe` the
    // eight counters are read first (one round trip) and the queues already empty are skipped without
    // drawing from them: a workgroup whose queue has run dry near the end of the kernel leaves after one
    // round trip, not eight.
    auto draw_now = [&](bool probe) -> int {
        for (;;) {
            if (probe) {
                if (threadIdx.x < 64) {
                    bool live = false;
                    if (threadIdx.x < 8 && (int)threadIdx.x >= qx) {
                        const int x = (xcd + threadIdx.x) & 7;
                        const int c = (int)__hip_atomic_load(g.sched + x * kSchedStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const int L = (((c >> 5) * 8 + x) << 5) + (c & 31);
                        live = c >= 0 && L >= 0 && L < total_tiles;
                    }
                    const uint64_t m = __ballot(live);
                    if (threadIdx.x == 0) s_draw[0] = m ? __builtin_ctzll(m) : 8;
                }
                __syncthreads();
                qx = s_draw[0];
                __syncthreads();
            }
            if (qx >= 8) return total_tiles;
            if (threadIdx.x == 0)
                s_draw[0] = (int)__hip_atomic_fetch_add(queue_counter(), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const int c = s_draw[0];
            __syncthreads();
            const int L = tile_of_draw(c);
            if (c >= 0 && L >= 0 && L < total_tiles) return L;
            ++qx;
            probe = true;
        }
    };
    auto decode = [&](int L) -> TileDesc {
        TileDesc t;
        t.valid = L < total_tiles;
        t.e = 0; t.m0 = 0; t.m_lim = 0; t.n0 = 0; t.kbeg = 0; t.kend = 0; t.nk = 0;
        t.half = false;
        if (!t.valid) return t;
        int part = -1;  // which half of a split tile
        if (L >= split_from) {
            part = (L - split_from) & 1;
            L = split_from + ((L - split_from) >> 1);
        }
        int m, nt;
        if constexpr (RAGK) {
            const int per = m_tiles_k * n_tiles;
            const int oi = L / per;
            t.e = g.order ? g.order[oi] : oi;  // heaviest experts first
            walk_tile(L - oi * per, m_tiles_k, n_tiles, m, nt);
            t.m0 = m * TM;
            t.m_lim = g.M;
            t.kbeg = t_off[t.e];
            t.kend = t_off[t.e + 1];
        } else {
            // the expert whose tile range holds L: every lane tests a few experts, a ballot picks it
            int found = 0;
            for (int j = 0; j < MOE_MAX_EXPERTS / 64; ++j) {
                const int e = lane + 64 * j;
                const bool hit = e < g.E && t_pref[e] <= L && L < t_pref[e + 1];
                const uint64_t bal = __ballot(hit);
                if (bal) found = 64 * j + __builtin_ctzll(bal);
            }
            t.e = __builtin_amdgcn_readfirstlane(found);
            const int b = t_off[t.e], en = t_off[t.e + 1];
            walk_tile(L - t_pref[t.e], (en - b + TM - 1) / TM, n_tiles, m, nt);
            t.m0 = b + m * TM;
            t.m_lim = en;
            t.kend = g.K;
            if (part >= 0) {  // rows [m0 + 128*part, m0 + 128*part + 128) of the tile, as far as the expert reaches
                t.m0 += part * (TM / 2);
                t.m_lim = min(en, t.m0 + TM / 2);
            }
        }
        t.n0 = nt * n_out;
        t.nk = (t.kend - t.kbeg + TK - 1) / TK;  // exact when M is ragged (K % 64 == 0)
        if (!RAGK && t.m0 >= t.m_lim) t.nk = 0;   // the lower half of a tile of at most 128 rows: nothing to do
        t.e = __builtin_amdgcn_readfirstlane(t.e);
        t.m0 = __builtin_amdgcn_readfirstlane(t.m0);
        t.m_lim = __builtin_amdgcn_readfirstlane(t.m_lim);
        t.n0 = __builtin_amdgcn_readfirstlane(t.n0);
        t.kbeg = __builtin_amdgcn_readfirstlane(t.kbeg);
        t.kend = __builtin_amdgcn_readfirstlane(t.kend);
        t.nk = __builtin_amdgcn_readfirstlane(t.nk);
        if constexpr (!RAGK) t.half = t.m_lim - t.m0 <= TM / 2;
        return t;
    };

    // ================= issue side: DMA loads of k-stage s into stage buffer s & 1 =================
    const int64_t lda = g.lda, ldb = g.ldb;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_AS char*)smem;
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * (CPW * 1024));
    // row form: chunk c = wave*CPW + i covers rows 8c .. 8c+7; lane -> row 8c + lane/8, slot lane%8
    // k-row form: chunk c covers k-rows 2c, 2c+1; lane -> k-row 2c + lane/32, slot lane%32
    // k-row form, two matrices: chunk c covers k-rows 4(c%16) .. +3 of matrix c/16 (wavefronts 0-3 load the
    //   first matrix, 4-7 the second); lane -> k-row 4(c%16) + lane/16, slot lane%16
    TileDesc di;                  // tile whose stages are being issued
    di.valid = false; di.half = false; di.e = 0; di.m0 = 0; di.m_lim = 0; di.n0 = 0; di.kbeg = 0; di.kend = 0; di.nk = 0;
    // Ragged M: per-lane byte offsets of this lane's 16-byte pieces relative to a wave-uniform base of the tile
    // (sA / sB per K segment; with two B matrices sB is the base of the matrix this wavefront loads).
    // Ragged K: byte offsets relative to the first k-row of the stage (the base moves by scalar adds); only a
    // stage that reaches past the expert's last row forms full per-lane addresses.
    constexpr bool kBDual = DUAL && BT == 0;   // the B tile is two half-width k-row tiles
    const int b_mat = kBDual ? __builtin_amdgcn_readfirstlane(wave / (kWaves / 2)) : 0;  // the matrix this wavefront's B chunks come from
    uint32_t a_off[CPW], b_off[CPW];
    const char* sA[2];
    const char* sB[2];
    const bf16_t* iA[2];
    const bf16_t* iB[2];   // ragged K: the matrix this wavefront's B chunks come from
    int qa_row[CPW], qb_row[CPW];  // k-row form: the k-row inside the stage of this lane's piece in chunk i
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int c = wave * CPW + i;
        qa_row[i] = c * 2 + (lane >> 5);
        qb_row[i] = kBDual ? (c & 15) * 4 + (lane >> 4) : c * 2 + (lane >> 5);
    }

    auto setup_issue = [&]() {
#pragma unroll
        for (int sgi = 0; sgi < 2; ++sgi) {
            const int q = sgi < g.nseg ? sgi : 0;
            const int64_t eoff = RAGK ? 0 : (int64_t)weight_index(g, di.e) * g.strideB;
            iA[sgi] = static_cast<const bf16_t*>(g.seg[q].A);
            iB[sgi] = static_cast<const bf16_t*>(kBDual && b_mat ? g.seg[q].B2 : g.seg[q].B) + eoff;
        }
#pragma unroll
        for (int sgi = 0; sgi < 2; ++sgi) {
            if constexpr (AT == 0) sA[sgi] = reinterpret_cast<const char*>(iA[sgi] + (int64_t)di.m0 * lda);
            if constexpr (BT == 1) sB[sgi] = reinterpret_cast<const char*>(iB[sgi] + (int64_t)di.n0 * ldb);
            else sB[sgi] = reinterpret_cast<const char*>(iB[sgi] + di.n0);
        }
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            const int c = wave * CPW + i;
            if constexpr (AT == 0) {
                const int r = c * 8 + (lane >> 3);
                const int last = di.m_lim - 1 - di.m0;  // rows past the expert's end: any valid row (masked at the store)
                const int rl = r < last ? r : last;
                a_off[i] = ((uint32_t)rl * (uint32_t)lda + ((lane & 7) ^ swz_rows(r)) * 8) * 2;
            } else {
                int col = di.m0 + ((lane & 31) ^ swz_krow(qa_row[i])) * 8;
                col = col < g.M ? col : g.M - 8;
                a_off[i] = ((uint32_t)qa_row[i] * (uint32_t)lda + (uint32_t)col) * 2;
            }
            if constexpr (BT == 1) {
                const int r = c * 8 + (lane >> 3);
                const int last = g.N - 1 - di.n0;
                const int rl = r < last ? r : last;
                b_off[i] = ((uint32_t)rl * (uint32_t)ldb + ((lane & 7) ^ swz_rows(r)) * 8) * 2;
            } else {
                int col;
                if constexpr (kBDual) col = di.n0 + ((lane & 15) ^ swz_krow(qb_row[i])) * 8;
                else col = di.n0 + ((lane & 31) ^ swz_krow(qb_row[i])) * 8;
                col = col < g.N ? col : g.N - 8;
                if constexpr (RAGK) b_off[i] = ((uint32_t)qb_row[i] * (uint32_t)ldb + (uint32_t)col) * 2;
                else b_off[i] = ((uint32_t)qb_row[i] * (uint32_t)ldb + (uint32_t)(col - di.n0)) * 2;
            }
        }
    };
    // k-stage `stage` of tile di -> stage buffer `buf`: always exactly 2*CPW DMA instructions per wavefront,
    // numbered idx = 0 .. 2*CPW-1 (A chunks first); issue_part issues the idx range [lo, hi).
    auto issue_part = [&](int stage, int buf, int lo, int hi) {
        const int sg = stage >= di.nk ? 1 : 0;
        const int k0 = di.kbeg + (stage - sg * di.nk) * TK;
        const uint32_t st = __builtin_amdgcn_readfirstlane(lds_wave + buf * kStageBytes);
        if constexpr (!RAGK) {
            const char* Ab = (sg ? sA[1] : sA[0]) + (int64_t)k0 * 2;
            const char* Bb = (sg ? sB[1] : sB[0]) + (BT == 1 ? (int64_t)k0 * 2 : (int64_t)k0 * ldb * 2);
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                if (i < lo || i >= hi) continue;
                dma16_s(Ab, a_off[i], st + i * 1024);
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                if (CPW + i < lo || CPW + i >= hi) continue;
                dma16_s(Bb, b_off[i], st + kBOff + i * 1024);
            }
        } else {
            const char* Ab = reinterpret_cast<const char*>(sg ? iA[1] : iA[0]) + (int64_t)k0 * lda * 2;
            const char* Bb = reinterpret_cast<const char*>(sg ? iB[1] : iB[0]) + (int64_t)k0 * ldb * 2;
            if (k0 + TK <= di.kend) {  // (wave-uniform) every k-row of the stage belongs to the expert
#pragma unroll
                for (int i = 0; i < CPW; ++i) {
                    if (i < lo || i >= hi) continue;
                    dma16_s(Ab, a_off[i], st + i * 1024);
                }
#pragma unroll
                for (int i = 0; i < CPW; ++i) {
                    if (CPW + i < lo || CPW + i >= hi) continue;
                    dma16_s(Bb, b_off[i], st + kBOff + i * 1024);
                }
            } else {
                const int left = di.kend - k0;  // k-rows of the stage that exist, 1 .. TK-1
#pragma unroll
                for (int i = 0; i < CPW; ++i) {
                    if (i < lo || i >= hi) continue;
                    // k-rows past the expert's rows read a row of zeros: they add nothing to the sums
                    const char* src = qa_row[i] < left ? Ab + a_off[i]
                                                       : static_cast<const char*>(g.zero_row) + (lane & 31) * 16;
                    dma16(src, st + i * 1024);
                }
#pragma unroll
                for (int i = 0; i < CPW; ++i) {
                    if (CPW + i < lo || CPW + i >= hi) continue;
                    // any valid (finite) row: it meets zeros
                    const int over = qb_row[i] < left ? 0 : qb_row[i] - (left - 1);
                    dma16(Bb + (b_off[i] - (uint32_t)over * (uint32_t)ldb * 2), st + kBOff + i * 1024);
                }
            }
        }
    };
    auto issue = [&](int stage, int buf) { issue_part(stage, buf, 0, 2 * CPW); };

    // ================= compute side =================
    const int l32 = lane & 31, kg = lane >> 5;
    const int a_sw = swz_rows(l32);  // the same for all tiles of 32 rows
    // k-row form (transposing reads): lane -> group g16 = lane/16, i16 = lane%16
    const int g16 = lane >> 4, i16 = lane & 15;
    const int tr_krow = (g16 >> 1) * 8 + (i16 >> 2);  // + kk*16 + t*4
    const int tr_sw = swz_krow(tr_krow);              // kk*16 + t*4 do not change the swizzle
    const int tr_lane_col = (g16 & 1) * 16 + (i16 & 3) * 4;
    constexpr int kBRow = kBDual ? 256 : 512;         // bytes per k-row of the B tile
    int a_rd[4], b_rd[NJ];  // byte offsets inside the operand tile, without the k-step term
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (AT == 0) {
            a_rd[i] = (wm * 128 + i * 32 + l32) * 128;
        } else {
            const int col = wm * 128 + i * 32 + tr_lane_col;
            a_rd[i] = tr_krow * 512 + (((col >> 3) ^ tr_sw) << 4) + (col & 7) * 2;
        }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if constexpr (BT == 1) {
            // DUAL with row-form B does not occur (the two-matrix products have their weights in k-row form)
            b_rd[j] = (wn * NJ * 32 + j * 32 + l32) * 128;
        } else if constexpr (kBDual) {
            // blocks j < NJ/2 lie in the first matrix' half of the B tile, the others in the second
            const int col = wn * (NJ / 2) * 32 + (j % (NJ / 2)) * 32 + tr_lane_col;
            b_rd[j] = (j / (NJ / 2)) * (kBOff / 2) + tr_krow * 256 + (((col >> 3) ^ tr_sw) << 4) + (col & 7) * 2;
        } else {
            const int col = wn * NJ * 32 + j * 32 + tr_lane_col;
            b_rd[j] = tr_krow * 512 + (((col >> 3) ^ tr_sw) << 4) + (col & 7) * 2;
        }
    }
    // fragments of k-step kk (0 .. kSteps-1) of a stage -> registers.  B first: the MFMAs below walk
    // a[0] x b[0..1], a[1] x b[0..1], ..., so the operands requested last are the ones needed last.
    // NI = row blocks per wavefront: 4 (128 x 64 per wavefront, 256-row tile) or 2 (64 x 64, 128-row tile:
    // wavefront row wm then starts at row 64*wm, which is taken off the A offsets).
    auto load_frags = [&](auto ni_tag, const char* st, int kk, bf16x8 (&a)[4], bf16x8 (&b)[NJ]) {
        constexpr int NI = decltype(ni_tag)::value;
        const char* sb = st + kBOff;
        if constexpr (NI == 2 && AT == 0) st -= wm * 64 * 128;
        const int rowform = ((kk * 2 + kg) ^ a_sw) << 4;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if constexpr (BT == 1) {
                b[j] = *reinterpret_cast<const bf16x8*>(sb + b_rd[j] + rowform);
            } else {
                const char* p = sb + b_rd[j] + kk * (16 * kBRow);
                const bf16x4 h0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_AS bf16x4*)p);
                const bf16x4 h1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_AS bf16x4*)(p + 4 * kBRow));
                b[j] = __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if constexpr (AT == 0) {
                a[i] = *reinterpret_cast<const bf16x8*>(st + a_rd[i] + rowform);
            } else {
                const char* p = st + a_rd[i] + kk * 8192;
                const bf16x4 h0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_AS bf16x4*)p);
                const bf16x4 h1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_AS bf16x4*)(p + 2048));
                a[i] = __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    // The MFMAs take the B fragment as their first operand and the A fragment as their second: each 32x32
    // block is accumulated transposed, so that a lane holds runs of four consecutive COLUMNS of one row
    // (row = lane%32, column = 8*(r/4) + 4*(lane/32) + r%4) and the epilogues write whole 8- or 16-byte
    // pieces of output rows without exchanging values between lanes.
    f32x16 acc[4][NJ];
    auto zero_acc = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    };
    auto mma = [&](auto ni_tag, const bf16x8 (&a)[4], const bf16x8 (&b)[NJ]) {
        constexpr int NI = decltype(ni_tag)::value;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    };
    // The accumulators as operands of an empty volatile asm: every MFMA issued so far stays in front of
    // the waits and the barrier that follow (instruction selection otherwise moves most of a k-step's
    // MFMAs behind the barrier, which then drains the matrix pipe while the wavefronts wait).
    auto pin_one = [](f32x16& v) {
        asm volatile("" : "+v"(v));
    };
    auto pin_acc = [&](auto ni_tag) {
        constexpr int NI = decltype(ni_tag)::value;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) pin_one(acc[i][j]);
    };

    // ---- epilogue of one tile.  The accumulators (row = lane%32, col = 8*(r/4) + 4*(lane/32) + r%4
    // inside a 32x32 block) go through LDS, 16 KB (bf16) or 32 KB (fp32) at a time, so that global memory
    // sees 16-byte accesses along rows.  `stg` is the staging area; both stage buffers already receive the
    // next tile's first two stages (but for the chunks the staging area overlaps).
    auto epilogue_zero = [&](const TileDesc& t) {  // ragged K, expert without rows: exact zeros, no staging needed
        const int64_t cbase = RAGK ? (int64_t)t.e * g.strideC : 0;
        {
            constexpr int PPR = 32;
            for (int item = threadIdx.x; item < 256 * PPR; item += kThreads) {
                const int row = t.m0 + item / PPR;
                int col = (item % PPR) * 8;
                bf16_t* dst = static_cast<bf16_t*>(g.C0);
                if (DUAL && col >= 128) { col -= 128; dst = static_cast<bf16_t*>(g.C1); }
                if (row < t.m_lim && t.n0 + col < g.N) {
                    if constexpr (EPI == EPI_STORE_F32) {
                        float* d = static_cast<float*>(g.C0) + cbase + (int64_t)row * g.ldc + t.n0 + col;
                        for (int z = 0; z < 8; ++z) d[z] = 0.f;
                    } else {
                        *reinterpret_cast<u32x4*>(dst + cbase + (int64_t)row * g.ldc + t.n0 + col) = (u32x4){0, 0, 0, 0};
                    }
                }
            }
        }
    };
    auto epilogue = [&](const TileDesc& t, char* stg) {
        // The thread's coordinates, derived afresh from an opaque copy of its index: everything the epilogue
        // computes from them is then recomputed per tile (a few VALU instructions) instead of living in
        // registers through the main loop, where the budget is 256 VGPRs.
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63, wave = tid >> 6;
        const int wm = wave / kWN, wn = wave % kWN, l32 = lane & 31, kg = lane >> 5;
        const int64_t cbase = RAGK ? (int64_t)t.e * g.strideC : 0;
        // a 128-row tile holds two row blocks per wavefront, the rows of wavefront row 1 start at 64
        const bool half = !RAGK && t.half;
        const int ni = half ? 2 : 4, wrows = half ? 64 : 128;
        if constexpr (EPI == EPI_STORE_F32) {  // narrow fp32 output (gate weight gradient): direct stores
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i >= ni) continue;
                const int row = t.m0 + wm * wrows + i * 32 + l32;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const int col = t.n0 + wn * NJ * 32 + j * 32 + g4 * 8 + kg * 4;
                        if (row >= t.m_lim) continue;
                        float* d = static_cast<float*>(g.C0) + cbase + (int64_t)row * g.ldc + col;
#pragma unroll
                        for (int z = 0; z < 4; ++z)
                            if (col + z < g.N) d[z] = acc[i][j][4 * g4 + z];
                    }
            }
        } else if constexpr (EPI == EPI_DH || EPI == EPI_DHP || EPI == EPI_ADD) {
            // dH in fp32 through LDS, 64 rows x 128 columns at a time; then 8 columns per thread: read A, B,
            // write H = silu(A)*B, dA = dH*B*silu'(A), dB = dH*silu(A).  Staging rows are 512 B; a lane writes
            // 16-byte pieces of its row, and the piece index is XORed with row%32 so that the 32 rows of a
            // write fall into different banks.
            // EPI_DHP is the same epilogue for activations saved as products (P = B*silu'(A), Q = silu(A); H is
            // saved too and not rewritten): dA = dH*P, dB = dH*Q, two multiplications per element.
            // The arithmetic bounds this epilogue (about 20 VALU issue slots per element, the exponential and
            // the reciprocal at a quarter of the rate), so nothing else may add to it: the global operands of
            // pass q+1 (saved A and B, or the old C) are requested at the top of pass q into a second set of
            // registers and have a whole pass to arrive.  Every lane loads (dead items from a clamped address)
            // and every lane consumes what it loaded; only the stores are predicated.  The wait for the
            // operands of pass q leaves the loads of pass q+1 outstanding: vmcnt(loads per pass); loads return in
            // order, so whatever the stores of pass q-1 do, the older loads have landed when at most the
            // younger ones are pending.
            constexpr int IPT = 64 * 16 / kThreads;                  // 8-column items per thread and pass
            constexpr int NLD = (EPI == EPI_ADD ? 1 : 2) * IPT;      // loads per thread and pass
            static_assert(NLD == 2 || NLD == 4, "the waits below are written for these counts");
            const int64_t tile_base = cbase + (int64_t)t.m0 * g.ldc + t.n0;
            uint32_t ldc_u = (uint32_t)g.ldc;  // (opaque per tile, as in the bf16 path)
            asm volatile("" : "+s"(ldc_u));
            const int last_row = t.m_lim - 1 - t.m0, last_col = g.N - 8 - t.n0;
            u32x4 pre0[2][IPT], pre1[2][IPT];
            auto load_pass = [&](int q, u32x4 (&p0)[IPT], u32x4 (&p1)[IPT]) {
#pragma unroll
                for (int u = 0; u < IPT; ++u) {
                    const int item = tid + u * kThreads;
                    const int sr = item >> 4, cg = item & 15;
                    const int trow = (sr >> 5) * wrows + (q >> 1) * 32 + (sr & 31), tcol = (q & 1) * 128 + cg * 8;
                    const int lrow = trow < last_row ? trow : last_row, lcol = tcol < last_col ? tcol : last_col;
                    const uint32_t off = (uint32_t)lrow * ldc_u + (uint32_t)lcol;
                    if constexpr (EPI == EPI_ADD) {
                        p0[u] = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(g.C0) + tile_base + off);
                        p1[u] = (u32x4){0, 0, 0, 0};
                    } else {
                        p0[u] = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(g.S0) + tile_base + off);
                        p1[u] = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(g.S1) + tile_base + off);
                    }
                }
            };
            // (the number of passes is a compile-time constant of each instance, so that the compiler's
            // bookkeeping of pending loads is exact and it adds no waits of its own in the next tile's loop)
            auto run_passes = [&](auto np_tag) {
            constexpr int NP = decltype(np_tag)::value;
            load_pass(0, pre0[0], pre1[0]);
            __builtin_amdgcn_sched_barrier(0);  // the loads of pass 0 stay in front of those of pass 1
#pragma unroll
            for (int q = 0; q < NP; ++q) {
                const int i = q >> 1, p = q & 1;
                const bool more = q + 1 < NP;
                if (more) load_pass(q + 1, pre0[(q + 1) & 1], pre1[(q + 1) & 1]);
                {
                    const int sr = wm * 32 + l32;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int g4 = 0; g4 < 4; ++g4) {
                            const int tcol = wn * NJ * 32 + j * 32 + g4 * 8 + kg * 4;  // column inside the 256-wide tile
                            const int piece = ((tcol & 127) >> 2) ^ (sr & 31);
                            if ((tcol >> 7) == p)
                                *reinterpret_cast<f32x4v*>(stg + sr * 512 + piece * 16) =
                                    (f32x4v){acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]};
                        }
                }
                __syncthreads();
                // (builtins, so that the compiler's own bookkeeping of pending loads agrees)
                if (more) __builtin_amdgcn_s_waitcnt(NLD == 4 ? 0x0F74 : 0x0F72);  // vmcnt(NLD)
                else __builtin_amdgcn_s_waitcnt(0x0F70);                           // vmcnt(0)
#pragma unroll
                for (int u = 0; u < IPT; ++u) {
                    const int item = tid + u * kThreads;
                    const int sr = item >> 4, cg = item & 15;
                    const int trow = (sr >> 5) * wrows + i * 32 + (sr & 31), tcol = p * 128 + cg * 8;
                    const bool live = t.m0 + trow < t.m_lim && t.n0 + tcol < g.N;
                    const uint32_t off = (uint32_t)trow * ldc_u + (uint32_t)tcol;
                    const int sw = sr & 31;
                    const f32x4v d0 = *reinterpret_cast<const f32x4v*>(stg + sr * 512 + ((2 * cg) ^ sw) * 16);
                    const f32x4v d1 = *reinterpret_cast<const f32x4v*>(stg + sr * 512 + ((2 * cg + 1) ^ sw) * 16);
                    const float dh[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
                    if constexpr (EPI == EPI_ADD) {  // C += tile: the bf16 values plus the tile in fp32, one rounding
                        const u32x4 old = pre0[q & 1][u];
                        u32x4 o;
#pragma unroll
                        for (int z = 0; z < 4; ++z) {
                            const float lo = __uint_as_float(old[z] << 16) + dh[2 * z];
                            const float hi = __uint_as_float(old[z] & 0xFFFF0000u) + dh[2 * z + 1];
                            o[z] = pack_bf16x2(lo, hi);
                        }
                        if (live) *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C0) + tile_base + off) = o;
                    } else {
                        const u32x4 av = pre0[q & 1][u], bv = pre1[q & 1][u];
                        u32x4 oh, oa, ob;
                        if constexpr (EPI == EPI_DHP) {
#pragma unroll
                            for (int z4 = 0; z4 < 4; ++z4) {
                                const float p_lo = __uint_as_float(av[z4] << 16), p_hi = __uint_as_float(av[z4] & 0xFFFF0000u);
                                const float q_lo = __uint_as_float(bv[z4] << 16), q_hi = __uint_as_float(bv[z4] & 0xFFFF0000u);
                                oa[z4] = pack_bf16x2(dh[2 * z4] * p_lo, dh[2 * z4 + 1] * p_hi);
                                ob[z4] = pack_bf16x2(dh[2 * z4] * q_lo, dh[2 * z4 + 1] * q_hi);
                            }
                            if (live) {
                                *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C1) + tile_base + off) = oa;
                                *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C2) + tile_base + off) = ob;
                            }
                            continue;
                        }
#pragma unroll
                        for (int z4 = 0; z4 < 4; ++z4) {
                            float hh[2], da[2], db[2];
#pragma unroll
                            for (int z = 0; z < 2; ++z) {
                                const float A = __uint_as_float(z ? (av[z4] & 0xFFFF0000u) : (av[z4] << 16));
                                const float B = __uint_as_float(z ? (bv[z4] & 0xFFFF0000u) : (bv[z4] << 16));
                                const float sg = sigmoid_f(A);             // one exp and one reciprocal per element
                                const float sA = A * sg;                   // silu(A)
                                const float gr = sg + sA * (1.0f - sg);    // silu'(A) = s (1 + A (1 - s))
                                hh[z] = sA * B;
                                da[z] = dh[2 * z4 + z] * B * gr;
                                db[z] = dh[2 * z4 + z] * sA;
                            }
                            oh[z4] = pack_bf16x2(hh[0], hh[1]);
                            oa[z4] = pack_bf16x2(da[0], da[1]);
                            ob[z4] = pack_bf16x2(db[0], db[1]);
                        }
                        if (live) {
                            *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C0) + tile_base + off) = oh;
                            *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C1) + tile_base + off) = oa;
                            *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C2) + tile_base + off) = ob;
                        }
                    }
                }
                __syncthreads();
            }
            };
            if (ni == 4) run_passes(IntTag<8>{});  // pass q: row block q/2, column half q%2
            else run_passes(IntTag<4>{});          // (a 128-row tile has two row blocks)
        } else {
            // bf16 tiles: stage [RPP rows][ROWB bytes] with swizzled 16-byte pieces, then 16 bytes per lane along
            // rows.  A pass fills one of two 16 KB areas: block i of both wavefront rows (64 rows of 256 B) or of
            // one wavefront row (32 rows of 512 B).  The areas take the passes in turn, so one barrier per pass is
            // enough: a wavefront that writes pass p+2 has passed the barrier of pass p+1, which every wavefront
            // reaches only after it has read pass p.
            constexpr int ROWB = (DUAL && EPI == EPI_SWIGLU) ? 256 : 512;
            constexpr int PPR = ROWB / 16;               // pieces per row
            constexpr int RPP = kStagingBytes / 2 / ROWB;  // rows per pass: 64 or 32
            constexpr int ITEMS = RPP * PPR / kThreads;   // 16-byte pieces per thread and pass
            static_assert(ITEMS * kThreads == RPP * PPR, "a pass is a whole number of pieces per thread");
            // Four accumulators r = 4g .. 4g+3 of a lane are four consecutive columns of its row: one 8-byte
            // LDS write.  Staging swizzle: piece ^ (row % PPR), so that the rows of one write (32 lanes, 32
            // rows, the same piece) fall into different banks.
            auto stg_sw = [](int sr) { return sr & (PPR - 1); };
            auto put4 = [&](char* sb, int g4, int colbase, float v0, float v1, float v2, float v3) {
                u32x2 o;
                o[0] = pack_bf16x2(v0, v1);
                o[1] = pack_bf16x2(v2, v3);
                const int sr = (RPP == 64 ? wm * 32 : 0) + l32;
                const int col = colbase + g4 * 8 + kg * 4;
                *reinterpret_cast<u32x2*>(sb + sr * ROWB + (((col >> 3) ^ stg_sw(sr)) << 4) + (col & 7) * 2) = o;
            };
            const int64_t tile_base = cbase + (int64_t)t.m0 * g.ldc + t.n0;
            // (opaque per tile: the store offsets below do not change from tile to tile, and the compiler would
            // otherwise compute them once per kernel and keep them in scratch memory)
            uint32_t ldc_u = (uint32_t)g.ldc;
            asm volatile("" : "+s"(ldc_u));
            // h: the wavefront row whose 32 rows the pass holds (RPP == 32)
            auto flush = [&](const char* sb, int i, int h, bf16_t* dst0, bf16_t* dst1, int cols0) {
                __syncthreads();
                u32x4 v[ITEMS];
#pragma unroll
                for (int u = 0; u < ITEMS; ++u) {
                    const int item = tid + u * kThreads;
                    const int sr = item / PPR, pc = item % PPR;
                    v[u] = *reinterpret_cast<const u32x4*>(sb + sr * ROWB + ((pc ^ stg_sw(sr)) << 4));
                }
#pragma unroll
                for (int u = 0; u < ITEMS; ++u) {
                    const int item = tid + u * kThreads;
                    const int sr = item / PPR, pc = item % PPR;
                    const int trow = (RPP == 64 ? (sr >> 5) : h) * wrows + i * 32 + (sr & 31);  // row inside the tile
                    int col = pc * 8;
                    bf16_t* dst = dst0;
                    if (dst1 && col >= cols0) { col -= cols0; dst = dst1; }
                    // (offsets inside a tile fit 32 bits: at most 256 rows of ldc < 2^22 elements)
                    const uint32_t off = (uint32_t)trow * ldc_u + (uint32_t)col;
                    if (t.m0 + trow < t.m_lim && t.n0 + col < g.N)
                        *reinterpret_cast<u32x4*>(dst + tile_base + off) = v[u];
                }
            };
            int pn = 0;  // passes so far
            auto next_buf = [&]() { return stg + ((pn++ & 1) ? kStagingBytes / 2 : 0); };  // the two areas in turn
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i >= ni) break;
                if constexpr (EPI == EPI_SWIGLU) {
                    for (int pass = 0; pass < (g.S0 ? 3 : 1); ++pass) {
                        char* sb = next_buf();
#pragma unroll
                        for (int j = 0; j < NJ / 2; ++j)
#pragma unroll
                            for (int g4 = 0; g4 < 4; ++g4) {
                                float v[4];
#pragma unroll
                                for (int z = 0; z < 4; ++z) {
                                    const float a = acc[i][j][4 * g4 + z], b = acc[i][j + NJ / 2][4 * g4 + z];
                                    if (pass == 0) {
                                        v[z] = silu_f(a) * b;
                                    } else if (!g.products) {
                                        v[z] = pass == 1 ? a : b;
                                    } else {  // P = b * silu'(a), Q = silu(a)
                                        const float sg = sigmoid_f(a), sA = a * sg;
                                        v[z] = pass == 1 ? b * (sg + sA * (1.0f - sg)) : sA;
                                    }
                                }
                                put4(sb, g4, wn * (NJ / 2) * 32 + j * 32, v[0], v[1], v[2], v[3]);
                            }
                        bf16_t* dst = pass == 0 ? static_cast<bf16_t*>(g.C0)
                                                : const_cast<bf16_t*>(static_cast<const bf16_t*>(pass == 1 ? g.S0 : g.S1));
                        flush(sb, i, 0, dst, nullptr, 0);
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        char* sb = next_buf();
                        if (wm == h) {
                            if constexpr (DUAL) {  // EPI_STORE2: first 128 columns -> C0, second 128 -> C1
#pragma unroll
                                for (int j = 0; j < NJ / 2; ++j)
#pragma unroll
                                    for (int g4 = 0; g4 < 4; ++g4) {
                                        const int r = 4 * g4;
                                        put4(sb, g4, wn * (NJ / 2) * 32 + j * 32, acc[i][j][r], acc[i][j][r + 1], acc[i][j][r + 2],
                                             acc[i][j][r + 3]);
                                        put4(sb, g4, 128 + wn * (NJ / 2) * 32 + j * 32, acc[i][j + NJ / 2][r], acc[i][j + NJ / 2][r + 1],
                                             acc[i][j + NJ / 2][r + 2], acc[i][j + NJ / 2][r + 3]);
                                    }
                            } else {  // EPI_STORE
#pragma unroll
                                for (int j = 0; j < NJ; ++j)
#pragma unroll
                                    for (int g4 = 0; g4 < 4; ++g4) {
                                        const int r = 4 * g4;
                                        put4(sb, g4, wn * NJ * 32 + j * 32, acc[i][j][r], acc[i][j][r + 1], acc[i][j][r + 2], acc[i][j][r + 3]);
                                    }
                            }
                        }
                        if constexpr (DUAL) flush(sb, i, h, static_cast<bf16_t*>(g.C0), static_cast<bf16_t*>(g.C1), 128);
                        else flush(sb, i, h, static_cast<bf16_t*>(g.C0), nullptr, 0);
                    }
                }
            }
            __syncthreads();  // the last two passes have been read: the chunks under the staging area may be requested
        }
    };

    // ================= the tiles of this workgroup =================
    // Per tile: stages 0 and 1 are in flight when its loop starts (both were requested before the previous
    // tile's epilogue, three chunks of stage 1 after it).  Iteration `it` runs the four k-steps of stage `it`; the barrier in
    // front of the last k-step publishes stage it+1 and frees the buffer of stage it, into which stage it+2 is
    // requested at once: a stage has one whole iteration (about 2 us) to land.
    bf16x8 fa[2][4], fb[2][NJ];
    int round = 0;
    auto static_tile = [&]() { return logical_tile(blockIdx.x + round++ * gridDim.x); };
    TileDesc t = decode(dyn ? draw_now(false) : static_tile());
    while (t.valid && t.nk == 0) {  // ragged K: experts without rows; ragged M: empty halves of split tiles
        if constexpr (RAGK) epilogue_zero(t);
        t = decode(dyn ? draw_now(false) : static_tile());
    }
    if (!t.valid) return;
    di = t;
    setup_issue();
    {
        const int tot0 = t.nk * g.nseg;
        for (int sq = 0; sq < kStages && sq < tot0; ++sq) issue(sq, sq);
    }
    // The main loop of one tile; NI as in load_frags.  `ahead` (lane 0 of wavefront 0): the queue draw made
    // when the tile started; it goes to LDS in front of the loop's last barrier.
    auto run_tile = [&](auto ni_tag, const int total, const int ahead) {
        constexpr int NI = decltype(ni_tag)::value;
        constexpr int kReads = (AT == 0 ? NI : 2 * NI) + (BT == 1 ? NJ : 2 * NJ);
        constexpr int kDeal = 2 * CPW / NI;                         // DMA instructions behind each row of MFMAs
        // stage 0 must have landed: behind it at most the 2*CPW loads of stage 1 are pending
        if (total >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * CPW) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        load_frags(ni_tag, smem, 0, fa[0], fb[0]);
        // k-steps 0 .. kSteps-2 of a stage: the fragments of the next k-step are read while the MFMAs of this one issue
        auto steps_before_barrier = [&](const char* st) {
#pragma unroll
            for (int kk = 0; kk < kSteps - 1; ++kk) {
                load_frags(ni_tag, st, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
                mma(ni_tag, fa[kk & 1], fb[kk & 1]);
                interleave_mfma_dsread<NI * NJ, kReads>();
            }
            pin_acc(ni_tag);
        };
        int it = 0;
        // ---- hot loop: branch-free ----
        for (; it + kStages < total; ++it) {
            const char* st = smem + (it & 1) * kStageBytes;
            const char* nx = smem + ((it + 1) & 1) * kStageBytes;
            steps_before_barrier(st);
            // this wavefront's reads of stage `it` have returned and its share of stage it+1 has landed
            // (nothing else is in flight: stage it+2 is requested below)
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __syncthreads();
            // last k-step: the DMA instructions of stage it+2 (and their address arithmetic) are dealt out
            // between the MFMAs, an equal share after each row of MFMA blocks, so that the matrix pipe stays
            // fed while they issue; the pins keep each row of MFMAs in front of its share.
            load_frags(ni_tag, nx, 0, fa[0], fb[0]);
#pragma unroll
            for (int i = 0; i < NI; ++i) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[1][j], fa[1][i], acc[i][j], 0, 0, 0);
                    pin_one(acc[i][j]);
                }
                issue_part(it + kStages, it & 1, i * kDeal, (i + 1) * kDeal);
                if (i < NI - 1) pin_one(acc[i + 1][0]);  // the next row's MFMAs read this value: they stay behind the DMA
            }
        }
        // ---- the last (up to two) stages: nothing left to issue for this tile ----
        for (; it < total; ++it) {
            const char* st = smem + (it & 1) * kStageBytes;
            const char* nx = smem + ((it + 1) & 1) * kStageBytes;
            steps_before_barrier(st);
            const int rem = total - 1 - it;  // stages after this one, all issued already
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            if (rem == 0 && threadIdx.x == 0) s_draw[1] = ahead;  // (every load of this wavefront has returned)
            __syncthreads();
            if (rem > 0) load_frags(ni_tag, nx, 0, fa[0], fb[0]);
            mma(ni_tag, fa[1], fb[1]);
            interleave_mfma_dsread<NI * NJ, kReads>();
        }
    };
    // The first two stages of the next tile are requested before this tile's epilogue, all but the chunks
    // of the second stage buffer that lie under the staging area: wavefront 7 requests those after it.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    constexpr int kEarly = 2 * CPW - kDeferChunks;
    for (;;) {
        const int total = t.nk * g.nseg;
        zero_acc();
        // The draw for the next tile, as inline assembly: the compiler would wait for the returned value on
        // the spot (it broadcasts it inside the wavefront), which stalls the first stages of the tile behind
        // the round trip.  Like the DMA loads, this one is waited for by the loop's own vmcnt waits; the
        // value is first read behind the vmcnt(0) of the tile's last stage.  The register is tied in and out
        // ("+v"), so the value the asm statement defines is the one the later store reads: no copy of it can
        // be made before the wait.
        int ahead = 0;
        if (dyn && threadIdx.x == 0) {
            const uint32_t one = 1u;
            asm volatile("global_atomic_add %0, %1, %2, off sc0" : "+v"(ahead) : "v"(queue_counter()), "v"(one) : "memory");
        }
        if constexpr (!RAGK) {
            if (t.half) run_tile(IntTag<2>{}, total, ahead);
            else run_tile(IntTag<4>{}, total, ahead);
        } else {
            run_tile(IntTag<4>{}, total, ahead);
        }
        // Nothing is outstanding here (the loop ended with vmcnt(0)); said with the builtin so that the
        // compiler's own bookkeeping agrees and no load counts as pending in the next tile's loop.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        // ---- next tile: its first stage is requested before this tile's epilogue ----
        // (every DMA load of this tile has landed and every wavefront is past the last barrier, after
        // which nobody reads LDS any more: both buffers are free)
        auto next_tile = [&](bool first) -> int {
            if (!dyn) return static_tile();
            if (first) {  // the draw made ahead; from an empty queue it is void, like every later draw from it
                const int c = s_draw[1];
                const int L = tile_of_draw(c);
                if (c >= 0 && L >= 0 && L < total_tiles) return L;
                ++qx;
                return draw_now(true);
            }
            return draw_now(false);
        };
        TileDesc nt = decode(next_tile(true));
        while (nt.valid && nt.nk == 0) {
            if constexpr (RAGK) epilogue_zero(nt);
            nt = decode(next_tile(false));
        }
        int ntot = 0;
        if (nt.valid) {
            di = nt;
            setup_issue();
            ntot = nt.nk * g.nseg;
            issue(0, 0);
            if (ntot >= 2) {
                issue_part(1, 1, 0, kEarly);
                if (wave_u != kWaves - 1) issue_part(1, 1, kEarly, 2 * CPW);
            }
        }
        epilogue(t, smem + kStagingOff);
        if (!nt.valid) break;
        if (ntot >= 2 && wave_u == kWaves - 1) issue_part(1, 1, kEarly, 2 * CPW);
        t = nt;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Experts sorted by row count, heaviest first (one workgroup; E <= 256): the wgrad tiles of a
// heavy expert take longest, so they are started first.  Also clears the row of zeros and the tile queues.
__global__ __launch_bounds__(256) void expert_order_kernel(const int32_t* __restrict__ offsets, int E,
                                                           int32_t* __restrict__ order, uint32_t* __restrict__ zero_row,
                                                           uint32_t* __restrict__ sched, int sched_words) {
    const int e = threadIdx.x;
    if (e < 128) zero_row[e] = 0u;  // the 512-byte row of zeros the wgrad loads read past an expert's last row
    for (int i = e; i < sched_words; i += 256) sched[i] = 0u;  // the tile queues of the GEMMs that follow
    if (e >= E) return;
    const int mine = offsets[e + 1] - offsets[e];
    int rank = 0;
    for (int j = 0; j < E; ++j) {
        const int c = offsets[j + 1] - offsets[j];
        rank += (c > mine) || (c == mine && j < e);
    }
    order[rank] = e;
}

}  // namespace moe
