// Expert computation: moe_grouped_ffn_fwd and moe_grouped_ffn_bwd.
//
// Every expert is a SwiGLU MLP (paper section 3.1) applied to the rows the gate
// sent to it; the rows of one expert are contiguous after moe_permute and their
// number is whatever the (skewed) routing produced.  All six products are
// "grouped GEMMs": one GEMM per expert whose ragged dimension is the expert's
// row count, either as M (forward, dgrad) or as the contraction length K
// (wgrad).  One kernel template covers them:
//
//   C[m,n] = sum_k A(m,k) * B(k,n)          per expert, fp32 accumulate
//
//   forward 1   [A|B] = Xp_e * [W1_e|W3_e]         -> H = silu(A) (.) B
//   forward 2   Yp_e  = H_e * W2_e
//   dgrad 1     dH    = dYp_e * W2_e^T              -> dA, dB (and H again)
//   dgrad 2     dXp_e = dA_e * W1_e^T + dB_e * W3_e^T      (two K segments)
//   wgrad       dW2_e = H_e^T * dYp_e,  [dW1_e|dW3_e] = Xp_e^T * [dA_e|dB_e]
//
// bf16 path: the persistent 256x256x64 kernel of grouped_gemm_bf16.h (8 wavefronts,
// MFMA 32x32x16 bf16 with fp32 accumulators, operands brought into LDS by DMA in
// memory order, transposing LDS reads where the contraction index is not the
// contiguous one).  Shapes it does not take (leading dimensions that are not a
// multiple of 8, K not a multiple of 64) run on the plain 128x128x64 kernel below.
// fp32 path (parity mode): plain FMA tiles, same tile walk and epilogues.
#include "moe_internal.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum { EPI_STORE = 0, EPI_STORE2 = 1, EPI_SWIGLU = 2, EPI_DH = 3, EPI_STORE_F32 = 4, EPI_ADD = 5, EPI_DHP = 6 };

struct Seg {
    const void* A;
    const void* B;
    const void* B2;
};

struct GArgs {
    const int32_t* offsets;  // [E+1] rows of each expert
    int E;
    int M, N, K;           // fixed extents (M unused when M is ragged, K unused when K is ragged)
    int nseg;              // K segments accumulated into one tile
    Seg seg[2];
    int64_t lda, ldb;      // leading dimensions in elements
    int64_t strideB;       // per-expert stride of B (ragged M);
    int64_t strideC;       // per-expert stride of C (ragged K)
    void* C0;
    void* C1;
    void* C2;
    const void* S0;        // saved A (EPI_DH: read; EPI_SWIGLU: written if non-null)
    const void* S1;        // saved B
    int products;          // the saved pair is P = B*silu'(A), Q = silu(A) instead of A, B (EPI_SWIGLU writes it, EPI_DHP reads it)
    int64_t ldc;
    const int32_t* order;  // ragged K: experts by row count, heaviest first (may be null)
    const void* zero_row;  // ragged K: 512 bytes of zeros in device memory
    const int32_t* expert_of_group;  // ragged M: weights of group e are those of expert expert_of_group[e] (null: e itself)
    int n_weights;                   // experts in the weight arrays (the table's entries are clamped to it)
    uint32_t* sched;                 // tile queues of the persistent kernel (kSchedWords words, zero at launch); null: static tile order
};

// index of the weight matrices of group e
__device__ __forceinline__ int weight_index(const GArgs& g, int e) {
    if (!g.expert_of_group) return e;
    const int w = g.expert_of_group[e];
    return w < 0 ? 0 : (w >= g.n_weights ? g.n_weights - 1 : w);
}

template <class T, int EPI>
__device__ __forceinline__ void epilogue_elem(const GArgs& g, int64_t idx, float a, float b) {
    if constexpr (EPI == EPI_STORE_F32) {
        static_cast<float*>(g.C0)[idx] = a;
    } else if constexpr (EPI == EPI_STORE) {
        Elem<T>::store(static_cast<T*>(g.C0) + idx, a);
    } else if constexpr (EPI == EPI_STORE2) {
        Elem<T>::store(static_cast<T*>(g.C0) + idx, a);
        Elem<T>::store(static_cast<T*>(g.C1) + idx, b);
    } else if constexpr (EPI == EPI_SWIGLU) {
        Elem<T>::store(static_cast<T*>(g.C0) + idx, silu_f(a) * b);
        if (g.S0) {
            Elem<T>::store(const_cast<T*>(static_cast<const T*>(g.S0)) + idx, g.products ? b * silu_grad_f(a) : a);
            Elem<T>::store(const_cast<T*>(static_cast<const T*>(g.S1)) + idx, g.products ? silu_f(a) : b);
        }
    } else if constexpr (EPI == EPI_DHP) {  // a = dH; saved P, Q
        const float P = Elem<T>::load(static_cast<const T*>(g.S0) + idx);
        const float Q = Elem<T>::load(static_cast<const T*>(g.S1) + idx);
        Elem<T>::store(static_cast<T*>(g.C1) + idx, a * P);
        Elem<T>::store(static_cast<T*>(g.C2) + idx, a * Q);
    } else {  // EPI_DH: a = dH
        const float A = Elem<T>::load(static_cast<const T*>(g.S0) + idx);
        const float B = Elem<T>::load(static_cast<const T*>(g.S1) + idx);
        const float sA = silu_f(A);
        Elem<T>::store(static_cast<T*>(g.C0) + idx, sA * B);
        Elem<T>::store(static_cast<T*>(g.C1) + idx, a * B * silu_grad_f(A));
        Elem<T>::store(static_cast<T*>(g.C2) + idx, a * sA);
    }
}

// Which expert and which row block does m-tile `mt` (counted over all experts) belong to?
// Returns false if mt is past the last tile.  Uniform across the workgroup.
template <int BM>
__device__ __forceinline__ bool find_m_tile(const int32_t* __restrict__ offsets, int E, int mt, int& e_out,
                                            int& row0, int& row_end) {
    int acc = 0;
    for (int e = 0; e < E; ++e) {
        const int b = offsets[e], en = offsets[e + 1];
        const int nt = (en - b + BM - 1) / BM;
        if (mt < acc + nt) {
            e_out = e;
            row0 = b + (mt - acc) * BM;
            row_end = en;
            return true;
        }
        acc += nt;
    }
    return false;
}

// =============================== bf16 MFMA path ===============================
constexpr int BM = 128, BN = 128, BK = 64, BKP = BK + 8;

// contraction-contiguous source: tile rows [row0, row0+128) x k [k0, k0+64)
__device__ __forceinline__ void ld_kcontig(u32x4 (&r)[4], const bf16_t* __restrict__ base, int64_t ld, int row0,
                                           int row_lim, int k0, int k_lim) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = threadIdx.x + i * 256;
        const int row = row0 + (v >> 3), kk = k0 + (v & 7) * 8;
        if (row < row_lim && kk < k_lim)
            r[i] = *reinterpret_cast<const u32x4*>(base + (int64_t)row * ld + kk);
        else
            r[i] = (u32x4){0, 0, 0, 0};
    }
}
__device__ __forceinline__ void st_kcontig(bf16_t (*dst)[BKP], const u32x4 (&r)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = threadIdx.x + i * 256;
        *reinterpret_cast<u32x4*>(&dst[v >> 3][(v & 7) * 8]) = r[i];
    }
}
// other-index-contiguous source: k rows [k0, k0+64) x cols [col0, col0+128)
__device__ __forceinline__ void ld_strided(u32x4 (&r)[4], const bf16_t* __restrict__ base, int64_t ld, int k0,
                                           int k_lim, int col0, int col_lim) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = threadIdx.x + i * 256;
        const int kk = k0 + (v >> 4), col = col0 + (v & 15) * 8;
        if (kk < k_lim && col < col_lim)
            r[i] = *reinterpret_cast<const u32x4*>(base + (int64_t)kk * ld + col);
        else
            r[i] = (u32x4){0, 0, 0, 0};
    }
}
__device__ __forceinline__ void st_strided(bf16_t (*dst)[BKP], const u32x4 (&r)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = threadIdx.x + i * 256;
        const int kk = v >> 4, c = (v & 15) * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = r[i][j];
            dst[c + 2 * j][kk] = (bf16_t)(w & 0xFFFFu);
            dst[c + 2 * j + 1][kk] = (bf16_t)(w >> 16);
        }
    }
}

// AT: 0 = A stored [M][K] (K contiguous), 1 = A stored [K][M]
// BT: 0 = B stored [K][N] (N contiguous), 1 = B stored [N][K]
template <int AT, int BT, bool DUAL, int EPI, bool RAGK>
__global__ __launch_bounds__(256) void gg_bf16_kernel(const GArgs g) {
    __shared__ __attribute__((aligned(16))) bf16_t As[BM][BKP];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN][BKP];
    __shared__ __attribute__((aligned(16))) bf16_t Bs2[DUAL ? BN : 1][BKP];

    int e, m0, m_lim, kbeg, kend;
    const int n0 = blockIdx.x * BN;
    if constexpr (RAGK) {
        e = blockIdx.z;
        m0 = blockIdx.y * BM;
        m_lim = g.M;
        kbeg = g.offsets[e];
        kend = g.offsets[e + 1];
    } else {
        if (!find_m_tile<BM>(g.offsets, g.E, blockIdx.y, e, m0, m_lim)) return;
        kbeg = 0;
        kend = g.K;
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

    f32x16 acc[2][2], acc2[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[i][j][r] = 0.f;
                acc2[i][j][r] = 0.f;
            }

    const int nk = (kend - kbeg + BK - 1) / BK;
    const int total = nk * g.nseg;
    u32x4 ra[4], rb[4], rb2[4];

    auto gload = [&](int it) {
        const int sg = it / nk, k0 = kbeg + (it - sg * nk) * BK;
        const bf16_t* A = static_cast<const bf16_t*>(g.seg[sg].A);
        const bf16_t* B = static_cast<const bf16_t*>(g.seg[sg].B) + (RAGK ? 0 : (int64_t)weight_index(g, e) * g.strideB);
        if constexpr (AT == 0) ld_kcontig(ra, A, g.lda, m0, m_lim, k0, kend);
        else ld_strided(ra, A, g.lda, k0, kend, m0, m_lim);
        if constexpr (BT == 1) ld_kcontig(rb, B, g.ldb, n0, g.N, k0, kend);
        else ld_strided(rb, B, g.ldb, k0, kend, n0, g.N);
        if constexpr (DUAL) {
            const bf16_t* B2 = static_cast<const bf16_t*>(g.seg[sg].B2) + (RAGK ? 0 : (int64_t)weight_index(g, e) * g.strideB);
            if constexpr (BT == 1) ld_kcontig(rb2, B2, g.ldb, n0, g.N, k0, kend);
            else ld_strided(rb2, B2, g.ldb, k0, kend, n0, g.N);
        }
    };

    if (total > 0) gload(0);
    for (int it = 0; it < total; ++it) {
        __syncthreads();  // previous tile fully consumed
        if constexpr (AT == 0) st_kcontig(As, ra); else st_strided(As, ra);
        if constexpr (BT == 1) st_kcontig(Bs, rb); else st_strided(Bs, rb);
        if constexpr (DUAL) { if constexpr (BT == 1) st_kcontig(Bs2, rb2); else st_strided(Bs2, rb2); }
        __syncthreads();
        if (it + 1 < total) gload(it + 1);  // next tile's HBM reads overlap the MFMAs below
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 a[2], b[2], b2[2];
            const int ko = kk + (lane >> 5) * 8;
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&As[wm + i * 32 + (lane & 31)][ko]);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                b[j] = *reinterpret_cast<const bf16x8*>(&Bs[wn + j * 32 + (lane & 31)][ko]);
                if constexpr (DUAL) b2[j] = *reinterpret_cast<const bf16x8*>(&Bs2[wn + j * 32 + (lane & 31)][ko]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
                    if constexpr (DUAL)
                        acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b2[j], acc2[i][j], 0, 0, 0);
                }
        }
    }

    // epilogue: 32x32 accumulator layout: col = lane%32, row = 8*(r/4) + 4*(lane/32) + r%4
    const int64_t cbase = RAGK ? (int64_t)e * g.strideC : 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (row < m_lim && col < g.N)
                    epilogue_elem<bf16_t, EPI>(g, cbase + (int64_t)row * g.ldc + col, acc[i][j][r],
                                               DUAL ? acc2[i][j][r] : 0.f);
            }
        }
}

}  // namespace moe
#include "grouped_gemm_bf16.h"
namespace moe {

// =============================== fp32 FMA path ================================
// 64x64 tiles, 16x16 threads with 4x4 outputs each, BK = 16; operands addressed
// with explicit strides so every layout uses the same loader.
struct F32Strides {
    int64_t sam, sak, sbk, sbn;
};

template <bool DUAL, int EPI, bool RAGK>
__global__ __launch_bounds__(256) void gg_f32_kernel(const GArgs g, const F32Strides st) {
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float As[TK][TM + 1];
    __shared__ float Bs[TK][TN + 1];
    __shared__ float Bs2[DUAL ? TK : 1][TN + 1];

    int e, m0, m_lim, kbeg, kend;
    const int n0 = blockIdx.x * TN;
    if constexpr (RAGK) {
        e = blockIdx.z;
        m0 = blockIdx.y * TM;
        m_lim = g.M;
        kbeg = g.offsets[e];
        kend = g.offsets[e + 1];
    } else {
        if (!find_m_tile<TM>(g.offsets, g.E, blockIdx.y, e, m0, m_lim)) return;
        kbeg = 0;
        kend = g.K;
    }
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4], acc2[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = acc2[i][j] = 0.f;

    for (int sg = 0; sg < g.nseg; ++sg) {
        const float* A = static_cast<const float*>(g.seg[sg].A);
        const float* B = static_cast<const float*>(g.seg[sg].B) + (RAGK ? 0 : (int64_t)weight_index(g, e) * g.strideB);
        const float* B2 = DUAL ? static_cast<const float*>(g.seg[sg].B2) + (RAGK ? 0 : (int64_t)weight_index(g, e) * g.strideB) : nullptr;
        for (int k0 = kbeg; k0 < kend; k0 += TK) {
            __syncthreads();
            for (int idx = threadIdx.x; idx < TK * TM; idx += 256) {
                // pick the thread->element map that walks the contiguous index fastest
                int kk, mm;
                if (st.sak == 1) { kk = idx % TK; mm = idx / TK; } else { mm = idx % TM; kk = idx / TM; }
                const int m = m0 + mm, k = k0 + kk;
                As[kk][mm] = (m < m_lim && k < kend) ? A[(int64_t)m * st.sam + (int64_t)k * st.sak] : 0.f;
            }
            for (int idx = threadIdx.x; idx < TK * TN; idx += 256) {
                int kk, nn;
                if (st.sbk == 1) { kk = idx % TK; nn = idx / TK; } else { nn = idx % TN; kk = idx / TN; }
                const int n = n0 + nn, k = k0 + kk;
                const bool ok = n < g.N && k < kend;
                Bs[kk][nn] = ok ? B[(int64_t)k * st.sbk + (int64_t)n * st.sbn] : 0.f;
                if constexpr (DUAL) Bs2[kk][nn] = ok ? B2[(int64_t)k * st.sbk + (int64_t)n * st.sbn] : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < TK; ++kk) {
                float a[4], b[4], b2[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    b[j] = Bs[kk][tx * 4 + j];
                    if constexpr (DUAL) b2[j] = Bs2[kk][tx * 4 + j];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                        if constexpr (DUAL) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
                    }
            }
        }
    }
    const int64_t cbase = RAGK ? (int64_t)e * g.strideC : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
            if (row < m_lim && col < g.N)
                epilogue_elem<float, EPI>(g, cbase + (int64_t)row * g.ldc + col, acc[i][j], DUAL ? acc2[i][j] : 0.f);
        }
}

// =============================== host dispatch ================================
// A(m,k) layout AT, B(k,n) layout BT as in the bf16 kernel.
template <int AT, int BT, bool DUAL, int EPI, bool RAGK>
static void launch_gg(const moe_shape* s, const GArgs& g, int64_t R, hipStream_t st) {
    if (s->dtype == MOE_BF16) {
        constexpr bool fast_form = RAGK ? (AT == 1 && BT == 0) : (AT == 0);
        if constexpr (fast_form) {
            // (the kernel keeps per-lane offsets in 32 bits; inside a tile they stay below 2^31 bytes)
            const bool ok = g.lda % 8 == 0 && g.ldb % 8 == 0 && g.N >= 8 && g.lda < (1 << 21) && g.ldb < (1 << 21) && g.ldc < (1 << 22) &&
                            (uint64_t)R * (uint64_t)g.lda < (1ull << 32) && (uint64_t)g.N * (uint64_t)g.ldb < (1ull << 32) &&
                            (RAGK ? (g.M >= 8) : (g.K % TK == 0));
            if (ok) {
                auto kern = gg256_kernel<AT, BT, DUAL, EPI, RAGK>;
                ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kGemmLds);
                (void)R;
                kern<<<dim3(256), kThreads, kGemmLds, st>>>(g);  // persistent: one workgroup per CU
                return;
            }
        }
        dim3 grid;
        if (RAGK) grid = dim3((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, g.E);
        else grid = dim3((g.N + BN - 1) / BN, (unsigned)((R + BM - 1) / BM + g.E), 1);
        gg_bf16_kernel<AT, BT, DUAL, EPI, RAGK><<<grid, 256, 0, st>>>(g);
    } else {
        F32Strides fs;
        fs.sam = AT == 0 ? g.lda : 1;
        fs.sak = AT == 0 ? 1 : g.lda;
        fs.sbk = BT == 0 ? g.ldb : 1;
        fs.sbn = BT == 0 ? 1 : g.ldb;
        dim3 grid;
        if (RAGK) grid = dim3((g.N + 63) / 64, (g.M + 63) / 64, g.E);
        else grid = dim3((g.N + 63) / 64, (unsigned)((R + 63) / 64 + g.E), 1);
        gg_f32_kernel<DUAL, EPI, RAGK><<<grid, 256, 0, st>>>(g, fs);
    }
}

void launch_gate_dwg_gemm(const void* x, const void* dl_hi, const void* dl_lo, const int32_t* chunk_offsets,
                          int nchunks, int d, int n_pad, float* partial, const void* zero_row, hipStream_t st) {
    GArgs g{};
    g.zero_row = zero_row;
    g.offsets = chunk_offsets; g.E = nchunks; g.M = d; g.N = n_pad; g.nseg = 2;
    g.seg[0] = {x, dl_hi, nullptr};
    g.seg[1] = {x, dl_lo, nullptr};
    g.lda = d; g.ldb = n_pad; g.strideC = (int64_t)d * n_pad;
    g.C0 = partial; g.ldc = n_pad;
    auto kern = gg256_kernel<1, 0, false, EPI_STORE_F32, true>;
    ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kGemmLds);
    kern<<<dim3(256), kThreads, kGemmLds, st>>>(g);
}

void launch_gate_dx_gemm(const void* dl_hi, const void* dl_lo, const void* wg_pad, const int32_t* whole, int d, int n_pad,
                         void* dx, hipStream_t st) {
    GArgs g{};
    g.offsets = whole; g.E = 1; g.N = d; g.K = n_pad; g.nseg = 2;
    g.seg[0] = {dl_hi, wg_pad, nullptr};
    g.seg[1] = {dl_lo, wg_pad, nullptr};
    g.lda = n_pad; g.ldb = n_pad; g.strideB = 0;
    g.C0 = dx; g.ldc = d;
    auto kern = gg256_kernel<0, 1, false, EPI_ADD, false>;
    ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kGemmLds);
    kern<<<dim3(256), kThreads, kGemmLds, st>>>(g);
}

// Tile queues: the two wgrad launches draw their tiles (a tile costs as much as its expert has rows, so a
// fixed deal leaves workgroups idle at the end: 2-4 % of the backward pass on the skewed workloads); the
// kernels with ragged M keep the fixed order, where drawing measured no gain.
constexpr size_t kSchedBytes = kSchedWords * sizeof(uint32_t);  // tile queues of one GEMM launch
constexpr int kBwdLaunches = 2;

size_t ffn_fwd_workspace_bytes(const moe_shape* s) {
    return align_up((size_t)s->T * s->k * s->f * el_size(s), 256);  // H
}
size_t ffn_bwd_workspace_bytes(const moe_shape* s) {
    // H, dA, dB, (A, B when recomputing), expert order, a row of zeros, tile queues
    return 5 * align_up((size_t)s->T * s->k * s->f * el_size(s), 256) + 2048 + kBwdLaunches * kSchedBytes;
}


}  // namespace moe

using namespace moe;

// groups: number of row groups described by offsets (the experts themselves, or replica groups whose weights
// are those of expert expert_of_group[g])
static void run_fwd1(const moe_shape* s, const void* x_perm, const int32_t* offsets, const void* w1, const void* w3,
                     void* H, void* a_save, void* b_save, hipStream_t st, int groups = 0,
                     const int32_t* expert_of_group = nullptr, bool products = false) {
    GArgs g{};
    g.offsets = offsets; g.E = groups ? groups : s->E; g.N = s->f; g.K = s->d; g.nseg = 1;
    g.expert_of_group = expert_of_group; g.n_weights = s->E;
    g.seg[0] = {x_perm, w1, w3};
    g.lda = s->d; g.ldb = s->f; g.strideB = (int64_t)s->d * s->f;
    g.C0 = H; g.S0 = a_save; g.S1 = b_save; g.ldc = s->f; g.products = products ? 1 : 0;
    launch_gg<0, 0, true, EPI_SWIGLU, false>(s, g, (int64_t)s->T * s->k, st);
}

static moe_status ffn_fwd_impl(const char* who, const moe_shape* s, int groups, const int32_t* expert_of_group,
                               const void* x_perm, const int32_t* offsets, const void* w1, const void* w3,
                               const void* w2, void* y_perm, void* a_save, void* b_save, void* ws, size_t ws_bytes,
                               void* stream, void* h_save = nullptr) {
    // h_save: the products form (H is kept, the saved pair is P = B*silu'(A), Q = silu(A)); no workspace then
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(x_perm, "x_perm", who));
    MOE_RETURN_IF(check_ptr(offsets, "offsets", who));
    MOE_RETURN_IF(check_ptr(w1, "w1", who));
    MOE_RETURN_IF(check_ptr(w3, "w3", who));
    MOE_RETURN_IF(check_ptr(w2, "w2", who));
    MOE_RETURN_IF(check_ptr(y_perm, "y_perm", who));
    MOE_RETURN_IF(check_ptr(a_save, "a_save", who, true));
    MOE_RETURN_IF(check_ptr(b_save, "b_save", who, true));
    if (!h_save) MOE_RETURN_IF(check_ptr(ws, "ws", who));
    if ((a_save == nullptr) != (b_save == nullptr)) {
        set_error("%s: a_save and b_save must both be given or both be NULL", who);
        return MOE_ERR_INVALID_ARG;
    }
    MOE_RETURN_IF(check_device(who));
    if (!h_save && ws_bytes < ffn_fwd_workspace_bytes(s)) {
        set_error("%s: workspace %zu < %zu bytes", who, ws_bytes, ffn_fwd_workspace_bytes(s));
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t R = (int64_t)s->T * s->k;
    void* H = h_save ? h_save : ws;
    run_fwd1(s, x_perm, offsets, w1, w3, H, a_save, b_save, st, groups, expert_of_group, h_save != nullptr);
    GArgs g{};
    g.offsets = offsets; g.E = groups; g.N = s->d; g.K = s->f; g.nseg = 1;
    g.expert_of_group = expert_of_group; g.n_weights = s->E;
    g.seg[0] = {H, w2, nullptr};
    g.lda = s->f; g.ldb = s->d; g.strideB = (int64_t)s->f * s->d;
    g.C0 = y_perm; g.ldc = s->d;
    launch_gg<0, 0, false, EPI_STORE, false>(s, g, R, st);
    return launch_status(who);
}

extern "C" moe_status moe_grouped_ffn_fwd(const moe_shape* s, const void* x_perm, const int32_t* offsets,
                                          const void* w1, const void* w3, const void* w2, void* y_perm, void* a_save,
                                          void* b_save, void* ws, size_t ws_bytes, void* stream) {
    return ffn_fwd_impl("moe_grouped_ffn_fwd", s, s ? s->E : 0, nullptr, x_perm, offsets, w1, w3, w2, y_perm, a_save,
                        b_save, ws, ws_bytes, stream);
}

extern "C" moe_status moe_grouped_ffn_fwd_groups(const moe_shape* s, int32_t G, const int32_t* expert_of_group,
                                                 const void* x_perm, const int32_t* group_offsets, const void* w1,
                                                 const void* w3, const void* w2, void* y_perm, void* a_save,
                                                 void* b_save, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "moe_grouped_ffn_fwd_groups";
    if (G < 1 || G > MOE_MAX_EXPERTS) {
        set_error("%s: G=%d must be in [1, %d]", who, G, MOE_MAX_EXPERTS);
        return MOE_ERR_INVALID_ARG;
    }
    MOE_RETURN_IF(check_ptr(expert_of_group, "expert_of_group", who));
    return ffn_fwd_impl(who, s, G, expert_of_group, x_perm, group_offsets, w1, w3, w2, y_perm, a_save, b_save, ws,
                        ws_bytes, stream);
}

// groups / expert_of_group as in ffn_fwd_impl; the weight gradients are written per group
static moe_status ffn_bwd_impl(const char* who, const moe_shape* s, int groups, const int32_t* expert_of_group,
                               const void* x_perm, const int32_t* offsets, const void* w1, const void* w3,
                               const void* w2, const void* a_save, const void* b_save, const void* dy_perm,
                               void* dx_perm, void* dw1, void* dw3, void* dw2, void* ws, size_t ws_bytes,
                               void* stream, const void* h_save = nullptr) {
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(x_perm, "x_perm", who));
    MOE_RETURN_IF(check_ptr(offsets, "offsets", who));
    MOE_RETURN_IF(check_ptr(w1, "w1", who));
    MOE_RETURN_IF(check_ptr(w3, "w3", who));
    MOE_RETURN_IF(check_ptr(w2, "w2", who));
    MOE_RETURN_IF(check_ptr(a_save, "a_save", who, true));
    MOE_RETURN_IF(check_ptr(b_save, "b_save", who, true));
    MOE_RETURN_IF(check_ptr(dy_perm, "dy_perm", who));
    MOE_RETURN_IF(check_ptr(dx_perm, "dx_perm", who));
    MOE_RETURN_IF(check_ptr(dw1, "dw1", who));
    MOE_RETURN_IF(check_ptr(dw3, "dw3", who));
    MOE_RETURN_IF(check_ptr(dw2, "dw2", who));
    MOE_RETURN_IF(check_ptr(ws, "ws", who));
    if (h_save && (!a_save || !b_save)) {
        set_error("%s: the products form needs h_save, p_save and q_save", who);
        return MOE_ERR_INVALID_ARG;
    }
    MOE_RETURN_IF(check_device(who));
    if (ws_bytes < ffn_bwd_workspace_bytes(s)) {
        set_error("%s: workspace %zu < %zu bytes", who, ws_bytes, ffn_bwd_workspace_bytes(s));
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t R = (int64_t)s->T * s->k;
    const size_t rf = (size_t)R * s->f * el_size(s);
    Carver cv(ws);
    void* H = cv.take(rf);  // (not used in the products form, which reads h_save)
    void* dA = cv.take(rf);
    void* dB = cv.take(rf);
    int32_t* order = static_cast<int32_t*>(cv.take(1024));
    void* zero_row = cv.take(512);
    uint32_t* sched = static_cast<uint32_t*>(cv.take(kBwdLaunches * kSchedBytes));
    expert_order_kernel<<<1, 256, 0, st>>>(offsets, groups, order, static_cast<uint32_t*>(zero_row), sched,
                                           kBwdLaunches * kSchedWords);
    if (!a_save || !b_save) {  // expert-only recomputation: rebuild A and B (H is rewritten below anyway)
        void* A = cv.take(rf);
        void* B = cv.take(rf);
        run_fwd1(s, x_perm, offsets, w1, w3, H, A, B, st, groups, expert_of_group);
        a_save = A;
        b_save = B;
    }
    {  // dH = dYp * W2^T, then the SwiGLU derivative in the epilogue
        GArgs g{};
        g.offsets = offsets; g.E = groups; g.N = s->f; g.K = s->d; g.nseg = 1;
        g.expert_of_group = expert_of_group; g.n_weights = s->E;
        g.seg[0] = {dy_perm, w2, nullptr};
        g.lda = s->d; g.ldb = s->d; g.strideB = (int64_t)s->f * s->d;
        g.C0 = H; g.C1 = dA; g.C2 = dB; g.S0 = a_save; g.S1 = b_save; g.ldc = s->f;
        if (h_save) launch_gg<0, 1, false, EPI_DHP, false>(s, g, R, st);  // dA = dH*P, dB = dH*Q
        else launch_gg<0, 1, false, EPI_DH, false>(s, g, R, st);
    }
    {  // dXp = dA * W1^T + dB * W3^T
        GArgs g{};
        g.offsets = offsets; g.E = groups; g.N = s->d; g.K = s->f; g.nseg = 2;
        g.expert_of_group = expert_of_group; g.n_weights = s->E;
        g.seg[0] = {dA, w1, nullptr};
        g.seg[1] = {dB, w3, nullptr};
        g.lda = s->f; g.ldb = s->f; g.strideB = (int64_t)s->d * s->f;
        g.C0 = dx_perm; g.ldc = s->d;
        launch_gg<0, 1, false, EPI_STORE, false>(s, g, R, st);
    }
    {  // dW2[e] = H_e^T * dYp_e
        GArgs g{};
        g.offsets = offsets; g.E = groups; g.M = s->f; g.N = s->d; g.nseg = 1;
        g.seg[0] = {h_save ? h_save : H, dy_perm, nullptr};
        g.lda = s->f; g.ldb = s->d; g.strideC = (int64_t)s->f * s->d;
        g.C0 = dw2; g.ldc = s->d; g.order = order; g.zero_row = zero_row;
        g.sched = sched;
        launch_gg<1, 0, false, EPI_STORE, true>(s, g, R, st);
    }
    {  // [dW1|dW3][e] = Xp_e^T * [dA_e|dB_e]
        GArgs g{};
        g.offsets = offsets; g.E = groups; g.M = s->d; g.N = s->f; g.nseg = 1;
        g.seg[0] = {x_perm, dA, dB};
        g.lda = s->d; g.ldb = s->f; g.strideC = (int64_t)s->d * s->f;
        g.C0 = dw1; g.C1 = dw3; g.ldc = s->f; g.order = order; g.zero_row = zero_row;
        g.sched = sched + kSchedWords;
        launch_gg<1, 0, true, EPI_STORE2, true>(s, g, R, st);
    }
    return launch_status(who);
}


extern "C" moe_status moe_grouped_ffn_bwd(const moe_shape* s, const void* x_perm, const int32_t* offsets,
                                          const void* w1, const void* w3, const void* w2, const void* a_save,
                                          const void* b_save, const void* dy_perm, void* dx_perm, void* dw1, void* dw3,
                                          void* dw2, void* ws, size_t ws_bytes, void* stream) {
    return ffn_bwd_impl("moe_grouped_ffn_bwd", s, s ? s->E : 0, nullptr, x_perm, offsets, w1, w3, w2, a_save, b_save,
                        dy_perm, dx_perm, dw1, dw3, dw2, ws, ws_bytes, stream);
}

extern "C" moe_status moe_grouped_ffn_fwd_products(const moe_shape* s, const void* x_perm, const int32_t* offsets,
                                                   const void* w1, const void* w3, const void* w2, void* y_perm,
                                                   void* h_save, void* p_save, void* q_save, void* stream) {
    const char* who = "moe_grouped_ffn_fwd_products";
    MOE_RETURN_IF(check_ptr(h_save, "h_save", who));
    MOE_RETURN_IF(check_ptr(p_save, "p_save", who));
    MOE_RETURN_IF(check_ptr(q_save, "q_save", who));
    return ffn_fwd_impl(who, s, s ? s->E : 0, nullptr, x_perm, offsets, w1, w3, w2, y_perm, p_save, q_save, nullptr, 0,
                        stream, h_save);
}

extern "C" moe_status moe_grouped_ffn_bwd_products(const moe_shape* s, const void* x_perm, const int32_t* offsets,
                                                   const void* w1, const void* w3, const void* w2, const void* h_save,
                                                   const void* p_save, const void* q_save, const void* dy_perm,
                                                   void* dx_perm, void* dw1, void* dw3, void* dw2, void* ws,
                                                   size_t ws_bytes, void* stream) {
    const char* who = "moe_grouped_ffn_bwd_products";
    MOE_RETURN_IF(check_ptr(h_save, "h_save", who));
    MOE_RETURN_IF(check_ptr(p_save, "p_save", who));
    MOE_RETURN_IF(check_ptr(q_save, "q_save", who));
    return ffn_bwd_impl(who, s, s ? s->E : 0, nullptr, x_perm, offsets, w1, w3, w2, p_save, q_save, dy_perm, dx_perm,
                        dw1, dw3, dw2, ws, ws_bytes, stream, h_save);
}

extern "C" moe_status moe_grouped_ffn_bwd_groups(const moe_shape* s, int32_t G, const int32_t* expert_of_group,
                                                 const void* x_perm, const int32_t* group_offsets, const void* w1,
                                                 const void* w3, const void* w2, const void* a_save,
                                                 const void* b_save, const void* dy_perm, void* dx_perm,
                                                 void* dw1_groups, void* dw3_groups, void* dw2_groups, void* ws,
                                                 size_t ws_bytes, void* stream) {
    const char* who = "moe_grouped_ffn_bwd_groups";
    if (G < 1 || G > MOE_MAX_EXPERTS) {
        set_error("%s: G=%d must be in [1, %d]", who, G, MOE_MAX_EXPERTS);
        return MOE_ERR_INVALID_ARG;
    }
    MOE_RETURN_IF(check_ptr(expert_of_group, "expert_of_group", who));
    return ffn_bwd_impl(who, s, G, expert_of_group, x_perm, group_offsets, w1, w3, w2, a_save, b_save, dy_perm, dx_perm,
                        dw1_groups, dw3_groups, dw2_groups, ws, ws_bytes, stream);
}
