// Gate of the MoE layer: moe_gate_topk and moe_gate_topk_bwd.
//
// g(x) = Softmax(TopK(x * W_g)) (paper, Preliminary section).  Logits are
// accumulated in fp32 from exact products of the stored values, a per-expert
// bias is added, and the k largest are picked by a wavefront: every lane holds
// the logits of the experts (lane, lane+64, ...), k rounds of a 64-lane
// arg-max (value descending, expert index ascending on ties) pick the slots in
// order, and the softmax runs over the k picked values only.
#include "moe_internal.h"

namespace moe {

constexpr int kGateTokens = 16;   // tokens per workgroup
constexpr int kGateKC = 256;      // hidden-dimension chunk staged in LDS
constexpr int kGateMaxNE = MOE_MAX_EXPERTS / 64;

size_t gate_workspace_bytes(const moe_shape* s) { return align_up((size_t)MOE_MAX_EXPERTS * s->d * 2, 256); }

// One workgroup = 4 wavefronts = 16 tokens; wave w owns tokens w, w+4, w+8, w+12
// of the block, lane l owns experts l, l+64, ...
template <class T>
__global__ __launch_bounds__(256) void gate_topk_kernel(const T* __restrict__ x, const T* __restrict__ wg,
                                                        const float* __restrict__ bias, int32_t* __restrict__ ids,
                                                        float* __restrict__ wout, float* __restrict__ logits_out,
                                                        int Tn, int d, int E, int k) {
    __shared__ float xs[kGateTokens][kGateKC];
    __shared__ float sel[4][MOE_MAX_EXPERTS];  // per wave: the picked logits of the token in flight
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t0 = blockIdx.x * kGateTokens;
    const int ne = (E + 63) >> 6;

    float acc[4][kGateMaxNE];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < kGateMaxNE; ++j) acc[i][j] = 0.f;

    for (int c0 = 0; c0 < d; c0 += kGateKC) {
        const int kc = min(kGateKC, d - c0);
        __syncthreads();
        for (int idx = threadIdx.x; idx < kGateTokens * kGateKC; idx += 256) {
            const int tt = idx / kGateKC, c = idx - tt * kGateKC;
            const int t = t0 + tt;
            xs[tt][c] = (t < Tn && c < kc) ? Elem<T>::load(x + (size_t)t * d + c0 + c) : 0.f;
        }
        __syncthreads();
        for (int c = 0; c < kc; ++c) {
            float wv[kGateMaxNE];
#pragma unroll
            for (int j = 0; j < kGateMaxNE; ++j) {
                const int e = lane + 64 * j;
                wv[j] = (j < ne && e < E) ? Elem<T>::load(wg + (size_t)(c0 + c) * E + e) : 0.f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float xv = xs[wave + 4 * i][c];
#pragma unroll
                for (int j = 0; j < kGateMaxNE; ++j) acc[i][j] = fmaf(xv, wv[j], acc[i][j]);
            }
        }
    }

    // top-k and softmax, one token at a time per wave
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + wave + 4 * i;
        if (t >= Tn) continue;  // uniform per wave
        float v[kGateMaxNE];
#pragma unroll
        for (int j = 0; j < kGateMaxNE; ++j) {
            const int e = lane + 64 * j;
            if (e < E) {
                v[j] = acc[i][j] + (bias ? bias[e] : 0.f);
                if (logits_out) logits_out[(size_t)t * E + e] = v[j];
            } else {
                v[j] = -INFINITY;
            }
        }
        for (int s = 0; s < k; ++s) {
            // lane-local best (lowest index first on ties: j ascending, strict >)
            float bv = v[0];
            int be = lane;
#pragma unroll
            for (int j = 1; j < kGateMaxNE; ++j)
                if (v[j] > bv) { bv = v[j]; be = lane + 64 * j; }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                const float ov = __shfl_xor(bv, m, 64);
                const int oe = __shfl_xor(be, m, 64);
                if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
            }
            // every lane now holds the same winner
            if ((be & 63) == lane) {
#pragma unroll
                for (int j = 0; j < kGateMaxNE; ++j)
                    if (be == lane + 64 * j) v[j] = -INFINITY;
            }
            if (lane == 0) {
                ids[(size_t)t * k + s] = be;
                sel[wave][s] = bv;
            }
        }
        __builtin_amdgcn_wave_barrier();
        const float m0 = sel[wave][0];
        float z = 0.f;
        for (int s = 0; s < k; ++s) z += __expf(sel[wave][s] - m0);
        for (int s = lane; s < k; s += 64) wout[(size_t)t * k + s] = __expf(sel[wave][s] - m0) / z;
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- bf16 forward on the matrix cores ------------------------------------------------------
// One workgroup = 32 tokens, 4 wavefronts; wavefront w contracts the quarter
// [w*d/4, (w+1)*d/4) of the hidden dimension for all 32 tokens and all experts with MFMA
// 32x32x16 (operands straight from global memory: a lane reads 64 contiguous bytes of its
// token row / of its expert's row of the transposed gate weight per 64-wide k chunk), the
// four partial sums meet in LDS and are added in a fixed order, then each wavefront runs
// the top-k of 8 tokens.
typedef __bf16 gbf16x8 __attribute__((ext_vector_type(8)));
typedef float gf32x16 __attribute__((ext_vector_type(16)));
constexpr int kGateMT = 32;

// The gate weight in the order the MFMA lanes of gate_topk_mfma_kernel consume it ("fragment-major"): the
// 64 lanes x 8 values of one B operand are 1 KB of consecutive memory, so that every operand load of a
// wavefront is one fully coalesced 1 KB read (a plain transposed copy makes each lane read 16 bytes of a
// different row: 32 cache lines per load instruction).  Block index: ((wavefront's K range, 64-wide chunk),
// expert tile j, k-step s4); inside a block lane (l32, kg) holds expert j*32 + l32,
// k = range*kq + chunk*64 + kg*32 + s4*8 + 0..7.  Experts past E are zero.
__global__ void gate_pack_wg_kernel(const bf16_t* __restrict__ wg, bf16_t* __restrict__ wfrag, int d, int E, int NT,
                                    int NW) {
    const int64_t n = (int64_t)d * NT * 32;
    const int kq = d / NW, nchunk = kq / 64;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int z = (int)(i & 7), lane = (int)((i >> 3) & 63), s4 = (int)((i >> 9) & 3);
        const int64_t blk = i >> 11;  // (range*nchunk + chunk)*NT + j
        const int j = (int)(blk % NT);
        const int64_t rc = blk / NT;
        const int ci = (int)(rc % nchunk), w = (int)(rc / nchunk);
        const int e = j * 32 + (lane & 31);
        const int k = w * kq + ci * 64 + (lane >> 5) * 32 + s4 * 8 + z;
        wfrag[i] = e < E ? wg[(size_t)k * E + e] : (bf16_t)0;
    }
}

__device__ __forceinline__ void topk_softmax_token(float (&v)[kGateMaxNE], int lane, int k, float* sel,
                                                   int32_t* ids_t, float* w_t) {
    for (int s = 0; s < k; ++s) {
        float bv = v[0];
        int be = lane;
#pragma unroll
        for (int j = 1; j < kGateMaxNE; ++j)
            if (v[j] > bv) { bv = v[j]; be = lane + 64 * j; }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            const float ov = __shfl_xor(bv, m, 64);
            const int oe = __shfl_xor(be, m, 64);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        }
        if ((be & 63) == lane) {
#pragma unroll
            for (int j = 0; j < kGateMaxNE; ++j)
                if (be == lane + 64 * j) v[j] = -INFINITY;
        }
        if (lane == 0) {
            ids_t[s] = be;
            sel[s] = bv;
        }
    }
    __builtin_amdgcn_wave_barrier();
    const float m0 = sel[0];
    float z = 0.f;
    for (int s = 0; s < k; ++s) z += __expf(sel[s] - m0);
    for (int s = lane; s < k; s += 64) w_t[s] = __expf(sel[s] - m0) / z;
    __builtin_amdgcn_wave_barrier();
}

// Maximum over the 64 lanes, returned wave-uniform: DPP row shifts build the maximum of each
// row of 16 in its last lane, two row broadcasts carry it to lane 63.
__device__ __forceinline__ float wave_max_f32(float v) {
#define MOE_DPP_MAX(ctrl, rmask)                                                                              \
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v),            \
                                                                       __builtin_bit_cast(int, v), ctrl, rmask, 0xf, false)))
    MOE_DPP_MAX(0x111, 0xf);  // row_shr:1
    MOE_DPP_MAX(0x112, 0xf);  // row_shr:2
    MOE_DPP_MAX(0x114, 0xf);  // row_shr:4
    MOE_DPP_MAX(0x118, 0xf);  // row_shr:8
    MOE_DPP_MAX(0x142, 0xa);  // row_bcast:15 into rows 1 and 3
    MOE_DPP_MAX(0x143, 0xc);  // row_bcast:31 into rows 2 and 3
#undef MOE_DPP_MAX
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

template <int NT, int NW>  // expert tiles of 32; wavefronts (the contraction is split NW ways)
__global__ __launch_bounds__(NW * 64) void gate_topk_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wgT,
                                                             const float* __restrict__ bias, int32_t* __restrict__ ids,
                                                             float* __restrict__ wout, float* __restrict__ logits_out,
                                                             int Tn, int d, int E, int k) {
    extern __shared__ float part[];  // [NW][32][NT*32] partial logits, then the picked logits [32][MOE_MAX_EXPERTS]
    constexpr int TPW = kGateMT / NW;  // tokens finished by each wavefront
    constexpr int NE = (NT * 32 + 63) / 64;  // experts per lane in the top-k phase
    constexpr int EP = NT * 32;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, kg = lane >> 5;
    const int t0 = blockIdx.x * kGateMT;
    int trow = t0 + l32;
    trow = trow < Tn ? trow : Tn - 1;
    const int kq = d / NW;
    const bf16_t* xa = x + (size_t)trow * d + wave * kq + kg * 32;
    const bf16_t* wb = wgT + ((size_t)wave * (kq / 64) * NT) * 2048 + lane * 8;  // fragment-major, see gate_pack_wg_kernel

    gf32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    // operands of chunk c+1 are requested before the MFMAs of chunk c (HBM latency, not
    // bandwidth, is what a 32-token tile has to hide)
    gbf16x8 a[2][4], b[2][NT][4];
    auto load_chunk = [&](int c, gbf16x8 (&aa)[4], gbf16x8 (&bb)[NT][4]) {
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) aa[s4] = *reinterpret_cast<const gbf16x8*>(xa + c + s4 * 8);
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
                bb[j][s4] = *reinterpret_cast<const gbf16x8*>(wb + (((size_t)(c >> 6) * NT + j) * 4 + s4) * 512);
    };
    auto mma_chunk = [&](const gbf16x8 (&aa)[4], const gbf16x8 (&bb)[NT][4]) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aa[s4], bb[j][s4], acc[j], 0, 0, 0);
    };
    load_chunk(0, a[0], b[0]);
    for (int c = 0; c < kq; c += 128) {   // kq is a multiple of 64
        const int c1 = c + 64 < kq ? c + 64 : c, c2 = c + 128 < kq ? c + 128 : c;
        load_chunk(c1, a[1], b[1]);
        mma_chunk(a[0], b[0]);
        load_chunk(c2, a[0], b[0]);
        if (c + 64 < kq) mma_chunk(a[1], b[1]);
    }
    // partial sums -> LDS (accumulator layout: col = lane%32, row = 8*(r/4) + 4*(lane/32) + r%4)
    float* mine = part + (size_t)wave * kGateMT * EP;
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = (r >> 2) * 8 + kg * 4 + (r & 3);
            mine[row * EP + j * 32 + l32] = acc[j][r];
        }
    __syncthreads();
    // wave w finishes tokens TPW*w .. TPW*w + TPW-1; lane owns experts lane, lane+64, ...
    float vals[TPW][NE];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int row = wave * TPW + i;
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            const int e = lane + 64 * j;
            float v = -INFINITY;
            if (e < E) {
                v = part[row * EP + e];
#pragma unroll
                for (int q = 1; q < NW; ++q) v += part[(q * kGateMT + row) * EP + e];  // fixed order
                v += bias ? bias[e] : 0.f;
            }
            vals[i][j] = v;
        }
    }
    __syncthreads();  // partial sums consumed; LDS is reused for the picked logits
    // top-k of the wave's 8 tokens, all 8 arg-max reductions of a round in flight together
    float* sel = part + wave * TPW * MOE_MAX_EXPERTS;  // [TPW][k]
    if (logits_out) {
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int t = t0 + wave * TPW + i;
#pragma unroll
            for (int j = 0; j < NE; ++j)
                if (t < Tn && lane + 64 * j < E) logits_out[(size_t)t * E + lane + 64 * j] = vals[i][j];
        }
    }
    for (int s = 0; s < k; ++s) {
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            float lv = vals[i][0];
#pragma unroll
            for (int j = 1; j < NE; ++j) lv = fmaxf(lv, vals[i][j]);
            const float m = wave_max_f32(lv);  // uniform
            // lowest expert index holding the maximum: experts are laid out e = lane + 64*j
            int be = -1;
#pragma unroll
            for (int j = NE - 1; j >= 0; --j) {
                const uint64_t bal = __ballot(vals[i][j] == m);
                if (bal) be = 64 * j + __builtin_ctzll(bal);
            }
            if ((be & 63) == lane) {
#pragma unroll
                for (int j = 0; j < NE; ++j)
                    if (be == lane + 64 * j) vals[i][j] = -INFINITY;
            }
            const int t = t0 + wave * TPW + i;
            if (lane == 0 && t < Tn) {
                ids[(size_t)t * k + s] = be;
                sel[i * MOE_MAX_EXPERTS + s] = m;
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int t = t0 + wave * TPW + i;
        if (t >= Tn) continue;
        const float* sl = sel + i * MOE_MAX_EXPERTS;
        const float m0 = sl[0];
        float z = 0.f;
        for (int s = 0; s < k; ++s) z += __expf(sl[s] - m0);
        for (int s = lane; s < k; s += 64) wout[(size_t)t * k + s] = __expf(sl[s] - m0) / z;
    }
}

// ---- backward -----------------------------------------------------------------------

// wgT[e][c] = w_gate[c][e] as fp32 (makes the dx update a contiguous read)
template <class T>
__global__ void gate_transpose_kernel(const T* __restrict__ wg, float* __restrict__ wgT, int d, int E) {
    const int64_t n = (int64_t)d * E;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int e = (int)(i / d), c = (int)(i - (int64_t)e * d);
        wgT[i] = Elem<T>::load(wg + (size_t)c * E + e);
    }
}

// dl[t,s] = w_s (dw_s - sum_j w_j dw_j)
__global__ void gate_dl_kernel(const float* __restrict__ w, const float* __restrict__ dw, float* __restrict__ dl,
                               int Tn, int k) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= Tn) return;
    float dot = 0.f;
    for (int s = 0; s < k; ++s) dot += w[(size_t)t * k + s] * dw[(size_t)t * k + s];
    for (int s = 0; s < k; ++s) dl[(size_t)t * k + s] = w[(size_t)t * k + s] * (dw[(size_t)t * k + s] - dot);
}

// dx[t,c] += sum_s dl[t,s] * wgT[ids[t,s]][c]      (4 columns per thread)
// 16 bytes of dx per thread (8 bf16 / 4 fp32 columns); KT > 0: k at compile time, the k gate-weight rows are
// requested together with the dx piece.  d is a multiple of the vector width (checked with the shape).
template <class T, int VEC, int KT>
__global__ __launch_bounds__(256) void gate_bwd_dx_kernel(T* __restrict__ dx, const float* __restrict__ wgT,
                                                          const int32_t* __restrict__ ids,
                                                          const float* __restrict__ dl, int Tn, int d, int k) {
    const int q = d / VEC;
    const int64_t total = (int64_t)Tn * q;
    constexpr int KU = KT > 0 ? KT : 1;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int t = (int)(i / q), c = (int)(i - (int64_t)t * q) * VEC;
        T raw[VEC];
        static_assert(VEC * sizeof(T) == 16, "one 16-byte piece per thread");
        *reinterpret_cast<uint4*>(raw) = *reinterpret_cast<const uint4*>(dx + (size_t)t * d + c);
        float a[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) a[j] = Elem<T>::load(raw + j);
        if constexpr (KT > 0) {
            float g[KU], wv[KU][VEC];
#pragma unroll
            for (int s = 0; s < KU; ++s) {
                g[s] = dl[(size_t)t * KU + s];
                const float* row = wgT + (size_t)ids[(size_t)t * KU + s] * d + c;
#pragma unroll
                for (int j = 0; j < VEC; j += 4) {
                    const float4 v4 = *reinterpret_cast<const float4*>(row + j);
                    wv[s][j] = v4.x; wv[s][j + 1] = v4.y; wv[s][j + 2] = v4.z; wv[s][j + 3] = v4.w;
                }
            }
#pragma unroll
            for (int s = 0; s < KU; ++s)
#pragma unroll
                for (int j = 0; j < VEC; ++j) a[j] = fmaf(g[s], wv[s][j], a[j]);
        } else {
            for (int s = 0; s < k; ++s) {
                const float g = dl[(size_t)t * k + s];
                const float* row = wgT + (size_t)ids[(size_t)t * k + s] * d + c;
#pragma unroll
                for (int j = 0; j < VEC; ++j) a[j] = fmaf(g, row[j], a[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < VEC; ++j) Elem<T>::store(raw + j, a[j]);
        *reinterpret_cast<uint4*>(dx + (size_t)t * d + c) = *reinterpret_cast<const uint4*>(raw);
    }
}

template <class T>
static void launch_gate_bwd_dx(T* dx, const float* wgT, const int32_t* ids, const float* dl, int Tn, int d, int k,
                               hipStream_t st) {
    constexpr int VEC = 16 / sizeof(T);
    const int64_t items = (int64_t)Tn * (d / VEC);
    const int grid = (int)((items + 255) / 256 > 4096 ? 4096 : (items + 255) / 256);
    if (k == 1) gate_bwd_dx_kernel<T, VEC, 1><<<grid, 256, 0, st>>>(dx, wgT, ids, dl, Tn, d, k);
    else if (k == 2) gate_bwd_dx_kernel<T, VEC, 2><<<grid, 256, 0, st>>>(dx, wgT, ids, dl, Tn, d, k);
    else if (k == 4) gate_bwd_dx_kernel<T, VEC, 4><<<grid, 256, 0, st>>>(dx, wgT, ids, dl, Tn, d, k);
    else gate_bwd_dx_kernel<T, VEC, 0><<<grid, 256, 0, st>>>(dx, wgT, ids, dl, Tn, d, k);
}

// partial[chunk][e][c] = sum over the chunk's tokens of x[t,c] * dL[t,e]; a thread
// owns one column c of a slab, the accumulators of all experts live in LDS.
constexpr int kDwgSlab = 128;    // columns per workgroup (= threads)
constexpr int kDwgTokens = 256;  // tokens per chunk

template <class T>
__global__ __launch_bounds__(kDwgSlab) void gate_bwd_dwg_partial_kernel(
    const T* __restrict__ x, const int32_t* __restrict__ ids, const float* __restrict__ dl,
    float* __restrict__ partial, int Tn, int d, int E, int k) {
    extern __shared__ float accs[];  // [E][kDwgSlab]
    const int c = blockIdx.x * kDwgSlab + threadIdx.x;
    const int chunk = blockIdx.y;
    for (int e = 0; e < E; ++e) accs[e * kDwgSlab + threadIdx.x] = 0.f;
    const int t1 = min(Tn, (chunk + 1) * kDwgTokens);
    if (c < d) {
        for (int t = chunk * kDwgTokens; t < t1; ++t) {
            const float xv = Elem<T>::load(x + (size_t)t * d + c);
            // the k experts of one token are distinct, so their k read-modify-writes are
            // independent: read up to 8 accumulators, add, write back
            for (int s0 = 0; s0 < k; s0 += 8) {
                float v[8];
                int eo[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    eo[u] = (s0 + u < k ? ids[(size_t)t * k + s0 + u] : 0) * kDwgSlab + threadIdx.x;
                    v[u] = accs[eo[u]];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < k) accs[eo[u]] = fmaf(xv, dl[(size_t)t * k + s0 + u], v[u]);
            }
        }
        for (int e = 0; e < E; ++e)
            partial[((size_t)chunk * E + e) * d + c] = accs[e * kDwgSlab + threadIdx.x];
    }
}

// dw_gate[c][e] = sum over chunks, in chunk order
__global__ void gate_bwd_dwg_reduce_kernel(const float* __restrict__ partial, float* __restrict__ dwg, int nchunks,
                                           int d, int E) {
    const int64_t n = (int64_t)d * E;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int e = (int)(i / d), c = (int)(i - (int64_t)e * d);
        float a = 0.f;
        for (int ch = 0; ch < nchunks; ++ch) a += partial[((size_t)ch * E + e) * d + c];
        dwg[(size_t)c * E + e] = a;
    }
}

static inline int dwg_chunks(int Tn) { return (Tn + kDwgTokens - 1) / kDwgTokens; }

// ---- bf16: dW_g through the grouped GEMM --------------------------------------------------
// dL is written out densely as two bf16 matrices hi + lo (the pair carries 16 mantissa bits
// of the fp32 value), tokens are cut into chunks, each chunk's X^T * dL is one
// ragged-K GEMM group, and the chunk partials are added in chunk order.
// (512 tokens, or more for very long batches: the GEMM's group table holds MOE_MAX_EXPERTS groups)
static inline int mma_chunk_tokens(int Tn) {
    const int need = (Tn + MOE_MAX_EXPERTS - 1) / MOE_MAX_EXPERTS;
    return need <= 512 ? 512 : (need + 31) / 32 * 32;
}
static inline int mma_chunks(int Tn) { const int c = mma_chunk_tokens(Tn); return (Tn + c - 1) / c; }
static inline int pad64(int v) { return (v + 63) / 64 * 64; }  // the dense dL is a K operand: whole 64-wide k-stages

// one wavefront per token: dl[t,s] (fp32, for the dx update) and the dense hi/lo rows
__global__ __launch_bounds__(256) void gate_dl_dense_kernel(const int32_t* __restrict__ ids, const float* __restrict__ w,
                                                            const float* __restrict__ dw, float* __restrict__ dl,
                                                            bf16_t* __restrict__ hi, bf16_t* __restrict__ lo, int Tn,
                                                            int k, int n_pad) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;
    float dot = 0.f;
    for (int s = 0; s < k; ++s) dot += w[(size_t)t * k + s] * dw[(size_t)t * k + s];
    for (int s = lane; s < k; s += 64) dl[(size_t)t * k + s] = w[(size_t)t * k + s] * (dw[(size_t)t * k + s] - dot);
    for (int e = lane; e < n_pad; e += 64) {
        float v = 0.f;
        for (int s = 0; s < k; ++s)
            if (ids[(size_t)t * k + s] == e) v = w[(size_t)t * k + s] * (dw[(size_t)t * k + s] - dot);
        const bf16_t h = f32_to_bf16(v);
        hi[(size_t)t * n_pad + e] = h;
        lo[(size_t)t * n_pad + e] = f32_to_bf16(v - bf16_to_f32(h));
    }
}

__global__ void gate_chunk_offsets_kernel(int32_t* __restrict__ off, int nchunks, int chunk_tokens, int Tn,
                                          uint32_t* __restrict__ zero_row, int32_t* __restrict__ whole) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 128) zero_row[i] = 0u;
    if (i == 0) {  // the token range as a single group
        whole[0] = 0;
        whole[1] = Tn;
    }
    if (i <= nchunks) off[i] = (int)min((int64_t)i * chunk_tokens, (int64_t)Tn);
}

// wg_pad[c][j] = w_gate[c][j] for j < E, zero up to n_pad: the gate weight as a [N][K] operand with whole k-stages
__global__ void gate_pad_wg_kernel(const bf16_t* __restrict__ wg, bf16_t* __restrict__ wg_pad, int d, int E, int n_pad) {
    const int64_t n = (int64_t)d * n_pad;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i / n_pad), j = (int)(i - (int64_t)c * n_pad);
        wg_pad[i] = j < E ? wg[(size_t)c * E + j] : (bf16_t)0;
    }
}

// dw_gate[c][e] = sum over chunks (in chunk order) of partial[chunk][c][e]
__global__ void gate_bwd_dwg_reduce_mma_kernel(const float* __restrict__ partial, float* __restrict__ dwg, int nchunks,
                                               int d, int E, int n_pad) {
    const int64_t n = (int64_t)d * E;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i / E), e = (int)(i - (int64_t)c * E);
        float a = 0.f;
        int ch = 0;
        for (; ch + 8 <= nchunks; ch += 8) {  // eight loads in flight, added in chunk order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[((size_t)(ch + u) * d + c) * n_pad + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += v[u];
        }
        for (; ch < nchunks; ++ch) a += partial[((size_t)ch * d + c) * n_pad + e];
        dwg[i] = a;
    }
}

size_t gate_bwd_workspace_bytes(const moe_shape* s) {
    size_t b = align_up((size_t)pad64(s->E) * s->d * 4, 256);          // wgT (fp32), or the padded bf16 gate weight
    b += align_up((size_t)s->T * s->k * 4, 256);                       // dl
    const size_t p_valu = (size_t)dwg_chunks(s->T) * s->E * s->d * 4;
    const size_t p_mma = (size_t)mma_chunks(s->T) * s->d * pad64(s->E) * 4;
    b += align_up(p_valu > p_mma ? p_valu : p_mma, 256);               // partial sums
    b += 2 * align_up((size_t)s->T * pad64(s->E) * 2, 256);             // dense dL, hi and lo
    b += align_up((size_t)(mma_chunks(s->T) + 1) * 4, 256) + 512 + 256;  // token chunk offsets, a row of zeros, {0, T}
    return b;
}

}  // namespace moe

using namespace moe;

extern "C" moe_status moe_gate_topk(const moe_shape* s, const void* x, const void* w_gate, const float* bias,
                                    int32_t* topk_ids, float* topk_w, float* logits_out, void* ws, size_t ws_bytes,
                                    void* stream) {
    const char* who = "moe_gate_topk";
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(x, "x", who));
    MOE_RETURN_IF(check_ptr(w_gate, "w_gate", who));
    MOE_RETURN_IF(check_ptr(bias, "bias", who, true));
    MOE_RETURN_IF(check_ptr(topk_ids, "topk_ids", who));
    MOE_RETURN_IF(check_ptr(topk_w, "topk_w", who));
    MOE_RETURN_IF(check_ptr(logits_out, "logits_out", who, true));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (s->dtype == MOE_BF16 && s->d % 256 == 0) {
        MOE_RETURN_IF(check_ptr(ws, "ws", who));
        if (ws_bytes < gate_workspace_bytes(s)) {
            set_error("%s: workspace %zu < %zu bytes", who, ws_bytes, gate_workspace_bytes(s));
            return MOE_ERR_WORKSPACE_TOO_SMALL;
        }
        const int nt = (s->E + 31) / 32;
        const int NT = nt <= 1 ? 1 : nt <= 2 ? 2 : nt <= 4 ? 4 : 8;
        bf16_t* wgT = static_cast<bf16_t*>(ws);
        const int grid = (s->T + kGateMT - 1) / kGateMT;
        // 8 wavefronts (the contraction split 8 ways) halve the chain of dependent loads of a 32-token tile;
        // from 128 padded experts on, 4 wavefronts and half the partial-sum area (two workgroups per CU) do better.
        const int NW = (s->d % 512 == 0 && NT <= 2) ? 8 : 4;
        gate_pack_wg_kernel<<<256, 256, 0, st>>>(static_cast<const bf16_t*>(w_gate), wgT, s->d, s->E, NT, NW);
        size_t lds = (size_t)NW * kGateMT * NT * 32 * sizeof(float);            // partial logits
        if (lds < (size_t)kGateMT * MOE_MAX_EXPERTS * sizeof(float)) lds = (size_t)kGateMT * MOE_MAX_EXPERTS * sizeof(float);
#define MOE_GATE_LAUNCH(N, W)                                                                                      \
    {                                                                                                              \
        ensure_dynamic_lds(reinterpret_cast<const void*>(&gate_topk_mfma_kernel<N, W>), 4 * kGateMT * 256 * 4);    \
        gate_topk_mfma_kernel<N, W><<<grid, W * 64, lds, st>>>(static_cast<const bf16_t*>(x), wgT, bias, topk_ids, \
                                                               topk_w, logits_out, s->T, s->d, s->E, s->k);        \
    }
        if (NW == 8) {
            if (NT == 1) MOE_GATE_LAUNCH(1, 8) else if (NT == 2) MOE_GATE_LAUNCH(2, 8) else MOE_GATE_LAUNCH(4, 8)
        } else {
            if (NT == 1) MOE_GATE_LAUNCH(1, 4) else if (NT == 2) MOE_GATE_LAUNCH(2, 4) else if (NT == 4) MOE_GATE_LAUNCH(4, 4) else MOE_GATE_LAUNCH(8, 4)
        }
#undef MOE_GATE_LAUNCH
        return launch_status(who);
    }
    const int grid = (s->T + kGateTokens - 1) / kGateTokens;
    if (s->dtype == MOE_BF16)
        gate_topk_kernel<bf16_t><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(x),
                                                       static_cast<const bf16_t*>(w_gate), bias, topk_ids, topk_w,
                                                       logits_out, s->T, s->d, s->E, s->k);
    else
        gate_topk_kernel<float><<<grid, 256, 0, st>>>(static_cast<const float*>(x),
                                                      static_cast<const float*>(w_gate), bias, topk_ids, topk_w,
                                                      logits_out, s->T, s->d, s->E, s->k);
    return launch_status(who);
}

template <class T>
static moe_status gate_bwd_launch(const moe_shape* s, const T* x, const T* w_gate, const int32_t* ids,
                                  const float* w, const float* dw, T* dx, float* dwg, void* ws, hipStream_t st) {
    Carver cv(ws);
    float* wgT = static_cast<float*>(cv.take((size_t)pad64(s->E) * s->d * 4));  // fp32 transpose, or the padded bf16 copy
    float* dl = static_cast<float*>(cv.take((size_t)s->T * s->k * 4));
    const int nchunks = dwg_chunks(s->T);
    const size_t p_valu = (size_t)nchunks * s->E * s->d * 4;
    const size_t p_mma = (size_t)mma_chunks(s->T) * s->d * pad64(s->E) * 4;
    float* partial = static_cast<float*>(cv.take(p_valu > p_mma ? p_valu : p_mma));
    const bool mma = sizeof(T) == 2 && s->d % 8 == 0;
    if (mma) {
        const int n_pad = pad64(s->E), nch = mma_chunks(s->T);
        bf16_t* hi = static_cast<bf16_t*>(cv.take((size_t)s->T * n_pad * 2));
        bf16_t* lo = static_cast<bf16_t*>(cv.take((size_t)s->T * n_pad * 2));
        int32_t* coff = static_cast<int32_t*>(cv.take((size_t)(nch + 1) * 4));
        gate_dl_dense_kernel<<<(s->T + 3) / 4, 256, 0, st>>>(ids, w, dw, dl, hi, lo, s->T, s->k, n_pad);
        uint32_t* zero_row = static_cast<uint32_t*>(cv.take(512));
        int32_t* whole = static_cast<int32_t*>(cv.take(256));
        gate_chunk_offsets_kernel<<<(nch + 256) / 256, 256, 0, st>>>(coff, nch, mma_chunk_tokens(s->T), s->T, zero_row, whole);
        if (dx && s->k >= 4) {
            // dx += dL * W_g^T as a GEMM over the dense (hi + lo) dL: reads and writes dx once; the gate
            // weight stays in bf16 (padded to whole k-stages in the space of the fp32 transpose).  The
            // gather form below reads k rows of the fp32 gate weight per token from L2, which is what
            // costs from k = 4 on (measured: k = 8: 54 us against 89 us; k = 2: 93 us against 87 us).
            bf16_t* wg_pad = reinterpret_cast<bf16_t*>(wgT);
            gate_pad_wg_kernel<<<256, 256, 0, st>>>(reinterpret_cast<const bf16_t*>(w_gate), wg_pad, s->d, s->E, n_pad);
            launch_gate_dx_gemm(hi, lo, wg_pad, whole, s->d, n_pad, dx, st);
        } else if (dx) {
            gate_transpose_kernel<T><<<256, 256, 0, st>>>(w_gate, wgT, s->d, s->E);
            launch_gate_bwd_dx<T>(dx, wgT, ids, dl, s->T, s->d, s->k, st);
        }
        launch_gate_dwg_gemm(x, hi, lo, coff, nch, s->d, n_pad, partial, zero_row, st);
        gate_bwd_dwg_reduce_mma_kernel<<<256, 256, 0, st>>>(partial, dwg, nch, s->d, s->E, n_pad);
        return launch_status("moe_gate_topk_bwd");
    }
    gate_dl_kernel<<<(s->T + 255) / 256, 256, 0, st>>>(w, dw, dl, s->T, s->k);
    if (dx) {
        gate_transpose_kernel<T><<<256, 256, 0, st>>>(w_gate, wgT, s->d, s->E);
        launch_gate_bwd_dx<T>(dx, wgT, ids, dl, s->T, s->d, s->k, st);
    }
    const size_t lds = (size_t)s->E * kDwgSlab * sizeof(float);
    ensure_dynamic_lds(reinterpret_cast<const void*>(&gate_bwd_dwg_partial_kernel<T>), MOE_MAX_EXPERTS * kDwgSlab * 4);
    dim3 grid((s->d + kDwgSlab - 1) / kDwgSlab, nchunks);
    gate_bwd_dwg_partial_kernel<T><<<grid, kDwgSlab, lds, st>>>(x, ids, dl, partial, s->T, s->d, s->E, s->k);
    gate_bwd_dwg_reduce_kernel<<<256, 256, 0, st>>>(partial, dwg, nchunks, s->d, s->E);
    return launch_status("moe_gate_topk_bwd");
}

extern "C" moe_status moe_gate_topk_bwd(const moe_shape* s, const void* x, const void* w_gate,
                                        const int32_t* topk_ids, const float* topk_w, const float* dtopk_w,
                                        void* dx_inout, float* dw_gate, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "moe_gate_topk_bwd";
    MOE_RETURN_IF(check_shape(s, who));
    MOE_RETURN_IF(check_ptr(x, "x", who));
    MOE_RETURN_IF(check_ptr(w_gate, "w_gate", who));
    MOE_RETURN_IF(check_ptr(topk_ids, "topk_ids", who));
    MOE_RETURN_IF(check_ptr(topk_w, "topk_w", who));
    MOE_RETURN_IF(check_ptr(dtopk_w, "dtopk_w", who));
    MOE_RETURN_IF(check_ptr(dx_inout, "dx_inout", who, true));
    MOE_RETURN_IF(check_ptr(dw_gate, "dw_gate", who));
    MOE_RETURN_IF(check_ptr(ws, "ws", who));
    if (s->dtype == MOE_BF16 && s->d % 8 == 0) MOE_RETURN_IF(check_device(who));  // (this path runs the grouped GEMM)
    if (ws_bytes < gate_bwd_workspace_bytes(s)) {
        set_error("%s: workspace %zu < %zu bytes", who, ws_bytes, gate_bwd_workspace_bytes(s));
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (s->dtype == MOE_BF16)
        return gate_bwd_launch<bf16_t>(s, static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w_gate), topk_ids,
                                       topk_w, dtopk_w, static_cast<bf16_t*>(dx_inout), dw_gate, ws, st);
    return gate_bwd_launch<float>(s, static_cast<const float*>(x), static_cast<const float*>(w_gate), topk_ids, topk_w,
                                  dtopk_w, static_cast<float*>(dx_inout), dw_gate, ws, st);
}
