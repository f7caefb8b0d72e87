// FSEP parameter layout (paper section 3.1, executor): shard, unshard, reshard for the buffers of N
// ranks held in one device's memory.  Pure data movement: 16-byte pieces, every source read once,
// non-temporal accesses (nothing is reused), index arithmetic per piece.
#include "moe_internal.h"
#include "moe_fsep.h"

namespace moe {

typedef uint32_t fu32x4 __attribute__((ext_vector_type(4)));
constexpr int kFsepMaxSlots = 4096;

// piece index -> (row, piece in row) without 64-bit division in the loop body where it can be avoided
__global__ __launch_bounds__(256) void fsep_shard_kernel(const fu32x4* __restrict__ experts, fu32x4* __restrict__ shards,
                                                         int N, int E, int64_t chunk_p) {
    // output piece v = ((n*E + e)*chunk_p + o)  <-  experts[(e*N + n)*chunk_p + o]
    const int64_t total = (int64_t)N * E * chunk_p;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = v / chunk_p, o = v - row * chunk_p;
        const int n = (int)(row / E), e = (int)(row - (int64_t)n * E);
        __builtin_nontemporal_store(__builtin_nontemporal_load(&experts[((int64_t)e * N + n) * chunk_p + o]), &shards[v]);
    }
}

__global__ __launch_bounds__(256) void fsep_unshard_kernel(const fu32x4* __restrict__ shards,
                                                           const int32_t* __restrict__ hosted,
                                                           fu32x4* __restrict__ restored, int N, int E, int C,
                                                           int64_t chunk_p) {
    // output piece v = (((i*C + c)*N + n)*chunk_p + o)  <-  shards[(n*E + hosted[i][c])*chunk_p + o]
    const int64_t total = (int64_t)N * C * N * chunk_p;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = v / chunk_p, o = v - row * chunk_p;
        const int64_t slot = row / N;
        const int n = (int)(row - slot * N);
        const int e = hosted[slot];
        fu32x4 val = {0u, 0u, 0u, 0u};
        if (e >= 0 && e < E) val = __builtin_nontemporal_load(&shards[((int64_t)n * E + e) * chunk_p + o]);
        __builtin_nontemporal_store(val, &restored[v]);
    }
}

// One expert per blockIdx.y.  The slots that host it are collected once per workgroup (ascending
// order), then every thread adds up its pieces over them.
template <class T>
__global__ __launch_bounds__(256) void fsep_reshard_kernel(const fu32x4* __restrict__ grads,
                                                           const int32_t* __restrict__ hosted,
                                                           fu32x4* __restrict__ grad_shards, int N, int E, int C,
                                                           int64_t chunk_p) {
    __shared__ int32_t slots[kFsepMaxSlots];
    __shared__ int32_t n_slots;
    const int e = blockIdx.y;
    if (threadIdx.x == 0) {
        int cnt = 0;
        for (int q = 0; q < N * C; ++q)
            if (hosted[q] == e) slots[cnt++] = q;
        n_slots = cnt;
    }
    __syncthreads();
    const int cnt = n_slots;
    const int64_t total = (int64_t)N * chunk_p;  // pieces of this expert over all destination ranks = psi / piece
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (int64_t)gridDim.x * blockDim.x) {
        const int n = (int)(v / chunk_p);
        const int64_t o = v - (int64_t)n * chunk_p;
        constexpr int VALS = 16 / sizeof(T);
        float acc[VALS];
#pragma unroll
        for (int z = 0; z < VALS; ++z) acc[z] = 0.f;
        for (int s = 0; s < cnt; ++s) {
            // slot q of (rank i, slot c) holds psi values; chunk n of it starts at piece n*chunk_p: that is piece v
            const fu32x4 g = __builtin_nontemporal_load(&grads[(int64_t)slots[s] * total + v]);
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int z = 0; z < 4; ++z) {
                    acc[2 * z] += __uint_as_float(g[z] << 16);
                    acc[2 * z + 1] += __uint_as_float(g[z] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int z = 0; z < 4; ++z) acc[z] += __uint_as_float(g[z]);
            }
        }
        fu32x4 out;
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int z = 0; z < 4; ++z)
                out[z] = pack_bf16x2(acc[2 * z], acc[2 * z + 1]);
        } else {
#pragma unroll
            for (int z = 0; z < 4; ++z) out[z] = __float_as_uint(acc[z]);
        }
        __builtin_nontemporal_store(out, &grad_shards[((int64_t)n * E + e) * chunk_p + o]);
    }
}

static moe_status fsep_check(const char* who, int32_t N, int32_t E, int32_t C, int64_t psi, int32_t dtype) {
    if (dtype != MOE_F32 && dtype != MOE_BF16) {
        set_error("%s: dtype %d is neither MOE_F32 nor MOE_BF16", who, dtype);
        return MOE_ERR_INVALID_ARG;
    }
    const int64_t per_piece = dtype == MOE_BF16 ? 8 : 4;
    if (N < 1 || E < 1 || C < 1 || (int64_t)N * C > kFsepMaxSlots || psi < 1 || psi % (per_piece * N) != 0) {
        set_error("%s: N=%d E=%d C=%d psi=%lld: all >= 1, N*C <= %d, psi a multiple of %lld*N", who, N, E, C,
                  (long long)psi, kFsepMaxSlots, (long long)per_piece);
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

static int fsep_grid(int64_t pieces) {
    int64_t g = (pieces + 255) / 256;
    return (int)(g > 256 * 16 ? 256 * 16 : (g < 1 ? 1 : g));
}

}  // namespace moe

using namespace moe;

extern "C" moe_status moe_fsep_shard(int32_t N, int32_t E, int64_t psi, int32_t dtype, const void* experts, void* shards,
                                     void* stream) {
    const char* who = "moe_fsep_shard";
    MOE_RETURN_IF(fsep_check(who, N, E, 1, psi, dtype));
    MOE_RETURN_IF(check_ptr(experts, "experts", who));
    MOE_RETURN_IF(check_ptr(shards, "shards", who));
    const int64_t chunk_p = psi / N / (dtype == MOE_BF16 ? 8 : 4);
    fsep_shard_kernel<<<fsep_grid((int64_t)N * E * chunk_p), 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const fu32x4*>(experts), static_cast<fu32x4*>(shards), N, E, chunk_p);
    return launch_status(who);
}

extern "C" moe_status moe_fsep_unshard(int32_t N, int32_t E, int32_t C, int64_t psi, int32_t dtype, const void* shards,
                                       const int32_t* hosted, void* restored, void* stream) {
    const char* who = "moe_fsep_unshard";
    MOE_RETURN_IF(fsep_check(who, N, E, C, psi, dtype));
    MOE_RETURN_IF(check_ptr(shards, "shards", who));
    MOE_RETURN_IF(check_ptr(hosted, "hosted", who));
    MOE_RETURN_IF(check_ptr(restored, "restored", who));
    const int64_t chunk_p = psi / N / (dtype == MOE_BF16 ? 8 : 4);
    fsep_unshard_kernel<<<fsep_grid((int64_t)N * C * N * chunk_p), 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const fu32x4*>(shards), hosted, static_cast<fu32x4*>(restored), N, E, C, chunk_p);
    return launch_status(who);
}

extern "C" moe_status moe_fsep_reshard(int32_t N, int32_t E, int32_t C, int64_t psi, int32_t dtype, const void* grads,
                                       const int32_t* hosted, void* grad_shards, void* stream) {
    const char* who = "moe_fsep_reshard";
    MOE_RETURN_IF(fsep_check(who, N, E, C, psi, dtype));
    if (E > 65535) {
        set_error("%s: E=%d exceeds the grid's second dimension", who, E);
        return MOE_ERR_INVALID_ARG;
    }
    MOE_RETURN_IF(check_ptr(grads, "grads", who));
    MOE_RETURN_IF(check_ptr(hosted, "hosted", who));
    MOE_RETURN_IF(check_ptr(grad_shards, "grad_shards", who));
    const int64_t chunk_p = psi / N / (dtype == MOE_BF16 ? 8 : 4);
    int gx = fsep_grid((int64_t)N * chunk_p);
    const int cap = (256 * 16 + E - 1) / E;  // about 16 workgroups per CU over all experts
    if (gx > cap) gx = cap < 1 ? 1 : cap;
    dim3 grid(gx, E);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == MOE_BF16)
        fsep_reshard_kernel<bf16_t><<<grid, 256, 0, st>>>(static_cast<const fu32x4*>(grads), hosted,
                                                          static_cast<fu32x4*>(grad_shards), N, E, C, chunk_p);
    else
        fsep_reshard_kernel<float><<<grid, 256, 0, st>>>(static_cast<const fu32x4*>(grads), hosted,
                                                         static_cast<fu32x4*>(grad_shards), N, E, C, chunk_p);
    return launch_status(who);
}
