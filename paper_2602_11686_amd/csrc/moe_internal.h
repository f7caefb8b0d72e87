// Internal helpers shared by the HIP translation units of libmoe (host-side
// validation, error text, launch checks, bf16 conversion).  Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "moe.h"

namespace moe {

void set_error(const char* fmt, ...);
moe_status check_shape(const moe_shape* s, const char* who);
bool aligned16(const void* p);
moe_status check_ptr(const void* p, const char* name, const char* who, bool nullable = false);
moe_status launch_status(const char* who);
// The persistent grouped GEMM is laid out for a whole MI355X: 256 workgroups, one per compute unit, dealt
// round-robin to 8 XCDs.  MOE_OK on such a device (the answer is looked up once per device and kept),
// MOE_ERR_DEVICE if no device can be queried, MOE_ERR_UNSUPPORTED on anything else (another architecture, a
// compute-unit mask).
moe_status check_device(const char* who);
// hipFuncSetAttribute(MaxDynamicSharedMemorySize) once per (kernel, device); safe to call from any thread.
void ensure_dynamic_lds(const void* kernel, int bytes);

inline size_t el_size(const moe_shape* s) { return s->dtype == MOE_BF16 ? 2 : 4; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace layout of the grouped FFN calls: carve regions off one buffer.
struct Carver {
    char* base;
    size_t used = 0;
    explicit Carver(void* p) : base(static_cast<char*>(p)) {}
    void* take(size_t bytes) {
        void* r = base ? base + used : nullptr;
        used += align_up(bytes, 256);
        return r;
    }
};

size_t gate_workspace_bytes(const moe_shape* s);
size_t permute_workspace_bytes(const moe_shape* s);
size_t ffn_fwd_workspace_bytes(const moe_shape* s);
size_t ffn_bwd_workspace_bytes(const moe_shape* s);
size_t gate_bwd_workspace_bytes(const moe_shape* s);

// dW_g partials on the matrix cores (implemented next to the grouped GEMM):
//   partial[c][m][n] = sum over the tokens t of chunk c of x[t][m] * (dl_hi[t][n] + dl_lo[t][n])
// x [T][d] bf16, dl_hi / dl_lo [T][n_pad] bf16, chunk_offsets [nchunks+1] token ranges,
// partial [nchunks][d][n_pad] fp32; zero_row: 512 bytes of zeros in device memory.
void launch_gate_dwg_gemm(const void* x, const void* dl_hi, const void* dl_lo, const int32_t* chunk_offsets,
                          int nchunks, int d, int n_pad, float* partial, const void* zero_row, hipStream_t st);

// dx += (dl_hi + dl_lo) * wg_pad^T on the matrix cores (implemented next to the grouped GEMM):
// dl_hi / dl_lo [T][n_pad] bf16, wg_pad [d][n_pad] bf16 (gate weight, columns past E zero), n_pad a multiple
// of 64, whole = {0, T} in device memory, dx [T][d] bf16 read and written.
void launch_gate_dx_gemm(const void* dl_hi, const void* dl_lo, const void* wg_pad, const int32_t* whole, int d, int n_pad,
                         void* dx, hipStream_t st);

// ---- device-side element helpers -------------------------------------------
typedef uint16_t bf16_t;  // raw bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest, ties to even (inputs are finite by contract)
__device__ __forceinline__ bf16_t f32_to_bf16(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// two fp32 values -> two bf16 in one dword (low half first), round to nearest even, with the packed conversion
// instruction of gfx950 (inputs are finite by contract)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    f32x2_t v;
    v[0] = lo;
    v[1] = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <class T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// silu and its derivative with the hardware exp2 / reciprocal (about 1 ulp each): these run on
// 128 accumulators per lane in the GEMM epilogues, where a full-precision division is what costs.
__device__ __forceinline__ float sigmoid_f(float a) { return __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }
__device__ __forceinline__ float silu_f(float a) { return a * sigmoid_f(a); }
__device__ __forceinline__ float silu_grad_f(float a) {
    const float s = sigmoid_f(a);
    return s * (1.0f + a * (1.0f - s));
}

}  // namespace moe

#define MOE_RETURN_IF(expr)                    \
    do {                                       \
        moe_status _st = (expr);               \
        if (_st != MOE_OK) return _st;         \
    } while (0)
