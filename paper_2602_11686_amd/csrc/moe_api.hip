// Host-side plumbing of the C ABI: status text, thread-local error detail,
// argument validation and the workspace bound.  No kernels here.
#include <stdarg.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <utility>
#include <vector>

#include "moe_internal.h"

namespace moe {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

moe_status check_ptr(const void* p, const char* name, const char* who, bool nullable) {
    if (!p) {
        if (nullable) return MOE_OK;
        set_error("%s: %s is NULL", who, name);
        return MOE_ERR_INVALID_ARG;
    }
    if (!aligned16(p)) {
        set_error("%s: %s is not 16-byte aligned", who, name);
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

moe_status check_shape(const moe_shape* s, const char* who) {
    if (!s) {
        set_error("%s: shape is NULL", who);
        return MOE_ERR_INVALID_ARG;
    }
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) {
        set_error("%s: dtype %d is neither MOE_F32 nor MOE_BF16", who, s->dtype);
        return MOE_ERR_INVALID_ARG;
    }
    if (s->T < 1 || s->d < 1 || s->f < 1 || s->E < 1 || s->k < 1) {
        set_error("%s: T=%d d=%d f=%d E=%d k=%d must all be >= 1", who, s->T, s->d, s->f, s->E, s->k);
        return MOE_ERR_INVALID_ARG;
    }
    if (s->k > s->E) {
        set_error("%s: k=%d exceeds E=%d", who, s->k, s->E);
        return MOE_ERR_INVALID_ARG;
    }
    if (s->E > MOE_MAX_EXPERTS) {
        set_error("%s: E=%d exceeds MOE_MAX_EXPERTS=%d", who, s->E, MOE_MAX_EXPERTS);
        return MOE_ERR_UNSUPPORTED;
    }
    const int q = s->dtype == MOE_BF16 ? 8 : 4;
    if (s->d % q || s->f % q) {
        set_error("%s: d=%d and f=%d must be multiples of %d for this dtype", who, s->d, s->f, q);
        return MOE_ERR_UNSUPPORTED;
    }
    const int64_t R = (int64_t)s->T * s->k;
    if (R >= (int64_t(1) << 31) || R * std::max(s->d, s->f) >= (int64_t(1) << 37) ||
        (int64_t)s->E * s->d * s->f >= (int64_t(1) << 37)) {
        set_error("%s: problem too large (T*k=%lld)", who, (long long)R);
        return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

static std::mutex g_dev_mutex;
static int g_dev_state[64];  // per device: 0 unknown, 1 supported, 2 unsupported
static char g_dev_why[64][96];

moe_status check_device(const char* who) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        set_error("%s: no usable GPU (hipGetDevice: %s)", who, hipGetErrorString(e));
        return MOE_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (g_dev_state[dev] == 0) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            set_error("%s: hipGetDeviceProperties failed: %s", who, hipGetErrorString(e));
            return MOE_ERR_DEVICE;
        }
        const bool arch = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        const bool cus = prop.multiProcessorCount == 256;
        g_dev_state[dev] = arch && cus ? 1 : 2;
        snprintf(g_dev_why[dev], sizeof(g_dev_why[dev]), "%.40s with %d compute units", prop.gcnArchName,
                 prop.multiProcessorCount);
    }
    if (g_dev_state[dev] == 2) {
        set_error("%s: device %d is %s; the grouped GEMM needs gfx950 with all 256 compute units", who, dev,
                  g_dev_why[dev]);
        return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

void ensure_dynamic_lds(const void* kernel, int bytes) {
    static std::mutex m;
    static std::vector<std::pair<const void*, int>> done;
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::lock_guard<std::mutex> lock(m);
    for (const auto& d : done)
        if (d.first == kernel && d.second == dev) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    done.emplace_back(kernel, dev);
}

moe_status launch_status(const char* who) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: HIP launch failed: %s", who, hipGetErrorString(e));
        return MOE_ERR_DEVICE;
    }
    return MOE_OK;
}

}  // namespace moe

extern "C" {

const char* moe_status_string(moe_status s) {
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported shape or type";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

const char* moe_last_error(void) { return moe::g_err; }

int moe_abi_version(void) { return 1; }

size_t moe_workspace_bytes(const moe_shape* s) {
    if (moe::check_shape(s, "moe_workspace_bytes") != MOE_OK) return 0;
    size_t b = moe::gate_workspace_bytes(s);
    b = std::max(b, moe::permute_workspace_bytes(s));
    b = std::max(b, moe::ffn_fwd_workspace_bytes(s));
    b = std::max(b, moe::ffn_bwd_workspace_bytes(s));
    b = std::max(b, moe::gate_bwd_workspace_bytes(s));
    return b;
}

}  // extern "C"
