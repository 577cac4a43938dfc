// Shared internals of the conststn library: status/error plumbing, device buffers, the
// device-resident CSF handle.  Nothing here is visible across the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/conststn.h"

namespace cst {

// ---- error plumbing --------------------------------------------------------------------
void set_error(const char *fmt, ...);
const char *get_error();
void clear_error();

#define CST_HIP(expr)                                                                   \
    do {                                                                                \
        hipError_t e__ = (expr);                                                        \
        if (e__ != hipSuccess) {                                                        \
            cst::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__),      \
                           __FILE__, __LINE__);                                         \
            return (e__ == hipErrorOutOfMemory) ? CONSTSTN_ENOMEM : CONSTSTN_EHIP;      \
        }                                                                               \
    } while (0)

#define CST_TRY(expr)                                \
    do {                                             \
        conststn_status s__ = (expr);                \
        if (s__ != CONSTSTN_OK) return s__;          \
    } while (0)

// ---- owned device buffer ---------------------------------------------------------------
template <typename T>
struct DevBuf {
    T *p = nullptr;
    size_t n = 0;
    DevBuf() = default;
    DevBuf(const DevBuf &) = delete;
    DevBuf &operator=(const DevBuf &) = delete;
    ~DevBuf() { release(); }
    void release() {
        if (p) (void)hipFree(p);
        p = nullptr;
        n = 0;
    }
    conststn_status alloc(size_t count) {
        release();
        if (count == 0) count = 1;   // keep a valid pointer for empty arrays
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&p), count * sizeof(T));
        if (e != hipSuccess) {
            p = nullptr;
            set_error("hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
            (void)hipGetLastError();
            return CONSTSTN_ENOMEM;
        }
        n = count;
        return CONSTSTN_OK;
    }
};

static inline int ceil_log2_u64(uint64_t v) {   // bits needed to hold values 0..v-1
    int b = 0;
    while (b < 64 && (uint64_t(1) << b) < v) ++b;
    return b;
}

static inline int64_t div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace cst

// The CSF handle.  Level l: idx[l] (nodes[l] entries), ptr[l] (nodes[l]+1 entries, l < order-1).
struct conststn_csf_s {
    int order = 0;
    int64_t dims[CONSTSTN_MAX_ORDER] = {0};
    int mode_order[CONSTSTN_MAX_ORDER] = {0};
    int64_t nnz = 0;
    int64_t nodes[CONSTSTN_MAX_ORDER] = {0};
    cst::DevBuf<int32_t> idx[CONSTSTN_MAX_ORDER];
    cst::DevBuf<int64_t> ptr[CONSTSTN_MAX_ORDER];
    cst::DevBuf<double> vals;
    int device = 0;
};
