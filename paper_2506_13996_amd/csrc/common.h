// Pieces shared by the translation units of libalst: error macro, per-kernel timing, launch helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>

#include "../../include/alst.h"
#include "gemm_tile.h"

namespace alst {

#define ALST_HIP(call)                                   \
    do {                                                 \
        if ((call) != hipSuccess) return ALST_ERR_HIP;   \
    } while (0)

// Optional per-kernel timing (alst_profile_*): while enabled, each launch of a block GEMM (and each
// group of small kernels between them) is bracketed by a pair of HIP events on the launch stream.
// A benchmarking aid; its list of spans is process-wide and guarded by a lock.
// The kinds are the indices of alst_profile_read().
enum {
    PROF_LOGITS = 0, PROF_DHIDDEN = 1, PROF_DW = 2, PROF_OTHER = 3,
    PROF_MLP_LINEAR = 4, PROF_MLP_WGRAD = 5, PROF_MLP_OTHER = 6, PROF_KINDS = 8
};

struct ProfScope {
    hipEvent_t a, b;
    int kind;
    hipStream_t s;
    bool on;
    ProfScope(int kind, hipStream_t stream);
    ~ProfScope();
};

// The attribute below is per device: the first call on each device (up to kMaxDevices) sets it.
constexpr int kMaxDevices = 64;
static inline int current_device_slot() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

// Upper bound of the workgroups of a launch over tiles_r x tiles_c output blocks (4 x 8 patches;
// another patch shape is only chosen when it needs fewer); 0 if that does not fit a grid.
static inline int64_t checked_grid(int64_t tiles_r, int64_t tiles_c) {
    const int64_t patches = ((tiles_r + 3) / 4) * ((tiles_c + 7) / 8);
    const int64_t blocks = ((patches + 7) / 8) * 8 * 32;
    return blocks <= 0x7fffffff ? blocks : 0;
}

// Lets a kernel use the LDS of a compute unit beyond the default limit.
template <typename K>
static int allow_big_lds(K kernel, int bytes = kLdsBytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
               ? ALST_OK : ALST_ERR_HIP;
}

// Workgroups of a launch of persistent workgroups (one per compute unit, each walking its share of
// the launch's blocks): the compute units of the current device, a multiple of 8 so that the
// workgroups dealt to one XCD keep their XCD from block to block.  Looked up once per device.
static inline int persistent_grid() {
    static std::atomic<int> cached[kMaxDevices];
    const int dev = current_device_slot();
    if (dev < 0) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        int cu = 0;
        if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 8)
            cu = 256;
        n = cu / 8 * 8;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

}  // namespace alst
