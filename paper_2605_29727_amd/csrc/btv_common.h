// Internal helpers shared by the HIP translation units of libbastion_tv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "bastion_tv.h"

#define BTV_WS_ALIGN 256

int btv_fail(int code, const char *fmt, ...);   // records the thread-local message, returns code

#define BTV_REQUIRE(cond, ...)                         \
    do {                                               \
        if (!(cond)) return btv_fail(BTV_EINVAL, __VA_ARGS__); \
    } while (0)

#define BTV_HIP(call)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess) return btv_fail(BTV_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

static inline size_t btv_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace layout used by every entry point: word 0 of the workspace is the data-error flag.
#define BTV_WS_HEADER 256

static inline int btv_check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return BTV_OK;
    if (!ws) return btv_fail(BTV_EWORKSPACE, "workspace is NULL, %zu bytes needed", need);
    if (((uintptr_t)ws) % BTV_WS_ALIGN) return btv_fail(BTV_EWORKSPACE, "workspace not %d-byte aligned", BTV_WS_ALIGN);
    if (have < need) return btv_fail(BTV_EWORKSPACE, "workspace too small: %zu < %zu bytes", have, need);
    return BTV_OK;
}

// ---- internal launchers (defined in the .hip files) --------------------------------------------
int btv_launch_anc_mask(const int32_t *parent, const int32_t *q_offset, int batch, int M_max, int total_M,
                        uint32_t *anc, uint32_t *flag, hipStream_t st);
