// Error reporting and small host-side entry points of libbastion_tv.
#include "btv_common.h"

namespace {
thread_local char g_err[512] = "";
}

int btv_fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" {

const char *btv_last_error(void) { return g_err; }

int btv_version(void) { return 1; }

int btv_workspace_status(void *ws, void *stream)
{
    if (!ws) return btv_fail(BTV_EWORKSPACE, "workspace is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t flag = 0, zero = 0;
    BTV_HIP(hipMemcpyAsync(&flag, ws, sizeof(flag), hipMemcpyDeviceToHost, st));
    BTV_HIP(hipStreamSynchronize(st));
    if (flag) {
        BTV_HIP(hipMemcpyAsync(ws, &zero, sizeof(zero), hipMemcpyHostToDevice, st));
        BTV_HIP(hipStreamSynchronize(st));
        return btv_fail(BTV_EDATA, "a kernel flagged invalid data (flag=0x%x)", flag);
    }
    return BTV_OK;
}

}  // extern "C"
