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

namespace {
// Streaming read for the bandwidth ceiling: every workgroup owns a contiguous piece, a wave reads 1 KiB per load
// instruction, four loads in flight per thread; the words are folded into one per workgroup so that the loads
// cannot be dropped.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ src, size_t per_wg, size_t n16,
                                                          uint32_t *__restrict__ sink)
{
    const size_t lo = (size_t)blockIdx.x * per_wg, hi = lo + per_wg < n16 ? lo + per_wg : n16;
    uint32_t acc = 0;
    size_t i = lo + threadIdx.x;
    for (; i + 3 * 256 < hi; i += 4 * 256) {
        const uint4 a = src[i], b = src[i + 256], c = src[i + 512], d = src[i + 768];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < hi; i += 256) { const uint4 a = src[i]; acc ^= a.x ^ a.y ^ a.z ^ a.w; }
    for (int off = 32; off >= 1; off >>= 1) acc ^= __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], acc);
}

// Register-resident matrix-core loop for the arithmetic ceiling: every wave keeps four independent 32x32 fp32
// accumulators and issues `iters` rounds of four v_mfma_f32_32x32x16_bf16 on operands that never leave registers.
// The accumulators are folded into one word per wave so that the work cannot be dropped.
typedef __bf16 pk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512, 1) void mfma_peak_kernel(int iters, uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    pk_bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(0.001f * (float)((lane + e) & 15)); b[e] = (__bf16)(0.002f * (float)((lane ^ e) & 7)); }
    pk_f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int v = 0; v < 16; ++v) { c0[v] = 0.f; c1[v] = 0.f; c2[v] = 0.f; c3[v] = 0.f; }
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float f = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) f += c0[v] + c1[v] + c2[v] + c3[v];
    if (lane == 0) atomicXor(&sink[(blockIdx.x * 8 + (threadIdx.x >> 6)) & 4095], __float_as_uint(f));
}
}  // namespace

extern "C" {

int btv_mfma_peak(int workgroups, int iters, void *sink, size_t sink_bytes, double *flops, void *stream)
{
    BTV_REQUIRE(sink != nullptr && flops != nullptr, "null pointer");
    BTV_REQUIRE(workgroups >= 1 && workgroups <= 65536 && iters >= 1 && iters <= (1 << 24), "workgroups=%d or iters=%d out of range",
                workgroups, iters);
    BTV_REQUIRE(sink_bytes >= 4096 * 4, "sink needs %d bytes", 4096 * 4);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(workgroups), dim3(512), 0, static_cast<hipStream_t>(stream), iters,
                       static_cast<uint32_t *>(sink));
    BTV_HIP(hipGetLastError());
    *flops = (double)workgroups * 8.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
    return BTV_OK;
}

int btv_stream_read(const void *src, size_t bytes, void *sink, size_t sink_bytes, void *stream)
{
    BTV_REQUIRE(src != nullptr && sink != nullptr, "null pointer");
    BTV_REQUIRE((reinterpret_cast<uintptr_t>(src) & 15) == 0 && bytes % 16 == 0, "src must be 16-byte aligned, bytes a multiple of 16");
    const int wgs = 256 * 16;
    BTV_REQUIRE(sink_bytes >= (size_t)wgs * 4, "sink needs %d bytes", wgs * 4);
    const size_t n16 = bytes / 16, per_wg = ((n16 + wgs - 1) / wgs + 1023) / 1024 * 1024;
    hipLaunchKernelGGL(stream_read_kernel, dim3(wgs), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), per_wg, n16, static_cast<uint32_t *>(sink));
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

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

// Verifier cost model (App. E), host arithmetic only.  The two totals are the appendix's displayed sums: FLOPs =
// layers * (projections + scores and PV + FFN) + LM head; traffic = weights (embedding and LM head counted apart)
// + KV cache read and write + activations, in elements times bytes per element.
int btv_verify_cost(double s, double c, double layers, double h, double nq, double nkv, double d, double hffn, double V,
                    double bp, double peak_flops, double bandwidth, double calib_scale, double calib_offset, double *out)
{
    BTV_REQUIRE(out != nullptr, "null pointer");
    BTV_REQUIRE(s >= 0 && c >= 0 && layers >= 0 && h > 0 && nq > 0 && nkv > 0 && d > 0 && hffn >= 0 && V > 0 && bp > 0,
                "negative or zero model dimension");
    BTV_REQUIRE(peak_flops > 0 && bandwidth > 0, "peak_flops and bandwidth must be positive");
    const double hq = nq * d, hkv = nkv * d;
    const double flops = layers * (4.0 * s * h * hq + 4.0 * s * h * hkv + 4.0 * s * (c + s) * hq + 6.0 * s * h * hffn) +
                         2.0 * s * h * V;
    const double elems = 2.0 * V * h + s * (h + V) +
                         layers * (2.0 * h * (hq + hkv) + 3.0 * h * hffn + 2.0 * hkv * (c + 2.0 * s) +
                                   4.0 * s * (h + hq + hffn) + 2.0 * nq * s * (c + s));
    const double bytes = bp * elems;
    const double tf = flops / peak_flops, tb = bytes / bandwidth;
    const double r = tf > tb ? tf : tb;
    out[0] = flops; out[1] = bytes; out[2] = r; out[3] = calib_scale * r + calib_offset;
    return BTV_OK;
}

// Static calibration (Sec. 5.2): least-squares line through (pred, obs), two passes (means, then centred moments).
int btv_calib_fit_linear(const double *pred, const double *obs, int n, double *calib_scale, double *calib_offset)
{
    BTV_REQUIRE(pred != nullptr && obs != nullptr && calib_scale != nullptr && calib_offset != nullptr, "null pointer");
    BTV_REQUIRE(n >= 2, "a line needs at least two points");
    double sum_p = 0.0, sum_o = 0.0;
    for (int i = 0; i < n; ++i) {
        BTV_REQUIRE(std::isfinite(pred[i]) && std::isfinite(obs[i]), "non-finite sample");
        sum_p += pred[i];
        sum_o += obs[i];
    }
    const double mean_p = sum_p / n, mean_o = sum_o / n;
    double var = 0.0, cov = 0.0;
    for (int i = 0; i < n; ++i) {
        const double dp = pred[i] - mean_p;
        var += dp * dp;
        cov += dp * (obs[i] - mean_o);
    }
    BTV_REQUIRE(var > 0.0, "all predictions are equal: the slope is undetermined");
    *calib_scale = cov / var;
    *calib_offset = mean_o - (cov / var) * mean_p;
    return BTV_OK;
}

// Online calibration (Sec. 5.2): exponential moving average of the observed / predicted latency ratio.
int btv_calib_ema_update(double *c, double alpha, double obs, double pred)
{
    BTV_REQUIRE(c != nullptr, "null pointer");
    BTV_REQUIRE(alpha >= 0.0 && alpha <= 1.0, "alpha outside [0, 1]");
    BTV_REQUIRE(pred > 0.0 && obs >= 0.0 && std::isfinite(obs) && std::isfinite(pred), "latencies must be positive and finite");
    *c = (1.0 - alpha) * *c + alpha * (obs / pred);
    return BTV_OK;
}

// Cost curve for the budget controller (Eq. 6): C(N) = t_other + c_ema * (calibrated T_verify of N + 1 tokens).
int btv_verify_cost_curve(int N_max, double c, double layers, double h, double nq, double nkv, double d, double hffn,
                          double V, double bp, double peak_flops, double bandwidth, double calib_scale,
                          double calib_offset, double c_ema, double t_other, double *cost)
{
    BTV_REQUIRE(cost != nullptr, "null pointer");
    BTV_REQUIRE(N_max >= 0 && N_max <= BTV_MAX_NODES, "N_max outside [0, BTV_MAX_NODES]");
    BTV_REQUIRE(std::isfinite(c_ema) && std::isfinite(t_other), "non-finite calibration state");
    for (int n = 1; n <= N_max; ++n) {
        double out[4];
        const int rc = btv_verify_cost(n + 1.0, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale,
                                       calib_offset, out);
        if (rc != BTV_OK) return rc;
        cost[n - 1] = t_other + c_ema * out[3];
    }
    return BTV_OK;
}

}  // extern "C"
