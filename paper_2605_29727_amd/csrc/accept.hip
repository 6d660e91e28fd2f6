// Acceptance walk on the GPU (gfx950): target argmax per tree row, greedy walk, and the
// token-level rejection walk at temperature 1.
//
// App. C "Acceptance" / Sec. 3.1: the committed tokens are the longest root-to-node path the
// target itself would have produced.  Rows of `logits`: 0 = root, 1+i = node i.
#include "btv_common.h"

#include <algorithm>
#include <climits>

namespace {

constexpr int ACHUNK = 8192;     // vocabulary elements per argmax workgroup

struct Best { float v; int i; };

__device__ __forceinline__ void best_take(Best &b, float v, int i)
{   // larger value wins; equal values: lower index wins; NaN never wins
    if (v > b.v || (v == b.v && i < b.i)) { b.v = v; b.i = i; }
}

__device__ __forceinline__ Best best_wave(Best b)
{
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = __shfl_xor(b.v, off);
        int oi = __shfl_xor(b.i, off);
        best_take(b, ov, oi);
    }
    return b;
}

// grid = (chunks, rows).  part[(row*chunks + chunk)] = best of the chunk.
template <bool BF16>
__global__ __launch_bounds__(256) void argmax_chunks(const void *logits, int V, Best *part)
{
    __shared__ Best wb[4];
    const int tid = threadIdx.x, chunk = blockIdx.x, row = blockIdx.y;
    const int v0 = chunk * ACHUNK, v1 = min(v0 + ACHUNK, V);
    Best b = { -INFINITY, INT_MAX };
    if (BF16) {
        const uint16_t *x = static_cast<const uint16_t *>(logits) + (size_t)row * V;
        if ((((size_t)row * V * 2) & 15) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0) {
            for (int v = v0 + tid * 8; v < v1; v += 256 * 8) {
                if (v + 8 <= v1) {
                    uint4 q = *reinterpret_cast<const uint4 *>(x + v);
                    uint32_t wds[4] = { q.x, q.y, q.z, q.w };
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        best_take(b, __uint_as_float(wds[e] << 16), v + 2 * e);
                        best_take(b, __uint_as_float(wds[e] & 0xFFFF0000u), v + 2 * e + 1);
                    }
                } else {
                    for (int e = v; e < v1; ++e) best_take(b, __uint_as_float((uint32_t)x[e] << 16), e);
                }
            }
        } else {
            for (int v = v0 + tid; v < v1; v += 256) best_take(b, __uint_as_float((uint32_t)x[v] << 16), v);
        }
    } else {
        const float *x = static_cast<const float *>(logits) + (size_t)row * V;
        if ((((size_t)row * V * 4) & 15) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0) {
            for (int v = v0 + tid * 4; v < v1; v += 256 * 4) {
                if (v + 4 <= v1) {
                    float4 q = *reinterpret_cast<const float4 *>(x + v);
                    best_take(b, q.x, v); best_take(b, q.y, v + 1); best_take(b, q.z, v + 2); best_take(b, q.w, v + 3);
                } else {
                    for (int e = v; e < v1; ++e) best_take(b, x[e], e);
                }
            }
        } else {
            for (int v = v0 + tid; v < v1; v += 256) best_take(b, x[v], v);
        }
    }
    b = best_wave(b);
    if ((tid & 63) == 0) wb[tid >> 6] = b;
    __syncthreads();
    if (tid == 0) {
        Best r = wb[0];
        best_take(r, wb[1].v, wb[1].i); best_take(r, wb[2].v, wb[2].i); best_take(r, wb[3].v, wb[3].i);
        part[(size_t)row * gridDim.x + chunk] = r;
    }
}

// One workgroup: finish the argmax of every row, then walk the tree.
__global__ __launch_bounds__(256) void greedy_walk(const Best *part, int chunks, const int32_t *parent,
                                                   const int32_t *token, int M, int32_t *path, int32_t *n_acc,
                                                   int32_t *bonus, int32_t *argmax_out)
{
    __shared__ int t[BTV_MAX_NODES + 1];
    __shared__ int par[BTV_MAX_NODES], tok[BTV_MAX_NODES];
    __shared__ int next;
    const int tid = threadIdx.x;
    for (int r = tid; r <= M; r += 256) {
        Best b = part[(size_t)r * chunks];
        for (int c = 1; c < chunks; ++c) best_take(b, part[(size_t)r * chunks + c].v, part[(size_t)r * chunks + c].i);
        t[r] = b.i == INT_MAX ? 0 : b.i;
        if (argmax_out) argmax_out[r] = t[r];
    }
    for (int c = tid; c < M; c += 256) { par[c] = parent[c]; tok[c] = token[c]; }
    __syncthreads();
    int cur = -1, n = 0;
    for (;;) {
        if (tid == 0) next = INT_MAX;
        __syncthreads();
        const int want = t[cur + 1];
        for (int c = tid; c < M; c += 256)
            if (par[c] == cur && tok[c] == want) atomicMin(&next, c);
        __syncthreads();
        const int nx = next;
        __syncthreads();
        if (nx == INT_MAX || n >= M) break;
        if (tid == 0) path[n] = nx;
        cur = nx; ++n;
    }
    if (tid == 0) { *n_acc = n; *bonus = t[cur + 1]; }
}

// ------------------------------------------------------------------------------------------------
// Stochastic walk: one workgroup of 1024 threads; p and q live in the workspace (fp32), every
// vocabulary-wide sum is accumulated in fp64.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ double block_sum(double x, double *sh, int tid)
{
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((tid & 63) == 0) sh[tid >> 6] = x;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < 16; ++w) s += sh[w];
    return s;
}

__device__ __forceinline__ float block_max(float x, float *sh, int tid)
{
    for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    __syncthreads();
    if ((tid & 63) == 0) sh[tid >> 6] = x;
    __syncthreads();
    float s = sh[0];
    for (int w = 1; w < 16; ++w) s = fmaxf(s, sh[w]);
    return s;
}

template <bool BF16>
__device__ __forceinline__ float load_logit(const void *logits, size_t idx)
{
    if (BF16) return __uint_as_float((uint32_t)static_cast<const uint16_t *>(logits)[idx] << 16);
    return static_cast<const float *>(logits)[idx];
}

template <bool BF16>
__global__ __launch_bounds__(1024) void stochastic_walk(const void *logits, const float *marg, int B,
                                                        const int32_t *parent, const int32_t *token, int M, int V,
                                                        const float *uniforms, float *p, float *q, int32_t *path,
                                                        int32_t *n_acc, int32_t *bonus)
{
    __shared__ double shd[16];
    __shared__ float shf[16];
    __shared__ double seg[1024];
    __shared__ int found, lastpos;
    const int tid = threadIdx.x;
    int cur = -1, n = 0, ui = 0, d = 0;
    for (;;) {
        // p = softmax(logits[row(cur)])
        const size_t base = (size_t)(cur + 1) * V;
        float mx = -INFINITY;
        for (int v = tid; v < V; v += 1024) mx = fmaxf(mx, load_logit<BF16>(logits, base + v));
        mx = block_max(mx, shf, tid);
        double z = 0.0;
        for (int v = tid; v < V; v += 1024) {
            float e = expf(load_logit<BF16>(logits, base + v) - mx);
            p[v] = e; z += (double)e;
        }
        z = block_sum(z, shd, tid);
        for (int v = tid; v < V; v += 1024) p[v] = (float)((double)p[v] / z);
        int accepted = -1;
        if (d < B) {
            for (int v = tid; v < V; v += 1024) q[v] = marg[(size_t)d * V + v];
            __syncthreads();
            for (int c = 0; c < M; ++c) {
                if (parent[c] != cur) continue;            // uniform across the workgroup
                const int tk = token[c];
                const double u = (double)uniforms[ui++];
                const double lhs = u * (double)q[tk], rhs = (double)p[tk];
                if (lhs < rhs) { accepted = c; break; }
                __syncthreads();                             // everyone has read p[tk], q[tk]
                double zr = 0.0;
                for (int v = tid; v < V; v += 1024) { float r = p[v] - q[v]; zr += (double)(r > 0.f ? r : 0.f); }
                zr = block_sum(zr, shd, tid);
                if (zr > 0.0)
                    for (int v = tid; v < V; v += 1024) { float r = p[v] - q[v]; p[v] = (float)((double)(r > 0.f ? r : 0.f) / zr); }
                __syncthreads();
                if (tid == 0) q[tk] = 0.f;
                __syncthreads();
                double zq = 0.0;
                for (int v = tid; v < V; v += 1024) zq += (double)q[v];
                zq = block_sum(zq, shd, tid);
                if (zq > 0.0)
                    for (int v = tid; v < V; v += 1024) q[v] = (float)((double)q[v] / zq);
                __syncthreads();
            }
        }
        if (accepted >= 0) {
            if (tid == 0) path[n] = accepted;
            cur = accepted; ++n; ++d;
            __syncthreads();
            continue;
        }
        // bonus: smallest v with cumsum(p)[v] > u; each thread owns a contiguous segment
        const double u = (double)uniforms[ui++];
        const int per = (V + 1023) / 1024, s0 = min(tid * per, V), s1 = min(s0 + per, V);
        __syncthreads();
        double loc = 0.0;
        int lp = -1;
        for (int v = s0; v < s1; ++v) { loc += (double)p[v]; if (p[v] > 0.f) lp = v; }
        seg[tid] = loc;
        if (tid == 0) { found = INT_MAX; lastpos = 0; }
        __syncthreads();
        double cum = 0.0;
        for (int s = 0; s < tid; ++s) cum += seg[s];
        for (int v = s0; v < s1; ++v) {
            cum += (double)p[v];
            if (cum > u) { atomicMin(&found, v); break; }
        }
        if (lp >= 0) atomicMax(&lastpos, lp);
        __syncthreads();
        if (tid == 0) { *bonus = found == INT_MAX ? lastpos : found; *n_acc = n; }
        break;
    }
}

int check_accept(const void *logits, int dtype, const int32_t *parent, const int32_t *token, int M, int V,
                 int32_t *path, int32_t *n_acc, int32_t *bonus)
{
    BTV_REQUIRE(logits && parent && token && path && n_acc && bonus, "null pointer");
    BTV_REQUIRE(dtype == BTV_F32 || dtype == BTV_BF16, "dtype=%d unsupported", dtype);
    BTV_REQUIRE(M >= 1 && M <= BTV_MAX_NODES, "M=%d outside [1,%d]", M, BTV_MAX_NODES);
    BTV_REQUIRE(V >= 1, "V=%d", V);
    return BTV_OK;
}

}  // namespace

extern "C" {

size_t btv_tree_accept_workspace(int M, int V, int stochastic)
{
    if (M < 1 || M > BTV_MAX_NODES || V < 1) return 0;
    if (stochastic) return BTV_WS_HEADER + 2 * btv_align_up((size_t)V * 4, BTV_WS_ALIGN);
    int chunks = (V + ACHUNK - 1) / ACHUNK;
    return BTV_WS_HEADER + btv_align_up((size_t)(M + 1) * chunks * sizeof(Best), BTV_WS_ALIGN);
}

int btv_tree_accept_greedy(const void *logits, int dtype, const int32_t *parent, const int32_t *token, int M, int V,
                           int32_t *path, int32_t *n_acc, int32_t *bonus, int32_t *argmax_out, void *ws,
                           size_t ws_bytes, void *stream)
{
    int rc = check_accept(logits, dtype, parent, token, M, V, path, n_acc, bonus);
    if (rc) return rc;
    rc = btv_check_ws(ws, ws_bytes, btv_tree_accept_workspace(M, V, 0));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Best *part = reinterpret_cast<Best *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    int chunks = (V + ACHUNK - 1) / ACHUNK;
    if (dtype == BTV_BF16) hipLaunchKernelGGL(argmax_chunks<true>, dim3(chunks, M + 1), dim3(256), 0, st, logits, V, part);
    else hipLaunchKernelGGL(argmax_chunks<false>, dim3(chunks, M + 1), dim3(256), 0, st, logits, V, part);
    BTV_HIP(hipGetLastError());
    hipLaunchKernelGGL(greedy_walk, dim3(1), dim3(256), 0, st, part, chunks, parent, token, M, path, n_acc, bonus,
                       argmax_out);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

int btv_tree_accept_stochastic(const void *logits, int dtype, const float *marginals, int B, const int32_t *parent,
                               const int32_t *token, int M, int V, const float *uniforms, int32_t *path,
                               int32_t *n_acc, int32_t *bonus, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_accept(logits, dtype, parent, token, M, V, path, n_acc, bonus);
    if (rc) return rc;
    BTV_REQUIRE(marginals && uniforms, "null pointer");
    BTV_REQUIRE(B >= 1 && B <= BTV_MAX_DEPTH, "B=%d outside [1,%d]", B, BTV_MAX_DEPTH);
    rc = btv_check_ws(ws, ws_bytes, btv_tree_accept_workspace(M, V, 1));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    size_t vb = btv_align_up((size_t)V * 4, BTV_WS_ALIGN);
    float *p = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    float *q = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER + vb);
    if (dtype == BTV_BF16)
        hipLaunchKernelGGL(stochastic_walk<true>, dim3(1), dim3(1024), 0, st, logits, marginals, B, parent, token, M, V,
                           uniforms, p, q, path, n_acc, bonus);
    else
        hipLaunchKernelGGL(stochastic_walk<false>, dim3(1), dim3(1024), 0, st, logits, marginals, B, parent, token, M, V,
                           uniforms, p, q, path, n_acc, bonus);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

}  // extern "C"
