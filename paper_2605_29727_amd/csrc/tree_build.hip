// Best-first draft-tree construction on the GPU (gfx950).
//
// Sec. 3.3 / Prop. 3.3 / Algorithm 1's frontier rule at a fixed budget N: repeatedly emit the
// frontier prefix with the largest path score rho (Eq. 1), then push its best child and its next
// sibling.  Two steps:
//   1. per-position exact top-K of the marginals (K = min(V, N): a rank-j token is preceded by its
//      j earlier siblings, so ranks >= N can never be emitted), ordered (probability desc, id asc);
//      done as LDS bitonic sorts of 64-bit keys  prob_bits << 32 | ~id  over 2048-element chunks,
//      followed by rounds that merge the per-chunk winners;
//   2. the expansion itself: one wavefront, frontier in LDS, wave-wide arg-best per emitted node.
// rho(child) = rho(parent) * q is one fp32 multiply (never fused), the root has rho = 1.
// Frontier order: rho desc, depth asc, rank path lexicographic asc (ranks < 256 pack into 16 bytes).
#include "btv_common.h"

#include <algorithm>

namespace {

constexpr int CHUNK = 2048;      // elements sorted per workgroup
constexpr int MAXB = 16;         // draft positions supported by the expansion kernel (rank path = 16 bytes)

__device__ __forceinline__ unsigned long long make_key(float prob, uint32_t id)
{
    uint32_t b = __float_as_uint(prob);
    if (b == 0x80000000u) b = 0u;                  // -0.0 sorts as 0
    return ((unsigned long long)b << 32) | (unsigned long long)(0xFFFFFFFFu - id);
}

// Descending bitonic sort of CHUNK 64-bit keys held in LDS by 256 threads.
__device__ __forceinline__ void bitonic_desc(unsigned long long *keys, int tid)
{
    for (int k = 2; k <= CHUNK; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
#pragma unroll
            for (int e = 0; e < CHUNK / 512; ++e) {
                int t = tid + e * 256;                    // compare-exchange index 0..CHUNK/2-1
                int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int p = i | j;
                unsigned long long a = keys[i], b = keys[p];
                bool desc = (i & k) == 0;
                if ((a < b) == desc) { keys[i] = b; keys[p] = a; }
            }
        }
    }
    __syncthreads();
}

// Round 0: keys from the marginals.  grid = (chunks, B).  Writes the KP best keys of each chunk.
__global__ __launch_bounds__(256) void topk_chunks(const float *marg, int V, int KP, unsigned long long *out)
{
    __shared__ unsigned long long keys[CHUNK];
    const int tid = threadIdx.x, chunk = blockIdx.x, row = blockIdx.y;
    const float *src = marg + (size_t)row * V;
    for (int e = tid; e < CHUNK; e += 256) {
        int v = chunk * CHUNK + e;
        keys[e] = v < V ? make_key(src[v], (uint32_t)v) : 0ull;
    }
    bitonic_desc(keys, tid);
    unsigned long long *dst = out + ((size_t)row * gridDim.x + chunk) * KP;
    for (int e = tid; e < KP; e += 256) dst[e] = keys[e];
}

// Later rounds: merge CHUNK/KP lists of KP keys into one.  grid = (groups, B).
__global__ __launch_bounds__(256) void topk_merge(const unsigned long long *in, int lists, int KP,
                                                  unsigned long long *out)
{
    __shared__ unsigned long long keys[CHUNK];
    const int tid = threadIdx.x, grp = blockIdx.x, row = blockIdx.y;
    const int per = CHUNK / KP;
    const int first = grp * per, cnt = min(per, lists - first);
    const unsigned long long *src = in + ((size_t)row * lists + first) * KP;
    for (int e = tid; e < CHUNK; e += 256) keys[e] = e < cnt * KP ? src[e] : 0ull;
    bitonic_desc(keys, tid);
    unsigned long long *dst = out + ((size_t)row * gridDim.x + grp) * KP;
    for (int e = tid; e < KP; e += 256) dst[e] = keys[e];
}

// ------------------------------------------------------------------------------------------------
// Expansion: one wavefront.  top[k*KP + r] = key of rank r at position k (0 where V < KP).
// ------------------------------------------------------------------------------------------------
struct Cand {
    float rho;
    int depth, parent, rank;
    uint32_t path[4];         // rank bytes, first rank in the most significant byte of path[0]
};

__device__ __forceinline__ bool cand_before(const Cand &a, const Cand &b)
{
    if (a.rho != b.rho) return a.rho > b.rho;
    if (a.depth != b.depth) return a.depth < b.depth;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        if (a.path[w] != b.path[w]) return a.path[w] < b.path[w];
    return false;
}

__device__ __forceinline__ Cand shfl_cand(const Cand &c, int src)
{
    Cand r;
    r.rho = __shfl(c.rho, src); r.depth = __shfl(c.depth, src); r.parent = __shfl(c.parent, src);
    r.rank = __shfl(c.rank, src);
#pragma unroll
    for (int w = 0; w < 4; ++w) r.path[w] = __shfl(c.path[w], src);
    return r;
}

__global__ __launch_bounds__(64) void bestfirst_expand(const unsigned long long *top, int B, int K, int KP, int N,
                                                       int32_t *parent, int32_t *token, int32_t *depth, float *rho,
                                                       int32_t *n_out, float *ahat)
{
    constexpr int CAP = BTV_MAX_NODES + 2;
    __shared__ float f_rho[CAP];
    __shared__ int f_meta[CAP];                   // depth | rank << 8 | (parent + 1) << 16
    __shared__ uint32_t f_path[CAP][4];
    __shared__ float n_rho[BTV_MAX_NODES];
    const int lane = threadIdx.x;
    int nf = 0, n = 0;
    float a = 1.0f;
    auto topq = [&](int k, int r) { return __uint_as_float((uint32_t)(top[(size_t)k * KP + r] >> 32)); };
    auto topid = [&](int k, int r) { return (int32_t)(0xFFFFFFFFu - (uint32_t)(top[(size_t)k * KP + r])); };
    if (lane == 0) {
        f_rho[0] = __fmul_rn(1.0f, topq(0, 0));
        f_meta[0] = 1;
        f_path[0][0] = f_path[0][1] = f_path[0][2] = f_path[0][3] = 0u;
    }
    nf = 1;
    __syncthreads();
    while (n < N && nf > 0) {
        // lane-local best over entries lane, lane+64, ...
        Cand best; int bj = -1;
        best.rho = -1.f; best.depth = 0; best.parent = 0; best.rank = 0;
        best.path[0] = best.path[1] = best.path[2] = best.path[3] = 0u;
        for (int j = lane; j < nf; j += 64) {
            Cand cnd;
            cnd.rho = f_rho[j];
            int mt = f_meta[j];
            cnd.depth = mt & 0xFF; cnd.rank = (mt >> 8) & 0xFF; cnd.parent = (mt >> 16) - 1;
#pragma unroll
            for (int w = 0; w < 4; ++w) cnd.path[w] = f_path[j][w];
            if (bj < 0 || cand_before(cnd, best)) { best = cnd; bj = j; }
        }
        // wave-wide best (lanes without an entry carry bj = -1)
        for (int off = 32; off >= 1; off >>= 1) {
            Cand o = shfl_cand(best, lane ^ off);
            int oj = __shfl(bj, lane ^ off);
            if (oj >= 0 && (bj < 0 || cand_before(o, best))) { best = o; bj = oj; }
        }
        // every lane now holds the same (best, bj)
        const Cand u = best;
        if (lane == 0) {
            parent[n] = u.parent; token[n] = topid(u.depth - 1, u.rank);
            if (depth) depth[n] = u.depth;
            if (rho) rho[n] = u.rho;
            n_rho[n] = u.rho;
            // remove by moving the last entry into the hole
            int last = nf - 1;
            if (bj != last) {
                f_rho[bj] = f_rho[last]; f_meta[bj] = f_meta[last];
#pragma unroll
                for (int w = 0; w < 4; ++w) f_path[bj][w] = f_path[last][w];
            }
        }
        a += u.rho;
        nf -= 1;
        __syncthreads();
        if (lane == 0) {
            int k = nf;
            if (u.depth < B) {                                    // best child of u
                f_rho[k] = __fmul_rn(u.rho, topq(u.depth, 0));
                f_meta[k] = (u.depth + 1) | (0 << 8) | ((n + 1) << 16);
#pragma unroll
                for (int w = 0; w < 4; ++w) f_path[k][w] = u.path[w];
                ++k;
            }
            if (u.rank + 1 < K) {                                 // next sibling of u
                float prho = u.parent < 0 ? 1.0f : n_rho[u.parent];
                f_rho[k] = __fmul_rn(prho, topq(u.depth - 1, u.rank + 1));
                f_meta[k] = u.depth | ((u.rank + 1) << 8) | ((u.parent + 1) << 16);
                int pos = u.depth - 1, wd = pos >> 2, sh = 24 - 8 * (pos & 3);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t pw = u.path[w];
                    if (w == wd) pw = (pw & ~(0xFFu << sh)) | ((uint32_t)(u.rank + 1) << sh);
                    f_path[k][w] = pw;
                }
                ++k;
            }
        }
        nf += (u.depth < B ? 1 : 0) + (u.rank + 1 < K ? 1 : 0);
        ++n;
        __syncthreads();
    }
    if (lane == 0) {
        *n_out = n;
        if (ahat) *ahat = a;
    }
}

int next_pow2(int x) { int p = 1; while (p < x) p <<= 1; return p; }

struct TopkPlan { int K, KP, chunks; size_t buf_keys; };

TopkPlan topk_plan(int B, int V, int N)
{
    TopkPlan t;
    t.K = std::min(V, N);
    t.KP = std::max(next_pow2(t.K), 1);
    t.chunks = (V + CHUNK - 1) / CHUNK;
    t.buf_keys = (size_t)B * t.chunks * t.KP;
    return t;
}

}  // namespace

extern "C" {

size_t btv_tree_build_workspace(int B, int V, int N)
{
    if (B < 1 || B > MAXB || V < 1 || N < 1 || N > BTV_MAX_NODES) return 0;
    TopkPlan t = topk_plan(B, V, N);
    return BTV_WS_HEADER + 2 * btv_align_up(t.buf_keys * 8, BTV_WS_ALIGN);
}

int btv_tree_build(const float *marginals, int B, int V, int N, int32_t *parent, int32_t *token, int32_t *depth,
                   float *rho, int32_t *n_out, float *ahat, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(marginals && parent && token && n_out, "null pointer");
    BTV_REQUIRE(B >= 1 && B <= MAXB, "B=%d outside [1,%d]", B, MAXB);
    BTV_REQUIRE(V >= 1, "V=%d", V);
    BTV_REQUIRE(N >= 1 && N <= BTV_MAX_NODES, "N=%d outside [1,%d]", N, BTV_MAX_NODES);
    int rc = btv_check_ws(ws, ws_bytes, btv_tree_build_workspace(B, V, N));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TopkPlan t = topk_plan(B, V, N);
    size_t half = btv_align_up(t.buf_keys * 8, BTV_WS_ALIGN);
    unsigned long long *bufA = reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    unsigned long long *bufB = reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER + half);
    hipLaunchKernelGGL(topk_chunks, dim3(t.chunks, B), dim3(256), 0, st, marginals, V, t.KP, bufA);
    BTV_HIP(hipGetLastError());
    int lists = t.chunks;
    const int per = CHUNK / t.KP;
    while (lists > 1) {
        int groups = (lists + per - 1) / per;
        hipLaunchKernelGGL(topk_merge, dim3(groups, B), dim3(256), 0, st, bufA, lists, t.KP, bufB);
        BTV_HIP(hipGetLastError());
        std::swap(bufA, bufB);
        lists = groups;
    }
    hipLaunchKernelGGL(bestfirst_expand, dim3(1), dim3(64), 0, st, bufA, B, t.K, t.KP, N, parent, token, depth, rho,
                       n_out, ahat);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

}  // extern "C"
