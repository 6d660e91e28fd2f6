// Best-first draft-tree construction on the GPU (gfx950).
//
// Sec. 3.3 / Prop. 3.3 / Algorithm 1's frontier rule at a fixed budget N: repeatedly emit the
// frontier prefix with the largest path score rho (Eq. 1), then push its best child and its next
// sibling.  Two steps:
//   1. per-position exact top-K of the marginals (K = min(V, N): a rank-j token is preceded by its
//      j earlier siblings, so ranks >= N can never be emitted), ordered (probability desc, id asc).
//      Keys are 64-bit  prob_bits << 32 | ~id  (probabilities are non-negative, so the bit pattern
//      orders like the value).  Every workgroup selects the K best of 2048 keys: LDS histogram of a
//      12-bit digit, the digit of the K-th key, compaction, and a bitonic sort of the few survivors
//      (exchanges in registers, by DPP / lane-permute instructions, and through LDS only across
//      waves); rounds of the same kernel then merge the per-chunk winners.
//   2. the expansion itself: one wavefront, the top lists and the frontier in LDS, a wave-wide
//      arg-best per emitted node.
// rho(child) = rho(parent) * q is one fp32 multiply (never fused), the root has rho = 1.
// Frontier order: rho desc, depth asc, rank path lexicographic asc (ranks < 256 pack into 16 bytes).
#include "btv_common.h"

#include <algorithm>

namespace {

typedef unsigned long long u64;

constexpr int CHUNK = 2048;      // keys merged per workgroup in the later rounds (256 threads x 8)
constexpr int CHUNK0 = 4096;     // marginals scanned per workgroup in round 0 (256 threads x 16)
constexpr int MAXB = BTV_MAX_DEPTH;
constexpr int BINS = 4096;       // selection histogram: 12 bits below the sign bit of the probability

__device__ __forceinline__ u64 make_key(float prob, uint32_t id)
{
    uint32_t b = __float_as_uint(prob);
    if (b == 0x80000000u) b = 0u;                  // -0.0 sorts as 0
    return ((u64)b << 32) | (u64)(0xFFFFFFFFu - id);
}

__device__ __forceinline__ int key_bin(u64 key) { return (int)((key >> 51) & (BINS - 1)); }   // float bits [30:19]

// value of lane (lane ^ MASK), by DPP / lane-permute instructions only (no LDS traffic)
template <int MASK>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int lane)
{
    if constexpr (MASK == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false);
    else if constexpr (MASK == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false);
    else if constexpr (MASK == 4) {
        const uint32_t up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x104, 0xF, 0xF, false);   // lane + 4
        const uint32_t dn = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, false);   // lane - 4
        return (lane & 4) ? dn : up;
    } else if constexpr (MASK == 8) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xF, 0xF, false);
    else if constexpr (MASK == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16) ? r[0] : r[1];
    } else {
        static_assert(MASK == 32, "lane mask");
        auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        return (lane & 32) ? r[0] : r[1];
    }
}

template <int MASK>
__device__ __forceinline__ u64 lane_xor64(u64 x, int lane)
{
    return ((u64)lane_xor<MASK>((uint32_t)(x >> 32), lane) << 32) | lane_xor<MASK>((uint32_t)x, lane);
}

template <int EPT, int J>
__device__ __forceinline__ void inthread_step(u64 (&x)[EPT], int tid, int k)
{
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int p = i ^ J;
        if (p > i) {
            const bool desc = (((tid * EPT + i) & k) == 0);
            const u64 a = x[i], b = x[p];
            const bool sw = (a < b) == desc;
            x[i] = sw ? b : a;
            x[p] = sw ? a : b;
        }
    }
}

template <int EPT, int TJ>
__device__ __forceinline__ void wave_step(u64 (&x)[EPT], int tid, bool keep_max)
{
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const u64 o = lane_xor64<TJ>(x[i], tid & 63);
        x[i] = ((x[i] < o) == keep_max) ? o : x[i];      // keys are distinct (or both padding)
    }
}

// Descending bitonic sort of 256*EPT keys by 256 threads; thread t holds elements EPT*t .. EPT*t+EPT-1 in x[].
// `lds` has room for 256*EPT keys.
template <int EPT>
__device__ __forceinline__ void sort_desc(u64 (&x)[EPT], u64 *lds, int tid)
{
    constexpr int NKEYS = 256 * EPT;
#pragma unroll 1
    for (int k = 2; k <= NKEYS; k <<= 1) {
#pragma unroll 1
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j < EPT) {
                // both elements live in this thread
                if (EPT > 8 && j == 8) inthread_step<EPT, 8>(x, tid, k);
                else if (EPT > 4 && j == 4) inthread_step<EPT, 4>(x, tid, k);
                else if (EPT > 2 && j == 2) inthread_step<EPT, 2>(x, tid, k);
                else inthread_step<EPT, 1>(x, tid, k);
            } else {
                const int tj = j / EPT;                                   // partner thread = tid ^ tj
                const bool lower = (tid & tj) == 0;
                const bool desc = ((tid * EPT) & k) == 0;                 // same for all elements of the thread here
                const bool keep_max = lower == desc;
                if (tj == 1) wave_step<EPT, 1>(x, tid, keep_max);
                else if (tj == 2) wave_step<EPT, 2>(x, tid, keep_max);
                else if (tj == 4) wave_step<EPT, 4>(x, tid, keep_max);
                else if (tj == 8) wave_step<EPT, 8>(x, tid, keep_max);
                else if (tj == 16) wave_step<EPT, 16>(x, tid, keep_max);
                else if (tj == 32) wave_step<EPT, 32>(x, tid, keep_max);
                else {
                    __syncthreads();
#pragma unroll
                    for (int i = 0; i < EPT; ++i) lds[i * 256 + tid] = x[i];      // element-major: conflict-free
                    __syncthreads();
#pragma unroll
                    for (int i = 0; i < EPT; ++i) {
                        const u64 o = lds[i * 256 + (tid ^ tj)];
                        x[i] = ((x[i] < o) == keep_max) ? o : x[i];
                    }
                }
            }
        }
    }
}

// One workgroup selects, in order, the KP largest of up to 256*EPT keys (EPT per thread, 0 = padding):
// histogram of a 12-bit digit -> the digit of the KP-th largest key -> compaction of the keys at or above that
// digit -> a bitonic sort of just those (512 slots when they fit, else all 256*EPT, which always fits).
// Round 0 (EPT = 16, from marginals): keys come from chunk `blockIdx.x` of row `blockIdx.y` of the marginals.
// Later rounds (EPT = 8): the keys are `per` lists of KP winners of the previous round.
template <int EPT, bool FROM_MARGINALS>
__global__ __launch_bounds__(256) void topk_round(const float *marg, int V, const u64 *in, int lists, int KP, u64 *out)
{
    constexpr int NKEYS = 256 * EPT;
    __shared__ u64 lds[NKEYS];            // candidates, then sort exchange buffer
    __shared__ int hist[BINS];
    __shared__ int wsum[4];
    __shared__ int sel_bin, ncand;
    const int tid = threadIdx.x, grp = blockIdx.x, row = blockIdx.y, lane = tid & 63, w = tid >> 6;
    u64 x[EPT];
    if (FROM_MARGINALS) {
        const float *src = marg + (size_t)row * V;
        const bool aligned = (((size_t)row * V) & 3) == 0 && (reinterpret_cast<uintptr_t>(marg) & 15) == 0;
#pragma unroll
        for (int q4 = 0; q4 < EPT / 4; ++q4) {
            const int v0 = grp * NKEYS + q4 * 1024 + tid * 4;        // coalesced: a wave reads 1 KiB per load
            if (aligned && v0 + 4 <= V) {
                const float4 a = *reinterpret_cast<const float4 *>(src + v0);
                x[q4 * 4 + 0] = make_key(a.x, v0); x[q4 * 4 + 1] = make_key(a.y, v0 + 1);
                x[q4 * 4 + 2] = make_key(a.z, v0 + 2); x[q4 * 4 + 3] = make_key(a.w, v0 + 3);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) x[q4 * 4 + i] = v0 + i < V ? make_key(src[v0 + i], (uint32_t)(v0 + i)) : 0ull;
            }
        }
    } else {
        const int per = NKEYS / KP;
        const int first = grp * per, cnt = min(per, lists - first);
        const u64 *src = in + ((size_t)row * lists + first) * KP;
#pragma unroll
        for (int i = 0; i < EPT; ++i) x[i] = i * 256 + tid < cnt * KP ? src[i * 256 + tid] : 0ull;
    }
    // ---- histogram of the digit ------------------------------------------------------------------------
    for (int b = tid; b < BINS; b += 256) hist[b] = 0;
    if (tid == 0) { ncand = 0; sel_bin = 0; }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < EPT; ++i) atomicAdd(&hist[key_bin(x[i])], 1);
    __syncthreads();
    // ---- digit of the KP-th largest key: thread t owns bins 16t .. 16t+15; suffix sums over threads ----------
    int own = 0;
#pragma unroll
    for (int b = 0; b < 16; ++b) own += hist[tid * 16 + b];
    int suf = own;                         // inclusive suffix sum within the wave (over higher lanes)
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_down(suf, off);
        if (lane + off < 64) suf += o;
    }
    if (lane == 0) wsum[w] = suf;
    __syncthreads();
    int above = suf - own;                 // keys in bins owned by higher threads
    for (int ww = w + 1; ww < 4; ++ww) above += wsum[ww];
    if (above < KP && above + own >= KP) {
        int cum = above;
        for (int b = 15; b >= 0; --b) {
            const int hb = hist[tid * 16 + b];
            if (cum + hb >= KP) { sel_bin = tid * 16 + b; break; }
            cum += hb;
        }
    }
    __syncthreads();
    // ---- compaction of the keys at or above that digit -----------------------------------------------------
    const int tb = sel_bin;
#pragma unroll
    for (int i = 0; i < EPT; ++i)
        if (key_bin(x[i]) >= tb) lds[atomicAdd(&ncand, 1)] = x[i];
    __syncthreads();
    const int nc = ncand;
    u64 *dst = out + ((size_t)row * gridDim.x + grp) * KP;
    if (nc <= 512) {
        u64 y[2];
        y[0] = 2 * tid < nc ? lds[2 * tid] : 0ull;
        y[1] = 2 * tid + 1 < nc ? lds[2 * tid + 1] : 0ull;
        __syncthreads();
        sort_desc<2>(y, lds, tid);
        if (2 * tid < KP) dst[2 * tid] = y[0];
        if (2 * tid + 1 < KP) dst[2 * tid + 1] = y[1];
    } else {
#pragma unroll
        for (int i = 0; i < EPT; ++i) x[i] = tid * EPT + i < nc ? lds[tid * EPT + i] : 0ull;
        __syncthreads();
        sort_desc<EPT>(x, lds, tid);
#pragma unroll
        for (int i = 0; i < EPT; ++i)
            if (tid * EPT + i < KP) dst[tid * EPT + i] = x[i];
    }
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

__global__ __launch_bounds__(64) void bestfirst_expand(const u64 *top, int B, int K, int KP, int N, int32_t *parent,
                                                       int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat)
{
    constexpr int CAP = BTV_MAX_NODES + 2;
    __shared__ float q_s[MAXB * BTV_MAX_NODES];   // probability of rank r at position k: q_s[k*KP + r]
    __shared__ float f_rho[CAP];
    __shared__ int f_meta[CAP];                   // depth | rank << 8 | (parent + 1) << 16
    __shared__ uint32_t f_path[CAP][4];
    __shared__ float n_rho[BTV_MAX_NODES];
    __shared__ int n_meta[BTV_MAX_NODES];         // (depth - 1) * KP + rank of emitted node: index of its token in `top`
    __shared__ int n_parent[BTV_MAX_NODES], n_depth[BTV_MAX_NODES];   // outputs are staged: no global store in the loop
    const int lane = threadIdx.x;
    for (int e = lane; e < B * KP; e += 64) q_s[e] = __uint_as_float((uint32_t)(top[e] >> 32));
    if (lane == 0) {
        f_meta[0] = 1;
        f_path[0][0] = f_path[0][1] = f_path[0][2] = f_path[0][3] = 0u;
    }
    __syncthreads();
    if (lane == 0) f_rho[0] = __fmul_rn(1.0f, q_s[0]);
    __syncthreads();
    int nf = 1, n = 0;
    float a = 1.0f;
    while (n < N && nf > 0) {
        // lane-local best over entries lane, lane+64, ...
        Cand best; int bj = -1;
        best.rho = -1.f; best.depth = 0; best.parent = 0; best.rank = 0;
        best.path[0] = best.path[1] = best.path[2] = best.path[3] = 0u;
        for (int j = lane; j < nf; j += 64) {
            Cand cnd;
            cnd.rho = f_rho[j];
            const int mt = f_meta[j];
            cnd.depth = mt & 0xFF; cnd.rank = (mt >> 8) & 0xFF; cnd.parent = (mt >> 16) - 1;
#pragma unroll
            for (int w = 0; w < 4; ++w) cnd.path[w] = f_path[j][w];
            if (bj < 0 || cand_before(cnd, best)) { best = cnd; bj = j; }
        }
        // wave-wide best.  Primary key (rho desc, depth asc) as one 64-bit maximum; the rank path only decides
        // when several lanes tie on it, which is rare.
        const u64 pk = bj < 0 ? 0ull : (((u64)__float_as_uint(best.rho) << 32) | (u64)(0x100 - best.depth) << 8 | 1ull);
        u64 mx = pk;
        { u64 o;
          o = lane_xor64<1>(mx, lane); mx = o > mx ? o : mx;   o = lane_xor64<2>(mx, lane); mx = o > mx ? o : mx;
          o = lane_xor64<4>(mx, lane); mx = o > mx ? o : mx;   o = lane_xor64<8>(mx, lane); mx = o > mx ? o : mx;
          o = lane_xor64<16>(mx, lane); mx = o > mx ? o : mx;  o = lane_xor64<32>(mx, lane); mx = o > mx ? o : mx; }
        const u64 tied = __builtin_amdgcn_ballot_w64(pk == mx);
        int src = __builtin_ctzll(tied);
        if (__builtin_popcountll(tied) > 1) {
            // lexicographic minimum of the rank paths among the tied lanes, word by word
            u64 alive = tied;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t v = ((alive >> lane) & 1ull) ? best.path[w] : 0xFFFFFFFFu;
                uint32_t mn = v;
                for (int off = 32; off >= 1; off >>= 1) { const uint32_t o = __shfl_xor(mn, off); mn = o < mn ? o : mn; }
                alive &= __builtin_amdgcn_ballot_w64(v == mn && ((alive >> lane) & 1ull));
            }
            src = __builtin_ctzll(alive);
        }
        Cand u;    // broadcast of lane `src` (wave-uniform index: scalar lane reads)
        u.rho = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(best.rho), src));
        u.depth = __builtin_amdgcn_readlane(best.depth, src); u.parent = __builtin_amdgcn_readlane(best.parent, src);
        u.rank = __builtin_amdgcn_readlane(best.rank, src);
#pragma unroll
        for (int w = 0; w < 4; ++w) u.path[w] = __builtin_amdgcn_readlane(best.path[w], src);
        bj = __builtin_amdgcn_readlane(bj, src);
        const bool has_child = u.depth < B, has_sib = u.rank + 1 < K;
        if (lane == 0) {
            n_rho[n] = u.rho;
            n_meta[n] = (u.depth - 1) * KP + u.rank;
            n_parent[n] = u.parent;
            n_depth[n] = u.depth;
            // the emitted entry's slot takes the child (or the sibling, or the last entry)
            int slot = bj;
            if (has_child) {
                f_rho[slot] = __fmul_rn(u.rho, q_s[u.depth * KP]);
                f_meta[slot] = (u.depth + 1) | (0 << 8) | ((n + 1) << 16);
                // path unchanged: the child's own rank byte is 0
                slot = nf;
            }
            if (has_sib) {
                const float prho = u.parent < 0 ? 1.0f : n_rho[u.parent];
                f_rho[slot] = __fmul_rn(prho, q_s[(u.depth - 1) * KP + u.rank + 1]);
                f_meta[slot] = u.depth | ((u.rank + 1) << 8) | ((u.parent + 1) << 16);
                const int pos = u.depth - 1, wd = pos >> 2, sh = 24 - 8 * (pos & 3);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t pw = u.path[w];
                    if (w == wd) pw = (pw & ~(0xFFu << sh)) | ((uint32_t)(u.rank + 1) << sh);
                    f_path[slot][w] = pw;
                }
            }
            if (!has_child && !has_sib && bj != nf - 1) {
                f_rho[bj] = f_rho[nf - 1]; f_meta[bj] = f_meta[nf - 1];
#pragma unroll
                for (int w = 0; w < 4; ++w) f_path[bj][w] = f_path[nf - 1][w];
            }
        }
        a += u.rho;
        nf += (has_child ? 1 : 0) + (has_sib ? 1 : 0) - 1;
        ++n;
        __syncthreads();
    }
    // token ids of the emitted nodes, read from the top lists in parallel
    for (int i = lane; i < n; i += 64) {
        token[i] = (int32_t)(0xFFFFFFFFu - (uint32_t)top[n_meta[i]]);
        parent[i] = n_parent[i];
        if (depth) depth[i] = n_depth[i];
        if (rho) rho[i] = n_rho[i];
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
    t.chunks = (V + CHUNK0 - 1) / CHUNK0;
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
    u64 *bufA = reinterpret_cast<u64 *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    u64 *bufB = reinterpret_cast<u64 *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER + half);
    hipLaunchKernelGGL((topk_round<16, true>), dim3(t.chunks, B), dim3(256), 0, st, marginals, V, nullptr, 0, t.KP, bufA);
    BTV_HIP(hipGetLastError());
    int lists = t.chunks;
    const int per = CHUNK / t.KP;
    while (lists > 1) {
        int groups = (lists + per - 1) / per;
        hipLaunchKernelGGL((topk_round<8, false>), dim3(groups, B), dim3(256), 0, st, nullptr, 0, bufA, lists, t.KP, bufB);
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
