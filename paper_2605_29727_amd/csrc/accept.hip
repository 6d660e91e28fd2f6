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
// LM head fused with the argmax (App. E: 2*s*h*V FLOPs and s*V activation elements for the logits;
// App. C "Acceptance": only their top-1 is used).  logit[r, v] = sum_k H[r, k] W[v, k] is formed on the
// matrix cores and reduced to one (value, token) pair per row and workgroup: the logits never reach
// memory, the 2*V*h bytes of W are streamed once.
//
// Transposed product, C^T = W_tile * H^T (v_mfma_f32_32x32x16_bf16): a wave owns 32 vocabulary rows
// and every row of H, so a lane's accumulator registers run over vocabulary rows of one H row and
// the argmax is a per-lane scan.  The operand layout wants lane l to hold row l % 32, which as a
// direct load would touch 64 cache lines per instruction and use 16 bytes of each; instead every
// load instruction fetches four whole 256-byte row segments (16 lanes per row), and the block is
// turned round through a wave-private LDS tile.  H blocks [rows, KB] are shared by the waves through
// a double-buffered LDS slab.  All tiles store the 16-byte chunks of a row XOR-permuted by the row
// number, so operand reads (ds_read_b128, 16 lanes = 16 different rows) are conflict-free.
// ------------------------------------------------------------------------------------------------
typedef __bf16 lm_bf16x8 __attribute__((ext_vector_type(8)));
typedef float lm_f32x16 __attribute__((ext_vector_type(16)));

template <int RT, int WAVES, int KB>
struct LmShape {
    static constexpr int THREADS = WAVES * 64, ROWS = RT * 32;
    static constexpr int RB = KB * 2;                     // bytes of a tile row
    static constexpr int CPR = RB / 16;                   // 16-byte chunks per row
    static constexpr int WTILE = 32 * RB, SLAB = ROWS * RB;
    static constexpr int LDS_BYTES = WAVES * WTILE + 2 * SLAB;
    static constexpr int WLD = 32 * CPR / 64;             // load instructions per wave and block for W
    static constexpr int HLD = (ROWS * CPR + THREADS - 1) / THREADS;   // chunks of the H slab per thread and block
    static constexpr bool HEVEN = ROWS * CPR % THREADS == 0;
    static_assert(CPR == 8 || CPR == 16, "KB is 64 or 128");
    // byte offset of 16-byte chunk `col` of tile row `row`: 16 lanes reading one chunk index of 16 consecutive
    // rows must land in 16 different 16-byte bank groups of the 256-byte bank line
    __device__ static constexpr int at(int row, int col)
    {
        return row * RB + ((col ^ (CPR == 16 ? (row & 15) : ((row >> 1) & 7))) << 4);
    }
};

template <int RT, int WAVES, int KB>
__global__ __launch_bounds__(WAVES * 64) void lm_head_argmax(const uint16_t *__restrict__ H,
                                                              const uint16_t *__restrict__ W, int R, int h, int V,
                                                              Best *__restrict__ part)
{
    using S = LmShape<RT, WAVES, KB>;
    extern __shared__ __align__(16) unsigned char lm_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r32 = lane & 31, half = lane >> 5;
    const int v0 = (blockIdx.x * WAVES + wave) * 32;
    unsigned char *wtile = lm_lds + wave * S::WTILE;
    unsigned char *slab = lm_lds + WAVES * S::WTILE;
    const int nkb = h / KB;

    // W: instruction i moves rows i*(64/CPR) .. of the wave's tile, CPR lanes per row
    constexpr int RPI = 64 / S::CPR;                       // rows per load instruction
    const int wcol = lane % S::CPR, wrow0 = lane / S::CPR;
    const uint4 *wp[S::WLD];
    int wdst[S::WLD];
#pragma unroll
    for (int i = 0; i < S::WLD; ++i) {
        const int row = i * RPI + wrow0;
        wp[i] = reinterpret_cast<const uint4 *>(W + (size_t)min(v0 + row, V - 1) * h + wcol * 8);
        wdst[i] = S::at(row, wcol);
    }
    // H: chunk c of the slab -> row c / CPR, column c % CPR
    const uint4 *hp[S::HLD];
    int hdst[S::HLD];
#pragma unroll
    for (int i = 0; i < S::HLD; ++i) {
        const int c = tid + i * S::THREADS, row = c / S::CPR, col = c % S::CPR;
        hp[i] = reinterpret_cast<const uint4 *>(H + (size_t)min(row, R - 1) * h + col * 8);
        hdst[i] = S::at(row, col);
        if (!S::HEVEN && row >= S::ROWS) hdst[i] = -1;    // past the slab: fetched (row clamped), never stored
    }
    // operand reads: step j of a block uses chunk 2j + half of row r32 (same chunk on both sides)
    int osrc[KB / 16];
#pragma unroll
    for (int j = 0; j < KB / 16; ++j) osrc[j] = S::at(r32, 2 * j + half);

    lm_f32x16 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[rt][e] = 0.f;

    // Workgroups start at different blocks of the contraction and wrap round: rows of W are a multiple of 4 KB
    // apart, so workgroups marching in step would all hit the same few memory channels.
    int cur = (blockIdx.x * 5) % nkb;
    uint4 wn[S::WLD], hn[S::HLD];
#pragma unroll
    for (int i = 0; i < S::HLD; ++i) hn[i] = hp[i][cur * (KB / 8)];
#pragma unroll
    for (int i = 0; i < S::WLD; ++i) wn[i] = wp[i][cur * (KB / 8)];
#pragma unroll
    for (int i = 0; i < S::HLD; ++i)
        if (S::HEVEN || hdst[i] >= 0) *reinterpret_cast<uint4 *>(slab + hdst[i]) = hn[i];
#pragma unroll
    for (int i = 0; i < S::WLD; ++i) *reinterpret_cast<uint4 *>(wtile + wdst[i]) = wn[i];
    __syncthreads();

    for (int kb = 0; kb < nkb; ++kb) {
        // next block into registers (the last round fetches the first block again; it lands where nobody reads)
        cur = cur + 1 == nkb ? 0 : cur + 1;
        const int nb = cur * (KB / 8);
#pragma unroll
        for (int i = 0; i < S::HLD; ++i) hn[i] = hp[i][nb];
#pragma unroll
        for (int i = 0; i < S::WLD; ++i) wn[i] = wp[i][nb];
        const unsigned char *buf = slab + (kb & 1) * S::SLAB;
#pragma unroll
        for (int j = 0; j < KB / 16; ++j) {
            const uint4 a = *reinterpret_cast<const uint4 *>(wtile + osrc[j]);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const uint4 b = *reinterpret_cast<const uint4 *>(buf + rt * 32 * S::RB + osrc[j]);
                acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(lm_bf16x8, a),
                                                                  __builtin_bit_cast(lm_bf16x8, b), acc[rt], 0, 0, 0);
            }
        }
        // the wave's own W tile has been consumed (its reads precede these writes in program order); the H slab
        // written is the one nobody reads in this round
        unsigned char *nxt = slab + ((kb + 1) & 1) * S::SLAB;
#pragma unroll
        for (int i = 0; i < S::HLD; ++i)
            if (S::HEVEN || hdst[i] >= 0) *reinterpret_cast<uint4 *>(nxt + hdst[i]) = hn[i];
#pragma unroll
        for (int i = 0; i < S::WLD; ++i) *reinterpret_cast<uint4 *>(wtile + wdst[i]) = wn[i];
        __syncthreads();
    }

    // per-lane scan over the 16 vocabulary rows it holds (ascending), other half, then the waves
    Best *wb = reinterpret_cast<Best *>(lm_lds);            // [WAVES][ROWS]
    static_assert(S::LDS_BYTES >= WAVES * S::ROWS * (int)sizeof(Best), "exchange area must fit");
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        Best b = { -INFINITY, INT_MAX };
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int v = v0 + (e >> 2) * 8 + half * 4 + (e & 3);
            if (v < V) best_take(b, acc[rt][e], v);
        }
        const float ov = __shfl_xor(b.v, 32);
        const int oi = __shfl_xor(b.i, 32);
        best_take(b, ov, oi);
        if (half == 0) wb[wave * S::ROWS + rt * 32 + r32] = b;
    }
    __syncthreads();
    for (int row = tid; row < R; row += S::THREADS) {
        Best b = wb[row];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) best_take(b, wb[w * S::ROWS + row].v, wb[w * S::ROWS + row].i);
        part[(size_t)row * gridDim.x + blockIdx.x] = b;
    }
}

// grid = rows: best of a row's per-workgroup partials -> out[row]
__global__ __launch_bounds__(256) void argmax_merge(const Best *part, int chunks, Best *out)
{
    __shared__ Best wb[4];
    const int tid = threadIdx.x, row = blockIdx.x;
    Best b = { -INFINITY, INT_MAX };
    for (int c = tid; c < chunks; c += 256) best_take(b, part[(size_t)row * chunks + c].v, part[(size_t)row * chunks + c].i);
    b = best_wave(b);
    if ((tid & 63) == 0) wb[tid >> 6] = b;
    __syncthreads();
    if (tid == 0) {
        Best r = wb[0];
        best_take(r, wb[1].v, wb[1].i); best_take(r, wb[2].v, wb[2].i); best_take(r, wb[3].v, wb[3].i);
        out[row] = r;
    }
}

template <int RT, int WAVES, int KB>
int lm_head_launch(const uint16_t *H, const uint16_t *W, int R, int h, int V, Best *part, hipStream_t st)
{
    using S = LmShape<RT, WAVES, KB>;
    static bool configured = false;
    auto kern = lm_head_argmax<RT, WAVES, KB>;
    if (!configured) {
        BTV_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    S::LDS_BYTES));
        configured = true;
    }
    const int chunks = (V + WAVES * 32 - 1) / (WAVES * 32);
    hipLaunchKernelGGL(kern, dim3(chunks), dim3(WAVES * 64), S::LDS_BYTES, st, H, W, R, h, V, part);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

// Shapes: up to 96 rows two workgroups of four waves share a CU (80 KB of LDS each); above that one workgroup of
// eight waves, with half-length blocks from 224 rows on so that the slabs still fit.
inline int lm_waves(int R) { return R <= 96 ? 4 : 8; }
inline int lm_chunks(int R, int V) { return (V + lm_waves(R) * 32 - 1) / (lm_waves(R) * 32); }

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

size_t btv_tree_accept_lm_head_workspace(int M, int V)
{
    if (M < 1 || M > BTV_MAX_NODES || V < 1) return 0;
    const size_t rows = (size_t)M + 1;
    return BTV_WS_HEADER + btv_align_up(rows * lm_chunks(M + 1, V) * sizeof(Best), BTV_WS_ALIGN) +
           btv_align_up(rows * sizeof(Best), BTV_WS_ALIGN);
}

int btv_tree_accept_greedy_lm_head(const void *hidden, const void *W, int h, const int32_t *parent, const int32_t *token,
                                   int M, int V, int32_t *path, int32_t *n_acc, int32_t *bonus, int32_t *argmax_out,
                                   void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(hidden && W && parent && token && path && n_acc && bonus, "null pointer");
    BTV_REQUIRE(M >= 1 && M <= BTV_MAX_NODES, "M=%d outside [1,%d]", M, BTV_MAX_NODES);
    BTV_REQUIRE(V >= 1, "V=%d", V);
    BTV_REQUIRE(h >= 128 && h % 128 == 0, "h=%d must be a positive multiple of 128", h);
    BTV_REQUIRE((reinterpret_cast<uintptr_t>(hidden) & 15) == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0,
                "hidden and W must be 16-byte aligned");
    int rc = btv_check_ws(ws, ws_bytes, btv_tree_accept_lm_head_workspace(M, V));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int R = M + 1, chunks = lm_chunks(R, V);
    Best *part = reinterpret_cast<Best *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    Best *best = reinterpret_cast<Best *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER +
                                          btv_align_up((size_t)R * chunks * sizeof(Best), BTV_WS_ALIGN));
    const uint16_t *Hp = static_cast<const uint16_t *>(hidden), *Wp = static_cast<const uint16_t *>(W);
    switch ((R + 31) / 32) {
    case 1: rc = lm_head_launch<1, 4, 128>(Hp, Wp, R, h, V, part, st); break;
    case 2: rc = lm_head_launch<2, 4, 128>(Hp, Wp, R, h, V, part, st); break;
    case 3: rc = lm_head_launch<3, 4, 128>(Hp, Wp, R, h, V, part, st); break;
    case 4: rc = lm_head_launch<4, 8, 128>(Hp, Wp, R, h, V, part, st); break;
    case 5: rc = lm_head_launch<5, 8, 128>(Hp, Wp, R, h, V, part, st); break;
    case 6: rc = lm_head_launch<6, 8, 128>(Hp, Wp, R, h, V, part, st); break;
    case 7: rc = lm_head_launch<7, 8, 64>(Hp, Wp, R, h, V, part, st); break;
    case 8: rc = lm_head_launch<8, 8, 64>(Hp, Wp, R, h, V, part, st); break;
    default: rc = lm_head_launch<9, 8, 64>(Hp, Wp, R, h, V, part, st); break;
    }
    if (rc) return rc;
    hipLaunchKernelGGL(argmax_merge, dim3(R), dim3(256), 0, st, part, chunks, best);
    BTV_HIP(hipGetLastError());
    hipLaunchKernelGGL(greedy_walk, dim3(1), dim3(256), 0, st, best, 1, parent, token, M, path, n_acc, bonus, argmax_out);
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
