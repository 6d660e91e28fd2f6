// Acceptance walk on the GPU (gfx950): target argmax per tree row, greedy walk, and the
// token-level rejection walk at temperature 1.
//
// App. C "Acceptance" / Sec. 3.1: the committed tokens are the longest root-to-node path the
// target itself would have produced.  Rows of `logits`: 0 = root, 1+i = node i.
#include "btv_common.h"

#include <atomic>

#include <algorithm>
#include <climits>

namespace {

constexpr int ACHUNK = 8192;     // vocabulary elements per argmax workgroup

struct alignas(8) Best { float v; int i; };


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

// Best element of vocabulary chunk `chunk` of row `row` as seen by this thread (256 threads per workgroup).  Whole,
// 16-byte aligned chunks take four (bf16) or eight (fp32) 16-byte loads per thread, all in flight before the first
// is looked at.
template <bool BF16>
__device__ __forceinline__ Best chunk_scan(const void *logits, int V, int row, int chunk, int tid)
{
    const int v0 = chunk * ACHUNK, v1 = min(v0 + ACHUNK, V);
    Best b = { -INFINITY, INT_MAX };
    if (BF16) {
        const uint16_t *x = static_cast<const uint16_t *>(logits) + (size_t)row * V;
        if ((((size_t)row * V * 2) & 15) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0) {
            if (v1 - v0 == ACHUNK) {
                uint4 q[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) q[j] = *reinterpret_cast<const uint4 *>(x + v0 + tid * 8 + j * 2048);
                // the thread meets its elements in rising index order: "larger than the best so far" keeps the first of
                // equal values, the place is the element's number (a constant of the instruction); elements equal to
                // the start value, -inf, are not taken, and a wavefront in which a thread ends without a place takes
                // the exact pass below
                float bv = -INFINITY;
                int bk = -1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t wds[4] = { q[j].x, q[j].y, q[j].z, q[j].w };
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(wds[e] << 16), hi = __uint_as_float(wds[e] & 0xFFFF0000u);
                        if (lo > bv) { bv = lo; bk = j * 8 + 2 * e; }
                        if (hi > bv) { bv = hi; bk = j * 8 + 2 * e + 1; }
                    }
                }
                if (__builtin_amdgcn_ballot_w64(bk < 0) == 0ull) {
                    b.v = bv;
                    b.i = v0 + tid * 8 + (bk >> 3) * 2048 + (bk & 7);
                    return b;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t wds[4] = { q[j].x, q[j].y, q[j].z, q[j].w };
                    const int v = v0 + tid * 8 + j * 2048;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        best_take(b, __uint_as_float(wds[e] << 16), v + 2 * e);
                        best_take(b, __uint_as_float(wds[e] & 0xFFFF0000u), v + 2 * e + 1);
                    }
                }
                return b;
            }
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
            if (v1 - v0 == ACHUNK) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float4 q[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) q[j] = *reinterpret_cast<const float4 *>(x + v0 + tid * 4 + (h * 4 + j) * 1024);
                    float bv = b.v;                              // (as for bf16: rising order, exact pass on demand)
                    int bk = -1;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float f[4] = { q[j].x, q[j].y, q[j].z, q[j].w };
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (f[e] > bv) { bv = f[e]; bk = j * 4 + e; }
                    }
                    const bool none = bk < 0 && b.i == INT_MAX;
                    if (__builtin_amdgcn_ballot_w64(none) == 0ull) {
                        if (bk >= 0) { b.v = bv; b.i = v0 + tid * 4 + (h * 4 + (bk >> 2)) * 1024 + (bk & 3); }
                        continue;
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int v = v0 + tid * 4 + (h * 4 + j) * 1024;
                        best_take(b, q[j].x, v); best_take(b, q[j].y, v + 1); best_take(b, q[j].z, v + 2); best_take(b, q[j].w, v + 3);
                    }
                }
                return b;
            }
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
    return b;
}

// grid = (chunks, rows).  part[(row*chunks + chunk)] = best of the chunk.
template <bool BF16>
__global__ __launch_bounds__(256) void argmax_chunks(const void *logits, int V, Best *part)
{
    __shared__ Best wb[4];
    const int tid = threadIdx.x, chunk = blockIdx.x, row = blockIdx.y;
    Best b = best_wave(chunk_scan<BF16>(logits, V, row, chunk, tid));
    if ((tid & 63) == 0) wb[tid >> 6] = b;
    __syncthreads();
    if (tid == 0) {
        Best r = wb[0];
        best_take(r, wb[1].v, wb[1].i); best_take(r, wb[2].v, wb[2].i); best_take(r, wb[3].v, wb[3].i);
        part[(size_t)row * gridDim.x + chunk] = r;
    }
}

// ------------------------------------------------------------------------------------------------
// Greedy acceptance of one request in one launch.  A wavefront scans one unit of WCHUNK vocabulary elements of one
// row; the waves of a workgroup fold the units that belong to the same row and leave one 64-bit key per row they
// touched in the workgroup's own slots of the workspace.  The workgroup with the highest index (the last one to be
// placed on the chip) then collects: it takes every slot with an atomic exchange against zero, again while a slot
// is still empty, merges the keys per row and walks the tree on its first wavefront.  Nobody else waits for
// anything, so every wait of the collector ends as soon as the other workgroups have run; a wall-clock limit
// (s_memrealtime) bounds it all the same, and running into it raises the workspace's flag.  The exchange leaves the
// slots at zero for the next call.
// The L2 caches of the 8 XCDs are not coherent with each other, and a device-scope fence writes back and
// invalidates a whole cache; the only words other workgroups must see are the slots, moved by relaxed device-scope
// atomics (executed at the memory side).  Counting the workgroups in instead (each waits for its key updates to be
// acknowledged, adds itself to a counter, the last one reads the keys) puts three dependent round trips to the
// memory side, about 2 us each, behind the scan; here it is the flight of a store and one exchange.
// Key = value bits made monotonic << 32 | ~index: the larger value wins, then the lower index; a key's upper half is
// never zero, so 1 stands for "only NaN seen": a row without a key has argmax 0, as in the two-launch path.
// The walk keeps node c in lane c % 64, register row c / 64: `ok` = the node's token is the target's argmax at its
// parent; a step is a ballot over "child of the current node and ok" per row, lowest node index first.
// ------------------------------------------------------------------------------------------------
constexpr int WALK_ROWS = (BTV_MAX_NODES + 63) / 64;
constexpr int WCHUNK = 4096;     // vocabulary elements per wavefront unit of the one-launch kernel
constexpr int OL_WAVES = 8;      // wavefronts per workgroup of the one-launch kernel (16: 8.7 us at 65 rows, 8: 7.7 us)
static_assert(OL_WAVES * 64 > BTV_MAX_NODES, "the collector gives every logit row a thread");
constexpr unsigned long long OL_NO_KEY = 1ull;
constexpr long long OL_WAIT_TICKS = 100000000ll;    // collector's limit: one second of the 100 MHz wall clock

// Rows that OL_WAVES consecutive units can touch: the slots a workgroup owns.
__host__ __device__ inline int ol_slots_per_wg(int chunks)
{
    const int r = (OL_WAVES - 1) / chunks + 2;
    return r < OL_WAVES ? r : OL_WAVES;
}

__device__ __forceinline__ unsigned long long best_key(Best b)
{
    if (b.i == INT_MAX) return 0ull;
    const uint32_t u = __float_as_uint(b.v + 0.0f);              // -0 counts as +0
    const uint32_t mono = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)mono << 32) | (uint32_t)~(uint32_t)b.i;
}

// Best element of elements v0 .. v1-1 of a row as seen by this lane.  Where the row is 16-byte aligned the unit is
// fetched with eight 16-byte loads per lane at a time, all in flight before the first is looked at; a ragged unit (the
// last of a row) takes the same loads with the pieces past its end redirected to its first piece and left out, and
// the elements behind the last whole piece one per lane.  Nothing here loads inside a loop whose next trip needs
// the value: twenty such trips for the last 1280 elements of a row were two thirds of the kernel's time.
template <bool BF16, bool WHOLE>
__device__ __forceinline__ void wave_scan_pieces(Best &b, const uint4 *x, int v0, int npiece, int lane)
{
    constexpr int PER = BF16 ? 8 : 4;                            // elements per 16-byte piece
    for (int h = 0; h * 512 < npiece; ++h) {
        uint4 q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int p = (h * 8 + j) * 64 + lane;
            q[j] = x[WHOLE || p < npiece ? p : 0];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int p = (h * 8 + j) * 64 + lane;
            if (!WHOLE && p >= npiece) continue;
            const int v = v0 + p * PER;
            const uint32_t wds[4] = { q[j].x, q[j].y, q[j].z, q[j].w };
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (BF16) {
                    best_take(b, __uint_as_float(wds[e] << 16), v + 2 * e);
                    best_take(b, __uint_as_float(wds[e] & 0xFFFF0000u), v + 2 * e + 1);
                } else {
                    best_take(b, __uint_as_float(wds[e]), v + e);
                }
            }
        }
    }
}

// A whole unit, the cheap way: the lane meets its elements in rising index order, so "larger than the best so far"
// alone keeps the first of equal values, and the place is kept as the number of the element within the trip (a
// constant in the instruction).  Three instructions per element against eight for best_take: with four wavefronts per
// SIMD the scan was bound by this arithmetic, not by memory.  Elements equal to the start value, -inf, are not
// taken here: a lane that ends without a place sends the wavefront through wave_scan_pieces after all.
template <bool BF16>
__device__ __forceinline__ void wave_scan_whole(Best &b, const uint4 *x, int v0, int lane)
{
    constexpr int PER = BF16 ? 8 : 4;
    for (int h = 0; h < WCHUNK / (512 * PER); ++h) {
        uint4 q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = x[(h * 8 + j) * 64 + lane];
        float bv = b.v;
        int bk = -1;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t wds[4] = { q[j].x, q[j].y, q[j].z, q[j].w };
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (BF16) {
                    const float lo = __uint_as_float(wds[e] << 16), hi = __uint_as_float(wds[e] & 0xFFFF0000u);
                    if (lo > bv) { bv = lo; bk = j * PER + 2 * e; }
                    if (hi > bv) { bv = hi; bk = j * PER + 2 * e + 1; }
                } else {
                    const float f = __uint_as_float(wds[e]);
                    if (f > bv) { bv = f; bk = j * PER + e; }
                }
            }
        }
        if (bk >= 0) {
            b.v = bv;
            b.i = v0 + ((h * 8 + bk / PER) * 64 + lane) * PER + bk % PER;
        }
    }
}

template <bool BF16>
__device__ __forceinline__ float wave_scan_one(const void *logits, size_t idx)
{
    if (BF16) return __uint_as_float((uint32_t)static_cast<const uint16_t *>(logits)[idx] << 16);
    return static_cast<const float *>(logits)[idx];
}

template <bool BF16>
__device__ __forceinline__ Best wave_scan(const void *logits, int V, int row, int v0, int v1, int lane)
{
    Best b = { -INFINITY, INT_MAX };
    constexpr int ES = BF16 ? 2 : 4, PER = 16 / ES;              // element size, elements per 16-byte load
    const bool aligned = (((size_t)row * V * ES) & 15) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0;
    const size_t base = (size_t)row * V;
    if (aligned) {                                               // (v0 is a multiple of WCHUNK)
        const uint4 *x = reinterpret_cast<const uint4 *>(static_cast<const unsigned char *>(logits) + (base + v0) * ES);
        const int npiece = (v1 - v0) / PER;
        if (v1 - v0 == WCHUNK) {
            wave_scan_whole<BF16>(b, x, v0, lane);
            if (__builtin_amdgcn_ballot_w64(b.i == INT_MAX) == 0ull) return b;
            b = Best{ -INFINITY, INT_MAX };                      // (a lane saw nothing above -inf)
            wave_scan_pieces<BF16, true>(b, x, v0, npiece, lane);
            return b;
        }
        wave_scan_pieces<BF16, false>(b, x, v0, npiece, lane);
        const int v = v0 + npiece * PER + lane;                  // fewer than PER elements are left
        const float last = wave_scan_one<BF16>(logits, base + (v < v1 ? v : v0));
        if (v < v1) best_take(b, last, v);
        return b;
    }
    for (int vb = v0; vb < v1; vb += 64 * 8) {                   // eight loads in flight
        float xv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int v = vb + j * 64 + lane;
            xv[j] = wave_scan_one<BF16>(logits, base + (v < v1 ? v : v0));
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int v = vb + j * 64 + lane;
            if (v < v1) best_take(b, xv[j], v);
        }
    }
    return b;
}

template <bool BF16>
__global__ __launch_bounds__(OL_WAVES * 64) void accept_greedy_one_launch(
    const void *logits, int V, int chunks, unsigned long long *slot, uint32_t *flag, const int32_t *parent,
    const int32_t *token, int M, int32_t *path, int32_t *n_acc, int32_t *bonus, int32_t *argmax_out, long long wait_ticks)
{
    __shared__ Best wbest[OL_WAVES];
    __shared__ int wrow[OL_WAVES];
    __shared__ int t[BTV_MAX_NODES + 1];
    __shared__ unsigned long long rowmax[BTV_MAX_NODES + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, units = (M + 1) * chunks;
    const int RS = ol_slots_per_wg(chunks);
    const bool collector = blockIdx.x == gridDim.x - 1;
    // the collector's walk needs the tree: asked for now, used after the scan
    int par[WALK_ROWS], tok[WALK_ROWS];
#pragma unroll
    for (int r = 0; r < WALK_ROWS; ++r) {
        const int c = r * 64 + lane;
        const bool mine = collector && wave == 0 && c < M;
        par[r] = mine ? parent[c] : INT_MIN;
        tok[r] = mine ? token[c] : -1;
    }
    {
        const int u = blockIdx.x * OL_WAVES + wave;              // (the grid covers the units exactly once)
        Best b = { -INFINITY, INT_MAX };
        int row = -1;
        if (u < units) {
            row = u / chunks;
            const int chunk = u - row * chunks;
            b = best_wave(wave_scan<BF16>(logits, V, row, chunk * WCHUNK, min(chunk * WCHUNK + WCHUNK, V), lane));
        }
        if (lane == 0) { wbest[wave] = b; wrow[wave] = row; }
        if (collector)
            for (int i = tid; i <= M; i += OL_WAVES * 64) rowmax[i] = 0ull;
        __syncthreads();
        if (tid < OL_WAVES && wrow[tid] >= 0 && (tid == 0 || wrow[tid - 1] != wrow[tid])) {
            // first unit of a row within this workgroup: fold the row's other units, leave the key
            Best r = wbest[tid];
            for (int j = tid + 1; j < OL_WAVES && wrow[j] == wrow[tid]; ++j) best_take(r, wbest[j].v, wbest[j].i);
            const unsigned long long key = best_key(r);
            __hip_atomic_store(slot + (size_t)blockIdx.x * RS + (wrow[tid] - wrow[0]), key != 0ull ? key : OL_NO_KEY,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (!collector) return;
    // workgroup w owns units OL_WAVES w .. OL_WAVES (w + 1) - 1 (as far as they exist); its slot j belongs to row
    // (OL_WAVES w) / chunks + j
    {
        const long long t0 = (long long)__builtin_amdgcn_s_memrealtime();
        bool late = wait_ticks < 0;                              // (a negative limit: give up at once, for tests of this path)
        for (int s = tid; s < (int)gridDim.x * RS && !late; s += OL_WAVES * 64) {
            const int w = s / RS, j = s - w * RS;
            const int r0 = (w * OL_WAVES) / chunks, r1 = min(w * OL_WAVES + OL_WAVES - 1, units - 1) / chunks;
            if (j > r1 - r0) continue;
            unsigned long long key = 0ull;
            for (;;) {
                key = __hip_atomic_exchange(slot + s, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (key != 0ull) break;
                if ((long long)__builtin_amdgcn_s_memrealtime() - t0 > wait_ticks) { late = true; break; }
                __builtin_amdgcn_s_sleep(8);
            }
            if (key > 0xFFFFFFFFull) atomicMax(&rowmax[r0 + j], key);
        }
        if (late) atomicOr(flag, 128u);
    }
    __syncthreads();
    if (tid <= M) {
        const unsigned long long key = rowmax[tid];
        t[tid] = key == 0ull ? 0 : (int)~(uint32_t)key;
        if (argmax_out) argmax_out[tid] = t[tid];
    }
    __syncthreads();
    if (tid >= 64) return;
    bool ok[WALK_ROWS];
#pragma unroll
    for (int r = 0; r < WALK_ROWS; ++r) {
        const int c = r * 64 + tid;
        ok[r] = c < M && par[r] >= -1 && par[r] < M && tok[r] == t[par[r] + 1];
    }
    int cur = -1, n = 0;
    while (n < M) {
        int nx = -1;
#pragma unroll
        for (int r = WALK_ROWS - 1; r >= 0; --r) {
            const unsigned long long m = __builtin_amdgcn_ballot_w64(ok[r] && par[r] == cur);
            if (m != 0ull) nx = r * 64 + __builtin_ctzll(m);
        }
        if (nx < 0) break;
        if (tid == 0) path[n] = nx;
        cur = nx;
        ++n;
    }
    if (tid == 0) { *n_acc = n; *bonus = t[cur + 1]; }
}

// One workgroup per request: finish the argmax of every row, then walk the tree.  With q_offset (a batch),
// request r owns nodes q_offset[r] .. q_offset[r+1] - 1 and logit rows q_offset[r] + r .. q_offset[r+1] + r (its
// root row first); without, there is one request of M nodes.
__global__ __launch_bounds__(256) void greedy_walk(const Best *part, int chunks, const int32_t *parent,
                                                   const int32_t *token, int M, int32_t *path, int32_t *n_acc,
                                                   int32_t *bonus, int32_t *argmax_out, const int32_t *q_offset,
                                                   int total_M, uint32_t *flag)
{
    __shared__ int t[BTV_MAX_NODES + 1];
    __shared__ int par[BTV_MAX_NODES], tok[BTV_MAX_NODES];
    __shared__ int next;
    const int tid = threadIdx.x;
    if (q_offset) {
        const int rq = blockIdx.x, o0 = q_offset[rq], m = q_offset[rq + 1] - o0;
        n_acc += rq; bonus += rq;
        // M = the largest request the caller announced; a request may not reach past the total_M rows of the arrays
        if (o0 < 0 || m < 1 || m > M || (long long)o0 + m > (long long)total_M) {
            if (tid == 0) { atomicOr(flag, 32u); *n_acc = 0; *bonus = 0; }
            return;
        }
        M = m;
        part += (size_t)(o0 + rq) * chunks;
        parent += o0; token += o0; path += o0;
        if (argmax_out) argmax_out += o0 + rq;
    }
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
// Transposed product, C^T = W_tile * H^T (v_mfma_f32_32x32x16_bf16): a wave owns TV tiles of 32
// vocabulary rows and every row of H, so a lane's accumulator registers run over vocabulary rows of
// one H row and the argmax is a per-lane scan.  The operand layout wants lane l to hold row l % 32,
// which as a direct load would touch 64 cache lines per instruction and use 16 bytes of each;
// instead every load instruction fetches whole row segments (8 or 16 lanes per row), and the block
// is turned round through a wave-private LDS tile.  H blocks [rows, KB] are shared by the waves
// through a double-buffered LDS slab.  All tiles store the 16-byte chunks of a row XOR-permuted by
// the row number, so operand reads (ds_read_b128, 16 lanes = 16 different rows) are conflict-free.
// ------------------------------------------------------------------------------------------------
typedef __bf16 lm_bf16x8 __attribute__((ext_vector_type(8)));
typedef float lm_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int lm_u32x4 __attribute__((ext_vector_type(4)));

template <int RT, int WAVES, int KB, int TV>
struct LmShape {
    static constexpr int THREADS = WAVES * 64, ROWS = RT * 32;
    static constexpr int VROWS = TV * 32;                 // vocabulary rows of a wave
    static constexpr int RB = KB * 2;                     // bytes of a tile row
    static constexpr int CPR = RB / 16;                   // 16-byte chunks per row
    static constexpr int WTILE = VROWS * RB, SLAB = ROWS * RB;
    static constexpr int LDS_BYTES = WAVES * WTILE + 2 * SLAB;
    static constexpr int WLD = VROWS * CPR / 64;          // load instructions per wave and block for W
    static constexpr int HLD = (ROWS * CPR + THREADS - 1) / THREADS;   // chunks of the H slab per thread and block
    static constexpr bool HEVEN = ROWS * CPR % THREADS == 0;
    static_assert(CPR == 8 || CPR == 16, "KB is 64 or 128");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of a CU");
    // byte offset of 16-byte chunk `col` of tile row `row`: 16 lanes reading one chunk index of 16 consecutive
    // rows must land in 16 different 16-byte bank groups of the 256-byte bank line
    __device__ static constexpr int at(int row, int col)
    {
        return row * RB + ((col ^ (CPR == 16 ? (row & 15) : ((row >> 1) & 7))) << 4);
    }
};

// One block of the contraction for a wave: KB / 16 steps of TV + RT operand reads and TV * RT MFMAs.  Here the
// reads are raw instructions with hand-placed waits (as ordinary loads each is waited for right before its MFMA,
// which leaves the matrix core idle for an LDS round trip): the reads of step j + 1 are issued before the MFMAs
// of step j, and the in-order counter tells when step j's have landed.
template <int RT, int TV>
__device__ __forceinline__ void lm_read_step(uint32_t wt, uint32_t hb, int tile_bytes, lm_u32x4 (&a)[TV], lm_u32x4 (&b)[RT])
{
#pragma unroll
    for (int tv = 0; tv < TV; ++tv)
        asm volatile("ds_read_b128 %0, %1" : "=v"(a[tv]) : "v"(wt + (uint32_t)(tv * tile_bytes)) : "memory");
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
        asm volatile("ds_read_b128 %0, %1" : "=v"(b[rt]) : "v"(hb + (uint32_t)(rt * tile_bytes)) : "memory");
}

template <int RT, int TV, int YOUNGER>
__device__ __forceinline__ void lm_wait_step(lm_u32x4 (&a)[TV], lm_u32x4 (&b)[RT])
{
    static_assert(YOUNGER >= 0 && YOUNGER <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(YOUNGER) : "memory");
#pragma unroll
    for (int tv = 0; tv < TV; ++tv) asm volatile("" : "+v"(a[tv]));     // uses below may not move above the wait
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) asm volatile("" : "+v"(b[rt]));
}

// ob = offset of this lane's operand chunk at step 0 within a 32-row tile; step j sits at ob ^ (j << 5)
template <int RT, int TV, int KB, int RB>
__device__ __forceinline__ void lm_multiply(uint32_t wt, uint32_t hb, uint32_t ob, lm_f32x16 (&acc)[TV][RT])
{
    constexpr int STEPS = KB / 16, N = TV + RT;
    static_assert(N <= 15, "lgkmcnt range");
    lm_u32x4 a[2][TV], b[2][RT];
    lm_read_step<RT, TV>(wt + ob, hb + ob, 32 * RB, a[0], b[0]);
#pragma unroll
    for (int j = 0; j < STEPS; ++j) {
        if (j + 1 < STEPS) {
            const uint32_t o = ob ^ (uint32_t)((j + 1) << 5);
            lm_read_step<RT, TV>(wt + o, hb + o, 32 * RB, a[(j + 1) & 1], b[(j + 1) & 1]);
            lm_wait_step<RT, TV, N>(a[j & 1], b[j & 1]);
        } else {
            lm_wait_step<RT, TV, 0>(a[j & 1], b[j & 1]);
        }
#pragma unroll
        for (int tv = 0; tv < TV; ++tv)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                acc[tv][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(lm_bf16x8, a[j & 1][tv]),
                                                                      __builtin_bit_cast(lm_bf16x8, b[j & 1][rt]),
                                                                      acc[tv][rt], 0, 0, 0);
    }
}

// The same block with ordinary loads, scheduled by the compiler: leaner in registers, used when the accumulators
// of many row tiles leave no room for a second set of operands.
template <int RT, int TV, int KB, int RB>
__device__ __forceinline__ void lm_multiply_plain(const unsigned char *wt, const unsigned char *hb, uint32_t ob,
                                                  lm_f32x16 (&acc)[TV][RT])
{
#pragma unroll
    for (int j = 0; j < KB / 16; ++j) {
        const uint32_t o = ob ^ (uint32_t)(j << 5);
        lm_u32x4 a[TV];
#pragma unroll
        for (int tv = 0; tv < TV; ++tv) a[tv] = *reinterpret_cast<const lm_u32x4 *>(wt + tv * 32 * RB + o);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const lm_u32x4 b = *reinterpret_cast<const lm_u32x4 *>(hb + rt * 32 * RB + o);
#pragma unroll
            for (int tv = 0; tv < TV; ++tv)
                acc[tv][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(lm_bf16x8, a[tv]),
                                                                      __builtin_bit_cast(lm_bf16x8, b), acc[tv][rt], 0, 0, 0);
        }
    }
}

template <int RT, int WAVES, int KB, int TV, bool RAW>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void lm_head_argmax(
    const uint16_t *__restrict__ H, const uint16_t *__restrict__ W, int R, int h, int V, Best *__restrict__ part)
{
    using S = LmShape<RT, WAVES, KB, TV>;
    extern __shared__ __align__(16) unsigned char lm_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r32 = lane & 31, half = lane >> 5;
    const int vwg = blockIdx.x * WAVES * S::VROWS, v0 = vwg + wave * S::VROWS;
    unsigned char *wtile = lm_lds + wave * S::WTILE;
    unsigned char *slab = lm_lds + WAVES * S::WTILE;
    const int nkb = h / KB;

    // Addresses are a wave-uniform base (block of the contraction, first row of the workgroup) plus a 32-bit
    // per-lane offset that never changes.
    // W: instruction i moves rows i*(64/CPR) .. of the wave's tile, CPR lanes per row
    constexpr int RPI = 64 / S::CPR;                       // rows per load instruction
    const int wcol = lane % S::CPR, wrow0 = lane / S::CPR;
    const unsigned char *wbase = reinterpret_cast<const unsigned char *>(W) + (size_t)vwg * h * 2;
    const unsigned char *hbase = reinterpret_cast<const unsigned char *>(H);
    uint32_t woff[S::WLD], hoff[S::HLD];
    // LDS destinations: rows 16 apart share the swizzle, so only the first 16 / RPI of a tile's store addresses
    // differ by more than a constant
    constexpr int WDN = 16 / RPI < S::WLD ? 16 / RPI : S::WLD;
    int wdst[WDN];
#pragma unroll
    for (int i = 0; i < S::WLD; ++i) {
        const int row = i * RPI + wrow0;
        woff[i] = (uint32_t)(min(v0 + row, V - 1) - vwg) * (uint32_t)(h * 2) + wcol * 16;
        if (i < WDN) wdst[i] = S::at(row, wcol);
    }
    // H: chunk c of the slab -> row c / CPR, column c % CPR
#pragma unroll
    for (int i = 0; i < S::HLD; ++i) {
        const int c = tid + i * S::THREADS, row = c / S::CPR, col = c % S::CPR;
        hoff[i] = (uint32_t)min(row, R - 1) * (uint32_t)(h * 2) + col * 16;
    }
    // a thread's chunks are THREADS / CPR rows apart, a multiple of 16: same swizzle, constant distance
    constexpr int HSTEP = S::THREADS / S::CPR;
    static_assert(HSTEP % 16 == 0, "H chunks of a thread must share the swizzle");
    const int hrow0 = tid / S::CPR, hdst0 = S::at(hrow0, tid % S::CPR);
    // operand reads: step j of a block uses chunk 2j + half of row r32 (same chunk on both sides), which sits at
    // at(r32, half) ^ (j << 5): the swizzle is an XOR and 2j + half = 2j ^ half
    const uint32_t ob = (uint32_t)S::at(r32, half);

    lm_f32x16 acc[TV][RT];
#pragma unroll
    for (int tv = 0; tv < TV; ++tv)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[tv][rt][e] = 0.f;

    // Workgroups start at different blocks of the contraction and wrap round: rows of W are a multiple of 4 KB
    // apart, so workgroups marching in step would all hit the same few memory channels.
    int curw = (blockIdx.x * 5) % nkb, curh = curw;
    // (staging arrays are of a native vector type: arrays of the uint4 struct were left in scratch memory)
#define LM_FETCH_W(w)                                                                                      \
    {                                                                                                      \
        const unsigned char *b_ = wbase + (size_t)curw * (KB * 2);                                         \
        curw = curw + 1 == nkb ? 0 : curw + 1;                                                             \
        _Pragma("unroll") for (int i = 0; i < S::WLD; ++i) w[i] = *reinterpret_cast<const lm_u32x4 *>(b_ + woff[i]); \
    }
#define LM_FETCH_H(x)                                                                                      \
    {                                                                                                      \
        const unsigned char *b_ = hbase + (size_t)curh * (KB * 2);                                         \
        curh = curh + 1 == nkb ? 0 : curh + 1;                                                             \
        _Pragma("unroll") for (int i = 0; i < S::HLD; ++i) x[i] = *reinterpret_cast<const lm_u32x4 *>(b_ + hoff[i]); \
    }
#define LM_STORE_W(w)                                                                                   \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < S::WLD; ++i)                                              \
            *reinterpret_cast<lm_u32x4 *>(wtile + wdst[i % WDN] + (i / WDN) * 16 * S::RB) = w[i];       \
    }
#define LM_STORE_H(x, dst)                                                                              \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < S::HLD; ++i)                                              \
            if (S::HEVEN || hrow0 + i * HSTEP < S::ROWS)   /* past the slab: fetched, never stored */   \
                *reinterpret_cast<lm_u32x4 *>((dst) + hdst0 + i * HSTEP * S::RB) = x[i];                \
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) void *)lm_lds);
    const uint32_t wt_addr = lds0 + wave * S::WTILE, slab_addr = lds0 + WAVES * S::WTILE;
#define LM_MULTIPLY(sl)                                                                                      \
    {                                                                                                        \
        if constexpr (RAW) lm_multiply<RT, TV, KB, S::RB>(wt_addr, slab_addr + (sl) * S::SLAB, ob, acc);     \
        else lm_multiply_plain<RT, TV, KB, S::RB>(wtile, slab + (sl) * S::SLAB, ob, acc);                    \
    }

    // While block t is multiplied from LDS, the weights of blocks t + 1 and t + 2 are in registers or on their way
    // (they come from HBM); H comes from the L2 and is fetched one block ahead.  Fetches past the end wrap round to
    // blocks already seen; they land where nobody reads.
    lm_u32x4 w0[S::WLD], w1[S::WLD], x[S::HLD];
    LM_FETCH_W(w0)
    LM_FETCH_H(x)
    LM_FETCH_W(w1)
    LM_STORE_H(x, slab)
    LM_STORE_W(w0)
    __syncthreads();
    for (int kb = 0; kb + 1 < nkb; kb += 2) {
        // even round: slab 0 and the W tile hold block kb, w1 block kb + 1
        LM_FETCH_H(x)                                   // block kb + 1
        LM_FETCH_W(w0)                                  // block kb + 2
        LM_MULTIPLY(0)
        LM_STORE_H(x, slab + S::SLAB)                   // slab 1 is idle in this round
        LM_STORE_W(w1)                                  // own W tile: consumed by the multiply above
        __syncthreads();
        LM_FETCH_H(x)                                   // block kb + 2
        LM_FETCH_W(w1)                                  // block kb + 3
        LM_MULTIPLY(1)
        LM_STORE_H(x, slab)
        LM_STORE_W(w0)
        __syncthreads();
    }
    if (nkb & 1) {                                      // the last block of an odd count sits in slab 0
        LM_MULTIPLY(0)
        __syncthreads();
    }
#undef LM_MULTIPLY
#undef LM_FETCH_W
#undef LM_FETCH_H
#undef LM_STORE_W
#undef LM_STORE_H

    // per-lane scan over the 16 vocabulary rows of a tile that it holds (ascending), other half, then the waves
    Best *wb = reinterpret_cast<Best *>(lm_lds);            // [WAVES][ROWS]
    static_assert(S::LDS_BYTES >= WAVES * S::ROWS * (int)sizeof(Best), "exchange area must fit");
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        Best b = { -INFINITY, INT_MAX };
#pragma unroll
        for (int tv = 0; tv < TV; ++tv)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int v = v0 + tv * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                if (v < V) best_take(b, acc[tv][rt][e], v);
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

// Shape of the LM-head kernel for R rows of H: row tiles, waves per workgroup, contraction block, vocabulary
// tiles per wave, raw or compiler-scheduled operand reads.
struct LmPlan { int rt, waves, kb, tv, raw; };

inline LmPlan lm_plan(int R)
{
    // Measured at h = 4096, V = 128256: every shape up to 160 rows runs within 10 % of the 1 or 2 row-tile case,
    // which is bound by the stream of W; pipelined raw reads pay only while a second set of operands fits beside
    // the accumulators, and two vocabulary tiles per wave bought nothing.
    const int rt = (R + 31) / 32;
    if (rt <= 2) return { rt, 4, 128, 1, 1 };
    if (rt <= 6) return { rt, 8, 128, 1, 0 };
    return { rt, 8, 64, 1, 0 };
}

inline int lm_chunks(int R, int V)
{
    const LmPlan p = lm_plan(R);
    return (V + p.waves * p.tv * 32 - 1) / (p.waves * p.tv * 32);
}

template <int RT, int WAVES, int KB, int TV, bool RAW>
int lm_head_launch(const uint16_t *H, const uint16_t *W, int R, int h, int V, Best *part, hipStream_t st)
{
    using S = LmShape<RT, WAVES, KB, TV>;
    static std::atomic<bool> configured{false};         // (one GPU per process: the attribute is set once)
    auto kern = lm_head_argmax<RT, WAVES, KB, TV, RAW>;
    if (!configured.load(std::memory_order_acquire)) {
        BTV_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    S::LDS_BYTES));
        configured.store(true, std::memory_order_release);
    }
    const int chunks = (V + WAVES * S::VROWS - 1) / (WAVES * S::VROWS);
    hipLaunchKernelGGL(kern, dim3(chunks), dim3(WAVES * 64), S::LDS_BYTES, st, H, W, R, h, V, part);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

int lm_head_dispatch(const uint16_t *H, const uint16_t *W, int R, int h, int V, Best *part, hipStream_t st)
{
    const LmPlan p = lm_plan(R);
#define LM_CASE(rt_, w_, kb_, tv_, raw_)                                                              \
    if (p.rt == rt_ && p.waves == w_ && p.kb == kb_ && p.tv == tv_ && p.raw == raw_)                  \
        return lm_head_launch<rt_, w_, kb_, tv_, raw_ != 0>(H, W, R, h, V, part, st);
    LM_CASE(1, 4, 128, 1, 1) LM_CASE(2, 4, 128, 1, 1)
    LM_CASE(3, 8, 128, 1, 0)
    LM_CASE(4, 8, 128, 1, 0) LM_CASE(5, 8, 128, 1, 0) LM_CASE(6, 8, 128, 1, 0)
    LM_CASE(7, 8, 64, 1, 0) LM_CASE(8, 8, 64, 1, 0) LM_CASE(9, 8, 64, 1, 0)
#undef LM_CASE
    return btv_fail(BTV_EINVAL, "no LM-head kernel for %d rows", R);
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

// Sum of x over the wavefront, returned in every lane: quad swaps, row mirrors, then the row totals travel down the
// rows (DPP moves of the two halves; lanes a step does not write add zero).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double x)
{
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, ROW_MASK, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, ROW_MASK, 0xF, true);
    return x + __longlong_as_double(((long long)(uint32_t)hi << 32) | (long long)(uint32_t)lo);
}
__device__ __forceinline__ double wave_sum_f64(double x)
{
    x = dpp_add<0xB1, 0xF>(x);      // quad_perm [1,0,3,2]
    x = dpp_add<0x4E, 0xF>(x);      // quad_perm [2,3,0,1]
    x = dpp_add<0x141, 0xF>(x);     // row_half_mirror
    x = dpp_add<0x140, 0xF>(x);     // row_mirror: every lane holds its row's total
    x = dpp_add<0x142, 0xA>(x);     // row_bcast15 into rows 1 and 3
    x = dpp_add<0x143, 0xC>(x);     // row_bcast31 into rows 2 and 3: lane 63 holds the total
    const long long b = __double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, 63), hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), 63);
    return __longlong_as_double(((long long)hi << 32) | (long long)lo);
}

template <bool BF16>
__device__ __forceinline__ float load_logit(const void *logits, size_t idx)
{
    if (BF16) return __uint_as_float((uint32_t)static_cast<const uint16_t *>(logits)[idx] << 16);
    return static_cast<const float *>(logits)[idx];
}

// Nothing is rewritten per rejection.  With e[v] = exp(logit[v] - max) and q0 = the draft marginal of the depth,
// the target distribution after k rejections at a node is  p_k[v] = max(alpha * e[v] - beta * q0[v], 0)  and the
// draft distribution  q_k[v] = q0[v] / T  for the tokens not yet tried (a rejected token has q_k > p_k, so its
// residual is zero from then on and the same formula covers it).  A rejection needs
//     Z = sum_v max(p_k[v] - q_k[v], 0) = sum_v max(alpha * e[v] - b1 * q0[v], 0),   b1 = beta + 1/T,
// then  alpha /= Z,  beta = b1 / Z,  T -= q0[x];  Z = 0 leaves p as it was.  Scalars are fp64; e is stored once
// per node in fp32.
// A rejection at a node with few children gets Z from a read-only pass over the vocabulary.  A node with a wide fan
// of children still to try sorts its tokens once into SW_BINS bins of the ratio q0/e (counting sort on the float's
// exponent and three mantissa bits, the (e, q0) pairs moved into bin order): token v contributes iff q0/e < alpha/b1,
// so Z is a prefix sum over the sorted pairs below the threshold's bin plus an exact scan of that one bin.
constexpr int SW_BINS = 2048;
constexpr int SW_PBINS = 2048;      // bins of a row that is prepared ahead of the walk (sw_bin_at); 4096 measured slower:
                                    // what the walk saves per rejection, the scatter kernel pays in histogram reads
constexpr int SW_BUILD_MIN = 40;    // children still untried at a node for the sort to be worth its cost (about 30 passes)
constexpr int SW_PRE_MIN = 6;       // children of the root from which its row is sorted ahead of the walk (a few passes' worth)
constexpr int SW_WIN = 11264;       // sorted pairs kept in LDS around the threshold

__device__ __forceinline__ int sw_bin(float ratio)
{
    const uint32_t b = (__float_as_uint(ratio) & 0x7FFFFFFFu) >> 20;      // NaN (0/0) and inf (e = 0) land on top: never active
    return (int)(b < (uint32_t)SW_BINS ? b : (uint32_t)SW_BINS - 1u);
}

// The same order-preserving map with the bins spent where the ratios are: binades elo .. (biased exponents) get 2^m
// bins each, what lies below shares bin 0 and what lies above (inf and NaN included) the last bin.  { 0, 3 } is sw_bin.
struct SwBin { int elo, m; };

__device__ __forceinline__ int sw_bin_at(float ratio, SwBin p)
{
    const uint32_t u = __float_as_uint(ratio) & 0x7FFFFFFFu;
    const int d = (int)(u >> 23) - p.elo;
    if (d < 0) return 0;
    const uint32_t b = ((uint32_t)d << p.m) | ((u & 0x7FFFFFu) >> (23 - p.m));
    return (int)(b < (uint32_t)SW_PBINS ? b : (uint32_t)SW_PBINS - 1u);
}

// Sorted pairs per prefix-sum chunk: 2^s with s the smallest value from 6 up that leaves at most SW_BINS chunks (a
// power of two, so that the chunk of a sorted position is a shift: the walk asks once per rejection).
__device__ __forceinline__ int sw_chunk_shift(int V)
{
    int s = 6;
    while (((V + (1 << s) - 1) >> s) > SW_BINS) ++s;
    return s;
}

// ---- the root's row sorted ahead of the walk, by many workgroups ---------------------------------------------------
// Wide fans sit under the root (the best-first tree puts up to N children there when the first position's
// marginal is flat), and a sort on the walk's single CU costs about 250 us.  When the root has at least SW_BUILD_MIN
// children, SW_PRE_WGS workgroups prepare the root's row before the walk starts: row maximum, e = exp(logit - max)
// with its sum, a bin histogram per workgroup, the (e, q0) pairs moved into bin order (bin offsets per workgroup),
// and the sums of e and q0 per chunk of the sorted pairs.  Every step is its own launch (the grid-wide
// dependencies are kernel boundaries); with fewer children every one of them returns at once.  The walk picks the
// prepared row up if SwPre::ready says so.  Each workgroup owns a contiguous slice of the vocabulary; all sums
// that cross workgroups are added in workgroup order, so they are the same in every run.
constexpr int SW_PRE_WGS = 32;

struct SwPre {                      // in the workspace, behind es and eq_sorted
    int ready;                      // 1: the root's row is prepared (written by sw_pre_scatter)
    float mx;
    double z, tq;
    float wg_max[SW_PRE_WGS];
    float wg_tlo[SW_PRE_WGS], wg_thi[SW_PRE_WGS];         // range of log2(q0) - logit * log2(e) over the slice's tokens with q0 > 0
    double wg_z[SW_PRE_WGS], wg_tq[SW_PRE_WGS];
    int start[SW_PBINS + 1];
    double chunk_e[SW_BINS], chunk_q[SW_BINS];            // sums over chunk c of the sorted pairs (not yet prefix sums)
    int hist[SW_PRE_WGS][SW_PBINS];                       // pairs of workgroup w in bin b
    // what the walk leaves for the bonus draw, and the draw's per-wavefront totals
    double b_alpha, b_beta, b_u;
    int b_has_q, b_depth;
    int b_count;                                          // workgroups of the bonus kernel that have left their totals
    double b_tot[SW_PRE_WGS * 16];
    int b_last[SW_PRE_WGS * 16];
};

__device__ __forceinline__ bool sw_root_is_wide(const int32_t *parent, int M, int tid, double *shd)
{
    int mine = 0;
    for (int c = tid; c < M; c += 1024) mine += parent[c] == -1 ? 1 : 0;
    return (int)block_sum((double)mine, shd, tid) >= SW_PRE_MIN;
}

__device__ __forceinline__ void sw_slice(int V, int wg, int &v0, int &v1)
{
    const int per = ((V + SW_PRE_WGS - 1) / SW_PRE_WGS + 3) & ~3;      // a multiple of four: slices keep the row's alignment
    v0 = min(wg * per, V);
    v1 = min(v0 + per, V);
}

// Bins of the prepared row: log2(q0 / e) = log2(q0) - (logit - max) * log2(e) lies within the range that sw_pre_max
// found (plus a binade of slack at either end for the roundings on the way); the binades of that range share the
// bins, as many per binade as fit.  With the fixed map a row whose ratios span 30 binades used 240 of the 2048 bins
// and the bin that the falling threshold sits in held 1500 pairs, all of which a rejection must look at.  Every
// kernel works the parameters out from the same numbers, so they agree.
__device__ __forceinline__ SwBin sw_bin_params(const SwPre *pre, float mx)
{
    float tlo = INFINITY, thi = -INFINITY;
    for (int w = 0; w < SW_PRE_WGS; ++w) { tlo = fminf(tlo, pre->wg_tlo[w]); thi = fmaxf(thi, pre->wg_thi[w]); }
    SwBin p = { 0, 3 };
    const float shift = mx * 1.44269504f;
    const float lo2 = tlo + shift, hi2 = thi + shift;
    if (!(lo2 <= hi2) || !(lo2 > -200.f) || !(hi2 < 200.f)) return p;      // no token with q0 > 0, or a range beyond fp32's
    const int elo = max((int)floorf(lo2) - 1 + 127, 0), ehi = min(max((int)ceilf(hi2) + 1 + 127, elo), 254);
    const int span = ehi - elo + 1;
    int m = 3;
    while (m < 10 && (span << (m + 1)) <= SW_PBINS) ++m;
    if ((span << m) > SW_PBINS) return p;
    p.elo = elo; p.m = m;
    return p;
}

template <bool BF16>
__global__ __launch_bounds__(1024) void sw_pre_max(const void *__restrict__ logits, const float *__restrict__ q0,
                                                   const int32_t *__restrict__ parent, int M, int V, SwPre *pre)
{
    __shared__ double shd[16];
    __shared__ float shf[16];
    const int tid = threadIdx.x;
    if (blockIdx.x == 0 && tid == 0) pre->ready = 0;
    if (!sw_root_is_wide(parent, M, tid, shd)) return;
    int v0, v1;
    sw_slice(V, blockIdx.x, v0, v1);
    float mx = -INFINITY, tlo = INFINITY, thi = -INFINITY;
    for (int v = v0 + tid; v < v1; v += 1024) {
        const float x = load_logit<BF16>(logits, v), q = q0[v];
        mx = fmaxf(mx, x);
        const float t = __log2f(q) - x * 1.44269504f;
        if (q > 0.f && fabsf(t) < 1e30f) { tlo = fminf(tlo, t); thi = fmaxf(thi, t); }
    }
    mx = block_max(mx, shf, tid);
    __syncthreads();
    tlo = -block_max(-tlo, shf, tid);
    __syncthreads();
    thi = block_max(thi, shf, tid);
    if (tid == 0) { pre->wg_max[blockIdx.x] = mx; pre->wg_tlo[blockIdx.x] = tlo; pre->wg_thi[blockIdx.x] = thi; }
}

template <bool BF16>
__global__ __launch_bounds__(1024) void sw_pre_exp(const void *__restrict__ logits, const float *__restrict__ q0,
                                                   const int32_t *__restrict__ parent, int M, int V, float *__restrict__ es,
                                                   SwPre *pre)
{
    __shared__ double shd[16];
    __shared__ int hist[SW_PBINS];
    const int tid = threadIdx.x;
    if (!sw_root_is_wide(parent, M, tid, shd)) return;
    float mx = pre->wg_max[0];
    for (int w = 1; w < SW_PRE_WGS; ++w) mx = fmaxf(mx, pre->wg_max[w]);
    for (int b = tid; b < SW_PBINS; b += 1024) hist[b] = 0;
    const SwBin bp = sw_bin_params(pre, mx);
    __syncthreads();
    int v0, v1;
    sw_slice(V, blockIdx.x, v0, v1);
    double z = 0.0, tq = 0.0;
    for (int v = v0 + tid; v < v1; v += 1024) {
        const float e = expf(load_logit<BF16>(logits, v) - mx), q = q0[v];
        es[v] = e;
        z += (double)e;
        tq += (double)q;
        atomicAdd(&hist[sw_bin_at(__fdiv_rn(q, e), bp)], 1);
    }
    z = block_sum(z, shd, tid);
    tq = block_sum(tq, shd, tid);                            // (the barriers also complete the histogram)
    if (tid == 0) { pre->wg_z[blockIdx.x] = z; pre->wg_tq[blockIdx.x] = tq; if (blockIdx.x == 0) pre->mx = mx; }
    for (int b = tid; b < SW_PBINS; b += 1024) pre->hist[blockIdx.x][b] = hist[b];
}

// Bin offsets and scatter in one launch: every workgroup adds up the histograms of all of them (the same 256 KB for
// each: cheaper than a launch of its own for one workgroup to do it), scans the bins, and moves its slice's pairs to
// where its share of each bin starts.  Workgroup 0 also leaves the bin starts and the row's sums for the walk.
__global__ __launch_bounds__(1024) void sw_pre_scatter(const float *__restrict__ q0, const int32_t *__restrict__ parent, int M, int V,
                                                       const float *__restrict__ es, float2 *__restrict__ eq_sorted, SwPre *pre)
{
    __shared__ double shd[16];
    __shared__ int wsum[16];
    __shared__ double part[2][SW_PRE_WGS];
    __shared__ int cursor[SW_PBINS];
    constexpr int PB = SW_PBINS / 1024;                      // bins per thread: PB * tid .. PB * tid + PB - 1
    static_assert(PB == 2 || PB == 4, "a thread's bins are fetched as one int2 or int4");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, me = blockIdx.x;
    if (!sw_root_is_wide(parent, M, tid, shd)) return;
    if (me == 0 && tid < SW_PRE_WGS) { part[0][tid] = pre->wg_z[tid]; part[1][tid] = pre->wg_tq[tid]; }
    int c[PB], mb[PB];                                       // all workgroups; those before this one
#pragma unroll
    for (int k = 0; k < PB; ++k) { c[k] = 0; mb[k] = 0; }
#pragma unroll
    for (int w = 0; w < SW_PRE_WGS; ++w) {
        int h[PB];
        if constexpr (PB == 4) {
            const int4 x = *reinterpret_cast<const int4 *>(&pre->hist[w][PB * tid]);
            h[0] = x.x; h[1] = x.y; h[2] = x.z; h[3] = x.w;
        } else {
            const int2 x = *reinterpret_cast<const int2 *>(&pre->hist[w][PB * tid]);
            h[0] = x.x; h[1] = x.y;
        }
#pragma unroll
        for (int k = 0; k < PB; ++k) { mb[k] = w == me ? c[k] : mb[k]; c[k] += h[k]; }
    }
    int own = 0;
#pragma unroll
    for (int k = 0; k < PB; ++k) own += c[k];
    int ci = own;
    for (int off = 1; off < 64; off <<= 1) {
        const int co = __shfl_up(ci, off);
        if (lane >= off) ci += co;
    }
    if (lane == 63) wsum[wv] = ci;
    __syncthreads();
    int cb = 0;
    for (int w = 0; w < wv; ++w) cb += wsum[w];
    int st[PB + 1];                                          // where the thread's bins start
    st[0] = cb + ci - own;
#pragma unroll
    for (int k = 0; k < PB; ++k) st[k + 1] = st[k] + c[k];
#pragma unroll
    for (int k = 0; k < PB; ++k) cursor[PB * tid + k] = st[k] + mb[k];
    if (me == 0) {
#pragma unroll
        for (int k = 0; k < PB; ++k) pre->start[PB * tid + k] = st[k];
        if (tid == 1023) pre->start[SW_PBINS] = st[PB];
        if (tid == 0) {
            double z = 0.0, tq = 0.0;
            for (int w = 0; w < SW_PRE_WGS; ++w) { z += part[0][w]; tq += part[1][w]; }
            pre->z = z; pre->tq = tq;
            pre->ready = 1;
        }
    }
    __syncthreads();
    int v0, v1;
    sw_slice(V, me, v0, v1);
    const SwBin bp = sw_bin_params(pre, pre->mx);
    for (int vb = v0; vb < v1; vb += 4 * 1024) {             // four tokens per thread at a time, their loads issued together
        float e[4], q[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int v = vb + tid + 1024 * k;
            e[k] = es[v < v1 ? v : v0];
            q[k] = q0[v < v1 ? v : v0];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int v = vb + tid + 1024 * k;
            if (v < v1) {
                const int pos = atomicAdd(&cursor[sw_bin_at(__fdiv_rn(q[k], e[k]), bp)], 1);
                eq_sorted[pos] = make_float2(e[k], q[k]);
            }
        }
    }
}

__global__ __launch_bounds__(1024) void sw_pre_chunks(const int32_t *__restrict__ parent, int M, int V,
                                                      const float2 *__restrict__ eq_sorted, SwPre *pre)
{
    __shared__ double shd[16];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (!sw_root_is_wide(parent, M, tid, shd)) return;
    const int CH = 1 << sw_chunk_shift(V);
    constexpr int PER = SW_BINS / (SW_PRE_WGS * 16);          // chunks per wavefront
    if (CH == 64) {                                          // one pair per lane and chunk: the wavefront's loads all at once
        float2 x[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = (blockIdx.x * 16 + wv + k * SW_PRE_WGS * 16) * 64 + lane;
            x[k] = eq_sorted[i < V ? i : 0];
            if (i >= V) x[k] = make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const double se = wave_sum_f64((double)x[k].x), sq = wave_sum_f64((double)x[k].y);
            const int c = blockIdx.x * 16 + wv + k * SW_PRE_WGS * 16;
            if (lane == 0) { pre->chunk_e[c] = se; pre->chunk_q[c] = sq; }
        }
        return;
    }
    for (int c = blockIdx.x * 16 + wv; c < SW_BINS; c += SW_PRE_WGS * 16) {
        double se = 0.0, sq = 0.0;
        for (int i = c * CH + lane; i < min(c * CH + CH, V); i += 64) {
            const float2 x = eq_sorted[i];
            se += (double)x.x; sq += (double)x.y;
        }
        se = wave_sum_f64(se); sq = wave_sum_f64(sq);
        if (lane == 0) { pre->chunk_e[c] = se; pre->chunk_q[c] = sq; }
    }
}

// The window of sorted pairs [lo, hi), hi - lo <= SW_WIN, by 1024 threads: every thread's loads are issued before the
// first is stored (a load and its store per loop trip is a round trip to the L2 per trip).
__device__ __forceinline__ void load_window(float2 *win, const float2 *eq_sorted, int lo, int hi, int tid)
{
    static_assert(SW_WIN % 1024 == 0, "whole trips of the workgroup");
    float2 t[SW_WIN / 1024];
#pragma unroll
    for (int q = 0; q < SW_WIN / 1024; ++q) {
        const int i = lo + tid + 1024 * q;
        t[q] = eq_sorted[i < hi ? i : lo];
    }
#pragma unroll
    for (int q = 0; q < SW_WIN / 1024; ++q) {
        const int i = lo + tid + 1024 * q;
        if (i < hi) win[i - lo] = t[q];
    }
}

template <bool BF16>
__global__ __launch_bounds__(1024) void stochastic_walk(const void *__restrict__ logits, const float *__restrict__ marg, int B,
                                                        const int32_t *__restrict__ parent, const int32_t *__restrict__ token,
                                                        int M, int V, const float *__restrict__ uniforms,
                                                        float *__restrict__ es, float2 *__restrict__ eq_sorted,
                                                        SwPre *__restrict__ pre, int32_t *path, int32_t *n_acc,
                                                        uint32_t *flag)
{
    __shared__ double shd[16];
    __shared__ float shf[16];
    __shared__ double seg[1024];
    __shared__ double chunkE[SW_BINS], chunkQ[SW_BINS];  // sums of e and q0 over the sorted pairs before chunk c
    __shared__ int start[SW_PBINS + 1], cursor[SW_BINS];
    __shared__ float2 win[SW_WIN + 256];                  // sorted pairs win_lo .. win_hi - 1 (the threshold only falls,
                                                          // so the window is refilled towards lower positions)
    __shared__ float2 child_eq[BTV_MAX_NODES];            // (e, q0) of node c's token, fetched for all nodes at once
    __shared__ int kid_node[BTV_MAX_NODES];               // the current node's children in node order (prepared row only)
    __shared__ float kid_u[BTV_MAX_NODES];
    __shared__ float2 kid_eq[BTV_MAX_NODES];              // (e, q0) of child j's token
    __shared__ double kid_invT[BTV_MAX_NODES], kid_lhs[BTV_MAX_NODES];    // 1/T when child j is tried; u * q_k[x] of its test
    __shared__ struct { double alpha, beta, T; int next, accepted, reload_hi, done, nkids, wcount[4]; } fast;
    const int tid = threadIdx.x;
    int cur = -1, n = 0, ui = 0, d = 0;
    for (;;) {
        const size_t base = (size_t)(cur + 1) * V;
        const float *q0 = marg + (size_t)(d < B ? d : 0) * V;    // (unused when d == B: no children there)
        const bool vec4 = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(q0) & 15) == 0;
        const int CS = sw_chunk_shift(V), CH = 1 << CS;           // sorted pairs per prefix-sum chunk
        // (the passes are unrolled so that several loads are in flight: one load per iteration leaves a pass bound
        // by the round trip to the L2)
        const bool prepared = cur == -1 && pre->ready == 1;      // the root's row was sorted ahead of this kernel
        double z = 0.0, tq = 0.0;
        const bool has_q = d < B;
        if (prepared) {
            z = pre->z; tq = pre->tq;
        } else {
            float mx = -INFINITY;
#pragma unroll 8
            for (int v = tid; v < V; v += 1024) mx = fmaxf(mx, load_logit<BF16>(logits, base + v));
            mx = block_max(mx, shf, tid);
#pragma unroll 8
            for (int v = tid; v < V; v += 1024) {
                const float e = expf(load_logit<BF16>(logits, base + v) - mx);
                es[v] = e; z += (double)e;
                tq += has_q ? (double)q0[v] : 0.0;
            }
            z = block_sum(z, shd, tid);                          // (its barriers also publish es)
            tq = block_sum(tq, shd, tid);
        }
        double alpha = 1.0 / z, beta = 0.0, T = tq;
        int accepted = -1, untried = 0;
        bool binned = false;
        int win_lo = 0, win_hi = 0;                              // (empty)
        auto scan_chunks = [&]() {                                // chunkE / chunkQ: per-chunk sums -> sums before the chunk
            const int lane = tid & 63, wv = tid >> 6;
            const double e0 = chunkE[2 * tid], e1 = chunkE[2 * tid + 1], q0s = chunkQ[2 * tid], q1s = chunkQ[2 * tid + 1];
            double ei = e0 + e1, qi = q0s + q1s;
            for (int off = 1; off < 64; off <<= 1) {
                const double eo = __shfl_up(ei, off), qo = __shfl_up(qi, off);
                if (lane >= off) { ei += eo; qi += qo; }
            }
            if (lane == 63) { seg[wv] = ei; seg[16 + wv] = qi; }
            __syncthreads();
            double eb = 0.0, qb = 0.0;
            for (int w = 0; w < wv; ++w) { eb += seg[w]; qb += seg[16 + w]; }
            const double ex = eb + ei - (e0 + e1), qxs = qb + qi - (q0s + q1s);
            chunkE[2 * tid] = ex; chunkE[2 * tid + 1] = ex + e0;
            chunkQ[2 * tid] = qxs; chunkQ[2 * tid + 1] = qxs + q0s;
            __syncthreads();
        };
        if (prepared) {                                          // (prepared implies d == 0 < B)
            {   // every load before the first store: one round trip to the L2, not one per loop trip
                int sb[SW_PBINS / 1024];
                double ce[SW_BINS / 1024], cq[SW_BINS / 1024];
#pragma unroll
                for (int k = 0; k < SW_PBINS / 1024; ++k) sb[k] = pre->start[tid + 1024 * k];
#pragma unroll
                for (int k = 0; k < SW_BINS / 1024; ++k) { ce[k] = pre->chunk_e[tid + 1024 * k]; cq[k] = pre->chunk_q[tid + 1024 * k]; }
                if (tid == 0) start[SW_PBINS] = pre->start[SW_PBINS];
#pragma unroll
                for (int k = 0; k < SW_PBINS / 1024; ++k) start[tid + 1024 * k] = sb[k];
#pragma unroll
                for (int k = 0; k < SW_BINS / 1024; ++k) { chunkE[tid + 1024 * k] = ce[k]; chunkQ[tid + 1024 * k] = cq[k]; }
            }
            __syncthreads();
            scan_chunks();
            binned = true;
        }
        if (prepared) {
            // ---- the sorted row is at hand: the children are tried by the first wavefront alone, out of LDS, with no
            // workgroup barrier per rejection; the others only help to move the window of sorted pairs --------------
            const int lane = tid & 63, wv = tid >> 6;
            const SwBin bp = sw_bin_params(pre, pre->mx);
            {   // the children in node order: (node, uniform), their tokens' (e, q0)
                const bool mine = tid < M && parent[tid] == cur;
                const unsigned long long bal = __builtin_amdgcn_ballot_w64(mine);
                if (wv < 4 && lane == 0) fast.wcount[wv] = __builtin_popcountll(bal);
                __syncthreads();
                if (mine) {
                    int j = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
                    for (int w = 0; w < wv; ++w) j += fast.wcount[w];
                    const int tk = token[tid];
                    kid_node[j] = tk >= 0 && tk < V ? tid : -1 - tid;      // (negative: not a vocabulary id)
                    kid_u[j] = uniforms[ui + j];
                    if (tk >= 0 && tk < V) child_eq[tid] = make_float2(es[tk], q0[tk]);
                }
                if (tid == 0) {
                    fast.alpha = alpha; fast.beta = beta; fast.T = T;
                    fast.next = 0; fast.accepted = -1; fast.done = 0;
                    fast.nkids = fast.wcount[0] + fast.wcount[1] + fast.wcount[2] + fast.wcount[3];
                }
                __syncthreads();
            }
            auto recip = [](double x) {                           // 1/x to within a few ulp: hardware estimate, two Newton steps
                double r = __builtin_amdgcn_rcp(x);
                r = __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
                r = __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
                return r;
            };
            // T falls by the tried token's q0 whatever the test decides, so every child's 1/T and the left side of its
            // test are known before the loop: an exclusive prefix sum over the children, 64 at a time
            if (wv == 0) {
                double carry = 0.0;
                for (int j0 = 0; j0 < fast.nkids; j0 += 64) {
                    const int j = j0 + lane;
                    const int c = j < fast.nkids ? kid_node[j] : -1;
                    const double qx = c >= 0 ? (double)child_eq[c].y : 0.0;
                    double incl = qx;
                    for (int off = 1; off < 64; off <<= 1) {
                        const double o = __shfl_up(incl, off);
                        if (lane >= off) incl += o;
                    }
                    const double Tj = T - (carry + (incl - qx));
                    if (j < fast.nkids) {
                        const double invT = Tj > 0.0 ? recip(Tj) : 0.0;
                        kid_eq[j] = c >= 0 ? child_eq[c] : make_float2(0.f, 0.f);
                        kid_invT[j] = invT;
                        kid_lhs[j] = (double)kid_u[j] * (qx * invT);
                    }
                    carry += __shfl(incl, 63);
                }
            }
            __syncthreads();
            for (;;) {
                if (wv == 0) {
                    int j = fast.next;
                    const int nk = fast.nkids;
                    int acc = -1, want_hi = -1;
                    alpha = fast.alpha; beta = fast.beta; T = fast.T;
                    // child j + 1's entries are read while child j is tested: nothing in them depends on the tests
                    const int jf = max(min(j, nk - 1), 0);
                    int c_nx = kid_node[jf];
                    float2 own_nx = kid_eq[jf];
                    double invT_nx = kid_invT[jf], lhs_nx = kid_lhs[jf];
                    for (; j < nk; ++j) {
                        const int c = c_nx;
                        const float2 own = own_nx;
                        const double invT = invT_nx, lhs = lhs_nx;
                        {
                            const int j1 = min(j + 1, nk - 1);
                            c_nx = kid_node[j1]; own_nx = kid_eq[j1]; invT_nx = kid_invT[j1]; lhs_nx = kid_lhs[j1];
                        }
                        if (__builtin_expect(c < 0, 0)) {        // spent uniform, raised flag, nothing indexed
                            if (lane == 0) atomicOr(flag, 64u);
                            continue;
                        }
                        const double px = alpha * (double)own.x - beta * (double)own.y;
                        if (__builtin_expect(lhs < (px > 0.0 ? px : 0.0), 0)) { acc = c; ++j; break; }
                        const double b1 = beta + invT;
                        const int b = sw_bin_at((float)(b1 > 0.0 ? alpha * recip(b1) : INFINITY), bp);
                        const int p0 = start[b], p1 = start[b + 1];
                        const int ch = min(p0 >> CS, SW_BINS - 1), lo = ch << CS;
                        const double ce = chunkE[ch], cq = chunkQ[ch];      // (asked for ahead of the scan's reads)
                        double zr = 0.0;
                        if (__builtin_expect(p1 - lo <= SW_WIN, 1)) {
                            if (__builtin_expect(lo < win_lo || p1 > win_hi, 0)) { want_hi = p1; break; }      // the others help to move the window
                            // four reads in flight per trip, none behind a branch (one read, its arithmetic and the loop
                            // branch per trip made a trip cost an LDS round trip: the larger part of a rejection)
                            // (the reads run up to 255 entries past p1, into the pad behind the window: what they bring is
                            // not used)
                            double z4[4] = { 0.0, 0.0, 0.0, 0.0 };
                            const float2 *wp = win + (lo - win_lo + lane);
                            const int trips = (p1 - lo + 255) >> 8;
                            for (int t = 0, i = lo + lane; t < trips; ++t, i += 256, wp += 256) {
                                float2 x[4];
#pragma unroll
                                for (int q = 0; q < 4; ++q) x[q] = wp[64 * q];
#pragma unroll
                                for (int q = 0; q < 4; ++q) {
                                    const double r = alpha * (double)x[q].x - b1 * (double)x[q].y;
                                    z4[q] += i + 64 * q < p1 && r > 0.0 ? r : 0.0;
                                }
                            }
                            zr = (z4[0] + z4[1]) + (z4[2] + z4[3]);
                        } else {                                 // a bin larger than the window (ratios that nearly all coincide)
                            for (int i = lo + lane; i < p1; i += 64) {
                                const float2 x = eq_sorted[i];
                                const double r = alpha * (double)x.x - b1 * (double)x.y;
                                zr += r > 0.0 ? r : 0.0;
                            }
                        }
                        zr = wave_sum_f64(zr);
                        const double below = alpha * ce - b1 * cq;
                        zr += below > 0.0 ? below : 0.0;
                        if (__builtin_expect(zr > 0.0, 1)) { const double iz = recip(zr); alpha *= iz; beta = b1 * iz; }
                    }
                    if (lane == 0) {
                        fast.alpha = alpha; fast.beta = beta; fast.T = T;
                        fast.next = j; fast.accepted = acc; fast.reload_hi = want_hi;
                        fast.done = want_hi < 0;
                    }
                }
                __syncthreads();
                if (fast.done) break;
                win_hi = fast.reload_hi;
                win_lo = max(win_hi - SW_WIN, 0);
                load_window(win, eq_sorted, win_lo, win_hi, tid);
                __syncthreads();
            }
            alpha = fast.alpha; beta = fast.beta; T = fast.T;
            accepted = fast.accepted;
            ui += fast.next;                                     // one uniform per child tried
            __syncthreads();                                     // (fast is rewritten at the next node only after everyone has read it)
        } else if (d < B) {
            // one round trip for every child's own e and q0, instead of one per child inside the loop
            for (int c = tid; c < M; c += 1024) {
                const bool mine = parent[c] == cur;
                untried += mine ? 1 : 0;
                const int tk = token[c];
                if (mine && tk >= 0 && tk < V) child_eq[c] = make_float2(es[tk], q0[tk]);
            }
            untried = (int)block_sum((double)untried, shd, tid);          // children of this node still to be tried
            for (int c = 0; c < M; ++c) {
                if (parent[c] != cur) continue;                  // uniform across the workgroup
                const int tk = token[c];
                const double u = (double)uniforms[ui++];
                if (tk < 0 || tk >= V) {                         // not a vocabulary id: the child is rejected (its uniform is
                    if (tid == 0) atomicOr(flag, 64u);           // spent), nothing is indexed with it, the data flag is raised
                    --untried;
                    continue;
                }
                const float2 own = child_eq[c];
                const double invT = T > 0.0 ? 1.0 / T : 0.0, qx = (double)own.y;
                const double px = alpha * (double)own.x - beta * qx;     // p_k of the child's token
                if (u * (qx * invT) < (px > 0.0 ? px : 0.0)) { accepted = c; break; }
                const double b1 = beta + invT;
                --untried;
                if (!binned && untried >= SW_BUILD_MIN) {         // enough tests may follow for the sort to pay
                    // ---- counting sort of the (e, q0) pairs by the bin of q0/e, then prefix sums over the sorted pairs ----
                    for (int b = tid; b < SW_BINS; b += 1024) start[b] = 0;
                    __syncthreads();
                    for (int v = tid; v < V; v += 1024) atomicAdd(&start[sw_bin(__fdiv_rn(q0[v], es[v]))], 1);
                    __syncthreads();
                    {   // exclusive scan of the bin counts (two bins per thread)
                        const int c0 = start[2 * tid], c1 = start[2 * tid + 1];
                        int ci = c0 + c1;
                        for (int off = 1; off < 64; off <<= 1) {
                            const int co = __shfl_up(ci, off);
                            if ((tid & 63) >= off) ci += co;
                        }
                        __syncthreads();
                        if ((tid & 63) == 63) cursor[tid >> 6] = ci;
                        __syncthreads();
                        int cb = 0;
                        for (int w = 0; w < (tid >> 6); ++w) cb += cursor[w];
                        __syncthreads();
                        const int cx = cb + ci - (c0 + c1);          // exclusive prefix of this thread's first bin
                        start[2 * tid] = cx; start[2 * tid + 1] = cx + c0;
                        cursor[2 * tid] = cx; cursor[2 * tid + 1] = cx + c0;
                        if (tid == 1023) start[SW_BINS] = cx + c0 + c1;
                    }
                    __syncthreads();
                    for (int v = tid; v < V; v += 1024) {
                        const float e = es[v], q = q0[v];
                        const int pos = atomicAdd(&cursor[sw_bin(__fdiv_rn(q, e))], 1);
                        eq_sorted[pos] = make_float2(e, q);          // one 8-byte store: the scattered stores are what the sort costs
                    }
                    __syncthreads();
                    {   // chunk c = sorted positions c*CH .. c*CH + CH - 1 (CH a power of two from 64 up, at most SW_BINS chunks): a
                        // wave sums a chunk with coalesced loads; then an exclusive scan over the chunk sums
                        const int lane = tid & 63, wv = tid >> 6;
                        for (int c = wv; c < SW_BINS; c += 16) {
                            double se = 0.0, sq = 0.0;
                            for (int i = c * CH + lane; i < min(c * CH + CH, V); i += 64) {
                                const float2 x = eq_sorted[i];
                                se += (double)x.x; sq += (double)x.y;
                            }
                            for (int off = 32; off >= 1; off >>= 1) { se += __shfl_xor(se, off); sq += __shfl_xor(sq, off); }
                            if (lane == 0) { chunkE[c] = se; chunkQ[c] = sq; }
                        }
                        __syncthreads();
                    }
                    scan_chunks();
                    binned = true;
                }
                double zr = 0.0;                                 // residual max(p_k - q_k, 0): its sum
                auto resid = [&](float ev, float qv) {
                    const double r = alpha * (double)ev - b1 * (double)qv;
                    zr += r > 0.0 ? r : 0.0;
                };
                if (binned) {
                    // pairs before the threshold's bin all contribute: whole chunks through the prefix sums, the rest
                    // of the chunk that holds the bin's start one by one; the threshold's own bin is scanned exactly
                    const int b = sw_bin((float)(alpha / b1));   // b1 = 0: the threshold is +inf, every finite ratio is below it
                    const int p0 = start[b], p1 = start[b + 1];
                    const int ch = min(p0 >> CS, SW_BINS - 1), lo = ch << CS;
                    if (p1 - lo <= SW_WIN) {
                        if (lo < win_lo || p1 > win_hi) {        // (uniform) refill: the window ends at this bin's end
                            __syncthreads();
                            win_hi = p1;
                            win_lo = max(p1 - SW_WIN, 0);
                            load_window(win, eq_sorted, win_lo, win_hi, tid);
                            __syncthreads();
                        }
                        for (int i = lo + tid; i < p1; i += 1024) { const float2 x = win[i - win_lo]; resid(x.x, x.y); }
                    } else {                                     // a bin larger than the window (ratios that nearly all coincide)
                        for (int i = lo + tid; i < p1; i += 1024) { const float2 x = eq_sorted[i]; resid(x.x, x.y); }
                    }
                    zr = block_sum(zr, shd, tid);
                    const double below = alpha * chunkE[ch] - b1 * chunkQ[ch];
                    zr += below > 0.0 ? below : 0.0;
                } else {
                    if (vec4) {
#pragma unroll 4
                        for (int v = tid * 4; v < V; v += 4096) {
                            const float4 a = *reinterpret_cast<const float4 *>(es + v), q = *reinterpret_cast<const float4 *>(q0 + v);
                            resid(a.x, q.x); resid(a.y, q.y); resid(a.z, q.z); resid(a.w, q.w);
                        }
                    } else {
                        for (int v = tid; v < V; v += 1024) resid(es[v], q0[v]);
                    }
                    zr = block_sum(zr, shd, tid);
                }
                if (zr > 0.0) { const double iz = 1.0 / zr; alpha *= iz; beta = b1 * iz; }
                T -= qx;                                         // drafted without replacement
            }
        }
        if (accepted >= 0) {
            if (tid == 0) path[n] = accepted;
            cur = accepted; ++n; ++d;
            __syncthreads();                                     // everyone is done with es before it is rewritten
            continue;
        }
        // The bonus token is drawn by the kernel that follows (a pass over the vocabulary in fp64 is bound by the
        // arithmetic of the one CU this kernel runs on: 16 us of its time): the residual's parameters, the uniform
        // and the row go to the workspace.
        if (tid == 0) {
            pre->b_alpha = alpha; pre->b_beta = beta; pre->b_u = (double)uniforms[ui];
            pre->b_has_q = has_q ? 1 : 0; pre->b_depth = has_q ? d : 0;
            pre->b_count = 0;
            *n_acc = n;
        }
        break;
    }
}

// Bonus draw: smallest v with cumsum(p_k)[v] > u, p_k = max(alpha e - beta q0, 0).  Wavefront g of SW_PRE_WGS * 16 owns
// a contiguous stretch of the vocabulary (whole wave instructions of 256 tokens, four per lane, when the rows allow
// 16-byte loads) and leaves its total and its last positive token; the workgroup that counts itself in last picks
// the token (sw_bonus_pick) on its first wavefront.  Totals, last tokens and the counter cross workgroups as relaxed
// device-scope atomics, the counter only after the stores are acknowledged (the L2s of the XCDs are not coherent
// with each other).
__device__ __forceinline__ double sw_resid(double alpha, double beta, bool has_q, float ev, float qv)
{
    const double x = has_q ? alpha * (double)ev - beta * (double)qv : alpha * (double)ev;
    return x > 0.0 ? x : 0.0;
}

__device__ __forceinline__ void sw_stretch(int V, bool wide, int g, int &w0, int &w1)
{
    const int waves = SW_PRE_WGS * 16;
    const int stretch = wide ? ((V + waves - 1) / waves + 255) / 256 * 256 : ((V + waves - 1) / waves + 63) / 64 * 64;
    w0 = (int)min((long long)g * stretch, (long long)V);
    w1 = min(w0 + stretch, V);
}

__device__ void sw_bonus_pick(const float *__restrict__ marg, int V, const float *__restrict__ es, SwPre *pre, int32_t *bonus,
                              int lane);

__global__ __launch_bounds__(1024) void sw_bonus_draw(const float *__restrict__ marg, int V, const float *__restrict__ es, SwPre *pre,
                                                      int32_t *bonus)
{
    __shared__ int is_last;
    const int tid = threadIdx.x, lane = tid & 63, g = blockIdx.x * 16 + (tid >> 6);
    const double alpha = pre->b_alpha, beta = pre->b_beta;
    const bool has_q = pre->b_has_q != 0;
    const float *q0 = marg + (size_t)pre->b_depth * V;
    const bool wide = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(q0) & 15) == 0 && (reinterpret_cast<uintptr_t>(es) & 15) == 0;
    int w0, w1;
    sw_stretch(V, wide, g, w0, w1);
    double loc = 0.0;
    int lp = -1;
    if (wide) {
        const int trips = (w1 - w0 + 255) / 256;                  // (wave-uniform)
        for (int t0 = 0; t0 < trips; t0 += 4) {                   // the loads of a trip issued together, none behind a branch
            float4 a[4], q[4];
            int vv[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int v = w0 + (t0 + k) * 256 + lane * 4;
                vv[k] = t0 + k < trips && v < w1 ? v : -1;
                a[k] = *reinterpret_cast<const float4 *>(es + (vv[k] < 0 ? 0 : v));
                q[k] = has_q ? *reinterpret_cast<const float4 *>(q0 + (vv[k] < 0 ? 0 : v)) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool ok = vv[k] >= 0;
                const double x0 = ok ? sw_resid(alpha, beta, has_q, a[k].x, q[k].x) : 0.0, x1 = ok ? sw_resid(alpha, beta, has_q, a[k].y, q[k].y) : 0.0,
                             x2 = ok ? sw_resid(alpha, beta, has_q, a[k].z, q[k].z) : 0.0, x3 = ok ? sw_resid(alpha, beta, has_q, a[k].w, q[k].w) : 0.0;
                loc += (x0 + x1) + (x2 + x3);
                lp = x3 > 0.0 ? vv[k] + 3 : x2 > 0.0 ? vv[k] + 2 : x1 > 0.0 ? vv[k] + 1 : x0 > 0.0 ? vv[k] : lp;
            }
        }
    } else {
        for (int v = w0 + lane; v < w1; v += 64) {
            const double x = sw_resid(alpha, beta, has_q, es[v], has_q ? q0[v] : 0.f);
            loc += x;
            lp = x > 0.0 ? v : lp;
        }
    }
    loc = wave_sum_f64(loc);
    for (int off = 32; off >= 1; off >>= 1) lp = max(lp, __shfl_xor(lp, off));
    if (lane == 0) {
        __hip_atomic_store(reinterpret_cast<unsigned long long *>(pre->b_tot) + g, (unsigned long long)__double_as_longlong(loc),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pre->b_last + g, lp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) is_last = __hip_atomic_fetch_add(&pre->b_count, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == SW_PRE_WGS - 1;
    __syncthreads();
    if (is_last && tid < 64) sw_bonus_pick(marg, V, es, pre, bonus, tid);
}

// One wavefront: the totals in order tell which stretch holds the crossing; that stretch is looked at again, a wave
// instruction's worth of tokens at a time: its total, then the lanes' prefix inside it, then the token inside the lane.
__device__ void sw_bonus_pick(const float *__restrict__ marg, int V, const float *__restrict__ es, SwPre *pre, int32_t *bonus,
                              int lane)
{
    constexpr int WAVES = SW_PRE_WGS * 16, PER = WAVES / 64;
    const double alpha = pre->b_alpha, beta = pre->b_beta, u = pre->b_u;
    const bool has_q = pre->b_has_q != 0;
    const float *q0 = marg + (size_t)pre->b_depth * V;
    const bool wide = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(q0) & 15) == 0 && (reinterpret_cast<uintptr_t>(es) & 15) == 0;
    // lane l holds stretches PER * l .. PER * l + PER - 1: sums before each of them, added in stretch order
    double t[PER];
    int lastpos = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        t[k] = __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<unsigned long long *>(pre->b_tot) + PER * lane + k,
                                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        lastpos = max(lastpos, __hip_atomic_load(pre->b_last + PER * lane + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    for (int off = 32; off >= 1; off >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, off));
    double own = 0.0;
#pragma unroll
    for (int k = 0; k < PER; ++k) own += t[k];
    double incl = own;
    for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    double before = incl - own;
    int gsel = INT_MAX;
    double bsel = 0.0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        if (gsel == INT_MAX && u >= before && u < before + t[k]) { gsel = PER * lane + k; bsel = before; }
        before += t[k];
    }
    const unsigned long long has = __builtin_amdgcn_ballot_w64(gsel != INT_MAX);
    int found = INT_MAX;
    if (has != 0ull) {                                           // (uniform) none if u is past the total
        const int src = __builtin_ctzll(has);
        const int g = __shfl(gsel, src);
        double running = __shfl(bsel, src);
        int w0, w1;
        sw_stretch(V, wide, g, w0, w1);
        int hit = INT_MAX;
        if (wide) {
            for (int g0 = w0; g0 < w1 && hit == INT_MAX; g0 += 256) {
                const int v = g0 + lane * 4;
                const bool ok = v < w1;
                const float4 a = *reinterpret_cast<const float4 *>(es + (ok ? v : 0));
                const float4 q = has_q ? *reinterpret_cast<const float4 *>(q0 + (ok ? v : 0)) : make_float4(0.f, 0.f, 0.f, 0.f);
                const double x0 = ok ? sw_resid(alpha, beta, has_q, a.x, q.x) : 0.0, x1 = ok ? sw_resid(alpha, beta, has_q, a.y, q.y) : 0.0,
                             x2 = ok ? sw_resid(alpha, beta, has_q, a.z, q.z) : 0.0, x3 = ok ? sw_resid(alpha, beta, has_q, a.w, q.w) : 0.0;
                double inc = (x0 + x1) + (x2 + x3);
                const double mine_sum = inc;
                const double tot = wave_sum_f64(inc);
                if (running + tot > u) {                         // (uniform) the crossing lies in these 256 tokens
                    for (int off = 1; off < 64; off <<= 1) {     // inclusive prefix over the lanes
                        const double o = __shfl_up(inc, off);
                        if (lane >= off) inc += o;
                    }
                    const double excl = running + (inc - mine_sum);
                    int mine = INT_MAX;                          // first of this lane's four tokens whose cumulative sum passes u
                    if (ok) {
                        if (excl + x0 > u) mine = v;
                        else if (excl + (x0 + x1) > u) mine = v + 1;
                        else if (excl + ((x0 + x1) + x2) > u) mine = v + 2;
                        else if (excl + ((x0 + x1) + (x2 + x3)) > u) mine = v + 3;
                    }
                    for (int off = 32; off >= 1; off >>= 1) mine = min(mine, __shfl_xor(mine, off));
                    if (mine != INT_MAX) hit = mine;             // (else rounding: the crossing is the next positive token)
                }
                running += tot;
            }
        } else {
            for (int v0 = w0; v0 < w1 && hit == INT_MAX; v0 += 64) {
                const int v = v0 + lane;
                double x = v < w1 ? sw_resid(alpha, beta, has_q, es[v], has_q ? q0[v] : 0.f) : 0.0;
                for (int off = 1; off < 64; off <<= 1) {         // inclusive prefix over the 64 tokens
                    const double o = __shfl_up(x, off);
                    if (lane >= off) x += o;
                }
                const unsigned long long over = __builtin_amdgcn_ballot_w64(v < w1 && running + x > u);
                if (over) hit = v0 + __builtin_ctzll(over);
                running += __shfl(x, 63);
            }
        }
        // rounding left the crossing just past the stretch
        found = hit != INT_MAX ? hit : max(__hip_atomic_load(pre->b_last + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), 0);
    }
    if (lane == 0) *bonus = found == INT_MAX ? lastpos : found;
}

// workgroups of the one-launch greedy kernel: OL_WAVES units each, every unit once
int greedy_wgs(int M, int V)
{
    const long long chunks = (V + WCHUNK - 1) / WCHUNK;
    return (int)(((long long)(M + 1) * chunks + OL_WAVES - 1) / OL_WAVES);
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
    if (stochastic) return BTV_WS_HEADER + 3 * btv_align_up((size_t)V * 4, BTV_WS_ALIGN) + btv_align_up(sizeof(SwPre), BTV_WS_ALIGN);
    const int chunks = (V + WCHUNK - 1) / WCHUNK;
    return BTV_WS_HEADER + btv_align_up((size_t)greedy_wgs(M, V) * ol_slots_per_wg(chunks) * sizeof(unsigned long long), BTV_WS_ALIGN);
}

int btv_tree_accept_greedy_tuned(const void *logits, int dtype, const int32_t *parent, const int32_t *token, int M, int V,
                                 int32_t *path, int32_t *n_acc, int32_t *bonus, int32_t *argmax_out, void *ws,
                                 size_t ws_bytes, void *stream, long long wait_ticks)
{
    int rc = check_accept(logits, dtype, parent, token, M, V, path, n_acc, bonus);
    if (rc) return rc;
    rc = btv_check_ws(ws, ws_bytes, btv_tree_accept_workspace(M, V, 0));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned long long *slot = reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    uint32_t *flag = static_cast<uint32_t *>(ws);
    const int chunks = (V + WCHUNK - 1) / WCHUNK, wgs = greedy_wgs(M, V);
    if (dtype == BTV_BF16)
        hipLaunchKernelGGL(accept_greedy_one_launch<true>, dim3(wgs), dim3(OL_WAVES * 64), 0, st, logits, V, chunks, slot,
                           flag, parent, token, M, path, n_acc, bonus, argmax_out, wait_ticks);
    else
        hipLaunchKernelGGL(accept_greedy_one_launch<false>, dim3(wgs), dim3(OL_WAVES * 64), 0, st, logits, V, chunks, slot,
                           flag, parent, token, M, path, n_acc, bonus, argmax_out, wait_ticks);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

int btv_tree_accept_greedy(const void *logits, int dtype, const int32_t *parent, const int32_t *token, int M, int V,
                           int32_t *path, int32_t *n_acc, int32_t *bonus, int32_t *argmax_out, void *ws,
                           size_t ws_bytes, void *stream)
{
    return btv_tree_accept_greedy_tuned(logits, dtype, parent, token, M, V, path, n_acc, bonus, argmax_out, ws, ws_bytes, stream,
                                        OL_WAIT_TICKS);
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
    rc = lm_head_dispatch(Hp, Wp, R, h, V, part, st);
    if (rc) return rc;
    hipLaunchKernelGGL(argmax_merge, dim3(R), dim3(256), 0, st, part, chunks, best);
    BTV_HIP(hipGetLastError());
    hipLaunchKernelGGL(greedy_walk, dim3(1), dim3(256), 0, st, best, 1, parent, token, M, path, n_acc, bonus, argmax_out,
                       static_cast<const int32_t *>(nullptr), 0, static_cast<uint32_t *>(nullptr));
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

size_t btv_tree_accept_batch_workspace(int batch, int total_M, int V)
{
    if (batch < 1 || total_M < 1 || V < 1) return 0;
    int chunks = (V + ACHUNK - 1) / ACHUNK;
    return BTV_WS_HEADER + btv_align_up(((size_t)total_M + batch) * chunks * sizeof(Best), BTV_WS_ALIGN);
}

int btv_tree_accept_greedy_batch(const void *logits, int dtype, const int32_t *parent, const int32_t *token,
                                 const int32_t *q_offset, int batch, int total_M, int M_max, int V, int32_t *path,
                                 int32_t *n_acc, int32_t *bonus, int32_t *argmax_out, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(logits && parent && token && q_offset && path && n_acc && bonus, "null pointer");
    BTV_REQUIRE(dtype == BTV_F32 || dtype == BTV_BF16, "dtype=%d unsupported", dtype);
    BTV_REQUIRE(batch >= 1 && total_M >= batch, "batch=%d, total_M=%d", batch, total_M);
    BTV_REQUIRE(M_max >= 1 && M_max <= BTV_MAX_NODES, "M_max=%d outside [1,%d]", M_max, BTV_MAX_NODES);
    BTV_REQUIRE(V >= 1, "V=%d", V);
    int rc = btv_check_ws(ws, ws_bytes, btv_tree_accept_batch_workspace(batch, total_M, V));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Best *part = reinterpret_cast<Best *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    const int chunks = (V + ACHUNK - 1) / ACHUNK, rows = total_M + batch;
    if (dtype == BTV_BF16) hipLaunchKernelGGL(argmax_chunks<true>, dim3(chunks, rows), dim3(256), 0, st, logits, V, part);
    else hipLaunchKernelGGL(argmax_chunks<false>, dim3(chunks, rows), dim3(256), 0, st, logits, V, part);
    BTV_HIP(hipGetLastError());
    hipLaunchKernelGGL(greedy_walk, dim3(batch), dim3(256), 0, st, part, chunks, parent, token, M_max, path, n_acc, bonus,
                       argmax_out, q_offset, total_M, static_cast<uint32_t *>(ws));
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
    const size_t vb = btv_align_up((size_t)V * 4, BTV_WS_ALIGN);
    float *es = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER);
    float2 *eq_sorted = reinterpret_cast<float2 *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER + vb);
    SwPre *pre = reinterpret_cast<SwPre *>(static_cast<unsigned char *>(ws) + BTV_WS_HEADER + 3 * vb);
    uint32_t *flag = static_cast<uint32_t *>(ws);
    // the root's row, prepared by many workgroups when the root has a wide fan (each kernel finds that out itself)
    if (dtype == BTV_BF16) {
        hipLaunchKernelGGL(sw_pre_max<true>, dim3(SW_PRE_WGS), dim3(1024), 0, st, logits, marginals, parent, M, V, pre);
        hipLaunchKernelGGL(sw_pre_exp<true>, dim3(SW_PRE_WGS), dim3(1024), 0, st, logits, marginals, parent, M, V, es, pre);
    } else {
        hipLaunchKernelGGL(sw_pre_max<false>, dim3(SW_PRE_WGS), dim3(1024), 0, st, logits, marginals, parent, M, V, pre);
        hipLaunchKernelGGL(sw_pre_exp<false>, dim3(SW_PRE_WGS), dim3(1024), 0, st, logits, marginals, parent, M, V, es, pre);
    }
    hipLaunchKernelGGL(sw_pre_scatter, dim3(SW_PRE_WGS), dim3(1024), 0, st, marginals, parent, M, V, es, eq_sorted, pre);
    hipLaunchKernelGGL(sw_pre_chunks, dim3(SW_PRE_WGS), dim3(1024), 0, st, parent, M, V, eq_sorted, pre);
    BTV_HIP(hipGetLastError());
    if (dtype == BTV_BF16)
        hipLaunchKernelGGL(stochastic_walk<true>, dim3(1), dim3(1024), 0, st, logits, marginals, B, parent, token, M, V,
                           uniforms, es, eq_sorted, pre, path, n_acc, flag);
    else
        hipLaunchKernelGGL(stochastic_walk<false>, dim3(1), dim3(1024), 0, st, logits, marginals, B, parent, token, M, V,
                           uniforms, es, eq_sorted, pre, path, n_acc, flag);
    // the bonus token: per-wavefront totals of the residual on 32 workgroups, the last of which finds the crossing
    hipLaunchKernelGGL(sw_bonus_draw, dim3(SW_PRE_WGS), dim3(1024), 0, st, marginals, V, es, pre, bonus);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

}  // extern "C"
