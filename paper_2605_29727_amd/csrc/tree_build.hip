// Best-first draft-tree construction on the GPU (gfx950).
//
// Sec. 3.3 / Prop. 3.3 / Algorithm 1's frontier rule at a fixed budget N: repeatedly emit the
// frontier prefix with the largest path score rho (Eq. 1), then push its best child and its next
// sibling.  Two kernels:
//   1. tb_thread_max   per slot of 32 marginals (one thread's share of a chunk): the largest, its place in the
//                      slot, and the second largest (one pass over [B, V], all CUs);
//   2. tb_rank_expand  workgroup k derives from the maxima of position k a bound below which no token can be
//                      among its K best (K = min(V, N): a rank-j token is preceded by its j earlier siblings, so
//                      ranks >= N can never be emitted); a slot whose maximum reaches the bound and whose second
//                      largest does not gives its maximum as a candidate, the few other slots that reach the
//                      bound are read again; the candidates are ranked (order: probability desc, token id asc);
//                      the workgroup that finishes last runs the expansion.
// Keys are 64-bit  prob_bits << 32 | ~id  (probabilities are non-negative, so the bit pattern orders like
// the value; keys are distinct).
// rho(child) = rho(parent) * q is one fp32 multiply (never fused), the root has rho = 1.
// Frontier order: rho desc, depth asc, rank path lexicographic asc.
#include "btv_common.h"

#include <algorithm>
#include <type_traits>

namespace {

typedef unsigned long long u64;

constexpr int MAXB = BTV_MAX_DEPTH;
constexpr int SCAN = 8192;        // marginals scanned per workgroup (256 threads x 32)

__device__ __forceinline__ u64 make_key(float prob, uint32_t id)
{
    uint32_t b = __float_as_uint(prob);
    if (b == 0x80000000u) b = 0u;                  // -0.0 sorts as 0
    return ((u64)b << 32) | (u64)(0xFFFFFFFFu - id);
}

__device__ __forceinline__ uint32_t prob_bits(float p) { return __float_as_uint(p) & 0x7FFFFFFFu; }   // -0.0 counts as 0

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Wave-wide maximum as a wave-uniform value: quad swaps, row mirrors, then the row maxima travel down the rows
// (row_bcast), so that lane 63 ends up with the maximum.  The DPP operand sits on the max instruction itself;
// lanes whose source is masked out keep their value.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    uint32_t out;
    asm volatile("s_nop 1\n"
                 "v_max_u32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n s_nop 1\n"
                 "v_max_u32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n s_nop 1\n"
                 "v_max_u32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n s_nop 1\n"
                 "v_max_u32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n s_nop 1\n"
                 "v_max_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n s_nop 1\n"
                 "v_max_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n s_nop 1\n"
                 "v_readlane_b32 %1, %0, 63"
                 : "+v"(v), "=s"(out));
    return out;
}

// Inclusive prefix sum over the wavefront on the vector ALU: shifts within the rows of 16 lanes (zeros enter from
// outside a row), then the row totals travel down the rows.
__device__ __forceinline__ int wave_incl_scan(int x)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);    // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);    // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);    // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);    // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
    return x;
}

__device__ __forceinline__ int wave_incl_max(int x)               // the same with max, for values >= 0
{
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false));
    return x;
}

// The ranked lists travel from the workgroups that rank to the one that expands through memory, within one launch and
// between compute dies whose L2 caches do not see each other: they are written and read as relaxed device-scope
// atomics, which go through to memory, and the writer waits for its stores before it counts itself as done.
__device__ __forceinline__ void publish(float *q_row, uint32_t *tok_row, int r, float q, uint32_t tok)
{
    __hip_atomic_store(q_row + r, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(tok_row + r, tok, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}


// ------------------------------------------------------------------------------------------------
// Step 1: per-thread maxima.  Workgroup (chunk, row) scans elements chunk*SCAN .. chunk*SCAN + SCAN - 1 of the
// row; thread t looks at elements 4t..4t+3 of every 1024 (its slot: 32 elements, numbered k = 4 * piece + element)
// and keeps the largest probability it saw, where it saw it, and the second largest:
// part[row][chunk][t] = { bits of the largest, bits of the second largest with k of the largest in the low 5 bits }.
// The second largest is only ever compared with a bound whose low 19 bits are zero, so the 5 bits cost nothing.
// Among equal probabilities the first one counts as the largest and the next as the second largest.
// ------------------------------------------------------------------------------------------------
struct TbCounters { int done; };

template <typename F>
__device__ __forceinline__ void scan_chunk(const float *src, bool aligned, int V, int chunk, int tid, F f)
{
#pragma unroll
    for (int j = 0; j < SCAN / 1024; ++j) {
        const int v0 = chunk * SCAN + j * 1024 + tid * 4;        // coalesced: a wave reads 1 KiB per load
        if (aligned && v0 + 4 <= V) {
            const float4 a = *reinterpret_cast<const float4 *>(src + v0);
            f(a.x, 4 * j); f(a.y, 4 * j + 1); f(a.z, 4 * j + 2); f(a.w, 4 * j + 3);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (v0 + i < V) f(src[v0 + i], 4 * j + i);
        }
    }
}

__global__ __launch_bounds__(256) void tb_thread_max(const float *marg, int V, int B, int chunks, uint2 *part, TbCounters *ctr)
{
    const int tid = threadIdx.x, chunk = blockIdx.x, row = blockIdx.y;
    const float *src = marg + (size_t)row * V;
    const bool aligned = (((size_t)row * V) & 3) == 0 && (reinterpret_cast<uintptr_t>(marg) & 15) == 0;
    uint32_t m1 = 0u, m2 = 0u, k1 = 0u;
    scan_chunk(src, aligned, V, chunk, tid, [&](float p, int k) {
        const uint32_t b = prob_bits(p);
        m2 = umax(m2, b < m1 ? b : m1);                          // the smaller of the newcomer and the best so far
        k1 = b > m1 ? (uint32_t)k : k1;
        m1 = umax(m1, b);
    });
    part[((size_t)row * chunks + chunk) * 256 + tid] = make_uint2(m1, (m2 & ~31u) | k1);
    if (chunk == 0 && row % B == 0 && tid == 0) ctr[row / B].done = 0;   // the next kernel starts after this one has ended
}

constexpr int TBINS = 4096;

// ------------------------------------------------------------------------------------------------
// Step 2 (inside tb_rank_expand): the bound and the candidates of one position.  Every per-thread maximum of
// step 1 is a different token of the row, so the K-th largest of them (K <= 256 <= their number) is a lower bound
// of the row's K-th largest probability, and a tight one: it only falls short by the few tokens of the K best
// that share a slot with a better one.  The workgroup finds the 12-bit bin (sign-less float bits [30:19]: an
// eighth of a binade) that holds it from a histogram of the chunks*256 maxima and takes the lower edge of that bin
// as the bound; only slots whose maximum reaches the bound can hold candidates (about K of the chunks*256).  Where
// the slot's second largest stays below the bound, the maximum is the slot's one candidate and goes to the list
// from what step 1 recorded; the other slots, a handful, are read again, 32 elements each, and their elements at
// or above the bound join the list in LDS: K plus a few.
// Step 3, part A: the candidates are ranked by counting the candidates above each (order: probability desc, token
// id asc) and the K best go to the position's top list.  More than SELCAP candidates (heavily tied or otherwise
// degenerate probabilities): the K-th largest key of the whole row is found by radix selection, one byte of the
// key per pass (histogram of 256 bins, one wavefront), and the K keys at or above it are ranked the same way.
// ------------------------------------------------------------------------------------------------
constexpr int SELCAP = 512;
constexpr int SLOTCAP = 1024;

__device__ __forceinline__ int bin_at(int b) { return b + (b >> 4); }

// Element i of sixteen registers for a lane-dependent i, by halving.  The values arrive one by one and pass through an
// empty asm, which hides from the compiler that they are the elements of one array: it would turn the selects into
// an indexed load and move the array into scratch memory.
__device__ __forceinline__ uint32_t pick16v(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3, uint32_t x4, uint32_t x5, uint32_t x6, uint32_t x7, uint32_t x8, uint32_t x9, uint32_t x10, uint32_t x11, uint32_t x12, uint32_t x13, uint32_t x14, uint32_t x15, int i)
{
    asm volatile("" : "+v"(x0)); asm volatile("" : "+v"(x1)); asm volatile("" : "+v"(x2)); asm volatile("" : "+v"(x3)); asm volatile("" : "+v"(x4)); asm volatile("" : "+v"(x5)); asm volatile("" : "+v"(x6)); asm volatile("" : "+v"(x7)); asm volatile("" : "+v"(x8)); asm volatile("" : "+v"(x9)); asm volatile("" : "+v"(x10)); asm volatile("" : "+v"(x11)); asm volatile("" : "+v"(x12)); asm volatile("" : "+v"(x13)); asm volatile("" : "+v"(x14)); asm volatile("" : "+v"(x15));
    const uint32_t a0 = (i & 8) ? x8 : x0, a1 = (i & 8) ? x9 : x1, a2 = (i & 8) ? x10 : x2, a3 = (i & 8) ? x11 : x3;
    const uint32_t a4 = (i & 8) ? x12 : x4, a5 = (i & 8) ? x13 : x5, a6 = (i & 8) ? x14 : x6, a7 = (i & 8) ? x15 : x7;
    const uint32_t b0 = (i & 4) ? a4 : a0, b1 = (i & 4) ? a5 : a1, b2 = (i & 4) ? a6 : a2, b3 = (i & 4) ? a7 : a3;
    const uint32_t c0 = (i & 2) ? b2 : b0, c1 = (i & 2) ? b3 : b1;
    return (i & 1) ? c1 : c0;
}
#define BTV_PICK16(x, i) pick16v(x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7], x[8], x[9], x[10], x[11], x[12], x[13], x[14], x[15], i)

struct alignas(16) RankLds {                // bound and ranking of one position
    union {
        int bins[TBINS + TBINS / 16];       // histogram of the per-thread maxima (before the candidates exist); bin b at
                                            // b + b / 16, so that a thread's 16 bins and its neighbours' fall into different banks
        struct {
            alignas(16) u64 sel[SELCAP + 64];   // the candidates (+ a place per lane for the stores that store nothing)
            uint16_t slot[SLOTCAP + 64];        // slots (chunk * 256 + thread) whose maximum reaches the bound
        };
    };
    int hist[256];
    int wsum[4];
    int sel_bin;
    int nslot;
    int nsel;
    int last;
};

struct ExpandLds {                          // the expansion
    float q[MAXB * BTV_MAX_NODES + 64];     // q[k*KP + r]: probability of rank r at position k (+ padding: q[..][r+1] is
                                            // fetched, not used, also for the last rank of the last position)
    double cost[BTV_MAX_NODES];             // adaptive budget: estimated cycle latency at budget n + 1
    uint32_t tok[MAXB * BTV_MAX_NODES];     // token ids of the same lists (fetched with q: a read from memory per emitted
                                            // node at the end of the expansion would be one more round trip)
};

// The level-synchronous expansion: pool = the best nodes found so far, in emission order; candidates of one level.
constexpr int LV_CAND = 2048;
constexpr int LV_PAD = 80;                  // zero keys behind a list that is counted over: the reads overrun by up to 66 keys
struct alignas(16) LevelLds {
    alignas(16) u64 ckey[LV_CAND + LV_PAD];
    alignas(16) u64 pkey[2][BTV_MAX_NODES + LV_PAD];   // (+ zero keys behind the pool)
    uint32_t pval[2][BTV_MAX_NODES];
    uint16_t lex2id[BTV_MAX_NODES];         // node id by lexicographic place, for the level whose children are proposed
    uint16_t mark[BTV_MAX_NODES];           // index + 1 of the pool entry whose proposals start at this candidate, else 0
    uint16_t rcap[BTV_MAX_NODES];           // min(K, N / (i + 1))
    int hist[BTV_MAX_NODES + 8];            // proposals that land right behind pool entry i - 1
    int wmax[4];
    uint16_t pos_of[MAXB * BTV_MAX_NODES];  // place in the pool by node id (level, index within the level)
    int off[BTV_MAX_NODES];                 // exclusive scan of the candidates per pool entry
    int cnt_lex[BTV_MAX_NODES];             // nodes of the new level per parent (by the parent's lexicographic place)
    int wsum[4], wsum2[4];
    uint32_t wtop[4];                       // per wavefront: score of its first node of the new level (0: none)
    double dsum[4];
    int n_stop;
};

struct Batch {                              // several requests in one launch (n_nodes == nullptr: one request)
    const int32_t *n_nodes;                 // [batch] budget of each request (device)
    const int32_t *q_offset;                // [batch + 1] first output row of each request (device)
    uint32_t *flag;
};

struct Adaptive {                           // Algorithm 1's early stop (cost == nullptr: fixed budget)
    const double *cost;
    double L_AR;
    double *s_best;
    uint32_t *flag;
};

// sel[0..n): distinct keys; those of rank < K (rank = number of keys above) go to q_row / tok_row (global).
// Threads tid, tid + nthreads, ... take one key each.
__device__ __forceinline__ void rank_keys(const u64 *sel, int n, int K, int KP, float *q_row, uint32_t *tok_row, int tid, int nthreads)
{
    for (int i0 = 0; i0 < n; i0 += 2 * nthreads) {            // two keys per thread at a time
        u64 mine[2];
        int rank[2] = { 0, 0 };
#pragma unroll
        for (int c = 0; c < 2; ++c) mine[c] = i0 + c * nthreads + tid < n ? sel[i0 + c * nthreads + tid] : ~0ull;
        for (int j = 0; j < n; ++j) {
            const u64 kj = sel[j];
#pragma unroll
            for (int c = 0; c < 2; ++c) rank[c] += kj > mine[c] ? 1 : 0;
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
            if (i0 + c * nthreads + tid < n && rank[c] < K) {
                publish(q_row, tok_row, rank[c], __uint_as_float((uint32_t)(mine[c] >> 32)), 0xFFFFFFFFu - (uint32_t)mine[c]);
            }
    }
    for (int i = K + tid; i < KP; i += nthreads) publish(q_row, tok_row, i, 0.f, 0u);
}

// The same for at most 256 keys on a workgroup of 256: a key belongs to T = 1, 2 or 4 neighbouring lanes, which take
// the list's pairs in turn (lane `part` reads pairs part, part + T, ...), two keys per LDS read and eight reads in
// flight; the shares meet by quad swaps.  Every address is the trip's base plus a constant (a compare, a select and
// an address sum per read had been half of the loop's instructions), none of the reads is conditional (the compiler
// would wait for each conditional read on its own), and they run past the end of the list into RANK_PAD zero keys,
// which are above nothing.
constexpr int RANK_PAD = 80;
template <int T>
__device__ __forceinline__ int rank_count(const ulonglong2 *two, int n, int part, u64 mine)
{
    const int pairs = (n + 1) >> 1, per = (pairs + T - 1) / T;
    const ulonglong2 *at = two + part;
    int cnt = 0;
    for (int r = 0; r < per; r += 8, at += 8 * T) {            // (uniform)
        ulonglong2 kk[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) kk[u] = at[u * T];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            cnt += kk[u].x > mine ? 1 : 0;
            cnt += kk[u].y > mine ? 1 : 0;
        }
    }
    return cnt;
}

__device__ __forceinline__ void rank_keys_split(u64 *sel, int n, int K, int KP, float *q_row, uint32_t *tok_row, int tid)
{
    const int lgT = n <= 64 ? 2 : n <= 128 ? 1 : 0, T = 1 << lgT;
    const int i = tid >> lgT, part = tid & (T - 1);
    if (tid < RANK_PAD) sel[n + tid] = 0ull;                   // n <= 256 of the list's 512 places are taken
    __syncthreads();
    const u64 mine = sel[min(i, n)];
    const ulonglong2 *two = reinterpret_cast<const ulonglong2 *>(sel);
    int cnt = lgT == 2 ? rank_count<4>(two, n, part, mine) : lgT == 1 ? rank_count<2>(two, n, part, mine) : rank_count<1>(two, n, part, mine);
    if (T >= 2) cnt += __builtin_amdgcn_update_dpp(0, cnt, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
    if (T == 4) cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
    if (part == 0 && i < n && cnt < K) publish(q_row, tok_row, cnt, __uint_as_float((uint32_t)(mine >> 32)), 0xFFFFFFFFu - (uint32_t)mine);
    for (int e = K + tid; e < KP; e += 256) publish(q_row, tok_row, e, 0.f, 0u);
}

template <typename ForEach>
__device__ __forceinline__ u64 wave_kth_largest(ForEach for_each, int K, int *hist, int lane)
{
    u64 prefix = 0;
    int krem = K;
    for (int byte = 7; byte >= 0; --byte) {
        *reinterpret_cast<int4 *>(&hist[lane * 4]) = make_int4(0, 0, 0, 0);
        __builtin_amdgcn_wave_barrier();
        const int sh = 8 * byte;
        for_each([&](u64 key) {
            if (byte == 7 || (key >> (sh + 8)) == (prefix >> (sh + 8))) atomicAdd(&hist[(int)((key >> sh) & 255)], 1);
        });
        __builtin_amdgcn_wave_barrier();
        const int4 h = *reinterpret_cast<const int4 *>(&hist[lane * 4]);
        const int own = h.x + h.y + h.z + h.w;
        int suf = own;                         // inclusive suffix sum over the higher lanes
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_down(suf, off);
            if (lane + off < 64) suf += o;
        }
        const int above = suf - own;
        int sel = 0, kn = 0;
        const bool here = above < krem && above + own >= krem;
        if (here) {
            int cum = above;
            const int hb[4] = { h.x, h.y, h.z, h.w };
#pragma unroll
            for (int b = 3; b >= 0; --b) {
                if (kn == 0 && cum + hb[b] >= krem) { sel = lane * 4 + b; kn = krem - cum; }
                cum += hb[b];
            }
        }
        const int srcl = __builtin_ctzll(__builtin_amdgcn_ballot_w64(here));
        sel = __builtin_amdgcn_readlane(sel, srcl);
        krem = __builtin_amdgcn_readlane(kn, srcl);
        prefix |= (u64)sel << sh;
        __builtin_amdgcn_wave_barrier();
    }
    return prefix;
}

template <typename ForEach>
__device__ __forceinline__ void wave_select_rank(ForEach for_each, int K, int KP, int *hist, u64 *sel, int *nsel, float *q_row,
                                                 uint32_t *tok_row, int lane)
{
    const u64 kth = wave_kth_largest(for_each, K, hist, lane);
    if (lane == 0) *nsel = 0;
    __builtin_amdgcn_wave_barrier();
    for_each([&](u64 key) {
        if (key >= kth) {
            const int pos = atomicAdd(nsel, 1);
            if (pos < SELCAP) sel[pos] = key;                  // exactly K keys: they are distinct
        }
    });
    __builtin_amdgcn_wave_barrier();
    rank_keys(sel, K, K, KP, q_row, tok_row, lane, 64);
}

// ------------------------------------------------------------------------------------------------
// Step 3, part B: the expansion, one wavefront, the frontier in registers.
// A single wavefront issues an instruction every few cycles at best, so the loop is written for few instructions
// per emitted node rather than for parallel work.
// A frontier entry stands for "the children of one node, from rank r on".  The entry for the children of node i
// lives in slot i + 1 (slot 0: the children of the root), slot s = lane s % 64 of register row s / 64; slots are
// never reused, so no search for a free one is needed and the parent of an entry is its slot number minus one.
// Per entry: key = bits(rho of rank r) + 1 (0 = empty or exhausted), rho of the parent, x = LDS address of
// q[depth-1][r] (depth and r are read back from it: KP is a power of two), and qn = q[depth-1][r+1], the
// probability of the next sibling (every lane re-reads qn after every pop: one gather, whose latency is off the
// critical path because qn is used one pop later at the earliest).  Popping an entry emits (parent, depth, r)
// and advances the entry in place to rank r + 1; the emitted node's own children become the entry of the next
// slot.  Emitted node i is kept in lane i % 64 of row i / 64 as rec = index of q[depth-1][r] | slot << 13.
// Order of emission: rho desc, depth asc, rank path lexicographic asc.  The wave maximum of the keys decides
// almost always; on ties the depth decides, then the rank paths, rebuilt by walking the parents of the tied
// entries through the emitted nodes.
// ------------------------------------------------------------------------------------------------
// ADAPT: the budget is chosen online (Sec. 3.4, Eq. 6): with Ahat summed in fp64 in emission order, the popped node
// is kept only while Ahat(N) * L_AR / C(N) strictly improves, compared as Ahat(N) * C(N*) > Ahat(N*) * C(N).
// An empty volatile asm in the body of a wave-uniform `if` keeps it a real (scalar) branch: with several register
// rows the compiler would otherwise turn the row selection into select chains over every row, which costs more
// instructions than the branches do.
#define BTV_KEEP_BRANCH() asm volatile("" ::: "memory")

template <int R, bool ADAPT>
__device__ __forceinline__ void expand_wave(ExpandLds &S, int B, int K, int KP, int N, int lane, int32_t *parent, int32_t *token,
                                            int32_t *depth, float *rho, int32_t *n_out, float *ahat, const Adaptive &ad)
{
    const float *q_s = S.q;
    const uint32_t q_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)q_s;
    const int lg = 31 - __builtin_clz((unsigned)KP);           // KP = 1 << lg
    const float qfirst = lane < B ? q_s[lane * KP] : 0.f;      // lane k: probability of the best token at position k
    uint32_t e_key[R], e_x[R], o_rec[R];
    float e_prho[R], e_qn[R], o_rho[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { e_key[r] = 0u; e_prho[r] = 0.f; e_qn[r] = 0.f; e_x[r] = q_base; o_rec[r] = 0u; o_rho[r] = 0.f; }
    if (lane == 0) {       // slot 0: the children of the root
        e_key[0] = __float_as_uint(__fmul_rn(1.0f, q_s[0])) + 1u;
        e_qn[0] = q_s[1];                                      // padding when K == 1: never used
        e_prho[0] = 1.0f;
    }
    int n = 0;
    double run_a = 1.0, best_a = 0.0, best_c = 0.0;            // Ahat so far; Ahat and cost at the best budget so far
    bool stop = false;
    // Slots are handed out in node order, so before node 64*RA - 1 is emitted only the first RA register rows can
    // hold anything: the loop runs in phases over RA = 1..R, each compiled for its number of live rows.
    auto phase = [&](auto ra_c, int n_end) {
        constexpr int RA = decltype(ra_c)::value;
        while (n < n_end) {
            double c_n = 0.0;
            if (ADAPT) c_n = S.cost[n];                            // fetched early: used after the wave maximum
            uint32_t lm = e_key[0];
    #pragma unroll
            for (int r = 1; r < RA; ++r) lm = umax(lm, e_key[r]);
            const uint32_t m = wave_max_u32(lm);
            if (__builtin_expect(m == 0u, 0)) { stop = true; break; }     // frontier empty: the lattice is exhausted
            if (ADAPT) {
                const double a_new = run_a + (double)__uint_as_float(m - 1u);
                if (__builtin_expect(!(c_n > 0.0), 0)) {           // invalid cost: stop here and tell
                    if (lane == 0) atomicOr(ad.flag, 4u);
                    stop = true;
                    break;
                }
                if (n > 0 && !(a_new * best_c > best_a * c_n)) { stop = true; break; }   // the estimated speedup did not improve
                run_a = a_new; best_a = a_new; best_c = c_n;
            }
            u64 al[RA];
            int cnt = 0;
    #pragma unroll
            for (int r = 0; r < RA; ++r) { al[r] = __builtin_amdgcn_ballot_w64(e_key[r] == m); cnt += __builtin_popcountll(al[r]); }
            if (__builtin_expect(cnt > 1, 0)) {
                // ties on rho: shallower first (x grows with the depth) ...
                uint32_t cl = 0u;
    #pragma unroll
                for (int r = 0; r < RA; ++r)
                    if ((al[r] >> lane) & 1ull) cl = umax(cl, 0x100u - ((e_x[r] - q_base) >> (2 + lg)));
                const uint32_t cm = wave_max_u32(cl);
                cnt = 0;
    #pragma unroll
                for (int r = 0; r < RA; ++r) {
                    al[r] = __builtin_amdgcn_ballot_w64(((al[r] >> lane) & 1ull) && 0x100u - ((e_x[r] - q_base) >> (2 + lg)) == cm);
                    cnt += __builtin_popcountll(al[r]);
                }
                if (cnt > 1) {
                    // ... then the smaller rank path: one byte per position, first position in the most significant
                    // byte of word 0; the walk fetches the emitted ancestors from the lanes that hold them
                    uint32_t path[RA][4];
    #pragma unroll
                    for (int r = 0; r < RA; ++r) {
    #pragma unroll
                        for (int w = 0; w < 4; ++w) path[r][w] = 0u;
                    }
    #pragma unroll
                    for (int r = 0; r < RA; ++r) {                  // every lane walks, tied or not: the fetches are wave-wide
                        uint32_t idx = (e_x[r] - q_base) >> 2;     // index of q[depth-1][rank]
                        int node = r * 64 + lane - 1;              // the entry's parent
                        bool live = (al[r] >> lane) & 1ull;
                        while (__builtin_amdgcn_ballot_w64(live) != 0ull) {
                            const int pos = (int)(idx >> lg), sh = 24 - 8 * (pos & 3);
                            const uint32_t byte = (idx & (uint32_t)(KP - 1)) << sh;
                            if (live) {
    #pragma unroll
                                for (int w = 0; w < 4; ++w) if (w == (pos >> 2)) path[r][w] |= byte;
                            }
                            live = live && node >= 0;
                            const int src = node >= 0 ? node : 0;
                            uint32_t rec = 0u;
    #pragma unroll
                            for (int rr = 0; rr < RA; ++rr) {
                                const uint32_t got = (uint32_t)__shfl((int)o_rec[rr], src & 63);
                                if (rr == (src >> 6)) rec = got;
                            }
                            idx = rec & 0x1FFFu;
                            node = (int)(rec >> 13) - 1;
                        }
                    }
    #pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        if (cnt <= 1) break;
                        uint32_t pl = 0u;
    #pragma unroll
                        for (int r = 0; r < RA; ++r)
                            if ((al[r] >> lane) & 1ull) pl = umax(pl, ~path[r][w]);
                        const uint32_t pm = wave_max_u32(pl);
                        cnt = 0;
    #pragma unroll
                        for (int r = 0; r < RA; ++r) {
                            al[r] = __builtin_amdgcn_ballot_w64(((al[r] >> lane) & 1ull) && ~path[r][w] == pm);
                            cnt += __builtin_popcountll(al[r]);
                        }
                    }
                }
            }
            int wr = 0;
    #pragma unroll
            for (int r = RA - 1; r >= 1; --r) if (al[r] != 0ull) wr = r;
            if (al[0] != 0ull) wr = 0;
            u64 alw = al[0];
            uint32_t s_x = e_x[0];
    #pragma unroll
            for (int r = 1; r < RA; ++r)
                if (r == wr) { alw = al[r]; s_x = e_x[r]; }
            const int wl = __builtin_ctzll(alw);
            const uint32_t u_idx = (__builtin_amdgcn_readlane(s_x, wl) - q_base) >> 2;
            const float u_rho = __uint_as_float(m - 1u);
            const int d = (int)(u_idx >> lg) + 1, rank = u_idx & (uint32_t)(KP - 1);
            // emit node n into its lane
            {
                const uint32_t rec = u_idx | ((uint32_t)(wr * 64 + wl) << 13);     // parent + 1 = the entry's slot
    #pragma unroll
                for (int r = 0; r < RA; ++r)
                    if (r == (n >> 6)) {                           // wave-uniform
                        BTV_KEEP_BRANCH();
                        const bool me = lane == (n & 63);
                        o_rec[r] = me ? rec : o_rec[r];
                        o_rho[r] = me ? u_rho : o_rho[r];
                    }
            }
            // the entry moves on to the next sibling, in its own lane
            const bool has_next = rank + 1 < K;
    #pragma unroll
            for (int r = 0; r < RA; ++r)
                if (r == wr) {                                     // wave-uniform
                    BTV_KEEP_BRANCH();
                    const bool me = lane == wl;
                    const uint32_t nk = has_next ? __float_as_uint(__fmul_rn(e_prho[r], e_qn[r])) + 1u : 0u;
                    e_key[r] = me ? nk : e_key[r];
                    e_x[r] += me ? 4u : 0u;
                }
            // the emitted node's children: the entry of slot n + 1 (a slot past the last row is simply not written)
            if (d < B) {
                const int cs = n + 1;
                const float q_child = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(qfirst), d));
                const uint32_t key_child = __float_as_uint(__fmul_rn(u_rho, q_child)) + 1u;
                const uint32_t x_child = q_base + ((uint32_t)d << (2 + lg));
    #pragma unroll
                for (int r = 0; r < RA; ++r)
                    if (r == (cs >> 6)) {                          // wave-uniform
                        BTV_KEEP_BRANCH();
                        const bool me = lane == (cs & 63);
                        e_key[r] = me ? key_child : e_key[r];
                        e_prho[r] = me ? u_rho : e_prho[r];
                        e_x[r] = me ? x_child : e_x[r];
                    }
            }
    #pragma unroll
            for (int r = 0; r < RA; ++r)
                e_qn[r] = *reinterpret_cast<const __attribute__((address_space(3))) float *>((uintptr_t)(e_x[r] + 4u));
            ++n;
        }
    };
    phase(std::integral_constant<int, 1>{}, min(N, 63));
    if (R >= 2 && !stop) phase(std::integral_constant<int, (R >= 2 ? 2 : 1)>{}, min(N, 127));
    if (R >= 3 && !stop) phase(std::integral_constant<int, (R >= 3 ? 3 : 1)>{}, min(N, 191));
    if (R >= 4 && !stop) phase(std::integral_constant<int, (R >= 4 ? 4 : 1)>{}, N);
    if (R < 4 && !stop) phase(std::integral_constant<int, R>{}, N);
    double a = 0.0;                  // the surrogate: summed in fp64 and rounded once
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * 64 + lane;
        if (i < n) {
            const uint32_t idx = o_rec[r] & 0x1FFFu;
            token[i] = (int32_t)S.tok[idx];
            parent[i] = (int32_t)(o_rec[r] >> 13) - 1;
            if (depth) depth[i] = (int)(idx >> lg) + 1;
            if (rho) rho[i] = o_rho[r];
            a += (double)o_rho[r];
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);
    if (lane == 0) {
        *n_out = n;
        if (ahat) *ahat = ADAPT ? (float)run_a : (float)(1.0 + a);
        if (ADAPT && ad.s_best) *ad.s_best = n > 0 ? best_a * ad.L_AR / best_c : -INFINITY;
    }
}

// ------------------------------------------------------------------------------------------------
// Step 3, part B'': the same tree, level by level, on the whole workgroup.
// The emission order (rho desc, depth asc, rank path asc) is a total order of the lattice in which a node comes
// after its parent and after its elder siblings, so the tree is the set of the N first prefixes of that order and
// the emission order is that order: nothing about it needs the frontier.  Level d of the tree is among the
// children of the level d-1 nodes kept so far.  The pool holds the best N nodes found up to the level before, in
// order; every pool node of depth d-1 proposes its children of rank r < min(K, N / (i + 1)), i being its place
// among the depth d-1 nodes (the child is preceded by the (i+1)(r+1) children of rank <= r of the parents up to its
// own), cut further at the score of the pool's last node once the pool is full.  Up to 256 proposals (the rule
// once the pool is full) are placed by counting: one per thread, its new place = the proposals above it + the pool
// nodes above it; more are sorted (bitonic, 64-bit keys, in LDS) and merged into the pool by binary searches from
// both sides.  The loop ends at depth B or when a level proposes nothing.
// Key of a node = bits(rho) << 32 | (31 - depth) << 16 | (0xFFFF - lexkey); lexkey = place of the parent in the
// lexicographic order of its level * KP + rank, which orders the nodes of one level by rank path; the place of a
// new node in that order is the number of level nodes under parents before its parent, plus its rank (siblings
// in the pool are always ranks 0 .. c-1).  Value = node id (level - 1) * 256 + place within the level | id of the
// parent << 12 | lexicographic place << 24; places within a level never change once assigned, because the pool
// only ever loses its last nodes.
// A level costs a few microseconds whatever it holds, a node of the one-wavefront expansion a quarter to half a
// microsecond whatever the tree looks like: the host of this function picks by the depth the tree can reach.
// ------------------------------------------------------------------------------------------------
// Bitonic sort of P2 (a power of two, at least 128) 64-bit keys in LDS, largest first, by 256 threads.  Every
// compare-exchange at a distance below 128 happens in registers: a wavefront holds a block of 128 keys two per lane
// (key e * 64 + lane of the block in register e), distance 64 pairs a lane's own two registers, shorter distances pair
// lanes (the network is unrolled, every stage takes the cross-lane move that fits its distance).  Only the distances from 128 up go through LDS, one block barrier
// each.  base = index of the block's first key in the whole array: it fixes each pair's direction.
// x of lane (l ^ J) for J = 1 .. 32, on the vector ALU alone: quad permutes for 1 and 2, two row shifts (each written
// to the banks of four lanes it is right for) for 4 and 8, the row / half-wave swaps for 16 and 32.  The same data
// through ds_bpermute costs a trip through the LDS crossbar per 32 bits and stage.
template <int J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int lane)
{
    const int v = (int)x;
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false);      // quad_perm [1,0,3,2]
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false); // quad_perm [2,3,0,1]
    else if constexpr (J == 4) {
        const int t = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xF, 0x5, false);                  // row_shl:4 -> lanes with bit 2 clear
        return (uint32_t)__builtin_amdgcn_update_dpp(t, v, 0x114, 0xF, 0xA, false);               // row_shr:4 -> lanes with bit 2 set
    } else if constexpr (J == 8) {
        const int t = __builtin_amdgcn_update_dpp(v, v, 0x108, 0xF, 0x3, false);                  // row_shl:8 -> lanes 0-7 of a row
        return (uint32_t)__builtin_amdgcn_update_dpp(t, v, 0x118, 0xF, 0xC, false);               // row_shr:8 -> lanes 8-15
    } else if constexpr (J == 16) {
        const auto sw = __builtin_amdgcn_permlane16_swap(x, x, false, false);                       // odd rows of [0] <-> even rows of [1]
        return (lane & 16) ? sw[0] : sw[1];
    } else {
        const auto sw = __builtin_amdgcn_permlane32_swap(x, x, false, false);                       // upper half of [0] <-> lower half of [1]
        return (lane & 32) ? sw[0] : sw[1];
    }
}

// One compare-exchange stage at distance J of the bitonic network over a block of 128 keys (two per lane); kbit = the
// merge size the stage belongs to (its bit of a key's index gives the direction).
template <int J>
__device__ __forceinline__ void wave_stage(u64 &k0, u64 &k1, int base, int kbit, int lane)
{
    if constexpr (J == 64) {
        const bool desc = ((base + lane) & kbit) == 0;
        const u64 hi = k0 > k1 ? k0 : k1, lo = k0 > k1 ? k1 : k0;
        k0 = desc ? hi : lo;
        k1 = desc ? lo : hi;
    } else {
        const bool lower = (lane & J) == 0;                       // this lane holds the pair's lower index
        const u64 p0 = ((u64)lane_xor<J>((uint32_t)(k0 >> 32), lane) << 32) | lane_xor<J>((uint32_t)k0, lane);
        const u64 p1 = ((u64)lane_xor<J>((uint32_t)(k1 >> 32), lane) << 32) | lane_xor<J>((uint32_t)k1, lane);
        const bool max0 = lower == (((base + lane) & kbit) == 0), max1 = lower == (((base + 64 + lane) & kbit) == 0);
        k0 = (max0 == (k0 > p0)) ? k0 : p0;
        k1 = (max1 == (k1 > p1)) ? k1 : p1;
    }
}

// the stages of one merge of size kbit, from distance J down to 1
template <int J>
__device__ __forceinline__ void wave_merge(u64 &k0, u64 &k1, int base, int kbit, int lane)
{
    wave_stage<J>(k0, k1, base, kbit, lane);
    if constexpr (J > 1) wave_merge<J / 2>(k0, k1, base, kbit, lane);
}

// the whole network on one block of 128: merges of size 2, 4, ..., 128
template <int K>
__device__ __forceinline__ void wave_sort(u64 &k0, u64 &k1, int base, int lane)
{
    if constexpr (K > 2) wave_sort<K / 2>(k0, k1, base, lane);
    wave_merge<K / 2>(k0, k1, base, K, lane);
}

__device__ __forceinline__ void bitonic_desc(u64 *key, int P2, int tid)
{
    const int lane = tid & 63, w = tid >> 6;
    __syncthreads();
    for (int blk = w; blk * 128 < P2; blk += 4) {                  // every block of 128 sorted on its own
        u64 k0 = key[blk * 128 + lane], k1 = key[blk * 128 + 64 + lane];
        wave_sort<128>(k0, k1, blk * 128, lane);
        key[blk * 128 + lane] = k0;
        key[blk * 128 + 64 + lane] = k1;
    }
    for (int k = 256; k <= P2; k <<= 1) {
        for (int j = k >> 1; j >= 128; j >>= 1) {
            __syncthreads();
            for (int idx = tid; idx < P2 / 2; idx += 256) {
                const int i1 = 2 * idx - (idx & (j - 1)), i2 = i1 + j;
                const u64 a = key[i1], b = key[i2];
                if ((a < b) == ((i1 & k) == 0)) { key[i1] = b; key[i2] = a; }
            }
        }
        __syncthreads();
        for (int blk = w; blk * 128 < P2; blk += 4) {
            u64 k0 = key[blk * 128 + lane], k1 = key[blk * 128 + 64 + lane];
            wave_merge<64>(k0, k1, blk * 128, k, lane);
            key[blk * 128 + lane] = k0;
            key[blk * 128 + 64 + lane] = k1;
        }
    }
    __syncthreads();
}

template <bool ADAPT>
__device__ __forceinline__ void expand_levels(ExpandLds &S, LevelLds &L, int B, int K, int KP, int N, int tid, int32_t *parent,
                                              int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat,
                                              const Adaptive &ad)
{
    const int lane = tid & 63, w = tid >> 6;
    const int lg = 31 - __builtin_clz((unsigned)KP);
    const u64 below = (1ull << lane) - 1ull;
    int cur = 0, np = min(K, N);
    L.rcap[tid] = (uint16_t)min(K, N / (tid + 1));
    if (tid < np) {                                            // level 1: the K best tokens of position 0, already in order
        L.pkey[0][tid] = ((u64)__float_as_uint(__fmul_rn(1.0f, S.q[tid])) << 32) | (30u << 16) | (0xFFFFu - (uint32_t)tid);
        L.pval[0][tid] = (uint32_t)tid | (0xFFFu << 12) | ((uint32_t)tid << 24);
        L.lex2id[tid] = (uint16_t)tid;
    }
    if (tid < LV_PAD) L.pkey[0][np + tid] = 0ull;         // the zero keys behind the pool
    __syncthreads();
    // No LDS read of the loop sits behind a lane-dependent branch (the compiler would wait for each on its own):
    // lanes without work read place 0 and drop the result.  The searches run a fixed, wave-uniform number of steps.
    const int search_steps = 32 - __builtin_clz((unsigned)min(K, N));
    uint32_t top = __float_as_uint(__fmul_rn(1.0f, S.q[0]));   // the largest score among the nodes of the level before d
    for (int d = 2; d <= B; ++d) {
        // ---- how many children each pool node of depth d-1 proposes ------------------------------------------------
        const float *qd = S.q + (d - 1) * KP;
        const u64 k = L.pkey[cur][tid < np ? tid : 0];
        const uint32_t v = L.pval[cur][tid < np ? tid : 0];
        const uint32_t g32 = (uint32_t)(L.pkey[cur][N - 1] >> 32);   // the pool's last score (read, not used, before the pool is full)
        // The pool is full and not even the best child of the level's best node reaches its last score (the product
        // rises with the parent's score): nobody proposes anything, as the counts below would find out at the cost
        // of a search per parent.
        if (np == N && __float_as_uint(__fmul_rn(__uint_as_float(top), qd[0])) < g32) break;      // (uniform)
        const int rcap = L.rcap[v & 0xFFu];
        const float rp = __uint_as_float((uint32_t)(k >> 32));
        int c = tid < np && 31 - (int)((k >> 16) & 31u) == d - 1 ? rcap : 0;
        if (np == N) {                                         // only scores that reach the pool's last node; they fall with the rank
            int lo = 0, hi = c;
            for (int st = 0; st < search_steps; ++st) {
                const int mid = (lo + hi) >> 1;
                const bool ge = __float_as_uint(__fmul_rn(rp, qd[mid])) >= g32;
                const bool open = lo < hi;
                lo = open && ge ? mid + 1 : lo;
                hi = open && !ge ? mid : hi;
            }
            c = lo;
        }
        const int incl = wave_incl_scan(c);
        if (lane == 63) L.wsum[w] = incl;
        L.mark[tid] = 0;
        L.hist[tid] = 0;
        if (tid == 0) L.hist[BTV_MAX_NODES] = 0;
        __syncthreads();
        const int ws0 = L.wsum[0], ws1 = L.wsum[1], ws2 = L.wsum[2], ws3 = L.wsum[3];
        const int base = (w > 0 ? ws0 : 0) + (w > 1 ? ws1 : 0) + (w > 2 ? ws2 : 0);
        const int C = ws0 + ws1 + ws2 + ws3;
        const int off = base + incl - c;
        L.off[tid] = off;
        if (C == 0) break;                                     // (uniform)
        if (C > LV_CAND) {                                     // cannot happen (sum over i of N / (i+1) <= 1570 at N = 256)
            if (tid == 0) atomicOr(ad.flag, 8u);
            break;
        }
        const int nxt = cur ^ 1;
        if (C <= 256) {
            // ---- few proposals: one per thread, placed by counting ---------------------------------------------------
            // Candidate j belongs to the last pool entry whose offset does not exceed j: the entries mark where their
            // proposals start and a running maximum carries the marks along.
            if (c > 0) L.mark[off] = (uint16_t)(tid + 1);
            __syncthreads();
            const int mk = wave_incl_max((int)L.mark[tid]);
            if (lane == 63) L.wmax[w] = mk;
            __syncthreads();
            const int wm0 = L.wmax[0], wm1 = L.wmax[1], wm2 = L.wmax[2];
            const int carry = max(max(w > 0 ? wm0 : 0, w > 1 ? wm1 : 0), w > 2 ? wm2 : 0);
            const bool live = tid < C;
            const int pe = live ? max(mk, carry) - 1 : 0;
            const int r = live ? tid - L.off[pe] : 0;
            const u64 pk = L.pkey[cur][pe];
            const uint32_t plex = L.pval[cur][pe] >> 24;
            const uint32_t sc = __float_as_uint(__fmul_rn(__uint_as_float((uint32_t)(pk >> 32)), qd[r]));
            L.ckey[tid] = live ? ((u64)sc << 32) | ((uint32_t)(31 - d) << 16) | (0xFFFFu - ((plex << lg) + (uint32_t)r)) : 0ull;
            if (tid < LV_PAD) L.ckey[256 + tid] = 0ull;        // with the zeros from C on: the zero keys behind the list
            __syncthreads();
            // A candidate's new place = the candidates above it + the pool nodes above it, both counted (T = 1, 2 or 4
            // neighbouring lanes share a candidate, two keys per LDS read, eight reads in flight); a pool node moves
            // down by the candidates above it = the candidates with at most its own place in pool nodes above them.
            const int lgT = C <= 64 ? 2 : C <= 128 ? 1 : 0, T = 1 << lgT;
            const int ci = tid >> lgT, part = tid & (T - 1);
            const u64 mine = L.ckey[ci];                        // zero from C on: never placed
            const uint32_t cval = (uint32_t)L.lex2id[(0xFFFFu - (uint32_t)(mine & 0xFFFFu)) >> lg] << 12;
            const ulonglong2 *two = reinterpret_cast<const ulonglong2 *>(L.ckey);
            const ulonglong2 *ptwo = reinterpret_cast<const ulonglong2 *>(L.pkey[cur]);
            // The T lanes of a candidate take the pairs of a list in turn (lane `part` reads pairs part, part + T, ...),
            // eight reads in flight, every address the trip's base plus a constant: with a compare, a select and an
            // address sum per read the loop spent half its instructions on addresses.  The reads run past the list's
            // end into LV_PAD zero keys, which are above nothing.
            auto count_above = [&](auto t_c, const ulonglong2 *list, int n) {
                constexpr int TT = decltype(t_c)::value;
                const int pairs = (n + 1) >> 1, per = (pairs + TT - 1) / TT;
                const ulonglong2 *at = list + part;
                int cnt = 0;
                for (int q = 0; q < per; q += 8, at += 8 * TT) {          // (uniform)
                    ulonglong2 kk[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) kk[u] = at[u * TT];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        cnt += kk[u].x > mine ? 1 : 0;
                        cnt += kk[u].y > mine ? 1 : 0;
                    }
                }
                return cnt;
            };
            auto count_list = [&](const ulonglong2 *list, int n) {
                if (lgT == 2) return count_above(std::integral_constant<int, 4>{}, list, n);
                if (lgT == 1) return count_above(std::integral_constant<int, 2>{}, list, n);
                return count_above(std::integral_constant<int, 1>{}, list, n);
            };
            int above_c = count_list(two, C), above_p = 0;
            if (np <= 128) {
                above_p = count_list(ptwo, np);
            } else if (part == 0) {                            // a long pool: binary search, by the candidate's first lane
                int lo = 0, hi = np;
                for (int st = 0; st < 9; ++st) {
                    const int mid = (lo + hi) >> 1;
                    const bool gt = L.pkey[cur][mid] > mine;
                    const bool open = lo < hi;
                    lo = open && gt ? mid + 1 : lo;
                    hi = open && !gt ? mid : hi;
                }
                above_p = lo;
            }
            if (T >= 2) {
                above_c += __builtin_amdgcn_update_dpp(0, above_c, 0xB1, 0xF, 0xF, false);
                above_p += __builtin_amdgcn_update_dpp(0, above_p, 0xB1, 0xF, 0xF, false);
            }
            if (T == 4) {
                above_c += __builtin_amdgcn_update_dpp(0, above_c, 0x4E, 0xF, 0xF, false);
                above_p += __builtin_amdgcn_update_dpp(0, above_p, 0x4E, 0xF, 0xF, false);
            }
            if (part == 0 && ci < C) {
                atomicAdd(&L.hist[above_p], 1);
                if (above_c + above_p < N) {
                    L.pkey[nxt][above_c + above_p] = mine;
                    L.pval[nxt][above_c + above_p] = cval;
                }
            }
            __syncthreads();
            const int hs = wave_incl_scan(L.hist[tid]);
            if (lane == 63) L.wsum2[w] = hs;
            __syncthreads();
            const int h0 = L.wsum2[0], h1 = L.wsum2[1], h2 = L.wsum2[2];
            const int moved = hs + (w > 0 ? h0 : 0) + (w > 1 ? h1 : 0) + (w > 2 ? h2 : 0);
            if (tid < np && tid + moved < N) { L.pkey[nxt][tid + moved] = k; L.pval[nxt][tid + moved] = v; }
        } else {
            __syncthreads();
            // ---- the proposals: candidate j belongs to the last pool entry whose offset does not exceed j -----------
            int P2 = 512;
            while (P2 < C) P2 <<= 1;
            for (int j = tid; j < P2; j += 256) {
                u64 key = 0ull;
                if (j < C) {
                    int lo = 0, hi = np;                       // first entry with off > j
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (L.off[mid] <= j) lo = mid + 1; else hi = mid;
                    }
                    const int pe = lo - 1, r = j - L.off[pe];
                    const u64 pk = L.pkey[cur][pe];
                    const uint32_t sc = __float_as_uint(__fmul_rn(__uint_as_float((uint32_t)(pk >> 32)), qd[r]));
                    key = ((u64)sc << 32) | ((uint32_t)(31 - d) << 16) | (0xFFFFu - (((L.pval[cur][pe] >> 24) << lg) + (uint32_t)r));
                }
                L.ckey[j] = key;
            }
            bitonic_desc(L.ckey, P2, tid);
            // ---- merge: a node's new place = its place in its own list + the nodes of the other list ahead of it ----
            for (int j = tid; j < C; j += 256) {
                const u64 ck = L.ckey[j];
                int lo = 0, hi = np;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (L.pkey[cur][mid] > ck) lo = mid + 1; else hi = mid;
                }
                if (j + lo < N) {
                    L.pkey[nxt][j + lo] = ck;
                    L.pval[nxt][j + lo] = (uint32_t)L.lex2id[(0xFFFFu - (uint32_t)(ck & 0xFFFFu)) >> lg] << 12;
                }
            }
            if (tid < np) {
                int lo = 0, hi = C;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (L.ckey[mid] > k) lo = mid + 1; else hi = mid;
                }
                if (tid + lo < N) { L.pkey[nxt][tid + lo] = k; L.pval[nxt][tid + lo] = v; }
            }
        }
        L.cnt_lex[tid] = 0;
        np = min(np + C, N);
        cur = nxt;
        if (tid < LV_PAD) L.pkey[cur][np + tid] = 0ull;
        __syncthreads();
        // ---- the new level's nodes get their id and their lexicographic place --------------------------------------
        const u64 k2 = L.pkey[cur][tid < np ? tid : 0];
        const bool mine2 = tid < np && 31 - (int)((k2 >> 16) & 31u) == d;
        const uint32_t lexkey = 0xFFFFu - (uint32_t)(k2 & 0xFFFFu);
        const u64 bal = __builtin_amdgcn_ballot_w64(mine2);
        {   // the pool is in falling order: a wavefront's first node of the new level is its best
            const uint32_t first = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(k2 >> 32), bal != 0ull ? __builtin_ctzll(bal) : 0);
            if (lane == 0) { L.wsum2[w] = __builtin_popcountll(bal); L.wtop[w] = bal != 0ull ? first : 0u; }
        }
        if (mine2) atomicAdd(&L.cnt_lex[lexkey >> lg], 1);
        __syncthreads();
        top = umax(umax(L.wtop[0], L.wtop[1]), umax(L.wtop[2], L.wtop[3]));
        const int p0 = L.wsum2[0], p1 = L.wsum2[1], p2 = L.wsum2[2];
        const int place = __builtin_popcountll(bal & below) + (w > 0 ? p0 : 0) + (w > 1 ? p1 : 0) + (w > 2 ? p2 : 0);
        const int cl = L.cnt_lex[tid];
        const int il = wave_incl_scan(cl);
        if (lane == 63) L.wsum[w] = il;
        __syncthreads();
        const int l0 = L.wsum[0], l1 = L.wsum[1], l2 = L.wsum[2];
        L.cnt_lex[tid] = il - cl + (w > 0 ? l0 : 0) + (w > 1 ? l1 : 0) + (w > 2 ? l2 : 0);
        __syncthreads();
        const uint32_t lexpos = (uint32_t)L.cnt_lex[mine2 ? lexkey >> lg : 0] + (lexkey & (uint32_t)(KP - 1));
        const uint32_t pv2 = L.pval[cur][tid < np ? tid : 0];
        if (mine2) {
            L.pval[cur][tid] = (uint32_t)((d - 1) * 256 + place) | (pv2 & 0x00FFF000u) | (lexpos << 24);
            L.lex2id[lexpos] = (uint16_t)((d - 1) * 256 + place);
        }
        __syncthreads();
    }
    __syncthreads();
    // ---- the pool is the tree, in emission order ---------------------------------------------------------------------
    int n = np;
    if (ADAPT) {
        // Sec. 3.4, Eq. 6: the budget stops at the first node that does not improve Ahat(n) * L_AR / C(n); Ahat is summed
        // in emission order in fp64, by one thread
        if (tid == 0) {
            double run_a = 1.0, best_a = 0.0, best_c = 0.0;
            int m = 0;
            for (; m < np; ++m) {
                const double c_n = S.cost[m];
                const double a_new = run_a + (double)__uint_as_float((uint32_t)(L.pkey[cur][m] >> 32));
                if (!(c_n > 0.0)) { atomicOr(ad.flag, 4u); break; }
                if (m > 0 && !(a_new * best_c > best_a * c_n)) break;
                run_a = a_new; best_a = a_new; best_c = c_n;
            }
            L.n_stop = m;
            *n_out = m;
            if (ahat) *ahat = (float)run_a;
            if (ad.s_best) *ad.s_best = m > 0 ? best_a * ad.L_AR / best_c : -INFINITY;
        }
        __syncthreads();
        n = L.n_stop;
    }
    if (tid < np) L.pos_of[L.pval[cur][tid] & 0xFFFu] = (uint16_t)tid;
    __syncthreads();
    double a = 0.0;
    if (tid < n) {
        const u64 k = L.pkey[cur][tid];
        const uint32_t v = L.pval[cur][tid];
        const int dep = 31 - (int)((k >> 16) & 31u);
        const uint32_t lexkey = 0xFFFFu - (uint32_t)(k & 0xFFFFu);
        const int idx = (dep - 1) * KP + (int)(lexkey & (uint32_t)(KP - 1));
        const uint32_t pu = (v >> 12) & 0xFFFu;
        const float r = __uint_as_float((uint32_t)(k >> 32));
        token[tid] = (int32_t)S.tok[idx];
        parent[tid] = pu == 0xFFFu ? -1 : (int32_t)L.pos_of[pu];
        if (depth) depth[tid] = dep;
        if (rho) rho[tid] = r;
        a = (double)r;
    }
    if (!ADAPT) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);
        if (lane == 0) L.dsum[w] = a;
        __syncthreads();
        if (tid == 0) {
            *n_out = n;
            if (ahat) *ahat = (float)(1.0 + ((L.dsum[0] + L.dsum[1]) + (L.dsum[2] + L.dsum[3])));
        }
    }
}

// Workgroup `row` ranks the candidates of its position into top_q / top_tok (global, [B][KP]); the workgroup that
// finishes last then runs the expansion on its first wavefront.
// ------------------------------------------------------------------------------------------------
// Step 3, part B': the beam-search tree (Sec. 4.3's comparison topology): depth by depth, the `width` extensions
// with the largest path score among all extensions of the prefixes kept at the previous depth.  Only the `width`
// best tokens of a position can be kept (an extension of rank r is preceded by r extensions of the same prefix),
// so a depth has at most width * width <= 256 candidates: one per thread, ranked by counting.  Order within a
// depth: rho desc, then the parent's place in the previous depth, then the token's rank.
// ------------------------------------------------------------------------------------------------
constexpr int MAXW = 16;

struct BeamLds {
    u64 key[MAXW * MAXW];
    float rho[2][MAXW];
    int node[2][MAXW];
    double part[4];
};

__device__ __forceinline__ void beam_block(const ExpandLds &S, BeamLds &Bm, int depth_max, int K, int KP, int width, int tid,
                                           int32_t *parent, int32_t *token, int32_t *depth, float *rho, int32_t *n_out,
                                           float *ahat)
{
    int n = 0, kept = 1;                                    // nodes so far, prefixes kept at the previous depth
    double mine_sum = 0.0;
    if (tid == 0) { Bm.rho[0][0] = 1.f; Bm.node[0][0] = -1; }
    __syncthreads();
    for (int k = 0; k < depth_max; ++k) {
        const int cur = k & 1, nc = kept * K, keep = min(nc, width);
        const int b = tid / K, rk = tid - b * K;            // candidate tid = (kept prefix b, rank rk)
        float r = 0.f;
        u64 mine = 0;
        if (tid < nc) {
            r = __fmul_rn(Bm.rho[cur][b], S.q[k * KP + rk]);
            mine = ((u64)__float_as_uint(r) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)tid);
            Bm.key[tid] = mine;
        }
        __syncthreads();
        if (tid < nc) {
            int rank = 0;
            for (int j = 0; j < nc; ++j) rank += Bm.key[j] > mine ? 1 : 0;
            if (rank < keep) {
                const int nd = n + rank;
                parent[nd] = Bm.node[cur][b];
                token[nd] = (int32_t)S.tok[k * KP + rk];
                if (depth) depth[nd] = k + 1;
                if (rho) rho[nd] = r;
                Bm.rho[cur ^ 1][rank] = r;
                Bm.node[cur ^ 1][rank] = nd;
                mine_sum += (double)r;
            }
        }
        n += keep;
        kept = keep;
        __syncthreads();
    }
    for (int off = 32; off >= 1; off >>= 1) mine_sum += __shfl_xor(mine_sum, off);
    if ((tid & 63) == 0) Bm.part[tid >> 6] = mine_sum;
    __syncthreads();
    if (tid == 0) {
        *n_out = n;
        if (ahat) *ahat = (float)(1.0 + ((Bm.part[0] + Bm.part[1]) + (Bm.part[2] + Bm.part[3])));
    }
}

__global__ __launch_bounds__(256) void tb_rank_expand(const float *marg, int V, int B, int K, int KP, int N, int chunks,
                                                      TbCounters *ctr, const uint2 *part, float *top_q, uint32_t *top_tok,
                                                      int32_t *parent,
                                                      int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat,
                                                      Adaptive ad, int beam_width, Batch bt, int algo)
{
    __shared__ union RankOrLevels { RankLds rank; LevelLds lev; } U;     // the ranking is over when the expansion starts
    __shared__ ExpandLds S;
    __shared__ BeamLds BM;
    __shared__ int use_levels;
    RankLds &RL = U.rank;
    // Fetch every argument in one round trip: left to the compiler the scalar loads follow the code in four
    // dependent steps over an argument block of several cache lines that is cold in every launch.
    asm volatile("" ::"s"(marg), "s"(V), "s"(B), "s"(K), "s"(KP), "s"(N), "s"(chunks), "s"(ctr), "s"(part), "s"(top_q),
                 "s"(top_tok), "s"(parent), "s"(token), "s"(depth), "s"(rho), "s"(n_out), "s"(ahat), "s"(ad.cost), "s"(ad.L_AR),
                 "s"(ad.s_best), "s"(ad.flag), "s"(beam_width), "s"(bt.n_nodes), "s"(bt.q_offset), "s"(bt.flag));
    // Workgroup `row` = position row % B of request row / B; marginals, per-thread maxima and top lists are laid out
    // request after request, outputs start at the request's q_offset.
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), row = blockIdx.x;
    const int req = row / B;
    float *q_row = top_q + (size_t)row * KP;
    uint32_t *tok_row = top_tok + (size_t)row * KP;
    const float *src = marg + (size_t)row * V;
    const bool aligned = (((size_t)row * V) & 3) == 0 && (reinterpret_cast<uintptr_t>(marg) & 15) == 0;
    const uint2 *pr = part + (size_t)row * chunks * 256 + tid;
    // ---- the bound: K-th largest per-thread maximum of the row, down to the lower edge of its histogram bin ---
    uint32_t pv[16], pw[16];                                   // the loads are in flight while the histogram is cleared
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const uint2 x = pr[(size_t)(j < chunks ? j : 0) * 256];      // no load behind a branch: all of them in flight at once
        pv[j] = j < chunks ? x.x : 0u;
        pw[j] = x.y;
    }
    for (int b = tid; b < (TBINS + TBINS / 16) / 4; b += 256) reinterpret_cast<int4 *>(RL.bins)[b] = make_int4(0, 0, 0, 0);
    if (tid == 0) { RL.nsel = 0; RL.nslot = 0; }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) if (j < chunks) atomicAdd(&RL.bins[bin_at((int)(pv[j] >> 19))], 1);
    for (int j = 16; j < chunks; ++j) atomicAdd(&RL.bins[bin_at((int)(pr[(size_t)j * 256].x >> 19))], 1);
    __syncthreads();
    {
        int hb[16], own = 0;                                   // thread t owns bins 16t .. 16t+15
#pragma unroll
        for (int b = 0; b < 16; ++b) { hb[b] = RL.bins[tid * 17 + b]; own += hb[b]; }
        const int incl = wave_incl_scan(own), wtot = __builtin_amdgcn_readlane(incl, 63);
        if (lane == 0) RL.wsum[w] = wtot;
        __syncthreads();
        int above = wtot - incl;                               // in the bins of the higher threads
        for (int ww = w + 1; ww < 4; ++ww) above += RL.wsum[ww];
        if (above < K && above + own >= K) {
            int cum = above, sel = tid * 16;
#pragma unroll
            for (int b = 15; b >= 0; --b) {
                if (cum < K && cum + hb[b] >= K) sel = tid * 16 + b;
                cum += hb[b];
            }
            RL.sel_bin = sel;
        }
        __syncthreads();                                       // the histogram is dead from here on: sel[] takes its place
    }
    const uint32_t tau = (uint32_t)RL.sel_bin << 19;
    // ---- the candidates.  A slot whose maximum reaches the bound holds a candidate; when its second largest stays
    // below the bound, which is the rule (K of thousands of slots are taken), that maximum is the slot's only one
    // and goes to the list as it stands, with the token id that its place in the slot gives.  The other slots
    // are listed and read again, one 16-byte piece of a slot per thread and four pieces in flight per thread.
    // Places in the lists are handed out per wavefront: every lane counts what it has, a scan places the lanes,
    // one lane takes the wavefront's range from the shared counter (one LDS round trip, not one per entry).
    // A lane rarely holds more than one entry: it keeps its entries as a bit mask and the wavefront loops until
    // every mask is empty, each lane storing one entry per trip (to a place of its own behind the list when it has
    // none left), which costs less than a branch or a store per possible entry. ----------------------------------
    auto wave_range = [&](int mine, int *counter) {            // first place of this lane's `mine` entries
        const int incl = wave_incl_scan(mine), total = __builtin_amdgcn_readlane(incl, 63);
        int first = 0;
        if (total > 0) {                                       // (wave-uniform)
            if (lane == 0) first = atomicAdd(counter, total);
            first = __builtin_amdgcn_readfirstlane(first);
        }
        return first + incl - mine;
    };
    {
        uint32_t one = 0u, more = 0u;                           // chunks whose slot holds one candidate / maybe several
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (j < chunks && pv[j] >= tau) {
                if (pw[j] >= tau) more |= 1u << j; else one |= 1u << j;
            }
        int pos = wave_range(__builtin_popcount(one), &RL.nsel);
        while (__builtin_amdgcn_ballot_w64(one != 0u) != 0ull) {
            const bool has = one != 0u;
            const int j = has ? __builtin_ctz(one) : 0;
            const uint32_t k = BTV_PICK16(pw, j) & 31u;
            const uint32_t v = (uint32_t)(j * SCAN + tid * 4) + (k >> 2) * 1024u + (k & 3u);
            RL.sel[has && pos < SELCAP ? pos : SELCAP + lane] = ((u64)BTV_PICK16(pv, j) << 32) | (u64)(0xFFFFFFFFu - v);
            pos += has ? 1 : 0;
            one &= one - 1u;
        }
        int mine = __builtin_popcount(more);
        for (int j = 16; j < chunks && j < 256; ++j) mine += pr[(size_t)j * 256].x >= tau ? 1 : 0;
        pos = wave_range(mine, &RL.nslot);
        while (__builtin_amdgcn_ballot_w64(more != 0u) != 0ull) {
            const bool has = more != 0u;
            const int j = has ? __builtin_ctz(more) : 0;
            RL.slot[has && pos < SLOTCAP ? pos : SLOTCAP + lane] = (uint16_t)(j * 256 + tid);
            pos += has ? 1 : 0;
            more &= more - 1u;
        }
        for (int j = 16; j < chunks && j < 256; ++j)
            if (pr[(size_t)j * 256].x >= tau) {
                if (pos < SLOTCAP) RL.slot[pos] = (uint16_t)(j * 256 + tid);
                ++pos;
            }
    }
    __syncthreads();
    const int nslot = RL.nslot;
    if (nslot == 0 && chunks <= 256) {
        // nothing to read again
    } else if (nslot <= SLOTCAP && chunks <= 256) {
        constexpr int PPS = SCAN / 1024;                       // 16-byte pieces per slot
        const int total = nslot * PPS;
        const bool whole = aligned && (V & 3) == 0;            // every piece that starts inside the row ends inside it
        for (int base = 0; base < total; base += 4 * 256) {
            float pe[16];
            int v0[4];
            uint32_t ok = 0u;                                   // bit 4u + e: element e of piece u is a candidate
            if (whole) {                                        // no load depends on a branch: four in flight at once
                int sl[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + u * 256 + tid;
                    sl[u] = RL.slot[(i < total ? i : 0) / PPS];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + u * 256 + tid;
                    v0[u] = (sl[u] >> 8) * SCAN + (i % PPS) * 1024 + (sl[u] & 255) * 4;
                    if (i >= total || v0[u] >= V) v0[u] = -1;
                    const float4 a = *reinterpret_cast<const float4 *>(src + (v0[u] < 0 ? 0 : v0[u]));
                    pe[4 * u] = a.x; pe[4 * u + 1] = a.y; pe[4 * u + 2] = a.z; pe[4 * u + 3] = a.w;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (v0[u] >= 0 && prob_bits(pe[4 * u + e]) >= tau) ok |= 1u << (4 * u + e);
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + u * 256 + tid;
                    v0[u] = -1;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pe[4 * u + e] = 0.f;
                    if (i < total) {
                        const int sl = RL.slot[i / PPS];
                        v0[u] = (sl >> 8) * SCAN + (i % PPS) * 1024 + (sl & 255) * 4;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (v0[u] + e < V) {
                                pe[4 * u + e] = src[v0[u] + e];
                                if (prob_bits(pe[4 * u + e]) >= tau) ok |= 1u << (4 * u + e);
                            }
                    }
                }
            }
            int pos = wave_range(__builtin_popcount(ok), &RL.nsel);
            while (__builtin_amdgcn_ballot_w64(ok != 0u) != 0ull) {
                const bool has = ok != 0u;
                const int bit = has ? __builtin_ctz(ok) : 0;
                const float pq = __uint_as_float(pick16v(__float_as_uint(pe[0]), __float_as_uint(pe[1]), __float_as_uint(pe[2]),
                    __float_as_uint(pe[3]), __float_as_uint(pe[4]), __float_as_uint(pe[5]), __float_as_uint(pe[6]), __float_as_uint(pe[7]),
                    __float_as_uint(pe[8]), __float_as_uint(pe[9]), __float_as_uint(pe[10]), __float_as_uint(pe[11]), __float_as_uint(pe[12]),
                    __float_as_uint(pe[13]), __float_as_uint(pe[14]), __float_as_uint(pe[15]), bit));
                int va = (bit & 8) ? v0[2] : v0[0], vb = (bit & 8) ? v0[3] : v0[1];
                asm volatile("" : "+v"(va), "+v"(vb));
                const int v = ((bit & 4) ? vb : va) + (bit & 3);
                RL.sel[has && pos < SELCAP ? pos : SELCAP + lane] = make_key(pq, (uint32_t)v);
                pos += has ? 1 : 0;
                ok &= ok - 1u;
            }
        }
    } else if (tid == 0) {
        RL.nsel = SELCAP + 1;                                  // too many slots tie at the bound: select from the row
    }
    __syncthreads();
    const int nc = RL.nsel;
    if (nc <= 256) {
        rank_keys_split(RL.sel, nc, K, KP, q_row, tok_row, tid);
    } else if (nc <= SELCAP) {
        rank_keys(RL.sel, nc, K, KP, q_row, tok_row, tid, 256);
    } else if (w == 0) {                       // rare: one wavefront selects the K best of the row first
        wave_select_rank([&](auto f) { for (int v = lane; v < V; v += 64) f(make_key(src[v], (uint32_t)v)); },
                         K, KP, RL.hist, RL.sel, &RL.nsel, q_row, tok_row, lane);
    }
    // ---- the workgroup that finishes last expands -------------------------------------------------------------
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // this thread's part of the lists has reached memory
    __syncthreads();
    if (tid == 0) RL.last = __hip_atomic_fetch_add(&ctr[req].done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == B - 1;
    __syncthreads();
    if (!RL.last) return;
    {   // all of a thread's loads are issued before the first is stored (a load and its store per loop trip would
        // make every trip a round trip to memory): 1, 4 or MAXB entries of each list per thread
        const size_t lists = (size_t)req * B * KP;
        const int n = B * KP;
        auto fetch = [&](auto per_thread) {
            constexpr int PT = decltype(per_thread)::value;
            float qv[PT];
            uint32_t tv[PT];
#pragma unroll
            for (int i = 0; i < PT; ++i) {
                const int e = tid + 256 * i, ee = e < n ? e : 0;
                qv[i] = __hip_atomic_load(top_q + lists + ee, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                tv[i] = __hip_atomic_load(top_tok + lists + ee, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int i = 0; i < PT; ++i) {
                const int e = tid + 256 * i;
                if (e < n) { S.q[e] = qv[i]; S.tok[e] = tv[i]; }
            }
        };
        if (n <= 256) fetch(std::integral_constant<int, 1>{});
        else if (n <= 1024) fetch(std::integral_constant<int, 4>{});
        else fetch(std::integral_constant<int, MAXB>{});
    }

    if (bt.n_nodes) {                          // this request's budget and output rows
        const int o0 = bt.q_offset[req], room = bt.q_offset[req + 1] - o0, want = bt.n_nodes[req];
        const bool bad = o0 < 0 || want < 0 || want > N || want > room;
        if (bad && tid == 0) atomicOr(bt.flag, 16u);
        N = bad ? 0 : want;
        parent += o0; token += o0;
        if (depth) depth += o0;
        if (rho) rho += o0;
        n_out += req;
        if (ahat) ahat += req;
        if (N == 0) {
            if (tid == 0) { *n_out = 0; if (ahat) *ahat = 1.0f; }
            return;
        }
    }
    if (ad.cost)
        for (int e = tid; e < N; e += 256) S.cost[e] = ad.cost[e];
    __syncthreads();
    if (beam_width > 0) {                      // B rows = depths of the beam tree, K = min(V, width)
        beam_block(S, BM, B, K, KP, beam_width, tid, parent, token, depth, rho, n_out, ahat);
        return;
    }
    // Which expansion: the level-synchronous one pays per level (measured: about 2.5 us up to 32 nodes, 3.0 to 64,
    // 3.6 to 128, 4.2 beyond), the one-wavefront one per node (0.27 / 0.31 / 0.41 us up to 64 / 128 / 256 nodes), and
    // with the early stop it ends at the chosen budget, typically a quarter of N_max.  The tree cannot be deeper than
    // the greedy chain stays above the N-th best token of the first position (every node scores at least as much as
    // the tree's last one, which scores at least that); a tree of depth 1 is the first level's list as it stands.
    if (tid == 0) {
        int reach = 0;
        if (algo == 0) {
            const float g_est = S.q[min(K, N) - 1];
            float chain = 1.0f;
            for (int k = 0; k < B; ++k) {
                chain = __fmul_rn(chain, S.q[k * KP]);
                if (!(chain >= g_est)) break;
                reach = k + 1;
            }
        }
        const float per_level = N <= 32 ? 2.5f : N <= 64 ? 3.0f : N <= 128 ? 3.6f : 4.2f;
        const float per_node = N <= 64 ? 0.27f : N <= 128 ? 0.31f : 0.41f;
        const float nodes = ad.cost ? 0.25f * (float)N : (float)N;
        use_levels = algo == 2 || (algo == 0 && (reach <= 1 || (float)reach * per_level < nodes * per_node));
    }
    __syncthreads();
    if (use_levels) {
        if (ad.cost) expand_levels<true>(S, U.lev, B, K, KP, N, tid, parent, token, depth, rho, n_out, ahat, ad);
        else expand_levels<false>(S, U.lev, B, K, KP, N, tid, parent, token, depth, rho, n_out, ahat, ad);
        return;
    }
    if (w != 0) return;
    if (ad.cost) {
        if (N <= 64) expand_wave<1, true>(S, B, K, KP, N, lane, parent, token, depth, rho, n_out, ahat, ad);
        else if (N <= 128) expand_wave<2, true>(S, B, K, KP, N, lane, parent, token, depth, rho, n_out, ahat, ad);
        else expand_wave<4, true>(S, B, K, KP, N, lane, parent, token, depth, rho, n_out, ahat, ad);
    } else {
        if (N <= 64) expand_wave<1, false>(S, B, K, KP, N, lane, parent, token, depth, rho, n_out, ahat, ad);
        else if (N <= 128) expand_wave<2, false>(S, B, K, KP, N, lane, parent, token, depth, rho, n_out, ahat, ad);
        else expand_wave<4, false>(S, B, K, KP, N, lane, parent, token, depth, rho, n_out, ahat, ad);
    }
}

int next_pow2(int x) { int p = 1; while (p < x) p <<= 1; return p; }

struct TopkPlan { int K, KP, chunks; size_t ctr_bytes, part_bytes, top_bytes; };

TopkPlan topk_plan(int batch, int B, int V, int N)
{
    TopkPlan t;
    t.K = std::min(V, N);
    t.KP = std::max(next_pow2(t.K), 1);
    t.chunks = (V + SCAN - 1) / SCAN;
    t.ctr_bytes = btv_align_up((size_t)batch * sizeof(TbCounters), BTV_WS_ALIGN);
    t.part_bytes = btv_align_up((size_t)batch * B * t.chunks * 256 * sizeof(uint2), BTV_WS_ALIGN);
    t.top_bytes = btv_align_up((size_t)batch * B * t.KP * 4, BTV_WS_ALIGN);
    return t;
}

constexpr int MAX_BATCH = 1024;

size_t tree_build_ws(int batch, int B, int V, int N)
{
    if (batch < 1 || batch > MAX_BATCH || B < 1 || B > MAXB || V < 1 || N < 1 || N > BTV_MAX_NODES) return 0;
    TopkPlan t = topk_plan(batch, B, V, N);
    return BTV_WS_HEADER + t.ctr_bytes + t.part_bytes + 2 * t.top_bytes;
}

}  // namespace

extern "C" {

size_t btv_tree_build_workspace(int B, int V, int N) { return tree_build_ws(1, B, V, N); }

size_t btv_tree_build_batch_workspace(int batch, int B, int V, int N_max) { return tree_build_ws(batch, B, V, N_max); }

static int tree_build_launch(const float *marginals, int batch, int B, int V, int N, const Adaptive &ad_in, int beam_width,
                             Batch bt, int algo, int32_t *parent, int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat,
                             void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(marginals && parent && token && n_out, "null pointer");
    BTV_REQUIRE(batch >= 1 && batch <= MAX_BATCH, "batch=%d outside [1,%d]", batch, MAX_BATCH);
    BTV_REQUIRE(B >= 1 && B <= MAXB, "B=%d outside [1,%d]", B, MAXB);
    BTV_REQUIRE(V >= 1, "V=%d", V);
    BTV_REQUIRE(N >= 1 && N <= BTV_MAX_NODES, "N=%d outside [1,%d]", N, BTV_MAX_NODES);
    int rc = btv_check_ws(ws, ws_bytes, tree_build_ws(batch, B, V, N));
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TopkPlan t = topk_plan(batch, B, V, N);
    unsigned char *base = static_cast<unsigned char *>(ws);
    TbCounters *ctr = reinterpret_cast<TbCounters *>(base + BTV_WS_HEADER);
    uint2 *part = reinterpret_cast<uint2 *>(base + BTV_WS_HEADER + t.ctr_bytes);
    float *top_q = reinterpret_cast<float *>(base + BTV_WS_HEADER + t.ctr_bytes + t.part_bytes);
    uint32_t *top_tok = reinterpret_cast<uint32_t *>(base + BTV_WS_HEADER + t.ctr_bytes + t.part_bytes + t.top_bytes);
    Adaptive ad = ad_in;
    ad.flag = reinterpret_cast<uint32_t *>(base);
    bt.flag = reinterpret_cast<uint32_t *>(base);
    hipLaunchKernelGGL(tb_thread_max, dim3(t.chunks, B * batch), dim3(256), 0, st, marginals, V, B, t.chunks, part, ctr);
    BTV_HIP(hipGetLastError());
    hipLaunchKernelGGL(tb_rank_expand, dim3(B * batch), dim3(256), 0, st, marginals, V, B, t.K, t.KP, N, t.chunks, ctr, part, top_q,
                       top_tok, parent, token, depth, rho, n_out, ahat, ad, beam_width, bt, algo);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

static const Batch kOneRequest = { nullptr, nullptr, nullptr };

int btv_tree_build(const float *marginals, int B, int V, int N, int32_t *parent, int32_t *token, int32_t *depth,
                   float *rho, int32_t *n_out, float *ahat, void *ws, size_t ws_bytes, void *stream)
{
    const Adaptive none = { nullptr, 0.0, nullptr, nullptr };
    return tree_build_launch(marginals, 1, B, V, N, none, 0, kOneRequest, 0, parent, token, depth, rho, n_out, ahat, ws, ws_bytes, stream);
}

int btv_tree_build_beam(const float *marginals, int B, int V, int width, int depth_max, int32_t *parent, int32_t *token,
                        int32_t *depth, float *rho, int32_t *n_out, float *ahat, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(width >= 1 && width <= MAXW, "width=%d outside [1,%d]", width, MAXW);
    BTV_REQUIRE(B >= 1 && B <= MAXB, "B=%d outside [1,%d]", B, MAXB);
    BTV_REQUIRE(depth_max >= 1 && depth_max <= B, "depth=%d outside [1,B=%d]", depth_max, B);
    // the first depth_max positions are ranked for their `width` best tokens; the rest of the path is shared
    const Adaptive none = { nullptr, 0.0, nullptr, nullptr };
    return tree_build_launch(marginals, 1, depth_max, V, width, none, width, kOneRequest, 0, parent, token, depth, rho, n_out, ahat,
                             ws, ws_bytes, stream);
}

int btv_tree_build_adaptive(const float *marginals, int B, int V, int N_max, const double *cost, double L_AR,
                            int32_t *parent, int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat,
                            double *s_best, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(cost != nullptr, "null pointer");
    BTV_REQUIRE(L_AR > 0.0, "L_AR must be positive");
    const Adaptive ad = { cost, L_AR, s_best, nullptr };
    return tree_build_launch(marginals, 1, B, V, N_max, ad, 0, kOneRequest, 0, parent, token, depth, rho, n_out, ahat, ws, ws_bytes, stream);
}

int btv_tree_build_tuned(const float *marginals, int B, int V, int N, const double *cost, double L_AR, int algo,
                         int32_t *parent, int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat,
                         double *s_best, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(algo >= 0 && algo <= 2, "algo=%d outside [0,2]", algo);
    BTV_REQUIRE(cost == nullptr || L_AR > 0.0, "L_AR must be positive");
    const Adaptive ad = { cost, L_AR, cost ? s_best : nullptr, nullptr };
    return tree_build_launch(marginals, 1, B, V, N, ad, 0, kOneRequest, algo, parent, token, depth, rho, n_out, ahat, ws, ws_bytes,
                             stream);
}

int btv_tree_build_batch(const float *marginals, int batch, int B, int V, const int32_t *n_nodes, const int32_t *q_offset,
                         int N_max, int32_t *parent, int32_t *token, int32_t *depth, float *rho, int32_t *n_out, float *ahat,
                         void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(n_nodes && q_offset, "null pointer");
    const Adaptive none = { nullptr, 0.0, nullptr, nullptr };
    const Batch bt = { n_nodes, q_offset, nullptr };
    return tree_build_launch(marginals, batch, B, V, N_max, none, 0, bt, 0, parent, token, depth, rho, n_out, ahat, ws, ws_bytes,
                             stream);
}

}  // extern "C"
