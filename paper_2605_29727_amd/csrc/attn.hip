// Tree-masked attention for gfx950 (MI355X): ancestor bitmask, bf16 MFMA split-K kernel,
// fp32 reference-precision kernel, split-K combine, and the two C-ABI entry points.
//
// What is computed (App. C, "Linearization and verification mask"): node i attends to the L
// prefix rows of the KV cache and to the tree rows of its ancestors and itself.
//
// bf16 kernel layout.  For one KV head the G = Hq/Hkv query heads of every node are packed
// into rows r = i*G + j, so the whole GQA group shares each K/V byte that is streamed.
// A workgroup (4 wavefronts of 64 lanes) owns WR rows and a range of 32-key tiles; K and V
// tiles are staged through LDS once per workgroup (ring of stages filled by direct-to-LDS loads).
// Scores are computed transposed, S^T = K . Q^T with 32x32x16 bf16 MFMA: in the accumulator
// layout a lane then holds ONE query column and 16 keys, so the running max / sum of the
// online softmax are per-lane scalars (one cross-half exchange per tile), the P^T tile is
// already in B-operand layout for O^T += V^T . P^T, and the O^T accumulator is rescaled by a
// per-lane factor.  V^T operands come from transposing LDS reads.  The tree mask is applied only on tiles
// that touch tree rows, from a 32-bit visibility word per (query, tile) built from the node's
// ancestor bitmask.
#include "btv_common.h"

#include <algorithm>
#include <cmath>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 32;          // keys per tile = per LDS stage
constexpr float NEG_BIG = -1.0e30f;

struct AttnParams {
    const void *Q, *K, *V;
    void *O;
    const uint32_t *anc;          // [total_M][BTV_ANC_WORDS]
    const int32_t *block_table;   // paged only
    const int32_t *q_offset;      // paged only, [batch+1]
    const int32_t *prefix_len;    // paged only, [batch]
    float *Opart;                 // [nsplit][total_rows][D]
    float *ML;                    // [nsplit][total_rows][2]
    uint32_t *flag;
    int M, L;                     // contiguous: actual sizes; paged: host upper bounds
    int Hq, Hkv, G;
    int max_blocks, num_blocks;
    int total_rows;               // rows of the partial buffers (>= total_M * Hq)
    int total_M;
    int sps;                      // stages per split
    int nsplit;                   // grid.x
    float scale;                  // softmax scale
    float scale_log2;             // scale * log2(e)
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{   // round to nearest even; inputs here are finite
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Request geometry: contiguous calls have one request; paged calls read it from device arrays
// and clamp against the host-provided bounds so that no access can leave its buffer.
struct Req { int q0, M, L; bool ok; };

template <bool PAGED>
__device__ __forceinline__ Req load_req(const AttnParams &p, int r)
{
    Req q;
    if (!PAGED) { q.q0 = 0; q.M = p.M; q.L = p.L; q.ok = true; return q; }
    q.q0 = p.q_offset[r];
    q.M = p.q_offset[r + 1] - q.q0;
    q.L = p.prefix_len[r];
    q.ok = q.M >= 1 && q.M <= p.M && q.L >= 0 && q.L <= p.L && q.q0 >= 0 &&
           q.q0 + q.M <= p.total_M && (long long)q.L + q.M <= (long long)p.max_blocks * BTV_PAGE;
    return q;
}

template <bool PAGED>
__device__ __forceinline__ long long phys_row(const AttnParams &p, int r, int j)
{
    if (!PAGED) return j;
    int b = p.block_table[(long long)r * p.max_blocks + (j >> 4)];
    b = min(max(b, 0), p.num_blocks - 1);
    return (long long)b * BTV_PAGE + (j & 15);
}

// Visibility of keys kb..kb+31 for node i: bit c set iff key kb+c is a prefix row, or a tree
// row L+a with a in anc(i).  Bits of anc past the request's node count are zero.
__device__ __forceinline__ uint32_t vis_word(const uint32_t *anc_i, int kb, int L)
{
    int off = kb - L;
    if (off <= -32) return 0xFFFFFFFFu;
    if (off < 0) {
        int n = -off;
        return ((1u << n) - 1u) | (anc_i[0] << n);
    }
    int w = off >> 5, sh = off & 31;
    uint32_t lo = (w < BTV_ANC_WORDS) ? anc_i[w] : 0u;
    uint32_t hi = (w + 1 < BTV_ANC_WORDS) ? anc_i[w + 1] : 0u;
    return sh ? ((lo >> sh) | (hi << (32 - sh))) : lo;
}

// ------------------------------------------------------------------------------------------------
// Ancestor bitmask: anc[i] = {i} u anc[parent[i]].  One workgroup per request, one thread per node,
// each walking its own chain (parents are strictly decreasing, so the walk ends; an out-of-range
// parent is treated as -1 and flagged).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void anc_mask_kernel(const int32_t *parent, const int32_t *q_offset, int M_max,
                                                       int total_M, uint32_t *anc, uint32_t *flag)
{
    __shared__ int32_t par[BTV_MAX_NODES];
    int r = blockIdx.x, i = threadIdx.x;
    int q0 = q_offset ? q_offset[r] : 0;
    int M = q_offset ? q_offset[r + 1] - q0 : M_max;
    if (M < 1 || M > M_max || q0 < 0 || q0 + M > total_M) return;   // flagged by the attention kernel's own check
    bool bad = false;
    if (i < M) {
        int pa = parent[q0 + i];
        if (pa < -1 || pa >= i) { bad = true; pa = -1; }
        par[i] = pa;
    }
    __syncthreads();
    if (i < M) {
        uint32_t w[BTV_ANC_WORDS];
#pragma unroll
        for (int k = 0; k < BTV_ANC_WORDS; ++k) w[k] = 0u;
        for (int a = i; a >= 0; a = par[a]) {
#pragma unroll
            for (int k = 0; k < BTV_ANC_WORDS; ++k)
                if ((a >> 5) == k) w[k] |= 1u << (a & 31);
        }
        uint4 *dst = reinterpret_cast<uint4 *>(anc + (size_t)(q0 + i) * BTV_ANC_WORDS);
        dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
        dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
    }
    if (bad) atomicOr(flag, 1u);
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel
//
// LDS holds a ring of NS stages; a stage is one 32-key tile: the K rows and the V rows exactly as
// they lie in memory ([key][channel], 2*D bytes per row).  Stages are filled by direct-to-LDS
// global loads (each lane moves 16 bytes, a wave instruction fills 1 KiB of LDS), so no staging
// registers and no VALU work are spent on data movement and NS-1 stages stay in flight.
// Bank conflicts are avoided by choosing which 16-byte chunk of a row each lane fetches: the chunk
// stored at physical position pc of LDS row r is chunk pc ^ f(r) of the source row.
//   K: LDS row i holds key kb + swap_bits_2_3(i) (the MFMA A-row order that makes a lane's 16 score
//      registers two runs of 8 consecutive keys); A operands are 16-byte LDS reads.
//   V: LDS row r holds key kb + r; the V^T A operand (one channel, 8 consecutive keys per lane) comes
//      from two transposing LDS reads (ds_read_b64_tr_b16): a 16-lane group reads 4 keys x 16 channels
//      and every lane receives the 4 keys of its own channel.
// ------------------------------------------------------------------------------------------------
template <int D>
struct Lds {
    static constexpr int ROWB = 2 * D;                       // bytes per K or V row
    static constexpr int TILEB = 32 * ROWB;                  // one K (or V) tile
    static constexpr int STAGE = 2 * TILEB;                  // K tile then V tile
    static constexpr int LPW = STAGE / 1024 / 4;             // load instructions per wave per stage
};

__device__ __forceinline__ int swap_bits_2_3(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

template <int D> __device__ __forceinline__ int swz_k(int row) { return row & (D / 8 - 1); }
template <int D> __device__ __forceinline__ int swz_v(int row) { return (row & (D / 8 - 1)) ^ (((row >> 3) & 1) << 2); }

#define BTV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

template <bool PAGED>
struct StageCtx {
    const uint16_t *Kp, *Vp;
    const int32_t *block_table;   // row of this request
    int num_blocks, Hkv, g, S;
};

// Issue the direct-to-LDS loads of tile `st` (keys 32*st ..) into ring slot `slot`.  Keys past the end of
// the sequence re-read the last valid row (finite data; their scores are masked).
template <int D, bool PAGED>
__device__ __forceinline__ void issue_stage(const StageCtx<PAGED> &cx, unsigned char *smem, int slot, int st, int w, int l)
{
    using LD = Lds<D>;
    constexpr int CH = D / 8;                 // 16-byte chunks per row
    constexpr int RPI = 1024 / LD::ROWB;      // rows filled by one wave instruction
    const int kb = st * 32;
    // a 32-key tile spans two 16-token pages; their ids are wave-uniform (scalar loads, so the vector-memory
    // counter only ever counts the LDS fills)
    long long page0 = 0, page1 = 0;
    if (PAGED) {
        const int last_page = (cx.S - 1) >> 4;
        typedef const __attribute__((address_space(4))) int32_t *const_i32;   // constant space: scalar loads
        const_i32 bt = reinterpret_cast<const_i32>(reinterpret_cast<uintptr_t>(cx.block_table));
        const int i0 = __builtin_amdgcn_readfirstlane(min(2 * st, last_page));
        const int i1 = __builtin_amdgcn_readfirstlane(min(2 * st + 1, last_page));
        int b0 = bt[i0], b1 = bt[i1];
        page0 = (long long)min(max(b0, 0), cx.num_blocks - 1) * BTV_PAGE;
        page1 = (long long)min(max(b1, 0), cx.num_blocks - 1) * BTV_PAGE;
    }
#pragma unroll
    for (int jj = 0; jj < LD::LPW; ++jj) {
        const int j = w * LD::LPW + jj;                       // instruction index within the stage
        const bool isv = j >= LD::TILEB / 1024;
        const int jt = isv ? j - LD::TILEB / 1024 : j;        // instruction index within the K or V tile
        const int r = jt * RPI + l / CH, pc = l % CH;         // LDS row and physical chunk of this lane
        const int key = min(kb + (isv ? r : swap_bits_2_3(r)), cx.S - 1);
        const int chunk = pc ^ (isv ? swz_v<D>(r) : swz_k<D>(r));
        const long long prow = PAGED ? (((key - kb) & 16) ? page1 : page0) + (key & 15) : (long long)key;
        const uint16_t *src = (isv ? cx.Vp : cx.Kp) + (prow * cx.Hkv + cx.g) * D + chunk * 8;
        __builtin_amdgcn_global_load_lds(src, BTV_LDS_PTR(smem + slot * LD::STAGE + j * 1024), 16, 0, 0);
    }
}

// One 32-key tile of one wave: S^T = K.Q^T, tree mask, online softmax, O^T += V^T.P^T.
template <int D, int QB>
__device__ __forceinline__ void do_tile(const unsigned char *stage, int kb, int Lr, int l, float sl2,
                                        const uint32_t *anc, int q0, const int (&node)[QB],
                                        const bf16x8 (&qreg)[QB][D / 16], float (&m_run)[QB], float (&l_run)[QB],
                                        f32x16 (&oacc)[D / 32][QB])
{
    constexpr int DS = D / 16, DT = D / 32;
    using LD = Lds<D>;
    const int c = l & 31, h = l >> 5;
    const unsigned char *Ks = stage, *Vs = stage + LD::TILEB;
    f32x16 sacc[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[qb][v] = 0.f;
    const int kswz = swz_k<D>(c);
#pragma unroll
    for (int s = 0; s < DS; ++s) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(Ks + c * LD::ROWB + (((2 * s + h) ^ kswz) << 4));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            sacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][s], sacc[qb], 0, 0, 0);
    }
    if (kb + 32 > Lr) {     // the tile touches tree rows (or the end of the sequence): apply the mask
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            uint32_t vis = vis_word(anc + (size_t)(q0 + node[qb]) * BTV_ANC_WORDS, kb, Lr);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int bit = 16 * (v >> 3) + 8 * h + (v & 7);
                if (!((vis >> bit) & 1u)) sacc[qb][v] = -INFINITY;
            }
        }
    }
    bf16x8 pb[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float tmax = sacc[qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, sacc[qb][v]);
        {   // other half of the wave holds the other 16 keys of the same query
            auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
            tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        float mnew = fmaxf(m_run[qb], tmax);
        float alpha = __builtin_amdgcn_exp2f((m_run[qb] - mnew) * sl2);
        float mc = mnew * sl2;
        m_run[qb] = mnew;
        float rs = 0.f;
        float pv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            pv[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[qb][v], sl2, -mc));
            rs += pv[v];
        }
        l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[dt][qb][v] *= alpha;
#pragma unroll
        for (int mm = 0; mm < 2; ++mm)
#pragma unroll
            for (int e = 0; e < 8; ++e) pb[qb][mm][e] = (__bf16)pv[mm * 8 + e];
    }
    // V^T operands: lane l sits in 16-lane group l/16 = 2h + dhalf; it supplies the address of key row
    // 16mm + 8h + 4i + (l%16)/4, channels 32dt + 16dhalf + 4(l%4) .. +3, and receives keys 16mm + 8h + 4i .. +3
    // of channel 32dt + (l%32).
    const int dhalf = (l >> 4) & 1, rr = (l & 15) >> 2, q = l & 3;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            bf16x4 lo, hi;
            {
                const int r0 = 16 * mm + 8 * h + rr, r1 = r0 + 4;
                const int chunk = 4 * dt + 2 * dhalf + (q >> 1);
                lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (__attribute__((address_space(3))) bf16x4 *)BTV_LDS_PTR(Vs + r0 * LD::ROWB + ((chunk ^ swz_v<D>(r0)) << 4) + ((q & 1) << 3)));
                hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (__attribute__((address_space(3))) bf16x4 *)BTV_LDS_PTR(Vs + r1 * LD::ROWB + ((chunk ^ swz_v<D>(r1)) << 4) + ((q & 1) << 3)));
            }
            bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                oacc[dt][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][mm], oacc[dt][qb], 0, 0, 0);
        }
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int D, int QB, int KW, int NS, bool PAGED>
__global__ __launch_bounds__(256, 1) void tv_attn_bf16(AttnParams p)
{
    constexpr int RW = 4 / KW;
    constexpr int WR = RW * QB * 32;
    constexpr int DS = D / 16;
    constexpr int DT = D / 32;
    using LD = Lds<D>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, c = l & 31, h = l >> 5;
    const int kw = w % KW, rw = w / KW;
    const int rq = blockIdx.z / p.Hkv, g = blockIdx.z % p.Hkv;
    const Req rq_ = load_req<PAGED>(p, rq);
    if (!rq_.ok) {
        if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) atomicOr(p.flag, 2u);
        return;
    }
    const int Mr = rq_.M, Lr = rq_.L, S = Lr + Mr;
    const int rows_g = Mr * p.G;
    if ((int)blockIdx.y * WR >= rows_g) return;
    const int tiles = (S + 31) / 32;
    const int nsplit_r = (tiles + p.sps - 1) / p.sps;
    if ((int)blockIdx.x >= nsplit_r) return;
    const int st0 = blockIdx.x * p.sps, st1 = min(st0 + p.sps, tiles);

    const uint16_t *Qp = static_cast<const uint16_t *>(p.Q);
    const StageCtx<PAGED> cx = { static_cast<const uint16_t *>(p.K), static_cast<const uint16_t *>(p.V),
                                 PAGED ? p.block_table + (long long)rq * p.max_blocks : nullptr, p.num_blocks, p.Hkv, g, S };

    // ---- start filling the ring: NS-1 tiles in flight ------------------------------------------
    int issued = st0, islot = 0;
#pragma unroll
    for (int k = 0; k < NS - 1; ++k)
        if (issued < st1) { issue_stage<D, PAGED>(cx, smem, islot, issued, w, l); ++issued; ++islot; }
    // ---- per-lane query rows -------------------------------------------------------------------
    int node[QB];
    long long orow[QB];       // row index into Q/O viewed as [total_M*Hq, D]
    bool rvalid[QB];
    bf16x8 qreg[QB][DS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int r = blockIdx.y * WR + (rw * QB + qb) * 32 + c;
        rvalid[qb] = r < rows_g;
        int rr = rvalid[qb] ? r : 0;
        node[qb] = rr / p.G;
        orow[qb] = (long long)(rq_.q0 + node[qb]) * p.Hq + g * p.G + (rr % p.G);
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (rvalid[qb]) v = *reinterpret_cast<const uint4 *>(Qp + orow[qb] * D + s * 16 + h * 8);
            qreg[qb][s] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // Pin the Q registers here: the compiler then waits for the Q loads in straight-line code, before the loop,
    // instead of draining the whole vector-memory queue at their first use inside it.
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(qreg[qb][s]));

    float m_run[QB], l_run[QB];
    f32x16 oacc[DT][QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = NEG_BIG; l_run[qb] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[dt][qb][v] = 0.f;
    }

    // ---- main loop: one barrier per tile --------------------------------------------------------
    // At the top of iteration st the tiles st+1 .. issued-1 may still be in flight; the barrier also tells
    // that every wave is done with tile st-1, whose ring slot the next issue overwrites.
    int cslot = 0, turn = 0;
    if (islot == NS) islot = 0;
    for (int st = st0; st < st1; ++st) {
        if (issued - st - 1 == NS - 2) wait_vmcnt<(NS - 2) * LD::LPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (issued < st1) {
            issue_stage<D, PAGED>(cx, smem, islot, issued, w, l);
            ++issued;
            if (++islot == NS) islot = 0;
        }
        if (turn == kw)
            do_tile<D, QB>(smem + cslot * LD::STAGE, st * 32, Lr, l, p.scale_log2, p.anc, rq_.q0, node, qreg, m_run, l_run,
                           oacc);
        if (++cslot == NS) cslot = 0;
        if (++turn == KW) turn = 0;
    }

    // both halves of a wave hold partial row sums of the same queries
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += __shfl_xor(l_run[qb], 32);

    // ---- merge the key-split waves of this workgroup through LDS, one donor wave at a time ----
    if (KW > 1) {
        constexpr int SLOT = (DT * QB * 16 + 2 * QB) * 64;    // floats per row-wave slot
        float *mg = reinterpret_cast<float *>(smem) + rw * SLOT;
#pragma unroll
        for (int donor = 1; donor < KW; ++donor) {
            __syncthreads();
            if (kw == donor) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) mg[((dt * QB + qb) * 16 + v) * 64 + l] = oacc[dt][qb][v];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    mg[(DT * QB * 16 + qb) * 64 + l] = m_run[qb];
                    mg[(DT * QB * 16 + QB + qb) * 64 + l] = l_run[qb];
                }
            }
            __syncthreads();
            if (kw == 0) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    float m1 = mg[(DT * QB * 16 + qb) * 64 + l], l1 = mg[(DT * QB * 16 + QB + qb) * 64 + l];
                    float mn = fmaxf(m_run[qb], m1);
                    float a0 = __builtin_amdgcn_exp2f((m_run[qb] - mn) * p.scale_log2);
                    float a1 = __builtin_amdgcn_exp2f((m1 - mn) * p.scale_log2);
                    m_run[qb] = mn;
                    l_run[qb] = l_run[qb] * a0 + l1 * a1;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            oacc[dt][qb][v] = oacc[dt][qb][v] * a0 + mg[((dt * QB + qb) * 16 + v) * 64 + l] * a1;
                }
            }
        }
    }
    if (kw != 0) return;

    // ---- write: final bf16 rows when this request has a single split, fp32 partials otherwise ---
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        if (!rvalid[qb]) continue;
        if (nsplit_r == 1) {
            float inv = 1.0f / l_run[qb];
            uint16_t *Op = static_cast<uint16_t *>(p.O) + orow[qb] * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    uint32_t lo = float_to_bf16_bits(oacc[dt][qb][q4 * 4 + 0] * inv) |
                                  (float_to_bf16_bits(oacc[dt][qb][q4 * 4 + 1] * inv) << 16);
                    uint32_t hi = float_to_bf16_bits(oacc[dt][qb][q4 * 4 + 2] * inv) |
                                  (float_to_bf16_bits(oacc[dt][qb][q4 * 4 + 3] * inv) << 16);
                    *reinterpret_cast<uint2 *>(Op + dt * 32 + q4 * 8 + h * 4) = make_uint2(lo, hi);
                }
        } else {
            size_t prow = (size_t)blockIdx.x * p.total_rows + orow[qb];
            float *Pp = p.Opart + prow * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 o = { oacc[dt][qb][q4 * 4 + 0], oacc[dt][qb][q4 * 4 + 1], oacc[dt][qb][q4 * 4 + 2],
                                oacc[dt][qb][q4 * 4 + 3] };
                    *reinterpret_cast<f32x4 *>(Pp + dt * 32 + q4 * 8 + h * 4) = o;
                }
            if (h == 0) *reinterpret_cast<float2 *>(p.ML + prow * 2) = make_float2(m_run[qb], l_run[qb]);
        }
    }
}

// Split-K combine: O[row] = sum_s w_s O_s / sum_s w_s l_s with w_s = exp2((m_s - max m) * scale*log2 e).
// 8 rows per workgroup, 32 lanes per row.
template <int D, bool PAGED>
__global__ __launch_bounds__(256) void tv_combine_bf16(AttnParams p)
{
    constexpr int E = D / 32;
    const int rq = blockIdx.y;
    const Req rq_ = load_req<PAGED>(p, rq);
    if (!rq_.ok) return;
    const int stages = (rq_.L + rq_.M + TK - 1) / TK;
    const int nsplit_r = (stages + p.sps - 1) / p.sps;
    if (nsplit_r == 1) return;                      // the attention kernel wrote O directly
    const int lr = blockIdx.x * 8 + (threadIdx.x >> 5), lane = threadIdx.x & 31;
    if (lr >= rq_.M * p.Hq) return;
    const size_t row = (size_t)rq_.q0 * p.Hq + lr;
    float mmax = NEG_BIG;
    for (int s = 0; s < nsplit_r; ++s) mmax = fmaxf(mmax, p.ML[((size_t)s * p.total_rows + row) * 2]);
    float acc[E], den = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    for (int s = 0; s < nsplit_r; ++s) {
        size_t pr = (size_t)s * p.total_rows + row;
        float2 ml = *reinterpret_cast<const float2 *>(p.ML + pr * 2);
        float wgt = __builtin_amdgcn_exp2f((ml.x - mmax) * p.scale_log2);
        den += wgt * ml.y;
        const float *src = p.Opart + pr * D + lane * E;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] += wgt * src[e];
    }
    float inv = 1.0f / den;
    uint16_t *dst = static_cast<uint16_t *>(p.O) + row * D + lane * E;
#pragma unroll
    for (int e = 0; e < E; ++e) dst[e] = (uint16_t)float_to_bf16_bits(acc[e] * inv);
}

// ------------------------------------------------------------------------------------------------
// fp32 kernel: one workgroup per (node, query head); threads stride over the visible keys with a
// private online softmax, then the 256 partial states are merged.  Precision path, not the fast one.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void tv_attn_f32(AttnParams p)
{
    __shared__ float qs[D];
    __shared__ float red[4][D + 2];
    const int i = blockIdx.x, hq = blockIdx.y, tid = threadIdx.x, g = hq / p.G;
    const float *Q = static_cast<const float *>(p.Q), *K = static_cast<const float *>(p.K),
                *V = static_cast<const float *>(p.V);
    const uint32_t *anc_i = p.anc + (size_t)i * BTV_ANC_WORDS;
    for (int d = tid; d < D; d += 256) qs[d] = Q[((size_t)i * p.Hq + hq) * D + d];
    __syncthreads();
    float m = NEG_BIG, lsum = 0.f, o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;
    const int S = p.L + p.M;
    for (int j = tid; j < S; j += 256) {
        if (j >= p.L) {
            int a = j - p.L;
            if (!((anc_i[a >> 5] >> (a & 31)) & 1u)) continue;
        }
        const float4 *kr = reinterpret_cast<const float4 *>(K + ((size_t)j * p.Hkv + g) * D);
        float s = 0.f;
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            float4 kv = kr[d4];
            s = fmaf(qs[4 * d4 + 0], kv.x, s); s = fmaf(qs[4 * d4 + 1], kv.y, s);
            s = fmaf(qs[4 * d4 + 2], kv.z, s); s = fmaf(qs[4 * d4 + 3], kv.w, s);
        }
        s *= p.scale;
        float mn = fmaxf(m, s);
        float alpha = expf(m - mn), pj = expf(s - mn);
        m = mn;
        lsum = lsum * alpha + pj;
        const float4 *vr = reinterpret_cast<const float4 *>(V + ((size_t)j * p.Hkv + g) * D);
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            float4 vv = vr[d4];
            o[4 * d4 + 0] = o[4 * d4 + 0] * alpha + pj * vv.x;
            o[4 * d4 + 1] = o[4 * d4 + 1] * alpha + pj * vv.y;
            o[4 * d4 + 2] = o[4 * d4 + 2] * alpha + pj * vv.z;
            o[4 * d4 + 3] = o[4 * d4 + 3] * alpha + pj * vv.w;
        }
    }
    // merge: global max, rescale, sum
    float mw = m;
    for (int off = 32; off >= 1; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
    if ((tid & 63) == 0) red[tid >> 6][0] = mw;
    __syncthreads();
    float mb = fmaxf(fmaxf(red[0][0], red[1][0]), fmaxf(red[2][0], red[3][0]));
    __syncthreads();
    float f = expf(m - mb);
    lsum *= f;
    for (int off = 32; off >= 1; off >>= 1) lsum += __shfl_xor(lsum, off);
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float x = o[d] * f;
        for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
        o[d] = x;
    }
    if ((tid & 63) == 0) {
        red[tid >> 6][D] = lsum;
#pragma unroll
        for (int d = 0; d < D; ++d) red[tid >> 6][d] = o[d];
    }
    __syncthreads();
    float den = red[0][D] + red[1][D] + red[2][D] + red[3][D];
    float *Op = static_cast<float *>(p.O) + ((size_t)i * p.Hq + hq) * D;
    for (int d = tid; d < D; d += 256) Op[d] = (red[0][d] + red[1][d] + red[2][d] + red[3][d]) / den;
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
int g_split_override = 0;

struct Plan { int qb, kw, wr, row_blocks, stages, sps, nsplit; };

// Kernel shape by the number of packed rows per KV head (G*M): few rows -> all four waves share the rows and
// split the keys (KW = 4 or 2); many rows -> four row-waves of 64 rows, workgroups tile the rows in blocks of 256.
Plan make_plan(int M, int L, int Hq, int Hkv, int batch)
{
    Plan pl;
    int G = Hq / Hkv, rows_g = G * M;
    if (rows_g <= 32) { pl.qb = 1; pl.kw = 4; }
    else if (rows_g <= 64) { pl.qb = 2; pl.kw = 4; }
    else if (rows_g <= 128) { pl.qb = 2; pl.kw = 2; }
    else { pl.qb = 2; pl.kw = 1; }
    pl.wr = (4 / pl.kw) * pl.qb * 32;
    pl.row_blocks = (rows_g + pl.wr - 1) / pl.wr;
    pl.stages = (L + M + TK - 1) / TK;
    int base = Hkv * pl.row_blocks * batch;
    int want = g_split_override > 0 ? g_split_override : (256 + base - 1) / base;
    // a split should stream at least 8 tiles (256 keys) unless the caller forces it
    if (g_split_override <= 0) want = std::min(want, std::max(1, pl.stages / 8));
    want = std::max(1, std::min(want, pl.stages));
    pl.sps = (pl.stages + want - 1) / want;
    pl.nsplit = (pl.stages + pl.sps - 1) / pl.sps;
    return pl;
}

struct WsLayout { size_t anc, ml, opart, total; };

WsLayout ws_layout(int total_M, int Hq, int D, int nsplit)
{
    WsLayout w;
    size_t off = BTV_WS_HEADER;
    w.anc = off; off += btv_align_up((size_t)total_M * BTV_ANC_WORDS * 4, BTV_WS_ALIGN);
    size_t rows = (size_t)total_M * Hq;
    size_t ns = nsplit > 1 ? nsplit : 0;
    w.ml = off; off += btv_align_up(ns * rows * 2 * 4, BTV_WS_ALIGN);
    w.opart = off; off += btv_align_up(ns * rows * D * 4, BTV_WS_ALIGN);
    w.total = off;
    return w;
}

template <int D, int QB, int KW, int NS, bool PAGED>
int launch_bf16(const AttnParams &p, dim3 grid, hipStream_t st)
{
    constexpr int RING = NS * Lds<D>::STAGE;
    constexpr int MERGE = KW > 1 ? (4 / KW) * ((D / 32) * QB * 16 + 2 * QB) * 64 * 4 : 0;
    constexpr int LDS_BYTES = RING > MERGE ? RING : MERGE;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static bool configured = false;
    auto kern = tv_attn_bf16<D, QB, KW, NS, PAGED>;
    if (!configured) {
        BTV_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    LDS_BYTES));
        configured = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), LDS_BYTES, st, p);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

template <bool PAGED>
int dispatch_bf16(const AttnParams &p, const Plan &pl, int D, int batch, hipStream_t st)
{
    dim3 grid(pl.nsplit, pl.row_blocks, p.Hkv * batch);
#define BTV_CASE(DD, QQ, KK, NN) \
    if (D == DD && pl.qb == QQ && pl.kw == KK) return launch_bf16<DD, QQ, KK, NN, PAGED>(p, grid, st);
    BTV_CASE(128, 1, 4, 4) BTV_CASE(128, 2, 4, 6) BTV_CASE(128, 2, 2, 6) BTV_CASE(128, 2, 1, 6)
    BTV_CASE(64, 1, 4, 4) BTV_CASE(64, 2, 4, 6) BTV_CASE(64, 2, 2, 6) BTV_CASE(64, 2, 1, 6)
#undef BTV_CASE
    return btv_fail(BTV_EINVAL, "no kernel for D=%d", D);
}

int check_shape(int M, int L, int Hq, int Hkv, int D)
{
    BTV_REQUIRE(M >= 1 && M <= BTV_MAX_NODES, "M=%d outside [1,%d]", M, BTV_MAX_NODES);
    BTV_REQUIRE(L >= 0 && (long long)L + M < (1ll << 30), "L=%d out of range", L);
    BTV_REQUIRE(Hq >= 1 && Hkv >= 1 && Hq % Hkv == 0 && Hq / Hkv <= 16, "bad heads Hq=%d Hkv=%d", Hq, Hkv);
    BTV_REQUIRE(D == 64 || D == 128, "D=%d not in {64,128}", D);
    return BTV_OK;
}

}  // namespace

int btv_launch_anc_mask(const int32_t *parent, const int32_t *q_offset, int batch, int M_max, int total_M,
                        uint32_t *anc, uint32_t *flag, hipStream_t st)
{
    hipLaunchKernelGGL(anc_mask_kernel, dim3(batch), dim3(256), 0, st, parent, q_offset, M_max, total_M, anc, flag);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

extern "C" {

void btv_set_attn_splits(int nsplit) { g_split_override = nsplit > 0 ? nsplit : 0; }

int btv_tree_ancestor_mask(const int32_t *parent, int M, uint32_t *anc, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(parent && anc, "null pointer");
    BTV_REQUIRE(M >= 1 && M <= BTV_MAX_NODES, "M=%d outside [1,%d]", M, BTV_MAX_NODES);
    int rc = btv_check_ws(ws, ws_bytes, BTV_WS_HEADER);
    if (rc) return rc;
    return btv_launch_anc_mask(parent, nullptr, 1, M, M, anc, static_cast<uint32_t *>(ws),
                               static_cast<hipStream_t>(stream));
}

size_t btv_tree_verify_attn_workspace(int M, int L, int Hq, int Hkv, int D, int dtype)
{
    if (check_shape(M, L, Hq, Hkv, D) != BTV_OK) return 0;
    int nsplit = dtype == BTV_BF16 ? make_plan(M, L, Hq, Hkv, 1).nsplit : 1;
    return ws_layout(M, Hq, D, nsplit).total;
}

int btv_tree_verify_attn(const void *Q, const void *K, const void *V, const int32_t *parent, int M, int L, int Hq,
                         int Hkv, int D, int dtype, float scale, void *O, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(Q && K && V && parent && O, "null pointer");
    int rc = check_shape(M, L, Hq, Hkv, D);
    if (rc) return rc;
    BTV_REQUIRE(dtype == BTV_F32 || dtype == BTV_BF16, "dtype=%d unsupported", dtype);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Plan pl = make_plan(M, L, Hq, Hkv, 1);
    if (dtype == BTV_F32) pl.nsplit = 1;
    WsLayout wl = ws_layout(M, Hq, D, pl.nsplit);
    rc = btv_check_ws(ws, ws_bytes, wl.total);
    if (rc) return rc;
    unsigned char *w8 = static_cast<unsigned char *>(ws);
    AttnParams p = {};
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.anc = reinterpret_cast<uint32_t *>(w8 + wl.anc);
    p.ML = reinterpret_cast<float *>(w8 + wl.ml);
    p.Opart = reinterpret_cast<float *>(w8 + wl.opart);
    p.flag = reinterpret_cast<uint32_t *>(w8);
    p.M = M; p.L = L; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.total_rows = M * Hq; p.total_M = M;
    p.sps = pl.sps; p.nsplit = pl.nsplit;
    p.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    p.scale_log2 = p.scale * 1.4426950408889634f;
    rc = btv_launch_anc_mask(parent, nullptr, 1, M, M, const_cast<uint32_t *>(p.anc), p.flag, st);
    if (rc) return rc;
    if (dtype == BTV_F32) {
        if (D == 64) hipLaunchKernelGGL(tv_attn_f32<64>, dim3(M, Hq), dim3(256), 0, st, p);
        else hipLaunchKernelGGL(tv_attn_f32<128>, dim3(M, Hq), dim3(256), 0, st, p);
        BTV_HIP(hipGetLastError());
        return BTV_OK;
    }
    rc = dispatch_bf16<false>(p, pl, D, 1, st);
    if (rc) return rc;
    if (pl.nsplit > 1) {
        dim3 cg((M * Hq + 7) / 8, 1);
        if (D == 64) hipLaunchKernelGGL((tv_combine_bf16<64, false>), cg, dim3(256), 0, st, p);
        else hipLaunchKernelGGL((tv_combine_bf16<128, false>), cg, dim3(256), 0, st, p);
        BTV_HIP(hipGetLastError());
    }
    return BTV_OK;
}

size_t btv_tree_verify_attn_paged_workspace(int batch, int M_max, int L_max, int Hq, int Hkv, int D)
{
    if (batch < 1 || batch > 4096 || check_shape(M_max, L_max, Hq, Hkv, D) != BTV_OK) return 0;
    Plan pl = make_plan(M_max, L_max, Hq, Hkv, batch);
    return ws_layout(batch * M_max, Hq, D, pl.nsplit).total;
}

int btv_tree_verify_attn_paged(const void *Q, const void *Kpool, const void *Vpool, int num_blocks,
                               const int32_t *block_table, int max_blocks, const int32_t *q_offset,
                               const int32_t *prefix_len, const int32_t *parent, int batch, int total_M, int M_max,
                               int L_max, int Hq, int Hkv, int D, float scale, void *O, void *ws, size_t ws_bytes,
                               void *stream)
{
    BTV_REQUIRE(Q && Kpool && Vpool && block_table && q_offset && prefix_len && parent && O, "null pointer");
    BTV_REQUIRE(batch >= 1 && batch <= 4096, "batch=%d outside [1,4096]", batch);
    int rc = check_shape(M_max, L_max, Hq, Hkv, D);
    if (rc) return rc;
    BTV_REQUIRE(total_M >= 1 && total_M <= batch * M_max, "total_M=%d inconsistent with batch*M_max", total_M);
    BTV_REQUIRE(num_blocks >= 1 && max_blocks >= 1, "bad block counts");
    BTV_REQUIRE((long long)max_blocks * BTV_PAGE >= (long long)L_max + 1, "max_blocks too small for L_max");
    hipStream_t st = static_cast<hipStream_t>(stream);
    Plan pl = make_plan(M_max, L_max, Hq, Hkv, batch);
    WsLayout wl = ws_layout(batch * M_max, Hq, D, pl.nsplit);
    rc = btv_check_ws(ws, ws_bytes, wl.total);
    if (rc) return rc;
    unsigned char *w8 = static_cast<unsigned char *>(ws);
    AttnParams p = {};
    p.Q = Q; p.K = Kpool; p.V = Vpool; p.O = O;
    p.anc = reinterpret_cast<uint32_t *>(w8 + wl.anc);
    p.ML = reinterpret_cast<float *>(w8 + wl.ml);
    p.Opart = reinterpret_cast<float *>(w8 + wl.opart);
    p.flag = reinterpret_cast<uint32_t *>(w8);
    p.block_table = block_table; p.q_offset = q_offset; p.prefix_len = prefix_len;
    p.max_blocks = max_blocks; p.num_blocks = num_blocks;
    p.M = M_max; p.L = L_max; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.total_rows = batch * M_max * Hq;    // partial buffers are sized for the bound; rows index by q_offset
    p.total_M = total_M;
    p.sps = pl.sps; p.nsplit = pl.nsplit;
    p.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    p.scale_log2 = p.scale * 1.4426950408889634f;
    rc = btv_launch_anc_mask(parent, q_offset, batch, M_max, total_M, const_cast<uint32_t *>(p.anc), p.flag, st);
    if (rc) return rc;
    rc = dispatch_bf16<true>(p, pl, D, batch, st);
    if (rc) return rc;
    if (pl.nsplit > 1) {
        dim3 cg((M_max * Hq + 7) / 8, batch);
        if (D == 64) hipLaunchKernelGGL((tv_combine_bf16<64, true>), cg, dim3(256), 0, st, p);
        else hipLaunchKernelGGL((tv_combine_bf16<128, true>), cg, dim3(256), 0, st, p);
        BTV_HIP(hipGetLastError());
    }
    return BTV_OK;
}

}  // extern "C"
