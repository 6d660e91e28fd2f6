// Tree-masked attention for gfx950 (MI355X): ancestor bitmask, bf16 MFMA split-K kernel,
// fp32 reference-precision kernel, split-K combine, and the two C-ABI entry points.
//
// What is computed (App. C, "Linearization and verification mask"): node i attends to the L
// prefix rows of the KV cache and to the tree rows of its ancestors and itself.
//
// bf16 kernel layout.  For one KV head the G = Hq/Hkv query heads of every node are packed
// into rows r = i*G + j, so the whole GQA group shares each K/V byte that is streamed.
// A workgroup (4 wavefronts of 64 lanes) owns WR rows and a range of 64-key stages; K and V
// stages are staged through LDS once per workgroup (double buffered, register prefetch).
// Scores are computed transposed, S^T = K . Q^T with 32x32x16 bf16 MFMA: in the accumulator
// layout a lane then holds ONE query column and 16 keys, so the running max / sum of the
// online softmax are per-lane scalars (one cross-half exchange per tile), the P^T tile is
// already in B-operand layout for O^T += V^T . P^T, and the O^T accumulator is rescaled by a
// per-lane factor.  V is transposed on its way into LDS (pairs of keys per dword, XOR
// swizzled) so V^T tiles are plain 16-byte LDS reads.  The tree mask is applied only on tiles
// that touch tree rows, from a 32-bit visibility word per (query, tile) built from the node's
// ancestor bitmask.
#include "btv_common.h"

#include <algorithm>
#include <cmath>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 64;          // keys per LDS stage
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
// ------------------------------------------------------------------------------------------------
template <int D>
struct Lds {
    static constexpr int KROW = D + 8;                       // bf16 elements per K row (16 B pad)
    static constexpr int KBYTES = TK * KROW * 2;             // one K stage
    static constexpr int VBYTES = D * TK * 2;                // one V^T stage: D rows of TK keys
    static constexpr int STAGE = KBYTES + VBYTES;
    static constexpr int TOTAL = 2 * STAGE;
};

__device__ __forceinline__ int swap_bits_2_3(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// dword index inside a V^T stage for (row d, key-pair kp): 32 dwords per row, 16-byte columns XOR-swizzled.
__device__ __forceinline__ int vt_dword(int d, int kp)
{
    int sw = (d & 7) ^ ((d >> 3) & 7);
    return d * (TK / 2) + ((((kp >> 2) ^ sw) & 7) << 2) + (kp & 3);
}


template <bool PAGED>
struct StageCtx {
    const uint16_t *Kp, *Vp;
    const int32_t *block_table;
    int rq, max_blocks, num_blocks, Hkv, g, S;
    __device__ __forceinline__ long long row(int j) const
    {
        if (!PAGED) return j;
        int b = block_table[(long long)rq * max_blocks + (j >> 4)];
        b = min(max(b, 0), num_blocks - 1);
        return (long long)b * BTV_PAGE + (j & 15);
    }
};

// Global -> registers for one 64-key stage: each thread fetches D/32 16-byte pieces of K and of V.
// Keys past the end of the sequence re-read the last valid row (finite data; they are masked later).
template <int D, bool PAGED>
__device__ __forceinline__ void load_stage(const StageCtx<PAGED> &cx, int st, int tid, uint4 (&kreg)[D / 32],
                                           uint4 (&vreg)[D / 32])
{
    constexpr int CH = D / 8, NP = CH / 4, KPI = 128 / CH;
    const int kb = st * TK, w = tid >> 6, l = tid & 63;
#pragma unroll
    for (int r = 0; r < NP; ++r) {
        int piece = r * 256 + tid;
        int key = min(kb + piece / CH, cx.S - 1);
        kreg[r] = *reinterpret_cast<const uint4 *>(cx.Kp + (cx.row(key) * cx.Hkv + cx.g) * D + (piece % CH) * 8);
    }
#pragma unroll
    for (int r = 0; r < NP; ++r) {
        int key = min(kb + r * (4 * KPI) + w * KPI + 2 * (l / (2 * CH)) + (l & 1), cx.S - 1);
        vreg[r] = *reinterpret_cast<const uint4 *>(cx.Vp + (cx.row(key) * cx.Hkv + cx.g) * D + ((l >> 1) % CH) * 8);
    }
}

// Registers -> LDS.  K rows are stored in MFMA A-row order (bits 2 and 3 of the key index swapped) so that
// a lane's 16 score registers cover two runs of 8 consecutive keys; V is transposed: lanes 2x and 2x+1 hold
// two consecutive keys of the same 8 channels, exchange halves, and each writes 4 (channel, key-pair) dwords.
template <int D>
__device__ __forceinline__ void store_stage(unsigned char *smem, int buf, int tid, const uint4 (&kreg)[D / 32],
                                            const uint4 (&vreg)[D / 32])
{
    constexpr int CH = D / 8, NP = CH / 4, KPI = 128 / CH;
    using LD = Lds<D>;
    const int w = tid >> 6, l = tid & 63;
    uint16_t *Ks = reinterpret_cast<uint16_t *>(smem + buf * LD::STAGE);
    uint32_t *Vt = reinterpret_cast<uint32_t *>(smem + buf * LD::STAGE + LD::KBYTES);
#pragma unroll
    for (int r = 0; r < NP; ++r) {
        int piece = r * 256 + tid;
        int kk = piece / CH;
        int lrow = (kk & 32) | swap_bits_2_3(kk & 31);
        *reinterpret_cast<uint4 *>(Ks + lrow * LD::KROW + (piece % CH) * 8) = kreg[r];
    }
#pragma unroll
    for (int r = 0; r < NP; ++r) {
        const int par = l & 1;
        uint4 v = vreg[r];
        uint32_t s0 = par ? v.x : v.z, s1 = par ? v.y : v.w;
        uint32_t r0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)s0, 0xB1, 0xF, 0xF, true);
        uint32_t r1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)s1, 0xB1, 0xF, 0xF, true);
        uint32_t a0 = par ? r0 : v.x, a1 = par ? r1 : v.y;      // even key of the pair
        uint32_t b0 = par ? v.z : r0, b1 = par ? v.w : r1;      // odd key of the pair
        uint32_t o0 = (a0 & 0xFFFFu) | (b0 << 16);
        uint32_t o1 = (a0 >> 16) | (b0 & 0xFFFF0000u);
        uint32_t o2 = (a1 & 0xFFFFu) | (b1 << 16);
        uint32_t o3 = (a1 >> 16) | (b1 & 0xFFFF0000u);
        int kp = (r * (4 * KPI) + w * KPI + 2 * (l / (2 * CH))) >> 1;
        int d0 = ((l >> 1) % CH) * 8 + par * 4;
        Vt[vt_dword(d0 + 0, kp)] = o0;
        Vt[vt_dword(d0 + 1, kp)] = o1;
        Vt[vt_dword(d0 + 2, kp)] = o2;
        Vt[vt_dword(d0 + 3, kp)] = o3;
    }
}

// One 32-key tile of one wave: S^T = K.Q^T, tree mask, online softmax, O^T += V^T.P^T.
template <int D, int QB>
__device__ __forceinline__ void do_tile(const unsigned char *stage, int t, int kb, int Lr, int c, int h, float sl2,
                                        const uint32_t *anc, int q0, const int (&node)[QB],
                                        const bf16x8 (&qreg)[QB][D / 16], float (&m_run)[QB], float (&l_run)[QB],
                                        f32x16 (&oacc)[D / 32][QB])
{
    constexpr int DS = D / 16, DT = D / 32;
    using LD = Lds<D>;
    const uint16_t *Ks = reinterpret_cast<const uint16_t *>(stage);
    const uint32_t *Vt = reinterpret_cast<const uint32_t *>(stage + LD::KBYTES);
    f32x16 sacc[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[qb][v] = 0.f;
#pragma unroll
    for (int s = 0; s < DS; ++s) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(Ks + (t * 32 + c) * LD::KROW + s * 16 + h * 8);
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
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
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
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            int d = dt * 32 + c;
            int gi = t * 4 + mm * 2 + h;
            int sw = (d & 7) ^ ((d >> 3) & 7);
            bf16x8 a = *reinterpret_cast<const bf16x8 *>(Vt + d * (TK / 2) + (((gi ^ sw) & 7) << 2));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                oacc[dt][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][mm], oacc[dt][qb], 0, 0, 0);
        }
}

template <int D, int QB, int KW, bool PAGED>
__global__ __launch_bounds__(256, 1) void tv_attn_bf16(AttnParams p)
{
    constexpr int RW = 4 / KW;
    constexpr int WR = RW * QB * 32;
    constexpr int DS = D / 16;
    constexpr int DT = D / 32;
    constexpr int NP = D / 32;           // 16-byte pieces per thread per stage (K and V each)
    using LD = Lds<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

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
    const int stages = (S + TK - 1) / TK;
    const int nsplit_r = (stages + p.sps - 1) / p.sps;
    if ((int)blockIdx.x >= nsplit_r) return;
    const int st0 = blockIdx.x * p.sps, st1 = min(st0 + p.sps, stages);

    const uint16_t *Qp = static_cast<const uint16_t *>(p.Q);
    const uint16_t *Kp = static_cast<const uint16_t *>(p.K);
    const uint16_t *Vp = static_cast<const uint16_t *>(p.V);

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

    // ---- main loop over the stages of this split -----------------------------------------------
    uint4 kreg[NP], vreg[NP];
    const StageCtx<PAGED> cx = { Kp, Vp, p.block_table, rq, p.max_blocks, p.num_blocks, p.Hkv, g, S };
    load_stage<D, PAGED>(cx, st0, tid, kreg, vreg);
    store_stage<D>(smem, 0, tid, kreg, vreg);
    __syncthreads();
    for (int st = st0; st < st1; ++st) {
        const int buf = (st - st0) & 1;
        const bool more = st + 1 < st1;
        if (more) load_stage<D, PAGED>(cx, st + 1, tid, kreg, vreg);
#pragma unroll
        for (int t = 0; t < TK / 32; ++t) {
            if (t % KW != kw) continue;
            int kb = st * TK + t * 32;
            if (kb < S)
                do_tile<D, QB>(smem + buf * LD::STAGE, t, kb, Lr, c, h, p.scale_log2, p.anc, rq_.q0, node, qreg, m_run,
                               l_run, oacc);
        }
        if (more) store_stage<D>(smem, buf ^ 1, tid, kreg, vreg);
        __syncthreads();
    }

    // both halves of a wave hold partial row sums of the same queries
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += __shfl_xor(l_run[qb], 32);

    // ---- merge the key-split waves of this workgroup through LDS -----------------------------
    if (KW > 1) {
        constexpr int SLOT = (DT * QB * 16 + 2 * QB) * 64;    // floats per row-wave slot
        float *mg = reinterpret_cast<float *>(smem) + rw * SLOT;
        if (kw == 1) {
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

Plan make_plan(int M, int L, int Hq, int Hkv, int batch)
{
    Plan pl;
    int G = Hq / Hkv, rows_g = G * M;
    if (rows_g <= 64) { pl.qb = 1; pl.kw = 2; }
    else if (rows_g <= 128) { pl.qb = 2; pl.kw = 2; }
    else { pl.qb = 2; pl.kw = 1; }
    pl.wr = (4 / pl.kw) * pl.qb * 32;
    pl.row_blocks = (rows_g + pl.wr - 1) / pl.wr;
    pl.stages = (L + M + TK - 1) / TK;
    int base = Hkv * pl.row_blocks * batch;
    int want = g_split_override > 0 ? g_split_override : (256 + base - 1) / base;
    // a split should stream at least 4 stages (256 keys) unless the caller forces it
    if (g_split_override <= 0) want = std::min(want, std::max(1, pl.stages / 4));
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

template <int D, int QB, int KW, bool PAGED>
int launch_bf16(const AttnParams &p, dim3 grid, hipStream_t st)
{
    static bool configured = false;
    auto kern = tv_attn_bf16<D, QB, KW, PAGED>;
    if (!configured) {
        BTV_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    Lds<D>::TOTAL));
        configured = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), Lds<D>::TOTAL, st, p);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

template <bool PAGED>
int dispatch_bf16(const AttnParams &p, const Plan &pl, int D, int batch, hipStream_t st)
{
    dim3 grid(pl.nsplit, pl.row_blocks, p.Hkv * batch);
#define BTV_CASE(DD, QQ, KK) \
    if (D == DD && pl.qb == QQ && pl.kw == KK) return launch_bf16<DD, QQ, KK, PAGED>(p, grid, st);
    BTV_CASE(128, 1, 2) BTV_CASE(128, 2, 2) BTV_CASE(128, 2, 1)
    BTV_CASE(64, 1, 2) BTV_CASE(64, 2, 2) BTV_CASE(64, 2, 1)
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
