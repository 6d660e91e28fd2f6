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

#include <atomic>

#include <algorithm>
#include <cmath>
#include <type_traits>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 32;          // keys per tile = per LDS stage
constexpr float NEG_BIG = -1.0e30f;

struct AttnParams {
    const void *Q, *K, *V;
    void *O;
    const int32_t *parent;        // [total_M], indices local to each request
    const uint32_t *anc;          // [total_M][BTV_ANC_WORDS], fp32 path only
    const int32_t *block_table;   // paged only
    const int32_t *q_offset;      // paged only, [batch+1]
    const int32_t *prefix_len;    // paged only, [batch]
    _Float16 *Opart;              // [nsplit][total_rows][D]: split partial of O^T's row, divided by its largest magnitude
    float *ML;                    // [nsplit][total_rows][4]: reference max, row sum, that magnitude, unused
    uint32_t *flag;
    int M, L;                     // contiguous: actual sizes; paged: host upper bounds
    int Hq, Hkv, G;
    int max_blocks, num_blocks;
    int total_rows;               // rows of the partial buffers (>= total_M * Hq)
    int total_M;
    int sps;                      // stages per split
    int nsplit;                   // key splits of the longest request
    int row_blocks, units;        // row blocks per (split, head, request) unit; number of units
    float scale;                  // softmax scale
    float scale_log2;             // scale * log2(e) (times the key scale of an FP8 cache)
    float out_scale;              // 1, or the value scale of an FP8 cache
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

// Visibility of keys kb..kb+31 for a node: bit c set iff key kb+c is a prefix row, or a tree
// row L+a with a in anc(node).  Bits of anc past the request's node count are zero.
// AncT is either a pointer to the node's BTV_ANC_WORDS words or a register array of them.
template <typename AncT>
__device__ __forceinline__ uint32_t anc_word(const AncT &anc, int w)
{
    uint32_t r = 0u;
#pragma unroll
    for (int k = 0; k < BTV_ANC_WORDS; ++k) r = (k == w) ? anc[k] : r;
    return r;
}

template <typename AncT>
__device__ __forceinline__ uint32_t vis_word(const AncT &anc, int kb, int L)
{
    int off = kb - L;
    if (off <= -32) return 0xFFFFFFFFu;
    if (off < 0) {
        int n = -off;
        return ((1u << n) - 1u) | (anc_word(anc, 0) << n);
    }
    int w = off >> 5, sh = off & 31;
    uint32_t lo = anc_word(anc, w), hi = anc_word(anc, w + 1);
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
// EB = bytes per K/V element in memory and in LDS: 2 (bf16) or 1 (FP8 E4M3, converted to bf16 in registers after
// the operand reads: every E4M3 number is a bf16 number, so the conversion is exact).
template <int D, int EB = 2>
struct Lds {
    static constexpr int ROWB = EB * D;                      // bytes per K or V row
    static constexpr int TILEB = 32 * ROWB;                  // one K (or V) tile
    static constexpr int STAGE = 2 * TILEB;                  // K tile then V tile
    static constexpr int INSTR = STAGE / 1024;               // wave-wide 1 KiB fills per tile
    static constexpr int CHUNKS = ROWB / 16;                 // 16-byte chunks per row
};

__device__ __forceinline__ int swap_bits_2_3(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// bf16 rows (2*D bytes): consecutive rows start on the same bank, so the chunk is rotated by the row number.
// FP8 rows of 128 bytes: even and odd rows already sit in different halves of the 64 banks, so pairs of rows share a
// rotation.
template <int D, int EB = 2> __device__ __forceinline__ int swz_k(int row)
{
    return EB == 2 ? (row & (D / 8 - 1)) : ((row >> 1) & (Lds<D, EB>::CHUNKS - 1));
}
// V rows, bf16: the four rows a 16-lane group of a transposing read touches (row % 4 = 0..3) are moved 64 bytes
// apart.  FP8: a group touches 8 rows x 16 bytes and two groups (32 bytes per row) are served together; the four
// even (and the four odd) rows among them are moved 32 bytes apart.
template <int D, int EB = 2> __device__ __forceinline__ int swz_v(int row)
{
    return EB == 2 ? (((row & 3) << 2) & (D / 8 - 1)) : ((((row >> 1) & 3) << 1) & (Lds<D, EB>::CHUNKS - 1));
}

#define BTV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// Per-wave, loop-invariant part of the ring fills.  A wave issues LPW fills per tile; fill jj of wave w is
// instruction j = w*LPW + jj of the tile (K part first).  Lane l of it fills LDS row r, physical chunk pc, with
// source row key_off (relative to the tile's first key) and source chunk pc ^ swizzle(r).
template <int D, int WAVES, bool PAGED, int EB = 2>
struct Fill {
    static constexpr int LPW = Lds<D, EB>::INSTR / WAVES;
    static_assert(LPW >= 1 && LPW * WAVES == Lds<D, EB>::INSTR, "fills must divide evenly over the waves");
    const unsigned char *base[LPW]; // K or V base of this KV head for fill jj (wave-uniform)
    const int32_t *block_table;     // row of this request (paged)
    int num_blocks, S;
    uint32_t row_bytes;             // Hkv * D * EB: distance between consecutive keys
    uint32_t lane_off[LPW];         // contiguous: key_off*row_bytes + chunk*16;  paged: (key_off & 15)*row_bytes + chunk*16
};

template <int D, int WAVES, bool PAGED, int EB = 2>
__device__ __forceinline__ Fill<D, WAVES, PAGED, EB> make_fill(const void *K, const void *V, const int32_t *bt, int num_blocks,
                                                               int Hkv, int g, int S, int w, int l)
{
    using LD = Lds<D, EB>;
    constexpr int CH = LD::CHUNKS, RPI = 1024 / LD::ROWB;
    Fill<D, WAVES, PAGED, EB> f;
    const uintptr_t Kb = reinterpret_cast<uintptr_t>(K) + (size_t)g * D * EB, Vb = reinterpret_cast<uintptr_t>(V) + (size_t)g * D * EB;
    f.block_table = bt; f.num_blocks = num_blocks; f.S = S;
    f.row_bytes = (uint32_t)Hkv * D * EB;
#pragma unroll
    for (int jj = 0; jj < f.LPW; ++jj) {
        const int j = w * f.LPW + jj;
        const bool isv = j >= LD::TILEB / 1024;      // wave-uniform: this fill belongs to the V part
        f.base[jj] = reinterpret_cast<const unsigned char *>(isv ? Vb : Kb);
        const int jt = isv ? j - LD::TILEB / 1024 : j;
        const int r = jt * RPI + l / CH, pc = l % CH;
        const int key_off = isv ? r : swap_bits_2_3(r);
        const int chunk = pc ^ (isv ? swz_v<D, EB>(r) : swz_k<D, EB>(r));
        f.lane_off[jj] = (uint32_t)(PAGED ? (key_off & 15) : key_off) * f.row_bytes + chunk * 16;
    }
    return f;
}

// Source row (relative to the tile's first key) of lane l in fill jj of wave w: recomputed where it is needed (the
// clamped last tile, paged addressing) rather than kept in registers through the main loop.
template <int D, int WAVES, int EB>
__device__ __forceinline__ int fill_key_off(int w, int jj, int l)
{
    using LD = Lds<D, EB>;
    constexpr int CH = LD::CHUNKS, RPI = 1024 / LD::ROWB, LPW = LD::INSTR / WAVES;
    const int j = w * LPW + jj;
    const bool isv = j >= LD::TILEB / 1024;
    const int r = (isv ? j - LD::TILEB / 1024 : j) * RPI + l / CH;
    return isv ? r : swap_bits_2_3(r);
}

// Issue this wave's share of the direct-to-LDS loads of tile `st` (keys 32*st ..) into ring slot `slot`.
// Keys past the end of the sequence re-read the last valid row (finite data; their scores are masked).
// JB .. JE - 1: which of the wave's LPW fills (all by default; the pipelined loop issues them one by one, each behind a
// group of MFMAs, because an issue holds its wave for about a hundred cycles).
template <int D, int WAVES, bool PAGED, int EB = 2, int JB = 0, int JE = Lds<D, EB>::INSTR / WAVES>
__device__ __forceinline__ void issue_tile(const Fill<D, WAVES, PAGED, EB> &f, unsigned char *smem, int slot, int st, int w, int l)
{
    using LD = Lds<D, EB>;
    const int kb = st * 32;
    const bool whole = kb + 32 <= f.S;       // uniform: no key of this tile needs clamping
    if (!PAGED) {
        const size_t tile_off = (size_t)kb * f.row_bytes;
#pragma unroll
        for (int jj = JB; jj < JE; ++jj) {
            const unsigned char *base = f.base[jj] + tile_off;          // uniform
            uint32_t off = f.lane_off[jj];
            if (!whole) {
                const int ko = fill_key_off<D, WAVES, EB>(w, jj, l);
                off = off - (uint32_t)ko * f.row_bytes + (uint32_t)(min(kb + ko, f.S - 1) - kb) * f.row_bytes;
            }
            __builtin_amdgcn_global_load_lds(base + off, BTV_LDS_PTR(smem + slot * LD::STAGE + (w * f.LPW + jj) * 1024), 16, 0, 0);
        }
    } else {
        // a 32-key tile spans two 16-token pages; their ids are wave-uniform (scalar loads, so the vector-memory
        // counter only ever counts the LDS fills)
        const int last_page = (f.S - 1) >> 4;
        typedef const __attribute__((address_space(4))) int32_t *const_i32;   // constant space: scalar loads
        const_i32 bt = reinterpret_cast<const_i32>(reinterpret_cast<uintptr_t>(f.block_table));
        const int i0 = __builtin_amdgcn_readfirstlane(min(2 * st, last_page));
        const int i1 = __builtin_amdgcn_readfirstlane(min(2 * st + 1, last_page));
        const int id0 = bt[i0], id1 = bt[i1];
        asm volatile("" ::"s"(id0), "s"(id1));                   // both loads are issued before either id is used: one wait, not two
        const size_t page0 = (size_t)min(max(id0, 0), f.num_blocks - 1) * BTV_PAGE * f.row_bytes;
        const size_t page1 = (size_t)min(max(id1, 0), f.num_blocks - 1) * BTV_PAGE * f.row_bytes;
        if (whole) {
            // The rows of one fill instruction all lie in the same half of the tile (an instruction covers 4 or 8
            // consecutive LDS rows, and the K rows' permutation stays within 16), so the page is the instruction's,
            // not the lane's: a scalar base plus the lane's fixed offset, as in the contiguous form.
            // The rows of one fill instruction all lie in the same half of the tile (an instruction covers 4 or 8
            // consecutive LDS rows, and the permutation of the K rows stays within 16), so the page is the
            // instruction's, not the lane's: a scalar base plus the lane's fixed offset, as in the contiguous form.
#pragma unroll
            for (int jj = JB; jj < JE; ++jj) {
                const unsigned char *b = f.base[jj];
                const int row0 = fill_key_off<D, WAVES, EB>(w, jj, 0);      // (uniform: the key of the instruction's first lane)
                const unsigned char *src = b + ((row0 & 16) ? page1 : page0) + f.lane_off[jj];
                __builtin_amdgcn_global_load_lds(src, BTV_LDS_PTR(smem + slot * LD::STAGE + (w * f.LPW + jj) * 1024), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int jj = JB; jj < JE; ++jj) {
                const unsigned char *b = f.base[jj];
                const int ko = fill_key_off<D, WAVES, EB>(w, jj, l);
                const int kc = min(kb + ko, f.S - 1) - kb;
                const uint32_t off = f.lane_off[jj] - (uint32_t)(ko & 15) * f.row_bytes + (uint32_t)(kc & 15) * f.row_bytes;
                const unsigned char *src = b + ((kc & 16) ? page1 : page0) + off;
                __builtin_amdgcn_global_load_lds(src, BTV_LDS_PTR(smem + slot * LD::STAGE + (w * f.LPW + jj) * 1024), 16, 0, 0);
            }
        }
    }
}

// ---- LDS operand reads ---------------------------------------------------------------------------
// All operand reads are raw instructions with explicit counter waits: as ordinary loads / builtins the
// compiler would drain the whole vector-memory queue (the ring fills still in flight) in front of every tile.
// Each wait takes the registers it covers as in/out operands, so no use can be scheduled above it.
//
// K A-operands: lane (c = l%32, h = l/32) reads chunk (2s+h) ^ swz_k(c) of LDS row c for s = 0..D/16-1.  Row
// starts are 2*D-byte aligned, so the address is  (tile + lane part) ^ (s << 5).
template <int D> __device__ __forceinline__ uint32_t lane_k_off(int l)
{
    const int c = l & 31, h = l >> 5;
    return (uint32_t)(c * Lds<D>::ROWB + ((h ^ swz_k<D>(c)) << 4));
}

template <int D> __device__ __forceinline__ void lds_read_k(uint32_t a, u32x4 (&ka)[D / 16])
{
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        const uint32_t addr = a ^ (uint32_t)(s << 5);
        asm volatile("ds_read_b128 %0, %1" : "=v"(ka[s]) : "v"(addr));
    }
}

template <int DS, int YOUNGER> __device__ __forceinline__ void lds_wait_k(u32x4 (&ka)[DS])
{
    static_assert(DS == 4 || DS == 8, "D in {64,128}");
    if constexpr (DS == 8)
        asm volatile("s_waitcnt lgkmcnt(%8)"
                     : "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]), "+v"(ka[4]), "+v"(ka[5]), "+v"(ka[6]), "+v"(ka[7])
                     : "n"(YOUNGER));
    else
        asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]) : "n"(YOUNGER));
}

// V^T A-operands (ds_read_b64_tr_b16): lane l sits in 16-lane group l/16 = 2h + dhalf; for (dt, mm, i) it
// supplies the address of key row 16mm + 8h + 4i + (l%16)/4, channels 32dt + 16dhalf + 4(l%4) .. +3, and
// receives keys 16mm + 8h + 4i .. +3 of channel 32dt + (l%32).  With the V swizzle the address is
// ((tile + lane part) ^ (dt << 6)) + (16mm + 4i) * row bytes, the last term an immediate offset.
template <int D> __device__ __forceinline__ uint32_t lane_v_off(int l)
{
    const int h = l >> 5, dhalf = (l >> 4) & 1, rr = (l & 15) >> 2, q = l & 3;
    const int x = 2 * dhalf + (q >> 1);
    return (uint32_t)((8 * h + rr) * Lds<D>::ROWB + ((swz_v<D>(rr) ^ x) << 4) + ((q & 1) << 3));
}

// The reads for keys 16*MM .. 16*MM + 15 (the operands of the PV MFMAs with index mm = MM): 2*D/32 instructions.
template <int D, int MM> __device__ __forceinline__ void lds_read_vt(uint32_t a, bf16x4 (&va)[D / 32][2][2])
{
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
        const uint32_t addr = a ^ (uint32_t)(dt << 6);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                         : "=v"(va[dt][MM][i])
                         : "v"(addr), "n"((16 * MM + 4 * i) * Lds<D>::ROWB));
    }
}

template <int DT>
__device__ __forceinline__ void lds_wait_vt(bf16x4 (&va)[DT][2][2])
{
    static_assert(DT == 2 || DT == 4, "D in {64,128}");
    if constexpr (DT == 4)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(va[0][0][0]), "+v"(va[0][0][1]), "+v"(va[0][1][0]), "+v"(va[0][1][1]), "+v"(va[1][0][0]),
                       "+v"(va[1][0][1]), "+v"(va[1][1][0]), "+v"(va[1][1][1]), "+v"(va[2][0][0]), "+v"(va[2][0][1]),
                       "+v"(va[2][1][0]), "+v"(va[2][1][1]), "+v"(va[3][0][0]), "+v"(va[3][0][1]), "+v"(va[3][1][0]),
                       "+v"(va[3][1][1]));
    else
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(va[0][0][0]), "+v"(va[0][0][1]), "+v"(va[0][1][0]), "+v"(va[0][1][1]), "+v"(va[1][0][0]),
                       "+v"(va[1][0][1]), "+v"(va[1][1][0]), "+v"(va[1][1][1]));
}

// ---- the arithmetic steps of one 32-key tile of one wave (32 query rows) ---------------------------------
// S^T = K . Q^T
template <int DS>
__device__ __forceinline__ f32x16 qk_tile(const u32x4 (&ka)[DS], const bf16x8 (&qreg)[DS], f32x16 s)
{
#pragma unroll
    for (int k = 0; k < DS; ++k)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[k]), qreg[k], s, 0, 0, 0);
    return s;
}

// largest score of the lane's query over the 32 keys (the other half of the wave holds the other 16)
__device__ __forceinline__ float tile_max(const f32x16 &s)
{
    float t = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) t = fmaxf(t, s[v]);
    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

// Scores arrive in log2 units: the queries were multiplied by scale * log2(e) once, in the prologue, so a
// probability is exp2(score - reference) with no multiply per element.
//
// Lazy reference maximum: m_run only moves when the tile maximum exceeds it by more than LAZY, so probabilities
// stay below 2^LAZY and the O^T / row-sum rescale is skipped on most tiles.  The result is unchanged: numerator
// and denominator refer to the same m_run.
template <int DT>
__device__ __forceinline__ void lazy_rescale(float tmax, float &m_run, float &l_run, f32x16 (&oacc)[DT])
{
    constexpr float LAZY = 8.0f;
    const bool grow = tmax - m_run > LAZY;
    if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
        const float mnew = grow ? tmax : m_run;
        const float alpha = __builtin_amdgcn_exp2f(m_run - mnew);
        m_run = mnew;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
    }
}

// P^T = exp2(S^T - m_run) as bf16 B-operands; the row sum adds the rounded values PV uses
// (v_dot2c_f32_bf16 against (1, 1): two probabilities per instruction).
__device__ __forceinline__ void softmax_tile(const f32x16 &s, float m_run, float &l_run, bf16x8 (&pb)[2])
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = { (__bf16)1.0f, (__bf16)1.0f };
    float ls[2] = { l_run, 0.f };
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(s[mm * 8 + e] - m_run);
            const float p1 = __builtin_amdgcn_exp2f(s[mm * 8 + e + 1] - m_run);
            const bf16x2 pp = { (__bf16)p0, (__bf16)p1 };
            pb[mm][e] = pp[0];
            pb[mm][e + 1] = pp[1];
            ls[mm] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, ls[mm], false);
        }
    l_run = ls[0] + ls[1];
}

// One half (keys 8 mm .. 8 mm + 7 of the lane's 16) of a tile whose scores already are relative to the reference:
// P = exp2(x) as a B operand, its rounded values added to `sum`.
__device__ __forceinline__ void exp_half(const f32x16 &x, int mm, bf16x8 &pbm, float &sum)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = { (__bf16)1.0f, (__bf16)1.0f };
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(x[mm * 8 + e]);
        const float p1 = __builtin_amdgcn_exp2f(x[mm * 8 + e + 1]);
        const bf16x2 pp = { (__bf16)p0, (__bf16)p1 };
        pbm[e] = pp[0];
        pbm[e + 1] = pp[1];
        sum = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, sum, false);
    }
}

// The reference of the step-by-step tiles enters through the matrix cores as well: the score accumulator starts from
// -base (negb: the same value in all 16 registers), base being the running maximum once there is one (0 before), so
// the scores arrive relative to it and a probability is exp2 of the accumulator as it stands.  Only when the maximum
// moves (the lazy rule of lazy_rescale, on the scores' true values) are the tile's scores shifted by hand.
template <int DT>
__device__ __forceinline__ void rebase_tile(f32x16 &srel, float &base, f32x16 &negb, float &m_run, float &l_run, f32x16 (&oacc)[DT])
{
    constexpr float LAZY = 8.0f;
    const float rmax = tile_max(srel);
    const bool grow = (rmax + base) - m_run > LAZY;
    if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
        const float mnew = grow ? rmax + base : m_run;
        const float alpha = __builtin_amdgcn_exp2f(m_run - mnew);
        m_run = mnew;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
        const float nb = m_run > 0.5f * NEG_BIG ? m_run : 0.f;
        const float d = nb - base;
        base = nb;
#pragma unroll
        for (int v = 0; v < 16; ++v) { srel[v] -= d; negb[v] = -nb; }
    }
}

// P^T = exp2(x) for scores x already relative to the reference; the row sum adds the rounded values PV uses.
__device__ __forceinline__ void softmax_rel(const f32x16 &x, float &l_run, bf16x8 (&pb)[2])
{
    float ls[2] = { l_run, 0.f };
    exp_half(x, 0, pb[0], ls[0]);
    exp_half(x, 1, pb[1], ls[1]);
    l_run = ls[0] + ls[1];
}

// O^T += V^T . P^T
template <int DT>
__device__ __forceinline__ void pv_tile(const bf16x4 (&va)[DT][2][2], const bf16x8 (&pb)[2], f32x16 (&oacc)[DT])
{
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const bf16x8 a = __builtin_shufflevector(va[dt][mm][0], va[dt][mm][1], 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[mm], oacc[dt], 0, 0, 0);
        }
}

// tree mask of a tile that touches tree rows (or the end of the sequence)
__device__ __forceinline__ void mask_tile(f32x16 &s, uint32_t vis, int h)
{
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int bit = 16 * (v >> 3) + 8 * h + (v & 7);
        if (!((vis >> bit) & 1u)) s[v] = -INFINITY;
    }
}

// One whole tile, step after step (no overlap between the steps): used for the tiles that need the mask and
// by the workgroup shapes whose wave pairs alternate over the tiles.
template <int D>
__device__ __forceinline__ void do_tile(uint32_t stage, int kb, int Lr, int l,
                                        const uint32_t (&anc_i)[BTV_ANC_WORDS],
                                        const bf16x8 (&qreg)[D / 16], float &m_run, float &l_run, f32x16 (&oacc)[D / 32],
                                        float &base, f32x16 &negb)
{
    constexpr int DS = D / 16, DT = D / 32;
    u32x4 ka[DS];
    bf16x4 va[DT][2][2];
    const uint32_t va_addr = stage + Lds<D>::TILEB + lane_v_off<D>(l);
    lds_read_k<D>(stage + lane_k_off<D>(l), ka);
    lds_read_vt<D, 0>(va_addr, va);
    lds_wait_k<DS, DT * 2>(ka);          // the counter completes in order: K has landed when 2*DT reads remain
    lds_read_vt<D, 1>(va_addr, va);
    f32x16 s = qk_tile<DS>(ka, qreg, negb);
    if (kb + 32 > Lr) mask_tile(s, vis_word(anc_i, kb, Lr), l >> 5);
    rebase_tile<DT>(s, base, negb, m_run, l_run, oacc);
    bf16x8 pb[2];
    softmax_rel(s, l_run, pb);
    lds_wait_vt<DT>(va);
    pv_tile<DT>(va, pb, oacc);
}

// ---- FP8 (E4M3) K/V: operand reads and exact conversion to bf16 ---------------------------------------
// K: a lane reads 16 consecutive channels (16 bytes) of its key row, channels 32 s + 16 h .. + 15 for s = 0 .. D/32-1,
// and uses the first 8 for contraction step 2s, the last 8 for step 2s+1.  The contraction steps thus take the
// channels in another order than the bf16 layout; the query operands are loaded in the same order, so the sum is
// over the same products.  Address: (tile + lane part) ^ (s << 5), as for bf16 with 128-byte rows.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int D> __device__ __forceinline__ uint32_t lane_k8_off(int l)
{
    const int c = l & 31, h = l >> 5;
    return (uint32_t)(c * Lds<D, 1>::ROWB + ((h ^ swz_k<D, 1>(c)) << 4));
}

template <int D> __device__ __forceinline__ void lds_read_k8(uint32_t a, u32x4 (&k8)[D / 32])
{
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        const uint32_t addr = a ^ (uint32_t)(s << 5);
        asm volatile("ds_read_b128 %0, %1" : "=v"(k8[s]) : "v"(addr));
    }
}

template <int YOUNGER> __device__ __forceinline__ void lds_wait_k8(u32x4 (&k8)[4])
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(k8[0]), "+v"(k8[1]), "+v"(k8[2]), "+v"(k8[3]) : "n"(YOUNGER));
}

// Two E4M3 codes (one 16-bit half of a register) to two bf16, scale 1: exact for every code.
__device__ __forceinline__ uint32_t fp8x2_to_bf16x2(uint32_t w, bool high)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 r = high ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true)
                          : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
    return __builtin_bit_cast(uint32_t, r);
}

// eight consecutive codes (two registers) -> one bf16 MFMA operand
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t w0, uint32_t w1)
{
    const u32x4 r = { fp8x2_to_bf16x2(w0, false), fp8x2_to_bf16x2(w0, true), fp8x2_to_bf16x2(w1, false),
                      fp8x2_to_bf16x2(w1, true) };
    return __builtin_bit_cast(bf16x8, r);
}

// V^T operands (ds_read_b64_tr_b8): a 16-lane group reads 8 key rows x 16 channels; lane j of the group supplies
// the address of row j/2, bytes 8 (j%2) .. + 7 of the group's 16 channels, and receives the 8 keys of channel j.
// Lane l sits in group l/16 = 2h + dhalf; for (dt, mm) the group reads keys 16mm + 8h .. + 7, channels
// 32dt + 16dhalf .. + 15, so the lane receives keys 16mm + 8h .. + 7 of channel 32dt + (l%32): one whole operand
// of the PV MFMA with index mm.  With the V swizzle the address is ((tile + lane part) ^ (dt << 5)) + 16mm * row
// bytes, the last term an immediate offset.
template <int D> __device__ __forceinline__ uint32_t lane_v8_off(int l)
{
    const int h = l >> 5, dhalf = (l >> 4) & 1, j = l & 15;
    const int row = 8 * h + (j >> 1);
    return (uint32_t)(row * Lds<D, 1>::ROWB + ((swz_v<D, 1>(row) ^ dhalf) << 4) + ((j & 1) << 3));
}

template <int D, int MM> __device__ __forceinline__ void lds_read_vt8(uint32_t a, u32x2 (&v8)[D / 32][2])
{
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
        const uint32_t addr = a ^ (uint32_t)(dt << 5);
        asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(v8[dt][MM]) : "v"(addr), "n"(16 * MM * Lds<D, 1>::ROWB));
    }
}

__device__ __forceinline__ void lds_wait_vt8(u32x2 (&v8)[4][2])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(v8[0][0]), "+v"(v8[0][1]), "+v"(v8[1][0]), "+v"(v8[1][1]), "+v"(v8[2][0]), "+v"(v8[2][1]),
                   "+v"(v8[3][0]), "+v"(v8[3][1]));
}

// One whole tile of an FP8 cache: the same steps as do_tile with half the operand reads and the conversions.
template <int D>
__device__ __forceinline__ void do_tile8(uint32_t stage, int kb, int Lr, int l,
                                         const uint32_t (&anc_i)[BTV_ANC_WORDS],
                                         const bf16x8 (&qreg)[D / 16], float &m_run, float &l_run, f32x16 (&oacc)[D / 32])
{
    static_assert(D == 128, "FP8 K/V: head dimension 128 only");
    constexpr int DS = D / 16, DT = D / 32;
    u32x4 k8[DS / 2];
    u32x2 v8[DT][2];
    const uint32_t va_addr = stage + Lds<D, 1>::TILEB + lane_v8_off<D>(l);
    lds_read_k8<D>(stage + lane_k8_off<D>(l), k8);
    lds_read_vt8<D, 0>(va_addr, v8);
    lds_wait_k8<DT>(k8);                 // the counter completes in order: K has landed when DT reads remain
    lds_read_vt8<D, 1>(va_addr, v8);
    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int k = 0; k < DS / 2; ++k) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fp8x8_to_bf16x8(k8[k][0], k8[k][1]), qreg[2 * k], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fp8x8_to_bf16x8(k8[k][2], k8[k][3]), qreg[2 * k + 1], s, 0, 0, 0);
    }
    if (kb + 32 > Lr) mask_tile(s, vis_word(anc_i, kb, Lr), l >> 5);
    lazy_rescale<DT>(tile_max(s), m_run, l_run, oacc);
    bf16x8 pb[2];
    softmax_tile(s, m_run, l_run, pb);
    lds_wait_vt8(v8);
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fp8x8_to_bf16x8(v8[dt][mm][0], v8[dt][mm][1]), pb[mm],
                                                               oacc[dt], 0, 0, 0);
}

// ---- half-tile operand buffers of the software-pipelined loop ----------------------------------------------
// The loop keeps 16 registers of K operands and 16 of V^T operands (D = 128): half a tile each, refilled right
// after the MFMAs that consumed the previous contents were issued.  Addresses are loop-invariant registers (one
// per contraction step / channel block, the XOR of the swizzle already applied); the ring slot is an immediate
// offset, which reaches SPB slots from one base (the offset field has 16 bits).
template <int OFF> __device__ __forceinline__ void ds_read_k_imm(uint32_t a, u32x4 &r)
{
    static_assert(OFF >= 0 && OFF < 65536, "immediate offset range");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(a), "n"(OFF));
}
template <int OFF> __device__ __forceinline__ void ds_read_vt_imm(uint32_t a, bf16x4 &r)
{
    static_assert(OFF >= 0 && OFF < 65536, "immediate offset range");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(a), "n"(OFF));
}

// K operands of contraction steps HALF * DS/2 .. + DS/2 - 1 of the tile in slot SLOT (relative to the base in ak).
template <int D, int SLOT, int HALF> __device__ __forceinline__ void read_k_half(const uint32_t (&ak)[D / 16], u32x4 (&kh)[D / 32])
{
#pragma unroll
    for (int s = 0; s < D / 32; ++s) ds_read_k_imm<SLOT * Lds<D>::STAGE>(ak[HALF * (D / 32) + s], kh[s]);
}
// V^T operands of keys 16 MM .. 16 MM + 15 (the PV MFMAs with index MM), all channel blocks.
template <int D, int SLOT, int MM> __device__ __forceinline__ void read_v_half(const uint32_t (&av)[D / 32], bf16x4 (&vh)[D / 32][2])
{
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
        ds_read_vt_imm<SLOT * Lds<D>::STAGE + (16 * MM) * Lds<D>::ROWB>(av[dt], vh[dt][0]);
        ds_read_vt_imm<SLOT * Lds<D>::STAGE + (16 * MM + 4) * Lds<D>::ROWB>(av[dt], vh[dt][1]);
    }
}
// the same reads with the stage address in a register (prologue and epilogue of the loop)
template <int D, int HALF> __device__ __forceinline__ void read_k_half_at(uint32_t a, u32x4 (&kh)[D / 32])
{
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        const uint32_t addr = a ^ (uint32_t)((HALF * (D / 32) + s) << 5);
        asm volatile("ds_read_b128 %0, %1" : "=v"(kh[s]) : "v"(addr));
    }
}
template <int D, int MM> __device__ __forceinline__ void read_v_half_at(uint32_t a, bf16x4 (&vh)[D / 32][2])
{
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
        const uint32_t addr = a ^ (uint32_t)(dt << 6);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[dt][i]) : "v"(addr), "n"((16 * MM + 4 * i) * Lds<D>::ROWB));
    }
}
// Wait until at most YOUNGER LDS reads issued after these are still in flight (the counter completes in order).
template <int KH, int YOUNGER> __device__ __forceinline__ void wait_k_half(u32x4 (&kh)[KH])
{
    static_assert((KH == 2 || KH == 4) && YOUNGER >= 0 && YOUNGER < 16, "D in {64,128}");
    if constexpr (KH == 4) asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(kh[0]), "+v"(kh[1]), "+v"(kh[2]), "+v"(kh[3]) : "n"(YOUNGER));
    else asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(kh[0]), "+v"(kh[1]) : "n"(YOUNGER));
}
template <int DT, int YOUNGER> __device__ __forceinline__ void wait_v_half(bf16x4 (&vh)[DT][2])
{
    static_assert((DT == 2 || DT == 4) && YOUNGER >= 0 && YOUNGER < 16, "D in {64,128}");
    if constexpr (DT == 4)
        asm volatile("s_waitcnt lgkmcnt(%8)"
                     : "+v"(vh[0][0]), "+v"(vh[0][1]), "+v"(vh[1][0]), "+v"(vh[1][1]), "+v"(vh[2][0]), "+v"(vh[2][1]),
                       "+v"(vh[3][0]), "+v"(vh[3][1])
                     : "n"(YOUNGER));
    else
        asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(vh[0][0]), "+v"(vh[0][1]), "+v"(vh[1][0]), "+v"(vh[1][1]) : "n"(YOUNGER));
}
// half of S^T = K . Q^T: contraction steps HALF * DS/2 .. on top of c
template <int DS, int HALF>
__device__ __forceinline__ f32x16 qk_half(const u32x4 (&kh)[DS / 2], const bf16x8 (&qreg)[DS], f32x16 c)
{
#pragma unroll
    for (int k = 0; k < DS / 2; ++k)
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kh[k]), qreg[HALF * (DS / 2) + k], c, 0, 0, 0);
    return c;
}
// half of O^T += V^T . P^T: the keys of one P operand
template <int DT> __device__ __forceinline__ void pv_half(const bf16x4 (&vh)[DT][2], const bf16x8 &pbm, f32x16 (&oacc)[DT])
{
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        const bf16x8 a = __builtin_shufflevector(vh[dt][0], vh[dt][1], 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pbm, oacc[dt], 0, 0, 0);
    }
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most `tiles` (wave-uniform, clamped to [0, MAXT]) tiles of LPW fills each are in flight.
template <int LPW, int MAXT> __device__ __forceinline__ void wait_tiles(int tiles)
{
    static_assert(MAXT * LPW < 64, "vmcnt range");
    if constexpr (MAXT > 0) {
        if (tiles >= MAXT) { wait_vmcnt<MAXT * LPW>(); return; }
        wait_tiles<LPW, MAXT - 1>(tiles);
    } else {
        wait_vmcnt<0>();
    }
}

// LDS map of one workgroup: the ring of NT stages; the query tiles (one per row-wave: its 32 rows as they lie in
// memory, 2*D bytes each, chunk-rotated like a bf16 K tile) in the top of the ring when the prologue's fills leave
// that free, else behind them; 1 KiB for the staged parent[] in a stage the prologue leaves free, else behind the
// query tiles.  Queries and parents are consumed before the main loop's first barrier, after which the ring owns
// every stage.  The merge of the key-waves re-uses the same memory after the loop.
template <int D, int RW, int KW, int NT, int EB>
struct WgLds {
    static constexpr int STAGE = Lds<D, EB>::STAGE;
    static constexpr int PREFILL = KW == 1 ? (NT - 1 < 3 ? NT - 1 : 3) : NT - KW;   // tiles issued before the main loop
    static constexpr int RING = NT * STAGE;
    static constexpr int QTILE = 32 * D * 2;
    static constexpr int QBYTES = RW * QTILE;
    static constexpr int PRE_B = PREFILL * STAGE;
    static constexpr int QOFF = RING - QBYTES > PRE_B ? RING - QBYTES : PRE_B;
    // parent[]: in a stage the prologue leaves free, else behind the query tiles; behind the ring for the pipelined
    // shape, which reads it after the plain prefix tiles
    static constexpr int PAROFF = KW == 1 ? (RING > QOFF + QBYTES ? RING : QOFF + QBYTES) : (QOFF - PRE_B >= 1024 ? PRE_B : QOFF + QBYTES);
    static constexpr int USED = (PAROFF + 1024 > QOFF + QBYTES ? PAROFF + 1024 : QOFF + QBYTES) > RING
                                    ? (PAROFF + 1024 > QOFF + QBYTES ? PAROFF + 1024 : QOFF + QBYTES) : RING;
    // two key-waves exchange half a row each (+ m, l, bound); more key-waves: donors to wave 0
    static constexpr int MERGE = KW == 2 ? RW * 2 * ((D / 64) * 16 + 3) * 64 * 4 : RW * (KW - 1) * ((D / 32) * 16 + 2) * 64 * 4;
    static constexpr int BYTES = USED > MERGE ? USED : MERGE;
    static_assert(QOFF % 1024 == 0 && PAROFF % 1024 == 0 && BYTES <= 160 * 1024, "LDS budget");
    static_assert(BTV_MAX_NODES * 4 <= 1024, "parent[] staging");
};

// Wait until at most n (wave-uniform, clamped to [0, MAXN]) vector-memory operations are in flight.
template <int MAXN> __device__ __forceinline__ void wait_vm_ops(int n)
{
    if constexpr (MAXN > 0) {
        if (n >= MAXN) { wait_vmcnt<MAXN>(); return; }
        wait_vm_ops<MAXN - 1>(n);
    } else {
        wait_vmcnt<0>();
    }
}

// A lane's query row: row r of a KV head's packed rows is node r / G, query head r % G of the group.  Worked out where
// it is needed (mask construction, final store) rather than held in registers through the main loop.  Padding rows
// (r >= rows_g) recompute row 0 and are never written.
struct LaneRow { bool valid; int node; long long orow; };
__device__ __forceinline__ LaneRow lane_row(int r, int rows_g, int G, int Hq, int g, int q0)
{
    LaneRow x;
    x.valid = r < rows_g;
    const int rr = x.valid ? r : 0;
    x.node = rr / G;
    x.orow = (long long)(q0 + x.node) * Hq + g * G + (rr % G);       // row of Q/O as [total_M*Hq, D]
    return x;
}

// Workgroup = RW row-waves x KW key-waves; wave (rw, kw) owns query rows [32 rw, 32 rw + 32) of the block and,
// in every round of KW consecutive tiles, tile number kw.  LDS ring of NT tiles; one barrier per round.
template <int D, int RW, int KW, int NT, bool PAGED, int EB = 2>
__global__ __launch_bounds__(RW * KW * 64, 2) void tv_attn_bf16(AttnParams p)
{
    static_assert(EB == 2 || (EB == 1 && KW >= 2), "FP8 K/V runs in the shapes whose waves alternate over the tiles");
    constexpr int WAVES = RW * KW;
    constexpr int WR = RW * 32;
    constexpr int DS = D / 16;
    constexpr int DT = D / 32;
    // Waves that issue the ring fills.  With two waves per SIMD the hardware favours the older wave of each pair,
    // which then idles at the round's barrier: those four waves issue every fill (an issue stalls its wave for
    // about a hundred cycles), the younger four only compute.
    constexpr int IW = WAVES;
    constexpr int LPW = Lds<D, EB>::INSTR / IW;
    constexpr int AHEAD = NT - 2 * KW;            // tiles still in flight when a round's tiles have landed
    static_assert(AHEAD >= 0 && AHEAD * LPW < 64, "ring too small or too deep for the counter");
    using LD = Lds<D, EB>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // Fetch every argument now, in one round trip.  Left to the compiler the scalar loads follow the early-exit tests
    // below in five dependent steps, three of which miss the cache (the argument block spans three lines and is cold
    // in every launch): about two microseconds before the first fill is issued.
    asm volatile("" ::"s"(p.Q), "s"(p.K), "s"(p.V), "s"(p.O), "s"(p.parent), "s"(p.block_table), "s"(p.q_offset),
                 "s"(p.prefix_len), "s"(p.Opart), "s"(p.ML), "s"(p.flag), "s"(p.M), "s"(p.L), "s"(p.Hq), "s"(p.Hkv), "s"(p.G),
                 "s"(p.max_blocks), "s"(p.num_blocks), "s"(p.total_rows), "s"(p.total_M), "s"(p.sps), "s"(p.nsplit),
                 "s"(p.row_blocks), "s"(p.units), "s"(p.scale_log2), "s"(p.out_scale));
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, c = l & 31, h = l >> 5;
    const int kw = w % KW, rw = w / KW;
    // Workgroups go to the 8 XCDs round-robin by their linear id.  A unit = (key split, KV head, request); the row
    // blocks of one unit stream the same K/V bytes, so they get ids that are congruent mod 8 and share one L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int by = slot % p.row_blocks, unit = (slot / p.row_blocks) * 8 + xcd;
    if (unit >= p.units) return;
    // Ragged batches: the split index is rotated by the (request, head) number.  Without it a split count that is
    // a multiple of 8 ties split i to XCD i % 8, and the requests with few splits load only the first XCDs.
    const int bz = unit / p.nsplit;
    const int bx = PAGED ? (unit % p.nsplit + 3 * bz) % p.nsplit : unit % p.nsplit;
    const int rq = bz / p.Hkv, g = bz % p.Hkv;
    const Req rq_ = load_req<PAGED>(p, rq);
    if (!rq_.ok) {
        if (tid == 0 && bx == 0 && by == 0) atomicOr(p.flag, 2u);
        return;
    }
    const int Mr = rq_.M, Lr = rq_.L, S = Lr + Mr;
    const int rows_g = Mr * p.G;
    if (by * WR >= rows_g) return;
    const int tiles = (S + 31) / 32;
    const int nsplit_r = (tiles + p.sps - 1) / p.sps;
    if (bx >= nsplit_r) return;
    const int st0 = bx * p.sps;
    int st1 = min(st0 + p.sps, tiles);
    {   // tree rows past the last node of this row block are invisible to all of its rows: their tiles are dropped
        const int node_hi = (min((by + 1) * WR, rows_g) - 1) / p.G;
        st1 = min(st1, max((Lr + node_hi + 1 + 31) / 32, st0 + 1));
    }

    using WL = WgLds<D, RW, KW, NT, EB>;

    // ---- prologue loads, oldest first: parent[] (one entry per thread), this wave's share of its row-wave's query
    // tile, the first ring tiles.  All are raw instructions counted by hand.
    // parent[]: every wave moves 64 entries straight into LDS (index clamped to the request's nodes), whether or not
    // the workgroup reaches the tree rows; entries are checked where they are read.
#pragma unroll
    for (int i0 = 0; i0 < BTV_MAX_NODES; i0 += WAVES * 64)
        if (tid + i0 < BTV_MAX_NODES) {              // wave-uniform: whole waves
            const int32_t *pp = p.parent + rq_.q0 + min(tid + i0, Mr - 1);
            const int dst = __builtin_amdgcn_readfirstlane(WL::PAROFF + ((tid + i0) >> 6) * 256);
            __builtin_amdgcn_global_load_lds(pp, BTV_LDS_PTR(smem + dst), 4, 0, 0);
        }
    // Query tile: direct-to-LDS like a K tile (each wave instruction moves 1 KiB: whole rows, coalesced); as
    // per-lane operand loads the same bytes cost 64 separate 16-byte pieces per instruction and held the ring fills
    // back by about two microseconds.  The KW waves of a row-wave share the tile's instructions.
    constexpr int QCH = D / 8, QRPI = 1024 / (2 * D), QINSTR = WL::QTILE / 1024, QPW = QINSTR / KW;
    static_assert(QPW * KW == QINSTR, "query tile instructions must divide over the key-waves");
#pragma unroll
    for (int jj = 0; jj < QPW; ++jj) {
        const int j = kw * QPW + jj;
        const int qrow = j * QRPI + l / QCH, pc = l % QCH;
        const int rf = by * WR + rw * 32 + qrow;
        const int rrf = rf < rows_g ? rf : 0;
        const long long of = (long long)(rq_.q0 + rrf / p.G) * p.Hq + g * p.G + (rrf % p.G);
        const unsigned char *src = static_cast<const unsigned char *>(p.Q) + of * (D * 2) + ((pc ^ swz_k<D, 2>(qrow)) << 4);
        // the destination must be wave-uniform: rw and kw are, but the compiler cannot know
        const int dst = __builtin_amdgcn_readfirstlane(WL::QOFF + rw * WL::QTILE + j * 1024);
        __builtin_amdgcn_global_load_lds(src, BTV_LDS_PTR(smem + dst), 16, 0, 0);
    }

    // ---- start filling the ring ------------------------------------------------------------------------
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const bool issuer = wu < IW;
    const Fill<D, IW, PAGED, EB> fill = make_fill<D, IW, PAGED, EB>(p.K, p.V, PAGED ? p.block_table + (long long)rq * p.max_blocks : nullptr,
                                                                    p.num_blocks, p.Hkv, g, S, issuer ? wu : 0, l);
    // KW == 1: three tiles up front (the first compute needs two), the rest of the ring fills during the first
    // rounds; an issue holds its wave for about a hundred cycles, so a full prefill would only delay the start.
    constexpr int PREFILL = WL::PREFILL;
    int issued = st0, islot = 0;
#pragma unroll
    for (int k = 0; k < PREFILL; ++k)
        if (issued < st1) {
            if (issuer) issue_tile<D, IW, PAGED, EB>(fill, smem, islot, issued, wu, l);
            ++issued; ++islot;
        }
    if (islot >= NT) islot -= NT;

    // ---- parent[] and the query tile have landed when only the ring fills are in flight ------------------------
    wait_vm_ops<PREFILL * LPW>(issuer ? (issued - st0) * LPW : 0);
    // A bare barrier, and raw LDS reads below: with the fence of a full synchronisation, or with ordinary reads of
    // memory that direct-to-LDS loads wrote, the compiler drains the ring fills first.
    __builtin_amdgcn_s_barrier();                    // query tiles (filled by KW waves) and parent[] are visible
    const bool tree_wg = st1 * 32 > Lr;              // this workgroup's keys reach the tree rows
    const uint32_t par_lds = (uint32_t)(uintptr_t)BTV_LDS_PTR(smem) + WL::PAROFF;
    auto par_at = [&](int i) {
        int v;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(par_lds + 4u * (uint32_t)i) : "memory");
        return v;
    };
    // Operand s holds the 8 channels that contraction step s takes from this lane's half: 16 s + 8 h .. + 7 for
    // bf16 K, 32 (s/2) + 16 h + 8 (s%2) .. + 7 for FP8 K (the order of its 16-byte operand reads).
    u32x4 qv[DS];
    {
        const uint32_t qa = (uint32_t)(uintptr_t)BTV_LDS_PTR(smem) + WL::QOFF + rw * WL::QTILE + c * (2 * D);
        const int sw = swz_k<D, 2>(c);
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            const int chunk = EB == 2 ? 2 * s + h : 4 * (s / 2) + 2 * h + (s % 2);
            const uint32_t addr = qa + (uint32_t)((chunk ^ sw) << 4);
            asm volatile("ds_read_b128 %0, %1" : "=v"(qv[s]) : "v"(addr));
        }
    }

    // ---- ancestor bitmask of this lane's node, only in workgroups whose keys reach the tree rows ----------
    // parent[] is checked (every entry, once per workgroup) and walked from its copy in LDS.
    uint32_t anc_i[BTV_ANC_WORDS];
#pragma unroll
    for (int k = 0; k < BTV_ANC_WORDS; ++k) anc_i[k] = 0u;
    // Built where a shape needs it: shapes whose waves alternate over the tiles stage parent[] inside the ring and
    // must read it before the main loop; the pipelined shape keeps it behind the ring and builds the masks after
    // the plain prefix tiles, so that they are not live through that loop.
#define BTV_BUILD_MASK()                                                                                              \
    if (tree_wg) {                                                                                                    \
        bool bad_ = false;                                                                                            \
        for (int i_ = tid; i_ < Mr; i_ += WAVES * 64) {                                                               \
            const int pa_ = par_at(i_);                                                                               \
            bad_ = bad_ || pa_ < -1 || pa_ >= i_;                                                                     \
        }                                                                                                             \
        if (bad_) atomicOr(p.flag, 1u);                                                                               \
        const LaneRow lr_ = lane_row(by * WR + rw * 32 + c, rows_g, p.G, p.Hq, g, rq_.q0);                            \
        for (int a_ = lr_.node; a_ >= 0;) {                                                                           \
            _Pragma("unroll") for (int k_ = 0; k_ < BTV_ANC_WORDS; ++k_)                                              \
                if ((a_ >> 5) == k_) anc_i[k_] |= 1u << (a_ & 31);                                                    \
            const int pa_ = par_at(a_);                                                                               \
            a_ = (pa_ < -1 || pa_ >= a_) ? -1 : pa_; /* an invalid entry ends the walk (flagged above) */             \
        }                                                                                                             \
    }
    if constexpr (KW > 1) { BTV_BUILD_MASK() }

    float m_run = NEG_BIG, l_run = 0.f;
    float base = 0.f;                 // what the step-by-step tiles' scores are relative to (rebase_tile)
    f32x16 negb;
#pragma unroll
    for (int v = 0; v < 16; ++v) negb[v] = 0.f;
    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;

    bf16x8 qreg[DS];
    if constexpr (DS == 8)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(qv[0]), "+v"(qv[1]), "+v"(qv[2]), "+v"(qv[3]), "+v"(qv[4]), "+v"(qv[5]), "+v"(qv[6]), "+v"(qv[7]));
    else
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(qv[0]), "+v"(qv[1]), "+v"(qv[2]), "+v"(qv[3]));
    const uint32_t ring = (uint32_t)(uintptr_t)BTV_LDS_PTR(smem);
    auto issue_one = [&]() {                             // the next tile of this split, if there is one
        if (issued < st1) {
            if (issuer) issue_tile<D, IW, PAGED, EB>(fill, smem, islot, issued, wu, l);
            ++issued;
            if (++islot == NT) islot = 0;
        }
    };
    // one half of the wave's fills of the next tile (LPW = 2 in the pipelined shape); the caller advances the counters
    auto issue_part = [&](auto part) {
        constexpr int P = decltype(part)::value;
        constexpr int MID = (LPW + 1) / 2, JB = P == 0 ? 0 : MID, JE = P == 0 ? MID : LPW;
        if constexpr (JB < JE)
            if (issuer) issue_tile<D, IW, PAGED, EB, JB, JE>(fill, smem, islot, issued, wu, l);
    };
    if constexpr (KW == 1) {
        // Every wave has its queries in registers and parent[] is consumed: the ring owns all stages from here on.
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int k = PREFILL; k < NT - 1; ++k) issue_one();
    }
    // The queries take the softmax scale and the change of base once (rounded to bf16 again, to nearest even: a
    // relative 2^-9 per element, as if the caller's projection had produced the scaled queries): scores then
    // are in log2 units and a probability costs no multiply.
    {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const float qs = p.scale_log2;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            u32x4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t wd = qv[s][j];
                const bf16x2 pr = { (__bf16)(__uint_as_float(wd << 16) * qs), (__bf16)(__uint_as_float(wd & 0xFFFF0000u) * qs) };
                r[j] = __builtin_bit_cast(uint32_t, pr);
            }
            qreg[s] = __builtin_bit_cast(bf16x8, r);
        }
    }
    if constexpr (KW == 1 && EB == 2) {
        // ---- main loop, one tile per round, software-pipelined over the plain prefix tiles ------------------------
        // Local tile j = tile st0 + j lives in ring slot j % NT.  Tiles whose 32 keys all are prefix rows ("plain":
        // no mask) run through a pipeline in which iteration i issues
        //     the PV MFMAs of tile i-1 among the exponentials of tile i,  then the score MFMAs of tile i+1.
        // Scores come out of the matrix cores relative to the running reference (the accumulator starts at minus
        // the reference), so P = exp2(x) with no other arithmetic per element.  The reference is the maximum of
        // the split's first tile and moves only when a tile's row sum shows that some x exceeded 16 (checked on
        // the sum: no maximum per tile); then the tile is redone against its own maximum and everything rescaled.
        // K and V^T operands live in two half-tile buffers, each refilled right after the MFMAs that read it.
        static_assert(NT == 8, "the pipelined loop is written for a ring of 8 stages");
        constexpr int KH = DS / 2;                               // LDS reads per K half (a V^T half takes 2 * DT)
        constexpr float GROW = 1048576.0f;                       // 2^20: a half-row sum of 16 terms above it means some x > 16
        int Tf = min(st1, Lr / 32) - st0;                        // plain tiles at the start of this split
        if (Tf < 3) Tf = 0;
        int j0 = 0;                                              // first local tile the step-by-step loop below takes
        if (Tf > 0) {
            const uint32_t kbase = ring + lane_k_off<D>(l), vbase = ring + LD::TILEB + lane_v_off<D>(l);
            auto slot_off = [](int j) { return (uint32_t)((j & (NT - 1)) * LD::STAGE); };      // wave-uniform
            u32x4 kh[KH];
            bf16x4 vh[DT][2];
            f32x16 x;
            bf16x8 pa[2], pc[2];
            float negm;                                          // minus the reference: what the score accumulator starts from
            f32x16 negm16;                                       // ... kept splatted: the first score MFMA of a tile takes it as its
                                                                 // addend and writes x, so no tile pays sixteen moves for it
            // the tile's probabilities against a new reference: its own maximum joins the old one; sums, accumulator follow
            auto regrow = [&](bf16x8 (&pn)[2], float &ts) {
                const float dlt = fmaxf(tile_max(x), 0.f), alpha = __builtin_amdgcn_exp2f(-dlt);
                negm -= dlt;
#pragma unroll
                for (int v = 0; v < 16; ++v) negm16[v] = negm;
                l_run *= alpha;
#pragma unroll
                for (int v = 0; v < 16; ++v) x[v] -= dlt;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
                ts = 0.f;
                exp_half(x, 0, pn[0], ts);
                exp_half(x, 1, pn[1], ts);
            };
            // tiles 0 .. 2 have landed when at most the later ones are in flight
            wait_tiles<LPW, NT - 4>(issued - st0 - 3);
            __builtin_amdgcn_s_barrier();
            // ---- prologue: scores of tile 0 set the reference; its probabilities; scores of tile 1 ----
            {
#pragma unroll
                for (int v = 0; v < 16; ++v) x[v] = 0.f;
                read_k_half_at<D, 0>(kbase, kh); wait_k_half<KH, 0>(kh); x = qk_half<DS, 0>(kh, qreg, x);
                read_k_half_at<D, 1>(kbase, kh); wait_k_half<KH, 0>(kh); x = qk_half<DS, 1>(kh, qreg, x);
                read_k_half_at<D, 0>(kbase + slot_off(1), kh);
                negm = -tile_max(x);
#pragma unroll
                for (int v = 0; v < 16; ++v) x[v] += negm;
                exp_half(x, 0, pa[0], l_run);                    // x <= 0 here: no growth check
                exp_half(x, 1, pa[1], l_run);
#pragma unroll
                for (int v = 0; v < 16; ++v) negm16[v] = negm;
                wait_k_half<KH, 0>(kh); x = qk_half<DS, 0>(kh, qreg, negm16);
                read_k_half_at<D, 1>(kbase + slot_off(1), kh); wait_k_half<KH, 0>(kh); x = qk_half<DS, 1>(kh, qreg, x);
                read_v_half_at<D, 0>(vbase, vh);                 // queue: V(0) first half, K(2) low half
                read_k_half_at<D, 0>(kbase + slot_off(2), kh);
            }
            // ---- iteration i (1 <= i <= Tf - 2): x holds the scores of tile i, pprev the probabilities of tile i-1, pcur
            // receives those of tile i ----
            // On entry the LDS queue holds [V(i-1) first half, K(i+1) low half].
            // Loop-invariant operand addresses for the trips whose ring slots are known at compile time (eight trips
            // unrolled, one per slot): the slot is an immediate offset then, which reaches four slots from one base,
            // and a trip needs no address arithmetic at all (20 instructions of it otherwise).
            uint32_t ak[DS], akh[DS], av[DT], avh[DT];
#pragma unroll
            for (int s2 = 0; s2 < DS; ++s2) { ak[s2] = kbase ^ (uint32_t)(s2 << 5); akh[s2] = ak[s2] + 4u * LD::STAGE; }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) { av[dt] = vbase ^ (uint32_t)(dt << 6); avh[dt] = av[dt] + 4u * LD::STAGE; }
            auto rk = [&](auto slot, auto half) {
                constexpr int S = decltype(slot)::value & 7, H = decltype(half)::value;
                if constexpr (S < 4) read_k_half<D, S, H>(ak, kh); else read_k_half<D, S - 4, H>(akh, kh);
            };
            auto rv = [&](auto slot, auto mm) {
                constexpr int S = decltype(slot)::value & 7, MM = decltype(mm)::value;
                if constexpr (S < 4) read_v_half<D, S, MM>(av, vh); else read_v_half<D, S - 4, MM>(avh, vh);
            };
            // ph: the trip's tile number modulo 8 as a constant, or -1 for a trip with its addresses in registers
            auto iter = [&](bf16x8 (&pprev)[2], bf16x8 (&pcur)[2], int i, auto ph) {
                constexpr int PH = decltype(ph)::value;
                using C0 = std::integral_constant<int, 0>;
                using C1 = std::integral_constant<int, 1>;
                // tiles <= i+2 are read in this iteration; the barrier also tells that every wave is done with
                // iteration i-1, i.e. with tile i-2, whose slot the next fill takes
                wait_tiles<LPW, 3>(issued - st0 - i - 3);
                __builtin_amdgcn_s_barrier();
                const bool fill_now = issued < st1;              // tile i+6 goes into the slot tile i-2 left
                uint32_t k1 = 0, k2 = 0, v0 = 0, v1 = 0;
                if constexpr (PH < 0) {
                    k1 = kbase + slot_off(i + 1); k2 = kbase + slot_off(i + 2);
                    v0 = vbase + slot_off(i - 1); v1 = vbase + slot_off(i);
                }
                float ts = 0.f;
                wait_v_half<DT, KH>(vh);                          // V(i-1) first half
                pv_half<DT>(vh, pprev[0], oacc);
                if (fill_now) issue_part(std::integral_constant<int, 0>{});      // behind four MFMAs: its issue stall is covered
                if constexpr (PH < 0) read_v_half_at<D, 1>(v0, vh);                     // V(i-1) second half  queue: K(i+1)lo, V(i-1)b
                else rv(std::integral_constant<int, PH + 7>{}, C1{});
                exp_half(x, 0, pcur[0], ts);
                __builtin_amdgcn_sched_barrier(0);                // (the exponentials stay in front of the wait: they cover the reads)
                wait_v_half<DT, 0>(vh);                           // V(i-1) second half (and K(i+1) low)
                pv_half<DT>(vh, pprev[1], oacc);
                if (fill_now) issue_part(std::integral_constant<int, 1>{});
                if constexpr (PH < 0) read_v_half_at<D, 0>(v1, vh);                     // V(i) first half     queue: V(i)a
                else rv(std::integral_constant<int, PH>{}, C0{});
                exp_half(x, 1, pcur[1], ts);
                __builtin_amdgcn_sched_barrier(0);
                if (__builtin_amdgcn_ballot_w64(!(ts <= GROW)) != 0ull) regrow(pcur, ts);     // rare
                l_run += ts;
                wait_k_half<KH, 2 * DT>(kh);                      // K(i+1) low (landed above; binds the registers)
                x = qk_half<DS, 0>(kh, qreg, negm16);
                if constexpr (PH < 0) read_k_half_at<D, 1>(k1, kh);                     // K(i+1) high         queue: V(i)a, K(i+1)hi
                else rk(std::integral_constant<int, PH + 1>{}, C1{});
                wait_k_half<KH, 0>(kh);                           // K(i+1) high (and V(i) first half)
                x = qk_half<DS, 1>(kh, qreg, x);
                if constexpr (PH < 0) read_k_half_at<D, 0>(k2, kh);                     // K(i+2) low          queue: K(i+2)lo (V(i)a has landed)
                else rk(std::integral_constant<int, PH + 2>{}, C0{});
                if (fill_now) { ++issued; if (++islot == NT) islot = 0; }
            };
            // ---- epilogue: tile e = Tf - 1 has its scores, tile e-1 its probabilities (pp); nothing left to overlap ----
            auto drain = [&](bf16x8 (&pp)[2], bf16x8 (&pn)[2]) {
                const int e = Tf - 1;
                const uint32_t ve1 = vbase + slot_off(e - 1), ve = vbase + slot_off(e);
                wait_k_half<KH, 0>(kh);                          // (the low half of tile e+1's K: not used)
                wait_v_half<DT, 0>(vh);                          // V(e-1) first half
                pv_half<DT>(vh, pp[0], oacc);
                read_v_half_at<D, 1>(ve1, vh);
                float ts = 0.f;
                exp_half(x, 0, pn[0], ts);
                exp_half(x, 1, pn[1], ts);
                wait_v_half<DT, 0>(vh);
                pv_half<DT>(vh, pp[1], oacc);
                read_v_half_at<D, 0>(ve, vh);
                if (__builtin_amdgcn_ballot_w64(!(ts <= GROW)) != 0ull) regrow(pn, ts);
                l_run += ts;
                wait_v_half<DT, 0>(vh);
                pv_half<DT>(vh, pn[0], oacc);
                read_v_half_at<D, 1>(ve, vh);
                wait_v_half<DT, 0>(vh);
                pv_half<DT>(vh, pn[1], oacc);
                m_run = -negm;
            };
            // One iteration per trip, the new probabilities copied into place at its end (8 moves): with the roles of
            // two register sets alternating over an unrolled pair the allocator shuffles tuples and spills.
            int i = 1;
            for (; i + 7 <= Tf - 2; i += 8) {                    // tile i is in ring slot 1 here: eight trips, one per slot
                // (the two probability buffers swap roles from trip to trip: no copies inside the group)
                // (one barrier for two trips, with the fills one tile less ahead, measured the same)
#define BTV_TRIP(k, slot, from, to) iter(from, to, i + k, std::integral_constant<int, slot>{});
                BTV_TRIP(0, 1, pa, pc) BTV_TRIP(1, 2, pc, pa) BTV_TRIP(2, 3, pa, pc) BTV_TRIP(3, 4, pc, pa)
                BTV_TRIP(4, 5, pa, pc) BTV_TRIP(5, 6, pc, pa) BTV_TRIP(6, 7, pa, pc) BTV_TRIP(7, 0, pc, pa)
#undef BTV_TRIP
            }
            for (; i <= Tf - 2; ++i) {
                iter(pa, pc, i, std::integral_constant<int, -1>{});
#pragma unroll
                for (int mm = 0; mm < 2; ++mm) pa[mm] = pc[mm];
            }
            drain(pa, pc);
            j0 = Tf;
        }
        // ---- the remaining tiles (those that touch tree rows, or all of a short split), step by step ----
        if (j0 > 0) {                                            // (m_run is a real maximum after the pipelined part)
            base = m_run;
#pragma unroll
            for (int v = 0; v < 16; ++v) negb[v] = -m_run;
        }
        BTV_BUILD_MASK()
        for (int j = j0; j < st1 - st0; ++j) {
            wait_tiles<LPW, NT - 1>(issued - st0 - j - 1);       // tile j has landed
            __builtin_amdgcn_s_barrier();                        // ... for every wave, and all are done with tile j-1
#pragma unroll
            for (int k = 0; k < 2; ++k)
                if (issued - st0 - j < NT) issue_one();
            do_tile<D>(ring + (j & 7) * LD::STAGE, (st0 + j) * 32, Lr, l, anc_i, qreg, m_run, l_run, oacc, base, negb);
        }
    } else if constexpr (KW > 1) {
        // ---- main loop: one barrier per round of KW tiles, wave kw takes tile number kw of the round ------
        // At the top of the round starting at tile st, tiles st+KW .. issued-1 may still be in flight.  The
        // barrier also tells that every wave is done with the previous round, whose KW ring slots the next
        // issues overwrite.
        int cslot = kw;
        for (int st = st0; st < st1; st += KW) {
            if (issued - st - KW == AHEAD) wait_vmcnt<AHEAD * LPW>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int k = 0; k < KW; ++k)
                if (issued < st1) {
                    issue_tile<D, IW, PAGED, EB>(fill, smem, islot, issued, wu, l);
                    ++issued;
                    if (++islot == NT) islot = 0;
                }
            if (st + kw < st1) {
                if constexpr (EB == 2)
                    do_tile<D>(ring + cslot * LD::STAGE, (st + kw) * 32, Lr, l, anc_i, qreg, m_run, l_run, oacc, base, negb);
                else
                    do_tile8<D>(ring + cslot * LD::STAGE, (st + kw) * 32, Lr, l, anc_i, qreg, m_run, l_run, oacc);
            }
            cslot += KW;
            if (cslot >= NT) cslot -= NT;
        }
    }
    const LaneRow lrow = lane_row(by * WR + rw * 32 + c, rows_g, p.G, p.Hq, g, rq_.q0);
    const bool rvalid = lrow.valid;
    const long long orow = lrow.orow;
    // both halves of a wave hold partial row sums of the same queries
    l_run += __shfl_xor(l_run, 32);

    // ---- merge the key-waves of each row-wave through LDS ---------------------------------------------------
    // Two key-waves: each keeps one half of the channels and hands the other half to its partner, so both merge,
    // scale and store half a row.  dt0 .. dt0 + DTK - 1 are the channel blocks this wave ends up with.
    int dt0 = 0;
    constexpr int DTK = KW == 2 ? DT / 2 : DT;
    float fin[DTK][16];                             // what this wave stores
    float amax = 0.f;                               // bound on the row's largest magnitude (for the fp16 partials)
    if constexpr (KW == 2) {
        constexpr int SLOT = (DTK * 16 + 3) * 64;   // floats a wave hands over
        float *mg = reinterpret_cast<float *>(smem) + rw * 2 * SLOT;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) amax = fmaxf(amax, fabsf(oacc[dt][v]));
        amax = fmaxf(amax, __shfl_xor(amax, 32));   // the other half of the wave holds the row's other channels
        wait_vmcnt<0>();
        __syncthreads();                            // every wave is done with the ring
        float *out = mg + kw * SLOT;
        auto give = [&](auto first) {               // the channel blocks first .. first + DTK - 1 go to the partner
            constexpr int F = decltype(first)::value;
#pragma unroll
            for (int dt = 0; dt < DTK; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) out[(dt * 16 + v) * 64 + l] = oacc[F + dt][v];
        };
        if (kw == 0) give(std::integral_constant<int, DTK>{}); else give(std::integral_constant<int, 0>{});
        out[(DTK * 16) * 64 + l] = m_run;
        out[(DTK * 16 + 1) * 64 + l] = l_run;
        out[(DTK * 16 + 2) * 64 + l] = amax;
        __syncthreads();
        const float *in = mg + (kw ^ 1) * SLOT;
        const float m1 = in[(DTK * 16) * 64 + l], l1 = in[(DTK * 16 + 1) * 64 + l], x1 = in[(DTK * 16 + 2) * 64 + l];
        const float mn = fmaxf(m_run, m1);
        const float a0 = __builtin_amdgcn_exp2f(m_run - mn);
        const float a1 = __builtin_amdgcn_exp2f(m1 - mn);
        // both waves must arrive at the same l and bound: sums of the same two products, order fixed by kw
        const float la = kw == 0 ? l_run * a0 : l1 * a1, lb = kw == 0 ? l1 * a1 : l_run * a0;
        const float xa = kw == 0 ? amax * a0 : x1 * a1, xb = kw == 0 ? x1 * a1 : amax * a0;
        m_run = mn;
        l_run = la + lb;
        amax = xa + xb;                             // >= the merged row's largest magnitude, at most twice it
        auto take = [&](auto first) {
            constexpr int F = decltype(first)::value;
#pragma unroll
            for (int dt = 0; dt < DTK; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) fin[dt][v] = oacc[F + dt][v] * a0 + in[(dt * 16 + v) * 64 + l] * a1;
        };
        if (kw == 0) take(std::integral_constant<int, 0>{}); else take(std::integral_constant<int, DTK>{});
        dt0 = kw * DTK;                             // the kept blocks now sit in oacc[0 .. DTK)
    } else if (KW > 1) {                            // donors write side by side, wave kw = 0 reduces
        constexpr int SLOT = (DT * 16 + 2) * 64;    // floats per donor
        float *mg = reinterpret_cast<float *>(smem) + (rw * (KW - 1)) * SLOT;
        wait_vmcnt<0>();
        __syncthreads();                            // every wave is done with the ring
        if (kw > 0) {
            float *d = mg + (kw - 1) * SLOT;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) d[(dt * 16 + v) * 64 + l] = oacc[dt][v];
            d[(DT * 16) * 64 + l] = m_run;
            d[(DT * 16 + 1) * 64 + l] = l_run;
        }
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int donor = 0; donor < KW - 1; ++donor) {
                const float *d = mg + donor * SLOT;
                const float m1 = d[(DT * 16) * 64 + l], l1 = d[(DT * 16 + 1) * 64 + l];
                const float mn = fmaxf(m_run, m1);
                const float a0 = __builtin_amdgcn_exp2f(m_run - mn);
                const float a1 = __builtin_amdgcn_exp2f(m1 - mn);
                m_run = mn;
                l_run = l_run * a0 + l1 * a1;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] = oacc[dt][v] * a0 + d[(dt * 16 + v) * 64 + l] * a1;
            }
        }
    }
    if ((KW != 2 && kw != 0) || !rvalid) return;
    if constexpr (KW != 2) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) { fin[dt][v] = oacc[dt][v]; amax = fmaxf(amax, fabsf(oacc[dt][v])); }
        amax = fmaxf(amax, __shfl_xor(amax, 32));
    }

    // ---- write: final bf16 rows when this request has a single split, scaled fp16 partials otherwise ---
    if (nsplit_r == 1) {
        const float inv = p.out_scale / l_run;
        uint16_t *Op = static_cast<uint16_t *>(p.O) + orow * D + dt0 * 32;
#pragma unroll
        for (int dt = 0; dt < DTK; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                uint32_t lo = float_to_bf16_bits(fin[dt][q4 * 4 + 0] * inv) | (float_to_bf16_bits(fin[dt][q4 * 4 + 1] * inv) << 16);
                uint32_t hi = float_to_bf16_bits(fin[dt][q4 * 4 + 2] * inv) | (float_to_bf16_bits(fin[dt][q4 * 4 + 3] * inv) << 16);
                *reinterpret_cast<uint2 *>(Op + dt * 32 + q4 * 8 + h * 4) = make_uint2(lo, hi);
            }
    } else {
        // Partials travel as fp16 relative to (a bound within a factor two of) the row's largest magnitude, kept
        // in fp32 beside m and l: half the bytes of fp32 to write, flush at the end of the kernel and read back, at
        // a relative error of at most 2^-10 of that magnitude, below the final bf16 rounding.
        const float sc = amax > 0.f ? 1.0f / amax : 0.f;
        const size_t prow = (size_t)bx * p.total_rows + orow;
        _Float16 *Pp = p.Opart + prow * D + dt0 * 32;
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int dt = 0; dt < DTK; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const h2 lo = { (_Float16)(fin[dt][q4 * 4 + 0] * sc), (_Float16)(fin[dt][q4 * 4 + 1] * sc) };
                const h2 hi = { (_Float16)(fin[dt][q4 * 4 + 2] * sc), (_Float16)(fin[dt][q4 * 4 + 3] * sc) };
                *reinterpret_cast<uint2 *>(Pp + dt * 32 + q4 * 8 + h * 4) =
                    make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
            }
        if (h == 0 && kw == 0) *reinterpret_cast<float4 *>(p.ML + prow * 4) = make_float4(m_run, l_run, amax, 0.f);
    }
}

// Split-K combine: O[row] = sum_s w_s a_s O'_s / sum_s w_s l_s with w_s = exp2((m_s - max m) * scale*log2 e), O'_s the
// fp16 partial and a_s the magnitude it was divided by.
// 8 rows per workgroup, 32 lanes per row, each lane owns D/32 consecutive channels.  Lane j of a row fetches the
// (m, l) pairs of splits j, j + 32, ... and computes their weights; the partial rows of up to 32 splits are fetched
// by independent loads issued before anything is waited for, so the kernel costs about one memory round trip
// whatever the number of splits.  What happens between the lanes of a row stays off the LDS crossbar where it can:
// maximum and sum over the 32 lanes are DPP steps within the rows of 16 and one swap between the two rows (they were
// five dependent ds_bpermute round trips each), and the 32 weights reach every lane through one LDS store and eight
// 16-byte reads of the same address (they were 32 shuffles, each waited for before its multiply-adds).
__device__ __forceinline__ float row32_max(float x, int lane)
{
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0xB1, 0xF, 0xF, false)));    // quad_perm [1,0,3,2]
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x4E, 0xF, 0xF, false)));    // quad_perm [2,3,0,1]
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x141, 0xF, 0xF, false)));   // row_half_mirror
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x140, 0xF, 0xF, false)));   // row_mirror
    const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(x, __uint_as_float((lane & 16) ? sw[0] : sw[1]));                                               // the other row of 16
}

__device__ __forceinline__ float row32_sum(float x, int lane)
{
    x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0xB1, 0xF, 0xF, false));
    x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x4E, 0xF, 0xF, false));
    x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x141, 0xF, 0xF, false));
    x += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x140, 0xF, 0xF, false));
    const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return x + __uint_as_float((lane & 16) ? sw[0] : sw[1]);
}

template <int D, bool PAGED>
__global__ __launch_bounds__(256) void tv_combine_bf16(AttnParams p)
{
    constexpr int E = D / 32;
    typedef _Float16 hvec __attribute__((ext_vector_type(E)));
    __shared__ __attribute__((aligned(16))) float wsh[8][32];
    // every argument in one round trip (the argument block is cold in every launch)
    asm volatile("" ::"s"(p.O), "s"(p.q_offset), "s"(p.prefix_len), "s"(p.Opart), "s"(p.ML), "s"(p.M), "s"(p.L), "s"(p.Hq),
                 "s"(p.max_blocks), "s"(p.total_rows), "s"(p.total_M), "s"(p.sps), "s"(p.out_scale));
    const int rq = blockIdx.y;
    const Req rq_ = load_req<PAGED>(p, rq);
    if (!rq_.ok) return;
    const int stages = (rq_.L + rq_.M + TK - 1) / TK;
    const int nsplit_r = (stages + p.sps - 1) / p.sps;
    if (nsplit_r == 1) return;                      // the attention kernel wrote O directly
    const int rin = threadIdx.x >> 5, lr = blockIdx.x * 8 + rin, lane = threadIdx.x & 31;
    if (lr >= rq_.M * p.Hq) return;
    const size_t row = (size_t)rq_.q0 * p.Hq + lr;
    const size_t sstride = (size_t)p.total_rows;
    // reference maximum over all splits: with more than 32 of them it takes a round trip of its own
    float mmax = NEG_BIG;
    for (int s = lane + 32; s < nsplit_r; s += 32) mmax = fmaxf(mmax, p.ML[(s * sstride + row) * 4]);
    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    float den = 0.f;
    for (int s0 = 0; s0 < nsplit_r; s0 += 32) {     // one pass for up to 32 splits
        const int s_mine = s0 + lane;
        const float4 mlr = *reinterpret_cast<const float4 *>(p.ML + ((size_t)min(s_mine, nsplit_r - 1) * sstride + row) * 4);
        const float4 ml = s_mine < nsplit_r ? mlr : make_float4(NEG_BIG, 0.f, 0.f, 0.f);
        hvec part[32];
#pragma unroll
        for (int g = 0; g < 4; ++g)
            if (s0 + 8 * g < nsplit_r) {             // uniform within the row's lanes: whole groups of 8 loads
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const int s = min(s0 + 8 * g + b, nsplit_r - 1);
                    part[8 * g + b] = *reinterpret_cast<const hvec *>(p.Opart + (s * sstride + row) * D + lane * E);
                }
            }
        if (s0 == 0) mmax = row32_max(fmaxf(mmax, ml.x), (int)threadIdx.x);
        const float w = s_mine < nsplit_r ? __builtin_amdgcn_exp2f(ml.x - mmax) : 0.f;
        den += w * ml.y;
        wsh[rin][lane] = w * ml.z;                              // weight times the partial's magnitude; 0 past the last split
        // (the row's 32 lanes are one half of a wavefront: its LDS operations complete in order, no barrier needed)
        float wgt[32];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float4 x = *reinterpret_cast<const float4 *>(&wsh[rin][4 * q]);
            wgt[4 * q] = x.x; wgt[4 * q + 1] = x.y; wgt[4 * q + 2] = x.z; wgt[4 * q + 3] = x.w;
        }
#pragma unroll
        for (int g = 0; g < 4; ++g)
            if (s0 + 8 * g < nsplit_r) {
#pragma unroll
                for (int b = 0; b < 8; ++b) {
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[e] += wgt[8 * g + b] * (float)part[8 * g + b][e];
                }
            }
    }
    den = row32_sum(den, (int)threadIdx.x);
    const float inv = p.out_scale / den;
    uint16_t *dst = static_cast<uint16_t *>(p.O) + row * D + lane * E;
    if (E == 4) {
        uint32_t lo = float_to_bf16_bits(acc[0] * inv) | (float_to_bf16_bits(acc[1] * inv) << 16);
        uint32_t hi = float_to_bf16_bits(acc[E - 2] * inv) | (float_to_bf16_bits(acc[E - 1] * inv) << 16);
        *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
    } else {
        *reinterpret_cast<uint32_t *>(dst) = float_to_bf16_bits(acc[0] * inv) | (float_to_bf16_bits(acc[E - 1] * inv) << 16);
    }
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
// ---- scratch of the entry point that allocates nothing ---------------------------------------------------------
// One array per GPU, part of the loaded code object (zero until first used), held until the process ends.  Host code
// never uses the array's name as an address: the device address is asked for once per device and kept.
constexpr size_t SCRATCH_BYTES = (size_t)32 << 20;
constexpr int SCRATCH_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];
void *g_scratch_ptr[SCRATCH_MAX_DEVICES];
std::atomic<bool> g_scratch_known[SCRATCH_MAX_DEVICES];

// Device address of the current device's copy of `scratch` (looked up on the first call per device).
int scratch_address(void **out)
{
    int dev = -1;
    BTV_HIP(hipGetDevice(&dev));
    BTV_REQUIRE(dev >= 0 && dev < SCRATCH_MAX_DEVICES, "device index %d outside [0,%d)", dev, SCRATCH_MAX_DEVICES);
    if (!g_scratch_known[dev].load(std::memory_order_acquire)) {
        void *ptr = nullptr;
        BTV_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        BTV_REQUIRE(ptr != nullptr, "no device address for the scratch array");
        g_scratch_ptr[dev] = ptr;                   // (two racing first calls store the same address)
        g_scratch_known[dev].store(true, std::memory_order_release);
    }
    *out = g_scratch_ptr[dev];
    return BTV_OK;
}

// Clears the first `words` 32-bit words at p (a kernel rather than a memset node, so that the call can be captured).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *p, int words)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < words) p[i] = 0u;
}

struct Plan { int rw, kw, nt, wr, row_blocks, stages, sps, nsplit; };

// Kernel shape by the number of packed rows per KV head (G*M).  Every wave owns 32 rows.  Measured on MI355X at
// L = 8192 (8 KV heads): what counts is one workgroup per CU and as few key splits as that allows (the split
// partials are written and read back), so few rows get small row blocks and many rows get 128-row blocks, both
// with pairs of waves alternating over the tiles (KW = 2); very many rows over a very long prefix take the
// 256-row software-pipelined shape (KW = 1), which measures the same there within run-to-run noise.
// `force_split` > 0 and `force_shape` in 1..3 replace the heuristic's choices (the tuning entry point passes them).
Plan make_plan(int M, int L, int Hq, int Hkv, int batch, int eb = 2, int force_split = 0, int force_shape = 0)
{
    Plan pl;
    int G = Hq / Hkv, rows_g = G * M;
    // Ragged batches take the small workgroup whatever the largest tree: 64-row blocks pad the smaller trees less,
    // and two such workgroups share a CU, so one's prologue and store overlap the other's main loop.
    if (rows_g <= 128 || batch > 1) { pl.rw = 2; pl.kw = 2; pl.nt = 5; }
    // 768 packed rows or more (192 nodes at 4 query heads per KV head, 96 at 8): the software-pipelined 256-row
    // shape, measured 12 % ahead at the 70B shape with a 32k prefix, 4 % at 256 nodes of the 8B shape, 2 % at 192;
    // below, pairs of waves alternating over the tiles are 3-8 % ahead.  The FP8 cache has only the latter.
    else if (eb == 2 && rows_g >= 768) { pl.rw = 8; pl.kw = 1; pl.nt = 8; }
    else { pl.rw = 4; pl.kw = 2; pl.nt = 8; }
    if (force_shape == 1) { pl.rw = 2; pl.kw = 2; pl.nt = 5; }
    if (force_shape == 2) { pl.rw = 4; pl.kw = 2; pl.nt = 8; }
    if (force_shape == 3 && eb == 2) { pl.rw = 8; pl.kw = 1; pl.nt = 8; }
    pl.wr = pl.rw * 32;
    pl.row_blocks = (rows_g + pl.wr - 1) / pl.wr;
    pl.stages = (L + M + TK - 1) / TK;
    // Tiles that hold tree rows cost more than plain tiles (mask; in the pipelined loop also a second row maximum)
    // and all sit in the last split: sizing the splits as if there were `extra` more tiles leaves the last one
    // that much shorter.
    const int tree_tiles = pl.stages - L / TK;
    const int extra = pl.kw == 1 ? (7 * tree_tiles + 9) / 10 : (tree_tiles + 3) / 4;
    int base = Hkv * pl.row_blocks * batch;
    // 64 rows or fewer: finer splits still pay.  Batches: the host only knows the largest request, so the longest
    // request is cut into up to 8 units of at least 32 tiles and the dispatcher evens out the requests' lengths
    // (measured on ragged and uniform batches of 4 to 16 requests: within 1.5x of the best shape and split count
    // found for each; a uniform batch would do best with one unit per CU, which the host cannot tell from here).
    int target = rows_g <= 64 ? 512 : 256;
    // (rounded down: one split more than the CUs hold sends a second, nearly empty round of workgroups through the
    // chip, e.g. 6 splits x 48 = 288 workgroups at 192 nodes took 61 us against 43 us for 5 x 48 = 240)
    int want = force_split > 0 ? force_split : std::max(1, target / base);
    if (batch > 1 && force_split <= 0) want = std::max(1, std::min(8, pl.stages / 32));
    // a split should stream at least 8 tiles (256 keys) unless the caller forces it
    if (force_split <= 0) want = std::min(want, std::max(1, pl.stages / 8));
    want = std::max(1, std::min(want, pl.stages));
    pl.sps = (pl.stages + (want > 1 ? extra : 0) + want - 1) / want;
    pl.sps = (pl.sps + pl.kw - 1) / pl.kw * pl.kw;         // whole rounds of KW tiles
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
    w.ml = off; off += btv_align_up(ns * rows * 4 * 4, BTV_WS_ALIGN);
    w.opart = off; off += btv_align_up(ns * rows * D * 2, BTV_WS_ALIGN);
    w.total = off;
    return w;
}

template <int D, int RW, int KW, int NT, bool PAGED, int EB = 2>
int launch_bf16(const AttnParams &p, dim3 grid, hipStream_t st)
{
    constexpr int LDS_BYTES = WgLds<D, RW, KW, NT, EB>::BYTES;
    static std::atomic<bool> configured{false};         // (one GPU per process: the attribute is set once)
    auto kern = tv_attn_bf16<D, RW, KW, NT, PAGED, EB>;
    if (!configured.load(std::memory_order_acquire)) {
        BTV_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    LDS_BYTES));
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, grid, dim3(RW * KW * 64), LDS_BYTES, st, p);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

template <bool PAGED>
int dispatch_bf16(AttnParams &p, const Plan &pl, int D, int batch, int eb, hipStream_t st)
{
    p.row_blocks = pl.row_blocks;
    p.units = pl.nsplit * p.Hkv * batch;
    const int units = pl.nsplit * p.Hkv * batch;
    dim3 grid(((units + 7) / 8) * pl.row_blocks * 8);
    if (eb == 1) {      // FP8 K/V
        if (D == 128 && pl.rw == 2 && pl.kw == 2 && pl.nt == 5) return launch_bf16<128, 2, 2, 5, PAGED, 1>(p, grid, st);
        if (D == 128 && pl.rw == 4 && pl.kw == 2 && pl.nt == 8) return launch_bf16<128, 4, 2, 8, PAGED, 1>(p, grid, st);
        return btv_fail(BTV_EINVAL, "no FP8-KV kernel for D=%d", D);
    }
#define BTV_CASE(DD, RR, KK, NN) \
    if (D == DD && pl.rw == RR && pl.kw == KK && pl.nt == NN) return launch_bf16<DD, RR, KK, NN, PAGED>(p, grid, st);
    BTV_CASE(128, 2, 2, 5) BTV_CASE(128, 4, 2, 8) BTV_CASE(128, 8, 1, 8)
    BTV_CASE(64, 2, 2, 5) BTV_CASE(64, 4, 2, 8) BTV_CASE(64, 8, 1, 8)
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

int check_fp8(int D, float k_scale, float v_scale)
{
    BTV_REQUIRE(D == 128, "FP8 K/V: D=%d, only 128 is built", D);
    BTV_REQUIRE(k_scale > 0.f && k_scale <= 3.0e38f && v_scale > 0.f && v_scale <= 3.0e38f,
                "FP8 K/V scales must be positive and finite");
    return BTV_OK;
}

bool aligned16(const void *a) { return (reinterpret_cast<uintptr_t>(a) & 15u) == 0; }

// eb = bytes per K/V element (2: the dtype's own; 1: E4M3 codes, bf16 Q and O).  The key scale multiplies every
// score, so it joins the softmax scale; the value scale multiplies the weighted sum, so it joins the final division.
void set_scales(AttnParams &p, int D, float scale, float k_scale, float v_scale)
{
    p.scale = (scale > 0.f ? scale : 1.0f / sqrtf((float)D)) * k_scale;
    p.scale_log2 = p.scale * 1.4426950408889634f;
    p.out_scale = v_scale;
}

int attn_contiguous(const void *Q, const void *K, const void *V, const int32_t *parent, int M, int L, int Hq, int Hkv,
                    int D, int dtype, int eb, float scale, float k_scale, float v_scale, void *O, void *ws,
                    size_t ws_bytes, void *stream, int force_split = 0, int force_shape = 0, uint32_t *flag_out = nullptr)
{
    BTV_REQUIRE(Q && K && V && parent && O, "null pointer");
    BTV_REQUIRE(aligned16(Q) && aligned16(K) && aligned16(V) && aligned16(O), "Q, K, V and O must be 16-byte aligned");
    int rc = check_shape(M, L, Hq, Hkv, D);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Plan pl = make_plan(M, L, Hq, Hkv, 1, eb, force_split, force_shape);
    if (dtype == BTV_F32) pl.nsplit = 1;
    WsLayout wl = ws_layout(M, Hq, D, pl.nsplit);
    rc = btv_check_ws(ws, ws_bytes, wl.total);
    if (rc) return rc;
    unsigned char *w8 = static_cast<unsigned char *>(ws);
    AttnParams p = {};
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.anc = reinterpret_cast<uint32_t *>(w8 + wl.anc);
    p.ML = reinterpret_cast<float *>(w8 + wl.ml);
    p.Opart = reinterpret_cast<_Float16 *>(w8 + wl.opart);
    p.flag = flag_out ? flag_out : reinterpret_cast<uint32_t *>(w8);
    p.M = M; p.L = L; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.total_rows = M * Hq; p.total_M = M;
    p.sps = pl.sps; p.nsplit = pl.nsplit;
    set_scales(p, D, scale, k_scale, v_scale);
    p.parent = parent;
    if (dtype == BTV_F32) {
        rc = btv_launch_anc_mask(parent, nullptr, 1, M, M, const_cast<uint32_t *>(p.anc), p.flag, st);
        if (rc) return rc;
        if (D == 64) hipLaunchKernelGGL(tv_attn_f32<64>, dim3(M, Hq), dim3(256), 0, st, p);
        else hipLaunchKernelGGL(tv_attn_f32<128>, dim3(M, Hq), dim3(256), 0, st, p);
        BTV_HIP(hipGetLastError());
        return BTV_OK;
    }
    rc = dispatch_bf16<false>(p, pl, D, 1, eb, st);
    if (rc) return rc;
    if (pl.nsplit > 1) {
        dim3 cg((M * Hq + 7) / 8, 1);
        if (D == 64) hipLaunchKernelGGL((tv_combine_bf16<64, false>), cg, dim3(256), 0, st, p);
        else hipLaunchKernelGGL((tv_combine_bf16<128, false>), cg, dim3(256), 0, st, p);
        BTV_HIP(hipGetLastError());
    }
    return BTV_OK;
}

int attn_paged(const void *Q, const void *Kpool, const void *Vpool, int num_blocks, const int32_t *block_table,
               int max_blocks, const int32_t *q_offset, const int32_t *prefix_len, const int32_t *parent, int batch,
               int total_M, int M_max, int L_max, int Hq, int Hkv, int D, int eb, float scale, float k_scale,
               float v_scale, void *O, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(Q && Kpool && Vpool && block_table && q_offset && prefix_len && parent && O, "null pointer");
    BTV_REQUIRE(aligned16(Q) && aligned16(Kpool) && aligned16(Vpool) && aligned16(O),
                "Q, K, V and O must be 16-byte aligned");
    BTV_REQUIRE(batch >= 1 && batch <= 4096, "batch=%d outside [1,4096]", batch);
    int rc = check_shape(M_max, L_max, Hq, Hkv, D);
    if (rc) return rc;
    BTV_REQUIRE(total_M >= 1 && total_M <= batch * M_max, "total_M=%d inconsistent with batch*M_max", total_M);
    BTV_REQUIRE(num_blocks >= 1 && max_blocks >= 1, "bad block counts");
    BTV_REQUIRE((long long)max_blocks * BTV_PAGE >= (long long)L_max + 1, "max_blocks too small for L_max");
    hipStream_t st = static_cast<hipStream_t>(stream);
    Plan pl = make_plan(M_max, L_max, Hq, Hkv, batch, eb);
    WsLayout wl = ws_layout(batch * M_max, Hq, D, pl.nsplit);
    rc = btv_check_ws(ws, ws_bytes, wl.total);
    if (rc) return rc;
    unsigned char *w8 = static_cast<unsigned char *>(ws);
    AttnParams p = {};
    p.Q = Q; p.K = Kpool; p.V = Vpool; p.O = O;
    p.anc = reinterpret_cast<uint32_t *>(w8 + wl.anc);
    p.ML = reinterpret_cast<float *>(w8 + wl.ml);
    p.Opart = reinterpret_cast<_Float16 *>(w8 + wl.opart);
    p.flag = reinterpret_cast<uint32_t *>(w8);
    p.block_table = block_table; p.q_offset = q_offset; p.prefix_len = prefix_len;
    p.max_blocks = max_blocks; p.num_blocks = num_blocks;
    p.M = M_max; p.L = L_max; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.total_rows = batch * M_max * Hq;    // partial buffers are sized for the bound; rows index by q_offset
    p.total_M = total_M;
    p.sps = pl.sps; p.nsplit = pl.nsplit;
    set_scales(p, D, scale, k_scale, v_scale);
    p.parent = parent;
    rc = dispatch_bf16<true>(p, pl, D, batch, eb, st);
    if (rc) return rc;
    if (pl.nsplit > 1) {
        dim3 cg((M_max * Hq + 7) / 8, batch);
        if (D == 64) hipLaunchKernelGGL((tv_combine_bf16<64, true>), cg, dim3(256), 0, st, p);
        else hipLaunchKernelGGL((tv_combine_bf16<128, true>), cg, dim3(256), 0, st, p);
        BTV_HIP(hipGetLastError());
    }
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
    BTV_REQUIRE(dtype == BTV_F32 || dtype == BTV_BF16, "dtype=%d unsupported", dtype);
    return attn_contiguous(Q, K, V, parent, M, L, Hq, Hkv, D, dtype, 2, scale, 1.0f, 1.0f, O, ws, ws_bytes, stream);
}

int btv_tree_verify_attn_noalloc(const void *Q, const void *K, const void *V, const int32_t *parent, int M, int L, int Hq,
                                 int Hkv, int D, int dtype, float scale, void *O, uint32_t *status, void *stream)
{
    BTV_REQUIRE(dtype == BTV_F32 || dtype == BTV_BF16, "dtype=%d unsupported", dtype);
    int rc = check_shape(M, L, Hq, Hkv, D);
    if (rc) return rc;
    const size_t need = btv_tree_verify_attn_workspace(M, L, Hq, Hkv, D, dtype);
    if (need > SCRATCH_BYTES)
        return btv_fail(BTV_EWORKSPACE, "this shape needs %zu bytes of scratch, the built-in array holds %zu: use "
                        "btv_tree_verify_attn with a workspace", need, SCRATCH_BYTES);
    void *ws = nullptr;
    rc = scratch_address(&ws);
    if (rc) return rc;
    // the header (data flag, counters) must start at zero whatever an earlier call left behind
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint32_t *>(ws), (int)(BTV_WS_HEADER / 4));
    BTV_HIP(hipGetLastError());
    return attn_contiguous(Q, K, V, parent, M, L, Hq, Hkv, D, dtype, 2, scale, 1.0f, 1.0f, O, ws, SCRATCH_BYTES, stream, 0, 0,
                           status);
}

size_t btv_tree_verify_attn_fp8kv_workspace(int M, int L, int Hq, int Hkv, int D)
{
    if (check_shape(M, L, Hq, Hkv, D) != BTV_OK || D != 128) return 0;
    return ws_layout(M, Hq, D, make_plan(M, L, Hq, Hkv, 1, 1).nsplit).total;
}

int btv_tree_verify_attn_fp8kv(const void *Q, const void *K8, const void *V8, float k_scale, float v_scale,
                               const int32_t *parent, int M, int L, int Hq, int Hkv, int D, float scale, void *O,
                               void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_fp8(D, k_scale, v_scale);
    if (rc) return rc;
    return attn_contiguous(Q, K8, V8, parent, M, L, Hq, Hkv, D, BTV_BF16, 1, scale, k_scale, v_scale, O, ws, ws_bytes,
                           stream);
}

size_t btv_tree_verify_attn_tuned_workspace(int M, int L, int Hq, int Hkv, int D, int kv_fp8, int nsplit, int shape)
{
    if (check_shape(M, L, Hq, Hkv, D) != BTV_OK || (kv_fp8 && D != 128) || nsplit < 0 || shape < 0 || shape > 3) return 0;
    return ws_layout(M, Hq, D, make_plan(M, L, Hq, Hkv, 1, kv_fp8 ? 1 : 2, nsplit, shape).nsplit).total;
}

int btv_tree_verify_attn_tuned(const void *Q, const void *K, const void *V, int kv_fp8, float k_scale, float v_scale,
                               const int32_t *parent, int M, int L, int Hq, int Hkv, int D, float scale, int nsplit,
                               int shape, void *O, void *ws, size_t ws_bytes, void *stream)
{
    BTV_REQUIRE(nsplit >= 0 && shape >= 0 && shape <= 3, "nsplit=%d or shape=%d out of range", nsplit, shape);
    if (kv_fp8) {
        int rc = check_fp8(D, k_scale, v_scale);
        if (rc) return rc;
        BTV_REQUIRE(shape != 3, "shape 3 is not built for an FP8 cache");
    }
    return attn_contiguous(Q, K, V, parent, M, L, Hq, Hkv, D, BTV_BF16, kv_fp8 ? 1 : 2, scale, kv_fp8 ? k_scale : 1.0f,
                           kv_fp8 ? v_scale : 1.0f, O, ws, ws_bytes, stream, nsplit, shape);
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
    return attn_paged(Q, Kpool, Vpool, num_blocks, block_table, max_blocks, q_offset, prefix_len, parent, batch, total_M,
                      M_max, L_max, Hq, Hkv, D, 2, scale, 1.0f, 1.0f, O, ws, ws_bytes, stream);
}

size_t btv_tree_verify_attn_paged_fp8kv_workspace(int batch, int M_max, int L_max, int Hq, int Hkv, int D)
{
    if (batch < 1 || batch > 4096 || check_shape(M_max, L_max, Hq, Hkv, D) != BTV_OK || D != 128) return 0;
    Plan pl = make_plan(M_max, L_max, Hq, Hkv, batch, 1);
    return ws_layout(batch * M_max, Hq, D, pl.nsplit).total;
}

int btv_tree_verify_attn_paged_fp8kv(const void *Q, const void *K8pool, const void *V8pool, float k_scale,
                                     float v_scale, int num_blocks, const int32_t *block_table, int max_blocks,
                                     const int32_t *q_offset, const int32_t *prefix_len, const int32_t *parent,
                                     int batch, int total_M, int M_max, int L_max, int Hq, int Hkv, int D, float scale,
                                     void *O, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_fp8(D, k_scale, v_scale);
    if (rc) return rc;
    return attn_paged(Q, K8pool, V8pool, num_blocks, block_table, max_blocks, q_offset, prefix_len, parent, batch,
                      total_M, M_max, L_max, Hq, Hkv, D, 1, scale, k_scale, v_scale, O, ws, ws_bytes, stream);
}

}  // extern "C"
