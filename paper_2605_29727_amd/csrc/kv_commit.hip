// KV commit on the GPU (gfx950): once a path is accepted, only its nodes' K/V rows are still needed behind the
// prefix (App. C, "Acceptance").  The j-th accepted node's row moves to sequence position L + j, for j < n_acc, in
// every layer, in K and in V.
//
// In place, without a second buffer: an accepted path lists node ids in increasing order with path[j] >= j, so
// the destination of a move never is the source of a LATER move; moves are done in ascending j, a batch of rows
// at a time (all sources of a batch are read into LDS before any of its destinations is written), which also
// covers a destination that is the source of an earlier move.  A path that breaks the rule (data error) still
// touches rows of its own request only: ids are clamped to [0, M).
// One workgroup per (layer, request, K or V); rows are moved as 16-byte pieces, coalesced.
#include "btv_common.h"

namespace {

constexpr int STAGE_BYTES = 32 * 1024;

struct CommitParams {
    unsigned char *K, *V;
    long long layer_stride;           // bytes between layers
    const int32_t *block_table;       // paged: [batch][max_blocks]; contiguous: nullptr
    const int32_t *prefix_len;        // paged: [batch]
    const int32_t *path;              // request r's ids start at q_offset[r] (ragged), else at r * M_max
    const int32_t *q_offset;          // paged, optional: [batch + 1], the ragged layout the batch acceptance writes
    const int32_t *n_acc;             // [batch]
    int32_t *new_len;                 // [batch] optional
    uint32_t *flag;                   // optional data flag
    int L, M_max, max_blocks, num_blocks, row_bytes, total_M;
};

__device__ __forceinline__ size_t row_offset(const CommitParams &p, const int32_t *bt, int pos)
{
    if (!bt) return (size_t)pos * p.row_bytes;
    int blk = bt[min(pos / BTV_PAGE, p.max_blocks - 1)];       // no access leaves the table ...
    blk = min(max(blk, 0), p.num_blocks - 1);                  // ... or the pool
    return ((size_t)blk * BTV_PAGE + pos % BTV_PAGE) * p.row_bytes;
}

__global__ __launch_bounds__(256) void kv_commit_kernel(CommitParams p)
{
    __shared__ __attribute__((aligned(16))) unsigned char stage[STAGE_BYTES];
    const int tid = threadIdx.x, layer = blockIdx.x, rq = blockIdx.y;
    unsigned char *base = (blockIdx.z == 0 ? p.K : p.V) + (size_t)layer * p.layer_stride;
    const int32_t *bt = p.block_table ? p.block_table + (size_t)rq * p.max_blocks : nullptr;
    const int L = p.prefix_len ? p.prefix_len[rq] : p.L;
    int room = p.M_max;                                        // nodes this request may name
    size_t path0 = (size_t)rq * p.M_max;
    bool bad = false;
    if (p.q_offset) {
        const int o0 = p.q_offset[rq];
        room = p.q_offset[rq + 1] - o0;
        bad = o0 < 0 || room < 0 || room > p.M_max || (long long)o0 + room > (long long)p.total_M;
        path0 = bad ? 0 : (size_t)o0;
        if (bad) room = 0;
    }
    const int32_t *path = p.path + path0;
    int n = p.n_acc[rq];
    bad = bad || n < 0 || n > room || L < 0 || (bt && (long long)L + n > (long long)p.max_blocks * BTV_PAGE);
    if (bad) n = 0;
    if (layer == 0 && blockIdx.z == 0 && tid == 0) {
        if (p.new_len) p.new_len[rq] = L + n;
        if (bad && p.flag) atomicOr(p.flag, 8u);
    }
    const int per_row = p.row_bytes / 16;                      // 16-byte pieces per row
    const int rows_per_batch = STAGE_BYTES / p.row_bytes;
    for (int j0 = 0; j0 < n; j0 += rows_per_batch) {
        const int rows = min(rows_per_batch, n - j0);
        for (int e = tid; e < rows * per_row; e += 256) {
            const int j = j0 + e / per_row, piece = e % per_row;
            int src = path[j];
            src = min(max(src, 0), room - 1);
            const uint4 v = *reinterpret_cast<const uint4 *>(base + row_offset(p, bt, L + src) + (size_t)piece * 16);
            *reinterpret_cast<uint4 *>(stage + (size_t)e * 16) = v;
        }
        __syncthreads();
        for (int e = tid; e < rows * per_row; e += 256) {
            const int j = j0 + e / per_row, piece = e % per_row;
            if (path[j] != j)                                   // a row already in place is left alone
                *reinterpret_cast<uint4 *>(base + row_offset(p, bt, L + j) + (size_t)piece * 16) =
                    *reinterpret_cast<const uint4 *>(stage + (size_t)e * 16);
        }
        __syncthreads();
    }
}

int check_common(const void *K, const void *V, int layers, long long layer_stride, int M, int row_bytes, const int32_t *path,
                 const int32_t *n_acc)
{
    BTV_REQUIRE(K && V && path && n_acc, "null pointer");
    BTV_REQUIRE(layers >= 1 && layers <= 65535, "layers=%d outside [1,65535]", layers);
    BTV_REQUIRE(M >= 1 && M <= BTV_MAX_NODES, "M=%d outside [1,%d]", M, BTV_MAX_NODES);
    BTV_REQUIRE(row_bytes >= 16 && row_bytes % 16 == 0 && row_bytes <= STAGE_BYTES, "row_bytes=%d not a multiple of 16 in [16,%d]",
                row_bytes, STAGE_BYTES);
    BTV_REQUIRE(layer_stride >= 0 && layer_stride % 16 == 0, "layer stride %lld not a multiple of 16", layer_stride);
    BTV_REQUIRE((reinterpret_cast<uintptr_t>(K) & 15) == 0 && (reinterpret_cast<uintptr_t>(V) & 15) == 0, "K, V not 16-byte aligned");
    return BTV_OK;
}

}  // namespace

extern "C" {

int btv_kv_commit(void *K, void *V, int layers, long long layer_stride_bytes, int L, int M, int row_bytes,
                  const int32_t *path, const int32_t *n_acc, int32_t *new_len, void *stream)
{
    int rc = check_common(K, V, layers, layer_stride_bytes, M, row_bytes, path, n_acc);
    if (rc) return rc;
    BTV_REQUIRE(L >= 0 && (long long)L + M < (1ll << 30), "L=%d out of range", L);
    BTV_REQUIRE(layers == 1 || layer_stride_bytes >= (long long)(L + M) * row_bytes, "layers overlap");
    CommitParams p = {};
    p.K = static_cast<unsigned char *>(K); p.V = static_cast<unsigned char *>(V);
    p.layer_stride = layer_stride_bytes; p.path = path; p.n_acc = n_acc; p.new_len = new_len;
    p.L = L; p.M_max = M; p.row_bytes = row_bytes; p.num_blocks = 1;
    hipLaunchKernelGGL(kv_commit_kernel, dim3(layers, 1, 2), dim3(256), 0, static_cast<hipStream_t>(stream), p);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

int btv_kv_commit_paged(void *Kpool, void *Vpool, int layers, long long layer_stride_bytes, int num_blocks,
                        const int32_t *block_table, int max_blocks, const int32_t *prefix_len, const int32_t *path,
                        const int32_t *q_offset, int total_M, const int32_t *n_acc, int batch, int M_max, int row_bytes,
                        int32_t *new_len, void *ws, void *stream)
{
    int rc = check_common(Kpool, Vpool, layers, layer_stride_bytes, M_max, row_bytes, path, n_acc);
    if (rc) return rc;
    BTV_REQUIRE(block_table && prefix_len, "null pointer");
    BTV_REQUIRE(batch >= 1 && batch <= 65535, "batch=%d outside [1,65535]", batch);
    BTV_REQUIRE(!q_offset || (total_M >= 1 && total_M <= batch * M_max), "total_M=%d inconsistent with batch*M_max", total_M);
    BTV_REQUIRE(num_blocks >= 1 && max_blocks >= 1, "num_blocks=%d max_blocks=%d", num_blocks, max_blocks);
    BTV_REQUIRE(layers == 1 || layer_stride_bytes >= (long long)num_blocks * BTV_PAGE * row_bytes, "layers overlap");
    CommitParams p = {};
    p.K = static_cast<unsigned char *>(Kpool); p.V = static_cast<unsigned char *>(Vpool);
    p.layer_stride = layer_stride_bytes; p.block_table = block_table; p.prefix_len = prefix_len;
    p.path = path; p.q_offset = q_offset; p.total_M = total_M; p.n_acc = n_acc; p.new_len = new_len;
    p.flag = static_cast<uint32_t *>(ws);
    p.M_max = M_max; p.max_blocks = max_blocks; p.num_blocks = num_blocks; p.row_bytes = row_bytes;
    hipLaunchKernelGGL(kv_commit_kernel, dim3(layers, batch, 2), dim3(256), 0, static_cast<hipStream_t>(stream), p);
    BTV_HIP(hipGetLastError());
    return BTV_OK;
}

}  // extern "C"
