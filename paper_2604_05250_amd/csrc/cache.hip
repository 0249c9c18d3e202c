// Token-granular maintenance of the drafter's K/V cache.
//
// The drafters cited in Sec. 2.3 differ in WHEN a position's key/value enter the cache: block-wise caches
// refresh a whole block when it is complete (dd_block_attention_refresh), dKV-Cache inserts the rows of the
// tokens decoded at the previous step, one step late.  Either way the operation on the cache is the same:
// rows computed by the model this step replace the cache rows of chosen positions.  This file holds the
// scatter form: for every (batch, kv head), row r of a dense [n, d] tensor goes to cache row pos[b][r].
#include "dd_internal.h"

namespace dd {
namespace {

// one thread per 16-byte chunk of the larger of the two row types; K and V rows of a position travel together
__global__ __launch_bounds__(256) void cache_insert_rows_kernel(const uint4 *__restrict__ krows,
                                                                const uint4 *__restrict__ vrows,
                                                                uint4 *__restrict__ kc, uint4 *__restrict__ vc,
                                                                const int32_t *__restrict__ pos,
                                                                int Hkv, int n, int N, int kchunks, int vchunks,
                                                                long total_rows)
{
    const int cmax = kchunks > vchunks ? kchunks : vchunks;              // chunks per row: 4 .. 32, a power of two
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long row = gid / cmax;                                        // (b * Hkv + g) * n + r
    const int ch = (int)(gid - row * cmax);
    if (row >= total_rows) return;
    const long bg = row / n;
    const int r = (int)(row - bg * n);
    const long b = bg / Hkv;
    const int p = pos[b * n + r];
    if (p < 0 || p >= N) return;                                         // not a position of the cache: skipped
    const long dst = bg * N + p;
    if (ch < kchunks) kc[dst * kchunks + ch] = krows[row * kchunks + ch];
    if (ch < vchunks) vc[dst * vchunks + ch] = vrows[row * vchunks + ch];
}

}  // namespace

hipError_t launch_cache_insert_rows(const void *Krows, const void *Vrows, void *Kc, void *Vc, const int32_t *pos,
                                    int n, int B, int Hkv, int N, int d, int k_elem_bytes, int v_elem_bytes,
                                    hipStream_t stream)
{
    const int kchunks = d * k_elem_bytes / 16, vchunks = d * v_elem_bytes / 16;
    const int cmax = kchunks > vchunks ? kchunks : vchunks;
    const long total_rows = (long)B * Hkv * n;
    if (total_rows == 0) return hipSuccess;
    const long threads = total_rows * cmax;
    return launch(cache_insert_rows_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), stream,
                  static_cast<const uint4 *>(Krows), static_cast<const uint4 *>(Vrows), static_cast<uint4 *>(Kc),
                  static_cast<uint4 *>(Vc), pos, Hkv, n, N, kchunks, vchunks, total_rows);
}

}  // namespace dd
