// Device-side argument block and work decomposition shared by the attention kernels.
//
// Both the verifier's full bidirectional attention (Sec. 2.2) and the drafter's block
// attention over a cached K/V (Sec. 2.3) are softmax(Q K^T / sqrt(d_k)) V (Eq. 3) over
// every key position; they differ only in which query rows exist and where a key row is
// read from.  The kernels therefore work on "virtual rows": for one (batch, kv head) the
// query rows of the `group` query heads that share it, v = (head - kvh*group) * Nq + i.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dd {

struct AttnKernelArgs {
    const void *Q, *K, *V, *Kblk, *Vblk;
    void *O;                   // final output (splits == 1)
    float *part_o;             // [rows][splits][d] unnormalised partial outputs (splits > 1)
    float *part_ml;            // [rows][splits][2] (running max in log2 units, partial sum)
    const float *q_scale, *k_scale;
    const float *v_scale;      // [B*Hkv] or nullptr: multiplier of the decoded V values (fp8 V)
    const uint8_t *q_mx, *k_mx, *v_mx;   // block-scaled inputs: E8M0 scales [rows][d / 32] of Q, K, V; nullptr otherwise
    int B, H, Hkv, Nq, N;
    int kv_stride;             // rows between consecutive (batch, kv head) in K and V (N unless the call sees a window)
    int group;                 // H / Hkv
    int rows_per_wg;           // query rows per workgroup (a multiple of a wave's rows)
    int row_tiles;             // ceil(group * Nq / rows_per_wg)
    int splits;                // key-range splits
    int keys_per_split;        // multiple of the key tile
    int block_start, block_len;
    const int32_t *block_starts;   // [B] or nullptr: the block's first row per batch entry (overrides block_start)
    float scale_log2;          // log2(e) / sqrt(d)
};

constexpr int kAttnThreads = 256;

struct AttnArgs;
// Host side: derive the launch decomposition (row tiles, key splits, partial buffers).
void fill_kernel_args(const AttnArgs &a, AttnKernelArgs &k, int rows_per_wg, int key_tile);

}  // namespace dd
