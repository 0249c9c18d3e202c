// Internal launch interfaces between the C-ABI layer (dd_api.hip) and the kernels.
// Everything here takes validated arguments; shapes were checked by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <utility>

namespace dd {

// Launch through the runtime call that RETURNS the status of this launch, so that a stale
// error left in the thread by an unrelated earlier runtime call is never reported as ours.
template <typename... Params, size_t... I>
inline hipError_t launch_impl(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream,
                              std::tuple<Params...> &vals, std::index_sequence<I...>)
{
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, 0, stream);
}
template <typename... Params, typename... Args>
inline hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args... args)
{
    std::tuple<Params...> vals{args...};
    return launch_impl(kernel, grid, block, stream, vals, std::index_sequence_for<Params...>{});
}

// Test hooks.  The kernel a call runs on is chosen from its shape alone; so that the tests can reach every
// kernel with every shape, a process started with DD_TUNE=1 in its environment (looked at once) lets the
// variables below override single choices, read at every call.  Without DD_TUNE no call reads the environment.
//   DD_TUNE_ATTN_WIDE=0/1      verifier attention off / on the wide-wave kernel
//   DD_TUNE_ATTN_WIDE_GRID=n   at most n persistent workgroups on that kernel
//   DD_TUNE_BIDIR_STREAM=0/1   small bf16 verifier calls off / on the streaming kernel
//   DD_TUNE_BLOCK_STREAM=0     drafter calls with few query rows off the streaming kernel
//   DD_TUNE_BLOCK_WIDE=0       drafter calls with many query rows off the wide-wave kernel
//   DD_TUNE_BLOCK_SPLITS=n     key splits of a drafter call on the streaming / MFMA kernels (still at least 128 keys each)
//   DD_TUNE_BLOCK_WIDE_ROWS=128/256   query rows per workgroup of such a call
//   DD_TUNE_BLOCK_WIDE_MIN_ROWS=n     query rows per kv head from which it takes that kernel
// Returns the variable's integer value, or `dflt` when hooks are off or the variable is unset.
int tune(const char *name, int dflt);

// ---- verification (verify.hip) -------------------------------------------------
// Number of workgroups one logit row is split over, and workspace size.
int verify_splits(int P, int V, int elem_bytes);
size_t verify_workspace_bytes(int P, int V, int elem_bytes);
// `mode`: a dd_mode value, or one of the two below for the drafter's unmasking step (logits_v then holds the
// drafter's logits, logits_d is unused, and x_tokens - optional - receives the tokens of the selected rows).
constexpr int kModeUnmaskThresh = 100, kModeUnmaskTopk = 101;
// kModeScores: no rule and no mask; out_scores gets the divergence, out_tokens the verifier's argmax, and the
// fields of `extra` the remaining per-position quantities (conf_v required, the drafter's two optional).
constexpr int kModeScores = 200;
struct VerifyExtra {
    float *conf_v = nullptr;
    float *conf_d = nullptr;
    int32_t *tok_d = nullptr;
};
hipError_t launch_verify(const void *logits_d, const void *logits_v, const uint8_t *mask,
                         int mode, float threshold, uint64_t seed,
                         uint8_t *out_mask, int32_t *out_tokens, float *out_scores,
                         int B, int G, int V, int logit_is_bf16, void *workspace, hipStream_t stream,
                         int32_t *x_tokens = nullptr, const VerifyExtra *extra = nullptr);

// ---- attention (attention_mfma.hip, attention_f32.hip) -------------------------
// One description serves the verifier's full attention and the drafter's block attention:
// for every (batch, kv head) the `group * Nq` query rows of the heads sharing that kv head
// attend keys [0, N); key row j is taken from (Kblk, Vblk) when Kblk != nullptr and
// block_start <= j < block_start + block_len, else from (K, V).
struct AttnArgs {
    const void *Q;       // [B, H, Nq, d]
    const void *K;       // [B, Hkv, N, d]
    const void *V;       // [B, Hkv, N, d]
    const void *Kblk;    // [B, Hkv, block_len, d] or nullptr
    const void *Vblk;
    void *O;             // [B, H, Nq, d]
    const float *q_scale;  // [B*H] or nullptr
    const float *k_scale;  // [B*Hkv] or nullptr
    const float *v_scale = nullptr;  // [B*Hkv]: multiplier of the decoded V values; required when V is fp8
    // block-scaled inputs (all three or none): E8M0 scale bytes, one per 32 elements of the head dimension, of Q
    // [B*H*Nq][d/32], K and V [B*Hkv*N][d/32]; Q and K then hold e4m3 codes, V packed e2m1 codes (d/2 bytes per row)
    const uint8_t *q_mx = nullptr, *k_mx = nullptr, *v_mx = nullptr;
    int B, H, Hkv, Nq, N, d;
    int kv_stride = 0;       // rows between consecutive (batch, kv head) of K and V; 0 = N (dense).  A call on a
                             // window of the cache passes K/V at the window's first row, N = the window length
    int block_start, block_len;
    const int32_t *block_starts = nullptr;   // device [B] or nullptr: the block's first row per batch entry
                                             // (overrides block_start; not served by the wide kernel)
    int qk_dtype, v_dtype;   // dd_dtype values
    int splits;              // key-range splits (1 = write O directly)
    void *workspace;         // partial states when splits > 1
    // Block-completion refresh: when set (both or neither; Kblk/Vblk then required) the rows
    // [block_start, block_start + block_len) of the cache are overwritten with Kblk / Vblk by the same call.
    // No workgroup of the call reads those cache rows, so the copy may run at any point of it.
    void *K_refresh = nullptr;   // = K, writable
    void *V_refresh = nullptr;   // = V, writable
};

int attn_block_splits(int block_len, int B, int H, int Hkv, int N, int d);
int attn_block_rows_per_wg(int block_len, int B, int H, int Hkv);
size_t attn_partial_bytes(int B, int H, int Nq, int d, int splits);
hipError_t launch_attention_mfma(const AttnArgs &a, hipStream_t stream);   // bf16 / fp8 inputs
hipError_t launch_attention_f32(const AttnArgs &a, hipStream_t stream);    // fp32 inputs
hipError_t launch_attention_wide(const AttnArgs &a, hipStream_t stream);   // bf16 verifier form, 64 rows per wave
hipError_t launch_attention_stream(const AttnArgs &a, hipStream_t stream);  // bf16 drafter form, few query rows
// drafter form on the wide kernel (a few hundred query rows per kv head): whether the call qualifies, the
// key splits it then uses (a.splits must hold them), the launch (+ merge kernel)
bool attn_wide_block_fits(const AttnArgs &a);
int attn_wide_block_splits(int block_len, int B, int H, int Hkv, int N);
int attn_wide_block_rows(int block_len, int B, int H, int Hkv, int N);      // 256 or 128 query rows per workgroup
hipError_t launch_attention_wide_block(const AttnArgs &a, hipStream_t stream);
bool attn_stream_fits(const AttnArgs &a);

// ---- cache maintenance (cache.hip) ----------------------------------------------
// Row r of Krows/Vrows [B, Hkv, n, d] replaces cache row pos[b * n + r] of every kv head of batch b
// (entries outside [0, N) are skipped by the kernel).
hipError_t launch_cache_insert_rows(const void *Krows, const void *Vrows, void *Kc, void *Vc, const int32_t *pos,
                                    int n, int B, int Hkv, int N, int d, int k_elem_bytes, int v_elem_bytes,
                                    hipStream_t stream);
// merge of the partial states (a.splits > 1), carrying the cache refresh on extra workgroups when one is asked for
hipError_t launch_attention_combine(const AttnArgs &a, hipStream_t stream);
// what every attention launcher ends with: the merge if the key range was split (`splits_used` > 1),
// else the cache refresh alone if one is asked for, else nothing
hipError_t finish_attention(const AttnArgs &a, int splits_used, hipStream_t stream);

}  // namespace dd
