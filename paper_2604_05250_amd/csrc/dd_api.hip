// C ABI of the library: argument validation (host only, before any GPU call) and dispatch
// to the kernels.  See include/dd.h for the contract of every entry point.
#include "../../include/dd.h"
#include "dd_internal.h"

#include <cstdlib>
#include <mutex>

namespace {

// Scratch memory of dd_verify_remask_static: one copy per GPU, at its own address on each, held from the moment
// the library's code is loaded on that GPU until the process ends.  The name below is a host-side handle only;
// the device address is looked up once per device (scratch_of_current_device) and is what the kernels get.
constexpr size_t kStaticScratchBytes = 128u * 1024u;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];            // device address of `scratch` on device i, or nullptr: not looked up yet
std::mutex g_scratch_mutex;

int scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DD_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return DD_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DD_OK;
}

inline bool misaligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_attention_common(int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                           const float *q_scale, const float *k_scale, const float *v_scale = nullptr)
{
    if (B < 1 || H < 1 || Hkv < 1 || N < 1) return DD_ERR_SHAPE;
    if (H % Hkv != 0) return DD_ERR_SHAPE;
    if (d != 64 && d != 128) return DD_ERR_SHAPE;
    if ((double)B * H * N * d >= 1099511627776.0) return DD_ERR_SHAPE;
    // (fp8 V - with fp8 Q/K - only through the entry points that carry its scale)
    const bool ok = (qk_dtype == DD_F32 && v_dtype == DD_F32) || (qk_dtype == DD_BF16 && v_dtype == DD_BF16) ||
                    (qk_dtype == DD_FP8_E4M3 && v_dtype == DD_BF16) ||
                    (qk_dtype == DD_FP8_E4M3 && v_dtype == DD_FP8_E4M3 && v_scale != nullptr);
    if (!ok) return DD_ERR_DTYPE;
    if (qk_dtype == DD_FP8_E4M3 && (!q_scale || !k_scale)) return DD_ERR_NULL;
    return DD_OK;
}

int check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return DD_OK;
    if (!ws || have < need) return DD_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return DD_ERR_WORKSPACE;
    return DD_OK;
}

}  // namespace

namespace dd {

int tune(const char *name, int dflt)
{
    static const bool hooks = [] { const char *e = getenv("DD_TUNE"); return e && e[0] == '1'; }();
    if (!hooks) return dflt;
    const char *e = getenv(name);
    return e && *e ? atoi(e) : dflt;
}

// Query rows per workgroup of the drafter's MFMA kernel.  Smaller row tiles (64, 32: more workgroups that
// stream the same K/V side by side) were measured and lose on every benchmark shape.
int attn_block_rows_per_wg(int block_len, int B, int H, int Hkv)
{
    (void)block_len; (void)B; (void)H; (void)Hkv;
    return 128;
}

int attn_block_splits(int block_len, int B, int H, int Hkv, int N, int d)
{
    (void)d;
    const int group = H / Hkv;
    const int r = attn_block_rows_per_wg(block_len, B, H, Hkv);
    const long base = (long)B * Hkv * ((group * block_len + r - 1) / r);
    // Every extra split adds partial-state traffic and merge work, so the key range is only split until
    // there is about one workgroup per compute unit.
    const int target = 256;
    long s = (target + base - 1) / base;
    const long forced = tune("DD_TUNE_BLOCK_SPLITS", 0);
    if (forced >= 1) s = forced;
    const long max_s = N / 128 > 1 ? N / 128 : 1;   // at least 128 keys per split
    if (s > max_s) s = max_s;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    return (int)s;
}

size_t attn_partial_bytes(int B, int H, int Nq, int d, int splits)
{
    if (splits <= 1) return 0;
    return (size_t)B * H * Nq * (size_t)splits * (size_t)(d + 2) * sizeof(float);
}

}  // namespace dd

extern "C" {

const char *dd_strerror(int status)
{
    switch (status) {
    case DD_OK: return "ok";
    case DD_ERR_NULL: return "a required pointer is NULL";
    case DD_ERR_SHAPE: return "a size is out of range or inconsistent";
    case DD_ERR_DTYPE: return "unsupported element type or combination";
    case DD_ERR_MODE: return "unknown remask mode";
    case DD_ERR_WORKSPACE: return "workspace is NULL, too small or not 256-byte aligned";
    case DD_ERR_ALIGN: return "a pointer or row pitch is not 16-byte aligned";
    case DD_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
    }
}

int dd_version(void) { return 100; }

size_t dd_bidir_attention_workspace_bytes(int, int, int, int, int, dd_dtype, dd_dtype) { return 0; }

int dd_bidir_attention(const void *Q, const void *K, const void *V, void *O,
                       int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                       const float *q_scale, const float *k_scale,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace; (void)workspace_bytes;
    if (!Q || !K || !V || !O) return DD_ERR_NULL;
    const int rc = check_attention_common(B, H, Hkv, N, d, qk_dtype, v_dtype, q_scale, k_scale);
    if (rc != DD_OK) return rc;
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O)) return DD_ERR_ALIGN;
    dd::AttnArgs a{};
    a.Q = Q; a.K = K; a.V = V; a.Kblk = nullptr; a.Vblk = nullptr; a.O = O;
    a.q_scale = q_scale; a.k_scale = k_scale;
    a.B = B; a.H = H; a.Hkv = Hkv; a.Nq = N; a.N = N; a.d = d;
    a.block_start = 0; a.block_len = 0;
    a.qk_dtype = qk_dtype; a.v_dtype = v_dtype;
    a.splits = 1; a.workspace = nullptr;
    const hipError_t e = (qk_dtype == DD_F32) ? dd::launch_attention_f32(a, static_cast<hipStream_t>(stream))
                                              : dd::launch_attention_mfma(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

size_t dd_block_attention_cached_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d,
                                                 dd_dtype qk_dtype, dd_dtype v_dtype)
{
    if (check_attention_common(B, H, Hkv, N, d, qk_dtype, v_dtype, (const float *)16, (const float *)16) != DD_OK) return 0;
    if (block_len < 1 || block_len > N) return 0;
    // which kernel serves the call also depends on block_start: enough for either plan
    const size_t narrow = dd::attn_partial_bytes(B, H, block_len, d, dd::attn_block_splits(block_len, B, H, Hkv, N, d));
    const size_t wide = dd::attn_partial_bytes(B, H, block_len, d, dd::attn_wide_block_splits(block_len, B, H, Hkv, N));
    return narrow > wide ? narrow : wide;
}

}  // extern "C"

// the drafter's call, with (refresh) or without the block's rows written back into the cache, over the
// whole cache (win_len == 0) or over the key rows [win_start, win_start + win_len) only
static int block_attention(const void *Qblk, const void *Kc, const void *Vc, void *O,
                           int block_start, int block_len, const void *Kblk, const void *Vblk,
                           int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                           const float *q_scale, const float *k_scale,
                           void *workspace, size_t workspace_bytes, void *stream, bool refresh,
                           int win_start = 0, int win_len = 0, const int32_t *block_starts = nullptr,
                           const float *v_scale = nullptr)
{
    if (!Qblk || !Kc || !Vc || !O) return DD_ERR_NULL;
    if ((Kblk == nullptr) != (Vblk == nullptr)) return DD_ERR_NULL;
    if (refresh && !Kblk) return DD_ERR_NULL;
    if (refresh && block_len > (1 << 25)) return DD_ERR_SHAPE;   // the copy indexes a block's 16-byte chunks with 32 bits
    int rc = check_attention_common(B, H, Hkv, N, d, qk_dtype, v_dtype, q_scale, k_scale, v_scale);
    if (rc != DD_OK) return rc;
    if (block_start < 0 || block_len < 1 || (long)block_start + block_len > N) return DD_ERR_SHAPE;
    const int full_N = N;
    if (win_len != 0) {
        // a window is a shorter sequence that starts win_start rows into every (batch, kv head) of the cache:
        // same kernels, K/V based at the window's first row, the cache's own row count as the stride
        if (win_start < 0 || win_len < 1 || (long)win_start + win_len > N) return DD_ERR_SHAPE;
        if (block_start < win_start || (long)block_start + block_len > (long)win_start + win_len) return DD_ERR_SHAPE;
        const size_t ebk = qk_dtype == DD_F32 ? 4 : qk_dtype == DD_BF16 ? 2 : 1;
        const size_t ebv = v_dtype == DD_F32 ? 4 : v_dtype == DD_BF16 ? 2 : 1;
        Kc = static_cast<const uint8_t *>(Kc) + (size_t)win_start * d * ebk;
        Vc = static_cast<const uint8_t *>(Vc) + (size_t)win_start * d * ebv;
        block_start -= win_start;
        N = win_len;
    }
    if (misaligned16(Qblk) || misaligned16(Kc) || misaligned16(Vc) || misaligned16(O) ||
        misaligned16(Kblk) || misaligned16(Vblk))
        return DD_ERR_ALIGN;
    dd::AttnArgs a{};
    a.Q = Qblk; a.K = Kc; a.V = Vc; a.Kblk = Kblk; a.Vblk = Vblk; a.O = O;
    a.q_scale = q_scale; a.k_scale = k_scale; a.v_scale = v_scale;
    a.B = B; a.H = H; a.Hkv = Hkv; a.Nq = block_len; a.N = N; a.d = d;
    a.block_start = block_start; a.block_len = block_len;
    a.qk_dtype = qk_dtype; a.v_dtype = v_dtype;
    a.workspace = workspace;
    a.kv_stride = full_N;
    a.block_starts = block_starts;
    if (refresh) {
        a.K_refresh = const_cast<void *>(Kc);
        a.V_refresh = const_cast<void *>(Vc);
    }
    const bool wide = dd::tune("DD_TUNE_BLOCK_WIDE", 1) != 0 && dd::attn_wide_block_fits(a);
    const int splits = wide ? dd::attn_wide_block_splits(block_len, B, H, Hkv, N)
                            : dd::attn_block_splits(block_len, B, H, Hkv, N, d);
    rc = check_workspace(workspace, workspace_bytes, dd::attn_partial_bytes(B, H, block_len, d, splits));
    if (rc != DD_OK) return rc;
    a.splits = splits;
    if (wide)
        return dd::launch_attention_wide_block(a, static_cast<hipStream_t>(stream)) == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
    const hipError_t e = (qk_dtype == DD_F32) ? dd::launch_attention_f32(a, static_cast<hipStream_t>(stream))
                                              : dd::launch_attention_mfma(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

extern "C" {

int dd_block_attention_cached(const void *Qblk, const void *Kc, const void *Vc, void *O,
                              int block_start, int block_len, const void *Kblk, const void *Vblk,
                              int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                              const float *q_scale, const float *k_scale,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return block_attention(Qblk, Kc, Vc, O, block_start, block_len, Kblk, Vblk, B, H, Hkv, N, d, qk_dtype, v_dtype,
                           q_scale, k_scale, workspace, workspace_bytes, stream, false);
}

int dd_bidir_attention_fp8v(const void *Q, const void *K, const void *V, void *O,
                            int B, int H, int Hkv, int N, int d,
                            const float *q_scale, const float *k_scale, const float *v_scale, void *stream)
{
    if (!Q || !K || !V || !O || !v_scale) return DD_ERR_NULL;
    const int rc = check_attention_common(B, H, Hkv, N, d, DD_FP8_E4M3, DD_FP8_E4M3, q_scale, k_scale, v_scale);
    if (rc != DD_OK) return rc;
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O)) return DD_ERR_ALIGN;
    dd::AttnArgs a{};
    a.Q = Q; a.K = K; a.V = V; a.Kblk = nullptr; a.Vblk = nullptr; a.O = O;
    a.q_scale = q_scale; a.k_scale = k_scale; a.v_scale = v_scale;
    a.B = B; a.H = H; a.Hkv = Hkv; a.Nq = N; a.N = N; a.d = d;
    a.block_start = 0; a.block_len = 0;
    a.qk_dtype = DD_FP8_E4M3; a.v_dtype = DD_FP8_E4M3;
    a.splits = 1; a.workspace = nullptr;
    return dd::launch_attention_mfma(a, static_cast<hipStream_t>(stream)) == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

int dd_bidir_attention_mx(const void *Q, const void *Qs, const void *K, const void *Ks, const void *V, const void *Vs,
                          void *O, int B, int H, int Hkv, int N, int d, void *stream)
{
    if (!Q || !Qs || !K || !Ks || !V || !Vs || !O) return DD_ERR_NULL;
    const float one = 1.0f;                    // (the per-head scales of the plain fp8 form are not part of this one)
    const int rc = check_attention_common(B, H, Hkv, N, d, DD_FP8_E4M3, DD_BF16, &one, &one);
    if (rc != DD_OK) return rc;
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O)) return DD_ERR_ALIGN;
    // (a row's scale bytes are read as one word)
    if (((reinterpret_cast<uintptr_t>(Qs) | reinterpret_cast<uintptr_t>(Ks) | reinterpret_cast<uintptr_t>(Vs)) & 3u) != 0) return DD_ERR_ALIGN;
    dd::AttnArgs a{};
    a.Q = Q; a.K = K; a.V = V; a.Kblk = nullptr; a.Vblk = nullptr; a.O = O;
    a.q_scale = nullptr; a.k_scale = nullptr;
    a.q_mx = static_cast<const uint8_t *>(Qs); a.k_mx = static_cast<const uint8_t *>(Ks); a.v_mx = static_cast<const uint8_t *>(Vs);
    a.B = B; a.H = H; a.Hkv = Hkv; a.Nq = N; a.N = N; a.d = d;
    a.block_start = 0; a.block_len = 0;
    a.qk_dtype = DD_FP8_E4M3; a.v_dtype = DD_BF16;     // (storage of V: packed e2m1; its decoded form is bf16)
    a.splits = 1; a.workspace = nullptr;
    return dd::launch_attention_mfma(a, static_cast<hipStream_t>(stream)) == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

size_t dd_block_attention_cached_fp8v_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d)
{
    return dd_block_attention_cached_workspace_bytes(block_len, B, H, Hkv, N, d, DD_FP8_E4M3, DD_BF16);
}

int dd_block_attention_cached_fp8v(const void *Qblk, const void *Kc, const void *Vc, void *O,
                                   int block_start, int block_len, const void *Kblk, const void *Vblk,
                                   int B, int H, int Hkv, int N, int d,
                                   const float *q_scale, const float *k_scale, const float *v_scale,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!v_scale) return DD_ERR_NULL;
    return block_attention(Qblk, Kc, Vc, O, block_start, block_len, Kblk, Vblk, B, H, Hkv, N, d, DD_FP8_E4M3,
                           DD_FP8_E4M3, q_scale, k_scale, workspace, workspace_bytes, stream, false, 0, 0, nullptr, v_scale);
}

size_t dd_block_attention_refresh_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d,
                                                  dd_dtype qk_dtype, dd_dtype v_dtype)
{
    return dd_block_attention_cached_workspace_bytes(block_len, B, H, Hkv, N, d, qk_dtype, v_dtype);
}

int dd_block_attention_refresh(const void *Qblk, void *Kc, void *Vc, void *O,
                               int block_start, int block_len, const void *Kblk, const void *Vblk,
                               int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                               const float *q_scale, const float *k_scale,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    return block_attention(Qblk, Kc, Vc, O, block_start, block_len, Kblk, Vblk, B, H, Hkv, N, d, qk_dtype, v_dtype,
                           q_scale, k_scale, workspace, workspace_bytes, stream, true);
}

size_t dd_block_attention_batched_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d,
                                                  dd_dtype qk_dtype, dd_dtype v_dtype)
{
    return dd_block_attention_cached_workspace_bytes(block_len, B, H, Hkv, N, d, qk_dtype, v_dtype);
}

int dd_block_attention_batched(const void *Qblk, const void *Kc, const void *Vc, void *O,
                               const int32_t *block_starts, int block_len, const void *Kblk, const void *Vblk,
                               int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                               const float *q_scale, const float *k_scale,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    if (!block_starts || !Kblk || !Vblk) return DD_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(block_starts) & 3u) != 0) return DD_ERR_ALIGN;
    return block_attention(Qblk, Kc, Vc, O, 0, block_len, Kblk, Vblk, B, H, Hkv, N, d, qk_dtype, v_dtype,
                           q_scale, k_scale, workspace, workspace_bytes, stream, false, 0, 0, block_starts);
}

size_t dd_block_attention_window_workspace_bytes(int block_len, int win_len, int B, int H, int Hkv, int N, int d,
                                                 dd_dtype qk_dtype, dd_dtype v_dtype)
{
    if (win_len < 1 || win_len > N) return 0;
    if (check_attention_common(B, H, Hkv, N, d, qk_dtype, v_dtype, (const float *)16, (const float *)16) != DD_OK) return 0;
    return dd_block_attention_cached_workspace_bytes(block_len, B, H, Hkv, win_len, d, qk_dtype, v_dtype);
}

int dd_block_attention_window(const void *Qblk, const void *Kc, const void *Vc, void *O,
                              int block_start, int block_len, int win_start, int win_len,
                              const void *Kblk, const void *Vblk,
                              int B, int H, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype,
                              const float *q_scale, const float *k_scale,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (win_len < 1) return DD_ERR_SHAPE;
    return block_attention(Qblk, Kc, Vc, O, block_start, block_len, Kblk, Vblk, B, H, Hkv, N, d, qk_dtype, v_dtype,
                           q_scale, k_scale, workspace, workspace_bytes, stream, false, win_start, win_len);
}

int dd_cache_insert_rows(void *Kc, void *Vc, const void *Krows, const void *Vrows, const int32_t *positions, int n,
                         int B, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype, void *stream)
{
    if (n < 0) return DD_ERR_SHAPE;
    const int rc = check_attention_common(B, Hkv, Hkv, N, d, qk_dtype, v_dtype, (const float *)16, (const float *)16);
    if (rc != DD_OK) return rc;
    if ((double)B * Hkv * n * d >= 1099511627776.0) return DD_ERR_SHAPE;
    if (n == 0) return DD_OK;
    if (!Kc || !Vc || !Krows || !Vrows || !positions) return DD_ERR_NULL;
    if (misaligned16(Kc) || misaligned16(Vc) || misaligned16(Krows) || misaligned16(Vrows)) return DD_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(positions) & 3u) != 0) return DD_ERR_ALIGN;
    const int ebk = qk_dtype == DD_F32 ? 4 : qk_dtype == DD_BF16 ? 2 : 1, ebv = v_dtype == DD_F32 ? 4 : 2;
    const hipError_t e = dd::launch_cache_insert_rows(Krows, Vrows, Kc, Vc, positions, n, B, Hkv, N, d, ebk, ebv,
                                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

size_t dd_verify_remask_workspace_bytes(int B, int G, int V, dd_dtype logit_dtype)
{
    if (B < 0 || G < 0 || V < 1 || (logit_dtype != DD_F32 && logit_dtype != DD_BF16)) return 0;
    if ((double)B * G >= 2147483648.0) return 0;
    return dd::verify_workspace_bytes(B * G, V, logit_dtype == DD_BF16 ? 2 : 4);
}

}  // extern "C"

// everything dd_verify_remask checks before it launches, except the workspace; DD_OK with *empty set for a no-op
static int check_verify_remask(const void *logits_d, const void *logits_v, const uint8_t *mask, int mode, float threshold,
                               const uint8_t *out_mask, const int32_t *out_tokens, const float *out_scores,
                               int B, int G, int V, int logit_dtype, bool *empty)
{
    *empty = false;
    if (mode < DD_TRUST || mode > DD_CONF_TOPK) return DD_ERR_MODE;
    if ((mode == DD_KL_TOPK || mode == DD_CONF_TOPK) && !(threshold >= 0.0f && threshold <= 3.0e38f)) return DD_ERR_SHAPE;
    if (logit_dtype != DD_F32 && logit_dtype != DD_BF16) return DD_ERR_DTYPE;
    if (B < 0 || G < 0 || V < 1) return DD_ERR_SHAPE;
    if ((double)B * G >= 2147483648.0) return DD_ERR_SHAPE;
    const int eb = logit_dtype == DD_BF16 ? 2 : 4;
    if (((long)V * eb) % 16 != 0) return DD_ERR_ALIGN;
    if (B == 0 || G == 0) {
        *empty = true;
        return DD_OK;
    }
    const bool kl = (mode == DD_KL_THRESH || mode == DD_KL_PROB || mode == DD_KL_TOPK);
    if (!logits_v || !mask || !out_mask || !out_tokens || !out_scores) return DD_ERR_NULL;
    if (kl && !logits_d) return DD_ERR_NULL;
    {
        // The per-row rules read mask[i] and write out_mask[i] in one lane, so updating the mask in place is
        // safe; the per-sequence rules (Eq. 6, the budgeted ones) read every mask byte of a sequence while other
        // workgroups write out_mask.  Ranges that overlap without being identical are never meaningful.
        const uintptr_t m0 = reinterpret_cast<uintptr_t>(mask), o0 = reinterpret_cast<uintptr_t>(out_mask);
        const uintptr_t n = (uintptr_t)B * (uintptr_t)G;
        const bool overlap = m0 < o0 + n && o0 < m0 + n;
        const bool per_sequence = mode == DD_KL_PROB || mode == DD_KL_TOPK || mode == DD_CONF_TOPK;
        if (overlap && (per_sequence || m0 != o0)) return DD_ERR_SHAPE;
    }
    if (misaligned16(logits_v) || (kl && misaligned16(logits_d))) return DD_ERR_ALIGN;
    return DD_OK;
}

static int verify_remask(const void *logits_d, const void *logits_v, const uint8_t *mask, int mode, float threshold,
                         uint64_t seed, uint8_t *out_mask, int32_t *out_tokens, float *out_scores, int B, int G, int V,
                         int logit_dtype, void *workspace, size_t workspace_bytes, void *stream, bool static_scratch)
{
    bool empty = false;
    int rc = check_verify_remask(logits_d, logits_v, mask, mode, threshold, out_mask, out_tokens, out_scores, B, G, V,
                                 logit_dtype, &empty);
    if (rc != DD_OK || empty) return rc;
    const int eb = logit_dtype == DD_BF16 ? 2 : 4;
    const size_t need = dd::verify_workspace_bytes(B * G, V, eb);
    if (static_scratch) {
        if (need > kStaticScratchBytes) return DD_ERR_WORKSPACE;  // more partial states than the static array holds
        workspace = nullptr;
        workspace_bytes = need;
        if (need > 0 && (rc = scratch_of_current_device(&workspace)) != DD_OK) return rc;
    }
    rc = check_workspace(workspace, workspace_bytes, need);
    if (rc != DD_OK) return rc;
    const bool kl = (mode == DD_KL_THRESH || mode == DD_KL_PROB || mode == DD_KL_TOPK);
    const hipError_t e = dd::launch_verify(kl ? logits_d : nullptr, logits_v, mask, mode, threshold, seed,
                                           out_mask, out_tokens, out_scores, B, G, V, logit_dtype == DD_BF16,
                                           workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

extern "C" {

int dd_verify_remask(const void *logits_d, const void *logits_v, const uint8_t *mask,
                     dd_mode mode, float threshold, uint64_t seed,
                     uint8_t *out_mask, int32_t *out_tokens, float *out_scores,
                     int B, int G, int V, dd_dtype logit_dtype,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    return verify_remask(logits_d, logits_v, mask, (int)mode, threshold, seed, out_mask, out_tokens, out_scores, B, G, V,
                         (int)logit_dtype, workspace, workspace_bytes, stream, false);
}

int dd_verify_remask_static(const void *logits_d, const void *logits_v, const uint8_t *mask,
                            dd_mode mode, float threshold, uint64_t seed,
                            uint8_t *out_mask, int32_t *out_tokens, float *out_scores,
                            int B, int G, int V, dd_dtype logit_dtype, void *stream)
{
    // every partial state the finishing kernel reads is written by the streaming kernel of the same call:
    // nothing in the static array has to be cleared between calls
    return verify_remask(logits_d, logits_v, mask, (int)mode, threshold, seed, out_mask, out_tokens, out_scores, B, G, V,
                         (int)logit_dtype, nullptr, 0, stream, true);
}

size_t dd_unmask_workspace_bytes(int B, int G, int V, dd_dtype logit_dtype)
{
    return dd_verify_remask_workspace_bytes(B, G, V, logit_dtype);
}

int dd_unmask(const void *logits_d, const uint8_t *mask, dd_unmask_mode mode, float threshold,
              int32_t *x_tokens, uint8_t *out_mask, int32_t *out_tokens, float *out_conf,
              int B, int G, int V, dd_dtype logit_dtype,
              void *workspace, size_t workspace_bytes, void *stream)
{
    if (mode != DD_UNMASK_THRESH && mode != DD_UNMASK_TOPK) return DD_ERR_MODE;
    if (mode == DD_UNMASK_TOPK && !(threshold >= 0.0f && threshold <= 3.0e38f)) return DD_ERR_SHAPE;
    if (logit_dtype != DD_F32 && logit_dtype != DD_BF16) return DD_ERR_DTYPE;
    if (B < 0 || G < 0 || V < 1) return DD_ERR_SHAPE;
    if ((double)B * G >= 2147483648.0) return DD_ERR_SHAPE;
    const int eb = logit_dtype == DD_BF16 ? 2 : 4;
    if (((long)V * eb) % 16 != 0) return DD_ERR_ALIGN;
    if (B == 0 || G == 0) return DD_OK;
    if (!logits_d || !mask || !out_mask || !out_tokens || !out_conf) return DD_ERR_NULL;
    {
        // the selection reads every mask byte of a sequence while other lanes write out_mask
        const uintptr_t m0 = reinterpret_cast<uintptr_t>(mask), o0 = reinterpret_cast<uintptr_t>(out_mask);
        const uintptr_t n = (uintptr_t)B * (uintptr_t)G;
        if (m0 < o0 + n && o0 < m0 + n) return DD_ERR_SHAPE;
    }
    if (misaligned16(logits_d)) return DD_ERR_ALIGN;
    const int rc = check_workspace(workspace, workspace_bytes, dd::verify_workspace_bytes(B * G, V, eb));
    if (rc != DD_OK) return rc;
    const hipError_t e = dd::launch_verify(nullptr, logits_d, mask,
                                           mode == DD_UNMASK_TOPK ? dd::kModeUnmaskTopk : dd::kModeUnmaskThresh,
                                           threshold, 0, out_mask, out_tokens, out_conf, B, G, V,
                                           logit_dtype == DD_BF16, workspace, static_cast<hipStream_t>(stream), x_tokens);
    return e == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

size_t dd_verify_scores_workspace_bytes(int P, int V, dd_dtype logit_dtype)
{
    return dd_verify_remask_workspace_bytes(1, P, V, logit_dtype);
}

int dd_verify_scores(const void *logits_d, const void *logits_v,
                     float *out_kl, float *out_conf_v, int32_t *out_tok_v, float *out_conf_d, int32_t *out_tok_d,
                     int P, int V, dd_dtype logit_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    if (logit_dtype != DD_F32 && logit_dtype != DD_BF16) return DD_ERR_DTYPE;
    if (P < 0 || V < 1) return DD_ERR_SHAPE;
    const int eb = logit_dtype == DD_BF16 ? 2 : 4;
    if (((long)V * eb) % 16 != 0) return DD_ERR_ALIGN;
    if (P == 0) return DD_OK;
    if (!logits_d || !logits_v || !out_kl || !out_conf_v || !out_tok_v) return DD_ERR_NULL;
    if (misaligned16(logits_v) || misaligned16(logits_d)) return DD_ERR_ALIGN;
    const int rc = check_workspace(workspace, workspace_bytes, dd::verify_workspace_bytes(P, V, eb));
    if (rc != DD_OK) return rc;
    dd::VerifyExtra ex;
    ex.conf_v = out_conf_v;
    ex.conf_d = out_conf_d;
    ex.tok_d = out_tok_d;
    const hipError_t e = dd::launch_verify(logits_d, logits_v, nullptr, dd::kModeScores, 0.0f, 0, nullptr, out_tok_v,
                                           out_kl, 1, P, V, logit_dtype == DD_BF16, workspace,
                                           static_cast<hipStream_t>(stream), nullptr, &ex);
    return e == hipSuccess ? DD_OK : DD_ERR_LAUNCH;
}

}  // extern "C"
