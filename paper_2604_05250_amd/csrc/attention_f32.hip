// fp32 attention, softmax(Q K^T / sqrt(d_k)) V (Eq. 3) over all key positions (Sec. 2.2),
// computed in fp32 throughout on the vector ALUs.  It serves fp32 inputs (the small
// CPU-checkable configuration) for both the verifier's full attention and the drafter's
// block attention over the cached K/V (Sec. 2.3); the bf16 / fp8 workloads run on the
// matrix cores in attention_mfma.hip.
//
// d/32 adjacent lanes share one query row, each owning 32 of its dims.  A tile of 32 keys
// (K and V rows, fp32) is staged in LDS; K rows are read as wave-wide broadcasts.
#include "attention_common.h"
#include "dd_internal.h"

namespace dd {
namespace {

constexpr int TKF = 32;   // keys per LDS tile

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D>
__global__ __launch_bounds__(kAttnThreads) void attn_f32_kernel(const AttnKernelArgs a)
{
    constexpr int LPQ = D / 32;                 // lanes per query row
    constexpr int ROWS = kAttnThreads / LPQ;    // query rows per workgroup
    constexpr int CH = D / 4;                   // float4 chunks per row
    __shared__ float4 Ks[TKF * CH];
    __shared__ float4 Vs[TKF * CH];

    const int tid = threadIdx.x;
    int bid = blockIdx.x;
    const int sp = bid % a.splits; bid /= a.splits;
    const int rt = bid % a.row_tiles; bid /= a.row_tiles;
    const int kvh = bid % a.Hkv;
    const int b = bid / a.Hkv;
    const int rows_total = a.group * a.Nq;
    const int v = rt * ROWS + tid / LPQ;
    const int sub = tid % LPQ;
    const bool row_ok = v < rows_total;
    const int vv = row_ok ? v : rows_total - 1;
    const int head = kvh * a.group + vv / a.Nq;
    const int qi = vv % a.Nq;
    const size_t orow = ((size_t)b * a.H + head) * (size_t)a.Nq + qi;

    float q[32], o[32];
    {
        const float4 *qp = reinterpret_cast<const float4 *>(static_cast<const float *>(a.Q) + orow * D + sub * 32);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float4 w = qp[i];
            q[4 * i] = w.x; q[4 * i + 1] = w.y; q[4 * i + 2] = w.z; q[4 * i + 3] = w.w;
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) o[i] = 0.f;
    }
    float c = a.scale_log2;
    if (a.q_scale) c *= a.q_scale[b * a.H + head];
    if (a.k_scale) c *= a.k_scale[b * a.Hkv + kvh];

    const int k_begin = sp * a.keys_per_split;
    const int k_end = min(a.N, k_begin + a.keys_per_split);
    const size_t kv_head = (size_t)b * a.Hkv + kvh;
    const int bstart = a.block_starts ? a.block_starts[b] : a.block_start;   // any value is safe: rows are chosen by range test
    float m_run = -INFINITY, l_run = 0.f;

    for (int k0 = k_begin; k0 < k_end; k0 += TKF) {
        __syncthreads();
        for (int id = tid; id < TKF * CH; id += kAttnThreads) {
            const int row = id / CH, ch = id % CH;
            const int j = k0 + row;
            float4 kw = make_float4(0.f, 0.f, 0.f, 0.f), vw = kw;
            if (j < k_end) {
                const bool in_blk = a.Kblk != nullptr && (unsigned)j - (unsigned)bstart < (unsigned)a.block_len;
                const size_t off = in_blk ? (kv_head * a.block_len + (size_t)(j - bstart)) * D
                                          : (kv_head * a.kv_stride + (size_t)j) * D;
                const float *kp = static_cast<const float *>(in_blk ? a.Kblk : a.K) + off;
                const float *vp = static_cast<const float *>(in_blk ? a.Vblk : a.V) + off;
                kw = reinterpret_cast<const float4 *>(kp)[ch];
                vw = reinterpret_cast<const float4 *>(vp)[ch];
            }
            Ks[id] = kw;
            Vs[id] = vw;
        }
        __syncthreads();

        float s[TKF];
        float tmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < TKF; ++j) {
            float dot = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float4 kw = Ks[j * CH + sub * 8 + i];
                dot = fmaf(q[4 * i], kw.x, dot);
                dot = fmaf(q[4 * i + 1], kw.y, dot);
                dot = fmaf(q[4 * i + 2], kw.z, dot);
                dot = fmaf(q[4 * i + 3], kw.w, dot);
            }
#pragma unroll
            for (int w = 1; w < LPQ; w <<= 1) dot += __shfl_xor(dot, w);
            if (k0 + j >= k_end) dot = -INFINITY;
            s[j] = dot;
            tmax = fmaxf(tmax, dot);
        }
        const float m_new = fmaxf(m_run, tmax);
        const float corr = fast_exp2((m_run - m_new) * c);
        m_run = m_new;
        const float mc = m_new * c;
#pragma unroll
        for (int i = 0; i < 32; ++i) o[i] *= corr;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < TKF; ++j) {
            const float p = fast_exp2(fmaf(s[j], c, -mc));
            psum += p;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float4 vw = Vs[j * CH + sub * 8 + i];
                o[4 * i] = fmaf(p, vw.x, o[4 * i]);
                o[4 * i + 1] = fmaf(p, vw.y, o[4 * i + 1]);
                o[4 * i + 2] = fmaf(p, vw.z, o[4 * i + 2]);
                o[4 * i + 3] = fmaf(p, vw.w, o[4 * i + 3]);
            }
        }
        l_run = l_run * corr + psum;
    }

    if (!row_ok) return;
    if (a.splits == 1) {
        const float inv = 1.0f / l_run;
        float4 *op = reinterpret_cast<float4 *>(static_cast<float *>(a.O) + orow * D + sub * 32);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            op[i] = make_float4(o[4 * i] * inv, o[4 * i + 1] * inv, o[4 * i + 2] * inv, o[4 * i + 3] * inv);
    } else {
        float4 *op = reinterpret_cast<float4 *>(a.part_o + (orow * a.splits + sp) * D + sub * 32);
#pragma unroll
        for (int i = 0; i < 8; ++i) op[i] = make_float4(o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]);
        if (sub == 0) {
            float *ml = a.part_ml + (orow * a.splits + sp) * 2;
            ml[0] = m_run * c;
            ml[1] = l_run;
        }
    }
}

}  // namespace

hipError_t launch_attention_f32(const AttnArgs &a, hipStream_t stream)
{
    AttnKernelArgs k;
    const int rows_per_wg = kAttnThreads / (a.d / 32);
    fill_kernel_args(a, k, rows_per_wg, TKF);
    const long blocks = (long)a.B * a.Hkv * k.row_tiles * k.splits;
    const dim3 grid((unsigned)blocks), block(kAttnThreads);
    const hipError_t e = a.d == 128 ? launch(attn_f32_kernel<128>, grid, block, stream, k)
                                    : launch(attn_f32_kernel<64>, grid, block, stream, k);
    return e != hipSuccess ? e : finish_attention(a, k.splits, stream);
}

}  // namespace dd
