// Matrix-core attention for bf16 (and fp8-e4m3 Q/K) inputs on gfx950:
//     O = softmax(Q K^T / sqrt(d_k)) V            (Eq. 3, over all key positions: Sec. 2.2)
// used by the verifier's full attention and, with a split key range, by the drafter's
// block attention over the cached K/V (Sec. 2.3).
//
// Layout of the computation (one wave = 32 query rows, one workgroup = 4 waves):
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K tile (from LDS), B = Q (registers).
//                 The 32x32 result puts one QUERY per lane column and 16 KEYS in the lane's
//                 registers, so the softmax row reductions are in-register plus one
//                 exchange between the two lane halves.
//   O^T += V^T P^T  A = V^T (LDS, keys contiguous), B = P^T.  The accumulator layout of
//                 S^T is exactly the B-operand layout of this product once the keys of a
//                 16-key step are taken in the order the accumulator holds them, so the
//                 probabilities never leave registers; V is transposed once per tile while
//                 it is staged into LDS, in that same key order.
//   The rescale factor of the online softmax is per query = per lane: a plain multiply.
// K/V tiles are prefetched into registers while the previous tile is being multiplied, and
// both LDS tiles are XOR-swizzled at 16-byte granularity so that the 16-byte operand reads
// and the staging writes are bank-conflict free without padding.
#include "attention_common.h"
#include "dd_internal.h"

namespace dd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int TK = 64;            // keys per LDS tile
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerWG = 128;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ unsigned pack_bf16_trunc(float lo, float hi)
{
    // exact when the inputs are representable in bf16 (decoded fp8 values are)
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
}

__device__ __forceinline__ unsigned pack_bf16_rne(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    floatx2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(unsigned, b);
}

// eight OCP e4m3 codes -> eight bf16 (exact)
__device__ __forceinline__ uint4 fp8x8_to_bf16x8(uint2 w)
{
    const floatx2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, false);
    const floatx2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, true);
    const floatx2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, false);
    const floatx2 d = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, true);
    return make_uint4(pack_bf16_trunc(a.x, a.y), pack_bf16_trunc(b.x, b.y),
                      pack_bf16_trunc(c.x, c.y), pack_bf16_trunc(d.x, d.y));
}

template <int D, bool FP8>
__global__ __launch_bounds__(kAttnThreads, 2) void attn_mfma_kernel(const AttnKernelArgs a)
{
    constexpr int CH = D / 8;                        // 16-byte chunks (8 bf16) per K row
    constexpr int KCH = TK * CH / kAttnThreads;      // K chunks staged per thread
    constexpr int VTASKS = (TK / 8) * CH * 2;        // V transpose tasks per tile (4 keys x 8 dims)
    constexpr int KS = D / 16;                       // MFMA k-steps over the head dim
    constexpr int DC = D / 32;                       // 32-wide chunks of the head dim
    static_assert(KCH >= 1 && VTASKS <= kAttnThreads, "tile does not fit the staging scheme");

    __shared__ uint4 Ks[TK * CH];                    // [key][chunk ^ (key & 7)]
    __shared__ uint4 Vt[D * (TK / 8)];               // [dim][keygroup ^ swz(dim)], 8 keys per 16 bytes

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;

    int bid = blockIdx.x;
    const int sp = bid % a.splits; bid /= a.splits;
    const int rt = bid % a.row_tiles; bid /= a.row_tiles;
    const int kvh = bid % a.Hkv;
    const int b = bid / a.Hkv;
    const int rows_total = a.group * a.Nq;
    const int v = rt * kRowsPerWG + wave * kRowsPerWave + l32;
    const bool row_ok = v < rows_total;
    const int vv = row_ok ? v : rows_total - 1;
    const int head = kvh * a.group + vv / a.Nq;
    const int qi = vv % a.Nq;
    const bool wave_active = rt * kRowsPerWG + wave * kRowsPerWave < rows_total;
    const size_t orow = ((size_t)b * a.H + head) * (size_t)a.Nq + qi;

    // ---- Q fragments (B operand of S^T = K Q^T): lane (query l32, half hh) holds dims 16*ks + 8*hh .. +7
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const size_t off = orow * D + ks * 16 + hh * 8;
        uint4 w;
        if (FP8) w = fp8x8_to_bf16x8(*reinterpret_cast<const uint2 *>(static_cast<const uint8_t *>(a.Q) + off));
        else w = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.Q) + off);
        qf[ks] = __builtin_bit_cast(bf16x8, w);
    }
    float c = a.scale_log2;
    if (a.q_scale) c *= a.q_scale[b * a.H + head];
    if (a.k_scale) c *= a.k_scale[b * a.Hkv + kvh];

    const int k_begin = sp * a.keys_per_split;
    const int k_end = min(a.N, k_begin + a.keys_per_split);
    const int ntiles = (k_end - k_begin + TK - 1) / TK;
    const size_t kv_head = (size_t)b * a.Hkv + kvh;

    // ---- staging: global -> registers -> LDS
    uint4 kreg[KCH];
    uint4 vreg[4];
    const int vt_dchunk = tid % CH, vt_e4 = (tid / CH) & 1, vt_g = tid / (2 * CH);   // V task of this thread
    // keys of task (g, e4): tile-local index (g/4)*32 + ((g/2)&1)*16 + 8*e4 + 4*(g&1) + e,  e = 0..3
    const int vt_key0 = (vt_g >> 2) * 32 + ((vt_g >> 1) & 1) * 16 + 8 * vt_e4 + 4 * (vt_g & 1);

    auto src_row = [&](int j, const void *cache, const void *blk, int elem_bytes) -> const uint8_t * {
        // row j of the key/value sequence: the fresh block tensor inside the active block, else the cache
        if (blk != nullptr && j >= a.block_start && j < a.block_start + a.block_len)
            return static_cast<const uint8_t *>(blk) +
                   ((kv_head * a.block_len + (size_t)(j - a.block_start)) * D) * elem_bytes;
        return static_cast<const uint8_t *>(cache) + ((kv_head * a.N + (size_t)j) * D) * elem_bytes;
    };
    auto load_tile = [&](int t) {
        const int k0 = k_begin + t * TK;
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int id = tid + i * kAttnThreads;
            const int row = id / CH, ch = id % CH;
            const int j = k0 + row;
            uint4 w = make_uint4(0, 0, 0, 0);
            if (j < k_end) {
                if (FP8) {
                    const uint2 r = *reinterpret_cast<const uint2 *>(src_row(j, a.K, a.Kblk, 1) + ch * 8);
                    w = make_uint4(r.x, r.y, 0, 0);
                } else {
                    w = *reinterpret_cast<const uint4 *>(src_row(j, a.K, a.Kblk, 2) + ch * 16);
                }
            }
            kreg[i] = w;
        }
        if (tid < VTASKS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = k0 + vt_key0 + e;
                uint4 w = make_uint4(0, 0, 0, 0);
                if (j < k_end) w = *reinterpret_cast<const uint4 *>(src_row(j, a.V, a.Vblk, 2) + vt_dchunk * 16);
                vreg[e] = w;
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int id = tid + i * kAttnThreads;
            const int row = id / CH, ch = id % CH;
            uint4 w = kreg[i];
            if (FP8) w = fp8x8_to_bf16x8(make_uint2(w.x, w.y));
            Ks[row * CH + (ch ^ (row & 7))] = w;
        }
        if (tid < VTASKS) {
            // 4 keys x 8 dims -> 8 dims x 4 keys
            const unsigned r0[4] = {vreg[0].x, vreg[0].y, vreg[0].z, vreg[0].w};
            const unsigned r1[4] = {vreg[1].x, vreg[1].y, vreg[1].z, vreg[1].w};
            const unsigned r2[4] = {vreg[2].x, vreg[2].y, vreg[2].z, vreg[2].w};
            const unsigned r3[4] = {vreg[3].x, vreg[3].y, vreg[3].z, vreg[3].w};
            uint2 *vt2 = reinterpret_cast<uint2 *>(Vt);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                // dims 2p (low halves) and 2p+1 (high halves)
                const uint2 even = make_uint2((r0[p] & 0xFFFFu) | (r1[p] << 16), (r2[p] & 0xFFFFu) | (r3[p] << 16));
                const uint2 odd = make_uint2((r0[p] >> 16) | (r1[p] & 0xFFFF0000u), (r2[p] >> 16) | (r3[p] & 0xFFFF0000u));
                const int d0 = vt_dchunk * 8 + 2 * p, d1 = d0 + 1;
                vt2[(d0 * (TK / 8) + (vt_g ^ ((d0 ^ (d0 >> 3)) & 7))) * 2 + vt_e4] = even;
                vt2[(d1 * (TK / 8) + (vt_g ^ ((d1 ^ (d1 >> 3)) & 7))) * 2 + vt_e4] = odd;
            }
        }
    };

    // ---- online softmax state: per lane = per (query, lane half)
    floatx16 acc[DC];
#pragma unroll
    for (int i = 0; i < DC; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    float m_run = -INFINITY;     // running max of raw scores (same in both lane halves)
    float l_run = 0.f;           // this lane half's share of the running sum

    load_tile(0);
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
        store_tile();
        __syncthreads();
        if (t + 1 < ntiles) load_tile(t + 1);
        if (!wave_active) continue;

        // S^T tiles: two 32-key x 32-query blocks
        floatx16 s[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
            const int krow = sub * 32 + l32;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint4 w = Ks[krow * CH + ((2 * ks + hh) ^ (krow & 7))];
                s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), qf[ks], s[sub], 0, 0, 0);
            }
        }
        // keys past the end of the range score -inf (only the last tile can be ragged)
        const int k0 = k_begin + t * TK;
        if (k0 + TK > k_end) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kk = sub * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (k0 + kk >= k_end) s[sub][r] = -INFINITY;
                }
        }
        float tmax = s[0][0];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[sub][r]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        const float corr = fast_exp2((m_run - m_new) * c);   // first tile: exp2(-inf) = 0
        m_run = m_new;
        const float mc = m_new * c;
        unsigned pk[2][2][4];     // [sub][16-key step][4 dwords = 8 bf16], already in B-operand order
        float psum = 0.f;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = fast_exp2(fmaf(s[sub][r], c, -mc));
                const float p1 = fast_exp2(fmaf(s[sub][r + 1], c, -mc));
                psum += p0 + p1;
                pk[sub][r >> 3][(r & 7) >> 1] = pack_bf16_rne(p0, p1);
            }
        l_run = l_run * corr + psum;
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] *= corr;

        // O^T += V^T P^T
#pragma unroll
        for (int i = 0; i < DC; ++i) {
            const int drow = i * 32 + l32;
            const int swz = (drow ^ (drow >> 3)) & 7;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const int g = sub * 4 + st * 2 + hh;
                    const uint4 w = Vt[drow * (TK / 8) + (g ^ swz)];
                    const uint4 pw = make_uint4(pk[sub][st][0], pk[sub][st][1], pk[sub][st][2], pk[sub][st][3]);
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w),
                                                                     __builtin_bit_cast(bf16x8, pw), acc[i], 0, 0, 0);
                }
        }
    }

    if (!wave_active) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!row_ok) return;
    // accumulator register r of chunk i holds dim 32*i + 8*(r/4) + 4*hh + (r%4) of this lane's query
    if (a.splits == 1) {
        const float inv = 1.0f / l_tot;
        uint16_t *o = static_cast<uint16_t *>(a.O) + orow * D;
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const uint2 w = make_uint2(pack_bf16_rne(acc[i][4 * q4] * inv, acc[i][4 * q4 + 1] * inv),
                                           pack_bf16_rne(acc[i][4 * q4 + 2] * inv, acc[i][4 * q4 + 3] * inv));
                *reinterpret_cast<uint2 *>(o + i * 32 + q4 * 8 + hh * 4) = w;
            }
    } else {
        float *po = a.part_o + (orow * a.splits + sp) * D;
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<float4 *>(po + i * 32 + q4 * 8 + hh * 4) =
                    make_float4(acc[i][4 * q4], acc[i][4 * q4 + 1], acc[i][4 * q4 + 2], acc[i][4 * q4 + 3]);
        if (hh == 0) {
            float *ml = a.part_ml + (orow * a.splits + sp) * 2;
            ml[0] = m_run * c;
            ml[1] = l_tot;
        }
    }
}

// Merge the per-split partial states of each query row: O = sum_s 2^{m_s-M} O_s / sum_s 2^{m_s-M} l_s.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml, void *__restrict__ O,
                                                           long rows, int splits, int d)
{
    const int per_row = d / 4;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long row = gid / per_row;
    const int c4 = (int)(gid % per_row);
    if (row >= rows) return;
    const float *ml = part_ml + row * splits * 2;
    float M = -INFINITY;
    for (int s = 0; s < splits; ++s) M = fmaxf(M, ml[2 * s]);
    float L = 0.f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < splits; ++s) {
        const float w = fast_exp2(ml[2 * s] - M);
        L += w * ml[2 * s + 1];
        const float4 p = *reinterpret_cast<const float4 *>(part_o + (row * splits + s) * d + c4 * 4);
        o.x += w * p.x; o.y += w * p.y; o.z += w * p.z; o.w += w * p.w;
    }
    const float inv = 1.0f / L;
    if (OUT_BF16) {
        const uint2 w = make_uint2(pack_bf16_rne(o.x * inv, o.y * inv), pack_bf16_rne(o.z * inv, o.w * inv));
        *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(O) + row * d + c4 * 4) = w;
    } else {
        *reinterpret_cast<float4 *>(static_cast<float *>(O) + row * d + c4 * 4) =
            make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
    }
}

}  // namespace

void fill_kernel_args(const AttnArgs &a, AttnKernelArgs &k, int rows_per_wg, int key_tile)
{
    k.Q = a.Q; k.K = a.K; k.V = a.V; k.Kblk = a.Kblk; k.Vblk = a.Vblk; k.O = a.O;
    k.q_scale = a.q_scale; k.k_scale = a.k_scale;
    k.B = a.B; k.H = a.H; k.Hkv = a.Hkv; k.Nq = a.Nq; k.N = a.N;
    k.group = a.H / a.Hkv;
    k.row_tiles = (k.group * a.Nq + rows_per_wg - 1) / rows_per_wg;
    k.splits = a.splits;
    int per = (a.N + a.splits - 1) / a.splits;
    per = (per + key_tile - 1) / key_tile * key_tile;
    k.keys_per_split = per;
    // drop trailing splits that would be empty after rounding the split length up to whole tiles
    k.splits = (a.N + per - 1) / per;
    k.block_start = a.block_start; k.block_len = a.block_len;
    k.scale_log2 = 1.44269504088896340736f / sqrtf((float)a.d);
    const size_t rows = (size_t)a.B * a.H * a.Nq;
    k.part_o = static_cast<float *>(a.workspace);
    k.part_ml = k.part_o ? k.part_o + rows * (size_t)k.splits * a.d : nullptr;
}

hipError_t launch_attention_mfma(const AttnArgs &a, hipStream_t stream)
{
    AttnKernelArgs k;
    fill_kernel_args(a, k, kRowsPerWG, TK);
    const long blocks = (long)a.B * a.Hkv * k.row_tiles * k.splits;
    const dim3 grid((unsigned)blocks), block(kAttnThreads);
    const bool fp8 = a.qk_dtype == 2;
    hipError_t e;
    if (a.d == 128) {
        if (fp8) e = launch(attn_mfma_kernel<128, true>, grid, block, stream, k);
        else     e = launch(attn_mfma_kernel<128, false>, grid, block, stream, k);
    } else {
        if (fp8) e = launch(attn_mfma_kernel<64, true>, grid, block, stream, k);
        else     e = launch(attn_mfma_kernel<64, false>, grid, block, stream, k);
    }
    if (e != hipSuccess || k.splits == 1) return e;
    AttnArgs c = a;
    c.splits = k.splits;
    return launch_attention_combine(c, stream);
}

hipError_t launch_attention_combine(const AttnArgs &a, hipStream_t stream)
{
    const long rows = (long)a.B * a.H * a.Nq;
    const float *po = static_cast<const float *>(a.workspace);
    const float *pml = po + (size_t)rows * a.splits * a.d;
    const long threads = rows * (a.d / 4);
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (a.v_dtype == 1)
        return launch(attn_combine_kernel<true>, grid, block, stream, po, pml, a.O, rows, a.splits, a.d);
    return launch(attn_combine_kernel<false>, grid, block, stream, po, pml, a.O, rows, a.splits, a.d);
}

}  // namespace dd
