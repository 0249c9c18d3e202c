// Drafter attention over the cached K/V (Sec. 2.3), streaming form (bf16):
//     O = softmax(Q_blk K^T / sqrt(d_k)) V     for the block_len queries of the active block (Eq. 3),
// key/value row j coming from the block tensors inside the block and from the cache elsewhere.
//
// With a few dozen query rows per head this call is bound by reading K and V once, so the kernel is
// built around the memory pipeline, not the matrix cores:
//   - K/V tiles of 64 keys go from global memory straight into LDS (global_load_lds_dwordx4, no
//     staging registers) through a ring of four tile buffers: three tiles (96 KB per compute unit) are
//     always in flight while a fourth is consumed.  The barrier that opens a tile only waits until the
//     two newest tiles are the only loads outstanding (memory operations complete in order).  The
//     compiler would wait for every outstanding LDS load before any read of such a buffer, so the
//     operand reads of the tiles are written as inline assembly with their own wait;
//   - one workgroup = 4 waves (one per SIMD) owns up to 64 query rows of one (batch, kv head): wave w holds
//     the 32-row block w % 2 and takes unit w / 2 of every tile (two key phases), so all four waves work on
//     every tile; the two phases of a row block merge their (max, sum, O) states through LDS at the end.
//     Calls with more than 64 rows per kv head stay with the MFMA kernel of attention_mfma.hip;
//   - per unit a wave simply runs S = K Q^T, the online softmax and O += V P back to back.
// K is XOR-swizzled for its 16-byte operand reads; V stays row-major (swizzled in 64-byte granules) and
// its transposed operand comes from ds_read_b64_tr_b16.
// The key range can also be split over workgroups; their partial states go to the workspace and are
// merged by the combine kernel of attention_mfma.hip.
#include "attention_common.h"
#include "dd_internal.h"

#include <type_traits>

namespace dd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

constexpr int TKS = 64;                 // keys per tile
constexpr int kRing = 4;                // tile buffers
constexpr int QBS = 1;                  // 32-row query blocks per wave
constexpr int kRowsWaveS = 32 * QBS;
constexpr float kSlackS = 8.0f;         // the maximum in use is raised when exceeded by 2^8

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ unsigned pack2_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}
__device__ __forceinline__ float swap_max(float x)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float swap_sum(float x)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}

template <int D>
__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_stream_kernel(const AttnKernelArgs a)
{
    constexpr int CH = D / 8;                        // 16-byte chunks (8 bf16) per row
    constexpr int KS = D / 16;                       // MFMA k-steps over the head dim
    constexpr int DC = D / 32;                       // 32-wide chunks of the head dim
    constexpr int ROWB = D * 2;                      // bytes per K / V row
    constexpr int DMA_ROWS = 1024 / ROWB;            // rows moved by one wave-wide 16-byte-per-lane load
    constexpr int NDMA = TKS / DMA_ROWS / 4;         // such loads per wave per K or V tile
    static_assert((4 * DMA_ROWS) % 8 == 0, "swizzle phase must not depend on the load index");

    constexpr int TILEB = TKS * ROWB;                // bytes of one K or V tile
    static_assert(QBS * DC * 16 * 64 * 4 <= 2 * TILEB, "a wave's O state must fit a quarter of the ring");
    __shared__ __attribute__((aligned(1024))) uint4 KV[2 * kRing * TKS * CH];   // K ring [key][chunk ^ (key & 7)], then
                                                     // V ring [key][chunk ^ ((key % (CH/4)) << 2)]
    __shared__ float ml_sh[4][2][64];                // per wave: (max, sum) of its query block, for the phase merge

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;
    const int rg = wave & 1, ph = wave >> 1;         // row block, key phase

    // ---- which (batch, kv head, row tile, key split); same XCD for workgroups that share K/V
    int bid = blockIdx.x;
    {
        const int total = gridDim.x, per = total >> 3, rem = total & 7;
        const int xcd = bid & 7, slot = bid >> 3;
        bid = xcd * per + min(xcd, rem) + slot;
    }
    const int sp = bid % a.splits; bid /= a.splits;
    const int rt = bid % a.row_tiles; bid /= a.row_tiles;
    const int kvh = bid % a.Hkv;
    const int b = bid / a.Hkv;
    const int rows_total = a.group * a.Nq;           // query rows of this (batch, kv head): contiguous in memory
    const int v_first = rt * a.rows_per_wg + rg * kRowsWaveS;   // rows_per_wg = 64
    const bool wave_active = v_first < rows_total;
    const size_t row_base = ((size_t)b * a.H + (size_t)kvh * a.group) * a.Nq;
    const int kbeg = sp * a.keys_per_split;
    const int kend = min(a.N, kbeg + a.keys_per_split);
    const int bstart = a.block_starts ? a.block_starts[b] : a.block_start;   // any value is safe: rows are chosen by range test
    const int ntiles = (kend - kbeg + TKS - 1) / TKS;

    // ---- staging by LDS DMA: load i of this wave moves rows (4i + wave) * DMA_ROWS .. of a tile; lane l
    // lands at chunk position l % CH of row l / CH and therefore fetches the chunk the swizzle maps there.
    const int dma_row = lane / CH, dma_pos = lane % CH;
    const int dma_row0 = wave * DMA_ROWS + dma_row;
    const unsigned dma_koff = (dma_pos ^ (dma_row0 & 7)) * 16;
    const unsigned dma_voff = (dma_pos ^ ((dma_row0 & (CH / 4 - 1)) << 2)) * 16;
    const size_t kv_head = (size_t)b * a.Hkv + kvh;
    const uint8_t *const kc = static_cast<const uint8_t *>(a.K) + kv_head * a.kv_stride * (size_t)ROWB;
    const uint8_t *const vc = static_cast<const uint8_t *>(a.V) + kv_head * a.kv_stride * (size_t)ROWB;
    const uint8_t *const kb_ = a.block_len ? static_cast<const uint8_t *>(a.Kblk) + kv_head * a.block_len * (size_t)ROWB : nullptr;
    const uint8_t *const vb_ = a.block_len ? static_cast<const uint8_t *>(a.Vblk) + kv_head * a.block_len * (size_t)ROWB : nullptr;
    // rows of the last tile at or past the end of the key range repeat its last row (finite stand-ins, masked later)
    auto dma_tile = [&](int tile) __attribute__((always_inline)) {
        uint4 *kd = KV + (tile % kRing) * (TKS * CH), *vd = KV + (kRing + tile % kRing) * (TKS * CH);
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            const int r0 = (i * 4 + wave) * DMA_ROWS;
            const int j = min(kbeg + tile * TKS + i * 4 * DMA_ROWS + dma_row0, kend - 1);
            const bool in_blk = (unsigned)j - (unsigned)bstart < (unsigned)a.block_len;
            const size_t roff = (size_t)(in_blk ? j - bstart : j) * ROWB;
            const uint8_t *ks = (in_blk ? kb_ : kc) + roff + dma_koff;
            const uint8_t *vs = (in_blk ? vb_ : vc) + roff + dma_voff;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)ks,
                                             (__attribute__((address_space(3))) void *)(kd + r0 * CH), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)vs,
                                             (__attribute__((address_space(3))) void *)(vd + r0 * CH), 16, 0, 0);
        }
    };

    // ---- Q fragments (B operand of S^T = K Q^T): lane (query l32, half hh) holds dims 16 ks + 8 hh .. +7
    bool row_ok[QBS];
    float c[QBS];                                    // scores are exponentiated as 2^(s*c)
    bf16x8 qf[QBS][KS];
#pragma unroll
    for (int q = 0; q < QBS; ++q) {
        const int v = v_first + q * 32 + l32;
        row_ok[q] = v < rows_total;
        const int vv = row_ok[q] ? v : rows_total - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[q][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(
                            static_cast<const uint16_t *>(a.Q) + (row_base + vv) * D + ks * 16 + hh * 8));
        c[q] = a.scale_log2;
        if (a.q_scale) c[q] *= a.q_scale[b * a.H + kvh * a.group + vv / a.Nq];
        if (a.k_scale) c[q] *= a.k_scale[b * a.Hkv + kvh];
    }

    // the first three tiles; the Q loads above are older, so the first partial wait below covers them too
#pragma unroll
    for (int t0 = 0; t0 < kRing - 1; ++t0)
        if (t0 < ntiles) dma_tile(t0);

    floatx16 acc[QBS][DC];                           // O^T, unnormalised
#pragma unroll
    for (int q = 0; q < QBS; ++q)
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[q][i][r] = 0.f;
    float mc[QBS] = {-INFINITY};                     // maximum in use (log2 units), equal in both lane halves
    float l_run[QBS] = {0.f};                        // this lane half's share of the running sums

    // operand addresses inside a tile buffer (bytes), without the unit offset
    int k_off[KS], v_off[DC];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_off[ks] = (l32 * CH + ((2 * ks + hh) ^ (l32 & 7))) * 16;
    {
        const int t = lane & 15, gq = l32 >> 4, row = 4 * hh + (t >> 2);
#pragma unroll
        for (int i = 0; i < DC; ++i) {
            const int chunk = 4 * i + 2 * gq + ((t & 3) >> 1);
            v_off[i] = (row * CH + (chunk ^ ((row & (CH / 4 - 1)) << 2))) * 16 + (t & 1) * 8;
        }
    }

    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void *)KV;   // LDS byte address of the ring
    // One 32-key unit: S = K Q^T, online softmax, O += V P.  kaddr / vaddr = LDS byte addresses of the
    // unit's first K / V row, key0 = global index of its first key.
    auto unit = [&](unsigned kaddr, unsigned vaddr, int key0) __attribute__((always_inline)) {
        // ---- all K fragments of the unit (keys l32, dims 16 ks + 8 hh .. +7) in one go, with their wait
        uint4 kf[KS];
        if constexpr (KS == 8) {
            asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
                         "ds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\tds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(kf[0]), "=&v"(kf[1]), "=&v"(kf[2]), "=&v"(kf[3]), "=&v"(kf[4]), "=&v"(kf[5]), "=&v"(kf[6]), "=&v"(kf[7])
                         : "v"(kaddr + k_off[0]), "v"(kaddr + k_off[1]), "v"(kaddr + k_off[2]), "v"(kaddr + k_off[3]),
                           "v"(kaddr + k_off[4]), "v"(kaddr + k_off[5]), "v"(kaddr + k_off[6]), "v"(kaddr + k_off[7])
                         : "memory");
        } else {
            asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(kf[0]), "=&v"(kf[1]), "=&v"(kf[2]), "=&v"(kf[3])
                         : "v"(kaddr + k_off[0]), "v"(kaddr + k_off[1]), "v"(kaddr + k_off[2]), "v"(kaddr + k_off[3])
                         : "memory");
        }
        floatx16 s[QBS];
#pragma unroll
        for (int q = 0; q < QBS; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[q][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int q = 0; q < QBS; ++q)
                s[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[ks]), qf[q][ks], s[q], 0, 0, 0);
        // score register r of a block is key key0 + 8 (r / 4) + 4 hh + (r % 4) for query row l32
        if (key0 + 32 > kend) {
#pragma unroll
            for (int q = 0; q < QBS; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (key0 + 8 * (r >> 2) + 4 * hh + (r & 3) >= kend) s[q][r] = -INFINITY;
        }
        float tm[QBS];
        bool need = false;
#pragma unroll
        for (int q = 0; q < QBS; ++q) {
            float t = s[q][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) t = fmaxf(t, s[q][r]);
            tm[q] = swap_max(t) * c[q];
            need = need || (tm[q] > mc[q] + kSlackS);
        }
        if (__any(need)) {                                   // rare after the first units: raise the maxima in use
#pragma unroll
            for (int q = 0; q < QBS; ++q) {
                const float mn = fmaxf(mc[q], tm[q]);
                const float corr = exp2_fast(mc[q] - mn);    // first unit: 2^(-inf) = 0
                mc[q] = mn;
                l_run[q] *= corr;
#pragma unroll
                for (int i = 0; i < DC; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[q][i][r] *= corr;
            }
        }
        unsigned pk[QBS][2][4];                              // P^T as the B operand of O^T += V^T P^T
#pragma unroll
        for (int q = 0; q < QBS; ++q) {
            float lsum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = exp2_fast(fmaf(s[q][r], c[q], -mc[q]));
                const float p1 = exp2_fast(fmaf(s[q][r + 1], c[q], -mc[q]));
                lsum += p0 + p1;
                pk[q][r >> 3][(r & 7) >> 1] = pack2_bf16(p0, p1);
            }
            l_run[q] += lsum;
        }
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            // V^T fragments of 16 keys: dims 32 i + l32, keys 16 st + 4 hh + {0..3, 8..11} of the unit
            uint2 lo[DC], hi[DC];
            const unsigned va = vaddr + 16 * st * ROWB;
            if constexpr (DC == 4) {
                asm volatile("ds_read_b64_tr_b16 %0, %8\n\tds_read_b64_tr_b16 %1, %8 offset:%12\n\t"
                             "ds_read_b64_tr_b16 %2, %9\n\tds_read_b64_tr_b16 %3, %9 offset:%12\n\t"
                             "ds_read_b64_tr_b16 %4, %10\n\tds_read_b64_tr_b16 %5, %10 offset:%12\n\t"
                             "ds_read_b64_tr_b16 %6, %11\n\tds_read_b64_tr_b16 %7, %11 offset:%12\n\t"
                             "s_waitcnt lgkmcnt(0)"
                             : "=&v"(lo[0]), "=&v"(hi[0]), "=&v"(lo[1]), "=&v"(hi[1]), "=&v"(lo[2]), "=&v"(hi[2]), "=&v"(lo[3]), "=&v"(hi[3])
                             : "v"(va + v_off[0]), "v"(va + v_off[1]), "v"(va + v_off[2]), "v"(va + v_off[3]), "n"(8 * ROWB)
                             : "memory");
            } else {
                asm volatile("ds_read_b64_tr_b16 %0, %4\n\tds_read_b64_tr_b16 %1, %4 offset:%6\n\t"
                             "ds_read_b64_tr_b16 %2, %5\n\tds_read_b64_tr_b16 %3, %5 offset:%6\n\t"
                             "s_waitcnt lgkmcnt(0)"
                             : "=&v"(lo[0]), "=&v"(hi[0]), "=&v"(lo[1]), "=&v"(hi[1])
                             : "v"(va + v_off[0]), "v"(va + v_off[1]), "n"(8 * ROWB)
                             : "memory");
            }
#pragma unroll
            for (int i = 0; i < DC; ++i) {
                const uint4 w = make_uint4(lo[i].x, lo[i].y, hi[i].x, hi[i].y);
#pragma unroll
                for (int q = 0; q < QBS; ++q) {
                    const uint4 pw = make_uint4(pk[q][st][0], pk[q][st][1], pk[q][st][2], pk[q][st][3]);
                    acc[q][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, pw),
                                                                        acc[q][i], 0, 0, 0);
                }
            }
        }
    };

    // ---- tiles.  Tile t sits in ring slot t % 4.  Its barrier waits until this wave's loads of the (up to
    // two) newer tiles are the only ones outstanding - i.e. tile t has landed - and tells that every wave is
    // done with tile t-1, whose slot then receives tile t+3.  A wave takes the unit of its key phase.
    for (int t = 0; t < ntiles; ++t) {
        const int newer = ntiles - 1 - t;                    // tiles after t (all requested up to t + 2)
        if (newer >= 2) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * 2 * NDMA) : "memory");
        else if (newer == 1) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * NDMA) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        if (t + kRing - 1 < ntiles) dma_tile(t + kRing - 1);
        if (wave_active) {
            const unsigned slot = (unsigned)(t % kRing);
            const int key0 = kbeg + t * TKS + 32 * ph;
            if (key0 < kend) unit(lds0 + slot * TILEB + ph * 32 * ROWB, lds0 + (kRing + slot) * TILEB + ph * 32 * ROWB, key0);
        }
    }

    float l_tot[QBS];
#pragma unroll
    for (int q = 0; q < QBS; ++q) l_tot[q] = swap_sum(l_run[q]);

    // ---- merge the two key phases of a row block through LDS: phase 1 parks its state in quarter `wave`
    // of the ring (register r of chunk i at [i 16 + r][lane]), phase 0 adds it to its own
    __syncthreads();                                         // all waves are done with the ring; its loads have landed
    float *region = reinterpret_cast<float *>(KV) + wave * (2 * TILEB / 4);
    if (ph != 0 && wave_active) {
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                *reinterpret_cast<float4 *>(region + ((i * 4 + r4) * 64 + lane) * 4) =
                    make_float4(acc[0][i][4 * r4], acc[0][i][4 * r4 + 1], acc[0][i][4 * r4 + 2], acc[0][i][4 * r4 + 3]);
        ml_sh[wave][0][lane] = mc[0];
        ml_sh[wave][1][lane] = l_tot[0];
    }
    __syncthreads();
    if (ph == 0 && wave_active) {
        const int w = wave + 2;
        const float *src = reinterpret_cast<const float *>(KV) + w * (2 * TILEB / 4);
        const float mo = ml_sh[w][0][lane], lo = ml_sh[w][1][lane];
        const float mn = fmaxf(mc[0], mo);
        // a phase that saw no key at all has max -inf and weighs nothing
        const float ws = mc[0] == -INFINITY ? 0.f : exp2_fast(mc[0] - mn);
        const float wo = mo == -INFINITY ? 0.f : exp2_fast(mo - mn);
        l_tot[0] = l_tot[0] * ws + lo * wo;
        mc[0] = mn;
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const float4 o = *reinterpret_cast<const float4 *>(src + ((i * 4 + r4) * 64 + lane) * 4);
                acc[0][i][4 * r4] = acc[0][i][4 * r4] * ws + o.x * wo;
                acc[0][i][4 * r4 + 1] = acc[0][i][4 * r4 + 1] * ws + o.y * wo;
                acc[0][i][4 * r4 + 2] = acc[0][i][4 * r4 + 2] * ws + o.z * wo;
                acc[0][i][4 * r4 + 3] = acc[0][i][4 * r4 + 3] * ws + o.w * wo;
            }
    }
    if (ph != 0 || !wave_active) return;

    // ---- output: O^T register r of chunk i holds dim 32 i + 8 (r / 4) + 4 hh + (r % 4) of query row l32
#pragma unroll
    for (int q = 0; q < QBS; ++q) {
        if (!row_ok[q]) continue;
        const size_t orow = row_base + v_first + q * 32 + l32;
        if (a.splits == 1) {
            const float inv = 1.0f / l_tot[q];
            uint16_t *o = static_cast<uint16_t *>(a.O) + orow * D;
#pragma unroll
            for (int i = 0; i < DC; ++i)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const uint2 w = make_uint2(pack2_bf16(acc[q][i][4 * q4] * inv, acc[q][i][4 * q4 + 1] * inv),
                                               pack2_bf16(acc[q][i][4 * q4 + 2] * inv, acc[q][i][4 * q4 + 3] * inv));
                    *reinterpret_cast<uint2 *>(o + i * 32 + q4 * 8 + hh * 4) = w;
                }
        } else {
            float *po = a.part_o + (orow * a.splits + sp) * D;
#pragma unroll
            for (int i = 0; i < DC; ++i)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<float4 *>(po + i * 32 + q4 * 8 + hh * 4) =
                        make_float4(acc[q][i][4 * q4], acc[q][i][4 * q4 + 1], acc[q][i][4 * q4 + 2], acc[q][i][4 * q4 + 3]);
            if (hh == 0) {
                float *ml = a.part_ml + (orow * a.splits + sp) * 2;
                ml[0] = mc[q];
                ml[1] = l_tot[q];
            }
        }
    }
}

}  // namespace

// The streaming kernel serves calls with at most this many query rows per (batch, kv head).
bool attn_stream_fits(const AttnArgs &a) { return (long)(a.H / a.Hkv) * a.Nq <= 2 * kRowsWaveS; }

hipError_t launch_attention_stream(const AttnArgs &a, hipStream_t stream)
{
    AttnKernelArgs k;
    fill_kernel_args(a, k, 2 * kRowsWaveS, TKS);
    if (a.Kblk == nullptr) k.block_len = 0;                 // no row is taken from the block tensors
    const dim3 grid((unsigned)((long)a.B * a.Hkv * k.row_tiles * k.splits)), block(kAttnThreads);
    const hipError_t e = a.d == 128 ? launch(attn_stream_kernel<128>, grid, block, stream, k)
                                    : launch(attn_stream_kernel<64>, grid, block, stream, k);
    return e != hipSuccess ? e : finish_attention(a, k.splits, stream);
}

}  // namespace dd
