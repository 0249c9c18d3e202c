// Verifier attention, wide-wave form (bf16):  O = softmax(Q K^T / sqrt(d_k)) V over all positions
// (Eq. 3 applied bidirectionally, Sec. 2.2) -- the O(N^2)-per-step cost of a masked diffusion model.
//
// Why a second kernel.  With 32 query rows per wave every matrix-core instruction needs its own 1 KB
// operand fragment from LDS, and the 128 B/clk LDS port can only just feed four SIMDs at the MFMA rate.
// Here one wave owns 64 query rows (two 32-row blocks) and is alone on its SIMD (up to 512 registers);
// one workgroup = 4 waves = 256 query rows of one (batch, kv head).  Every K fragment and every V
// fragment read from LDS feeds two MFMAs (one per block): half the LDS bytes per FLOP.
//
// A single wave per SIMD has no other wave to overlap with, and a wave issues in order: a matrix
// instruction only overlaps with the vector instructions that directly follow it.  Each pipeline step
// (one 32-key unit u) is therefore a fixed sequence of "pieces" = one MFMA + its share of everything else:
//     matrix cores   S(u+1) = K(u+1) Q^T,   O^T += V(u-1)^T P(u-1)^T,   l += 1^T P(u-1)^T (row sums)
//     vector ALUs    row maxima of S(u), then P(u) = 2^(S(u) c - m), packed to bf16
//     memory         LDS fragment reads two MFMAs ahead, one global->LDS tile load per piece
// The maximum in use is raised (accumulators rescaled) in a rare branch at the end of a step.
//
// Register files.  S lives in architectural VGPRs (the vector ALUs cannot read accumulation VGPRs and a
// copy costs as much as two FMAs and does not overlap with the matrix cores); O, the row sums and the Q
// fragments live in accumulation VGPRs, which the matrix cores read directly.  The compiler picks one
// register file for all MFMA results of a function, so the S = K Q^T instructions are written as inline
// assembly.  The hazards the compiler would otherwise pad are kept apart by construction: a score block
// is written by the first half of step u's MFMAs and first read by a vector instruction in step u+1.
//
// Staging.  K and V tiles (64 keys) are double-buffered in four separate LDS arrays and filled by
// global_load_lds_dwordx4 (no registers, no LDS store instructions); the arrays are distinct objects and
// selected statically, so the compiler only waits for those loads at the barrier that ends a stage.
// K is XOR-swizzled for its 16-byte operand reads; V stays row-major (swizzled in 64-byte granules) and
// its transposed operand comes from ds_read_b64_tr_b16 (lane j of a 16-lane group receives column j of
// the 4-row x 16-column block whose row r is addressed by lanes 4r..4r+3).
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
typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr int TKW = 64;                 // keys per tile
constexpr int QB = 2;                   // 32-row query blocks per wave
constexpr int kRowsWave = 32 * QB;
constexpr int kRowsWGWide = 4 * kRowsWave;
constexpr float kSlack = 8.0f;          // the maximum in use is raised when exceeded by 2^8

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ unsigned pack_bf16_rne(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}
__device__ __forceinline__ float half_swap_max(float x)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
// S = K Q^T step with the result in architectural VGPRs and the Q fragment read from accumulation VGPRs.
__device__ __forceinline__ void qk_first(floatx16 &s, const intx4 kf, const intx4 qfrag)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(kf), "a"(qfrag));
}
__device__ __forceinline__ void qk_next(floatx16 &s, const intx4 kf, const intx4 qfrag)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(kf), "a"(qfrag));
}

template <int N> using I_ = std::integral_constant<int, N>;
using T_ = std::true_type;
using F_ = std::false_type;

template <int D>
__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_wide_kernel(const AttnKernelArgs a)
{
    constexpr int CH = D / 8;                        // 16-byte chunks (8 bf16) per row
    constexpr int KS = D / 16;                       // MFMA k-steps over the head dim
    constexpr int DC = D / 32;                       // 32-wide chunks of the head dim
    constexpr int ROWB = D * 2;                      // bytes per K / V row
    constexpr int DMA_ROWS = 1024 / ROWB;            // rows moved by one wave-wide 16-byte-per-lane load
    constexpr int NDMA = TKW / DMA_ROWS / 4;         // such loads per wave per tile
    constexpr int NQK = KS * QB;                     // pieces of a step: S(u+1) ...
    constexpr int NPV = 2 * DC * QB;                 // ... O += V P ...
    constexpr int NP = NQK + NPV + 2 * QB;           // ... and the row sums
    constexpr int MAXC = NP >= 32 ? 8 : 4;           // pieces that carry the row maxima
    constexpr int EXC = NP - MAXC;                   // pieces that carry the 32 exponentials
    static_assert(2 * NDMA + 1 <= NP, "one tile load per piece");
    static_assert(KS >= 3 && 2 * DC >= 3, "fragment rings are three deep");

    __shared__ uint4 K0[TKW * CH], K1[TKW * CH];     // [key][chunk ^ (key & 7)]
    __shared__ uint4 V0[TKW * CH], V1[TKW * CH];     // [key][chunk ^ ((key % (CH/4)) << 2)]  (row-major, 64-byte granules)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;

    // workgroups sharing one (batch, kv head) - hence the same K/V - run on the same XCD (own L2 each)
    int bid = blockIdx.x;
    {
        const int total = gridDim.x, per = total >> 3, rem = total & 7;
        const int xcd = bid & 7, slot = bid >> 3;
        bid = xcd * per + min(xcd, rem) + slot;
    }
    const int rt = bid % a.row_tiles; bid /= a.row_tiles;
    const int kvh = bid % a.Hkv;
    const int b = bid / a.Hkv;
    const int rows_total = a.group * a.Nq;
    const bool wave_active = rt * kRowsWGWide + wave * kRowsWave < rows_total;
    const int nkeys = a.N;
    const int ntiles = (nkeys + TKW - 1) / TKW;
    const size_t kv_head = (size_t)b * a.Hkv + kvh;

    // ---- staging by LDS DMA: load i of this wave moves rows (4i + wave) * DMA_ROWS .. of a tile; lane l
    // lands at chunk position l % CH of row l / CH and therefore fetches the chunk the swizzle maps there.
    // Both swizzles only depend on the row modulo 4 DMA_ROWS, so the chunk a lane fetches is the same for every load.
    const int dma_row = lane / CH, dma_pos = lane % CH;
    const uint8_t *const k_glob = static_cast<const uint8_t *>(a.K) + kv_head * a.N * (size_t)ROWB;
    const uint8_t *const v_glob = static_cast<const uint8_t *>(a.V) + kv_head * a.N * (size_t)ROWB;
    const int dma_row0 = wave * DMA_ROWS + dma_row;                        // row of load 0; load i: + 4 i DMA_ROWS
    const unsigned dma_koff = (dma_pos ^ (dma_row0 & 7)) * 16;
    const unsigned dma_voff = (dma_pos ^ ((dma_row0 & (CH / 4 - 1)) << 2)) * 16;
    static_assert((4 * DMA_ROWS) % 8 == 0, "swizzle phase must not depend on the load index");
    // one load (index i) of a tile; rows past the last key repeat it (finite stand-ins, masked later)
    auto dma_one = [&](uint4 *dst, const uint8_t *glob, unsigned lane_off, int tile, int i) __attribute__((always_inline)) {
        const int r0 = (i * 4 + wave) * DMA_ROWS;
        const int row = min(tile * TKW + i * 4 * DMA_ROWS + dma_row0, nkeys - 1);
        const uint8_t *src = glob + (size_t)((unsigned)row * (unsigned)ROWB + lane_off);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                         (__attribute__((address_space(3))) void *)(dst + r0 * CH), 16, 0, 0);
    };
    auto dma_tile = [&](uint4 *dst, const uint8_t *glob, unsigned lane_off, int tile) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NDMA; ++i) dma_one(dst, glob, lane_off, tile, i);
    };
    auto kbuf = [&](auto p) __attribute__((always_inline)) -> uint4 * { if constexpr (decltype(p)::value == 0) return K0; else return K1; };
    auto vbuf = [&](auto p) __attribute__((always_inline)) -> uint4 * { if constexpr (decltype(p)::value == 0) return V0; else return V1; };

    // ---- prologue loads: K tiles 0 and 1, V tile 0 go straight to LDS while the Q fragments are fetched
    dma_tile(K0, k_glob, dma_koff, 0);
    dma_tile(V0, v_glob, dma_voff, 0);
    dma_tile(K1, k_glob, dma_koff, 1);

    bool row_ok[QB];
    size_t orow[QB];
    float c[QB];                                     // scores are exponentiated as 2^(s*c)
    intx4 qf[QB][KS];                                // B operand of S^T = K Q^T (8 bf16), kept in accumulation VGPRs
#pragma unroll
    for (int q = 0; q < QB; ++q) {
        const int v = rt * kRowsWGWide + wave * kRowsWave + q * 32 + l32;
        row_ok[q] = v < rows_total;
        const int vv = row_ok[q] ? v : rows_total - 1;
        const int head = kvh * a.group + vv / a.Nq;
        orow[q] = ((size_t)b * a.H + head) * (size_t)a.Nq + vv % a.Nq;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[q][ks] = __builtin_bit_cast(intx4, *reinterpret_cast<const uint4 *>(
                            static_cast<const uint16_t *>(a.Q) + orow[q] * D + ks * 16 + hh * 8));
        c[q] = a.scale_log2;
        if (a.q_scale) c[q] *= a.q_scale[b * a.H + head];
        if (a.k_scale) c[q] *= a.k_scale[b * a.Hkv + kvh];
    }
#pragma unroll
    for (int q = 0; q < QB; ++q)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[q][ks]));

    // ---- per-lane state of the two query blocks
    floatx16 acc[QB][DC], acc_l[QB];                 // O^T (unnormalised) and the row sums (all 16 registers equal)
#pragma unroll
    for (int q = 0; q < QB; ++q) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_l[q][r] = 0.f;
#pragma unroll
        for (int i = 0; i < DC; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[q][i][r] = 0.f;
    }
    float mc[QB] = {-INFINITY, -INFINITY};           // maximum in use (log2 units), equal in both lane halves
    intx4 ones = {0x3F803F80, 0x3F803F80, 0x3F803F80, 0x3F803F80};         // eight bf16 1.0
    asm volatile("" : "+v"(ones));                   // held in registers instead of being rebuilt per use

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
    // K fragment ks of the unit `sub` (0/1) of a tile buffer: keys 32 sub + l32, dims 16ks + 8hh .. +7
    auto k_frag = [&](const uint4 *kb, int sub, int ks) __attribute__((always_inline)) {
        return __builtin_bit_cast(intx4, *reinterpret_cast<const uint4 *>(
                   reinterpret_cast<const char *>(kb) + sub * 32 * ROWB + k_off[ks]));
    };
    // V^T fragment jv of the unit `sub` of a tile buffer: dims 32i + l32 (i = jv % DC),
    // keys 32 sub + 16 st + 4hh + {0..3, 8..11} (st = jv / DC)
    auto v_frag = [&](const uint4 *vb, int sub, int jv) __attribute__((always_inline)) {
        const int st = jv / DC, i = jv % DC;
        const char *p = reinterpret_cast<const char *>(vb) + (sub * 32 + 16 * st) * ROWB + v_off[i];
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)(p));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)(p + 8 * ROWB));
        const short8v w = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, w);
    };

    constexpr int RD = 3;                                    // fragment rings: fetched RD uses (2 RD MFMAs) ahead
    intx4 kfr[RD];
    bf16x8 vfr[RD];
    // Pipeline step u.  In: s_cur = S(u), pk_prev = P(u-1).  Out: pk_cur = P(u), s_nxt = S(u+1).
    // kb / ksub: tile buffer and unit of K(u+1); vb / vsub: those of V(u-1).
    // Every step has the same shape: units at or past the end of the keys are computed on finite
    // stand-in rows and masked to -inf, so they contribute exact zeros; P(-1) is zero.
    // `chain`: the next step reads unit 1 of the same tile buffers, so its first K fragments are fetched
    // in this step's last pieces; `primed`: the previous step did that for this one.
    // `dma`: this step also issues the tile loads of its stage (K tile into dk, V tile into dv).
    auto step = [&](int u, floatx16 (&s_cur)[QB], floatx16 (&s_nxt)[QB], unsigned (&pk_prev)[QB][2][4],
                    unsigned (&pk_cur)[QB][2][4], const uint4 *kb, int ksub, const uint4 *vb, int vsub,
                    auto primed, auto chain, auto dma, uint4 *dk, int ktile, uint4 *dv, int vtile)
                    __attribute__((always_inline)) {
        constexpr bool PRIMED = decltype(primed)::value, CHAIN = decltype(chain)::value;
        constexpr bool DMA = decltype(dma)::value;
        if (!PRIMED) {
#pragma unroll
            for (int j = 0; j < RD; ++j) kfr[j] = k_frag(kb, ksub, j);
        }
        if (__builtin_expect(32 * (u + 1) > nkeys, 0)) {     // uniform branch: keys at or past the end score -inf
#pragma unroll
            for (int q = 0; q < QB; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * u + 8 * (r >> 2) + 4 * hh + (r & 3) >= nkeys) s_cur[q][r] = -INFINITY;
        }
        float corr[QB], tm[QB], tpart[QB], pe[32];
        bool changed = false;
        // element e = 2 pr + (0/1) of the exponential stream is S(u)[q = pr & 1][r = 2 (pr >> 1) + (0/1)]
        auto exp_piece = [](int e) constexpr { int t = MAXC; while (!(e < 32 * (t - MAXC + 1) / EXC)) ++t; return t; };
        auto pack_pair = [&](int pr) __attribute__((always_inline)) {
            const int q = pr & 1, r = (pr >> 1) * 2;
            unsigned w = pack_bf16_rne(pe[2 * pr], pe[2 * pr + 1]);
            asm volatile("" : "+v"(w));                      // P(u) is only consumed a step later: keep its
            pk_cur[q][r >> 3][(r & 7) >> 1] = w;             // computation here, beside the matrix-core work
        };
        // everything of the step that is not an MFMA, dealt out over the NP pieces
        auto piece = [&](int t) __attribute__((always_inline)) {
            if (DMA && t >= 1 && t <= 2 * NDMA) {
                if (t <= NDMA) dma_one(dk, k_glob, dma_koff, ktile, t - 1);
                else dma_one(dv, v_glob, dma_voff, vtile, t - 1 - NDMA);
            }
            if (t < MAXC) {
                // row maxima of S(u) decide, without a divergent branch, whether the maxima in use are raised
#pragma unroll
                for (int v = 32 * t / MAXC; v < 32 * (t + 1) / MAXC; ++v) {
                    const int q = v >> 4, r = v & 15;
                    tpart[q] = r == 0 ? s_cur[q][0] : fmaxf(tpart[q], s_cur[q][r]);
                }
                if (t == MAXC - 1) {
                    bool need = false;
#pragma unroll
                    for (int q = 0; q < QB; ++q) {
                        tm[q] = half_swap_max(tpart[q]) * c[q];
                        need = need || (tm[q] > mc[q] + kSlack);
                    }
                    changed = __any(need);                   // wave-uniform; always true for the first unit
#pragma unroll
                    for (int q = 0; q < QB; ++q) {
                        const float mn = changed ? fmaxf(mc[q], tm[q]) : mc[q];
                        corr[q] = fast_exp2(mc[q] - mn);     // first unit: 2^(-inf) = 0
                        mc[q] = mn;
                    }
                }
            } else {
#pragma unroll
                for (int e = 32 * (t - MAXC) / EXC; e < 32 * (t - MAXC + 1) / EXC; ++e) {
                    const int pr = e >> 1, q = pr & 1, r = (pr >> 1) * 2 + (e & 1);
                    pe[e] = fast_exp2(fmaf(s_cur[q][r], c[q], -mc[q]));
                }
            }
            // pairs completed in the previous piece are packed now: a transcendental result cannot be
            // consumed by the very next instruction without a bubble
#pragma unroll
            for (int pr = 0; pr < 16; ++pr)
                if (exp_piece(2 * pr + 1) == t - 1) pack_pair(pr);
            __builtin_amdgcn_sched_barrier(0);               // nothing moves between pieces
        };
        // ---- S(u+1): the first V fragments are fetched meanwhile
#pragma unroll
        for (int j = 0; j < KS; ++j) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                if (j == 0) qk_first(s_nxt[q], kfr[0], qf[q][0]);
                else qk_next(s_nxt[q], kfr[j % RD], qf[q][j]);
                if (q == QB - 1 && j + RD < KS) kfr[j % RD] = k_frag(kb, ksub, j + RD);
                if (q == 0 && j >= KS - RD) vfr[j - (KS - RD)] = v_frag(vb, vsub, j - (KS - RD));
                piece(j * QB + q);
            }
        }
        // ---- O += V(u-1) P(u-1) and the row sums of P(u-1)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
#pragma unroll
            for (int i = 0; i < DC; ++i) {
                const int jv = st * DC + i;
#pragma unroll
                for (int q = 0; q < QB; ++q) {
                    const uint4 pw = make_uint4(pk_prev[q][st][0], pk_prev[q][st][1], pk_prev[q][st][2], pk_prev[q][st][3]);
                    acc[q][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[jv % RD], __builtin_bit_cast(bf16x8, pw),
                                                                        acc[q][i], 0, 0, 0);
                    if (q == QB - 1) {
                        if (jv + RD < 2 * DC) vfr[jv % RD] = v_frag(vb, vsub, jv + RD);
                        else if (CHAIN) kfr[jv + RD - 2 * DC] = k_frag(kb, 1, jv + RD - 2 * DC);
                    }
                    piece(NQK + st * (DC + 1) * QB + i * QB + q);
                }
            }
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                const uint4 pw = make_uint4(pk_prev[q][st][0], pk_prev[q][st][1], pk_prev[q][st][2], pk_prev[q][st][3]);
                acc_l[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ones),
                                                                   __builtin_bit_cast(bf16x8, pw), acc_l[q], 0, 0, 0);
                piece(NQK + st * (DC + 1) * QB + DC * QB + q);
            }
        }
#pragma unroll
        for (int pr = 0; pr < 16; ++pr)
            if (exp_piece(2 * pr + 1) == NP - 1) pack_pair(pr);
        if (__builtin_expect(changed, 0)) {                  // rare: everything accumulated so far changes units
#pragma unroll
            for (int q = 0; q < QB; ++q) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_l[q][r] *= corr[q];
#pragma unroll
                for (int i = 0; i < DC; ++i) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[q][i][r] *= corr[q];
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    floatx16 s0[QB], s1[QB];                                 // S(u) lives in s{u & 1}
    unsigned pk0[QB][2][4], pk1[QB][2][4];                   // P(u) lives in pk{u & 1}

    // Stage sp = steps 2sp+1 and 2sp+2.  With PAR = sp & 1 it reads K tile sp+1 from K[1-PAR] and V tile sp
    // from V[PAR], while K tile sp+2 streams into K[PAR] and V tile sp+1 into V[1-PAR] (stand-ins past the end).
    auto stage = [&](int sp, auto par) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par)::value;
        if (wave_active) {
            step(2 * sp + 1, s1, s0, pk0, pk1, kbuf(I_<1 - PAR>{}), 0, vbuf(I_<PAR>{}), 0, F_{}, T_{}, T_{},
                 kbuf(I_<PAR>{}), sp + 2, vbuf(I_<1 - PAR>{}), sp + 1);
            step(2 * sp + 2, s0, s1, pk1, pk0, kbuf(I_<1 - PAR>{}), 1, vbuf(I_<PAR>{}), 1, T_{}, F_{}, F_{},
                 kbuf(I_<PAR>{}), 0, vbuf(I_<1 - PAR>{}), 0);
        } else {
            dma_tile(kbuf(I_<PAR>{}), k_glob, dma_koff, sp + 2);
            dma_tile(vbuf(I_<1 - PAR>{}), v_glob, dma_voff, sp + 1);
        }
        __syncthreads();                                     // also the point where the streamed tiles are waited for
    };

    // ---- prologue: S(0), then step 0 (its P(-1) is zero)
    __syncthreads();
    if (wave_active) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                if (ks == 0) qk_first(s0[q], k_frag(K0, 0, 0), qf[q][0]);
                else qk_next(s0[q], k_frag(K0, 0, ks), qf[q][ks]);
            }
#pragma unroll
        for (int q = 0; q < QB; ++q)
#pragma unroll
            for (int t = 0; t < 8; ++t) pk1[q][t >> 2][t & 3] = 0u;
        // the compiler does not know that the statements above are matrix instructions whose results
        // need 11 more wait states before a vector instruction may read them
        asm volatile("s_nop 15\n\ts_nop 15" : "+v"(s0[0]), "+v"(s0[1]));
        step(0, s0, s1, pk1, pk0, K0, 1, V0, 0, F_{}, F_{}, F_{}, K0, 0, V0, 0);
    }
    __syncthreads();   // K tile 0 is overwritten during stage 0: every wave must be done with it

    // ---- stages 0 .. ntiles-1 = steps 1 .. 2 ntiles: the product with P(u) happens in step u+1, so this
    // covers every unit; the one or two surplus steps work on masked stand-in units
    int sp = 0;
    for (; sp + 1 < ntiles; sp += 2) {
        stage(sp, I_<0>{});
        stage(sp + 1, I_<1>{});
    }
    if (sp < ntiles) stage(sp, I_<0>{});

    if (!wave_active) return;
    // ---- normalise, transpose through LDS, write whole rows.  The tile buffers are free now (the barrier
    // that ended the last stage also waited for its loads); wave w uses buffer w: 64 rows of ROWB bytes.
    // O^T register r of chunk i holds dim 32 i + 8 (r / 4) + 4 hh + (r % 4) of query row l32 of its block.
    {
        constexpr int SL = D / 4;                                          // 8-byte slots per row
        char *region = reinterpret_cast<char *>(wave == 0 ? K0 : wave == 1 ? K1 : wave == 2 ? V0 : V1);
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const float inv = 1.0f / acc_l[q][0];
            const int row = q * 32 + l32;
#pragma unroll
            for (int i = 0; i < DC; ++i)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const uint2 w = make_uint2(pack_bf16_rne(acc[q][i][4 * q4] * inv, acc[q][i][4 * q4 + 1] * inv),
                                               pack_bf16_rne(acc[q][i][4 * q4 + 2] * inv, acc[q][i][4 * q4 + 3] * inv));
                    const int slot = i * 8 + q4 * 2 + hh;
                    // slots are XOR-ed with the row so that the 16 rows written together hit different banks
                    *reinterpret_cast<uint2 *>(region + row * ROWB + (slot ^ ((row & (SL / 2 - 1)) << 1)) * 8) = w;
                }
        }
        // query rows of one (batch, kv head) are contiguous in memory: row of virtual row v = first row + v
        uint8_t *og = static_cast<uint8_t *>(a.O) + ((size_t)b * a.H + (size_t)kvh * a.group) * a.Nq * ROWB;
        constexpr int LPR = ROWB / 16, RPI = 64 / LPR;                     // lanes per row, rows per store
        const int v_first = rt * kRowsWGWide + wave * kRowsWave;
#pragma unroll
        for (int it = 0; it < kRowsWave / RPI; ++it) {
            const int row = it * RPI + lane / LPR, ch = lane % LPR;
            const uint4 w = *reinterpret_cast<const uint4 *>(region + row * ROWB + (ch ^ (row & (SL / 2 - 1))) * 16);
            if (v_first + row < rows_total) *reinterpret_cast<uint4 *>(og + (size_t)(v_first + row) * ROWB + ch * 16) = w;
        }
    }
}

}  // namespace

hipError_t launch_attention_wide(const AttnArgs &a, hipStream_t stream)
{
    AttnKernelArgs k;
    fill_kernel_args(a, k, kRowsWGWide, TKW);
    const dim3 grid((unsigned)((long)a.B * a.Hkv * k.row_tiles)), block(kAttnThreads);
    if (a.d == 128) return launch(attn_wide_kernel<128>, grid, block, stream, k);
    return launch(attn_wide_kernel<64>, grid, block, stream, k);
}

}  // namespace dd
