// Matrix-core attention for bf16 (and fp8-e4m3 Q/K) inputs on gfx950:
//     O = softmax(Q K^T / sqrt(d_k)) V            (Eq. 3, over all key positions: Sec. 2.2)
// used by the verifier's full attention and, with a split key range, by the drafter's
// block attention over the cached K/V (Sec. 2.3).
//
// Layout of the computation (one wave = 32 query rows, one workgroup = 4 waves = 128 rows):
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K fragment (from LDS), B = Q (registers); fp8 Q/K: the 64-deep
//                 fp8 instruction on the e4m3 bytes as stored (see KRAW below).
//                 The 32x32 result puts one QUERY per lane column and 16 KEYS in the lane's
//                 registers, so the softmax row reductions are in-register plus one
//                 exchange between the two lane halves (v_permlane32_swap).
//   O^T += V^T P^T  A = V^T (LDS, keys contiguous), B = P^T.  The accumulator layout of
//                 S^T is exactly the B-operand layout of this product once the keys of a
//                 16-key step are taken in the order the accumulator holds them, so the
//                 probabilities never leave registers; V is transposed once per tile while
//                 it is staged into LDS, in that same key order.
//   The rescale factor of the online softmax is per query = per lane: a plain multiply, and
//   it is applied lazily (only when a unit's maximum exceeds the maximum in use by 2^8).
// Pipeline: the softmax works on 32-key units.  While the exponentials of unit u run on the
// vector ALUs, the matrix-core steps producing the scores of unit u+1 are issued in between
// them; then the PV product of unit u follows.  K lives in a 128-row LDS ring whose 64-key
// staging windows are offset by half a tile against the V tiles, so one barrier per 64 keys
// suffices; the next window / tile is prefetched into registers during the current one.
// Both LDS arrays are XOR-swizzled at 16-byte granularity: operand reads and staging writes
// are bank-conflict free without padding.  Workgroups are renumbered so that those sharing
// one (batch, kv head) run on the same XCD and hit its L2.
// Row sums use plain adds: v_dot2c_f32_bf16 was measured to serialise with the MFMA pipe.
#include "attention_common.h"
#include "dd_internal.h"

namespace dd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef int intx8 __attribute__((ext_vector_type(8)));

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

// Block-scaled ("MX") storage, OCP Microscaling Formats v1.0: 32 consecutive elements of the head dimension share
// one E8M0 scale 2^(code - 127).  Decoding is exact in bf16 as long as the result is a normal bf16 number (or zero).
__device__ __forceinline__ float e8m0_to_f32(unsigned code)
{
    return __uint_as_float(code ? code << 23 : 0x00400000u);     // code 0 = 2^-127, a subnormal fp32
}
// eight bf16 (in four registers) times a power of two
__device__ __forceinline__ uint4 bf16x8_times(uint4 w, float s)
{
    const unsigned u[4] = {w.x, w.y, w.z, w.w};
    unsigned r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        r[i] = pack_bf16_trunc(__uint_as_float(u[i] << 16) * s, __uint_as_float(u[i] & 0xFFFF0000u) * s);
    return make_uint4(r[0], r[1], r[2], r[3]);
}
// eight e2m1 codes (sign, two exponent bits with bias 1, one mantissa bit; four bits each, element 0 lowest) -> bf16
__device__ __forceinline__ uint4 fp4x8_to_bf16x8(unsigned w)
{
    unsigned h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned c = (w >> (4 * i)) & 15u, e = (c >> 1) & 3u, m = c & 1u;
        const unsigned mag = e ? ((126u + e) << 7) | (m << 6) : (m ? 0x3F00u : 0u);   // (1 + m/2) 2^(e-1); 0.5 m
        h[i] = mag | ((c & 8u) << 12);
    }
    return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// The same decode and the multiplication by the block's scale 2^(sc - 127) in one go, by table lookup: the bf16
// pattern of magnitude code c = 2 e + m (e >= 1) times the scale is ((e + sc - 1) << 7) | (m << 6) = (c << 6) + K with
// K = (sc - 1) << 7, that of c = 1 (0.5) is K, that of c = 0 is 0 - eight 16-bit entries that depend on the scale only.
// Split into a table of low and one of high bytes (eight bytes = two registers each), v_perm_b32 looks up four codes
// per instruction (selector bytes 0-3 pick from its second operand, 4-7 from its first); the signs go into the high
// bytes, and four more byte permutes put the halves together.  29 vector instructions for eight elements instead of
// about 80.  Exact while every result is a normal bf16 number, i.e. for 2 <= sc <= 252; other scales take the plain path.
__device__ __forceinline__ uint4 fp4x8_scaled_to_bf16x8(unsigned w, unsigned sc)
{
    if (__builtin_expect(sc - 2u > 250u, 0)) return bf16x8_times(fp4x8_to_bf16x8(w), e8m0_to_f32(sc));
    const unsigned k2 = ((sc - 1u) << 7) * 0x00010001u;
    const unsigned t01 = k2 & 0xFFFF0000u, t23 = k2 + 0x00C00080u, t45 = k2 + 0x01400100u, t67 = k2 + 0x01C00180u;
    const unsigned l0 = __builtin_amdgcn_perm(t23, t01, 0x06040200u), h0 = __builtin_amdgcn_perm(t23, t01, 0x07050301u);
    const unsigned l1 = __builtin_amdgcn_perm(t67, t45, 0x06040200u), h1 = __builtin_amdgcn_perm(t67, t45, 0x07050301u);
    const unsigned se = w & 0x07070707u, so = (w >> 4) & 0x07070707u;       // codes of elements 0,2,4,6 / 1,3,5,7
    const unsigned le = __builtin_amdgcn_perm(l1, l0, se), lo = __builtin_amdgcn_perm(l1, l0, so);
    const unsigned he = __builtin_amdgcn_perm(h1, h0, se) | ((w & 0x08080808u) << 4);
    const unsigned ho = __builtin_amdgcn_perm(h1, h0, so) | (w & 0x80808080u);
    const unsigned e01 = __builtin_amdgcn_perm(he, le, 0x05010400u), e23 = __builtin_amdgcn_perm(he, le, 0x07030602u);   // elements (0, 2), (4, 6)
    const unsigned o01 = __builtin_amdgcn_perm(ho, lo, 0x05010400u), o23 = __builtin_amdgcn_perm(ho, lo, 0x07030602u);   // elements (1, 3), (5, 7)
    return make_uint4(__builtin_amdgcn_perm(o01, e01, 0x05040100u), __builtin_amdgcn_perm(o01, e01, 0x07060302u),
                      __builtin_amdgcn_perm(o23, e23, 0x05040100u), __builtin_amdgcn_perm(o23, e23, 0x07060302u));
}

// exchange between lane l and lane l^32 (one v_permlane32_swap), then combine
__device__ __forceinline__ float half_swap_max(float x)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float half_swap_sum(float x)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}

// The running maximum used for exponentiation is raised only when a tile's maximum exceeds it
// by more than this many powers of two; until then probabilities are at most 2^8, which bf16
// and the fp32 accumulators hold without loss, and the 64 accumulator multiplies are skipped.
constexpr float kRescaleSlack = 8.0f;

// BLOCK = false: verifier attention (all rows of a head attend all keys, O written directly).
// BLOCK = true : drafter block attention (key rows of the active block may come from the fresh
//                block tensors, the key range may be split, partial states go to the workspace).
// V8: V (and Vblk) are fp8 e4m3 as well, decoded exactly to bf16 on their way into LDS; their per-head
//      scale multiplies the output once, at the end.
// MX: block-scaled inputs (verifier form only): Q and K with e4m3 elements, V with e2m1 elements (two per byte), each
//      with one E8M0 scale per 32 elements of the head dimension (a.q_mx, a.k_mx, a.v_mx: [rows][D / 32] bytes).
//      S = K Q^T runs on the block-scaled matrix instruction (v_mfma_scale_f32_32x32x64_f8f6f4: 64 head dims per
//      instruction, the E8M0 scales of both operands applied by the hardware), K staying e4m3 in LDS; V's scales run
//      along the head dimension, not along the keys its product contracts over, so V is decoded, times its block's
//      scale, to bf16 (exact) on its way into LDS and O += V P runs as in the other forms.
//      Operand layout of that instruction, found by comparing it with a plain sum for random operands and scales: of
//      a lane's 32 operand bytes (row = lane % 32) the first 16 are elements 16 hh .. 16 hh + 15 of the 64 (hh = lane /
//      32) and belong to scale block 0, the last 16 are elements 32 + 16 hh .. and belong to block 1; the scale of
//      (row, block b) is taken from lane row + 32 b (its selected byte).
template <int D, bool FP8, bool BLOCK, bool V8 = false, bool MX = false>
__global__ __launch_bounds__(kAttnThreads, 2) void attn_mfma_kernel(const AttnKernelArgs a)
{
    static_assert(!MX || (FP8 && !BLOCK && !V8), "block-scaled inputs: e4m3 Q/K, e2m1 V, verifier form");
    // KRAW: every fp8 form keeps Q and K as e4m3 bytes - K in LDS as stored, Q in registers - and computes S = K Q^T on
    // the 64-deep fp8 matrix instruction (twice the bf16 rate, and no vector instruction decodes K); without block
    // scales the instruction's scale operands are the neutral code 127 (2^0) and the per-head fp32 scales stay in the
    // exponent's factor.  "MX" in the names below is historical: the code path is this one.
    constexpr bool KRAW = FP8;
    static_assert(!KRAW || D % 64 == 0, "an fp8 matrix instruction takes 64 head dims");
    constexpr int CH = D / 8;                        // 16-byte chunks (8 bf16) per K row
    constexpr int KCH = TK * CH / kAttnThreads;      // K chunks staged per thread
    constexpr int KROWS = kAttnThreads / CH;         // K rows covered by one pass of the workgroup
    constexpr int VTASKS = (TK / 8) * CH * 2;        // V transpose tasks per tile (4 keys x 8 dims)
    constexpr int KS = D / 16;                       // MFMA k-steps over the head dim
    constexpr int DC = D / 32;                       // 32-wide chunks of the head dim
    constexpr int KELEM = FP8 ? 1 : 2;               // bytes per K element in memory
    constexpr int VB8 = MX ? 4 : V8 ? 8 : 16;        // bytes of eight V elements in memory
    constexpr int VROWB = D / 8 * VB8;               // bytes of a V row
    static_assert(KCH >= 1 && VTASKS <= kAttnThreads, "tile does not fit the staging scheme");

    constexpr int KSX = D / 64;                      // MX: block-scaled matrix instructions per 32-key unit
    constexpr int KCR = D / 16;                      // MX: 16-byte chunks of a K row as stored (e4m3)
    __shared__ uint4 Ks[2 * TK * CH];                // ring of 128 key rows: [key % 128][chunk ^ (key & 7)]
    __shared__ unsigned Ksc[MX ? 2 * TK : 1];        // MX: the rows' E8M0 scales, D / 32 bytes each in one word
    __shared__ uint4 Vt[2][D * (TK / 8)];            // [dim][keygroup ^ swz(dim)], 8 keys per 16 bytes

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;

    // ---- which (batch, kv head, row tile, key split) this workgroup owns
    int bid = blockIdx.x;
    {
        // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Remap so that the
        // workgroups sharing one (batch, kv head) - hence the same K/V - run on the same XCD.
        const int total = gridDim.x, per = total >> 3, rem = total & 7;
        const int xcd = bid & 7, slot = bid >> 3;
        bid = xcd * per + min(xcd, rem) + slot;
    }
    const int sp = bid % a.splits; bid /= a.splits;
    const int rt = bid % a.row_tiles; bid /= a.row_tiles;
    const int kvh = bid % a.Hkv;
    const int b = bid / a.Hkv;
    const int rows_total = a.group * a.Nq;
    const int v = rt * a.rows_per_wg + wave * kRowsPerWave + l32;
    const bool row_ok = v < rows_total;
    const int vv = row_ok ? v : rows_total - 1;
    const int head = kvh * a.group + vv / a.Nq;
    const int qi = vv % a.Nq;
    // waves past the workgroup's rows only help to stage the tiles
    const bool wave_active = wave * kRowsPerWave < a.rows_per_wg && rt * a.rows_per_wg + wave * kRowsPerWave < rows_total;
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
    // MX: the operand bytes as they are (see the layout above) and the row's scales, this lane's block in byte 0 (+ 2 j)
    intx8 qx[KRAW ? KSX : 1];
    unsigned qsw = 0x7F7F7F7Fu;                      // (neutral scales unless the input is block-scaled)
    if constexpr (KRAW) {
        const uint8_t *qrow = static_cast<const uint8_t *>(a.Q) + orow * D;
#pragma unroll
        for (int j = 0; j < KSX; ++j) {
            const uint4 lo = *reinterpret_cast<const uint4 *>(qrow + 64 * j + 16 * hh);
            const uint4 hi = *reinterpret_cast<const uint4 *>(qrow + 64 * j + 32 + 16 * hh);
            qx[j] = intx8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
        if constexpr (MX)
            qsw = (D == 128 ? *reinterpret_cast<const unsigned *>(a.q_mx + orow * 4)
                            : (unsigned)*reinterpret_cast<const unsigned short *>(a.q_mx + orow * 2)) >> (8 * hh);
    }
    float c = a.scale_log2;                          // scores are exponentiated as 2^(s*c)
    if (a.q_scale) c *= a.q_scale[b * a.H + head];
    if (a.k_scale) c *= a.k_scale[b * a.Hkv + kvh];

    const int k_begin = sp * a.keys_per_split;
    const int k_end = min(a.N, k_begin + a.keys_per_split);
    const int ntiles = (k_end - k_begin + TK - 1) / TK;
    const size_t kv_head = (size_t)b * a.Hkv + kvh;
    const int bstart = a.block_starts ? a.block_starts[b] : a.block_start;   // any value is safe: rows are chosen by range test

    // ---- staging: global -> registers -> LDS
    uint4 kreg[KCH];
    uint4 vreg[4];
    const int k_row0 = tid / CH, k_ch = tid % CH;                                  // K chunk i: row k_row0 + i*KROWS
    const int vt_dchunk = tid % CH, vt_e4 = (tid / CH) & 1, vt_g = tid / (2 * CH);   // V task of this thread
    // keys of task (g, e4): tile-local index (g/4)*32 + ((g/2)&1)*16 + 8*e4 + 4*(g&1) + e,  e = 0..3
    const int vt_key0 = (vt_g >> 2) * 32 + ((vt_g >> 1) & 1) * 16 + 8 * vt_e4 + 4 * (vt_g & 1);
    const uint8_t *const k_base = static_cast<const uint8_t *>(a.K) + kv_head * a.kv_stride * (size_t)(D * KELEM) + k_ch * (8 * KELEM);
    const uint8_t *const v_base = static_cast<const uint8_t *>(a.V) + kv_head * a.kv_stride * (size_t)VROWB + vt_dchunk * VB8;

    // address of key row j's chunk for this thread; rows past the range are clamped to the last
    // valid row (their scores are masked to -inf, their values multiply a zero probability)
    auto k_src = [&](int j) -> const uint8_t * {
        j = min(j, k_end - 1);
        if (BLOCK && (unsigned)j - (unsigned)bstart < (unsigned)a.block_len)
            return static_cast<const uint8_t *>(a.Kblk) +
                   (kv_head * a.block_len + (size_t)(j - bstart)) * (size_t)(D * KELEM) + k_ch * (8 * KELEM);
        return k_base + (size_t)j * (D * KELEM);
    };
    auto v_src = [&](int j) -> const uint8_t * {
        j = min(j, k_end - 1);
        if (BLOCK && (unsigned)j - (unsigned)bstart < (unsigned)a.block_len)
            return static_cast<const uint8_t *>(a.Vblk) +
                   (kv_head * a.block_len + (size_t)(j - bstart)) * (size_t)VROWB + vt_dchunk * VB8;
        return v_base + (size_t)j * VROWB;
    };
    // K is staged in windows of 64 keys that are offset by half a tile against the V tiles:
    // window w = keys [64w+32, 64w+96) relative to the range start.  A ring of 128 rows then always
    // holds the two 32-key units the current stage multiplies while the next window is written.
    const int nkeys = k_end - k_begin;
    auto load_k = [&](uint4 (&dst)[KCH], int j0, int nch) {   // rows j0 + k_row0 + i*KROWS, i < nch
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            if (i < nch) {
                const uint8_t *p = k_src(k_begin + j0 + k_row0 + i * KROWS);
                if (FP8) {
                    const uint2 r = *reinterpret_cast<const uint2 *>(p);
                    dst[i] = make_uint4(r.x, r.y, 0, 0);
                    if (MX) {                          // the row's scales travel with it
                        const size_t rg = kv_head * a.kv_stride + (size_t)min(k_begin + j0 + k_row0 + i * KROWS, k_end - 1);
                        dst[i].z = D == 128 ? *reinterpret_cast<const unsigned *>(a.k_mx + rg * 4)
                                            : (unsigned)*reinterpret_cast<const unsigned short *>(a.k_mx + rg * 2);
                    }
                } else {
                    dst[i] = *reinterpret_cast<const uint4 *>(p);
                }
            }
        }
    };
    auto load_v = [&](int t) {
        const int k0 = k_begin + t * TK;
        if (tid < VTASKS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (MX) {
                    const int j = min(k0 + vt_key0 + e, k_end - 1);
                    vreg[e] = make_uint4(*reinterpret_cast<const unsigned *>(v_src(j)),
                                         a.v_mx[(kv_head * a.kv_stride + (size_t)j) * (D / 32) + vt_dchunk / 4], 0, 0);
                } else if (V8) {
                    const uint2 r = *reinterpret_cast<const uint2 *>(v_src(k0 + vt_key0 + e));
                    vreg[e] = make_uint4(r.x, r.y, 0, 0);    // decoded when it is stored to LDS
                } else {
                    vreg[e] = *reinterpret_cast<const uint4 *>(v_src(k0 + vt_key0 + e));
                }
            }
        }
    };
    auto store_k = [&](const uint4 (&src)[KCH], int j0, int nch) {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            if (i < nch) {
                const int row = (j0 + k_row0 + i * KROWS) & (2 * TK - 1);
                uint4 w = src[i];
                if constexpr (KRAW) {
                    // e4m3 as stored: 8 bytes into [row][16-byte chunk ^ (row % KCR)]
                    char *p = reinterpret_cast<char *>(Ks) + (row * KCR + ((k_ch >> 1) ^ (row & (KCR - 1)))) * 16 + (k_ch & 1) * 8;
                    *reinterpret_cast<uint2 *>(p) = make_uint2(w.x, w.y);
                    if (MX && k_ch == 0) Ksc[row] = w.z;
                } else {
                    if (FP8) w = fp8x8_to_bf16x8(make_uint2(w.x, w.y));
                    Ks[row * CH + (k_ch ^ (row & 7))] = w;
                }
            }
        }
    };
    auto store_v = [&](int buf) {
        if (tid < VTASKS) {
            // 4 keys x 8 dims -> 8 dims x 4 keys
            uint4 vr[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                vr[e] = MX ? fp4x8_scaled_to_bf16x8(vreg[e].x, vreg[e].y)
                      : V8 ? fp8x8_to_bf16x8(make_uint2(vreg[e].x, vreg[e].y)) : vreg[e];
            const unsigned r0[4] = {vr[0].x, vr[0].y, vr[0].z, vr[0].w};
            const unsigned r1[4] = {vr[1].x, vr[1].y, vr[1].z, vr[1].w};
            const unsigned r2[4] = {vr[2].x, vr[2].y, vr[2].z, vr[2].w};
            const unsigned r3[4] = {vr[3].x, vr[3].y, vr[3].z, vr[3].w};
            uint2 *vt2 = reinterpret_cast<uint2 *>(Vt[buf]);
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
    float mc = -INFINITY;        // maximum in use, in log2 units (raw score * c); equal in both lane halves
    float l_run = 0.f;           // this lane half's share of the running sum

    // The softmax works on units of 32 keys x 32 queries (one accumulator block, 16 scores per
    // lane); an LDS tile holds two units.

    // matrix-core step ks (16 head dims) of S^T = K Q^T for the 32-key unit u (keys 32u .. 32u+31)
    auto qk_step = [&](int u, int ks, floatx16 &s) {
        const int krow = (u & 3) * 32 + l32;
        const uint4 w = Ks[krow * CH + ((2 * ks + hh) ^ (krow & 7))];
        floatx16 cin = s;
        if (ks == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) cin[r] = 0.f;
        }
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), qf[ks], cin, 0, 0, 0);
    };

    // MX: the 16-byte chunk `half` (0 / 1) of this lane's operand of block-scaled instruction j for key row `krow`
    // of the ring: elements 64 j + 32 half + 16 hh .. +15 of the row
    auto kx_chunk = [&](int krow, int j, int half) -> uint4 {
        return Ks[krow * KCR + ((4 * j + 2 * half + hh) ^ (krow & (KCR - 1)))];
    };
    auto mx_mfma = [&](const uint4 &lo, const uint4 &hi, unsigned ksw, int j, const floatx16 &cin) -> floatx16 {
        const intx8 kx = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        // both operands e4m3; scale byte 0 of each scale register (the words are shifted so that it is this lane's
        // block of this instruction)
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kx, qx[j], cin, 0, 0, 0, (int)(ksw >> (16 * j)), 0,
                                                               (int)(qsw >> (16 * j)));
    };
    auto qk_unit_mx = [&](int u, floatx16 &s) {         // S^T of unit u, all of it
        const int krow = (u & 3) * 32 + l32;
        const unsigned ksw = MX ? Ksc[krow] >> (8 * hh) : 0x7F7F7F7Fu;
        floatx16 cin;
#pragma unroll
        for (int r = 0; r < 16; ++r) cin[r] = 0.f;
#pragma unroll
        for (int j = 0; j < KSX; ++j) cin = mx_mfma(kx_chunk(krow, j, 0), kx_chunk(krow, j, 1), ksw, j, cin);
        s = cin;
    };

    // keys past the end of the range score -inf (only the last tile can be ragged)
    auto mask_tail = [&](int t, int sub, floatx16 &s) {
        const int k0 = k_begin + t * TK + sub * 32;
        if (k0 + 32 > k_end) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (k0 + 8 * (r >> 2) + 4 * hh + (r & 3) >= k_end) s[r] = -INFINITY;
        }
    };

    // unit maximum; raise the maximum in use (and rescale the running state) only when needed
    auto update_max = [&](const floatx16 &s) {
        float tmax = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
        const float tm = half_swap_max(tmax) * c;
        if (__any(tm > mc + kRescaleSlack)) {        // always true on the first unit (mc = -inf)
            const float mn = fmaxf(mc, tm);
            const float corr = fast_exp2(mc - mn);
            mc = mn;
            l_run *= corr;
#pragma unroll
            for (int i = 0; i < DC; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][r] *= corr;
        }
    };

    // probabilities of scores (2*step, 2*step+1) of a unit, packed to bf16 in B-operand order
    auto exp_step = [&](int step, const floatx16 &s, unsigned (&pk)[2][4]) {
        const int r = step * 2;
        const float p0 = fast_exp2(fmaf(s[r], c, -mc));
        const float p1 = fast_exp2(fmaf(s[r + 1], c, -mc));
        const unsigned w = pack_bf16_rne(p0, p1);
        l_run += p0 + p1;     // plain adds: v_dot2c_f32_bf16 would serialise with the matrix cores
        pk[r >> 3][(r & 7) >> 1] = w;
    };

    // O^T += V^T P^T for one unit
    auto pv = [&](int buf, int sub, const unsigned (&pk)[2][4]) {   // buf = tile & 1, sub = unit within the tile
#pragma unroll
        for (int i = 0; i < DC; ++i) {
            const int drow = i * 32 + l32;
            const int swz = (drow ^ (drow >> 3)) & 7;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const int g = sub * 4 + st * 2 + hh;
                const uint4 w = Vt[buf][drow * (TK / 8) + (g ^ swz)];
                const uint4 pw = make_uint4(pk[st][0], pk[st][1], pk[st][2], pk[st][3]);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w),
                                                                 __builtin_bit_cast(bf16x8, pw), acc[i], 0, 0, 0);
            }
        }
    };

    // Softmax + PV of unit u (scores in s_cur) while, if have_next, the scores of unit u+1 are
    // produced into s_nxt: the matrix-core steps are interleaved one by one with the exponentials,
    // so the vector ALU work runs in the shadow of the matrix cores within the same wave.
    // LDS fragment m of a unit's 16 matrix-core slots: slots 0..KS-1 are the K fragments of unit u+1,
    // the following 2*DC are the V fragments of unit u (k-step major, 32-dim chunk minor)
    auto frag = [&](int u, int m) -> uint4 {
        if (m < KS) {
            const int krow = ((u + 1) & 3) * 32 + l32;
            return Ks[krow * CH + ((2 * m + hh) ^ (krow & 7))];
        }
        const int j = m - KS, st = j / DC, i = j % DC;
        const int drow = i * 32 + l32;
        const int g = (u & 1) * 4 + st * 2 + hh;
        return Vt[(u >> 1) & 1][drow * (TK / 8) + (g ^ ((drow ^ (drow >> 3)) & 7))];
    };
    auto unit = [&](int u, floatx16 &s_cur, bool have_next, floatx16 &s_nxt) {
        unsigned pk[2][4];
        update_max(s_cur);
        if constexpr (KRAW) {
            if (have_next) {
                // the K operands of unit u+1 and the first V fragments of unit u, then: a block-scaled instruction
                // every 8 / KSX exponential steps, the V products after them
                const int krow = ((u + 1) & 3) * 32 + l32;
                uint4 kf[2 * KSX];
#pragma unroll
                for (int m = 0; m < 2 * KSX; ++m) kf[m] = kx_chunk(krow, m >> 1, m & 1);
                const unsigned ksw = MX ? Ksc[krow] >> (8 * hh) : 0x7F7F7F7Fu;
                constexpr int PD = 3;
                uint4 fv[2 * DC];
#pragma unroll
                for (int j = 0; j < PD; ++j) fv[j] = frag(u, KS + j);
                floatx16 cin;
#pragma unroll
                for (int r = 0; r < 16; ++r) cin[r] = 0.f;
#pragma unroll
                for (int step = 0; step < 8; ++step) {
                    if (step % (8 / KSX) == 0) {
                        const int j = step / (8 / KSX);
                        cin = mx_mfma(kf[2 * j], kf[2 * j + 1], ksw, j, cin);
                    }
                    exp_step(step, s_cur, pk);
                }
                s_nxt = cin;
#pragma unroll
                for (int j = 0; j < 2 * DC; ++j) {
                    const int st = j / DC, i = j % DC;
                    if (j + PD < 2 * DC) fv[j + PD] = frag(u, KS + j + PD);
                    const uint4 pw = make_uint4(pk[st][0], pk[st][1], pk[st][2], pk[st][3]);
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fv[j]),
                                                                     __builtin_bit_cast(bf16x8, pw), acc[i], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int step = 0; step < 8; ++step) exp_step(step, s_cur, pk);
                pv((u >> 1) & 1, u & 1, pk);
            }
        } else if (have_next) {
            constexpr int NSLOT = KS + 2 * DC;              // matrix-core slots of the unit
            constexpr int PD = 3;                           // fragments requested this many slots ahead
            uint4 fq[NSLOT];
#pragma unroll
            for (int m = 0; m < PD; ++m) fq[m] = frag(u, m);
            constexpr int every = 8 / KS > 0 ? 8 / KS : 1;
#pragma unroll
            for (int step = 0; step < 8; ++step) {
                if (step % every == 0) {
                    const int m = step / every;
                    if (m + PD < NSLOT) fq[m + PD] = frag(u, m + PD);
                    floatx16 cin = s_nxt;
                    if (m == 0) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) cin[r] = 0.f;
                    }
                    s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fq[m]), qf[m], cin, 0, 0, 0);
                }
                exp_step(step, s_cur, pk);
            }
#pragma unroll
            for (int j = 0; j < 2 * DC; ++j) {
                const int m = KS + j, st = j / DC, i = j % DC;
                if (m + PD < NSLOT) fq[m + PD] = frag(u, m + PD);
                const uint4 pw = make_uint4(pk[st][0], pk[st][1], pk[st][2], pk[st][3]);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fq[m]),
                                                                 __builtin_bit_cast(bf16x8, pw), acc[i], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int step = 0; step < 8; ++step) exp_step(step, s_cur, pk);
            pv((u >> 1) & 1, u & 1, pk);
        }
    };

    constexpr int UNIT0_CH = 32 / KROWS;               // chunks per thread to stage keys 0..31
    {
        // all prologue loads are in flight together: keys 0..31, window 0 (units 1 and 2), V tile 0
        uint4 k0[KCH];
        load_k(k0, 0, UNIT0_CH);
        if (32 < nkeys) load_k(kreg, 32, KCH);
        load_v(0);
        store_k(k0, 0, UNIT0_CH);
        if (32 < nkeys) store_k(kreg, 32, KCH);
        store_v(0);
    }
    __syncthreads();
    floatx16 s_a, s_b;
    if (wave_active) {
        if constexpr (KRAW) qk_unit_mx(0, s_a);
        else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qk_step(0, ks, s_a);
        }
    }
    __syncthreads();   // unit 0's ring slot is rewritten at the end of stage 0: every wave must have read it
    // Stage t: on entry units 2t .. 2t+2 of K and tile t of V are in LDS, s_a holds the scores of unit 2t.
    for (int t = 0; t + 1 < ntiles; ++t) {
        const bool more_k = TK * (t + 1) + 32 < nkeys;  // window t+1 = units 2t+3, 2t+4
        if (more_k) load_k(kreg, TK * (t + 1) + 32, KCH);
        load_v(t + 1);
        if (wave_active) {
            unit(2 * t, s_a, true, s_b);
            unit(2 * t + 1, s_b, true, s_a);
        }
        if (more_k) store_k(kreg, TK * (t + 1) + 32, KCH);   // overwrites units 2t-1, 2t: read one stage ago
        store_v((t + 1) & 1);                          // overwrites V(t-1): read one stage ago
        __syncthreads();
    }
    if (wave_active) {                                  // last tile: nothing to prefetch, possibly ragged
        const int t = ntiles - 1;
        const bool two_units = TK * t + 32 < nkeys;
        mask_tail(t, 0, s_a);
        if (two_units) {
            unit(2 * t, s_a, true, s_b);
            mask_tail(t, 1, s_b);
            unit(2 * t + 1, s_b, false, s_a);
        } else {
            unit(2 * t, s_a, false, s_b);
        }
    }

    if (!wave_active) return;
    const float l_tot = half_swap_sum(l_run);
    if (!row_ok) return;
    // accumulator register r of chunk i holds dim 32*i + 8*(r/4) + 4*hh + (r%4) of this lane's query
    const float vs = V8 ? a.v_scale[kv_head] : 1.0f;     // the decoded V values times this are the real ones
    if (!BLOCK || a.splits == 1) {
        const float inv = vs / l_tot;
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
                    make_float4(acc[i][4 * q4] * vs, acc[i][4 * q4 + 1] * vs, acc[i][4 * q4 + 2] * vs, acc[i][4 * q4 + 3] * vs);
        if (hh == 0) {
            float *ml = a.part_ml + (orow * a.splits + sp) * 2;
            ml[0] = mc;
            ml[1] = l_tot;
        }
    }
}

// Block-completion refresh of the cache (Sec. 2.3: the cache is brought up to date when a block is done):
// the block's K and V rows, dense in [B*Hkv, block_len, d], replace rows block_start.. of every (batch, kv head)
// of the cache.  Everything in 16-byte chunks; workgroups `first_wg`.. of the launch do the copying.
struct RefreshArgs {
    const uint4 *src[2];       // Kblk, Vblk
    uint4 *dst[2];             // Kc, Vc at row 0 of (batch 0, kv head 0)
    int per_bh[2];             // chunks of the block per (batch, kv head)
    long bh_stride[2];         // chunks between consecutive (batch, kv head) in the cache
    long offset[2];            // chunks from a cache (batch, kv head) base to row block_start
    int wgs_per_bh;            // copying workgroups per (batch, kv head)
    int first_wg;              // workgroups below this one merge partial states
};

__device__ __forceinline__ void refresh_cache_rows(const RefreshArgs &r)
{
    const int cw = (int)blockIdx.x - r.first_wg;
    const int bh = cw / r.wgs_per_bh;
    const int first = (cw - bh * r.wgs_per_bh) * (int)blockDim.x + (int)threadIdx.x;
    const int step = r.wgs_per_bh * (int)blockDim.x;
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const uint4 *src = r.src[w] + (long)bh * r.per_bh[w];
        uint4 *dst = r.dst[w] + (long)bh * r.bh_stride[w] + r.offset[w];
        for (int in = first; in < r.per_bh[w]; in += step) dst[in] = src[in];
    }
}

// Merge the per-split partial states of each query row: O = sum_s 2^{m_s-M} O_s / sum_s 2^{m_s-M} l_s.
template <bool OUT_BF16>
__device__ __forceinline__ void combine_rows(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                             void *__restrict__ O, long rows, int splits, int d)
{
    const int per_row = d / 4;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long row = gid / per_row;
    const int c4 = (int)(gid % per_row);
    if (row >= rows) return;
    // every load of the row is issued before the first use (at most 16 splits): one memory round trip
    constexpr int kMaxSplits = 16;
    const float2 *ml = reinterpret_cast<const float2 *>(part_ml + row * splits * 2);
    float2 st[kMaxSplits];
    float4 po[kMaxSplits];
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
        st[s] = make_float2(-INFINITY, 0.f);
        po[s] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (s < splits) {
            st[s] = ml[s];
            po[s] = *reinterpret_cast<const float4 *>(part_o + (row * splits + s) * d + c4 * 4);
        }
    }
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) M = fmaxf(M, st[s].x);
    float L = 0.f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
        if (s < splits) {
            const float w = fast_exp2(st[s].x - M);
            L += w * st[s].y;
            o.x += w * po[s].x; o.y += w * po[s].y; o.z += w * po[s].z; o.w += w * po[s].w;
        }
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

template <bool OUT_BF16>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml, void *__restrict__ O,
                                                           long rows, int splits, int d)
{
    combine_rows<OUT_BF16>(part_o, part_ml, O, rows, splits, d);
}

// the same launch with the block-completion copy on the workgroups past the merging ones
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void attn_combine_refresh_kernel(const float *__restrict__ part_o,
                                                                   const float *__restrict__ part_ml,
                                                                   void *__restrict__ O, long rows, int splits, int d,
                                                                   const RefreshArgs refresh)
{
    if ((int)blockIdx.x >= refresh.first_wg) {             // workgroup-uniform: these only copy
        refresh_cache_rows(refresh);
        return;
    }
    combine_rows<OUT_BF16>(part_o, part_ml, O, rows, splits, d);
}

}  // namespace

void fill_kernel_args(const AttnArgs &a, AttnKernelArgs &k, int rows_per_wg, int key_tile)
{
    k.Q = a.Q; k.K = a.K; k.V = a.V; k.Kblk = a.Kblk; k.Vblk = a.Vblk; k.O = a.O;
    k.q_scale = a.q_scale; k.k_scale = a.k_scale; k.v_scale = a.v_scale;
    k.q_mx = a.q_mx; k.k_mx = a.k_mx; k.v_mx = a.v_mx;
    k.B = a.B; k.H = a.H; k.Hkv = a.Hkv; k.Nq = a.Nq; k.N = a.N;
    k.kv_stride = a.kv_stride > 0 ? a.kv_stride : a.N;
    k.group = a.H / a.Hkv;
    k.rows_per_wg = rows_per_wg;
    k.row_tiles = (k.group * a.Nq + rows_per_wg - 1) / rows_per_wg;
    k.splits = a.splits;
    int per = (a.N + a.splits - 1) / a.splits;
    per = (per + key_tile - 1) / key_tile * key_tile;
    k.keys_per_split = per;
    // drop trailing splits that would be empty after rounding the split length up to whole tiles
    k.splits = (a.N + per - 1) / per;
    k.block_start = a.block_start; k.block_len = a.block_len;
    k.block_starts = a.block_starts;
    k.scale_log2 = 1.44269504088896340736f / sqrtf((float)a.d);
    const size_t rows = (size_t)a.B * a.H * a.Nq;
    k.part_o = static_cast<float *>(a.workspace);
    k.part_ml = k.part_o ? k.part_o + rows * (size_t)k.splits * a.d : nullptr;
}

hipError_t launch_attention_mfma(const AttnArgs &a, hipStream_t stream)
{
    AttnKernelArgs k;
    const bool fp8 = a.qk_dtype == 2;
    const bool blk = a.Nq != a.N || a.Kblk != nullptr || a.splits > 1;   // drafter form of the call
    fill_kernel_args(a, k, blk && a.Nq != a.N ? attn_block_rows_per_wg(a.Nq, a.B, a.H, a.Hkv) : kRowsPerWG, TK);
    const long blocks = (long)a.B * a.Hkv * k.row_tiles * k.splits;
    const dim3 grid((unsigned)blocks), block(kAttnThreads);
    if (a.Kblk == nullptr) k.block_len = 0;                                // no row is taken from block tensors
    hipError_t e;
    if (a.q_mx != nullptr) {
        // block-scaled inputs, verifier form
        if (blk || a.k_mx == nullptr || a.v_mx == nullptr) return hipErrorInvalidValue;
        return a.d == 128 ? launch(attn_mfma_kernel<128, true, false, false, true>, grid, block, stream, k)
                          : launch(attn_mfma_kernel<64, true, false, false, true>, grid, block, stream, k);
    }
    if (a.v_dtype == 2) {
        // fp8 V (with fp8 Q/K): this file's kernel serves every shape of the workload
        if (!blk) return a.d == 128 ? launch(attn_mfma_kernel<128, true, false, true>, grid, block, stream, k)
                                    : launch(attn_mfma_kernel<64, true, false, true>, grid, block, stream, k);
        e = a.d == 128 ? launch(attn_mfma_kernel<128, true, true, true>, grid, block, stream, k)
                       : launch(attn_mfma_kernel<64, true, true, true>, grid, block, stream, k);
        return e != hipSuccess ? e : finish_attention(a, k.splits, stream);
    }
    if (!blk && (!fp8 || a.d == 128)) {
        // The wide-wave kernel (256 query rows per workgroup, one wave per SIMD; bf16, or fp8 Q/K with
        // d = 128) wins once there are enough row tiles to occupy the chip; below that smaller workgroups
        // spread better.
        const long tiles = (long)a.B * a.Hkv * (((long)(a.H / a.Hkv) * a.Nq + 255) / 256);
        const bool wide = tune("DD_TUNE_ATTN_WIDE", tiles >= 192 && a.N >= 512) != 0;
        if (wide && a.N >= 64) return launch_attention_wide(a, stream);   // its K/V tiles are 64 whole rows
        // A small bf16 call leaves most compute units idle with 128-row workgroups: the streaming kernel's
        // 64-row workgroups (two row blocks x two key phases) spread it over more of them.
        const bool small = tune("DD_TUNE_BIDIR_STREAM", blocks < 256) != 0;
        if (small && !fp8) return launch_attention_stream(a, stream);
    }
    if (blk && !fp8 && a.Nq != a.N && attn_stream_fits(a)) {
        // The drafter's call is bound by streaming K/V once: a kernel built around the memory pipeline
        // serves it.
        if (tune("DD_TUNE_BLOCK_STREAM", 1) != 0) return launch_attention_stream(a, stream);
    }
    if (!blk) {
        if (a.d == 128) e = fp8 ? launch(attn_mfma_kernel<128, true, false>, grid, block, stream, k)
                                : launch(attn_mfma_kernel<128, false, false>, grid, block, stream, k);
        else            e = fp8 ? launch(attn_mfma_kernel<64, true, false>, grid, block, stream, k)
                                : launch(attn_mfma_kernel<64, false, false>, grid, block, stream, k);
        return e;
    }
    if (a.d == 128) e = fp8 ? launch(attn_mfma_kernel<128, true, true>, grid, block, stream, k)
                            : launch(attn_mfma_kernel<128, false, true>, grid, block, stream, k);
    else            e = fp8 ? launch(attn_mfma_kernel<64, true, true>, grid, block, stream, k)
                            : launch(attn_mfma_kernel<64, false, true>, grid, block, stream, k);
    return e != hipSuccess ? e : finish_attention(a, k.splits, stream);
}

static int elem_bytes(int dtype) { return dtype == 0 ? 4 : dtype == 1 ? 2 : 1; }

// merge workgroups first (none when the key range was not split), then the copying ones
static hipError_t launch_combine_refresh(const AttnArgs &a, bool merge, hipStream_t stream)
{
    const long rows = merge ? (long)a.B * a.H * a.Nq : 0;
    const float *po = static_cast<const float *>(a.workspace);
    const float *pml = merge ? po + (size_t)rows * a.splits * a.d : nullptr;
    const long threads = rows * (a.d / 4);
    const long merge_wgs = (threads + 255) / 256;
    RefreshArgs r{};
    r.first_wg = (int)merge_wgs;
    long copy_wgs = 0;
    if (a.K_refresh != nullptr) {
        const int eb[2] = {elem_bytes(a.qk_dtype), elem_bytes(a.v_dtype)};
        r.src[0] = static_cast<const uint4 *>(a.Kblk); r.src[1] = static_cast<const uint4 *>(a.Vblk);
        r.dst[0] = static_cast<uint4 *>(a.K_refresh);  r.dst[1] = static_cast<uint4 *>(a.V_refresh);
        int most = 0;
        for (int w = 0; w < 2; ++w) {
            const long row_chunks = (long)a.d * eb[w] / 16;            // d is 64 or 128: whole chunks
            r.per_bh[w] = (int)(a.block_len * row_chunks);             // block_len <= N < 2^31 / 32
            r.bh_stride[w] = (long)(a.kv_stride > 0 ? a.kv_stride : a.N) * row_chunks;
            r.offset[w] = (long)a.block_start * row_chunks;
            most = r.per_bh[w] > most ? r.per_bh[w] : most;
        }
        const long nbh = (long)a.B * a.Hkv;
        long per = (most + 255) / 256;                                 // one K and one V chunk per lane ...
        const long cap = nbh >= 2048 ? 1 : 2048 / nbh;                 // ... or a few each
        r.wgs_per_bh = (int)(per < cap ? per : cap);
        copy_wgs = nbh * r.wgs_per_bh;
    }
    if (merge_wgs + copy_wgs == 0) return hipSuccess;
    const dim3 grid((unsigned)(merge_wgs + copy_wgs)), block(256);
    if (copy_wgs == 0) {
        if (a.v_dtype != 0)                 // bf16 output (V bf16 or fp8)
            return launch(attn_combine_kernel<true>, grid, block, stream, po, pml, a.O, rows, a.splits, a.d);
        return launch(attn_combine_kernel<false>, grid, block, stream, po, pml, a.O, rows, a.splits, a.d);
    }
    if (a.v_dtype != 0)                 // bf16 output (V bf16 or fp8)
        return launch(attn_combine_refresh_kernel<true>, grid, block, stream, po, pml, a.O, rows, a.splits, a.d, r);
    return launch(attn_combine_refresh_kernel<false>, grid, block, stream, po, pml, a.O, rows, a.splits, a.d, r);
}

hipError_t launch_attention_combine(const AttnArgs &a, hipStream_t stream)
{
    return launch_combine_refresh(a, true, stream);
}

hipError_t finish_attention(const AttnArgs &a, int splits_used, hipStream_t stream)
{
    if (splits_used > 1) {
        AttnArgs c = a;
        c.splits = splits_used;
        return launch_combine_refresh(c, true, stream);
    }
    return a.K_refresh != nullptr ? launch_combine_refresh(a, false, stream) : hipSuccess;
}

}  // namespace dd
