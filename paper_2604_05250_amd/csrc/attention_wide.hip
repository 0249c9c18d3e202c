// Verifier attention, wide-wave form (bf16, or fp8 e4m3 Q/K with bf16 V):  O = softmax(Q K^T / sqrt(d_k)) V over all positions
// (Eq. 3 applied bidirectionally, Sec. 2.2) -- the O(N^2)-per-step cost of a masked diffusion model.
//
// Why a second kernel.  With 32 query rows per wave every matrix-core instruction needs its own 1 KB
// operand fragment from LDS, twice the fragment reads (and, with two workgroups per compute unit, twice the
// tile loads) of this form; measured on a drafter call, two such waves per SIMD are slower than the one below.
// Here one wave owns 64 query rows (two 32-row blocks) and is alone on its SIMD (up to 512 registers);
// one workgroup = 4 waves = 256 query rows of one (batch, kv head).  Every K fragment and every V
// fragment read from LDS feeds two MFMAs (one per block): half the LDS bytes per FLOP.
//
// A single wave per SIMD has no other wave to overlap with, and a wave issues in order, one instruction
// per ~4 cycles whatever its kind: a matrix instruction (32 cycles of matrix-core time) only overlaps with
// the handful of instructions that directly follow it.  Each pipeline step (one 32-key unit u) is therefore
// a fixed sequence of "pieces" = one MFMA + its share of everything else, and what counts is the number of
// instructions per piece:
//     matrix cores   S(u+1) = K(u+1) Q^T,   O^T += V(u-1)^T P(u-1)^T,   l += 1^T P(u-1)^T (row sums)
//     vector ALUs    row maxima of S(u), then P(u) = 2^(S(u) c - m), packed to bf16
//     memory         LDS fragment reads three uses ahead, one global->LDS tile load per piece
// Whether a score exceeds the maximum in use (by more than 2^8) is one comparison per row block against a
// threshold in raw score units; raising the maximum and rescaling the accumulators are rare branches.
//
// Register files.  S lives in architectural VGPRs (the vector ALUs cannot read accumulation VGPRs and a
// copy costs as much as two FMAs and does not overlap with the matrix cores); O, the row sums and the Q
// fragments live in accumulation VGPRs, which the matrix cores read directly.  The compiler picks one
// register file for all MFMA results of a function, so the S = K Q^T instructions are written as inline
// assembly.  The hazards the compiler would otherwise pad are kept apart by construction: a score block
// is written by the first half of step u's MFMAs and first read by a vector instruction in step u+1.
//
// Persistence.  A lone wave cannot hide the start (operand loads, pipeline fill) and the end (normalise,
// store) of a row tile behind another workgroup's work, so a workgroup walks through every G-th row
// tile (G workgroups) and the K/V tile stream simply wraps into the next row tile: the two surplus steps that drain
// one tile's pipeline compute the first two score blocks of the next.  The next tile's Q rows are
// prefetched into LDS one stage earlier; the finished tile is normalised, transposed through the same
// LDS region and written out in full rows.
//
// Staging.  K and V tiles (64 keys) are double-buffered in four LDS arrays and filled by
// global_load_lds_dwordx4 (no registers, no LDS store instructions).  A tile always holds 64 whole rows -
// the last one of a pass overlaps its predecessor and the repeated keys score -inf - so a load's address is
// "scalar tile base + constant lane offset + immediate" with no vector arithmetic; the loads are written
// as assembly to keep that form, and every wait for them is explicit (only the barrier that ends a stage
// waits, and it lets the requests issued after the tile loads stay in flight).
// K is XOR-swizzled for its 16-byte operand reads; V stays row-major (swizzled in 64-byte granules) and
// its transposed operand comes from ds_read_b64_tr_b16 (lane j of a 16-lane group receives column j of
// the 4-row x 16-column block whose row r is addressed by lanes 4r..4r+3).
//
// Measured on MI355X: with realistic operand data the matrix cores are power-limited (a register-only
// MFMA loop runs at about 1.65 GHz and 1.75 PFLOP/s on all 256 CUs, against 2.2 GHz with constant
// operands), and so is this kernel: instructions removed from the pieces come back partly as a lower clock.
#include "attention_common.h"
#include "dd_internal.h"

#include <type_traits>

namespace dd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef int intx8 __attribute__((ext_vector_type(8)));

constexpr int TKW = 64;                 // keys per tile
constexpr int kRowsWGWide = 256;        // query rows per workgroup: four waves of two 32-row blocks each ...
constexpr int kRowsWGNarrow = 128;      // ... or of one (the drafter's form when that spares it the key splits)
[[maybe_unused]] constexpr int kPackLag = 2;             // pieces between an exponential and its conversion to bf16
[[maybe_unused]] constexpr float kSlack = 8.0f;         // the maximum in use is raised when exceeded by 2^8
constexpr int kFoldMinKeys = 1024;      // key rows from which scaling Q once per row tile pays (see FOLD below)
[[maybe_unused]] constexpr float kFoldMargin = 7.0f;    // folded form: the reference is set this far above a unit's maximum (log2 units)

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
    return __uint_as_float(r.x) > __uint_as_float(r.y) ? __uint_as_float(r.x) : __uint_as_float(r.y);
}
// Maxima as single instructions: fmaxf() on values the compiler cannot prove canonical (results of inline
// assembly, lane swaps) costs an extra instruction per operand.
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// S = K Q^T step with the result in architectural VGPRs and the Q fragment read from accumulation VGPRs.
// bf16: 8 values per lane and operand (16 bytes), 16 head dims per instruction.  fp8 e4m3: 32 values per lane and
// operand (32 bytes), 64 head dims per instruction - the only fp8 matrix instruction that runs at twice the bf16
// rate (64 cycles for four times the products; the 32x32x16 fp8 one takes the 32 cycles of its bf16 twin).  Any
// assignment of head dims to the bytes of the operands will do as long as K and Q use the same.
template <bool FP8, typename KT, typename QT>
__device__ __forceinline__ void qk_first(floatx16 &s, const KT kf, const QT qfrag)
{
    if constexpr (FP8) asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0" : "=&v"(s) : "v"(kf), "a"(qfrag));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(kf), "a"(qfrag));
}
// the same from an addend: the block starts from `init` (minus the softmax reference of its query rows)
template <typename KT, typename QT>
__device__ __forceinline__ void qk_first_from(floatx16 &s, const KT kf, const QT qfrag, const floatx16 &init)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(s) : "v"(kf), "a"(qfrag), "v"(init));
}
template <bool FP8, typename KT, typename QT>
__device__ __forceinline__ void qk_next(floatx16 &s, const KT kf, const QT qfrag)
{
    if constexpr (FP8) asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+v"(s) : "v"(kf), "a"(qfrag));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(kf), "a"(qfrag));
}

// A wave-uniform pointer that the compiler happens to hold in vector registers, as a scalar register pair
// (a no-op when it already is one).
__device__ __forceinline__ const uint8_t *scalar_ptr(const uint8_t *p)
{
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return reinterpret_cast<const uint8_t *>(((unsigned long long)hi << 32) | lo);
}

// s_waitcnt immediate: wait until at most n vector-memory operations are outstanding, nothing else
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

template <int N> using I_ = std::integral_constant<int, N>;
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(I_<I>{});
        static_for<N, I + 1>(f);
    }
}
using T_ = std::true_type;
using F_ = std::false_type;

// FP8: Q and K are fp8 e4m3 (with per-head scales folded into the exponent's factor), V and O bf16.
// BLOCK: the drafter's form of the call (Sec. 2.3) - the rows are the active block's queries, the key stream
// is cache rows [0, block_start), the block tensors' rows, cache rows [block_start + block_len, N) (each
// part tiled by the same rule of 64-row windows with a valid range), a workgroup takes one row tile and one of `splits` ranges of the tile list, and
// with splits > 1 writes its unnormalised state for the merge kernel instead of O.
// FOLD (bf16 Q/K without per-head scales, key ranges of kFoldMinKeys rows or more): the factor
// c = log2(e)/sqrt(d_k) is multiplied into the Q fragments once per row tile (rounded to bf16 again; this second
// rounding perturbs a score by about 2^-10 of the typical score magnitude, as much as the bf16 rounding of the
// weights does), and every score block starts from minus the softmax reference m of its query rows instead of
// from zero - the first matrix instruction of a block takes -m, held in sixteen registers per row block, as its
// addend - so the matrix cores deliver S' = c q.k - m and the weight of a key is exp2(S') with no other
// arithmetic per score.  The reference only has to be NEAR the running maximum (weights and sums are floating
// point, any common factor 2^-m cancels in O = sum(P v) / sum(P)): it is set to the maximum of a row tile's
// first unit plus a margin, and raised when some weight reaches 2, which shows as one bit of its bf16 pattern -
// the packed weights are or-ed together as they are produced (one instruction per four scores) and tested once
// per unit.  Scaling Q costs some 1600 cycles per row tile and wave; measured against the row-maximum form
// below, the call is 5 % faster at 4096 keys and 3 % at 1024.  (Tried: the reference refilled into the score
// registers by LDS reads instead of kept in registers - half the gain; the same mechanism without the folded
// scale, one multiplication per score - slower than the row-maximum form, which therefore stays for fp8 and
// per-head scales.)
// QB: 32-row query blocks per wave.  2 is the form described above; 1 (the drafter's call only) halves the row
// tile to 128 rows - every K and V fragment then feeds one matrix instruction instead of two, but twice as many
// workgroups share the call, which can spare it the key splits, their partial states and the merge launch.
template <int D, bool FP8, bool BLOCK, bool FOLD = false, int QB = 2>
__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_wide_kernel(const AttnKernelArgs a)
{
    // The body exists in the device pass only.  The host pass needs the kernel's handle, not its code, and, given
    // lambdas whose parameter types depend on a template parameter around assembly it cannot check, it was seen to
    // drop the handle without a diagnostic: the library then fails to load with an undefined symbol.
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(!(FOLD && FP8), "the scale cannot be folded into fp8 operands");
    static_assert(QB == 2 || (QB == 1 && BLOCK), "one or two row blocks per wave");
    constexpr int kRowsWave = 32 * QB, kRowsWG = 4 * kRowsWave;
    constexpr int NE = 16 * QB;                      // scores per lane and unit
    constexpr int CH = D / 8;                        // 16-byte chunks (8 bf16) per V / O row
    static_assert(!FP8 || D % 64 == 0, "an fp8 matrix instruction takes 64 head dims");
    constexpr int KS = FP8 ? D / 64 : D / 16;        // S = K Q^T: matrix instructions per 32-key unit and row block
    constexpr int DC = D / 32;                       // 32-wide chunks of the head dim
    constexpr int ROWB = D * 2;                      // bytes per V / O row
    constexpr int KROWB = FP8 ? D : 2 * D;           // bytes per Q / K row
    constexpr int KCH = KROWB / 16;                  // 16-byte chunks per Q / K row
    constexpr int KF = KROWB / 32;                   // 16-byte fragments per lane and Q / K row; an instruction takes ...
    constexpr int FPM = KF / KS;                     // ... this many of them (bf16 1, fp8 2)
    static_assert(FPM == (FP8 ? 2 : 1), "operand widths");
    constexpr int DMA_ROWS = 1024 / ROWB;            // rows moved by one wave-wide 16-byte-per-lane load (V)
    constexpr int KDMA_ROWS = 1024 / KROWB;          // ... (Q, K)
    constexpr int NDMA = TKW / DMA_ROWS / 4;         // such loads per wave per V tile
    constexpr int NDMA_K = TKW / KDMA_ROWS / 4;      // ... per K tile
    constexpr int NQDMA = kRowsWave / KDMA_ROWS;     // ... per wave for its Q rows
    constexpr int NQK = KS * QB;                     // pieces of a step: S(u+1) ...
    constexpr int NPV = 2 * DC * QB;                 // ... O += V P ...
    constexpr int NP = NQK + NPV + 2 * QB;           // ... and the row sums
    constexpr int MAXC = FOLD ? 0 : NP >= 32 ? 8 : 4;   // pieces that carry the row maxima
    constexpr int CHK = NP - 6;                      // FOLD: the piece that tests the unit's weights, after the last pack ...
    constexpr int EXC = FOLD ? CHK - kPackLag : NP - MAXC;   // pieces that carry the 32 exponentials
    constexpr int RD = 3;                            // fragment rings: fetched RD uses (2 RD MFMAs) ahead
    static_assert(NDMA_K + NDMA + 1 <= NP, "one tile load per piece");
    static_assert(FOLD || 16 % (2 * MAXC) == 0, "whole pairs of scores per maximum piece");
    static_assert(KF >= RD && 2 * DC >= RD, "fragment rings are three deep");
    static_assert((4 * DMA_ROWS) % 8 == 0 && DMA_ROWS <= 8, "swizzle phase must not depend on the load index");
    static_assert((4 * KDMA_ROWS) % 8 == 0 && KDMA_ROWS <= 8, "swizzle phase must not depend on the load index");

    __shared__ __attribute__((aligned(4096))) uint4 K0[TKW * KCH], K1[TKW * KCH];   // [key][chunk ^ (key & 7)]
    __shared__ __attribute__((aligned(4096))) uint4 V0[TKW * CH], V1[TKW * CH];     // [key][chunk ^ ((key % (CH/4)) << 2)]  (row-major, 64-byte granules)
    // Per wave: the next tile's 64 Q rows [row][chunk ^ (row & 7)], later the finished tile's O rows on
    // their way out, in rows of OPITCH bytes (8 bytes of padding rotate the banks from row to row).
    constexpr int OPITCH = ROWB + 8;
    constexpr int QOW = kRowsWave * OPITCH;          // bytes per wave
    static_assert(QOW % 16 == 0, "wave regions stay 16-byte aligned");
    __shared__ uint4 QO[4 * QOW / 16];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;

    // ---- this workgroup's row tiles.  Tile t = ((b * Hkv + kvh) * row_tiles + rt); workgroup w takes tiles
    // w, w + G, w + 2G ...: at any time the G workgroups are on consecutive tiles, so neighbours work on the
    // same K/V, and neighbours are placed on the same XCD (own L2 each).
    const int tiles_total = a.B * a.Hkv * a.row_tiles;
    int t_stride = gridDim.x;
    int t_cur, split = 0;
    {
        const int G = gridDim.x, per = G >> 3, rem = G & 7;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        t_cur = xcd * per + min(xcd, rem) + slot;
    }
    if (BLOCK) {                                     // one (row tile, key split) per workgroup, no second tile
        split = t_cur % a.splits;
        t_cur /= a.splits;
        t_stride = tiles_total;
    }
    const int rows_total = a.group * a.Nq;           // query rows per (batch, kv head); contiguous in memory
    const int nkeys = a.N;
    // Key stream as a list of 64-row tiles.  Not BLOCK: one part, rows [0, N).  BLOCK: up to three parts - cache
    // rows [0, lo), block-tensor rows [lo - bs, hi - bs), cache rows [hi, N), where [lo, hi) = [bs, bs + block_len)
    // cut to the sequence and bs is the block's first row: the call's, or this batch entry's own (any value).
    int blk_lo = 0, blk_hi = 0, blk_first = 0;       // rows [lo, hi) come from the block tensors, from their row blk_first on
    if (BLOCK && a.block_len) {
        const int bsel = a.block_starts ? a.block_starts[(t_cur / a.row_tiles) / a.Hkv] : a.block_start;
        const long s0 = bsel, s1 = (long)bsel + a.block_len;
        blk_lo = (int)(s0 < 0 ? 0 : s0 > nkeys ? nkeys : s0);
        blk_hi = (int)(s1 < 0 ? 0 : s1 > nkeys ? nkeys : s1);
        blk_first = (int)(blk_lo - s0);              // 0 <= blk_first <= block_len whenever the part is not empty
        if (blk_hi <= blk_lo) blk_first = 0;
    }
    const int len_a = BLOCK && a.block_len ? blk_lo : nkeys;
    const int len_b = BLOCK ? blk_hi - blk_lo : 0;
    const int len_c = BLOCK && a.block_len ? nkeys - blk_hi : 0;
    const int nt_a = (len_a + TKW - 1) / TKW, nt_b = (len_b + TKW - 1) / TKW, nt_c = (len_c + TKW - 1) / TKW;
    const int nt_all = nt_a + nt_b + nt_c;
    const int nt_per_split = BLOCK ? (nt_all + a.splits - 1) / a.splits : nt_all;
    const int t_first = split * nt_per_split;                               // this workgroup's tiles of the list
    const int nt_local = min(nt_all, t_first + nt_per_split) - t_first;
    const int nt_even = (nt_local + 1) & ~1;         // tiles per pass, padded to an even count
    struct Tile { const uint8_t *k, *v, *kb, *vb; size_t row_base; int v0, bh0, kvs; };
    auto tile_of = [&](int t) __attribute__((always_inline)) {
        const int rt = t % a.row_tiles, bk = t / a.row_tiles, kvh = bk % a.Hkv, b = bk / a.Hkv;
        Tile r;
        r.k = static_cast<const uint8_t *>(a.K) + (size_t)bk * a.kv_stride * (size_t)KROWB;
        r.v = static_cast<const uint8_t *>(a.V) + (size_t)bk * a.kv_stride * (size_t)ROWB;
        r.kb = r.vb = nullptr;
        if (BLOCK && a.block_len) {
            r.kb = static_cast<const uint8_t *>(a.Kblk) + (size_t)bk * a.block_len * (size_t)KROWB;
            r.vb = static_cast<const uint8_t *>(a.Vblk) + (size_t)bk * a.block_len * (size_t)ROWB;
        }
        r.bh0 = b * a.H + kvh * a.group;             // first query head of the group
        r.row_base = (size_t)r.bh0 * a.Nq;           // row of virtual row 0 in Q and O
        r.v0 = rt * kRowsWG;                     // first virtual row of the tile
        r.kvs = bk;                                  // index into k_scale
        return r;
    };

    // ---- staging by LDS DMA: load i of this wave moves rows (4i + wave) * DMA_ROWS .. of a tile; lane l
    // lands at chunk position l % CH of row l / CH and therefore fetches the chunk the swizzle maps there.
    // Both swizzles only depend on the row modulo 4 DMA_ROWS, so the chunk a lane fetches is the same for
    // every load, and a tile has the same row pitch in LDS as in memory: load i differs from load 0 by the
    // same 4096 i bytes on both sides, which is what the instruction's immediate offset adds.  Its range is
    // +-4 KB, so loads pair up around bases 4 KB and 12 KB into the tile.  All address arithmetic per load
    // is then scalar.
    // A tile always holds 64 valid rows: tile T covers rows a(T) = min(64 T, N - 64) .. a(T) + 63, and the
    // rows before 64 T (already seen in the previous tile, or all of them for a tile past the end) are
    // masked in the scores.
    auto lds_addr = [](const void *p) __attribute__((always_inline)) {
        return (unsigned)(size_t)(__attribute__((address_space(3))) const void *)p;
    };
    const int dma_row0 = wave * DMA_ROWS + lane / CH;                      // row of load 0; load i: + 4 i DMA_ROWS
    const int dma_krow0 = wave * KDMA_ROWS + lane / KCH;
    const unsigned dma_koff = dma_krow0 * KROWB + ((lane % KCH) ^ (dma_krow0 & 7)) * 16;
    const unsigned dma_voff = dma_row0 * ROWB + ((lane % CH) ^ ((dma_row0 & (CH / 4 - 1)) << 2)) * 16;
    // Tile `tile` of this workgroup's pass: where its 64 rows start in memory (K and V side), and which of them
    // count: rows [vlo, vhi) of the tile.  A tile is always 64 whole rows of its source (the cache, or the block
    // tensors): the window is pushed back into the source where the nominal rows 64 T .. of the part would hang
    // over its end, so a last tile repeats rows of its predecessor, and the tile of a part shorter than 64 rows
    // holds rows of the neighbouring part as well - all of those are masked in the scores, as is every row of a
    // stand-in tile past the end of the pass.  All of it is scalar arithmetic.
    struct TileAt { const uint8_t *k, *v; int vlo, vhi; };
    auto tile_at = [&](const Tile &t, int tile) __attribute__((always_inline)) {
        // (every captured value is copied before any choice is made between them: the compiler otherwise
        // turns "choose one of several loaded values" into a load through a chosen address, which pins the
        // captured variables in scratch memory)
        const int la = len_a, lb = len_b, lc = len_c, na = nt_a, nb = nt_b, nl = nt_local, tf = t_first;
        const int c_row0 = blk_hi, b_row0 = blk_first, nk = nkeys, bl = a.block_len;
        const uint8_t *const ck = t.k, *const cv = t.v, *const bk = t.kb, *const bv = t.vb;
        const bool standin = tile >= nl;
        int T = tf + min(tile, nl - 1);                                      // position in the list
        const bool in_c = BLOCK && T >= na + nb, in_b = BLOCK && !in_c && T >= na;
        T -= in_c ? na + nb : in_b ? na : 0;                                 // position in its part
        const int len = in_c ? lc : in_b ? lb : la;                          // rows of the part
        const int off = in_c ? c_row0 : in_b ? b_row0 : 0;                   // its first row in its source
        const int src_rows = in_b ? bl : nk;                                 // rows of the source (>= 64: the launcher checks)
        const uint8_t *kp = in_b ? bk : ck, *vp = in_b ? bv : cv;
        const int first = off + T * TKW;                                     // nominal first row of the tile
        const int win = min(first, src_rows - TKW);                          // first row actually loaded
        TileAt r;
        r.k = kp + (size_t)win * KROWB;
        r.v = vp + (size_t)win * ROWB;
        r.vlo = standin ? TKW : first - win;
        r.vhi = standin ? TKW : off + min(T * TKW + TKW, len) - win;
        return r;
    };
    // one load (index i) of the tile whose first row is at `glob`
    auto dma_one = [&](uint4 *dst, const uint8_t *glob, unsigned lane_off, int i) __attribute__((always_inline)) {
        static_assert(4 * DMA_ROWS * ROWB == 4096 && 4 * KDMA_ROWS * KROWB == 4096, "loads of a wave are 4 KB apart");
        const int mid = 4096 + 8192 * (i >> 1);
        const uint8_t *sbase = scalar_ptr(glob + mid);                     // uniform: a scalar register pair
        const unsigned d = lds_addr(dst) + wave * 1024 + mid;
        // Written as assembly so that the address stays "scalar base + 32-bit lane offset + immediate" (the
        // compiler prefers to carry a 64-bit address per lane and per load).  It therefore knows nothing of
        // these loads: every wait for them in this kernel is explicit.
        if (i & 1)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(d), "v"(lane_off), "s"(sbase) : "memory", "m0");
        else
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 offset:-4096" : : "s"(d), "v"(lane_off), "s"(sbase) : "memory", "m0");
    };
    // Wait until at most `pending` of this wave's memory operations are outstanding, then meet the other
    // waves.  (The barrier by itself is no fence for the compiler: the empty statements keep it from
    // moving LDS accesses across.)
    auto wait_loads_and_sync = [&](auto pending) __attribute__((always_inline)) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(decltype(pending)::value));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto dma_tile = [&](uint4 *dst, const uint8_t *glob, unsigned lane_off, auto n) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < decltype(n)::value; ++i) dma_one(dst, glob, lane_off, i);
    };
    // this wave's 64 query rows of a tile -> its region of QO (rows past the end repeat the last one)
    auto dma_q = [&](const Tile &t) __attribute__((always_inline)) {
        const uint8_t *qg = static_cast<const uint8_t *>(a.Q) + (t.row_base + t.v0 + wave * kRowsWave) * KROWB;
        const unsigned dst = lds_addr(QO) + wave * QOW;
        // Rarely executed code derives its per-lane values from an opaque copy of the lane number: otherwise
        // they are all computed once at kernel start and occupy registers (or scratch) throughout.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int drow = ln / KCH, dpos = ln % KCH;
        if (__builtin_expect(t.v0 + kRowsWG <= rows_total, 1)) {
            // whole tile: 1 KB per load, contiguous on both sides - scalar bases 8 KB apart and immediates;
            // the chunk a lane fetches depends on the row modulo 8, hence on the parity of a 4-row load
            unsigned off[2];
#pragma unroll
            for (int par = 0; par < 2; ++par)
                off[par] = drow * KROWB + (dpos ^ ((par * KDMA_ROWS + drow) & 7)) * 16;
            static_for<NQDMA>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value, mid = 4096 + 8192 * (i / 8), imm = i * 1024 - mid;
                const uint8_t *sbase = scalar_ptr(qg + mid);
                const unsigned d = dst + mid, o = off[(i * KDMA_ROWS / 4) & 1];
                if constexpr (imm >= 0)
                    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                                 : : "s"(d), "v"(o), "s"(sbase), "n"(imm) : "memory", "m0");
                else
                    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 offset:-%3"
                                 : : "s"(d), "v"(o), "s"(sbase), "n"(-imm) : "memory", "m0");
            });
        } else {
#pragma unroll
            for (int i = 0; i < NQDMA; ++i) {
                const int row = min(i * KDMA_ROWS + drow, rows_total - 1 - t.v0 - wave * kRowsWave);
                const uint8_t *src = qg + (ptrdiff_t)row * KROWB + (dpos ^ ((i * KDMA_ROWS + drow) & 7)) * 16;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst + i * 1024), "v"(src) : "memory", "m0");
            }
        }
    };
    auto kbuf = [&](auto p) __attribute__((always_inline)) -> uint4 * { if constexpr (decltype(p)::value == 0) return K0; else return K1; };
    auto vbuf = [&](auto p) __attribute__((always_inline)) -> uint4 * { if constexpr (decltype(p)::value == 0) return V0; else return V1; };

    // ---- per-lane state of the two query blocks
    float c[QB], c_next[QB];                         // scores are exponentiated as 2^(s*c); the next row tile's factor
    using qfrag_t = std::conditional_t<FP8, intx8, intx4>;
    qfrag_t qf[QB][KS];                              // B operands of S^T = K Q^T (one per instruction), kept in accumulation VGPRs
    // O^T (unnormalised), and the row sums of the weights.  The sums come from a 16x16x32 matrix instruction (half the
    // matrix-core time of the 32x32x16 one) that takes the weights' B fragment as it is.  Read as that instruction's
    // 16 x 32 B operand, lane l (column l % 16, k = 8 (l / 16) ..) holds, for column n: k 0-7 and 16-23 = the sixteen
    // keys of row n, k 8-15 and 24-31 = those of row n + 16.  An A operand whose row 0 is one on the first kind of k and
    // whose row 1 is one on the second (all else zero) therefore gives C[0][n] = sum of row n, C[1][n] = sum of row
    // n + 16: lane n < 16 holds them in registers 0 and 1, every other lane and register holds zero.
    floatx16 acc[QB][DC];
    floatx4 acc_l[QB];
    auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < QB; ++q) {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc_l[q][r] = 0.f;
#pragma unroll
            for (int i = 0; i < DC; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[q][i][r] = 0.f;
        }
    };
    clear_acc();
    // The same between two row tiles: ten matrix instructions with zero operands instead of 160 register
    // writes (written as assembly: the results stay in accumulation VGPRs and are next read, as the addend
    // of a matrix instruction, a whole step later).
    auto clear_acc_mfma = [&]() __attribute__((always_inline)) {
        intx4 z = {0, 0, 0, 0};
        asm volatile("s_nop 3" : "+v"(z));                   // the zeros are in place before a matrix instruction reads them
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %1, 0" : "=a"(acc_l[q]) : "v"(z));
#pragma unroll
            for (int i = 0; i < DC; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(acc[q][i]) : "v"(z));
        }
    };
    float mc[QB];                                    // maximum (FOLD: reference) in use, log2 units, equal in both lane halves
    float thr[QB];                                   // raw scores above (mc + slack) / c raise the maximum in use
    float mc_done[QB];                               // the finished tile's maximum in use (BLOCK: part of its state)
#pragma unroll
    for (int q = 0; q < QB; ++q) {
        mc[q] = FOLD ? 0.f : -INFINITY;
        thr[q] = mc_done[q] = -INFINITY;
    }
    bool ref_unset = false;                          // FOLD: a row tile has begun with wholly masked units, no reference yet (uniform)
    unsigned seen0 = 0u;                             // ... what the or of a unit's weights starts from: the tested bit while that is so
    floatx16 cinit[QB];                              // FOLD: what a score block starts from: -mc in all 16 registers
    if constexpr (FOLD) {
#pragma unroll
        for (int q = 0; q < QB; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) cinit[q][r] = 0.f;
    }
    // A operand of the row-sum instruction (see acc_l): lane l holds A[l % 16][8 (l / 16) .. + 7]
    const int lsel_on = (lane == 0 || lane == 32 || lane == 17 || lane == 49) ? 0x3F803F80 : 0;   // bf16 1.0 twice, or zero
    intx4 ones = {lsel_on, lsel_on, lsel_on, lsel_on};
    asm volatile("" : "+v"(ones));                   // held in registers instead of being rebuilt per use
    // the sum of this lane's row (l32) of row block q: from lane l32 % 16, register l32 / 16 (every lane must call it)
    auto row_sum = [&](int q) __attribute__((always_inline)) {
        const float lo = __shfl(acc_l[q][0], lane & 15), hi = __shfl(acc_l[q][1], lane & 15);
        return (lane & 16) ? hi : lo;
    };

    // operand addresses inside a tile buffer (bytes), without the unit offset
    int k_off[KF], v_off[DC];
#pragma unroll
    for (int f = 0; f < KF; ++f) k_off[f] = (l32 * KCH + ((2 * f + hh) ^ (l32 & 7))) * 16;
    {
        const int t = lane & 15, gq = l32 >> 4, row = 4 * hh + (t >> 2);
#pragma unroll
        for (int i = 0; i < DC; ++i) {
            const int chunk = 4 * i + 2 * gq + ((t & 3) >> 1);
            v_off[i] = (row * CH + (chunk ^ ((row & (CH / 4 - 1)) << 2))) * 16 + (t & 1) * 8;
        }
    }
    // K fragment f of the unit `sub` (0/1) of a tile buffer: key 32 sub + l32, bytes 32 f + 16 hh .. +15 of its
    // row: bf16 dims 16 f + 8 hh .. +7 (one MFMA); fp8 dims 32 f + 16 hh .. +15 (half of one MFMA's operand: fragments
    // 2 j and 2 j + 1 make up instruction j's - any split of the head dim over instructions, operand bytes and lane
    // halves will do as long as Q uses the same)
    auto k_frag = [&](const uint4 *kb, int sub, int f) __attribute__((always_inline)) {
        return __builtin_bit_cast(intx4, *reinterpret_cast<const uint4 *>(
                   reinterpret_cast<const char *>(kb) + sub * 32 * KROWB + k_off[f]));
    };
    // the A operand of an fp8 instruction out of its two fragments
    auto k_pair = [](const intx4 &f0, const intx4 &f1) __attribute__((always_inline)) {
        return intx8{f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
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
    // Q fragments of a tile out of this wave's quarter of QO (same addressing as a K tile), and its scales
    auto install_q = [&](const Tile &t) __attribute__((always_inline)) {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        intx4 q_half = {0, 0, 0, 0};
#pragma unroll
        for (int q = 0; q < QB; ++q) {
#pragma unroll
            for (int f = 0; f < KF; ++f) {
                // addresses derived from the opaque lane copy: see dma_q
                const int lo = ((ln & 31) * KCH + ((2 * f + (ln >> 5)) ^ (ln & 7))) * 16;
                const intx4 w = __builtin_bit_cast(intx4, *reinterpret_cast<const uint4 *>(
                                    reinterpret_cast<const char *>(QO) + wave * QOW + q * 32 * KROWB + lo));
                if constexpr (FOLD) {
                    // c q, rounded to bf16 once more (two values per register)
                    intx4 ws;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const unsigned u = (unsigned)w[k];
                        ws[k] = (int)pack_bf16_rne(__uint_as_float(u << 16) * a.scale_log2,
                                                   __uint_as_float(u & 0xFFFF0000u) * a.scale_log2);
                    }
                    qf[q][f] = ws;
                    asm volatile("" : "+a"(qf[q][f]));
                } else if constexpr (FP8) {
                    // fragments 2 j and 2 j + 1 are the two halves of instruction j's operand
                    if (f % 2 == 0) q_half = w;
                    else {
                        qf[q][f / 2] = k_pair(q_half, w);
                        asm volatile("" : "+a"(qf[q][f / 2]));
                    }
                } else {
                    qf[q][f] = w;
                    asm volatile("" : "+a"(qf[q][f]));
                }
            }
            const int v = min(t.v0 + wave * kRowsWave + q * 32 + (ln & 31), rows_total - 1);
            c_next[q] = a.scale_log2;                        // takes effect with the tile's first score block
            if (a.q_scale) c_next[q] *= a.q_scale[t.bh0 + v / a.Nq];
            if (a.k_scale) c_next[q] *= a.k_scale[t.kvs];
        }
        // the matrix instructions written as assembly are invisible to the compiler's hazard padding:
        // keep them clear of the register writes above
        asm volatile("s_nop 15" : "+a"(qf[0][0]), "+a"(qf[QB - 1][KS - 1]));
    };
    // Finished tile: normalise, transpose through this wave's region of QO, write whole rows.
    // O^T register r of chunk i holds dim 32 i + 8 (r / 4) + 4 hh + (r % 4) of query row l32 of its block:
    // four consecutive dims = one 8-byte slot (i * 8 + (r / 4) * 2 + hh) of the row.  All addresses are one
    // per-lane base plus constants.
    auto write_out = [&](const Tile &t) __attribute__((always_inline)) {
        char *region = reinterpret_cast<char *>(QO) + wave * QOW;
        int ln = lane;
        asm volatile("" : "+v"(ln));
        if constexpr (BLOCK) {
            if (a.splits > 1) {
                // one of several key ranges: the unnormalised state (O, maximum in use, row sum) goes to the
                // merge kernel, row r of the call at [(r * splits + split)]
#pragma unroll
                for (int q = 0; q < QB; ++q) {
                    const float l_row = row_sum(q);
                    const int v = t.v0 + wave * kRowsWave + q * 32 + (ln & 31);
                    if (v >= rows_total) continue;
                    const size_t slot = (t.row_base + v) * (size_t)a.splits + split;
                    float *po = a.part_o + slot * D + (ln >> 5) * 4;
#pragma unroll
                    for (int i = 0; i < DC; ++i)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4)
                            *reinterpret_cast<float4 *>(po + i * 32 + q4 * 8) =
                                make_float4(acc[q][i][4 * q4], acc[q][i][4 * q4 + 1], acc[q][i][4 * q4 + 2], acc[q][i][4 * q4 + 3]);
                    if ((ln >> 5) == 0) {
                        a.part_ml[slot * 2] = mc_done[q];
                        a.part_ml[slot * 2 + 1] = l_row;
                    }
                }
                return;
            }
        }
        char *wbase = region + (ln & 31) * OPITCH + (ln >> 5) * 8;
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const float inv = __builtin_amdgcn_rcpf(row_sum(q));          // 1 ulp; the result is rounded to bf16
#pragma unroll
            for (int i = 0; i < DC; ++i)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const uint2 w = make_uint2(pack_bf16_rne(acc[q][i][4 * q4] * inv, acc[q][i][4 * q4 + 1] * inv),
                                               pack_bf16_rne(acc[q][i][4 * q4 + 2] * inv, acc[q][i][4 * q4 + 3] * inv));
                    *reinterpret_cast<uint2 *>(wbase + q * 32 * OPITCH + (i * 8 + q4 * 2) * 8) = w;
                }
        }
        constexpr int LPR = ROWB / 16, RPI = 64 / LPR;                     // lanes per row, rows per store
        const int row0 = ln / LPR, ch = ln % LPR;
        const char *rbase = region + row0 * OPITCH + ch * 16;
        const int v_first = t.v0 + wave * kRowsWave;                       // virtual row of the wave's row 0
        uint8_t *og = static_cast<uint8_t *>(a.O) + (t.row_base + v_first) * ROWB;      // uniform
        const unsigned goff = row0 * ROWB + ch * 16;
        const bool whole = v_first + kRowsWave <= rows_total;              // uniform
        auto staged = [&](int it) __attribute__((always_inline)) {
            const uint2 lo = *reinterpret_cast<const uint2 *>(rbase + it * RPI * OPITCH);
            const uint2 hi = *reinterpret_cast<const uint2 *>(rbase + it * RPI * OPITCH + 8);
            return make_uint4(lo.x, lo.y, hi.x, hi.y);
        };
        constexpr int NIT = kRowsWave / RPI, BATCH = NIT < 8 ? NIT : 8;   // (32 rows of 128 bytes are four stores)
        static_assert(NIT % BATCH == 0, "whole batches of output stores");
        if (__builtin_expect(whole, 1)) {
            // reads in batches, so that their latencies overlap instead of adding up
#pragma unroll
            for (int b = 0; b < NIT; b += BATCH) {
                uint4 w[BATCH];
#pragma unroll
                for (int k = 0; k < BATCH; ++k) w[k] = staged(b + k);
#pragma unroll
                for (int k = 0; k < BATCH; ++k) *reinterpret_cast<uint4 *>(og + (b + k) * RPI * ROWB + goff) = w[k];
            }
        } else {
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const uint4 w = staged(it);
                if (v_first + it * RPI + row0 < rows_total) *reinterpret_cast<uint4 *>(og + it * RPI * ROWB + goff) = w;
            }
        }
    };

    constexpr int RDK = FP8 ? KF : RD;               // K fragment ring (fp8: a unit's four fragments, taken two at a time)
    intx4 kfr[RDK];
    bf16x8 vfr[RD];
    // Pipeline step.  In: s_cur = S(u), pk_prev = P(u-1).  Out: pk_cur = P(u), s_nxt = S(u+1).
    // kb / ksub: tile buffer and unit of K(u+1); vb / vsub: those of V(u-1).
    // Every step has the same shape: units at or past the end of the keys are computed on finite
    // stand-in rows and masked to -inf, so they contribute exact zeros; P(-1) is zero.
    // `chain`: the next step reads unit 1 of the same tile buffers, so its first K fragments are fetched
    // in this step's last pieces; `primed`: the previous step did that for this one.
    // `dma`: this step also issues the tile loads of its stage (the K tile at kg into dk, the V tile at vg into dv).
    // `fin` (run time, only looked at when `can_finish`): S(u) is the first score block of the NEXT row
    // tile and this step's products are the last of the current one, which is then written out.
    auto step = [&](int u, floatx16 (&s_cur)[QB], floatx16 (&s_nxt)[QB], unsigned (&pk_prev)[QB][2][4],
                    unsigned (&pk_cur)[QB][2][4], const uint4 *kb, int ksub, const uint4 *vb, int vsub,
                    auto primed, auto chain, auto dma, uint4 *dk, const uint8_t *kg,
                    uint4 *dv, const uint8_t *vg, auto can_finish, bool fin, const Tile &cur, auto maskable, auto first)
                    __attribute__((always_inline)) {
        // `first` (FOLD): S(u) is the first score block of a row tile - the softmax reference is set from it
        constexpr bool FIRST = decltype(first)::value;
        constexpr bool PRIMED = decltype(primed)::value, CHAIN = decltype(chain)::value;
        constexpr bool DMA = decltype(dma)::value, CANFIN = decltype(can_finish)::value;
        // `maskable` false: the caller knows that unit u lies in a tile that starts at its nominal row (any tile
        // of the verifier's pass before the last one), so there is nothing to mask and nothing to test
        constexpr bool MASKABLE = BLOCK || decltype(maskable)::value;
        if (!PRIMED) {
#pragma unroll
            for (int j = 0; j < RDK; ++j) kfr[j] = k_frag(kb, ksub, j);
        }
        // keys of unit u's tile outside the rows that count (see tile_at) score -inf
        const TileAt cur_at = tile_at(cur, u >> 1);
        const int lo_u = MASKABLE ? cur_at.vlo - 32 * (u & 1) : 0, hi_u = MASKABLE ? cur_at.vhi - 32 * (u & 1) : 32;
        if (MASKABLE && __builtin_expect(lo_u > 0 || hi_u < 32, 0)) {      // uniform branch
            int k0 = 4 * hh;
            asm volatile("" : "+v"(k0));
#pragma unroll
            for (int q = 0; q < QB; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kk = k0 + 8 * (r >> 2) + (r & 3);
                    if (kk < lo_u || kk >= hi_u) s_cur[q][r] = -INFINITY;
                }
            // A key range that starts with a wholly masked unit (BLOCK: a split may begin at a part's
            // overlapping last tile) has no maximum yet: give it a finite one, so that its weights are 0, not NaN.
            if (BLOCK && !FOLD && (lo_u >= 32 || hi_u <= 0)) {
#pragma unroll
                for (int q = 0; q < QB; ++q)
                    if (mc[q] == -INFINITY) {
                        mc[q] = 0.f;
                        thr[q] = kSlack / c[q];
                    }
            }
        }
        float corr[QB], tpart[QB], pe[NE];
        bool changed = false;
        // element e = 2 pr + (0/1) of the exponential stream is S(u)[q = pr % QB][r = 2 (pr / QB) + (0/1)]
        auto exp_piece = [](int e) constexpr { int t = MAXC; while (!(e < NE * (t - MAXC + 1) / EXC)) ++t; return t; };
        unsigned seen = seen0, w_even = 0u;                  // FOLD: the weights' bit patterns or-ed together
        auto pack_pair = [&](int pr) __attribute__((always_inline)) {
            const int q = pr % QB, r = (pr / QB) * 2;
            unsigned w = pack_bf16_rne(pe[2 * pr], pe[2 * pr + 1]);
            asm volatile("" : "+v"(w));                      // P(u) is only consumed a step later: keep its
            pk_cur[q][r >> 3][(r & 7) >> 1] = w;             // computation here, beside the matrix-core work
            if constexpr (FOLD) {
                if (pr & 1) asm volatile("v_or3_b32 %0, %0, %1, %2" : "+v"(seen) : "v"(w_even), "v"(w));
                else w_even = w;
            }
        };
        // FOLD, once per unit after its last weight is packed.  Some weight reached 2 (bit 14 of a bf16 pattern:
        // exponent field >= 128; an overflowed weight is +inf and shows the same bit), or the unit opens a row tile:
        // move the reference of every row to the maximum of this unit plus the margin - never down, except when
        // opening a tile - and redo what was computed with the old one: this unit's weights and the next unit's
        // scores here, the accumulated sums at the end of the step (`changed`).
        auto check_reference = [&]() __attribute__((always_inline)) {
            if (__builtin_expect(FIRST || __builtin_amdgcn_ballot_w64((seen & 0x40004000u) != 0u) != 0, FIRST)) {
                const bool opening = FIRST || ref_unset;     // nothing but zeros accumulated so far
#pragma unroll
                for (int q = 0; q < QB; ++q) {
                    float rm = vmax(s_cur[q][0], s_cur[q][1]);
#pragma unroll
                    for (int r = 2; r < 16; r += 2) rm = vmax3(rm, s_cur[q][r], s_cur[q][r + 1]);
                    rm = half_swap_max(rm);                  // both lane halves hold keys of the same query row
                    float delta = rm + kFoldMargin;
                    if (opening) delta = rm == -INFINITY ? 0.f : delta;  // a wholly masked unit leaves the reference alone
                    else delta = delta > 0.f ? delta : 0.f;
                    if (q == 0) {                            // masks are the same for every row
                        ref_unset = opening && __builtin_amdgcn_ballot_w64(rm != -INFINITY) == 0;
                        seen0 = ref_unset ? 0x4000u : 0u;
                    }
                    mc[q] += delta;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s_cur[q][r] -= delta;
                        s_nxt[q][r] -= delta;                // (written by matrix instructions many pieces ago)
                        cinit[q][r] = -mc[q];
                    }
#pragma unroll
                    for (int r = 0; r < 16; r += 2)
                        pk_cur[q][r >> 3][(r & 7) >> 1] = pack_bf16_rne(fast_exp2(s_cur[q][r]), fast_exp2(s_cur[q][r + 1]));
                    corr[q] = fast_exp2(-delta);
                }
                changed = !opening;                          // (zeros need no rescaling, and 2^-delta may overflow there)
                // written by vector instructions, read as the addend of the next S = K Q^T, which the compiler's
                // hazard padding does not see
                if constexpr (QB == 2) asm volatile("s_nop 7" : "+v"(cinit[0]), "+v"(cinit[QB - 1]));
                else asm volatile("s_nop 7" : "+v"(cinit[0]));
            }
        };
        // everything of the step that is not an MFMA, dealt out over the NP pieces
        auto piece = [&](int t) __attribute__((always_inline)) {
            if (DMA && t >= 1 && t <= NDMA_K + NDMA) {
                if (t <= NDMA_K) dma_one(dk, kg, dma_koff, t - 1);
                else dma_one(dv, vg, dma_voff, t - 1 - NDMA_K);
            }
            if constexpr (MAXC > 0) if (t < MAXC) {
                // row maxima of S(u) decide, without a divergent branch, whether the maxima in use are raised
#pragma unroll
                for (int r = 16 * t / MAXC; r < 16 * (t + 1) / MAXC; r += 2)
#pragma unroll
                    for (int q = 0; q < QB; ++q)             // alternating blocks: no back-to-back dependence
                        tpart[q] = r == 0 ? vmax(s_cur[q][0], s_cur[q][1]) : vmax3(tpart[q], s_cur[q][r], s_cur[q][r + 1]);
                if (t == MAXC - 1) {
                    // Each lane half compares the maximum of its own keys with the threshold; whether any
                    // lane is above it is wave-uniform (always true for the first unit of a row tile).
                    changed = (__builtin_amdgcn_ballot_w64(tpart[0] > thr[0]) | __builtin_amdgcn_ballot_w64(tpart[QB - 1] > thr[QB - 1])) != 0;
                    if (__builtin_expect(changed, 0)) {      // rare: raise the maxima in use
#pragma unroll
                        for (int q = 0; q < QB; ++q) {
                            const float tmq = half_swap_max(tpart[q]) * c[q];
                            const float mn = tmq > mc[q] ? tmq : mc[q];
                            corr[q] = fast_exp2(mc[q] - mn); // first unit: 2^(-inf) = 0
                            mc[q] = mn;
                            thr[q] = (mn + kSlack) / c[q];
                        }
                    }
                }
            }
            if (t >= MAXC && t < MAXC + EXC) {               // (FOLD: the last pieces carry no exponentials)
#pragma unroll
                for (int e = NE * (t - MAXC) / EXC; e < NE * (t - MAXC + 1) / EXC; ++e) {
                    const int pr = e >> 1, q = pr % QB, r = (pr / QB) * 2 + (e & 1);
                    if constexpr (FOLD) pe[e] = fast_exp2(s_cur[q][r]);
                    else pe[e] = fast_exp2(fmaf(s_cur[q][r], c[q], -mc[q]));
                }
            }
            // pairs completed in the previous piece are packed now: a transcendental result cannot be
            // consumed by the very next instruction without a bubble
#pragma unroll
            for (int pr = 0; pr < NE / 2; ++pr)
                if (exp_piece(2 * pr + 1) == t - kPackLag) pack_pair(pr);
            if constexpr (FOLD) {
                if (t == CHK) check_reference();
            }
            __builtin_amdgcn_sched_barrier(0);               // nothing moves between pieces
        };
        // ---- S(u+1): the first V fragments are fetched meanwhile
#pragma unroll
        for (int j = 0; j < KS; ++j) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                if constexpr (FP8) {
                    // the unit's four fragments are all in registers; the first V fragments: two with the first
                    // instruction, one with the second
                    if (j == 0) qk_first<true>(s_nxt[q], k_pair(kfr[0], kfr[1]), qf[q][0]);
                    else qk_next<true>(s_nxt[q], k_pair(kfr[2 * j], kfr[2 * j + 1]), qf[q][j]);
                    static_assert(!FP8 || (KS == 2 && RD == 3), "V fragment schedule of the fp8 form");
                    if (q == 0 && j == 0) { vfr[0] = v_frag(vb, vsub, 0); vfr[1] = v_frag(vb, vsub, 1); }
                    if (q == 0 && j == 1) vfr[2] = v_frag(vb, vsub, 2);
                } else {
                    const int f = j;                             // fragment of this k-step; it is free after its use
                    if constexpr (FOLD) {
                        if (j == 0) qk_first_from(s_nxt[q], kfr[0], qf[q][0], cinit[q]);   // starts from minus the reference
                        else qk_next<false>(s_nxt[q], kfr[f % RD], qf[q][j]);
                    } else {
                        if (j == 0) qk_first<false>(s_nxt[q], kfr[0], qf[q][0]);
                        else qk_next<false>(s_nxt[q], kfr[f % RD], qf[q][j]);
                    }
                    if (q == QB - 1 && f + RD < KF) kfr[f % RD] = k_frag(kb, ksub, f + RD);
                    if (q == 0 && j >= KS - RD) vfr[j - (KS - RD)] = v_frag(vb, vsub, j - (KS - RD));
                }
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
                        else if (CHAIN) {
                            kfr[jv + RD - 2 * DC] = k_frag(kb, 1, jv + RD - 2 * DC);
                            if (FP8 && jv == 2 * DC - 1) kfr[RDK - 1] = k_frag(kb, 1, RDK - 1);   // (the fourth of four)
                        }
                    }
                    piece(NQK + st * (DC + 1) * QB + i * QB + q);
                }
            }
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                const uint4 pw = make_uint4(pk_prev[q][st][0], pk_prev[q][st][1], pk_prev[q][st][2], pk_prev[q][st][3]);
                acc_l[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ones),
                                                                   __builtin_bit_cast(bf16x8, pw), acc_l[q], 0, 0, 0);
                piece(NQK + st * (DC + 1) * QB + DC * QB + q);
            }
        }
        // The score instructions are written as assembly, so the compiler takes their results for complete at
        // once.  Where S(u+1) is never read (the drafter's last step) it would hand those registers to a V
        // fragment, whose load can return before the instruction, still in flight, writes over it.  This use
        // keeps them allocated until the instructions are long done.
#pragma unroll
        for (int q = 0; q < QB; ++q) asm volatile("" :: "v"(s_nxt[q]));
#pragma unroll
        for (int pr = 0; pr < NE / 2; ++pr)
            if (exp_piece(2 * pr + 1) >= NP - kPackLag) pack_pair(pr);
        if (CANFIN && fin) {                                 // uniform: the row tile is complete
            write_out(cur);
            clear_acc_mfma();
        }
        else if (__builtin_expect(changed, 0)) {           // rare: everything accumulated so far changes units
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                // (sixteen registers at a time, each block back in accumulation registers before the next is read:
                // left alone, the compiler holds all 160 products in vector registers at once)
                asm volatile("" : "+a"(acc_l[q]));
                // (register 0 of lanes 0-15 is the sum of the lane's own row, register 1 that of the row sixteen on,
                // whose factor lane + 16 holds; everything else is zero)
                acc_l[q][0] *= corr[q];
                acc_l[q][1] *= __shfl(corr[q], (lane + 16) & 63);
                asm volatile("" : "+a"(acc_l[q]));
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < DC; ++i) {
                    asm volatile("" : "+a"(acc[q][i]));
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[q][i][r] *= corr[q];
                    asm volatile("" : "+a"(acc[q][i]));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    floatx16 s0[QB], s1[QB];                                 // S(u) lives in s{u & 1}
    unsigned pk0[QB][2][4], pk1[QB][2][4];                   // P(u) lives in pk{u & 1}
    Tile cur = tile_of(t_cur), nxt = cur;
    bool has_next = false;

    // Stage sp = steps 2sp+1 and 2sp+2 of a pass over one row tile (nt_even stages).  With PAR = sp & 1 it
    // reads K tile sp+1 from K[1-PAR] and V tile sp from V[PAR], while K tile sp+2 streams into K[PAR] and
    // V tile sp+1 into V[1-PAR]; tile numbers at or past nt_even are tiles of the next row tile.
    // The last stage of a pass (always PAR = 1) therefore already works for the next row tile: its first
    // step computes that tile's S(0) - with that tile's Q - and its second step S(1) and P(0), while
    // their products still belong to the current tile, which the second step then writes out.
    // `kind`: 0 = a stage in the middle of a pass (the hot loop: no tile-boundary logic at all),
    //         1 = the last but one stage (PAR = 0; its K load is tile 0 of the next row tile),
    //         2 = the last stage (PAR = 1).
    auto stage = [&](int sp, auto par, auto kind, auto maskable) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par)::value, KIND = decltype(kind)::value;
        static_assert(KIND == 0 || (KIND == 1 && PAR == 0) || (KIND == 2 && PAR == 1), "stage kinds");
        constexpr bool last = KIND == 2;
        if (!BLOCK && last && has_next) {
            // the Q rows were requested a stage ago and deliberately not waited for at its barrier
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
            install_q(nxt);
        }
        const int ktile = KIND == 0 ? sp + 2 : KIND - 1, vtile = last ? 0 : sp + 1;
        step(2 * sp + 1, s1, s0, pk0, pk1, kbuf(I_<1 - PAR>{}), 0, vbuf(I_<PAR>{}), 0, F_{}, T_{}, T_{},
             kbuf(I_<PAR>{}), tile_at(KIND == 0 || BLOCK ? cur : nxt, ktile).k,
             vbuf(I_<1 - PAR>{}), tile_at(last && !BLOCK ? nxt : cur, vtile).v, F_{}, false, cur, maskable, F_{});
        if (!BLOCK && KIND == 1 && has_next) dma_q(nxt);               // after this stage's tile loads: see the barrier below
        if (last) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                mc_done[q] = mc[q];
                if constexpr (!FOLD) {
                    mc[q] = thr[q] = -INFINITY;              // the second step starts the next tile's softmax
                    c[q] = c_next[q];
                }
            }                                                // (FOLD: the second step is a tile's first and resets the reference)
        }
        step(last ? 0 : 2 * sp + 2, s0, s1, pk1, pk0, kbuf(I_<1 - PAR>{}), 1, vbuf(I_<PAR>{}), 1, T_{}, F_{}, F_{},
             kbuf(I_<PAR>{}), cur.k, vbuf(I_<1 - PAR>{}), cur.v, std::integral_constant<bool, last>{}, last, cur, maskable,
             std::integral_constant<bool, last>{});
        // The barrier that ends a stage waits for the stage's tile loads.  Memory operations complete in
        // order, so the requests issued after those loads - the next tile's Q rows, the finished tile's
        // output rows - can stay in flight: wait until only that many are outstanding.
        constexpr int NST = kRowsWave / (64 / (ROWB / 16));  // output stores per wave
        if (!BLOCK && KIND == 1 && has_next) wait_loads_and_sync(I_<NQDMA>{});
        else if (last && cur.v0 + kRowsWG <= rows_total) {
            wait_loads_and_sync(I_<NST>{});
        }
        else wait_loads_and_sync(I_<0>{});
    };

    if (BLOCK && nt_local <= 0) {
        // A batch entry whose tile list is shorter than the launch planned for (its block hangs over an end of the
        // sequence) leaves the last key range empty: a state that weighs nothing in the merge, and done.
        if (lane < 32) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                const int v = cur.v0 + wave * kRowsWave + q * 32 + lane;
                if (v >= rows_total) continue;
                const size_t slot = (cur.row_base + v) * (size_t)a.splits + split;
                for (int c4 = 0; c4 < D / 4; ++c4)
                    reinterpret_cast<float4 *>(a.part_o + slot * D)[c4] = make_float4(0.f, 0.f, 0.f, 0.f);
                a.part_ml[slot * 2] = -INFINITY;
                a.part_ml[slot * 2 + 1] = 0.f;
            }
        }
        return;
    }
    // ---- prologue of the first row tile: Q rows and K tiles 0, 1 and V tile 0 go straight to LDS
    dma_q(cur);
    dma_tile(K0, tile_at(cur, 0).k, dma_koff, I_<NDMA_K>{});
    dma_tile(V0, tile_at(cur, 0).v, dma_voff, I_<NDMA>{});
    dma_tile(K1, tile_at(cur, 1).k, dma_koff, I_<NDMA_K>{});
    // the Q rows (first in line, and this wave's own) are turned into fragments while the tiles still arrive
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(2 * NDMA_K + NDMA));
    asm volatile("" ::: "memory");
    install_q(cur);
    wait_loads_and_sync(I_<0>{});
#pragma unroll
    for (int q = 0; q < QB; ++q) c[q] = c_next[q];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            if constexpr (FP8) {
                const intx8 kx = k_pair(k_frag(K0, 0, 2 * ks), k_frag(K0, 0, 2 * ks + 1));
                if (ks == 0) qk_first<true>(s0[q], kx, qf[q][0]);
                else qk_next<true>(s0[q], kx, qf[q][ks]);
            } else {
                if (ks == 0) qk_first<false>(s0[q], k_frag(K0, 0, 0), qf[q][0]);       // (FOLD: from zero, the reference is 0)
                else qk_next<false>(s0[q], k_frag(K0, 0, ks), qf[q][ks]);
            }
        }
#pragma unroll
    for (int q = 0; q < QB; ++q)
#pragma unroll
        for (int t = 0; t < 8; ++t) pk1[q][t >> 2][t & 3] = 0u;
    // the compiler does not know that the statements above are matrix instructions whose results
    // need 11 more wait states before a vector instruction may read them
    if constexpr (QB == 2) asm volatile("s_nop 15\n\ts_nop 15" : "+v"(s0[0]), "+v"(s0[QB - 1]));
    else asm volatile("s_nop 15\n\ts_nop 15" : "+v"(s0[0]));
    if constexpr (FP8) asm volatile("s_nop 15\n\ts_nop 15" : "+v"(s0[0]));                     // (an instruction of twice the passes)
    step(0, s0, s1, pk1, pk0, K0, 1, V0, 0, F_{}, F_{}, F_{}, K0, cur.k, V0, cur.v, F_{}, false, cur, T_{}, T_{});
    __syncthreads();   // K tile 0 is overwritten during stage 0: every wave must be done with it

    // ---- passes: stages 0 .. nt_even-1 = steps 1 .. 2 nt_even; the product with P(u) happens in step u+1,
    // so this covers every unit, and the surplus steps work for the next row tile (or on masked stand-ins)
    for (;;) {
        has_next = !BLOCK && t_cur + t_stride < tiles_total;
        if (!BLOCK && has_next) nxt = tile_of(t_cur + t_stride);
        int sp = 0;
        // stages sp <= nt_even - 4 only touch units of tiles <= nt_even - 3 <= nt_local - 2: never the last
        // tile of the key range, the only one of the verifier's pass that can overlap its predecessor
        for (; sp + 4 < nt_even; sp += 2) {
            stage(sp, I_<0>{}, I_<0>{}, F_{});
            stage(sp + 1, I_<1>{}, I_<0>{}, F_{});
        }
        for (; sp + 2 < nt_even; sp += 2) {
            stage(sp, I_<0>{}, I_<0>{}, T_{});
            stage(sp + 1, I_<1>{}, I_<0>{}, T_{});
        }
        stage(sp, I_<0>{}, I_<1>{}, T_{});
        stage(sp + 1, I_<1>{}, I_<2>{}, T_{});
        if (BLOCK || !has_next) break;
        cur = nxt;
        t_cur += t_stride;
    }
#endif  // __HIP_DEVICE_COMPILE__
}

}  // namespace

hipError_t launch_attention_wide(const AttnArgs &a, hipStream_t stream)
{
    if (a.N < TKW) return hipErrorInvalidValue;            // a K/V tile is 64 whole rows
    AttnKernelArgs k;
    fill_kernel_args(a, k, kRowsWGWide, TKW);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus = n;
    }
    const long tiles = (long)a.B * a.Hkv * k.row_tiles;
    long wgs = tiles < cus ? tiles : cus;                  // one persistent workgroup per compute unit
    const long cap = tune("DD_TUNE_ATTN_WIDE_GRID", 0);
    if (cap >= 1 && cap < wgs) wgs = cap;
    const dim3 grid((unsigned)wgs), block(kAttnThreads);
    if (a.qk_dtype == 2) {
        if (a.d != 128) return hipErrorInvalidValue;      // 64-byte fp8 rows are not worth a variant
        return launch(attn_wide_kernel<128, true, false>, grid, block, stream, k);
    }
    // bf16 without per-head scales, long key ranges: the form with the softmax scale folded into Q
    const bool fold = a.q_scale == nullptr && a.k_scale == nullptr && a.N >= kFoldMinKeys;
    if (a.d == 128) return fold ? launch(attn_wide_kernel<128, false, false, true>, grid, block, stream, k)
                                : launch(attn_wide_kernel<128, false, false>, grid, block, stream, k);
    return fold ? launch(attn_wide_kernel<64, false, false, true>, grid, block, stream, k)
                : launch(attn_wide_kernel<64, false, false>, grid, block, stream, k);
}

// The drafter's call on the wide kernel: worth it from 65 query rows per kv head (GQA groups times the block
// length; up to 64 the bf16 call streams), which makes the call compute bound.  Every part of the key stream must
// be empty or at least one tile long.
bool attn_wide_block_fits(const AttnArgs &a)
{
    if (a.qk_dtype == 0 || a.v_dtype != 1 || (a.qk_dtype == 2 && a.d != 128)) return false;
    if ((long)(a.H / a.Hkv) * a.Nq < tune("DD_TUNE_BLOCK_WIDE_MIN_ROWS", 65)) return false;
    // a tile is 64 whole rows of its source: the cache, and the block tensors when rows are spliced in from them
    return a.N >= TKW && (a.Kblk == nullptr || a.block_len >= TKW);
}

// Key splits of that form for `tiles` row tiles: as many as keep the workgroups at or under one per compute unit
// (more would run in a second round, and every split adds partial-state traffic and merge work), at least two
// key tiles each.
static int wide_block_splits_for(long tiles, int N)
{
    long s = 256 / tiles;
    const long max_s = N / (2 * TKW) > 1 ? N / (2 * TKW) : 1;
    if (s > max_s) s = max_s;
    if (s > 16) s = 16;
    return (int)(s < 1 ? 1 : s);
}

// Rows per workgroup of that form: 256, or 128 where a kv head has no more rows than that, or where the smaller
// tile alone gives every compute unit a workgroup, so that the call needs no key splits.
int attn_wide_block_rows(int block_len, int B, int H, int Hkv, int N)
{
    const long forced = tune("DD_TUNE_BLOCK_WIDE_ROWS", 0);
    if (forced == kRowsWGNarrow || forced == kRowsWGWide) return (int)forced;
    const long rows = (long)(H / Hkv) * block_len, heads = (long)B * Hkv;
    if (rows <= kRowsWGNarrow) return kRowsWGNarrow;
    const long t_wide = heads * ((rows + kRowsWGWide - 1) / kRowsWGWide);
    const long t_narrow = heads * ((rows + kRowsWGNarrow - 1) / kRowsWGNarrow);
    return wide_block_splits_for(t_wide, N) > 1 && wide_block_splits_for(t_narrow, N) == 1 ? kRowsWGNarrow : kRowsWGWide;
}

int attn_wide_block_splits(int block_len, int B, int H, int Hkv, int N)
{
    const int per_wg = attn_wide_block_rows(block_len, B, H, Hkv, N);
    return wide_block_splits_for((long)B * Hkv * (((long)(H / Hkv) * block_len + per_wg - 1) / per_wg), N);
}

hipError_t launch_attention_wide_block(const AttnArgs &a, hipStream_t stream)
{
    AttnKernelArgs k;
    const bool narrow = attn_wide_block_rows(a.Nq, a.B, a.H, a.Hkv, a.N) == kRowsWGNarrow;
    fill_kernel_args(a, k, narrow ? kRowsWGNarrow : kRowsWGWide, TKW);
    if (a.Kblk == nullptr) k.block_len = 0;                // no row is taken from the block tensors
    // the kernel splits the LIST of tiles (not the key range) evenly
    int splits;
    if (a.block_starts != nullptr) {
        // positions known on the device only: a list has between ceil(N / 64) and two more tiles; a batch entry
        // with a shorter list than others leaves its last split empty, which the kernel handles
        const int nt_min = (a.N + TKW - 1) / TKW;
        splits = a.splits < nt_min ? a.splits : nt_min;
    } else {
        // drop splits that would be empty
        const int spliced = a.Kblk != nullptr;
        const int la = spliced ? a.block_start : a.N, lb = spliced ? a.block_len : 0, lc = spliced ? a.N - a.block_start - a.block_len : 0;
        const int nt = (la + TKW - 1) / TKW + (lb + TKW - 1) / TKW + (lc + TKW - 1) / TKW;
        splits = a.splits < nt ? a.splits : nt;
        const int per = (nt + splits - 1) / splits;
        splits = (nt + per - 1) / per;
    }
    k.splits = splits;
    const size_t rows = (size_t)a.B * a.H * a.Nq;
    k.part_ml = k.part_o ? k.part_o + rows * (size_t)splits * a.d : nullptr;
    const dim3 grid((unsigned)((long)a.B * a.Hkv * k.row_tiles * splits)), block(kAttnThreads);
    const bool fold = a.q_scale == nullptr && a.k_scale == nullptr && a.N >= kFoldMinKeys;
    hipError_t e;
    if (narrow)
        e = a.qk_dtype == 2 ? launch(attn_wide_kernel<128, true, true, false, 1>, grid, block, stream, k)
          : a.d == 128 ? (fold ? launch(attn_wide_kernel<128, false, true, true, 1>, grid, block, stream, k)
                               : launch(attn_wide_kernel<128, false, true, false, 1>, grid, block, stream, k))
                       : (fold ? launch(attn_wide_kernel<64, false, true, true, 1>, grid, block, stream, k)
                               : launch(attn_wide_kernel<64, false, true, false, 1>, grid, block, stream, k));
    else
        e = a.qk_dtype == 2 ? launch(attn_wide_kernel<128, true, true>, grid, block, stream, k)
          : a.d == 128 ? (fold ? launch(attn_wide_kernel<128, false, true, true>, grid, block, stream, k)
                               : launch(attn_wide_kernel<128, false, true>, grid, block, stream, k))
                       : (fold ? launch(attn_wide_kernel<64, false, true, true>, grid, block, stream, k)
                               : launch(attn_wide_kernel<64, false, true>, grid, block, stream, k));
    return e != hipSuccess ? e : finish_attention(a, splits, stream);
}

}  // namespace dd
