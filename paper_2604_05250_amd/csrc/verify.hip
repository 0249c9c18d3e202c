// Verification pass over the vocabulary (Sec. 3.2): one streaming read of the verifier
// logits (and, in the KL modes, the drafter logits) produces per position the verifier
// confidence c_V = max_x p_V(x) (Eq. 7), its argmax, and KL(p_D || p_V) (Eq. 5); a small
// finishing kernel applies the remask rule (Eq. 4, the KL / confidence thresholds, Eq. 6,
// and the 1 - c_V rule).
//
// HBM-bound design: every logit is loaded exactly once with 16-byte coalesced loads.
// A row is split over `S` workgroups.  Each wave keeps wave-uniform references (the
// running verifier and drafter maxima) so the per-element work
// is one fma + one exp2 + one add per logit, and the argmax / rescale logic runs only
// when some lane of the wave sees a new maximum (a few times per row).  Partial states
//     (ref_D, sum e^{l_D-ref_D}, sum e^{l_D-ref_D}(l_D-l_V), max l_V, sum e^{l_V-max}, argmax)
// are merged in a fixed order (lanes -> waves -> splits), so results are run-to-run
// identical; the last merge and the log / divide are done in fp64.
#include "dd_internal.h"

#include <limits.h>
#include <math.h>

namespace dd {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;   // independent 16-byte loads per matrix in flight per lane
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kNegInf = -INFINITY;
// The drafter reference is raised when a logit exceeds it by more than this.  Zero keeps it
// equal to the running maximum, exactly as on the verifier side, so identical drafter and
// verifier rows go through identical arithmetic and give KL = 0 exactly.
constexpr float kLazyMargin = 0.0f;

struct __align__(32) VerifyPartial {
    float ref_d, s_d, a;   // drafter reference, sum e^{l_D-ref}, sum e^{l_D-ref} (l_D - l_V)
    float best_v, s_v;     // verifier maximum, sum e^{l_V-best}
    int idx;               // lowest index attaining best_v
    int idx_d;             // lowest index attaining ref_d (the drafter's most likely token)
    int pad1;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// streaming 16-byte load: every logit is read once, so it need not displace cached lines
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const uint4 *p)
{
    const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(w.x, w.y, w.z, w.w);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ int wave_min(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// e^{ref - m} with the convention that an empty state (ref = -inf) weighs nothing
__device__ __forceinline__ float rescale_factor(float ref, float m)
{
    return ref == kNegInf ? 0.0f : fast_exp2((ref - m) * kLog2e);
}

template <bool BF16> struct VecTraits;
template <> struct VecTraits<true> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&x)[8])
    {
        const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};
template <> struct VecTraits<false> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&x)[4])
    {
        x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
    }
};

struct LaneState {
    float ref_d = kNegInf, s_d = 0.f, a = 0.f;   // ref_d is wave-uniform
    float best_v = kNegInf, s_v = 0.f;           // best_v, idx_v are wave-uniform
    int idx_v = INT_MAX, idx_d = INT_MAX;        // idx_d: where the drafter reference was found (wave-uniform)
};

// Fold one 16-byte vector of verifier logits (and the matching drafter vector) into the state.
// Must be called by all lanes of a wave together; `valid` masks lanes past the row chunk's end.
// TRACKD: also keep the index of the drafter's maximum (only the all-scores entry point asks for it)
template <bool BF16, bool KL, bool TRACKD>
__device__ __forceinline__ void consume(const uint4 &rv, const uint4 &rd, bool valid, int elem_base, LaneState &st)
{
    constexpr int E = VecTraits<BF16>::kElems;
    float xv[E], xd[E];
    VecTraits<BF16>::unpack(rv, xv);
    float bmax = xv[0];
#pragma unroll
    for (int e = 1; e < E; ++e) bmax = fmaxf(bmax, xv[e]);
    if (!valid) bmax = kNegInf;

    if (__any(bmax > st.best_v)) {
        // rare: a new verifier maximum appears in this wave
        const float wmax = wave_max(bmax);
        int cand = INT_MAX;
        if (valid && bmax == wmax) {
#pragma unroll
            for (int e = E - 1; e >= 0; --e)
                if (xv[e] == wmax) cand = elem_base + e;
        }
        const int widx = wave_min(cand);
        st.s_v *= rescale_factor(st.best_v, wmax);
        st.best_v = wmax;
        st.idx_v = widx;
    }
    if (KL) {
        VecTraits<BF16>::unpack(rd, xd);
        float dmax = xd[0];
#pragma unroll
        for (int e = 1; e < E; ++e) dmax = fmaxf(dmax, xd[e]);
        if (!valid) dmax = kNegInf;
        if (__any(dmax > st.ref_d + kLazyMargin)) {
            const float wmax = wave_max(dmax);
            if (TRACKD) {
                int cand = INT_MAX;
                if (valid && dmax == wmax) {
#pragma unroll
                    for (int e = E - 1; e >= 0; --e)
                        if (xd[e] == wmax) cand = elem_base + e;
                }
                st.idx_d = wave_min(cand);
            }
            const float c = rescale_factor(st.ref_d, wmax);
            st.s_d *= c;
            st.a *= c;
            st.ref_d = wmax;
        }
    }
    if (valid) {
        const float mv = st.best_v * kLog2e;
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc += fast_exp2(fmaf(xv[e], kLog2e, -mv));
        st.s_v += acc;
        if (KL) {
            const float md = st.ref_d * kLog2e;
            float accs = 0.f, acca = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float ed = fast_exp2(fmaf(xd[e], kLog2e, -md));
                accs += ed;
                acca = fmaf(ed, xd[e] - xv[e], acca);
            }
            st.s_d += accs;
            st.a += acca;
        }
    }
}

struct WaveState {
    float ref_d, s_d, a, best_v, s_v;
    int idx, idx_d;
};

// associative merge of two partial states (b comes after a in index order)
__device__ __forceinline__ WaveState merge(const WaveState &x, const WaveState &y)
{
    WaveState r;
    const float mv = fmaxf(x.best_v, y.best_v);
    r.s_v = x.s_v * rescale_factor(x.best_v, mv) + y.s_v * rescale_factor(y.best_v, mv);
    const bool take_y = (y.best_v > x.best_v) || (y.best_v == x.best_v && y.idx < x.idx);
    r.best_v = mv;
    r.idx = take_y ? y.idx : x.idx;
    const float md = fmaxf(x.ref_d, y.ref_d);
    const float cx = rescale_factor(x.ref_d, md), cy = rescale_factor(y.ref_d, md);
    r.idx_d = ((y.ref_d > x.ref_d) || (y.ref_d == x.ref_d && y.idx_d < x.idx_d)) ? y.idx_d : x.idx_d;
    r.ref_d = md;
    r.s_d = x.s_d * cx + y.s_d * cy;
    r.a = x.a * cx + y.a * cy;
    return r;
}

// Reduce vectors [vbeg, vend) of one row with a workgroup of THREADS lanes.  Returns true on thread 0,
// whose `out` then holds the merged state of the range (lanes -> waves -> workgroup, fixed order).
template <bool BF16, bool KL, int THREADS, bool TRACKD>
__device__ __forceinline__ bool reduce_range(const uint4 *__restrict__ pv, const uint4 *__restrict__ pd,
                                             int vbeg, int vend, WaveState &out)
{
    constexpr int E = VecTraits<BF16>::kElems;
    constexpr int NW = THREADS / 64;
    const int tid = threadIdx.x;
    LaneState st;
    int base = vbeg;
    // full iterations: kUnroll independent 16-byte loads per matrix in flight per lane
    for (; base + THREADS * kUnroll <= vend; base += THREADS * kUnroll) {
        uint4 rv[kUnroll], rd[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int idx = base + u * THREADS + tid;
            rv[u] = stream_load16(pv + idx);
            if (KL) rd[u] = stream_load16(pd + idx);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            consume<BF16, KL, TRACKD>(rv[u], rd[u], true, (base + u * THREADS + tid) * E, st);
    }
    // ragged remainder of the range
    if (base < vend) {
        uint4 rv[kUnroll], rd[kUnroll];
        bool ok[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int idx = base + u * THREADS + tid;
            ok[u] = idx < vend;
            rv[u] = make_uint4(0, 0, 0, 0);
            rd[u] = make_uint4(0, 0, 0, 0);
            if (ok[u]) {
                rv[u] = stream_load16(pv + idx);
                if (KL) rd[u] = stream_load16(pd + idx);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            consume<BF16, KL, TRACKD>(rv[u], rd[u], ok[u], (base + u * THREADS + tid) * E, st);
    }

    // lanes -> wave (references are already wave-uniform), waves -> workgroup
    __shared__ WaveState ws[NW];
    WaveState w;
    w.ref_d = st.ref_d;
    w.s_d = wave_sum(st.s_d);
    w.a = wave_sum(st.a);
    w.best_v = st.best_v;
    w.s_v = wave_sum(st.s_v);
    w.idx = st.idx_v;
    w.idx_d = st.idx_d;
    if ((tid & 63) == 0) ws[tid >> 6] = w;
    __syncthreads();
    if (tid != 0) return false;
    WaveState r = ws[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = merge(r, ws[i]);
    out = r;
    return true;
}

// grid: P * S workgroups; workgroup (row, split) reduces vectors [split*chunk, (split+1)*chunk) of its row
template <bool BF16, bool KL, bool TRACKD = false>
__global__ __launch_bounds__(kThreads) void verify_partial_kernel(const uint4 *__restrict__ logits_d,
                                                                  const uint4 *__restrict__ logits_v,
                                                                  int nvec, int S, int chunk,
                                                                  VerifyPartial *__restrict__ part)
{
    const int row = blockIdx.x / S;
    const int split = blockIdx.x - row * S;
    const size_t rbase = (size_t)row * (size_t)nvec;
    const int vbeg = split * chunk;
    const int vend = min(nvec, vbeg + chunk);
    WaveState r;
    if (reduce_range<BF16, KL, kThreads, TRACKD>(logits_v + rbase, KL ? logits_d + rbase : nullptr, vbeg, vend, r)) {
        VerifyPartial p;
        p.ref_d = r.ref_d; p.s_d = r.s_d; p.a = r.a;
        p.best_v = r.best_v; p.s_v = r.s_v; p.idx = r.idx;
        p.idx_d = r.idx_d; p.pad1 = 0;
        part[(size_t)row * S + split] = p;
    }
}

// Philox-4x32 with ten rounds (Salmon et al., SC'11): counter-based, so the uniform of a
// row depends only on (seed, row index) and not on the launch geometry.
__device__ __forceinline__ unsigned philox_word0(uint64_t seed, uint64_t row)
{
    unsigned c0 = (unsigned)row, c1 = (unsigned)(row >> 32), c2 = 0u, c3 = 0u;
    unsigned k0 = (unsigned)seed, k1 = (unsigned)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}
__device__ __forceinline__ double row_uniform(uint64_t seed, uint64_t row)
{
    return (double)(philox_word0(seed, row) >> 8) * (1.0 / 16777216.0);
}

// Finish one row from its merged sums (fp64): score, token, remask rule.
//   KL = E_D[l_D - l_V] - lse_D + lse_V = a/s_D - (m_D + ln s_D) + (m_V + ln s_V);   c_V = e^{max - lse_V} = 1/s_V
__device__ __forceinline__ void finish_row(int row, double md, double sd, double a, double mv, double sv, int idx,
                                           const uint8_t *__restrict__ mask, int mode, float threshold, uint64_t seed,
                                           int kl_mode, uint8_t *__restrict__ out_mask,
                                           int32_t *__restrict__ out_tokens, float *__restrict__ out_scores,
                                           int idx_d = 0, const VerifyExtra ex = VerifyExtra{})
{
    const double score = kl_mode ? a / sd - (md + log(sd)) + (mv + log(sv)) : 1.0 / sv;
    const float s32 = (float)score;
    out_scores[row] = s32;
    out_tokens[row] = idx;
    if (mode == kModeScores) {                   // every per-position quantity, no rule: c = e^{max - lse} = 1 / sum
        ex.conf_v[row] = (float)(1.0 / sv);
        if (ex.conf_d) ex.conf_d[row] = (float)(1.0 / sd);
        if (ex.tok_d) ex.tok_d[row] = idx_d;
        return;
    }
    const uint8_t m = mask[row];
    bool remask = false;
    switch (mode) {
    case 1: remask = s32 > threshold; break;                                // KL threshold
    case 2: remask = s32 < threshold; break;                                // confidence threshold
    case 4: remask = row_uniform(seed, (uint64_t)row) < 1.0 - (double)s32; break;
    default: break;                                                         // trust; per-sequence rules decided later
    }
    out_mask[row] = (uint8_t)((m != 0) || remask);
}

// Sixteen lanes per row (S <= 16): lane s takes the partial state of split s, the group merges them in fp64
// with xor-butterflies (every lane ends with the same totals: a + b == b + a exactly), lane 0 finishes the row.
constexpr int kFinalizeLanes = 16;
// Called by whole groups of sixteen consecutive lanes (lane sp of the group takes split sp of `row`); `row_ok`
// false for a group without a row: it still takes part in the shuffles.
__device__ __forceinline__ void merge_splits_and_finish(const VerifyPartial *__restrict__ part, int S, long row,
                                                        bool row_ok, int sp, const uint8_t *__restrict__ mask,
                                                        int mode, float threshold, uint64_t seed, int kl_mode,
                                                        uint8_t *__restrict__ out_mask,
                                                        int32_t *__restrict__ out_tokens,
                                                        float *__restrict__ out_scores, const VerifyExtra &ex)
{
    const bool have = row_ok && sp < S;                    // no early exit: the shuffles below need every lane
    VerifyPartial p;
    p.ref_d = kNegInf; p.s_d = 0.f; p.a = 0.f; p.best_v = kNegInf; p.s_v = 0.f; p.idx = INT_MAX; p.idx_d = INT_MAX;
    if (have) p = part[(size_t)row * S + sp];
    float mv = p.best_v, md = kl_mode ? p.ref_d : kNegInf;
    int idx = p.idx, idx_d = p.idx_d;
#pragma unroll
    for (int o = kFinalizeLanes / 2; o > 0; o >>= 1) {
        const float ov = __shfl_xor(mv, o), od = __shfl_xor(md, o);
        const int oi = __shfl_xor(idx, o), oid = __shfl_xor(idx_d, o);
        if (ov > mv || (ov == mv && oi < idx)) { mv = ov; idx = oi; }
        if (od > md || (od == md && oid < idx_d)) { md = od; idx_d = oid; }
    }
    double sv = 0.0, sd = 0.0, a = 0.0;
    if (p.best_v != kNegInf) sv = (double)p.s_v * exp((double)p.best_v - (double)mv);
    if (kl_mode && p.ref_d != kNegInf) {
        const double c = exp((double)p.ref_d - (double)md);
        sd = (double)p.s_d * c;
        a = (double)p.a * c;
    }
#pragma unroll
    for (int o = kFinalizeLanes / 2; o > 0; o >>= 1) {
        sv += __shfl_xor(sv, o);
        sd += __shfl_xor(sd, o);
        a += __shfl_xor(a, o);
    }
    if (sp == 0 && row_ok)
        finish_row((int)row, md, sd, a, mv, sv, idx, mask, mode, threshold, seed, kl_mode, out_mask, out_tokens,
                   out_scores, idx_d, ex);
}

__global__ __launch_bounds__(256) void verify_finalize_kernel(const VerifyPartial *__restrict__ part, int S, int P,
                                                              const uint8_t *__restrict__ mask, int mode,
                                                              float threshold, uint64_t seed, int kl_mode,
                                                              uint8_t *__restrict__ out_mask,
                                                              int32_t *__restrict__ out_tokens,
                                                              float *__restrict__ out_scores, VerifyExtra ex)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    const int row = gid / kFinalizeLanes;
    merge_splits_and_finish(part, S, row, row < P, gid % kFinalizeLanes, mask, mode, threshold, seed, kl_mode, out_mask,
                            out_tokens, out_scores, ex);
}

// One workgroup per row: stream the whole row and finish it in the same kernel (no partial states,
// no second launch).  Used whenever there are enough rows to fill the chip with such workgroups.
template <bool BF16, bool KL, int THREADS, bool TRACKD = false>
__global__ __launch_bounds__(THREADS) void verify_row_kernel(const uint4 *__restrict__ logits_d,
                                                             const uint4 *__restrict__ logits_v, int nvec,
                                                             const uint8_t *__restrict__ mask, int mode,
                                                             float threshold, uint64_t seed,
                                                             uint8_t *__restrict__ out_mask,
                                                             int32_t *__restrict__ out_tokens,
                                                             float *__restrict__ out_scores, VerifyExtra ex)
{
    const int row = blockIdx.x;
    const size_t rbase = (size_t)row * (size_t)nvec;
    WaveState r;
    if (reduce_range<BF16, KL, THREADS, TRACKD>(logits_v + rbase, KL ? logits_d + rbase : nullptr, 0, nvec, r))
        finish_row(row, (double)r.ref_d, (double)r.s_d, (double)r.a, (double)r.best_v, (double)r.s_v, r.idx,
                   mask, mode, threshold, seed, KL ? 1 : 0, out_mask, out_tokens, out_scores, r.idx_d, ex);
}

// Eq. 6: one workgroup per sequence sums the divergences of its eligible rows, then draws
template <int THREADS>
__device__ __forceinline__ void klprob_sequence(const float *__restrict__ scores, const uint8_t *__restrict__ mask,
                                                size_t base, int G, uint64_t seed, uint8_t *__restrict__ out_mask,
                                                double *red)
{
    const int tid = threadIdx.x;
    double local = 0.0;
    for (int g = tid; g < G; g += THREADS) {
        const float s = scores[base + g];
        if (mask[base + g] == 0 && s > 0.0f) local += (double)s;
    }
    red[tid] = local;
    __syncthreads();
    for (int o = THREADS / 2; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    const double total = red[0];
    for (int g = tid; g < G; g += THREADS) {
        const size_t i = base + g;
        const float s = scores[i];
        const double k = s > 0.0f ? (double)s : 0.0;
        const double p = total > 0.0 ? k / total : 0.0;
        const bool remask = mask[i] == 0 && row_uniform(seed, (uint64_t)i) < p;
        out_mask[i] = (uint8_t)(mask[i] != 0 || remask);
    }
}

__global__ __launch_bounds__(256) void verify_klprob_kernel(const float *__restrict__ scores,
                                                            const uint8_t *__restrict__ mask, int G, uint64_t seed,
                                                            uint8_t *__restrict__ out_mask)
{
    __shared__ double red[256];
    klprob_sequence<256>(scores, mask, (size_t)blockIdx.x * G, G, seed, out_mask, red);
}

// Budgeted remasking: rank the eligible rows of a sequence by badness (KL: larger score, confidence: smaller
// score; equal scores: lower row first) and remask those of rank < k.  The rank of a row is the number of
// eligible rows of its sequence that are worse.  One workgroup takes 64 rows of one sequence, four lanes per
// row, each lane a quarter of the comparisons; the sequence's scores pass through LDS in chunks and are
// read back 16 bytes at a time (a scalar loop here is bound by the LDS latency of every single read).
constexpr int kTopkRows = 64, kTopkChunk = 2048;
// Rank of row g among the rows of its sequence whose mask byte equals `want` (the candidates), ordered by
// sign * score descending, equal values by row; -1 for a row that is no candidate.  Called by all THREADS lanes
// of a workgroup (it contains barriers); lanes 4r..4r+3 hold row r of the workgroup's THREADS / 4 and all four
// return its rank.
template <int THREADS>
__device__ __forceinline__ int sequence_rank(const float *__restrict__ scores, const uint8_t *__restrict__ mask,
                                             size_t base, int G, int g, uint8_t want, float sign, float *bad_sh)
{
    const int tid = threadIdx.x, sub = tid % 4;
    const bool candidate = g < G && mask[base + g] == want;
    const float bad = candidate ? sign * scores[base + g] : 0.0f;
    int rank = 0;
    for (int c0 = 0; c0 < G; c0 += kTopkChunk) {             // uniform trip count: every lane reaches the barriers
        const int n = min(kTopkChunk, G - c0), n16 = (n + 15) & ~15;
        __syncthreads();
        for (int j = tid; j < n16; j += THREADS)             // -inf marks a row that is no candidate
            bad_sh[j] = (j < n && mask[base + c0 + j] == want) ? sign * scores[base + c0 + j] : kNegInf;
        __syncthreads();
        if (candidate) {
#pragma unroll 4
            for (int j = 4 * sub; j < n16; j += 16) {
                const float4 o = *reinterpret_cast<const float4 *>(&bad_sh[j]);
                const int i = c0 + j;
                rank += (o.x > bad || (o.x == bad && i < g)) ? 1 : 0;
                rank += (o.y > bad || (o.y == bad && i + 1 < g)) ? 1 : 0;
                rank += (o.z > bad || (o.z == bad && i + 2 < g)) ? 1 : 0;
                rank += (o.w > bad || (o.w == bad && i + 3 < g)) ? 1 : 0;
            }
        }
    }
    rank += __shfl_xor(rank, 1);
    rank += __shfl_xor(rank, 2);
    return candidate ? rank : -1;
}

// rows [slab * THREADS / 4, + THREADS / 4) of the sequence at `base`; called by all lanes of a workgroup
template <int THREADS>
__device__ __forceinline__ void topk_slab(const float *__restrict__ scores, const uint8_t *__restrict__ mask,
                                          size_t base, int G, int slab, int kl_mode, float budget,
                                          uint8_t *__restrict__ out_mask, float *bad_sh)
{
    const int tid = threadIdx.x;
    const int g = slab * (THREADS / 4) + tid / 4;
    const int rank = sequence_rank<THREADS>(scores, mask, base, G, g, 0, kl_mode ? 1.0f : -1.0f, bad_sh);
    if (g < G && tid % 4 == 0) out_mask[base + g] = (uint8_t)(mask[base + g] != 0 || (rank >= 0 && (float)rank < budget));
}

__global__ __launch_bounds__(256) void verify_topk_kernel(const float *__restrict__ scores,
                                                          const uint8_t *__restrict__ mask, int G, int kl_mode,
                                                          float budget, uint8_t *__restrict__ out_mask)
{
    __shared__ __attribute__((aligned(16))) float bad_sh[kTopkChunk];
    const int slabs = (G + kTopkRows - 1) / kTopkRows;        // workgroups per sequence
    topk_slab<256>(scores, mask, (size_t)(blockIdx.x / slabs) * G, G, blockIdx.x % slabs, kl_mode, budget, out_mask, bad_sh);
}

// Drafter unmasking (Alg. 1, drafting phase): of the positions that still hold [MASK], those selected by
// confidence are decoded to the drafter's most likely token.  mode 0: confidence above the threshold, and
// always the most confident one of the sequence; mode 1: the k most confident ones.
template <int THREADS>
__device__ __forceinline__ void unmask_slab(const float *__restrict__ conf, const uint8_t *__restrict__ mask,
                                            const int32_t *__restrict__ tokens, size_t base, int G, int slab, int mode,
                                            float threshold, uint8_t *__restrict__ out_mask, int32_t *__restrict__ x,
                                            float *bad_sh)
{
    const int tid = threadIdx.x;
    const int g = slab * (THREADS / 4) + tid / 4;
    const int rank = sequence_rank<THREADS>(conf, mask, base, G, g, 1, 1.0f, bad_sh);
    if (g < G && tid % 4 == 0) {
        const bool take = rank >= 0 && (mode == 0 ? (rank == 0 || conf[base + g] > threshold) : (float)rank < threshold);
        out_mask[base + g] = (uint8_t)(mask[base + g] != 0 && !take);
        if (take && x) x[base + g] = tokens[base + g];
    }
}

__global__ __launch_bounds__(256) void unmask_select_kernel(const float *__restrict__ conf,
                                                            const uint8_t *__restrict__ mask,
                                                            const int32_t *__restrict__ tokens, int G, int mode,
                                                            float threshold, uint8_t *__restrict__ out_mask,
                                                            int32_t *__restrict__ x)
{
    __shared__ __attribute__((aligned(16))) float bad_sh[kTopkChunk];
    const int slabs = (G + kTopkRows - 1) / kTopkRows;
    unmask_slab<256>(conf, mask, tokens, (size_t)(blockIdx.x / slabs) * G, G, blockIdx.x % slabs, mode, threshold, out_mask,
                     x, bad_sh);
}

// Split path with a per-sequence rule (Eq. 6, the budgeted rules, the unmasking step): one workgroup per
// sequence first finishes the rows of its sequence from their partial states, then applies the rule to them
// - the second and third launch of such a call in one.  The scores and tokens the rule reads were written by
// this workgroup; the barrier between the two phases makes them visible to all of its lanes.
constexpr int kSeqThreads = 1024;
__global__ __launch_bounds__(kSeqThreads) void verify_finalize_seq_kernel(const VerifyPartial *__restrict__ part, int S, int G,
                                                                  const uint8_t *__restrict__ mask, int mode,
                                                                  float threshold, uint64_t seed, int kl_mode,
                                                                  uint8_t *__restrict__ out_mask,
                                                                  int32_t *__restrict__ out_tokens,
                                                                  float *__restrict__ out_scores,
                                                                  int32_t *__restrict__ x_tokens)
{
    __shared__ __attribute__((aligned(16))) float bad_sh[kTopkChunk];
    __shared__ double red[kSeqThreads];
    const int tid = threadIdx.x;
    const size_t base = (size_t)blockIdx.x * G;
    constexpr int kRowsPerPass = kSeqThreads / kFinalizeLanes;
    for (int g0 = 0; g0 < G; g0 += kRowsPerPass) {           // uniform trip count
        const int g = g0 + tid / kFinalizeLanes;
        merge_splits_and_finish(part, S, (long)base + g, g < G, tid % kFinalizeLanes, mask, mode, threshold, seed, kl_mode,
                                out_mask, out_tokens, out_scores, VerifyExtra{});
    }
    __threadfence_block();
    __syncthreads();
    const int slabs = (G + kSeqThreads / 4 - 1) / (kSeqThreads / 4);
    if (mode == 3) {
        klprob_sequence<kSeqThreads>(out_scores, mask, base, G, seed, out_mask, red);
    } else if (mode == 5 || mode == 6) {
        for (int slab = 0; slab < slabs; ++slab)
            topk_slab<kSeqThreads>(out_scores, mask, base, G, slab, kl_mode, floorf(threshold), out_mask, bad_sh);
    } else {
        for (int slab = 0; slab < slabs; ++slab)
            unmask_slab<kSeqThreads>(out_scores, mask, out_tokens, base, G, slab, mode - kModeUnmaskThresh,
                                     mode == kModeUnmaskTopk ? floorf(threshold) : threshold, out_mask, x_tokens, bad_sh);
    }
}

}  // namespace

// Rows are handled by one workgroup each (fused finish) once there are enough of them to occupy the
// chip; the workgroup grows as the row count shrinks so that the bytes in flight stay about constant.
int verify_fused_threads(int P)
{
    if (P < 192) return 0;               // too few rows: split them over several workgroups instead
    return P >= 2048 ? 256 : 512;        // measured: 512 lanes per row stream best for 256..1024 rows
}

// Vectors per split: a whole number of full iterations (kThreads * kUnroll vectors), so that only the last
// split of a row has a ragged remainder - every load round of a workgroup is a dependent memory round trip,
// and with few rows those round trips are the call.
static int verify_split_chunk(int P, int V, int elem_bytes)
{
    const long nvec = (long)V * elem_bytes / 16;
    long s = (2048 + P - 1) / P;         // about 2048 workgroups in all
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    const long iter = (long)kThreads * kUnroll;
    long chunk = (nvec + s - 1) / s;
    chunk = (chunk + iter - 1) / iter * iter;
    return (int)chunk;
}

int verify_splits(int P, int V, int elem_bytes)
{
    if (P <= 0 || verify_fused_threads(P) != 0) return 1;
    const long nvec = (long)V * elem_bytes / 16;
    const long chunk = verify_split_chunk(P, V, elem_bytes);
    const long s = (nvec + chunk - 1) / chunk;
    return (int)(s < 1 ? 1 : s);
}

size_t verify_workspace_bytes(int P, int V, int elem_bytes)
{
    if (P <= 0 || verify_fused_threads(P) != 0) return 0;
    return (size_t)P * (size_t)verify_splits(P, V, elem_bytes) * sizeof(VerifyPartial);
}

template <bool BF16, bool KL, bool TRACKD = false>
static hipError_t launch_row_kernel(int threads, dim3 grid, hipStream_t stream, const uint4 *ld, const uint4 *lv,
                                    int nvec, const uint8_t *mask, int mode, float threshold, uint64_t seed,
                                    uint8_t *out_mask, int32_t *out_tokens, float *out_scores, VerifyExtra ex)
{
    if (threads == 256)
        return launch(verify_row_kernel<BF16, KL, 256, TRACKD>, grid, dim3(256), stream, ld, lv, nvec, mask, mode,
                      threshold, seed, out_mask, out_tokens, out_scores, ex);
    return launch(verify_row_kernel<BF16, KL, 512, TRACKD>, grid, dim3(512), stream, ld, lv, nvec, mask, mode,
                  threshold, seed, out_mask, out_tokens, out_scores, ex);
}

hipError_t launch_verify(const void *logits_d, const void *logits_v, const uint8_t *mask,
                         int mode, float threshold, uint64_t seed,
                         uint8_t *out_mask, int32_t *out_tokens, float *out_scores,
                         int B, int G, int V, int logit_is_bf16, void *workspace, hipStream_t stream,
                         int32_t *x_tokens, const VerifyExtra *extra)
{
    const int P = B * G;
    if (P == 0) return hipSuccess;
    const int eb = logit_is_bf16 ? 2 : 4;
    const int nvec = (int)((long)V * eb / 16);
    const bool kl = (mode == 1 || mode == 3 || mode == 5 || mode == kModeScores);
    const VerifyExtra ex = extra ? *extra : VerifyExtra{};
    const uint4 *ld = static_cast<const uint4 *>(logits_d);
    const uint4 *lv = static_cast<const uint4 *>(logits_v);
    hipError_t e;
    const int fused = verify_fused_threads(P);
    const bool track_d = mode == kModeScores && ex.tok_d != nullptr;     // the drafter's argmax is wanted as well
    if (fused != 0 && track_d) {
        const dim3 grid((unsigned)P);
        e = logit_is_bf16 ? launch_row_kernel<true, true, true>(fused, grid, stream, ld, lv, nvec, mask, mode, threshold, seed, out_mask, out_tokens, out_scores, ex)
                          : launch_row_kernel<false, true, true>(fused, grid, stream, ld, lv, nvec, mask, mode, threshold, seed, out_mask, out_tokens, out_scores, ex);
    } else if (fused != 0) {
        const dim3 grid((unsigned)P);
        if (logit_is_bf16)
            e = kl ? launch_row_kernel<true, true>(fused, grid, stream, ld, lv, nvec, mask, mode, threshold, seed, out_mask, out_tokens, out_scores, ex)
                   : launch_row_kernel<true, false>(fused, grid, stream, ld, lv, nvec, mask, mode, threshold, seed, out_mask, out_tokens, out_scores, ex);
        else
            e = kl ? launch_row_kernel<false, true>(fused, grid, stream, ld, lv, nvec, mask, mode, threshold, seed, out_mask, out_tokens, out_scores, ex)
                   : launch_row_kernel<false, false>(fused, grid, stream, ld, lv, nvec, mask, mode, threshold, seed, out_mask, out_tokens, out_scores, ex);
    } else {
        const int S = verify_splits(P, V, eb);
        const int chunk = verify_split_chunk(P, V, eb);
        VerifyPartial *part = static_cast<VerifyPartial *>(workspace);
        const dim3 grid((unsigned)((long)P * S)), block(kThreads);
        if (track_d) {
            e = logit_is_bf16 ? launch(verify_partial_kernel<true, true, true>, grid, block, stream, ld, lv, nvec, S, chunk, part)
                              : launch(verify_partial_kernel<false, true, true>, grid, block, stream, ld, lv, nvec, S, chunk, part);
        } else if (logit_is_bf16) {
            if (kl) e = launch(verify_partial_kernel<true, true>, grid, block, stream, ld, lv, nvec, S, chunk, part);
            else    e = launch(verify_partial_kernel<true, false>, grid, block, stream, ld, lv, nvec, S, chunk, part);
        } else {
            if (kl) e = launch(verify_partial_kernel<false, true>, grid, block, stream, ld, lv, nvec, S, chunk, part);
            else    e = launch(verify_partial_kernel<false, false>, grid, block, stream, ld, lv, nvec, S, chunk, part);
        }
        if (e != hipSuccess) return e;
        if (mode == 3 || mode == 5 || mode == 6 || mode == kModeUnmaskThresh || mode == kModeUnmaskTopk)
            return launch(verify_finalize_seq_kernel, dim3((unsigned)B), dim3(kSeqThreads), stream, (const VerifyPartial *)part, S,
                          G, mask, mode, threshold, seed, kl ? 1 : 0, out_mask, out_tokens, out_scores, x_tokens);
        e = launch(verify_finalize_kernel, dim3((unsigned)(((long)P * kFinalizeLanes + 255) / 256)), dim3(256), stream,
                   (const VerifyPartial *)part, S, P, mask, mode, threshold, seed, kl ? 1 : 0, out_mask, out_tokens, out_scores,
                   ex);
    }
    if (e != hipSuccess) return e;
    if (mode == 3)
        e = launch(verify_klprob_kernel, dim3(B), dim3(256), stream, (const float *)out_scores, mask, G, seed, out_mask);
    if (mode == kModeUnmaskThresh || mode == kModeUnmaskTopk)
        // the pass above ran as for the Trust rule on the drafter's logits: confidence and argmax of every row
        return launch(unmask_select_kernel, dim3((unsigned)((long)((G + kTopkRows - 1) / kTopkRows) * B)), dim3(256),
                      stream, (const float *)out_scores, mask, (const int32_t *)out_tokens, G, mode - kModeUnmaskThresh,
                      mode == kModeUnmaskTopk ? floorf(threshold) : threshold, out_mask, x_tokens);
    if (mode == 5 || mode == 6)
        e = launch(verify_topk_kernel, dim3((unsigned)((long)((G + kTopkRows - 1) / kTopkRows) * B)), dim3(256), stream,
                   (const float *)out_scores, mask, G, kl ? 1 : 0, floorf(threshold), out_mask);
    return e;
}

}  // namespace dd
