// Bulk prefill of an empty WeightedKV cache with a prompt of P tokens, gfx950.
//
// The paper streams tokens one by one (Algorithm 1) and gives no procedure for a prompt that
// arrives at once.  What is computed here: row t of the prompt is softmax attention of q_t over
// tokens 0..t of the UNcompressed prompt (Section III-A, scale of Section III-B); the score list
// is what Algorithm 1's bookkeeping accumulates over these rows, a_i = sum_t A_t[i], with
// n_i = P - i; then, while more than m entries remain, Algorithm 1's selection and merge are
// repeated with these (now fixed) scores.  For P <= m + 1 this is exactly Algorithm 1 fed token
// by token; beyond that it is a different function (streamed tokens attend to an already
// compressed cache).
//
// Three kernels:
//   1. wkv_prefill_rows: causal attention, one wave per tile of 16 queries, keys in tiles of 16.
//      The logits are a dense contraction: v_mfma_f64_16x16x4_f64, fp16/bf16 inputs converted to
//      fp64 (products and sums then reproduce an fp64 reference to ~1e-16, which is what makes
//      the later selection reproduce it exactly, as in the decode kernels).  Online softmax in
//      fp64; P.V with v_mfma_f32_16x16x16_f16 / _bf16 (fp32 accumulation): the weights go in as
//      hi + lo 16-bit pairs straight from the registers the logits arrive in, the values as the raw
//      cache words.  Writes o_t and the log-sum-exp of every row.
//   2. wkv_prefill_scores: the column sums a_i = sum_{t >= i} exp(s_ti - lse_t): one wave per
//      tile of 16 keys, looping over the query tiles below the diagonal, the same fp64 MFMA
//      contraction again (recomputing the logits costs less than storing P^2/2 of them);
//      sums stay in registers, no atomics, fixed order.
//   3. wkv_prefill_compress: one workgroup per unit: rank of every candidate by (score, token),
//      the P - m lowest are removed; survivors are laid out in token order in the cache; every
//      run of removed tokens is folded into the survivor on its right with the weights that the
//      sequence of pairwise merges in ascending score order gives each raw row.
//
// MFMA operand layouts (one wave; g = lane / 16, x = lane % 16), as measured on gfx950:
//   both: A operand = A[row x][k = g], B operand = B[k = g][column x];
//   f64 16x16x4: result register r holds D[row g + 4r][column x];
//   f32 16x16x4: result register r holds D[row 4g + r][column x];
//   f32 16x16x16 (16-bit inputs): A operand = A[row x][k = 4g .. 4g+3], B operand = B[k = 4g .. 4g+3][column x],
//   result as f32 16x16x4.
// The reduction index of a contraction may be permuted at will as long as A and B agree, so a lane
// simply takes a contiguous quarter of its row: MFMA step kk uses element g*(D/4) + kk of both.
#include "../../include/wkv.h"
#include "wkv_internal.h"
#include <mutex>
#include "wkv_device.h"

namespace {

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float  float4_t  __attribute__((ext_vector_type(4)));

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short    short4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t  __attribute__((ext_vector_type(2)));

constexpr int TILE = 16;
constexpr int WKV_PREFILL_MAX_TOKENS = 4096;   // prompt length the compression stages in LDS (WKV_MAX_PROMPT)

// element e of a row fragment held as raw 32-bit words (two 16-bit elements per word)
template <class TT> __device__ __forceinline__ float frag_elem(const uint32_t* w, int e) {
    const uint32_t x = w[e >> 1];
    if constexpr (__is_same(TT, TF16)) {
        const half2_t h = __builtin_bit_cast(half2_t, x);
        return (e & 1) ? (float)h.y : (float)h.x;
    } else {
        return __builtin_bit_cast(float, (e & 1) ? (x & 0xFFFF0000u) : (x << 16));
    }
}

// Workgroups are dealt to the chip's eight partitions (each with its own L2) round-robin by index.
// All workgroups of a unit re-read that unit's 1-2 MB of Q, K and V, so a unit is given to ONE
// partition: workgroup b belongs to partition b % 8, and there to unit 8 * ((b / 8) / groups) + b % 8.
// (With units dealt across the partitions instead, every L2 sees the ~10 units in flight at once,
// more than it holds, and the operands come from the memory-side cache.)
constexpr int XCDS = 8;
__device__ __forceinline__ int xcd_unit(unsigned b, int groups) { return (int)((b >> 3) / groups) * XCDS + (int)(b & 7); }
inline int xcd_grid(int units, int groups) { return (units + XCDS - 1) / XCDS * XCDS * groups; }

// Four softmax weights p >= 0, each as a sum of 16-bit numbers of the cache format, packed as MFMA
// operands, so that P.V can run on the 16-bit matrix instruction without costing accuracy against
// an fp32 P.V.  Every part but the last is the running remainder cut to the format's significand
// (a mask: exact in the format, and the next remainder is exact in fp32).
//   fp16: two parts, 11 + 11 bits, the last one cut (2^-22; weights below 2^-14 lose bits below
//         2^-24 absolute);
//   bf16: three parts, 8 + 8 + 8 bits, the last one rounded to nearest.  Two parts (2^-17) were not
//         enough: in entries that cancel to 1e-4 of their row's scale the error of the weights
//         showed, about one element in 1e8 beyond the test's bound.
// No conversion of a double to 16 bits appears here: the compiler expands that one into some
// thirty integer instructions.
typedef _Float16 half2v_t __attribute__((ext_vector_type(2)));
typedef float    float2v_t __attribute__((ext_vector_type(2)));
typedef __bf16   bf16x2_t  __attribute__((ext_vector_type(2)));
template <class TT> constexpr int weight_parts() { return __is_same(TT, TF16) ? 2 : 3; }
template <class TT> __device__ __forceinline__ void split16x4(const float (&p)[4], uint2_t (&part)[weight_parts<TT>()]) {
    constexpr uint32_t keep = __is_same(TT, TF16) ? 0xFFFFE000u : 0xFFFF0000u;
    auto cut = [](float x) { return __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x) & keep); };
    if constexpr (__is_same(TT, TF16)) {
        float h[4], l[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) { h[r] = cut(p[r]); l[r] = p[r] - h[r]; }
        part[0] = uint2_t{ __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(h[0], h[1])),
                           __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(h[2], h[3])) };
        part[1] = uint2_t{ __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(l[0], l[1])),
                           __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(l[2], l[3])) };
    } else {
        auto pack = [](float a, float b) {                   // the upper halves of two words: exact for cut values
            return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, a), 0x07060302u);
        };
        auto round2 = [](float a, float b) {                 // v_cvt_pk_bf16_f32: to nearest even
            return __builtin_bit_cast(uint32_t, __builtin_convertvector(float2v_t{a, b}, bf16x2_t));
        };
        float h[4], m[4], l[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) { h[r] = cut(p[r]); const float rem = p[r] - h[r]; m[r] = cut(rem); l[r] = rem - m[r]; }
        part[0] = uint2_t{ pack(h[0], h[1]), pack(h[2], h[3]) };
        part[1] = uint2_t{ pack(m[0], m[1]), pack(m[2], m[3]) };
        part[2] = uint2_t{ round2(l[0], l[1]), round2(l[2], l[3]) };
    }
}

// D += A.B with 16-bit operands (four per lane, packed in two words) and fp32 accumulation
template <class TT> __device__ __forceinline__ float4_t mfma16(uint2_t a, uint2_t b, float4_t c) {
    if constexpr (__is_same(TT, TF16))
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, a), __builtin_bit_cast(half4_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4_t, a), __builtin_bit_cast(short4_t, b), c, 0, 0, 0);
}

// exp(x) for the arguments a softmax produces: x <= 0 (a rounding error above 0 is fine), -inf
// included.  x = (64 n + j + f) ln2 / 64 with integers n, 0 <= j < 64 and |f| <= 1/2:
// exp(x) = 2^n . 2^(j/64) . exp(f ln2 / 64); the middle factor comes from a 64-entry table in LDS,
// the last one from the Taylor quartic (remainder below r^5 / 120 < 4e-14 for |r| <= ln2 / 128), the
// first is applied by ldexp, which also takes care of gradual underflow.  Relative error about
// 1e-13 -- eight orders below what separates two scores that may legitimately be ranked either
// way -- at ten double-precision instructions, against the library routine's two dozen; on this
// part they do not overlap with the fp64 matrix instruction, so they count in full.
__device__ __forceinline__ void exp_table_init(double* tab) {
    if (threadIdx.x < 64) tab[threadIdx.x] = exp2((double)threadIdx.x * (1.0 / 64.0));
    __syncthreads();
}
__device__ __forceinline__ double exp_nonpos(double x, const double* tab) {
    const double xc = (x < -750.0) ? -750.0 : x;                         // exp(-750) = 0 in fp64; keeps n in range; NaN stays NaN
    const double kd = __builtin_rint(xc * 92.332482616893656877);        // 64 / ln 2
    const double r = fma(kd, -0.010830424696249145, xc);                 // ln 2 / 64
    const int k = (int)kd;
    const double tj = tab[k & 63];
    double p = fma(r, 1.0 / 24.0, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(tj * p, k >> 6);
}

// S^T tile: rows = 16 keys, columns = 16 queries; register r of lane (g, x) = key g + 4r, query x.
// Both operands are the exact storage values; the softmax scale is applied to the four results.
template <class TT, int D>
__device__ __forceinline__ double4_t logits_tile(const uint32_t (&kfrag)[D / 8], const double (&qd)[D / 4]) {
    // two accumulators: an MFMA that continues the chain of the one before it waits for that
    // one's result; alternating chains keeps the matrix unit issuing back to back
    double4_t s0 = {0.0, 0.0, 0.0, 0.0}, s1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int kk = 0; kk < D / 4; kk += 2) {
        s0 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)frag_elem<TT>(kfrag, kk), qd[kk], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)frag_elem<TT>(kfrag, kk + 1), qd[kk + 1], s1, 0, 0, 0);
    }
    const double scale = 1.0 / sqrt((double)D);
    return (s0 + s1) * scale;
}

// The same tile with both operands already in fp64: for a loop in which one operand never changes
// (its conversions are then paid once, not once per tile).
template <int D>
__device__ __forceinline__ double4_t logits_tile(const double (&kd)[D / 4], const double (&qd)[D / 4]) {
    double4_t s0 = {0.0, 0.0, 0.0, 0.0}, s1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int kk = 0; kk < D / 4; kk += 2) {
        s0 = __builtin_amdgcn_mfma_f64_16x16x4f64(kd[kk], qd[kk], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f64_16x16x4f64(kd[kk + 1], qd[kk + 1], s1, 0, 0, 0);
    }
    const double scale = 1.0 / sqrt((double)D);
    return (s0 + s1) * scale;
}

// ------------------------------------------------------------------ 1. rows
// q, k, v, out: [P][units][D] (token-major, as a decode step sees them one token at a time).
// lse: [units][P].  One workgroup = 4 waves = 4 consecutive query tiles of one unit.
template <class TT, int D>
__global__ __launch_bounds__(256, 2)
void wkv_prefill_rows(const void* __restrict__ q_, const void* __restrict__ k_, const void* __restrict__ v_,
                      void* __restrict__ out_, double* __restrict__ lse, int P, int units)
{
    constexpr int CH = D / 4;                 // elements of a row per lane group
    constexpr int ROWB = D * TT::BYTES;
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int g = lane >> 4, x = lane & 15;
    const int ntiles = (P + TILE - 1) / TILE;
    const int groups = (ntiles + 3) / 4;
    const int u = xcd_unit(blockIdx.x, groups);
    const int qt = (groups - 1 - (int)((blockIdx.x >> 3) % groups)) * 4 + wid;   // long rows are scheduled first
    __shared__ double etab[64];
    exp_table_init(etab);                     // every wave of the workgroup: ahead of the early exit
    if (u >= units || qt >= ntiles) return;
    const size_t tok = (size_t)units * ROWB;                              // bytes from one token to the next
    const char* qb = reinterpret_cast<const char*>(q_) + (size_t)u * ROWB;
    const char* kb = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;
    const char* vb = reinterpret_cast<const char*>(v_) + (size_t)u * ROWB;

    // the query fragment: row 16 qt + x (clamped), elements g*CH .. g*CH+CH-1, scaled, fp64
    double qd[CH];
    {
        const int tq = min(qt * TILE + x, P - 1);
        uint32_t w[CH / 2];
        load_words<CH / 2>(qb + (size_t)tq * tok + g * CH * TT::BYTES, w);
#pragma unroll
        for (int e = 0; e < CH; ++e) qd[e] = (double)frag_elem<TT>(w, e);
    }
    double mrow = -INFINITY, lrow = 0.0;      // running maximum and sum of query x (same in the 4 lanes x, x+16, ...)
    constexpr int NE = D / 16;                // output column sets: lane (g, x) owns columns NE*x .. NE*x+NE-1
    float4_t o[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) o[e] = float4_t{0.f, 0.f, 0.f, 0.f};

    // K fragment of a key tile: key 16 kt + x, the same quarter of the row as the query fragment.
    // V fragments: keys 16 kt + g + 4r, columns NE*x .. NE*x+NE-1.  Two sets of fragment registers
    // take turns: the next tile is requested into one set before the current tile is worked on
    // from the other, so no fragment is ever copied.  A lane's byte offsets inside a tile never
    // change; the tile's base address is uniform (scalar arithmetic), so a request costs one vector
    // add per load.  Only a tile that reaches past the end of the prompt clamps its rows.
    const size_t koff = (size_t)x * tok + g * CH * TT::BYTES;
    size_t voff[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) voff[r] = (size_t)(g + 4 * r) * tok + x * NE * TT::BYTES;
    auto request = [&](int kt, uint32_t (&kf)[CH / 2], uint32_t (&vf)[4][NE / 2]) __attribute__((always_inline)) {
        if (kt * TILE + TILE <= P) {                          // uniform
            const size_t base = (size_t)kt * TILE * tok;
            load_words<CH / 2>(kb + base + koff, kf);
#pragma unroll
            for (int r = 0; r < 4; ++r) load_words<NE / 2>(vb + base + voff[r], vf[r]);
        } else {
            load_words<CH / 2>(kb + (size_t)min(kt * TILE + x, P - 1) * tok + g * CH * TT::BYTES, kf);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                load_words<NE / 2>(vb + (size_t)min(kt * TILE + g + 4 * r, P - 1) * tok + x * NE * TT::BYTES, vf[r]);
        }
    };
    auto tile = [&](int kt, const uint32_t (&kfrag)[CH / 2], const uint32_t (&vfrag)[4][NE / 2]) __attribute__((always_inline)) {
        double4_t s = logits_tile<TT, D>(kfrag, qd);
        if (kt == qt) {                       // the diagonal tile: key g + 4r may be attended by query x only if <= x
#pragma unroll
            for (int r = 0; r < 4; ++r) if (g + 4 * r > x) s[r] = -INFINITY;
        }
        double tmax = fmax(fmax(s[0], s[1]), fmax(s[2], s[3]));
        tmax = pair_max<32>(pair_max<16>(tmax));               // over the four lane groups: all 16 keys of the tile
        const double mnew = fmax(mrow, tmax);                 // finite: key 16 kt + 0 <= every query of a later tile,
                                                              // and on the diagonal key x is attended by query x
        // A running maximum that has not moved needs no rescaling, and after the first few key
        // tiles of a row it rarely moves: the rescaling (an exp, the running sum and all output
        // accumulators of the wave) is skipped unless some query of the tile needs it.
        if (__any(mnew > mrow)) {
            const double resc = exp_nonpos(mrow - mnew, etab);             // 0 on the first tile (mrow = -inf), 1 where nothing moved
            lrow *= resc;
            mrow = mnew;
            const float rf = (float)resc;                     // the output rows this lane holds (queries 4g + r') by their own factor
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float f = __shfl(rf, 4 * g + r);
#pragma unroll
                for (int e = 0; e < NE; ++e) o[e][r] *= f;
            }
        }
        float p[4];
        double psum = 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r) { const double e = exp_nonpos(s[r] - mrow, etab); psum += e; p[r] = (float)e; }
        psum = rows_sum(psum);
        lrow += psum;
        // O[query][column] += sum over keys P[query][key] V[key][column] with the 16-bit matrix
        // instruction (k = 16 keys at once): lane (g, x) supplies k-slots 4g + r, which stand for the
        // keys g + 4r it already holds -- as A operand P[query x][key g + 4r], as B operand
        // V[key g + 4r][column NE*x + e], the raw cache values.  P goes in as a sum of 16-bit parts.
        uint2_t pa[weight_parts<TT>()];
        split16x4<TT>(p, pa);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;      // high / low halves of two words
            const uint2_t vb = { __builtin_amdgcn_perm(vfrag[1][e >> 1], vfrag[0][e >> 1], sel),
                                 __builtin_amdgcn_perm(vfrag[3][e >> 1], vfrag[2][e >> 1], sel) };
#pragma unroll
            for (int w = 0; w < weight_parts<TT>(); ++w) o[e] = mfma16<TT>(pa[w], vb, o[e]);
        }
    };
    uint32_t kf0[CH / 2], vf0[4][NE / 2], kf1[CH / 2], vf1[4][NE / 2];
    request(0, kf0, vf0);
    for (int kt = 0; kt <= qt; kt += 2) {
        request(min(kt + 1, qt), kf1, vf1);                   // past the last tile: a repeat, unused
        tile(kt, kf0, vf0);
        if (kt + 1 > qt) break;
        request(min(kt + 2, qt), kf0, vf0);
        tile(kt + 1, kf1, vf1);
    }

    // o_t = O / l, log-sum-exp = m + log l
    const float linv = (float)(1.0 / lrow);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int t = qt * TILE + 4 * g + r;
        const float f = __shfl(linv, 4 * g + r);
        if (t < P && out_ != nullptr) {
            char* dst = reinterpret_cast<char*>(out_) + (size_t)t * tok + (size_t)u * ROWB + x * NE * TT::BYTES;
#pragma unroll
            for (int e = 0; e < NE; ++e) store_elem<TT>(dst, e, o[e][r] * f);
        }
    }
    if (g == 0 && qt * TILE + x < P) lse[(size_t)u * P + qt * TILE + x] = mrow + log(lrow);
}

// ------------------------------------------------------------------ 2. scores
// a[u][i] = sum over rows t >= i of exp(s_ti - lse_t).  One wave per key tile.
template <class TT, int D>
__global__ __launch_bounds__(256)
void wkv_prefill_scores(const void* __restrict__ q_, const void* __restrict__ k_, const double* __restrict__ lse,
                        double* __restrict__ a, int P, int units)
{
    constexpr int CH = D / 4;
    constexpr int ROWB = D * TT::BYTES;
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int g = lane >> 4, x = lane & 15;
    const int ntiles = (P + TILE - 1) / TILE;
    const int groups = (ntiles + 3) / 4;
    const int u = xcd_unit(blockIdx.x, groups);
    const int kt = (int)((blockIdx.x >> 3) % groups) * 4 + wid;           // low key tiles have the most rows: first
    __shared__ double etab[64];
    exp_table_init(etab);                     // every wave of the workgroup: ahead of the early exit
    if (u >= units || kt >= ntiles) return;
    const size_t tok = (size_t)units * ROWB;
    const char* qb = reinterpret_cast<const char*>(q_) + (size_t)u * ROWB;
    const char* kb = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;

    // the wave's key fragment never changes: converted to fp64 once (64 registers), not once per query tile
    double kd[CH];
    {
        uint32_t kfrag[CH / 2];
        load_words<CH / 2>(kb + (size_t)min(kt * TILE + x, P - 1) * tok + g * CH * TT::BYTES, kfrag);
#pragma unroll
        for (int e = 0; e < CH; ++e) kd[e] = (double)frag_elem<TT>(kfrag, e);
    }
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    uint32_t wnext[CH / 2];
    double lnext;
    auto request = [&](int qt) {
        const int tqc = min(qt * TILE + x, P - 1);
        load_words<CH / 2>(qb + (size_t)tqc * tok + g * CH * TT::BYTES, wnext);
        lnext = lse[(size_t)u * P + tqc];
    };
    // Software pipeline: the MFMA chain of the next query tile is issued in the same stretch of
    // straight-line code as the exponentials of the current one, so the matrix unit and the
    // vector unit of a SIMD work at the same time.  (Waves left to themselves run in lockstep --
    // all in their MFMA chain, then all in their exponentials -- and the two units take turns.)
    request(kt);
    double4_t s_cur;
    double l_cur = lnext;
    {
        double qd[CH];
#pragma unroll
        for (int e = 0; e < CH; ++e) qd[e] = (double)frag_elem<TT>(wnext, e);
        request(min(kt + 1, ntiles - 1));
        s_cur = logits_tile<D>(kd, qd);
    }
    for (int qt = kt; qt < ntiles; ++qt) {
        const int tq = qt * TILE + x;
        double qd[CH];
#pragma unroll
        for (int e = 0; e < CH; ++e) qd[e] = (double)frag_elem<TT>(wnext, e);
        const double l_next = lnext;
        request(min(qt + 2, ntiles - 1));
        __builtin_amdgcn_sched_barrier(0);                                 // the requests are issued here, not later
        double4_t s_next = logits_tile<D>(kd, qd);                 // tile qt + 1 (a repeat on the last round)
        // The fragment just requested may be touched only once this chain has been issued: without
        // these opaque uses the compiler converts it right behind its request, i.e. every round
        // waits for the loads it has just issued.
        {
            double pin = s_next[0];
#pragma unroll
            for (int w = 0; w < CH / 2; ++w) asm volatile("" : "+v"(pin), "+v"(wnext[w]));
            asm volatile("" : "+v"(pin), "+v"(lnext));
            s_next[0] = pin;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int key = kt * TILE + g + 4 * r;
            const bool on = tq < P && key <= tq;                           // causal, and inside the prompt
            acc[r] += exp_nonpos(on ? s_cur[r] - l_cur : -INFINITY, etab);  // exp(-inf) = 0; no branch
        }
        s_cur = s_next;
        l_cur = l_next;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const double c = row_allsum(acc[r]);                               // over the 16 queries x
        const int key = kt * TILE + g + 4 * r;
        if (x == 0 && key < P) a[(size_t)u * P + key] = c;
    }
}

// ------------------------------------------------------------------ 3. compress
// One workgroup per unit.  Scores are fixed during the compression, so the P - L tokens that
// the repeated selection removes are the candidates of lowest (score, token), in that order.
//
// Values.  A removed token j folds into the nearest token on its right that is still present
// when its turn comes, i.e. the nearest one with a higher rank (survivors rank above everything):
// its parent.  The merges therefore form a forest whose roots are the survivors, and a node
// receives its children in ascending rank.  With s the scores, a child c of p contributes
//     g_c * prod_{children c' of p ranked after c} f_c',   f_c' = s_p / (s_c' + s_p),  g_c = s_c / (s_c + s_p)
// of its accumulated value to p's, and p's own raw value keeps prod_{children} f_c'.  The weight
// of a raw token in its survivor's row is the product of these coefficients up the tree, and the
// row is the weighted sum of the raw rows of the run -- the same numbers as the sequence of pairwise
// merges (Algorithm 1) in fp64, with no dependent chain of row updates.  Rows are rounded to the
// cache format once, when they are written.
//
// LDS: sc[P] score, then list products, finally weight | ae[P] f, then edge coefficient | a0[P] g, then
//      own coefficient | slot[P] | wcnt[NT] | rk[P] rank (16 bit) | par[P] parent (16 bit) |
//      ptr[P] list successor (16 bit) | bmax[64].  The sort keys borrow ae[], a0[] and slot[].
template <class TT, int D>
__global__ __launch_bounds__(1024)
void wkv_prefill_compress(WkvCache c, const void* __restrict__ k_, const void* __restrict__ v_,
                          const double* __restrict__ a, int P)
{
    constexpr int ROWB = D * TT::BYTES;
    constexpr int EPW = (D + 63) / 64;
    const int tid = threadIdx.x, NT = blockDim.x, lane = tid & 63, wid = tid >> 6, NW = NT >> 6;
    const int u = blockIdx.x, m = c.m;
    const size_t tok = (size_t)c.units * ROWB;
    const char* kb = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;
    const char* vb = reinterpret_cast<const char*>(v_) + (size_t)u * ROWB;
    char* Kc = reinterpret_cast<char*>(c.K) + (size_t)u * m * ROWB;
    char* Vc = reinterpret_cast<char*>(c.V) + (size_t)u * m * ROWB;
    double*  au = c.a + (size_t)u * m;
    int32_t* pu = c.pos + (size_t)u * m;
    int32_t* nu = c.nxt + (size_t)u * m;
    const double* ap = a + (size_t)u * P;

    extern __shared__ double lds[];
    double*   sc   = lds;
    double*   ae   = sc + P;
    double*   a0   = ae + P;
    int32_t*  slot = reinterpret_cast<int32_t*>(a0 + P);      // slot of a survivor, -1 for a removed token
    int32_t*  wcnt = slot + P;
    uint16_t* rk   = reinterpret_cast<uint16_t*>(wcnt + NT);
    uint16_t* par  = rk + P;
    uint16_t* ptr  = par + P;                                 // successor in the list a product runs along
    uint16_t* bmax = ptr + P;                                 // [64] highest rank in a block of 64 tokens
    const int L = (P < m) ? P : m;
    const int nrem = P - L;                                   // tokens to remove
    const int lo = c.n_sink, hi = P - c.R;                    // candidates: lo <= token < hi

    for (int i = tid; i < P; i += NT) {
        const double ai = ap[i];
        double s = (c.score_mode == 0) ? ai / (double)(P - i) : ai;       // abar = a / n, n_i = P - i
        if (!(s == s) || s == INFINITY) { s = INFINITY; atomicAdd(&c.status[1], 1); }
        sc[i] = s;
    }
    __syncthreads();
    // rank among the candidates by (score, token); the nrem lowest are removed.  A bitonic sort of
    // (score bits, token) in LDS (the key arrays borrow ae[], a0[] and slot[], not yet in use).
    for (int i = tid; i < P; i += NT) rk[i] = 0xFFFF;
    if (nrem > 0) {
        unsigned long long* key = reinterpret_cast<unsigned long long*>(ae);   // [N2]
        uint16_t* kid = reinterpret_cast<uint16_t*>(slot);                     // [N2]
        int N2 = 1;
        while (N2 < P) N2 <<= 1;
        for (int i = tid; i < N2; i += NT) {
            unsigned long long kb64 = ~0ull;                                   // not a candidate, or padding: sorts last
            if (i >= lo && i < hi) {
                const unsigned long long bits = (unsigned long long)__double_as_longlong(sc[i]);
                kb64 = (bits >> 63) ? ~bits : (bits | 0x8000000000000000ull);  // order of the doubles as order of integers
                if (kb64 == ~0ull) kb64 = ~0ull - 1;                           // (no score maps there; keep the sentinel unique)
            }
            key[i] = kb64;
            kid[i] = (uint16_t)i;
        }
        __syncthreads();
        for (int k = 2; k <= N2; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int t = tid; t < (N2 >> 1); t += NT) {
                    const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), l = i | j;
                    const unsigned long long ki = key[i], kl = key[l];
                    const uint16_t di = kid[i], dl = kid[l];
                    const bool gt = ki > kl || (ki == kl && di > dl);
                    if (gt == ((i & k) == 0)) { key[i] = kl; key[l] = ki; kid[i] = dl; kid[l] = di; }
                }
                __syncthreads();
            }
        }
        for (int r = tid; r < nrem; r += NT) rk[kid[r]] = (uint16_t)r;         // the nrem lowest keys are candidates
        __syncthreads();
    } else {
        __syncthreads();
    }
    for (int i = tid; i < P; i += NT) slot[i] = (rk[i] != 0xFFFF) ? -1 : 0;
    __syncthreads();
    // survivors get consecutive slots in token order: exclusive scan over the keep flags
    const int per = (P + NT - 1) / NT;
    const int b0 = min(tid * per, P), b1 = min(b0 + per, P);
    int mine = 0;
    for (int i = b0; i < b1; ++i) mine += (slot[i] == 0) ? 1 : 0;
    wcnt[tid] = mine;
    __syncthreads();
    if (tid == 0) { int run = 0; for (int w = 0; w < NT; ++w) { const int t = wcnt[w]; wcnt[w] = run; run += t; } }
    __syncthreads();
    {
        int sidx = wcnt[tid];
        for (int i = b0; i < b1; ++i) if (slot[i] == 0) slot[i] = sidx++;
    }
    __syncthreads();
    // score sums, token indices, links and keys of the survivors
    for (int i = tid; i < P; i += NT) {
        const int sidx = slot[i];
        if (sidx >= 0) { au[sidx] = ap[i]; pu[sidx] = i; nu[sidx] = (sidx + 1 < L) ? sidx + 1 : -1; }
    }
    for (int i = wid; i < P; i += NW) {                       // one wave per row
        const int sidx = slot[i];
        if (sidx < 0) continue;
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const int col = lane + 64 * e;
            if (col < D) store_bits<TT>(Kc + (size_t)sidx * ROWB, col, load_bits<TT>(kb + (size_t)i * tok, col));
        }
    }

    const bool merging = c.merge_mode == 0 && nrem > 0;
    if (merging) {
        // Parent of a removed token: the nearest token to its right that outranks it (survivors
        // outrank everything: rank 0xFFFF); also the nearest one to its LEFT that outranks it.  Both by
        // a search that skips whole blocks of 64 tokens whose highest rank is too low, so a token
        // looks at < 200 entries however long the runs are.
        constexpr int NIL = 0xFFFF;
        const int nblk = (P + 63) >> 6;
        for (int b = wid; b < nblk; b += NW) {
            const int i = b * 64 + lane;
            int r = (i < P) ? (int)rk[i] : 0;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) r = max(r, __shfl_xor(r, off));
            if (lane == 0) bmax[b] = (uint16_t)r;
        }
        __syncthreads();
        for (int i = tid; i < P; i += NT) {
            int right = i, left = NIL;                        // a survivor is its own parent
            if (slot[i] < 0) {
                const int ri = rk[i];
                {
                    const int e = min((i | 63) + 1, P);
                    int k = i + 1;
                    while (k < e && rk[k] <= ri) ++k;
                    if (k == e) {                              // a survivor lies to the right (the newest tokens are never removed)
                        int b = (i >> 6) + 1;
                        while (b < nblk - 1 && bmax[b] <= ri) ++b;
                        k = b * 64;
                        while (k < P - 1 && rk[k] <= ri) ++k;
                    }
                    right = k;
                }
                {
                    const int e = (i & ~63) - 1;
                    int k = i - 1;
                    while (k > e && rk[k] <= ri) --k;
                    if (k == e) {
                        int b = (i >> 6) - 1;
                        while (b >= 0 && bmax[b] <= ri) --b;
                        if (b >= 0) { k = b * 64 + 63; while (rk[k] <= ri) --k; }   // bmax[b] > ri: the scan ends inside block b
                        else k = -1;
                    }
                    left = (k >= 0) ? k : NIL;
                }
            }
            par[i] = (uint16_t)right;
            ptr[i] = (uint16_t)left;
        }
        __syncthreads();
        // f and g of every removed token with respect to its parent (one division each): f -> ae[], g -> a0[]
        for (int i = tid; i < P; i += NT) {
            if (slot[i] >= 0) continue;
            const double sp = sc[par[i]], si = sc[i], den = si + sp;
            ae[i] = (den > 0.0) ? sp / den : 0.5;
            a0[i] = (den > 0.0) ? si / den : 0.5;
            if (!(den > 0.0)) atomicAdd(&c.status[0], 1);
        }
        __syncthreads();
        // Products along lists by pointer jumping: every removed token i has a successor (held in
        // ptr[i], NIL at the end); on return sc[i] = product of val[] over all tokens after i in its
        // list.  log2(list length) rounds, each token's update held in registers across a barrier.
        // sc[] (the scores) is free from here on.
        constexpr int MAXTOK = (WKV_PREFILL_MAX_TOKENS + 1023) / 1024;   // tokens per thread
        auto list_products = [&](const double* val) {
            for (int i = tid; i < P; i += NT) {
                const int j = (slot[i] < 0) ? (int)ptr[i] : NIL;
                sc[i] = (j != NIL) ? val[j] : 1.0;
            }
            __syncthreads();
            for (;;) {
                double wn[MAXTOK];
                int jn[MAXTOK];
                int pending = 0;
#pragma unroll
                for (int kk = 0; kk < MAXTOK; ++kk) {
                    const int i = tid + kk * NT;
                    jn[kk] = NIL;
                    wn[kk] = 1.0;
                    if (i < P && slot[i] < 0) {
                        const int j = ptr[i];
                        wn[kk] = sc[i];
                        if (j != NIL) { wn[kk] *= sc[j]; jn[kk] = ptr[j]; pending |= (jn[kk] != NIL) ? 1 : 0; }
                    }
                }
                __syncthreads();
#pragma unroll
                for (int kk = 0; kk < MAXTOK; ++kk) {
                    const int i = tid + kk * NT;
                    if (i < P && slot[i] < 0) { sc[i] = wn[kk]; ptr[i] = (uint16_t)jn[kk]; }
                }
                if (!__syncthreads_or(pending)) break;
            }
        };
        // Siblings.  The children of p, from p - 1 leftwards, have ascending rank, i.e. they are merged
        // into p in that order; the one after child i is the nearest token on i's left that outranks
        // i, as long as it does not outrank p as well.  ptr[] holds that left neighbour: cut the lists.
        for (int i = tid; i < P; i += NT) {
            if (slot[i] >= 0) continue;
            const int l = ptr[i];
            if (l != NIL && rk[l] >= rk[par[i]]) ptr[i] = NIL;     // (a survivor has rank 0xFFFF)
        }
        __syncthreads();
        list_products(ae);                                     // sc[i] = product of f over the siblings merged after i
        // edge coefficient of a removed token within its parent: g_i times the f of the later siblings;
        // own coefficient of any token: the f of all its children = f of the first child (the token on
        // its left, if that is a child) times the f of that child's later siblings.
        {
            double edge[MAXTOK], own[MAXTOK];
#pragma unroll
            for (int kk = 0; kk < MAXTOK; ++kk) {
                const int i = tid + kk * NT;
                edge[kk] = 0.0; own[kk] = 1.0;
                if (i >= P) continue;
                if (slot[i] < 0) edge[kk] = a0[i] * sc[i];
                if (i > 0 && slot[i - 1] < 0 && par[i - 1] == i) own[kk] = ae[i - 1] * sc[i - 1];
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < MAXTOK; ++kk) {
                const int i = tid + kk * NT;
                if (i >= P) continue;
                if (slot[i] < 0) ae[i] = edge[kk];
                a0[i] = own[kk];
            }
        }
        // Ancestors: the weight of a raw token in its survivor's row is its own coefficient times the
        // edge coefficients up the tree.
        for (int i = tid; i < P; i += NT) {
            if (slot[i] >= 0) continue;
            const int q = par[i];
            ptr[i] = (slot[q] < 0) ? (uint16_t)q : (uint16_t)NIL;
        }
        __syncthreads();
        list_products(ae);                                     // sc[i] = product of the edge coefficients of i's removed ancestors
        for (int i = tid; i < P; i += NT)
            if (slot[i] < 0) sc[i] *= ae[i] * a0[i];
        __syncthreads();
    }
    // acc += sum over rows k = first, first + stride, ... <= last of weight(k) * V_k, where the last
    // row of a run is the survivor itself (own coefficient).  Eight rows are requested at a time:
    // the sum is a chain of dependent FMAs, the loads need not be.
    auto weighted_rows = [&](double (&acc)[EPW], int first, int last, int stride) {
        for (int k0 = first; k0 <= last; k0 += 8 * stride) {
            uint32_t raw[8][EPW];
            double w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int k = k0 + j * stride;
                const int kc = min(k, last);
                w[j] = (k > last) ? 0.0 : (k < last) ? sc[kc] : a0[last];
#pragma unroll
                for (int e = 0; e < EPW; ++e)
                    raw[j][e] = load_bits<TT>(vb + (size_t)kc * tok, min(lane + 64 * e, D - 1));
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int e = 0; e < EPW; ++e) acc[e] = fma(w[j], (double)bits_elem<TT>(raw[j][e]), acc[e]);
        }
    };
    // values of the survivors.  rk[] is free now: it takes the number of tokens that fold into a survivor.
    constexpr int LONG = 32;                                  // runs from this length on are summed by the whole workgroup
    const bool coop = merging && P >= NW * D;                 // (the partial sums borrow ae[], P doubles)
    for (int i = tid; i < P; i += NT) {
        if (slot[i] < 0) continue;
        int i0 = i - 1;
        while (i0 >= 0 && slot[i0] < 0) --i0;                  // previous survivor (or -1)
        rk[i] = (uint16_t)(merging ? i - 1 - i0 : 0);
    }
    __syncthreads();
    for (int i = wid; i < P; i += NW) {                       // short runs: one wave per survivor
        const int sidx = slot[i];
        if (sidx < 0) continue;
        const int len = rk[i];
        if (coop && len >= LONG) continue;
        const char* own = vb + (size_t)i * tok;
        if (len == 0) {                                        // nothing folds into this token
#pragma unroll
            for (int e = 0; e < EPW; ++e) {
                const int col = lane + 64 * e;
                if (col < D) store_bits<TT>(Vc + (size_t)sidx * ROWB, col, load_bits<TT>(own, col));
            }
            continue;
        }
        double acc[EPW];
#pragma unroll
        for (int e = 0; e < EPW; ++e) acc[e] = 0.0;
        weighted_rows(acc, i - len, i, 1);
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const int col = lane + 64 * e;
            if (col < D) store_elem_f64<TT>(Vc + (size_t)sidx * ROWB, col, acc[e]);
        }
    }
    if (coop) {                                                // long runs: every wave takes every NW-th row
        double* part = ae;                                     // [NW][D]
        for (int i = 0; i < P; ++i) {                          // uniform over the workgroup
            if (slot[i] < 0 || rk[i] < LONG) continue;
            const int len = rk[i];
            double acc[EPW];
#pragma unroll
            for (int e = 0; e < EPW; ++e) acc[e] = 0.0;
            weighted_rows(acc, i - len + wid, i, NW);
            __syncthreads();                                   // the previous long run's partial sums have been read
#pragma unroll
            for (int e = 0; e < EPW; ++e) {
                const int col = lane + 64 * e;
                if (col < D) part[wid * D + col] = acc[e];
            }
            __syncthreads();
            if (tid < D) {
                double y = 0.0;
                for (int w = 0; w < NW; ++w) y += part[w * D + tid];
                store_elem_f64<TT>(Vc + (size_t)slot[i] * ROWB, tid, y);
            }
        }
    }
}

template <class TT, int D>
hipError_t run(const WkvCache& c, const void* q, const void* k, const void* v, void* out,
               double* lse, double* a, int P, hipStream_t stream)
{
    const int ntiles = (P + TILE - 1) / TILE, groups = (ntiles + 3) / 4;
    hipLaunchKernelGGL((wkv_prefill_rows<TT, D>), dim3(xcd_grid(c.units, groups)), dim3(256), 0, stream, q, k, v, out, lse, P, c.units);
    hipLaunchKernelGGL((wkv_prefill_scores<TT, D>), dim3(xcd_grid(c.units, groups)), dim3(256), 0, stream, q, k, lse, a, P, c.units);
    const size_t lds = wkv_prefill_lds_bytes(P);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wkv_prefill_compress<TT, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((wkv_prefill_compress<TT, D>), dim3(c.units), dim3(1024), lds, stream, c, k, v, a, P);
    return hipGetLastError();
}

}  // namespace

size_t wkv_prefill_lds_bytes(int P) { return (size_t)P * 34 + 1024 * 4 + 64 * 2; }

// ---- scratch of wkv_prefill_noalloc: a static device array, so that the call allocates nothing.
// Every GPU holds its own copy at its own address; in host code the array's name is only a
// stand-in for hipGetSymbolAddress, never an address to hand to a kernel.
static __device__ __align__(256) unsigned char wkv_noalloc_scratch[WKV_NOALLOC_SCRATCH_BYTES];

hipError_t wkv_prefill_static_scratch(int device, double** ptr)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void* addr[MAX_DEVICES] = {};
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(wkv_noalloc_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[device] = p;
    }
    *ptr = static_cast<double*>(addr[device]);
    return hipSuccess;
}

hipError_t wkv_launch_prefill(const WkvCache& c, int dtype, int head_dim, const void* q, const void* k,
                              const void* v, void* out, double* lse, double* a, int P, hipStream_t stream)
{
    if (dtype == 1 && head_dim == 64)  return run<TF16, 64>(c, q, k, v, out, lse, a, P, stream);
    if (dtype == 1 && head_dim == 128) return run<TF16, 128>(c, q, k, v, out, lse, a, P, stream);
    if (dtype == 2 && head_dim == 64)  return run<TBF16, 64>(c, q, k, v, out, lse, a, P, stream);
    if (dtype == 2 && head_dim == 128) return run<TBF16, 128>(c, q, k, v, out, lse, a, P, stream);
    return hipErrorInvalidValue;
}
