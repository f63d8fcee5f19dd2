// One WeightedKV decode step for every (sequence, head) unit, gfx950.
//
// Per unit and per incoming token (Algorithm 1 and Sections III-A, IV of the
// WeightedKV paper, arXiv 2503.01330):
//   append k_t, v_t; A_t = softmax(q_t^T K_t / sqrt(d)); o_t = A_t^T V_t;
//   a += A_t, n += 1; if more than m entries: abar = a/n, j = arg-min abar over
//   unprotected entries, V[right(j)] <- convex merge weighted by abar, drop j.
//
// Mapping to CDNA4
//   * one workgroup per unit; a K or V row (d elements) is spread over 16
//     lanes, so one wave64 load instruction fetches 4 consecutive rows (1 KiB
//     for d=128 half precision) fully coalesced, and the 16-lane dot-product
//     reduction is four DPP steps (quad_perm, quad_perm, row_half_mirror,
//     row_mirror) with no LDS traffic;
//   * K and V are each streamed exactly once.  Phase 1 streams K and leaves the
//     logit of every entry, in fp64, in LDS.  Phase 2 streams V and accumulates
//     exp(logit - max) . V in fp32 (fp64 for an fp32 cache);
//   * phase 2 is wave-specialised: wave 0 does the score bookkeeping of
//     Algorithm 1 (softmax denominator, a += A_t, abar = a/n, arg-min, right
//     neighbour, merge weights) from the staged logit row while the other waves
//     stream V, so the dependent chain of the compression hides behind the
//     second half of the memory traffic;
//   * the bookkeeping is fp64 throughout.  That costs one extra convert per K
//     element on a memory-bound kernel and makes the eviction decision reproduce
//     an fp64 reference exactly (differences ~1e-15 relative in abar) instead of
//     drifting apart after the first near-tie;
//   * the path is a GEMV per unit with no reuse across units: no MFMA.
//
// Slot order in memory is not token order (see wkv_internal.h): the incoming
// token is attended straight from the caller's k_new/v_new buffers and then
// written into the slot the victim vacates, so compression moves no K/V row.
//
// Latency matters as much as bandwidth here (one launch streams ~50 MB, ~7 us
// at peak): everything the bookkeeping needs from memory (score sums, token
// positions) is requested before the streaming loop starts, the workgroup meets
// at two barriers only, and wave-level reductions use DPP row operations plus
// v_readlane, not LDS permutes.
#include "wkv_internal.h"

#include <math.h>

namespace {

constexpr int ROW_LANES = 16;   // lanes that share one K/V row

struct TF32  { static constexpr int BYTES = 4; using soft_t = double; };
struct TF16  { static constexpr int BYTES = 2; using soft_t = float;  };
struct TBF16 { static constexpr int BYTES = 2; using soft_t = float;  };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------- raw row I/O
template <int NW>
__device__ __forceinline__ void load_words(const void* p, uint32_t (&w)[NW]) {
    if constexpr (NW == 2) {
        uint2 x = *reinterpret_cast<const uint2*>(p);
        w[0] = x.x; w[1] = x.y;
    } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i) {
            uint4 x = reinterpret_cast<const uint4*>(p)[i];
            w[4 * i] = x.x; w[4 * i + 1] = x.y; w[4 * i + 2] = x.z; w[4 * i + 3] = x.w;
        }
    }
}

template <int NW>
__device__ __forceinline__ void store_words(void* p, const uint32_t (&w)[NW]) {
    if constexpr (NW == 2) {
        *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]);
    } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i)
            reinterpret_cast<uint4*>(p)[i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
    }
}

// storage words -> exact fp32 values
template <class TT, int EPL, int NW>
__device__ __forceinline__ void decode(const uint32_t (&w)[NW], float (&x)[EPL]) {
    if constexpr (TT::BYTES == 4) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) x[e] = __builtin_bit_cast(float, w[e]);
    } else if constexpr (__is_same(TT, TF16)) {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            half2_t h = __builtin_bit_cast(half2_t, w[i]);
            x[2 * i] = (float)h.x; x[2 * i + 1] = (float)h.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            x[2 * i]     = __builtin_bit_cast(float, w[i] << 16);
            x[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
        }
    }
}

// one storage element -> fp32 / fp32 -> one storage element (round to nearest even)
template <class TT> __device__ __forceinline__ float load_elem(const void* base, int idx) {
    if constexpr (TT::BYTES == 4) return reinterpret_cast<const float*>(base)[idx];
    else if constexpr (__is_same(TT, TF16)) return (float)reinterpret_cast<const _Float16*>(base)[idx];
    else return __builtin_bit_cast(float, (uint32_t)reinterpret_cast<const uint16_t*>(base)[idx] << 16);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40);   // NaN stays NaN
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

template <class TT> __device__ __forceinline__ void store_elem(void* base, int idx, float f) {
    if constexpr (TT::BYTES == 4) reinterpret_cast<float*>(base)[idx] = f;
    else if constexpr (__is_same(TT, TF16)) reinterpret_cast<_Float16*>(base)[idx] = (_Float16)f;
    else reinterpret_cast<uint16_t*>(base)[idx] = f32_to_bf16_rne(f);
}

// fp64 -> fp32 with round-to-odd, so that the following fp32 -> 16-bit rounding
// (nearest even) gives the correctly rounded 16-bit value of the fp64 input.
__device__ __forceinline__ float f64_to_f32_round_odd(double x) {
    float f = (float)x;
    double back = (double)f;
    if (back != x && __builtin_isfinite(f)) {
        uint32_t b = __builtin_bit_cast(uint32_t, f);
        if (fabs(back) > fabs(x)) b -= 1u;   // step to the neighbour nearer zero
        b |= 1u;                             // inexact: force the odd neighbour
        f = __builtin_bit_cast(float, b);
    }
    return f;
}

template <class TT> __device__ __forceinline__ void store_elem_f64(void* base, int idx, double x) {
    if constexpr (TT::BYTES == 4) reinterpret_cast<float*>(base)[idx] = (float)x;
    else store_elem<TT>(base, idx, f64_to_f32_round_odd(x));
}

// ------------------------------------------------------------- lane exchange
template <int CTRL, class X> __device__ __forceinline__ X dpp(X x) {
    return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false);
}

// Sum over the 16 lanes of a DPP row; every lane ends with the same bits.
template <class X> __device__ __forceinline__ X row_allsum(X x) {
    x += dpp<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp<0x141>(x);   // row_half_mirror
    x += dpp<0x140>(x);   // row_mirror
    return x;
}

__device__ __forceinline__ float  soft_exp(float x)  { return __expf(x); }
__device__ __forceinline__ double soft_exp(double x) { return exp(x); }

template <class S> __device__ __forceinline__ S neg_inf() { return (S)(-INFINITY); }

// scale factor exp(m - M) of a partial whose running maximum is m; 0 for an empty partial
template <class S> __device__ __forceinline__ S rescale(S m, S M) {
    return (m == neg_inf<S>()) ? (S)0 : soft_exp(m - M);
}

// ------------------------------------------------------- wave-level reductions
// All 64 lanes active.  Results are uniform across the wave and depend only on
// the data (fixed combination order), never on timing.
__device__ __forceinline__ double readlane_f64(double x, int l) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), l);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), l);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum(double x) {
    x = row_allsum(x);
    return ((readlane_f64(x, 0) + readlane_f64(x, 16)) + readlane_f64(x, 32)) + readlane_f64(x, 48);
}

__device__ __forceinline__ int wave_sum(int x) {
    x = row_allsum(x);
    return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) +
           __builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48);
}

// candidate victim: lexicographic (score, token index), so ties go to the oldest token
struct Best { double s; int pos; int phys; };

__device__ __forceinline__ bool better(double s, int pos, const Best& b) {
    return (s < b.s) || (s == b.s && pos < b.pos);
}

template <int CTRL> __device__ __forceinline__ void best_step(Best& b) {
    const Best o = { dpp<CTRL>(b.s), dpp<CTRL>(b.pos), dpp<CTRL>(b.phys) };
    if (better(o.s, o.pos, b)) b = o;
}

__device__ __forceinline__ Best wave_argmin(Best b) {
    best_step<0xB1>(b); best_step<0x4E>(b); best_step<0x141>(b); best_step<0x140>(b);
    Best r = { readlane_f64(b.s, 0), __builtin_amdgcn_readlane(b.pos, 0), __builtin_amdgcn_readlane(b.phys, 0) };
#pragma unroll
    for (int l = 16; l < 64; l += 16) {
        const Best o = { readlane_f64(b.s, l), __builtin_amdgcn_readlane(b.pos, l),
                         __builtin_amdgcn_readlane(b.phys, l) };
        if (better(o.s, o.pos, r)) r = o;
    }
    return r;
}

// right-hand neighbour of the victim: the live entry with the smallest token
// index above the victim's (token indices are unique), with its slot and score
struct Next { int pos; int phys; double s; };

template <int CTRL> __device__ __forceinline__ void next_step(Next& n) {
    const Next o = { dpp<CTRL>(n.pos), dpp<CTRL>(n.phys), dpp<CTRL>(n.s) };
    if (o.pos < n.pos) n = o;
}

__device__ __forceinline__ Next wave_next(Next n) {
    next_step<0xB1>(n); next_step<0x4E>(n); next_step<0x141>(n); next_step<0x140>(n);
    Next r = { __builtin_amdgcn_readlane(n.pos, 0), __builtin_amdgcn_readlane(n.phys, 0), readlane_f64(n.s, 0) };
#pragma unroll
    for (int l = 16; l < 64; l += 16) {
        const Next o = { __builtin_amdgcn_readlane(n.pos, l), __builtin_amdgcn_readlane(n.phys, l),
                         readlane_f64(n.s, l) };
        if (o.pos < r.pos) r = o;
    }
    return r;
}

constexpr int MAXPT = 4;       // entries whose a/pos one thread fetches ahead of the streaming loop
constexpr int NONE_POS = 0x7FFFFFFF;

// ------------------------------------------------------------------ the kernel
// Entries attended in step t: the Lc = min(t, m) cached slots, then the incoming
// token as entry Lc (its row is read from k_new / v_new).  L = Lc + 1.
template <class TT, int D, int U>
__global__ __launch_bounds__(1024)
void wkv_step_kernel(WkvCache c, const void* __restrict__ q_, const void* __restrict__ k_,
                     const void* __restrict__ v_, void* __restrict__ out_, int t)
{
    using S = typename TT::soft_t;
    constexpr int EPL  = D / ROW_LANES;          // elements of a row per lane
    constexpr int NW32 = EPL * TT::BYTES / 4;    // 32-bit words per lane per row
    constexpr int ROWB = D * TT::BYTES;          // bytes per row
    constexpr int LANEB = EPL * TT::BYTES;       // bytes per lane per row
    constexpr int EPW  = (D + 63) / 64;          // row elements per lane of the bookkeeping wave

    const int tid = threadIdx.x, NT = blockDim.x;
    const int NG = NT >> 4, gid = tid >> 4, sub = tid & 15;
    const int NW = NT >> 6, wid = tid >> 6, lane = tid & 63;
    const int u = blockIdx.x;
    const int m = c.m;
    const int Lc = (t < m) ? t : m;                        // cached entries
    const int L = Lc + 1;                                  // entries attended
    const bool compress = t >= m;                          // the cache would exceed m

    // ---- LDS carve-up
    extern __shared__ double lds[];
    double* sl   = lds;                                    // [m+1] fp64 logit of every entry
    double* al   = sl + m + 1;                             // [m+1] score sums a
    double* wmax = al + m + 1;                             // [16] per-wave maximum logit
    S*      part = reinterpret_cast<S*>(wmax + 16);        // [NW][D] per-wave P.V partials
    S*      plw  = part + NW * D;                          // [16] per-wave sum of weights
    int*    pl   = reinterpret_cast<int*>(plw + 16);       // [m+1] token index of every entry

    char*       Kc = reinterpret_cast<char*>(c.K) + (size_t)u * m * ROWB;
    char*       Vc = reinterpret_cast<char*>(c.V) + (size_t)u * m * ROWB;
    const char* qu = reinterpret_cast<const char*>(q_) + (size_t)u * ROWB;
    const char* ku = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;
    const char* vu = reinterpret_cast<const char*>(v_) + (size_t)u * ROWB;
    double*  au = c.a + (size_t)u * m;
    int32_t* pu = c.pos + (size_t)u * m;

    // ---- everything the bookkeeping needs from memory, requested before the streaming loop
    double a_reg[MAXPT];
    int pos_reg[MAXPT];
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        const int i = tid + k * NT;
        a_reg[k] = (i < Lc) ? au[i] : 0.0;                 // a = [a, 0]
        pos_reg[k] = (i < Lc) ? pu[i] : ((i == Lc) ? t : NONE_POS);
    }
    float knew_e[EPW], vnew_e[EPW];                        // the incoming row, for wave 0's write-back
    if (wid == 0) {
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const int col = lane + 64 * e;
            knew_e[e] = (col < D) ? load_elem<TT>(ku, col) : 0.f;
            vnew_e[e] = (col < D) ? load_elem<TT>(vu, col) : 0.f;
        }
    }

    // ---- the query, pre-scaled by 1/sqrt(d), in fp64
    double qd[EPL];
    {
        uint32_t w[NW32]; float x[EPL];
        load_words<NW32>(qu + sub * LANEB, w);
        decode<TT, EPL, NW32>(w, x);
        const double scale = 1.0 / sqrt((double)D);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qd[e] = (double)x[e] * scale;
    }

    // ---- phase 1: stream K, logits in fp64 to LDS
    double mx = -INFINITY;
    for (int base = gid; base < L; base += NG * U) {
        uint32_t kw[U][NW32];
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            int i = base + uu * NG;
            if (i >= L) i = base;                           // harmless duplicate load
            const char* kp = (i == Lc) ? ku : Kc + (size_t)i * ROWB;
            load_words<NW32>(kp + sub * LANEB, kw[uu]);
        }
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int i = base + uu * NG;
            float kx[EPL];
            decode<TT, EPL, NW32>(kw[uu], kx);
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = fma((double)kx[e], qd[e], dot);
            dot = row_allsum(dot);
            if (i < L) {
                if (sub == 0) sl[i] = dot;
                mx = fmax(mx, dot);
            }
        }
    }
    // mx is uniform within each 16-lane row: combine the four rows of the wave
    mx = fmax(fmax(readlane_f64(mx, 0), readlane_f64(mx, 16)), fmax(readlane_f64(mx, 32), readlane_f64(mx, 48)));
    if (lane == 0) wmax[wid] = mx;
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        const int i = tid + k * NT;
        if (i < L) { al[i] = a_reg[k]; pl[i] = pos_reg[k]; }
    }
    __syncthreads();     // barrier 1: logits, score sums and token indices are staged

    double Mx = wmax[0];
    for (int w = 1; w < NW; ++w) Mx = fmax(Mx, wmax[w]);

    // state wave 0 carries across barrier 2
    int dest = t;        // slot that receives the incoming token (fill phase: the next free one)
    int ev_pos = -1, ev_rank = -1, j = -1, r = -1;
    double merged[EPW];
    bool zero_den = false;

    if (wid != 0) {
        // ---- phase 2, waves 1..NW-1: stream V, accumulate exp(logit - max) . V
        const int g2 = gid - 4, NG2 = NG - 4;
        S l_run = (S)0;
        S acc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = (S)0;
        for (int base = g2; base < L; base += NG2 * U) {
            uint32_t vw[U][NW32];
#pragma unroll
            for (int uu = 0; uu < U; ++uu) {
                int i = base + uu * NG2;
                if (i >= L) i = base;
                const char* vp = (i == Lc) ? vu : Vc + (size_t)i * ROWB;
                load_words<NW32>(vp + sub * LANEB, vw[uu]);
            }
#pragma unroll
            for (int uu = 0; uu < U; ++uu) {
                const int i = base + uu * NG2;
                const S p = (i < L) ? soft_exp((S)(sl[(i < L) ? i : base] - Mx)) : (S)0;
                float vx[EPL];
                decode<TT, EPL, NW32>(vw[uu], vx);
                l_run += p;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] += p * (S)vx[e];
            }
        }
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            l_run += __shfl_xor(l_run, off);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], off);
        }
        if (lane < ROW_LANES) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) part[wid * D + lane * EPL + e] = acc[e];
            if (lane == 0) plw[wid] = l_run;
        }
    } else {
        // ---- phase 2, wave 0: the bookkeeping of Algorithm 1, in fp64, from LDS
        double psum = 0.0;
        for (int i = lane; i < L; i += 64) psum += exp(sl[i] - Mx);
        const double denom = wave_sum(psum);

        Best best = { INFINITY, NONE_POS, -1 };
        int nonfinite = 0;
        for (int i = lane; i < L; i += 64) {
            const double p = exp(sl[i] - Mx) / denom;                // A_t[i]
            const double ai = al[i] + p;                             // a = [a, 0] + A_t
            al[i] = ai;
            if (compress) {
                const int pi = pl[i];
                const double ni = (double)(t - pi + 1);              // n: steps this token has been attended
                double score = (c.score_mode == 0) ? ai / ni : (c.score_mode == 1) ? ai : p;
                if (!(score == score) || score == INFINITY) { score = INFINITY; nonfinite = 1; }
                if (pi <= t - c.R && pi >= c.n_sink && better(score, pi, best)) best = { score, pi, i };
            }
        }
        if (nonfinite) atomicAdd(&c.status[1], 1);

        if (compress) {
            best = wave_argmin(best);
            j = best.phys;
            const int pj = best.pos;
            Next nx = { NONE_POS, -1, 0.0 };
            int cnt = 0;
            for (int i = lane; i < L; i += 64) {
                const int pi = pl[i];
                if (pi < pj) ++cnt;
                else if (pi > pj && pi < nx.pos) nx = { pi, i, 0.0 };
            }
            nx = wave_next(nx);
            cnt = wave_sum(cnt);
            r = nx.phys;
            ev_pos = pj; ev_rank = cnt;
            // A candidate and a right neighbour always exist (n_sink + R <= m, and the
            // incoming token is newer than any candidate).  Should the cache ever be
            // inconsistent, touch nothing out of range and flag it.
            if (j < 0 || r < 0) {
                if (lane == 0) atomicAdd(&c.status[1], 1);
                j = r = -1;
            } else {
                dest = j;
            }
        }
        // score sums back to memory: every entry but the victim; the incoming token's goes to its slot
        for (int i = lane; i < Lc; i += 64)
            if (i != j) au[i] = al[i];
        if (lane == 0 && (!compress || j >= 0)) { au[dest] = al[Lc]; pu[dest] = t; }

        if (compress && j >= 0 && c.merge_mode == 0) {
            // V[r] <- (abar_j V[j] + abar_r V[r]) / (abar_j + abar_r)     (Algorithm 1, Section IV)
            const double sj = best.s;
            const double sr = al[r] / (double)(t - pl[r] + 1);
            const double den = sj + sr;
            zero_den = !(den > 0.0);
#pragma unroll
            for (int e = 0; e < EPW; ++e) {
                const int col = lane + 64 * e;
                if (col < D) {
                    const double vj = (double)load_elem<TT>(Vc + (size_t)j * ROWB, col);
                    const double vr = (double)((r == Lc) ? vnew_e[e] : load_elem<TT>(Vc + (size_t)r * ROWB, col));
                    merged[e] = zero_den ? 0.5 * vj + 0.5 * vr : (sj * vj + sr * vr) / den;
                }
            }
        }
    }
    __syncthreads();     // barrier 2: every V row has been read, partials are staged

    if (tid < D) {       // o_t = A_t^T V_t   (Section III-A)
        const int col = tid;
        S num = (S)0, den = (S)0;
        for (int w = 1; w < NW; ++w) { num += part[w * D + col]; den += plw[w]; }
        const S o = num / den;
        if constexpr (TT::BYTES == 4) reinterpret_cast<float*>(out_)[(size_t)u * D + col] = (float)o;
        else store_elem<TT>(out_, (size_t)u * D + col, (float)o);
    }
    if (wid == 0 && (!compress || j >= 0)) {
        // ---- write-back of the rows: merged value, then the incoming token into its slot
        const bool merge = compress && c.merge_mode == 0;
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const int col = lane + 64 * e;
            if (col < D) {
                if (merge && r == Lc) {
                    store_elem_f64<TT>(Vc + (size_t)dest * ROWB, col, merged[e]);   // folded straight into the new token
                } else {
                    if (merge) store_elem_f64<TT>(Vc + (size_t)r * ROWB, col, merged[e]);
                    store_elem<TT>(Vc + (size_t)dest * ROWB, col, vnew_e[e]);
                }
                store_elem<TT>(Kc + (size_t)dest * ROWB, col, knew_e[e]);
            }
        }
        if (lane == 0) {
            int32_t* nm = c.nmerged + (size_t)u * m;
            if (merge) {
                const int nj = nm[j];
                if (r == Lc) nm[dest] = 1 + nj;
                else { nm[r] += nj; nm[dest] = 1; }
                if (zero_den) atomicAdd(&c.status[0], 1);
            } else {
                nm[dest] = 1;
            }
        }
    }
    if (tid == 0) {
        const size_t row = (size_t)(t % c.log_cap) * c.units + u;
        c.log_pos[row] = ev_pos;
        c.log_slot[row] = ev_rank;
    }
}

template <class TT, int D>
hipError_t launch(const WkvCache& c, int threads, size_t lds, const void* q, const void* k,
                  const void* v, void* out, int t, hipStream_t stream)
{
    hipLaunchKernelGGL((wkv_step_kernel<TT, D, 4>), dim3(c.units), dim3(threads), lds, stream,
                       c, q, k, v, out, t);
    return hipGetLastError();
}

}  // namespace

size_t wkv_step_lds_bytes(int m, int dtype, int head_dim, int threads)
{
    const size_t s = (dtype == 0) ? 8 : 4;     // sizeof(soft_t)
    const size_t nw = (size_t)threads / 64;
    return ((size_t)m + 1) * 20 + 16 * 8 + (nw * (size_t)head_dim + 16) * s;
}

int wkv_step_max_entries(int threads) { return MAXPT * threads; }

hipError_t wkv_launch_step(const WkvCache& c, int dtype, int head_dim, int threads,
                           const void* q, const void* k_new, const void* v_new, void* out,
                           int64_t t, hipStream_t stream)
{
    const size_t lds = wkv_step_lds_bytes(c.m, dtype, head_dim, threads);
    const int ti = (int)t;
#define WKV_CASE(DT, TT, DD) \
    if (dtype == DT && head_dim == DD) return launch<TT, DD>(c, threads, lds, q, k_new, v_new, out, ti, stream);
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return hipErrorInvalidValue;
}
