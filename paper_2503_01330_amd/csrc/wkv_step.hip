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
//   * K and V are streamed once, in one pass: the P.V accumulation uses an
//     online (running-max) softmax per 16-lane group, rescaled when combined;
//   * the logit of every slot is kept in fp64 and staged in LDS.  The score
//     bookkeeping (softmax denominator, a += p, abar, arg-min, merge weights)
//     is done in fp64 from that staged row after the streaming pass.  This
//     costs one extra convert per K element on a memory-bound kernel and makes
//     the eviction decision reproduce an fp64 reference exactly (differences
//     ~1e-15 relative in abar) instead of drifting apart after the first
//     near-tie;
//   * the path is a GEMV per unit with no reuse across units: no MFMA.
//
// Slot order in memory is not token order (see wkv_internal.h): the victim's
// slot is reused for the next token, so compression moves no K/V row at all.
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

// --------------------------------------------------------- block reductions
// red: LDS scratch of >= 16 doubles.  Results are identical in every thread and
// do not depend on timing (fixed tree).
__device__ __forceinline__ double block_max(double x, double* red, int tid, int nw) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmax(x, __shfl_xor(x, o));
    if ((tid & 63) == 0) red[tid >> 6] = x;
    __syncthreads();
    double r = red[0];
    for (int w = 1; w < nw; ++w) r = fmax(r, red[w]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ double block_sum(double x, double* red, int tid, int nw) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    if ((tid & 63) == 0) red[tid >> 6] = x;
    __syncthreads();
    double r = red[0];
    for (int w = 1; w < nw; ++w) r += red[w];
    __syncthreads();
    return r;
}

struct Best { double s; int pos; int phys; };

// lexicographic (score, token index): ties go to the oldest token
__device__ __forceinline__ bool better(double s, int pos, const Best& b) {
    return (s < b.s) || (s == b.s && pos < b.pos);
}

// ------------------------------------------------------------------ the kernel
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

    const int tid = threadIdx.x, NT = blockDim.x;
    const int NG = NT >> 4, gid = tid >> 4, sub = tid & 15;
    const int NW = NT >> 6, wid = tid >> 6, lane = tid & 63;
    const int u = blockIdx.x;
    const int cap = c.cap;
    const int L = (t + 1 < cap) ? t + 1 : cap;            // slots attended this step
    const bool compress = t >= c.m;                        // cache exceeds m after the append
    const int f = (t < c.m) ? t : c.free_slot[u];          // slot of the incoming token

    // ---- LDS carve-up
    extern __shared__ double lds[];
    double* sl   = lds;                                    // [cap] logit -> exp -> score
    double* red  = sl + cap;                               // [32] reduction scratch
    S*      part = reinterpret_cast<S*>(red + 32);         // [NW][D] per-wave P.V partials
    S*      pm   = part + NW * D;                          // [16] per-wave running max
    S*      plw  = pm + 16;                                // [16] per-wave denominator
    int*    pl   = reinterpret_cast<int*>(plw + 16);       // [cap] token index of each slot
    int*    redi = pl + cap;                               // [64] integer reduction scratch

    const char* Kc = reinterpret_cast<const char*>(c.K) + (size_t)u * cap * ROWB;
    char*       Kw = reinterpret_cast<char*>(c.K) + (size_t)u * cap * ROWB;
    char*       Vc = reinterpret_cast<char*>(c.V) + (size_t)u * cap * ROWB;
    const char* qu = reinterpret_cast<const char*>(q_) + (size_t)u * ROWB;
    const char* ku = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;
    const char* vu = reinterpret_cast<const char*>(v_) + (size_t)u * ROWB;

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

    // ---- streaming pass over the L slots: logits (fp64, to LDS) and online softmax . V
    S m_run = neg_inf<S>(), l_run = (S)0;
    S acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = (S)0;

    for (int base = gid; base < L; base += NG * U) {
        uint32_t kw[U][NW32], vw[U][NW32];
        bool valid[U];
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            int i = base + uu * NG;
            valid[uu] = i < L;
            if (!valid[uu]) i = base;                       // harmless duplicate load
            const char* kp = (i == f) ? ku : Kc + (size_t)i * ROWB;
            const char* vp = (i == f) ? vu : Vc + (size_t)i * ROWB;
            load_words<NW32>(kp + sub * LANEB, kw[uu]);
            load_words<NW32>(vp + sub * LANEB, vw[uu]);
        }
        S sv[U];
        S mnew = m_run;
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int i = base + uu * NG;
            float kx[EPL];
            decode<TT, EPL, NW32>(kw[uu], kx);
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = fma((double)kx[e], qd[e], dot);
            dot = row_allsum(dot);
            if (valid[uu]) {
                if (sub == 0) sl[i] = dot;
                if (i == f) store_words<NW32>(Kw + (size_t)f * ROWB + sub * LANEB, kw[uu]);   // append k_t
            }
            sv[uu] = valid[uu] ? (S)dot : neg_inf<S>();
            mnew = (sv[uu] > mnew) ? sv[uu] : mnew;
        }
        const S sc = rescale(m_run, mnew);
        l_run *= sc;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= sc;
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const S p = rescale(sv[uu], mnew);
            float vx[EPL];
            decode<TT, EPL, NW32>(vw[uu], vx);
            l_run += p;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += p * (S)vx[e];
        }
        m_run = mnew;
    }

    // ---- combine the four 16-lane groups of each wave, then the waves
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const S mo = __shfl_xor(m_run, off), lo = __shfl_xor(l_run, off);
        const S M = (mo > m_run) ? mo : m_run;
        const S sa = rescale(m_run, M), sb = rescale(mo, M);
        l_run = l_run * sa + lo * sb;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = acc[e] * sa + __shfl_xor(acc[e], off) * sb;
        m_run = M;
    }
    if (lane < ROW_LANES) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) part[wid * D + lane * EPL + e] = acc[e];
        if (lane == 0) { pm[wid] = m_run; plw[wid] = l_run; }
    }
    __syncthreads();     // also publishes sl[0..L)

    if (tid < D) {       // o_t = A_t^T V_t   (Section III-A)
        S M = pm[0];
        for (int w = 1; w < NW; ++w) M = (pm[w] > M) ? pm[w] : M;
        S num = (S)0, den = (S)0;
        for (int w = 0; w < NW; ++w) {
            const S sc = rescale(pm[w], M);
            num += part[w * D + tid] * sc;
            den += plw[w] * sc;
        }
        const S o = num / den;
        if constexpr (TT::BYTES == 4) reinterpret_cast<float*>(out_)[(size_t)u * D + tid] = (float)o;
        else store_elem<TT>(out_, (size_t)u * D + tid, (float)o);
    }

    // ---- score bookkeeping in fp64 from the staged logit row
    double mx = -INFINITY;
    for (int i = tid; i < L; i += NT) mx = fmax(mx, sl[i]);
    mx = block_max(mx, red, tid, NW);
    double part_sum = 0.0;
    for (int i = tid; i < L; i += NT) { const double e = exp(sl[i] - mx); sl[i] = e; part_sum += e; }
    const double denom = block_sum(part_sum, red, tid, NW);

    double*  au = c.a + (size_t)u * cap;
    int32_t* pu = c.pos + (size_t)u * cap;
    Best best = { INFINITY, 0x7FFFFFFF, -1 };
    int nonfinite = 0;
    for (int i = tid; i < L; i += NT) {
        const double p = sl[i] / denom;                          // A_t[i]
        const double ai = ((i == f) ? 0.0 : au[i]) + p;          // a = [a, 0] + A_t
        au[i] = ai;
        const int pi = (i == f) ? t : pu[i];
        pl[i] = pi;
        if (compress) {
            const double ni = (double)(t - pi + 1);              // n = steps this token has been attended
            double score = (c.score_mode == 0) ? ai / ni : (c.score_mode == 1) ? ai : p;
            if (!(score == score) || score == INFINITY) { score = INFINITY; nonfinite = 1; }
            sl[i] = score;
            if (pi <= t - c.R && pi >= c.n_sink && better(score, pi, best)) best = { score, pi, i };
        }
    }
    if (tid == 0) pu[f] = t;

    int ev_pos = -1, ev_rank = -1;
    if (compress) {      // uniform over the workgroup
        // arg-min over the workgroup
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            Best b2 = { __shfl_xor(best.s, o), __shfl_xor(best.pos, o), __shfl_xor(best.phys, o) };
            if (better(b2.s, b2.pos, best)) best = b2;
        }
        if (lane == 0) { red[wid] = best.s; redi[wid] = best.pos; redi[16 + wid] = best.phys; }
        __syncthreads();   // also publishes pl[] and the scores in sl[]
        best = { red[0], redi[0], redi[16] };
        for (int w = 1; w < NW; ++w)
            if (better(red[w], redi[w], best)) best = { red[w], redi[w], redi[16 + w] };
        __syncthreads();
        const int j = best.phys, pj = best.pos;

        // right-hand neighbour in token order and the victim's rank
        int rpos = 0x7FFFFFFF, rphys = -1, cnt = 0;
        for (int i = tid; i < L; i += NT) {
            const int pi = pl[i];
            if (pi < pj) ++cnt;
            else if (pi > pj && pi < rpos) { rpos = pi; rphys = i; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const int rp2 = __shfl_xor(rpos, o), rh2 = __shfl_xor(rphys, o);
            if (rp2 < rpos) { rpos = rp2; rphys = rh2; }
            cnt += __shfl_xor(cnt, o);
        }
        if (lane == 0) { redi[wid] = rpos; redi[16 + wid] = rphys; redi[32 + wid] = cnt; }
        __syncthreads();
        rpos = redi[0]; rphys = redi[16]; cnt = redi[32];
        for (int w = 1; w < NW; ++w) {
            if (redi[w] < rpos) { rpos = redi[w]; rphys = redi[16 + w]; }
            cnt += redi[32 + w];
        }
        const int r = rphys;
        ev_pos = pj; ev_rank = cnt;
        // A candidate and a right neighbour always exist (n_sink + R <= m, and the
        // incoming token is newer than any candidate).  Should the cache ever be
        // inconsistent, touch nothing out of range and flag it.
        const bool sane = j >= 0 && r >= 0;
        if (!sane && tid == 0) atomicAdd(&c.status[1], 1);

        if (tid < D && sane) {
            if (c.merge_mode == 0) {
                // V[r] <- (abar_j V[j] + abar_r V[r]) / (abar_j + abar_r)     (Algorithm 1, Section IV)
                const double wj = sl[j], wr = sl[r];
                const double den = wj + wr;
                const double vj = (double)load_elem<TT>(Vc + (size_t)j * ROWB, tid);
                const double vr = (double)((r == f) ? load_elem<TT>(vu, tid)
                                                    : load_elem<TT>(Vc + (size_t)r * ROWB, tid));
                const double x = (den > 0.0) ? (wj * vj + wr * vr) / den : 0.5 * vj + 0.5 * vr;
                store_elem_f64<TT>(Vc + (size_t)r * ROWB, tid, x);
                if (tid == 0 && !(den > 0.0)) atomicAdd(&c.status[0], 1);
            }
            if (r != f || c.merge_mode != 0)                                   // append v_t
                store_elem<TT>(Vc + (size_t)f * ROWB, tid, load_elem<TT>(vu, tid));
        }
        if (tid == 0 && sane) {
            int32_t* nm = c.nmerged + (size_t)u * cap;
            const int nm_r = (r == f) ? 1 : nm[r];
            if (c.merge_mode == 0) nm[r] = nm_r + nm[j]; else if (r == f) nm[r] = 1;
            if (r != f) nm[f] = 1;
            c.free_slot[u] = j;
        }
    } else {
        if (tid < D) store_elem<TT>(Vc + (size_t)f * ROWB, tid, load_elem<TT>(vu, tid));     // append v_t
        if (tid == 0) c.nmerged[(size_t)u * cap + f] = 1;
    }
    if (nonfinite) atomicAdd(&c.status[1], 1);
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
    hipLaunchKernelGGL((wkv_step_kernel<TT, D, 2>), dim3(c.units), dim3(threads), lds, stream,
                       c, q, k, v, out, t);
    return hipGetLastError();
}

}  // namespace

size_t wkv_step_lds_bytes(int cap, int dtype, int head_dim, int threads)
{
    const size_t s = (dtype == 0) ? 8 : 4;     // sizeof(soft_t)
    const size_t nw = (size_t)threads / 64;
    return (size_t)cap * 8 + 32 * 8 + (nw * (size_t)head_dim + 32) * s + (size_t)cap * 4 + 64 * 4;
}

hipError_t wkv_launch_step(const WkvCache& c, int dtype, int head_dim, int threads,
                           const void* q, const void* k_new, const void* v_new, void* out,
                           int64_t t, hipStream_t stream)
{
    const size_t lds = wkv_step_lds_bytes(c.cap, dtype, head_dim, threads);
    const int ti = (int)t;
#define WKV_CASE(DT, TT, DD) \
    if (dtype == DT && head_dim == DD) return launch<TT, DD>(c, threads, lds, q, k_new, v_new, out, ti, stream);
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return hipErrorInvalidValue;
}
