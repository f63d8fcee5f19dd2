// The WeightedKV decode step for caches with few units, gfx950.
//
// wkv_step.hip gives every (sequence, head) unit one workgroup, i.e. one compute unit.  A
// single sequence of a 32-head model then occupies 32 of the 256 compute units and is bound
// by what one compute unit can pull from memory.  Here a unit's entries are cut into S slices
// and the grid is units x S workgroups:
//
//   phase A (every workgroup): stream the slice's K rows, logits in fp64 to LDS, then the
//     slice's V rows weighted by exp(logit - slice maximum).  The fp64 exponentials that the
//     score bookkeeping needs are taken here too, one entry per thread while V arrives, so that
//     they are spread over all workgroups of the unit.  The exponentials, their sum, the
//     partial output row, its weight total and the slice maximum go to device memory.  Then
//     the workgroup draws a ticket from the unit's arrival counter.
//   phase B (the workgroup that draws the last ticket; the others have left): everything of
//     Algorithm 1 that needs the whole score row -- softmax denominator, a += A_t,
//     abar = a / n, arg-min over the unprotected entries, right neighbour, convex merge of
//     the two V rows -- one entry per thread, in fp64; o_t from the S partial sums; the
//     incoming token's rows into the slot the victim vacates.
//
// Nobody waits for anybody: a workgroup either leaves after its ticket or finds all S partial
// results complete.  What the slices hand over (logits, partial sums, maxima) is written and read
// with device-coherent accesses, and a workgroup draws its ticket only after all its stores have
// been acknowledged; cache write-backs or invalidations, which cost microseconds per wave here,
// are not needed.  The counter is zero between launches; the finishing workgroup resets it.
//
// Results are those of wkv_step.hip up to summation order: the same fp64 score path (so the
// same eviction decisions), the same write-back; o_t is assembled from S partial sums with
// their own maxima instead of one sum with the global maximum.
#include "wkv_internal.h"
#include "wkv_device.h"

namespace {

template <class TT, int D, int U, int MAXT, bool STREAM>
__global__ __launch_bounds__(MAXT)
void wkv_split_kernel(WkvCache c, WkvSplit sp, const void* __restrict__ q_, const void* __restrict__ k_,
                      const void* __restrict__ v_, void* __restrict__ out_, int t_arg)
{
    using S = typename TT::soft_t;
    const int t = step_index(c, t_arg);          // from the host, or (replayable handles) from device memory
    constexpr int EPL  = D / ROW_LANES;
    constexpr int NW32 = EPL * TT::BYTES / 4;
    constexpr int ROWB = D * TT::BYTES;
    constexpr int LANEB = EPL * TT::BYTES;

    const int tid = threadIdx.x, NT = blockDim.x;
    const int NG = NT >> 4, gid = tid >> 4, sub = tid & 15;
    const int NW = NT >> 6, wid = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int NS = sp.S;
    const int u = blockIdx.x / NS, s = blockIdx.x - u * NS;
    const int m = c.m;
    const int Lc = (t < m) ? t : m;
    const int L = Lc + 1;
    const bool compress = t >= m;
    const int per = (L + NS - 1) / NS;                     // entries per slice
    const int lo = (s * per < L) ? s * per : L;            // this slice: entries lo .. hi-1 (may be empty)
    const int hi = (lo + per < L) ? lo + per : L;
    // Rounds of RB = NG * U rows; full rounds are dealt group by group, the last, partial one wave
    // by wave in blocks of BR = 4 U consecutive rows from wave 0 upwards, and a wave whose block
    // lies beyond the end of the slice skips it (as in wkv_step.hip, where the reasons are given).
    constexpr int BR = 4 * U;
    const int g4 = gid & 3;
    const int RB = NG * U;
    const int nfull = (hi - lo) >> __builtin_ctz(RB);
    const int tail_blocks = (hi - lo - nfull * RB + BR - 1) / BR;
    const int nrounds = nfull + (wid < tail_blocks ? 1 : 0);   // rounds of this wave

    // ---- LDS carve-up
    extern __shared__ double lds[];
    double*   sl   = lds;                                  // [m+1] phase A: logits of the slice; phase B: unused
    double*   al   = sl + m + 1;                           // [m+1] phase B: updated score sums
    double*   wmax = al + m + 1;                           // [16] phase A: per-wave maximum; phase B: per-slice factor
    double*   wsum = wmax + 16;                            // [16] per-wave sum of the exponentials
    double*   bs   = wsum + 16;                            // [16] per-wave best score
    S*        part = reinterpret_cast<S*>(bs + 16);        // [NW][D] per-wave P.V partials
    S*        plw  = part + NW * D;                        // [16]
    int*      pl   = reinterpret_cast<int*>(plw + 16);     // [m+1] token index of every entry
    int*      nl   = pl + m + 1;                           // [m+1] entry that follows in token order
    int*      bp   = nl + m + 1;                           // [16] per-wave best token index
    int*      bi   = bp + 16;                              // [16] per-wave best entry
    int*      misc = bi + 16;                              // [4] ticket, rank, ...

    char*       Kc = reinterpret_cast<char*>(c.K) + (size_t)u * m * ROWB;
    char*       Vc = reinterpret_cast<char*>(c.V) + (size_t)u * m * ROWB;
    const char* qu = reinterpret_cast<const char*>(q_) + (size_t)u * ROWB;
    const char* ku = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;
    const char* vu = reinterpret_cast<const char*>(v_) + (size_t)u * ROWB;
    double*  au = c.a + (size_t)u * m;
    int32_t* pu = c.pos + (size_t)u * m;
    int32_t* nu = c.nxt + (size_t)u * m;
    double*  lgu = sp.lg + (size_t)u * (m + 1);
    S*       pou = reinterpret_cast<S*>(sp.po) + (size_t)u * NS * D;
    double*  pmu = sp.pm + (size_t)u * NS;
    double*  plu = sp.pl + (size_t)u * NS;
    double*  peu = sp.pe + (size_t)u * NS;

    // =========================================================== phase A: the slice
    uint32_t qw[NW32];
    load_words<NW32>(qu + sub * LANEB, qw);
    // Round r of the slice: entries row_base(r) + uu * row_stride(r), uu < U.  Entry Lc is the incoming
    // token, read from the caller's buffers.  Rows past the end of the slice re-read a valid row.
    auto row_base = [&](int r) { return lo + r * RB + (r < nfull ? gid : wid * BR + g4); };
    auto row_stride = [&](int r) { return r < nfull ? NG : 4; };
    uint32_t kw[U][NW32], vw[U][NW32];
    // all addresses of a round first, then its loads back to back (see wkv_step.hip)
    auto row_ptrs = [&](const char* (&rp)[U], const char* cached, const char* incoming, int r) {
        const int base = row_base(r), stride = row_stride(r);
        const int dup = (base < hi) ? base : 0;            // entry 0 always has an address (slot 0, or the incoming row)
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            int i = base + uu * stride;
            if (i >= hi) i = dup;
            rp[uu] = ((i == Lc) ? incoming : cached + (size_t)i * ROWB) + sub * LANEB;
        }
    };
    auto issue = [&](uint32_t (&dst)[U][NW32], const char* const (&rp)[U]) {
#pragma unroll
        for (int uu = 0; uu < U; ++uu) load_words<NW32, STREAM>(rp[uu], dst[uu]);
    };
    auto request = [&](uint32_t (&dst)[U][NW32], const char* cached, const char* incoming, int r) {
        const char* rp[U];
        row_ptrs(rp, cached, incoming, r);
        issue(dst, rp);
    };
    request(kw, Kc, ku, 0);
    // where the first round of V rows lies: worked out now, while the K rows are on their way, so that
    // the V requests go out the moment the last K row is used (the address arithmetic of eight rows is
    // some hundred instructions, a third of a microsecond with two waves on a SIMD)
    const char* vp0[U];
    row_ptrs(vp0, Vc, vu, 0);

    double qd[EPL];
    {
        float x[EPL];
        decode<TT, EPL, NW32>(qw, x);
        const double scale = 1.0 / sqrt((double)D);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qd[e] = (double)x[e] * scale;
    }

    double mx = -INFINITY;
    auto logits = [&](int r) {
        const int base = row_base(r), stride = row_stride(r);
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int i = base + uu * stride;
            float kx[EPL];
            decode<TT, EPL, NW32>(kw[uu], kx);
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = fma((double)kx[e], qd[e], dot);
            dot = row_allsum(dot);
            if (i < hi) {
                if (sub == 0) sl[i - lo] = dot;
                mx = fmax(mx, dot);
            }
        }
    };
    {
        int r = 0;
        for (; r + 1 < nrounds; ++r) { logits(r); request(kw, Kc, ku, r + 1); }
        if (r < nrounds) logits(r);
    }
    issue(vw, vp0);

    mx = fmax(fmax(readlane_f64(mx, 0), readlane_f64(mx, 16)), fmax(readlane_f64(mx, 32), readlane_f64(mx, 48)));
    if (lane == 0) wmax[wid] = mx;
    // the slice's logits and the per-wave maxima are in LDS; the V rows stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const double Ms = combine_max(wmax, NW, lane);         // slice maximum (-inf for an empty slice)

    // exp(logit - slice maximum) in fp64 for the bookkeeping, one entry per thread and round; kept
    // in registers until the V rows are used up (a store here would sit between the V requests and
    // their use, and the rounds are data dependent, which makes every later wait conservative)
    double e_reg[MAXPT];
    double esum = 0.0;
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        e_reg[k] = 0.0;
        if (k * NT < hi - lo) {                            // uniform
            const int i = lo + tid + k * NT;
            if (i < hi) e_reg[k] = exp(sl[i - lo] - Ms);
            esum += e_reg[k];
        }
    }
    esum = wave_sum(esum);
    if (lane == 0) wsum[wid] = esum;

    S l_run = (S)0;
    S acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = (S)0;
    auto weighted_sum = [&](int r) {
        const int base = row_base(r), stride = row_stride(r);
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int i = base + uu * stride;
            const S p = (i < hi) ? soft_exp((S)(sl[(i < hi) ? i - lo : 0] - Ms)) : (S)0;
            // touched here and not before: left alone, the compiler converts the first V rows right
            // behind their request, i.e. waits for them ahead of the barrier (see wkv_step.hip)
#pragma unroll
            for (int w = 0; w < NW32; ++w) asm volatile("" : "+v"(vw[uu][w]));
            float vx[EPL];
            decode<TT, EPL, NW32>(vw[uu], vx);
            l_run += p;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += p * (S)vx[e];
        }
    };
    if (nrounds > 0) weighted_sum(0);
    for (int r = 1; r < nrounds; ++r) { request(vw, Vc, vu, r); weighted_sum(r); }
    {
        l_run = rows_sum(l_run);                           // over the wave's four groups
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = rows_sum(acc[e]);
        if (lane < ROW_LANES) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) part[wid * D + lane * EPL + e] = acc[e];
            if (lane == 0) plw[wid] = l_run;
        }
    }
    __syncthreads();
    if (tid < D) {
        S num = (S)0;
        for (int w = 0; w < NW; ++w) num += part[w * D + tid];
        store_agent(&pou[s * D + tid], num);
    }
    if (tid == 64) {                                       // (a workgroup has at least four waves)
        S den = (S)0;
        double es = 0.0;
        for (int w = 0; w < NW; ++w) { den += plw[w]; es += wsum[w]; }
        store_agent(&plu[s], (double)den);
        store_agent(&peu[s], es);
        store_agent(&pmu[s], Ms);
    }
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        const int i = lo + tid + k * NT;
        if (i < hi) store_agent(&lgu[i], e_reg[k]);
    }
    // every wave waits for the acknowledgement of its own stores (vmcnt(0)), the barrier collects
    // the waves, then one thread draws the ticket: whoever sees the last ticket sees all results
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                         // vmcnt(0) expcnt(0) lgkmcnt(0)
    __syncthreads();
    if (tid == 0) {
        misc[0] = (int)atomicAdd(&sp.cnt[u], 1u);
        step_done(c, t, gridDim.x);                        // every wave of this workgroup has read the index long ago
    }
    __syncthreads();
    if (misc[0] != NS - 1) return;                         // uniform: somebody else finishes this unit

    // =========================================================== phase B: the whole score row
    // one entry per thread and round (MAXPT * NT >= L is checked on the host): its exponential,
    // relative to the maximum of the slice that produced it, and what the previous step left for
    // it (score sum, token index, link).  Only the finishing workgroup reads these.
    double a_reg[MAXPT];
    int pos_reg[MAXPT], nxt_reg[MAXPT];
    // (rounds that hold no entry and slices that do not exist are left out -- uniform conditions --:
    //  every load instruction of 512 threads occupies the memory pipeline for a dozen cycles or more,
    //  and four rounds of four loads plus sixteen partial rows were a microsecond of issue alone)
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        e_reg[k] = 0.0; a_reg[k] = 0.0; pos_reg[k] = 0; nxt_reg[k] = -1;
        if (k * NT < L) {
            const int i = tid + k * NT;
            const int ic = (i < Lc) ? i : 0;
            e_reg[k] = load_agent(&lgu[(i < L) ? i : 0]);
            a_reg[k] = au[ic];
            pos_reg[k] = pu[ic];
            nxt_reg[k] = nu[ic];
        }
    }
    // ... and the partial output rows, by the waves that will form o_t (the last ones: they own the
    // fewest entries), requested now so that they arrive with the rest
    const bool o_wave = tid >= NT - D;                     // uniform per wave
    const int ocol = o_wave ? tid - (NT - D) : 0;
    S po_reg[16];
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        po_reg[w] = (S)0;
        if (o_wave && w < NS) po_reg[w] = load_agent(&pou[w * D + ocol]);
    }
    // softmax over the whole row: lane w of the first wave takes slice w; global maximum, factor
    // exp(slice maximum - maximum), denominator; wmax[w] := factor / denominator, so that
    // A_t[i] = e_i * wmax[slice of i]
    if (wid == 0) {
        const bool has = lane < NS;
        const double pm_s = has ? load_agent(&pmu[has ? lane : 0]) : -INFINITY;
        const double pe_s = has ? load_agent(&peu[has ? lane : 0]) : 0.0;
        if (lane < 16) wsum[lane] = has ? load_agent(&plu[has ? lane : 0]) : 0.0;
        double x = pm_s;
        x = fmax(x, dpp<0xB1>(x)); x = fmax(x, dpp<0x4E>(x)); x = fmax(x, dpp<0x141>(x)); x = fmax(x, dpp<0x140>(x));
        const double f = has ? exp(pm_s - x) : 0.0;        // 0 for an empty slice
        const double den = row_allsum(f * pe_s);
        if (lane < 16) wmax[lane] = f / den;
        if (lane == 0) { misc[1] = 0; misc[2] = 0; }
    }
    __syncthreads();

    if (o_wave) {   // o_t = A_t^T V_t from the S partial sums                  (Section III-A)
        // here and not at the end: it needs the softmax factors only, not the victim, and its store
        // is acknowledged while the scores are still being ranked
        S num = (S)0, dn = (S)0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            if (w < NS) {                                  // the common 1/denominator cancels
                const S f = (S)wmax[w];
                num += f * po_reg[w];
                dn += f * (S)wsum[w];
            }
        }
        const S o = num / dn;
        if constexpr (TT::BYTES == 4) reinterpret_cast<float*>(out_)[(size_t)u * D + ocol] = (float)o;
        else store_elem<TT>(out_, (size_t)u * D + ocol, (float)o);
    }

    // a = [a, 0] + A_t; abar = a / n; candidates                           (Algorithm 1)
    Best best = { INFINITY, NONE_POS, -1 };
    int nonfinite = 0;
    const float rper = 1.0f / (float)per;
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        const int i = tid + k * NT;
        if (k * NT >= L) break;                                              // uniform: rounds nobody needs
        if (i < L) {
            // slice of entry i: (i + 0.5) / per is at least 0.5 / per away from an integer, far
            // more than the rounding error of the fp32 product for i, per < 4096
            const int si = (int)(((float)i + 0.5f) * rper);
            const double p = e_reg[k] * wmax[si];                            // A_t[i]
            const double ai = ((i < Lc) ? a_reg[k] : 0.0) + p;
            const int pi = (i < Lc) ? pos_reg[k] : t;
            a_reg[k] = ai;
            al[i] = ai;
            pl[i] = pi;
            nl[i] = (i < Lc) ? ((nxt_reg[k] < 0) ? Lc : nxt_reg[k]) : -1;
            if (compress) {
                const double ni = (double)(t - pi + 1);
                double score = (c.score_mode == 0) ? ai / ni : (c.score_mode == 1) ? ai : p;
                if (!(score == score) || score == INFINITY) { score = INFINITY; nonfinite = 1; }
                if (pi <= t - c.R && pi >= c.n_sink && better(score, pi, best)) best = { score, pi, i };
            }
        }
    }
    if (nonfinite) atomicAdd(&c.status[1], 1);
    if (compress) {
        best = wave_argmin(best);
        if (lane == 0) { bs[wid] = best.s; bp[wid] = best.pos; bi[wid] = best.phys; }
    }
    __syncthreads();

    int j = -1, r = -1, pj = -1;
    double sj = 0.0, sr = 0.0;
    bool sane = true;
    if (compress) {
        // lane w takes wave w's candidate; one DPP row reduction; lane 0 holds the winner
        Best b = { INFINITY, NONE_POS, -1 };
        if (lane < NW) b = { bs[lane], bp[lane], bi[lane] };
        best_step<0xB1>(b); best_step<0x4E>(b); best_step<0x141>(b); best_step<0x140>(b);
        j = __builtin_amdgcn_readlane(b.phys, 0); pj = __builtin_amdgcn_readlane(b.pos, 0); sj = readlane_f64(b.s, 0);
        // a candidate always exists (n_sink + R <= m) and is never the newest entry; should the
        // cache ever be inconsistent, touch nothing and flag it
        sane = j >= 0 && j < Lc;
        if (sane) { r = nl[j]; sane = r >= 0 && r <= Lc && r != j; }
        if (sane) sr = al[r] / (double)(t - pl[r] + 1);
        else if (tid == 0) atomicAdd(&c.status[1], 1);
    }
    const int dest = compress ? j : t;

    // the two V rows of the merge are requested as soon as they are known
    const bool merge = compress && sane && c.merge_mode == 0;
    const int colc = (tid < D) ? tid : 0;
    uint32_t vj_b = 0, vr_b = 0;
    if (merge) {
        vj_b = load_bits<TT>(Vc + (size_t)j * ROWB, colc);
        vr_b = load_bits<TT>((r == Lc) ? vu : Vc + (size_t)r * ROWB, colc);
    }
    const uint32_t vnew = load_bits<TT>(vu, colc), knew = load_bits<TT>(ku, colc);

    if (sane) {
        // score sums, token indices, links: every entry's owner stores its own (see wkv_step.hip)
        int cnt = 0;
#pragma unroll
        for (int k = 0; k < MAXPT; ++k) {
            const int i = tid + k * NT;
            if (k * NT >= L) break;
            if (i < Lc) {
                cnt += (pos_reg[k] < pj) ? 1 : 0;
                if (i != j) {
                    au[i] = a_reg[k];
                    const int n = nxt_reg[k];
                    int nn = n;
                    if (n < 0) nn = dest;
                    else if (n == j) nn = (r == Lc) ? dest : r;
                    if (nn != n) nu[i] = nn;
                }
            } else if (i == Lc) {
                au[dest] = a_reg[k]; pu[dest] = t; nu[dest] = -1;
            }
        }
        if (compress) {
            cnt = wave_sum(cnt);
            if (lane == 0 && cnt) atomicAdd(&misc[1], cnt);
        }
        // rows: merged value, then the incoming token into its slot.  Thread col owns column col
        // of every row it touches, so its read of V[j] precedes its write into that slot.
        if (tid < D) {
            const int col = tid;
            if (merge) {
                // V[r] <- (abar_j V[j] + abar_r V[r]) / (abar_j + abar_r)       (Algorithm 1, Section IV)
                const double dsum = sj + sr;
                const bool zero_den = !(dsum > 0.0);
                const double vj = (double)bits_elem<TT>(vj_b), vr = (double)bits_elem<TT>(vr_b);
                const double y = zero_den ? 0.5 * vj + 0.5 * vr : (sj * vj + sr * vr) / dsum;
                if (r == Lc) {
                    store_elem_f64<TT>(Vc + (size_t)dest * ROWB, col, y);
                } else {
                    store_elem_f64<TT>(Vc + (size_t)r * ROWB, col, y);
                    store_bits<TT>(Vc + (size_t)dest * ROWB, col, vnew);
                }
                if (col == 0 && zero_den) atomicAdd(&c.status[0], 1);
            } else {
                store_bits<TT>(Vc + (size_t)dest * ROWB, col, vnew);
            }
            store_bits<TT>(Kc + (size_t)dest * ROWB, col, knew);
        }
    }
    __syncthreads();
    if (tid == 0) {
        const size_t row = (size_t)(t % c.log_cap) * c.units + u;
        c.log_pos[row] = (compress && sane) ? pj : -1;
        c.log_slot[row] = (compress && sane) ? misc[1] : -1;
        store_agent(&sp.cnt[u], 0u);                       // ready for the next launch
    }
}

template <class TT, int D, int MAXT>
hipError_t prepare(size_t lds)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wkv_split_kernel<TT, D, unroll<TT, D, MAXT>(), MAXT, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&wkv_split_kernel<TT, D, unroll<TT, D, MAXT>(), MAXT, true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

template <class TT, int D, int MAXT>
hipError_t launch(const WkvCache& c, const WkvSplit& sp, int threads, size_t lds, bool stream_loads, const void* q,
                  const void* k, const void* v, void* out, int t, hipStream_t stream)
{
    if (stream_loads)
        hipLaunchKernelGGL((wkv_split_kernel<TT, D, unroll<TT, D, MAXT>(), MAXT, true>), dim3(c.units * sp.S),
                           dim3(threads), lds, stream, c, sp, q, k, v, out, t);
    else
        hipLaunchKernelGGL((wkv_split_kernel<TT, D, unroll<TT, D, MAXT>(), MAXT, false>), dim3(c.units * sp.S),
                           dim3(threads), lds, stream, c, sp, q, k, v, out, t);
    return hipGetLastError();
}

}  // namespace

size_t wkv_split_lds_bytes(int m, int dtype, int head_dim, int threads)
{
    const size_t s = (dtype == 0) ? 8 : 4;     // sizeof(soft_t)
    const size_t nw = (size_t)threads / 64;
    return ((size_t)m + 1) * 24 + 48 * 8 + (nw * (size_t)head_dim + 16) * s + 36 * 4;
}

hipError_t wkv_split_prepare(int dtype, int head_dim, size_t lds)
{
#define WKV_CASE(DT, TT, DD) if (dtype == DT && head_dim == DD) { \
        hipError_t e = prepare<TT, DD, 1024>(lds); return e != hipSuccess ? e : prepare<TT, DD, 512>(lds); }
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return hipErrorInvalidValue;
}

hipError_t wkv_launch_split(const WkvCache& c, const WkvSplit& sp, int dtype, int head_dim, int threads,
                            bool stream_loads, const void* q, const void* k_new, const void* v_new, void* out,
                            int64_t t, hipStream_t stream)
{
    const size_t lds = wkv_split_lds_bytes(c.m, dtype, head_dim, threads);
    const int ti = (int)t;
#define WKV_CASE(DT, TT, DD) \
    if (dtype == DT && head_dim == DD) return threads > 512 \
        ? launch<TT, DD, 1024>(c, sp, threads, lds, stream_loads, q, k_new, v_new, out, ti, stream) \
        : launch<TT, DD, 512>(c, sp, threads, lds, stream_loads, q, k_new, v_new, out, ti, stream);
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return hipErrorInvalidValue;
}
