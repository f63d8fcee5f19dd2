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
//   * K and V are each streamed exactly once.  The K phase leaves the logit of
//     every entry, in fp64, in LDS; a wave requests its V rows as soon as it has
//     used its last K row.  The V phase accumulates exp(logit - max) . V in fp32
//     (fp64 for an fp32 cache);
//   * the score bookkeeping of Algorithm 1 (softmax denominator, a += A_t,
//     abar = a/n, arg-min, right neighbour, merge weights) is done by wave 0
//     -- in the 1024-thread workgroups by waves 0..3, one on each SIMD of the
//     compute unit -- from the staged logit row while V is in flight, so the
//     dependent chain of the compression hides behind the second half of the
//     memory traffic;
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
// indices, links) is requested before the streaming loop starts, wave-level
// reductions use DPP row operations plus v_readlane instead of LDS permutes,
// per-wave results are combined by one DPP row reduction per wave, and the two
// V rows of the merge are requested the moment a bookkeeping wave knows its
// candidate, well ahead of the barrier after which they are needed.
#include "wkv_internal.h"
#include <type_traits>

#include "wkv_device.h"

// Phase markers for an out-of-tree timing harness; they compile to nothing in the library.
#ifndef WKV_MARK
#define WKV_MARK(k)
#endif

namespace {

// ------------------------------------------------------------------ the kernel
// Entries attended in step t: the Lc = min(t, m) cached slots, then the incoming
// token as entry Lc (its row is read from k_new / v_new).  L = Lc + 1.
//
// Shape of the kernel (one workgroup per unit):
//   1. small loads (query, score sums, token indices, links, incoming row), then the K
//      rows of the first round, are requested before anything is waited for.  Every wave
//      issues its row loads in straight-line code: s_waitcnt counts are derived per
//      control-flow path by the compiler, and a request under a condition between a load and
//      its use would make every later wait conservative (conditions ahead of the first row
//      request are harmless: which small loads a wave issues is decided there);
//   2. K phase: logits in fp64, to LDS.  A wave requests its first round of V rows as soon
//      as it has used its last K row, so the memory system is never idle but mostly serves
//      K before V;
//   3. barrier 1 (LDS traffic only; the V requests stay in flight).  Then the bookkeeping
//      of Algorithm 1 in fp64 (softmax denominator, a += A_t, abar = a/n, arg-min, right
//      neighbour) from LDS, by wave 0 or by waves 0..3 (QUAD below), while V arrives and the
//      waves accumulate exp(logit - max) . V;
//   4. barrier 2: victim and neighbour are known.  The wave that requested the two V rows of
//      the merge writes the merged row, wave 0 the incoming token's rows; every thread writes
//      back the score sum and link of the entry it owns; the last waves write o_t; barrier 3;
//      the log entry (the 1024-thread workgroups need no third barrier: a bookkeeping wave has
//      ranked the victim for the log while it waited for the second).
//
// SEP: the incoming token is attended outside the rounds (by the wave whose block would have
// held it).  Chosen by the host when the budget is a multiple of the block, where entry m would
// otherwise cost that wave one more round of K and of V for a single row.
//
// DED: wave 0 streams K like every other wave but takes no V rows: the V phase is spread over the
// other waves, and wave 0 has only the bookkeeping between the two barriers.
// Without it wave 0 does the bookkeeping (~2 us for 411 entries) and then its share of V, and
// the other waves wait for it at the second barrier.  Chosen by the host (dedicated_wave below).
template <class TT, int D, int U, int MAXT, bool SEP, bool DED, bool STREAM>
__global__ __launch_bounds__(MAXT, 4)
void wkv_step_kernel(WkvCache c, const void* __restrict__ q_, const void* __restrict__ k_,
                     const void* __restrict__ v_, void* __restrict__ out_, int t_arg)
{
    using S = typename TT::soft_t;
    const int t = step_index(c, t_arg);          // from the host, or (replayable handles) from device memory
    // QUAD (the 1024-thread workgroups, one per compute unit): Algorithm 1's bookkeeping is shared by
    // four waves, one on each SIMD of the compute unit, which stream V like everybody else.  A wave
    // issues one instruction every four cycles at best, whatever the instruction, and the
    // bookkeeping of 411 entries is ~600 of them in a chain: 2.6 us in one wave, measured, with
    // the rest of the workgroup waiting at the second barrier for the last microsecond of it.
    // Four waves on four SIMDs take a quarter of the entries each; waves 1..3 publish their best
    // candidate through LDS and wave 0, after a short wait on an LDS counter, picks among the four.
    constexpr bool QUAD = MAXT > 512;
    constexpr int NBK = QUAD ? 4 : 1;            // waves that keep the books
    static_assert(!(QUAD && DED), "the four bookkeeping waves stream V too");
    // wave 0 also ranks the victim for the log: in small launches with a dedicated wave (uniform
    // over the launch); with four bookkeeping waves, wave 1 does it after the second barrier
    const bool RANK0 = DED && gridDim.x <= 768;
    constexpr int EPL  = D / ROW_LANES;          // elements of a row per lane
    constexpr int NW32 = EPL * TT::BYTES / 4;    // 32-bit words per lane per row
    constexpr int ROWB = D * TT::BYTES;          // bytes per row
    constexpr int LANEB = EPL * TT::BYTES;       // bytes per lane per row
    constexpr int EPW  = (D + 63) / 64;          // row elements per lane when one wave handles a row

    const int tid = threadIdx.x, NT = blockDim.x;
    const int NG = NT >> 4, gid = tid >> 4, sub = tid & 15;
    const int NW = NT >> 6, wid = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // wid: scalar, so that what depends on it branches without a lane mask
    const int u = blockIdx.x;
    const int m = c.m;
    const int Lc = (t < m) ? t : m;                        // cached entries
    const int L = Lc + 1;                                  // entries attended
    const bool compress = t >= m;                          // the cache would exceed m
    // Rows are streamed in rounds of RB = NG * U rows: every 16-lane group takes U of them.  In a
    // round that lies wholly inside the cache the rows are dealt group by group (row = start + gid
    // + uu * NG), so that the requests the workgroup issues together cover consecutive rows.  The
    // last, partial round is dealt wave by wave instead, in blocks of BR = 4 U consecutive rows,
    // from wave 0 upwards: a wave whose block lies beyond the end skips the round, so a
    // cache that ends in the middle of a round costs no request for what is not there (dealt group
    // by group, the missing rows would be every wave's last requests, and leaving those out would
    // take requests under a condition, which makes every later wait conservative).
    constexpr int BR = 4 * U;
    static_assert((BR & (BR - 1)) == 0, "block size must be a power of two");
    const int g4 = gid & 3;                                // group within the wave
    const int Ls = SEP ? Lc : L;                           // entries streamed in rounds
    const int RB = NG * U, RBs = __builtin_ctz(RB);       // (a power of two)
    const int nfull = Ls >> RBs;                           // full rounds
    const int tail_blocks = (Ls - nfull * RB + BR - 1) / BR;
    const bool in_tail = wid < tail_blocks;       // this wave has a block of the partial round
    const int nrounds = nfull + (in_tail ? 1 : 0);         // rounds of this wave
    // the wave that attends the incoming entry when it is kept out of the rounds (SEP; then Lc is a
    // multiple of BR): the one that would get the block it opens
    const int w_in = (Lc & (RB - 1)) / BR;
    const bool own_in = SEP && wid == w_in;
    // V phase: which waves stream V rows (all, or all but wave 0), dealt the same way among them
    const int NWv = DED ? NW - 1 : NW, NGv = 4 * NWv;
    const int vwid = DED ? wid - 1 : wid, vgid = DED ? gid - 4 : gid;    // (negative in wave 0 with DED: unused)
    const bool has_v = !DED || wid != 0;
    const int RBv = NGv * U;
    const int nfull_v = Ls / RBv;
    const int tail_blocks_v = (Ls - nfull_v * RBv + BR - 1) / BR;
    // the partial round of V goes to the V waves in order -- but to wave 0 last when it streams V
    // too: it has the bookkeeping to do first (2048 units x 410 slots: 77.6 -> 76.3 us per step)
    // (with four bookkeeping waves: to those four last)
    const int vtail = QUAD ? (wid < NBK ? NW - NBK + wid : wid - NBK) : DED ? vwid : (wid == 0 ? NW - 1 : wid - 1);
    const bool in_tail_v = has_v && vtail < tail_blocks_v;
    const int nrounds_v = nfull_v + (in_tail_v ? 1 : 0);
    const int wv_in = (Lc % RBv) / BR;
    const bool own_in_v = SEP && has_v && vtail == wv_in;   // SEP: the wave that adds the incoming value

    // ---- LDS carve-up
    extern __shared__ double lds[];
    double*   sl     = lds;                                // [m+1] fp64 logit of every entry
    double*   el     = sl + m + 1;                         // [m+1] exp(logit - maximum of the producing wave)
    double*   al     = el + m + 1;                         // [m+1] score sums a
    double*   wmax   = al + m + 1;                         // [16] per-wave maximum logit
    double*   wsum   = wmax + 16;                          // [16] per-wave sum of el
    double*   fw     = wsum + 16;                          // [16] exp(wmax - max) / softmax denominator
    double*   bk_d   = fw + 16;                            // [16] bookkeeping result: victim's and neighbour's score
    S*        part   = reinterpret_cast<S*>(bk_d + 16);    // [NW][D] per-wave P.V partials
    S*        plw    = part + NW * D;                      // [16] per-wave sum of weights
    int*      pl     = reinterpret_cast<int*>(plw + 16);   // [m+1] token index of every entry
    int*      nl     = pl + m + 1;                         // [m+1] entry that follows in token order
    int*      bk_i   = nl + m + 1;                         // [16] bookkeeping result: victim, neighbour, token, rank

    char*       Kc = reinterpret_cast<char*>(c.K) + (size_t)u * m * ROWB;
    char*       Vc = reinterpret_cast<char*>(c.V) + (size_t)u * m * ROWB;
    const char* qu = reinterpret_cast<const char*>(q_) + (size_t)u * ROWB;
    const char* ku = reinterpret_cast<const char*>(k_) + (size_t)u * ROWB;
    const char* vu = reinterpret_cast<const char*>(v_) + (size_t)u * ROWB;
    double*  au = c.a + (size_t)u * m;
    int32_t* pu = c.pos + (size_t)u * m;
    int32_t* nu = c.nxt + (size_t)u * m;

    WKV_MARK(0);
    // ---- small loads first; raw (clamped addresses, no selects or conversions yet).
    // Thread tid owns entries tid, tid + NT, ... for staging and write-back.
    uint32_t qw[NW32];
    load_words<NW32>(qu + sub * LANEB, qw);
    // A wave whose 64 entries of a round all lie beyond the cache skips that round's loads (a scalar
    // condition; with 411 entries and 1024 threads that is nine waves of sixteen in the first round
    // and everybody in the other three -- requests that would all have fetched slot 0).  These
    // conditions sit ahead of the first row request, where they cost nothing: a request under a
    // condition spoils the waits for requests that are OLDER than it, and nothing older is waited
    // for separately (rows are younger, and waiting for a row waits for everything before it).
    double a_reg[MAXPT] = {};
    int pos_reg[MAXPT] = {}, nxt_reg[MAXPT] = {};
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        if (k * NT + wid * 64 < Lc) {
            const int i = tid + k * NT;
            const int ic = (i < Lc) ? i : 0;               // slot 0 always exists in memory
            a_reg[k] = au[ic];
            pos_reg[k] = pu[ic];
            nxt_reg[k] = nu[ic];
        }
    }
    uint32_t knew_b[EPW] = {}, vnew_b[EPW] = {};           // the incoming row (raw), for wave 0's write-back
    if (wid == 0) {
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const int col = (lane + 64 * e < D) ? lane + 64 * e : 0;
            knew_b[e] = load_bits<TT>(ku, col);
            vnew_b[e] = load_bits<TT>(vu, col);
        }
    }
    [[maybe_unused]] uint32_t kin[NW32] = {};               // SEP: the incoming key in row layout
    if constexpr (SEP) { if (own_in) load_words<NW32>(ku + sub * LANEB, kin); }

    // ---- row requests.  Round r of a matrix: entries row_base + uu * row_stride, uu < U.
    uint32_t kw[U][NW32], vw[U][NW32];
    auto request_rows = [&](uint32_t (&dst)[U][NW32], const char* cached, const char* incoming, int base, int stride) {
        const int dup = (base < Ls) ? base : 0;            // where out-of-range groups point (harmless duplicate)
        // all addresses first, then the loads back to back: computed in between, an address may be
        // given a register that an earlier load of the batch is still going to write, and the
        // compiler then waits for that load -- a whole memory round trip -- before it goes on
        const char* rp[U];
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            int i = base + uu * stride;
            if (i >= Ls) i = dup;
            rp[uu] = ((!SEP && i == Lc) ? incoming : cached + (size_t)i * ROWB) + sub * LANEB;
        }
#pragma unroll
        for (int uu = 0; uu < U; ++uu) load_words<NW32, STREAM>(rp[uu], dst[uu]);
    };
    auto k_base = [&](int r) { return r * RB + (r < nfull ? gid : wid * BR + g4); };
    auto k_stride = [&](int r) { return r < nfull ? NG : 4; };
    auto v_base = [&](int r) { return r * RBv + (r < nfull_v ? vgid : vtail * BR + g4); };
    auto v_stride = [&](int r) { return r < nfull_v ? NGv : 4; };
    auto request = [&](uint32_t (&dst)[U][NW32], const char* cached, const char* incoming, int r) {
        request_rows(dst, cached, incoming, k_base(r), k_stride(r));
    };
    auto request_v = [&](int r) { request_rows(vw, Vc, vu, v_base(r), v_stride(r)); };

    request(kw, Kc, ku, 0);                                // a wave without a round gets harmless duplicates

    double qd[EPL];                                        // the query, pre-scaled by 1/sqrt(d), in fp64
    {
        float x[EPL];
        decode<TT, EPL, NW32>(qw, x);
        const double scale = 1.0 / sqrt((double)D);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qd[e] = (double)x[e] * scale;
    }

    // ---- K phase: logits q.K / sqrt(d) in fp64, to LDS
    double mx = -INFINITY;
    auto logits = [&](int r) {
        const int base = k_base(r), stride = k_stride(r);
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int i = base + uu * stride;
            float kx[EPL];
            decode<TT, EPL, NW32>(kw[uu], kx);
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = fma((double)kx[e], qd[e], dot);
            dot = row_allsum(dot);
            if (i < Ls) {
                if (sub == 0) sl[i] = dot;
                mx = fmax(mx, dot);
            }
        }
    };
    if constexpr (SEP) {
        if (own_in) {                                      // the incoming token's logit (its key arrived first)
            float kx[EPL];
            decode<TT, EPL, NW32>(kin, kx);
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = fma((double)kx[e], qd[e], dot);
            dot = row_allsum(dot);
            if (lane == 0) sl[Lc] = dot;
            mx = fmax(mx, dot);
        }
    }
    {
        int r = 0;
        for (; r + 1 < nrounds; ++r) { logits(r); request(kw, Kc, ku, r + 1); }
        if (r < nrounds) logits(r);
    }
    [[maybe_unused]] uint32_t vin[NW32];                    // SEP: the incoming value in row layout
    if constexpr (SEP) load_words<NW32>(vu + sub * LANEB, vin);   // (by every wave: a condition here, between the
                                                                  //  K requests and their use, would spoil the waits)
    // stage what the bookkeeping needs (these loads are older than the K rows: they have
    // arrived): score sums, token indices, and token order as a linked list (nl[i] = entry that
    // follows entry i; the newest cached token is followed by the incoming one, entry Lc)
#pragma unroll
    for (int k = 0; k < MAXPT; ++k) {
        const int i = tid + k * NT;
        if (i < Lc) { al[i] = a_reg[k]; pl[i] = pos_reg[k]; nl[i] = (nxt_reg[k] < 0) ? Lc : nxt_reg[k]; }
        else if (i == Lc) { al[i] = 0.0; pl[i] = t; nl[i] = -1; }      // a = [a, 0]
    }
    if (tid == 0) { bk_i[0] = -1; bk_i[1] = -1; bk_i[2] = -1; bk_i[3] = 0; bk_i[4] = 0; bk_i[5] = 0; bk_i[7] = 0; }
    if (has_v) request_v(0);                               // this wave's K is done: its V rows may queue now
    WKV_MARK(1);

    // mx is uniform within each 16-lane row: combine the four rows of the wave
    mx = fmax(fmax(readlane_f64(mx, 0), readlane_f64(mx, 16)), fmax(readlane_f64(mx, 32), readlane_f64(mx, 48)));
    // exp(logit - wave maximum) of the entries this wave produced, one entry per lane: the
    // fp64 exponentials of the softmax are spread over all waves, ahead of the barrier
    {
        double psum = 0.0;
        for (int idx = lane; idx < nrounds * BR; idx += 64) {
            const int r = idx / BR, j = idx & (BR - 1);
            const int i = r * RB + (r < nfull ? (j >> 2) * NG + 4 * wid + (j & 3) : wid * BR + j);
            if (i < Ls) { const double e = exp(sl[i] - mx); el[i] = e; psum += e; }
        }
        if constexpr (SEP) {
            if (own_in && lane == 0) { const double e = exp(sl[Lc] - mx); el[Lc] = e; psum += e; }
        }
        psum = wave_sum(psum);
        if (lane == 0) { wmax[wid] = mx; wsum[wid] = psum; }
    }
    WKV_MARK(2);
    // barrier 1: logits, exponentials, score sums, token indices and links are staged.  Only
    // LDS traffic has to be complete; the V rows requested above stay in flight.
#define WKV_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")
    WKV_LDS_BARRIER();
    WKV_MARK(3);
    const double Mx = combine_max(wmax, NW, lane);

    // ---- V phase (all waves): accumulate exp(logit - max) . V
    S l_run = (S)0;
    S acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = (S)0;
    auto weighted_sum_from = [&](uint32_t (&src)[U][NW32], int r) {
        const int base = v_base(r), stride = v_stride(r);
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int i = base + uu * stride;
            const S p = (i < Ls) ? soft_exp((S)(sl[(i < Ls) ? i : 0] - Mx)) : (S)0;
            // The row is touched here and not before: left alone, the compiler converts the first V
            // rows right behind their request, ahead of the first barrier, and every wave then
            // waits for its V rows before the bookkeeping can even start.
#pragma unroll
            for (int w = 0; w < NW32; ++w) asm volatile("" : "+v"(src[uu][w]));
            float vx[EPL];
            decode<TT, EPL, NW32>(src[uu], vx);
            l_run += p;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += p * (S)vx[e];
        }
    };
    auto weighted_sum = [&](int r) { weighted_sum_from(vw, r); };
    auto v_first_round = [&]() { weighted_sum(0); };

    uint32_t vj_b[EPW] = {}, vr_b[EPW] = {};               // wave 0: the two V rows of the merge (raw)
    if (wid < NBK) {
        // ---- the bookkeeping of Algorithm 1, in fp64, from LDS, while V arrives: wave 0, or waves 0..3
        {   // softmax denominator from the per-wave partial sums; fw[w] rescales wave w's exponentials
            // (with four bookkeeping waves each computes all of it: same instructions, same bits)
            const double f = (lane < NW) ? exp(wmax[lane] - Mx) : 0.0;
            double den = (lane < NW) ? wsum[lane] * f : 0.0;
            den = readlane_f64(row_allsum(den), 0);
            if (lane < NW) fw[lane] = f / den;
        }
        WKV_MARK(9);
        Best best = { INFINITY, NONE_POS, -1 };
        int nonfinite = 0;
        // BK entries per lane at a time, in straight-line code: their LDS reads are in flight
        // together and their divisions interleave (one entry at a time, each trip is a chain of
        // two LDS round trips and a 14-instruction fp64 division that nothing overlaps).  Bookkeeping
        // wave w of NBK takes the 64-entry stretches w, w + NBK, ...
        constexpr int BK = QUAD ? 2 : 4;
        const int newest_cand = t - c.R, n_sink = c.n_sink;
        auto batches = [&](auto mode_c) {                            // the scoring rule as a constant: no branch per entry
            constexpr int MODE = decltype(mode_c)::value;
            for (int b0 = 0; b0 < L; b0 += 64 * BK * NBK) {
                double e[BK], a[BK], f[BK];
                int pi[BK], ie[BK];
#pragma unroll
                for (int k = 0; k < BK; ++k) {
                    const int i = b0 + 64 * (k * NBK + (QUAD ? wid : 0)) + lane;
                    ie[k] = i;
                    const int ic = (i < L) ? i : L - 1;              // past the end: a duplicate, never stored or ranked
                    e[k] = el[ic]; a[k] = al[ic]; pi[k] = pl[ic];
                    const int ir = ic & (RB - 1);                    // the wave that produced the entry
                    f[k] = fw[(ic == Lc && SEP) ? w_in : (ic - ir < nfull * RB) ? (ir & (NG - 1)) >> 2 : ir / BR];
                }
                double p[BK], ai[BK];
#pragma unroll
                for (int k = 0; k < BK; ++k) {
                    p[k] = e[k] * f[k];                              // A_t[i]
                    ai[k] = a[k] + p[k];                             // a = [a, 0] + A_t
                    if (ie[k] < L) al[ie[k]] = ai[k];
                }
                if (compress) {
                    double score[BK];
#pragma unroll
                    for (int k = 0; k < BK; ++k) {
                        double sc;
                        if constexpr (MODE == 0) sc = ai[k] / (double)(t - pi[k] + 1);   // abar = a / n, n = steps attended
                        else if constexpr (MODE == 1) sc = ai[k];
                        else sc = p[k];
                        const bool bad = !(sc == sc) | (sc == INFINITY);
                        score[k] = bad ? INFINITY : sc;
                        nonfinite |= (bad & (ie[k] < L)) ? 1 : 0;
                    }
#pragma unroll
                    for (int k = 0; k < BK; ++k) {                   // selects, no short-circuit: stays one basic block
                        const bool cand = (ie[k] < L) & (pi[k] <= newest_cand) & (pi[k] >= n_sink);
                        const bool take = cand & ((score[k] < best.s) | ((score[k] == best.s) & (pi[k] < best.pos)));
                        best.s = take ? score[k] : best.s;
                        best.pos = take ? pi[k] : best.pos;
                        best.phys = take ? ie[k] : best.phys;
                    }
                }
            }
        };
        if (c.score_mode == 0) batches(std::integral_constant<int, 0>{});
        else if (c.score_mode == 1) batches(std::integral_constant<int, 1>{});
        else batches(std::integral_constant<int, 2>{});
        WKV_MARK(10);
        bool insane = false;
        if (compress) best = wave_argmin(best);
        WKV_MARK(11);
        if constexpr (QUAD) {
        // Each of the four waves requests the two V rows a merge of ITS candidate would need
        // (the candidate's and its right neighbour's), now, 0.6 us before the winner is known:
        // the winner's rows are then there when the second barrier opens, and the wave that
        // holds them forms the merged row.  Requested whatever the case (row 0 when there is
        // no candidate): these waves have their own V rows in flight, and a request under a
        // condition would make the wait for those wait for everything.
        {
            const int jb = best.phys;
            const bool okb = jb >= 0 && jb < Lc;
            const int rb = okb ? nl[jb] : -1;
            const bool use = okb && rb >= 0 && rb <= Lc && rb != jb;
            const char* rj = Vc + (size_t)(use ? jb : 0) * ROWB;
            const char* rr = (use && rb == Lc) ? vu : Vc + (size_t)(use ? rb : 0) * ROWB;
#pragma unroll
            for (int e = 0; e < EPW; ++e) {
                const int col = (lane + 64 * e < D) ? lane + 64 * e : 0;
                vj_b[e] = load_bits<TT>(rj, col);
                vr_b[e] = load_bits<TT>(rr, col);
            }
        }
        }
        if (compress) {
            if constexpr (QUAD) {
                // Waves 1..3 hand their candidate to wave 0: record, then a release increment of the
                // counter (their LDS writes, the score sums of their entries included, are visible
                // before it).  Wave 0 waits for the three increments; they come unconditionally and
                // depend on nothing wave 0 does, so the wait ends.
                double* wb_s = bk_d + 4;                             // [4] candidate scores
                int* wb_pos = bk_i + 8;                              // [4] their tokens
                int* wb_phy = bk_i + 12;                             // [4] their entries
                if (lane == 0) { wb_s[wid] = best.s; wb_pos[wid] = best.pos; wb_phy[wid] = best.phys; }
                if (wid != 0) {
                    if (lane == 0) __hip_atomic_fetch_add(&bk_i[5], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                } else {
                    while (__hip_atomic_load(&bk_i[5], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < NBK - 1) {}
                    Best b = { (lane < NBK) ? wb_s[lane & 3] : INFINITY, (lane < NBK) ? wb_pos[lane & 3] : NONE_POS,
                               (lane < NBK) ? wb_phy[lane & 3] : -1 };
                    best_step<0xB1>(b); best_step<0x4E>(b);          // over lanes 0..3
                    best = { readlane_f64(b.s, 0), __builtin_amdgcn_readlane(b.pos, 0), __builtin_amdgcn_readlane(b.phys, 0) };
                }
            }
            if (wid == 0) {
                int j = best.phys, r = -1;
                // A candidate always exists (n_sink + R <= m) and is never the newest entry, so it has
                // a right neighbour.  Should the cache ever be inconsistent, touch nothing and flag it.
                bool sane = j >= 0 && j < Lc;
                if (sane) { r = nl[j]; sane = r >= 0 && r <= Lc && r != j; }
                insane = !sane;
                if constexpr (!QUAD) {
                    // The merge needs the V rows of the victim and of its right neighbour: requested here,
                    // used after the second barrier, so that their round trip overlaps the V phase.
                    if (sane && c.merge_mode == 0) {
                        const char* rj = Vc + (size_t)j * ROWB;
                        const char* rr = (r == Lc) ? vu : Vc + (size_t)r * ROWB;
#pragma unroll
                        for (int e = 0; e < EPW; ++e) {
                            const int col = (lane + 64 * e < D) ? lane + 64 * e : 0;
                            vj_b[e] = load_bits<TT>(rj, col);
                            vr_b[e] = load_bits<TT>(rr, col);
                        }
                    }
                }
                if (lane == 0) {
                    if (sane) {
                        bk_i[0] = j; bk_i[1] = r; bk_i[2] = best.pos;
                        bk_i[6] = (j >> 6) & (NBK - 1);              // the bookkeeping wave that ranked (and fetched for) the victim
                        bk_d[0] = best.s;
                        bk_d[1] = al[r] / (double)(t - pl[r] + 1);   // abar of the right neighbour
                    } else {
                        bk_i[3] = 1;
                    }
                    if constexpr (QUAD)     // the victim is published: wave 1, which ranks it for the log, may go on
                        __hip_atomic_store(&bk_i[7], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                if (RANK0) {
                    // the victim's rank in token order, for the log: this wave has nothing else to do
                    // until the second barrier, and the other waves are spared a count, a reduction, an
                    // LDS atomic and a third barrier at the very end of the kernel (512 units x 410
                    // slots 21.2 -> 20.9 us; in large launches it does not pay: 1024 x 1024 88.2 -> 89.4)
                    int cnt = 0;
                    for (int i = lane; i < Lc; i += 64) cnt += (pl[i] < best.pos) ? 1 : 0;
                    cnt = wave_sum(cnt);
                    if (lane == 0) bk_i[4] = cnt;
                }
                WKV_MARK(8);
            }
        }
        if constexpr (QUAD) {
            // These waves' own V rows, here and not below; the flags for the status word wait until
            // after: an atomic under a condition would spoil the wait.
            if (nrounds_v > 0) v_first_round();
            if (compress && wid == 1) {
                // The victim's rank in token order, for the log, from the staged token indices: by wave
                // 1, which has handed in its candidate and used its V rows, ahead of the second barrier
                // (it waits for wave 0 to publish the victim: that comes unconditionally).
                while (__hip_atomic_load(&bk_i[7], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) {}
                const int pv = bk_i[2];
                int cnt = 0;
                for (int i = lane; i < Lc; i += 64) cnt += (pl[i] < pv) ? 1 : 0;
                cnt = wave_sum(cnt);
                if (lane == 0) bk_i[4] = cnt;
            }
        }
        if (nonfinite) atomicAdd(&c.status[1], 1);
        if (insane && lane == 0) atomicAdd(&c.status[1], 1);
    }

    // ---- V phase (all waves)
    auto incoming_value = [&]() {
        if constexpr (SEP) {
            if (own_in_v) {                                // the incoming token, counted by one group only
                const S p = (g4 == 0) ? soft_exp((S)(sl[Lc] - Mx)) : (S)0;
                float vx[EPL];
                decode<TT, EPL, NW32>(vin, vx);
                l_run += p;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] += p * (S)vx[e];
            }
        }
    };
    if constexpr (QUAD) {
        if (wid >= NBK) {
            if (nrounds_v > 1) {
                // A wave with a second round of V rows requests it now, into the K buffer (free since
                // the K phase), and only then uses the first: a workgroup that got its K rows late --
                // the kind a launch of a few hundred units ends with -- pays one memory round trip for
                // its V rows instead of two.  (Both rounds ahead of the barrier stall the wave at the
                // request: the compute unit's memory pipeline is full of its siblings' V rows by then.)
                // A path of its own, so that the wait for the first round leaves the second in flight.
                request_rows(kw, Vc, vu, v_base(1), v_stride(1));
                weighted_sum_from(vw, 0);
                incoming_value();
                weighted_sum_from(kw, 1);
                for (int r = 2; r < nrounds_v; ++r) { request_v(r); weighted_sum(r); }
            } else {
                if (nrounds_v > 0) weighted_sum(0);        // the round requested during the K phase
                incoming_value();
            }
        } else {                                           // the bookkeeping waves have used their first round
            incoming_value();
            for (int r = 1; r < nrounds_v; ++r) { request_v(r); weighted_sum(r); }
        }
    } else if (has_v) {
        if (nrounds_v > 0) weighted_sum(0);                // the round requested during the K phase
        incoming_value();
        for (int r = 1; r < nrounds_v; ++r) { request_v(r); weighted_sum(r); }
    }
    if (has_v) {                                           // a wave without V rows has nothing to add
        S l_w = l_run;
        S acc_w[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc_w[e] = acc[e];
        l_w = rows_sum(l_w);                               // over the wave's four groups
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc_w[e] = rows_sum(acc_w[e]);
        if (lane < ROW_LANES) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) part[wid * D + lane * EPL + e] = acc_w[e];
            if (lane == 0) plw[wid] = l_w;
        }
    }
    WKV_MARK(4);
    if constexpr (QUAD) {
        // The rows a bookkeeping wave fetched for its candidate include the victim's, whose slot wave 0
        // overwrites with the incoming token right after the barrier: those loads have to be complete,
        // in every bookkeeping wave, before anybody passes it.  They were issued a microsecond ago.
        if (wid < NBK) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    WKV_LDS_BARRIER();   // barrier 2: victim and neighbour are known, per-wave partials are staged
    WKV_MARK(5);

    const int j = bk_i[0], r = bk_i[1], pj = bk_i[2];
    const bool sane = bk_i[3] == 0;
    const int dest = compress ? j : t;   // slot that receives the incoming token (fill phase: the next free one)

    if (tid >= NT - D) {  // o_t = A_t^T V_t   (Section III-A); the last waves, wave 0 has the row write-back
        const int col = tid - (NT - D);
        S num = (S)0, den = (S)0;
        for (int w = DED ? 1 : 0; w < NW; ++w) { num += part[w * D + col]; den += plw[w]; }
        const S o = num / den;
        if constexpr (TT::BYTES == 4) reinterpret_cast<float*>(out_)[(size_t)u * D + col] = (float)o;
        else store_elem<TT>(out_, (size_t)u * D + col, (float)o);
    }

    if constexpr (QUAD) {
        // ---- write-back of the rows.  The merged value by the bookkeeping wave that ranked the victim:
        // it requested the victim's and the neighbour's rows when it picked its candidate.  The
        // incoming token's rows by wave 0.
        const bool merge = compress && sane && c.merge_mode == 0;
        if (merge && wid == bk_i[6]) {
            const double sj = bk_d[0], sr = bk_d[1];
            const double den = sj + sr;
            const bool zero_den = !(den > 0.0);
            char* dst = Vc + (size_t)(r == Lc ? dest : r) * ROWB;   // r == Lc: folded straight into the new token
#pragma unroll
            for (int e = 0; e < EPW; ++e) {
                const int col = lane + 64 * e;
                if (col < D) {
                    // V[r] <- (abar_j V[j] + abar_r V[r]) / (abar_j + abar_r)     (Algorithm 1, Section IV)
                    const double vj = (double)bits_elem<TT>(vj_b[e]);
                    const double vr = (double)bits_elem<TT>(vr_b[e]);
                    store_elem_f64<TT, STREAM>(dst, col, zero_den ? 0.5 * vj + 0.5 * vr : (sj * vj + sr * vr) / den);
                }
            }
            if (lane == 0 && zero_den) atomicAdd(&c.status[0], 1);
        }
        if (wid == 0 && sane) {
#pragma unroll
            for (int e = 0; e < EPW; ++e) {
                const int col = lane + 64 * e;
                if (col < D) {
                    if (!(merge && r == Lc)) store_bits<TT, STREAM>(Vc + (size_t)dest * ROWB, col, vnew_b[e]);
                    store_bits<TT, STREAM>(Kc + (size_t)dest * ROWB, col, knew_b[e]);
                }
            }
        }
    } else if (wid == 0 && sane) {
        // ---- write-back of the rows: merged value, then the incoming token into its slot
        const bool merge = compress && c.merge_mode == 0;
        const double sj = bk_d[0], sr = bk_d[1];
        const double den = sj + sr;
        const bool zero_den = !(den > 0.0);
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const int col = lane + 64 * e;
            if (col < D) {
                if (merge) {
                    // V[r] <- (abar_j V[j] + abar_r V[r]) / (abar_j + abar_r)     (Algorithm 1, Section IV)
                    const double vj = (double)bits_elem<TT>(vj_b[e]);
                    const double vr = (double)bits_elem<TT>(vr_b[e]);
                    const double x = zero_den ? 0.5 * vj + 0.5 * vr : (sj * vj + sr * vr) / den;
                    if (r == Lc) {
                        store_elem_f64<TT, STREAM>(Vc + (size_t)dest * ROWB, col, x);   // folded straight into the new token
                    } else {
                        store_elem_f64<TT, STREAM>(Vc + (size_t)r * ROWB, col, x);
                        store_bits<TT, STREAM>(Vc + (size_t)dest * ROWB, col, vnew_b[e]);
                    }
                } else {
                    store_bits<TT, STREAM>(Vc + (size_t)dest * ROWB, col, vnew_b[e]);
                }
                store_bits<TT, STREAM>(Kc + (size_t)dest * ROWB, col, knew_b[e]);
            }
        }
        if (lane == 0 && merge && zero_den) atomicAdd(&c.status[0], 1);
    }

    if (sane) {
        // score sums, token indices and links back to memory: every entry's owner stores its
        // own, the victim's owner stores nothing, the incoming token's owner stores into the
        // destination.  Links: the newest cached token is now followed by the incoming one
        // (which lands in slot dest); the victim's predecessor skips over the victim.
        int cnt = 0;
#pragma unroll
        for (int k = 0; k < MAXPT; ++k) {
            if (k * NT < L) {                               // uniform: skip rounds no thread needs
                const int i = tid + k * NT;
                if (i < Lc) {
                    if (!RANK0 && !QUAD) cnt += (pos_reg[k] < pj) ? 1 : 0;   // the victim's rank in token order, for the log
                    if (i != j) {
                        store_state<STREAM>(&au[i], al[i]);
                        const int n = nxt_reg[k];
                        int nn = n;
                        if (n < 0) nn = dest;
                        else if (n == j) nn = (r == Lc) ? dest : r;
                        if (nn != n) store_state<STREAM>(&nu[i], nn);
                    }
                } else if (i == Lc) {
                    store_state<STREAM>(&au[dest], al[Lc]); store_state<STREAM>(&pu[dest], (int32_t)t); store_state<STREAM>(&nu[dest], (int32_t)-1);
                }
            }
        }
        if (!RANK0 && !QUAD) {
            if (compress) {
                cnt = wave_sum(cnt);
                if (lane == 0 && cnt) atomicAdd(&bk_i[4], cnt);
            }
        }
    }
    WKV_MARK(6);
    if constexpr (QUAD) {
        // the log entry, by wave 1, which ranked the victim ahead of the barrier
        if (tid == 64) {
            const size_t row = (size_t)(t % c.log_cap) * c.units + u;
            c.log_pos[row] = (compress && sane) ? pj : -1;
            c.log_slot[row] = (compress && sane) ? bk_i[4] : -1;
            step_done(c, t, gridDim.x);
        }
    } else {
        if (!RANK0) WKV_LDS_BARRIER();   // barrier 3: the victim's rank is complete (global stores keep flying)
        if (tid == 0) {
            const size_t row = (size_t)(t % c.log_cap) * c.units + u;
            c.log_pos[row] = (compress && sane) ? pj : -1;
            c.log_slot[row] = (compress && sane) ? bk_i[4] : -1;
            step_done(c, t, gridDim.x);
        }
    }
#undef WKV_LDS_BARRIER
    WKV_MARK(7);
}

// The incoming token is attended outside the rounds (SEP at the kernel) when it alone would open
// another block of rows, i.e. cost one wave another round of K and of V for a single row.
inline bool separate_incoming(int m, int rows_per_group) { return m % (4 * rows_per_group) == 0; }

// Depth of a round.  Deep rounds (U rows per group) keep more bytes in flight per wave; shallow
// ones leave more, smaller steps for the workgroups of a compute unit to interleave, and more
// rounds make the dedicated bookkeeping wave pay (below).  Workgroups of up to 512 threads exist
// with U and with U / 2 rows per group.  The shallower one is taken by 512-thread workgroups in
// launches of up to 1024 units (MI355X, d = 128, 16-bit, us per step: 384 units x 410 slots 19.7
// -> 18.7, 512 x 410 22.3 -> 20.7, 512 x 1024 48.8 -> 44.9, 1024 x 512 48.7 -> 46.0, 1024 x 1024
// 92.3 -> 87.8; larger launches lose: 2048 x 512 91.7 -> 92.5, 8192 x 512 356 -> 371, 4096 x 256
// 98 -> 106), and otherwise when m + 1 sits just above a multiple of the deep round (1024 units x
// 520 slots bf16, 256 threads: 51.8 with U = 8, 47.9 with U = 4).
template <class TT, int D, int MAXT> constexpr bool has_half_chunk() { return MAXT <= 512 && unroll<TT, D, MAXT>() >= 8; }
inline int round_slots(int m, int round) { const int ls = (m % round == 0) ? m : m + 1; return (ls + round - 1) / round * round; }
inline bool shallow_rounds(int m, int ng, int rows_per_group, int units = 1 << 30)
{
    if (units <= 1024 && ng == 32) return true;
    return round_slots(m, ng * (rows_per_group / 2)) * 10 <= round_slots(m, ng * rows_per_group) * 9;
}

// Wave 0 is kept free of V rows (DED at the kernel) in workgroups of up to 512 threads only (the
// 1024-thread workgroups share the bookkeeping among four waves instead, which all stream V).  In
// those of 512 threads when a matrix takes three rounds or more (one wave fewer among eight then
// adds little to each of the others, and wave 0's bookkeeping stops being the longest job of the
// workgroup); with fewer rounds, and in workgroups of 256 threads, only when the launch is not
// large enough for many workgroups per compute unit to overlap each other's serial stretches
// and the V rows still fit the same number of rounds with one wave fewer.  Measured (512 threads,
// d = 128, 16-bit, us per step with / without): 384 units x 410 slots 19.7 / 20.2, 512 x 410
// 22.4 / 23.0, 4096 x 300 (three rounds of four rows) 110.7 / 118.4, 2048 x 350 65.8 / 68.9,
// 512 x 1024 48.7 / 52.1, 1024 x 640 57.0 / 59.4, 1024 x 1024 92.2 / 94.5, 2048 x 1024 184.0 /
// 187.9; two rounds: 2048 x 512 91.2 / 91.4, 8192 x 512 360.9 / 355.6, 2048 x 410 76.8 / 76.3;
// one round: 4096 x 256 99.1 / 97.8; 256 threads: 768 x 410 29.9 / 29.3.
inline bool dedicated_wave(const WkvCache& c, int threads, size_t row_bytes, int rows_per_group, bool sep)
{
    const int ls = sep ? c.m : c.m + 1, ng = threads / ROW_LANES;
    const int chunk = ng * rows_per_group, chunk_v = (ng - 4) * rows_per_group;
    const int rounds = (ls + chunk - 1) / chunk, rounds_v = (ls + chunk_v - 1) / chunk_v;
    const bool small = (size_t)c.units * (size_t)(c.m + 1) * row_bytes * 2 <= (size_t)400 << 20;
    if (threads == 512 && rounds >= 3) return true;
    return rounds == rounds_v && small;
}

template <class TT, int D, int U, int MAXT>
hipError_t prepare_u(size_t lds)
{
    const void* ks[] = {
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, false, (MAXT <= 512), false>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, true, (MAXT <= 512), false>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, false, false, false>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, true, false, false>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, false, (MAXT <= 512), true>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, true, (MAXT <= 512), true>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, false, false, true>),
        reinterpret_cast<const void*>(&wkv_step_kernel<TT, D, U, MAXT, true, false, true>),
    };
    for (const void* k : ks) {
        hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <class TT, int D, int MAXT>
hipError_t prepare(size_t lds)
{
    constexpr int U = unroll<TT, D, MAXT>();
    hipError_t e = prepare_u<TT, D, U, MAXT>(lds);
    if constexpr (has_half_chunk<TT, D, MAXT>()) {
        if (e == hipSuccess) e = prepare_u<TT, D, U / 2, MAXT>(lds);
    }
    return e;
}

template <class TT, int D, int U, int MAXT, bool DED, bool STREAM>
hipError_t launch_uds(const WkvCache& c, int threads, size_t lds, bool sep, const void* q, const void* k,
                      const void* v, void* out, int t, hipStream_t stream)
{
    if (sep)
        hipLaunchKernelGGL((wkv_step_kernel<TT, D, U, MAXT, true, DED, STREAM>), dim3(c.units), dim3(threads), lds,
                           stream, c, q, k, v, out, t);
    else
        hipLaunchKernelGGL((wkv_step_kernel<TT, D, U, MAXT, false, DED, STREAM>), dim3(c.units), dim3(threads), lds,
                           stream, c, q, k, v, out, t);
    return hipGetLastError();
}

template <class TT, int D, int U, int MAXT, bool DED>
hipError_t launch_ud(const WkvCache& c, int threads, size_t lds, bool sep, bool stream_loads, const void* q,
                     const void* k, const void* v, void* out, int t, hipStream_t stream)
{
    return stream_loads ? launch_uds<TT, D, U, MAXT, DED, true>(c, threads, lds, sep, q, k, v, out, t, stream)
                        : launch_uds<TT, D, U, MAXT, DED, false>(c, threads, lds, sep, q, k, v, out, t, stream);
}

template <class TT, int D, int U, int MAXT>
hipError_t launch_u(const WkvCache& c, int threads, size_t lds, bool sep, bool stream_loads, const void* q,
                    const void* k, const void* v, void* out, int t, hipStream_t stream)
{
    if constexpr (MAXT <= 512) {
        if (dedicated_wave(c, threads, (size_t)D * TT::BYTES, U, sep))
            return launch_ud<TT, D, U, MAXT, true>(c, threads, lds, sep, stream_loads, q, k, v, out, t, stream);
    }
    return launch_ud<TT, D, U, MAXT, false>(c, threads, lds, sep, stream_loads, q, k, v, out, t, stream);
}

template <class TT, int D, int MAXT>
hipError_t launch(const WkvCache& c, int threads, size_t lds, bool stream_loads, const void* q, const void* k,
                  const void* v, void* out, int t, hipStream_t stream)
{
    constexpr int U = unroll<TT, D, MAXT>();
    if constexpr (has_half_chunk<TT, D, MAXT>()) {
        if (shallow_rounds(c.m, threads / ROW_LANES, U, c.units))
            return launch_u<TT, D, U / 2, MAXT>(c, threads, lds, separate_incoming(c.m, U / 2), stream_loads, q, k, v, out, t, stream);
    }
    return launch_u<TT, D, U, MAXT>(c, threads, lds, separate_incoming(c.m, U), stream_loads, q, k, v, out, t, stream);
}

}  // namespace

size_t wkv_step_lds_bytes(int m, int dtype, int head_dim, int threads)
{
    const size_t s = (dtype == 0) ? 8 : 4;     // sizeof(soft_t)
    const size_t nw = (size_t)threads / 64;
    return ((size_t)m + 1) * 32 + 64 * 8 + (nw * (size_t)head_dim + 16) * s + 16 * 4;
}

int wkv_step_max_entries(int threads) { return MAXPT * threads; }

namespace {
template <class TT, int D, int MAXT> int padded_rows(int m, int threads, int units)
{
    constexpr int U = unroll<TT, D, MAXT>();
    const int ng = threads / ROW_LANES;
    if constexpr (has_half_chunk<TT, D, MAXT>()) {
        if (shallow_rounds(m, ng, U, units)) return round_slots(m, ng * (U / 2));
    }
    return round_slots(m, ng * U);
}
}  // namespace

int wkv_step_padded_rows(int m, int dtype, int head_dim, int threads, int units)
{
#define WKV_CASE(DT, TT, DD) \
    if (dtype == DT && head_dim == DD) return threads > 512 ? padded_rows<TT, DD, 1024>(m, threads, units) : padded_rows<TT, DD, 512>(m, threads, units);
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return 0;
}

namespace {
__global__ void wkv_set_clock_kernel(WkvCache c, long long tokens) { *c.tdev = tokens; *c.tick = 0u; }
}  // namespace

hipError_t wkv_launch_set_clock(const WkvCache& c, int64_t tokens, hipStream_t stream)
{
    hipLaunchKernelGGL(wkv_set_clock_kernel, dim3(1), dim3(1), 0, stream, c, (long long)tokens);
    return hipGetLastError();
}

hipError_t wkv_step_prepare(int dtype, int head_dim, size_t lds)
{
#define WKV_CASE(DT, TT, DD) if (dtype == DT && head_dim == DD) { \
        hipError_t e = prepare<TT, DD, 1024>(lds); return e != hipSuccess ? e : prepare<TT, DD, 512>(lds); }
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return hipErrorInvalidValue;
}

hipError_t wkv_launch_step(const WkvCache& c, int dtype, int head_dim, int threads, bool stream_loads,
                           const void* q, const void* k_new, const void* v_new, void* out,
                           int64_t t, hipStream_t stream)
{
    const size_t lds = wkv_step_lds_bytes(c.m, dtype, head_dim, threads);
    const int ti = (int)t;
#define WKV_CASE(DT, TT, DD) \
    if (dtype == DT && head_dim == DD) return threads > 512 \
        ? launch<TT, DD, 1024>(c, threads, lds, stream_loads, q, k_new, v_new, out, ti, stream) \
        : launch<TT, DD, 512>(c, threads, lds, stream_loads, q, k_new, v_new, out, ti, stream);
    WKV_CASE(0, TF32, 64)  WKV_CASE(0, TF32, 128)
    WKV_CASE(1, TF16, 64)  WKV_CASE(1, TF16, 128)  WKV_CASE(1, TF16, 256)
    WKV_CASE(2, TBF16, 64) WKV_CASE(2, TBF16, 128) WKV_CASE(2, TBF16, 256)
#undef WKV_CASE
    return hipErrorInvalidValue;
}
