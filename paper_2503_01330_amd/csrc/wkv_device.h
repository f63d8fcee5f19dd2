// Device-side helpers shared by the kernels of libwkv (wkv_step.hip, wkv_split.hip): row I/O in
// the three storage types, DPP lane exchange, wave-level reductions, the victim ordering.
// Everything is forceinline device code in an unnamed namespace: each kernel file gets its own copy.
#ifndef WKV_DEVICE_H
#define WKV_DEVICE_H

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace {

constexpr int ROW_LANES = 16;   // lanes that share one K/V row

struct TF32  { static constexpr int BYTES = 4; using soft_t = double; };
struct TF16  { static constexpr int BYTES = 2; using soft_t = float;  };
struct TBF16 { static constexpr int BYTES = 2; using soft_t = float;  };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------- raw row I/O
// STREAM: the data is used once per launch and the next use is a whole pass over everything else
// away: loaded non-temporally (global_load ... nt), so that it does not push anything out of the
// caches on its way.  On an MI355X this alone took the decode step of 2048 units x 512 slots
// from 102 to 92 us (0.69 -> 0.77 of the HBM peak).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <int NW, bool STREAM = false>
__device__ __forceinline__ void load_words(const void* p, uint32_t (&w)[NW]) {
    if constexpr (NW == 2) {
        const u32x2_t* src = reinterpret_cast<const u32x2_t*>(p);
        const u32x2_t x = STREAM ? __builtin_nontemporal_load(src) : *src;
        w[0] = x.x; w[1] = x.y;
    } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i) {
            const u32x4_t* src = reinterpret_cast<const u32x4_t*>(p) + i;
            const u32x4_t x = STREAM ? __builtin_nontemporal_load(src) : *src;
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

// one storage element as raw bits (no conversion: nothing waits on the load)
template <class TT> __device__ __forceinline__ uint32_t load_bits(const void* base, int idx) {
    if constexpr (TT::BYTES == 4) return reinterpret_cast<const uint32_t*>(base)[idx];
    else return reinterpret_cast<const uint16_t*>(base)[idx];
}
// raw bits of one storage element -> fp32
template <class TT> __device__ __forceinline__ float bits_elem(uint32_t b) {
    if constexpr (TT::BYTES == 4) return __builtin_bit_cast(float, b);
    else if constexpr (__is_same(TT, TF16)) return (float)__builtin_bit_cast(_Float16, (uint16_t)b);
    else return __builtin_bit_cast(float, b << 16);
}
// Stores of cache state (rows, score sums, links).  NT: non-temporal, for handles whose rows are
// loaded non-temporally too -- what a step writes is not in any cache any more when the next step
// of the handle reads it, and lines left dirty in L2 only lengthen the end of the launch
// (256 units x 410 slots, 32 handles in turn: 12.66 -> 12.56 us per step).
template <bool NT, class X> __device__ __forceinline__ void store_state(X* p, X x) {
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}
template <class TT, bool NT = false> __device__ __forceinline__ void store_bits(void* base, int idx, uint32_t b) {
    if constexpr (TT::BYTES == 4) store_state<NT>(&reinterpret_cast<uint32_t*>(base)[idx], b);
    else store_state<NT>(&reinterpret_cast<uint16_t*>(base)[idx], (uint16_t)b);
}
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40);   // NaN stays NaN
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

template <class TT, bool NT = false> __device__ __forceinline__ void store_elem(void* base, int idx, float f) {
    if constexpr (TT::BYTES == 4) store_state<NT>(&reinterpret_cast<float*>(base)[idx], f);
    else if constexpr (__is_same(TT, TF16)) store_state<NT>(&reinterpret_cast<_Float16*>(base)[idx], (_Float16)f);
    else store_state<NT>(&reinterpret_cast<uint16_t*>(base)[idx], f32_to_bf16_rne(f));
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

template <class TT, bool NT = false> __device__ __forceinline__ void store_elem_f64(void* base, int idx, double x) {
    if constexpr (TT::BYTES == 4) store_state<NT>(&reinterpret_cast<float*>(base)[idx], (float)x);
    else store_elem<TT, NT>(base, idx, f64_to_f32_round_odd(x));
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

// Exchange between the 16-lane rows of a wave: v_permlane16_swap / v_permlane32_swap (gfx950) hand
// every lane, in one VALU instruction and without a trip through the LDS crossbar, its own value
// and that of the lane 16 (32) lanes away.  Called with the same register twice they return, as
// measured on the hardware, .x = the value held by the even row (the lower half) of each pair and
// .y = that of the odd row (the upper half), identical in both lanes of a pair.  Summing or taking
// the maximum of .x and .y is the butterfly step x op shfl_xor(x, W), with the same bits in both
// partners (the operands are taken in the same order on both sides).
typedef unsigned uint2v_t __attribute__((ext_vector_type(2)));
template <int W> __device__ __forceinline__ void lane_pair(unsigned v, unsigned& even, unsigned& odd) {
    static_assert(W == 16 || W == 32, "rows 16 apart or halves 32 apart");
    uint2v_t p;
    if constexpr (W == 16) p = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    else p = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    even = p.x; odd = p.y;        // as scalars: __builtin_bit_cast applied to p.y itself reads p.x (hipcc of ROCm 7.2)
}
template <int W> __device__ __forceinline__ void lane_pair(float v, float& even, float& odd) {
    unsigned a, b;
    lane_pair<W>(__builtin_bit_cast(unsigned, v), a, b);
    even = __builtin_bit_cast(float, a); odd = __builtin_bit_cast(float, b);
}
template <int W> __device__ __forceinline__ void lane_pair(double v, double& even, double& odd) {
    unsigned la, lb, ha, hb;
    lane_pair<W>((unsigned)__double2loint(v), la, lb);
    lane_pair<W>((unsigned)__double2hiint(v), ha, hb);
    even = __hiloint2double((int)ha, (int)la); odd = __hiloint2double((int)hb, (int)lb);
}
template <int W, class X> __device__ __forceinline__ X pair_sum(X v) { X a, b; lane_pair<W>(v, a, b); return a + b; }
template <int W> __device__ __forceinline__ double pair_max(double v) { double a, b; lane_pair<W>(v, a, b); return fmax(a, b); }
// over the four rows of a wave: lanes x, x + 16, x + 32, x + 48
template <class X> __device__ __forceinline__ X rows_sum(X v) { return pair_sum<32>(pair_sum<16>(v)); }

__device__ __forceinline__ float  soft_exp(float x)  { return __expf(x); }
__device__ __forceinline__ double soft_exp(double x) { return exp(x); }

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
    // Fast path: the smallest score by a plain fp64 minimum (three instructions per exchange
    // instead of a compare-and-select of the whole record); if exactly one lane holds it, that
    // lane's record is the answer.  Scores are never NaN here.  Ties take the full reduction.
    {
        double mn = b.s;
        mn = fmin(mn, dpp<0xB1>(mn)); mn = fmin(mn, dpp<0x4E>(mn)); mn = fmin(mn, dpp<0x141>(mn)); mn = fmin(mn, dpp<0x140>(mn));
        mn = fmin(fmin(readlane_f64(mn, 0), readlane_f64(mn, 16)), fmin(readlane_f64(mn, 32), readlane_f64(mn, 48)));
        const unsigned long long holders = __ballot(b.s == mn);
        if (__popcll(holders) == 1) {
            const int l = __ffsll((long long)holders) - 1;
            return { mn, __builtin_amdgcn_readlane(b.pos, l), __builtin_amdgcn_readlane(b.phys, l) };
        }
    }
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

// Combining the per-wave results that sit in LDS arrays of nw <= 16 entries: lane w takes
// entry w, one DPP row reduction, lane 0 broadcasts.  Every wave does this for itself
// (a few dozen instructions) instead of every thread scanning the arrays serially.
__device__ __forceinline__ double combine_max(const double* arr, int nw, int lane) {
    double x = (lane < nw) ? arr[lane] : -INFINITY;
    x = fmax(x, dpp<0xB1>(x)); x = fmax(x, dpp<0x4E>(x)); x = fmax(x, dpp<0x141>(x)); x = fmax(x, dpp<0x140>(x));
    return readlane_f64(x, 0);
}

// Device-coherent accesses for the few values that workgroups of one launch hand to each other
// (relaxed atomics at agent scope: they bypass the caches that are not coherent between the
// chip's partitions, so no cache write-back or invalidation is needed around them).
template <class X> __device__ __forceinline__ void store_agent(X* p, X v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class X> __device__ __forceinline__ X load_agent(X* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The token index of a step.  Normally a kernel argument from the host.  A handle created
// "replayable" keeps it in device memory instead, so that a step recorded into a HIP graph advances
// with every replay.  Every workgroup reads it at its start; when a workgroup is done with it, one
// of its threads draws a ticket, and the thread that draws the last ticket of the launch -- every
// workgroup has read the index by then -- stores index + 1 for the next launch and clears the
// tickets.  (Visibility to the next launch comes with the kernel boundary.)
template <class Cache> __device__ __forceinline__ int step_index(const Cache& c, int t_arg) {
    return c.tdev ? (int)*c.tdev : t_arg;
}
template <class Cache> __device__ __forceinline__ void step_done(const Cache& c, int t, unsigned workgroups) {
    if (c.tdev) {
        const unsigned ticket = atomicAdd(c.tick, 1u);
        if (ticket == workgroups - 1) { *c.tick = 0u; *c.tdev = (int64_t)t + 1; }
    }
}

constexpr int MAXPT = 4;       // entries whose a/pos one thread fetches ahead of the streaming loop
constexpr int NONE_POS = 0x7FFFFFFF;

// Rows per 16-lane group requested per round, sized so that one round of K and one of V (both
// raw, in registers) fit the register file: 128 VGPRs per thread for a 1024-thread workgroup,
// 256 for 512 threads or fewer.  The 1024-thread workgroups take four rows also where eight
// would fit (128-byte rows): measured on an MI355X, 256 units x 410 slots x 64 bf16 11.1 -> 10.4
// us per step, 256 x 512 13.5 -> 12.8, 128 x 410 10.5 -> 9.8 (256 x 819 17.0 -> 17.2).
template <class TT, int D, int MAXT> constexpr int unroll() {
    constexpr int words = D / ROW_LANES * TT::BYTES / 4;     // registers per row per lane
    if (MAXT > 512) return words <= 4 ? 4 : 2;
    return words <= 4 ? 8 : 4;
}

}  // namespace

#endif
