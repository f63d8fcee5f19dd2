// Internal contract between the host side of libwkv (wkv_api.cpp) and its
// kernels (wkv_step.hip).  Not part of the public boundary (include/wkv.h).
#ifndef WKV_INTERNAL_H
#define WKV_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

// Device-resident cache of one handle: m = budget physical slots per unit.
//
// While a step runs, the cache logically has m+1 entries (Algorithm 1 computes
// A_t over the cache including the new token before it compresses); the extra
// entry is the incoming token itself, read straight from the caller's k_new /
// v_new buffers.  When the step ends the token is written into the slot the
// victim vacated (or, while the cache is still filling, into slot t).
//
// Physical slot order is therefore NOT token order.  Attention is a sum over
// slots, so any order gives the same result; token order -- needed only to find
// the right-hand neighbour of the victim -- is carried by pos[] (for readback) and
// by the linked list nxt[] (for the kernel).  No row of K or V is ever moved.
struct WkvCache {
    void*    K;          // [units][m][D] storage dtype; a row is written once per token it holds
    void*    V;          // [units][m][D] storage dtype; one row rewritten per compression
    double*  a;          // [units][m] accumulated attention weight (Algorithm 1's list a), fp64
    int32_t* pos;        // [units][m] original token index of the slot's key
    int32_t* nxt;        // [units][m] slot of the next token in token order, -1 for the newest
    int32_t* log_pos;    // [log_cap][units] evicted token index per step (ring), -1 = none
    int32_t* log_slot;   // [log_cap][units] its rank in token order
    int32_t* status;     // [2] {zero-denominator merges, non-finite scores / inconsistencies}
    int64_t* tdev;       // null, or (replayable handles) [1] the token index of the next step, kept on the device
    uint32_t* tick;      // with tdev: [1] workgroups of the running step that have finished with the index
    int units, m, R, n_sink, score_mode, merge_mode, log_cap;
};

// Sets a replayable handle's device-side token index (after a prefill or a load): one tiny kernel.
hipError_t wkv_launch_set_clock(const WkvCache& c, int64_t tokens, hipStream_t stream);

// Launches one decode step for every unit.  t = 0-based index of the incoming
// token.  threads in {256,512,1024}, with m + 1 <= wkv_step_max_entries(threads).
// stream_loads: cached K/V rows are loaded non-temporally.  Returns the launch's hipError_t.
hipError_t wkv_launch_step(const WkvCache& c, int dtype, int head_dim, int threads, bool stream_loads,
                           const void* q, const void* k_new, const void* v_new, void* out,
                           int64_t t, hipStream_t stream);

// Row requests per matrix, group and step that wkv_launch_step issues for a budget of m slots in a
// launch of `units` units, padding of the last chunk included (the chunk depth it would choose for
// that launch is taken into account).
int wkv_step_padded_rows(int m, int dtype, int head_dim, int threads, int units);

// Bytes of dynamic LDS wkv_launch_step needs for this shape.
size_t wkv_step_lds_bytes(int m, int dtype, int head_dim, int threads);

// Raises the kernel's dynamic-LDS limit to `lds` bytes (needed above 64 KiB).
hipError_t wkv_step_prepare(int dtype, int head_dim, size_t lds);

// Largest number of attended entries (m + 1) a workgroup of this size handles.
int wkv_step_max_entries(int threads);

// ---- the variant for few units (wkv_split.hip): S workgroups per unit
//
// Device scratch of a handle that splits: what the S slices of a unit hand to the workgroup
// that finishes the unit.  Rewritten by every step; only cnt carries state (zero between steps).
struct WkvSplit {
    double*   lg;        // [units][m+1] exp(logit - maximum of its slice) of every entry of the current step
    void*     po;        // [units][S][D] per-slice sum of exp(logit - slice maximum) . V; 8 bytes per
                         //              element are allocated, fp32 is stored for 16-bit caches, fp64 for fp32
    double*   pm;        // [units][S] slice maximum of the logits (-inf for an empty slice)
    double*   pl;        // [units][S] per-slice sum of the weights the partial output row was built with
    double*   pe;        // [units][S] per-slice sum of exp(logit - slice maximum), fp64
    uint32_t* cnt;       // [units] slices of the unit that have delivered
    int S;
};

// Same contract as wkv_launch_step, grid = units * sp.S workgroups.
hipError_t wkv_launch_split(const WkvCache& c, const WkvSplit& sp, int dtype, int head_dim, int threads,
                            bool stream_loads, const void* q, const void* k_new, const void* v_new, void* out,
                            int64_t t, hipStream_t stream);
size_t wkv_split_lds_bytes(int m, int dtype, int head_dim, int threads);
hipError_t wkv_split_prepare(int dtype, int head_dim, size_t lds);


// ---- bulk prefill of an empty cache (wkv_prefill.hip).  q, k, v, out: [P][units][D] device
// memory (out may be null); lse, a: [units][P] fp64 scratch.  16-bit caches, D in {64,128}.
hipError_t wkv_launch_prefill(const WkvCache& c, int dtype, int head_dim, const void* q, const void* k,
                              const void* v, void* out, double* lse, double* a, int P, hipStream_t stream);
size_t wkv_prefill_lds_bytes(int P);

// Device address of the library's static prefill scratch (WKV_NOALLOC_SCRATCH_BYTES, declared in
// wkv_prefill.hip) on `device`, which must be the current device.  Looked up once per device.
hipError_t wkv_prefill_static_scratch(int device, double** ptr);


// ---- measurement aid (wkv_probe.hip): `workgroups` x `threads` read `bytes` of device memory,
// each workgroup its own contiguous share, and do nothing else.
hipError_t wkv_launch_probe_read(const void* src, size_t bytes, int workgroups, int threads, bool nontemporal,
                                 void* sink, hipStream_t stream);

#endif
