// Internal contract between the host side of libwkv (wkv_api.cpp) and its
// kernels (wkv_step.hip).  Not part of the public boundary (include/wkv.h).
#ifndef WKV_INTERNAL_H
#define WKV_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

// Device-resident cache of one handle.  "cap" = budget + 1 physical slots per
// unit: the extra slot is where the incoming token lives while attention runs
// over all m+1 entries (Algorithm 1 computes A_t before it compresses).
//
// Physical slot order is NOT token order.  Attention is a sum over slots, so
// any order gives the same result; token order -- needed only to find the
// right-hand neighbour of the victim -- is carried by pos[].  After a
// compression the victim's slot is simply the one the next token is written
// to (free_slot), so no row of K or V is ever moved.
struct WkvCache {
    void*    K;          // [units][cap][D] storage dtype; rows are written once, never modified
    void*    V;          // [units][cap][D] storage dtype; one row rewritten per compression
    double*  a;          // [units][cap] accumulated attention weight (Algorithm 1's list a), fp64
    int32_t* pos;        // [units][cap] original token index of the slot's key
    int32_t* nmerged;    // [units][cap] raw values folded into the slot
    int32_t* free_slot;  // [units] slot vacated by the last compression
    int32_t* log_pos;    // [log_cap][units] evicted token index per step (ring), -1 = none
    int32_t* log_slot;   // [log_cap][units] its rank in token order
    int32_t* status;     // [2] {zero-denominator merges, non-finite scores}
    int units, cap, m, R, n_sink, score_mode, merge_mode, log_cap;
};

// Launches one decode step for every unit.  t = 0-based index of the incoming
// token.  threads in {256,512,1024}.  Returns the launch's hipError_t.
hipError_t wkv_launch_step(const WkvCache& c, int dtype, int head_dim, int threads,
                           const void* q, const void* k_new, const void* v_new, void* out,
                           int64_t t, hipStream_t stream);

// Bytes of dynamic LDS wkv_launch_step needs for this shape.
size_t wkv_step_lds_bytes(int cap, int dtype, int head_dim, int threads);

#endif
