// Host side of libwkv: handle management, argument checking, state readback.
// The arithmetic of the method lives in the kernels (wkv_step.hip, wkv_split.hip, wkv_prefill.hip); nothing here computes
// attention, scores or merges.  See include/wkv.h for the contract.
#include "../../include/wkv.h"
#include "wkv_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <numeric>
#include <string>
#include <vector>

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int dtype_bytes(int dtype) { return dtype == WKV_FP32 ? 4 : 2; }

constexpr size_t LDS_LIMIT = 160 * 1024;    // LDS per compute unit on gfx950

// K and V bytes of all live handles, per device: what WKV_LOADS_AUTO goes by.
constexpr int MAX_DEVICES = 64;
std::atomic<long long> g_live_kv[MAX_DEVICES];
constexpr long long LAST_LEVEL_CACHE = 256ll << 20;   // MI355X: 256 MB memory-side cache

void count_live(int device, long long bytes)
{
    if (device >= 0 && device < MAX_DEVICES) g_live_kv[device] += bytes;
}

// Non-temporal row loads: asked for, or (AUTO) nothing a step loads can still be cached at the next
// step.  Measured on an MI355X: 2048 units x 512 slots x 256 B, one handle (538 MB): 102 -> 91 us
// per step; handles of 54 MB (256 units x 410 slots) stepped in turn, us per step cached / non-temporal:
// 4 handles 12.2 / -, 5 (270 MB) 12.32 / 12.43, 6 (324 MB) 12.86 / 12.47, 8 13.75 / 12.54, 12 13.63 / 12.61;
// one handle of 273 MB: 44.5 / 46.5.  The two cross a little above the size of the cache.  Rows of
// 512 B lose 11 % at any size (a lane's two 16-byte loads of a row share their 64-byte segments,
// which then travel twice).
bool stream_loads(const wkv_options& o, int device)
{
    if (o.streaming == WKV_LOADS_STREAMING) return true;
    if (o.streaming == WKV_LOADS_CACHED) return false;
    const long long live = (device >= 0 && device < MAX_DEVICES) ? g_live_kv[device].load() : 0;
    return o.head_dim * dtype_bytes(o.dtype) <= 256 && live >= LAST_LEVEL_CACHE + LAST_LEVEL_CACHE / 8;
}

// Returns 0 and fills *threads and *split, or a negative code with the reason in g_err.
int validate(const wkv_options& o, int* threads, int* split)
{
    if (o.batch <= 0 || o.heads <= 0) return fail(WKV_EINVAL, "batch and heads must be positive");
    if ((long long)o.batch * o.heads > (1 << 24)) return fail(WKV_ESIZE, "batch*heads exceeds 2^24 units");
    if (o.dtype != WKV_FP32 && o.dtype != WKV_FP16 && o.dtype != WKV_BF16)
        return fail(WKV_EINVAL, "dtype must be WKV_FP32, WKV_FP16 or WKV_BF16");
    const bool d_ok = o.head_dim == 64 || o.head_dim == 128 || (o.head_dim == 256 && o.dtype != WKV_FP32);
    if (!d_ok) return fail(WKV_EINVAL, "head_dim %d unsupported for this dtype (64, 128; 256 for 16-bit)", o.head_dim);
    if (o.budget < 1) return fail(WKV_EINVAL, "budget must be at least 1");
    if (o.budget > WKV_MAX_BUDGET) return fail(WKV_ESIZE, "budget %d exceeds WKV_MAX_BUDGET %d", o.budget, WKV_MAX_BUDGET);
    if (o.recent_window < 1 || o.recent_window > o.budget)
        return fail(WKV_EINVAL, "recent_window must be in 1..budget");
    if (o.n_sink < 0 || (long long)o.n_sink + o.recent_window > o.budget)
        return fail(WKV_EINVAL, "n_sink must be >= 0 with n_sink + recent_window <= budget");
    if (o.score_mode < 0 || o.score_mode > 2) return fail(WKV_EINVAL, "unknown score_mode");
    if (o.merge_mode < 0 || o.merge_mode > 1) return fail(WKV_EINVAL, "unknown merge_mode");
    if (o.score_mode != WKV_SCORE_AVERAGE && o.merge_mode != WKV_MERGE_NONE)
        return fail(WKV_EINVAL, "cumulative / last-step scoring are eviction rules: use WKV_MERGE_NONE");
    if (o.log_capacity < 0) return fail(WKV_EINVAL, "log_capacity must be >= 0");
    if (o.streaming < 0 || o.streaming > 2) return fail(WKV_EINVAL, "streaming must be WKV_LOADS_AUTO, _CACHED or _STREAMING");
    if (o.replayable != 0 && o.replayable != 1) return fail(WKV_EINVAL, "replayable must be 0 or 1");
    if (o.max_prompt < 0 || o.max_prompt > WKV_MAX_PROMPT) return fail(WKV_EINVAL, "max_prompt must be in 0..WKV_MAX_PROMPT");
    if (o.max_prompt > 0 && (o.dtype == WKV_FP32 || o.head_dim > 128))
        return fail(WKV_ESIZE, "max_prompt: wkv_prefill is built for 16-bit caches with head_dim 64 or 128");
    for (int r : o.reserved) if (r != 0) return fail(WKV_EINVAL, "reserved fields must be zero");
    int th = o.threads, sp = o.split;
    const int units = o.batch * o.heads;
    if (sp != 0 && sp != 1 && sp != 2 && sp != 4 && sp != 8 && sp != 16)
        return fail(WKV_EINVAL, "split must be 1, 2, 4, 8 or 16");
    if (sp == 0) {
        // One workgroup per unit keeps the score bookkeeping hidden behind the V traffic and has
        // the shorter chain of dependent memory round trips; it is the better shape whenever the
        // units alone occupy the 256 compute units, and for short rows of scores.  Otherwise cut
        // every unit into slices of at least ~200 rows (of 256 bytes), up to 256 workgroups.
        // Measured on an MI355X (fp16, d = 128): 32 units x 819 slots 17.6 -> 12.7 us per step,
        // 64 x 2048 34 -> 23, 16 x 4095 59 -> 19, 32 x 410 no gain.
        const long long rows = (long long)(o.budget + 1) * o.head_dim * dtype_bytes(o.dtype) / 256;
        sp = 1;
        if (rows >= 600)
            while (sp < 16 && units * sp * 2 <= 256 && rows / (sp * 2) >= 200) sp *= 2;
    }
    auto fits = [&](int n) {
        const size_t lds = sp > 1 ? wkv_split_lds_bytes(o.budget, o.dtype, o.head_dim, n)
                                  : wkv_step_lds_bytes(o.budget, o.dtype, o.head_dim, n);
        return lds <= LDS_LIMIT && o.budget + 1 <= wkv_step_max_entries(n);
    };
    if (th == 0) {
        // up to one unit per compute unit (256): large workgroups, so that one unit's rows are spread
        // over many waves (a compute unit holds only one workgroup of 1024 threads: 384 units take
        // 26.3 us with 1024 threads, 23.4 with 512); more
        // units: 512 threads (measured 2-9 % ahead of 256 for rows of 256 bytes at 1024-8192
        // units), except for 128-byte rows, where 256 threads are 20 % ahead; slices: 512
        const int row_bytes = o.head_dim * dtype_bytes(o.dtype);
        th = sp > 1 ? 512 : units >= 1024 ? (row_bytes < 256 ? 256 : 512) : units > 256 ? 512 : 1024;
        // from 768 to about 1200 units, 256 threads where m + 1 sits clearly closer above a multiple
        // of their (smaller) round than of the 512-thread one (m = 410: 448 against 512 rows):
        // 768 x 410 30.5 -> 29.3 us, 1024 x 410 39.4 -> 37.5, 1024 x 520 49.3 -> 46.8; where the two
        // are equally close (m = 512) 512 threads stay ahead, and beyond they win either way
        // (1400 x 410: 55.3 against 58.6, 2048 x 410: 77.2 against 79.0); below 768 units too
        if (sp == 1 && units >= 768 && units < 1200 && row_bytes == 256 && th == 512 && fits(256) &&
            wkv_step_padded_rows(o.budget, o.dtype, o.head_dim, 256, units) * 20 <=
            wkv_step_padded_rows(o.budget, o.dtype, o.head_dim, 512, units) * 19)
            th = 256;
        while (th < 1024 && !fits(th)) th *= 2;
    }
    if (th != 256 && th != 512 && th != 1024) return fail(WKV_EINVAL, "threads must be 256, 512 or 1024");
    if (!fits(th))
        return fail(WKV_ESIZE, "a score row of %d entries does not fit a workgroup of %d threads", o.budget + 1, th);
    *threads = th;
    *split = sp;
    return WKV_OK;
}

struct Sizes { size_t kv, a, i32, log, status, lg, po, ps, cnt, total; };

Sizes sizes(const wkv_options& o, int split)
{
    const size_t units = (size_t)o.batch * o.heads, cap = (size_t)o.budget;
    const size_t logc = o.log_capacity ? o.log_capacity : 1024;
    Sizes s;
    s.kv = units * cap * o.head_dim * dtype_bytes(o.dtype);
    s.a = units * cap * sizeof(double);
    s.i32 = units * cap * sizeof(int32_t);
    s.log = logc * units * sizeof(int32_t);
    s.status = 2 * sizeof(int32_t);
    // scratch of the split variant (nothing when every unit has one workgroup)
    s.lg = split > 1 ? units * (cap + 1) * sizeof(double) : 0;
    s.po = split > 1 ? units * split * o.head_dim * sizeof(double) : 0;
    s.ps = split > 1 ? units * split * sizeof(double) : 0;
    s.cnt = split > 1 ? units * sizeof(uint32_t) : 0;
    // wkv_prefill's scratch, when reserved at creation
    const size_t pf = 2 * units * (size_t)(o.max_prompt > 0 ? o.max_prompt : 0) * sizeof(double);
    s.total = 2 * s.kv + s.a + 2 * s.i32 + 2 * s.log + s.status + s.lg + s.po + 3 * s.ps + s.cnt + pf +
              (o.replayable ? 16 : 0);
    return s;
}

}  // namespace

struct wkv_handle {
    wkv_options opt;
    WkvCache c;
    WkvSplit sp;      // all null with S = 1 when every unit has one workgroup
    int device;
    int threads;
    int64_t t;        // tokens processed
    int64_t log_from; // first step whose eviction log entry is valid (after wkv_load)
    double* pf_scratch;  // wkv_prefill's scratch: [2][units][pf_tokens] fp64, or null
    int pf_tokens;
};

namespace {

// The handle's memory and the kernels' attributes belong to one device; calls come from it.
int on_device(const wkv_handle* h)
{
    int dev;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(WKV_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev != h->device) return fail(WKV_EINVAL, "handle belongs to device %d, current device is %d", h->device, dev);
    return WKV_OK;
}

// Argument checks shared by the two prefill entry points; nothing is launched or allocated here.
int prefill_check(wkv_handle* h, const void* q, const void* k, const void* v, void* out, int n_tokens)
{
    if (!h) return fail(WKV_EINVAL, "null handle");
    if (!q || !k || !v) return fail(WKV_EINVAL, "null device pointer");
    if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) != 0)
        return fail(WKV_EINVAL, "q, k, v and out must be 16-byte aligned");
    if (h->t != 0) return fail(WKV_EINVAL, "wkv_prefill needs an empty cache (%lld tokens processed)", (long long)h->t);
    if (n_tokens < 1) return fail(WKV_EINVAL, "n_tokens must be positive");
    if (n_tokens > WKV_MAX_PROMPT) return fail(WKV_ESIZE, "n_tokens %d exceeds WKV_MAX_PROMPT %d", n_tokens, WKV_MAX_PROMPT);
    const wkv_options& o = h->opt;
    if (o.dtype == WKV_FP32 || o.head_dim > 128)
        return fail(WKV_ESIZE, "wkv_prefill is built for 16-bit caches with head_dim 64 or 128");
    if (o.score_mode == WKV_SCORE_LAST)
        return fail(WKV_EINVAL, "the last-step scoring rule is not defined for a prompt");
    const int rc = on_device(h);
    if (rc != WKV_OK) return rc;
    int lds_max = 0;
    const hipError_t e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device);
    if (e == hipSuccess && wkv_prefill_lds_bytes(n_tokens) > (size_t)lds_max)
        return fail(WKV_ESIZE, "a prompt of %d tokens needs %zu bytes of LDS, the device offers %d", n_tokens,
                    wkv_prefill_lds_bytes(n_tokens), lds_max);
    return WKV_OK;
}

// The handle's own prefill scratch (row log-sum-exps and column sums, fp64 each): sized for
// `tokens` prompt tokens, grown when a longer prompt comes, freed by wkv_destroy.
int prefill_reserve(wkv_handle* h, int tokens)
{
    if (tokens <= h->pf_tokens) return WKV_OK;
    const size_t n = (size_t)h->c.units * (size_t)tokens * sizeof(double);
    double* p = nullptr;
    const hipError_t e = hipMalloc((void**)&p, 2 * n);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? WKV_ENOMEM : WKV_EHIP, "scratch for a prompt of %d tokens: %s",
                    tokens, hipGetErrorString(e));
    }
    if (h->pf_scratch) {
        // an earlier, shorter prompt's kernels may still be reading the old block
        (void)hipDeviceSynchronize();
        (void)hipFree(h->pf_scratch);
    }
    h->pf_scratch = p;
    h->pf_tokens = tokens;
    return WKV_OK;
}

}  // namespace

extern "C" {

const char* wkv_last_error(void) { return g_err.c_str(); }
int wkv_version(void) { return 100; }

size_t wkv_workspace_bytes(const wkv_options* opt)
{
    int th, sp;
    if (!opt || validate(*opt, &th, &sp) != WKV_OK) return 0;
    return sizes(*opt, sp).total;
}

size_t wkv_step_bytes(const wkv_options* opt)
{
    int th, sp;
    if (!opt || validate(*opt, &th, &sp) != WKV_OK) return 0;
    const size_t units = (size_t)opt->batch * opt->heads, L = (size_t)opt->budget + 1;
    const size_t row = (size_t)opt->head_dim * dtype_bytes(opt->dtype);
    // What the method itself has to move (implementation extras such as the next-token
    // links are left out):
    //   per attended entry: K row + V row + score sum read and written (fp64) + token index read
    //   per unit: q, k_new, v_new in, out out; the new token's K and V rows written;
    //             the merged V row written (its two inputs are among the rows already read)
    return units * (L * (2 * row + 16 + 4) + 4 * row + 2 * row + 1 * row);
}

int wkv_launch_shape(const wkv_options* opt, int* workgroups, int* threads)
{
    if (!opt || !workgroups || !threads) return fail(WKV_EINVAL, "null argument");
    int th, sp;
    const int rc = validate(*opt, &th, &sp);
    if (rc != WKV_OK) return rc;
    *workgroups = opt->batch * opt->heads * sp;
    *threads = th;
    return WKV_OK;
}

int wkv_create_ex(wkv_handle** hp, const wkv_options* opt)
{
    if (!hp || !opt) return fail(WKV_EINVAL, "null argument");
    int threads, split;
    int rc = validate(*opt, &threads, &split);
    if (rc != WKV_OK) return rc;
    wkv_handle* h = new (std::nothrow) wkv_handle();
    if (!h) return fail(WKV_ENOMEM, "host allocation failed");
    h->opt = *opt;
    if (h->opt.log_capacity == 0) h->opt.log_capacity = 1024;
    h->threads = threads;
    h->t = 0;
    h->log_from = 0;
    h->pf_scratch = nullptr;
    h->pf_tokens = 0;
    hipError_t e = hipGetDevice(&h->device);
    if (e != hipSuccess) {
        delete h;
        return fail(WKV_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    }
    {
        int lds_max = 0;
        const size_t lds = split > 1 ? wkv_split_lds_bytes(opt->budget, opt->dtype, opt->head_dim, threads)
                                     : wkv_step_lds_bytes(opt->budget, opt->dtype, opt->head_dim, threads);
        e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device);
        if (e == hipSuccess && lds > (size_t)lds_max) {
            delete h;
            return fail(WKV_ESIZE, "a score row of %d entries needs %zu bytes of LDS, the device offers %d",
                        opt->budget + 1, lds, lds_max);
        }
        if (e == hipSuccess)
            e = split > 1 ? wkv_split_prepare(opt->dtype, opt->head_dim, lds)
                          : wkv_step_prepare(opt->dtype, opt->head_dim, lds);
        if (e != hipSuccess) {
            delete h;
            return fail(WKV_EHIP, "preparing the kernel: %s", hipGetErrorString(e));
        }
    }
    const Sizes s = sizes(h->opt, split);
    WkvCache& c = h->c;
    WkvSplit& sp = h->sp;
    memset(&c, 0, sizeof c);
    memset(&sp, 0, sizeof sp);
    sp.S = split;
    c.units = opt->batch * opt->heads; c.m = opt->budget;
    c.R = opt->recent_window; c.n_sink = opt->n_sink; c.score_mode = opt->score_mode;
    c.merge_mode = opt->merge_mode; c.log_cap = h->opt.log_capacity;

    struct { void** p; size_t n; int fill; } bufs[] = {
        { &c.K, s.kv, 0 }, { &c.V, s.kv, 0 }, { (void**)&c.a, s.a, 0 },
        { (void**)&c.pos, s.i32, 0xFF }, { (void**)&c.nxt, s.i32, 0xFF },
        { (void**)&c.log_pos, s.log, 0xFF },
        { (void**)&c.log_slot, s.log, 0xFF }, { (void**)&c.status, s.status, 0 },
        { (void**)&sp.lg, s.lg, 0 }, { &sp.po, s.po, 0 }, { (void**)&sp.pm, s.ps, 0 },
        { (void**)&sp.pl, s.ps, 0 }, { (void**)&sp.pe, s.ps, 0 }, { (void**)&sp.cnt, s.cnt, 0 },
    };
    for (auto& b : bufs) {
        if (b.n == 0) continue;
        e = hipMalloc(b.p, b.n);
        if (e == hipSuccess) e = hipMemset(*b.p, b.fill, b.n);
        if (e != hipSuccess) {
            const bool oom = (e == hipErrorOutOfMemory);
            rc = fail(oom ? WKV_ENOMEM : WKV_EHIP, "device allocation of %zu bytes: %s", b.n, hipGetErrorString(e));
            (void)hipGetLastError();
            for (auto& b2 : bufs) if (*b2.p) (void)hipFree(*b2.p);
            delete h;
            return rc;
        }
    }
    if (opt->max_prompt > 0) {
        rc = prefill_reserve(h, opt->max_prompt);
        if (rc != WKV_OK) {
            for (auto& b2 : bufs) if (*b2.p) (void)hipFree(*b2.p);
            delete h;
            return rc;
        }
    }
    if (opt->replayable) {
        // token index and ticket counter on the device (both start at zero)
        void* clk = nullptr;
        e = hipMalloc(&clk, 16);
        if (e == hipSuccess) e = hipMemset(clk, 0, 16);
        if (e != hipSuccess) {
            rc = fail(e == hipErrorOutOfMemory ? WKV_ENOMEM : WKV_EHIP, "device allocation of the step counter: %s", hipGetErrorString(e));
            (void)hipGetLastError();
            if (clk) (void)hipFree(clk);
            for (auto& b2 : bufs) if (*b2.p) (void)hipFree(*b2.p);
            if (h->pf_scratch) (void)hipFree(h->pf_scratch);
            delete h;
            return rc;
        }
        c.tdev = static_cast<int64_t*>(clk);
        c.tick = reinterpret_cast<uint32_t*>(static_cast<char*>(clk) + 8);
    }
    count_live(h->device, 2 * (long long)s.kv);
    *hp = h;
    return WKV_OK;
}

int wkv_create(wkv_handle** h, int batch, int heads, int head_dim, int budget, int recent_window, int dtype)
{
    wkv_options o;
    memset(&o, 0, sizeof o);
    o.batch = batch; o.heads = heads; o.head_dim = head_dim; o.budget = budget;
    o.recent_window = recent_window; o.dtype = dtype;
    return wkv_create_ex(h, &o);
}

int wkv_step(wkv_handle* h, const void* q, const void* k_new, const void* v_new, void* out, void* stream)
{
    if (!h) return fail(WKV_EINVAL, "null handle");
    if (!q || !k_new || !v_new || !out) return fail(WKV_EINVAL, "null device pointer");
    if ((((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)out) & 15) != 0)
        return fail(WKV_EINVAL, "q, k_new, v_new and out must be 16-byte aligned");
    if (h->t >= 0x7FFFFFF0LL) return fail(WKV_ESIZE, "token counter would overflow");
    const int rc = on_device(h);
    if (rc != WKV_OK) return rc;
    const hipError_t e = h->sp.S > 1
        ? wkv_launch_split(h->c, h->sp, h->opt.dtype, h->opt.head_dim, h->threads, stream_loads(h->opt, h->device),
                           q, k_new, v_new, out, h->t, (hipStream_t)stream)
        : wkv_launch_step(h->c, h->opt.dtype, h->opt.head_dim, h->threads, stream_loads(h->opt, h->device),
                          q, k_new, v_new, out, h->t, (hipStream_t)stream);
    if (e != hipSuccess) return fail(WKV_EHIP, "kernel launch: %s", hipGetErrorString(e));
    h->t += 1;
    return WKV_OK;
}

int wkv_prefill(wkv_handle* h, const void* q, const void* k, const void* v, void* out, int n_tokens,
                void* stream)
{
    int rc = prefill_check(h, q, k, v, out, n_tokens);
    if (rc != WKV_OK) return rc;
    rc = prefill_reserve(h, n_tokens);
    if (rc != WKV_OK) return rc;
    double* lse = h->pf_scratch;
    double* a = lse + (size_t)h->c.units * (size_t)n_tokens;
    const hipError_t e = wkv_launch_prefill(h->c, h->opt.dtype, h->opt.head_dim, q, k, v, out, lse, a, n_tokens,
                                            (hipStream_t)stream);
    if (e != hipSuccess) return fail(WKV_EHIP, "kernel launch: %s", hipGetErrorString(e));
    if (h->c.tdev) {
        const hipError_t e3 = wkv_launch_set_clock(h->c, n_tokens, (hipStream_t)stream);
        if (e3 != hipSuccess) return fail(WKV_EHIP, "kernel launch: %s", hipGetErrorString(e3));
    }
    h->t = n_tokens;
    h->log_from = n_tokens;
    return WKV_OK;
}

int wkv_prefill_noalloc(wkv_handle* h, const void* q, const void* k, const void* v, void* out, int n_tokens,
                        void* stream)
{
    int rc = prefill_check(h, q, k, v, out, n_tokens);
    if (rc != WKV_OK) return rc;
    const size_t need = 2 * (size_t)h->c.units * (size_t)n_tokens * sizeof(double);
    if (need > WKV_NOALLOC_SCRATCH_BYTES)
        return fail(WKV_ESIZE, "units x n_tokens = %zu exceeds the %zu the static scratch of wkv_prefill_noalloc holds",
                    (size_t)h->c.units * (size_t)n_tokens, (size_t)WKV_NOALLOC_SCRATCH_BYTES / 16);
    double* base = nullptr;
    hipError_t e = wkv_prefill_static_scratch(h->device, &base);
    if (e != hipSuccess) return fail(WKV_EHIP, "address of the static scratch: %s", hipGetErrorString(e));
    double* lse = base;
    double* a = lse + (size_t)h->c.units * (size_t)n_tokens;
    e = wkv_launch_prefill(h->c, h->opt.dtype, h->opt.head_dim, q, k, v, out, lse, a, n_tokens, (hipStream_t)stream);
    if (e != hipSuccess) return fail(WKV_EHIP, "kernel launch: %s", hipGetErrorString(e));
    if (h->c.tdev) {
        const hipError_t e3 = wkv_launch_set_clock(h->c, n_tokens, (hipStream_t)stream);
        if (e3 != hipSuccess) return fail(WKV_EHIP, "kernel launch: %s", hipGetErrorString(e3));
    }
    h->t = n_tokens;
    h->log_from = n_tokens;
    return WKV_OK;
}

static int state_impl(wkv_handle* h, int what, void* dst, size_t bytes)
{
    const WkvCache& c = h->c;
    const size_t units = c.units, cap = c.m;
    if (c.tdev) {
        // replayable handle: the device counts the steps (graph replays advance it without the host)
        int rc0 = on_device(h);
        if (rc0 != WKV_OK) return rc0;
        hipError_t e0 = hipDeviceSynchronize();
        int64_t td = 0;
        if (e0 == hipSuccess) e0 = hipMemcpy(&td, c.tdev, sizeof td, hipMemcpyDeviceToHost);
        if (e0 != hipSuccess) return fail(WKV_EHIP, "reading the step counter: %s", hipGetErrorString(e0));
        h->t = td;
    }
    const int64_t T = h->t;
    const size_t len = (size_t)std::min<int64_t>(T, c.m);
    if (what == WKV_STEP) {
        if (bytes < sizeof(int64_t)) return fail(WKV_ESIZE, "need 8 bytes");
        memcpy(dst, &T, sizeof T);
        return WKV_OK;
    }
    if (what == WKV_LEN) {
        if (bytes < sizeof(int32_t)) return fail(WKV_ESIZE, "need 4 bytes");
        const int32_t l = (int32_t)len;
        memcpy(dst, &l, sizeof l);
        return WKV_OK;
    }
    int rc = on_device(h);
    if (rc != WKV_OK) return rc;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail(WKV_EHIP, "hipDeviceSynchronize: %s", hipGetErrorString(e));

    if (what == WKV_STATUS) {
        if (bytes < 2 * sizeof(int32_t)) return fail(WKV_ESIZE, "need 8 bytes");
        e = hipMemcpy(dst, c.status, 2 * sizeof(int32_t), hipMemcpyDeviceToHost);
        return e == hipSuccess ? WKV_OK : fail(WKV_EHIP, "hipMemcpy: %s", hipGetErrorString(e));
    }
    if (what == WKV_EVICT_POS || what == WKV_EVICT_SLOT) {
        if (bytes % (4 * units) != 0) return fail(WKV_EINVAL, "bytes must be a multiple of 4*units");
        const int64_t n = (int64_t)(bytes / (4 * units));
        const int64_t avail = std::min<int64_t>(T - h->log_from, c.log_cap);
        if (n > avail)
            return fail(WKV_ESIZE, "asked for %lld steps of log, %lld available", (long long)n, (long long)avail);
        const int32_t* src = (what == WKV_EVICT_POS) ? c.log_pos : c.log_slot;
        for (int64_t s = T - n; s < T; ++s) {       // ring: at most two contiguous pieces; keep it simple
            e = hipMemcpy((char*)dst + (size_t)(s - (T - n)) * units * 4, src + (size_t)(s % c.log_cap) * units,
                          units * 4, hipMemcpyDeviceToHost);
            if (e != hipSuccess) return fail(WKV_EHIP, "hipMemcpy: %s", hipGetErrorString(e));
        }
        return WKV_OK;
    }

    const size_t d = h->opt.head_dim, eb = dtype_bytes(h->opt.dtype);
    size_t need;
    switch (what) {
    case WKV_K: case WKV_V: need = units * len * d * eb; break;
    case WKV_SCORE_SUM: need = units * len * sizeof(double); break;
    case WKV_COUNT: case WKV_POS: case WKV_NMERGED: need = units * len * sizeof(int32_t); break;
    default: return fail(WKV_EINVAL, "unknown state item %d", what);
    }
    if (bytes < need) return fail(WKV_ESIZE, "need %zu bytes, got %zu", need, bytes);
    if (len == 0) return WKV_OK;

    // token order of the live slots (physical slots 0..len-1) of every unit
    std::vector<int32_t> pos(units * cap);
    e = hipMemcpy(pos.data(), c.pos, pos.size() * 4, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(WKV_EHIP, "hipMemcpy: %s", hipGetErrorString(e));
    std::vector<int32_t> order(units * len);
    for (size_t u = 0; u < units; ++u) {
        int32_t* idx = order.data() + u * len;
        std::iota(idx, idx + len, 0);
        const int32_t* pu = pos.data() + u * cap;
        std::sort(idx, idx + len, [pu](int32_t x, int32_t y) { return pu[x] < pu[y]; });
    }

    auto gather = [&](const void* dev, size_t elem, auto&& emit) -> int {
        std::vector<char> raw(units * cap * elem);
        hipError_t e2 = hipMemcpy(raw.data(), dev, raw.size(), hipMemcpyDeviceToHost);
        if (e2 != hipSuccess) return fail(WKV_EHIP, "hipMemcpy: %s", hipGetErrorString(e2));
        for (size_t u = 0; u < units; ++u)
            for (size_t l = 0; l < len; ++l)
                emit(u * len + l, raw.data() + (u * cap + order[u * len + l]) * elem);
        return WKV_OK;
    };
    switch (what) {
    case WKV_K: case WKV_V: {
        const size_t rb = d * eb;
        return gather(what == WKV_K ? c.K : c.V, rb,
                      [&](size_t o, const char* src) { memcpy((char*)dst + o * rb, src, rb); });
    }
    case WKV_SCORE_SUM:
        return gather(c.a, sizeof(double),
                      [&](size_t o, const char* src) { memcpy((char*)dst + o * 8, src, 8); });
    case WKV_POS:
        return gather(c.pos, 4, [&](size_t o, const char* src) { memcpy((char*)dst + o * 4, src, 4); });
    case WKV_NMERGED: {
        // Raw values folded into a slot.  Merging only ever joins a token with its right
        // neighbour, so a slot holds the contiguous run of tokens that ends at its own key:
        // the count is the distance to the previous retained key.  Without merging it is 1.
        const bool merging = h->opt.merge_mode == WKV_MERGE_CONVEX;
        for (size_t u = 0; u < units; ++u) {
            int32_t prev = -1;
            for (size_t l = 0; l < len; ++l) {
                const int32_t p = pos[u * cap + order[u * len + l]];
                const int32_t n = merging ? p - prev : 1;
                memcpy((char*)dst + (u * len + l) * 4, &n, 4);
                prev = p;
            }
        }
        return WKV_OK;
    }
    case WKV_COUNT:     // n = steps attended = tokens - pos (every live slot is attended once per step)
        return gather(c.pos, 4, [&](size_t o, const char* src) {
            int32_t p; memcpy(&p, src, 4);
            const int32_t n = (int32_t)(T - p);
            memcpy((char*)dst + o * 4, &n, 4);
        });
    }
    return fail(WKV_EINVAL, "unknown state item %d", what);
}

int wkv_state(wkv_handle* h, int what, void* dst, size_t bytes)
{
    if (!h || !dst) return fail(WKV_EINVAL, "null argument");
    try {
        return state_impl(h, what, dst, bytes);
    } catch (const std::bad_alloc&) {
        return fail(WKV_ENOMEM, "host allocation failed");
    }
}

static int load_impl(wkv_handle* h, int64_t tokens, int len, const void* K, const void* V,
                     const double* score_sum, const int32_t* pos)
{
    WkvCache& c = h->c;
    const size_t units = c.units, m = c.m;
    if (tokens < 0 || tokens >= 0x7FFFFFF0LL) return fail(WKV_EINVAL, "tokens out of range");
    if (len != (int)std::min<int64_t>(tokens, c.m)) return fail(WKV_EINVAL, "len must equal min(tokens, budget)");
    if (len > 0 && (!K || !V || !score_sum || !pos)) return fail(WKV_EINVAL, "null state array");
    for (size_t u = 0; u < units && len > 0; ++u) {
        const int32_t* pu = pos + u * len;
        for (int l = 0; l < len; ++l)
            if (pu[l] < 0 || pu[l] >= tokens || (l > 0 && pu[l] <= pu[l - 1]))
                return fail(WKV_EINVAL, "pos of unit %zu is not strictly increasing within [0, tokens)", u);
        if (pu[len - 1] != tokens - 1) return fail(WKV_EINVAL, "the newest token must be retained (unit %zu)", u);
    }
    int rc = on_device(h);
    if (rc != WKV_OK) return rc;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail(WKV_EHIP, "hipDeviceSynchronize: %s", hipGetErrorString(e));
    // device layout: slot l of a unit holds the l-th token in token order, links run l -> l+1
    const size_t rb = (size_t)h->opt.head_dim * dtype_bytes(h->opt.dtype);
    std::vector<int32_t> hp(units * m, -1), hn(units * m, -1);
    std::vector<double> ha(units * m, 0.0);
    for (size_t u = 0; u < units; ++u)
        for (int l = 0; l < len; ++l) {
            hp[u * m + l] = pos[u * len + l];
            hn[u * m + l] = (l + 1 < len) ? l + 1 : -1;
            ha[u * m + l] = score_sum[u * len + l];
        }
    if (len > 0) {
        e = hipMemcpy2D(c.K, m * rb, K, (size_t)len * rb, (size_t)len * rb, units, hipMemcpyHostToDevice);
        if (e == hipSuccess)
            e = hipMemcpy2D(c.V, m * rb, V, (size_t)len * rb, (size_t)len * rb, units, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMemcpy(c.a, ha.data(), ha.size() * sizeof(double), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c.pos, hp.data(), hp.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c.nxt, hn.data(), hn.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(c.log_pos, 0xFF, (size_t)c.log_cap * units * 4);
    if (e == hipSuccess) e = hipMemset(c.log_slot, 0xFF, (size_t)c.log_cap * units * 4);
    if (e == hipSuccess && c.tdev) {
        e = wkv_launch_set_clock(c, tokens, nullptr);
        if (e == hipSuccess) e = hipDeviceSynchronize();
    }
    if (e != hipSuccess) return fail(WKV_EHIP, "uploading the state: %s (the cache may be partly overwritten)", hipGetErrorString(e));
    h->t = tokens;
    h->log_from = tokens;
    return WKV_OK;
}

int wkv_load(wkv_handle* h, int64_t tokens, int len, const void* K, const void* V,
             const double* score_sum, const int32_t* pos)
{
    if (!h) return fail(WKV_EINVAL, "null handle");
    try {
        return load_impl(h, tokens, len, K, V, score_sum, pos);
    } catch (const std::bad_alloc&) {
        return fail(WKV_ENOMEM, "host allocation failed");
    }
}

int wkv_probe_read(const void* src, size_t bytes, int workgroups, int threads, int nontemporal, void* sink, void* stream)
{
    if (!src) return fail(WKV_EINVAL, "null device pointer");
    if (((uintptr_t)src & 15) != 0) return fail(WKV_EINVAL, "src must be 16-byte aligned");
    if (workgroups < 1 || threads < 64 || threads > 1024 || threads % 64 != 0)
        return fail(WKV_EINVAL, "workgroups must be positive, threads a multiple of 64 in 64..1024");
    if (bytes == 0 || bytes % (16 * (size_t)workgroups) != 0)
        return fail(WKV_EINVAL, "bytes must be a positive multiple of 16*workgroups");
    const hipError_t e = wkv_launch_probe_read(src, bytes, workgroups, threads, nontemporal != 0, sink, (hipStream_t)stream);
    if (e != hipSuccess) return fail(WKV_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return WKV_OK;
}

int wkv_destroy(wkv_handle* h)
{
    if (!h) return WKV_OK;
    // wait for the handle's device, whichever is current
    int cur = -1;
    const bool moved = hipGetDevice(&cur) == hipSuccess && cur != h->device && hipSetDevice(h->device) == hipSuccess;
    (void)hipDeviceSynchronize();
    WkvCache& c = h->c;
    void* bufs[] = { c.K, c.V, c.a, c.pos, c.nxt, c.log_pos, c.log_slot, c.status,
                     h->sp.lg, h->sp.po, h->sp.pm, h->sp.pl, h->sp.pe, h->sp.cnt };
    for (void* b : bufs) if (b) (void)hipFree(b);
    if (h->pf_scratch) (void)hipFree(h->pf_scratch);
    if (c.tdev) (void)hipFree(c.tdev);
    count_live(h->device, -2 * (long long)sizes(h->opt, h->sp.S).kv);
    if (moved) (void)hipSetDevice(cur);
    delete h;
    return WKV_OK;
}

}  // extern "C"
