/*
 * A plain C caller of libwkv: no Python, no PyTorch.  It streams a few tokens through a
 * small cache on device 0 and checks facts that hold for any input: with every value row
 * equal to one constant vector, every output and every (merged) cached value equals that
 * vector; the cache holds min(tokens, budget) slots; token positions are strictly increasing
 * and end at the newest token; merge counts sum to the number of tokens; the eviction log
 * names tokens outside the recent window.  Then the same facts for a prompt that goes through
 * wkv_prefill into an fp16 cache, followed by one decode step; the same through wkv_create_ex
 * (device-side token index) and wkv_prefill_noalloc; wkv_launch_shape; wkv_probe_read.
 * Prints "c_abi ok" and exits 0 on success.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/wkv.h"

#define B 2
#define H 3
#define D 64
#define M 5
#define R 2
#define T 23
#define UNITS (B * H)

#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip: %s (line %d)\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define WKV(x) do { int r_ = (x); if (r_ != WKV_OK) { printf("wkv: %d %s (line %d)\n", r_, wkv_last_error(), __LINE__); return 3; } } while (0)
#define CHECK(c) do { if (!(c)) { printf("check failed: %s (line %d)\n", #c, __LINE__); return 4; } } while (0)

/* values k/64 with |k| <= 64 are exact in fp16: sign, exponent, 10 fraction bits, no rounding needed */
static uint16_t half_of_64th(int k)
{
    if (k == 0) return 0;
    const uint16_t sign = k < 0 ? 0x8000 : 0;
    unsigned a = (unsigned)(k < 0 ? -k : k);          /* value = a / 64, 1 <= a <= 64 */
    int e = 0;
    while ((a >> e) > 1) ++e;                          /* leading bit of a */
    const unsigned frac = (a << (10 - e)) & 0x3FF;     /* bits below the leading one, left aligned */
    return (uint16_t)(sign | ((unsigned)(e - 6 + 15) << 10) | frac);
}
static float half_value(uint16_t h)
{
    const int e = (h >> 10) & 31;
    const float m = (float)(h & 0x3FF) / 1024.0f;
    const float v = e ? ldexpf(1.0f + m, e - 15) : ldexpf(m, -14);
    return (h & 0x8000) ? -v : v;
}

static float lcg(unsigned* s) { *s = *s * 1664525u + 1013904223u; return ((*s >> 8) & 0xFFFF) / 32768.0f - 1.0f; }

int main(void)
{
    const size_t n = (size_t)UNITS * D;
    float *hq = malloc(n * 4), *hk = malloc(n * 4), *hv = malloc(n * 4), *ho = malloc(n * 4);
    float *dq, *dk, *dv, *dout;
    HIP(hipMalloc((void**)&dq, n * 4)); HIP(hipMalloc((void**)&dk, n * 4));
    HIP(hipMalloc((void**)&dv, n * 4)); HIP(hipMalloc((void**)&dout, n * 4));
    wkv_handle* h = NULL;
    CHECK(wkv_create(&h, B, H, 96, M, R, WKV_FP32) == WKV_EINVAL && h == NULL);   /* bad head_dim is refused */
    WKV(wkv_create(&h, B, H, D, M, R, WKV_FP32));

    float cvec[D];
    unsigned seed = 7;
    for (int c = 0; c < D; ++c) cvec[c] = lcg(&seed);
    for (int t = 0; t < T; ++t) {
        for (size_t i = 0; i < n; ++i) { hq[i] = lcg(&seed); hk[i] = lcg(&seed); hv[i] = cvec[i % D]; }
        HIP(hipMemcpy(dq, hq, n * 4, hipMemcpyHostToDevice));
        HIP(hipMemcpy(dk, hk, n * 4, hipMemcpyHostToDevice));
        HIP(hipMemcpy(dv, hv, n * 4, hipMemcpyHostToDevice));
        WKV(wkv_step(h, dq, dk, dv, dout, NULL));
        HIP(hipMemcpy(ho, dout, n * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < n; ++i) CHECK(fabsf(ho[i] - cvec[i % D]) <= 1e-5f * fabsf(cvec[i % D]) + 1e-7f);
    }

    int64_t tokens = 0; int32_t len = 0;
    WKV(wkv_state(h, WKV_STEP, &tokens, sizeof tokens));
    WKV(wkv_state(h, WKV_LEN, &len, sizeof len));
    CHECK(tokens == T && len == M);
    int32_t pos[UNITS * M], nm[UNITS * M], cnt[UNITS * M], ev[T * UNITS];
    float V[UNITS * M * D];
    WKV(wkv_state(h, WKV_POS, pos, sizeof pos));
    WKV(wkv_state(h, WKV_NMERGED, nm, sizeof nm));
    WKV(wkv_state(h, WKV_COUNT, cnt, sizeof cnt));
    WKV(wkv_state(h, WKV_V, V, sizeof V));
    WKV(wkv_state(h, WKV_EVICT_POS, ev, sizeof ev));
    CHECK(wkv_state(h, WKV_POS, pos, sizeof pos - 4) == WKV_ESIZE);
    for (int u = 0; u < UNITS; ++u) {
        int total = 0;
        for (int l = 0; l < M; ++l) {
            if (l) CHECK(pos[u * M + l] > pos[u * M + l - 1]);
            CHECK(cnt[u * M + l] == T - pos[u * M + l]);
            total += nm[u * M + l];
            for (int c = 0; c < D; ++c)
                CHECK(fabsf(V[(u * M + l) * D + c] - cvec[c]) <= 1e-6f * fabsf(cvec[c]) + 1e-7f);
        }
        CHECK(pos[u * M + M - 1] == T - 1 && total == T);
        for (int t = 0; t < T; ++t) {
            const int e = ev[t * UNITS + u];
            if (t < M) CHECK(e == -1); else CHECK(e >= 0 && e <= t - R);
        }
    }
    WKV(wkv_destroy(h));
    HIP(hipFree(dq)); HIP(hipFree(dk)); HIP(hipFree(dv)); HIP(hipFree(dout));
    free(hq); free(hk); free(hv); free(ho);

    /* ---- a prompt of PT tokens through wkv_prefill (fp16 cache), then one decode step */
    {
#define PT 37
        const size_t np = (size_t)(PT + 1) * UNITS * D;
        uint16_t *pq = malloc(np * 2), *pk = malloc(np * 2), *pv = malloc(np * 2), *po = malloc(np * 2);
        uint16_t chalf[D];
        for (int c = 0; c < D; ++c) chalf[c] = half_of_64th((int)(lcg(&seed) * 64.0f));
        for (size_t i = 0; i < np; ++i) {
            pq[i] = half_of_64th((int)(lcg(&seed) * 64.0f));
            pk[i] = half_of_64th((int)(lcg(&seed) * 64.0f));
            pv[i] = chalf[i % D];
        }
        uint16_t *gq, *gk, *gv, *go;
        HIP(hipMalloc((void**)&gq, np * 2)); HIP(hipMalloc((void**)&gk, np * 2));
        HIP(hipMalloc((void**)&gv, np * 2)); HIP(hipMalloc((void**)&go, np * 2));
        HIP(hipMemcpy(gq, pq, np * 2, hipMemcpyHostToDevice));
        HIP(hipMemcpy(gk, pk, np * 2, hipMemcpyHostToDevice));
        HIP(hipMemcpy(gv, pv, np * 2, hipMemcpyHostToDevice));
        HIP(hipMemset(go, 0, np * 2));
        WKV(wkv_create(&h, B, H, D, M, R, WKV_FP16));
        CHECK(wkv_prefill(h, gq, gk, gv, go, 0, NULL) == WKV_EINVAL);
        WKV(wkv_prefill(h, gq, gk, gv, go, PT, NULL));
        CHECK(wkv_prefill(h, gq, gk, gv, go, PT, NULL) == WKV_EINVAL);       /* the cache is no longer empty */
        const size_t step = (size_t)UNITS * D;
        WKV(wkv_step(h, gq + PT * step, gk + PT * step, gv + PT * step, go + PT * step, NULL));
        HIP(hipDeviceSynchronize());
        HIP(hipMemcpy(po, go, np * 2, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < np; ++i) {
            const float want = half_value(chalf[i % D]);
            CHECK(fabsf(half_value(po[i]) - want) <= 2e-3f * fabsf(want) + 1e-6f);
        }
        WKV(wkv_state(h, WKV_STEP, &tokens, sizeof tokens));
        WKV(wkv_state(h, WKV_LEN, &len, sizeof len));
        CHECK(tokens == PT + 1 && len == M);
        WKV(wkv_state(h, WKV_POS, pos, sizeof pos));
        WKV(wkv_state(h, WKV_NMERGED, nm, sizeof nm));
        for (int u = 0; u < UNITS; ++u) {
            int total = 0;
            for (int l = 0; l < M; ++l) {
                if (l) CHECK(pos[u * M + l] > pos[u * M + l - 1]);
                total += nm[u * M + l];
            }
            CHECK(pos[u * M + M - 1] == PT && total == PT + 1);
        }
        WKV(wkv_destroy(h));

        /* ---- the same prompt through wkv_prefill_noalloc, into a handle made with wkv_create_ex whose
         * token index lives on the device (replayable): the retained tokens must be the same */
        {
            wkv_options o;
            memset(&o, 0, sizeof o);
            o.batch = B; o.heads = H; o.head_dim = D; o.budget = M; o.recent_window = R; o.dtype = WKV_FP16;
            o.max_prompt = PT; o.replayable = 1;
            int groups = 0, threads = 0;
            WKV(wkv_launch_shape(&o, &groups, &threads));
            CHECK(groups >= UNITS && groups % UNITS == 0 && (threads == 256 || threads == 512 || threads == 1024));
            o.reserved[0] = 1;
            CHECK(wkv_launch_shape(&o, &groups, &threads) == WKV_EINVAL);   /* reserved fields must be zero */
            o.reserved[0] = 0;
            wkv_handle* h2 = NULL;
            WKV(wkv_create_ex(&h2, &o));
            WKV(wkv_prefill_noalloc(h2, gq, gk, gv, go, PT, NULL));
            WKV(wkv_step(h2, gq + PT * step, gk + PT * step, gv + PT * step, go + PT * step, NULL));
            int64_t tokens2 = 0;
            int32_t pos2[UNITS * M];
            WKV(wkv_state(h2, WKV_STEP, &tokens2, sizeof tokens2));
            WKV(wkv_state(h2, WKV_POS, pos2, sizeof pos2));
            CHECK(tokens2 == PT + 1);
            CHECK(memcmp(pos2, pos, sizeof pos2) == 0);
            WKV(wkv_destroy(h2));
        }
        /* ---- the streaming-read yardstick: argument checks and one launch */
        CHECK(wkv_probe_read(NULL, 4096, 4, 256, 0, NULL, NULL) == WKV_EINVAL);
        CHECK(wkv_probe_read(gq, 4096 + 16, 4, 256, 0, NULL, NULL) == WKV_EINVAL);
        WKV(wkv_probe_read(gq, (np * 2) / 64 * 64, 4, 256, 1, NULL, NULL));
        HIP(hipDeviceSynchronize());
        HIP(hipFree(gq)); HIP(hipFree(gk)); HIP(hipFree(gv)); HIP(hipFree(go));
        free(pq); free(pk); free(pv); free(po);
    }
    printf("c_abi ok\n");
    return 0;
}
