/*
 * A caller of libvatp written in plain C: device memory from the HIP runtime, the entry points of vatp.h,
 * no Python and no torch.  One head group of a tiny model: prompt pass, prompt prune, three decode steps
 * through vatp_decode_prune_step.  Checks what can be checked without a reference implementation:
 *   - every softmax row sums to one, so the prompt scores sum to the prompt length;
 *   - the survivor indices are ascending, contain the forced prefix and the recent window, and there are
 *     exactly `budget` of them;
 *   - a decode step adds exactly one to the sum of scores before the evicted row's share leaves, so the sum
 *     of the surviving scores is positive and at most the previous sum plus one.
 * Prints "c_abi_demo ok" and returns 0 on success.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "vatp.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_VATP(x) do { vatp_status s_ = (x); if (s_ != VATP_OK) { fprintf(stderr, "%s: %s\n", #x, vatp_strerror(s_)); return 3; } } while (0)

enum { H = 3, D = 64, L = 200, CAP = 200, B = 80, F = 2, R = 8, STEPS = 3 };

static float frand(unsigned *state)
{
    *state = *state * 1664525u + 1013904223u;
    return ((*state >> 8) & 0xffff) / 32768.0f - 1.0f;
}

static void *dev_alloc(size_t bytes)
{
    void *p = NULL;
    if (hipMalloc(&p, bytes) != hipSuccess) return NULL;
    hipMemset(p, 0, bytes);
    return p;
}

int main(void)
{
    const size_t n_prompt = (size_t)H * CAP * D, n_cache = (size_t)H * (B + 1) * D;
    float *hQ = malloc(n_prompt * 4), *hK = malloc(n_prompt * 4), *hV = malloc(n_prompt * 4);
    float *hS = malloc((size_t)H * CAP * 4);
    int32_t *hkept = malloc((size_t)H * (B + 1) * 4);
    unsigned seed = 12345u;
    size_t i;
    int h, t, r;
    for (i = 0; i < n_prompt; ++i) { hQ[i] = 2.f * frand(&seed); hK[i] = 2.f * frand(&seed); hV[i] = frand(&seed); }

    vatp_ctx *ctx = NULL;
    CHECK_VATP(vatp_create(&ctx, 0));
    int32_t len[1] = { L }, budget[1] = { B };
    vatp_params p;
    memset(&p, 0, sizeof p);
    p.batch = 1; p.n_heads = H; p.head_dim = D; p.dtype = VATP_F32; p.n_sink = F; p.recent = R;
    p.cap = CAP; p.cap_out = B + 1; p.len = len; p.budget = budget;

    float *Q = dev_alloc(n_prompt * 4), *K = dev_alloc(n_prompt * 4), *V = dev_alloc(n_prompt * 4);
    float *S = dev_alloc((size_t)H * CAP * 4), *nrm = dev_alloc((size_t)H * CAP * 4);
    float *Kc[2], *Vc[2], *Sc[2], *Nc[2];
    int32_t *synced[2], *kept = dev_alloc((size_t)H * (B + 1) * 4);
    for (t = 0; t < 2; ++t) {
        Kc[t] = dev_alloc(n_cache * 4); Vc[t] = dev_alloc(n_cache * 4);
        Sc[t] = dev_alloc((size_t)H * (B + 1) * 4); Nc[t] = dev_alloc((size_t)H * (B + 1) * 4);
        synced[t] = dev_alloc(H * 4);
    }
    CHECK_HIP(hipMemcpy(Q, hQ, n_prompt * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(K, hK, n_prompt * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(V, hV, n_prompt * 4, hipMemcpyHostToDevice));

    size_t ws_bytes = vatp_workspace_bytes(ctx, &p, VATP_CALL_PREFILL_SCORE);
    void *ws = dev_alloc(ws_bytes);
    CHECK_VATP(vatp_prefill_score(ctx, &p, Q, K, V, S, nrm, ws, ws_bytes, NULL));
    CHECK_HIP(hipMemcpy(hS, S, (size_t)H * CAP * 4, hipMemcpyDeviceToHost));
    for (h = 0; h < H; ++h) {
        double sum = 0;
        for (r = 0; r < L; ++r) sum += hS[h * CAP + r];
        if (fabs(sum - L) > 1e-3 * L) { fprintf(stderr, "head %d: prompt scores sum to %f, not %d\n", h, sum, L); return 1; }
    }

    CHECK_VATP(vatp_select_compact(ctx, &p, K, V, S, nrm, NULL, Kc[0], Vc[0], Sc[0], Nc[0], NULL, kept, NULL, 0, NULL));
    CHECK_HIP(hipMemcpy(hkept, kept, (size_t)H * (B + 1) * 4, hipMemcpyDeviceToHost));
    for (h = 0; h < H; ++h) {
        const int32_t *k = hkept + h * (B + 1);
        for (r = 1; r < B; ++r) if (k[r] <= k[r - 1]) { fprintf(stderr, "head %d: survivors not ascending\n", h); return 1; }
        for (r = 0; r < F; ++r) if (k[r] != r) { fprintf(stderr, "head %d: forced prefix missing\n", h); return 1; }
        for (r = 0; r < R; ++r) if (k[B - R + r] != L - R + r) { fprintf(stderr, "head %d: recent window missing\n", h); return 1; }
    }

    /* decode: the cache now holds B rows per head */
    p.cap = B + 1; p.cap_out = B + 1; len[0] = B;
    size_t ws2_bytes = vatp_workspace_bytes(ctx, &p, VATP_CALL_DECODE_PRUNE_STEP);
    void *ws2 = dev_alloc(ws2_bytes);
    float *q = dev_alloc((size_t)H * D * 4), *kn = dev_alloc((size_t)H * D * 4), *vn = dev_alloc((size_t)H * D * 4);
    float hq[H * D];
    float *hSc = malloc((size_t)H * (B + 1) * 4);
    double prev[H];
    CHECK_HIP(hipMemcpy(hSc, Sc[0], (size_t)H * (B + 1) * 4, hipMemcpyDeviceToHost));
    for (h = 0; h < H; ++h) { prev[h] = 0; for (r = 0; r < B; ++r) prev[h] += hSc[h * (B + 1) + r]; }
    int cur = 0;
    for (t = 0; t < STEPS; ++t) {
        for (i = 0; i < (size_t)H * D; ++i) hq[i] = 2.f * frand(&seed);
        CHECK_HIP(hipMemcpy(q, hq, sizeof hq, hipMemcpyHostToDevice));
        for (i = 0; i < (size_t)H * D; ++i) hq[i] = 2.f * frand(&seed);
        CHECK_HIP(hipMemcpy(kn, hq, sizeof hq, hipMemcpyHostToDevice));
        for (i = 0; i < (size_t)H * D; ++i) hq[i] = frand(&seed);
        CHECK_HIP(hipMemcpy(vn, hq, sizeof hq, hipMemcpyHostToDevice));
        CHECK_VATP(vatp_decode_prune_step(ctx, &p, q, kn, vn, Kc[cur], Vc[cur], Sc[cur], Nc[cur], NULL, NULL, Kc[1 - cur],
                                          Vc[1 - cur], Sc[1 - cur], Nc[1 - cur], NULL, kept, synced[cur], synced[1 - cur], NULL,
                                          ws2, ws2_bytes, NULL));
        cur = 1 - cur;
        CHECK_HIP(hipMemcpy(hSc, Sc[cur], (size_t)H * (B + 1) * 4, hipMemcpyDeviceToHost));
        for (h = 0; h < H; ++h) {
            double sum = 0;
            for (r = 0; r < B; ++r) sum += hSc[h * (B + 1) + r];
            if (sum > prev[h] + 1.0 + 1e-4 || !(sum > 0)) {
                fprintf(stderr, "step %d head %d: scores went from %f to %f\n", t, h, prev[h], sum);
                return 1;
            }
            prev[h] = sum;
        }
    }
    CHECK_HIP(hipDeviceSynchronize());
    vatp_destroy(ctx);
    printf("c_abi_demo ok\n");
    return 0;
}
