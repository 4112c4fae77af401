/* A plain C11 consumer of the C ABI: proves that include/power_smc.h is C, that the library needs nothing but device
 * pointers and sizes, and that one step + resampling + reorder run from C.  Exit status 0 and "c_abi_client ok" on
 * success.  Built by __graft_entry__.build(); run by tests/test_gpu_c_client.py. */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "power_smc.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_SMC(x) do { smc_status s_ = (x); if (s_ != SMC_OK) { printf("%s -> %s (line %d)\n", #x, smc_status_str(s_), __LINE__); return 3; } } while (0)
#define EXPECT(c) do { if (!(c)) { printf("expectation failed: %s (line %d)\n", #c, __LINE__); return 4; } } while (0)

int main(void)
{
    smc_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.B = 3; cfg.N = 4; cfg.V = 4096; cfg.T_max = 8; cfg.logits_dtype = SMC_F32; cfg.eos_id = -1;
    cfg.kappa = 1.0; cfg.seed = 7;
    cfg.kv_tensors = 2; cfg.kv_H = 2; cfg.kv_S = 8; cfg.kv_D = 64; cfg.kv_elem_bytes = 2;
    const int R = cfg.B * cfg.N;
    const size_t row_bytes = (size_t)cfg.kv_H * cfg.kv_S * cfg.kv_D * 2;

    /* argument errors are found on the host, before any device work */
    smc_ctx* ctx = NULL;
    EXPECT(smc_init(NULL, NULL, 0, NULL, &ctx) == SMC_E_NULL);
    EXPECT(smc_step(NULL, NULL, 0, 1, 4.0, 4.0, -1.0, NULL) == SMC_E_NULL);
    EXPECT(strcmp(smc_status_str(SMC_OK), "ok") == 0);

    const size_t ws_bytes = smc_workspace_bytes(&cfg);
    EXPECT(ws_bytes > 0);
    void* d_ws = NULL; float* d_logits = NULL; int32_t* d_tokens = NULL; int32_t* d_anc = NULL; int32_t* d_res = NULL;
    double* d_ess = NULL; void* d_kv[4] = {0}; int32_t* d_hist[2] = {0};
    CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
    CHECK_HIP(hipMalloc((void**)&d_logits, (size_t)R * cfg.V * sizeof(float)));
    CHECK_HIP(hipMalloc((void**)&d_tokens, R * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&d_anc, R * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&d_res, cfg.B * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&d_ess, cfg.B * sizeof(double)));
    for (int i = 0; i < 4; ++i) CHECK_HIP(hipMalloc(&d_kv[i], R * row_bytes));
    for (int i = 0; i < 2; ++i) CHECK_HIP(hipMalloc((void**)&d_hist[i], (size_t)R * cfg.T_max * sizeof(int32_t)));

    /* every row's cache is filled with its own row number, so the reorder can be checked byte by byte */
    unsigned short* h_row = (unsigned short*)malloc(row_bytes);
    for (int t = 0; t < 2; ++t)
        for (int r = 0; r < R; ++r) {
            for (size_t i = 0; i < row_bytes / 2; ++i) h_row[i] = (unsigned short)(1000 * t + r);
            CHECK_HIP(hipMemcpy((char*)d_kv[t] + (size_t)r * row_bytes, h_row, row_bytes, hipMemcpyHostToDevice));
        }
    float* h_logits = (float*)malloc((size_t)R * cfg.V * sizeof(float));
    unsigned x = 12345u;
    for (size_t i = 0; i < (size_t)R * cfg.V; ++i) { x = x * 1664525u + 1013904223u; h_logits[i] = (float)(x >> 8) / 16777216.0f * 12.0f - 6.0f; }
    CHECK_HIP(hipMemcpy(d_logits, h_logits, (size_t)R * cfg.V * sizeof(float), hipMemcpyHostToDevice));

    CHECK_SMC(smc_init(&cfg, d_ws, ws_bytes, NULL, &ctx));
    void* bufA[2] = {d_kv[0], d_kv[1]}; void* bufB[2] = {d_kv[2], d_kv[3]};
    CHECK_SMC(smc_kv_bind(ctx, bufA, bufB, d_hist[0], d_hist[1]));
    EXPECT(smc_step(ctx, d_logits, cfg.V - 1, 1, 4.0, 4.0, -1.0, d_tokens) == SMC_E_SHAPE);   /* stride shorter than a row */
    CHECK_SMC(smc_step(ctx, d_logits, cfg.V, 1, 4.0, 4.0, -1.0, d_tokens));
    CHECK_SMC(smc_resample(ctx, 1, d_anc, d_res, d_ess));
    CHECK_SMC(smc_kv_reindex(ctx, d_anc, d_res, cfg.kv_S, 1));
    CHECK_HIP(hipDeviceSynchronize());

    int32_t tokens[12], anc[12], res[3], parity[12];
    double ess[3], logW[12];
    CHECK_HIP(hipMemcpy(tokens, d_tokens, sizeof tokens, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(anc, d_anc, sizeof anc, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(res, d_res, sizeof res, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(ess, d_ess, sizeof ess, hipMemcpyDeviceToHost));
    CHECK_SMC(smc_get_state(ctx, logW, NULL, parity));
    for (int r = 0; r < R; ++r) {
        EXPECT(tokens[r] >= 0 && tokens[r] < cfg.V);
        EXPECT(anc[r] >= (r / cfg.N) * cfg.N && anc[r] < (r / cfg.N + 1) * cfg.N);    /* ancestors stay inside the prompt */
        EXPECT(parity[r] == (res[r / cfg.N] && anc[r] != r));                          /* exactly the moved rows changed buffer */
        if (res[r / cfg.N]) EXPECT(logW[r] == 0.0);                                    /* weights reset after resampling */
        /* the live row of every tensor holds its ancestor's bytes */
        for (int t = 0; t < 2; ++t) {
            const void* live = (const char*)(parity[r] ? bufB[t] : bufA[t]) + (size_t)r * row_bytes;
            CHECK_HIP(hipMemcpy(h_row, live, row_bytes, hipMemcpyDeviceToHost));
            const unsigned short want = (unsigned short)(1000 * t + (res[r / cfg.N] ? anc[r] : r));
            for (size_t i = 0; i < row_bytes / 2; ++i) EXPECT(h_row[i] == want);
        }
    }
    for (int b = 0; b < cfg.B; ++b) EXPECT(ess[b] >= 1.0 - 1e-9 && ess[b] <= cfg.N + 1e-9);
    CHECK_SMC(smc_destroy(ctx));
    printf("c_abi_client ok\n");
    return 0;
}
