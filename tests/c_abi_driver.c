/*
 * The library used from plain C through include/distattn.h, with no Python and no torch: device memory from the HIP
 * runtime, one KV append, one fused attention call, one MicroAttention + aggregation pair, all checked against
 * attention written out in double precision in this file.  Built by paper_2401_02669_amd/build.py (gcc) and run by
 * tests/test_gpu_c_abi.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include "../include/distattn.h"

#define CHECK_HIP(x)                                                        \
    do {                                                                    \
        hipError_t e_ = (x);                                                \
        if (e_ != hipSuccess) {                                             \
            fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__); \
            return 2;                                                       \
        }                                                                   \
    } while (0)
#define CHECK_DA(x)                                                                          \
    do {                                                                                     \
        da_status s_ = (x);                                                                  \
        if (s_ != DA_OK) {                                                                   \
            fprintf(stderr, "%s at line %d\n", da_status_string(s_), __LINE__);              \
            return 3;                                                                        \
        }                                                                                    \
    } while (0)

enum { B = 3, HQ = 8, HKV = 2, D = 128, T = 16, MAXB = 8, NPHYS = B * MAXB };

static uint64_t lcg = 20240102;
static float rnd(void)
{
    lcg = lcg * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((double)(lcg >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

/* softmax(scale q K^T) V for one (request, q-head), written out */
static void reference(const float *q, const float *kp, const float *vp, const int32_t *table, int L, int r, int h,
                      float scale, double *out)
{
    const int g = h / (HQ / HKV);
    double m = -INFINITY, e = 0.0, s[MAXB * T];
    for (int i = 0; i < L; ++i) {
        const size_t row = (((size_t)table[r * MAXB + i / T] * HKV + g) * T + i % T) * D;
        double acc = 0.0;
        for (int c = 0; c < D; ++c) acc += (double)q[((size_t)r * HQ + h) * D + c] * (double)kp[row + c];
        s[i] = acc * scale;
        if (s[i] > m) m = s[i];
    }
    for (int c = 0; c < D; ++c) out[c] = 0.0;
    for (int i = 0; i < L; ++i) {
        const size_t row = (((size_t)table[r * MAXB + i / T] * HKV + g) * T + i % T) * D;
        const double w = exp(s[i] - m);
        e += w;
        for (int c = 0; c < D; ++c) out[c] += w * (double)vp[row + c];
    }
    for (int c = 0; c < D; ++c) out[c] = L > 0 ? out[c] / e : 0.0;
}

int main(void)
{
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
        fprintf(stderr, "no GPU\n");
        return 4;
    }
    const size_t pool_elems = (size_t)NPHYS * HKV * T * D;
    float *kp = malloc(pool_elems * 4), *vp = malloc(pool_elems * 4);
    float *q = malloc((size_t)B * HQ * D * 4), *knew = malloc((size_t)B * HKV * D * 4), *vnew = malloc((size_t)B * HKV * D * 4);
    int32_t table[B * MAXB], lens[B] = {100, 0, 47};
    for (size_t i = 0; i < pool_elems; ++i) { kp[i] = rnd(); vp[i] = rnd(); }
    for (size_t i = 0; i < (size_t)B * HQ * D; ++i) q[i] = rnd();
    for (size_t i = 0; i < (size_t)B * HKV * D; ++i) { knew[i] = rnd(); vnew[i] = rnd(); }
    for (int i = 0; i < B * MAXB; ++i) table[i] = (i * 7 + 3) % NPHYS;   /* 7 is coprime to 24: a permutation */

    void *d_k, *d_v, *d_q, *d_kn, *d_vn, *d_table, *d_lens, *d_out, *d_lse, *d_ws, *d_po, *d_pm, *d_pe;
    CHECK_HIP(hipMalloc(&d_k, pool_elems * 4));
    CHECK_HIP(hipMalloc(&d_v, pool_elems * 4));
    CHECK_HIP(hipMalloc(&d_q, (size_t)B * HQ * D * 4));
    CHECK_HIP(hipMalloc(&d_kn, (size_t)B * HKV * D * 4));
    CHECK_HIP(hipMalloc(&d_vn, (size_t)B * HKV * D * 4));
    CHECK_HIP(hipMalloc(&d_table, sizeof table));
    CHECK_HIP(hipMalloc(&d_lens, sizeof lens));
    CHECK_HIP(hipMalloc(&d_out, (size_t)B * HQ * D * 4));
    CHECK_HIP(hipMalloc(&d_lse, (size_t)B * HQ * 4));
    CHECK_HIP(hipMemcpy(d_k, kp, pool_elems * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_v, vp, pool_elems * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_q, q, (size_t)B * HQ * D * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_kn, knew, (size_t)B * HKV * D * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_vn, vnew, (size_t)B * HKV * D * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_table, table, sizeof table, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_lens, lens, sizeof lens, hipMemcpyHostToDevice));

    da_problem p;
    memset(&p, 0, sizeof p);
    p.batch = B; p.num_q_heads = HQ; p.num_kv_heads = HKV; p.head_dim = D; p.block_tokens = T;
    p.max_blocks_per_seq = MAXB; p.num_phys_blocks = NPHYS; p.kv_dtype = DA_F32; p.q_dtype = DA_F32;
    p.scale = 0.0883883f; p.kv_token_stride = D; p.kv_head_stride = (int64_t)T * D; p.kv_block_stride = (int64_t)HKV * T * D;
    p.q_len = 1;

    /* the new token joins the cache (host mirror updated the same way) */
    CHECK_DA(da_append(&p, d_kn, d_vn, d_k, d_v, d_table, d_lens, NULL, NULL));
    for (int r = 0; r < B; ++r) {
        const int L = lens[r];
        for (int g = 0; g < HKV; ++g) {
            const size_t row = (((size_t)table[r * MAXB + L / T] * HKV + g) * T + L % T) * D;
            memcpy(kp + row, knew + ((size_t)r * HKV + g) * D, D * 4);
            memcpy(vp + row, vnew + ((size_t)r * HKV + g) * D, D * 4);
        }
        lens[r] = L + 1;
    }

    da_plan *plan = NULL;
    CHECK_DA(da_plan_create(&p, lens, NULL, NULL, &plan));
    size_t ws_bytes = 0;
    int64_t nparts = 0;
    CHECK_DA(da_workspace_bytes(plan, &ws_bytes));
    CHECK_DA(da_plan_num_partials(plan, &nparts));
    CHECK_HIP(hipMalloc(&d_ws, ws_bytes ? ws_bytes : 256));
    CHECK_HIP(hipMalloc(&d_po, (size_t)nparts * D * 4));
    CHECK_HIP(hipMalloc(&d_pm, (size_t)nparts * 4));
    CHECK_HIP(hipMalloc(&d_pe, (size_t)nparts * 4));

    float *out = malloc((size_t)B * HQ * D * 4), *out2 = malloc((size_t)B * HQ * D * 4);
    CHECK_DA(da_attention(plan, d_q, d_k, d_v, d_table, d_lens, d_out, d_lse, d_ws, ws_bytes ? ws_bytes : 256, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(out, d_out, (size_t)B * HQ * D * 4, hipMemcpyDeviceToHost));
    CHECK_DA(da_partial(plan, d_q, d_k, d_v, d_table, d_lens, d_po, d_pm, d_pe, NULL));
    CHECK_DA(da_combine(plan, d_po, d_pm, d_pe, d_out, NULL, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(out2, d_out, (size_t)B * HQ * D * 4, hipMemcpyDeviceToHost));
    int32_t flags = -1, dev_lens[B];
    CHECK_DA(da_plan_error(plan, NULL, &flags));
    CHECK_HIP(hipMemcpy(dev_lens, d_lens, sizeof dev_lens, hipMemcpyDeviceToHost));

    double worst = 0.0, ref[D];
    for (int r = 0; r < B; ++r)
        for (int h = 0; h < HQ; ++h) {
            reference(q, kp, vp, table, lens[r], r, h, p.scale, ref);
            for (int c = 0; c < D; ++c) {
                const double a = fabs((double)out[((size_t)r * HQ + h) * D + c] - ref[c]);
                const double b = fabs((double)out2[((size_t)r * HQ + h) * D + c] - ref[c]);
                if (a > worst) worst = a;
                if (b > worst) worst = b;
            }
        }
    CHECK_DA(da_plan_destroy(plan));
    printf("c abi driver: lens %d %d %d, flags %d, %lld partial rows, max-abs %.3e\n", dev_lens[0], dev_lens[1], dev_lens[2],
           flags, (long long)nparts, worst);
    if (flags != 0 || dev_lens[0] != 101 || dev_lens[1] != 1 || dev_lens[2] != 48 || !(worst <= 1e-5)) {
        printf("c abi driver: FAILED\n");
        return 1;
    }
    printf("c abi driver: ok\n");
    return 0;
}
