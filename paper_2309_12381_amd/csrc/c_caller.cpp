/*
 * A caller of the C interface alone (no Python, no PyTorch): allocates the state of a
 * Llama-shaped parameter list with hipMalloc, asks mpo_place_second where res, v and the reused
 * gradient buffer should go, steps the list per layer in backward order with mpo_step_layer
 * (arXiv 2309.12381, Section 3.2) and prints one JSON line with the rate it reached.  What a
 * C or C++ program gets from include/mpo.h and include/mpo_probe.h; bench.py --c-caller runs it.
 *
 * usage: mpo_c_caller [hidden intermediate layers vocab [steps [place]]]
 *        defaults: 4096 11008 32 32000 (the Llama-7B shape), 20 steps, place = 1
 */
#include <hip/hip_runtime_api.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "mpo.h"
#include "mpo_probe.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)
#define MPO_OK_(x) do { mpo_status s_ = (x); if (s_ != MPO_OK) { fprintf(stderr, "%s failed: %s\n", #x, mpo_status_string(s_)); return 1; } } while (0)

static uint64_t round_up(uint64_t x, uint64_t k) { return (x + k - 1) / k * k; }

int main(int argc, char **argv)
{
    const uint64_t h = argc > 4 ? strtoull(argv[1], NULL, 10) : 4096, inter = argc > 4 ? strtoull(argv[2], NULL, 10) : 11008;
    const int L = argc > 4 ? atoi(argv[3]) : 32;
    const uint64_t vocab = argc > 4 ? strtoull(argv[4], NULL, 10) : 32000;
    const int steps = argc > 5 ? atoi(argv[5]) : 20, place = argc > 6 ? atoi(argv[6]) : 1;
    if (h == 0 || inter == 0 || L < 1 || L > 200 || vocab == 0 || steps < 1) { fprintf(stderr, "bad arguments\n"); return 2; }

    /* the list: embedding (layer 0), L blocks of 9 tensors, final norm, head */
    const int nt = 1 + 9 * L + 2;
    uint64_t *len = (uint64_t *)malloc(sizeof(uint64_t) * nt);
    int32_t *layer = (int32_t *)malloc(sizeof(int32_t) * nt);
    mpo_tensor *ts = (mpo_tensor *)calloc(nt, sizeof(mpo_tensor));
    if (!len || !layer || !ts) return 1;
    int k = 0;
    len[k] = vocab * h; layer[k++] = 0;
    for (int i = 0; i < L; ++i) {
        const uint64_t block[9] = {h, h * h, h * h, h * h, h * h, h, h * inter, h * inter, inter * h};
        for (int j = 0; j < 9; ++j) { len[k] = block[j]; layer[k++] = i + 1; }
    }
    len[k] = h; layer[k++] = L + 1;
    len[k] = vocab * h; layer[k++] = L + 2;

    /* every tensor starts on a 128-byte line of the 16-bit arrays; one gradient buffer as large as the largest layer */
    uint64_t total = 0, *off = (uint64_t *)malloc(sizeof(uint64_t) * nt), *goff = (uint64_t *)malloc(sizeof(uint64_t) * nt);
    uint64_t layer_fill[256] = {0}, grad_len = 0, params = 0;
    if (!off || !goff) return 1;
    for (int i = 0; i < nt; ++i) {
        off[i] = total; total += round_up(len[i], 64); params += len[i];
        goff[i] = layer_fill[layer[i]]; layer_fill[layer[i]] += round_up(len[i], 64);
        if (layer_fill[layer[i]] > grad_len) grad_len = layer_fill[layer[i]];
    }

    uint16_t *hi = NULL; float *m = NULL; char *block = NULL;
    HIP_OK(hipMalloc((void **)&hi, total * 2));
    HIP_OK(hipMalloc((void **)&m, total * 4));
    mpo_place_report rep;
    memset(&rep, 0, sizeof rep);
    if (place) {
        const int rc = mpo_place_second(hi, total * 2, m, total * 4, total * 2, total * 4, grad_len * 2, 0, 0, (void **)&block, &rep, NULL);
        if (rc != 0) { fprintf(stderr, "mpo_place_second failed (%d)\n", rc); return 1; }
    } else {
        rep.v_offset = round_up(total * 2, 256); rep.grad_offset = rep.v_offset + round_up(total * 4, 256);
        HIP_OK(hipMalloc((void **)&block, rep.grad_offset + grad_len * 2));
    }
    uint16_t *res = (uint16_t *)block; float *v = (float *)(block + rep.v_offset); uint16_t *grad = (uint16_t *)(block + rep.grad_offset);
    /* synthetic values: weights 0x3C3C (bf16, about 0.0115) with residual 0x1111, gradients 0x3838 (about 4.4e-5), moments 0 */
    HIP_OK(hipMemset(hi, 0x3C, total * 2));
    HIP_OK(hipMemset(res, 0x11, total * 2));
    HIP_OK(hipMemset(grad, 0x38, grad_len * 2));
    HIP_OK(hipMemset(m, 0, total * 4));
    HIP_OK(hipMemset(v, 0, total * 4));
    for (int i = 0; i < nt; ++i) {
        ts[i].hi = hi + off[i]; ts[i].res = res + off[i]; ts[i].grad = grad + goff[i];
        ts[i].m = m + off[i]; ts[i].v = v + off[i]; ts[i].n = len[i]; ts[i].layer = layer[i];
    }
    mpo_plan *plan = NULL;
    MPO_OK_(mpo_plan_create(ts, (uint64_t)nt, &plan));
    mpo_adam_cfg cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.lr = 1e-3; cfg.beta1 = 0.9; cfg.beta2 = 0.999; cfg.eps = 1e-8; cfg.loss_scale = 1.0;
    cfg.weight_fmt = MPO_BF16; cfg.grad_fmt = MPO_BF16; cfg.round = MPO_ROUND_TRUNC;

    hipEvent_t e0, e1;
    HIP_OK(hipEventCreate(&e0));
    HIP_OK(hipEventCreate(&e1));
    uint64_t step = 0;
    for (int rep_ = 0; rep_ < 2; ++rep_) {                     /* two untimed steps, then the timed ones */
        const int count = rep_ == 0 ? 2 : steps;
        if (rep_ == 1) HIP_OK(hipEventRecord(e0, NULL));
        for (int s = 0; s < count; ++s) {
            ++step;
            for (int ly = L + 2; ly >= 0; --ly) MPO_OK_(mpo_step_layer(plan, ly, NULL, 0, MPO_OPT_ADAM, &cfg, step, NULL));
        }
    }
    HIP_OK(hipEventRecord(e1, NULL));
    HIP_OK(hipEventSynchronize(e1));
    float ms = 0.0f;
    HIP_OK(hipEventElapsedTime(&ms, e0, e1));
    const double per_step = ms / steps, gbps = 26.0 * (double)params / (per_step * 1e6);
    printf("{\"caller\": \"C interface only\", \"params\": %llu, \"tensors\": %d, \"launches_per_step\": %d, \"steps\": %d, "
           "\"ms_per_step\": %.4f, \"params_per_s\": %.6g, \"GBps\": %.1f, \"frac_of_peak\": %.4f, "
           "\"placement\": {\"searched\": %s, \"split\": %s, \"candidates\": %d, \"chosen\": %d, "
           "\"one_region_GBps\": [%.0f, %.0f, %.0f, %.0f], \"chosen_GBps\": [%.0f, %.0f, %.0f, %.0f], \"peak_transient_bytes\": %llu}}\n",
           (unsigned long long)params, nt, L + 3, steps, per_step, (double)params / (per_step * 1e-3), gbps, gbps / 8000.0,
           place ? "true" : "false", rep.split ? "true" : "false", rep.candidates, rep.chosen,
           rep.one_region_GBps[0], rep.one_region_GBps[1], rep.one_region_GBps[2], rep.one_region_GBps[3],
           rep.chosen_GBps[0], rep.chosen_GBps[1], rep.chosen_GBps[2], rep.chosen_GBps[3],
           (unsigned long long)rep.peak_transient_bytes);
    MPO_OK_(mpo_plan_destroy(plan));
    (void)mpo_place_free(block);
    (void)hipFree(m);
    (void)hipFree(hi);
    free(goff); free(off); free(ts); free(layer); free(len);
    return 0;
}
