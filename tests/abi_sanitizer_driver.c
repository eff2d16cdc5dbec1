/* Calls every entry point of libsamo with arguments its host-side validation must reject before
 * anything is enqueued (so no GPU is needed), plus the host-only entries.  The test builds the
 * library's sources together with this file with AddressSanitizer and UBSan on the HOST code. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "samo.h"

static int failures = 0;
#define EXPECT(call, want)                                                                      \
    do {                                                                                        \
        const samo_status got_ = (call);                                                        \
        if (got_ != (want)) { printf("%s -> %d, expected %d\n", #call, (int)got_, (int)(want)); ++failures; } \
    } while (0)

int main(void)
{
    void *fake = (void *)(uintptr_t)0x7000000000ull;          /* aligned, never dereferenced on the host */
    void *odd = (void *)(uintptr_t)0x7000000004ull;           /* not 16-byte aligned */
    samo_adam_cfg adam = {1e-4f, 0.9f, 0.999f, 1e-8f, 0.0f, 0, 1};
    samo_adam_cfg bad_adam = adam;
    samo_sgd_cfg sgd = {0.1f, 0.9f, 0.0f};
    samo_sgd_cfg bad_sgd = {0.1f, 1.5f, 0.0f};
    int64_t a = 0, b = 0, c = 0;
    size_t bytes = 0;
    samo_plan plan;

    if (samo_abi_version() != SAMO_ABI_VERSION) { printf("abi version\n"); ++failures; }
    for (int s = 1; s >= -10; --s) if (!samo_status_string(s) || !strlen(samo_status_string(s))) ++failures;
    if (samo_seg_ptr_len(0) != 1 || samo_seg_ptr_len(1025) != 3 || samo_seg_ptr_len(-1) != -1) ++failures;
    EXPECT(samo_memory_model(1000, 100, &a, &b, &c), SAMO_OK);
    if (a != 20000 || b != 4400 || c != 3600) { printf("memory model\n"); ++failures; }
    EXPECT(samo_memory_model(10, 11, &a, &b, &c), SAMO_ERR_SIZE);

    EXPECT(samo_count_nonzero(NULL, 10, fake, fake, NULL), SAMO_ERR_NULL);
    EXPECT(samo_count_nonzero(fake, -1, fake, fake, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_build_index(fake, 10, NULL, 5, fake, fake, NULL), SAMO_ERR_NULL);
    EXPECT(samo_build_index(fake, 10, odd, 5, fake, fake, NULL), SAMO_ERR_ALIGN);
    EXPECT(samo_build_index_batched(NULL, 2, NULL), SAMO_ERR_NULL);
    EXPECT(samo_build_index_batched(NULL, -1, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_build_index_batched(NULL, 0, NULL), SAMO_OK);
    EXPECT(samo_build_seg_ptr(fake, 11, 10, fake, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_validate_index(fake, 5, 10, NULL, NULL, NULL), SAMO_ERR_NULL);

    EXPECT(samo_decompress(fake, fake, fake, 5, NULL, 10, NULL), SAMO_ERR_NULL);
    EXPECT(samo_decompress(fake, fake, fake, 11, fake, 10, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_decompress(fake, NULL, NULL, 5, fake, 10, NULL), SAMO_ERR_SIZE);     /* dense needs nnz == n */
    EXPECT(samo_gather_grads(fake, 10, fake, 5, 0.0f, fake, NULL), SAMO_ERR_ARG);
    EXPECT(samo_gather_grads(fake, 10, fake, 5, NAN, fake, NULL), SAMO_ERR_ARG);
    EXPECT(samo_gather_grads(fake, 10, fake, 5, 1.0f, odd, NULL), SAMO_ERR_ALIGN);
    EXPECT(samo_gather_grads_fp16(fake, 10, fake, 5, NULL, 0, NULL), SAMO_ERR_NULL);
    bad_adam.beta1 = 1.0f;
    EXPECT(samo_adam_step(fake, fake, fake, fake, 5, &bad_adam, NULL), SAMO_ERR_ARG);
    bad_adam = adam; bad_adam.step = 0;
    EXPECT(samo_adam_step(fake, fake, fake, fake, 5, &bad_adam, NULL), SAMO_ERR_ARG);
    bad_adam = adam; bad_adam.eps = 0.0f;
    EXPECT(samo_adam_step(fake, fake, fake, fake, 5, &bad_adam, NULL), SAMO_ERR_ARG);
    EXPECT(samo_adam_step(fake, fake, fake, fake, 5, NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_adam_step(fake, fake, fake, fake, -1, &adam, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_sgd_step(fake, fake, fake, 5, &bad_sgd, NULL), SAMO_ERR_ARG);
    EXPECT(samo_sgd_step(fake, NULL, fake, 5, &sgd, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_step(fake, fake, 10, fake, fake, 5, fake, fake, NULL, 1.0f, &adam, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_step(fake, fake, 10, fake, NULL, 5, fake, fake, fake, 1.0f, &adam, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_step(fake, fake, 10, fake, fake, 5, fake, fake, fake, -1.0f, &adam, NULL), SAMO_ERR_ARG);
    EXPECT(samo_adam_expand_step(NULL, fake, 10, fake, fake, 5, fake, fake, fake, 1.0f, &adam, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_sgd_step(fake, fake, 10, fake, fake, 5, fake, fake, 1.0f, &bad_sgd, NULL), SAMO_ERR_ARG);
    EXPECT(samo_fused_step_fp32(fake, NULL, 10, fake, fake, 5, fake, fake, 1.0f, &adam, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_step_fp32(fake, fake, 10, fake, fake, 5, fake, fake, INFINITY, &adam, NULL), SAMO_ERR_ARG);
    EXPECT(samo_fused_step_fp32(fake, fake, 10, fake, fake, 5, odd, fake, 1.0f, &adam, NULL), SAMO_ERR_ALIGN);
    EXPECT(samo_wgrad_gather(fake, fake, 4, 8, 12, NULL, NULL, 96, 1.0f, fake, NULL), SAMO_ERR_SIZE);      /* in % 8 */
    EXPECT(samo_wgrad_gather(fake, fake, -1, 8, 16, NULL, NULL, 128, 1.0f, fake, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_wgrad_gather(fake, fake, 4, 65536, 65536, NULL, NULL, 1, 1.0f, fake, NULL), SAMO_ERR_SIZE); /* out * in >= 2^31 */
    EXPECT(samo_wgrad_gather(fake, fake, 4, 8, 16, NULL, NULL, 90, 1.0f, fake, NULL), SAMO_ERR_NULL);       /* no index, nnz < out * in */
    EXPECT(samo_wgrad_gather(fake, fake, 4, 8, 16, fake, NULL, 90, 1.0f, fake, NULL), SAMO_ERR_NULL);       /* index without seg_ptr */
    EXPECT(samo_wgrad_gather(NULL, fake, 4, 8, 16, fake, fake, 90, 1.0f, fake, NULL), SAMO_ERR_NULL);
    EXPECT(samo_wgrad_gather(fake, fake, 4, 8, 16, fake, fake, 90, 0.0f, fake, NULL), SAMO_ERR_ARG);
    EXPECT(samo_wgrad_gather(fake, odd, 4, 8, 16, fake, fake, 90, 1.0f, fake, NULL), SAMO_ERR_ALIGN);
    EXPECT(samo_wgrad_gather(fake, fake, 4, 8, 16, fake, fake, 0, 1.0f, NULL, NULL), SAMO_OK);              /* nothing kept: nothing to do */
    EXPECT(samo_wgrad_gather_fp16(fake, fake, 4, 8, 16, fake, fake, 90, NULL, 0, NULL), SAMO_ERR_NULL);
    EXPECT(samo_wgrad_gather_fp16(fake, fake, 4, 8, 16, fake, fake, 129, fake, 1, NULL), SAMO_ERR_SIZE);
    {
        samo_wgrad_job jobs[SAMO_WGRAD_MAX_JOBS + 1];
        for (int j = 0; j <= SAMO_WGRAD_MAX_JOBS; ++j) {
            samo_wgrad_job ok = {fake, fake, 4, 8, 16, fake, fake, 0, NULL};     /* nothing kept: skipped */
            jobs[j] = ok;
        }
        EXPECT(samo_wgrad_gather_batched(0, NULL, 1.0f, NULL), SAMO_OK);
        EXPECT(samo_wgrad_gather_batched(SAMO_WGRAD_MAX_JOBS, jobs, 1.0f, NULL), SAMO_OK);
        EXPECT(samo_wgrad_gather_batched(SAMO_WGRAD_MAX_JOBS + 1, jobs, 1.0f, NULL), SAMO_ERR_SIZE);
        EXPECT(samo_wgrad_gather_batched(-1, jobs, 1.0f, NULL), SAMO_ERR_SIZE);
        EXPECT(samo_wgrad_gather_batched(2, NULL, 1.0f, NULL), SAMO_ERR_NULL);
        EXPECT(samo_wgrad_gather_batched(2, jobs, 0.0f, NULL), SAMO_ERR_ARG);
        jobs[1].in = 12;                                                        /* one bad job rejects the call */
        EXPECT(samo_wgrad_gather_batched(2, jobs, 1.0f, NULL), SAMO_ERR_SIZE);
        EXPECT(samo_wgrad_gather_fp16_batched(2, jobs, 0, NULL), SAMO_ERR_SIZE);
        jobs[1].in = 16; jobs[1].nnz = 90;                                      /* kept entries but no output */
        EXPECT(samo_wgrad_gather_fp16_batched(2, jobs, 0, NULL), SAMO_ERR_NULL);
    }

    {
        samo_layer layers[2];
        memset(layers, 0, sizeof(layers));
        memset(&plan, 0, sizeof(plan));
        layers[0].n = 10; layers[0].nnz = 11;
        EXPECT(samo_plan_workspace_bytes(layers, 1, &bytes), SAMO_ERR_SIZE);
        EXPECT(samo_plan_init(layers, 1, fake, 1u << 20, NULL, &plan), SAMO_ERR_SIZE);
        layers[0].nnz = 5; layers[0].idx = fake;                      /* seg_ptr missing */
        EXPECT(samo_plan_init(layers, 1, fake, 1u << 20, NULL, &plan), SAMO_ERR_NULL);
        layers[0].seg_ptr = fake;                                     /* no parameters in either form */
        EXPECT(samo_plan_init(layers, 1, fake, 1u << 20, NULL, &plan), SAMO_ERR_NULL);
        layers[0].p = (float *)odd;
        EXPECT(samo_plan_init(layers, 1, fake, 1u << 20, NULL, &plan), SAMO_ERR_ALIGN);
        layers[0].p = (float *)fake;
        EXPECT(samo_plan_workspace_bytes(layers, 1, &bytes), SAMO_OK);
        if (bytes == 0 || bytes % 256 != 0) { printf("plan workspace size\n"); ++failures; }
        EXPECT(samo_plan_init(layers, 1, NULL, bytes, NULL, &plan), SAMO_ERR_WORKSPACE);
        EXPECT(samo_plan_init(layers, 1, fake, bytes - 1, NULL, &plan), SAMO_ERR_WORKSPACE);
        EXPECT(samo_plan_init(layers, 1, odd, bytes, NULL, &plan), SAMO_ERR_ALIGN);
        EXPECT(samo_plan_init(layers, -1, fake, bytes, NULL, &plan), SAMO_ERR_SIZE);
        EXPECT(samo_plan_init(layers, 1, fake, bytes, NULL, NULL), SAMO_ERR_NULL);
        EXPECT(samo_plan_workspace_bytes(layers, 1, NULL), SAMO_ERR_NULL);
        EXPECT(samo_plan_workspace_bytes(NULL, 1, &bytes), SAMO_ERR_NULL);
        EXPECT(samo_plan_workspace_bytes(NULL, 0, &bytes), SAMO_OK);
        if (plan.d_layers != NULL || plan.num_layers != 0) { printf("a rejected plan must stay untouched\n"); ++failures; }
        /* a plan that lacks what an entry needs: rejected before anything is enqueued */
        plan.num_layers = 1; plan.num_tiles = 1; plan.num_chunks = 1; plan.n_total = 10; plan.nnz_total = 5;
        plan.d_layers = plan.d_tiles = plan.d_chunks = fake; plan.buffers = 0;
        EXPECT(samo_fused_step_batched(&plan, 1.0f, &adam, NULL, NULL), SAMO_ERR_PLAN);
        EXPECT(samo_decompress_batched(&plan, NULL), SAMO_ERR_PLAN);
        plan.buffers = ~0u;
        EXPECT(samo_fused_step_batched(&plan, 0.0f, &adam, NULL, NULL), SAMO_ERR_ARG);
        EXPECT(samo_grad_stats_batched(&plan, 0, 1.0f, fake, NULL, 0, NULL), SAMO_ERR_WORKSPACE);
        EXPECT(samo_grad_stats_batched(&plan, 0, 1.0f, fake, fake, 64, NULL), SAMO_ERR_WORKSPACE);
        EXPECT(samo_grad_stats_batched(&plan, 7, 1.0f, fake, fake, 1u << 20, NULL), SAMO_ERR_ARG);
    }
    EXPECT(samo_index_workspace_bytes(1025, &bytes), SAMO_OK);
    if (bytes != 12) { printf("index workspace size\n"); ++failures; }
    EXPECT(samo_index_workspace_bytes(-1, &bytes), SAMO_ERR_SIZE);
    EXPECT(samo_index_workspace_bytes(10, NULL), SAMO_ERR_NULL);
    EXPECT(samo_debug_set(SAMO_KNOB_COUNT, 1), SAMO_ERR_ARG);
    EXPECT(samo_debug_set(-1, 1), SAMO_ERR_ARG);
    EXPECT(samo_debug_set(SAMO_KNOB_WGRAD_TILE, 128), SAMO_OK);
    EXPECT(samo_debug_set(SAMO_KNOB_WGRAD_TILE, SAMO_KNOB_DEFAULT), SAMO_OK);
    EXPECT(samo_plan_stats_workspace_bytes(NULL, &bytes), SAMO_ERR_NULL);
    EXPECT(samo_decompress_batched(NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_gather_batched(NULL, 1.0f, NULL, NULL, 0, NULL), SAMO_ERR_NULL);
    EXPECT(samo_gather_fp16_batched(NULL, 0, 1.0f, NULL, NULL, 0, NULL), SAMO_ERR_NULL);
    EXPECT(samo_grad_stats_batched(NULL, 0, 1.0f, NULL, NULL, 0, NULL), SAMO_ERR_NULL);
    EXPECT(samo_adam_batched(NULL, &adam, NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_step_batched(NULL, 1.0f, &adam, NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_adam_expand_batched(NULL, 1.0f, &adam, NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_sgd_step_batched(NULL, 1.0f, &sgd, NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_fused_step_fp32_batched(NULL, 1.0f, &adam, NULL, NULL), SAMO_ERR_NULL);
    EXPECT(samo_stream_copy(fake, fake, 15, NULL), SAMO_ERR_SIZE);
    EXPECT(samo_stream_copy(fake, NULL, 16, NULL), SAMO_ERR_NULL);

    printf(failures ? "FAILED %d\n" : "all rejected as documented\n", failures);
    return failures ? 1 : 0;
}
