/* Plain C99 translation unit against the public header: checks that cnr.h is valid C, that every
 * entry point links, and exercises the host-only calls.  Built and run by tests/test_library_host.py
 * (no GPU needed: cnr_create is expected to fail cleanly when there is none). */
#include <stdio.h>
#include <string.h>

#include "cnr.h"

int main(void) {
    /* take the address of every export so that the linker has to resolve it */
    typedef void (*fn)(void);
    const fn exports[] = {
        (fn)cnr_create, (fn)cnr_destroy, (fn)cnr_bitmap_words, (fn)cnr_packed_row_bytes, (fn)cnr_scratch_bytes,
        (fn)cnr_mark_scratch_bytes, (fn)cnr_greedy_iterations, (fn)cnr_clear_bitmap, (fn)cnr_mark_touched,
        (fn)cnr_compact_dirty, (fn)cnr_quantize_rows, (fn)cnr_pack, (fn)cnr_restore_rows, (fn)cnr_quant_error,
        (fn)cnr_poll_errors, (fn)cnr_status_str, (fn)cnr_last_hip_error, (fn)cnr_full_checkpoint_due,
        (fn)cnr_policy_init, (fn)cnr_policy_next, (fn)cnr_clear_bitmap_batch, (fn)cnr_mark_touched_batch,
        (fn)cnr_compact_dirty_batch, (fn)cnr_quantize_rows_batch, (fn)cnr_restore_rows_batch,
        (fn)cnr_host_writer_device_bytes, (fn)cnr_host_writer_create, (fn)cnr_host_writer_destroy,
        (fn)cnr_encode_to_host, (fn)cnr_host_writer_wait, (fn)cnr_select_scratch_bytes,
        (fn)cnr_select_greedy_params, (fn)cnr_select_bits, (fn)cnr_restore_from_host,
        (fn)cnr_compact_dirty_noalloc};
    size_t i, n_exports = sizeof(exports) / sizeof(exports[0]);
    for (i = 0; i < n_exports; ++i)
        if (!exports[i]) return 10;

    if (cnr_bitmap_words(33) != 2 || cnr_packed_row_bytes(64, 3) != 24 || cnr_packed_row_bytes(12, 3) != 0) return 11;
    if (cnr_greedy_iterations(25, 0.6f) != 15 || cnr_greedy_iterations(100, 1.0f) != 99) return 12;
    if (cnr_mark_scratch_bytes(1000) < 1000 || cnr_scratch_bytes(40000000u) < 4u * 2442u) return 13;
    {
        double s[2] = {0.5, 0.8};
        if (!cnr_full_checkpoint_due(s, 2) || cnr_full_checkpoint_due(s, 1)) return 14;
    }
    {
        cnr_policy p;
        cnr_policy_decision d;
        int k, first_full = 0;
        if (cnr_policy_init(&p, CNR_POLICY_INTERMITTENT) != CNR_OK) return 15;
        for (k = 0; k < 12 && !first_full; ++k) {
            d = cnr_policy_next(&p, 0.25 + 0.03 * k);
            if (d.take_full) first_full = k + 1;
        }
        if (first_full != 8) return 16;
        if (cnr_policy_init(&p, (cnr_policy_kind)7) != CNR_E_INVALID) return 17;
    }
    if (strcmp(cnr_status_str(CNR_OK), "ok") != 0) return 18;
    if (cnr_select_bits(1, 0) != 2 || cnr_select_bits(3, 3) != 3 || cnr_select_bits(20, 0) != 4 ||
        cnr_select_bits(21, 0) != 8 || cnr_select_bits(1, 2) != 8)
        return 19;
    if (cnr_select_scratch_bytes(100, 64, 4) != 400u + 400u + 3200u + 800u + 16u) return 27;
    if (cnr_host_writer_device_bytes(64, 4, 1024) != 2u * 1024u * 44u || cnr_host_writer_device_bytes(12, 3, 16) != 0) return 26;
    {
        cnr_ctx *ctx = NULL;
        cnr_status st = cnr_create(&ctx, 0);
        if (st == CNR_OK) {
            /* a GPU is present: argument checks must come back without touching it */
            if (cnr_quantize_rows(ctx, NULL, 10, 64, NULL, NULL, 10, 5, CNR_RANGE_MINMAX, NULL, NULL, NULL, NULL,
                                  NULL, NULL, NULL, NULL) != CNR_E_BITS) return 19;
            if (cnr_restore_rows(ctx, NULL, 10, 12, NULL, NULL, 10, 3, NULL, NULL, NULL, NULL) != CNR_E_DIM) return 20;
            {
                cnr_table_job job;
                memset(&job, 0, sizeof job);
                if (cnr_quantize_rows_batch(ctx, &job, 1, 64, 4, (cnr_range_mode)9, NULL, NULL) != CNR_E_INVALID) return 23;
                if (cnr_quantize_rows_batch(ctx, &job, 1, 64, 4, CNR_RANGE_MINMAX, NULL, NULL) != CNR_OK) return 24;
                job.n_rows = (uint64_t)1 << 32;
                if (cnr_mark_touched_batch(ctx, &job, 1, CNR_IDX_I64, NULL) != CNR_E_INVALID) return 25;
            }
            if (cnr_compact_dirty_noalloc(ctx, NULL, CNR_NOALLOC_MAX_ROWS + 1, NULL, 0, NULL, NULL) != CNR_E_TOO_LARGE)
                return 28;
            if (cnr_destroy(ctx) != CNR_OK) return 21;
        } else if (st != CNR_E_HIP || ctx != NULL) {
            return 22;
        }
    }
    printf("abi ok: %u exports\n", (unsigned)n_exports);
    return 0;
}
