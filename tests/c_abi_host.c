/* A C99 translation unit that uses the library through include/rec.h alone: compiled with
 * `gcc -std=c99 -pedantic -Wall -Werror` and linked against librec.so by tests/test_abi_exports.py.
 * Calls only entry points (or error paths) that return before anything touches a device. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "rec.h"

#define CHECK(c)                                                      \
    do {                                                              \
        if (!(c)) {                                                   \
            printf("FAILED line %d: %s\n", __LINE__, #c);             \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main(void) {
    int64_t start[8], count[8];
    double arrival[4] = {0.0, 1.0, 2.0, 10.0}, service[4] = {2.0, 2.0, 2.0, 1.0}, lat[4];
    double qps[5] = {0.0, 0.0, 3.0, 5.0, 4.0}, table[5] = {0.0, 1.0, 1.5, 2.0, 2.5};
    int32_t widths[4] = {884, 512, 128, 1}, top[3] = {87, 64, 1}, bottom[2] = {13, 32};
    int64_t rows[1] = {10};
    rec_model_desc d;
    rec_model* m = NULL;
    rec_stream_pool* pool = NULL;

    CHECK(strcmp(rec_status_string(REC_OK), "REC_OK") == 0);
    CHECK(strcmp(rec_status_string(REC_ERR_WORKSPACE), "REC_ERR_WORKSPACE") == 0);

    CHECK(rec_split_query(70, 32, start, count) == 3);
    CHECK(start[2] == 64 && count[2] == 6 && count[0] == 32);
    CHECK(rec_split_query(-1, 4, NULL, NULL) == -1);

    CHECK(rec_sls_workspace_bytes(40, 1024) >= (size_t)(40 * 1024 + 1) * 8);
    CHECK(rec_mlp_workspace_bytes(widths, 3, 1024, REC_F32) >= (size_t)2 * 1024 * 512 * 4);
    CHECK(rec_mlp_workspace_bytes(NULL, 3, 1024, REC_F32) == 0);

    /* argument errors are reported before anything is launched */
    CHECK(rec_sls_forward(NULL, NULL, 0, 64, NULL, 0, NULL, 4, NULL, 0, 0, NULL, 0, NULL) == REC_ERR_BAD_SHAPE);
    CHECK(rec_sls_forward(NULL, NULL, 1, 64, NULL, 0, NULL, 0, NULL, 0, 0, NULL, 0, NULL) == REC_ERR_NULL);
    CHECK(rec_sls_forward_static((const float* const*)rows, rows, 1, 64, NULL, 0, (const int32_t*)rows, REC_SLS_STATIC_MAX_BAGS,
                                 NULL, 0, 0, NULL) == REC_ERR_WORKSPACE);
    CHECK(rec_sls_offsets(NULL, -1, NULL, NULL) == REC_ERR_BAD_SHAPE);
    CHECK(rec_mlp_forward(NULL, NULL, NULL, 1, REC_F32, REC_ACT_RELU, REC_ACT_RELU, NULL, 1, NULL, 1, 1, NULL, 0, NULL) == REC_ERR_NULL);
    CHECK(rec_interact(NULL, 0, 9, 32, NULL, 68, NULL) == REC_OK);
    CHECK(rec_f32_to_bf16(NULL, NULL, -1, NULL) == REC_ERR_BAD_SHAPE);
    CHECK(rec_model_create(NULL, &m) == REC_ERR_NULL && m == NULL);
    CHECK(rec_model_forward(NULL, NULL, NULL, 0, NULL, 0, NULL, NULL, 0, NULL) == REC_ERR_NULL);
    CHECK(rec_model_workspace_bytes(NULL, 16) == 0);
    rec_model_destroy(NULL);

    /* padded-weights size query: host only, from widths and dtype (87 columns -> 88) */
    memset(&d, 0, sizeof d);
    d.T = 10;
    d.D = 32;
    d.n_bottom = 1;
    d.bottom_widths = bottom;
    d.n_top = 2;
    d.top_widths = top;
    d.mlp_dtype = REC_F32;
    d.interaction = REC_INTERACT_DOT;
    CHECK(rec_model_padded_weight_bytes(&d) == 64 * 88 * 4);
    d.mlp_dtype = REC_BF16;
    CHECK(rec_model_padded_weight_bytes(&d) == 64 * 88 * 2);
    top[0] = 88;
    CHECK(rec_model_padded_weight_bytes(&d) == 0);
    CHECK(rec_model_padded_weight_bytes(NULL) == 0);

    /* serving model */
    CHECK(rec_sched_query_service(7, 4, table) == 2.5 + 2.0);
    CHECK(rec_sched_fifo_latencies(arrival, service, 4, lat) == REC_OK);
    CHECK(lat[0] == 2.0 && lat[1] == 3.0 && lat[2] == 4.0 && lat[3] == 1.0);
    CHECK(rec_sched_percentile(lat, 4, 0.5) == 2.0);
    CHECK(isnan(rec_sched_percentile(lat, 0, 0.5)));
    CHECK(rec_sched_hill_climb(qps, 5) == 3);
    CHECK(rec_sched_max_qps(arrival, service, 4, 0.95, 0.5, 10) == 0.0);

    CHECK(rec_stream_pool_create(0, &pool) == REC_ERR_BAD_SHAPE && pool == NULL);
    CHECK(rec_stream_pool_size(NULL) == 0);
    printf("c abi ok\n");
    return 0;
}
