/*
 * A plain C client of the C ABI (include/dmi.h): no Python, no torch.  Reads a bf16
 * matrix from a file, puts it into device memory with the HIP runtime, captures three
 * selections of its rows through dmi_observe (raw with summaries, fp8, with a keep
 * vector) and, through dmi_observe_batch, the two halves of the matrix as two observation points in
 * one launch; drains, polls the pinned host ring and writes the records, in order, to a file.
 *
 *   c_client <in.bin> <rows> <elems> <out.bin>
 *
 * Selection used (the test that runs this builds the same one for the oracle):
 *   request i of 6: req_id 100+i, rows i*7 .. i*7+(i%3), step 1      (6 requests, 1-3 rows each)
 *   keep vector for the third observe: requests 1 and 4 are out.
 *   batch: rows 2, 5, 8 and the last row of each half, as fp16 with the mean.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "dmi.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_DMI(x) do { dmi_status_t s_ = (x); if (s_ < 0) { \
    fprintf(stderr, "%s: %d (%s)\n", #x, (int)s_, dmi_last_error()); return 3; } } while (0)

int main(int argc, char **argv)
{
    if (argc != 5) { fprintf(stderr, "usage: %s in.bin rows elems out.bin\n", argv[0]); return 1; }
    const long rows = atol(argv[2]), elems = atol(argv[3]);
    const size_t bytes = (size_t)rows * (size_t)elems * 2u;
    void *host = malloc(bytes);
    FILE *f = fopen(argv[1], "rb");
    if (!host || !f || fread(host, 1, bytes, f) != bytes) { fprintf(stderr, "cannot read %s\n", argv[1]); return 1; }
    fclose(f);

    void *dev = NULL;
    uint8_t *keep_dev = NULL;
    CHECK_HIP(hipSetDevice(0));
    CHECK_HIP(hipMalloc(&dev, bytes));
    CHECK_HIP(hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice));
    const uint8_t keep[6] = {1, 0, 1, 1, 0, 1};
    CHECK_HIP(hipMalloc((void **)&keep_dev, sizeof keep));
    CHECK_HIP(hipMemcpy(keep_dev, keep, sizeof keep, hipMemcpyHostToDevice));

    dmi_ring_config_t cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.device_ring_bytes = 1u << 20;
    cfg.host_ring_bytes = 1u << 20;
    cfg.device_id = 0;
    cfg.rank_tag = 7;
    dmi_ring_t *ring = NULL;
    CHECK_DMI(dmi_ring_create(&cfg, &ring));

    dmi_req_sel_t reqs[6];
    for (uint32_t i = 0; i < 6; i++) {
        reqs[i].req_id = 100u + i;
        reqs[i].row_base = i * 7u;
        reqs[i].tok_start = 0;
        reqs[i].tok_count = 1u + i % 3u;
        reqs[i].tok_step = 1;
    }
    dmi_tensor_t t;
    t.data = dev;
    t.dtype = DMI_DTYPE_BF16;
    t.shape[0] = rows; t.shape[1] = elems;
    t.stride[0] = elems; t.stride[1] = 1;
    dmi_selection_t sel = {6, reqs, NULL, NULL};
    dmi_transform_t raw_sum = {DMI_DTYPE_BF16, DMI_SUM_L2 | DMI_SUM_ABSMAX};
    dmi_transform_t fp8 = {DMI_DTYPE_FP8_E4M3FN, 0};
    CHECK_DMI(dmi_observe(ring, 1, &t, &sel, &raw_sum, 40, NULL));
    CHECK_DMI(dmi_observe(ring, 2, &t, &sel, &fp8, 40, NULL));
    sel.keep_mask_dev = keep_dev;
    CHECK_DMI(dmi_observe(ring, 3, &t, &sel, &raw_sum, 41, NULL));
    /* two observation points in one launch: the two halves of the tensor as two tensors of one
     * shape, one selection (rows 2, 5, 8 and the last row of each half), stored as fp16 */
    dmi_req_sel_t reqs2[2] = {{200, 2, 0, 3, 3}, {201, (uint32_t)(rows / 2 - 1), 0, 1, 1}};
    dmi_selection_t sel2 = {2, reqs2, NULL, NULL};
    dmi_tensor_t half = t;
    half.data = NULL;                   /* ignored: the addresses travel in data[] */
    half.shape[0] = rows / 2;
    const uint32_t points[2] = {4, 5};
    const void *data[2] = {dev, (const char *)dev + (size_t)(rows / 2) * elems * 2u};
    dmi_transform_t fp16 = {DMI_DTYPE_FP16, DMI_SUM_MEAN};
    uint32_t n_done = 0;
    CHECK_DMI(dmi_observe_batch(ring, 2, points, data, &half, &sel2, &fp16, 42, NULL, &n_done));
    if (n_done != 2) { fprintf(stderr, "batch stopped after %u of 2\n", n_done); return 5; }
    uint64_t moved = 0;
    CHECK_DMI(dmi_drain(ring, DMI_DRAIN_FLUSH, &moved));

    dmi_record_view_t views[8];
    uint32_t n = 0;
    CHECK_DMI(dmi_poll_host(ring, views, 8, &n));
    FILE *o = fopen(argv[4], "wb");
    if (!o) { fprintf(stderr, "cannot write %s\n", argv[4]); return 1; }
    for (uint32_t i = 0; i < n; i++) {
        fwrite(views[i].p0, 1, views[i].n0, o);
        if (views[i].n1) fwrite(views[i].p1, 1, views[i].n1, o);
    }
    fclose(o);
    if (n) CHECK_DMI(dmi_release_host(ring, views[n - 1].seq));
    dmi_stats_t st;
    CHECK_DMI(dmi_get_stats(ring, &st));
    printf("%u records, %llu bytes drained, %llu rows captured\n", n, (unsigned long long)moved,
           (unsigned long long)st.captured_rows);
    CHECK_DMI(dmi_ring_destroy(ring));
    CHECK_HIP(hipFree(keep_dev));
    CHECK_HIP(hipFree(dev));
    free(host);
    return n == 5 ? 0 : 4;
}
