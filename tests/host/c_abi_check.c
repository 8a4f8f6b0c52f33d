/* The boundary is a C ABI: this file is compiled as C99 against include/caramel.h, linked with
 * the shared library and exercises the host-only entry points (no GPU call). */
#include <stdio.h>
#include <string.h>

#include "caramel.h"

#define CHECK(c)                                                     \
  do {                                                               \
    if (!(c)) {                                                      \
      printf("FAIL line %d: %s (%s)\n", __LINE__, #c, caramel_last_error()); \
      return 1;                                                      \
    }                                                                \
  } while (0)

int main(void) {
  /* the MLP configuration: 6 tensors in update order, W = 4, threshold 64 KiB */
  const uint64_t elems[6] = {10, 2560, 256, 65536, 256, 200704};
  caramel_config cfg;
  caramel_plan* plan = NULL;
  uint32_t n_units = 0, n_entries = 0;
  uint64_t fused = 0, seg[5], thr = 0;
  caramel_unit units[3];
  caramel_entry entries[6];
  unsigned char image[1024];
  size_t len = 0;
  double a = 0, b = 0;

  memset(&cfg, 0, sizeof cfg);
  cfg.world = 4;
  cfg.dtype = CARAMEL_F32;
  cfg.batch_threshold_bytes = 65536;
  cfg.split_mode = CARAMEL_SPLIT_NONE;
  cfg.max_depth = 8;
  cfg.align_bytes = 16;
  cfg.num_streams = 2;
  cfg.pattern = CARAMEL_PATTERN_RING;

  CHECK(caramel_version() >= 100);
  CHECK(caramel_plan_create(&cfg, elems, 6, &plan) == CARAMEL_OK && plan != NULL);
  CHECK(caramel_plan_counts(plan, &n_units, &n_entries, &fused) == CARAMEL_OK);
  CHECK(n_units == 3 && n_entries == 6 && fused == 3084);
  CHECK(caramel_plan_units(plan, units, 3) == CARAMEL_OK);
  CHECK(units[0].kind == CARAMEL_KIND_CHUNK && units[0].elems == 65536 && units[0].stream == 0);
  CHECK(units[1].kind == CARAMEL_KIND_CHUNK && units[1].elems == 200704 && units[1].stream == 1);
  CHECK(units[2].kind == CARAMEL_KIND_BATCH && units[2].elems == 3084 && units[2].n_entries == 4);
  CHECK(caramel_plan_entries(plan, entries, 6) == CARAMEL_OK);
  CHECK(entries[3].tensor == 1 && entries[3].unit_off == 12 && entries[5].unit_off == 2828);
  CHECK(caramel_plan_entries(plan, entries, 5) == CARAMEL_EINVAL);
  CHECK(caramel_plan_segments(plan, 2, seg) == CARAMEL_OK);
  CHECK(seg[0] == 0 && seg[1] == 772 && seg[2] == 1544 && seg[3] == 2316 && seg[4] == 3084);
  CHECK(caramel_plan_serialize(plan, NULL, &len) == CARAMEL_OK && len > 0 && len <= sizeof image);
  CHECK(caramel_plan_serialize(plan, image, &len) == CARAMEL_OK && memcmp(image, "CARAMEL1", 8) == 0);
  /* device calls on an unbound plan are refused before anything touches a GPU */
  CHECK(caramel_allreduce(plan, NULL) == CARAMEL_ESTATE);
  CHECK(strlen(caramel_last_error()) > 0);
  caramel_plan_destroy(plan);
  caramel_plan_destroy(NULL);

  cfg.world = 0;
  CHECK(caramel_plan_create(&cfg, elems, 6, &plan) == CARAMEL_EINVAL && plan == NULL);

  CHECK(caramel_net_model_fit(64, 40.0 + 32.0, 4096, 40.0 + 2048.0, &a, &b) == CARAMEL_OK);
  CHECK(a > 39.999 && a < 40.001 && b > 0.4999 && b < 0.5001);
  CHECK(caramel_threshold_estimate(40.0, 0.5, &thr) == CARAMEL_OK && thr == 121);
  {
    /* section 4.3: one group fits behind its update time, the other must wait for the forward pass */
    const uint64_t bytes[2] = {8, 4};
    const double ready[2] = {6.0, 7.0}, need[2] = {5.0, 4.0};
    caramel_slot slots[2];
    caramel_schedule_summary sum;
    CHECK(caramel_schedule_transfers(bytes, ready, need, 2, 10.0, 5.0, 0.0, 0.5, slots, &sum) == CARAMEL_OK);
    CHECK(slots[0].bin == CARAMEL_BIN_BACKWARD && slots[0].start == 6.0 && slots[0].end == 10.0);
    CHECK(slots[1].bin == CARAMEL_BIN_FORWARD && slots[1].start == 2.0 && slots[1].end == 4.0);
    CHECK(sum.iteration_time == 15.0 && sum.utilization == 1.0);
    CHECK(caramel_schedule_transfers(bytes, ready, need, 2, 5.0, 5.0, 0.0, 0.5, slots, &sum) == CARAMEL_EINVAL);
  }
  printf("c_abi_check ok\n");
  return 0;
}
