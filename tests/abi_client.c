/* A client of the library written in C99: shows that the header is plain C and that the calls that
 * need no GPU (host-only handle) behave the same from C as through the Python binding.
 * Prints "key value" lines that the test compares with the binding's answers. */
#include <stdio.h>
#include <string.h>

#include "dadam.h"

/* pair timings of a memory whose thirds begin at arena offsets 40 and 136 GiB */
static double model_rate(uint64_t a, uint64_t b, void* ctx) {
  const uint64_t gib = 1024ull * 1024ull * 1024ull;
  const int ta = a < 40 * gib ? 0 : a < 136 * gib ? 1 : 2, tb = b < 40 * gib ? 0 : b < 136 * gib ? 1 : 2;
  (void)ctx;
  return ta != tb ? 0.79 : 0.66;
}

int main(void) {
  dadam_tensor_desc tensors[3];
  dadam_stretch stretches[DADAM_MAX_STRETCHES];
  uint32_t n_stretches = 0u, every = 0u;
  uint64_t sizes[8], regions[4], placed[8];
  int32_t order[4];
  uint64_t numel[3] = {1000, 24, 5001};
  uint64_t offsets[3];
  uint64_t d = 0;
  dadam_config cfg;
  dadam_handle* h = NULL;
  dadam_plan_info info;
  /* ring of 4, weights 1/3 */
  int32_t row_ptr[5] = {0, 3, 6, 9, 12};
  int32_t col[12] = {3, 0, 1, 0, 1, 2, 1, 2, 3, 2, 3, 0};
  float w[12];
  uint32_t warn = 77u;
  int rc, i;

  rc = dadam_pack_offsets(numel, 3u, 8u, offsets, &d);
  printf("pack_rc %d\n", rc);
  printf("d %llu\n", (unsigned long long)d);
  for (i = 0; i < 3; ++i) {
    tensors[i].offset_elems = offsets[i];
    tensors[i].numel = numel[i];
    tensors[i].weight_decay = 0.0f;
    tensors[i].flags = 0u;
    printf("offset%d %llu\n", i, (unsigned long long)offsets[i]);
  }
  memset(&cfg, 0, sizeof cfg);
  cfg.abi_version = DADAM_ABI_VERSION;
  cfg.n_rows = 4u;
  cfg.n_cols = 4u;
  cfg.d = d;
  cfg.n_tensors = 3u;
  cfg.tensors = tensors;
  cfg.param_dtype = DADAM_F32;
  cfg.grad_dtype = DADAM_F32;
  cfg.lr = 1e-3f;
  cfg.beta1 = 0.9f;
  cfg.beta2 = 0.999f;
  cfg.eps = 1e-8f;
  cfg.accum_s = 2u;
  cfg.beta_vhat = -1.0f;
  cfg.device = DADAM_DEVICE_NONE;
  rc = dadam_init(&cfg, &h);
  printf("init_rc %d\n", rc);
  if (rc != DADAM_OK || h == NULL) return 1;

  for (i = 0; i < 12; ++i) w[i] = 1.0f / 3.0f;
  rc = dadam_set_topology(h, 0u, row_ptr, col, w, &warn);
  printf("topology_rc %d\n", rc);
  printf("warn %u\n", warn);

  col[1] = 9; /* out of range */
  rc = dadam_set_topology(h, 1u, row_ptr, col, w, &warn);
  printf("bad_topology_rc %d\n", rc);
  printf("bad_topology_has_message %d\n", dadam_last_error(h) != NULL && dadam_last_error(h)[0] != '\0');

  rc = dadam_get_plan_info(h, &info);
  printf("plan_rc %d\n", rc);
  printf("n_segments %u\n", info.n_segments);
  printf("tile_elems %u\n", info.tile_elems);
  printf("n_tiles_tile %llu\n", (unsigned long long)info.n_tiles_tile);
  printf("n_tiles_direct %llu\n", (unsigned long long)info.n_tiles_direct);
  printf("lds_bytes_tile %u\n", info.lds_bytes_tile);

  rc = dadam_get_row_order(h, 0u, order);
  printf("row_order_rc %d\n", rc);
  printf("row_order %d%d%d%d\n", (int)order[0], (int)order[1], (int)order[2], (int)order[3]);

  /* placement bookkeeping with a model in place of the device's timings */
  rc = dadam_find_stretches(200ull << 30, model_rate, NULL, stretches, &n_stretches);
  printf("stretches_rc %d\n", rc);
  printf("n_stretches %u\n", n_stretches);
  for (i = 0; i < 8; ++i) sizes[i] = 3ull << 30;
  rc = dadam_regions_from_stretches(stretches, n_stretches, sizes, 8u, regions, &every);
  printf("regions_found %d\n", rc);
  printf("every %u\n", every);
  rc = dadam_deal_offsets(sizes, 8u, regions[0], regions[1], regions[2], regions[3], every, placed);
  printf("deal_rc %d\n", rc);
  printf("first_in_region0 %d\n", placed[0] >= regions[0] && placed[0] + sizes[0] <= regions[1]);
  printf("second_in_region1 %d\n", placed[1] >= regions[2] && placed[1] + sizes[1] <= regions[3]);

  /* a host-only handle cannot launch: an error code, not a crash */
  rc = dadam_mix(h, 0u, 0u, NULL);
  printf("mix_on_host_only_handle_rc %d\n", rc);
  rc = dadam_set_lr(h, 5e-4f);
  printf("set_lr_rc %d\n", rc);
  dadam_destroy(h);
  dadam_destroy(NULL);
  printf("done 1\n");
  return 0;
}
