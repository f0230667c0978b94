// Test infrastructure: drives the library's host-side logic (plan building, weight table, workspace layout, step
// accounting, argument checks) with no GPU, in a build whose host code is compiled with -fsanitize=address,undefined
// (tests/test_sanitizers.py).  Nothing here launches a kernel.
#include <stdio.h>
#include <string.h>

#include "wmdec.h"
#include "wmdec_measure.h"

static int fails = 0;
#define CHECK(cond) do { if (!(cond)) { printf("host_sanitize_check: failed: %s (line %d): %s\n", #cond, __LINE__, wmdec_last_error()); ++fails; } } while (0)

static void exercise(const wmdec_decoder_config& cfg) {
  wmdec_decoder* dec = nullptr;
  CHECK(decoder_create(&cfg, &dec) == WMDEC_OK && dec);
  if (!dec) return;
  const size_t wb = decoder_weights_bytes(dec);
  CHECK(wb > 0 && decoder_packed_bytes(dec) > 0);
  const int nw = decoder_num_weights(dec);
  size_t end = 0;
  for (int i = 0; i < nw; ++i) {
    const char* name = nullptr; size_t off = 0, bytes = 0; int dtype = -1, shape[4] = {0, 0, 0, 0};
    CHECK(decoder_weight_info(dec, i, &name, &off, &bytes, &dtype, shape) == WMDEC_OK && name && bytes > 0);
    size_t off2 = 0, bytes2 = 0;
    CHECK(decoder_weight_offset(dec, name, &off2, &bytes2) == WMDEC_OK && off2 == off && bytes2 == bytes);
    CHECK(off % 256 == 0 && off >= end);
    end = off + bytes;
  }
  CHECK(end <= wb);
  size_t o = 0, b = 0;
  CHECK(decoder_weight_offset(dec, "no.such.weight", &o, &b) != WMDEC_OK);
  CHECK(decoder_weight_info(dec, nw, nullptr, nullptr, nullptr, nullptr, nullptr) != WMDEC_OK);
  size_t prev = 0;
  for (int batch = 1; batch <= cfg.max_batch; ++batch) {
    const size_t ws = decoder_workspace_bytes(dec, batch);
    CHECK(ws > prev);
    prev = ws;
  }
  CHECK(decoder_workspace_bytes(dec, cfg.max_batch + 1) == 0);
  const int steps = decoder_num_steps(dec);
  double flops = 0.0;
  for (int i = 0; i < steps; ++i) {
    const char* kernel = nullptr; double f = 0, by = 0;
    CHECK(decoder_step_info(dec, i, &kernel, &f, &by) == WMDEC_OK && kernel && strlen(kernel) > 0 && f >= 0 && by >= 0);
    flops += f;
  }
  CHECK(steps >= 1 && steps <= decoder_num_launches(dec));   // a step is one or two launches
  CHECK(flops > 0 && flops <= decoder_flops_per_frame(dec) * (1 + 1e-12) && flops >= decoder_flops_per_frame(dec) * (1 - 1e-12));
  CHECK(decoder_dense_flops_per_frame(dec) >= decoder_flops_per_frame(dec));
  // argument checks that return before anything is enqueued
  CHECK(decoder_run(dec, nullptr, nullptr, nullptr, 1, nullptr) != WMDEC_OK);
  CHECK(decoder_set_workspace(dec, nullptr, 0) != WMDEC_OK);
  float ms = 0.f;
  CHECK(decoder_step_times(dec, &ms, 1) != WMDEC_OK);
  CHECK(decoder_destroy(dec) == WMDEC_OK);
}

int main() {
  wmdec_decoder_config cfg;
  decoder_default_config(&cfg);
  exercise(cfg);
  for (int variant = 0; variant < 3; ++variant) {
    wmdec_decoder_config c = cfg;
    if (variant == 0) c.separate_stats_pass = 1;
    if (variant == 1) c.separate_merge_launch = 1;
    if (variant == 2) c.separate_shortcut = 1;
    exercise(c);
  }
  {   // a narrow decoder on an odd latent, both 16-bit types
    wmdec_decoder_config c = cfg;
    c.latent_h = 7; c.latent_w = 9; c.level_channels[1] = 128; c.level_channels[2] = 64; c.level_channels[3] = 32;
    c.resblocks_per_level = 2; c.max_batch = 3;
    exercise(c);
    c.act_dtype = WMDEC_BF16;
    exercise(c);
  }
  {   // rejected configurations
    wmdec_decoder* dec = nullptr;
    wmdec_decoder_config c = cfg;
    c.groups = 7;
    CHECK(decoder_create(&c, &dec) != WMDEC_OK && dec == nullptr);
    c = cfg; c.max_batch = 0;
    CHECK(decoder_create(&c, &dec) != WMDEC_OK);
    CHECK(decoder_create(nullptr, &dec) != WMDEC_OK);
  }
  // size helpers and argument errors of the per-operator entries
  CHECK(wmdec_gn_stats_workspace_bytes(1, 480, 720, 128, 32) > 0);
  CHECK(wmdec_conv_packed_bytes(512, 512, 3, WMDEC_F16) == (size_t)9 * 512 * 512 * 2);
  CHECK(wmdec_upconv_packed_bytes(256, 256, WMDEC_F16) > wmdec_conv_packed_bytes(256, 256, 3, WMDEC_F16));
  CHECK(wmdec_attention_workspace_bytes(1, 60, 90, 512) > 0);
  CHECK(wmdec_conv_stats_workspace_bytes(WMDEC_F16, WMDEC_F16, 1, 60, 90, 512, 512, 32) > 0);
  CHECK(wmdec_adaln_max_batch(1920) >= 1);
  CHECK(wmdec_gn_stats(nullptr, WMDEC_F16, 1, 8, 8, 32, 32, 1e-6f, nullptr, nullptr, nullptr, 0, nullptr) != WMDEC_OK);
  CHECK(wmdec_upsample2x_nearest(nullptr, nullptr, WMDEC_F16, 1, 4, 4, 8, nullptr) != WMDEC_OK);
  CHECK(wmdec_latent_extrapolate(nullptr, nullptr, WMDEC_BF16, 0.5f, 1, nullptr, WMDEC_BF16, 16, nullptr) != WMDEC_OK);
  CHECK(strlen(wmdec_status_string(WMDEC_ERR_SHAPE)) > 0);
  if (fails) { printf("host_sanitize_check: %d checks failed\n", fails); return 1; }
  printf("host_sanitize_check: ok\n");
  return 0;
}
