// Host-only driver for a sanitizer-instrumented build of the library: walks the configuration
// checks, the scratch-layout arithmetic and the decode launch planner through ordinary, edge and
// hostile inputs.  No call here touches a GPU.  Any AddressSanitizer / UndefinedBehaviorSanitizer
// report aborts the program; otherwise it prints a summary and exits 0.
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "linear_kv.h"
#include "linear_kv_diag.h"

static linear_cfg_t base() {
  linear_cfg_t c = {};
  c.n_layers = 2; c.batch = 2; c.n_heads = 4; c.head_dim = 64; c.n_cond = 1; c.line_len = 24; c.n_lines = 24;
  c.budget = 96; c.n_init = 24; c.n_recent_lines = 1; c.dtype = LINEAR_BF16;
  return c;
}

#define CHECK(x) do { if (!(x)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__); std::exit(1); } } while (0)

int main() {
  long plans = 0, configs = 0, accepted = 0;
  // 1. planner sweep: every cache length of several shapes, every tuning
  struct Shape { int heads, d, cond, n, h, budget, init, dtype, batch; };
  const Shape shapes[] = {
      {20, 64, 1, 24, 24, 96, 24, LINEAR_BF16, 64},   {20, 64, 1, 24, 24, 576, 24, LINEAR_BF16, 64},
      {32, 128, 256, 49, 48, 294, 49, LINEAR_BF16, 8}, {32, 128, 256, 49, 48, 2352, 49, LINEAR_BF16, 8},
      {4, 64, 8, 8, 8, 24, 4, LINEAR_F32, 1},          {2, 128, 0, 1, 12, 4, 1, LINEAR_F32, 1},
      {3, 64, 5, 8, 211, 1672, 0, LINEAR_BF16, 1}};
  for (const Shape& sh : shapes) {
    linear_cfg_t c = base();
    c.n_heads = sh.heads; c.head_dim = sh.d; c.n_cond = sh.cond; c.line_len = sh.n; c.n_lines = sh.h;
    c.budget = sh.budget; c.n_init = sh.init; c.dtype = sh.dtype; c.batch = sh.batch;
    for (int mode = 0; mode <= 3; ++mode) {
      c.score_mode = mode;
      size_t cache = 0, scratch = 0;
      CHECK(linear_workspace_bytes(&c, &cache, &scratch) == LINEAR_OK);
      CHECK(cache == (size_t)sh.batch * sh.heads * (sh.cond + sh.budget) * sh.d * (sh.dtype == LINEAR_BF16 ? 2 : 4));
      CHECK(scratch % 256 == 0);
      for (int gpw : {0, 1, 5, 16})
        for (int ns : {0, 1, 3, 64})
          for (int keys = 0; keys < sh.cond + sh.budget; keys += (keys < 300 ? 1 : 7)) {
            int32_t p[6];
            const int rc = linear_plan_shape(&c, keys, gpw, ns, p);
            CHECK(rc == LINEAR_OK);
            CHECK(p[0] >= 1 && p[0] <= 64 && (long)p[0] * p[1] >= keys && p[2] >= 1 && p[2] <= 16 && p[4] >= 0 && p[4] < p[2]);
            ++plans;
          }
      int32_t p[6];
      CHECK(linear_plan_shape(&c, sh.cond + sh.budget, 0, 0, p) == LINEAR_EINVAL);
      CHECK(linear_plan_shape(&c, -1, 0, 0, p) == LINEAR_EINVAL);
      CHECK(linear_plan_shape(&c, 0, 17, 0, p) == LINEAR_EINVAL);
    }
  }
  // 2. hostile configurations: every field at extreme values, alone and together
  const int extremes[] = {INT_MIN, INT_MIN + 1, -1, 0, 1, 2, 7, 63, 64, 65, 127, 128, 1 << 10, 1 << 20, (1 << 20) + 1,
                          1 << 24, 1 << 30, INT_MAX - 1, INT_MAX};
  for (int field = 0; field < 14; ++field)
    for (int v : extremes)
      for (int w : {INT_MAX, 1, 3}) {
        linear_cfg_t c = base();
        int32_t* f = &c.n_layers;          // the first thirteen members are int32_t, in declaration order
        if (field < 13) f[field] = v; else c.out_dtype = v;
        if (field != 9) c.n_recent_lines = w == 3 ? c.n_recent_lines : w;
        if (field == 7 && w == 1) c.budget = c.line_len * c.n_lines;     // full cache with the extreme elsewhere
        size_t cache = 0, scratch = 0;
        const int rc = linear_workspace_bytes(&c, &cache, &scratch);
        CHECK(rc == LINEAR_OK || rc == LINEAR_EINVAL);
        accepted += rc == LINEAR_OK;
        ++configs;
      }
  for (int a : extremes)
    for (int b : extremes) {
      linear_cfg_t c = base();
      c.line_len = a; c.n_lines = b; c.budget = a;                       // products and sums of extremes
      size_t cache = 0, scratch = 0;
      int rc = linear_workspace_bytes(&c, &cache, &scratch);
      CHECK(rc == LINEAR_OK || rc == LINEAR_EINVAL);
      c = base(); c.n_init = a; c.n_recent_lines = b;
      rc = linear_workspace_bytes(&c, &cache, &scratch);
      CHECK(rc == LINEAR_OK || rc == LINEAR_EINVAL);
      c = base(); c.batch = a; c.n_heads = b;
      rc = linear_workspace_bytes(&c, &cache, &scratch);
      CHECK(rc == LINEAR_OK || rc == LINEAR_EINVAL);
      c = base(); c.n_cond = a; c.budget = b; c.n_lines = INT_MAX;
      rc = linear_workspace_bytes(&c, &cache, &scratch);
      CHECK(rc == LINEAR_OK || rc == LINEAR_EINVAL);
      c = base(); c.budget = c.line_len * c.n_lines; c.n_recent_lines = a; c.n_init = b;   // full cache: r, N_init unused
      rc = linear_workspace_bytes(&c, &cache, &scratch);
      CHECK(rc == LINEAR_OK || rc == LINEAR_EINVAL);
      configs += 5;
    }
  // 3. argument checks of the calls that would launch (none gets as far as a device call)
  void* two[2] = {(void*)256, (void*)512};
  linear_kv_t* h = nullptr;
  linear_cfg_t c = base();
  CHECK(kv_init(&c, two, two, (void*)4096, nullptr, nullptr, nullptr, &h) == LINEAR_ENULL);
  CHECK(kv_init(nullptr, two, two, (void*)4096, nullptr, nullptr, nullptr, &h) == LINEAR_ENULL);
  for (int a : extremes)
    for (int b : extremes) {
      // q is not 16-byte aligned: whatever survives the value checks stops at the alignment check
      const int rc = decode_step_static(LINEAR_BF16, 128, a, b, b == INT_MAX ? b : b + 1, (void*)256, (void*)256,
                                        (void*)264, (void*)256, (void*)256, 0.f, 0, (void*)256, nullptr);
      CHECK(rc == LINEAR_EINVAL || rc == LINEAR_EALIGN);
    }
  for (int pairs : {1 << 12, 1 << 20, 1 << 24})
    for (int keys : {4096, 30000, (1 << 20) - 1}) {
      // valid arguments whose 64-way split partials cannot fit the library's own scratch array
      const int rc = decode_step_static(LINEAR_F32, 128, pairs, keys, keys + 1, (void*)256, (void*)256, (void*)256,
                                        (void*)256, (void*)256, 0.f, 64, (void*)256, nullptr);
      CHECK(rc == LINEAR_ECAPACITY || rc == LINEAR_EINVAL);
    }
  CHECK(decode_step_layers(nullptr, 0, 1, nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr) == LINEAR_ENULL);
  CHECK(end_of_line_evict_layers(nullptr, 0, 1, nullptr) == LINEAR_ENULL);
  CHECK(kv_free(nullptr) == LINEAR_OK);
  std::printf("sanitize_driver ok: %ld plans, %ld configurations (%ld accepted)\n", plans, configs, accepted);
  return 0;
}
