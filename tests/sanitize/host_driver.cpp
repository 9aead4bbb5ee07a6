// Drives the host-only paths of the C ABI: every call here must return before anything is enqueued
// (bad arguments, unbound workspace), so it runs without a GPU.  Built with -fsanitize=address,undefined.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "treekv.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: CHECK failed: %s\n", __FILE__, __LINE__, #cond); exit(1); } } while (0)

static treekv_config base() {
  treekv_config c;
  memset(&c, 0, sizeof(c));
  c.budget = 64; c.q_heads = 4; c.kv_heads = 4; c.head_dim = 128; c.batch = 1; c.dtype = TREEKV_BF16;
  return c;
}

int main() {
  treekv_ctx* h = nullptr;
  // configurations that must be refused
  { treekv_config c = base(); c.budget = 0; CHECK(treekv_init_ex(&h, &c) == TREEKV_EINVAL); }
  { treekv_config c = base(); c.q_heads = 6; CHECK(treekv_init_ex(&h, &c) == TREEKV_EINVAL); }
  { treekv_config c = base(); c.n_sink = 40; c.n_recent = 24; CHECK(treekv_init_ex(&h, &c) == TREEKV_EINVAL); }
  { treekv_config c = base(); c.flags = 2; CHECK(treekv_init_ex(&h, &c) == TREEKV_EINVAL); }
  { treekv_config c = base(); c.softmax_scale = NAN; CHECK(treekv_init_ex(&h, &c) == TREEKV_EINVAL); }
  { treekv_config c = base(); c.head_dim = 96; CHECK(treekv_init_ex(&h, &c) == TREEKV_EUNSUPPORTED); }
  { treekv_config c = base(); c.n_sink = TREEKV_DEFAULT_LAYOUT; c.n_recent = 2; CHECK(treekv_init_ex(&h, &c) == TREEKV_EINVAL); }
  CHECK(treekv_init_ex(nullptr, nullptr) == TREEKV_EINVAL);
  CHECK(treekv_init(&h, 8, 4, 128) == TREEKV_EINVAL);
  CHECK(h == nullptr);

  // a sweep of valid shapes: the workspace and snapshot layouts are computed without overflow or misalignment
  const int budgets[] = {1, 2, 17, 64, 1024, 2048, 4096}, dims[] = {64, 128}, groups[] = {1, 2, 4, 8};
  for (int b : budgets) for (int d : dims) for (int g : groups) for (int dt = 0; dt < 2; ++dt) for (int rr = 0; rr < 2; ++rr) {
    treekv_config c = base();
    c.budget = b; c.head_dim = d; c.kv_heads = 3; c.q_heads = 3 * g; c.batch = 5; c.dtype = dt;
    c.n_sink = b >= 8 ? 2 : 0; c.n_recent = b >= 8 ? b / 3 : 0;
    c.max_prompt = rr ? 4096 : 0; c.flags = rr ? TREEKV_POSITION_RERANK : 0;
    CHECK(treekv_init_ex(&h, &c) == TREEKV_OK);
    treekv_config e;
    CHECK(treekv_get_config(h, &e) == TREEKV_OK && e.max_chunk == 512 && e.kv_splits >= 1 && e.softmax_scale > 0);
    const size_t ws = treekv_workspace_bytes(h);
    const size_t rows = (size_t)2 * 15 * (b + 1) * d * (dt == TREEKV_BF16 ? 2 : 4);
    CHECK(ws > rows && ws % 256 == 0);
    treekv_state_layout l;
    CHECK(treekv_get_state_layout(h, &l) == TREEKV_OK && l.bytes == treekv_state_bytes(h));
    CHECK(l.header == 0 && l.positions % 256 == 0 && l.slots > l.positions && l.S > l.slots && l.K > l.S && l.V > l.K && l.bytes > l.V);
    // nothing bound: every call that needs the workspace refuses; bad pointers are refused first
    char fake[64];
    CHECK(treekv_reset(h, nullptr) == TREEKV_ENOWS);
    CHECK(treekv_decode_step(h, nullptr, fake, fake, fake, (int32_t*)fake, nullptr, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_decode_step(h, (void*)0x1000, (void*)0x1000, (void*)0x1000, (void*)0x1000, (int32_t*)0x1000, nullptr, nullptr, nullptr) == TREEKV_ENOWS);
    CHECK(treekv_decode_step(h, (void*)0x1004, (void*)0x1000, (void*)0x1000, (void*)0x1000, (int32_t*)0x1000, nullptr, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_prefill_chunk(h, (void*)0x1000, (void*)0x1000, (void*)0x1000, 513, (void*)0x1000, (int32_t*)0x1000, nullptr, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_prefill_chunk(h, (void*)0x1000, (void*)0x1000, (void*)0x1000, 0, (void*)0x1000, (int32_t*)0x1000, nullptr, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_prefill_prompt(h, (void*)0x1000, (void*)0x1000, (void*)0x1000, 100000, 64, (int32_t*)0x1000, nullptr, nullptr, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_scores(h, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_scores(h, (float*)0x1000, nullptr) == TREEKV_ENOWS);
    CHECK(treekv_gather_kv(h, (void*)0x1000, (void*)0x1000, nullptr) == TREEKV_ENOWS);
    CHECK(treekv_export_state(h, (void*)0x1000, l.bytes, nullptr) == TREEKV_ENOWS);
    CHECK(treekv_export_state(h, (void*)0x1000, l.bytes - 1, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_import_state(h, (void*)0x1010, l.bytes, nullptr, nullptr) == TREEKV_EINVAL);
    CHECK(treekv_bind_workspace(h, (void*)0x1001, ws) == TREEKV_ENOWS);
    CHECK(treekv_bind_workspace(h, (void*)0x1000, ws - 1) == TREEKV_ENOWS);
    CHECK(treekv_bind_workspace(h, nullptr, ws) == TREEKV_EINVAL);
    CHECK(strlen(treekv_last_hip_error(h)) == 0);
    treekv_destroy(h);
    h = nullptr;
  }
  CHECK(treekv_wavelet_components(nullptr, nullptr, 0, 1, 32, 128, 5, nullptr, nullptr, nullptr) == TREEKV_EINVAL);
  CHECK(treekv_wavelet_components((float*)0x1000, (void*)0x1000, 0, 1, 33, 128, 5, (float*)0x1000, nullptr, nullptr) == TREEKV_EINVAL);
  CHECK(treekv_wavelet_components((float*)0x1000, (void*)0x1000, 0, 1, 64, 96, 5, (float*)0x1000, nullptr, nullptr) == TREEKV_EUNSUPPORTED);
  for (int s = 1; s >= -6; --s) CHECK(strlen(treekv_strerror(s)) > 0);
  CHECK(treekv_workspace_bytes(nullptr) == 0 && treekv_state_bytes(nullptr) == 0);
  treekv_destroy(nullptr);
  puts("host paths clean");
  return 0;
}
