// Drives the host layer of the C ABI (csrc/api.hip built for the CPU with stub launchers, see stub_kernels.cpp) under
// AddressSanitizer + UndefinedBehaviorSanitizer: parameter validation, workspace arithmetic at small, benchmark and
// extreme sizes, the chunked-prefill layouts, the closed forms, the profiling record store and the error strings.
// Pointers handed to the launch paths are fake but non-NULL and aligned; the stubs never dereference them.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <initializer_list>

#include "rattn.h"

namespace rattn { extern int g_stub_launches; }

static int failures = 0;
#define CHECK(cond)                                                                  \
  do {                                                                               \
    if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

// a path that reaches the (stub) launchers ends in hipGetLastError(): RATTN_OK on a GPU box, RATTN_ERR_HIP ("no device")
// on a CPU-only box; both mean that validation and layout arithmetic went through
static bool launched(rattn_status st) { return st == RATTN_OK || st == RATTN_ERR_HIP; }

static rattn_params params(int B, int T, int Hq, int Hkv, int D, int W, int dtype) {
  rattn_params p;
  memset(&p, 0, sizeof(p));
  p.B = B; p.T = T; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.window = W; p.dtype = dtype;
  p.softmax_scale = 0.088f; p.rms_eps = 1e-6f;
  return p;
}

int main() {
  void* fake = (void*)(uintptr_t)0x7f0000001000ull;  // aligned, never dereferenced
  size_t f = 0, b = 0, s = 0;
  // ---- validation
  rattn_params p = params(2, 300, 4, 2, 64, 32, RATTN_F32);
  CHECK(rattn_workspace_bytes(&p, &f, &b, &s) == RATTN_OK && f > 0 && b > f && s > 0);
  CHECK(rattn_workspace_bytes(NULL, &f, &b, &s) == RATTN_ERR_INVALID_ARG);
  CHECK(rattn_workspace_bytes(&p, NULL, NULL, NULL) == RATTN_OK);
  struct { int field, value; rattn_status want; } bad[] = {
      {0, 0, RATTN_ERR_INVALID_ARG}, {1, 0, RATTN_ERR_INVALID_ARG}, {2, 3, RATTN_ERR_INVALID_ARG},
      {4, 96, RATTN_ERR_UNSUPPORTED}, {5, 0, RATTN_ERR_INVALID_ARG}, {6, -1, RATTN_ERR_INVALID_ARG},
      {7, 7, RATTN_ERR_UNSUPPORTED}, {11, 3, RATTN_ERR_UNSUPPORTED}, {12, 2, RATTN_ERR_UNSUPPORTED},
      {13, 3, RATTN_ERR_UNSUPPORTED}, {13, -1, RATTN_ERR_UNSUPPORTED},
      {0, 70000, RATTN_ERR_UNSUPPORTED}, {1, 2000000000, RATTN_ERR_UNSUPPORTED}};
  for (auto& c : bad) {
    rattn_params q = p;
    ((int32_t*)&q)[c.field >= 8 ? c.field + 0 : c.field] = c.value;   // fields 8, 9 are the two floats
    CHECK(rattn_workspace_bytes(&q, &f, &b, &s) == c.want);
    CHECK(strlen(rattn_last_error()) > 0);
  }
  { rattn_params q = p; q.rms_eps = 0.f; CHECK(rattn_workspace_bytes(&q, &f, &b, &s) == RATTN_ERR_INVALID_ARG); }
  { rattn_params q = p; q.softmax_scale = 0.f; CHECK(rattn_workspace_bytes(&q, &f, &b, &s) == RATTN_ERR_INVALID_ARG); }
  // ---- sizes: benchmark shapes, ragged, extreme
  int shapes[][7] = {{4, 4096, 24, 8, 128, 512, 1}, {2, 8192, 32, 8, 128, 512, 1}, {4, 8192, 24, 8, 128, 8192, 1},
                     {1, 32768, 2, 1, 128, 512, 1}, {3, 1100, 6, 2, 128, 513, 1}, {1, 1, 1, 1, 64, 1, 0},
                     {65535, 8000, 1, 1, 128, 9, 1}, {1, 300, 65535, 65535, 64, 1000000, 0}, {2, 127, 8, 1, 128, 64, 1}};
  for (auto& sh : shapes) {
    rattn_params q = params(sh[0], sh[1], sh[2], sh[3], sh[4], sh[5], sh[6]);
    for (int variant = 0; variant < 8; ++variant) {
      const int policies[4] = {RATTN_STATES_KEEP, RATTN_STATES_REBUILD, RATTN_STATES_KEEP_EVERY_2ND, RATTN_STATES_KEEP_EVERY_4TH};
      q.kernel_path = variant & 1;
      q.state_policy = policies[variant >> 1];
      q.chunk = variant == 2 ? 64 : 0;
      rattn_status st = rattn_workspace_bytes(&q, &f, &b, &s);
      CHECK(st == RATTN_OK || st == RATTN_ERR_UNSUPPORTED);
      if (st != RATTN_OK) continue;
      // launch paths with the stubs: too-small workspace is refused, the right size goes through
      q.save_for_bwd = 1;
      if (f > 0) CHECK(rattn_fwd(&q, fake, fake, fake, NULL, NULL, fake, fake, fake, f - 1, NULL) == RATTN_ERR_WORKSPACE);
      int before = rattn::g_stub_launches;
      CHECK(launched(rattn_fwd(&q, fake, fake, fake, NULL, NULL, fake, fake, fake, f, NULL)));
      CHECK(rattn::g_stub_launches > before);
      CHECK(rattn_bwd(&q, fake, fake, fake, NULL, NULL, fake, fake, fake, fake, fake, NULL, NULL, fake, b - 1, NULL) ==
            RATTN_ERR_WORKSPACE);
      CHECK(launched(rattn_bwd(&q, fake, fake, fake, NULL, NULL, fake, fake, fake, fake, fake, NULL, NULL, fake, b, NULL)));
      CHECK(rattn_fwd(&q, fake, fake, fake, NULL, NULL, fake, NULL, fake, f, NULL) == RATTN_ERR_INVALID_ARG);  // save, no buffer
      CHECK(rattn_fwd(&q, (char*)fake + 2, fake, fake, NULL, NULL, fake, fake, fake, f, NULL) == RATTN_ERR_INVALID_ARG);
      size_t e = 0, c = 0;
      CHECK(rattn_prefill_export_workspace_bytes(&q, &e) == RATTN_OK);
      CHECK(launched(rattn_prefill_export(&q, fake, fake, fake, fake, (float*)fake, fake, e, NULL)));
      for (int pos0 : {0, 1, 64, 128, 511, 512, 513, 4096, 100000}) {
        rattn_status sc = rattn_prefill_chunk_workspace_bytes(&q, pos0, &c);
        CHECK(sc == RATTN_OK || sc == RATTN_ERR_UNSUPPORTED);
        if (sc == RATTN_OK) {
          CHECK(launched(rattn_prefill_chunk(&q, pos0, fake, fake, fake, NULL, NULL, fake, fake, (float*)fake, fake, fake, c, NULL)));
          CHECK(rattn_prefill_chunk(&q, pos0, fake, fake, fake, NULL, NULL, fake, fake, (float*)fake, fake, fake, c - 1, NULL) == RATTN_ERR_WORKSPACE);
        }
      }
      CHECK(rattn_prefill_chunk_workspace_bytes(&q, -1, &c) == RATTN_ERR_INVALID_ARG);
      CHECK(rattn_prefill_chunk_workspace_bytes(&q, 2147483647, &c) != RATTN_OK);
    }
  }
  // the allocation-free entry refuses what does not fit its buffer before touching any device
  { rattn_params q = params(4, 8192, 24, 8, 128, 512, 1);
    CHECK(rattn_fwd_static(&q, fake, fake, fake, NULL, NULL, fake, NULL, NULL) == RATTN_ERR_WORKSPACE); }
  // ---- decode validation
  rattn_decode_params d;
  memset(&d, 0, sizeof(d));
  d.N = 4; d.Hq = 4; d.Hkv = 2; d.D = 64; d.window = 16; d.dtype = RATTN_BF16; d.softmax_scale = 1.f; d.rms_eps = 1e-6f;
  CHECK(rattn_decode_step(&d, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == RATTN_ERR_INVALID_ARG);
  CHECK(launched(rattn_decode_step(&d, fake, fake, fake, (const int32_t*)fake, fake, fake, (float*)fake, NULL, NULL, fake, NULL)));
  d.D = 80; CHECK(rattn_decode_step(&d, fake, fake, fake, (const int32_t*)fake, fake, fake, (float*)fake, NULL, NULL, fake, NULL) == RATTN_ERR_UNSUPPORTED);
  d.D = 64; d.N = 70000; CHECK(rattn_decode_step(&d, fake, fake, fake, (const int32_t*)fake, fake, fake, (float*)fake, NULL, NULL, fake, NULL) == RATTN_ERR_UNSUPPORTED);
  CHECK(rattn_decode_step(NULL, fake, fake, fake, (const int32_t*)fake, fake, fake, (float*)fake, NULL, NULL, fake, NULL) == RATTN_ERR_INVALID_ARG);
  // ---- closed forms
  double out = 0;
  CHECK(rattn_cache_bytes(40, 4, 4096, 1024, 0, 8, 128, 2, &out) == RATTN_OK && out == (10.0 * 4096 + 30.0 * 1024) * 2 * 8 * 128 * 2);
  CHECK(rattn_cache_bytes(40, 4, 4096, 1024, 0, 8, 128, 2, NULL) == RATTN_ERR_INVALID_ARG);
  CHECK(rattn_cache_bytes(-1, 4, 4096, 1024, 0, 8, 128, 2, &out) == RATTN_ERR_INVALID_ARG);
  CHECK(rattn_step_time_model(128, 1e9, 3e9, 6e9, 8e12, 2.5e15, &out) == RATTN_OK && out > 0);
  CHECK(rattn_step_time_model(128, 1e9, 3e9, 6e9, 0, 2.5e15, &out) == RATTN_ERR_INVALID_ARG);
  double fl = 0;
  CHECK(rattn_probe_mfma(NULL, 10, 10, &fl, NULL) == RATTN_ERR_INVALID_ARG);
  CHECK(launched(rattn_probe_mfma(fake, 10, 10, &fl, NULL)) && fl > 0);
  CHECK(rattn_probe_mfma(fake, 0, 10, &fl, NULL) == RATTN_ERR_INVALID_ARG);
  // ---- strings and the profiling store (without a device no event pair can be created: the store stays empty)
  for (int st = -5; st <= 1; ++st) CHECK(strlen(rattn_status_string((rattn_status)st)) > 0);
  CHECK(strlen(rattn_version()) > 0);
  rattn_profile_enable(1);
  p = params(1, 256, 2, 1, 128, 64, RATTN_BF16);
  CHECK(rattn_workspace_bytes(&p, &f, &b, &s) == RATTN_OK);
  CHECK(launched(rattn_fwd(&p, fake, fake, fake, NULL, NULL, fake, NULL, fake, f, NULL)));
  const char* name = NULL; float ms = 0;
  CHECK(rattn_profile_get(rattn_profile_count(), &name, &ms) == RATTN_ERR_INVALID_ARG);
  CHECK(rattn_profile_get(-1, &name, &ms) == RATTN_ERR_INVALID_ARG);
  rattn_profile_reset();
  CHECK(rattn_profile_count() == 0);
  rattn_profile_enable(0);
  if (failures == 0) printf("ALL OK (%d stub launches)\n", rattn::g_stub_launches);
  return failures == 0 ? 0 : 1;
}
