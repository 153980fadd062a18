// Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the library's HOST code
// (csrc/itemset.hip and csrc/draft.hip compiled for the host only): every entry point of
// include/nezha.h is called on the paths that must end before anything reaches a GPU -- argument
// errors, workspace queries, the registry of live sets, the allocation-failure hook -- with fake
// (never dereferenced) device pointers.  No device code is compiled into this program (the symbols
// that would hold it stay unresolved at link time), and nothing here launches a kernel.
// Exit status 0 = clean.  Built and run by tests/test_sanitizers.py.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "nezha.h"

#define REQUIRE(cond)                                                   \
  do {                                                                  \
    if (!(cond)) {                                                      \
      fprintf(stderr, "%s:%d: %s failed (last error: %s)\n", __FILE__, __LINE__, #cond, \
              nezha_last_error());                                      \
      return 1;                                                         \
    }                                                                   \
  } while (0)

static void* fake(uintptr_t a) { return reinterpret_cast<void*>(a); }

static int step(const nezha_step_desc& d, const void* H, const void* key_out, const void* state_out,
                const void* ws, size_t ws_bytes, const nezha_itemset* set = nullptr) {
  return nezha_draft_step(&d, H, fake(0x2000), fake(0x3000), fake(0x4000),
                          (const uint64_t*)fake(0x5000), (const float*)fake(0x6000), set,
                          (uint64_t*)key_out, (float*)fake(0x8000), (int32_t*)fake(0x9000),
                          (int32_t*)fake(0xA000), const_cast<void*>(state_out),
                          (int32_t*)fake(0xC000), const_cast<void*>(ws), ws_bytes, nullptr);
}

int main() {
  REQUIRE(nezha_last_error() != nullptr);
  const int32_t rad3[3] = {256, 256, 256};
  int32_t codes[6] = {0, 1, 2, 3, 4, 5};
  nezha_itemset* set = fake(0x1) ? (nezha_itemset*)fake(0x1234) : nullptr;

  // ---- nezha_build_itemset: argument errors, then the allocation hook ------------------------
  REQUIRE(nezha_build_itemset(codes, 2, 3, rad3, 0, 0.5, nullptr, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_build_itemset(codes, -1, 3, rad3, 0, 0.5, nullptr, &set) == NEZHA_EINVAL && !set);
  REQUIRE(nezha_build_itemset(nullptr, 2, 3, rad3, 0, 0.5, nullptr, &set) == NEZHA_EINVAL);
  REQUIRE(nezha_build_itemset(codes, 2, 3, nullptr, 0, 0.5, nullptr, &set) == NEZHA_EINVAL);
  REQUIRE(nezha_build_itemset(codes, 2, 0, rad3, 0, 0.5, nullptr, &set) == NEZHA_EINVAL);
  REQUIRE(nezha_build_itemset(codes, 2, 9, rad3, 0, 0.5, nullptr, &set) == NEZHA_EINVAL);
  REQUIRE(nezha_build_itemset(codes, 2, 3, rad3, 0, 0.0, nullptr, &set) == NEZHA_EINVAL);
  REQUIRE(nezha_build_itemset(codes, 2, 3, rad3, 0, 0.91, nullptr, &set) == NEZHA_EINVAL);
  {
    const int32_t big[3] = {1 << 30, 1 << 30, 1 << 30}, zero[3] = {4, 0, 4};
    REQUIRE(nezha_build_itemset(codes, 2, 3, big, 0, 0.5, nullptr, &set) == NEZHA_ERANGE);
    REQUIRE(nezha_build_itemset(codes, 2, 3, zero, 0, 0.5, nullptr, &set) == NEZHA_ERANGE);
  }
  for (const char* nth : {"1", "2"}) {
    setenv("NEZHA_TEST_FAIL_ALLOC", nth, 1);
    set = (nezha_itemset*)fake(0x1234);
    REQUIRE(nezha_build_itemset(codes, 2, 3, rad3, 0, 0.5, nullptr, &set) == NEZHA_ENOMEM);
    REQUIRE(set == nullptr);
  }
  unsetenv("NEZHA_TEST_FAIL_ALLOC");

  // ---- a pointer that is not a live set is refused without being read ------------------------
  nezha_itemset* bogus = (nezha_itemset*)fake(0x1000);
  int64_t n64 = 0;
  REQUIRE(nezha_free_itemset(nullptr) == NEZHA_OK);
  REQUIRE(nezha_free_itemset(bogus) == NEZHA_EINVAL);
  REQUIRE(nezha_itemset_info(bogus, &n64, nullptr, nullptr, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_itemset_info(nullptr, &n64, nullptr, nullptr, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_verify_tuples(bogus, (const int32_t*)fake(0x2000), 8, (uint8_t*)fake(0x3000), nullptr,
                              nullptr, fake(0x4000), 1 << 20, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_verify_tuples_static(bogus, (const int32_t*)fake(0x2000), 8, (uint8_t*)fake(0x3000),
                                     nullptr, nullptr, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_check_itemset(bogus, (const int32_t*)fake(0x2000), 8, 1, nullptr, &n64) == NEZHA_EINVAL);

  // ---- workspace queries -------------------------------------------------------------------------
  REQUIRE(nezha_verify_workspace(-1) == 0 && nezha_verify_workspace(0) > 0);
  REQUIRE(nezha_verify_workspace(4000000) >= 3907 * 12);
  nezha_step_desc d;
  memset(&d, 0, sizeof(d));
  d.B = 4; d.L = 3; d.level = 2; d.K = 4; d.K_in = 4; d.d = 64; d.e = 64;
  d.radices = rad3; d.dtype = NEZHA_F32; d.h_row_stride = 64;
  const size_t need = nezha_draft_step_workspace(&d);
  REQUIRE(need > 0 && nezha_draft_levels_workspace(&d) >= need);
  REQUIRE(nezha_draft_step_workspace(nullptr) == 0);
  REQUIRE(nezha_packed_weights_bytes(&d) == 0);           // float32 weights are not packed

  // ---- nezha_draft_step: everything it refuses ---------------------------------------------------
  const void* H = fake(0x1000);
  const void* ws = fake(0x10000);
  auto bad = [&](nezha_step_desc v, int want) {
    const int rc = step(v, H, fake(0x7000), fake(0xB000), ws, (size_t)1 << 24);
    if (rc != want) fprintf(stderr, "got %d, wanted %d: %s\n", rc, want, nezha_last_error());
    return rc == want && (want == NEZHA_OK || nezha_last_error()[0] != 0);
  };
  { auto v = d; v.level = 0; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.level = 4; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.K = 0; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.K = 257; REQUIRE(bad(v, NEZHA_EINVAL)); }                 // K > T_level
  { auto v = d; v.K_in = 0; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.K = 1025; v.K_in = 1025; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.e = 6; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.e = 512; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.h_row_stride = 32; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.radices = nullptr; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.dtype = NEZHA_BF16; v.d = 48; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.transition = 2; REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.transition = NEZHA_TRANSITION_RNN; REQUIRE(bad(v, NEZHA_EINVAL)); }   // no matrix
  { auto v = d; v.transition = NEZHA_TRANSITION_RNN; v.U_l = fake(0x1008); REQUIRE(bad(v, NEZHA_EINVAL)); }
  { auto v = d; v.user_part = (const float*)fake(0x1004); REQUIRE(bad(v, NEZHA_EINVAL)); }
  {
    const int32_t big[3] = {1 << 30, 1 << 30, 1 << 30};
    auto v = d; v.radices = big; REQUIRE(bad(v, NEZHA_ERANGE));
  }
  REQUIRE(step(d, nullptr, fake(0x7000), fake(0xB000), ws, 1 << 24) == NEZHA_EINVAL);
  REQUIRE(step(d, H, nullptr, fake(0xB000), ws, 1 << 24) == NEZHA_EINVAL);
  REQUIRE(step(d, H, fake(0x7000), nullptr, ws, 1 << 24) == NEZHA_EINVAL);   // state_out below L
  REQUIRE(step(d, H, fake(0x7000), fake(0xB000), nullptr, 1 << 24) == NEZHA_EINVAL);
  REQUIRE(step(d, H, fake(0x7000), fake(0xB000), ws, 16) == NEZHA_EINVAL);
  REQUIRE(step(d, H, fake(0x7000), fake(0xB000), fake(0x10010), 1 << 24) == NEZHA_EINVAL);
  REQUIRE(step(d, fake(0x1002), fake(0x7000), fake(0xB000), ws, 1 << 24) == NEZHA_EINVAL);
  REQUIRE(step(d, H, fake(0x7000), fake(0xB008), ws, 1 << 24) == NEZHA_EINVAL);
  REQUIRE(step(d, H, fake(0x7000), fake(0xB000), ws, 1 << 24, bogus) == NEZHA_EINVAL);
  { auto v = d; v.B = 0; REQUIRE(bad(v, NEZHA_OK)); }                          // an empty batch
  REQUIRE(nezha_draft_step(nullptr, H, H, H, H, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                           nullptr, nullptr, nullptr, nullptr, 0, nullptr) == NEZHA_EINVAL);

  // ---- nezha_draft_levels / nezha_decode: all levels are checked before anything is enqueued ----
  nezha_step_desc p = d;
  p.dtype = NEZHA_BF16; p.w_packed = 1; p.K = 40; p.radices = rad3;
  const int32_t rad_big[3] = {2048, 2048, 2048};
  p.radices = rad_big;
  nezha_level_io io[3];
  memset(io, 0, sizeof(io));
  for (int l = 0; l < 3; ++l) {
    const uintptr_t base = 0x100000 * (l + 1);
    io[l].H_l = fake(base); io[l].W_l = fake(base); io[l].E_l = fake(base);
    io[l].key_out = (uint64_t*)fake(base); io[l].score_out = (float*)fake(base);
    io[l].parent_out = (int32_t*)fake(base); io[l].code_out = (int32_t*)fake(base);
    io[l].state_out = l < 2 ? fake(base) : nullptr; io[l].count_out = (int32_t*)fake(base);
  }
  REQUIRE(nezha_draft_levels(nullptr, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_draft_levels(&p, nullptr, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);
  io[2].key_out = nullptr;                         // only the last level is wrong
  REQUIRE(nezha_draft_levels(&p, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);
  REQUIRE(strstr(nezha_last_error(), "output pointer") != nullptr);
  io[2].key_out = (uint64_t*)fake(0x300000);
  p.state_init = fake(0x1008);
  REQUIRE(nezha_draft_levels(&p, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);
  p.state_init = nullptr;
  io[1].set = bogus;
  REQUIRE(nezha_draft_levels(&p, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);
  io[1].set = nullptr;
  REQUIRE(nezha_draft_levels(&p, io, fake(0x10000000), 1024, nullptr) == NEZHA_EINVAL);   // workspace
  { auto v = p; v.L = 9; REQUIRE(nezha_draft_levels(&v, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL); }
  REQUIRE(nezha_decode(&p, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);   // no user_part buffers
  REQUIRE(strstr(nezha_last_error(), "user_part") != nullptr);
  for (int l = 0; l < 3; ++l) io[l].user_part = (const float*)fake(0x400000 * (l + 1));
  io[2].code_out = nullptr;                        // caught before the projections are enqueued
  REQUIRE(nezha_decode(&p, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL);
  { auto v = p; v.w_packed = 0; REQUIRE(nezha_decode(&v, io, fake(0x10000000), (size_t)1 << 40, nullptr) == NEZHA_EINVAL); }
  REQUIRE(nezha_decode(nullptr, io, nullptr, 0, nullptr) == NEZHA_EINVAL);

  // ---- projections and weight packing ------------------------------------------------------------
  {
    const void* Hs[3] = {fake(0x1000), fake(0x2000), fake(0x3000)};
    float* As[3] = {(float*)fake(0x4000), (float*)fake(0x5000), (float*)fake(0x6000)};
    REQUIRE(nezha_user_projection_levels(&p, 0, Hs, Hs, As, nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_user_projection_levels(&p, 4, Hs, Hs, As, nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_user_projection_levels(&p, 3, nullptr, Hs, As, nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_user_projection_levels(&d, 3, Hs, Hs, As, nullptr) == NEZHA_EINVAL);     // float32
    REQUIRE(nezha_user_projection_levels(nullptr, 3, Hs, Hs, As, nullptr) == NEZHA_EINVAL);
    const void* Hm[3] = {fake(0x1000), fake(0x2004), fake(0x3000)};
    REQUIRE(nezha_user_projection_levels(&p, 3, Hm, Hs, As, nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_user_projection(&d, nullptr, fake(0x2000), As[0], fake(0x10000), 1 << 24, nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_user_projection(&d, Hs[0], fake(0x2000), (float*)fake(0x4004), fake(0x10000), 1 << 24, nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_pack_weights(&d, Hs[0], fake(0x8000), nullptr) == NEZHA_EINVAL);         // float32
    REQUIRE(nezha_pack_weights(&p, nullptr, fake(0x8000), nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_pack_weights(&p, Hs[0], fake(0x8004), nullptr) == NEZHA_EINVAL);
    REQUIRE(nezha_packed_weights_bytes(&p) >= (size_t)(64 + 64) * 2048 * 2);
  }

  // ---- measurement aids, host helpers ------------------------------------------------------------
  REQUIRE(nezha_profile_kinds() > 0);
  REQUIRE(nezha_profile_enable(0) == NEZHA_OK && nezha_profile_reset() == NEZHA_OK);
  const char* name = nullptr;
  double ms = -1;
  REQUIRE(nezha_profile_read(0, &name, &n64, &ms) == NEZHA_OK && name && n64 == 0 && ms == 0.0);
  REQUIRE(nezha_profile_read(-1, &name, &n64, &ms) == NEZHA_EINVAL);
  REQUIRE(nezha_profile_read(nezha_profile_kinds(), &name, &n64, &ms) == NEZHA_EINVAL);
  REQUIRE(nezha_profile_event_overhead(0, nullptr, &ms) == NEZHA_EINVAL);
  REQUIRE(nezha_profile_event_overhead(10, nullptr, nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_random_gather(nullptr, 1024, 4, 64, 1, fake(0x1000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_random_gather(fake(0x1000), 1024, 4, 32, 1, fake(0x1000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_random_gather(fake(0x1040), 1024, 4, 64, 1, fake(0x1000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_mfma_rate(nullptr, 4096, 10, 4, (uint64_t*)fake(0x1000), (float*)fake(0x2000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_mfma_rate(fake(0x1008), 4096, 10, 4, (uint64_t*)fake(0x1000), (float*)fake(0x2000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_mfma_rate(fake(0x1000), 4096, 0, 4, (uint64_t*)fake(0x1000), (float*)fake(0x2000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_tile_step(3, 10, 4, (const float*)fake(0x1000), (uint64_t*)fake(0x1000), (float*)fake(0x2000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_tile_step(2, 0, 4, (const float*)fake(0x1000), (uint64_t*)fake(0x1000), (float*)fake(0x2000), nullptr) == NEZHA_EINVAL);
  REQUIRE(nezha_bench_tile_step(2, 10, 4, nullptr, (uint64_t*)fake(0x1000), (float*)fake(0x2000), nullptr) == NEZHA_EINVAL);
  {
    const uint64_t keys[2] = {852723ull, 104ull};
    const int32_t r512[3] = {512, 512, 512}, r357[3] = {3, 5, 7};
    int32_t out[3];
    REQUIRE(nezha_unpack_keys(keys, 1, 3, r512, out) == NEZHA_OK && out[0] == 243 && out[1] == 129 && out[2] == 3);
    REQUIRE(nezha_unpack_keys(keys + 1, 1, 3, r357, out) == NEZHA_OK && out[0] == 2 && out[1] == 4 && out[2] == 6);
    REQUIRE(nezha_unpack_keys(keys, 1, 0, r512, out) == NEZHA_EINVAL);
    REQUIRE(nezha_unpack_keys(nullptr, 1, 3, r512, out) == NEZHA_EINVAL);
    REQUIRE(nezha_unpack_keys(keys, 0, 3, r512, nullptr) == NEZHA_OK);
  }
  puts("abi: clean");
  return 0;
}
