// Shared host/device helpers of the library (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>

#include "nezha.h"

namespace nezha {

constexpr uint64_t kEmpty = 0xFFFFFFFFFFFFFFFFull;  // never a valid index: prod T_l <= 2^64-1
constexpr int kBucketSlots = 8;                     // 8 keys x 8 B = one 64-byte bucket

// ---- error text (thread local) -------------------------------------------------------
char* error_buffer();
int fail(int code, const char* fmt, ...);
#define NEZHA_HIP_CHECK(expr)                                                         \
  do {                                                                                \
    hipError_t _e = (expr);                                                           \
    if (_e != hipSuccess)                                                             \
      return ::nezha::fail(NEZHA_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e)); \
  } while (0)

// Positional multipliers of Eq. 4; false if prod T_l > 2^64-1 or a radix < 1.
bool radix_multipliers(int32_t L, const int32_t* radices, uint64_t* mult);

// ---- optional per-kernel timing with HIP events (off by default) ------------------------
enum KernelKind {
  kPackWeights = 0, kUserGemm, kExpand, kMerge, kVerifyProbe, kVerifyScan, kVerifyScatter,
  kInsert, kGather, kLevelFused, kExpandRequest, kKernelKinds
};
// Brackets the launches made while it is alive with two events on `stream` when timing is on.
struct ProfileScope {
  ProfileScope(KernelKind kind, hipStream_t stream);
  ~ProfileScope();
  int slot;
  hipStream_t stream;
};

struct SetView {  // what kernels need from an item set
  const uint64_t* slots;
  uint64_t n_buckets;
};

// ---- device helpers --------------------------------------------------------------------
// 64-bit finaliser; spreads every key bit over the whole word (hot first-level codes share
// the low digits of Eq. 4, so the bucket index must depend on all bits).
__device__ __forceinline__ uint64_t hash64(uint64_t k) {
  k ^= k >> 33;
  k *= 0xFF51AFD7ED558CCDull;
  k ^= k >> 33;
  k *= 0xC4CEB9FE1A85EC53ull;
  k ^= k >> 33;
  return k;
}
__device__ __forceinline__ uint64_t home_bucket(uint64_t key, uint64_t n_buckets) {
  return __umul64hi(hash64(key), n_buckets);  // range reduction without a modulo
}

// Membership of one key: scan the home bucket, then following buckets, until the key or an
// empty slot is seen.  The table is never full, so the scan ends; it is bounded anyway.
__device__ __forceinline__ bool set_contains(const SetView& s, uint64_t key) {
  uint64_t b = home_bucket(key, s.n_buckets);
  for (uint64_t step = 0; step < s.n_buckets; ++step) {
    const ulonglong2* p = reinterpret_cast<const ulonglong2*>(s.slots + b * kBucketSlots);
    ulonglong2 q0 = p[0], q1 = p[1], q2 = p[2], q3 = p[3];
    bool hit = (q0.x == key) | (q0.y == key) | (q1.x == key) | (q1.y == key) |
               (q2.x == key) | (q2.y == key) | (q3.x == key) | (q3.y == key);
    if (hit) return true;
    bool hole = (q0.x == kEmpty) | (q0.y == kEmpty) | (q1.x == kEmpty) | (q1.y == kEmpty) |
                (q2.x == kEmpty) | (q2.y == kEmpty) | (q3.x == kEmpty) | (q3.y == kEmpty);
    if (hole) return false;
    b = (b + 1 == s.n_buckets) ? 0 : b + 1;
  }
  return false;
}

}  // namespace nezha

struct nezha_itemset {
  uint64_t* slots;      // device, n_buckets * kBucketSlots keys, kEmpty = free
  uint64_t n_buckets;
  int64_t n_distinct;
  int32_t L;
  int32_t radices[NEZHA_MAX_LEVELS];
  uint64_t mult[NEZHA_MAX_LEVELS];
  int device;
  uint32_t magic;
};
constexpr uint32_t kSetMagic = 0x4E5A4853u;
