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

// Whether `set` is a handle nezha_build_itemset returned and nezha_free_itemset has not taken yet
// (answered from a registry, without reading the handle's memory).
bool set_is_live(const nezha_itemset* set);

// Positional multipliers of Eq. 4; false if prod T_l > 2^64-1 or a radix < 1.
bool radix_multipliers(int32_t L, const int32_t* radices, uint64_t* mult);

// ---- optional per-kernel timing with HIP events (off by default) ------------------------
enum KernelKind {
  kPackWeights = 0, kUserGemm, kExpand, kMerge, kVerifyProbe, kVerifyScan, kVerifyScatter,
  kInsert, kGather, kLevelFused, kExpandRequest, kDecodeFused, kWideLogits, kWideRows, kWideSelect,
  kKernelKinds
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
  // optional prefilter (NULL: none): 64-byte blocks of 512 bits.  The block of a key is chosen by
  // its prefix (all digits but the last) and the upper bits of its last digit, the bit inside the
  // block is the last digit modulo 512: a bitmap of the last codes present, shared by the
  // prefixes that hash to the block.  The candidates of one beam differ in the last digit only,
  // so their filter reads fall on the same few lines.  A clear bit: the key is not in the set.
  const uint64_t* filter;
  uint64_t n_blocks;
  uint64_t mult_last;   // positional multiplier of the set's last digit (Eq. 4)
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

// Prefilter: word index of (prefix, last code); the bit inside the word is code & 63.
__device__ __forceinline__ uint64_t filter_word(uint64_t prefix, uint32_t code, uint64_t n_blocks) {
  const uint64_t block = __umul64hi(hash64(prefix * 8 + (code >> 9)), n_blocks);
  return block * 8 + ((code >> 6) & 7);
}

// A pointer known to address global memory, typed so: loads and stores through it are global
// instructions even where the compiler cannot trace the pointer back to a kernel argument
// (a generic access is a flat instruction, which also counts as an LDS access at every barrier).
template <typename T>
using global_ptr = __attribute__((address_space(1))) T*;
template <typename T>
__device__ __forceinline__ global_ptr<T> as_global(T* p) {
  return (global_ptr<T>)p;
}
// 16-byte global loads / stores (the HIP vector classes cannot be read through such a pointer)
typedef uint32_t nezha_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long nezha_u64x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_global_u4(const void* p) {
  const nezha_u32x4 v = *(global_ptr<const nezha_u32x4>)p;
  return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ void store_global_u4(void* p, uint4 v) {
  *(global_ptr<nezha_u32x4>)p = nezha_u32x4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ ulonglong2 load_global_u64x2(const void* p) {
  const nezha_u64x2 v = *(global_ptr<const nezha_u64x2>)p;
  return ulonglong2{v.x, v.y};
}

// Membership of one key in the table: scan the home bucket, then following buckets, until the
// key or an empty slot is seen.  The table is never full, so the scan ends; it is bounded anyway.
__device__ __forceinline__ bool set_probe(const SetView& s, uint64_t key) {
  uint64_t b = home_bucket(key, s.n_buckets);
  for (uint64_t step = 0; step < s.n_buckets; ++step) {
    const uint64_t* p = s.slots + b * kBucketSlots;
    const ulonglong2 q0 = load_global_u64x2(p), q1 = load_global_u64x2(p + 2),
                     q2 = load_global_u64x2(p + 4), q3 = load_global_u64x2(p + 6);
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

// The same for the key prefix + code * mult_last, through the prefilter where the view has one.
__device__ __forceinline__ bool set_contains(const SetView& s, uint64_t prefix, uint32_t code) {
  if (s.filter) {
    const uint64_t w = *(global_ptr<const uint64_t>)(s.filter + filter_word(prefix, code, s.n_blocks));
    if (((w >> (code & 63)) & 1ull) == 0ull) return false;
  }
  return set_probe(s, prefix + (uint64_t)code * s.mult_last);
}

// Membership of N keys (prefix[i] + code[i] * mult_last) with all N lookups in flight at once
// (the probes of one lane are independent random lines; one at a time leaves the memory system
// idle).  live[i] == false: key i is not looked up and in[i] is false.
template <int N>
__device__ __forceinline__ void set_contains_many(const SetView& s, const uint64_t (&prefix)[N],
                                                  const uint32_t (&code)[N], const bool (&live)[N],
                                                  bool (&in)[N]) {
  bool go[N];                                          // still to be looked up in the table
  uint64_t key[N];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    go[i] = live[i];
    key[i] = prefix[i] + (uint64_t)code[i] * s.mult_last;
  }
  if (s.filter) {
    uint64_t w[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
      w[i] = ~0ull;
      if (live[i])
        w[i] = *(global_ptr<const uint64_t>)(s.filter + filter_word(prefix[i], code[i], s.n_blocks));
    }
#pragma unroll
    for (int i = 0; i < N; ++i) go[i] = live[i] && ((w[i] >> (code[i] & 63)) & 1ull);
  }
  ulonglong2 q[N][4];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const uint64_t* p = s.slots + (go[i] ? home_bucket(key[i], s.n_buckets) : 0) * kBucketSlots;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      q[i][c] = ulonglong2{kEmpty, kEmpty};
      if (go[i]) q[i][c] = load_global_u64x2(p + 2 * c);
    }
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
    bool hit = false, hole = false;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      hit |= (q[i][c].x == key[i]) | (q[i][c].y == key[i]);
      hole |= (q[i][c].x == kEmpty) | (q[i][c].y == kEmpty);
    }
    in[i] = go[i] && hit;
    // a full home bucket without the key (rare at the load factors in use): the general scan
    if (go[i] && !hit && !hole) in[i] = set_probe(s, key[i]);
  }
}

}  // namespace nezha

struct nezha_itemset {
  uint64_t* slots;      // device, n_buckets * kBucketSlots keys, kEmpty = free
  uint64_t n_buckets;
  uint64_t* filter;     // device, n_blocks blocks of 8 words (see SetView), or NULL
  uint64_t n_blocks;
  int64_t n_distinct;
  int32_t L;
  int32_t radices[NEZHA_MAX_LEVELS];
  uint64_t mult[NEZHA_MAX_LEVELS];
  int device;
  uint32_t magic;
};
constexpr uint32_t kSetMagic = 0x4E5A4853u;
