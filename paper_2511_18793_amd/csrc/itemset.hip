// The model-free verifier (Sec. 3.3): an open-addressing hash set of the packed 64-bit item
// indices of Eq. 4 in device memory, its parallel build, and the stand-alone batch
// verification of Eq. 5 with order-preserving compaction of the accepted tuples.
#include <stdlib.h>

#include <mutex>
#include <new>
#include <unordered_set>
#include <vector>

#include "nezha_internal.h"

namespace nezha {

char* error_buffer() {
  static thread_local char buf[512] = "";
  return buf;
}
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

// ---- per-kernel timing -------------------------------------------------------------------
namespace {
struct ProfileRecord {
  KernelKind kind;
  hipEvent_t start, stop;
};
std::mutex g_prof_mutex;
std::vector<ProfileRecord> g_prof_records;
bool g_prof_on = false;
const char* const kKernelNames[kKernelKinds] = {
    "pack_weights_kernel", "user_gemm_kernel", "expand_kernel", "merge_kernel",
    "verify_probe_kernel", "verify_scan_kernel", "verify_scatter_kernel", "insert_kernel",
    "random_gather_kernel", "level_small_kernel", "expand_request_kernel",
    "decode_small_kernel", "wide_logits_kernel", "wide_rows_kernel", "wide_select_kernel"};
}  // namespace

ProfileScope::ProfileScope(KernelKind kind, hipStream_t s) : slot(-1), stream(s) {
  if (!g_prof_on) return;
  ProfileRecord r;
  r.kind = kind;
  if (hipEventCreate(&r.start) != hipSuccess) return;
  if (hipEventCreate(&r.stop) != hipSuccess) {
    (void)hipEventDestroy(r.start);
    return;
  }
  (void)hipEventRecord(r.start, stream);
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof_records.push_back(r);
  slot = (int)g_prof_records.size() - 1;
}
ProfileScope::~ProfileScope() {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (slot < (int)g_prof_records.size()) (void)hipEventRecord(g_prof_records[slot].stop, stream);
}

bool radix_multipliers(int32_t L, const int32_t* radices, uint64_t* mult) {
  unsigned __int128 p = 1;
  for (int32_t l = 0; l < L; ++l) {
    if (radices[l] < 1) return false;
    mult[l] = (uint64_t)p;
    p *= (unsigned __int128)(uint32_t)radices[l];
    if (p > (unsigned __int128)0xFFFFFFFFFFFFFFFFull) return false;
  }
  return true;
}

// ---- registry of live sets ------------------------------------------------------------------
// A handle is valid from the moment nezha_build_itemset returns it until nezha_free_itemset takes
// it; the registry answers that question without reading the handle's memory, so a handle that
// was freed (or never was one) is refused instead of dereferenced.
namespace {
std::mutex g_sets_mutex;
std::unordered_set<const nezha_itemset*>& live_sets() {
  static std::unordered_set<const nezha_itemset*> sets;
  return sets;
}
}  // namespace
bool set_is_live(const nezha_itemset* set) {
  if (!set) return false;
  std::lock_guard<std::mutex> lock(g_sets_mutex);
  return live_sets().count(set) != 0;
}

namespace {

// Test hook for the failure path of nezha_build_itemset: with NEZHA_TEST_FAIL_ALLOC=N in the
// environment the N-th allocation of a build (1 = the host-side handle, 2 = the table, 3 = the
// status words, then the staging buffer when the catalog is in host memory, last the prefilter)
// is reported as failed without being attempted.  Unset, empty or 0: no effect.
struct BuildAllocs {
  int failing = 0, made = 0;
  BuildAllocs() {
    const char* v = getenv("NEZHA_TEST_FAIL_ALLOC");
    if (v && *v) failing = atoi(v);
  }
  bool fails() { return ++made == failing; }
  hipError_t device(void** p, size_t bytes) {
    if (fails()) {
      *p = nullptr;
      return hipErrorOutOfMemory;
    }
    return hipMalloc(p, bytes);
  }
};

struct Radix {
  int32_t L;
  int32_t T[NEZHA_MAX_LEVELS];
  uint64_t mult[NEZHA_MAX_LEVELS];
};

// Eq. 4 on one tuple; false if a code is outside its radix.
__device__ __forceinline__ bool pack_tuple(const int32_t* t, const Radix& r, uint64_t& key) {
  key = 0;
  bool ok = true;
  for (int l = 0; l < r.L; ++l) {
    int32_t c = t[l];
    ok &= (uint32_t)c < (uint32_t)r.T[l];
    key += (uint64_t)(uint32_t)c * r.mult[l];
  }
  return ok;
}

__global__ void fill_empty_kernel(uint64_t* slots, uint64_t n) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) slots[i] = kEmpty;
}

// One thread per catalog tuple: pack, then claim the first free slot on the probe path with a
// 64-bit compare-and-swap.  Only the value the CAS returns decides, so a stale plain read
// can do no harm.  status[0]: tuples with a bad code; status[1]: keys that found no slot;
// status[2]: distinct keys stored.
__global__ void insert_kernel(const int32_t* __restrict__ codes, int64_t n, Radix r,
                              uint64_t* slots, uint64_t n_buckets,
                              unsigned long long* status) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    uint64_t key;
    if (!pack_tuple(codes + i * r.L, r, key)) {
      atomicAdd(&status[0], 1ull);
      continue;
    }
    uint64_t b = home_bucket(key, n_buckets);
    bool done = false;
    for (uint64_t step = 0; step < n_buckets && !done; ++step) {
      unsigned long long* bucket = reinterpret_cast<unsigned long long*>(slots + b * kBucketSlots);
      for (int s = 0; s < kBucketSlots && !done; ++s) {
        unsigned long long cur = __atomic_load_n(&bucket[s], __ATOMIC_RELAXED);
        if (cur == kEmpty) cur = atomicCAS(&bucket[s], (unsigned long long)kEmpty, key);
        if (cur == kEmpty) {
          atomicAdd(&status[2], 1ull);
          done = true;
        } else if (cur == key) {
          done = true;  // duplicate tuple: stored once
        }
      }
      b = (b + 1 == n_buckets) ? 0 : b + 1;
    }
    if (!done) atomicAdd(&status[1], 1ull);
  }
}

// The prefilter from the finished table: every stored key sets its bit.
__global__ void filter_kernel(const uint64_t* __restrict__ slots, uint64_t n_slots,
                              unsigned long long* filter, uint64_t n_blocks, uint64_t mult_last) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (; i < n_slots; i += stride) {
    const uint64_t key = slots[i];
    if (key == kEmpty) continue;
    const uint64_t code = key / mult_last, prefix = key - code * mult_last;
    atomicOr(&filter[filter_word(prefix, (uint32_t)code, n_blocks)], 1ull << (code & 63));
  }
}

// ---- stand-alone verification ----------------------------------------------------------
constexpr int kVerifyThreads = 256;
constexpr int kPerThread = 4;                                 // consecutive tuples per lane
constexpr int kVerifyBlock = kVerifyThreads * kPerThread;     // tuples per workgroup
constexpr int64_t kFusedPrefixBlocks = 16384;                 // above this a scan kernel runs

// Pass 1: pack + probe, write the mask bytes and the number of accepted tuples per block.
// A lane per tuple, four consecutive tuples each, probed one after the other: few registers, so
// that the chip holds as many waves as it can, which is where the memory-level parallelism comes
// from.  (Measured against this on the stress workload, 78 us per call: all of a lane's home
// buckets requested at once, 4 / 8 / 16 per lane: 138 / 156 / 195 us; eight lanes per bucket with
// the keys staged through LDS: 90 us.)
template <int L>
__global__ __launch_bounds__(kVerifyThreads) void verify_probe_kernel(
    const int32_t* __restrict__ codes, int64_t n, Radix r, SetView set,
    uint8_t* __restrict__ mask, int32_t* __restrict__ block_count) {
  __shared__ int32_t wave_count[kVerifyThreads / 64];
  const int64_t base = ((int64_t)blockIdx.x * kVerifyThreads + threadIdx.x) * kPerThread;
  uint64_t key[kPerThread];
  bool ok[kPerThread];
#pragma unroll
  for (int j = 0; j < kPerThread; ++j) {
    ok[j] = false;
    key[j] = 0;
    if (base + j < n) {
      int32_t t[NEZHA_MAX_LEVELS];
      const int LL = (L > 0) ? L : r.L;
#pragma unroll
      for (int l = 0; l < (L > 0 ? L : NEZHA_MAX_LEVELS); ++l)
        if (l < LL) t[l] = codes[(base + j) * LL + l];
      ok[j] = pack_tuple(t, r, key[j]);
    }
  }
  int cnt = 0;
  uint32_t bits = 0;
#pragma unroll
  for (int j = 0; j < kPerThread; ++j) {
    bool in = ok[j] && set_probe(set, key[j]);
    bits |= (in ? 1u : 0u) << (8 * j);
    cnt += in ? 1 : 0;
  }
  if (base + kPerThread <= n && (reinterpret_cast<uintptr_t>(mask) & 3) == 0) {
    *reinterpret_cast<uint32_t*>(mask + base) = bits;
  } else {
#pragma unroll
    for (int j = 0; j < kPerThread; ++j)
      if (base + j < n) mask[base + j] = (bits >> (8 * j)) & 1u;
  }
  // block total: wave reduction by cross-lane adds, then a 4-entry LDS sum
  for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off);
  if ((threadIdx.x & 63) == 0) wave_count[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int s = 0;
    for (int w = 0; w < kVerifyThreads / 64; ++w) s += wave_count[w];
    block_count[blockIdx.x] = s;
  }
}

// Pass 2 (one workgroup): exclusive scan of the per-block counts, total to out_count.
__global__ __launch_bounds__(1024) void verify_scan_kernel(const int32_t* __restrict__ block_count,
                                                           int64_t n_blocks,
                                                           int64_t* __restrict__ block_offset,
                                                           int64_t* __restrict__ out_count) {
  __shared__ int64_t wave_sum[16];
  __shared__ int64_t carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int64_t start = 0; start < n_blocks; start += 1024) {
    int64_t i = start + threadIdx.x;
    int64_t v = (i < n_blocks) ? block_count[i] : 0;
    int64_t incl = v;
    for (int off = 1; off < 64; off <<= 1) {
      int64_t t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int64_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (i < n_blocks) block_offset[i] = before + incl - v;
    __syncthreads();
    if (threadIdx.x == 1023) carry_s = before + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0 && out_count) *out_count = carry_s;
}

// Pass 3: every block turns its mask bytes into ascending indices at its offset
// (ballot-free per-lane popcounts, wave prefix by cross-lane adds, LDS across waves).
//
// block_offset != NULL: the offsets come from verify_scan_kernel.  block_offset == NULL: every
// block sums the counts of the blocks before it itself (cheap up to a few thousand blocks) and
// the last block writes the grand total to out_count.
__global__ __launch_bounds__(kVerifyThreads) void verify_scatter_kernel(
    const uint8_t* __restrict__ mask, int64_t n, const int64_t* __restrict__ block_offset,
    const int32_t* __restrict__ block_count, int64_t* __restrict__ out_index,
    int64_t* __restrict__ out_count) {
  __shared__ int32_t wave_total[kVerifyThreads / 64];
  __shared__ int64_t wave_before[kVerifyThreads / 64];
  int64_t offset = 0;
  if (block_offset) {
    offset = block_offset[blockIdx.x];
  } else {
    int64_t part = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kVerifyThreads) part += block_count[i];
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off);
    if ((threadIdx.x & 63) == 0) wave_before[threadIdx.x >> 6] = part;
    __syncthreads();
    for (int w = 0; w < kVerifyThreads / 64; ++w) offset += wave_before[w];
    if (out_count && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0)
      *out_count = offset + block_count[blockIdx.x];
    if (!out_index) return;
  }
  const int64_t base = ((int64_t)blockIdx.x * kVerifyThreads + threadIdx.x) * kPerThread;
  uint32_t bits = 0;
  if (base + kPerThread <= n && (reinterpret_cast<uintptr_t>(mask) & 3) == 0) {
    bits = *reinterpret_cast<const uint32_t*>(mask + base);
  } else {
    for (int j = 0; j < kPerThread; ++j)
      if (base + j < n) bits |= (uint32_t)(mask[base + j] & 1u) << (8 * j);
  }
  const int mine = __popc(bits);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = mine;
  for (int off = 1; off < 64; off <<= 1) {
    int t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  if (lane == 63) wave_total[wave] = incl;
  __syncthreads();
  int64_t pos = offset + incl - mine;
  for (int w = 0; w < wave; ++w) pos += wave_total[w];
#pragma unroll
  for (int j = 0; j < kPerThread; ++j)
    if ((bits >> (8 * j)) & 1u) out_index[pos++] = base + j;
}

// Probes every tuple of `codes` (as the draft step does: through the prefilter, then the table)
// and counts those that are not found.
__global__ void check_kernel(const int32_t* __restrict__ codes, int64_t n, Radix r, SetView set,
                             unsigned long long* missing) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    uint64_t key;
    bool ok = pack_tuple(codes + i * r.L, r, key);
    if (ok) {
      const uint64_t code = key / set.mult_last, prefix = key - code * set.mult_last;
      ok = set_contains(set, prefix, (uint32_t)code);
    }
    if (!ok) atomicAdd(missing, 1ull);
  }
}
// Measurement aid: n independent reads of whole lines (LINE bytes, LINE-aligned) at pseudo-random
// places of a buffer.  DEPTH lines are in flight per lane (COOP = false: a lane reads a whole line,
// as a verifier lane reads a bucket), or per group of eight lanes that share each line eight
// bytes apiece (COOP = true, 64-byte lines).  The loaded words are folded into one value so the
// reads cannot be dropped.
template <int LINE, int DEPTH, bool COOP>
__global__ __launch_bounds__(256) void random_gather_kernel(const uint64_t* __restrict__ buf,
                                                            uint64_t n_lines, int64_t n,
                                                            uint64_t seed, uint64_t* sink) {
  uint64_t acc = 0;
  if constexpr (COOP) {
    const int64_t group = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 3;
    const int part = threadIdx.x & 7;
    uint64_t v[DEPTH];
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      v[j] = 0;
      const int64_t i = group * DEPTH + j;
      if (i < n) {
        const uint64_t line = __umul64hi(hash64(seed + (uint64_t)i), n_lines);
        v[j] = *(global_ptr<const uint64_t>)(buf + line * (LINE / 8) + part);
      }
    }
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) acc ^= v[j];
  } else {
    const int64_t base = ((int64_t)blockIdx.x * 256 + threadIdx.x) * DEPTH;
    ulonglong2 v[DEPTH][LINE / 16];
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      const bool live = base + j < n;
      const uint64_t line = live ? __umul64hi(hash64(seed + (uint64_t)(base + j)), n_lines) : 0;
#pragma unroll
      for (int q = 0; q < LINE / 16; ++q) {
        v[j][q] = ulonglong2{0, 0};
        if (live) v[j][q] = load_global_u64x2(buf + line * (LINE / 8) + 2 * q);
      }
    }
#pragma unroll
    for (int j = 0; j < DEPTH; ++j)
#pragma unroll
      for (int q = 0; q < LINE / 16; ++q) acc ^= v[j][q].x + v[j][q].y;
  }
  if (acc == 0x0123456789ABCDEFull) sink[0] = acc;   // practically never; keeps the loads alive
}

}  // namespace
}  // namespace nezha

using namespace nezha;

extern "C" {

const char* nezha_last_error(void) { return error_buffer(); }

int nezha_build_itemset(const int32_t* codes, int64_t n, int32_t L, const int32_t* radices,
                        int codes_on_device, double load_factor, void* hip_stream,
                        nezha_itemset** out) {
  if (!out) return fail(NEZHA_EINVAL, "out is NULL");
  *out = nullptr;
  if (n < 0) return fail(NEZHA_EINVAL, "n = %lld is negative", (long long)n);
  if (n > 0 && !codes) return fail(NEZHA_EINVAL, "codes is NULL");
  if (!radices) return fail(NEZHA_EINVAL, "radices is NULL");
  if (L < 1 || L > NEZHA_MAX_LEVELS)
    return fail(NEZHA_EINVAL, "L = %d outside 1..%d", L, NEZHA_MAX_LEVELS);
  if (!(load_factor > 0.0 && load_factor <= 0.9))
    return fail(NEZHA_EINVAL, "load_factor %g outside (0, 0.9]", load_factor);
  Radix r;
  r.L = L;
  for (int l = 0; l < NEZHA_MAX_LEVELS; ++l) {
    r.T[l] = l < L ? radices[l] : 1;
    r.mult[l] = 0;
  }
  if (!radix_multipliers(L, radices, r.mult))
    return fail(NEZHA_ERANGE, "radices must be >= 1 with a product of at most 2^64-1");

  double want = (double)n / load_factor;
  if (want > 9.0e15) return fail(NEZHA_EINVAL, "table too large");
  uint64_t n_slots = (uint64_t)want;
  if ((double)n_slots < want) ++n_slots;
  uint64_t n_buckets = (n_slots + kBucketSlots - 1) / kBucketSlots;
  if (n_buckets == 0) n_buckets = 1;
  n_slots = n_buckets * kBucketSlots;

  hipStream_t stream = (hipStream_t)hip_stream;
  BuildAllocs allocs;
  nezha_itemset* s = allocs.fails() ? nullptr : new (std::nothrow) nezha_itemset;
  if (!s) return fail(NEZHA_ENOMEM, "host allocation failed");
  s->slots = nullptr;
  s->filter = nullptr;
  s->n_blocks = 0;
  s->n_buckets = n_buckets;
  s->n_distinct = 0;
  s->L = L;
  for (int l = 0; l < NEZHA_MAX_LEVELS; ++l) {
    s->radices[l] = r.T[l];
    s->mult[l] = r.mult[l];
  }
  s->magic = kSetMagic;

  unsigned long long* status = nullptr;
  int32_t* staged = nullptr;
  int rc = NEZHA_OK;
  auto cleanup = [&](int code) {
    if (status) (void)hipFree(status);
    if (staged) (void)hipFree(staged);
    if (code != NEZHA_OK) {
      if (s->slots) (void)hipFree(s->slots);
      if (s->filter) (void)hipFree(s->filter);
      s->magic = 0;
      delete s;
    }
    return code;
  };
#define BUILD_CHECK(expr)                                                                  \
  do {                                                                                     \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess) {                                                                \
      rc = fail(_e == hipErrorOutOfMemory ? NEZHA_ENOMEM : NEZHA_EHIP, "%s failed: %s",    \
                #expr, hipGetErrorString(_e));                                             \
      return cleanup(rc);                                                                  \
    }                                                                                      \
  } while (0)

  s->device = -1;
  BUILD_CHECK(allocs.device((void**)&s->slots, n_slots * sizeof(uint64_t)));
  BUILD_CHECK(hipGetDevice(&s->device));
  BUILD_CHECK(allocs.device((void**)&status, 4 * sizeof(unsigned long long)));
  BUILD_CHECK(hipMemsetAsync(status, 0, 4 * sizeof(unsigned long long), stream));
  {
    uint64_t blocks = (n_slots + 1023) / 1024;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_empty_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, s->slots,
                       n_slots);
    BUILD_CHECK(hipGetLastError());
  }
  const int64_t chunk_max = (int64_t)1 << 25;  // tuples staged per copy when codes are on the host
  if (!codes_on_device && n > 0) {
    int64_t cap = n < chunk_max ? n : chunk_max;
    BUILD_CHECK(allocs.device((void**)&staged, (size_t)cap * L * sizeof(int32_t)));
  }
  for (int64_t start = 0; start < n; start += chunk_max) {
    int64_t m = n - start < chunk_max ? n - start : chunk_max;
    const int32_t* src = codes + start * L;
    if (!codes_on_device) {
      BUILD_CHECK(hipMemcpyAsync(staged, src, (size_t)m * L * sizeof(int32_t),
                                 hipMemcpyHostToDevice, stream));
      src = staged;
    }
    int64_t blocks = (m + 255) / 256;
    if (blocks > 262144) blocks = 262144;
    {
      ProfileScope prof(kInsert, stream);
      hipLaunchKernelGGL(insert_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, m, r,
                         s->slots, n_buckets, status);
    }
    BUILD_CHECK(hipGetLastError());
    if (!codes_on_device) BUILD_CHECK(hipStreamSynchronize(stream));
  }
  unsigned long long host_status[4] = {0, 0, 0, 0};
  BUILD_CHECK(hipMemcpyAsync(host_status, status, sizeof(host_status), hipMemcpyDeviceToHost,
                             stream));
  BUILD_CHECK(hipStreamSynchronize(stream));
#undef BUILD_CHECK
  if (host_status[0] != 0) {
    rc = fail(NEZHA_ERANGE, "%llu catalog tuples have a code outside [0, T_l)", host_status[0]);
    return cleanup(rc);
  }
  if (host_status[1] != 0) {
    rc = fail(NEZHA_EFULL, "%llu keys found no free slot", host_status[1]);
    return cleanup(rc);
  }
  s->n_distinct = (int64_t)host_status[2];
  {
    // The prefilter: 512-bit blocks, one per 16 keys on average (4 bytes per item).  Most
    // candidates of the draft step are not items; a filter word is a small, cache-resident access
    // that turns most of their table probes (a random HBM line each) away.  It can only say "not
    // in the set" for keys that are not in it, so results do not change.
    s->n_blocks = (uint64_t)(s->n_distinct / 16 + 1);
    hipError_t fe = allocs.device((void**)&s->filter, s->n_blocks * 64);
    if (fe == hipSuccess) {
      fe = hipMemsetAsync(s->filter, 0, s->n_blocks * 64, stream);
      if (fe == hipSuccess) {
        uint64_t blocks = (n_slots + 1023) / 1024;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(filter_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, s->slots,
                           (uint64_t)n_slots, reinterpret_cast<unsigned long long*>(s->filter),
                           s->n_blocks, s->mult[L - 1]);
        fe = hipGetLastError();
      }
      if (fe == hipSuccess) fe = hipStreamSynchronize(stream);
    }
    if (fe != hipSuccess) {
      // A filter that is not known to be complete would turn valid items away (a clear bit means
      // "not in the set"): the set then works without one.
      if (s->filter) (void)hipFree(s->filter);
      s->filter = nullptr;
      s->n_blocks = 0;
      (void)hipGetLastError();
    }
  }
  {
    std::lock_guard<std::mutex> lock(g_sets_mutex);
    live_sets().insert(s);
  }
  *out = s;
  return cleanup(NEZHA_OK);
}

int nezha_itemset_info(const nezha_itemset* set, int64_t* n_distinct, int64_t* n_slots,
                       int32_t* L, int32_t* radices) {
  if (!set_is_live(set)) return fail(NEZHA_EINVAL, "not an item set");
  if (n_distinct) *n_distinct = set->n_distinct;
  if (n_slots) *n_slots = (int64_t)(set->n_buckets * kBucketSlots);
  if (L) *L = set->L;
  if (radices)
    for (int l = 0; l < set->L; ++l) radices[l] = set->radices[l];
  return NEZHA_OK;
}

int nezha_free_itemset(nezha_itemset* set) {
  if (!set) return NEZHA_OK;
  {
    // the registry decides, so a handle that was freed before is refused without being read
    std::lock_guard<std::mutex> lock(g_sets_mutex);
    if (live_sets().erase(set) == 0) return fail(NEZHA_EINVAL, "not an item set (freed twice?)");
  }
  set->magic = 0;
  if (set->filter) (void)hipFree(set->filter);
  hipError_t e = set->slots ? hipFree(set->slots) : hipSuccess;
  delete set;
  if (e != hipSuccess) return fail(NEZHA_EHIP, "hipFree failed: %s", hipGetErrorString(e));
  return NEZHA_OK;
}

size_t nezha_verify_workspace(int64_t n) {
  if (n < 0) return 0;
  size_t blocks = (size_t)((n + kVerifyBlock - 1) / kVerifyBlock);
  if (blocks == 0) blocks = 1;
  size_t counts = (blocks * sizeof(int32_t) + 15) & ~(size_t)15;
  return counts + blocks * sizeof(int64_t);
}

// The launches of the stand-alone verifier; `workspace` is known to be large enough.
static int verify_launch(const nezha_itemset* set, const int32_t* codes, int64_t n,
                         uint8_t* out_mask, int64_t* out_index, int64_t* out_count,
                         void* workspace, hipStream_t stream) {
  const bool compact = out_index || out_count;
  const int64_t blocks = (n + kVerifyBlock - 1) / kVerifyBlock;
  const size_t counts_bytes = ((size_t)blocks * sizeof(int32_t) + 15) & ~(size_t)15;
  // (the probe pass writes its block counts whether or not they are wanted afterwards)
  int32_t* block_count = static_cast<int32_t*>(workspace);
  int64_t* block_offset = reinterpret_cast<int64_t*>(static_cast<char*>(workspace) + counts_bytes);
  Radix r;
  r.L = set->L;
  for (int l = 0; l < NEZHA_MAX_LEVELS; ++l) {
    r.T[l] = set->radices[l];
    r.mult[l] = set->mult[l];
  }
  // (the stand-alone verifier's queries are mostly present keys: the prefilter would only add an
  // access, so it is left out of the view)
  SetView view{set->slots, set->n_buckets, nullptr, 0, 0};
  dim3 grid((unsigned)blocks), block(kVerifyThreads);
  {
  ProfileScope prof(kVerifyProbe, stream);
  switch (set->L) {
    case 3:
      hipLaunchKernelGGL(verify_probe_kernel<3>, grid, block, 0, stream, codes, n, r, view,
                         out_mask, block_count);
      break;
    case 4:
      hipLaunchKernelGGL(verify_probe_kernel<4>, grid, block, 0, stream, codes, n, r, view,
                         out_mask, block_count);
      break;
    default:
      hipLaunchKernelGGL(verify_probe_kernel<0>, grid, block, 0, stream, codes, n, r, view,
                         out_mask, block_count);
  }
  }
  NEZHA_HIP_CHECK(hipGetLastError());
  if (compact && blocks <= kFusedPrefixBlocks) {
    // few blocks: the scatter pass forms its own offsets, no separate scan launch
    ProfileScope prof(kVerifyScatter, stream);
    hipLaunchKernelGGL(verify_scatter_kernel, grid, block, 0, stream, (const uint8_t*)out_mask, n,
                       (const int64_t*)nullptr, (const int32_t*)block_count, out_index, out_count);
    NEZHA_HIP_CHECK(hipGetLastError());
  } else if (compact) {
    {
      ProfileScope prof(kVerifyScan, stream);
      hipLaunchKernelGGL(verify_scan_kernel, dim3(1), dim3(1024), 0, stream,
                         (const int32_t*)block_count, blocks, block_offset, out_count);
    }
    NEZHA_HIP_CHECK(hipGetLastError());
    if (out_index) {
      ProfileScope prof(kVerifyScatter, stream);
      hipLaunchKernelGGL(verify_scatter_kernel, grid, block, 0, stream,
                         (const uint8_t*)out_mask, n, (const int64_t*)block_offset,
                         (const int32_t*)block_count, out_index, (int64_t*)nullptr);
    }
    NEZHA_HIP_CHECK(hipGetLastError());
  }
  return NEZHA_OK;
}

// Argument checks shared by the two verifier entry points (everything but the workspace).
static int verify_check(const nezha_itemset* set, const int32_t* codes, int64_t n,
                        const uint8_t* out_mask) {
  if (!set_is_live(set)) return fail(NEZHA_EINVAL, "not an item set");
  if (n < 0) return fail(NEZHA_EINVAL, "n = %lld is negative", (long long)n);
  if (n > 0 && (!codes || !out_mask)) return fail(NEZHA_EINVAL, "codes or out_mask is NULL");
  if (n > (int64_t)kVerifyBlock * 0x7FFFFFFF) return fail(NEZHA_EINVAL, "n too large");
  return NEZHA_OK;
}

// n == 0: nothing to probe; the count, if wanted, is written by a one-block launch.
static int verify_empty(int64_t* out_count, hipStream_t stream) {
  if (out_count) {
    hipLaunchKernelGGL(verify_scan_kernel, dim3(1), dim3(1024), 0, stream, (const int32_t*)nullptr,
                       (int64_t)0, (int64_t*)nullptr, out_count);
    NEZHA_HIP_CHECK(hipGetLastError());
  }
  return NEZHA_OK;
}

int nezha_verify_tuples(const nezha_itemset* set, const int32_t* codes, int64_t n,
                        uint8_t* out_mask, int64_t* out_index, int64_t* out_count,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = verify_check(set, codes, n, out_mask);
  if (rc != NEZHA_OK) return rc;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (n == 0) return verify_empty(out_count, stream);
  if (!workspace) return fail(NEZHA_EINVAL, "workspace is NULL");
  if (workspace_bytes < nezha_verify_workspace(n))
    return fail(NEZHA_EINVAL, "workspace has %zu bytes, %zu needed", workspace_bytes,
                nezha_verify_workspace(n));
  if (reinterpret_cast<uintptr_t>(workspace) & 15)
    return fail(NEZHA_EINVAL, "workspace is not 16-byte aligned");
  return verify_launch(set, codes, n, out_mask, out_index, out_count, workspace, stream);
}

}  // extern "C"

// ---- the verifier for callers that cannot allocate -------------------------------------------
// The block counts and offsets of nezha_verify_tuples live in a fixed array in device memory that
// belongs to the library's code object (one copy per GPU, held until the process ends).
namespace nezha {
namespace {
constexpr int64_t kStaticVerifyBlocks = NEZHA_VERIFY_STATIC_MAX / kVerifyBlock;
constexpr size_t kStaticVerifyBytes =
    (size_t)kStaticVerifyBlocks * sizeof(int32_t) + (size_t)kStaticVerifyBlocks * sizeof(int64_t);
static_assert(NEZHA_VERIFY_STATIC_MAX % kVerifyBlock == 0, "whole blocks");
static_assert(((size_t)kStaticVerifyBlocks * sizeof(int32_t)) % 16 == 0, "offsets stay aligned");
static __device__ __align__(256) unsigned char scratch[kStaticVerifyBytes];

// The array's address on each device, asked for once per device with that device current.  (In
// host code the array's name is only a handle for this query, never an address.)
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  NEZHA_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(NEZHA_EINVAL, "device %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    NEZHA_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(NEZHA_EHIP, "hipGetSymbolAddress gave no address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return NEZHA_OK;
}
}  // namespace
}  // namespace nezha

extern "C" {

int nezha_verify_tuples_static(const nezha_itemset* set, const int32_t* codes, int64_t n,
                               uint8_t* out_mask, int64_t* out_index, int64_t* out_count,
                               void* hip_stream) {
  int rc = verify_check(set, codes, n, out_mask);
  if (rc != NEZHA_OK) return rc;
  if (n > NEZHA_VERIFY_STATIC_MAX)
    return fail(NEZHA_EINVAL, "n = %lld exceeds NEZHA_VERIFY_STATIC_MAX = %lld; use "
                "nezha_verify_tuples with a workspace", (long long)n,
                (long long)NEZHA_VERIFY_STATIC_MAX);
  hipStream_t stream = (hipStream_t)hip_stream;
  if (n == 0) return verify_empty(out_count, stream);
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != NEZHA_OK) return rc;
  // Nothing in the array has to start at zero: the probe pass writes the count of every block of
  // this call before any other pass reads it, and the scan writes every offset that is read.
  return verify_launch(set, codes, n, out_mask, out_index, out_count, ws, stream);
}

int nezha_check_itemset(const nezha_itemset* set, const int32_t* codes, int64_t n,
                        int codes_on_device, void* hip_stream, int64_t* n_missing) {
  if (!set_is_live(set)) return fail(NEZHA_EINVAL, "not an item set");
  if (n < 0 || (n > 0 && !codes) || !n_missing) return fail(NEZHA_EINVAL, "bad argument");
  *n_missing = 0;
  if (n == 0) return NEZHA_OK;
  hipStream_t stream = (hipStream_t)hip_stream;
  Radix r;
  r.L = set->L;
  for (int l = 0; l < NEZHA_MAX_LEVELS; ++l) {
    r.T[l] = set->radices[l];
    r.mult[l] = set->mult[l];
  }
  SetView view{set->slots, set->n_buckets, set->filter, set->n_blocks, set->mult[set->L - 1]};
  unsigned long long* missing = nullptr;
  int32_t* staged = nullptr;
  int rc = NEZHA_OK;
  auto done = [&](int code) {
    if (missing) (void)hipFree(missing);
    if (staged) (void)hipFree(staged);
    return code;
  };
#define CHECK_OR_DONE(expr)                                                                \
  do {                                                                                     \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess) {                                                                \
      rc = fail(_e == hipErrorOutOfMemory ? NEZHA_ENOMEM : NEZHA_EHIP, "%s failed: %s",    \
                #expr, hipGetErrorString(_e));                                             \
      return done(rc);                                                                     \
    }                                                                                      \
  } while (0)
  CHECK_OR_DONE(hipMalloc((void**)&missing, sizeof(unsigned long long)));
  CHECK_OR_DONE(hipMemsetAsync(missing, 0, sizeof(unsigned long long), stream));
  const int64_t chunk_max = (int64_t)1 << 25;
  if (!codes_on_device) {
    const int64_t cap = n < chunk_max ? n : chunk_max;
    CHECK_OR_DONE(hipMalloc((void**)&staged, (size_t)cap * set->L * sizeof(int32_t)));
  }
  for (int64_t start = 0; start < n; start += chunk_max) {
    const int64_t m = n - start < chunk_max ? n - start : chunk_max;
    const int32_t* src = codes + start * set->L;
    if (!codes_on_device) {
      CHECK_OR_DONE(hipMemcpyAsync(staged, src, (size_t)m * set->L * sizeof(int32_t),
                                   hipMemcpyHostToDevice, stream));
      src = staged;
    }
    int64_t blocks = (m + 255) / 256;
    if (blocks > 262144) blocks = 262144;
    hipLaunchKernelGGL(check_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, m, r, view,
                       missing);
    CHECK_OR_DONE(hipGetLastError());
    if (!codes_on_device) CHECK_OR_DONE(hipStreamSynchronize(stream));
  }
  unsigned long long host_missing = 0;
  CHECK_OR_DONE(hipMemcpyAsync(&host_missing, missing, sizeof(host_missing), hipMemcpyDeviceToHost,
                               stream));
  CHECK_OR_DONE(hipStreamSynchronize(stream));
#undef CHECK_OR_DONE
  *n_missing = (int64_t)host_missing;
  return done(NEZHA_OK);
}

int nezha_bench_random_gather_depth(const void* buf, size_t bytes, int64_t n, int line_bytes,
                                    int depth, int lanes_per_line, uint64_t seed, void* sink,
                                    void* hip_stream) {
  if (!buf || !sink || n < 0 || (line_bytes != 64 && line_bytes != 128) ||
      bytes < (size_t)line_bytes || (reinterpret_cast<uintptr_t>(buf) & 127))
    return fail(NEZHA_EINVAL, "bad argument");
  if (depth != 1 && depth != 2 && depth != 4 && depth != 8 && depth != 16)
    return fail(NEZHA_EINVAL, "depth must be 1, 2, 4, 8 or 16");
  if (lanes_per_line != 1 && !(lanes_per_line == 8 && line_bytes == 64))
    return fail(NEZHA_EINVAL, "lanes_per_line is 1, or 8 with 64-byte lines");
  if (line_bytes == 128 && depth == 16) return fail(NEZHA_EINVAL, "depth 16 needs 64-byte lines");
  if (n == 0) return NEZHA_OK;
  hipStream_t stream = (hipStream_t)hip_stream;
  const uint64_t n_lines = bytes / (size_t)line_bytes;
  const int64_t per_block = lanes_per_line == 8 ? (int64_t)32 * depth : (int64_t)256 * depth;
  dim3 grid((unsigned)((n + per_block - 1) / per_block)), block(256);
  const uint64_t* b = static_cast<const uint64_t*>(buf);
  uint64_t* sk = static_cast<uint64_t*>(sink);
  ProfileScope prof(kGather, stream);
#define GATHER(LINEV, DEPTHV, COOPV)                                                            \
  hipLaunchKernelGGL((random_gather_kernel<LINEV, DEPTHV, COOPV>), grid, block, 0, stream, b,   \
                     n_lines, n, seed, sk)
#define GATHER_DEPTH(LINEV, COOPV)                    \
  do {                                                \
    if (depth == 1) GATHER(LINEV, 1, COOPV);          \
    else if (depth == 2) GATHER(LINEV, 2, COOPV);     \
    else if (depth == 4) GATHER(LINEV, 4, COOPV);     \
    else GATHER(LINEV, 8, COOPV);                     \
  } while (0)
  if (lanes_per_line == 8) {
    if (depth == 16) GATHER(64, 16, true);
    else GATHER_DEPTH(64, true);
  } else if (line_bytes == 64) {
    if (depth == 16) GATHER(64, 16, false);
    else GATHER_DEPTH(64, false);
  } else {
    GATHER_DEPTH(128, false);
  }
#undef GATHER_DEPTH
#undef GATHER
  NEZHA_HIP_CHECK(hipGetLastError());
  return NEZHA_OK;
}

int nezha_bench_random_gather(const void* buf, size_t bytes, int64_t n, int line_bytes,
                              uint64_t seed, void* sink, void* hip_stream) {
  return nezha_bench_random_gather_depth(buf, bytes, n, line_bytes, 4, 1, seed, sink, hip_stream);
}

int nezha_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof_on = on != 0;
  return NEZHA_OK;
}

int nezha_profile_reset(void) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (ProfileRecord& r : g_prof_records) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof_records.clear();
  return NEZHA_OK;
}

int nezha_profile_kinds(void) { return (int)kKernelKinds; }

namespace nezha {
namespace {
__global__ void empty_kernel() {}
}  // namespace
}  // namespace nezha

int nezha_profile_event_overhead(int launches, void* hip_stream, double* mean_us) {
  if (launches < 1 || launches > 10000 || !mean_us) return fail(NEZHA_EINVAL, "bad argument");
  hipStream_t stream = (hipStream_t)hip_stream;
  std::vector<hipEvent_t> ev(2 * (size_t)launches);
  for (auto& e : ev) NEZHA_HIP_CHECK(hipEventCreate(&e));
  for (int i = 0; i < launches; ++i) {
    NEZHA_HIP_CHECK(hipEventRecord(ev[2 * i], stream));
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, stream);
    NEZHA_HIP_CHECK(hipEventRecord(ev[2 * i + 1], stream));
  }
  NEZHA_HIP_CHECK(hipStreamSynchronize(stream));
  double total = 0.0;
  for (int i = 0; i < launches; ++i) {
    float t = 0.f;
    NEZHA_HIP_CHECK(hipEventElapsedTime(&t, ev[2 * i], ev[2 * i + 1]));
    total += t;
  }
  for (auto& e : ev) (void)hipEventDestroy(e);
  *mean_us = 1e3 * total / launches;
  return NEZHA_OK;
}

int nezha_profile_read(int kind, const char** name, int64_t* launches, double* total_ms) {
  if (kind < 0 || kind >= (int)kKernelKinds) return fail(NEZHA_EINVAL, "kind out of range");
  if (name) *name = kKernelNames[kind];
  int64_t n = 0;
  double ms = 0.0;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (const ProfileRecord& r : g_prof_records) {
    if ((int)r.kind != kind) continue;
    hipError_t e = hipEventSynchronize(r.stop);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
    if (e != hipSuccess)
      return fail(NEZHA_EHIP, "reading a timing event failed: %s", hipGetErrorString(e));
    ms += t;
    ++n;
  }
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  return NEZHA_OK;
}

int nezha_unpack_keys(const uint64_t* keys, int64_t n, int32_t L, const int32_t* radices,
                      int32_t* codes) {
  if (n < 0 || L < 1 || L > NEZHA_MAX_LEVELS || !radices || (n > 0 && (!keys || !codes)))
    return fail(NEZHA_EINVAL, "bad argument");
  for (int l = 0; l < L; ++l)
    if (radices[l] < 1) return fail(NEZHA_EINVAL, "radix < 1");
  for (int64_t i = 0; i < n; ++i) {
    uint64_t k = keys[i];
    for (int l = 0; l < L; ++l) {
      uint64_t T = (uint64_t)radices[l];
      codes[i * L + l] = (int32_t)(k % T);
      k /= T;
    }
  }
  return NEZHA_OK;
}

}  // extern "C"
