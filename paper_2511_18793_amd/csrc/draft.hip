// One level of the draft head's beam search (Alg. 3, inference loop body; Eq. 2-3) with the
// last level's hash-set verification (Eq. 4-5) for a batch of requests.
//
// Kernels (which of them take a level follows from its shape alone):
//   pack_weights_kernel     W_l (bf16, row major) -> MFMA operand order (bf16 workloads only)
//   user_gemm_*             A_l = H_l * W_l[0:d]           (the beam-independent part of Eq. 2)
//   expand_*_kernel         per beam: z = A_l + c * W_l[d:d+e] by MFMA, log-sum-exp and the K best
//                           codes; logits never leave the chip.  expand_request_kernel also does
//                           the request's selection where no set is consulted
//   first_level_kernel      a level with one entering beam and no state (level 1): the logits are
//                           the user part; selection, outputs and Transition in one launch
//   merge_kernel            per request: cumulative scores, Eq. 4 indices, Eq. 5 probes, the K
//                           best surviving candidates, and the Transition of Eq. 3
//   level_small_kernel,     all of the above after the projection in one launch per level / per
//   decode_small_kernel     decode, for small shapes
//   wide_*_kernel           beams wider than 128 (wide_beam.h)
//   mfma_rate_kernel,       measurement aids: what the chip sustains on the bare instruction mixes
//   tile_step_kernel        of the projection and of the per-request expansion (the rooflines'
//                           measured denominators)
#include "nezha_internal.h"

#include <atomic>
#include <type_traits>

namespace nezha {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_to_float(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// max(a, b) for operands that are never NaN, as the single instruction it is (the generic maximum
// first rewrites both operands into canonical form, two more instructions per call).
__device__ __forceinline__ float max_of_numbers(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// Two running maxima in one register: (a, b) rounded towards zero to half precision, packed, and
// the element-wise maximum of two such pairs.  A maximum kept this way is off by less than one
// half-precision unit in the last place (2^-10 relative; below 2^-14 in magnitude: 2^-24
// absolute); half_floor / half_ceil turn it back into a float32 bound on the true maximum from
// below / above.  Values beyond the half range (|x| > 65504) are clamped by the conversion and
// must be detected by the caller (half_out_of_range).
__device__ __forceinline__ uint32_t pack_halves_rtz(float a, float b) {
  auto p = __builtin_amdgcn_cvt_pkrtz(a, b);
  uint32_t r;
  __builtin_memcpy(&r, &p, 4);
  return r;
}
__device__ __forceinline__ uint32_t max_of_half_pairs(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
  const uint16_t x = (uint16_t)h;
  _Float16 f;
  __builtin_memcpy(&f, &x, 2);
  return (float)f;
}
__device__ __forceinline__ float half_floor(float m) { return m - fabsf(m) * 0.0009765625f - 1e-7f; }
__device__ __forceinline__ float half_ceil(float m) { return m + fabsf(m) * 0.0009765625f + 1e-7f; }
__device__ __forceinline__ bool half_out_of_range(float m) {
  return fabsf(m) >= 60000.f && fabsf(m) < INFINITY;
}
// Order-preserving map float -> uint32 (larger float <=> larger integer) and back.
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float unordered_bits(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o ^ 0x80000000u) : ~o;
  return __uint_as_float(u);
}

// ---- cross-lane helpers (wave64) ---------------------------------------------------------
// Orders this wave's LDS traffic: the hardware runs one wave's LDS instructions in issue
// order, so only the compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
}

// Value of lane (lane ^ M) for a compile-time M.  Distances 1, 2 and 8 are one DPP move
// (quad permutes, rotation by 8 inside a row of 16 lanes); 4 takes the two rotations by 4 and
// 12; 16 and 32 use the gfx950 row / half-wave swaps.
template <int M>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v, int lane) {
  if constexpr (M == 1) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
  } else if constexpr (M == 2) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
  } else if constexpr (M == 4) {
    const uint32_t down = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x124, 0xF, 0xF, true);
    const uint32_t up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x12C, 0xF, 0xF, true);
    return (lane & 4) ? down : up;   // row_ror:4 reads lane-4, row_ror:12 reads lane+4
  } else if constexpr (M == 8) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, true);
  } else if constexpr (M == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return (lane & 16) ? r[0] : r[1];
  } else {
    static_assert(M == 32, "lane distance");
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (lane & 32) ? r[0] : r[1];
  }
}

// One compare-exchange step of the bitonic network across lanes at distance LM, for R
// independent sequences at once (independent work hides the cross-lane latency).
template <int NPL, int R, int LM, typename T>
__device__ __forceinline__ void cross_step(T (&key)[R][NPL], int lane, bool keep_max) {
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
      T other;
      if constexpr (sizeof(T) == 8) {
        const uint32_t lo = lane_xor<LM>((uint32_t)key[r][j], lane);
        const uint32_t hi = lane_xor<LM>((uint32_t)(key[r][j] >> 32), lane);
        other = ((uint64_t)hi << 32) | lo;
      } else {
        other = lane_xor<LM>(key[r][j], lane);
      }
      const bool gt = key[r][j] > other;
      key[r][j] = (gt == keep_max) ? key[r][j] : other;
    }
}

// Bitonic sort of R sequences of 64*NPL keys (64- or 32-bit unsigned), NPL per lane, descending
// in position p = lane*NPL + j.
template <int NPL, int R, typename T = uint64_t>
__device__ __forceinline__ void sort_desc(T (&key)[R][NPL]) {
  const int lane = threadIdx.x & 63;
  constexpr int N = 64 * NPL;
#pragma unroll
  for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
    for (int dist = k >> 1; dist >= 1; dist >>= 1) {
      if (dist < NPL) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int j = 0; j < NPL; ++j) {
            if ((j & dist) == 0) {
              const int j2 = j | dist;
              // block direction: descending where bit k of the position is clear
              const bool desc = (k < NPL) ? ((j & k) == 0)
                                          : (k == N ? true : ((lane & (k / NPL)) == 0));
              const T a = key[r][j], b = key[r][j2];
              const bool a_gt = a > b;
              const bool swap = desc ? !a_gt : a_gt;
              key[r][j] = swap ? b : a;
              key[r][j2] = swap ? a : b;
            }
          }
      } else {
        const int lm = dist / NPL;
        const bool is_lo = (lane & lm) == 0;
        const bool desc = (k == N) ? true : ((lane & (k / NPL)) == 0);
        const bool keep_max = (is_lo == desc);
        if (lm == 1) cross_step<NPL, R, 1, T>(key, lane, keep_max);
        else if (lm == 2) cross_step<NPL, R, 2, T>(key, lane, keep_max);
        else if (lm == 4) cross_step<NPL, R, 4, T>(key, lane, keep_max);
        else if (lm == 8) cross_step<NPL, R, 8, T>(key, lane, keep_max);
        else if (lm == 16) cross_step<NPL, R, 16, T>(key, lane, keep_max);
        else cross_step<NPL, R, 32, T>(key, lane, keep_max);
      }
    }
  }
}

// Cuts R LDS buffers (R rows) back to their K largest keys, sorted descending at buf[0..):
// rows[r] points at CAP keys of which cnt[r] are in use.  On return cnt[r] = min(cnt[r], K)
// and tau[r] is the K-th largest key (0 while fewer than K are held).  Wave uniform.
template <int CAP, int NPL, int R>
__device__ __forceinline__ void compact_rows_n(uint64_t* const (&rows)[R], int (&cnt)[R],
                                               uint64_t (&tau)[R], int K) {
  const int lane = threadIdx.x & 63;
  uint64_t key[R][NPL];
  wave_sync();
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
      const int e = j * 64 + lane;
      key[r][j] = e < cnt[r] ? rows[r][e] : 0ull;
    }
  sort_desc<NPL, R>(key);
  wave_sync();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int keep = cnt[r] < K ? cnt[r] : K;
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
      const int p = lane * NPL + j;
      if (p < keep) rows[r][p] = key[r][j];
    }
    cnt[r] = keep;
  }
  wave_sync();
#pragma unroll
  for (int r = 0; r < R; ++r) tau[r] = (cnt[r] == K) ? rows[r][K - 1] : 0ull;
}

// Picks the smallest network that holds every row (all counts are wave uniform).
template <int CAP, int R>
__device__ __forceinline__ void compact_rows(uint64_t* const (&rows)[R], int (&cnt)[R],
                                             uint64_t (&tau)[R], int K) {
  int most = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) most = cnt[r] > most ? cnt[r] : most;
  if (most <= 64) {
    compact_rows_n<CAP, 1, R>(rows, cnt, tau, K);
  } else if (CAP == 128 || most <= 128) {
    compact_rows_n<CAP, 2, R>(rows, cnt, tau, K);
  } else {
    compact_rows_n<CAP, CAP / 64, R>(rows, cnt, tau, K);
  }
}

// A streaming top-K of 64-bit keys for one wave.  The buffer lives in LDS (CAP keys); keys
// that beat the threshold are appended with a ballot prefix; when fewer than 64 free places
// remain the buffer is sorted and cut back to the K largest, which raises the threshold.
template <int CAP>
struct WaveTopK {
  uint64_t* buf;   // LDS, CAP entries, private to the wave
  int cnt;         // wave uniform
  uint64_t tau;    // keys must be > tau to enter; wave uniform
  int K;

  __device__ __forceinline__ void init(uint64_t* b, int k) {
    buf = b;
    cnt = 0;
    tau = 0;
    K = k;
  }
  // Sort, keep the K largest at buf[0..), update tau.
  __device__ __forceinline__ void compact() {
    uint64_t* const rows[1] = {buf};
    int c[1] = {cnt};
    uint64_t t[1] = {0};
    compact_rows<CAP, 1>(rows, c, t, K);
    cnt = c[0];
    tau = t[0];
  }
  // One key per lane (0 = nothing).  All lanes of the wave must call this together.
  __device__ __forceinline__ void push(uint64_t key) {
    const bool pass = key > tau;
    const uint64_t bal = __ballot(pass);
    if (bal) {
      const int pos = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                      __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
      if (pass) buf[pos] = key;
      cnt += __popcll(bal);
      if (cnt > CAP - 64) compact();
    }
  }
};

// ---- weight packing -------------------------------------------------------------------------
// W_l (bf16, [(d+e), V] row major) is rearranged into MFMA operand order, two regions:
//  user part (rows 0..d-1), for v_mfma_f32_32x32x16_bf16:
//    Wu[((ct*KSu + ks)*64 + lane)*8 + j] = W[16*ks + 8*(lane/32) + j][32*ct + lane%32]
//    (KSu = d/16; columns at or beyond V are clamped to V-1 and never used)
//  beam part (rows d..d+e-1), for v_mfma_f32_16x16x32_bf16:
//    Wb[((ct*KSb + ks)*64 + lane)*8 + j] = W[d + 32*ks + 8*(lane/16) + j][16*ct + lane%16]
//    (KSb = e/32)
// so that the 64 lanes' B operands of one MFMA are one contiguous 1 KiB block.
__host__ __device__ inline int64_t packed_user_elems(int d, int V) {
  return (int64_t)((V + 31) / 32) * 32 * d;
}
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t* __restrict__ W,
                                                           uint16_t* __restrict__ Wp, int d, int e,
                                                           int V) {
  const int KSu = d / 16, KSb = e / 32;
  const int64_t n_user = (int64_t)((V + 31) / 32) * KSu * 64;
  const int64_t n_beam = (int64_t)(V / 16) * KSb * 64;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_user + n_beam) return;
  int col, k0;
  if (idx < n_user) {
    const int lane = (int)(idx & 63);
    const int64_t blk = idx >> 6;
    const int ks = (int)(blk % KSu), ct = (int)(blk / KSu);
    col = ct * 32 + (lane & 31);
    col = col < V ? col : V - 1;
    k0 = ks * 16 + 8 * (lane >> 5);
  } else {
    const int64_t r = idx - n_user;
    const int lane = (int)(r & 63);
    const int64_t blk = r >> 6;
    const int ks = (int)(blk % KSb), ct = (int)(blk / KSb);
    col = ct * 16 + (lane & 15);
    k0 = d + ks * 32 + 8 * (lane >> 4);
  }
  uint16_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = W[(int64_t)(k0 + j) * V + col];
  uint4 out;
  out.x = v[0] | ((uint32_t)v[1] << 16);
  out.y = v[2] | ((uint32_t)v[3] << 16);
  out.z = v[4] | ((uint32_t)v[5] << 16);
  out.w = v[6] | ((uint32_t)v[7] << 16);
  reinterpret_cast<uint4*>(Wp)[idx] = out;
}

// ---- user-part projection, bf16: A[B,V] = H[B,d] * W[0:d, V] -----------------------------
// Operand blocks: 1 KiB = the 64 lanes' 16-byte operands of one v_mfma_f32_32x32x16_bf16 (lane l:
// row or column l%32, k = 8*(l/32)..+7).  Result layout of the 32x32 MFMA: register r of lane l is
// row 8*(r/4) + 4*(l/32) + r%4, column l%32.
__device__ __forceinline__ void load_block_to_lds(const void* gptr, void* lds_block) {
  // 16 bytes per lane from global memory straight into LDS at lds_block + 16*lane
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_block, 16, 0, 0);
}

// Workgroup of NWM x NWN waves, each wave TM x TN tiles of 32x32.  K advances 32 per stage (two
// MFMA steps of 16).  The H tile is brought by global_load_lds (no staging registers) into one of
// four buffers, three stages ahead of use.  The packed W operands are loaded straight from global
// memory / L2 into registers, also three stages ahead (at these wave tiles LDS bandwidth is what
// binds; the waves of one column strip read the same lines).  One barrier per stage.  Workgroup
// ids are remapped so that the tiles that run on one XCD (ids equal modulo 8) are neighbours and
// share its L2.  (The largest products take user_gemm_big_tile below instead.)
constexpr int kGemmBuffers = 4;
// KSPLIT > 1 (small problems, whose time is the length of the k loop): the workgroup has KSPLIT
// groups of NWM x NWN waves, group s takes the s-th part of k with its own H buffers, and the
// groups' partial results are added through LDS at the end (d must be a multiple of 32 * KSPLIT).
template <int NWM, int NWN, int TM, int TN, int KSPLIT = 1>
__device__ __forceinline__ void user_gemm_tile(
    const uint16_t* __restrict__ H, int64_t h_stride, const uint16_t* __restrict__ Wu,
    float* __restrict__ A, int B, int d, int V, int tiles_n, int tiles_total, int tile_id) {
  typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
  constexpr int NW = NWM * NWN;
  constexpr int BM = NWM * TM * 32, BN = NWN * TN * 32;
  constexpr int CT = BN / 32;                        // 32-column tiles per workgroup
  constexpr int ASLOTS = BM * 4;                     // 16-byte slots of the H tile (64 B per row)
  constexpr int SSLOTS = ASLOTS;                     // one stage's buffer
  extern __shared__ __align__(16) uint4 smem_all[];  // [KSPLIT][kGemmBuffers][H tile]
  const int tid = threadIdx.x, lane = tid & 63;
  const int ksplit = (tid >> 6) / NW, wave = (tid >> 6) % NW;   // wave: index inside its group
  uint4* const smem = smem_all + ksplit * kGemmBuffers * SSLOTS;
  const int wm = wave / NWN, wn = wave % NWN;
  // Workgroup ids equal modulo 8 run on the same XCD.  When the grid allows it every XCD gets
  // 4 x 8 blocks of tiles (4 H panels and 8 W panels live in its L2 at a time); otherwise a
  // contiguous run of tiles.
  int tile_m, tile_n;
  {
    const int t = tile_id, xcd = t & 7, local = t >> 3;
    if (tiles_total % 256 == 0 && tiles_n % 8 == 0 && (tiles_total / tiles_n) % 4 == 0) {
      const int group = xcd + 8 * (local >> 5), groups_n = tiles_n >> 3;
      tile_m = (group / groups_n) * 4 + ((local & 31) >> 3);
      tile_n = (group % groups_n) * 8 + (local & 7);
    } else {
      const int per_xcd = tiles_total / 8;
      const int lin = (per_xcd * 8 == tiles_total) ? xcd * per_xcd + local : t;
      tile_m = lin / tiles_n;
      tile_n = lin - tile_m * tiles_n;
    }
  }
  const int row0 = tile_m * BM, ct0 = tile_n * CT;
  const int n_ct = (V + 31) / 32;
  const int KSu = d / 16;
  const int stages = d / 32 / KSPLIT;                // of this group
  const int stage0 = ksplit * stages;                // its first stage in the whole k range

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // H tile in LDS: row major, 64 bytes (this stage's 32 k) per row, with the 16-byte chunk index
  // XOR-ed with (row/4)%4 so that operand reads are free of bank conflicts.  One fetch
  // instruction brings 16 rows x 64 bytes; since lane l always lands at block + 16*l, the swizzle
  // is applied to the global address the lane reads.  Rows beyond B are clamped (their results
  // are never stored).  Wave w issues fetch instructions w, w+NW, ...
  constexpr int AINS = BM / 16;
  constexpr int APW = (AINS + NW - 1) / NW;
  const uint16_t* a_ptr[APW];
#pragma unroll
  for (int u = 0; u < APW; ++u) {
    int ins = wave + NW * u;
    ins = ins < AINS ? ins : AINS - 1;               // surplus waves repeat the last instruction
    int row = row0 + ins * 16 + (lane >> 2);
    row = row < B ? row : B - 1;
    a_ptr[u] = H + (int64_t)row * h_stride + 8 * ((lane & 3) ^ ((lane >> 4) & 3));
  }
  // packed W: operand block of column tile ct, step ks is 64 uint4 at (ct*KSu + ks)*64
  const uint4* b_ptr[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    int ct = ct0 + wn * TN + j;
    ct = ct < n_ct ? ct : n_ct - 1;                  // tiles beyond V: clamped, never stored
    b_ptr[j] = reinterpret_cast<const uint4*>(Wu) + (int64_t)ct * KSu * 64 + lane;
  }
  uint4 fb[kGemmBuffers][2][TN];                     // W operands of the stages in flight
  auto fetch = [&](int stage, uint4 (&b)[2][TN]) {
    uint4* sa = smem + (stage % kGemmBuffers) * SSLOTS;
#pragma unroll
    for (int u = 0; u < APW; ++u) {
      int ins = wave + NW * u;
      ins = ins < AINS ? ins : AINS - 1;
      load_block_to_lds(a_ptr[u] + (stage0 + stage) * 32, sa + ins * 64);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < TN; ++j) b[ks][j] = b_ptr[j][((stage0 + stage) * 2 + ks) * 64];
  };
  // LDS slot of this lane's A operand for row tile i, step ks: row = (wm*TM+i)*32 + lane%32,
  // chunk = 2*ks + lane/32, slot = row*4 + (chunk ^ (row/4)%4)
  int a_slot[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_slot[i] = ((wm * TM + i) * 32 + (lane & 31)) * 4;
  const int a_sw = (lane >> 2) & 3, a_hi = lane >> 5;
  constexpr int LOADS = APW + 2 * TN;                // loads per wave and stage
  // at most `newer` stages' worth of this wave's loads still in flight (they complete in order)
  auto wait_fetches = [&](int newer) {
    constexpr int L1 = LOADS < 15 ? LOADS : 15, L2 = 2 * LOADS < 63 ? 2 * LOADS : 63;
    if (newer >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | (L2 & 15) | ((L2 >> 4) << 14));
    else if (newer == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (L1 & 15) | ((L1 >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  };
  auto read_a = [&](int stage, int ks, bf16x8 (&fa)[TM]) {
    const uint4* sa = smem + (stage % kGemmBuffers) * SSLOTS;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      fa[i] = *reinterpret_cast<const bf16x8*>(&sa[a_slot[i] + ((2 * ks + a_hi) ^ a_sw)]);
  };
  auto multiply = [&](bf16x8 (&fa)[TM], uint4 (&b)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            fa[i], *reinterpret_cast<bf16x8*>(&b[j]), acc[i][j], 0, 0, 0);
  };

  // Software pipeline, unrolled over the four buffers so that every register set is addressed
  // statically.  The H operands of the next MFMA step are read from LDS while the current
  // step's MFMAs run.
#pragma unroll
  for (int p = 0; p < kGemmBuffers - 1; ++p)
    if (p < stages) fetch(p, fb[p]);
  bf16x8 fa0[TM], fa1[TM];
  {
    const int ahead = stages - 1;
    wait_fetches(ahead < kGemmBuffers - 2 ? ahead : kGemmBuffers - 2);
    __syncthreads();
    read_a(0, 0, fa0);
  }
  for (int base = 0; base < stages; base += kGemmBuffers) {
#pragma unroll
    for (int q = 0; q < kGemmBuffers; ++q) {
      const int stage = base + q;
      if (stage < stages) {
        read_a(stage, 1, fa1);
        multiply(fa0, fb[q][0]);
        if (stage + 1 < stages) {
          const int ahead = stages - 2 - stage;      // fetched stages after stage+1
          wait_fetches(ahead < kGemmBuffers - 3 ? ahead : kGemmBuffers - 3);
          __syncthreads();  // stage+1 has landed everywhere; the buffer of stage-1 is free everywhere
          if (stage + kGemmBuffers - 1 < stages)
            fetch(stage + kGemmBuffers - 1, fb[(q + kGemmBuffers - 1) % kGemmBuffers]);
          read_a(stage + 1, 0, fa0);
        }
        multiply(fa1, fb[q][1]);
      }
    }
  }
  if constexpr (KSPLIT > 1) {
    // partial results of the groups 1.. -> LDS (over the H buffers, which nobody reads any more),
    // group 0 adds them to its own
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem_all);
    constexpr int PER_WAVE = TM * TN * 16 * 64;
    if (ksplit > 0) {
      float* mine = red + ((ksplit - 1) * NW + wave) * PER_WAVE;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) mine[((i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
    }
    __syncthreads();
    if (ksplit > 0) return;
#pragma unroll
    for (int g = 1; g < KSPLIT; ++g) {
      const float* theirs = red + ((g - 1) * NW + wave) * PER_WAVE;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] += theirs[((i * TN + j) * 16 + r) * 64 + lane];
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = (ct0 + wn * TN + j) * 32 + (lane & 31);
      if (col >= V) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < B) A[(int64_t)row * V + col] = acc[i][j][r];
      }
    }
}

template <int NWM, int NWN, int TM, int TN, int KSPLIT = 1>
__global__ __launch_bounds__(64 * NWM * NWN * KSPLIT, 1) void user_gemm_bf16_kernel(
    const uint16_t* __restrict__ H, int64_t h_stride, const uint16_t* __restrict__ Wu,
    float* __restrict__ A, int B, int d, int V, int tiles_n, int tiles_total) {
  user_gemm_tile<NWM, NWN, TM, TN, KSPLIT>(H, h_stride, Wu, A, B, d, V, tiles_n, tiles_total,
                                           blockIdx.x);
}

// Several levels' projections in one launch: they do not depend on each other (all the hidden
// states come out of the same prefill), so the level loop need not pay for them one by one.
struct GemmGroup {
  const uint16_t* H[NEZHA_MAX_LEVELS];
  const uint16_t* Wu[NEZHA_MAX_LEVELS];
  float* A[NEZHA_MAX_LEVELS];
  int V[NEZHA_MAX_LEVELS];
  int tiles_n[NEZHA_MAX_LEVELS];
  int tile_begin[NEZHA_MAX_LEVELS + 1];
  int n;
};
template <int NWM, int NWN, int TM, int TN, int KSPLIT>
__global__ __launch_bounds__(64 * NWM * NWN * KSPLIT, 1) void user_gemm_bf16_grouped_kernel(
    GemmGroup grp, int64_t h_stride, int B, int d) {
  int p = 0;
  while (p + 1 < grp.n && (int)blockIdx.x >= grp.tile_begin[p + 1]) ++p;
  // an odd tile count defeats the XCD remapping inside, which is what small problems want
  user_gemm_tile<NWM, NWN, TM, TN, KSPLIT>(grp.H[p], h_stride, grp.Wu[p], grp.A[p], B, d, grp.V[p],
                                           grp.tiles_n[p], 1, (int)blockIdx.x - grp.tile_begin[p]);
}

// ---- the largest products: 256 x 256 tiles, both operands through LDS ------------------------------
// Four waves (2 x 2), each 128 x 128 = 4 x 4 accumulator tiles of 32 x 32 (256 accumulator
// registers, one wave per SIMD: the tile shape that moves the fewest LDS and L2 bytes per flop).
// A stage is 32 k: the H tile (256 rows x 64 B, XOR-swizzled as above) and the packed W tile (16
// operand blocks of 1 KiB) are brought by global_load_lds into one of four 32 KiB buffers, and
// stage s+4 is requested as soon as the barrier of iteration s has shown that every wave is done
// with buffer s: three stages are in flight while a wave waits for the next one.  The instruction
// order inside an iteration is pinned (scheduling groups): the LDS operand reads of the next MFMA
// step go out under the first MFMAs of the current one, the barrier sits behind eight MFMAs, and
// the eight fetch instructions are spread one per MFMA, so that the matrix pipe is not left idle
// while the wave issues memory instructions (in-kernel clock reads: 39 cycles per MFMA against 33.6
// for a loop of MFMAs alone).
// The product is accumulated TRANSPOSED (W fragment as the first MFMA operand): a lane then holds
// four consecutive output columns of one row per accumulator quad and writes them as one 16-byte
// store (64 store instructions per wave instead of 256).
constexpr int kBigSlotsA = 1024, kBigSlotsStage = 2048;   // 16-byte slots: H tile, H + W tiles
__host__ __device__ constexpr size_t big_gemm_lds() {
  return (size_t)kGemmBuffers * kBigSlotsStage * sizeof(uint4);
}
__device__ __forceinline__ void user_gemm_big_tile(
    const uint16_t* __restrict__ H, int64_t h_stride, const uint16_t* __restrict__ Wu,
    float* __restrict__ A, int B, int d, int V, int tiles_n, int tiles_total, int tile_id) {
  typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
  typedef float float4v __attribute__((ext_vector_type(4)));
  extern __shared__ __align__(16) uint4 smem_all[];
  uint4* const smem = smem_all;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  {
    // (the same XCD-aware order as user_gemm_tile)
    const int t = tile_id, xcd = t & 7, local = t >> 3;
    if (tiles_total % 256 == 0 && tiles_n % 8 == 0 && (tiles_total / tiles_n) % 4 == 0) {
      const int group = xcd + 8 * (local >> 5), groups_n = tiles_n >> 3;
      tile_m = (group / groups_n) * 4 + ((local & 31) >> 3);
      tile_n = (group % groups_n) * 8 + (local & 7);
    } else {
      const int per_xcd = tiles_total / 8;
      const int lin = (per_xcd * 8 == tiles_total) ? xcd * per_xcd + local : t;
      tile_m = lin / tiles_n;
      tile_n = lin - tile_m * tiles_n;
    }
  }
  const int row0 = tile_m * 256, ct0 = tile_n * 8;
  const int n_ct = (V + 31) / 32;
  const int KSu = d / 16;
  const int stages = d / 32;

  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Wave w issues H fetch instructions w, w+4, w+8, w+12 (16 rows x 64 B each) and W operand
  // blocks w, w+4, w+8, w+12 of the stage's 16 (block 2*jb + ks: column tile jb, MFMA step ks).
  // Rows beyond B and column tiles beyond T_l are clamped (their results are never stored).
  const uint16_t* a_ptr[4];
  const uint4* b_ptr[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int ins = wave + 4 * u;
    int row = row0 + ins * 16 + (lane >> 2);
    row = row < B ? row : B - 1;
    a_ptr[u] = H + (int64_t)row * h_stride + 8 * ((lane & 3) ^ ((lane >> 4) & 3));
    int ct = ct0 + (ins >> 1);
    ct = ct < n_ct ? ct : n_ct - 1;
    b_ptr[u] = reinterpret_cast<const uint4*>(Wu) + ((int64_t)ct * KSu + (ins & 1)) * 64 + lane;
  }
  auto fetch = [&](int stage) {
    uint4* sa = smem + (stage & (kGemmBuffers - 1)) * kBigSlotsStage;
#pragma unroll
    for (int u = 0; u < 4; ++u) load_block_to_lds(a_ptr[u] + stage * 32, sa + (wave + 4 * u) * 64);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      load_block_to_lds(b_ptr[u] + (int64_t)stage * 128, sa + kBigSlotsA + (wave + 4 * u) * 64);
  };
  int a_slot[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) a_slot[i] = ((wm * 4 + i) * 32 + (lane & 31)) * 4;
  const int a_sw = (lane >> 2) & 3, a_hi = lane >> 5;
  auto read_a = [&](int stage, int ks, bf16x8 (&fa)[4]) {
    const uint4* sa = smem + (stage & (kGemmBuffers - 1)) * kBigSlotsStage;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      fa[i] = *reinterpret_cast<const bf16x8*>(&sa[a_slot[i] + ((2 * ks + a_hi) ^ a_sw)]);
  };
  auto read_b = [&](int stage, int ks, bf16x8 (&fb)[4]) {
    const uint4* sb = smem + (stage & (kGemmBuffers - 1)) * kBigSlotsStage + kBigSlotsA;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      fb[j] = *reinterpret_cast<const bf16x8*>(&sb[(2 * (wn * 4 + j) + ks) * 64 + lane]);
  };
  auto mm = [&](bf16x8 (&fa)[4], bf16x8 (&fb)[4], int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  };
  constexpr int kMfma = 0x008, kVmemRead = 0x020, kDsRead = 0x100;   // scheduling group masks

  fetch(0);
  if (stages > 1) fetch(1);
  if (stages > 2) fetch(2);
  if (stages > 3) fetch(3);
  bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];
  // stage 0 has landed: at most the 24 loads of stages 1..3 are still in flight
  if (stages > 3) __builtin_amdgcn_s_waitcnt(0x0F70 | (24 & 15) | ((24 >> 4) << 14));
  else __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  read_a(0, 0, fa0);
  read_b(0, 0, fb0);
  auto iteration = [&](int s, auto fetch_c, auto drain_c) {
    constexpr bool FETCH = decltype(fetch_c)::value;     // s + 4 < stages: stage s+4 is requested
    constexpr bool DRAIN = decltype(drain_c)::value;     // s + 3 >= stages: nothing newer in flight
    // first half of MFMA step (s, 0); the operands of step (s, 1) go out under its first MFMAs
    read_a(s, 1, fa1);
    read_b(s, 1, fb1);
    mm(fa0, fb0, 0, 2);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kDsRead, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(kMfma, 4, 0);
    __builtin_amdgcn_sched_barrier(0);
    // this wave's part of stage s+1 has landed (its loads complete in order: 16 newer ones may
    // be in flight) and its reads of buffer s are complete; then everybody's
    if (DRAIN) __builtin_amdgcn_s_waitcnt(0x0070);
    else __builtin_amdgcn_s_waitcnt(0x0070 | (16 & 15) | ((16 >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (FETCH) fetch(s + 4);                             // buffer s is free now
    mm(fa0, fb0, 2, 4);
    read_a(s + 1, 0, fa0);
    read_b(s + 1, 0, fb0);
    mm(fa1, fb1, 0, 4);
    if (FETCH) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kVmemRead, 1, 0);
      }
    } else {
      __builtin_amdgcn_sched_group_barrier(kMfma, 8, 0);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kDsRead, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(kMfma, 12, 0);
  };
  int s = 0;
  for (; s + 4 < stages; ++s) iteration(s, std::true_type{}, std::false_type{});
  for (; s + 3 < stages; ++s) iteration(s, std::false_type{}, std::false_type{});
  for (; s + 1 < stages; ++s) iteration(s, std::false_type{}, std::true_type{});
  read_a(s, 1, fa1);                                     // the last stage
  read_b(s, 1, fb1);
  mm(fa0, fb0, 0, 4);
  mm(fa1, fb1, 0, 4);
  // register 4q + t of lane l: row l%32 of row tile i, column 8q + 4*(l/32) + t of column tile j
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = row0 + (wm * 4 + i) * 32 + (lane & 31);
    if (row >= B) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int colb = (ct0 + wn * 4 + j) * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = colb + 8 * q;                    // T_l is a multiple of 16: all four or none
        if (col < V)
          *reinterpret_cast<float4v*>(A + (int64_t)row * V + col) = float4v{
              acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
      }
    }
  }
}

__global__ __launch_bounds__(256, 1) void user_gemm_big_kernel(
    const uint16_t* __restrict__ H, int64_t h_stride, const uint16_t* __restrict__ Wu,
    float* __restrict__ A, int B, int d, int V, int tiles_n, int tiles_total) {
  user_gemm_big_tile(H, h_stride, Wu, A, B, d, V, tiles_n, tiles_total, blockIdx.x);
}
// All levels' tiles in one launch: a CU takes its next tile as soon as the waves of the one before
// have issued their result stores, so the 4 * B * T_l bytes of one level drain to memory under the
// next level's k loop instead of at the end of a launch of their own.
__global__ __launch_bounds__(256, 1) void user_gemm_big_grouped_kernel(GemmGroup grp,
                                                                       int64_t h_stride, int B,
                                                                       int d) {
  int p = 0;
  while (p + 1 < grp.n && (int)blockIdx.x >= grp.tile_begin[p + 1]) ++p;
  user_gemm_big_tile(grp.H[p], h_stride, grp.Wu[p], grp.A[p], B, d, grp.V[p], grp.tiles_n[p],
                     grp.tile_begin[p + 1] - grp.tile_begin[p], (int)blockIdx.x - grp.tile_begin[p]);
}

// Measurement aid for the projection's roofline: the loop of user_gemm_big_tile with everything but
// its MFMAs taken out (one wave per SIMD, 32 independent 32x32x16 bf16 MFMAs per iteration on
// operand values read from the caller's buffer), timed from inside with the core-clock counter and
// the constant 100 MHz counter.  The chip lowers its clock under matrix load by an amount that
// depends on the operand values (all-zero operands run faster than random ones), so the product
// of unit count and nominal clock is not what a projection on real values can reach; this gives
// the rate that is sustained with the values at hand, and the clock it runs at.
__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(const uint4* __restrict__ operands,
                                                           int n_vec, int iters,
                                                           unsigned long long* __restrict__ ticks,
                                                           float* __restrict__ sink) {
  typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
  const int tid = threadIdx.x;
  bf16x8 fa[2][4], fb[2][4];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 x = operands[(int)(((unsigned)blockIdx.x * 2048u + (h * 8 + i) * 256 + tid) % (unsigned)n_vec)];
      const uint4 y = operands[(int)(((unsigned)blockIdx.x * 2048u + (h * 8 + 4 + i) * 256 + tid) % (unsigned)n_vec)];
      fa[h][i] = *reinterpret_cast<const bf16x8*>(&x);
      fb[h][i] = *reinterpret_cast<const bf16x8*>(&y);
    }
  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  __syncthreads();
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[h][j], fa[h][i], acc[i][j], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) t += acc[i][j][r];
  if (t == 123.456f) sink[0] = t;                        // keeps every accumulator alive
  if (tid == 0) {
    ticks[2 * blockIdx.x] = c1 - c0;
    ticks[2 * blockIdx.x + 1] = r1 - r0;
  }
}

// Measurement aid for the per-request expansion's roofline: one "tile step" of its first sweep as
// a wave issues it, without the LDS traffic: four dependent 16x16x32 bf16 MFMAs (one logit tile at
// e = 128) and the vector work on the tile before (per lane four logits: fused multiply-add,
// exponential, addition; two conversions to packed halves, two packed maxima; three moves for the
// accumulator's start value), the pieces issued between the MFMAs as the kernel does.  MODE 0:
// the MFMAs alone, 1: the vector work alone, 2: both.  Matrix and vector instructions of a SIMD
// overlap only in part on this chip, so neither unit's peak bounds such a loop; the rate of mode 2
// at the kernel's occupancy is the bound that the kernel's tile rate is compared with.
template <int MODE>
__global__ __launch_bounds__(256) void tile_step_kernel(const float* __restrict__ values, int iters,
                                                        unsigned long long* __restrict__ ticks,
                                                        float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 fa[4], fb[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      fa[ks][j] = (__bf16)values[(lane * 7 + ks * 8 + j) & 255];
      fb[ks][j] = (__bf16)values[(lane * 3 + ks * 8 + j + 64) & 255];
    }
  }
  float a0 = values[lane], nml[4], ssum[4] = {0.f, 0.f, 0.f, 0.f};
  uint32_t gmax[2] = {0xFC00FC00u, 0xFC00FC00u};
  floatx4 prev = floatx4{values[lane + 1], values[lane + 2], values[lane + 3], values[lane + 4]};
#pragma unroll
  for (int i = 0; i < 4; ++i) nml[i] = -(prev[i] + 20.f) * kLog2e;
  __syncthreads();
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
    floatx4 t = floatx4{a0, a0, a0, a0};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if constexpr (MODE != 1) {
        t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ks], fb[ks], t, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (MODE != 0) {
        const float z = prev[ks];
        if ((ks & 1) == 0)
          gmax[ks >> 1] = max_of_half_pairs(gmax[ks >> 1], pack_halves_rtz(z, prev[ks + 1]));
        ssum[ks] += __builtin_amdgcn_exp2f(fmaf(z, kLog2e, nml[ks]));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (MODE != 1) prev = t;
    else asm volatile("" : "+v"(prev));       // the vector work stays in the loop
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  const float r = prev[0] + prev[1] + prev[2] + prev[3] + ssum[0] + ssum[1] + ssum[2] + ssum[3] +
                  __uint_as_float(gmax[0] ^ gmax[1]);
  if (r == 12345.678f) *sink = r;
  if (threadIdx.x == 0) {
    ticks[2 * blockIdx.x] = c1 - c0;
    ticks[2 * blockIdx.x + 1] = r1 - r0;
  }
}

// ---- user-part projection, fp32 (small correctness-first shapes) -----------------------------
__global__ __launch_bounds__(256) void user_gemm_f32_kernel(const float* __restrict__ H,
                                                            int64_t h_stride,
                                                            const float* __restrict__ W,
                                                            float* __restrict__ A, int B, int d,
                                                            int V) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (v >= V || b >= B) return;
  const float* h = H + (int64_t)b * h_stride;
  float s = 0.f;
  for (int i = 0; i < d; ++i) s = fmaf(h[i], W[(int64_t)i * V + v], s);
  A[(int64_t)b * V + v] = s;
}

// ---- beam-part projection + log-softmax + per-beam top-K --------------------------------------
struct ExpandArgs {
  const void* state;     // [rows, e] or NULL (level 1: the state is zero)
  const void* Wbeam;     // bf16: packed beam part of W; f32: row-major W (whole matrix)
  const float* A;        // [B, V] user part
  int32_t* cand_code;    // [rows, K]
  float* cand_logp;      // [rows, K]
  int rows;              // B * K_in
  int K_in, K, V, d, e;
  const uint8_t* redo;   // expand_chunked_kernel: only rows with redo[row] != 0 (NULL: every row)
};

// A workgroup of NW waves owns 16 beams (rows); wave w takes the blocks of 64 codes
// w, w+NW, ...  For each block the wave forms the 16x64 logits in four 16x16 MFMA
// accumulators (initialised with the user part), updates every row's running (max, sum of
// exponentials) and appends the logits above the row's current threshold to the row's LDS
// buffer.  Buffers are cut back to the K best by a sort when they run short of room, which
// raises the threshold.  Register i of lane l belongs to row 4*(l/16)+i and code column l%16
// of the tile.  With NW > 1 the waves' per-row lists are merged at the end (NW*K <= CAP).
// KST: compile-time bound on the number of MFMA steps over e (bf16: e/32, f32: e/4).
template <bool BF16, int CAP, int KST, int NW>
__global__ __launch_bounds__(64 * NW) void expand_kernel(ExpandArgs a) {
  extern __shared__ __align__(16) uint64_t lds[];
  uint64_t* buf_all = lds;                                            // [NW][16][CAP]
  float* part_m = reinterpret_cast<float*>(lds + NW * 16 * CAP);      // [NW][16]
  float* part_s = part_m + NW * 16;                                   // [NW][16]
  int* part_cnt = reinterpret_cast<int*>(part_s + NW * 16);           // [NW][16]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, c = lane & 15;
  const int R0 = blockIdx.x * 16;
  const int V = a.V, K = a.K, e = a.e;
  const bool has_beam = a.state != nullptr;
  const int KS = BF16 ? e / 32 : e / 4;
  uint64_t* buf = buf_all + wave * 16 * CAP;

  // A operands of the MFMA: this lane's row is R0 + c
  bf16x8 fa16[BF16 ? KST : 1];
  float fa32[BF16 ? 1 : KST];
  if (has_beam) {
    const int row = R0 + c;
    if constexpr (BF16) {
      const uint16_t* st = static_cast<const uint16_t*>(a.state);
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) {
        uint4 v = uint4{0, 0, 0, 0};
        if (ks < KS && row < a.rows)
          v = *reinterpret_cast<const uint4*>(st + (int64_t)row * e + ks * 32 + 8 * g);
        fa16[ks] = *reinterpret_cast<bf16x8*>(&v);
      }
    } else {
      const float* st = static_cast<const float*>(a.state);
#pragma unroll
      for (int ks = 0; ks < KST; ++ks)
        fa32[ks] = (ks < KS && row < a.rows) ? st[(int64_t)row * e + ks * 4 + g] : 0.f;
    }
  }

  // per-row state, replicated over the 16 lanes of a group: rows 4g+i
  float tau[4], m[4], s[4];
  int cnt[4];
  int64_t a_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = R0 + 4 * g + i;
    const bool ok = row < a.rows;
    tau[i] = ok ? -INFINITY : INFINITY;
    m[i] = -INFINITY;
    s[i] = 0.f;
    cnt[i] = 0;
    a_off[i] = (int64_t)((ok ? row : 0) / a.K_in) * V;
  }
  constexpr int lim = CAP - 64;
  const int n_ct = V / 16;
  const int n_blk = (n_ct + 3) / 4;

  // operands of one block of 64 codes: the user part (accumulator start values) and, for
  // bf16, the packed B operands, fetched one block ahead of their use
  float aq[4][4];
  uint4 bq[4][BF16 ? KST : 1];
  auto fetch = [&](int blk) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int ct = blk * 4 + t;
      if (ct < n_ct) {
#pragma unroll
        for (int i = 0; i < 4; ++i) aq[t][i] = a.A[a_off[i] + ct * 16 + c];
        if constexpr (BF16) {
          if (has_beam) {
            const uint4* wp = static_cast<const uint4*>(a.Wbeam) + (int64_t)ct * KS * 64 + lane;
#pragma unroll
            for (int ks = 0; ks < KST; ++ks)
              if (ks < KS) bq[t][ks] = wp[ks * 64];
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) aq[t][i] = -INFINITY;
      }
    }
  };
  auto project = [&](int blk, floatx4 (&acc)[4]) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      acc[t] = floatx4{aq[t][0], aq[t][1], aq[t][2], aq[t][3]};
      const int ct = blk * 4 + t;
      if (has_beam && ct < n_ct) {
        if constexpr (BF16) {
#pragma unroll
          for (int ks = 0; ks < KST; ++ks)
            if (ks < KS)
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  fa16[ks], *reinterpret_cast<bf16x8*>(&bq[t][ks]), acc[t], 0, 0, 0);
        } else {
          const float* w = static_cast<const float*>(a.Wbeam) + (int64_t)a.d * V + ct * 16 + c;
#pragma unroll
          for (int ks = 0; ks < KST; ++ks)
            if (ks < KS)
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                  fa32[ks], w[(int64_t)(ks * 4 + g) * V], acc[t], 0, 0, 0);
        }
      }
    }
  };

  floatx4 acc[4], acc_next[4];
  int blk = wave;
  if (blk < n_blk) {
    fetch(blk);
    project(blk, acc);
    if (blk + NW < n_blk) fetch(blk + NW);
  }
  for (; blk < n_blk; blk += NW) {
    if (blk + NW < n_blk) {
      project(blk + NW, acc_next);                 // MFMAs run while the block below is scanned
      if (blk + 2 * NW < n_blk) fetch(blk + 2 * NW);
    }
    // running log-sum-exp, one (max, sum) pair per lane and row
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float mx = fmaxf(fmaxf(acc[0][i], acc[1][i]), fmaxf(acc[2][i], acc[3][i]));
      const float mn = fmaxf(m[i], mx);
      float sum = s[i] * __builtin_amdgcn_exp2f((m[i] - mn) * kLog2e);
#pragma unroll
      for (int t = 0; t < 4; ++t) sum += __builtin_amdgcn_exp2f((acc[t][i] - mn) * kLog2e);
      s[i] = sum;
      m[i] = mn;
    }
    // threshold filter and append
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float z = acc[t][i];
        const bool pass = z > tau[i];
        const uint64_t bal = __ballot(pass);
        if (bal) {
          const uint32_t grp = (uint32_t)(bal >> (16 * g)) & 0xFFFFu;
          const int pos = cnt[i] + __popc(grp & ((1u << c) - 1u));
          if (pass) {
            const uint32_t code = (uint32_t)((blk * 4 + t) * 16 + c);
            buf[(4 * g + i) * CAP + pos] = ((uint64_t)ordered_bits(z) << 32) | (uint32_t)~code;
          }
          cnt[i] += __popc(grp);
        }
      }
    }
    // rows that could overflow on the next block are cut back to their K best, four rows
    // (one accumulator register index) at a time
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (__ballot(cnt[i] > lim)) {
        uint64_t* const rows[4] = {buf + (0 + i) * CAP, buf + (4 + i) * CAP, buf + (8 + i) * CAP,
                                   buf + (12 + i) * CAP};
        int rc[4] = {__builtin_amdgcn_readlane(cnt[i], 0), __builtin_amdgcn_readlane(cnt[i], 16),
                     __builtin_amdgcn_readlane(cnt[i], 32), __builtin_amdgcn_readlane(cnt[i], 48)};
        uint64_t rt[4];
        compact_rows<CAP, 4>(rows, rc, rt, K);
        const int my_cnt = g == 0 ? rc[0] : g == 1 ? rc[1] : g == 2 ? rc[2] : rc[3];
        const uint64_t my_tau = g == 0 ? rt[0] : g == 1 ? rt[1] : g == 2 ? rt[2] : rt[3];
        cnt[i] = my_cnt;
        if (tau[i] != INFINITY)
          tau[i] = (my_cnt == K) ? unordered_bits((uint32_t)(my_tau >> 32)) : -INFINITY;
      }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = acc_next[t];
  }

  // this wave's (max, sum) of each row: merge the 16 lanes of every group
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float mm = m[i], ss = s[i];
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
      const float om = __shfl_xor(mm, off);
      const float os = __shfl_xor(ss, off);
      const float mn = fmaxf(mm, om);
      const float wa = (mm == mn) ? 1.f : __builtin_amdgcn_exp2f((mm - mn) * kLog2e);
      const float wb = (om == mn) ? 1.f : __builtin_amdgcn_exp2f((om - mn) * kLog2e);
      ss = ss * wa + os * wb;
      mm = mn;
    }
    if (c == 0) {
      part_m[wave * 16 + 4 * g + i] = mm;
      part_s[wave * 16 + 4 * g + i] = ss;
      part_cnt[wave * 16 + 4 * g + i] = cnt[i];
    }
  }
  wave_sync();
  // final cut of this wave's 16 rows: sorted K best at the front of each buffer
  for (int r0 = 0; r0 < 16; r0 += 4) {
    uint64_t* const rows[4] = {buf + r0 * CAP, buf + (r0 + 1) * CAP, buf + (r0 + 2) * CAP,
                               buf + (r0 + 3) * CAP};
    int rc[4];
    uint64_t rt[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
      rc[r] = __builtin_amdgcn_readfirstlane(part_cnt[wave * 16 + r0 + r]);
    compact_rows<CAP, 4>(rows, rc, rt, K);
    if (lane == 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) part_cnt[wave * 16 + r0 + r] = rc[r];
    }
  }
  if constexpr (NW == 1) {
    wave_sync();
    for (int r = 0; r < 16; ++r) {
      const int row = R0 + r;
      if (row >= a.rows) break;
      const float lse = part_m[r] + __builtin_amdgcn_logf(part_s[r]) * kLn2;
      const int n = part_cnt[r];
      for (int p = lane; p < n; p += 64) {
        const uint64_t key = buf[r * CAP + p];
        a.cand_code[(int64_t)row * K + p] = (int32_t)(~(uint32_t)key);
        a.cand_logp[(int64_t)row * K + p] = unordered_bits((uint32_t)(key >> 32)) - lse;
      }
    }
  } else {
    __syncthreads();
    // wave w merges rows w*RPW .. : every row's NW sorted lists (at most NW*K <= CAP keys)
    constexpr int RPW = 16 / NW;
    constexpr int NPL = CAP / 64;
    static_assert(RPW >= 1 && RPW <= 4, "rows per wave in the merge");
    uint64_t key[RPW][NPL];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
      const int lr = wave * RPW + r;
#pragma unroll
      for (int j = 0; j < NPL; ++j) {
        const int el = j * 64 + lane;
        const int w = el / K, idx = el - w * K;
        key[r][j] = (w < NW && idx < part_cnt[w * 16 + lr]) ? buf_all[(w * 16 + lr) * CAP + idx]
                                                            : 0ull;
      }
    }
    sort_desc<NPL, RPW>(key);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
      const int lr = wave * RPW + r, row = R0 + lr;
      if (row < a.rows) {
        float mm = part_m[lr], ss = part_s[lr];
        int total = part_cnt[lr];
#pragma unroll
        for (int w = 1; w < NW; ++w) {
          const float om = part_m[w * 16 + lr], os = part_s[w * 16 + lr];
          const float mn = fmaxf(mm, om);
          const float wa = (mm == mn) ? 1.f : __builtin_amdgcn_exp2f((mm - mn) * kLog2e);
          const float wb = (om == mn) ? 1.f : __builtin_amdgcn_exp2f((om - mn) * kLog2e);
          ss = ss * wa + os * wb;
          mm = mn;
          total += part_cnt[w * 16 + lr];
        }
        const float lse = mm + __builtin_amdgcn_logf(ss) * kLn2;
        const int n = total < K ? total : K;
#pragma unroll
        for (int j = 0; j < NPL; ++j) {
          const int p = lane * NPL + j;
          if (p < n) {
            a.cand_code[(int64_t)row * K + p] = (int32_t)(~(uint32_t)key[r][j]);
            a.cand_logp[(int64_t)row * K + p] =
                unordered_bits((uint32_t)(key[r][j] >> 32)) - lse;
          }
        }
      }
    }
  }
}

// Element j (wave uniform, 0 <= j < N) of a small register array, without indexing it.
template <int N>
__device__ __forceinline__ uint32_t pick_element(const uint32_t (&v)[N], int j) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8, "1, 2, 4 or 8 elements");
  if constexpr (N == 1) {
    return v[0];
  } else if constexpr (N == 2) {
    return v[0] ^ ((v[0] ^ v[1]) & (0u - (uint32_t)(j & 1)));
  } else if constexpr (N == 4) {
    const uint32_t m1 = 0u - (uint32_t)(j & 1), m2 = 0u - (uint32_t)((j >> 1) & 1);
    const uint32_t lo = v[0] ^ ((v[0] ^ v[1]) & m1), hi = v[2] ^ ((v[2] ^ v[3]) & m1);
    return lo ^ ((lo ^ hi) & m2);
  } else {
    const uint32_t a[4] = {v[0], v[1], v[2], v[3]}, b[4] = {v[4], v[5], v[6], v[7]};
    const uint32_t lo = pick_element<4>(a, j & 3), hi = pick_element<4>(b, j & 3);
    return lo ^ ((lo ^ hi) & (0u - (uint32_t)((j >> 2) & 1)));
  }
}
// Two rows of float32 logits in LDS (T_l = V values each, V/64 per lane): log-sum-exp and the K
// best (logit, code) keys of each, handed to emit(row 0|1, place, key, lse) in code order (not
// sorted by logit: what follows orders equal scores by parent and code, so the place of a
// candidate inside its beam's list only has to respect the code order of equal logits).  All
// sorting is on the 32-bit ordered logits alone.  The K-th largest of the 64 per-lane maxima is
// a lower bound of the row's K-th largest logit, so only the few logits at or above it are
// appended, in code order, to the wave's LDS list (scratch, CAP keys, half per row); a sort of
// those gives the K-th largest logit itself, and the entries above it plus the first (lowest
// code) of its ties are the K best.  The two rows run side by side: independent work hides the
// cross-lane latency.  K <= 64.  Whole wave.
template <int NVT, int CAP, class Emit>
__device__ __forceinline__ void two_rows_topk(const float* z0, const float* z1, bool live0,
                                              bool live1, int V, int K, uint64_t* scratch,
                                              Emit emit) {
  const int lane = threadIdx.x & 63;
  const int NV = (V + 63) / 64;
  const float* zrow[2] = {z0, z1};
  bool live[2] = {live0, live1};
  float zv[2][NVT], m[2], ssum[2];
  uint32_t zk[2][NVT], best[2][1];
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    m[rr] = -INFINITY;
#pragma unroll
    for (int j = 0; j < NVT; ++j) {
      const int col = j * 64 + lane;
      zv[rr][j] = (j < NV && col < V && live[rr]) ? zrow[rr][col] : -INFINITY;
      m[rr] = fmaxf(m[rr], zv[rr][j]);
    }
  }
  auto reduce_max = [&](float (&x)[2]) {
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      float v = x[rr];
      v = fmaxf(v, __uint_as_float(lane_xor<1>(__float_as_uint(v), lane)));
      v = fmaxf(v, __uint_as_float(lane_xor<2>(__float_as_uint(v), lane)));
      v = fmaxf(v, __uint_as_float(lane_xor<4>(__float_as_uint(v), lane)));
      v = fmaxf(v, __uint_as_float(lane_xor<8>(__float_as_uint(v), lane)));
      v = fmaxf(v, __uint_as_float(lane_xor<16>(__float_as_uint(v), lane)));
      v = fmaxf(v, __uint_as_float(lane_xor<32>(__float_as_uint(v), lane)));
      x[rr] = v;
    }
  };
  auto reduce_sum = [&](float (&x)[2]) {
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      float v = x[rr];
      v += __uint_as_float(lane_xor<1>(__float_as_uint(v), lane));
      v += __uint_as_float(lane_xor<2>(__float_as_uint(v), lane));
      v += __uint_as_float(lane_xor<4>(__float_as_uint(v), lane));
      v += __uint_as_float(lane_xor<8>(__float_as_uint(v), lane));
      v += __uint_as_float(lane_xor<16>(__float_as_uint(v), lane));
      v += __uint_as_float(lane_xor<32>(__float_as_uint(v), lane));
      x[rr] = v;
    }
  };
  reduce_max(m);
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    ssum[rr] = 0.f;
    best[rr][0] = 0;
#pragma unroll
    for (int j = 0; j < NVT; ++j) {
      const int col = j * 64 + lane;
      const bool ok = j < NV && col < V && live[rr];
      ssum[rr] += ok ? __builtin_amdgcn_exp2f((zv[rr][j] - m[rr]) * kLog2e) : 0.f;
      zk[rr][j] = ok ? ordered_bits(zv[rr][j]) : 0u;       // ordered bits of a finite logit are > 0
      best[rr][0] = zk[rr][j] > best[rr][0] ? zk[rr][j] : best[rr][0];
    }
  }
  reduce_sum(ssum);
  // K-th largest of the per-lane maxima: every one of the row's K best logits is >= it
  sort_desc<1, 2, uint32_t>(best);
  uint64_t* rows[2] = {scratch, scratch + CAP / 2};
  int rc[2];
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    const uint32_t bound = (uint32_t)__builtin_amdgcn_readlane((int)best[rr][0], K - 1);
    // append the logits >= bound in code order; a row gets CAP/2 places, which K * T_l/64 keys
    // could exceed only in contrived cases: then the row falls back to the streaming top-K below
    int cnt = 0;
    bool overflow = false;
#pragma unroll
    for (int j = 0; j < NVT; ++j) {
      if (j < NV) {
        const bool pass = zk[rr][j] >= bound && zk[rr][j] != 0;
        const uint64_t bal = __ballot(pass);
        const int pos = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
        const int n = __popcll(bal);
        if (cnt + n > CAP / 2) overflow = true;
        if (pass && pos < CAP / 2)
          rows[rr][pos] = ((uint64_t)zk[rr][j] << 32) | (uint32_t)~(uint32_t)(j * 64 + lane);
        cnt += n;
      }
    }
    rc[rr] = overflow ? -1 : cnt;
  }
  if (rc[0] < 0 || rc[1] < 0) {
    // rare: too many keys tie with the bound; redo both rows with the general streaming top-K
    for (int rr = 0; rr < 2; ++rr) {
      wave_sync();
      WaveTopK<CAP> q;
      q.init(scratch, K);
      for (int j = 0; j < NV; ++j) {                       // keys rebuilt from the LDS tile
        const int col = j * 64 + lane;
        const bool ok = col < V && live[rr];
        const float z = ok ? zrow[rr][col] : 0.f;
        q.push(ok ? (((uint64_t)ordered_bits(z) << 32) | (uint32_t)~(uint32_t)col) : 0ull);
      }
      q.compact();
      wave_sync();
      if (live[rr]) {
        const float lse = m[rr] + __builtin_amdgcn_logf(ssum[rr]) * kLn2;
        for (int p = lane; p < q.cnt; p += 64) emit(rr, p, q.buf[p], lse);
      }
    }
    return;
  }
  wave_sync();
  // the lists hold K .. CAP/2 entries each, in code order: find the K-th largest logit and keep
  // what is above it and the first of its ties
  auto select = [&](auto npl_c) {
    constexpr int NPL = decltype(npl_c)::value;
    uint64_t ent[2][NPL];
    uint32_t zz[2][NPL], sk[2][NPL];
#pragma unroll
    for (int rr = 0; rr < 2; ++rr)
#pragma unroll
      for (int j = 0; j < NPL; ++j) {
        const int idx = j * 64 + lane;
        ent[rr][j] = idx < rc[rr] ? rows[rr][idx] : 0ull;
        zz[rr][j] = (uint32_t)(ent[rr][j] >> 32);
        sk[rr][j] = zz[rr][j];
      }
    sort_desc<NPL, 2, uint32_t>(sk);                                    // position NPL*lane + j
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      if (!live[rr]) continue;
      const uint32_t tau = (uint32_t)__builtin_amdgcn_readlane(
          (int)pick_element<NPL>(sk[rr], (K - 1) % NPL), (K - 1) / NPL);
      int n_gt = 0;
#pragma unroll
      for (int j = 0; j < NPL; ++j) n_gt += __popcll(__ballot(zz[rr][j] > tau));
      const int need = K - n_gt;                                         // ties to take, in list order
      const float lse = m[rr] + __builtin_amdgcn_logf(ssum[rr]) * kLn2;
      int base = 0, ties = 0;
#pragma unroll
      for (int j = 0; j < NPL; ++j) {
        const bool eq = zz[rr][j] == tau;
        const uint64_t bal_eq = __ballot(eq);
        const int tie_rank = ties + __builtin_amdgcn_mbcnt_hi(
                                        (uint32_t)(bal_eq >> 32),
                                        __builtin_amdgcn_mbcnt_lo((uint32_t)bal_eq, 0));
        const bool take = zz[rr][j] > tau || (eq && tie_rank < need);
        const uint64_t bal = __ballot(take);
        const int p = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                       __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
        if (take) emit(rr, p, ent[rr][j], lse);
        base += __popcll(bal);
        ties += __popcll(bal_eq);
      }
    }
  };
  const int most = rc[0] > rc[1] ? rc[0] : rc[1];
  if (most <= 64) select(std::integral_constant<int, 1>{});
  else select(std::integral_constant<int, 2>{});
}

// ---- the same step for small codebooks (T_l <= 1024, K <= 64) ------------------------------------
// A workgroup of 8 waves owns 16 beams.  Phase A: the waves share out the 16-column MFMA tiles
// and write the 16 x T_l logits (float32) to LDS.  Phase B: every wave takes two rows; a row's
// logits sit T_l/64 per lane.  The K-th largest of the 64 per-lane maxima is a lower bound of the
// row's K-th largest logit, so only the few logits at or above it are appended to the wave's
// LDS list, which one small sort then cuts to the K best.  More waves work on fewer rows each
// than in expand_kernel, which is what a small batch needs.
template <int KST, int NVT>
__global__ __launch_bounds__(512, 1) void expand_small_kernel(ExpandArgs a) {
  extern __shared__ __align__(16) uint64_t lds[];
  constexpr int CAP = 256;
  uint64_t* scratch = lds;                                   // [8 waves][CAP]
  float* ztile = reinterpret_cast<float*>(lds + 8 * CAP);    // [16][V]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, c = lane & 15;
  const int R0 = blockIdx.x * 16;
  const int V = a.V, K = a.K, e = a.e;
  const bool has_beam = a.state != nullptr;
  const int KS = e / 32;
  const int n_ct = V / 16;

  {  // phase A
    bf16x8 fa16[KST];
    if (has_beam) {
      const int row = R0 + c;
      const uint16_t* st = static_cast<const uint16_t*>(a.state);
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) {
        uint4 v = uint4{0, 0, 0, 0};
        if (ks < KS && row < a.rows)
          v = *reinterpret_cast<const uint4*>(st + (int64_t)row * e + ks * 32 + 8 * g);
        fa16[ks] = *reinterpret_cast<bf16x8*>(&v);
      }
    }
    int64_t a_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = R0 + 4 * g + i;
      a_off[i] = (int64_t)((row < a.rows ? row : 0) / a.K_in) * V;
    }
    // two tiles (ct, ct + 8) per trip, all their loads issued before the first MFMA
    for (int ct = wave; ct < n_ct; ct += 16) {
      const bool two = ct + 8 < n_ct;
      const int ct2 = two ? ct + 8 : ct;
      floatx4 acc0, acc1;
      uint4 w0[KST], w1[KST];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc0[i] = a.A[a_off[i] + ct * 16 + c];
        acc1[i] = a.A[a_off[i] + ct2 * 16 + c];
      }
      if (has_beam) {
        const uint4* wp0 = static_cast<const uint4*>(a.Wbeam) + (int64_t)ct * KS * 64 + lane;
        const uint4* wp1 = static_cast<const uint4*>(a.Wbeam) + (int64_t)ct2 * KS * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
          if (ks < KS) {
            w0[ks] = wp0[ks * 64];
            w1[ks] = wp1[ks * 64];
          }
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
          if (ks < KS) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                fa16[ks], *reinterpret_cast<bf16x8*>(&w0[ks]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                fa16[ks], *reinterpret_cast<bf16x8*>(&w1[ks]), acc1, 0, 0, 0);
          }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ztile[(4 * g + i) * V + ct * 16 + c] = acc0[i];
        if (two) ztile[(4 * g + i) * V + ct2 * 16 + c] = acc1[i];
      }
    }
  }
  __syncthreads();

  // phase B: this wave's two rows side by side
  const int r0 = wave * 2;
  if (R0 + r0 >= a.rows) return;
  const bool live0 = true, live1 = R0 + r0 + 1 < a.rows;
  two_rows_topk<NVT, CAP>(ztile + r0 * V, ztile + (r0 + 1) * V, live0, live1, V, K,
                          scratch + wave * CAP, [&](int rr, int p, uint64_t kk, float lse) {
                            const int row = R0 + r0 + rr;
                            a.cand_code[(int64_t)row * K + p] = (int32_t)(~(uint32_t)kk);
                            a.cand_logp[(int64_t)row * K + p] =
                                unordered_bits((uint32_t)(kk >> 32)) - lse;
                          });
}

// ---- per-request merge, verification, pruning and state update ---------------------------------
struct MergeArgs {
  const int32_t* cand_code;
  const float* cand_logp;
  const uint64_t* key_in;   // [B, K_in] or NULL
  const float* score_in;    // [B, K_in] or NULL
  const void* state_in;     // [B, K_in, e] or NULL
  const void* E;            // [V, e] (used when state_out != NULL)
  SetView set;              // slots == NULL: no verification
  uint64_t mult;            // prod_{j<level} T_j
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  void* state_out;          // or NULL
  int32_t* count_out;       // or NULL
  int K_in, K, e;
  const void* U;            // [e, e] row major (recurrent Transition), else unused
  int transition;
  const uint8_t* redo_req;  // only requests with redo_req[b] != 0 (NULL: every request)
};

// Eq. 3 with the additive Transition for the K survivors of request b: c' = c_parent + E[code]
// (zero for unused slots); 8 (bf16) or 4 (f32) elements per thread and step.
// lds_in / lds_out (bf16 only, may be NULL): the parents' states [K_in, e] and a second copy of
// the new states [K, e] in LDS, for a caller that runs the next level in the same workgroup.
template <bool BF16>
__device__ __forceinline__ void update_states(const void* state_in, const void* E, void* state_out,
                                              int b, int K, int K_in, int e,
                                              const int32_t* fin_parent, const int32_t* fin_code,
                                              int tid, int nthreads,
                                              const uint16_t* lds_in = nullptr,
                                              uint16_t* lds_out = nullptr) {
  {
    const int per = e / (BF16 ? 8 : 4);
    for (int idx = tid; idx < K * per; idx += nthreads) {
      const int j = idx / per, t = idx - j * per;
      const int par = fin_parent[j], code = fin_code[j];
      if constexpr (BF16) {
        uint16_t* out = static_cast<uint16_t*>(state_out) + ((int64_t)b * K + j) * e + t * 8;
        uint4 r = uint4{0, 0, 0, 0};
        if (par >= 0) {
          const uint4 ev = load_global_u4(static_cast<const uint16_t*>(E) + (int64_t)code * e + t * 8);
          uint4 sv = uint4{0, 0, 0, 0};
          if (lds_in)
            sv = *reinterpret_cast<const uint4*>(lds_in + par * e + t * 8);
          else if (state_in)
            sv = load_global_u4(static_cast<const uint16_t*>(state_in) +
                                ((int64_t)b * K_in + par) * e + t * 8);
          const uint32_t ew[4] = {ev.x, ev.y, ev.z, ev.w}, sw[4] = {sv.x, sv.y, sv.z, sv.w};
          uint32_t ow[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float lo = bf16_to_float((uint16_t)ew[u]) + bf16_to_float((uint16_t)sw[u]);
            const float hi = bf16_to_float((uint16_t)(ew[u] >> 16)) +
                             bf16_to_float((uint16_t)(sw[u] >> 16));
            ow[u] = (uint32_t)float_to_bf16(lo) | ((uint32_t)float_to_bf16(hi) << 16);
          }
          r = uint4{ow[0], ow[1], ow[2], ow[3]};
        }
        store_global_u4(out, r);
        if (lds_out) *reinterpret_cast<uint4*>(lds_out + j * e + t * 8) = r;
      } else {
        float* out = static_cast<float*>(state_out) + ((int64_t)b * K + j) * e + t * 4;
        float4 r = float4{0.f, 0.f, 0.f, 0.f};
        if (par >= 0) {
          const float4 ev = *reinterpret_cast<const float4*>(static_cast<const float*>(E) +
                                                             (int64_t)code * e + t * 4);
          float4 sv = float4{0.f, 0.f, 0.f, 0.f};
          if (state_in)
            sv = *reinterpret_cast<const float4*>(static_cast<const float*>(state_in) +
                                                  ((int64_t)b * K_in + par) * e + t * 4);
          r = float4{ev.x + sv.x, ev.y + sv.y, ev.z + sv.z, ev.w + sv.w};
        }
        *reinterpret_cast<float4*>(out) = r;
      }
    }
  }
}

// Eq. 3 with the recurrent Transition for the K survivors of request b:
// c'[j] = tanh(sum_i U[j][i] c_parent[i] + E[code][j]) (zero for unused slots).  bf16: 16x16
// output tiles (16 survivors x 16 state elements) by v_mfma_f32_16x16x32_bf16, spread over the
// workgroup's waves; the accumulator starts at the code embedding; the A operand is the parent
// state row, the B operand B[k][n] = U[n][k] is 16 contiguous bytes of row n of U.
template <bool BF16>
__device__ __forceinline__ void update_states_rnn(const void* state_in, const void* E, const void* U,
                                                  void* state_out, int b, int K, int K_in, int e,
                                                  const int32_t* fin_parent,
                                                  const int32_t* fin_code, int tid, int nthreads,
                                                  const uint16_t* lds_in = nullptr,
                                                  uint16_t* lds_out = nullptr) {
  if constexpr (BF16) {
    const int lane = tid & 63, wave = tid >> 6, n_waves = nthreads >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int RT = (K + 15) / 16, CT = e / 16, KS = e / 32;
    const uint16_t* Eh = static_cast<const uint16_t*>(E);
    const uint16_t* Uh = static_cast<const uint16_t*>(U);
    const uint16_t* Sh = static_cast<const uint16_t*>(state_in);
    uint16_t* Oh = static_cast<uint16_t*>(state_out);
    for (int t = wave; t < RT * CT; t += n_waves) {
      const int rt = t / CT, ct = t - rt * CT;
      floatx4 acc;
      int code[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = rt * 16 + 4 * g + i;
        code[i] = j < K ? fin_code[j] : -1;
        acc[i] = code[i] >= 0 ? bf16_to_float(as_global(Eh)[(int64_t)code[i] * e + ct * 16 + c]) : 0.f;
      }
      const int ja = rt * 16 + c;
      const int pa = ja < K ? fin_parent[ja] : -1;
      if (Sh || lds_in) {
        for (int ks = 0; ks < KS; ++ks) {
          uint4 av = uint4{0, 0, 0, 0};
          if (pa >= 0) {
            if (lds_in)
              av = *reinterpret_cast<const uint4*>(lds_in + pa * e + ks * 32 + 8 * g);
            else
              av = load_global_u4(Sh + ((int64_t)b * K_in + pa) * e + ks * 32 + 8 * g);
          }
          const uint4 bv = load_global_u4(Uh + (int64_t)(ct * 16 + c) * e + ks * 32 + 8 * g);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8*>(&av),
                                                        *reinterpret_cast<const bf16x8*>(&bv), acc,
                                                        0, 0, 0);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = rt * 16 + 4 * g + i;
        if (j < K) {
          const uint16_t v = code[i] >= 0 ? float_to_bf16(tanhf(acc[i])) : (uint16_t)0;
          as_global(Oh)[((int64_t)b * K + j) * e + ct * 16 + c] = v;
          if (lds_out) lds_out[j * e + ct * 16 + c] = v;
        }
      }
    }
  } else {
    const float* Ef = static_cast<const float*>(E);
    const float* Uf = static_cast<const float*>(U);
    const float* Sf = static_cast<const float*>(state_in);
    float* Of = static_cast<float*>(state_out);
    for (int idx = tid; idx < K * e; idx += nthreads) {
      const int j = idx / e, col = idx - j * e;
      const int par = fin_parent[j], code = fin_code[j];
      float r = 0.f;
      if (par >= 0) {
        float acc = Ef[(int64_t)code * e + col];
        if (Sf) {
          const float* srow = Sf + ((int64_t)b * K_in + par) * e;
          const float* urow = Uf + (int64_t)col * e;
          for (int i = 0; i < e; ++i) acc = fmaf(urow[i], srow[i], acc);
        }
        r = tanhf(acc);
      }
      Of[((int64_t)b * K + j) * e + col] = r;
    }
  }
}

// One workgroup (4 or 16 waves) per request.  Every candidate (parent p, within-beam rank r) gets
// the sort key (ordered score, ~(p*K+r)), or 0 if the verifier rejects it; all keys go to LDS.
// Each lane remembers its two largest keys; the K-th largest of a wave's lane maxima bounds the
// request's K-th largest key from below, so wave 0 then only has to sort the few keys at or above
// the best of the waves' bounds.  The keys fill most of a CU's LDS for large K_in * K, so the
// hash-set probes in flight are what the workgroup's own waves issue: 16 waves then.
constexpr int kMergeMaxWaves = 16;
template <bool BF16>
__global__ __launch_bounds__(64 * kMergeMaxWaves) void merge_kernel(MergeArgs a) {
  constexpr int CAP = 256;
  extern __shared__ __align__(16) uint64_t dyn[];   // [n_c keys][CAP top buffer]
  __shared__ uint64_t bounds[kMergeMaxWaves];
  __shared__ int32_t fin_parent[NEZHA_MAX_BEAM], fin_code[NEZHA_MAX_BEAM];
  const int b = blockIdx.x;
  if (a.redo_req && a.redo_req[b] == 0) return;      // a pass over what another kernel left
  // the wave id is made scalar: loops and branches on it are then uniform for the compiler
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_threads = blockDim.x, n_waves = n_threads >> 6;
  const int K = a.K, K_in = a.K_in;
  const int n_c = K_in * K;
  const bool verify = a.set.slots != nullptr;
  uint64_t* keys = dyn;
  uint64_t* topbuf = dyn + ((n_c + 1) & ~1);

  // Sort keys (score, ~candidate number) of the candidates that exist and, where a set is
  // consulted, are in it, packed at keys[0 .. n_valid): with verification a few per cent of the
  // candidates survive, and the selection below then reads those instead of all K_in * K.
  // A lane takes NB candidates at a time: their inputs, then the filter words of all of them, are
  // in flight together.  The few that pass the filter are gathered per wave (64 at a time, in
  // LDS) and looked up in the table one per lane, so a round of table accesses has full waves
  // instead of a lane or two per instruction.  (One candidate after the other, a workgroup's ten
  // rounds of three dependent memory accesses each were most of this kernel's time.)
  __shared__ int n_valid;
  __shared__ uint64_t staged_key[kMergeMaxWaves][64], staged_sk[kMergeMaxWaves][64];
  if (tid == 0) n_valid = 0;
  __syncthreads();
  constexpr int NB = 8;
  uint32_t top0 = 0, top1 = 0;                       // this lane's two largest scores (ordered bits)
  auto keep = [&](bool ok, uint64_t sk) {            // all lanes of the wave together
    const uint64_t bal = __ballot(ok);
    if (bal) {
      int at = 0;
      if (lane == 0) at = atomicAdd(&n_valid, __popcll(bal));
      at = __builtin_amdgcn_readfirstlane(at);
      if (ok)
        keys[at + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                            __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0))] = sk;
      const uint32_t s32 = ok ? (uint32_t)(sk >> 32) : 0u;
      const uint32_t lo = s32 > top0 ? top0 : s32;   // the smaller of (score, top0)
      top0 = s32 > top0 ? s32 : top0;
      top1 = lo > top1 ? lo : top1;
    }
  };
  int staged = 0;                                    // wave uniform
  auto look_up_staged = [&]() {
    wave_sync();
    bool ok = false;
    uint64_t sk = 0;
    if (lane < staged) {
      ok = set_probe(a.set, staged_key[wave][lane]);
      sk = staged_sk[wave][lane];
    }
    keep(ok, sk);
    wave_sync();
    staged = 0;
  };
  for (int base = wave * 64; base < n_c; base += n_threads * NB) {   // wave uniform trip count
    uint64_t prefix[NB];
    uint32_t code[NB];
    float score[NB];
    bool live[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int i = base + j * n_threads + lane;
      prefix[j] = 0ull;
      code[j] = 0u;
      score[j] = 0.f;
      live[j] = false;
      if (i < n_c) {
        const int p = i / K;
        const int64_t o = (int64_t)(b * K_in + p) * K + (i - p * K);
        score[j] = (a.score_in ? a.score_in[b * K_in + p] : 0.f) + a.cand_logp[o];
        prefix[j] = a.key_in ? a.key_in[b * K_in + p] : 0ull;
        live[j] = prefix[j] != kEmpty;               // an empty beam slot has no children
        if (verify) code[j] = (uint32_t)a.cand_code[o];
      }
    }
    uint64_t word[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      word[j] = ~0ull;
      if (verify && a.set.filter && live[j])
        word[j] = *(global_ptr<const uint64_t>)(a.set.filter +
                                                filter_word(prefix[j], code[j], a.set.n_blocks));
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int i = base + j * n_threads + lane;
      const bool go = live[j] && ((word[j] >> (code[j] & 63)) & 1ull);
      const uint64_t sk = ((uint64_t)ordered_bits(score[j]) << 32) | (uint32_t)~(uint32_t)i;
      if (!verify) {
        keep(go, sk);
        continue;
      }
      const uint64_t bal = __ballot(go);
      const int n = __popcll(bal);
      if (n == 0) continue;
      if (staged + n > 64) look_up_staged();
      if (go) {
        const int at = staged + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
        staged_key[wave][at] = prefix[j] + (uint64_t)code[j] * a.set.mult_last;
        staged_sk[wave][at] = sk;
      }
      staged += n;
    }
  }
  if (staged) look_up_staged();
  {
    // scores alone: a lower bound of the K-th largest key may ignore how ties are ordered
    uint32_t b32;
    if (K <= 64) {
      uint32_t mk[1][1] = {{top0}};
      sort_desc<1, 1, uint32_t>(mk);
      b32 = (uint32_t)__builtin_amdgcn_readlane((int)mk[0][0], K - 1);
    } else {
      uint32_t mk[1][2] = {{top0, top1}};
      sort_desc<2, 1, uint32_t>(mk);                 // position 2*lane + j
      b32 = (uint32_t)__builtin_amdgcn_readlane((int)pick_element<2>(mk[0], (K - 1) & 1),
                                                (K - 1) >> 1);
    }
    if (lane == 0) bounds[wave] = (uint64_t)b32 << 32;
  }
  __syncthreads();
  if (wave == 0) {
    uint64_t tau = bounds[0];
    for (int w = 1; w < n_waves; ++w) tau = bounds[w] > tau ? bounds[w] : tau;
    WaveTopK<CAP> f;
    f.init(topbuf, K);
    f.tau = tau ? tau - 1ull : 0ull;                 // keys >= tau enter
    const int n_in = n_valid;                        // (written before the barrier above)
    for (int base = 0; base < n_in; base += 64) f.push(base + lane < n_in ? keys[base + lane] : 0ull);
    f.compact();
    wave_sync();
    constexpr int NPL = (NEZHA_MAX_BEAM + 63) / 64;
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
      const int p = lane + 64 * j;
      if (p < K) {
        const int64_t o = (int64_t)b * K + p;
        if (p < f.cnt) {
          const uint64_t sk = f.buf[p];
          const int i = (int)(~(uint32_t)sk);
          const int par = i / K;
          const int32_t code = a.cand_code[(int64_t)(b * K_in + par) * K + (i - par * K)];
          a.key_out[o] = (a.key_in ? a.key_in[b * K_in + par] : 0ull) +
                         (uint64_t)(uint32_t)code * a.mult;
          a.score_out[o] = unordered_bits((uint32_t)(sk >> 32));
          a.parent_out[o] = par;
          a.code_out[o] = code;
          fin_parent[p] = par;
          fin_code[p] = code;
        } else {
          a.key_out[o] = kEmpty;
          a.score_out[o] = -INFINITY;
          a.parent_out[o] = -1;
          a.code_out[o] = -1;
          fin_parent[p] = -1;
          fin_code[p] = -1;
        }
      }
    }
    if (lane == 0 && a.count_out) a.count_out[b] = f.cnt;
  }
  __syncthreads();
  if (a.state_out) {
    if (a.transition == NEZHA_TRANSITION_RNN)
      update_states_rnn<BF16>(a.state_in, a.E, a.U, a.state_out, b, K, K_in, a.e, fin_parent,
                              fin_code, tid, n_threads);
    else
      update_states<BF16>(a.state_in, a.E, a.state_out, b, K, K_in, a.e, fin_parent, fin_code, tid,
                          n_threads);
  }
}

// ---- a level with one entering beam whose state is zero (level 1 of a decode) -------------------
// The logits are the user part itself (Eq. 2 with c = 0), so there is nothing to multiply: one
// workgroup of four waves per request holds the row in registers (16 per thread, T_l <= 4096),
// forms the log-sum-exp, and selects the K best codes: every lane's two largest keys give each
// wave a lower bound of its K-th largest (one small sort), the largest of the waves' bounds is a
// lower bound of the row's K-th largest, the keys at or above it are gathered in LDS and wave 0
// sorts them (score first, lower code first among equal scores).  Outputs and the Transition as
// merge_kernel writes them; no candidate arrays, no second launch.
struct FirstLevelArgs {
  const float* A;           // [B, V] user part
  const void* E;            // [V, e] (used when state_out != NULL)
  const void* U;            // recurrent Transition, else unused
  uint64_t mult;            // prod_{j<level} T_j
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  void* state_out;          // or NULL
  int32_t* count_out;       // or NULL
  int K, V, e, transition;
};
constexpr int kFirstThreads = 256, kFirstPerThread = 16, kFirstListCap = 1024;
template <bool BF16>
__global__ __launch_bounds__(kFirstThreads) void first_level_kernel(FirstLevelArgs a) {
  __shared__ uint64_t list[kFirstListCap + 256];        // gathered keys, then wave 0's sort buffer
  __shared__ float red[8];
  __shared__ uint32_t bounds[4];
  __shared__ int n_listed;
  __shared__ int32_t fin_parent[NEZHA_MAX_BEAM], fin_code[NEZHA_MAX_BEAM];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int V = a.V, K = a.K;
  float z[kFirstPerThread];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < kFirstPerThread; ++j) {
    const int v = tid + j * kFirstThreads;
    z[j] = v < V ? a.A[(int64_t)b * V + v] : -INFINITY;
    m = fmaxf(m, z[j]);
  }
  auto wave_max = [&](float x) {
    x = fmaxf(x, __uint_as_float(lane_xor<1>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(lane_xor<2>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(lane_xor<4>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(lane_xor<8>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(lane_xor<16>(__float_as_uint(x), lane)));
    x = fmaxf(x, __uint_as_float(lane_xor<32>(__float_as_uint(x), lane)));
    return x;
  };
  auto wave_sum = [&](float x) {
    x += __uint_as_float(lane_xor<1>(__float_as_uint(x), lane));
    x += __uint_as_float(lane_xor<2>(__float_as_uint(x), lane));
    x += __uint_as_float(lane_xor<4>(__float_as_uint(x), lane));
    x += __uint_as_float(lane_xor<8>(__float_as_uint(x), lane));
    x += __uint_as_float(lane_xor<16>(__float_as_uint(x), lane));
    x += __uint_as_float(lane_xor<32>(__float_as_uint(x), lane));
    return x;
  };
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  if (tid == 0) n_listed = 0;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float ssum = 0.f;
  uint32_t top0 = 0, top1 = 0;                       // the lane's two largest keys
#pragma unroll
  for (int j = 0; j < kFirstPerThread; ++j) {
    const int v = tid + j * kFirstThreads;
    if (v < V) ssum += __builtin_amdgcn_exp2f((z[j] - m) * kLog2e);
    const uint32_t k = v < V ? ordered_bits(z[j]) : 0u;
    const uint32_t lo = k > top0 ? top0 : k;
    top0 = k > top0 ? k : top0;
    top1 = lo > top1 ? lo : top1;
  }
  ssum = wave_sum(ssum);
  if (lane == 0) red[4 + wave] = ssum;
  {
    uint32_t mk[1][2] = {{top0, top1}};
    sort_desc<2, 1, uint32_t>(mk);                   // position 2*lane + j; K <= 128
    const uint32_t bw = (uint32_t)__builtin_amdgcn_readlane((int)pick_element<2>(mk[0], (K - 1) & 1),
                                                            (K - 1) >> 1);
    if (lane == 0) bounds[wave] = bw;
  }
  __syncthreads();
  const float lse = m + __builtin_amdgcn_logf((red[4] + red[5]) + (red[6] + red[7])) * kLn2;
  uint32_t tau = bounds[0];
#pragma unroll
  for (int w = 1; w < 4; ++w) tau = bounds[w] > tau ? bounds[w] : tau;
  bool over = false;
#pragma unroll
  for (int j = 0; j < kFirstPerThread; ++j) {
    const int v = tid + j * kFirstThreads;
    const uint32_t k = v < V ? ordered_bits(z[j]) : 0u;
    const bool take = v < V && k >= tau;
    const uint64_t bal = __ballot(take);
    if (bal) {
      int at = 0;
      if (lane == 0) at = atomicAdd(&n_listed, __popcll(bal));
      at = __builtin_amdgcn_readfirstlane(at) +
           __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
      if (take && at < kFirstListCap) list[at] = ((uint64_t)k << 32) | (uint32_t)~(uint32_t)v;
    }
  }
  __syncthreads();
  int n = n_listed;
  over = n > kFirstListCap;
  if (wave == 0) {
    WaveTopK<256> f;
    f.init(list + kFirstListCap, K);
    if (!over) {
      for (int base = 0; base < n; base += 64) f.push(base + lane < n ? list[base + lane] : 0ull);
    } else {
      // more keys tie with the bound than the list holds: stream the whole row
      for (int v0 = 0; v0 < V; v0 += 64) {
        const int v = v0 + lane;
        f.push(v < V ? (((uint64_t)ordered_bits(a.A[(int64_t)b * V + v]) << 32) | (uint32_t)~(uint32_t)v)
                     : 0ull);
      }
    }
    f.compact();
    wave_sync();
    constexpr int NPLK = (NEZHA_MAX_BEAM + 63) / 64;
#pragma unroll
    for (int j = 0; j < NPLK; ++j) {
      const int p = lane + 64 * j;
      if (p < K) {
        const int64_t o = (int64_t)b * K + p;
        if (p < f.cnt) {
          const uint64_t sk = f.buf[p];
          const int32_t code = (int32_t)(~(uint32_t)sk);
          a.key_out[o] = (uint64_t)(uint32_t)code * a.mult;
          a.score_out[o] = unordered_bits((uint32_t)(sk >> 32)) - lse;
          a.parent_out[o] = 0;
          a.code_out[o] = code;
          fin_parent[p] = 0;
          fin_code[p] = code;
        } else {
          a.key_out[o] = kEmpty;
          a.score_out[o] = -INFINITY;
          a.parent_out[o] = -1;
          a.code_out[o] = -1;
          fin_parent[p] = -1;
          fin_code[p] = -1;
        }
      }
    }
    if (lane == 0 && a.count_out) a.count_out[b] = f.cnt;
  }
  __syncthreads();
  if (a.state_out) {
    if (a.transition == NEZHA_TRANSITION_RNN)
      update_states_rnn<BF16>(nullptr, a.E, a.U, a.state_out, b, K, 1, a.e, fin_parent, fin_code, tid,
                              kFirstThreads);
    else
      update_states<BF16>(nullptr, a.E, a.state_out, b, K, 1, a.e, fin_parent, fin_code, tid,
                          kFirstThreads);
  }
}

// ---- the same step for large codebooks: two sweeps over the codes, no running top-K -----------
// A workgroup of 8 waves owns 16 beams and walks the T_l codes in chunks of 256: phase A puts the
// chunk's 16 x 256 logits into one of two LDS tiles by MFMA (operands of the next chunk are
// fetched meanwhile), phase B gives every wave two rows with the row spread over all 64 lanes.
//   sweep 1: running (max, sum of exponentials) and each lane's two largest logits per row.  The
//            K-th largest of a row's 128 lane maxima is a lower bound of its K-th largest logit.
//   sweep 2: the logits are formed again and those at or above the bound (K .. about 1.5 K of them)
//            are appended to the row's LDS list; one sort per row then gives the K best.
// The MFMA work is done twice, but nothing is sorted while streaming.  A row whose list would
// overflow (more than 256 logits tie with the bound) is redone in a third sweep with the
// general streaming top-K.  K <= 128.
constexpr int kChunk = 256;
// The 16 beams R0 .. R0+15 (one workgroup; redo_flag is a word of static LDS).
template <int KST>
__device__ __forceinline__ void expand_chunked_group(const ExpandArgs& a, const int R0,
                                                     uint64_t* lds, int& redo_flag) {
  constexpr int CAP = 256;
  uint64_t* lists = lds;                                              // [16 rows][CAP]
  float* ztile = reinterpret_cast<float*>(lds + 16 * CAP);            // [2][16][kChunk]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, c = lane & 15;
  const int V = a.V, K = a.K, e = a.e;
  const bool has_beam = a.state != nullptr;
  const int KS = e / 32;
  const int n_ct = V / 16;
  const int n_chunks = (V + kChunk - 1) / kChunk;

  bf16x8 fa16[KST];
  if (has_beam) {
    const int row = R0 + c;
    const uint16_t* st = static_cast<const uint16_t*>(a.state);
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) {
      uint4 v = uint4{0, 0, 0, 0};
      if (ks < KS && row < a.rows)
        v = *reinterpret_cast<const uint4*>(st + (int64_t)row * e + ks * 32 + 8 * g);
      fa16[ks] = *reinterpret_cast<bf16x8*>(&v);
    }
  }
  int64_t a_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = R0 + 4 * g + i;
    a_off[i] = (int64_t)((row < a.rows ? row : 0) / a.K_in) * V;
  }
  // operands of this wave's two tiles of a chunk (column tiles 16*ch + wave and + 8)
  float aq[2][4];
  uint4 wq[2][KST];
  auto prefetch = [&](int ch) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      int ct = ch * 16 + wave + 8 * t;
      ct = ct < n_ct ? ct : n_ct - 1;                                 // clamped; masked at the store
#pragma unroll
      for (int i = 0; i < 4; ++i) aq[t][i] = a.A[a_off[i] + ct * 16 + c];
      if (has_beam) {
        const uint4* wp = static_cast<const uint4*>(a.Wbeam) + (int64_t)ct * KS * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
          if (ks < KS) wq[t][ks] = wp[ks * 64];
      }
    }
  };
  auto project = [&](int ch) {                                        // phase A of chunk ch
    float* zt = ztile + (ch & 1) * 16 * kChunk;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx4 acc = floatx4{aq[t][0], aq[t][1], aq[t][2], aq[t][3]};
      if (has_beam) {
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
          if (ks < KS)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                fa16[ks], *reinterpret_cast<bf16x8*>(&wq[t][ks]), acc, 0, 0, 0);
      }
      const bool in_range = ch * 16 + wave + 8 * t < n_ct;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        zt[(4 * g + i) * kChunk + (wave + 8 * t) * 16 + c] = in_range ? acc[i] : -INFINITY;
    }
  };

  // phase B state of this wave's rows 2*wave, 2*wave+1
  const int r0 = wave * 2;
  float m[2] = {-INFINITY, -INFINITY}, ssum[2] = {0.f, 0.f};
  float top0[2] = {-INFINITY, -INFINITY}, top1[2] = {-INFINITY, -INFINITY};
  float bound[2] = {INFINITY, INFINITY};
  int cnt[2] = {0, 0};
  bool over[2] = {false, false};
  WaveTopK<CAP> q[2];

  for (int sweep = 0; sweep < 3; ++sweep) {
    if (sweep == 2) {
      // third sweep only if some row overflowed (decided for the whole workgroup)
      if (threadIdx.x == 0) redo_flag = 0;
      __syncthreads();
      if (lane == 0 && (over[0] || over[1])) redo_flag = 1;
      __syncthreads();
      if (!redo_flag) break;
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) q[rr].init(lists + (r0 + rr) * CAP, K);
    }
    prefetch(0);
    for (int ch = 0; ch < n_chunks; ++ch) {
      project(ch);
      if (ch + 1 < n_chunks) prefetch(ch + 1);
      __syncthreads();          // tile ch complete; everyone is past phase B of tile ch-1
      const float* zt = ztile + (ch & 1) * 16 * kChunk;
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        float z[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) z[j] = zt[(r0 + rr) * kChunk + j * 64 + lane];
        if (sweep == 0) {
          const float mx = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
          const float mn = fmaxf(m[rr], mx);
          float sum = (m[rr] == mn) ? ssum[rr] : ssum[rr] * __builtin_amdgcn_exp2f((m[rr] - mn) * kLog2e);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            sum += (z[j] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((z[j] - mn) * kLog2e);
            const float lo = fminf(z[j], top0[rr]);
            top0[rr] = fmaxf(z[j], top0[rr]);
            top1[rr] = fmaxf(top1[rr], lo);
          }
          ssum[rr] = sum;
          m[rr] = mn;
        } else if (sweep == 1) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const bool pass = z[j] >= bound[rr];
            const uint64_t bal = __ballot(pass);
            if (bal) {
              const int pos = cnt[rr] + __builtin_amdgcn_mbcnt_hi(
                                            (uint32_t)(bal >> 32),
                                            __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
              const uint32_t code = (uint32_t)(ch * kChunk + j * 64 + lane);
              if (pass && pos < CAP)
                lists[(r0 + rr) * CAP + pos] = ((uint64_t)ordered_bits(z[j]) << 32) | (uint32_t)~code;
              cnt[rr] += __popcll(bal);
              if (cnt[rr] > CAP) over[rr] = true;
            }
          }
        } else if (over[rr]) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t code = (uint32_t)(ch * kChunk + j * 64 + lane);
            q[rr].push(z[j] == -INFINITY ? 0ull
                                         : (((uint64_t)ordered_bits(z[j]) << 32) | (uint32_t)~code));
          }
        }
      }
    }
    if (sweep == 0) {
      // log-sum-exp: merge the 64 lanes' (max, sum); bound: K-th largest of the 128 lane maxima
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        float mm = m[rr], ss = ssum[rr];
        auto merge_with = [&](float om, float os) {
          const float mn = fmaxf(mm, om);
          const float wa = (mm == mn) ? 1.f : __builtin_amdgcn_exp2f((mm - mn) * kLog2e);
          const float wb = (om == mn) ? 1.f : __builtin_amdgcn_exp2f((om - mn) * kLog2e);
          ss = ss * wa + os * wb;
          mm = mn;
        };
        merge_with(__uint_as_float(lane_xor<1>(__float_as_uint(mm), lane)),
                   __uint_as_float(lane_xor<1>(__float_as_uint(ss), lane)));
        merge_with(__uint_as_float(lane_xor<2>(__float_as_uint(mm), lane)),
                   __uint_as_float(lane_xor<2>(__float_as_uint(ss), lane)));
        merge_with(__uint_as_float(lane_xor<4>(__float_as_uint(mm), lane)),
                   __uint_as_float(lane_xor<4>(__float_as_uint(ss), lane)));
        merge_with(__uint_as_float(lane_xor<8>(__float_as_uint(mm), lane)),
                   __uint_as_float(lane_xor<8>(__float_as_uint(ss), lane)));
        merge_with(__uint_as_float(lane_xor<16>(__float_as_uint(mm), lane)),
                   __uint_as_float(lane_xor<16>(__float_as_uint(ss), lane)));
        merge_with(__uint_as_float(lane_xor<32>(__float_as_uint(mm), lane)),
                   __uint_as_float(lane_xor<32>(__float_as_uint(ss), lane)));
        m[rr] = mm;
        ssum[rr] = ss;
      }
      uint64_t mk[2][2];
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        mk[rr][0] = (uint64_t)ordered_bits(top0[rr]) << 32;
        mk[rr][1] = (uint64_t)ordered_bits(top1[rr]) << 32;
      }
      sort_desc<2, 2>(mk);                                            // position 2*lane + j
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const uint64_t pick = ((K - 1) & 1) ? mk[rr][1] : mk[rr][0];
        bound[rr] = unordered_bits(
            (uint32_t)__builtin_amdgcn_readlane((uint32_t)(pick >> 32), (K - 1) >> 1));
      }
    }
    __syncthreads();            // the tiles are free again before the next sweep's first phase A
  }

  // the K best of each list, sorted; rows redone in the third sweep take their streaming result
  if (R0 + r0 >= a.rows) return;
#pragma unroll
  for (int rr = 0; rr < 2; ++rr)
    if (over[rr]) {
      q[rr].compact();
      cnt[rr] = q[rr].cnt;
    }
  if (!over[0] || !over[1]) {
    uint64_t* const crows[2] = {lists + r0 * CAP, lists + (r0 + 1) * CAP};
    int rc[2] = {over[0] ? 0 : cnt[0], over[1] ? 0 : cnt[1]};
    uint64_t rt[2];
    compact_rows<CAP, 2>(crows, rc, rt, K);
    if (!over[0]) cnt[0] = rc[0];
    if (!over[1]) cnt[1] = rc[1];
  }
  wave_sync();
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    const int row = R0 + r0 + rr;
    if (row < a.rows && (!a.redo || a.redo[row] != 0)) {
      const float lse = m[rr] + __builtin_amdgcn_logf(ssum[rr]) * kLn2;
      for (int p = lane; p < cnt[rr]; p += 64) {
        const uint64_t kk = lists[(r0 + rr) * CAP + p];
        a.cand_code[(int64_t)row * K + p] = (int32_t)(~(uint32_t)kk);
        a.cand_logp[(int64_t)row * K + p] = unordered_bits((uint32_t)(kk >> 32)) - lse;
      }
    }
  }
}
// Without a.redo: workgroup i takes beams 16 i .. 16 i + 15.  With a.redo (a pass over the beams
// another kernel left, usually a handful among tens of thousands): every workgroup of a small grid
// looks through its share of the groups of 16 beams, one group per thread and one 16-byte load
// per group, and then takes the flagged ones of its share in turn.  (A workgroup per
// group that leaves at once costs more in dispatch than the pass does in work.)  The flags are
// padded to a multiple of 256 bytes and 16-byte aligned.
constexpr int kRedoScanGroups = 256;   // workgroups of a redo pass
template <int KST>
__global__ __launch_bounds__(512, 4) void expand_chunked_kernel(ExpandArgs a) {
  extern __shared__ __align__(16) uint64_t lds[];
  __shared__ int redo_flag;
  if (!a.redo) {
    expand_chunked_group<KST>(a, blockIdx.x * 16, lds, redo_flag);
    return;
  }
  __shared__ int n_found;
  __shared__ int found[512];
  const int n_groups = (a.rows + 15) / 16;
  // thread t of workgroup w looks at groups w + (t + 512 k) * (number of workgroups): the groups of
  // one flagged request (neighbours) go to different workgroups
  const int G = (int)gridDim.x;
  for (int base = 0; base * G + (int)blockIdx.x < n_groups; base += 512) {
    if (threadIdx.x == 0) n_found = 0;
    __syncthreads();
    const int gi = (base + (int)threadIdx.x) * G + (int)blockIdx.x;
    if (gi < n_groups) {
      const uint4 f = load_global_u4(a.redo + (int64_t)gi * 16);
      const int live = a.rows - gi * 16;                   // rows of the group inside the batch
      const uint32_t word[4] = {f.x, f.y, f.z, f.w};
      bool any = false;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = live - 4 * i;                         // bytes of this word that are flags
        const uint32_t mask = n >= 4 ? 0xFFFFFFFFu : (n <= 0 ? 0u : (1u << (8 * n)) - 1u);
        any = any || (word[i] & mask) != 0;
      }
      if (any) found[atomicAdd(&n_found, 1)] = gi;
    }
    __syncthreads();
    const int n = n_found;
    for (int k = 0; k < n; ++k) {
      expand_chunked_group<KST>(a, found[k] * 16, lds, redo_flag);
      __syncthreads();                                      // the lists and tiles are reused
    }
  }
}

// ---- the same step with one workgroup per request (bf16, K_in >= 16) ---------------------------
// The beams of a request share its user-part row and all beams share W_l: wave w owns the
// request's beams 16w .. 16w+15 as one MFMA row tile, and the packed beam part of W_l is streamed
// through LDS in chunks of 128 codes (global_load_lds, two buffers) that every wave reads, so W_l
// crosses L2 -> CU once per request and sweep instead of once per 16 beams.  Logits stay in the
// MFMA result layout (register i of lane l: beam 4*(l/16)+i of the tile, code column l%16):
//   sweep 1: per lane and beam a running sum of exponentials about a reference point and the
//            maxima of 8 code groups (column tile modulo 8).  A beam's 16 lanes x 8 groups give
//            128 group maxima; the K-th largest of them is a lower bound of the beam's K-th
//            largest logit.
//   sweep 2: logits at or above the bound are appended to the beam's list of 384 (logit, code)
//            pairs in global scratch, the place taken from a counter in LDS.  The scratch belongs
//            to the workgroup and is reused for each of its requests, so it lives in L2 / MALL.
//            (A list per (beam, lane) pair with its counter in a register needs no atomic, but
//            its stores fall on 64 different lines per instruction: measured, 23 % slower.)
//   Then, per beam, a sort of the listed logits alone (32-bit keys) gives the K-th largest; the
//   entries above it and the lowest codes among those equal to it are written out, in list order.
//   (The merge step orders equal scores by parent and code, so the order inside a beam's
//   candidates carries no meaning.)
// A beam whose list would overflow (ties, or large logits crowded into few groups) is flagged in
// redo[] and left to a pass of expand_chunked_kernel.
constexpr int kReqCap = 384;         // list entries per beam (about 190 are used at K = 100, T_l = 4096)
constexpr int kReqTiles = 8;         // column tiles per chunk = code groups per lane and beam
constexpr int kReqMaxGroups = 1024;  // workgroups that own list scratch
__host__ __device__ inline size_t request_w_region(int e, int n_waves) {
  const size_t chunks = (size_t)2 * kReqTiles * (e / 32) * 1024;   // two chunk buffers
  const size_t maxima = (size_t)n_waves * 16 * 128 * 4;            // group maxima between sweeps
  return chunks > maxima ? chunks : maxima;
}
// WHOLE = true (a level without verification): the per-beam lists and the merge step are skipped.
// The K best of the request's K_in * T_l candidates are the same set whether or not each beam is
// first cut to its own K best, so the selection is done on cumulative scores for the request as a
// whole: after sweep 1 every wave turns the 16 largest group maxima of each of its beams into
// scores (parent score + logit - log-sum-exp, formed exactly as the final scores are), and the
// K-th largest of a wave's 256 such scores bounds the request's K-th best score from below; the
// best of the waves' bounds is the threshold.  Sweep 2 appends the few candidates at or above it
// (about 1.5 K .. 6 K per request instead of 1.3 K per beam) to one list in LDS as final sort keys
// (score, parent, code); wave 0 sorts them, writes the level's outputs, and the workgroup applies
// the Transition.  A request whose list overflows is flagged and left to the general kernels.
struct RequestLevelArgs {
  const uint64_t* key_in;   // [B, K_in] or NULL
  const float* score_in;    // [B, K_in] or NULL
  const void* E;            // [V, e] (used when state_out != NULL)
  const void* U;            // recurrent Transition, else unused
  uint64_t mult;            // prod_{j<level} T_j
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  void* state_out;          // or NULL
  int32_t* count_out;       // or NULL
  uint8_t* redo_req;        // [B]: 1 = the request is left to the general kernels
  int transition;
};
constexpr int kReqListCap = 768;     // WHOLE: candidates per request kept for the final sort
constexpr int kReqForced = 1 << 30;  // WHOLE: bit of the request's counter that hands it to the general kernels
__host__ __device__ inline size_t request_whole_lds() {
  // request list, wave 0's sorting buffer, per-wave bounds + counter, survivors' parents / codes
  return (size_t)kReqListCap * 8 + 256 * 8 + 16 * 4 + 2 * NEZHA_MAX_BEAM * 4;
}
template <int KST, bool WHOLE>
__global__ __launch_bounds__(512, KST <= 4 ? 4 : 2) void expand_request_kernel(
    ExpandArgs a, uint64_t* __restrict__ lists_all, uint8_t* __restrict__ redo,
    RequestLevelArgs la) {
  extern __shared__ __align__(16) uint8_t req_lds[];
  // wave-uniform values are made scalar so that what is derived from them needs no vector registers
  const int lane = threadIdx.x & 63, NW = blockDim.x >> 6;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int V = a.V, K = a.K, K_in = a.K_in, e = a.e;
  constexpr int KS = KST;                                   // e = 32 * KST exactly
  const int n_ct = V / 16;
  const int n_chunks = (n_ct + kReqTiles - 1) / kReqTiles;
  constexpr int chunk_blocks = kReqTiles * KS;              // 1 KiB operand blocks per chunk
  const int total_blocks = n_ct * KS;
  uint8_t* const wbuf = req_lds;                                                  // [2][chunk]
  float* const abuf = reinterpret_cast<float*>(req_lds + request_w_region(e, NW));   // [2][128]
  // per wave: bound[16], lse[16], count[16] (WHOLE: the parents' scores instead of the counts)
  float* const my_info = abuf + 2 * kReqTiles * 16 + wave * 48;
  // list form: entries listed per beam, four 16-bit counts to a word (word g: beams 4g .. 4g+3), so
  // that a lane reserves places for its four beams with one LDS atomic
  unsigned long long* const my_cnt4 = reinterpret_cast<unsigned long long*>(my_info + 32);
  uint64_t* const my_lists = lists_all + ((int64_t)blockIdx.x * 128 + wave * 16) * kReqCap;
  // WHOLE only (after the NW waves' info):
  uint64_t* const req_list = reinterpret_cast<uint64_t*>(abuf + 2 * kReqTiles * 16 + NW * 48);
  uint64_t* const topbuf = req_list + kReqListCap;
  uint32_t* const tau_s = reinterpret_cast<uint32_t*>(topbuf + 256);   // [8] bounds, [8] = counter
  int* const req_cnt = reinterpret_cast<int*>(tau_s + 8);
  int32_t* const fin_parent = reinterpret_cast<int32_t*>(tau_s + 16);
  int32_t* const fin_code = fin_parent + NEZHA_MAX_BEAM;
  const int B = a.rows / K_in;
  const uint4* const Wb = static_cast<const uint4*>(a.Wbeam);

  auto stage = [&](int b, int ch) {       // chunk ch of W_l and of the request's user-part row
    uint8_t* dst = wbuf + (ch & 1) * chunk_blocks * 1024;
    for (int blk = wave; blk < chunk_blocks; blk += NW) {
      int gb = ch * chunk_blocks + blk;
      gb = gb < total_blocks ? gb : total_blocks - 1;       // past the end: a block nobody uses
      load_block_to_lds(Wb + (int64_t)gb * 64 + lane, dst + blk * 1024);
    }
    if (wave == NW - 1 && lane < kReqTiles * 4) {
      int col = ch * kReqTiles * 16 + lane * 4;
      col = col < V ? col : 0;
      load_block_to_lds(a.A + (int64_t)b * V + col, abuf + (ch & 1) * kReqTiles * 16);
    }
  };

  for (int b = blockIdx.x; b < B; b += gridDim.x) {
    bf16x8 fa16[KST];
    {
      const int g = lane >> 4, c = lane & 15;
      const int r = wave * 16 + c;
      const uint16_t* st = static_cast<const uint16_t*>(a.state);
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) {
        uint4 v = uint4{0, 0, 0, 0};
        if (st && r < K_in)
          v = *reinterpret_cast<const uint4*>(st + ((int64_t)b * K_in + r) * e + ks * 32 + 8 * g);
        fa16[ks] = *reinterpret_cast<bf16x8*>(&v);
      }
    }
    // sweep 1 state: sum of exp(z - m) with the reference m held as nml = -m * log2(e)
    // (as few values as possible live through the first sweep: it is the one short of registers)
    // What the second sweep needs (bounds, parent scores, log-sum-exps, threshold) is handed over
    // through LDS and read at its start, so that nothing but this lives through the first sweep.
    // group maxima of beams (4g, 4g+1) and (4g+2, 4g+3) as packed half pairs: half the registers
    uint32_t gmaxp[2][kReqTiles];
    float nml[4], ssum[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      nml[i] = 0.f;
      ssum[i] = 0.f;
#pragma unroll
      for (int j = 0; j < kReqTiles; ++j) gmaxp[i >> 1][j] = 0xFC00FC00u;   // (-inf, -inf)
    }
    if constexpr (WHOLE) {
      const int g = lane >> 4, c = lane & 15;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = wave * 16 + 4 * g + i;
        float v = -INFINITY;
        if (row < K_in) {
          const bool dead = la.key_in && la.key_in[(int64_t)b * K_in + row] == kEmpty;
          if (!dead) v = la.score_in ? la.score_in[(int64_t)b * K_in + row] : 0.f;
        }
        if (c == 0) my_info[32 + 4 * g + i] = v;   // read back after the first sweep
      }
      if (threadIdx.x == 0) {
        *req_cnt = 0;
        tau_s[0] = 0;
      }
    } else {
      if (lane < 4) my_cnt4[lane] = 0ull;
    }

    auto run_sweep = [&](auto sweep_c) {
      constexpr int sweep = decltype(sweep_c)::value;
      // a copy of the lane id the compiler cannot see through: addresses derived from it are
      // formed here and not kept in registers across the other phases
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int g = ln >> 4, c = ln & 15;
      // second sweep: per-beam logit bounds (and, WHOLE, what turns a logit into its final score)
      float bound[4], sp[4], lse_r[4];
      uint32_t tau = 0;                       // WHOLE: ordered bits of the score threshold
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bound[i] = INFINITY;
        sp[i] = 0.f;
        lse_r[i] = 0.f;
      }
      if constexpr (sweep == 1) {
        if constexpr (WHOLE) {
          tau = (uint32_t)__builtin_amdgcn_readfirstlane((int)tau_s[0]);
          // a logit bound per beam that no candidate with score >= tau can fall below: the
          // threshold moved back through the (rounded) score formula, minus a margin far above
          // the rounding of two float32 additions
          const float tf = unordered_bits(tau);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            sp[i] = my_info[32 + 4 * g + i];
            lse_r[i] = my_info[16 + 4 * g + i];
            const float margin = 1e-5f * (fabsf(tf) + fabsf(sp[i]) + fabsf(lse_r[i]) + 1.f);
            const float bz = (tf - sp[i]) + lse_r[i] - margin;
            bound[i] = (sp[i] == -INFINITY) ? INFINITY : bz;
          }
          // No threshold (fewer than K candidates with a finite score, i.e. nearly all entering
          // beams are empty slots): everything would be listed; the general kernels take the
          // request.
          if (!(tf > -INFINITY)) {
            if (threadIdx.x == 0) atomicOr(req_cnt, kReqForced);
#pragma unroll
            for (int i = 0; i < 4; ++i) bound[i] = INFINITY;
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            bound[i] = (wave * 16 + 4 * g + i < K_in) ? my_info[4 * g + i] : INFINITY;
        }
      }
      stage(b, 0);
      for (int ch = 0; ch < n_chunks; ++ch) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of chunk ch has landed
        __syncthreads();                      // chunk ch is whole; the other buffer is free
        if (ch + 1 < n_chunks) stage(b, ch + 1);
        const uint8_t* wb = wbuf + (ch & 1) * chunk_blocks * 1024;
        const float* ab = abuf + (ch & 1) * kReqTiles * 16;
        const int tiles = n_ct - ch * kReqTiles;            // >= kReqTiles except in the last chunk
        auto chunk_body = [&](auto ragged_c) {
          constexpr bool ragged = decltype(ragged_c)::value;
          // One operand set, two accumulators.  The matrix instructions of a tile form a dependent
          // chain (each adds to the result of the one before), so a wave that issued them back to
          // back would sit out each one's latency; instead the vector work on the previous tile's
          // logits is cut into four pieces (one per beam of the lane) that are issued between the
          // chain's links, and each operand register is requested again (for the next tile) right
          // after the instruction that consumed it.  The scheduling fences pin that order.
          // (Worth 2 % here: with four waves on a SIMD the other waves already fill most of such
          // gaps, and matrix and vector instructions of one SIMD overlap only in part: a loop of
          // both takes the vector time plus about half the matrix time, however they are ordered.)
          uint4 w[KST];
          float a0;
          floatx4 acc[2];
          auto read_operand = [&](int ct, int ks) {
            w[ks] = *reinterpret_cast<const uint4*>(wb + ((ct * KS + ks) * 64 + ln) * 16);
            if (ks == 0) a0 = ab[ct * 16 + c];
          };
          // piece i of the vector work on tile ct (the lane's logit of beam 4g+i)
          auto piece = [&](int ct, int buf, int i) {
            const bool live = !ragged || ct < tiles;
            auto zv = [&](int j) { return live ? acc[buf][j] : -INFINITY; };
            const float z = zv(i);
            if constexpr (sweep == 0) {
              // Sum of exp(z - m) about a fixed reference m = (the lane's first logit of the
              // beam) + 20, held as nml = -m * log2(e): no rescaling while streaming.  A beam with
              // a logit more than 64 above a lane's reference is redone by the general kernel.
              if (ct == 0 && ch == 0) nml[i] = -(z + 20.f) * kLog2e;
              // (the whole-level form only uses the lane's largest logit per beam: one group)
              if ((i & 1) == 0)
                gmaxp[i >> 1][WHOLE ? 0 : ct] =
                    max_of_half_pairs(gmaxp[i >> 1][WHOLE ? 0 : ct], pack_halves_rtz(z, zv(i + 1)));
              ssum[i] += __builtin_amdgcn_exp2f(fmaf(z, kLog2e, nml[i]));
            } else if constexpr (WHOLE) {
              // The accumulators started at (user part - bound of the beam), so the lane's four
              // values are logit - bound and one test serves all four; candidates are so rare
              // after the request-wide threshold that the branch is almost never taken.
              if (i == 3) {
                const float most = fmaxf(fmaxf(zv(0), zv(1)), fmaxf(zv(2), zv(3)));
                if (most >= 0.f) {
#pragma unroll
                  for (int k = 0; k < 4; ++k) {
                    const float over = zv(k);
                    if (over >= 0.f) {                       // the logit cannot be missed
                      const float zl = over + bound[k];
                      const uint32_t key = ordered_bits(sp[k] + (zl - lse_r[k]));   // the final score
                      if (key >= tau) {
                        const uint32_t code = (uint32_t)((ch * kReqTiles + ct) * 16 + c);
                        const int pos = atomicAdd(req_cnt, 1);
                        const uint32_t who = ((uint32_t)(wave * 16 + 4 * g + k) << 24) | code;
                        if (pos < kReqListCap) req_list[pos] = ((uint64_t)key << 32) | (uint32_t)~who;
                      }
                    }
                  }
                }
              }
            } else {
              // all four beams of the lane after the chain's last link: one atomic on the lane's
              // word of counts reserves a place in each list the lane appends to
              if (i == 3) {
                bool pass[4];
                unsigned long long add = 0ull;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                  pass[k] = live && zv(k) >= bound[k];
                  add |= pass[k] ? (1ull << (16 * k)) : 0ull;
                }
                if (add != 0ull) {
                  const unsigned long long before = atomicAdd(&my_cnt4[g], add);
                  const uint32_t code = (uint32_t)((ch * kReqTiles + ct) * 16 + c);
#pragma unroll
                  for (int k = 0; k < 4; ++k) {
                    const int pos = (int)((before >> (16 * k)) & 0xFFFFull);
                    if (pass[k] && pos < kReqCap)
                      my_lists[(4 * g + k) * kReqCap + pos] =
                          ((uint64_t)__float_as_uint(zv(k)) << 32) | code;
                  }
                }
              }
            }
          };
#pragma unroll
          for (int ks = 0; ks < KST; ++ks) read_operand(0, ks);
#pragma unroll
          for (int ct = 0; ct <= kReqTiles; ++ct) {
            floatx4 t = floatx4{a0, a0, a0, a0};
            if constexpr (WHOLE && sweep == 1)
              t = floatx4{a0 - bound[0], a0 - bound[1], a0 - bound[2], a0 - bound[3]};
#pragma unroll
            for (int ks = 0; ks < KST; ++ks) {
              if (ct < kReqTiles) {
                t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    fa16[ks], *reinterpret_cast<const bf16x8*>(&w[ks]), t, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (ct + 1 < kReqTiles) read_operand(ct + 1, ks);
                __builtin_amdgcn_sched_barrier(0);
              }
              if (ct > 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  if ((i * KST) / 4 == ks) piece(ct - 1, (ct - 1) & 1, i);
                __builtin_amdgcn_sched_barrier(0);
              }
            }
            if (ct < kReqTiles) acc[ct & 1] = t;
          }
        };
        if (tiles >= kReqTiles) chunk_body(std::false_type{});
        else chunk_body(std::true_type{});
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);     // list stores are done before anyone reads them
      __syncthreads();                        // every wave is done with the chunk buffers
      if constexpr (sweep == 0) {
        uint32_t lane_key[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 4; ++i) {         // (reference, sum) over the beam's 16 lanes
          const float m_ref = -nml[i] * kLn2;                // the reference the sum was taken about
          float mm = m_ref, ss = ssum[i];
          auto merge_with = [&](float om, float os) {
            const float mn = fmaxf(mm, om);
            ss = ss * __builtin_amdgcn_exp2f((mm - mn) * kLog2e) +
                 os * __builtin_amdgcn_exp2f((om - mn) * kLog2e);
            mm = mn;
          };
          merge_with(__uint_as_float(lane_xor<1>(__float_as_uint(mm), lane)),
                     __uint_as_float(lane_xor<1>(__float_as_uint(ss), lane)));
          merge_with(__uint_as_float(lane_xor<2>(__float_as_uint(mm), lane)),
                     __uint_as_float(lane_xor<2>(__float_as_uint(ss), lane)));
          merge_with(__uint_as_float(lane_xor<4>(__float_as_uint(mm), lane)),
                     __uint_as_float(lane_xor<4>(__float_as_uint(ss), lane)));
          merge_with(__uint_as_float(lane_xor<8>(__float_as_uint(mm), lane)),
                     __uint_as_float(lane_xor<8>(__float_as_uint(ss), lane)));
          const float lse_i = mm + __builtin_amdgcn_logf(ss) * kLn2;   // the same in the beam's 16 lanes
          if (c == 0) my_info[16 + 4 * g + i] = lse_i;
          float top = -INFINITY;
          bool clamped = false;
#pragma unroll
          for (int j = 0; j < (WHOLE ? 1 : kReqTiles); ++j) {
            const float m = half_bits_to_float(gmaxp[i >> 1][j] >> (16 * (i & 1)));
            top = fmaxf(top, m);
            clamped |= half_out_of_range(m);
          }
          // this lane's sum may have overflowed, or a maximum left the half range: push the
          // beam's (the request's) count past the list size
          if (half_ceil(top) > m_ref + 64.f || clamped) {
            if constexpr (WHOLE) atomicOr(req_cnt, kReqForced);
            else atomicAdd(&my_cnt4[g], (unsigned long long)(kReqCap + 1) << (16 * i));
          }
          if constexpr (WHOLE) {
            // the lane's largest logit of this beam, as a score no larger than the true one
            // (formed as the final scores are: parent score + (logit - log-sum-exp); the margin
            // covers the last-place differences between the 16 lanes' copies of the log-sum-exp)
            const float sp_i = my_info[32 + 4 * g + i];
            const float low = sp_i + (half_floor(top) - lse_i);
            lane_key[i] = ordered_bits(low - 4e-6f * (fabsf(lse_i) + fabsf(sp_i) + 1.f));
          }
        }
        if constexpr (WHOLE) {
          // Threshold of the request: each lane holds, per beam, the largest of its 256 logits: 16
          // distinct candidates per beam, 256 per wave, 256 NW in the workgroup, whose scores
          // bound the K-th best score of the request from below by their K-th largest.  Every
          // wave sorts its 256 and leaves its 128 best (K <= 128) in the chunk buffers; then each
          // lane ranks two of its wave's entries among all waves' lists (a binary search per
          // list): the largest entry with at least K entries at or above it is that K-th largest.
          uint32_t uk[1][4] = {{lane_key[0], lane_key[1], lane_key[2], lane_key[3]}};
          sort_desc<4, 1, uint32_t>(uk);                                  // position 4*lane + j
          uint32_t* const best = reinterpret_cast<uint32_t*>(req_lds);    // [NW][128], descending
          if (lane < 32)
            *reinterpret_cast<uint4*>(best + wave * 128 + 4 * lane) =
                uint4{uk[0][0], uk[0][1], uk[0][2], uk[0][3]};
          __syncthreads();                    // all lists are in
          uint32_t mine[2], at_least[2] = {0u, 0u};
#pragma unroll
          for (int t = 0; t < 2; ++t) mine[t] = best[wave * 128 + lane + 64 * t];
          for (int v = 0; v < NW; ++v) {
            const uint32_t* list = best + v * 128;
            uint32_t lo[2] = {0u, 0u}, hi[2] = {128u, 128u};   // entries [0, lo) are >= mine, [hi, 128) are not
#pragma unroll
            for (int step = 0; step < 8; ++step)           // 129 possible answers
#pragma unroll
              for (int t = 0; t < 2; ++t) {
                const bool open = lo[t] < hi[t];
                const uint32_t mid = (lo[t] + hi[t]) >> 1;   // < 128 while the interval is open
                const bool ge = open && list[open ? mid : 0u] >= mine[t];
                lo[t] = ge ? mid + 1 : lo[t];
                hi[t] = (open && !ge) ? mid : hi[t];
              }
#pragma unroll
            for (int t = 0; t < 2; ++t) at_least[t] += lo[t];
          }
          uint32_t cand = 0;
#pragma unroll
          for (int t = 0; t < 2; ++t)
            if (at_least[t] >= (uint32_t)K && mine[t] > cand) cand = mine[t];
          if (cand != 0) atomicMax(&tau_s[0], cand);
          __syncthreads();                    // the threshold is in; the lists may be overwritten
        } else {
          // the beams' 128 group maxima each, through this wave's part of the chunk buffers
          float* gm = reinterpret_cast<float*>(req_lds) + wave * (16 * 128);
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h)
              *reinterpret_cast<float4*>(gm + (4 * g + i) * 128 + c * 8 + h * 4) = float4{
                  half_floor(half_bits_to_float(gmaxp[i >> 1][4 * h] >> (16 * (i & 1)))),
                  half_floor(half_bits_to_float(gmaxp[i >> 1][4 * h + 1] >> (16 * (i & 1)))),
                  half_floor(half_bits_to_float(gmaxp[i >> 1][4 * h + 2] >> (16 * (i & 1)))),
                  half_floor(half_bits_to_float(gmaxp[i >> 1][4 * h + 3] >> (16 * (i & 1))))};
          wave_sync();
#pragma unroll 1
          for (int q = 0; q < 4; ++q) {
            uint32_t mk[4][2];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
              for (int j = 0; j < 2; ++j) mk[r][j] = ordered_bits(gm[(4 * q + r) * 128 + j * 64 + ln]);
            sort_desc<2, 4, uint32_t>(mk);                                // position 2*lane + j
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const uint32_t pick = pick_element<2>(mk[r], (K - 1) & 1);
              const float bnd =
                  unordered_bits((uint32_t)__builtin_amdgcn_readlane((int)pick, (K - 1) >> 1));
              if (lane == 0) my_info[4 * q + r] = bnd;
            }
          }
          wave_sync();
          __syncthreads();                    // maxima read before the next chunk lands on them
        }
      }
    };
    run_sweep(std::integral_constant<int, 0>{});
    for (int attempt = 0;; ++attempt) {
      run_sweep(std::integral_constant<int, 1>{});
      if constexpr (!WHOLE) {
        break;
      } else {
        // More candidates at or above the threshold than the list holds (one beam far ahead of
        // the others gives few of the candidates the threshold was taken from): the K-th best of
        // the listed ones, all of them real candidates, is a tighter threshold; sweep again.
        const int n0 = *req_cnt;              // (the sweep ended with a barrier)
        if (n0 <= kReqListCap || n0 >= kReqForced || attempt == 2) break;
        __syncthreads();                      // everyone has read the counter
        if (wave == 0) {
          WaveTopK<256> f;
          f.init(topbuf, K);
          for (int base = 0; base < kReqListCap; base += 64) f.push(req_list[base + lane]);
          f.compact();
          wave_sync();
          if (lane == 0) {
            tau_s[0] = (uint32_t)(f.buf[K - 1] >> 32);
            *req_cnt = 0;
          }
        }
        __syncthreads();
      }
    }

    if constexpr (WHOLE) {
      const int n = *req_cnt;                 // (the sweep ended with a barrier)
      const bool over = n > kReqListCap;
      if ((int)threadIdx.x < K_in) redo[(int64_t)b * K_in + threadIdx.x] = over ? 1 : 0;
      if (threadIdx.x == 0) la.redo_req[b] = over ? 1 : 0;
      if (!over) {
        if (wave == 0) {
          WaveTopK<256> f;
          f.init(topbuf, K);
          for (int base = 0; base < n; base += 64) f.push(base + lane < n ? req_list[base + lane] : 0ull);
          f.compact();
          wave_sync();
          constexpr int NPLK = (NEZHA_MAX_BEAM + 63) / 64;
#pragma unroll
          for (int j = 0; j < NPLK; ++j) {
            const int p = lane + 64 * j;
            if (p < K) {
              const int64_t o = (int64_t)b * K + p;
              if (p < f.cnt) {
                const uint64_t sk = f.buf[p];
                const uint32_t who = ~(uint32_t)sk;
                const int par = (int)(who >> 24);
                const int32_t code = (int32_t)(who & 0xFFFFFFu);
                la.key_out[o] = (la.key_in ? la.key_in[(int64_t)b * K_in + par] : 0ull) +
                                (uint64_t)(uint32_t)code * la.mult;
                la.score_out[o] = unordered_bits((uint32_t)(sk >> 32));
                la.parent_out[o] = par;
                la.code_out[o] = code;
                fin_parent[p] = par;
                fin_code[p] = code;
              } else {
                la.key_out[o] = kEmpty;
                la.score_out[o] = -INFINITY;
                la.parent_out[o] = -1;
                la.code_out[o] = -1;
                fin_parent[p] = -1;
                fin_code[p] = -1;
              }
            }
          }
          if (lane == 0 && la.count_out) la.count_out[b] = f.cnt;
        }
        __syncthreads();
        if (la.state_out) {
          if (la.transition == NEZHA_TRANSITION_RNN)
            update_states_rnn<true>(a.state, la.E, la.U, la.state_out, b, K, K_in, e, fin_parent,
                                    fin_code, threadIdx.x, blockDim.x);
          else
            update_states<true>(a.state, la.E, la.state_out, b, K, K_in, e, fin_parent, fin_code,
                                threadIdx.x, blockDim.x);
        }
      }
      __syncthreads();                        // the request's LDS state is reused by the next one
      continue;
    }
    // per beam: the K-th largest listed logit, then the entries that belong to the K best
    auto emit = [&](auto npl_c, int q, const int (&n)[2]) {
      constexpr int NPL = decltype(npl_c)::value;
      int ln = lane;
      asm volatile("" : "+v"(ln));
      uint32_t zk[2][NPL], code[2][NPL];
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int j = 0; j < NPL; ++j) {
          const int idx = j * 64 + ln;
          uint64_t ent = 0;
          if (idx < n[r]) ent = my_lists[(2 * q + r) * kReqCap + idx];
          zk[r][j] = idx < n[r] ? ordered_bits(__uint_as_float((uint32_t)(ent >> 32))) : 0u;
          code[r][j] = (uint32_t)ent;
        }
      // A threshold T per beam with exactly K listed keys >= T, or, where keys tie there, the
      // K-th largest key itself: bit by bit from the top, T takes a bit while at least K keys stay
      // at or above it (a compare per register and scalar counting per step; the whole kernel is
      // bound by the number of instructions issued, and a sort of the keys takes three times as
      // many).  The bits that the listed keys share (they lie between the beam's bound and its
      // largest logit: sign, exponent and a little more) are set at the start, and the walk ends
      // as soon as both beams hold exactly K keys, some ten steps later as a rule.
      uint32_t kth[2] = {0u, 0u};
      int held[2], top_bit = -1;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        held[r] = n[r] ? n[r] : K;                          // keys >= kth[r] (no beam: nothing to find)
        if (n[r] == 0) continue;
        uint32_t hi = zk[r][0];
#pragma unroll
        for (int j = 1; j < NPL; ++j) hi = hi > zk[r][j] ? hi : zk[r][j];
        auto wider = [&](uint32_t o) { hi = hi > o ? hi : o; };
        wider(lane_xor<1>(hi, ln));
        wider(lane_xor<2>(hi, ln));
        wider(lane_xor<4>(hi, ln));
        wider(lane_xor<8>(hi, ln));
        wider(lane_xor<16>(hi, ln));
        wider(lane_xor<32>(hi, ln));
        hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)hi);
        const uint32_t lo = ordered_bits(my_info[2 * q + r]);   // every listed logit is >= the bound
        const uint32_t differ = lo ^ hi;
        const int top = differ ? 31 - __builtin_clz(differ) : -1;
        kth[r] = top < 0 ? hi : (hi & ~((2u << top) - 1u));
        top_bit = top > top_bit ? top : top_bit;
      }
#pragma unroll 1
      for (int bit = top_bit; bit >= 0 && (held[0] != K || held[1] != K); --bit) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const uint32_t cand = kth[r] | (1u << bit);
          int at_least = 0;
#pragma unroll
          for (int j = 0; j < NPL; ++j) at_least += __popcll(__ballot(zk[r][j] >= cand));
          if (at_least >= K) {
            kth[r] = cand;
            held[r] = at_least;
          }
        }
      }
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        if (n[r] == 0) continue;
        const uint32_t tau = kth[r];
        int n_gt = 0, n_eq = 0;
#pragma unroll
        for (int j = 0; j < NPL; ++j) {
          n_gt += __popcll(__ballot(zk[r][j] > tau));
          n_eq += __popcll(__ballot(zk[r][j] == tau));
        }
        const int need = K - n_gt;                                      // >= 1 of the n_eq ties
        uint32_t cthr = 0;                                              // ~code must reach this
        if (n_eq > need) {
          constexpr int NP2 = NPL <= 1 ? 1 : NPL <= 2 ? 2 : NPL <= 4 ? 4 : 8;   // the sort's size
          uint32_t ck[1][NP2];
#pragma unroll
          for (int j = 0; j < NP2; ++j) ck[0][j] = (j < NPL && zk[r][j < NPL ? j : 0] == tau) ? ~code[r][j < NPL ? j : 0] : 0u;
          sort_desc<NP2, 1, uint32_t>(ck);
          cthr = (uint32_t)__builtin_amdgcn_readlane(
              (int)pick_element<NP2>(ck[0], (need - 1) % NP2), (need - 1) / NP2);
        }
        const int64_t row = (int64_t)b * K_in + wave * 16 + 2 * q + r;
        const float lse = my_info[16 + 2 * q + r];
        int base = 0;
#pragma unroll
        for (int j = 0; j < NPL; ++j) {
          const bool take = zk[r][j] > tau || (zk[r][j] == tau && ~code[r][j] >= cthr);
          const uint64_t bal = __ballot(take);
          const int p = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
          if (take && p < K) {
            a.cand_code[row * K + p] = (int32_t)code[r][j];
            a.cand_logp[row * K + p] = unordered_bits(zk[r][j]) - lse;
          }
          base += __popcll(bal);
        }
      }
    };
#pragma unroll 1
    for (int q = 0; q < 8; ++q) {
      const int ra = wave * 16 + 2 * q;
      if (ra >= K_in) break;
      int n[2];
      // (a count that was pushed past the list's size by up to 16 lanes still fits its 16 bits)
      const unsigned long long word = my_cnt4[q >> 1];
      const uint32_t pair = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(word >> (32 * (q & 1))));
      n[0] = (int)(pair & 0xFFFFu);
      n[1] = ra + 1 < K_in ? (int)(pair >> 16) : 0;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const bool over = n[r] > kReqCap;
        if (lane == 0 && ra + r < K_in) redo[(int64_t)b * K_in + ra + r] = over ? 1 : 0;
        if (over) n[r] = 0;
      }
      const int most = n[0] > n[1] ? n[0] : n[1];
      if (most == 0) continue;
      if (most <= 64) emit(std::integral_constant<int, 1>{}, q, n);
      else if (most <= 128) emit(std::integral_constant<int, 2>{}, q, n);
      else if (most <= 256) emit(std::integral_constant<int, 4>{}, q, n);
      else emit(std::integral_constant<int, 6>{}, q, n);
    }
    wave_sync();                              // counters and info are rewritten for the next request
  }
}

// ---- whole level in one kernel for small shapes (bf16, T_l <= 512, K and K_in <= 32) -----------
// One workgroup of 16 waves per request.  Phase A: the request's K_in x T_l logits by MFMA into
// LDS (the user-part row is the accumulators' start value).  Phase B: two rows per wave,
// two_rows_topk, the per-beam lists stay in LDS.  Phase C: every candidate gets its cumulative
// score, its Eq. 4 index and (last level) its hash-set probe; the K best survivors are found as in
// merge_kernel.  Then the additive Transition.  Nothing but the level's outputs leaves the chip.
struct LevelArgs {
  const void* state_in;     // [B, K_in, e] or NULL
  const void* Wbeam;        // packed beam part of W
  const float* A;           // [B, V] user part
  const uint64_t* key_in;   // [B, K_in] or NULL
  const float* score_in;    // [B, K_in] or NULL
  const void* E;            // [V, e] (used when state_out != NULL)
  SetView set;              // slots == NULL: no verification
  uint64_t mult;            // prod_{j<level} T_j
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  void* state_out;          // or NULL
  int32_t* count_out;       // or NULL
  int K_in, K, V, e;
  const void* U;            // [e, e] row major (recurrent Transition), else unused
  int transition;
};
constexpr int kLevelWaves = 16, kLevelRows = 32, kLevelBeam = 32;
// What a workgroup that runs several levels in one launch carries from one level to the next:
// which of the two LDS state buffers holds the states of the entering beams.  (Requesting the
// next level's weight operands a level ahead into registers was tried and lost: the kernel is
// bound by instruction issue with four waves per SIMD, and the extra live registers cost more
// than the hidden latency gained.)
struct LevelCarry {
  int state_buf;        // 0 / 1: that LDS buffer; -1: the states are read from global memory
};
constexpr int kLevelStateElems = kLevelBeam * 256;     // one LDS state buffer: 32 beams x e <= 256

template <int KST, int NVT>
__device__ __forceinline__ void level_small_body(const LevelArgs& a, uint64_t* lds, bool has_next,
                                                 LevelCarry& carry) {
  constexpr int CAP = 256;
  uint64_t* scratch = lds;                                            // [16 waves][CAP]
  uint64_t* lists = scratch + kLevelWaves * CAP;                      // [32 rows][32]
  uint64_t* keys2 = lists + kLevelRows * kLevelBeam;                  // [32*32]
  uint64_t* topbuf = keys2 + kLevelRows * kLevelBeam;                 // [CAP]
  uint16_t* state_lds = reinterpret_cast<uint16_t*>(topbuf + CAP);    // [2][32 beams][e]
  float* ztile = reinterpret_cast<float*>(state_lds + 2 * kLevelStateElems);   // [32][V]
  __shared__ float row_lse[kLevelRows];
  __shared__ uint64_t bounds[kLevelWaves];
  __shared__ int32_t fin_parent[NEZHA_MAX_BEAM], fin_code[NEZHA_MAX_BEAM];
  // the wave id is made scalar: loops and branches on it are then uniform for the compiler
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  const int b = blockIdx.x;
  const int V = a.V, K = a.K, K_in = a.K_in, e = a.e;
  const bool has_beam = a.state_in != nullptr;
  const int n_ct = V / 16;
  const int RT = (K_in + 15) / 16;                                    // 1 or 2 row tiles

  {  // phase A: wave w takes column tiles w, w+16, ... for both row tiles (same W operands).
     // Every load of the first tile is issued before anything waits: one memory round trip.
    constexpr int KS = KST;                                           // e = 32 * KST exactly
    uint4 w[KST];
    float start = 0.f;
    int ct = wave;
    auto fetch = [&](int t) {
      if (has_beam) {
        const uint4* wp = static_cast<const uint4*>(a.Wbeam) + (int64_t)t * KS * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) w[ks] = load_global_u4(wp + ks * 64);
      }
      start = as_global(a.A)[(int64_t)b * V + t * 16 + c];
    };
    if (ct < n_ct) fetch(ct);
    bf16x8 fa16[2][KST];
    if (has_beam) {
      const uint16_t* st = static_cast<const uint16_t*>(a.state_in) + (int64_t)b * K_in * e;
      const uint16_t* sl = state_lds + (carry.state_buf > 0 ? kLevelStateElems : 0);
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        const int row = rt * 16 + c;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) {
          uint4 v = uint4{0, 0, 0, 0};
          if (row < K_in) {
            if (carry.state_buf >= 0)     // (two loads, not one load through a chosen pointer)
              v = *reinterpret_cast<const uint4*>(sl + row * e + ks * 32 + 8 * g);
            else
              v = load_global_u4(st + (int64_t)row * e + ks * 32 + 8 * g);
          }
          fa16[rt][ks] = *reinterpret_cast<bf16x8*>(&v);
        }
      }
    }
    for (; ct < n_ct; ct += kLevelWaves) {
      floatx4 acc0 = floatx4{start, start, start, start}, acc1 = acc0;
      if (has_beam) {
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) {
          acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              fa16[0][ks], *reinterpret_cast<bf16x8*>(&w[ks]), acc0, 0, 0, 0);
          if (RT > 1)
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                fa16[1][ks], *reinterpret_cast<bf16x8*>(&w[ks]), acc1, 0, 0, 0);
        }
      }
      const int here = ct;
      if (ct + kLevelWaves < n_ct) fetch(ct + kLevelWaves);           // next tile's operands
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ztile[(4 * g + i) * V + here * 16 + c] = acc0[i];
        if (RT > 1) ztile[(16 + 4 * g + i) * V + here * 16 + c] = acc1[i];
      }
    }
  }
  __syncthreads();

  const bool verify = a.set.slots != nullptr;
  {  // phase B: rows 2*wave and 2*wave+1
    const int r0 = wave * 2;
    if (r0 < K_in) {
      two_rows_topk<NVT, CAP>(ztile + r0 * V, ztile + (r0 + 1) * V, true, r0 + 1 < K_in, V, K,
                              scratch + wave * CAP, [&](int rr, int p, uint64_t kk, float lse) {
                                lists[(r0 + rr) * kLevelBeam + p] = kk;
                                if (p == 0) row_lse[r0 + rr] = lse;
                              });
    }
  }
  if (K_in == 1) {
    // One entering beam (level 1): its K best codes are the level's beams, so wave 0, which has
    // just found them, also does the probes and the ordering by score: no candidate matrix, no
    // bounds, two barriers fewer.
    if (wave == 0) {
      wave_sync();
      uint64_t sk1[1][1] = {{0ull}};
      if (lane < K) {
        const uint64_t zk = lists[lane];
        const uint32_t code = ~(uint32_t)zk;
        const float logp = unordered_bits((uint32_t)(zk >> 32)) - row_lse[0];
        const float score = (a.score_in ? as_global(a.score_in)[b] : 0.f) + logp;
        const uint64_t pkey = a.key_in ? as_global(a.key_in)[b] : 0ull;
        bool ok = pkey != kEmpty;                                       // an empty beam slot has no children
        if (verify && ok) ok = set_contains(a.set, pkey, code);
        if (ok) sk1[0][0] = ((uint64_t)ordered_bits(score) << 32) | (uint32_t)~(uint32_t)lane;
      }
      sort_desc<1, 1, uint64_t>(sk1);                                   // (score, place in code order)
      const int cnt = __popcll(__ballot(sk1[0][0] != 0ull));
      if (lane < K) {
        const int64_t o = (int64_t)b * K + lane;
        if (lane < cnt) {
          const uint64_t s2 = sk1[0][0];
          const int32_t code = (int32_t)(~(uint32_t)lists[(int)(~(uint32_t)s2)]);
          as_global(a.key_out)[o] =
              (a.key_in ? as_global(a.key_in)[b] : 0ull) + (uint64_t)(uint32_t)code * a.mult;
          as_global(a.score_out)[o] = unordered_bits((uint32_t)(s2 >> 32));
          as_global(a.parent_out)[o] = 0;
          as_global(a.code_out)[o] = code;
          fin_parent[lane] = 0;
          fin_code[lane] = code;
        } else {
          as_global(a.key_out)[o] = kEmpty;
          as_global(a.score_out)[o] = -INFINITY;
          as_global(a.parent_out)[o] = -1;
          as_global(a.code_out)[o] = -1;
          fin_parent[lane] = -1;
          fin_code[lane] = -1;
        }
      }
      if (lane == 0 && a.count_out) as_global(a.count_out)[b] = cnt;
    }
  } else {
    __syncthreads();

    // phase C: candidate (parent p, rank r) -> sort key (ordered score, ~(p*K+r)), 0 if rejected
    const int n_c = K_in * K;                                           // <= 1024 = one per thread
    uint64_t sk = 0;
    if (tid < n_c) {
      const int p = tid / K;
      const uint64_t zk = lists[p * kLevelBeam + (tid - p * K)];
      const uint32_t code = ~(uint32_t)zk;
      const float logp = unordered_bits((uint32_t)(zk >> 32)) - row_lse[p];
      const float score = (a.score_in ? as_global(a.score_in)[b * K_in + p] : 0.f) + logp;
      const uint64_t pkey = a.key_in ? as_global(a.key_in)[b * K_in + p] : 0ull;
      bool ok = pkey != kEmpty;                                         // an empty beam slot has no children
      if (verify && ok) ok = set_contains(a.set, pkey, code);
      if (ok) sk = ((uint64_t)ordered_bits(score) << 32) | (uint32_t)~(uint32_t)tid;
      keys2[tid] = sk;
    }
    {
      // K-th largest score of this wave's 64 candidates (scores alone: a bound may ignore ties)
      uint32_t mk[1][1] = {{(uint32_t)(sk >> 32)}};
      sort_desc<1, 1, uint32_t>(mk);                                    // K <= 32 <= 64
      const uint64_t bound = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mk[0][0], K - 1) << 32;
      if (lane == 0) bounds[wave] = bound;
    }
    __syncthreads();
    if (wave == 0) {
      uint64_t tau = bounds[0];
  #pragma unroll
      for (int w = 1; w < kLevelWaves; ++w) tau = bounds[w] > tau ? bounds[w] : tau;
      WaveTopK<CAP> f;
      f.init(topbuf, K);
      f.tau = tau ? tau - 1ull : 0ull;                                  // keys >= tau enter
      for (int base = 0; base < n_c; base += 64) f.push(base + lane < n_c ? keys2[base + lane] : 0ull);
      f.compact();
      wave_sync();
      if (lane < K) {
        const int64_t o = (int64_t)b * K + lane;
        if (lane < f.cnt) {
          const uint64_t s2 = f.buf[lane];
          const int i = (int)(~(uint32_t)s2);
          const int par = i / K;
          const int32_t code = (int32_t)(~(uint32_t)lists[par * kLevelBeam + (i - par * K)]);
          as_global(a.key_out)[o] =
              (a.key_in ? as_global(a.key_in)[b * K_in + par] : 0ull) + (uint64_t)(uint32_t)code * a.mult;
          as_global(a.score_out)[o] = unordered_bits((uint32_t)(s2 >> 32));
          as_global(a.parent_out)[o] = par;
          as_global(a.code_out)[o] = code;
          fin_parent[lane] = par;
          fin_code[lane] = code;
        } else {
          as_global(a.key_out)[o] = kEmpty;
          as_global(a.score_out)[o] = -INFINITY;
          as_global(a.parent_out)[o] = -1;
          as_global(a.code_out)[o] = -1;
          fin_parent[lane] = -1;
          fin_code[lane] = -1;
        }
      }
      if (lane == 0 && a.count_out) as_global(a.count_out)[b] = f.cnt;
    }
  }
  __syncthreads();
  if (a.state_out) {
    // with a next level in the same launch the new states also go to the other LDS buffer
    const uint16_t* lds_in =
        (has_beam && carry.state_buf >= 0) ? state_lds + (carry.state_buf > 0 ? kLevelStateElems : 0)
                                           : nullptr;
    const int out_buf = carry.state_buf > 0 ? 0 : 1;
    uint16_t* lds_out = has_next ? state_lds + (out_buf > 0 ? kLevelStateElems : 0) : nullptr;
    if (a.transition == NEZHA_TRANSITION_RNN)
      update_states_rnn<true>(a.state_in, a.E, a.U, a.state_out, b, K, K_in, e, fin_parent, fin_code,
                              tid, 64 * kLevelWaves, lds_in, lds_out);
    else
      update_states<true>(a.state_in, a.E, a.state_out, b, K, K_in, e, fin_parent, fin_code, tid,
                          64 * kLevelWaves, lds_in, lds_out);
    carry.state_buf = has_next ? out_buf : -1;
  }
}

template <int KST, int NVT>
__global__ __launch_bounds__(64 * kLevelWaves, 1) void level_small_kernel(LevelArgs a) {
  extern __shared__ __align__(16) uint64_t lds[];
  LevelCarry carry;
  carry.state_buf = -1;
  level_small_body<KST, NVT>(a, lds, false, carry);
}

// All levels of a decode in one launch: the workgroup of request b runs level 1, 2, ... in turn.
// Keys and scores of the beams are read back from the level's output arrays in global memory
// (written by the same workgroup); the states stay in LDS.
struct DecodeArgs {
  LevelArgs lv[NEZHA_MAX_LEVELS];
  int L;
};
template <int KST, int NVT>
__global__ __launch_bounds__(64 * kLevelWaves, 1) void decode_small_kernel(DecodeArgs d) {
  extern __shared__ __align__(16) uint64_t lds[];
  LevelCarry carry;
  carry.state_buf = -1;
  for (int l = 0; l < d.L; ++l) {
    level_small_body<KST, NVT>(d.lv[l], lds, l + 1 < d.L, carry);
    __threadfence_block();      // this level's outputs are the next level's inputs
    __syncthreads();
  }
}

// ---- host side ---------------------------------------------------------------------------------
#include "wide_beam.h"

struct Plan {
  size_t wp_off, a_off, code_off, logp_off, list_off, redo_off, redo_req_off, total;
  int cap;
  bool per_request;   // expand_request_kernel takes the expansion
  bool wide;          // beams wider than NEZHA_MAX_BEAM: code_off is where the level's logits go
};
inline bool wide_beam(int K, int K_in) { return K > NEZHA_MAX_BEAM || K_in > NEZHA_MAX_BEAM; }
// wide_fused_bf16_kernel: waves that share the code tiles of one group of 32 beams, so that even
// a small batch gives the chip a few thousand waves; at most 16 (their parts are merged per beam).
inline int wide_fused_col_splits(int B, int K_in, int V) {
  const int64_t groups = (int64_t)B * ((K_in + 31) / 32);
  int64_t cs = (4096 + groups - 1) / (groups > 0 ? groups : 1);
  const int64_t most = V / 16 < 16 ? V / 16 : 16;
  return (int)(cs < 1 ? 1 : cs > most ? most : cs);
}

// Which kernels take a level is a function of the shape alone, so that the workspace can be sized
// without the buffers.
inline bool level_fits_one_launch(bool bf16, int K, int K_in, int V, int e) {
  return bf16 && K <= kLevelBeam && K_in <= kLevelRows && V <= 512 &&
         (e == 32 || e == 64 || e == 128 || e == 256);
}
inline bool codebook_fits_lds(bool bf16, int K, int V) { return bf16 && V <= 1024 && K <= 64; }
inline bool expand_per_request(bool bf16, int K, int K_in, int V, int e) {
  // (T_l <= 32768: the kernel counts a beam's list entries, at most T_l plus 16 flags of 385, in 16 bits)
  return bf16 && K_in >= 16 && V <= (1 << 15) && (e == 32 || e == 64 || e == 128 || e == 256) &&
         !level_fits_one_launch(bf16, K, K_in, V, e) && !codebook_fits_lds(bf16, K, V);
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_desc(const nezha_step_desc* dsc, Plan* plan) {
  if (!dsc) return fail(NEZHA_EINVAL, "desc is NULL");
  if (dsc->B < 0) return fail(NEZHA_EINVAL, "B = %d is negative", dsc->B);
  if (dsc->L < 1 || dsc->L > NEZHA_MAX_LEVELS)
    return fail(NEZHA_EINVAL, "L = %d outside 1..%d", dsc->L, NEZHA_MAX_LEVELS);
  if (dsc->level < 1 || dsc->level > dsc->L)
    return fail(NEZHA_EINVAL, "level = %d outside 1..L = %d", dsc->level, dsc->L);
  if (!dsc->radices) return fail(NEZHA_EINVAL, "radices is NULL");
  uint64_t mult[NEZHA_MAX_LEVELS];
  if (!radix_multipliers(dsc->L, dsc->radices, mult))
    return fail(NEZHA_ERANGE, "radices must be >= 1 with a product of at most 2^64-1");
  const int V = dsc->radices[dsc->level - 1];
  if (dsc->K < 1 || dsc->K > NEZHA_MAX_WIDE_BEAM || dsc->K > V)
    return fail(NEZHA_EINVAL, "K = %d outside 1..min(T_level = %d, %d)", dsc->K, V,
                NEZHA_MAX_WIDE_BEAM);
  if (dsc->K_in < 1 || dsc->K_in > NEZHA_MAX_WIDE_BEAM)
    return fail(NEZHA_EINVAL, "K_in = %d outside 1..%d", dsc->K_in, NEZHA_MAX_WIDE_BEAM);
  if (dsc->dtype != NEZHA_F32 && dsc->dtype != NEZHA_BF16)
    return fail(NEZHA_EINVAL, "unknown dtype %d", (int)dsc->dtype);
  if (dsc->w_packed != 0 && (dsc->w_packed != 1 || dsc->dtype != NEZHA_BF16))
    return fail(NEZHA_EINVAL, "w_packed must be 0, or 1 with NEZHA_BF16");
  if (V % 16 != 0) return fail(NEZHA_EINVAL, "T_level = %d is not a multiple of 16", V);
  const bool bf16 = dsc->dtype == NEZHA_BF16;
  if (dsc->d < 1 || (bf16 && dsc->d % 32 != 0))
    return fail(NEZHA_EINVAL, "d = %d must be >= 1 (a multiple of 32 for bf16)", dsc->d);
  if (dsc->e < 1 || dsc->e > 256 || dsc->e % (bf16 ? 32 : 4) != 0)
    return fail(NEZHA_EINVAL, "e = %d must be a multiple of %d in 1..256", dsc->e, bf16 ? 32 : 4);
  if (dsc->h_row_stride < dsc->d || (bf16 && dsc->h_row_stride % 8 != 0))
    return fail(NEZHA_EINVAL, "h_row_stride = %lld must be >= d (a multiple of 8 for bf16)",
                (long long)dsc->h_row_stride);
  if ((int64_t)dsc->B * dsc->K_in > 0x7FFFFFFF / NEZHA_MAX_BEAM)
    return fail(NEZHA_EINVAL, "B * K_in too large");
  const bool wide = wide_beam(dsc->K, dsc->K_in);
  if (wide && (int64_t)dsc->K_in * V > 0x7FFFFFFF)
    return fail(NEZHA_EINVAL, "K_in * T_level = %lld exceeds 2^31-1 (beams wider than %d)",
                (long long)dsc->K_in * V, NEZHA_MAX_BEAM);
  if (plan) {
    const size_t rows = (size_t)dsc->B * dsc->K_in;
    size_t off = 0;
    plan->wp_off = off;
    if (bf16 && !dsc->w_packed)
      off += align_up((size_t)(packed_user_elems(dsc->d, V) + (int64_t)dsc->e * V) * 2, 256);
    plan->a_off = off;
    off += align_up((size_t)dsc->B * V * 4, 256);
    plan->code_off = off;
    plan->wide = wide;
    if (wide) {
      off += align_up(rows * (size_t)V * 4, 256);
      plan->logp_off = plan->list_off = plan->redo_off = plan->redo_req_off = off;
      // the largest keys of every share of a request (batches too small for one workgroup per
      // request), the request's list of keys at or above the bound / found in the set, its length
      const int splits = wide_select_splits(dsc->B);
      const int groups = (dsc->K_in + 31) / 32;
      const int cs = wide_fused_col_splits(dsc->B, dsc->K_in, V);
      size_t n_tops = (size_t)splits * dsc->K;
      if ((size_t)groups * cs * 128 > n_tops) n_tops = (size_t)groups * cs * 128;
      off += align_up((size_t)dsc->B * n_tops * 4, 256);
      plan->list_off = off;
      off += align_up((size_t)dsc->B * kWideListCap * 8, 256);
      plan->redo_off = off;
      off += align_up((size_t)dsc->B * 4, 256);
      plan->redo_req_off = off;                          // (max, sum) of every beam and column share
      off += align_up(rows * (size_t)cs * 8, 256);
      plan->per_request = false;
      plan->total = off;
      plan->cap = 0;
      return NEZHA_OK;
    }
    off += align_up(rows * dsc->K * 4, 256);
    plan->logp_off = off;
    off += align_up(rows * dsc->K * 4, 256);
    plan->per_request = expand_per_request(bf16, dsc->K, dsc->K_in, V, dsc->e);
    plan->list_off = plan->redo_off = plan->redo_req_off = off;
    if (plan->per_request) {
      const size_t groups = dsc->B < kReqMaxGroups ? (size_t)dsc->B : (size_t)kReqMaxGroups;
      off += align_up(groups * 128 * kReqCap * 8, 256);
      plan->redo_off = off;
      off += align_up(rows, 256);
      plan->redo_req_off = off;
      off += align_up((size_t)dsc->B, 256);
    }
    plan->total = off < 256 ? 256 : off;
    plan->cap = dsc->K <= 32 ? 128 : 256;
  }
  return NEZHA_OK;
}

template <typename Kern>
int allow_lds(Kern kern, size_t bytes) {
  if (bytes > 64 * 1024) {
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (err != hipSuccess)
      return fail(NEZHA_EHIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(err));
  }
  return NEZHA_OK;
}

// Products with fewer outputs than this are "small": 128 x 128 tiles would leave most of the 256
// CUs without a workgroup (B = T_l = 1024: 64 tiles), so they get 32 x 64 tiles, and their k
// loop runs in four parts side by side (user_gemm_tile, KSPLIT).
constexpr int64_t kSmallGemmElems = (int64_t)128 * 128 * 256;
constexpr int64_t kBigGemmElems = (int64_t)256 * 256 * 128;   // from here on: 256 x 256 tiles
inline bool small_gemm_splits_k(int d) { return (d / 32) % 4 == 0 && d >= 256; }

int launch_pack(const nezha_step_desc* desc, const void* W_l, uint16_t* Wp, hipStream_t stream) {
  const int d = desc->d, e = desc->e, V = desc->radices[desc->level - 1];
  const int64_t total = (int64_t)((V + 31) / 32) * (d / 16) * 64 + (int64_t)(V / 16) * (e / 32) * 64;
  ProfileScope prof(kPackWeights, stream);
  hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const uint16_t*>(W_l), Wp, d, e, V);
  NEZHA_HIP_CHECK(hipGetLastError());
  return NEZHA_OK;
}

// a1: packs W_l (bf16, unless it comes packed) and forms A = H_l * W_l[0:d] on `stream`.
int launch_user_part(const nezha_step_desc* desc, const void* H_l, const void* W_l, uint16_t* Wp,
                     float* A, hipStream_t stream) {
  const int B = desc->B, d = desc->d;
  const int V = desc->radices[desc->level - 1];
  const bool bf16 = desc->dtype == NEZHA_BF16;
  int rc = NEZHA_OK;
  if (bf16) {
    if (!desc->w_packed) {
      rc = launch_pack(desc, W_l, Wp, stream);
      if (rc != NEZHA_OK) return rc;
    }
    ProfileScope prof(kUserGemm, stream);
    const uint16_t* Hp = static_cast<const uint16_t*>(H_l);
#define LAUNCH_GEMM(NWM, NWN, TM, TN, KSPLIT)                                                  \
  do {                                                                                         \
    constexpr int BM = NWM * TM * 32, BN = NWN * TN * 32;                                      \
    const int tiles_m = (B + BM - 1) / BM, tiles_n = (V + BN - 1) / BN;                        \
    const size_t lds = (size_t)KSPLIT * kGemmBuffers * (BM * 4) * sizeof(uint4);               \
    rc = allow_lds(user_gemm_bf16_kernel<NWM, NWN, TM, TN, KSPLIT>, lds);                      \
    if (rc != NEZHA_OK) return rc;                                                             \
    hipLaunchKernelGGL((user_gemm_bf16_kernel<NWM, NWN, TM, TN, KSPLIT>),                      \
                       dim3(tiles_m * tiles_n), dim3(64 * NWM * NWN * KSPLIT), lds, stream, Hp, \
                       desc->h_row_stride, (const uint16_t*)Wp, A, B, d, V, tiles_n,           \
                       tiles_m * tiles_n);                                                     \
  } while (0)
    const int64_t out_elems = (int64_t)B * V;
    if (out_elems >= kBigGemmElems) {                                             // 256 x 256 tiles
      const int tiles_m = (B + 255) / 256, tiles_n = (V + 255) / 256;
      rc = allow_lds(user_gemm_big_kernel, big_gemm_lds());
      if (rc != NEZHA_OK) return rc;
      hipLaunchKernelGGL(user_gemm_big_kernel, dim3(tiles_m * tiles_n), dim3(256), big_gemm_lds(),
                         stream, Hp, desc->h_row_stride, (const uint16_t*)Wp, A, B, d, V, tiles_n,
                         tiles_m * tiles_n);
    }
    else if (out_elems >= kSmallGemmElems) LAUNCH_GEMM(2, 2, 2, 2, 1);             // 128 x 128 tiles
    // small products: the same tiles and the same order of summation as the grouped launch of
    // nezha_user_projection_levels, so that both give the same bits
    else if (small_gemm_splits_k(d)) LAUNCH_GEMM(1, 2, 1, 1, 4);                  // 32 x 64, k in four parts
    else LAUNCH_GEMM(1, 2, 1, 1, 1);                                              // 32 x 64 tiles
#undef LAUNCH_GEMM
    NEZHA_HIP_CHECK(hipGetLastError());
  } else {
    dim3 grid((V + 255) / 256, B);
    ProfileScope prof(kUserGemm, stream);
    hipLaunchKernelGGL(user_gemm_f32_kernel, grid, dim3(256), 0, stream,
                       static_cast<const float*>(H_l), desc->h_row_stride,
                       static_cast<const float*>(W_l), A, B, d, V);
    NEZHA_HIP_CHECK(hipGetLastError());
  }

  return NEZHA_OK;
}

}  // namespace
}  // namespace nezha

using namespace nezha;

extern "C" {

int nezha_user_projection(const nezha_step_desc* desc, const void* H_l, const void* W_l,
                          float* A_out, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Plan plan;
  int rc = check_desc(desc, &plan);
  if (rc != NEZHA_OK) return rc;
  if (desc->B == 0) return NEZHA_OK;
  const bool bf16 = desc->dtype == NEZHA_BF16;
  if (!H_l || !W_l || !A_out) return fail(NEZHA_EINVAL, "H_l, W_l or A_out is NULL");
  if (bf16 && !desc->w_packed && (!workspace || workspace_bytes < plan.a_off))
    return fail(NEZHA_EINVAL, "workspace has %zu bytes, %zu needed", workspace_bytes, plan.a_off);
  if (bf16 && !desc->w_packed && (reinterpret_cast<uintptr_t>(workspace) & 255))
    return fail(NEZHA_EINVAL, "workspace is not 256-byte aligned");
  const uintptr_t hw_mask = bf16 ? 15 : 3;
  if ((reinterpret_cast<uintptr_t>(H_l) | reinterpret_cast<uintptr_t>(W_l)) & hw_mask)
    return fail(NEZHA_EINVAL, "H_l and W_l must be %d-byte aligned", (int)hw_mask + 1);
  if (reinterpret_cast<uintptr_t>(A_out) & 15) return fail(NEZHA_EINVAL, "A_out is not 16-byte aligned");
  uint16_t* Wp = desc->w_packed ? static_cast<uint16_t*>(const_cast<void*>(W_l))
                                : static_cast<uint16_t*>(workspace);
  return launch_user_part(desc, H_l, W_l, Wp, A_out, (hipStream_t)hip_stream);
}

int nezha_user_projection_levels(const nezha_step_desc* desc, int32_t n_levels,
                                 const void* const* H, const void* const* W_packed,
                                 float* const* A_out, void* hip_stream) {
  if (!desc) return fail(NEZHA_EINVAL, "desc is NULL");
  nezha_step_desc probe = *desc;
  probe.level = 1;
  probe.K = 1;
  probe.K_in = 1;
  if (n_levels < 1 || n_levels > desc->L) return fail(NEZHA_EINVAL, "n_levels outside 1..L");
  if (desc->dtype != NEZHA_BF16 || !desc->w_packed)
    return fail(NEZHA_EINVAL, "needs NEZHA_BF16 weights packed by nezha_pack_weights");
  if (!H || !W_packed || !A_out) return fail(NEZHA_EINVAL, "a pointer array is NULL");
  // small projections are bound by the length of the k loop, not by the tile: 32 x 64 tiles by two
  // waves give the chip more workgroups than 64 x 64 ones (9.2 against 10.5 us for three 256 x 512
  // x 256 products)
  constexpr int kGroupedBM = 32, kGroupedBN = 64;
  GemmGroup grp;
  grp.n = n_levels;
  int tiles = 0;
  const int B = desc->B, d = desc->d;
  for (int i = 0; i < n_levels; ++i) {
    probe.level = i + 1;
    int rc = check_desc(&probe, nullptr);
    if (rc != NEZHA_OK) return rc;
    if (!H[i] || !W_packed[i] || !A_out[i]) return fail(NEZHA_EINVAL, "a level's pointer is NULL");
    if ((reinterpret_cast<uintptr_t>(H[i]) | reinterpret_cast<uintptr_t>(W_packed[i]) |
         reinterpret_cast<uintptr_t>(A_out[i])) & 15)
      return fail(NEZHA_EINVAL, "H, W_packed and A_out must be 16-byte aligned");
    const int V = desc->radices[i];
    grp.H[i] = static_cast<const uint16_t*>(H[i]);
    grp.Wu[i] = static_cast<const uint16_t*>(W_packed[i]);
    grp.A[i] = A_out[i];
    grp.V[i] = V;
    grp.tiles_n[i] = (V + kGroupedBN - 1) / kGroupedBN;
    grp.tile_begin[i] = tiles;
    tiles += ((B + kGroupedBM - 1) / kGroupedBM) * grp.tiles_n[i];
  }
  grp.tile_begin[n_levels] = tiles;
  for (int i = n_levels; i < NEZHA_MAX_LEVELS; ++i) {
    grp.H[i] = nullptr;
    grp.Wu[i] = nullptr;
    grp.A[i] = nullptr;
    grp.V[i] = 0;
    grp.tiles_n[i] = 0;
    grp.tile_begin[i + 1] = tiles;
  }
  if (B == 0) return NEZHA_OK;
  hipStream_t stream = (hipStream_t)hip_stream;
  int max_v = 0;
  for (int i = 0; i < n_levels; ++i) max_v = desc->radices[i] > max_v ? desc->radices[i] : max_v;
  int min_v = max_v;
  for (int i = 0; i < n_levels; ++i) min_v = desc->radices[i] < min_v ? desc->radices[i] : min_v;
  if ((int64_t)B * min_v >= kBigGemmElems) {
    // the largest projections: the 256 x 256 tiles of all levels in one launch
    GemmGroup big = grp;
    int big_tiles = 0;
    const int tiles_m = (B + 255) / 256;
    for (int i = 0; i < n_levels; ++i) {
      big.tiles_n[i] = (desc->radices[i] + 255) / 256;
      big.tile_begin[i] = big_tiles;
      big_tiles += tiles_m * big.tiles_n[i];
    }
    for (int i = n_levels; i <= NEZHA_MAX_LEVELS; ++i) big.tile_begin[i] = big_tiles;
    int rc = allow_lds(user_gemm_big_grouped_kernel, big_gemm_lds());
    if (rc != NEZHA_OK) return rc;
    ProfileScope prof(kUserGemm, stream);
    hipLaunchKernelGGL(user_gemm_big_grouped_kernel, dim3(big_tiles), dim3(256), big_gemm_lds(),
                       stream, big, desc->h_row_stride, B, d);
    NEZHA_HIP_CHECK(hipGetLastError());
    return NEZHA_OK;
  }
  if ((int64_t)B * max_v >= kSmallGemmElems) {
    // large projections fill the chip on their own: one launch each, with the large tiles
    for (int i = 0; i < n_levels; ++i) {
      probe.level = i + 1;
      int rc = launch_user_part(&probe, H[i], W_packed[i],
                                static_cast<uint16_t*>(const_cast<void*>(W_packed[i])), A_out[i],
                                stream);
      if (rc != NEZHA_OK) return rc;
    }
    return NEZHA_OK;
  }
  ProfileScope prof(kUserGemm, stream);
  if (small_gemm_splits_k(d)) {
    // the k range in four parts, each by its own pair of waves; LDS: the four groups' H buffers,
    // later three groups' partial results (2 waves x 16 x 64 floats each)
    constexpr size_t lds = (size_t)4 * kGemmBuffers * (kGroupedBM * 4) * sizeof(uint4);
    static_assert(lds >= (size_t)3 * 2 * 16 * 64 * 4, "room for the partial results");
    hipLaunchKernelGGL((user_gemm_bf16_grouped_kernel<1, 2, 1, 1, 4>), dim3(tiles), dim3(512), lds,
                       stream, grp, desc->h_row_stride, B, d);
  } else {
    const size_t lds = (size_t)kGemmBuffers * (kGroupedBM * 4) * sizeof(uint4);
    hipLaunchKernelGGL((user_gemm_bf16_grouped_kernel<1, 2, 1, 1, 1>), dim3(tiles), dim3(128), lds,
                       stream, grp, desc->h_row_stride, B, d);
  }
  NEZHA_HIP_CHECK(hipGetLastError());
  return NEZHA_OK;
}

size_t nezha_packed_weights_bytes(const nezha_step_desc* desc) {
  if (check_desc(desc, nullptr) != NEZHA_OK || desc->dtype != NEZHA_BF16) return 0;
  const int V = desc->radices[desc->level - 1];
  return align_up((size_t)(packed_user_elems(desc->d, V) + (int64_t)desc->e * V) * 2, 256);
}

int nezha_pack_weights(const nezha_step_desc* desc, const void* W_l, void* W_packed,
                       void* hip_stream) {
  int rc = check_desc(desc, nullptr);
  if (rc != NEZHA_OK) return rc;
  if (desc->dtype != NEZHA_BF16) return fail(NEZHA_EINVAL, "only NEZHA_BF16 weights are packed");
  if (!W_l || !W_packed) return fail(NEZHA_EINVAL, "W_l or W_packed is NULL");
  if ((reinterpret_cast<uintptr_t>(W_l) | reinterpret_cast<uintptr_t>(W_packed)) & 15)
    return fail(NEZHA_EINVAL, "W_l and W_packed must be 16-byte aligned");
  return launch_pack(desc, W_l, static_cast<uint16_t*>(W_packed), (hipStream_t)hip_stream);
}

int nezha_bench_mfma_rate(const void* operands, size_t bytes, int iters, int workgroups,
                          uint64_t* ticks, float* sink, void* hip_stream) {
  if (!operands || !ticks || !sink || bytes < 16 || bytes > ((size_t)1 << 34) || iters < 1 ||
      iters > (1 << 20) || workgroups < 1 || workgroups > 65536 ||
      (reinterpret_cast<uintptr_t>(operands) & 15))
    return fail(NEZHA_EINVAL, "bad argument");
  hipStream_t stream = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(256), 0, stream,
                     static_cast<const uint4*>(operands), (int)(bytes / 16), iters,
                     reinterpret_cast<unsigned long long*>(ticks), sink);
  NEZHA_HIP_CHECK(hipGetLastError());
  return NEZHA_OK;
}

int nezha_bench_tile_step(int mode, int iters, int workgroups, const float* values,
                          uint64_t* ticks, float* sink, void* hip_stream) {
  if (!values || !ticks || !sink || mode < 0 || mode > 2 || iters < 1 || iters > (1 << 24) ||
      workgroups < 1 || workgroups > 65536)
    return fail(NEZHA_EINVAL, "bad argument");
  hipStream_t stream = (hipStream_t)hip_stream;
  unsigned long long* tk = reinterpret_cast<unsigned long long*>(ticks);
  if (mode == 0)
    hipLaunchKernelGGL(tile_step_kernel<0>, dim3(workgroups), dim3(256), 0, stream, values, iters, tk, sink);
  else if (mode == 1)
    hipLaunchKernelGGL(tile_step_kernel<1>, dim3(workgroups), dim3(256), 0, stream, values, iters, tk, sink);
  else
    hipLaunchKernelGGL(tile_step_kernel<2>, dim3(workgroups), dim3(256), 0, stream, values, iters, tk, sink);
  NEZHA_HIP_CHECK(hipGetLastError());
  return NEZHA_OK;
}

size_t nezha_draft_step_workspace(const nezha_step_desc* desc) {
  Plan p;
  if (check_desc(desc, &p) != NEZHA_OK) return 0;
  return p.total;
}

// Arguments of the single-launch level kernel from those of nezha_draft_step.
static LevelArgs make_level_args(const nezha_step_desc* desc, const uint16_t* Wp, const float* A,
                                 const void* E_l, const void* state_in, const uint64_t* key_in,
                                 const float* score_in, const nezha_itemset* set, uint64_t* key_out,
                                 float* score_out, int32_t* parent_out, int32_t* code_out,
                                 void* state_out, int32_t* count_out, uint64_t mult) {
  const int level = desc->level;
  const int V = desc->radices[level - 1];
  LevelArgs la;
  la.state_in = state_in;
  la.Wbeam = Wp + packed_user_elems(desc->d, V);
  la.A = A;
  la.key_in = key_in;
  la.score_in = score_in;
  la.E = E_l;
  la.set = SetView{(set && set->L == level) ? set->slots : nullptr, set ? set->n_buckets : 0,
                   set ? set->filter : nullptr, set ? set->n_blocks : 0,
                   set ? set->mult[set->L - 1] : 0};
  la.U = desc->U_l;
  la.transition = desc->transition;
  la.mult = mult;
  la.key_out = key_out;
  la.score_out = score_out;
  la.parent_out = parent_out;
  la.code_out = code_out;
  la.state_out = state_out;
  la.count_out = count_out;
  la.K_in = desc->K_in;
  la.K = desc->K;
  la.V = V;
  la.e = desc->e;
  return la;
}
static size_t level_small_lds(int V) {
  return (size_t)(kLevelWaves * 256 + 2 * kLevelRows * kLevelBeam + 256) * 8 +
         (size_t)2 * kLevelStateElems * 2 + (size_t)kLevelRows * V * 4;
}

// Argument checks of one level (everything nezha_draft_step refuses); fills the workspace plan.
static int validate_step(const nezha_step_desc* desc, const void* H_l, const void* W_l,
                         const void* E_l, const void* state_in, const nezha_itemset* set,
                         const uint64_t* key_out, const float* score_out,
                         const int32_t* parent_out, const int32_t* code_out,
                         const void* state_out, const void* workspace, size_t workspace_bytes,
                         Plan* plan_out) {
  Plan plan;
  int rc = check_desc(desc, &plan);
  if (rc != NEZHA_OK) return rc;
  *plan_out = plan;
  const int level = desc->level, L = desc->L;
  const bool bf16 = desc->dtype == NEZHA_BF16;
  if (desc->B == 0) return NEZHA_OK;  // an empty batch has nothing to read or write
  if ((!H_l && !desc->user_part) || !W_l) return fail(NEZHA_EINVAL, "H_l or W_l is NULL");
  if (reinterpret_cast<uintptr_t>(desc->user_part) & 15)
    return fail(NEZHA_EINVAL, "user_part is not 16-byte aligned");
  if (!key_out || !score_out || !parent_out || !code_out)
    return fail(NEZHA_EINVAL, "an output pointer is NULL");
  if (level < L && !state_out) return fail(NEZHA_EINVAL, "state_out is NULL below the last level");
  if (state_out && !E_l) return fail(NEZHA_EINVAL, "E_l is NULL but state_out is wanted");
  if (desc->transition != NEZHA_TRANSITION_ADD && desc->transition != NEZHA_TRANSITION_RNN)
    return fail(NEZHA_EINVAL, "unknown transition %d", (int)desc->transition);
  if (state_out && desc->transition == NEZHA_TRANSITION_RNN) {
    if (!desc->U_l) return fail(NEZHA_EINVAL, "U_l is NULL with NEZHA_TRANSITION_RNN");
    if (reinterpret_cast<uintptr_t>(desc->U_l) & 15)
      return fail(NEZHA_EINVAL, "U_l is not 16-byte aligned");
  }
  if (!workspace) return fail(NEZHA_EINVAL, "workspace is NULL");
  if (workspace_bytes < plan.total)
    return fail(NEZHA_EINVAL, "workspace has %zu bytes, %zu needed", workspace_bytes, plan.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255)
    return fail(NEZHA_EINVAL, "workspace is not 256-byte aligned");
  // bf16 operands are fetched 16 bytes at a time; the float32 path reads H and W element-wise
  const uintptr_t hw_mask = bf16 ? 15 : 3;
  if ((reinterpret_cast<uintptr_t>(H_l) | reinterpret_cast<uintptr_t>(W_l)) & hw_mask)
    return fail(NEZHA_EINVAL, "H_l and W_l must be %d-byte aligned", (int)hw_mask + 1);
  if ((reinterpret_cast<uintptr_t>(E_l) | reinterpret_cast<uintptr_t>(state_in) |
       reinterpret_cast<uintptr_t>(state_out)) & 15)
    return fail(NEZHA_EINVAL, "E_l and the states must be 16-byte aligned");
  if (set) {
    if (!set_is_live(set)) return fail(NEZHA_EINVAL, "not an item set");
    if (set->L != L && set->L != level)
      return fail(NEZHA_EINVAL, "the set's tuples have %d digits; %d (items) or %d (prefixes of this level) expected",
                  set->L, L, level);
    for (int l = 0; l < set->L; ++l)
      if (set->radices[l] != desc->radices[l])
        return fail(NEZHA_EINVAL, "item set and desc disagree on radix %d", l + 1);
  }
  return NEZHA_OK;
}

int nezha_draft_step(const nezha_step_desc* desc, const void* H_l, const void* W_l,
                     const void* E_l, const void* state_in, const uint64_t* key_in,
                     const float* score_in, const nezha_itemset* set, uint64_t* key_out,
                     float* score_out, int32_t* parent_out, int32_t* code_out,
                     void* state_out, int32_t* count_out, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  Plan plan;
  int rc = validate_step(desc, H_l, W_l, E_l, state_in, set, key_out, score_out, parent_out,
                         code_out, state_out, workspace, workspace_bytes, &plan);
  if (rc != NEZHA_OK) return rc;
  const int B = desc->B, K = desc->K, K_in = desc->K_in, d = desc->d, e = desc->e;
  const int level = desc->level, L = desc->L;
  const int V = desc->radices[level - 1];
  const bool bf16 = desc->dtype == NEZHA_BF16;
  if (desc->B == 0) return NEZHA_OK;
  uint64_t mult[NEZHA_MAX_LEVELS];
  radix_multipliers(L, desc->radices, mult);

  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = static_cast<char*>(workspace);
  uint16_t* Wp = desc->w_packed ? static_cast<uint16_t*>(const_cast<void*>(W_l))
                                : reinterpret_cast<uint16_t*>(ws + plan.wp_off);
  float* A = reinterpret_cast<float*>(ws + plan.a_off);
  int32_t* cand_code = reinterpret_cast<int32_t*>(ws + plan.code_off);
  float* cand_logp = reinterpret_cast<float*>(ws + plan.logp_off);
  const int rows = B * K_in;

  if (desc->user_part) {
    // the caller formed A_l already (nezha_user_projection / nezha_user_projection_levels)
    A = const_cast<float*>(desc->user_part);
    if (bf16 && !desc->w_packed) {
      rc = launch_pack(desc, W_l, Wp, stream);
      if (rc != NEZHA_OK) return rc;
    }
  } else {
    rc = launch_user_part(desc, H_l, W_l, Wp, A, stream);
    if (rc != NEZHA_OK) return rc;
  }

  if (plan.wide) {
    // beams wider than 128: the level's logits go through HBM (wide_beam.h)
    WideArgs wa;
    wa.state = state_in;
    wa.Wbeam = bf16 ? static_cast<const void*>(Wp + packed_user_elems(d, V)) : W_l;
    wa.A = A;
    wa.zk = reinterpret_cast<uint32_t*>(ws + plan.code_off);
    wa.key_in = key_in;
    wa.score_in = score_in;
    const bool verify = set && set->L == level;
    wa.set = SetView{verify ? set->slots : nullptr, set ? set->n_buckets : 0,
                     set ? set->filter : nullptr, set ? set->n_blocks : 0,
                   set ? set->mult[set->L - 1] : 0};
    wa.mult = mult[level - 1];
    wa.rows = rows;
    wa.K_in = K_in;
    wa.K = K;
    wa.V = V;
    wa.d = d;
    wa.e = e;
    wa.col_splits = 1;
    wa.glist = reinterpret_cast<uint64_t*>(ws + plan.list_off);
    wa.gcount = verify ? reinterpret_cast<int32_t*>(ws + plan.redo_off) : nullptr;
    const bool fused = bf16 && !verify;                  // logits never stored (wide_beam.h)
    WideSelectArgs sa;
    sa.splits = wide_select_splits(B);
    sa.n_tops = sa.splits * K;
    if (fused) {
      WideFusedArgs fa;
      fa.w = wa;
      fa.w.gcount = reinterpret_cast<int32_t*>(ws + plan.redo_off);
      fa.w.col_splits = wide_fused_col_splits(B, K_in, V);
      fa.part = reinterpret_cast<float2*>(ws + plan.redo_req_off);
      fa.tops = reinterpret_cast<uint32_t*>(ws + plan.logp_off);
      fa.groups = (K_in + 31) / 32;
      sa.n_tops = fa.groups * fa.w.col_splits * 128;
      const int64_t units = (int64_t)B * fa.groups * fa.w.col_splits;
      const unsigned blocks = (unsigned)((units + 3) / 4);
      ProfileScope prof(kWideLogits, stream);
#define LAUNCH_FUSED(KSTV)                                                                         \
  do {                                                                                             \
    hipLaunchKernelGGL((wide_fused_bf16_kernel<KSTV, false>), dim3(blocks), dim3(256), 0, stream, fa); \
    hipLaunchKernelGGL((wide_fused_bf16_kernel<KSTV, true>), dim3(blocks), dim3(256), 0, stream, fa);  \
  } while (0)
      if (e <= 64) LAUNCH_FUSED(2);
      else if (e <= 128) LAUNCH_FUSED(4);
      else LAUNCH_FUSED(8);
#undef LAUNCH_FUSED
      NEZHA_HIP_CHECK(hipGetLastError());
    } else {
      ProfileScope prof(kWideLogits, stream);
      if (bf16) {
        const int64_t row_groups = ((int64_t)rows + 31) / 32;
        int64_t cs = (4096 + row_groups - 1) / row_groups;       // enough waves to fill the chip
        cs = cs < 1 ? 1 : cs > V / 16 ? V / 16 : cs;
        wa.col_splits = (int)cs;
        const int64_t blocks = (row_groups * cs + 3) / 4;
        if (e <= 64)
          hipLaunchKernelGGL((wide_logits_bf16_kernel<2>), dim3((unsigned)blocks), dim3(256), 0,
                             stream, wa);
        else if (e <= 128)
          hipLaunchKernelGGL((wide_logits_bf16_kernel<4>), dim3((unsigned)blocks), dim3(256), 0,
                             stream, wa);
        else
          hipLaunchKernelGGL((wide_logits_bf16_kernel<8>), dim3((unsigned)blocks), dim3(256), 0,
                             stream, wa);
      } else {
        const int64_t blocks = (((int64_t)rows + 15) / 16) * ((V + 255) / 256);
        hipLaunchKernelGGL(wide_logits_f32_kernel, dim3((unsigned)blocks), dim3(256),
                           (size_t)16 * e * 4, stream, wa);
      }
      NEZHA_HIP_CHECK(hipGetLastError());
    }
    if (!fused) {
      ProfileScope prof(kWideRows, stream);
#define LAUNCH_ROWS(VERIFYV, NVV)                                                                  \
  hipLaunchKernelGGL((wide_rows_kernel<VERIFYV, NVV>), dim3((unsigned)rows), dim3(kWideRowThreads), \
                     0, stream, wa)
      if (V <= 16 * kWideRowThreads) {
        if (verify) LAUNCH_ROWS(true, 16);
        else LAUNCH_ROWS(false, 16);
      } else {
        if (verify) LAUNCH_ROWS(true, 0);
        else LAUNCH_ROWS(false, 0);
      }
#undef LAUNCH_ROWS
      NEZHA_HIP_CHECK(hipGetLastError());
    }
    sa.zk = wa.zk;
    sa.key_in = key_in;
    sa.score_in = score_in;
    sa.state_in = state_in;
    sa.E = E_l;
    sa.U = desc->U_l;
    sa.mult = mult[level - 1];
    sa.key_out = key_out;
    sa.score_out = score_out;
    sa.parent_out = parent_out;
    sa.code_out = code_out;
    sa.state_out = state_out;
    sa.count_out = count_out;
    sa.K_in = K_in;
    sa.K = K;
    sa.V = V;
    sa.e = e;
    sa.transition = desc->transition;
    sa.tops = reinterpret_cast<uint32_t*>(ws + plan.logp_off);
    sa.glist = reinterpret_cast<uint64_t*>(ws + plan.list_off);
    sa.gcount = reinterpret_cast<int32_t*>(ws + plan.redo_off);
    {
      const size_t lds = wide_select_lds();
      ProfileScope prof(kWideSelect, stream);
      const size_t collect_lds = (size_t)kWideListCap * 8;
      if (fused || (sa.splits > 1 && !verify)) {
        rc = allow_lds(wide_collect_kernel, collect_lds);
        if (rc != NEZHA_OK) return rc;
      }
      if (fused) {
        // the bound comes from the keys the fused kernel kept
        hipLaunchKernelGGL(wide_collect_kernel, dim3(B * sa.splits), dim3(kWideThreads), collect_lds,
                           stream, sa);
      } else if (sa.splits > 1 && !verify) {
        hipLaunchKernelGGL(wide_bound_kernel, dim3(B * sa.splits), dim3(kWideThreads), 0, stream, sa);
        hipLaunchKernelGGL(wide_collect_kernel, dim3(B * sa.splits), dim3(kWideThreads), collect_lds,
                           stream, sa);
      }
#define LAUNCH_SELECT(KERN)                                                             \
  do {                                                                                  \
    rc = allow_lds(KERN, lds);                                                          \
    if (rc != NEZHA_OK) return rc;                                                      \
    hipLaunchKernelGGL(KERN, dim3(B), dim3(kWideThreads), lds, stream, sa);             \
  } while (0)
      if (sa.splits > 1 || verify || fused) {
        if (bf16) LAUNCH_SELECT(wide_finish_kernel<true>);
        else LAUNCH_SELECT(wide_finish_kernel<false>);
      } else {
        if (bf16) LAUNCH_SELECT(wide_select_kernel<true>);
        else LAUNCH_SELECT(wide_select_kernel<false>);
      }
#undef LAUNCH_SELECT
      NEZHA_HIP_CHECK(hipGetLastError());
    }
    return NEZHA_OK;
  }

  if (level_fits_one_launch(bf16, K, K_in, V, e)) {
    // small shapes: the whole level after the projection in one launch, one workgroup per request
    const LevelArgs la = make_level_args(desc, Wp, A, E_l, state_in, key_in, score_in, set, key_out,
                                         score_out, parent_out, code_out, state_out, count_out,
                                         mult[level - 1]);
    const size_t lds = level_small_lds(V);
    dim3 grid(B), block(64 * kLevelWaves);
    ProfileScope prof(kLevelFused, stream);
#define LAUNCH_LEVEL(KSTV, NVTV)                                                           \
  do {                                                                                     \
    rc = allow_lds(level_small_kernel<KSTV, NVTV>, lds);                                   \
    if (rc != NEZHA_OK) return rc;                                                         \
    hipLaunchKernelGGL((level_small_kernel<KSTV, NVTV>), grid, block, lds, stream, la);    \
  } while (0)
    if (V <= 256) {
      if (e == 32) LAUNCH_LEVEL(1, 4);
      else if (e == 64) LAUNCH_LEVEL(2, 4);
      else if (e == 128) LAUNCH_LEVEL(4, 4);
      else LAUNCH_LEVEL(8, 4);
    } else {
      if (e == 32) LAUNCH_LEVEL(1, 8);
      else if (e == 64) LAUNCH_LEVEL(2, 8);
      else if (e == 128) LAUNCH_LEVEL(4, 8);
      else LAUNCH_LEVEL(8, 8);
    }
#undef LAUNCH_LEVEL
    NEZHA_HIP_CHECK(hipGetLastError());
    return NEZHA_OK;
  }

  if (K_in == 1 && !state_in && !key_in && !score_in && !(set && set->L == level) &&
      V <= kFirstThreads * kFirstPerThread &&
      K <= NEZHA_MAX_BEAM) {
    // level 1 of a decode: the logits are the user part; one launch
    FirstLevelArgs fa;
    fa.A = A;
    fa.E = E_l;
    fa.U = desc->U_l;
    fa.mult = mult[level - 1];
    fa.key_out = key_out;
    fa.score_out = score_out;
    fa.parent_out = parent_out;
    fa.code_out = code_out;
    fa.state_out = state_out;
    fa.count_out = count_out;
    fa.K = K;
    fa.V = V;
    fa.e = e;
    fa.transition = desc->transition;
    ProfileScope prof(kExpand, stream);
    if (bf16)
      hipLaunchKernelGGL(first_level_kernel<true>, dim3(B), dim3(kFirstThreads), 0, stream, fa);
    else
      hipLaunchKernelGGL(first_level_kernel<false>, dim3(B), dim3(kFirstThreads), 0, stream, fa);
    NEZHA_HIP_CHECK(hipGetLastError());
    return NEZHA_OK;
  }

  ExpandArgs ea;
  ea.state = state_in;
  ea.Wbeam = bf16 ? static_cast<const void*>(Wp + packed_user_elems(d, V)) : W_l;
  ea.A = A;
  ea.cand_code = cand_code;
  ea.cand_logp = cand_logp;
  ea.rows = rows;
  ea.K_in = K_in;
  ea.K = K;
  ea.V = V;
  ea.d = d;
  ea.e = e;
  ea.redo = nullptr;
  const uint8_t* redo_req = nullptr;   // set when a kernel above has already finished most requests
  if (plan.per_request) {
    // one workgroup per request, resident workgroups walk the batch
    // compute units of the current device (asked once per device; the cache is per device)
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cu_of_device[kMaxDevices];
    int dev = 0;
    NEZHA_HIP_CHECK(hipGetDevice(&dev));
    int n_cu = (dev >= 0 && dev < kMaxDevices) ? cu_of_device[dev].load(std::memory_order_relaxed) : 0;
    if (n_cu == 0) {
      int v = 0;
      NEZHA_HIP_CHECK(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
      n_cu = v > 0 ? v : 1;
      if (dev >= 0 && dev < kMaxDevices) cu_of_device[dev].store(n_cu, std::memory_order_relaxed);
    }
    const int n_waves = (K_in + 15) / 16;
    int groups = B < 2 * n_cu ? B : 2 * n_cu;
    groups = groups < kReqMaxGroups ? groups : kReqMaxGroups;
    // without verification at this level the kernel also does the merge and the Transition
    const bool whole = !(set && set->L == level);
    const size_t lds = request_w_region(e, n_waves) + (size_t)2 * kReqTiles * 16 * 4 +
                       (size_t)n_waves * 48 * 4 + (whole ? request_whole_lds() : 0);
    uint64_t* lists = reinterpret_cast<uint64_t*>(ws + plan.list_off);
    uint8_t* redo = reinterpret_cast<uint8_t*>(ws + plan.redo_off);
    RequestLevelArgs rl;
    rl.key_in = key_in;
    rl.score_in = score_in;
    rl.E = E_l;
    rl.U = desc->U_l;
    rl.mult = mult[level - 1];
    rl.key_out = key_out;
    rl.score_out = score_out;
    rl.parent_out = parent_out;
    rl.code_out = code_out;
    rl.state_out = state_out;
    rl.count_out = count_out;
    rl.redo_req = reinterpret_cast<uint8_t*>(ws + plan.redo_req_off);
    rl.transition = desc->transition;
    ProfileScope prof(kExpandRequest, stream);
#define LAUNCH_REQUEST(KSTV, WHOLEV)                                                               \
  do {                                                                                             \
    rc = allow_lds(expand_request_kernel<KSTV, WHOLEV>, lds);                                      \
    if (rc != NEZHA_OK) return rc;                                                                 \
    hipLaunchKernelGGL((expand_request_kernel<KSTV, WHOLEV>), dim3(groups), dim3(64 * n_waves),    \
                       lds, stream, ea, lists, redo, rl);                                          \
  } while (0)
#define LAUNCH_REQUEST_E(WHOLEV)                  \
  do {                                            \
    if (e == 32) LAUNCH_REQUEST(1, WHOLEV);       \
    else if (e == 64) LAUNCH_REQUEST(2, WHOLEV);  \
    else if (e == 128) LAUNCH_REQUEST(4, WHOLEV); \
    else LAUNCH_REQUEST(8, WHOLEV);               \
  } while (0)
    if (whole) LAUNCH_REQUEST_E(true);
    else LAUNCH_REQUEST_E(false);
#undef LAUNCH_REQUEST_E
#undef LAUNCH_REQUEST
    NEZHA_HIP_CHECK(hipGetLastError());
    redo_req = whole ? rl.redo_req : nullptr;
    ea.redo = redo;   // the chunked kernel below redoes the flagged beams only
  }
  {
    const int groups = (rows + 15) / 16;
    ProfileScope prof(kExpand, stream);
    if (codebook_fits_lds(bf16, K, V)) {
      // small codebook: 16 x T_l logits fit in LDS; 8 waves share 16 beams
      const size_t lds = (size_t)8 * 256 * 8 + (size_t)16 * V * 4;
      dim3 grid(groups), block(512);
#define LAUNCH_SMALL(KSTV, NVTV)                                                            \
  do {                                                                                      \
    rc = allow_lds(expand_small_kernel<KSTV, NVTV>, lds);                                   \
    if (rc != NEZHA_OK) return rc;                                                          \
    hipLaunchKernelGGL((expand_small_kernel<KSTV, NVTV>), grid, block, lds, stream, ea);    \
  } while (0)
      if (V <= 256) {
        if (e <= 64) LAUNCH_SMALL(2, 4);
        else if (e <= 128) LAUNCH_SMALL(4, 4);
        else LAUNCH_SMALL(8, 4);
      } else {
        if (e <= 64) LAUNCH_SMALL(2, 16);
        else if (e <= 128) LAUNCH_SMALL(4, 16);
        else LAUNCH_SMALL(8, 16);
      }
#undef LAUNCH_SMALL
    } else {
      const size_t lds = (size_t)16 * plan.cap * 8 + (size_t)16 * 12;
      dim3 grid(groups), block(64);
#define LAUNCH_EXPAND(BF, CAPV, KSTV)                                                         \
  do {                                                                                        \
    rc = allow_lds(expand_kernel<BF, CAPV, KSTV, 1>, lds);                                    \
    if (rc != NEZHA_OK) return rc;                                                            \
    hipLaunchKernelGGL((expand_kernel<BF, CAPV, KSTV, 1>), grid, block, lds, stream, ea);     \
  } while (0)
#define LAUNCH_EXPAND_BF16(CAPV)                                 \
  do {                                                           \
    if (e <= 64) LAUNCH_EXPAND(true, CAPV, 2);                   \
    else if (e <= 128) LAUNCH_EXPAND(true, CAPV, 4);             \
    else LAUNCH_EXPAND(true, CAPV, 8);                           \
  } while (0)
      if (bf16) {
        // large codebook (or K > 64): two sweeps in chunks of 256 codes, 8 waves per 16 beams
        const size_t lds2 = (size_t)16 * 256 * 8 + (size_t)2 * 16 * kChunk * 4;
        dim3 grid2(ea.redo && groups > kRedoScanGroups ? kRedoScanGroups : groups), block2(512);
#define LAUNCH_CHUNKED(KSTV)                                                              \
  do {                                                                                    \
    rc = allow_lds(expand_chunked_kernel<KSTV>, lds2);                                    \
    if (rc != NEZHA_OK) return rc;                                                        \
    hipLaunchKernelGGL((expand_chunked_kernel<KSTV>), grid2, block2, lds2, stream, ea);   \
  } while (0)
        if (e <= 64) LAUNCH_CHUNKED(2);
        else if (e <= 128) LAUNCH_CHUNKED(4);
        else LAUNCH_CHUNKED(8);
#undef LAUNCH_CHUNKED
      } else {
        if (plan.cap == 128) LAUNCH_EXPAND(false, 128, 64);
        else LAUNCH_EXPAND(false, 256, 64);
      }
#undef LAUNCH_EXPAND_BF16
#undef LAUNCH_EXPAND
    }
    NEZHA_HIP_CHECK(hipGetLastError());
  }

  MergeArgs ma;
  ma.cand_code = cand_code;
  ma.cand_logp = cand_logp;
  ma.key_in = key_in;
  ma.score_in = score_in;
  ma.state_in = state_in;
  ma.E = E_l;
  ma.set = SetView{(set && set->L == level) ? set->slots : nullptr, set ? set->n_buckets : 0,
                   set ? set->filter : nullptr, set ? set->n_blocks : 0,
                   set ? set->mult[set->L - 1] : 0};
  ma.U = desc->U_l;
  ma.transition = desc->transition;
  ma.redo_req = redo_req;
  ma.mult = mult[level - 1];
  ma.key_out = key_out;
  ma.score_out = score_out;
  ma.parent_out = parent_out;
  ma.code_out = code_out;
  ma.state_out = state_out;
  ma.count_out = count_out;
  ma.K_in = K_in;
  ma.K = K;
  ma.e = e;
  {
    dim3 grid(B), block(K_in * K >= 4096 ? 64 * kMergeMaxWaves : 256);
    const size_t lds = ((size_t)((K_in * K + 1) & ~1) + 256) * sizeof(uint64_t);
    ProfileScope prof(kMerge, stream);
    if (bf16) {
      rc = allow_lds(merge_kernel<true>, lds);
      if (rc != NEZHA_OK) return rc;
      hipLaunchKernelGGL((merge_kernel<true>), grid, block, lds, stream, ma);
    } else {
      rc = allow_lds(merge_kernel<false>, lds);
      if (rc != NEZHA_OK) return rc;
      hipLaunchKernelGGL((merge_kernel<false>), grid, block, lds, stream, ma);
    }
    NEZHA_HIP_CHECK(hipGetLastError());
  }
  return NEZHA_OK;
}

// Argument checks of all L levels of nezha_draft_levels / nezha_decode, in the order the levels
// would run, before anything is enqueued.
static int validate_levels(const nezha_step_desc* desc, const nezha_level_io* io,
                           const void* workspace, size_t workspace_bytes) {
  if (!desc || !io) return fail(NEZHA_EINVAL, "desc or io is NULL");
  const int L = desc->L;
  if (L < 1 || L > NEZHA_MAX_LEVELS)
    return fail(NEZHA_EINVAL, "L = %d outside 1..%d", L, NEZHA_MAX_LEVELS);
  if (!desc->radices) return fail(NEZHA_EINVAL, "radices is NULL");
  if (reinterpret_cast<uintptr_t>(desc->state_init) & 15)
    return fail(NEZHA_EINVAL, "state_init is not 16-byte aligned");
  nezha_step_desc dl = *desc;
  const void* state = desc->state_init;
  for (int l = 1; l <= L; ++l) {
    const nezha_level_io& x = io[l - 1];
    dl.level = l;
    dl.K_in = l == 1 ? 1 : desc->K;
    dl.user_part = x.user_part;
    dl.U_l = x.U_l;
    Plan plan;
    int rc = validate_step(&dl, x.H_l, x.W_l, x.E_l, state, x.set, x.key_out, x.score_out,
                           x.parent_out, x.code_out, x.state_out, workspace, workspace_bytes, &plan);
    if (rc != NEZHA_OK) return rc;
    state = x.state_out;
  }
  return NEZHA_OK;
}

static int draft_levels_checked(const nezha_step_desc* desc, const nezha_level_io* io,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

int nezha_decode(const nezha_step_desc* desc, const nezha_level_io* io, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  if (!desc || !io) return fail(NEZHA_EINVAL, "desc or io is NULL");
  if (desc->L < 1 || desc->L > NEZHA_MAX_LEVELS)
    return fail(NEZHA_EINVAL, "L = %d outside 1..%d", desc->L, NEZHA_MAX_LEVELS);
  const void* H[NEZHA_MAX_LEVELS];
  const void* W[NEZHA_MAX_LEVELS];
  float* A[NEZHA_MAX_LEVELS];
  for (int l = 0; l < desc->L; ++l) {
    if (!io[l].H_l || !io[l].user_part)
      return fail(NEZHA_EINVAL, "level %d: H_l and user_part (the buffer of the level's user part) are needed",
                  l + 1);
    H[l] = io[l].H_l;
    W[l] = io[l].W_l;
    A[l] = const_cast<float*>(io[l].user_part);
  }
  if (desc->dtype != NEZHA_BF16 || !desc->w_packed)
    return fail(NEZHA_EINVAL, "needs NEZHA_BF16 weights packed by nezha_pack_weights");
  // every level's arguments are checked before the projections (which write user_part) are enqueued
  int rc = validate_levels(desc, io, workspace, workspace_bytes);
  if (rc != NEZHA_OK) return rc;
  rc = nezha_user_projection_levels(desc, desc->L, H, W, A, hip_stream);
  if (rc != NEZHA_OK) return rc;
  return draft_levels_checked(desc, io, workspace, workspace_bytes, hip_stream);
}

size_t nezha_draft_levels_workspace(const nezha_step_desc* desc) {
  if (!desc || desc->L < 1 || desc->L > NEZHA_MAX_LEVELS) return 0;
  size_t most = 0;
  nezha_step_desc dl = *desc;
  for (int l = 1; l <= desc->L; ++l) {
    dl.level = l;
    dl.K_in = l == 1 ? 1 : desc->K;
    const size_t n = nezha_draft_step_workspace(&dl);
    if (n == 0) return 0;
    most = n > most ? n : most;
  }
  return most;
}

int nezha_draft_levels(const nezha_step_desc* desc, const nezha_level_io* io, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  int rc = validate_levels(desc, io, workspace, workspace_bytes);
  if (rc != NEZHA_OK) return rc;
  return draft_levels_checked(desc, io, workspace, workspace_bytes, hip_stream);
}

// The level loop; validate_levels has passed.
static int draft_levels_checked(const nezha_step_desc* desc, const nezha_level_io* io,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int L = desc->L;
  const bool bf16 = desc->dtype == NEZHA_BF16;
  const int K = desc->K;
  // one launch for all levels when every level fits the single-launch kernel and has its user part
  bool one_launch = bf16 && desc->w_packed == 1 && desc->B > 0;
  int max_v = 0;
  for (int l = 1; l <= L && one_launch; ++l) {
    const int V = desc->radices[l - 1];
    one_launch = level_fits_one_launch(bf16, K, l == 1 ? 1 : K, V, desc->e) &&
                 io[l - 1].user_part != nullptr;
    max_v = V > max_v ? V : max_v;
  }
  nezha_step_desc dl = *desc;
  const void* state = desc->state_init;
  const uint64_t* key = nullptr;
  const float* score = nullptr;
  DecodeArgs da;
  da.L = L;
  uint64_t mult[NEZHA_MAX_LEVELS];
  if (one_launch && !radix_multipliers(L, desc->radices, mult))
    return fail(NEZHA_ERANGE, "radices must be >= 1 with a product of at most 2^64-1");
  for (int l = 1; l <= L; ++l) {
    const nezha_level_io& x = io[l - 1];
    dl.level = l;
    dl.K_in = l == 1 ? 1 : K;
    dl.user_part = x.user_part;
    dl.U_l = x.U_l;
    if (one_launch) {
      da.lv[l - 1] = make_level_args(&dl, static_cast<const uint16_t*>(x.W_l), x.user_part, x.E_l,
                                     state, key, score, x.set, x.key_out, x.score_out, x.parent_out,
                                     x.code_out, x.state_out, x.count_out, mult[l - 1]);
    } else {
      int rc = nezha_draft_step(&dl, x.H_l, x.W_l, x.E_l, state, key, score, x.set, x.key_out,
                                x.score_out, x.parent_out, x.code_out, x.state_out, x.count_out,
                                workspace, workspace_bytes, hip_stream);
      if (rc != NEZHA_OK) return rc;
    }
    state = x.state_out;
    key = x.key_out;
    score = x.score_out;
  }
  if (!one_launch) return NEZHA_OK;
  for (int l = L; l < NEZHA_MAX_LEVELS; ++l) da.lv[l] = da.lv[L - 1];
  hipStream_t stream = (hipStream_t)hip_stream;
  const size_t lds = level_small_lds(max_v);
  const int e = desc->e;
  int rc = NEZHA_OK;
  dim3 grid(desc->B), block(64 * kLevelWaves);
  ProfileScope prof(kDecodeFused, stream);
#define LAUNCH_DECODE(KSTV, NVTV)                                                           \
  do {                                                                                      \
    rc = allow_lds(decode_small_kernel<KSTV, NVTV>, lds);                                   \
    if (rc != NEZHA_OK) return rc;                                                          \
    hipLaunchKernelGGL((decode_small_kernel<KSTV, NVTV>), grid, block, lds, stream, da);    \
  } while (0)
  if (max_v <= 256) {
    if (e == 32) LAUNCH_DECODE(1, 4);
    else if (e == 64) LAUNCH_DECODE(2, 4);
    else if (e == 128) LAUNCH_DECODE(4, 4);
    else LAUNCH_DECODE(8, 4);
  } else {
    if (e == 32) LAUNCH_DECODE(1, 8);
    else if (e == 64) LAUNCH_DECODE(2, 8);
    else if (e == 128) LAUNCH_DECODE(4, 8);
    else LAUNCH_DECODE(8, 8);
  }
#undef LAUNCH_DECODE
  NEZHA_HIP_CHECK(hipGetLastError());
  return NEZHA_OK;
}

}  // extern "C"
