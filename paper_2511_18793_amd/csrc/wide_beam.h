// Beams wider than NEZHA_MAX_BEAM (the recall setting of Sec. 1 and Table 1: beam 512, up to
// 1000 in item retrieval): one level of Alg. 3 with up to 1024 beams in and out.
//
// K * K reaches 10^6 candidates per request here, so nothing of a request fits in registers or
// LDS any more.  The level's logits go through HBM once instead:
//   wide_logits_*_kernel  z = A_l + c * W_l[d:d+e] for all B*K_in beams        -> zk (float32)
//   wide_rows_kernel      per beam: log-sum-exp, cumulative score of every code as a 32-bit sort
//                         key (in place).  Where a set is consulted: the beam's K best codes
//                         (exact radix selection, ties to the lower code) are probed (Eq. 4-5);
//                         every other code gets key 0 = not a candidate
//   wide_select_kernel    per request: the K best keys of its K_in * T_l, ordered by (score,
//                         parent, code); outputs and the Transition of Eq. 3
// Included by draft.hip only (inside its unnamed namespace).
#pragma once

constexpr int kWideThreads = 1024;          // wide_select_kernel
constexpr int kWideListCap = 8192;          // keys at or above the first bound that LDS can take
constexpr int kWideRowThreads = 256;        // wide_rows_kernel

struct WideArgs {
  const void* state;        // [B*K_in, e] or NULL
  const void* Wbeam;        // bf16: packed beam part of W_l; float32: W_l itself, row major
  const float* A;           // [B, T_l] user part
  uint32_t* zk;             // [B*K_in, T_l]: logits as float bits, then sort keys, in place
  const uint64_t* key_in;   // [B*K_in] or NULL
  const float* score_in;    // [B*K_in] or NULL
  SetView set;              // slots == NULL: no set is consulted at this level
  uint64_t mult;
  int64_t rows;
  int K_in, K, V, d, e;
  int col_splits;           // wide_logits_bf16_kernel: waves sharing one group of 32 beams
  // where a set is consulted: the request's surviving candidates as (key, ~index), at most
  // kWideListCap per request are stored, and how many there are
  uint64_t* glist;          // [B, kWideListCap]
  int32_t* gcount;          // [B], cleared by the logits kernel (wide_fused_bf16_kernel: always)
};

// ---- logits --------------------------------------------------------------------------------
// bf16: one wave = 32 beams (two 16-row MFMA tiles) x a contiguous share of the code tiles; the
// packed operands of W_l are read straight from L2 (every wave walks them in the same order),
// one tile ahead of the MFMAs.
template <int KST>
__global__ __launch_bounds__(256) void wide_logits_bf16_kernel(WideArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int g = lane >> 4, c = lane & 15;
  if (blockIdx.x == 0 && a.gcount)
    for (int64_t b = threadIdx.x; b < a.rows / a.K_in; b += 256) a.gcount[b] = 0;
  const int64_t unit = (int64_t)blockIdx.x * 4 + wave;
  const int64_t rg = unit / a.col_splits;
  const int cs = (int)(unit - rg * a.col_splits);
  const int64_t row0 = rg * 32;
  if (row0 >= a.rows) return;
  const int V = a.V, e = a.e, KS = e >> 5;
  const int n_tiles = V >> 4;
  const int t_begin = (int)((int64_t)n_tiles * cs / a.col_splits);
  const int t_end = (int)((int64_t)n_tiles * (cs + 1) / a.col_splits);
  const uint16_t* S = static_cast<const uint16_t*>(a.state);
  const uint16_t* Wb = static_cast<const uint16_t*>(a.Wbeam);

  uint4 fa[2][KST];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int64_t r = row0 + 16 * t + c;
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) {
      fa[t][ks] = uint4{0, 0, 0, 0};
      if (S && r < a.rows && ks < KS) fa[t][ks] = load_global_u4(S + r * e + ks * 32 + 8 * g);
    }
  }
  int64_t arow[2][4], zrow[2][4];
  bool live[2][4];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t r = row0 + 16 * t + 4 * g + i;
      live[t][i] = r < a.rows;
      arow[t][i] = live[t][i] ? (r / a.K_in) * V : 0;
      zrow[t][i] = live[t][i] ? r * V : 0;
    }
  uint4 w[KST], wn[KST];
  auto fetch = [&](uint4 (&dst)[KST], int ct) {
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) {
      dst[ks] = uint4{0, 0, 0, 0};
      if (ks < KS) dst[ks] = load_global_u4(Wb + ((int64_t)(ct * KS + ks) * 64 + lane) * 8);
    }
  };
  if (t_begin < t_end) fetch(w, t_begin);
  for (int ct = t_begin; ct < t_end; ++ct) {
    if (ct + 1 < t_end) fetch(wn, ct + 1);
    const int col = ct * 16 + c;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx4 acc;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = as_global(a.A)[arow[t][i] + col];
#pragma unroll
      for (int ks = 0; ks < KST; ++ks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8*>(&fa[t][ks]),
                                                      *reinterpret_cast<const bf16x8*>(&w[ks]), acc,
                                                      0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (live[t][i]) as_global(a.zk)[zrow[t][i] + col] = __float_as_uint(acc[i]);
    }
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) w[ks] = wn[ks];
  }
}

// bf16, levels where no set is consulted: the logits never reach HBM.  Two launches walk the same
// MFMA tiles; a wave = up to 32 beams of ONE request x a contiguous share of the code tiles:
//   wide_fused_bf16_kernel<KST, false>  running (max, sum of exponentials) per beam and share
//                                       -> part
//   wide_fused_bf16_kernel<KST, true>   log-sum-exp from the shares' parts; the logits are formed
//                                       again and written as sort keys; every lane keeps the two
//                                       largest keys it wrote (distinct candidates of one request)
//                                       -> tops, from which the selection takes its bound without
//                                       another pass over the keys
struct WideFusedArgs {
  WideArgs w;
  float2* part;             // [B*K_in, col_splits] (max, sum of exp(z - max))
  uint32_t* tops;           // [B, groups * col_splits * 128]
  int groups;               // ceil(K_in / 32)
};
__device__ __forceinline__ void softmax_merge(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  s = (m == mn ? s : s * __expf(m - mn)) + (m2 == mn ? s2 : s2 * __expf(m2 - mn));
  m = mn;
}
template <int KST, bool KEYS>
__global__ __launch_bounds__(256) void wide_fused_bf16_kernel(WideFusedArgs f) {
  const WideArgs& a = f.w;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int g = lane >> 4, c = lane & 15;
  const int CS = a.col_splits;
  const int64_t unit = (int64_t)blockIdx.x * 4 + wave;
  const int64_t n_req = a.rows / a.K_in;
  if (KEYS && blockIdx.x == 0)                           // the selection's list counters start at 0
    for (int64_t q = threadIdx.x; q < n_req; q += 256) a.gcount[q] = 0;
  if (unit >= n_req * f.groups * CS) return;
  const int cs = (int)(unit % CS);
  const int gr = (int)((unit / CS) % f.groups);
  const int64_t b = unit / ((int64_t)CS * f.groups);
  const int V = a.V, e = a.e, KS = e >> 5;
  const int n_tiles = V >> 4;
  const int t_begin = (int)((int64_t)n_tiles * cs / CS);
  const int t_end = (int)((int64_t)n_tiles * (cs + 1) / CS);
  const uint16_t* S = static_cast<const uint16_t*>(a.state);
  const uint16_t* Wb = static_cast<const uint16_t*>(a.Wbeam);
  // The wave's 32 beams are every groups-th beam of the request, starting at gr: beams enter a
  // level ordered by score, so a run of 32 consecutive beams would put the request's best
  // candidates into the lanes of one wave, and the two keys a lane keeps would miss most of them.
  auto beam_of = [&](int j) { return gr + f.groups * j; };    // j = 0..31, may reach past K_in

  uint4 fa[2][KST];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int r = beam_of(16 * t + c);
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) {
      fa[t][ks] = uint4{0, 0, 0, 0};
      if (S && r < a.K_in && ks < KS)
        fa[t][ks] = load_global_u4(S + (b * a.K_in + r) * e + ks * 32 + 8 * g);
    }
  }
  // per accumulator row: KEYS: (parent score - log-sum-exp, live); else running (max, sum)
  float p0[2][4], p1[2][4];
  bool live[2][4], in_req[2][4];
  int64_t zoff[2][4];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = beam_of(16 * t + 4 * g + i);
      const int64_t row = b * a.K_in + r;
      live[t][i] = in_req[t][i] = r < a.K_in;
      zoff[t][i] = in_req[t][i] ? row * V : 0;
      if constexpr (KEYS) {
        float m = -INFINITY, sm = 0.f;
        if (live[t][i])
          for (int k = 0; k < CS; ++k) {
            const float2 q = f.part[row * CS + k];
            softmax_merge(m, sm, q.x, q.y);
          }
        p0[t][i] = m + __logf(sm);                                       // log-sum-exp
        p1[t][i] = (live[t][i] && a.score_in) ? a.score_in[row] : 0.f;   // parent score
        if (live[t][i] && a.key_in && a.key_in[row] == kEmpty) live[t][i] = false;   // no children
      } else {
        p0[t][i] = -INFINITY;
        p1[t][i] = 0.f;
      }
    }
  uint32_t top0 = 0, top1 = 0;
  const float* Arow = a.A + b * V;
  uint4 w[KST], wn[KST];
  auto fetch = [&](uint4 (&dst)[KST], int ct) {
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) {
      dst[ks] = uint4{0, 0, 0, 0};
      if (ks < KS) dst[ks] = load_global_u4(Wb + ((int64_t)(ct * KS + ks) * 64 + lane) * 8);
    }
  };
  if (t_begin < t_end) fetch(w, t_begin);
  for (int ct = t_begin; ct < t_end; ++ct) {
    if (ct + 1 < t_end) fetch(wn, ct + 1);
    const int col = ct * 16 + c;
    const float a0 = as_global(Arow)[col];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx4 acc = floatx4{a0, a0, a0, a0};
#pragma unroll
      for (int ks = 0; ks < KST; ++ks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8*>(&fa[t][ks]),
                                                      *reinterpret_cast<const bf16x8*>(&w[ks]), acc,
                                                      0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (KEYS) {
          const uint32_t k = live[t][i] ? ordered_bits(p1[t][i] + (acc[i] - p0[t][i])) : 0u;
          if (in_req[t][i]) as_global(a.zk)[zoff[t][i] + col] = k;
          const uint32_t lo = k > top0 ? top0 : k;
          top0 = k > top0 ? k : top0;
          top1 = lo > top1 ? lo : top1;
        } else {
          const float mn = fmaxf(p0[t][i], acc[i]);
          p1[t][i] = p1[t][i] * __expf(p0[t][i] - mn) + __expf(acc[i] - mn);
          p0[t][i] = mn;
        }
      }
    }
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) w[ks] = wn[ks];
  }
  if constexpr (KEYS) {
    uint32_t* tp = f.tops + (b * f.groups * CS + (int64_t)gr * CS + cs) * 128 + 2 * lane;
    as_global(tp)[0] = top0;
    as_global(tp)[1] = top1;
  } else {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float m = p0[t][i], sm = p1[t][i];
#pragma unroll
        for (int x = 1; x < 16; x <<= 1) {               // the 16 lanes that hold this beam's columns
          const float m2 = __shfl_xor(m, x), s2 = __shfl_xor(sm, x);
          softmax_merge(m, sm, m2, s2);
        }
        if (c == 0 && live[t][i])
          f.part[(b * a.K_in + beam_of(16 * t + 4 * g + i)) * CS + cs] = float2{m, sm};
      }
  }
}

// float32: a workgroup forms 16 beams x 256 codes; the beams' states sit in LDS, a thread owns
// one code column and walks the e rows of the beam part of W_l (coalesced across the threads).
__global__ __launch_bounds__(256) void wide_logits_f32_kernel(WideArgs a) {
  extern __shared__ float wide_states[];   // [16][e]
  const int V = a.V, e = a.e;
  if (blockIdx.x == 0 && a.gcount)
    for (int64_t b = threadIdx.x; b < a.rows / a.K_in; b += 256) a.gcount[b] = 0;
  const int col_tiles = (V + 255) / 256;
  const int64_t rt = blockIdx.x / col_tiles;
  const int vt = (int)(blockIdx.x - rt * col_tiles);
  const int64_t row0 = rt * 16;
  const float* S = static_cast<const float*>(a.state);
  const float* W = static_cast<const float*>(a.Wbeam);
  for (int idx = threadIdx.x; idx < 16 * e; idx += 256) {
    const int r = idx / e, i = idx - r * e;
    wide_states[idx] = (S && row0 + r < a.rows) ? S[(row0 + r) * e + i] : 0.f;
  }
  __syncthreads();
  const int v = vt * 256 + (int)threadIdx.x;
  if (v >= V) return;
  float acc[16];
#pragma unroll
  for (int r = 0; r < 16; ++r)
    acc[r] = row0 + r < a.rows ? a.A[((row0 + r) / a.K_in) * V + v] : 0.f;
  if (S) {
    for (int i = 0; i < e; ++i) {
      const float wv = W[(int64_t)(a.d + i) * V + v];
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = fmaf(wide_states[r * e + i], wv, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (row0 + r < a.rows) a.zk[(row0 + r) * V + v] = __float_as_uint(acc[r]);
}

// ---- workgroup-wide helpers ------------------------------------------------------------------
template <int NT>
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
  __syncthreads();                                   // red may still be read from a call before
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r = fmaxf(r, red[w]);
  return r;
}
template <int NT>
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r += red[w];
  return r;
}

// Where the K-th largest nonzero key of keys[0..n) lies: keys above tau are among the K largest,
// and so are `need` of the n_eq keys equal to tau (need >= 1).  all == true: there are at most K
// nonzero keys, all of them count (tau, need, n_eq unset).
struct RadixPick {
  uint32_t tau;
  int need, n_eq;
  bool all;
};
// Exact radix selection by a workgroup of NT threads: a pass for the smallest and largest nonzero
// key, then passes over the keys for digits of up to 12 bits, starting at the highest bit in which
// those two differ (keys of one request share their top bits; a histogram of those would be one
// bin, and LDS atomics on one address run one after the other).  Each pass is a histogram in LDS
// of the keys that match the digits found so far.
// hist: 4096 + 256 words of LDS, bc: 4 words of LDS.  Every thread gets the result.
// BOUND_ONLY: stop after the first digit; tau is then the smallest key that has that digit (the
// low bits zero), a lower bound of the K-th largest key, and need / n_eq mean nothing.
template <int NT, bool BOUND_ONLY = false>
__device__ RadixPick block_radix_select(const uint32_t* keys, int64_t n, int K, uint32_t* hist,
                                        uint32_t* bc) {
  const int tid = threadIdx.x, lane = tid & 63;
  RadixPick r;
  r.tau = 0;
  r.need = K;
  r.n_eq = 0;
  r.all = false;
  uint32_t* psum = hist + 4096;
  uint32_t mx = 0, mn_inv = 0, n_mine = 0;
  for (int64_t i0 = tid; i0 < n; i0 += 8 * NT) {          // eight loads in flight per thread
    uint32_t kk[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) kk[u] = i0 + u * NT < n ? as_global(keys)[i0 + u * NT] : 0u;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t k = kk[u], inv = k ? ~k : 0u;
      mx = k > mx ? k : mx;
      mn_inv = inv > mn_inv ? inv : mn_inv;
      n_mine += k != 0u;
    }
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const uint32_t o0 = (uint32_t)__shfl_xor((int)mx, m), o1 = (uint32_t)__shfl_xor((int)mn_inv, m);
    mx = o0 > mx ? o0 : mx;
    mn_inv = o1 > mn_inv ? o1 : mn_inv;
    n_mine += (uint32_t)__shfl_xor((int)n_mine, m);
  }
  __syncthreads();                                       // psum may still be read from a call before
  if (lane == 0) {
    psum[3 * (tid >> 6)] = mx;
    psum[3 * (tid >> 6) + 1] = mn_inv;
    psum[3 * (tid >> 6) + 2] = n_mine;
  }
  __syncthreads();
  uint32_t n_valid = 0;
  mx = 0;
  mn_inv = 0;
  for (int w = 0; w < NT / 64; ++w) {
    mx = psum[3 * w] > mx ? psum[3 * w] : mx;
    mn_inv = psum[3 * w + 1] > mn_inv ? psum[3 * w + 1] : mn_inv;
    n_valid += psum[3 * w + 2];
  }
  __syncthreads();
  if (n_valid < (uint32_t)K) {                           // fewer than K keys: all of them count
    r.all = true;
    return r;
  }
  const uint32_t kmax = mx, kmin = ~mn_inv;
  if (kmin == kmax) {                                    // every key the same
    r.tau = kmax;
    r.n_eq = (int)n_valid;
    return r;
  }
  int remaining = 32 - __clz((int)(kmin ^ kmax));        // low bits that are not common to all keys
  uint64_t prefix = (uint64_t)kmax >> remaining;
  int need = K;
#pragma unroll 1
  while (remaining > 0) {                                // uniform: at most three rounds
    const int bits = remaining < 12 ? remaining : 12;
    const int shift = remaining - bits;
    // the histogram always has 4096 or 256 bins (digits narrower than that leave the top ones empty)
    const int nb = bits > 8 ? 4096 : 256;
    for (int i = tid; i < nb; i += NT) hist[i] = 0;
    __syncthreads();
    for (int64_t i0 = tid; i0 < n; i0 += 8 * NT) {
      uint32_t kk[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) kk[u] = i0 + u * NT < n ? as_global(keys)[i0 + u * NT] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (kk[u] != 0 && ((uint64_t)kk[u] >> remaining) == prefix)
          atomicAdd(&hist[(kk[u] >> shift) & (uint32_t)((1 << bits) - 1)], 1u);
    }
    __syncthreads();
    // sums of 16 bins, top first: psum[t] = bins nb-1-16t .. nb-1-16t-15
    const int np = nb / 16;                               // 256 or 16
    if (tid < np) {
      uint32_t sum = 0;
      for (int i = 0; i < 16; ++i) sum += hist[nb - 1 - (16 * tid + ((i + tid) & 15))];
      psum[tid] = sum;
    }
    __syncthreads();
    if (tid < 64) {
      // lane l owns psum[4l .. 4l+3] (nothing when np is 16 and l >= 4)
      uint32_t mine = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) mine += 4 * lane + i < np ? psum[4 * lane + i] : 0u;
      uint32_t incl = mine;
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) {
        const uint32_t up = __shfl_up(incl, m);
        if (lane >= m) incl += up;
      }
      // the keys that match `prefix` number at least `need`, so some lane reaches it
      const uint64_t reach = __ballot(incl >= (uint32_t)need);
      const int first = __ffsll((unsigned long long)reach) - 1;
      if (lane == first) {
        uint32_t above = incl - mine;                   // keys in the bins above this lane's
        int pi = 4 * lane;
        while (above + psum[pi] < (uint32_t)need) above += psum[pi++];   // ends inside the lane's four
        int digit = nb - 1 - 16 * pi;
        for (int i = 0; i < 16; ++i, --digit) {
          const uint32_t h = hist[digit];
          if (above + h >= (uint32_t)need) {
            bc[0] = (uint32_t)digit;
            bc[1] = above;
            bc[2] = h;
            break;
          }
          above += h;
        }
      }
    }
    __syncthreads();
    need -= (int)bc[1];
    r.n_eq = (int)bc[2];
    prefix = (prefix << bits) | bc[0];
    remaining = shift;
    __syncthreads();                                    // bc and hist are reused by the next pass
    if constexpr (BOUND_ONLY) {
      r.tau = (uint32_t)(prefix << remaining);
      return r;
    }
  }
  r.tau = (uint32_t)prefix;
  r.need = need;
  return r;
}

// Which of the keys equal to tau are taken: the first `need` in index order.  Calls visit(i,
// taken) for every i in [0, n) with keys[i] == tau, in chunks of NT consecutive indices.
// cnt: NT/64 words of LDS.
template <int NT, class Visit>
__device__ __forceinline__ void block_take_ties(const uint32_t* keys, int64_t n, uint32_t tau,
                                                int need, int* cnt, Visit visit) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int running = 0;
  for (int64_t base = 0; base < n; base += NT) {        // uniform trip count
    const int64_t i = base + tid;
    const bool tie = i < n && as_global(keys)[i] == tau;
    const uint64_t bal = __ballot(tie);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) cnt[wave] = __popcll(bal);
    __syncthreads();
    int before = running, total = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
      const int cw = cnt[w];
      if (w < wave) before += cw;
      total += cw;
    }
    if (tie) visit(i, before + rank < need);
    running += total;
  }
}

// Bitonic sort, descending, of P (a power of two) 64-bit keys in LDS by NT threads.
template <int NT>
__device__ __forceinline__ void block_sort_desc(uint64_t* v, int P) {
  const int tid = threadIdx.x;
  for (int k = 2; k <= P; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (P >> 1); t += NT) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int l = i | j;
        const bool desc = (i & k) == 0;
        const uint64_t x = v[i], y = v[l];
        if ((x < y) == desc) {
          v[i] = y;
          v[l] = x;
        }
      }
      __syncthreads();
    }
}
template <int NT>
__device__ __forceinline__ void block_sort_desc(uint32_t* v, int P) {
  const int tid = threadIdx.x;
  for (int k = 2; k <= P; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (P >> 1); t += NT) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int l = i | j;
        const bool desc = (i & k) == 0;
        const uint32_t x = v[i], y = v[l];
        if ((x < y) == desc) {
          v[i] = y;
          v[l] = x;
        }
      }
      __syncthreads();
    }
}

// ---- per beam: scores as sort keys, per-beam cut and probes -------------------------------------
template <int NT>
__device__ __forceinline__ uint32_t block_max_u32(uint32_t v, uint32_t* red) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)v, m);
    v = o > v ? o : v;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  uint32_t r = red[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r = red[w] > r ? red[w] : r;
  return r;
}

// The same selection as block_radix_select for keys held in registers (NV per thread, 0 = unused
// slot, at least K + 1 of them nonzero): digits of 8 bits, starting at the highest bit in which
// the smallest and the largest key differ, so that the first histogram already spreads the keys.
// hist: 256 words of LDS, bc: 4 words, red: NT/64 words.
template <int NT, int NV>
__device__ RadixPick regs_radix_select(const uint32_t (&key)[NV], int K, uint32_t* hist,
                                       uint32_t* bc, uint32_t* red) {
  const int tid = threadIdx.x, lane = tid & 63;
  RadixPick r;
  r.all = false;
  uint32_t mx = 0, mn_inv = 0;
  int n_mine = 0;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    mx = key[j] > mx ? key[j] : mx;
    const uint32_t inv = key[j] ? ~key[j] : 0u;
    mn_inv = inv > mn_inv ? inv : mn_inv;
    n_mine += key[j] != 0u;
  }
  const uint32_t kmax = block_max_u32<NT>(mx, red);
  const uint32_t kmin = ~block_max_u32<NT>(mn_inv, red);
  if (kmin == kmax) {                                   // every key the same
    r.tau = kmax;
    r.need = K;
    r.n_eq = (int)block_sum<NT>((float)n_mine, reinterpret_cast<float*>(red));
    return r;
  }
  int remaining = 32 - __clz((int)(kmin ^ kmax));        // low bits that are not common to all keys
  uint64_t pre = (uint64_t)kmax >> remaining;
  int need = K, n_eq = 0;
  while (remaining > 0) {                                // uniform: at most four rounds
    const int bits = remaining < 8 ? remaining : 8;
    const int shift = remaining - bits;
    const int nb = 1 << bits;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    // (32-bit forms of "the bits above `remaining` equal pre"; remaining == 32: no such bits)
    const uint32_t hi_mask = remaining >= 32 ? 0u : ~0u << remaining;
    const uint32_t hi_want = remaining >= 32 ? 0u : (uint32_t)pre << remaining;
#pragma unroll
    for (int j = 0; j < NV; ++j)
      if (key[j] != 0u && (key[j] & hi_mask) == hi_want)
        atomicAdd(&hist[(key[j] >> shift) & (uint32_t)(nb - 1)], 1u);
    __syncthreads();
    if (tid < 64) {
      // lane l owns the bins nb-1-4l .. nb-1-4l-3 (none when nb is smaller): top first
      uint32_t h[4], mine = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int bin = nb - 1 - (4 * lane + i);
        h[i] = bin >= 0 ? hist[bin] : 0u;
        mine += h[i];
      }
      uint32_t incl = mine;
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, m);
        if (lane >= m) incl += up;
      }
      const uint64_t reach = __ballot(incl >= (uint32_t)need);
      const int first = __ffsll((unsigned long long)reach) - 1;     // exists: the keys matching
      if (lane == first) {                                          // `pre` number at least `need`
        uint32_t above = incl - mine;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (above + h[i] >= (uint32_t)need) {
            bc[0] = (uint32_t)(nb - 1 - (4 * lane + i));
            bc[1] = above;
            bc[2] = h[i];
            break;
          }
          above += h[i];
        }
      }
    }
    __syncthreads();
    need -= (int)bc[1];
    n_eq = (int)bc[2];
    pre = (pre << bits) | bc[0];
    remaining = shift;
    __syncthreads();
  }
  r.tau = (uint32_t)pre;
  r.need = need;
  r.n_eq = n_eq;
  return r;
}

// Set membership of two children (codes c0, c1) of one beam with both lookups in flight at once.
__device__ __forceinline__ void set_contains_pair(const SetView& s, uint64_t pkey, uint32_t c0,
                                                  bool live0, uint32_t c1, bool live1, bool& in0,
                                                  bool& in1) {
  const uint64_t prefix[2] = {pkey, pkey};
  const uint32_t code[2] = {c0, c1};
  const bool live[2] = {live0, live1};
  bool in[2];
  set_contains_many<2>(s, prefix, code, live, in);
  in0 = in[0];
  in1 = in[1];
}

// One workgroup per beam.  VERIFY: a set is consulted at this level, so the beam is cut to its K
// most probable codes first (that cut decides which candidates are verified; without a set the
// request-level selection alone gives the same result) and the survivors are probed.
// NV > 0: T_l <= NV * 256, the beam's logits and keys stay in registers (one read and one write of
// the row; the K survivors are gathered in LDS so that every lane has probes in flight);
// NV == 0: any T_l, the row is read again from L2 for every pass.
template <bool VERIFY, int NV>
__global__ __launch_bounds__(kWideRowThreads) void wide_rows_kernel(WideArgs a) {
  constexpr int NT = kWideRowThreads;
  constexpr bool kRegs = NV > 0;
  __shared__ float red[NT / 64];
  __shared__ uint32_t hist[VERIFY ? (kRegs ? 256 : 4096 + 256) : 1];
  __shared__ uint64_t cand[VERIFY && kRegs ? NEZHA_MAX_WIDE_BEAM : 1];    // (key, code) of the survivors
  __shared__ uint32_t bc[4];
  __shared__ int cnt[NT / 64];
  __shared__ uint64_t kept[VERIFY ? NEZHA_MAX_WIDE_BEAM : 1];            // those found in the set
  __shared__ uint32_t member[VERIFY && kRegs ? NV * NT / 32 : 1];         // the same as a bitmap over the codes
  __shared__ int n_cand, n_kept, kept_base;
  const int64_t row = blockIdx.x;
  const int V = a.V, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t* zk = a.zk + row * V;
  const uint64_t pkey = a.key_in ? a.key_in[row] : 0ull;
  const float sp = a.score_in ? a.score_in[row] : 0.f;
  if (pkey == kEmpty) {                                  // an empty beam slot has no children
    for (int v = tid; v < V; v += NT) as_global(zk)[v] = 0u;
    return;
  }
  const int64_t req = row / a.K_in;
  const uint32_t idx0 = (uint32_t)(row - req * a.K_in) * (uint32_t)V;   // index of code 0 in the request
  if (tid == 0) n_kept = 0;                              // (barriers follow before its first use)
  // a candidate found in the set: its key stays, and it joins the request's list
  auto keep = [&](int v, uint32_t k) {
    kept[atomicAdd(&n_kept, 1)] = ((uint64_t)k << 32) | (uint32_t)~(idx0 + (uint32_t)v);
  };
  if constexpr (kRegs) {
    float z[NV];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int v = tid + j * NT;
      z[j] = v < V ? __uint_as_float(as_global(zk)[v]) : -INFINITY;
      m = fmaxf(m, z[j]);
    }
    m = block_max<NT>(m, red);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) s += __expf(z[j] - m);
    s = block_sum<NT>(s, red);
    const float lse = m + logf(s);
    uint32_t key[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) key[j] = tid + j * NT < V ? ordered_bits(sp + (z[j] - lse)) : 0u;
    if constexpr (!VERIFY) {
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (tid + j * NT < V) as_global(zk)[tid + j * NT] = key[j];
    } else {
      if (a.K >= V) {
        // no cut: every code is probed, two at a time
#pragma unroll
        for (int j = 0; j < NV; j += 2) {
          const int v0 = tid + j * NT, v1 = v0 + NT;
          bool in0, in1;
          set_contains_pair(a.set, pkey, (uint32_t)v0, v0 < V, (uint32_t)v1, v1 < V, in0, in1);
          if (v0 < V) as_global(zk)[v0] = in0 ? key[j] : 0u;
          if (v1 < V) as_global(zk)[v1] = in1 ? key[j + 1] : 0u;
          if (in0) keep(v0, key[j]);
          if (in1) keep(v1, key[j + 1]);
        }
      } else {
        if (tid == 0) n_cand = 0;
        const RadixPick p = regs_radix_select<NT, NV>(key, a.K, hist, bc,
                                                      reinterpret_cast<uint32_t*>(red));
        const bool ordered_ties = p.need < p.n_eq;       // more codes tie with the K-th than fit
        int running = 0;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          const int v = tid + j * NT;
          bool take = key[j] > p.tau || (key[j] == p.tau && !ordered_ties);
          if (ordered_ties) {                            // uniform branch: the lower codes stay
            const bool tie = key[j] == p.tau;
            const uint64_t bal = __ballot(tie);
            __syncthreads();
            if (lane == 0) cnt[wave] = __popcll(bal);
            __syncthreads();
            int before = running, total = 0;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) {
              if (w < wave) before += cnt[w];
              total += cnt[w];
            }
            running += total;
            if (tie) take = before + (int)__popcll(bal & ((1ull << lane) - 1ull)) < p.need;
          }
          // one LDS reservation per wave (atomics on one address run one after the other)
          const uint64_t tb = __ballot(take);
          int at = 0;
          if (lane == 0 && tb) at = atomicAdd(&n_cand, __popcll(tb));
          at = __shfl(at, 0) + __popcll(tb & ((1ull << lane) - 1ull));
          if (take) cand[at] = ((uint64_t)key[j] << 32) | (uint32_t)v;    // K entries in all
        }
        if (tid < NV * NT / 32) member[tid] = 0u;
        __syncthreads();
        const int n = n_cand;
        for (int i = tid; i < n; i += 2 * NT) {
          const bool live1 = i + NT < n;
          const uint64_t c0 = cand[i], c1 = live1 ? cand[i + NT] : 0ull;
          bool in0, in1;
          set_contains_pair(a.set, pkey, (uint32_t)c0, true, (uint32_t)c1, live1, in0, in1);
          if (in0) {
            atomicOr(&member[(uint32_t)c0 >> 5], 1u << ((uint32_t)c0 & 31u));
            keep((int)(uint32_t)c0, (uint32_t)(c0 >> 32));
          }
          if (in1) {
            atomicOr(&member[(uint32_t)c1 >> 5], 1u << ((uint32_t)c1 & 31u));
            keep((int)(uint32_t)c1, (uint32_t)(c1 >> 32));
          }
        }
        // the row is written by the threads that hold its keys, in full lines: survivors keep
        // their key, everything else becomes 0
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          const int v = tid + j * NT;
          if (v < V) as_global(zk)[v] = (member[v >> 5] >> (v & 31)) & 1u ? key[j] : 0u;
        }
      }
    }
  } else {
    float m = -INFINITY;
    for (int v = tid; v < V; v += NT) m = fmaxf(m, __uint_as_float(as_global(zk)[v]));
    m = block_max<NT>(m, red);
    float s = 0.f;
    for (int v = tid; v < V; v += NT) s += expf(__uint_as_float(as_global(zk)[v]) - m);
    s = block_sum<NT>(s, red);
    const float lse = m + logf(s);
    for (int v = tid; v < V; v += NT) {
      const float z = __uint_as_float(as_global(zk)[v]);
      as_global(zk)[v] = ordered_bits(sp + (z - lse));
    }
    if constexpr (VERIFY) {
      __syncthreads();                                   // the keys are read back by other threads
      uint32_t tau = 0;
      if (a.K < V) {
        const RadixPick p = block_radix_select<NT>(zk, V, a.K, hist, bc);
        if (!p.all) {
          tau = p.tau;
          if (p.need < p.n_eq) {
            // more codes tie with the K-th than fit: the lower codes stay
            block_take_ties<NT>(zk, V, tau, p.need, cnt, [&](int64_t i, bool taken) {
              if (!taken) as_global(zk)[i] = 0u;
            });
            __syncthreads();
          }
        }
      }
      for (int v = tid; v < V; v += NT) {
        const uint32_t k = as_global(zk)[v];
        if (k == 0u) continue;
        const bool in = k >= tau && set_contains(a.set, pkey, (uint32_t)v);
        if (!in) as_global(zk)[v] = 0u;
        else keep(v, k);
      }
    }
  }
  if constexpr (VERIFY) {
    // the row's survivors join the request's list (one reservation per row)
    __syncthreads();
    const int n = n_kept;
    if (tid == 0) kept_base = atomicAdd(&a.gcount[req], n);
    __syncthreads();
    uint64_t* glist = a.glist + req * kWideListCap;
    for (int i = tid; i < n; i += NT)
      if (kept_base + i < kWideListCap) glist[kept_base + i] = kept[i];
  }
}

// ---- per request: the K best keys --------------------------------------------------------------
struct WideSelectArgs {
  const uint32_t* zk;       // [B, K_in * T_l] sort keys, 0 = not a candidate
  const uint64_t* key_in;
  const float* score_in;
  const void* state_in;
  const void* E;
  const void* U;
  uint64_t mult;
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  void* state_out;
  int32_t* count_out;
  int K_in, K, V, e, transition;
  // when a request is shared by `splits` > 1 workgroups (small batches):
  int splits;
  int n_tops;               // keys per request in tops
  uint32_t* tops;           // [B, n_tops] distinct candidates of the request (each share's K largest,
                            // or what wide_fused_bf16_kernel kept), among them the bound is sought
  uint64_t* glist;          // [B, kWideListCap] (key, ~index) at or above the bound
  int32_t* gcount;          // [B]
};
inline size_t wide_select_lds() {
  return (size_t)kWideListCap * 8 + (size_t)2 * kWideThreads * 4 + (size_t)2 * 1024 * 4 + 64;
}
// Workgroups per request: a request's keys are walked by one workgroup when the batch fills the
// chip on its own, by up to 16 when it does not.
inline int wide_select_splits(int B) {
  if (B >= 256) return 1;
  int s = 512 / (B > 0 ? B : 1);
  return s > 16 ? 16 : s < 1 ? 1 : s;
}

// The LDS of the selection kernels.
struct WideLds {
  uint64_t* list;        // [kWideListCap]
  uint32_t* top;         // [2 * kWideThreads]; later the tie counters
  int32_t* fin_parent;   // [1024]
  int32_t* fin_code;     // [1024]
  uint32_t* bc;          // [4]
  int* n_list;           // [1]
  uint32_t* hist;        // 4096 + 256 words inside list (exact selection only)
};
__device__ __forceinline__ WideLds wide_lds_layout(uint64_t* base) {
  WideLds l;
  l.list = base;
  l.top = reinterpret_cast<uint32_t*>(base + kWideListCap);
  l.fin_parent = reinterpret_cast<int32_t*>(l.top + 2 * kWideThreads);
  l.fin_code = l.fin_parent + 1024;
  l.bc = reinterpret_cast<uint32_t*>(l.fin_code + 1024);
  l.n_list = reinterpret_cast<int*>(l.bc + 4);
  l.hist = reinterpret_cast<uint32_t*>(base + 2048);
  return l;
}

// First pass: every thread keeps the two largest keys of the 16-byte groups [q_begin, q_end) it
// visits.  A thread visits one group of each run of 1024 groups, at a position that rotates from
// run to run: with T_l = 4096 a fixed position would be the same four codes of every beam, and
// the codes the user part favours are the same for all beams of a request, so the best keys would
// crowd into few threads and the bound would be weak.
__device__ __forceinline__ void wide_thread_top2(const uint32_t* keys, int64_t q_begin,
                                                 int64_t q_end, uint32_t& t0, uint32_t& t1) {
  constexpr int NT = kWideThreads;
  const int tid = threadIdx.x;
  auto note = [&](const uint4& k4) {
    const uint32_t kk[4] = {k4.x, k4.y, k4.z, k4.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = kk[j] > t0 ? t0 : kk[j];
      t0 = kk[j] > t0 ? kk[j] : t0;
      t1 = lo > t1 ? lo : t1;
    }
  };
  int64_t q0 = q_begin;
  int run = 0;
  for (; q0 + 4 * NT <= q_end; q0 += 4 * NT, run += 4) {   // four loads in flight per thread
    uint4 k4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      k4[u] = load_global_u4(keys + 4 * (q0 + u * NT + ((tid + 37 * (run + u)) & (NT - 1))));
#pragma unroll
    for (int u = 0; u < 4; ++u) note(k4[u]);
  }
  for (; q0 < q_end; q0 += NT, ++run) {
    const int64_t q = q0 + ((tid + 37 * run) & (NT - 1));
    if (q < q_end) note(load_global_u4(keys + 4 * q));
  }
}

// Second pass: keys of the groups [q_begin, q_end) at or above tau0 are handed to put(count) ->
// first position, wave by wave, and stored through store(position, entry) as (key, ~index).
template <class Reserve, class Store>
__device__ __forceinline__ void wide_collect(const uint32_t* keys, int64_t q_begin, int64_t q_end,
                                             uint32_t tau0, Reserve reserve, Store store) {
  constexpr int NT = kWideThreads;
  const int tid = threadIdx.x, lane = tid & 63;
  auto collect = [&](const uint4& k4, int64_t q) {          // called by whole waves
    const uint32_t kk[4] = {k4.x, k4.y, k4.z, k4.w};
    const bool any = (kk[0] >= tau0) | (kk[1] >= tau0) | (kk[2] >= tau0) | (kk[3] >= tau0);
    if (__ballot(any) == 0ull) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool in = kk[j] >= tau0;
      const uint64_t bal = __ballot(in);
      if (bal == 0ull) continue;
      int base = 0;
      if (lane == 0) base = reserve(__popcll(bal));
      base = __shfl(base, 0);
      const int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
      if (in && pos < kWideListCap)
        store(pos, ((uint64_t)kk[j] << 32) | (uint32_t)~(uint32_t)(4 * q + j));
    }
  };
  int64_t q0 = q_begin;
  for (; q0 + 4 * NT <= q_end; q0 += 4 * NT) {
    uint4 k4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) k4[u] = load_global_u4(keys + 4 * (q0 + u * NT + tid));
#pragma unroll
    for (int u = 0; u < 4; ++u) collect(k4[u], q0 + u * NT + tid);
  }
  for (; q0 < q_end; q0 += NT) {                            // uniform trip count
    const int64_t q = q0 + tid;
    uint4 k4 = uint4{0, 0, 0, 0};
    if (q < q_end) k4 = load_global_u4(keys + 4 * q);
    collect(k4, q);
  }
}

// From the n_in entries of the LDS list (or, when the list overflowed, from an exact radix
// selection over all keys) to the level's outputs: sort by (score, parent, code), write the K
// best, apply the Transition.
template <bool BF16>
__device__ __forceinline__ void wide_finish(const WideSelectArgs& a, int b, const uint32_t* keys,
                                            int64_t n, const WideLds& l, int n_in) {
  constexpr int NT = kWideThreads;
  const int tid = threadIdx.x, lane = tid & 63;
  const int K = a.K, V = a.V;
  uint64_t* list = l.list;
  if (n_in > kWideListCap) {
    // exact selection; the list is rebuilt from the keys above the K-th and its first ties
    const RadixPick p = block_radix_select<NT>(keys, n, K, l.hist, l.bc);
    if (tid == 0) *l.n_list = 0;
    __syncthreads();
    const uint32_t tau = p.all ? 1u : p.tau;
    for (int64_t i0 = 0; i0 < n; i0 += NT) {
      const int64_t i = i0 + tid;
      const uint32_t k = i < n ? as_global(keys)[i] : 0u;
      const bool in = p.all ? (k != 0u) : (k > tau);
      const uint64_t bal = __ballot(in);
      if (bal == 0ull) continue;
      int base = 0;
      if (lane == 0) base = atomicAdd(l.n_list, __popcll(bal));
      base = __shfl(base, 0);
      const int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
      if (in) list[pos] = ((uint64_t)k << 32) | (uint32_t)~(uint32_t)i;   // at most K entries
    }
    if (!p.all) {
      block_take_ties<NT>(keys, n, tau, p.need, reinterpret_cast<int*>(l.top),
                          [&](int64_t i, bool taken) {
        if (taken) list[atomicAdd(l.n_list, 1)] = ((uint64_t)tau << 32) | (uint32_t)~(uint32_t)i;
      });
    }
    __syncthreads();
    n_in = *l.n_list;
    __syncthreads();
  }
  int P = 2;
  while (P < n_in) P <<= 1;
  for (int i = n_in + tid; i < P; i += NT) list[i] = 0ull;
  __syncthreads();
  block_sort_desc<NT>(list, P);

  const int cnt = n_in < K ? n_in : K;
  for (int j = tid; j < K; j += NT) {
    const int64_t o = (int64_t)b * K + j;
    if (j < cnt) {
      const uint64_t sk = list[j];
      const uint32_t idx = ~(uint32_t)sk;
      const int par = (int)(idx / (uint32_t)V);
      const int code = (int)(idx - (uint32_t)par * (uint32_t)V);
      a.key_out[o] = (a.key_in ? a.key_in[(int64_t)b * a.K_in + par] : 0ull) +
                     (uint64_t)(uint32_t)code * a.mult;
      a.score_out[o] = unordered_bits((uint32_t)(sk >> 32));
      a.parent_out[o] = par;
      a.code_out[o] = code;
      l.fin_parent[j] = par;
      l.fin_code[j] = code;
    } else {
      a.key_out[o] = kEmpty;
      a.score_out[o] = -INFINITY;
      a.parent_out[o] = -1;
      a.code_out[o] = -1;
      l.fin_parent[j] = -1;
      l.fin_code[j] = -1;
    }
  }
  if (tid == 0 && a.count_out) a.count_out[b] = cnt;
  __syncthreads();
  if (a.state_out) {
    if (a.transition == NEZHA_TRANSITION_RNN)
      update_states_rnn<BF16>(a.state_in, a.E, a.U, a.state_out, b, K, a.K_in, a.e, l.fin_parent,
                              l.fin_code, tid, NT);
    else
      update_states<BF16>(a.state_in, a.E, a.state_out, b, K, a.K_in, a.e, l.fin_parent, l.fin_code,
                          tid, NT);
  }
}

// One workgroup of 1024 threads per request.  First pass over the request's K_in * T_l keys:
// every thread keeps the two largest keys of the indices it visits; the K-th largest of those
// 2048 keys is a lower bound of the K-th largest key (they are K distinct candidates).  Second
// pass: keys at or above the bound go to an LDS list as (key, ~index); the list is sorted, which
// orders equal scores by parent and code, and its first K entries are the level's beams.  When
// the list would overflow (scores crowded into the indices of few threads, massive ties) the
// selection is done exactly by radix passes instead.
template <bool BF16>
__global__ __launch_bounds__(kWideThreads) void wide_select_kernel(WideSelectArgs a) {
  constexpr int NT = kWideThreads;
  extern __shared__ __align__(16) uint64_t wide_lds[];
  const WideLds l = wide_lds_layout(wide_lds);
  const int b = blockIdx.x, tid = threadIdx.x;
  const int64_t n = (int64_t)a.K_in * a.V;               // a multiple of 16
  const uint32_t* keys = a.zk + (int64_t)b * n;

  uint32_t t0 = 0, t1 = 0;
  wide_thread_top2(keys, 0, n >> 2, t0, t1);
  l.top[2 * tid] = t0;
  l.top[2 * tid + 1] = t1;
  if (tid == 0) *l.n_list = 0;
  __syncthreads();
  block_sort_desc<NT>(l.top, 2 * NT);
  uint32_t tau0 = l.top[a.K - 1];
  if (tau0 == 0u) tau0 = 1u;                             // fewer than K candidates seen: take all
  __syncthreads();
  wide_collect(keys, 0, n >> 2, tau0, [&](int c) { return atomicAdd(l.n_list, c); },
               [&](int pos, uint64_t v) { l.list[pos] = v; });
  __syncthreads();
  const int n_in = *l.n_list;
  __syncthreads();
  wide_finish<BF16>(a, b, keys, n, l, n_in);
}

// Where a set was consulted the survivors are few and wide_rows_kernel has listed them already:
// wide_finish_kernel alone follows.  Otherwise, for batches too small to fill the chip with one
// workgroup per request, the selection runs in three launches: blockIdx.x = request * splits + share.
//   wide_bound_kernel    every share's K largest (thread top-2) keys -> tops
//   wide_collect_kernel  bound = K-th largest of the request's splits * K such keys (every
//                        workgroup of the request finds it again); the share's keys at or above
//                        it -> the request's list in global memory
//   wide_finish_kernel   one workgroup per request: list -> LDS -> outputs
__global__ __launch_bounds__(kWideThreads) void wide_bound_kernel(WideSelectArgs a) {
  constexpr int NT = kWideThreads;
  __shared__ uint32_t top[2 * NT];
  const int b = blockIdx.x / a.splits, s = blockIdx.x - b * a.splits, tid = threadIdx.x;
  const int64_t n = (int64_t)a.K_in * a.V, n4 = n >> 2;
  const uint32_t* keys = a.zk + (int64_t)b * n;
  uint32_t t0 = 0, t1 = 0;
  wide_thread_top2(keys, n4 * s / a.splits, n4 * (s + 1) / a.splits, t0, t1);
  top[2 * tid] = t0;
  top[2 * tid + 1] = t1;
  if (s == 0 && tid == 0) a.gcount[b] = 0;
  __syncthreads();
  block_sort_desc<NT>(top, 2 * NT);
  for (int j = tid; j < a.K; j += NT) a.tops[((int64_t)b * a.splits + s) * a.K + j] = top[j];
}

__global__ __launch_bounds__(kWideThreads) void wide_collect_kernel(WideSelectArgs a) {
  constexpr int NT = kWideThreads;
  // the histogram of the bound search, then this workgroup's part of the list (kWideListCap
  // entries: one reservation in the request's list per workgroup, not one per wave)
  extern __shared__ __align__(16) uint64_t wide_lds[];
  __shared__ uint32_t bc[4];
  __shared__ int n_local, base;
  uint32_t* hist = reinterpret_cast<uint32_t*>(wide_lds);
  uint64_t* list = wide_lds;
  const int b = blockIdx.x / a.splits, s = blockIdx.x - b * a.splits, tid = threadIdx.x;
  const int64_t n = (int64_t)a.K_in * a.V, n4 = n >> 2;
  const uint32_t* keys = a.zk + (int64_t)b * n;
  // any lower bound of the K-th largest of these keys will do: one digit is enough
  const RadixPick p = block_radix_select<NT, true>(a.tops + (int64_t)b * a.n_tops, a.n_tops, a.K, hist,
                                                   bc);
  const uint32_t tau0 = p.all ? 1u : p.tau;              // fewer than K candidates seen: take all
  if (tid == 0) n_local = 0;
  __syncthreads();
  wide_collect(keys, n4 * s / a.splits, n4 * (s + 1) / a.splits, tau0,
               [&](int c) { return atomicAdd(&n_local, c); },
               [&](int pos, uint64_t v) { list[pos] = v; });
  __syncthreads();
  const int m = n_local;                                 // may exceed what was stored: then the
  if (tid == 0) base = atomicAdd(&a.gcount[b], m);       // request's count exceeds the cap as well
  __syncthreads();
  uint64_t* glist = a.glist + (int64_t)b * kWideListCap;
  for (int i = tid; i < m && i < kWideListCap; i += NT)
    if (base + i < kWideListCap) glist[base + i] = list[i];
}

template <bool BF16>
__global__ __launch_bounds__(kWideThreads) void wide_finish_kernel(WideSelectArgs a) {
  constexpr int NT = kWideThreads;
  extern __shared__ __align__(16) uint64_t wide_lds[];
  const WideLds l = wide_lds_layout(wide_lds);
  const int b = blockIdx.x, tid = threadIdx.x;
  const int64_t n = (int64_t)a.K_in * a.V;
  const uint32_t* keys = a.zk + (int64_t)b * n;
  const int n_in = a.gcount[b];
  if (n_in <= kWideListCap) {
    const uint64_t* glist = a.glist + (int64_t)b * kWideListCap;
    for (int i = tid; i < n_in; i += NT) l.list[i] = glist[i];
  }
  __syncthreads();
  wide_finish<BF16>(a, b, keys, n, l, n_in);
}
