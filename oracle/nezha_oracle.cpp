// CPU oracle for the NEZHA draft + verify step.  TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, literal implementation of what the decoding step computes,
// written from the paper (Sec. 3.2 Eq. 1-3, Sec. 3.3 Eq. 4-5, Alg. 3 inference
// part).  It exists so that the GPU library can be checked against it; only the
// tests, the smoke check and the CPU-baseline leg of the benchmark may call it.
// It shares no code with the GPU library and must never be used as a fallback.
//
// Conventions fixed here where the paper is silent (each is listed with its
// reason in the design notes): the logit head of Eq. 2 is one linear layer on
// the concatenation [h_l ; c_l] with no bias; the state c lives in the code-
// embedding space, starts at zero and is updated by addition (the Transition
// the paper defines completely, its ablation variant 3); probabilities are a
// softmax over the level's codes only; cumulative probability is carried as a
// sum of log-probabilities; ties go to the lower code, then to the better
// ranked parent; verification happens at the last level only.
//
// Two widenings beyond that path, each behind an argument that defaults to the
// path above: the recurrent Transition c' = tanh(U c + e_l) (the paper's main
// variant says "an RNN" without giving the cell; the plain Elman cell without
// bias is the reading taken), and verification below the last level against a
// set of valid prefixes (the per-level filter the paper mentions in passing).
//
// Arithmetic: inputs are float32 (bf16 workloads pass bf16 values widened to
// float32); every dot product, the log-sum-exp and the log-probabilities are in
// double; cumulative scores are stored as float32.
//
// Parity pins (tests/test_oracle_*.py): the printed example of Eq. 4, bijection
// by enumeration, membership against a sorted array and a bitmap, logits and
// log-softmax against a library float64 matmul / log_softmax, the tie rule on
// all-zero weights, and brute-force enumeration of every tuple on tiny
// codebooks.  Draft *quality* (hit rate etc.) is parity unpinned: it needs the
// paper's datasets and trained weights.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <numeric>
#include <thread>
#include <unordered_set>
#include <vector>

namespace {

struct ItemSet {
  std::unordered_set<uint64_t> keys;
  int32_t L;
  std::vector<int32_t> radices;
};

// Positional multipliers of Eq. 4: mult[l] = prod_{j<l} T_j, empty product = 1.
// Returns false when prod_l T_l does not fit below 2^64 - 1.
bool multipliers(int32_t L, const int32_t* radices, std::vector<uint64_t>& mult) {
  mult.assign(L, 1);
  unsigned __int128 p = 1;
  for (int32_t l = 0; l < L; ++l) {
    if (radices[l] < 1) return false;
    mult[l] = (uint64_t)p;
    p *= (unsigned __int128)radices[l];
    if (p > (unsigned __int128)std::numeric_limits<uint64_t>::max()) return false;
  }
  return true;
}

// Eq. 4: V_i = sum_l t_l * prod_{j<l} T_j  (level 1 is the least significant digit).
bool pack_one(const int32_t* t, int32_t L, const int32_t* radices,
              const std::vector<uint64_t>& mult, uint64_t& key) {
  key = 0;
  for (int32_t l = 0; l < L; ++l) {
    if (t[l] < 0 || t[l] >= radices[l]) return false;
    key += (uint64_t)t[l] * mult[l];
  }
  return true;
}

float round_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) return x;  // inf / nan unchanged
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  u &= 0xFFFF0000u;
  float y;
  std::memcpy(&y, &u, 4);
  return y;
}

struct Cand {
  uint64_t key;
  float score;
  int32_t parent;
  int32_t code;
};

struct LevelArgs {
  int32_t B, L, level, K, K_in, d, e;
  const int32_t* radices;
  const float* H;
  int64_t h_row_stride;
  const float* W;
  const float* E;
  const float* state_in;
  const uint64_t* key_in;
  const float* score_in;
  const ItemSet* set;
  const float* U;       // [e, e] row major, used when transition == 1
  int transition;       // 0: c' = c + e_l;  1: c'[j] = tanh(sum_i U[j][i] c[i] + e_l[j])
  int round_state_bf16;
  uint64_t* key_out;
  float* score_out;
  int32_t* parent_out;
  int32_t* code_out;
  float* state_out;
  int32_t* count_out;
  double* logp_out;
  uint64_t mult;
};

// One request, one level of Alg. 3 (inference part).
void level_one_request(const LevelArgs& a, int32_t b) {
  const int32_t V = a.radices[a.level - 1];
  const int32_t d = a.d, e = a.e, K = a.K, K_in = a.K_in;
  std::vector<double> x(d + e), z(V), logp(V);
  std::vector<int32_t> order(V);
  std::vector<Cand> cands;
  cands.reserve((size_t)K_in * K);

  for (int32_t k = 0; k < K_in; ++k) {
    // An empty beam slot (index 2^64-1: fewer than K beams survived the level before)
    // has no children.
    const bool empty_slot =
        a.key_in && a.key_in[(int64_t)b * K_in + k] == std::numeric_limits<uint64_t>::max();
    if (empty_slot) {
      if (a.logp_out)
        for (int32_t v = 0; v < V; ++v)
          a.logp_out[((int64_t)b * K_in + k) * V + v] = -std::numeric_limits<double>::infinity();
      continue;
    }
    // Eq. 2: logits of beam k from the placeholder hidden h_l and the beam's state.
    for (int32_t i = 0; i < d; ++i) x[i] = (double)a.H[(int64_t)b * a.h_row_stride + i];
    for (int32_t i = 0; i < e; ++i)
      x[d + i] = a.state_in ? (double)a.state_in[((int64_t)b * K_in + k) * e + i] : 0.0;
    std::fill(z.begin(), z.end(), 0.0);
    for (int32_t i = 0; i < d + e; ++i) {
      const float* wrow = a.W + (int64_t)i * V;
      const double xi = x[i];
      for (int32_t v = 0; v < V; ++v) z[v] += xi * (double)wrow[v];
    }
    // log-softmax over the level's codes.
    double m = z[0];
    for (int32_t v = 1; v < V; ++v) m = std::max(m, z[v]);
    double s = 0.0;
    for (int32_t v = 0; v < V; ++v) s += std::exp(z[v] - m);
    const double lse = m + std::log(s);
    for (int32_t v = 0; v < V; ++v) logp[v] = z[v] - lse;
    if (a.logp_out)
      std::memcpy(a.logp_out + ((int64_t)b * K_in + k) * V, logp.data(), sizeof(double) * V);
    // The K most probable codes of this beam; equal probabilities: lower code first.
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t p, int32_t q) { return logp[p] > logp[q]; });
    const uint64_t pkey = a.key_in ? a.key_in[(int64_t)b * K_in + k] : 0;
    const double pscore = a.score_in ? (double)a.score_in[(int64_t)b * K_in + k] : 0.0;
    for (int32_t r = 0; r < std::min(K, V); ++r) {
      Cand c;
      c.code = order[r];
      c.parent = k;
      c.key = pkey + (uint64_t)c.code * a.mult;           // Eq. 4, one more digit
      c.score = (float)(pscore + logp[c.code]);            // log of the cumulative probability
      cands.push_back(c);
    }
  }
  // Eq. 5: drop candidates that are not in the set, keeping order.  A set of full tuples
  // (its L equals the step's L) is consulted at the last level; a set of prefixes of
  // length `level` at that level.
  if (a.set && a.set->L == a.level) {
    std::vector<Cand> kept;
    for (const Cand& c : cands)
      if (a.set->keys.count(c.key)) kept.push_back(c);
    cands.swap(kept);
  }
  // Keep the K candidates of largest cumulative probability (stable: ties keep
  // the (parent rank, within-beam rank) order in which they were generated).
  std::stable_sort(cands.begin(), cands.end(),
                   [](const Cand& p, const Cand& q) { return p.score > q.score; });
  const int32_t cnt = (int32_t)std::min<size_t>((size_t)K, cands.size());
  a.count_out[b] = cnt;
  for (int32_t j = 0; j < K; ++j) {
    const int64_t o = (int64_t)b * K + j;
    if (j < cnt) {
      a.key_out[o] = cands[j].key;
      a.score_out[o] = cands[j].score;
      a.parent_out[o] = cands[j].parent;
      a.code_out[o] = cands[j].code;
    } else {
      a.key_out[o] = std::numeric_limits<uint64_t>::max();
      a.score_out[o] = -std::numeric_limits<float>::infinity();
      a.parent_out[o] = -1;
      a.code_out[o] = -1;
    }
    // Eq. 3: state of the survivor, by addition or by the recurrent cell.
    if (a.state_out) {
      float* so = a.state_out + o * e;
      if (j < cnt) {
        const float* erow = a.E + (int64_t)cands[j].code * e;
        const float* prow =
            a.state_in ? a.state_in + ((int64_t)b * K_in + cands[j].parent) * e : nullptr;
        for (int32_t i = 0; i < e; ++i) {
          float next;
          if (a.transition == 1) {
            double acc = (double)erow[i];
            if (prow)
              for (int32_t t = 0; t < e; ++t) acc += (double)a.U[(int64_t)i * e + t] * (double)prow[t];
            next = (float)std::tanh(acc);
          } else {
            next = (prow ? prow[i] : 0.0f) + erow[i];
          }
          so[i] = a.round_state_bf16 ? round_bf16(next) : next;
        }
      } else {
        for (int32_t i = 0; i < e; ++i) so[i] = 0.0f;
      }
    }
  }
}

}  // namespace

extern "C" {

// Eq. 4 on n tuples.  ok[i] = 0 (and keys[i] = 2^64-1) when a code is out of range.
// Returns -4 when prod T_l does not fit, else 0.
int orc_pack(const int32_t* codes, int64_t n, int32_t L, const int32_t* radices,
             uint64_t* keys, uint8_t* ok) {
  std::vector<uint64_t> mult;
  if (!multipliers(L, radices, mult)) return -4;
  for (int64_t i = 0; i < n; ++i) {
    uint64_t k;
    const bool good = pack_one(codes + i * L, L, radices, mult, k);
    keys[i] = good ? k : std::numeric_limits<uint64_t>::max();
    if (ok) ok[i] = good ? 1 : 0;
  }
  return 0;
}

// Inverse of Eq. 4 (successive division by the radices, level 1 first).
int orc_unpack(const uint64_t* keys, int64_t n, int32_t L, const int32_t* radices,
               int32_t* codes) {
  for (int64_t i = 0; i < n; ++i) {
    uint64_t k = keys[i];
    for (int32_t l = 0; l < L; ++l) {
      codes[i * L + l] = (int32_t)(k % (uint64_t)radices[l]);
      k /= (uint64_t)radices[l];
    }
  }
  return 0;
}

// The set of valid item indices of Eq. 5.  *err: 0 ok, -4 code out of range or overflow.
void* orc_set_new(const int32_t* codes, int64_t n, int32_t L, const int32_t* radices, int* err) {
  std::vector<uint64_t> mult;
  *err = 0;
  if (!multipliers(L, radices, mult)) {
    *err = -4;
    return nullptr;
  }
  ItemSet* s = new ItemSet;
  s->L = L;
  s->radices.assign(radices, radices + L);
  s->keys.reserve((size_t)n * 2);
  for (int64_t i = 0; i < n; ++i) {
    uint64_t k;
    if (!pack_one(codes + i * L, L, radices, mult, k)) {
      delete s;
      *err = -4;
      return nullptr;
    }
    s->keys.insert(k);
  }
  return s;
}

int64_t orc_set_size(const void* h) { return (int64_t) static_cast<const ItemSet*>(h)->keys.size(); }

void orc_set_free(void* h) { delete static_cast<ItemSet*>(h); }

void orc_set_contains_keys(const void* h, const uint64_t* keys, int64_t n, uint8_t* mask) {
  const ItemSet* s = static_cast<const ItemSet*>(h);
  for (int64_t i = 0; i < n; ++i) mask[i] = s->keys.count(keys[i]) ? 1 : 0;
}

// Eq. 4 + Eq. 5 on n query tuples: mask, ascending indices of the accepted
// tuples, and their number.  A tuple with a code outside its radix is rejected.
void orc_verify_tuples(const void* h, const int32_t* codes, int64_t n, uint8_t* mask,
                       int64_t* index, int64_t* count) {
  const ItemSet* s = static_cast<const ItemSet*>(h);
  std::vector<uint64_t> mult;
  multipliers(s->L, s->radices.data(), mult);
  int64_t c = 0;
  for (int64_t i = 0; i < n; ++i) {
    uint64_t k;
    const bool in = pack_one(codes + i * s->L, s->L, s->radices.data(), mult, k) &&
                    s->keys.count(k) != 0;
    if (mask) mask[i] = in ? 1 : 0;
    if (in) {
      if (index) index[c] = i;
      ++c;
    }
  }
  if (count) *count = c;
}

// One level (1-based `level`) of the inference part of Alg. 3 for B requests.
// H [B,d] with h_row_stride floats between requests; W [(d+e),T_level]; E
// [T_level,e] (needed when state_out != NULL); state_in [B,K_in,e] or NULL
// (zeros); key_in/score_in [B,K_in] or NULL (0 / 0), a slot with key 2^64-1 is
// empty; set or NULL (no verification; consulted when its L equals `level`);
// U [e,e] with transition == 1, else ignored.  Outputs [B,K] (+ state_out
// [B,K,e], count_out [B]); slots beyond count hold key 2^64-1, score -inf,
// parent -1, code -1.  logp_out (optional) [B,K_in,T_level] doubles.
int orc_draft_level(int32_t B, int32_t L, int32_t level, int32_t K, int32_t K_in, int32_t d,
                    int32_t e, const int32_t* radices, const float* H, int64_t h_row_stride,
                    const float* W, const float* E, const float* state_in,
                    const uint64_t* key_in, const float* score_in, const void* set,
                    const float* U, int transition, int round_state_bf16, uint64_t* key_out,
                    float* score_out,
                    int32_t* parent_out, int32_t* code_out, float* state_out,
                    int32_t* count_out, double* logp_out, int threads) {
  std::vector<uint64_t> mult;
  if (level < 1 || level > L || K < 1 || K_in < 1 || B < 0) return -1;
  if (!multipliers(L, radices, mult)) return -4;
  if (state_out && !E) return -1;
  if (transition != 0 && transition != 1) return -1;
  if (state_out && transition == 1 && !U) return -1;
  const ItemSet* iset = static_cast<const ItemSet*>(set);
  if (iset) {
    if (iset->L != L && iset->L != level) return -1;
    for (int32_t l = 0; l < iset->L; ++l)
      if (iset->radices[l] != radices[l]) return -1;
  }
  LevelArgs a{B, L, level, K, K_in, d, e, radices, H, h_row_stride, W, E, state_in, key_in,
              score_in, iset, U, transition, round_state_bf16, key_out, score_out,
              parent_out, code_out, state_out, count_out, logp_out, mult[level - 1]};
  const int nt = std::max(1, std::min(threads, (int)B));
  if (nt == 1) {
    for (int32_t b = 0; b < B; ++b) level_one_request(a, b);
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t)
      pool.emplace_back([&a, t, nt, B]() {
        for (int32_t b = t; b < B; b += nt) level_one_request(a, b);
      });
    for (auto& th : pool) th.join();
  }
  return 0;
}

}  // extern "C"
