// Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the CPU oracle: it runs
// every exported function of oracle/nezha_oracle.cpp on small inputs, edge cases included (K above
// the number of codes, an empty batch, out-of-range codes, duplicates, several threads), checks a
// few facts that must hold, and leaves the memory and arithmetic checking to the sanitizers.
// Exit status 0 = clean.  Built and run by tests/test_sanitizers.py.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
int orc_pack(const int32_t*, int64_t, int32_t, const int32_t*, uint64_t*, uint8_t*);
int orc_unpack(const uint64_t*, int64_t, int32_t, const int32_t*, int32_t*);
void* orc_set_new(const int32_t*, int64_t, int32_t, const int32_t*, int*);
int64_t orc_set_size(const void*);
void orc_set_free(void*);
void orc_set_contains_keys(const void*, const uint64_t*, int64_t, uint8_t*);
void orc_verify_tuples(const void*, const int32_t*, int64_t, uint8_t*, int64_t*, int64_t*);
int orc_draft_level(int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, const int32_t*,
                    const float*, int64_t, const float*, const float*, const float*,
                    const uint64_t*, const float*, const void*, const float*, int, int, uint64_t*,
                    float*, int32_t*, int32_t*, float*, int32_t*, double*, int);
}

#define REQUIRE(cond)                                                      \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #cond); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static uint32_t rng_state = 12345u;
static float rnd() {  // small deterministic generator, values in [-1, 1)
  rng_state = rng_state * 1664525u + 1013904223u;
  return (float)((rng_state >> 8) & 0xFFFF) / 32768.0f - 1.0f;
}

int main() {
  // Eq. 4 on the printed example, its inverse, an out-of-range code, a radix product that overflows
  {
    const int32_t rad[3] = {512, 512, 512};
    const int32_t t[6] = {243, 129, 3, 512, 0, 0};
    uint64_t keys[2];
    uint8_t ok[2];
    REQUIRE(orc_pack(t, 2, 3, rad, keys, ok) == 0);
    REQUIRE(keys[0] == 852723ull && ok[0] == 1 && ok[1] == 0 && keys[1] == ~0ull);
    int32_t back[3];
    REQUIRE(orc_unpack(keys, 1, 3, rad, back) == 0);
    REQUIRE(back[0] == 243 && back[1] == 129 && back[2] == 3);
    const int32_t big[3] = {1 << 30, 1 << 30, 1 << 30};
    REQUIRE(orc_pack(t, 1, 3, big, keys, ok) == -4);
    const int32_t edge[2] = {65536, 65536};          // 2^32 tuples: the largest key is 2^32 - 1
    const int32_t last[2] = {65535, 65535};
    REQUIRE(orc_pack(last, 1, 2, edge, keys, nullptr) == 0 && keys[0] == 0xFFFFFFFFull);
  }
  // the set: duplicates, membership, verification with a bad tuple, refusal of a bad catalog
  const int32_t rad[3] = {6, 6, 6};
  std::vector<int32_t> cat;
  for (int i = 0; i < 60; ++i) {
    cat.push_back(i % 6);
    cat.push_back((i / 6) % 6);
    cat.push_back((i * 7) % 6);
  }
  for (int i = 0; i < 9; ++i) cat.push_back(cat[i]);  // three duplicates
  int err = 1;
  void* set = orc_set_new(cat.data(), 63, 3, rad, &err);
  REQUIRE(set && err == 0 && orc_set_size(set) <= 60 && orc_set_size(set) > 0);
  {
    const int32_t q[12] = {0, 0, 0, 5, 5, 5, 6, 0, 0, -1, 2, 2};
    uint8_t mask[4];
    int64_t index[4], count = -1;
    orc_verify_tuples(set, q, 4, mask, index, &count);
    REQUIRE(mask[0] == 1 && mask[2] == 0 && mask[3] == 0 && count >= 1 && index[0] == 0);
    orc_verify_tuples(set, q, 0, nullptr, nullptr, &count);
    REQUIRE(count == 0);
    const uint64_t keys[2] = {0, ~0ull};
    orc_set_contains_keys(set, keys, 2, mask);
    REQUIRE(mask[0] == 1 && mask[1] == 0);
    const int32_t bad[3] = {0, 6, 0};
    REQUIRE(orc_set_new(bad, 1, 3, rad, &err) == nullptr && err == -4);
  }
  // the level loop: B = 3 requests, d = 5, e = 4, K = 4, then K above the number of codes, with
  // both Transitions, on one and on several threads
  const int B = 3, d = 5, e = 4, V = 6, L = 3;
  std::vector<float> H(B * L * d), W(L * (d + e) * V), E(L * V * e), U(e * e);
  for (auto& v : H) v = rnd();
  for (auto& v : W) v = rnd();
  for (auto& v : E) v = 0.5f * rnd();
  for (auto& v : U) v = 0.5f * rnd();
  for (int K : {4, 9}) {
    for (int transition : {0, 1}) {
      for (int threads : {1, 4}) {
        std::vector<uint64_t> key(B * K), key_in;
        std::vector<float> score(B * K), score_in, state(B * K * e), state_in;
        std::vector<int32_t> parent(B * K), code(B * K), count(B);
        std::vector<double> logp;
        int K_in = 1;
        for (int level = 1; level <= L; ++level) {
          logp.assign((size_t)B * K_in * V, 0.0);
          const int rc = orc_draft_level(
              B, L, level, K, K_in, d, e, rad, H.data() + (level - 1) * d, (int64_t)L * d,
              W.data() + (level - 1) * (d + e) * V, E.data() + (level - 1) * V * e,
              level > 1 ? state_in.data() : nullptr, level > 1 ? key_in.data() : nullptr,
              level > 1 ? score_in.data() : nullptr, set, U.data(), transition, /*bf16*/ level & 1,
              key.data(), score.data(), parent.data(), code.data(),
              level < L ? state.data() : nullptr, count.data(), logp.data(), threads);
          REQUIRE(rc == 0);
          for (int b = 0; b < B; ++b) {
            REQUIRE(count[b] >= 0 && count[b] <= K);
            for (int k = 1; k < count[b]; ++k) REQUIRE(score[b * K + k] <= score[b * K + k - 1]);
            for (int k = count[b]; k < K; ++k) REQUIRE(key[b * K + k] == ~0ull && code[b * K + k] == -1);
            for (int r = 0; r < K_in; ++r) {             // probabilities of a live beam sum to 1
              double s = 0;
              for (int v = 0; v < V; ++v) s += std::exp(logp[((size_t)b * K_in + r) * V + v]);
              if (level == 1 || key_in[b * K_in + r] != ~0ull) REQUIRE(std::fabs(s - 1.0) < 1e-9);
            }
          }
          key_in = key;
          score_in = score;
          state_in = state;
          K_in = K;
        }
      }
    }
  }
  // an empty batch, and argument errors
  {
    uint64_t key[4];
    float score[4];
    int32_t parent[4], code[4], count[1];
    REQUIRE(orc_draft_level(0, L, 1, 4, 1, d, e, rad, H.data(), d, W.data(), E.data(), nullptr,
                            nullptr, nullptr, nullptr, nullptr, 0, 0, key, score, parent, code,
                            nullptr, count, nullptr, 2) == 0);
    REQUIRE(orc_draft_level(1, L, 4, 4, 1, d, e, rad, H.data(), d, W.data(), E.data(), nullptr,
                            nullptr, nullptr, nullptr, nullptr, 0, 0, key, score, parent, code,
                            nullptr, count, nullptr, 1) == -1);
  }
  orc_set_free(set);
  std::puts("oracle: clean");
  return 0;
}
