// Standalone driver for the CPU oracle under AddressSanitizer / UndefinedBehaviorSanitizer:
// includes the oracle's one translation unit and calls every exported function on small seeded
// inputs, among them the degenerate shapes (one token, budget equal to the sequence, no
// representatives, nothing important, units, protected ends with no middle, paged gather).
// Output buffers are sized exactly, so any access past an end aborts the run.  Exit status 0 and
// the last line "oracle sanitizer run ok" mean a clean pass.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../oracle/kvcrush_oracle.cpp"

namespace {
uint64_t rng_state = 0x1234567ull;
double uniform() {  // xorshift; only the shapes matter here
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 9007199254740992.0;
}
std::vector<float> random_floats(size_t n, bool positive) {
  std::vector<float> v(n);
  for (auto& x : v) x = positive ? (float)(0.01 + uniform()) : (float)(2.0 * uniform() - 1.0);
  return v;
}
int fails = 0;
void expect(bool ok, const char* what) {
  if (!ok) {
    std::printf("FAILED: %s\n", what);
    ++fails;
  }
}

void scores_case(int B, int Hq, int Hkv, int S, int D, int rg, int window) {
  const int Hs = rg ? Hkv : Hq;
  auto q = random_floats((size_t)B * Hq * S * D, false), k = random_floats((size_t)B * Hkv * S * D, false);
  std::vector<float> sc((size_t)B * Hs * S), lse((size_t)B * Hq * S);
  expect(kvcrush_oracle_scores(B, Hq, Hkv, S, D, 0, rg, window, 0.0, q.data(), k.data(), sc.data(), lse.data()) == 0,
         "scores");
  std::vector<double> c(S, 0.0), l(S, 0.0);
  expect(kvcrush_oracle_head_colsums(S, D, 0, q.data(), k.data(), 0, S, 0.0, c.data(), l.data()) == 0, "head_colsums");
}

void select_case(int B, int Hs, int S, int budget, int n_imp, int kbit, int sink, int recent, int anchor, int unit) {
  auto sc = random_floats((size_t)B * Hs * S, true);
  std::vector<int32_t> idx((size_t)B * budget);
  std::vector<uint8_t> kind((size_t)B * budget);
  const int W = (Hs + 63) / 64;
  if (unit > 1) {
    const int n_units = (S - sink - recent) / unit, Wu = (Hs * unit + 63) / 64;
    std::vector<uint64_t> ub((size_t)B * n_units * Wu + 1);
    expect(kvcrush_oracle_select_units(B, Hs, S, unit, budget, n_imp, kbit, sink, recent, anchor, 7, nullptr, sc.data(),
                                       idx.data(), kind.data(), ub.data()) == 0, "select_units");
  } else {
    std::vector<uint64_t> bits((size_t)B * S * W);
    expect(kvcrush_oracle_select_protected(B, Hs, S, budget, n_imp, kbit, sink, recent, anchor, 7, nullptr, sc.data(),
                                           idx.data(), kind.data(), bits.data()) == 0, "select_protected");
  }
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < budget; ++j) {
      const int t = idx[(size_t)b * budget + j];
      expect(t >= 0 && t < S && (j == 0 || t > idx[(size_t)b * budget + j - 1]), "indices ascending and in range");
    }
}
}  // namespace

int main() {
  scores_case(1, 1, 1, 1, 8, 0, 0);      // one token
  scores_case(2, 4, 2, 37, 16, 1, 0);    // ragged length, grouped
  scores_case(1, 2, 2, 20, 8, 0, 5);     // observation window
  scores_case(1, 2, 1, 9, 8, 1, 100);    // window longer than the sequence

  select_case(1, 4, 1, 1, 1, 0, 0, 0, 2, 1);        // one token kept
  select_case(1, 4, 1, 0, 0, 0, 0, 0, 2, 1);        // nothing kept
  select_case(2, 8, 100, 100, 30, 0, 0, 0, 1, 1);   // budget == S
  select_case(1, 8, 130, 40, 40, 0, 0, 0, 0, 1);    // no representatives
  select_case(1, 8, 130, 40, 0, 0, 0, 0, 1, 1);     // nothing important
  select_case(2, 70, 90, 30, 10, 60, 0, 0, 1, 1);   // two bit words, mean anchor with one-bits
  select_case(1, 8, 64, 64, 0, 0, 40, 24, 0, 1);    // protected ends, no middle
  select_case(1, 8, 200, 60, 20, 0, 7, 13, 2, 1);   // protected ends, ragged middle
  select_case(1, 3, 96, 48, 24, 0, 0, 0, 1, 8);     // units of 8 tokens
  select_case(1, 4, 104, 40, 16, 0, 4, 4, 0, 8);    // units between protected ends
  select_case(1, 32, 64, 32, 32, 0, 0, 0, 2, 32);   // 1024-bit vectors, no representatives

  {  // gathers: dense, paged, capacity-strided
    const int B = 2, Hkv = 3, S = 32, D = 8, budget = 5, bs = 16;
    auto k = random_floats((size_t)B * Hkv * S * D, false), v = random_floats((size_t)B * Hkv * S * D, false);
    std::vector<int32_t> idx = {0, 3, 17, 30, 31, 1, 2, 15, 16, 31};
    std::vector<float> ko((size_t)B * Hkv * budget * D), vo(ko.size());
    expect(kvcrush_oracle_compact(B, Hkv, S, D, 0, budget, k.data(), v.data(), idx.data(), nullptr, 0, ko.data(),
                                  vo.data()) == 0, "compact dense");
    std::vector<int32_t> bt = {3, 0, 1, 2};  // [B, S / bs] pool blocks
    expect(kvcrush_oracle_compact(B, Hkv, S, D, 0, budget, k.data(), v.data(), idx.data(), bt.data(), bs, ko.data(),
                                  vo.data()) == 0, "compact paged");
    const int Hs = 2, cap_dst = 6;
    auto sc = random_floats((size_t)B * Hs * S, true);
    std::vector<float> k2((size_t)B * Hkv * cap_dst * D), v2(k2.size()), s2((size_t)B * Hs * cap_dst);
    expect(kvcrush_oracle_compact_cache(B, Hkv, Hs, D, 0, S, cap_dst, budget, k.data(), v.data(), sc.data(), idx.data(),
                                        k2.data(), v2.data(), s2.data()) == 0, "compact_cache");
  }
  {  // decoding step, pooling, top-k, generator, bits, grouping
    const int B = 1, Hq = 4, Hkv = 2, S = 11, cap = 11, D = 8;
    auto qn = random_floats((size_t)B * Hq * D, false), kc = random_floats((size_t)B * Hkv * cap * D, false);
    auto sc = random_floats((size_t)B * Hkv * cap, true);
    expect(kvcrush_oracle_scores_append(B, Hq, Hkv, S, cap, D, 0, 1, 0.25, qn.data(), kc.data(), sc.data()) == 0, "append");
    expect(kvcrush_oracle_scores_append(B, Hq, Hkv, 1, cap, D, 0, 1, 0.0, qn.data(), kc.data(), sc.data()) == 0, "append S=1");
    auto in = random_floats(3 * 17, true);
    std::vector<float> out(in.size());
    expect(kvcrush_oracle_maxpool(3, 17, 5, in.data(), out.data()) == 0, "maxpool");
    expect(kvcrush_oracle_maxpool(3, 17, 33, in.data(), out.data()) == 0, "maxpool wider than the row");
    std::vector<int32_t> top(17);
    expect(kvcrush_oracle_topk(in.data(), 17, 17, top.data()) == 0 && kvcrush_oracle_topk(in.data(), 17, 0, top.data()) == 0,
           "topk");
    uint64_t words[3];
    kvcrush_oracle_splitmix64(0, 3, words);
    const int Hs = 5, St = 40;
    auto rows = random_floats((size_t)Hs * St, true);
    std::vector<uint64_t> bits(St);
    expect(kvcrush_oracle_bits(Hs, St, 13, rows.data(), bits.data()) == 0, "bits");
    std::vector<uint8_t> imp(St, 0);
    for (int t = 0; t < St; t += 4) imp[t] = 1;
    std::vector<int32_t> reps(7);
    uint64_t anchor = 0;
    expect(kvcrush_oracle_group(Hs, St, bits.data(), imp.data(), 7, 1, 3, 0, nullptr, reps.data(), &anchor) == 0, "group");
  }
  if (fails) return 1;
  std::printf("oracle sanitizer run ok\n");
  return 0;
}
