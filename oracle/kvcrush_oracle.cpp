// KVCrush oracle: a plain, slow, single-threaded CPU statement of the per-layer
// KV-cache compression step.  TEST INFRASTRUCTURE ONLY: it exists so that the
// GPU library can be checked against something written straight from the
// paper.  It shares no code with the GPU sources, is never linked into the
// product, and nothing on the product path may call it.
//
// What it follows (KVCrush, arXiv 2503.00022):
//   * Algorithm 1 + Sec. 3.1  -- per-head attention weights, a per-head
//     threshold keeping a target fraction of tokens, one bit per head.
//   * Algorithm 2 + Sec. 3.2  -- anchor vector, Hamming distance to it,
//     B_representative buckets, one representative nearest each bucket centroid.
//   * Sec. 3 (first paragraph) -- budget B = B_important + B_representative,
//     the important set chosen by the baseline (H2O: largest accumulated
//     attention, Sec. 2.3 and Sec. 4.1.1); final cache = union of both sets.
//
// Readings taken where the paper is silent or garbled (listed in the design
// notes too):
//   * The printed score of Alg. 1 sums a softmax row, which is 1 for every
//     token.  The H2O meaning is used instead: the attention a token RECEIVES,
//     c_h[t] = sum over queries i >= t of A_h(i, t), causal mask, no 1/S factor.
//   * theta_h is described as the cut that keeps a fixed share of the tokens
//     of each head: exact per-head top-k, ties resolved towards the lower index.
//   * Alg. 2 only says that the bucket of a token follows from d_t: tokens are
//     ordered by (d_t, token index) and cut into B_representative contiguous
//     rank ranges [floor(j*N/Br), floor((j+1)*N/Br)).
//   * Only tokens NOT kept as important are grouped (Sec. 3 presents the
//     representatives as stand-ins for what is evicted), so the two sets are
//     disjoint and the cache holds exactly B.
//   * Nearness to the bucket centroid is measured as L1 distance to the
//     fractional centroid times the bucket size, an integer:
//     sum_r (bit_r ? n - cnt_r : cnt_r).
//   * Every tie goes to the lower token index.  Output ascending by position.
//
// Beyond the five stages the same file states the variants the paper pairs the
// method with: scoring from an observation window of the last queries and max
// pooling of the scores (the SnapKV baseline as Sec. 2.3 / 4.1.1 summarise it),
// protected initial and recent tokens (Table 1's cache layout), chunk- / page-
// level selection (Sec. 4.3.4, 4.3.5), and the decoding-time steps (one more
// query row per generated token, eviction on capacity-strided caches).
//
// Parity pins (tests/test_oracle_*.py): brute force with the full SxS matrix,
// the harmonic closed form for uniform attention, column sums totalling the
// number of query rows, float64 library softmax, hand-worked Hamming/bucket
// examples (token and page level), splitmix64's published first outputs, an
// independent big-integer implementation of the whole selection (also on the
// middle between protected ends and on pages), library max pooling, the
// identity "prefix scored at once + one append per later token = the whole
// sequence scored at once", strided gathers against a library gather; and a
// mutation test that plants single mistakes in a copy of this file and checks
// that a named pin notices each.  Whether the retained tokens preserve model
// accuracy is "parity unpinned" (needs the paper's datasets and weights).
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
enum { ANCHOR_RANDOM = 0, ANCHOR_MEAN = 1, ANCHOR_ALTERNATING = 2, ANCHOR_EXPLICIT = 3 };

// bf16 is the upper 16 bits of an IEEE binary32; widening is exact.
double widen(const void* base, size_t i, int dtype) {
  if (dtype == ORC_F32) return (double)((const float*)base)[i];
  if (dtype == ORC_F16) {
    // IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits; exact in double.
    const uint16_t h = ((const uint16_t*)base)[i];
    const int e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0) v = std::ldexp((double)f, -24);                       // zero and subnormals
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = std::ldexp((double)(1024 + f), e - 25);
    return (h & 0x8000) ? -v : v;
  }
  uint32_t u = (uint32_t)((const uint16_t*)base)[i] << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return (double)f;
}

size_t elem_size(int dtype) { return dtype == ORC_F32 ? 4 : 2; }

int words_for(int Hs) { return (Hs + 63) / 64; }

// One splitmix64 step (public-domain generator by S. Vigna): advances the
// state by the golden-ratio increment and returns the mixed value.
uint64_t splitmix64_next(uint64_t* state) {
  *state += 0x9E3779B97F4A7C15ull;
  uint64_t z = *state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Indices of the k largest values, ties to the lower index: a full stable sort
// by descending value (stability keeps equal values in index order).
std::vector<int> topk_indices(const float* v, int n, int k) {
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [v](int a, int b) { return v[a] > v[b]; });
  order.resize(k);
  return order;
}

bool get_bit(const uint64_t* w, int r) { return (w[r / 64] >> (r % 64)) & 1ull; }

}  // namespace

extern "C" {

// Alg. 1 (attention weights) with the received-attention reading: for one
// head, adds to c[t] the probability that each query row i in
// [row_begin, row_end) puts on key t <= i.  q_head, k_head: [S, D] row-major.
// lse (nullable, [S]) receives log(sum_j exp(s_ij)) for the rows visited.
// c is accumulated into (caller zeroes it), so disjoint row ranges add up.
// scale: factor on the dot products; 0 means the usual 1 / sqrt(D) (heads stored with padding, or
// models with their own attention scale, pass theirs).
int kvcrush_oracle_head_colsums(int S, int D, int dtype, const void* q_head, const void* k_head,
                                int row_begin, int row_end, double scale, double* c, double* lse) {
  if (S < 1 || D < 1 || row_begin < 0 || row_end > S || row_begin > row_end) return 1;
  std::vector<double> kd((size_t)S * D), qrow(D), s(S), p(S);
  for (size_t i = 0; i < (size_t)S * D; ++i) kd[i] = widen(k_head, i, dtype);
  const double inv_sqrt_d = scale != 0.0 ? scale : 1.0 / std::sqrt((double)D);
  for (int i = row_begin; i < row_end; ++i) {
    for (int d = 0; d < D; ++d) qrow[d] = widen(q_head, (size_t)i * D + d, dtype);
    double m = -INFINITY;
    for (int j = 0; j <= i; ++j) {
      double dot = 0.0;
      const double* kr = &kd[(size_t)j * D];
      for (int d = 0; d < D; ++d) dot += qrow[d] * kr[d];
      s[j] = dot * inv_sqrt_d;
      if (s[j] > m) m = s[j];
    }
    double L = 0.0;
    for (int j = 0; j <= i; ++j) {
      p[j] = std::exp(s[j] - m);
      L += p[j];
    }
    for (int j = 0; j <= i; ++j) c[j] += p[j] / L;
    if (lse) lse[i] = m + std::log(L);
  }
  return 0;
}

// Whole score tensor.  q: [B,Hq,S,D], k: [B,Hkv,S,D]; query head h reads KV
// head h / (Hq/Hkv).  scores: [B,Hs,S] fp32 with Hs = Hkv when reduce_groups
// (the heads of a group are summed in double, ascending, and rounded once),
// else Hs = Hq.  lse_out (nullable): [B,Hq,S] fp32.
// obs_window = 0: every query row contributes.  obs_window = W > 0: only the last
// min(W, S) query rows do (SnapKV's observation window over the end of the
// prompt, as Sec. 2.3 summarises that baseline); lse_out rows before the
// window are left at zero.
int kvcrush_oracle_scores(int B, int Hq, int Hkv, int S, int D, int dtype, int reduce_groups,
                          int obs_window, double scale, const void* q, const void* k, float* scores,
                          float* lse_out) {
  if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 || D < 1 || obs_window < 0) return 1;
  const int row_begin = (obs_window == 0 || obs_window >= S) ? 0 : S - obs_window;
  const int G = Hq / Hkv;
  const size_t es = elem_size(dtype), head_elems = (size_t)S * D;
  std::vector<double> c(S), acc(S), lse(S);
  for (int b = 0; b < B; ++b) {
    for (int g = 0; g < Hkv; ++g) {
      std::fill(acc.begin(), acc.end(), 0.0);
      for (int hh = 0; hh < G; ++hh) {
        const int h = g * G + hh;
        std::fill(c.begin(), c.end(), 0.0);
        const char* qh = (const char*)q + ((size_t)b * Hq + h) * head_elems * es;
        const char* kh = (const char*)k + ((size_t)b * Hkv + g) * head_elems * es;
        std::fill(lse.begin(), lse.end(), 0.0);
        int rc = kvcrush_oracle_head_colsums(S, D, dtype, qh, kh, row_begin, S, scale, c.data(), lse.data());
        if (rc) return rc;
        if (lse_out)
          for (int t = 0; t < S; ++t) lse_out[((size_t)b * Hq + h) * S + t] = (float)lse[t];
        if (reduce_groups) {
          for (int t = 0; t < S; ++t) acc[t] += c[t];
        } else {
          for (int t = 0; t < S; ++t) scores[((size_t)b * Hq + h) * S + t] = (float)c[t];
        }
      }
      if (reduce_groups)
        for (int t = 0; t < S; ++t) scores[((size_t)b * Hkv + g) * S + t] = (float)acc[t];
    }
  }
  return 0;
}

// One decoding step (Sec. 1: the cache grows by one entry per generated token;
// the H2O importance keeps accumulating over decoding steps, Sec. 2.3).  The
// new token's query of every head attends to the S cached keys, its own (the
// last, position S-1) included; the probabilities are added to the running
// scores.  q_new: [B,Hq,D]; k: [B,Hkv,capacity,D] of which the first S tokens
// are valid; scores: [B,Hs,capacity], updated in place for t < S-1, position
// S-1 (the new token, which had no score yet) is overwritten; entries at or
// beyond S are not touched.  With reduce_groups the probabilities of a
// group's heads are summed in double, heads ascending, before the single
// rounding to float of old + sum.
int kvcrush_oracle_scores_append(int B, int Hq, int Hkv, int S, int capacity, int D, int dtype,
                                 int reduce_groups, double scale, const void* q_new, const void* k,
                                 float* scores) {
  if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 || capacity < S || D < 1) return 1;
  const int G = Hq / Hkv, Hs = reduce_groups ? Hkv : Hq;
  const double inv_sqrt_d = scale != 0.0 ? scale : 1.0 / std::sqrt((double)D);
  std::vector<double> logit(S), add(S);
  for (int b = 0; b < B; ++b)
    for (int r = 0; r < Hs; ++r) {
      std::fill(add.begin(), add.end(), 0.0);
      const int h0 = reduce_groups ? r * G : r, h1 = reduce_groups ? h0 + G : h0 + 1;
      for (int h = h0; h < h1; ++h) {
        const int g = h / G;
        double m = -INFINITY;
        for (int j = 0; j < S; ++j) {
          double dot = 0.0;
          for (int d = 0; d < D; ++d)
            dot += widen(q_new, ((size_t)b * Hq + h) * D + d, dtype) *
                   widen(k, (((size_t)b * Hkv + g) * capacity + j) * D + d, dtype);
          logit[j] = dot * inv_sqrt_d;
          if (logit[j] > m) m = logit[j];
        }
        double L = 0.0;
        for (int j = 0; j < S; ++j) L += std::exp(logit[j] - m);
        for (int j = 0; j < S; ++j) add[j] += std::exp(logit[j] - m) / L;
      }
      float* row = scores + ((size_t)b * Hs + r) * capacity;
      for (int j = 0; j < S; ++j) row[j] = (float)((j == S - 1 ? 0.0 : (double)row[j]) + add[j]);
    }
  return 0;
}

// Eviction during decoding: the kept tokens of a capacity-strided cache and
// their running scores move to the front of another one.
// k, v: [B,Hkv,cap_src,D]; scores: [B,Hs,cap_src]; idx: [B,budget];
// k_out, v_out: [B,Hkv,cap_dst,D]; scores_out: [B,Hs,cap_dst].  Only the first
// `budget` tokens of every output row are written.
int kvcrush_oracle_compact_cache(int B, int Hkv, int Hs, int D, int dtype, int cap_src, int cap_dst,
                                 int budget, const void* k, const void* v, const float* scores,
                                 const int32_t* idx, void* k_out, void* v_out, float* scores_out) {
  if (B < 1 || Hkv < 1 || Hs < 1 || D < 1 || budget < 0 || budget > cap_src || budget > cap_dst)
    return 1;
  const size_t row = (size_t)D * elem_size(dtype);
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < budget; ++j) {
      const int t = idx[(size_t)b * budget + j];
      if (t < 0 || t >= cap_src) return 2;
      for (int h = 0; h < Hkv; ++h) {
        const size_t src = (((size_t)b * Hkv + h) * cap_src + t) * row;
        const size_t dst = (((size_t)b * Hkv + h) * cap_dst + j) * row;
        std::memcpy((char*)k_out + dst, (const char*)k + src, row);
        std::memcpy((char*)v_out + dst, (const char*)v + src, row);
      }
      for (int r = 0; r < Hs; ++r)
        scores_out[((size_t)b * Hs + r) * cap_dst + j] = scores[((size_t)b * Hs + r) * cap_src + t];
    }
  return 0;
}

// 1-D max pooling along the token axis, window `kernel` (odd), centred, the
// sequence ends padded with -inf (the pooling step by which SnapKV also keeps
// the neighbours of strong tokens, Sec. 2.3 / 4.1.1).  in, out: [rows, S].
int kvcrush_oracle_maxpool(int rows, int S, int kernel, const float* in, float* out) {
  if (rows < 0 || S < 1 || kernel < 1 || kernel % 2 == 0) return 1;
  const int half = kernel / 2;
  for (int r = 0; r < rows; ++r)
    for (int t = 0; t < S; ++t) {
      float best = -INFINITY;
      for (int u = t - half; u <= t + half; ++u)
        if (u >= 0 && u < S && in[(size_t)r * S + u] > best) best = in[(size_t)r * S + u];
      out[(size_t)r * S + t] = best;
    }
  return 0;
}

// The k largest of v[0..n), ties to the lower index, in rank order.
int kvcrush_oracle_topk(const float* v, int n, int k, int32_t* out) {
  if (n < 0 || k < 0 || k > n) return 1;
  std::vector<int> sel = topk_indices(v, n, k);
  for (int i = 0; i < k; ++i) out[i] = sel[i];
  return 0;
}

// First `count` outputs of splitmix64 started at `seed`.
void kvcrush_oracle_splitmix64(uint64_t seed, int count, uint64_t* out) {
  uint64_t st = seed;
  for (int i = 0; i < count; ++i) out[i] = splitmix64_next(&st);
}

// Alg. 1's thresholding for one sequence: bit r of token t is set iff t is in
// the top-kbit of score row r.  scores: [Hs,S]; bits: [S,W] (W = ceil(Hs/64)),
// head r -> bit r%64 of word r/64.
int kvcrush_oracle_bits(int Hs, int S, int kbit, const float* scores, uint64_t* bits) {
  if (Hs < 1 || S < 1 || kbit < 0 || kbit > S) return 1;
  const int W = words_for(Hs);
  std::memset(bits, 0, sizeof(uint64_t) * (size_t)S * W);
  for (int r = 0; r < Hs; ++r) {
    std::vector<int> sel = topk_indices(scores + (size_t)r * S, S, kbit);
    for (int t : sel) bits[(size_t)t * W + r / 64] |= 1ull << (r % 64);
  }
  return 0;
}

// Alg. 2 for one sequence.  bits: [S,W]; is_important: [S] flags (those tokens
// are left out of the grouping); Br buckets; anchor per `mode` (batch_index
// enters the random anchor's seed; anchor_explicit: [W], EXPLICIT only).
// reps: [Br] token ids in bucket order.  anchor_out (nullable): [W].
int kvcrush_oracle_group(int Hs, int S, const uint64_t* bits, const uint8_t* is_important, int Br,
                         int mode, uint64_t anchor_seed, int batch_index,
                         const uint64_t* anchor_explicit, int32_t* reps, uint64_t* anchor_out) {
  if (Hs < 1 || S < 1 || Br < 0) return 1;
  const int W = words_for(Hs);
  std::vector<int> disc;  // discarded tokens, ascending
  for (int t = 0; t < S; ++t)
    if (!is_important[t]) disc.push_back(t);
  const long long N = (long long)disc.size();
  if (Br > N) return 1;

  // anchor
  std::vector<uint64_t> a(W, 0);
  if (mode == ANCHOR_RANDOM) {
    uint64_t st = anchor_seed + (uint64_t)batch_index;
    for (int w = 0; w < W; ++w) a[w] = splitmix64_next(&st);
  } else if (mode == ANCHOR_ALTERNATING) {
    for (int r = 0; r < Hs; ++r)
      if (r & 1) a[r / 64] |= 1ull << (r % 64);
  } else if (mode == ANCHOR_MEAN) {
    for (int r = 0; r < Hs; ++r) {
      long long cnt = 0;
      for (int t : disc) cnt += get_bit(bits + (size_t)t * W, r) ? 1 : 0;
      if (2 * cnt > N) a[r / 64] |= 1ull << (r % 64);
    }
  } else if (mode == ANCHOR_EXPLICIT) {
    if (!anchor_explicit) return 1;
    for (int w = 0; w < W; ++w) a[w] = anchor_explicit[w];
  } else {
    return 1;
  }
  // keep only the Hs meaningful bits
  for (int r = Hs; r < W * 64; ++r) a[r / 64] &= ~(1ull << (r % 64));
  if (anchor_out)
    for (int w = 0; w < W; ++w) anchor_out[w] = a[w];
  if (Br == 0) return 0;

  // Hamming distance of every grouped token to the anchor, bit by bit.
  std::vector<int> dist(S, 0);
  for (int t : disc) {
    int d = 0;
    for (int r = 0; r < Hs; ++r)
      d += (get_bit(bits + (size_t)t * W, r) != get_bit(a.data(), r)) ? 1 : 0;
    dist[t] = d;
  }
  // order by distance; equal distances stay in token order
  std::vector<int> order = disc;
  std::stable_sort(order.begin(), order.end(), [&dist](int x, int y) { return dist[x] < dist[y]; });

  for (long long j = 0; j < Br; ++j) {
    const long long lo = j * N / Br, hi = (j + 1) * N / Br;
    const long long n = hi - lo;
    std::vector<long long> cnt(Hs, 0);
    for (long long m = lo; m < hi; ++m)
      for (int r = 0; r < Hs; ++r) cnt[r] += get_bit(bits + (size_t)order[m] * W, r) ? 1 : 0;
    long long best_cost = -1;
    int best_t = -1;
    for (long long m = lo; m < hi; ++m) {
      const int t = order[m];
      long long cost = 0;
      for (int r = 0; r < Hs; ++r) cost += get_bit(bits + (size_t)t * W, r) ? (n - cnt[r]) : cnt[r];
      if (best_t < 0 || cost < best_cost || (cost == best_cost && t < best_t)) {
        best_cost = cost;
        best_t = t;
      }
    }
    reps[j] = best_t;
  }
  return 0;
}

// Stages 2-4 for a batch, with protected ends (the cache layout of the paper's
// lm-eval-harness runs, Table 1: initial tokens + compressed middle + recent
// tokens).  scores: [B,Hs,S] fp32.  The first n_sink and the last n_recent
// tokens are always kept; the middle tokens [n_sink, S - n_recent) are
// compressed to budget - n_sink - n_recent tokens exactly as a sequence of their
// own would be: per-row top-bit_topk (0 = the middle's budget), importance
// top-n_important, grouping of the rest (Alg. 1, Alg. 2).
// Outputs: idx [B,budget] ascending token ids; kind (nullable) [B,budget]:
// 0 = kept as important, 1 = kept as representative, 2 = protected; bits
// (nullable) [B,S,W], zero for protected tokens.
// Token importance is the fp32 sum of the Hs rows taken in row order.
int kvcrush_oracle_select_protected(int B, int Hs, int S, int budget, int n_important,
                                    int bit_topk, int n_sink, int n_recent, int anchor_mode,
                                    uint64_t anchor_seed, const uint64_t* anchor_bits,
                                    const float* scores, int32_t* idx, uint8_t* kind,
                                    uint64_t* bits_out) {
  if (B < 1 || Hs < 1 || S < 1 || budget < 0 || budget > S || n_sink < 0 || n_recent < 0 ||
      n_sink + n_recent > budget)
    return 1;
  const int Sm = S - n_sink - n_recent;        // middle tokens
  const int Bm = budget - n_sink - n_recent;   // their budget
  if (n_important < 0 || n_important > Bm) return 1;
  const int kbit = bit_topk == 0 ? Bm : bit_topk;
  if (kbit < 0 || kbit > Sm) return 1;
  const int W = words_for(Hs), Br = Bm - n_important;
  std::vector<float> mid((size_t)Hs * (Sm > 0 ? Sm : 1));
  std::vector<uint64_t> bits((size_t)(Sm > 0 ? Sm : 1) * W);
  std::vector<float> imp(Sm > 0 ? Sm : 1);
  std::vector<uint8_t> is_imp(Sm > 0 ? Sm : 1), is_rep(Sm > 0 ? Sm : 1);
  std::vector<int32_t> reps(Br > 0 ? Br : 1);
  for (int b = 0; b < B; ++b) {
    const float* sc = scores + (size_t)b * Hs * S;
    std::fill(is_imp.begin(), is_imp.end(), 0);
    std::fill(is_rep.begin(), is_rep.end(), 0);
    if (Sm > 0) {
      for (int r = 0; r < Hs; ++r)
        for (int u = 0; u < Sm; ++u) mid[(size_t)r * Sm + u] = sc[(size_t)r * S + n_sink + u];
      int rc = kvcrush_oracle_bits(Hs, Sm, kbit, mid.data(), bits.data());
      if (rc) return rc;
      for (int u = 0; u < Sm; ++u) {
        float acc = 0.0f;
        for (int r = 0; r < Hs; ++r) acc = acc + mid[(size_t)r * Sm + u];
        imp[u] = acc;
      }
      for (int u : topk_indices(imp.data(), Sm, n_important)) is_imp[u] = 1;
      rc = kvcrush_oracle_group(Hs, Sm, bits.data(), is_imp.data(), Br, anchor_mode, anchor_seed, b,
                                anchor_bits ? anchor_bits + (size_t)b * W : nullptr, reps.data(),
                                nullptr);
      if (rc) return rc;
      for (int j = 0; j < Br; ++j) {
        if (is_imp[reps[j]] || is_rep[reps[j]]) return 2;  // must be disjoint and distinct
        is_rep[reps[j]] = 1;
      }
    }
    int o = 0;
    for (int t = 0; t < S; ++t) {
      const bool prot = t < n_sink || t >= S - n_recent;
      const int u = t - n_sink;
      if (prot || is_imp[u] || is_rep[u]) {
        if (o >= budget) return 2;
        idx[(size_t)b * budget + o] = t;
        if (kind) kind[(size_t)b * budget + o] = prot ? 2 : (is_rep[u] ? 1 : 0);
        ++o;
      }
    }
    if (o != budget) return 2;
    if (bits_out) {
      uint64_t* dst = bits_out + (size_t)b * S * W;
      std::fill(dst, dst + (size_t)S * W, 0ull);
      if (Sm > 0) std::memcpy(dst + (size_t)n_sink * W, bits.data(), sizeof(uint64_t) * Sm * W);
    }
  }
  return 0;
}

// Chunk- / page-level KVCrush (Sec. 4.3.4: baselines that work on chunks;
// Sec. 4.3.5: paged caches).  The unit of selection is a run of `unit`
// consecutive tokens.  As that section describes the paged variant:
//   * a unit's importance is the baseline's token importance added up over the
//     unit's tokens (here: fp32, tokens ascending, each token's importance being
//     the fp32 sum of the score rows in row order);
//   * a unit's binary vector is the concatenation of the head vectors of its
//     tokens: bit j*Hs + r of the unit is bit r of its j-th token, the token
//     bits being those of Alg. 1 (per-row top-bit_topk over TOKENS);
//   * Alg. 2 then runs on units: anchor of unit*Hs bits, Hamming distance,
//     buckets, one representative unit per bucket.
// budget, n_important, n_sink, n_recent count tokens; budget - n_sink - n_recent,
// n_important and the middle's length must be multiples of `unit`.
// idx, kind: [B,budget] tokens (every token of a kept unit, ascending).
// unit_bits_out (nullable): [B, Nu, Wu] with Nu = middle / unit units and
// Wu = ceil(unit*Hs / 64) words each.
int kvcrush_oracle_select_units(int B, int Hs, int S, int unit, int budget, int n_important,
                                int bit_topk, int n_sink, int n_recent, int anchor_mode,
                                uint64_t anchor_seed, const uint64_t* anchor_bits,
                                const float* scores, int32_t* idx, uint8_t* kind,
                                uint64_t* unit_bits_out) {
  if (B < 1 || Hs < 1 || S < 1 || unit < 1 || budget < 0 || budget > S || n_sink < 0 ||
      n_recent < 0 || n_sink + n_recent > budget)
    return 1;
  const int Sm = S - n_sink - n_recent, Bm = budget - n_sink - n_recent;
  if (Sm % unit != 0 || Bm % unit != 0 || n_important < 0 || n_important > Bm ||
      n_important % unit != 0)
    return 1;
  const int kbit = bit_topk == 0 ? Bm : bit_topk;
  if (kbit < 0 || kbit > Sm) return 1;
  const int Nu = Sm / unit, Bu = Bm / unit, Iu = n_important / unit, Ru = Bu - Iu;
  const int W = words_for(Hs), Hu = Hs * unit, Wu = words_for(Hu);
  const size_t one = 1;
  std::vector<float> mid((size_t)Hs * std::max(Sm, 1)), tok_imp(std::max(Sm, 1)), unit_imp(std::max(Nu, 1));
  std::vector<uint64_t> tok_bits(std::max((size_t)Sm * W, one)), unit_bits(std::max((size_t)Nu * Wu, one));
  std::vector<uint8_t> is_imp(std::max(Nu, 1)), is_rep(std::max(Nu, 1));
  std::vector<int32_t> reps(std::max(Ru, 1));
  for (int b = 0; b < B; ++b) {
    const float* sc = scores + (size_t)b * Hs * S;
    std::fill(is_imp.begin(), is_imp.end(), 0);
    std::fill(is_rep.begin(), is_rep.end(), 0);
    if (Nu > 0) {
      for (int r = 0; r < Hs; ++r)
        for (int t = 0; t < Sm; ++t) mid[(size_t)r * Sm + t] = sc[(size_t)r * S + n_sink + t];
      int rc = kvcrush_oracle_bits(Hs, Sm, kbit, mid.data(), tok_bits.data());
      if (rc) return rc;
      for (int t = 0; t < Sm; ++t) {
        float acc = 0.0f;
        for (int r = 0; r < Hs; ++r) acc = acc + mid[(size_t)r * Sm + t];
        tok_imp[t] = acc;
      }
      std::fill(unit_bits.begin(), unit_bits.end(), 0ull);
      for (int u = 0; u < Nu; ++u) {
        float acc = 0.0f;
        for (int j = 0; j < unit; ++j) {
          const int t = u * unit + j;
          acc = acc + tok_imp[t];
          for (int r = 0; r < Hs; ++r)
            if (get_bit(tok_bits.data() + (size_t)t * W, r)) {
              const int pos = j * Hs + r;
              unit_bits[(size_t)u * Wu + pos / 64] |= 1ull << (pos % 64);
            }
        }
        unit_imp[u] = acc;
      }
      for (int u : topk_indices(unit_imp.data(), Nu, Iu)) is_imp[u] = 1;
      rc = kvcrush_oracle_group(Hu, Nu, unit_bits.data(), is_imp.data(), Ru, anchor_mode, anchor_seed,
                                b, anchor_bits ? anchor_bits + (size_t)b * Wu : nullptr, reps.data(),
                                nullptr);
      if (rc) return rc;
      for (int j = 0; j < Ru; ++j) {
        if (is_imp[reps[j]] || is_rep[reps[j]]) return 2;
        is_rep[reps[j]] = 1;
      }
    }
    int o = 0;
    for (int t = 0; t < S; ++t) {
      const bool prot = t < n_sink || t >= S - n_recent;
      const int u = prot ? 0 : (t - n_sink) / unit;
      if (prot || is_imp[u] || is_rep[u]) {
        if (o >= budget) return 2;
        idx[(size_t)b * budget + o] = t;
        if (kind) kind[(size_t)b * budget + o] = prot ? 2 : (is_rep[u] ? 1 : 0);
        ++o;
      }
    }
    if (o != budget) return 2;
    if (unit_bits_out && Nu > 0)
      std::memcpy(unit_bits_out + (size_t)b * Nu * Wu, unit_bits.data(), sizeof(uint64_t) * Nu * Wu);
  }
  return 0;
}

// Stages 2-4 for a batch without protected tokens.
int kvcrush_oracle_select(int B, int Hs, int S, int budget, int n_important, int bit_topk,
                          int anchor_mode, uint64_t anchor_seed, const uint64_t* anchor_bits,
                          const float* scores, int32_t* idx, uint8_t* kind, uint64_t* bits_out) {
  return kvcrush_oracle_select_protected(B, Hs, S, budget, n_important, bit_topk, 0, 0, anchor_mode,
                                         anchor_seed, anchor_bits, scores, idx, kind, bits_out);
}

// Stage 5.  Dense source: k, v [B,Hkv,S,D].  Paged source (block_table
// non-null): pool [n_blocks, block_size, Hkv, D], block_table [B, S/block_size]
// gives the physical block of each logical block.  Output [B,Hkv,budget,D].
int kvcrush_oracle_compact(int B, int Hkv, int S, int D, int dtype, int budget, const void* k,
                           const void* v, const int32_t* idx, const int32_t* block_table,
                           int block_size, void* k_out, void* v_out) {
  if (B < 1 || Hkv < 1 || S < 1 || D < 1 || budget < 0 || budget > S) return 1;
  if (block_table && (block_size < 1 || S % block_size != 0)) return 1;
  const size_t row = (size_t)D * elem_size(dtype);
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hkv; ++h)
      for (int j = 0; j < budget; ++j) {
        const int t = idx[(size_t)b * budget + j];
        if (t < 0 || t >= S) return 1;
        size_t src;
        if (block_table) {
          const size_t blk = (size_t)block_table[(size_t)b * (S / block_size) + t / block_size];
          src = ((blk * block_size + t % block_size) * Hkv + h) * row;
        } else {
          src = (((size_t)b * Hkv + h) * S + t) * row;
        }
        const size_t dst = (((size_t)b * Hkv + h) * budget + j) * row;
        std::memcpy((char*)k_out + dst, (const char*)k + src, row);
        std::memcpy((char*)v_out + dst, (const char*)v + src, row);
      }
  return 0;
}

}  // extern "C"
