// CPU oracle for the Residual Gradient Compression (RGC) hot path.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
// correct implementation used only by tests, the smoke check and the
// cpu_baseline leg of the benchmark.  It shares no code, header, table or
// helper with the HIP library and must never be called from the product path.
//
// What it computes (RedSync paper, Algorithm 1, inner loop over layers):
//   V_j += G_j                      (residual accumulate)
//   Masks = select(V_j, D)          (communication-set = top-k by magnitude,
//                                    Section 2.1, first paragraph: the largest
//                                    0.1 % of every layer's elements)
//   message = compress(V_j . Masks) (k indices + k values + a length element,
//                                    Section 2.2 first sentence, Section 2.3)
//   V_j = V_j . (1 - Masks)         (sent entries leave the residual)
// and the decompression of Section 2.3 (sparse array added into a dense array,
// message after message), followed by one scaling.
//
// The paper's own fast selection schemes (Algorithms 2 and 3) are NOT what is
// implemented here: Algorithm 2 plus its radixSelect step yields exactly the
// top-k set (Section 2.1: the compression ratio stays at exactly 0.1 % with it),
// so the oracle is that definition written out with a full sort.
//
// Readings taken where the paper is silent:
//   * k = max(1, ceil(n * ppm / 1e6)) in integer arithmetic.
//   * magnitude order = order of the IEEE-754 bit pattern with the sign bit
//     cleared (monotone in |x| for every non-NaN float; NaN sorts above Inf).
//   * ties in magnitude: the lowest index wins.
//   * the message lists indices ascending; values are the accumulated, signed
//     residual entries; masked residual entries become +0.0f bits.
//   * momentum-corrected variant (named in Section 2.5, formulas from DGC):
//       u = fma(m, u, g)   (one rounding)
//       a = V + u
//     and the sent entries are cleared from u as well (momentum masking).
//   * Nesterov form of the momentum correction (Section 2.5 names it for
//     Nesterov momentum SGD and defers to DGC, whose rule is
//     U <- m*(U + G), V <- V + U + G), every operation rounded on its own, the
//     additions taken from the left:
//       u = m * (u + g)
//       a = (V + u) + g
//   * local gradient clipping (Section 2.4: every worker clips its own
//     gradients before they enter the residuals, and with N workers the
//     clipping threshold is divided by sqrt(N)): with the L2 norm taken over
//     all layers of the call (the squares, exact in fp64, summed without
//     rounding and the sum rounded to fp64 once),
//       c = norm > t ? t / norm : 1,   t = max_norm / sqrt(N)   (fp64, then
//     rounded to fp32 once), and every gradient element enters the
//     accumulate as fl(c * g).
//   * Alternating Signs Quantization (Section 2.2, "Quantization of Sparsified
//     Residuals"): in one iteration the communication-set is the k largest
//     elements of the layer, in the next the k smallest, and one average is
//     sent in place of the k values.  "Largest" and "smallest" are taken as
//     they read: by value, sign included (the paper expects the k largest to
//     be positive; a layer with fewer than k positive elements goes on with
//     its zeros and then its negative elements closest to zero), equal values
//     to the lowest index as everywhere, +0 and -0 being equal values; NaNs
//     rank by their bit pattern like the other keys here (sign bit clear: above
//     +Inf, set: below -Inf).  The message lists the k indices ascending
//     and the mean of the k accumulated values: their sum without rounding,
//     rounded to fp64 once, divided by k in fp64 and rounded to fp32; the sent
//     entries leave the residual (and the velocity) exactly as in Algorithm 1.
//     Decompression adds the message's one value at each of its indices.
//   * threshold binary search selection (Section 2.1, Algorithm 3): the
//     communication-set is every element whose magnitude exceeds a threshold,
//     and the threshold is found by bisection so that more than k and fewer
//     than 2k elements pass.  The thresholds tried lie between the mean and the
//     maximum of |a|: threshold = mean + ratio * (max - mean) with ratio the
//     midpoint of an interval that starts as [0, 1]; a count of at most k moves
//     the interval's upper end to the midpoint (the threshold must come down), a
//     count of 2k or more moves its lower end there, a count in between ends
//     the search, and so does an interval no wider than eps.
//     Readings: the printed listing tests "nnz < k/2" in its second branch,
//     which would push the threshold up while too few elements pass and
//     contradicts the section's text (the threshold is to end between the k-th
//     and the 2k-th largest element): read as just described.  eps is not
//     given: 2^-10, i.e. at most ten counts.  Precision is not given: mean =
//     the sum of |a| without rounding, rounded to fp64 once, divided by n in
//     fp64 and rounded to fp32; the midpoint, max - mean, the product and the
//     sum in fp32, each operation rounded on its own.  A search that ends on the interval width
//     uses the last threshold tried.  The message is as long as it comes out;
//     a message buffer of `cap` entries takes the first cap elements in index
//     order and the others stay in the residual.  The sampled variant of the
//     same section reuses a threshold found earlier: the search is skipped and
//     the given threshold is applied.  Inputs must be finite.
//   * the three long sums (squares of the gradients, the k values of a one-value
//     message, |a| over a layer): the paper fixes neither their precision nor
//     the order of their additions, and a sum that depends on the order is one
//     that only a single schedule can reproduce.  They are therefore read as
//     the sum of the terms itself, rounded once to fp64 (nearest, ties to
//     even): whatever the order and the grouping, every correct implementation
//     arrives at the same bits.  A NaN term, or infinite terms of both signs,
//     give NaN; infinite terms of one sign give that infinity.
//   * decompression: acc starts at +0, workers are added in order 0..N-1 and
//     entries in message order, all in fp32; then either dense = acc*scale or
//     dense = dense + acc*scale (two roundings, no fused multiply-add).
//
// Build: g++ -std=c++17 -O2 -ffp-contract=off -fPIC -shared
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <utility>
#include <vector>

namespace {

inline uint32_t float_bits(float x) {
  uint32_t b;
  std::memcpy(&b, &x, sizeof b);
  return b;
}

// Monotone unsigned image of |x|.
inline uint32_t magnitude_key(float x) { return float_bits(x) & 0x7FFFFFFFu; }

// The sum of any number of doubles with one rounding at its end: the terms are
// added as integers (in units of 2^-1074, the smallest step of the format), the
// positive ones into one long integer and the magnitudes of the negative ones
// into another; the difference of the two is rounded to the nearest double,
// a tie to the one with an even last bit.  A NaN among the terms, or infinities
// of both signs, give NaN; infinities of one sign give that infinity.
class ExactSum {
 public:
  void add(double x) {
    if (std::isnan(x)) { nan_ = true; return; }
    if (std::isinf(x)) { (x > 0 ? pinf_ : ninf_) = true; return; }
    if (x == 0.0) return;
    int e;
    const double f = std::frexp(std::fabs(x), &e);              // |x| = f * 2^e, f in [1/2, 1)
    uint64_t mant = static_cast<uint64_t>(std::ldexp(f, 53));   // |x| = mant * 2^(e - 53)
    int pos = e - 53 + 1074;                                    // position of mant's last bit
    if (pos < 0) { mant >>= -pos; pos = 0; }                    // subnormal: the bits shifted out are zeros
    uint32_t* w = x > 0 ? pos_ : neg_;
    unsigned __int128 t = static_cast<unsigned __int128>(mant) << (pos % 32);
    uint64_t carry = 0;
    for (int i = pos / 32; i < kWords && (t != 0 || carry != 0); ++i) {
      const uint64_t v = static_cast<uint64_t>(w[i]) + static_cast<uint32_t>(t) + carry;
      w[i] = static_cast<uint32_t>(v);
      carry = v >> 32;
      t >>= 32;
    }
  }

  double rounded() const {
    if (nan_ || (pinf_ && ninf_)) return std::nan("");
    if (pinf_) return HUGE_VAL;
    if (ninf_) return -HUGE_VAL;
    int cmp = 0;
    for (int i = kWords - 1; i >= 0 && cmp == 0; --i)
      if (pos_[i] != neg_[i]) cmp = pos_[i] > neg_[i] ? 1 : -1;
    if (cmp == 0) return 0.0;
    const uint32_t* big = cmp > 0 ? pos_ : neg_;
    const uint32_t* small = cmp > 0 ? neg_ : pos_;
    uint32_t d[kWords];
    int64_t borrow = 0;
    for (int i = 0; i < kWords; ++i) {
      int64_t v = static_cast<int64_t>(big[i]) - static_cast<int64_t>(small[i]) - borrow;
      borrow = v < 0 ? 1 : 0;
      if (v < 0) v += int64_t(1) << 32;
      d[i] = static_cast<uint32_t>(v);
    }
    auto bit = [&](int p) { return p < 0 ? 0u : (d[p / 32] >> (p % 32)) & 1u; };
    int top = kWords * 32 - 1;
    while (bit(top) == 0u) --top;                               // the difference is not zero
    const int last = top >= 53 ? top - 52 : 0;                  // last bit that is kept
    uint64_t mant = 0;
    for (int p = top; p >= last; --p) mant = (mant << 1) | bit(p);
    if (last > 0) {
      bool rest = false;                                        // anything below the first dropped bit
      for (int p = last - 2; p >= 0 && !rest; --p) rest = bit(p) != 0u;
      if (bit(last - 1) != 0u && (rest || (mant & 1u) != 0u)) ++mant;
    }
    const double r = std::ldexp(static_cast<double>(mant), last - 1074);
    return cmp > 0 ? r : -r;
  }

 private:
  static constexpr int kWords = 68;      // 2176 bits: the format's 2098 and room for 2^64 terms
  uint32_t pos_[kWords] = {};
  uint32_t neg_[kWords] = {};
  bool nan_ = false, pinf_ = false, ninf_ = false;
};

// Step 1 of the layer loop: produce the accumulated tensor a (and the updated
// velocity when momentum correction is on).  Writes a into `acc`.
// `scale` (may be NULL) is the clipping coefficient applied to every gradient
// element first; `nesterov` selects the Nesterov form of the correction.
void accumulate(const float* grad, const float* residual, float* momentum,
                int64_t n, float m, int nesterov, const float* scale, std::vector<float>& acc) {
  acc.resize(static_cast<size_t>(n));
  for (int64_t i = 0; i < n; ++i) {
    float g = grad[i];
    if (scale != nullptr) g = *scale * g;
    if (momentum == nullptr) {
      acc[i] = residual[i] + g;
    } else if (!nesterov) {
      float u = std::fmaf(m, momentum[i], g);
      momentum[i] = u;
      acc[i] = residual[i] + u;
    } else {
      float t = momentum[i] + g;
      float u = m * t;
      momentum[i] = u;
      float s = residual[i] + u;
      acc[i] = s + g;
    }
  }
}

// Emit the message and the masked residual from the selected index set
// (`sel`, any order).
void emit(const std::vector<float>& acc, std::vector<int32_t>& sel,
          float* residual, float* momentum, int mask_momentum, int64_t n,
          int32_t* out_idx, float* out_val, int32_t* out_count) {
  std::sort(sel.begin(), sel.end());
  for (int64_t i = 0; i < n; ++i) residual[i] = acc[i];
  const float pos_zero = 0.0f;
  for (size_t j = 0; j < sel.size(); ++j) {
    int32_t i = sel[j];
    out_idx[j] = i;
    out_val[j] = acc[i];
    residual[i] = pos_zero;
    if (momentum != nullptr && mask_momentum) momentum[i] = pos_zero;
  }
  *out_count = static_cast<int32_t>(sel.size());
}

}  // namespace

extern "C" {

// k for a density given in parts per million.
int32_t rgc_oracle_k_for_density(int64_t n, uint32_t density_ppm) {
  if (n < 1) return 0;
  // ceil(n*ppm/1e6) without overflow for n < 2^31, ppm <= 1e6.
  unsigned long long num = static_cast<unsigned long long>(n) * density_ppm;
  unsigned long long k = (num + 999999ull) / 1000000ull;
  if (k < 1) k = 1;
  if (k > static_cast<unsigned long long>(n)) k = static_cast<unsigned long long>(n);
  return static_cast<int32_t>(k);
}

// One layer of the compression step, exact top-k by a full sort of
// (magnitude key descending, index ascending).  `momentum` may be NULL.
// Returns 0, or -1 on bad arguments.
// `nesterov` and `scale` (NULL: none) as described at the top of this file.
int rgc_oracle_compress_layer_ex(const float* grad, float* residual, float* momentum,
                                 int64_t n, int32_t k, float m, int mask_momentum, int nesterov,
                                 const float* scale,
                                 int32_t* out_idx, float* out_val, int32_t* out_count) {
  if (!grad || !residual || !out_idx || !out_val || !out_count) return -1;
  if (n < 1 || n >= (int64_t(1) << 31) || k < 1 || k > n) return -1;
  std::vector<float> acc;
  accumulate(grad, residual, momentum, n, m, nesterov, scale, acc);

  std::vector<std::pair<uint32_t, int32_t>> order(static_cast<size_t>(n));
  for (int64_t i = 0; i < n; ++i)
    order[i] = {magnitude_key(acc[i]), static_cast<int32_t>(i)};
  std::sort(order.begin(), order.end(),
            [](const std::pair<uint32_t, int32_t>& a, const std::pair<uint32_t, int32_t>& b) {
              if (a.first != b.first) return a.first > b.first;
              return a.second < b.second;
            });
  std::vector<int32_t> sel(static_cast<size_t>(k));
  for (int32_t j = 0; j < k; ++j) sel[j] = order[j].second;
  emit(acc, sel, residual, momentum, mask_momentum, n, out_idx, out_val, out_count);
  return 0;
}

int rgc_oracle_compress_layer(const float* grad, float* residual, float* momentum,
                              int64_t n, int32_t k, float m, int mask_momentum,
                              int32_t* out_idx, float* out_val, int32_t* out_count) {
  return rgc_oracle_compress_layer_ex(grad, residual, momentum, n, k, m, mask_momentum, 0, nullptr,
                                      out_idx, out_val, out_count);
}

// Selection key of Alternating Signs Quantization: an unsigned integer that
// grows with the value of x (sign = +1) or of -x (sign = -1); both zeros map
// to the same key.
inline uint32_t asq_key(float x, int sign) {
  uint32_t b = float_bits(x);
  if (sign < 0) b ^= 0x80000000u;               // -x
  if ((b & 0x7FFFFFFFu) == 0u) b = 0u;          // -0 and +0 are the same value
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// One layer of the compression step with Alternating Signs Quantization (see
// the top of this file).  out_idx[k]; *out_mean is the one value of the message.
// bruteforce != 0 (tiny n only): k rounds of "largest remaining key, first
// occurrence" instead of the sort.
int rgc_oracle_compress_layer_asq(const float* grad, float* residual, float* momentum,
                                  int64_t n, int32_t k, float m, int mask_momentum, int sign,
                                  int bruteforce, int32_t* out_idx, float* out_mean,
                                  int32_t* out_count) {
  if (!grad || !residual || !out_idx || !out_mean || !out_count) return -1;
  if (n < 1 || n >= (int64_t(1) << 31) || k < 1 || k > n || (sign != 1 && sign != -1)) return -1;
  if (bruteforce && n > 4096) return -1;
  std::vector<float> acc;
  accumulate(grad, residual, momentum, n, m, 0, nullptr, acc);
  std::vector<int32_t> sel;
  if (bruteforce) {
    std::vector<char> taken(static_cast<size_t>(n), 0);
    for (int32_t round = 0; round < k; ++round) {
      int64_t best = -1;
      for (int64_t i = 0; i < n; ++i) {
        if (taken[i]) continue;
        if (best < 0 || asq_key(acc[i], sign) > asq_key(acc[best], sign)) best = i;
      }
      taken[best] = 1;
      sel.push_back(static_cast<int32_t>(best));
    }
  } else {
    std::vector<std::pair<uint32_t, int32_t>> order(static_cast<size_t>(n));
    for (int64_t i = 0; i < n; ++i) order[i] = {asq_key(acc[i], sign), static_cast<int32_t>(i)};
    std::sort(order.begin(), order.end(),
              [](const std::pair<uint32_t, int32_t>& a, const std::pair<uint32_t, int32_t>& b) {
                if (a.first != b.first) return a.first > b.first;
                return a.second < b.second;
              });
    for (int32_t j = 0; j < k; ++j) sel.push_back(order[j].second);
  }
  std::vector<float> values(static_cast<size_t>(k));
  emit(acc, sel, residual, momentum, mask_momentum, n, out_idx, values.data(), out_count);
  ExactSum sum;
  for (int32_t j = 0; j < k; ++j) sum.add(static_cast<double>(values[j]));
  *out_mean = static_cast<float>(sum.rounded() / static_cast<double>(k));
  return 0;
}

// One layer of the compression step with threshold binary search selection
// (see the top of this file).  `scale` (NULL: none) is the clipping coefficient
// of the accumulate.  search != 0: Algorithm 3 finds *threshold;
// search == 0: *threshold is applied as given.  out_idx / out_val hold cap
// entries; *out_count = min(nnz, cap); *out_nnz = the number of elements above
// the threshold.  out_trace (may be NULL, 4 floats): mean, max, number of
// counts taken, last ratio.
int rgc_oracle_compress_layer_threshold(const float* grad, float* residual, float* momentum,
                                        int64_t n, int32_t k, float m, int mask_momentum,
                                        int nesterov, const float* scale, int search, float* threshold,
                                        int32_t cap,
                                        int32_t* out_idx, float* out_val, int32_t* out_count,
                                        int64_t* out_nnz, float* out_trace) {
  if (!grad || !residual || !threshold || !out_idx || !out_val || !out_count || !out_nnz) return -1;
  if (n < 1 || n >= (int64_t(1) << 31) || k < 1 || k > n || cap < 1) return -1;
  std::vector<float> acc;
  accumulate(grad, residual, momentum, n, m, nesterov, scale, acc);
  auto count_above = [&](float t) {
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i) c += (std::fabs(acc[i]) > t) ? 1 : 0;
    return c;
  };
  if (search) {
    ExactSum sum;
    float max = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      const float mag = std::fabs(acc[i]);
      sum.add(static_cast<double>(mag));
      if (mag > max) max = mag;
    }
    const float mean = static_cast<float>(sum.rounded() / static_cast<double>(n));
    const float eps = 1.0f / 1024.0f;
    float l = 0.0f, r = 1.0f, thr = 0.0f, ratio = 0.0f;
    int counts = 0;
    while (r - l > eps) {
      const float half = (r - l) / 2.0f;
      ratio = l + half;
      const float span = max - mean;
      const float offset = ratio * span;
      thr = mean + offset;
      const int64_t nnz = count_above(thr);
      ++counts;
      if (nnz > k && nnz < 2 * static_cast<int64_t>(k)) break;
      if (nnz <= k) r = ratio; else l = ratio;
    }
    *threshold = thr;
    if (out_trace) {
      out_trace[0] = mean;
      out_trace[1] = max;
      out_trace[2] = static_cast<float>(counts);
      out_trace[3] = ratio;
    }
  }
  const float thr = *threshold;
  std::vector<int32_t> sel;
  int64_t nnz = 0;
  for (int64_t i = 0; i < n; ++i) {
    if (std::fabs(acc[i]) > thr) {
      if (nnz < cap) sel.push_back(static_cast<int32_t>(i));
      ++nnz;
    }
  }
  *out_nnz = nnz;
  emit(acc, sel, residual, momentum, mask_momentum, n, out_idx, out_val, out_count);
  return 0;
}

// Decompression of messages that carry one value each (Alternating Signs
// Quantization): worker w adds value[w] at each of its indices.
int rgc_oracle_decompress_scalar(const int32_t* const* idx, const float* value,
                                 const int32_t* count, int32_t num_workers, float* dense,
                                 int64_t n, float scale, int add_to_dst) {
  if (!dense || n < 1 || num_workers < 0) return -1;
  std::vector<float> acc(static_cast<size_t>(n), 0.0f);
  for (int32_t w = 0; w < num_workers; ++w) {
    if (count[w] < 0) return -1;
    for (int32_t j = 0; j < count[w]; ++j) {
      int32_t i = idx[w][j];
      if (i < 0 || i >= n) return -1;
      acc[i] = acc[i] + value[w];
    }
  }
  if (add_to_dst) {
    for (int64_t i = 0; i < n; ++i) {
      float scaled = acc[i] * scale;
      dense[i] = dense[i] + scaled;
    }
  } else {
    for (int64_t i = 0; i < n; ++i) dense[i] = acc[i] * scale;
  }
  return 0;
}

// Same result by brute force, for tiny n only: k rounds of "largest remaining
// magnitude, first occurrence".  Exists to pin the sort-based version.
int rgc_oracle_compress_layer_bruteforce(const float* grad, float* residual, float* momentum,
                                         int64_t n, int32_t k, float m, int mask_momentum,
                                         int32_t* out_idx, float* out_val, int32_t* out_count) {
  if (!grad || !residual || !out_idx || !out_val || !out_count) return -1;
  if (n < 1 || n > 4096 || k < 1 || k > n) return -1;
  std::vector<float> acc;
  accumulate(grad, residual, momentum, n, m, 0, nullptr, acc);
  std::vector<char> taken(static_cast<size_t>(n), 0);
  std::vector<int32_t> sel;
  for (int32_t round = 0; round < k; ++round) {
    int64_t best = -1;
    for (int64_t i = 0; i < n; ++i) {
      if (taken[i]) continue;
      if (best < 0 || magnitude_key(acc[i]) > magnitude_key(acc[best])) best = i;
    }
    taken[best] = 1;
    sel.push_back(static_cast<int32_t>(best));
  }
  emit(acc, sel, residual, momentum, mask_momentum, n, out_idx, out_val, out_count);
  return 0;
}

// A whole layer set: Algorithm 1's inner loop over the layers, which are
// independent of each other, so layer l goes to host thread l mod `threads`
// (threads <= 1 runs the plain sequential loop).  Every multi-layer reference of
// the parity tests, the smoke check and the benchmark's CPU timing comes from
// here; the pins compare it with one call per layer for several thread counts.
int rgc_oracle_compress_layers_ex(const float* const* grad, float* const* residual,
                                  float* const* momentum, const int64_t* n, const int32_t* k,
                                  int32_t num_layers, float m, int mask_momentum, int nesterov,
                                  const float* scale,
                                  int32_t* const* out_idx, float* const* out_val,
                                  int32_t* out_count, int32_t threads) {
  if (num_layers < 0) return -1;
  std::vector<int> rc(static_cast<size_t>(num_layers), 0);
  auto work = [&](int32_t first, int32_t step) {
    for (int32_t l = first; l < num_layers; l += step)
      rc[l] = rgc_oracle_compress_layer_ex(grad[l], residual[l], momentum ? momentum[l] : nullptr,
                                           n[l], k[l], m, mask_momentum, nesterov, scale,
                                           out_idx[l], out_val[l], &out_count[l]);
  };
  if (threads <= 1) {
    work(0, 1);
  } else {
    std::vector<std::thread> pool;
    for (int32_t t = 0; t < threads; ++t) pool.emplace_back(work, t, threads);
    for (auto& th : pool) th.join();
  }
  for (int32_t l = 0; l < num_layers; ++l)
    if (rc[l] != 0) return -1;
  return 0;
}

int rgc_oracle_compress_layers(const float* const* grad, float* const* residual,
                               float* const* momentum, const int64_t* n, const int32_t* k,
                               int32_t num_layers, float m, int mask_momentum,
                               int32_t* const* out_idx, float* const* out_val,
                               int32_t* out_count, int32_t threads) {
  return rgc_oracle_compress_layers_ex(grad, residual, momentum, n, k, num_layers, m, mask_momentum,
                                       0, nullptr, out_idx, out_val, out_count, threads);
}

// Local gradient clipping coefficient over all layers of one call (see the top
// of this file).  Also stores the squared norm (fp64) if sqnorm is not NULL.
float rgc_oracle_clip_coefficient(const float* const* grad, const int64_t* n, int32_t num_layers,
                                  float max_norm, int32_t num_workers, double* sqnorm) {
  ExactSum squares;
  for (int32_t l = 0; l < num_layers; ++l)
    for (int64_t i = 0; i < n[l]; ++i) {
      double g = static_cast<double>(grad[l][i]);
      squares.add(g * g);                  // 24 bits times 24 bits: the product is exact in fp64
    }
  const double sum = squares.rounded();
  if (sqnorm) *sqnorm = sum;
  double norm = std::sqrt(sum);
  double t = static_cast<double>(max_norm) / std::sqrt(static_cast<double>(num_workers));
  double c = norm > t ? t / norm : 1.0;
  return static_cast<float>(c);
}

// Decompression of one layer: N messages (idx[w], val[w], count[w]) added in
// worker order into an fp32 accumulator that starts at +0, then scaled once.
// add_to_dst = 0: dense = acc*scale;  1: dense = dense + acc*scale.
int rgc_oracle_decompress(const int32_t* const* idx, const float* const* val,
                          const int32_t* count, int32_t num_workers, float* dense,
                          int64_t n, float scale, int add_to_dst) {
  if (!dense || n < 1 || num_workers < 0) return -1;
  std::vector<float> acc(static_cast<size_t>(n), 0.0f);
  for (int32_t w = 0; w < num_workers; ++w) {
    if (count[w] < 0) return -1;
    for (int32_t j = 0; j < count[w]; ++j) {
      int32_t i = idx[w][j];
      if (i < 0 || i >= n) return -1;
      acc[i] = acc[i] + val[w][j];
    }
  }
  if (add_to_dst) {
    for (int64_t i = 0; i < n; ++i) {
      float scaled = acc[i] * scale;
      dense[i] = dense[i] + scaled;
    }
  } else {
    for (int64_t i = 0; i < n; ++i) dense[i] = acc[i] * scale;
  }
  return 0;
}

// The exactly rounded sum the three reductions above are built on, by itself
// (for the tests that pin it).
double rgc_oracle_exact_sum(const double* x, int64_t n) {
  ExactSum sum;
  for (int64_t i = 0; i < n; ++i) sum.add(x[i]);
  return sum.rounded();
}

// Number of host threads the machine reports (for the benchmark's "cores").
int32_t rgc_oracle_hardware_threads() {
  unsigned t = std::thread::hardware_concurrency();
  return t ? static_cast<int32_t>(t) : 1;
}

}  // extern "C"
