// Drives every entry point of the CPU oracle on small seeded inputs; built together with
// rgc_oracle.cpp under -fsanitize=address,undefined by tests/test_oracle_sanitizers.py, so that an
// out-of-bounds index, a use after free or undefined arithmetic in the oracle fails a CPU test.
// TEST INFRASTRUCTURE like the oracle itself.  Exit status 0 = every call returned what it should.
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>

extern "C" {
int32_t rgc_oracle_k_for_density(int64_t n, uint32_t density_ppm);
int rgc_oracle_compress_layer_ex(const float*, float*, float*, int64_t, int32_t, float, int, int, const float*,
                                 int32_t*, float*, int32_t*);
int rgc_oracle_compress_layer_bruteforce(const float*, float*, float*, int64_t, int32_t, float, int, int32_t*, float*,
                                         int32_t*);
int rgc_oracle_compress_layer_asq(const float*, float*, float*, int64_t, int32_t, float, int, int, int, int32_t*,
                                  float*, int32_t*);
int rgc_oracle_compress_layer_threshold(const float*, float*, float*, int64_t, int32_t, float, int, int,
                                        const float*, int, float*, int32_t, int32_t*, float*, int32_t*, int64_t*,
                                        float*);
int rgc_oracle_compress_layers_ex(const float* const*, float* const*, float* const*, const int64_t*, const int32_t*,
                                  int32_t, float, int, int, const float*, int32_t* const*, float* const*, int32_t*,
                                  int32_t);
float rgc_oracle_clip_coefficient(const float* const*, const int64_t*, int32_t, float, int32_t, double*);
double rgc_oracle_exact_sum(const double*, int64_t);
int rgc_oracle_decompress(const int32_t* const*, const float* const*, const int32_t*, int32_t, float*, int64_t, float,
                          int);
int rgc_oracle_decompress_scalar(const int32_t* const*, const float*, const int32_t*, int32_t, float*, int64_t, float,
                                 int);
}

#define CHECK(cond) if (!(cond)) { std::fprintf(stderr, "sanitize_check: %s failed (line %d)\n", #cond, __LINE__); return 1; }

int main() {
  std::mt19937 gen(12345);
  std::normal_distribution<float> normal(0.0f, 1.0f);
  const int64_t sizes[] = {1, 2, 7, 64, 1000, 4097};
  for (int64_t n : sizes) {
    for (int32_t k : {int32_t(1), int32_t((n + 1) / 2), int32_t(n)}) {
      std::vector<float> g(n), v(n), u(n);
      for (int64_t i = 0; i < n; ++i) { g[i] = normal(gen) * 1e-3f; v[i] = normal(gen) * 1e-2f; u[i] = normal(gen) * 1e-3f; }
      if (n > 3) { v[1] = v[2]; g[1] = g[2]; }                    // a tie
      std::vector<int32_t> idx(2 * static_cast<size_t>(k) + 1);
      std::vector<float> val(2 * static_cast<size_t>(k) + 1);
      int32_t cnt = -1;
      const float scale = 0.5f;
      std::vector<float> v1 = v, u1 = u;
      CHECK(rgc_oracle_compress_layer_ex(g.data(), v1.data(), u1.data(), n, k, 0.9f, 1, 0, nullptr, idx.data(), val.data(), &cnt) == 0 && cnt == k);
      v1 = v; u1 = u;
      CHECK(rgc_oracle_compress_layer_ex(g.data(), v1.data(), u1.data(), n, k, 0.9f, 0, 1, &scale, idx.data(), val.data(), &cnt) == 0 && cnt == k);
      v1 = v;
      if (n <= 4096) CHECK(rgc_oracle_compress_layer_bruteforce(g.data(), v1.data(), nullptr, n, k, 0.0f, 1, idx.data(), val.data(), &cnt) == 0 && cnt == k);
      for (int sign : {1, -1}) {
        float mean = 0.0f;
        v1 = v; u1 = u;
        CHECK(rgc_oracle_compress_layer_asq(g.data(), v1.data(), u1.data(), n, k, 0.9f, 1, sign, 0, idx.data(), &mean, &cnt) == 0 && cnt == k);
        v1 = v;
        if (n <= 4096) CHECK(rgc_oracle_compress_layer_asq(g.data(), v1.data(), nullptr, n, k, 0.0f, 1, sign, 1, idx.data(), &mean, &cnt) == 0 && cnt == k);
      }
      for (int search : {1, 0}) {
        float thr = 1e-3f, trace[4];
        int64_t nnz = -1;
        v1 = v; u1 = u;
        CHECK(rgc_oracle_compress_layer_threshold(g.data(), v1.data(), u1.data(), n, k, 0.9f, 1, 0, nullptr, search, &thr,
                                                  2 * k, idx.data(), val.data(), &cnt, &nnz, trace) == 0);
        CHECK(cnt >= 0 && cnt <= 2 * k && nnz >= cnt);
      }
      CHECK(rgc_oracle_compress_layer_ex(g.data(), v1.data(), nullptr, n, k + static_cast<int32_t>(n), 0.0f, 1, 0, nullptr, idx.data(), val.data(), &cnt) == -1);
    }
  }
  {
    // a layer set on several threads, more layers than threads and fewer
    const int32_t L = 5;
    std::vector<std::vector<float>> g(L), v(L), u(L), val(L);
    std::vector<std::vector<int32_t>> idx(L);
    std::vector<const float*> gp(L);
    std::vector<float*> vp(L), up(L), valp(L);
    std::vector<int32_t*> idxp(L);
    std::vector<int64_t> n(L);
    std::vector<int32_t> k(L), cnt(L, -1);
    for (int32_t l = 0; l < L; ++l) {
      n[l] = 10 + 300 * l;
      k[l] = rgc_oracle_k_for_density(n[l], 50000);
      g[l].resize(n[l]); v[l].resize(n[l]); u[l].resize(n[l]); val[l].resize(k[l]); idx[l].resize(k[l]);
      for (int64_t i = 0; i < n[l]; ++i) { g[l][i] = normal(gen); v[l][i] = normal(gen); u[l][i] = normal(gen); }
      gp[l] = g[l].data(); vp[l] = v[l].data(); up[l] = u[l].data(); valp[l] = val[l].data(); idxp[l] = idx[l].data();
    }
    for (int32_t threads : {1, 3, 16})
      CHECK(rgc_oracle_compress_layers_ex(gp.data(), vp.data(), up.data(), n.data(), k.data(), L, 0.9f, 1, 0, nullptr,
                                          idxp.data(), valp.data(), cnt.data(), threads) == 0);
    double sq = 0.0;
    const float c = rgc_oracle_clip_coefficient(gp.data(), n.data(), L, 1.0f, 4, &sq);
    CHECK(c > 0.0f && c <= 1.0f && sq > 0.0);
    // the exactly rounded sum at both ends of the format's range, with cancellation
    const double ends[] = {1.7976931348623157e308, 4.9406564584124654e-324, -1.7976931348623157e308,
                           1.0, -4.9406564584124654e-324, 1e-320, 1.7976931348623157e308};
    CHECK(rgc_oracle_exact_sum(ends, 7) == 1.7976931348623157e308);
    CHECK(rgc_oracle_exact_sum(ends, 6) == 1.0);
    CHECK(rgc_oracle_exact_sum(ends, 0) == 0.0);
  }
  {
    // decompression: overlapping workers, an empty one, both destination modes, one-value messages
    const int64_t n = 300;
    const int32_t N = 4;
    std::vector<std::vector<int32_t>> idx(N);
    std::vector<std::vector<float>> val(N);
    std::vector<const int32_t*> ip(N);
    std::vector<const float*> vp(N);
    std::vector<int32_t> cnt(N);
    std::vector<float> one(N);
    for (int32_t w = 0; w < N; ++w) {
      for (int32_t i = w; i < n && w != 2; i += 3 + w) { idx[w].push_back(i); val[w].push_back(normal(gen)); }
      ip[w] = idx[w].data(); vp[w] = val[w].data(); cnt[w] = static_cast<int32_t>(idx[w].size()); one[w] = normal(gen);
    }
    std::vector<float> dense(n, 1.0f);
    CHECK(rgc_oracle_decompress(ip.data(), vp.data(), cnt.data(), N, dense.data(), n, 0.25f, 0) == 0);
    CHECK(rgc_oracle_decompress(ip.data(), vp.data(), cnt.data(), N, dense.data(), n, 0.25f, 1) == 0);
    CHECK(rgc_oracle_decompress_scalar(ip.data(), one.data(), cnt.data(), N, dense.data(), n, 1.0f, 0) == 0);
    CHECK(rgc_oracle_decompress(ip.data(), vp.data(), cnt.data(), 0, dense.data(), n, 1.0f, 0) == 0);
    idx[0][0] = static_cast<int32_t>(n);                        // out of range: rejected, nothing written beyond the buffer
    CHECK(rgc_oracle_decompress(ip.data(), vp.data(), cnt.data(), N, dense.data(), n, 1.0f, 0) == -1);
  }
  std::puts("sanitize_check ok");
  return 0;
}
