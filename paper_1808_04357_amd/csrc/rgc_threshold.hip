// gfx950 kernels of the compression step with threshold binary search selection (RedSync,
// Section 2.1, Algorithm 3, and the sampled variant of the same section that reuses a threshold):
// the communication-set of a layer is every element whose magnitude exceeds a threshold, the
// threshold is searched on  mean + ratio * (max - mean),  ratio bisected in [0, 1] until between
// k and 2k elements pass or the interval is shorter than 2^-10.
//
// The paper's listing counts the elements above the threshold once per bisection step, i.e. up to
// ten passes over the layer.  Here the ten counts cost ONE pass: the interval ends are multiples
// of 2^-10, so the search can only ever try the 1023 thresholds  T(j) = mean + (j/1024)(max - mean);
// a histogram of  bin(x) = #{j : T(j) < |x|}  over the layer gives the count above every T(j) as a
// suffix sum, and the bisection runs on those sums.  T(j) is computed with the very operations
// of the listing (fp32, every operation rounded), so the counts are the listing's counts.
//
// Launches of one call (same workgroup -> layer -> wave-chunk decomposition as the exact path):
//   search:  accumulate (+ partial sums and maxima of |a|)  ->  moments  ->  histogram  ->  search
//            ->  count  ->  offsets  ->  emit
//   reuse:   accumulate (+ the elements above the given threshold, listed per wave-chunk)  ->  offsets
//            ->  emit from the lists
#include "rgc_exact.h"

namespace rgc {

namespace {

constexpr uint32_t kSteps = 1024;   // 1 / epsilon of the search: ratios are multiples of 2^-10

typedef uint32_t vu2 __attribute__((ext_vector_type(2)));   // a listed element: (float bits, index)

// T(j), j = 1 .. 1023; the operations and their order are those of Algorithm 3.
__device__ __forceinline__ float threshold_at(float mean, float span, uint32_t j) {
  const float ratio = static_cast<float>(j) * (1.0f / static_cast<float>(kSteps));   // exact
  return __fadd_rn(mean, __fmul_rn(ratio, span));
}

// #{j in 1..1023 : T(j) < x}.  T is non-decreasing in j (span >= 0, rounding is monotone), so this is
// the largest j with T(j) < x, or 0.  A guess from the inverse map is checked against T itself; where
// the guess is off, a binary search over j finds it.
__device__ __forceinline__ uint32_t bin_of(float x, float mean, float span, float inv) {
  const float g = __fmul_rn(__fsub_rn(x, mean), inv);
  uint32_t j = g > 0.0f ? (g < static_cast<float>(kSteps - 1u) ? static_cast<uint32_t>(g) : kSteps - 1u) : 0u;   // NaN -> 0
  const bool lo_ok = (j == 0u) || (threshold_at(mean, span, j) < x);
  const bool hi_ok = (j == kSteps - 1u) || !(threshold_at(mean, span, j + 1u) < x);
  if (lo_ok && hi_ok) return j;
  uint32_t lo = 0u, hi = kSteps - 1u;
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1u) >> 1;
    if (threshold_at(mean, span, mid) < x) lo = mid; else hi = mid - 1u;
  }
  return lo;
}

struct Place {           // where a wave works
  uint32_t l;            // layer
  uint32_t wc;           // its wave-chunk, global number
  uint32_t begin, end;   // element range inside the layer; begin == end: nothing to do
};

__device__ __forceinline__ Place place_of(const ThresholdArgs& A, const LayerDesc& L, uint32_t l, uint32_t wg) {
  Place p;
  p.l = l;
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  p.wc = L.wc_first + wc_local;
  if (wc_local < L.wc_count) {
    p.begin = wc_local * A.chunk;
    p.end = (L.n - p.begin) < A.chunk ? L.n : p.begin + A.chunk;
  } else {
    p.begin = p.end = 0u;
  }
  return p;
}

// Calls f(a, nvalid, idx0) for the groups of 256 elements of [begin, end) of tensor p: lane-major,
// four consecutive elements per lane; whole groups of an aligned tensor four at a time.
template <typename F>
__device__ __forceinline__ void read_groups(const float* generic_p, bool vec, uint32_t begin, uint32_t end, F&& f) {
  const gptr<const float> p = as_global(generic_p);
  const uint32_t lane = lane_id();
  uint32_t base = begin;
  if (vec) {
    constexpr uint32_t kUnroll = 4u;
    for (; base + kUnroll * kGroupElems <= end; base += kUnroll * kGroupElems) {
      vf4 q[kUnroll];
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) q[t] = *reinterpret_cast<gptr<const vf4>>(p + base + t * kGroupElems + lane * 4u);
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) {
        const float a[4] = {q[t].x, q[t].y, q[t].z, q[t].w};
        f(a, 4u, base + t * kGroupElems + lane * 4u);
      }
    }
  }
  for (; base < end; base += kGroupElems) {
    const uint32_t idx0 = base + lane * 4u;
    float a[4] = {0.f, 0.f, 0.f, 0.f};
    uint32_t nvalid;
    if (vec && base + kGroupElems <= end) {
      const vf4 q = *reinterpret_cast<gptr<const vf4>>(p + idx0);
      a[0] = q.x; a[1] = q.y; a[2] = q.z; a[3] = q.w;
      nvalid = 4u;
    } else {
      nvalid = idx0 < end ? ((end - idx0) < 4u ? (end - idx0) : 4u) : 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (static_cast<uint32_t>(j) < nvalid) a[j] = p[idx0 + j];
    }
    f(a, nvalid, idx0);
  }
}

// The accumulate of Algorithm 1 over [begin, end) of a layer (same arithmetic as the exact path:
// accum4), handing every group of accumulated values to f.  Whole groups of an aligned layer are
// taken four (two with a velocity) at a time, all their loads issued before the first use.
template <bool kMom, bool kNest, typename F>
__device__ __forceinline__ void accumulate_groups(const LayerDesc& L, uint32_t begin, uint32_t end, const AccumRule& rule, F&& f) {
  const gptr<const float> G = as_global(L.grad);
  const gptr<float> V = as_global(L.resid);
  const gptr<float> U = as_global(L.mom);
  const uint32_t lane = lane_id();
  uint32_t base = begin;
  if (L.vec_ok) {
    constexpr uint32_t kUnroll = kMom ? 2u : 4u;
    for (; base + kUnroll * kGroupElems <= end; base += kUnroll * kGroupElems) {
      vf4 gq[kUnroll], vq[kUnroll], uq[kUnroll];
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) {
        const uint32_t idx0 = base + t * kGroupElems + lane * 4u;
        gq[t] = __builtin_nontemporal_load(reinterpret_cast<gptr<const vf4>>(G + idx0));
        vq[t] = *reinterpret_cast<gptr<const vf4>>(V + idx0);
        if constexpr (kMom) uq[t] = *reinterpret_cast<gptr<const vf4>>(U + idx0);
      }
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) {
        const uint32_t idx0 = base + t * kGroupElems + lane * 4u;
        const float g[4] = {gq[t].x, gq[t].y, gq[t].z, gq[t].w};
        const float v[4] = {vq[t].x, vq[t].y, vq[t].z, vq[t].w};
        float u[4] = {0.f, 0.f, 0.f, 0.f}, a[4];
        if constexpr (kMom) { u[0] = uq[t].x; u[1] = uq[t].y; u[2] = uq[t].z; u[3] = uq[t].w; }
        accum4<kMom, kNest>(g, v, u, rule, a);
        *reinterpret_cast<gptr<vf4>>(V + idx0) = vf4{a[0], a[1], a[2], a[3]};
        if constexpr (kMom) *reinterpret_cast<gptr<vf4>>(U + idx0) = vf4{u[0], u[1], u[2], u[3]};
        f(a, 4u, idx0);
      }
    }
  }
  for (; base < end; base += kGroupElems) {
    const uint32_t idx0 = base + lane * 4u;
    float g[4] = {0.f, 0.f, 0.f, 0.f}, v[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f}, a[4];
    if (L.vec_ok && base + kGroupElems <= end) {
      const vf4 gq = __builtin_nontemporal_load(reinterpret_cast<gptr<const vf4>>(G + idx0));
      const vf4 vq = *reinterpret_cast<gptr<const vf4>>(V + idx0);
      g[0] = gq.x; g[1] = gq.y; g[2] = gq.z; g[3] = gq.w;
      v[0] = vq.x; v[1] = vq.y; v[2] = vq.z; v[3] = vq.w;
      if constexpr (kMom) {
        const vf4 uq = *reinterpret_cast<gptr<const vf4>>(U + idx0);
        u[0] = uq.x; u[1] = uq.y; u[2] = uq.z; u[3] = uq.w;
      }
      accum4<kMom, kNest>(g, v, u, rule, a);
      *reinterpret_cast<gptr<vf4>>(V + idx0) = vf4{a[0], a[1], a[2], a[3]};
      if constexpr (kMom) *reinterpret_cast<gptr<vf4>>(U + idx0) = vf4{u[0], u[1], u[2], u[3]};
      f(a, 4u, idx0);
    } else {
      const uint32_t nvalid = idx0 < end ? ((end - idx0) < 4u ? (end - idx0) : 4u) : 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (static_cast<uint32_t>(j) < nvalid) {
          g[j] = G[idx0 + j];
          v[j] = V[idx0 + j];
          if constexpr (kMom) u[j] = U[idx0 + j];
        }
      }
      accum4<kMom, kNest>(g, v, u, rule, a);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (static_cast<uint32_t>(j) < nvalid) {
          V[idx0 + j] = a[j];
          if constexpr (kMom) U[idx0 + j] = u[j];
        }
      }
      f(a, nvalid, idx0);
    }
  }
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}

}  // namespace

// ------------------------------------------------------------------ accumulate (+ moments or counts)
// kCount = false (a search follows): leaves per workgroup its part of the exactly rounded sum of |a|
// (rgc_exact.h) and the maximum of |a|.
// kCount = true (the threshold is given): leaves per wave-chunk the number of |a| > threshold and, in
// the wave-chunk's list, those elements themselves (as many as the list holds).
template <bool kCount, bool kReverse>
__global__ void __launch_bounds__(kBlockThreads) threshold_accumulate_kernel(ThresholdArgs A) {
  __shared__ ExactShared sh;
  __shared__ float wave_mx[kWavesPerBlock];
  if constexpr (!kCount) {
    exact_shared_init(sh);
    __syncthreads();
  }
  const uint32_t wg = (kReverse != (A.reverse != 0u)) ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  const Place p = place_of(A, L, l, wg);
  ExactAcc acc{0.0, 0.0, 0u};
  float mx = 0.0f;
  if (p.begin != p.end) {
    const float thr = kCount ? *as_global(A.thresholds + l) : 0.0f;
    uint32_t cnt = 0u;                      // kCount: elements above the threshold so far, the same in every lane
    const gptr<vu2> slot = as_global(reinterpret_cast<vu2*>(A.slots + static_cast<size_t>(p.wc) * A.cap));
    auto take = [&](const float (&a)[4], uint32_t nvalid, uint32_t idx0) {
      if constexpr (kCount) {
        // the elements above the threshold go to the wave-chunk's list in index order (ballot ranks);
        // a list that is full only counts on, and the emit pass reads that wave-chunk from V instead
        bool f[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = static_cast<uint32_t>(j) < nvalid && fabsf(a[j]) > thr;
        const unsigned long long m0 = __ballot(f[0]), m1 = __ballot(f[1]), m2 = __ballot(f[2]), m3 = __ballot(f[3]);
        if ((m0 | m1 | m2 | m3) == 0ull) return;
        uint32_t pos = cnt + rank_below(m0) + rank_below(m1) + rank_below(m2) + rank_below(m3);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (f[j]) {
            if (pos < A.cap) slot[pos] = vu2{fbits(a[j]), idx0 + static_cast<uint32_t>(j)};
            ++pos;
          }
        }
        cnt += popc64(m0) + popc64(m1) + popc64(m2) + popc64(m3);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (static_cast<uint32_t>(j) < nvalid) {
            const float mag = fabsf(a[j]);
            exact_add_f32(acc, mag, sh.digits);
            mx = fmaxf(mx, mag);
          }
        }
      }
    };
    AccumRule rule;
    rule.m = A.m;
    rule.scale = A.grad_scale ? *as_global(A.grad_scale) : 1.0f;
    if (L.mom == nullptr) accumulate_groups<false, false>(L, p.begin, p.end, rule, take);
    else if (!A.nesterov) accumulate_groups<true, false>(L, p.begin, p.end, rule, take);
    else accumulate_groups<true, true>(L, p.begin, p.end, rule, take);
    if constexpr (kCount) {
      if (lane_id() == 0u) {
        A.counts[p.wc] = cnt;
        A.listed[p.wc] = cnt;
      }
    }
  }
  if constexpr (!kCount) {
    const float m = wave_max(mx);
    if (lane_id() == 0u) wave_mx[threadIdx.x >> 6] = m;
    const ExactAcc total = exact_block_total(acc, sh);      // its barriers also order wave_mx
    if (threadIdx.x == 0u) {
      exact_store_part(A.sum_parts, wg, total, sh);
      float bm = wave_mx[0];
#pragma unroll
      for (int w = 1; w < kWavesPerBlock; ++w) bm = fmaxf(bm, wave_mx[w]);
      A.part_max[wg] = bm;
    }
  }
}

// ------------------------------------------------------------------ moments of a layer
// One workgroup per layer adds the parts of the layer's workgroups up, rounds the sum once, takes the
// maximum, stores mean, max and max - mean, and clears the layer's histogram for the pass that follows.
__global__ void __launch_bounds__(kBlockThreads) threshold_moments_kernel(ThresholdArgs A) {
  __shared__ ExactShared sh;
  __shared__ float redm[kBlockThreads];
  exact_shared_init(sh);
  __syncthreads();
  const uint32_t l = blockIdx.x;
  const LayerDesc L = A.layers[l];
  ExactPair acc;
  float mx = 0.0f;
  exact_take_parts(acc, A.sum_parts, L.wg_first, L.wg_count, sh);
  for (uint32_t i = threadIdx.x; i < L.wg_count; i += kBlockThreads) mx = fmaxf(mx, A.part_max[L.wg_first + i]);
  redm[threadIdx.x] = mx;
  const double sum = exact_finish(acc, sh);                 // holds barriers
  for (uint32_t step = kBlockThreads / 2u; step >= 1u; step >>= 1) {
    if (threadIdx.x < step) redm[threadIdx.x] = fmaxf(redm[threadIdx.x], redm[threadIdx.x + step]);
    __syncthreads();
  }
  if (threadIdx.x == 0u) {
    ThresholdMoments M;
    M.mean = static_cast<float>(sum / static_cast<double>(L.n));
    M.max = redm[0];
    M.span = __fsub_rn(M.max, M.mean);
    M.counts_taken = 0u;
    A.moments[l] = M;
  }
  uint32_t* hist = A.hist + static_cast<size_t>(l) * kHistBins;
  for (uint32_t b = threadIdx.x; b < kSteps; b += kBlockThreads) hist[b] = 0u;
}

// ------------------------------------------------------------------ histogram over the candidate thresholds
template <bool kReverse>
__global__ void __launch_bounds__(kBlockThreads) threshold_histogram_kernel(ThresholdArgs A) {
  __shared__ uint32_t lds_hist[kSteps];
  const uint32_t wg = (kReverse != (A.reverse != 0u)) ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  const Place p = place_of(A, L, l, wg);
  for (uint32_t b = threadIdx.x; b < kSteps; b += kBlockThreads) lds_hist[b] = 0u;
  __syncthreads();
  const ThresholdMoments M = A.moments[l];
  const float inv = M.span > 0.0f ? static_cast<float>(kSteps) / M.span : 0.0f;
  uint32_t below = 0u;     // bin 0 is by far the fullest: counted in a register
  read_groups(L.resid, L.vec_ok != 0u, p.begin, p.end, [&](const float (&a)[4], uint32_t nvalid, uint32_t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (static_cast<uint32_t>(j) < nvalid) {
        const uint32_t b = bin_of(fabsf(a[j]), M.mean, M.span, inv);
        if (b != 0u) atomicAdd(&lds_hist[b], 1u);
        else ++below;
      }
    }
  });
  if (below) atomicAdd(&lds_hist[0], below);
  __syncthreads();
  uint32_t* hist = A.hist + static_cast<size_t>(l) * kHistBins;
  for (uint32_t b = threadIdx.x; b < kSteps; b += kBlockThreads) {
    const uint32_t c = lds_hist[b];
    if (c) atomicAdd(&hist[b], c);
  }
}

// ------------------------------------------------------------------ the threshold search (Section 2.1, Algorithm 3)
// One workgroup per layer; the number of elements above T(j) is the number of elements in the bins j .. 1023.
__global__ void __launch_bounds__(kBlockThreads) threshold_search_kernel(ThresholdArgs A) {
  __shared__ uint32_t above[kSteps + 1];
  __shared__ uint32_t part[kBlockThreads];
  const uint32_t l = blockIdx.x;
  const LayerDesc L = A.layers[l];
  uint32_t* hist = A.hist + static_cast<size_t>(l) * kHistBins;
  // suffix sums: thread t owns the bins 4t .. 4t+3 (and leaves them zero: the exact path, which
  // shares the array, expects it cleared)
  constexpr uint32_t kPer = kSteps / kBlockThreads;
  uint32_t h[kPer], mine = 0u;
#pragma unroll
  for (uint32_t i = 0; i < kPer; ++i) {
    h[i] = hist[threadIdx.x * kPer + i];
    hist[threadIdx.x * kPer + i] = 0u;
    mine += h[i];
  }
  part[threadIdx.x] = mine;
  __syncthreads();
  if (threadIdx.x == 0u) {
    uint32_t run = 0u;
    for (int t = kBlockThreads - 1; t >= 0; --t) { const uint32_t v = part[t]; part[t] = run; run += v; }   // bins of higher threads
  }
  __syncthreads();
  uint32_t run = part[threadIdx.x];
#pragma unroll
  for (int i = static_cast<int>(kPer) - 1; i >= 0; --i) { run += h[i]; above[threadIdx.x * kPer + static_cast<uint32_t>(i)] = run; }
  __syncthreads();
  if (threadIdx.x == 0u) {
    // The search interval of Algorithm 3 starts as [0, 1] and is halved until it is 2^-10 wide, so its ends and
    // midpoints are the multiples j / 1024 and the bisection can run on the integers j: [lo, hi] starts as
    // [0, 1024], every midpoint is exact, and at most ten thresholds T(j) are tried.  More than k but fewer than
    // 2k elements above T(j) end the search; k or fewer mean the threshold has to come down (hi = j), otherwise up.
    ThresholdMoments M = A.moments[l];
    const unsigned long long k = L.k;
    uint32_t lo = 0u, hi = kSteps, counts = 0u;
    float thr = 0.0f;
    while (hi - lo > 1u) {
      const uint32_t j = lo + (hi - lo) / 2u;
      thr = threshold_at(M.mean, M.span, j);
      const unsigned long long nnz = above[j];
      ++counts;
      if (nnz > k && nnz < 2ull * k) break;
      if (nnz <= k) hi = j; else lo = j;
    }
    *as_global(A.thresholds + l) = thr;
    A.moments[l].counts_taken = counts;
  }
}

// ------------------------------------------------------------------ count, offsets, emit
template <bool kReverse>
__global__ void __launch_bounds__(kBlockThreads) threshold_count_kernel(ThresholdArgs A) {
  const uint32_t wg = (kReverse != (A.reverse != 0u)) ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  const Place p = place_of(A, L, l, wg);
  if (p.begin == p.end) return;
  const float thr = *as_global(A.thresholds + l);
  uint32_t cnt = 0u;
  read_groups(L.resid, L.vec_ok != 0u, p.begin, p.end, [&](const float (&a)[4], uint32_t nvalid, uint32_t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) cnt += (static_cast<uint32_t>(j) < nvalid && fabsf(a[j]) > thr) ? 1u : 0u;
  });
  const uint32_t total = wave_total(wave_incl_scan(cnt));
  if (lane_id() == 0u) A.counts[p.wc] = total;
}

// One workgroup per layer: the wave-chunk counts become the wave-chunks' first output positions.
__global__ void __launch_bounds__(kBlockThreads) threshold_offsets_kernel(ThresholdArgs A) {
  __shared__ uint32_t lds_scan[kWavesPerBlock];
  const uint32_t l = blockIdx.x;
  const LayerDesc L = A.layers[l];
  uint32_t* c = A.counts + L.wc_first;
  constexpr uint32_t kItems = 8;          // independent loads in flight per thread: this is a serial step
  uint32_t carry = 0u;
  for (uint32_t base = 0; base < L.wc_count; base += kBlockThreads * kItems) {
    const uint32_t i0 = base + threadIdx.x * kItems;
    uint32_t v[kItems], sum = 0u;
#pragma unroll
    for (uint32_t j = 0; j < kItems; ++j) {
      v[j] = (i0 + j < L.wc_count) ? c[i0 + j] : 0u;
      sum += v[j];
    }
    uint32_t total;
    uint32_t ex = carry + block_excl_scan(sum, lds_scan, total);
#pragma unroll
    for (uint32_t j = 0; j < kItems; ++j) {
      if (i0 + j < L.wc_count) c[i0 + j] = ex;
      ex += v[j];
    }
    carry += total;
  }
  if (threadIdx.x == 0u) {
    const uint32_t cap = 2u * L.k;
    *as_global(L.out_count) = static_cast<int32_t>(carry < cap ? carry : cap);
    if (A.nnz) *as_global(A.nnz + l) = static_cast<int32_t>(carry);
  }
}

// kLists: the accumulate pass of this call left the elements above the threshold in the wave-chunk
// lists; a wave-chunk whose list holds them all is written from it, without another look at V.
template <bool kReverse, bool kLists>
__global__ void __launch_bounds__(kBlockThreads) threshold_emit_kernel(ThresholdArgs A) {
  const uint32_t wg = (kReverse != (A.reverse != 0u)) ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  const Place p = place_of(A, L, l, wg);
  if (p.begin == p.end) return;
  const uint32_t cap = 2u * L.k;
  uint32_t out_pos = A.counts[p.wc];
  if (out_pos >= cap) return;                      // the buffer is full: the rest stays in the residual
  const bool clear_mom = (L.mom != nullptr) && A.mask_momentum;
  const gptr<int32_t> out_idx = as_global(L.out_idx);
  const gptr<float> out_val = as_global(L.out_val);
  const gptr<float> resid = as_global(L.resid);
  const gptr<float> mom = as_global(L.mom);
  if constexpr (kLists) {
    const uint32_t listed = A.listed[p.wc];
    if (listed <= A.cap) {
      const gptr<const vu2> slot = as_global(reinterpret_cast<const vu2*>(A.slots + static_cast<size_t>(p.wc) * A.cap));
      for (uint32_t i = lane_id(); i < listed; i += kWaveSize) {
        const uint32_t pos = out_pos + i;
        if (pos < cap) {
          const vu2 e = slot[i];
          out_idx[pos] = static_cast<int32_t>(e.y);
          out_val[pos] = __uint_as_float(e.x);
          mask_store(resid + e.y);
          if (clear_mom) mask_store(mom + e.y);
        }
      }
      return;
    }
  }
  const float thr = *as_global(A.thresholds + l);
  read_groups(L.resid, L.vec_ok != 0u, p.begin, p.end, [&](const float (&a)[4], uint32_t nvalid, uint32_t idx0) {
    bool sel[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) sel[j] = static_cast<uint32_t>(j) < nvalid && fabsf(a[j]) > thr;
    const unsigned long long s0 = __ballot(sel[0]), s1 = __ballot(sel[1]), s2 = __ballot(sel[2]), s3 = __ballot(sel[3]);
    if ((s0 | s1 | s2 | s3) == 0ull) return;
    uint32_t pos = out_pos + rank_below(s0) + rank_below(s1) + rank_below(s2) + rank_below(s3);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (sel[j]) {
        if (pos < cap) {
          out_idx[pos] = static_cast<int32_t>(idx0 + j);
          out_val[pos] = a[j];
          mask_store(resid + idx0 + j);
          if (clear_mom) mask_store(mom + idx0 + j);
        }
        ++pos;
      }
    }
    out_pos += popc64(s0) + popc64(s1) + popc64(s2) + popc64(s3);
  });
}

hipError_t launch_threshold_compress(const ThresholdArgs& a, uint32_t num_wgs, uint32_t num_layers, hipStream_t s) {
  const dim3 block(kBlockThreads);
#define RGC_LAUNCHED() do { hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return e_; } while (0)
  // Each pass over the tensors runs against the direction of the one before it: what that one touched last
  // (still in the memory-side cache) is read first.  a.reverse turns the whole sequence round.
  if (a.search) {
    hipLaunchKernelGGL((threshold_accumulate_kernel<false, false>), dim3(num_wgs), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL(threshold_moments_kernel, dim3(num_layers), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL(threshold_histogram_kernel<true>, dim3(num_wgs), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL(threshold_search_kernel, dim3(num_layers), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL(threshold_count_kernel<false>, dim3(num_wgs), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL(threshold_offsets_kernel, dim3(num_layers), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL((threshold_emit_kernel<true, false>), dim3(num_wgs), block, 0, s, a);
  } else {
    hipLaunchKernelGGL((threshold_accumulate_kernel<true, false>), dim3(num_wgs), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL(threshold_offsets_kernel, dim3(num_layers), block, 0, s, a);
    RGC_LAUNCHED();
    hipLaunchKernelGGL((threshold_emit_kernel<true, true>), dim3(num_wgs), block, 0, s, a);
  }
#undef RGC_LAUNCHED
  return hipGetLastError();
}

}  // namespace rgc
