// gfx950 kernels of the compression step (RedSync, Algorithm 1, inner loop over layers):
//   V += G (or the momentum-corrected form of Section 2.5), exact top-k selection by
//   magnitude (Section 2.1 defines the communication-set as the top 0.1 % of each layer),
//   packing into (index, value) messages (Sections 2.2 / 2.3) and masking of the residual.
//
// Work decomposition: a layer is cut into wave-chunks of `chunk` consecutive elements; one
// wave64 owns one wave-chunk, four waves form a workgroup, all layers of a call share one
// launch (workgroup -> layer through a table).  A wave keeps everything it emits in ascending
// index order using ballot + popcount ranks, so every list below is ordered without a sort.
//
// Two ways to the same result:
//  * hinted, one pass over G/V: the streaming pass appends every element whose magnitude key
//    is >= a cached threshold tau to its wave-chunk's candidate list and counts candidates in
//    a coarse histogram of (key - tau).  If at least k candidates were seen and no list
//    overflowed, the exact k-th key is found among the candidates (PH_SEL) and the message is
//    written from the lists (PH_OUT_C).  tau only decides speed: a bad tau is detected and the
//    layer falls back to
//  * multi-pass radix select: three histogram passes over 12+12+7 key bits give the exact
//    k-th key T and the number r of admitted ties, a counting pass and an ordered-compaction
//    pass write the message (lowest indices win among keys equal to T).
// Per layer decisions are taken by the last workgroup of the layer to finish a phase (a two-level
// election with device-scope atomic counters; what it reads was written with device-scope stores, so no
// fence, no host round trip and no spinning is needed).
#include "rgc_exact.h"

#include <mutex>

#include "../../include/rgc.h"

#ifndef RGC_RECOMPUTE_UNROLL
#define RGC_RECOMPUTE_UNROLL 2
#endif

namespace rgc {

namespace {

typedef uint32_t vu2 __attribute__((ext_vector_type(2))); // a candidate: (float bits, index)

struct Collector {
  gptr<vu2> slot;    // this wave-chunk's candidate list
  uint32_t* coarse;  // the workgroup's coarse histogram in LDS (flushed when the workgroup ends)
  uint32_t cap;
  uint32_t count;    // candidates seen so far (wave-uniform)
  uint32_t tau;
  uint32_t shift;
  uint32_t sign_xor, sign_filter;   // see key_of()
  uint32_t clip;     // dense layers: candidates of the coarse bins from this one upwards are masked by the streaming pass itself
};

// The selection key of an element with bit pattern `bits`.  Plain top-k (Section 2.1): its
// magnitude, sign bit cleared.  Alternating Signs Quantization (Section 2.2: the k largest
// elements in one iteration, the k smallest in the next): the magnitude of the elements that
// carry the iteration's sign bit, 0 for all others, which thereby rank last and equal.
//   sign_filter = 0:                      key = bits & 0x7FFFFFFF
//   sign_filter = ~0, sign_xor = 0:       key = sign bit clear ? bits              : 0   (largest)
//   sign_filter = ~0, sign_xor = 1 << 31: key = sign bit set   ? bits & 0x7FFFFFFF : 0   (smallest)
// One AND with a wave-uniform mask, one XOR, one signed maximum: after the XOR the elements of the
// other sign are the negative integers.
__device__ __forceinline__ uint32_t key_of(uint32_t bits, uint32_t sign_xor, uint32_t sign_filter) {
  const int32_t t = static_cast<int32_t>((bits & (kKeyMask | sign_filter)) ^ sign_xor);
  return static_cast<uint32_t>(t > 0 ? t : 0);
}

// The key of the multi-pass selection.  Plain top-k: the magnitude key (31 bits).  Alternating Signs
// Quantization: a 32-bit key that grows with the value of the element (largest) or of its negative
// (smallest), both zeros being one value: the order "by value" that Section 2.2 words, also for a layer
// with fewer than k elements of the expected sign (its zeros come next, then the elements of the other
// sign closest to zero).  For the elements that key_of() ranks (expected sign, not zero) the two keys
// agree up to the top bit: ordered = key_of | 0x80000000; every other element lies below 0x80000000.
__device__ __forceinline__ uint32_t ordered_key(uint32_t bits, uint32_t sign_xor, uint32_t sign_filter) {
  if (sign_filter == 0u) return bits & kKeyMask;
  uint32_t b = bits ^ sign_xor;
  b = (b & kKeyMask) == 0u ? 0u : b;
  const uint32_t neg = static_cast<uint32_t>(static_cast<int32_t>(b) >> 31);
  return b ^ (neg | 0x80000000u);
}

// Digits of the multi-pass key: 12 + 12 + low bits, low = 7 (31-bit magnitude key) or 8 (32-bit ordered key).
__device__ __forceinline__ uint32_t low_bits_of(uint32_t sign_filter) { return sign_filter ? 8u : 7u; }

__device__ __forceinline__ uint32_t coarse_bin(uint32_t key, uint32_t tau, uint32_t shift) {
  const uint32_t b = (key - tau) >> shift;
  return b < static_cast<uint32_t>(kCoarseBins - 1) ? b : static_cast<uint32_t>(kCoarseBins - 1);
}

// Dense layers: the clip bin as the kernels use it (whatever the state holds).
__device__ __forceinline__ uint32_t dense_clip(uint32_t clip) {
  return clip < static_cast<uint32_t>(kCoarseBins - 1) ? clip : static_cast<uint32_t>(kCoarseBins - 1);
}
// Dense layers: the smallest key whose coarse bin is the clip bin or a higher one (clip <= kCoarseBins - 1, where
// coarse_bin() does not saturate yet); 2^31, which no key reaches, if there is none.
__device__ __forceinline__ uint32_t dense_clip_key(uint32_t tau, uint32_t shift, uint32_t clip) {
  const unsigned long long k = static_cast<unsigned long long>(tau) + (static_cast<unsigned long long>(clip) << shift);
  return k < 0x80000000ull ? static_cast<uint32_t>(k) : 0x80000000u;
}
// Dense layers: the key from which the streaming pass masks at once, as the kernels use it (whatever the state
// holds, only candidates are masked: they are the ones the lists can put back).
__device__ __forceinline__ uint32_t dense_mask_key(uint32_t mask_key, uint32_t tau) { return mask_key > tau ? mask_key : tau; }
// ... and where the next call's k-th key is expected: as far above the new threshold as this call's k-th key T lies
// above the (undrifted) threshold tn of the same rank.
__device__ __forceinline__ uint32_t mask_key_for(uint32_t T, uint32_t tn, uint32_t tau_new) {
  const unsigned long long k = static_cast<unsigned long long>(tau_new) + (T >= tn ? T - tn : 0u);
  return k < 0x80000000ull ? static_cast<uint32_t>(k) : 0x80000000u;
}
// Dense layers: a wave-chunk whose list could not be sure to hold another group stores this bit with the number of
// entries it had listed by then (as a count that is beyond every capacity, so the layer's hint counts as missed).
constexpr uint32_t kListStopped = 0x80000000u;

// Consume the four accumulated values a lane holds (elements idx0 .. idx0+3, the first
// `nvalid` of which exist).  Element order inside the wave is lane-major.
template <bool kCollect>
__device__ __forceinline__ void consume(const float (&a)[4], uint32_t nvalid, uint32_t idx0,
                                        Collector& c, uint32_t* lds_hist, uint32_t& zeros) {
  uint32_t bits[4], key[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    bits[j] = fbits(a[j]);
    key[j] = key_of(bits[j], c.sign_xor, c.sign_filter);
  }
  if constexpr (kCollect) {
    bool f[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) f[j] = (static_cast<uint32_t>(j) < nvalid) && (key[j] >= c.tau);
    const unsigned long long any = __ballot(f[0] | f[1] | f[2] | f[3]);
    if (any != 0ull) {
      const unsigned long long m0 = __ballot(f[0]), m1 = __ballot(f[1]), m2 = __ballot(f[2]),
                               m3 = __ballot(f[3]);
      uint32_t pos = c.count + rank_below(m0) + rank_below(m1) + rank_below(m2) + rank_below(m3);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (f[j]) {
          if (pos < c.cap) {
            c.slot[pos] = vu2{bits[j], idx0 + j};
            atomicAdd(&c.coarse[coarse_bin(key[j], c.tau, c.shift)], 1u);
          }
          ++pos;
        }
      }
      c.count += popc64(m0) + popc64(m1) + popc64(m2) + popc64(m3);
    }
  } else {
    const uint32_t sh1 = low_bits_of(c.sign_filter) + 12u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (static_cast<uint32_t>(j) < nvalid) {
        if ((bits[j] & kKeyMask) != 0u) atomicAdd(&lds_hist[ordered_key(bits[j], c.sign_xor, c.sign_filter) >> sh1], 1u);
        else ++zeros;            // the zeros of a sparse tensor would all hit one bin: counted in a register
      }
    }
  }
}

// The first-digit bin of the value zero (where the zeros counted in registers are added).
__device__ __forceinline__ uint32_t zero_bin(uint32_t sign_xor, uint32_t sign_filter) {
  return ordered_key(0u, sign_xor, sign_filter) >> (low_bits_of(sign_filter) + 12u);
}

// Streaming pass over one wave-chunk [begin, end) of a layer.
template <bool kMom, bool kCollect, bool kNest = false>
__device__ __forceinline__ void stream_chunk(const LayerDesc& L, uint32_t begin, uint32_t end,
                                             const AccumRule m, Collector& c, uint32_t* lds_hist) {
  const uint32_t lane = lane_id();
  uint32_t zeros = 0;
  uint32_t base = begin;
  if (L.vec_ok) {
    const uint32_t nfull = (end - begin) / kGroupElems;
    const gptr<const vf4> G4 = as_global(reinterpret_cast<const vf4*>(L.grad + begin));
    const gptr<vf4> V4 = as_global(reinterpret_cast<vf4*>(L.resid + begin));
    const gptr<vf4> U4 = as_global(kMom ? reinterpret_cast<vf4*>(L.mom + begin) : nullptr);
    constexpr uint32_t kUnroll = kMom ? 2u : 4u;   // 16-byte loads in flight per lane: 6 or 8
    uint32_t g = 0;
    for (; g + kUnroll <= nfull; g += kUnroll) {
      vf4 gv[kUnroll], vv[kUnroll], uv[kUnroll];
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) {
        const uint32_t o = (g + t) * kWaveSize + lane;
        gv[t] = __builtin_nontemporal_load(&G4[o]);
        vv[t] = V4[o];
        if constexpr (kMom) uv[t] = U4[o];
      }
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) {
        const uint32_t o = (g + t) * kWaveSize + lane;
        const float gg[4] = {gv[t].x, gv[t].y, gv[t].z, gv[t].w};
        const float vvv[4] = {vv[t].x, vv[t].y, vv[t].z, vv[t].w};
        float uu[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (kMom) { uu[0] = uv[t].x; uu[1] = uv[t].y; uu[2] = uv[t].z; uu[3] = uv[t].w; }
        float a[4];
        accum4<kMom, kNest>(gg, vvv, uu, m, a);
        V4[o] = vf4{a[0], a[1], a[2], a[3]};
        if constexpr (kMom) U4[o] = vf4{uu[0], uu[1], uu[2], uu[3]};
        consume<kCollect>(a, 4u, begin + o * 4u, c, lds_hist, zeros);
      }
    }
    for (; g < nfull; ++g) {
      const uint32_t o = g * kWaveSize + lane;
      const vf4 gq = __builtin_nontemporal_load(&G4[o]);
      const vf4 vq = V4[o];
      const float gg[4] = {gq.x, gq.y, gq.z, gq.w};
      const float vvv[4] = {vq.x, vq.y, vq.z, vq.w};
      float uu[4] = {0.f, 0.f, 0.f, 0.f};
      if constexpr (kMom) { const vf4 uq = U4[o]; uu[0] = uq.x; uu[1] = uq.y; uu[2] = uq.z; uu[3] = uq.w; }
      float a[4];
      accum4<kMom, kNest>(gg, vvv, uu, m, a);
      V4[o] = vf4{a[0], a[1], a[2], a[3]};
      if constexpr (kMom) U4[o] = vf4{uu[0], uu[1], uu[2], uu[3]};
      consume<kCollect>(a, 4u, begin + o * 4u, c, lds_hist, zeros);
    }
    base = begin + nfull * kGroupElems;
  }
  // scalar groups: the ragged tail of an aligned layer, or every group of an unaligned one
  const gptr<const float> Gs = as_global(L.grad);
  const gptr<float> Vs = as_global(L.resid);
  const gptr<float> Us = as_global(L.mom);
  for (; base < end; base += kGroupElems) {
    const uint32_t idx0 = base + lane * 4u;
    const uint32_t nvalid = idx0 < end ? ((end - idx0) < 4u ? (end - idx0) : 4u) : 0u;
    float gg[4] = {0.f, 0.f, 0.f, 0.f}, vvv[4] = {0.f, 0.f, 0.f, 0.f}, uu[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (static_cast<uint32_t>(j) < nvalid) {
        gg[j] = Gs[idx0 + j];
        vvv[j] = Vs[idx0 + j];
        if constexpr (kMom) uu[j] = Us[idx0 + j];
      }
    }
    float a[4];
    accum4<kMom, kNest>(gg, vvv, uu, m, a);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (static_cast<uint32_t>(j) < nvalid) {
        Vs[idx0 + j] = a[j];
        if constexpr (kMom) Us[idx0 + j] = uu[j];
      }
    }
    consume<kCollect>(a, nvalid, idx0, c, lds_hist, zeros);
  }
  if constexpr (!kCollect) {
    if (zeros) atomicAdd(&lds_hist[zero_bin(c.sign_xor, c.sign_filter)], zeros);
  }
}

// Read-only walk over one wave-chunk of the updated residual, four elements per lane per step,
// same element order as the streaming pass.  f(a[4], nvalid, idx0) must be wave-uniform code.
template <typename F>
__device__ __forceinline__ void for_each_group(const float* generic_p, bool vec, uint32_t begin,
                                               uint32_t end, F&& f) {
  const gptr<const float> p = as_global(generic_p);
  const uint32_t lane = lane_id();
  for (uint32_t base = begin; base < end; base += kGroupElems) {
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

__device__ __forceinline__ void flush_hist(const uint32_t* lds_hist, uint32_t* ghist, uint32_t bins) {
  for (uint32_t b = threadIdx.x; b < bins; b += kBlockThreads) {
    const uint32_t v = lds_hist[b];
    if (v) atomicAdd(&ghist[b], v);
  }
}

__device__ __forceinline__ uint32_t bit_length(uint32_t x) { return x ? 32u - __clz(x) : 0u; }

// Coarse-bin shift for the next call so that the k-th key lands in the second quarter of the
// coarse bins (kCoarseBins / 4 .. kCoarseBins / 2).
__device__ __forceinline__ uint32_t shift_for(uint32_t T, uint32_t tau) {
  const uint32_t d = T >= tau ? T - tau : 0u;
  const uint32_t bl = bit_length(d);
  constexpr uint32_t kKeep = 9u;   // log2(kCoarseBins / 2)
  static_assert(kCoarseBins == 1024, "kKeep is tied to the number of coarse bins");
  return bl > kKeep ? bl - kKeep : 0u;
}

// Dense layers: the ranking step of the next call looks at the keys from the hinted threshold tau up to twice as far
// above the k-th key T of this call as tau lies below it (in coarse bins of the next call's shift, as far as the
// bins reach); what lies above that is sure to be selected.  (A k-th key that rises costs a miss, one that falls
// only list entries, and the band costs an LDS atomic per candidate in it: hence the lopsided band.)
__device__ __forceinline__ uint32_t clip_for(uint32_t T, uint32_t tau, uint32_t shift) {
  const uint32_t d = T >= tau ? T - tau : 0u;
  const uint32_t b = 3u * (d >> shift) + 2u;
  return b < static_cast<uint32_t>(kCoarseBins - 1) ? b : static_cast<uint32_t>(kCoarseBins - 1);
}

// Threshold for the next call = rank-based estimate from this call + the observed drift of the
// k-th key between the last two calls (a steadily growing or shrinking residual moves the
// threshold by about the same amount every call).  Speed only.
__device__ __forceinline__ uint32_t drifted_tau(uint32_t tau_rank, uint32_t T, uint32_t T_prev, bool has_prev) {
  long long d = has_prev ? static_cast<long long>(T) - static_cast<long long>(T_prev) : 0ll;
  const long long lim = 1ll << 22;               // half an octave per call at most
  d = d > lim ? lim : (d < -lim ? -lim : d);
  if (d > 0) d -= d >> 3;                        // raising tau is the risky direction
  long long t = static_cast<long long>(tau_rank) + d;
  if (t < 0) t = 0;
  if (t > static_cast<long long>(kKeyMask)) t = kKeyMask;
  return static_cast<uint32_t>(t);
}

constexpr uint32_t kOffsetGroup = 64;   // wave-chunks whose output offsets one wave of PH_OUT_C derives by itself
static_assert(kOffsetGroup == kWaveSize, "one lane per wave-chunk of the group");

struct ResolveShared {
  uint32_t scan[4];
  uint32_t flag;
  uint32_t bin, above, cnt;     // bin holding the k-th key, keys above it, keys in it
  uint32_t hbin, hcum, hcnt;    // bin where the cumulative count reaches the hint's target rank
  uint32_t bad;
};

// Copy a (possibly replicated) global histogram into LDS, summing the replicas, and clear the
// global copy for its next use.  The global bins were filled with device-scope atomics, so they
// are read with device-scope loads; all loads of a thread are issued before the first use so
// that their round trips overlap (this runs on the critical path of a layer's last workgroup).
template <uint32_t kBins, uint32_t kReps>
__device__ __forceinline__ void stage_hist(uint32_t* g, uint32_t* lds) {
  constexpr uint32_t kPer = (kBins + kBlockThreads - 1) / kBlockThreads;
  constexpr uint32_t kBatch = (kPer * kReps > 16u) ? (16u / kReps ? 16u / kReps : 1u) : kPer;   // <= 16 loads in flight
  for (uint32_t i0 = 0; i0 < kPer; i0 += kBatch) {
    uint32_t v[kBatch][kReps];
#pragma unroll
    for (uint32_t i = 0; i < kBatch; ++i) {
      const uint32_t b = (i0 + i) * kBlockThreads + threadIdx.x;
#pragma unroll
      for (uint32_t rep = 0; rep < kReps; ++rep)
        v[i][rep] = (i0 + i < kPer && b < kBins) ? ld_agent(&g[rep * kBins + b]) : 0u;
    }
#pragma unroll
    for (uint32_t i = 0; i < kBatch; ++i) {
      const uint32_t b = (i0 + i) * kBlockThreads + threadIdx.x;
      if (i0 + i < kPer && b < kBins) {
        uint32_t sum = 0;
#pragma unroll
        for (uint32_t rep = 0; rep < kReps; ++rep) {
          sum += v[i][rep];
          g[rep * kBins + b] = 0u;
        }
        lds[b] = sum;
      }
    }
  }
  __syncthreads();
}

// Walk the LDS histogram from its top bin downwards and find the bins where the cumulative
// count first reaches want_k and want_h.  Results go to sh.{bin,above,cnt} and
// sh.{hbin,hcum,hcnt} (bin = ~0 when the total stays below the wanted count); returns the total.
// Kept light on registers: this code shares a kernel with the streaming loop.
__device__ uint32_t locate_from_top(const uint32_t* lds, uint32_t bins, uint32_t want_k, uint32_t want_h,
                                    ResolveShared& sh) {
  const uint32_t t = threadIdx.x;
  const uint32_t per = bins >= static_cast<uint32_t>(kBlockThreads) ? bins / kBlockThreads : 1u;
  const bool active = t * per < bins;
  uint32_t s = 0;
  if (active) {
#pragma unroll 1
    for (uint32_t i = 0; i < per; ++i) s += lds[bins - 1u - (t * per + i)];
  }
  if (t == 0) { sh.bin = 0xFFFFFFFFu; sh.hbin = 0xFFFFFFFFu; sh.above = 0; sh.cnt = 0; sh.hcum = 0; sh.hcnt = 0; }
  uint32_t total;
  const uint32_t ex = block_excl_scan(s, sh.scan, total);   // barriers inside: the init is visible
  if (active && ((ex < want_k && want_k <= ex + s) || (ex < want_h && want_h <= ex + s))) {
    uint32_t cum = ex;
#pragma unroll 1
    for (uint32_t i = 0; i < per; ++i) {
      const uint32_t b = bins - 1u - (t * per + i);
      const uint32_t h = lds[b];
      if (cum < want_k && cum + h >= want_k) { sh.bin = b; sh.above = cum; sh.cnt = h; }
      if (cum < want_h && cum + h >= want_h) { sh.hbin = b; sh.hcum = cum + h; sh.hcnt = h; }
      cum += h;
    }
  }
  __syncthreads();
  return total;
}

// Multi-pass path, one radix digit: the layer's histogram of this digit is complete.  Find the
// bin holding the k_rem-th largest key, update prefix / k_rem, derive the threshold hint for
// the next call on the way, clear the histogram, schedule the next phase.
// `lds` holds the bins of this level (kHistBins words, 128 at the last level) and is free for use.
template <int kLevel>
__device__ void resolve_digit(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st,
                              ResolveShared& sh, uint32_t* lds, uint32_t cur_launch) {
  constexpr uint32_t kBins = (kLevel == 3) ? 256u : static_cast<uint32_t>(kHistBins);   // the last digit has 7 or 8 bits
  const uint32_t low = low_bits_of(A.sign_filter);
  const uint32_t k_rem = (kLevel == 1) ? L.k : st->k_rem;
  const uint32_t above_scope = L.k - k_rem;          // keys above the current scope
  // The k entries selected now leave the residual, so the next call's top-k come from ranks
  // k+1.. of this call: aim the next threshold at rank 2k + margin.
  const uint32_t target = L.target;
  const uint32_t pending = (kLevel == 1) ? 1u : st->hint_pending;
  const uint32_t prefix = (kLevel == 1) ? 0u : st->prefix;
  stage_hist<kBins, 1u>(A.hist + static_cast<size_t>(l) * kHistBins, lds);
  (void)locate_from_top(lds, kBins, k_rem, target - above_scope, sh);
  if (threadIdx.x == 0) {
    if (sh.bin == 0xFFFFFFFFu) { atomicOr(A.errflag, 1u); sh.bin = 0; }
    const uint32_t D = sh.bin;
    const uint32_t hcum = above_scope + sh.hcum;
    auto edge = [&](uint32_t b) -> uint32_t {
      if (kLevel == 1) return b << (low + 12u);
      if (kLevel == 2) return (prefix << (low + 12u)) | (b << low);
      return (prefix << low) | b;
    };
    // ---- hint derivation (speed only)
    uint32_t pend = pending;
    if (pend == 1u) {
      if (sh.hbin == 0xFFFFFFFFu) {          // the whole layer holds fewer keys than the target rank
        st->tau_next = 0u; pend = 2u;
      } else if (hcum <= L.cmax) {
        st->tau_next = edge(sh.hbin); pend = 2u;
      } else if (sh.hbin == D) {
        pend = (kLevel < 3) ? 1u : 3u;      // refine inside the same bin, or give up (heavy ties)
      } else {
        st->tau_next = edge(sh.hbin + 1u); pend = 2u;   // one bin up: fewer keys than aimed at, still >= k
      }
    }
    const uint32_t new_rem = k_rem - sh.above;
    st->k_rem = new_rem;
    if (kLevel == 1) {
      st->prefix = D;
      st->next_phase = PH_HIST2;
      // A hint-free call needs no further digits if the keys from the first digit's bin upwards fit the
      // candidate lists: one more pass over the residual collects them (threshold = the bin's lower edge,
      // so at least k of them exist) and the call ends like a hinted one (PH_SEL, PH_OUT_C): two passes
      // less.  Only straight after the streaming pass (a call that already lost a launch to a missed hint
      // has too few launches left for the fall-back should a list overflow), and not for callers who asked
      // for the hints to be left alone (the collection uses the hint's fields).
      const uint32_t lower = edge(D);
      const bool in_key_space = A.sign_filter == 0u || lower > 0x80000000u;   // see ordered_key / key_of
      if (cur_launch == 1u && A.update_hints && L.hintable && in_key_space && sh.above + sh.cnt <= L.cmax) {
        const uint32_t tau = (lower & kKeyMask) ? (lower & kKeyMask) : 1u;
        st->tau = tau;
        st->shift = shift_for(tau + ((1u << (low + 12u)) - 1u), tau);
        st->next_phase = PH_COLLECT;
      }
    } else if (kLevel == 2) {
      st->prefix = (prefix << 12) | D;
      st->next_phase = PH_HIST3;
    } else {
      const uint32_t T = (prefix << low) | D;
      st->T = T;
      st->r = new_rem;
      st->next_phase = PH_COUNT;
      if (A.update_hints && L.dense && st->dense_skip != 0u) st->dense_skip -= 1u;   // one more call without its hint
      if (A.update_hints) {
        // The hints live in the key space of the one-pass path (key_of).  With the ordered key a hint
        // exists only if the k-th key and the threshold aimed at both lie among the elements key_of()
        // ranks (top bit set); a layer short of such elements has none and stays on this path.
        uint32_t Th = T, tn = st->tau_next;
        bool usable = (pend == 2u);
        if (A.sign_filter) {
          usable = usable && T > 0x80000000u && tn >= 0x80000000u;
          Th = T & kKeyMask;
          tn = (tn & kKeyMask) ? (tn & kKeyMask) : 1u;
        }
        if (usable) {
          st->tau = drifted_tau(tn, Th, st->T_prev, A.use_hints && st->has_prev);
          st->shift = shift_for(Th, tn);
          st->clip = clip_for(Th, tn, st->shift);
          st->mask_key = mask_key_for(Th, tn, st->tau);
          st->hint_valid = 1u;
          st->T_prev = Th;
          st->has_prev = 1u;
        } else {
          st->hint_valid = 0u;
          st->has_prev = A.sign_filter ? 0u : 1u;
          st->T_prev = Th;
        }
      }
    }
    st->hint_pending = pend;
    st->next_launch = cur_launch + 1u;
  }
}

// A dense layer's hint missed: a pass over the lists and five more passes for nothing, so the layer goes without its
// hint for a while, twice as long after every further miss.
__device__ __forceinline__ void dense_missed(LayerState* st) {
  const uint32_t wait = st->dense_backoff ? 2u * st->dense_backoff : 1u;
  st->dense_backoff = wait < kDenseBackoffMax ? wait : kDenseBackoffMax;
  st->dense_skip = st->dense_backoff + 1u;       // (the count-down at the end of this call's own fall-back included)
}

// Hinted path, end of the streaming pass: validate the candidate lists, locate the coarse bin
// holding the k-th key, clear the coarse histogram, schedule PH_SEL or fall back.
// `lds` holds >= kCoarseBins words and is free for use.
// `after_first_digit`: the lists come from PH_COLLECT of a hint-free call rather than from the streaming pass
// of a hinted one; should they not do, the call goes on with the second digit.
// `dense`: the lists are those of a dense layer's streaming pass (collect_kernel), which has already masked the
// candidates of the coarse bins from the layer's clip bin upwards: the k-th key must lie below that bin, and
// should it not, or should anything else be off, those entries are put back first (PH_RESTORE).
__device__ void resolve_collect(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st,
                                ResolveShared& sh, uint32_t* lds, bool after_first_digit, uint32_t cur_launch,
                                bool dense = false) {
  const uint32_t t = threadIdx.x;
  uint32_t total = 0, bad = 0;
  for (uint32_t c0 = 0; c0 < L.wc_count; c0 += 8u * kBlockThreads) {
    uint32_t v[8];
#pragma unroll
    for (uint32_t j = 0; j < 8u; ++j) {
      const uint32_t c = c0 + j * kBlockThreads + t;
      v[j] = c < L.wc_count ? ld_agent(&A.cand_cnt[L.wc_first + c]) : 0u;
    }
#pragma unroll
    for (uint32_t j = 0; j < 8u; ++j) {
      bad |= (v[j] > (dense ? L.list_cap : A.cap)) ? 1u : 0u;
      total += v[j];
    }
  }
  uint32_t cand_total;
  (void)block_excl_scan(total, sh.scan, cand_total);
  bad = __syncthreads_or(static_cast<int>(bad)) ? 1u : 0u;
  stage_hist<kCoarseBins, kCoarseRep>(A.coarse + static_cast<size_t>(l) * kCoarseRep * kCoarseBins, lds);
  const uint32_t k = L.k, target = L.target;   // see resolve_digit
  const uint32_t hist_total = locate_from_top(lds, kCoarseBins, k, target, sh);
  // PH_SEL adds the selected counts of every kOffsetGroup wave-chunks up in wc_b: start from zero
  for (uint32_t g = t; g < (L.wc_count + kOffsetGroup - 1u) / kOffsetGroup; g += kBlockThreads)
    st_agent(&A.wc_b[L.wc_first + g], 0u);
  if (dense && t < kMemberLists) st_agent(&A.shard_cnt[(static_cast<size_t>(l) * kMemberLists + t) * kShardStride], 0u);
  if (t == 0) {
    if (dense) {
      st->cur_tau = st->tau;
      st->cur_shift = st->shift;
      st->cur_mask_key = dense_mask_key(st->mask_key, st->tau);
    }
    st->stat_candidates = cand_total;
    st->stat_members = sh.cnt;
    const bool ok = !bad && cand_total >= k && hist_total == cand_total && sh.bin != 0xFFFFFFFFu &&
                    sh.cnt <= (dense ? L.mem_cap / 4u : static_cast<uint32_t>(kMemberMax)) && (!dense || sh.bin < dense_clip(st->clip));
    if (ok) {
      const uint32_t tau = st->tau, shift = st->shift;
      st->bstar = sh.bin;
      st->k_rem = k - sh.above;
      st->nmembers = 0u;
      if (!after_first_digit) st->path = 0u;
      st->next_phase = dense ? PH_SEL2 : PH_SEL;
      unsigned long long tn;
      if (sh.hbin != 0xFFFFFFFFu) {
        tn = static_cast<unsigned long long>(tau) + (static_cast<unsigned long long>(sh.hbin) << shift);
        if (tn > kKeyMask) tn = kKeyMask;
      } else {
        // the lists end above rank 2k + margin: extend tau downwards assuming the key density
        // seen between rank k and the end of the lists (it grows further down, so this errs
        // towards more candidates)
        const unsigned long long d = (static_cast<unsigned long long>(sh.bin) + 1ull) << shift;
        const unsigned long long have = cand_total > k ? cand_total - k : 1u;
        const unsigned long long need = target - cand_total;
        const unsigned long long delta = (d * need + have - 1ull) / have + 1ull;
        tn = delta < tau ? tau - delta : 0ull;
      }
      st->tau_next = static_cast<uint32_t>(tn);
    } else if (after_first_digit) {
      st->next_phase = PH_HIST2;          // prefix and k_rem are still those of the first digit
    } else if (dense) {
      st->path = 2u;
      st->stat_misses += 1u;
      st->next_phase = PH_RESTORE;        // the multi-pass path on the restored residual
      dense_missed(st);
    } else {
      st->path = 2u;
      st->stat_misses += 1u;
      st->next_phase = PH_HIST1;
    }
    st->next_launch = cur_launch + 1u;
  }
}

// In-place exclusive scan over the per wave-chunk counters of one layer (one workgroup).
// with_ties: a[] = keys > T, b[] = keys == T  ->  a[] = output offset of the chunk
//            (= prefix(a) + min(prefix(b), r)), b[] = prefix(b).
__device__ void scan_chunks(uint32_t* a, uint32_t* b, uint32_t count, uint32_t r, bool with_ties,
                            uint32_t* lds_scan, uint32_t* out_total) {
  constexpr uint32_t kItems = 16;   // many independent device-scope loads in flight per thread: this is a serial step
  uint32_t carry_a = 0, carry_b = 0;
  for (uint32_t base = 0; base < count; base += kBlockThreads * kItems) {
    uint32_t va[kItems], vb[kItems];
    uint32_t sa = 0, sb = 0;
    const uint32_t i0 = base + threadIdx.x * kItems;
#pragma unroll
    for (uint32_t j = 0; j < kItems; ++j) {
      va[j] = (i0 + j < count) ? ld_agent(&a[i0 + j]) : 0u;
      vb[j] = (with_ties && i0 + j < count) ? ld_agent(&b[i0 + j]) : 0u;
      sa += va[j];
      sb += vb[j];
    }
    uint32_t ta, tb = 0;
    uint32_t ea = block_excl_scan(sa, lds_scan, ta) + carry_a;
    uint32_t eb = 0;
    if (with_ties) eb = block_excl_scan(sb, lds_scan, tb) + carry_b;
#pragma unroll
    for (uint32_t j = 0; j < kItems; ++j) {
      if (i0 + j < count) {
        if (with_ties) {
          a[i0 + j] = ea + (eb < r ? eb : r);
          b[i0 + j] = eb;
        } else {
          a[i0 + j] = ea;
        }
      }
      ea += va[j];
      eb += vb[j];
    }
    carry_a += ta;
    carry_b += tb;
  }
  if (threadIdx.x == 0) *out_total = carry_a + (with_ties ? (carry_b < r ? carry_b : r) : 0u);
}

// The kk-th largest (1-based) of the m distinct 64-bit values v[0..m) in LDS, by radix selection
// from the top byte in which the values differ at all (the members of one coarse bin share
// their leading bytes) downwards: a 256-bin histogram of the values that match the bytes fixed
// so far, a scan from the top bin, the next byte; stops as soon as one value is left.  One
// barrier per byte: every wave scans the finished histogram for itself (four bins a lane), and
// three histograms take turns, the one two bytes ahead being cleared meanwhile.  (A bitonic
// sort of the same values took 55 dependent LDS round trips.)  All threads of the workgroup call
// it; hist holds 3 * 256 words.
static_assert(kBlockThreads == 256, "one thread per histogram bin");   // (PH_SEL also counts on hist holding 3 * kBlockThreads words)
__device__ unsigned long long select_kth_largest(const unsigned long long* v, uint32_t m, uint32_t kk,
                                                 uint32_t* hist, ResolveShared& sh) {
  const uint32_t t = threadIdx.x, lane = lane_id();
  const unsigned long long v0 = v[0];
  unsigned long long diff = 0ull;
  for (uint32_t i = t; i < m; i += kBlockThreads) diff |= v[i] ^ v0;
  int top = diff ? 63 - __clzll(static_cast<long long>(diff)) : -1;   // highest differing bit this thread saw
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int other = __shfl_xor(top, o);
    top = other > top ? other : top;
  }
  if (lane == 0) sh.scan[t >> 6] = static_cast<uint32_t>(top + 1);
  hist[t] = 0u; hist[256u + t] = 0u; hist[512u + t] = 0u;
  __syncthreads();
  {
    const uint32_t a = sh.scan[0], b = sh.scan[1], c = sh.scan[2], d = sh.scan[3];
    const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
    top = static_cast<int>(ab > cd ? ab : cd) - 1;
  }
  if (top < 0) return v0;                                   // a single value
  int shift = (top >> 3) << 3;
  unsigned long long prefix = shift == 56 ? 0ull : (v0 & (~0ull << (shift + 8)));
  for (uint32_t pass = 0;; ++pass, shift -= 8) {
    uint32_t* const H = hist + (pass % 3u) * 256u;
    const unsigned long long himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
    for (uint32_t i = t; i < m; i += kBlockThreads) {
      const unsigned long long x = v[i];
      if ((x & himask) == prefix) atomicAdd(&H[static_cast<uint32_t>(x >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[((pass + 2u) % 3u) * 256u + t] = 0u;
    // each wave for itself: lane L holds bins 4L .. 4L+3
    const uint32_t h0 = H[4u * lane], h1 = H[4u * lane + 1u], h2 = H[4u * lane + 2u], h3 = H[4u * lane + 3u];
    const uint32_t mine = h0 + h1 + h2 + h3;
    const uint32_t incl = wave_incl_scan(mine);
    const uint32_t higher = wave_total(incl) - incl;        // values in the bins of higher lanes
    const bool here = higher < kk && kk <= higher + mine;
    uint32_t bin = 0, above = 0, cnt = 0;
    if (here) {
      uint32_t a = higher;
      if (kk <= a + h3) { bin = 3u; cnt = h3; }
      else { a += h3; if (kk <= a + h2) { bin = 2u; cnt = h2; }
      else { a += h2; if (kk <= a + h1) { bin = 1u; cnt = h1; }
      else { a += h1; bin = 0u; cnt = h0; } } }
      bin += 4u * lane;
      above = a;
    }
    const unsigned long long who = __ballot(here);          // exactly one lane when 1 <= kk <= values in scope
    const int src = who ? static_cast<int>(__ffsll(static_cast<long long>(who))) - 1 : 0;
    bin = static_cast<uint32_t>(__shfl(static_cast<int>(bin), src));
    above = static_cast<uint32_t>(__shfl(static_cast<int>(above), src));
    cnt = static_cast<uint32_t>(__shfl(static_cast<int>(cnt), src));
    prefix |= static_cast<unsigned long long>(bin) << shift;
    kk -= above;
    if (shift == 0) return prefix;
    if (cnt <= 1u) break;
  }
  // one value is left under these leading bytes: whoever holds it tells the others
  const unsigned long long lomask = ~0ull << shift;
  for (uint32_t i = t; i < m; i += kBlockThreads) {
    const unsigned long long x = v[i];
    if ((x & lomask) == prefix) { sh.hbin = static_cast<uint32_t>(x); sh.hcum = static_cast<uint32_t>(x >> 32); }
  }
  __syncthreads();
  const unsigned long long r = (static_cast<unsigned long long>(sh.hcum) << 32) | sh.hbin;
  __syncthreads();
  return r;
}

__device__ __forceinline__ unsigned long long composite(uint32_t key, uint32_t idx) {
  return (static_cast<unsigned long long>(key) << 32) | static_cast<unsigned long long>(0xFFFFFFFFu - idx);
}

}  // namespace

// =================================================================== launch 1: streaming pass
__global__ void __launch_bounds__(kBlockThreads) accumulate_kernel(CompressArgs A) {
  __shared__ uint32_t lds_hist[kHistBins];
  __shared__ ResolveShared sh;
  // Every other call walks through the tensors from the end: when calls follow each other closely,
  // what the previous one wrote last (the tails of V and u, still in the memory-side cache) is what
  // this one reads first.
  const uint32_t wg = A.reverse ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  LayerState* st = A.state + l;
  // (with a sign filter a threshold of 0 would let the elements that key_of() ranks last and equal into the lists)
  const bool hinted = A.use_hints && (st->hint_valid != 0u) && !(A.sign_filter != 0u && st->tau == 0u);
  if (A.dense_ok && L.dense && hinted && st->dense_skip == 0u) return;     // collect_kernel has this layer
  const bool collect = hinted && L.hintable;
  // the same LDS array serves as 4096-bin digit histogram (hint-free) or 1024-bin coarse one
  const uint32_t lds_bins = collect ? static_cast<uint32_t>(kCoarseBins) : static_cast<uint32_t>(kHistBins);
  for (uint32_t b = threadIdx.x; b < lds_bins; b += kBlockThreads) lds_hist[b] = 0u;
  __syncthreads();
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + wave;
  if (wc_local < L.wc_count) {
    const uint32_t begin = wc_local * A.chunk;
    const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
    Collector c;
    c.slot = as_global(reinterpret_cast<vu2*>(A.slots + static_cast<size_t>(L.wc_first + wc_local) * A.cap));
    c.coarse = lds_hist;
    c.cap = A.cap;
    c.count = 0;
    c.tau = st->tau;
    c.shift = st->shift;
    c.sign_xor = A.sign_xor;
    c.sign_filter = A.sign_filter;
    const bool mom = (L.mom != nullptr);
    AccumRule rule;
    rule.m = A.m;
    rule.scale = A.grad_scale ? *as_global(A.grad_scale) : 1.0f;
    if (collect) {
      if (!mom) stream_chunk<false, true>(L, begin, end, rule, c, lds_hist);
      else if (!A.nesterov) stream_chunk<true, true>(L, begin, end, rule, c, lds_hist);
      else stream_chunk<true, true, true>(L, begin, end, rule, c, lds_hist);
      if (lane_id() == 0) st_agent(&A.cand_cnt[L.wc_first + wc_local], c.count);
    } else {
      if (!mom) stream_chunk<false, false>(L, begin, end, rule, c, lds_hist);
      else if (!A.nesterov) stream_chunk<true, false>(L, begin, end, rule, c, lds_hist);
      else stream_chunk<true, false, true>(L, begin, end, rule, c, lds_hist);
    }
  }
  __syncthreads();
  if (collect) {
    // Global atomics only here, in one burst per workgroup: inside the streaming loop each one
    // would stall the wave's later loads behind the atomic's round trip.
    flush_hist(lds_hist, A.coarse + (static_cast<size_t>(l) * kCoarseRep + (wg & (kCoarseRep - 1))) * kCoarseBins,
               kCoarseBins);
  } else {
    flush_hist(lds_hist, A.hist + static_cast<size_t>(l) * kHistBins, kHistBins);
  }
  if (last_block_of_layer(&st->done, A.group_done + L.grp_first, wg - L.wg_first, L.wg_count, &sh.flag)) {
    if (collect) {
      resolve_collect(A, l, L, st, sh, lds_hist, false, 1u);
    } else {
      if (threadIdx.x == 0) { st->path = 1u; st->stat_candidates = 0u; st->stat_members = 0u; }
      resolve_digit<1>(A, l, L, st, sh, lds_hist, 1u);
    }
  }
}

// =================================================================== launches 2..6: phases
namespace {

// PH_RESTORE, a dense layer whose hint missed: the entries its streaming pass masked on the strength of the hint
// (keys from the expected k-th key upwards) get their accumulated value and their velocity back from the wave-chunk's
// list; V and u are then exactly what an ordinary streaming pass leaves.  The wave goes on to the first digit's
// histogram of the same wave-chunk at once (phase_hist<1>), which reads what it has just written.
__device__ void dense_restore(const CompressArgs& A, const LayerDesc& L, const LayerState* st, uint32_t wc_local) {
  if (wc_local < L.wc_count) {
    const uint32_t mask_key = st->cur_mask_key;
    const bool clear_mom = (L.mom != nullptr) && A.mask_momentum;
    const gptr<float> resid = as_global(L.resid);
    const gptr<float> mom = as_global(L.mom);
    const size_t list = L.list_first + static_cast<size_t>(wc_local) * L.list_cap;
    const gptr<const vu2> slot = as_global(reinterpret_cast<const vu2*>(A.slots2 + list));
    const gptr<const float> slot_u = as_global(static_cast<const float*>(A.slots_u + list));
    uint32_t cnt = A.cand_cnt[L.wc_first + wc_local] & ~kListStopped;   // (a list that stopped early: what it held by then)
    cnt = cnt < L.list_cap ? cnt : L.list_cap;
    for (uint32_t p = lane_id(); p < cnt; p += kWaveSize) {
      const vu2 e = slot[p];
      const uint32_t key = key_of(e.x, A.sign_xor, A.sign_filter);
      if (key >= mask_key && e.y < L.n) {
        resid[e.y] = __uint_as_float(e.x);
        if (clear_mom) mom[e.y] = slot_u[p];
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the wave's stores have arrived before it reads the wave-chunk
}

template <int kLevel>
__device__ void phase_hist(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st, uint32_t wg,
                           uint32_t wc_local, uint32_t* lds_hist, ResolveShared& sh) {
  constexpr uint32_t kBins = (kLevel == 3) ? 256u : static_cast<uint32_t>(kHistBins);
  for (uint32_t b = threadIdx.x; b < kBins; b += kBlockThreads) lds_hist[b] = 0u;
  __syncthreads();
  const uint32_t prefix = st->prefix;
  const uint32_t low = low_bits_of(A.sign_filter), low_mask = (1u << low) - 1u;
  if (wc_local < L.wc_count) {
    const uint32_t begin = wc_local * A.chunk;
    const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
    uint32_t zeros = 0;
    for_each_group(L.resid, L.vec_ok != 0u, begin, end,
                   [&](const float (&a)[4], uint32_t nvalid, uint32_t) {
#pragma unroll
                     for (int j = 0; j < 4; ++j) {
                       if (static_cast<uint32_t>(j) < nvalid) {
                         const uint32_t bits = fbits(a[j]);
                         const uint32_t key = ordered_key(bits, A.sign_xor, A.sign_filter);
                         if (kLevel == 1) {
                           if ((bits & kKeyMask) != 0u) atomicAdd(&lds_hist[key >> (low + 12u)], 1u);
                           else ++zeros;
                         } else if (kLevel == 2) {
                           if ((key >> (low + 12u)) == prefix) atomicAdd(&lds_hist[(key >> low) & 0xFFFu], 1u);
                         } else {
                           if ((key >> low) == prefix) atomicAdd(&lds_hist[key & low_mask], 1u);
                         }
                       }
                     }
                   });
    if (kLevel == 1 && zeros) atomicAdd(&lds_hist[zero_bin(A.sign_xor, A.sign_filter)], zeros);
  }
  __syncthreads();
  flush_hist(lds_hist, A.hist + static_cast<size_t>(l) * kHistBins, kBins);
  if (last_block_of_layer(&st->done, A.group_done + L.grp_first, wg - L.wg_first, L.wg_count, &sh.flag)) resolve_digit<kLevel>(A, l, L, st, sh, lds_hist, A.launch);
}

// PH_COLLECT: the streaming pass's candidate collection, from the updated residual (see resolve_digit<1>).
__device__ void phase_collect(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st, uint32_t wg,
                              uint32_t wc_local, uint32_t* lds_hist, ResolveShared& sh) {
  for (uint32_t b = threadIdx.x; b < static_cast<uint32_t>(kCoarseBins); b += kBlockThreads) lds_hist[b] = 0u;
  __syncthreads();
  if (wc_local < L.wc_count) {
    const uint32_t begin = wc_local * A.chunk;
    const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
    Collector c;
    c.slot = as_global(reinterpret_cast<vu2*>(A.slots + static_cast<size_t>(L.wc_first + wc_local) * A.cap));
    c.coarse = lds_hist;
    c.cap = A.cap;
    c.count = 0;
    c.tau = st->tau;
    c.shift = st->shift;
    c.sign_xor = A.sign_xor;
    c.sign_filter = A.sign_filter;
    uint32_t zeros = 0;
    for_each_group(L.resid, L.vec_ok != 0u, begin, end,
                   [&](const float (&a)[4], uint32_t nvalid, uint32_t idx0) {
                     consume<true>(a, nvalid, idx0, c, lds_hist, zeros);
                   });
    if (lane_id() == 0) st_agent(&A.cand_cnt[L.wc_first + wc_local], c.count);
  }
  __syncthreads();
  flush_hist(lds_hist, A.coarse + (static_cast<size_t>(l) * kCoarseRep + (wg & (kCoarseRep - 1))) * kCoarseBins,
             kCoarseBins);
  if (last_block_of_layer(&st->done, A.group_done + L.grp_first, wg - L.wg_first, L.wg_count, &sh.flag))
    resolve_collect(A, l, L, st, sh, lds_hist, true, A.launch);
}

__device__ void phase_count(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st, uint32_t wg,
                            uint32_t wc_local, ResolveShared& sh) {
  const uint32_t T = st->T;
  if (wc_local < L.wc_count) {
    const uint32_t begin = wc_local * A.chunk;
    const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
    uint32_t gt = 0, eq = 0;
    for_each_group(L.resid, L.vec_ok != 0u, begin, end,
                   [&](const float (&a)[4], uint32_t nvalid, uint32_t) {
#pragma unroll
                     for (int j = 0; j < 4; ++j) {
                       if (static_cast<uint32_t>(j) < nvalid) {
                         const uint32_t key = ordered_key(fbits(a[j]), A.sign_xor, A.sign_filter);
                         gt += (key > T) ? 1u : 0u;
                         eq += (key == T) ? 1u : 0u;
                       }
                     }
                   });
    const uint32_t gt_all = wave_total(wave_incl_scan(gt));
    const uint32_t eq_all = wave_total(wave_incl_scan(eq));
    if (lane_id() == 0) {
      st_agent(&A.wc_a[L.wc_first + wc_local], gt_all);
      st_agent(&A.wc_b[L.wc_first + wc_local], eq_all);
    }
  }
  if (last_block_of_layer(&st->done, A.group_done + L.grp_first, wg - L.wg_first, L.wg_count, &sh.flag)) {
    scan_chunks(A.wc_a + L.wc_first, A.wc_b + L.wc_first, L.wc_count, st->r, true, sh.scan, &sh.cnt);
    __syncthreads();
    if (threadIdx.x == 0) {
      if (sh.cnt != L.k) atomicOr(A.errflag, 2u);
      st->next_phase = PH_OUT_V;
      st->next_launch = A.launch + 1u;
    }
  }
}

__device__ void phase_out_v(const CompressArgs& A, const LayerDesc& L, LayerState* st, uint32_t wc_local) {
  if (wc_local >= L.wc_count) return;
  const uint32_t T = st->T, r = st->r;
  const uint32_t begin = wc_local * A.chunk;
  const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
  uint32_t out_pos = A.wc_a[L.wc_first + wc_local];
  uint32_t eq_seen = A.wc_b[L.wc_first + wc_local];
  const bool clear_mom = (L.mom != nullptr) && A.mask_momentum;
  const gptr<int32_t> out_idx = as_global(L.out_idx);
  const gptr<float> out_val = as_global(L.out_val);
  const gptr<float> resid = as_global(L.resid);
  const gptr<float> mom = as_global(L.mom);
  for_each_group(L.resid, L.vec_ok != 0u, begin, end,
                 [&](const float (&a)[4], uint32_t nvalid, uint32_t idx0) {
                   bool gt[4], eq[4];
#pragma unroll
                   for (int j = 0; j < 4; ++j) {
                     const uint32_t key = ordered_key(fbits(a[j]), A.sign_xor, A.sign_filter);
                     const bool valid = static_cast<uint32_t>(j) < nvalid;
                     gt[j] = valid && key > T;
                     eq[j] = valid && key == T;
                   }
                   const unsigned long long any =
                       __ballot(gt[0] | gt[1] | gt[2] | gt[3] | eq[0] | eq[1] | eq[2] | eq[3]);
                   if (any == 0ull) return;
                   const unsigned long long e0 = __ballot(eq[0]), e1 = __ballot(eq[1]),
                                            e2 = __ballot(eq[2]), e3 = __ballot(eq[3]);
                   uint32_t my_eq = eq_seen + rank_below(e0) + rank_below(e1) + rank_below(e2) + rank_below(e3);
                   bool sel[4];
#pragma unroll
                   for (int j = 0; j < 4; ++j) {
                     sel[j] = gt[j] || (eq[j] && my_eq < r);
                     my_eq += eq[j] ? 1u : 0u;
                   }
                   eq_seen += popc64(e0) + popc64(e1) + popc64(e2) + popc64(e3);
                   const unsigned long long s0 = __ballot(sel[0]), s1 = __ballot(sel[1]),
                                            s2 = __ballot(sel[2]), s3 = __ballot(sel[3]);
                   uint32_t pos = out_pos + rank_below(s0) + rank_below(s1) + rank_below(s2) + rank_below(s3);
#pragma unroll
                   for (int j = 0; j < 4; ++j) {
                     if (sel[j]) {
                       if (pos < L.k) {   // always true when the counts are consistent
                         out_idx[pos] = static_cast<int32_t>(idx0 + j);
                         out_val[pos] = a[j];
                         resid[idx0 + j] = 0.0f;
                         if (clear_mom) mom[idx0 + j] = 0.0f;
                       }
                       ++pos;
                     }
                   }
                   out_pos += popc64(s0) + popc64(s1) + popc64(s2) + popc64(s3);
                 });
  if (wc_local == 0 && lane_id() == 0) *as_global(L.out_count) = static_cast<int32_t>(L.k);
}

// Hinted path: every wave looks at its own candidate list; candidates of the coarse bin that
// holds the k-th key become "members" (ranked exactly by the last workgroup), candidates of
// higher bins are counted as certainly selected.
__device__ void phase_sel(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st, uint32_t wg,
                          unsigned long long* sortbuf, uint32_t* sel_hist, ResolveShared& sh) {
  // The lists are short (a few dozen entries), so this phase is a chain of dependent loads per
  // workgroup and little else: one workgroup in A.list_group takes the lists of that many
  // workgroups, with the loads of all of them in flight together; the others leave at once.
  const uint32_t wgl = wg - L.wg_first;
  const uint32_t group = A.list_group, group_log2 = group == 1u ? 0u : kListGroupLog2;   // (1 or kListGroup)
  if ((wgl & (group - 1u)) != 0u) return;
  const uint32_t tau = st->tau, shift = st->shift, bstar = st->bstar;
  unsigned long long* members = A.members + static_cast<size_t>(l) * kMemberMax;
  const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) sh.hcnt = 0u;              // what this workgroup's lists add to their offset group
  __syncthreads();
  uint32_t wc[kListGroup], cnt[kListGroup];
#pragma unroll
  for (uint32_t i = 0; i < kListGroup; ++i) {
    const uint32_t wc_local = (wgl + i) * kWavesPerBlock + wave;
    wc[i] = L.wc_first + wc_local;
    cnt[i] = (i < group && wc_local < L.wc_count) ? A.cand_cnt[wc[i]] : 0xFFFFFFFFu;   // ~0: no such list
  }
  // the first 64 slots of every list are asked for together with the lists' lengths, not after them
  // (the slots exist whatever the length; what lies beyond it is not looked at)
  uint2 first[kListGroup];
#pragma unroll
  for (uint32_t i = 0; i < kListGroup; ++i) {
    first[i] = make_uint2(0u, 0u);
    if (i < group && (wgl + i) * kWavesPerBlock + wave < L.wc_count && lane < A.cap) first[i] = (A.slots + static_cast<size_t>(wc[i]) * A.cap)[lane];
  }
#pragma unroll
  for (uint32_t i = 0; i < kListGroup; ++i) {
    if (cnt[i] == 0xFFFFFFFFu) continue;
    const uint2* slot = A.slots + static_cast<size_t>(wc[i]) * A.cap;
    uint32_t hi = 0;
    for (uint32_t p0 = 0; p0 < cnt[i]; p0 += kWaveSize) {
      const uint32_t p = p0 + lane;
      if (p < cnt[i]) {
        const uint2 e = p0 == 0u ? first[i] : slot[p];
        const uint32_t key = key_of(e.x, A.sign_xor, A.sign_filter);
        const uint32_t bin = coarse_bin(key, tau, shift);
        if (bin > bstar) {
          ++hi;
        } else if (bin == bstar) {
          const uint32_t at = atomicAdd(&st->nmembers, 1u);
          if (at < static_cast<uint32_t>(kMemberMax))
            __hip_atomic_store(&members[at], composite(key, e.y), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
    const uint32_t hi_all = wave_total(wave_incl_scan(hi));
    if (lane == 0) {
      st_agent(&A.wc_a[wc[i]], hi_all);
      if (hi_all) atomicAdd(&sh.hcnt, hi_all);
    }
  }
  // one device-scope atomic per workgroup (its 16 wave-chunks lie in one offset group): such atomics
  // on one address take their turns at a fraction of a microsecond each
  __syncthreads();
  if (threadIdx.x == 0 && sh.hcnt != 0u) atomicAdd(&A.wc_b[L.wc_first + (wgl * kWavesPerBlock) / kOffsetGroup], sh.hcnt);
  if (!last_block_of_layer(&st->done, A.group_done + L.grp_first, wgl >> group_log2,
                           (L.wg_count + group - 1u) >> group_log2, &sh.flag)) return;

  const uint32_t m = ld_agent(&st->nmembers);
  const uint32_t k_rem = st->k_rem;
  if (m > static_cast<uint32_t>(kMemberMax) || k_rem == 0u || k_rem > m) {
    if (threadIdx.x == 0) atomicOr(A.errflag, 4u);
    return;   // cannot happen when the histogram and the lists agree; leave the layer unscheduled
  }
  // Output offsets: only the sums of groups of kOffsetGroup wave-chunks are scanned here (this is a
  // serial step of one workgroup); PH_OUT_C scans inside its group itself.  Up to kLdsGroups groups
  // (every layer below 400 M elements) the sums are fetched now, three a thread, while the members
  // are ranked; the members' own credits to them are then counted in LDS, which spares the round
  // trip of device-scope atomics followed by loads of the same words.
  constexpr uint32_t kLdsGroups = 3u * kBlockThreads;
  const uint32_t groups = (L.wc_count + kOffsetGroup - 1u) / kOffsetGroup;
  const bool in_lds = groups <= kLdsGroups;
  uint32_t gsum[3] = {0u, 0u, 0u};
  if (in_lds) {
#pragma unroll
    for (uint32_t j = 0; j < 3u; ++j) {
      const uint32_t g = 3u * threadIdx.x + j;
      if (g < groups) gsum[j] = ld_agent(&A.wc_b[L.wc_first + g]);
    }
  }
  for (uint32_t i = threadIdx.x; i < m; i += kBlockThreads)
    sortbuf[i] = __hip_atomic_load(&members[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  const unsigned long long thr = select_kth_largest(sortbuf, m, k_rem, sel_hist, sh);
  __syncthreads();                                  // every wave is done with the selection's histograms
  if (in_lds) {
    sel_hist[threadIdx.x] = 0u; sel_hist[kBlockThreads + threadIdx.x] = 0u; sel_hist[2u * kBlockThreads + threadIdx.x] = 0u;
    __syncthreads();
  }
  // members not below thr are selected: credit them to their wave-chunks (and to the chunks' groups)
  for (uint32_t i = threadIdx.x; i < m; i += kBlockThreads) {
    if (sortbuf[i] < thr) continue;
    const uint32_t idx = 0xFFFFFFFFu - static_cast<uint32_t>(sortbuf[i] & 0xFFFFFFFFull);
    const uint32_t c = idx / A.chunk;
    atomicAdd(&A.wc_a[L.wc_first + c], 1u);
    if (in_lds) atomicAdd(&sel_hist[c / kOffsetGroup], 1u);
    else atomicAdd(&A.wc_b[L.wc_first + c / kOffsetGroup], 1u);
  }
  if (in_lds) {
    __syncthreads();
    uint32_t v[3], mine = 0u;
#pragma unroll
    for (uint32_t j = 0; j < 3u; ++j) {
      const uint32_t g = 3u * threadIdx.x + j;
      v[j] = g < groups ? gsum[j] + sel_hist[g] : 0u;
      mine += v[j];
    }
    uint32_t total;
    uint32_t ex = block_excl_scan(mine, sh.scan, total);
#pragma unroll
    for (uint32_t j = 0; j < 3u; ++j) {
      const uint32_t g = 3u * threadIdx.x + j;
      if (g < groups) A.wc_b[L.wc_first + g] = ex;
      ex += v[j];
    }
    if (threadIdx.x == 0) sh.cnt = total;
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the credits are device-scope atomics
    __syncthreads();
    scan_chunks(A.wc_b + L.wc_first, nullptr, groups, 0u, false, sh.scan, &sh.cnt);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (sh.cnt != L.k) atomicOr(A.errflag, 8u);
    const uint32_t T = static_cast<uint32_t>(thr >> 32);
    st->thr = thr;
    st->T = T;
    if (A.update_hints) {
      const uint32_t tn = st->tau_next <= T ? st->tau_next : T;
      st->tau = drifted_tau(tn, T, st->T_prev, st->has_prev != 0u);
      st->shift = shift_for(T, tn);
      st->hint_valid = 1u;               // (a hint-free call that collected after its first digit gets its hint here)
      st->T_prev = T;
      st->has_prev = 1u;
    }
    st->next_phase = PH_OUT_C;
    st->next_launch = A.launch + 1u;
  }
}

__device__ void phase_out_c(const CompressArgs& A, const LayerDesc& L, LayerState* st, uint32_t wg) {
  const uint32_t wgl = wg - L.wg_first;
  const uint32_t group = A.list_group;              // (1 or kListGroup)
  if ((wgl & (group - 1u)) != 0u) return;           // see phase_sel
  const unsigned long long thr = st->thr;
  const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
  const bool clear_mom = (L.mom != nullptr) && A.mask_momentum;
  const gptr<int32_t> out_idx = as_global(L.out_idx);
  const gptr<float> out_val = as_global(L.out_val);
  const gptr<float> resid = as_global(L.resid);
  const gptr<float> mom = as_global(L.mom);
  uint32_t wc[kListGroup], cnt[kListGroup], out_at[kListGroup];
  // this wave's lists are wave-chunks (wgl + i) * 4 + wave: all inside one group of kOffsetGroup
  const uint32_t grp = (wgl * kWavesPerBlock) / kOffsetGroup;
  uint32_t excl;
  {
    const uint32_t c = grp * kOffsetGroup + lane;
    const uint32_t mine = c < L.wc_count ? A.wc_a[L.wc_first + c] : 0u;   // selected entries of the group's chunks
    excl = wave_incl_scan(mine) - mine + A.wc_b[L.wc_first + grp];
  }
#pragma unroll
  for (uint32_t i = 0; i < kListGroup; ++i) {
    const uint32_t wc_local = (wgl + i) * kWavesPerBlock + wave;
    wc[i] = L.wc_first + wc_local;
    cnt[i] = 0u;
    out_at[i] = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(excl),
                                                                 static_cast<int>(__builtin_amdgcn_readfirstlane(wc_local % kOffsetGroup))));
    if (i < group && wc_local < L.wc_count) cnt[i] = A.cand_cnt[wc[i]];
  }
  uint2 first[kListGroup];
#pragma unroll
  for (uint32_t i = 0; i < kListGroup; ++i) {
    first[i] = make_uint2(0u, 0u);
    if (lane < cnt[i]) first[i] = (A.slots + static_cast<size_t>(wc[i]) * A.cap)[lane];
  }
#pragma unroll
  for (uint32_t i = 0; i < kListGroup; ++i) {
    const uint2* slot = A.slots + static_cast<size_t>(wc[i]) * A.cap;
    uint32_t out_pos = out_at[i];
    for (uint32_t p0 = 0; p0 < cnt[i]; p0 += kWaveSize) {
      const uint32_t p = p0 + lane;
      uint2 e = make_uint2(0u, 0u);
      bool sel = false;
      if (p < cnt[i]) {
        e = p0 == 0u ? first[i] : slot[p];
        sel = composite(key_of(e.x, A.sign_xor, A.sign_filter), e.y) >= thr;
      }
      const unsigned long long sm = __ballot(sel);
      const uint32_t pos = out_pos + rank_below(sm);
      if (sel && pos < L.k && e.y < L.n) {   // the bounds always hold when the counts are consistent
        out_idx[pos] = static_cast<int32_t>(e.y);
        out_val[pos] = __uint_as_float(e.x);
        mask_store(&resid[e.y]);
        if (clear_mom) mask_store(&mom[e.y]);
      }
      out_pos += popc64(sm);
    }
  }
  if (wgl == 0u && threadIdx.x == 0u) *as_global(L.out_count) = static_cast<int32_t>(L.k);
}

}  // namespace

// The phase launches always take the workgroups in ascending order, largest layers first: their
// serial per-layer steps then start as early as possible.  (Letting consecutive launches alternate
// like the streaming passes of consecutive calls do makes the multi-pass path 6 % faster, each pass
// starting with what the one before touched last, but the steady state 2 us slower.)
__device__ __forceinline__ uint32_t phase_workgroup(const CompressArgs&) { return blockIdx.x; }

__global__ void __launch_bounds__(kBlockThreads) phase_kernel(CompressArgs A) {
  __shared__ union {
    uint32_t hist[kHistBins];
    unsigned long long sortbuf[kMemberMax];
  } sm;
  __shared__ ResolveShared sh;
  __shared__ __attribute__((aligned(16))) uint32_t sel_hist[3 * 256];
  const uint32_t wg = phase_workgroup(A);
  const uint32_t l = A.wg2layer[wg];
  LayerState* st = A.state + l;
  if (st->next_launch != A.launch) return;
  const LayerDesc L = A.layers[l];
  const uint32_t phase = st->next_phase;
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  switch (phase) {
    case PH_SEL:   phase_sel(A, l, L, st, wg, sm.sortbuf, sel_hist, sh); break;
    case PH_OUT_C: phase_out_c(A, L, st, wg); break;
    case PH_HIST1: phase_hist<1>(A, l, L, st, wg, wc_local, sm.hist, sh); break;
    case PH_RESTORE: dense_restore(A, L, st, wc_local); phase_hist<1>(A, l, L, st, wg, wc_local, sm.hist, sh); break;
    case PH_HIST2: phase_hist<2>(A, l, L, st, wg, wc_local, sm.hist, sh); break;
    case PH_HIST3: phase_hist<3>(A, l, L, st, wg, wc_local, sm.hist, sh); break;
    case PH_COUNT: phase_count(A, l, L, st, wg, wc_local, sh); break;
    case PH_OUT_V: phase_out_v(A, L, st, wc_local); break;
    case PH_COLLECT: phase_collect(A, l, L, st, wg, wc_local, sm.hist, sh); break;
    default: break;
  }
}

// Launches 4..6 can only meet the last three phases of the multi-pass path (a layer that missed
// its hint is at PH_HIST3 in launch 4 at the earliest) or the output phase of a hint-free call that
// collected its candidates in launch 2, and in steady state they meet nothing at
// all.  They get a kernel of their own that needs next to no LDS: twice as many of its
// workgroups fit on the device at once, so the launches that find nothing to do are over sooner.
constexpr uint32_t kFirstLateLaunch = 4;
__global__ void __launch_bounds__(kBlockThreads) phase_late_kernel(CompressArgs A) {
  __shared__ uint32_t hist[256];   // the last digit: 7 or 8 bits
  __shared__ ResolveShared sh;
  const uint32_t wg = phase_workgroup(A);
  const uint32_t l = A.wg2layer[wg];
  LayerState* st = A.state + l;
  if (st->next_launch != A.launch) return;
  const LayerDesc L = A.layers[l];
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  switch (st->next_phase) {
    case PH_HIST3: phase_hist<3>(A, l, L, st, wg, wc_local, hist, sh); break;
    case PH_COUNT: phase_count(A, l, L, st, wg, wc_local, sh); break;
    case PH_OUT_V: phase_out_v(A, L, st, wc_local); break;
    case PH_OUT_C: phase_out_c(A, L, st, wg); break;                  // a hint-free call that collected after its first digit
    default: if (threadIdx.x == 0) atomicOr(A.errflag, 16u); break;   // no other phase can be due this late
  }
}

// =================================================================== dense layers (high densities)
// At the densities of a warm-up period (Section 2.5: 25 %, 6.25 %, 1.5625 % before 0.1 %) the candidate
// lists of the one-pass path cannot hold every element from the hinted threshold upwards, and masking the
// sent entries out of the residual one by one afterwards would dirty most cache lines of V and u a second
// time.  Such a layer ("dense"), once it has a hint, is streamed by a kernel of its own:
//  1. collect_kernel reads G, V (, u), computes the accumulated values and lists EVERY candidate
//     (key >= tau) in the wave-chunk's list, in index order (lists of the layer's own, long enough for twice
//     the expected number).  The hint also says where the k-th key is expected (mask_key): the pass writes +0
//     into V (and u) in place of every candidate from there upwards, taking it as sent, and keeps its velocity
//     in a second array.  The candidates up to a clip bin well above the expected k-th key ("the band") enter
//     the coarse histogram one by one; those above it are sure to be selected, are counted per lane and added
//     to the top bin once.
//  2. lists_kernel, launch 2 (PH_SEL2): every wave walks its list; the members of the k-th key's coarse bin
//     are ranked exactly by the layer's last workgroup, as on the one-pass path.
//  3. lists_kernel, launch 3 (PH_EMIT): the message straight from the ordered lists.  What step 1 guessed
//     wrong is put right here: a sent entry below mask_key is masked now, a masked entry that is not sent gets
//     its value and velocity back (as many isolated writes as the k-th key lies ranks away from where it was
//     expected, whatever the width of the band).
// If the hint misses (too few candidates, the k-th key at or above the clip bin, a list that ran over, more
// members than can be ranked), what step 1 masked is put back from the lists at launch 2 (PH_RESTORE: V and u
// are then exactly the accumulated values, as after an ordinary streaming pass), and the layer starts on the
// multi-pass path in the same launch.
// A wave-chunk whose list may not hold the next group stops listing AND masking there, so the lists always
// hold what was masked.
namespace {

// What the streaming pass of a dense layer keeps per wave-chunk beside the Collector.
// The list entries pass through a staging area in LDS of the wave's own: appended one by one to global memory they
// would cost up to eight sparse store instructions per group of 256 elements (and leave cache lines partly written);
// from the staging area they go out 64 at a time, one full 512-byte store per array.
constexpr uint32_t kStageEntries = 5u * kWaveSize;   // what a flush leaves (< 64) plus one group's candidates (<= 256)
struct DenseChunk {
  gptr<float> slot_u;   // the velocity of the listed elements (null: the velocity is not masked, nothing is kept)
  vu2* stage;           // [kStageEntries] in LDS: the list's entries from number `flushed` on
  float* stage_u;       // [kStageEntries] their velocities
  uint32_t flushed;     // entries of the list that are in global memory already (a multiple of 64 until the end)
  uint32_t mask_key;    // candidates with keys from here upwards are masked at once (where the k-th key is expected)
  uint32_t clip_key;    // candidates with keys from here upwards lie in the coarse bins from the clip bin upwards: sure to be selected
  uint32_t certain;     // how many candidates from clip_key upwards this lane has seen (they enter the histogram's top bin in one
                        // addition per wave-chunk: one by one they would all queue up on that word)
  bool overflow;        // the list may not hold the next group: from here on the pass neither lists nor masks
};

// The four accumulated values a lane holds (elements idx0 .. idx0+3, the first `nvalid` exist): which of them the
// pass masks at once.  Known before any rank is, so the stores of V (and u) go out first, as in stream_chunk.
__device__ __forceinline__ void masked_dense(const float (&a)[4], uint32_t nvalid, const Collector& c, const DenseChunk& dc,
                                             uint32_t (&key)[4], bool (&masked)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    key[j] = key_of(fbits(a[j]), c.sign_xor, c.sign_filter);
    masked[j] = !dc.overflow && (static_cast<uint32_t>(j) < nvalid) && key[j] >= dc.mask_key;
  }
}

// Writes the staged entries [0, n) (n <= 64) behind the list's flushed part.  Lanes read what other lanes of the wave
// staged: the wave barriers keep the compiler from moving LDS accesses across them (the hardware keeps a wave's LDS
// operations in order).
__device__ __forceinline__ void flush_staged(Collector& c, DenseChunk& dc, uint32_t from, uint32_t n) {
  const uint32_t lane = lane_id();
  if (lane < n) {
    c.slot[dc.flushed + lane] = dc.stage[from + lane];
    if (dc.slot_u != nullptr) dc.slot_u[dc.flushed + lane] = dc.stage_u[from + lane];
  }
}

// Appends the group's candidates to the wave-chunk's list in index order (the caller has seen that 256 more
// entries fit).  The candidates of the band (keys below clip_key) enter the coarse histogram one by one.
__device__ __forceinline__ void list_dense(const float (&a)[4], const float (&u)[4], const uint32_t (&key)[4],
                                           uint32_t nvalid, uint32_t idx0, Collector& c, DenseChunk& dc) {
  bool cand[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) cand[j] = (static_cast<uint32_t>(j) < nvalid) && (key[j] >= c.tau);
  const unsigned long long m0 = __ballot(cand[0]), m1 = __ballot(cand[1]), m2 = __ballot(cand[2]), m3 = __ballot(cand[3]);
  if ((m0 | m1 | m2 | m3) == 0ull) return;
  uint32_t pos = (c.count - dc.flushed) + rank_below(m0) + rank_below(m1) + rank_below(m2) + rank_below(m3);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (cand[j]) {
      dc.stage[pos] = vu2{fbits(a[j]), idx0 + j};
      if (dc.slot_u != nullptr) dc.stage_u[pos] = u[j];
      if (key[j] >= dc.clip_key) ++dc.certain;
      else atomicAdd(&c.coarse[coarse_bin(key[j], c.tau, c.shift)], 1u);
      ++pos;
    }
  }
  c.count += popc64(m0) + popc64(m1) + popc64(m2) + popc64(m3);
  uint32_t pend = c.count - dc.flushed;               // wave-uniform
  if (pend >= kWaveSize) {
    __builtin_amdgcn_wave_barrier();
    uint32_t from = 0;
    do {
      flush_staged(c, dc, from, kWaveSize);
      from += kWaveSize;
      dc.flushed += kWaveSize;
      pend -= kWaveSize;
    } while (pend >= kWaveSize);
    // what is left moves to the front of the staging area
    const uint32_t lane = lane_id();
    vu2 e = vu2{0u, 0u};
    float eu = 0.0f;
    if (lane < pend) { e = dc.stage[from + lane]; eu = dc.stage_u[from + lane]; }
    __builtin_amdgcn_wave_barrier();
    if (lane < pend) { dc.stage[lane] = e; dc.stage_u[lane] = eu; }
    __builtin_amdgcn_wave_barrier();
  }
}

// Streaming pass over one wave-chunk [begin, end) of a dense layer that has a hint: stream_chunk's loop, with the
// candidates far above the hinted threshold masked on the way.
template <bool kMom, bool kNest>
__device__ __forceinline__ void stream_chunk_dense(const LayerDesc& L, uint32_t begin, uint32_t end, const AccumRule m,
                                                   bool clear_mom, Collector& c, DenseChunk& dc) {
  const uint32_t lane = lane_id();
  uint32_t base = begin;
  if (L.vec_ok) {
    const uint32_t nfull = (end - begin) / kGroupElems;
    const gptr<const vf4> G4 = as_global(reinterpret_cast<const vf4*>(L.grad + begin));
    const gptr<vf4> V4 = as_global(reinterpret_cast<vf4*>(L.resid + begin));
    const gptr<vf4> U4 = as_global(kMom ? reinterpret_cast<vf4*>(L.mom + begin) : nullptr);
    constexpr uint32_t kUnroll = kMom ? 2u : 4u;
    auto group = [&](const vf4& gq, const vf4& vq, const vf4& uq, uint32_t o) __attribute__((always_inline)) {
      const float gg[4] = {gq.x, gq.y, gq.z, gq.w};
      const float vvv[4] = {vq.x, vq.y, vq.z, vq.w};
      float uu[4] = {0.f, 0.f, 0.f, 0.f};
      if constexpr (kMom) { uu[0] = uq.x; uu[1] = uq.y; uu[2] = uq.z; uu[3] = uq.w; }
      float a[4];
      accum4<kMom, kNest>(gg, vvv, uu, m, a);
      dc.overflow = dc.overflow || (c.count + 4u * kWaveSize > c.cap);
      uint32_t key[4];
      bool masked[4];
      masked_dense(a, 4u, c, dc, key, masked);
      V4[o] = vf4{masked[0] ? 0.0f : a[0], masked[1] ? 0.0f : a[1], masked[2] ? 0.0f : a[2], masked[3] ? 0.0f : a[3]};
      if constexpr (kMom)
        U4[o] = vf4{(masked[0] && clear_mom) ? 0.0f : uu[0], (masked[1] && clear_mom) ? 0.0f : uu[1],
                    (masked[2] && clear_mom) ? 0.0f : uu[2], (masked[3] && clear_mom) ? 0.0f : uu[3]};
      if (!dc.overflow) list_dense(a, uu, key, 4u, begin + o * 4u, c, dc);
    };
    uint32_t g = 0;
    for (; g + kUnroll <= nfull; g += kUnroll) {
      vf4 gv[kUnroll], vv[kUnroll], uv[kUnroll];
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) {
        const uint32_t o = (g + t) * kWaveSize + lane;
        gv[t] = __builtin_nontemporal_load(&G4[o]);
        vv[t] = V4[o];
        if constexpr (kMom) uv[t] = U4[o];
      }
#pragma unroll
      for (uint32_t t = 0; t < kUnroll; ++t) group(gv[t], vv[t], uv[t], (g + t) * kWaveSize + lane);
    }
    for (; g < nfull; ++g) {
      const uint32_t o = g * kWaveSize + lane;
      const vf4 gq = __builtin_nontemporal_load(&G4[o]);
      const vf4 vq = V4[o];
      vf4 uq = vf4{0.f, 0.f, 0.f, 0.f};
      if constexpr (kMom) uq = U4[o];
      group(gq, vq, uq, o);
    }
    base = begin + nfull * kGroupElems;
  }
  // scalar groups: the ragged tail of an aligned layer, or every group of an unaligned one
  const gptr<const float> Gs = as_global(L.grad);
  const gptr<float> Vs = as_global(L.resid);
  const gptr<float> Us = as_global(L.mom);
  for (; base < end; base += kGroupElems) {
    const uint32_t idx0 = base + lane * 4u;
    const uint32_t nvalid = idx0 < end ? ((end - idx0) < 4u ? (end - idx0) : 4u) : 0u;
    float gg[4] = {0.f, 0.f, 0.f, 0.f}, vvv[4] = {0.f, 0.f, 0.f, 0.f}, uu[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (static_cast<uint32_t>(j) < nvalid) {
        gg[j] = Gs[idx0 + j];
        vvv[j] = Vs[idx0 + j];
        if constexpr (kMom) uu[j] = Us[idx0 + j];
      }
    }
    float a[4];
    accum4<kMom, kNest>(gg, vvv, uu, m, a);
    dc.overflow = dc.overflow || (c.count + 4u * kWaveSize > c.cap);
    uint32_t key[4];
    bool masked[4];
    masked_dense(a, nvalid, c, dc, key, masked);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (static_cast<uint32_t>(j) < nvalid) {
        Vs[idx0 + j] = masked[j] ? 0.0f : a[j];
        if constexpr (kMom) Us[idx0 + j] = (masked[j] && clear_mom) ? 0.0f : uu[j];
      }
    }
    if (!dc.overflow) list_dense(a, uu, key, nvalid, idx0, c, dc);
  }
  // the list's last entries (fewer than 64)
  __builtin_amdgcn_wave_barrier();
  flush_staged(c, dc, 0u, c.count - dc.flushed);
  dc.flushed = c.count;
}

}  // namespace

// Launch 1 for the dense layers that have a hint (accumulate_kernel leaves exactly these out).
__global__ void __launch_bounds__(kBlockThreads) collect_kernel(CompressArgs A) {
  __shared__ uint32_t lds_hist[kCoarseBins];
  __shared__ ResolveShared sh;
  __shared__ vu2 stage[kWavesPerBlock][kStageEntries];
  __shared__ float stage_u[kWavesPerBlock][kStageEntries];
  const uint32_t wg = A.reverse ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  if (!L.dense) return;
  LayerState* st = A.state + l;
  // the same condition as in accumulate_kernel
  const bool hinted = A.use_hints && (st->hint_valid != 0u) && !(A.sign_filter != 0u && st->tau == 0u);
  if (!hinted || st->dense_skip != 0u) return;
  for (uint32_t b = threadIdx.x; b < static_cast<uint32_t>(kCoarseBins); b += kBlockThreads) lds_hist[b] = 0u;
  __syncthreads();
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  if (wc_local < L.wc_count) {
    const uint32_t begin = wc_local * A.chunk;
    const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
    const size_t list = L.list_first + static_cast<size_t>(wc_local) * L.list_cap;
    const bool mom = L.mom != nullptr;
    const bool clear_mom = mom && A.mask_momentum;
    Collector c;
    c.slot = as_global(reinterpret_cast<vu2*>(A.slots2 + list));
    c.coarse = lds_hist;
    c.cap = L.list_cap;
    c.count = 0;
    c.tau = st->tau;
    c.shift = st->shift;
    c.sign_xor = A.sign_xor;
    c.sign_filter = A.sign_filter;
    c.clip = dense_clip(st->clip);
    DenseChunk dc;
    // (the velocity is kept only where the masking clears it)
    dc.slot_u = clear_mom ? as_global(A.slots_u + list) : gptr<float>(nullptr);
    dc.stage = stage[threadIdx.x >> 6];
    dc.stage_u = stage_u[threadIdx.x >> 6];
    dc.flushed = 0u;
    dc.clip_key = dense_clip_key(c.tau, c.shift, c.clip);
    dc.mask_key = dense_mask_key(st->mask_key, c.tau);
    dc.certain = 0u;
    dc.overflow = false;
    AccumRule rule;
    rule.m = A.m;
    rule.scale = A.grad_scale ? *as_global(A.grad_scale) : 1.0f;
    if (!mom) stream_chunk_dense<false, false>(L, begin, end, rule, clear_mom, c, dc);
    else if (!A.nesterov) stream_chunk_dense<true, false>(L, begin, end, rule, clear_mom, c, dc);
    else stream_chunk_dense<true, true>(L, begin, end, rule, clear_mom, c, dc);
    const uint32_t certain = wave_total(wave_incl_scan(dc.certain));
    if (lane_id() == 0) {
      // (a list that stopped early says so, and where: nothing was listed or masked after that entry)
      st_agent(&A.cand_cnt[L.wc_first + wc_local], dc.overflow ? (kListStopped | c.count) : c.count);
      if (certain) atomicAdd(&lds_hist[kCoarseBins - 1], certain);
    }
  }
  __syncthreads();
  flush_hist(lds_hist, A.coarse + (static_cast<size_t>(l) * kCoarseRep + (wg & (kCoarseRep - 1))) * kCoarseBins, kCoarseBins);
  if (last_block_of_layer(&st->done, A.group_done + L.grp_first, wg - L.wg_first, L.wg_count, &sh.flag))
    resolve_collect(A, l, L, st, sh, lds_hist, false, 1u, true);
}

namespace {

// The members of a dense layer: kMemberLists lists in global memory (region + s * shard_cap, n[s] entries; the last
// one, for what the others could not hold, is longer), which other workgroups filled with device-scope stores.
// A thread asks for one value of every list at a time, so that their round trips overlap.
struct MemberLists {
  const unsigned long long* region;
  uint32_t shard_cap;
  const uint32_t* first;  // [kMemberLists + 1], in LDS: running number of each list's first member; [kMemberLists] = all
};

template <typename F>
__device__ __forceinline__ void for_each_member(const MemberLists& M, F&& f) {
  // one step takes the i-th member of every list: kMemberLists independent loads of a thread in flight
  uint32_t n[kMemberLists], nmax = 0u;
#pragma unroll
  for (uint32_t s = 0; s < kMemberLists; ++s) {
    n[s] = M.first[s + 1] - M.first[s];
    nmax = n[s] > nmax ? n[s] : nmax;
  }
  for (uint32_t i = threadIdx.x; i < nmax; i += kBlockThreads) {
    unsigned long long x[kMemberLists];
#pragma unroll
    for (uint32_t s = 0; s < kMemberLists; ++s)
      x[s] = i < n[s] ? __hip_atomic_load(&M.region[static_cast<size_t>(s) * M.shard_cap + i], __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT)
                      : 0ull;
#pragma unroll
    for (uint32_t s = 0; s < kMemberLists; ++s)
      if (i < n[s]) f(x[s]);
  }
}

// select_kth_largest() for such members (there may be more of them than the LDS holds): the same radix
// selection, every digit one more pass over the values.  `any` is one of the values.  hist holds 3 * 256 words.
__device__ unsigned long long select_kth_largest_global(const MemberLists& M, unsigned long long any, uint32_t kk,
                                                        uint32_t* hist, ResolveShared& sh) {
  const uint32_t t = threadIdx.x, lane = lane_id();
  const unsigned long long v0 = any;
  unsigned long long diff = 0ull;
  for_each_member(M, [&](unsigned long long x) { diff |= x ^ v0; });
  int top = diff ? 63 - __clzll(static_cast<long long>(diff)) : -1;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int other = __shfl_xor(top, o);
    top = other > top ? other : top;
  }
  if (lane == 0) sh.scan[t >> 6] = static_cast<uint32_t>(top + 1);
  hist[t] = 0u; hist[256u + t] = 0u; hist[512u + t] = 0u;
  __syncthreads();
  {
    const uint32_t a = sh.scan[0], b = sh.scan[1], c = sh.scan[2], d = sh.scan[3];
    const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
    top = static_cast<int>(ab > cd ? ab : cd) - 1;
  }
  if (top < 0) return v0;                                   // a single value
  int shift = (top >> 3) << 3;
  unsigned long long prefix = shift == 56 ? 0ull : (v0 & (~0ull << (shift + 8)));
  for (uint32_t pass = 0;; ++pass, shift -= 8) {
    uint32_t* const H = hist + (pass % 3u) * 256u;
    const unsigned long long himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
    for_each_member(M, [&](unsigned long long x) {
      if ((x & himask) == prefix) atomicAdd(&H[static_cast<uint32_t>(x >> shift) & 255u], 1u);
    });
    __syncthreads();
    hist[((pass + 2u) % 3u) * 256u + t] = 0u;
    const uint32_t h0 = H[4u * lane], h1 = H[4u * lane + 1u], h2 = H[4u * lane + 2u], h3 = H[4u * lane + 3u];
    const uint32_t mine = h0 + h1 + h2 + h3;
    const uint32_t incl = wave_incl_scan(mine);
    const uint32_t higher = wave_total(incl) - incl;
    const bool here = higher < kk && kk <= higher + mine;
    uint32_t bin = 0, above = 0, cnt = 0;
    if (here) {
      uint32_t a = higher;
      if (kk <= a + h3) { bin = 3u; cnt = h3; }
      else { a += h3; if (kk <= a + h2) { bin = 2u; cnt = h2; }
      else { a += h2; if (kk <= a + h1) { bin = 1u; cnt = h1; }
      else { a += h1; bin = 0u; cnt = h0; } } }
      bin += 4u * lane;
      above = a;
    }
    const unsigned long long who = __ballot(here);          // exactly one lane when 1 <= kk <= values in scope
    const int src = who ? static_cast<int>(__ffsll(static_cast<long long>(who))) - 1 : 0;
    bin = static_cast<uint32_t>(__shfl(static_cast<int>(bin), src));
    above = static_cast<uint32_t>(__shfl(static_cast<int>(above), src));
    cnt = static_cast<uint32_t>(__shfl(static_cast<int>(cnt), src));
    prefix |= static_cast<unsigned long long>(bin) << shift;
    kk -= above;
    if (shift == 0) return prefix;                          // the composites are distinct: this is the value itself
    if (cnt <= 1u) break;
  }
  // one value is left under these leading bytes: whoever holds it tells the others
  const unsigned long long lomask = ~0ull << shift;
  for_each_member(M, [&](unsigned long long x) {
    if ((x & lomask) == prefix) { sh.hbin = static_cast<uint32_t>(x); sh.hcum = static_cast<uint32_t>(x >> 32); }
  });
  __syncthreads();
  const unsigned long long r = (static_cast<unsigned long long>(sh.hcum) << 32) | sh.hbin;
  __syncthreads();
  return r;
}

// Launch 2 of a call with dense layers (PH_SEL2), for the layers whose streaming pass found the k-th key below
// its clip bin.  Every wave takes its own wave-chunk's list; the layer's last workgroup ranks the members of the
// k-th key's coarse bin (in global memory: there may be more of them than one workgroup's LDS holds), credits the
// selected ones to their wave-chunks, scans the group sums into offsets and schedules the output step.
__device__ void dense_rank(const CompressArgs& A, uint32_t l, const LayerDesc& L, LayerState* st, uint32_t wg,
                           ResolveShared& sh, uint32_t* sel_hist, uint32_t* shard_first) {
  const uint32_t tau = st->cur_tau, shift = st->cur_shift, bstar = st->bstar;
  unsigned long long* const region = A.members2 + L.mem_first;
  const uint32_t shard_cap = L.mem_cap / kMemberShards, spill_cap = L.mem_cap / 4u;
  const uint32_t lane = lane_id();
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  if (threadIdx.x == 0) sh.hcnt = 0u;              // what this workgroup's lists add to their offset group
  __syncthreads();
  const bool have = wc_local < L.wc_count;
  const uint32_t wc = L.wc_first + wc_local;
  const gptr<const vu2> slot = as_global(reinterpret_cast<const vu2*>(A.slots2 + L.list_first + static_cast<size_t>(have ? wc_local : 0u) * L.list_cap));
  uint32_t cnt = 0, hi = 0, nm = 0;
  unsigned long long keep0 = 0ull, keep1 = 0ull;
  if (have) {
    // One walk through the list, eight entries of a lane on their way at a time (every round trip counts); the
    // first eight are asked for together with the list's length (the slots exist whatever the length), the next
    // eight while these are looked at.  A lane keeps the first two members it meets; only a wave in which some
    // lane met more walks again.
    constexpr uint32_t kBatch = 8;
    vu2 e[kBatch];
#pragma unroll
    for (uint32_t j = 0; j < kBatch; ++j) {
      const uint32_t p = j * kWaveSize + lane;
      e[j] = p < L.list_cap ? slot[p] : vu2{0u, 0u};
    }
    cnt = A.cand_cnt[wc];                              // (<= list_cap: the streaming pass's resolve step has checked)
    for (uint32_t p0 = 0; p0 < cnt; p0 += kBatch * kWaveSize) {
      vu2 nx[kBatch];
#pragma unroll
      for (uint32_t j = 0; j < kBatch; ++j) {
        const uint32_t p = p0 + (kBatch + j) * kWaveSize + lane;
        nx[j] = p < cnt ? slot[p] : vu2{0u, 0u};
      }
#pragma unroll
      for (uint32_t j = 0; j < kBatch; ++j) {
        if (p0 + j * kWaveSize + lane < cnt) {
          const uint32_t key = key_of(e[j].x, A.sign_xor, A.sign_filter);
          const uint32_t bin = coarse_bin(key, tau, shift);
          hi += bin > bstar ? 1u : 0u;
          if (bin == bstar) {
            const unsigned long long c = composite(key, e[j].y);
            if (nm == 0u) keep0 = c; else if (nm == 1u) keep1 = c;
            ++nm;
          }
        }
      }
#pragma unroll
      for (uint32_t j = 0; j < kBatch; ++j) e[j] = nx[j];
    }
  }
  // The members of the workgroup's four lists are appended to its sub-list with ONE device-scope atomic (such
  // atomics on one address take their turns): the waves' counts meet in LDS, thread 0 reserves the room.
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t nm_incl = wave_incl_scan(nm);
  const uint32_t nm_all = wave_total(nm_incl);
  if (lane == 0) sh.scan[wave] = nm_all;
  __syncthreads();
  const uint32_t shard = (wg - L.wg_first) % kMemberShards;
  if (threadIdx.x == 0) {
    const uint32_t wg_all = sh.scan[0] + sh.scan[1] + sh.scan[2] + sh.scan[3];
    uint32_t base = 0, spill_base = 0;
    if (wg_all != 0u) {
      // the members go to the sub-list as far as that has room, the others to the overflow list (which can
      // hold every member the streaming pass's resolve step accepts): no sub-list is left with a gap
      base = atomicAdd(&A.shard_cnt[(static_cast<size_t>(l) * kMemberLists + shard) * kShardStride], wg_all);
      const uint32_t from = base > shard_cap ? base : shard_cap;
      if (base + wg_all > from)
        spill_base = atomicAdd(&A.shard_cnt[(static_cast<size_t>(l) * kMemberLists + kMemberShards) * kShardStride], base + wg_all - from);
    }
    sh.bin = base;
    sh.above = spill_base;
  }
  __syncthreads();
  if (nm_all != 0u) {
    const uint32_t wg_base = sh.bin, spill_base = sh.above;
    uint32_t before = 0;                               // members of the workgroup's waves before this one
    for (uint32_t w = 0; w < wave; ++w) before += sh.scan[w];
    const uint32_t from = wg_base > shard_cap ? wg_base : shard_cap;
    auto put = [&](uint32_t at, unsigned long long c) {        // `at`: position in the sub-list as if it had no end
      unsigned long long* to = nullptr;
      if (at < shard_cap) to = region + static_cast<size_t>(shard) * shard_cap + at;
      else if (spill_base + (at - from) < spill_cap) to = region + L.mem_cap + spill_base + (at - from);
      if (to != nullptr) __hip_atomic_store(to, c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    uint32_t at = wg_base + before + (nm_incl - nm);
    if (__ballot(nm > 2u) == 0ull) {
      if (nm >= 1u) put(at, keep0);
      if (nm >= 2u) put(at + 1u, keep1);
    } else {
      for (uint32_t p = lane; p < cnt; p += kWaveSize) {
        const vu2 e = slot[p];
        const uint32_t key = key_of(e.x, A.sign_xor, A.sign_filter);
        if (coarse_bin(key, tau, shift) == bstar) put(at++, composite(key, e.y));
      }
    }
  }
  if (have) {
    const uint32_t hi_all = wave_total(wave_incl_scan(hi));
    if (lane == 0) {
      st_agent(&A.wc_a[wc], hi_all);
      if (hi_all) atomicAdd(&sh.hcnt, hi_all);
    }
  }
  // one device-scope atomic per workgroup (its four wave-chunks lie in one offset group)
  __syncthreads();
  if (threadIdx.x == 0 && sh.hcnt != 0u)
    atomicAdd(&A.wc_b[L.wc_first + ((wg - L.wg_first) * kWavesPerBlock) / kOffsetGroup], sh.hcnt);
  if (!last_block_of_layer(&st->done, A.group_done + L.grp_first, wg - L.wg_first, L.wg_count, &sh.flag)) return;

  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (uint32_t s = 0; s < kMemberLists; ++s) {
      const uint32_t c = ld_agent(&A.shard_cnt[(static_cast<size_t>(l) * kMemberLists + s) * kShardStride]);
      const uint32_t cap = s < kMemberShards ? shard_cap : spill_cap;
      shard_first[s] = run;
      run += c < cap ? c : cap;
    }
    shard_first[kMemberLists] = run;
  }
  __syncthreads();
  const uint32_t m = shard_first[kMemberLists];
  const uint32_t k_rem = st->k_rem;
  if (k_rem == 0u || k_rem > m) {
    if (threadIdx.x == 0) atomicOr(A.errflag, 32u);
    return;   // cannot happen when the histogram and the lists agree; leave the layer unscheduled
  }
  MemberLists M{region, shard_cap, shard_first};
  unsigned long long any = 0ull;
  for (uint32_t s = 0; s < kMemberLists; ++s)
    if (shard_first[s + 1] != shard_first[s]) { any = __hip_atomic_load(&region[static_cast<size_t>(s) * shard_cap], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
  const unsigned long long thr = select_kth_largest_global(M, any, k_rem, sel_hist, sh);
  // members not below thr are selected: credit them to their wave-chunks and to the chunks' groups
  // (the groups' credits are counted in LDS where the groups fit, as in PH_SEL: their counters share a few cache lines)
  const uint32_t groups = (L.wc_count + kOffsetGroup - 1u) / kOffsetGroup;
  const bool in_lds = groups <= 3u * kBlockThreads;
  __syncthreads();                                  // every wave is done with the selection's histograms
  if (in_lds) {
    sel_hist[threadIdx.x] = 0u; sel_hist[kBlockThreads + threadIdx.x] = 0u; sel_hist[2u * kBlockThreads + threadIdx.x] = 0u;
    __syncthreads();
  }
  for_each_member(M, [&](unsigned long long x) {
    if (x < thr) return;
    const uint32_t idx = 0xFFFFFFFFu - static_cast<uint32_t>(x & 0xFFFFFFFFull);
    const uint32_t c = idx / A.chunk;
    atomicAdd(&A.wc_a[L.wc_first + c], 1u);
    if (in_lds) atomicAdd(&sel_hist[c / kOffsetGroup], 1u);
    else atomicAdd(&A.wc_b[L.wc_first + c / kOffsetGroup], 1u);
  });
  __syncthreads();
  if (in_lds) {
    for (uint32_t g = threadIdx.x; g < groups; g += kBlockThreads)
      if (sel_hist[g] != 0u) atomicAdd(&A.wc_b[L.wc_first + g], sel_hist[g]);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the credits are device-scope atomics
  __syncthreads();
  scan_chunks(A.wc_b + L.wc_first, nullptr, groups, 0u, false, sh.scan, &sh.cnt);
  __syncthreads();
  if (threadIdx.x == 0) {
    if (sh.cnt != L.k) atomicOr(A.errflag, 64u);
    const uint32_t T = static_cast<uint32_t>(thr >> 32);
    st->thr = thr;
    st->T = T;
    if (A.update_hints) {
      const uint32_t tn = st->tau_next <= T ? st->tau_next : T;
      st->tau = drifted_tau(tn, T, st->T_prev, st->has_prev != 0u);
      st->shift = shift_for(T, tn);
      st->clip = clip_for(T, tn, st->shift);
      st->mask_key = mask_key_for(T, tn, st->tau);
      st->dense_backoff = 0u;            // the hint did its job
      st->hint_valid = 1u;
      st->T_prev = T;
      st->has_prev = 1u;
    }
    st->next_phase = PH_EMIT;
    st->next_launch = A.launch + 1u;
  }
}

// Launch 3 (PH_EMIT): the composite of the k-th entry is known, and a listed element is sent if and only if its
// composite (key, then lower index first) is not below it.  The lists are in index order, so a wave writes its
// wave-chunk's part of the message in one walk; of the sent entries those of the coarse bins below the clip bin
// are still in V (and u) and are masked here, the others were masked by the streaming pass.
__device__ void dense_emit(const CompressArgs& A, const LayerDesc& L, LayerState* st, uint32_t wg) {
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  if (wc_local >= L.wc_count) return;
  const uint32_t lane = lane_id();
  // everything that depends on the wave-chunk's number alone is asked for together: the list's length, its first
  // entries (the slots exist whatever the length), the counts the output offset is made of
  const size_t list = L.list_first + static_cast<size_t>(wc_local) * L.list_cap;
  const gptr<const vu2> slot = as_global(reinterpret_cast<const vu2*>(A.slots2 + list));
  const gptr<const float> slot_u = as_global(static_cast<const float*>(A.slots_u + list));
  constexpr uint32_t kBatch = 4;
  vu2 e[kBatch];
#pragma unroll
  for (uint32_t j = 0; j < kBatch; ++j) {
    const uint32_t p = j * kWaveSize + lane;
    e[j] = p < L.list_cap ? slot[p] : vu2{0u, 0u};
  }
  const uint32_t cnt = A.cand_cnt[L.wc_first + wc_local];
  const unsigned long long thr = st->thr;
  const uint32_t mask_key = st->cur_mask_key;
  // the first output position of this wave-chunk: the offset of its group of kOffsetGroup wave-chunks (wc_b)
  // plus the selected entries of the group's chunks before it (wc_a), as in PH_OUT_C
  uint32_t out_pos;
  {
    const uint32_t grp = wc_local / kOffsetGroup;
    const uint32_t c = grp * kOffsetGroup + lane;
    const uint32_t mine = c < L.wc_count ? A.wc_a[L.wc_first + c] : 0u;
    const uint32_t excl = wave_incl_scan(mine) - mine + A.wc_b[L.wc_first + grp];
    out_pos = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(excl),
                                                              static_cast<int>(__builtin_amdgcn_readfirstlane(wc_local % kOffsetGroup))));
  }
  const bool clear_mom = (L.mom != nullptr) && A.mask_momentum;
  const gptr<int32_t> out_idx = as_global(L.out_idx);
  const gptr<float> out_val = as_global(L.out_val);
  const gptr<float> resid = as_global(L.resid);
  const gptr<float> mom = as_global(L.mom);
  for (uint32_t p0 = 0; p0 < cnt; p0 += kBatch * kWaveSize) {
    vu2 nx[kBatch];                                   // the next entries are on their way while these are written
#pragma unroll
    for (uint32_t j = 0; j < kBatch; ++j) {
      const uint32_t p = p0 + (kBatch + j) * kWaveSize + lane;
      nx[j] = p < cnt ? slot[p] : vu2{0u, 0u};
    }
#pragma unroll
    for (uint32_t j = 0; j < kBatch; ++j) {
      const uint32_t key = key_of(e[j].x, A.sign_xor, A.sign_filter);
      const bool sel = (p0 + j * kWaveSize + lane < cnt) && composite(key, e[j].y) >= thr;
      const unsigned long long sm = __ballot(sel);
      const uint32_t pos = out_pos + rank_below(sm);
      const uint32_t p = p0 + j * kWaveSize + lane;
      if (sel && pos < L.k && e[j].y < L.n) {   // the bounds always hold when the counts are consistent
        out_idx[pos] = static_cast<int32_t>(e[j].y);
        out_val[pos] = __uint_as_float(e[j].x);
        if (key < mask_key) {                   // (the streaming pass has masked the others)
          mask_store(&resid[e[j].y]);
          if (clear_mom) mask_store(&mom[e[j].y]);
        }
      } else if (!sel && p < cnt && key >= mask_key && e[j].y < L.n) {
        // masked by the streaming pass on the strength of the hint, and not sent after all: back it goes
        // (isolated 4-byte writes like the masking ones: stored with the streaming hint for the same reason)
        __builtin_nontemporal_store(__uint_as_float(e[j].x), &resid[e[j].y]);
        if (clear_mom) __builtin_nontemporal_store(slot_u[p], &mom[e[j].y]);
      }
      out_pos += popc64(sm);
    }
#pragma unroll
    for (uint32_t j = 0; j < kBatch; ++j) e[j] = nx[j];
  }
  if (wc_local == 0 && lane == 0) *as_global(L.out_count) = static_cast<int32_t>(L.k);
}

}  // namespace

__global__ void __launch_bounds__(kBlockThreads) lists_kernel(CompressArgs A) {
  __shared__ ResolveShared sh;
  __shared__ __attribute__((aligned(16))) uint32_t sel_hist[3 * 256];
  __shared__ uint32_t shard_first[kMemberLists + 1];
  const uint32_t wg = blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  LayerState* st = A.state + l;
  if (st->next_launch != A.launch) return;
  const LayerDesc L = A.layers[l];
  switch (st->next_phase) {
    case PH_SEL2: dense_rank(A, l, L, st, wg, sh, sel_hist, shard_first); break;
    case PH_EMIT: dense_emit(A, L, st, wg); break;
    default: break;                                   // the other phases belong to phase_kernel
  }
}

// Overwrite the cached thresholds with wrong values (test hook: results must not change).
__global__ void poison_kernel(LayerState* st, uint32_t num_layers, int mode) {
  const uint32_t l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= num_layers) return;
  uint32_t h = (l + 1u) * 2654435761u;
  h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
  st[l].hint_valid = 1u;
  if (mode == 0) { st[l].tau = 0x7F000000u; st[l].shift = 0u; }
  else if (mode == 1) { st[l].tau = 0u; st[l].shift = 0u; }
  else { st[l].tau = h & 0x3FFFFFFFu; st[l].shift = (h >> 7) % 24u; }
}

__global__ void wave_scan_selftest_kernel(uint32_t* io) {
  // io[0..255] in: values; out: block-exclusive scan.  io[256]: total.
  __shared__ uint32_t lds[4];
  uint32_t total;
  const uint32_t v = io[threadIdx.x];
  const uint32_t ex = block_excl_scan(v, lds, total);
  const unsigned long long odd = __ballot((v & 1u) != 0u);
  io[threadIdx.x] = ex;
  io[512 + threadIdx.x] = rank_below(odd);
  if (threadIdx.x == 0) io[256] = total;
}

// ------------------------------------------------------------------ local gradient clipping
// Section 2.4: the gradients of all layers are clipped by their common L2 norm, locally and
// before they are added to the residuals; with N workers the threshold is max_norm / sqrt(N).
// The norm is the square root of the exactly rounded sum of the squares (rgc_exact.h), so the same
// coefficient comes out whatever the tiling.  Two launches: every workgroup leaves one part of the
// sum for its four wave-chunks of the gradient; one workgroup then adds the parts up, rounds, and
// stores  c = norm > threshold ? threshold / norm : 1  as a float.
//
// The squares of one wave-chunk, fast: one error-free addition per element into s, its error added
// to c with an ordinary addition, and the smallest and largest magnitude seen kept beside them.  The
// ordinary additions were exact if every error is a multiple of q, the last bit of the smallest
// square, and their sums stay below 2^53 q; a lane checks that afterwards from the exponents (the
// errors of the at most 2^k additions of a lane are at most half a last bit of its final s each).  A
// wave in which a lane cannot show it (elements some 2^23 apart, an element that is not finite) takes
// its chunk again the careful way (kCareful), which needs no such condition.
struct SquareSums {
  ExactAcc acc{0.0, 0.0, 0u};
  uint32_t least = 0xFFFFFFFFu;   // smallest magnitude bits - 1 over the non-zero elements
  uint32_t most = 0u;             // largest magnitude bits
};

template <bool kCareful>
__device__ __forceinline__ void add_square(SquareSums& S, float x, long long* digits) {
  if constexpr (kCareful) {
    exact_add_square(S.acc, x, digits);
  } else {
    const uint32_t b = fbits(x) & 0x7FFFFFFFu;
    S.most = b > S.most ? b : S.most;
    S.least = (b - 1u) < S.least ? (b - 1u) : S.least;        // zero wraps around and never counts
    const double d = static_cast<double>(x);
    double sum, err;
    two_sum(S.acc.s, d * d, sum, err);
    S.acc.s = sum;
    S.acc.c += err;
  }
}

template <bool kCareful>
__device__ __forceinline__ void squares_of_chunk(const float* grad, uint32_t begin, uint32_t end, SquareSums& S, long long* digits) {
  const uint32_t lane = lane_id();
  uint32_t base = begin;
  if ((reinterpret_cast<uintptr_t>(grad) & 15u) == 0u) {
    // whole groups of 64 x 4 elements, eight 16-byte loads of a lane in flight
    const gptr<const vf4> G4 = as_global(reinterpret_cast<const vf4*>(grad + begin));
    const uint32_t nfull = (end - begin) / kGroupElems;
    uint32_t g = 0;
    for (; g + 8u <= nfull; g += 8u) {
      vf4 q[8];
#pragma unroll
      for (uint32_t t = 0; t < 8u; ++t) q[t] = G4[(g + t) * kWaveSize + lane];
#pragma unroll
      for (uint32_t t = 0; t < 8u; ++t) {
        add_square<kCareful>(S, q[t].x, digits);
        add_square<kCareful>(S, q[t].y, digits);
        add_square<kCareful>(S, q[t].z, digits);
        add_square<kCareful>(S, q[t].w, digits);
      }
    }
    base = begin + g * kGroupElems;
  }
  for_each_group(grad, false, base, end,
                 [&](const float (&a)[4], uint32_t nvalid, uint32_t) {
#pragma unroll
                   for (int j = 0; j < 4; ++j) {
                     if (static_cast<uint32_t>(j) < nvalid) add_square<kCareful>(S, a[j], digits);
                   }
                 });
}

// True if the fast sums of this lane are the exact ones (see above); terms: at most 2^k per lane.
__device__ __forceinline__ bool square_sums_exact(const SquareSums& S, uint32_t k) {
  if (S.most >= 0x7F800000u) return false;                   // an infinity or a NaN
  if (S.least == 0xFFFFFFFFu) return true;                   // nothing but zeros
  uint32_t fmin = (S.least + 1u) >> 23;                      // exponent field of the smallest non-zero magnitude
  fmin = fmin ? fmin : 1u;                                   // subnormal: the same last bit as the field 1
  const uint32_t sf = static_cast<uint32_t>(static_cast<unsigned long long>(__double_as_longlong(S.acc.s)) >> 52) & 0x7FFu;
  // errors: multiples of q = 2^(2 (fmin - 150)), their sums at most 2^(k-1) 2^(sf - 1075); exact up to 2^53 q
  return sf + k <= 2u * fmin + 829u;
}

__global__ void __launch_bounds__(kBlockThreads) grad_sqnorm_kernel(CompressArgs A) {
  __shared__ ExactShared sh;
  exact_shared_init(sh);
  __syncthreads();
  // The workgroups walk through the gradients against the direction of the streaming pass that
  // follows: what this pass reads last is what that one reads first, and finds in the memory-side
  // cache (the pair of calls is 18 us shorter on the VGG16-shaped set than with both walking the
  // same way).
  const uint32_t wg = A.reverse ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint32_t l = A.wg2layer[wg];
  const LayerDesc L = A.layers[l];
  const uint32_t wc_local = (wg - L.wg_first) * kWavesPerBlock + (threadIdx.x >> 6);
  SquareSums S;
  if (wc_local < L.wc_count) {
    const uint32_t begin = wc_local * A.chunk;
    const uint32_t end = (L.n - begin) < A.chunk ? L.n : begin + A.chunk;
    squares_of_chunk<false>(L.grad, begin, end, S, sh.digits);
    const uint32_t per_lane = A.chunk / kWaveSize;           // elements of a lane at most (the chunk is a multiple of 256)
    const uint32_t k = 32u - static_cast<uint32_t>(__clz(static_cast<int>(per_lane - 1u)));
    if (__any(!square_sums_exact(S, k))) {
      S = SquareSums{};
      squares_of_chunk<true>(L.grad, begin, end, S, sh.digits);
    }
  }
  const ExactAcc total = exact_block_total(S.acc, sh);
  if (threadIdx.x == 0u) exact_store_part(A.norm_parts, wg, total, sh);
}

__global__ void __launch_bounds__(kBlockThreads) clip_coefficient_kernel(ExactParts parts, uint32_t count,
                                                                          float threshold, float* coef) {
  __shared__ ExactShared sh;
  exact_shared_init(sh);
  __syncthreads();
  ExactPair acc;
  exact_take_parts(acc, parts, 0u, count, sh);
  const double sum = exact_finish(acc, sh);
  if (threadIdx.x == 0u) {
    const double norm = sqrt(sum);
    const double t = static_cast<double>(threshold);
    *coef = static_cast<float>(norm > t ? t / norm : 1.0);
  }
}

hipError_t launch_clip_coefficient(const CompressArgs& a, uint32_t num_wgs, float threshold, float* d_coef, hipStream_t s) {
  hipLaunchKernelGGL(grad_sqnorm_kernel, dim3(num_wgs), dim3(kBlockThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(clip_coefficient_kernel, dim3(1), dim3(kBlockThreads), 0, s, a.norm_parts, num_wgs, threshold, d_coef);
  return hipGetLastError();
}

// ------------------------------------------------------------------ one value per message
// Section 2.2 (quantization of the sparsified residuals): the k values of a message are replaced by
// their average, so that the message carries its indices and one value.  The sum of the values is the
// exactly rounded one (rgc_exact.h), divided by the count in fp64 and rounded to fp32.  The values are
// cut into parts of `part` elements (a multiple of 256, at least 2048, and large enough that the
// longest message has at most kMeanPartsMax parts); workgroup (l, p) takes part p of layer l, a second
// launch adds each layer's parts up and stores the mean.  How the values are cut changes nothing.
// Where the two kernels find a layer's message: in the descriptor table of a compression plan, or in
// the kernel arguments themselves (the entry point that allocates nothing has no table to put them in).
struct MessageRef {
  const float* val;        // the message's values
  const int32_t* count;    // device word: how many there are
  uint32_t cap;            // how many the buffer holds (the layer's k); a larger count is read as this
};

struct TableMessages {
  const LayerDesc* layers;
  __device__ __forceinline__ MessageRef get(uint32_t l) const {
    const LayerDesc& L = layers[l];
    return MessageRef{L.out_val, L.out_count, L.k};
  }
};

constexpr uint32_t kInlineMessagesMax = 64;
struct InlineMessages {
  const float* val[kInlineMessagesMax];
  const int32_t* count[kInlineMessagesMax];
  uint32_t cap[kInlineMessagesMax];
  __device__ __forceinline__ MessageRef get(uint32_t l) const { return MessageRef{val[l], count[l], cap[l]}; }
};

// The length of a message as both kernels read it: never beyond the buffer, so that the parts the
// second kernel adds up are exactly the parts the first one wrote (the grid is sized from the buffers).
__device__ __forceinline__ uint32_t message_length(const MessageRef& M) {
  const int32_t c = *as_global(M.count);
  return c <= 0 ? 0u : (static_cast<uint32_t>(c) < M.cap ? static_cast<uint32_t>(c) : M.cap);
}

template <typename Messages>
__global__ void __launch_bounds__(kBlockThreads) message_part_sums_kernel(Messages src, uint32_t part, ExactParts parts) {
  __shared__ ExactShared sh;
  exact_shared_init(sh);
  __syncthreads();
  const MessageRef M = src.get(blockIdx.x);
  const uint32_t count = message_length(M);
  const uint64_t first = static_cast<uint64_t>(blockIdx.y) * part;
  if (first >= count) return;                               // uniform over the workgroup
  const uint32_t len = static_cast<uint32_t>(count - first < part ? count - first : part);
  const gptr<const float> val = as_global(M.val) + first;
  ExactAcc acc{0.0, 0.0, 0u};
  uint32_t i = threadIdx.x;
  for (; i + 7u * kBlockThreads < len; i += 8u * kBlockThreads) {   // eight loads in flight
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = val[i + static_cast<uint32_t>(j) * kBlockThreads];
#pragma unroll
    for (int j = 0; j < 8; ++j) exact_add_f32(acc, v[j], sh.digits);
  }
  for (; i < len; i += kBlockThreads) exact_add_f32(acc, val[i], sh.digits);
  const ExactAcc total = exact_block_total(acc, sh);
  if (threadIdx.x == 0u) exact_store_part(parts, static_cast<size_t>(blockIdx.x) * kMeanPartsMax + blockIdx.y, total, sh);
}

template <typename Messages>
__global__ void __launch_bounds__(kBlockThreads) message_means_kernel(Messages src, uint32_t part, ExactParts parts, float* means) {
  __shared__ ExactShared sh;
  exact_shared_init(sh);
  __syncthreads();
  const MessageRef M = src.get(blockIdx.x);
  const uint32_t count = message_length(M);
  const uint32_t nparts = static_cast<uint32_t>((static_cast<uint64_t>(count) + part - 1u) / part);
  ExactPair acc;
  exact_take_parts(acc, parts, static_cast<size_t>(blockIdx.x) * kMeanPartsMax, nparts, sh);
  const double sum = exact_finish(acc, sh);
  if (threadIdx.x == 0u) {
    means[blockIdx.x] = count ? static_cast<float>(sum / static_cast<double>(count)) : 0.0f;
  }
}

// Elements per part for messages of at most max_k values: a multiple of 256, at least 2048, and large
// enough that the longest message has at most kMeanPartsMax parts.
static uint32_t mean_part_size(uint32_t max_k) {
  uint32_t part = (max_k + kMeanPartsMax - 1u) / kMeanPartsMax;
  part = (part + 255u) / 256u * 256u;
  return part < 2048u ? 2048u : part;
}

template <typename Messages>
static hipError_t launch_message_means_from(const Messages& src, uint32_t num_layers, uint32_t max_k, const ExactParts& parts,
                                            float* d_means, hipStream_t s) {
  const uint32_t part = mean_part_size(max_k);
  const uint32_t parts_max = (max_k + part - 1u) / part;    // <= kMeanPartsMax
  hipLaunchKernelGGL(message_part_sums_kernel<Messages>, dim3(num_layers, parts_max ? parts_max : 1u), dim3(kBlockThreads), 0, s,
                     src, part, parts);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(message_means_kernel<Messages>, dim3(num_layers), dim3(kBlockThreads), 0, s, src, part, parts, d_means);
  return hipGetLastError();
}

hipError_t launch_message_means(const CompressArgs& a, uint32_t num_layers, uint32_t max_k, const ExactParts& parts,
                                float* d_means, hipStream_t s) {
  return launch_message_means_from(TableMessages{a.layers}, num_layers, max_k, parts, d_means, s);
}

hipError_t launch_accumulate(const CompressArgs& a, uint32_t num_wgs, hipStream_t s) {
  hipLaunchKernelGGL(accumulate_kernel, dim3(num_wgs), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_collect(const CompressArgs& a, uint32_t num_wgs, hipStream_t s) {
  hipLaunchKernelGGL(collect_kernel, dim3(num_wgs), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_lists(const CompressArgs& a, uint32_t num_wgs, hipStream_t s) {
  hipLaunchKernelGGL(lists_kernel, dim3(num_wgs), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_phase(const CompressArgs& a, uint32_t num_wgs, hipStream_t s) {
  if (a.launch >= kFirstLateLaunch) hipLaunchKernelGGL(phase_late_kernel, dim3(num_wgs), dim3(kBlockThreads), 0, s, a);
  else hipLaunchKernelGGL(phase_kernel, dim3(num_wgs), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_poison(LayerState* st, uint32_t num_layers, int mode, hipStream_t s) {
  hipLaunchKernelGGL(poison_kernel, dim3((num_layers + 255u) / 256u), dim3(256), 0, s, st, num_layers, mode);
  return hipGetLastError();
}

hipError_t launch_wave_scan_selftest(uint32_t* io, hipStream_t s) {
  hipLaunchKernelGGL(wave_scan_selftest_kernel, dim3(1), dim3(kBlockThreads), 0, s, io);
  return hipGetLastError();
}

}  // namespace rgc

// ------------------------------------------------------------------ one value per message without any allocation
// rgc_message_means for callers that cannot allocate: no context, no descriptor table, no hipMalloc.  The
// messages are named in the kernel arguments and the partial sums live in an array of the code object,
// of which every device holds its own copy at its own address for as long as the process lives.
static_assert(RGC_NOALLOC_MAX_LAYERS == rgc::kInlineMessagesMax, "the header states the limit of the kernel arguments");
static __device__ __align__(256) long long scratch[rgc::kInlineMessagesMax * rgc::kMeanPartsMax * rgc::kExactWordsPerPart];   // 1.44 MiB

namespace {
constexpr int kScratchDevices = 64;
std::mutex g_scratch_mutex;
long long* g_scratch_ptr[kScratchDevices] = {};    // device address of `scratch` on each device, once asked for
}  // namespace

extern "C" int rgc_message_means_noalloc(const float* const* values, const int32_t* const* counts,
                                         const int32_t* capacity, int32_t num_layers, float* means,
                                         void* hip_stream) {
  if (!values || !counts || !capacity || !means || num_layers < 1) return RGC_EINVAL;
  if (num_layers > RGC_NOALLOC_MAX_LAYERS) return RGC_ENOMEM;          // beyond what the static scratch holds
  if (reinterpret_cast<uintptr_t>(means) & 3u) return RGC_EINVAL;
  rgc::InlineMessages src{};
  uint32_t max_k = 0;
  for (int32_t l = 0; l < num_layers; ++l) {
    if (!values[l] || !counts[l] || capacity[l] < 1) return RGC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(values[l]) | reinterpret_cast<uintptr_t>(counts[l])) & 3u) return RGC_EINVAL;
    src.val[l] = values[l];
    src.count[l] = counts[l];
    src.cap[l] = static_cast<uint32_t>(capacity[l]);
    max_k = src.cap[l] > max_k ? src.cap[l] : max_k;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return rgc::fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= kScratchDevices) return RGC_EINVAL;
  long long* ptr = nullptr;
  {
    // In host code the array's name is only a handle for the symbol; its address on the current device
    // is asked for once per device and used from then on.
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) return rgc::fail_hip(e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
      g_scratch_ptr[dev] = static_cast<long long*>(p);
    }
    ptr = g_scratch_ptr[dev];
  }
  // Nothing in the array has to start at zero: the second kernel reads exactly the parts the first one
  // has just written (both derive them from the same message lengths).
  const rgc::ExactParts parts = rgc::exact_parts_at(ptr, static_cast<size_t>(rgc::kInlineMessagesMax) * rgc::kMeanPartsMax);
  e = rgc::launch_message_means_from(src, static_cast<uint32_t>(num_layers), max_k, parts, means,
                                     static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return rgc::fail_hip(e, "rgc_message_means_noalloc launch");
  return RGC_OK;
}
