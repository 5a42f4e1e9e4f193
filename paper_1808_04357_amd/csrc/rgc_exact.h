// Device side of the exactly rounded sums: the squared norm behind the clipping coefficient
// (Section 2.4), the mean of a one-value message (Section 2.2) and the mean of |a| that starts the
// threshold search (Algorithm 3).  The paper fixes neither precision nor order for these additions;
// they are taken as the sum of the terms rounded ONCE to fp64 (nearest, ties to even), which no
// grouping of the work over lanes, waves and workgroups can change.
//
// How: a lane keeps a running fp64 sum s and, beside it, the sum c of the rounding errors of s
// (each addition's error is itself a double and is recovered without rounding).  c has errors of its
// own only when terms more than about a hundred binary orders apart meet; such an error goes, as an
// integer, into a long fixed-point number ("digits": 32 bits each, held in 64-bit words so that
// carries can wait) in the LDS.  Lanes, waves and workgroups are combined the same way (two
// error-free additions, anything left over into the digits), every workgroup leaves (s, c, flags)
// and, if it used them, its digits; the last kernel adds the parts up the same way once more, puts
// the final s and c into the digits as well, carries, and rounds the integer to fp64.
// Terms that are not finite are counted in flags instead: a NaN, or infinities of both signs, make
// the sum NaN, infinities of one sign make it that infinity.
#pragma once

#include "rgc_device.h"

namespace rgc {

constexpr int kExactBias = 298;             // digit 0, bit 0 stands for 2^-298: the square of the smallest fp32 step
constexpr uint32_t kExactSpilled = 1u;      // the part's digits are in use
constexpr uint32_t kExactNaN = 2u;
constexpr uint32_t kExactPosInf = 4u;
constexpr uint32_t kExactNegInf = 8u;

struct ExactAcc {
  double s;
  double c;
  uint32_t flags;
};

struct ExactShared {                        // one per workgroup, in the LDS
  long long digits[kExactDigits];
  double s[kBlockThreads / kWaveSize];
  double c[kBlockThreads / kWaveSize];
  uint32_t flags[kBlockThreads / kWaveSize];
};

// s + e == a + b, s the rounded sum (Knuth's branch-free form: no order of magnitudes assumed).
__device__ __forceinline__ void two_sum(double a, double b, double& s, double& e) {
  s = a + b;
  const double bv = s - a;
  e = (a - (s - bv)) + (b - bv);
}

// Adds the finite double x, a multiple of 2^-298 below 2^342, to the digits.
__device__ __noinline__ void exact_spill(double x, long long* digits) {
  const unsigned long long bits = static_cast<unsigned long long>(__double_as_longlong(x));
  const uint32_t field = static_cast<uint32_t>(bits >> 52) & 0x7FFu;
  unsigned long long mant = bits & 0xFFFFFFFFFFFFFull;
  int pos;                                  // bit position of mant's last bit in the long number
  if (field != 0u) {
    mant |= 1ull << 52;
    pos = static_cast<int>(field) - 1075 + kExactBias;
  } else {
    pos = -1074 + kExactBias;
  }
  if (pos < 0) {                            // the bits below 2^-298 are zeros
    mant = pos > -64 ? mant >> -pos : 0ull;
    pos = 0;
  }
  if (mant == 0ull) return;
  const uint32_t d = static_cast<uint32_t>(pos) >> 5, r = static_cast<uint32_t>(pos) & 31u;
  if (d + 2u >= static_cast<uint32_t>(kExactDigits)) return;   // beyond any sum of fp32 terms or squares
  const unsigned long long low = mant << r;
  const unsigned long long high = r ? mant >> (64u - r) : 0ull;
  unsigned long long piece[3] = {low & 0xFFFFFFFFull, low >> 32, high};
  const bool neg = (bits >> 63) != 0ull;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    if (piece[i] != 0ull)
      atomicAdd(reinterpret_cast<unsigned long long*>(digits + d + i), neg ? 0ull - piece[i] : piece[i]);
  }
}

__device__ __forceinline__ void exact_add(ExactAcc& a, double x, long long* digits) {
  double s, e1;
  two_sum(a.s, x, s, e1);
  a.s = s;
  if (e1 != 0.0) {
    double c, e2;
    two_sum(a.c, e1, c, e2);
    a.c = c;
    if (e2 != 0.0) {
      exact_spill(e2, digits);
      a.flags |= kExactSpilled;
    }
  }
}

__device__ __forceinline__ uint32_t exact_class(float v) {      // 0 for a finite value
  const uint32_t b = fbits(v);
  if ((b & 0x7F800000u) != 0x7F800000u) return 0u;
  return (b & 0x007FFFFFu) ? kExactNaN : ((b >> 31) ? kExactNegInf : kExactPosInf);
}

__device__ __forceinline__ void exact_add_f32(ExactAcc& a, float v, long long* digits) {
  const uint32_t cls = exact_class(v);
  a.flags |= cls;
  exact_add(a, cls ? 0.0 : static_cast<double>(v), digits);
}

// v * v: 24 bits times 24 bits, exact in fp64 and never out of its range.
__device__ __forceinline__ void exact_add_square(ExactAcc& a, float v, long long* digits) {
  const uint32_t cls = exact_class(v);
  a.flags |= cls == kExactNegInf ? kExactPosInf : cls;
  const double x = cls ? 0.0 : static_cast<double>(v);
  exact_add(a, x * x, digits);
}

// (s, c) of b joins a; what neither double can hold goes to the digits if `spill` (the caller lets
// exactly one lane of those that compute the same combination do that).
__device__ __forceinline__ void exact_join(ExactAcc& a, double bs, double bc, uint32_t bflags, bool spill, long long* digits) {
  double s, e1, c, e2, c2, e3;
  two_sum(a.s, bs, s, e1);
  two_sum(a.c, bc, c, e2);
  two_sum(c, e1, c2, e3);
  a.s = s;
  a.c = c2;
  a.flags |= bflags;
  if (spill && (e2 != 0.0 || e3 != 0.0)) {
    if (e2 != 0.0) exact_spill(e2, digits);
    if (e3 != 0.0) exact_spill(e3, digits);
    a.flags |= kExactSpilled;
  }
}

// Clears the digits; the caller puts a barrier between this and the first addition.
__device__ __forceinline__ void exact_shared_init(ExactShared& sh) {
  if (threadIdx.x < static_cast<uint32_t>(kExactDigits)) sh.digits[threadIdx.x] = 0ll;
}

// Every thread of the workgroup brings its accumulator (all zero if it had nothing to add); thread 0
// returns with the workgroup's, and the workgroup's digits are complete then.  Holds two barriers.
__device__ __forceinline__ ExactAcc exact_block_total(ExactAcc a, ExactShared& sh) {
  const uint32_t lane = lane_id();
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t waves = blockDim.x >> 6;
#pragma unroll
  for (uint32_t off = 32u; off >= 1u; off >>= 1) {
    const double bs = __shfl_down(a.s, off);
    const double bc = __shfl_down(a.c, off);
    const uint32_t bf = __shfl_down(a.flags, off);
    exact_join(a, bs, bc, bf, lane < off, sh.digits);
  }
  // (the flags, the note of a spill among them, have travelled down the tree with the sums)
  if (lane == 0u) {
    sh.s[wave] = a.s;
    sh.c[wave] = a.c;
    sh.flags[wave] = a.flags;
  }
  __syncthreads();
  if (threadIdx.x == 0u) {
    a.flags = sh.flags[0];
    for (uint32_t w = 1u; w < waves; ++w) exact_join(a, sh.s[w], sh.c[w], sh.flags[w], true, sh.digits);
  }
  __syncthreads();
  return a;
}

// Thread 0 stores the workgroup's part.
__device__ __forceinline__ void exact_store_part(const ExactParts& P, size_t part, const ExactAcc& total, const ExactShared& sh) {
  const gptr<double> sc = as_global(P.sc);
  sc[2u * part] = total.s;
  sc[2u * part + 1u] = total.c;
  as_global(P.flags)[part] = total.flags;
  if (total.flags & kExactSpilled) {
    const gptr<long long> dg = as_global(P.digits) + part * kExactDigits;
    for (int i = 0; i < kExactDigits; ++i) dg[i] = sh.digits[i];
  }
}

// The last kernel of a sum.  Every thread of the workgroup takes the parts first + threadIdx.x,
// first + threadIdx.x + blockDim.x, ... below first + count, eight of them asked for at a time (one thread
// adding up a few dozen parts is a chain of memory round trips otherwise).  The parts' running sums go to one
// accumulator and their error sums to another: the two kinds lie some fifty binary orders apart, and one
// accumulator for both would have to put nearly every error sum into the digits.
struct ExactPair {
  ExactAcc sums{0.0, 0.0, 0u};
  ExactAcc errs{0.0, 0.0, 0u};
};

__device__ __forceinline__ void exact_take_parts(ExactPair& a, const ExactParts& P, size_t first, uint32_t count, ExactShared& sh) {
  constexpr uint32_t kBatch = 8u;
  const gptr<const double> sc = as_global(static_cast<const double*>(P.sc));
  const gptr<const unsigned long long> fl = as_global(static_cast<const unsigned long long*>(P.flags));
  for (uint32_t i0 = threadIdx.x; i0 < count; i0 += kBatch * blockDim.x) {
    double s[kBatch], c[kBatch];
    uint32_t f[kBatch];
#pragma unroll
    for (uint32_t j = 0; j < kBatch; ++j) {
      const uint32_t i = i0 + j * blockDim.x;
      const bool in = i < count;
      const size_t part = first + (in ? i : i0);
      s[j] = sc[2u * part];
      c[j] = sc[2u * part + 1u];
      f[j] = in ? static_cast<uint32_t>(fl[part]) : 0xFFFFFFFFu;      // ~0: no such part
    }
#pragma unroll
    for (uint32_t j = 0; j < kBatch; ++j) {
      if (f[j] == 0xFFFFFFFFu) continue;
      exact_add(a.sums, s[j], sh.digits);
      exact_add(a.errs, c[j], sh.digits);
      a.sums.flags |= f[j];
      if (f[j] & kExactSpilled) {
        const gptr<const long long> dg = as_global(static_cast<const long long*>(P.digits)) + (first + i0 + j * blockDim.x) * kExactDigits;
        long long v[kExactDigits];                     // all asked for before the first is used
#pragma unroll
        for (int d = 0; d < kExactDigits; ++d) v[d] = dg[d];
#pragma unroll
        for (int d = 0; d < kExactDigits; ++d)
          if (v[d] != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&sh.digits[d]), static_cast<unsigned long long>(v[d]));
      }
    }
  }
}

// Thread 0, after exact_block_total: the sum of everything the workgroup took, rounded once.
__device__ __noinline__ double exact_round(const ExactAcc& total, ExactShared& sh);

// Every thread brings what exact_take_parts gave it; thread 0 returns with the sum of all parts, rounded once
// (the other threads with nothing of use).  Holds barriers.
__device__ __forceinline__ double exact_finish(const ExactPair& mine, ExactShared& sh) {
  const ExactAcc errs = exact_block_total(mine.errs, sh);
  ExactAcc sums = exact_block_total(mine.sums, sh);
  if (threadIdx.x != 0u) return 0.0;
  if (errs.s != 0.0) exact_spill(errs.s, sh.digits);
  if (errs.c != 0.0) exact_spill(errs.c, sh.digits);
  sums.flags |= errs.flags;
  return exact_round(sums, sh);
}

__device__ __noinline__ double exact_round(const ExactAcc& total, ExactShared& sh) {
  const uint32_t f = total.flags;
  if ((f & kExactNaN) || ((f & kExactPosInf) && (f & kExactNegInf))) return __longlong_as_double(0x7FF8000000000000ll);
  if (f & kExactPosInf) return __longlong_as_double(0x7FF0000000000000ll);
  if (f & kExactNegInf) return __longlong_as_double(static_cast<long long>(0xFFF0000000000000ull));
  long long* dg = sh.digits;
  if (total.s != 0.0) exact_spill(total.s, dg);
  if (total.c != 0.0) exact_spill(total.c, dg);
  long long carry = 0;
  for (int i = 0; i < kExactDigits; ++i) {            // every digit into [0, 2^32), the sign ends up in carry
    const long long t = dg[i] + carry;
    dg[i] = t & 0xFFFFFFFFll;
    carry = t >> 32;
  }
  const bool neg = carry < 0;
  if (neg) {                                          // magnitude of a negative total: two's complement
    long long c2 = 1;
    for (int i = 0; i < kExactDigits; ++i) {
      const long long t = ((~dg[i]) & 0xFFFFFFFFll) + c2;
      dg[i] = t & 0xFFFFFFFFll;
      c2 = t >> 32;
    }
  }
  int td = kExactDigits - 1;
  while (td >= 0 && dg[td] == 0ll) --td;
  if (td < 0) return 0.0;
  const int top = td * 32 + (31 - __clz(static_cast<int>(static_cast<uint32_t>(dg[td]))));
  const int last = top >= 53 ? top - 52 : 0;          // last bit that is kept
  const int w = last >> 5, r = last & 31;
  auto digit = [&](int i) { return i < kExactDigits ? static_cast<unsigned long long>(dg[i]) : 0ull; };
  const unsigned long long low = digit(w) | (digit(w + 1) << 32);
  unsigned long long mant = (low >> r) | (r ? digit(w + 2) << (64 - r) : 0ull);
  mant &= (1ull << 53) - 1ull;
  if (last > 0) {
    const int h = last - 1;                           // the first dropped bit
    const bool half = ((digit(h >> 5) >> (h & 31)) & 1ull) != 0ull;
    bool rest = (digit(h >> 5) & ((1ull << (h & 31)) - 1ull)) != 0ull;
    for (int i = 0; i < (h >> 5) && !rest; ++i) rest = dg[i] != 0ll;
    if (half && (rest || (mant & 1ull))) ++mant;
  }
  const double v = ldexp(static_cast<double>(mant), last - kExactBias);
  return neg ? -v : v;
}

}  // namespace rgc
