// Wave64 / workgroup primitives for the gfx950 kernels: ballot-popcount ranks, DPP prefix
// scans, a 256-thread block scan.  Device code only.
#pragma once

#include "rgc_internal.h"

namespace rgc {

// Tensor pointers reach the kernels through descriptor tables in memory, so the compiler sees
// generic ("flat") pointers and would emit flat_load/flat_store, which also tick the LDS
// counter and make every LDS wait a wait for all outstanding global traffic.  Everything the
// library touches through such pointers is global memory: say so.
template <typename T>
using gptr = __attribute__((address_space(1))) T*;

template <typename T>
__device__ __forceinline__ gptr<T> as_global(T* p) {
  return (gptr<T>)p;
}

__device__ __forceinline__ uint32_t lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Number of set bits of `mask` that belong to lanes below the calling lane.
__device__ __forceinline__ uint32_t rank_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t popc64(unsigned long long m) {
  return static_cast<uint32_t>(__popcll(m));
}

template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_shift_add(uint32_t v) {
  // lanes without a source (shifted in from outside the row, or rows masked off) add 0
  uint32_t t = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
      0, static_cast<int>(v), kCtrl, kRowMask, 0xF, false));
  return v + t;
}

// Inclusive prefix sum over the 64 lanes of a wave using DPP row shifts and row broadcasts.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  v = dpp_shift_add<0x111, 0xF>(v);  // row_shr:1
  v = dpp_shift_add<0x112, 0xF>(v);  // row_shr:2
  v = dpp_shift_add<0x114, 0xF>(v);  // row_shr:4
  v = dpp_shift_add<0x118, 0xF>(v);  // row_shr:8   -> inclusive scan inside each row of 16
  v = dpp_shift_add<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
  v = dpp_shift_add<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
  return v;
}

__device__ __forceinline__ uint32_t wave_total(uint32_t incl) {
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(incl), 63));
}

// Exclusive prefix sum over the 256 threads of a workgroup.  `lds` holds >= 4 words.
// Contains barriers: every thread of the workgroup must call it.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* lds, uint32_t& total) {
  const uint32_t incl = wave_incl_scan(v);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 63u) lds[wave] = incl;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (uint32_t w = 0; w < kWavesPerBlock; ++w) {
    const uint32_t t = lds[w];
    off += (w < wave) ? t : 0u;
    tot += t;
  }
  total = tot;
  return off + incl - v;
}

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// "Last workgroup of the layer" election.  Contract: everything the elected workgroup will
// read from this phase was written with device-scope atomics or st_agent() (both go to the
// device's coherence point, unlike plain stores which may sit in one XCD's L2 until the kernel
// ends), and is read back with ld_agent().  Waiting for the wave's outstanding memory
// operations before the counter increment is then all the ordering needed; a full
// __threadfence() here would force an L2 write-back per workgroup and costs several times the
// streaming pass itself.
// Returns true in every thread of exactly one workgroup per (layer, phase): the one whose
// increment completes the count.  That workgroup also resets the counter.
// The election is two-level: workgroups first count themselves into the counter of their group of
// kElectGroup consecutive workgroups, the last of a group counts the group into the layer's
// counter.  Thousands of workgroups finishing a short phase together otherwise queue up on one
// address (a same-address device atomic takes ~10-25 ns, i.e. ~100 us for 4000 workgroups).
constexpr uint32_t kElectGroup = 32;

__device__ __forceinline__ bool last_block_of_layer(uint32_t* layer_done, uint32_t* group_done, uint32_t wg_in_layer,
                                                    uint32_t wg_count, uint32_t* lds_flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t grp = wg_in_layer / kElectGroup;
    const uint32_t groups = (wg_count + kElectGroup - 1u) / kElectGroup;
    const uint32_t in_grp = (grp + 1u == groups) ? wg_count - grp * kElectGroup : kElectGroup;
    bool last = false;
    if (atomicAdd(&group_done[grp], 1u) + 1u == in_grp) {
      st_agent(&group_done[grp], 0u);
      if (atomicAdd(layer_done, 1u) + 1u == groups) {
        st_agent(layer_done, 0u);
        last = true;
      }
    }
    *lds_flag = last ? 1u : 0u;
  }
  __syncthreads();
  return *lds_flag != 0u;
}

// ---------------------------------------------------------------- shared by every pass over a layer
__device__ __forceinline__ uint32_t fbits(float x) { return __float_as_uint(x); }

typedef float vf4 __attribute__((ext_vector_type(4)));   // one 16-byte access per lane

// The accumulate of Algorithm 1 and its variants (Sections 2.4, 2.5): every gradient element is
// first multiplied with the clipping coefficient (1 when there is none: an exact product), then
//   plain:                a = V + g
//   momentum correction:  u = fma(m, u, g),   a = V + u
//   its Nesterov form:    u = m * (u + g),    a = (V + u) + g      (every operation rounded)
struct AccumRule {
  float m;       // momentum factor
  float scale;   // clipping coefficient
};

template <bool kMom, bool kNest>
__device__ __forceinline__ void accum4(const float (&g)[4], const float (&v)[4], float (&u)[4],
                                       const AccumRule& r, float (&a)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float gs = __fmul_rn(r.scale, g[j]);
    if constexpr (kMom && kNest) {
      u[j] = __fmul_rn(r.m, __fadd_rn(u[j], gs));
      a[j] = __fadd_rn(__fadd_rn(v[j], u[j]), gs);
    } else if constexpr (kMom) {
      u[j] = __fmaf_rn(r.m, u[j], gs);
      a[j] = __fadd_rn(v[j], u[j]);
    } else {
      a[j] = __fadd_rn(v[j], gs);
    }
  }
}

// The zeros that mask a sent entry out of the residual (and the velocity) are isolated 4-byte
// writes, one cache line in a thousand.  Left dirty in the caches they are written to DRAM one
// by one while the next streaming pass runs and cost it about a tenth of its bandwidth; stored
// with the streaming hint they leave the caches early and cost half of that.
__device__ __forceinline__ void mask_store(gptr<float> p) { __builtin_nontemporal_store(0.0f, p); }

}  // namespace rgc
