// gfx950 kernels of the decompression step (RedSync, Section 2.3: after the Allgather every
// node adds the N gathered sparse messages into a dense array).
//
// Tile ownership: one workgroup owns kTile consecutive positions of one dense buffer, keeps
// them in LDS, adds every worker's entries that fall into the tile and writes the tile once
// (scaled).  Entries of one worker are unique inside a tile, so positions hit by a single
// worker need no ordering; positions hit by several workers are summed strictly in worker
// order by one lane each: a per-position bitmask of the hitting workers (built with
// order-independent atomic ORs) gives every colliding entry its rank among them, the values
// are placed by rank and then added left to right.  The result is therefore independent of
// scheduling and equals the sequential sum bit for bit; no floating-point atomics are used.
//
// A first kernel builds a table with the offset of the first entry of every tile in every
// (worker, layer) message (the messages are sorted by index); rows are tiles, columns are
// workers, so a tile reads all its offsets from two contiguous rows.
//
// The tile kernel is persistent and XCD-aware: every XCD gets one contiguous range of tiles and
// every workgroup a contiguous piece of it, so neighbouring tiles share table rows and message
// cache lines inside one L2.  Inside a run of tiles of one layer the kernel is software
// pipelined: while tile i is accumulated in LDS, the entries of tile i+1 are already being
// loaded into registers and the table row of tile i+2 is in flight, so no tile waits for a
// chain of dependent global loads.
#include "rgc_device.h"

namespace rgc {

namespace {

constexpr uint32_t kTableBlockEntries = 1024;
constexpr uint32_t kPerThread = kEntryCap / kBlockThreads;   // staged entries per thread (4)
constexpr uint32_t kNone = 0xFFFFFFFFu;

constexpr uint32_t kFastR = 8;                         // entries a thread keeps in registers per tile
constexpr uint32_t kStagedCap = 2 * kEntryCap;          // colliding values placed by rank

struct TileLds {
  float acc[kTile];
  uint32_t cnt32[kTile / 4];          // one byte counter per position
  uint32_t cb[kTile / 32];            // positions hit more than once in this batch
  uint32_t cbpre[kTile / 32];         // exclusive popcount prefix of cb
  uint32_t masks[kQMax * kMaskWords]; // per colliding position: which workers hit it
  uint32_t qbase[kQMax];
  union {
    float staged[kStagedCap];         // colliding values in worker order, one run per position
    struct {                          // unpipelined path only: the batch's entries
      uint32_t e_pw[kEntryCap];       // position | local worker << 16, or ~0 if unusable
      float e_val[kEntryCap];
    };
  };
  float staged_generic[kEntryCap];    // the unpipelined path needs its entries and the runs at once
  uint32_t w_start[2][kBatchWorkers];
  uint32_t w_pref[2][kBatchWorkers + 1];
  const int32_t* w_idx[kBatchWorkers];
  const float* w_val[kBatchWorkers];
  uint32_t scan_lds[4];
  uint32_t sh_end, sh_entries, sh_cursor;
};

struct TileGeom {          // one tile, derived arithmetically from its layer
  float* dense;            // start of the tile
  uint32_t first;          // layer-local index of its first position
  uint32_t len;            // positions in it (<= kTile)
  uint32_t row;            // its table row; row + 1 closes it
  uint32_t layer;
};

__device__ __forceinline__ uint32_t layer_of_tile(const DecompressArgs& A, uint32_t tile_id) {
  uint32_t lo = 0, hi = A.num_layers;       // tile_base[lo] <= tile_id < tile_base[hi]
  while (hi - lo > 1u) {
    const uint32_t mid = (lo + hi) >> 1;
    if (A.layers[mid].tile_base <= tile_id) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ TileGeom tile_geom(const DecompressLayer& L, uint32_t layer, uint32_t tile_id) {
  TileGeom g;
  const uint32_t t = tile_id - L.tile_base;
  g.first = t << kTileShift;
  g.dense = L.dense + g.first;
  g.len = (L.n - g.first) < static_cast<uint32_t>(kTile) ? (L.n - g.first) : static_cast<uint32_t>(kTile);
  g.row = L.row_base + t;
  g.layer = layer;
  return g;
}

__device__ __forceinline__ void clear_tile(TileLds& S) {
  for (uint32_t i = threadIdx.x; i < static_cast<uint32_t>(kTile); i += kBlockThreads) S.acc[i] = 0.0f;
}

__device__ __forceinline__ void clear_batch(TileLds& S) {
  for (uint32_t i = threadIdx.x; i < static_cast<uint32_t>(kTile / 4); i += kBlockThreads) S.cnt32[i] = 0u;
  if (threadIdx.x < static_cast<uint32_t>(kTile / 32)) S.cb[threadIdx.x] = 0u;
  if (threadIdx.x == 0) S.sh_cursor = 0u;
}

__device__ __forceinline__ uint32_t hits_of(const TileLds& S, uint32_t p) {
  return (S.cnt32[p >> 2] >> ((p & 3u) * 8u)) & 0xFFu;
}

__device__ __forceinline__ void worker_rank(const TileLds& S, uint32_t q, uint32_t wl, uint32_t& rank, uint32_t& total) {
  rank = 0;
  total = 0;
#pragma unroll
  for (uint32_t mw = 0; mw < static_cast<uint32_t>(kMaskWords); ++mw) {
    const uint32_t mk = S.masks[q * kMaskWords + mw];
    total += static_cast<uint32_t>(__popc(mk));
    if (mw < (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk));
    else if (mw == (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk & ((1u << (wl & 31u)) - 1u)));
  }
}

// The batch's E entries are staged in S.e_pw / S.e_val and counted in S.cnt32 (the staging is
// followed by a barrier).  Adds them into S.acc in worker order.  `pref` = exclusive prefix of
// the per-worker entry counts of the batch (nw + 1 values), used by the rare slow path only.
// Ends with a barrier.
__device__ void accumulate_staged(TileLds& S, uint32_t E, uint32_t nw, const uint32_t* pref) {
  const uint32_t tid = threadIdx.x;
  // ---- positions hit once are final; mark the others
  for (uint32_t e = tid; e < E; e += kBlockThreads) {
    const uint32_t pw = S.e_pw[e];
    if (pw == kNone) continue;
    const uint32_t p = pw & 0xFFFFu;
    if (hits_of(S, p) == 1u) S.acc[p] = __fadd_rn(S.acc[p], S.e_val[e]);
    else atomicOr(&S.cb[p >> 5], 1u << (p & 31u));
  }
  __syncthreads();
  // ---- dense numbering of the colliding positions
  uint32_t nq;
  {
    const uint32_t pc = tid < static_cast<uint32_t>(kTile / 32) ? static_cast<uint32_t>(__popc(S.cb[tid])) : 0u;
    const uint32_t pex = block_excl_scan(pc, S.scan_lds, nq);
    if (tid < static_cast<uint32_t>(kTile / 32)) S.cbpre[tid] = pex;
  }
  __syncthreads();
  if (nq == 0u) return;
  if (nq > static_cast<uint32_t>(kQMax)) {
    // too many colliding positions for the mask table: add worker after worker
    for (uint32_t wl = 0; wl < nw; ++wl) {
      for (uint32_t e = pref[wl] + tid; e < pref[wl + 1u]; e += kBlockThreads) {
        const uint32_t pw = S.e_pw[e];
        if (pw == kNone) continue;
        const uint32_t p = pw & 0xFFFFu;
        if (hits_of(S, p) > 1u) S.acc[p] = __fadd_rn(S.acc[p], S.e_val[e]);
      }
      __syncthreads();
    }
    return;
  }
  for (uint32_t i = tid; i < nq * kMaskWords; i += kBlockThreads) S.masks[i] = 0u;
  __syncthreads();
  // every colliding entry keeps its dense position id in a register across the next phases
  uint32_t myq[kPerThread];
#pragma unroll
  for (uint32_t it = 0; it < kPerThread; ++it) {
    const uint32_t e = tid + it * kBlockThreads;
    myq[it] = kNone;
    if (e < E) {
      const uint32_t pw = S.e_pw[e];
      if (pw != kNone) {
        const uint32_t p = pw & 0xFFFFu, wl = pw >> 16;
        const uint32_t word = S.cb[p >> 5], bit = 1u << (p & 31u);
        if (word & bit) {
          const uint32_t q = S.cbpre[p >> 5] + static_cast<uint32_t>(__popc(word & (bit - 1u)));
          myq[it] = q;
          atomicOr(&S.masks[q * kMaskWords + (wl >> 5)], 1u << (wl & 31u));   // who hits this position
        }
      }
    }
  }
  __syncthreads();
  // ---- the lowest worker of each position reserves its run of staged values
  uint32_t myrank[kPerThread], mytotal[kPerThread];
#pragma unroll
  for (uint32_t it = 0; it < kPerThread; ++it) {
    myrank[it] = 0;
    mytotal[it] = 0;
    if (myq[it] != kNone) {
      const uint32_t wl = S.e_pw[tid + it * kBlockThreads] >> 16;
      worker_rank(S, myq[it], wl, myrank[it], mytotal[it]);
      if (myrank[it] == 0u) S.qbase[myq[it]] = atomicAdd(&S.sh_cursor, mytotal[it]);
    }
  }
  __syncthreads();
  // ---- place the values by rank
#pragma unroll
  for (uint32_t it = 0; it < kPerThread; ++it) {
    if (myq[it] != kNone) {
      const uint32_t at = S.qbase[myq[it]] + myrank[it];
      if (at < static_cast<uint32_t>(kEntryCap)) S.staged_generic[at] = S.e_val[tid + it * kBlockThreads];
    }
  }
  __syncthreads();
  // ---- one lane per colliding position adds its run in worker order
#pragma unroll
  for (uint32_t it = 0; it < kPerThread; ++it) {
    if (myq[it] != kNone && myrank[it] == 0u) {
      const uint32_t p = S.e_pw[tid + it * kBlockThreads] & 0xFFFFu;
      const uint32_t b = S.qbase[myq[it]];
      float sum = S.acc[p];
      for (uint32_t i = 0; i < mytotal[it] && b + i < static_cast<uint32_t>(kEntryCap); ++i)
        sum = __fadd_rn(sum, S.staged_generic[b + i]);
      S.acc[p] = sum;
    }
  }
  __syncthreads();
}

// Same accumulation for entries that live in registers: thread (worker wl, slot) holds up to kFastR
// entries of its worker, p[r] = position in the tile or kNone.  S.cnt32 already counts every
// entry (barrier passed).  Ends with a barrier.
__device__ void accumulate_regs(TileLds& S, const uint32_t (&p)[kFastR], const float (&v)[kFastR], uint32_t wl,
                                uint32_t nw) {
  const uint32_t tid = threadIdx.x;
  bool coll[kFastR];
#pragma unroll
  for (uint32_t r = 0; r < kFastR; ++r) {
    coll[r] = false;
    if (p[r] != kNone) {
      if (hits_of(S, p[r]) == 1u) S.acc[p[r]] = __fadd_rn(S.acc[p[r]], v[r]);
      else { coll[r] = true; atomicOr(&S.cb[p[r] >> 5], 1u << (p[r] & 31u)); }
    }
  }
  __syncthreads();
  uint32_t nq;
  {
    const uint32_t pc = tid < static_cast<uint32_t>(kTile / 32) ? static_cast<uint32_t>(__popc(S.cb[tid])) : 0u;
    const uint32_t pex = block_excl_scan(pc, S.scan_lds, nq);
    if (tid < static_cast<uint32_t>(kTile / 32)) S.cbpre[tid] = pex;
  }
  __syncthreads();
  if (nq == 0u) return;
  if (nq > static_cast<uint32_t>(kQMax)) {
    // too many colliding positions for the mask table: add worker after worker
    for (uint32_t w = 0; w < nw; ++w) {
      if (wl == w) {
#pragma unroll
        for (uint32_t r = 0; r < kFastR; ++r)
          if (coll[r]) S.acc[p[r]] = __fadd_rn(S.acc[p[r]], v[r]);
      }
      __syncthreads();
    }
    return;
  }
  for (uint32_t i = tid; i < nq * kMaskWords; i += kBlockThreads) S.masks[i] = 0u;
  __syncthreads();
  uint32_t q[kFastR];
#pragma unroll
  for (uint32_t r = 0; r < kFastR; ++r) {
    q[r] = kNone;
    if (coll[r]) {
      const uint32_t word = S.cb[p[r] >> 5], bit = 1u << (p[r] & 31u);
      q[r] = S.cbpre[p[r] >> 5] + static_cast<uint32_t>(__popc(word & (bit - 1u)));
      atomicOr(&S.masks[q[r] * kMaskWords + (wl >> 5)], 1u << (wl & 31u));
    }
  }
  __syncthreads();
  uint32_t rank[kFastR], total[kFastR];
#pragma unroll
  for (uint32_t r = 0; r < kFastR; ++r) {
    rank[r] = 0;
    total[r] = 0;
    if (coll[r]) {
      worker_rank(S, q[r], wl, rank[r], total[r]);
      if (rank[r] == 0u) S.qbase[q[r]] = atomicAdd(&S.sh_cursor, total[r]);
    }
  }
  __syncthreads();
#pragma unroll
  for (uint32_t r = 0; r < kFastR; ++r) {
    if (coll[r]) {
      const uint32_t at = S.qbase[q[r]] + rank[r];
      if (at < kStagedCap) S.staged[at] = v[r];
    }
  }
  __syncthreads();
#pragma unroll
  for (uint32_t r = 0; r < kFastR; ++r) {
    if (coll[r] && rank[r] == 0u) {
      const uint32_t b = S.qbase[q[r]];
      const uint32_t n = (b + total[r] <= kStagedCap) ? total[r] : (b < kStagedCap ? kStagedCap - b : 0u);
      float sum = S.acc[p[r]];
      uint32_t i = 0;
      for (; i + 4u <= n; i += 4u) {          // loads first, then the dependent adds, in worker order
        const float a0 = S.staged[b + i], a1 = S.staged[b + i + 1u], a2 = S.staged[b + i + 2u], a3 = S.staged[b + i + 3u];
        sum = __fadd_rn(__fadd_rn(__fadd_rn(__fadd_rn(sum, a0), a1), a2), a3);
      }
      for (; i < n; ++i) sum = __fadd_rn(sum, S.staged[b + i]);
      S.acc[p[r]] = sum;
    }
  }
  __syncthreads();
}

// Write the finished tile once (scaled).  Followed by a barrier at the caller.
__device__ __forceinline__ void write_tile(const TileLds& S, const TileGeom& g, float scale, uint32_t add_to_dst) {
  const uint32_t tid = threadIdx.x;
  const gptr<float> d = as_global(g.dense);
  const bool vec = ((reinterpret_cast<uintptr_t>(g.dense) & 15u) == 0u) && ((g.len & 3u) == 0u);
  if (vec) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    const gptr<vf4> d4 = as_global(reinterpret_cast<vf4*>(g.dense));
    for (uint32_t i = tid; i < g.len / 4u; i += kBlockThreads) {
      vf4 o;
      o.x = __fmul_rn(S.acc[4 * i + 0], scale);
      o.y = __fmul_rn(S.acc[4 * i + 1], scale);
      o.z = __fmul_rn(S.acc[4 * i + 2], scale);
      o.w = __fmul_rn(S.acc[4 * i + 3], scale);
      if (add_to_dst) {
        const vf4 old = d4[i];
        o.x = __fadd_rn(old.x, o.x); o.y = __fadd_rn(old.y, o.y);
        o.z = __fadd_rn(old.z, o.z); o.w = __fadd_rn(old.w, o.w);
      }
      d4[i] = o;
    }
  } else {
    for (uint32_t i = tid; i < g.len; i += kBlockThreads) {
      float o = __fmul_rn(S.acc[i], scale);
      if (add_to_dst) o = __fadd_rn(d[i], o);
      d[i] = o;
    }
  }
}

// One tile, any number of workers, any number of entries: workers are taken in batches that fit
// the staging buffers; every batch fetches its own offsets and entries (no prefetching).
// S.acc must be cleared (barrier passed); ends with the tile accumulated in S.acc and a barrier.
__device__ void tile_generic(const DecompressArgs& A, TileLds& S, const TileGeom& g) {
  const uint32_t tid = threadIdx.x;
  const uint32_t N = A.num_workers;
  uint32_t w0 = 0;
  while (w0 < N) {
    const uint32_t nb = (N - w0) < static_cast<uint32_t>(kBatchWorkers) ? (N - w0) : static_cast<uint32_t>(kBatchWorkers);
    uint32_t s = 0, c = 0;
    const int32_t* ip = nullptr;
    const float* vp = nullptr;
    if (tid < nb) {
      const MsgDesc md = A.msgs[static_cast<size_t>(g.layer) * N + w0 + tid];
      const uint32_t* row = A.tab + static_cast<size_t>(g.row) * N + w0 + tid;
      s = row[0];
      uint32_t e = row[N];
      if (e > md.count) e = md.count;     // the table never exceeds the message; stay in bounds anyway
      c = e > s ? e - s : 0u;
      ip = md.idx;
      vp = md.val;
    }
    if (tid == 0) S.sh_end = nb;
    clear_batch(S);
    uint32_t batch_total;
    const uint32_t ex = block_excl_scan(c, S.scan_lds, batch_total);
    if (tid < nb && ex + c > static_cast<uint32_t>(kEntryCap)) atomicMin(&S.sh_end, tid);
    __syncthreads();
    const uint32_t nw = S.sh_end;
    if (nw == 0u) {
      // the first worker alone exceeds the staging capacity: its positions are unique, add directly
      if (tid == 0) { S.w_start[0][0] = s; S.w_pref[0][0] = c; S.w_idx[0] = ip; S.w_val[0] = vp; }
      __syncthreads();
      const uint32_t s0 = S.w_start[0][0], c0 = S.w_pref[0][0];
      const gptr<const int32_t> ip0 = as_global(S.w_idx[0]);
      const gptr<const float> vp0 = as_global(S.w_val[0]);
      for (uint32_t j = tid; j < c0; j += kBlockThreads) {
        const uint32_t p = static_cast<uint32_t>(ip0[s0 + j]) - g.first;
        if (p < g.len) S.acc[p] = __fadd_rn(S.acc[p], vp0[s0 + j]);
      }
      __syncthreads();
      w0 += 1u;
      continue;
    }
    if (tid < nw) { S.w_start[0][tid] = s; S.w_pref[0][tid] = ex; S.w_idx[tid] = ip; S.w_val[tid] = vp; }
    if (tid == nw - 1u) { S.w_pref[0][nw] = ex + c; S.sh_entries = ex + c; }
    __syncthreads();
    const uint32_t E = S.sh_entries;
    if (E != 0u) {
      // fetch: all loads of a thread are issued before the first is used
      uint32_t lo_[kPerThread], idx_[kPerThread];
      float val_[kPerThread];
#pragma unroll
      for (uint32_t it = 0; it < kPerThread; ++it) {
        const uint32_t e = tid + it * kBlockThreads;
        lo_[it] = kNone;
        idx_[it] = 0;
        val_[it] = 0.0f;
        if (e < E) {
          uint32_t lo = 0, hi = nw;
          while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (S.w_pref[0][mid] <= e) lo = mid; else hi = mid;
          }
          const uint32_t j = S.w_start[0][lo] + (e - S.w_pref[0][lo]);
          lo_[it] = lo;
          idx_[it] = static_cast<uint32_t>(as_global(S.w_idx[lo])[j]);
          val_[it] = as_global(S.w_val[lo])[j];
        }
      }
#pragma unroll
      for (uint32_t it = 0; it < kPerThread; ++it) {
        const uint32_t e = tid + it * kBlockThreads;
        if (e < E) {
          const uint32_t p = idx_[it] - g.first;
          if (p < g.len) {
            S.e_pw[e] = p | (lo_[it] << 16);
            S.e_val[e] = val_[it];
            atomicAdd(&S.cnt32[p >> 2], 1u << ((p & 3u) * 8u));
          } else {
            S.e_pw[e] = kNone;
          }
        }
      }
      __syncthreads();
      accumulate_staged(S, E, nw, S.w_pref[0]);
    }
    w0 += nw;
    __syncthreads();
  }
}

}  // namespace

// ------------------------------------------------------------------ tile-offset table
__global__ void __launch_bounds__(kBlockThreads) decompress_table_kernel(DecompressArgs A) {
  const BlockDesc bd = A.blocks[blockIdx.x];
  const MsgDesc md = A.msgs[bd.msg];              // messages are stored [layer][worker]
  const uint32_t N = A.num_workers;
  const uint32_t layer = bd.msg / N, w = bd.msg % N;
  const DecompressLayer L = A.layers[layer];
  const uint32_t ntiles = L.tiles;
  uint32_t* col = A.tab + static_cast<size_t>(L.row_base) * N + w;   // col[t * N] = first entry of tile t
  const gptr<const int32_t> midx = as_global(md.idx);
  if (md.count == 0u) {
    for (uint32_t t = threadIdx.x; t <= ntiles; t += kBlockThreads) col[static_cast<size_t>(t) * N] = 0u;
    return;
  }
  const uint32_t stop = (md.count - bd.first) < kTableBlockEntries ? md.count : bd.first + kTableBlockEntries;
  for (uint32_t j = bd.first + threadIdx.x; j < stop; j += kBlockThreads) {
    uint32_t cur = static_cast<uint32_t>(midx[j]) >> kTileShift;
    if (cur >= ntiles) cur = ntiles - 1u;                 // out-of-range index: stay inside the table
    uint32_t first = 0u;
    if (j != 0u) {
      uint32_t prev = static_cast<uint32_t>(midx[j - 1u]) >> kTileShift;
      if (prev >= ntiles) prev = ntiles - 1u;
      first = prev + 1u;
    }
    for (uint32_t t = first; t <= cur; ++t) col[static_cast<size_t>(t) * N] = j;
    if (j == md.count - 1u)
      for (uint32_t t = cur + 1u; t <= ntiles; ++t) col[static_cast<size_t>(t) * N] = md.count;
  }
}

// ------------------------------------------------------------------ tile accumulation
__global__ void __launch_bounds__(kBlockThreads) decompress_tiles_kernel(DecompressArgs A) {
  __shared__ TileLds S;
  const uint32_t tid = threadIdx.x;
  const uint32_t N = A.num_workers;
  // Workgroups are dealt to the 8 XCDs round-robin by index.  Every XCD gets one contiguous
  // range of tiles, and the workgroups of an XCD take its tiles round-robin, so at any moment
  // they work on neighbouring tiles: one 128-byte line of a message holds the entries of about
  // 8 tiles, is fetched from HBM once and is then found in that XCD's L2 by the 7 other
  // workgroups that need it (a blocked assignment makes the concurrent working set of an XCD
  // as large as its L2 and fetches every line 8 times).
  uint32_t t_first, t_last, stride;
  {
    const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const uint32_t per_xcd = (A.num_tiles + 7u) >> 3;
    const uint32_t x0 = xcd * per_xcd < A.num_tiles ? xcd * per_xcd : A.num_tiles;
    const uint32_t x1 = x0 + per_xcd < A.num_tiles ? x0 + per_xcd : A.num_tiles;
    if (A.debug & 8u) {          // blocked: a contiguous piece per workgroup
      const uint32_t per_slot = (x1 - x0 + slots - 1u) / slots;
      t_first = x0 + slot * per_slot < x1 ? x0 + slot * per_slot : x1;
      t_last = t_first + per_slot < x1 ? t_first + per_slot : x1;
      stride = 1u;
    } else {
      t_first = x0 + slot < x1 ? x0 + slot : x1;
      t_last = x1;
      stride = slots;
    }
  }
  const bool pipelined = N >= 1u && N <= static_cast<uint32_t>(kBatchWorkers);
  // threads per worker on the pipelined path: 256 / (N rounded up to a power of two), >= 2
  uint32_t tpw_shift = 1;
  while (tpw_shift < 8u && (N << (tpw_shift + 1u)) <= static_cast<uint32_t>(kBlockThreads)) ++tpw_shift;
  const uint32_t tpw = 1u << tpw_shift;

  uint32_t tile_id = t_first;
  while (tile_id < t_last) {
    // ---- a run of consecutive tiles of one layer
    const uint32_t layer = layer_of_tile(A, tile_id);
    const DecompressLayer L = A.layers[layer];
    const uint32_t run_end = (L.tile_base + L.tiles) < t_last ? (L.tile_base + L.tiles) : t_last;

    if (!pipelined) {
      for (; tile_id < run_end; tile_id += stride) {
        const TileGeom g = tile_geom(L, layer, tile_id);
        clear_tile(S);
        __syncthreads();
        tile_generic(A, S, g);
        write_tile(S, g, A.scale, A.add_to_dst);
        __syncthreads();
      }
      continue;
    }

    // ---- pipelined run.  Thread (worker wl, part) owns, of its worker's entries inside a tile,
    // the groups of four consecutive entries number part, part + T, ... (T threads per worker),
    // kFastR entries at most, fetched with one 16-byte load per group and array: an L1 lookup
    // costs the same for 4 bytes as for 16, and one-entry gathers made this kernel bound by
    // them.  A tile where some worker has more entries takes the unpipelined path.  The
    // entries stay in registers from the prefetch to the end of their tile.
    const uint32_t wl = tid & ((static_cast<uint32_t>(kBlockThreads) >> tpw_shift) - 1u);
    const uint32_t part = tid >> (8u - tpw_shift);
    const bool has_worker = wl < N;
    uint32_t my_count = 0;
    gptr<const int32_t> my_idx = nullptr;
    gptr<const float> my_val = nullptr;
    if (has_worker) {
      const MsgDesc md = A.msgs[static_cast<size_t>(layer) * N + wl];
      my_idx = as_global(md.idx);
      my_val = as_global(md.val);
      my_count = md.count;
    }
    const uint32_t* tabw = A.tab + (has_worker ? wl : 0u);
    auto row_at = [&](uint32_t row) -> uint32_t {
      if (!has_worker) return 0u;
      const uint32_t v = tabw[static_cast<size_t>(row) * N];
      return v < my_count ? v : my_count;        // the table never exceeds the message; stay in bounds anyway
    };
    const uint32_t row0 = L.row_base + (tile_id - L.tile_base);
    uint32_t r_start = row_at(row0);             // entry range of the tile being prefetched
    uint32_t r_end = row_at(row0 + 1u);
    uint32_t r_start2 = 0, r_end2 = 0;           // entry range of this workgroup's tile after it
    if (tile_id + stride < run_end) {
      r_start2 = row_at(row0 + stride);
      r_end2 = row_at(row0 + stride + 1u);
    }

    uint32_t nx_idx[kFastR];
    float nx_val[kFastR];
    uint32_t nx_cnt = 0;                         // how many of them exist (this thread)
    bool nx_generic = false;
    typedef uint32_t vu4 __attribute__((ext_vector_type(4), aligned(4)));
    typedef float vf4u __attribute__((ext_vector_type(4), aligned(4)));
    auto prefetch = [&]() {
      const uint32_t c = r_end > r_start ? r_end - r_start : 0u;
      nx_generic = __syncthreads_or(c > tpw * kFastR ? 1 : 0) != 0;
      nx_cnt = 0;
#pragma unroll
      for (uint32_t r = 0; r < kFastR / 4u; ++r) {
        const uint32_t off = 4u * (part + r * tpw);          // first entry of this group inside the tile
#pragma unroll
        for (uint32_t j = 0; j < 4u; ++j) { nx_idx[4u * r + j] = 0; nx_val[4u * r + j] = 0.0f; }
        if (!nx_generic && off < c) {
          const uint32_t at = r_start + off;
          const uint32_t have = (c - off) < 4u ? (c - off) : 4u;
          if (at + 4u <= my_count) {                         // the 16-byte load stays inside the message
            const vu4 qi = *reinterpret_cast<gptr<const vu4>>(my_idx + at);
            const vf4u qv = *reinterpret_cast<gptr<const vf4u>>(my_val + at);
            nx_idx[4u * r + 0] = qi.x; nx_idx[4u * r + 1] = qi.y; nx_idx[4u * r + 2] = qi.z; nx_idx[4u * r + 3] = qi.w;
            nx_val[4u * r + 0] = qv.x; nx_val[4u * r + 1] = qv.y; nx_val[4u * r + 2] = qv.z; nx_val[4u * r + 3] = qv.w;
          } else {
#pragma unroll
            for (uint32_t j = 0; j < 4u; ++j) {
              if (j < have) {
                nx_idx[4u * r + j] = static_cast<uint32_t>(my_idx[at + j]);
                nx_val[4u * r + j] = my_val[at + j];
              }
            }
          }
          nx_cnt = 4u * r + have;
        }
      }
    };
    prefetch();

    for (; tile_id < run_end; tile_id += stride) {
      const TileGeom g = tile_geom(L, layer, tile_id);
      const bool generic = nx_generic;
      clear_tile(S);
      clear_batch(S);
      __syncthreads();
      // ---- this tile's entries were prefetched during the previous tile: count the hits
      uint32_t cur_p[kFastR];
      float cur_v[kFastR];
#pragma unroll
      for (uint32_t r = 0; r < kFastR; ++r) {
        cur_p[r] = kNone;
        cur_v[r] = nx_val[r];
        if (!generic && r < nx_cnt) {
          const uint32_t p = nx_idx[r] - g.first;
          if (p < g.len) {
            cur_p[r] = p;
            atomicAdd(&S.cnt32[p >> 2], 1u << ((p & 3u) * 8u));
          }
        }
      }
      __syncthreads();
      // ---- start fetching the next tile of the run
      if (tile_id + stride < run_end) {
        r_start = r_start2;
        r_end = r_end2;
        if (tile_id + 2u * stride < run_end) {
          const uint32_t row2 = L.row_base + (tile_id - L.tile_base) + 2u * stride;
          r_start2 = row_at(row2);
          r_end2 = row_at(row2 + 1u);
        }
        if (!(A.debug & 2u)) prefetch();
      }
      // ---- accumulate and write this tile
      if (generic) {
        tile_generic(A, S, g);                   // some worker has too many entries here: unpipelined
      } else if (!(A.debug & 1u)) {
        accumulate_regs(S, cur_p, cur_v, wl, N);
      }
      if (!(A.debug & 4u)) write_tile(S, g, A.scale, A.add_to_dst);
      __syncthreads();
    }
  }
}

hipError_t launch_decompress_table(const DecompressArgs& a, hipStream_t s) {
  if (a.num_blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(decompress_table_kernel, dim3(a.num_blocks), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_decompress_tiles(const DecompressArgs& a, hipStream_t s) {
  if (a.num_tiles == 0) return hipSuccess;
  // persistent: at most 4 workgroups per CU (LDS), a multiple of 8 so that every XCD gets its share
  uint32_t grid = ((a.num_tiles + 7u) / 8u) * 8u;
  if (grid > a.max_grid) grid = a.max_grid;
  hipLaunchKernelGGL(decompress_tiles_kernel, dim3(grid), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace rgc
