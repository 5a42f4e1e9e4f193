// gfx950 kernels of the decompression step (RedSync, Section 2.3: after the Allgather every
// node adds the N gathered sparse messages into a dense array).
//
// Tile ownership: one workgroup owns kTile consecutive positions of one dense buffer, adds every
// worker's entries that fall into the tile and writes the tile once (scaled).  Entries of one
// worker are unique inside a tile, so positions hit by a single worker need no ordering: the
// first entry to reach a position stores its value there.  A position hit by several workers
// gets a row with one slot per worker: every later hitter stores its value into its own slot,
// the first one's value is moved from the tile into its slot, the other slots hold +0, and one
// lane adds the row from slot 0 upwards.  Adding +0 leaves a partial sum as it is, so this is
// the sequential sum over the workers bit for bit, independent of scheduling; no floating-point
// atomics are used.
//
// The fast kernel (up to kBatchWorkers workers) is persistent and XCD-aware: every XCD gets one
// contiguous range of tiles and every workgroup a contiguous piece of it, which it walks through
// once.  Four lanes serve one worker and keep a window of its (sorted) message in registers, so
// a message is read once, front to back, in 64-byte pieces, and no table of per-tile offsets is
// needed: a binary search finds where the workgroup's first tile of a layer starts, afterwards
// the count of consumed entries says where the next tile starts.  Blocks that enter the window
// are loaded while the current tile is being finished.
//
// A tile with more colliding positions than the kernel has rows (rare) takes them a row-set at a
// time.  With more than kBatchWorkers workers a second kernel does the job instead: workers in
// batches, colliding entries sorted by their rank in a per-position worker bitmask, entry ranges
// from a table of per-tile offsets that a third kernel builds first.
#include "rgc_device.h"

namespace rgc {

namespace {

constexpr uint32_t kTableBlockEntries = 1024;
constexpr uint32_t kPerThread = kEntryCap / kBlockThreads;   // staged entries per thread (4)
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint32_t kWords = kTile / 32;                 // words of a one-bit-per-position map

typedef uint32_t vu2l __attribute__((ext_vector_type(2)));
typedef uint32_t vu4l __attribute__((ext_vector_type(4)));
typedef float vf4 __attribute__((ext_vector_type(4)));

struct TileGeom {          // one tile, derived arithmetically from its layer
  float* dense;            // start of the tile
  uint32_t first;          // layer-local index of its first position
  uint32_t len;            // positions in it (<= kTile)
  uint32_t row;            // its table entry inside a worker's row; row + 1 closes it
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

// The tiles of workgroup `wg` of a persistent grid: t_first, t_first + stride, ... < t_last.
// Workgroups are dealt to the 8 XCDs round-robin by index.  Every XCD gets one contiguous range
// of tiles, and the workgroups of an XCD take its tiles round-robin, so at any moment they work on
// neighbouring tiles: one 128-byte line of a message holds the entries of about 4 tiles, is
// fetched from HBM once and is then found in that XCD's L2 by the other workgroups that need it
// (a blocked assignment makes the concurrent working set of an XCD as large as its L2 and fetches
// every line 8 times).
__device__ __forceinline__ void tiles_of_workgroup(uint32_t num_tiles, uint32_t& t_first, uint32_t& t_last,
                                                   uint32_t& stride) {
  const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
  const uint32_t per_xcd = (num_tiles + 7u) >> 3;
  const uint32_t x0 = xcd * per_xcd < num_tiles ? xcd * per_xcd : num_tiles;
  const uint32_t x1 = x0 + per_xcd < num_tiles ? x0 + per_xcd : num_tiles;
  t_first = x0 + slot < x1 ? x0 + slot : x1;
  t_last = x1;
  stride = slots;
}

// =================================================================== generic tiles
// Any number of workers and entries.  Workers are taken in batches of kBatchWorkers; inside a
// batch a per-position bitmask of the hitting workers (built with order-independent atomic ORs)
// gives every colliding entry its rank among them, the values are placed by rank and then added
// left to right by one lane per position.
struct alignas(16) GenericLds {
  float acc[kTile];
  uint32_t cnt32[kTile / 4];          // one byte counter per position
  uint32_t cb[kWords];                // positions hit more than once in this batch
  uint32_t cbpre[kWords];             // exclusive popcount prefix of cb
  uint32_t masks[kQMax * kMaskWords]; // per colliding position: which workers hit it
  uint32_t qbase[kQMax];
  uint32_t e_pw[kEntryCap];           // position | local worker << 16, or ~0 if unusable
  float e_val[kEntryCap];
  float staged[kEntryCap];            // colliding values in worker order, one run per position
  uint32_t w_start[kBatchWorkers];
  uint32_t w_pref[kBatchWorkers + 1];
  const int32_t* w_idx[kBatchWorkers];
  const float* w_val[kBatchWorkers];
  uint32_t scan_lds[4];
  uint32_t sh_end, sh_entries, sh_cursor;
};

__device__ __forceinline__ void clear_tile(GenericLds& S) {
  for (uint32_t i = threadIdx.x; i < static_cast<uint32_t>(kTile); i += kBlockThreads) S.acc[i] = 0.0f;
}

__device__ __forceinline__ void clear_batch(GenericLds& S) {
  for (uint32_t i = threadIdx.x; i < static_cast<uint32_t>(kTile / 4); i += kBlockThreads) S.cnt32[i] = 0u;
  if (threadIdx.x < kWords) S.cb[threadIdx.x] = 0u;
  if (threadIdx.x == 0) S.sh_cursor = 0u;
}

__device__ __forceinline__ uint32_t hits_of(const GenericLds& S, uint32_t p) {
  return (S.cnt32[p >> 2] >> ((p & 3u) * 8u)) & 0xFFu;
}

// Rank of worker `wl` among the workers in the mask of colliding position q, and their number.
__device__ __forceinline__ void worker_rank(const uint32_t* masks, uint32_t q, uint32_t wl, uint32_t& rank,
                                            uint32_t& total) {
  rank = 0;
  total = 0;
#pragma unroll
  for (uint32_t mw = 0; mw < static_cast<uint32_t>(kMaskWords); ++mw) {
    const uint32_t mk = masks[q * kMaskWords + mw];
    total += static_cast<uint32_t>(__popc(mk));
    if (mw < (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk));
    else if (mw == (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk & ((1u << (wl & 31u)) - 1u)));
  }
}

// The batch's E entries are staged in S.e_pw / S.e_val and counted in S.cnt32 (the staging is
// followed by a barrier).  Adds them into S.acc in worker order.  `pref` = exclusive prefix of
// the per-worker entry counts of the batch (nw + 1 values), used by the rare slow path only.
// Ends with a barrier.
__device__ void accumulate_staged(GenericLds& S, uint32_t E, uint32_t nw, const uint32_t* pref) {
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
    const uint32_t pc = tid < kWords ? static_cast<uint32_t>(__popc(S.cb[tid])) : 0u;
    const uint32_t pex = block_excl_scan(pc, S.scan_lds, nq);
    if (tid < kWords) S.cbpre[tid] = pex;
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
      worker_rank(S.masks, myq[it], wl, myrank[it], mytotal[it]);
      if (myrank[it] == 0u) S.qbase[myq[it]] = atomicAdd(&S.sh_cursor, mytotal[it]);
    }
  }
  __syncthreads();
  // ---- place the values by rank
#pragma unroll
  for (uint32_t it = 0; it < kPerThread; ++it) {
    if (myq[it] != kNone) {
      const uint32_t at = S.qbase[myq[it]] + myrank[it];
      if (at < static_cast<uint32_t>(kEntryCap)) S.staged[at] = S.e_val[tid + it * kBlockThreads];
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
        sum = __fadd_rn(sum, S.staged[b + i]);
      S.acc[p] = sum;
    }
  }
  __syncthreads();
}

// Write the finished tile once (scaled).  Followed by a barrier at the caller.
__device__ __forceinline__ void write_tile(const GenericLds& S, const TileGeom& g, float scale, uint32_t add_to_dst) {
  const uint32_t tid = threadIdx.x;
  const gptr<float> d = as_global(g.dense);
  const bool vec = ((reinterpret_cast<uintptr_t>(g.dense) & 15u) == 0u) && ((g.len & 3u) == 0u);
  if (vec) {
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
__device__ __forceinline__ uint32_t lower_bound_idx(gptr<const int32_t> idx, uint32_t count, uint32_t target) {
  uint32_t lo = 0, hi = count;                        // idx[lo - 1] < target <= idx[hi]
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (static_cast<uint32_t>(idx[mid]) < target) lo = mid + 1u; else hi = mid;
  }
  return lo;
}

__device__ void tile_generic(const DecompressArgs& A, GenericLds& S, const TileGeom& g) {
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
      const uint32_t* row = A.tab + static_cast<size_t>(w0 + tid) * A.tab_stride + g.row;
      s = row[0];
      uint32_t e = row[1];
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
      if (tid == 0) { S.w_start[0] = s; S.w_pref[0] = c; S.w_idx[0] = ip; S.w_val[0] = vp; }
      __syncthreads();
      const uint32_t s0 = S.w_start[0], c0 = S.w_pref[0];
      const gptr<const int32_t> ip0 = as_global(S.w_idx[0]);
      const gptr<const float> vp0 = as_global(S.w_val[0]);
      for (uint32_t j = tid; j < c0; j += kBlockThreads) {
        const uint32_t p = static_cast<uint32_t>(ip0[s0 + j]) - g.first;
        if (p < g.len) S.acc[p] = __fadd_rn(S.acc[p], vp0[A.one_value ? 0u : s0 + j]);
      }
      __syncthreads();
      w0 += 1u;
      continue;
    }
    if (tid < nw) { S.w_start[tid] = s; S.w_pref[tid] = ex; S.w_idx[tid] = ip; S.w_val[tid] = vp; }
    if (tid == nw - 1u) { S.w_pref[nw] = ex + c; S.sh_entries = ex + c; }
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
            if (S.w_pref[mid] <= e) lo = mid; else hi = mid;
          }
          const uint32_t j = S.w_start[lo] + (e - S.w_pref[lo]);
          lo_[it] = lo;
          idx_[it] = static_cast<uint32_t>(as_global(S.w_idx[lo])[j]);
          val_[it] = as_global(S.w_val[lo])[A.one_value ? 0u : j];   // one value for the whole message (Section 2.2), or one per entry
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
      accumulate_staged(S, E, nw, S.w_pref);
    }
    w0 += nw;
    __syncthreads();
  }
}

// =================================================================== fast tiles
constexpr uint32_t kFastShift = 9;
constexpr uint32_t kFastThreads = 1u << kFastShift;   // 8 waves per tile
constexpr uint32_t kRows = 48;                  // positions hit more than once in one tile
constexpr uint32_t kRowStride = kBatchWorkers + 4;   // floats; the +4 spreads the rows over the LDS banks

// seen / cb / nq exist twice: tile i uses set i & 1 while the other set is being cleared.
struct alignas(16) FastLds {
  float acc[kTile];                          // the tile; all zero between tiles
  float rows[kRows * kRowStride];            // per colliding position one slot per worker; all +0 between tiles
  uint32_t seen[2][kWords];                  // positions hit at all
  uint32_t cb[2][kWords];                    // positions hit more than once
  uint32_t nq[2];                            // how many of those
  uint16_t run_p[kRows];                     // the position a row belongs to
  uint32_t pre_cb[kWords];                   // exclusive popcount prefix of cb (only when the rows do not suffice)
  uint8_t qmap[kTile];                       // the row of a colliding position (valid where cb is set)
  uint8_t who[kTile];                        // the worker whose entry reached a position first (valid where seen is set)
};
static_assert(sizeof(FastLds) <= 80 * 1024, "two 8-wave workgroups per CU");
static_assert(kWords % 64u == 0u, "a wave scans the colliding-position bitmap, a whole number of words per lane");
static_assert(kRows <= 64 && kRows < 256, "one wave adds the rows; row numbers are bytes");

// threadIdx.x behind a veil: what is derived from it is recomputed where it is used instead of
// being kept in a register across the whole tile loop (the loop is short of registers for eight
// waves per SIMD, and a spilled value comes back through a vector-memory wait).
__device__ __forceinline__ uint32_t fresh_tid() {
  uint32_t t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
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
  const gptr<uint32_t> col = as_global(A.tab + static_cast<size_t>(w) * A.tab_stride + L.row_base);   // col[t] = first entry of tile t
  const gptr<const int32_t> midx = as_global(md.idx);
  if (md.count == 0u) {
    for (uint32_t t = threadIdx.x; t <= ntiles; t += kBlockThreads) col[t] = 0u;
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
    for (uint32_t t = first; t <= cur; ++t) col[t] = j;
    if (j == md.count - 1u)
      for (uint32_t t = cur + 1u; t <= ntiles; ++t) col[t] = md.count;
  }
}

// ------------------------------------------------------------------ tile accumulation, fast path
namespace {

// Sum over the four lanes of a quad (lanes 4k .. 4k+3), in every lane of it.
__device__ __forceinline__ uint32_t quad_sum(uint32_t v) {
  v += static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  return v;
}

__device__ __forceinline__ uint32_t quad_lane0(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0x00, 0xF, 0xF, true));  // quad_perm [0,0,0,0]
}

}  // namespace

// A workgroup owns a contiguous range of tiles and walks through it once.  Four neighbouring lanes
// serve one worker and keep a window of its message in registers: two blocks of 16 consecutive
// entries (block b in slot b & 1, four entries per lane), so that a block comes from memory once,
// as one 64-byte piece per array, and serves the four or so tiles its entries fall into.  E is
// the number of the worker's entries that lie before the current tile; the window is the two
// blocks starting at the one that holds entry E, and the blocks that enter it are loaded while
// the tile is being finished.  There is no per-tile offset table: E starts from a binary search
// at the first tile of a layer and then advances by what each tile consumes.
template <bool kStreamMsgs, bool kOneValue>
__global__ void __launch_bounds__(kFastThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
decompress_tiles_kernel(DecompressArgs A) {
  __shared__ FastLds S;
  const uint32_t tid = threadIdx.x;
  const uint32_t N = A.num_workers;                    // 1 .. kBatchWorkers (the host checks)
  // this workgroup's tiles: a contiguous piece of its XCD's contiguous range
  uint32_t t_first, t_last;
  {
    const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const uint32_t per_xcd = (A.num_tiles + 7u) >> 3;
    const uint32_t x0 = xcd * per_xcd < A.num_tiles ? xcd * per_xcd : A.num_tiles;
    const uint32_t x1 = x0 + per_xcd < A.num_tiles ? x0 + per_xcd : A.num_tiles;
    const uint32_t per_slot = (x1 - x0 + slots - 1u) / slots;
    t_first = x0 + slot * per_slot < x1 ? x0 + slot * per_slot : x1;
    t_last = t_first + per_slot < x1 ? t_first + per_slot : x1;
  }
  const uint32_t wl = tid >> 2, q = tid & 3u;          // worker, lane of the worker
  const bool has_worker = wl < N;
  const uint32_t row_groups = (N + 3u) / 4u;           // a row's slots, in groups of four

  for (uint32_t i = tid; i < static_cast<uint32_t>(kTile); i += kFastThreads) S.acc[i] = 0.0f;
  for (uint32_t i = tid; i < kRows * kRowStride; i += kFastThreads) S.rows[i] = 0.0f;
  for (uint32_t i = tid; i < 2u * kWords; i += kFastThreads) { (&S.seen[0][0])[i] = 0u; (&S.cb[0][0])[i] = 0u; }
  if (tid < 2u) S.nq[tid] = 0u;
  __syncthreads();
  uint32_t par = 0;                                    // which set of maps the current tile uses

  typedef uint32_t vu4 __attribute__((ext_vector_type(4), aligned(4)));
  typedef float vf4u __attribute__((ext_vector_type(4), aligned(4)));

  uint32_t tile_id = t_first;
  while (tile_id < t_last) {
    // ---- a run of this workgroup's tiles inside one layer
    const uint32_t layer = layer_of_tile(A, tile_id);
    const DecompressLayer L = A.layers[layer];
    const uint32_t run_end = (L.tile_base + L.tiles) < t_last ? (L.tile_base + L.tiles) : t_last;

    uint32_t my_count = 0;
    gptr<const int32_t> my_idx = nullptr;
    gptr<const float> my_val = nullptr;
    if (has_worker) {
      const MsgDesc md = A.msgs[static_cast<size_t>(layer) * N + wl];
      my_idx = as_global(md.idx);
      my_val = as_global(md.val);
      my_count = md.count;
    }
    // messages that carry one value for all their entries (the average of Section 2.2's
    // quantization): it is read once per run and stands in for every entry's value
    float my_one = 0.0f;
    if constexpr (kOneValue) {
      if (my_count != 0u) my_one = my_val[0];
    }
    auto value_at = [&](uint32_t e) -> float {
      if constexpr (kOneValue) return my_one; else return my_val[e];
    };
    // E: entries of the worker before the run's first tile (the messages are sorted by index)
    // The four lanes of a worker search together: each step they probe the four inner fifth points
    // of the range at once, so the search is log5 deep instead of log2.  A run that starts a
    // layer needs no search.
    uint32_t E = 0;
    {
      const uint32_t target = (tile_id - L.tile_base) << kTileShift;
      uint32_t lo = 0, hi = target != 0u ? my_count : 0u;   // idx[lo - 1] < target <= idx[hi]
      while (__builtin_amdgcn_ballot_w64(lo < hi) != 0ull) {
        const uint32_t span = hi - lo;                       // the same in the four lanes of a quad
        const uint32_t s5 = span / 5u, r5 = span % 5u;
        auto fifths = [&](uint32_t j) { return s5 * j + (r5 * j + 4u) / 5u; };   // ceil(j * span / 5)
        // probe points lo + ceil((q+1) * span / 5) - 1: ascending, all inside [lo, hi)
        const uint32_t at = lo + fifths(q + 1u) - 1u;
        uint32_t below = 0;
        if (lo < hi) below = static_cast<uint32_t>(my_idx[at]) < target ? 1u : 0u;
        const uint32_t nb = quad_sum(below);                 // the probes are ordered: the first nb lie below
        if (lo < hi) {
          const uint32_t new_lo = nb == 0u ? lo : lo + fifths(nb);              // one past probe nb-1
          const uint32_t new_hi = nb == 4u ? hi : lo + fifths(nb + 1u) - 1u;    // probe nb
          lo = new_lo; hi = new_hi;
        }
      }
      E = lo;
    }

    // the window: slot s holds block have[s] (kNone: nothing), this lane its entries 4q .. 4q+3
    uint32_t b_idx[2][4];
    float b_val[2][4];
    uint32_t have[2] = {kNone, kNone};
#pragma unroll
    for (uint32_t sl = 0; sl < 2u; ++sl)
#pragma unroll
      for (uint32_t r = 0; r < 4u; ++r) { b_idx[sl][r] = kNone; b_val[sl][r] = 0.0f; }
    // Bring the blocks that hold entries E .. (two blocks) into their slots; entries past the
    // end of the message read as index kNone, which no tile contains.
    auto fill_window = [&]() {
      const uint32_t bc = E >> 4;
#pragma unroll
      for (uint32_t sl = 0; sl < 2u; ++sl) {
        const uint32_t want = bc + ((sl ^ bc) & 1u);
        if (want != have[sl]) {
          have[sl] = want;
          const uint32_t at = want * 16u + 4u * q;
          if (at + 4u <= my_count) {
            // Streaming loads when the caller alternates compression and decompression: what the
            // memory-side cache holds of the compression's tensors is worth more to the next call than
            // the other half of this 128-byte line, which then comes from DRAM again four tiles later.
            // (a template parameter, not a run-time flag: merged into one branch-free load the two
            // flavours would lose the hint)
            vu4 qi;
            vf4u qv;
            if constexpr (kStreamMsgs) {
              qi = __builtin_nontemporal_load(reinterpret_cast<gptr<const vu4>>(my_idx + at));
              if constexpr (!kOneValue) qv = __builtin_nontemporal_load(reinterpret_cast<gptr<const vf4u>>(my_val + at));
            } else {
              qi = *reinterpret_cast<gptr<const vu4>>(my_idx + at);
              if constexpr (!kOneValue) qv = *reinterpret_cast<gptr<const vf4u>>(my_val + at);
            }
            if constexpr (kOneValue) qv = vf4u{my_one, my_one, my_one, my_one};
            b_idx[sl][0] = qi.x; b_idx[sl][1] = qi.y; b_idx[sl][2] = qi.z; b_idx[sl][3] = qi.w;
            b_val[sl][0] = qv.x; b_val[sl][1] = qv.y; b_val[sl][2] = qv.z; b_val[sl][3] = qv.w;
          } else {
#pragma unroll
            for (uint32_t r = 0; r < 4u; ++r) {
              b_idx[sl][r] = kNone;
              b_val[sl][r] = 0.0f;
              if (at + r < my_count) {
                b_idx[sl][r] = static_cast<uint32_t>(my_idx[at + r]);
                b_val[sl][r] = value_at(at + r);
              }
            }
          }
        }
      }
    };
    fill_window();

    for (; tile_id < run_end; ++tile_id, par ^= 1u) {
      const TileGeom g = tile_geom(L, layer, tile_id);
      uint32_t* const seen = S.seen[par];
      uint32_t* const cb = S.cb[par];
      // ---- mark the positions hit, and those hit again; whoever finds a position hit for the
      // second time gives it a row (the numbering depends on timing, the sums do not)
      // The first entry to reach a position puts its value straight into the tile and leaves its
      // worker's number there; should the position turn out to be hit again, the lane that adds the
      // position's row up moves that value into the row first.  Returns whether the entry came later.
      auto mark = [&](uint32_t p, float v) -> bool {
        const uint32_t bit = 1u << (p & 31u);
        if (atomicOr(&seen[p >> 5], bit) & bit) {
          if (!(atomicOr(&cb[p >> 5], bit) & bit)) {
            const uint32_t qq = atomicAdd(&S.nq[par], 1u);
            if (qq < kRows) { S.qmap[p] = static_cast<uint8_t>(qq); S.run_p[qq] = static_cast<uint16_t>(p); }
          }
          return true;
        }
        S.acc[p] = __fadd_rn(0.0f, v);
        S.who[p] = static_cast<uint8_t>(fresh_tid() >> 2);
        return false;
      };
      uint32_t mine = 0;                           // entries of this lane inside the tile
      uint32_t last_in = 0;                        // the window's last entry is inside the tile
      uint32_t late = 0;                           // bit 4*sl+r: that window entry was not the first at its position
#pragma unroll
      for (uint32_t sl = 0; sl < 2u; ++sl) {
#pragma unroll
        for (uint32_t r = 0; r < 4u; ++r) {
          const uint32_t p = b_idx[sl][r] - g.first;
          if (p < g.len) {
            if (mark(p, b_val[sl][r])) late |= 1u << (4u * sl + r);
            ++mine;
            if (r == 3u && q == 3u && have[sl] == (E >> 4) + 1u) last_in = 1u;
          }
        }
      }
      // the worker's entries inside the tile go on beyond the window (rare): straight from memory,
      // here and again below
      const uint32_t beyond = (E >> 4) * 16u + 32u;
      const bool more = quad_sum(last_in) != 0u;
      if (more) {
        for (uint32_t e = beyond + q; e < my_count; e += 4u) {
          const uint32_t p = static_cast<uint32_t>(my_idx[e]) - g.first;
          if (p >= g.len) break;
          (void)mark(p, value_at(e));
          ++mine;
        }
      }
      const uint32_t consumed = quad_sum(mine);
      __syncthreads();
      const uint32_t nq = S.nq[par];
      // ---- clear the maps the previous tile used
      if (tid == 0u) S.nq[par ^ 1u] = 0u;
      if (tid < kWords) { S.seen[par ^ 1u][tid] = 0u; S.cb[par ^ 1u][tid] = 0u; }
      // one lane per row adds the row's slots in worker order; the slots of the workers that did
      // not hit the position hold +0, which leaves every partial sum as it is (a partial sum is
      // never -0)
      auto sum_rows = [&](uint32_t count) {
        const uint32_t row = fresh_tid();
        if (row < count) {
          {
            const uint32_t p = S.run_p[row];
            S.rows[row * kRowStride + S.who[p]] = S.acc[p];   // the position's first arrival (it may be there already)
          }
          const vf4* const r4 = reinterpret_cast<const vf4*>(S.rows + row * kRowStride);
          float sum = 0.0f;
          uint32_t gi = 0;
          vf4 c0 = r4[0], c1 = r4[1];            // the next eight slots are on their way while these are added
          for (;;) {
            gi += 2u;
            const bool again = gi < row_groups;
            vf4 n0 = c0, n1 = c1;
            if (again) { n0 = r4[gi]; n1 = r4[gi + 1u]; }
            sum = __fadd_rn(__fadd_rn(__fadd_rn(__fadd_rn(sum, c0.x), c0.y), c0.z), c0.w);
            sum = __fadd_rn(__fadd_rn(__fadd_rn(__fadd_rn(sum, c1.x), c1.y), c1.z), c1.w);
            if (!again) break;
            c0 = n0; c1 = n1;
          }
          S.acc[S.run_p[row]] = sum;
        }
        __syncthreads();
        // the rows go back to +0
        for (uint32_t i = row; i < count * (kRowStride / 4u); i += kFastThreads)
          reinterpret_cast<vf4*>(S.rows)[i] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
      };
      // run f(position, value) over this lane's entries inside the tile
      auto for_my_entries = [&](auto&& f) {
        if (mine == 0u) return;
        uint32_t first = g.first;
        asm volatile("" : "+s"(first));          // recompute the positions here rather than keep (and spill) them
#pragma unroll
        for (uint32_t sl = 0; sl < 2u; ++sl) {
#pragma unroll
          for (uint32_t r = 0; r < 4u; ++r) {
            const uint32_t p = b_idx[sl][r] - first;
            if (p < g.len) f(p, b_val[sl][r]);
          }
        }
        if (more) {
          for (uint32_t e = beyond + q; e < my_count; e += 4u) {
            const uint32_t p = static_cast<uint32_t>(my_idx[e]) - first;
            if (p >= g.len) break;
            f(p, value_at(e));
          }
        }
      };
      if (nq > kRows) {
        // ---- more colliding positions than rows (rare): they are taken kRows at a time, numbered by
        // position (popcount prefix over the bitmap; every wave computes the same prefix and writes
        // it, so it may read it back at once)
        {
          constexpr uint32_t kPerLane = kWords / 64u;     // words of the bitmap a lane takes
          const uint32_t ln = fresh_tid() & 63u;
          uint32_t c[kPerLane], total = 0u;
#pragma unroll
          for (uint32_t i = 0; i < kPerLane; ++i) {
            c[i] = static_cast<uint32_t>(__popc(cb[kPerLane * ln + i]));
            total += c[i];
          }
          uint32_t run = wave_incl_scan(total) - total;
#pragma unroll
          for (uint32_t i = 0; i < kPerLane; ++i) {
            S.pre_cb[kPerLane * ln + i] = run;
            run += c[i];
          }
        }
        const uint32_t my_slot = fresh_tid() >> 2;   // = wl
        for (uint32_t d0 = 0; d0 < nq; d0 += kRows) {
          for_my_entries([&](uint32_t p, float v) {
            const uint32_t word = cb[p >> 5], sh = p & 31u;
            if ((word >> sh) & 1u) {
              const uint32_t d = S.pre_cb[p >> 5] + static_cast<uint32_t>(__popc(word & ((1u << sh) - 1u))) - d0;
              if (d < kRows) { S.rows[d * kRowStride + my_slot] = v; S.run_p[d] = static_cast<uint16_t>(p); }
            }
          });
          __syncthreads();
          sum_rows(nq - d0 < kRows ? nq - d0 : kRows);
          __syncthreads();
        }
        E += consumed;
        fill_window();
      } else {
        // ---- positions hit once are final; the entries that came later put their value into their
        // worker's slot of the position's row
        if (nq != 0u) {
          const uint32_t my_slot = fresh_tid() >> 2;   // = wl
          if (late != 0u) {
            uint32_t first = g.first;
            asm volatile("" : "+s"(first));        // recompute the positions here rather than keep (and spill) them
#pragma unroll
            for (uint32_t sl = 0; sl < 2u; ++sl) {
#pragma unroll
              for (uint32_t r = 0; r < 4u; ++r) {
                if ((late >> (4u * sl + r)) & 1u) {
                  const uint32_t p = b_idx[sl][r] - first;
                  S.rows[static_cast<uint32_t>(S.qmap[p]) * kRowStride + my_slot] = b_val[sl][r];
                }
              }
            }
          }
          if (more) {                              // beyond the window: whoever is on a colliding position (a first arrival twice: harmless)
            for (uint32_t e = beyond + q; e < my_count; e += 4u) {
              const uint32_t p = static_cast<uint32_t>(my_idx[e]) - g.first;
              if (p >= g.len) break;
              if ((cb[p >> 5] >> (p & 31u)) & 1u) S.rows[static_cast<uint32_t>(S.qmap[p]) * kRowStride + my_slot] = value_at(e);
            }
          }
          __syncthreads();
        }
        // the tile's entries are used up: move the window on; its new blocks arrive while the tile is finished
        E += consumed;
        fill_window();
        if (nq != 0u) sum_rows(nq);
      }
      // ---- write the tile (scaled) and leave its accumulator cleared
      const bool vec = ((reinterpret_cast<uintptr_t>(g.dense) & 15u) == 0u) && ((g.len & 3u) == 0u);
      const uint32_t out_tid = fresh_tid();
      if (vec) {
        const gptr<vf4> d4 = as_global(reinterpret_cast<vf4*>(g.dense));
        vf4* const acc4 = reinterpret_cast<vf4*>(S.acc);
#pragma unroll
        for (uint32_t j = 0; j < static_cast<uint32_t>(kTile) / (4u * kFastThreads); ++j) {
          const uint32_t i4 = out_tid + j * kFastThreads;
          if (4u * i4 < g.len) {
            const vf4 a = acc4[i4];
            acc4[i4] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
            vf4 o;
            o.x = __fmul_rn(a.x, A.scale); o.y = __fmul_rn(a.y, A.scale);
            o.z = __fmul_rn(a.z, A.scale); o.w = __fmul_rn(a.w, A.scale);
            if (A.add_to_dst) {
              const vf4 old = d4[i4];
              o.x = __fadd_rn(old.x, o.x); o.y = __fadd_rn(old.y, o.y);
              o.z = __fadd_rn(old.z, o.z); o.w = __fadd_rn(old.w, o.w);
            }
            __builtin_nontemporal_store(o, &d4[i4]);       // written once, not read here again: keep it from pushing the message lines out of the L2
          }
        }
      } else {
        const gptr<float> d = as_global(g.dense);
        for (uint32_t i = out_tid; i < g.len; i += kFastThreads) {
          float o = __fmul_rn(S.acc[i], A.scale);
          S.acc[i] = 0.0f;
          if (A.add_to_dst) o = __fadd_rn(d[i], o);
          d[i] = o;
        }
      }
      __syncthreads();                             // the next tile's first arrivals write into the accumulator that this one has just cleared
    }
  }
}

// ------------------------------------------------------------------ tile accumulation, any number of workers
__global__ void __launch_bounds__(kBlockThreads) decompress_generic_kernel(DecompressArgs A) {
  __shared__ GenericLds S;
  uint32_t t_first, t_last, stride;
  tiles_of_workgroup(A.num_tiles, t_first, t_last, stride);
  for (uint32_t tile_id = t_first; tile_id < t_last; tile_id += stride) {
    const uint32_t layer = layer_of_tile(A, tile_id);
    const TileGeom g = tile_geom(A.layers[layer], layer, tile_id);
    clear_tile(S);
    __syncthreads();
    tile_generic(A, S, g);
    write_tile(S, g, A.scale, A.add_to_dst);
    __syncthreads();
  }
}

// ------------------------------------------------------------------ precondition check (on request)
// One workgroup per message: every index must lie inside the layer and exceed its predecessor
// (Section 2.3: a message is what compression emitted).  Violations are ORed into *status
// (bit 0: range, bit 1: order); nothing else is touched.
__global__ void __launch_bounds__(kBlockThreads) decompress_validate_kernel(DecompressArgs A, uint32_t* status) {
  const MsgDesc md = A.msgs[blockIdx.x];            // messages are stored [layer][worker]
  const uint32_t n = A.layers[blockIdx.x / A.num_workers].n;
  const gptr<const int32_t> idx = as_global(md.idx);
  uint32_t bad = 0;
  for (uint32_t j = threadIdx.x; j < md.count; j += kBlockThreads) {
    const uint32_t v = static_cast<uint32_t>(idx[j]);                 // a negative index reads as a huge one
    if (v >= n) bad |= 1u;
    if (j != 0u && static_cast<uint32_t>(idx[j - 1u]) >= v) bad |= 2u;
  }
  if (bad != 0u) atomicOr(status, bad);
}

hipError_t launch_decompress_validate(const DecompressArgs& a, uint32_t* status, hipStream_t s) {
  const uint32_t msgs = a.num_workers * a.num_layers;
  if (msgs == 0) return hipSuccess;
  hipLaunchKernelGGL(decompress_validate_kernel, dim3(msgs), dim3(kBlockThreads), 0, s, a, status);
  return hipGetLastError();
}

hipError_t launch_decompress_table(const DecompressArgs& a, hipStream_t s) {
  // only the kernel that takes any number of workers reads the table
  if (a.num_blocks == 0 || a.num_workers <= static_cast<uint32_t>(kBatchWorkers)) return hipSuccess;
  hipLaunchKernelGGL(decompress_table_kernel, dim3(a.num_blocks), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

// Persistent grids: as many workgroups as fit on the device at once, a multiple of 8 so that
// every XCD gets its share.  cus = compute units of the current device.
static uint32_t resident_grid(const void* kernel, uint32_t threads, uint32_t cus) {
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, static_cast<int>(threads), 0) != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    per_cu = 1;
  }
  const uint32_t g = (static_cast<uint32_t>(per_cu) * cus / 8u) * 8u;
  return g < 8u ? 8u : g;
}

hipError_t launch_decompress_tiles(const DecompressArgs& a, hipStream_t s) {
  if (a.num_tiles == 0) return hipSuccess;
  static uint32_t per_cu_fast = 0, per_cu_generic = 0;   // workgroups per CU; a property of the code object
  if (per_cu_fast == 0) {
    per_cu_fast = resident_grid(reinterpret_cast<const void*>(decompress_tiles_kernel<false, false>), kFastThreads, 8u) / 8u;
    per_cu_generic = resident_grid(reinterpret_cast<const void*>(decompress_generic_kernel), kBlockThreads, 8u) / 8u;
  }
  const uint32_t want = ((a.num_tiles + 7u) / 8u) * 8u;
  const uint32_t cus8 = a.cus < 8u ? 8u : (a.cus / 8u) * 8u;
  const bool fast = a.num_workers >= 1u && a.num_workers <= static_cast<uint32_t>(kBatchWorkers);
  const uint32_t cap = (fast ? per_cu_fast : per_cu_generic) * cus8;
  const uint32_t grid = want < cap ? want : cap;
  if (fast && a.one_value) {
    if (a.stream_msgs) hipLaunchKernelGGL((decompress_tiles_kernel<true, true>), dim3(grid), dim3(kFastThreads), 0, s, a);
    else hipLaunchKernelGGL((decompress_tiles_kernel<false, true>), dim3(grid), dim3(kFastThreads), 0, s, a);
  } else if (fast) {
    if (a.stream_msgs) hipLaunchKernelGGL((decompress_tiles_kernel<true, false>), dim3(grid), dim3(kFastThreads), 0, s, a);
    else hipLaunchKernelGGL((decompress_tiles_kernel<false, false>), dim3(grid), dim3(kFastThreads), 0, s, a);
  }
  else hipLaunchKernelGGL(decompress_generic_kernel, dim3(grid), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace rgc
