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
// A first kernel builds, for every (worker, layer) message, the offset of the first entry of
// every tile (the messages are sorted by index), so that the tile kernel finds its entries
// without searching.
#include "rgc_device.h"

namespace rgc {

namespace {
constexpr uint32_t kTableBlockEntries = 1024;
}

// ------------------------------------------------------------------ tile-offset table
__global__ void __launch_bounds__(kBlockThreads) decompress_table_kernel(DecompressArgs A) {
  const BlockDesc bd = A.blocks[blockIdx.x];
  const MsgDesc md = A.msgs[bd.msg];
  const uint32_t layer = bd.msg % A.num_layers;
  const uint32_t ntiles = A.layer_tiles[layer];
  uint32_t* row = A.tab + md.tab_base;   // ntiles + 1 words: first entry of tile t; row[ntiles] = count
  const gptr<const int32_t> midx = as_global(md.idx);
  if (md.count == 0u) {
    for (uint32_t t = threadIdx.x; t <= ntiles; t += kBlockThreads) row[t] = 0u;
    return;
  }
  const uint32_t stop = (md.count - bd.first) < kTableBlockEntries ? md.count : bd.first + kTableBlockEntries;
  for (uint32_t j = bd.first + threadIdx.x; j < stop; j += kBlockThreads) {
    uint32_t cur = static_cast<uint32_t>(midx[j]) >> kTileShift;
    if (cur >= ntiles) cur = ntiles - 1u;                 // out-of-range index: stay inside the row
    uint32_t first = 0u;
    if (j != 0u) {
      uint32_t prev = static_cast<uint32_t>(midx[j - 1u]) >> kTileShift;
      if (prev >= ntiles) prev = ntiles - 1u;
      first = prev + 1u;
    }
    for (uint32_t t = first; t <= cur; ++t) row[t] = j;
    if (j == md.count - 1u)
      for (uint32_t t = cur + 1u; t <= ntiles; ++t) row[t] = md.count;
  }
}

// ------------------------------------------------------------------ tile accumulation
__global__ void __launch_bounds__(kBlockThreads) decompress_tiles_kernel(DecompressArgs A) {
  __shared__ float acc[kTile];
  __shared__ uint32_t cnt32[kTile / 4];          // one byte counter per position
  __shared__ uint32_t cb[kTile / 32];            // positions hit more than once in this batch
  __shared__ uint32_t cbpre[kTile / 32];         // exclusive popcount prefix of cb
  __shared__ uint32_t masks[kQMax * kMaskWords]; // per colliding position: which workers hit it
  __shared__ uint32_t qbase[kQMax];
  __shared__ float staged[kEntryCap];
  __shared__ uint32_t e_pw[kEntryCap];           // position | local worker << 16, or ~0 if unusable
  __shared__ float e_val[kEntryCap];
  __shared__ uint32_t w_start[kBatchWorkers];
  __shared__ uint32_t w_pref[kBatchWorkers + 1];
  __shared__ const int32_t* w_idx[kBatchWorkers];
  __shared__ const float* w_val[kBatchWorkers];
  __shared__ uint32_t scan_lds[4];
  __shared__ uint32_t sh_end, sh_entries, sh_cursor;

  const uint32_t tid = threadIdx.x;
  const TileDesc tile = A.tiles[blockIdx.x];
  const uint32_t N = A.num_workers, NL = A.num_layers;

  for (uint32_t i = tid; i < static_cast<uint32_t>(kTile); i += kBlockThreads) acc[i] = 0.0f;

  uint32_t w0 = 0;
  while (w0 < N) {
    const uint32_t nb = (N - w0) < static_cast<uint32_t>(kBatchWorkers) ? (N - w0) : static_cast<uint32_t>(kBatchWorkers);
    // ---- which workers fit into this batch
    uint32_t s = 0, c = 0;
    const int32_t* ip = nullptr;
    const float* vp = nullptr;
    if (tid < nb) {
      const MsgDesc md = A.msgs[static_cast<size_t>(w0 + tid) * NL + tile.layer];
      const uint32_t* row = A.tab + md.tab_base + tile.tab_col;
      s = row[0];
      uint32_t e = row[1];
      if (e > md.count) e = md.count;     // the table never exceeds the message; stay in bounds anyway
      c = e > s ? e - s : 0u;
      ip = md.idx;
      vp = md.val;
    }
    if (tid == 0) { sh_end = nb; sh_cursor = 0u; }
    uint32_t batch_total;
    const uint32_t ex = block_excl_scan(c, scan_lds, batch_total);
    if (tid < nb && ex + c > static_cast<uint32_t>(kEntryCap)) atomicMin(&sh_end, tid);
    __syncthreads();
    const uint32_t nw = sh_end;
    if (nw == 0u) {
      // the first worker alone exceeds the staging capacity: its positions are unique, add directly
      __syncthreads();
      if (tid == 0) { w_start[0] = s; w_pref[0] = c; w_idx[0] = ip; w_val[0] = vp; }
      __syncthreads();
      const uint32_t s0 = w_start[0], c0 = w_pref[0];
      const gptr<const int32_t> ip0 = as_global(w_idx[0]);
      const gptr<const float> vp0 = as_global(w_val[0]);
      for (uint32_t j = tid; j < c0; j += kBlockThreads) {
        const uint32_t p = static_cast<uint32_t>(ip0[s0 + j]) - tile.first;
        if (p < tile.len) acc[p] = __fadd_rn(acc[p], vp0[s0 + j]);
      }
      __syncthreads();
      w0 += 1u;
      continue;
    }
    if (tid < nw) { w_start[tid] = s; w_pref[tid] = ex; w_idx[tid] = ip; w_val[tid] = vp; }
    if (tid == nw - 1u) { w_pref[nw] = ex + c; sh_entries = ex + c; }
    // ---- clear the per-batch structures
    for (uint32_t i = tid; i < static_cast<uint32_t>(kTile / 4); i += kBlockThreads) cnt32[i] = 0u;
    if (tid < static_cast<uint32_t>(kTile / 32)) cb[tid] = 0u;
    __syncthreads();
    const uint32_t E = sh_entries;
    if (E == 0u) { w0 += nw; __syncthreads(); continue; }

    // ---- P1: fetch the entries, count hits per position
    for (uint32_t e = tid; e < E; e += kBlockThreads) {
      uint32_t lo = 0, hi = nw;
      while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (w_pref[mid] <= e) lo = mid; else hi = mid;
      }
      const uint32_t j = w_start[lo] + (e - w_pref[lo]);
      const uint32_t p = static_cast<uint32_t>(as_global(w_idx[lo])[j]) - tile.first;
      if (p < tile.len) {
        e_pw[e] = p | (lo << 16);
        e_val[e] = as_global(w_val[lo])[j];
        atomicAdd(&cnt32[p >> 2], 1u << ((p & 3u) * 8u));
      } else {
        e_pw[e] = 0xFFFFFFFFu;
      }
    }
    __syncthreads();
    // ---- P2: positions hit once are final; mark the others
    for (uint32_t e = tid; e < E; e += kBlockThreads) {
      const uint32_t pw = e_pw[e];
      if (pw == 0xFFFFFFFFu) continue;
      const uint32_t p = pw & 0xFFFFu;
      const uint32_t hits = (cnt32[p >> 2] >> ((p & 3u) * 8u)) & 0xFFu;
      if (hits == 1u) acc[p] = __fadd_rn(acc[p], e_val[e]);
      else atomicOr(&cb[p >> 5], 1u << (p & 31u));
    }
    __syncthreads();
    // ---- P3: dense numbering of the colliding positions
    uint32_t nq;
    {
      const uint32_t pc = tid < static_cast<uint32_t>(kTile / 32) ? static_cast<uint32_t>(__popc(cb[tid])) : 0u;
      const uint32_t pex = block_excl_scan(pc, scan_lds, nq);
      if (tid < static_cast<uint32_t>(kTile / 32)) cbpre[tid] = pex;
    }
    __syncthreads();
    if (nq == 0u) { w0 += nw; continue; }
    if (nq > static_cast<uint32_t>(kQMax)) {
      // too many colliding positions for the mask table: add worker after worker
      for (uint32_t wl = 0; wl < nw; ++wl) {
        const uint32_t eb = w_pref[wl], ee = w_pref[wl + 1u];
        for (uint32_t e = eb + tid; e < ee; e += kBlockThreads) {
          const uint32_t pw = e_pw[e];
          if (pw == 0xFFFFFFFFu) continue;
          const uint32_t p = pw & 0xFFFFu;
          const uint32_t hits = (cnt32[p >> 2] >> ((p & 3u) * 8u)) & 0xFFu;
          if (hits > 1u) acc[p] = __fadd_rn(acc[p], e_val[e]);
        }
        __syncthreads();
      }
      w0 += nw;
      continue;
    }
    for (uint32_t i = tid; i < nq * kMaskWords; i += kBlockThreads) masks[i] = 0u;
    __syncthreads();
    // ---- P4: who hits each colliding position
    for (uint32_t e = tid; e < E; e += kBlockThreads) {
      const uint32_t pw = e_pw[e];
      if (pw == 0xFFFFFFFFu) continue;
      const uint32_t p = pw & 0xFFFFu, wl = pw >> 16;
      const uint32_t word = cb[p >> 5], bit = 1u << (p & 31u);
      if (word & bit) {
        const uint32_t q = cbpre[p >> 5] + static_cast<uint32_t>(__popc(word & (bit - 1u)));
        atomicOr(&masks[q * kMaskWords + (wl >> 5)], 1u << (wl & 31u));
      }
    }
    __syncthreads();
    // ---- P5: the lowest worker of each position reserves its run of staged values
    for (uint32_t e = tid; e < E; e += kBlockThreads) {
      const uint32_t pw = e_pw[e];
      if (pw == 0xFFFFFFFFu) continue;
      const uint32_t p = pw & 0xFFFFu, wl = pw >> 16;
      const uint32_t word = cb[p >> 5], bit = 1u << (p & 31u);
      if (word & bit) {
        const uint32_t q = cbpre[p >> 5] + static_cast<uint32_t>(__popc(word & (bit - 1u)));
        uint32_t rank = 0, total = 0;
#pragma unroll
        for (uint32_t mw = 0; mw < kMaskWords; ++mw) {
          const uint32_t mk = masks[q * kMaskWords + mw];
          total += static_cast<uint32_t>(__popc(mk));
          if (mw < (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk));
          else if (mw == (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk & ((1u << (wl & 31u)) - 1u)));
        }
        if (rank == 0u) qbase[q] = atomicAdd(&sh_cursor, total);
      }
    }
    __syncthreads();
    // ---- P6: place the values by rank
    for (uint32_t e = tid; e < E; e += kBlockThreads) {
      const uint32_t pw = e_pw[e];
      if (pw == 0xFFFFFFFFu) continue;
      const uint32_t p = pw & 0xFFFFu, wl = pw >> 16;
      const uint32_t word = cb[p >> 5], bit = 1u << (p & 31u);
      if (word & bit) {
        const uint32_t q = cbpre[p >> 5] + static_cast<uint32_t>(__popc(word & (bit - 1u)));
        uint32_t rank = 0;
#pragma unroll
        for (uint32_t mw = 0; mw < kMaskWords; ++mw) {
          const uint32_t mk = masks[q * kMaskWords + mw];
          if (mw < (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk));
          else if (mw == (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk & ((1u << (wl & 31u)) - 1u)));
        }
        const uint32_t at = qbase[q] + rank;
        if (at < static_cast<uint32_t>(kEntryCap)) staged[at] = e_val[e];
      }
    }
    __syncthreads();
    // ---- P7: one lane per colliding position adds its run in worker order
    for (uint32_t e = tid; e < E; e += kBlockThreads) {
      const uint32_t pw = e_pw[e];
      if (pw == 0xFFFFFFFFu) continue;
      const uint32_t p = pw & 0xFFFFu, wl = pw >> 16;
      const uint32_t word = cb[p >> 5], bit = 1u << (p & 31u);
      if (word & bit) {
        const uint32_t q = cbpre[p >> 5] + static_cast<uint32_t>(__popc(word & (bit - 1u)));
        uint32_t rank = 0, total = 0;
#pragma unroll
        for (uint32_t mw = 0; mw < kMaskWords; ++mw) {
          const uint32_t mk = masks[q * kMaskWords + mw];
          total += static_cast<uint32_t>(__popc(mk));
          if (mw < (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk));
          else if (mw == (wl >> 5)) rank += static_cast<uint32_t>(__popc(mk & ((1u << (wl & 31u)) - 1u)));
        }
        if (rank == 0u) {
          const uint32_t b = qbase[q];
          float sum = acc[p];
          for (uint32_t i = 0; i < total && b + i < static_cast<uint32_t>(kEntryCap); ++i)
            sum = __fadd_rn(sum, staged[b + i]);
          acc[p] = sum;
        }
      }
    }
    __syncthreads();
    w0 += nw;
  }
  __syncthreads();

  // ---- write the tile once
  const gptr<float> d = as_global(tile.dense);
  const float scale = A.scale;
  const bool vec = ((reinterpret_cast<uintptr_t>(tile.dense) & 15u) == 0u) && ((tile.len & 3u) == 0u);
  if (vec) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    const gptr<vf4> d4 = as_global(reinterpret_cast<vf4*>(tile.dense));
    for (uint32_t i = tid; i < tile.len / 4u; i += kBlockThreads) {
      vf4 o;
      o.x = __fmul_rn(acc[4 * i + 0], scale);
      o.y = __fmul_rn(acc[4 * i + 1], scale);
      o.z = __fmul_rn(acc[4 * i + 2], scale);
      o.w = __fmul_rn(acc[4 * i + 3], scale);
      if (A.add_to_dst) {
        const vf4 old = d4[i];
        o.x = __fadd_rn(old.x, o.x); o.y = __fadd_rn(old.y, o.y);
        o.z = __fadd_rn(old.z, o.z); o.w = __fadd_rn(old.w, o.w);
      }
      d4[i] = o;
    }
  } else {
    for (uint32_t i = tid; i < tile.len; i += kBlockThreads) {
      float o = __fmul_rn(acc[i], scale);
      if (A.add_to_dst) o = __fadd_rn(d[i], o);
      d[i] = o;
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
  hipLaunchKernelGGL(decompress_tiles_kernel, dim3(a.num_tiles), dim3(kBlockThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace rgc
