// Internal declarations shared by the host API and the gfx950 kernels of librgc.
// Nothing here is visible through the C ABI (include/rgc.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rgc {

// ---------------------------------------------------------------- geometry (compile time)
constexpr int kWaveSize = 64;
constexpr int kBlockThreads = 256;                 // 4 waves per workgroup
constexpr int kWavesPerBlock = kBlockThreads / kWaveSize;
constexpr int kGroupElems = kWaveSize * 4;         // one float4 per lane per step
constexpr int kHistBins = 4096;                    // radix digit of 12 bits (31-bit key = 12+12+7)
constexpr int kCoarseBins = 1024;                  // candidate histogram bins (hinted path)
constexpr int kCoarseRep = 8;                      // replicas of it, to spread same-address atomics
constexpr int kMemberMax = 4096;                   // candidates of one coarse bin ranked in LDS
constexpr uint32_t kKeyMask = 0x7FFFFFFFu;

// Phase a layer has to run at a given launch of the phase kernel.
enum Phase : uint32_t {
  PH_NONE = 0,
  PH_SEL = 1,      // hinted: rank the members of the candidate bin holding the k-th key
  PH_OUT_C = 2,    // hinted: ordered output from the candidate lists
  PH_HIST1 = 3,    // multi-pass: digit-1 histogram over the updated residual (after a miss)
  PH_HIST2 = 4,    // multi-pass: digit-2 histogram
  PH_HIST3 = 5,    // multi-pass: digit-3 histogram
  PH_COUNT = 6,    // multi-pass: per wave-chunk counts of keys > T and == T
  PH_OUT_V = 7,    // multi-pass: ordered compaction from the updated residual
  PH_COLLECT = 8,  // after the first digit: candidate lists from the updated residual, then PH_SEL / PH_OUT_C
  PH_RESTORE = 9,  // dense layers whose hint missed: the entries masked on the strength of the hint go back into residual and
                   // velocity, then PH_HIST1 in the same launch
  PH_EMIT = 10,    // dense layers: the message from the lists, with the k-th entry known
  PH_SEL2 = 11,    // dense layers: PH_SEL on the layer's own lists (lists_kernel)
};

// Dense layers: after a call whose hint missed, the layer goes without its hint for a number of calls that
// doubles with every further miss, up to this many.
// Workgroups' worth of candidate lists one workgroup of PH_SEL / PH_OUT_C takes (CompressArgs::list_group:
// kListGroup, or 1 for a call whose workgroups all fit on the device at once, where spreading the lists wins).
constexpr uint32_t kListGroupLog2 = 2, kListGroup = 1u << kListGroupLog2;
constexpr uint32_t kDenseBackoffMax = 64;
// Dense layers: the members of the k-th key's coarse bin are appended to this many sub-lists, each with a counter
// of its own (thousands of waves appending through one counter take their turns at ~20 ns each), and what a
// sub-list cannot hold to one more list that can hold them all.
constexpr uint32_t kMemberShards = 16;
constexpr uint32_t kMemberLists = kMemberShards + 1;
constexpr uint32_t kShardStride = 64;    // words between two counters: atomics on one cache line take their turns like atomics on one word

// Per call, per layer descriptor (device copy of the caller's rgc_layer plus the tiling).
struct LayerDesc {
  const float* grad;
  float* resid;
  float* mom;
  int32_t* out_idx;
  float* out_val;
  int32_t* out_count;
  uint32_t n;
  uint32_t k;
  uint32_t wc_first;   // first wave-chunk of this layer in the per-wave-chunk arrays
  uint32_t wc_count;   // number of wave-chunks = ceil(n / chunk)
  uint32_t wg_first;   // first workgroup of this layer
  uint32_t wg_count;   // = ceil(wc_count / 4)
  uint32_t grp_first;  // first election-group counter of this layer
  uint32_t vec_ok;     // every tensor pointer is 16-byte aligned
  uint32_t hintable;   // one-pass layer: the candidate lists can hold every element from the hinted threshold upwards
  uint32_t margin;     // extra candidates aimed for beyond k
  uint32_t cmax;       // largest candidate total a hint may aim at
  uint32_t target;     // rank the next call's threshold hint is aimed at (2k + margin, dense layers: k + margin)
  uint32_t dense;      // high-density layer (never set together with hintable): with a hint, its streaming pass lists every
                       // candidate in lists of its own and masks those far enough above the hinted threshold at once
  uint32_t mem_cap;    // dense layers: entries of the layer's kMemberShards sub-lists together (a multiple of kMemberShards); the
                       // overflow list behind them holds mem_cap / 4, which is also the most members a call accepts
  uint32_t list_cap;   // dense layers: entries of one wave-chunk's list
  uint32_t pad_;
  uint64_t mem_first;  // dense layers: where the layer's region of the member pool starts
  uint64_t list_first; // dense layers: where the layer's lists start (wave-chunk c of the layer: list_first + c * list_cap)
};

// Per layer state living in the context (device memory).  Everything but the hint fields is
// rewritten by every call before it is read.
struct LayerState {
  uint32_t next_phase;   // Phase to run ...
  uint32_t next_launch;  // ... at this launch number (2..6)
  uint32_t done;         // workgroups of the layer that finished the current phase
  uint32_t prefix;       // multi-pass: key bits fixed so far (digits 1 and 2)
  uint32_t k_rem;        // rank of the k-th key inside the current bin (1-based)
  uint32_t T;            // threshold key: the k-th largest key of the layer
  uint32_t r;            // multi-pass: how many keys == T are admitted (lowest indices)
  uint32_t bstar;        // hinted: coarse bin holding the k-th key
  uint32_t nmembers;     // hinted: members appended so far
  uint32_t path;         // 0 hinted one-pass, 1 hint-free multi-pass, 2 miss then multi-pass
  unsigned long long thr;  // hinted: composite (key<<32 | ~idx) of the k-th entry
  // speed hints (never influence results)
  uint32_t hint_valid;
  uint32_t tau;          // candidate threshold key for the next call
  uint32_t shift;        // coarse bin = min((key - tau) >> shift, kCoarseBins - 1)
  uint32_t tau_next;     // being derived during this call
  uint32_t hint_pending; // multi-pass: 0 none found yet / 1 refine in the next digit / 2 final
  uint32_t T_prev;       // threshold key of the previous call (drift estimate), if has_prev
  uint32_t has_prev;
  uint32_t stat_candidates;  // diagnostics of the last call
  uint32_t stat_members;
  uint32_t stat_misses;      // calls so far in which this layer's hint missed (never reset)
  // dense layers (speed only, like the hints)
  uint32_t clip;             // candidates of the coarse bins from this one upwards are sure to be selected: counted, not ranked
  uint32_t dense_backoff;    // calls the layer went without its hint after the last miss
  uint32_t dense_skip;       // calls it still goes without it
  uint32_t cur_tau;          // tau, shift and mask_key as this call's streaming pass used them (the ranking step rewrites
  uint32_t cur_shift;        // the hint for the next call before the output step has read it)
  uint32_t cur_mask_key;
  uint32_t mask_key;         // dense layers: where the k-th key of the next call is expected; its streaming pass masks the candidates
                             // from here upwards at once and the output step puts right what that got wrong
};

// Where the kernels of an exactly rounded sum leave their parts (one per workgroup): the running sum
// and the sum of its rounding errors, the flags (digits in use, non-finite terms seen) and, only where
// the flags say so, the part's fixed-point digits.
constexpr int kExactDigits = 20;            // 32 bits each, from 2^-298 upwards: any sum of fp32 terms or of their squares
constexpr size_t kExactWordsPerPart = 3 + kExactDigits;   // 8-byte words of one part
struct ExactParts {
  double* sc;                  // [parts][2]
  unsigned long long* flags;   // [parts]
  long long* digits;           // [parts][kExactDigits]
};
inline ExactParts exact_parts_at(void* base, size_t parts) {
  ExactParts P;
  P.sc = static_cast<double*>(base);
  P.flags = reinterpret_cast<unsigned long long*>(P.sc + 2 * parts);
  P.digits = reinterpret_cast<long long*>(P.flags + parts);
  return P;
}

struct CompressArgs {
  const LayerDesc* layers;
  LayerState* state;
  const uint32_t* wg2layer;
  uint32_t* hist;        // [layers][kHistBins]
  uint32_t* coarse;      // [layers][kCoarseRep][kCoarseBins]
  unsigned long long* members;  // [layers][kMemberMax]
  uint32_t* cand_cnt;    // [wave-chunks]
  uint2* slots;          // [wave-chunks][cap] (float bits, index), ascending index per chunk
  uint32_t* wc_a;        // [wave-chunks] counts, then output offsets
  uint32_t* wc_b;        // [wave-chunks] tie counts, then tie prefixes
  uint2* slots2;         // the lists of the dense layers (LayerDesc::list_first, list_cap; allocated when such a layer is first seen)
  float* slots_u;        // the velocity of every listed element, same layout (restores a masked entry after a miss)
  unsigned long long* members2;  // member pool of the dense layers (LayerDesc::mem_first, mem_cap)
  uint32_t* shard_cnt;   // [layers][kMemberLists][kShardStride] members appended to each sub-list, one counter per 256 bytes
  uint32_t* group_done;  // [election groups] workgroups of the group that finished the current phase
  uint32_t* errflag;     // set non-zero on an internal inconsistency
  uint32_t chunk;        // elements per wave-chunk (multiple of 256)
  uint32_t cap;          // candidate slots per wave-chunk
  uint32_t use_hints;
  uint32_t dense_ok;     // the lists of the dense layers exist: such a layer may take its hinted path (collect_kernel)
  uint32_t update_hints;
  uint32_t mask_momentum;
  float m;
  uint32_t launch;       // launch number of the phase kernel (2..6)
  uint32_t sign_xor;     // selection key: see key_of() (0 / 0x80000000: which sign bit keeps an element in the ranking)
  uint32_t sign_filter;  // 0: every element ranks by magnitude; ~0: elements of the other sign rank last (key 0)
  uint32_t reverse;      // the streaming pass takes its workgroups in descending order
  uint32_t nesterov;     // momentum correction in its Nesterov form: u = m (u + g), a = (V + u) + g
  uint32_t list_group;   // workgroups' worth of candidate lists one workgroup of PH_SEL / PH_OUT_C takes (1 or 4)
  const float* grad_scale;   // device word every gradient element is multiplied with first, or null
  ExactParts norm_parts; // [workgroups] parts of the sum of squares (clipping coefficient only)
};

// ---------------------------------------------------------------- threshold binary search selection
struct ThresholdMoments {   // per layer, written by the moments kernel
  float mean;               // mean of |a|
  float max;                // max of |a|
  float span;               // max - mean, rounded
  uint32_t counts_taken;    // counts the bisection took (diagnostics)
};

struct ThresholdArgs {
  const LayerDesc* layers;
  const uint32_t* wg2layer;
  float* thresholds;        // [layers] the caller's: written by a search, read otherwise
  int32_t* nnz;             // [layers] the caller's, or null: elements above the threshold
  const float* grad_scale;  // device word every gradient element is multiplied with first, or null
  ExactParts sum_parts;     // [workgroups] parts of the sum of |a|
  float* part_max;          // [workgroups] partial maxima of |a|
  uint32_t* counts;         // [wave-chunks] elements above the threshold, then first output positions
  uint32_t* listed;         // [wave-chunks] elements above the threshold (kept; more than cap: list incomplete)
  uint2* slots;             // [wave-chunks][cap] (float bits, index) of the elements above a reused threshold
  uint32_t cap;             // list slots per wave-chunk
  uint32_t* hist;           // [layers][kHistBins], the first 1024 bins of each are used
  ThresholdMoments* moments;  // [layers]
  uint32_t chunk;           // elements per wave-chunk
  uint32_t search;          // 1: Algorithm 3 finds the thresholds; 0: they are given
  uint32_t reverse;         // the first pass takes its workgroups in descending order (and every pass after it the other way)
  uint32_t mask_momentum;
  uint32_t nesterov;
  float m;
};

hipError_t launch_threshold_compress(const ThresholdArgs& a, uint32_t num_wgs, uint32_t num_layers, hipStream_t s);

// ---------------------------------------------------------------- decompress
// 8192 positions: most of a tile's instructions (window checks, map clearing, barriers) are paid per tile,
// not per position; 4096 was 28 % slower, 16384 leaves room for one workgroup per CU only and is slower too.
constexpr int kTileShift = 13;
constexpr int kTile = 1 << kTileShift;            // dense positions owned by one workgroup
constexpr int kEntryCap = 1024;                   // entries staged per worker batch (generic tiles)
constexpr int kBatchWorkers = 128;                // workers per batch (mask of 4 words)
constexpr int kMaskWords = kBatchWorkers / 32;
constexpr int kQMax = 128;                        // positions hit more than once per batch

struct MsgDesc {                                   // one (worker, layer) message
  const int32_t* idx;
  const float* val;
  uint32_t count;
  uint32_t tab_base;    // first table row of the message's layer
};

struct DecompressLayer {   // one dense buffer
  float* dense;
  uint32_t n;
  uint32_t tiles;         // ceil(n / kTile)
  uint32_t tile_base;     // global id of its first tile
  uint32_t row_base;      // first table row (the layer owns tiles + 1 rows)
  uint32_t pad[2];
};

struct BlockDesc {      // one block of the table-building kernel
  uint32_t msg;         // index into the MsgDesc array
  uint32_t first;       // first entry handled by the block
};

struct DecompressArgs {
  const MsgDesc* msgs;        // [layers][workers]
  const DecompressLayer* layers;
  const BlockDesc* blocks;
  uint32_t* tab;              // [workers][tab_stride]: first entry of each tile; one closing entry per layer
  uint32_t tab_stride;
  uint32_t cus;               // compute units of the device (sizes the persistent grids)
  uint32_t num_workers;
  uint32_t num_layers;
  uint32_t num_tiles;
  uint32_t num_blocks;
  uint32_t add_to_dst;
  uint32_t stream_msgs;       // read the messages with streaming loads (see decompress_tiles_kernel)
  uint32_t one_value;         // every message's val points to ONE float that all its entries carry
  float scale;
};

// Records the text of a failed HIP call for rgc_strerror and returns RGC_EHIP (defined with the host API).
int fail_hip(hipError_t e, const char* what);

// kernel launchers (defined in the .hip files)
hipError_t launch_accumulate(const CompressArgs& a, uint32_t num_wgs, hipStream_t s);
hipError_t launch_collect(const CompressArgs& a, uint32_t num_wgs, hipStream_t s);   // streaming pass of the dense layers
hipError_t launch_lists(const CompressArgs& a, uint32_t num_wgs, hipStream_t s);     // their ranking and output steps
hipError_t launch_phase(const CompressArgs& a, uint32_t num_wgs, hipStream_t s);
constexpr uint32_t kMeanPartsMax = 128;    // parts per layer at most (rgc_message_means)
hipError_t launch_message_means(const CompressArgs& a, uint32_t num_layers, uint32_t max_k, const ExactParts& parts,
                                float* d_means, hipStream_t s);
hipError_t launch_clip_coefficient(const CompressArgs& a, uint32_t num_wgs, float threshold, float* d_coef, hipStream_t s);
hipError_t launch_poison(LayerState* st, uint32_t num_layers, int mode, hipStream_t s);
hipError_t launch_decompress_table(const DecompressArgs& a, hipStream_t s);
hipError_t launch_decompress_tiles(const DecompressArgs& a, hipStream_t s);
hipError_t launch_decompress_validate(const DecompressArgs& a, uint32_t* status, hipStream_t s);
hipError_t launch_wave_scan_selftest(uint32_t* io, hipStream_t s);

}  // namespace rgc
