// Host side of librgc: the C ABI declared in include/rgc.h.  Validates arguments, turns the
// caller's layer / message lists into device descriptor tables (cached while the lists do not
// change) and enqueues the kernels.  No kernel arithmetic lives here.
#include "../../include/rgc.h"
#include "../../include/rgc_diag.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <numeric>
#include <string>
#include <vector>

#include "rgc_internal.h"

using namespace rgc;

namespace {

thread_local std::string g_hip_error = "no HIP error recorded";

}  // namespace

int rgc::fail_hip(hipError_t e, const char* what) {
  char buf[256];
  std::snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
  g_hip_error = buf;
  return RGC_EHIP;
}

namespace {

#define RGC_HIP(call)                                   \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return fail_hip(e_, #call);   \
  } while (0)

constexpr uint32_t kSmallCallWorkgroups = 256;   // one workgroup per compute unit
constexpr uint32_t kChunkSmallest = 4096;  // elements per wave-chunk for small layer sets
// Candidate slots per wave-chunk = chunk / 16: sixty times the average number of candidates of a chunk at
// density 0.1 %.  Tensors whose large values sit in a few rows (embedding gradients) fill single lists far
// beyond the average; with chunk / 32 such a layer overflowed a list, and so missed its hint, in 20 of its first
// 50 calls, with chunk / 16 in 2.
constexpr uint32_t kCapDiv = 16;
// Dense layers (high densities) list every candidate in lists of their own, long enough for twice the number the
// hint aims at (allocated when a plan with such a layer is first used); the members of the k-th key's coarse bin
// go to a pool in which every such layer owns max(4096, n / 64) entries.

// -DRGC_CHUNK=<elements> (a multiple of 256, >= 1024) at build time fixes the wave-chunk size for tuning
// experiments; not defined = automatic.  (There are no run-time switches: nothing here reads the environment.)
#ifdef RGC_CHUNK
static_assert(RGC_CHUNK >= 1024 && RGC_CHUNK <= (1 << 20) && RGC_CHUNK % 256 == 0, "RGC_CHUNK: a multiple of 256, at least 1024");
constexpr uint32_t chunk_override() { return RGC_CHUNK; }
#else
constexpr uint32_t chunk_override() { return 0u; }
#endif

// Elements per wave-chunk for a call over `total` elements.  Larger chunks mean fewer per-chunk
// counters for the per-layer serial steps, smaller ones more workgroups to fill 256 CUs.
uint32_t chunk_for(int64_t total) {
  if (chunk_override()) return chunk_override();
  if (total >= (int64_t(8) << 20)) return 8192;
  return kChunkSmallest;
}

// Smallest chunk any call may use: the scratch is sized for it.
uint32_t chunk_smallest() { return chunk_override() ? std::min(chunk_override(), kChunkSmallest) : kChunkSmallest; }
constexpr int kPlanCache = 8;
constexpr uint32_t kElectGroupHost = 32;   // = kElectGroup of the kernels (workgroups per election group)
constexpr int kLaunches = 6;               // streaming pass + at most five phase launches

struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

template <typename T>
struct DevBuf {
  T* p = nullptr;
  size_t n = 0;
  hipError_t alloc(size_t count) {
    release();
    if (count == 0) count = 1;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&p), count * sizeof(T));
    if (e == hipSuccess) n = count; else p = nullptr;
    return e;
  }
  void release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    n = 0;
  }
};

struct PinnedBuf {
  void* p = nullptr;
  size_t bytes = 0;
  hipError_t ensure(size_t b) {
    if (b <= bytes) return hipSuccess;
    if (p) (void)hipHostFree(p);
    p = nullptr;
    bytes = 0;
    hipError_t e = hipHostMalloc(&p, b, hipHostMallocDefault);
    if (e == hipSuccess) bytes = b; else p = nullptr;
    return e;
  }
  void release() {
    if (p) (void)hipHostFree(p);
    p = nullptr;
    bytes = 0;
  }
};

// One cached translation of a layer list into device tables.
struct CompressPlan {
  std::vector<rgc_layer> key;       // the caller's list this plan was built from
  uint32_t chunk = 0;               // elements per wave-chunk of this plan
  DevBuf<LayerDesc> d_layers;
  DevBuf<uint32_t> d_wg2layer;
  PinnedBuf staging;
  hipEvent_t uploaded = nullptr;    // recorded after the uploads
  uint32_t num_wgs = 0;
  uint32_t num_chunks = 0;                 // wave-chunks over all layers
  uint64_t write_bytes = 0;                // what the streaming pass writes (V, and u where there is one)
  uint32_t max_k = 0;                      // the largest k of the list
  bool any_dense = false;                  // some layer is streamed by collect_kernel when it has a hint
  uint64_t list_entries = 0;               // list entries of the dense layers
  uint64_t member_entries = 0;             // entries of the member pool they own
  uint64_t last_use = 0;
  bool valid = false;
};

struct DecompressPlan {
  std::vector<rgc_msg> key_msgs;
  std::vector<float*> key_dense;
  std::vector<int64_t> key_n;
  int32_t workers = 0, layers = 0;
  DevBuf<unsigned char> d_tables;   // MsgDesc[], DecompressLayer[], BlockDesc[]
  DevBuf<uint32_t> d_tab;
  PinnedBuf staging;
  hipEvent_t uploaded = nullptr;
  DecompressArgs args{};
  bool valid = false;
};

}  // namespace

struct rgc_ctx {
  int device = 0;
  int64_t max_total = 0;
  int32_t max_layers = 0;
  uint32_t wc_max = 0;
  uint32_t cus = 0;                        // compute units of the device (sizes the persistent decompression grids)
  DevBuf<LayerState> d_state;
  DevBuf<uint32_t> d_hist, d_coarse, d_cand_cnt, d_wc_a, d_wc_b, d_err, d_group;
  DevBuf<unsigned long long> d_members;
  DevBuf<long long> d_norm_part;           // [workgroups] parts of the sum of squares / of |a| (ExactParts)
  DevBuf<long long> d_mean_part;           // [layers][kMeanPartsMax] parts of the sums of message values (ExactParts)
  DevBuf<ThresholdMoments> d_moments;      // [max_layers] threshold binary search: mean, max of each layer
  DevBuf<uint2> d_slots;
  DevBuf<uint2> d_slots2;                  // the lists of the dense layers (first use)
  DevBuf<float> d_slots_u;                 // the velocity of every listed element (first use)
  DevBuf<unsigned long long> d_members2;   // member pool of the dense layers (first use)
  DevBuf<uint32_t> d_shards;               // their sub-list counters (first use)
  CompressPlan plans[kPlanCache];
  uint64_t tick = 0;
  int64_t optional_scratch_cap = -1;       // bytes the dense layers' lists may take (diagnostics); negative: no cap
  bool compressed_since_decompress = false;
  uint64_t compress_calls = 0;             // its parity is the direction of the next streaming pass
  uint32_t threshold_reverse = 0;          // direction of the next threshold-selection call's first pass
  // Speed hints are kept per selection mode (0 magnitude, 1 largest, 2 smallest: the thresholds of
  // the positive and the negative tail differ, and Alternating Signs Quantization switches between
  // them from call to call): bank b uses the layer states [b * max_layers, (b + 1) * max_layers).
  std::vector<std::pair<int64_t, int32_t>> hint_sig[3];   // (n, k) per layer slot the hints belong to
  bool hints_reset[3] = {true, true, true};
  int last_bank = 0;
  int32_t last_layers = 0;
  DecompressPlan dplan;
  // benchmark timing: events recorded around the kernels of each call while enabled
  bool profiling = false;
  std::vector<hipEvent_t> ev_compress;     // triples: before accumulate, after it, after the phases
  std::vector<hipEvent_t> ev_decompress;   // triples: before table, after it, after the tiles
  std::vector<hipEvent_t> ev_pool;
};

namespace {

int build_compress_plan(rgc_ctx* ctx, CompressPlan& P, const rgc_layer* layers, int32_t L,
                        hipStream_t stream) {
  if (P.uploaded) RGC_HIP(hipEventSynchronize(P.uploaded));   // an older upload may still read staging
  else RGC_HIP(hipEventCreateWithFlags(&P.uploaded, hipEventDisableTiming));
  P.valid = false;
  // workgroups are handed out largest layer first so that the long per-layer tails start early
  std::vector<int32_t> order(L);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int32_t a, int32_t b) { return layers[a].n > layers[b].n; });
  std::vector<LayerDesc> desc(L);
  int64_t total_elems = 0;
  for (int32_t l = 0; l < L; ++l) total_elems += layers[l].n;
  const uint32_t kChunk = chunk_for(total_elems), kCap = kChunk / kCapDiv;
  P.chunk = kChunk;
  uint32_t wc = 0, wg = 0, grp = 0;
  uint64_t mem = 0;                        // entries of the member pool handed out to dense layers
  uint64_t lists = 0;                      // list entries handed out to them
  for (int32_t o = 0; o < L; ++o) {
    const int32_t l = order[o];
    const rgc_layer& in = layers[l];
    LayerDesc& d = desc[l];
    d.grad = in.grad;
    d.resid = in.residual;
    d.mom = in.momentum;
    d.out_idx = in.out_idx;
    d.out_val = in.out_val;
    d.out_count = in.out_count;
    d.n = static_cast<uint32_t>(in.n);
    d.k = static_cast<uint32_t>(in.k);
    d.wc_first = wc;
    d.wc_count = static_cast<uint32_t>((in.n + kChunk - 1) / kChunk);
    d.wg_first = wg;
    d.wg_count = (d.wc_count + kWavesPerBlock - 1) / kWavesPerBlock;
    d.grp_first = grp;
    grp += (d.wg_count + kElectGroupHost - 1) / kElectGroupHost;
    d.mem_cap = 0;
    d.mem_first = 0;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(in.grad) | reinterpret_cast<uintptr_t>(in.residual) |
                           reinterpret_cast<uintptr_t>(in.momentum);
    d.vec_ok = (bits & 15u) == 0 ? 1u : 0u;
    // speed-hint policy: aim the threshold at rank 2k + margin of this call, accept up to cmax
    const uint64_t k = d.k;
    uint64_t margin = std::max<uint64_t>(k / 2, 32);
    if (d.n <= kChunk) margin = std::min<uint64_t>(margin, std::max<uint64_t>(kCap / 4, 8));   // one list holds it all
    const uint64_t span = std::max<uint64_t>(d.n, kChunk);
    const uint64_t target = 2 * k + margin;   // rank the next threshold is aimed at
    const uint64_t per_chunk = (target * kChunk + span - 1) / span;         // expected per wave-chunk
    d.hintable = (2 * per_chunk + 16 <= kCap) ? 1u : 0u;
    // The candidates between the threshold aimed at and the k-th key fall into several hundred coarse
    // bins, and the one bin that holds the k-th key must fit the member list: beyond about a million
    // selected entries per layer it would not, and the hint would miss on every call.
    if (k > static_cast<uint64_t>(kMemberMax) * 256u) d.hintable = 0u;
    d.margin = static_cast<uint32_t>(margin);
    uint64_t cmax = std::min<uint64_t>(2 * target, (kCap / 2) * (span / kChunk));
    d.target = static_cast<uint32_t>(std::min<uint64_t>(target, 0xFFFFFFFFu));
    d.dense = 0;
    d.list_cap = 0;
    d.list_first = 0;
    d.pad_ = 0;
    if (!d.hintable) {
      // High densities (the warm-up period of Section 2.5): the short lists of the one-pass path cannot hold every
      // element from the threshold upwards.  Such a layer gets lists of its own, long enough for twice the number of
      // candidates aimed at, and its hint is aimed at rank k + margin and accepted from rank k to rank k + 2 margin.
      // The margin is wide (on the benchmark's tensors at 25 % the count above the hinted threshold comes out within
      // 3 % of k of the rank aimed at, 10 % now and then, and a miss costs more than a whole hint-free call): what it
      // costs is list entries, a twenty-fourth of the layer at most (at 1.5625 % a margin of k / 2 missed on most calls).
      const uint64_t margin2 = std::max<uint64_t>(std::min<uint64_t>(2 * k, d.n / 24), 64);
      if (k + 2 * margin2 < d.n) {
        const uint64_t aimed_per_chunk = ((k + margin2) * kChunk + span - 1) / span;
        d.dense = 1;
        // (twice the number aimed at, and the 256 slots a wave wants to see free before it lists another group)
        d.list_cap = static_cast<uint32_t>(std::min<uint64_t>(kChunk, (2 * aimed_per_chunk + 256 + 64 + 63) / 64 * 64));
        d.list_first = lists;
        lists += static_cast<uint64_t>(d.wc_count) * d.list_cap;
        d.mem_cap = static_cast<uint32_t>(std::max<uint64_t>(4096, d.n / 64) / kMemberShards * kMemberShards);
        d.mem_first = mem;
        mem += d.mem_cap + d.mem_cap / 4;       // (the sub-lists and the list for what they cannot hold)
        d.margin = static_cast<uint32_t>(margin2);
        d.target = static_cast<uint32_t>(k + margin2);
        cmax = k + 2 * margin2;
      }
    }
    d.cmax = static_cast<uint32_t>(std::min<uint64_t>(cmax, 0x7FFFFFFFu));
    wc += d.wc_count;
    wg += d.wg_count;
  }
  if (wc > ctx->wc_max) return RGC_ENOMEM;
  const size_t bytes_layers = sizeof(LayerDesc) * static_cast<size_t>(L);
  const size_t bytes_map = sizeof(uint32_t) * static_cast<size_t>(wg);
  RGC_HIP(P.staging.ensure(bytes_layers + bytes_map));
  if (P.d_layers.n < static_cast<size_t>(L)) RGC_HIP(P.d_layers.alloc(static_cast<size_t>(L)));
  if (P.d_wg2layer.n < wg) RGC_HIP(P.d_wg2layer.alloc(wg));
  std::memcpy(P.staging.p, desc.data(), bytes_layers);
  uint32_t* map = reinterpret_cast<uint32_t*>(static_cast<char*>(P.staging.p) + bytes_layers);
  for (int32_t o = 0; o < L; ++o) {
    const int32_t l = order[o];
    for (uint32_t i = 0; i < desc[l].wg_count; ++i) map[desc[l].wg_first + i] = static_cast<uint32_t>(l);
  }
  RGC_HIP(hipMemcpyAsync(P.d_layers.p, P.staging.p, bytes_layers, hipMemcpyHostToDevice, stream));
  RGC_HIP(hipMemcpyAsync(P.d_wg2layer.p, map, bytes_map, hipMemcpyHostToDevice, stream));
  RGC_HIP(hipEventRecord(P.uploaded, stream));
  P.key.resize(static_cast<size_t>(L));
  for (int32_t l = 0; l < L; ++l) {
    rgc_layer c{};
    c.grad = layers[l].grad; c.residual = layers[l].residual; c.momentum = layers[l].momentum; c.n = layers[l].n;
    c.k = layers[l].k; c.out_idx = layers[l].out_idx; c.out_val = layers[l].out_val; c.out_count = layers[l].out_count;
    P.key[l] = c;
  }
  P.num_wgs = wg;
  P.num_chunks = wc;
  P.write_bytes = 0;
  P.max_k = 0;
  P.any_dense = false;
  P.list_entries = lists;
  P.member_entries = mem;
  for (int32_t l = 0; l < L; ++l) {
    P.any_dense = P.any_dense || desc[l].dense != 0;
    P.write_bytes += static_cast<uint64_t>(layers[l].n) * (layers[l].momentum ? 8u : 4u);
    P.max_k = std::max(P.max_k, static_cast<uint32_t>(layers[l].k));
  }
  P.valid = true;
  return RGC_OK;
}

hipError_t take_event(rgc_ctx* ctx, hipStream_t stream, std::vector<hipEvent_t>& into) {
  hipEvent_t e = nullptr;
  if (!ctx->ev_pool.empty()) {
    e = ctx->ev_pool.back();
    ctx->ev_pool.pop_back();
  } else {
    hipError_t r = hipEventCreate(&e);
    if (r != hipSuccess) return r;
  }
  into.push_back(e);
  return hipEventRecord(e, stream);
}

void destroy_plan(CompressPlan& P) {
  if (P.uploaded) { (void)hipEventSynchronize(P.uploaded); (void)hipEventDestroy(P.uploaded); }
  P.uploaded = nullptr;
  P.d_layers.release();
  P.d_wg2layer.release();
  P.staging.release();
  P.valid = false;
}

}  // namespace

extern "C" {

int32_t rgc_k_for_density(int64_t n, uint32_t density_ppm) {
  if (n < 1) return 0;
  if (n >= (int64_t(1) << 31)) n = (int64_t(1) << 31) - 1;
  const unsigned long long num = static_cast<unsigned long long>(n) * density_ppm;
  unsigned long long k = (num + 999999ull) / 1000000ull;
  if (k < 1) k = 1;
  if (k > static_cast<unsigned long long>(n)) k = static_cast<unsigned long long>(n);
  return static_cast<int32_t>(k);
}

const char* rgc_strerror(int status) {
  switch (status) {
    case RGC_OK: return "ok";
    case RGC_EINVAL: return "invalid argument";
    case RGC_ENOMEM: return "scratch too small or allocation failed";
    case RGC_EHIP: return g_hip_error.c_str();
    case RGC_EINTERNAL: return "internal inconsistency reported by a kernel";
    default: return "unknown status";
  }
}

int rgc_create(rgc_ctx** out, int device_id, int64_t max_total_elems, int32_t max_layers) {
  if (!out) return RGC_EINVAL;
  *out = nullptr;
  if (max_total_elems < 1 || max_layers < 1 || device_id < 0) return RGC_EINVAL;
  int ndev = 0;
  RGC_HIP(hipGetDeviceCount(&ndev));
  if (device_id >= ndev) return RGC_EINVAL;
  DeviceGuard guard(device_id);
  if (!guard.ok) return fail_hip(hipErrorInvalidDevice, "hipSetDevice");
  std::unique_ptr<rgc_ctx> c(new (std::nothrow) rgc_ctx);
  if (!c) return RGC_ENOMEM;
  c->device = device_id;
  {
    int cus = 0;
    RGC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device_id));
    c->cus = static_cast<uint32_t>(std::max(1, cus));
  }
  c->max_total = max_total_elems;
  c->max_layers = max_layers;
  const uint32_t kChunk = chunk_smallest(), kCap = kChunk / kCapDiv;
  const uint64_t wc_max = static_cast<uint64_t>((max_total_elems + kChunk - 1) / kChunk) + static_cast<uint64_t>(max_layers);
  if (wc_max > 0x7FFFFFFFull) return RGC_ENOMEM;
  c->wc_max = static_cast<uint32_t>(wc_max);
  const size_t L = static_cast<size_t>(max_layers);
  hipError_t e = hipSuccess;
  auto chk = [&](hipError_t r) { if (e == hipSuccess && r != hipSuccess) e = r; };
  chk(c->d_state.alloc(3 * L));
  chk(c->d_hist.alloc(L * kHistBins));
  chk(c->d_coarse.alloc(L * kCoarseRep * kCoarseBins));
  chk(c->d_members.alloc(L * kMemberMax));
  chk(c->d_cand_cnt.alloc(wc_max));
  chk(c->d_wc_a.alloc(wc_max));
  chk(c->d_wc_b.alloc(wc_max));
  {
    // every wave-chunk owns chunk / kCapDiv slots whatever the chunk size: total / kCapDiv slots
    // plus one (partly used) chunk per layer at the largest chunk size a plan may pick
    const uint64_t largest = std::max<uint64_t>(16384, chunk_override());
    (void)kCap;
    chk(c->d_slots.alloc(static_cast<uint64_t>(max_total_elems) / kCapDiv + (static_cast<uint64_t>(max_layers) + 1) * (largest / kCapDiv)));
  }
  chk(c->d_err.alloc(2));                  // [0] internal inconsistencies of compression, [1] status of the message checks
  const uint64_t grp_max = wc_max / (kWavesPerBlock * kElectGroupHost) + 2 * L + 2;
  chk(c->d_group.alloc(grp_max));
  if (e == hipSuccess) chk(hipMemset(c->d_state.p, 0, sizeof(LayerState) * 3 * L));
  if (e == hipSuccess) chk(hipMemset(c->d_hist.p, 0, sizeof(uint32_t) * L * kHistBins));
  if (e == hipSuccess) chk(hipMemset(c->d_coarse.p, 0, sizeof(uint32_t) * L * kCoarseRep * kCoarseBins));
  if (e == hipSuccess) chk(hipMemset(c->d_cand_cnt.p, 0, sizeof(uint32_t) * wc_max));
  if (e == hipSuccess) chk(hipMemset(c->d_err.p, 0, 2 * sizeof(uint32_t)));
  if (e == hipSuccess) chk(hipMemset(c->d_group.p, 0, sizeof(uint32_t) * grp_max));
  if (e == hipSuccess) chk(hipDeviceSynchronize());
  if (e != hipSuccess) {
    rgc_ctx* raw = c.release();
    rgc_destroy(raw);
    if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return RGC_ENOMEM; }
    return fail_hip(e, "rgc_create allocation");
  }
  *out = c.release();
  return RGC_OK;
}

int rgc_destroy(rgc_ctx* ctx) {
  if (!ctx) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  for (auto& P : ctx->plans) destroy_plan(P);
  if (ctx->dplan.uploaded) { (void)hipEventSynchronize(ctx->dplan.uploaded); (void)hipEventDestroy(ctx->dplan.uploaded); }
  ctx->dplan.d_tables.release();
  ctx->dplan.d_tab.release();
  ctx->dplan.staging.release();
  ctx->d_state.release();
  ctx->d_hist.release();
  ctx->d_coarse.release();
  ctx->d_members.release();
  ctx->d_cand_cnt.release();
  ctx->d_wc_a.release();
  ctx->d_wc_b.release();
  ctx->d_slots.release();
  ctx->d_slots2.release();
  ctx->d_slots_u.release();
  ctx->d_members2.release();
  ctx->d_shards.release();
  ctx->d_err.release();
  ctx->d_group.release();
  ctx->d_norm_part.release();
  ctx->d_mean_part.release();
  ctx->d_moments.release();
  for (auto* v : {&ctx->ev_compress, &ctx->ev_decompress, &ctx->ev_pool})
    for (hipEvent_t e : *v) (void)hipEventDestroy(e);
  delete ctx;
  return RGC_OK;
}

int rgc_reset_hints(rgc_ctx* ctx) {
  if (!ctx) return RGC_EINVAL;
  for (bool& r : ctx->hints_reset) r = true;
  return RGC_OK;
}

int rgc_limit_optional_scratch(rgc_ctx* ctx, int64_t max_bytes) {
  if (!ctx) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  ctx->optional_scratch_cap = max_bytes;
  const uint64_t held = ctx->d_slots2.n * (sizeof(uint2) + sizeof(float)) + ctx->d_members2.n * sizeof(unsigned long long);
  if (max_bytes >= 0 && ctx->d_slots2.p && held > static_cast<uint64_t>(max_bytes)) {
    RGC_HIP(hipDeviceSynchronize());
    ctx->d_slots2.release();
    ctx->d_slots_u.release();
    ctx->d_members2.release();
  }
  return RGC_OK;
}

int rgc_poison_hints(rgc_ctx* ctx, int mode, void* hip_stream) {
  if (!ctx || mode < 0 || mode > 2) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  RGC_HIP(launch_poison(ctx->d_state.p, 3u * static_cast<uint32_t>(ctx->max_layers), mode,
                        static_cast<hipStream_t>(hip_stream)));
  for (bool& r : ctx->hints_reset) r = false;   // the poisoned values are to be used
  return RGC_OK;
}

}  // extern "C"

namespace {

// The caller's structs have padding bytes that a C caller need not initialise: the cached lists are compared
// field by field.
bool same_layers(const std::vector<rgc_layer>& key, const rgc_layer* layers, int32_t num_layers) {
  if (key.size() != static_cast<size_t>(num_layers)) return false;
  for (int32_t l = 0; l < num_layers; ++l) {
    const rgc_layer &a = key[l], &b = layers[l];
    if (a.grad != b.grad || a.residual != b.residual || a.momentum != b.momentum || a.n != b.n || a.k != b.k ||
        a.out_idx != b.out_idx || a.out_val != b.out_val || a.out_count != b.out_count)
      return false;
  }
  return true;
}

bool same_messages(const std::vector<rgc_msg>& key, const rgc_msg* msgs, size_t count) {
  if (key.size() != count) return false;
  for (size_t i = 0; i < count; ++i)
    if (key[i].idx != msgs[i].idx || key[i].val != msgs[i].val || key[i].count != msgs[i].count) return false;
  return true;
}

// Checks a layer list and finds (or builds) its plan.  On success *out is the plan and the device
// of the context is current.
int plan_for_layers(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, hipStream_t stream,
                    CompressPlan** out) {
  int64_t total = 0;
  for (int32_t l = 0; l < num_layers; ++l) {
    const rgc_layer& a = layers[l];
    if (!a.grad || !a.residual || !a.out_idx || !a.out_val || !a.out_count) return RGC_EINVAL;
    if (a.n < 1 || a.n >= (int64_t(1) << 31) || a.k < 1 || a.k > a.n) return RGC_EINVAL;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(a.grad) | reinterpret_cast<uintptr_t>(a.residual) |
                           reinterpret_cast<uintptr_t>(a.momentum) | reinterpret_cast<uintptr_t>(a.out_idx) |
                           reinterpret_cast<uintptr_t>(a.out_val) | reinterpret_cast<uintptr_t>(a.out_count);
    if (bits & 3u) return RGC_EINVAL;
    total += a.n;
  }
  if (total > ctx->max_total) return RGC_ENOMEM;

  // ---- find or build the plan for this exact layer list
  CompressPlan* plan = nullptr;
  for (auto& P : ctx->plans) {
    if (P.valid && same_layers(P.key, layers, num_layers)) {
      plan = &P;
      break;
    }
  }
  if (!plan) {
    CompressPlan* victim = &ctx->plans[0];
    for (auto& P : ctx->plans) {
      if (!P.valid) { victim = &P; break; }
      if (P.last_use < victim->last_use) victim = &P;
    }
    const int rc = build_compress_plan(ctx, *victim, layers, num_layers, stream);
    if (rc != RGC_OK) return rc;
    plan = victim;
  }
  plan->last_use = ++ctx->tick;
  *out = plan;
  return RGC_OK;
}

// Direction of the streaming pass of compression call number `call` (0: workgroups ascending).
// Every other call goes backwards when the call writes more than the memory-side cache holds
// (256 MB on MI355X): the tail of what the previous call wrote is then still cached and is read
// first.  Smaller layer sets stay cached whatever the order, and ascending order (largest layers
// first) is the better one for them.
constexpr uint64_t kMemorySideCacheBytes = 256ull << 20;
uint32_t streaming_direction(const CompressPlan* plan, uint64_t call) {
  return (plan->write_bytes > kMemorySideCacheBytes) ? static_cast<uint32_t>(call & 1u) : 0u;
}

void fill_plan_args(rgc_ctx* ctx, const CompressPlan* plan, CompressArgs& A) {
  A.layers = plan->d_layers.p;
  A.wg2layer = plan->d_wg2layer.p;
  A.chunk = plan->chunk;
  A.norm_parts = exact_parts_at(ctx->d_norm_part.p, ctx->wc_max);
}

}  // namespace

extern "C" {

int rgc_clip_coefficient(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float max_norm,
                         int32_t num_workers, float* coefficient, void* hip_stream) {
  if (!ctx || !layers || !coefficient || num_layers < 1 || num_layers > ctx->max_layers) return RGC_EINVAL;
  if (!(max_norm > 0.0f) || num_workers < 1 || (reinterpret_cast<uintptr_t>(coefficient) & 3u)) return RGC_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail_hip(hipErrorInvalidDevice, "hipSetDevice");
  CompressPlan* plan = nullptr;
  const int rc = plan_for_layers(ctx, layers, num_layers, stream, &plan);
  if (rc != RGC_OK) return rc;
  if (ctx->d_norm_part.n < ctx->wc_max * kExactWordsPerPart)                              // first use only
    RGC_HIP(ctx->d_norm_part.alloc(ctx->wc_max * kExactWordsPerPart));                    // (no more workgroups than wave-chunks)
  CompressArgs A{};
  fill_plan_args(ctx, plan, A);
  A.reverse = streaming_direction(plan, ctx->compress_calls) ^ 1u;   // against the direction of the compression call to come
  const float threshold = static_cast<float>(static_cast<double>(max_norm) / std::sqrt(static_cast<double>(num_workers)));
  RGC_HIP(launch_clip_coefficient(A, plan->num_wgs, threshold, coefficient, stream));
  return RGC_OK;
}

int rgc_message_means(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float* means,
                      void* hip_stream) {
  if (!ctx || !layers || !means || num_layers < 1 || num_layers > ctx->max_layers) return RGC_EINVAL;
  if (reinterpret_cast<uintptr_t>(means) & 3u) return RGC_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail_hip(hipErrorInvalidDevice, "hipSetDevice");
  CompressPlan* plan = nullptr;
  const int rc = plan_for_layers(ctx, layers, num_layers, stream, &plan);
  if (rc != RGC_OK) return rc;
  const size_t parts = static_cast<size_t>(ctx->max_layers) * kMeanPartsMax;
  if (ctx->d_mean_part.n < parts * kExactWordsPerPart)      // first use only
    RGC_HIP(ctx->d_mean_part.alloc(parts * kExactWordsPerPart));
  CompressArgs A{};
  fill_plan_args(ctx, plan, A);
  RGC_HIP(launch_message_means(A, static_cast<uint32_t>(num_layers), plan->max_k,
                               exact_parts_at(ctx->d_mean_part.p, parts), means, stream));
  return RGC_OK;
}

int rgc_compress_layers_threshold(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float momentum,
                                  const float* grad_scale, float* thresholds, int32_t* nnz, uint32_t flags,
                                  void* hip_stream) {
  if (!ctx || !layers || !thresholds || num_layers < 1 || num_layers > ctx->max_layers) return RGC_EINVAL;
  if (flags & ~(RGC_NO_MOMENTUM_MASK | RGC_NESTEROV | RGC_THRESHOLD_SEARCH)) return RGC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(thresholds) | reinterpret_cast<uintptr_t>(nnz) |
       reinterpret_cast<uintptr_t>(grad_scale)) & 3u) return RGC_EINVAL;
  for (int32_t l = 0; l < num_layers; ++l)
    if (layers[l].k > (int32_t(1) << 30)) return RGC_EINVAL;              // 2k entries must be countable
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail_hip(hipErrorInvalidDevice, "hipSetDevice");
  CompressPlan* plan = nullptr;
  const int rc = plan_for_layers(ctx, layers, num_layers, stream, &plan);
  if (rc != RGC_OK) return rc;
  if (ctx->d_norm_part.n < ctx->wc_max * kExactWordsPerPart)                              // first use only
    RGC_HIP(ctx->d_norm_part.alloc(ctx->wc_max * kExactWordsPerPart));
  if (ctx->d_moments.n < static_cast<size_t>(ctx->max_layers))
    RGC_HIP(ctx->d_moments.alloc(static_cast<size_t>(ctx->max_layers)));
  ThresholdArgs A{};
  A.layers = plan->d_layers.p;
  A.wg2layer = plan->d_wg2layer.p;
  A.thresholds = thresholds;
  A.nnz = nnz;
  A.grad_scale = grad_scale;
  A.sum_parts = exact_parts_at(ctx->d_norm_part.p, ctx->wc_max);
  A.part_max = reinterpret_cast<float*>(ctx->d_wc_b.p);
  A.counts = ctx->d_wc_a.p;
  A.listed = ctx->d_cand_cnt.p;
  A.slots = ctx->d_slots.p;
  A.cap = plan->chunk / kCapDiv;
  A.hist = ctx->d_hist.p;
  A.moments = ctx->d_moments.p;
  A.chunk = plan->chunk;
  A.search = (flags & RGC_THRESHOLD_SEARCH) ? 1u : 0u;
  A.mask_momentum = (flags & RGC_NO_MOMENTUM_MASK) ? 0u : 1u;
  A.nesterov = (flags & RGC_NESTEROV) ? 1u : 0u;
  A.m = momentum;
  // A searching call passes over the tensors four times and ends where it began; a reusing call passes once:
  // the call after it starts from the end it stopped at, whose data the memory-side cache still holds.
  const bool alternate = plan->write_bytes > kMemorySideCacheBytes;
  A.reverse = alternate ? ctx->threshold_reverse : 0u;
  RGC_HIP(launch_threshold_compress(A, plan->num_wgs, static_cast<uint32_t>(num_layers), stream));
  if (!A.search) ctx->threshold_reverse ^= 1u;
  ctx->compressed_since_decompress = true;
  return RGC_OK;
}

int rgc_compress_layers(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float momentum,
                        uint32_t flags, void* hip_stream) {
  return rgc_compress_layers_scaled(ctx, layers, num_layers, momentum, nullptr, flags, hip_stream);
}

int rgc_compress_layers_scaled(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float momentum,
                               const float* grad_scale, uint32_t flags, void* hip_stream) {
  if (!ctx || !layers || num_layers < 1 || num_layers > ctx->max_layers) return RGC_EINVAL;
  if (flags & ~(RGC_NO_MOMENTUM_MASK | RGC_NO_HINTS | RGC_NESTEROV | RGC_SELECT_LARGEST | RGC_SELECT_SMALLEST)) return RGC_EINVAL;
  if ((flags & RGC_SELECT_LARGEST) && (flags & RGC_SELECT_SMALLEST)) return RGC_EINVAL;
  if (reinterpret_cast<uintptr_t>(grad_scale) & 3u) return RGC_EINVAL;
  const int bank = (flags & RGC_SELECT_LARGEST) ? 1 : (flags & RGC_SELECT_SMALLEST) ? 2 : 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail_hip(hipErrorInvalidDevice, "hipSetDevice");
  CompressPlan* plan = nullptr;
  {
    const int rc = plan_for_layers(ctx, layers, num_layers, stream, &plan);
    if (rc != RGC_OK) return rc;
  }

  // ---- hints belong to a (n, k) sequence; anything else starts hint-free
  auto& hint_sig = ctx->hint_sig[bank];
  bool sig_same = !ctx->hints_reset[bank] && hint_sig.size() == static_cast<size_t>(num_layers);
  if (sig_same) {
    for (int32_t l = 0; l < num_layers; ++l)
      if (hint_sig[l].first != layers[l].n || hint_sig[l].second != layers[l].k) { sig_same = false; break; }
  }
  const bool no_hints = (flags & RGC_NO_HINTS) != 0;

  CompressArgs A{};
  A.layers = plan->d_layers.p;
  A.state = ctx->d_state.p + static_cast<size_t>(bank) * ctx->max_layers;
  A.sign_filter = bank ? 0xFFFFFFFFu : 0u;
  A.sign_xor = bank == 2 ? 0x80000000u : 0u;
  A.wg2layer = plan->d_wg2layer.p;
  A.hist = ctx->d_hist.p;
  A.coarse = ctx->d_coarse.p;
  A.members = ctx->d_members.p;
  A.cand_cnt = ctx->d_cand_cnt.p;
  A.slots = ctx->d_slots.p;
  A.wc_a = ctx->d_wc_a.p;
  A.wc_b = ctx->d_wc_b.p;
  A.errflag = ctx->d_err.p;
  A.group_done = ctx->d_group.p;
  A.chunk = plan->chunk;
  A.cap = A.chunk / kCapDiv;
  A.use_hints = (sig_same && !no_hints) ? 1u : 0u;
  A.update_hints = no_hints ? 0u : 1u;
  A.mask_momentum = (flags & RGC_NO_MOMENTUM_MASK) ? 0u : 1u;
  // The lists of dense layers are allocated by the first call that shows the context a plan with such layers (or one
  // that needs longer lists; hipFree waits for the kernels that may still use the old ones).  Without them (the device
  // is short of memory) those layers simply take the hint-free path, as they would on a first call.
  bool dense_ok = plan->any_dense;
  if (plan->any_dense && (ctx->d_slots2.n < plan->list_entries || ctx->d_members2.n < plan->member_entries || !ctx->d_shards.p)) {
    const uint64_t want = plan->list_entries * (sizeof(uint2) + sizeof(float)) + plan->member_entries * sizeof(unsigned long long);
    const bool capped = ctx->optional_scratch_cap >= 0 && want > static_cast<uint64_t>(ctx->optional_scratch_cap);
    hipError_t e = capped ? hipErrorOutOfMemory : ctx->d_slots2.alloc(plan->list_entries);
    if (e == hipSuccess) e = ctx->d_slots_u.alloc(plan->list_entries);
    if (e == hipSuccess) e = ctx->d_members2.alloc(plan->member_entries);
    if (e == hipSuccess && !ctx->d_shards.p) e = ctx->d_shards.alloc(static_cast<size_t>(ctx->max_layers) * kMemberLists * kShardStride);
    if (e != hipSuccess) {
      ctx->d_slots2.release();
      ctx->d_slots_u.release();
      ctx->d_members2.release();
      ctx->d_shards.release();
      if (e != hipErrorOutOfMemory) return fail_hip(e, "scratch allocation for dense layers");
      (void)hipGetLastError();
      dense_ok = false;
    }
  }
  A.dense_ok = dense_ok ? 1u : 0u;
  const bool dense = dense_ok && A.use_hints;
  A.slots2 = ctx->d_slots2.p;
  A.slots_u = ctx->d_slots_u.p;
  A.members2 = ctx->d_members2.p;
  A.shard_cnt = ctx->d_shards.p;
  A.reverse = streaming_direction(plan, ctx->compress_calls);
  ++ctx->compress_calls;
  ctx->compressed_since_decompress = true;
  A.nesterov = (flags & RGC_NESTEROV) ? 1u : 0u;
  // a call that leaves most of the device idle spreads its candidate lists over as many workgroups as it has
  A.list_group = plan->num_wgs <= kSmallCallWorkgroups ? 1u : kListGroup;
  A.grad_scale = grad_scale;
  A.m = momentum;
  A.launch = 1;
  // Dense layers that have a hint are streamed by a kernel of their own and skipped by accumulate_kernel (both
  // decide from the same state, which neither changes before its layer is done).  They are ranked at launch 2 and
  // written at launch 3 by lists_kernel; one whose hint misses has its residual put right at launch 2, where it
  // also starts on the five passes.
  if (ctx->profiling) RGC_HIP(take_event(ctx, stream, ctx->ev_compress));
  RGC_HIP(launch_accumulate(A, plan->num_wgs, stream));
  if (dense) RGC_HIP(launch_collect(A, plan->num_wgs, stream));
  if (ctx->profiling) RGC_HIP(take_event(ctx, stream, ctx->ev_compress));
  for (int launch = 2; launch <= kLaunches; ++launch) {
    A.launch = static_cast<uint32_t>(launch);
    RGC_HIP(launch_phase(A, plan->num_wgs, stream));
    if (dense && launch <= 3) RGC_HIP(launch_lists(A, plan->num_wgs, stream));
  }
  if (ctx->profiling) RGC_HIP(take_event(ctx, stream, ctx->ev_compress));
  if (!no_hints) {
    hint_sig.resize(num_layers);
    for (int32_t l = 0; l < num_layers; ++l) hint_sig[l] = {layers[l].n, layers[l].k};
    ctx->hints_reset[bank] = false;
  }
  ctx->last_bank = bank;
  ctx->last_layers = num_layers;
  return RGC_OK;
}

int rgc_last_paths(rgc_ctx* ctx, int32_t* out, int32_t num_layers, void* hip_stream) {
  if (!ctx || !out || num_layers < 1 || num_layers > ctx->max_layers) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  std::vector<LayerState> st(num_layers);
  uint32_t err = 0;
  RGC_HIP(hipMemcpyAsync(st.data(), ctx->d_state.p + static_cast<size_t>(ctx->last_bank) * ctx->max_layers,
                         sizeof(LayerState) * num_layers, hipMemcpyDeviceToHost, stream));
  RGC_HIP(hipMemcpyAsync(&err, ctx->d_err.p, sizeof err, hipMemcpyDeviceToHost, stream));
  RGC_HIP(hipStreamSynchronize(stream));
  for (int32_t l = 0; l < num_layers; ++l) out[l] = static_cast<int32_t>(st[l].path);
  return err ? RGC_EINTERNAL : RGC_OK;
}

int rgc_last_error(rgc_ctx* ctx, void* hip_stream) {
  if (!ctx) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  uint32_t err = 0;
  RGC_HIP(hipMemcpyAsync(&err, ctx->d_err.p, sizeof err, hipMemcpyDeviceToHost, stream));
  RGC_HIP(hipStreamSynchronize(stream));
  return err ? RGC_EINTERNAL : RGC_OK;
}

int rgc_last_stats(rgc_ctx* ctx, int64_t* out, int32_t num_layers, void* hip_stream) {
  if (!ctx || !out || num_layers < 1 || num_layers > ctx->max_layers) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  std::vector<LayerState> st(num_layers);
  RGC_HIP(hipMemcpyAsync(st.data(), ctx->d_state.p + static_cast<size_t>(ctx->last_bank) * ctx->max_layers,
                         sizeof(LayerState) * num_layers, hipMemcpyDeviceToHost, stream));
  RGC_HIP(hipStreamSynchronize(stream));
  for (int32_t l = 0; l < num_layers; ++l) {
    out[5 * l + 0] = st[l].path;
    out[5 * l + 1] = st[l].stat_candidates;
    out[5 * l + 2] = st[l].stat_members;
    out[5 * l + 3] = st[l].T;
    out[5 * l + 4] = st[l].stat_misses;
  }
  return RGC_OK;
}

int rgc_selftest(rgc_ctx* ctx, void* hip_stream) {
  if (!ctx) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DevBuf<uint32_t> io;
  RGC_HIP(io.alloc(768));
  std::vector<uint32_t> h(768, 0), ref(768, 0);
  uint32_t x = 12345u, sum = 0;
  for (int i = 0; i < 256; ++i) {
    x = x * 1664525u + 1013904223u;
    h[i] = (x >> 20) & 0x3FFu;
  }
  for (int i = 0; i < 256; ++i) { ref[i] = sum; sum += h[i]; }
  ref[256] = sum;
  for (int w = 0; w < 4; ++w) {
    uint32_t r = 0;
    for (int lane = 0; lane < 64; ++lane) { ref[512 + w * 64 + lane] = r; r += h[w * 64 + lane] & 1u; }
  }
  hipError_t e = hipMemcpyAsync(io.p, h.data(), 768 * 4, hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) e = launch_wave_scan_selftest(io.p, stream);
  if (e == hipSuccess) e = hipMemcpyAsync(h.data(), io.p, 768 * 4, hipMemcpyDeviceToHost, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  io.release();
  if (e != hipSuccess) return fail_hip(e, "rgc_selftest");
  for (int i = 0; i <= 256; ++i) if (h[i] != ref[i]) return RGC_EINTERNAL;
  for (int i = 512; i < 768; ++i) if (h[i] != ref[i]) return RGC_EINTERNAL;
  return RGC_OK;
}

int rgc_decompress_accumulate(rgc_ctx* ctx, const rgc_msg* msgs, int32_t num_workers, int32_t num_layers,
                              float* const* dense, const int64_t* n, float scale, uint32_t flags,
                              void* hip_stream) {
  if (!ctx || !dense || !n || num_layers < 1 || num_workers < 0) return RGC_EINVAL;
  if (num_workers > 0 && !msgs) return RGC_EINVAL;
  const bool validate = (flags & RGC_VALIDATE) != 0;
  const bool one_value = (flags & RGC_ONE_VALUE) != 0;
  flags &= ~(RGC_VALIDATE | RGC_ONE_VALUE);
  if (flags != RGC_OVERWRITE && flags != RGC_ADD_TO_DST) return RGC_EINVAL;
  if (static_cast<int64_t>(num_workers) * num_layers > (int64_t(1) << 24)) return RGC_EINVAL;
  for (int32_t l = 0; l < num_layers; ++l) {
    if (!dense[l] || n[l] < 1 || n[l] >= (int64_t(1) << 31)) return RGC_EINVAL;
    if (reinterpret_cast<uintptr_t>(dense[l]) & 3u) return RGC_EINVAL;
  }
  const size_t NM = static_cast<size_t>(num_workers) * num_layers;
  for (size_t i = 0; i < NM; ++i) {
    const rgc_msg& m = msgs[i];
    if (m.count < 0 || m.count > n[i % num_layers]) return RGC_EINVAL;
    if (m.count > 0 && (!m.idx || !m.val)) return RGC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(m.idx) | reinterpret_cast<uintptr_t>(m.val)) & 3u) return RGC_EINVAL;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail_hip(hipErrorInvalidDevice, "hipSetDevice");

  DecompressPlan& P = ctx->dplan;
  const bool same = P.valid && P.workers == num_workers && P.layers == num_layers &&
                    same_messages(P.key_msgs, msgs, NM) &&
                    std::memcmp(P.key_dense.data(), dense, sizeof(float*) * num_layers) == 0 &&
                    std::memcmp(P.key_n.data(), n, sizeof(int64_t) * num_layers) == 0;
  if (!same) {
    if (P.uploaded) RGC_HIP(hipEventSynchronize(P.uploaded));
    else RGC_HIP(hipEventCreateWithFlags(&P.uploaded, hipEventDisableTiming));
    P.valid = false;
    // geometry
    std::vector<uint32_t> layer_tiles(num_layers), layer_col(num_layers);
    uint64_t tiles = 0, stride = 0;
    for (int32_t l = 0; l < num_layers; ++l) {
      layer_tiles[l] = static_cast<uint32_t>((n[l] + kTile - 1) >> kTileShift);
      layer_col[l] = static_cast<uint32_t>(stride);
      tiles += layer_tiles[l];
      stride += layer_tiles[l] + 1u;
    }
    const bool need_table = num_workers > kBatchWorkers;   // only the any-number-of-workers kernel reads the offset table
    uint64_t blocks = 0;                                    // ... which is built by one workgroup per 1024 entries of a message
    if (need_table)
      for (size_t i = 0; i < NM; ++i) blocks += std::max<uint64_t>(1, (static_cast<uint64_t>(msgs[i].count) + 1023) / 1024);
    const uint64_t tab_words = stride * static_cast<uint64_t>(std::max(num_workers, 1));
    if (tiles > 0x7FFFFFFFull || blocks > 0x7FFFFFFFull || tab_words > 0xFFFFFFFFull) return RGC_ENOMEM;
    const size_t off_msgs = 0;
    const size_t off_layers = off_msgs + sizeof(MsgDesc) * std::max<size_t>(NM, 1);
    const size_t off_blocks = off_layers + sizeof(DecompressLayer) * num_layers;
    const size_t bytes = off_blocks + sizeof(BlockDesc) * std::max<uint64_t>(blocks, 1);
    RGC_HIP(P.staging.ensure(bytes));
    if (P.d_tables.n < bytes) {
      hipError_t e = P.d_tables.alloc(bytes);
      if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return RGC_ENOMEM; }
      RGC_HIP(e);
    }
    if (need_table && P.d_tab.n < tab_words) {
      hipError_t e = P.d_tab.alloc(tab_words);
      if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return RGC_ENOMEM; }
      RGC_HIP(e);
    }
    char* base = static_cast<char*>(P.staging.p);
    MsgDesc* hm = reinterpret_cast<MsgDesc*>(base + off_msgs);
    DecompressLayer* hl = reinterpret_cast<DecompressLayer*>(base + off_layers);
    BlockDesc* hb = reinterpret_cast<BlockDesc*>(base + off_blocks);
    uint64_t nb = 0;
    for (uint32_t l = 0; l < static_cast<uint32_t>(num_layers); ++l) {
      for (uint32_t w = 0; w < static_cast<uint32_t>(num_workers); ++w) {
        const rgc_msg& in = msgs[static_cast<size_t>(w) * num_layers + l];
        const size_t i = static_cast<size_t>(l) * num_workers + w;      // device order: [layer][worker]
        hm[i].idx = in.idx;
        hm[i].val = in.val;
        hm[i].count = static_cast<uint32_t>(in.count);
        hm[i].tab_base = layer_col[l];
        if (need_table) {
          const uint32_t cnt = hm[i].count;
          uint32_t first = 0;
          do {
            hb[nb].msg = static_cast<uint32_t>(i);
            hb[nb].first = first;
            ++nb;
            first += 1024;
          } while (first < cnt);
        }
      }
    }
    uint32_t tile_base = 0;
    for (int32_t l = 0; l < num_layers; ++l) {
      hl[l].dense = dense[l];
      hl[l].n = static_cast<uint32_t>(n[l]);
      hl[l].tiles = layer_tiles[l];
      hl[l].tile_base = tile_base;
      hl[l].row_base = layer_col[l];
      hl[l].pad[0] = hl[l].pad[1] = 0;
      tile_base += layer_tiles[l];
    }
    RGC_HIP(hipMemcpyAsync(P.d_tables.p, P.staging.p, bytes, hipMemcpyHostToDevice, stream));
    RGC_HIP(hipEventRecord(P.uploaded, stream));
    DecompressArgs& A = P.args;
    A.msgs = reinterpret_cast<const MsgDesc*>(P.d_tables.p + off_msgs);
    A.layers = reinterpret_cast<const DecompressLayer*>(P.d_tables.p + off_layers);
    A.blocks = reinterpret_cast<const BlockDesc*>(P.d_tables.p + off_blocks);
    A.tab = P.d_tab.p;
    A.tab_stride = static_cast<uint32_t>(stride);
    A.cus = ctx->cus;
    A.num_workers = static_cast<uint32_t>(num_workers);
    A.num_layers = static_cast<uint32_t>(num_layers);
    A.num_tiles = static_cast<uint32_t>(tiles);
    A.num_blocks = static_cast<uint32_t>(nb);
    P.key_msgs.resize(NM);
    for (size_t i = 0; i < NM; ++i) {
      rgc_msg c{};
      c.idx = msgs[i].idx; c.val = msgs[i].val; c.count = msgs[i].count;
      P.key_msgs[i] = c;
    }
    P.key_dense.assign(dense, dense + num_layers);
    P.key_n.assign(n, n + num_layers);
    P.workers = num_workers;
    P.layers = num_layers;
    P.valid = true;
  }
  DecompressArgs A = P.args;
  A.add_to_dst = (flags == RGC_ADD_TO_DST) ? 1u : 0u;
  A.scale = scale;
  // A compression call since the last decompression: the tails of its tensors are in the memory-side
  // cache and its next call will start with them, so this call leaves them there.
  A.one_value = one_value ? 1u : 0u;
  A.stream_msgs = ctx->compressed_since_decompress ? 1u : 0u;
  ctx->compressed_since_decompress = false;
  if (validate) RGC_HIP(launch_decompress_validate(A, ctx->d_err.p + 1, stream));
  if (ctx->profiling) RGC_HIP(take_event(ctx, stream, ctx->ev_decompress));
  RGC_HIP(launch_decompress_table(A, stream));
  if (ctx->profiling) RGC_HIP(take_event(ctx, stream, ctx->ev_decompress));
  RGC_HIP(launch_decompress_tiles(A, stream));
  if (ctx->profiling) RGC_HIP(take_event(ctx, stream, ctx->ev_decompress));
  return RGC_OK;
}

int rgc_decompress_status(rgc_ctx* ctx, uint32_t* out_status, void* hip_stream) {
  if (!ctx || !out_status) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  uint32_t word = 0;
  RGC_HIP(hipMemcpyAsync(&word, ctx->d_err.p + 1, sizeof word, hipMemcpyDeviceToHost, stream));
  RGC_HIP(hipMemsetAsync(ctx->d_err.p + 1, 0, sizeof word, stream));
  RGC_HIP(hipStreamSynchronize(stream));
  *out_status = word;
  return RGC_OK;
}

int rgc_profile_enable(rgc_ctx* ctx, int enable) {
  if (!ctx) return RGC_EINVAL;
  ctx->profiling = enable != 0;
  return RGC_OK;
}

int rgc_profile_read(rgc_ctx* ctx, double* out_ms, int64_t* out_calls) {
  if (!ctx || !out_ms || !out_calls) return RGC_EINVAL;
  DeviceGuard guard(ctx->device);
  for (int i = 0; i < 4; ++i) out_ms[i] = 0.0;
  auto drain = [&](std::vector<hipEvent_t>& ev, double* ms, int64_t* calls) -> int {
    *calls = static_cast<int64_t>(ev.size() / 3);
    for (size_t i = 0; i + 2 < ev.size(); i += 3) {
      float a = 0.f, b = 0.f;
      RGC_HIP(hipEventSynchronize(ev[i + 2]));
      RGC_HIP(hipEventElapsedTime(&a, ev[i], ev[i + 1]));
      RGC_HIP(hipEventElapsedTime(&b, ev[i + 1], ev[i + 2]));
      ms[0] += a;
      ms[1] += b;
    }
    for (hipEvent_t e : ev) ctx->ev_pool.push_back(e);
    ev.clear();
    return RGC_OK;
  };
  int rc = drain(ctx->ev_compress, out_ms, &out_calls[0]);
  if (rc != RGC_OK) return rc;
  return drain(ctx->ev_decompress, out_ms + 2, &out_calls[1]);
}

}  // extern "C"
