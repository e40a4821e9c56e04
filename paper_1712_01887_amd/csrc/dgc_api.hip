// Host side of libdgc: argument checks, the host arithmetic of the method
// (k_j, sample plan, warm-up table), workspace management and launch order.
// Every step of the path itself runs in the kernels of dgc_compress.hip, dgc_receive.hip and
// dgc_wire.hip.

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "dgc_internal.h"

using namespace dgc;

struct dgc_handle {
  dgc_config cfg;
  uint64_t id = 0;                   // unique in the process: what the workspace registry records
  int32_t num_tensors = 0;
  int64_t n = 0;
  std::vector<int64_t> offsets;      // T + 1
  std::vector<double> warmup;        // densities
  int64_t warmup_stage_len = 1;      // iterations every entry of the table is held
  // plan under cfg.density
  std::vector<TensorPlan> plans;     // T
  std::vector<int64_t> k;            // T
  std::vector<int64_t> draws;        // T
  std::vector<uint32_t> tile_info;   // ceil(n / kWaveTile)
  std::vector<float> tile_thr_init;  // ceil(n / kWaveTile): NaN where a tile is not wholly inside one tensor
  std::vector<EmitBlock> emit_blocks;  // work list of the emit pass
  std::vector<MergeBlock> merge_blocks;  // work list of the receive side: ranges of several emit parts
  std::vector<MergeBlock> part_blocks;   // the same with one emit part per range (warm-up densities)
  bool layout_may_overflow = true;       // some region of the registered layout is smaller than its tensor
  int64_t last_replace_expected = 0;     // pairs per range the payloads of the last dgc_decompress_replace_regions call let expect
  WorkspaceLayout lay{};
  // what the bound workspace currently holds
  void* ws = nullptr;
  bool ws_static_valid = false;      // offsets + tile table
  bool ws_plan_valid = false;
  bool ws_layout_valid = false;
  std::vector<int64_t> ws_out_offsets;
  std::vector<uint32_t> wire_first_block;  // T + 1: encoder workgroup slots per region of the bound layout
  size_t wire_slots = 0;                   // words reserved for block sums of the wire-format passes
  // optional kernel timing: five events per dgc_compress call
  // (start, after norm, after select, after stream, after emit)
  std::vector<hipEvent_t> prof_events;
  int32_t prof_capacity = 0;  // calls that can be recorded before a collect
  int32_t prof_calls = 0;
};

namespace {

// Text of the most recent failed HIP call on this thread (for dgc_last_error_string).
thread_local char g_last_error[256] = "";

bool hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  std::snprintf(g_last_error, sizeof(g_last_error), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
  (void)hipGetLastError();  // clear the sticky launch error so later calls start clean
  return false;
}

// Which handle's tables a workspace holds.  A handle keeps host-side flags for what it has
// uploaded into the workspace it used last; they mean something only while no other handle has
// written its own tables there in between, which this map records (workspace address -> id of
// the handle that uploaded last).
std::mutex g_registry_mutex;
std::unordered_map<const void*, uint64_t> g_workspace_owner;
std::atomic<uint64_t> g_next_handle_id{1};

bool workspace_owned_by(const void* ws, uint64_t id) {
  std::lock_guard<std::mutex> lock(g_registry_mutex);
  auto it = g_workspace_owner.find(ws);
  return it != g_workspace_owner.end() && it->second == id;
}

void workspace_claim(const void* ws, uint64_t id) {
  std::lock_guard<std::mutex> lock(g_registry_mutex);
  g_workspace_owner[ws] = id;
}

void workspace_release_all(uint64_t id) {
  std::lock_guard<std::mutex> lock(g_registry_mutex);
  for (auto it = g_workspace_owner.begin(); it != g_workspace_owner.end();)
    it = it->second == id ? g_workspace_owner.erase(it) : std::next(it);
}

// Scratch memory for callers that cannot allocate (dgc_compress_static): a workspace that is
// part of the library's code object.  Every GPU the process uses holds its own copy at its own
// address; in host code the array's name is only a handle for hipGetSymbolAddress, which is
// asked once per device, with that device current, and whose answer is what host code passes
// on (to the kernels, as the workspace pointer of dgc_compress).
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

constexpr size_t kAlign = 256;
constexpr double kMergeMaxDensity = 0.005;   // receive side: merge by element range in LDS up to here
constexpr double kStagedMinDensity = 0.005;  // compress: staged streaming pass above this density
constexpr int kProfEvents = 5;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Device address of this device's copy of `scratch`; *known_only: do not ask the runtime, fail if
// the address has not been asked for yet.
dgc_status static_scratch(void** out, bool known_only) {
  int dev = -1;
  if (!hip_ok(hipGetDevice(&dev), "query the current device")) return DGC_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return DGC_ERR_CAPACITY;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    if (known_only) return DGC_ERR_STATE;
    void* p = nullptr;
    if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "address of the static scratch array")) return DGC_ERR_HIP;
    if (!p) return DGC_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DGC_OK;
}

bool valid_density(double d) { return d > 0.0 && d <= 1.0; }

// paper: Section 4.1 lists the warm-up sparsities 75 %, 93.75 %, 98.4375 %, 99.6 %, 99.9 %.
const double kDefaultWarmup[5] = {0.25, 0.0625, 0.015625, 0.004, 0.001};

int64_t topk_count(double density, int64_t n) {
  int64_t k = (int64_t)std::ceil(density * (double)n);
  if (k < 1) k = 1;
  if (k > n) k = n;
  return k;
}

// Host arithmetic of the sampled threshold (paper: Section 5).  The wanted
// sample size is ratio * n clamped to [sample_min, sample_max]; a tensor no
// larger than that is used whole.  Otherwise ceil(s / B) aligned blocks of B
// consecutive elements are drawn and the threshold is the magnitude of
// descending rank ceil(d * draws * B) in the sample.
void build_plan(dgc_handle* h) {
  const dgc_config& c = h->cfg;
  const int64_t B = c.sample_block;
  for (int32_t j = 0; j < h->num_tensors; ++j) {
    const int64_t n = h->offsets[j + 1] - h->offsets[j];
    TensorPlan& p = h->plans[j];
    p.offset = h->offsets[j];
    p.n = n;
    const int64_t k = topk_count(c.density, n);
    h->k[j] = k;
    p.k = (int32_t)k;
    {
      const double lim = std::floor((double)c.refine_alpha * (double)k);
      p.refine_limit = lim >= 2147483647.0 ? 2147483647 : (int32_t)lim;
    }
    int64_t want = (int64_t)std::ceil(c.sample_ratio * (double)n);
    if (want > c.sample_max) want = c.sample_max;
    if (want < c.sample_min) want = c.sample_min;
    const int64_t s = want < n ? want : n;
    if ((c.flags & DGC_FLAG_EXACT_SELECT) || s >= n || n / B < 1) {
      p.exact = 1;
      p.count = (int32_t)n;
      p.rank = (int32_t)k;
      p.nblocks = 0;
      h->draws[j] = 0;
    } else {
      const int64_t draws = (s + B - 1) / B;
      const int64_t count = draws * B;
      int64_t rank = (int64_t)std::ceil(c.density * (double)count);
      if (rank < 1) rank = 1;
      p.exact = 0;
      p.count = (int32_t)count;
      p.rank = (int32_t)rank;
      p.nblocks = (uint32_t)(n / B);
      h->draws[j] = draws;
    }
  }
  h->ws_plan_valid = false;
}

void build_layout(dgc_handle* h) {
  const size_t T = (size_t)h->num_tensors;
  const size_t tiles = (size_t)((h->n + kWaveTile - 1) / kWaveTile);
  WorkspaceLayout& l = h->lay;
  size_t off = 0;
  l.state = off;        off = align_up(off + sizeof(DeviceState));
  l.partials = off;     off = align_up(off + sizeof(double) * kNormMaxBlocks);
  l.offsets = off;      off = align_up(off + sizeof(int64_t) * (T + 1));
  l.out_offsets = off;  off = align_up(off + sizeof(int64_t) * (T + 1));
  l.plans = off;        off = align_up(off + sizeof(TensorPlan) * T);
  l.thr = off;          off = align_up(off + sizeof(float) * T);
  l.tile_info = off;    off = align_up(off + sizeof(uint32_t) * tiles);
  l.tile_thr = off;     off = align_up(off + sizeof(float) * tiles);
  l.emit_blocks = off;  off = align_up(off + sizeof(EmitBlock) * h->emit_blocks.size());
  l.tile_count = off;   off = align_up(off + sizeof(uint32_t) * tiles);
  l.merge_blocks = off; off = align_up(off + sizeof(MergeBlock) * h->merge_blocks.size());
  l.part_blocks = off;  off = align_up(off + sizeof(MergeBlock) * h->part_blocks.size());
  // (first pair, pairs) of every payload inside every part, left by the search that precedes the part kernels
  l.part_found = off;   off = align_up(off + 2 * sizeof(int32_t) * kMaxPayloads * h->part_blocks.size());
  // wire format: one block sum per kWireChunk pairs of every region (encoder, at most
  // n / kWireChunk + T) or per kWireChunk entries of every payload (decoder, an entry
  // stream of a set of n elements has at most n + (n >> 16) entries)
  {
    const size_t enc = (size_t)(h->n / kWireChunk) + T + 1;
    const size_t dec = (size_t)kMaxPayloads * ((size_t)((h->n + (h->n >> 16)) / kWireChunk) + 2);
    h->wire_slots = enc > dec ? enc : dec;
  }
  l.wire_first_block = off; off = align_up(off + sizeof(uint32_t) * (T + 1));
  l.wire_sums = off;    off = align_up(off + sizeof(uint32_t) * h->wire_slots);
  l.mask = off;         off = align_up(off + sizeof(uint16_t) * 64 * tiles);
  l.total = off;
  // optional: staging arrays of the streaming pass at warm-up densities
  l.stage_v = off;      off = align_up(off + sizeof(float) * (size_t)h->n);
  l.stage_u = off;      off = align_up(off + sizeof(float) * (size_t)h->n);
  l.total_staged = off;
}

template <typename T>
T* at(void* ws, size_t off) {
  return reinterpret_cast<T*>(static_cast<char*>(ws) + off);
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

dgc_status check_layout(const dgc_handle* h, const int64_t* oo) {
  if (!oo || oo[0] != 0) return DGC_ERR_INVALID_ARG;
  for (int32_t j = 0; j < h->num_tensors; ++j)
    if (oo[j + 1] < oo[j]) return DGC_ERR_INVALID_ARG;
  if (oo[h->num_tensors] >= (int64_t)1 << 31) return DGC_ERR_INVALID_ARG;
  return DGC_OK;
}

// Make the workspace hold the static tables, the current plan and the payload
// layout.  Copies are stream-ordered; the sources are host vectors that stay
// alive in the handle (the runtime stages pageable memory before returning).
// The host-side flags say what has been ENQUEUED, so nothing may be uploaded while the stream
// is being captured into a graph (a capture runs nothing, and may be thrown away): such a call
// is refused with DGC_ERR_STATE, and the caller makes its first call on a workspace, and the
// first one after a change of density or payload layout, eagerly.
dgc_status sync_workspace(dgc_handle* h, void* ws, size_t ws_bytes, const int64_t* out_offsets,
                          bool need_plan, hipStream_t stream) {
  if (!ws) return DGC_ERR_INVALID_ARG;
  if (!aligned(ws, kAlign)) return DGC_ERR_ALIGNMENT;
  if (ws_bytes < h->lay.total) return DGC_ERR_CAPACITY;
  const size_t T = (size_t)h->num_tensors;
  if (ws != h->ws || !workspace_owned_by(ws, h->id)) {
    h->ws = ws;
    h->ws_static_valid = h->ws_plan_valid = h->ws_layout_valid = false;
  }
  const bool layout_same = !out_offsets ||
                           (h->ws_layout_valid &&
                            std::memcmp(h->ws_out_offsets.data(), out_offsets, sizeof(int64_t) * (T + 1)) == 0);
  if (!h->ws_static_valid || (need_plan && !h->ws_plan_valid) || !layout_same) {
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (!hip_ok(hipStreamIsCapturing(stream, &capturing), "query stream capture")) return DGC_ERR_HIP;
    if (capturing != hipStreamCaptureStatusNone) {
      std::snprintf(g_last_error, sizeof(g_last_error),
                    "the workspace tables must be uploaded, which cannot be captured: make this call once outside the capture");
      return DGC_ERR_STATE;
    }
  }
  if (!h->ws_static_valid) {
    workspace_claim(ws, h->id);
    if (!hip_ok(launch_clear_words(at<uint32_t>(ws, h->lay.state), sizeof(DeviceState) / sizeof(uint32_t), stream),
                "clear workspace state"))
      return DGC_ERR_HIP;
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.offsets), h->offsets.data(),
                               sizeof(int64_t) * (T + 1), hipMemcpyHostToDevice, stream),
                "upload offsets"))
      return DGC_ERR_HIP;
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.tile_info), h->tile_info.data(),
                               sizeof(uint32_t) * h->tile_info.size(), hipMemcpyHostToDevice, stream),
                "upload tile table"))
      return DGC_ERR_HIP;
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.tile_thr), h->tile_thr_init.data(),
                               sizeof(float) * h->tile_thr_init.size(), hipMemcpyHostToDevice, stream),
                "upload tile thresholds"))
      return DGC_ERR_HIP;
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.emit_blocks), h->emit_blocks.data(),
                               sizeof(EmitBlock) * h->emit_blocks.size(), hipMemcpyHostToDevice, stream),
                "upload emit work list"))
      return DGC_ERR_HIP;
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.merge_blocks), h->merge_blocks.data(),
                               sizeof(MergeBlock) * h->merge_blocks.size(), hipMemcpyHostToDevice, stream),
                "upload merge work list"))
      return DGC_ERR_HIP;
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.part_blocks), h->part_blocks.data(),
                               sizeof(MergeBlock) * h->part_blocks.size(), hipMemcpyHostToDevice, stream),
                "upload part work list"))
      return DGC_ERR_HIP;
    h->ws_static_valid = true;
  }
  if (need_plan && !h->ws_plan_valid) {
    if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.plans), h->plans.data(), sizeof(TensorPlan) * T,
                               hipMemcpyHostToDevice, stream),
                "upload selection plan"))
      return DGC_ERR_HIP;
    h->ws_plan_valid = true;
  }
  if (out_offsets) {
    if (!layout_same) {
      h->ws_out_offsets.assign(out_offsets, out_offsets + T + 1);
      if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.out_offsets), h->ws_out_offsets.data(),
                                 sizeof(int64_t) * (T + 1), hipMemcpyHostToDevice, stream),
                  "upload payload layout"))
        return DGC_ERR_HIP;
      h->layout_may_overflow = false;
      for (size_t j = 0; j < T; ++j)
        if (out_offsets[j + 1] - out_offsets[j] < h->offsets[j + 1] - h->offsets[j]) h->layout_may_overflow = true;
      uint64_t slots = 0;
      for (size_t j = 0; j < T; ++j) {
        h->wire_first_block[j] = (uint32_t)slots;
        slots += (uint64_t)((out_offsets[j + 1] - out_offsets[j] + kWireChunk - 1) / kWireChunk);
      }
      h->wire_first_block[T] = (uint32_t)slots;
      if (!hip_ok(hipMemcpyAsync(at<char>(ws, h->lay.wire_first_block), h->wire_first_block.data(),
                                 sizeof(uint32_t) * (T + 1), hipMemcpyHostToDevice, stream),
                  "upload encoder slots"))
        return DGC_ERR_HIP;
      h->ws_layout_valid = true;
    }
  }
  return DGC_OK;
}

}  // namespace

extern "C" {

int32_t dgc_version(void) { return 1001; }

const char* dgc_last_error_string(void) { return g_last_error; }

const char* dgc_status_string(dgc_status s) {
  switch (s) {
    case DGC_OK: return "ok";
    case DGC_ERR_INVALID_ARG: return "invalid argument";
    case DGC_ERR_ALIGNMENT: return "buffer not aligned";
    case DGC_ERR_CAPACITY: return "capacity exceeded";
    case DGC_ERR_HIP: return "HIP runtime error";
    case DGC_ERR_STATE: return "invalid state";
    default: return "unknown status";
  }
}

dgc_status dgc_config_default(dgc_config* cfg) {
  if (!cfg) return DGC_ERR_INVALID_ARG;
  std::memset(cfg, 0, sizeof(*cfg));
  cfg->momentum = 0.9f;
  cfg->clip_threshold = 0.0f;
  cfg->num_workers = 1;
  cfg->flags = 0;
  cfg->density = 0.001;
  cfg->sample_ratio = 0.01;
  cfg->sample_min = 4096;
  cfg->sample_max = 32768;
  cfg->sample_block = 32;
  cfg->scale_override = std::nanf("");
  cfg->seed = 0;
  cfg->refine_alpha = 0.0f;
  cfg->reserved = 0;
  return DGC_OK;
}

dgc_status dgc_create(dgc_handle** out, const dgc_config* cfg, int32_t num_tensors,
                      const int64_t* offsets_host) {
  if (!out) return DGC_ERR_INVALID_ARG;
  *out = nullptr;
  if (!cfg || !offsets_host || num_tensors < 1) return DGC_ERR_INVALID_ARG;
  if (!valid_density(cfg->density) || cfg->num_workers < 1) return DGC_ERR_INVALID_ARG;
  if (!(cfg->momentum >= 0.0f) || !(cfg->momentum <= 1.0f)) return DGC_ERR_INVALID_ARG;
  if (!(cfg->sample_ratio > 0.0) || !(cfg->sample_ratio <= 1.0)) return DGC_ERR_INVALID_ARG;
  const int32_t B = cfg->sample_block;
  if (B < 1 || B > 64 || (B & (B - 1)) != 0) return DGC_ERR_INVALID_ARG;
  if (cfg->sample_min < B || cfg->sample_max < cfg->sample_min) return DGC_ERR_INVALID_ARG;
  if (cfg->clip_threshold != cfg->clip_threshold) return DGC_ERR_INVALID_ARG;
  if (!(cfg->refine_alpha == 0.0f || cfg->refine_alpha >= 1.0f)) return DGC_ERR_INVALID_ARG;
  if (offsets_host[0] != 0) return DGC_ERR_INVALID_ARG;
  for (int32_t j = 0; j < num_tensors; ++j)
    if (offsets_host[j + 1] <= offsets_host[j]) return DGC_ERR_INVALID_ARG;
  if (offsets_host[num_tensors] > ((int64_t)1 << 31) - 65536) return DGC_ERR_CAPACITY;

  dgc_handle* h = new (std::nothrow) dgc_handle();
  if (!h) return DGC_ERR_CAPACITY;
  try {
    h->cfg = *cfg;
    h->id = g_next_handle_id.fetch_add(1);
    h->num_tensors = num_tensors;
    h->offsets.assign(offsets_host, offsets_host + num_tensors + 1);
    h->n = offsets_host[num_tensors];
    h->warmup.assign(kDefaultWarmup, kDefaultWarmup + 5);
    h->plans.resize(num_tensors);
    h->k.resize(num_tensors);
    h->draws.resize(num_tensors);
    const int64_t tiles = (h->n + kWaveTile - 1) / kWaveTile;
    h->tile_info.resize((size_t)tiles);
    h->tile_thr_init.resize((size_t)tiles);
    int32_t j = 0;
    for (int64_t t = 0; t < tiles; ++t) {
      const int64_t first = t * kWaveTile;
      const int64_t last = first + kWaveTile;  // one past the tile
      while (h->offsets[j + 1] <= first) ++j;
      const bool whole = last <= h->n && last <= h->offsets[j + 1];
      h->tile_info[(size_t)t] = (uint32_t)j | (whole ? 0u : kTileMixed);
      h->tile_thr_init[(size_t)t] = whole ? 0.0f : std::nanf("");
    }
    for (int32_t t = 0; t < num_tensors; ++t) {
      const int64_t t0 = h->offsets[t] / kWaveTile;
      const int64_t t1 = (h->offsets[t + 1] - 1) / kWaveTile;
      const int32_t nb = (int32_t)((t1 - t0) / kEmitTiles + 1);
      for (int64_t f = t0; f <= t1; f += kEmitTiles)
        h->emit_blocks.push_back(EmitBlock{t, (int32_t)f, nb, 0, h->offsets[t], h->offsets[t + 1]});
    }
    // element ranges of the receive side: kMergeEmitBlocks consecutive emit workgroups' parts of one tensor
    for (size_t b = 0; b < h->emit_blocks.size();) {
      const int32_t t = h->emit_blocks[b].tensor;
      size_t e = b;
      while (e < h->emit_blocks.size() && e < b + kMergeEmitBlocks && h->emit_blocks[e].tensor == t) ++e;
      int64_t begin = (int64_t)h->emit_blocks[b].first_tile * kWaveTile;
      int64_t end = (int64_t)(h->emit_blocks[e - 1].first_tile + kEmitTiles) * kWaveTile;
      if (begin < h->offsets[t]) begin = h->offsets[t];
      if (end > h->offsets[t + 1]) end = h->offsets[t + 1];
      h->merge_blocks.push_back(MergeBlock{begin, end, t, 0});
      b = e;
    }
    for (const EmitBlock& eb : h->emit_blocks) {
      int64_t begin = (int64_t)eb.first_tile * kWaveTile;
      int64_t end = (int64_t)(eb.first_tile + kEmitTiles) * kWaveTile;
      if (begin < h->offsets[eb.tensor]) begin = h->offsets[eb.tensor];
      if (end > h->offsets[eb.tensor + 1]) end = h->offsets[eb.tensor + 1];
      h->part_blocks.push_back(MergeBlock{begin, end, eb.tensor, 0});
    }
    h->ws_out_offsets.resize(num_tensors + 1);
    h->wire_first_block.resize(num_tensors + 1);
  } catch (...) {
    delete h;
    return DGC_ERR_CAPACITY;
  }
  build_plan(h);
  build_layout(h);
  *out = h;
  return DGC_OK;
}

static void profile_release(dgc_handle* h);

dgc_status dgc_destroy(dgc_handle* h) {
  if (h) {
    profile_release(h);
    workspace_release_all(h->id);
  }
  delete h;
  return DGC_OK;
}

dgc_status dgc_invalidate_workspace(dgc_handle* h) {
  if (!h) return DGC_ERR_INVALID_ARG;
  workspace_release_all(h->id);
  h->ws = nullptr;
  h->ws_static_valid = h->ws_plan_valid = h->ws_layout_valid = false;
  return DGC_OK;
}

dgc_status dgc_set_scale_override(dgc_handle* h, float scale) {
  if (!h) return DGC_ERR_INVALID_ARG;
  if (scale - scale != 0.0f && scale == scale) return DGC_ERR_INVALID_ARG;  // an infinity
  h->cfg.scale_override = scale;
  return DGC_OK;
}

dgc_status dgc_set_density(dgc_handle* h, double density) {
  if (!h || !valid_density(density)) return DGC_ERR_INVALID_ARG;
  if (density != h->cfg.density) {
    h->cfg.density = density;
    build_plan(h);
  }
  return DGC_OK;
}

dgc_status dgc_set_warmup_schedule(dgc_handle* h, const double* densities_host, int32_t len) {
  if (!h || !densities_host || len < 1) return DGC_ERR_INVALID_ARG;
  for (int32_t i = 0; i < len; ++i)
    if (!valid_density(densities_host[i])) return DGC_ERR_INVALID_ARG;
  h->warmup.assign(densities_host, densities_host + len);
  return DGC_OK;
}

dgc_status dgc_set_warmup_stage_length(dgc_handle* h, int64_t iterations_per_stage) {
  if (!h || iterations_per_stage < 1) return DGC_ERR_INVALID_ARG;
  h->warmup_stage_len = iterations_per_stage;
  return DGC_OK;
}

dgc_status dgc_set_iteration_density(dgc_handle* h, int64_t iteration) {
  if (!h || iteration < 0) return DGC_ERR_INVALID_ARG;
  const size_t last = h->warmup.size() - 1;
  const uint64_t stage = (uint64_t)(iteration / h->warmup_stage_len);
  const size_t i = stage < last ? (size_t)stage : last;
  return dgc_set_density(h, h->warmup[i]);
}

dgc_status dgc_query_plan(const dgc_handle* h, int32_t j, int64_t* k, int64_t* sample_count,
                          int64_t* rank, int64_t* draws) {
  if (!h || j < 0 || j >= h->num_tensors) return DGC_ERR_INVALID_ARG;
  if (k) *k = h->k[j];
  if (sample_count) *sample_count = h->plans[j].count;
  if (rank) *rank = h->plans[j].rank;
  if (draws) *draws = h->draws[j];
  return DGC_OK;
}

dgc_status dgc_workspace_bytes(const dgc_handle* h, size_t* bytes) {
  if (!h || !bytes) return DGC_ERR_INVALID_ARG;
  *bytes = h->lay.total;
  return DGC_OK;
}

dgc_status dgc_workspace_bytes_warmup(const dgc_handle* h, size_t* bytes) {
  if (!h || !bytes) return DGC_ERR_INVALID_ARG;
  *bytes = h->lay.total_staged;
  return DGC_OK;
}

dgc_status dgc_recommended_payload_layout(const dgc_handle* h, double density,
                                          int64_t* out_offsets_host) {
  if (!h || !out_offsets_host || !valid_density(density)) return DGC_ERR_INVALID_ARG;
  int64_t off = 0;
  for (int32_t j = 0; j < h->num_tensors; ++j) {
    out_offsets_host[j] = off;
    const int64_t n = h->offsets[j + 1] - h->offsets[j];
    const int64_t k = topk_count(density, n);
    // A threshold taken at rank r of a sample lets through a Beta(r + 1, s - r) share of the tensor:
    // with r as small as 5 that exceeds 4 k about once in a thousand calls, 8 k practically never.
    int64_t cap = 8 * k > k + 256 ? 8 * k : k + 256;
    if (cap > n) cap = n;
    off += cap;
  }
  out_offsets_host[h->num_tensors] = off;
  if (off >= (int64_t)1 << 31) return DGC_ERR_CAPACITY;
  return DGC_OK;
}

dgc_status dgc_compress(dgc_handle* h, const float* g, float* u, float* v, int32_t* out_idx,
                        float* out_val, const int64_t* out_offsets_host, int32_t* out_counts,
                        float* out_thr, uint64_t iteration, void* workspace,
                        size_t workspace_bytes, void* stream_) {
  if (!h || !g || !u || !v || !out_idx || !out_val || !out_counts) return DGC_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(u, 16) || !aligned(v, 16)) return DGC_ERR_ALIGNMENT;
  if (!aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(out_counts, 4)) return DGC_ERR_ALIGNMENT;
  dgc_status st = check_layout(h, out_offsets_host);
  if (st != DGC_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  st = sync_workspace(h, workspace, workspace_bytes, out_offsets_host, true, stream);
  if (st != DGC_OK) return st;

  const dgc_config& c = h->cfg;
  const bool clip = c.clip_threshold > 0.0f;
  const bool have_override = c.scale_override == c.scale_override;
  DeviceState* state = at<DeviceState>(workspace, h->lay.state);

  hipEvent_t* ev = nullptr;
  if (h->prof_capacity > 0 && h->prof_calls < h->prof_capacity) {
    ev = &h->prof_events[(size_t)h->prof_calls * kProfEvents];
    ++h->prof_calls;
    if (!hip_ok(hipEventRecord(ev[0], stream), "record event")) return DGC_ERR_HIP;
  }

  // paper: Appendix C equation 12 -- the local threshold is N^-1/2 times the global one.
  const double thr_local = clip ? (double)c.clip_threshold / std::sqrt((double)c.num_workers) : 0.0;
  if (clip) {
    if (!hip_ok(launch_norm(g, h->n, at<double>(workspace, h->lay.partials), stream), "launch norm kernel"))
      return DGC_ERR_HIP;
  }
  if (ev && !hip_ok(hipEventRecord(ev[1], stream), "record event")) return DGC_ERR_HIP;
  const float scale_const = have_override ? c.scale_override : 1.0f;

  SelectArgs sa{};
  sa.g = g;
  sa.u = u;
  sa.v = v;
  sa.plans = at<TensorPlan>(workspace, h->lay.plans);
  sa.state = state;
  sa.thr = at<float>(workspace, h->lay.thr);
  sa.out_thr = out_thr;
  sa.tile_thr = at<float>(workspace, h->lay.tile_thr);
  sa.partials = at<double>(workspace, h->lay.partials);
  sa.thr_local = thr_local;
  sa.num_partials = clip ? norm_blocks(h->n) : 0;
  sa.scale_override = c.scale_override;
  sa.momentum = c.momentum;
  sa.scale_const = scale_const;
  sa.scale_from_state = clip ? 1 : 0;
  sa.nesterov = (c.flags & DGC_FLAG_NESTEROV) ? 1 : 0;
  int shift = 0;
  while ((1 << shift) < c.sample_block) ++shift;
  sa.block_shift = shift;
  sa.seed_lo = (uint32_t)(c.seed & 0xFFFFFFFFu);
  sa.seed_hi = (uint32_t)(c.seed >> 32);
  sa.iter_lo = (uint32_t)(iteration & 0xFFFFFFFFu);
  sa.iter_hi = (uint32_t)(iteration >> 32);
  if (!hip_ok(launch_select(sa, h->num_tensors, stream), "launch select kernel")) return DGC_ERR_HIP;
  if (ev && !hip_ok(hipEventRecord(ev[2], stream), "record event")) return DGC_ERR_HIP;

  StreamArgs ta{};
  ta.g = g;
  ta.u = u;
  ta.v = v;
  ta.mask = at<uint16_t>(workspace, h->lay.mask);
  ta.offsets = at<int64_t>(workspace, h->lay.offsets);
  ta.thr = sa.thr;
  ta.tile_info = at<uint32_t>(workspace, h->lay.tile_info);
  ta.tile_thr = sa.tile_thr;
  ta.tile_count = at<uint32_t>(workspace, h->lay.tile_count);
  ta.state = state;
  ta.n = h->n;
  ta.num_tensors = h->num_tensors;
  ta.momentum = c.momentum;
  ta.scale_const = scale_const;
  ta.scale_from_state = sa.scale_from_state;
  ta.nesterov = sa.nesterov;
  // paper: Section 4, warm-up training -- at the densities of the first epochs the masking of u and v
  // is folded into the streaming pass and the selected values wait in staging arrays, if the
  // workspace has them.  (The re-threshold pass drops elements after the streaming pass and
  // expects them untouched in u and v: it keeps the plain pass.)
  const bool factor_masking = (c.flags & DGC_FLAG_NO_FACTOR_MASKING) == 0;
  const bool staged = c.density > kStagedMinDensity && c.refine_alpha <= 0.0f && workspace_bytes >= h->lay.total_staged;
  ta.factor_masking = factor_masking ? 1 : 0;
  const bool sorted = (c.flags & DGC_FLAG_SORTED_OUTPUT) != 0;
  // At the densities the method runs at (Section 4.1: 99.9 % sparsity after the warm-up) a tile holds
  // one or two selected elements: the streaming pass parks them in the tile's slots and masks u and v
  // itself, and the emit pass copies, in index order.
  const bool slotted = !staged && c.density <= kStagedMinDensity;
  if (staged) {
    ta.stage_v = at<float>(workspace, h->lay.stage_v);
    ta.stage_u = (factor_masking && h->layout_may_overflow) ? at<float>(workspace, h->lay.stage_u) : nullptr;
  }
  ta.slotted = slotted ? 1 : 0;
  if (!hip_ok(launch_stream(ta, stream), "launch stream kernel")) return DGC_ERR_HIP;
  if (ev && !hip_ok(hipEventRecord(ev[3], stream), "record event")) return DGC_ERR_HIP;

  // paper: Section 5 -- a tensor that lets through far more elements than wanted gets an exact
  // threshold, computed among the elements that passed
  if (c.refine_alpha > 0.0f) {
    RefineArgs ra{};
    ra.plans = sa.plans;
    ra.v = v;
    ra.mask = ta.mask;
    ra.offsets = ta.offsets;
    ra.out_offsets = at<int64_t>(workspace, h->lay.out_offsets);
    ra.out_idx = out_idx;
    ra.out_val = out_val;
    ra.thr = sa.thr;
    ra.out_thr = out_thr;
    ra.tile_count = ta.tile_count;
    ra.slotted = ta.slotted;
    ra.factor_masking = ta.factor_masking;
    ra.u_out = u;
    ra.v_out = v;
    if (!hip_ok(launch_refine(ra, h->num_tensors, stream), "launch refine kernel"))
      return DGC_ERR_HIP;
  }

  EmitArgs ea{};
  ea.blocks = at<EmitBlock>(workspace, h->lay.emit_blocks);
  ea.tile_count = at<uint32_t>(workspace, h->lay.tile_count);
  ea.u = u;
  ea.v = v;
  ea.mask = ta.mask;
  ea.out_idx = out_idx;
  ea.out_val = out_val;
  ea.offsets = ta.offsets;
  ea.out_offsets = at<int64_t>(workspace, h->lay.out_offsets);
  ea.out_counts = out_counts;
  ea.state = state;
  ea.factor_masking = factor_masking ? 1 : 0;
  ea.stage_v = ta.stage_v;
  ea.stage_u = ta.stage_u;
  ea.slotted = ta.slotted;
  if (!hip_ok(launch_emit(ea, (int32_t)h->emit_blocks.size(), sorted, stream), "launch emit kernel"))
    return DGC_ERR_HIP;
  if (ev && !hip_ok(hipEventRecord(ev[4], stream), "record event")) return DGC_ERR_HIP;
  return DGC_OK;
}

dgc_status dgc_compress_static(dgc_handle* h, const float* g, float* u, float* v, int32_t* out_idx,
                               float* out_val, const int64_t* out_offsets_host, int32_t* out_counts,
                               float* out_thr, uint64_t iteration, void* stream) {
  if (!h) return DGC_ERR_INVALID_ARG;
  if (h->lay.total > kStaticScratchBytes) {
    std::snprintf(g_last_error, sizeof(g_last_error),
                  "dgc_compress_static: this gradient set needs a workspace of %zu bytes, the static array has %zu",
                  h->lay.total, kStaticScratchBytes);
    return DGC_ERR_CAPACITY;
  }
  void* ws = nullptr;
  const dgc_status st = static_scratch(&ws, false);
  if (st != DGC_OK) return st;
  // The array keeps what the last call left in it.  What must start at zero (the state record)
  // is cleared, and every table uploaded again, whenever another handle has used the array since
  // this one did: sync_workspace sees that in the owner registry.
  return dgc_compress(h, g, u, v, out_idx, out_val, out_offsets_host, out_counts, out_thr, iteration, ws,
                      kStaticScratchBytes, stream);
}

static void profile_release(dgc_handle* h) {
  for (hipEvent_t e : h->prof_events) (void)hipEventDestroy(e);
  h->prof_events.clear();
  h->prof_capacity = 0;
  h->prof_calls = 0;
}

dgc_status dgc_profile_enable(dgc_handle* h, int32_t max_calls) {
  if (!h || max_calls < 1 || max_calls > 65536) return DGC_ERR_INVALID_ARG;
  profile_release(h);
  h->prof_events.reserve((size_t)max_calls * kProfEvents);
  for (int32_t i = 0; i < max_calls * kProfEvents; ++i) {
    hipEvent_t e;
    if (!hip_ok(hipEventCreate(&e), "create event")) {
      profile_release(h);
      return DGC_ERR_HIP;
    }
    h->prof_events.push_back(e);
  }
  h->prof_capacity = max_calls;
  return DGC_OK;
}

dgc_status dgc_profile_collect(dgc_handle* h, int32_t* calls, double* norm_ms, double* select_ms,
                               double* stream_ms, double* emit_ms) {
  if (!h || !calls || !norm_ms || !select_ms || !stream_ms || !emit_ms) return DGC_ERR_INVALID_ARG;
  if (h->prof_capacity < 1) return DGC_ERR_STATE;
  *calls = h->prof_calls;
  *norm_ms = *select_ms = *stream_ms = *emit_ms = 0.0;
  for (int32_t i = 0; i < h->prof_calls; ++i) {
    hipEvent_t* ev = &h->prof_events[(size_t)i * kProfEvents];
    if (!hip_ok(hipEventSynchronize(ev[4]), "wait for event")) return DGC_ERR_HIP;
    float a = 0.f, b = 0.f, c = 0.f, d = 0.f;
    if (!hip_ok(hipEventElapsedTime(&a, ev[0], ev[1]), "event time") ||
        !hip_ok(hipEventElapsedTime(&b, ev[1], ev[2]), "event time") ||
        !hip_ok(hipEventElapsedTime(&c, ev[2], ev[3]), "event time") ||
        !hip_ok(hipEventElapsedTime(&d, ev[3], ev[4]), "event time"))
      return DGC_ERR_HIP;
    *norm_ms += a;
    *select_ms += b;
    *stream_ms += c;
    *emit_ms += d;
  }
  h->prof_calls = 0;
  return DGC_OK;
}

dgc_status dgc_profile_disable(dgc_handle* h) {
  if (!h) return DGC_ERR_INVALID_ARG;
  profile_release(h);
  return DGC_OK;
}

dgc_status dgc_profile_stream_ceiling(const float* a, float* b, float* c, int64_t n, int32_t groups_per_cu,
                                      void* stream) {
  if (!a || !b || !c || n < 0 || n >= (int64_t)1 << 31) return DGC_ERR_INVALID_ARG;
  if (groups_per_cu < 0 || groups_per_cu > 16) return DGC_ERR_INVALID_ARG;
  if (!aligned(a, 16) || !aligned(b, 16) || !aligned(c, 16)) return DGC_ERR_ALIGNMENT;
  if (!hip_ok(launch_ceiling(a, b, c, n, groups_per_cu, static_cast<hipStream_t>(stream)), "launch ceiling kernel"))
    return DGC_ERR_HIP;
  return DGC_OK;
}

dgc_status dgc_get_diagnostics(dgc_handle* h, const void* workspace, dgc_diagnostics* out_host,
                               void* stream_) {
  if (!h || !out_host) return DGC_ERR_INVALID_ARG;
  if (!workspace) {  // the static array of dgc_compress_static on the current device
    void* ws = nullptr;
    const dgc_status st = static_scratch(&ws, true);
    if (st != DGC_OK) return st == DGC_ERR_STATE ? DGC_ERR_INVALID_ARG : st;
    workspace = ws;
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  DeviceState s;
  if (!hip_ok(hipMemcpyAsync(&s, static_cast<const char*>(workspace) + h->lay.state, sizeof(s),
                             hipMemcpyDeviceToHost, stream),
              "read diagnostics"))
    return DGC_ERR_HIP;
  if (!hip_ok(hipStreamSynchronize(stream), "synchronize stream")) return DGC_ERR_HIP;
  out_host->norm = s.norm;
  out_host->scale = s.scale;
  out_host->flags = s.flags;
  return DGC_OK;
}

namespace {
enum class ScatterOp { kAccumulate, kClear, kSgd, kReplace };
}

static dgc_status scatter_pairs(dgc_handle* h, float* dense, int64_t n, int32_t num_payloads,
                                const int32_t* const* idx_ptrs_host, const float* const* val_ptrs_host,
                                const int64_t* pair_counts_host, uint32_t* diag_flags_dev, void* stream_,
                                ScatterOp op, float scale) {
  if (!h || !dense || !idx_ptrs_host || !val_ptrs_host || !pair_counts_host) return DGC_ERR_INVALID_ARG;
  if (n < 1 || n >= (int64_t)1 << 31) return DGC_ERR_INVALID_ARG;
  if (num_payloads < 1) return DGC_ERR_INVALID_ARG;
  if (num_payloads > kMaxPayloads) return DGC_ERR_CAPACITY;
  if (!aligned(dense, 4)) return DGC_ERR_ALIGNMENT;
  PairPayloads p{};
  int64_t max_count = 0;
  for (int32_t w = 0; w < num_payloads; ++w) {
    const int64_t c = pair_counts_host[w];
    if (c < 0 || c >= (int64_t)1 << 31) return DGC_ERR_INVALID_ARG;
    if (c > 0 && (!idx_ptrs_host[w] || !val_ptrs_host[w])) return DGC_ERR_INVALID_ARG;
    p.idx[w] = idx_ptrs_host[w];
    p.val[w] = val_ptrs_host[w];
    p.count[w] = c;
    if (c > max_count) max_count = c;
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const bool sgd = op == ScatterOp::kSgd;
  if (h->cfg.flags & DGC_FLAG_DETERMINISTIC_ACCUMULATE) {
    // one launch per worker, in order: within a payload every index is distinct
    for (int32_t w = 0; w < num_payloads; ++w)
      if (!hip_ok(launch_scatter_pairs(dense, n, p, w, 1, p.count[w], sgd ? kScatterPlainSgd : kScatterPlainAdd,
                                       scale, diag_flags_dev, stream),
                  "launch scatter kernel"))
        return DGC_ERR_HIP;
  } else {
    if (!hip_ok(launch_scatter_pairs(dense, n, p, 0, num_payloads, max_count,
                                     sgd ? kScatterAtomicSgd : kScatterAtomicAdd, scale, diag_flags_dev, stream),
                "launch scatter kernel"))
      return DGC_ERR_HIP;
  }
  return DGC_OK;
}

dgc_status dgc_decompress_accumulate(dgc_handle* h, float* dense, int64_t n, int32_t num_payloads,
                                     const int32_t* const* idx_ptrs_host,
                                     const float* const* val_ptrs_host,
                                     const int64_t* pair_counts_host, uint32_t* diag_flags_dev,
                                     void* stream) {
  return scatter_pairs(h, dense, n, num_payloads, idx_ptrs_host, val_ptrs_host, pair_counts_host,
                       diag_flags_dev, stream, ScatterOp::kAccumulate, 0.0f);
}

dgc_status dgc_sparse_sgd_apply(dgc_handle* h, float* theta, int64_t n, float learning_rate,
                                int32_t num_payloads, const int32_t* const* idx_ptrs_host,
                                const float* const* val_ptrs_host, const int64_t* pair_counts_host,
                                uint32_t* diag_flags_dev, void* stream) {
  if (!(learning_rate == learning_rate)) return DGC_ERR_INVALID_ARG;
  return scatter_pairs(h, theta, n, num_payloads, idx_ptrs_host, val_ptrs_host, pair_counts_host,
                       diag_flags_dev, stream, ScatterOp::kSgd, -learning_rate);
}

static dgc_status scatter_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                  const int32_t* const* idx_ptrs_host,
                                  const float* const* val_ptrs_host,
                                  const int32_t* const* count_ptrs_host,
                                  const int64_t* out_offsets_host, void* workspace,
                                  size_t workspace_bytes, void* stream_, ScatterOp op, float scale,
                                  int32_t num_old = 0, const int32_t* const* old_idx_host = nullptr,
                                  const int32_t* const* old_count_host = nullptr) {
  const bool clear = op == ScatterOp::kClear;
  const bool sgd = op == ScatterOp::kSgd;
  const bool replace = op == ScatterOp::kReplace;
  if (num_old < 0 || (num_old > 0 && (!old_idx_host || !old_count_host))) return DGC_ERR_INVALID_ARG;
  if (num_old > kMaxPayloads) return DGC_ERR_CAPACITY;
  RegionPayloads was{};
  for (int32_t w = 0; w < num_old; ++w) {
    if (!old_idx_host[w] || !old_count_host[w]) return DGC_ERR_INVALID_ARG;
    was.idx[w] = old_idx_host[w];
    was.counts[w] = old_count_host[w];
  }
  if (!h || !dense || !idx_ptrs_host || !count_ptrs_host) return DGC_ERR_INVALID_ARG;
  if (!clear && !val_ptrs_host) return DGC_ERR_INVALID_ARG;
  if (num_payloads < 1) return DGC_ERR_INVALID_ARG;
  if (num_payloads > kMaxPayloads) return DGC_ERR_CAPACITY;
  dgc_status st = check_layout(h, out_offsets_host);
  if (st != DGC_OK) return st;
  RegionPayloads p{};
  for (int32_t w = 0; w < num_payloads; ++w) {
    if (!idx_ptrs_host[w] || !count_ptrs_host[w] || (!clear && !val_ptrs_host[w]))
      return DGC_ERR_INVALID_ARG;
    p.idx[w] = idx_ptrs_host[w];
    p.val[w] = clear ? nullptr : val_ptrs_host[w];
    p.counts[w] = count_ptrs_host[w];
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  st = sync_workspace(h, workspace, workspace_bytes, out_offsets_host, false, stream);
  if (st != DGC_OK) return st;
  const int64_t* oo = at<int64_t>(workspace, h->lay.out_offsets);
  const int64_t widest = out_offsets_host[h->num_tensors];  // pairs a payload can hold
  // No atomics at any density, workers in order.  At the densities the method runs at, a
  // workgroup merges the pairs of a range of up to 128 Ki elements in LDS and touches only
  // the elements that occur; at warm-up densities a workgroup keeps one emit part's whole
  // range of `dense` in LDS.
  // Pairs a range of kMergeMaxRange elements can expect (the sampled threshold lets through up to a
  // quarter more than the density on the inputs seen so far): the range kernel wants them, and the
  // previous payloads' indices when it replaces, in its registers and accumulator, and takes a much
  // slower way when they do not fit.  (Replacing an aggregate whose index lists are that long:
  // writing the whole of `dense` once, which needs none of them, is the cheaper way.)
  const int64_t expected_new = (int64_t)std::ceil(1.25 * h->cfg.density * (double)kMergeMaxRange * (double)num_payloads);
  const int64_t expected_old = (replace && num_old > 0) ? h->last_replace_expected : 0;
  const int64_t expected_pairs = expected_new > expected_old ? expected_new : expected_old;
  const bool fits = h->cfg.density <= kMergeMaxDensity && expected_new <= kMergeCapLarge;
  const bool few = fits && expected_old <= kMergeCapLarge;
  if (replace) h->last_replace_expected = fits ? expected_new : (int64_t)kMergeCapLarge + 1;
  const MergeBlock* parts = at<MergeBlock>(workspace, h->lay.part_blocks);
  const int32_t num_parts = (int32_t)h->part_blocks.size();
  void* found = at<char>(workspace, h->lay.part_found);
  if (clear) {
    if (few) {
      // the launch is sized for the pairs the density lets expect (the kernel strides over whatever
      // there is), not for regions that were laid out for a higher density
      int64_t expected = 0;
      for (int32_t j = 0; j < h->num_tensors; ++j) expected += 8 * h->k[j] + 256;
      const int64_t sized_for = expected < widest ? expected : widest;
      if (!hip_ok(launch_scatter_regions(dense, h->n, p, 0, num_payloads, oo, h->num_tensors, sized_for,
                                         kScatterClear, 0.0f, nullptr, stream),
                  "launch scatter kernel"))
        return DGC_ERR_HIP;
    } else if (!hip_ok(launch_clear_parts(dense, p, num_payloads, oo, parts, num_parts, found, stream),
                       "launch clear kernel")) {
      return DGC_ERR_HIP;
    }
  } else if (few) {
    if (!hip_ok(launch_merge_regions(dense, p, num_payloads, replace ? &was : nullptr, num_old, oo,
                                     at<MergeBlock>(workspace, h->lay.merge_blocks), (int32_t)h->merge_blocks.size(),
                                     expected_pairs, sgd, scale, stream),
                "launch merge kernel"))
      return DGC_ERR_HIP;
  } else if (!hip_ok(launch_merge_parts(dense, p, num_payloads, oo, parts, num_parts, found, replace, sgd, scale,
                                        stream),
                     "launch merge kernel")) {
    return DGC_ERR_HIP;
  }
  return DGC_OK;
}

dgc_status dgc_decompress_accumulate_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                             const int32_t* const* idx_ptrs_host,
                                             const float* const* val_ptrs_host,
                                             const int32_t* const* count_ptrs_host,
                                             const int64_t* out_offsets_host, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  return scatter_regions(h, dense, num_payloads, idx_ptrs_host, val_ptrs_host, count_ptrs_host,
                         out_offsets_host, workspace, workspace_bytes, stream, ScatterOp::kAccumulate, 0.0f);
}

dgc_status dgc_decompress_replace_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                          const int32_t* const* idx_ptrs_host,
                                          const float* const* val_ptrs_host,
                                          const int32_t* const* count_ptrs_host, int32_t num_previous,
                                          const int32_t* const* previous_idx_ptrs_host,
                                          const int32_t* const* previous_count_ptrs_host,
                                          const int64_t* out_offsets_host, void* workspace,
                                          size_t workspace_bytes, void* stream) {
  return scatter_regions(h, dense, num_payloads, idx_ptrs_host, val_ptrs_host, count_ptrs_host,
                         out_offsets_host, workspace, workspace_bytes, stream, ScatterOp::kReplace, 0.0f,
                         num_previous, previous_idx_ptrs_host, previous_count_ptrs_host);
}

dgc_status dgc_sparse_sgd_apply_regions(dgc_handle* h, float* theta, float learning_rate,
                                        int32_t num_payloads, const int32_t* const* idx_ptrs_host,
                                        const float* const* val_ptrs_host,
                                        const int32_t* const* count_ptrs_host,
                                        const int64_t* out_offsets_host, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  if (!(learning_rate == learning_rate)) return DGC_ERR_INVALID_ARG;
  return scatter_regions(h, theta, num_payloads, idx_ptrs_host, val_ptrs_host, count_ptrs_host,
                         out_offsets_host, workspace, workspace_bytes, stream, ScatterOp::kSgd, -learning_rate);
}

dgc_status dgc_dense_clear_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                   const int32_t* const* idx_ptrs_host,
                                   const int32_t* const* count_ptrs_host,
                                   const int64_t* out_offsets_host, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return scatter_regions(h, dense, num_payloads, idx_ptrs_host, nullptr, count_ptrs_host,
                         out_offsets_host, workspace, workspace_bytes, stream, ScatterOp::kClear, 0.0f);
}

dgc_status dgc_encode_max_entries(const dgc_handle* h, int64_t pairs, int64_t* entries) {
  if (!h || !entries || pairs < 0) return DGC_ERR_INVALID_ARG;
  // every filler entry accounts for 65536 positions of the set
  *entries = pairs + (h->n >> 16);
  return DGC_OK;
}

dgc_status dgc_encode(dgc_handle* h, const int32_t* idx, const float* val, const int32_t* counts,
                      const int64_t* out_offsets_host, uint16_t* runs, float* vals, int64_t entry_capacity,
                      int32_t* num_entries, void* workspace, size_t workspace_bytes, void* stream_) {
  if (!h || !idx || !val || !counts || !runs || !vals || !num_entries) return DGC_ERR_INVALID_ARG;
  if (entry_capacity < 0) return DGC_ERR_INVALID_ARG;
  if (!aligned(idx, 4) || !aligned(val, 4) || !aligned(counts, 4) || !aligned(runs, 2) || !aligned(vals, 4) ||
      !aligned(num_entries, 4))
    return DGC_ERR_ALIGNMENT;
  dgc_status st = check_layout(h, out_offsets_host);
  if (st != DGC_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  st = sync_workspace(h, workspace, workspace_bytes, out_offsets_host, false, stream);
  if (st != DGC_OK) return st;
  int64_t widest = 0;
  for (int32_t j = 0; j < h->num_tensors; ++j)
    if (out_offsets_host[j + 1] - out_offsets_host[j] > widest) widest = out_offsets_host[j + 1] - out_offsets_host[j];
  const uint32_t total_blocks = h->wire_first_block[(size_t)h->num_tensors];
  if ((size_t)total_blocks > h->wire_slots) return DGC_ERR_CAPACITY;
  EncodeArgs ea{};
  ea.idx = idx;
  ea.val = val;
  ea.counts = counts;
  ea.out_offsets = at<int64_t>(workspace, h->lay.out_offsets);
  ea.first_block = at<uint32_t>(workspace, h->lay.wire_first_block);
  ea.sums = at<uint32_t>(workspace, h->lay.wire_sums);
  ea.runs = runs;
  ea.vals = vals;
  ea.num_entries = num_entries;
  ea.state = at<DeviceState>(workspace, h->lay.state);
  ea.capacity = entry_capacity;
  ea.num_tensors = h->num_tensors;
  if (!hip_ok(launch_encode(ea, widest, (int32_t)total_blocks, stream), "launch encode kernels")) return DGC_ERR_HIP;
  return DGC_OK;
}

dgc_status dgc_decode_accumulate(dgc_handle* h, float* dense, int64_t n, int32_t num_payloads,
                                 const uint16_t* const* runs_ptrs_host, const float* const* vals_ptrs_host,
                                 const int64_t* entry_counts_host, uint32_t* diag_flags_dev, void* workspace,
                                 size_t workspace_bytes, void* stream_) {
  if (!h || !dense || !runs_ptrs_host || !vals_ptrs_host || !entry_counts_host) return DGC_ERR_INVALID_ARG;
  if (n < 1 || n >= (int64_t)1 << 31) return DGC_ERR_INVALID_ARG;
  if (num_payloads < 1) return DGC_ERR_INVALID_ARG;
  if (num_payloads > kMaxPayloads) return DGC_ERR_CAPACITY;
  if (!aligned(dense, 4)) return DGC_ERR_ALIGNMENT;
  DecodeArgs da{};
  int64_t slots = 0;
  for (int32_t w = 0; w < num_payloads; ++w) {
    const int64_t c = entry_counts_host[w];
    if (c < 0 || c >= (int64_t)1 << 31) return DGC_ERR_INVALID_ARG;
    if (c > 0 && (!runs_ptrs_host[w] || !vals_ptrs_host[w])) return DGC_ERR_INVALID_ARG;
    if (c > 0 && (!aligned(runs_ptrs_host[w], 2) || !aligned(vals_ptrs_host[w], 4))) return DGC_ERR_ALIGNMENT;
    da.runs[w] = runs_ptrs_host[w];
    da.vals[w] = vals_ptrs_host[w];
    da.count[w] = c;
    da.seg.begin[w] = (int32_t)slots;
    slots += (c + kWireChunk - 1) / kWireChunk;
    if (slots > (int64_t)h->wire_slots) return DGC_ERR_CAPACITY;
  }
  da.seg.begin[num_payloads] = (int32_t)slots;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  dgc_status st = sync_workspace(h, workspace, workspace_bytes, nullptr, false, stream);
  if (st != DGC_OK) return st;
  da.sums = at<uint32_t>(workspace, h->lay.wire_sums);
  da.dense = dense;
  da.n = n;
  da.diag_flags = diag_flags_dev;
  if (h->cfg.flags & DGC_FLAG_DETERMINISTIC_ACCUMULATE) {
    // one payload after the other: inside a payload every position is distinct
    for (int32_t w = 0; w < num_payloads; ++w)
      if (!hip_ok(launch_decode(da, w, 1, false, stream), "launch decode kernels")) return DGC_ERR_HIP;
  } else {
    if (!hip_ok(launch_decode(da, 0, num_payloads, true, stream), "launch decode kernels")) return DGC_ERR_HIP;
  }
  return DGC_OK;
}

}  // extern "C"
