// Shared between the host side of libdgc and its kernels: workspace layout,
// kernel argument blocks and launch geometry.  Nothing here is visible through
// the C ABI.
#ifndef DGC_INTERNAL_H_
#define DGC_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dgc.h"

namespace dgc {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- launch geometry -------------------------------------------------------
// Streaming pass: one wavefront owns a contiguous run of kWaveTile elements and
// reads it as kStreamUnroll rounds of one float4 per lane (64 lanes x 16 B =
// 1 KiB per round, fully coalesced).
#ifndef DGC_STREAM_UNROLL
#define DGC_STREAM_UNROLL 4
#endif
constexpr int kStreamUnroll = DGC_STREAM_UNROLL;
constexpr int kWaveTile = 64 * 4 * kStreamUnroll;  // elements per wavefront
constexpr int kStreamThreads = 128;                 // 2 wavefronts per workgroup
constexpr int kStreamWaves = kStreamThreads / 64;
// Workgroups of the streaming pass a compute unit holds at a time.  The pass is faster with few
// wavefronts in flight than with the 32 a compute unit could hold (six per compute unit move 5 %
// more bytes per second than 32: fewer streams for the memory side to interleave), so every
// launch asks for as much LDS as leaves room for this many workgroups in a compute unit's 160 KB.
constexpr int kStreamResidentGroups = 3;
constexpr int kStreamGroupsAfterNorm = 6;  // with clipping on: see launch_stream
constexpr size_t kLdsPerComputeUnit = (size_t)160 * 1024;
// Tile table: one int32 per wave tile = index of the tensor that holds the tile's
// first element, with the top bit set when the tile is not wholly inside one
// tensor or is the ragged last tile (such tiles look up every element's tensor).
constexpr uint32_t kTileMixed = 0x80000000u;

// Emit pass: a workgroup takes kEmitTiles consecutive wave tiles of one tensor.
constexpr int kEmitThreads = 256;
constexpr int kEmitElements = 32768;                  // elements per workgroup
constexpr int kEmitTiles = kEmitElements / kWaveTile;
static_assert(kEmitTiles % (kEmitThreads / 64) == 0, "tiles are dealt round-robin to wavefronts");
constexpr int kEmitList = 4096;                       // elements listed in LDS at a time
// Slots: at the densities the method runs at, a tile of 1024 elements holds one or two selected
// elements.  The streaming pass parks up to kSlotsPerTile of them in a record (kSlotsPerTile
// indices, their v', their u', padding) that it writes in place of the tile's mask words, and
// masks u and v itself, so that the emit pass neither decodes mask words nor goes back to u
// and v for such a tile.  One thread of the emit workgroup per slot of its part.
constexpr int kSlotsPerTile = 8;
constexpr int kSlotRecord = 32;  // 32-bit words per tile: the 128 bytes of the tile's 64 mask words
// Per-tile count of the slotted pass: the top bit says that the tile's line holds mask words although
// the tile lies wholly inside one tensor (it selected more elements than a record holds).
constexpr uint32_t kTileCountHasMask = 0x80000000u;
constexpr uint32_t kTileCountMask = 0x7FFFFFFFu;
static_assert(3 * kSlotsPerTile <= kSlotRecord, "index, v' and u' of every slot");
constexpr int kEmitSlotThreads = 128;  // emit pass over records: two slots per thread
static_assert(kEmitTiles * kSlotsPerTile == 2 * kEmitSlotThreads, "two slots of the workgroup's tiles per emit thread");
constexpr int kRefineThreads = 1024;                  // the re-threshold pass: one workgroup per tensor

// Receive side: pairs of one payload handled by one workgroup (kFlatPer per thread) and
// tensors whose counts a workgroup stages in LDS at a time.
constexpr int kFlatThreads = 256;
constexpr int kFlatPer = 4;
constexpr int kFlatChunk = kFlatThreads * kFlatPer;
constexpr int kFlatTensors = 1024;

// Receive side without atomics: a workgroup owns a range of one tensor's elements (a
// whole number of emit workgroups' parts, which follow each other in index order in
// every payload's region), finds the pairs of every payload that fall into it by search,
// and adds them up in LDS.
constexpr int kMergeMaxThreads = 1024;   // 512 threads when there are at most eight payloads
constexpr int kMergeMaxRange = 131072;   // elements per workgroup at most (one bitmap bit each)
constexpr int kMergeEmitBlocks = kMergeMaxRange / kEmitElements;  // emit workgroups' parts per range
// pairs of a range a workgroup takes into registers and its LDS accumulator (512 and 1024 threads);
// a range with more takes a slower way through the same kernel
constexpr int kMergeCapSmall = 4096;
constexpr int kMergeCapLarge = 6144;
static_assert((kMergeMaxRange / 128) % kMergeMaxThreads == 0, "dealt evenly to threads");

// Receive side at warm-up densities: a workgroup owns one emit workgroup's part and keeps
// the whole range of the dense vector in LDS.
constexpr int kPartThreads = 1024;
constexpr int kPartPer = 4;  // pairs a thread holds per round (8: 5 to 15 % slower at every warm-up density; 2: slower at 25 %)
constexpr int kPartRound = kPartThreads * kPartPer;
constexpr int kPartClearThreads = 256;
static_assert(kEmitElements <= 65536 && kEmitElements % kPartThreads == 0 &&
                  (kEmitElements / 32) % kPartClearThreads == 0,
              "dealt evenly");

// Wire format (32-bit values + 16-bit zero-run lengths): pairs or entries handled by one
// workgroup, kWirePerThread consecutive ones per thread.
constexpr int kWireThreads = 256;
constexpr int kWirePerThread = 16;
constexpr int kWireChunk = kWireThreads * kWirePerThread;
constexpr int kScanThreads = 1024;

// Threshold selection: one workgroup per tensor.
constexpr int kSelectThreads = 1024;
constexpr int kSelectRegKeys = 32;    // candidate keys a thread keeps in registers (32 * 1024 in all)
constexpr int kSelectDirect = 256;    // a bin with at most this many members is ranked directly
constexpr int kSelectBins = 2048;     // 11-bit digits
constexpr int kSelectFloorRounds = 8; // ranks below 16 * this take the short cut over the threads' largest keys
constexpr int kSelectInFlight = 8;    // candidates each thread gathers before using any

// Clipping norm: a fixed number of partial sums keeps the result reproducible.
constexpr int kNormThreads = 256;
constexpr int kNormMaxBlocks = 512;

constexpr int kMaxPayloads = 64;
static_assert(kMaxPayloads <= 32768, "a payload's number is packed above a 16-bit index");

// ---- device-resident state (start of the workspace) ------------------------
struct DeviceState {
  double norm;           // L2 norm of g (clipping on)
  float scale;           // factor applied to g
  uint32_t flags;        // DGC_DIAG_*
  uint32_t pad[4];
};

// Per-tensor selection plan (host arithmetic, uploaded when the density changes).
struct TensorPlan {
  int64_t offset;   // first element of the tensor in the flat buffers
  int64_t n;        // elements
  int32_t count;    // candidates: n (whole tensor) or draws * block
  int32_t rank;     // 0-based descending rank that becomes the threshold
  uint32_t nblocks; // aligned sample blocks in the tensor (sampled mode)
  int32_t exact;    // 1: candidates are elements 0..n-1
  int32_t k;             // clamp(ceil(d n), 1, n)
  int32_t refine_limit;  // floor(refine_alpha * k): more passes than this trigger the re-threshold
};

struct WorkspaceLayout {
  size_t state, partials, offsets, out_offsets, plans, thr, tile_info, tile_thr, emit_blocks,
      tile_count, merge_blocks, part_blocks, part_found, wire_first_block, wire_sums, mask, total,
      stage_v, stage_u, total_staged;  // staging arrays lie behind `total`: a workspace may end before them
};

struct SelectArgs {
  const float* g;
  const float* u;
  const float* v;
  const TensorPlan* plans;
  DeviceState* state;
  float* thr;
  float* out_thr;       // may be null
  float* tile_thr;      // device, one word per wave tile: the threshold of every tile that lies
                        // wholly inside one tensor; the others hold a NaN put there once by the host
  const double* partials;  // partial sums of the squared norm (clipping on)
  double thr_local;        // thr_G / sqrt(N)
  int32_t num_partials;
  float scale_override;    // NaN: unused
  float momentum;
  float scale_const;
  int32_t scale_from_state;  // 1: clipping is on; the scale comes from `partials` and is filed in `state`
  int32_t nesterov;
  int32_t block_shift;  // log2(sample_block)
  uint32_t seed_lo, seed_hi, iter_lo, iter_hi;
};

struct StreamArgs {
  const float* g;
  float* u;
  float* v;
  uint16_t* mask;              // device, 64 words per wave tile
  const int64_t* offsets;      // device, T + 1
  const float* thr;            // device, T
  const uint32_t* tile_info;   // device, ceil(n / kWaveTile), see kTileMixed
  const float* tile_thr;       // device, ceil(n / kWaveTile), see SelectArgs
  uint32_t* tile_count;        // device, ceil(n / kWaveTile): mask bits set in every tile
  const DeviceState* state;
  int64_t n;
  int32_t num_tensors;
  float momentum;
  float scale_const;
  int32_t scale_from_state;
  int32_t nesterov;
  // staged pass (warm-up densities): selected v' (and u') of every whole tile, masking of u, v in the pass
  float* stage_v;              // device, n floats, or null: plain pass
  float* stage_u;              // device, n floats, or null: no region can overflow, or no factor masking
  int32_t factor_masking;
  int32_t slotted;             // slotted pass (densities up to 0.5 %): records in place of mask words
};

struct EmitBlock {
  int32_t tensor;
  int32_t first_tile;     // first wave tile of the workgroup's run inside that tensor
  int32_t tensor_blocks;  // workgroups that share this tensor
  int32_t pad;
  int64_t lo, hi;         // the tensor's elements [lo, hi): here, so that no workgroup waits for a second table
};

struct RefineArgs {
  const TensorPlan* plans;
  const float* v;              // pre-mask v' as left by the streaming pass
  uint16_t* mask;
  const int64_t* offsets;
  const int64_t* out_offsets;  // payload regions: free until the emit pass, used as scratch
  int32_t* out_idx;
  float* out_val;
  float* thr;
  float* out_thr;              // may be null
  uint32_t* tile_count;        // kept in step with the mask bits the pass clears
  int32_t slotted;             // the streaming pass was a slotted one: records in place of some tiles' mask words
  int32_t factor_masking;
  float* u_out;                // u and v, to put back what is dropped from a record
  float* v_out;
};

struct EmitArgs {
  const EmitBlock* blocks;     // device, one entry per workgroup
  float* u;
  float* v;
  const uint16_t* mask;
  int32_t* out_idx;
  float* out_val;
  const int64_t* offsets;      // device, T + 1
  const int64_t* out_offsets;  // device, T + 1
  int32_t* out_counts;         // device, T
  DeviceState* state;
  int32_t factor_masking;
  const uint32_t* tile_count;  // mask bits per tile, left by the streaming pass
  const float* stage_v;        // as in StreamArgs; null: the streaming pass was a plain one
  const float* stage_u;
  int32_t slotted;             // as in StreamArgs
};

struct MergeBlock {
  int64_t begin;   // first element (flat index) of the range
  int64_t end;     // one past its last element; the range lies inside one tensor
  int32_t tensor;
  int32_t pad;
};

struct PairPayloads {
  const int32_t* idx[kMaxPayloads];
  const float* val[kMaxPayloads];
  int64_t count[kMaxPayloads];
};

struct RegionPayloads {
  const int32_t* idx[kMaxPayloads];
  const float* val[kMaxPayloads];
  const int32_t* counts[kMaxPayloads];
};

// Encoder: regions in, entries out.
struct EncodeArgs {
  const int32_t* idx;            // region layout, ascending inside every region
  const float* val;
  const int32_t* counts;         // device, T
  const int64_t* out_offsets;    // device, T + 1
  const uint32_t* first_block;   // device, T + 1: first workgroup slot of every tensor
  uint32_t* sums;                // device, one word per workgroup slot
  uint16_t* runs;
  float* vals;
  int32_t* num_entries;          // device
  DeviceState* state;
  int64_t capacity;              // entries that fit in runs / vals
  int32_t num_tensors;
};

// Segments of the block-sum array handed to the scan kernel: segment s is
// [begin[s], begin[s + 1]).
struct ScanSegments {
  int32_t begin[kMaxPayloads + 1];
};

struct DecodeArgs {
  const uint16_t* runs[kMaxPayloads];
  const float* vals[kMaxPayloads];
  int64_t count[kMaxPayloads];   // entries
  ScanSegments seg;              // workgroup slots of every payload in `sums`
  uint32_t* sums;
  float* dense;
  int64_t n;
  uint32_t* diag_flags;          // may be null
};

enum ScatterMode : int32_t {
  kScatterAtomicAdd = 0,
  kScatterPlainAdd = 1,
  kScatterClear = 2,
  kScatterAtomicSgd = 3,  // target += scale * value, scale = -learning rate
  kScatterPlainSgd = 4
};

// ---- launchers (dgc_compress.hip, dgc_receive.hip, dgc_wire.hip) --------------
hipError_t launch_clear_words(uint32_t* p, size_t words, hipStream_t stream);  // p[0 .. words) <- 0
int32_t norm_blocks(int64_t n);  // partial sums launch_norm leaves
hipError_t launch_norm(const float* g, int64_t n, double* partials, hipStream_t stream);
hipError_t launch_select(const SelectArgs& a, int32_t num_tensors, hipStream_t stream);
hipError_t launch_stream(const StreamArgs& a, hipStream_t stream);
hipError_t launch_ceiling(const float* a, float* b, float* c, int64_t n, int groups, hipStream_t stream);
hipError_t launch_refine(const RefineArgs& a, int32_t num_tensors, hipStream_t stream);
hipError_t launch_emit(const EmitArgs& a, int32_t num_blocks, bool sorted, hipStream_t stream);
hipError_t launch_scatter_pairs(float* dense, int64_t n, const PairPayloads& p, int32_t first,
                                int32_t num, int64_t max_count, ScatterMode mode, float scale,
                                uint32_t* diag_flags, hipStream_t stream);
hipError_t launch_scatter_regions(float* dense, int64_t n, const RegionPayloads& p, int32_t first,
                                  int32_t num, const int64_t* out_offsets_dev, int32_t num_tensors,
                                  int64_t total_capacity, ScatterMode mode, float scale,
                                  uint32_t* diag_flags, hipStream_t stream);

hipError_t launch_merge_regions(float* dense, const RegionPayloads& p, int32_t num, const RegionPayloads* old,
                                int32_t num_old, const int64_t* out_offsets_dev, const MergeBlock* blocks,
                                int32_t num_blocks, int64_t expected_pairs, bool scaled, float scale,
                                hipStream_t stream);
hipError_t launch_merge_parts(float* dense, const RegionPayloads& p, int32_t num, const int64_t* out_offsets_dev,
                              const MergeBlock* parts, int32_t num_parts, void* found, bool replace, bool scaled,
                              float scale, hipStream_t stream);
hipError_t launch_clear_parts(float* dense, const RegionPayloads& p, int32_t num, const int64_t* out_offsets_dev,
                              const MergeBlock* parts, int32_t num_parts, void* found, hipStream_t stream);
hipError_t launch_encode(const EncodeArgs& a, int64_t widest_region, int32_t total_blocks, hipStream_t stream);
hipError_t launch_decode(const DecodeArgs& a, int32_t first, int32_t num, bool atomic, hipStream_t stream);

}  // namespace dgc
#endif  // DGC_INTERNAL_H_
