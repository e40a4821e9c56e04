// HIP kernels of the wire format of the DGC payload for gfx950 (wave64, CDNA4): 32-bit
// values with 16-bit run lengths of zeros, both directions.

#include "dgc_internal.h"

namespace dgc {
namespace {

// ---------------------------------------------------------------------------
// Wire format (paper: Section 3.1 -- encode() packs the 32-bit nonzero values and
// 16-bit run lengths of zeros; footnote of Table 3)
// ---------------------------------------------------------------------------
// An entry (run, value) stands for `run` zeros followed by `value`, in the order of the
// flat index.  Sixteen bits hold a run of at most 65535, so a longer gap is bridged by
// entries (65535, 0.0f), each of which covers 65536 positions.  A pair whose
// predecessor in the whole set leaves `gap` zeros before it therefore takes
// 1 + (gap >> 16) entries, the last of them (gap & 0xFFFF, value).  Trailing zeros are
// not encoded.  Encoding needs every tensor's region in ascending index order
// (DGC_FLAG_SORTED_OUTPUT); regions follow each other in tensor order, which is index
// order.  Both directions are a prefix sum: three launches each (block sums, scan of
// the block sums, write).

// Exclusive prefix sum of `x` over the workgroup (kWireThreads threads); `total` gets the sum.
__device__ __forceinline__ uint32_t wire_block_scan(uint32_t x, uint32_t* wave_sums, uint32_t& total) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint32_t incl = x;
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(incl, d);
    if (lane >= d) incl += t;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  uint32_t before = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < kWireThreads / 64; ++w) {
    const uint32_t t = wave_sums[w];
    if (w < wave) before += t;
    total += t;
  }
  __syncthreads();
  return before + incl - x;
}

// Index of the last pair of the nearest non-empty region before tensor j, or -1.
// Called by one whole wavefront; every lane returns the same value.
__device__ __forceinline__ int32_t last_index_before(const EncodeArgs& a, int j) {
  const int lane = threadIdx.x & 63;
  for (int base = j - 1; base >= 0; base -= 64) {
    const int jj = base - lane;
    int64_t cnt = 0, region = 0;
    if (jj >= 0) {
      region = a.out_offsets[jj];
      const int64_t cap = a.out_offsets[jj + 1] - region;
      cnt = a.counts[jj];
      if (cnt > cap) cnt = cap;
    }
    const unsigned long long have = __ballot(cnt > 0);
    if (have) {
      const int src = __ffsll((long long)have) - 1;  // lowest lane = nearest tensor
      int32_t last = 0;
      if (lane == src) last = a.idx[region + cnt - 1];
      return __shfl(last, src);
    }
  }
  return -1;
}

// PASS 0: entries needed by the workgroup's pairs.  PASS 1: write them.
// grid = (chunks of the widest region, tensors)
template <int PASS>
__global__ __launch_bounds__(kWireThreads) void encode_kernel(EncodeArgs a) {
  __shared__ uint32_t wave_sums[kWireThreads / 64];
  __shared__ int32_t region_prev;
  const int j = blockIdx.y;
  const uint32_t slot0 = a.first_block[j];
  const uint32_t slots = a.first_block[j + 1] - slot0;
  if (blockIdx.x >= slots) return;  // beyond this tensor's region
  const int64_t region = a.out_offsets[j];
  const int64_t cap = a.out_offsets[j + 1] - region;
  int64_t count = a.counts[j];
  if (count > cap) count = cap;
  const int64_t begin = (int64_t)blockIdx.x * kWireChunk;
  if (begin >= count) {
    if (PASS == 0 && threadIdx.x == 0) a.sums[slot0 + blockIdx.x] = 0;
    return;
  }
  if (blockIdx.x == 0) {
    if (threadIdx.x < 64) {
      const int32_t prev = last_index_before(a, j);
      if (threadIdx.x == 0) region_prev = prev;
    }
    __syncthreads();
  }
  const int32_t* __restrict__ idx = a.idx + region;
  const int64_t p0 = begin + (int64_t)threadIdx.x * kWirePerThread;
  int32_t mine[kWirePerThread];
  int32_t prev = -1;
  if (p0 < count) prev = p0 > 0 ? idx[p0 - 1] : region_prev;
#pragma unroll
  for (int k = 0; k < kWirePerThread; ++k) mine[k] = p0 + k < count ? idx[p0 + k] : 0;
  uint32_t need = 0;
  bool unsorted = false;
  {
    int32_t q = prev;
#pragma unroll
    for (int k = 0; k < kWirePerThread; ++k) {
      if (p0 + k < count) {
        int32_t gap = mine[k] - q - 1;
        if (gap < 0) {  // not ascending: flagged, encoded as if adjacent
          gap = 0;
          unsorted = true;
        }
        need += 1u + ((uint32_t)gap >> 16);
        q = mine[k];
      }
    }
  }
  uint32_t total;
  const uint32_t excl = wire_block_scan(need, wave_sums, total);
  if (PASS == 0) {
    if (threadIdx.x == 0) a.sums[slot0 + blockIdx.x] = total;
    if (unsorted) atomicOr(&a.state->flags, (uint32_t)DGC_DIAG_UNSORTED);
    return;
  }
  const float* __restrict__ val = a.val + region;
  int64_t pos = (int64_t)a.sums[slot0 + blockIdx.x] + excl;  // sums hold the exclusive scan by now
  bool overflow = false;
  int32_t q = prev;
#pragma unroll 1
  for (int k = 0; k < kWirePerThread; ++k) {
    if (p0 + k >= count) break;
    int32_t gap = mine[k] - q - 1;
    if (gap < 0) gap = 0;
    for (uint32_t f = (uint32_t)gap >> 16; f > 0; --f) {
      if (pos < a.capacity) {
        a.runs[pos] = 0xFFFFu;
        a.vals[pos] = 0.0f;
      } else {
        overflow = true;
      }
      ++pos;
    }
    if (pos < a.capacity) {
      a.runs[pos] = (uint16_t)((uint32_t)gap & 0xFFFFu);
      a.vals[pos] = val[p0 + k];
    } else {
      overflow = true;
    }
    ++pos;
    q = mine[k];
  }
  if (overflow) atomicOr(&a.state->flags, (uint32_t)DGC_DIAG_OVERFLOW);
}

// In-place exclusive prefix sum of every segment of `sums`; one workgroup per segment.
// `total_out` (may be null) receives the sum of segment 0.
__global__ __launch_bounds__(kScanThreads) void scan_kernel(uint32_t* sums, ScanSegments seg, int32_t* total_out) {
  __shared__ uint32_t wave_sums[kScanThreads / 64];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int32_t begin = seg.begin[blockIdx.x];
  const int32_t end = seg.begin[blockIdx.x + 1];
  uint32_t carry = 0;
  for (int32_t base = begin; base < end; base += kScanThreads) {
    const int32_t i = base + threadIdx.x;
    const uint32_t x = i < end ? sums[i] : 0u;
    uint32_t incl = x;
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t t = __shfl_up(incl, d);
      if (lane >= d) incl += t;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
      const uint32_t t = wave_sums[w];
      if (w < wave) before += t;
      total += t;
    }
    if (i < end) sums[i] = carry + before + incl - x;
    carry += total;
    __syncthreads();
  }
  if (total_out && blockIdx.x == 0 && threadIdx.x == 0) *total_out = (int32_t)carry;
}

// PASS 0: positions covered by the workgroup's entries (run + 1 each).
// PASS 1: dense[position] += value.  grid = (chunks, payloads)
template <int PASS, bool ATOMIC>
__global__ __launch_bounds__(kWireThreads) void decode_kernel(DecodeArgs a, int32_t first) {
  __shared__ uint32_t wave_sums[kWireThreads / 64];
  const int w = first + blockIdx.y;
  const int64_t count = a.count[w];
  const int64_t begin = (int64_t)blockIdx.x * kWireChunk;
  if (begin >= count) return;
  const uint16_t* __restrict__ runs = a.runs[w];
  const int64_t e0 = begin + (int64_t)threadIdx.x * kWirePerThread;
  uint32_t run[kWirePerThread];
  uint32_t span = 0;
#pragma unroll
  for (int k = 0; k < kWirePerThread; ++k) {
    run[k] = e0 + k < count ? (uint32_t)runs[e0 + k] : 0u;
    if (e0 + k < count) span += run[k] + 1u;
  }
  uint32_t total;
  const uint32_t excl = wire_block_scan(span, wave_sums, total);
  const int32_t slot = a.seg.begin[w] + (int32_t)blockIdx.x;
  if (PASS == 0) {
    if (threadIdx.x == 0) a.sums[slot] = total;
    return;
  }
  const float* __restrict__ vals = a.vals[w];
  int64_t pos = (int64_t)a.sums[slot] + excl;
  bool bad = false;
#pragma unroll
  for (int k = 0; k < kWirePerThread; ++k) {
    if (e0 + k < count) {
      pos += run[k];
      const float x = vals[e0 + k];
      if (pos < a.n) {
        if (ATOMIC) unsafeAtomicAdd(a.dense + pos, x);
        else a.dense[pos] = a.dense[pos] + x;
      } else {
        bad = true;
      }
      ++pos;
    }
  }
  if (bad && a.diag_flags) atomicOr(a.diag_flags, (uint32_t)DGC_DIAG_BAD_INDEX);
}

}  // namespace

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
hipError_t launch_encode(const EncodeArgs& a, int64_t widest_region, int32_t total_blocks, hipStream_t stream) {
  if (widest_region <= 0 || total_blocks <= 0) {  // nothing can have been emitted
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, a.sums, ScanSegments{}, a.num_entries);
    return hipGetLastError();
  }
  const int64_t chunks = ceil_div(widest_region, kWireChunk);
  if (chunks > 0x7FFFFFFF || a.num_tensors > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)chunks, (unsigned)a.num_tensors);
  hipLaunchKernelGGL(encode_kernel<0>, grid, dim3(kWireThreads), 0, stream, a);
  ScanSegments seg{};
  seg.begin[0] = 0;
  seg.begin[1] = total_blocks;
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, a.sums, seg, a.num_entries);
  hipLaunchKernelGGL(encode_kernel<1>, grid, dim3(kWireThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_decode(const DecodeArgs& a, int32_t first, int32_t num, bool atomic, hipStream_t stream) {
  int64_t most = 0;
  for (int32_t w = first; w < first + num; ++w)
    if (a.count[w] > most) most = a.count[w];
  if (num <= 0 || most <= 0) return hipSuccess;
  const dim3 grid((unsigned)ceil_div(most, kWireChunk), (unsigned)num);
  ScanSegments seg{};
  for (int32_t w = 0; w <= num; ++w) seg.begin[w] = a.seg.begin[first + w];
  hipLaunchKernelGGL((decode_kernel<0, true>), grid, dim3(kWireThreads), 0, stream, a, first);
  hipLaunchKernelGGL(scan_kernel, dim3((unsigned)num), dim3(kScanThreads), 0, stream, a.sums, seg,
                     (int32_t*)nullptr);
  if (atomic)
    hipLaunchKernelGGL((decode_kernel<1, true>), grid, dim3(kWireThreads), 0, stream, a, first);
  else
    hipLaunchKernelGGL((decode_kernel<1, false>), grid, dim3(kWireThreads), 0, stream, a, first);
  return hipGetLastError();
}

}  // namespace dgc
