// HIP kernels of the receive side of the DGC hot path for gfx950 (wave64, CDNA4): the sum
// of N workers' sparse payloads into one dense vector, without float atomics on the paths
// that take payloads as dgc_compress writes them.

#include "dgc_internal.h"

namespace dgc {
namespace {

// ---------------------------------------------------------------------------
// Receive side (paper: the sum in Algorithm 3's all-reduce line)
// ---------------------------------------------------------------------------
// `scale` multiplies the value first in the two SGD modes (it is -learning rate there:
// theta - lr*x and theta + (-lr)*x round identically) and is ignored otherwise.
__device__ __forceinline__ void scatter_one(float* dense, int64_t n, int32_t i, float x, float scale,
                                            ScatterMode mode, uint32_t* diag_flags) {
  if (i < 0 || (int64_t)i >= n) {
    if (diag_flags) atomicOr(diag_flags, (uint32_t)DGC_DIAG_BAD_INDEX);
    return;
  }
  if (mode == kScatterAtomicSgd || mode == kScatterPlainSgd) x = scale * x;
  if (mode == kScatterAtomicAdd || mode == kScatterAtomicSgd) {
    unsafeAtomicAdd(dense + i, x);  // hardware float add at the L2 / memory side
  } else if (mode == kScatterPlainAdd || mode == kScatterPlainSgd) {
    dense[i] = dense[i] + x;
  } else {
    dense[i] = 0.0f;
  }
}

// grid = (chunks, payloads)
__global__ __launch_bounds__(256) void scatter_pairs_kernel(float* dense, int64_t n, PairPayloads p,
                                                            int32_t first, ScatterMode mode,
                                                            float scale, uint32_t* diag_flags) {
  const int w = first + blockIdx.y;
  const int64_t count = p.count[w];
  const int32_t* __restrict__ idx = p.idx[w];
  const float* __restrict__ val = p.val[w];
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < count; q += stride)
    scatter_one(dense, n, idx[q], mode == kScatterClear ? 0.0f : val[q], scale, mode, diag_flags);
}

// Payloads in the per-tensor region layout written by the emit pass.
// grid = (workgroups per payload, payloads).  The pairs of a payload are numbered
// through all its regions (tensor by tensor, only the filled part of each region), and a
// workgroup takes chunks of kFlatChunk consecutive numbers, grid-strided until the pairs
// run out, so that every thread that runs has a pair to move however unevenly the
// tensors are filled and however little of the capacity is used.  The numbering needs the prefix
// sum of the per-tensor counts: every workgroup forms it in LDS, kFlatTensors tensors at
// a time, and a thread finds the tensor of its pair by bisection there.
__global__ __launch_bounds__(kFlatThreads) void scatter_regions_kernel(float* dense, int64_t n,
                                                                       RegionPayloads p, int32_t first,
                                                                       const int64_t* __restrict__ out_offsets,
                                                                       int32_t num_tensors, ScatterMode mode,
                                                                       float scale, uint32_t* diag_flags) {
  constexpr int kPerThread = kFlatTensors / kFlatThreads;  // tensors a thread stages per round
  __shared__ int64_t s_off[kFlatTensors];
  __shared__ uint32_t s_pre[kFlatTensors];   // pairs in the staged tensors before each one
  __shared__ uint32_t wave_sums[kFlatThreads / 64];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int w = first + blockIdx.y;
  const int32_t* __restrict__ counts = p.counts[w];
  const int32_t* __restrict__ idx = p.idx[w];
  const float* __restrict__ val = mode == kScatterClear ? nullptr : p.val[w];
  int64_t carry = 0;                                    // pairs in the tensors before the staged ones
  for (int32_t c0 = 0; c0 < num_tensors; c0 += kFlatTensors) {
    uint32_t cnt[kPerThread];
    int64_t off[kPerThread];
    uint32_t mine = 0;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      const int32_t j = c0 + tid * kPerThread + k;
      cnt[k] = 0;
      off[k] = 0;
      if (j < num_tensors) {
        off[k] = out_offsets[j];
        const int64_t cap = out_offsets[j + 1] - off[k];
        int64_t c = counts[j];
        if (c > cap) c = cap;
        if (c < 0) c = 0;
        cnt[k] = (uint32_t)c;
      }
      mine += cnt[k];
    }
    uint32_t incl = mine;
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t t = __shfl_up(incl, d);
      if (lane >= d) incl += t;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t before = 0, staged = 0;
#pragma unroll
    for (int v = 0; v < kFlatThreads / 64; ++v) {
      const uint32_t t = wave_sums[v];
      if (v < wave) before += t;
      staged += t;
    }
    uint32_t run = before + incl - mine;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      s_pre[tid * kPerThread + k] = run;
      s_off[tid * kPerThread + k] = off[k];
      run += cnt[k];
    }
    __syncthreads();
    // chunks of this workgroup that reach into the staged tensors
    for (int64_t x0 = (int64_t)blockIdx.x * kFlatChunk; x0 < carry + (int64_t)staged;
         x0 += (int64_t)gridDim.x * kFlatChunk) {
      if (x0 + kFlatChunk <= carry) continue;
      int64_t slot[kFlatPer];
#pragma unroll
      for (int k = 0; k < kFlatPer; ++k) {
        const int64_t q = x0 + tid + k * kFlatThreads - carry;
        slot[k] = -1;
        if (q >= 0 && q < (int64_t)staged) {
          int lo = 0, hi = kFlatTensors - 1;  // largest i with s_pre[i] <= q
          while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if ((int64_t)s_pre[mid] <= q) lo = mid;
            else hi = mid - 1;
          }
          slot[k] = s_off[lo] + (q - (int64_t)s_pre[lo]);
        }
      }
      int32_t i[kFlatPer];
      float x[kFlatPer];
#pragma unroll
      for (int k = 0; k < kFlatPer; ++k) {
        i[k] = slot[k] >= 0 ? idx[slot[k]] : 0;
        x[k] = (slot[k] >= 0 && mode != kScatterClear) ? val[slot[k]] : 0.0f;
      }
#pragma unroll
      for (int k = 0; k < kFlatPer; ++k)
        if (slot[k] >= 0) scatter_one(dense, n, i[k], x[k], scale, mode, diag_flags);
    }
    carry += staged;
    __syncthreads();
  }
}

// Receive side without float atomics: workers are added in the order given, so the
// result is that of the plain definition, bit for bit, in one launch.
//
// A workgroup owns a range of one tensor's elements that consists of whole parts of emit
// workgroups; in every payload's region those parts follow each other in index order
// (inside a part the order is free), so "index below the range's end" is monotone along
// a region and the payload's pairs inside the range are found by search: one wavefront
// per payload, both ends at once (half the lanes probe for each, 32 probes per round).
// Every thread then takes a few of the pairs into registers and marks their indices in
// an LDS bitmap of the range; a prefix sum over the bitmap numbers the distinct
// indices, which gives every index a slot in an LDS accumulator.  The slots start from
// dense[idx], the payloads are added one after the other with a barrier between them
// (inside one payload the indices are distinct), and the sums are stored.  Every index
// belongs to one workgroup, so plain loads and stores do.  (Float atomics complete at
// about 20 G/s on this part wherever they are executed, plain scattered stores at 80 G/s.)
//
// Positions [lo, hi) of the list L[0, m) whose values lie in [xa, xb), for a list in which
// "value < xa" and "value < xb" are monotone; every lane of the wavefront takes part and
// gets the same answer.
__device__ __forceinline__ void wave_equal_range(const int32_t* __restrict__ L, int m, int32_t xa, int32_t xb,
                                                 int lane, int& out_lo, int& out_hi) {
  const int half = lane >> 5;  // 0: lower bound of xa, 1: lower bound of xb
  const int sub = lane & 31;
  const int32_t x = half ? xb : xa;
  int lo = 0, hi = m;  // the answer of this lane's half lies in [lo, hi]
  while (__ballot(hi > lo)) {
    const int span = hi - lo;
    const int step = (span + 31) >> 5;
    const int pos = lo + sub * step;
    const bool less = span > 0 && pos < hi && L[pos] < x;
    const unsigned long long votes = __ballot(less);
    const int c = __popc((uint32_t)(votes >> (32 * half)));  // probes below x form a prefix
    if (span > 0) {
      if (c == 0) {
        hi = lo;
      } else {
        const int next = lo + c * step;
        lo = lo + (c - 1) * step + 1;
        hi = next < hi ? next : hi;
      }
    }
  }
  out_lo = __shfl(lo, 0);
  out_hi = __shfl(lo, 32);
}

// The same for two lists at once, with the probes of both in flight together (`safe` is any
// readable word: it is read in place of a probe that has nothing left to ask).
__device__ __forceinline__ void wave_equal_range2(const int32_t* __restrict__ L0, int m0, const int32_t* __restrict__ L1,
                                                  int m1, const int32_t* __restrict__ safe, int32_t xa, int32_t xb,
                                                  int lane, int& lo_0, int& hi_0, int& lo_1, int& hi_1) {
  const int half = lane >> 5;
  const int sub = lane & 31;
  const int32_t x = half ? xb : xa;
  const int32_t* __restrict__ A = m0 > 0 ? L0 : safe;
  const int32_t* __restrict__ B = m1 > 0 ? L1 : safe;
  int lo0 = 0, hi0 = m0, lo1 = 0, hi1 = m1;
  while (__ballot(hi0 > lo0 || hi1 > lo1)) {
    const int span0 = hi0 - lo0, span1 = hi1 - lo1;
    const int step0 = (span0 + 31) >> 5, step1 = (span1 + 31) >> 5;
    const int pos0 = lo0 + sub * step0, pos1 = lo1 + sub * step1;
    const bool ask0 = span0 > 0 && pos0 < hi0, ask1 = span1 > 0 && pos1 < hi1;
    const int32_t v0 = A[ask0 ? pos0 : 0];
    const int32_t v1 = B[ask1 ? pos1 : 0];
    const unsigned long long votes0 = __ballot(ask0 && v0 < x);
    const unsigned long long votes1 = __ballot(ask1 && v1 < x);
    const int c0 = __popc((uint32_t)(votes0 >> (32 * half)));
    const int c1 = __popc((uint32_t)(votes1 >> (32 * half)));
    if (span0 > 0) {
      if (c0 == 0) {
        hi0 = lo0;
      } else {
        const int next = lo0 + c0 * step0;
        lo0 = lo0 + (c0 - 1) * step0 + 1;
        hi0 = next < hi0 ? next : hi0;
      }
    }
    if (span1 > 0) {
      if (c1 == 0) {
        hi1 = lo1;
      } else {
        const int next = lo1 + c1 * step1;
        lo1 = lo1 + (c1 - 1) * step1 + 1;
        hi1 = next < hi1 ? next : hi1;
      }
    }
  }
  lo_0 = __shfl(lo0, 0);
  hi_0 = __shfl(lo0, 32);
  lo_1 = __shfl(lo1, 0);
  hi_1 = __shfl(lo1, 32);
}

// Finds every payload's pairs inside [blk.begin, blk.end) and fills begin[], idx_at[] and
// val_at[] (in LDS: a payload's pointers looked up per pair in the kernel's argument block
// would put a load from memory in front of every pair load).
template <typename Shared>
__device__ __forceinline__ int locate_pairs(Shared& sh, const RegionPayloads& p, int32_t num_payloads, int64_t region,
                                            int64_t cap, const MergeBlock& blk, int tid, int waves) {
  const int lane = tid & 63;
  const int wave = tid >> 6;
  for (int w = wave; w < num_payloads; w += waves) {
    int64_t cnt = p.counts[w][blk.tensor];
    if (cnt > cap) cnt = cap;
    if (cnt < 0) cnt = 0;
    int lo, hi;
    wave_equal_range(p.idx[w] + region, (int)cnt, (int32_t)blk.begin, (int32_t)blk.end, lane, lo, hi);
    if (lane == 0) {
      sh.idx_at[w] = p.idx[w] + region + lo;
      sh.val_at[w] = p.val[w] ? p.val[w] + region + lo : nullptr;
      sh.begin[w + 1] = hi - lo;  // length for now
    }
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    sh.begin[0] = 0;
    for (int w = 0; w < num_payloads; ++w) {
      const int len = sh.begin[w + 1];
      sh.begin[w + 1] = run + len;
      run += len;
    }
  }
  __syncthreads();
  return sh.begin[num_payloads];
}

// Two sets of payloads at once (the new ones and the previous ones of a replacing merge):
// wavefront w searches payload w of both sets with the probes of the two searches in flight
// together.  `total2` gets the second set's number of pairs, the first set's is returned.
template <typename Shared, typename Shared2>
__device__ __forceinline__ int locate_pairs2(Shared& sh, const RegionPayloads& p, int32_t num_payloads, Shared2& sh2,
                                             const RegionPayloads& p2, int32_t num_payloads2, int64_t region,
                                             int64_t cap, const MergeBlock& blk, const int32_t* __restrict__ safe,
                                             int tid, int waves, int& total2) {
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int most = num_payloads > num_payloads2 ? num_payloads : num_payloads2;
  for (int w = wave; w < most; w += waves) {
    int64_t cnt = w < num_payloads ? (int64_t)p.counts[w][blk.tensor] : 0;
    int64_t cnt2 = w < num_payloads2 ? (int64_t)p2.counts[w][blk.tensor] : 0;
    if (cnt > cap) cnt = cap;
    if (cnt < 0) cnt = 0;
    if (cnt2 > cap) cnt2 = cap;
    if (cnt2 < 0) cnt2 = 0;
    const int32_t* __restrict__ list = w < num_payloads ? p.idx[w] + region : safe;
    const int32_t* __restrict__ list2 = w < num_payloads2 ? p2.idx[w] + region : safe;
    int lo, hi, lo2, hi2;
    wave_equal_range2(list, (int)cnt, list2, (int)cnt2, safe, (int32_t)blk.begin, (int32_t)blk.end, lane, lo, hi, lo2,
                      hi2);
    if (lane == 0) {
      if (w < num_payloads) {
        sh.idx_at[w] = list + lo;
        sh.val_at[w] = p.val[w] ? p.val[w] + region + lo : nullptr;
        sh.begin[w + 1] = hi - lo;  // length for now
      }
      if (w < num_payloads2) {
        sh2.idx_at[w] = list2 + lo2;
        sh2.val_at[w] = nullptr;
        sh2.begin[w + 1] = hi2 - lo2;
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    sh.begin[0] = 0;
    for (int w = 0; w < num_payloads; ++w) {
      const int len = sh.begin[w + 1];
      sh.begin[w + 1] = run + len;
      run += len;
    }
  }
  if (tid == 64) {
    int run = 0;
    sh2.begin[0] = 0;
    for (int w = 0; w < num_payloads2; ++w) {
      const int len = sh2.begin[w + 1];
      sh2.begin[w + 1] = run + len;
      run += len;
    }
  }
  __syncthreads();
  total2 = sh2.begin[num_payloads2];
  return sh.begin[num_payloads];
}

// Largest w with begin[w] <= q.
__device__ __forceinline__ int payload_of(const int32_t* begin, int num_payloads, int q) {
  int w = 0, e = num_payloads;
  while (e - w > 1) {
    const int mid = (w + e) >> 1;
    if (begin[mid] <= q) w = mid;
    else e = mid;
  }
  return w;
}

template <int CAP>
struct MergeShared {
  alignas(16) uint32_t bitmap[kMergeMaxRange / 32];
  uint32_t prefix[kMergeMaxRange / 128];  // distinct indices before each group of four bitmap words
  float acc[CAP];
  uint32_t wave_sums[kMergeMaxThreads / 64];
  int32_t begin[kMaxPayloads + 1];  // number of pairs of the payloads before w inside the range
  const int32_t* idx_at[kMaxPayloads];  // payload w's first pair inside the range
  const float* val_at[kMaxPayloads];
};

// `scale` multiplies every value first (1 for the plain sum; -learning rate for the SGD
// apply, where `dense` is the parameter vector).
//
// REPLACE: `dense` becomes the sum of the payloads instead of growing by it.  It holds
// the sum of an earlier set of payloads (`old`: their index lists are all that is needed),
// i.e. zero wherever none of those has an index.  The accumulator then starts from zero,
// which saves the scattered reads of `dense`, and an index of the earlier set that is in
// none of the new payloads gets a zero: one launch instead of a clear and an accumulate.
struct OldLists {
  int32_t begin[kMaxPayloads + 1];
  const int32_t* idx_at[kMaxPayloads];
  const float* val_at[kMaxPayloads];  // unused
};

// Number of the distinct index r (relative to the range) among those of the range: the indices
// marked before its group of 128 bits, plus the marked bits below it inside the group.
template <int CAP>
__device__ __forceinline__ int merge_slot(const MergeShared<CAP>& sh, int32_t r) {
  const uint4 g = reinterpret_cast<const uint4*>(sh.bitmap)[r >> 7];
  const int word = (r >> 5) & 3;
  const uint32_t own = word == 0 ? g.x : word == 1 ? g.y : word == 2 ? g.z : g.w;
  uint32_t c = (uint32_t)__popc(own & ((1u << (r & 31)) - 1u));
  c += word > 0 ? (uint32_t)__popc(g.x) : 0u;
  c += word > 1 ? (uint32_t)__popc(g.y) : 0u;
  c += word > 2 ? (uint32_t)__popc(g.z) : 0u;
  return (int)(sh.prefix[r >> 7] + c);
}

// THREADS: 512 when there are at most eight payloads (one wavefront searches one payload's region,
// and four workgroups of eight wavefronts fit a compute unit, LDS included: the 970 ranges of a
// 122 M-element set then run all at once instead of in two rounds), 1024 otherwise.  kMergeCap:
// pairs a workgroup takes into registers, slots of its LDS accumulator (a range with more takes
// the slow way at the end of the kernel).
template <bool REPLACE, int THREADS>
__global__ __launch_bounds__(THREADS) void merge_regions_kernel(float* __restrict__ dense, RegionPayloads p,
                                                                      int32_t num_payloads, RegionPayloads old,
                                                                      int32_t num_old,
                                                                      const int64_t* __restrict__ out_offsets,
                                                                      const MergeBlock* __restrict__ blocks,
                                                                      float scale, int32_t scaled) {
  constexpr int kMergeThreads = THREADS;
  constexpr int kMergeWaves = THREADS / 64;
  constexpr int kMergeCap = THREADS == 512 ? kMergeCapSmall : kMergeCapLarge;
  constexpr int kPerThread = kMergeCap / kMergeThreads;
  constexpr int kWordsPerThread = kMergeMaxRange / 32 / kMergeThreads;
  static_assert(kMergeCap % THREADS == 0 && kWordsPerThread % 4 == 0 && THREADS <= kMergeMaxThreads, "dealt evenly to threads");
  __shared__ MergeShared<kMergeCap> sh;
  __shared__ OldLists was;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const MergeBlock blk = blocks[blockIdx.x];
  const int j = blk.tensor;
  const int64_t region = out_offsets[j];
  const int64_t cap = out_offsets[j + 1] - region;
  const int32_t length = (int32_t)(blk.end - blk.begin);  // <= kMergeMaxRange
#pragma unroll
  for (int k = 0; k < kWordsPerThread; ++k) sh.bitmap[tid * kWordsPerThread + k] = 0;
  int old_total = 0;
  const int total = (REPLACE && num_old > 0)
                        ? locate_pairs2(sh, p, num_payloads, was, old, num_old, region, cap, blk,
                                        reinterpret_cast<const int32_t*>(blocks), tid, kMergeWaves, old_total)
                        : locate_pairs(sh, p, num_payloads, region, cap, blk, tid, kMergeWaves);
  if (total == 0 && old_total == 0) return;
  // Whether the accumulator may start from zero: the earlier set's indices of this range fit
  // the registers too.  Otherwise they are cleared in `dense` first and the sum is added
  // to what `dense` holds then, as without REPLACE.
  const bool from_zero = REPLACE && total <= kMergeCap && old_total <= kMergeCap;
  if (REPLACE && !from_zero) {
    for (int q = tid; q < old_total; q += kMergeThreads) {
      const int w = payload_of(was.begin, num_old, q);
      const int64_t r = (int64_t)was.idx_at[w][q - was.begin[w]] - blk.begin;
      if (r >= 0 && r < length) dense[blk.begin + r] = 0.0f;
    }
    __syncthreads();  // the zeros are in place before any thread of the workgroup reads `dense`
  }
  if (total == 0 && !from_zero) return;

  if (total <= kMergeCap) {
    // the earlier set's indices of this range, asked for first and not looked at before the
    // new pairs are in: their loads are in flight together with those of the pairs
    int32_t was_idx[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      const int q = tid + k * kMergeThreads;
      was_idx[k] = 0;
      if (from_zero && q < old_total) {
        const int w = payload_of(was.begin, num_old, q);
        was_idx[k] = was.idx_at[w][q - was.begin[w]];
      }
    }
    // this thread's pairs: payload, index relative to the range (-1: none), value
    int pw[kPerThread];
    int32_t rel[kPerThread];
    float x[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      const int q = tid + k * kMergeThreads;
      rel[k] = -1;
      pw[k] = 0;
      x[k] = 0.0f;
      if (q < total) {
        int w = 0, e = num_payloads;  // largest w with begin[w] <= q
        while (e - w > 1) {
          const int mid = (w + e) >> 1;
          if (sh.begin[mid] <= q) w = mid;
          else e = mid;
        }
        const int src = q - sh.begin[w];
        const int64_t r = (int64_t)sh.idx_at[w][src] - blk.begin;
        const float value = sh.val_at[w][src];
        x[k] = scaled ? scale * value : value;
        pw[k] = w;
        if (r >= 0 && r < length) {  // anything else can only come from a region that does not ascend
          rel[k] = (int32_t)r;
          atomicOr(&sh.bitmap[r >> 5], 1u << (r & 31));
        }
      }
    }
    __syncthreads();
    if (from_zero) {  // an index of the earlier set that no new payload has becomes zero
#pragma unroll
      for (int k = 0; k < kPerThread; ++k) {
        const int64_t r = (int64_t)was_idx[k] - blk.begin;
        if (tid + k * kMergeThreads < old_total && r >= 0 && r < length && !((sh.bitmap[r >> 5] >> (r & 31)) & 1u))
          dense[blk.begin + r] = 0.0f;
      }
      if (total == 0) return;
    }
    {
      uint32_t mine = 0, c[kWordsPerThread];
#pragma unroll
      for (int k = 0; k < kWordsPerThread; ++k) {
        c[k] = (uint32_t)__popc(sh.bitmap[tid * kWordsPerThread + k]);
        mine += c[k];
      }
      uint32_t incl = mine;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
      }
      if (lane == 63) sh.wave_sums[wave] = incl;
      __syncthreads();
      uint32_t run = incl - mine;
      for (int v = 0; v < wave; ++v) run += sh.wave_sums[v];
#pragma unroll
      for (int k = 0; k < kWordsPerThread; ++k) {
        if ((k & 3) == 0) sh.prefix[(tid * kWordsPerThread + k) >> 2] = run;
        run += c[k];
      }
    }
    __syncthreads();
    int id[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      id[k] = -1;
      if (rel[k] >= 0) {
        id[k] = merge_slot(sh, rel[k]);
        // pairs of several payloads with one index write the same
        sh.acc[id[k]] = from_zero ? 0.0f : dense[blk.begin + rel[k]];
      }
    }
    __syncthreads();
    for (int w = 0; w < num_payloads; ++w) {  // payloads in the order given
#pragma unroll
      for (int k = 0; k < kPerThread; ++k)
        if (id[k] >= 0 && pw[k] == w) sh.acc[id[k]] = sh.acc[id[k]] + x[k];
      __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < kPerThread; ++k)
      if (id[k] >= 0) dense[blk.begin + rel[k]] = sh.acc[id[k]];
  } else {
    // More pairs than a thread's registers and the accumulator hold (many workers, or a
    // density above what this kernel is chosen for): the same steps with the pairs read
    // from the payloads' arrays each time, the distinct indices taken kMergeCap at a time.
    auto pair_of = [&](int q, int& w, int& src) {
      int lo_w = 0, e = num_payloads;  // largest w with begin[w] <= q
      while (e - lo_w > 1) {
        const int mid = (lo_w + e) >> 1;
        if (sh.begin[mid] <= q) lo_w = mid;
        else e = mid;
      }
      w = lo_w;
      src = q - sh.begin[w];
    };
    auto slot_of = [&](int64_t r) { return merge_slot(sh, (int32_t)r); };
    for (int q = tid; q < total; q += kMergeThreads) {
      int w;
      int src;
      pair_of(q, w, src);
      const int64_t r = (int64_t)sh.idx_at[w][src] - blk.begin;
      if (r >= 0 && r < length) atomicOr(&sh.bitmap[r >> 5], 1u << (r & 31));
    }
    __syncthreads();
    int distinct;
    {
      uint32_t mine = 0, c[kWordsPerThread];
#pragma unroll
      for (int k = 0; k < kWordsPerThread; ++k) {
        c[k] = (uint32_t)__popc(sh.bitmap[tid * kWordsPerThread + k]);
        mine += c[k];
      }
      uint32_t incl = mine;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
      }
      if (lane == 63) sh.wave_sums[wave] = incl;
      __syncthreads();
      uint32_t run = incl - mine, all = 0;
      for (int v = 0; v < kMergeWaves; ++v) {
        if (v < wave) run += sh.wave_sums[v];
        all += sh.wave_sums[v];
      }
      distinct = (int)all;
#pragma unroll
      for (int k = 0; k < kWordsPerThread; ++k) {
        if ((k & 3) == 0) sh.prefix[(tid * kWordsPerThread + k) >> 2] = run;
        run += c[k];
      }
    }
    __syncthreads();
    for (int first_slot = 0; first_slot < distinct; first_slot += kMergeCap) {
      for (int q = tid; q < total; q += kMergeThreads) {
        int w;
        int src;
        pair_of(q, w, src);
        const int64_t r = (int64_t)sh.idx_at[w][src] - blk.begin;
        if (r < 0 || r >= length) continue;
        const int id = slot_of(r) - first_slot;
        if (id >= 0 && id < kMergeCap) sh.acc[id] = dense[blk.begin + r];
      }
      __syncthreads();
      for (int w = 0; w < num_payloads; ++w) {  // payloads in the order given
        const int len = sh.begin[w + 1] - sh.begin[w];
        for (int q = tid; q < len; q += kMergeThreads) {
          const int64_t r = (int64_t)sh.idx_at[w][q] - blk.begin;
          if (r < 0 || r >= length) continue;
          const int id = slot_of(r) - first_slot;
          if (id >= 0 && id < kMergeCap) {
            const float value = sh.val_at[w][q];
            const float x = scaled ? scale * value : value;
            sh.acc[id] = sh.acc[id] + x;
          }
        }
        __syncthreads();
      }
      for (int q = tid; q < total; q += kMergeThreads) {
        int w;
        int src;
        pair_of(q, w, src);
        const int64_t r = (int64_t)sh.idx_at[w][src] - blk.begin;
        if (r < 0 || r >= length) continue;
        const int id = slot_of(r) - first_slot;
        if (id >= 0 && id < kMergeCap) dense[blk.begin + r] = sh.acc[id];
      }
      __syncthreads();
    }
  }
}

// Receive side at warm-up densities (paper: Section 4, warm-up training -- 25 % down to
// 0.4 % of the elements are sent during the first epochs): with millions of pairs per
// payload, adding them one by one to `dense` costs a scattered read-modify-write each.
// Here a workgroup owns one emit workgroup's part of a tensor (at most kEmitElements
// elements, contiguous in index order in every payload's region, see above), keeps the
// whole range of `dense` in LDS, adds the payloads' pairs to it in the order of the
// payloads, and writes the range back: `dense` is read and written once, coalesced,
// the pairs are read once, coalesced, and the sums are those of the plain definition,
// bit for bit.
//
// The pairs are taken a round at a time: up to kPartRound consecutive pairs of one
// payload, kPartPer per thread, with the loads of the next two rounds in flight.  Pairs
// of one payload have distinct indices and are added without synchronisation; a
// barrier separates one payload from the next.
//
// At these densities a region holds up to millions of pairs and the search for a part's
// pairs is several rounds of dependent loads: with one workgroup per compute unit (the
// accumulator fills LDS) nothing else would run meanwhile.  So the searches of all parts
// and payloads run first, spread over the chip, and leave (first pair, number of pairs)
// of every part in every payload's region in a table (a part ends where the next one of
// its tensor starts, so one bound per part is searched for).  The probes are what this
// launch costs (each one a 64-byte sector from HBM: 350 MB with 32 probes per round and
// two bounds per part), so eight lanes share a search: 8 probes per round, about seven
// rounds for a region of a million pairs.
__global__ __launch_bounds__(kFlatThreads) void locate_parts_kernel(RegionPayloads p, int32_t num_payloads,
                                                                    const int64_t* __restrict__ out_offsets,
                                                                    const MergeBlock* __restrict__ blocks,
                                                                    int32_t num_blocks, int2* __restrict__ found) {
  // A wavefront takes seven consecutive parts of one payload; its eighth group finds the
  // start of the part after them, which is where the seventh ends.
  const int lane = threadIdx.x & 63;
  const int group = lane >> 3;
  const int sub = lane & 7;
  const int waves_per_payload = (num_blocks + 6) / 7;
  const int64_t wave_id = (int64_t)blockIdx.x * (kFlatThreads / 64) + (threadIdx.x >> 6);
  const int w = (int)(wave_id / waves_per_payload);
  const int b = (int)(wave_id % waves_per_payload) * 7 + group;
  const bool valid = w < num_payloads && b < num_blocks;
  const int32_t* __restrict__ list = nullptr;
  int32_t x = 0;
  int lo = 0, hi = 0;  // the answer lies in [lo, hi]
  int cnt = 0;
  bool last = true;    // the tensor's last part: it ends where the region's pairs end
  if (valid) {
    const MergeBlock blk = blocks[b];
    const int64_t region = out_offsets[blk.tensor];
    const int64_t cap = out_offsets[blk.tensor + 1] - region;
    int64_t c = p.counts[w][blk.tensor];
    if (c > cap) c = cap;
    if (c < 0) c = 0;
    cnt = (int)c;
    last = b + 1 >= num_blocks || blocks[b + 1].tensor != blk.tensor;
    list = p.idx[w] + region;
    x = (int32_t)blk.begin;
    hi = cnt;
  }
  // first position whose index is not below x ("index < x" is monotone along a region)
  while (__ballot(hi > lo)) {
    const int span = hi - lo;
    const int step = (span + 7) >> 3;
    const int pos = lo + sub * step;
    const bool less = span > 0 && pos < hi && list[pos] < x;
    const unsigned long long votes = __ballot(less);
    const int c = __popc((uint32_t)(votes >> (8 * group)) & 0xFFu);  // probes below x form a prefix
    if (span > 0) {
      if (c == 0) {
        hi = lo;
      } else {
        const int next = lo + c * step;
        lo = lo + (c - 1) * step + 1;
        hi = next < hi ? next : hi;
      }
    }
  }
  const int next_lo = __shfl(lo, (lane + 8) & 63);  // of the part after this one (group 7 does not use it)
  if (valid && group < 7 && sub == 0) {
    const int end = last ? cnt : next_lo;
    found[(int64_t)b * num_payloads + w] = make_int2(lo, end > lo ? end - lo : 0);
  }
}

// Fills begin[], idx_at[] and val_at[] from that table; returns the number of pairs.
template <typename Shared>
__device__ __forceinline__ int located_pairs(Shared& sh, const RegionPayloads& p, int32_t num_payloads, int64_t region,
                                             const int2* __restrict__ found, int part, int tid) {
  if (tid < num_payloads) {
    const int2 f = found[(int64_t)part * num_payloads + tid];
    sh.idx_at[tid] = p.idx[tid] + region + f.x;
    sh.val_at[tid] = p.val[tid] ? p.val[tid] + region + f.x : nullptr;
    sh.begin[tid + 1] = f.y;  // length for now
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    sh.begin[0] = 0;
    for (int w = 0; w < num_payloads; ++w) {
      const int len = sh.begin[w + 1];
      sh.begin[w + 1] = run + len;
      run += len;
    }
  }
  __syncthreads();
  return sh.begin[num_payloads];
}

struct PartShared {
  float acc[kEmitElements];
  int32_t begin[kMaxPayloads + 1];  // number of pairs of the payloads before w inside the range
  const int32_t* idx_at[kMaxPayloads];  // payload w's first pair inside the range
  const float* val_at[kMaxPayloads];
};

// REPLACE: `dense` becomes the sum of the payloads: the accumulator starts from zero instead of
// the range of `dense`, and every range is written, also one that no pair falls into.
template <bool REPLACE>
__global__ __launch_bounds__(kPartThreads) void merge_parts_kernel(float* __restrict__ dense, RegionPayloads p,
                                                                   int32_t num_payloads,
                                                                   const int64_t* __restrict__ out_offsets,
                                                                   const MergeBlock* __restrict__ blocks,
                                                                   int32_t num_blocks,
                                                                   const int2* __restrict__ found, float scale,
                                                                   int32_t scaled) {
  constexpr int kElems = kEmitElements / kPartThreads;
  __shared__ PartShared sh;
  const int tid = threadIdx.x;
  // The accumulator fills LDS, so a workgroup is alone on its compute unit: the grid is one
  // workgroup per compute unit and every workgroup takes parts b, b + grid, ...; the range of
  // the next part is requested before the finished one is written back, so that neither
  // the write-back nor the table look-up leaves the memory pipeline of the unit empty.
  int b = blockIdx.x;
  if (b >= num_blocks) return;
  MergeBlock blk = blocks[b];
  float d[kElems];
  {
    const int32_t len = REPLACE ? 0 : (int32_t)(blk.end - blk.begin);
    const float* __restrict__ src = dense + blk.begin;
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
      const int e = tid + i * kPartThreads;
      d[i] = e < len ? __builtin_nontemporal_load(src + e) : 0.0f;
    }
  }
  for (;;) {
    const int next_b = b + (int)gridDim.x;
    const bool more = next_b < num_blocks;
    const MergeBlock next = blocks[more ? next_b : b];
    const int32_t length = (int32_t)(blk.end - blk.begin);  // <= kEmitElements
    float* __restrict__ range = dense + blk.begin;
    const int total = located_pairs(sh, p, num_payloads, out_offsets[blk.tensor], found, b, tid);
    if (total > 0) {
#pragma unroll
      for (int k = 0; k < kElems; ++k) sh.acc[tid + k * kPartThreads] = d[k];

      if (total <= kPartRound) {
        // Few pairs (many payloads of a low density): all of them at once, whatever payload they
        // belong to, so that their loads are one wait; then payload after payload from registers.
        int32_t at[kPartPer];  // payload << 16 | index relative to the range; -1: none
        float x[kPartPer];
#pragma unroll
        for (int k = 0; k < kPartPer; ++k) {
          const int q = tid + k * kPartThreads;
          at[k] = -1;
          x[k] = 0.0f;
          if (q < total) {
            const int w = payload_of(sh.begin, num_payloads, q);
            const int src = q - sh.begin[w];
            const int64_t r = (int64_t)__builtin_nontemporal_load(sh.idx_at[w] + src) - blk.begin;
            const float value = __builtin_nontemporal_load(sh.val_at[w] + src);
            x[k] = scaled ? scale * value : value;
            if (r >= 0 && r < length) at[k] = (int32_t)r | (w << 16);  // anything else: a foreign region
          }
        }
        __syncthreads();  // the accumulator is filled
        for (int w = 0; w < num_payloads; ++w) {  // payloads in the order given
          if (sh.begin[w + 1] == sh.begin[w]) continue;
          float sum[kPartPer];
#pragma unroll
          for (int k = 0; k < kPartPer; ++k)
            sum[k] = (at[k] >= 0 && (at[k] >> 16) == w) ? sh.acc[at[k] & 0xFFFF] + x[k] : 0.0f;
#pragma unroll
          for (int k = 0; k < kPartPer; ++k)
            if (at[k] >= 0 && (at[k] >> 16) == w) sh.acc[at[k] & 0xFFFF] = sum[k];
          __syncthreads();
        }
      } else {
      // A round: up to kPartRound consecutive pairs of one payload.  Two rounds are on their way
      // while a third is added, and nothing in fetch() depends on the loaded words.
      struct Loaded {
        int32_t idx[kPartPer];
        float x[kPartPer];
        int w;  // payload
        int n;  // pairs of the round; 0: there is no further round
      };
      int cursor_w = 0, cursor_at = 0;  // next pair to fetch: payload, position among its pairs inside the range
      auto fetch = [&](Loaded& L) {
        L.n = 0;
        L.w = 0;
        while (cursor_w < num_payloads) {
          const int len = sh.begin[cursor_w + 1] - sh.begin[cursor_w];
          if (cursor_at < len) break;
          ++cursor_w;
          cursor_at = 0;
        }
        if (cursor_w >= num_payloads) return;
        const int left = sh.begin[cursor_w + 1] - sh.begin[cursor_w] - cursor_at;
        L.w = cursor_w;
        L.n = left < kPartRound ? left : kPartRound;
        const int32_t* __restrict__ ip = sh.idx_at[cursor_w] + cursor_at;
        const float* __restrict__ vp = sh.val_at[cursor_w] + cursor_at;
        cursor_at += L.n;
#pragma unroll
        for (int k = 0; k < kPartPer; ++k) {
          const int q = tid + k * kPartThreads;
          L.idx[k] = 0;
          L.x[k] = 0.0f;
          if (q < L.n) {
            L.idx[k] = __builtin_nontemporal_load(ip + q);
            L.x[k] = __builtin_nontemporal_load(vp + q);
          }
        }
      };
      int last_w = -1;
      // Adds the round in L and refills L with the next round to fetch.
      auto add = [&](Loaded& L) {
        int32_t at[kPartPer];  // index relative to the range; -1: none
        float x[kPartPer];
#pragma unroll
        for (int k = 0; k < kPartPer; ++k) {
          const int64_t r = (int64_t)L.idx[k] - blk.begin;
          // an index outside the range can only come from a foreign region
          at[k] = (tid + k * kPartThreads < L.n && r >= 0 && r < length) ? (int32_t)r : -1;
          x[k] = scaled ? scale * L.x[k] : L.x[k];
        }
        const int w = L.w;
        fetch(L);
        if (w != last_w) __syncthreads();  // the payload before is added (the first time: the accumulator is filled)
        last_w = w;
        // the indices of one payload are distinct: all reads, then all writes, no barrier between its rounds
        float sum[kPartPer];
#pragma unroll
        for (int k = 0; k < kPartPer; ++k) sum[k] = at[k] >= 0 ? sh.acc[at[k]] + x[k] : 0.0f;
#pragma unroll
        for (int k = 0; k < kPartPer; ++k)
          if (at[k] >= 0) sh.acc[at[k]] = sum[k];
      };
      Loaded A, B;
      fetch(A);
      fetch(B);
      for (;;) {
        if (A.n == 0) break;
        add(A);
        if (B.n == 0) break;
        add(B);
      }
      __syncthreads();
      }
    }
    {  // (every d[i] is assigned anew: the old values must not stay alive through the rounds above)
      const int32_t len = (more && !REPLACE) ? (int32_t)(next.end - next.begin) : 0;
      const float* __restrict__ src = dense + next.begin;
#pragma unroll
      for (int i = 0; i < kElems; ++i) {
        const int e = tid + i * kPartThreads;
        d[i] = e < len ? __builtin_nontemporal_load(src + e) : 0.0f;
      }
    }
    if (total > 0) {
#pragma unroll
      for (int k = 0; k < kElems; ++k) {
        const int e = tid + k * kPartThreads;
        if (e < length) __builtin_nontemporal_store(sh.acc[e], range + e);
      }
    } else if (REPLACE) {
#pragma unroll
      for (int k = 0; k < kElems; ++k) {
        const int e = tid + k * kPartThreads;
        if (e < length) __builtin_nontemporal_store(0.0f, range + e);
      }
    }
    if (!more) break;
    b = next_b;
    blk = next;
    __syncthreads();  // the accumulator and the tables are free again
  }
}

// The sparse clear at the same densities: the indices of all payloads inside the part
// are marked in an LDS bitmap and zeros stored where a bit is set, every element once.
struct PartClearShared {
  uint32_t bitmap[kEmitElements / 32];
  int32_t begin[kMaxPayloads + 1];
  const int32_t* idx_at[kMaxPayloads];
  const float* val_at[kMaxPayloads];
};

__global__ __launch_bounds__(kPartClearThreads) void clear_parts_kernel(float* __restrict__ dense, RegionPayloads p,
                                                                        int32_t num_payloads,
                                                                        const int64_t* __restrict__ out_offsets,
                                                                        const MergeBlock* __restrict__ blocks,
                                                                        const int2* __restrict__ found) {
  constexpr int kWords = kEmitElements / 32 / kPartClearThreads;
  __shared__ PartClearShared sh;
  const int tid = threadIdx.x;
  const MergeBlock blk = blocks[blockIdx.x];
  const int j = blk.tensor;
  const int64_t region = out_offsets[j];
  const int32_t length = (int32_t)(blk.end - blk.begin);
#pragma unroll
  for (int k = 0; k < kWords; ++k) sh.bitmap[tid + k * kPartClearThreads] = 0;
  const int total = located_pairs(sh, p, num_payloads, region, found, (int)blockIdx.x, tid);
  if (total == 0) return;
  for (int w = 0; w < num_payloads; ++w) {
    const int n = sh.begin[w + 1] - sh.begin[w];
    const int32_t* __restrict__ ip = sh.idx_at[w];
    for (int first = 0; first < n; first += kPartClearThreads * kPartPer) {
      int32_t r[kPartPer];
#pragma unroll
      for (int k = 0; k < kPartPer; ++k) {
        const int q = first + tid + k * kPartClearThreads;
        r[k] = q < n ? __builtin_nontemporal_load(ip + q) : -1;
      }
#pragma unroll
      for (int k = 0; k < kPartPer; ++k) {
        const int64_t rr = (int64_t)r[k] - blk.begin;  // outside the range: a foreign region, or no pair
        if (r[k] >= 0 && rr >= 0 && rr < length) atomicOr(&sh.bitmap[rr >> 5], 1u << (rr & 31));
      }
    }
  }
  __syncthreads();
  float* __restrict__ range = dense + blk.begin;
  // Lane after lane along the range, four consecutive elements per lane.  A store of part
  // of a 64-byte sector costs the memory system a read-modify-write of its own, so a sector
  // with any element to clear is written whole by its four lanes, each of which reads its
  // 16 bytes first unless all of them are cleared.
  const bool aligned = ((reinterpret_cast<uintptr_t>(range) & 15) == 0);
  if (aligned) {
    constexpr int kGroups = kEmitElements / 4 / kPartClearThreads;
    constexpr int kBatch = 8;
    for (int i0 = 0; i0 < kGroups; i0 += kBatch) {
      uint32_t nib[kBatch];
      bool touch[kBatch];  // the lane's sector has an element to clear
      float4 old[kBatch];
#pragma unroll
      for (int i = 0; i < kBatch; ++i) {
        const int e4 = tid + (i0 + i) * kPartClearThreads;
        const int e = e4 * 4;
        const uint32_t word = e < length ? sh.bitmap[e4 >> 3] : 0u;
        nib[i] = (word >> ((e4 & 7) * 4)) & 15u;
        touch[i] = ((word >> ((e4 & 4) * 4)) & 0xFFFFu) != 0;
        old[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (touch[i] && nib[i] != 15u && e + 4 <= length) old[i] = *reinterpret_cast<const float4*>(range + e);
      }
#pragma unroll
      for (int i = 0; i < kBatch; ++i) {
        if (!touch[i]) continue;
        const int e = (tid + (i0 + i) * kPartClearThreads) * 4;
        if (e + 4 <= length) {
          float4 v = old[i];
          if (nib[i] & 1u) v.x = 0.0f;
          if (nib[i] & 2u) v.y = 0.0f;
          if (nib[i] & 4u) v.z = 0.0f;
          if (nib[i] & 8u) v.w = 0.0f;
          *reinterpret_cast<float4*>(range + e) = v;
        } else {  // the last, incomplete group of the range
#pragma unroll
          for (int b = 0; b < 4; ++b)
            if (((nib[i] >> b) & 1u) && e + b < length) range[e + b] = 0.0f;
        }
      }
    }
  } else {
    for (int e4 = tid; e4 * 4 < length; e4 += kPartClearThreads) {
      const uint32_t nib = (sh.bitmap[e4 >> 3] >> ((e4 & 7) * 4)) & 15u;
      const int e = e4 * 4;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if (((nib >> b) & 1u) && e + b < length) range[e + b] = 0.0f;
    }
  }
}

}  // namespace

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
hipError_t launch_scatter_pairs(float* dense, int64_t n, const PairPayloads& p, int32_t first,
                                int32_t num, int64_t max_count, ScatterMode mode, float scale,
                                uint32_t* diag_flags, hipStream_t stream) {
  if (num <= 0 || max_count <= 0) return hipSuccess;
  int64_t chunks = ceil_div(max_count, 256 * 4);
  if (chunks > 4096) chunks = 4096;
  hipLaunchKernelGGL(scatter_pairs_kernel, dim3((unsigned)chunks, (unsigned)num), dim3(256), 0, stream,
                     dense, n, p, first, mode, scale, diag_flags);
  return hipGetLastError();
}

hipError_t launch_scatter_regions(float* dense, int64_t n, const RegionPayloads& p, int32_t first,
                                  int32_t num, const int64_t* out_offsets_dev, int32_t num_tensors,
                                  int64_t total_capacity, ScatterMode mode, float scale,
                                  uint32_t* diag_flags, hipStream_t stream) {
  if (num <= 0 || total_capacity <= 0) return hipSuccess;
  // a quarter of the capacity: regions sized as recommended hold eight times the expected
  // pairs, so most workgroups find one chunk; fuller regions make them loop
  int64_t chunks = ceil_div(total_capacity, 4 * kFlatChunk);
  if (chunks > 65536) chunks = 65536;
  hipLaunchKernelGGL(scatter_regions_kernel, dim3((unsigned)chunks, (unsigned)num), dim3(kFlatThreads), 0, stream,
                     dense, n, p, first, out_offsets_dev, num_tensors, mode, scale, diag_flags);
  return hipGetLastError();
}

hipError_t launch_merge_regions(float* dense, const RegionPayloads& p, int32_t num, const RegionPayloads* old,
                                int32_t num_old, const int64_t* out_offsets_dev, const MergeBlock* blocks,
                                int32_t num_blocks, int64_t expected_pairs, bool scaled, float scale,
                                hipStream_t stream) {
  if (num <= 0 || num_blocks <= 0) return hipSuccess;
  const dim3 grid((unsigned)num_blocks);
  const int sc = scaled ? 1 : 0;
  // one wavefront per payload in a workgroup of eight, if the pairs a range can expect fit its accumulator
  const bool few = num <= 8 && num_old <= 8 && expected_pairs <= kMergeCapSmall;
  if (old) {  // dense becomes the sum (it holds the sum of `old` now)
    if (few)
      hipLaunchKernelGGL((merge_regions_kernel<true, 512>), grid, dim3(512), 0, stream, dense, p, num, *old, num_old,
                         out_offsets_dev, blocks, scale, sc);
    else
      hipLaunchKernelGGL((merge_regions_kernel<true, 1024>), grid, dim3(1024), 0, stream, dense, p, num, *old, num_old,
                         out_offsets_dev, blocks, scale, sc);
  } else {
    if (few)
      hipLaunchKernelGGL((merge_regions_kernel<false, 512>), grid, dim3(512), 0, stream, dense, p, num, p, 0,
                         out_offsets_dev, blocks, scale, sc);
    else
      hipLaunchKernelGGL((merge_regions_kernel<false, 1024>), grid, dim3(1024), 0, stream, dense, p, num, p, 0,
                         out_offsets_dev, blocks, scale, sc);
  }
  return hipGetLastError();
}

static void launch_locate_parts(const RegionPayloads& p, int32_t num, const int64_t* out_offsets_dev,
                                const MergeBlock* parts, int32_t num_parts, int2* found, hipStream_t stream) {
  const int64_t waves = ceil_div(num_parts, 7) * num;  // seven parts of one payload per wavefront
  hipLaunchKernelGGL(locate_parts_kernel, dim3((unsigned)ceil_div(waves, kFlatThreads / 64)), dim3(kFlatThreads), 0,
                     stream, p, num, out_offsets_dev, parts, num_parts, found);
}

hipError_t launch_merge_parts(float* dense, const RegionPayloads& p, int32_t num, const int64_t* out_offsets_dev,
                              const MergeBlock* parts, int32_t num_parts, void* found, bool replace, bool scaled,
                              float scale, hipStream_t stream) {
  if (num <= 0 || num_parts <= 0) return hipSuccess;
  launch_locate_parts(p, num, out_offsets_dev, parts, num_parts, static_cast<int2*>(found), stream);
  static int compute_units = 0;  // one workgroup of this kernel fits a compute unit
  if (compute_units <= 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&compute_units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || compute_units <= 0)
      compute_units = 256;
  }
  const int grid = num_parts < compute_units ? num_parts : compute_units;
  if (replace)
    hipLaunchKernelGGL(merge_parts_kernel<true>, dim3((unsigned)grid), dim3(kPartThreads), 0, stream, dense, p, num,
                       out_offsets_dev, parts, num_parts, static_cast<const int2*>(found), scale, scaled ? 1 : 0);
  else
    hipLaunchKernelGGL(merge_parts_kernel<false>, dim3((unsigned)grid), dim3(kPartThreads), 0, stream, dense, p, num,
                       out_offsets_dev, parts, num_parts, static_cast<const int2*>(found), scale, scaled ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_clear_parts(float* dense, const RegionPayloads& p, int32_t num, const int64_t* out_offsets_dev,
                              const MergeBlock* parts, int32_t num_parts, void* found, hipStream_t stream) {
  if (num <= 0 || num_parts <= 0) return hipSuccess;
  launch_locate_parts(p, num, out_offsets_dev, parts, num_parts, static_cast<int2*>(found), stream);
  hipLaunchKernelGGL(clear_parts_kernel, dim3((unsigned)num_parts), dim3(kPartClearThreads), 0, stream, dense, p, num,
                     out_offsets_dev, parts, static_cast<const int2*>(found));
  return hipGetLastError();
}

}  // namespace dgc
