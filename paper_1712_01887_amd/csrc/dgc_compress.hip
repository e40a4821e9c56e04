// HIP kernels of the DGC hot path for gfx950 (wave64, CDNA4).
//
// The path is memory-bound: one streaming pass reads g, u, v and writes u, v
// (20 bytes per element); everything else touches a sample or the sparse
// payload only.  No kernel here is a contraction, so no MFMA is used.
//
// Arithmetic contract (shared with nothing, stated for the reader): binary32,
// one rounding per operation, in this order
//     gs = g * scale;  t = m * u;  u' = t + gs;  v' = v + u'          (vanilla)
//     gs = g * scale;  s = u + gs; u' = m * s;   w = v + u'; v' = w + gs  (Nesterov)
// The file must be compiled with -ffp-contract=off so that no pair of these is
// fused; the threshold pass and the streaming pass evaluate v' with the same
// inline function, which makes the sampled threshold an exact member of the
// values the streaming pass later compares against it.

#include "dgc_internal.h"

namespace dgc {
namespace {

// ---------------------------------------------------------------------------
// Momentum correction (paper: equation 7; Algorithm 3 / Algorithm 4 update lines)
// ---------------------------------------------------------------------------
__device__ __forceinline__ void momentum_update(float g, float u, float v, float m, float scale,
                                                bool nesterov, float& u1, float& v1) {
  const float gs = g * scale;
  if (!nesterov) {
    const float t = m * u;
    u1 = t + gs;
    v1 = v + u1;
  } else {
    const float s = u + gs;
    u1 = m * s;
    const float w = v + u1;
    v1 = w + gs;
  }
}

// Zero fill of small pieces of the workspace (a kernel rather than a memset: the calls of
// the library may be captured into a HIP graph).
__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t* __restrict__ p, size_t words) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

// ---------------------------------------------------------------------------
// Clipping norm (paper: Section 3.2 "Local Gradient Clipping"; Appendix C eq. 12)
// ---------------------------------------------------------------------------
// Every workgroup accumulates squares in binary64 over a grid-stride range and stores
// one partial sum; nothing else.  The partials are added up, in a fixed order, by the
// kernel that runs next (every workgroup of the threshold selection does it for itself),
// so that the result does not depend on scheduling and no workgroup has to wait for
// another: a version in which the last workgroup to arrive finished the sum needed two
// chained device-scope atomics per workgroup and ran 6 us longer (52 against 46 us on
// 66 M elements).
__global__ __launch_bounds__(kNormThreads) void norm_kernel(const float* __restrict__ g, int64_t n,
                                                            double* __restrict__ partials) {
  __shared__ double red[kNormThreads / 64];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t nvec = n >> 2;
  const float4* __restrict__ g4 = reinterpret_cast<const float4*>(g);
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  const int64_t stride = (int64_t)gridDim.x * kNormThreads;
  int64_t i = (int64_t)blockIdx.x * kNormThreads + tid;
  // four independent 16-byte loads in flight per thread; ordinary (cached) loads, because
  // the streaming pass reads g again right after this kernel
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    const float4 x0 = g4[i];
    const float4 x1 = g4[i + stride];
    const float4 x2 = g4[i + 2 * stride];
    const float4 x3 = g4[i + 3 * stride];
    a0 += (double)x0.x * (double)x0.x;
    a1 += (double)x0.y * (double)x0.y;
    a2 += (double)x0.z * (double)x0.z;
    a3 += (double)x0.w * (double)x0.w;
    a0 += (double)x1.x * (double)x1.x;
    a1 += (double)x1.y * (double)x1.y;
    a2 += (double)x1.z * (double)x1.z;
    a3 += (double)x1.w * (double)x1.w;
    a0 += (double)x2.x * (double)x2.x;
    a1 += (double)x2.y * (double)x2.y;
    a2 += (double)x2.z * (double)x2.z;
    a3 += (double)x2.w * (double)x2.w;
    a0 += (double)x3.x * (double)x3.x;
    a1 += (double)x3.y * (double)x3.y;
    a2 += (double)x3.z * (double)x3.z;
    a3 += (double)x3.w * (double)x3.w;
  }
  for (; i < nvec; i += stride) {
    const float4 x = g4[i];
    a0 += (double)x.x * (double)x.x;
    a1 += (double)x.y * (double)x.y;
    a2 += (double)x.z * (double)x.z;
    a3 += (double)x.w * (double)x.w;
  }
  if (blockIdx.x == 0 && tid < (int)(n & 3)) {
    const double x = (double)g[(nvec << 2) + tid];
    a0 += x * x;
  }
  double acc = (a0 + a1) + (a2 + a3);
  for (int d = 32; d >= 1; d >>= 1) acc += __shfl_down(acc, d);
  if (lane == 0) red[wave] = acc;
  __syncthreads();
  if (tid == 0) {
    double s = 0.0;
    for (int w = 0; w < kNormThreads / 64; ++w) s += red[w];
    partials[blockIdx.x] = s;
  }
}

// ---------------------------------------------------------------------------
// Sampled threshold (paper: Section 5 -- top-k on a sample estimates the
// threshold of the whole tensor; Algorithm 3 "thr <- s% of |V[j]|")
// ---------------------------------------------------------------------------
// 32-bit xorshift-multiply finaliser; a bijection on 32-bit words.
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

struct Candidates {
  const float* g;
  const float* u;
  const float* v;
  int64_t offset;
  uint32_t key;      // folded (seed, iteration, tensor)
  uint32_t nblocks;
  int32_t block_shift;
  int32_t exact;
  float m, scale;
  bool nesterov;

  // Position (relative to the tensor) of candidate p.
  __device__ __forceinline__ int64_t position(int32_t p) const {
    if (exact) return p;
    const uint32_t draw = (uint32_t)p >> block_shift;
    const uint32_t r = mix32(key ^ (draw * 0x9E3779B1u));
    const uint32_t blk = __umulhi(r, nblocks);
    return ((int64_t)blk << block_shift) + (p & ((1 << block_shift) - 1));
  }
};

// One workgroup per tensor finds the candidate key of a given descending rank
// exactly.  Keys are the bit patterns of |v'| (order-isomorphic to the
// magnitudes).  Up to three histogram passes over 11 + 11 + 9 key bits, most
// significant first, narrow the key down; as soon as the bin that holds the
// rank has few enough members they are gathered and ranked directly, which at
// the paper's densities happens after the first pass.
//
// Up to kSelectRegKeys * kSelectThreads candidates live in registers (each
// thread gathers its own once and keeps them); a larger candidate set (exact
// selection on a big tensor) is re-evaluated from g, u, v in every pass.
struct SelectShared {
  double red[kSelectThreads / 64];
  float scale;
  uint32_t hist[kSelectBins];
  uint32_t wave_tot[kSelectThreads / 64];
  uint32_t surv[kSelectThreads];
  uint32_t sel[3];
  uint32_t surv_n, result;
};

// After a histogram pass: the bin that holds descending rank `rank`, how many
// candidates lie above it, and how many it holds.  Every thread returns the same.
// `sel` is three words of LDS, `wave_tot` one word per wavefront.
template <int THREADS>
__device__ __forceinline__ void find_bin(const uint32_t* hist, uint32_t* wave_tot, uint32_t* sel, int tid,
                                         uint32_t rank, uint32_t& bin, uint32_t& above_out,
                                         uint32_t& members) {
  constexpr int PER = kSelectBins / THREADS;  // consecutive bins owned by a thread
  const int lane = tid & 63;
  const int wave = tid >> 6;
  uint32_t h[PER];
  uint32_t local = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    h[i] = hist[PER * tid + i];
    local += h[i];
  }
  uint32_t incl = local;  // suffix sum: this thread's bins and everything above
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_down(incl, d);
    if (lane + d < 64) incl += t;
  }
  if (lane == 0) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t run = incl - local;  // candidates above this thread's bins
  for (int w = wave + 1; w < THREADS / 64; ++w) run += wave_tot[w];
#pragma unroll
  for (int i = PER - 1; i >= 0; --i) {
    if (run <= rank && rank < run + h[i]) {
      sel[0] = PER * tid + i;
      sel[1] = run;
      sel[2] = h[i];
    }
    run += h[i];
  }
  __syncthreads();
  bin = sel[0];
  above_out = sel[1];
  members = sel[2];
}

// The `m` <= kSelectThreads keys in sh.surv: the one of descending rank `rank`.  (Splitting the
// comparisons of one key over several threads, with the partial counts added in LDS, was measured:
// no faster for the 100 to 200 keys that get here.)
__device__ __forceinline__ uint32_t rank_directly(SelectShared& sh, int tid, uint32_t m, uint32_t rank) {
  if (tid < (int)m) {
    const uint32_t x = sh.surv[tid];
    uint32_t greater = 0, equal = 0;
    for (uint32_t i = 0; i < m; ++i) {
      const uint32_t y = sh.surv[i];
      greater += y > x;
      equal += y == x;
    }
    if (greater <= rank && rank < greater + equal) sh.result = x;  // ties write the same value
  }
  __syncthreads();
  return sh.result;
}

// Key of descending rank `rank` among the keys a workgroup holds in registers (NKEYS per
// thread), ignoring empty slots (kNoKey) and keys below `floor_key`; the caller
// guarantees that more than `rank` keys are considered.  Every thread returns the same.
constexpr uint32_t kNoKey = 0xFFFFFFFFu;  // real keys have the sign bit clear

template <int NKEYS>
__device__ __forceinline__ uint32_t select_in_registers(SelectShared& sh, const uint32_t (&key)[NKEYS],
                                                        uint32_t floor_key, uint32_t rank, int tid) {
  uint32_t prefix = 0;
  int consumed = 0;  // key bits fixed so far (below the sign bit)
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int bits = pass == 2 ? 9 : 11;
    const int shift = 31 - consumed - bits;
    const uint32_t digit_mask = (1u << bits) - 1u;
    for (int i = tid; i < kSelectBins; i += kSelectThreads) sh.hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NKEYS; ++i) {
      const uint32_t k = key[i];
      if (k != kNoKey && k >= floor_key && (pass == 0 || (k >> (shift + bits)) == prefix))
        atomicAdd(&sh.hist[(k >> shift) & digit_mask], 1u);
    }
    __syncthreads();
    uint32_t bin, above, members;
    find_bin<kSelectThreads>(sh.hist, sh.wave_tot, sh.sel, tid, rank, bin, above, members);
    prefix = (prefix << bits) | bin;
    rank -= above;
    consumed += bits;
    if (consumed == 31) return prefix;
    if (members <= (uint32_t)kSelectDirect) {
      if (tid == 0) sh.surv_n = 0;
      __syncthreads();
      const int low = 31 - consumed;  // key bits not yet fixed
#pragma unroll
      for (int i = 0; i < NKEYS; ++i) {
        const uint32_t k = key[i];
        if (k != kNoKey && k >= floor_key && (k >> low) == prefix) sh.surv[atomicAdd(&sh.surv_n, 1u)] = k;
      }
      __syncthreads();
      return rank_directly(sh, tid, members, rank);
    }
  }
  return prefix;
}

template <bool NESTEROV>
__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a) {
  __shared__ SelectShared sh;
  const int tid = threadIdx.x;
  const int j = blockIdx.x;
  const TensorPlan plan = a.plans[j];

  // Clipping scale (paper: Appendix C equation 12).  With clipping on, the norm kernel
  // has left its partial sums; every workgroup adds them in the same fixed order (thread
  // t takes partials t, t + 1024, ...; lanes, then wavefronts, in order), so all of them
  // get the same bits, and the first one also files the result for the streaming pass
  // and for the diagnostics.
  float scale = a.scale_const;
  if (a.scale_from_state) {
    double s = 0.0;
    for (int i = tid; i < a.num_partials; i += kSelectThreads) s += a.partials[i];
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_down(s, d);
    if ((tid & 63) == 0) sh.red[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
      double total = 0.0;
      for (int w = 0; w < kSelectThreads / 64; ++w) total += sh.red[w];
      const double norm = sqrt(total);
      float sc = 1.0f;
      if (norm > a.thr_local) sc = (float)(a.thr_local / norm);
      if (a.scale_override == a.scale_override) sc = a.scale_override;
      sh.scale = sc;
      if (j == 0) {
        uint32_t flags = 0;
        if (!(norm <= 1.79769313486231570e308)) flags |= DGC_DIAG_NONFINITE;  // NaN or infinity
        a.state->norm = norm;
        a.state->scale = sc;
        a.state->flags = flags;
      }
    }
    __syncthreads();
    scale = sh.scale;
  } else if (tid == 0 && j == 0) {  // no clipping: start a clean record
    a.state->norm = __longlong_as_double(0x7FF8000000000000ll);
    a.state->scale = a.scale_const;
    a.state->flags = 0;
  }
  // Tiles that lie wholly inside this tensor get the threshold written into the per-tile
  // table, which is all the streaming pass looks at on its fast path.
  const int64_t tile_first = (plan.offset + kWaveTile - 1) / kWaveTile;
  const int64_t tile_end = (plan.offset + plan.n) / kWaveTile;
  if (plan.rank >= plan.count) {  // the strict comparison then passes everything
    if (tid == 0) {
      a.thr[j] = -1.0f;
      if (a.out_thr) a.out_thr[j] = -1.0f;
    }
    for (int64_t t = tile_first + tid; t < tile_end; t += kSelectThreads) a.tile_thr[t] = -1.0f;
    return;
  }

  Candidates c;
  c.g = a.g;
  c.u = a.u;
  c.v = a.v;
  c.offset = plan.offset;
  c.nblocks = plan.nblocks;
  c.block_shift = a.block_shift;
  c.exact = plan.exact;
  c.m = a.momentum;
  c.scale = scale;
  c.nesterov = NESTEROV;
  {
    uint32_t h = mix32(a.seed_lo ^ 0x9E3779B9u);
    h = mix32(h ^ a.seed_hi);
    h = mix32(h ^ a.iter_lo);
    h = mix32(h ^ a.iter_hi);
    c.key = mix32(h ^ (uint32_t)j);
  }

  const int32_t count = plan.count;
  uint32_t prefix = 0;
  uint32_t rank = (uint32_t)plan.rank;
  uint32_t thr_bits = 0;

  if (count <= kSelectRegKeys * kSelectThreads) {
    // ---- candidates in registers ------------------------------------------------
    uint32_t key[kSelectRegKeys];
#pragma unroll
    for (int i = 0; i < kSelectRegKeys; ++i) key[i] = kNoKey;
    // The gather is written without branches around the loads and without conditional stores into
    // key[]: a candidate beyond the count reads candidate 0 instead and its key is replaced by the
    // empty mark afterwards.  (With `if (p < count)` around them the compiler copied the whole
    // register array at every such branch: some 400 moves per thread in a kernel that spends as
    // much time issuing instructions as waiting for memory, 16 wavefronts sharing four SIMDs.)
    if (!plan.exact && a.block_shift >= 2) {
      // Sampled blocks of at least four elements: a thread takes four consecutive elements of a
      // drawn block at a time (one 16-byte load per array; a block starts at a multiple of its size
      // from the tensor's start, which need not be 16-byte aligned: dword-aligned vector loads), so
      // that the draw's position is worked out once per four candidates.  Which thread holds which
      // candidate does not matter: the rank is taken over all of them.
      typedef float vec4u __attribute__((ext_vector_type(4), aligned(4)));
      constexpr int kQuads = kSelectRegKeys / 4;       // per thread
      constexpr int kQuadsInFlight = 4;
      const int32_t quads = count >> 2;                // blocks are whole multiples of four elements
      const int qshift = a.block_shift - 2;            // log2(quads per block)
#pragma unroll
      for (int r = 0; r < kQuads / kQuadsInFlight; ++r) {
        if (r == 0 || r * kQuadsInFlight * kSelectThreads < quads) {  // uniform
          vec4u gg[kQuadsInFlight], uu[kQuadsInFlight], vv[kQuadsInFlight];
#pragma unroll
          for (int q = 0; q < kQuadsInFlight; ++q) {
            const int32_t qd = tid + (r * kQuadsInFlight + q) * kSelectThreads;
            const int32_t qq = qd < quads ? qd : 0;
            const int64_t e = c.offset + c.position((qq >> qshift) << a.block_shift) + ((qq & ((1 << qshift) - 1)) << 2);
            gg[q] = *reinterpret_cast<const vec4u*>(c.g + e);
            uu[q] = *reinterpret_cast<const vec4u*>(c.u + e);
            vv[q] = *reinterpret_cast<const vec4u*>(c.v + e);
          }
#pragma unroll
          for (int q = 0; q < kQuadsInFlight; ++q) {
            const bool ok = tid + (r * kQuadsInFlight + q) * kSelectThreads < quads;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              float u1, v1;
              momentum_update(gg[q][k], uu[q][k], vv[q][k], c.m, c.scale, NESTEROV, u1, v1);
              key[4 * (r * kQuadsInFlight + q) + k] = ok ? (__float_as_uint(v1) & 0x7FFFFFFFu) : kNoKey;
            }
          }
        }
      }
    } else {
      // one candidate per load: kSelectInFlight of them are loaded before any is used
#pragma unroll
      for (int r = 0; r < kSelectRegKeys / kSelectInFlight; ++r) {
        if (r == 0 || r * kSelectInFlight * kSelectThreads < count) {  // uniform
          float gg[kSelectInFlight], uu[kSelectInFlight], vv[kSelectInFlight];
#pragma unroll
          for (int q = 0; q < kSelectInFlight; ++q) {
            const int32_t p = tid + (r * kSelectInFlight + q) * kSelectThreads;
            const int64_t e = c.offset + c.position(p < count ? p : 0);
            gg[q] = c.g[e];
            uu[q] = c.u[e];
            vv[q] = c.v[e];
          }
#pragma unroll
          for (int q = 0; q < kSelectInFlight; ++q) {
            const bool ok = tid + (r * kSelectInFlight + q) * kSelectThreads < count;
            float u1, v1;
            momentum_update(gg[q], uu[q], vv[q], c.m, c.scale, NESTEROV, u1, v1);
            key[r * kSelectInFlight + q] = ok ? (__float_as_uint(v1) & 0x7FFFFFFFu) : kNoKey;
          }
        }
      }
    }
    // Gradients of one tensor share a few exponents, so a histogram over the leading key
    // bits of all candidates piles tens of thousands of LDS atomics on a handful of bins,
    // and every histogram pass costs half a dozen barriers of 1024 threads (ranking 32 Ki
    // keys that way took 20 us, against 3 us this way).  At the paper's densities the
    // rank r is a few dozen, and a floor below which no key matters is cheap to get: if
    // every one of the 16 wavefronts names the t-th largest of its threads' largest
    // keys, 16 t > r, then the smallest of the 16 answers has more than r keys at or
    // above it.  What lies at or above that floor (a few times r keys) is listed in LDS
    // and ranked by direct counting.  Anything that does not fit this pattern takes the
    // histogram passes.
    constexpr int kWaves = kSelectThreads / 64;
    const uint32_t t_rounds = rank / kWaves + 1;  // kWaves * t_rounds > rank
    bool done = false;
    if (count > 2 * kSelectThreads && t_rounds <= (uint32_t)kSelectFloorRounds) {
      const int lane = tid & 63;
      uint32_t top = 0;  // this thread's largest key (every thread has keys: count > 2048)
#pragma unroll
      for (int i = 0; i < kSelectRegKeys; ++i)
        if (key[i] != kNoKey) top = key[i] > top ? key[i] : top;
      uint32_t tth = 0;
      for (uint32_t round = 0; round < t_rounds; ++round) {
        uint32_t m = top;
        for (int d = 32; d >= 1; d >>= 1) {
          const uint32_t o = __shfl_xor(m, d);
          m = o > m ? o : m;
        }
        tth = m;
        const unsigned long long holders = __ballot(top == m);
        if (lane == __ffsll((long long)holders) - 1) top = 0;  // one holder of the maximum steps down
      }
      if (lane == 0) sh.wave_tot[tid >> 6] = tth;
      if (tid == 0) sh.surv_n = 0;
      __syncthreads();
      uint32_t floor_key = sh.wave_tot[0];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) floor_key = sh.wave_tot[w] < floor_key ? sh.wave_tot[w] : floor_key;
#pragma unroll
      for (int i = 0; i < kSelectRegKeys; ++i)
        if (key[i] != kNoKey && key[i] >= floor_key) {
          const uint32_t pos = atomicAdd(&sh.surv_n, 1u);
          if (pos < (uint32_t)kSelectThreads) sh.surv[pos] = key[i];
        }
      __syncthreads();
      const uint32_t listed = sh.surv_n;
      if (listed <= (uint32_t)kSelectThreads) {
        thr_bits = rank_directly(sh, tid, listed, rank);
        done = true;
      }
      __syncthreads();
    }
    if (!done) thr_bits = select_in_registers<kSelectRegKeys>(sh, key, 0u, rank, tid);
  } else {
    // ---- candidates re-evaluated in every pass -----------------------------------
    int consumed = 0;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int bits = pass == 2 ? 9 : 11;
      const int shift = 31 - consumed - bits;
      const uint32_t digit_mask = (1u << bits) - 1u;
      for (int i = tid; i < kSelectBins; i += kSelectThreads) sh.hist[i] = 0;
      __syncthreads();
      for (int32_t p0 = tid; p0 < count; p0 += kSelectInFlight * kSelectThreads) {
        float gg[kSelectInFlight], uu[kSelectInFlight], vv[kSelectInFlight];
#pragma unroll
        for (int q = 0; q < kSelectInFlight; ++q) {
          const int32_t p = p0 + q * kSelectThreads;
          gg[q] = uu[q] = vv[q] = 0.0f;
          if (p < count) {
            const int64_t e = c.offset + c.position(p);
            gg[q] = c.g[e];
            uu[q] = c.u[e];
            vv[q] = c.v[e];
          }
        }
#pragma unroll
        for (int q = 0; q < kSelectInFlight; ++q) {
          const int32_t p = p0 + q * kSelectThreads;
          if (p < count) {
            float u1, v1;
            momentum_update(gg[q], uu[q], vv[q], c.m, c.scale, c.nesterov, u1, v1);
            const uint32_t k = __float_as_uint(v1) & 0x7FFFFFFFu;
            if (pass == 0 || (k >> (shift + bits)) == prefix)
              atomicAdd(&sh.hist[(k >> shift) & digit_mask], 1u);
          }
        }
      }
      __syncthreads();
      uint32_t bin, above, members;
      find_bin<kSelectThreads>(sh.hist, sh.wave_tot, sh.sel, tid, rank, bin, above, members);
      prefix = (prefix << bits) | bin;
      rank -= above;
      consumed += bits;
    }
    thr_bits = prefix;
  }
  const float thr = __uint_as_float(thr_bits);
  if (tid == 0) {
    a.thr[j] = thr;
    if (a.out_thr) a.out_thr[j] = thr;
  }
  for (int64_t t = tile_first + tid; t < tile_end; t += kSelectThreads) a.tile_thr[t] = thr;
}

// ---------------------------------------------------------------------------
// Streaming pass: momentum correction + mask
// (paper: Algorithm 3, the U and V update lines and the Mask line)
// ---------------------------------------------------------------------------
// A wavefront owns kWaveTile consecutive elements, read as kStreamUnroll rounds
// of one 16-byte vector per lane.  g, u and v are touched exactly once per
// iteration, so they are loaded and stored with the non-temporal hint.  The
// pass writes the pre-mask u', v' and one bit per element (|v'| > thr) and
// nothing else: no atomics, no scattered stores, nothing that depends on how
// many elements pass.  The emit pass below turns the bits into the payload and
// applies the mask to u and v.
//
// Mask layout: lane l of the wavefront that owns tile t stores a 16-bit word at
// mask[t * 64 + l]; bit q = r * 4 + c of it belongs to element
// t * kWaveTile + r * 256 + l * 4 + c.
//
// Tiles that lie inside one tensor (all but a few hundred) compare against one
// threshold.  Tiles that straddle tensors, and the ragged last tile, look up each
// element's tensor.
typedef float vec4 __attribute__((ext_vector_type(4)));

static_assert(kStreamUnroll >= 1 && kStreamUnroll <= 4, "mask words hold at most 16 bits per lane");

__device__ __forceinline__ int64_t tile_element(int64_t tile, int lane, int q) {
  return tile * kWaveTile + (q >> 2) * 256 + lane * 4 + (q & 3);
}

// Mask bits of a lane's sixteen elements in a tile that is not wholly inside one tensor.  `zq`
// points at the lane's column of the wavefront's v' in LDS (element q of the lane at zq[q * 64]).
// `j0` is the tensor of the tile's first element.  The starts of the tensors after it are
// fetched 64 at a time, one per lane (those inside the tile form a prefix of the lanes because
// the offsets ascend) and handed round with readlane, so that the tile is walked segment by
// segment, each with its tensor's threshold: one round of loads per 64 tensors, however many
// tensors share the tile.  A few hundred tiles of a launch come here; the loops are kept rolled
// and the values in LDS so that this path does not set the register allocation of the whole
// kernel (unrolled over register-held values it cost the streaming pass a wavefront per SIMD).
__device__ __forceinline__ uint32_t mixed_tile_mask(const StreamArgs& a, int64_t base, int lane, int32_t j0,
                                                    const float* zq) {
  constexpr int kElems = 4 * kStreamUnroll;
  const int32_t tile_end = base + kWaveTile <= a.n ? kWaveTile : (int32_t)(a.n - base);
  const int32_t lane4 = lane * 4;
  uint32_t cand = 0;
  int32_t seg_lo = 0;            // the segment being closed starts here (relative to the tile)
  float seg_thr = a.thr[j0];     // ... and belongs to a tensor with this threshold
  for (int32_t jb = j0 + 1; jb < a.num_tensors; jb += 64) {
    const int32_t jj = jb + lane;
    int32_t rel = kWaveTile;  // start of tensor jj relative to the tile, kWaveTile = not inside it
    float t = 0.0f;
    if (jj < a.num_tensors) {
      const int64_t o = a.offsets[jj];
      if (o < base + tile_end) {
        rel = o > base ? (int32_t)(o - base) : 0;
        t = a.thr[jj];
      }
    }
    const int cnt = __popcll(__ballot(rel < kWaveTile));
    for (int i = 0; i < cnt; ++i) {
      const int32_t seg_hi = __builtin_amdgcn_readlane(rel, i);
#pragma unroll 1
      for (int q = 0; q < kElems; ++q) {
        const int32_t p = (q >> 2) * 256 + lane4 + (q & 3);
        if (p >= seg_lo && p < seg_hi && fabsf(zq[q * 64]) > seg_thr) cand |= 1u << q;
      }
      seg_lo = seg_hi;
      seg_thr = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int32_t)__float_as_uint(t), i));
    }
    if (cnt < 64) break;
  }
#pragma unroll 1
  for (int q = 0; q < kElems; ++q) {
    const int32_t p = (q >> 2) * 256 + lane4 + (q & 3);
    if (p >= seg_lo && p < tile_end && fabsf(zq[q * 64]) > seg_thr) cand |= 1u << q;
  }
  return cand;
}

// NESTEROV and SCALED are compile-time so that the sixteen updates of a lane are straight
// code: SCALED = false is the case scale == 1 exactly (no clipping), where g * 1.0f == g
// bit for bit and the multiplication is left out.  The kernel is memory-bound but a
// wave64 instruction occupies its SIMD for four cycles, so instructions saved per tile
// show in the run time.
//
// Every tile, whatever it holds, asks for its data first and all at once, then learns from
// ONE table word (a scalar load that depends on nothing) whether it lies wholly inside one
// tensor, in which case the word is its threshold, or not (NaN), in which case it fetches
// the tensor starts and thresholds it needs in one more round of loads.  A tile that took
// several dependent rounds, as a first version did, held up the end of the whole launch
// whenever it was dispatched late: 5 us of 88 on the 161-tensor set.
//
// STAGED (densities of the warm-up epochs, paper: Section 4): with a quarter of the elements
// selected, an emit pass that comes back for them reads every sector of v and rewrites
// every sector of u and v a second time.  Here a tile that lies wholly inside one tensor
// applies the mask to u and v before it stores them, and parks the selected v' (and u',
// which a full payload region needs to put back) in the tile's 1024 slots of a staging
// array, in index order: the emit pass then copies from there and touches u and v only
// where a region overflows.  An element's position among the tile's selected ones is
// rows before it + bits of its row in lower lanes (from the votes) + lower bits of its
// nibble.  Tiles shared between tensors are left to the emit pass as before.
//
// SLOTTED (densities up to 0.5 %, i.e. the 99.9 % sparsity the method runs at after its
// warm-up): a tile holds one or two selected elements, seldom more than a handful.  A tile
// that lies wholly inside one tensor and selects at most kSlotsPerTile elements parks their
// index, v' and u' (which a full payload region needs to put back) in a record that takes the
// place of the tile's mask words, in index order, and stores u and v masked: the emit pass copies
// from the record and neither decodes a mask word nor reads or rewrites u and v for such a tile.  Tiles with more selected elements, and tiles shared between tensors, are
// left to the emit pass as in the plain case (u', v' unmasked, mask bits set).
enum StreamMode : int { kStreamPlain = 0, kStreamStaged = 1, kStreamSlotted = 2 };

template <bool NESTEROV, bool SCALED, int MODE>
__global__ __launch_bounds__(kStreamThreads) void stream_kernel(StreamArgs a) {
  constexpr bool STAGED = MODE == kStreamStaged;
  __shared__ float mixed_z[kStreamWaves][4 * kStreamUnroll][64];  // for tiles shared between tensors only
  constexpr int U = kStreamUnroll;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: table reads go scalar
  const int64_t tile = (int64_t)blockIdx.x * kStreamWaves + wave;
  const int64_t base = tile * kWaveTile;
  if (base >= a.n) return;
  const float scale = SCALED ? (a.scale_from_state ? a.state->scale : a.scale_const) : 1.0f;
  const bool full = base + kWaveTile <= a.n;
  const vec4* __restrict__ g4 = reinterpret_cast<const vec4*>(a.g + base) + lane;
  vec4* __restrict__ u4 = reinterpret_cast<vec4*>(a.u + base) + lane;
  vec4* __restrict__ v4 = reinterpret_cast<vec4*>(a.v + base) + lane;
  vec4 x[U], y[U], z[U];
  if (full) {
#pragma unroll
    for (int r = 0; r < U; ++r) {
      x[r] = __builtin_nontemporal_load(g4 + r * 64);
      y[r] = __builtin_nontemporal_load(u4 + r * 64);
      z[r] = __builtin_nontemporal_load(v4 + r * 64);
    }
  } else {  // the ragged last tile: element by element, zero beyond the end
#pragma unroll
    for (int r = 0; r < U; ++r) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int64_t e = base + r * 256 + lane * 4 + c;
        const bool in = e < a.n;
        x[r][c] = in ? a.g[e] : 0.0f;
        y[r][c] = in ? a.u[e] : 0.0f;
        z[r][c] = in ? a.v[e] : 0.0f;
      }
    }
  }
  const float thr = a.tile_thr[tile];
  const int32_t j0 = (int32_t)(a.tile_info[tile] & ~kTileMixed);

  const float m = a.momentum;
#pragma unroll
  for (int r = 0; r < U; ++r) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float gs = SCALED ? x[r][c] * scale : x[r][c];
      float u1, v1;
      if (!NESTEROV) {
        const float t = m * y[r][c];
        u1 = t + gs;
        v1 = z[r][c] + u1;
      } else {
        const float s = y[r][c] + gs;
        u1 = m * s;
        const float w = z[r][c] + u1;
        v1 = w + gs;
      }
      y[r][c] = u1;
      z[r][c] = v1;
    }
  }
  if (STAGED && thr == thr) {  // wholly inside one tensor (and so a whole tile)
    uint32_t cand = 0;
#pragma unroll
    for (int q = 0; q < 4 * U; ++q)
      if (fabsf(z[q >> 2][q & 3]) > thr) cand |= 1u << q;
    float* __restrict__ stage_v = a.stage_v + base;
    float* __restrict__ stage_u = a.stage_u ? a.stage_u + base : nullptr;
    const bool clear_u = a.factor_masking != 0;
    int row_base = 0;
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const uint32_t nib = (cand >> (4 * r)) & 0xFu;
      int lower = 0, row = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const unsigned long long vote = __ballot((nib >> c) & 1u);
        lower += (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vote >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vote, 0u));
        row += __popcll(vote);
      }
      int pos = row_base + lower;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if ((nib >> c) & 1u) {
          stage_v[pos] = z[r][c];
          if (stage_u) stage_u[pos] = y[r][c];
          z[r][c] = 0.0f;
          if (clear_u) y[r][c] = 0.0f;
          ++pos;
        }
      }
      row_base += row;
    }
#pragma unroll
    for (int r = 0; r < U; ++r) {
      __builtin_nontemporal_store(y[r], u4 + r * 64);
      __builtin_nontemporal_store(z[r], v4 + r * 64);
    }
    a.mask[tile * 64 + lane] = (uint16_t)cand;
    if (lane == 0) a.tile_count[tile] = (uint32_t)row_base;
    return;
  }
  if (MODE == kStreamSlotted && thr == thr) {  // wholly inside one tensor (and so a whole tile)
    uint32_t cand = 0;
#pragma unroll
    for (int q = 0; q < 4 * U; ++q)
      if (fabsf(z[q >> 2][q & 3]) > thr) cand |= 1u << q;
    // A row (one 16-byte vector per lane) without a selected element, which is most rows, goes out
    // at once: how long a wavefront holds on to its data after the loads have come back is what
    // the pass's throughput hangs on, and the bookkeeping below is long enough to show.
    unsigned long long row_holders[U];
#pragma unroll
    for (int r = 0; r < U; ++r) {
      row_holders[r] = __ballot(((cand >> (4 * r)) & 0xFu) != 0);
      if (row_holders[r] == 0) {
        __builtin_nontemporal_store(y[r], u4 + r * 64);
        __builtin_nontemporal_store(z[r], v4 + r * 64);
      }
    }
    int total = __popc(cand);
    for (int d = 32; d >= 1; d >>= 1) total += __shfl_xor(total, d);
    if (total > 0 && total <= kSlotsPerTile) {  // uniform
      // The few selected elements are taken row by row, one at a time, everything about them in
      // scalar registers (which lane, which of its four elements): the values are read from that
      // lane, and the tile's record is put together across lanes 0 .. 31 (index of element p in
      // lane p, its v' in lane 8 + p, its u' in lane 16 + p) and stored whole, as one 128-byte
      // line.  (Scattered 4-byte stores from inside this pass cost 26 us on a 122 M-element set:
      // every one is a partial write of a line; a record array of its own with a line for every
      // tile that has a record, a stream of stores with holes in it, 7 us.)
      const bool clear_u = a.factor_masking != 0;
      int record = 0;
      int pos = 0;
#pragma unroll
      for (int r = 0; r < U; ++r) {
        unsigned long long holders = row_holders[r];
        if (holders == 0) continue;
        const uint32_t nib = (cand >> (4 * r)) & 0xFu;
        do {
          const int l = __ffsll((long long)holders) - 1;
          holders &= holders - 1;
          uint32_t w = (uint32_t)__builtin_amdgcn_readlane((int)nib, l);
          do {
            const int c = __ffs(w) - 1;  // uniform: the component is picked in every lane, then read from lane l
            w &= w - 1;
            const float zc = c == 0 ? z[r][0] : c == 1 ? z[r][1] : c == 2 ? z[r][2] : z[r][3];
            const float yc = c == 0 ? y[r][0] : c == 1 ? y[r][1] : c == 2 ? y[r][2] : y[r][3];
            const int zv = __builtin_amdgcn_readlane(__float_as_int(zc), l);
            const int yv = __builtin_amdgcn_readlane(__float_as_int(yc), l);
            const int e = (int32_t)(base + r * 256 + l * 4 + c);
            if (lane == pos) record = e;
            if (lane == kSlotsPerTile + pos) record = zv;
            if (lane == 2 * kSlotsPerTile + pos) record = yv;
            ++pos;
          } while (w);
        } while (holders);
        // the mask applied to this row of u and v
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const bool sel = (nib >> c) & 1u;
          z[r][c] = sel ? 0.0f : z[r][c];
          if (clear_u) y[r][c] = sel ? 0.0f : y[r][c];
        }
      }
      // the record takes the place of the tile's mask words (both are one 128-byte line per tile;
      // the count says which of the two the line holds)
      if (lane < kSlotRecord) reinterpret_cast<int32_t*>(a.mask)[tile * kSlotRecord + lane] = record;
    } else {  // (an empty tile's line is written too: a stream of stores with holes in it runs slower)
      a.mask[tile * 64 + lane] = (uint16_t)cand;
    }
#pragma unroll
    for (int r = 0; r < U; ++r) {
      if (row_holders[r] != 0) {
        __builtin_nontemporal_store(y[r], u4 + r * 64);
        __builtin_nontemporal_store(z[r], v4 + r * 64);
      }
    }
    // (the flag: this line holds mask words although the tile lies inside one tensor -- a count that
    // the re-threshold pass lowers to kSlotsPerTile or less must not make the line pass for a record)
    if (lane == 0) a.tile_count[tile] = (uint32_t)total | (total > kSlotsPerTile ? kTileCountHasMask : 0u);
    return;
  }
  // u' and v' go out first: once stored, u' need not be kept while the mask is worked out
  if (full) {
#pragma unroll
    for (int r = 0; r < U; ++r) {
      __builtin_nontemporal_store(y[r], u4 + r * 64);
      __builtin_nontemporal_store(z[r], v4 + r * 64);
    }
  } else {
#pragma unroll
    for (int r = 0; r < U; ++r) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int64_t e = base + r * 256 + lane * 4 + c;
        if (e < a.n) {
          a.u[e] = y[r][c];
          a.v[e] = z[r][c];
        }
      }
    }
  }
  uint32_t cand = 0;
  if (thr == thr) {  // the whole tile belongs to one tensor
#pragma unroll
    for (int q = 0; q < 4 * U; ++q)
      if (fabsf(z[q >> 2][q & 3]) > thr) cand |= 1u << q;
  } else {
    float* zq = &mixed_z[wave][0][lane];  // this lane's column: written and read by this lane only
#pragma unroll
    for (int q = 0; q < 4 * U; ++q) zq[q * 64] = z[q >> 2][q & 3];
    cand = mixed_tile_mask(a, base, lane, j0, zq);
  }
  a.mask[tile * 64 + lane] = (uint16_t)cand;
  // bits set in the tile, for the index-ordered emit pass (measured: no cost here)
  int bits = __popc(cand);
  for (int d = 32; d >= 1; d >>= 1) bits += __shfl_xor(bits, d);
  if (lane == 0) a.tile_count[tile] = (uint32_t)bits;
}

// Yardstick for the streaming pass: the same traffic (three arrays read, two written,
// non-temporal, one wave tile per wavefront) with next to no arithmetic, no table and no
// mask.  What this kernel reaches on a box is the ceiling the streaming pass can be held
// against besides the nominal HBM peak.  Whole tiles only.
__global__ __launch_bounds__(64) void ceiling_kernel(const float* __restrict__ a, float* __restrict__ b,
                                                     float* __restrict__ c, int64_t tiles) {
  constexpr int U = kStreamUnroll;
  const int lane = threadIdx.x;
  const int64_t tile = blockIdx.x;  // one wavefront per workgroup: the residency is set in wavefronts
  if (tile >= tiles) return;
  const vec4* a4 = reinterpret_cast<const vec4*>(a + tile * kWaveTile) + lane;
  vec4* b4 = reinterpret_cast<vec4*>(b + tile * kWaveTile) + lane;
  vec4* c4 = reinterpret_cast<vec4*>(c + tile * kWaveTile) + lane;
  vec4 x[U], y[U], z[U];
#pragma unroll
  for (int r = 0; r < U; ++r) {
    x[r] = __builtin_nontemporal_load(a4 + r * 64);
    y[r] = __builtin_nontemporal_load(b4 + r * 64);
    z[r] = __builtin_nontemporal_load(c4 + r * 64);
  }
#pragma unroll
  for (int r = 0; r < U; ++r) {
    y[r] = y[r] + x[r];
    z[r] = z[r] + y[r];
    __builtin_nontemporal_store(y[r], b4 + r * 64);
    __builtin_nontemporal_store(z[r], c4 + r * 64);
  }
}

// This thread's share of the sum of tile_count[b .. e) (the counts proper: the flag of the slotted
// pass is masked off): the counts are fetched four to a load
// (the last workgroup of a 4.7 M-element tensor adds up 4600 of them: with one count per load
// that was three rounds of loads in a row, 6 us of the emit pass on a 122 M-element set).
template <int THREADS>
__device__ __forceinline__ int tile_counts_partial(const uint32_t* __restrict__ tc, int64_t b, int64_t e, int tid) {
  int sum = 0;
  if (b >= e) return 0;
  int64_t b4 = (b + 3) & ~(int64_t)3;  // first multiple of four at or above b
  if (b4 > e) b4 = e;
  int64_t e4 = e & ~(int64_t)3;
  if (e4 < b4) e4 = b4;
  // at most three counts before the aligned body and three behind it
  if (tid < (int)(b4 - b)) sum += (int)(tc[b + tid] & kTileCountMask);
  if (tid < (int)(e - e4)) sum += (int)(tc[e4 + tid] & kTileCountMask);
  const uint4* __restrict__ tc4 = reinterpret_cast<const uint4*>(tc);  // the table starts on a 256-byte boundary
  const int64_t q0 = b4 >> 2, q1 = e4 >> 2;
  int64_t q = q0 + tid;
  for (; q + 3 * THREADS < q1; q += 4 * THREADS) {  // four loads in flight per thread
    uint4 c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) c[k] = tc4[q + k * THREADS];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      sum += (int)((c[k].x & kTileCountMask) + (c[k].y & kTileCountMask) + (c[k].z & kTileCountMask) + (c[k].w & kTileCountMask));
  }
  for (; q < q1; q += THREADS) {
    const uint4 c = tc4[q];
    sum += (int)((c.x & kTileCountMask) + (c.y & kTileCountMask) + (c.z & kTileCountMask) + (c.w & kTileCountMask));
  }
  return sum;
}

// ---------------------------------------------------------------------------
// Re-threshold on over-selection
// (paper: Section 5 -- the exact threshold among the elements that passed, for a
//  tensor that let too many pass)
// ---------------------------------------------------------------------------
// Runs between the streaming and the emit pass, one workgroup per tensor.  The workgroup adds up
// the mask-bit counts the streaming pass has left for the tensor's tiles; only if the total
// exceeds refine_limit does it go on: three histogram passes over |v'| of the selected elements
// find the magnitude of descending rank k exactly, and a last walk clears the mask bits of
// elements that do not exceed it.  What the emit pass then extracts is the exact top k of the
// tensor.  (A first version ran over the emit work list: every workgroup recounted its part's
// mask words and took a ticket on the tensor's counter, the last to arrive went on; 17 us on the
// 161-tensor set and 34 us on the 122 M-element set for what the per-tile counts already say.)
struct RefineShared {
  uint32_t hist[kSelectBins];
  uint32_t wave_tot[kRefineThreads / 64];
  uint32_t sel[3];
  int red[kRefineThreads / 64];
  int go;
  uint32_t passed;
  uint32_t listed;
};

// This thread's filtered mask word `wi` (0-based within the tensor's tiles) of tensor [lo, hi).
__device__ __forceinline__ uint32_t tensor_mask_word(const uint16_t* mask, int64_t t0, int64_t wi, int64_t lo,
                                                     int64_t hi, int64_t& tile, int& lane) {
  constexpr int kBits = kStreamUnroll * 4;
  tile = t0 + (wi >> 6);
  lane = (int)(wi & 63);
  uint32_t w = mask[tile * 64 + lane];
  if (w && (tile * kWaveTile < lo || (tile + 1) * kWaveTile > hi)) {
    uint32_t keep = 0;
    for (int q = 0; q < kBits; ++q) {
      const int64_t e = tile_element(tile, lane, q);
      if (e >= lo && e < hi) keep |= 1u << q;
    }
    w &= keep;
  }
  return w;
}

__global__ __launch_bounds__(kRefineThreads) void refine_kernel(RefineArgs a) {
  constexpr int kWaves = kRefineThreads / 64;
  __shared__ RefineShared sh;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int j = blockIdx.x;
  const TensorPlan plan = a.plans[j];
  const int64_t region = a.out_offsets[j];  // asked for early: needed late
  const int64_t cap = a.out_offsets[j + 1] - region;
  const int64_t lo = plan.offset;
  const int64_t hi = plan.offset + plan.n;
  const int64_t t0 = lo / kWaveTile;
  const int64_t t1 = (hi - 1) / kWaveTile;

  // How many elements of the tensor passed: the counts the streaming pass has left for the tiles
  // that lie wholly inside the tensor, and the tensor's share of a first or last tile that it
  // shares with a neighbour (or that is the ragged end of the set), recounted from the mask words.
  const bool shared0 = t0 * kWaveTile < lo || (t0 == t1 && (t1 + 1) * kWaveTile > hi);
  const bool shared1 = t1 != t0 && (t1 + 1) * kWaveTile > hi;
  int cnt = tile_counts_partial<kRefineThreads>(a.tile_count, shared0 ? t0 + 1 : t0, shared1 ? t1 : t1 + 1, tid);
  {
    int64_t tile;
    int l;
    if (shared0 && wave == 0) cnt += __popc(tensor_mask_word(a.mask, t0, lane, lo, hi, tile, l));
    if (shared1 && wave == 1) cnt += __popc(tensor_mask_word(a.mask, t0, (t1 - t0) * 64 + lane, lo, hi, tile, l));
  }
  for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_down(cnt, d);
  if (lane == 0) sh.red[wave] = cnt;
  __syncthreads();
  if (tid == 0) {
    int total = 0;
    for (int w = 0; w < kWaves; ++w) total += sh.red[w];
    sh.passed = (uint32_t)total;
    sh.go = (uint32_t)total > (uint32_t)plan.refine_limit;
  }
  __syncthreads();
  if (!sh.go) return;

  // ---- exact threshold among the selected elements of tensor j (rare) ---------------
  // After a slotted streaming pass a tile that lies wholly inside the tensor and selected 1 to
  // kSlotsPerTile elements holds a record in place of its mask words (indices, v', u'), and u and
  // v are masked there already; every other tile has mask words and u', v' as they were.
  const int64_t words = (t1 - t0 + 1) * 64;
  const int64_t passed = sh.passed;
  uint32_t prefix = 0;
  uint32_t rank = (uint32_t)plan.k;
  int consumed = 0;
  uint32_t* mask32 = reinterpret_cast<uint32_t*>(a.mask);
  const int32_t* records = reinterpret_cast<const int32_t*>(a.mask);
  auto is_record = [&](int64_t tile) {
    if (!a.slotted || tile * kWaveTile < lo || (tile + 1) * kWaveTile > hi) return false;
    const uint32_t c = a.tile_count[tile];  // (with the flag: mask words, whatever the count)
    return c >= 1u && c <= (uint32_t)kSlotsPerTile;
  };
  constexpr uint32_t kFromRecord = 0x80000000u;  // list entry: the element sits in a record (indices are below 2^31)

  if (passed <= cap) {
    // The tensor's payload region is free until the emit pass: list the selected elements
    // there, then their keys, so that everything after one walk over the tiles is coalesced.
    uint32_t* list = reinterpret_cast<uint32_t*>(a.out_idx + region);
    uint32_t* keys = reinterpret_cast<uint32_t*>(a.out_val + region);
    if (tid == 0) sh.listed = 0;
    __syncthreads();
    // records: one thread per tile (keys come with them)
    if (a.slotted) {
      for (int64_t tile = t0 + tid; tile <= t1; tile += kRefineThreads) {
        if (!is_record(tile)) continue;
        const int c = (int)a.tile_count[tile];
        int pos = (int)atomicAdd(&sh.listed, (uint32_t)c);
        for (int q = 0; q < c; ++q) {
          list[pos] = (uint32_t)records[tile * kSlotRecord + q] | kFromRecord;
          keys[pos] = (uint32_t)records[tile * kSlotRecord + kSlotsPerTile + q] & 0x7FFFFFFFu;
          ++pos;
        }
      }
    }
    // mask words: eight (16 bytes) per load, four loads in flight per thread
    const uint4* mask128 = reinterpret_cast<const uint4*>(a.mask + t0 * 64);
    const int64_t chunks = words >> 3;
    for (int64_t c0 = tid; c0 < chunks; c0 += 4 * kRefineThreads) {
      uint4 m[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int64_t c = c0 + k * kRefineThreads;
        m[k] = c < chunks ? mask128[c] : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int64_t c = c0 + k * kRefineThreads;
        if ((m[k].x | m[k].y | m[k].z | m[k].w) == 0) continue;
        if (c < chunks && is_record(t0 + (c >> 3))) continue;  // that line is a record, taken above
        const uint32_t pair[4] = {m[k].x, m[k].y, m[k].z, m[k].w};
#pragma unroll
        for (int h = 0; h < 8; ++h) {
          uint32_t w = (pair[h >> 1] >> (16 * (h & 1))) & 0xFFFFu;
          if (!w) continue;
          const int64_t wi = c * 8 + h;
          const int64_t tile = t0 + (wi >> 6);
          const int l = (int)(wi & 63);
          if (tile * kWaveTile < lo || (tile + 1) * kWaveTile > hi) {  // tile shared with a neighbour
            uint32_t keep = 0;
            for (int q = 0; q < kStreamUnroll * 4; ++q) {
              const int64_t e = tile_element(tile, l, q);
              if (e >= lo && e < hi) keep |= 1u << q;
            }
            w &= keep;
            if (!w) continue;
          }
          int pos = (int)atomicAdd(&sh.listed, (uint32_t)__popc(w));
          while (w) {
            const int q = __ffs(w) - 1;
            w &= w - 1;
            list[pos++] = (uint32_t)tile_element(tile, l, q);
          }
        }
      }
    }
    __syncthreads();
    const int count = (int)passed;
    for (int p0 = tid; p0 < count; p0 += 4 * kRefineThreads) {
      uint32_t e[4];
      float x[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = p0 + q * kRefineThreads;
        e[q] = p < count ? list[p] : kFromRecord;
        x[q] = (e[q] & kFromRecord) ? 0.0f : a.v[e[q]];
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = p0 + q * kRefineThreads;
        if (p < count && !(e[q] & kFromRecord)) keys[p] = __float_as_uint(x[q]) & 0x7FFFFFFFu;
      }
    }
    __syncthreads();
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int bits = pass == 2 ? 9 : 11;
      const int shift = 31 - consumed - bits;
      const uint32_t digit_mask = (1u << bits) - 1u;
      for (int i = tid; i < kSelectBins; i += kRefineThreads) sh.hist[i] = 0;
      __syncthreads();
      for (int p = tid; p < count; p += kRefineThreads) {
        const uint32_t key = keys[p];
        if (pass == 0 || (key >> (shift + bits)) == prefix) atomicAdd(&sh.hist[(key >> shift) & digit_mask], 1u);
      }
      __syncthreads();
      uint32_t bin, above, members;
      find_bin<kRefineThreads>(sh.hist, sh.wave_tot, sh.sel, tid, rank, bin, above, members);
      prefix = (prefix << bits) | bin;
      rank -= above;
      consumed += bits;
    }
    // Clear the mask bit of every selected element that does not exceed the new threshold.
    // A 16-bit mask word of a tile shared with a neighbour tensor also holds that tensor's
    // bits, and its re-threshold may run at the same time: atomic AND on the 32-bit word.
    // (Elements in records are dropped tile by tile below.)
    for (int p = tid; p < count; p += kRefineThreads) {
      if (!(keys[p] > prefix) && !(list[p] & kFromRecord)) {
        const int64_t e = list[p];
        const int64_t tile = e / kWaveTile;
        const int r = (int)(e % kWaveTile);
        const int64_t h = tile * 64 + ((r & 255) >> 2);        // the lane's 16-bit word
        const int q = (r >> 8) * 4 + (r & 3);
        atomicAnd(&mask32[h >> 1], ~((1u << q) << (16 * (int)(h & 1))));
        atomicSub(&a.tile_count[tile], 1u);
      }
    }
  } else {
    // More passed than the payload region holds (the caller's capacity is below the
    // over-selection): walk the tiles in every pass and read v' element by element.
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int bits = pass == 2 ? 9 : 11;
      const int shift = 31 - consumed - bits;
      const uint32_t digit_mask = (1u << bits) - 1u;
      for (int i = tid; i < kSelectBins; i += kRefineThreads) sh.hist[i] = 0;
      __syncthreads();
      if (a.slotted) {
        for (int64_t tile = t0 + tid; tile <= t1; tile += kRefineThreads) {
          if (!is_record(tile)) continue;
          const int c = (int)a.tile_count[tile];
          for (int q = 0; q < c; ++q) {
            const uint32_t key = (uint32_t)records[tile * kSlotRecord + kSlotsPerTile + q] & 0x7FFFFFFFu;
            if (pass == 0 || (key >> (shift + bits)) == prefix) atomicAdd(&sh.hist[(key >> shift) & digit_mask], 1u);
          }
        }
      }
      for (int64_t wi = tid; wi < words; wi += kRefineThreads) {
        if (is_record(t0 + (wi >> 6))) continue;
        int64_t tile;
        int l;
        uint32_t w = tensor_mask_word(a.mask, t0, wi, lo, hi, tile, l);
        while (w) {
          const int q = __ffs(w) - 1;
          w &= w - 1;
          const uint32_t key = __float_as_uint(a.v[tile_element(tile, l, q)]) & 0x7FFFFFFFu;
          if (pass == 0 || (key >> (shift + bits)) == prefix)
            atomicAdd(&sh.hist[(key >> shift) & digit_mask], 1u);
        }
      }
      __syncthreads();
      uint32_t bin, above, members;
      find_bin<kRefineThreads>(sh.hist, sh.wave_tot, sh.sel, tid, rank, bin, above, members);
      prefix = (prefix << bits) | bin;
      rank -= above;
      consumed += bits;
    }
    for (int64_t wi = tid; wi < words; wi += kRefineThreads) {
      if (is_record(t0 + (wi >> 6))) continue;
      int64_t tile;
      int l;
      uint32_t w = tensor_mask_word(a.mask, t0, wi, lo, hi, tile, l);
      uint32_t drop = 0;
      while (w) {
        const int q = __ffs(w) - 1;
        w &= w - 1;
        const uint32_t key = __float_as_uint(a.v[tile_element(tile, l, q)]) & 0x7FFFFFFFu;
        if (!(key > prefix)) drop |= 1u << q;
      }
      if (drop) {
        const int64_t h = tile * 64 + l;  // index of the 16-bit word
        atomicAnd(&mask32[h >> 1], ~(drop << (16 * (int)(h & 1))));
        atomicSub(&a.tile_count[tile], (uint32_t)__popc(drop));
      }
    }
  }
  // Records: an element that does not exceed the new threshold goes back to where the streaming
  // pass took it from (v', and u' under factor masking), the others close ranks in the record, in
  // their order.  One thread per tile: a record belongs to this tensor alone.  (Whether a tile has
  // a record is read off its count, which this loop changes: each tile is looked at once, by one
  // thread, and a count that falls to zero makes the emit pass skip the tile.)
  if (a.slotted) {
    __syncthreads();  // every walk over records and counts above is over
    int32_t* rec = reinterpret_cast<int32_t*>(a.mask);
    for (int64_t tile = t0 + tid; tile <= t1; tile += kRefineThreads) {
      if (!is_record(tile)) continue;
      const int c = (int)a.tile_count[tile];
      int32_t* r = rec + tile * kSlotRecord;
      int kept = 0;
      for (int q = 0; q < c; ++q) {
        const int32_t e = r[q];
        const int32_t xv = r[kSlotsPerTile + q];
        const int32_t xu = r[2 * kSlotsPerTile + q];
        if (((uint32_t)xv & 0x7FFFFFFFu) > prefix) {
          r[kept] = e;
          r[kSlotsPerTile + kept] = xv;
          r[2 * kSlotsPerTile + kept] = xu;
          ++kept;
        } else {
          a.v_out[e] = __int_as_float(xv);
          if (a.factor_masking) a.u_out[e] = __int_as_float(xu);
        }
      }
      if (kept != c) a.tile_count[tile] = (uint32_t)kept;
    }
  }
  if (tid == 0) {
    const float thr = __uint_as_float(prefix);
    a.thr[j] = thr;
    if (a.out_thr) a.out_thr[j] = thr;
  }
}

// ---------------------------------------------------------------------------
// Emit pass: sparse extract + residual + momentum factor masking
// (paper: Algorithm 3, the three lines after Mask; Section 3.3)
// ---------------------------------------------------------------------------
// One workgroup per entry of a host-built list of (tensor, first tile): it owns up
// to kEmitTiles consecutive tiles of that tensor, counts the mask bits that fall
// inside the tensor, obtains that many slots of the tensor's payload region, then
// for every set bit moves v' into the payload and clears v and u.  An element that
// finds the region full is left untouched (it stays in u, v) and the overflow flag
// is set.
//
// The streaming pass has left the number of mask bits of every tile; a workgroup starts
// after the sum over the tensor's tiles before its own, so the workgroups' parts follow
// each other in index order and the region is the same on every run.  Inside its part a
// workgroup places its elements
//   plain   in the order wavefront, lane, tile, bit (whatever is cheapest), or
//   sorted  in index order (DGC_FLAG_SORTED_OUTPUT): the whole region ascends, and a
//           full region keeps the lowest indices.
// (A first version reserved slots with one atomic per workgroup in order of arrival; the
// receive side can find a range of elements in a region by search only if the parts are
// in order.)

// This lane's mask word of tile t with the bits outside tensor [lo, hi) removed.
__device__ __forceinline__ uint32_t tensor_tile_word(const uint16_t* __restrict__ mask, int64_t t, int lane,
                                                     int64_t lo, int64_t hi) {
  constexpr int kBits = kStreamUnroll * 4;
  uint32_t w = mask[t * 64 + lane];
  // (the test must not depend on w: the loads of several tiles are to be in flight together)
  if (t * kWaveTile < lo || (t + 1) * kWaveTile > hi) {  // tile shared with a neighbour tensor
    uint32_t keep = 0;
    for (int q = 0; q < kBits; ++q) {
      const int64_t e = tile_element(t, lane, q);
      if (e >= lo && e < hi) keep |= 1u << q;
    }
    w &= keep;
  }
  return w;
}

// Moves the `in_win` elements listed in `list` to slots slot0, slot0 + 1, ... of the
// tensor's region [region, region + cap): reads v', writes the pair, clears v and u.
// Returns true if some element found the region full.
__device__ __forceinline__ bool emit_move(const EmitArgs& a, const int32_t* list, int in_win, int64_t slot0,
                                          int64_t region, int64_t cap) {
  float* __restrict__ u = a.u;
  float* __restrict__ v = a.v;
  int32_t* __restrict__ out_idx = a.out_idx;
  float* __restrict__ out_val = a.out_val;
  bool overflow = false;
  for (int p0 = threadIdx.x; p0 < in_win; p0 += 4 * kEmitThreads) {
    int32_t e[4];
    float x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int p = p0 + k * kEmitThreads;
      e[k] = p < in_win ? list[p] : -1;
      if (e[k] >= 0 && slot0 + p >= cap) {  // region full: leave the element where it is
        e[k] = -1;
        overflow = true;
      }
      x[k] = e[k] >= 0 ? v[e[k]] : 0.0f;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (e[k] >= 0) {
        const int64_t slot = slot0 + p0 + k * kEmitThreads;
        out_idx[region + slot] = e[k];
        out_val[region + slot] = x[k];
        v[e[k]] = 0.0f;
        if (a.factor_masking) u[e[k]] = 0.0f;
      }
    }
  }
  return overflow;
}

__global__ __launch_bounds__(kEmitThreads) void emit_kernel(EmitArgs a) {
  constexpr int kWaves = kEmitThreads / 64;
  constexpr int kPerWave = kEmitTiles / kWaves;
  __shared__ int wave_tot[kWaves];
  __shared__ int pre_tot[kWaves];
  __shared__ int32_t list[kEmitList];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const EmitBlock blk = a.blocks[blockIdx.x];
  const int j = blk.tensor;
  const int64_t region = a.out_offsets[j];  // asked for early: needed late
  const int64_t cap = a.out_offsets[j + 1] - region;
  const int64_t lo = blk.lo;
  const int64_t hi = blk.hi;
  const int64_t t0 = lo / kWaveTile;
  const int64_t t1 = (hi - 1) / kWaveTile;
  const int64_t first = blk.first_tile;

  // Everything the workgroup needs before it can place its elements is asked for at once: the
  // mask words of its own tiles, and the mask-bit counts the streaming pass has left for the
  // tiles of this tensor before them (every tile strictly between the tensor's first tile and
  // this workgroup's lies wholly inside the tensor; the tensor's share of its first tile is
  // recounted from the mask words).  A version that summed its own words first and only then,
  // behind a barrier, asked for the counts had two memory round trips in a row here.
  uint32_t word[kPerWave];
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int64_t t = first + wave + i * kWaves;
    word[i] = t <= t1 ? tensor_tile_word(a.mask, t, lane, lo, hi) : 0u;
  }
  int pre = tile_counts_partial<kEmitThreads>(a.tile_count, t0 + 1, first, threadIdx.x);
  if (first > t0 && wave == 0) pre += __popc(tensor_tile_word(a.mask, t0, lane, lo, hi));
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) cnt += __popc(word[i]);
  int incl = cnt;
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(incl, d);
    if (lane >= d) incl += t;
  }
  for (int d = 32; d >= 1; d >>= 1) pre += __shfl_xor(pre, d);
  if (lane == 63) wave_tot[wave] = incl;
  if (lane == 0) pre_tot[wave] = pre;
  __syncthreads();
  // Slots taken by the tensor's tiles before the workgroup's first one, and by the wavefronts
  // before this one: no atomics, no tickets, the workgroups of a tensor fill its region in index
  // order, so the region is the same on every run.
  int before = 0, total = 0, base = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int t = wave_tot[w];
    if (w < wave) before += t;
    total += t;
    base += pre_tot[w];
  }
  if (threadIdx.x == 0 && (int)((first - t0) / kEmitTiles) == blk.tensor_blocks - 1) a.out_counts[j] = base + total;
  if (total == 0) return;
  const int64_t base_slot = base;
  const int my_first = before + (incl - cnt);  // position of this lane's first element in the workgroup
  bool overflow = false;
  // The elements to move are first listed in LDS in their slot order, kEmitList at a
  // time, then dealt out one per thread: every thread has the same amount of work and
  // the reads of v are independent of each other.
  for (int win = 0; win < total; win += kEmitList) {
    int pos = my_first;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      uint32_t w = word[i];
      const int64_t t = first + wave + i * kWaves;
      while (w) {
        const int q = __ffs(w) - 1;
        w &= w - 1;
        if (pos >= win && pos < win + kEmitList) list[pos - win] = (int32_t)tile_element(t, lane, q);
        ++pos;
      }
    }
    __syncthreads();
    const int in_win = total - win < kEmitList ? total - win : kEmitList;
    overflow |= emit_move(a, list, in_win, base_slot + win, region, cap);
    __syncthreads();
  }
  if (overflow) atomicOr(&a.state->flags, (uint32_t)DGC_DIAG_OVERFLOW);
}

struct EmitTiles {
  uint16_t words[kEmitTiles * 64];  // the workgroup's mask words, bits outside the tensor removed
  int tile_tot[kEmitTiles];         // selected elements per tile
  int tile_base[kEmitTiles];        // ... and in the workgroup's tiles before it
  int wave_tot[kEmitThreads / 64];
  int block_base, block_total;      // slots taken before the workgroup's part; elements of the part
};

// Parks the workgroup's mask words in LDS, counts per tile, finds where the workgroup's part
// starts in the tensor's region and, in the tensor's last workgroup, writes the tensor's count.
__device__ __forceinline__ void emit_tiles(const EmitArgs& a, const EmitBlock& blk, EmitTiles& sh) {
  constexpr int kWaves = kEmitThreads / 64;
  constexpr int kPerWave = kEmitTiles / kWaves;
  static_assert(kEmitTiles <= 64, "one wavefront scans the tile totals");
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int j = blk.tensor;
  const int64_t lo = blk.lo;
  const int64_t hi = blk.hi;
  const int64_t t1 = (hi - 1) / kWaveTile;
  const int64_t first = blk.first_tile;

  // Slots taken by the tiles of this tensor before the workgroup's first one.  Every tile
  // strictly between the tensor's first tile and this workgroup's lies wholly inside the
  // tensor, so its count left by the streaming pass (and kept up by the re-threshold pass)
  // is what it contributes; the tensor's first tile may be shared with the tensor before
  // and is recounted from its mask words.
  const int64_t t0 = lo / kWaveTile;
  const int in_tensor = (int)((first - t0) / kEmitTiles);
  int before = tile_counts_partial<kEmitThreads>(a.tile_count, t0 + 1, first, threadIdx.x);
  if (first > t0 && wave == 0) before += __popc(tensor_tile_word(a.mask, t0, lane, lo, hi));
  static_assert(kPerWave % 2 == 0, "tile totals are reduced two to a register");
  {
    uint32_t word[kPerWave];
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int64_t t = first + wave + i * kWaves;
      word[i] = t <= t1 ? tensor_tile_word(a.mask, t, lane, lo, hi) : 0u;
    }
    // elements per tile: the lanes' bit counts of two tiles share a register (16 bits each,
    // a tile holds at most 1024) and are summed over the wavefront by a butterfly
    uint32_t pair[kPerWave / 2];
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      sh.words[(wave + i * kWaves) * 64 + lane] = (uint16_t)word[i];
      if (i & 1) pair[i / 2] |= (uint32_t)__popc(word[i]) << 16;
      else pair[i / 2] = (uint32_t)__popc(word[i]);
    }
    for (int d = 32; d >= 1; d >>= 1) {
#pragma unroll
      for (int i = 0; i < kPerWave / 2; ++i) pair[i] += __shfl_xor(pair[i], d);
      before += __shfl_xor(before, d);
    }
    if (lane == 0) {
      sh.wave_tot[wave] = before;
#pragma unroll
      for (int i = 0; i < kPerWave; ++i)
        sh.tile_tot[wave + i * kWaves] = (int)((pair[i / 2] >> (16 * (i & 1))) & 0xFFFFu);
    }
  }
  __syncthreads();
  if (wave == 0) {
    const int own = lane < kEmitTiles ? sh.tile_tot[lane] : 0;
    int incl = own;
    for (int d = 1; d < 64; d <<= 1) {
      const int t = __shfl_up(incl, d);
      if (lane >= d) incl += t;
    }
    if (lane < kEmitTiles) sh.tile_base[lane] = incl - own;
    if (lane == 63) {
      int base = 0;
      for (int w = 0; w < kWaves; ++w) base += sh.wave_tot[w];
      sh.block_base = base;
      sh.block_total = incl;
      if (in_tensor == blk.tensor_blocks - 1) a.out_counts[j] = base + incl;
    }
  }
  __syncthreads();
}

// Sorted variant.  The workgroup's mask words are parked in LDS; everything that
// follows walks the tiles one at a time from there, which keeps the register count low
// (the kernel is latency-bound: what matters is how many workgroups a CU holds).
__global__ __launch_bounds__(kEmitThreads) void emit_sorted_kernel(EmitArgs a) {
  constexpr int kWaves = kEmitThreads / 64;
  constexpr int kPerWave = kEmitTiles / kWaves;
  constexpr int kRows = kStreamUnroll;  // rounds of 256 elements per tile
  __shared__ EmitTiles sh;
  __shared__ int32_t list[kEmitList];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const EmitBlock blk = a.blocks[blockIdx.x];
  const int j = blk.tensor;
  const int64_t region = a.out_offsets[j];  // asked for early: needed late
  const int64_t cap = a.out_offsets[j + 1] - region;
  const int64_t first = blk.first_tile;
  emit_tiles(a, blk, sh);
  const int total = sh.block_total;
  if (total == 0) return;
  const int64_t base_slot = sh.block_base;
  bool overflow = false;
  for (int win = 0; win < total; win += kEmitList) {
    // Index order inside a tile is row (round of 256 elements), lane, component: an
    // element's position is the tile's base, plus the rows before it, plus the bits of
    // its row in lower lanes (counted from the votes), plus the lower bits of its nibble.
#pragma unroll 1
    for (int i = 0; i < kPerWave; ++i) {
      const int tl = wave + i * kWaves;
      if (sh.tile_tot[tl] == 0) continue;
      const uint32_t w = sh.words[tl * 64 + lane];
      const int64_t t = first + tl;
      int row_base = sh.tile_base[tl];
#pragma unroll
      for (int r = 0; r < kRows; ++r) {
        const uint32_t nib = (w >> (4 * r)) & 0xFu;
        if (__ballot(nib != 0) == 0) continue;  // nothing in this row of the tile
        int lower = 0, row = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const unsigned long long vote = __ballot((nib >> c) & 1u);
          lower += (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vote >> 32),
                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)vote, 0u));
          row += __popcll(vote);
        }
        int pos = row_base + lower;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if ((nib >> c) & 1u) {
            if (pos >= win && pos < win + kEmitList) list[pos - win] = (int32_t)tile_element(t, lane, 4 * r + c);
            ++pos;
          }
        }
        row_base += row;
      }
    }
    __syncthreads();
    const int in_win = total - win < kEmitList ? total - win : kEmitList;
    overflow |= emit_move(a, list, in_win, base_slot + win, region, cap);
    __syncthreads();
  }
  if (overflow) atomicOr(&a.state->flags, (uint32_t)DGC_DIAG_OVERFLOW);
}

// Emit pass after a STAGED streaming pass: the selected values of a tile that lies wholly
// inside one tensor wait in the tile's slots of the staging array, in index order, and u
// and v are masked already.  The part's payload is written in index order (as the sorted
// variant does, with the same positions), values copied from the staging array; nothing
// is listed in LDS and u, v are touched only where the region is full (the element is put
// back: v' and, under factor masking, u') and in tiles shared between tensors, which the
// streaming pass leaves alone.
__global__ __launch_bounds__(kEmitThreads) void emit_staged_kernel(EmitArgs a) {
  constexpr int kWaves = kEmitThreads / 64;
  constexpr int kPerWave = kEmitTiles / kWaves;
  constexpr int kRows = kStreamUnroll;
  __shared__ EmitTiles sh;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const EmitBlock blk = a.blocks[blockIdx.x];
  const int j = blk.tensor;
  const int64_t first = blk.first_tile;
  emit_tiles(a, blk, sh);
  if (sh.block_total == 0) return;
  const int64_t lo = blk.lo;
  const int64_t hi = blk.hi;
  const int64_t region = a.out_offsets[j];
  const int64_t cap = a.out_offsets[j + 1] - region;
  int32_t* __restrict__ out_idx = a.out_idx + region;
  float* __restrict__ out_val = a.out_val + region;
  float* __restrict__ u = a.u;
  float* __restrict__ v = a.v;
  bool overflow = false;
  // What a tile of the wavefront is, as far as the copy of its values goes.
  auto tile_of = [&](int i, const float*& stage, float*& vals, int& room) {
    const int tl = wave + i * kWaves;
    const int64_t t = first + tl;
    const int tile_total = sh.tile_tot[tl];
    const bool staged = t * kWaveTile >= lo && (t + 1) * kWaveTile <= hi;
    const int64_t slot0 = (int64_t)sh.block_base + sh.tile_base[tl];
    stage = a.stage_v + t * kWaveTile;
    vals = out_val + slot0;
    // slots of the tile that exist (the rest of the tile overflows); none to copy for a shared tile
    room = cap - slot0 >= tile_total ? tile_total : (cap > slot0 ? (int)(cap - slot0) : 0);
    return staged;
  };
  // The values are a straight copy: the staging array holds a tile's in slot order.  The first
  // 256 of every tile of the wavefront are loaded before any is stored (one wait for all).
  {
    float x[kPerWave][4];
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const float* stage;
      float* vals;
      int room;
      const bool staged = tile_of(i, stage, vals, room);
#pragma unroll
      for (int k = 0; k < 4; ++k) x[i][k] = (staged && k * 64 + lane < room) ? stage[k * 64 + lane] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const float* stage;
      float* vals;
      int room;
      const bool staged = tile_of(i, stage, vals, room);
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (staged && k * 64 + lane < room) vals[k * 64 + lane] = x[i][k];
    }
  }
#pragma unroll 1
  for (int i = 0; i < kPerWave; ++i) {
    const int tl = wave + i * kWaves;
    const int tile_total = sh.tile_tot[tl];
    if (tile_total == 0) continue;
    const uint32_t w = sh.words[tl * 64 + lane];
    const int64_t t = first + tl;
    const float* __restrict__ stage_v;
    float* __restrict__ tile_val;
    int room;
    {
      const float* stage;
      float* vals;
      const bool st = tile_of(i, stage, vals, room);
      stage_v = stage;
      tile_val = vals;
      if (st) {
        for (int s = 256 + lane; s < room; s += 64) vals[s] = stage[s];  // beyond a quarter of the tile
      }
    }
    const bool staged = t * kWaveTile >= lo && (t + 1) * kWaveTile <= hi;
    const float* __restrict__ stage_u = a.stage_u ? a.stage_u + t * kWaveTile : nullptr;
    int32_t* __restrict__ tile_idx = out_idx + ((int64_t)sh.block_base + sh.tile_base[tl]);
    // the indices: an element's slot is rows before it + bits of its row in lower lanes + lower bits of its nibble
    if (staged && tile_total < 256 && room == tile_total) {
      // Fewer than 256 elements, all with a slot (at 1.6 % a tile selects 16): the counts of the
      // lane's four rows ride in the bytes of one word (no byte can overflow), one scan over the
      // lanes gives every row's "bits in lower lanes", the rows' totals shifted up by one, two and
      // three bytes the "rows before it", and a lane walks its own bits, lowest first: two or
      // three rounds instead of sixteen votes.
      uint32_t x = w - ((w >> 1) & 0x5555u);
      x = (x & 0x3333u) + ((x >> 2) & 0x3333u);  // a count per nibble
      const uint32_t cnt = (x & 0xFu) | ((x & 0xF0u) << 4) | ((x & 0xF00u) << 8) | ((x & 0xF000u) << 12);
      uint32_t incl = cnt;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
      }
      const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
      uint32_t at = (incl - cnt) + ((tot << 8) + (tot << 16) + (tot << 24));  // next slot of each of the lane's rows
      const int32_t e_lane = (int32_t)tile_element(t, lane, 0);
      uint32_t rem = w;
      while (__ballot(rem != 0u)) {
        if (rem != 0u) {
          const int b = __ffs((int)rem) - 1;  // bit 4 r + c
          const int r8 = (b >> 2) * 8;
          tile_idx[(at >> r8) & 0xFFu] = e_lane + (b >> 2) * 256 + (b & 3);
          at += 1u << r8;
          rem &= rem - 1u;
        }
      }
      continue;
    }
    int row_base = 0;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const uint32_t nib = (w >> (4 * r)) & 0xFu;
      int lower = 0, row = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const unsigned long long vote = __ballot((nib >> c) & 1u);
        lower += (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vote >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vote, 0u));
        row += __popcll(vote);
      }
      int pos = row_base + lower;
      const int32_t e0 = (int32_t)tile_element(t, lane, 4 * r);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if ((nib >> c) & 1u) {
          if (pos < room) {
            tile_idx[pos] = e0 + c;
            if (!staged) {  // a tile shared between tensors: value taken and u, v masked here
              tile_val[pos] = v[e0 + c];
              v[e0 + c] = 0.0f;
              if (a.factor_masking) u[e0 + c] = 0.0f;
            }
          } else {
            overflow = true;
            if (staged) {  // region full: the element goes back to where the streaming pass took it from
              v[e0 + c] = stage_v[pos];
              if (a.factor_masking && stage_u) u[e0 + c] = stage_u[pos];
            }
          }
        }
        pos += (int)((nib >> c) & 1u);
      }
      row_base += row;
    }
  }
  if (overflow) atomicOr(&a.state->flags, (uint32_t)DGC_DIAG_OVERFLOW);
}

// Emit pass after a SLOTTED streaming pass.  Four threads per tile of the workgroup's 32 tiles,
// two slots each: a thread asks for its slots' indices and values at once with the tile's count
// and the counts of the tensor's tiles before the workgroup (two wavefronts per workgroup: the
// parts of a 122 M-element set are all resident at once); a tile that lies wholly inside the tensor and selected
// at most kSlotsPerTile elements is a straight copy (its u and v are masked already; an element
// that finds the region full is put back).  The other tiles -- shared with a neighbour tensor, or
// with more selected elements than slots -- are taken by the wavefront that holds them, one after
// the other, from their mask words as in the plain pass: read v', write the pair, clear v and u.
// Order inside the workgroup's part: tile by tile, index order inside a tile (a record is in index
// order, and the tiles taken from mask words are placed by the votes of their rows), so the
// whole region ascends, and a full region keeps the lowest indices: this pass also serves
// DGC_FLAG_SORTED_OUTPUT.
struct EmitSlotsShared {
  uint16_t words[kEmitTiles * 64];  // mask words of the tiles that are not copied from slots
  int cnt[kEmitTiles];              // elements of every tile that belong to this tensor
  int pre_tot[kEmitSlotThreads / 64];
};

__global__ __launch_bounds__(kEmitSlotThreads) void emit_slots_kernel(EmitArgs a) {
  constexpr int kWaves = kEmitSlotThreads / 64;
  constexpr int kLanesPerTile = kEmitSlotThreads / kEmitTiles;
  constexpr int kPerLane = kSlotsPerTile / kLanesPerTile;
  static_assert(kPerLane == 2 && kLanesPerTile * kPerLane == kSlotsPerTile, "a thread takes two neighbouring slots");
  constexpr int kEmitWalk = 6;  // selected elements of one lane the short way takes
  constexpr int kTilesPerWave = 64 / kLanesPerTile;
  static_assert(kEmitTiles <= 32 && kTilesPerWave * kWaves == kEmitTiles, "tile counts are scanned by half a wavefront");
  __shared__ EmitSlotsShared sh;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const EmitBlock blk = a.blocks[blockIdx.x];
  const int j = blk.tensor;
  const int64_t region = a.out_offsets[j];  // asked for early: needed late
  const int64_t cap = a.out_offsets[j + 1] - region;
  const int64_t lo = blk.lo;
  const int64_t hi = blk.hi;
  const int64_t t0 = lo / kWaveTile;
  const int64_t t1 = (hi - 1) / kWaveTile;
  const int64_t first = blk.first_tile;

  const int tl = tid / kLanesPerTile;             // this thread's tile of the part ...
  const int s = (tid % kLanesPerTile) * kPerLane;  // ... and the first of its two slots of that tile
  const int64_t t = first + tl;
  const bool exists = t <= t1;
  const bool inside = exists && t * kWaveTile >= lo && (t + 1) * kWaveTile <= hi;
  const uint32_t c_raw = exists ? a.tile_count[t] : 0u;
  const uint32_t c_own = c_raw & kTileCountMask;
  int2 e_slot = make_int2(0, 0);
  int2 x_slot = make_int2(0, 0);  // bits of the values
  const int32_t* __restrict__ records = reinterpret_cast<const int32_t*>(a.mask);  // see the streaming pass
  if (inside) {  // (a record only if the count says so; loaded before the count is known)
    e_slot = *reinterpret_cast<const int2*>(records + t * kSlotRecord + s);
    x_slot = *reinterpret_cast<const int2*>(records + t * kSlotRecord + kSlotsPerTile + s);
  }
  // Slots taken by the tensor's tiles before the workgroup's first one.  The tensor's first tile
  // counts like the others when it lies wholly inside the tensor (its line may hold a record);
  // shared with the tensor before, it has mask words, from which the tensor's share is recounted.
  const bool first_shared = t0 * kWaveTile < lo;
  int pre = tile_counts_partial<kEmitSlotThreads>(a.tile_count, first_shared ? t0 + 1 : t0, first, tid);
  if (first > t0 && first_shared && wave == 0) pre += __popc(tensor_tile_word(a.mask, t0, lane, lo, hi));
  for (int d = 32; d >= 1; d >>= 1) pre += __shfl_xor(pre, d);
  if (lane == 0) sh.pre_tot[wave] = pre;

  const bool from_slots = inside && c_raw <= (uint32_t)kSlotsPerTile;  // (a flagged count is a large number)
  // tiles of this wavefront that are taken from their mask words: one bit per tile, at its first lane
  const unsigned long long others = __ballot(exists && !from_slots && s == 0);
  if (from_slots && s == 0) sh.cnt[tl] = (int)c_own;
  if (!exists && s == 0) sh.cnt[tl] = 0;
  for (unsigned long long m = others; m; m &= m - 1) {
    const int k = wave * kTilesPerWave + (__ffsll((long long)m) - 1) / kLanesPerTile;
    const uint32_t w = tensor_tile_word(a.mask, first + k, lane, lo, hi);
    sh.words[k * 64 + lane] = (uint16_t)w;
    int c = __popc(w);
    for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d);
    if (lane == 0) sh.cnt[k] = c;
  }
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) base += sh.pre_tot[w];
  // where every tile starts in the part: each wavefront scans the 32 counts for itself
  const int own = lane < kEmitTiles ? sh.cnt[lane] : 0;
  int incl = own;
  for (int d = 1; d < 32; d <<= 1) {
    const int up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  const int total = __shfl(incl, kEmitTiles - 1);
  if (tid == 0 && (int)((first - t0) / kEmitTiles) == blk.tensor_blocks - 1) a.out_counts[j] = base + total;
  if (total == 0) return;
  const int excl = incl - own;
  int32_t* __restrict__ out_idx = a.out_idx + region;
  float* __restrict__ out_val = a.out_val + region;
  float* __restrict__ u = a.u;
  float* __restrict__ v = a.v;
  bool overflow = false;
  {
    const int tile_start = __shfl(excl, tl & 31);
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) {
      const int32_t e_q = q == 0 ? e_slot.x : e_slot.y;
      const float x_q = __int_as_float(q == 0 ? x_slot.x : x_slot.y);
      if (from_slots && s + q < (int)c_own) {
        const int64_t slot = (int64_t)base + tile_start + s + q;
        if (slot < cap) {
          out_idx[slot] = e_q;
          out_val[slot] = x_q;
        } else {  // region full: the element goes back to where the streaming pass took it from
          overflow = true;
          v[e_q] = x_q;
          if (a.factor_masking) u[e_q] = __int_as_float(records[t * kSlotRecord + 2 * kSlotsPerTile + s + q]);
        }
      }
    }
  }
  for (unsigned long long m = others; m; m &= m - 1) {
    const int k = wave * kTilesPerWave + (__ffsll((long long)m) - 1) / kLanesPerTile;
    const int64_t tk = first + k;
    const uint32_t w = sh.words[k * 64 + lane];
    const int64_t tile_slot = (int64_t)base + __shfl(excl, k);
    // Index order inside the tile is row (one 16-byte vector per lane), lane, component: an element's
    // position is the rows before it, plus the bits of its row in lower lanes, plus the lower bits of
    // its nibble.
    int most = __popc(w);  // bits of the lane that has most
    for (int d = 32; d >= 1; d >>= 1) {
      const int o = __shfl_xor(most, d);
      most = o > most ? o : most;
    }
    most = __builtin_amdgcn_readfirstlane(most);  // the same in every lane: branches on it are scalar
    const int tile_count = __shfl(own, k);
    if (tile_count < 256 && most <= kEmitWalk) {
      // The usual case (a tile shared between tensors, or a dozen elements in one tile): positions
      // from one packed scan (the counts of the lane's four rows in the bytes of a word, as in the
      // staged pass), and every lane walks its own bits: all of the tile's reads of v are on their
      // way before the first store, one round trip to memory per tile instead of one per row.
      uint32_t xw = w - ((w >> 1) & 0x5555u);
      xw = (xw & 0x3333u) + ((xw >> 2) & 0x3333u);  // a count per nibble
      const uint32_t cnt = (xw & 0xFu) | ((xw & 0xF0u) << 4) | ((xw & 0xF00u) << 8) | ((xw & 0xF000u) << 12);
      uint32_t inc = cnt;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(inc, d);
        if (lane >= d) inc += up;
      }
      const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
      uint32_t next = (inc - cnt) + ((tot << 8) + (tot << 16) + (tot << 24));  // next position of each of the lane's rows
      const int32_t e_lane = (int32_t)tile_element(tk, lane, 0);
      uint32_t rem = w;
      int32_t e[kEmitWalk];
      int ps[kEmitWalk];
      float x[kEmitWalk];
#pragma unroll
      for (int i = 0; i < kEmitWalk; ++i) {
        e[i] = -1;
        ps[i] = 0;
        x[i] = 0.0f;
        if (i < most) {
          if (rem != 0u) {
            const int b = __ffs((int)rem) - 1;  // bit 4 r + c
            const int r8 = (b >> 2) * 8;
            ps[i] = (int)((next >> r8) & 0xFFu);
            next += 1u << r8;
            rem &= rem - 1u;
            if (tile_slot + ps[i] < cap) e[i] = e_lane + (b >> 2) * 256 + (b & 3);
            else overflow = true;  // region full: the element stays where it is
          }
          if (e[i] >= 0) x[i] = v[e[i]];
        }
      }
#pragma unroll
      for (int i = 0; i < kEmitWalk; ++i) {
        if (i < most && e[i] >= 0) {
          out_idx[tile_slot + ps[i]] = e[i];
          out_val[tile_slot + ps[i]] = x[i];
          v[e[i]] = 0.0f;
          if (a.factor_masking) u[e[i]] = 0.0f;
        }
      }
      continue;
    }
    // Otherwise row by row, positions from votes; a row's (up to four) elements of a lane are read together.
    int row_base = 0;
#pragma unroll
    for (int r = 0; r < kStreamUnroll; ++r) {
      const uint32_t nib = (w >> (4 * r)) & 0xFu;
      if (__ballot(nib != 0) == 0) continue;  // nothing in this row of the tile
      int lower = 0, row = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const unsigned long long vote = __ballot((nib >> c) & 1u);
        lower += (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vote >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vote, 0u));
        row += __popcll(vote);
      }
      int pos = row_base + lower;
      int32_t e[4];
      int64_t at[4];
      float x[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        e[c] = -1;
        at[c] = tile_slot + pos;
        if ((nib >> c) & 1u) {
          if (at[c] < cap) e[c] = (int32_t)tile_element(tk, lane, 4 * r + c);
          else overflow = true;  // region full: the element stays where it is
          ++pos;
        }
        x[c] = e[c] >= 0 ? v[e[c]] : 0.0f;
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (e[c] >= 0) {
          out_idx[at[c]] = e[c];
          out_val[at[c]] = x[c];
          v[e[c]] = 0.0f;
          if (a.factor_masking) u[e[c]] = 0.0f;
        }
      }
      row_base += row;
    }
  }
  if (overflow) atomicOr(&a.state->flags, (uint32_t)DGC_DIAG_OVERFLOW);
}

}  // namespace

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
hipError_t launch_clear_words(uint32_t* p, size_t words, hipStream_t stream) {
  if (words == 0) return hipSuccess;
  size_t blocks = (words + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, words);
  return hipGetLastError();
}

int32_t norm_blocks(int64_t n) {
  int64_t blocks = ceil_div(n >> 2, (int64_t)kNormThreads * 8);
  if (blocks < 1) blocks = 1;
  if (blocks > kNormMaxBlocks) blocks = kNormMaxBlocks;
  return (int32_t)blocks;
}

hipError_t launch_norm(const float* g, int64_t n, double* partials, hipStream_t stream) {
  hipLaunchKernelGGL(norm_kernel, dim3((unsigned)norm_blocks(n)), dim3(kNormThreads), 0, stream, g, n, partials);
  return hipGetLastError();
}

hipError_t launch_select(const SelectArgs& a, int32_t num_tensors, hipStream_t stream) {
  if (a.nesterov)
    hipLaunchKernelGGL(select_kernel<true>, dim3((unsigned)num_tensors), dim3(kSelectThreads), 0, stream, a);
  else
    hipLaunchKernelGGL(select_kernel<false>, dim3((unsigned)num_tensors), dim3(kSelectThreads), 0, stream, a);
  return hipGetLastError();
}

// Dynamic LDS that nothing uses: it caps the workgroups a compute unit holds at `groups`.
constexpr size_t kStreamStaticLds = sizeof(float) * kStreamWaves * 4 * kStreamUnroll * 64;  // mixed_z of stream_kernel
static size_t stream_lds_pad(int groups, size_t static_lds) {
  const size_t per = kLdsPerComputeUnit / (size_t)groups - 2048;  // (2 KB of slack for the allocation granule)
  const size_t limit = 64 * 1024;                                  // a workgroup's LDS without a function attribute
  const size_t want = per < limit ? per : limit;
  return want > static_lds ? want - static_lds : 0;
}

template <bool NESTEROV, bool SCALED>
static void launch_stream_mode(const StreamArgs& a, int mode, int groups, dim3 grid, dim3 block, hipStream_t stream) {
  const size_t pad = stream_lds_pad(groups, kStreamStaticLds);
  if (mode == kStreamStaged) hipLaunchKernelGGL((stream_kernel<NESTEROV, SCALED, kStreamStaged>), grid, block, pad, stream, a);
  else if (mode == kStreamSlotted) hipLaunchKernelGGL((stream_kernel<NESTEROV, SCALED, kStreamSlotted>), grid, block, pad, stream, a);
  else hipLaunchKernelGGL((stream_kernel<NESTEROV, SCALED, kStreamPlain>), grid, block, pad, stream, a);
}

hipError_t launch_stream(const StreamArgs& a, hipStream_t stream) {
  const int64_t tiles = ceil_div(a.n, kWaveTile);
  const int64_t blocks = ceil_div(tiles, kStreamWaves);
  // scale is known to be exactly 1 when neither the norm kernel nor an override supplies it
  const bool scaled = a.scale_from_state != 0 || a.scale_const != 1.0f;
  const dim3 grid((unsigned)blocks), block(kStreamThreads);
  const int mode = a.stage_v ? kStreamStaged : a.slotted ? kStreamSlotted : kStreamPlain;
  // right after the norm pass part of g comes from the last-level cache, and more wavefronts pay
  const int groups = a.scale_from_state ? kStreamGroupsAfterNorm : kStreamResidentGroups;
  if (a.nesterov) {
    if (scaled) launch_stream_mode<true, true>(a, mode, groups, grid, block, stream);
    else launch_stream_mode<true, false>(a, mode, groups, grid, block, stream);
  } else {
    if (scaled) launch_stream_mode<false, true>(a, mode, groups, grid, block, stream);
    else launch_stream_mode<false, false>(a, mode, groups, grid, block, stream);
  }
  return hipGetLastError();
}

hipError_t launch_ceiling(const float* a, float* b, float* c, int64_t n, int groups, hipStream_t stream) {
  const int64_t tiles = n / kWaveTile;
  if (tiles < 1) return hipSuccess;
  if (groups < 1) groups = kStreamResidentGroups * kStreamWaves;
  hipLaunchKernelGGL(ceiling_kernel, dim3((unsigned)tiles), dim3(64), stream_lds_pad(groups, 0), stream, a, b, c, tiles);
  return hipGetLastError();
}

hipError_t launch_refine(const RefineArgs& a, int32_t num_tensors, hipStream_t stream) {
  hipLaunchKernelGGL(refine_kernel, dim3((unsigned)num_tensors), dim3(kRefineThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_emit(const EmitArgs& a, int32_t num_blocks, bool sorted, hipStream_t stream) {
  if (a.stage_v)
    hipLaunchKernelGGL(emit_staged_kernel, dim3((unsigned)num_blocks), dim3(kEmitThreads), 0, stream, a);
  else if (a.slotted)
    hipLaunchKernelGGL(emit_slots_kernel, dim3((unsigned)num_blocks), dim3(kEmitSlotThreads), 0, stream, a);
  else if (sorted)
    hipLaunchKernelGGL(emit_sorted_kernel, dim3((unsigned)num_blocks), dim3(kEmitThreads), 0, stream, a);
  else
    hipLaunchKernelGGL(emit_kernel, dim3((unsigned)num_blocks), dim3(kEmitThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace dgc
