// Calibration-side kernels: min/max activation steps per K-segment (Sec. 4.3.2: s_- = |min x| / q, s_+ = max x / q;
// App. B sensitivity study: the strict min/max rule) with running maxima over calibration batches.  One pass over
// the activations, HBM-bandwidth-bound.
#include "sq_kernels.hpp"

#include <cmath>
#include <mutex>

namespace sq {

constexpr int kCalibRows = 8;   // token rows per workgroup

__global__ void calib_init_kernel(float* __restrict__ amax, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) amax[i] = 0.0f;
}

// grid: (row blocks, K-segments).  Maxima are >= 0, so their fp32 bit patterns order like unsigned integers and
// the cross-workgroup combine is an integer atomic max.
template <bool BF16, bool VEC8>
__global__ __launch_bounds__(256) void calib_amax_kernel(const void* __restrict__ x, int M, int K, const ActTable tb,
                                                         float* __restrict__ amax) {
  const int ks = blockIdx.y;
  int k0 = 0, k1 = 0;
  bool dual = false;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.kseg_off[s]; k1 = tb.kseg_off[s + 1]; dual = tb.dual[s] != 0; }
  const int L = k1 - k0;
  const int r0 = blockIdx.x * kCalibRows;
  const int nrows = (M - r0) < kCalibRows ? (M - r0) : kCalibRows;
  float mp = 0.0f, mn = 0.0f;
  auto take = [&](float v) {
    if (dual) {
      mp = __builtin_fmaxf(mp, v);
      mn = __builtin_fmaxf(mn, -v);
    } else {
      mp = __builtin_fmaxf(mp, __builtin_fabsf(v));
    }
  };
  if (VEC8) {
    const int cpr = L >> 3;                                 // 8-element chunks per row of the segment
    for (int cc = threadIdx.x; cc < cpr; cc += 256) {       // the rows of the block are independent loads in flight
      v4i raw[kCalibRows][BF16 ? 1 : 2];
#pragma unroll
      for (int r = 0; r < kCalibRows; ++r) {
        const int rr = r < nrows ? r : nrows - 1;           // ragged M: re-read the last row (a maximum does not mind)
        const size_t e = (size_t)(r0 + rr) * K + k0 + cc * 8;
        if (BF16) {
          raw[r][0] = *reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(x) + e);
        } else {
          raw[r][0] = *reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + e);
          raw[r][BF16 ? 0 : 1] = *reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + e + 4);
        }
      }
#pragma unroll
      for (int r = 0; r < kCalibRows; ++r) {
        if (BF16) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t u = (uint32_t)raw[r][0][i];
            take(__uint_as_float(u << 16));
            take(__uint_as_float(u & 0xFFFF0000u));
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) { take(__int_as_float(raw[r][0][i])); take(__int_as_float(raw[r][BF16 ? 0 : 1][i])); }
        }
      }
    }
  } else {
    for (int c = threadIdx.x; c < nrows * L; c += 256) {
      const int r = c / L, cc = c - r * L;
      const size_t e = (size_t)(r0 + r) * K + k0 + cc;
      take(BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(x)[e]) : reinterpret_cast<const float*>(x)[e]);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    mp = __builtin_fmaxf(mp, __shfl_xor(mp, off, 64));
    mn = __builtin_fmaxf(mn, __shfl_xor(mn, off, 64));
  }
  __shared__ float red[2][4];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][wave] = mp; red[1][wave] = mn; }
  __syncthreads();
  if (threadIdx.x == 0) {
    mp = __builtin_fmaxf(__builtin_fmaxf(red[0][0], red[0][1]), __builtin_fmaxf(red[0][2], red[0][3]));
    mn = __builtin_fmaxf(__builtin_fmaxf(red[1][0], red[1][1]), __builtin_fmaxf(red[1][2], red[1][3]));
    // Look before combining (an uncached read): the running maximum only grows, so a value that already is at least
    // this workgroup's maximum makes the atomic unnecessary; same-address atomics serialize at ~20 ns each.
    // Measured alternatives, all slower on the headline layer (45 us as is): fewer rows or one column tile per
    // workgroup (more, shorter workgroups: 70-220 us), per-wave combining without the barrier (78 us), an ordinary
    // cached read for the test (stale zeros: every workgroup takes the atomic, 219 us), one 8-element chunk per thread
    // (186 us), 512 workgroups walking the row blocks (54 us).
    unsigned int* gp = reinterpret_cast<unsigned int*>(amax) + ks;
    unsigned int* gn = reinterpret_cast<unsigned int*>(amax) + tb.S + ks;
    if (__float_as_uint(mp) > *reinterpret_cast<volatile unsigned int*>(gp)) atomicMax(gp, __float_as_uint(mp));
    if (__float_as_uint(mn) > *reinterpret_cast<volatile unsigned int*>(gn)) atomicMax(gn, __float_as_uint(mn));
  }
}

// steps[ks] = s_+ , steps[S + ks] = s_- : amax / 127, the neutral step 1.0 where the maximum is 0
__global__ void calib_steps_kernel(const float* __restrict__ amax, float* __restrict__ steps, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const float a = amax[i];
    steps[i] = (a == 0.0f) ? 1.0f : a / kQmax;
  }
}

hipError_t launch_calibrate_act(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, float* amax, float* steps,
                                bool accumulate, hipStream_t st) {
  const int n = 2 * tb.S;
  if (!accumulate) hipLaunchKernelGGL(calib_init_kernel, dim3(1), dim3(128), 0, st, amax, n);
  bool vec = (K % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) vec = vec && (tb.kseg_off[s] % 8 == 0);
  dim3 grid((M + kCalibRows - 1) / kCalibRows, tb.S);
#define SQ_CALIB(B, V) hipLaunchKernelGGL((calib_amax_kernel<B, V>), grid, dim3(256), 0, st, x, M, K, tb, amax)
  if (x_is_bf16) { if (vec) SQ_CALIB(true, true); else SQ_CALIB(true, false); }
  else           { if (vec) SQ_CALIB(false, true); else SQ_CALIB(false, false); }
#undef SQ_CALIB
  hipLaunchKernelGGL(calib_steps_kernel, dim3(1), dim3(128), 0, st, amax, steps, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// Percentile clipping (App. B, dual-scale sensitivity study: p <= 0.9999 against the min/max rule).  Per K-segment
// and polarity the threshold is the nearest-rank quantile of max(x,0), max(-x,0) or |x| over the batch, zeros
// included.  The values are >= 0, so their fp32 bit patterns order like unsigned integers and the exact order
// statistic comes from a radix select on those bits, most significant digit first: a histogram pass over the
// activations per digit (one pass per 8 bits: two for bf16 inputs, four for fp32), each followed by a tiny kernel
// that walks the 256 bins from the top, picks the bin holding the wanted rank and narrows the search to it.
// Digit 0 is never counted (it would make the zeros of the other polarity one hot bin): its count is the rest of
// the bucket.
// ------------------------------------------------------------------------------------------------------------
struct PctState {                                 // the caller's workspace
  unsigned int hist[SQ_MAX_SEGMENTS][2][256];     // [ks][polarity][digit], zero between passes
  unsigned int rank[SQ_MAX_SEGMENTS][2];          // wanted rank from the top (1 = largest) inside the bucket
  unsigned int bucket[SQ_MAX_SEGMENTS][2];        // elements that share the prefix found so far
  unsigned int prefix[SQ_MAX_SEGMENTS][2];        // magnitude bits found so far
};
struct PctRanks {                                 // per K-segment: elements of a batch, rank from the top
  unsigned int n[SQ_MAX_SEGMENTS];
  unsigned int r[SQ_MAX_SEGMENTS];
};

constexpr int kPctCopies = 8;

size_t calibrate_workspace_bytes() { return sizeof(PctState); }

__global__ void pct_init_kernel(PctState* __restrict__ st, const PctRanks rk, int S) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < S * 2 * 256) (&st->hist[0][0][0])[i] = 0u;
  if (i < S * 2) {
    const int ks = i >> 1, pol = i & 1;
    st->rank[ks][pol] = rk.r[ks];
    st->bucket[ks][pol] = rk.n[ks];
    st->prefix[ks][pol] = 0u;
  }
}

// grid: (row blocks, K-segments), as the maximum pass.  Counts digit (bits >> shift) & dmask of every value whose
// bits above the digit (himask) equal the prefix found so far.
template <bool BF16, bool VEC8>
__global__ __launch_bounds__(256) void pct_hist_kernel(const void* __restrict__ x, int M, int K, const ActTable tb,
                                                       PctState* __restrict__ st, int shift, unsigned int dmask,
                                                       unsigned int himask) {
  const int ks = blockIdx.y;
  int k0 = 0, k1 = 0;
  bool dual = false;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.kseg_off[s]; k1 = tb.kseg_off[s + 1]; dual = tb.dual[s] != 0; }
  const int L = k1 - k0;
  const int r0 = blockIdx.x * kCalibRows;
  const int nrows = (M - r0) < kCalibRows ? (M - r0) : kCalibRows;
  // kPctCopies copies of every bin, consecutive in LDS (so in different banks), one per lane class: activations
  // put a third of a wave's lanes on one exponent bin, and same-address LDS atomics serialize
  __shared__ unsigned int h[2][256][kPctCopies];
  for (int i = threadIdx.x; i < 2 * 256 * kPctCopies; i += 256) (&h[0][0][0])[i] = 0u;
  const unsigned int pre_p = st->prefix[ks][0], pre_n = st->prefix[ks][1];
  const int copy = threadIdx.x & (kPctCopies - 1);
  __syncthreads();
  auto count = [&](int pol, unsigned int bits, unsigned int pre) {
    if ((bits & himask) == pre) {
      const unsigned int d = (bits >> shift) & dmask;
      if (d != 0u) atomicAdd(&h[pol][d][copy], 1u);
    }
  };
  auto take = [&](float v) {
    const unsigned int bits = __float_as_uint(v), mag = bits & 0x7FFFFFFFu;
    if (dual) {
      count(0, v > 0.0f ? bits : 0u, pre_p);
      count(1, v < 0.0f ? mag : 0u, pre_n);
    } else {
      count(0, mag, pre_p);
    }
  };
  if (VEC8) {
    const int cpr = L >> 3;
    for (int cc = threadIdx.x; cc < cpr; cc += 256) {
      v4i raw[kCalibRows][BF16 ? 1 : 2];
#pragma unroll
      for (int r = 0; r < kCalibRows; ++r) {
        const int rr = r < nrows ? r : nrows - 1;           // ragged M: in-bounds load, not counted below
        const size_t e = (size_t)(r0 + rr) * K + k0 + cc * 8;
        if (BF16) {
          raw[r][0] = *reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(x) + e);
        } else {
          raw[r][0] = *reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + e);
          raw[r][BF16 ? 0 : 1] = *reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + e + 4);
        }
      }
#pragma unroll
      for (int r = 0; r < kCalibRows; ++r) {
        if (r >= nrows) continue;
        if (BF16) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t u = (uint32_t)raw[r][0][i];
            take(__uint_as_float(u << 16));
            take(__uint_as_float(u & 0xFFFF0000u));
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) { take(__int_as_float(raw[r][0][i])); take(__int_as_float(raw[r][BF16 ? 0 : 1][i])); }
        }
      }
    }
  } else {
    for (int c = threadIdx.x; c < nrows * L; c += 256) {
      const int r = c / L, cc = c - r * L;
      const size_t e = (size_t)(r0 + r) * K + k0 + cc;
      take(BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(x)[e]) : reinterpret_cast<const float*>(x)[e]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int pol = 0; pol < 2; ++pol) {
    unsigned int c = 0u;
#pragma unroll
    for (int i = 0; i < kPctCopies; ++i) c += h[pol][threadIdx.x][i];
    if (c != 0u) atomicAdd(&st->hist[ks][pol][threadIdx.x], c);
  }
}

// One 256-thread workgroup per (K-segment, polarity): suffix sums of the 256 bins from the top (a log-step scan in
// LDS); the bin d >= 1 whose suffix sum first reaches the wanted rank holds it, else it lies in the uncounted digit 0.
// The bucket is narrowed to that bin and the histogram cleared for the next pass.  After the last digit the prefix is
// the threshold: fold it into the running maxima and write the steps (amax, steps: [2][S], as the min/max calibration).
__global__ __launch_bounds__(256) void pct_select_kernel(PctState* __restrict__ st, int S, int shift, int last, int accumulate,
                                                         float* __restrict__ amax, float* __restrict__ steps) {
  const int i = blockIdx.x;                                  // grid: 2 S
  const int pol = i / S, ks = i - pol * S;
  const int d = threadIdx.x;
  unsigned int* h = st->hist[ks][pol];
  __shared__ unsigned int suf[256];
  const unsigned int own = d >= 1 ? h[d] : 0u;               // digit 0 is not counted
  h[d] = 0u;
  suf[d] = own;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {                  // suf[d] = sum of bins d .. 255
    const unsigned int add = d + off < 256 ? suf[d + off] : 0u;
    __syncthreads();
    suf[d] += add;
    __syncthreads();
  }
  const unsigned int r = st->rank[ks][pol], bucket = st->bucket[ks][pol], pre = st->prefix[ks][pol];
  const unsigned int above = d < 255 ? suf[d + 1] : 0u;      // elements in bins above d
  const unsigned int total = suf[1];                         // all counted elements (bins 1 .. 255)
  __syncthreads();
  // exactly one thread holds the rank: bin d >= 1 with above < r <= above + own, or d == 0 when r > total
  const bool mine = d >= 1 ? (above < r && r <= above + own) : (r > total);
  if (mine) {
    const unsigned int taken = d >= 1 ? above : total;
    const unsigned int npre = pre | ((unsigned int)d << shift);
    st->rank[ks][pol] = r - taken;
    st->bucket[ks][pol] = d >= 1 ? own : bucket - total;
    st->prefix[ks][pol] = npre;
    if (last) {
      const float t = __uint_as_float(npre);
      float a = accumulate ? amax[i] : 0.0f;
      a = __builtin_fmaxf(a, t);
      amax[i] = a;
      steps[i] = (a == 0.0f) ? 1.0f : a / kQmax;
    }
  }
}

hipError_t launch_calibrate_act_percentile(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, double p,
                                           float* amax, float* steps, void* workspace, bool accumulate, hipStream_t st) {
  PctState* ws = reinterpret_cast<PctState*>(workspace);
  PctRanks rk;
  for (int s = 0; s < tb.S; ++s) {
    const long long n = (long long)M * (tb.kseg_off[s + 1] - tb.kseg_off[s]);
    long long k = (long long)std::ceil(p * (double)n);      // nearest rank, in IEEE double
    k = k < 1 ? 1 : (k > n ? n : k);
    rk.n[s] = (unsigned int)n;
    rk.r[s] = (unsigned int)(n - k + 1);                    // k-th smallest = (n - k + 1)-th largest
  }
  const int nclear = tb.S * 2 * 256;
  hipLaunchKernelGGL(pct_init_kernel, dim3((nclear + 255) / 256), dim3(256), 0, st, ws, rk, tb.S);
  bool vec = (K % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) vec = vec && (tb.kseg_off[s] % 8 == 0);
  dim3 grid((M + kCalibRows - 1) / kCalibRows, tb.S);
  // digits of the magnitude bits, most significant first; a bf16 value has nothing below bit 16
  static const int kShift[4] = {23, 15, 7, 0};
  static const unsigned int kMask[4] = {0xFFu, 0xFFu, 0xFFu, 0x7Fu};
  const int npass = x_is_bf16 ? 2 : 4;
  for (int ps = 0; ps < npass; ++ps) {
    int shift = kShift[ps];
    unsigned int dmask = kMask[ps];
    if (x_is_bf16 && ps == 1) { shift = 16; dmask = 0x7Fu; }
    const unsigned int himask = 0x7FFFFFFFu & ~((dmask << shift) | ((1u << shift) - 1u));
#define SQ_PCT(B, V) hipLaunchKernelGGL((pct_hist_kernel<B, V>), grid, dim3(256), 0, st, x, M, K, tb, ws, shift, dmask, himask)
    if (x_is_bf16) { if (vec) SQ_PCT(true, true); else SQ_PCT(true, false); }
    else           { if (vec) SQ_PCT(false, true); else SQ_PCT(false, false); }
#undef SQ_PCT
    hipLaunchKernelGGL(pct_select_kernel, dim3(2 * tb.S), dim3(256), 0, st, ws, tb.S, shift,
                       ps == npass - 1 ? 1 : 0, accumulate ? 1 : 0, amax, steps);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// The same calibration for callers that cannot allocate or pass a workspace (HIP graph capture, serving loops,
// harnesses that forbid hipMalloc): the radix-select state lives in a file-scope device array.  Every device the
// library runs on holds its own copy of the array at its own address; the address is looked up once per device
// (with that device current) and used from then on — the array's name is a host-side stand-in, never a device
// address.  All calls on one device share the array: calls that overlap on a device race.  Nothing has to be zero
// on entry: pct_init_kernel clears the histograms and sets ranks, buckets and prefixes at the start of every call.
// ------------------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[sizeof(PctState)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

size_t calibrate_static_scratch_bytes() { return sizeof(PctState); }

hipError_t launch_calibrate_act_percentile_static(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, double p,
                                                  float* amax, float* steps, bool accumulate, hipStream_t st) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
      void* found = nullptr;
      e = hipGetSymbolAddress(&found, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (found == nullptr) return hipErrorInvalidSymbol;
      g_scratch_ptr[dev] = found;
    }
    ptr = g_scratch_ptr[dev];
  }
  return launch_calibrate_act_percentile(x, x_is_bf16, M, K, tb, p, amax, steps, ptr, accumulate, st);
}

}  // namespace sq
