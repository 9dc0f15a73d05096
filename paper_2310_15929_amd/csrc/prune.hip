// Offline pruning stage on the GPU: channel statistics (Section 3.2, eq. 1-2), pruning metric
// (eq. 3), global naive shuffle and local block shuffle (Section 3.3, Algorithm 1), n:m mask.
//
// Everything that decides an integer (a bin, a rank, an exchange, a kept position) is computed so
// that the result does not depend on the order in which threads run:
//   - histogram counts, minima and maxima are integer / ordered-integer atomics;
//   - sums of squares and column sums of |w| are accumulated EXACTLY: every term is split by its
//     binary exponent into one of a few 64-bit integer accumulators (16 exponents per accumulator),
//     and the host adds the accumulators exactly and rounds once;
//   - the retained metric of a candidate group is summed over the output rows in a FIXED order (16
//     interleaved sub-sums, see ROW_LANES) in float64 without contraction, so repeated runs make the
//     same exchanges; eq. (5) fixes no order for that sum, and the exchanges Algorithm 1 makes do not
//     hinge on it where candidates are not tied to the last bit (the tests compare them with a plain
//     ascending-row sum);
//   - logs, square roots and the sort of K channel means run on the host (K values each).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <thread>

#include "common.h"

// ------------------------------------------------------------------------------------------------
// exact exponent-binned accumulation
// ------------------------------------------------------------------------------------------------
// squares of 16-bit values: exponent in [-266, 255], at most 22 significant bits
#define SQ_NB 33
#define SQ_EOFF 272
#define SQ_SIG 21
// |w|: exponent in [-133, 127], at most 11 significant bits
#define AB_NB 17
#define AB_EOFF 144
#define AB_SIG 10

__device__ __forceinline__ void exact_bin(double v, int eoff, int sig, int* bin, unsigned long long* q) {
  // v > 0 finite.  bin = floor((e + eoff) / 16); q = v / 2^(16 bin - eoff - sig), an exact integer.
  int e = ilogb(v);
  int b = (e + eoff) >> 4;
  *bin = b;
  *q = (unsigned long long)ldexp(v, -(16 * b - eoff - sig));
}

__device__ __forceinline__ unsigned int ordered_bits(float f) {
  unsigned int u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ------------------------------------------------------------------------------------------------
// Channel statistics in two scans of the calibration features, each at memory speed.
// Both kernels: block 1024 = 32 column lanes of CPL channels (CPL = 4: 8-byte loads, needs K % 4 == 0;
// CPL = 2 otherwise) x 32 row lanes, eight rows in flight per thread; grid (ceil(K / (32 CPL)), row chunks).
//
// Scan A: per-channel min / max and the exact sum of squares.  A 16-bit value is m * 2^E with an integer m of
// at most 11 bits, so its square is the integer m * m at binary position 2 E: bin and quotient of the exponent-
// binned accumulation come from integer shifts (no float64 arithmetic, no ilogb / ldexp).
// Scan B: the histogram over [min, max].  The bin of x is floor(((x - lo) * bins) / (hi - lo)) evaluated in
// float64, clamped to bins - 1 (the definition).  A float32 estimate q of that quotient is at most 5e-5 off for
// bins <= 256 (three roundings of 2^-24 relative), the float64 quotient at most 2^-44: whenever q is farther
// than 1e-4 from the nearest integer both have the same floor, so only the lanes near a bin edge (and the lanes
// where the estimate overflowed) evaluate the definition itself.
// ------------------------------------------------------------------------------------------------
// bin and quotient of the square of a 16-bit value for the exponent-binned exact accumulation, from the bits of the
// (exact) floating-point square: fp16 squares have at most 22 significant bits and fit float32, bf16 squares have 16
// and fit float64 (their exponents go beyond float32).  With t = ilogb(x^2) + SQ_EOFF the bin is t / 16 and the
// quotient x^2 / 2^(16 bin - SQ_EOFF - SQ_SIG) is the square's integer significand shifted left by t % 16 (less than
// 2^37).  Zero gives quotient 0.
template <int DT>
__device__ __forceinline__ void square_bin(float x, unsigned int* bin, unsigned long long* q) {
  if (DT == ESPARSE_F16) {
    const float xs = x * x;
    const uint32_t bits = __float_as_uint(xs);
    const uint32_t t = (bits >> 23) + (uint32_t)(SQ_EOFF - 127);
    uint32_t mant = ((bits & 0x7fffffu) | 0x800000u) >> 2;  // 24-bit significand, its two low bits are zero: SQ_SIG + 1 = 22 bits
    mant = bits ? mant : 0u;
    *bin = t >> 4;
    *q = (unsigned long long)mant << (t & 15u);
  } else {
    const double xs = (double)x * (double)x;
    const uint32_t hi = (uint32_t)(__double_as_longlong(xs) >> 32);  // the low word of the significand is zero
    const uint32_t t = (hi >> 20) + (uint32_t)(SQ_EOFF - 1023);
    uint32_t mant = (hi & 0xfffffu) | 0x100000u;  // top 21 bits of the significand
    mant = hi ? mant : 0u;
    *bin = t >> 4;
    *q = (unsigned long long)mant << ((t & 15u) + 1u);
  }
}

// the 16-bit values of ROWS rows (32 rows apart) x CPL channels of one thread; FULL: all rows exist, else rows past the
// end are replaced by the thread's first row (callers give those no weight)
template <int CPL, int ROWS, bool FULL>
__device__ __forceinline__ void load_rows(const uint16_t* __restrict__ p, long long stride32, long long rb, long long r1,
                                          uint32_t (&w)[ROWS][CPL / 2]) {
#pragma unroll
  for (int u = 0; u < ROWS; u++) {
    const uint16_t* src = (FULL || rb + 32 * u < r1) ? p + u * stride32 : p;
    if (CPL == 4) {
      const uint2 v = *reinterpret_cast<const uint2*>(src);
      w[u][0] = v.x;
      w[u][1 % (CPL / 2)] = v.y;
    } else {
      w[u][0] = *reinterpret_cast<const uint32_t*>(src);
    }
  }
}

template <int DT, int CPL, int ROWS, bool FULL>
__device__ __forceinline__ void minmax_sumsq_trip(const uint16_t* __restrict__ p, long long stride32, long long rb, long long r1,
                                                  float (&lo)[CPL], float (&hi)[CPL], unsigned long long* s_sq_lane, int want_sq) {
  uint32_t w[ROWS][CPL / 2];
  load_rows<CPL, ROWS, FULL>(p, stride32, rb, r1, w);
#pragma unroll
  for (int u = 0; u < ROWS; u++) {
    // a repeated row changes neither min nor max; its square is replaced by zero (no branches in this loop)
    const bool live = FULL || rb + 32 * u < r1;
#pragma unroll
    for (int j = 0; j < CPL; j++) {
      const float x = esp_to_float<DT>((uint16_t)(w[u][j / 2] >> (16 * (j & 1))));
      lo[j] = fminf(lo[j], x);
      hi[j] = fmaxf(hi[j], x);
      if (want_sq) {
        unsigned int bi;
        unsigned long long q;
        square_bin<DT>(live ? x : 0.0f, &bi, &q);
        atomicAdd(s_sq_lane + j * (32 * SQ_NB) + bi, q);
      }
    }
  }
}

template <int DT, int CPL>
__global__ void __launch_bounds__(1024) k_minmax_sumsq(const uint16_t* __restrict__ X, long long T, long long K,
                                                        long long rows_per_block, unsigned int* __restrict__ omin,
                                                        unsigned int* __restrict__ omax,
                                                        unsigned long long* __restrict__ sq /*[K][SQ_NB]*/, int want_sq) {
  constexpr int CH = 32 * CPL;  // channels per block
  // LDS row of a channel = j * 32 + cl (cl: column lane, j: which of the lane's CPL channels)
  __shared__ unsigned long long s_sq[CH * SQ_NB];
  __shared__ unsigned int s_lo[CH], s_hi[CH];
  const int tid = threadIdx.x, cl = tid & 31, rl = tid >> 5;
  for (int i = tid; i < CH * SQ_NB; i += 1024) s_sq[i] = 0ull;
  if (tid < CH) {
    s_lo[tid] = 0xffffffffu;
    s_hi[tid] = 0u;
  }
  __syncthreads();
  const long long c = ((long long)blockIdx.x * 32 + cl) * CPL;
  const long long r0 = (long long)blockIdx.y * rows_per_block;
  const long long r1 = r0 + rows_per_block < T ? r0 + rows_per_block : T;
  if (c < K && r0 + rl < r1) {
    float lo[CPL], hi[CPL];
#pragma unroll
    for (int j = 0; j < CPL; j++) {
      lo[j] = INFINITY;
      hi[j] = -INFINITY;
    }
    constexpr int ROWS = 8;
    const long long stride32 = 32 * K;
    const uint16_t* p = X + (r0 + rl) * K + c;
    unsigned long long* s_sq_lane = s_sq + cl * SQ_NB;
    long long rb = r0 + rl;
    for (; rb + 32 * (ROWS - 1) < r1; rb += 32 * ROWS, p += ROWS * stride32)
      minmax_sumsq_trip<DT, CPL, ROWS, true>(p, stride32, rb, r1, lo, hi, s_sq_lane, want_sq);
    if (rb < r1) minmax_sumsq_trip<DT, CPL, ROWS, false>(p, stride32, rb, r1, lo, hi, s_sq_lane, want_sq);
#pragma unroll
    for (int j = 0; j < CPL; j++) {
      atomicMin(&s_lo[j * 32 + cl], ordered_bits(lo[j]));
      atomicMax(&s_hi[j * 32 + cl], ordered_bits(hi[j]));
    }
  }
  __syncthreads();
  const long long cbase = (long long)blockIdx.x * CH;
  if (tid < CH && r0 < r1) {
    const long long ch = cbase + (long long)(tid & 31) * CPL + (tid >> 5);  // LDS row tid = j * 32 + cl
    if (ch < K) {
      atomicMin(&omin[ch], s_lo[tid]);
      atomicMax(&omax[ch], s_hi[tid]);
    }
  }
  if (want_sq)
    for (int i = tid; i < CH * SQ_NB; i += 1024) {
      const int row = i / SQ_NB;
      const long long ch = cbase + (long long)(row & 31) * CPL + (row >> 5);
      const unsigned long long v = s_sq[i];
      if (ch < K && v) atomicAdd(&sq[ch * SQ_NB + (i % SQ_NB)], v);
    }
}

__device__ __forceinline__ float float_from_ordered_bits(unsigned int o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}

__device__ __forceinline__ float fraction_of(float q) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_fractf(q);
#else
  return q - floorf(q);
#endif
}

// the float32 estimate of a value's bin and whether it can be trusted: farther than 1e-4 from both neighbouring
// integers and inside [0, bins)
__device__ __forceinline__ bool bin_estimate(float x, float lo32, float c32, int bins, int* bi) {
  const float q = (x - lo32) * c32;
  *bi = (int)q;
  return fabsf(fraction_of(q) - 0.5f) < 0.4999f && (unsigned int)*bi < (unsigned int)bins;
}

template <int DT, int CPL, int ROWS, bool FULL>
__device__ __forceinline__ void hist_trip(const uint16_t* __restrict__ p, long long stride32, long long rb, long long r1,
                                          const float (&lo32)[CPL], const float (&c32)[CPL], const double (&lo)[CPL],
                                          const double (&wd)[CPL], int bins, unsigned int* s_hist_lane, int row_stride) {
  uint32_t w[ROWS][CPL / 2];
  load_rows<CPL, ROWS, FULL>(p, stride32, rb, r1, w);
  // all estimates first, without branches (whether all can be trusted is kept in a lane mask, not in registers);
  // the rare values near a bin edge are redone afterwards from the definition
  int bsel[ROWS][CPL];
  bool all_ok = true;
#pragma unroll
  for (int u = 0; u < ROWS; u++)
#pragma unroll
    for (int j = 0; j < CPL; j++)
      all_ok &= bin_estimate(esp_to_float<DT>((uint16_t)(w[u][j / 2] >> (16 * (j & 1)))), lo32[j], c32[j], bins, &bsel[u][j]);
  if (!all_ok) {
    const double nb = (double)bins;
#pragma unroll
    for (int u = 0; u < ROWS; u++)
#pragma unroll
      for (int j = 0; j < CPL; j++) {
        const float x = esp_to_float<DT>((uint16_t)(w[u][j / 2] >> (16 * (j & 1))));
        int b;
        if (!bin_estimate(x, lo32[j], c32[j], bins, &b)) {
          b = 0;
          if (wd[j] > 0.0) {
            const double d = ((double)x - lo[j]) * nb / wd[j];  // the definition
            b = (int)floor(d);
            if (b > bins - 1) b = bins - 1;
          }
          bsel[u][j] = b;
        }
      }
  }
#pragma unroll
  for (int u = 0; u < ROWS; u++) {
    const unsigned int one = (FULL || rb + 32 * u < r1) ? 1u : 0u;  // a repeated row counts nothing
#pragma unroll
    for (int j = 0; j < CPL; j++) atomicAdd(s_hist_lane + j * (32 * row_stride) + bsel[u][j], one);
  }
}

template <int DT, int CPL>
__global__ void __launch_bounds__(1024) k_hist(const uint16_t* __restrict__ X, long long T, long long K,
                                                long long rows_per_block, int bins, const unsigned int* __restrict__ omin,
                                                const unsigned int* __restrict__ omax, unsigned int* __restrict__ hist /*[K][bins]*/) {
  constexpr int CH = 32 * CPL;
  extern __shared__ unsigned int s_hist[];  // [CH rows][stride]: the row of a channel is j * 32 + cl, the stride odd, so
  const int stride = bins | 1;              // that the column lanes of one instruction start in 32 different banks
  const int tid = threadIdx.x, cl = tid & 31, rl = tid >> 5;
  for (int i = tid; i < CH * stride; i += 1024) s_hist[i] = 0u;
  __syncthreads();
  const long long c = ((long long)blockIdx.x * 32 + cl) * CPL;
  const long long r0 = (long long)blockIdx.y * rows_per_block;
  const long long r1 = r0 + rows_per_block < T ? r0 + rows_per_block : T;
  if (c < K && r0 + rl < r1) {
    float lo32[CPL], c32[CPL];
    double lo[CPL], wd[CPL];
    const double nb = (double)bins;
#pragma unroll
    for (int j = 0; j < CPL; j++) {
      lo32[j] = float_from_ordered_bits(omin[c + j]);
      lo[j] = (double)lo32[j];
      wd[j] = (double)float_from_ordered_bits(omax[c + j]) - lo[j];
      // the estimate's factor; a constant channel (width 0) gets NaN, which sends every value to the definition
      c32[j] = wd[j] > 0.0 ? (float)(nb / wd[j]) : __uint_as_float(0x7fc00000u);
    }
    constexpr int ROWS = 8;
    const long long stride32 = 32 * K;
    const uint16_t* p = X + (r0 + rl) * K + c;
    unsigned int* s_hist_lane = s_hist + cl * stride;
    long long rb = r0 + rl;
    for (; rb + 32 * (ROWS - 1) < r1; rb += 32 * ROWS, p += ROWS * stride32)
      hist_trip<DT, CPL, ROWS, true>(p, stride32, rb, r1, lo32, c32, lo, wd, bins, s_hist_lane, stride);
    if (rb < r1) hist_trip<DT, CPL, ROWS, false>(p, stride32, rb, r1, lo32, c32, lo, wd, bins, s_hist_lane, stride);
  }
  __syncthreads();
  const long long cbase = (long long)blockIdx.x * CH;
  for (int i = tid; i < CH * bins; i += 1024) {
    const int row = i / bins, b = i - row * bins;
    const long long ch = cbase + (long long)(row & 31) * CPL + (row >> 5);
    const unsigned int v = s_hist[row * stride + b];
    if (ch < K && v) atomicAdd(&hist[ch * bins + b], v);
  }
}

// ------------------------------------------------------------------------------------------------
// exact column sums of |W|: grid (ceil(K/64), row chunks), block 256 = 8 row lanes x 32 channel pairs
// ------------------------------------------------------------------------------------------------
template <int DT>
__global__ void __launch_bounds__(256) k_abs_colsum(const uint16_t* __restrict__ W, long long N, long long K,
                                                     long long rows_per_block, unsigned long long* __restrict__ out /*[K][AB_NB]*/) {
  __shared__ unsigned long long s_acc[64 * AB_NB];
  const int tid = threadIdx.x;
  for (int i = tid; i < 64 * AB_NB; i += 256) s_acc[i] = 0ull;
  __syncthreads();
  const int cp = tid & 31, rl = tid >> 5;
  const long long c = (long long)blockIdx.x * 64 + cp * 2;
  if (c < K) {
    long long r0 = (long long)blockIdx.y * rows_per_block;
    long long r1 = r0 + rows_per_block < N ? r0 + rows_per_block : N;
    for (long long r = r0 + rl; r < r1; r += 8) {
      uint32_t two = *reinterpret_cast<const uint32_t*>(W + r * K + c);
      double x[2] = {fabs((double)esp_to_float<DT>((uint16_t)(two & 0xffffu))), fabs((double)esp_to_float<DT>((uint16_t)(two >> 16)))};
#pragma unroll
      for (int h = 0; h < 2; h++)
        if (x[h] > 0.0) {
          int bi;
          unsigned long long q;
          exact_bin(x[h], AB_EOFF, AB_SIG, &bi, &q);
          atomicAdd(&s_acc[(cp * 2 + h) * AB_NB + bi], q);
        }
    }
  }
  __syncthreads();
  const long long cbase = (long long)blockIdx.x * 64;
  for (int i = tid; i < 64 * AB_NB; i += 256) {
    long long ch = cbase + i / AB_NB;
    unsigned long long v = s_acc[i];
    if (ch < K && v) atomicAdd(&out[ch * AB_NB + (i % AB_NB)], v);
  }
}

// ------------------------------------------------------------------------------------------------
// host driver of the statistics
// ------------------------------------------------------------------------------------------------
int esp_stats_device(esparse_ctx* ctx, const void* calib, long long T, long long K, int dtype, int bins,
                     std::vector<double>* ir, std::vector<double>* am) {
  if (!ir && !am) return ESPARSE_OK;
  hipStream_t st = ctx->stream;
  DevBuf dmin, dmax, dhist, dsq;
  if (dmin.alloc(K * 4) != hipSuccess || dmax.alloc(K * 4) != hipSuccess ||
      dhist.alloc((size_t)K * bins * 4) != hipSuccess || dsq.alloc((size_t)K * SQ_NB * 8) != hipSuccess)
    return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation for channel statistics failed");
  ESP_HIP(ctx, hipMemsetAsync(dmin.p, 0xff, K * 4, st));
  ESP_HIP(ctx, hipMemsetAsync(dmax.p, 0x00, K * 4, st));
  ESP_HIP(ctx, hipMemsetAsync(dhist.p, 0, (size_t)K * bins * 4, st));
  ESP_HIP(ctx, hipMemsetAsync(dsq.p, 0, (size_t)K * SQ_NB * 8, st));
  const uint16_t* X = reinterpret_cast<const uint16_t*>(calib);
  const int cpl = K % 4 == 0 ? 4 : 2;  // channels per lane: 8-byte loads where the rows allow them
  const long long gx = (K + 32 * cpl - 1) / (32 * cpl);
  // about 1024 workgroups (four per CU over the two that fit at once), whole trips of 256 rows
  const long long nchunk = std::max<long long>(1, std::min<long long>((T + 255) / 256, 1024 / gx + 1));
  long long rpb = (T + nchunk - 1) / nchunk;
  rpb = (rpb + 255) / 256 * 256;
  dim3 grid((unsigned)gx, (unsigned)((T + rpb - 1) / rpb));
#define ESP_SCAN_A(DTv, CPLv)                                                                                        \
  hipLaunchKernelGGL((k_minmax_sumsq<DTv, CPLv>), grid, dim3(1024), 0, st, X, T, K, rpb, dmin.as<unsigned int>(),     \
                     dmax.as<unsigned int>(), dsq.as<unsigned long long>(), am ? 1 : 0)
#define ESP_SCAN_B(DTv, CPLv)                                                                                        \
  hipLaunchKernelGGL((k_hist<DTv, CPLv>), grid, dim3(1024), (size_t)32 * CPLv * (bins | 1) * 4, st, X, T, K, rpb, bins,     \
                     dmin.as<unsigned int>(), dmax.as<unsigned int>(), dhist.as<unsigned int>())
  if (dtype == ESPARSE_F16) {
    if (cpl == 4) ESP_SCAN_A(ESPARSE_F16, 4);
    else ESP_SCAN_A(ESPARSE_F16, 2);
  } else {
    if (cpl == 4) ESP_SCAN_A(ESPARSE_BF16, 4);
    else ESP_SCAN_A(ESPARSE_BF16, 2);
  }
  ESP_HIP(ctx, hipGetLastError());
  if (ir) {
    // 32 * 4 channels x 256 bins x 4 bytes = 128 KiB of LDS at most
    const size_t smem = (size_t)32 * cpl * (bins | 1) * 4;
    if (smem > 48 * 1024) {
      ESP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<ESPARSE_F16, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
      ESP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<ESPARSE_BF16, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
      ESP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<ESPARSE_F16, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
      ESP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<ESPARSE_BF16, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    }
    if (dtype == ESPARSE_F16) {
      if (cpl == 4) ESP_SCAN_B(ESPARSE_F16, 4);
      else ESP_SCAN_B(ESPARSE_F16, 2);
    } else {
      if (cpl == 4) ESP_SCAN_B(ESPARSE_BF16, 4);
      else ESP_SCAN_B(ESPARSE_BF16, 2);
    }
    ESP_HIP(ctx, hipGetLastError());
  }
#undef ESP_SCAN_A
#undef ESP_SCAN_B
  std::vector<unsigned int> hist;
  std::vector<unsigned long long> sq;
  if (ir) {
    hist.resize((size_t)K * bins);
    ESP_HIP(ctx, hipMemcpyAsync(hist.data(), dhist.p, hist.size() * 4, hipMemcpyDeviceToHost, st));
  }
  if (am) {
    sq.resize((size_t)K * SQ_NB);
    ESP_HIP(ctx, hipMemcpyAsync(sq.data(), dsq.p, sq.size() * 8, hipMemcpyDeviceToHost, st));
  }
  ESP_HIP(ctx, hipStreamSynchronize(st));
  if (ir) {
    // eq. 1: IR_c = - sum_k p_k ln p_k, ascending k, empty bins skipped
    ir->assign((size_t)K, 0.0);
    auto entropy_of = [&](long long c0, long long c1) {
      for (long long c = c0; c < c1; c++) {
        double acc = 0.0;
        for (int k = 0; k < bins; k++) {
          unsigned int nk = hist[(size_t)c * bins + k];
          if (nk) {
            double p = (double)nk / (double)T;
            double t = p * std::log(p);
            acc = acc + t;
          }
        }
        (*ir)[c] = -acc;
      }
    };
    // K * bins logarithms on the host (the host's log is the one the result is defined by): channels are independent
    const int nthr = (int)std::max<long long>(1, std::min<long long>(8, K * bins / 65536));
    std::vector<std::thread> pool;
    for (int i = 1; i < nthr; i++) pool.emplace_back(entropy_of, K * i / nthr, K * (i + 1) / nthr);
    entropy_of(0, K / nthr);
    for (auto& th : pool) th.join();
  }
  if (am) {
    // eq. 2: AM_c = sqrt(exact sum of squares rounded once)
    am->assign((size_t)K, 0.0);
    for (long long c = 0; c < K; c++)
      (*am)[c] = std::sqrt(esp_exact_bins_to_double(&sq[(size_t)c * SQ_NB], SQ_NB, -SQ_EOFF - SQ_SIG));
  }
  return ESPARSE_OK;
}

// ------------------------------------------------------------------------------------------------
// local block shuffle
// ------------------------------------------------------------------------------------------------
// Panel: P[j][p] = |W[j, theta0[p]]| as raw 16-bit magnitudes, p in GNS order (so the B channels of a
// block are contiguous in every row).
template <int DT>
__global__ void __launch_bounds__(256) k_build_panel(const uint16_t* __restrict__ W, const int32_t* __restrict__ theta0,
                                                      long long N, long long K, uint16_t* __restrict__ P) {
  long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= N * K) return;
  long long j = e / K, p = e % K;
  P[e] = W[j * K + theta0[p]] & 0x7fffu;
}

template <int NKEEP, int MG>
__device__ __forceinline__ double top_n_sum(double* v) {
  // the NKEEP largest of v[0..MG), added largest first
#pragma unroll
  for (int a = 0; a < NKEEP; a++) {
#pragma unroll
    for (int b = MG - 1; b > a; b--) {
      // bubble the maximum of v[a..MG) to v[a]
      double hi = fmax(v[b - 1], v[b]), lo = fmin(v[b - 1], v[b]);
      v[b - 1] = hi;
      v[b] = lo;
    }
  }
  double t = v[0];
#pragma unroll
  for (int a = 1; a < NKEEP; a++) t = t + v[a];
  return t;
}

// Order of every sum over output rows (eq. 5 prescribes none): ROW_LANES = 16 interleaved sub-sums -
// sub-sum l adds the rows j = l, l + 16, l + 32, ... in ascending order - which are then added in
// ascending l.  A fixed order that 16 lanes can work on at once; the lanes of one sum are 16
// neighbouring lanes of a wave.  It differs from an ascending-row sum in the last bits only.
#define ROW_LANES 16

__device__ __forceinline__ double lanes_total(double part) {
  // lane 0 of each group of 16 neighbouring lanes gets ((part_0 + part_1) + part_2) + ... + part_15
  double acc = __shfl(part, 0, ROW_LANES);
#pragma unroll
  for (int l = 1; l < ROW_LANES; l++) acc = acc + __shfl(part, l, ROW_LANES);
  return acc;
}

// V[blk][g][i][x] = retained metric of group g of block blk with its i-th member replaced by panel
// column x of the block (x == the member itself gives v(g)).  grid (entries / 64, blocks), block 1024 =
// 64 entries x 16 row lanes.  `groups` = list of 2 group numbers per block to refresh (or NULL = all
// groups).  Entries whose x sits in group g (other than the member itself) are skipped.
// The block's metric values go through LDS in chunks of rows_chunk rows (a multiple of 16; rows are
// padded by one value so that the 16 row lanes of an entry read different banks); the panel values of
// the next chunk are loaded into registers before the current chunk is evaluated.
template <int DT, int NKEEP, int MG>
__global__ void __launch_bounds__(1024) k_lbs_eval(const uint16_t* __restrict__ P, const double* __restrict__ sp /*[K] score in panel order*/,
                                                    const int* __restrict__ lp /*[nblk][B] position -> panel column*/,
                                                    const int* __restrict__ groups /*[nblk][2] or null*/,
                                                    const int* __restrict__ done /*[nblk]*/, long long N, long long K, int B,
                                                    int rows_chunk, double* __restrict__ V /*[nblk][G][MG][B]*/) {
  extern __shared__ unsigned char smem_raw[];
  double* s_xi = reinterpret_cast<double*>(smem_raw);  // [rows_chunk][B + 1]
  __shared__ int s_lp[1024];
  const int blk = blockIdx.y;
  if (done[blk]) return;
  const int G = B / MG;
  const int tid = threadIdx.x;
  const int rl = tid & (ROW_LANES - 1);                  // row lane
  const int eid = blockIdx.x * 64 + (tid >> 4);          // entry within this block's refresh list
  const int per_group = MG * B;
  const int ngroups = groups ? 2 : G;
  const int stride = B + 1;
  for (int i = tid; i < B; i += 1024) s_lp[i] = lp[blk * B + i];
  __syncthreads();
  bool active = eid < ngroups * per_group;
  int g = 0, i = 0, x = 0;
  int cols[MG];
#pragma unroll
  for (int k = 0; k < MG; k++) cols[k] = 0;
  if (active) {
    int gsel = eid / per_group;
    g = groups ? groups[blk * 2 + gsel] : gsel;
    i = (eid / B) % MG;
    x = eid % B;
    if (g < 0) active = false;
  }
  if (active) {
    bool in_group = false;
#pragma unroll
    for (int k = 0; k < MG; k++) {
      int ck = s_lp[g * MG + k];
      if (ck == x && k != i) in_group = true;
      cols[k] = (k == i) ? x : ck;
    }
    if (in_group) active = false;
  }
  const uint16_t* Pb = P + (long long)blk * B;
  const double* spb = sp + (long long)blk * B;
  // this thread's share of a chunk: values tid, tid + 1024, ... of the rows_chunk x B values (the same
  // places in every chunk)
  constexpr int EPT = 4;
  const int elems = rows_chunk * B;  // <= EPT * 1024: the host picks rows_chunk <= 4096 / B (B <= 256)
  uint16_t nextv[EPT];
  int rq[EPT], cq[EPT];
  double sq[EPT];
#pragma unroll
  for (int q = 0; q < EPT; q++) {
    const int e = tid + 1024 * q;
    rq[q] = e < elems ? e / B : rows_chunk;  // rows_chunk = "no such value"
    cq[q] = e % B;
    sq[q] = spb[cq[q]];
  }
  auto fetch = [&](long long r0) {
    const int nr = (int)((N - r0) < rows_chunk ? (N - r0) : rows_chunk);
#pragma unroll
    for (int q = 0; q < EPT; q++) nextv[q] = (rq[q] < nr) ? Pb[(r0 + rq[q]) * K + cq[q]] : (uint16_t)0;
  };
  double acc = 0.0;  // this lane's sub-sum
  fetch(0);
  for (long long r0 = 0; r0 < N; r0 += rows_chunk) {
    const int nr = (int)((N - r0) < rows_chunk ? (N - r0) : rows_chunk);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < EPT; q++)
      if (rq[q] < nr) s_xi[rq[q] * stride + cq[q]] = (double)esp_to_float<DT>(nextv[q]) * sq[q];
    __syncthreads();
    if (r0 + rows_chunk < N) fetch(r0 + rows_chunk);
    if (active) {
      // rows r0 + rl, r0 + rl + 16, ...: r0 is a multiple of 16, so they are this lane's rows
#pragma unroll 4
      for (int rr = rl; rr < nr; rr += ROW_LANES) {
        double v[MG];
#pragma unroll
        for (int k = 0; k < MG; k++) v[k] = s_xi[rr * stride + cols[k]];
        acc = acc + top_n_sum<NKEEP, MG>(v);
      }
    }
  }
  const double total = lanes_total(active ? acc : 0.0);
  if (active && rl == 0) V[(((long long)blk * G + g) * MG + i) * B + x] = total;
}

// The same table for 2:4, several times faster.  The B candidates x of one (group g, member i)
// combination share the group's three other members, so the two largest of those three are found
// once per row (m1 >= m2) and a candidate's retained metric in that row is
// max(m1, xi_x) + max(m2, min(m1, xi_x)): the two largest of the four values, the same two doubles
// the general network adds.  A workgroup (1024 threads = up to 64 candidates x 16 row lanes) stages the
// block's metric values once per chunk and evaluates NC units with them; a unit is a combination and
// a slice of XL = min(B, 64) candidates.  grid (ceil(units / NC), blocks); B % 64 == 0 or B < 64.
template <int DT, int NC>
__global__ void __launch_bounds__(1024) k_lbs_eval_2_4(const uint16_t* __restrict__ P, const double* __restrict__ sp,
                                                        const int* __restrict__ lp, const int* __restrict__ groups,
                                                        const int* __restrict__ done, long long N, long long K, int B, int rows_chunk,
                                                        double* __restrict__ V) {
  constexpr int MG = 4;
  extern __shared__ unsigned char smem_raw[];
  double* s_xi = reinterpret_cast<double*>(smem_raw);  // [rows_chunk][B + 1]
  __shared__ int s_lp[256];
  const int blk = blockIdx.y;
  if (done[blk]) return;
  const int G = B / MG;
  const int tid = threadIdx.x;
  const int rl = tid & (ROW_LANES - 1), xl = tid >> 4;
  const int XL = B < 64 ? B : 64, xslices = B / XL;
  const int ngroups = groups ? 2 : G;
  const int nunits = ngroups * MG * xslices;
  const int stride = B + 1;
  double* s_pair = s_xi + (size_t)rows_chunk * stride;  // [NC][rows_chunk][2]: the 16 row lanes read 256 contiguous bytes
  for (int i = tid; i < B; i += 1024) s_lp[i] = lp[blk * B + i];
  __syncthreads();
  // per unit: group, member, candidate of this thread, and whether the entry exists
  int ug[NC], ui[NC], ux[NC];
  bool uact[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) {
    const int u = blockIdx.x * NC + c;
    const int cmb = u / xslices;
    ux[c] = (u % xslices) * XL + xl;
    ui[c] = cmb % MG;
    const int gsel = cmb / MG;
    ug[c] = -1;
    if (u < nunits) ug[c] = groups ? groups[blk * 2 + gsel] : gsel;
    uact[c] = ug[c] >= 0 && xl < XL;
    if (!uact[c]) ux[c] = 0;
    if (uact[c]) {
#pragma unroll
      for (int k = 0; k < MG; k++)
        if (k != ui[c] && s_lp[ug[c] * MG + k] == ux[c]) uact[c] = false;  // x is another member of the group
    }
  }
  const uint16_t* Pb = P + (long long)blk * B;
  const double* spb = sp + (long long)blk * B;
  constexpr int EPT = 4;
  const int elems = rows_chunk * B;  // <= EPT * 1024
  uint16_t nextv[EPT];
  int rq[EPT], cq[EPT];
  double sq[EPT];
#pragma unroll
  for (int q = 0; q < EPT; q++) {
    const int e = tid + 1024 * q;
    rq[q] = e < elems ? e / B : rows_chunk;
    cq[q] = e % B;
    sq[q] = spb[cq[q]];
  }
  auto fetch = [&](long long r0) {
    const int nr = (int)((N - r0) < rows_chunk ? (N - r0) : rows_chunk);
#pragma unroll
    for (int q = 0; q < EPT; q++) nextv[q] = (rq[q] < nr) ? Pb[(r0 + rq[q]) * K + cq[q]] : (uint16_t)0;
  };
  double acc[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) acc[c] = 0.0;
  fetch(0);
  for (long long r0 = 0; r0 < N; r0 += rows_chunk) {
    const int nr = (int)((N - r0) < rows_chunk ? (N - r0) : rows_chunk);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < EPT; q++)
      if (rq[q] < nr) s_xi[rq[q] * stride + cq[q]] = (double)esp_to_float<DT>(nextv[q]) * sq[q];
    __syncthreads();
    if (r0 + rows_chunk < N) fetch(r0 + rows_chunk);
    for (int t = tid; t < nr * NC; t += 1024) {
      const int row = t / NC, c = t % NC;
      const int u = blockIdx.x * NC + c;
      const int cmb = u / xslices, mi = cmb % MG, gsel = cmb / MG;
      double m1 = 0.0, m2 = 0.0;
      if (u < nunits) {
        const int gg = groups ? groups[blk * 2 + gsel] : gsel;
        if (gg >= 0) {
          double o[3];
          int c3 = 0;
#pragma unroll
          for (int k = 0; k < MG; k++)
            if (k != mi) o[c3++] = s_xi[row * stride + s_lp[gg * MG + k]];
          const double hi = fmax(o[0], o[1]), lo = fmin(o[0], o[1]);
          m1 = fmax(hi, o[2]);
          m2 = fmax(lo, fmin(hi, o[2]));
        }
      }
      s_pair[2 * (c * rows_chunk + row)] = m1;
      s_pair[2 * (c * rows_chunk + row) + 1] = m2;
    }
    __syncthreads();
    // rows r0 + rl, r0 + rl + 16, ...: r0 is a multiple of 16, so they are this lane's rows
    for (int rr = rl; rr < nr; rr += ROW_LANES) {
#pragma unroll
      for (int c = 0; c < NC; c++) {  // entries that do not exist compute along (column 0) and are dropped at the end
        const double xv = s_xi[rr * stride + ux[c]];
        const double2 mm = *reinterpret_cast<const double2*>(s_pair + 2 * (c * rows_chunk + rr));
        acc[c] = acc[c] + (fmax(mm.x, xv) + fmax(mm.y, fmin(mm.x, xv)));
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NC; c++) {
    const double total = lanes_total(uact[c] ? acc[c] : 0.0);
    if (uact[c] && rl == 0) V[(((long long)blk * G + ug[c]) * MG + ui[c]) * B + ux[c]] = total;
  }
}

// One workgroup per block: best exchange (largest delta, ties -> smallest (i, j)), applied if delta > 0.
template <int MG>
__global__ void __launch_bounds__(256) k_lbs_select(const double* __restrict__ V, int* __restrict__ lp, int* __restrict__ groups,
                                                     int* __restrict__ done, long long* __restrict__ swaps, long long max_swaps,
                                                     int B, int* __restrict__ n_active) {
  const int blk = blockIdx.x;
  if (done[blk]) return;
  const int G = B / MG;
  const int tid = threadIdx.x;
  __shared__ int s_lp[256];
  __shared__ double s_best[256];
  __shared__ int s_pair[256];
  for (int i = tid; i < B; i += 256) s_lp[i] = lp[blk * B + i];
  __syncthreads();
  const double* Vb = V + (long long)blk * G * MG * B;
  double best = 0.0;
  int best_pair = -1;
  for (int pid = tid; pid < B * B; pid += 256) {  // pid = i * B + j, ascending per thread
    int i = pid / B, j = pid % B;
    int a = i / MG, b = j / MG;
    if (j <= i || a == b) continue;
    double va2 = Vb[((a * MG) + (i % MG)) * B + s_lp[j]];
    double vb2 = Vb[((b * MG) + (j % MG)) * B + s_lp[i]];
    double va = Vb[(a * MG) * B + s_lp[a * MG]];
    double vb = Vb[(b * MG) * B + s_lp[b * MG]];
    double delta = (va2 + vb2) - (va + vb);
    if (delta > 0.0 && (best_pair < 0 || delta > best)) {
      best = delta;
      best_pair = pid;
    }
  }
  s_best[tid] = best;
  s_pair[tid] = best_pair;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      double ob = s_best[tid + s];
      int op = s_pair[tid + s];
      int mp = s_pair[tid];
      if (op >= 0 && (mp < 0 || ob > s_best[tid] || (ob == s_best[tid] && op < mp))) {
        s_best[tid] = ob;
        s_pair[tid] = op;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    int pr = s_pair[0];
    if (pr < 0) {
      done[blk] = 1;
      atomicSub(n_active, 1);
    } else {
      int i = pr / B, j = pr % B;
      int ci = s_lp[i], cj = s_lp[j];
      lp[blk * B + i] = cj;
      lp[blk * B + j] = ci;
      groups[blk * 2 + 0] = i / MG;
      groups[blk * 2 + 1] = j / MG;
      long long sw = swaps[blk] + 1;
      swaps[blk] = sw;
      if (max_swaps > 0 && sw >= max_swaps) {
        done[blk] = 1;
        atomicSub(n_active, 1);
      }
    }
  }
}

__global__ void k_lbs_init(int* lp, int* done, long long* swaps, int nblk, int B) {
  int t = blockIdx.x * 256 + threadIdx.x;
  if (t < nblk * B) lp[t] = t % B;
  if (t < nblk) {
    done[t] = 0;
    swaps[t] = 0;
  }
}

__global__ void k_lbs_final_theta(const int32_t* theta0, const int* lp, int B, long long K, int32_t* theta) {
  long long p = (long long)blockIdx.x * 256 + threadIdx.x;
  if (p >= K) return;
  long long blk = p / B;
  theta[p] = theta0[blk * B + lp[p]];
}

// ------------------------------------------------------------------------------------------------
// n:m mask on the final order, one thread per (row, group); ties -> lower position kept
// ------------------------------------------------------------------------------------------------
template <int DT, int NKEEP, int MG>
__global__ void __launch_bounds__(256) k_nm_mask(const uint16_t* __restrict__ W, const double* __restrict__ s /*original order*/,
                                                  const int32_t* __restrict__ theta, long long N, long long K,
                                                  uint8_t* __restrict__ mask) {
  const long long ng = K / MG;
  long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= N * ng) return;
  long long j = e / ng, g = e % ng;
  double xi[MG];
#pragma unroll
  for (int k = 0; k < MG; k++) {
    int c = theta[g * MG + k];
    xi[k] = fabs((double)esp_to_float<DT>(W[j * K + c])) * s[c];
  }
  uint8_t out[MG];
#pragma unroll
  for (int k = 0; k < MG; k++) {
    int ahead = 0;
#pragma unroll
    for (int q = 0; q < MG; q++) ahead += (xi[q] > xi[k] || (xi[q] == xi[k] && q < k)) ? 1 : 0;
    out[k] = ahead < NKEEP ? 1 : 0;
  }
  uint8_t* dst = mask + j * K + g * MG;
  if (MG == 4) {
    *reinterpret_cast<uint32_t*>(dst) = (uint32_t)out[0] | ((uint32_t)out[1] << 8) | ((uint32_t)out[2] << 16) | ((uint32_t)out[3] << 24);
  } else {
#pragma unroll
    for (int k = 0; k < MG; k++) dst[k] = out[k];
  }
}

// retained metric of every group under the final order (eq. 5 terms), rows summed in order
template <int DT, int NKEEP, int MG>
__global__ void __launch_bounds__(64) k_group_values(const uint16_t* __restrict__ W, const double* __restrict__ s,
                                                      const int32_t* __restrict__ theta, long long N, long long K,
                                                      double* __restrict__ out) {
  // 4 groups per workgroup, 16 row lanes per group
  const int rl = threadIdx.x & (ROW_LANES - 1);
  const long long g = (long long)blockIdx.x * 4 + (threadIdx.x >> 4);
  const bool active = g < K / MG;
  int c[MG];
  double sc[MG];
#pragma unroll
  for (int k = 0; k < MG; k++) {
    c[k] = active ? theta[g * MG + k] : 0;
    sc[k] = active ? s[c[k]] : 0.0;
  }
  double acc = 0.0;
  if (active) {
    for (long long j = rl; j < N; j += ROW_LANES) {
      double v[MG];
#pragma unroll
      for (int k = 0; k < MG; k++) v[k] = fabs((double)esp_to_float<DT>(W[j * K + c[k]])) * sc[k];
      acc = acc + top_n_sum<NKEEP, MG>(v);
    }
  }
  const double total = lanes_total(acc);
  if (active && rl == 0) out[g] = total;
}

// ------------------------------------------------------------------------------------------------
// host driver: GNS -> LBS -> mask
// ------------------------------------------------------------------------------------------------
#define DISPATCH_DT_NM(dtype, n, KERNEL, ...)                                      \
  do {                                                                             \
    if ((dtype) == ESPARSE_F16 && (n) == 2) KERNEL(ESPARSE_F16, 2, 4, __VA_ARGS__); \
    else if ((dtype) == ESPARSE_F16) KERNEL(ESPARSE_F16, 4, 8, __VA_ARGS__);        \
    else if ((n) == 2) KERNEL(ESPARSE_BF16, 2, 4, __VA_ARGS__);                     \
    else KERNEL(ESPARSE_BF16, 4, 8, __VA_ARGS__);                                   \
  } while (0)

int esp_prune_device(esparse_ctx* ctx, const double* score, const void* Wv, long long N, long long K, int dtype,
                     const esparse_prune_opts* o, int32_t* perm_out, uint8_t* mask_out, int64_t* swaps_out,
                     double* retained_out) {
  hipStream_t st = ctx->stream;
  const uint16_t* W = reinterpret_cast<const uint16_t*>(Wv);
  const int n = o->n_keep, m = o->m_group;
  const bool use_gns = o->flags & ESPARSE_USE_GNS, use_lbs = o->flags & ESPARSE_USE_LBS;
  const int B = o->block;
  const long long nblk = use_lbs ? K / B : 0;
  if (swaps_out && !use_lbs && o->block > 0 && K % o->block == 0) memset(swaps_out, 0, sizeof(int64_t) * (K / o->block));

  DevBuf d_s;
  if (d_s.alloc(K * 8) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
  ESP_HIP(ctx, hipMemcpyAsync(d_s.p, score, K * 8, hipMemcpyHostToDevice, st));

  // ---- global naive shuffle: g_c = (s_c * sum_j |w_jc|) / N, stable descending sort, round-robin deal
  std::vector<int32_t> theta0((size_t)K);
  if (use_gns) {
    DevBuf d_cs;
    if (d_cs.alloc((size_t)K * AB_NB * 8) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
    ESP_HIP(ctx, hipMemsetAsync(d_cs.p, 0, (size_t)K * AB_NB * 8, st));
    long long nchunk = std::max<long long>(1, std::min<long long>(N / 64, 1024 / std::max<long long>(1, (K + 63) / 64) + 1));
    long long rpb = ((N + nchunk - 1) / nchunk + 7) / 8 * 8;
    dim3 grid((unsigned)((K + 63) / 64), (unsigned)((N + rpb - 1) / rpb));
    if (dtype == ESPARSE_F16)
      hipLaunchKernelGGL(k_abs_colsum<ESPARSE_F16>, grid, dim3(256), 0, st, W, N, K, rpb, d_cs.as<unsigned long long>());
    else
      hipLaunchKernelGGL(k_abs_colsum<ESPARSE_BF16>, grid, dim3(256), 0, st, W, N, K, rpb, d_cs.as<unsigned long long>());
    ESP_HIP(ctx, hipGetLastError());
    std::vector<unsigned long long> cs((size_t)K * AB_NB);
    ESP_HIP(ctx, hipMemcpyAsync(cs.data(), d_cs.p, cs.size() * 8, hipMemcpyDeviceToHost, st));
    ESP_HIP(ctx, hipStreamSynchronize(st));
    std::vector<double> g((size_t)K);
    for (long long c = 0; c < K; c++) {
      double colsum = esp_exact_bins_to_double(&cs[(size_t)c * AB_NB], AB_NB, -AB_EOFF - AB_SIG);
      double t = score[c] * colsum;
      g[c] = t / (double)N;
    }
    std::vector<int32_t> order((size_t)K);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return g[a] > g[b]; });
    const long long G = K / m;
    for (long long r = 0; r < K; r++) theta0[(size_t)((r % G) * m + r / G)] = order[(size_t)r];
  } else {
    std::iota(theta0.begin(), theta0.end(), 0);
  }
  DevBuf d_theta0;
  if (d_theta0.alloc(K * 4) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
  ESP_HIP(ctx, hipMemcpyAsync(d_theta0.p, theta0.data(), K * 4, hipMemcpyHostToDevice, st));

  // ---- local block shuffle
  if (use_lbs) {
    const int G = B / m;
    DevBuf d_P, d_sp, d_lp, d_groups, d_done, d_swaps, d_V, d_nact;
    std::vector<double> sp((size_t)K);
    for (long long p = 0; p < K; p++) sp[p] = score[theta0[p]];
    if (d_P.alloc((size_t)N * K * 2) != hipSuccess || d_sp.alloc(K * 8) != hipSuccess || d_lp.alloc(K * 4) != hipSuccess ||
        d_groups.alloc(nblk * 8) != hipSuccess || d_done.alloc(nblk * 4) != hipSuccess || d_swaps.alloc(nblk * 8) != hipSuccess ||
        d_V.alloc((size_t)nblk * G * m * B * 8) != hipSuccess || d_nact.alloc(4) != hipSuccess)
      return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation for the block shuffle failed");
    ESP_HIP(ctx, hipMemcpyAsync(d_sp.p, sp.data(), K * 8, hipMemcpyHostToDevice, st));
    {
      dim3 grid((unsigned)((N * K + 255) / 256));
      if (dtype == ESPARSE_F16)
        hipLaunchKernelGGL(k_build_panel<ESPARSE_F16>, grid, dim3(256), 0, st, W, d_theta0.as<int32_t>(), N, K, d_P.as<uint16_t>());
      else
        hipLaunchKernelGGL(k_build_panel<ESPARSE_BF16>, grid, dim3(256), 0, st, W, d_theta0.as<int32_t>(), N, K, d_P.as<uint16_t>());
      ESP_HIP(ctx, hipGetLastError());
    }
    hipLaunchKernelGGL(k_lbs_init, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, d_lp.as<int>(), d_done.as<int>(),
                       d_swaps.as<long long>(), (int)nblk, B);
    int nact = (int)nblk;
    ESP_HIP(ctx, hipMemcpyAsync(d_nact.p, &nact, 4, hipMemcpyHostToDevice, st));
    // rows per LDS chunk: a multiple of the 16 row lanes, about 4096 metric values (at most 16 per thread)
    const int rows_chunk = std::max(16, (4096 / B) / 16 * 16);
    const size_t smem = (size_t)rows_chunk * (B + 1) * 8;
    bool first = true;
    long long iter = 0;
    while (nact > 0) {
      const int entries = (first ? G : 2) * m * B;
      const int* grp = first ? nullptr : d_groups.as<int>();
      if (n == 2 && m == 4 && (B % 64 == 0 || B < 64)) {
        // 2:4: 8 units per workgroup while every group is evaluated, 2 in the refresh rounds (more workgroups)
        const int units = (first ? G : 2) * m * (B < 64 ? 1 : B / 64);
        const int nc = first ? 8 : 2;
        dim3 grid((unsigned)((units + nc - 1) / nc), (unsigned)nblk);
        const size_t smem2 = (size_t)rows_chunk * (B + 1) * 8 + (size_t)rows_chunk * nc * 16;
#define LAUNCH_EVAL24(DTv, NCv)                                                                                             \
  hipLaunchKernelGGL((k_lbs_eval_2_4<DTv, NCv>), grid, dim3(1024), smem2, st, d_P.as<uint16_t>(), d_sp.as<double>(), d_lp.as<int>(), \
                     grp, d_done.as<int>(), N, K, B, rows_chunk, d_V.as<double>())
        if (dtype == ESPARSE_F16) {
          if (first) LAUNCH_EVAL24(ESPARSE_F16, 8);
          else LAUNCH_EVAL24(ESPARSE_F16, 2);
        } else {
          if (first) LAUNCH_EVAL24(ESPARSE_BF16, 8);
          else LAUNCH_EVAL24(ESPARSE_BF16, 2);
        }
#undef LAUNCH_EVAL24
      } else {
        dim3 grid((unsigned)((entries + 63) / 64), (unsigned)nblk);
#define LAUNCH_EVAL(DT, NK, MGv, ...)                                                                                  \
  hipLaunchKernelGGL((k_lbs_eval<DT, NK, MGv>), grid, dim3(1024), smem, st, d_P.as<uint16_t>(), d_sp.as<double>(), d_lp.as<int>(), \
                     grp, d_done.as<int>(), N, K, B, rows_chunk, d_V.as<double>())
        DISPATCH_DT_NM(dtype, n, LAUNCH_EVAL, 0);
#undef LAUNCH_EVAL
      }
      ESP_HIP(ctx, hipGetLastError());
      if (m == 4)
        hipLaunchKernelGGL(k_lbs_select<4>, dim3((unsigned)nblk), dim3(256), 0, st, d_V.as<double>(), d_lp.as<int>(), d_groups.as<int>(),
                           d_done.as<int>(), d_swaps.as<long long>(), o->max_swaps, B, d_nact.as<int>());
      else
        hipLaunchKernelGGL(k_lbs_select<8>, dim3((unsigned)nblk), dim3(256), 0, st, d_V.as<double>(), d_lp.as<int>(), d_groups.as<int>(),
                           d_done.as<int>(), d_swaps.as<long long>(), o->max_swaps, B, d_nact.as<int>());
      ESP_HIP(ctx, hipGetLastError());
      ESP_HIP(ctx, hipMemcpyAsync(&nact, d_nact.p, 4, hipMemcpyDeviceToHost, st));
      ESP_HIP(ctx, hipStreamSynchronize(st));
      first = false;
      if (++iter > (long long)B * B * 64)
        return esp_fail(ctx, ESPARSE_EHIP, "block shuffle did not terminate after %lld rounds", iter);
    }
    hipLaunchKernelGGL(k_lbs_final_theta, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, d_theta0.as<int32_t>(), d_lp.as<int>(), B,
                       K, perm_out);
    ESP_HIP(ctx, hipGetLastError());
    if (swaps_out) {
      ESP_HIP(ctx, hipMemcpyAsync(swaps_out, d_swaps.p, nblk * 8, hipMemcpyDeviceToHost, st));
    }
    ESP_HIP(ctx, hipStreamSynchronize(st));
  } else {
    ESP_HIP(ctx, hipMemcpyAsync(perm_out, d_theta0.p, K * 4, hipMemcpyDeviceToDevice, st));
  }

  // ---- n:m mask under the final order
  {
    dim3 grid((unsigned)((N * (K / m) + 255) / 256));
#define LAUNCH_MASK(DT, NK, MGv, ...) \
  hipLaunchKernelGGL((k_nm_mask<DT, NK, MGv>), grid, dim3(256), 0, st, W, d_s.as<double>(), perm_out, N, K, mask_out)
    DISPATCH_DT_NM(dtype, n, LAUNCH_MASK, 0);
#undef LAUNCH_MASK
    ESP_HIP(ctx, hipGetLastError());
  }
  if (retained_out) {
    DevBuf d_gv;
    const long long ng = K / m;
    if (d_gv.alloc(ng * 8) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
    dim3 grid((unsigned)((ng + 3) / 4));
#define LAUNCH_GV(DT, NK, MGv, ...) \
  hipLaunchKernelGGL((k_group_values<DT, NK, MGv>), grid, dim3(64), 0, st, W, d_s.as<double>(), perm_out, N, K, d_gv.as<double>())
    DISPATCH_DT_NM(dtype, n, LAUNCH_GV, 0);
#undef LAUNCH_GV
    ESP_HIP(ctx, hipGetLastError());
    std::vector<double> gv((size_t)ng);
    ESP_HIP(ctx, hipMemcpyAsync(gv.data(), d_gv.p, ng * 8, hipMemcpyDeviceToHost, st));
    ESP_HIP(ctx, hipStreamSynchronize(st));
    double tot = 0.0;
    for (long long g = 0; g < ng; g++) tot = tot + gv[g];
    *retained_out = tot;
  }
  ESP_HIP(ctx, hipStreamSynchronize(st));
  return ESPARSE_OK;
}
