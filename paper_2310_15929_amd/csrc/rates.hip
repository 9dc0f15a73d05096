// What the matrix pipes of this chip sustain when they have nothing else to do - the ceiling the product kernels are
// measured against beside the published peak.  One workgroup of 8 waves per CU (two waves per SIMD, as in the tile
// kernels) issues the matrix instruction of those kernels back to back, 16 per trip into 8 independent accumulator
// tiles, on operands that stay in registers: no LDS, no memory.  With operands of random mantissas and signs the chip
// holds a lower clock than with zeros (the multipliers' switching power counts against the board limit), so both are
// reported: the figure that matters for a product of real data is the first.
//
// mix > 0 adds, per trip of 16 multiplies (= one 64-channel stage of the 8-wave prefill kernel), what that kernel does
// beside them, without its data dependencies on memory:
//   mix 1: the stage's operand reads out of LDS (8 weight + 8 activation operands of 16 bytes per lane and 8 index
//          words per wave: 144 KiB per workgroup) feeding the multiplies;
//   mix 2: ... and the DMA of a coming stage's operands from an L2-resident region of global memory into LDS (6 copies
//          of 16 bytes per lane + 2 of 4 bytes per wave: 52 KiB per workgroup, each copy behind one multiply, none behind
//          the stage's last four), the stage's counted wait and its barrier.
// The rate of mix 2 is what this instruction mix can reach on the chip when every global access hits the L2 and nothing
// waits for data: the distance between it and a product kernel is the kernel's to close, the distance between it and
// mix 0 is not.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "common.h"

namespace {

typedef unsigned int esp_read4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t rate_hash(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

// two 16-bit values with random sign and mantissa and magnitude in [1, 2): fp16 0x3c00 | 10 mantissa bits, bf16 0x3f80 | 7
template <int DT>
__device__ __forceinline__ uint32_t rate_pair(uint32_t i) {
  const uint32_t r = rate_hash(i);
  return DT == ESPARSE_F16 ? ((r & 0x83ff83ffu) | 0x3c003c00u) : ((r & 0x807f807fu) | 0x3f803f80u);
}

struct RateOps {
  uint4 a[4];   // four weight operands
  uint4 b[2];   // one activation operand (the sparse instruction reads both halves, the dense one the first)
  int idx;
};

template <int DT, int SPARSE>
__device__ __forceinline__ floatx16_t rate_multiply(const RateOps& o, int m, floatx16_t c) {
#if defined(__HIP_DEVICE_COMPILE__)
  struct B2 {
    uint4 lo, hi;
  } bb = {o.b[0], o.b[1]};
  if (SPARSE) {
    if (DT == ESPARSE_F16)
      return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(half8_t, o.a[m]), __builtin_bit_cast(half16_t, bb), c, o.idx, 0, 0);
    return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8_t, o.a[m]), __builtin_bit_cast(bf16x16_t, bb), c, o.idx, 0, 0);
  }
  if (DT == ESPARSE_F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, o.a[m]), __builtin_bit_cast(half8_t, o.b[0]), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, o.a[m]), __builtin_bit_cast(bf16x8_t, o.b[0]), c, 0, 0, 0);
#else
  (void)o;
  (void)m;
  return c;
#endif
}

template <int DT, int SPARSE>
__global__ void __launch_bounds__(512) k_matrix_rate(int random_operands, int trips, float* __restrict__ sink) {
  const uint32_t id = blockIdx.x * 512u + threadIdx.x;
  RateOps o;
#pragma unroll
  for (int m = 0; m < 4; m++)
    o.a[m] = random_operands ? uint4{rate_pair<DT>(id * 24 + 4 * m), rate_pair<DT>(id * 24 + 4 * m + 1), rate_pair<DT>(id * 24 + 4 * m + 2),
                                     rate_pair<DT>(id * 24 + 4 * m + 3)}
                             : uint4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int h = 0; h < 2; h++)
    o.b[h] = random_operands ? uint4{rate_pair<DT>(id * 24 + 16 + 4 * h), rate_pair<DT>(id * 24 + 17 + 4 * h), rate_pair<DT>(id * 24 + 18 + 4 * h),
                                     rate_pair<DT>(id * 24 + 19 + 4 * h)}
                             : uint4{0u, 0u, 0u, 0u};
  // index pairs of a 2:4 operand: any two distinct positions per group; 0x4 = positions 0 and 1, 0xe = 2 and 3
  o.idx = random_operands ? (int)(0x4e4e4e4eu ^ (rate_hash(id) & 0x88888888u)) : 0x44444444;
  floatx16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) acc[i][j] = 0.f;
  for (int t = 0; t < trips; t++) {
#pragma unroll
    for (int g = 0; g < 4; g++)
#pragma unroll
      for (int m = 0; m < 4; m++) acc[(g & 1) * 4 + m] = rate_multiply<DT, SPARSE>(o, m, acc[(g & 1) * 4 + m]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) s += acc[i][j];
  sink[id] = s;
}


template <int DT, int MIX>
__global__ void __launch_bounds__(512) k_stage_rate(int trips, const uint4* __restrict__ gsrc, float* __restrict__ sink) {
  __shared__ uint4 s_rd[4096];  // 64 KiB the operand reads use: random values, written once
  __shared__ uint4 s_wr[4096];  // 64 KiB the DMA lands in, never read
  const int tid = threadIdx.x, lane = tid & 63;
#if defined(__HIP_DEVICE_COMPILE__)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#else
  const int wave = tid >> 6;
#endif
  const uint32_t id = blockIdx.x * 512u + threadIdx.x;
  for (int i = tid; i < 4096; i += 512)
    s_rd[i] = uint4{rate_pair<DT>(4 * i), rate_pair<DT>(4 * i + 1), rate_pair<DT>(4 * i + 2), rate_pair<DT>(4 * i + 3)};
  __syncthreads();
  const uint32_t* s_rd4 = reinterpret_cast<const uint32_t*>(s_rd);
  floatx16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) acc[i][j] = 0.f;
  // 64 lanes x 16 bytes per read, the 64 chunks of s_rd visited in an order that differs per wave and trip
  auto rd = [&](int x, int ph) -> uint4 { return s_rd[lane + 64 * ((wave * 8 + x + ph * 16) & 63)]; };
  auto rd4 = [&](int x, int ph) -> uint32_t { return s_rd4[lane + 64 * ((wave * 8 + x + ph * 16) & 255)]; };
  const uint4* gw = gsrc + ((size_t)blockIdx.x * 8 + wave) * 512 + lane;  // 8 KiB of global memory per wave
  uint4* dw = s_wr + wave * 512;
  constexpr int ND16 = 6, ND = 8;  // copies of 16 and (the rest) of 4 bytes per lane, per wave and stage
  for (int t = 0; t < trips; t++) {
    const int ph = t & 3;
    RateOps o;
#pragma unroll
    for (int i = 0; i < 4; i++) o.a[i] = rd(i, ph);
    uint32_t ix[4];
#pragma unroll
    for (int i = 0; i < 4; i++) ix[i] = rd4(i, ph);
    int issued = 0;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      o.b[0] = rd(8 + 2 * g, ph);
      o.b[1] = rd(9 + 2 * g, ph);
      if (g == 2) {  // the weight operands of the stage's second half
#pragma unroll
        for (int i = 0; i < 4; i++) {
          o.a[i] = rd(4 + i, ph);
          ix[i] = rd4(4 + i, ph);
        }
      }
#pragma unroll
      for (int m = 0; m < 4; m++) {
        o.idx = (int)ix[m];
        acc[(g & 1) * 4 + m] = rate_multiply<DT, 1>(o, m, acc[(g & 1) * 4 + m]);
        if (MIX >= 2 && g < 3 && m < 3 && issued < ND) {  // the order of the tile kernel: a copy after each of the first three
                                                            // multiplies of the first three groups of four
          const int q = issued++;
#if defined(__HIP_DEVICE_COMPILE__)
          if (q < ND16)
            __builtin_amdgcn_global_load_lds(gw + (((t * ND + q) & 7) * 64), dw + (q & 7) * 64, 16, 0, 0);
          else
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(gw + (((t * ND + q) & 7) * 64)),
                                             reinterpret_cast<uint32_t*>(dw + (q & 7) * 64), 4, 0, 0);
#endif
        }
      }
#if defined(__HIP_DEVICE_COMPILE__)
      __builtin_amdgcn_sched_barrier(0);
#endif
    }
#if defined(__HIP_DEVICE_COMPILE__)
    if (MIX >= 2) {
      __builtin_amdgcn_s_waitcnt((ND & 15) | ((ND >> 4) << 14) | 0x0070);  // vmcnt(ND): the newest stage's copies may be under way
      __builtin_amdgcn_s_barrier();
    }
#endif
  }
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no copy into this workgroup's LDS is left in flight
#endif
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) s += acc[i][j];
  sink[id] = s;
}


// plain streaming read: a workgroup of 16 waves reads a contiguous share of the buffer, 16 bytes per lane and load, four
// loads under way per thread; the values are folded into one word per thread so that the loads cannot be dropped
__global__ void __launch_bounds__(1024) k_read_rate(const uint4* __restrict__ src, size_t units_per_wg, uint32_t* __restrict__ sink) {
  const uint4* p = src + (size_t)blockIdx.x * units_per_wg;
  uint32_t f = 0u;
  size_t u = threadIdx.x;
  for (; u + 3072 < units_per_wg; u += 4096) {
    const esp_read4 a = __builtin_nontemporal_load(reinterpret_cast<const esp_read4*>(p + u));
    const esp_read4 b = __builtin_nontemporal_load(reinterpret_cast<const esp_read4*>(p + u + 1024));
    const esp_read4 c = __builtin_nontemporal_load(reinterpret_cast<const esp_read4*>(p + u + 2048));
    const esp_read4 d = __builtin_nontemporal_load(reinterpret_cast<const esp_read4*>(p + u + 3072));
    f ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; u < units_per_wg; u += 1024) {
    const esp_read4 a = __builtin_nontemporal_load(reinterpret_cast<const esp_read4*>(p + u));
    f ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  sink[blockIdx.x * 1024 + threadIdx.x] = f;
}

}  // namespace

int esp_matrix_rate_device(esparse_ctx* ctx, int sparse, int dtype, int random_operands, int mix, double* tflops) {
  int cus = 0;
  ESP_HIP(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device));
  if (cus < 1) return esp_fail(ctx, ESPARSE_EHIP, "the device reports no compute units");
  DevBuf sink, src;
  if (sink.alloc((size_t)cus * 512 * 4) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
  if (mix >= 2) {  // 64 KiB per workgroup: 2 MiB per XCD, which its L2 holds
    if (src.alloc((size_t)cus * 65536) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
    int rc = esp_fill_pattern_device(ctx, src.p, (size_t)cus * 65536);
    if (rc) return rc;
  }
  const int trips = 12000;  // 8 - 13 ms per launch
  hipEvent_t e0, e1;
  ESP_HIP(ctx, hipEventCreate(&e0));
  ESP_HIP(ctx, hipEventCreate(&e1));
  auto launch = [&]() {
#define ESP_RATE(DTv, SPv) \
  hipLaunchKernelGGL((k_matrix_rate<DTv, SPv>), dim3((unsigned)cus), dim3(512), 0, ctx->stream, random_operands, trips, sink.as<float>())
#define ESP_STAGE(DTv, MIXv) \
  hipLaunchKernelGGL((k_stage_rate<DTv, MIXv>), dim3((unsigned)cus), dim3(512), 0, ctx->stream, trips, src.as<uint4>(), sink.as<float>())
    if (mix == 0) {
      if (dtype == ESPARSE_F16) {
        if (sparse) ESP_RATE(ESPARSE_F16, 1);
        else ESP_RATE(ESPARSE_F16, 0);
      } else {
        if (sparse) ESP_RATE(ESPARSE_BF16, 1);
        else ESP_RATE(ESPARSE_BF16, 0);
      }
    } else if (mix == 1) {
      if (dtype == ESPARSE_F16) ESP_STAGE(ESPARSE_F16, 1);
      else ESP_STAGE(ESPARSE_BF16, 1);
    } else {
      if (dtype == ESPARSE_F16) ESP_STAGE(ESPARSE_F16, 2);
      else ESP_STAGE(ESPARSE_BF16, 2);
    }
#undef ESP_RATE
#undef ESP_STAGE
  };
  // two launches for the clocks to settle under this load, then three timed as one interval
  launch();
  launch();
  hipError_t e = hipEventRecord(e0, ctx->stream);
  for (int i = 0; i < 3 && e == hipSuccess; i++) launch();
  if (e == hipSuccess) e = hipGetLastError();
  if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  ESP_HIP(ctx, e);
  // effective (dense-equivalent) flops of one instruction: 2 x 32 x 32 x 32 for the 2:4 form, 2 x 32 x 32 x 16 dense
  const double per_instr = sparse ? 65536.0 : 32768.0;
  const double flops = 3.0 * (double)cus * 8.0 * (double)trips * 16.0 * per_instr;
  *tflops = ms > 0.f ? flops / ((double)ms * 1e-3) / 1e12 : 0.0;
  return ESPARSE_OK;
}

// What the memory system gives a plain read of `bytes` bytes in one launch, cold: the launches walk through a buffer
// larger than the last-level cache, so every launch reads from HBM.  The decode kernels read 1.125 N K bytes per launch
// and can be no faster than this for their size (launch, ramp-up and drain are a fixed few microseconds).
int esp_read_rate_device(esparse_ctx* ctx, size_t bytes, double* gbs) {
  // one workgroup of 1024 threads per compute unit: the fastest of the grids tried (103 MB per launch: 17.0 us against
  // 18.6 with 2048 workgroups of 256 threads and 20.5 with 8192; 19 MB: 5.0 against 5.1 and 6.8)
  int cus = 0;
  ESP_HIP(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device));
  if (cus < 1) return esp_fail(ctx, ESPARSE_EHIP, "the device reports no compute units");
  const size_t wgs = std::min<size_t>((size_t)cus, std::max<size_t>(1, bytes / 16384));  // at least 16 KiB per workgroup
  const size_t units_per_wg = (bytes / 16 + wgs - 1) / wgs;
  const size_t span = wgs * units_per_wg * 16;                                    // bytes one launch reads
  const size_t ncopies = std::max<size_t>(2, ((size_t)640 << 20) / span + 1);
  DevBuf buf, sink;
  if (buf.alloc(span * ncopies) != hipSuccess || sink.alloc(wgs * 1024 * 4) != hipSuccess)
    return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
  int rc = esp_fill_pattern_device(ctx, buf.p, span * ncopies);
  if (rc) return rc;
  hipEvent_t e0, e1;
  ESP_HIP(ctx, hipEventCreate(&e0));
  ESP_HIP(ctx, hipEventCreate(&e1));
  const int reps = 24;
  auto launch = [&](int i) {
    const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(buf.p) + (size_t)(i % ncopies) * span);
    hipLaunchKernelGGL(k_read_rate, dim3((unsigned)wgs), dim3(1024), 0, ctx->stream, src, units_per_wg, sink.as<uint32_t>());
  };
  for (int i = 0; i < 4; i++) launch(i);
  hipError_t e = hipEventRecord(e0, ctx->stream);
  for (int i = 0; i < reps && e == hipSuccess; i++) launch(i + 4);
  if (e == hipSuccess) e = hipGetLastError();
  if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  ESP_HIP(ctx, e);
  *gbs = ms > 0.f ? (double)span * reps / ((double)ms * 1e-3) / 1e9 : 0.0;
  return ESPARSE_OK;
}
