// Sparse (2:4, v_smfmac) and dense (v_mfma) products Y[M,N] = X[M,K] . W[N,K]^T on gfx950
// (Section 4 of the paper: the Sparse-GEMM and its dense baseline, Table 5).
//
// Operand layouts of the matrix instructions used here (wave of 64 lanes, lane l, c = l % 16,
// g = l / 16), measured on the hardware with one-hot operands:
//   v_mfma_f32_16x16x32_{f16,bf16}    A: row c, k = 8 g + e (e = 0..7)      B: column c, k = 8 g + e
//   v_smfmac_f32_16x16x64_{f16,bf16}  A: row c, the 8 kept values of channels [16 g, 16 g + 16) in
//                                        order; value e sits at channel 16 g + 4 (e / 2) + idx_e where
//                                        idx_e = bits [2e+1 : 2e] of the low (ABID = 0) or high
//                                        (ABID = 1) half of the index register of the SAME lane
//                                     B: column c, e < 8 : k = 8 g + e ;  e >= 8 : k = 32 + 8 g + (e - 8)
//                                        (two B operands of the dense 16x16x32 instruction back to back)
//   both                              D: column c, rows 4 g + j (j = 0..3)
// W is the A operand (rows of D = output features), the activations are the B operand (columns of
// D = tokens), so D is a 16 x 16 tile of Y^T.
//
// Memory formats
//   sparse weights ("native"): see include/esparse.h; the 16-byte unit u = (rt * nks + ks) * 64 + l is
//     exactly what lane l feeds to the instruction for row tile rt and 64-channel step ks, and the
//     8-byte index unit (rt * nks/4 + ks/4) * 64 + l holds the lane's index halves of 4 steps.
//   dense weights (packed): 16-byte unit (rt * ns + s) * 64 + l for 32-channel step s.
//   activations ("fragment-major" X', built by k_gather_x in the workspace): 16-byte unit
//     (tt * ns + s) * 64 + l = tokens 16 tt + c, re-ordered channels 32 s + 8 g .. + 7, i.e. the B
//     operand of the dense instruction for token tile tt and step s; the channel re-ordering theta
//     of Section 3.3 is applied here (X'[t, p] = X[t, theta[p]]), zero padded in both directions.
#include <algorithm>
#include <cstring>
#include <cstdlib>
#include <atomic>

#include "common.h"

#define WS_HEADER_BYTES 65536
#define MAX_SPLIT 16
// Kernels that need more than the default 64 KiB of dynamic LDS have that limit raised once per device; `done` is the
// kernel's own mask of the devices where that has happened.
template <class F>
static hipError_t raise_dynamic_lds(std::atomic<unsigned long long>& done, int device, F* kernel, size_t bytes) {
  const unsigned long long bit = 1ull << (device & 63);
  if (device < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && device < 64) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// fp32 partial tiles the workspace has room for: 16 K splits up to 128 tokens, 4 up to 512, none beyond
static inline int esp_split_capacity(long long M) { return M <= 128 ? MAX_SPLIT : (M <= 512 ? 4 : 1); }
#define ESP_MAX_GROUP 4  // products of one shape that may share a launch

// ------------------------------------------------------------------------------------------------
// device-only intrinsics (hipcc also parses kernels in its host pass, where these do not exist)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int wave_uniform(int v) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_readfirstlane(v);
#else
  return v;
#endif
}
// 16 bytes per lane from global memory straight into LDS: lane l lands at lds_wave_base + 16 l
__device__ __forceinline__ void global_to_lds_16(const uint4* gsrc, uint4* lds_wave_base) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(gsrc, lds_wave_base, 16, 0, 0);
#else
  (void)gsrc;
  (void)lds_wave_base;
#endif
}
// scheduling hint: the next SIZE instructions of class MASK (0x008 matrix, 0x100 LDS read) form one
// group; consecutive groups are issued in the order the hints are written
template <int MASK, int SIZE>
__device__ __forceinline__ void sched_group() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_sched_group_barrier(MASK, SIZE, 0);
#endif
}
// 4 bytes per lane from global memory straight into LDS: lane l lands at lds_wave_base + 4 l
__device__ __forceinline__ void global_to_lds_4(const uint32_t* gsrc, uint32_t* lds_wave_base) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(gsrc, lds_wave_base, 4, 0, 0);
#else
  (void)gsrc;
  (void)lds_wave_base;
#endif
}
// streaming load: the line is not kept in the caches once read (weights are read once per product)
typedef unsigned int esp_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream_16(const uint4* p) {
  const esp_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const esp_u32x4*>(p));
  return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ uint32_t load_stream_4(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void sched_fence() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_sched_barrier(0);
#endif
}
// NM matrix instructions with ND copies into LDS and NA LDS reads spread evenly among them: after each multiply one copy
// and a share of the reads.  A matrix instruction occupies its pipe for 16 or 32 clocks, during which the wave can issue
// other work; issued in bursts (all multiplies, then all copies, then all reads) the copies queue up at the
// vector-memory issue while the matrix pipe runs dry - measured 5-6 % slower on the prefill shapes.  READS_FIRST: the
// reads ahead of the copy in each slot (same-box comparisons: 2 % faster for the 8-wave 32x32x32 kernel, 4-8 % slower
// for the 4-wave kernel with its deeper operand read-ahead, no difference for the other 8-wave kernels).
template <int NM, int ND, int NA, bool READS_FIRST = false>
__device__ __forceinline__ void sched_spread() {
  constexpr int AP = (NA + NM - 1) / NM;
#pragma unroll
  for (int p = 0; p < NM; p++) {
    sched_group<0x008, 1>();
    if (READS_FIRST && AP > 0) sched_group<0x100, AP>();
    if (p < ND) sched_group<0x010, 1>();
    if (!READS_FIRST && AP > 0) sched_group<0x100, AP>();
  }
  if (ND > NM) sched_group<0x010, ND - NM>();
}

// ------------------------------------------------------------------------------------------------
// instruction wrappers
// ------------------------------------------------------------------------------------------------
template <int DT, int ABID>
__device__ __forceinline__ floatx4_t smfmac16(uint4 a, uint4 b0, uint4 b1, floatx4_t c, int idx) {
  struct B2 {
    uint4 lo, hi;
  } bb = {b0, b1};
  if (DT == ESPARSE_F16) {
    return __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half16_t, bb), c, idx, 0, ABID);
  } else {
    return __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x16_t, bb), c, idx, 0, ABID);
  }
}

// byte permute: byte i of the result is byte sel[i] of {hi, lo} (0-3: lo, 4-7: hi) or 0x00 for sel[i] = 0x0c
__device__ __forceinline__ uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_perm(hi, lo, sel);
#else
  (void)hi;
  (void)lo;
  (void)sel;
  return 0;
#endif
}

// 4:8: byte-permute selectors that spread a group's 4 kept values over its 8 positions, one 16-byte entry per pattern
// code (the index of the group's bitmap among the 70 bitmaps with four bits set, in ascending order - what the native
// form stores per group): output half e takes value number popcount(bitmap below bit e) if bit e is set and 0 otherwise
// (selector byte 0x0c yields 0x00).  COPIES copies of the table stand side by side, entry code * COPIES + c: with
// COPIES = 16 and c = lane % 16 the 16 lanes that one pass of a 16-byte LDS read serves fall into 16 different groups of
// four banks whatever their codes are (measured: the rate of a conflict-free read; one copy: half of it).
// Threads 0 .. 255 of the workgroup take one bitmap each; the caller synchronises.
constexpr int LUT48_CODES = 70;
template <int COPIES>
__device__ __forceinline__ void fill_expand_lut(uint4* s_lut, int tid) {
  if (tid < 256 && __builtin_popcount(tid) == 4) {
    uint32_t sel[4] = {0x0c0c0c0cu, 0x0c0c0c0cu, 0x0c0c0c0cu, 0x0c0c0c0cu};
    int code = 0, r = 0;
#pragma unroll
    for (int e = 0; e < 8; e++)
      if ((tid >> e) & 1) {
        const int sh = 16 * (e & 1);
        sel[e >> 1] = (sel[e >> 1] & ~(0xffffu << sh)) | (((2u * r) | ((2u * r + 1u) << 8)) << sh);
        r++;
        int c = 1;  // C(e, r): bitmaps below this one that agree with it above bit e and have a zero at bit e
        for (int t = 0; t < r; t++) c = c * (e - t) / (t + 1);
        code += c;
      }
    for (int c = 0; c < COPIES; c++) s_lut[code * COPIES + c] = uint4{sel[0], sel[1], sel[2], sel[3]};
  }
}

// the dense operands of the two half steps of a 4:8 unit: v.x, v.y hold the 4 kept values of the first group of 8, v.z, v.w
// those of the second; codes = the two pattern codes (bits 0-7, 8-15); copy = the lane's copy of the table
template <int COPIES>
__device__ __forceinline__ void expand_4_8(const uint4 v, uint32_t codes, const uint4* s_lut, unsigned copy, uint4& e0, uint4& e1) {
  const unsigned c0 = codes & 0xffu, c1 = (codes >> 8) & 0xffu;  // a code past the table (corrupt input) reads the last entry
  const uint4 s0 = s_lut[(c0 < LUT48_CODES ? c0 : LUT48_CODES - 1) * COPIES + copy];
  const uint4 s1 = s_lut[(c1 < LUT48_CODES ? c1 : LUT48_CODES - 1) * COPIES + copy];
  e0 = uint4{byte_perm(v.y, v.x, s0.x), byte_perm(v.y, v.x, s0.y), byte_perm(v.y, v.x, s0.z), byte_perm(v.y, v.x, s0.w)};
  e1 = uint4{byte_perm(v.w, v.z, s1.x), byte_perm(v.w, v.z, s1.y), byte_perm(v.w, v.z, s1.z), byte_perm(v.w, v.z, s1.w)};
}

template <int DT>
__device__ __forceinline__ floatx4_t mfma16(uint4 a, uint4 b, floatx4_t c) {
  if (DT == ESPARSE_F16) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
}

// ------------------------------------------------------------------------------------------------
// activation staging: X[M,K] (original channel order) -> fragment-major X' through theta
// one thread per 16-byte unit
// ------------------------------------------------------------------------------------------------
// Up to ESP_MAX_GROUP products of one shape go through one launch (blockIdx.y picks the member): at
// decode sizes a product of a 4096 x 4096 matrix is a 5 us kernel, mostly launch and ramp-up.
struct GatherArgs {
  const uint16_t* X[ESP_MAX_GROUP];
  const int32_t* perm[ESP_MAX_GROUP];
  uint4* Xf[ESP_MAX_GROUP];
};
struct KsplitArgs {
  const uint4* A[ESP_MAX_GROUP];
  const uint16_t* meta16[ESP_MAX_GROUP];
  const uint4* Xf[ESP_MAX_GROUP];
  uint16_t* Y[ESP_MAX_GROUP];
  float* partial;  // single products with K split over workgroups (gridDim.z > 1): fp32 partial tiles [split][Mp][Np]
  int sps;         // ... and the steps per split
  // FOLD kernels (one or two tokens): the activations in original channel order and theta; the workgroup gathers them itself
  const uint16_t* X[ESP_MAX_GROUP];
  const int32_t* perm[ESP_MAX_GROUP];
  long long K;
};

// mc > 0 (at most 16 tokens): a second, compact copy follows the fragment-major one (units [units, units + mc Kp / 8)):
// unit (8-channel unit) * mc + token for tokens 0 .. mc - 1 only - the decode kernels then load the real tokens'
// 16 bytes instead of a 16-token tile that is mostly padding.
__global__ void __launch_bounds__(256) k_gather_x(GatherArgs args, long long M, long long K, long long Kp, long long units, int mc) {
  const uint16_t* __restrict__ X = args.X[blockIdx.y];
  const int32_t* __restrict__ perm = args.perm[blockIdx.y];
  uint4* __restrict__ Xf = args.Xf[blockIdx.y];
  long long u = (long long)blockIdx.x * 256 + threadIdx.x;
  if (u >= units + (long long)mc * (Kp / 8)) return;
  long long t, k0;
  if (u >= units) {
    t = (u - units) % mc;
    k0 = ((u - units) / mc) * 8;
  } else {
    const int lane = (int)(u & 63);
    const long long ns = Kp / 32;
    const long long s = (u >> 6) % ns, tt = (u >> 6) / ns;
    t = tt * 16 + (lane & 15);
    k0 = s * 32 + (lane >> 4) * 8;
  }
  uint16_t v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (t < M && k0 < K) {
    const uint16_t* xr = X + t * K;
    if (perm) {
      if (k0 + 8 <= K) {
        const int4 p0 = *reinterpret_cast<const int4*>(perm + k0);
        const int4 p1 = *reinterpret_cast<const int4*>(perm + k0 + 4);
        v[0] = xr[p0.x];
        v[1] = xr[p0.y];
        v[2] = xr[p0.z];
        v[3] = xr[p0.w];
        v[4] = xr[p1.x];
        v[5] = xr[p1.y];
        v[6] = xr[p1.z];
        v[7] = xr[p1.w];
      } else {
        for (int e = 0; e < 8; e++)
          if (k0 + e < K) v[e] = xr[perm[k0 + e]];
      }
    } else {
      for (int e = 0; e < 8; e++)
        if (k0 + e < K) v[e] = xr[k0 + e];
    }
  }
  uint4 o;
  o.x = v[0] | ((uint32_t)v[1] << 16);
  o.y = v[2] | ((uint32_t)v[3] << 16);
  o.z = v[4] | ((uint32_t)v[5] << 16);
  o.w = v[6] | ((uint32_t)v[7] << 16);
  Xf[u] = o;
}

// The same staging for many tokens: a workgroup copies TOK whole rows of X into LDS with coalesced
// 16-byte reads and gathers through theta out of LDS (the element-wise gather above reads 2 bytes per
// lane from 64 different cache lines per instruction).  Rows are padded by 8 elements so that the TOK
// tokens of one channel sit in different banks.  Lane l of a wave works on token l % TOK and 8-channel
// unit l / TOK, so consecutive lanes write consecutive 16-byte units of X'.  Needs K % 8 == 0.
template <int TOK>
__global__ void __launch_bounds__(512) k_gather_rows(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm, long long M,
                                                      long long Mp, long long K, long long Kp, uint4* __restrict__ Xf) {
  extern __shared__ uint4 s_rows4[];
  uint16_t* s_rows = reinterpret_cast<uint16_t*>(s_rows4);
  const int tid = threadIdx.x;
  // Workgroups b, b + 8, b + 16, ... run on one XCD (round-robin dispatch): the 16 / TOK workgroups whose tokens
  // share a token tile - and with it every 256-byte run of X' - are numbered that way, so that their 16 TOK-byte
  // pieces meet in that XCD's L2 and leave it as whole lines
  constexpr int PER = 16 / TOK;
  const long long j = blockIdx.x / 8;
  const long long tile = (j / PER) * 8 + blockIdx.x % 8;
  const long long t0 = tile * 16 + (j % PER) * TOK;
  if (t0 >= Mp) return;
  const int stride = (int)K + 8;
  const long long nrows = (M - t0) < TOK ? (M - t0 > 0 ? M - t0 : 0) : TOK;
  const int kc = (int)(K / 8);  // 16-byte chunks per row
  const uint4* src = reinterpret_cast<const uint4*>(X + t0 * K);
  for (int i = tid; i < (int)nrows * kc; i += 512) {
    const int row = i / kc, col = i - row * kc;
    s_rows4[(row * stride) / 8 + col] = src[i];
  }
  __syncthreads();
  constexpr int UPW = 64 / TOK;  // units per wave and pass
  const int lane = tid & 63, wave = tid >> 6;
  const int c = lane % TOK, q = lane / TOK;
  const long long t = t0 + c;
  const long long ns = Kp / 32;
  const long long obase = (t / 16) * ns * 64 + (t % 16);
  const uint16_t* row = s_rows + c * stride;
  const bool live = t < M;
  const int nunits = (int)(Kp / 8);
  for (int u = wave * UPW + q; u < nunits; u += 8 * UPW) {
    const int k0 = u * 8;
    uint16_t v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (live && k0 < K) {  // K % 8 == 0: a unit is entirely inside or outside the real channels
      if (perm) {
        const int4 p0 = *reinterpret_cast<const int4*>(perm + k0);
        const int4 p1 = *reinterpret_cast<const int4*>(perm + k0 + 4);
        v[0] = row[p0.x];
        v[1] = row[p0.y];
        v[2] = row[p0.z];
        v[3] = row[p0.w];
        v[4] = row[p1.x];
        v[5] = row[p1.y];
        v[6] = row[p1.z];
        v[7] = row[p1.w];
      } else {
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = row[k0 + e];
      }
    }
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    // unit u = 4 s32 + g of token tile t / 16: X' unit (tt ns + s32) 64 + 16 g + t % 16
    Xf[obase + (long long)(u >> 2) * 64 + (u & 3) * 16] = o;
  }
}

// ------------------------------------------------------------------------------------------------
// epilogue helpers
// ------------------------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void store_y4(uint16_t* __restrict__ Y, long long M, long long N, long long t, long long n,
                                         floatx4_t acc) {
  if (t >= M) return;
  uint16_t h[4];
#pragma unroll
  for (int j = 0; j < 4; j++) h[j] = esp_from_float<DT>(acc[j]);
  uint16_t* dst = Y + t * N + n;
  if ((N & 3) == 0 && n + 3 < N) {
    uint2 v;
    v.x = h[0] | ((uint32_t)h[1] << 16);
    v.y = h[2] | ((uint32_t)h[3] << 16);
    *reinterpret_cast<uint2*>(dst) = v;
  } else {
#pragma unroll
    for (int j = 0; j < 4; j++)
      if (n + j < N) dst[j] = h[j];
  }
}

// partial[split][t][n] (fp32, padded Mp x Np) -> Y, splits added in ascending order
template <int DT>
__global__ void __launch_bounds__(256) k_reduce_splits(const float* __restrict__ partial, int nsplit, long long M, long long N,
                                                        long long Mp, long long Np, uint16_t* __restrict__ Y) {
  const long long n4 = Np / 4;
  long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= M * n4) return;
  const long long t = e / n4, n = (e % n4) * 4;
  floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < nsplit; s++) {
    const floatx4_t v = *reinterpret_cast<const floatx4_t*>(partial + ((long long)s * Mp + t) * Np + n);
    acc += v;
  }
  store_y4<DT>(Y, M, N, t, n, acc);
}

// partial[piece][t][n] -> Y for the stream kernels: the steps of all row blocks (rows_per_block rows, nks steps
// each) form one sequence cut into spans of `span` steps, one per workgroup; row block rb is covered by the
// spans first(rb) .. last(rb), whose partial tiles are pieces 0 .. last - first, added in ascending order.
// A row block inside a single span was stored to Y by its workgroup and is skipped here.
template <int DT>
__global__ void __launch_bounds__(256) k_reduce_pieces(const float* __restrict__ partial, long long M, long long N, long long Mp,
                                                        long long Np, uint16_t* __restrict__ Y, long long nks, long long span,
                                                        long long rows_per_block) {
  const long long n4 = Np / 4;
  long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= M * n4) return;
  const long long t = e / n4, n = (e % n4) * 4;
  const long long rb = n / rows_per_block;
  const long long first = (rb * nks) / span, last = ((rb + 1) * nks - 1) / span;
  if (first == last) return;
  floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (long long s = 0; s <= last - first; s++) {
    const floatx4_t v = *reinterpret_cast<const floatx4_t*>(partial + (s * Mp + t) * Np + n);
    acc += v;
  }
  store_y4<DT>(Y, M, N, t, n, acc);
}

// ------------------------------------------------------------------------------------------------
// variant "wave-tile": every wave owns RT row tiles x TT token tiles x one K split and streams
// both operands straight from global memory (fragment-major, 16 bytes per lane, fully coalesced).
// No LDS, no barriers.  Items are numbered with the row block fastest.
// ------------------------------------------------------------------------------------------------
template <int DT, int SPARSE, int RT, int TT>
__global__ void __launch_bounds__(256) k_mm_wave_tile(const uint4* __restrict__ A, const uint2* __restrict__ meta,
                                                       const uint4* __restrict__ Xf, uint16_t* __restrict__ Y,
                                                       float* __restrict__ partial, long long M, long long N, long long Mp,
                                                       long long Np, long long Kp, int nsplit, int steps_per_split,
                                                       long long n_items) {
  const int lane = threadIdx.x & 63;
  const long long item = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= n_items) return;
  const long long nrt = Np / 16, ntt = Mp / 16;
  const long long nrb = (nrt + RT - 1) / RT, ntb = (ntt + TT - 1) / TT;
  const long long rb = item % nrb;
  const long long tb = (item / nrb) % ntb;
  const int split = (int)(item / (nrb * ntb));
  const long long nks = Kp / 64;  // 64-channel steps
  const long long ks0 = (long long)split * steps_per_split;
  const long long ks1 = (ks0 + steps_per_split < nks) ? ks0 + steps_per_split : nks;

  floatx4_t acc[RT][TT];
#pragma unroll
  for (int i = 0; i < RT; i++)
#pragma unroll
    for (int j = 0; j < TT; j++) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  long long rts[RT], tts[TT];
#pragma unroll
  for (int i = 0; i < RT; i++) {
    long long rt = rb * RT + i;
    rts[i] = rt < nrt ? rt : nrt - 1;  // clamp: duplicate work, discarded in the epilogue
  }
#pragma unroll
  for (int j = 0; j < TT; j++) {
    long long tt = tb * TT + j;
    tts[j] = tt < ntt ? tt : ntt - 1;
  }

  for (long long ks = ks0; ks < ks1; ks += 4) {
    if (SPARSE) {
      uint2 md[RT];
#pragma unroll
      for (int i = 0; i < RT; i++) md[i] = meta[(rts[i] * (nks / 4) + ks / 4) * 64 + lane];
#pragma unroll
      for (int q = 0; q < 4; q++) {
        uint4 a[RT], b0[TT], b1[TT];
#pragma unroll
        for (int i = 0; i < RT; i++) a[i] = A[(rts[i] * nks + ks + q) * 64 + lane];
#pragma unroll
        for (int j = 0; j < TT; j++) {
          b0[j] = Xf[(tts[j] * (2 * nks) + 2 * (ks + q)) * 64 + lane];
          b1[j] = Xf[(tts[j] * (2 * nks) + 2 * (ks + q) + 1) * 64 + lane];
        }
#pragma unroll
        for (int i = 0; i < RT; i++) {
          const int idx = (int)((q < 2) ? md[i].x : md[i].y);
#pragma unroll
          for (int j = 0; j < TT; j++) {
            if (q & 1)
              acc[i][j] = smfmac16<DT, 1>(a[i], b0[j], b1[j], acc[i][j], idx);
            else
              acc[i][j] = smfmac16<DT, 0>(a[i], b0[j], b1[j], acc[i][j], idx);
          }
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < 8; q++) {
        const long long s = 2 * ks + q;  // 32-channel step
        uint4 a[RT], b[TT];
#pragma unroll
        for (int i = 0; i < RT; i++) a[i] = A[(rts[i] * (2 * nks) + s) * 64 + lane];
#pragma unroll
        for (int j = 0; j < TT; j++) b[j] = Xf[(tts[j] * (2 * nks) + s) * 64 + lane];
#pragma unroll
        for (int i = 0; i < RT; i++)
#pragma unroll
          for (int j = 0; j < TT; j++) acc[i][j] = mfma16<DT>(a[i], b[j], acc[i][j]);
      }
    }
  }

  const int c = lane & 15, g = lane >> 4;
#pragma unroll
  for (int i = 0; i < RT; i++) {
    const long long rt = rb * RT + i;
    if (rt >= nrt) continue;
#pragma unroll
    for (int j = 0; j < TT; j++) {
      const long long tt = tb * TT + j;
      if (tt >= ntt) continue;
      const long long t = tt * 16 + c, n = rt * 16 + g * 4;
      if (nsplit == 1)
        store_y4<DT>(Y, M, N, t, n, acc[i][j]);
      else
        *reinterpret_cast<floatx4_t*>(partial + ((long long)split * Mp + t) * Np + n) = acc[i][j];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// variant "ksplit" (decode sizes, M <= 32, HBM-bound): a workgroup of NW waves owns RT row tiles
// (16*RT output features) over the WHOLE of K; wave w takes the 64-channel steps w, w+NW, w+2NW, ...
// so the workgroup reads the compressed rows as contiguous NW KiB runs and has NW*(RT + 2*MT) KiB of
// loads in flight.  Operands go straight from memory to registers (weights from HBM, the staged
// activations from L2).  The NW partial tiles meet in LDS and are added in ascending wave order, so
// the result does not depend on timing and no global synchronisation is needed.
// grid = ceil(row tiles / RT), block = 64 * NW.
// ------------------------------------------------------------------------------------------------
// FOLD (one or two tokens, MT = 1): there is no staged copy and no staging launch; the workgroup applies the channel
// re-ordering of Section 3.3 itself: it gathers X[t, theta[p]] for all p into LDS (2 Kp bytes per token, the layout of the
// compact copy) while its first weight loads are under way, and the waves read their activation operands from there.
template <int DT, int SPARSE, int MT, int RT, int NW, int IDXM, bool FOLD = false>
__global__ void __launch_bounds__(NW * 64) k_mm_ksplit(KsplitArgs args, long long M, long long N, long long Mp, long long Np,
                                                        long long Kp, int mc) {
  static_assert(!FOLD || MT == 1, "the fold exists for the compact activation layout only");
  const uint4* __restrict__ A = args.A[blockIdx.y];
  const uint16_t* __restrict__ meta16 = args.meta16[blockIdx.y];
  const uint4* __restrict__ Xf = args.Xf[blockIdx.y];
  uint16_t* __restrict__ Y = args.Y[blockIdx.y];
  extern __shared__ floatx4_t s_red[];  // [NW][RT * MT][64]; FOLD: followed by the gathered activations [Kp / 8][mc]
  uint4* s_x = reinterpret_cast<uint4*>(s_red + NW * RT * MT * 64);
  if (FOLD) {
    const uint16_t* __restrict__ X = args.X[blockIdx.y];
    const int32_t* __restrict__ perm = args.perm[blockIdx.y];
    const long long K = args.K;
    for (long long u = threadIdx.x; u < Kp / 8; u += NW * 64) {
      const long long k0 = u * 8;
      int p[8];
      if (perm && k0 + 8 <= K) {
        const int4 p0 = *reinterpret_cast<const int4*>(perm + k0);
        const int4 p1 = *reinterpret_cast<const int4*>(perm + k0 + 4);
        p[0] = p0.x, p[1] = p0.y, p[2] = p0.z, p[3] = p0.w, p[4] = p1.x, p[5] = p1.y, p[6] = p1.z, p[7] = p1.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; e++) p[e] = k0 + e < K ? (perm ? perm[k0 + e] : (int)(k0 + e)) : -1;
      }
      for (int c = 0; c < mc; c++) {
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = (c < M && p[e] >= 0) ? X[(long long)c * K + p[e]] : (uint16_t)0;
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        s_x[u * mc + c] = o;
      }
    }
    __syncthreads();
  }
  __shared__ uint4 s_lut[SPARSE == 2 ? LUT48_CODES : 1];  // 4:8: the byte-permute selectors of every pattern code
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (SPARSE == 2) {
    fill_expand_lut<1>(s_lut, tid);
    __syncthreads();
  }
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  const long long rt0 = (long long)blockIdx.x * RT;
  long long rts[RT];
#pragma unroll
  for (int i = 0; i < RT; i++) rts[i] = (rt0 + i < nrt) ? rt0 + i : nrt - 1;

  floatx4_t acc[RT][MT];
#pragma unroll
  for (int i = 0; i < RT; i++)
#pragma unroll
    for (int j = 0; j < MT; j++) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // IDXM = how a wave takes its steps and reads their index halves: 0 = steps w, w + NW, ... with a 16-bit load each;
  // 1 = step pairs; 2 = quads (below).
  // Two steps per trip (all loads of both steps are issued before the first multiply).  Pairs (chosen by the host where
  // the step pairs divide evenly among the waves and there are two or more token tiles): a trip takes the two steps of
  // a pair, whose index halves are one 32-bit word - one load per row tile instead of two; the vector-memory path of
  // the CU, which these kernels saturate, counts instructions as well as bytes.  Otherwise wave w takes steps
  // w, w + NW, ... as they come.
  constexpr bool pairs = IDXM == 1;
  const uint32_t* meta32 = reinterpret_cast<const uint32_t*>(meta16);
  // K split over workgroups (matrices with few rows and many tokens, where every workgroup re-reading all the
  // activations costs more than the weights): workgroup z takes steps [kb, ke), an even kb
  const long long kb = gridDim.z > 1 ? (long long)blockIdx.z * args.sps : 0;
  const long long ke = gridDim.z > 1 && kb + args.sps < nks ? kb + args.sps : nks;
  if constexpr (IDXM == 2) {
    // quads (2:4 and 4:8): wave w takes the four steps 4 w .. 4 w + 3, then 4 (w + NW) .., whose index halves are one 8-byte
    // unit per lane: one index load per row tile and quad instead of four.  The vector-memory path of a CU works
    // through a load lane by lane whatever its width, so a 2-byte index load costs what a 16-byte weight load costs.
    const uint2* meta64 = reinterpret_cast<const uint2*>(meta16);
    for (long long ks = kb + 4 * wave; ks < ke; ks += 4 * NW) {
      uint32_t iw[2][RT];
#pragma unroll
      for (int i = 0; i < RT; i++) {
        const uint2 w = meta64[(rts[i] * (nks / 4) + ks / 4) * 64 + lane];
        iw[0][i] = w.x;
        iw[1][i] = w.y;
      }
      uint4 a[4][RT], b0[4][MT], b1[4][MT];
      if (MT == 1 && mc) {
        // the padding lanes hold zeros; set before the loads (and opaque to the compiler), so that the loads of the
        // live lanes land on top of them: a zero moved in after the load would have to wait for the load
#pragma unroll
        for (int u = 0; u < 4; u++) {
          b0[u][0] = uint4{0u, 0u, 0u, 0u};
          b1[u][0] = uint4{0u, 0u, 0u, 0u};
          asm volatile("" : "+v"(b0[u][0].x), "+v"(b0[u][0].y), "+v"(b0[u][0].z), "+v"(b0[u][0].w));
          asm volatile("" : "+v"(b1[u][0].x), "+v"(b1[u][0].y), "+v"(b1[u][0].z), "+v"(b1[u][0].w));
        }
      }
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const long long k = ks + u;
#pragma unroll
        for (int i = 0; i < RT; i++) a[u][i] = load_stream_16(A + (rts[i] * nks + k) * 64 + lane);
      }
      if (MT == 1 && mc) {
        const int c = lane & 15, g = lane >> 4;
        const uint4* Xc = Xf + Kp * 2;  // the compact copy behind the 16 x Kp fragment-major one
        if (c < mc) {
#pragma unroll
          for (int u = 0; u < 4; u++) {
            const long long k = ks + u;
            if (FOLD) {
              b0[u][0] = s_x[((2 * k) * 4 + g) * mc + c];
              b1[u][0] = s_x[((2 * k + 1) * 4 + g) * mc + c];
            } else {
              b0[u][0] = Xc[((2 * k) * 4 + g) * mc + c];
              b1[u][0] = Xc[((2 * k + 1) * 4 + g) * mc + c];
            }
          }
        }
      } else {
#pragma unroll
        for (int u = 0; u < 4; u++) {
          const long long k = ks + u;
#pragma unroll
          for (int j = 0; j < MT; j++) {
            const long long tt = (j < ntt) ? j : ntt - 1;
            b0[u][j] = Xf[(tt * (2 * nks) + 2 * k) * 64 + lane];
            b1[u][j] = Xf[(tt * (2 * nks) + 2 * k + 1) * 64 + lane];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; u++)
#pragma unroll
        for (int i = 0; i < RT; i++) {
          const uint32_t half = (u & 1) ? iw[u >> 1][i] >> 16 : iw[u >> 1][i];  // index half (2:4) or two pattern codes (4:8)
          if constexpr (SPARSE == 2) {
            uint4 e0, e1;
            expand_4_8<1>(a[u][i], half, s_lut, 0u, e0, e1);
#pragma unroll
            for (int j = 0; j < MT; j++) {
              acc[i][j] = mfma16<DT>(e0, b0[u][j], acc[i][j]);
              acc[i][j] = mfma16<DT>(e1, b1[u][j], acc[i][j]);
            }
          } else {
#pragma unroll
            for (int j = 0; j < MT; j++) acc[i][j] = smfmac16<DT, 0>(a[u][i], b0[u][j], b1[u][j], acc[i][j], (int)half);
          }
        }
    }
  } else
  for (long long ks = kb + (pairs ? 2 * wave : wave); ks < ke; ks += 2 * NW) {
    const bool second = pairs || ks + NW < ke;  // wave-uniform
    const long long kk[2] = {ks, pairs ? ks + 1 : (second ? ks + NW : ks)};
    uint4 a[2][RT], a2[2][RT], b0[2][MT], b1[2][MT];
    int idx[2][RT];
    if (pairs) {
#pragma unroll
      for (int i = 0; i < RT; i++) {
        const uint32_t w = meta32[((rts[i] * (nks / 4) + ks / 4) * 64 + lane) * 2 + ((ks >> 1) & 1)];
        idx[0][i] = (int)w;           // the instruction reads the low half
        idx[1][i] = (int)(w >> 16);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
#pragma unroll
      for (int i = 0; i < RT; i++) {
        if (SPARSE) {  // 2:4: kept values + index half; 4:8: kept values of two groups + their two bitmaps
          a[u][i] = load_stream_16(A + (rts[i] * nks + kk[u]) * 64 + lane);
          if (!pairs) idx[u][i] = (int)meta16[((rts[i] * (nks / 4) + kk[u] / 4) * 64 + lane) * 4 + (kk[u] & 3)];
        } else {
          a[u][i] = load_stream_16(A + (rts[i] * (2 * nks) + 2 * kk[u]) * 64 + lane);
          a2[u][i] = load_stream_16(A + (rts[i] * (2 * nks) + 2 * kk[u] + 1) * 64 + lane);
        }
      }
      if (MT == 1 && mc) {
        // compact activations (at most 16 tokens): lane (g, c) holds token c's channels 8 g .. 8 g + 7 of each half step
        const uint4 zero = {0u, 0u, 0u, 0u};
        const int c = lane & 15, g = lane >> 4;
        const bool live = c < mc;
        const uint4* Xc = Xf + Kp * 2;  // behind the 16 x Kp fragment-major copy
        if (FOLD) {
          b0[u][0] = live ? s_x[((2 * kk[u]) * 4 + g) * mc + c] : zero;
          b1[u][0] = live ? s_x[((2 * kk[u] + 1) * 4 + g) * mc + c] : zero;
        } else {
          b0[u][0] = live ? Xc[((2 * kk[u]) * 4 + g) * mc + c] : zero;
          b1[u][0] = live ? Xc[((2 * kk[u] + 1) * 4 + g) * mc + c] : zero;
        }
      } else {
#pragma unroll
        for (int j = 0; j < MT; j++) {
          const long long tt = (j < ntt) ? j : ntt - 1;
          b0[u][j] = Xf[(tt * (2 * nks) + 2 * kk[u]) * 64 + lane];
          b1[u][j] = Xf[(tt * (2 * nks) + 2 * kk[u] + 1) * 64 + lane];
        }
      }
    }
    if (SPARSE == 2) {
#pragma unroll
      for (int u = 0; u < 2; u++)
#pragma unroll
        for (int i = 0; i < RT; i++) {
          const uint4 v = a[u][i];
          expand_4_8<1>(v, (uint32_t)idx[u][i], s_lut, 0u, a[u][i], a2[u][i]);
        }
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
      if (u == 1 && !second) break;
#pragma unroll
      for (int i = 0; i < RT; i++)
#pragma unroll
        for (int j = 0; j < MT; j++) {
          if (SPARSE == 1) {
            acc[i][j] = smfmac16<DT, 0>(a[u][i], b0[u][j], b1[u][j], acc[i][j], idx[u][i]);
          } else {
            acc[i][j] = mfma16<DT>(a[u][i], b0[u][j], acc[i][j]);
            acc[i][j] = mfma16<DT>(a2[u][i], b1[u][j], acc[i][j]);
          }
        }
    }
  }

#pragma unroll
  for (int i = 0; i < RT; i++)
#pragma unroll
    for (int j = 0; j < MT; j++) s_red[(wave * (RT * MT) + i * MT + j) * 64 + lane] = acc[i][j];
  __syncthreads();
  const int c = lane & 15, g = lane >> 4;
  for (int q = wave; q < RT * MT; q += NW) {
    const int i = q / MT, j = q % MT;
    floatx4_t sum = s_red[q * 64 + lane];
    for (int w = 1; w < NW; w++) sum += s_red[(w * (RT * MT) + q) * 64 + lane];
    if (rt0 + i < nrt && j < ntt) {
      if (gridDim.z > 1)
        *reinterpret_cast<floatx4_t*>(args.partial + (((long long)blockIdx.z * Mp + (long long)j * 16 + c) * Np + (rt0 + i) * 16 + g * 4)) = sum;
      else
        store_y4<DT>(Y, M, N, (long long)j * 16 + c, (rt0 + i) * 16 + g * 4, sum);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// variant "tile" (prefill sizes, MFMA-bound): a workgroup of 4 waves (2 x 2) owns a macro tile of
// RTM row tiles x 2*TC token tiles (of 16); each wave owns TR x TC tiles (sparse: TR = TC = 8, i.e.
// 128 x 128 outputs and 256 accumulator registers, one wave per SIMD; RTM = 2 TR).
// The K loop runs in 64-channel stages, software pipelined TWO stages ahead:
//   - the macro tile's slice of the staged activations (4*TC KiB per stage), of the weights (16 KiB
//     per stage) and of the index words (4 KiB per stage pair) are copied by DMA from global memory
//     straight into LDS (three buffers each, no registers involved);
//   - a stage ends with a counted wait (all vector-memory operations but the newest stage's DMA have
//     finished, so the next stage's buffers are full) and a barrier.
// The LDS buffers are separate __shared__ arrays handed to the pipeline as __restrict__ pointers:
// that is what lets the compiler see that reading buffer k does not have to wait for the DMA into
// buffer k+2.  Each wave reads its TR A operands once per stage and each B operand once for TR
// multiplies.  Macro tiles are numbered so that the workgroups of one XCD (blockIdx % 8) cover
// neighbouring tiles and share weight rows in that XCD's L2.
// ------------------------------------------------------------------------------------------------
// Order of the macro tiles: bands of `band` row blocks; within a band the token blocks are outermost.  The workgroups an
// XCD runs at the same time take consecutive tiles, i.e. a patch of band row blocks x (32 / band) token blocks, and
// share those operand panels in that XCD's L2 (band = 1: the token blocks of one row block after another).
__device__ __forceinline__ void tile_coords(long long tile, long long n_tiles, long long ntb, int band, long long& rb, long long& tb) {
  const long long nrb = n_tiles / ntb;
  const long long b = tile / (band * ntb), base = b * band;
  const long long gh = nrb - base < band ? nrb - base : band;
  const long long t = tile - b * band * ntb;
  rb = base + t % gh;
  tb = t / gh;
}

template <int SPARSE, int TR, int TC, int NWC>
struct TileState {
  static constexpr int NW = 2 * NWC;                        // waves: 2 along the rows x NWC along the tokens
  static constexpr int NT = 64 * NW;                        // threads
  static constexpr bool HALF = SPARSE == 3;                 // dense, 32-channel stages (one half step per stage)
  static constexpr bool META = SPARSE == 1 || SPARSE == 2;  // index words (2:4) or bitmaps (4:8) travel beside the weights
  static constexpr int BSTEP = HALF ? 64 : 128;             // 16-byte units of activations per token tile and stage
  static constexpr int BCOPIES = (NWC * TC * BSTEP) / NT;   // ... per lane and stage
  static constexpr int RTM = 2 * TR;                        // row tiles of 16 in the macro tile
  static constexpr int AUNITS = RTM * (SPARSE ? 64 : 128);  // 16-byte units of weights per stage
  static constexpr int ACOPIES = (AUNITS + NT - 1) / NT;    // ... per lane; when the chunks do not divide among the waves the
  static constexpr int ASLOTS = ACOPIES * NT;               //     last copies fetch a row tile past the macro tile into spare slots
  static_assert((NWC * TC * BSTEP) % NT == 0, "every wave copies whole 64-unit chunks");
  floatx4_t acc[TR][TC];
  const uint4* a_src[ACOPIES];  // wave-uniform global bases of this wave's DMA copies
  const uint4* x_src[BCOPIES];
  const uint32_t* m_src[ACOPIES];  // index words (two stages of index halves per lane) of the copied row tiles
  unsigned lane, x_lane, wave, wr, wc;
  unsigned k0, k1;  // this workgroup's stages [k0, k1) of the K loop (all of them unless K is split)
  const uint4* lut;  // 4:8: the byte-permute selectors of every pattern code, 16 copies (LDS)
};

// every vector-memory operation of the pipeline is a DMA into LDS: they keep their program order,
// which the stage-end wait counts on
template <int SPARSE, int TR, int TC, int NWC>
__device__ __forceinline__ void tile_prefetch_b(TileState<SPARSE, TR, TC, NWC>& st, uint4* sb, unsigned kn) {
  using State = TileState<SPARSE, TR, TC, NWC>;
#pragma unroll
  for (int p = 0; p < State::BCOPIES; p++) {
    if (State::HALF)  // chunk q = NW p + w: half step kn of token tile q
      global_to_lds_16(st.x_src[p] + (kn * 64u + st.lane), sb + State::NT * p + st.wave * 64);
    else
      global_to_lds_16(st.x_src[p] + (kn * 128u + st.x_lane), sb + State::NT * p + st.wave * 64);
  }
}

template <int SPARSE, int TR, int TC, int NWC>
__device__ __forceinline__ void tile_prefetch_a(TileState<SPARSE, TR, TC, NWC>& st, uint4* sa, uint32_t* sm, unsigned kn) {
  using State = TileState<SPARSE, TR, TC, NWC>;
#pragma unroll
  for (int p = 0; p < State::ACOPIES; p++) {
    // chunk q = NW p + w of 64 units.  sparse and dense half-step stages: row tile q; dense: row tile q / 2, half q % 2
    // (NW is even: half w % 2)
    const unsigned off = SPARSE ? kn * 64u + st.lane : kn * 128u + (st.wave & 1u) * 64u + st.lane;
    global_to_lds_16(st.a_src[p] + off, sa + State::NT * p + st.wave * 64);
    // the lane's index word holding stage kn: 8 bytes per lane and group of 4 stages, word (kn % 4) / 2
    if (State::META)
      global_to_lds_4(st.m_src[p] + ((kn >> 2) * 128u + st.lane * 2u + ((kn >> 1) & 1u)), sm + State::NT * p + st.wave * 64);
  }
}

// the A side of one stage in registers: the wave's TR weight operands and their raw index words; 4:8: the dense operands
// of the stage's two half steps, expanded from the kept values and the bitmaps as they are read
template <int SPARSE, int TR>
struct TileRegs {
  uint4 a[(SPARSE == 1 || SPARSE == 3) ? TR : 2 * TR];
  uint32_t m[SPARSE == 1 ? TR : 1];
};

template <int SPARSE, int TR, int TC, int NWC>
__device__ __forceinline__ void tile_load_a(TileState<SPARSE, TR, TC, NWC>& st, const uint4* sa, const uint32_t* sm,
                                            TileRegs<SPARSE, TR>& r, unsigned k) {
  if constexpr (SPARSE == 2) {
    // all pattern codes first, then the kept values, then the selectors: the selector reads depend on the codes, and
    // with the reads issued in this order (spread one by one among the multiplies) a code is back long before its
    // selector read comes up.  The word holds the codes of an even and an odd stage; k = the stage of these operands.
    uint32_t codes[TR];
    uint4 raw[TR];
#pragma unroll
    for (int i = 0; i < TR; i++) codes[i] = sm[(st.wr * TR + i) * 64 + st.lane] >> ((k & 1u) * 16u);
#pragma unroll
    for (int i = 0; i < TR; i++) raw[i] = sa[(st.wr * TR + i) * 64 + st.lane];
#pragma unroll
    for (int i = 0; i < TR; i++) expand_4_8<16>(raw[i], codes[i], st.lut, st.lane & 15u, r.a[2 * i], r.a[2 * i + 1]);
  } else {
#pragma unroll
    for (int i = 0; i < TR; i++) {
      if constexpr (SPARSE != 0) {
        r.a[i] = sa[(st.wr * TR + i) * 64 + st.lane];
        if constexpr (SPARSE == 1) r.m[i] = sm[(st.wr * TR + i) * 64 + st.lane];
      } else {
        r.a[2 * i] = sa[(st.wr * TR + i) * 128 + st.lane];
        r.a[2 * i + 1] = sa[(st.wr * TR + i) * 128 + 64 + st.lane];
      }
    }
  }
}

// the B operand (two 16-byte halves of a 64-channel step) of one token tile
struct TileB {
  uint4 b0, b1;
};

// multiplies of token tiles J0 .. J1 - 1 of stage k.  The B operands stream from LDS D token tiles ahead through a ring
// of D register sets: on entry bq[(j + OFF) % D] holds the operand of tile j for j = J0 .. J0 + D - 1; while tile j is
// multiplied the operand of tile j + D is read into the set it frees (from `sb` for tiles of this stage; past the stage's
// last tile - if NEXT - tile j + D - TC of `sb_next`, the next stage's buffer).  The next stage therefore finds its tile t
// in set (t + OFF + TC) % D: its OFF is (OFF + TC) % D.
template <int DT, int SPARSE, int TR, int TC, int NWC, int J0, int J1, bool NEXT, int D, int OFF>
__device__ __forceinline__ void tile_multiply(TileState<SPARSE, TR, TC, NWC>& st, const TileRegs<SPARSE, TR>& r, TileB (&bq)[D],
                                              const uint4* sb, const uint4* sb_next, unsigned k) {
  using State = TileState<SPARSE, TR, TC, NWC>;
  constexpr int BS = State::BSTEP;
  int idx[TR];
  if constexpr (SPARSE == 1) {
    const unsigned sh = (k & 1u) * 16u;  // the word holds the index halves of an even and an odd stage
#pragma unroll
    for (int i = 0; i < TR; i++) idx[i] = (int)(r.m[i] >> sh);
  }
  const uint4* b = sb + (st.wc * TC) * BS + st.lane;
  const uint4* bn = sb_next + (st.wc * TC) * BS + st.lane;
#pragma unroll
  for (int j = J0; j < J1; j++) {
    const TileB cur = bq[(j + OFF) % D];
    TileB nx = cur;
    if (j + D < TC) {
      nx.b0 = b[(j + D) * BS];
      if (!State::HALF) nx.b1 = b[(j + D) * BS + 64];
    } else if (NEXT) {
      nx.b0 = bn[(j + D - TC) * BS];
      if (!State::HALF) nx.b1 = bn[(j + D - TC) * BS + 64];
    }
#pragma unroll
    for (int i = 0; i < TR; i++) {
      if constexpr (SPARSE == 1) {
        st.acc[i][j] = smfmac16<DT, 0>(r.a[i], cur.b0, cur.b1, st.acc[i][j], idx[i]);
      } else if constexpr (State::HALF) {
        st.acc[i][j] = mfma16<DT>(r.a[i], cur.b0, st.acc[i][j]);
      } else {  // dense, or 4:8 expanded to dense operands
        st.acc[i][j] = mfma16<DT>(r.a[2 * i], cur.b0, st.acc[i][j]);
        st.acc[i][j] = mfma16<DT>(r.a[2 * i + 1], cur.b1, st.acc[i][j]);
      }
    }
    bq[(j + OFF) % D] = nx;
  }
}

// End of a stage: wait until at most the DMA operations of the newest prefetch are outstanding (they
// are the last vector-memory operations issued, and DMA keeps its program order), so every older DMA
// - in particular the ones that filled the next stage's buffers - has landed, and until this wave's
// LDS reads have returned (the buffer they read is overwritten by the next stage's DMA); then meet
// the other waves.
template <int DMA_PER_STAGE>
__device__ __forceinline__ void tile_arrive() {
#if defined(__HIP_DEVICE_COMPILE__)
  // s_waitcnt: vmcnt = DMA_PER_STAGE (6 bits, split 3:0 / 15:14), lgkmcnt = 0, expcnt left at "do not wait"
  __builtin_amdgcn_s_waitcnt((DMA_PER_STAGE & 15) | ((DMA_PER_STAGE >> 4) << 14) | 0x0070);
  __builtin_amdgcn_s_barrier();
#endif
}

// One pipeline stage k.  On entry the wave holds the A side of stage k in `cur` and the B operand of its first
// token tile in `bq`; the LDS buffers hold B(k) (b_cur), A(k+1) (a_nxt / m_nxt) and, landed or landing, B(k+1)
// (b_nxt) and A(k+2).  The stage
//   - issues the DMA of B(k+2) into the buffer B(k-1) was in and of A(k+3) into the buffer A(k) was in,
//   - copies A(k+1) from LDS to `nxt` (off the critical path: those registers are used one stage on),
//   - multiplies all token tiles but the last, B operands streaming from LDS one token tile ahead,
//   - waits for the DMA issued in stage k-1 (B(k+1), A(k+2)) and meets the other waves,
//   - reads the first B operand of stage k+1 and, while that read is under way, multiplies the last token tile:
//     the matrix pipe has work across the barrier and the LDS latency behind it.
// With fewer than four token tiles per wave holding one back leaves too little ahead of the barrier to spread the
// DMA over (measured slower): all tiles are multiplied first and the next stage's operand is read after the barrier.
// D = how many token tiles ahead the B operands are read (1 with two waves per SIMD, where the other wave covers the LDS
// latency; more with one wave per SIMD); the last D token tiles of a stage are multiplied after the barrier.
template <int DT, int SPARSE, int TR, int TC, int NWC, int D, int OFF>
__device__ __forceinline__ void tile_stage(TileState<SPARSE, TR, TC, NWC>& st, const TileRegs<SPARSE, TR>& cur,
                                           TileRegs<SPARSE, TR>& nxt, TileB (&bq)[D], const uint4* b_cur, const uint4* b_nxt,
                                           const uint4* a_nxt, const uint32_t* m_nxt, uint4* b_pre, uint4* a_pre, uint32_t* m_pre,
                                           unsigned k) {
  using State = TileState<SPARSE, TR, TC, NWC>;
  constexpr int DMA = State::BCOPIES + (State::META ? 2 : 1) * State::ACOPIES;
  constexpr int BR = State::HALF ? 1 : 2;                    // LDS reads per B operand
  constexpr bool STRADDLE = TC >= 4;
  static_assert(D == 1 || (STRADDLE && D < TC), "deeper operand streams exist for the straddling schedule only");
  constexpr int TH = STRADDLE ? TC - D : TC;                 // token tiles multiplied ahead of the barrier
  constexpr int DPJ = (DMA + TH - 1) / TH;                   // DMA operations issued per token tile
  constexpr int AREADS = State::HALF ? TR : (SPARSE == 2 ? 4 : 2) * TR;  // LDS reads of tile_load_a (4:8: + two selector reads)
  constexpr int APJ = (AREADS + TH - 1) / TH;
  constexpr int MM = (SPARSE == 1 || SPARSE == 3) ? TR : 2 * TR;  // matrix instructions per token tile
  const unsigned last = st.k1 - 1;                           // past the end: reload the last stage (never used)
  tile_prefetch_b<SPARSE, TR, TC, NWC>(st, b_pre, k + 2 < st.k1 ? k + 2 : last);
  tile_prefetch_a<SPARSE, TR, TC, NWC>(st, a_pre, m_pre, k + 3 < st.k1 ? k + 3 : last);
  tile_multiply<DT, SPARSE, TR, TC, NWC, 0, TH, false, D, OFF>(st, cur, bq, b_cur, b_nxt, k);
  tile_load_a<SPARSE, TR, TC, NWC>(st, a_nxt, m_nxt, nxt, k + 1);
  // the order wanted ahead of the barrier: per token tile "read a coming B operand; then multiplies, each followed by
  // one copy of the DMA's share and a share of the reads of the next stage's A side" (sched_spread).
#pragma unroll
  for (int j = 0; j < TH; j++) {
    if (j + D < TC) sched_group<0x100, BR>();
    sched_spread<MM, DPJ, APJ>();
  }
  sched_fence();
  tile_arrive<DMA>();
  sched_fence();
  if (STRADDLE) {
    tile_multiply<DT, SPARSE, TR, TC, NWC, TH, TC, true, D, OFF>(st, cur, bq, b_cur, b_nxt, k);
#pragma unroll
    for (int j = TH; j < TC; j++) {
      sched_group<0x100, BR>();
      sched_group<0x008, MM>();
    }
    sched_fence();
  } else {
    const uint4* bn = b_nxt + (st.wc * TC) * State::BSTEP + st.lane;  // D == 1 here
    bq[0].b0 = bn[0];
    if (!State::HALF) bq[0].b1 = bn[64];
  }
}

template <int DT, int SPARSE, int TR, int TC, int NWC, int D>
__device__ __attribute__((always_inline)) void tile_pipeline(
    uint4* __restrict__ sa0, uint4* __restrict__ sa1, uint4* __restrict__ sa2, uint4* __restrict__ sb0, uint4* __restrict__ sb1,
    uint4* __restrict__ sb2, uint32_t* __restrict__ sm0, uint32_t* __restrict__ sm1, uint32_t* __restrict__ sm2,
    const uint4* __restrict__ A, const uint16_t* __restrict__ meta16, const uint4* __restrict__ Xf,
    uint16_t* __restrict__ Y, float* __restrict__ partial, long long M, long long N, long long Mp, long long Np, long long Kp,
    long long n_tiles, long long ntb, int nsplit, int sps, int band, const uint4* lut = nullptr) {
  constexpr int NTT = NWC * TC;               // token tiles of 16 in the macro tile
  constexpr int RTM = 2 * TR;                 // row tiles of 16 in the macro tile
  using State = TileState<SPARSE, TR, TC, NWC>;
  const int tid = threadIdx.x;
  State st;
  st.lane = (unsigned)(tid & 63);
  st.wave = (unsigned)wave_uniform(tid >> 6);  // wave-uniform: keeps the operand bases in SGPRs
  st.wr = st.wave / NWC;
  st.wc = st.wave % NWC;
  st.lut = lut;
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  const long long nst = State::HALF ? 2 * nks : nks;  // stages of the K loop
  // XCD-aware numbering: XCD x (= blockIdx % 8) works through items [x * per, (x + 1) * per); an item is
  // a macro tile and one of the nsplit ranges of K stages (the split varies fastest)
  const long long n_items = n_tiles * nsplit;
  const long long per = (n_items + 7) / 8;
  const long long item = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((long long)(blockIdx.x >> 3) >= per || item >= n_items) return;
  const long long tile = item / nsplit;
  const int split = (int)(item % nsplit);
  st.k0 = (unsigned)((long long)split * sps);
  st.k1 = (unsigned)(((long long)(split + 1) * sps < nst) ? (long long)(split + 1) * sps : nst);
  long long rb, tb;
  tile_coords(tile, n_tiles, ntb, band, rb, tb);
  const long long rt_macro = rb * RTM;  // first row tile of the macro tile
  const long long tt_base = tb * NTT;   // first token tile of the macro tile
#pragma unroll
  for (int p = 0; p < State::ACOPIES; p++) {
    const long long rtl = SPARSE ? State::NW * p + st.wave : (State::NW / 2) * p + (st.wave >> 1);  // row tile this wave copies
    const long long rt = (rt_macro + rtl < nrt) ? rt_macro + rtl : nrt - 1;
    st.a_src[p] = A + (State::META ? rt * nks : rt * (2 * nks)) * 64;
    st.m_src[p] = reinterpret_cast<const uint32_t*>(meta16) + rt * (nks / 4) * 128;
  }
#pragma unroll
  for (int p = 0; p < State::BCOPIES; p++) {
    // token tile (within the macro tile) of this wave's p-th copy
    const long long ttl = State::HALF ? State::NW * p + st.wave : (State::NW / 2) * p + (st.wave >> 1);
    const long long tt = (tt_base + ttl < ntt) ? tt_base + ttl : ntt - 1;
    st.x_src[p] = Xf + tt * (2 * nks) * 64;
  }
  st.x_lane = (unsigned)(tid & 127);  // chunk q = NW p + w is half q % 2 = w % 2 of its token tile
#pragma unroll
  for (int i = 0; i < TR; i++)
#pragma unroll
    for (int j = 0; j < TC; j++) st.acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // prologue: B and A of the first two stages and A of the third in flight; wait for all of them; the first A side to registers
  const unsigned last = st.k1 - 1;
  const unsigned kb = st.k0;
  tile_prefetch_b<SPARSE, TR, TC, NWC>(st, sb0, kb);
  tile_prefetch_a<SPARSE, TR, TC, NWC>(st, sa0, sm0, kb);
  tile_prefetch_b<SPARSE, TR, TC, NWC>(st, sb1, kb + 1 < st.k1 ? kb + 1 : last);
  tile_prefetch_a<SPARSE, TR, TC, NWC>(st, sa1, sm1, kb + 1 < st.k1 ? kb + 1 : last);
  tile_prefetch_a<SPARSE, TR, TC, NWC>(st, sa2, sm2, kb + 2 < st.k1 ? kb + 2 : last);
  sched_fence();
  tile_arrive<0>();
  TileRegs<SPARSE, TR> r0, r1;
  tile_load_a<SPARSE, TR, TC, NWC>(st, sa0, sm0, r0, kb);
  sched_fence();
  tile_arrive<0>();  // every wave has its first A side in registers before the first stage overwrites its buffer
  TileB bq[D];       // the B operands of the coming stage's first D token tiles
#pragma unroll
  for (int d = 0; d < D; d++) {
    bq[d].b0 = sb0[(st.wc * TC + d) * State::BSTEP + st.lane];
    if (!State::HALF) bq[d].b1 = sb0[(st.wc * TC + d) * State::BSTEP + 64 + st.lane];
  }
  // the register set a stage finds its first operand in moves by TC % D from stage to stage and is back after three
  constexpr int O1 = TC % D, O2 = (2 * TC) % D;
  static_assert((3 * TC) % D == 0, "the operand ring must be back in place after the three unrolled stages");
  unsigned k = kb;
  for (; k + 3 <= st.k1; k += 3) {
    tile_stage<DT, SPARSE, TR, TC, NWC, D, 0>(st, r0, r1, bq, sb0, sb1, sa1, sm1, sb2, sa0, sm0, k);
    tile_stage<DT, SPARSE, TR, TC, NWC, D, O1>(st, r1, r0, bq, sb1, sb2, sa2, sm2, sb0, sa1, sm1, k + 1);
    tile_stage<DT, SPARSE, TR, TC, NWC, D, O2>(st, r0, r1, bq, sb2, sb0, sa0, sm0, sb1, sa2, sm2, k + 2);
    r0 = r1;
  }
  if (k < st.k1) tile_stage<DT, SPARSE, TR, TC, NWC, D, 0>(st, r0, r1, bq, sb0, sb1, sa1, sm1, sb2, sa0, sm0, k);
  if (k + 1 < st.k1) tile_stage<DT, SPARSE, TR, TC, NWC, D, O1>(st, r1, r0, bq, sb1, sb2, sa2, sm2, sb0, sa1, sm1, k + 1);
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no DMA into this workgroup's LDS is left in flight when the wave ends
#endif

  const int c = (int)(st.lane & 15), g = (int)(st.lane >> 4);
  if (nsplit == 1 && (N & 7) == 0) {
    // Outputs through LDS: a wave transposes its TR x TC tiles, CH tokens at a time, in a private slice of the (now idle)
    // operand rings and stores runs of 32 TR bytes (the wave's 16 TR output features of one token) in 16-byte pieces;
    // stored straight from the accumulators a lane would write 8 bytes of 16 different rows of Y per instruction.
    constexpr int CHT = TC >= 2 ? 2 : 1;                   // token tiles per pass
    constexpr unsigned ROWB = TR * 32 + 16;                // bytes per token in the slice (padded: the 16 tokens of a
    constexpr unsigned SLICE = CHT * 16 * ROWB;            //   tile start in different banks)
    constexpr unsigned ABYTES = State::ASLOTS * 16, BBYTES = NTT * State::BSTEP * 16;
    constexpr int FA = ABYTES / SLICE, FB = BBYTES / SLICE;  // slices per weight / activation buffer
    constexpr int SLOTS = 3 * (FA + FB) < State::NW ? 3 * (FA + FB) : State::NW;
    static_assert(SLOTS >= 1, "no operand buffer holds an output slice");
    constexpr int PHASES = (State::NW + SLOTS - 1) / SLOTS;  // waves take turns where the rings hold fewer slices than waves
    constexpr int FAd = FA ? FA : 1, FBd = FB ? FB : 1;
    const int slot = (int)st.wave % SLOTS, phase = (int)st.wave / SLOTS;
    unsigned char* ep;
    if (slot < 3 * FB) {
      uint4* base = slot / FBd == 0 ? sb0 : (slot / FBd == 1 ? sb1 : sb2);
      ep = reinterpret_cast<unsigned char*>(base) + (slot % FBd) * SLICE;
    } else {
      const int s2 = slot - 3 * FB;
      uint4* base = s2 / FAd == 0 ? sa0 : (s2 / FAd == 1 ? sa1 : sa2);
      ep = reinterpret_cast<unsigned char*>(base) + (s2 % FAd) * SLICE;
    }
    const long long t_wave = (tt_base + st.wc * TC) * 16, n_wave = (rt_macro + st.wr * TR) * 16;
    __syncthreads();  // every wave is done with the rings
#pragma unroll
    for (int ph = 0; ph < PHASES; ph++)
#pragma unroll
      for (int j0 = 0; j0 < TC; j0 += CHT) {
        const bool mine = PHASES == 1 || phase == ph;  // wave-uniform
        if (mine) {
#pragma unroll
          for (int jj = 0; jj < CHT; jj++)
#pragma unroll
            for (int i = 0; i < TR; i++) {
              const floatx4_t a = st.acc[i][j0 + jj];
              uint2 v;
              v.x = esp_from_float<DT>(a[0]) | ((uint32_t)esp_from_float<DT>(a[1]) << 16);
              v.y = esp_from_float<DT>(a[2]) | ((uint32_t)esp_from_float<DT>(a[3]) << 16);
              *reinterpret_cast<uint2*>(ep + (16 * jj + c) * ROWB + (16 * i + 4 * g) * 2) = v;
            }
        }
        __syncthreads();
        if (mine) {
          constexpr int PIECES = CHT * 16 * TR * 2;  // 16-byte pieces of the pass
#pragma unroll
          for (int p = 0; p < (PIECES + 63) / 64; p++) {
            const int pi = p * 64 + (int)st.lane;
            const int tl = pi / (2 * TR), piece = pi % (2 * TR);
            if (pi < PIECES) {
              const uint4 v = *reinterpret_cast<const uint4*>(ep + tl * ROWB + piece * 16);
              const long long t = t_wave + 16 * j0 + tl, n = n_wave + piece * 8;
              if (t < M && n + 8 <= N) *reinterpret_cast<uint4*>(Y + t * N + n) = v;
            }
          }
        }
        __syncthreads();
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < TR; i++) {
    const long long rt = rt_macro + st.wr * TR + i;
    if (rt >= nrt) continue;
#pragma unroll
    for (int j = 0; j < TC; j++) {
      const long long tt = tt_base + st.wc * TC + j;
      if (tt >= ntt) continue;
      if (nsplit > 1)  // fp32 partial tile of this K split; k_reduce_splits adds the splits in ascending order
        *reinterpret_cast<floatx4_t*>(partial + ((long long)split * Mp + tt * 16 + c) * Np + rt * 16 + g * 4) = st.acc[i][j];
      else
        store_y4<DT>(Y, M, N, tt * 16 + c, rt * 16 + g * 4, st.acc[i][j]);
    }
  }
}

// sparse: TR = 8 (macro tile of 16 row tiles) or 4; dense: half of that (operands twice as wide), or (SPARSE = 3) the
// sparse shape with stages of 32 channels: 256 x 256 outputs per workgroup for 32 KiB of operands per stage - half the
// operand bytes per multiply of the 128-row dense form, which is what the matrix pipe waits for.
template <int DT, int SPARSE, int TR, int TC, int NWC, int D = 1>
__global__ void __launch_bounds__(128 * NWC) k_mm_tile(const uint4* __restrict__ A, const uint16_t* __restrict__ meta16,
                                                        const uint4* __restrict__ Xf, uint16_t* __restrict__ Y,
                                                        float* __restrict__ partial, long long M, long long N, long long Mp,
                                                        long long Np, long long Kp, long long n_tiles, long long ntb, int nsplit,
                                                        int sps, int band) {
  constexpr int ASLOTS = TileState<SPARSE, TR, TC, NWC>::ASLOTS;
  __shared__ uint4 s_a0[ASLOTS];  // one stage of weights each
  __shared__ uint4 s_a1[ASLOTS];
  __shared__ uint4 s_a2[ASLOTS];
  constexpr int BSTEP = TileState<SPARSE, TR, TC, NWC>::BSTEP;
  __shared__ uint4 s_b0[NWC * TC * BSTEP];  // one stage of activations each: [NWC TC token tiles][2 half steps (or 1)][64 lanes]
  __shared__ uint4 s_b1[NWC * TC * BSTEP];
  __shared__ uint4 s_b2[NWC * TC * BSTEP];
  constexpr bool META = TileState<SPARSE, TR, TC, NWC>::META;
  __shared__ uint32_t s_m0[META ? ASLOTS : 1];  // one stage pair of index words (4:8: bitmaps) each: [row tiles][64 lanes]
  __shared__ uint32_t s_m1[META ? ASLOTS : 1];
  __shared__ uint32_t s_m2[META ? ASLOTS : 1];
  __shared__ uint4 s_lut[SPARSE == 2 ? LUT48_CODES * 16 : 1];
  if (SPARSE == 2) {
    fill_expand_lut<16>(s_lut, (int)threadIdx.x);
    __syncthreads();
  }
  tile_pipeline<DT, SPARSE, TR, TC, NWC, D>(s_a0, s_a1, s_a2, s_b0, s_b1, s_b2, s_m0, s_m1, s_m2, A, meta16, Xf, Y, partial, M, N, Mp,
                                         Np, Kp, n_tiles, ntb, nsplit, sps, band, s_lut);
}

// ------------------------------------------------------------------------------------------------
// variant "tile32" (2:4 only): the same workgroup, LDS ring and DMA schedule as the 8-wave 256 x 256 tile
// kernel above, but a wave's 128 rows x 64 tokens are 4 x 2 tiles of v_smfmac_f32_32x32x32 (half as many
// matrix instructions for the same operand bytes; the instruction also peaks 10 % higher), and the outputs
// leave through LDS: a wave transposes its tile 32 tokens at a time in a private LDS slice and stores 256-byte
// runs of Y (128 output features of one token) instead of 32-byte pieces.
// Operand layouts of v_smfmac_f32_32x32x32_{f16,bf16} (lane l, r = l % 32, h = l / 32), measured with one-hot
// operands:  A: row r, the 8 kept values of channels [16 h, 16 h + 16) of the 32-channel step, value e at channel
//            16 h + 4 (e / 2) + idx_e (idx_e = bits [2e+1 : 2e] of the low half of the lane's index register)
//            B: column r, e < 8: k = 8 h + e;  e >= 8: k = 16 + 8 h + (e - 8)
//            D: column r, register j holds row 8 (j / 4) + 4 h + j % 4
// Both operands are read out of the LDS images the DMA leaves (the 16-byte units of the native weight layout and
// of the fragment-major activations) by lane addressing alone: the A operand of the step's half q for rows
// 32 i .. 32 i + 31 is unit 16 (2 q + h) + r % 16 of row tile 2 i + r / 16; the B operand for tokens 32 j .. + 31 is
// units 16 h + r % 16 and 16 (2 + h) + r % 16 of half step q of token tile 2 j + r / 16.
// ------------------------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ floatx16_t smfmac32(uint4 a, uint4 b0, uint4 b1, floatx16_t c, int idx) {
  struct B2 {
    uint4 lo, hi;
  } bb = {b0, b1};
  if (DT == ESPARSE_F16) {
    return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half16_t, bb), c, idx, 0, 0);
  } else {
    return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x16_t, bb), c, idx, 0, 0);
  }
}

struct Tile32Regs {
  uint4 a[2][4];     // [half of the 64-channel stage][32-row tile]
  uint32_t m[2][4];  // raw index words (an even and an odd stage each)
};
struct Tile32Lane {
  unsigned a_base;  // unit (and index-word) number of this lane's A operand for half 0, row tile 0
  unsigned b_base;  // unit number of this lane's first B half for half 0, token tile 0
};

__device__ __forceinline__ void tile32_load_a(const Tile32Lane& ln, const uint4* sa, const uint32_t* sm, Tile32Regs& r) {
#pragma unroll
  for (int q = 0; q < 2; q++)
#pragma unroll
    for (int i = 0; i < 4; i++) {
      r.a[q][i] = sa[ln.a_base + i * 128 + q * 32];
      r.m[q][i] = sm[ln.a_base + i * 128 + q * 32];
    }
}

// multiplies of iterations IT0 .. IT1 - 1 of stage k; a wave owns TJ 32-token tiles and iteration it = (half q = it / TJ,
// tile j = it % TJ).  On entry `bq` holds the B operand of iteration IT0; the next iteration's operand is read while one
// is multiplied (after the stage's last iteration: the first operand of the next stage's buffer, if NEXT)
template <int DT, int TJ, int IT0, int IT1, bool NEXT>
__device__ __forceinline__ void tile32_multiply(const Tile32Lane& ln, const Tile32Regs& r, TileB& bq, const uint4* sb,
                                                const uint4* sb_next, unsigned k, floatx16_t (&acc)[4][TJ]) {
  const unsigned sh = (k & 1u) * 16u;
#pragma unroll
  for (int it = IT0; it < IT1; it++) {
    const int q = it / TJ, j = it % TJ;
    TileB nx = bq;
    if (it + 1 < 2 * TJ) {
      const int q2 = (it + 1) / TJ, j2 = (it + 1) % TJ;
      nx.b0 = sb[ln.b_base + j2 * 256 + q2 * 64];
      nx.b1 = sb[ln.b_base + j2 * 256 + q2 * 64 + 32];
    } else if (NEXT) {
      nx.b0 = sb_next[ln.b_base];
      nx.b1 = sb_next[ln.b_base + 32];
    }
#pragma unroll
    for (int i = 0; i < 4; i++) acc[i][j] = smfmac32<DT>(r.a[q][i], bq.b0, bq.b1, acc[i][j], (int)(r.m[q][i] >> sh));
    bq = nx;
  }
}

// one pipeline stage: the schedule of tile_stage (DMA of B(k+2) and A(k+3) issued, A(k+1) copied to registers, all
// iterations but the last ahead of the barrier, the last across it)
template <int DT, int TJ>
__device__ __forceinline__ void tile32_stage(TileState<1, 8, 2 * TJ, 4>& st, const Tile32Lane& ln, const Tile32Regs& cur,
                                             Tile32Regs& nxt, TileB& bq, const uint4* b_cur, const uint4* b_nxt, const uint4* a_nxt,
                                             const uint32_t* m_nxt, uint4* b_pre, uint4* a_pre, uint32_t* m_pre, unsigned k,
                                             floatx16_t (&acc)[4][TJ]) {
  using State = TileState<1, 8, 2 * TJ, 4>;
  constexpr int DMA = State::BCOPIES + 2 * State::ACOPIES;
  constexpr int ITERS = 2 * TJ, TH = ITERS - 1;
  constexpr int DPJ = (DMA + TH - 1) / TH;
  constexpr int APJ = (16 + TH - 1) / TH;
  const unsigned last = st.k1 - 1;
  tile_prefetch_b<1, 8, 2 * TJ, 4>(st, b_pre, k + 2 < st.k1 ? k + 2 : last);
  tile_prefetch_a<1, 8, 2 * TJ, 4>(st, a_pre, m_pre, k + 3 < st.k1 ? k + 3 : last);
  tile32_multiply<DT, TJ, 0, TH, false>(ln, cur, bq, b_cur, b_nxt, k, acc);
  tile32_load_a(ln, a_nxt, m_nxt, nxt);
#pragma unroll
  for (int j = 0; j < TH; j++) {
    sched_group<0x100, 2>();
    sched_spread<4, DPJ, APJ, true>();
  }
  sched_fence();
  tile_arrive<DMA>();
  sched_fence();
  tile32_multiply<DT, TJ, TH, ITERS, true>(ln, cur, bq, b_cur, b_nxt, k, acc);
  sched_group<0x100, 2>();
  sched_group<0x008, 4>();
  sched_fence();
}

// macro tile: 256 rows x 128 TJ tokens; waves 2 (rows) x 4 (tokens), a wave owns 128 rows x 32 TJ tokens.
// nsplit > 1: K is split over workgroups and a workgroup stores an fp32 partial tile (k_reduce_splits adds them).
template <int DT, int TJ>
__global__ void __launch_bounds__(512) k_mm_tile32(const uint4* __restrict__ A, const uint16_t* __restrict__ meta16,
                                                    const uint4* __restrict__ Xf, uint16_t* __restrict__ Y,
                                                    float* __restrict__ partial, long long M, long long N, long long Mp,
                                                    long long Np, long long Kp, long long n_tiles, long long ntb, int nsplit, int sps,
                                                    int band) {
  using State = TileState<1, 8, 2 * TJ, 4>;
  constexpr int ASLOTS = State::ASLOTS;
  constexpr int NTT = 8 * TJ;  // token tiles of 16 in the macro tile
  __shared__ uint4 s_a0[ASLOTS];
  __shared__ uint4 s_a1[ASLOTS];
  __shared__ uint4 s_a2[ASLOTS];
  __shared__ uint4 s_b0[NTT * 128];
  __shared__ uint4 s_b1[NTT * 128];
  __shared__ uint4 s_b2[NTT * 128];
  __shared__ uint32_t s_m0[ASLOTS];
  __shared__ uint32_t s_m1[ASLOTS];
  __shared__ uint32_t s_m2[ASLOTS];
  uint4* __restrict__ sa0 = s_a0;
  uint4* __restrict__ sa1 = s_a1;
  uint4* __restrict__ sa2 = s_a2;
  uint4* __restrict__ sb0 = s_b0;
  uint4* __restrict__ sb1 = s_b1;
  uint4* __restrict__ sb2 = s_b2;
  uint32_t* __restrict__ sm0 = s_m0;
  uint32_t* __restrict__ sm1 = s_m1;
  uint32_t* __restrict__ sm2 = s_m2;
  const int tid = threadIdx.x;
  State st;
  st.lane = (unsigned)(tid & 63);
  st.wave = (unsigned)wave_uniform(tid >> 6);
  st.wr = st.wave / 4;
  st.wc = st.wave % 4;
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  // XCD x (= blockIdx % 8) works through items [x * per, (x + 1) * per); an item is a macro tile and one of the
  // nsplit ranges of K stages (the split varies fastest)
  const long long n_items = n_tiles * nsplit;
  const long long per = (n_items + 7) / 8;
  const long long item = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((long long)(blockIdx.x >> 3) >= per || item >= n_items) return;
  const long long tile = item / nsplit;
  const int split = (int)(item % nsplit);
  st.k0 = (unsigned)((long long)split * sps);
  st.k1 = (unsigned)(((long long)(split + 1) * sps < nks) ? (long long)(split + 1) * sps : nks);
  long long rb, tb;
  tile_coords(tile, n_tiles, ntb, band, rb, tb);
  const long long rt_macro = rb * 16, tt_base = tb * NTT;
#pragma unroll
  for (int p = 0; p < State::ACOPIES; p++) {
    const long long rtl = State::NW * p + st.wave;
    const long long rt = (rt_macro + rtl < nrt) ? rt_macro + rtl : nrt - 1;
    st.a_src[p] = A + rt * nks * 64;
    st.m_src[p] = reinterpret_cast<const uint32_t*>(meta16) + rt * (nks / 4) * 128;
  }
#pragma unroll
  for (int p = 0; p < State::BCOPIES; p++) {
    const long long ttl = (State::NW / 2) * p + (st.wave >> 1);
    const long long tt = (tt_base + ttl < ntt) ? tt_base + ttl : ntt - 1;
    st.x_src[p] = Xf + tt * (2 * nks) * 64;
  }
  st.x_lane = (unsigned)(tid & 127);
  Tile32Lane ln;
  const unsigned r32 = st.lane & 31u, h = st.lane >> 5;
  ln.a_base = (st.wr * 8u + (r32 >> 4)) * 64u + 16u * h + (r32 & 15u);
  ln.b_base = (st.wc * (2u * TJ) + (r32 >> 4)) * 128u + 16u * h + (r32 & 15u);
  floatx16_t acc[4][TJ];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < TJ; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  const unsigned last = st.k1 - 1, kb = st.k0;
  tile_prefetch_b<1, 8, 2 * TJ, 4>(st, sb0, kb);
  tile_prefetch_a<1, 8, 2 * TJ, 4>(st, sa0, sm0, kb);
  tile_prefetch_b<1, 8, 2 * TJ, 4>(st, sb1, kb + 1 < st.k1 ? kb + 1 : last);
  tile_prefetch_a<1, 8, 2 * TJ, 4>(st, sa1, sm1, kb + 1 < st.k1 ? kb + 1 : last);
  tile_prefetch_a<1, 8, 2 * TJ, 4>(st, sa2, sm2, kb + 2 < st.k1 ? kb + 2 : last);
  sched_fence();
  tile_arrive<0>();
  Tile32Regs r0, r1;
  tile32_load_a(ln, sa0, sm0, r0);
  sched_fence();
  tile_arrive<0>();
  TileB bq;
  bq.b0 = sb0[ln.b_base];
  bq.b1 = sb0[ln.b_base + 32];
  unsigned k = kb;
  for (; k + 3 <= st.k1; k += 3) {
    tile32_stage<DT, TJ>(st, ln, r0, r1, bq, sb0, sb1, sa1, sm1, sb2, sa0, sm0, k, acc);
    tile32_stage<DT, TJ>(st, ln, r1, r0, bq, sb1, sb2, sa2, sm2, sb0, sa1, sm1, k + 1, acc);
    tile32_stage<DT, TJ>(st, ln, r0, r1, bq, sb2, sb0, sa0, sm0, sb1, sa2, sm2, k + 2, acc);
    r0 = r1;
  }
  if (k < st.k1) tile32_stage<DT, TJ>(st, ln, r0, r1, bq, sb0, sb1, sa1, sm1, sb2, sa0, sm0, k, acc);
  if (k + 1 < st.k1) tile32_stage<DT, TJ>(st, ln, r1, r0, bq, sb1, sb2, sa2, sm2, sb0, sa1, sm1, k + 1, acc);
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no DMA into this workgroup's LDS is left in flight
#endif
  __syncthreads();  // every wave is done with the ring: its buffers now carry the outputs

  const long long t_wave = (tt_base + st.wc * (2 * TJ)) * 16;  // first token and first output feature of this wave's tile
  const long long n_wave = (rt_macro + st.wr * 8) * 16;
  // epilogue: wave w transposes its 128 rows x 32 TJ tokens, 32 tokens at a time, in a private LDS slice (32 tokens x
  // (256 + 16) bytes, carved out of the weight and activation rings) and stores 256-byte runs of Y
  constexpr unsigned EP_ROW = 272, EP_SLICE = 32 * EP_ROW;
  // TJ = 2: eight slices at once (three in each of two activation buffers, one in each of two weight buffers);
  // TJ = 1 (buffers half the size): four slices, waves 0-3 first, then waves 4-7
  constexpr int PHASES = TJ == 1 ? 2 : 1;
  static_assert((TJ == 2 ? 3 * EP_SLICE : EP_SLICE) <= NTT * 128 * 16 && EP_SLICE <= ASLOTS * 16, "the epilogue slices fit the rings");
  unsigned char* ep;
  if (TJ == 2)
    ep = st.wave < 3 ? reinterpret_cast<unsigned char*>(s_b0) + st.wave * EP_SLICE
                     : (st.wave < 6 ? reinterpret_cast<unsigned char*>(s_b1) + (st.wave - 3u) * EP_SLICE
                                    : (st.wave == 6 ? reinterpret_cast<unsigned char*>(s_a0) : reinterpret_cast<unsigned char*>(s_a1)));
  else
    ep = (st.wave & 3u) == 0 ? reinterpret_cast<unsigned char*>(s_a0)
                             : ((st.wave & 3u) == 1 ? reinterpret_cast<unsigned char*>(s_a1)
                                                    : ((st.wave & 3u) == 2 ? reinterpret_cast<unsigned char*>(s_a2) : reinterpret_cast<unsigned char*>(s_b0)));
  const bool wide = (N & 7) == 0 && nsplit == 1;  // 16-byte stores of 8 output features
  if (wide) {
#pragma unroll
    for (int ph = 0; ph < PHASES; ph++)
#pragma unroll
      for (int j = 0; j < TJ; j++) {
        const bool mine = PHASES == 1 || (int)(st.wave >> 2) == ph;  // wave-uniform
        if (mine) {
#pragma unroll
          for (int i = 0; i < 4; i++)
#pragma unroll
            for (int a = 0; a < 4; a++) {
              uint2 v;
              v.x = esp_from_float<DT>(acc[i][j][4 * a]) | ((uint32_t)esp_from_float<DT>(acc[i][j][4 * a + 1]) << 16);
              v.y = esp_from_float<DT>(acc[i][j][4 * a + 2]) | ((uint32_t)esp_from_float<DT>(acc[i][j][4 * a + 3]) << 16);
              *reinterpret_cast<uint2*>(ep + r32 * EP_ROW + (32 * i + 8 * a + 4 * h) * 2) = v;
            }
        }
        __syncthreads();
        if (mine) {
#pragma unroll
          for (int p = 0; p < 8; p++) {
            const unsigned tl = p * 4u + (st.lane >> 4), piece = st.lane & 15u;
            const uint4 v = *reinterpret_cast<const uint4*>(ep + tl * EP_ROW + piece * 16u);
            const long long t = t_wave + 32 * j + tl;
            const long long n = n_wave + piece * 8;
            if (t < M && n + 8 <= N) *reinterpret_cast<uint4*>(Y + t * N + n) = v;
          }
        }
        __syncthreads();
      }
  } else {
#pragma unroll
    for (int j = 0; j < TJ; j++)
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int a = 0; a < 4; a++) {
          const long long t = t_wave + 32 * j + r32;
          const long long n = n_wave + 32 * i + 8 * a + 4 * h;
          const floatx4_t v = {acc[i][j][4 * a], acc[i][j][4 * a + 1], acc[i][j][4 * a + 2], acc[i][j][4 * a + 3]};
          if (nsplit > 1) {
            if (t < Mp && n < Np) *reinterpret_cast<floatx4_t*>(partial + ((long long)split * Mp + t) * Np + n) = v;
          } else {
            store_y4<DT>(Y, M, N, t, n, v);
          }
        }
  }
}

// ------------------------------------------------------------------------------------------------
// variant "stream" (M <= 128, bound by reading the weights): a workgroup of NW waves owns NW RT row
// tiles and all MT token tiles over a range of K; wave w owns row tiles (NW rb + w) RT .. + RT.
// Weights go HBM -> registers, one 64-channel step at a time, NB - 1 steps ahead (registers, not LDS,
// hold the bytes in flight: that is what lets a CU keep enough of them under way); the step's slice of
// the staged activations (MT * 2 KiB) is shared by the waves through a ring of NB LDS buffers filled
// by DMA.  Both kinds of load keep their program order, so one counted wait per step covers them.
// Work is cut without regard to row blocks: the steps of all row blocks, nks each, form one sequence
// that is cut into equal spans, one per workgroup, as many as the chip runs at once - no second, partly
// filled round of workgroups.  A span that covers a whole row block stores Y; otherwise it writes an
// fp32 partial tile, and k_reduce_pieces adds the pieces of a row block in ascending order.
//
// Two things keep the compiler's own waits out of the loop (it adds a full vmcnt(0) wherever it needs
// any wait on a register load while a DMA into LDS is pending): the loop body runs at least once and
// has no branches, so the loads stay in the order written here and the explicit counted wait already
// covers every register the multiplies read; steps past the end of the K range (the trip count is
// rounded up to whole rings) load the last real step again and multiply it by zeros.
// ------------------------------------------------------------------------------------------------
template <int SPARSE, int RT>
struct StreamRegs {
  uint4 a[RT];
  uint4 a2[SPARSE ? 1 : RT];
  int idx[RT];
};

template <int SPARSE, int MT, int RT, int NW>
struct StreamState {
  static constexpr int BC = (2 * MT + NW - 1) / NW;          // DMA copies of activations per lane and step
  static constexpr int GSZ = 2 * RT + BC;                    // vector-memory operations per step and wave
  const uint4* a_row[RT];     // per row tile: base of its weights
  const uint32_t* m_row[RT];  // ... and of its index words (one word = the 16-bit index halves of two steps)
  const uint4* x_src[BC];     // wave-uniform bases of this wave's DMA copies (token tile q / 2, half q % 2)
  unsigned x_dst[BC];         // ... and where they land in a ring buffer, in units
  unsigned lane, wave;
  const uint4* lut;           // 4:8: the byte-permute selectors of every pattern code (LDS)
};

template <int SPARSE, int MT, int RT, int NW>
__device__ __forceinline__ void stream_issue(const StreamState<SPARSE, MT, RT, NW>& st, StreamRegs<SPARSE, RT>& r, uint4* sb,
                                             unsigned ks) {
  using State = StreamState<SPARSE, MT, RT, NW>;
#pragma unroll
  for (int i = 0; i < RT; i++) {
    if (SPARSE) {
      r.a[i] = load_stream_16(st.a_row[i] + ((size_t)ks * 64 + st.lane));
      r.idx[i] = (int)st.m_row[i][((size_t)(ks >> 2) * 64 + st.lane) * 2 + ((ks >> 1) & 1u)];
    } else {
      r.a[i] = load_stream_16(st.a_row[i] + ((size_t)(2 * ks) * 64 + st.lane));
      r.a2[i] = load_stream_16(st.a_row[i] + ((size_t)(2 * ks + 1) * 64 + st.lane));
    }
  }
#pragma unroll
  for (int p = 0; p < State::BC; p++) global_to_lds_16(st.x_src[p] + ((size_t)(2 * ks) * 64 + st.lane), sb + st.x_dst[p]);
}

// PAR = parity of the step: which half of the index word belongs to it; live = false: multiply by zeros
template <int DT, int SPARSE, int MT, int RT, int NW, int PAR>
__device__ __forceinline__ void stream_multiply(const StreamState<SPARSE, MT, RT, NW>& st, const StreamRegs<SPARSE, RT>& r,
                                                const uint4* sb, floatx4_t (&acc)[RT][MT], bool live) {
  const uint32_t keep = live ? 0xffffffffu : 0u;
  uint4 a[RT], a2[SPARSE ? 1 : RT];
#pragma unroll
  for (int i = 0; i < RT; i++) {
    a[i] = uint4{r.a[i].x & keep, r.a[i].y & keep, r.a[i].z & keep, r.a[i].w & keep};
    if (!SPARSE) a2[i] = uint4{r.a2[i].x & keep, r.a2[i].y & keep, r.a2[i].z & keep, r.a2[i].w & keep};
  }
  // 4:8: the dense operands of the two half steps, from the unit's kept values and the step's two pattern codes
  uint4 e0[SPARSE == 2 ? RT : 1], e1[SPARSE == 2 ? RT : 1];
  if constexpr (SPARSE == 2) {
#pragma unroll
    for (int i = 0; i < RT; i++) expand_4_8<1>(a[i], (uint32_t)r.idx[i] >> (16 * PAR), st.lut, 0u, e0[i], e1[i]);
    sched_fence();  // the selector reads stay out of the read / multiply order set below
  }
  // the activations of token tile j + 1 are read while tile j is multiplied
  uint4 b0[2], b1[2];
  b0[0] = sb[st.lane];
  b1[0] = sb[64 + st.lane];
#pragma unroll
  for (int j = 0; j < MT; j++) {
    if (j + 1 < MT) {
      b0[(j + 1) & 1] = sb[(2 * j + 2) * 64 + st.lane];
      b1[(j + 1) & 1] = sb[(2 * j + 3) * 64 + st.lane];
    }
#pragma unroll
    for (int i = 0; i < RT; i++) {
      if constexpr (SPARSE == 1) {
        acc[i][j] = smfmac16<DT, PAR>(a[i], b0[j & 1], b1[j & 1], acc[i][j], r.idx[i]);
      } else if constexpr (SPARSE == 2) {
        acc[i][j] = mfma16<DT>(e0[i], b0[j & 1], acc[i][j]);
        acc[i][j] = mfma16<DT>(e1[i], b1[j & 1], acc[i][j]);
      } else {
        acc[i][j] = mfma16<DT>(a[i], b0[j & 1], acc[i][j]);
        acc[i][j] = mfma16<DT>(a2[i], b1[j & 1], acc[i][j]);
      }
    }
  }
  // issue order: reads of tile 0, then per tile the reads of the next one ahead of its multiplies
  constexpr int MM = (SPARSE == 1 ? 1 : 2) * RT;
  sched_group<0x100, 2>();
#pragma unroll
  for (int j = 0; j + 1 < MT; j++) {
    sched_group<0x100, 2>();
    sched_group<0x008, MM>();
  }
  sched_group<0x008, MM>();
}

// one step: wait for the loads of step ks (NB - 2 newer groups may be outstanding), meet the other waves (their
// DMA of this step has landed too, and they are done with the buffer the next DMA overwrites), issue the loads
// of step ks + NB - 1, multiply step ks
template <int DT, int SPARSE, int MT, int RT, int NW, int NB, int PAR>
__device__ __forceinline__ void stream_step(const StreamState<SPARSE, MT, RT, NW>& st, const StreamRegs<SPARSE, RT>& cur,
                                            StreamRegs<SPARSE, RT>& pre, const uint4* sb_cur, uint4* sb_pre, floatx4_t (&acc)[RT][MT],
                                            unsigned ks, unsigned k1) {
  constexpr int OUT = (NB - 2) * StreamState<SPARSE, MT, RT, NW>::GSZ;
  static_assert(OUT <= 63, "vmcnt is a 6-bit counter");
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_waitcnt((OUT & 15) | ((OUT >> 4) << 14) | 0x0F70);  // vmcnt(OUT)
  __builtin_amdgcn_s_barrier();
#endif
  const unsigned kp = ks + (NB - 1);
  stream_issue<SPARSE, MT, RT, NW>(st, pre, sb_pre, kp < k1 ? kp : k1 - 1);
  sched_fence();  // the loads of one step stay together: the counted wait relies on their order
  stream_multiply<DT, SPARSE, MT, RT, NW, PAR>(st, cur, sb_cur, acc, ks < k1);
  sched_fence();
}

template <int DT, int SPARSE, int MT, int RT, int NW, int NB>
__device__ __attribute__((always_inline)) void stream_pipeline(uint4* __restrict__ sb, const uint4* __restrict__ A,
                                                               const uint16_t* __restrict__ meta16, const uint4* __restrict__ Xf,
                                                               uint16_t* __restrict__ Y, float* __restrict__ partial, long long M,
                                                               long long N, long long Mp, long long Np, long long Kp, long long span,
                                                               const uint4* lut) {
  static_assert(NB % 2 == 0, "the parity of a step is that of its ring slot");
  using State = StreamState<SPARSE, MT, RT, NW>;
  constexpr int BUF = MT * 128;  // units per ring buffer: [MT token tiles][2 half steps][64 lanes]
  State st;
  const int tid = threadIdx.x;
  st.lane = (unsigned)(tid & 63);
  st.wave = (unsigned)wave_uniform(tid >> 6);
  st.lut = lut;
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  const long long nrb = (nrt + NW * RT - 1) / (NW * RT);
  const long long s_begin = (long long)blockIdx.x * span;
  const long long s_end = s_begin + span < nrb * nks ? s_begin + span : nrb * nks;
#pragma unroll
  for (int p = 0; p < State::BC; p++) {
    const long long q = ((long long)NW * p + st.wave) % (2 * MT);  // chunk of 64 units (more waves than chunks: copied twice)
    long long tt = q / 2;
    tt = tt < ntt ? tt : ntt - 1;
    st.x_src[p] = Xf + (tt * (2 * nks) + (q & 1)) * 64;
    st.x_dst[p] = (unsigned)q * 64;
  }
  // the segments of this span: one per row block it touches (spans and nks, and hence k0 and k1, are even)
  for (long long s = s_begin; s < s_end;) {
    const long long rb = s / nks;
    const unsigned k0 = (unsigned)(s - rb * nks);
    const unsigned k1 = (unsigned)((s_end - rb * nks) < nks ? (s_end - rb * nks) : nks);
    s += k1 - k0;
#pragma unroll
    for (int i = 0; i < RT; i++) {
      long long rt = (rb * NW + st.wave) * RT + i;
      rt = rt < nrt ? rt : nrt - 1;  // clamp: duplicate work, discarded in the epilogue
      st.a_row[i] = A + (SPARSE ? rt * nks : rt * (2 * nks)) * 64;
      st.m_row[i] = reinterpret_cast<const uint32_t*>(meta16) + rt * (nks / 4) * 128;
    }
    floatx4_t acc[RT][MT];
#pragma unroll
    for (int i = 0; i < RT; i++)
#pragma unroll
      for (int j = 0; j < MT; j++) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

    __syncthreads();  // the previous segment's reads of the ring are done
    // k0 is even, so the parity of a step is that of its ring slot
    StreamRegs<SPARSE, RT> r[NB];
#pragma unroll
    for (int q = 0; q < NB - 1; q++) {
      stream_issue<SPARSE, MT, RT, NW>(st, r[q], sb + q * BUF, k0 + q < k1 ? k0 + q : k1 - 1);
      sched_fence();
    }
    const unsigned trips = (k1 - k0 + NB - 1) / NB;
    unsigned ks = k0, t = 0;
    do {  // at least one trip
#pragma unroll
      for (int q = 0; q < NB; q++) {
        if (q & 1)
          stream_step<DT, SPARSE, MT, RT, NW, NB, 1>(st, r[q], r[(q + NB - 1) % NB], sb + q * BUF, sb + ((q + NB - 1) % NB) * BUF,
                                                     acc, ks + q, k1);
        else
          stream_step<DT, SPARSE, MT, RT, NW, NB, 0>(st, r[q], r[(q + NB - 1) % NB], sb + q * BUF, sb + ((q + NB - 1) % NB) * BUF,
                                                     acc, ks + q, k1);
      }
      ks += NB;
    } while (++t < trips);
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no DMA into the ring is left in flight
#endif
    // the store addresses are formed here, from a lane number the compiler cannot trace back: formed ahead of the
    // segment loop they would occupy registers all through the multiply loop
    unsigned lane_e = st.lane;
    asm volatile("" : "+v"(lane_e));
    const int c = (int)(lane_e & 15), g = (int)(lane_e >> 4);
    const bool whole = k0 == 0 && k1 == (unsigned)nks;
    const long long piece = (long long)blockIdx.x - (rb * nks) / span;
#pragma unroll
    for (int i = 0; i < RT; i++) {
      const long long rt = (rb * NW + st.wave) * RT + i;
      if (rt >= nrt) continue;
#pragma unroll
      for (int j = 0; j < MT; j++) {
        if (j >= ntt) continue;
        const long long tk = (long long)j * 16 + c, n = rt * 16 + g * 4;
        if (whole)
          store_y4<DT>(Y, M, N, tk, n, acc[i][j]);
        else
          *reinterpret_cast<floatx4_t*>(partial + (piece * Mp + tk) * Np + n) = acc[i][j];
      }
    }
  }
}

template <int DT, int SPARSE, int MT, int RT, int NW, int NB>
__global__ void __launch_bounds__(NW * 64) k_mm_stream(const uint4* __restrict__ A, const uint16_t* __restrict__ meta16,
                                                        const uint4* __restrict__ Xf, uint16_t* __restrict__ Y,
                                                        float* __restrict__ partial, long long M, long long N, long long Mp,
                                                        long long Np, long long Kp, long long span) {
  extern __shared__ uint4 s_stream[];  // NB ring buffers of MT * 128 units
  __shared__ uint4 s_lut[SPARSE == 2 ? LUT48_CODES : 1];
  if (SPARSE == 2) {
    fill_expand_lut<1>(s_lut, (int)threadIdx.x);
    __syncthreads();
  }
  stream_pipeline<DT, SPARSE, MT, RT, NW, NB>(s_stream, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, span, s_lut);
}

// ------------------------------------------------------------------------------------------------
// variant table and host launcher
// ------------------------------------------------------------------------------------------------
enum { KIND_WAVE = 0, KIND_KSPLIT = 1, KIND_TILE = 2, KIND_STREAM = 3 };
struct Variant {
  const char* name;
  int kind;
  int rt, tt;      // row tiles / token tiles per wave (ksplit: row tiles per workgroup, tt unused: MT follows M)
  int split_mode;  // wave and tile kinds: 0 = never split K, 1 = split K over workgroups to fill the chip
  int nw;          // ksplit kind: waves per workgroup; tile kind: waves along the tokens (the workgroup has 2 x nw waves)
  int quads;       // ksplit kind: 1 = a wave takes four consecutive steps with one index load (2:4 and 4:8, at most 16 tokens)
  int x32;         // tile kind: 1 = the 32x32x32 form of the sparse instruction and the epilogue through LDS (2:4 only)
  int depth;       // tile kind: token tiles the activation operands are read ahead (0 = 1)
  int half;        // tile kind: 1 = dense only, stages of 32 channels and the macro tile of the sparse form
  int four8;       // tile kind: 1 = 4:8 only, bitmaps expanded to dense operands in registers, dense instruction
};
static const Variant kVariants[] = {
    {"wave_r2_t1_splitk", KIND_WAVE, 2, 1, 1, 0},
    {"wave_r2_t2_splitk", KIND_WAVE, 2, 2, 1, 0},
    {"wave_r4_t2", KIND_WAVE, 4, 2, 0, 0},
    {"wave_r4_t4", KIND_WAVE, 4, 4, 0, 0},
    {"ksplit_w16_r1", KIND_KSPLIT, 1, 0, 0, 16},
    {"ksplit_w16_r2", KIND_KSPLIT, 2, 0, 0, 16},
    {"ksplit_w8_r1", KIND_KSPLIT, 1, 0, 0, 8},
    {"ksplit_w8_r2", KIND_KSPLIT, 2, 0, 0, 8},
    {"ksplit_w8_r4", KIND_KSPLIT, 4, 0, 0, 8},
    {"ksplit_w16_r3", KIND_KSPLIT, 3, 0, 0, 16},
    {"tile_t256", KIND_TILE, 8, 8, 0, 2},     // 256 rows (dense 128) x 256 tokens per workgroup, 4 waves
    {"tile_t128", KIND_TILE, 8, 4, 0, 2},     // 256 rows (dense 128) x 128 tokens per workgroup, 4 waves
    {"tile_w8_t256", KIND_TILE, 8, 4, 0, 4},  // 256 rows (dense 128) x 256 tokens per workgroup, 8 waves (two per SIMD)
    {"tile_w8_t128", KIND_TILE, 8, 2, 0, 4},  // 256 rows (dense 128) x 128 tokens per workgroup, 8 waves
    {"tile_w8_r128_t128", KIND_TILE, 4, 2, 0, 4},         // 128 rows (dense 64) x 128 tokens per workgroup, 8 waves
    {"tile_w8_r128_t128_splitk", KIND_TILE, 4, 2, 1, 4},  // ... with K split over workgroups (M <= 512)
    {"tile_w8_r128_t64_splitk", KIND_TILE, 4, 1, 1, 4},   // 128 rows (dense 64) x 64 tokens, K split
    // stream kind: nw waves x rt row tiles per workgroup, all tokens (M <= 128), K split; tt = ring slots
    {"stream_w8_r1_d3", KIND_STREAM, 1, 4, 1, 8},
    {"stream_w8_r1_d7", KIND_STREAM, 1, 8, 1, 8},
    {"stream_w8_r2_d3", KIND_STREAM, 2, 4, 1, 8},
    {"stream_w8_r2_d5", KIND_STREAM, 2, 6, 1, 8},
    {"ksplit_w8_r6", KIND_KSPLIT, 6, 0, 0, 8},  // M <= 32: 96 rows per workgroup, the activations are re-read by fewer workgroups
    {"ksplit_w8_r3", KIND_KSPLIT, 3, 0, 0, 8},
    {"tile_w8_t128_splitk", KIND_TILE, 8, 2, 1, 4},  // 256 rows (dense 128) x 128 tokens, K split (M <= 512)
    // decode kernels with K split over workgroups (tt = splits; single products): for matrices with few rows and
    // tens of tokens, where each workgroup re-reading all the staged activations costs several times the weights
    {"ksplit_w16_r4_k4", KIND_KSPLIT, 4, 4, 1, 16},
    {"ksplit_w16_r2_k2", KIND_KSPLIT, 2, 2, 1, 16},
    {"ksplit_w8_r4_k4", KIND_KSPLIT, 4, 4, 1, 8},
    // macro tiles of 288 / 320 rows x 128 tokens: row counts with a factor 9 or 5 (9216, 5120) then give a number of
    // macro tiles that fills the 256 CUs exactly where 256-row tiles leave a partly filled round
    {"tile_w8_r288_t128", KIND_TILE, 9, 2, 0, 4},
    {"tile_w8_r320_t128", KIND_TILE, 10, 2, 0, 4},
    // decode kernels for at most 16 tokens whose waves take four consecutive steps and read their index halves with
    // one 8-byte load (2:4: 7-13 % on 4096 x 11008, 2-5 % on q/k/v in one launch, level or behind elsewhere; 4:8: two pattern codes per step)
    {"ksplit_w8_r1_q", KIND_KSPLIT, 1, 0, 0, 8, 1},
    {"ksplit_w16_r1_q", KIND_KSPLIT, 1, 0, 0, 16, 1},
    {"ksplit_w8_r2_q", KIND_KSPLIT, 2, 0, 0, 8, 1},
    {"ksplit_w8_r4_q", KIND_KSPLIT, 4, 0, 0, 8, 1},
    // stream kernel with nine waves (144 rows per workgroup): 36864 rows are then exactly 256 row blocks, one per CU,
    // and no span cuts a row block (no partial tiles, no reduction launch)
    {"stream_w9_r1_d3", KIND_STREAM, 1, 4, 1, 9},
    // eleven waves (176 rows): 22016 rows are 126 row blocks, two aligned spans each
    {"stream_w11_r1_d3", KIND_STREAM, 1, 4, 1, 11},
    // the 8-wave 256 x 256 tile with v_smfmac_f32_32x32x32 and outputs stored in 256-byte runs (2:4 only)
    {"tile32_w8_t256", KIND_TILE, 8, 4, 0, 4, 0, 1},
    {"tile32_w8_t128", KIND_TILE, 8, 2, 0, 4, 0, 1},         // ... 256 rows x 128 tokens
    {"tile32_w8_t128_splitk", KIND_TILE, 8, 2, 1, 4, 0, 1},  // ... with K split over workgroups (M <= 512)
    // the 4-wave 256 x 256 tile (one wave per SIMD, 256 accumulators each: fewer LDS reads per multiply) with the
    // activation operands read three token tiles ahead, so that the wave's own multiplies cover the LDS latency
    {"tile_t256_d3", KIND_TILE, 8, 8, 0, 2, 0, 0, 3},
    // dense only: 256 rows x 256 (128) tokens per workgroup in stages of 32 channels - the operand bytes per multiply of
    // the sparse macro tile, half those of the 128-row dense forms above
    {"tile_w8_t256_h", KIND_TILE, 8, 4, 0, 4, 0, 0, 0, 1},
    {"tile_w8_t128_h", KIND_TILE, 8, 2, 0, 4, 0, 0, 0, 1},
    {"tile_w8_t256_h_splitk", KIND_TILE, 8, 4, 1, 4, 0, 0, 0, 1},  // ... with K split over workgroups (M <= 512)
    {"tile_w8_t128_h_splitk", KIND_TILE, 8, 2, 1, 4, 0, 0, 0, 1},
    // 4:8 only: the 2:4 kernel's copies, rings and 64-channel stages; while a wave reads the next stage's weight units out
    // of LDS it expands each unit and its two pattern codes into the dense operands of two 16x16x32 multiplies (selectors
    // from a table in LDS, replicated so that the lookups are free of bank conflicts).  128 rows x 256 tokens per
    // workgroup (a wave expands 4 row tiles for 4 token tiles) or 256 rows x 128 tokens
    {"tile48_w8_r128_t256", KIND_TILE, 4, 4, 0, 4, 0, 0, 0, 0, 1},
    {"tile48_w8_t128", KIND_TILE, 8, 2, 0, 4, 0, 0, 0, 0, 1},
    {"tile48_w8_t128_splitk", KIND_TILE, 8, 2, 1, 4, 0, 0, 0, 0, 1},  // ... with K split over workgroups (M <= 512)
};
static const int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

int esp_num_variants() { return kNumVariants; }
const char* esp_variant_name(int v) { return kVariants[v].name; }

bool esp_variant_applicable(int v, long long M, long long N, long long K, int sparse) {
  (void)N;
  (void)K;
  if (v < 0 || v >= kNumVariants) return false;
  const Variant& var = kVariants[v];
  if (var.four8 && (sparse != 2 || M < 64)) return false;
  if (sparse == 2 && var.kind == KIND_STREAM) return M <= 128 && var.tt == 4;  // the stream kernels with a ring of four slots
  if (sparse == 2 && !var.four8) {
    // 4:8: otherwise decode kernels only; longer inputs go through them 64 tokens at a time
    if (var.kind != KIND_KSPLIT || (var.quads && M > 16)) return false;
    const long long mc = M < 64 ? M : 64;
    const long long mt = mc <= 16 ? 1 : (mc <= 32 ? 2 : 4);
    return (long long)var.nw * var.rt * mt * 1024 <= 160 * 1024;
  }
  if (var.split_mode == 1 && esp_split_capacity(M) == 1) return false;  // no room for partial tiles beyond 512 tokens
  if (var.kind == KIND_KSPLIT) {
    if (M > 64) return false;
    if (var.quads && (sparse == 0 || M > 16)) return false;
    const long long mt = M <= 16 ? 1 : (M <= 32 ? 2 : 4);  // token tiles; the waves' partial tiles must fit the LDS
    if ((long long)var.nw * var.rt * mt * 1024 > 160 * 1024) return false;
  }
  if (var.kind == KIND_TILE && M < 64) return false;
  if (var.x32 && sparse != 1) return false;
  if (var.half && sparse != 0) return false;
  if (var.kind == KIND_STREAM && M > 128) return false;
  return true;
}

static int variant_index(const char* name) {
  for (int v = 0; v < kNumVariants; v++)
    if (!strcmp(kVariants[v].name, name)) return v;
  return -1;
}

int esp_default_variant(long long M, long long N, long long K, int sparse) {
  if (sparse == 2 && M > 128)  // 4:8 at prefill sizes; few macro tiles (and room for partial tiles): K split over workgroups
  {
    if (((N + 127) / 128) * ((M + 255) / 256) >= 128 || esp_split_capacity(M) == 1) return variant_index("tile48_w8_r128_t256");
    return variant_index("tile48_w8_t128_splitk");
  }
  if (M <= 32) {
    const long long nrt = esp_round_up(N, 16) / 16;
    return nrt <= 320 ? 4 : 5;  // ksplit_w16_r1 / ksplit_w16_r2
  }
  if (M <= 128) {
    // stream kernels: the number of waves (rows per workgroup) whose row blocks, each cut into p equal spans of an even
    // number of steps, come closest to one workgroup per CU without a span crossing a row block
    const long long nrt = esp_round_up(N, 16) / 16, nks = esp_round_up(K, 256) / 64;
    static const struct { int nw; const char* name; } cand[] = {{8, "stream_w8_r1_d3"}, {9, "stream_w9_r1_d3"}, {11, "stream_w11_r1_d3"}};
    long long best = 0;
    const char* pick = nullptr;
    for (const auto& c : cand) {
      const long long nrb = (nrt + c.nw - 1) / c.nw;
      if (nrb > 256) continue;
      long long pcs = 256 / nrb;
      while (pcs > 1 && (nks % pcs != 0 || (nks / pcs) % 2 != 0 || nks / pcs < 8)) pcs--;
      if (nrb * pcs > best) {
        best = nrb * pcs;
        pick = c.name;
      }
    }
    if (best >= 200) return variant_index(pick);
    return M <= 64 ? 19 : 17;  // stream_w8_r2_d3 / stream_w8_r1_d3 with spans cut where they fall
  }
  // 8-wave tile kernels: the largest macro tile that still gives half of the 256 CUs a tile
  const long long rows = sparse ? 256 : 128;
  const long long nrb = (N + rows - 1) / rows;
  if (nrb * ((M + 255) / 256) >= 128) {
    if (sparse == 1) return variant_index("tile32_w8_t256");
    // dense: the 256-row form with 32-channel stages once its macro tiles alone give half of the CUs a tile
    return ((N + 255) / 256) * ((M + 255) / 256) >= 128 ? variant_index("tile_w8_t256_h") : 12;  // else tile_w8_t256
  }
  if (nrb * ((M + 127) / 128) >= 128) return 13;  // tile_w8_t128
  return 14;                                       // tile_w8_r128_t128
}

// the built-in choice among the variants that keep no fp32 partial tiles in the workspace (for callers whose scratch
// is too small for them): a decode kernel up to 64 tokens, the tile kernels beyond
int esp_default_variant_without_partials(long long M, long long N, long long K, int sparse) {
  (void)K;
  if (M <= 64) return esp_round_up(N, 16) / 16 <= 320 ? 4 : 5;  // ksplit_w16_r1 / ksplit_w16_r2
  if (sparse == 2) return variant_index("tile48_w8_r128_t256");
  if (sparse == 1) return variant_index(M <= 128 ? "tile32_w8_t128" : "tile32_w8_t256");
  return variant_index(M <= 128 ? "tile_w8_t128_h" : "tile_w8_t256_h");
}

// tokens of the compact copy of the staged activations (0: none), written when there are at most 16 tokens
static int compact_tokens(long long M) {
  if (M > 16) return 0;
  int mc = 1;
  while (mc < M) mc *= 2;
  return mc;
}
// bytes of one staged activation matrix: the fragment-major form and, behind it, the compact copy
static size_t staged_bytes(long long M, long long K) {
  const size_t Mp = (size_t)esp_round_up(M, 16), Kp = (size_t)esp_round_up(K, 256);
  return (Mp + (size_t)compact_tokens(M)) * Kp * 2;  // a multiple of 512
}

size_t esp_workspace_bytes(long long M, long long N, long long K) {
  const size_t Mp = (size_t)esp_round_up(M, 16), Np = (size_t)esp_round_up(N, 16);
  size_t bytes = WS_HEADER_BYTES + staged_bytes(M, K);
  if (esp_split_capacity(M) > 1) bytes += (size_t)esp_split_capacity(M) * Mp * Np * 4;
  return bytes;
}

// what one variant really uses of the workspace: the header, the staged activations and - only for variants that split
// K over workgroups - the fp32 partial tiles
size_t esp_variant_workspace_bytes(int variant, long long M, long long N, long long K) {
  const Variant& v = kVariants[variant];
  const bool partial = v.split_mode == 1 || v.kind == KIND_STREAM;
  if (partial && esp_split_capacity(M) > 1) return esp_workspace_bytes(M, N, K);
  return (size_t)WS_HEADER_BYTES + staged_bytes(M, K);
}

// ------------------------------------------------------------------------------------------------
// Scratch for callers that cannot allocate: one array per GPU, in the library's own device image, held until the
// process ends.  The array's name is a host-side stand-in; its device address is looked up once per device (with
// that device current) and only that address is ever handed to kernels.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[ESPARSE_STATIC_SCRATCH_BYTES];
static std::atomic<void*> g_scratch_ptr[64];

int esp_static_scratch(esparse_ctx* ctx, void** out) {
  const int dev = ctx->device;
  ESP_REQUIRE(ctx, dev >= 0 && dev < 64, ESPARSE_EUNSUPPORTED, "device %d: the static scratch is kept for devices 0..63", dev);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    ESP_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));  // the caller has made ctx->device current
    ESP_REQUIRE(ctx, p && (reinterpret_cast<uintptr_t>(p) & 255u) == 0, ESPARSE_EHIP, "the static scratch has no usable device address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return ESPARSE_OK;
}

template <int DT, int SPARSE>
static void launch_wave_tile(const Variant& v, dim3 grid, hipStream_t st, const uint4* A, const uint2* meta, const uint4* Xf,
                             uint16_t* Y, float* partial, long long M, long long N, long long Mp, long long Np, long long Kp,
                             int nsplit, int sps, long long n_items) {
#define LAUNCH(R, T)                                                                                                      \
  hipLaunchKernelGGL((k_mm_wave_tile<DT, SPARSE, R, T>), grid, dim3(256), 0, st, A, meta, Xf, Y, partial, M, N, Mp, Np, Kp, \
                     nsplit, sps, n_items)
  if (v.rt == 2 && v.tt == 1) LAUNCH(2, 1);
  else if (v.rt == 2 && v.tt == 2) LAUNCH(2, 2);
  else if (v.rt == 4 && v.tt == 2) LAUNCH(4, 2);
  else LAUNCH(4, 4);
#undef LAUNCH
}

// Whether the decode kernel gathers the activations through theta itself (no staged copy, no staging launch): one or two
// tokens, a variant that keeps K inside the workgroup, the gathered copy (2 Kp bytes per token) fits beside the reduction
// buffer in the 64 KiB of LDS a launch may ask for without further ado - and the gather is cheap enough: every workgroup
// repeats it, so it pays while workgroups x channels stays small (4096 x 4096: 7.0 us against 6.5 + 2.1 for the staging
// launch; 36864 x 9216, 2304 workgroups: 77 us against 58 + 2.3, hence the limits).
static bool ksplit_folds(const Variant& v, long long M, long long Np, long long Kp) {
  if (v.kind != KIND_KSPLIT || v.split_mode != 0 || M > 2) return false;
  const long long mc = compact_tokens(M), groups = (Np / 16 + v.rt - 1) / v.rt;
  if (Kp * mc > 10240 || groups * Kp * mc > 3000000) return false;
  const size_t red = (size_t)v.nw * v.rt * 64 * 16, gathered = (size_t)2 * Kp * mc;
  return red + gathered <= 64 * 1024;
}

template <int DT, int SPARSE, int MT>
static void launch_ksplit(const Variant& v, hipStream_t st, KsplitArgs args, int count, long long M, long long N, long long Mp,
                          long long Np, long long Kp, int mc, int nsplit, bool fold) {
  const long long nrt = Np / 16, nks = Kp / 64;
  // K split over workgroups: single products only; splits of a multiple of four steps
  const long long sps = nsplit > 1 ? ((nks + nsplit - 1) / nsplit + 3) / 4 * 4 : nks;
  nsplit = (int)((nks + sps - 1) / sps);
  args.sps = (int)sps;
  dim3 grid((unsigned)((nrt + v.rt - 1) / v.rt), (unsigned)count, (unsigned)nsplit);
  fold = fold && MT == 1 && mc > 0 && nsplit == 1;
  const size_t smem = (size_t)v.nw * v.rt * MT * 64 * 16 + (fold ? (size_t)2 * Kp * mc : 0);
  const bool pairs = SPARSE != 0 && MT >= 2 && ((sps / 2) % v.nw) == 0 && nks % sps == 0;
  const bool quads = v.quads != 0;
#define LAUNCH(R, W)                                                                                                          \
  do {                                                                                                                        \
    if (MT == 1 && fold && SPARSE != 0 && quads && ((R == 1) || (W == 8 && (R == 2 || R == 4))))                              \
      hipLaunchKernelGGL((k_mm_ksplit<DT, SPARSE, MT, R, W, (SPARSE != 0 && MT == 1 && ((R == 1) || (W == 8 && (R == 2 || R == 4))) ? 2 : 0), MT == 1>), \
                         grid, dim3(W * 64), smem, st, args, M, N, Mp, Np, Kp, mc);                                           \
    else if (MT == 1 && fold)                                                                                                 \
      hipLaunchKernelGGL((k_mm_ksplit<DT, SPARSE, MT, R, W, 0, MT == 1>), grid, dim3(W * 64), smem, st, args, M, N, Mp, Np, Kp, mc); \
    else if (SPARSE != 0 && MT == 1 && quads && ((R == 1) || (W == 8 && (R == 2 || R == 4))))                                 \
      hipLaunchKernelGGL((k_mm_ksplit<DT, SPARSE, MT, R, W, (SPARSE != 0 && MT == 1 && ((R == 1) || (W == 8 && (R == 2 || R == 4))) ? 2 : 0)>), \
                         grid, dim3(W * 64), smem, st, args, M, N, Mp, Np, Kp, mc);                                           \
    else if (SPARSE != 0 && MT >= 2 && pairs)                                                                                 \
      hipLaunchKernelGGL((k_mm_ksplit<DT, SPARSE, MT, R, W, (SPARSE != 0 && MT >= 2 ? 1 : 0)>), grid, dim3(W * 64), smem, st, args, M, N, Mp, Np, \
                         Kp, mc);                                                                                             \
    else                                                                                                                      \
      hipLaunchKernelGGL((k_mm_ksplit<DT, SPARSE, MT, R, W, 0>), grid, dim3(W * 64), smem, st, args, M, N, Mp, Np, Kp, mc); \
  } while (0)
  if (v.nw == 16 && v.rt == 1) LAUNCH(1, 16);
  else if (v.nw == 16 && v.rt == 2) LAUNCH(2, 16);
  else if (v.nw == 16 && v.rt == 3) LAUNCH(3, 16);
  else if (v.nw == 8 && v.rt == 1) LAUNCH(1, 8);
  else if (v.nw == 8 && v.rt == 2) LAUNCH(2, 8);
  else if (v.nw == 8 && v.rt == 6) LAUNCH(6, 8);
  else if (v.nw == 8 && v.rt == 3) LAUNCH(3, 8);
  else if (v.nw == 16 && v.rt == 4) LAUNCH(4, 16);
  else LAUNCH(4, 8);
#undef LAUNCH
  if (nsplit > 1) {
    const long long e = M * (Np / 4);
    hipLaunchKernelGGL(k_reduce_splits<DT>, dim3((unsigned)((e + 255) / 256)), dim3(256), 0, st, args.partial, nsplit, M, N, Mp, Np, args.Y[0]);
  }
}

template <int DT, int SPARSE>
static int launch_tile(esparse_ctx* ctx, const Variant& v, hipStream_t st, const uint4* A, const uint16_t* meta16, const uint4* Xf,
                       uint16_t* Y, float* partial, long long M, long long N, long long Mp, long long Np, long long Kp) {
  // the dense operand is twice as wide: half the row tiles per wave
  const long long rtm = (SPARSE || v.half) ? 2 * v.rt : 2 * (v.rt / 2);  // row tiles per macro tile
  const long long nrt = Np / 16, ntt = Mp / 16, nks = (v.half ? 2 : 1) * (Kp / 64);  // nks: stages of the K loop
  const long long cols = (long long)v.nw * v.tt;  // token tiles per macro tile
  const long long nrb = (nrt + rtm - 1) / rtm, ntb = (ntt + cols - 1) / cols;
  const long long n_tiles = nrb * ntb;
  int nsplit = 1;
  long long sps = nks;
  if (v.split_mode == 1) {
    // about two workgroups per CU, splits of at least 8 stages (512 channels); no split once the macro
    // tiles alone cover half of the CUs (the fp32 partial tiles and their reduction then cost more)
    // M > 128 (at most 4 splits, larger partial tiles): as many splits as keep the items within one round of 256
    const long long want = M > 128 ? 256 / n_tiles : (n_tiles >= 128 ? 1 : (512 + n_tiles - 1) / n_tiles);
    nsplit = (int)std::max<long long>(1, std::min<long long>(std::min<long long>(want, nks / 8), esp_split_capacity(M)));
    sps = ((nks + nsplit - 1) / nsplit + 3) / 4 * 4;
    nsplit = (int)((nks + sps - 1) / sps);
  }
  const long long per = (n_tiles * nsplit + 7) / 8;
  dim3 grid((unsigned)(per * 8));
  // more than 8 token blocks: bands of 8 row blocks, so that the 32 workgroups an XCD runs at once share 8 weight panels
  // and 4 activation panels in its L2 instead of 1 and 32 (16384 tokens: 12-14 % faster); up to 8 token blocks the plain
  // order already gives each XCD a patch of 4 x 8
  const int band = ntb > 8 ? 8 : 1;
  if constexpr (SPARSE == 2) {
    if (!v.four8) return esp_fail(ctx, ESPARSE_EINVAL, "4:8 weights at prefill sizes go through the tile48 variants");
    if (v.tt == 4)
      hipLaunchKernelGGL((k_mm_tile<DT, 2, 4, 4, 4>), grid, dim3(512), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band);
    else
      hipLaunchKernelGGL((k_mm_tile<DT, 2, 8, 2, 4>), grid, dim3(512), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band);
    ESP_HIP(ctx, hipGetLastError());
  } else if (v.four8) {
    return esp_fail(ctx, ESPARSE_EINVAL, "the tile48 variants multiply 4:8 weights only");
  } else if (v.half) {
    if (SPARSE != 0) return esp_fail(ctx, ESPARSE_EINVAL, "the half-step tile kernel multiplies dense weights only");
    if (v.tt == 4)
      hipLaunchKernelGGL((k_mm_tile<DT, 3, 8, 4, 4>), grid, dim3(512), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band);
    else
      hipLaunchKernelGGL((k_mm_tile<DT, 3, 8, 2, 4>), grid, dim3(512), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band);
    ESP_HIP(ctx, hipGetLastError());
  } else if (v.x32) {
    if (SPARSE != 1) return esp_fail(ctx, ESPARSE_EINVAL, "the 32x32x32 tile kernel multiplies 2:4 weights only");
    if (v.tt == 4)
      hipLaunchKernelGGL((k_mm_tile32<DT, 2>), grid, dim3(512), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band);
    else
      hipLaunchKernelGGL((k_mm_tile32<DT, 1>), grid, dim3(512), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band);
    ESP_HIP(ctx, hipGetLastError());
  } else
  {
#define ESP_TILE(TRv, TCv, NWCv)                                                                                             \
  hipLaunchKernelGGL((k_mm_tile<DT, SPARSE, (SPARSE ? TRv : TRv / 2), TCv, NWCv>), grid, dim3(128 * NWCv), 0, st, A, meta16, Xf, Y, \
                     partial, M, N, Mp, Np, Kp, n_tiles, ntb, nsplit, (int)sps, band)
  if (v.rt == 8 && v.nw == 2 && v.tt == 8 && v.depth == 3)
    hipLaunchKernelGGL((k_mm_tile<DT, SPARSE, (SPARSE ? 8 : 4), 8, 2, 3>), grid, dim3(256), 0, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp,
                       n_tiles, ntb, nsplit, (int)sps, band);
  else if (v.rt == 8 && v.nw == 2 && v.tt == 8) ESP_TILE(8, 8, 2);
  else if (v.rt == 8 && v.nw == 2 && v.tt == 4) ESP_TILE(8, 4, 2);
  else if (v.rt == 8 && v.nw == 4 && v.tt == 4) ESP_TILE(8, 4, 4);
  else if (v.rt == 8 && v.nw == 4 && v.tt == 2) ESP_TILE(8, 2, 4);
  else if (v.rt == 4 && v.nw == 4 && v.tt == 2) ESP_TILE(4, 2, 4);
  else if (v.rt == 4 && v.nw == 4 && v.tt == 1) ESP_TILE(4, 1, 4);
  else if (v.rt == 9 && v.nw == 4 && v.tt == 2) ESP_TILE(9, 2, 4);
  else if (v.rt == 10 && v.nw == 4 && v.tt == 2) ESP_TILE(10, 2, 4);
  else return esp_fail(ctx, ESPARSE_EINVAL, "unknown tile variant");
#undef ESP_TILE
  ESP_HIP(ctx, hipGetLastError());
  }
  if (nsplit > 1) {
    const long long e = M * (Np / 4);
    if (DT == ESPARSE_F16)
      hipLaunchKernelGGL(k_reduce_splits<ESPARSE_F16>, dim3((unsigned)((e + 255) / 256)), dim3(256), 0, st, partial, nsplit, M, N, Mp, Np, Y);
    else
      hipLaunchKernelGGL(k_reduce_splits<ESPARSE_BF16>, dim3((unsigned)((e + 255) / 256)), dim3(256), 0, st, partial, nsplit, M, N, Mp, Np, Y);
    ESP_HIP(ctx, hipGetLastError());
  }
  return ESPARSE_OK;
}

template <int DT, int SPARSE, int MT, int RT, int NW, int NB>
static hipError_t launch_stream_kernel(int device, dim3 grid, hipStream_t st, const uint4* A, const uint16_t* meta16, const uint4* Xf, uint16_t* Y,
                                       float* partial, long long M, long long N, long long Mp, long long Np, long long Kp,
                                       long long span) {
  constexpr size_t smem = (size_t)NB * MT * 128 * 16;
  static std::atomic<unsigned long long> raised{0};
  if (smem > 64 * 1024) {
    hipError_t e = raise_dynamic_lds(raised, device, &k_mm_stream<DT, SPARSE, MT, RT, NW, NB>, smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k_mm_stream<DT, SPARSE, MT, RT, NW, NB>), grid, dim3(NW * 64), smem, st, A, meta16, Xf, Y, partial, M, N, Mp, Np,
                     Kp, span);
  return hipGetLastError();
}

// span of the stream kernels: steps per workgroup when `slots` workgroups share nrb row blocks of nks steps.
// An even number of steps (a step's index half is addressed by its parity within a pair, and its ring slot has
// that parity), at least 8, and long enough that a row block has at most MAX_SPLIT pieces.
static long long stream_span(long long nrb, long long nks, long long slots) {
  long long span = (nrb * nks + slots - 1) / slots;
  span = std::max<long long>(span, 8);
  span = std::max<long long>(span, (nks + MAX_SPLIT - 3) / (MAX_SPLIT - 2));  // pieces <= (nks - 1) / span + 2
  span = (span + 1) / 2 * 2;
  // a span that divides the steps of a row block keeps every span inside one row block (one segment and one partial
  // tile per workgroup instead of two): worth up to a fifth fewer workgroups
  for (long long a = span; a <= nks && a * 5 <= span * 6; a += 2)
    if (nks % a == 0) return a;
  return span;
}

template <int DT, int SPARSE>
static int launch_stream(esparse_ctx* ctx, const Variant& v, hipStream_t st, const uint4* A, const uint16_t* meta16, const uint4* Xf,
                         uint16_t* Y, float* partial, long long M, long long N, long long Mp, long long Np, long long Kp) {
  const long long nrt = Np / 16, nks = Kp / 64;
  const long long rows = (long long)v.nw * v.rt;  // row tiles per workgroup
  const long long nrb = (nrt + rows - 1) / rows;
  const int mt = Mp <= 16 ? 1 : (Mp <= 32 ? 2 : (Mp <= 64 ? 4 : 8));
  // one workgroup per CU: measured faster than two with half the span each
  const long long span = stream_span(nrb, nks, 256);
  dim3 grid((unsigned)((nrb * nks + span - 1) / span));
  hipError_t e = hipErrorInvalidValue;
#define ESP_STREAM(RTv, NWv, NBv)                                                                                           \
  if (v.rt == RTv && v.nw == NWv && v.tt == NBv)                                                                            \
  e = (mt == 1)   ? launch_stream_kernel<DT, SPARSE, 1, RTv, NWv, NBv>(ctx->device, grid, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, span) \
      : (mt == 2) ? launch_stream_kernel<DT, SPARSE, 2, RTv, NWv, NBv>(ctx->device, grid, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, span) \
      : (mt == 4) ? launch_stream_kernel<DT, SPARSE, 4, RTv, NWv, NBv>(ctx->device, grid, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, span) \
                  : launch_stream_kernel<DT, SPARSE, 8, RTv, NWv, NBv>(ctx->device, grid, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp, span)
  ESP_STREAM(1, 8, 4);
  ESP_STREAM(2, 8, 4);
  ESP_STREAM(1, 9, 4);
  ESP_STREAM(1, 11, 4);
  if constexpr (SPARSE != 2) {  // 4:8: the rings of four slots only
    ESP_STREAM(1, 8, 8);
    ESP_STREAM(2, 8, 6);
  }
#undef ESP_STREAM
  ESP_HIP(ctx, e);
  if (span % nks != 0) {  // some row block is cut
    const long long e4 = M * (Np / 4);
    if (DT == ESPARSE_F16)
      hipLaunchKernelGGL(k_reduce_pieces<ESPARSE_F16>, dim3((unsigned)((e4 + 255) / 256)), dim3(256), 0, st, partial, M, N, Mp, Np, Y, nks,
                         span, rows * 16);
    else
      hipLaunchKernelGGL(k_reduce_pieces<ESPARSE_BF16>, dim3((unsigned)((e4 + 255) / 256)), dim3(256), 0, st, partial, M, N, Mp, Np, Y, nks,
                         span, rows * 16);
    ESP_HIP(ctx, hipGetLastError());
  }
  return ESPARSE_OK;
}

// rows of X per workgroup of k_gather_rows (a power of two <= 16; 0 = a row does not fit the LDS)
static int gather_rows_tok(long long Mp, long long K) {
  const long long row = (K + 8) * 2, all = 160 * 1024;  // the kernel has no other LDS
  if (row > all) return 0;
  // two workgroups per CU (one loads while the other gathers) if that still leaves two tokens per workgroup,
  // else whatever fits one workgroup
  int tok = 16;
  while (tok > 2 && tok * row > all / 2) tok >>= 1;
  if (tok * row > all / 2) {
    tok = 16;
    while (tok > 1 && tok * row > all) tok >>= 1;
  }
  // fewer tokens where that fills the chip better, but single tokens (16-byte pieces of every line of X') only for
  // short inputs
  const int floor_tok = Mp >= 512 ? 2 : 1;
  while (tok > floor_tok && Mp / tok < 512) tok >>= 1;
  return tok;
}

template <int TOK>
static hipError_t launch_gather_rows(int device, hipStream_t st, const uint16_t* X, const int32_t* perm, long long M, long long K,
                                     long long Mp, long long Kp, uint4* Xf) {
  const size_t smem = (size_t)TOK * (K + 8) * 2;
  static std::atomic<unsigned long long> raised{0};
  hipError_t e = raise_dynamic_lds(raised, device, &k_gather_rows<TOK>, 160 * 1024);
  if (e != hipSuccess) return e;
  const long long ntiles = Mp / 16, per = 16 / TOK;
  hipLaunchKernelGGL(k_gather_rows<TOK>, dim3((unsigned)((ntiles + 7) / 8 * 8 * per)), dim3(512), smem, st, X, perm, M, Mp, K, Kp, Xf);
  return hipGetLastError();
}

static int stage_activations(esparse_ctx* ctx, const void* X, const int32_t* perm, long long M, long long K, long long Mp,
                             long long Kp, uint4* Xf, int mc) {
  const uint16_t* Xh = reinterpret_cast<const uint16_t*>(X);
  const int tok = (M >= 64 && K % 8 == 0) ? gather_rows_tok(Mp, K) : 0;
  if (tok) {
    hipStream_t st = ctx->stream;
    switch (tok) {
      case 16: ESP_HIP(ctx, launch_gather_rows<16>(ctx->device, st, Xh, perm, M, K, Mp, Kp, Xf)); break;
      case 8: ESP_HIP(ctx, launch_gather_rows<8>(ctx->device, st, Xh, perm, M, K, Mp, Kp, Xf)); break;
      case 4: ESP_HIP(ctx, launch_gather_rows<4>(ctx->device, st, Xh, perm, M, K, Mp, Kp, Xf)); break;
      case 2: ESP_HIP(ctx, launch_gather_rows<2>(ctx->device, st, Xh, perm, M, K, Mp, Kp, Xf)); break;
      default: ESP_HIP(ctx, launch_gather_rows<1>(ctx->device, st, Xh, perm, M, K, Mp, Kp, Xf)); break;
    }
    return ESPARSE_OK;
  }
  const long long units = Mp * Kp / 8, all = units + (long long)mc * (Kp / 8);
  GatherArgs ga = {};
  ga.X[0] = Xh;
  ga.perm[0] = perm;
  ga.Xf[0] = Xf;
  hipLaunchKernelGGL(k_gather_x, dim3((unsigned)((all + 255) / 256), 1), dim3(256), 0, ctx->stream, ga, M, K, Kp, units, mc);
  ESP_HIP(ctx, hipGetLastError());
  return ESPARSE_OK;
}

// the decode kernels on `count` products of one shape: members share M, N, K; ka holds their operands
static int launch_ksplit_any(esparse_ctx* ctx, const Variant& v, int sparse, int dtype, KsplitArgs ka, int count, long long M,
                             long long N, long long Np, long long Kp, bool fold = false) {
  const int mc = compact_tokens(M);
  // variants with K split over workgroups (tt = splits): single products of at most 64 tokens with room for the partial tiles
  const int nsplit = (v.split_mode == 1 && count == 1 && M <= 64 && ka.partial) ? v.tt : 1;
  hipStream_t st = ctx->stream;
  const long long nks = Kp / 64;
  for (long long t0 = 0; t0 < M; t0 += 64) {  // more than 64 tokens (4:8 only): 64 at a time
    const long long mcur = (M - t0) < 64 ? (M - t0) : 64, mcp = esp_round_up(mcur, 16);
    KsplitArgs kc = ka;
    for (int i = 0; i < count; i++) {
      kc.Xf[i] = ka.Xf[i] + (t0 / 16) * (2 * nks) * 64;
      kc.Y[i] = ka.Y[i] + t0 * N;
    }
#define ESP_KSPLIT(DTv, SPv)                                                          \
  do {                                                                                \
    if (mcp == 16) launch_ksplit<DTv, SPv, 1>(v, st, kc, count, mcur, N, mcp, Np, Kp, mc, nsplit, fold);  \
    else if (mcp == 32) launch_ksplit<DTv, SPv, 2>(v, st, kc, count, mcur, N, mcp, Np, Kp, 0, nsplit, false); \
    else launch_ksplit<DTv, SPv, 4>(v, st, kc, count, mcur, N, mcp, Np, Kp, 0, nsplit, false);            \
  } while (0)
    if (dtype == ESPARSE_F16) {
      if (sparse == 2) ESP_KSPLIT(ESPARSE_F16, 2);
      else if (sparse) ESP_KSPLIT(ESPARSE_F16, 1);
      else ESP_KSPLIT(ESPARSE_F16, 0);
    } else {
      if (sparse == 2) ESP_KSPLIT(ESPARSE_BF16, 2);
      else if (sparse) ESP_KSPLIT(ESPARSE_BF16, 1);
      else ESP_KSPLIT(ESPARSE_BF16, 0);
    }
#undef ESP_KSPLIT
    ESP_HIP(ctx, hipGetLastError());
  }
  return ESPARSE_OK;
}

int esp_matmul_device(esparse_ctx* ctx, int sparse, const void* X, long long M, const void* w, const int32_t* perm,
                      long long N, long long K, int dtype, void* Yv, void* workspace, int variant, int phases) {
  hipStream_t st = ctx->stream;
  const long long Mp = esp_round_up(M, 16), Np = esp_round_up(N, 16), Kp = esp_round_up(K, 256);
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  uint4* Xf = reinterpret_cast<uint4*>(ws + WS_HEADER_BYTES);
  float* partial = reinterpret_cast<float*>(ws + WS_HEADER_BYTES + staged_bytes(M, K));
  uint16_t* Y = reinterpret_cast<uint16_t*>(Yv);
  const uint4* A = reinterpret_cast<const uint4*>(w);
  const unsigned char* meta_bytes = sparse ? reinterpret_cast<const unsigned char*>(w) + (size_t)Np * Kp : nullptr;
  const uint2* meta = reinterpret_cast<const uint2*>(meta_bytes);
  const Variant& v = kVariants[variant];
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  int rc;
  // one or two tokens through a decode kernel, both halves in one call: the kernel gathers through theta itself
  const bool fold = phases == (ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY) && ksplit_folds(v, M, Np, Kp);
  if ((phases & ESP_PHASE_STAGE) && !fold && (rc = stage_activations(ctx, X, perm, M, K, Mp, Kp, Xf, compact_tokens(M)))) return rc;
  if (!(phases & ESP_PHASE_MULTIPLY)) return ESPARSE_OK;

  if (v.kind == KIND_KSPLIT) {
    KsplitArgs ka = {};
    ka.A[0] = A;
    ka.meta16[0] = reinterpret_cast<const uint16_t*>(meta_bytes);
    ka.Xf[0] = Xf;
    ka.Y[0] = Y;
    ka.partial = partial;
    ka.X[0] = reinterpret_cast<const uint16_t*>(X);
    ka.perm[0] = perm;
    ka.K = K;
    return launch_ksplit_any(ctx, v, sparse, dtype, ka, 1, M, N, Np, Kp, fold);
  }

  if (v.kind == KIND_TILE) {
    const uint16_t* meta16 = reinterpret_cast<const uint16_t*>(meta_bytes);
    if (sparse == 2)
      return dtype == ESPARSE_F16 ? launch_tile<ESPARSE_F16, 2>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp)
                                  : launch_tile<ESPARSE_BF16, 2>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp);
    if (dtype == ESPARSE_F16)
      return sparse ? launch_tile<ESPARSE_F16, 1>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp)
                    : launch_tile<ESPARSE_F16, 0>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp);
    return sparse ? launch_tile<ESPARSE_BF16, 1>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp)
                  : launch_tile<ESPARSE_BF16, 0>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp);
  }

  if (v.kind == KIND_STREAM) {
    const uint16_t* meta16 = reinterpret_cast<const uint16_t*>(meta_bytes);
    if (sparse == 2)
      return dtype == ESPARSE_F16 ? launch_stream<ESPARSE_F16, 2>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp)
                                  : launch_stream<ESPARSE_BF16, 2>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp);
    if (dtype == ESPARSE_F16)
      return sparse ? launch_stream<ESPARSE_F16, 1>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp)
                    : launch_stream<ESPARSE_F16, 0>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp);
    return sparse ? launch_stream<ESPARSE_BF16, 1>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp)
                  : launch_stream<ESPARSE_BF16, 0>(ctx, v, st, A, meta16, Xf, Y, partial, M, N, Mp, Np, Kp);

  }

  // ---- wave-tile kinds
  const long long nrb = (nrt + v.rt - 1) / v.rt, ntb = (ntt + v.tt - 1) / v.tt;
  int nsplit = 1;
  if (v.split_mode == 1) {
    // enough waves for ~8 per CU (256 CUs), splits of at least 4 steps (256 channels)
    long long want = (256 * 8 + nrb * ntb - 1) / (nrb * ntb);
    long long maxs = nks / 4;
    nsplit = (int)std::max<long long>(1, std::min<long long>(std::min<long long>(want, maxs), esp_split_capacity(M)));
  }
  long long sps = (nks + nsplit - 1) / nsplit;
  sps = (sps + 3) / 4 * 4;
  nsplit = (int)((nks + sps - 1) / sps);
  const long long n_items = nrb * ntb * nsplit;
  dim3 grid((unsigned)((n_items + 3) / 4));
  if (dtype == ESPARSE_F16) {
    if (sparse) launch_wave_tile<ESPARSE_F16, 1>(v, grid, st, A, meta, Xf, Y, partial, M, N, Mp, Np, Kp, nsplit, (int)sps, n_items);
    else launch_wave_tile<ESPARSE_F16, 0>(v, grid, st, A, meta, Xf, Y, partial, M, N, Mp, Np, Kp, nsplit, (int)sps, n_items);
  } else {
    if (sparse) launch_wave_tile<ESPARSE_BF16, 1>(v, grid, st, A, meta, Xf, Y, partial, M, N, Mp, Np, Kp, nsplit, (int)sps, n_items);
    else launch_wave_tile<ESPARSE_BF16, 0>(v, grid, st, A, meta, Xf, Y, partial, M, N, Mp, Np, Kp, nsplit, (int)sps, n_items);
  }
  ESP_HIP(ctx, hipGetLastError());
  if (nsplit > 1) {
    const long long e = M * (Np / 4);
    if (dtype == ESPARSE_F16)
      hipLaunchKernelGGL(k_reduce_splits<ESPARSE_F16>, dim3((unsigned)((e + 255) / 256)), dim3(256), 0, st, partial, nsplit, M, N, Mp, Np, Y);
    else
      hipLaunchKernelGGL(k_reduce_splits<ESPARSE_BF16>, dim3((unsigned)((e + 255) / 256)), dim3(256), 0, st, partial, nsplit, M, N, Mp, Np, Y);
    ESP_HIP(ctx, hipGetLastError());
  }
  return ESPARSE_OK;
}

// ------------------------------------------------------------------------------------------------
// several products of one shape
// ------------------------------------------------------------------------------------------------
size_t esp_group_workspace_bytes(int count, long long M, long long N, long long K) {
  return std::max(esp_workspace_bytes(M, N, K), (size_t)WS_HEADER_BYTES + (size_t)count * staged_bytes(M, K));
}

int esp_matmul_group_device(esparse_ctx* ctx, int sparse, int count, const void* const* X, long long M, const void* const* w,
                            const int32_t* const* perm, long long N, long long K, int dtype, void* const* Y, void* workspace,
                            int variant, int phases) {
  const Variant& v = kVariants[variant];
  if (v.kind != KIND_KSPLIT || v.split_mode == 1) {
    // no grouped form of the other kernels (nor of the decode kernels with K split over workgroups, whose partial
    // tiles live in the workspace of one product): one product after the other through the same workspace
    // (callers that split the phases get EUNSUPPORTED before they reach this point)
    for (int i = 0; i < count; i++) {
      int rc = esp_matmul_device(ctx, sparse, X[i], M, w[i], perm ? perm[i] : nullptr, N, K, dtype, Y[i], workspace, variant,
                                 ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY);
      if (rc) return rc;
    }
    return ESPARSE_OK;
  }
  const long long Mp = esp_round_up(M, 16), Np = esp_round_up(N, 16), Kp = esp_round_up(K, 256);
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  const size_t xbytes = staged_bytes(M, K);
  GatherArgs ga = {};
  KsplitArgs ka = {};
  const bool fold = phases == (ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY) && ksplit_folds(v, M, Np, Kp);
  ka.K = K;
  for (int i = 0; i < count; i++) {
    uint4* Xf = reinterpret_cast<uint4*>(ws + WS_HEADER_BYTES + (size_t)i * xbytes);
    if (fold) {
      ka.X[i] = reinterpret_cast<const uint16_t*>(X[i]);
      ka.perm[i] = perm ? perm[i] : nullptr;
    }
    if (phases & ESP_PHASE_STAGE) {
      ga.X[i] = reinterpret_cast<const uint16_t*>(X[i]);
      ga.perm[i] = perm ? perm[i] : nullptr;
      ga.Xf[i] = Xf;
    }
    if (phases & ESP_PHASE_MULTIPLY) {
      ka.A[i] = reinterpret_cast<const uint4*>(w[i]);
      ka.meta16[i] = sparse ? reinterpret_cast<const uint16_t*>(reinterpret_cast<const unsigned char*>(w[i]) + (size_t)Np * Kp) : nullptr;
      ka.Xf[i] = Xf;
      ka.Y[i] = reinterpret_cast<uint16_t*>(Y[i]);
    }
  }
  if ((phases & ESP_PHASE_STAGE) && !fold) {
    const int mc = compact_tokens(M);
    const long long units = Mp * Kp / 8, all = units + (long long)mc * (Kp / 8);
    hipLaunchKernelGGL(k_gather_x, dim3((unsigned)((all + 255) / 256), (unsigned)count), dim3(256), 0, ctx->stream, ga, M, K, Kp, units,
                       mc);
    ESP_HIP(ctx, hipGetLastError());
  }
  if (!(phases & ESP_PHASE_MULTIPLY)) return ESPARSE_OK;
  return launch_ksplit_any(ctx, v, sparse, dtype, ka, count, M, N, Np, Kp, fold);
}

bool esp_variant_is_decode_kernel(int v) {
  return v >= 0 && v < kNumVariants && kVariants[v].kind == KIND_KSPLIT && kVariants[v].split_mode == 0;
}
