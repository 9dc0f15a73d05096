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

#include "common.h"

#define WS_HEADER_BYTES 65536
#define MAX_SPLIT 16

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
__device__ __forceinline__ void sched_fence() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_sched_barrier(0);
#endif
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
__global__ void __launch_bounds__(256) k_gather_x(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm, long long M,
                                                   long long K, long long Kp, long long units, uint4* __restrict__ Xf) {
  long long u = (long long)blockIdx.x * 256 + threadIdx.x;
  if (u >= units) return;
  const int lane = (int)(u & 63);
  const long long ns = Kp / 32;
  const long long s = (u >> 6) % ns, tt = (u >> 6) / ns;
  const long long t = tt * 16 + (lane & 15);
  const long long k0 = s * 32 + (lane >> 4) * 8;
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
template <int DT, int SPARSE, int MT, int RT, int NW>
__global__ void __launch_bounds__(NW * 64) k_mm_ksplit(const uint4* __restrict__ A, const uint16_t* __restrict__ meta16,
                                                        const uint4* __restrict__ Xf, uint16_t* __restrict__ Y, long long M,
                                                        long long N, long long Mp, long long Np, long long Kp) {
  extern __shared__ floatx4_t s_red[];  // [NW][RT * MT][64]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

  // two steps per trip (all loads of both steps are issued before the first multiply)
  for (long long ks = wave; ks < nks; ks += 2 * NW) {
    const bool second = ks + NW < nks;  // wave-uniform
    const long long kk[2] = {ks, second ? ks + NW : ks};
    uint4 a[2][RT], a2[2][RT], b0[2][MT], b1[2][MT];
    int idx[2][RT];
#pragma unroll
    for (int u = 0; u < 2; u++) {
#pragma unroll
      for (int i = 0; i < RT; i++) {
        if (SPARSE) {
          a[u][i] = A[(rts[i] * nks + kk[u]) * 64 + lane];
          idx[u][i] = (int)meta16[((rts[i] * (nks / 4) + kk[u] / 4) * 64 + lane) * 4 + (kk[u] & 3)];
        } else {
          a[u][i] = A[(rts[i] * (2 * nks) + 2 * kk[u]) * 64 + lane];
          a2[u][i] = A[(rts[i] * (2 * nks) + 2 * kk[u] + 1) * 64 + lane];
        }
      }
#pragma unroll
      for (int j = 0; j < MT; j++) {
        const long long tt = (j < ntt) ? j : ntt - 1;
        b0[u][j] = Xf[(tt * (2 * nks) + 2 * kk[u]) * 64 + lane];
        b1[u][j] = Xf[(tt * (2 * nks) + 2 * kk[u] + 1) * 64 + lane];
      }
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
      if (u == 1 && !second) break;
#pragma unroll
      for (int i = 0; i < RT; i++)
#pragma unroll
        for (int j = 0; j < MT; j++) {
          if (SPARSE) {
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
    if (rt0 + i < nrt && j < ntt) store_y4<DT>(Y, M, N, (long long)j * 16 + c, (rt0 + i) * 16 + g * 4, sum);
  }
}

// ------------------------------------------------------------------------------------------------
// variant "tile" (prefill sizes, MFMA-bound): a workgroup of 4 waves (2 x 2) owns a macro tile of
// 32*TR output rows x 32*TC tokens; each wave owns TR x TC tiles of 16 x 16 (TR = TC = 8: 128 x 128,
// 256 accumulator registers).  Per 64-channel stage the workgroup copies the macro tile's slice of the
// staged activations (2*TC KiB per 16 tokens... 4*TC KiB in all) into LDS, double buffered, one barrier
// per stage; every wave takes its TR compressed weight operands (and their index halves) straight from
// memory into registers one stage ahead, and walks its TC token tiles reading each B operand from
// LDS once for TR multiplies.  Macro tiles are numbered so that the workgroups of one XCD
// (blockIdx % 8) cover neighbouring tiles and share weight rows in that XCD's L2.
// ------------------------------------------------------------------------------------------------
template <int DT, int SPARSE, int TR, int TC>
__global__ void __launch_bounds__(256) k_mm_tile(const uint4* __restrict__ A, const uint16_t* __restrict__ meta16,
                                                  const uint4* __restrict__ Xf, uint16_t* __restrict__ Y, long long M,
                                                  long long N, long long Mp, long long Np, long long Kp, long long n_tiles,
                                                  long long ntb) {
  extern __shared__ uint4 s_b[];  // [2 buffers][2 * TC token tiles][2 half steps][64 lanes]
  constexpr int NTT = 2 * TC;     // token tiles of 16 in the macro tile
  constexpr int STAGE_UNITS = NTT * 128;
  constexpr int COPIES = STAGE_UNITS / 256;  // 16-byte units per thread per stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = wave_uniform(tid >> 6);  // wave-uniform: keeps the operand bases in SGPRs
  const int wr = wave >> 1, wc = wave & 1;
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  // XCD-aware numbering: XCD x (= blockIdx % 8) works through tiles [x * per, (x + 1) * per)
  const long long per = (n_tiles + 7) / 8;
  const long long tile = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((long long)(blockIdx.x >> 3) >= per || tile >= n_tiles) return;
  const long long rb = tile / ntb, tb = tile % ntb;
  const long long rt_base = rb * (2 * TR) + wr * TR;  // first row tile of this wave
  const long long tt_base = tb * NTT;                 // first token tile of the macro tile

  // wave-uniform operand bases; per-lane offsets are 32-bit
  const uint4* a_ptr[TR];
  const uint16_t* m_ptr[TR];
#pragma unroll
  for (int i = 0; i < TR; i++) {
    const long long rt = (rt_base + i < nrt) ? rt_base + i : nrt - 1;
    a_ptr[i] = A + (SPARSE ? rt * nks : rt * (2 * nks)) * 64;
    m_ptr[i] = meta16 + rt * (nks / 4) * 256;
  }
  const uint4* x_ptr[COPIES];
#pragma unroll
  for (int p = 0; p < COPIES; p++) {
    const long long ttl = 2 * p + (wave >> 1);  // token tile (within the macro tile) of this wave's p-th copy
    const long long tt = (tt_base + ttl < ntt) ? tt_base + ttl : ntt - 1;
    x_ptr[p] = Xf + tt * (2 * nks) * 64;
  }
  const unsigned x_lane = (unsigned)(tid & 127);
  const unsigned nks32 = (unsigned)nks;

  floatx4_t acc[TR][TC];
#pragma unroll
  for (int i = 0; i < TR; i++)
#pragma unroll
    for (int j = 0; j < TC; j++) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  uint4 a[2][TR], a2[2][TR];
  int idx[2][TR];

  // prologue: stage 0.  The activations go from global memory straight into LDS (16 bytes per lane,
  // lane l of a wave lands at the wave's LDS base + 16 l), so they never occupy registers.
#pragma unroll
  for (int p = 0; p < COPIES; p++)
    global_to_lds_16(x_ptr[p] + x_lane, s_b + 256 * p + wave * 64);
#pragma unroll
  for (int i = 0; i < TR; i++) {
    if (SPARSE) {
      a[0][i] = a_ptr[i][lane];
      idx[0][i] = (int)m_ptr[i][lane * 4];
    } else {
      a[0][i] = a_ptr[i][lane];
      a2[0][i] = a_ptr[i][lane + 64];
    }
  }
  __syncthreads();

  for (unsigned ks = 0; ks < nks32; ks += 2) {
#pragma unroll
    for (int par = 0; par < 2; par++) {
      const unsigned k = ks + par;
      // loads of the next stage (the last stage reloads itself: no branch, the copy is never used)
      const unsigned kn = (k + 1 < nks32) ? k + 1 : k;
#pragma unroll
      for (int p = 0; p < COPIES; p++)
        global_to_lds_16(x_ptr[p] + (kn * 128u + x_lane), s_b + (par ^ 1) * STAGE_UNITS + 256 * p + wave * 64);
#pragma unroll
      for (int i = 0; i < TR; i++) {
        if (SPARSE) {
          a[par ^ 1][i] = a_ptr[i][kn * 64u + lane];
          idx[par ^ 1][i] = (int)m_ptr[i][(kn >> 2) * 256u + lane * 4u + (kn & 3u)];
        } else {
          a[par ^ 1][i] = a_ptr[i][kn * 128u + lane];
          a2[par ^ 1][i] = a_ptr[i][kn * 128u + 64u + lane];
        }
      }
      sched_fence();  // keep the next stage's loads ahead of this stage's multiplies
      // multiply stage k out of LDS buffer `par`
      const uint4* sb = s_b + par * STAGE_UNITS + (wc * TC) * 128 + lane;
#pragma unroll
      for (int j = 0; j < TC; j++) {
        const uint4 b0 = sb[j * 128];
        const uint4 b1 = sb[j * 128 + 64];
#pragma unroll
        for (int i = 0; i < TR; i++) {
          if (SPARSE) {
            acc[i][j] = smfmac16<DT, 0>(a[par][i], b0, b1, acc[i][j], idx[par][i]);
          } else {
            acc[i][j] = mfma16<DT>(a[par][i], b0, acc[i][j]);
            acc[i][j] = mfma16<DT>(a2[par][i], b1, acc[i][j]);
          }
        }
      }
      __syncthreads();
    }
  }

  const int c = lane & 15, g = lane >> 4;
#pragma unroll
  for (int i = 0; i < TR; i++) {
    const long long rt = rt_base + i;
    if (rt >= nrt) continue;
#pragma unroll
    for (int j = 0; j < TC; j++) {
      const long long tt = tt_base + wc * TC + j;
      if (tt >= ntt) continue;
      store_y4<DT>(Y, M, N, tt * 16 + c, rt * 16 + g * 4, acc[i][j]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// variant table and host launcher
// ------------------------------------------------------------------------------------------------
enum { KIND_WAVE = 0, KIND_KSPLIT = 1, KIND_TILE = 2 };
struct Variant {
  const char* name;
  int kind;
  int rt, tt;      // row tiles / token tiles per wave (ksplit: row tiles per workgroup, tt unused: MT follows M)
  int split_mode;  // wave kind: 0 = never split K, 1 = split K over workgroups to fill the chip
  int nw;          // ksplit kind: waves per workgroup
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
    {"tile_256x256", KIND_TILE, 8, 8, 0, 0},
    {"tile_256x128", KIND_TILE, 8, 4, 0, 0},
    {"tile_128x128", KIND_TILE, 4, 4, 0, 0},
};
static const int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

int esp_num_variants() { return kNumVariants; }
const char* esp_variant_name(int v) { return kVariants[v].name; }

bool esp_variant_applicable(int v, long long M, long long N, long long K, int sparse) {
  (void)N;
  (void)K;
  (void)sparse;
  if (v < 0 || v >= kNumVariants) return false;
  const Variant& var = kVariants[v];
  if (var.kind == KIND_WAVE && var.split_mode == 1 && M > 128) return false;  // partial buffers are sized for decode only
  if (var.kind == KIND_KSPLIT && M > 32) return false;
  if (var.kind == KIND_TILE && M < 64) return false;
  return true;
}

int esp_default_variant(long long M, long long N, long long K, int sparse) {
  (void)K;
  (void)sparse;
  if (M <= 32) {
    const long long nrt = esp_round_up(N, 16) / 16;
    return nrt <= 320 ? 4 : 5;  // ksplit_w16_r1 / ksplit_w16_r2
  }
  if (M <= 128) return 1;  // wave_r2_t2_splitk
  return 12;               // tile_128x128
}

size_t esp_workspace_bytes(long long M, long long N, long long K) {
  const size_t Mp = (size_t)esp_round_up(M, 16), Np = (size_t)esp_round_up(N, 16), Kp = (size_t)esp_round_up(K, 256);
  size_t bytes = WS_HEADER_BYTES + Mp * Kp * 2;
  bytes = (bytes + 255) / 256 * 256;
  if (M <= 128) bytes += (size_t)MAX_SPLIT * Mp * Np * 4;
  return bytes;
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

template <int DT, int SPARSE, int MT>
static void launch_ksplit(const Variant& v, hipStream_t st, const uint4* A, const uint16_t* meta16, const uint4* Xf, uint16_t* Y,
                          long long M, long long N, long long Mp, long long Np, long long Kp) {
  const long long nrt = Np / 16;
  dim3 grid((unsigned)((nrt + v.rt - 1) / v.rt));
  const size_t smem = (size_t)v.nw * v.rt * MT * 64 * 16;
#define LAUNCH(R, W) \
  hipLaunchKernelGGL((k_mm_ksplit<DT, SPARSE, MT, R, W>), grid, dim3(W * 64), smem, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp)
  if (v.nw == 16 && v.rt == 1) LAUNCH(1, 16);
  else if (v.nw == 16 && v.rt == 2) LAUNCH(2, 16);
  else if (v.nw == 16 && v.rt == 3) LAUNCH(3, 16);
  else if (v.nw == 8 && v.rt == 1) LAUNCH(1, 8);
  else if (v.nw == 8 && v.rt == 2) LAUNCH(2, 8);
  else LAUNCH(4, 8);
#undef LAUNCH
}

template <int DT, int SPARSE>
static int launch_tile(esparse_ctx* ctx, const Variant& v, hipStream_t st, const uint4* A, const uint16_t* meta16, const uint4* Xf,
                       uint16_t* Y, long long M, long long N, long long Mp, long long Np, long long Kp) {
  const long long nrt = Np / 16, ntt = Mp / 16;
  const long long nrb = (nrt + 2 * v.rt - 1) / (2 * v.rt), ntb = (ntt + 2 * v.tt - 1) / (2 * v.tt);
  const long long n_tiles = nrb * ntb;
  const long long per = (n_tiles + 7) / 8;
  dim3 grid((unsigned)(per * 8));
  const size_t smem = (size_t)2 * (2 * v.tt) * 128 * 16;
#define LAUNCH(R, T)                                                                                                   \
  do {                                                                                                                 \
    if (smem > 48 * 1024)                                                                                              \
      ESP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_mm_tile<DT, SPARSE, R, T>),                    \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));                        \
    hipLaunchKernelGGL((k_mm_tile<DT, SPARSE, R, T>), grid, dim3(256), smem, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp, n_tiles, ntb); \
  } while (0)
  if (v.rt == 8 && v.tt == 8) LAUNCH(8, 8);
  else if (v.rt == 8 && v.tt == 4) LAUNCH(8, 4);
  else LAUNCH(4, 4);
#undef LAUNCH
  ESP_HIP(ctx, hipGetLastError());
  return ESPARSE_OK;
}

static int stage_activations(esparse_ctx* ctx, const void* X, const int32_t* perm, long long M, long long K, long long Mp,
                             long long Kp, uint4* Xf) {
  const long long units = Mp * Kp / 8;
  hipLaunchKernelGGL(k_gather_x, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, ctx->stream,
                     reinterpret_cast<const uint16_t*>(X), perm, M, K, Kp, units, Xf);
  ESP_HIP(ctx, hipGetLastError());
  return ESPARSE_OK;
}

int esp_matmul_device(esparse_ctx* ctx, int sparse, const void* X, long long M, const void* w, const int32_t* perm,
                      long long N, long long K, int dtype, void* Yv, void* workspace, int variant, int phases) {
  hipStream_t st = ctx->stream;
  const long long Mp = esp_round_up(M, 16), Np = esp_round_up(N, 16), Kp = esp_round_up(K, 256);
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  uint4* Xf = reinterpret_cast<uint4*>(ws + WS_HEADER_BYTES);
  size_t xbytes = ((size_t)Mp * Kp * 2 + 255) / 256 * 256;
  float* partial = reinterpret_cast<float*>(ws + WS_HEADER_BYTES + xbytes);
  uint16_t* Y = reinterpret_cast<uint16_t*>(Yv);
  const uint4* A = reinterpret_cast<const uint4*>(w);
  const unsigned char* meta_bytes = sparse ? reinterpret_cast<const unsigned char*>(w) + (size_t)Np * Kp : nullptr;
  const uint2* meta = reinterpret_cast<const uint2*>(meta_bytes);
  const Variant& v = kVariants[variant];
  const long long nrt = Np / 16, ntt = Mp / 16, nks = Kp / 64;
  int rc;
  if ((phases & ESP_PHASE_STAGE) && (rc = stage_activations(ctx, X, perm, M, K, Mp, Kp, Xf))) return rc;
  if (!(phases & ESP_PHASE_MULTIPLY)) return ESPARSE_OK;

  if (v.kind == KIND_KSPLIT) {
    const uint16_t* meta16 = reinterpret_cast<const uint16_t*>(meta_bytes);
    if (dtype == ESPARSE_F16) {
      if (sparse && ntt == 1) launch_ksplit<ESPARSE_F16, 1, 1>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
      else if (sparse) launch_ksplit<ESPARSE_F16, 1, 2>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
      else if (ntt == 1) launch_ksplit<ESPARSE_F16, 0, 1>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
      else launch_ksplit<ESPARSE_F16, 0, 2>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
    } else {
      if (sparse && ntt == 1) launch_ksplit<ESPARSE_BF16, 1, 1>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
      else if (sparse) launch_ksplit<ESPARSE_BF16, 1, 2>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
      else if (ntt == 1) launch_ksplit<ESPARSE_BF16, 0, 1>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
      else launch_ksplit<ESPARSE_BF16, 0, 2>(v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
    }
    ESP_HIP(ctx, hipGetLastError());
    return ESPARSE_OK;
  }

  if (v.kind == KIND_TILE) {
    const uint16_t* meta16 = reinterpret_cast<const uint16_t*>(meta_bytes);
    if (dtype == ESPARSE_F16)
      return sparse ? launch_tile<ESPARSE_F16, 1>(ctx, v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp)
                    : launch_tile<ESPARSE_F16, 0>(ctx, v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
    return sparse ? launch_tile<ESPARSE_BF16, 1>(ctx, v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp)
                  : launch_tile<ESPARSE_BF16, 0>(ctx, v, st, A, meta16, Xf, Y, M, N, Mp, Np, Kp);
  }

  // ---- wave-tile kinds
  const long long nrb = (nrt + v.rt - 1) / v.rt, ntb = (ntt + v.tt - 1) / v.tt;
  int nsplit = 1;
  if (v.split_mode == 1) {
    // enough waves for ~8 per CU (256 CUs), splits of at least 4 steps (256 channels)
    long long want = (256 * 8 + nrb * ntb - 1) / (nrb * ntb);
    long long maxs = nks / 4;
    nsplit = (int)std::max<long long>(1, std::min<long long>(std::min<long long>(want, maxs), MAX_SPLIT));
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
