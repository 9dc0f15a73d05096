// Compression of n:m-pruned weights (Section 4, step 1): kept values + 2 bits of index per kept
// value, written both in the canonical row-major form and in the order the sparse-MFMA kernels
// stream (the layout is documented in include/esparse.h).  Pure data movement: HBM-bound.
#include <algorithm>

#include "common.h"

// flags[0] |= 1 : a group does not keep exactly n ; flags[0] |= 2 : perm is not a bijection
__global__ void k_perm_count(const int32_t* __restrict__ perm, long long K, int* __restrict__ count, int* __restrict__ flags) {
  long long p = (long long)blockIdx.x * 256 + threadIdx.x;
  if (p >= K) return;
  int c = perm[p];
  if (c < 0 || c >= K)
    atomicOr(flags, 2);
  else if (atomicAdd(&count[c], 1) != 0)
    atomicOr(flags, 2);
}

// ---- 2:4 ----------------------------------------------------------------------------------------
// One unit = (row, 16 re-ordered channels): 4 groups, 8 kept values, 16 index bits.
// wrow points at the row's weights in ORIGINAL channel order (global memory or an LDS copy).
// Units beyond N or K (padding of the native tiling) are written as zeros.
__device__ __forceinline__ void compress_unit_2_4(const uint16_t* wrow, const uint8_t* __restrict__ mrow /*mask row or null*/,
                                                  const int32_t* __restrict__ perm, bool live, long long row, long long ch,
                                                  long long K, long long Kp, uint16_t* __restrict__ values,
                                                  uint32_t* __restrict__ meta, uint16_t* __restrict__ nvalues,
                                                  uint16_t* __restrict__ nmeta, int* __restrict__ flags) {
  uint16_t kept[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  uint32_t bits = 0;
  int nk = 0;  // kept values in this unit (8 unless the unit is cut by K or is padding)
  const long long p0 = ch * 16;
  if (live && p0 < K) {
    const int ngroups = (int)((K - p0) >= 16 ? 4 : (K - p0) / 4);
    uint32_t mk4[4] = {0, 0, 0, 0};
    if (mrow) {
      if (ngroups == 4 && (K & 15) == 0) {
        const uint4 mv = *reinterpret_cast<const uint4*>(mrow + p0);
        mk4[0] = mv.x; mk4[1] = mv.y; mk4[2] = mv.z; mk4[3] = mv.w;
      } else {
        for (int g = 0; g < ngroups; g++) mk4[g] = *reinterpret_cast<const uint32_t*>(mrow + p0 + g * 4);
      }
    }
    bool bad = false;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      if (g >= ngroups) break;
      uint16_t w[4];
      int c4[4];
      if (perm) {
        const int4 pv = *reinterpret_cast<const int4*>(perm + p0 + g * 4);
        c4[0] = pv.x; c4[1] = pv.y; c4[2] = pv.z; c4[3] = pv.w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; i++) c4[i] = (int)(p0 + g * 4 + i);
      }
#pragma unroll
      for (int i = 0; i < 4; i++) w[i] = wrow[c4[i]];
      uint32_t mk;  // one byte per position, non-zero = kept
      if (mrow) {
        mk = mk4[g];
      } else {
        // keep the non-zero weights, topped up with the lowest-position zeros
        mk = 0;
        int nz = 0;
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (w[i] & 0x7fffu) {
            mk |= 1u << (8 * i);
            nz++;
          }
        if (nz > 2) bad = true;
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (nz < 2 && !((mk >> (8 * i)) & 0xffu)) {
            mk |= 1u << (8 * i);
            nz++;
          }
      }
      int cnt = 0;
#pragma unroll
      for (int i = 0; i < 4; i++)
        if ((mk >> (8 * i)) & 0xffu) {
          if (cnt < 2) {
            // nk = 2 g + cnt : compile-time g, so the two slots are selected without dynamic indexing
            if (cnt == 0) kept[2 * g] = w[i];
            else kept[2 * g + 1] = w[i];
            bits |= (uint32_t)i << (2 * (2 * g + cnt));
          }
          cnt++;
        }
      if (cnt != 2) bad = true;  // the call reports EBADMASK; the slot layout stays well-formed
      nk = 2 * g + 2;
    }
    if (bad) atomicOr(flags, 1);
    // canonical: values[row][ch*8 .. ch*8+nk), index half-words
    if (values) {
      uint16_t* dst = values + row * (K / 2) + ch * 8;
      if (nk == 8 && ((K / 2) % 8 == 0)) {
        uint4 v;
        v.x = kept[0] | ((uint32_t)kept[1] << 16);
        v.y = kept[2] | ((uint32_t)kept[3] << 16);
        v.z = kept[4] | ((uint32_t)kept[5] << 16);
        v.w = kept[6] | ((uint32_t)kept[7] << 16);
        *reinterpret_cast<uint4*>(dst) = v;
      } else {
#pragma unroll
        for (int i = 0; i < 8; i++)
          if (i < nk) dst[i] = kept[i];
      }
    }
    if (meta) {
      // uint32 words per row: ceil(K/32); this unit is half-word (ch & 1) of word ch / 2
      uint16_t* m16 = reinterpret_cast<uint16_t*>(meta + row * ((K / 2 + 15) / 16));
      m16[ch] = (uint16_t)bits;
      if (p0 + 16 >= K && (ch & 1) == 0) m16[ch + 1] = 0;  // unused half of the row's last word
    }
  }
  if (nvalues) {
    const long long nchunk = Kp / 16;
    const long long rt = row >> 4, ks = ch >> 2;
    const int r = (int)(row & 15), ga = (int)(ch & 3);
    uint4 v;
    v.x = kept[0] | ((uint32_t)kept[1] << 16);
    v.y = kept[2] | ((uint32_t)kept[3] << 16);
    v.z = kept[4] | ((uint32_t)kept[5] << 16);
    v.w = kept[6] | ((uint32_t)kept[7] << 16);
    reinterpret_cast<uint4*>(nvalues)[((rt * (nchunk / 4) + ks) * 4 + ga) * 16 + r] = v;
    // index unit order [rt][ks/4][ga][r][ks%4]
    nmeta[(((rt * (nchunk / 16) + ks / 4) * 4 + ga) * 16 + r) * 4 + (ks & 3)] = (uint16_t)bits;
  }
}

// Generic form: one thread per unit, weights gathered from global memory (any K).
__global__ void __launch_bounds__(256) k_compress_2_4(const uint16_t* __restrict__ W, const uint8_t* __restrict__ mask,
                                                       const int32_t* __restrict__ perm, long long N, long long K, long long Np,
                                                       long long Kp, uint16_t* __restrict__ values, uint32_t* __restrict__ meta,
                                                       uint16_t* __restrict__ nvalues, uint16_t* __restrict__ nmeta,
                                                       int* __restrict__ flags) {
  const long long nchunk = Kp / 16;
  long long u = (long long)blockIdx.x * 256 + threadIdx.x;
  if (u >= Np * nchunk) return;
  // thread order = native unit order, so the native stores are coalesced
  const int r = (int)(u & 15), ga = (int)((u >> 4) & 3);
  const long long t = u >> 6;
  const long long ks = t % (nchunk / 4), rt = t / (nchunk / 4);
  const long long row = rt * 16 + r, ch = ks * 4 + ga;
  const bool live = row < N;
  compress_unit_2_4(W + (live ? row : 0) * K, mask ? mask + (live ? row : 0) * K : nullptr, perm, live, row, ch, K, Kp, values,
                    meta, nvalues, nmeta, flags);
}

// Fast form: a workgroup copies RB whole rows of W into LDS with coalesced loads and gathers the
// permuted channels from there, so HBM sees W exactly once, in order.  Needs 2*K*RB bytes of LDS.
__global__ void __launch_bounds__(512) k_compress_2_4_rows(const uint16_t* __restrict__ W, const uint8_t* __restrict__ mask,
                                                            const int32_t* __restrict__ perm, long long N, long long K,
                                                            long long Np, long long Kp, int RB, uint16_t* __restrict__ values,
                                                            uint32_t* __restrict__ meta, uint16_t* __restrict__ nvalues,
                                                            uint16_t* __restrict__ nmeta, int* __restrict__ flags) {
  extern __shared__ uint2 s_w2[];  // [RB][K / 4] groups of 4 weights
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * RB;
  const int k4 = (int)(K / 4);
  const uint2* W2 = reinterpret_cast<const uint2*>(W);
  for (int r = 0; r < RB; r++) {
    const long long row = row0 + r;
    if (row >= N) break;
    for (int c = tid; c < k4; c += 512) s_w2[r * k4 + c] = W2[row * k4 + c];
  }
  __syncthreads();
  const uint16_t* s_w = reinterpret_cast<const uint16_t*>(s_w2);
  const int nchunk = (int)(Kp / 16);
  for (int e = tid; e < RB * nchunk; e += 512) {
    const int r = e % RB, ch = e / RB;
    const long long row = row0 + r;
    if (row >= Np) continue;
    const bool live = row < N;
    compress_unit_2_4(s_w + (size_t)r * K, (mask && live) ? mask + row * K : nullptr, perm, live, row, ch, K, Kp, values, meta,
                      nvalues, nmeta, flags);
  }
}

// ---- 4:8 ----------------------------------------------------------------------------------------
// One thread per (row, group of 8) of the padded matrix: 4 kept values + one bitmap byte.
// Native form (what the 4:8 product streams; same size and unit numbering as the 2:4 one): the group
// of row 16 rt + r that covers channels 64 ks + 32 h + 8 g .. + 8 is the A operand of lane 16 g + r of
// the dense 16x16x32 instruction for half-step h of step ks.  Its 4 kept values (8 bytes) sit at byte
// 8 h of the 16-byte unit (rt nks + ks) 64 + lane; its pattern code is byte h of the 16-bit word at the place
// where the 2:4 form keeps that lane's index half for step ks.  The pattern code of a group is the index of its
// bitmap among the 70 bitmaps with four bits set, in ascending order (the product kernels look their byte-permute
// selectors up by it, and 70 entries can be replicated in LDS where 256 cannot).  Padding rows and channels hold
// zero values and code 0.
__device__ __forceinline__ uint32_t pattern_code_4_8(uint32_t bm) {
  // sum over the set positions p_1 < p_2 < ... of C(p_j, j): the bitmaps below bm that first differ from it at p_j
  uint32_t code = 0;
  int j = 0;
#pragma unroll
  for (int e = 0; e < 8; e++)
    if ((bm >> e) & 1u) {
      j++;
      int c = 1;
      for (int t = 0; t < j; t++) c = c * (e - t) / (t + 1);
      code += (uint32_t)c;
    }
  return code;
}

__global__ void __launch_bounds__(256) k_compress_4_8(const uint16_t* __restrict__ W, const uint8_t* __restrict__ mask,
                                                       const int32_t* __restrict__ perm, long long N, long long K, long long Np,
                                                       long long Kp, uint16_t* __restrict__ values, uint8_t* __restrict__ meta,
                                                       unsigned char* __restrict__ nvalues, uint8_t* __restrict__ nmeta,
                                                       int* __restrict__ flags) {
  const long long ng = K / 8, ngp = Kp / 8;
  long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= Np * ngp) return;
  const long long row = e / ngp, g = e % ngp;
  uint16_t kept[4] = {0, 0, 0, 0};
  uint32_t bm = 0;
  if (row < N && g < ng) {
    uint16_t w[8];
    uint8_t mk[8];
    int nz = 0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      long long p = g * 8 + i;
      long long c = perm ? perm[p] : p;
      w[i] = W[row * K + c];
      mk[i] = mask ? (mask[row * K + p] ? 1 : 0) : ((w[i] & 0x7fffu) ? 1 : 0);
      nz += mk[i];
    }
    if (!mask) {
      if (nz > 4) atomicOr(flags, 1);
#pragma unroll
      for (int i = 0; i < 8; i++)
        if (nz < 4 && !mk[i]) {
          mk[i] = 1;
          nz++;
        }
    }
    if (nz != 4) atomicOr(flags, 1);
    int nk = 0;
#pragma unroll
    for (int i = 0; i < 8; i++)
      if (mk[i] && nk < 4) {
        kept[nk++] = w[i];
        bm |= 1u << i;
      }
    if (values) {
      uint2 v;
      v.x = kept[0] | ((uint32_t)kept[1] << 16);
      v.y = kept[2] | ((uint32_t)kept[3] << 16);
      *reinterpret_cast<uint2*>(values + row * (K / 2) + g * 4) = v;
    }
    if (meta) meta[row * ng + g] = (uint8_t)bm;
  }
  if (nvalues) {
    const long long nks = Kp / 64;
    const long long rt = row >> 4, ks = g >> 3;
    const int r = (int)(row & 15), h = (int)((g >> 2) & 1), gg = (int)(g & 3);
    const int lane = gg * 16 + r;
    uint2 v;
    v.x = kept[0] | ((uint32_t)kept[1] << 16);
    v.y = kept[2] | ((uint32_t)kept[3] << 16);
    *reinterpret_cast<uint2*>(nvalues + ((rt * nks + ks) * 64 + lane) * 16 + 8 * h) = v;
    nmeta[(((rt * (nks / 4) + ks / 4) * 64 + lane) * 4 + (ks & 3)) * 2 + h] = (uint8_t)pattern_code_4_8(bm);
  }
}

int esp_compress_device(esparse_ctx* ctx, const void* Wv, const uint8_t* mask, const int32_t* perm, long long N,
                        long long K, int dtype, int n, int m, void* values_out, void* meta_out, void* native_out) {
  (void)dtype;  // both dtypes are 16-bit patterns here
  (void)n;
  hipStream_t st = ctx->stream;
  int* flags = ctx->d_flags;
  ESP_HIP(ctx, hipMemsetAsync(flags, 0, sizeof(int), st));
  DevBuf count;
  if (perm) {
    if (count.alloc(K * 4) != hipSuccess) return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation failed");
    ESP_HIP(ctx, hipMemsetAsync(count.p, 0, K * 4, st));
    hipLaunchKernelGGL(k_perm_count, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, perm, K, count.as<int>(), flags);
    ESP_HIP(ctx, hipGetLastError());
    int h = 0;
    ESP_HIP(ctx, hipMemcpyAsync(&h, flags, sizeof(int), hipMemcpyDeviceToHost, st));
    ESP_HIP(ctx, hipStreamSynchronize(st));
    if (h & 2) return esp_fail(ctx, ESPARSE_EBADPERM, "perm is not a bijection on [0, %lld)", K);
  }
  const uint16_t* W = reinterpret_cast<const uint16_t*>(Wv);
  if (m == 4) {
    const long long Np = esp_round_up(N, 16);
    const long long Kp = esp_round_up(K, 256);
    uint16_t* nvalues = reinterpret_cast<uint16_t*>(native_out);
    uint16_t* nmeta = native_out ? reinterpret_cast<uint16_t*>(reinterpret_cast<unsigned char*>(native_out) + (size_t)Np * Kp) : nullptr;
    const long long units = Np * (Kp / 16);
    const size_t row_bytes = (size_t)K * 2;
    const size_t lds_budget = row_bytes <= 64 * 1024 ? 64 * 1024 : 144 * 1024;
    int RB = (int)std::min<size_t>(16, lds_budget / row_bytes);
    if (RB >= 1) {
      const size_t smem = (size_t)RB * row_bytes;
      if (smem > 64 * 1024)
        ESP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_compress_2_4_rows),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
      hipLaunchKernelGGL(k_compress_2_4_rows, dim3((unsigned)((Np + RB - 1) / RB)), dim3(512), smem, st, W, mask, perm, N, K, Np, Kp,
                         RB, reinterpret_cast<uint16_t*>(values_out), reinterpret_cast<uint32_t*>(meta_out), nvalues, nmeta, flags);
    } else {
      hipLaunchKernelGGL(k_compress_2_4, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st, W, mask, perm, N, K, Np, Kp,
                         reinterpret_cast<uint16_t*>(values_out), reinterpret_cast<uint32_t*>(meta_out), nvalues, nmeta, flags);
    }
  } else {
    const long long Np = native_out ? esp_round_up(N, 16) : N;
    const long long Kp = native_out ? esp_round_up(K, 256) : K;
    const long long groups = Np * (Kp / 8);
    unsigned char* nvalues = reinterpret_cast<unsigned char*>(native_out);
    uint8_t* nmeta = native_out ? reinterpret_cast<uint8_t*>(native_out) + (size_t)Np * Kp : nullptr;
    hipLaunchKernelGGL(k_compress_4_8, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, W, mask, perm, N, K, Np, Kp,
                       reinterpret_cast<uint16_t*>(values_out), reinterpret_cast<uint8_t*>(meta_out), nvalues, nmeta, flags);
  }
  ESP_HIP(ctx, hipGetLastError());
  int h = 0;
  ESP_HIP(ctx, hipMemcpyAsync(&h, flags, sizeof(int), hipMemcpyDeviceToHost, st));
  ESP_HIP(ctx, hipStreamSynchronize(st));
  if (h & 1) return esp_fail(ctx, ESPARSE_EBADMASK, "a group of %d does not keep exactly %d weights", m, n);
  return ESPARSE_OK;
}

// ---- dense re-tiling (the dense GEMM streams W the same way the sparse one streams its values) ----
// unit = (row, 8 channels) = 16 bytes; order [row/16][chunk/4][chunk%4][row%16]; zero padded.
__global__ void __launch_bounds__(256) k_dense_pack(const uint16_t* __restrict__ W, long long N, long long K, long long Np,
                                                     long long Kp, uint4* __restrict__ out) {
  const long long nchunk = Kp / 8;
  long long u = (long long)blockIdx.x * 256 + threadIdx.x;
  if (u >= Np * nchunk) return;
  const int r = (int)(u & 15), g = (int)((u >> 4) & 3);
  const long long t = u >> 6;
  const long long ks = t % (nchunk / 4), rt = t / (nchunk / 4);
  const long long row = rt * 16 + r, k0 = (ks * 4 + g) * 8;
  uint16_t v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < N)
    for (int e = 0; e < 8; e++)
      if (k0 + e < K) v[e] = W[row * K + k0 + e];
  uint4 o;
  o.x = v[0] | ((uint32_t)v[1] << 16);
  o.y = v[2] | ((uint32_t)v[3] << 16);
  o.z = v[4] | ((uint32_t)v[5] << 16);
  o.w = v[6] | ((uint32_t)v[7] << 16);
  out[u] = o;
}

int esp_dense_pack_device(esparse_ctx* ctx, const void* W, long long N, long long K, int dtype, void* packed) {
  (void)dtype;
  const long long Np = esp_round_up(N, 16), Kp = esp_round_up(K, 256);
  const long long units = Np * (Kp / 8);
  hipLaunchKernelGGL(k_dense_pack, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, ctx->stream,
                     reinterpret_cast<const uint16_t*>(W), N, K, Np, Kp, reinterpret_cast<uint4*>(packed));
  ESP_HIP(ctx, hipGetLastError());
  return ESPARSE_OK;
}
