// Internal declarations shared by the translation units of libesparse (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <map>
#include <tuple>
#include <vector>

#include "../../include/esparse.h"

struct esparse_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  std::string err;
  // (sparse, dtype, M, N, K) -> variant chosen by esparse_tune
  std::map<std::tuple<int, int, int, long long, long long, long long>, int> tuned;  // (products per launch, mode, dtype, M, N, K) -> variant
  int* d_flags = nullptr;     // 64 ints of device scratch for error flags
};

int esp_fail(esparse_ctx* ctx, int code, const char* fmt, ...);

#define ESP_HIP(ctx, call)                                                                    \
  do {                                                                                        \
    hipError_t e__ = (call);                                                                  \
    if (e__ != hipSuccess)                                                                    \
      return esp_fail((ctx), ESPARSE_EHIP, "%s failed: %s (%s:%d)", #call,                    \
                      hipGetErrorString(e__), __FILE__, __LINE__);                            \
  } while (0)

#define ESP_REQUIRE(ctx, cond, code, ...)                                                     \
  do {                                                                                        \
    if (!(cond)) return esp_fail((ctx), (code), __VA_ARGS__);                                 \
  } while (0)

static inline bool esp_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline long long esp_round_up(long long v, long long q) { return (v + q - 1) / q * q; }

// device scratch that frees itself (offline stages only)
struct DevBuf {
  void* p = nullptr;
  ~DevBuf() {
    if (p) (void)hipFree(p);
  }
  hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1); }
  template <class T>
  T* as() const { return reinterpret_cast<T*>(p); }
};

// ---- 16-bit element helpers on the device ----------------------------------------------------
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16_t __attribute__((ext_vector_type(16)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

// raw 16 bits -> float (exact) for either dtype
template <int DT>
__device__ __forceinline__ float esp_to_float(uint16_t raw) {
  if (DT == ESPARSE_F16) {
    _Float16 h;
    __builtin_memcpy(&h, &raw, 2);
    return (float)h;
  } else {
    uint32_t u = ((uint32_t)raw) << 16;
    float f;
    __builtin_memcpy(&f, &u, 4);
    return f;
  }
}

// float -> 16 bits, round to nearest even
template <int DT>
__device__ __forceinline__ uint16_t esp_from_float(float f) {
  uint16_t raw;
  if (DT == ESPARSE_F16) {
    _Float16 h = (_Float16)f;
    __builtin_memcpy(&raw, &h, 2);
  } else {
    __bf16 b = (__bf16)f;
    __builtin_memcpy(&raw, &b, 2);
  }
  return raw;
}

// ---- entry points implemented in the kernel files (host side launchers) ----------------------
// statistics / prune
int esp_stats_device(esparse_ctx* ctx, const void* calib, long long T, long long K, int dtype,
                     int bins, std::vector<double>* ir, std::vector<double>* am);
int esp_prune_device(esparse_ctx* ctx, const double* score_host, const void* W, long long N,
                     long long K, int dtype, const esparse_prune_opts* o, int32_t* perm_out,
                     uint8_t* mask_out, int64_t* swaps_out, double* retained_out);
// compression
int esp_compress_device(esparse_ctx* ctx, const void* W, const uint8_t* mask, const int32_t* perm,
                        long long N, long long K, int dtype, int n, int m, void* values_out,
                        void* meta_out, void* native_out);
int esp_dense_pack_device(esparse_ctx* ctx, const void* W, long long N, long long K, int dtype,
                          void* packed);
// products
// report (eq. 4)
int esp_fill_pattern_device(esparse_ctx* ctx, void* dst, size_t bytes);
int esp_output_error_device(esparse_ctx* ctx, const void* Yref, const void* Y, long long count, int dtype, double* num_out,
                            double* den_out);
int esp_matrix_rate_device(esparse_ctx* ctx, int sparse, int dtype, int random_operands, int mix, double* tflops);
int esp_read_rate_device(esparse_ctx* ctx, size_t bytes, double* gbs);

int esp_num_variants();
const char* esp_variant_name(int v);
bool esp_variant_applicable(int v, long long M, long long N, long long K, int sparse);
int esp_default_variant(long long M, long long N, long long K, int sparse);
int esp_default_variant_without_partials(long long M, long long N, long long K, int sparse);
size_t esp_workspace_bytes(long long M, long long N, long long K);
size_t esp_variant_workspace_bytes(int variant, long long M, long long N, long long K);
int esp_static_scratch(esparse_ctx* ctx, void** out);  // device address of this GPU's static scratch (ctx->device current)
#define ESP_PHASE_STAGE 1     // gather X through theta into the workspace
#define ESP_PHASE_MULTIPLY 2  // multiply the staged activations with the weights
int esp_matmul_device(esparse_ctx* ctx, int sparse, const void* X, long long M, const void* w,
                      const int32_t* perm, long long N, long long K, int dtype, void* Y,
                      void* workspace, int variant, int phases);

size_t esp_group_workspace_bytes(int count, long long M, long long N, long long K);
int esp_matmul_group_device(esparse_ctx* ctx, int sparse, int count, const void* const* X, long long M,
                            const void* const* w, const int32_t* const* perm, long long N, long long K,
                            int dtype, void* const* Y, void* workspace, int variant, int phases);
bool esp_variant_is_decode_kernel(int v);

// exact accumulation helpers (host)
// value = sum_b bins[b] * 2^(unit0 + 16*b), rounded once to nearest-even double
double esp_exact_bins_to_double(const unsigned long long* bins, int nb, int unit0);
