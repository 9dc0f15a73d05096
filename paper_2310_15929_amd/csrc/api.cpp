// C ABI of libesparse: context, argument validation, dispatch.  Every argument check in this
// file runs before the first HIP call of the entry point, so the error paths need no GPU.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cmath>

#include "common.h"

int esp_fail(esparse_ctx* ctx, int code, const char* fmt, ...) {
  if (ctx) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    ctx->err = buf;
  }
  return code;
}

// value = sum_b bins[b] * 2^(unit0 + 16 b), exact, then one round-to-nearest-even to double.
double esp_exact_bins_to_double(const unsigned long long* bins, int nb, int unit0) {
  // little-endian limbs of 32 bits, limb i has weight 2^(unit0 + 32 i)
  const int NL = 2 * 40;
  unsigned long long limb[NL];
  for (int i = 0; i < NL; i++) limb[i] = 0;
  for (int b = 0; b < nb; b++) {
    unsigned long long v = bins[b];
    if (!v) continue;
    int pos = 16 * b;  // bit offset relative to unit0
    int li = pos / 32, sh = pos % 32;
    // v << sh spans up to 96 bits: add three 32-bit pieces
    unsigned long long lo = (v & 0xffffffffull) << sh;  // < 2^64
    unsigned long long hi = (v >> 32) << sh;            // weight 2^32 more
    limb[li] += lo & 0xffffffffull;
    limb[li + 1] += (lo >> 32) + (hi & 0xffffffffull);
    limb[li + 2] += hi >> 32;
  }
  for (int i = 0; i + 1 < NL; i++) {  // carry propagation (each limb holds < 2^40 before this)
    limb[i + 1] += limb[i] >> 32;
    limb[i] &= 0xffffffffull;
  }
  int top = -1;
  for (int i = NL - 1; i >= 0 && top < 0; i--)
    if (limb[i]) {
      int bit = 31;
      while (!((limb[i] >> bit) & 1ull)) bit--;
      top = 32 * i + bit;
    }
  if (top < 0) return 0.0;
  auto bit_at = [&](int p) -> int { return p < 0 ? 0 : (int)((limb[p / 32] >> (p % 32)) & 1ull); };
  // 53 significant bits: positions top .. top-52
  unsigned long long mant = 0;
  for (int p = top; p > top - 53; p--) mant = (mant << 1) | (unsigned long long)bit_at(p);
  int guard = bit_at(top - 53);
  int sticky = 0;
  for (int p = top - 54; p >= 0 && !sticky; p--) sticky |= bit_at(p);
  if (guard && (sticky || (mant & 1ull))) mant++;  // may become 2^53: ldexp handles it
  return std::ldexp((double)mant, unit0 + top - 52);
}

extern "C" {

const char* esparse_version(void) { return "esparse-gfx950 0.1"; }

int esparse_create(esparse_ctx** out, int device, void* hip_stream) {
  if (!out || device < 0) return ESPARSE_EINVAL;
  esparse_ctx* c = new (std::nothrow) esparse_ctx();
  if (!c) return ESPARSE_ENOMEM;
  c->device = device;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  *out = c;
  return ESPARSE_OK;
}

void esparse_destroy(esparse_ctx* ctx) {
  if (!ctx) return;
  if (ctx->d_flags) (void)hipFree(ctx->d_flags);
  delete ctx;
}

int esparse_set_stream(esparse_ctx* ctx, void* hip_stream) {
  if (!ctx) return ESPARSE_EINVAL;
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  return ESPARSE_OK;
}

const char* esparse_last_error(const esparse_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

static int check_dtype(esparse_ctx* ctx, int dtype) {
  ESP_REQUIRE(ctx, dtype == ESPARSE_F16 || dtype == ESPARSE_BF16, ESPARSE_EUNSUPPORTED,
              "dtype %d is not f16 / bf16", dtype);
  return ESPARSE_OK;
}

static int check_pattern(esparse_ctx* ctx, int n, int m) {
  ESP_REQUIRE(ctx, (n == 2 && m == 4) || (n == 4 && m == 8), ESPARSE_EUNSUPPORTED,
              "n:m = %d:%d is not 2:4 or 4:8", n, m);
  return ESPARSE_OK;
}

static int bind_device(esparse_ctx* ctx) {
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  if (!ctx->d_flags) ESP_HIP(ctx, hipMalloc((void**)&ctx->d_flags, 64 * sizeof(int)));
  return ESPARSE_OK;
}

int esparse_channel_stats(esparse_ctx* ctx, const void* calib, long long T, long long K,
                          esparse_dtype dtype, int bins, double* ir_out, double* am_out) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, calib, ESPARSE_EINVAL, "calib is null");
  ESP_REQUIRE(ctx, T >= 1 && T <= (1ll << 24), ESPARSE_EINVAL, "T = %lld outside [1, 2^24]", T);
  ESP_REQUIRE(ctx, K >= 2 && K % 2 == 0, ESPARSE_EINVAL, "K = %lld must be even and >= 2", K);
  ESP_REQUIRE(ctx, bins >= 1 && bins <= 256, ESPARSE_EINVAL, "bins = %d outside [1, 256]", bins);
  ESP_REQUIRE(ctx, esp_aligned16(calib), ESPARSE_EINVAL, "calib is not 16-byte aligned");
  if ((rc = bind_device(ctx))) return rc;
  std::vector<double> ir, am;
  if ((rc = esp_stats_device(ctx, calib, T, K, dtype, bins, ir_out ? &ir : nullptr, am_out ? &am : nullptr)))
    return rc;
  if (ir_out) memcpy(ir_out, ir.data(), sizeof(double) * K);
  if (am_out) memcpy(am_out, am.data(), sizeof(double) * K);
  return ESPARSE_OK;
}

static int check_prune_args(esparse_ctx* ctx, const void* W, long long N, long long K, int dtype,
                            const esparse_prune_opts* o, const int32_t* perm_out,
                            const uint8_t* mask_out) {
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, o, ESPARSE_EINVAL, "opts is null");
  if ((rc = check_pattern(ctx, o->n_keep, o->m_group))) return rc;
  ESP_REQUIRE(ctx, W && perm_out && mask_out, ESPARSE_EINVAL, "W / perm_out / mask_out is null");
  ESP_REQUIRE(ctx, N >= 1 && N < (1ll << 31), ESPARSE_EINVAL, "N = %lld out of range", N);
  ESP_REQUIRE(ctx, K >= o->m_group && K < (1ll << 31), ESPARSE_EINVAL, "K = %lld out of range", K);
  ESP_REQUIRE(ctx, K % o->m_group == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of m = %d", K,
              o->m_group);
  ESP_REQUIRE(ctx, (o->flags & ~ESPARSE_USE_ALL) == 0, ESPARSE_EINVAL, "unknown flag bits 0x%x", o->flags);
  ESP_REQUIRE(ctx, (o->flags & (ESPARSE_USE_ENTROPY | ESPARSE_USE_NORM)) != 0, ESPARSE_EINVAL,
              "flags select neither the entropy nor the norm term");
  if (o->flags & ESPARSE_USE_LBS) {
    ESP_REQUIRE(ctx, o->block >= 2 * o->m_group && o->block <= 256, ESPARSE_EINVAL,
                "block = %d outside [2 m, 256]", o->block);
    ESP_REQUIRE(ctx, o->block % o->m_group == 0, ESPARSE_EINVAL, "block = %d is not a multiple of m = %d",
                o->block, o->m_group);
    ESP_REQUIRE(ctx, K % o->block == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of block = %d", K,
                o->block);
  }
  ESP_REQUIRE(ctx, o->max_swaps >= 0, ESPARSE_EINVAL, "max_swaps < 0");
  ESP_REQUIRE(ctx, esp_aligned16(W) && esp_aligned16(perm_out) && esp_aligned16(mask_out), ESPARSE_EINVAL,
              "W / perm_out / mask_out is not 16-byte aligned");
  return ESPARSE_OK;
}

int esparse_prune_with_scores(esparse_ctx* ctx, const double* score, const void* W, long long N,
                              long long K, esparse_dtype dtype, const esparse_prune_opts* opts,
                              int32_t* perm_out, uint8_t* mask_out, int64_t* swaps_out,
                              double* retained_out) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_prune_args(ctx, W, N, K, dtype, opts, perm_out, mask_out);
  if (rc) return rc;
  ESP_REQUIRE(ctx, score, ESPARSE_EINVAL, "score is null");
  if ((rc = bind_device(ctx))) return rc;
  return esp_prune_device(ctx, score, W, N, K, dtype, opts, perm_out, mask_out, swaps_out, retained_out);
}

int esparse_prune(esparse_ctx* ctx, const void* calib, long long T, const void* W, long long N,
                  long long K, esparse_dtype dtype, const esparse_prune_opts* opts,
                  int32_t* perm_out, uint8_t* mask_out, double* score_out, int64_t* swaps_out,
                  double* retained_out) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_prune_args(ctx, W, N, K, dtype, opts, perm_out, mask_out);
  if (rc) return rc;
  ESP_REQUIRE(ctx, calib, ESPARSE_EINVAL, "calib is null");
  ESP_REQUIRE(ctx, T >= 1 && T <= (1ll << 24), ESPARSE_EINVAL, "T = %lld outside [1, 2^24]", T);
  ESP_REQUIRE(ctx, opts->bins >= 1 && opts->bins <= 256, ESPARSE_EINVAL, "bins = %d outside [1, 256]",
              opts->bins);
  ESP_REQUIRE(ctx, std::isfinite(opts->alpha), ESPARSE_EINVAL, "alpha is not finite");
  ESP_REQUIRE(ctx, esp_aligned16(calib), ESPARSE_EINVAL, "calib is not 16-byte aligned");
  if ((rc = bind_device(ctx))) return rc;
  const bool use_e = opts->flags & ESPARSE_USE_ENTROPY, use_n = opts->flags & ESPARSE_USE_NORM;
  std::vector<double> ir, am;
  if ((rc = esp_stats_device(ctx, calib, T, K, dtype, opts->bins, use_e ? &ir : nullptr, use_n ? &am : nullptr)))
    return rc;
  // eq. 3: s_c = IR_c + alpha * AM_c, each term behind its switch
  std::vector<double> s((size_t)K, 0.0);
  for (long long c = 0; c < K; c++) {
    double v = 0.0;
    if (use_e) v = v + ir[c];
    if (use_n) {
      double t = opts->alpha * am[c];
      v = v + t;
    }
    s[c] = v;
  }
  if (score_out) memcpy(score_out, s.data(), sizeof(double) * K);
  return esp_prune_device(ctx, s.data(), W, N, K, dtype, opts, perm_out, mask_out, swaps_out, retained_out);
}

int esparse_compressed_size(long long N, long long K, int n, int m, esparse_dtype dtype,
                            size_t* values_bytes, size_t* meta_bytes, size_t* native_bytes) {
  if (!((n == 2 && m == 4) || (n == 4 && m == 8))) return ESPARSE_EUNSUPPORTED;
  if (dtype != ESPARSE_F16 && dtype != ESPARSE_BF16) return ESPARSE_EUNSUPPORTED;
  if (N < 0 || K < 0 || K % m != 0) return ESPARSE_EINVAL;
  if (values_bytes) *values_bytes = (size_t)N * (size_t)(K / m * n) * 2;
  if (meta_bytes) *meta_bytes = (m == 4) ? (size_t)N * (size_t)((K / 2 + 15) / 16) * 4 : (size_t)N * (size_t)(K / 8);
  if (native_bytes) {
    size_t Np = (size_t)esp_round_up(N, 16), Kp = (size_t)esp_round_up(K, 256);
    *native_bytes = Np * Kp + Np * Kp / 8;  // both forms: 1 byte of kept values + 1 bit of metadata per weight
  }
  return ESPARSE_OK;
}

int esparse_compress(esparse_ctx* ctx, const void* W, const uint8_t* mask, const int32_t* perm,
                     long long N, long long K, esparse_dtype dtype, int n, int m, void* values_out,
                     void* meta_out, void* native_out) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  if ((rc = check_pattern(ctx, n, m))) return rc;
  ESP_REQUIRE(ctx, W, ESPARSE_EINVAL, "W is null");
  ESP_REQUIRE(ctx, N >= 0 && N < (1ll << 31) && K >= 0 && K < (1ll << 31), ESPARSE_EINVAL, "N or K out of range");
  ESP_REQUIRE(ctx, K % m == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of m = %d", K, m);
  ESP_REQUIRE(ctx, esp_aligned16(W) && esp_aligned16(mask) && esp_aligned16(perm) && esp_aligned16(values_out) &&
                       esp_aligned16(meta_out) && esp_aligned16(native_out),
              ESPARSE_EINVAL, "a pointer is not 16-byte aligned");
  if (N == 0 || K == 0) return ESPARSE_OK;
  if ((rc = bind_device(ctx))) return rc;
  return esp_compress_device(ctx, W, mask, perm, N, K, dtype, n, m, values_out, meta_out, native_out);
}

static int check_matmul(esparse_ctx* ctx, const void* X, long long M, const void* w, long long N,
                        long long K, int dtype, const void* Y, const void* ws, size_t ws_bytes,
                        int variant, int sparse, int phases = 3, bool own_scratch = false) {
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, M >= 0 && M < (1ll << 24), ESPARSE_EINVAL, "M = %lld out of range", M);
  ESP_REQUIRE(ctx, N >= 1 && N < (1ll << 31) && K >= 4 && K < (1ll << 31), ESPARSE_EINVAL, "N or K out of range");
  ESP_REQUIRE(ctx, K % 4 == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of 4", K);
  if (M == 0) return ESPARSE_OK;
  ESP_REQUIRE(ctx, (ws || own_scratch) && ((phases & ESP_PHASE_STAGE) ? X != nullptr : true) &&
                       ((phases & ESP_PHASE_MULTIPLY) ? (w && Y) : true),
              ESPARSE_EINVAL, "X / weights / Y / workspace is null");
  ESP_REQUIRE(ctx, esp_aligned16(X) && esp_aligned16(w) && esp_aligned16(Y), ESPARSE_EINVAL,
              "X / weights / Y is not 16-byte aligned");
  ESP_REQUIRE(ctx, (reinterpret_cast<uintptr_t>(ws) & 255u) == 0, ESPARSE_EINVAL, "workspace is not 256-byte aligned");
  ESP_REQUIRE(ctx, variant >= -1 && variant < esp_num_variants(), ESPARSE_EINVAL, "variant %d does not exist", variant);
  ESP_REQUIRE(ctx, variant < 0 || esp_variant_applicable(variant, M, N, K, sparse), ESPARSE_EUNSUPPORTED,
              "variant %d (%s) cannot run M=%lld N=%lld K=%lld", variant, esp_variant_name(variant), M, N, K);
  // a named variant needs what esparse_spmm_workspace reports for it; the tuned choice (-1) may be any variant
  const size_t need = variant >= 0 ? esp_variant_workspace_bytes(variant, M, N, K) : esp_workspace_bytes(M, N, K);
  ESP_REQUIRE(ctx, own_scratch || ws_bytes >= need, ESPARSE_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
  return ESPARSE_OK;
}

// count = products in the launch: a group call looks for a choice tuned for its size first, then for the single product
static int pick_variant(esparse_ctx* ctx, int sparse, int dtype, long long M, long long N, long long K, int variant, int count = 1) {
  if (variant >= 0) return variant;
  for (int c : {count, 1}) {
    auto it = ctx->tuned.find(std::make_tuple(c, sparse, dtype, M, N, K));
    if (it != ctx->tuned.end() && esp_variant_applicable(it->second, M, N, K, sparse)) return it->second;
  }
  return esp_default_variant(M, N, K, sparse);
}

int esparse_spmm_workspace(long long M, long long N, long long K, int variant, size_t* bytes) {
  if (!bytes || M < 0 || N < 1 || K < 4 || variant < -1 || variant >= esp_num_variants()) return ESPARSE_EINVAL;
  *bytes = variant >= 0 ? esp_variant_workspace_bytes(variant, M, N, K) : esp_workspace_bytes(M, N, K);
  return ESPARSE_OK;
}

int esparse_spmm_num_variants(void) { return esp_num_variants(); }
const char* esparse_spmm_variant_name(int v) { return (v >= 0 && v < esp_num_variants()) ? esp_variant_name(v) : ""; }

static int spmm_phases(esparse_ctx* ctx, const void* X, long long M, const void* native_w, const int32_t* perm,
                       long long N, long long K, esparse_dtype dtype, int n, int m, void* Y, void* workspace,
                       size_t workspace_bytes, int variant, int phases) {
  if (!ctx) return ESPARSE_EINVAL;
  ESP_REQUIRE(ctx, (n == 2 && m == 4) || (n == 4 && m == 8), ESPARSE_EUNSUPPORTED,
              "the sparse product exists for 2:4 and 4:8 only (got %d:%d)", n, m);
  const int mode = m == 4 ? 1 : 2;  // 1: sparse MFMA; 2: bitmaps expanded in registers, dense MFMA
  int rc = check_matmul(ctx, X, M, native_w, N, K, dtype, Y, workspace, workspace_bytes, variant, mode, phases);
  if (rc) return rc;
  ESP_REQUIRE(ctx, K % m == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of %d", K, m);
  ESP_REQUIRE(ctx, esp_aligned16(perm), ESPARSE_EINVAL, "perm is not 16-byte aligned");
  if (M == 0) return ESPARSE_OK;
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_matmul_device(ctx, mode, X, M, native_w, perm, N, K, dtype, Y, workspace,
                           pick_variant(ctx, mode, dtype, M, N, K, variant), phases);
}

int esparse_spmm(esparse_ctx* ctx, const void* X, long long M, const void* native_w, const int32_t* perm,
                 long long N, long long K, esparse_dtype dtype, int n, int m, void* Y, void* workspace,
                 size_t workspace_bytes, int variant) {
  return spmm_phases(ctx, X, M, native_w, perm, N, K, dtype, n, m, Y, workspace, workspace_bytes, variant, 3);
}

int esparse_spmm_static(esparse_ctx* ctx, const void* X, long long M, const void* native_w, const int32_t* perm,
                        long long N, long long K, esparse_dtype dtype, int n, int m, void* Y, int variant) {
  if (!ctx) return ESPARSE_EINVAL;
  ESP_REQUIRE(ctx, (n == 2 && m == 4) || (n == 4 && m == 8), ESPARSE_EUNSUPPORTED,
              "the sparse product exists for 2:4 and 4:8 only (got %d:%d)", n, m);
  const int mode = m == 4 ? 1 : 2;
  int rc = check_matmul(ctx, X, M, native_w, N, K, dtype, Y, nullptr, 0, variant, mode, 3, true);
  if (rc) return rc;
  ESP_REQUIRE(ctx, K % m == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of %d", K, m);
  ESP_REQUIRE(ctx, esp_aligned16(perm), ESPARSE_EINVAL, "perm is not 16-byte aligned");
  if (M == 0) return ESPARSE_OK;
  int v = pick_variant(ctx, mode, dtype, M, N, K, variant);
  size_t need = esp_variant_workspace_bytes(v, M, N, K);
  if (variant < 0 && need > (size_t)ESPARSE_STATIC_SCRATCH_BYTES) {
    // the tuned or built-in choice keeps partial tiles that do not fit the array: the built-in choice among the
    // kernels without partial tiles instead
    v = esp_default_variant_without_partials(M, N, K, mode);
    need = esp_variant_workspace_bytes(v, M, N, K);
  }
  ESP_REQUIRE(ctx, need <= (size_t)ESPARSE_STATIC_SCRATCH_BYTES, ESPARSE_EWORKSPACE,
              "M=%lld N=%lld K=%lld with variant %s needs %zu bytes of scratch, the static scratch holds %zu: use esparse_spmm "
              "with a workspace of the caller's", M, N, K, esp_variant_name(v), need, (size_t)ESPARSE_STATIC_SCRATCH_BYTES);
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  void* ws = nullptr;
  if ((rc = esp_static_scratch(ctx, &ws))) return rc;
  return esp_matmul_device(ctx, mode, X, M, native_w, perm, N, K, dtype, Y, ws, v, ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY);
}

int esparse_stage_activations(esparse_ctx* ctx, const void* X, long long M, const int32_t* perm, long long N,
                              long long K, esparse_dtype dtype, void* workspace, size_t workspace_bytes) {
  return spmm_phases(ctx, X, M, nullptr, perm, N, K, dtype, 2, 4, nullptr, workspace, workspace_bytes, -1,
                     ESP_PHASE_STAGE);
}

int esparse_spmm_staged(esparse_ctx* ctx, long long M, const void* native_w, long long N, long long K,
                        esparse_dtype dtype, int n, int m, void* Y, void* workspace, size_t workspace_bytes,
                        int variant) {
  return spmm_phases(ctx, nullptr, M, native_w, nullptr, N, K, dtype, n, m, Y, workspace, workspace_bytes, variant,
                     ESP_PHASE_MULTIPLY);
}

int esparse_spmm_group_workspace(int count, long long M, long long N, long long K, size_t* bytes) {
  if (!bytes || count < 1 || count > 4 || M < 0 || N < 1 || K < 4) return ESPARSE_EINVAL;
  *bytes = esp_group_workspace_bytes(count, M, N, K);
  return ESPARSE_OK;
}

static int spmm_group_phases(esparse_ctx* ctx, int count, const void* const* X, long long M, const void* const* native_w,
                             const int32_t* const* perm, long long N, long long K, esparse_dtype dtype, int n, int m,
                             void* const* Y, void* workspace, size_t workspace_bytes, int variant, int phases) {
  if (!ctx) return ESPARSE_EINVAL;
  ESP_REQUIRE(ctx, count >= 1 && count <= 4, ESPARSE_EINVAL, "count = %d outside 1..4", count);
  ESP_REQUIRE(ctx, (n == 2 && m == 4) || (n == 4 && m == 8), ESPARSE_EUNSUPPORTED,
              "the sparse product exists for 2:4 and 4:8 only (got %d:%d)", n, m);
  ESP_REQUIRE(ctx, ((phases & ESP_PHASE_STAGE) ? X != nullptr : true) && ((phases & ESP_PHASE_MULTIPLY) ? (native_w && Y) : true),
              ESPARSE_EINVAL, "X / native_w / Y array is null");
  const int mode = m == 4 ? 1 : 2;
  for (int i = 0; i < count; i++) {
    int rc = check_matmul(ctx, X ? X[i] : nullptr, M, native_w ? native_w[i] : nullptr, N, K, dtype, Y ? Y[i] : nullptr, workspace,
                          workspace_bytes, variant, mode, phases);
    if (rc) return rc;
    ESP_REQUIRE(ctx, !perm || esp_aligned16(perm[i]), ESPARSE_EINVAL, "perm[%d] is not 16-byte aligned", i);
  }
  ESP_REQUIRE(ctx, K % m == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of %d", K, m);
  if (M == 0) return ESPARSE_OK;
  ESP_REQUIRE(ctx, workspace_bytes >= esp_group_workspace_bytes(count, M, N, K), ESPARSE_EWORKSPACE,
              "workspace has %zu bytes, %zu needed", workspace_bytes, esp_group_workspace_bytes(count, M, N, K));
  const int v = pick_variant(ctx, mode, dtype, M, N, K, variant, count);
  ESP_REQUIRE(ctx, phases == (ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY) || esp_variant_is_decode_kernel(v), ESPARSE_EUNSUPPORTED,
              "the two halves of a group call exist for the decode kernels only");
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_matmul_group_device(ctx, mode, count, X, M, native_w, perm, N, K, dtype, Y, workspace, v, phases);
}

int esparse_spmm_group(esparse_ctx* ctx, int count, const void* const* X, long long M, const void* const* native_w,
                       const int32_t* const* perm, long long N, long long K, esparse_dtype dtype, int n, int m,
                       void* const* Y, void* workspace, size_t workspace_bytes, int variant) {
  return spmm_group_phases(ctx, count, X, M, native_w, perm, N, K, dtype, n, m, Y, workspace, workspace_bytes, variant,
                           ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY);
}

int esparse_stage_activations_group(esparse_ctx* ctx, int count, const void* const* X, long long M,
                                    const int32_t* const* perm, long long N, long long K, esparse_dtype dtype, int n, int m,
                                    void* workspace, size_t workspace_bytes, int variant) {
  return spmm_group_phases(ctx, count, X, M, nullptr, perm, N, K, dtype, n, m, nullptr, workspace, workspace_bytes, variant,
                           ESP_PHASE_STAGE);
}

int esparse_spmm_group_staged(esparse_ctx* ctx, int count, long long M, const void* const* native_w, long long N, long long K,
                              esparse_dtype dtype, int n, int m, void* const* Y, void* workspace, size_t workspace_bytes,
                              int variant) {
  return spmm_group_phases(ctx, count, nullptr, M, native_w, nullptr, N, K, dtype, n, m, Y, workspace, workspace_bytes, variant,
                           ESP_PHASE_MULTIPLY);
}

int esparse_dense_gemm_group(esparse_ctx* ctx, int count, const void* const* X, long long M, const void* const* packed_w,
                             long long N, long long K, esparse_dtype dtype, void* const* Y, void* workspace,
                             size_t workspace_bytes, int variant) {
  if (!ctx) return ESPARSE_EINVAL;
  ESP_REQUIRE(ctx, count >= 1 && count <= 4, ESPARSE_EINVAL, "count = %d outside 1..4", count);
  ESP_REQUIRE(ctx, X && packed_w && Y, ESPARSE_EINVAL, "X / packed_w / Y array is null");
  for (int i = 0; i < count; i++) {
    int rc = check_matmul(ctx, X[i], M, packed_w[i], N, K, dtype, Y[i], workspace, workspace_bytes, variant, 0, 3);
    if (rc) return rc;
  }
  if (M == 0) return ESPARSE_OK;
  ESP_REQUIRE(ctx, workspace_bytes >= esp_group_workspace_bytes(count, M, N, K), ESPARSE_EWORKSPACE,
              "workspace has %zu bytes, %zu needed", workspace_bytes, esp_group_workspace_bytes(count, M, N, K));
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_matmul_group_device(ctx, 0, count, X, M, packed_w, nullptr, N, K, dtype, Y, workspace,
                                 pick_variant(ctx, 0, dtype, M, N, K, variant, count), ESP_PHASE_STAGE | ESP_PHASE_MULTIPLY);
}

int esparse_dense_packed_size(long long N, long long K, size_t* bytes) {
  if (!bytes || N < 0 || K < 0) return ESPARSE_EINVAL;
  *bytes = (size_t)esp_round_up(N, 16) * (size_t)esp_round_up(K, 256) * 2;
  return ESPARSE_OK;
}

int esparse_dense_pack(esparse_ctx* ctx, const void* W, long long N, long long K, esparse_dtype dtype,
                       void* packed_out) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, W && packed_out, ESPARSE_EINVAL, "W / packed_out is null");
  ESP_REQUIRE(ctx, N >= 1 && N < (1ll << 31) && K >= 4 && K < (1ll << 31) && K % 4 == 0, ESPARSE_EINVAL,
              "N or K out of range (K must be a multiple of 4)");
  ESP_REQUIRE(ctx, esp_aligned16(W) && esp_aligned16(packed_out), ESPARSE_EINVAL, "a pointer is not 16-byte aligned");
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_dense_pack_device(ctx, W, N, K, dtype, packed_out);
}

static int dense_phases(esparse_ctx* ctx, const void* X, long long M, const void* packed_w, long long N,
                        long long K, esparse_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                        int variant, int phases) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_matmul(ctx, X, M, packed_w, N, K, dtype, Y, workspace, workspace_bytes, variant, 0, phases);
  if (rc) return rc;
  if (M == 0) return ESPARSE_OK;
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_matmul_device(ctx, 0, X, M, packed_w, nullptr, N, K, dtype, Y, workspace,
                           pick_variant(ctx, 0, dtype, M, N, K, variant), phases);
}

int esparse_dense_gemm(esparse_ctx* ctx, const void* X, long long M, const void* packed_w, long long N,
                       long long K, esparse_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                       int variant) {
  return dense_phases(ctx, X, M, packed_w, N, K, dtype, Y, workspace, workspace_bytes, variant, 3);
}

int esparse_dense_gemm_staged(esparse_ctx* ctx, long long M, const void* packed_w, long long N, long long K,
                              esparse_dtype dtype, void* Y, void* workspace, size_t workspace_bytes, int variant) {
  return dense_phases(ctx, nullptr, M, packed_w, N, K, dtype, Y, workspace, workspace_bytes, variant,
                      ESP_PHASE_MULTIPLY);
}

static int tune_impl(esparse_ctx* ctx, int count, long long M, long long N, long long K, esparse_dtype dtype, int sparse,
                     int* best_variant, float* best_ms) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, count >= 1 && count <= 4, ESPARSE_EINVAL, "count = %d outside 1..4", count);
  ESP_REQUIRE(ctx, M >= 1 && M < (1ll << 24) && N >= 1 && N < (1ll << 31) && K >= 4 && K < (1ll << 31) && K % 4 == 0,
              ESPARSE_EINVAL, "shape out of range");
  sparse = sparse == 2 ? 2 : (sparse ? 1 : 0);
  ESP_REQUIRE(ctx, sparse != 2 || K % 8 == 0, ESPARSE_EINVAL, "K = %lld is not a multiple of 8", K);
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  const size_t Np = (size_t)esp_round_up(N, 16), Kp = (size_t)esp_round_up(K, 256);
  DevBuf w, x, y, ws;
  // the timed launches rotate over copies of the weight operand, more of them than the caches hold (256 MiB
  // last-level cache): in a model every matrix is read once per step, so the cold time is the one that counts
  const size_t wbytes = ((sparse ? Np * Kp + Np * Kp / 8 : Np * Kp * 2) + 255) / 256 * 256;
  const int ncopies = (int)std::max<size_t>(2 * count, std::min<size_t>(64, ((size_t)640 << 20) / wbytes + count));
  const size_t ybytes = ((size_t)M * N * 2 + 255) / 256 * 256;
  const size_t xbytes = ((size_t)M * K * 2 + 255) / 256 * 256;
  if (w.alloc(wbytes * ncopies) != hipSuccess || x.alloc(xbytes) != hipSuccess ||
      y.alloc(ybytes * count) != hipSuccess || ws.alloc(esp_group_workspace_bytes(count, M, N, K)) != hipSuccess)
    return esp_fail(ctx, ESPARSE_ENOMEM, "scratch allocation for tuning failed");
  // operands: finite pseudo-random 16-bit values (zeros would time differently, see esp_fill_pattern_device)
  if ((rc = esp_fill_pattern_device(ctx, w.p, wbytes * ncopies))) return rc;
  if ((rc = esp_fill_pattern_device(ctx, x.p, xbytes))) return rc;
  struct Events {  // destroyed on every way out
    hipEvent_t e[2] = {nullptr, nullptr};
    ~Events() {
      for (hipEvent_t ev : e)
        if (ev) (void)hipEventDestroy(ev);
    }
  } events;
  ESP_HIP(ctx, hipEventCreate(&events.e[0]));
  ESP_HIP(ctx, hipEventCreate(&events.e[1]));
  const hipEvent_t e0 = events.e[0], e1 = events.e[1];
  const int reps = 20;
  const unsigned char* wbase = reinterpret_cast<const unsigned char*>(w.p);
  unsigned char* ybase = reinterpret_cast<unsigned char*>(y.p);
  // average duration of `reps` launches of variant v after three untimed ones; launch i reads the weight copies
  // i count, i count + 1, ... (mod ncopies)
  auto time_variant = [&](int v, float* ms_out) -> int {
    auto launch = [&](int i) {
      const void* Xs[4];
      const void* Ws[4];
      void* Ys[4];
      for (int j = 0; j < count; j++) {
        Xs[j] = x.p;
        Ws[j] = wbase + (size_t)((i * count + j) % ncopies) * wbytes;
        Ys[j] = ybase + (size_t)j * ybytes;
      }
      if (count == 1) return esp_matmul_device(ctx, sparse, Xs[0], M, Ws[0], nullptr, N, K, dtype, Ys[0], ws.p, v, 3);
      return esp_matmul_group_device(ctx, sparse, count, Xs, M, Ws, nullptr, N, K, dtype, Ys, ws.p, v, 3);
    };
    int r = 0;
    for (int i = 0; i < 3; i++)
      if ((r = launch(i))) return r;
    (void)hipEventRecord(e0, ctx->stream);
    for (int i = 0; i < reps; i++)
      if ((r = launch(i + 3))) break;
    (void)hipEventRecord(e1, ctx->stream);
    if (r) return r;
    if (hipEventSynchronize(e1) != hipSuccess) return esp_fail(ctx, ESPARSE_EHIP, "event synchronize failed while tuning");
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    *ms_out = ms / reps;
    return ESPARSE_OK;
  };
  std::vector<std::pair<float, int>> timed;  // (ms, variant)
  for (int v = 0; v < esp_num_variants() && !rc; v++) {
    if (!esp_variant_applicable(v, M, N, K, sparse)) continue;
    float ms = 0.f;
    if (!(rc = time_variant(v, &ms))) timed.emplace_back(ms, v);
  }
  int best = -1;
  float best_t = 0.f;
  if (!rc && !timed.empty()) {
    // The first pass times every variant once, one after the other, while the clocks still move with the load: variants
    // within a few percent of each other come out in an order that changes from run to run.  The (at most four) variants
    // within 6 % of the fastest are therefore timed twice more, in alternating order, and ranked by their mean.
    std::sort(timed.begin(), timed.end());
    size_t nclose = 1;
    while (nclose < timed.size() && nclose < 4 && timed[nclose].first <= timed[0].first * 1.06f) nclose++;
    std::vector<float> sum(nclose);
    for (size_t i = 0; i < nclose; i++) sum[i] = timed[i].first;
    if (nclose > 1)
      for (int round = 0; round < 2 && !rc; round++)
        for (size_t q = 0; q < nclose && !rc; q++) {
          const size_t i = round == 0 ? nclose - 1 - q : q;
          float ms = 0.f;
          if (!(rc = time_variant(timed[i].second, &ms))) sum[i] += ms;
        }
    if (!rc) {
      size_t pick = 0;
      for (size_t i = 1; i < nclose; i++)
        if (sum[i] < sum[pick]) pick = i;
      best = timed[pick].second;
      best_t = nclose > 1 ? sum[pick] / 3.f : sum[pick];
    }
  }
  if (rc) return rc;
  ESP_REQUIRE(ctx, best >= 0, ESPARSE_EUNSUPPORTED, "no variant can run this shape");
  ctx->tuned[std::make_tuple(count, sparse, (int)dtype, M, N, K)] = best;
  if (best_variant) *best_variant = best;
  if (best_ms) *best_ms = best_t;
  return ESPARSE_OK;
}

int esparse_tune(esparse_ctx* ctx, long long M, long long N, long long K, esparse_dtype dtype, int sparse, int* best_variant,
                 float* best_ms) {
  return tune_impl(ctx, 1, M, N, K, dtype, sparse, best_variant, best_ms);
}

int esparse_tune_group(esparse_ctx* ctx, int count, long long M, long long N, long long K, esparse_dtype dtype, int sparse,
                       int* best_variant, float* best_ms) {
  return tune_impl(ctx, count, M, N, K, dtype, sparse, best_variant, best_ms);
}

int esparse_output_error(esparse_ctx* ctx, const void* Yref, const void* Y, long long M, long long N, esparse_dtype dtype,
                         double* err_num, double* err_den) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, err_num && err_den, ESPARSE_EINVAL, "err_num / err_den is null");
  ESP_REQUIRE(ctx, M >= 0 && N >= 0 && M < (1ll << 31) && N < (1ll << 31), ESPARSE_EINVAL, "M or N out of range");
  *err_num = 0.0;
  *err_den = 0.0;
  if (M == 0 || N == 0) return ESPARSE_OK;
  ESP_REQUIRE(ctx, Yref && Y, ESPARSE_EINVAL, "Yref / Y is null");
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_output_error_device(ctx, Yref, Y, M * N, dtype, err_num, err_den);
}

int esparse_matrix_rate(esparse_ctx* ctx, int sparse, esparse_dtype dtype, int random_operands, int mix, double* tflops) {
  if (!ctx) return ESPARSE_EINVAL;
  int rc = check_dtype(ctx, dtype);
  if (rc) return rc;
  ESP_REQUIRE(ctx, tflops != nullptr, ESPARSE_EINVAL, "tflops is null");
  ESP_REQUIRE(ctx, (sparse == 0 || sparse == 1) && (random_operands == 0 || random_operands == 1) && mix >= 0 && mix <= 2,
              ESPARSE_EINVAL, "sparse and random_operands are 0 or 1, mix is 0, 1 or 2");
  ESP_REQUIRE(ctx, mix == 0 || (sparse == 1 && random_operands == 1), ESPARSE_EUNSUPPORTED,
              "the stage mixes exist for the 2:4 instruction on random operands");
  *tflops = 0.0;
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_matrix_rate_device(ctx, sparse, dtype, random_operands, mix, tflops);
}

int esparse_read_rate(esparse_ctx* ctx, size_t bytes, double* gbs) {
  if (!ctx) return ESPARSE_EINVAL;
  ESP_REQUIRE(ctx, gbs != nullptr, ESPARSE_EINVAL, "gbs is null");
  ESP_REQUIRE(ctx, bytes >= 4096 && bytes <= ((size_t)8 << 30), ESPARSE_EINVAL, "bytes outside 4 KiB .. 8 GiB");
  *gbs = 0.0;
  ESP_HIP(ctx, hipSetDevice(ctx->device));
  return esp_read_rate_device(ctx, bytes, gbs);
}

int esparse_tune_save(const esparse_ctx* ctx, const char* path) {
  if (!ctx || !path) return ESPARSE_EINVAL;
  FILE* f = fopen(path, "w");
  if (!f) return ESPARSE_EINVAL;
  fprintf(f, "# sparse dtype M N K variant-name [products per launch, 1 if absent]\n");
  for (const auto& kv : ctx->tuned) {
    fprintf(f, "%d %d %lld %lld %lld %s", std::get<1>(kv.first), std::get<2>(kv.first), std::get<3>(kv.first),
            std::get<4>(kv.first), std::get<5>(kv.first), esp_variant_name(kv.second));
    if (std::get<0>(kv.first) != 1) fprintf(f, " %d", std::get<0>(kv.first));
    fprintf(f, "\n");
  }
  fclose(f);
  return ESPARSE_OK;
}

int esparse_tune_load(esparse_ctx* ctx, const char* path) {
  if (!ctx || !path) return ESPARSE_EINVAL;
  FILE* f = fopen(path, "r");
  if (!f) return esp_fail(ctx, ESPARSE_EINVAL, "cannot open %s", path);
  char line[256];
  while (fgets(line, sizeof line, f)) {
    if (line[0] == '#') continue;
    int sp, dt, count = 1;
    long long M, N, K;
    char name[128];
    const int got = sscanf(line, "%d %d %lld %lld %lld %127s %d", &sp, &dt, &M, &N, &K, name, &count);
    if (got < 6 || count < 1 || count > 4) continue;
    for (int v = 0; v < esp_num_variants(); v++)
      if (!strcmp(name, esp_variant_name(v))) ctx->tuned[std::make_tuple(count, sp, dt, M, N, K)] = v;
  }
  fclose(f);
  return ESPARSE_OK;
}

}  // extern "C"
