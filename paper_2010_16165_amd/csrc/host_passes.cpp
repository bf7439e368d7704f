// Host-side model transformation: batch-norm merge, filter selection, filter
// removal and packing to the device layout.  Pure functions on host memory.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

#include "fupr.h"
#include "layout.h"

extern "C" const char* fupr_status_str(fupr_status s) {
  switch (s) {
    case FUPR_OK: return "ok";
    case FUPR_ERR_NULL: return "null pointer";
    case FUPR_ERR_SHAPE: return "shape mismatch";
    case FUPR_ERR_DTYPE: return "bad or mixed dtype";
    case FUPR_ERR_MASK_EMPTY: return "mask keeps no filter";
    case FUPR_ERR_BN_VAR: return "var + eps is not positive and finite";
    case FUPR_ERR_WORKSPACE: return "workspace too small or misaligned";
    case FUPR_ERR_ALIGN: return "pointer or channel stride misaligned";
    case FUPR_ERR_LAUNCH: return "HIP runtime error";
    case FUPR_ERR_ARG: return "invalid argument";
    case FUPR_ERR_LIMIT: return "size exceeds 32-bit indexing";
    case FUPR_ERR_BN_SCALE: return "batch-norm scale to invert is zero";
    default: return "unknown status";
  }
}

namespace fupr {

bool shape_ok(const fupr_conv_shape* s) {
  return s->K > 0 && s->C > 0 && s->R > 0 && s->S > 0 && s->stride > 0 && s->pad >= 0 &&
         s->R <= 64 && s->S <= 64 && (int64_t)s->K * s->C * s->R * s->S < (int64_t(1) << 31);
}

}  // namespace fupr

using fupr::shape_ok;

// Sec. IV-B-2, Eq. 3-5 and the merge of Sec. VI-B-3.
extern "C" fupr_status fupr_fold(const fupr_conv_shape* shape, const float* W,
                                 const float* conv_bias, const float* gamma, const float* beta,
                                 const float* mean, const float* var, float eps,
                                 uint32_t fuse_flags, float* W_out, float* b_out) {
  if (!shape || !W || !W_out || !b_out) return FUPR_ERR_NULL;
  if (!shape_ok(shape)) return FUPR_ERR_SHAPE;
  if (fuse_flags & ~uint32_t(FUPR_FUSE_BN | FUPR_FUSE_RELU | FUPR_FUSE_ADD)) return FUPR_ERR_ARG;
  const int K = shape->K;
  const size_t crs = (size_t)shape->C * shape->R * shape->S;
  if (!(fuse_flags & FUPR_FUSE_BN)) {
    if (W_out != W) std::memmove(W_out, W, sizeof(float) * K * crs);
    for (int k = 0; k < K; ++k) b_out[k] = conv_bias ? conv_bias[k] : 0.0f;
    return FUPR_OK;
  }
  if (!gamma || !beta || !mean || !var) return FUPR_ERR_NULL;
  std::vector<double> omega(K), lambda(K);
  for (int k = 0; k < K; ++k) {
    const double v = (double)var[k] + (double)eps;
    if (!(v > 0.0) || !std::isfinite(v)) return FUPR_ERR_BN_VAR;
    omega[k] = (double)gamma[k] / std::sqrt(v);
    lambda[k] = (double)beta[k] - omega[k] * (double)mean[k];
  }
  for (int k = 0; k < K; ++k) {
    const float* src = W + (size_t)k * crs;
    float* dst = W_out + (size_t)k * crs;
    for (size_t i = 0; i < crs; ++i) dst[i] = (float)(omega[k] * (double)src[i]);
    const double b = conv_bias ? (double)conv_bias[k] : 0.0;
    b_out[k] = (float)(lambda[k] + omega[k] * b);
  }
  return FUPR_OK;
}

namespace {

// omega and lambda of Eq. 3-5 in double; false if var + eps is unusable.
bool affine_of(const fupr_bn& bn, int K, std::vector<double>* omega, std::vector<double>* lambda) {
  omega->resize(K);
  lambda->resize(K);
  for (int k = 0; k < K; ++k) {
    const double v = (double)bn.var[k] + (double)bn.eps;
    if (!(v > 0.0) || !std::isfinite(v)) return false;
    (*omega)[k] = (double)bn.gamma[k] / std::sqrt(v);
    (*lambda)[k] = (double)bn.beta[k] - (*omega)[k] * (double)bn.mean[k];
  }
  return true;
}

bool bn_present(const fupr_bn* bn) { return bn && bn->gamma && bn->beta && bn->mean && bn->var; }

}  // namespace

// Sec. IV-B-1 (auxiliary and padded convolutions) and IV-B-2 (batch norms).
extern "C" fupr_status fupr_xconv_fuse(const fupr_conv_shape* conv1, const float* W1,
                                       const fupr_bn* bn1, const fupr_conv_shape* conv2,
                                       const float* W2, const fupr_bn* bn2, int32_t shortcut,
                                       const fupr_conv_shape* proj, const float* Wp,
                                       const fupr_bn* bnp, float* W1_out,
                                       const fupr_bn_out* bn1_out, float* W2_out,
                                       float* beta2_out) {
  if (!conv1 || !W1 || !conv2 || !W2 || !W1_out || !W2_out || !beta2_out) return FUPR_ERR_NULL;
  if (!bn_present(bn1) || !bn_present(bn2)) return FUPR_ERR_NULL;
  if (!bn1_out || !bn1_out->gamma || !bn1_out->beta || !bn1_out->mean || !bn1_out->var)
    return FUPR_ERR_NULL;
  if (shortcut != FUPR_SHORTCUT_IDENTITY && shortcut != FUPR_SHORTCUT_SUBSAMPLE_PAD &&
      shortcut != FUPR_SHORTCUT_PROJECTION)
    return FUPR_ERR_ARG;
  if (!shape_ok(conv1) || !shape_ok(conv2)) return FUPR_ERR_SHAPE;
  const int k1 = conv1->K, c = conv1->C, R = conv1->R, S = conv1->S, k2 = conv2->K;
  if (conv2->C != k1 || conv2->R != R || conv2->S != S || R % 2 == 0 || S % 2 == 0 ||
      conv1->pad != R / 2 || conv1->pad != S / 2 || conv2->pad != conv1->pad || conv2->stride != 1)
    return FUPR_ERR_SHAPE;
  if (shortcut == FUPR_SHORTCUT_IDENTITY && (c != k2 || conv1->stride != 1)) return FUPR_ERR_SHAPE;
  if (shortcut == FUPR_SHORTCUT_SUBSAMPLE_PAD && c > k2) return FUPR_ERR_SHAPE;
  if (shortcut == FUPR_SHORTCUT_PROJECTION) {
    if (!proj || !Wp || !bn_present(bnp)) return FUPR_ERR_NULL;
    if (!shape_ok(proj) || proj->K != k2 || proj->C != c || proj->R != 1 || proj->S != 1 ||
        proj->pad != 0 || proj->stride != conv1->stride)
      return FUPR_ERR_SHAPE;
  }
  if ((int64_t)(k1 + c) * c * R * S >= (int64_t(1) << 31) ||
      (int64_t)k2 * (k1 + c) * R * S >= (int64_t(1) << 31))
    return FUPR_ERR_LIMIT;

  std::vector<double> omega2, lambda2, omega_p, lambda_p;
  if (!affine_of(*bn2, k2, &omega2, &lambda2)) return FUPR_ERR_BN_VAR;
  for (int k = 0; k < k2; ++k)
    if (omega2[k] == 0.0) return FUPR_ERR_BN_SCALE;
  if (shortcut == FUPR_SHORTCUT_PROJECTION && !affine_of(*bnp, k2, &omega_p, &lambda_p))
    return FUPR_ERR_BN_VAR;
  {
    const double v1 = 1.0 + (double)bn1->eps;
    if (!(v1 > 0.0) || !std::isfinite(v1)) return FUPR_ERR_BN_VAR;
  }

  const size_t rs = (size_t)R * S, centre = (size_t)(R / 2) * S + S / 2;
  // conv1': conv1's filters, then one identity filter per input channel
  const size_t crs1 = (size_t)c * rs;
  std::memcpy(W1_out, W1, sizeof(float) * k1 * crs1);
  std::memset(W1_out + (size_t)k1 * crs1, 0, sizeof(float) * c * crs1);
  for (int j = 0; j < c; ++j) W1_out[(size_t)(k1 + j) * crs1 + (size_t)j * rs + centre] = 1.0f;
  // bn1': bn1, then omega = 1, lambda = 0
  std::memcpy(bn1_out->gamma, bn1->gamma, sizeof(float) * k1);
  std::memcpy(bn1_out->beta, bn1->beta, sizeof(float) * k1);
  std::memcpy(bn1_out->mean, bn1->mean, sizeof(float) * k1);
  std::memcpy(bn1_out->var, bn1->var, sizeof(float) * k1);
  for (int j = 0; j < c; ++j) {
    bn1_out->gamma[k1 + j] = (float)std::sqrt(1.0 + (double)bn1->eps);
    bn1_out->beta[k1 + j] = 0.0f;
    bn1_out->mean[k1 + j] = 0.0f;
    bn1_out->var[k1 + j] = 1.0f;
  }
  // conv2': conv2's channels, then the auxiliary / padded weights at the centre tap
  const size_t crs2_in = (size_t)k1 * rs, crs2_out = (size_t)(k1 + c) * rs;
  for (int k = 0; k < k2; ++k) {
    float* dst = W2_out + (size_t)k * crs2_out;
    std::memcpy(dst, W2 + (size_t)k * crs2_in, sizeof(float) * crs2_in);
    std::memset(dst + crs2_in, 0, sizeof(float) * c * rs);
    if (shortcut == FUPR_SHORTCUT_PROJECTION) {
      for (int j = 0; j < c; ++j)
        dst[crs2_in + (size_t)j * rs + centre] =
            (float)(omega_p[k] / omega2[k] * (double)Wp[(size_t)k * c + j]);
      beta2_out[k] = (float)((double)bn2->beta[k] + lambda_p[k]);
    } else {
      if (k < c) dst[crs2_in + (size_t)k * rs + centre] = (float)(1.0 / omega2[k]);
      beta2_out[k] = bn2->beta[k];
    }
  }
  return FUPR_OK;
}

// Alg. 1: a non-fused operator loses p_phi * n filters.
// Sec. IV-B-1, projection-shortcut recipe: the shortcut's 1 x 1 convolution
// concatenated to the block's last 1 x 1 convolution along the channels.
extern "C" fupr_status fupr_proj_concat(const fupr_conv_shape* last, const float* W, const float* b,
                                        const fupr_conv_shape* proj, const float* Wp,
                                        const float* bp, fupr_conv_shape* out, float* W_out,
                                        float* b_out) {
  if (!last || !W || !proj || !Wp || !out || !W_out || !b_out) return FUPR_ERR_NULL;
  if (!shape_ok(last) || !shape_ok(proj)) return FUPR_ERR_SHAPE;
  if (last->R != 1 || last->S != 1 || proj->R != 1 || proj->S != 1 || last->pad != 0 ||
      proj->pad != 0 || last->stride != 1 || last->K != proj->K)
    return FUPR_ERR_SHAPE;
  const int K = last->K, C1 = last->C, C2 = proj->C;
  const int C1p = fupr::round_up(C1, FUPR_CAT_ALIGN);
  if ((int64_t)K * (C1p + C2) >= (int64_t(1) << 31)) return FUPR_ERR_SHAPE;
  const size_t C = (size_t)C1p + C2;
  for (int k = 0; k < K; ++k) {
    float* row = W_out + (size_t)k * C;
    std::copy(W + (size_t)k * C1, W + (size_t)(k + 1) * C1, row);
    std::fill(row + C1, row + C1p, 0.0f);
    std::copy(Wp + (size_t)k * C2, Wp + (size_t)(k + 1) * C2, row + C1p);
    b_out[k] = (b ? b[k] : 0.0f) + (bp ? bp[k] : 0.0f);
  }
  *out = fupr_conv_shape{K, C1p + C2, 1, 1, 1, 0};
  return FUPR_OK;
}

extern "C" int32_t fupr_prune_count(int32_t n, int32_t permille) {
  if (n <= 0 || permille < 0 || permille > 1000) return FUPR_ERR_ARG;
  const int64_t cut = ((int64_t)n * permille) / 1000;
  return (int32_t)std::min<int64_t>(cut, n - 1);
}

// Sec. IV-C, Eq. 6.
extern "C" fupr_status fupr_select_filters(const fupr_conv_shape* shape, const float* W,
                                           int32_t norm, int32_t n_prune, uint8_t* mask_out) {
  if (!shape || !W || !mask_out) return FUPR_ERR_NULL;
  if (!shape_ok(shape)) return FUPR_ERR_SHAPE;
  if (norm != 1 && norm != 2) return FUPR_ERR_ARG;
  const int K = shape->K;
  if (n_prune < 0 || n_prune >= K) return FUPR_ERR_ARG;
  const size_t crs = (size_t)shape->C * shape->R * shape->S;
  std::vector<double> score(K);
  for (int k = 0; k < K; ++k) {
    const float* f = W + (size_t)k * crs;
    double acc = 0.0;
    if (norm == 1) {
      for (size_t i = 0; i < crs; ++i) acc += std::fabs((double)f[i]);
      score[k] = acc;
    } else {
      for (size_t i = 0; i < crs; ++i) acc += (double)f[i] * (double)f[i];
      score[k] = std::sqrt(acc);
    }
  }
  std::vector<int> order(K);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int a, int b) { return score[a] < score[b]; });
  std::vector<uint8_t> mask(K, 1);
  for (int i = 0; i < n_prune; ++i) mask[order[i]] = 0;
  std::memcpy(mask_out, mask.data(), K);
  return FUPR_OK;
}

// Alg. 1, last step: masked filters are removed.
extern "C" fupr_status fupr_prune(const fupr_conv_shape* prod, const float* Wp, const float* bp,
                                  const uint8_t* mask, int32_t n_consumers,
                                  const fupr_conv_shape* cons, const float* const* Wc,
                                  int32_t* K_keep, int32_t* keep_idx, float* Wp_out, float* bp_out,
                                  float* const* Wc_out) {
  if (!prod || !Wp || !mask || !K_keep || !keep_idx || !Wp_out) return FUPR_ERR_NULL;
  if (bp && !bp_out) return FUPR_ERR_NULL;
  if (n_consumers < 0) return FUPR_ERR_ARG;
  if (n_consumers > 0 && (!cons || !Wc || !Wc_out)) return FUPR_ERR_NULL;
  if (!shape_ok(prod)) return FUPR_ERR_SHAPE;
  for (int i = 0; i < n_consumers; ++i) {
    if (!Wc[i] || !Wc_out[i]) return FUPR_ERR_NULL;
    if (!shape_ok(&cons[i]) || cons[i].C != prod->K) return FUPR_ERR_SHAPE;
  }
  std::vector<int32_t> keep;
  keep.reserve(prod->K);
  for (int k = 0; k < prod->K; ++k) {
    if (mask[k] > 1) return FUPR_ERR_ARG;
    if (mask[k]) keep.push_back(k);
  }
  if (keep.empty()) return FUPR_ERR_MASK_EMPTY;

  const int kk = (int)keep.size();
  const size_t crs = (size_t)prod->C * prod->R * prod->S;
  for (int j = 0; j < kk; ++j) {
    std::memcpy(Wp_out + (size_t)j * crs, Wp + (size_t)keep[j] * crs, sizeof(float) * crs);
    if (bp) bp_out[j] = bp[keep[j]];
    keep_idx[j] = keep[j];
  }
  for (int i = 0; i < n_consumers; ++i) {
    const size_t rs = (size_t)cons[i].R * cons[i].S;
    const float* src = Wc[i];
    float* dst = Wc_out[i];
    for (int k = 0; k < cons[i].K; ++k)
      for (int j = 0; j < kk; ++j)
        std::memcpy(dst + ((size_t)k * kk + j) * rs,
                    src + ((size_t)k * cons[i].C + keep[j]) * rs, sizeof(float) * rs);
  }
  *K_keep = kk;
  return FUPR_OK;
}

// ---------------------------------------------------------------- packing --

namespace {

// float -> bfloat16 bits, round to nearest even; NaN stays NaN.
uint16_t to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// float -> IEEE half bits, round to nearest even, overflow to infinity.
uint16_t to_f16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  const uint32_t sign = (u >> 16) & 0x8000u;
  const uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);
  if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);  // >= 65520 rounds to inf
  if (a < 0x33000001u) return (uint16_t)sign;               // <= 2^-25 rounds to zero
  int e = (int)(a >> 23) - 127;
  uint32_t mant = (a & 0x7fffffu) | 0x800000u;
  int shift;
  uint32_t base;
  if (e < -14) {  // subnormal half
    shift = 13 + (-14 - e);
    base = 0;
  } else {
    shift = 13;
    base = (uint32_t)(e + 15) << 10;
    mant &= 0x7fffffu;
  }
  uint32_t q = mant >> shift;
  const uint32_t rem = mant & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1);
  if (rem > half || (rem == half && (q & 1u))) ++q;
  return (uint16_t)(sign | (base + q));
}

}  // namespace

extern "C" size_t fupr_packed_bytes(const fupr_conv_shape* shape, fupr_dtype dt) {
  if (!shape || !shape_ok(shape)) return 0;
  if (dt != FUPR_F32 && dt != FUPR_BF16 && dt != FUPR_F16) return 0;
  const fupr::PackedLayout L = fupr::packed_layout(*shape, dt);
  return L.total_bytes;
}

extern "C" fupr_status fupr_pack(const fupr_conv_shape* shape, const float* W, const float* bias,
                                 fupr_dtype dt, void* blob_out) {
  if (!shape || !W || !blob_out) return FUPR_ERR_NULL;
  if (!shape_ok(shape)) return FUPR_ERR_SHAPE;
  if (dt != FUPR_F32 && dt != FUPR_BF16 && dt != FUPR_F16) return FUPR_ERR_DTYPE;
  const fupr::PackedLayout L = fupr::packed_layout(*shape, dt);
  const int K = shape->K, C = shape->C, R = shape->R, S = shape->S;
  std::memset(blob_out, 0, L.total_bytes);
  float* b = reinterpret_cast<float*>(blob_out);
  if (bias) std::memcpy(b, bias, sizeof(float) * K);
  char* wbase = reinterpret_cast<char*>(blob_out) + L.weight_offset;
  if (dt == FUPR_F32) {
    float* w = reinterpret_cast<float*>(wbase);
    for (int k = 0; k < K; ++k)
      for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r)
          for (int s = 0; s < S; ++s)
            w[((size_t)(r * S + s) * L.Cp + c) * L.Kp + k] =
                W[(((size_t)k * C + c) * R + r) * S + s];
    return FUPR_OK;
  }
  uint16_t* w = reinterpret_cast<uint16_t*>(wbase);
  const int cpt = L.Cp / 8;
  for (int k = 0; k < K; ++k)
    for (int c = 0; c < C; ++c)
      for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s) {
          const float v = W[(((size_t)k * C + c) * R + r) * S + s];
          const size_t chunk = (size_t)(r * S + s) * cpt + c / 8;
          w[(chunk * L.Kp + k) * 8 + (c % 8)] = dt == FUPR_BF16 ? to_bf16(v) : to_f16(v);
        }
  return FUPR_OK;
}
