// Host side of libbsp: the packer (mask + dense weights -> compressed block
// rows), its inverse, index validation, and the launch-plan builder.
// No device code and no HIP calls in this file.
#include "bsp.h"
#include "bsp_plan.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <vector>

bool bsp_rows_wanted(int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                     int32_t dtype);
int bsp_rows_section(const int32_t* row_ptr, const int32_t* col_idx, const uint16_t* payload,
                     int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                     std::vector<int32_t>* sec);
bool bsp_first_wanted(int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi, int32_t dtype);
int bsp_first_section(const int32_t* row_ptr, const int32_t* col_idx, const uint16_t* payload,
                      int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                      std::vector<int32_t>* sec);

namespace {

inline bool granularity_ok(int32_t bo, int32_t bi) {
  return (bo == 8 && bi == 8) || (bo == 4 && bi == 16) || (bo == 16 && bi == 4);
}

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// fp32 -> bf16, round to nearest, ties to even (finite values; NaN keeps a quiet pattern).
inline uint16_t f32_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
inline float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

int check_layer(int32_t O, int32_t I, int32_t bo, int32_t bi) {
  if (O <= 0 || I <= 0) return BSP_ERR_SHAPE;
  if (!granularity_ok(bo, bi)) return BSP_ERR_UNSUPPORTED;
  return BSP_OK;
}

template <typename Src, typename Dst> inline Dst convert(Src v);
template <> inline float convert<float, float>(float v) { return v; }
template <> inline uint16_t convert<uint16_t, uint16_t>(uint16_t v) { return v; }
template <> inline uint16_t convert<float, uint16_t>(float v) { return f32_to_bf16(v); }
template <> inline float convert<uint16_t, float>(uint16_t v) { return bf16_to_f32(v); }
template <> inline int8_t convert<int8_t, int8_t>(int8_t v) { return v; }

// Copy the kept blocks of W, block row by block row, column ascending.
template <typename Src, typename Dst>
void compact(const Src* W, const uint8_t* gamma, int32_t O, int32_t H, int32_t K, int32_t I,
             int32_t bo, int32_t bi, int32_t* row_ptr, int32_t* col_idx, Dst* payload) {
  const int64_t nbr = cdiv(O, bo), nbc = cdiv(I, bi);
  const int64_t HK = (int64_t)H * K;
  int64_t n = 0;
  row_ptr[0] = 0;
  for (int64_t l = 0; l < nbr; ++l) {
    for (int64_t c = 0; c < nbc; ++c) {
      if (!gamma[l * nbc + c]) continue;
      col_idx[n] = (int32_t)c;
      Dst* blk = payload + n * bo * HK * bi;
      const int64_t i0 = c * bi;
      const int64_t ni = (I - i0 < bi) ? (I - i0) : bi;
      for (int64_t r = 0; r < bo; ++r) {
        const int64_t o = l * bo + r;
        for (int64_t t = 0; t < HK; ++t) {
          Dst* d = blk + (r * HK + t) * bi;
          if (o < O) {
            const Src* s = W + (o * HK + t) * I + i0;
            for (int64_t j = 0; j < ni; ++j) d[j] = convert<Src, Dst>(s[j]);
            for (int64_t j = ni; j < bi; ++j) d[j] = Dst(0);
          } else {
            for (int64_t j = 0; j < bi; ++j) d[j] = Dst(0);
          }
        }
      }
      ++n;
    }
    row_ptr[l + 1] = (int32_t)n;
  }
}

template <typename T>
void expand(const int32_t* row_ptr, const int32_t* col_idx, const T* payload, int32_t O,
            int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi, T* W) {
  const int64_t nbr = cdiv(O, bo);
  const int64_t HK = (int64_t)H * K;
  std::memset(W, 0, sizeof(T) * (size_t)O * HK * I);
  for (int64_t l = 0; l < nbr; ++l)
    for (int64_t n = row_ptr[l]; n < row_ptr[l + 1]; ++n) {
      const int64_t i0 = (int64_t)col_idx[n] * bi;
      const int64_t ni = (I - i0 < bi) ? (I - i0) : bi;
      const T* blk = payload + n * bo * HK * bi;
      for (int64_t r = 0; r < bo && l * bo + r < O; ++r)
        for (int64_t t = 0; t < HK; ++t)
          std::memcpy(W + ((l * bo + r) * HK + t) * I + i0, blk + (r * HK + t) * bi,
                      sizeof(T) * (size_t)ni);
    }
}

}  // namespace

extern "C" {

const char* bsp_strerror(int code) {
  switch (code) {
    case BSP_OK: return "ok";
    case BSP_ERR_NULL: return "null pointer";
    case BSP_ERR_SHAPE: return "bad or inconsistent shape";
    case BSP_ERR_MASK: return "mask byte is neither 0 nor 1";
    case BSP_ERR_INDEX: return "row_ptr / col_idx malformed";
    case BSP_ERR_DTYPE: return "element type not supported";
    case BSP_ERR_UNSUPPORTED:
      return "unsupported: block granularity not in {8x8, 4x16, 16x4}, or a layer outside the "
             "requested kernel family";
    case BSP_ERR_CAPACITY: return "output buffer (or the fixed scratch memory of a *_static call) too small";
    case BSP_ERR_HIP: return "HIP runtime error at launch";
    case BSP_ERR_ALIGN: return "device pointer not 16-byte aligned";
    default: return "unknown status";
  }
}

int bsp_version(void) { return 1; }

int bsp_pack_count(const uint8_t* gamma, int32_t O, int32_t I, int32_t bo, int32_t bi,
                   int64_t* nnzb) {
  if (!gamma || !nnzb) return BSP_ERR_NULL;
  if (int rc = check_layer(O, I, bo, bi)) return rc;
  const int64_t total = cdiv(O, bo) * cdiv(I, bi);
  int64_t n = 0;
  for (int64_t t = 0; t < total; ++t) {
    if (gamma[t] > 1) return BSP_ERR_MASK;
    n += gamma[t];
  }
  *nnzb = n;
  return BSP_OK;
}

int bsp_pack(const void* W, int32_t w_dtype, const uint8_t* gamma, int32_t O, int32_t H,
             int32_t K, int32_t I, int32_t bo, int32_t bi, int32_t payload_dtype,
             int32_t* row_ptr, int32_t* col_idx, int64_t col_capacity, void* payload,
             int64_t payload_capacity_bytes) {
  if (!W || !gamma || !row_ptr) return BSP_ERR_NULL;
  if (H <= 0 || K <= 0) return BSP_ERR_SHAPE;
  int64_t nnzb = 0;
  if (int rc = bsp_pack_count(gamma, O, I, bo, bi, &nnzb)) return rc;
  const bool codes = w_dtype == BSP_I8 || payload_dtype == BSP_I8;
  if (codes ? (w_dtype != payload_dtype)
            : ((w_dtype != BSP_F32 && w_dtype != BSP_BF16) ||
               (payload_dtype != BSP_F32 && payload_dtype != BSP_BF16)))
    return BSP_ERR_DTYPE;
  if (nnzb > 0 && (!col_idx || !payload)) return BSP_ERR_NULL;
  if (nnzb > std::numeric_limits<int32_t>::max()) return BSP_ERR_SHAPE;
  const int64_t esz = payload_dtype == BSP_F32 ? 4 : payload_dtype == BSP_BF16 ? 2 : 1;
  if (col_capacity < nnzb) return BSP_ERR_CAPACITY;
  if (payload_capacity_bytes < nnzb * bo * bi * (int64_t)H * K * esz) return BSP_ERR_CAPACITY;
  if (codes)
    compact((const int8_t*)W, gamma, O, H, K, I, bo, bi, row_ptr, col_idx, (int8_t*)payload);
  else if (w_dtype == BSP_F32 && payload_dtype == BSP_F32)
    compact((const float*)W, gamma, O, H, K, I, bo, bi, row_ptr, col_idx, (float*)payload);
  else if (w_dtype == BSP_F32)
    compact((const float*)W, gamma, O, H, K, I, bo, bi, row_ptr, col_idx, (uint16_t*)payload);
  else if (payload_dtype == BSP_F32)
    compact((const uint16_t*)W, gamma, O, H, K, I, bo, bi, row_ptr, col_idx, (float*)payload);
  else
    compact((const uint16_t*)W, gamma, O, H, K, I, bo, bi, row_ptr, col_idx,
            (uint16_t*)payload);
  return BSP_OK;
}

int bsp_validate(const int32_t* row_ptr, const int32_t* col_idx, int32_t O, int32_t I,
                 int32_t bo, int32_t bi) {
  if (!row_ptr) return BSP_ERR_NULL;
  if (int rc = check_layer(O, I, bo, bi)) return rc;
  const int64_t nbr = cdiv(O, bo), nbc = cdiv(I, bi);
  if (row_ptr[0] != 0) return BSP_ERR_INDEX;
  for (int64_t l = 0; l < nbr; ++l) {
    const int64_t a = row_ptr[l], b = row_ptr[l + 1];
    if (b < a || b - a > nbc) return BSP_ERR_INDEX;
    if (b > a && !col_idx) return BSP_ERR_NULL;
    for (int64_t n = a; n < b; ++n) {
      if (col_idx[n] < 0 || col_idx[n] >= nbc) return BSP_ERR_INDEX;
      if (n > a && col_idx[n] <= col_idx[n - 1]) return BSP_ERR_INDEX;
    }
  }
  return BSP_OK;
}

int bsp_unpack(const int32_t* row_ptr, const int32_t* col_idx, const void* payload,
               int32_t payload_dtype, int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo,
               int32_t bi, void* W) {
  if (!W) return BSP_ERR_NULL;
  if (H <= 0 || K <= 0) return BSP_ERR_SHAPE;
  if (int rc = bsp_validate(row_ptr, col_idx, O, I, bo, bi)) return rc;
  if (payload_dtype != BSP_F32 && payload_dtype != BSP_BF16 && payload_dtype != BSP_I8)
    return BSP_ERR_DTYPE;
  const int64_t nnzb = row_ptr[cdiv(O, bo)];
  if (nnzb > 0 && !payload) return BSP_ERR_NULL;
  if (payload_dtype == BSP_I8)
    expand(row_ptr, col_idx, (const int8_t*)payload, O, H, K, I, bo, bi, (int8_t*)W);
  else if (payload_dtype == BSP_F32)
    expand(row_ptr, col_idx, (const float*)payload, O, H, K, I, bo, bi, (float*)W);
  else
    expand(row_ptr, col_idx, (const uint16_t*)payload, O, H, K, I, bo, bi, (uint16_t*)W);
  return BSP_OK;
}

}  // extern "C"

// ------------------------------------------------------------ choosing the mask
namespace {

// zero `count` kept entries with the lowest score (ties: lower index first)
void zero_lowest(const double* score, uint8_t* gamma, int64_t n, int64_t count) {
  std::vector<int64_t> kept;
  for (int64_t i = 0; i < n; ++i)
    if (gamma[i]) kept.push_back(i);
  std::stable_sort(kept.begin(), kept.end(),
                   [&](int64_t a, int64_t b) { return score[a] < score[b]; });
  for (int64_t i = 0; i < count && i < (int64_t)kept.size(); ++i) gamma[kept[i]] = 0;
}

}  // namespace

extern "C" {

int bsp_block_importance(const float* W, int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo,
                         int32_t bi, int32_t measure, double* score) {
  if (!W || !score) return BSP_ERR_NULL;
  if (H <= 0 || K <= 0) return BSP_ERR_SHAPE;
  if (int rc = check_layer(O, I, bo, bi)) return rc;
  if (measure < BSP_IMPORTANCE_L2 || measure > BSP_IMPORTANCE_VAR) return BSP_ERR_SHAPE;
  const int64_t nbr = cdiv(O, bo), nbc = cdiv(I, bi);
  const int64_t HK = (int64_t)H * K;
  const double n = (double)bo * (double)HK * (double)bi;
  for (int64_t l = 0; l < nbr; ++l)
    for (int64_t c = 0; c < nbc; ++c) {
      const int64_t no = std::min<int64_t>(bo, O - l * bo), ni = std::min<int64_t>(bi, I - c * bi);
      long double s1 = 0.0L, s2 = 0.0L, sa = 0.0L;  // extended sums: the rank must not hinge on rounding
      for (int64_t r = 0; r < no; ++r)
        for (int64_t t = 0; t < HK; ++t) {
          const float* w = W + ((l * bo + r) * HK + t) * I + c * bi;
          for (int64_t j = 0; j < ni; ++j) {
            const long double v = (long double)w[j];
            s1 += v;
            s2 += v * v;
            sa += v < 0 ? -v : v;
          }
        }
      double out;
      if (measure == BSP_IMPORTANCE_L2) {
        out = std::sqrt((double)s2);
      } else if (measure == BSP_IMPORTANCE_L1) {
        out = (double)sa;
      } else {
        // sum (w - mu)^2 over the n stored entries, the overhang's zeros included
        const long double mu = s1 / (long double)n;
        long double acc = 0.0L;
        for (int64_t r = 0; r < no; ++r)
          for (int64_t t = 0; t < HK; ++t) {
            const float* w = W + ((l * bo + r) * HK + t) * I + c * bi;
            for (int64_t j = 0; j < ni; ++j) {
              const long double d = (long double)w[j] - mu;
              acc += d * d;
            }
          }
        acc += ((long double)n - (long double)(no * HK * ni)) * mu * mu;
        out = (double)(acc / (long double)n);
      }
      score[l * nbc + c] = out;
    }
  return BSP_OK;
}

int bsp_select_mask(const float* W, int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo,
                    int32_t bi, int32_t measure, double density, int32_t per_row,
                    uint8_t* gamma) {
  if (!gamma) return BSP_ERR_NULL;
  if (!(density >= 0.0 && density <= 1.0)) return BSP_ERR_SHAPE;
  const int64_t nbr = cdiv(O, bo), nbc = cdiv(I, bi);
  if (O <= 0 || I <= 0) return BSP_ERR_SHAPE;
  std::vector<double> score((size_t)(nbr * nbc));
  if (int rc = bsp_block_importance(W, O, H, K, I, bo, bi, measure, score.data())) return rc;
  std::memset(gamma, 1, (size_t)(nbr * nbc));
  if (per_row) {
    const int64_t keep = (int64_t)std::nearbyint(density * (double)nbc);
    for (int64_t l = 0; l < nbr; ++l)
      zero_lowest(score.data() + l * nbc, gamma + l * nbc, nbc, nbc - keep);
  } else {
    const int64_t keep = (int64_t)std::nearbyint(density * (double)(nbr * nbc));
    zero_lowest(score.data(), gamma, nbr * nbc, nbr * nbc - keep);
  }
  return BSP_OK;
}

int bsp_mask_step(const float* W, int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo,
                  int32_t bi, int32_t measure, double target_density, uint8_t* gamma,
                  int32_t* zeroed) {
  if (!gamma || !zeroed) return BSP_ERR_NULL;
  if (!(target_density >= 0.0 && target_density <= 1.0)) return BSP_ERR_SHAPE;
  int64_t kept = 0;
  if (int rc = bsp_pack_count(gamma, O, I, bo, bi, &kept)) return rc;
  const int64_t n = cdiv(O, bo) * cdiv(I, bi);
  std::vector<double> score((size_t)n);
  if (int rc = bsp_block_importance(W, O, H, K, I, bo, bi, measure, score.data())) return rc;
  const int64_t k = kept - (int64_t)std::nearbyint(target_density * (double)n);
  *zeroed = 0;
  if (k <= 0) return BSP_OK;
  int64_t step = (int64_t)std::ceil(0.05 * (double)k);
  if (step < 1) step = 1;
  if (step > k) step = k;
  zero_lowest(score.data(), gamma, n, step);
  *zeroed = (int32_t)step;
  return BSP_OK;
}

}  // extern "C"

extern "C" {

int bsp_bcsr_segments(const int32_t* row_ptr, const int32_t* col_idx, int32_t rows, int32_t cols,
                      int32_t* seg_ptr) {
  if (!row_ptr || !seg_ptr) return BSP_ERR_NULL;
  if (rows <= 0 || cols <= 0) return BSP_ERR_SHAPE;
  if (int rc = bsp_validate(row_ptr, col_idx, rows * 8, cols * 8, 8, 8)) return rc;
  const int64_t nsub = (cols + 15) / 16;
  for (int64_t r = 0; r < rows; ++r) {
    int32_t* sp = seg_ptr + r * (nsub + 1);
    int64_t n = row_ptr[r];
    for (int64_t s = 0; s <= nsub; ++s) {  // col_idx is ascending within the row
      while (n < row_ptr[r + 1] && col_idx[n] < 16 * s) ++n;
      sp[s] = (int32_t)n;
    }
  }
  return BSP_OK;
}

int bsp_quantize(const float* W, int64_t n, int32_t bits, int8_t* codes, double* delta) {
  if (!delta || (n > 0 && (!W || !codes))) return BSP_ERR_NULL;
  if (n < 0 || bits < 2 || bits > 8) return BSP_ERR_SHAPE;
  double top = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    const double a = std::fabs((double)W[i]);
    if (a > top) top = a;
  }
  if (top == 0.0) {
    *delta = 0.0;
    for (int64_t i = 0; i < n; ++i) codes[i] = 0;
    return BSP_OK;
  }
  const double d = top / (double)(1 << (bits - 1));
  const double lo = -(double)(1 << (bits - 1)), hi = (double)((1 << (bits - 1)) - 1);
  for (int64_t i = 0; i < n; ++i) {
    double q = std::nearbyint((double)W[i] / d);  // default rounding mode: ties to even
    if (q < lo) q = lo;
    if (q > hi) q = hi;
    codes[i] = (int8_t)q;
  }
  *delta = d;
  return BSP_OK;
}

// ---------------------------------------------------------------- launch plan
// One pass serves both entry points: with out == nullptr it only counts.
static int plan_walk(const int32_t* row_ptr, const int32_t* col_idx, const void* payload,
                     int32_t dtype, int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo,
                     int32_t bi, int32_t* out, int64_t capacity_words, int64_t* words_needed) {
  if (H <= 0 || K <= 0) return BSP_ERR_SHAPE;
  if (dtype != BSP_F32 && dtype != BSP_BF16 && dtype != BSP_I8) return BSP_ERR_DTYPE;
  if (H > 255 || K > 255) return BSP_ERR_SHAPE;
  if (int rc = bsp_validate(row_ptr, col_idx, O, I, bo, bi)) return rc;
  const int64_t nbr = cdiv(O, bo);
  const int64_t HK = (int64_t)H * K;
  const int64_t blk_elems = (int64_t)bo * bi * HK;
  const int64_t nnzb = row_ptr[nbr];
  if (nnzb * blk_elems > std::numeric_limits<int32_t>::max()) return BSP_ERR_SHAPE;
  const int32_t nstrips = (int32_t)cdiv(O, BSP_STRIP);
  const int32_t nxc = (int32_t)cdiv(I, BSP_CHUNK);
  const int32_t rows_per_strip = BSP_STRIP / bo;  // 2, 4 or 1
  const bool steps_wanted = dtype == BSP_BF16 || dtype == BSP_I8;
  // the step section's chunks are 16 bytes of input channels per pixel: 8 bf16 or 16 int8
  const int32_t scw = dtype == BSP_I8 ? 2 : 1;  // 8-channel chunks per step-section chunk
  const int32_t nsc = (int32_t)cdiv(nxc, scw);
  const int32_t slab_chunks = bsp_slab_channels(nsc * BSP_CHUNK, H, K) / BSP_CHUNK;
  const int32_t slab = slab_chunks * BSP_CHUNK * scw;  // channels
  const int32_t nslabs = (int32_t)cdiv(nsc, slab_chunks);

  std::vector<int32_t> src((size_t)nxc * BSP_MAXSUB);
  std::vector<int32_t> strip_ptr((size_t)nstrips + 1, 0);
  std::vector<int32_t> xc_list, src_list;
  std::vector<int32_t> sc_list, sc_ptr((size_t)nstrips + 1, 0);  // step-section chunks per strip
  std::vector<int32_t> slab_ptr;  // [nstrips][nslabs+1]
  int32_t max_chunks = 0, max_steps = 0, max_slab_steps = 0;
  int64_t nsteps = 0;
  for (int32_t t = 0; t < nstrips; ++t) {
    std::fill(src.begin(), src.end(), -1);
    for (int32_t s = 0; s < rows_per_strip; ++s) {
      const int64_t l = (int64_t)t * rows_per_strip + s;
      if (l >= nbr) break;
      for (int64_t n = row_ptr[l]; n < row_ptr[l + 1]; ++n) {
        const int32_t c = col_idx[n];
        const int32_t base = (int32_t)(n * blk_elems);
        if (bi == 8) {
          src[(size_t)c * BSP_MAXSUB + s] = base;
        } else if (bi == 16) {
          for (int32_t half = 0; half < 2; ++half) {
            const int32_t xc = 2 * c + half;
            if (xc < nxc) src[(size_t)xc * BSP_MAXSUB + s] = base + half * 8;
          }
        } else {  // bi == 4: two block columns share one 8-channel group
          src[(size_t)(c / 2) * BSP_MAXSUB + (c % 2)] = base;
        }
      }
    }
    int32_t count = 0;
    const int64_t strip_first_step = nsteps;
    int32_t next_slab = 0, in_slab = 0;
    auto close_slabs_upto = [&](int32_t sl) {  // finish slabs < sl
      while (next_slab < sl) {
        if (next_slab == 0) slab_ptr.push_back((int32_t)nsteps);
        const int64_t st = cdiv((int64_t)in_slab * HK, 4);
        if (st > max_slab_steps) max_slab_steps = (int32_t)st;
        nsteps += st;
        slab_ptr.push_back((int32_t)nsteps);
        in_slab = 0;
        ++next_slab;
      }
    };
    int32_t last_sc = -1;
    for (int32_t xc = 0; xc < nxc; ++xc) {
      const int32_t* e = &src[(size_t)xc * BSP_MAXSUB];
      if (e[0] < 0 && e[1] < 0 && e[2] < 0 && e[3] < 0) continue;
      xc_list.push_back(xc);
      src_list.insert(src_list.end(), e, e + BSP_MAXSUB);
      ++count;
      const int32_t sc = xc / scw;
      if (sc != last_sc) {
        close_slabs_upto(sc / slab_chunks);
        sc_list.push_back(sc);
        ++in_slab;
        last_sc = sc;
      }
    }
    close_slabs_upto(nslabs);
    sc_ptr[(size_t)t + 1] = (int32_t)sc_list.size();
    strip_ptr[(size_t)t + 1] = strip_ptr[t] + count;
    if (count > max_chunks) max_chunks = count;
    if (nsteps - strip_first_step > max_steps) max_steps = (int32_t)(nsteps - strip_first_step);
  }
  if (!steps_wanted) nsteps = 0;
  const int64_t nchunks = (int64_t)xc_list.size();
  auto pad4 = [](int64_t w) { return (w + 3) & ~int64_t(3); };
  const int64_t off_strip = BSP_PLAN_HEADER_WORDS;
  const int64_t off_xc = off_strip + pad4(nstrips + 1);
  const int64_t off_src = off_xc + pad4(nchunks);
  const int64_t off_slab = off_src + nchunks * BSP_MAXSUB;
  const int64_t off_xdesc = off_slab + (steps_wanted ? pad4((int64_t)nstrips * (nslabs + 1)) : 0);
  const int64_t off_wfrag = off_xdesc + nsteps * 4;
  // 16 bytes (four words) per lane and step; then the row-band section, 16-byte aligned
  const int64_t off_rows = (off_wfrag + nsteps * 64 * 4 + 3) & ~int64_t(3);
  std::vector<int32_t> rows;
  if (bsp_rows_wanted(O, H, K, I, bo, bi, dtype))
    if (int rc = bsp_rows_section(row_ptr, col_idx, out ? (const uint16_t*)payload : nullptr, O, H,
                                  K, I, bo, bi, &rows))
      return rc;
  const int64_t off_first = (off_rows + (int64_t)rows.size() + 3) & ~int64_t(3);
  std::vector<int32_t> first;
  if (bsp_first_wanted(O, H, K, I, bo, bi, dtype))
    if (int rc = bsp_first_section(row_ptr, col_idx, out ? (const uint16_t*)payload : nullptr, O, H,
                                   K, I, bo, bi, &first))
      return rc;
  const int64_t total = first.empty() ? off_rows + (int64_t)rows.size() : off_first + (int64_t)first.size();
  if (total > std::numeric_limits<int32_t>::max()) return BSP_ERR_SHAPE;
  if (words_needed) *words_needed = total;
  if (!out) return BSP_OK;
  if (capacity_words < total) return BSP_ERR_CAPACITY;
  if (steps_wanted && nnzb > 0 && !payload) return BSP_ERR_NULL;
  std::memset(out, 0, sizeof(int32_t) * (size_t)total);
  out[BSP_PLAN_MAGIC_W] = BSP_PLAN_MAGIC;
  out[BSP_PLAN_VERSION_W] = BSP_PLAN_VERSION;
  out[BSP_PLAN_O_W] = O;
  out[BSP_PLAN_I_W] = I;
  out[BSP_PLAN_H_W] = H;
  out[BSP_PLAN_K_W] = K;
  out[BSP_PLAN_BO_W] = bo;
  out[BSP_PLAN_BI_W] = bi;
  out[BSP_PLAN_NSTRIPS_W] = nstrips;
  out[BSP_PLAN_NCHUNKS_W] = (int32_t)nchunks;
  out[BSP_PLAN_OFF_STRIP_W] = (int32_t)off_strip;
  out[BSP_PLAN_OFF_XC_W] = (int32_t)off_xc;
  out[BSP_PLAN_OFF_SRC_W] = (int32_t)off_src;
  out[BSP_PLAN_TOTAL_W] = (int32_t)total;
  out[BSP_PLAN_MAXCHUNKS_W] = max_chunks;
  out[BSP_PLAN_DTYPE_W] = dtype;
  out[BSP_PLAN_SLAB_W] = slab;
  out[BSP_PLAN_NSLABS_W] = nslabs;
  out[BSP_PLAN_NSTEPS_W] = (int32_t)nsteps;
  out[BSP_PLAN_OFF_SLAB_W] = (int32_t)off_slab;
  out[BSP_PLAN_OFF_XDESC_W] = (int32_t)off_xdesc;
  out[BSP_PLAN_OFF_WFRAG_W] = (int32_t)off_wfrag;
  out[BSP_PLAN_MAXSTEPS_W] = steps_wanted ? max_steps : 0;
  out[BSP_PLAN_MAXSLABSTEPS_W] = steps_wanted ? max_slab_steps : 0;
  out[BSP_PLAN_OFF_ROWS_W] = rows.empty() ? 0 : (int32_t)off_rows;
  if (!rows.empty()) std::memcpy(out + off_rows, rows.data(), sizeof(int32_t) * rows.size());
  out[BSP_PLAN_OFF_FIRST_W] = first.empty() ? 0 : (int32_t)off_first;
  if (!first.empty()) std::memcpy(out + off_first, first.data(), sizeof(int32_t) * first.size());
  std::memcpy(out + off_strip, strip_ptr.data(), sizeof(int32_t) * strip_ptr.size());
  if (nchunks) {
    std::memcpy(out + off_xc, xc_list.data(), sizeof(int32_t) * xc_list.size());
    std::memcpy(out + off_src, src_list.data(), sizeof(int32_t) * src_list.size());
  }
  if (!steps_wanted) return BSP_OK;

  // Step section: re-order the kept weights into MFMA operand order.
  std::memcpy(out + off_slab, slab_ptr.data(), sizeof(int32_t) * slab_ptr.size());
  if (dtype == BSP_I8) {
    // int8 codes, 16-channel chunks: lane 16g + j of a step holds the sixteen codes
    // W[16*strip + j][tap][16*chunk .. 16*chunk + 15] of the step's pair g (or zeros).
    const int8_t* pl8 = (const int8_t*)payload;
    int32_t* xdesc = out + off_xdesc;
    int8_t* wfrag = (int8_t*)(out + off_wfrag);
    const int64_t Ipad = (int64_t)nsc * 16;
    std::vector<int8_t> dense((size_t)(BSP_STRIP * HK * Ipad));  // the strip's masked rows
    for (int32_t t = 0; t < nstrips; ++t) {
      std::fill(dense.begin(), dense.end(), (int8_t)0);
      for (int32_t s = 0; s < rows_per_strip; ++s) {
        const int64_t l = (int64_t)t * rows_per_strip + s;
        if (l >= nbr) break;
        for (int64_t n = row_ptr[l]; n < row_ptr[l + 1]; ++n)
          for (int64_t r = 0; r < bo; ++r)
            for (int64_t tp = 0; tp < HK; ++tp)
              std::memcpy(&dense[(size_t)(((s * bo + r) * HK + tp) * Ipad + (int64_t)col_idx[n] * bi)],
                          pl8 + n * blk_elems + (r * HK + tp) * bi, (size_t)bi);
      }
      int32_t e = sc_ptr[t];
      for (int32_t sl = 0; sl < nslabs; ++sl) {
        const int32_t e0 = e;
        while (e < sc_ptr[(size_t)t + 1] && sc_list[e] / slab_chunks == sl) ++e;
        const int64_t pairs = (int64_t)(e - e0) * HK;
        const int64_t s0 = slab_ptr[(size_t)t * (nslabs + 1) + sl];
        for (int64_t q = 0; q < pairs; ++q) {
          const int64_t step = s0 + q / 4;
          const int32_t g = (int32_t)(q % 4);
          const int32_t sc = sc_list[e0 + (int32_t)(q / HK)];
          const int32_t tap = (int32_t)(q % HK);
          xdesc[step * 4 + g] = (sc - sl * slab_chunks) | ((tap / K) << 16) | ((tap % K) << 24);
          for (int32_t j = 0; j < BSP_STRIP; ++j)
            std::memcpy(wfrag + ((step * 64) + g * 16 + j) * 16,
                        &dense[(size_t)((j * HK + tap) * Ipad + (int64_t)sc * 16)], 16);
        }
      }
    }
    return BSP_OK;
  }
  const uint16_t* pl = (const uint16_t*)payload;
  int32_t* xdesc = out + off_xdesc;
  uint16_t* wfrag = (uint16_t*)(out + off_wfrag);
  for (int32_t t = 0; t < nstrips; ++t) {
    int32_t e = strip_ptr[t];  // walks the strip's chunks in slab order
    for (int32_t sl = 0; sl < nslabs; ++sl) {
      const int32_t e0 = e;
      while (e < strip_ptr[(size_t)t + 1] && xc_list[e] / slab_chunks == sl) ++e;
      const int64_t pairs = (int64_t)(e - e0) * HK;
      const int64_t s0 = slab_ptr[(size_t)t * (nslabs + 1) + sl];
      for (int64_t q = 0; q < pairs; ++q) {
        const int64_t step = s0 + q / 4;
        const int32_t g = (int32_t)(q % 4);
        const int32_t ce = e0 + (int32_t)(q / HK);
        const int32_t tap = (int32_t)(q % HK);
        const int32_t xc = xc_list[ce];
        xdesc[step * 4 + g] = (xc - sl * slab_chunks) | ((tap / K) << 16) | ((tap % K) << 24);
        const int32_t* sr = &src_list[(size_t)ce * BSP_MAXSUB];
        for (int32_t j = 0; j < BSP_STRIP; ++j) {
          uint16_t* d = wfrag + ((step * 64) + g * 16 + j) * 8;
          if (bi >= 8) {
            const int32_t so = sr[j / bo];
            if (so >= 0) std::memcpy(d, pl + so + ((int64_t)(j % bo) * HK + tap) * bi, 16);
          } else {
            for (int32_t s = 0; s < 2; ++s)
              if (sr[s] >= 0)
                std::memcpy(d + 4 * s, pl + sr[s] + ((int64_t)j * HK + tap) * 4, 8);
          }
        }
      }
    }
  }
  return BSP_OK;
}

int bsp_plan_size(const int32_t* row_ptr, const int32_t* col_idx, int32_t O, int32_t H,
                  int32_t K, int32_t I, int32_t bo, int32_t bi, int32_t payload_dtype,
                  int64_t* bytes) {
  if (!bytes) return BSP_ERR_NULL;
  int64_t words = 0;
  if (int rc = plan_walk(row_ptr, col_idx, nullptr, payload_dtype, O, H, K, I, bo, bi, nullptr,
                         0, &words))
    return rc;
  *bytes = words * 4;
  return BSP_OK;
}

int bsp_plan_build(const int32_t* row_ptr, const int32_t* col_idx, const void* payload,
                   int32_t payload_dtype, int32_t O, int32_t H, int32_t K, int32_t I,
                   int32_t bo, int32_t bi, void* plan, int64_t capacity_bytes) {
  if (!plan) return BSP_ERR_NULL;
  return plan_walk(row_ptr, col_idx, payload, payload_dtype, O, H, K, I, bo, bi,
                   (int32_t*)plan, capacity_bytes / 4, nullptr);
}

}  // extern "C"
