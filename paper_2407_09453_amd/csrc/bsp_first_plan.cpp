// Host: the plan section of the thin-input kernel (bsp_first.hip), see bsp_plan.h.
// The weights of a layer with at most four input channels, in matrix-core operand order with
// the whole window as the contraction and the output channels interleaved over the strips.
#include "bsp.h"
#include "bsp_plan.h"

#include <cstring>
#include <vector>

bool bsp_first_wanted(int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi, int32_t dtype) {
  (void)bo;
  if (dtype != BSP_BF16) return false;
  if (I > 4 || I > bi) return false;  // one block column
  if (O % 16 != 0 || O / 16 > 8) return false;
  if (H > 7 || K > 7) return false;
  return true;
}

// Fills `sec` (words) with the section; with payload == nullptr the weights are left zero
// (the size is what the caller is after).
int bsp_first_section(const int32_t* row_ptr, const int32_t* col_idx, const uint16_t* payload,
                      int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                      std::vector<int32_t>* sec) {
  (void)col_idx;
  const int32_t NS = O / 16, Kt = H * K * I, steps = (Kt + 31) / 32;
  const size_t frag_words = (size_t)steps * NS * 64 * 4;
  sec->assign(BSP_FIRST_HEADER_WORDS + frag_words, 0);
  int32_t* h = sec->data();
  h[BSP_FIRST_NS_W] = NS;
  h[BSP_FIRST_STEPS_W] = steps;
  h[BSP_FIRST_KT_W] = Kt;
  h[BSP_FIRST_OFF_FRAG_W] = BSP_FIRST_HEADER_WORDS;
  if (!payload) return BSP_OK;
  uint16_t* frag = (uint16_t*)(h + BSP_FIRST_HEADER_WORDS);
  const int64_t HK = (int64_t)H * K;
  for (int32_t t = 0; t < steps; ++t)
    for (int32_t s = 0; s < NS; ++s)
      for (int32_t lane = 0; lane < 64; ++lane) {
        const int32_t g = lane >> 4, j = lane & 15;
        const int32_t ch = (j >> 2) * 4 * NS + 4 * s + (j & 3);
        const int32_t l = ch / bo;  // its block row: kept when the row holds its one block
        if (row_ptr[l + 1] == row_ptr[l]) continue;
        const int64_t n = row_ptr[l];
        uint16_t* dst = frag + (((size_t)t * NS + s) * 64 + lane) * 8;
        for (int32_t e = 0; e < 8; ++e) {
          const int32_t k = 32 * t + 8 * g + e;
          if (k >= Kt) continue;
          const int32_t tap = k / I, i = k % I;
          dst[e] = payload[((n * bo + ch % bo) * HK + tap) * bi + i];
        }
      }
  return BSP_OK;
}
