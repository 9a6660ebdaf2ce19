// Attention for configurations with long key ranges (bf16, head width 64; the host selects it from the key capacity,
// kLongKeys and more): a chunk of up to 64 query rows that sees 129..512 keys goes to the body in which the four waves
// split the keys for all its row tiles (attn_split_tiles), everything else to the generic body (attn_block).
// A source file, hence a code object, of its own: the attention kernels are larger than the instruction cache, and the
// speed of the short-range ones, which are the batch-1 path, moved with every addition to their code object although
// their own instructions stayed the same (0.5 us per launch at 1152 rows).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "ad_device.h"

namespace ad {

__global__ __launch_bounds__(256) void k_attention_long(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb,
                                                        const bf16_t* __restrict__ Vb, bf16_t* __restrict__ out,
                                                        const SeqDesc* __restrict__ desc, int d, float scale, int nk_cap) {
  extern __shared__ unsigned att_long_lds[];
  const SeqDesc sd = desc[blockIdx.x];
  const int row_begin = blockIdx.z * 64;
  if (row_begin >= sd.nq) return;
  const int row_end = min(sd.nq, row_begin + 64);
  const int nk_all = sd.causal ? sd.nk_base + row_end : sd.nk_base;
  if (nk_all > 128 && nk_all <= 512) {
    attn_split_tiles(q, Kb, Vb, out, sd, row_begin, row_end, blockIdx.y, d, scale, nk_all, (bf16_t*)att_long_lds);
    return;
  }
  attn_block<bf16_t, 64, true>(q, Kb, Vb, out, sd, row_begin, row_end, blockIdx.y, d, scale, att_long_lds, nk_cap);
}

void launch_attention_long(const void* q, const void* K, const void* V, void* out, const SeqDesc* desc, dim3 grid, int d,
                           float scale, int max_keys, size_t lds_bytes, hipStream_t s) {
  static size_t set_for = 0;
  if (lds_bytes > set_for) {
    (void)hipFuncSetAttribute((const void*)k_attention_long, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    set_for = lds_bytes;
  }
  k_attention_long<<<grid, 256, lds_bytes, s>>>((const bf16_t*)q, (const bf16_t*)K, (const bf16_t*)V, (bf16_t*)out, desc, d, scale,
                                               max_keys);
}

// Cross-attention with its query projection for a source capacity of kLongKeys or more (head width 64, d 512 or 1024,
// bf16: launch_crossq_attention has checked that and chosen the rows per workgroup).  One row tile per workgroup: the
// waves split the keys (k_crossq_attention_split); several: every wave walks all keys with the four accumulators
// (k_crossq_attention<.., LONGK = true>).  false: the tiles do not fit in LDS, the caller launches projection and
// attention separately.
bool launch_crossq_attention_long(const LnA& ln, const void* A, const void* W, const float* bias, const void* K, const void* V,
                                  void* out, const SeqDesc* desc, int n_seq, int max_rows, int H, int chunk, int max_keys,
                                  hipStream_t s) {
  const int d = H * 64;
  const int mt = (std::min(max_rows, chunk) + 15) / 16;
  const float scale = 1.0f / sqrtf(64.0f);
  if (mt == 1 && 16 * (size_t)(d + 16) * 2 <= 4 * (size_t)kSplitWaveElems * 2) {
    if (n_seq <= 0 || max_rows <= 0) return true;
    const size_t shs = crossq_split_lds_bytes();
    dim3 g(n_seq, H, (max_rows + 15) / 16);
    auto go = [&](auto nv_c) {
      constexpr int NV = decltype(nv_c)::value;
      static bool set = false;
      if (!set) {
        (void)hipFuncSetAttribute((const void*)k_crossq_attention_split<NV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shs);
        set = true;
      }
      k_crossq_attention_split<NV><<<g, 256, shs, s>>>(desc, scale, (const bf16_t*)W, (const bf16_t*)K, (const bf16_t*)V, ln.x, ln.g,
                                                       ln.b, ln.y, (const bf16_t*)A, bias, (bf16_t*)out);
    };
    if (d == 512) go(std::integral_constant<int, 2>{});
    else go(std::integral_constant<int, 4>{});
    return true;
  }
  const size_t sh = crossq_lds_bytes(max_keys, mt, d);
  if (sh > 160 * 1024) return false;
  if (n_seq <= 0 || max_rows <= 0) return true;
  dim3 g(n_seq, H, (max_rows + chunk - 1) / chunk);
  auto go = [&](auto nv_c) {
    constexpr int NV = decltype(nv_c)::value;
    static size_t set_for = 0;
    if (sh > set_for) {
      (void)hipFuncSetAttribute((const void*)k_crossq_attention<NV, 0, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
      set_for = sh;
    }
    k_crossq_attention<NV, 0, true><<<g, 256, sh, s>>>(desc, chunk, scale, (const bf16_t*)W, (const bf16_t*)K, (const bf16_t*)V,
                                                           ln.x, ln.g, ln.b, ln.y, (const bf16_t*)A, bias, (bf16_t*)out);
  };
  if (d == 512) go(std::integral_constant<int, 2>{});
  else go(std::integral_constant<int, 4>{});
  return true;
}

}  // namespace ad
