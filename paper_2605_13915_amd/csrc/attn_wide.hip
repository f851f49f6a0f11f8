// Instances of the MSD attention-decode kernel for more than 8 query heads per KV head: 16 or 24 heads
// per pass over the KV tiles (one wave per SIMD), larger groups in passes of 16.
#include "attn_kernel.hpp"

namespace msd {

template <bool PER_TOKEN, bool LOWP>
static int launch_attn_wide_mode(const AttnParams& p, dim3 grid, hipStream_t stream) {
  if (p.G <= 16) return launch_attn_variant<2, PER_TOKEN, false, 2, LOWP>(p, grid, stream);
  if (p.G <= 24) return launch_attn_variant<2, PER_TOKEN, false, 3, LOWP>(p, grid, stream);
  return launch_attn_variant<2, PER_TOKEN, true, 2, LOWP>(p, grid, stream);  // passes of 16 heads (24 would spill)
}

int launch_attn_wide(const AttnParams& p, dim3 grid, bool per_token, bool lowprec, hipStream_t stream) {
  if (lowprec)
    return per_token ? launch_attn_wide_mode<true, true>(p, grid, stream) : launch_attn_wide_mode<false, true>(p, grid, stream);
  return per_token ? launch_attn_wide_mode<true, false>(p, grid, stream) : launch_attn_wide_mode<false, false>(p, grid, stream);
}

}  // namespace msd
