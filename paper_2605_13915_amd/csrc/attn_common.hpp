// Shared pieces of the two attention-decode kernels (MSD over the INT8 cache, attn.hip; the
// dequantise-then-BF16 comparison kernel, attn_dequant.hip): launch parameters, the flash-decode
// split plan, the 16-lane row reductions and the partial-result merge.
#pragma once
#include "kernels.hpp"

namespace msd {

struct AttnParams {
  const uint16_t* q;
  const int8_t* K;
  const int8_t* V;
  const float* k_scale;
  const float* v_scale;
  const int32_t* kv_len;
  int B, Hq, Hkv, G;
  int64_t L;
  int nsplit;
  int64_t tokens_per_split;
  float* part_o;  // [B*Hkv][nsplit][G][128]
  float* part_m;  // [B*Hkv][nsplit][G]
  float* part_l;
  void* out;
  int out_bf16;
  int8_t* tap_q1;
  int8_t* tap_q2;
  float* tap_alpha;
  int32_t* tap_s1;
  int32_t* tap_s2;
  int8_t* tap_p1;  // codes of the decomposed softmax numerator [B][Hq][L] (nullable pair)
  int8_t* tap_p2;
};

constexpr int kD = 128;
constexpr int kTile = 64;
constexpr int kAttnWaves = 4;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ v4i mfma_s8(v4i a, v4i b, v4i c) {
  return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// All-reduce over the 16 lanes sharing lane/16 (one DPP row): four rotate-and-combine steps.
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, row16_ror<8>(v));
  v = fmaxf(v, row16_ror<4>(v));
  v = fmaxf(v, row16_ror<2>(v));
  return fmaxf(v, row16_ror<1>(v));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += row16_ror<8>(v);
  v += row16_ror<4>(v);
  v += row16_ror<2>(v);
  return v + row16_ror<1>(v);
}

// 4x4 byte transpose: in[t] = 4 channel bytes of token t; out[c] = 4 token bytes of channel c
__device__ __forceinline__ void transpose4x4(uint32_t a, uint32_t b, uint32_t c, uint32_t d,
                                             uint32_t (&o)[4]) {
  const uint32_t ab_lo = __builtin_amdgcn_perm(b, a, 0x05010400u);
  const uint32_t ab_hi = __builtin_amdgcn_perm(b, a, 0x07030602u);
  const uint32_t cd_lo = __builtin_amdgcn_perm(d, c, 0x05010400u);
  const uint32_t cd_hi = __builtin_amdgcn_perm(d, c, 0x07030602u);
  o[0] = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x05040100u);
  o[1] = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x07060302u);
  o[2] = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x05040100u);
  o[3] = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x07060302u);
}

// number of KV splits per (batch, KV head): about two workgroups per CU (measured best: 256 as good, 384 and
// 1024 worse), at least two rounds
// of the four waves per split
inline int attn_plan_nsplit(int B, int Hkv, int64_t L) {
  const int64_t pairs = (int64_t)B * Hkv;
  int64_t ns = cdiv(512, pairs);
  int64_t max_by_len = L / (kAttnWaves * kTile * 2);
  if (max_by_len < 1) max_by_len = 1;
  if (ns > max_by_len) ns = max_by_len;
  if (ns > 64) ns = 64;
  if (ns < 1) ns = 1;
  return (int)ns;
}

// fills the split plan, the partial-result pointers inside the workspace and the output fields of p
void attn_fill_params(const AttnArgs& a, AttnParams& p);
// launches the kernel instances for more than 8 query heads per KV head (attn_wide.hip)
int launch_attn_wide(const AttnParams& p, dim3 grid, bool per_token, bool lowprec, hipStream_t stream);
// merges the split partials into p.out (attn.hip); call only when p.nsplit > 1
int launch_attn_combine(const AttnParams& p, int per_channel, hipStream_t stream);

}  // namespace msd
