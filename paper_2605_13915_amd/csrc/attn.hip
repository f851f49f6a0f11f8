// MSD attention decode over an INT8 KV cache for gfx950 (paper Sec. 4.2, Alg. 3; tiling of
// Sec. 4.3; fused-kernel steps of Sec. 3.9 "Attention decode example").
//
// K and V stay INT8 from HBM to the matrix unit.  Per (batch, KV head) the G = Hq/Hkv query
// rows are decomposed once into two INT8 components each; per 64-token tile a wave
//   (1) loads K_t, V_t once,
//   (2) computes S1 = Q1 K_t^T and S2 = Q2 K_t^T on v_mfma_i32_16x16x64_i8 with the rows
//       [Q1; Q2] of all heads stacked in one A fragment,
//   (3) merges S = (alpha_Q S1 + beta_Q S2)/sqrt(d) (times s_K[t] for per-token scales),
//   (4) runs the online softmax in fp32 and decomposes P (times s_V[t]) with a scale that
//       needs no reduction over P,
//   (5) computes O1 = P1 V_t, O2 = P2 V_t on the same MFMA and rescales the running output.
// The KV length is split over workgroups (flash-decode); a small second kernel merges the
// (m, l, O) partials -- the only cross-workgroup step (skipped when there is one split).
//
// Layout tricks.  A-fragment row i = 4*(lane/16)+r carries (head, component), chosen so that
// S1 and S2 (and later O1 and O2) of one head land in registers of the same lane: the
// merges are register-local.  The contraction index of an MFMA may be permuted freely as
// long as both operands agree; for P.V the k slot (kg, 4*jq+tt) stands for token
// 16*tt + 4*kg + jq of the tile, which lets P travel as one packed dword per lane and lets V
// be brought into "token-contiguous" order by 4x4 byte transposes (v_perm_b32) in registers.
#include "attn_kernel.hpp"

namespace msd {

template <bool PER_TOKEN, bool LOWP>
static int launch_attn_for_group(const AttnParams& p, dim3 grid, hipStream_t stream) {
  if (p.G <= 4) return launch_attn_variant<1, PER_TOKEN, false, 1, LOWP>(p, grid, stream);
  if (p.G <= 8) return launch_attn_variant<2, PER_TOKEN, false, 1, LOWP>(p, grid, stream);
  return launch_attn_wide(p, grid, PER_TOKEN, LOWP, stream);
}

// Merge the split partials: out = sum_s O_s 2^(m_s - m*) / sum_s l_s 2^(m_s - m*)
// (times s_V per channel in per-channel mode; Alg. 3 last two steps).  A second launch: a
// release/acquire handshake inside the main kernel costs far more than the launch (every
// workgroup's agent-scope release fence forces an L2 write-back under the KV stream).
__global__ __launch_bounds__(kD) void attn_combine_kernel(AttnParams p, int per_channel) {
  const int row = blockIdx.x;  // b*Hq + hq
  const int b = row / p.Hq, hq = row % p.Hq;
  const int hk = hq / p.G, h = hq % p.G;
  const int c = threadIdx.x;
  const int64_t base = ((int64_t)(b * p.Hkv + hk) * p.nsplit) * p.G + h;
  float ms = -INFINITY;
  for (int s = 0; s < p.nsplit; ++s) ms = fmaxf(ms, p.part_m[base + (int64_t)s * p.G]);
  float o = 0.f, l = 0.f;
  for (int s = 0; s < p.nsplit; ++s) {
    const int64_t pr = base + (int64_t)s * p.G;
    const float mv = p.part_m[pr];
    const float wgt = (mv == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mv - ms);
    o += p.part_o[pr * kD + c] * wgt;
    l += p.part_l[pr] * wgt;
  }
  float v = l > 0.f ? __fdiv_rn(o, l) : 0.f;
  if (per_channel) v *= p.v_scale[hk * kD + c];
  if (p.out_bf16)
    reinterpret_cast<uint16_t*>(p.out)[(int64_t)row * kD + c] = f32_to_bf16_bits(v);
  else
    reinterpret_cast<float*>(p.out)[(int64_t)row * kD + c] = v;
}

size_t attn_workspace_bytes(int B, int Hq, int Hkv, int d, int64_t L) {
  (void)d;
  const int ns = attn_plan_nsplit(B, Hkv, L);
  const size_t rows = (size_t)B * Hq * ns;
  return align_up(rows * kD * 4, 256) + 2 * align_up(rows * 4, 256);
}

void attn_fill_params(const AttnArgs& a, AttnParams& p) {
  p.q = a.q; p.K = a.K; p.V = a.V;
  p.k_scale = a.k_scale; p.v_scale = a.v_scale;
  p.kv_len = a.kv_len;
  p.B = a.B; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
  p.L = a.L;
  p.nsplit = attn_plan_nsplit(a.B, a.Hkv, a.L);
  int64_t tps = cdiv(a.L > 0 ? a.L : 1, p.nsplit);
  tps = cdiv(tps, kAttnWaves * kTile) * (kAttnWaves * kTile);
  p.tokens_per_split = tps;
  const size_t rows = (size_t)a.B * a.Hq * p.nsplit;
  char* ws = (char*)a.workspace;
  p.part_o = (float*)ws;
  p.part_m = (float*)(ws + align_up(rows * kD * 4, 256));
  p.part_l = (float*)(ws + align_up(rows * kD * 4, 256) + align_up(rows * 4, 256));
  p.out = a.out;
  p.out_bf16 = a.out_bf16;
}

int launch_attn_combine(const AttnParams& p, int per_channel, hipStream_t stream) {
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)(p.B * p.Hq)), dim3(kD), 0, stream, p, per_channel);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

int launch_attn_decode(const AttnArgs& a, hipStream_t stream) {
  AttnParams p{};
  attn_fill_params(a, p);
  if (a.taps) {
    p.tap_q1 = (int8_t*)a.taps->q1;
    p.tap_q2 = (int8_t*)a.taps->q2;
    p.tap_alpha = (float*)a.taps->scale;
    p.tap_s1 = a.taps->acc1;
    p.tap_s2 = a.taps->acc2;
    if (!(p.tap_q1 && p.tap_q2 && p.tap_alpha)) p.tap_q1 = p.tap_q2 = nullptr, p.tap_alpha = nullptr;
    if (!(p.tap_s1 && p.tap_s2)) p.tap_s1 = p.tap_s2 = nullptr;
    p.tap_p1 = (int8_t*)a.taps->p1;
    p.tap_p2 = (int8_t*)a.taps->p2;
    if (!(p.tap_p1 && p.tap_p2)) p.tap_p1 = p.tap_p2 = nullptr;
  }
  const dim3 grid((unsigned)((int64_t)a.B * a.Hkv * p.nsplit));
  const bool per_token = a.scale_mode == MSD_PER_TOKEN;
  int rc;
  if (a.lowprec)
    rc = per_token ? launch_attn_for_group<true, true>(p, grid, stream) : launch_attn_for_group<false, true>(p, grid, stream);
  else
    rc = per_token ? launch_attn_for_group<true, false>(p, grid, stream) : launch_attn_for_group<false, false>(p, grid, stream);
  if (rc) return rc;
  if (p.nsplit > 1) return launch_attn_combine(p, per_token ? 0 : 1, stream);
  return MSD_OK;
}

}  // namespace msd
