// MSD attention decode over an INT8 latent KV cache (multi-head latent attention; paper Sec. 4.2 /
// Alg. 3 with the shapes of Sec. 4.4 and Sec. 7.3: 512 latent channels plus 64 positional ones).
// One cached row per token serves every query head of a batch entry: its 576 channels are the key,
// its first 512 the value.  The steps are those of the grouped-query kernel (attn.hip) -- Q rows
// decomposed once, S1 / S2 on v_mfma_i32_16x16x64_i8 with [Q1; Q2] stacked, merge, online softmax in
// fp32, P decomposed with a scale that needs no reduction over P, O1 / O2 on the same instruction --
// reshaped around the one thing that differs: every head reads the same rows, so a tile of the cache
// is fetched once and shared.
//   * A 64-token tile (36 KB) goes global -> registers -> LDS with fully coalesced 16-byte loads,
//     fetched one tile ahead of its use; the key fragments (nine 64-channel chunks) and the value
//     fragments (16-channel blocks, through the transposing LDS read) both come from that LDS copy,
//     so HBM sees each cached row once per workgroup.  Both fragment streams are software-pipelined
//     by hand (reads a few fragments ahead of the MFMAs, MFMAs one step ahead of the merge).
//   * The query rows of a workgroup are decomposed in its prologue, all loads of a wave in flight at once,
//     straight into the A-fragment image in LDS (under the first tile fetches); with 64 heads per workgroup
//     that costs more than a launch, and a small kernel decomposes all rows once.  A wave owns 8 MG query
//     heads (MG 16-row A fragments: 8 heads x 2 components each) and keeps their running output in
//     registers, in units of alpha_P / 254 so that a tile contributes the exact integer 254 O1 + O2.
//   * The NW waves of a workgroup are laid out as HGW head groups x CH parts of the value channels x
//     TS token streams (HGW*CH*TS = NW); waves that split the value channels both compute the (cheap)
//     score product.  In use (MG = 1, NW = 8, two waves per SIMD):
//       up to 16 heads: 2 x 2 x 2,   up to 32 heads: 4 x 2 x 1,
//       more:           8 x 1 x 1, 64 heads per workgroup, further heads over blockIdx.y.
//   * One workgroup per CU; the KV length is split over workgroups and over the token streams inside
//     one; the streams of a workgroup merge through LDS at the end, every split writes one partial
//     (m, l, O) and a last kernel merges the splits.
#include <algorithm>
#include <type_traits>

#include "attn_common.hpp"
#include "decompose_int8_dev.hpp"

namespace msd {

namespace {

constexpr int kLatK = 576;    // key channels (latent + positional)
constexpr int kLatV = 512;    // value channels (latent)
// LDS image of a tile, laid out for the way the LDS serves a wave (measured with two-lane probes and the
// bank-conflict counter): a 16-byte read is served 16 lanes at a time, and the lanes served together are the
// 4-lane groups {0,3,5,6}, {1,2,4,7} (and the same +8) of the wave -- not 16 consecutive lanes; a 16-byte
// write goes 8 consecutive lanes at a time.  Row r (576 bytes, no padding: consecutive rows then fall into
// complementary halves of the banks for the writes) starts at 576 r + 16 E(r / 16), E = 0, 2, 8, 10, and its
// 16-byte columns are stored at column ^ ((-(r / 4)) & 3).  With that, the key reads (lane = token row r,
// column group g) of one service group cover all 64 banks exactly once, and the eight source rows of a
// transposing value read (16 apart, which the pitch alone would put on one bank) spread too.
constexpr int kPitch = 576;
constexpr int kTileBytes = kTile * kPitch + 192;
__device__ __forceinline__ int tile_row(int r) { return r * kPitch + 32 * ((r >> 4) & 1) + 128 * (r >> 5); }
__device__ __forceinline__ int tile_swz(int r) { return (-(r >> 2)) & 3; }

struct MlaParams {
  const uint16_t* q;   // [B][Hq][576]
  const int8_t* C;     // [B][L][ld]
  const float* scale;  // per token [B][L] or per channel [576]
  const int32_t* kv_len;
  int B, Hq;
  int64_t L, ld;
  int nsplit;  // workgroups along the KV length
  int nparts;  // partial results per (batch, head): one per KV split
  int64_t tokens_per_split;
  float sm_scale_log2;  // score scale times log2(e)
  int8_t* qc1;          // [B][Hq][576] query codes of both components and alpha_Q [B][Hq] (workspace; only
  int8_t* qc2;          // used by the layout that leaves the query decomposition to its own kernel)
  float* qalpha;
  float* part_o;        // [B][nparts][Hq][512]
  float* part_m;        // [B][nparts][Hq]
  float* part_l;
  void* out;
  int out_bf16;
  int8_t* tap_q1;
  int8_t* tap_q2;
  float* tap_alpha;
  int32_t* tap_s1;
  int32_t* tap_s2;
};

template <int MG, int NW, int HGW, int CH>
struct MlaCfg {
  static constexpr int kTS = NW / (HGW * CH);          // token streams
  static constexpr int kWS = HGW * CH;                 // waves sharing a tile
  static constexpr int kSlabs = 4 / CH;                // 128-channel value slabs per wave
  static constexpr int kLanesRow = kWS;                 // lanes of the stream's 64 kWS that fetch one cached row
  static constexpr int kLoads = (36 + kLanesRow - 1) / kLanesRow;  // 16-byte pieces per lane per tile
  static constexpr int kHeadsWave = 8 * MG;
  static constexpr int kHeadsWg = kHeadsWave * HGW;
  // tiles[streams][2] | sP[waves][MG frag][2 comp][8 heads][16] u32 | sAlpha[heads] |
  // sQ[HGW][MG][9 chunks][64 lanes][16 B]: the A fragments (over the tiles when they end up in registers)
  static constexpr bool kQReg = HGW <= 2;  // A fragments in registers: their LDS image is only a staging area
  static constexpr size_t kLds = (size_t)2 * kTS * kTileBytes + NW * MG * 2 * 8 * 64 + kHeadsWg * 4 +
                                 (kQReg ? 0 : HGW * MG * 9 * 1024);
  static_assert(kTS * kWS == NW && kTS >= 1, "wave layout");
  static_assert(kLds <= 160 * 1024, "LDS");
};

// Alg. 3 steps 1-2 for the query rows as a kernel of its own, one wave per (batch, head) row; the per-channel
// key scale, if any, is absorbed into the row first.  Used with the 64-heads-per-workgroup layout, where the
// prologue version would spend more vector-ALU time per CU (8 heads per wave, every KV split again) than this
// launch costs; codes and alpha_Q go to the workspace, where the main kernel picks up its A fragments.
__global__ __launch_bounds__(256) void mla_q_decompose_kernel(MlaParams p, int per_channel) {
  const int lane = threadIdx.x & 63;
  const int64_t qrow = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (qrow >= (int64_t)p.B * p.Hq) return;
  // a lane takes channels 4 lane .. +3 of the two 256-channel blocks and, lanes 0..15, of the last 64
  const uint16_t* src = p.q + qrow * kLatK + 4 * lane;
  float x[3][4];
  float mx = 0.f;
#pragma unroll
  for (int bi = 0; bi < 3; ++bi) {
    const v2i w2 = (bi < 2 || lane < 16) ? *reinterpret_cast<const v2i*>(src + 256 * bi) : v2i{0, 0};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = (uint32_t)w2[e >> 1];
      x[bi][e] = (e & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
      if (per_channel) x[bi][e] *= p.scale[min(256 * bi + 4 * lane + e, kLatK - 1)];
      mx = fmaxf(mx, fabsf(x[bi][e]));
    }
  }
  mx = wave_max(mx);
  const float alpha = mx > 0.f ? __fdiv_rn(mx, 127.0f) : 0.f;
  const float beta = __fdiv_rn(alpha, 254.0f);
  // reciprocal route with exact-division fallback (same codes); needs a normal beta
  const bool fast = beta >= 1.17549435e-38f;
  const float ra = fast ? __fdiv_rn(1.0f, alpha) : 0.f, rb = fast ? __fdiv_rn(1.0f, beta) : 0.f;
#pragma unroll
  for (int bi = 0; bi < 3; ++bi) {
    uint32_t w1 = 0, w2 = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int c1 = 0, c2 = 0;
      if (fast)
        int8_codes_fast(x[bi][e], alpha, ra, beta, rb, c1, c2);
      else if (mx > 0.f)
        int8_codes(x[bi][e], alpha, beta, c1, c2);
      w1 |= ((uint32_t)c1 & 0xFFu) << (8 * e);
      w2 |= ((uint32_t)c2 & 0xFFu) << (8 * e);
    }
    if (bi < 2 || lane < 16) {
      const int64_t at = qrow * kLatK + 256 * bi + 4 * lane;
      *reinterpret_cast<uint32_t*>(p.qc1 + at) = w1;
      *reinterpret_cast<uint32_t*>(p.qc2 + at) = w2;
      if (p.tap_q1) {
        *reinterpret_cast<uint32_t*>(p.tap_q1 + at) = w1;
        *reinterpret_cast<uint32_t*>(p.tap_q2 + at) = w2;
      }
    }
  }
  if (lane == 0) {
    p.qalpha[qrow] = alpha;
    if (p.tap_q1) p.tap_alpha[qrow] = alpha;
  }
}

template <bool PER_TOKEN, int MG, int NW, int HGW, int CH>
__global__ __launch_bounds__(NW * 64) void attn_mla_kernel(MlaParams p) {
  using Cfg = MlaCfg<MG, NW, HGW, CH>;
  constexpr int TS = Cfg::kTS, WS = Cfg::kWS, NSL = Cfg::kSlabs, NLD = Cfg::kLoads;
  extern __shared__ __attribute__((aligned(16))) uint8_t s_mla[];
  uint8_t* sTiles = s_mla;
  constexpr bool QREG = Cfg::kQReg;
  uint32_t(*sP)[MG][2][8][16] = reinterpret_cast<uint32_t(*)[MG][2][8][16]>(s_mla + 2 * TS * kTileBytes);
  float* sAlpha = reinterpret_cast<float*>(s_mla + 2 * TS * kTileBytes + NW * MG * 2 * 8 * 64);
  v4i* sQ = reinterpret_cast<v4i*>(QREG ? s_mla : s_mla + 2 * TS * kTileBytes + NW * MG * 2 * 8 * 64 + Cfg::kHeadsWg * 4);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int ts = wave / WS, hg = (wave / CH) % HGW, ch = wave % CH;
  const int b = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
  const int Hq = p.Hq;
  const int hb = blockIdx.y * Cfg::kHeadsWg;  // first head of this workgroup
  const int hw = hb + Cfg::kHeadsWave * hg;    // first head of this wave
  int64_t len = p.kv_len ? (int64_t)p.kv_len[b] : p.L;
  len = max((int64_t)0, min(len, p.L));
  const int64_t t_begin = (int64_t)split * p.tokens_per_split;
  const int64_t t_end = min(len, t_begin + p.tokens_per_split);
  const int64_t last = max(t_end - 1, (int64_t)0);
  const int8_t* Cb = p.C + (int64_t)b * p.L * p.ld;
  const float* sc_tok = p.scale + (int64_t)b * p.L;  // per-token mode only
  const v4i zero4 = {0, 0, 0, 0};
  uint8_t* tiles2 = sTiles + 2 * ts * kTileBytes;  // this stream's two tile buffers: tile k lives in buffer k & 1
  const int n_iter = (int)((max(t_end - t_begin, (int64_t)0) + TS * kTile - 1) / (TS * kTile));  // same for every wave

  // A-fragment row of this lane: slot j&3 of head pair j>>2 = (head, component)
  const int slot = j & 3;
  const int row_head = (j >> 2) * 2 + (slot >> 1);
  const int row_comp = slot & 1;

  // ---- tile fetch, two tiles ahead of their use (two register sets).  The 64 WS lanes of a stream take one
  // cached row per WS lanes: a lane fetches the 16-byte pieces fcol, fcol + WS, ... of its row, so the loads of a
  // lane share one base address and the LDS image needs no index arithmetic.  Fetches and LDS writes are
  // unconditional (rows past the end repeat the last valid one): straight-line code lets the compiler count
  // the loads in flight exactly, so the wait before an LDS write covers its own tile only.
  constexpr int LPR = Cfg::kLanesRow;
  const int frow = ((wave % WS) * 64 + lane) / LPR, fcol = ((wave % WS) * 64 + lane) % LPR;
  v4i G[2][NLD];
  auto fetch = [&](auto bufc, int it) __attribute__((always_inline)) {
    constexpr int BUF = decltype(bufc)::value;
    const int64_t t0 = t_begin + ((int64_t)it * TS + ts) * kTile;
    const int8_t* src = Cb + min(t0 + frow, last) * p.ld + 16 * fcol;
#pragma unroll
    for (int i = 0; i < NLD; ++i)
      if (36 % LPR == 0 || fcol + LPR * i < 36) G[BUF][i] = *reinterpret_cast<const v4i*>(src + 16 * LPR * i);
  };
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;
  if (n_iter > 0) {
    fetch(Buf0{}, 0);
    fetch(Buf1{}, 1);
  }

  // ---- Alg. 3 steps 1-2 for the query rows of this workgroup: a wave decomposes kHeadsWg / NW heads (all
  // their loads in flight at once) and writes the codes straight into the A-fragment image in LDS:
  // fragment (head group, chunk s) holds, for lane (g', j'), the 16 channels 64 s + 16 g' .. of fragment
  // row j' = (head pair, head in pair, component).  The per-channel key scale, if any, is absorbed first.
  // (Up to 32 heads per workgroup; with 64 the decomposition is a launch of its own, see mla_q_decompose_kernel.)
  constexpr bool QFUSED = Cfg::kHeadsWg <= 32;
  if (QFUSED) {
    constexpr int HPW = Cfg::kHeadsWg / NW;
    static_assert(HPW * NW == Cfg::kHeadsWg, "heads per wave");
    // a lane takes channels 4 lane .. +3 of the two 256-channel blocks and, lanes 0..15, of the last 64
    v2i xr[HPW][3];
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
      const int head = min(hb + wave + NW * u, Hq - 1);  // rows past Hq: results unused
      const uint16_t* qsrc16 = p.q + ((int64_t)b * Hq + head) * kLatK + 4 * lane;
#pragma unroll
      for (int bi = 0; bi < 3; ++bi)
        xr[u][bi] = (bi < 2 || lane < 16) ? *reinterpret_cast<const v2i*>(qsrc16 + 256 * bi) : v2i{0, 0};
    }
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
      const int hl = wave + NW * u;  // head within the workgroup
      float x[3][4];
      float mx = 0.f;
#pragma unroll
      for (int bi = 0; bi < 3; ++bi)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t w = (uint32_t)xr[u][bi][e >> 1];
          x[bi][e] = (e & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
          if (!PER_TOKEN) x[bi][e] *= p.scale[min(256 * bi + 4 * lane + e, kLatK - 1)];
          mx = fmaxf(mx, fabsf(x[bi][e]));
        }
      mx = wave_max(mx);
      const float alpha = mx > 0.f ? __fdiv_rn(mx, 127.0f) : 0.f;
      const float beta = __fdiv_rn(alpha, 254.0f);
      // reciprocal route with exact-division fallback (same codes); needs a normal beta
      const bool fast = beta >= 1.17549435e-38f;
      const float ra = fast ? __fdiv_rn(1.0f, alpha) : 0.f, rb = fast ? __fdiv_rn(1.0f, beta) : 0.f;
      const int hq = hl % 8;  // head within its A fragment
      const int jrow = 4 * (hq >> 1) + 2 * (hq & 1);
      // channel 256 bi + 4 lane: chunk 4 bi + lane / 16, column group (lane & 15) / 4, bytes 4 (lane & 3) ..
      uint8_t* frag = reinterpret_cast<uint8_t*>(sQ) + (size_t)(hl / 8) * 9 * 1024 + (lane >> 4) * 1024 +
                      (((lane & 15) >> 2) * 16 + jrow) * 16 + 4 * (lane & 3);
      const bool tap = p.tap_q1 && split == 0 && hb + hl < Hq;
      const int64_t qrow = (int64_t)b * Hq + hb + hl;
#pragma unroll
      for (int bi = 0; bi < 3; ++bi) {
        uint32_t w1 = 0, w2 = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int c1 = 0, c2 = 0;
          if (fast)
            int8_codes_fast(x[bi][e], alpha, ra, beta, rb, c1, c2);
          else if (mx > 0.f)
            int8_codes(x[bi][e], alpha, beta, c1, c2);
          w1 |= ((uint32_t)c1 & 0xFFu) << (8 * e);
          w2 |= ((uint32_t)c2 & 0xFFu) << (8 * e);
        }
        if (bi < 2 || lane < 16) {
          *reinterpret_cast<uint32_t*>(frag + bi * 4096) = w1;
          *reinterpret_cast<uint32_t*>(frag + bi * 4096 + 16) = w2;
          if (tap) {
            *reinterpret_cast<uint32_t*>(p.tap_q1 + qrow * kLatK + 256 * bi + 4 * lane) = w1;
            *reinterpret_cast<uint32_t*>(p.tap_q2 + qrow * kLatK + 256 * bi + 4 * lane) = w2;
          }
        }
      }
      if (lane == 0) {
        sAlpha[hl] = alpha;
        if (tap) p.tap_alpha[qrow] = alpha;
      }
    }
  }
  if (!QFUSED) {  // codes and alpha_Q come from mla_q_decompose_kernel
#pragma unroll
    for (int mg = 0; mg < MG; ++mg) {
      if (ts == 0 && ch == 0) {
        const int64_t qrow = (int64_t)b * Hq + min(hw + 8 * mg + row_head, Hq - 1);  // rows past Hq: results unused
        const int8_t* src = (row_comp ? p.qc2 : p.qc1) + qrow * kLatK + 16 * g;
#pragma unroll
        for (int sc = 0; sc < 9; ++sc)
          sQ[((hg * MG + mg) * 9 + sc) * 64 + lane] = *reinterpret_cast<const v4i*>(src + 64 * sc);
      }
    }
    if (tid < Cfg::kHeadsWg) sAlpha[tid] = p.qalpha[(int64_t)b * Hq + min(hb + tid, Hq - 1)];
  }
  __syncthreads();
  float aq[MG][2], bq[MG][2];
#pragma unroll
  for (int mg = 0; mg < MG; ++mg)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      aq[mg][hh] = sAlpha[Cfg::kHeadsWave * hg + 8 * mg + g * 2 + hh];
      bq[mg][hh] = __fdiv_rn(aq[mg][hh], 254.0f);
    }
  // with registers to spare (few head groups) the fragments stay in registers instead
  v4i qreg[MG][QREG ? 9 : 1];
  if (QREG) {
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
      for (int sc = 0; sc < 9; ++sc) qreg[mg][QREG ? sc : 0] = sQ[((hg * MG + mg) * 9 + sc) * 64 + lane];
    __syncthreads();  // the staging area is tile memory from here on
  }
  const v4i* qsrc = sQ + (hg * MG * 9) * 64 + lane;  // fragment (mg, s) at qsrc[(mg * 9 + s) * 64]

  float m_run[MG][2], l_run[MG][2], o_run[MG][NSL][2][8];  // o_run[mg][slab][hh][c]: head 8 mg + 2 g + hh, channel 128 slab + 16 c + j
  float unit = 0.f;                   // 0: no coded tile yet
  float top = PER_TOKEN ? 0.f : 1.f;  // bound on P (times the value scale) behind alpha_P
#pragma unroll
  for (int mg = 0; mg < MG; ++mg)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      m_run[mg][hh] = -INFINITY;
      l_run[mg][hh] = 0.f;
#pragma unroll
      for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
        for (int c = 0; c < 8; ++c) o_run[mg][sl][hh][c] = 0.f;
    }

  // LDS holds two tiles per stream, so a step needs one workgroup barrier: after it tile `it` is visible and
  // nobody reads tile it - 1 any more, whose buffer then takes tile it + 1 from the registers while the loads
  // of tiles it + 2 and it + 3 are in flight.
  auto stage = [&](auto bufc, int k) __attribute__((always_inline)) {  // registers of tile k -> LDS buffer k & 1
    constexpr int BUF = decltype(bufc)::value;
    uint8_t* dst = tiles2 + BUF * kTileBytes + tile_row(frow) + 16 * (fcol ^ tile_swz(frow));  // LPR is a multiple of 4
#pragma unroll
    for (int i = 0; i < NLD; ++i)
      if (36 % LPR == 0 || fcol + LPR * i < 36) *reinterpret_cast<v4i*>(dst + 16 * LPR * i) = G[BUF][i];
    fetch(bufc, k + 2);
  };
  auto step = [&](auto bufc, int it) __attribute__((always_inline)) {  // bufc: buffer of tile it + 1
    constexpr int BUF = decltype(bufc)::value;
    const uint8_t* tile = tiles2 + (1 - BUF) * kTileBytes;
    const int64_t t0 = t_begin + ((int64_t)it * TS + ts) * kTile;
    const bool tile_live = t0 < t_end;  // uniform over the waves of a stream
    __syncthreads();
    // the token scales of this tile: issued ahead of the next fetch, first used after the score product
    float sk[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) sk[tt] = PER_TOKEN ? sc_tok[min(t0 + 16 * tt + j, last)] : 1.f;
    stage(bufc, it + 1);
    __builtin_amdgcn_sched_barrier(0);
    if (!tile_live) return;

    bool live[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) live[tt] = t0 + 16 * tt + j < t_end;
    // ---- (2) S1, S2 over the nine 64-channel chunks; a key fragment serves both A fragments
    v4i sd[MG][4];
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) sd[mg][tt] = zero4;
    {
      // software pipeline over the 36 (chunk, token group) fragments: LDS reads three fragments ahead
      constexpr int NKF = 36, DEPTH = 4;
      v4i kf[DEPTH];
      v4i qf[2][MG];  // A fragments of the current and the next 64-channel chunk
      const uint8_t* ksrc = tile + j * kPitch + 16 * (g ^ tile_swz(j));  // rows 16 tt + j share the swizzle of j
      auto kload = [&](int i) __attribute__((always_inline)) {
        kf[i % DEPTH] = *reinterpret_cast<const v4i*>(ksrc + tile_row(16 * (i % 4)) + 64 * (i / 4));
      };
      auto qload = [&](int sc) __attribute__((always_inline)) {
#pragma unroll
        for (int mg = 0; mg < MG; ++mg) qf[sc & 1][mg] = QREG ? qreg[mg][sc] : qsrc[(mg * 9 + sc) * 64];
      };
      qload(0);
#pragma unroll
      for (int i = 0; i < DEPTH - 1; ++i) kload(i);
#pragma unroll
      for (int i = 0; i < NKF; ++i) {
        if (i + DEPTH - 1 < NKF) kload(i + DEPTH - 1);
        if (i % 4 == 0 && i / 4 + 1 < 9) qload(i / 4 + 1);
#pragma unroll
        for (int mg = 0; mg < MG; ++mg) sd[mg][i % 4] = mfma_s8(qf[(i / 4) & 1][mg], kf[i % DEPTH], sd[mg][i % 4]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (p.tap_s1 && ch == 0) {
#pragma unroll
      for (int mg = 0; mg < MG; ++mg)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int head = hw + 8 * mg + g * 2 + hh;
          if (head < Hq) {
            const int64_t row = ((int64_t)b * Hq + head) * p.L;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
              if (live[tt]) {
                p.tap_s1[row + t0 + 16 * tt + j] = sd[mg][tt][2 * hh];
                p.tap_s2[row + t0 + 16 * tt + j] = sd[mg][tt][2 * hh + 1];
              }
          }
        }
    }
    // scale of the P decomposition: alpha_P = top/127, top a bound on P (times the value scale): the largest
    // value scale this wave has met so far (the untiled algorithm takes the largest of all tokens; a running
    // maximum is never coarser than that and, being monotone, only ever shrinks the running output below)
    float sv[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) sv[tt] = live[tt] ? sk[tt] : 0.f;
    if (PER_TOKEN) top = fmaxf(top, row16_max(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]))));
    const bool coded = top > 1e-30f;  // below that every code of the tile is zero
    const float to_code = coded ? __fdiv_rn(127.0f, top) : 0.f;
    // The running output is kept in units of `unit` = alpha_P / 254, so that a tile's contribution is the
    // integer 254 O1 + O2 itself; a growing alpha_P rescales the running output (by a factor <= 1) together
    // with the softmax correction.
    float rescale = 1.f;
    if (coded) {
      const float unit_new = top * (1.0f / (127.0f * 254.0f));
      rescale = unit > 0.f ? __fdiv_rn(unit, unit_new) : 0.f;  // nothing accumulated before the first coded tile
      unit = unit_new;
    }
    // ---- (3)+(4) merge, online softmax, decompose P
    float corr[MG][2];
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        float s[4];
        float mx = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const float v = (aq[mg][hh] * (float)sd[mg][tt][2 * hh] + bq[mg][hh] * (float)sd[mg][tt][2 * hh + 1]) *
                          (p.sm_scale_log2 * sk[tt]);
          s[tt] = live[tt] ? v : -INFINITY;
          mx = fmaxf(mx, s[tt]);
        }
        mx = row16_max(mx);
        const float m_new = fmaxf(m_run[mg][hh], mx);
        const float cr = __builtin_amdgcn_exp2f(m_run[mg][hh] - m_new);
        corr[mg][hh] = cr * rescale;
        m_run[mg][hh] = m_new;
        float lsum = 0.f;
        uint32_t w1 = 0, w2 = 0;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const float pr = __builtin_amdgcn_exp2f(s[tt] - m_new);
          lsum += pr;
          const float t = pr * sv[tt] * to_code;
          const float c1 = fminf(rintf(t), 127.f);
          const float c2 = fminf(fmaxf(rintf((t - c1) * 254.0f), -127.f), 127.f);
          w1 |= ((uint32_t)(int)c1 & 0xFFu) << (8 * tt);
          w2 |= ((uint32_t)(int)c2 & 0xFFu) << (8 * tt);
        }
        l_run[mg][hh] = l_run[mg][hh] * cr + lsum;
        sP[wave][mg][0][g * 2 + hh][j] = w1;
        sP[wave][mg][1][g * 2 + hh][j] = w2;
      }
    __builtin_amdgcn_wave_barrier();
    v4i pa[MG];
#pragma unroll
    for (int mg = 0; mg < MG; ++mg) pa[mg] = *reinterpret_cast<const v4i*>(&sP[wave][mg][row_comp][row_head][4 * g]);
    __builtin_amdgcn_wave_barrier();
    // ---- (5) O1, O2 over this wave's 128-channel slabs of the same rows.  The B operand (64 tokens x 16
    // channels) comes from two transposing LDS reads: in each 16-lane group, source lane s points at 8
    // channel bytes of one token, and lane n receives byte n&7 of the eight source lanes 2k + (n>>3); with
    // even source lanes on channels 0..7 and odd ones on channels 8..15 of token(k), lane n ends up with
    // channel n of eight tokens.  token(k) follows the packing of the P codes (word 4g+i, byte t <-> token
    // 16 t + 4 g + i).
    const int vk = j >> 1;
    // rows 16 (vk & 3) + 4 g + (vk >> 2) (+ 2 for the second read): all in 4-row group g of their 16 rows
    const uint8_t* vsrc = tile + tile_row(16 * (vk & 3) + 4 * g + (vk >> 2)) + 8 * (j & 1);
    int vcol[4];  // byte offset of 16-byte column c within its group of four, c = 0..3
#pragma unroll
    for (int c = 0; c < 4; ++c) vcol[c] = 16 * (c ^ tile_swz(4 * g));
    // Software pipeline over the 16-channel blocks: LDS reads two blocks ahead, the two MFMAs of a block
    // issued one block before their results are merged on the vector ALU.
    constexpr int NST = NSL * 8;
    v2i rb[3][2];
    v4i acc[2][MG];
    auto vload = [&](int st) __attribute__((always_inline)) {
      const uint8_t* src = vsrc + 128 * (ch * NSL + st / 8) + 64 * ((st % 8) / 4) + vcol[st % 4];
      rb[st % 3][0] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) v2i*)src);
      rb[st % 3][1] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) v2i*)(src + 2 * kPitch));
    };
    vload(0);
    vload(1);
#pragma unroll
    for (int st = 0; st <= NST; ++st) {
      if (st + 2 < NST) vload(st + 2);
      if (st < NST) {
        const v4i bf = {rb[st % 3][0][0], rb[st % 3][0][1], rb[st % 3][1][0], rb[st % 3][1][1]};
#pragma unroll
        for (int mg = 0; mg < MG; ++mg) acc[st & 1][mg] = mfma_s8(pa[mg], bf, zero4);
      }
      __builtin_amdgcn_sched_barrier(0);  // the merge below covers the latency of the MFMAs above
      if (st >= 1) {
        const int sl = (st - 1) / 8, c = (st - 1) % 8;
#pragma unroll
        for (int mg = 0; mg < MG; ++mg)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const v4i od = acc[(st - 1) & 1][mg];
            const int merged = __mul24(od[2 * hh], 254) + od[2 * hh + 1];  // |O1| < 2^21: exact
            o_run[mg][sl][hh][c] = __builtin_fmaf(o_run[mg][sl][hh][c], corr[mg][hh], (float)merged);
          }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  if (n_iter > 0) stage(Buf0{}, 0);
  for (int it = 0; it < n_iter; it += 2) {  // an odd count is padded with a tile past the end
    step(Buf1{}, it);
    step(Buf0{}, it + 1);
  }

  float lsum[MG][2];
#pragma unroll
  for (int mg = 0; mg < MG; ++mg)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) lsum[mg][hh] = row16_sum(l_run[mg][hh]);
  if constexpr (TS == 2) {
    // ---- the two token streams of the workgroup merge here, through the tile buffers (free now): the waves of
    // stream 1 hand (m, l, O) to the waves of stream 0 that hold the same heads and channels, lane by lane, so
    // that a split writes one partial instead of two (half the partial-result traffic of the call)
    constexpr int NV = MG * 2 * (2 + NSL * 8);  // floats per lane
    static_assert((size_t)WS * NV * 64 * 4 <= (size_t)2 * TS * kTileBytes, "exchange area");
    float* xch = reinterpret_cast<float*>(sTiles) + (wave % WS) * NV * 64 + lane;
    // each stream keeps its output in its own unit (the alpha_P / 254 of its last coded tile): plain values from here
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
          for (int c = 0; c < 8; ++c) o_run[mg][sl][hh][c] *= unit;
    unit = 1.f;
    __syncthreads();  // every wave has left the tile buffers
    if (ts == 1) {
      int idx = 0;
#pragma unroll
      for (int mg = 0; mg < MG; ++mg)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          xch[64 * idx++] = m_run[mg][hh];
          xch[64 * idx++] = lsum[mg][hh];
#pragma unroll
          for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
            for (int c = 0; c < 8; ++c) xch[64 * idx++] = o_run[mg][sl][hh][c];
        }
    }
    __syncthreads();
    if (ts == 1) return;
    int idx = 0;
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const float m0 = m_run[mg][hh], m1 = xch[64 * idx++], l1 = xch[64 * idx++];
        const float mn = fmaxf(m0, m1);
        const float w0 = m0 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m0 - mn);
        const float w1 = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - mn);
        m_run[mg][hh] = mn;
        lsum[mg][hh] = lsum[mg][hh] * w0 + l1 * w1;
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
          for (int c = 0; c < 8; ++c) o_run[mg][sl][hh][c] = o_run[mg][sl][hh][c] * w0 + xch[64 * idx++] * w1;
      }
  }
  // ---- the partial (m, l, O) of this wave's heads and value channels: one per KV split
  static_assert(TS <= 2, "token streams are merged pairwise above");
  const int part = split;
#pragma unroll
  for (int mg = 0; mg < MG; ++mg)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const float l = lsum[mg][hh];
      const int head = hw + 8 * mg + g * 2 + hh;
      if (head >= Hq) continue;
      if (p.nparts == 1) {
        const int64_t orow = (int64_t)b * Hq + head;
        const float norm = l > 0.f ? __fdiv_rn(unit, l) : 0.f;
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            const int col = 128 * (ch * NSL + sl) + 16 * c + j;
            float v = o_run[mg][sl][hh][c] * norm;
            if (!PER_TOKEN) v *= p.scale[col];
            if (p.out_bf16)
              reinterpret_cast<uint16_t*>(p.out)[orow * kLatV + col] = f32_to_bf16_bits(v);
            else
              reinterpret_cast<float*>(p.out)[orow * kLatV + col] = v;
          }
      } else {
        const int64_t pr = ((int64_t)b * p.nparts + part) * Hq + head;
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
          for (int c = 0; c < 8; ++c)
            p.part_o[pr * kLatV + 128 * (ch * NSL + sl) + 16 * c + j] = o_run[mg][sl][hh][c] * unit;
        if (ch == 0 && j == 0) {
          p.part_m[pr] = m_run[mg][hh];
          p.part_l[pr] = l;
        }
      }
    }
}

// Merge the partials (Alg. 3 last two steps; see attn.hip for why this is a launch of its own).  One
// workgroup per (batch, head): the weights of the parts are formed once in LDS, then every thread sums
// four channels over the parts with independent 16-byte loads.
constexpr int kMlaMaxParts = 64;
__global__ __launch_bounds__(128) void attn_mla_combine_kernel(MlaParams p, int per_channel) {
  __shared__ float s_w[kMlaMaxParts];
  __shared__ float s_linv;
  const int row = blockIdx.x;  // b*Hq + h
  const int b = row / p.Hq, h = row % p.Hq;
  const int64_t base = (int64_t)b * p.nparts * p.Hq + h;
  if (threadIdx.x < 64) {
    const int s = threadIdx.x;
    const bool have = s < p.nparts;
    const float m = have ? p.part_m[base + (int64_t)s * p.Hq] : -INFINITY;
    const float lp = have ? p.part_l[base + (int64_t)s * p.Hq] : 0.f;
    const float ms = wave_max(m);
    const float w = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - ms);
    float l = lp * w;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off, 64);
    s_w[s] = w;
    if (s == 0) s_linv = l > 0.f ? __fdiv_rn(1.0f, l) : 0.f;
  }
  __syncthreads();
  const int c = 4 * threadIdx.x;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
  for (int s = 0; s < p.nparts; ++s) {
    const float w = s_w[s];
    const float4 v = *reinterpret_cast<const float4*>(p.part_o + (base + (int64_t)s * p.Hq) * kLatV + c);
    o.x += v.x * w; o.y += v.y * w; o.z += v.z * w; o.w += v.w * w;
  }
  const float linv = s_linv;
  float r[4] = {o.x * linv, o.y * linv, o.z * linv, o.w * linv};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (per_channel) r[i] *= p.scale[c + i];
    if (p.out_bf16)
      reinterpret_cast<uint16_t*>(p.out)[(int64_t)row * kLatV + c + i] = f32_to_bf16_bits(r[i]);
    else
      reinterpret_cast<float*>(p.out)[(int64_t)row * kLatV + c + i] = r[i];
  }
}

// Wave layout by head count, KV splits (about kMlaTargetWgs workgroups: one per CU holds the registers
// and LDS of this kernel; every token stream of a split gets at least two tiles) and partial count.
constexpr int kMlaTargetWgs = 256;
struct MlaPlan {
  int layout;  // 0: up to 16 heads, 1: up to 32, 2: 64 per workgroup
  int ts, heads_wg, head_blocks, nsplit, nparts;
  int64_t tokens_per_split;
};
// layout -> <MG, NW, HGW, CH>
#define MSD_MLA_LAYOUT_0 1, 8, 2, 2
#define MSD_MLA_LAYOUT_1 1, 8, 4, 2
#define MSD_MLA_LAYOUT_2 1, 8, 8, 1
MlaPlan mla_plan(int B, int Hq, int64_t L) {
  MlaPlan pl{};
  pl.layout = Hq <= 16 ? 0 : (Hq <= 32 ? 1 : 2);
  pl.ts = pl.layout == 0 ? MlaCfg<MSD_MLA_LAYOUT_0>::kTS : (pl.layout == 1 ? MlaCfg<MSD_MLA_LAYOUT_1>::kTS : MlaCfg<MSD_MLA_LAYOUT_2>::kTS);
  pl.heads_wg = pl.layout == 0 ? MlaCfg<MSD_MLA_LAYOUT_0>::kHeadsWg
                               : (pl.layout == 1 ? MlaCfg<MSD_MLA_LAYOUT_1>::kHeadsWg : MlaCfg<MSD_MLA_LAYOUT_2>::kHeadsWg);
  pl.head_blocks = (Hq + pl.heads_wg - 1) / pl.heads_wg;
  int64_t ns = cdiv((int64_t)kMlaTargetWgs, (int64_t)B * pl.head_blocks);
  const int64_t max_by_len = max((int64_t)1, L / (2 * pl.ts * kTile));
  ns = max((int64_t)1, min(min(ns, max_by_len), (int64_t)kMlaMaxParts));
  pl.nsplit = (int)ns;
  pl.nparts = pl.nsplit;  // the token streams of a workgroup merge inside it
  int64_t tps = cdiv(L > 0 ? L : 1, ns);
  pl.tokens_per_split = cdiv(tps, (int64_t)pl.ts * kTile) * (pl.ts * kTile);
  return pl;
}

template <bool PER_TOKEN, int MG, int NW, int HGW, int CH>
int launch_mla_layout(const MlaParams& p, const MlaPlan& pl, hipStream_t stream) {
  constexpr size_t lds = MlaCfg<MG, NW, HGW, CH>::kLds;
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mla_kernel<PER_TOKEN, MG, NW, HGW, CH>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  const dim3 grid((unsigned)((int64_t)p.B * p.nsplit), (unsigned)pl.head_blocks);
  hipLaunchKernelGGL((attn_mla_kernel<PER_TOKEN, MG, NW, HGW, CH>), grid, dim3(NW * 64), lds, stream, p);
  MSD_LAUNCH_CHECK();
  return MSD_OK;
}

template <bool PER_TOKEN>
int launch_mla_mode(const MlaParams& p, const MlaPlan& pl, hipStream_t stream) {
  switch (pl.layout) {
    case 0: return launch_mla_layout<PER_TOKEN, MSD_MLA_LAYOUT_0>(p, pl, stream);
    case 1: return launch_mla_layout<PER_TOKEN, MSD_MLA_LAYOUT_1>(p, pl, stream);
    default: return launch_mla_layout<PER_TOKEN, MSD_MLA_LAYOUT_2>(p, pl, stream);
  }
}

// ------------------------------------------------------------------ comparison kernel (latent cache)
// The conventional path of Sec. 4.1 on the latent-cache shape, as one fused kernel: every cache byte becomes BF16
// on the vector ALU (exact), Q C^T and P C run on v_mfma_f32_16x16x32_bf16 with fp32 accumulation, P (times the
// row's scale in per-token mode) is rounded to BF16; a per-channel scale is folded into Q (rounded to BF16) and
// multiplies the output.  Split plan, partial results and their merge are those of the MSD kernel.
//   A workgroup serves 16 heads (the rows of one A fragment) of a batch entry over one KV split; its four waves
//   take alternate 32-token tiles and each keeps the 16 x 512 output of its tokens in registers (128 per lane):
//   more heads per wave do not fit the register file, so further heads are further workgroups (blockIdx.y) that
//   read the same rows again, from L2.  Operands come straight from global memory in fragment order, as in the
//   grouped-query comparison kernel: the key reading as 16-byte loads (lane = token 16 tt + j, channels
//   64 s + 16 g ..), the value reading as 8-byte loads (channels 128 cb + 8 j .. of token 16 tt + 4 g + jq, so that
//   the bytes of the eight tokens of a B fragment sit in one lane).
constexpr int kCmpTile = 32;      // tokens per wave and step: the contraction extent of the P C product
constexpr int kCmpWaves = 4;
constexpr int kCmpQPitch = 584;   // BF16 elements per query row in LDS (576 + pad)
constexpr int kCmpPPitch = 40;    // BF16 elements per head row of a wave's P tile (32 + pad)
constexpr size_t kCmpLds = 16 * kCmpQPitch * 2 + kCmpWaves * 16 * kCmpPPitch * 2 + kCmpWaves * 16 * kLatV * 4 +
                           2 * kCmpWaves * 16 * 4;

typedef float cmp_v2f __attribute__((ext_vector_type(2)));
typedef __bf16 cmp_v2bf __attribute__((ext_vector_type(2)));
union CmpBf8 {
  uint32_t u[4];
  v8bf v;
};
__device__ __forceinline__ uint32_t cmp_pack2(float lo, float hi) {  // RNE, hardware convert
  const cmp_v2f f = {lo, hi};
  const cmp_v2bf b = __builtin_convertvector(f, cmp_v2bf);
  return *reinterpret_cast<const uint32_t*>(&b);
}
__device__ __forceinline__ float cmp_byte(uint32_t w, int i) {  // signed byte i of w as float
  return (float)(int)(int8_t)((w >> (8 * i)) & 0xFFu);
}

template <bool PER_TOKEN>
__global__ __launch_bounds__(kCmpWaves * 64) void attn_mla_dequant_kernel(MlaParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t s_cmp[];
  uint16_t* sQ = reinterpret_cast<uint16_t*>(s_cmp);                                     // [16][kCmpQPitch]
  uint16_t* sP = sQ + 16 * kCmpQPitch;                                                   // [waves][16][kCmpPPitch]
  float* sO = reinterpret_cast<float*>(sP + kCmpWaves * 16 * kCmpPPitch);                // [waves][16][512]
  float* sM = sO + kCmpWaves * 16 * kLatV;                                               // [waves][16]
  float* sL = sM + kCmpWaves * 16;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int b = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
  const int h0 = blockIdx.y * 16;
  int64_t len = p.kv_len ? (int64_t)p.kv_len[b] : p.L;
  len = max((int64_t)0, min(len, p.L));
  const int64_t t_begin = (int64_t)split * p.tokens_per_split;
  const int64_t t_end = min(len, t_begin + p.tokens_per_split);
  const int8_t* Cb = p.C + (int64_t)b * p.L * p.ld;
  const float* sb = p.scale + (int64_t)b * p.L;  // per token only

  // ---- the query rows as BF16 (per-channel mode: Q * scale rounded to BF16), zero rows past the last head
  for (int idx = tid; idx < 16 * kLatK; idx += kCmpWaves * 64) {
    const int h = idx / kLatK, c = idx % kLatK;
    uint16_t v = 0;
    if (h0 + h < p.Hq) {
      v = p.q[((int64_t)b * p.Hq + h0 + h) * kLatK + c];
      if (!PER_TOKEN) v = f32_to_bf16_bits(__uint_as_float((uint32_t)v << 16) * p.scale[c]);
    }
    sQ[h * kCmpQPitch + c] = v;
  }
  __syncthreads();

  const v4f zero4f = {0.f, 0.f, 0.f, 0.f};
  // per-lane state as a D lane: heads h0 + 4 g + r; output channels 128 cb + 8 j + c
  float m_run[4], l_run[4], o_run[4][8][4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    m_run[r] = -INFINITY;
    l_run[r] = 0.f;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int c = 0; c < 8; ++c) o_run[cb][c][r] = 0.f;
  }
  const int64_t last = max(t_end - 1, (int64_t)0);
  const int64_t t_first = t_begin + (int64_t)wave * kCmpTile;
  constexpr int64_t kStride = kCmpWaves * kCmpTile;
  v4i kx[2][9];      // [tt][s]: channels 64 s + 16 g .. + 15 of token 16 tt + j
  v2i vx[4][2][4];   // [jq][tt][cb]: channels 128 cb + 8 j .. + 7 of token 16 tt + 4 g + jq
  float sk[2];       // the row scale of token 16 tt + j (per token)
  auto load_k = [&](int64_t t0) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int64_t tok = min(t0 + 16 * tt + j, last);
#pragma unroll
      for (int s = 0; s < 9; ++s)
        kx[tt][s] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(Cb + tok * p.ld + 64 * s + 16 * g));
      sk[tt] = PER_TOKEN ? sb[tok] : 1.f;
    }
  };
  auto load_v = [&](int64_t t0) {
#pragma unroll
    for (int jq = 0; jq < 4; ++jq)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const int64_t tok = min(t0 + 16 * tt + 4 * g + jq, last);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
          vx[jq][tt][cb] = *reinterpret_cast<const v2i*>(Cb + tok * p.ld + 128 * cb + 8 * j);
      }
  };
  if (t_first < t_end) {
    load_k(t_first);
    load_v(t_first);
  }
  uint16_t* sPw = sP + wave * 16 * kCmpPPitch;
  for (int64_t t0 = t_first; t0 < t_end; t0 += kStride) {
    bool live[2];
    float sc_tok[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      live[tt] = t0 + 16 * tt + j < t_end;
      sc_tok[tt] = sk[tt];
    }
    // ---- key reading to BF16, S = Q C^T
    v4f sd[2] = {zero4f, zero4f};
#pragma unroll
    for (int s = 0; s < 9; ++s)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        CmpBf8 qa;
        const uint4 qv = *reinterpret_cast<const uint4*>(&sQ[j * kCmpQPitch + 64 * s + 16 * g + 8 * h]);
        qa.u[0] = qv.x; qa.u[1] = qv.y; qa.u[2] = qv.z; qa.u[3] = qv.w;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          CmpBf8 kb;
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const uint32_t w = (uint32_t)kx[tt][s][2 * h + d];
            kb.u[2 * d] = cmp_pack2(cmp_byte(w, 0), cmp_byte(w, 1));
            kb.u[2 * d + 1] = cmp_pack2(cmp_byte(w, 2), cmp_byte(w, 3));
          }
          sd[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa.v, kb.v, sd[tt], 0, 0, 0);
        }
      }
    if (t0 + kStride < t_end) load_k(t0 + kStride);  // the key registers are free: next tile under the rest of this one
    // ---- online softmax; P (times the row scale) to BF16
    float corr[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float sc[2];
      float mx = -INFINITY;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const float v = sd[tt][r] * (p.sm_scale_log2 * sc_tok[tt]);
        sc[tt] = live[tt] ? v : -INFINITY;
        mx = fmaxf(mx, sc[tt]);
      }
      mx = row16_max(mx);
      const float m_new = fmaxf(m_run[r], mx);
      corr[r] = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run[r] - m_new);
      m_run[r] = m_new;
      float lsum = 0.f;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const float pr = live[tt] ? __builtin_amdgcn_exp2f(sc[tt] - m_new) : 0.f;
        lsum += pr;
        sPw[(4 * g + r) * kCmpPPitch + 16 * tt + j] = f32_to_bf16_bits(PER_TOKEN ? pr * sc_tok[tt] : pr);
      }
      l_run[r] = l_run[r] * corr[r] + lsum;
    }
    __builtin_amdgcn_wave_barrier();
    CmpBf8 pa;
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const uint2 v = *reinterpret_cast<const uint2*>(&sPw[j * kCmpPPitch + 16 * t2 + 4 * g]);
      pa.u[2 * t2] = v.x;
      pa.u[2 * t2 + 1] = v.y;
    }
    __builtin_amdgcn_wave_barrier();
    // ---- value reading to BF16 (channel 128 cb + 8 j + c of the eight tokens this lane holds), O += P C
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        CmpBf8 vb;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          float f[4];
#pragma unroll
          for (int jq = 0; jq < 4; ++jq) f[jq] = cmp_byte((uint32_t)vx[jq][t2][cb][c >> 2], c & 3);
          vb.u[2 * t2] = cmp_pack2(f[0], f[1]);
          vb.u[2 * t2 + 1] = cmp_pack2(f[2], f[3]);
        }
        const v4f od = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.v, vb.v, zero4f, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) o_run[cb][c][r] = o_run[cb][c][r] * corr[r] + od[r];
      }
    if (t0 + kStride < t_end) load_v(t0 + kStride);
  }

  // ---- merge the waves of this workgroup; write the final rows (one split) or the split's partial (m, l, O)
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float lt = row16_sum(l_run[r]);
    const int hs = 4 * g + r;
    if (j == 0) {
      sM[wave * 16 + hs] = m_run[r];
      sL[wave * 16 + hs] = lt;
    }
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int c = 0; c < 8; ++c) sO[(wave * 16 + hs) * kLatV + 128 * cb + 8 * j + c] = o_run[cb][c][r];
  }
  __syncthreads();
  const int nh_here = min(16, p.Hq - h0);
  for (int idx = tid; idx < nh_here * kLatV; idx += kCmpWaves * 64) {
    const int hl = idx / kLatV, c = idx % kLatV;
    float ms = -INFINITY;
#pragma unroll
    for (int w = 0; w < kCmpWaves; ++w) ms = fmaxf(ms, sM[w * 16 + hl]);
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < kCmpWaves; ++w) {
      const float mw = sM[w * 16 + hl];
      const float wgt = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - ms);
      o += sO[(w * 16 + hl) * kLatV + c] * wgt;
      l += sL[w * 16 + hl] * wgt;
    }
    const int64_t orow = (int64_t)b * p.Hq + h0 + hl;
    if (p.nparts == 1) {
      float v = l > 0.f ? __fdiv_rn(o, l) : 0.f;
      if (!PER_TOKEN) v *= p.scale[c];
      if (p.out_bf16)
        reinterpret_cast<uint16_t*>(p.out)[orow * kLatV + c] = f32_to_bf16_bits(v);
      else
        reinterpret_cast<float*>(p.out)[orow * kLatV + c] = v;
    } else {
      const int64_t pr = ((int64_t)b * p.nparts + split) * p.Hq + h0 + hl;
      p.part_o[pr * kLatV + c] = o;
      if (c == 0) {
        p.part_m[pr] = ms;
        p.part_l[pr] = l;
      }
    }
  }
}

// KV splits of the comparison kernel: about one workgroup per CU, every wave of a split at least two tiles
struct MlaCmpPlan {
  int head_blocks, nsplit;
  int64_t tokens_per_split;
};
MlaCmpPlan mla_cmp_plan(int B, int Hq, int64_t L) {
  MlaCmpPlan pl{};
  pl.head_blocks = (Hq + 15) / 16;
  int64_t ns = cdiv((int64_t)kMlaTargetWgs, (int64_t)B * pl.head_blocks);
  const int64_t max_by_len = max((int64_t)1, L / (2 * kCmpWaves * kCmpTile));
  ns = max((int64_t)1, min(min(ns, max_by_len), (int64_t)16));
  pl.nsplit = (int)ns;
  const int64_t tps = cdiv(L > 0 ? L : 1, ns);
  pl.tokens_per_split = cdiv(tps, (int64_t)kCmpWaves * kCmpTile) * (kCmpWaves * kCmpTile);
  return pl;
}

}  // namespace

static size_t mla_partial_bytes(size_t rows) { return align_up(rows * kLatV * 4, 256) + 2 * align_up(rows * 4, 256); }

size_t attn_mla_workspace_bytes(int B, int Hq, int64_t L) {
  const size_t rows = (size_t)B * Hq * mla_plan(B, Hq, L).nparts;
  const size_t qrows = (size_t)B * Hq;
  const size_t msd = mla_partial_bytes(rows) + 2 * align_up(qrows * kLatK, 256) + align_up(qrows * 4, 256);
  // the comparison kernel shares the entry point's workspace contract (it never needs more in practice)
  return std::max(msd, mla_partial_bytes((size_t)B * Hq * mla_cmp_plan(B, Hq, L).nsplit));
}

int launch_attn_mla_dequant(const AttnMlaArgs& a, hipStream_t stream) {
  const MlaCmpPlan pl = mla_cmp_plan(a.B, a.Hq, a.L);
  MlaParams p{};
  p.q = a.q; p.C = a.C; p.scale = a.scale; p.kv_len = a.kv_len;
  p.B = a.B; p.Hq = a.Hq; p.L = a.L; p.ld = a.ld;
  p.nsplit = pl.nsplit;
  p.nparts = pl.nsplit;
  p.tokens_per_split = pl.tokens_per_split;
  p.sm_scale_log2 = a.sm_scale * kLog2e;
  const size_t rows = (size_t)a.B * a.Hq * p.nparts;
  char* ws = (char*)a.workspace;
  p.part_o = (float*)ws;
  p.part_m = (float*)(ws + align_up(rows * kLatV * 4, 256));
  p.part_l = (float*)(ws + align_up(rows * kLatV * 4, 256) + align_up(rows * 4, 256));
  p.out = a.out;
  p.out_bf16 = a.out_bf16;
  const bool per_token = a.scale_mode == MSD_PER_TOKEN;
  static bool attr_set = false;
  if (!attr_set) {
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mla_dequant_kernel<true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kCmpLds));
    MSD_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mla_dequant_kernel<false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kCmpLds));
    attr_set = true;
  }
  const dim3 grid((unsigned)((int64_t)a.B * p.nsplit), (unsigned)pl.head_blocks);
  if (per_token)
    hipLaunchKernelGGL((attn_mla_dequant_kernel<true>), grid, dim3(kCmpWaves * 64), kCmpLds, stream, p);
  else
    hipLaunchKernelGGL((attn_mla_dequant_kernel<false>), grid, dim3(kCmpWaves * 64), kCmpLds, stream, p);
  MSD_LAUNCH_CHECK();
  if (p.nparts > 1) {
    hipLaunchKernelGGL(attn_mla_combine_kernel, dim3((unsigned)(a.B * a.Hq)), dim3(128), 0, stream, p,
                       per_token ? 0 : 1);
    MSD_LAUNCH_CHECK();
  }
  return MSD_OK;
}

int launch_attn_mla(const AttnMlaArgs& a, hipStream_t stream) {
  const MlaPlan pl = mla_plan(a.B, a.Hq, a.L);
  MlaParams p{};
  p.q = a.q; p.C = a.C; p.scale = a.scale; p.kv_len = a.kv_len;
  p.B = a.B; p.Hq = a.Hq; p.L = a.L; p.ld = a.ld;
  p.nsplit = pl.nsplit;
  p.nparts = pl.nparts;
  p.tokens_per_split = pl.tokens_per_split;
  p.sm_scale_log2 = a.sm_scale * kLog2e;
  const size_t rows = (size_t)a.B * a.Hq * pl.nparts;
  char* ws = (char*)a.workspace;
  p.part_o = (float*)ws;
  p.part_m = (float*)(ws + align_up(rows * kLatV * 4, 256));
  p.part_l = (float*)(ws + align_up(rows * kLatV * 4, 256) + align_up(rows * 4, 256));
  char* qws = ws + align_up(rows * kLatV * 4, 256) + 2 * align_up(rows * 4, 256);
  const size_t qrows = (size_t)a.B * a.Hq;
  p.qc1 = (int8_t*)qws;
  p.qc2 = (int8_t*)(qws + align_up(qrows * kLatK, 256));
  p.qalpha = (float*)(qws + 2 * align_up(qrows * kLatK, 256));
  p.out = a.out;
  p.out_bf16 = a.out_bf16;
  if (a.taps) {
    p.tap_q1 = (int8_t*)a.taps->q1;
    p.tap_q2 = (int8_t*)a.taps->q2;
    p.tap_alpha = (float*)a.taps->scale;
    p.tap_s1 = a.taps->acc1;
    p.tap_s2 = a.taps->acc2;
    if (!(p.tap_q1 && p.tap_q2 && p.tap_alpha)) p.tap_q1 = p.tap_q2 = nullptr, p.tap_alpha = nullptr;
    if (!(p.tap_s1 && p.tap_s2)) p.tap_s1 = p.tap_s2 = nullptr;
  }
  const bool per_token = a.scale_mode == MSD_PER_TOKEN;
  if (pl.layout == 2) {
    hipLaunchKernelGGL(mla_q_decompose_kernel, dim3((unsigned)cdiv((int64_t)qrows, 4)), dim3(256), 0, stream, p,
                       per_token ? 0 : 1);
    MSD_LAUNCH_CHECK();
  }
  const int rc = per_token ? launch_mla_mode<true>(p, pl, stream) : launch_mla_mode<false>(p, pl, stream);
  if (rc != MSD_OK) return rc;
  if (p.nparts > 1) {
    hipLaunchKernelGGL(attn_mla_combine_kernel, dim3((unsigned)(a.B * a.Hq)), dim3(128), 0, stream, p,
                       per_token ? 0 : 1);
    MSD_LAUNCH_CHECK();
  }
  return MSD_OK;
}

}  // namespace msd
