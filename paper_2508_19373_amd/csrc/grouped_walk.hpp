// Grouped "NT" GEMM for decode-sized groups, register-resident activations (gfx950).
//
// Decode is bound by reading every active expert's weights from HBM once (paper, "Generative
// Inference": the decoding stage is memory-bound by weight loading).  Measured on MI355X, a
// kernel that re-reads the activation rows for every weight strip loses 10-40 % of the HBM
// rate to the extra L1 requests, so here the activations never leave the register file:
//  * a workgroup owns a contiguous range of the list of (expert, pass of 16*MT rows, 16-feature
//    strip) of one K slice; wavefront w owns k32 steps [w*STEPS, (w+1)*STEPS) of that slice and
//    loads its MFMA A operands (the pass's activation rows, padded by clamping) ONCE per
//    (expert, pass), before walking the strips;
//  * the weights then flow as one continuous stream of 1 KB loads (16 rows x 64 contiguous
//    bytes, the pattern that measured best: ~6.4 TB/s) through a register ring RING loads deep,
//    crossing strip boundaries without draining;
//  * v_mfma_f32_16x16x32_bf16; per strip the NW partial tiles meet in a double-buffered LDS
//    area (one barrier per strip) and are summed in wave order, so the result is deterministic;
//  * K slices (grid.z > 1, down projection only) write fp32 partial outputs that a small
//    second kernel adds in slice order;
//  * experts without rows have no entry in the list: their weights are never touched.
#pragma once
#include <type_traits>

#include "moe_internal.hpp"
#include "unit_list_wave.hpp"

namespace moe {
namespace gw {

__device__ __forceinline__ float silu_mul(float g, float u) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u; }

template <int LO, int HI, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (LO < HI) {
    f(std::integral_constant<int, LO>{});
    static_for<LO + 1, HI>(f);
  }
}

// largest divisor of n in [6, 12], else the largest one below 6
// largest divisor of n that is at most cap
constexpr int ring_cap(int n, int cap) {
  for (int r = cap; r >= 1; --r)
    if (n % r == 0) return r;
  return 1;
}
constexpr int ring_size(int n) {
  for (int r = 12; r >= 6; --r)
    if (n % r == 0) return r;
  for (int r = 5; r >= 1; --r)
    if (n % r == 0) return r;
  return 1;
}

// MT = 1 is compiled for 4 wavefronts per SIMD (at most 128 VGPRs: two 8-wave workgroups per CU),
// MT = 2 for 2 per SIMD.
// grid = (workgroups per K slice, 1, K slices).  GATEUP: Wa = gate, Wb = up, C = h (bf16).
// Else Wa = down and C = y (fp32) or, with K slices, the partial buffer [slice][cap_rows][n_out].
template <int NW, int STEPS, int MT, bool GATEUP>
__global__ __launch_bounds__(NW * 64, (MT == 1 ? 4 : 2)) void grouped_walk_kernel(
    const uint16_t* __restrict__ A, const int32_t* __restrict__ expert_offsets, const uint16_t* __restrict__ Wa,
    const uint16_t* __restrict__ Wb, int n_out, int K, void* __restrict__ Cv, int n_local, int cap_rows,
    const RowMap rows) {
  constexpr int NB = GATEUP ? 2 : 1;
  constexpr int ITEMS = NB * STEPS;  // weight loads (1 KB each) per strip per wave
  // MT = 1 has 128 VGPRs: 4 * STEPS hold the activations, and a ring that does not fit next to them
  // spills (8 slots beside 16 steps: 60 bytes of scratch per lane and 4 % of the HBM rate)
  // MT = 2 has 256 VGPRs and half the wavefronts per CU: a ring of up to 16 slots restores the
  // bytes in flight.
  constexpr int BUDGET2 = NW == 16 ? 96 : 216;  // registers for activations + ring with MT = 2 (16 wavefronts: 128 VGPRs)
  constexpr int RING = MT == 2 ? ring_cap(ITEMS, (BUDGET2 - 8 * STEPS) / 4 < 16 ? (BUDGET2 - 8 * STEPS) / 4 : 16)
                               : ((4 * STEPS + 4 * ring_size(ITEMS) > 92) ? ring_cap(ITEMS, (92 - 4 * STEPS) / 4)
                                                                           : ring_size(ITEMS));
  constexpr int TILES = NB * MT;
  __shared__ float red[2][NW][TILES][256];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, kq = lane >> 4;
  const int total_strips = n_out / 16;
  // The work of one K slice is the list of (expert, row pass, strip) in that order: an expert with
  // rows has ceil(rows / (16 MT)) passes, each walking all of its strips; one without rows has
  // none, so its weights are never read (with few tokens many experts are inactive: 40 of 60 at
  // 16 tokens).  The workgroups cut this list into equal contiguous ranges, so an expert that
  // needs a second pass (a skewed routing puts 20 rows on one expert when the average is 6) costs
  // its share of extra strips to everybody instead of doubling the run time of its own
  // workgroups.  Such a range may end one (expert, pass) and begin the next.  Lane l looks at experts
  // l, l + 64, ...; every wavefront computes the same values.
  const int chunks = (n_local + 63) >> 6;
  // The per-lane tables live only inside this function: a second range reads them again rather
  // than holding 16 registers through the strip loop.  Returns the number of (expert, pass) units;
  // with u >= 0 also that unit's expert, first row and the expert's end row.
  auto find_unit = [&](int u, int& e, int& m0, int& hi, int& g, int& g_end) {
    int pas[gg::kLaneChunks], pre[gg::kLaneChunks], lo_[gg::kLaneChunks], hi_[gg::kLaneChunks];
#pragma unroll
    for (int j = 0; j < gg::kLaneChunks; ++j) {
      const int ee = j * 64 + lane;
      const bool ok = j < chunks && ee < n_local;
      lo_[j] = ok ? expert_offsets[ee] : 0;
      hi_[j] = ok ? expert_offsets[ee + 1] : 0;
      pas[j] = (hi_[j] - lo_[j] + 16 * MT - 1) / (16 * MT);
    }
    const int units = gg::wave_prefix(pas, chunks, pre);
    if (u < 0) {  // first call: this workgroup's range [g, g_end) of the list, then its first unit
      const int n_wg = gridDim.x, total = units * total_strips;
      const int per_wg = (total + n_wg - 1) / n_wg;
      g = blockIdx.x * per_wg;
      g_end = min(g + per_wg, total);
      // A range that crosses into the next (expert, pass) reloads its activations and refills
      // the weight ring (about half a strip's time, with nothing else on the compute unit to
      // hide it), so when giving every (expert, pass) the same whole number of workgroups comes
      // out no longer than the equal cut, that is used instead and no range crosses.
      if (units > 0 && units <= n_wg) {
        const int share = n_wg / units, per_part = (total_strips + share - 1) / share;
        if (per_part <= per_wg) {
          const int uu = (int)blockIdx.x / share, part = (int)blockIdx.x - uu * share;
          g = uu * total_strips + part * per_part;
          g_end = uu < units ? min(g + per_part, (uu + 1) * total_strips) : g;
        }
      }
      if (g >= g_end) return;
      u = g / total_strips;
    }
    const gg::WaveHit h = gg::wave_find(pre, pas, chunks, u);
    e = __builtin_amdgcn_readfirstlane(h.lane + 64 * h.j);
    hi = __builtin_amdgcn_readfirstlane(gg::wave_pick(hi_, h));
    m0 = __builtin_amdgcn_readfirstlane(gg::wave_pick(lo_, h) + (u - gg::wave_pick(pre, h)) * 16 * MT);
  };
  int e = 0, m0 = 0, hi = 0, g = 0, g_end = 0;
  find_unit(-1, e, m0, hi, g, g_end);
  const int kbase = (blockIdx.z * NW + wave) * (STEPS * 32) + kq * 8;
  const size_t strip_stride = (size_t)16 * K;

  bool first = true;
  while (g < g_end) {
    const int u = g / total_strips;
    const int s_begin = g - u * total_strips;
    const int n_strips = min(total_strips - s_begin, g_end - g);
    if (!first) find_unit(u, e, m0, hi, g, g_end);
    first = false;
    g += n_strips;
    const size_t eoff = (size_t)e * n_out * K;
    const uint16_t* w_lane[NB];
    w_lane[0] = Wa + eoff + (size_t)(s_begin * 16 + l16) * K + kbase;
    if constexpr (GATEUP) w_lane[1] = Wb + eoff + (size_t)(s_begin * 16 + l16) * K + kbase;
    {
    const int m_hi = min(m0 + 16 * MT, hi);
    // ---- activations: loaded once, kept for every strip
    bf16x8 a[STEPS][MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const uint16_t* ap = A + (size_t)rows(min(m0 + t * 16 + l16, m_hi - 1)) * K + kbase;
#pragma unroll
      for (int s = 0; s < STEPS; ++s) a[s][t] = *reinterpret_cast<const bf16x8*>(ap + s * 32);
    }

    // ---- weight stream: item j of strip si is matrix j / STEPS, k32 step j % STEPS
    bf16x8 ring[RING];
    auto load_item = [&](int si, auto j_tag, auto slot_tag) {
      constexpr int j = decltype(j_tag)::value, slot = decltype(slot_tag)::value;
      const int sc = min(si, n_strips - 1);  // past the range: re-read the last strip (unused)
      ring[slot] = *reinterpret_cast<const bf16x8*>(w_lane[j / STEPS] + sc * strip_stride + (j % STEPS) * 32);
    };
    static_for<0, RING>([&](auto j_tag) { load_item(0, j_tag, j_tag); });

    for (int si = 0; si < n_strips; ++si) {
      f32x4 acc[NB][MT];
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[b][t] = f32x4{0.f, 0.f, 0.f, 0.f};
      static_for<0, ITEMS>([&](auto j_tag) {
        constexpr int j = decltype(j_tag)::value;
        constexpr int slot = j % RING, b = j / STEPS, s = j % STEPS;
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[b][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s][t], ring[slot], acc[b][t], 0, 0, 0);
        // refill the slot with the item RING ahead in the stream (next strip past the end)
        constexpr int jn = (j + RING) % ITEMS;
        load_item(si + ((j + RING) >= ITEMS ? 1 : 0), std::integral_constant<int, jn>{},
                  std::integral_constant<int, slot>{});
      });

      // ---- partial tiles -> LDS (buffer si & 1), one barrier, fixed-order sum, epilogue
      const int buf = si & 1;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) red[buf][wave][b * MT + t][(kq * 4 + i) * 16 + l16] = acc[b][t][i];
      __syncthreads();
      const int col = (s_begin + si) * 16;
      for (int idx = tid; idx < MT * 256; idx += NW * 64) {
        const int t = idx >> 8, r = (idx >> 4) & 15, c = idx & 15;
        const int row = m0 + t * 16 + r;
        float sum[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          float v = 0.f;
#pragma unroll
          for (int w = 0; w < NW; ++w) v += red[buf][w][b * MT + t][r * 16 + c];
          sum[b] = v;
        }
        if (row < m_hi) {
          if constexpr (GATEUP) {
            static_cast<uint16_t*>(Cv)[(size_t)row * n_out + col + c] =
                (uint16_t)f32_to_bf16_bits(silu_mul(sum[0], sum[1]));
          } else {
            static_cast<float*>(Cv)[((size_t)blockIdx.z * cap_rows + row) * n_out + col + c] = sum[0];
          }
        }
      }
      // no second barrier: buffer `buf` is written again two strips later, after the next barrier
    }
    }
    __syncthreads();  // before the next range reuses the LDS buffers
  }
}

// y[r, n] = sum over K slices, in slice order, of partial[slice][r, n] for the rows in use.
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ partial,
                                                        const int32_t* __restrict__ expert_offsets, int n_local,
                                                        int cap_rows, int n_out, int n_slices, float* __restrict__ y) {
  const int R = expert_offsets[n_local];
  const size_t total = (size_t)R * n_out / 4;
  const size_t slice_stride = (size_t)cap_rows * n_out / 4;
  const float4* p = reinterpret_cast<const float4*>(partial);
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    float4 s = p[i];
    for (int z = 1; z < n_slices; ++z) {
      const float4 v = p[z * slice_stride + i];
      s.x += v.x;
      s.y += v.y;
      s.z += v.z;
      s.w += v.w;
    }
    reinterpret_cast<float4*>(y)[i] = s;
  }
}

// How K is cut for the walk kernel: NW wavefronts x STEPS k32 steps per wavefront x slices.
struct WalkPlan {
  int nw, steps, slices;  // nw == 0: shape not covered, use the generic streaming kernel
};
// mt = 1 (at most 16 rows per pass, 128 VGPRs per lane): sixteen wavefronts per workgroup with at
// most 14 k32 steps each leave room for a weight ring as long as a strip, twice the bytes in flight
// per compute unit of the 8-wavefront split (measured 6.2 against 5.9 TB/s).  mt = 2 holds twice
// the activation registers and stays with 8 or 4 wavefronts at 256 VGPRs.
inline WalkPlan plan_for(int K, int mt, bool down = false) {
  const int steps32 = K / 32;
  if (K % 32 == 0) {
    if (mt == 1) {
      const int cand16[6] = {14, 11, 8, 7, 5, 4};  // instantiated with 16 wavefronts
      for (int st : cand16)
        if (steps32 % (16 * st) == 0) return WalkPlan{16, st, steps32 / (16 * st)};
    }
    if (mt == 2 && down) {
      // the down projection's registers (no second weight matrix) leave room for sixteen wavefronts of up
      // to 8 steps at 128 VGPRs also with 32 rows per pass (Mixtral TP=4 shard, K = 3584, 48-64 tokens:
      // 39.1-39.9 us replayed alone, tiled 43.0; layer 162.8 -> 160.6 us).  The gate/up projection spills
      // in that shape (97 us against 91 with eight wavefronts).
      const int cand16[4] = {8, 7, 5, 4};
      for (int st : cand16)
        if (steps32 == 16 * st) return WalkPlan{16, st, 1};
    }
    const int nws[2] = {8, 4};
    const int cand[7] = {16, 14, 11, 10, 8, 7, 5};
    for (int nw : nws)
      for (int st : cand) {
        // instantiated: (8,16) (8,14) (8,11) (8,10) (8,8) (8,7) (8,5) (4,11) (4,10) (4,8) (4,5)
        if (nw == 4 && !(st == 11 || st == 10 || st == 8 || st == 5)) continue;
        if (steps32 % (nw * st) == 0) return WalkPlan{nw, st, steps32 / (nw * st)};
      }
  }
  return WalkPlan{0, 0, 0};
}

}  // namespace gw
}  // namespace moe
