// Expert networks on the permuted rows (paper, "MoE Model Architectures": the Expert module's
// parallel expert networks, evaluated only for the tokens the gating network sent to them;
// "Tensor Parallelism": a shard may hold only a slice of the intermediate dimension, in which
// case the result is the unreduced partial sum).
//
// Two grouped GEMMs, both "NT" (activations and weights are K-contiguous):
//   GEMM1  h[r, i]  = silu(x_r . Wg_e[i,:]) * (x_r . Wu_e[i,:])      K = H,   N = I_s (gate+up fused)
//   GEMM2  y[r, n]  = h_r . Wd_e[n,:]                                K = I_s, N = H
// bf16 operands, fp32 accumulators.  Two kernel families cover the two regimes the paper
// distinguishes ("Generative Inference"): grouped_gemm.hpp (tiled, LDS-DMA, MFMA-bound) for
// prefill-sized groups, grouped_walk.hpp (weight streaming, HBM-bound; grouped_stream.hpp for the
// K extents it is not instantiated for) for decode-sized groups.  Each of the two GEMMs picks its
// family from a cost estimate (prefer_walk below).  In both, the work list is derived on the
// device from expert_offsets without a host round trip.
#include "grouped_gemm.hpp"
#include "grouped_stream.hpp"
#include "grouped_walk.hpp"
#include "moe_internal.hpp"

#include <cmath>

namespace moe {
namespace {

// Prefill-sized groups: LDS-DMA kernel, 256-column tiles of 256 / 128 / 64 rows.
template <int BN>
hipError_t launch_pair_dlds(const void* x_perm, RowMap rows, const int32_t* expert_offsets, int cap_rows, int est_rows, int n_local, int H,
                            int I_s, const void* w_gate, const void* w_up, const void* w_down, void* h_ws,
                            void* y_perm, void* workspace, uint32_t flags, hipStream_t stream) {
  const bool y_bf16 = (flags & MOE_Y_PERM_BF16) != 0;
  const dim3 block(256);
  const uint16_t* xp = static_cast<const uint16_t*>(x_perm);
  uint16_t* hw = static_cast<uint16_t*>(h_ws);
  auto grid_for = [&](int ncb) { return dim3((unsigned)gg::max_grid(cap_rows, n_local, ncb)); };
  if (!(flags & MOE_FFN_SKIP_GATEUP)) {
    const int ncb = (I_s + BN / 2 - 1) / (BN / 2);
    hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, true, uint16_t, false>), grid_for(ncb), block, 0, stream, xp,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_gate),
                       static_cast<const uint16_t*>(w_up), I_s, H, hw, ncb, static_cast<uint16_t*>(nullptr), 0, rows);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  if (flags & MOE_FFN_SKIP_DOWN) return hipSuccess;
  const int ncb = (H + BN - 1) / BN;
  if (y_bf16) {
    hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, false, uint16_t, false>), grid_for(ncb), block, 0, stream, hw,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_down),
                       static_cast<const uint16_t*>(nullptr), H, I_s, static_cast<uint16_t*>(y_perm), ncb,
                       static_cast<uint16_t*>(nullptr), 0, RowMap{nullptr, 1});
    return hipGetLastError();
  }
  const gg::SlicePlan sp = workspace == nullptr ? gg::SlicePlan{1, 0} : gg::slice_plan(cap_rows, ncb, I_s);
  float* yp = static_cast<float*>(y_perm);
  float* ws = static_cast<float*>(workspace);
  const uint16_t* wd = static_cast<const uint16_t*>(w_down);
  if (sp.max_slices == 1) {
    hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, false, float, false>), grid_for(ncb), block, 0, stream, hw,
                       expert_offsets, n_local, cap_rows, wd, static_cast<const uint16_t*>(nullptr), H, I_s, yp, ncb,
                       static_cast<float*>(nullptr), 0, RowMap{nullptr, 1});
    return hipGetLastError();
  }
  hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, false, float, true>),
                     dim3(gg::sliced_grid(cap_rows, n_local, ncb)), block, 0, stream, hw, expert_offsets, n_local,
                     cap_rows, wd, static_cast<const uint16_t*>(nullptr), H, I_s, ws, ncb, yp, sp.max_slices,
                     RowMap{nullptr, 1});
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(gg::sum_sliced_kernel, dim3(192, (H + 1023) / 1024), dim3(256), 0, stream, ws, expert_offsets, n_local, ncb,
                     I_s / gg::BK, sp.max_slices, H, yp);
  return hipGetLastError();
}

// A few hundred rows per expert: tiles of 160 rows from the one-height work list (unit_list_even.hpp).
hipError_t launch_pair_even(const void* x_perm, RowMap rows, const int32_t* expert_offsets, int cap_rows, int n_local,
                            int H, int I_s, const void* w_gate, const void* w_up, const void* w_down, void* h_ws,
                            void* y_perm, uint32_t flags, hipStream_t stream) {
  const dim3 block(256);
  uint16_t* hw = static_cast<uint16_t*>(h_ws);
  if (!(flags & MOE_FFN_SKIP_GATEUP)) {
    const int ncb = (I_s + 127) / 128;
    hipLaunchKernelGGL((gg::grouped_gemm_even_kernel<256, true, uint16_t>),
                       dim3((unsigned)gg::even_max_ids(cap_rows, n_local, ncb)), block, 0, stream,
                       static_cast<const uint16_t*>(x_perm), expert_offsets, n_local, cap_rows,
                       static_cast<const uint16_t*>(w_gate), static_cast<const uint16_t*>(w_up), I_s, H, hw, ncb, rows);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  if (flags & MOE_FFN_SKIP_DOWN) return hipSuccess;
  const int ncb = (H + 255) / 256;
  const dim3 grid((unsigned)gg::even_max_ids(cap_rows, n_local, ncb));
  if (flags & MOE_Y_PERM_BF16)
    hipLaunchKernelGGL((gg::grouped_gemm_even_kernel<256, false, uint16_t>), grid, block, 0, stream, hw, expert_offsets,
                       n_local, cap_rows, static_cast<const uint16_t*>(w_down), static_cast<const uint16_t*>(nullptr), H,
                       I_s, static_cast<uint16_t*>(y_perm), ncb, RowMap{nullptr, 1});
  else
    hipLaunchKernelGGL((gg::grouped_gemm_even_kernel<256, false, float>), grid, block, 0, stream, hw, expert_offsets,
                       n_local, cap_rows, static_cast<const uint16_t*>(w_down), static_cast<const uint16_t*>(nullptr), H,
                       I_s, static_cast<float*>(y_perm), ncb, RowMap{nullptr, 1});
  return hipGetLastError();
}

// Decode-sized groups, register-resident activations (grouped_walk.hpp).  Returns false when the
// K extent is not one of the instantiated (wavefronts x steps) splits.
constexpr int kWalkSlots = 512;  // 8-wavefront workgroups resident at once with MT = 1 (2 per CU); half of it
                                  // with MT = 2 or 16 wavefronts (1 per CU)

template <int MT, bool GATEUP>
bool launch_walk(const gw::WalkPlan& plan, const uint16_t* A, const int32_t* expert_offsets, int n_local,
                 const uint16_t* Wa, const uint16_t* Wb, int n_out, int K, void* C, int cap_rows, RowMap rows,
                 bool leave_room, hipStream_t stream) {
  // as many workgroups as are resident at once; the kernel cuts its work list into that many ranges
  int n_wg = (MT == 1 && plan.nw < 16 ? kWalkSlots : kWalkSlots / 2) / plan.slices;
  if (leave_room) n_wg = n_wg * 15 / 16;  // 16 compute units stay free for a tiled call on another stream
  n_wg = n_wg < 1 ? 1 : n_wg;
  const dim3 grid(n_wg, 1, plan.slices);
#define MOE_WALK(NW, ST)                                                                                        \
  if (plan.nw == NW && plan.steps == ST) {                                                                      \
    hipLaunchKernelGGL((gw::grouped_walk_kernel<NW, ST, MT, GATEUP>), grid, dim3(NW * 64), 0, stream, A,        \
                       expert_offsets, Wa, Wb, n_out, K, C, n_local, cap_rows, rows);                               \
    return true;                                                                                                \
  }
  if constexpr (MT == 1) {
    MOE_WALK(16, 14)
    MOE_WALK(16, 11)
  }
  if constexpr (MT == 1 || !GATEUP) {  // with 32 rows per pass only the down projection fits sixteen wavefronts
    MOE_WALK(16, 8)
    MOE_WALK(16, 7)
    MOE_WALK(16, 5)
    MOE_WALK(16, 4)
  }
  MOE_WALK(8, 16)
  MOE_WALK(8, 14)
  MOE_WALK(8, 11)
  MOE_WALK(8, 10)
  MOE_WALK(8, 8)
  MOE_WALK(8, 7)
  MOE_WALK(8, 5)
  MOE_WALK(4, 11)
  MOE_WALK(4, 10)
  MOE_WALK(4, 8)
  MOE_WALK(4, 5)
#undef MOE_WALK
  return false;
}

template <int MT>
hipError_t launch_pair_decode(const void* x_perm, RowMap rows, const int32_t* expert_offsets, int cap_rows, int n_local, int H,
                              int I_s, const void* w_gate, const void* w_up, const void* w_down, void* h_ws,
                              void* y_perm, void* workspace, uint32_t flags, hipStream_t stream) {
  const bool y_bf16 = (flags & MOE_Y_PERM_BF16) != 0;
  const uint16_t* xp = static_cast<const uint16_t*>(x_perm);
  uint16_t* hw = static_cast<uint16_t*>(h_ws);
  if (n_local > 65535) return hipErrorInvalidValue;
  if (!(flags & MOE_FFN_SKIP_GATEUP)) {
    const gw::WalkPlan p1 = gw::plan_for(H, MT);
    bool done = false;
    if (p1.nw != 0 && p1.slices == 1 && I_s % 16 == 0)
      done = launch_walk<MT, true>(p1, xp, expert_offsets, n_local, static_cast<const uint16_t*>(w_gate),
                                   static_cast<const uint16_t*>(w_up), I_s, H, hw, cap_rows, rows,
                                   (flags & MOE_FFN_LEAVE_ROOM) != 0, stream);
    if (!done) {
      const dim3 grid((I_s + gs::kStripN - 1) / gs::kStripN, n_local);
      hipLaunchKernelGGL((gs::grouped_stream_kernel<MT, true, uint16_t>), grid, dim3(gs::kWaves * 64), 0, stream, xp,
                         expert_offsets, static_cast<const uint16_t*>(w_gate), static_cast<const uint16_t*>(w_up),
                         I_s, H, hw, rows);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  if (flags & MOE_FFN_SKIP_DOWN) return hipSuccess;
  const gw::WalkPlan p2 = gw::plan_for(I_s, MT, true);
  if (!y_bf16 && p2.nw != 0 && H % 16 == 0 && (p2.slices == 1 || workspace != nullptr)) {
    void* out = p2.slices == 1 ? y_perm : workspace;
    if (launch_walk<MT, false>(p2, hw, expert_offsets, n_local, static_cast<const uint16_t*>(w_down),
                               static_cast<const uint16_t*>(nullptr), H, I_s, out, cap_rows, RowMap{nullptr, 1},
                               (flags & MOE_FFN_LEAVE_ROOM) != 0, stream)) {
      hipError_t err = hipGetLastError();
      if (err != hipSuccess || p2.slices == 1) return err;
      hipLaunchKernelGGL(gw::sum_slices_kernel, dim3(64), dim3(256), 0, stream, static_cast<const float*>(workspace),
                         expert_offsets, n_local, cap_rows, H, p2.slices, static_cast<float*>(y_perm));
      return hipGetLastError();
    }
  }
  const dim3 grid((H + gs::kStripN - 1) / gs::kStripN, n_local);
  if (y_bf16)
    hipLaunchKernelGGL((gs::grouped_stream_kernel<MT, false, uint16_t>), grid, dim3(gs::kWaves * 64), 0, stream, hw,
                       expert_offsets, static_cast<const uint16_t*>(w_down), static_cast<const uint16_t*>(nullptr),
                       H, I_s, static_cast<uint16_t*>(y_perm), RowMap{nullptr, 1});
  else
    hipLaunchKernelGGL((gs::grouped_stream_kernel<MT, false, float>), grid, dim3(gs::kWaves * 64), 0, stream, hw,
                       expert_offsets, static_cast<const uint16_t*>(w_down), static_cast<const uint16_t*>(nullptr),
                       H, I_s, static_cast<float*>(y_perm), RowMap{nullptr, 1});
  return hipGetLastError();
}

// Rows the fullest local expert is planned for.  A shard that holds every expert gets exactly the
// capacity, and only its spread over the experts is open: the average plus two sigma.  An
// expert-parallel shard's share of the batch follows the routing ("Expert Parallelism": load
// imbalance), and the shard that sets the latency of the step is the one that got more than its
// share, so it is planned for twice the balanced share (under Zipf(1.2) popularity the first of four
// shards receives 55 % of the rows, 2.2 times a quarter), never more than the whole capacity.
inline double planned_rows_hi(int cap_rows, int est_rows, int n_local) {
  double avg = (double)est_rows / n_local;
  if (n_local == 1 && est_rows == cap_rows) return avg;  // one expert that takes every row
  if (est_rows < cap_rows) avg = fmin(2.0 * avg, (double)cap_rows / n_local);
  return avg + 2.0 * sqrt(avg);
}

// MT = 1 (16 activation rows per pass) when the fullest expert is expected to stay within 16 rows
// (certain when the whole capacity is 16 rows): it keeps twice the bytes in flight, and an expert
// with more rows only pays another pass over its own weights.
inline int decode_mt(int cap_rows, int est_rows, int n_local) {
  return (cap_rows <= 16 || planned_rows_hi(cap_rows, est_rows, n_local) <= 16.0) ? 1 : 2;
}

// Which kernel family runs one of the two GEMMs: the weight-streaming walk (decode regime) or the
// tiled LDS-DMA kernel (prefill regime).  A few rows per expert are bound by streaming the
// weights once, many rows by the matrix cores; in between, what decides is how often the walk has
// to re-stream an expert (one pass per 16 or 32 rows) against how many tiles the tiled kernel can
// spread over the compute units (the down projection of a single shared expert has H / 256 = 14
// column blocks per row block: 14 CUs, which is why such a launch is also cut along K).
// Estimates in seconds, from measured rates on MI355X:
//   walk   passes * (bytes / rate + 5 us), rate 6.0 / 5.4 TB/s (GEMM1 / GEMM2) at 16 rows per pass,
//          5.3 / 4.9 TB/s at 32, 3 TB/s for K extents only the generic streaming kernel covers;
//          passes from the rows of the fullest expert (planned_rows_hi);
//   tiled  rounds * (tile time + 8 us), rounds = tiles * slices / 256, at least one; tile time is the
//          larger of streaming the tile's weight panel latency-bound (45 GB/s per compute unit) and
//          its MFMA pace (1.3 us per k-tile of a full 256-row tile); never faster than 1.2 PFLOP/s
//          overall.  What HBM allows when all compute units stream at once: for the gate/up
//          projection all panels together at 5.7 TB/s + 4 us (measured 5.4-5.9 TB/s); for the down
//          projection the per-unit rate is capped at 5.4 TB/s / busy units inside the tile time
//          (its partial sums and their addition ride on the 8 us).
// (Measured, Mixtral TP=4 shard at 48-64 tokens: gate/up streaming with 32 rows per pass 90.5-91.8 us,
// tiled 86.2-86.6; with 16 rows per pass at 16-32 tokens 80.5-81.8 against 85.7.  Qwen1.5 down
// projection at 64-128 tokens: streaming 68.0 / 73.7 us, tiled 61.8 / 66.0.)
inline bool prefer_walk(int cap_rows, int est_rows, int n_local, int n_out, int K, bool gateup) {
  const double mats = gateup ? 2.0 : 1.0;
  const bool exact = n_local == 1 && est_rows == cap_rows;  // one expert that takes every row
  const double rows_hi = planned_rows_hi(cap_rows, est_rows, n_local);
  const int mt = decode_mt(cap_rows, est_rows, n_local);
  const double passes = ceil(rows_hi / (16.0 * mt));
  const double bytes = mats * n_local * (double)n_out * K * 2.0;
  const gw::WalkPlan wp = gw::plan_for(K, mt, !gateup);
  const double rate = wp.nw == 0 ? 3.0e12
                                                  : (mt == 1 ? (gateup ? 6.0e12 : 5.4e12)
                                                             : (gateup ? 5.3e12 : (wp.nw == 16 ? 5.9e12 : 4.9e12)));
  const double walk = passes * (bytes / rate + 5e-6);
  const int ncb = (n_out + (gateup ? 127 : 255)) / (gateup ? 128 : 256);
  const int slices = gateup ? 1 : gg::k_slices_for(est_rows, n_local, ncb, K, exact);
  const double units = (double)gg::expected_tiles(est_rows, n_local, ncb, exact) * slices;
  const double k_slice = (double)K / slices;
  const double panel = 256.0 * k_slice * 2.0;  // bytes of weights one tile streams
  const double mfma_pace = k_slice / 64.0 * 1.3e-6 * fmin(1.0, rows_hi / 256.0);
  const double by_flops = 2.0 * mats * est_rows * (double)n_out * K / 1.2e15;
  double tiled;
  if (gateup) {
    const double by_rounds = fmax(units / 256.0, 1.0) * (fmax(panel / 45e9, mfma_pace) + 8e-6);
    const double by_hbm = units * panel / 5.7e12 + 4e-6;  // all tiles together: their panels at the HBM rate
    tiled = fmax(fmax(by_rounds, by_hbm), by_flops);
  } else {
    const double per_cu = fmin(45e9, 5.4e12 / fmin(units, 256.0));
    tiled = fmax(fmax(units / 256.0, 1.0) * (fmax(panel / per_cu, mfma_pace) + 8e-6), by_flops);
  }
  return walk < tiled;
}

// Row-block height of the tiled kernels for a call: 160 (the one-height list) or 256.
// The 160-row tiling pays where it saves the second stream of an expert's weights (or a padded
// 256-row tile) without adding a block: with the rows per expert just below a multiple of 160.
// Measured, gate/up + down projection in us, 256-row tiling against 160-row tiling, by average rows
// per expert: Qwen1.5-MoE (60 experts) 102: 243 / 243; 136: 275 / 254; 170: 296 / 359; 204: 301 / 392;
// 238: 323 / 397; 273: 441 / 402; 307: 488 / 435; 341: 497 / 522; 409: 512 / 534; Qwen2-57B (64
// experts) 128: 830 / 753; 192: 895 / 1141; 256: 1206 / 1172; 320: 1593 / 1408; 384: 1518 / 1645.
// With 30 local experts (273 rows each) the two are equal, with 8 large experts the 160-row tiling
// loses a fifth, hence the expert count in the rule.
#ifndef MOE_EVEN_MODE
#define MOE_EVEN_MODE 0  // 1: always 160, 2: never (tuning builds)
#endif
inline bool prefer_even(int est_rows, int n_local, int H, int I_s) {
  (void)H;
  (void)I_s;
  if (MOE_EVEN_MODE != 0) return MOE_EVEN_MODE == 1;
  const double avg = (double)est_rows / n_local;
  return n_local >= 32 && ((avg >= 115.0 && avg <= 148.0) || (avg >= 255.0 && avg <= 330.0));
}

}  // namespace

int tiled_block_rows(int cap_rows, int est_rows, int n_local, int H, int I_s) {
  (void)cap_rows;
  return prefer_even(est_rows, n_local, H, I_s) ? gg::kEvenRows : 256;
}

size_t ffn_workspace_bytes(int cap_rows, int est_rows, int n_local, int H, int I_s) {
  if (cap_rows == 0) return 0;
  // what the tiled kernels need is always covered: MOE_FFN_TILED may overrule the estimate
  const size_t tiled = (size_t)gg::slice_plan(cap_rows, (H + 255) / 256, I_s).scratch_rows * H * sizeof(float);
  if (!prefer_walk(cap_rows, est_rows, n_local, H, I_s, false)) return tiled;
  const gw::WalkPlan p2 = gw::plan_for(I_s, decode_mt(cap_rows, est_rows, n_local), true);
  const int slices = p2.nw == 0 ? 1 : p2.slices;
  const size_t walk = slices > 1 ? (size_t)slices * cap_rows * H * sizeof(float) : 0;
  return walk > tiled ? walk : tiled;
}

void ffn_plan(int cap_rows, int est_rows, int n_local, int H, int I_s, int32_t out[4]) {
  const bool walk1 = prefer_walk(cap_rows, est_rows, n_local, I_s, H, true),
             walk2 = prefer_walk(cap_rows, est_rows, n_local, H, I_s, false);
  const int mt = decode_mt(cap_rows, est_rows, n_local);
  out[0] = walk1;
  out[1] = walk2;
  out[2] = mt;
  if (walk2) {
    const gw::WalkPlan p2 = gw::plan_for(I_s, mt, true);
    out[3] = p2.nw == 0 ? 1 : p2.slices;
  } else {
    out[3] = gg::slice_plan(cap_rows, (H + 255) / 256, I_s).max_slices;
  }
}

hipError_t launch_expert_ffn(const void* x_perm, RowMap rows, const int32_t* expert_offsets, int cap_rows, int est_rows,
                             int n_local, int H, int I_s, const void* w_gate, const void* w_up, const void* w_down,
                             void* h_ws, void* y_perm, void* workspace, size_t workspace_bytes, uint32_t flags,
                             hipStream_t stream) {
  (void)workspace_bytes;
  if (cap_rows == 0) return hipSuccess;
  // each GEMM picks its kernel family on its own: h is row-major bf16 for both
  const int mt = decode_mt(cap_rows, est_rows, n_local);
  const bool even = prefer_even(est_rows, n_local, H, I_s);
  auto run = [&](bool walk, uint32_t f) {
    if (!walk && even)
      return launch_pair_even(x_perm, rows, expert_offsets, cap_rows, n_local, H, I_s, w_gate, w_up, w_down, h_ws,
                              y_perm, f, stream);
    if (!walk)
      return launch_pair_dlds<256>(x_perm, rows, expert_offsets, cap_rows, est_rows, n_local, H, I_s, w_gate, w_up, w_down,
                                   h_ws, y_perm, workspace, f, stream);
    if (mt == 1)
      return launch_pair_decode<1>(x_perm, rows, expert_offsets, cap_rows, n_local, H, I_s, w_gate, w_up, w_down, h_ws,
                                   y_perm, workspace, f, stream);
    return launch_pair_decode<2>(x_perm, rows, expert_offsets, cap_rows, n_local, H, I_s, w_gate, w_up, w_down, h_ws,
                                 y_perm, workspace, f, stream);
  };
  const bool tiled_only = (flags & MOE_FFN_TILED) != 0;
  const bool walk1 = !tiled_only && prefer_walk(cap_rows, est_rows, n_local, I_s, H, true),
             walk2 = !tiled_only && prefer_walk(cap_rows, est_rows, n_local, H, I_s, false);
  if (walk1 == walk2 || (flags & (MOE_FFN_SKIP_GATEUP | MOE_FFN_SKIP_DOWN)))
    return run((flags & MOE_FFN_SKIP_GATEUP) ? walk2 : walk1, flags);
  const hipError_t err = run(walk1, flags | MOE_FFN_SKIP_DOWN);
  if (err != hipSuccess) return err;
  return run(walk2, flags | MOE_FFN_SKIP_GATEUP);
}

}  // namespace moe
