// Token permutation by expert: the dispatch step of the Top-K mechanism (paper, "MoE Model
// Architectures"), restricted to the contiguous expert subset an expert-parallel shard holds
// ("Expert Parallelism").  A stable counting sort of assignment ids a = t*k + j by expert id.
//
// Index kernel for small batches: one 1024-thread workgroup.  Pass 1 builds the per-expert histogram with LDS
// integer atomics (order-independent result) and scans it.  Pass 2 walks the assignments in
// order, 1024 at a time: inside a wavefront the rank among equal experts comes from ballot +
// popcount, across the 16 wavefronts from a short serial prefix in LDS -- no order-dependent
// atomics, so the result is the unique stable order and is identical from run to run.
// Gather kernel: coalesced 16-byte-per-lane row copies x[row_src[r] / k] -> x_perm[r].
#include "moe_internal.hpp"

#include <mutex>

namespace moe {
namespace {

// Scratch of moe_permute_static: the per-workgroup expert counts of the large-batch path, in device
// memory that belongs to the library (each GPU the library runs on holds its own copy until the
// process ends).  The name below is a host-side handle only; host code uses the address that
// static_scratch() resolves per device.
constexpr size_t kStaticScratchInts = MOE_PERMUTE_STATIC_MAX_COUNTS;  // 1 MiB
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, resolved once per device.
hipError_t static_scratch(int32_t** out) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess) return err;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

constexpr int kIdxThreads = 1024;
constexpr int kIdxWaves = kIdxThreads / kWave;

__global__ __launch_bounds__(kIdxThreads) void permute_index_kernel(const int32_t* __restrict__ topk_idx, int A,
                                                                   int n_local, int offset,
                                                                   int32_t* __restrict__ expert_offsets,
                                                                   int32_t* __restrict__ row_src,
                                                                   int32_t* __restrict__ slot_row,
                                                                   const uint4* __restrict__ x, int k,
                                                                   int chunks_per_row, uint4* __restrict__ x_perm) {
  __shared__ int32_t base[MOE_MAX_EXPERTS];                   // next free row of each expert
  __shared__ int32_t wave_cnt[kIdxWaves][MOE_MAX_EXPERTS];    // per-wave counts, then per-wave bases
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;

  for (int e = tid; e < n_local; e += kIdxThreads) base[e] = 0;
  __syncthreads();
  for (int a = tid; a < A; a += kIdxThreads) {
    const int e = topk_idx[a] - offset;
    if (e >= 0 && e < n_local) atomicAdd(&base[e], 1);
  }
  __syncthreads();
  if (wv == 0) {  // exclusive scan of up to 256 counts by one wavefront, 64 at a time
    int carry = 0;
    for (int e0 = 0; e0 < n_local; e0 += kWave) {
      const int e = e0 + lane;
      const int c = (e < n_local) ? base[e] : 0;
      int incl = c;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int v = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += v;
      }
      if (e < n_local) {
        base[e] = carry + incl - c;
        expert_offsets[e] = carry + incl - c;
      }
      carry += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) expert_offsets[n_local] = carry;
  }
  __syncthreads();

  for (int a0 = 0; a0 < A; a0 += kIdxThreads) {
    for (int i = tid; i < kIdxWaves * n_local; i += kIdxThreads) wave_cnt[i / n_local][i % n_local] = 0;
    __syncthreads();
    const int a = a0 + tid;
    int e = -1;
    if (a < A) {
      e = topk_idx[a] - offset;
      if (e < 0 || e >= n_local) e = -1;
    }
    int rank = 0;
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int le = __shfl(e, leader, kWave);
      const unsigned long long m = __ballot(e == le);
      if (e == le) rank = __popcll(m & ((1ull << lane) - 1ull));
      if (lane == leader) wave_cnt[wv][le] = __popcll(m);
      todo &= ~m;
    }
    __syncthreads();
    for (int ee = tid; ee < n_local; ee += kIdxThreads) {
      int run = base[ee];
#pragma unroll
      for (int w = 0; w < kIdxWaves; ++w) {
        const int c = wave_cnt[w][ee];
        wave_cnt[w][ee] = run;
        run += c;
      }
      base[ee] = run;
    }
    __syncthreads();
    if (a < A) {
      if (e >= 0) {
        const int row = wave_cnt[wv][e] + rank;
        slot_row[a] = row;
        row_src[row] = a;
      } else {
        slot_row[a] = -1;
      }
    }
    __syncthreads();
  }
  // decode-sized batches: the same workgroup also gathers the rows (x != nullptr), saving a launch
  if (x != nullptr) {
    const int R = base[n_local - 1];  // after the last chunk, base[e] is the end of expert e's rows
    const int total = R * chunks_per_row;
    for (int i = tid; i < total; i += kIdxThreads) {
      const int r = i / chunks_per_row, c = i - r * chunks_per_row;
      x_perm[(size_t)r * chunks_per_row + c] = x[(size_t)(row_src[r] / k) * chunks_per_row + c];
    }
  }
}

// ---- large batches: the same stable order from three short kernels over many workgroups.
// (1) every workgroup ranks its own 1024 assignments (ballot inside a wavefront, serial prefix
// over its 16 wavefronts) and publishes its per-expert counts; (2) one workgroup turns the counts
// into per-(workgroup, expert) base rows (scan over workgroups, then over experts); (3) every
// workgroup adds its bases.  No atomics on the value path: the order is the unique stable one.
__global__ __launch_bounds__(kIdxThreads) void permute_rank_kernel(const int32_t* __restrict__ topk_idx, int A,
                                                                  int n_local, int offset,
                                                                  int32_t* __restrict__ block_counts,
                                                                  int32_t* __restrict__ slot_row) {
  __shared__ int32_t wave_cnt[kIdxWaves][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  for (int i = tid; i < kIdxWaves * n_local; i += kIdxThreads) wave_cnt[i / n_local][i % n_local] = 0;
  __syncthreads();
  const int a = blockIdx.x * kIdxThreads + tid;
  int e = -1;
  if (a < A) {
    e = topk_idx[a] - offset;
    if (e < 0 || e >= n_local) e = -1;
  }
  int rank = 0;
  unsigned long long todo = __ballot(e >= 0);
  while (todo) {
    const int leader = __ffsll((long long)todo) - 1;
    const int le = __shfl(e, leader, kWave);
    const unsigned long long m = __ballot(e == le);
    if (e == le) rank = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == leader) wave_cnt[wv][le] = __popcll(m);
    todo &= ~m;
  }
  __syncthreads();
  for (int ee = tid; ee < n_local; ee += kIdxThreads) {
    int run = 0;
#pragma unroll
    for (int w = 0; w < kIdxWaves; ++w) {
      const int c = wave_cnt[w][ee];
      wave_cnt[w][ee] = run;
      run += c;
    }
    block_counts[(size_t)blockIdx.x * n_local + ee] = run;
  }
  __syncthreads();
  // hand-over to the place kernel through slot_row: rank inside the workgroup (< 1024) in the low
  // 10 bits, local expert (< 256) above them
  if (a < A) slot_row[a] = (e >= 0) ? ((e << 10) | (wave_cnt[wv][e] + rank)) : -1;
}

__global__ __launch_bounds__(256) void permute_scan_kernel(int32_t* __restrict__ block_counts, int n_blocks,
                                                          int n_local, int32_t* __restrict__ expert_offsets) {
  __shared__ int32_t total[MOE_MAX_EXPERTS];
  const int tid = threadIdx.x;
  for (int e = tid; e < n_local; e += 256) {
    int run = 0;
    for (int b = 0; b < n_blocks; ++b) {
      const int c = block_counts[(size_t)b * n_local + e];
      block_counts[(size_t)b * n_local + e] = run;
      run += c;
    }
    total[e] = run;
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < n_local; ++e) {
      const int c = total[e];
      total[e] = run;
      expert_offsets[e] = run;
      run += c;
    }
    expert_offsets[n_local] = run;
  }
  __syncthreads();
  for (int i = tid; i < n_blocks * n_local; i += 256) block_counts[i] += total[i % n_local];
}

__global__ __launch_bounds__(kIdxThreads) void permute_place_kernel(int A, int n_local,
                                                                   const int32_t* __restrict__ block_bases,
                                                                   int32_t* __restrict__ row_src,
                                                                   int32_t* __restrict__ slot_row) {
  const int a = blockIdx.x * kIdxThreads + threadIdx.x;
  if (a >= A) return;
  const int v = slot_row[a];
  if (v < 0) return;
  const int e = v >> 10, rank = v & 1023;
  const int row = block_bases[(size_t)blockIdx.x * n_local + e] + rank;
  slot_row[a] = row;
  row_src[row] = a;
}

constexpr int kGatherThreads = 256;

__global__ __launch_bounds__(kGatherThreads) void gather_rows_kernel(const uint4* __restrict__ x,
                                                                    const int32_t* __restrict__ row_src,
                                                                    const int32_t* __restrict__ expert_offsets,
                                                                    int n_local, int k, int chunks_per_row,
                                                                    uint4* __restrict__ x_perm) {
  const int R = expert_offsets[n_local];
  for (int r = blockIdx.x; r < R; r += gridDim.x) {
    const int tok = row_src[r] / k;
    const uint4* src = x + (size_t)tok * chunks_per_row;
    uint4* dst = x_perm + (size_t)r * chunks_per_row;
    for (int c = threadIdx.x; c < chunks_per_row; c += kGatherThreads) dst[c] = src[c];
  }
}

}  // namespace

size_t permute_workspace_bytes(int T, int k, int n_local) {
  const size_t blocks = ((size_t)T * k + kIdxThreads - 1) / kIdxThreads;
  return 256 + blocks * n_local * sizeof(int32_t);
}

size_t permute_static_counts(int T, int k, int n_local) {
  const size_t A = (size_t)T * k;
  if (A <= 2 * kIdxThreads) return 0;  // the one-workgroup path keeps its counts in LDS
  return (A + kIdxThreads - 1) / kIdxThreads * n_local;
}

hipError_t launch_permute_static(const void* x, const int32_t* topk_idx, int T, int k, int H, int n_local, int offset,
                                 void* x_perm, int32_t* expert_offsets, int32_t* row_src, int32_t* slot_row,
                                 hipStream_t stream) {
  int32_t* ptr = nullptr;
  const hipError_t err = static_scratch(&ptr);
  if (err != hipSuccess) return err;
  // every count the scan and place kernels read was written by the rank kernel of the same call:
  // nothing has to start at zero, whatever the last call left behind
  return launch_permute(x, topk_idx, T, k, H, n_local, offset, x_perm, expert_offsets, row_src, slot_row, ptr, stream);
}

hipError_t launch_permute(const void* x, const int32_t* topk_idx, int T, int k, int H, int n_local, int offset,
                          void* x_perm, int32_t* expert_offsets, int32_t* row_src, int32_t* slot_row,
                          void* workspace, hipStream_t stream) {
  const int A = T * k;
  hipError_t err;
  if (A <= 2 * kIdxThreads) {  // small batch: one workgroup does it all in one launch
    const bool fuse = x_perm != nullptr && (size_t)A * H * 2 <= (256u << 10);
    hipLaunchKernelGGL(permute_index_kernel, dim3(1), dim3(kIdxThreads), 0, stream, topk_idx, A, n_local, offset,
                       expert_offsets, row_src, slot_row, fuse ? static_cast<const uint4*>(x) : nullptr, k, H / 8,
                       static_cast<uint4*>(x_perm));
    err = hipGetLastError();
    if (fuse) return err;
  } else {
    const int blocks = (A + kIdxThreads - 1) / kIdxThreads;
    int32_t* counts = static_cast<int32_t*>(workspace);
    hipLaunchKernelGGL(permute_rank_kernel, dim3(blocks), dim3(kIdxThreads), 0, stream, topk_idx, A, n_local, offset,
                       counts, slot_row);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(256), 0, stream, counts, blocks, n_local, expert_offsets);
    hipLaunchKernelGGL(permute_place_kernel, dim3(blocks), dim3(kIdxThreads), 0, stream, A, n_local, counts, row_src,
                       slot_row);
    err = hipGetLastError();
  }
  if (err != hipSuccess || A == 0 || x_perm == nullptr) return err;  // index only: the caller gathers on the fly
  const int grid = A < 8192 ? A : 8192;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(grid), dim3(kGatherThreads), 0, stream,
                     static_cast<const uint4*>(x), row_src, expert_offsets, n_local, k, H / 8,
                     static_cast<uint4*>(x_perm));
  return hipGetLastError();
}

}  // namespace moe
