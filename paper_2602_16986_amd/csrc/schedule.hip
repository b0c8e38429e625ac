// Jagged-offset tile scheduler and relative-bias expansion (gfx950).
//
// The scheduler turns seq_offsets (+ num_targets and the mask parameters K1, K2) into an
// ordered list of work items (sequence, block of rows, head).  Fully masked column tiles
// are never visited: every kernel enumerates the visible tiles of its block with
// tile_ranges()/row_tile_ranges(), and the scheduler uses the same functions to price
// each block so that expensive blocks start first (longest-processing-time order) while
// neighbouring blocks of one (sequence, head) stay adjacent in the list; the attention
// kernels then map list positions to accelerator dies so that such neighbours share one
// die's L2 for their K/V stream.  Semi-local attention costs O((K1+K2) L) only because
// of this skipping (paper Section 4.2.1).
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {

constexpr int kSchedThreads = 1024;
constexpr int kSortMax = 8192;       // lists up to this size are sorted by cost in LDS
constexpr int kSeqCache = 2048;      // batches up to this size keep their block prefix sums and lengths in LDS

// One workgroup builds one list; the backward pass launches two (dQ blocks and dK/dV blocks) side by side.
struct SchedJob {
  int block_rows, tile_cols, key_major;
  SchedHeader* header;
  WorkItem* items;
  int32_t* seq_base;
};

__global__ __launch_bounds__(kSchedThreads) void schedule_kernel(const int32_t* __restrict__ offsets,
                                                                 const int32_t* __restrict__ num_targets, int B, int H,
                                                                 int K1, int K2, SchedJob job0, SchedJob job1) {
  const SchedJob job = blockIdx.x == 0 ? job0 : job1;
  const int block_rows = job.block_rows, tile_cols = job.tile_cols, key_major = job.key_major;
  SchedHeader* header = job.header;
  WorkItem* items = job.items;
  int32_t* seq_base = job.seq_base;
  __shared__ int32_t scan[kSchedThreads];
  __shared__ uint32_t keys[kSortMax];
  __shared__ WorkItem staged[kSortMax];                  // items in natural order, permuted by the sort at the end
  __shared__ int32_t base_c[kSeqCache + 1], len_c[kSeqCache], hist_c[kSeqCache];
  const bool cached = B <= kSeqCache;                    // else the searches below read seq_base / offsets from global memory
  __shared__ int32_t carry_s;
  __shared__ unsigned long long tiles_s, dense_s;
  const int tid = threadIdx.x;
  if (tid == 0) { carry_s = 0; tiles_s = 0; dense_s = 0; }
  __syncthreads();

  // 1. exclusive scan of blocks-per-sequence -> seq_base[b] (per head)
  for (int c0 = 0; c0 < B; c0 += kSchedThreads) {
    const int b = c0 + tid;
    int nb = 0;
    if (b < B) nb = (offsets[b + 1] - offsets[b] + block_rows - 1) / block_rows;
    scan[tid] = nb;
    __syncthreads();
    for (int off = 1; off < kSchedThreads; off <<= 1) {
      int v = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += v;
      __syncthreads();
    }
    const int carry = carry_s;
    if (b < B) {
      seq_base[b] = carry + scan[tid] - nb;
      if (cached) {
        const int L = offsets[b + 1] - offsets[b];
        base_c[b] = carry + scan[tid] - nb;
        len_c[b] = L;
        hist_c[b] = L - (num_targets ? num_targets[b] : 0);
      }
    }
    __syncthreads();
    if (tid == kSchedThreads - 1) carry_s = carry + scan[tid];
    __syncthreads();
  }
  const int blocks_per_head = carry_s;
  if (tid == 0) {
    seq_base[B] = blocks_per_head;
    if (cached) base_c[B] = blocks_per_head;
  }
  __threadfence_block();
  __syncthreads();
  const int total = blocks_per_head * H;                 // <= max_items by construction of the bound

  // 2. natural order: sequence-major, then head, then block index descending.  Item idx -> (b, h, rb).
  const bool sorted = total <= kSortMax;
  // exact longest-first order measured best: the heaviest block is half of one compute unit's whole
  // share on the 8k-16k workload, so any coarsening of the order shows up as tail imbalance
  const int cost_quantum = 1;
  unsigned long long my_tiles = 0, my_dense = 0;
  for (int idx = tid; idx < total; idx += kSchedThreads) {
    // find b with seq_base[b]*H <= idx < seq_base[b+1]*H
    int lo = 0, hi = B;                                  // invariant: seq_base[lo]*H <= idx < seq_base[hi]*H
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if ((long long)(cached ? base_c[mid] : seq_base[mid]) * H <= idx) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int base_b = cached ? base_c[b] : seq_base[b];
    const int nb = (cached ? base_c[b + 1] : seq_base[b + 1]) - base_b;
    const int local = idx - base_b * H;
    const int h = local / nb;
    const int rb = nb - 1 - (local % nb);
    const int L = cached ? len_c[b] : offsets[b + 1] - offsets[b];
    SeqGeom g = {L, cached ? hist_c[b] : L - (num_targets ? num_targets[b] : 0), K1, K2};
    const int r0 = rb * block_rows, r1 = min(r0 + block_rows, L) - 1;
    const TileRanges tr = key_major ? row_tile_ranges(g, r0, r1, tile_cols) : tile_ranges(g, r0, r1, tile_cols);
    const int cost = tr.count();
    my_tiles += cost;
    my_dense += (L + tile_cols - 1) / tile_cols;
    if (sorted) {
      // ties keep the natural order: the heads of one (sequence, block) stay adjacent
      const uint32_t cq = min((uint32_t)cost / (uint32_t)cost_quantum, 0x7FFFFu);
      keys[idx] = ((0x7FFFFu - cq) << 13) | (uint32_t)idx;        // idx < 8192 = 2^13
      staged[idx].b = b;
      staged[idx].rb_h = (rb << 8) | h;
    } else {
      items[idx].b = b;
      items[idx].rb_h = (rb << 8) | h;
    }
  }
  for (int off = 32; off > 0; off >>= 1) {                 // one LDS atomic per wave, not per thread
    my_tiles += __shfl_xor(my_tiles, off, 64);
    my_dense += __shfl_xor(my_dense, off, 64);
  }
  if ((tid & 63) == 0) {
    atomicAdd(&tiles_s, my_tiles);
    atomicAdd(&dense_s, my_dense);
  }
  __syncthreads();
  if (tid == 0) {
    header->count = total;
    header->pad = 0;
    header->tiles = (int64_t)tiles_s;
    header->dense_tiles = (int64_t)dense_s;
  }
  if (!sorted) return;

  // 3. bitonic sort of the keys (ascending = most expensive first), padded to a power of two
  int n2 = 1;
  while (n2 < total) n2 <<= 1;
  for (int idx = total + tid; idx < n2; idx += kSchedThreads) keys[idx] = 0xFFFFFFFFu;
  __syncthreads();
  // Element i = tid + 1024*m is held by thread tid; compare-exchange partners at distance j < 64 are lanes of
  // the same wave, so those sub-stages run in registers with lane shuffles and need no barrier.
  const int lane = tid & 63;
  auto wave_stages = [&](int k, int jmax) {                // sub-stages j = jmax, jmax/2, ..., 1 of phase k
    for (int i = tid; i < n2; i += kSchedThreads) {
      uint32_t a = keys[i];
      const bool up = (i & k) == 0;
      for (int j = jmax; j > 0; j >>= 1) {
        const uint32_t c = (uint32_t)__shfl_xor((int)a, j, 64);
        const bool keep_min = ((lane & j) == 0) == up;
        a = keep_min ? min(a, c) : max(a, c);
      }
      keys[i] = a;
    }
    __syncthreads();
  };
  for (int k = 2; k <= n2; k <<= 1) {
    int j = k >> 1;
    for (; j >= 64; j >>= 1) {
      for (int i = tid; i < n2; i += kSchedThreads) {
        const int ixj = i ^ j;
        if (ixj > i) {
          const uint32_t a = keys[i], c = keys[ixj];
          const bool up = (i & k) == 0;
          if ((a > c) == up) { keys[i] = c; keys[ixj] = a; }
        }
      }
      __syncthreads();
    }
    if (j > 0) wave_stages(k, j);
  }
  for (int pos = tid; pos < total; pos += kSchedThreads) items[pos] = staged[keys[pos] & 0x1FFF];
}

hipError_t launch_schedule(const AttnArgs& a, int block_rows, int tile_cols, bool key_major, SchedHeader* header,
                           WorkItem* items, int32_t* seq_base, hipStream_t stream) {
  const SchedJob job = {block_rows, tile_cols, key_major ? 1 : 0, header, items, seq_base};
  hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(kSchedThreads), 0, stream, a.offsets, a.num_targets, a.B, a.H, a.K1,
                     a.K2, job, job);
  return hipGetLastError();
}

hipError_t launch_schedule_pair(const AttnArgs& a, const int block_rows[2], const int tile_cols[2], SchedHeader* const header[2],
                                WorkItem* const items[2], int32_t* const seq_base[2], hipStream_t stream) {
  const SchedJob j0 = {block_rows[0], tile_cols[0], 0, header[0], items[0], seq_base[0]};
  const SchedJob j1 = {block_rows[1], tile_cols[1], 1, header[1], items[1], seq_base[1]};
  hipLaunchKernelGGL(schedule_kernel, dim3(2), dim3(kSchedThreads), 0, stream, a.offsets, a.num_targets, a.B, a.H, a.K1,
                     a.K2, j0, j1);
  return hipGetLastError();
}

// bias_by_distance[h, x] = log2(e) * table[h, bucket(x)], bucket(x) = max{c : bounds[c] <= x}, for x in [0, len):
// the attention kernels keep their scores in units of ln 2.
__global__ __launch_bounds__(256) void bias_expand_kernel(const float* __restrict__ table,
                                                          const int32_t* __restrict__ bounds, int nb, int H, int len,
                                                          float* __restrict__ out) {
  const int x = blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= len) return;
  int lo = 0, hi = nb;                                   // bounds[lo] <= x < bounds[hi] (bounds[nb] = +inf)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (bounds[mid] <= x) lo = mid; else hi = mid;
  }
  for (int h = 0; h < H; ++h) out[(size_t)h * len + x] = table[(size_t)h * nb + lo] * 1.4426950408889634f;
}

hipError_t launch_bias_expand(const float* table, const int32_t* bounds, int num_buckets, int H, int len, float* out,
                              hipStream_t stream) {
  hipLaunchKernelGGL(bias_expand_kernel, dim3((len + 255) / 256), dim3(256), 0, stream, table, bounds, num_buckets, H,
                     len, out);
  return hipGetLastError();
}

}  // namespace hstu
