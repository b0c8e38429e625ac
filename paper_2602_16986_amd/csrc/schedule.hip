// Jagged-offset tile scheduler and relative-bias expansion (gfx950).
//
// The scheduler turns seq_offsets (+ num_targets and the mask parameters K1, K2) into an
// ordered list of work items (sequence, block of rows, head).  Fully masked column tiles
// are never visited: every kernel enumerates the visible tiles of its block with
// tile_ranges()/row_tile_ranges(), and the scheduler uses the same functions to price
// each block so that expensive blocks start first (longest-processing-time order).  In the
// key-major list of the dK/dV pass a block far longer than the average (the key blocks of a
// global prefix, which every query of the sequence sees) is cut into pieces along the query
// axis; the pieces write partial sums that a small kernel adds up in a fixed order.
// The cost of a block does not depend on the head, so pricing, cutting and sorting work on (sequence, block) pairs
// and every entry of the sorted list is written once per head (heads adjacent): a single workgroup does all of this,
// and its time grows with the number of keys it sorts.
// Semi-local attention costs O((K1+K2) L) only because of the skipping (paper Section 4.2.1).
#include "hstu_common.h"
#include "hstu_kernels.h"

namespace hstu {

constexpr int kSchedThreads = 1024;
constexpr int kSortMax = 8192;       // lists of up to this many (sequence, block) pairs are sorted by cost in LDS
constexpr int kSeqCache = 1024;      // batches up to this size keep their block prefix sums and lengths in LDS
constexpr int kItemsPerThread = kSortMax / kSchedThreads;
constexpr int kMinChunk = 8;         // a long key block is cut into pieces of at least this many tiles ...
constexpr int kTargetChunks = 2048;  // ... and of about 1/2048 of all scheduled tiles (4 per workgroup slot of the chip)
constexpr int kFwdTargetChunks = 1536;   // forward lists: 2 x chunk = one slot's share when 768 workgroups are resident
constexpr int kDqTargetChunks = 1024;    // dQ lists: the same with 512 resident workgroups

// One workgroup builds one list; the backward pass launches two (dQ blocks and dK/dV blocks) side by side.
struct SchedJob {
  int block_rows, tile_cols, key_major;
  int query_tail;                     // > 0 (query-major lists only): only the blocks that hold the last query_tail history rows or candidates
  int slot_cap;            // > 0: blocks much longer than the average may be cut along the streamed axis
  int even;                // cut blocks into equal pieces of at most 2 x chunk tiles (else: pieces of chunk tiles)
  int target_chunks;       // chunk = all scheduled tiles / target_chunks (at least kMinChunk)
  SchedHeader* header;
  WorkItem* items;
  int32_t* seq_base;
  SplitItem* splits;
};

// Exclusive scan of one 64-bit value per thread over the workgroup (three packed counters); returns the
// exclusive prefix and writes the grand total.
__device__ unsigned long long block_scan64(unsigned long long v, unsigned long long* lds, unsigned long long& total) {
  const int tid = threadIdx.x;
  lds[tid] = v;
  __syncthreads();
  for (int off = 1; off < kSchedThreads; off <<= 1) {
    const unsigned long long u = tid >= off ? lds[tid - off] : 0ull;
    __syncthreads();
    lds[tid] += u;
    __syncthreads();
  }
  const unsigned long long incl = lds[tid];
  total = lds[kSchedThreads - 1];
  __syncthreads();
  return incl - v;
}

__global__ __launch_bounds__(kSchedThreads) void schedule_kernel(const int32_t* __restrict__ offsets,
                                                                 const int32_t* __restrict__ num_targets, int B, int H,
                                                                 int K1, int K2, int T, int max_seqlen, SchedJob job0,
                                                                 SchedJob job1) {
  const SchedJob job = blockIdx.x == 0 ? job0 : job1;
  const int block_rows = job.block_rows, tile_cols = job.tile_cols, key_major = job.key_major, tail = job.query_tail;
  // first block of a sequence that holds a query row to compute
  auto first_block = [&](int hist) { return tail > 0 ? max(hist - tail, 0) / block_rows : 0; };
  SchedHeader* header = job.header;
  WorkItem* items = job.items;
  int32_t* seq_base = job.seq_base;
  __shared__ int32_t scan[kSchedThreads];
  __shared__ unsigned long long scan64[kSchedThreads];
  __shared__ uint32_t keys[kSortMax];                    // (inverted cost << 13) | entry
  __shared__ uint32_t entry_item[kSortMax];              // entry -> pair | (piece << 13)
  __shared__ uint16_t slot_c[kSortMax];                  // pair -> its first slot (x H: slot of head 0), 0xFFFF = not cut
  __shared__ int32_t base_c[kSeqCache + 1], len_c[kSeqCache], hist_c[kSeqCache];
  const bool cached = B <= kSeqCache;                    // else the searches below read seq_base / offsets from global memory
  __shared__ int32_t carry_s;
  __shared__ unsigned long long tiles_s, dense_s;
  const int tid = threadIdx.x;
  if (tid == 0) { carry_s = 0; tiles_s = 0; dense_s = 0; }
  __syncthreads();

  // 0. The offsets live on the device and the host may never have seen them: a batch whose offsets are not a non-decreasing
  // walk from 0 to at most T in steps of at most max_seqlen, or whose candidate counts leave [0, L], gets an empty list
  // (every kernel that follows then returns at once) instead of rows addressed outside the tensors.
  {
    int bad = 0;
    for (int b = tid; b < B; b += kSchedThreads) {
      const int o0 = offsets[b], o1 = offsets[b + 1];
      const int m = num_targets ? num_targets[b] : 0;
      bad |= (o0 < 0) | (o1 < o0) | (o1 - o0 > max_seqlen) | (o1 > T) | (m < 0) | (m > o1 - o0) | (b == 0 && o0 != 0);
    }
    if (__syncthreads_or(bad)) {
      if (tid == 0) *job.header = SchedHeader{0, 0, 0, 0, 0, 1};
      return;
    }
  }

  // 1. exclusive scan of blocks-per-sequence -> seq_base[b] (per head)
  for (int c0 = 0; c0 < B; c0 += kSchedThreads) {
    const int b = c0 + tid;
    int nb = 0;
    if (b < B) {
      const int L = offsets[b + 1] - offsets[b];
      nb = (L + block_rows - 1) / block_rows;
      if (tail > 0 && nb > 0) nb -= first_block(L - (num_targets ? num_targets[b] : 0));
    }
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
  const int pairs = blocks_per_head;                     // (sequence, block) pairs: what is priced, cut and sorted

  // natural order: sequence-major, then head, then block index descending.  Item idx of `heads` heads -> (b, h, rb) and
  // its tiles; heads = 1 enumerates the pairs.
  auto locate = [&](int idx, int heads, int& b, int& rb, int& h, int& cost, int& dense, bool want_cost) {
    int lo = 0, hi = B;                                  // invariant: seq_base[lo]*heads <= idx < seq_base[hi]*heads
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if ((long long)(cached ? base_c[mid] : seq_base[mid]) * heads <= idx) lo = mid; else hi = mid;
    }
    b = lo;
    const int base_b = cached ? base_c[b] : seq_base[b];
    const int nb = (cached ? base_c[b + 1] : seq_base[b + 1]) - base_b;
    const int local = idx - base_b * heads;
    h = local / nb;
    const int L = cached ? len_c[b] : offsets[b + 1] - offsets[b];
    SeqGeom g = {L, cached ? hist_c[b] : L - (num_targets ? num_targets[b] : 0), K1, K2};
    rb = (L + block_rows - 1) / block_rows - 1 - (local % nb);          // last block first; with a query tail the leading blocks are absent
    if (!want_cost) return;
    const int r0 = rb * block_rows, r1 = min(r0 + block_rows, L) - 1;
    const TileRanges tr = key_major ? row_tile_ranges(g, r0, r1, tile_cols) : tile_ranges(g, r0, r1, tile_cols);
    cost = tr.count();
    dense = (L + tile_cols - 1) / tile_cols;
  };

  // 2. price the pairs.  Sorted lists: thread tid owns the pairs [tid * ipt, (tid + 1) * ipt).
  const bool sorted = pairs <= kSortMax;
  const int ipt = (pairs + kSchedThreads - 1) / kSchedThreads;
  unsigned long long my_tiles = 0, my_dense = 0;
  int my_cost[kItemsPerThread];
  if (sorted) {
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
      const int idx = tid * ipt + k;
      my_cost[k] = 0;
      if (k < ipt && idx < pairs) {
        int b, rb, h, cost, dense;
        locate(idx, 1, b, rb, h, cost, dense, true);
        my_cost[k] = cost;
        my_tiles += (unsigned long long)cost * H;
        my_dense += (unsigned long long)dense * H;
      }
    }
  } else {
    for (int idx = tid; idx < total; idx += kSchedThreads) {
      int b, rb, h, cost, dense;
      locate(idx, H, b, rb, h, cost, dense, true);
      my_tiles += cost;
      my_dense += dense;
      const int Lb = offsets[b + 1] - offsets[b];
      items[idx] = WorkItem{b, (rb << 8) | h, 0, 0x7FFFFFFF, -1, offsets[b], Lb, Lb - (num_targets ? num_targets[b] : 0)};
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
  const unsigned long long all_tiles = tiles_s;
  if (!sorted) {
    if (tid == 0) *header = SchedHeader{total, 0, (int64_t)all_tiles, (int64_t)dense_s, 0, 0};
    return;
  }

  // 3. Cut blocks that are much longer than a workgroup slot's share into pieces of `chunk` tiles (key-major
  // lists only: the few key blocks of a global prefix are seen by every query of their sequence).  Each piece
  // becomes an entry of the list and accumulates into a partial-sum slot of its own (one per head).  The piece size
  // doubles until the slots and the list fit.  Packed counters, per pair: entries | slots << 20 | cut pairs << 40.
  int chunk = (int)min((unsigned long long)0x3FFFFFFF,
                       max((unsigned long long)kMinChunk, (all_tiles + job.target_chunks - 1) / (unsigned long long)job.target_chunks));
  // pieces of a block of `cost` tiles and their length: key-major lists take pieces of `chunk` tiles (a block of a global
  // prefix is hundreds of times longer than the rest); query-major lists, where the longest block is a few slot shares at
  // most, take the fewest equal pieces of at most 2 x chunk tiles (every piece costs a partial-sum slot and its traffic)
  auto pieces_of = [&](int cost, int ch) {
    if (!(job.slot_cap > 0 && cost > 2 * ch)) return 1;
    return job.even ? (cost + 2 * ch - 1) / (2 * ch) : (cost + ch - 1) / ch;
  };
  auto piece_len = [&](int cost, int pieces, int ch) { return job.even ? (cost + pieces - 1) / pieces : ch; };
  unsigned long long excl = (unsigned long long)min(tid * ipt, pairs), sum = (unsigned long long)pairs;
  while (job.slot_cap > 0) {                               // no slots: one entry per item, in natural order
    unsigned long long mine = 0;
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
      const int idx = tid * ipt + k;
      if (k < ipt && idx < pairs) {
        const int cost = my_cost[k];
        const unsigned long long pieces = (unsigned long long)pieces_of(cost, chunk);
        const bool cut = pieces > 1;
        mine += pieces | (cut ? (pieces << 20) | (1ull << 40) : 0ull);
      }
    }
    excl = block_scan64(mine, scan64, sum);
    const int entries = (int)(sum & 0xFFFFF), slots = (int)((sum >> 20) & 0xFFFFF);
    if (entries <= kSortMax && (long long)slots * H <= job.slot_cap) break;   // uniform: every thread sees the same totals
    chunk *= 2;                                                // ends: with no pair cut, entries = pairs <= kSortMax
  }
  const int entries = (int)(sum & 0xFFFFF), nsplit = (int)(sum >> 40);
  if (tid == 0) *header = SchedHeader{entries * H, nsplit * H, (int64_t)all_tiles, (int64_t)dense_s, chunk, 0};
  {
    int e = (int)(excl & 0xFFFFF), slot = (int)((excl >> 20) & 0xFFFFF), rank = (int)(excl >> 40);
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
      const int idx = tid * ipt + k;
      if (k < ipt && idx < pairs) {
        const int cost = my_cost[k];
        const int pieces = pieces_of(cost, chunk), plen = piece_len(cost, pieces, chunk);
        const bool cut = pieces > 1;
        slot_c[idx] = cut ? (uint16_t)slot : (uint16_t)0xFFFF;
        for (int c = 0; c < pieces; ++c) {
          // ties keep the natural order of the pairs (sequence-major, last block first)
          const uint32_t pc = (uint32_t)min(cut ? min(plen, cost - c * plen) : cost, 0x7FFFF);
          keys[e + c] = ((0x7FFFFu - pc) << 13) | (uint32_t)(e + c);      // entry < 8192 = 2^13
          entry_item[e + c] = (uint32_t)idx | ((uint32_t)c << 13);
        }
        if (cut) {                                       // the pieces of head h own the slots [(slot * H + h * pieces), + pieces)
          int b, rb, h, cost2, dense;
          locate(idx, 1, b, rb, h, cost2, dense, false);
          for (h = 0; h < H; ++h) job.splits[rank * H + h] = SplitItem{b, (rb << 8) | h, slot * H + h * pieces, pieces};
          slot += pieces;
          ++rank;
        }
        e += pieces;
      }
    }
  }

  // 4. bitonic sort of the keys (ascending = most expensive first), padded to a power of two
  int n2 = 1;
  while (n2 < entries) n2 <<= 1;
  __syncthreads();
  for (int idx = entries + tid; idx < n2; idx += kSchedThreads) keys[idx] = 0xFFFFFFFFu;
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
  // 5. the list.  The attention kernels keep runs of kXcdGroup consecutive items on one die; a run is made of consecutive
  // entries of one head (for equal costs these are neighbouring blocks of one sequence, which share most of the rows
  // they stream), so a group of kXcdGroup sorted entries becomes H runs, one per head.
  for (int e = tid; e < entries * H; e += kSchedThreads) {
    const int grp = e / (kXcdGroup * H), within = e - grp * (kXcdGroup * H);
    const int gsize = min(kXcdGroup, entries - grp * kXcdGroup);
    const int hh = within / gsize, pos = grp * kXcdGroup + within - hh * gsize;
    const uint32_t ei = entry_item[keys[pos] & 0x1FFF];
    const int idx = (int)(ei & 0x1FFF), c = (int)(ei >> 13);
    const bool cut = slot_c[idx] != 0xFFFF;
    int b, rb, h, cost = 0, dense;
    locate(idx, 1, b, rb, h, cost, dense, cut);
    const int pieces = cut ? pieces_of(cost, chunk) : 1, plen = piece_len(cost, pieces, chunk);
    const int sq0 = offsets[b], Lb = cached ? len_c[b] : offsets[b + 1] - sq0;
    const int hist = cached ? hist_c[b] : Lb - (num_targets ? num_targets[b] : 0);
    items[e] = cut ? WorkItem{b, (rb << 8) | hh, c * plen, min((c + 1) * plen, cost), (int)slot_c[idx] * H + hh * pieces + c, sq0, Lb, hist}
                   : WorkItem{b, (rb << 8) | hh, 0, 0x7FFFFFFF, -1, sq0, Lb, hist};
  }
}

hipError_t launch_schedule(const AttnArgs& a, int block_rows, int tile_cols, bool key_major, SchedHeader* header,
                           WorkItem* items, int32_t* seq_base, SplitItem* splits, int slot_cap, hipStream_t stream) {
  // forward lists (query-major): equal pieces of about one workgroup slot's share (768 slots at three workgroups per compute
  // unit); the forward over a query tail keeps the finer pieces of the key-major lists (few blocks, each against a whole history)
  const bool even = !key_major && a.query_tail == 0;
  const SchedJob job = {block_rows, tile_cols, key_major ? 1 : 0, key_major ? 0 : a.query_tail, splits ? slot_cap : 0, even ? 1 : 0,
                        even ? kFwdTargetChunks : kTargetChunks, header, items, seq_base, splits};
  hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(kSchedThreads), 0, stream, a.offsets, a.num_targets, a.B, a.H, a.K1,
                     a.K2, a.T, a.max_seqlen, job, job);
  return hipGetLastError();
}

hipError_t launch_schedule_pair(const AttnArgs& a, const int block_rows[2], const int tile_cols[2], SchedHeader* const header[2],
                                WorkItem* const items[2], int32_t* const seq_base[2], SplitItem* const splits[2],
                                const int slot_cap[2], hipStream_t stream) {
  // dQ list (query-major): equal pieces of about one slot's share, 512 slots at two workgroups per compute unit
  const SchedJob j0 = {block_rows[0], tile_cols[0], 0, 0, slot_cap[0], 1, kDqTargetChunks, header[0], items[0], seq_base[0], splits[0]};
  const SchedJob j1 = {block_rows[1], tile_cols[1], 1, 0, slot_cap[1], 0, kTargetChunks, header[1], items[1], seq_base[1], splits[1]};
  hipLaunchKernelGGL(schedule_kernel, dim3(2), dim3(kSchedThreads), 0, stream, a.offsets, a.num_targets, a.B, a.H, a.K1,
                     a.K2, a.T, a.max_seqlen, j0, j1);
  return hipGetLastError();
}

// bias_by_distance[h, x] = log2(e) * table[h, bucket(x)], bucket(x) = max{c : bounds[c] <= x}, for x in [0, len):
// the attention kernels keep their scores in units of ln 2.
__global__ __launch_bounds__(256) void bias_expand_kernel(const float* __restrict__ table,
                                                          const int32_t* __restrict__ bounds, int nb, int H, int len,
                                                          float* __restrict__ out, int32_t* __restrict__ bucket_end) {
  const int x = blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= len) return;
  int lo = 0, hi = nb;                                   // bounds[lo] <= x < bounds[hi] (bounds[nb] = +inf)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (bounds[mid] <= x) lo = mid; else hi = mid;
  }
  for (int h = 0; h < H; ++h) out[(size_t)h * len + x] = table[(size_t)h * nb + lo] * 1.4426950408889634f;
  if (bucket_end) bucket_end[x] = hi < nb ? bounds[hi] : 0x7FFFFFFF;
}

// Score seeds by distance (AttnArgs::seed): out[v][h][i], d = dmax - i.
__global__ __launch_bounds__(256) void seed_expand_kernel(const float* __restrict__ table, const int32_t* __restrict__ bounds,
                                                          int nb, int H, int max_seqlen, int K1, int dmax, int len,
                                                          float* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= len) return;
  const int d = dmax - i;
  const int x = d < 0 ? 0 : (d > max_seqlen ? max_seqlen : d);          // distances beyond any real pair take the last real one's bias
  int lo = 0;
  if (table) {
    int hi = nb;                                                         // bounds[lo] <= x < bounds[hi] (bounds[nb] = +inf)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (bounds[mid] <= x) lo = mid; else hi = mid;
    }
  }
  for (int h = 0; h < H; ++h) {
    const float b = table ? table[(size_t)h * nb + lo] * 1.4426950408889634f : 0.f;
    out[(size_t)h * len + i] = d < 0 ? -1e30f : b;
    out[((size_t)H + h) * len + i] = (d < 0 || (K1 >= 0 && d >= K1)) ? -1e30f : b;
  }
}

hipError_t launch_seed_expand(const float* table, const int32_t* bounds, int num_buckets, int H, int max_seqlen, int K1,
                              float* out, hipStream_t stream) {
  const int len = seed_len_for(max_seqlen);
  hipLaunchKernelGGL(seed_expand_kernel, dim3((len + 255) / 256), dim3(256), 0, stream, table, bounds, num_buckets, H,
                     max_seqlen, K1, seed_dmax_for(max_seqlen), len, out);
  return hipGetLastError();
}

hipError_t launch_bias_expand(const float* table, const int32_t* bounds, int num_buckets, int H, int len, float* out,
                              int32_t* bucket_end, hipStream_t stream) {
  hipLaunchKernelGGL(bias_expand_kernel, dim3((len + 255) / 256), dim3(256), 0, stream, table, bounds, num_buckets, H,
                     len, out, bucket_end);
  return hipGetLastError();
}

}  // namespace hstu
