// Order of the k blocks of a weight row block in memory (host and device; no HIP types, so that the host tests can
// include it).
#pragma once

#if defined(__HIPCC__)
#define RL_WEIGHT_ORDER_HD __host__ __device__
#else
#define RL_WEIGHT_ORDER_HD
#endif

namespace rl {

// The K range of a product is cut into segments of `seg` k blocks, four consecutive segments per K split, one per
// wave of a block.  Memory holds the k blocks of the four segments of a split interleaved -- block i of segment 0,
// of 1, of 2, of 3, then block i + 1 of each -- so that what the four waves of a block read at about the same time
// is one contiguous 16 KiB piece per row block instead of four pieces a quarter of the split apart (measured: 7 us of
// 42 on the gate/up stream at 32 rows).
RL_WEIGHT_ORDER_HD inline int weight_kb_slot(int kb, int seg) {
  const int s = kb / seg, i = kb - s * seg;
  return ((s >> 2) * seg + i) * 4 + (s & 3);
}

}  // namespace rl
