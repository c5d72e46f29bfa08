// Plain data shared by the host-side planning code and the kernels: no HIP types here, so that the
// planning code also builds with an ordinary host compiler (and its sanitizers).
#pragma once
#include <stdint.h>

namespace mc {

// One unit of attention work: a tile of stacked query rows of one (request, KV head).
// Stacked row index = token_in_chunk * G + head_in_group, so one K/V tile in LDS
// feeds all G query heads of the group.
struct AttnItem {
  int32_t req;
  int32_t kv_head;
  int32_t row0;   // first stacked row of the tile
  int32_t slice;  // key slice of the request this item covers (split launches only, else 0)
};

struct AttnReq {
  int32_t q_off;   // index of the request's first new token in q / out
  int32_t prefix;  // P_r
  int32_t chunk;   // C_r
  int32_t pages;   // ceil((P_r + C_r) / S): entries of the block-table row that may be read
};

// rows of stacked queries one attention workgroup covers (8 waves of 32 rows, both dtypes)
constexpr int kAttnTileRows = 256;
// keys of one LDS tile; key slices of the split form are whole tiles
constexpr int kAttnTileKeys = 64;
// 16-byte vectors of a page one copy workgroup moves (512 threads, one vector each)
constexpr int kKvCopySliceVecs = 512;
// the work list is kept in this many lists, one per XCD of the chip
constexpr int kXcds = 8;

}  // namespace mc
