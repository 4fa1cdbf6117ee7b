// Records shared by the host side (pool, batch translation) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace plora {

constexpr int kWave = 64;              // one work item = one wavefront = one workgroup
constexpr int kMaxSlotsPerLaunch = 128; // pointer pairs carried in the kernel arguments
constexpr int kShrinkRows = 8;         // rows of A per vector-ALU shrink item
constexpr int kValuTok = 4;            // tokens per vector-ALU item
constexpr int kMfmaTok = 64;           // tokens per matrix-core item (4 tiles of 16)
constexpr int kMfmaRows = 16;          // rows of A per matrix-core shrink item (one 16-wide tile)
constexpr int kMfmaCols = 128;         // columns of B per matrix-core expand item
constexpr int kPtWindow = 1024;        // page-table entries a shrink item may stage in LDS
constexpr int kMaxRank = 512;          // rows of B an expand item may stage page pairs for

// One group of tokens that share an adapter (a "segment" of the sorted batch).
struct SegRec {
  int32_t tok_start;  // first entry of the group in perm
  int32_t n_tok;
  int32_t rank;
  int32_t pt_off;     // first entry of the adapter's page table in the batch's table array
  float scale;
  int32_t adapter;
  int32_t n_pt;
  int32_t pad;
};

// One wavefront's worth of work.
struct ItemRec {
  int32_t seg;
  int32_t tok0;   // first token of the item inside its group
  int32_t ntok;   // tokens of the item (<= kValuTok or <= kMfmaTok)
  int32_t j0;     // shrink: first row of A;  expand: unused
};

struct SlotRec {
  int32_t d_in, d_out;
  int64_t cum;  // sum over earlier slots of (d_in + d_out): elements per rank before this slot
};

struct SlotPtrs {
  const void* a[kMaxSlotsPerLaunch];  // shrink: x   expand: v
  void* b[kMaxSlotsPerLaunch];        // shrink: v   expand: y
};

struct LaunchArgs {
  const uint8_t* slab;
  const SegRec* segs;
  const int32_t* perm;
  const int32_t* pt;
  const ItemRec* items;
  const SlotRec* slots;   // indexed by absolute slot number
  int32_t n_items;
  int32_t slot0;
  int32_t log2_page;
  int32_t v_stride;       // = max_rank
  int32_t pad;
};

// Launchers (plora_kernels.hip).  kind: 0 = vector-ALU items, 1 = matrix-core items.
// Shrink grid: (n_items, 1, n_slots).  Expand grid: (n_items, max_chunks, n_slots) where a chunk is
// 64 * 16 bytes of a row of B for vector-ALU items and kMfmaCols columns for matrix-core items.
hipError_t launch_shrink(int dtype, int kind, const LaunchArgs& a, const SlotPtrs& p, int n_slots, hipStream_t st);
hipError_t launch_expand(int dtype, int kind, const LaunchArgs& a, const SlotPtrs& p, int n_slots, int max_chunks,
                         hipStream_t st);

}  // namespace plora
