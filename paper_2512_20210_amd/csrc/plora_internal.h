// Records shared by the host side (pool, batch translation) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace plora {

constexpr int kWave = 64;               // one work item = one wavefront = one workgroup
constexpr int kMaxSlotsPerLaunch = 128; // pointer pairs carried in the kernel arguments
constexpr int kShrinkRows = 8;          // rows of A per vector-ALU shrink item
constexpr int kValuTok = 4;             // tokens per vector-ALU item (1, 2 or 4)
constexpr int kExpandU = 8;             // rows of B in flight per vector-ALU expand iteration
constexpr int kMfmaTokS = 32;           // tokens per matrix-core shrink item
constexpr int kMfmaTokE = 64;           // tokens per matrix-core expand item of the panel kernel
constexpr int kMfmaTokCols = 16;        // items of at most this many tokens take the column-split form
constexpr int kMfmaColsMaxGroup = 32;   // panel batches: groups (or last blocks of groups) of at most this many
                                        // tokens are cut into column-split items (default of an option)
constexpr int kMfmaRows = 32;           // rows of A per matrix-core shrink item
constexpr int kMfmaCols = 128;          // columns of B per matrix-core expand pass
constexpr int kPtWindow = 1024;         // page-table entries a shrink item may stage in LDS
constexpr int kMaxRank = 512;           // rows of B an expand item may stage page pairs for (4 KiB of LDS)
constexpr int kItemOnce = 0x100;        // flag in ItemRec::kind
constexpr int kItemContig = 0x200;      // flag in ItemRec::kind: the adapter's pages are physically consecutive and pt_off
                                        // is its first physical page (no page table to read)
constexpr int kXcds = 8;                // consecutive workgroups go to consecutive XCDs

// One wavefront's worth of work, self-contained so that a wavefront needs a single 32-byte read
// before it can start fetching page-table entries, activations and weights.
struct ItemRec {
  int16_t kind;    // -1 = padding (nothing to do), 0 = vector-ALU item, 1 = matrix-core item; + kItemOnce if no
                   // other item of the batch reads this item's weights (they are then fetched with streaming loads)
  int16_t ntok;    // tokens of the item
  int16_t rank;    // rank of the adapter (0 = tokens without adapter: shrink only clears v)
  int16_t j0;      // shrink: first row of A;  expand: unused
  float scale;
  int32_t pt_off;  // first entry of the adapter's page table in the batch's table array (kItemContig: first physical page)
  int32_t tok[4];  // vector-ALU item (kValuTok <= 4): the token indices (unused entries repeat the last one);
                   // matrix-core item: tok[0] = index of the item's first token in perm
};
static_assert(sizeof(ItemRec) == 32, "ItemRec must stay 32 bytes");

struct SlotRec {
  int32_t d_in, d_out;
  int64_t cum;  // sum over earlier slots of (d_in + d_out): elements per rank before this slot
};

struct SlotPtrs {
  const void* a[kMaxSlotsPerLaunch];  // shrink: x   expand: v
  void* b[kMaxSlotsPerLaunch];        // shrink: v   expand: y
  int32_t slot[kMaxSlotsPerLaunch];   // absolute slot number of each entry (a dword: scalar loads have no 16-bit form)
};

struct LaunchArgs {
  const uint8_t* slab;
  const int32_t* perm;
  const int32_t* pt;
  const ItemRec* items;
  const SlotRec* slots;   // indexed by absolute slot number
  int64_t elems_per_rank; // sum over all slots of (d_in + d_out)
  int32_t n_items;
  int32_t pad0;
  int32_t log2_page;
  int32_t v_stride;       // = max_rank
  int32_t slot_fastest;   // 1: grid = (slots, items, chunks); 0: grid = (items, chunks, slots); 2 (expand): (chunks, items, slots)
  int32_t pad;
};

// One launch that does shrink and then expand over a few slots (plora_delta on small calls): workgroup w
// of a persistent grid runs tasks w, w + grid, w + 2 grid, ... of a list that holds the shrink tasks of all
// slots and then the expand tasks.  An expand task waits until its slot's shrink tasks have all finished:
// every shrink task adds one to a per-slot counter, the one that completes the count publishes the
// count in kFlagCopies flag words (on separate cache lines, so that the waiting workgroups do not all
// poll one address), and expand tasks poll one of them.  The counters are never reset: the host keeps
// the value each slot's counter will have reached after every launch and hands it over as the target.
constexpr int kMaxSlotsFused = 32;
constexpr int kFlagCopies = 8, kFlagStride = 32;  // words between the copies (128 bytes)
constexpr int kQueueFlag0 = 64;                   // words [0, 32): counters; flags of slot q from kQueueFlag0 + q * kFlagCopies * kFlagStride
constexpr int kQueueWords = kQueueFlag0 + kMaxSlotsFused * kFlagCopies * kFlagStride;
struct FusedPtrs {
  const void* x[kMaxSlotsFused];
  float* v[kMaxSlotsFused];
  void* y[kMaxSlotsFused];
  int32_t slot[kMaxSlotsFused];
  uint32_t target[kMaxSlotsFused];  // value of the slot's counter once this launch's shrink tasks are done
};
struct FusedArgs {
  const uint8_t* slab;
  const int32_t* perm;
  const int32_t* pt;
  const ItemRec* items_s;  // shrink list: blocks of 4 records, or (coop_s) single records
  const ItemRec* items_e;  // expand list, likewise
  const SlotRec* slots;
  uint32_t* queue;         // kQueueWords words of the batch, zero when allocated and never reset
  uint32_t* timeouts;      // one word in page-locked host memory: expand tasks given up, counted for the host
  int64_t elems_per_rank;
  int32_t n_s, n_e;        // workgroup tasks per slot: shrink; expand per 512-column chunk
  int32_t chunks, n_slots;
  int32_t log2_page, v_stride;
  int32_t coop_s, coop_e;  // 1: the list holds single vector-ALU records that the four wavefronts share
  uint32_t spin_limit;     // polls of a slot's flag before an expand task gives up (and counts a timeout)
  int32_t pad;
};

// Runs of physically consecutive pages of one adapter, for the staged load's scatter kernel: run k
// covers the virtual pages first_vpage[k] .. (first_vpage[k+1] or the launch's end) and starts at
// physical page phys_page[k].
constexpr int kScatterRuns = 240;
constexpr int kScatterPiece = 16384;  // bytes one workgroup moves
struct ScatterRuns {
  int32_t n_runs;
  int32_t first_vpage[kScatterRuns];
  int32_t phys_page[kScatterRuns];
};

enum LaunchMode { kModeBlocks = 0, kModeCoop = 1, kModeDeep = 2, kModePanel = 2, kModePanelHalf = 3 };

// Launchers (plora_kernels.hip).  Both take a list of blocks of 4 records (one matrix-core item +
// 3 padding records, or up to 4 vector-ALU items) and run one 256-thread workgroup per block, slot
// and (expand) 512-column chunk.  kModeCoop: the list holds vector-ALU records only and every record
// gets a 256-thread workgroup whose four wavefronts share the record's work (for calls too small to
// fill the machine); kModeDeep (shrink): blocks, two runs in flight per matrix-core item; kModePanel
// (expand): matrix-core blocks only, B stationary in LDS; kModePanelHalf: the same with one workgroup
// per 256 columns instead of 512 (for launches of few workgroups).  Grid: (n_items, chunks, n_slots), or (n_slots, n_items, chunks) when
// a.slot_fastest is set: consecutive workgroups go to consecutive XCDs, so with a slot count that
// is a multiple of 8 every slot then lives on one XCD (its x, v and y rows meet in one L2) and all
// slots' copies of the first (longest) items start first.  A chunk is 64 lanes x 16 bytes of a row
// of B (shrink: chunks = 1).
// e0 / e1 (optional): events that take the start timestamp of the first and the end timestamp of the
// last kernel of the call.
hipError_t launch_shrink(int dtype, const LaunchArgs& a, const SlotPtrs& p, int n_slots, int mode, hipStream_t st,
                         hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);
hipError_t launch_expand(int dtype, const LaunchArgs& a, const SlotPtrs& p, int n_slots, int max_chunks, int mode,
                         hipStream_t st, hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr);

hipError_t launch_delta_queue(int dtype, const FusedArgs& f, const FusedPtrs& p, hipStream_t st, hipEvent_t e0 = nullptr,
                              hipEvent_t e1 = nullptr);

// The library's static device array (plora_delta_static keeps v there): its size, and its address on
// the current device (looked up once per device).
uint64_t static_scratch_bytes();
hipError_t static_scratch(void** out);

// Copies `bytes` bytes that lie contiguous at `staging` (device) into the pages pt[0 .. n_pages) (host
// array, ascending) of the slab, in virtual order; (n_pages - 1) pages < bytes <= n_pages pages,
// bytes a multiple of 16.
hipError_t launch_scatter(const uint8_t* staging, uint8_t* slab, int log2_page, uint64_t bytes, const int32_t* pt,
                          uint32_t n_pages, hipStream_t st);

}  // namespace plora
