// Internal declarations shared by the host side of librdkv and its kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <string>
#include <vector>

#include "rdkv.h"

namespace rdkv {

constexpr int kHeadDim = 128;
constexpr int kGroup = 32;             // quantization group (channels)
constexpr int kGroupsPerRow = kHeadDim / kGroup;
constexpr int kTile64 = 64;            // tier segments are padded to whole 64-row tiles
constexpr int kKTokenGroup = 32;       // mixed mode: a K channel's group = 32 consecutive retained tokens of a segment
constexpr int kSegAlign = 256;         // byte alignment of arena segments
constexpr int kNumPackTiers = 4;       // stored tiers, order 16, 8, 4, 2
constexpr int kDenseMaxSeqs = 64;      // sequences per dense-decode launch (kernel-argument table)

__host__ __device__ inline int pack_tier_bits(int ti) { return 16 >> ti; }          // 0..3 -> 16,8,4,2
__host__ __device__ inline int tier_row_bytes(int bits) { return kHeadDim * bits / 8; }
__host__ __device__ inline int tier_meta_bytes(int bits) { return bits == 16 ? 0 : kGroupsPerRow * 4; }

// One unit of decode work: a run of rows of one tier of one item.
struct Chunk {
  int64_t k_data, k_meta, v_data, v_meta;   // byte offsets into the arena
  int32_t rows;                             // valid rows in this chunk
  int32_t tier;                             // 16, 8, 4, 2
  int32_t item;                             // sequence * hkv + kv head
  int32_t slot;                             // partial-result slot
  int16_t k_word_end[4];                    // mixed mode: ItemK::word_end of the item (the shape of its K rows)
  int32_t row0;                             // appended-token zone: first row of the chunk inside the item's tail
  int32_t reserved;                         // mixed mode: index of the chunk's ItemK in the schedule's table
                                            // (generation * items + item)
  int32_t slot0, nslots;                    // the item's first partial slot and its number of slots (= chunks)
  int32_t next;                             // token-wise quantized tiers: index in the chunk table of the piece the same
                                            // workgroup goes on with (another tier of the same item), -1: none
  int32_t pad_;
};
constexpr int kTailChunkRows = 256;         // appended tokens per decode work item
constexpr int kTierTail = 17;               // Chunk::tier of a chunk of appended tokens (64-token tiles of bf16 rows)

// Channel-wise K (mixed mode): how one item's K tiles are laid out.  Channels are sorted by bit-width into
// slots: tiers 16, 8, 4, 2 in this order.  A retained token's K row is a run of 32-bit words (a 16-bit word holds
// 2 slots, an 8-bit word 4, a 4-bit word 8, a 2-bit word 16); every tier is padded to whole words, the 16-bit tier
// to whole word pairs, the row to an even number of words.  A step is 4 consecutive slots.
constexpr int kMaxSlots = 160;   // 128 channels + up to 3 + 3 + 7 + 15 padding slots
constexpr int kMaxKRowWords = 68;  // longest row: 125 channels at 16 bits, one each at 8, 4, 2 -> 64 + 1 + 1 + 1, evened
struct ItemK {
  int32_t kt_bytes;              // K tile (64 tokens) data bytes = 256 * n_words_padded
  int32_t km_bytes;              // K tile metadata bytes = 32 * n_qsteps (2 token groups x 16 bytes per quantized step)
  int16_t word_end[4];           // words per token up to and including tier 16, 8, 4, 2
  int16_t slot_base[4];          // first slot of each tier
  int16_t n_slots, n_words, n_words_padded;
  int16_t n_steps16, n_qsteps;   // steps of the 16-bit tier; steps of the quantized tiers
  int16_t slot_ch[kMaxSlots];    // channel held by a slot, -1 for padding
};

struct DenseArgs {
  const uint16_t* K;
  const uint16_t* V;
  const uint16_t* q;
  float* part_acc;     // [slots][g][128]
  float* part_ml;      // [slots][g][2]
  float* out;
  float* lse;
  int32_t hq, hkv, batch, chunk_rows, max_splits, seq_base;
  int32_t T[kDenseMaxSeqs];
  int64_t row_off[kDenseMaxSeqs];           // first row of the sequence block in K / V
};

// ---- launchers implemented in the .hip files ------------------------------
hipError_t launch_decode_dense_split(const DenseArgs& a, int g, int n_seqs, hipStream_t st);
hipError_t launch_decode_dense_merge(const DenseArgs& a, int g, int n_seqs, hipStream_t st);
struct MergeArgs;   // decode_merge.h
// 16-bit tier of a token-wise cache (row-major bf16 rows)
hipError_t launch_decode_tiered_split(const Chunk* chunks, int n_chunks, const uint8_t* arena, const uint16_t* q,
                                      const MergeArgs& ma, hipStream_t st);
// tail_state: the cache's device words {appended tokens so far, workgroups of the running append that are done}
hipError_t launch_append_rows(const uint16_t* k_new, const uint16_t* v_new, uint8_t* tail, int64_t n_items,
                              int32_t tail_tiles, int32_t tail_cap, int32_t* tail_state, hipStream_t st);
hipError_t launch_gather_tail_rows(const uint8_t* tail, int64_t n_items, int32_t tail_tiles, int32_t n,
                                   uint16_t* k_rows, uint16_t* v_rows, hipStream_t st);

// chunks: the whole chunk table; workgroup b starts with chunks[first + b] and, if `multi`, follows Chunk::next.
// tail_len: device word holding the appended tokens that exist so far (chunks of tier kTierTail end there)
hipError_t launch_decode_tiles(const Chunk* chunks, int first, int n_chunks, bool multi, const uint8_t* arena,
                               const uint16_t* q, const MergeArgs& ma, const int32_t* tail_len, hipStream_t st);
// one object per head-set count (hs1: up to 4 query heads per KV head, hs2: 8)
// One object per head-set count (hs1: up to 4 query heads per KV head, hs2: 8) and row length class (long0: K rows
// of up to 32 words, long1: up to 68).  waves: wavefronts per workgroup, 4 or 8 (8 only in hs1 / long0).
#define RDKV_DECLARE_MIXED(NAME_)                                                                                \
  hipError_t NAME_(const Chunk* chunks, int n_chunks, const uint8_t* arena, const ItemK* items_k, int max_words, \
                   int max_steps, int max_qsteps, const uint16_t* q, const MergeArgs& ma, const int32_t* tail_len, \
                   int per_unit, int waves, hipStream_t st);
RDKV_DECLARE_MIXED(launch_decode_mixed_hs1_long0)
RDKV_DECLARE_MIXED(launch_decode_mixed_hs1_long1)
RDKV_DECLARE_MIXED(launch_decode_mixed_hs2_long0)
RDKV_DECLARE_MIXED(launch_decode_mixed_hs2_long1)
#undef RDKV_DECLARE_MIXED
inline hipError_t launch_decode_mixed(const Chunk* chunks, int n_chunks, const uint8_t* arena, const ItemK* items_k,
                                      int max_words, int max_steps, int max_qsteps, const uint16_t* q,
                                      const MergeArgs& ma, const int32_t* tail_len, int per_unit, int waves,
                                      hipStream_t st);

// Optional event bracketing of the main kernels (rdkv_kernel_timing_*).
void timing_begin(int kind, hipStream_t st);
void timing_end(int kind, hipStream_t st);
struct TimedScope {
  int kind;
  hipStream_t st;
  TimedScope(int k, hipStream_t s) : kind(k), st(s) { timing_begin(kind, st); }
  ~TimedScope() { timing_end(kind, st); }
};

struct PackItemDesc;   // compress_kernels

}  // namespace rdkv

// The opaque handle of the C ABI.
struct rdkv_cache {
  int32_t batch = 0, hq = 0, hkv = 0, d = 0, k_mode = 0;
  int32_t k_per_unit = 0;               // mixed mode: one K scale per channel over all retained tokens (App. B)
  int32_t group_size = 32;              // channels per scale of a token row: 32, or 128 = one scale per row (App. B)
  std::vector<int32_t> seq_lens;
  int64_t n_items = 0;
  int64_t total_tokens = 0;             // sum_s hkv * T_s
  // host copies
  std::vector<int32_t> counts;          // [items][4]
  std::vector<int64_t> seg_off;         // [items][4][4]
  std::vector<rdkv::Chunk> chunks;
  int64_t arena_bytes = 0;
  int64_t kept_total = 0;
  int64_t n_chunks16 = 0;               // leading chunks of the 16-bit tier
  // device memory (owned): rdkv_pack takes one block for the arena and every table below; what later calls add or
  // replace (tail, rebuilt chunk tables, workspaces of other streams) are allocations of their own
  uint8_t* d_block = nullptr;
  int64_t block_bytes = 0;
  uint8_t* d_arena = nullptr;
  int32_t* d_tier_idx = nullptr;        // [kept_total]
  rdkv::Chunk* d_chunks = nullptr;
  // split workspaces, one per stream that has decoded from this cache: partial results [slots][g][128 + 2] floats and
  // the items' arrival counters (zero between steps)
  struct Workspace {
    hipStream_t stream;
    float* part_acc;
    float* part_ml;
    int32_t* arrive;
    void* block;                        // the one allocation behind the three
  };
  mutable std::vector<Workspace> workspaces;
  mutable std::mutex ws_mu;
  int64_t n_slots = 0;                  // partial slots of the whole schedule
  int32_t* d_tail_state = nullptr;      // {appended tokens so far, workgroups of the running append that are done}
  int32_t mixed_waves = 4;              // channel-wise mode: wavefronts per workgroup of the decode kernel (4 or 8)
  uint8_t* d_bits_tok = nullptr;        // copy of the token bit map
  uint8_t* d_bits_ch = nullptr;         // [items][128] K channel bit map (mixed mode)
  rdkv::ItemK* d_items_k = nullptr;     // [items] (mixed mode)
  std::vector<rdkv::ItemK> items_k;
  int32_t max_k_words = 0, max_k_steps = 0, max_k_qsteps = 0;   // largest K row shape over the items (mixed mode)
  // appended-token zone (Zone C): per item ceil(tail_cap / 64) tiles of 64 bf16 K rows (16 KiB each), then the same
  // for V, in one allocation (zero-filled: rows not yet appended read as zeros)
  std::vector<int32_t> slot_begin, slot_count;   // host copies of the partial-slot tables
  uint8_t* d_tail = nullptr;
  int64_t n_tail_chunks = 0;            // chunks of the tail, appended to d_chunks in (chunk index, item) order:
                                        // the first ceil(tail_len / 256) * items of them are live
  int32_t tail_cap = 0, tail_len = 0;
  // streaming re-budgeting: appended tokens that were compressed later, one packed cache per call (owned); their
  // chunks are part of this cache's decode schedule (d_chunks), with offsets relative to d_arena
  std::vector<rdkv_cache*> absorbed;
  std::vector<int32_t> own_slot_count;  // [items]: partial slots of this cache's own chunks (no tail, no absorbed)
  int64_t sched16 = 0, schedq = 0;      // chunks of the schedule: 16-bit tier, then the quantized tiers (all generations)
  int64_t n_cont = 0;                   // continuation pieces of this cache's own chunks: the last n_cont entries of `chunks`
  rdkv::ItemK* d_items_sched = nullptr; // mixed mode with absorbed generations: [generations][items] K row layouts
  int32_t sched_k_words = 0, sched_k_steps = 0, sched_k_qsteps = 0;   // largest K row shape over all generations
  double* d_lambda = nullptr;           // [items] (token map), channel-wise mode: + [items] (channel map): the
  int32_t* d_iters = nullptr;           // multiplier and the step count of every search (rdkv_compress only)
  int64_t stored_bytes = 0;             // bytes a decode step must read (unpadded)
  int64_t index_bytes = 0;
  rdkv_alloc_fn alloc = nullptr;
  rdkv_free_fn free_ = nullptr;
  void* alloc_user = nullptr;
};
