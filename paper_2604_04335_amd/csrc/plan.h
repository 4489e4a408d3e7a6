// Host-side work-list ("plan") for one packed denoising-step attention call.
//
// A batch handed to a GPU for one step mixes requests of very different length
// (paper Section 4.3: image requests are batched, Section 3 / Table 3: a video
// step has up to two orders of magnitude more tokens than an image step).  The
// plan cuts every (sequence, head) into query tiles and orders the tiles so
// that persistent workgroups, which take items in list order, finish together.
#pragma once
#include <cstdint>
#include <vector>

namespace dit {

// 16-byte record consumed by the kernel.
struct WorkItem {
  int32_t q_start;    // first global query row of the tile
  int32_t kv_start;   // first global key row (start of the tile's sequence)
  int32_t kv_len;     // keys in the sequence
  int32_t rows_head;  // (part << 28) | (q_rows << 16) | head, q_rows in 1..block_m, part = index of the key chunk (split-KV)
};
static_assert(sizeof(WorkItem) == 16, "WorkItem must be 16 bytes");

// Validate cu_seqlens: returns 0 if ok (cu[0]==0, non-decreasing, n_seqs>=0), else non-zero.
int plan_validate(const int32_t* cu_seqlens, int32_t n_seqs);

// Build the ordered work-list.  Longest sequences first (their tiles cost the
// most); inside a sequence, heads are the slow index and query tiles the fast
// one, so workgroups running side by side stream the same K/V rows; the ragged
// last query tile of every head comes after the sequence's whole tiles.
void plan_build(const int32_t* cu_seqlens, int32_t n_seqs, int32_t n_heads, int32_t block_m,
                std::vector<WorkItem>& items);

// The same with separate query and key boundaries (cross-attention, paper Section 2.1: DiT blocks attend to the text
// tokens): sequence i's query rows cu_q[i]..cu_q[i+1] of q see key rows cu_k[i]..cu_k[i+1] of k and v.  Sequences with
// no query rows or no key rows contribute no items (the caller zeroes the output rows of the latter).  Sequences with
// the most keys come first.
void plan_build_cross(const int32_t* cu_q, const int32_t* cu_k, int32_t n_seqs, int32_t n_heads, int32_t block_m,
                      std::vector<WorkItem>& items, int32_t n_splits = 1, int32_t block_n = 64);

// With n_splits > 1 (split-KV, for packs with fewer items than compute units) the keys of every sequence are cut into
// at most n_splits chunks of whole key tiles (block_n keys), and every (query tile, head) becomes one item per chunk:
// kv_start / kv_len describe the chunk, part its index.  The parts are combined by the merge kernel.

// Eviction policy of the per-context cache of uploaded work-lists: the least recently used entry among those that no
// captured graph refers to (pinned[i] == 0); -1 when every entry is pinned (the cache then grows instead).  A launch
// recorded into a HIP graph keeps reading its work-list on every replay, so such a list must never be freed.
int plan_cache_victim(const uint64_t* last_use, const uint8_t* pinned, int n);

}  // namespace dit
