// Internal declarations shared by the host side and the kernel launchers of libmixattn.
// Not installed; the public interface is include/mixattn.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "mixattn.h"

namespace mixattn {

// ---- tile geometry of the MFMA ("tiled") cache format: bf16, head_dim 128 ----------------------
// A cache is a sequence of 32-key blocks per (sequence, kv head).  One block holds 32 keys x 128 dims of K
// (8 KiB) in the K buffer and the same of V in the V buffer, each arranged so that lane l of a wavefront
// reads its MFMA operand as one 16-byte load at (fragment * 64 + l) * 16 bytes:
//   K block:  element (key, dim) at  (key/16)*2048 + (dim/8)*128 + (key%16)*8 + dim%8
//             -> fragment (t = key/16, kk = dim/32), lane = ((dim/8)%4)*16 + key%16   [A operand of 16x16x32]
//   V block:  element (key, dim) at  (dim/16)*512 + (((key%16)/4)*16 + dim%16)*8 + 4*(key/16) + key%4
//             -> fragment nn = dim/16, lane = ((key%16)/4)*16 + dim%16, the 8 keys of a lane being exactly the
//                keys whose scores that lane holds after the two 16-key QK products of the block.
constexpr int kBlockKeys = 32;
constexpr int kTiledDim = 128;
constexpr int kBlockElems = kBlockKeys * kTiledDim;  // 4096 elements = 8 KiB of bf16
constexpr int kMaxGroup = 8;                         // query heads per KV head on the MFMA decode path
constexpr int kIdle = -1;                             // length of a released sequence until a prompt chunk or load restarts it
constexpr int kMaxChunks = 64;                       // split-K chunks per (sequence, kv head)
constexpr int kMaxHeadDim = 256;
constexpr int kDecodeMinChunkBlocks = 4;              // a split-K chunk keeps every wavefront of its workgroup busy
// Split-K scratch held in the library's device image for mixattn_decode_noalloc (one copy per GPU, 16 MiB)
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
// bytes of split-K partials for `rows` (sequence, query head) rows with `stride` chunk slots each: fp32 accumulators
// of kTiledDim dims plus (max, sum)
inline int64_t static_scratch_bytes(int64_t rows, int64_t stride) { return rows * stride * (kTiledDim + 2) * 4; }

__host__ __device__ inline int k_tile_offset(int key, int dim) {
  return (key >> 4) * 2048 + (dim >> 3) * 128 + (key & 15) * 8 + (dim & 7);
}
__host__ __device__ inline int v_tile_offset(int key, int dim) {
  return (dim >> 4) * 512 + ((((key & 15) >> 2) << 4) + (dim & 15)) * 8 + 4 * (key >> 4) + (key & 3);
}

// Paged full caches: the blocks of (sequence b, kv head h) sit in pages of (1 << shift) blocks x n_kv_heads; the
// page of block blk is ids[b * max_pages + (blk >> shift)].  ids == nullptr: contiguous storage.
struct PageTable {
  const int32_t* ids = nullptr;
  int max_pages = 0;
  int shift = 0;
};
// Index (in blocks of kBlockElems elements) of block blk of (sequence b, kv head h) in a tile-format cache.
__device__ inline int64_t tiled_block_index(const int64_t* d_base, const int32_t* d_slots, const PageTable& pt,
                                            int Hkv, int b, int h, int blk) {
  if (pt.ids) {
    const int64_t pg = pt.ids[(int64_t)b * pt.max_pages + (blk >> pt.shift)];
    return ((pg * Hkv + h) << pt.shift) + (blk & ((1 << pt.shift) - 1));
  }
  return d_base[b] + (int64_t)h * (d_slots[b] >> 5) + blk;
}

// Prompt staging for prefill on the tiled path: tile-format copies that the MFMA kernel reads (V as fp16; for sliding
// layers also K, positions max(0, n_old - (W-1)) .. n_new-1).  Grown on demand.
struct Stage {
  void* K = nullptr;
  void* V = nullptr;
  int64_t blocks = 0;          // blocks per (b, h) currently allocated
  int cache = -1;              // cache whose chunk it holds (-1: none)
  std::vector<int32_t> lens;   // that chunk's length per sequence
  int64_t* d_base = nullptr;   // [batch] geometry tables of the area
  int32_t* d_slots = nullptr;  // [batch]
  // full caches: positions 0 .. d_done[b]-1 of sequence b already have their fp16 copy of V in the area (a prompt fed
  // in chunks converts every position once, not once per chunk); zero after the area moved, a reset or a release
  int32_t* d_done = nullptr;   // [batch]
};

struct Cache {
  int kind = 0;
  int window = 0;      // SLIDING only
  int writer = -1;     // layer index
  int64_t total_elems = 0;  // elements in each of K and V
  void* K = nullptr;   // device
  void* V = nullptr;   // device
  // per-sequence geometry (host copies; device copies in d_base / d_slots)
  std::vector<int64_t> base;   // tiled: first block index of (b, h=0); row-major: first row index of (b, h=0)
  std::vector<int32_t> slots;  // slots per (b, h): capacity rounded up to 32 (tiled) / capacity (row-major)
  int64_t* d_base = nullptr;
  int32_t* d_slots = nullptr;
  // device lengths, [batch], a slice of Layout::d_lens_all.  Always the same address (a captured launch stays valid):
  // appends advance them in place, a bulk store is followed by a small kernel that sets them.
  int32_t* d_lens = nullptr;
  int32_t* lens() const { return d_lens; }
  uint32_t* d_arrive = nullptr;  // arrival counter of fused append+decode launches on this cache (zero between launches)
  std::vector<int64_t> len;    // host mirror
  // paged storage (full caches of a paged layout): a pool of pages, handed to sequences as they grow
  bool paged = false;
  int page_shift = 0;                 // log2(blocks per page)
  int max_pages = 0;                  // table width: pages a sequence can hold at most
  std::vector<int32_t> free_pages;    // stack of free page ids
  std::vector<std::vector<int32_t>> seq_pages;  // [batch] pages of each sequence, in order
  int32_t* d_pages = nullptr;         // device [batch][max_pages]
  PageTable page_table() const {
    PageTable t;
    if (paged) { t.ids = d_pages; t.max_pages = max_pages; t.shift = page_shift; }
    return t;
  }
  // Every cache keeps the staged copy of its latest prompt chunk to itself, so that its readers can run at any later
  // point of the layer loop (a ring no longer holds the keys the chunk's first rows need).
  int n_users = 0;   // layers reading this cache, the writer included
  Stage own_stage;
  // memo of the last split-K plan (it only changes when a sequence crosses a block boundary)
  int64_t plan_key = -1;
  int plan_max_blocks = -1;
  int plan_chunk_blocks = 0;
};

struct DecodeScratch {
  // `layers` = most layers one group launch serves (1 when no ring has a reader)
  float* acc = nullptr;  // [layers][batch][n_q_heads][kMaxChunks][head_dim]
  float* ml = nullptr;   // [layers][batch][n_q_heads][kMaxChunks][2]  (max in log2 units, sum)
};

}  // namespace mixattn

struct mixattn_layout {
  int n_layers = 0;
  int batch = 0, Hq = 0, Hkv = 0, G = 0, D = 0;
  int kv_dtype = 0, out_dtype = 0;
  int elem = 0;  // bytes per cache element
  float scale = 0.f;
  bool tiled = false;  // MFMA tile format (bf16, D == 128, G <= 8) vs row-major
  std::vector<mixattn_layer_desc> layers;
  std::vector<int> layer_cache;  // layer -> cache index
  std::vector<mixattn::Cache> caches;
  std::vector<int32_t> capacity;  // [batch] for FULL caches
  int32_t* d_lens_all = nullptr;  // [n_caches][batch]
  uint32_t* d_arrive_all = nullptr;  // [n_caches]
  mixattn::DecodeScratch scratch;
  int64_t reserved_chunk = 0;     // longest prompt chunk the staging areas were sized for (mixattn_reserve_prefill)
  int fail_alloc_in = 0;          // testing: > 0 counts down device allocations, the one that reaches 0 fails
  int32_t* d_stage_lens = nullptr;  // [batch] device copy of seq_lens for load_kv / prefill commits
  int64_t* d_stage_src = nullptr;   // [batch] device: first packed token of each sequence
  int64_t* d_q_first = nullptr;     // [batch] device: first packed row of each sequence in a varlen prefill call
  int32_t* d_q_len = nullptr;       // [batch] device: chunk length of each sequence in a varlen prefill call
  void* d_readback = nullptr;       // 2 * kMaxHeadDim elements for mixattn_read_cache
  // tuning
  int64_t chunk_keys = 0;
  int64_t prefill_simple = 0;
  int64_t prefill_waves = 0; // 0 = automatic
  int64_t prefill_heads = 0; // 0 = automatic
  int64_t balanced = 1;      // 0 never, 1 when the batch is ragged, 2 always
  int group_layers = 1;      // most layers one group launch may serve (sizes the split-K scratch)
  int device = 0;
  int n_cus = 256;
};

namespace mixattn {

// ---- launchers implemented in the kernel files; all return hipError_t from hipGetLastError() ----
struct DecodeLaunch {
  const void* K; const void* V;
  const int64_t* d_base; const int32_t* d_slots; const int32_t* d_lens;
  PageTable pages;     // tiled path, full caches only
  int window;          // ring size of the cache, 0 = full cache
  int attn_window;     // > 0: sliding layer reading a full cache (attends the last attn_window positions)
  const void* q; void* out;
  int batch, Hq, Hkv, G, D;
  int kv_dtype, out_dtype;
  float scale;
  int max_blocks;      // over the batch, ceil(min(n_b, window)/32) (tiled path)
  int chunk_blocks;    // blocks per split-K chunk
  int n_chunks;        // grid.x
  DecodeScratch scratch;
  bool static_scratch = false;  // partials go to the library's static device area instead (checked to fit by the host)
  int device = 0;
  // fused append (tiled path): this step's k, v [batch, Hkv, D], the length array (advanced in place by the launch)
  // and the cache's arrival counter; nullptr = none
  const void* k_new = nullptr; const void* v_new = nullptr; int32_t* d_lens_rw = nullptr; uint32_t* arrive = nullptr;
  // > 0 (tiled path, rings only): q and out hold n_group layers, [n_group][batch][Hq][D]; scratch rows likewise
  int n_group = 0;
  // > 0 (tiled path, full caches): balanced launch of `balanced_runs` (>= 2) workgroups, each taking an equal run of
  // the batch's blocks (the run length is derived on the device from the lengths)
  int balanced_runs = 0;
};
hipError_t launch_decode_tiled(const DecodeLaunch& a, hipStream_t s);
// address of the static split-K scratch on `device` (looked up with that device current; once per device)
hipError_t static_scratch_init(int device);
void* static_scratch_ptr(int device);
hipError_t launch_decode_rowmajor(const DecodeLaunch& a, hipStream_t s);

// Bulk store of tokens into a cache or the staging area (prompt commit, bulk load, prefill staging).  A sequence
// holds n_old tokens before and n_old + add after; see kernels_cache.hip for the slot <-> position maps.
struct StoreLaunch {
  void* K = nullptr; void* V = nullptr;  // destination; tiled path: either may be nullptr (that tensor is skipped)
  int v_as_f16 = 0;            // tiled path: store V converted to fp16 (prefill staging), saturating at +-65504
  const int64_t* d_base = nullptr; const int32_t* d_slots = nullptr;  // destination geometry
  PageTable pages;             // destination is a paged cache (tiled path)
  int window = 0;              // 0 = linear destination; > 0 = ring of that many slots
  int stage_window = 0;        // linear only: > 0 = destination index 0 is position max(0, n_old - (stage_window-1))
  const void* k_src = nullptr; const void* v_src = nullptr;  // new tokens, [tokens, Hkv, D]
  const int64_t* d_src_first = nullptr;  // [batch] first packed token of each sequence; nullptr => b * uniform_len
  const int32_t* d_src_len = nullptr;    // [batch] new tokens of each sequence; nullptr => uniform_len
  int uniform_len = 0;
  const int32_t* d_n_old = nullptr;      // [batch] device lengths; nullptr => n_old = 0
  int old_sub = 0;                       // 1: d_n_old already include the new tokens (n_old = d_n_old[b] - add)
  // tokens before n_old (tiled path): read from this tile-format cache; nullptr => none are needed
  const void* Kold = nullptr; const void* Vold = nullptr;
  const int64_t* old_base = nullptr; const int32_t* old_slots = nullptr;
  PageTable old_pages;         // the old cache is paged
  int old_window = 0;          // ring size of the old cache (0 = full cache)
  int old_is_dest = 0;         // the old cache is the destination itself: blocks without new tokens are skipped
  const int32_t* d_done = nullptr;  // linear destinations from position 0: blocks wholly below d_done[b] are up to date
  int batch = 0, Hkv = 0, D = 0, elem = 0;
  int max_slots = 0;           // max over b of destination slots that can receive data (grid size)
};
hipError_t launch_store_tiled(const StoreLaunch& a, hipStream_t s);
hipError_t launch_store_rowmajor(const StoreLaunch& a, hipStream_t s);

struct AppendLaunch {
  void* K; void* V;
  const int64_t* d_base; const int32_t* d_slots; int32_t* d_lens;
  PageTable pages;
  int window;
  const void* k; const void* v;
  int batch, Hkv, D, elem;
};
hipError_t launch_append_tiled(const AppendLaunch& a, hipStream_t s);
hipError_t launch_append_rowmajor(const AppendLaunch& a, hipStream_t s);

// after a bulk store: lens[b] = tokens held once sequence b has received its new tokens (src_len[b], or uniform_len
// for every sequence when src_len is nullptr); an idle sequence (negative) given none stays idle
hipError_t launch_advance_lens(int32_t* lens, const int32_t* src_len, int uniform_len, int batch, hipStream_t s);
// done[b] = lens[b] for every sequence that received tokens (src_len[b] > 0, or all when src_len is nullptr and
// uniform_len > 0): the staged copy now covers all the sequence holds
hipError_t launch_mark_done(int32_t* done, const int32_t* lens, const int32_t* src_len, int uniform_len, int batch,
                            hipStream_t s);
hipError_t launch_fill_i32(int32_t* p, int32_t value, int64_t n, hipStream_t s);
// table[index[i]] = value[i] for i < n (host arrays; the values travel in the kernel arguments)
hipError_t launch_scatter_i32(int32_t* table, const int64_t* index, const int32_t* value, int n, hipStream_t s);
// d_first[i] = first[i], d_len[i] = len[i] for i < n (host arrays; the values travel in the kernel arguments)
hipError_t launch_set_seq_tables(int64_t* d_first, int32_t* d_len, const int64_t* first, const int32_t* len, int n,
                                 hipStream_t s);
hipError_t launch_gather_row(const void* K, const void* V, int64_t base, int32_t slots, int kv_head, int64_t slot,
                             int D, int elem, bool tiled, void* dst, hipStream_t s);

struct PrefillLaunch {
  const void* q = nullptr; void* out = nullptr;
  // tiled path: K in tile format (the full cache itself or the staging area), V in tile format as fp16 (staging)
  const void* Kt = nullptr; const int64_t* k_base = nullptr; const int32_t* k_slots = nullptr;
  PageTable k_pages;     // K comes from a paged full cache
  const void* Vt = nullptr; const int64_t* v_base = nullptr; const int32_t* v_slots = nullptr;
  int stage_window = 0;  // > 0: key index 0 of Kt/Vt is position max(0, n_old - (stage_window - 1))
  // row-major path: the caller's chunk tensors, and the row-major cache for positions before the chunk
  const void* k_src = nullptr; const void* v_src = nullptr;
  const void* Kc = nullptr; const void* Vc = nullptr; const int64_t* c_base = nullptr; const int32_t* c_slots = nullptr;
  int ring = 0;          // row-major: ring size of that cache (0 = full)
  // chunked prefill: n_old = d_lens[b] - old_sub tokens were held before this chunk (nullptr: empty caches)
  const int32_t* d_lens = nullptr; int old_sub = 0;  // old_sub: 1 = d_lens already include this chunk
  // chunks of different lengths: rows d_q_first[b] .. + d_q_len[b] - 1 of the packed q / out (and k_src / v_src)
  // tensors; nullptr: uniform, rows b*S .. b*S + S - 1.  S is the longest chunk.
  const int64_t* d_q_first = nullptr; const int32_t* d_q_len = nullptr;
  int window = 0;  // attention window of the layer, 0 = full causal
  int batch = 0, S = 0, Hq = 0, Hkv = 0, G = 0, D = 0;
  int kv_dtype = 0, out_dtype = 0;
  float scale = 0.f;
  int waves = 0;  // wavefronts per workgroup on the tiled path: 4, 8, or 0 = by layer kind (8 full, 4 sliding)
  int heads = 0;  // query heads of one KV head per workgroup on the tiled path: 1, 2, 4, or 0 = as many as divide G
};
hipError_t launch_prefill_tiled(const PrefillLaunch& a, hipStream_t s);
hipError_t launch_prefill_rowmajor(const PrefillLaunch& a, hipStream_t s);

}  // namespace mixattn
