// Decode-step attention over a KV cache (arXiv 2409.15012, Section 1: for long inputs the decode step is
// dominated by moving the KV cache out of HBM; Section 3: standard layers read the whole cache, sliding-window
// layers the last `window` tokens, grouped-query attention shares one KV head among several query heads).
//
// Tiled path (bf16, head_dim 128): a workgroup of 4 wavefronts streams the 32-key blocks of one split-K chunk of
// one (sequence, kv head).  K and V blocks arrive as 16-byte-per-lane loads that already are MFMA operands:
//   scores^T[key, head]   = K_block (A, 16 keys x 32 dims) x Q^T (B, 32 dims x 16 head columns), 4 k-steps, 2 key tiles
//   out^T[dim, head]     += V_block^T (A, 16 dims x 32 keys) x P^T (B, 32 keys x 16 head columns), 8 dim tiles
// The 16 head columns hold the G query heads of the KV head twice: columns 0..G-1 carry the bf16-rounded
// probabilities, columns G..2G-1 carry the bf16-rounded remainders, so that P enters the second product with
// about 16 significant bits at no extra MFMA cost (the columns would otherwise be padding).  Scores, softmax
// state and accumulators are fp32.  The online-softmax state of a head lives in the lanes of its column, so
// rescaling the accumulator is lane-local; the only cross-lane traffic per block is two shuffles for the maximum.
#include <algorithm>
#include <type_traits>

#include "mixattn_internal.h"

namespace mixattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

constexpr float kLog2e = 1.4426950408889634f;

__device__ inline uint32_t bf16_bits_rn(float f) {  // f finite, round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename OutT>
__device__ inline void store_out(OutT* p, float v);
template <>
__device__ inline void store_out<float>(float* p, float v) { *p = v; }
template <>
__device__ inline void store_out<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)bf16_bits_rn(v); }


constexpr int kDecodeWaves = 4;  // wavefronts per workgroup (8 were measured on launches that leave CUs idle: no gain)

struct TiledDecodeParams {
  const uint16_t* K; const uint16_t* V;
  const int64_t* d_base; const int32_t* d_slots; const int32_t* d_lens;
  PageTable pages;
  int window;       // ring size of a sliding cache (RING)
  int attn_window;  // WINDOWED: a sliding layer reading a full cache attends its last attn_window positions
  const uint16_t* q; void* out;
  int Hq, Hkv, G;
  float scale_log2;  // softmax scale times log2(e)
  int chunk_blocks, n_chunks;
  // split-K partials: row r, chunk c at (r * chunk_stride + c)
  float* p_acc; float* p_ml; int chunk_stride;
  // fused append (writer layers): this step's token, writable cache pointers, the length array once more (the
  // workgroup that finishes last advances it in place) and the arrival counter of this cache (zero between launches)
  const uint16_t* k_new; const uint16_t* v_new; uint16_t* Kw; uint16_t* Vw; int32_t* d_lens_rw; uint32_t* arrive;
  // group launch (GROUP): n_group layers of one sharing group in one pass over the ring; layer i's q and out
  // start layer_rows * i rows after the first layer's (a row = one query head of one sequence)
  int n_group; int64_t layer_rows;
  // sequences in the batch (balanced launches, fused append)
  int batch;
};

// merges the split-K partials of one (sequence, query head): thread d handles one output dim
template <typename OutT>
__device__ inline void merge_partials(const float* p_acc, const float* p_ml, int n_chunks_b, int d, OutT* out) {
  float M = -INFINITY;
  for (int c = 0; c < n_chunks_b; ++c) M = fmaxf(M, p_ml[2 * c]);
  float L = 0.f, acc = 0.f;
  for (int c = 0; c < n_chunks_b; ++c) {
    const float w = fast_exp2(p_ml[2 * c] - M);
    L += p_ml[2 * c + 1] * w;
    acc += p_acc[(int64_t)c * kTiledDim + d] * w;
  }
  store_out<OutT>(out + d, acc / L);
}

// RING selects the sliding-window instantiation (reads min(n, window) ring slots); it is a template parameter so
// that the two layer kinds are separate kernels in a profile.  Wave w takes blocks w, w + 4, ... of the chunk.
// FUSED: the launch also appends this step's token (k_new, v_new) of a writer layer: the sequence is one token
// longer than the length array says, the wavefront that owns the token's block patches it into the loaded
// fragments, stores it to the cache for later launches, and writes the new length to a second length array
// (the old one is still being read by other workgroups of this launch).
// WINDOWED (full caches only): the layer is a sliding-window layer that shares a standard layer's cache; it reads
// the blocks holding positions n - attn_window .. n - 1 and masks the keys before that range.
// GROUP (rings only): the 16 head columns carry the G query heads of up to 16 / G layers that read this ring, so one
// pass over the ring serves the whole sharing group.  No column is left for the remainders: they go through a
// second set of P x V products instead, which keeps the arithmetic of a column the same as in a one-layer launch.
//
// Fused append: the lengths are advanced in place by the workgroup of the launch that arrives last at a counter.
// Every workgroup has read all the lengths it uses before it arrives (they steer its loads, whose results it has
// consumed), so the one that finds every other arrival counted can overwrite them: no workgroup of this launch reads a
// length again, and the next launch on the stream sees the new values.  The counter is a device-scope atomic
// (workgroups of one launch run on several XCDs); the last arriver puts it back to zero for the next launch.
// Two-phase form for launches whose workgroups read the lengths once, at their start: arrive() is called by the first
// wavefront after a workgroup barrier that every wavefront reaches with its lengths in hand, and only requests the
// counter and the lengths the last arriver would advance; finish() consumes them after the merge of the wavefronts'
// results, so neither round trip is waited for at the end of the launch.  (If this workgroup is the last arriver,
// nobody writes the lengths before it does, so what it requested early is current.)
struct Arrival {
  uint32_t prev;   // lane 0 of the first wavefront
  int32_t len;     // lane bb < batch of the first wavefront: length of sequence bb
  int32_t slots;   // same, its capacity in slots (full caches)
  __device__ inline void arrive(const TiledDecodeParams& a) {
    if (threadIdx.x < 64) {
      if (threadIdx.x == 0)
        prev = __hip_atomic_fetch_add(a.arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const bool has = (int)threadIdx.x < a.batch;
      len = has ? a.d_lens_rw[threadIdx.x] : -1;
      slots = (has && a.window == 0) ? a.d_slots[threadIdx.x] : 0;
    }
  }
  __device__ inline void finish(const TiledDecodeParams& a, uint32_t total_workgroups) {
    if (threadIdx.x < 64) {
      if ((uint32_t)__builtin_amdgcn_readfirstlane((int)prev) == total_workgroups - 1) {
        if (threadIdx.x == 0) __hip_atomic_store(a.arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // idle sequences (negative) stay idle; a full cache at capacity stays as it is
        if (len >= 0 && (a.window > 0 || len < slots)) a.d_lens_rw[threadIdx.x] = len + 1;
        for (int bb = threadIdx.x + 64; bb < a.batch; bb += 64) {
          const int n = a.d_lens_rw[bb];
          if (n >= 0 && (a.window > 0 || n < a.d_slots[bb])) a.d_lens_rw[bb] = n + 1;
        }
      }
    }
  }
};

// decode_piece is the work of one workgroup on blocks blk0 .. blk1-1 of (sequence b, kv head h): piece c of the
// n_chunks_b pieces that (b, h) is cut into.  A workgroup may run it several times (balanced launches): the
// function ends with every wavefront past its last read of the shared arrays.
// n_old, slots_b, base_b: this sequence's entries of the length, slot-count and first-block tables (the caller loads
// the three together, so that the first K/V loads wait for one round trip, not three in a row).
// kr, vr: the two fragment sets of the load pipeline; preloaded (uniform for the wavefront): kr[0], vr[0] already
// hold, or are about to receive, block blk0 + wave.
template <typename OutT, bool RING, bool FUSED, bool WINDOWED, bool GROUP, bool BALANCED, int NW>
__device__ __attribute__((always_inline)) void decode_piece(const TiledDecodeParams& a, const int b, const int h,
                                                            const int blk0, const int blk1, const int c,
                                                            const int n_chunks_b, const int n_old, const int slots_b,
                                                            const int64_t base_b, Arrival& arrival,
                                                            u32x4_t (&kr)[2][8], u32x4_t (&vr)[2][8],
                                                            const bool preloaded) {
  constexpr int kCols = GROUP ? 16 : kMaxGroup;  // head columns that carry results
  // a fused launch sees the sequence one token longer; a full cache that is at capacity takes no token (the host
  // refuses such a call; replays of a captured step beyond the reserved capacity end up here)
  const bool room = FUSED && (RING || n_old < slots_b);
  int n = room ? n_old + 1 : n_old;
  if (RING && n > a.window) n = a.window;
  const int new_slot = RING ? n_old % a.window : n_old;  // where a fused launch puts its token
  const int new_blk = new_slot >> 5, new_key = new_slot & 31;
  const int nb_total = (n + kBlockKeys - 1) / kBlockKeys;
  const int lo = (WINDOWED && n > a.attn_window) ? n - a.attn_window : 0;  // first position attended

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the block loop on scalar branches
  const int col = lane & 15, g = lane >> 4;
  const int G = a.G;
  const int ncols = GROUP ? a.n_group * G : G;
  const bool is_hi = col < ncols, is_lo = !GROUP && (col >= G) && (col < 2 * G);
  const int col_layer = GROUP ? col / G : 0;
  const int head = GROUP ? col - col_layer * G : (is_hi ? col : col - G);  // meaningful when is_hi || is_lo

  // Q^T fragments: lane (col, g) holds dims kk*32 + g*8 .. +7 of its head, zeros in padding columns
  bf16x8_t qf[4];
  {
    const uint16_t* qp =
        a.q + (col_layer * a.layer_rows + (int64_t)b * a.Hq + (int64_t)h * G + head) * kTiledDim + g * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4_t raw = {0u, 0u, 0u, 0u};
      if (is_hi || is_lo) raw = *(const u32x4_t*)(qp + kk * 32);
      qf[kk] = __builtin_bit_cast(bf16x8_t, raw);
    }
  }

  // Block blk of this (sequence, kv head) sits at block index block_at(blk) of the cache: consecutive blocks when
  // the cache is contiguous; in a paged full cache the page id is looked up when the wavefront enters a new page
  // (its blocks are 4 apart, so a page of 2^shift blocks serves 2^shift / 4 consecutive iterations).
  const int64_t nblk = slots_b >> 5;
  const int64_t first_blk = base_b + (int64_t)h * nblk;
  const bool paged = !RING && a.pages.ids != nullptr;
  int cur_page = -1;
  int64_t cur_page_first = 0;
  auto block_at = [&](int blk) -> int64_t {
    if (!paged) return first_blk + blk;
    const int pi = blk >> a.pages.shift;
    if (pi != cur_page) {
      cur_page = pi;
      cur_page_first = ((int64_t)a.pages.ids[(int64_t)b * a.pages.max_pages + pi] * a.Hkv + h) << a.pages.shift;
    }
    return cur_page_first + (blk & ((1 << a.pages.shift) - 1));
  };
  const u32x4_t* Kb = (const u32x4_t*)a.K + lane;
  const u32x4_t* Vb = (const u32x4_t*)a.V + lane;

  floatx4_t o[8];
#pragma unroll
  for (int nn = 0; nn < 8; ++nn) o[nn] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, lsum = 0.f;

  auto load_block = [&](int blk, u32x4_t* kd, u32x4_t* vd) {
    const int64_t at = block_at(blk) * (kBlockElems / 8);
    const u32x4_t* kp = Kb + at;
    const u32x4_t* vp = Vb + at;
    // A full cache is streamed once per launch and is far larger than any cache level: nontemporal loads (+12 %
    // on a pure read stream).  A ring is read again by the next layers of its sharing group and is a few hundred
    // MiB at most: plain loads are 4-7 % faster on a working set of that size.  (Nontemporal loads only in the
    // writer's launch, which finds the ring cold, were measured too: the writer gains 2 us, each reader loses 2.)
#pragma unroll
    for (int i = 0; i < 8; ++i) kd[i] = RING ? kp[i * 64] : __builtin_nontemporal_load(kp + i * 64);
#pragma unroll
    for (int i = 0; i < 8; ++i) vd[i] = RING ? vp[i * 64] : __builtin_nontemporal_load(vp + i * 64);
  };

  // One 32-key block: scores, online softmax, accumulate.  TAIL = this is the last block of the sequence and it
  // is ragged: keys >= n are dropped and their V entries cleared (they may hold stale data).
  auto compute_block = [&](auto tail_tag, int blk, u32x4_t* kd, u32x4_t* vd) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    floatx4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kd[kk]), qf[kk], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kd[4 + kk]), qf[kk], s1, 0, 0, 0);
    }
    float sv[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sv[i] = s0[i] * a.scale_log2;      // key 4g + i of the block
      sv[4 + i] = s1[i] * a.scale_log2;  // key 16 + 4g + i
    }
    if constexpr (WINDOWED) {  // keys before the window (only the first block read has any)
      const int first = lo - blk * kBlockKeys;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = 16 * (j >> 2) + 4 * g + (j & 3);
        sv[j] = key < first ? -INFINITY : sv[j];
      }
    }
    if constexpr (TAIL) {
      const int valid = n - blk * kBlockKeys;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = 16 * (j >> 2) + 4 * g + (j & 3);
        const bool drop = key >= valid;
        sv[j] = drop ? -INFINITY : sv[j];
        const uint32_t keep = drop ? ((j & 1) ? 0x0000ffffu : 0xffff0000u) : 0xffffffffu;
#pragma unroll
        for (int nn = 0; nn < 8; ++nn) vd[nn][j >> 1] &= keep;
      }
    }
    float mx = sv[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) mx = fmaxf(mx, sv[j]);
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);  // finite: every block holds at least one valid key
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    float p[8], psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p[j] = fast_exp2(sv[j] - m_new);
      psum += p[j];
    }
    lsum = lsum * alpha + psum;
    uint32_t pb[8], pr[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t hi = bf16_bits_rn(p[j]);
      const float rem = p[j] - __uint_as_float(hi << 16);
      pr[j] = bf16_bits_rn(rem);
      pb[j] = is_lo ? pr[j] : hi;
    }
    u32x4_t pw = {pb[0] | (pb[1] << 16), pb[2] | (pb[3] << 16), pb[4] | (pb[5] << 16), pb[6] | (pb[7] << 16)};
    const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, pw);
#pragma unroll
    for (int nn = 0; nn < 8; ++nn) {
      o[nn] *= alpha;
      o[nn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vd[nn]), pf, o[nn], 0, 0, 0);
    }
    if constexpr (GROUP) {
      u32x4_t rw = {pr[0] | (pr[1] << 16), pr[2] | (pr[3] << 16), pr[4] | (pr[5] << 16), pr[6] | (pr[7] << 16)};
      const bf16x8_t rf = __builtin_bit_cast(bf16x8_t, rw);
#pragma unroll
      for (int nn = 0; nn < 8; ++nn)
        o[nn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vd[nn]), rf, o[nn], 0, 0, 0);
    }
  };
  using no_tail = std::integral_constant<bool, false>;
  using with_tail = std::integral_constant<bool, true>;
  auto compute_last = [&](int blk, u32x4_t* kd, u32x4_t* vd) {
    if (blk == nb_total - 1 && (n & (kBlockKeys - 1))) compute_block(with_tail{}, blk, kd, vd);
    else compute_block(no_tail{}, blk, kd, vd);
  };

  // Software pipeline over this wavefront's blocks blk0 + wave + NW*i, i < cnt.  The steady-state loop issues the
  // next block's loads unconditionally before it consumes the current one, so the wait before the MFMAs only
  // covers the older of the two blocks in flight; the last one or two blocks are peeled.
  // In a fused launch the wavefront that owns the block receiving the new token visits that block last: its loads
  // go through the pipeline like any other block's, and the token is patched into the fragments just before they
  // are consumed (the block as stored is one token short), so the steady-state loop stays free of conditions.
  const int first = blk0 + wave;
  const bool own_new = room && new_blk >= blk0 && new_blk < blk1 && ((new_blk - blk0) & (NW - 1)) == wave;
  const int i_new = own_new ? (new_blk - first) / NW : 0x7fffffff;
  // (balanced and group launches have no registers to spare for a patch inside the pipeline: they take the block out
  // of the sequence instead and handle it after the pipeline)
  constexpr bool kNewInPipeline = FUSED && !BALANCED && !GROUP;
  const int cnt = (blk1 - blk0 - wave + NW - 1) / NW - ((own_new && !kNewInPipeline) ? 1 : 0);  // may be <= 0
  auto blk_of = [&](int i) {
    return (kNewInPipeline && own_new && i == cnt - 1) ? new_blk : first + (i + (i >= i_new ? 1 : 0)) * NW;
  };
  // the new token's K pieces and V elements this lane would patch in: requested ahead of the block loads (balanced
  // launches fetch them when they patch)
  constexpr bool kTokenAhead = kNewInPipeline;
  u32x4_t k_tok[4] = {};
  uint32_t v_tok[8] = {};
  auto load_token = [&]() {
    const uint16_t* kn = a.k_new + ((int64_t)b * a.Hkv + h) * kTiledDim;
    const uint16_t* vn = a.v_new + ((int64_t)b * a.Hkv + h) * kTiledDim;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) k_tok[kk] = *(const u32x4_t*)(kn + kk * 32 + g * 8);
#pragma unroll
    for (int nn = 0; nn < 8; ++nn) v_tok[nn] = vn[nn * 16 + col];
  };
  if constexpr (kTokenAhead) {
    if (own_new) load_token();
  }
  auto patch_new = [&](u32x4_t* kd, u32x4_t* vd) {
    if constexpr (!kTokenAhead) load_token();
    // K fragments: lanes of MFMA row new_key % 16 take the token's dims kk*32 + g*8 .. +7 in key tile new_key / 16
    {
      const bool mine = col == (new_key & 15);
      const bool t1 = (new_key >> 4) != 0;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          kd[kk][w] = (mine && !t1) ? k_tok[kk][w] : kd[kk][w];
          kd[4 + kk][w] = (mine && t1) ? k_tok[kk][w] : kd[4 + kk][w];
        }
      }
    }
    // V fragments: lanes of key group (new_key % 16) / 4 hold the token as element j of every dim fragment
    {
      const bool mine = g == ((new_key & 15) >> 2);
      const int j = 4 * (new_key >> 4) + (new_key & 3);
      const uint32_t half_mask = (j & 1) ? 0xffff0000u : 0x0000ffffu;
#pragma unroll
      for (int nn = 0; nn < 8; ++nn) {
        const uint32_t val = v_tok[nn] << ((j & 1) * 16);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t msk = (mine && w == (j >> 1)) ? half_mask : 0u;
          vd[nn][w] = (vd[nn][w] & ~msk) | (val & msk);
        }
      }
    }
  };
  // the last block of this wavefront's sequence
  auto finish = [&](int blk, u32x4_t* kd, u32x4_t* vd) {
    if constexpr (kNewInPipeline) {
      if (own_new) patch_new(kd, vd);
    }
    compute_last(blk, kd, vd);
  };
  if (cnt > 0) {
    if (!preloaded) load_block(blk_of(0), kr[0], vr[0]);  // else the caller requested it before the length was known
    int i = 0;
    for (; i + 2 < cnt; i += 2) {
      load_block(blk_of(i + 1), kr[1], vr[1]);
      compute_block(no_tail{}, blk_of(i), kr[0], vr[0]);
      load_block(blk_of(i + 2), kr[0], vr[0]);
      compute_block(no_tail{}, blk_of(i + 1), kr[1], vr[1]);
    }
    if (i + 1 < cnt) {
      load_block(blk_of(i + 1), kr[1], vr[1]);
      compute_block(no_tail{}, blk_of(i), kr[0], vr[0]);
      finish(blk_of(i + 1), kr[1], vr[1]);
    } else {
      finish(blk_of(i), kr[0], vr[0]);
    }
  }
  if constexpr (FUSED && !kNewInPipeline) {
    if (own_new) {
      load_block(new_blk, kr[0], vr[0]);
      patch_new(kr[0], vr[0]);
      compute_last(new_blk, kr[0], vr[0]);
    }
  }
  if constexpr (FUSED) {
    if (own_new) {
      // the token goes to the cache for the launches that follow (no other wavefront of this launch reads the block)
      const uint16_t* kn = a.k_new + ((int64_t)b * a.Hkv + h) * kTiledDim;
      const uint16_t* vn = a.v_new + ((int64_t)b * a.Hkv + h) * kTiledDim;
      const int64_t new_at = block_at(new_blk) * kBlockElems;
      uint16_t* Kd = a.Kw + new_at;
      uint16_t* Vd = a.Vw + new_at;
      if (lane < 16) *(u32x4_t*)(Kd + k_tile_offset(new_key, lane * 8)) = *(const u32x4_t*)(kn + lane * 8);
      Vd[v_tile_offset(new_key, lane)] = vn[lane];
      Vd[v_tile_offset(new_key, lane + 64)] = vn[lane + 64];
    }
  }

  // ---- wave epilogue: total sum over the 4 lane groups, remainder columns folded into their head's column
  lsum += __shfl_xor(lsum, 16);
  lsum += __shfl_xor(lsum, 32);
  if constexpr (!GROUP) {
#pragma unroll
    for (int nn = 0; nn < 8; ++nn)
#pragma unroll
      for (int i = 0; i < 4; ++i) o[nn][i] += __shfl_down(o[nn][i], G);  // lane col+G of the same 16-lane row
  }

  __shared__ float s_o[NW][kCols][kTiledDim];
  __shared__ float s_m[NW][kCols];
  __shared__ float s_l[NW][kCols];
  if (is_hi) {
#pragma unroll
    for (int nn = 0; nn < 8; ++nn)
#pragma unroll
      for (int i = 0; i < 4; ++i) s_o[wave][col][nn * 16 + 4 * g + i] = o[nn][i];
    if (g == 0) {
      s_m[wave][col] = m;
      s_l[wave][col] = lsum;
    }
  }
  __syncthreads();
  // every wavefront of the workgroup is past its reads of the length array: the arrival's round trip runs under the merge
  if constexpr (FUSED && !BALANCED) arrival.arrive(a);

  const bool direct = (a.n_chunks == 1);
  // result row of head column hd: the layer's block of rows, then (sequence, query head)
  auto row_of = [&](int hd) -> int64_t {
    const int gl = GROUP ? hd / G : 0;
    return gl * a.layer_rows + (int64_t)b * a.Hq + (int64_t)h * G + (hd - gl * G);
  };
  for (int idx = tid; idx < ncols * kTiledDim; idx += NW * 64) {
    const int hd = idx >> 7, d = idx & 127;
    float M = s_m[0][hd];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[w][hd]);
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wgt = fast_exp2(s_m[w][hd] - M);  // a wave without blocks has m = -inf, weight 0
      L += s_l[w][hd] * wgt;
      acc += s_o[w][hd][d] * wgt;
    }
    const int64_t row = row_of(hd);
    if (direct) {
      store_out<OutT>((OutT*)a.out + row * kTiledDim + d, acc / L);
    } else {
      const int64_t pr = row * a.chunk_stride + c;
      a.p_acc[pr * kTiledDim + d] = acc;
      if (d == 0) {
        a.p_ml[2 * pr] = M;
        a.p_ml[2 * pr + 1] = L;
      }
    }
  }
  if constexpr (BALANCED) __syncthreads();  // the shared arrays are written again by this workgroup's next piece
}

// One-phase form of the arrival (balanced launches, whose workgroups read lengths again for every piece): called by
// every workgroup of the grid exactly once, at its end, from uniform control flow.
__device__ inline void arrive_and_advance(const TiledDecodeParams& a, uint32_t total_workgroups) {
  __shared__ int s_is_last;
  __syncthreads();  // every wavefront of this workgroup is past its reads of the length array
  if (threadIdx.x == 0) {
    const uint32_t prev = __hip_atomic_fetch_add(a.arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = prev == total_workgroups - 1;
    if (last) __hip_atomic_store(a.arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_is_last = last;
  }
  __syncthreads();
  if (s_is_last) {
    for (int bb = threadIdx.x; bb < a.batch; bb += blockDim.x) {
      const int n = a.d_lens_rw[bb];  // idle sequences (negative) stay idle; a full cache at capacity stays as it is
      if (n >= 0 && (a.window > 0 || n < a.d_slots[bb])) a.d_lens_rw[bb] = n + 1;
    }
  }
}

// output rows of an idle sequence (released, no new prompt yet): zeros for the G query heads of kv head h, in
// each of the `layers` layers of a group launch
template <typename OutT>
__device__ inline void zero_rows(const TiledDecodeParams& a, int b, int h, int layers) {
  for (int idx = threadIdx.x; idx < layers * a.G * kTiledDim; idx += blockDim.x) {
    const int hd = idx >> 7, d = idx & 127;
    const int gl = hd / a.G;
    const int64_t row = gl * a.layer_rows + (int64_t)b * a.Hq + (int64_t)h * a.G + (hd - gl * a.G);
    store_out<OutT>((OutT*)a.out + row * kTiledDim + d, 0.f);
  }
}

template <typename OutT, bool RING, bool FUSED, bool WINDOWED = false, bool GROUP = false, int NW = kDecodeWaves>
__global__ __launch_bounds__(NW * 64, 2) void decode_tiled_kernel(TiledDecodeParams a) {
  static_assert(!(WINDOWED && (RING || FUSED)), "a windowed reader of a full cache never writes it");
  static_assert(!GROUP || RING, "group launches serve ring caches");
  const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  constexpr bool kAhead = RING && !FUSED && !GROUP && !WINDOWED;  // first blocks requested ahead of the length
  int n_held = 0;
  if constexpr (!kAhead) n_held = a.d_lens[b];
  // a ring has the same geometry for every sequence: no table needed
  const int slots_b = RING ? ((a.window + kBlockKeys - 1) & ~(kBlockKeys - 1)) : a.d_slots[b];
  const int64_t base_b = RING ? (int64_t)b * a.Hkv * (slots_b >> 5) : a.d_base[b];
  u32x4_t kr[2][8], vr[2][8];
  // A reader of a ring that is not split knows where its wavefronts' first blocks are from the kernel arguments
  // alone: they are requested before the length arrives (a wavefront whose block turns out to be beyond the held
  // tokens drops what it loaded; the ring's storage is there whatever the length is).
  bool preloaded = false;
  if constexpr (kAhead) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (gridDim.x == 1 && wave < (slots_b >> 5)) {
      const int64_t at = (base_b + (int64_t)h * (slots_b >> 5) + wave) * (kBlockElems / 8) + (threadIdx.x & 63);
      const u32x4_t* kp = (const u32x4_t*)a.K + at;
      const u32x4_t* vp = (const u32x4_t*)a.V + at;
#pragma unroll
      for (int i = 0; i < 8; ++i) kr[0][i] = kp[i * 64];
#pragma unroll
      for (int i = 0; i < 8; ++i) vr[0][i] = vp[i * 64];
      preloaded = true;
    }
    __builtin_amdgcn_sched_barrier(0);  // the length is asked for after the loads above are on their way
    n_held = a.d_lens[b];
  }
  Arrival arrival;
  bool arrived = false;
  if (n_held < 0) {  // idle sequence: zero rows, stays idle
    if (c == 0) zero_rows<OutT>(a, b, h, GROUP ? a.n_group : 1);
  } else {
    int n = n_held + ((FUSED && (RING || n_held < slots_b)) ? 1 : 0);
    if (RING && n > a.window) n = a.window;
    const int nb_total = (n + kBlockKeys - 1) / kBlockKeys;
    const int lo = (WINDOWED && n > a.attn_window) ? n - a.attn_window : 0;  // first position attended
    const int fb = lo / kBlockKeys;                                           // first block read
    const int nb_read = nb_total - fb;
    // this sequence's blocks are cut into n_chunks_b chunks of equal length (+-1 block), so that workgroups of one
    // sequence finish together and a sequence a little longer than a multiple of the target does not grow a stub.
    // Never more chunks than the grid has workgroups for: a launch planned for shorter sequences (a captured step
    // replayed later) then simply takes longer chunks.
    const int n_chunks_b = min((nb_read + a.chunk_blocks - 1) / a.chunk_blocks, (int)gridDim.x);
    if (c < n_chunks_b) {  // uniform for the workgroup
      const int blk0 = fb + (int)(((int64_t)c * nb_read) / n_chunks_b);
      const int blk1 = fb + (int)(((int64_t)(c + 1) * nb_read) / n_chunks_b);
      decode_piece<OutT, RING, FUSED, WINDOWED, GROUP, false, NW>(a, b, h, blk0, blk1, c, n_chunks_b, n_held, slots_b,
                                                                  base_b, arrival, kr, vr, preloaded);
      arrived = true;
    }
  }
  if constexpr (FUSED) {
    if (!arrived) {  // uniform for the workgroup: it had no blocks to read
      __syncthreads();
      arrival.arrive(a);
    }
    arrival.finish(a, gridDim.x * gridDim.y * gridDim.z);
  }
}

// Balanced launch for full caches whose sequences differ in length.  The blocks of all (sequence, kv head) streams,
// laid end to end in (b, h) order, are cut into gridDim.x runs of `share` blocks: every workgroup streams the same
// number of blocks whatever the lengths are, and a stream is cut only where a run ends.  Piece c of a stream is the
// part inside the c-th run that touches it; the combine launch that follows merges the pieces.  `share` is derived
// on the device from the lengths and the grid size (balanced_share), so a launch set up for one set of lengths
// stays correct when they have grown (a captured step replayed later).
//   s_first[b] = blocks of one kv head held by sequences 0 .. b-1 (built by the first wavefront, a scan over the batch)
constexpr int kMaxBalancedBatch = 1024;

// blocks a decode reads for a sequence of length n (idle: none); a fused launch counts the token it appends
template <bool FUSED>
__device__ inline int blocks_of_length(int n, int slots) {
  if (n < 0) return 0;
  return (n + ((FUSED && n < slots) ? 1 : 0) + kBlockKeys - 1) / kBlockKeys;
}

// Blocks per run: the total spread over the runs, but no stream may fall into more than kMaxChunks pieces (a stream
// of nb blocks touches at most (nb - 1) / share + 2 runs) and a run keeps every wavefront of its workgroup busy.
__device__ inline int balanced_share(int64_t total, int max_nb, int runs) {
  int64_t share = (total + runs - 1) / runs;
  share = max(share, (int64_t)((max_nb + (kMaxChunks - 2) - 1) / (kMaxChunks - 2)));
  return (int)max(share, (int64_t)kDecodeMinChunkBlocks);
}

// s_first[0 .. batch] = exclusive scan of the block counts, *s_max = the largest count
template <bool FUSED>
__device__ inline void scan_block_counts(const int32_t* d_lens, const int32_t* d_slots, int batch, int* s_first,
                                         int* s_max) {
  const int lane = threadIdx.x & 63;
  if (threadIdx.x < 64) {
    int run = 0, mx = 0;
    for (int b0 = 0; b0 < batch; b0 += 64) {
      const int bb = b0 + lane;
      int inc = bb < batch ? blocks_of_length<FUSED>(d_lens[bb], d_slots[bb]) : 0;
      mx = max(mx, inc);
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
      }
      if (bb < batch) s_first[bb + 1] = run + inc;
      run += __shfl(inc, 63);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, __shfl_xor(mx, o));
    if (lane == 0) {
      s_first[0] = 0;
      *s_max = mx;
    }
  }
  __syncthreads();
}

// stream (b, h) starts at block s_first[b] * Hkv + h * nb_b of the end-to-end order; pieces of a stream starting at
// block gs with nb blocks, for runs of `share` blocks
__device__ inline int balanced_first_run(int64_t gs, int share) { return (int)(gs / share); }
__device__ inline int balanced_pieces(int64_t gs, int nb, int share) {
  return (int)((gs + nb - 1) / share) - (int)(gs / share) + 1;
}

template <typename OutT, bool FUSED>
__global__ __launch_bounds__(kDecodeWaves * 64, 2) void decode_balanced_kernel(TiledDecodeParams a) {
  __shared__ int s_first[kMaxBalancedBatch + 1];
  __shared__ int s_max;
  scan_block_counts<FUSED>(a.d_lens, a.d_slots, a.batch, s_first, &s_max);
  const int64_t total = (int64_t)s_first[a.batch] * a.Hkv;
  const int share = balanced_share(total, s_max, (int)gridDim.x);
  const int64_t g0 = (int64_t)blockIdx.x * share;
  const int64_t g1 = min(total, g0 + share);
  // sequence that holds block g0: the last b with s_first[b] * Hkv <= g0 (uniform binary search)
  int b = 0;
  {
    int hi = a.batch;  // invariant: s_first[b] * Hkv <= g0 < s_first[hi] * Hkv (when g0 < total)
    while (hi - b > 1) {
      const int mid = (b + hi) >> 1;
      if ((int64_t)s_first[mid] * a.Hkv <= g0) b = mid; else hi = mid;
    }
  }
  Arrival unused_arrival;  // balanced launches arrive once per workgroup, after the last piece
  u32x4_t kr[2][8], vr[2][8];
  for (int64_t g = g0; g < g1;) {
    while ((int64_t)s_first[b + 1] * a.Hkv <= g) ++b;  // g < total, so b stays below the batch size
    const int nb = s_first[b + 1] - s_first[b];
    const int off = (int)(g - (int64_t)s_first[b] * a.Hkv);
    const int h = off / nb;
    const int blk0 = off - h * nb;
    const int blk1 = (int)min((int64_t)nb, blk0 + (g1 - g));
    const int64_t gs = g - blk0;
    decode_piece<OutT, false, FUSED, false, false, true, kDecodeWaves>(
        a, b, h, blk0, blk1, blockIdx.x - balanced_first_run(gs, share), balanced_pieces(gs, nb, share), a.d_lens[b],
        a.d_slots[b], a.d_base[b], unused_arrival, kr, vr, false);
    g += blk1 - blk0;
  }
  if constexpr (FUSED) arrive_and_advance(a, gridDim.x);
}

// Merges the pieces of a balanced launch: one workgroup per (sequence, query head), thread d one output dim.  It
// runs after the decode launch, so a fused append has already advanced the lengths: the block counts it derives
// from them are the ones the decode launch worked with.  a.n_chunks = number of runs of that launch.
template <typename OutT>
__global__ __launch_bounds__(kTiledDim) void combine_balanced_kernel(TiledDecodeParams a) {
  const int hq = blockIdx.x, b = blockIdx.y;
  // blocks of one kv head held by the sequences before b, by all sequences, and the largest count
  __shared__ int s_part[3][kTiledDim / 64];
  int before = 0, all = 0, mx = 0;
  for (int bb = threadIdx.x; bb < a.batch; bb += kTiledDim) {
    const int nb_bb = blocks_of_length<false>(a.d_lens[bb], 0);
    before += bb < b ? nb_bb : 0;
    all += nb_bb;
    mx = max(mx, nb_bb);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    before += __shfl_xor(before, o);
    all += __shfl_xor(all, o);
    mx = max(mx, __shfl_xor(mx, o));
  }
  if ((threadIdx.x & 63) == 0) {
    s_part[0][threadIdx.x >> 6] = before;
    s_part[1][threadIdx.x >> 6] = all;
    s_part[2][threadIdx.x >> 6] = mx;
  }
  __syncthreads();
  before = all = mx = 0;
#pragma unroll
  for (int w = 0; w < kTiledDim / 64; ++w) {
    before += s_part[0][w];
    all += s_part[1][w];
    mx = max(mx, s_part[2][w]);
  }
  const int64_t row = (int64_t)b * a.Hq + hq;
  if (a.d_lens[b] < 0) {  // idle sequence: no workgroup of the balanced launch touched it
    store_out<OutT>((OutT*)a.out + row * kTiledDim + threadIdx.x, 0.f);
    return;
  }
  const int share = balanced_share((int64_t)all * a.Hkv, mx, a.n_chunks);
  const int nb = blocks_of_length<false>(a.d_lens[b], 0);
  const int64_t gs = (int64_t)before * a.Hkv + (int64_t)(hq / a.G) * nb;
  merge_partials<OutT>(a.p_acc + row * a.chunk_stride * kTiledDim, a.p_ml + row * a.chunk_stride * 2,
                       balanced_pieces(gs, nb, share), threadIdx.x, (OutT*)a.out + row * kTiledDim);
}

// Merges the chunks of a split launch (runs after it: a fused append has already advanced the lengths).
template <typename OutT>
__global__ __launch_bounds__(kTiledDim) void combine_kernel(TiledDecodeParams a) {
  const int hq = blockIdx.x, b = blockIdx.y;
  if (a.d_lens[b] < 0) return;  // idle sequence: the decode launch wrote its zero rows
  int n = a.d_lens[b];
  if (a.window > 0 && n > a.window) n = a.window;
  const int nb_total = (n + kBlockKeys - 1) / kBlockKeys;
  const int lo = (a.attn_window > 0 && n > a.attn_window) ? n - a.attn_window : 0;
  const int nb_read = nb_total - lo / kBlockKeys;
  const int n_chunks_b = min((nb_read + a.chunk_blocks - 1) / a.chunk_blocks, a.n_chunks);
  const int64_t row = blockIdx.z * a.layer_rows + (int64_t)b * a.Hq + hq;  // z: layer of a group launch
  merge_partials<OutT>(a.p_acc + row * a.chunk_stride * kTiledDim, a.p_ml + row * a.chunk_stride * 2, n_chunks_b,
                       threadIdx.x, (OutT*)a.out + row * kTiledDim);
}

// ------------------------------------------------------------------------------------------------
// Split-K scratch for callers that cannot allocate (mixattn_decode_noalloc): a fixed area in the library's device
// image.  Each GPU the library runs on holds its own copy at its own address, looked up once per device.  Nothing in
// it has to start at zero: a launch writes every partial that its combine launch reads.  Calls that overlap on one
// GPU share it and race.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

hipError_t static_scratch_init(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[device]) return hipSuccess;
  void* ptr = nullptr;
  const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));  // address on the current device
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  g_scratch_ptr[device] = ptr;
  return hipSuccess;
}

void* static_scratch_ptr(int device) {
  return (device >= 0 && device < kMaxDevices) ? g_scratch_ptr[device] : nullptr;
}

hipError_t launch_decode_tiled(const DecodeLaunch& L, hipStream_t s) {
  TiledDecodeParams p;
  p.K = (const uint16_t*)L.K; p.V = (const uint16_t*)L.V;
  p.d_base = L.d_base; p.d_slots = L.d_slots; p.d_lens = L.d_lens;
  p.pages = L.pages;
  p.window = L.window; p.attn_window = L.attn_window;
  p.q = (const uint16_t*)L.q; p.out = L.out;
  p.Hq = L.Hq; p.Hkv = L.Hkv; p.G = L.G;
  p.scale_log2 = L.scale * kLog2e;
  p.chunk_blocks = L.chunk_blocks; p.n_chunks = L.n_chunks;
  p.k_new = (const uint16_t*)L.k_new; p.v_new = (const uint16_t*)L.v_new;
  p.Kw = (uint16_t*)L.K; p.Vw = (uint16_t*)L.V; p.d_lens_rw = L.d_lens_rw; p.arrive = L.arrive;
  p.n_group = L.n_group; p.layer_rows = (int64_t)L.batch * L.Hq;
  p.batch = L.batch;
  const bool f32 = L.out_dtype == MIXATTN_F32, ring = L.window > 0, fused = L.k_new != nullptr;
  if (fused && (!L.d_lens_rw || !L.arrive)) return hipErrorInvalidValue;
  const bool balanced = L.balanced_runs > 0;
  const int n_pieces = balanced ? L.balanced_runs : L.n_chunks;  // partial results per row, at most
  if (L.static_scratch) {
    // partial rows packed as tightly as this launch allows; the host has checked that they fit the static area
    const int64_t rows = (int64_t)std::max(L.n_group, 1) * L.batch * L.Hq;
    p.chunk_stride = balanced ? kMaxChunks : n_pieces;
    unsigned char* base = (unsigned char*)static_scratch_ptr(L.device);
    if (!base || static_scratch_bytes(rows, p.chunk_stride) > (int64_t)kStaticScratchBytes) return hipErrorInvalidValue;
    p.p_acc = (float*)base;
    p.p_ml = p.p_acc + rows * p.chunk_stride * kTiledDim;
  } else {
    p.chunk_stride = kMaxChunks;
    p.p_acc = L.scratch.acc; p.p_ml = L.scratch.ml;
  }
  if (balanced) {
    if (ring || L.attn_window > 0 || L.n_group > 0 || L.batch > kMaxBalancedBatch) return hipErrorInvalidValue;
    p.n_chunks = L.balanced_runs;  // pieces always go through the combine launch (n_chunks != 1)
    if (p.n_chunks < 2) return hipErrorInvalidValue;
    const dim3 bgrid(L.balanced_runs), bblock(kDecodeWaves * 64);
    if (f32 && fused) hipLaunchKernelGGL((decode_balanced_kernel<float, true>), bgrid, bblock, 0, s, p);
    else if (f32) hipLaunchKernelGGL((decode_balanced_kernel<float, false>), bgrid, bblock, 0, s, p);
    else if (fused) hipLaunchKernelGGL((decode_balanced_kernel<uint16_t, true>), bgrid, bblock, 0, s, p);
    else hipLaunchKernelGGL((decode_balanced_kernel<uint16_t, false>), bgrid, bblock, 0, s, p);
    hipError_t be = hipGetLastError();
    if (be != hipSuccess) return be;
    const dim3 cgrid(L.Hq, L.batch), cblock(kTiledDim);
    if (f32) hipLaunchKernelGGL(combine_balanced_kernel<float>, cgrid, cblock, 0, s, p);
    else hipLaunchKernelGGL(combine_balanced_kernel<uint16_t>, cgrid, cblock, 0, s, p);
    return hipGetLastError();
  }
  if (L.n_chunks < 1 || L.n_chunks > kMaxChunks || L.chunk_blocks < 1) return hipErrorInvalidValue;
  const dim3 grid(L.n_chunks, L.Hkv, L.batch);
#define MIXATTN_LAUNCH_DECODE(OUT, RING, FUSED) \
  hipLaunchKernelGGL((decode_tiled_kernel<OUT, RING, FUSED>), grid, dim3(kDecodeWaves * 64), 0, s, p)
  if (L.n_group > 0) {  // several layers of one ring's sharing group in one launch
#define MIXATTN_LAUNCH_GROUP(OUT, FUSED) \
  hipLaunchKernelGGL((decode_tiled_kernel<OUT, true, FUSED, false, true>), grid, dim3(kDecodeWaves * 64), 0, s, p)
    if (!ring || L.n_group * L.G > 16) return hipErrorInvalidValue;
    if (f32 && fused) MIXATTN_LAUNCH_GROUP(float, true);
    else if (f32) MIXATTN_LAUNCH_GROUP(float, false);
    else if (fused) MIXATTN_LAUNCH_GROUP(uint16_t, true);
    else MIXATTN_LAUNCH_GROUP(uint16_t, false);
#undef MIXATTN_LAUNCH_GROUP
  } else if (L.attn_window > 0) {
    if (f32) hipLaunchKernelGGL((decode_tiled_kernel<float, false, false, true>), grid, dim3(kDecodeWaves * 64), 0, s, p);
    else hipLaunchKernelGGL((decode_tiled_kernel<uint16_t, false, false, true>), grid, dim3(kDecodeWaves * 64), 0, s, p);
  } else if (fused) {
    if (f32 && ring) MIXATTN_LAUNCH_DECODE(float, true, true);
    else if (f32) MIXATTN_LAUNCH_DECODE(float, false, true);
    else if (ring) MIXATTN_LAUNCH_DECODE(uint16_t, true, true);
    else MIXATTN_LAUNCH_DECODE(uint16_t, false, true);
  } else {
    if (f32 && ring) MIXATTN_LAUNCH_DECODE(float, true, false);
    else if (f32) MIXATTN_LAUNCH_DECODE(float, false, false);
    else if (ring) MIXATTN_LAUNCH_DECODE(uint16_t, true, false);
    else MIXATTN_LAUNCH_DECODE(uint16_t, false, false);
  }
#undef MIXATTN_LAUNCH_DECODE
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (L.n_chunks > 1) {
    const dim3 cgrid(L.Hq, L.batch, std::max(L.n_group, 1)), cblock(kTiledDim);
    if (L.out_dtype == MIXATTN_F32)
      hipLaunchKernelGGL(combine_kernel<float>, cgrid, cblock, 0, s, p);
    else
      hipLaunchKernelGGL(combine_kernel<uint16_t>, cgrid, cblock, 0, s, p);
    e = hipGetLastError();
  }
  return e;
}

// ------------------------------------------------------------------------------------------------
// Row-major path (fp32 caches, or bf16 shapes outside the MFMA path): one workgroup per (sequence, query
// head); each wavefront walks every 4th key, lanes split the head dimension.  Plain fp32 arithmetic.
// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ inline float load_as_float(const T* p);
template <>
__device__ inline float load_as_float<float>(const float* p) { return *p; }
template <>
__device__ inline float load_as_float<uint16_t>(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

struct RowDecodeParams {
  const void* K; const void* V;
  const int64_t* d_base; const int32_t* d_slots; const int32_t* d_lens;
  int window, attn_window;
  const void* q; void* out;
  int Hq, G, D;
  float scale;
};

template <typename T, typename OutT>
__global__ __launch_bounds__(256) void decode_rowmajor_kernel(RowDecodeParams a) {
  const int hq = blockIdx.x, b = blockIdx.y;
  const int h = hq / a.G;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  int n = a.d_lens[b];
  const int D = a.D;
  if (n < 0) {  // idle sequence: zero row
    for (int d = tid; d < D; d += 256) store_out<OutT>((OutT*)a.out + ((int64_t)b * a.Hq + hq) * D + d, 0.f);
    return;
  }
  if (a.window > 0 && n > a.window) n = a.window;
  const int lo = (a.attn_window > 0 && n > a.attn_window) ? n - a.attn_window : 0;  // sliding reader of a full cache
  const int slots = a.d_slots[b];
  const T* Kp = (const T*)a.K + (a.d_base[b] + (int64_t)h * slots) * D;
  const T* Vp = (const T*)a.V + (a.d_base[b] + (int64_t)h * slots) * D;
  const T* qp = (const T*)a.q + ((int64_t)b * a.Hq + hq) * D;
  float qv[4], acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int d = lane + 64 * i;
    qv[i] = d < D ? load_as_float<T>(qp + d) : 0.f;
    acc[i] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  for (int s = lo + wave; s < n; s += 4) {
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int d = lane + 64 * i;
      if (d < D) part += qv[i] * load_as_float<T>(Kp + (int64_t)s * D + d);
    }
    const float sc = wave_sum(part) * a.scale;
    const float m_new = fmaxf(m, sc);
    const float alpha = expf(m - m_new);
    const float p = expf(sc - m_new);
    l = l * alpha + p;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int d = lane + 64 * i;
      if (d < D) acc[i] = acc[i] * alpha + p * load_as_float<T>(Vp + (int64_t)s * D + d);
    }
    m = m_new;
  }
  __shared__ float s_acc[4][kMaxHeadDim];
  __shared__ float s_m[4], s_l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int d = lane + 64 * i;
    if (d < D) s_acc[wave][d] = acc[i];
  }
  if (lane == 0) {
    s_m[wave] = m;
    s_l[wave] = l;
  }
  __syncthreads();
  for (int d = tid; d < D; d += 256) {
    float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = (s_m[w] == -INFINITY) ? 0.f : expf(s_m[w] - M);
      L += s_l[w] * wgt;
      o += s_acc[w][d] * wgt;
    }
    store_out<OutT>((OutT*)a.out + ((int64_t)b * a.Hq + hq) * D + d, o / L);
  }
}

hipError_t launch_decode_rowmajor(const DecodeLaunch& L, hipStream_t s) {
  RowDecodeParams p;
  p.K = L.K; p.V = L.V; p.d_base = L.d_base; p.d_slots = L.d_slots; p.d_lens = L.d_lens;
  p.window = L.window; p.attn_window = L.attn_window;
  p.q = L.q; p.out = L.out; p.Hq = L.Hq; p.G = L.G; p.D = L.D; p.scale = L.scale;
  const dim3 grid(L.Hq, L.batch), block(256);
  const bool f32 = L.kv_dtype == MIXATTN_F32, of32 = L.out_dtype == MIXATTN_F32;
  if (f32 && of32) hipLaunchKernelGGL((decode_rowmajor_kernel<float, float>), grid, block, 0, s, p);
  else if (f32) hipLaunchKernelGGL((decode_rowmajor_kernel<float, uint16_t>), grid, block, 0, s, p);
  else if (of32) hipLaunchKernelGGL((decode_rowmajor_kernel<uint16_t, float>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((decode_rowmajor_kernel<uint16_t, uint16_t>), grid, block, 0, s, p);
  return hipGetLastError();
}

}  // namespace mixattn
