// Cache-side kernels: single-token append, bulk commit of prompt / packed K,V, row gather, int fill.
//
// arXiv 2409.15012, Section 3: a sliding-window layer keeps the K/V of the past `window` tokens only;
// here position p of such a cache lives in ring slot p mod window, a standard-attention cache keeps
// position p in slot p.  Both are pure integer maps, so cache contents are a function of the token count.
#include "mixattn_internal.h"

namespace mixattn {

__global__ void fill_i32_kernel(int32_t* p, int32_t v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t* p, int32_t value, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, value, n);
  return hipGetLastError();
}

// Lengths after a bulk store (a launch of its own: every workgroup of the store reads the old lengths).
__global__ void advance_lens_kernel(int32_t* lens, const int32_t* src_len, int uniform_len, int batch) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  const int add = src_len ? src_len[b] : uniform_len;
  const int held = lens[b];
  if (held < 0) {  // idle sequence: new tokens start it at position 0, none leave it idle
    if (add > 0) lens[b] = add;
  } else {
    lens[b] = held + add;
  }
}

hipError_t launch_advance_lens(int32_t* lens, const int32_t* src_len, int uniform_len, int batch, hipStream_t s) {
  hipLaunchKernelGGL(advance_lens_kernel, dim3((batch + 255) / 256), dim3(256), 0, s, lens, src_len, uniform_len, batch);
  return hipGetLastError();
}

__global__ void mark_done_kernel(int32_t* done, const int32_t* lens, const int32_t* src_len, int uniform_len, int batch) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  const int add = src_len ? src_len[b] : uniform_len;
  if (add > 0) done[b] = lens[b] < 0 ? 0 : lens[b];
}

hipError_t launch_mark_done(int32_t* done, const int32_t* lens, const int32_t* src_len, int uniform_len, int batch,
                            hipStream_t s) {
  hipLaunchKernelGGL(mark_done_kernel, dim3((batch + 255) / 256), dim3(256), 0, s, done, lens, src_len, uniform_len, batch);
  return hipGetLastError();
}

// Per-sequence tables (first packed row, row count) written by a kernel that carries the values in its arguments:
// stream-ordered, no host synchronisation and no pinned staging buffer to recycle.
struct SeqTableChunk {
  int64_t first[64];
  int32_t len[64];
};
__global__ __launch_bounds__(64) void set_seq_tables_kernel(int64_t* d_first, int32_t* d_len, SeqTableChunk c, int base,
                                                            int n) {
  const int i = threadIdx.x;
  if (i < n) {
    d_first[base + i] = c.first[i];
    d_len[base + i] = c.len[i];
  }
}

hipError_t launch_set_seq_tables(int64_t* d_first, int32_t* d_len, const int64_t* first, const int32_t* len, int n,
                                 hipStream_t s) {
  for (int base = 0; base < n; base += 64) {
    SeqTableChunk c;
    const int m = n - base < 64 ? n - base : 64;
    for (int i = 0; i < 64; ++i) {
      c.first[i] = i < m ? first[base + i] : 0;
      c.len[i] = i < m ? len[base + i] : 0;
    }
    hipLaunchKernelGGL(set_seq_tables_kernel, dim3(1), dim3(64), 0, s, d_first, d_len, c, base, m);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

struct ScatterChunk {
  int64_t index[64];
  int32_t value[64];
};
__global__ __launch_bounds__(64) void scatter_i32_kernel(int32_t* table, ScatterChunk c, int n) {
  const int i = threadIdx.x;
  if (i < n) table[c.index[i]] = c.value[i];
}

hipError_t launch_scatter_i32(int32_t* table, const int64_t* index, const int32_t* value, int n, hipStream_t s) {
  for (int base = 0; base < n; base += 64) {
    ScatterChunk c;
    const int m = n - base < 64 ? n - base : 64;
    for (int i = 0; i < 64; ++i) {
      c.index[i] = i < m ? index[base + i] : 0;
      c.value[i] = i < m ? value[base + i] : 0;
    }
    hipLaunchKernelGGL(scatter_i32_kernel, dim3(1), dim3(64), 0, s, table, c, m);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ------------------------------------------------------------------------------------------------
// Append one token per sequence.  One workgroup per sequence so that the length is read once, used by
// every thread, and bumped by one thread after all stores of this workgroup were issued.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void append_tiled_kernel(AppendLaunch a) {
  const int b = blockIdx.x;
  const int n = a.d_lens[b];
  if (n < 0) return;  // idle sequence (released, no new prompt yet): its row of k, v is ignored
  const int slot = a.window > 0 ? n % a.window : n;
  if (slot >= a.d_slots[b]) return;  // host checks capacity first; never taken for a consistent layout
  const int blk = slot >> 5, key = slot & 31;
  const uint16_t* ks = (const uint16_t*)a.k + (int64_t)b * a.Hkv * kTiledDim;
  const uint16_t* vs = (const uint16_t*)a.v + (int64_t)b * a.Hkv * kTiledDim;
  uint16_t* Kd = (uint16_t*)a.K;
  uint16_t* Vd = (uint16_t*)a.V;
  // K: 16-byte pieces (8 dims of one key stay together)
  for (int i = threadIdx.x; i < a.Hkv * 16; i += blockDim.x) {
    const int h = i >> 4, c = i & 15;
    const int64_t blk_elem = tiled_block_index(a.d_base, a.d_slots, a.pages, a.Hkv, b, h, blk) * kBlockElems;
    const uint4 val = *(const uint4*)(ks + h * kTiledDim + c * 8);
    *(uint4*)(Kd + blk_elem + k_tile_offset(key, c * 8)) = val;
  }
  // V: single elements (the 8 neighbours of an element in memory are other keys)
  for (int i = threadIdx.x; i < a.Hkv * kTiledDim; i += blockDim.x) {
    const int h = i >> 7, d = i & 127;
    const int64_t blk_elem = tiled_block_index(a.d_base, a.d_slots, a.pages, a.Hkv, b, h, blk) * kBlockElems;
    Vd[blk_elem + v_tile_offset(key, d)] = vs[h * kTiledDim + d];
  }
  __syncthreads();
  if (threadIdx.x == 0) a.d_lens[b] = n + 1;
}

template <typename T>
__global__ __launch_bounds__(256) void append_rowmajor_kernel(AppendLaunch a) {
  const int b = blockIdx.x;
  const int n = a.d_lens[b];
  if (n < 0) return;  // idle sequence
  const int slot = a.window > 0 ? n % a.window : n;
  const int slots = a.d_slots[b];
  if (slot >= slots) return;
  const T* ks = (const T*)a.k + (int64_t)b * a.Hkv * a.D;
  const T* vs = (const T*)a.v + (int64_t)b * a.Hkv * a.D;
  for (int i = threadIdx.x; i < a.Hkv * a.D; i += blockDim.x) {
    const int h = i / a.D, d = i - h * a.D;
    const int64_t row = a.d_base[b] + (int64_t)h * slots + slot;
    ((T*)a.K)[row * a.D + d] = ks[i];
    ((T*)a.V)[row * a.D + d] = vs[i];
  }
  __syncthreads();
  if (threadIdx.x == 0) a.d_lens[b] = n + 1;
}

hipError_t launch_append_tiled(const AppendLaunch& a, hipStream_t s) {
  hipLaunchKernelGGL(append_tiled_kernel, dim3(a.batch), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_append_rowmajor(const AppendLaunch& a, hipStream_t s) {
  if (a.elem == 4)
    hipLaunchKernelGGL(append_rowmajor_kernel<float>, dim3(a.batch), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(append_rowmajor_kernel<uint16_t>, dim3(a.batch), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Bulk store.  Destination driven: a workgroup (tiled) or wavefront (row-major) owns destination slots and
// fetches, for each slot, the token that ends up there.  A sequence held n_old tokens before the call and
// receives `add` new ones (n_new = n_old + add); positions n_old .. n_new-1 come from the caller's tensors,
// earlier positions (chunked prefill only) from an existing cache:
//   linear (ring == 0): destination index s <-> position p = off + s, valid while p < n_new.
//                       off = 0 for a full cache or a prompt copy; for the staging copy of a sliding layer's
//                       chunk, off = max(0, n_old - (stage_window - 1)): the window before the first new token.
//   ring   (ring  > 0): slot s <-> largest position p < n_new with p = s (mod ring), valid while s < min(n_new, ring).
// Slots of a touched block that receive nothing are zero-filled so that later MFMA reads see finite data.
// ------------------------------------------------------------------------------------------------
// bf16 -> fp16 bit pattern, round to nearest even, magnitudes above the fp16 range saturate to +-65504
__device__ inline uint16_t bf16_to_f16_sat(uint16_t b) {
  float f = __uint_as_float((uint32_t)b << 16);
  if (f == f) f = fminf(fmaxf(f, -65504.f), 65504.f);  // NaN passes through
  const _Float16 hval = (_Float16)f;
  return __builtin_bit_cast(uint16_t, hval);
}

struct SlotSource {
  int kind;       // 0: nothing (zero fill), 1: new token `index` of the caller's tensor, 2: slot `index` of the old cache
  int64_t index;
};

__device__ inline SlotSource slot_source(const StoreLaunch& a, int s, int n_old, int n_new, int off) {
  SlotSource r;
  r.kind = 0;
  r.index = 0;
  int64_t p;
  if (a.window == 0) {
    p = (int64_t)off + s;
    if (p >= n_new) return r;
  } else {
    if (s >= a.window || s >= n_new) return r;
    p = (int64_t)s + (int64_t)((n_new - 1 - s) / a.window) * a.window;
  }
  if (p >= n_old) {
    r.kind = 1;
    r.index = p - n_old;
  } else if (a.Kold || a.Vold) {
    r.kind = 2;
    r.index = a.old_window > 0 ? p % a.old_window : p;
  }
  return r;
}

__device__ inline void store_lengths(const StoreLaunch& a, int b, int& n_old, int& n_new, int& off) {
  const int add = a.d_src_len ? a.d_src_len[b] : a.uniform_len;
  const int held = a.d_n_old ? a.d_n_old[b] : 0;
  if (held < 0) {  // idle sequence (length -1): new tokens start it at position 0, none leave it idle
    n_old = add > 0 ? 0 : -1;
    n_new = add > 0 ? add : -1;
  } else {
    n_old = held - (a.old_sub ? add : 0);
    n_new = n_old + add;
  }
  off = (a.stage_window > 0 && n_old > a.stage_window - 1) ? n_old - (a.stage_window - 1) : 0;
}

__global__ __launch_bounds__(256) void store_tiled_kernel(StoreLaunch a) {
  __shared__ __attribute__((aligned(16))) uint16_t sK[kBlockKeys][kTiledDim + 8];
  __shared__ __attribute__((aligned(16))) uint16_t sV[kBlockKeys][kTiledDim + 8];
  const int blk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int slots = a.d_slots[b];
  if (blk * kBlockKeys >= slots) return;
  int n_old, n_new, off;
  store_lengths(a, b, n_old, n_new, off);
  const int add = n_new - n_old;
  const int64_t first = a.d_src_first ? a.d_src_first[b] : (int64_t)b * a.uniform_len;
  // a block no token maps to is left untouched (never read: it lies beyond the length)
  const int live = a.window > 0 ? (n_new < a.window ? n_new : a.window) : n_new - off;
  if (blk * kBlockKeys >= live) return;
  // linear store whose old tokens already sit in the destination: blocks made of old tokens only stay as they are
  if (a.old_is_dest && a.window == 0 && blk * kBlockKeys + kBlockKeys <= n_old - off) return;
  // ... or were brought up to date by an earlier call (fp16 copy of a full cache's V, chunk after chunk)
  if (a.d_done && a.window == 0 && off == 0 && blk * kBlockKeys + kBlockKeys <= a.d_done[b]) return;
  (void)add;

  const int64_t blk_elem = tiled_block_index(a.d_base, a.d_slots, a.pages, a.Hkv, b, h, blk) * kBlockElems;
  uint16_t* Kd = a.K ? (uint16_t*)a.K + blk_elem : nullptr;
  uint16_t* Vd = a.V ? (uint16_t*)a.V + blk_elem : nullptr;
  const uint16_t* ksrc = (const uint16_t*)a.k_src;
  const uint16_t* vsrc = (const uint16_t*)a.v_src;
  const uint16_t* kold = (const uint16_t*)a.Kold;
  const uint16_t* vold = (const uint16_t*)a.Vold;
  const bool has_old = a.Kold || a.Vold;
  auto old_block = [&](int ob) -> int64_t {  // block ob of this (sequence, head) in the old cache
    return tiled_block_index(a.old_base, a.old_slots, a.old_pages, a.Hkv, b, h, ob);
  };

  // Fast path (fp16 copy of a full cache's V, block made of old tokens only): same tile order on both sides,
  // so the block is converted piece by piece.
  if (!a.K && a.window == 0 && off == 0 && a.old_window == 0 && vold && !a.old_is_dest &&
      blk * kBlockKeys + kBlockKeys <= n_old) {
    const uint16_t* src = vold + old_block(blk) * kBlockElems;
    for (int o = threadIdx.x; o < kBlockElems / 8; o += blockDim.x) {
      uint4 v = *(const uint4*)(src + o * 8);
      if (a.v_as_f16) {
        uint16_t* e = (uint16_t*)&v;
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = bf16_to_f16_sat(e[j]);
      }
      *(uint4*)(Vd + o * 8) = v;
    }
    return;
  }

  for (int i = threadIdx.x; i < kBlockKeys * 16; i += blockDim.x) {
    const int key = i >> 4, c = i & 15;
    const SlotSource src = slot_source(a, blk * kBlockKeys + key, n_old, n_new, off);
    uint4 kq = make_uint4(0, 0, 0, 0), vq = make_uint4(0, 0, 0, 0);
    if (src.kind == 1) {
      const int64_t e = ((first + src.index) * a.Hkv + h) * kTiledDim + c * 8;
      if (Kd) kq = *(const uint4*)(ksrc + e);
      if (Vd) vq = *(const uint4*)(vsrc + e);
    } else if (src.kind == 2) {
      const int64_t be = has_old ? old_block((int)(src.index >> 5)) * kBlockElems : 0;
      const int within = (int)(src.index & 31);
      if (Kd && kold) kq = *(const uint4*)(kold + be + k_tile_offset(within, c * 8));
      if (Vd && vold) {
        uint16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = vold[be + v_tile_offset(within, c * 8 + j)];
        vq.x = e[0] | ((uint32_t)e[1] << 16);
        vq.y = e[2] | ((uint32_t)e[3] << 16);
        vq.z = e[4] | ((uint32_t)e[5] << 16);
        vq.w = e[6] | ((uint32_t)e[7] << 16);
      }
    }
    *(uint4*)&sK[key][c * 8] = kq;
    *(uint4*)&sV[key][c * 8] = vq;
  }
  __syncthreads();
  for (int o = threadIdx.x; o < kBlockElems / 8; o += blockDim.x) {
    // K piece o = t*256 + c*16 + r  holds key t*16+r, dims c*8..c*8+7
    if (Kd) {
      const int t = o >> 8, c = (o >> 4) & 15, r = o & 15;
      *(uint4*)(Kd + o * 8) = *(const uint4*)&sK[t * 16 + r][c * 8];
    }
    // V piece o = nn*64 + g*16 + c  holds dim nn*16+c of keys 16*(j/4) + 4g + j%4, j = 0..7
    if (Vd) {
      const int nn = o >> 6, g = (o >> 4) & 3, c = o & 15;
      const int d = nn * 16 + c;
      uint16_t e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        e[j] = sV[16 * (j >> 2) + 4 * g + (j & 3)][d];
        if (a.v_as_f16) e[j] = bf16_to_f16_sat(e[j]);
      }
      uint4 val;
      val.x = e[0] | ((uint32_t)e[1] << 16);
      val.y = e[2] | ((uint32_t)e[3] << 16);
      val.z = e[4] | ((uint32_t)e[5] << 16);
      val.w = e[6] | ((uint32_t)e[7] << 16);
      *(uint4*)(Vd + o * 8) = val;
    }
  }
}

// Row-major caches: one wavefront per destination slot; old tokens always already sit in the destination.
template <typename T>
__global__ __launch_bounds__(256) void store_rowmajor_kernel(StoreLaunch a) {
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63;
  const int slots = a.d_slots[b];
  int n_old, n_new, off;
  store_lengths(a, b, n_old, n_new, off);
  const int64_t first = a.d_src_first ? a.d_src_first[b] : (int64_t)b * a.uniform_len;
  if (slot >= slots) return;
  const SlotSource src = slot_source(a, slot, n_old, n_new, off);
  if (src.kind != 1) return;
  const int64_t se = ((first + src.index) * a.Hkv + h) * a.D;
  const int64_t de = (a.d_base[b] + (int64_t)h * slots + slot) * a.D;
  for (int d = lane; d < a.D; d += 64) {
    ((T*)a.K)[de + d] = ((const T*)a.k_src)[se + d];
    ((T*)a.V)[de + d] = ((const T*)a.v_src)[se + d];
  }
}

hipError_t launch_store_tiled(const StoreLaunch& a, hipStream_t s) {
  const int nblk = (a.max_slots + kBlockKeys - 1) / kBlockKeys;
  if (nblk <= 0) return hipSuccess;
  hipLaunchKernelGGL(store_tiled_kernel, dim3(nblk, a.Hkv, a.batch), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_store_rowmajor(const StoreLaunch& a, hipStream_t s) {
  const int nb = (a.max_slots + 3) / 4;
  if (nb <= 0) return hipSuccess;
  if (a.elem == 4)
    hipLaunchKernelGGL(store_rowmajor_kernel<float>, dim3(nb, a.Hkv, a.batch), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(store_rowmajor_kernel<uint16_t>, dim3(nb, a.Hkv, a.batch), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Read one logical row back (debug): dst[0..D) = K row, dst[D..2D) = V row, element size `elem`.
// ------------------------------------------------------------------------------------------------
__global__ void gather_row_kernel(const void* K, const void* V, int64_t base, int32_t slots, int kv_head,
                                  int64_t slot, int D, int elem, bool tiled, void* dst) {
  const int d = threadIdx.x;
  if (d >= D) return;
  int64_t koff, voff;
  if (tiled) {
    const int64_t nblk = slots >> 5;
    const int64_t blk_elem = (base + (int64_t)kv_head * nblk + (slot >> 5)) * kBlockElems;
    koff = blk_elem + k_tile_offset((int)(slot & 31), d);
    voff = blk_elem + v_tile_offset((int)(slot & 31), d);
  } else {
    koff = voff = (base + (int64_t)kv_head * slots + slot) * D + d;
  }
  if (elem == 4) {
    ((float*)dst)[d] = ((const float*)K)[koff];
    ((float*)dst)[D + d] = ((const float*)V)[voff];
  } else {
    ((uint16_t*)dst)[d] = ((const uint16_t*)K)[koff];
    ((uint16_t*)dst)[D + d] = ((const uint16_t*)V)[voff];
  }
}

hipError_t launch_gather_row(const void* K, const void* V, int64_t base, int32_t slots, int kv_head, int64_t slot,
                             int D, int elem, bool tiled, void* dst, hipStream_t s) {
  hipLaunchKernelGGL(gather_row_kernel, dim3(1), dim3(256), 0, s, K, V, base, slots, kv_head, slot, D, elem, tiled,
                     dst);
  return hipGetLastError();
}

}  // namespace mixattn
