// Prompt (prefill) attention: causal, and for sliding-window layers restricted to the last `window` keys
// including the query's own token (arXiv 2409.15012, Section 3, "Sliding Window Attention Layers"; Section 1 for
// the causal standard layer).
//
// Tiled path (bf16, head_dim 128): flash-attention forward on 32x32x16 MFMA.  K and V are read in the same
// 32-key block format the decode caches use (K: the full cache itself, or a staging copy of the prompt for
// sliding layers; V: a staging copy converted to fp16), so a block is copied verbatim into LDS and every operand
// fragment is one 16-byte LDS read per lane.  Scores use the bf16 MFMA (exact products of the bf16 inputs); the
// probabilities are rounded to fp16 (11 significant bits) and multiply fp16 V on the fp16 MFMA: a bf16 rounding
// of P would by itself cost about 1.6e-3 relative L2 error.
// A workgroup of NW wavefronts (32 query rows each) serves hg query heads of one KV head, NW/hg wavefronts and
// 32*NW/hg query rows per head, and walks the 64-key tiles its rows can see; a wavefront skips the tiles that are
// masked for all of its rows:
//   scores^T[key, row]  = K (A, 32 keys x 16 dims) x Q^T (B, 16 dims x 32 rows),  8 k-steps per 32-key block
//   out^T[dim, row]    += V^T (A, 32 dims x 16 keys) x P^T (B, 16 keys x 32 rows), both fp16
// Lane l holds query row l%32 in both products, so the online-softmax state and the accumulator rescale are
// lane-local; the row maximum needs one exchange with lane l^32.
#include "mixattn_internal.h"

namespace mixattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kPfKeys = 64;             // keys per iteration (two 32-key blocks)

__device__ inline uint32_t pf_bf16_bits_rn(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

struct TiledPrefillParams {
  const uint16_t* q; void* out;
  const uint16_t* Kt; const int64_t* k_base; const int32_t* k_slots;  // bf16 tiles
  PageTable k_pages;                                                   // ... of a paged full cache
  int Hkv;
  const uint16_t* Vt; const int64_t* v_base; const int32_t* v_slots;  // fp16 tiles
  int window, S, Hq, G;
  float scale_log2;
  // chunked prefill: sequence b held n_old = d_lens[b] - (old_sub ? chunk length : 0) tokens before this chunk
  // (d_lens == nullptr: 0).  Key index 0 of the K/V buffers is position 0 (stage_window == 0) or
  // max(0, n_old - (stage_window - 1)).
  const int32_t* d_lens; int old_sub; int stage_window;
  // chunks of different lengths: sequence b's rows are q_first[b] .. + q_len[b] - 1 of the packed q / out tensors
  // (nullptr: rows b*S .. b*S + S - 1); S is then the longest chunk
  const int64_t* q_first; const int32_t* q_len;
  int hg;  // query heads per workgroup (all of one KV head): 1, 2 or 4, divides G and the wavefront count
};

// MFMA row m of a 32-key block holds key pi(m): bits 3 and 4 of m swapped, so that the 8 scores a lane owns per
// 16-key slab are exactly the 8 keys of one 16-byte V fragment.
__device__ inline int pf_key_of_row(int m) { return (m & 7) | ((m & 8) << 1) | ((m & 16) >> 1); }

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 halfx2_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 halfx8_t;

// two floats -> packed fp16 pair, round to nearest even (one v_cvt_pk_f16_f32)
__device__ inline uint32_t pf_pack_f16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2_t{lo, hi}, halfx2_t));
}
// Probabilities enter the P.V product as fp16 scaled by 2^12 (so that weights down to 2^-26 of the row maximum
// stay normal numbers); the row sum carries the same factor and it cancels in the final division.
constexpr float kPShift = 12.0f;

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ inline uint32_t pf_pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2_t{lo, hi}, bf16x2_t));
}

template <typename OutT, int NW>
__global__ __launch_bounds__(NW * 64, 2) void prefill_tiled_kernel(TiledPrefillParams a) {
  // two stages of one 64-key tile each (2 blocks of K, 2 blocks of V), filled by direct global->LDS loads
  // 64 KiB: stage s holds K at smem + s*16384 and V at smem + s*16384 + 8192 (elements).  Before the first tile
  // lands in stage 1 that stage stages the query rows; after the last tile the whole array stages the output rows.
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * 2 * kBlockElems];
  auto sK = [&](int buf) { return smem + buf * (4 * kBlockElems); };
  auto sV = [&](int buf) { return smem + buf * (4 * kBlockElems) + 2 * kBlockElems; };

  // A workgroup serves hg query heads of one KV head (they read the same K/V tiles) with NW / hg wavefronts each, so
  // it spans 32 * NW / hg query rows: the more heads, the shorter the row span, the fewer keys a sliding-window
  // tile walks beyond its window, and the more MFMAs share each tile load and barrier.
  // Workgroup ids go round-robin over the 8 XCDs, each with its own L2.  Map them so that one XCD works on the
  // query tiles of one head group at a time (ids = 8*slot + xcd): its L2 then holds one K/V stream, not eight.
  const int wph = NW / a.hg;       // wavefronts per head
  const int rows_wg = 32 * wph;    // query rows per workgroup
  const int n_qt = (a.S + rows_wg - 1) / rows_wg;
  const int n_hg = a.Hq / a.hg;
  int qt, hgi;
  {
    const int id = blockIdx.x + gridDim.x * blockIdx.y;
    if ((n_hg & 7) == 0) {
      const int xcd = id & 7, slot = id >> 3;
      hgi = xcd + 8 * (slot / n_qt);
      qt = n_qt - 1 - (slot % n_qt);  // longest rows first
    } else {
      hgi = id / n_qt;
      qt = n_qt - 1 - (id % n_qt);
    }
  }
  const int b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hq = hgi * a.hg + wave / wph;  // this wavefront's query head
  const int h = hq / a.G;
  const int col = lane & 31, hh = lane >> 5;
  const int q0 = qt * rows_wg;
  const int r0 = q0 + (wave % wph) * 32;  // first row of this wavefront
  const int row = r0 + col;
  const int S = a.q_len ? a.q_len[b] : a.S;  // this sequence's chunk length
  const int W = a.window;
  if (q0 >= S) return;                         // the whole workgroup: nothing before this touches a barrier
  const int64_t qrow0 = a.q_first ? a.q_first[b] : (int64_t)b * a.S;  // first row of the sequence in q / out
  const float c2 = a.scale_log2;
  // query row i sits at key index i + qoff of the K/V buffers
  // (an idle sequence holds length -1 until its first chunk is committed: it starts at position 0)
  const int n_old = a.d_lens ? max(a.d_lens[b], 0) - (a.old_sub ? S : 0) : 0;
  const int qoff = (a.stage_window > 0 && n_old > a.stage_window - 1) ? a.stage_window - 1 : n_old;

  // Q^T fragments: lane (row, hh) holds dims kk*16 + hh*8 .. +7.  With 4 wavefronts each one first copies its 32
  // query rows (8 KiB) into a private slice of stage 1 with coalesced direct loads (4 whole rows per instruction)
  // and picks its fragments up from there; read straight from global memory, the fragment pattern touches 32
  // different rows per instruction.
  bf16x8_t qf[8];
  constexpr bool kStageQ = (NW == 4);
  if constexpr (kStageQ) {
    uint16_t* slice = smem + 4 * kBlockElems + wave * (32 * kTiledDim);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = min(r0 + 4 * i + (lane >> 4), S - 1);  // rows past the prompt re-read the last row (never stored)
      const uint16_t* src = a.q + ((qrow0 + r) * a.Hq + hq) * kTiledDim + (lane & 15) * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(slice + i * 512), 16, 0, 0);
    }
  } else {
    const uint16_t* qp = a.q + ((qrow0 + row) * a.Hq + hq) * kTiledDim + hh * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4_t raw = {0u, 0u, 0u, 0u};
      if (row < S) raw = *(const u32x4_t*)(qp + kk * 16);
      qf[kk] = __builtin_bit_cast(bf16x8_t, raw);
    }
  }

  const int nblk_valid = (qoff + S + kBlockKeys - 1) / kBlockKeys;
  const u32x4_t* Kt = (const u32x4_t*)a.Kt;
  const u32x4_t* Vg = (const u32x4_t*)(a.Vt + (a.v_base[b] + (int64_t)h * (a.v_slots[b] >> 5)) * kBlockElems);

  const int last_row = min(q0 + rows_wg, S) - 1;
  const int jt_hi = (last_row + qoff) / kPfKeys;
  const int jt_lo = W > 0 ? max(0, q0 + qoff - W + 1) / kPfKeys : 0;
  const int r0k = r0 + qoff, rowk = row + qoff;  // this wavefront's first row / this lane's row as key indices

  floatx16_t o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  float m = -INFINITY, lsum = 0.f;  // m in raw score units

  // Where block kb of this (sequence, kv head) sits in the K buffer.  Contiguous: one base, read once.  Paged: the
  // page ids of a tile's two blocks are looked up one tile ahead of their use (struct TilePages), because a wait
  // for such a lookup also waits for every direct load issued before it.
  const bool k_paged = a.k_pages.ids != nullptr;
  const int64_t k_first = k_paged ? 0 : a.k_base[b] + (int64_t)h * (a.k_slots[b] >> 5);
  const int32_t* k_ids = k_paged ? a.k_pages.ids + (int64_t)b * a.k_pages.max_pages : nullptr;
  const int k_shift = a.k_pages.shift, k_mask = (1 << a.k_pages.shift) - 1;
  // A block past the prompt (the second half of the last tile) is read from the last block that holds keys instead:
  // finite data for products that the causal mask discards, and no second code path in the tile loop.
  struct TilePages { int pg[2]; };
  auto pages_of = [&](int jt) {
    TilePages t;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int kb = min(jt * 2 + j, nblk_valid - 1);
      t.pg[j] = (k_paged && kb >= 0) ? k_ids[kb >> k_shift] : 0;
    }
    return t;
  };
  // block index in the K buffer, kept in scalar registers (everything about it is the same for the whole workgroup)
  auto k_block = [&](int kb, int pg) -> int64_t {
    if (!k_paged) return k_first + kb;
    const int pgs = __builtin_amdgcn_readfirstlane(pg);
    return (((int64_t)pgs * a.Hkv + h) << k_shift) + (kb & k_mask);
  };

  // Tile jt -> stage buf.  A block is 512 16-byte pieces of K and of V; piece p = T*i + tid, with T threads, lands at
  // LDS byte 16*p of its block, which is what a direct load does when the wave-uniform LDS base is that of the wave's
  // first lane.  The global address is a uniform block base plus the lane's 32-bit byte offset, so that per tile only
  // scalar arithmetic is left.
  const char* const Kbytes = (const char*)a.Kt;
  const char* const Vbytes = (const char*)Vg;
  auto issue = [&](int jt, int buf, const TilePages& tp) {
    constexpr int T = NW * 64;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int kb = min(jt * 2 + j, nblk_valid - 1);
      const char* kbase = Kbytes + k_block(kb, tp.pg[j]) * (int64_t)(kBlockElems * 2);
      const char* vbase = Vbytes + (int64_t)kb * (kBlockElems * 2);
#pragma unroll
      for (int i = 0; i < 512 / T; ++i) {
        const uint32_t off = (uint32_t)(T * i + tid) * 16u;
        uint16_t* lk = sK(buf) + j * kBlockElems + (T * i + wave * 64) * 8;
        uint16_t* lv = sV(buf) + j * kBlockElems + (T * i + wave * 64) * 8;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kbase + off),
                                         (__attribute__((address_space(3))) void*)lk, 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vbase + off),
                                         (__attribute__((address_space(3))) void*)lv, 16, 0, 0);
      }
    }
  };

  const int key_row = pf_key_of_row(col);  // key (within a block) this lane feeds as MFMA row `col`
  issue(jt_lo, 0, pages_of(jt_lo));
  TilePages next_pages = pages_of(jt_lo + 1);
  if constexpr (kStageQ) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the query rows (and the first tile) of this wavefront landed
    const uint16_t* slice = smem + 4 * kBlockElems + wave * (32 * kTiledDim) + col * kTiledDim + hh * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = *(const bf16x8_t*)(slice + kk * 16);
    // stage 1 is overwritten only after the first barrier of the loop, which this wavefront reaches after these reads
  }
  for (int jt = jt_lo; jt <= jt_hi; ++jt) {
    const int buf = (jt - jt_lo) & 1;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's direct loads of tile jt have landed
    __syncthreads();                     // ... and everybody's; everybody is also done reading the other stage
    if (jt < jt_hi) {
      issue(jt + 1, buf ^ 1, next_pages);
      next_pages = pages_of(jt + 2);  // arrives during this tile's arithmetic
    }

    const int k0 = jt * kPfKeys;
    // whole tile masked for every row of this wavefront?
    if (k0 > r0k + 31) continue;
    if (W > 0 && k0 + kPfKeys - 1 < r0k - W + 1) continue;
    const bool need_mask = (k0 + kPfKeys - 1 > r0k) || (W > 0 && k0 < r0k + 31 - W + 1);

    // All 16 K fragments of the tile are requested from LDS before the first MFMA (the scheduling barrier keeps the
    // compiler from sinking each read next to its use, which would expose the LDS latency sixteen times).
    bf16x8_t kf[2][8];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const uint16_t* kb = sK(buf) + sub * kBlockElems + (key_row >> 4) * 2048 + (key_row & 15) * 8;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) kf[sub][kk] = *(const bf16x8_t*)(kb + (2 * kk + hh) * 128);
    }
    __builtin_amdgcn_sched_barrier(0);
    // the wavefront feeding the matrix pipe wins issue arbitration over its SIMD mate's softmax arithmetic
    __builtin_amdgcn_s_setprio(3);
    floatx16_t s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[sub][i] = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)  // fragments are consumed in the order they were requested
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sub][kk], qf[kk], s[sub], 0, 0, 0);
    // The 16 V fragments are requested now, so that they arrive while the softmax arithmetic runs.
    halfx8_t vf[2][2][4];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        // dims 32*db + col, keys of piece g = 2u + hh
        const uint16_t* vb = sV(buf) + sub * kBlockElems + (col >> 4) * 512 + ((2 * u + hh) * 16 + (col & 15)) * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db) vf[sub][u][db] = *(const halfx8_t*)(vb + db * 1024);
      }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);
    if (need_mask) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          // register i is MFMA row 8*(i/4) + 4*hh + i%4, which holds key pi(row)
          const int key = k0 + sub * 32 + pf_key_of_row(8 * (i >> 2) + 4 * hh + (i & 3));
          const bool ok = (key <= rowk) && (W == 0 || key > rowk - W);
          s[sub][i] = ok ? s[sub][i] : -INFINITY;
        }
    }
    float mx = s[0][0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[0][i]);
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[1][i]);
    // the other half of the row lives in lane l ^ 32: exchanged with the lane-swap instruction (vector ALU), not with
    // an LDS permute, whose result would queue behind the V fragments requested just before
    {
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    const float m_new = fmaxf(m, mx);
    // rescale only when some row of the wavefront saw a new maximum (rare after the first tiles)
    if (__any(m_new > m)) {
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c2);  // m = -inf -> 0 (accumulators are 0 anyway)
      const float al = (m_new > m) ? alpha : 1.f;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= al;
      lsum *= al;
      m = m_new;
    }
    // row with nothing visible yet: all its scores are -inf, any finite offset gives p = 0
    const float mc = (m == -INFINITY) ? 0.f : m * c2 - kPShift;
    float psum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        u32x4_t pw;
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[sub][8 * u + 2 * jp], c2, -mc));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[sub][8 * u + 2 * jp + 1], c2, -mc));
          psum += p0 + p1;
          pw[jp] = pf_pack_f16(p0, p1);
        }
        const halfx8_t pf = __builtin_bit_cast(halfx8_t, pw);
#pragma unroll
        for (int db = 0; db < 4; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[sub][u][db], pf, o[db], 0, 0, 0);
      }
    }
    lsum += psum;
  }

  lsum += __shfl_xor(lsum, 32);
  const float inv = 1.f / lsum;
  if constexpr (sizeof(OutT) == 2 && NW == 4) {
    // bf16 output: transpose through LDS so that every store instruction writes 4 whole 256-byte rows
    constexpr int kRowPitch = kTiledDim + 8;  // elements; the pad spreads the rows over the LDS banks
    __syncthreads();                          // every wavefront is done with the K/V stages
    uint16_t* slice = smem + wave * (32 * kRowPitch);
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        uint2 w;
        w.x = pf_pack_bf16(o[db][4 * q4] * inv, o[db][4 * q4 + 1] * inv);
        w.y = pf_pack_bf16(o[db][4 * q4 + 2] * inv, o[db][4 * q4 + 3] * inv);
        *(uint2*)(slice + col * kRowPitch + 32 * db + 8 * q4 + 4 * hh) = w;
      }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's slice is complete (it is private to it)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rl = 4 * i + (lane >> 4);
      const u32x4_t v = *(const u32x4_t*)(slice + rl * kRowPitch + (lane & 15) * 8);
      if (r0 + rl < S)
        *(u32x4_t*)((uint16_t*)a.out + ((qrow0 + r0 + rl) * a.Hq + hq) * kTiledDim + (lane & 15) * 8) = v;
    }
  } else if (row < S) {
    OutT* op = (OutT*)a.out + ((qrow0 + row) * a.Hq + hq) * kTiledDim;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d = 32 * db + 8 * q4 + 4 * hh;
        const float v0 = o[db][4 * q4] * inv, v1 = o[db][4 * q4 + 1] * inv, v2 = o[db][4 * q4 + 2] * inv,
                    v3 = o[db][4 * q4 + 3] * inv;
        if constexpr (sizeof(OutT) == 4) {
          *(floatx4_t*)((float*)op + d) = floatx4_t{v0, v1, v2, v3};
        } else {
          uint2 w;
          w.x = pf_pack_bf16(v0, v1);
          w.y = pf_pack_bf16(v2, v3);
          *(uint2*)((uint16_t*)op + d) = w;
        }
      }
  }
}

hipError_t launch_prefill_tiled(const PrefillLaunch& L, hipStream_t s) {
  TiledPrefillParams p;
  p.q = (const uint16_t*)L.q; p.out = L.out;
  p.Kt = (const uint16_t*)L.Kt; p.k_base = L.k_base; p.k_slots = L.k_slots;
  p.k_pages = L.k_pages; p.Hkv = L.Hkv;
  p.Vt = (const uint16_t*)L.Vt; p.v_base = L.v_base; p.v_slots = L.v_slots;
  p.window = L.window; p.S = L.S; p.Hq = L.Hq; p.G = L.G;
  p.scale_log2 = L.scale * kLog2e;
  p.d_lens = L.d_lens; p.old_sub = L.old_sub; p.stage_window = L.stage_window;
  p.q_first = L.d_q_first; p.q_len = L.d_q_len;
  // Full causal layers: 8 wavefronts (256 query rows) share each K/V tile, which halves the tile loads per row
  // (about 6 % faster).  Sliding layers: 4 wavefronts (128 rows), because a taller workgroup spans more keys than
  // its rows can see (8 is about 20 % slower at W = 1024).
  const bool f32 = L.out_dtype == MIXATTN_F32;
  const int waves = L.waves ? L.waves : (L.window == 0 ? 8 : 4);
  // query heads per workgroup: the largest of 4, 2, 1 that divides the group size (and the wavefront count), unless set
  int hg = L.heads;
  if (hg <= 0) hg = (L.G % 4 == 0) ? 4 : (L.G % 2 == 0) ? 2 : 1;
  if (L.G % hg != 0 || waves % hg != 0) hg = 1;
  p.hg = hg;
  const int rows_wg = 32 * waves / hg;
  const dim3 grid((L.S + rows_wg - 1) / rows_wg, L.Hq / hg, L.batch), block(64 * waves);
  if (waves == 8) {
    if (f32) hipLaunchKernelGGL((prefill_tiled_kernel<float, 8>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((prefill_tiled_kernel<uint16_t, 8>), grid, block, 0, s, p);
  } else {
    if (f32) hipLaunchKernelGGL((prefill_tiled_kernel<float, 4>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((prefill_tiled_kernel<uint16_t, 4>), grid, block, 0, s, p);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Row-major path: one wavefront per (query row, query head), keys visited one by one from the caller's
// prompt tensors.  Plain fp32 arithmetic; used for fp32 and for shapes outside the MFMA path.
// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ inline float pf_load(const T* p);
template <>
__device__ inline float pf_load<float>(const float* p) { return *p; }
template <>
__device__ inline float pf_load<uint16_t>(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }

struct RowPrefillParams {
  const void* q; const void* k; const void* v; void* out;
  int window, S, Hq, Hkv, G, D;
  float scale;
  // chunked prefill: positions before n_old = d_lens[b] - old_sub come from the row-major cache (slot = position,
  // or position mod ring for a sliding cache that has not yet received this chunk)
  const void* Kc; const void* Vc; const int64_t* d_base; const int32_t* d_slots;
  const int32_t* d_lens; int old_sub; int ring;
  // chunks of different lengths: rows q_first[b] .. + q_len[b] - 1 of the packed tensors (nullptr: uniform S)
  const int64_t* q_first; const int32_t* q_len;
};

template <typename T, typename OutT>
__global__ __launch_bounds__(256) void prefill_rowmajor_kernel(RowPrefillParams a) {
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int hq = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63;
  const int S = a.q_len ? a.q_len[b] : a.S;
  if (i >= S) return;
  const int64_t qrow0 = a.q_first ? a.q_first[b] : (int64_t)b * a.S;
  const int h = hq / a.G, D = a.D;
  const T* qp = (const T*)a.q + ((qrow0 + i) * a.Hq + hq) * D;
  float qv[4], acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int d = lane + 64 * t;
    qv[t] = d < D ? pf_load<T>(qp + d) : 0.f;
    acc[t] = 0.f;
  }
  // (an idle sequence holds length -1 until its first chunk is committed: it starts at position 0)
  const int n_old = a.d_lens ? max(a.d_lens[b], 0) - (a.old_sub ? S : 0) : 0;
  const int pos = n_old + i;  // absolute position of this query row
  const int lo = a.window > 0 ? max(0, pos - a.window + 1) : 0;
  const int slots = a.d_lens ? a.d_slots[b] : 0;
  float m = -INFINITY, l = 0.f;
  for (int p = lo; p <= pos; ++p) {
    const T* kp;
    const T* vp;
    if (p >= n_old) {
      const int64_t off = ((qrow0 + (p - n_old)) * a.Hkv + h) * D;
      kp = (const T*)a.k + off;
      vp = (const T*)a.v + off;
    } else {
      const int64_t off = (a.d_base[b] + (int64_t)h * slots + (a.ring > 0 ? p % a.ring : p)) * D;
      kp = (const T*)a.Kc + off;
      vp = (const T*)a.Vc + off;
    }
    float part = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < D) part += qv[t] * pf_load<T>(kp + d);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
    const float sc = part * a.scale;
    const float m_new = fmaxf(m, sc);
    const float alpha = expf(m - m_new);
    const float pr = expf(sc - m_new);
    l = l * alpha + pr;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int d = lane + 64 * t;
      if (d < D) acc[t] = acc[t] * alpha + pr * pf_load<T>(vp + d);
    }
    m = m_new;
  }
  OutT* op = (OutT*)a.out + ((qrow0 + i) * a.Hq + hq) * D;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int d = lane + 64 * t;
    if (d < D) {
      const float v = acc[t] / l;
      if constexpr (sizeof(OutT) == 4) ((float*)op)[d] = v;
      else ((uint16_t*)op)[d] = (uint16_t)pf_bf16_bits_rn(v);
    }
  }
}

hipError_t launch_prefill_rowmajor(const PrefillLaunch& L, hipStream_t s) {
  RowPrefillParams p;
  p.q = L.q; p.k = L.k_src; p.v = L.v_src; p.out = L.out;
  p.window = L.window; p.S = L.S; p.Hq = L.Hq; p.Hkv = L.Hkv; p.G = L.G; p.D = L.D; p.scale = L.scale;
  p.Kc = L.Kc; p.Vc = L.Vc; p.d_base = L.c_base; p.d_slots = L.c_slots; p.d_lens = L.d_lens; p.old_sub = L.old_sub;
  p.ring = L.ring;
  p.q_first = L.d_q_first; p.q_len = L.d_q_len;
  const dim3 grid((L.S + 3) / 4, L.Hq, L.batch), block(256);
  const bool f32 = L.kv_dtype == MIXATTN_F32, of32 = L.out_dtype == MIXATTN_F32;
  if (f32 && of32) hipLaunchKernelGGL((prefill_rowmajor_kernel<float, float>), grid, block, 0, s, p);
  else if (f32) hipLaunchKernelGGL((prefill_rowmajor_kernel<float, uint16_t>), grid, block, 0, s, p);
  else if (of32) hipLaunchKernelGGL((prefill_rowmajor_kernel<uint16_t, float>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((prefill_rowmajor_kernel<uint16_t, uint16_t>), grid, block, 0, s, p);
  return hipGetLastError();
}

}  // namespace mixattn
