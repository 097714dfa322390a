// Chunk-prefill attention on the matrix cores (bf16, head_dim 128).
//
// The new chunk's queries attend to the retained cache and causally to their own
// chunk (Sec. 2.1: reuse of retained states; cost per chunk is fixed by the
// window sizes).  The work is a dense contraction: 4 * head_dim flops per
// (query, visible key, head), K/V read once per kv head, so the bound is bf16
// MFMA throughput.
//
// Tiling (64-wide wavefronts, v_mfma_f32_32x32x16_bf16):
//   * The G query heads that share a kv head are packed into one row space,
//     row = query * G + head_in_group, so one K/V tile serves all of them.
//   * A wavefront owns 32 rows; a workgroup of NW wavefronts owns NW * 32 rows of one
//     kv head and one key range (split-KV); key ranges are merged afterwards with
//     the log-sum-exp rule.  Two wavefronts share a SIMD (NW = 8, or two workgroups
//     of 4 per CU): inside ONE wavefront an MFMA and the vector instructions behind it
//     do not overlap (1 MFMA + 8 FMA measure 62 cycles, not 32), across two they do, as
//     long as the vector work sits in small pieces behind the MFMAs (about 20 cycles of
//     it per MFMA are hidden; the default kernel interleaves accordingly).
//   * Scores are computed transposed, S^T = K Q^T, so that a lane holds scores of
//     ONE query row: row max and row sum are in-lane plus one exchange between the
//     two half-wavefronts, and the output O^T = V^T P^T keeps one query row per
//     lane, so rescaling by the running max is a per-lane scalar.
//   * K tiles (64 keys) are staged in LDS with their rows permuted (bits 2 and 3 of
//     the key index swapped): the accumulator layout of S^T then hands every lane 8
//     consecutive keys per 16-key step, which is exactly the B-operand layout of
//     the second product, so P never moves between lanes.
//   * K and V^T tiles reach LDS with direct global -> LDS loads, four slots per tensor, and V^T fragments are
//     plain 16-byte LDS reads; the softmax of a tile is spread through the output MFMAs of the tile before
//     (see the kernel's own header).

#include <hip/hip_bf16.h>

#include <algorithm>
#include <type_traits>

#include "sv_internal.h"

namespace sv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));

constexpr int D = 128;               // head_dim
constexpr int TK = 64;               // keys per tile
constexpr int KROW = D * 2;          // bytes per K row in LDS (16-byte chunks XOR-swizzled by row)

__device__ __forceinline__ int perm_key(int key) {  // swap bits 2 and 3
  return (key & ~0xC) | ((key & 4) << 1) | ((key & 8) >> 1);
}
__device__ __forceinline__ int k_lds_off(int row, int chunk) {  // row: permuted key, chunk: 16-byte unit of head_dim
  return row * KROW + ((chunk ^ (row & 15)) << 4);   // 16 consecutive rows read 16 distinct chunks: no bank conflict
}

// ---------------------------------------------------------------------------------
// The kernel (8 wavefronts, one workgroup per CU).
//   * K/V tiles go from HBM to LDS with the direct global -> LDS load (16 bytes per lane, lane L lands at
//     base + 16 L; confirmed on the device), so staging costs no registers and no LDS store instructions.  The
//     swizzles are applied on the global side: each lane fetches the chunk that belongs at its LDS position.
//       K: LDS row m holds key perm_key(m); position p of the row holds chunk p ^ (m & 15).
//       V^T: LDS row = head dim (64 keys, 128 bytes); position p holds the 8-key chunk p ^ ((row >> 1) & 7).
//   * Four LDS slots per tensor: in iteration t tiles t-1 .. t+1 may be read while tile t+2 arrives.
//   * The matrix-core work of an iteration (scores of one tile, output of another) does not depend on the
//     softmax running in the same iteration; LDS operands are fetched one batch ahead of the MFMAs that use them.
// ---------------------------------------------------------------------------------
constexpr int PIPE_TILE = TK * D * 2;   // 16 KB per tile, unpadded
constexpr int PIPE_HROW = D + 8;         // halves per row of a wavefront's partial result on its way out through LDS

// 16 bytes per lane from global memory straight into LDS: lane L's bytes land at lds_dst + 16 L (lds_dst is
// uniform over the wavefront and travels in M0).  Written as assembly on purpose: the compiler then does not
// see a pending write to LDS and inserts no wait for ALL outstanding direct loads in front of later LDS
// reads; the kernel waits itself (vmcnt(0), then a workgroup barrier) before a tile is first read.
// (M0 is named as clobbered on purpose: nothing else in these kernels uses it, and the compiler must not assume it
// survives; clang notes that M0 is a reserved register, which is the point.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* base, uint32_t lane_off, char* lds_dst) {
  // base (uniform) travels in a scalar register pair, the lane's byte offset in one VGPR
  const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_dst);
  const uint64_t b = (uint64_t)base;
  // (the builtin returns a signed int: convert each half through uint32_t, or the low half sign-extends)
  const uint64_t bu = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32) |
                      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(lane_off), "s"(bu)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// causal 1 bit, key ranges 7 bits (kMaxChunkSplits), group 4 bits, kv heads 8 bits, row tiles 12 bits
__host__ __device__ inline uint32_t chunk_shape(int causal, int n_splits, int G, int n_kv_heads, int row_tiles) {
  return (uint32_t)(causal != 0) | (uint32_t)n_splits << 1 | (uint32_t)G << 8 | (uint32_t)n_kv_heads << 12 |
         (uint32_t)row_tiles << 20;
}
// STORE: the chunk's own K and V are not in the cache yet.  k_new / v_new hold them as the caller produced them
// ([n_q][n_kv_heads][128], K un-rotated) and cs_tab their cos/sin; a workgroup first stores, of its kv head, exactly the
// new keys it is about to read (K rows rotated, V into its V^T blocks), waits for its stores and then proceeds as
// ever.  Workgroups of different row tiles store the same keys with the same values: each reads what it wrote itself
// (through its own CU's and XCD's caches), the copies agree, and the last row tile's workgroups write every new key
// of their ranges, so the cache is complete when the launch ends.  One launch and one pass over the new rows fewer
// per layer; worth it while the chunk is short, since the store is repeated per row tile.
template <int NW, int KS, int VS, bool STORE>
__global__ __launch_bounds__(NW * 64, 2) void k_attn_chunk_pipe(
    __hip_bfloat16* kc, __hip_bfloat16* vc, int n_q, int n_kv, int keys_per_split,
    uint32_t head_stride_elems, uint32_t shape, int n_q_heads, const __hip_bfloat16* __restrict__ q,
    const float2* __restrict__ cs_tab, __hip_bfloat16* __restrict__ out, float* __restrict__ part_o,
    float* __restrict__ part_ml, const __hip_bfloat16* __restrict__ k_new, const __hip_bfloat16* __restrict__ v_new) {
  // (the arguments up to cs_tab are the 14 dwords that reach the wavefront in SGPRs at launch: everything the first
  // direct loads and the query loads need, the small integers in one word, see chunk_shape; the grid's size, which
  // would be a fetch of its own, follows from them)
  const int causal = shape & 1, n_splits = (shape >> 1) & 127, G = (shape >> 8) & 15, n_kv_heads = (shape >> 12) & 255,
            row_tiles = (int)(shape >> 20);
  constexpr float c_log2 = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
  constexpr int ROWS_WG = NW * 32;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  char* const sKbase = smem;
  char* const sVbase = smem + KS * PIPE_TILE;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;
  // One-dimensional grid of 8 x ceil(W / 8) workgroups for W = pairs x row tiles units of work, a pair being a
  // (key range, kv head).  Consecutive workgroup ids go to the 8 XCDs in turn; XCD x takes the units
  // [x * per_xcd, (x + 1) * per_xcd) in pair-major order, so the row tiles of a pair run on the same XCD (of two, where
  // a pair straddles the boundary) and share its L2 copy of the pair's K and V^T tiles, and every XCD gets the same
  // number of workgroups whatever the number of pairs (one workgroup fits a CU: 32 per XCD at most).
  const int per_xcd = (row_tiles * n_kv_heads * n_splits + 7) >> 3;   // = gridDim.x / 8
  const int unit = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
  const int pair = unit / row_tiles, rt = unit % row_tiles;
  if (pair >= n_kv_heads * n_splits) return;   // padding ids
  // (key range major: an XCD's pairs are one key range of several kv heads.  Kv head major, its pairs then share
  // their queries, cuts the launch's reads from 25 to 15 MB at 9 ranges and measured 1.7 us slower.)
  const int hk = pair % n_kv_heads, sp = pair / n_kv_heads;
  const int slot0 = n_kv - n_q;
  const int n_rows = n_q * G;

  const int row_last = min(n_rows, (rt + 1) * ROWS_WG) - 1;
  const int k_begin = sp * keys_per_split;
  int k_end = min(n_kv, k_begin + keys_per_split);
  if (causal) k_end = min(k_end, slot0 + row_last / G + 1);
  const int n_tiles = k_end > k_begin ? (k_end - k_begin + TK - 1) / TK : 0;
  if (n_tiles == 0) {   // nothing visible in this key range: an empty partial (weight zero, its row is never read)
    const int row = rt * ROWS_WG + wave * 32 + l32;
    if (row < n_rows && n_splits > 1 && hh == 0) {
      const size_t p = ((size_t)(row / G) * n_splits + sp) * n_q_heads + hk * G + row % G;
      *(float4*)(part_ml + p * 4) = make_float4(-INFINITY, 0.f, 1.f, 0.f);
    }
    return;
  }

  __hip_bfloat16* const kbase = kc + (size_t)hk * head_stride_elems;
  __hip_bfloat16* const vtbase = vc + (size_t)hk * head_stride_elems;   // V is stored as V^T in blocks of 8 keys

  if constexpr (STORE) {
    const int ks0 = max(k_begin, slot0), ks1 = k_end;   // the new keys this workgroup reads
    if (ks0 < ks1) {
      // K: 8 lanes per row, a lane owns 16 bytes of the low half and the matching 16 of the high half (the rotary
      // pairs are lane-local); 64 rows per pass, four passes' loads (row halves and cos/sin) in flight at once,
      // unconditional on a clamped row
      const int t8 = tid & 7, r8 = tid >> 3;
      for (int base = ks0; base < ks1; base += 4 * (NW * 8)) {
        uint4 lo[4], hi[4];
        float4 cs[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = min(base + i * (NW * 8) + r8, ks1 - 1) - slot0;
          const __hip_bfloat16* src = k_new + ((size_t)j * n_kv_heads + hk) * D + 8 * t8;
          lo[i] = *(const uint4*)src;
          hi[i] = *(const uint4*)(src + D / 2);
          const float4* c4 = (const float4*)(cs_tab + (size_t)j * (D / 2) + 8 * t8);
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) cs[i][e2] = c4[e2];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = base + i * (NW * 8) + r8;
          bf16x8 a8 = *(bf16x8*)&lo[i], b8 = *(bf16x8*)&hi[i];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float4 r4 = cs[i][e >> 1];
            const float cx = (e & 1) ? r4.z : r4.x, sx = (e & 1) ? r4.w : r4.y;
            const float a = (float)a8[e], b = (float)b8[e];
            a8[e] = (__bf16)(a * cx - b * sx);
            b8[e] = (__bf16)(b * cx + a * sx);
          }
          if (key < ks1) {
            __hip_bfloat16* dst = kbase + (size_t)key * D + 8 * t8;
            *(bf16x8*)dst = a8;
            *(bf16x8*)(dst + D / 2) = b8;
          }
        }
      }
      // V: a lane takes one head dim of the 8 keys of a block (eight 2-byte loads; a wavefront reads 128 contiguous
      // bytes of a row per instruction) and writes the block row, 16 bytes, consecutive lanes consecutive rows; where
      // a block is only partly this workgroup's (older tokens below the first new key, keys past its range above),
      // element by element.  Four blocks per lane in flight.
      const int dv = tid & (D - 1), bsub = tid / D;
      constexpr int BP = NW * 64 / D;   // blocks per pass of the workgroup
      const int b0 = ks0 >> 3, b1 = (ks1 - 1) >> 3;
      const unsigned short* vsrc = (const unsigned short*)v_new + (size_t)hk * D + dv;
      for (int base = b0; base <= b1; base += 4 * BP) {
        unsigned short x[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int be = min(base + u * BP + bsub, b1);
#pragma unroll
          for (int kk = 0; kk < 8; ++kk) {
            const int j = min(max(8 * be + kk, ks0), ks1 - 1) - slot0;
            x[u][kk] = vsrc[(size_t)j * n_kv_heads * D];
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int blk = base + u * BP + bsub;
          if (blk <= b1) {
            unsigned short* dst = (unsigned short*)vtbase + vt_elem(8 * (int64_t)blk, dv);
            if (8 * blk >= ks0 && 8 * blk + 8 <= ks1) {
              *(uint4*)dst = make_uint4(x[u][0] | (uint32_t)x[u][1] << 16, x[u][2] | (uint32_t)x[u][3] << 16,
                                        x[u][4] | (uint32_t)x[u][5] << 16, x[u][6] | (uint32_t)x[u][7] << 16);
            } else {
#pragma unroll
              for (int kk = 0; kk < 8; ++kk)
                if (8 * blk + kk >= ks0 && 8 * blk + kk < ks1) dst[kk] = x[u][kk];
            }
          }
        }
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);   // this wavefront's stores have reached the L2
      __syncthreads();                      // ... and everybody's: the tiles may be loaded
    }
  }

  // tile t -> LDS slot t & 3; each tile is 16 / NW direct-load instructions per wavefront, instruction wi
  // filling 1 KB of the slot.  The lane's source offset inside a tile does not depend on the tile:
  //   K:   LDS row m = 4 wi + lane / 16 holds key perm_key(m), its 16-byte chunks XOR-swizzled by m & 15;
  //   V^T: LDS row d = 8 wi + lane / 8 (128 bytes: 8 chunks of 8 keys); chunk c sits at position
  //        c ^ ((d >> 1) & 7), so that 16 lanes reading one chunk index of 16 consecutive rows touch 16
  //        distinct 16-byte bank groups.  In the cache a 64-key tile is 8 consecutive blocks of
  //        [128 head dims][8 keys] (2 KB each): chunk c of row d is row d of block c.
  // Tiles past the range re-read the last one.  The last tile may run up to 63 keys past the key range: those
  // K rows and V^T columns are other slots of the same head's plane (planes hold whole 64-key tiles); their
  // scores are replaced, not scaled, by the mask, and stale V values are finite (the store starts out cleared).
  uint32_t k_lane_off[16 / NW], v_lane_off[16 / NW];
#pragma unroll
  for (int i = 0; i < 16 / NW; ++i) {
    const int wi = wave + i * NW;
    const int m = 4 * wi + (lane >> 4), p = lane & 15;
    k_lane_off[i] = (uint32_t)(perm_key(m) * (D * 2) + ((p ^ (m & 15)) << 4));
    const int dd = 8 * wi + (lane >> 3), c = (lane & 7) ^ ((dd >> 1) & 7);
    v_lane_off[i] = (uint32_t)(c * (kVBElems * 2) + dd * (kVB * 2));
  }
  const char* const k_tiles = (const char*)(kbase + (size_t)k_begin * D);
  const char* const v_tiles = (const char*)(vtbase + (size_t)(k_begin / TK) * (TK * D));   // k_begin is a multiple of 64
  auto dma_tile = [&](int which, int t) {
    const int te = min(t, n_tiles - 1);
    char* slot = (which ? sVbase : sKbase) + (t % (which ? VS : KS)) * PIPE_TILE;
    const char* src = (which ? v_tiles : k_tiles) + (size_t)te * PIPE_TILE;
#pragma unroll
    for (int i = 0; i < 16 / NW; ++i)
      dma16(src, which ? v_lane_off[i] : k_lane_off[i], slot + (wave + i * NW) * 1024);
  };
  dma_tile(0, 0);   // the first pair of tiles
  dma_tile(0, 1);
  dma_tile(1, 0);

  const int row = rt * ROWS_WG + wave * 32 + l32;
  const bool rvalid = row < n_rows;
  const int rr = rvalid ? row : n_rows - 1;
  const int qi = rr / G, hg = rr % G;
  const int limit = min(causal ? slot0 + qi : n_kv - 1, k_end - 1);
  const int wg_first_limit = causal ? slot0 + (rt * ROWS_WG) / G : n_kv - 1;
  bf16x8 qf[8];
  {
    // rr is a valid row for every lane (lanes past the last row repeat it; nothing of theirs is stored), so all loads
    // are unconditional and issued together: queries and, for the rotation, their cos/sin in one memory round trip
    const __hip_bfloat16* qp = q + ((size_t)qi * n_q_heads + hk * G + hg) * D + hh * 8;
    uint4 raw[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) raw[kk] = *(const uint4*)(qp + kk * 16);
    if (cs_tab != nullptr) {
      // Un-rotated queries (the per-second step): rotate them here, with the cos/sin the run's registration
      // tabulated per (token, pair), and round to bf16 as a rotation pass in memory would have.  The lane holds
      // dims 16 kk + 8 hh + e, so the pair (i, i + 64) is (kk, kk + 4) of its own registers.
      const float4* cs = (const float4*)(cs_tab + (size_t)qi * (D / 2) + 8 * hh);   // pairs 16 kk + 8 hh + e
      float4 c4[4][4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) c4[kk][e2] = cs[8 * kk + e2];
      __builtin_amdgcn_sched_barrier(0);   // all 24 loads go out before the first of them is waited for
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qf[kk] = *(bf16x8*)&raw[kk];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float4 r4 = c4[kk][e >> 1];
          const float cx = (e & 1) ? r4.z : r4.x, sx = (e & 1) ? r4.w : r4.y;
          const float a = (float)qf[kk][e], b = (float)qf[kk + 4][e];
          qf[kk][e] = (__bf16)(a * cx - b * sx);
          qf[kk + 4][e] = (__bf16)(b * cx + a * sx);
        }
    } else {
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qf[kk] = *(bf16x8*)&raw[kk];
    }
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // V^T fragment of head-dim block db, key step ks: row 32 db + l32, chunk 2 ks + hh (swizzled as written)
  int v_ks_off[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) v_ks_off[ks] = l32 * 128 + (((2 * ks + hh) ^ ((l32 >> 1) & 7)) << 4);
  const float tau = 8.0f / c_log2;   // 8 binary orders, in score units
  auto rescale = [&](float alpha) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
  };
  // Matrix-core work of one phase: S^T of tile tq (groups 0..3: two 16-dim steps of both 32-key blocks each)
  // and O^T += V^T(tile tp) P^T (groups 4..7: one 16-key step of all four 32-dim blocks each), 4 MFMAs per
  // group.  The LDS operands of a group are requested two groups ahead of the MFMAs that use them, into three
  // rotating register sets; scheduling fences keep the compiler from sinking the reads back to their uses, so
  // the LDS latency hides behind 8 MFMAs (256 cycles) of this wavefront.
  auto matrix = [&](auto do_qk, auto do_pv, int tq, int tp, f32x16 (&sacc)[2], const bf16x8 (&pf)[4]) {
    constexpr int G0 = decltype(do_qk)::value ? 0 : 4, G1 = decltype(do_pv)::value ? 8 : 4;
    const char* sK = sKbase + (tq % KS) * PIPE_TILE;
    const char* sV = sVbase + (tp % VS) * PIPE_TILE;
    bf16x8 fb[3][4];
    auto fetch = [&](int g, bf16x8 (&f)[4]) {
      if (g < 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          f[i] = *(const bf16x8*)(sK + k_lds_off((i & 1) * 32 + l32, 2 * (2 * g + (i >> 1)) + hh));
      } else {
        const int ks = g - 4;
#pragma unroll
        for (int db = 0; db < 4; ++db) f[db] = *(const bf16x8*)(sV + v_ks_off[ks] + db * 4096);
      }
    };
    auto mm = [&](int g, const bf16x8 (&f)[4]) {
      if (g == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[0], qf[0], zero, 0, 0, 0);
        sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[1], qf[0], zero, 0, 0, 0);
        sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2], qf[1], sacc[0], 0, 0, 0);
        sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[3], qf[1], sacc[1], 0, 0, 0);
      } else if (g < 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          sacc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], qf[2 * g + (i >> 1)], sacc[i & 1], 0, 0, 0);
      } else {
#pragma unroll
        for (int db = 0; db < 4; ++db)
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[db], pf[g - 4], oacc[db], 0, 0, 0);
      }
    };
    fetch(G0, fb[G0 % 3]);
    fetch(G0 + 1, fb[(G0 + 1) % 3]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = G0; g < G1; ++g) {
      if (g + 2 < G1) fetch(g + 2, fb[(g + 2) % 3]);
      __builtin_amdgcn_sched_barrier(0);
      mm(g, fb[g % 3]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto arrive_all = [&]() {   // all of this wavefront's direct loads have landed; then everybody's
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
  };
  f32x16 sacc[2];
  bf16x8 pf[4];
  const int full_keys = min(wg_first_limit + 1, k_end) - k_begin;   // tiles every row of the workgroup sees whole
  const int n_full = full_keys > 0 ? min(full_keys / TK, n_tiles) : 0;
  arrive_all();
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  {
    // Interleaved order: iteration t = S(t) = QK(t), then the softmax of tile t with the 16 MFMAs of
    // O += P(t-1) V(t-1) spread through it (one MFMA, then the exp / pack / sum of two scores).  Inside one
    // wavefront an MFMA and the vector instructions behind it do not overlap, but the other wavefront of the
    // SIMD runs the same mix, and two such streams keep the matrix pipe busy where long separate phases do not.
    bf16x8 pfb[4];
    auto mixed = [&](auto do_pv, int t, const bf16x8 (&pp)[4], bf16x8 (&pc)[4]) {
      const char* sV = sVbase + ((t + VS - 1) % VS) * PIPE_TILE;   // tile t - 1
      bf16x8 fb[3][4];
      auto fetch = [&](int ks, bf16x8 (&f)[4]) {
#pragma unroll
        for (int db = 0; db < 4; ++db) f[db] = *(const bf16x8*)(sV + v_ks_off[ks] + db * 4096);
      };
      if constexpr (decltype(do_pv)::value) {
        fetch(0, fb[0]);
        fetch(1, fb[1]);
      }
      if (t >= n_full) {
        const int kt0 = k_begin + t * TK;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kt0 + 32 * kb + 16 * (r >> 3) + 8 * hh + (r & 7);
            if (key > limit) sacc[kb][r] = -INFINITY;
          }
      }
      // The probabilities are taken against the reference maximum as it stands (it moves
      // only in steps of more than 8 binary orders), so nothing waits for this tile's row maxima.  They are
      // not even computed unless a row's sum of the tile exceeds 2^8 (no p above 2^8 can hide under that) or a
      // row has no reference yet; then the exact maxima decide, and on a step the tile is redone.
      float mc = (m_run == -INFINITY ? 0.f : m_run) * c_log2;
      float psum = 0.f;
      typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
      bf16x2 ones;
      ones[0] = (__bf16)1.0f, ones[1] = (__bf16)1.0f;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          // One unit = one MFMA + the exp / pack / sum of two scores.  Empty volatile statements that
          // name a unit's input before it and its outputs (for the MFMA: the fragment it has read) after it
          // tie the units to this order; the scheduler otherwise gathers the 16 MFMAs behind the vector work.
          const int kb = ks >> 1, r = (ks & 1) * 8 + 2 * db;
          if constexpr (decltype(do_pv)::value) {
            asm volatile("" : "+v"(mc), "+v"(v_ks_off[(ks + 2) & 3]));
            if (db == 0 && ks + 2 < 4) fetch(ks + 2, fb[(ks + 2) % 3]);
            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks % 3][db], pp[ks], oacc[db], 0, 0, 0);
          }
          bf16x2 pk;
          pk[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[kb][r], c_log2, -mc));
          pk[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[kb][r + 1], c_log2, -mc));
          psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);   // row sum of the rounded P, as the MFMA sees it
          if constexpr (decltype(do_pv)::value)
            asm volatile("" : "+v"(pk), "+v"(psum), "+v"(fb[ks % 3][db]));
          pc[ks][2 * db] = pk[0], pc[ks][2 * db + 1] = pk[1];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      float alpha = 1.f;
      if (__any(!(psum <= 256.f) || m_run == -INFINITY)) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        if (__any(m_new > m_run + tau)) {   // a step of the reference maximum: exact new maxima, tile redone, O rescaled
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c_log2);
        m_run = m_new;
        mc = m_use * c_log2;
        psum = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const int kb = j >> 1, r = (j & 1) * 8 + e;
            bf16x2 pk;
            pk[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[kb][r], c_log2, -mc));
            pk[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[kb][r + 1], c_log2, -mc));
            psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);
            pc[j][e] = pk[0], pc[j][e + 1] = pk[1];
          }
        rescale(alpha);
        }
      }
      l_run = l_run * alpha + psum;
    };
    // Tiles go in pairs: at the start of pair (t0, t0 + 1) the direct loads of the next pair's tiles are issued
    // (K t0 + 2, t0 + 3 and V^T t0 + 1, t0 + 2 land in the slots the previous pair read), at its end one
    // wait + barrier: half the barriers of a per-tile scheme and twice the slack between the wavefronts.
    static_assert(KS == 4 && VS == 4, "pair schedule uses four slots per tensor");
    auto dma_pair = [&](int t0) {
      dma_tile(0, t0 + 2);
      dma_tile(0, t0 + 3);
      dma_tile(1, t0 + 1);
      dma_tile(1, t0 + 2);
    };
    dma_pair(0);
    matrix(yes, no, 0, 0, sacc, pf);
    mixed(no, 0, pfb, pf);
    if (n_tiles > 1) {
      matrix(yes, no, 1, 0, sacc, pf);
      mixed(yes, 1, pf, pfb);
    }
    arrive_all();
    for (int t0 = 2; t0 < n_tiles; t0 += 2) {   // even tiles leave P in pf, odd ones in pfb
      dma_pair(t0);
      matrix(yes, no, t0, 0, sacc, pf);
      mixed(yes, t0, pfb, pf);
      if (t0 + 1 < n_tiles) {
        matrix(yes, no, t0 + 1, 0, sacc, pf);
        mixed(yes, t0 + 1, pf, pfb);
      }
      arrive_all();
    }
    if (n_tiles & 1) matrix(no, yes, 0, n_tiles - 1, sacc, pf);
    else matrix(no, yes, 0, n_tiles - 1, sacc, pfb);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // no direct load may be in flight when the wavefront ends
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const int h = hk * G + hg;
  if (n_splits == 1) {
    if (!rvalid) return;
    const float inv = 1.0f / l_tot;
    __hip_bfloat16* op = out + ((size_t)qi * n_q_heads + h) * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int dv = 32 * db + 8 * r4 + 4 * hh;
        __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(oacc[db][r4 * 4 + e] * inv);
        *(uint2*)(op + dv) = *(uint2*)&pk;
      }
    return;
  }
  // Partial result of a key range.  What leaves is the NORMALISED partial o / l (a convex combination of V rows, so
  // its magnitude is bounded by the values of V) as fp16 scaled per row by a power of two that brings the row's
  // largest element into [1/2, 1): half the bytes of fp32 at 11 bits of mantissa relative to the row maximum, and no
  // fp16 range limit on V.  (max, sum, scale) go along in fp32; the merge weighs the rows by sum * 2^(max - M).
  // A lane holds one row in 8-byte pieces, so stored directly every instruction would touch 32 rows; the
  // wavefront's 32 rows go through LDS (its own 8.5 KB, rows padded to 136 halves) and leave as whole 256-byte rows.
  float amax = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(oacc[db][r]));
  amax = fmaxf(amax, __shfl_xor(amax, 32));
  const float inv_l = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  amax *= inv_l;
  // the power of two above the largest normalised element (1 for an all-zero row); exponent clamped below the top
  const uint32_t ebits = min((__float_as_uint(amax) & 0x7f800000u) + 0x00800000u, 0x7e800000u);
  const float scale = amax > 1e-30f ? __uint_as_float(ebits) : 1.f;   // (rows of vanishing magnitude keep scale 1)
  const float mul = inv_l / scale;
  __syncthreads();   // every wavefront is past its last read of the tile slots
  _Float16* so = (_Float16*)smem + wave * (32 * PIPE_HROW);
  if (rvalid) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int dv = 32 * db + 8 * r4 + 4 * hh;
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        h4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (_Float16)(oacc[db][r4 * 4 + e] * mul);
        *(h4*)(so + l32 * PIPE_HROW + dv) = pk;
      }
    if (hh == 0) {
      const size_t p = ((size_t)qi * n_splits + sp) * n_q_heads + h;
      *(float4*)(part_ml + p * 4) = make_float4(m_run == -INFINITY ? -INFINITY : m_run * c_log2, l_tot, scale, 0.f);
    }
  }
  // 16 lanes per row, 16 bytes per lane: four whole rows per store instruction
  _Float16* part_h = (_Float16*)part_o;
  const int l16 = lane & 15, rsub = lane >> 4;
#pragma unroll 4
  for (int i = 0; i < 8; ++i) {
    const int r = 4 * i + rsub, row2 = rt * ROWS_WG + wave * 32 + r;
    if (row2 < n_rows) {
      const size_t p2 = ((size_t)(row2 / G) * n_splits + sp) * n_q_heads + hk * G + row2 % G;
      *(uint4*)(part_h + p2 * D + 8 * l16) = *(const uint4*)(so + r * PIPE_HROW + 8 * l16);
    }
  }
}

// ---------------------------------------------------------------------------------
// Merge of the key ranges of a chunk-prefill launch: out = sum_s w_s o_s / sum_s w_s with w_s = l_s 2^(m_s - M)
// and o_s the normalised partial (fp16 x row scale, see above).  16 lanes per (query, head) row, 8 head dims per
// lane; 16 rows per workgroup.  Ranges go in passes of 8 while more than 12 are left, then one pass of exactly
// what is left; within a pass every load (one 16-byte piece and the (max, sum, scale) record per key range) is
// unconditional and issued before any is used, so a pass costs one memory round trip (guarded by the record's
// contents, the pieces' loads wait for the records': two).  A range of weight zero (nothing visible to the row:
// its piece was never written) is read all the same and left out by a select.
// grid: ceil(n_q * n_q_heads / 16), block: 256 threads.
// ---------------------------------------------------------------------------------
constexpr int kMaxChunkSplits = 64;
__global__ __launch_bounds__(256) void k_chunk_combine(const _Float16* __restrict__ part_h,
                                                       const float* __restrict__ part_ml,
                                                       __hip_bfloat16* __restrict__ out, int n_rows_total, int n_splits,
                                                       int n_q_heads) {
  const int row = blockIdx.x * 16 + (threadIdx.x >> 4), l16 = threadIdx.x & 15;
  if (row >= n_rows_total) return;
  const int qi = row / n_q_heads, h = row % n_q_heads;
  const size_t base = (size_t)qi * n_splits * n_q_heads + h;   // split s adds s * n_q_heads
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float wsum = 0.f, m_ref = -INFINITY;
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  auto pass = [&](auto Uc, int s0) {
    constexpr int U = decltype(Uc)::value;
    float4 ml[U];
    h8 v[U];
    // (the records first, then the pieces: measured 0.7 us per launch faster at 8 ranges than the two interleaved)
#pragma unroll
    for (int j = 0; j < U; ++j) ml[j] = *(const float4*)(part_ml + (base + (size_t)(s0 + j) * n_q_heads) * 4);
#pragma unroll
    for (int j = 0; j < U; ++j) v[j] = *(const h8*)(part_h + (base + (size_t)(s0 + j) * n_q_heads) * D + 8 * l16);
    float mx = m_ref;
#pragma unroll
    for (int j = 0; j < U; ++j) mx = fmaxf(mx, ml[j].x);
    const float resc = m_ref == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_ref - mx);
    wsum *= resc;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= resc;
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const bool any = ml[j].x != -INFINITY;
      const float w = any ? ml[j].y * __builtin_amdgcn_exp2f(ml[j].x - mx) : 0.f;
      const float ws = w * ml[j].z;
      wsum += w;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += any ? ws * (float)v[j][e] : 0.f;
    }
    m_ref = mx;
  };
  int s0 = 0;
  for (; n_splits - s0 > 12; s0 += 8) pass(std::integral_constant<int, 8>{}, s0);
  switch (n_splits - s0) {
    case 1: pass(std::integral_constant<int, 1>{}, s0); break;
    case 2: pass(std::integral_constant<int, 2>{}, s0); break;
    case 3: pass(std::integral_constant<int, 3>{}, s0); break;
    case 4: pass(std::integral_constant<int, 4>{}, s0); break;
    case 5: pass(std::integral_constant<int, 5>{}, s0); break;
    case 6: pass(std::integral_constant<int, 6>{}, s0); break;
    case 7: pass(std::integral_constant<int, 7>{}, s0); break;
    case 8: pass(std::integral_constant<int, 8>{}, s0); break;
    case 9: pass(std::integral_constant<int, 9>{}, s0); break;
    case 10: pass(std::integral_constant<int, 10>{}, s0); break;
    case 11: pass(std::integral_constant<int, 11>{}, s0); break;
    default: pass(std::integral_constant<int, 12>{}, s0); break;
  }
  const float inv = 1.0f / wsum;
  typedef __bf16 b8 __attribute__((ext_vector_type(8)));
  b8 o8;
#pragma unroll
  for (int e = 0; e < 8; ++e) o8[e] = (__bf16)(acc[e] * inv);
  *(b8*)(out + (size_t)row * D + 8 * l16) = o8;
}

constexpr int kNW = 8, kKS = 4, kVS = 4;   // 8 wavefronts, 4 + 4 tile slots: 128 KB of LDS, one workgroup per CU
constexpr int kLds = std::max((kKS + kVS) * PIPE_TILE, kNW * 32 * PIPE_HROW * 2);

}  // namespace

hipError_t attn_chunk_mfma_init() {
  // more than 64 KB of dynamic LDS has to be asked for, once per device
  hipError_t e = hipFuncSetAttribute((const void*)k_attn_chunk_pipe<kNW, kKS, kVS, false>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void*)k_attn_chunk_pipe<kNW, kKS, kVS, true>,
                             hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
}

// Key ranges of a chunk-prefill launch over n_kv keys: (count, keys per range).
static void chunk_ranges(const sv_cache* c, int n_q, int n_kv, int& n_splits, int& keys_per_split) {
  constexpr int ROWS_WG = kNW * 32;
  const int G = c->group, Hkv = c->cfg.n_kv_heads;
  const int row_tiles = (n_q * G + ROWS_WG - 1) / ROWS_WG;
  n_splits = c->opt[SV_OPT_CHUNK_SPLITS];
  if (n_splits <= 0) {
    // at most one workgroup per CU (256), ranges of at least 4 tiles; among those the count that leaves a workgroup
    // the fewest tiles, and of equals the smallest (fewer partial results to merge)
    const int most = std::min(std::max(1, 256 / std::max(1, row_tiles * Hkv)), std::max(1, n_kv / (4 * TK)));
    const int tiles = (n_kv + TK - 1) / TK;
    n_splits = 1;
    for (int s = 2; s <= most; ++s)
      if ((tiles + s - 1) / s < (tiles + n_splits - 1) / n_splits) n_splits = s;
  }
  n_splits = std::min<int64_t>(n_splits, std::max<int64_t>(1, c->part_rows / n_q));
  n_splits = std::min(n_splits, kMaxChunkSplits);
  keys_per_split = ((n_kv + n_splits - 1) / n_splits + TK - 1) / TK * TK;
  n_splits = (n_kv + keys_per_split - 1) / keys_per_split;
}

// Every key range's workgroups rotate the queries they load (about 2 us of vector work per workgroup): worth it
// against a rotation pass over Q in memory while a query row is loaded by few ranges (long chunks: 2 ranges at 1024
// tokens), not when 8 ranges repeat it (256 tokens).
bool attn_chunk_rotates_on_load(const sv_cache* c, int stream, int n_q) {
  int n_splits, kps;
  chunk_ranges(c, n_q, (int)c->st[stream].len, n_splits, kps);
  return n_splits <= 2;
}

// Whether the attention launch should store the chunk's K/V itself (see the kernel).  Every workgroup that reads new
// keys stores them first, the last row tile's all of them, at the pace of ONE CU's memory pipeline (measured: 0.8 us
// for 64 keys, 3.2 for 256, 6.5 for 384, 9.8 for 512), where a launch of its own spreads that over the device; doing
// without that launch takes about 3 us off the layer, of which the rotation of the queries on load gives 1.5 back.
// So it pays when the store hides behind the other workgroups' attention work, i.e. when the key ranges that hold
// new keys are that much shorter than a full range (at 4096 + 2 x 512 retained tokens and 272 new ones, 8 ranges of
// 10 tiles hold the retained keys and the ninth, 5 tiles, exactly the chunk: 36.5 -> 35.4 us per layer), or sticks
// out by no more than a microsecond.
bool attn_chunk_stores_tokens(const sv_cache* c, int stream, int n_q) {
  if (!c->use_mfma || n_q > 512 || c->opt[SV_OPT_CHUNK_STORE] == 1) return false;
  if (c->opt[SV_OPT_CHUNK_STORE] == 2) return true;
  const int n_kv = (int)c->st[stream].len, slot0 = n_kv - n_q;
  int n_splits, kps;
  chunk_ranges(c, n_q, n_kv, n_splits, kps);
  if (n_splits < 2) return false;
  const float us_tile = 1.9f;   // a 64-key tile of one workgroup in the steady loop
  for (int sp = slot0 / kps; sp < n_splits; ++sp) {
    const int k0 = sp * kps, k1 = std::min(n_kv, k0 + kps), n_new = k1 - std::max(k0, slot0);
    const float store_us = 0.2f + 0.0125f * (float)n_new + 0.013f * (float)std::max(0, n_new - 256);
    if ((float)((k1 - k0 + TK - 1) / TK) * us_tile + store_us > (float)(kps / TK) * us_tile + 1.0f) return false;
  }
  return true;
}

hipError_t launch_attn_chunk_mfma(const sv_cache* c, int stream, int layer, const void* q, int n_q, void* o,
                                  int causal, bool rotate_q, hipStream_t s, const void* k_new, const void* v_new) {
  if ((k_new != nullptr) != (v_new != nullptr) || (k_new != nullptr && !rotate_q)) return hipErrorInvalidValue;
  constexpr int ROWS_WG = kNW * 32;
  const StreamState& st = c->st[stream];
  const int n_kv = (int)st.len, G = c->group, Hkv = c->cfg.n_kv_heads;
  const int row_tiles = (n_q * G + ROWS_WG - 1) / ROWS_WG;
  int n_splits, keys_per_split;
  chunk_ranges(c, n_q, n_kv, n_splits, keys_per_split);
  const int units = row_tiles * Hkv * n_splits;
  if (n_splits > 127 || G > 15 || Hkv > 255 || row_tiles > 4095 || c->head_stride / 2 > 0xffffffffull)
    return hipErrorInvalidValue;   // what chunk_shape and the 32-bit head stride can carry
  auto kernel = k_new != nullptr ? k_attn_chunk_pipe<kNW, kKS, kVS, true> : k_attn_chunk_pipe<kNW, kKS, kVS, false>;
  hipLaunchKernelGGL(kernel, dim3((units + 7) / 8 * 8), dim3(kNW * 64), kLds, s,
                     (__hip_bfloat16*)c->kv_ptr(stream, st.cur, layer, 0),
                     (__hip_bfloat16*)c->kv_ptr(stream, st.cur, layer, 1), n_q, n_kv, keys_per_split,
                     (uint32_t)(c->head_stride / 2), chunk_shape(causal, n_splits, G, Hkv, row_tiles),
                     c->cfg.n_q_heads, (const __hip_bfloat16*)q,
                     rotate_q ? c->cs_tab + (size_t)stream * c->cfg.max_q_tokens * (D / 2) : nullptr,
                     (__hip_bfloat16*)o, c->part_o, c->part_ml, (const __hip_bfloat16*)k_new,
                     (const __hip_bfloat16*)v_new);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_splits == 1) return e;
  const int rows_total = n_q * c->cfg.n_q_heads;
  hipLaunchKernelGGL(k_chunk_combine, dim3((rows_total + 15) / 16), dim3(256), 0, s, (const _Float16*)c->part_o,
                     c->part_ml, (__hip_bfloat16*)o, rows_total, n_splits, c->cfg.n_q_heads);
  return hipGetLastError();
}

}  // namespace sv
