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
//     of 4 per CU), so one wavefront's softmax overlaps the other's MFMAs and the
//     vector ALU is fed every cycle (a single wavefront issues at half rate).
//   * Scores are computed transposed, S^T = K Q^T, so that a lane holds scores of
//     ONE query row: row max and row sum are in-lane plus one exchange between the
//     two half-wavefronts, and the output O^T = V^T P^T keeps one query row per
//     lane, so rescaling by the running max is a per-lane scalar.
//   * K tiles (64 keys) are staged in LDS with their rows permuted (bits 2 and 3 of
//     the key index swapped): the accumulator layout of S^T then hands every lane 8
//     consecutive keys per 16-key step, which is exactly the B-operand layout of
//     the second product, so P never moves between lanes.
//   * V tiles are staged row-major, exactly as loaded, and read back as the V^T
//     operand with the LDS transpose read (ds_read_b64_tr_b16), two per operand.
//   * LDS is double-buffered: the next tile's global loads are issued into registers
//     before the current tile's MFMAs and stored after them; one barrier per tile.

#include <hip/hip_bf16.h>

#include <algorithm>
#include <cstdlib>
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
constexpr int VROW = D * 2 + 64;     // bytes per V row in LDS: the 4 rows x 64 bytes that 32 lanes of a transpose read
                                     // touch fall in distinct banks (64 banks x 4 bytes)
constexpr int K_BYTES = TK * KROW;
constexpr int V_BYTES = TK * VROW;
constexpr int BUF_BYTES = K_BYTES + V_BYTES;

__device__ __forceinline__ int perm_key(int key) {  // swap bits 2 and 3
  return (key & ~0xC) | ((key & 4) << 1) | ((key & 8) >> 1);
}
__device__ __forceinline__ int k_lds_off(int row, int chunk) {  // row: permuted key, chunk: 16-byte unit of head_dim
  return row * KROW + ((chunk ^ (row & 15)) << 4);   // 16 consecutive rows read 16 distinct chunks: no bank conflict
}

// LDS transpose read: within each group of 16 lanes, lane j hands in the address of 4 consecutive 16-bit
// elements and receives element (j & 3) of the chunks of lanes (j >> 2) + 4 e, e = 0..3.  Pointing lane j
// at row r0 + (j >> 2), columns c0 + 4 (j & 3) .. + 3 of a row-major tile returns column c0 + j of rows
// r0 .. r0 + 3.  (Layout confirmed with an index pattern on the device.)
__device__ __forceinline__ v4i16 lds_read_tr(const char* base, int byte_off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (v4i16 __attribute__((address_space(3)))*)((__attribute__((address_space(3))) char*)base + byte_off));
}

template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void k_attn_chunk_mfma(
    const __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ kc, const __hip_bfloat16* __restrict__ vc,
    __hip_bfloat16* __restrict__ out, float* __restrict__ part_o, float* __restrict__ part_ml, int n_q, int n_kv,
    int causal, int n_splits, int keys_per_split, int n_q_heads, int G, size_t head_stride_elems, float c_log2) {
  constexpr int NT = NW * 64;
  constexpr int ROWS_WG = NW * 32;
  constexpr int CH = (TK * 16) / NT;   // 16-byte chunks of K (and of V) per thread per tile
  extern __shared__ __attribute__((aligned(16))) char smem[];   // two buffers of (K tile, V tile)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;
  const int rt = blockIdx.x, hk = blockIdx.y, sp = blockIdx.z;
  const int slot0 = n_kv - n_q;
  const int n_rows = n_q * G;

  // key range of this workgroup, trimmed to what its last query may see
  const int row_last = min(n_rows, (rt + 1) * ROWS_WG) - 1;
  const int k_begin = sp * keys_per_split;
  int k_end = min(n_kv, k_begin + keys_per_split);
  if (causal) k_end = min(k_end, slot0 + row_last / G + 1);
  const int n_tiles = k_end > k_begin ? (k_end - k_begin + TK - 1) / TK : 0;

  const __hip_bfloat16* kbase = kc + (size_t)hk * head_stride_elems;
  const __hip_bfloat16* vbase = vc + (size_t)hk * head_stride_elems;

  uint4 kreg[CH], vreg[CH];
  auto issue_loads = [&](int t) {
    const int kt0 = k_begin + t * TK;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int cid = tid + i * NT, key = cid >> 4, c16 = cid & 15;
      const bool ok = kt0 + key < k_end;   // rows past the range read as zero (finite, masked anyway)
      kreg[i] = ok ? *(const uint4*)(kbase + (size_t)(kt0 + key) * D + c16 * 8) : make_uint4(0, 0, 0, 0);
      vreg[i] = ok ? *(const uint4*)(vbase + (size_t)(kt0 + key) * D + c16 * 8) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_tile = [&](char* buf) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int cid = tid + i * NT, key = cid >> 4, c16 = cid & 15;
      *(uint4*)(buf + k_lds_off(perm_key(key), c16)) = kreg[i];
      *(uint4*)(buf + K_BYTES + key * VROW + c16 * 16) = vreg[i];
    }
  };

  if (n_tiles > 0) issue_loads(0);

  // this lane's query row
  const int row = rt * ROWS_WG + wave * 32 + l32;
  const bool rvalid = row < n_rows;
  const int rr = rvalid ? row : n_rows - 1;
  const int qi = rr / G, hg = rr % G;
  const int limit = min(causal ? slot0 + qi : n_kv - 1, k_end - 1);
  bf16x8 qf[8];
  {
    const __hip_bfloat16* qp = q + ((size_t)qi * n_q_heads + hk * G + hg) * D + hh * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      uint4 raw = rvalid ? *(const uint4*)(qp + kk * 16) : make_uint4(0, 0, 0, 0);
      qf[kk] = *(bf16x8*)&raw;
    }
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  if (n_tiles > 0) store_tile(smem);
  __syncthreads();

  // lane geometry of the V^T transpose reads: 16-lane group g16 covers dims 16 (g16 & 1) + j of a 32-dim
  // block and keys 8 (g16 >> 1) + e (+4 for the second read) of a 16-key step
  const int j16 = lane & 15, g16 = lane >> 4;
  const int v_lane_off = (8 * (g16 >> 1) + (j16 >> 2)) * VROW + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2;

  for (int t = 0; t < n_tiles; ++t) {
    const char* sK = smem + (t & 1) * BUF_BYTES;
    const char* sV = sK + K_BYTES;
    if (t + 1 < n_tiles) issue_loads(t + 1);
    const int kt0 = k_begin + t * TK;

    // S^T = K Q^T for 2 blocks of 32 keys
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 a = *(const bf16x8*)(sK + k_lds_off(kb * 32 + l32, 2 * kk + hh));
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], sacc[kb], 0, 0, 0);
      }
    }

    // online softmax, one query row per lane.  Register r of key block kb holds key
    // kt0 + 32 kb + 16 (r / 8) + 8 hh + r % 8.
    const bool need_mask = kt0 + TK - 1 > (causal ? slot0 + (rt * ROWS_WG) / G : n_kv - 1) || kt0 + TK > k_end;
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kt0 + 32 * kb + 16 * (r >> 3) + 8 * hh + (r & 7);
          if (key > limit) sacc[kb][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;   // a row may be fully masked in this tile
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c_log2);
    const float mc = m_use * c_log2;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][r], c_log2, -mc));
        psum += p;
        pf[kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
      }
    l_run = l_run * alpha + psum;
    if (__any(m_new > m_run)) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    m_run = m_new;

    // O^T += V^T P^T : 4 blocks of 32 dims, 4 steps of 16 keys
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const int off = v_lane_off + 16 * ks * VROW + 64 * db;
        const v4i16 a0 = lds_read_tr(sV, off), a1 = lds_read_tr(sV, off + 4 * VROW);
        const v8i16 a8 = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)&a8, pf[ks], oacc[db], 0, 0, 0);
      }
    }

    if (t + 1 < n_tiles) store_tile(smem + ((t + 1) & 1) * BUF_BYTES);
    __syncthreads();
  }

  // epilogue: lane holds its row, dims 32 db + 8 (r / 4) + 4 hh + r % 4
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (!rvalid) return;
  const int h = hk * G + hg;
  if (n_splits == 1) {
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
  } else {
    const size_t p = ((size_t)qi * n_splits + sp) * n_q_heads + h;
    float* po = part_o + p * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int dv = 32 * db + 8 * r4 + 4 * hh;
        *(float4*)(po + dv) = make_float4(oacc[db][r4 * 4], oacc[db][r4 * 4 + 1], oacc[db][r4 * 4 + 2],
                                          oacc[db][r4 * 4 + 3]);
      }
    if (hh == 0) {
      part_ml[p * 2] = m_run == -INFINITY ? -INFINITY : m_run * c_log2;
      part_ml[p * 2 + 1] = l_tot;
    }
  }
}

// ---------------------------------------------------------------------------------
// Pipelined variant (8 wavefronts, one workgroup per CU).
//   * K/V tiles go from HBM to LDS with the direct global -> LDS load (16 bytes per lane, lane L lands at
//     base + 16 L; confirmed on the device), so staging costs no registers and no LDS store instructions.  The
//     swizzles are applied on the global side: each lane fetches the chunk that belongs at its LDS position.
//       K: LDS row m holds key perm_key(m); position p of the row holds chunk p ^ (m & 15).
//       V: LDS row = key; position p holds chunk p ^ (4 (key & 3)), which puts the 4 rows x 64 bytes that
//          32 lanes of a transpose read touch into distinct banks without padding.
//   * Four LDS slots per tensor: in iteration t tiles t-1 .. t+1 may be read while tile t+2 arrives.
//   * The matrix-core work of an iteration (scores of one tile, output of another) does not depend on the
//     softmax running in the same iteration; LDS operands are fetched one batch ahead of the MFMAs that use them.
// ---------------------------------------------------------------------------------
constexpr int PIPE_SLOTS = 4;
constexpr int PIPE_TILE = TK * D * 2;   // 16 KB per tile, unpadded
constexpr int PIPE_LDS = 2 * PIPE_SLOTS * PIPE_TILE;

__device__ __forceinline__ void dma16(const void* gsrc, char* lds_dst) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)(__attribute__((address_space(3))) char*)lds_dst,
                                   16, 0, 0);
}

template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void k_attn_chunk_pipe(
    const __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ kc, const __hip_bfloat16* __restrict__ vc,
    __hip_bfloat16* __restrict__ out, float* __restrict__ part_o, float* __restrict__ part_ml, int n_q, int n_kv,
    int causal, int n_splits, int keys_per_split, int n_q_heads, int G, size_t head_stride_elems, float c_log2,
    int phase_mode) {
  constexpr int ROWS_WG = NW * 32;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  char* const sKbase = smem;
  char* const sVbase = smem + PIPE_SLOTS * PIPE_TILE;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;
  const int rt = blockIdx.x, hk = blockIdx.y, sp = blockIdx.z;
  const int slot0 = n_kv - n_q;
  const int n_rows = n_q * G;

  const int row_last = min(n_rows, (rt + 1) * ROWS_WG) - 1;
  const int k_begin = sp * keys_per_split;
  int k_end = min(n_kv, k_begin + keys_per_split);
  if (causal) k_end = min(k_end, slot0 + row_last / G + 1);
  const int n_tiles = k_end > k_begin ? (k_end - k_begin + TK - 1) / TK : 0;
  if (n_tiles == 0) {   // nothing visible in this key range: an empty partial
    const int row = rt * ROWS_WG + wave * 32 + l32;
    if (row < n_rows && n_splits > 1) {
      const size_t p = ((size_t)(row / G) * n_splits + sp) * n_q_heads + hk * G + row % G;
      for (int d = hh * 64; d < hh * 64 + 64; d += 4) *(float4*)(part_o + p * D + d) = make_float4(0.f, 0.f, 0.f, 0.f);
      if (hh == 0) part_ml[p * 2] = -INFINITY, part_ml[p * 2 + 1] = 0.f;
    }
    return;
  }

  const __hip_bfloat16* kbase = kc + (size_t)hk * head_stride_elems;
  const __hip_bfloat16* vbase = vc + (size_t)hk * head_stride_elems;

  // tile t -> LDS slot t & 3.  Rows past the key range re-read the last row (finite values, masked keys).
  auto dma_tile = [&](int t) {
    const int kt0 = k_begin + t * TK;
    char* kslot = sKbase + (t & (PIPE_SLOTS - 1)) * PIPE_TILE;
    char* vslot = sVbase + (t & (PIPE_SLOTS - 1)) * PIPE_TILE;
#pragma unroll
    for (int i = 0; i < 16 / NW; ++i) {
      const int wi = wave + i * NW;            // this instruction fills LDS rows 4 wi .. 4 wi + 3
      const int m = 4 * wi + (lane >> 4), p = lane & 15;
      const int gk = min(kt0 + perm_key(m), k_end - 1);
      dma16(kbase + (size_t)gk * D + ((p ^ (m & 15)) << 3), kslot + wi * 1024);
      const int gv = min(kt0 + m, k_end - 1);
      dma16(vbase + (size_t)gv * D + ((p ^ ((m & 3) << 2)) << 3), vslot + wi * 1024);
    }
  };

  dma_tile(0);
  dma_tile(1);

  const int row = rt * ROWS_WG + wave * 32 + l32;
  const bool rvalid = row < n_rows;
  const int rr = rvalid ? row : n_rows - 1;
  const int qi = rr / G, hg = rr % G;
  const int limit = min(causal ? slot0 + qi : n_kv - 1, k_end - 1);
  const int wg_first_limit = causal ? slot0 + (rt * ROWS_WG) / G : n_kv - 1;
  bf16x8 qf[8];
  {
    const __hip_bfloat16* qp = q + ((size_t)qi * n_q_heads + hk * G + hg) * D + hh * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      uint4 raw = rvalid ? *(const uint4*)(qp + kk * 16) : make_uint4(0, 0, 0, 0);
      qf[kk] = *(bf16x8*)&raw;
    }
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // V^T transpose-read geometry: 16-lane group g16 covers dims 16 (g16 & 1) + j of a 32-dim block and keys
  // 8 (g16 >> 1) + e of a 16-key step; x = row & 3 selects the swizzle of the 64-byte segment
  const int j16 = lane & 15, g16 = lane >> 4, vx = j16 >> 2;
  const int v_lane_off = (8 * (g16 >> 1) + vx) * 256 + ((2 * (g16 & 1) + ((j16 & 3) >> 1)) << 4) + (j16 & 1) * 8;
  int v_db_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) v_db_off[db] = (db ^ vx) << 6;
  const bool mfma_first = phase_mode == 0 ? true : (phase_mode == 1 ? ((wave >> 2) & 1) == 0 : (wave & 1) == 0);

  auto softmax = [&](auto masked, int t, f32x16 (&sacc)[2], bf16x8 (&pf)[4], bool& changed) -> float {
    const int kt0 = k_begin + t * TK;
    if constexpr (decltype(masked)::value) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kt0 + 32 * kb + 16 * (r >> 3) + 8 * hh + (r & 7);
          if (key > limit) sacc[kb][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c_log2);
    const float mc = m_use * c_log2;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][r], c_log2, -mc));
        psum += p;
        pf[kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
      }
    l_run = l_run * alpha + psum;
    changed = __any(m_new > m_run);
    m_run = m_new;
    return alpha;
  };
  auto rescale = [&](float alpha) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
  };
  auto qk_block = [&](int t, f32x16 (&sacc)[2]) {   // S^T of tile t
    const char* sK = sKbase + (t & (PIPE_SLOTS - 1)) * PIPE_TILE;
    bf16x8 fa[2][4];
    auto fetch = [&](int b, bf16x8 (&f)[4]) {   // fragments kk = 2b, 2b+1 of key blocks 0 and 1
#pragma unroll
      for (int i = 0; i < 4; ++i)
        f[i] = *(const bf16x8*)(sK + k_lds_off((i & 1) * 32 + l32, 2 * (2 * b + (i >> 1)) + hh));
    };
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
    fetch(0, fa[0]);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      if (b + 1 < 4) fetch(b + 1, fa[(b + 1) & 1]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        sacc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[b & 1][i], qf[2 * b + (i >> 1)], sacc[i & 1], 0, 0, 0);
    }
  };
  auto pv_block = [&](int t, const bf16x8 (&pf)[4]) {   // O^T += V^T(tile t) P^T
    const char* sV = sVbase + (t & (PIPE_SLOTS - 1)) * PIPE_TILE + v_lane_off;
    bf16x8 fa[2][4];
    auto fetch = [&](int ks, bf16x8 (&f)[4]) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const int off = 16 * ks * 256 + v_db_off[db];
        const v4i16 a0 = lds_read_tr(sV, off), a1 = lds_read_tr(sV, off + 4 * 256);
        const v8i16 a8 = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
        f[db] = *(const bf16x8*)&a8;
      }
    };
    fetch(0, fa[0]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks + 1 < 4) fetch(ks + 1, fa[(ks + 1) & 1]);
#pragma unroll
      for (int db = 0; db < 4; ++db)
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][db], pf[ks], oacc[db], 0, 0, 0);
    }
  };
  auto arrive = [&]() {   // this wavefront's direct loads have landed; then everybody's
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
  };

  // "matrix first":  iteration t = [S(t) = QK(t), O += PV(t-1)] then softmax(t)
  // "softmax first": iteration t = softmax(t) (S(t) from the previous iteration) then [O += PV(t), S(t+1)]
  f32x16 sacc[2];
  bf16x8 pf[4];
  bool changed;
  const int full_keys = min(wg_first_limit + 1, k_end) - k_begin;   // tiles every row of the workgroup sees whole
  const int n_full = full_keys > 0 ? min(full_keys / TK, n_tiles) : 0;
  arrive();
  if (mfma_first) {
    auto iter = [&](auto masked, int t) {
      dma_tile(t + 2);
      qk_block(t, sacc);
      if (t > 0) pv_block(t - 1, pf);
      const float alpha = softmax(masked, t, sacc, pf, changed);
      if (changed) rescale(alpha);
      arrive();
    };
    int t = 0;
    for (; t < n_full; ++t) iter(std::false_type{}, t);
    for (; t < n_tiles; ++t) iter(std::true_type{}, t);
    pv_block(n_tiles - 1, pf);
  } else {
    qk_block(0, sacc);
    auto iter = [&](auto masked, int t) {
      dma_tile(t + 2);
      const float alpha = softmax(masked, t, sacc, pf, changed);
      if (changed) rescale(alpha);
      pv_block(t, pf);
      if (t + 1 < n_tiles) qk_block(t + 1, sacc);
      arrive();
    };
    int t = 0;
    for (; t < n_full; ++t) iter(std::false_type{}, t);
    for (; t < n_tiles; ++t) iter(std::true_type{}, t);
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (!rvalid) return;
  const int h = hk * G + hg;
  if (n_splits == 1) {
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
  } else {
    const size_t p = ((size_t)qi * n_splits + sp) * n_q_heads + h;
    float* po = part_o + p * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int dv = 32 * db + 8 * r4 + 4 * hh;
        *(float4*)(po + dv) = make_float4(oacc[db][r4 * 4], oacc[db][r4 * 4 + 1], oacc[db][r4 * 4 + 2],
                                          oacc[db][r4 * 4 + 3]);
      }
    if (hh == 0) {
      part_ml[p * 2] = m_run == -INFINITY ? -INFINITY : m_run * c_log2;
      part_ml[p * 2 + 1] = l_tot;
    }
  }
}

int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  return v && *v ? std::atoi(v) : dflt;
}

template <int NW, bool PIPE>
hipError_t launch_t(const sv_cache* c, int stream, int layer, const void* q, int n_q, void* o, int causal,
                    hipStream_t s) {
  constexpr int ROWS_WG = NW * 32;
  constexpr int kLds = PIPE ? PIPE_LDS : 2 * BUF_BYTES;
  const void* kern = PIPE ? (const void*)k_attn_chunk_pipe<NW> : (const void*)k_attn_chunk_mfma<NW>;
  static bool attr_set = false;   // more than 64 KB of LDS has to be asked for once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const StreamState& st = c->st[stream];
  const int n_kv = (int)st.len, G = c->group, Hkv = c->cfg.n_kv_heads;
  const int row_tiles = (n_q * G + ROWS_WG - 1) / ROWS_WG;
  int n_splits = env_int("SV_CHUNK_SPLITS", 0);
  if (n_splits <= 0) {
    // fill 256 CUs with 8 wavefronts each (one workgroup of 8 or two of 4)
    const int slots = PIPE ? 256 : 256 * (8 / NW);
    n_splits = std::max(1, slots / std::max(1, row_tiles * Hkv));
    n_splits = std::min(n_splits, std::max(1, n_kv / (4 * TK)));
  }
  n_splits = std::min<int64_t>(n_splits, std::max<int64_t>(1, c->part_rows / n_q));
  n_splits = std::min(n_splits, 64);
  int keys_per_split = ((n_kv + n_splits - 1) / n_splits + TK - 1) / TK * TK;
  n_splits = (n_kv + keys_per_split - 1) / keys_per_split;
  const float c_log2 = 1.4426950408889634f / sqrtf((float)D);
  dim3 grid(row_tiles, Hkv, n_splits);
  if constexpr (PIPE)
    hipLaunchKernelGGL((k_attn_chunk_pipe<NW>), grid, dim3(NW * 64), kLds, s, (const __hip_bfloat16*)q,
                       (const __hip_bfloat16*)c->kv_ptr(stream, st.cur, layer, 0),
                       (const __hip_bfloat16*)c->kv_ptr(stream, st.cur, layer, 1), (__hip_bfloat16*)o, c->part_o,
                       c->part_ml, n_q, n_kv, causal ? 1 : 0, n_splits, keys_per_split, c->cfg.n_q_heads, G,
                       c->head_stride / 2, c_log2, env_int("SV_CHUNK_PHASE", 1));
  else
    hipLaunchKernelGGL((k_attn_chunk_mfma<NW>), grid, dim3(NW * 64), kLds, s, (const __hip_bfloat16*)q,
                       (const __hip_bfloat16*)c->kv_ptr(stream, st.cur, layer, 0),
                       (const __hip_bfloat16*)c->kv_ptr(stream, st.cur, layer, 1), (__hip_bfloat16*)o, c->part_o,
                       c->part_ml, n_q, n_kv, causal ? 1 : 0, n_splits, keys_per_split, c->cfg.n_q_heads, G,
                       c->head_stride / 2, c_log2);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_splits == 1) return e;
  return launch_attn_combine(c, n_q, n_splits, o, s);
}

}  // namespace

bool attn_mfma_supported(const sv_cache* c) {
  return c->cfg.dtype == SV_DTYPE_BF16 && c->cfg.head_dim == 128 && std::getenv("SV_NO_MFMA") == nullptr;
}

hipError_t launch_attn_chunk_mfma(const sv_cache* c, int stream, int layer, const void* q, int n_q, void* o,
                                  int causal, hipStream_t s) {
  // the pipelined kernel (tiles brought to LDS by direct loads) measured fastest on both chunk sizes; the
  // register-staged kernels stay selectable for comparison
  const int variant = env_int("SV_CHUNK_VARIANT", 2);
  if (variant == 0) return launch_t<8, false>(c, stream, layer, q, n_q, o, causal, s);
  if (variant == 2) return launch_t<8, true>(c, stream, layer, q, n_q, o, causal, s);
  return launch_t<4, false>(c, stream, layer, q, n_q, o, causal, s);
}

}  // namespace sv
