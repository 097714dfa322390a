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
//   * A wavefront owns RB blocks of 32 rows; a workgroup of NW wavefronts owns
//     NW * RB * 32 rows of one kv head and one key range (split-KV); key ranges
//     are merged afterwards with the log-sum-exp rule.
//   * Scores are computed transposed, S^T = K Q^T, so that a lane holds scores
//     of ONE query row: row max and row sum are in-lane plus one exchange
//     between the two half-wavefronts, and the output O^T = V^T P^T keeps one
//     query row per lane, so rescaling by the running max is a per-lane scalar.
//   * K tiles (64 keys) are staged in LDS row-wise with their rows permuted
//     (bits 2 and 3 of the key index swapped): the accumulator layout of S^T
//     then hands every lane 8 consecutive keys per 16-key step, which is exactly
//     the B-operand layout of the second product, so P never moves between lanes.
//   * V tiles are transposed on the way into LDS (4 keys x 8 dims per thread in
//     registers), so the A operand of V^T P^T is one 16-byte LDS read.
//   * Both LDS tiles use a 16-byte-chunk XOR swizzle: every 8 consecutive lanes
//     of a 16-byte read or an 8-byte write fall in distinct bank groups.
//   * The next tile's global loads are issued into registers before the current
//     tile's MFMAs.

#include <hip/hip_bf16.h>

#include <algorithm>
#include <cstdlib>

#include "sv_internal.h"

namespace sv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int D = 128;          // head_dim
constexpr int TK = 64;          // keys per tile
constexpr int KROW = D * 2;     // bytes per K row in LDS
constexpr int VROW = TK * 2;    // bytes per V^T row in LDS
constexpr int K_BYTES = TK * KROW;
constexpr int V_BYTES = D * VROW;

__device__ __forceinline__ int perm_key(int key) {  // swap bits 2 and 3
  return (key & ~0xC) | ((key & 4) << 1) | ((key & 8) >> 1);
}
__device__ __forceinline__ int k_lds_off(int row, int chunk) {  // row: permuted key, chunk: 16-byte unit of head_dim
  return row * KROW + ((chunk ^ (row & 7)) << 4);
}
__device__ __forceinline__ int v_swz(int dv) { return (dv & 7) ^ ((dv >> 3) & 7); }
__device__ __forceinline__ int vt_lds_off(int dv, int chunk) {  // chunk: 8 keys
  return dv * VROW + ((chunk ^ v_swz(dv)) << 4);
}

template <int NW, int RB>
__global__ __launch_bounds__(NW * 64) void k_attn_chunk_mfma(
    const __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ kc, const __hip_bfloat16* __restrict__ vc,
    __hip_bfloat16* __restrict__ out, float* __restrict__ part_o, float* __restrict__ part_ml, int n_q, int n_kv,
    int causal, int n_splits, int keys_per_split, int n_q_heads, int G, size_t head_stride_elems, float c_log2) {
  constexpr int NT = NW * 64;
  constexpr int ROWS_WG = NW * RB * 32;
  constexpr int KLD = (TK * 16) / NT;  // 16-byte K chunks per thread per tile
  constexpr int VUN = 256 / NT;        // (4 keys x 8 dims) V units per thread per tile
  __shared__ __attribute__((aligned(16))) char smem[K_BYTES + V_BYTES];
  char* sK = smem;
  char* sV = smem + K_BYTES;

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

  // per-lane query rows
  int qi[RB], hg[RB], limit[RB];
  bool rvalid[RB];
  bf16x8 qf[RB][8];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = rt * ROWS_WG + (wave * RB + rb) * 32 + l32;
    rvalid[rb] = row < n_rows;
    const int rr = rvalid[rb] ? row : n_rows - 1;
    qi[rb] = rr / G;
    hg[rb] = rr % G;
    limit[rb] = min(causal ? slot0 + qi[rb] : n_kv - 1, k_end - 1);
    const __hip_bfloat16* qp = q + ((size_t)qi[rb] * n_q_heads + hk * G + hg[rb]) * D + hh * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      uint4 raw = rvalid[rb] ? *(const uint4*)(qp + kk * 16) : make_uint4(0, 0, 0, 0);
      qf[rb][kk] = *(bf16x8*)&raw;
    }
  }

  f32x16 oacc[RB][4];
  float m_run[RB], l_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = -INFINITY;
    l_run[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[rb][db][r] = 0.f;
  }

  const __hip_bfloat16* kbase = kc + (size_t)hk * head_stride_elems;
  const __hip_bfloat16* vbase = vc + (size_t)hk * head_stride_elems;

  uint4 kreg[KLD];
  uint4 vreg[VUN][4];
  auto issue_loads = [&](int t) {
    const int kt0 = k_begin + t * TK;
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int cid = tid + i * NT, key = cid >> 4, c16 = cid & 15;
      kreg[i] = (kt0 + key < k_end) ? *(const uint4*)(kbase + (size_t)(kt0 + key) * D + c16 * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < VUN; ++u) {
      const int unit = tid + u * NT, dg = unit & 15, kg = unit >> 4;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int key = kt0 + 4 * kg + a;
        vreg[u][a] = key < k_end ? *(const uint4*)(vbase + (size_t)key * D + dg * 8) : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int cid = tid + i * NT, key = cid >> 4, c16 = cid & 15;
      *(uint4*)(sK + k_lds_off(perm_key(key), c16)) = kreg[i];
    }
#pragma unroll
    for (int u = 0; u < VUN; ++u) {
      const int unit = tid + u * NT, dg = unit & 15, kg = unit >> 4;
      const uint32_t* r0 = (const uint32_t*)&vreg[u][0];
      const uint32_t* r1 = (const uint32_t*)&vreg[u][1];
      const uint32_t* r2 = (const uint32_t*)&vreg[u][2];
      const uint32_t* r3 = (const uint32_t*)&vreg[u][3];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int w = e >> 1;
        uint2 t2;
        if (e & 1) {
          t2.x = (r0[w] >> 16) | (r1[w] & 0xffff0000u);
          t2.y = (r2[w] >> 16) | (r3[w] & 0xffff0000u);
        } else {
          t2.x = (r0[w] & 0xffffu) | (r1[w] << 16);
          t2.y = (r2[w] & 0xffffu) | (r3[w] << 16);
        }
        const int dv = dg * 8 + e;
        *(uint2*)(sV + vt_lds_off(dv, kg >> 1) + ((kg & 1) << 3)) = t2;
      }
    }
  };

  if (n_tiles > 0) issue_loads(0);
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();  // everyone is done reading the previous tile
    store_tile();
    __syncthreads();
    if (t + 1 < n_tiles) issue_loads(t + 1);
    const int kt0 = k_begin + t * TK;

    // S^T = K Q^T for 2 blocks of 32 keys x RB blocks of 32 rows
    f32x16 sacc[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[rb][kb][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 a = *(const bf16x8*)(sK + k_lds_off(kb * 32 + l32, 2 * kk + hh));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          sacc[rb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][kk], sacc[rb][kb], 0, 0, 0);
      }
    }

    // online softmax, one query row per lane.  Register r of key block kb holds key
    // kt0 + 32 kb + 16 (r / 8) + 8 hh + r % 8.
    const bool need_mask = kt0 + TK - 1 > (causal ? slot0 + (rt * ROWS_WG) / G : n_kv - 1) || kt0 + TK > k_end;
    bf16x8 pf[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kt0 + 32 * kb + 16 * (r >> 3) + 8 * hh + (r & 7);
            if (key > limit[rb]) sacc[rb][kb][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[rb][kb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[rb], mx);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = exp2f((m_run[rb] - m_use) * c_log2);
      const float mc = m_use * c_log2;
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = exp2f(fmaf(sacc[rb][kb][r], c_log2, -mc));
          psum += p;
          pf[rb][kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
        }
      l_run[rb] = l_run[rb] * alpha + psum;
      if (__any(m_new > m_run[rb])) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[rb][db][r] *= alpha;
      }
      m_run[rb] = m_new;
    }

    // O^T += V^T P^T : 4 blocks of 32 dims, 4 steps of 16 keys
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x8 a = *(const bf16x8*)(sV + vt_lds_off(db * 32 + l32, 2 * ks + hh));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          oacc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[rb][ks], oacc[rb][db], 0, 0, 0);
      }
    }
  }

  // epilogue: lane holds row l32 of each block, dims 32 db + 8 (r / 4) + 4 hh + r % 4
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
    if (!rvalid[rb]) continue;
    const int h = hk * G + hg[rb];
    if (n_splits == 1) {
      const float inv = 1.0f / l_tot;
      __hip_bfloat16* op = out + ((size_t)qi[rb] * n_q_heads + h) * D;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int dv = 32 * db + 8 * r4 + 4 * hh;
          __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(oacc[rb][db][r4 * 4 + e] * inv);
          *(uint2*)(op + dv) = *(uint2*)&pk;
        }
    } else {
      const size_t p = ((size_t)qi[rb] * n_splits + sp) * n_q_heads + h;
      float* po = part_o + p * D;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int dv = 32 * db + 8 * r4 + 4 * hh;
          *(float4*)(po + dv) = make_float4(oacc[rb][db][r4 * 4], oacc[rb][db][r4 * 4 + 1], oacc[rb][db][r4 * 4 + 2],
                                            oacc[rb][db][r4 * 4 + 3]);
        }
      if (hh == 0) {
        part_ml[p * 2] = m_run[rb] == -INFINITY ? -INFINITY : m_run[rb] * c_log2;
        part_ml[p * 2 + 1] = l_tot;
      }
    }
  }
}

int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  return v && *v ? std::atoi(v) : dflt;
}

template <int NW, int RB>
hipError_t launch_t(const sv_cache* c, int stream, int layer, const void* q, int n_q, void* o, int causal,
                    hipStream_t s) {
  constexpr int ROWS_WG = NW * RB * 32;
  const StreamState& st = c->st[stream];
  const int n_kv = (int)st.len, G = c->group, Hkv = c->cfg.n_kv_heads;
  const int row_tiles = (n_q * G + ROWS_WG - 1) / ROWS_WG;
  int n_splits = env_int("SV_CHUNK_SPLITS", 0);
  if (n_splits <= 0) {
    const int n_cu = 256;
    n_splits = std::max(1, n_cu / std::max(1, row_tiles * Hkv));
    n_splits = std::min(n_splits, std::max(1, n_kv / (4 * TK)));
  }
  n_splits = std::min<int64_t>(n_splits, std::max<int64_t>(1, c->part_rows / n_q));
  n_splits = std::min(n_splits, 64);
  int keys_per_split = ((n_kv + n_splits - 1) / n_splits + TK - 1) / TK * TK;
  n_splits = (n_kv + keys_per_split - 1) / keys_per_split;
  const float c_log2 = 1.4426950408889634f / sqrtf((float)D);
  dim3 grid(row_tiles, Hkv, n_splits);
  hipLaunchKernelGGL((k_attn_chunk_mfma<NW, RB>), grid, dim3(NW * 64), 0, s, (const __hip_bfloat16*)q,
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
  const int variant = env_int("SV_CHUNK_VARIANT", 0);
  switch (variant) {
    case 1: return launch_t<2, 2>(c, stream, layer, q, n_q, o, causal, s);
    case 3: return launch_t<4, 2>(c, stream, layer, q, n_q, o, causal, s);
    default: return launch_t<4, 1>(c, stream, layer, q, n_q, o, causal, s);
  }
}

}  // namespace sv
