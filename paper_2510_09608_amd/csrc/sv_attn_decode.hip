// Text-decode attention for bf16 / head_dim 128 / up to 8 query heads per kv head
// (Sec. 2.1, Sec. 3.3: each generated token attends to the compact cache).
//
// Bound: K and V of every cached token are read once per layer and step
// (2 * n_kv_heads * 128 * 2 bytes per token); arithmetic is negligible, so the
// kernel is organised to keep many 16-byte loads in flight and to spend as few
// instructions per key as possible:
//   * both products run on the matrix cores (v_mfma_f32_16x16x32_bf16).  Scores are
//     computed transposed, S^T[keys][heads] = K Q^T: K rows go from HBM straight into
//     the A-operand layout, the query heads of the kv head (padded to 16) are the B
//     operand held in registers, and a lane then owns scores of ONE head, so the tile
//     max needs two exchanges between lane groups and nothing else crosses lanes;
//   * the rows of the score MFMAs are assigned to keys such that each lane ends up
//     with 8 consecutive keys, i.e. the probabilities already sit in the B-operand
//     layout of the second product O^T = V^T P^T;
//   * V is stored in the cache as V^T in blocks of 8 keys ([head dim][key], 2 KB per kv head): a
//     32-key tile of the second product's A operand is 8 KB contiguous, each lane loads its 8 keys
//     of one head dim (one block row) with a 16-byte load straight from HBM, and keys are contracted
//     inside the MFMA: about 3 instructions per key in total, no LDS on the way;
//   * in the fused form the query and the new token's K are rotated in registers at
//     the new token's position (cos/sin from a 64-entry table written when the token
//     was registered), and K/V of the new token are stored by the lanes that hold them
//     (V as one 2-byte element per head dim into its V^T block);
//   * all global loads of a tile are issued before anything else the wavefront does;
//   * wavefronts of a workgroup take alternate tiles of the workgroup's key range and
//     are merged through LDS; key ranges are merged by a second, tiny kernel whose
//     threads issue all their loads at once (an in-kernel merge by the last workgroup
//     to arrive was measured slower: the device-scope fences it needs cost more than
//     a launch).

#include <hip/hip_bf16.h>

#include <algorithm>

#include "sv_internal.h"

// Measurement build (-DSV_TIMELINE, libsv_timeline.so): the two decode kernels stamp the 100 MHz real-time counter at
// a few points into a buffer set with sv_timeline_set, so that one decode step can be laid out on a common clock
// (dispatch, first memory round trip, tile work, merge through LDS, stores, the gap to the merge kernel).  The
// product build compiles none of it.
#ifdef SV_TIMELINE
static __device__ unsigned long long* g_ts = nullptr;   // [8 launch slots][2 kernels][1024 workgroups][8]
#define SV_TS_PARAM , int ts_slot
#define SV_TS_ARG(x) , x
#define SV_TS(kind, wg, i)                                                                                     \
  do {                                                                                                         \
    if (g_ts != nullptr && threadIdx.x == 0 && (wg) < 1024)                                                    \
      g_ts[((((size_t)ts_slot * 2 + (kind)) * 1024 + (wg)) << 3) + (i)] = __builtin_amdgcn_s_memrealtime();     \
  } while (0)
#else
#define SV_TS_PARAM
#define SV_TS_ARG(x)
#define SV_TS(kind, wg, i) \
  do {                     \
  } while (0)
#endif

namespace sv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int D = 128;
constexpr int GMAX = 8;       // query heads per kv head this kernel handles
constexpr int TK = 32;        // keys per wavefront tile
constexpr int kMaxSplitsD = 128;
constexpr int kMaxRowsD = 64;

struct DecRow {
  __hip_bfloat16* k;         // K of the layer: kv head 0, slot 0 (written only at the slot of a fused new token)
  __hip_bfloat16* v;
  const float2* cs;          // cos/sin of the query token's rotary angles, [64]
  int32_t len;               // visible keys: slots [0, len), the query token is slot len - 1
  int32_t kps;               // keys per key range of this row (a multiple of 128); ranges = ceil(len / kps)
};
struct RangeCounts {
  uint8_t n[kMaxRowsD];      // key ranges of each row of a launch
};
struct DecTable {
  DecRow r[kMaxRowsD];
};

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t bf_round_bits(float x) {
  uint32_t a = __float_as_uint(x);
  a += 0x7fffu + ((a >> 16) & 1u);
  return a >> 16;
}

// Rotate, in place, the two 16-byte chunks a lane holds of one row: `lo` covers
// dims [i0, i0 + 8), `hi` the partner dims [i0 + 64, i0 + 72); c/s are cos/sin of
// the 8 pairs.  Result is rounded to bf16, as it would be stored.
// 16 bytes of K or V for launches that read far more than the caches hold (many long streams), every byte once:
// a non-temporal load keeps the stream from displacing itself through L2 and the Infinity Cache (measured
// 16 x 32k tokens: 5.7 -> 6.4 TB/s with merge).  A single stream's 11 MB per layer are partly still cached from
// the step before, and there the plain load is the faster one (10.3 vs 10.9 us per layer-step).
__device__ __forceinline__ uint4 stream_load(const __hip_bfloat16* p) {
  typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ void rotate_pair_chunks(uint4& lo, uint4& hi, const float (&c)[8], const float (&s)[8]) {
  uint32_t* a = (uint32_t*)&lo;
  uint32_t* b = (uint32_t*)&hi;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float a0 = bf_lo(a[w]), a1 = bf_hi(a[w]), b0 = bf_lo(b[w]), b1 = bf_hi(b[w]);
    const float ra0 = a0 * c[2 * w] - b0 * s[2 * w], rb0 = b0 * c[2 * w] + a0 * s[2 * w];
    const float ra1 = a1 * c[2 * w + 1] - b1 * s[2 * w + 1], rb1 = b1 * c[2 * w + 1] + a1 * s[2 * w + 1];
    a[w] = bf_round_bits(ra0) | (bf_round_bits(ra1) << 16);
    b[w] = bf_round_bits(rb0) | (bf_round_bits(rb1) << 16);
  }
}


// ONE: a single row (one stream).  Its cache pointers, length and everything else needed to issue the first
// loads are the leading 16 dwords of the argument list, which reach the wavefront in SGPRs at launch (kernel
// argument preload) instead of through a first dependent fetch; the by-value table, at the end, is not read.
template <int NW, bool ONE, bool STREAM>
__global__ __launch_bounds__(NW * 64, 2) void k_decode_mfma(__hip_bfloat16* k0_, __hip_bfloat16* v0_, const float2* cs0_,
                                                         int len0_, int keys_per_split,
                                                         const __hip_bfloat16* __restrict__ q,
                                                         const __hip_bfloat16* __restrict__ k_new,
                                                         const __hip_bfloat16* __restrict__ v_new,
                                                         size_t head_stride_elems, int fused, int rotate,
                                                         __hip_bfloat16* __restrict__ out, float* __restrict__ part_o,
                                                         float* __restrict__ part_ml, int n_splits, int n_q_heads,
                                                         int n_kv_heads, int G, float c_log2, DecTable tab SV_TS_PARAM) {
  [[maybe_unused]] const int ts_wg = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
  SV_TS(0, ts_wg, 0);
  __shared__ float sO[NW][GMAX][D];                                 // wavefront results (merge)
  __shared__ float sML[NW][GMAX][2];

  const int sp = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  DecRow rd;
  if constexpr (ONE) rd = DecRow{k0_, v0_, cs0_, len0_};
  else rd = tab.r[b];
  const int len = rd.len;
  const int kps = ONE ? keys_per_split : rd.kps;   // rows of a batch are cut into ranges of their own size
  const int k0 = sp * kps, k1 = min(len, k0 + kps);
  if (k0 >= len) return;   // a shorter row of the batch has fewer ranges than the grid is wide
  const __hip_bfloat16* kp = rd.k + (size_t)hk * head_stride_elems;
  const __hip_bfloat16* vp = rd.v + (size_t)hk * head_stride_elems;
  const bool rot = fused && rotate;
  const size_t new_off = ((size_t)b * n_kv_heads + hk) * D;

  // Row m = l16 of score MFMA gi carries key 8 (m >> 2) + 4 gi + (m & 3) of the tile, so that the
  // accumulator of lane group lg holds keys 8 lg + 4 gi + r: eight consecutive keys per lane over the two
  // MFMAs, which is the B-operand layout of the second product.
  const int krow[2] = {8 * (l16 >> 2) + (l16 & 3), 8 * (l16 >> 2) + 4 + (l16 & 3)};

  uint4 kreg[2][4];
  uint4 vreg[8];
  // K: 8 loads per lane straight into the A-operand layout (dims 8 lg + 32 kk + j of key krow[gi]); the token
  // being decoded comes from the caller's buffer.
  // V^T: 8 loads per lane, again straight into the A-operand layout of the second product: head dim
  // 16 blk + l16, keys kt + 8 lg .. + 7 = one row of a V^T block.  Whole blocks are read whatever the range's
  // end: planes hold whole tiles, keys past the range get probability zero, and stale values are finite.
  auto issue_k = [&](int kt) {
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
      const int key = kt + krow[gi];
      const bool is_new = fused && key == len - 1;
      const __hip_bfloat16* src = is_new ? k_new + new_off + 8 * lg : kp + (size_t)key * D + 8 * lg;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        if constexpr (STREAM) kreg[gi][kk] = key < k1 ? stream_load(src + 32 * kk) : make_uint4(0, 0, 0, 0);
        else kreg[gi][kk] = key < k1 ? *(const uint4*)(src + 32 * kk) : make_uint4(0, 0, 0, 0);
    }
  };
  auto issue_v = [&](int kt) {
    const __hip_bfloat16* vb = vp + vt_elem(kt + 8 * lg, l16);   // block of the lane group's 8 keys, row l16
#pragma unroll
    for (int blk = 0; blk < 8; ++blk) {
      if constexpr (STREAM) vreg[blk] = stream_load(vb + blk * 16 * kVB);
      else vreg[blk] = *(const uint4*)(vb + blk * 16 * kVB);
    }
  };

  const int n_tiles = k1 > k0 ? (k1 - k0 + TK - 1) / TK : 0;
  if (wave < n_tiles) {   // memory first: everything below overlaps its latency
    issue_k(k0 + wave * TK);
    issue_v(k0 + wave * TK);
  }
  // the wavefront whose tile holds the token being decoded fetches that token's V (one element per head dim for
  // the lanes that will own it) along with its first loads
  unsigned short vnew_bits[8] = {};
  const bool owns_new = fused && len - 1 >= k0 && len - 1 < k1 && ((len - 1 - k0) / TK) % NW == wave;
  if (owns_new) {
#pragma unroll
    for (int blk = 0; blk < 8; ++blk) vnew_bits[blk] = *(const unsigned short*)(v_new + new_off + 16 * blk + l16);
  }

  // cos/sin of the 16 rotary pairs a lane touches (dims 8 lg + 32 kk + j, kk = 0, 1), from the table the
  // token's registration wrote
  float rc[2][8], rs[2][8];
  if (rot) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const float4 t4 = *(const float4*)(rd.cs + 8 * lg + 32 * kk + j);
        rc[kk][j] = t4.x, rs[kk][j] = t4.y, rc[kk][j + 1] = t4.z, rs[kk][j + 1] = t4.w;
      }
  }

  // query heads of this kv head as the B operand: lane holds head l16, dims 8 lg + 32 kk + j
  uint4 qraw[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    qraw[kk] = l16 < G ? *(const uint4*)(q + ((size_t)b * n_q_heads + hk * G + l16) * D + 8 * lg + 32 * kk)
                       : make_uint4(0, 0, 0, 0);
  if (rot) {
    rotate_pair_chunks(qraw[0], qraw[2], rc[0], rs[0]);
    rotate_pair_chunks(qraw[1], qraw[3], rc[1], rs[1]);
  }
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) qf[kk] = *(bf16x8*)&qraw[kk];

  // lane (head l16, lane group lg): running max of the head, its share of the sum, and
  // O^T[dims 16 blk + 4 lg + r][head l16]
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[8];
#pragma unroll
  for (int blk = 0; blk < 8; ++blk) oacc[blk] = (f32x4){0.f, 0.f, 0.f, 0.f};

#ifdef SV_TIMELINE
  __builtin_amdgcn_s_waitcnt(0x0F70);   // (measurement build only) the first tile's loads have landed
  SV_TS(0, ts_wg, 1);
#endif
  for (int t = wave; t < n_tiles; t += NW) {
    const int kt = k0 + t * TK;
    if (fused && len - 1 >= kt && len - 1 < kt + TK) {
      // this tile holds the token being decoded: rotate its K, store K and V to the cache
      const int rel = len - 1 - kt;
#pragma unroll
      for (int gi = 0; gi < 2; ++gi)
        if (rel == krow[gi]) {
          if (rot) {
            rotate_pair_chunks(kreg[gi][0], kreg[gi][2], rc[0], rs[0]);
            rotate_pair_chunks(kreg[gi][1], kreg[gi][3], rc[1], rs[1]);
          }
          __hip_bfloat16* dst = rd.k + (size_t)hk * head_stride_elems + (size_t)(len - 1) * D + 8 * lg;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) *(uint4*)(dst + 32 * kk) = kreg[gi][kk];
        }
      // V: the lanes of lane group rel / 8 hold the new token as element rel % 8 of each of their 8 head dims:
      // patch the registers (the cache does not hold the token yet) and store the elements into the block
      if ((rel >> 3) == lg) {
        const int wsel = (rel & 7) >> 1, hi = rel & 1;
        unsigned short* vdst = (unsigned short*)rd.v + (size_t)hk * head_stride_elems + vt_elem(len - 1, l16);
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
          const uint32_t x = vnew_bits[blk];
          uint32_t* w = (uint32_t*)&vreg[blk];
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (i == wsel) w[i] = hi ? (w[i] & 0x0000ffffu) | (x << 16) : (w[i] & 0xffff0000u) | x;
          vdst[blk * 16 * kVB] = vnew_bits[blk];
        }
      }
    }
    // ---- scores S^T = K Q^T: register r of MFMA gi is key kt + 8 lg + 4 gi + r, head l16
    f32x4 sacc[2];
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
      sacc[gi] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        sacc[gi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8*)&kreg[gi][kk], qf[kk], sacc[gi], 0, 0, 0);
    }
    // the K registers of this tile are consumed: fetch the wavefront's next K tile behind the softmax and the
    // second product (the next V^T block follows once that product has read this one)
    if (t + NW < n_tiles) issue_k(kt + NW * TK);
    float mx = -INFINITY;
#pragma unroll
    for (int gi = 0; gi < 2; ++gi)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (kt + 8 * lg + 4 * gi + r >= k1) sacc[gi][r] = -INFINITY;
        mx = fmaxf(mx, sacc[gi][r]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));   // every tile holds at least one valid key, so mx is finite
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
    const float mc = m_new * c_log2;
    float psum = 0.f;
    bf16x8 pf;
#pragma unroll
    for (int gi = 0; gi < 2; ++gi)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[gi][r], c_log2, -mc));
        psum += p;
        pf[4 * gi + r] = (__bf16)p;
      }
    l_run = l_run * alpha + psum;
    if (m_new > m_run) {
#pragma unroll
      for (int blk = 0; blk < 8; ++blk) oacc[blk] *= alpha;
    }
    m_run = m_new;
    // ---- O^T += V^T P^T: A operand = V^T[dims 16 blk + l16][keys 8 lg + j], as loaded
#pragma unroll
    for (int blk = 0; blk < 8; ++blk)
      oacc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)&vreg[blk], pf, oacc[blk], 0, 0, 0);
    if (t + NW < n_tiles) issue_v(kt + NW * TK);
  }

  SV_TS(0, ts_wg, 2);
  // ---- wavefront result to LDS: head l16 < G, dims 16 blk + 4 lg + r; the sum of a head is spread over
  // the four lane groups
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (l16 < GMAX) {
#pragma unroll
    for (int blk = 0; blk < 8; ++blk)
      *(float4*)&sO[wave][l16][16 * blk + 4 * lg] = make_float4(oacc[blk][0], oacc[blk][1], oacc[blk][2], oacc[blk][3]);
    if (lg == 0) {
      sML[wave][l16][0] = m_run == -INFINITY ? -INFINITY : m_run * c_log2;   // log2 units from here on
      sML[wave][l16][1] = l_run;
    }
  }
  __syncthreads();

  // ---- merge the wavefronts; with one split this is the result, else a partial for the merge kernel
  const size_t pbase = ((size_t)b * n_splits + sp) * n_q_heads + (size_t)hk * G;
  for (int idx = tid; idx < G * D; idx += NW * 64) {
    const int g = idx / D, d = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mn = fmaxf(mn, sML[w][g][0]);
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float mw = sML[w][g][0];
      const float a = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - mn);
      acc += sO[w][g][d] * a;
      lsum += sML[w][g][1] * a;
    }
    if (n_splits == 1) {
      out[((size_t)b * n_q_heads + hk * G + g) * D + d] = __float2bfloat16(acc / lsum);
    } else {
      part_o[(pbase + g) * D + d] = acc;
      if (d == 0) {
        part_ml[(pbase + g) * 2] = mn;
        part_ml[(pbase + g) * 2 + 1] = lsum;
      }
    }
  }
#ifdef SV_TIMELINE
  __builtin_amdgcn_s_waitcnt(0x0F70);   // (measurement build only) the stores have been acknowledged
  SV_TS(0, ts_wg, 3);
#endif
}

// ---------------------------------------------------------------------------------
// Merge of the key ranges of one decode step.  One workgroup of 128 threads per (head, row): thread
// (g, d4) = (tid / 32, tid % 32) takes the key ranges s = g, g + 4, g + 8, ... and 4 output dims, issues
// ALL its loads (up to 16 (max, sum) pairs and 16 float4) before using any of them, so the kernel costs
// one memory round trip for up to 64 key ranges; the four partial merges meet in LDS.
// grid: (n_q_heads, n_rows), block: 128 threads.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void k_decode_merge(const float* __restrict__ part_o,
                                                      const float* __restrict__ part_ml,
                                                      __hip_bfloat16* __restrict__ out, int n_splits, int n_q_heads,
                                                      RangeCounts cnt SV_TS_PARAM) {
  [[maybe_unused]] const int ts_wg = blockIdx.y * gridDim.x + blockIdx.x;
  SV_TS(1, ts_wg, 0);
  __shared__ float4 s_acc[4][32];
  __shared__ float2 s_ml[4];
  const int h = blockIdx.x, b = blockIdx.y, g = threadIdx.x >> 5, d4 = threadIdx.x & 31;
  const size_t rbase = (size_t)b * n_splits * n_q_heads + h;   // split s adds s * n_q_heads
  const int ns = cnt.n[b];                                      // ranges this row really has (<= n_splits)
  const float4* po = (const float4*)(part_o + rbase * D) + d4;
  const float2* pml = (const float2*)part_ml + rbase;
  const size_t ostride = (size_t)n_q_heads * D / 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float lsum = 0.f, m_ref = -INFINITY;
  for (int s0 = g; s0 < ns; s0 += 64) {
    float4 v[16];
    float2 ml[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int sidx = s0 + 4 * j;
      const bool ok = sidx < ns;
      ml[j] = ok ? pml[(size_t)sidx * n_q_heads] : make_float2(-INFINITY, 0.f);
      v[j] = ok ? po[(size_t)sidx * ostride] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float mx = m_ref;
#pragma unroll
    for (int j = 0; j < 16; ++j) mx = fmaxf(mx, ml[j].x);
    const float resc = m_ref == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_ref - mx);
    acc.x *= resc, acc.y *= resc, acc.z *= resc, acc.w *= resc;
    lsum *= resc;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float w = ml[j].x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml[j].x - mx);
      acc.x += w * v[j].x, acc.y += w * v[j].y, acc.z += w * v[j].z, acc.w += w * v[j].w;
      lsum += w * ml[j].y;
    }
    m_ref = mx;
  }
  s_acc[g][d4] = acc;
  if (d4 == 0) s_ml[g] = make_float2(m_ref, lsum);
  __syncthreads();
  if (g != 0) return;
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < 4; ++k) mx = fmaxf(mx, s_ml[k].x);
  float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
  float ltot = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float2 mlk = s_ml[k];
    const float w = mlk.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mlk.x - mx);
    const float4 a = s_acc[k][d4];
    tot.x += w * a.x, tot.y += w * a.y, tot.z += w * a.z, tot.w += w * a.w;
    ltot += w * mlk.y;
  }
  const float inv = 1.0f / ltot;
  __hip_bfloat16* op = out + ((size_t)b * n_q_heads + h) * D + 4 * d4;
  const uint32_t w0 = bf_round_bits(tot.x * inv) | (bf_round_bits(tot.y * inv) << 16);
  const uint32_t w1 = bf_round_bits(tot.z * inv) | (bf_round_bits(tot.w * inv) << 16);
  *(uint2*)op = make_uint2(w0, w1);
#ifdef SV_TIMELINE
  __builtin_amdgcn_s_waitcnt(0x0F70);
  SV_TS(1, ts_wg, 1);
#endif
}

#ifdef SV_TIMELINE
int g_ts_launch = 0;   // host: launches so far; the slot of a launch is this modulo 8
#endif

}  // namespace

template <int NW>
static hipError_t decode_launch(const sv_cache* c, const DecTable& tab, int fused, int nr, int max_len, int64_t total_tiles,
                         const void* q, const void* k_new, const void* v_new, void* o, size_t r0, float* part_o,
                         float* part_ml, int64_t part_rows, hipStream_t s) {
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads;
  // Key ranges.  A single stream is latency bound: ranges of 128 keys (one 32-key tile per wavefront) spread its
  // few hundred tiles over the most CUs and cost one memory round trip.  A batch is bandwidth bound: longer ranges
  // keep the partial results and their merge small, and all workgroups should be resident at once (two fit a CU:
  // 512), since one workgroup more than that and a second, nearly empty round follows the first (measured on 16
  // ragged rows: 516 workgroups 3.6 TB/s, 440 workgroups 4.2 TB/s).  So: the smallest target T, a multiple of 128
  // keys (whole tiles for each of the 4 wavefronts: ranges of 800 keys, 7 tiles for one wavefront and 6 for the
  // others, measured 6 % slower than ranges of 896), for which sum_b ceil(len_b / T) * kv heads <= 512; then every
  // row is cut into ceil(len_b / T) ranges of EQUAL size (rounded up to 128 keys), so that a row does not end in a
  // range much shorter than the others.
  constexpr int kSlots = 512;
  const int forced = std::min(c->opt[SV_OPT_DECODE_TILES_PER_WAVE], 64);
  const int64_t max_pairs = std::max<int64_t>(nr, part_rows);
  int T = forced > 0 ? TK * NW * forced : TK * NW;
  for (;; T += TK * NW) {
    int64_t pairs = 0;
    int widest = 0;
    for (int b = 0; b < nr; ++b) {
      const int nb = (tab.r[b].len + T - 1) / T;
      pairs += nb;
      widest = std::max(widest, nb);
    }
    const bool fits = widest <= kMaxSplitsD && widest * (int64_t)nr <= max_pairs;   // scratch: rows x widest ranges
    if (fits && (forced > 0 || pairs * Hkv <= kSlots || T >= max_len)) break;
  }
  DecTable tabk = tab;
  RangeCounts cnt = {};
  int n_splits = 1;
  for (int b = 0; b < nr; ++b) {
    const int len = tab.r[b].len, nb = std::max(1, (len + T - 1) / T);
    const int kps = ((len + nb - 1) / nb + TK * NW - 1) / (TK * NW) * (TK * NW);
    tabk.r[b].kps = kps;
    cnt.n[b] = (uint8_t)((len + kps - 1) / kps);
    n_splits = std::max(n_splits, (int)cnt.n[b]);
  }
  const int keys_per_split = tabk.r[0].kps;
  const float c_log2 = 1.4426950408889634f / sqrtf((float)D);
  const __hip_bfloat16* qp = (const __hip_bfloat16*)q + r0 * Hq * D;
  const __hip_bfloat16* knp = k_new ? (const __hip_bfloat16*)k_new + r0 * Hkv * D : nullptr;
  const __hip_bfloat16* vnp = v_new ? (const __hip_bfloat16*)v_new + r0 * Hkv * D : nullptr;
  __hip_bfloat16* op = (__hip_bfloat16*)o + r0 * Hq * D;
  const int rotate = c->cfg.rope_mode != SV_ROPE_NONE ? 1 : 0;
  const DecRow& r = tabk.r[0];
  // More than 96 MB of K and V in this launch, one long stream or many: non-temporal loads (rows that are the layers
  // of ONE stream keep the plain loads: their 308 MB are read again at the next token and the Infinity Cache still
  // holds most of them).
  const bool stream_loads = total_tiles * (int64_t)(TK * D * 2 * 2) * Hkv >= ((int64_t)96 << 20);
  if (nr == 1 && !stream_loads)
    hipLaunchKernelGGL((k_decode_mfma<NW, true, false>), dim3(n_splits, Hkv, 1), dim3(NW * 64), 0, s, r.k, r.v, r.cs, r.len,
                       keys_per_split, qp, knp, vnp, c->head_stride / 2, fused, rotate, op, part_o, part_ml,
                       n_splits, Hq, Hkv, c->group, c_log2, tabk SV_TS_ARG(g_ts_launch % 8));
  else if (stream_loads)
    hipLaunchKernelGGL((k_decode_mfma<NW, false, true>), dim3(n_splits, Hkv, nr), dim3(NW * 64), 0, s, r.k, r.v, r.cs, r.len,
                       keys_per_split, qp, knp, vnp, c->head_stride / 2, fused, rotate, op, part_o, part_ml,
                       n_splits, Hq, Hkv, c->group, c_log2, tabk SV_TS_ARG(g_ts_launch % 8));
  else
    hipLaunchKernelGGL((k_decode_mfma<NW, false, false>), dim3(n_splits, Hkv, nr), dim3(NW * 64), 0, s, r.k, r.v, r.cs, r.len,
                       keys_per_split, qp, knp, vnp, c->head_stride / 2, fused, rotate, op, part_o, part_ml,
                       n_splits, Hq, Hkv, c->group, c_log2, tabk SV_TS_ARG(g_ts_launch % 8));
  hipError_t e = hipGetLastError();
#ifdef SV_TIMELINE
  if (e != hipSuccess || n_splits == 1) ++g_ts_launch;
#endif
  if (e != hipSuccess || n_splits == 1) return e;
  hipLaunchKernelGGL(k_decode_merge, dim3(Hq, nr), dim3(128), 0, s, part_o, part_ml,
                     (__hip_bfloat16*)o + r0 * Hq * D, n_splits, Hq, cnt SV_TS_ARG(g_ts_launch % 8));
#ifdef SV_TIMELINE
  ++g_ts_launch;
#endif
  return hipGetLastError();
}

// Partial results of the key ranges live in the cache arena by default; sv_attn_decode_static keeps them in a
// file-scope device array instead (callers that cannot provide scratch memory).  The array's name is only a host-side
// handle: its device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kMaxDevices] = {};

hipError_t decode_static_scratch(void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr_out = g_scratch_ptr[dev];
  return hipSuccess;
}

int64_t decode_static_pairs(const sv_cache* c) {
  // one (row, key range) pair holds n_q_heads x (128 + 2) floats
  return (int64_t)(kStaticScratchBytes / ((size_t)c->cfg.n_q_heads * (D + 2) * sizeof(float)));
}

static hipError_t decode_rows(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused, const void* q,
                              const void* k_new, const void* v_new, void* o, float* part_o, float* part_ml,
                              int64_t part_rows, hipStream_t s) {
  for (int r0 = 0; r0 < n_list; r0 += kMaxRowsD) {
    const int nr = std::min(kMaxRowsD, n_list - r0);
    DecTable tab = {};
    int max_len = 1;
    int64_t total_tiles = 0;   // of the rows that are different streams: what decides the non-temporal loads
    for (int b = 0; b < nr; ++b) {
      // layer >= 0: row b is stream streams[b] at that layer; layer < 0: row b is layer b of stream streams[0]
      const int sid = layer >= 0 ? streams[r0 + b] : streams[0];
      const int lay = layer >= 0 ? layer : r0 + b;
      const StreamState& st = c->st[sid];
      tab.r[b].k = (__hip_bfloat16*)c->kv_ptr(sid, st.cur, lay, 0);
      tab.r[b].v = (__hip_bfloat16*)c->kv_ptr(sid, st.cur, lay, 1);
      tab.r[b].len = (int)st.len;
      tab.r[b].cs = c->last_cs + (size_t)sid * (D / 2);
      max_len = std::max(max_len, (int)st.len);
      if (layer >= 0) total_tiles += (st.len + TK - 1) / TK;
    }
    hipError_t e = decode_launch<4>(c, tab, fused, nr, max_len, total_tiles, q, k_new, v_new, o, (size_t)r0, part_o,
                                    part_ml, part_rows, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_attn_decode_mfma(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused,
                                   const void* q, const void* k_new, const void* v_new, void* o, hipStream_t s) {
  return decode_rows(c, layer, streams, n_list, fused, q, k_new, v_new, o, c->part_o, c->part_ml, c->part_rows, s);
}

hipError_t launch_attn_decode_mfma_static(const sv_cache* c, int layer, const int32_t* streams, int n_list,
                                          const void* q, void* o, hipStream_t s) {
  void* p = nullptr;
  hipError_t e = decode_static_scratch(&p);
  if (e != hipSuccess) return e;
  const int64_t pairs = decode_static_pairs(c);
  float* part_o = (float*)p;
  float* part_ml = part_o + (size_t)pairs * c->cfg.n_q_heads * D;
  return decode_rows(c, layer, streams, n_list, 0, q, nullptr, nullptr, o, part_o, part_ml, pairs, s);
}

}  // namespace sv

#ifdef SV_TIMELINE
// Measurement build only: where the decode kernels stamp their timeline (device memory of at least
// SV_TIMELINE_BYTES bytes, zeroed by the caller; NULL switches stamping off), and how many decode launches have
// been enqueued so far (the slot a launch stamps into is its index modulo 8).
extern "C" __attribute__((visibility("default"))) int sv_timeline_set(void* dev_buf, int* launches_out) {
  if (launches_out) *launches_out = sv::g_ts_launch;
  unsigned long long* p = (unsigned long long*)dev_buf;
  return hipMemcpyToSymbol(HIP_SYMBOL(g_ts), &p, sizeof(p)) == hipSuccess ? SV_OK : SV_ERR_HIP;
}
#endif
