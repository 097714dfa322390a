// Bandwidth-bound row movers: storing new K/V (K rotated at its assigned
// position), rotating fresh Q/K in place, and the compaction gather that moves
// every surviving K/V row of every layer to its new slot while re-rotating K by
// the position shift (Sec. 2.1: states are reused, positions stay contiguous).
//
// All three share one thread layout.  A row of head_dim elements is split into
// a low and a high half; the rotary pairing is (i, i + head_dim/2), so a thread
// that owns 16 bytes of the low half and the matching 16 bytes of the high half
// holds complete pairs.  Rows are 128-512 bytes, a wavefront therefore covers
// 4-16 whole rows with two fully coalesced 16-byte accesses per lane.

#include <hip/hip_bf16.h>

#include "sv_internal.h"

namespace sv {
namespace {

template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ float get(int e) const { return ((const float*)&raw)[e]; }
  __device__ void set(int e, float x) { ((float*)&raw)[e] = x; }
};
template <>
struct Vec16<__hip_bfloat16> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ float get(int e) const {
    const uint32_t w = ((const uint32_t*)&raw)[e >> 1];
    return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  __device__ void set(int e, float x) {  // round to nearest even
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    uint32_t& w = ((uint32_t*)&raw)[e >> 1];
    w = (e & 1) ? ((w & 0x0000ffffu) | (u & 0xffff0000u)) : ((w & 0xffff0000u) | (u >> 16));
  }
};

template <typename T, int D>
struct RowGeom {
  static constexpr int EPV = 16 / (int)sizeof(T);  // elements per 16-byte vector
  static constexpr int TPR = (D / 2) / EPV;        // threads per row
  static constexpr int ROWS = 256 / TPR;           // rows per 256-thread block
};

// cos/sin of angle for a rotation by pos * inv_freq; double for fp32 data (the
// fp32 workload is held to 1e-5), float for bf16 data.
template <typename T>
__device__ __forceinline__ void rot_cs(double angle, float& c, float& s) {
  if constexpr (sizeof(T) == 4) {
    double sd, cd;
    sincos(angle, &sd, &cd);
    c = (float)cd;
    s = (float)sd;
  } else {
    sincosf((float)angle, &s, &c);
  }
}

__device__ __forceinline__ int pos_of_freq(const int4& p, int i, int rope_mode, int s0, int s01) {
  if (rope_mode != SV_ROPE_3D) return p.x;
  return i < s0 ? p.x : (i < s01 ? p.y : p.z);
}

template <typename T, int D>
__device__ __forceinline__ void rotate_pair_vec(Vec16<T>& lo, Vec16<T>& hi, const int4 p, int i0, int rope_mode,
                                                int s0, int s01, const double* __restrict__ inv_freq) {
  double f[Vec16<T>::N];   // all frequencies first: loaded one by one between the sincos evaluations, each is a round trip
#pragma unroll
  for (int e = 0; e < Vec16<T>::N; ++e) f[e] = inv_freq[i0 + e];
#pragma unroll
  for (int e = 0; e < Vec16<T>::N; ++e) {
    const int i = i0 + e;
    float c, s;
    rot_cs<T>((double)pos_of_freq(p, i, rope_mode, s0, s01) * f[e], c, s);
    const float a = lo.get(e), b = hi.get(e);
    lo.set(e, a * c - b * s);
    hi.set(e, b * c + a * s);
  }
}

// ---------------------------------------------------------------------------------
// Store n new tokens of one layer: cache[K|V][h][slot0 + j] = (rotated K | V)[j][h].
// bx: block of ROWS tokens, h: kv head, which: 0 = K, 1 = V.
// ---------------------------------------------------------------------------------
template <typename T, int D>
__device__ __forceinline__ void append_rows(int bx, int h, int which, const T* __restrict__ k_in,
                                            const T* __restrict__ v_in, T* __restrict__ k_cache, T* __restrict__ v_cache,
                                            const int4* __restrict__ pos4, const double* __restrict__ inv_freq,
                                            int64_t slot0, int n, int n_kv_heads, size_t head_stride_elems,
                                            int rope_mode, int s0, int s01, const float2* __restrict__ cs_tab = nullptr) {
  using G = RowGeom<T, D>;
  const int j = bx * G::ROWS + threadIdx.x / G::TPR;
  if (j >= n) return;
  const int t = threadIdx.x % G::TPR;
  const T* src = (which == 0 ? k_in : v_in) + ((size_t)j * n_kv_heads + h) * D;
  T* dst = (which == 0 ? k_cache : v_cache) + (size_t)h * head_stride_elems + (size_t)(slot0 + j) * D;
  Vec16<T> lo, hi;
  // The (uniform) choice of where cos/sin come from is made BEFORE the row's loads, so that on the table's path the
  // row and its cos/sin go out together: with the choice behind the row's loads the compiler waited for the row
  // before it issued the table's loads, two memory round trips for a kernel that is little else.
  if (which == 0 && cs_tab != nullptr) {   // (a table is only ever given with a rotary mode)
    // cos/sin of the run's tokens were tabulated when it was registered: [token][pair]
    const float2* cs = cs_tab + (size_t)j * (D / 2) + t * G::EPV;
    lo.raw = *(const decltype(lo.raw)*)(src + t * G::EPV);
    hi.raw = *(const decltype(hi.raw)*)(src + D / 2 + t * G::EPV);
    float2 r[Vec16<T>::N];
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) r[e] = cs[e];
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) {
      const float a = lo.get(e), b = hi.get(e);
      lo.set(e, a * r[e].x - b * r[e].y);
      hi.set(e, b * r[e].x + a * r[e].y);
    }
  } else {
    lo.raw = *(const decltype(lo.raw)*)(src + t * G::EPV);
    hi.raw = *(const decltype(hi.raw)*)(src + D / 2 + t * G::EPV);
    if (which == 0 && rope_mode != SV_ROPE_NONE)
      rotate_pair_vec<T, D>(lo, hi, pos4[slot0 + j], t * G::EPV, rope_mode, s0, s01, inv_freq);
  }
  *(decltype(lo.raw)*)(dst + t * G::EPV) = lo.raw;
  *(decltype(hi.raw)*)(dst + D / 2 + t * G::EPV) = hi.raw;
}

// grid: (ceil(n / ROWS), n_kv_heads, 2)
template <typename T, int D>
__global__ __launch_bounds__(256) void k_append_kv(const T* __restrict__ k_in, const T* __restrict__ v_in,
                                                   T* __restrict__ k_cache, T* __restrict__ v_cache,
                                                   const int4* __restrict__ pos4, const double* __restrict__ inv_freq,
                                                   int64_t slot0, int n, int n_kv_heads, size_t head_stride_elems,
                                                   int rope_mode, int s0, int s01) {
  append_rows<T, D>(blockIdx.x, blockIdx.y, blockIdx.z, k_in, v_in, k_cache, v_cache, pos4, inv_freq, slot0, n,
                    n_kv_heads, head_stride_elems, rope_mode, s0, s01);
}

// ---------------------------------------------------------------------------------
// Rotate rows of x [n][n_heads][D] in place at the positions of slots slot0 + j.
// bx: block of ROWS (token, head) rows.
// ---------------------------------------------------------------------------------
template <typename T, int D>
__device__ __forceinline__ void rope_rows(int bx, T* __restrict__ x, const int4* __restrict__ pos4,
                                          const double* __restrict__ inv_freq, int64_t slot0, int n, int n_heads,
                                          int rope_mode, int s0, int s01, const float2* __restrict__ cs_tab = nullptr) {
  using G = RowGeom<T, D>;
  const int64_t row = (int64_t)bx * G::ROWS + threadIdx.x / G::TPR;
  if (row >= (int64_t)n * n_heads) return;
  const int t = threadIdx.x % G::TPR;
  const int j = (int)(row / n_heads);
  T* p = x + row * D;
  Vec16<T> lo, hi;
  if (cs_tab != nullptr) {   // cos/sin of the run's tokens, tabulated when it was registered: [token][pair]
    const float2* cs = cs_tab + (size_t)j * (D / 2) + t * G::EPV;   // (the row and its cos/sin go out together)
    lo.raw = *(const decltype(lo.raw)*)(p + t * G::EPV);
    hi.raw = *(const decltype(hi.raw)*)(p + D / 2 + t * G::EPV);
    float2 r[Vec16<T>::N];
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) r[e] = cs[e];
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) {
      const float a = lo.get(e), b = hi.get(e);
      lo.set(e, a * r[e].x - b * r[e].y);
      hi.set(e, b * r[e].x + a * r[e].y);
    }
  } else {
    lo.raw = *(const decltype(lo.raw)*)(p + t * G::EPV);
    hi.raw = *(const decltype(hi.raw)*)(p + D / 2 + t * G::EPV);
    rotate_pair_vec<T, D>(lo, hi, pos4[slot0 + j], t * G::EPV, rope_mode, s0, s01, inv_freq);
  }
  *(decltype(lo.raw)*)(p + t * G::EPV) = lo.raw;
  *(decltype(hi.raw)*)(p + D / 2 + t * G::EPV) = hi.raw;
}

// grid: ceil(n * n_heads / ROWS)
template <typename T, int D>
__global__ __launch_bounds__(256) void k_rope_rows(T* __restrict__ x, const int4* __restrict__ pos4,
                                                   const double* __restrict__ inv_freq, int64_t slot0, int n,
                                                   int n_heads, int rope_mode, int s0, int s01) {
  rope_rows<T, D>(blockIdx.x, x, pos4, inv_freq, slot0, n, n_heads, rope_mode, s0, s01);
}

// ---------------------------------------------------------------------------------
// Storing V of new tokens into the blocked V^T layout (see sv_internal.h): rows [slot0, slot0 + n) of one kv head
// that fall into the group of 32 slots [32 grp, 32 grp + 32) are staged row-major in LDS, then every thread
// collects two pieces of 8 keys x one head dim (a block row) and writes each as 16 bytes, or element by element
// where a piece is only partly new (its other keys belong to older tokens).  Consecutive lanes write
// consecutive rows of a block: 1 KB contiguous per store instruction.
// Slots past the end of a stream inside its last block hold zeros or old values, never NaN patterns (the store is
// cleared at create time): the attention kernels multiply them by probabilities of exactly zero.
// ---------------------------------------------------------------------------------
constexpr int VG = 32;                     // slots per workgroup of the V^T store (4 blocks)
constexpr int VT_D = kVD;
constexpr int VT_SROW = VT_D * 2 + 16;     // bytes per staged row in LDS

__device__ __forceinline__ void append_v_t_group(char* sT, int grp, int hk, const __hip_bfloat16* __restrict__ v_in,
                                                 __hip_bfloat16* __restrict__ v_cache, int64_t slot0, int n,
                                                 int n_kv_heads, size_t head_stride_elems) {
  const int tid = threadIdx.x;
  const int64_t key0 = (int64_t)grp * VG;
  // both loads of a thread are unconditional (a slot of the group outside the run reads the run's nearest row and
  // stages zeros) and issued together: guarded, the compiler waited for the first before it issued the second
  uint4 vin[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int cid = tid + 256 * i, key = cid >> 4, c16 = cid & 15;
    const int64_t kc = min(max(key0 + key, slot0), slot0 + n - 1);
    vin[i] = *(const uint4*)(v_in + ((size_t)(kc - slot0) * n_kv_heads + hk) * VT_D + c16 * 8);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int cid = tid + 256 * i, key = cid >> 4, c16 = cid & 15;
    const int64_t kk = key0 + key;
    const bool in_run = (kk >= slot0) & (kk < slot0 + n);
    *(uint4*)(sT + key * VT_SROW + c16 * 16) = in_run ? vin[i] : make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  unsigned short* head_base = (unsigned short*)v_cache + (size_t)hk * head_stride_elems;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int piece = tid + 256 * i, p = piece >> 7, d = piece & 127;   // block p of the group, head dim d
    unsigned short e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = *(const unsigned short*)(sT + (8 * p + j) * VT_SROW + d * 2);
    const int64_t k8 = key0 + 8 * p;
    unsigned short* dst = head_base + vt_elem(k8, d);
    if (k8 >= slot0 && k8 + 8 <= slot0 + n) {
      uint4 w;
      w.x = e[0] | ((uint32_t)e[1] << 16), w.y = e[2] | ((uint32_t)e[3] << 16);
      w.z = e[4] | ((uint32_t)e[5] << 16), w.w = e[6] | ((uint32_t)e[7] << 16);
      *(uint4*)dst = w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (k8 + j >= slot0 && k8 + j < slot0 + n) dst[j] = e[j];
    }
  }
}

// ---------------------------------------------------------------------------------
// Everything that stores a run of new tokens of one layer in a blocked-V^T cache, in ONE launch: K rows (rotated
// at their positions), V into its V^T blocks, and, when q is given, the rotation of the tokens' Q rows in place (the
// chunk prefill's prologue).  The three jobs are independent; workgroup ids [0, nb_k) do the first,
// [nb_k, nb_k + nb_q) the second, the rest the third.
// ---------------------------------------------------------------------------------
// All 14 dwords of its arguments reach the wavefront in SGPRs at launch, so no scalar fetch precedes the loads of a
// kernel that is little more than one memory round trip: the V plane follows the K plane of the layer, the job
// boundaries follow from n, slot0 and the head counts, and cos/sin come from the run's table only (cs_tab NULL: no
// rotary embedding, rows are copied; a cache with a rotary mode always has the table for a run this kernel is given).
// shape: bit 1 = rotate q, bits 8-15 kv heads, bits 16-31 query heads.
__global__ __launch_bounds__(256) void k_store_tokens_vt(
    __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ k_in, const __hip_bfloat16* __restrict__ v_in,
    __hip_bfloat16* __restrict__ k_cache, const float2* __restrict__ cs_tab, int slot0, int n, uint32_t head_stride_elems,
    uint32_t shape) {
  __shared__ __attribute__((aligned(16))) char sT[VG * VT_SROW];
  using T = __hip_bfloat16;
  using G = RowGeom<T, VT_D>;
  constexpr int D = VT_D;
  const int n_kv_heads = (shape >> 8) & 255, n_q_heads = (int)(shape >> 16);
  __hip_bfloat16* const v_cache = k_cache + (size_t)n_kv_heads * head_stride_elems;   // K and V planes of a layer are adjacent
  const int gx_k = (n + G::ROWS - 1) / G::ROWS, nb_k = gx_k * n_kv_heads;
  const int nb_q = (shape & 2) ? (n * n_q_heads + G::ROWS - 1) / G::ROWS : 0;
  const int blk0 = slot0 / VG, n_blk = (slot0 + n - 1) / VG - blk0 + 1;   // groups of 32 slots
  int b = blockIdx.x;
  if (b >= nb_k + nb_q) {
    b -= nb_k + nb_q;
    append_v_t_group(sT, blk0 + b % n_blk, b / n_blk, v_in, v_cache, slot0, n, n_kv_heads, head_stride_elems);
    return;
  }
  // a K row into the cache, or a Q row in place: the row and its token's cos/sin go out together, one round trip
  const bool is_k = b < nb_k;
  const int t = threadIdx.x % G::TPR;
  int j;
  const T* src;
  T* dst;
  if (is_k) {
    const int h = b / gx_k;
    j = (b % gx_k) * G::ROWS + threadIdx.x / G::TPR;
    if (j >= n) return;
    src = k_in + ((size_t)j * n_kv_heads + h) * D;
    dst = k_cache + (size_t)h * head_stride_elems + (size_t)(slot0 + j) * D;
  } else {
    const int64_t row = (int64_t)(b - nb_k) * G::ROWS + threadIdx.x / G::TPR;
    if (row >= (int64_t)n * n_q_heads) return;
    j = (int)(row / n_q_heads);
    dst = q + row * D;
    src = dst;
  }
  Vec16<T> lo, hi;
  lo.raw = *(const decltype(lo.raw)*)(src + t * G::EPV);
  hi.raw = *(const decltype(hi.raw)*)(src + D / 2 + t * G::EPV);
  if (cs_tab != nullptr) {   // [token of the run][pair]
    const float2* cs = cs_tab + (size_t)j * (D / 2) + t * G::EPV;
    float2 r[Vec16<T>::N];
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) r[e] = cs[e];
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) {
      const float a = lo.get(e), bb = hi.get(e);
      lo.set(e, a * r[e].x - bb * r[e].y);
      hi.set(e, bb * r[e].x + a * r[e].y);
    }
  }
  *(decltype(lo.raw)*)(dst + t * G::EPV) = lo.raw;
  *(decltype(hi.raw)*)(dst + D / 2 + t * G::EPV) = hi.raw;
}

// The same three jobs with cos/sin evaluated from the tokens' positions: runs that have no table (longer than the
// cache's max_q_tokens).
__global__ __launch_bounds__(256) void k_store_tokens_vt_pos(
    __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ k_in, const __hip_bfloat16* __restrict__ v_in,
    __hip_bfloat16* __restrict__ k_cache, __hip_bfloat16* __restrict__ v_cache, const int4* __restrict__ pos4,
    const double* __restrict__ inv_freq, int64_t slot0, int n, int n_q_heads, int n_kv_heads, size_t head_stride_elems,
    int rope_mode, int s0, int s01, int gx_k, int nb_k, int nb_q, int blk0, int n_blk,
    const float2* __restrict__ cs_tab) {
  __shared__ __attribute__((aligned(16))) char sT[VG * VT_SROW];
  using T = __hip_bfloat16;
  int b = blockIdx.x;
  if (b < nb_k) {
    append_rows<T, VT_D>(b % gx_k, b / gx_k, 0, k_in, v_in, k_cache, v_cache, pos4, inv_freq, slot0, n, n_kv_heads,
                         head_stride_elems, rope_mode, s0, s01, cs_tab);
    return;
  }
  b -= nb_k;
  if (b < nb_q) {
    rope_rows<T, VT_D>(b, q, pos4, inv_freq, slot0, n, n_q_heads, rope_mode, s0, s01, cs_tab);
    return;
  }
  b -= nb_q;
  append_v_t_group(sT, blk0 + b % n_blk, b / n_blk, v_in, v_cache, slot0, n, n_kv_heads, head_stride_elems);
}

// ---------------------------------------------------------------------------------
// Compaction gather over all layers: new[l][K|V][h][j] = old[l][K|V][h][src[j]],
// K re-rotated when delta[j] != 0.  old and new are the two halves of the
// ping-pong store, so no row is overwritten before it is read.
// Token groups (ROWS tokens) below x0 are not moved: the caller knows that the new half holds them already (tokens
// that two evictions in a row left in place, unshifted: the sink text at the front of a stream in steady state).
// grid: (ceil(n_new / ROWS) - x0, n_kv_heads, 2 * n_layers)
// ---------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void k_compact(const T* __restrict__ old_base, T* __restrict__ new_base,
                                                 const int32_t* __restrict__ src, const int32_t* __restrict__ delta,
                                                 const float2* __restrict__ dtab, int n_new,
                                                 size_t head_stride_elems, size_t tensor_stride_elems, int rotate,
                                                 int v_blocked, int x0) {
  using G = RowGeom<T, D>;
  const int bx = (int)blockIdx.x + x0;   // token group; the groups below x0 stay where they are
  const int h = blockIdx.y;
  const int which = blockIdx.z & 1;   // z = 2 * layer + which, tensors are laid out in that order
  const size_t plane = (size_t)blockIdx.z * tensor_stride_elems + (size_t)h * head_stride_elems;
  typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
  if constexpr (sizeof(T) == 2 && D == kVD) {
    if (which == 1 && v_blocked) {
      // V in the blocked V^T layout.  The workgroup moves the same 32 tokens as a workgroup of K rows: 4 new
      // blocks of 8 keys, 512 block rows of 16 bytes, two per thread (block p, head dim d), consecutive lanes
      // on consecutive rows.  A new block whose 8 tokens were consecutive in the old cache and started at a
      // multiple of 8 is a copy of an old block, 2 KB contiguous on both sides (the rule when runs of 8 k tokens
      // leave, as in the streaming workloads); otherwise its elements are gathered one by one.
      static_assert(G::ROWS == 32, "K rows and V^T blocks share the grid: 32 tokens per workgroup");
      const unsigned short* so = (const unsigned short*)old_base + plane;
      unsigned short* sn = (unsigned short*)new_base + plane;
      u32x4 w[2];
      bool live[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int piece = threadIdx.x + 256 * i, p = piece >> 7, d = piece & 127;
        const int jc = bx * 32 + 8 * p;
        live[i] = jc < n_new;   // a block wholly past the end: nothing to move
        if (!live[i]) continue;
        const int sa = src[jc];
        if (jc + 7 < n_new && src[jc + 7] == sa + 7 && (sa & 7) == 0) {
          w[i] = __builtin_nontemporal_load((const u32x4*)(so + vt_elem(sa, d)));
        } else {
          unsigned short e[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            e[j] = 0;
            if (jc + j < n_new) e[j] = so[vt_elem(src[jc + j], d)];
          }
          w[i][0] = e[0] | ((uint32_t)e[1] << 16), w[i][1] = e[2] | ((uint32_t)e[3] << 16);
          w[i][2] = e[4] | ((uint32_t)e[5] << 16), w[i][3] = e[6] | ((uint32_t)e[7] << 16);
        }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int piece = threadIdx.x + 256 * i, p = piece >> 7, d = piece & 127;
        if (live[i]) *(u32x4*)(sn + vt_elem((int64_t)bx * 32 + 8 * p, d)) = w[i];
      }
      return;
    }
  }
  const int j = bx * G::ROWS + threadIdx.x / G::TPR;
  if (j >= n_new) return;
  const int t = threadIdx.x % G::TPR;
  const T* s = old_base + plane + (size_t)src[j] * D;
  T* d = new_base + plane + (size_t)j * D;
  Vec16<T> lo, hi;
  // the old buffer is read once and dead afterwards: non-temporal loads (16 bytes as a native vector); measured
  // 92.8 -> 90 us for 28 layers at 5.1k retained tokens, non-temporal stores on top of that: no change
  static_assert(sizeof(lo.raw) == sizeof(u32x4), "16-byte vectors");
  {
    const u32x4 a = __builtin_nontemporal_load((const u32x4*)(s + t * G::EPV));
    const u32x4 b = __builtin_nontemporal_load((const u32x4*)(s + D / 2 + t * G::EPV));
    __builtin_memcpy(&lo.raw, &a, 16);
    __builtin_memcpy(&hi.raw, &b, 16);
  }
  if (which == 0 && rotate && delta[j] != 0) {
    const float2* cs = dtab + (size_t)j * (D / 2) + t * G::EPV;
#pragma unroll
    for (int e = 0; e < Vec16<T>::N; ++e) {
      const float2 r = cs[e];
      const float a = lo.get(e), b = hi.get(e);
      lo.set(e, a * r.x - b * r.y);
      hi.set(e, b * r.x + a * r.y);
    }
  }
  *(decltype(lo.raw)*)(d + t * G::EPV) = lo.raw;
  *(decltype(hi.raw)*)(d + D / 2 + t * G::EPV) = hi.raw;
}

template <typename T, int D>
hipError_t append_kv_t(const sv_cache* c, int stream, int layer, int64_t slot0, int n, const void* k, const void* v,
                       hipStream_t s) {
  using G = RowGeom<T, D>;
  const int cur = c->st[stream].cur;
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  const int s0 = c->cfg.mrope_sections[0], s01 = s0 + c->cfg.mrope_sections[1];
  dim3 grid((n + G::ROWS - 1) / G::ROWS, c->cfg.n_kv_heads, 2);
  hipLaunchKernelGGL((k_append_kv<T, D>), grid, dim3(256), 0, s, (const T*)k, (const T*)v,
                     (T*)c->kv_ptr(stream, cur, layer, 0), (T*)c->kv_ptr(stream, cur, layer, 1),
                     c->meta[cur].pos4 + off, c->inv_freq, slot0, n, c->cfg.n_kv_heads,
                     c->head_stride / sizeof(T), c->cfg.rope_mode, s0, s01);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t rope_apply_t(const sv_cache* c, int stream, int64_t slot0, int n, void* q, void* k, hipStream_t s) {
  using G = RowGeom<T, D>;
  const int cur = c->st[stream].cur;
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  const int s0 = c->cfg.mrope_sections[0], s01 = s0 + c->cfg.mrope_sections[1];
  void* ptrs[2] = {q, k};
  const int heads[2] = {c->cfg.n_q_heads, c->cfg.n_kv_heads};
  for (int a = 0; a < 2; ++a) {
    if (!ptrs[a]) continue;
    const int64_t rows = (int64_t)n * heads[a];
    dim3 grid((unsigned)((rows + G::ROWS - 1) / G::ROWS));
    hipLaunchKernelGGL((k_rope_rows<T, D>), grid, dim3(256), 0, s, (T*)ptrs[a], c->meta[cur].pos4 + off,
                       c->inv_freq, slot0, n, heads[a], c->cfg.rope_mode, s0, s01);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <typename T, int D>
hipError_t compact_t(const sv_cache* c, int stream, int64_t n_new, int64_t n_still, hipStream_t s) {
  using G = RowGeom<T, D>;
  const int cur = c->st[stream].cur;
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  const int rotate = c->cfg.rope_mode != SV_ROPE_NONE;
  float2* dtab = c->dtab + off * (D / 2);   // rows of the tokens with a shift, written by the eviction scan
  const int groups = (int)((n_new + G::ROWS - 1) / G::ROWS), x0 = (int)std::min<int64_t>(n_still / G::ROWS, groups);
  if (x0 == groups) return hipSuccess;
  dim3 grid((unsigned)(groups - x0), c->cfg.n_kv_heads, 2 * c->cfg.n_layers);
  hipLaunchKernelGGL((k_compact<T, D>), grid, dim3(256), 0, s, (const T*)c->kv_ptr(stream, cur, 0, 0),
                     (T*)c->kv_ptr(stream, cur ^ 1, 0, 0), c->src + off, c->delta + off, dtab, (int)n_new,
                     c->head_stride / sizeof(T), c->tensor_stride / sizeof(T), rotate, c->v_blocked ? 1 : 0, x0);
  return hipGetLastError();
}

}  // namespace

#define SV_DISPATCH(fn, ...)                                                                   \
  do {                                                                                         \
    if (c->cfg.dtype == SV_DTYPE_F32) {                                                        \
      return c->cfg.head_dim == 64 ? fn<float, 64>(__VA_ARGS__) : fn<float, 128>(__VA_ARGS__); \
    }                                                                                          \
    return c->cfg.head_dim == 64 ? fn<__hip_bfloat16, 64>(__VA_ARGS__)                         \
                                 : fn<__hip_bfloat16, 128>(__VA_ARGS__);                       \
  } while (0)

hipError_t launch_rope_apply(const sv_cache* c, int stream, int64_t slot0, int n, void* q, void* k,
                             hipStream_t s) {
  SV_DISPATCH(rope_apply_t, c, stream, slot0, n, q, k, s);
}

hipError_t launch_compact(const sv_cache* c, int stream, int64_t n_new, int64_t n_still, hipStream_t s) {
  SV_DISPATCH(compact_t, c, stream, n_new, n_still, s);
}

hipError_t launch_append_kv(const sv_cache* c, int stream, int layer, int64_t slot0, int n, const void* k,
                            const void* v, hipStream_t s) {
  if (c->v_blocked) return launch_store_tokens_vt(c, stream, layer, slot0, n, nullptr, k, v, s);
  SV_DISPATCH(append_kv_t, c, stream, layer, slot0, n, k, v, s);
}

hipError_t launch_store_tokens_vt(const sv_cache* c, int stream, int layer, int64_t slot0, int n, void* q, const void* k,
                                  const void* v, hipStream_t s) {
  using G = RowGeom<__hip_bfloat16, VT_D>;
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads, cur = c->st[stream].cur;
  const int gx_k = (n + G::ROWS - 1) / G::ROWS, nb_k = gx_k * Hkv;
  const bool rot_q = q && c->cfg.rope_mode != SV_ROPE_NONE;
  const int nb_q = rot_q ? (int)(((int64_t)n * Hq + G::ROWS - 1) / G::ROWS) : 0;
  const int blk0 = (int)(slot0 / VG), n_blk = (int)((slot0 + n - 1) / VG) - blk0 + 1;   // groups of 32 slots
  // what the kernel's packed arguments can carry, and the layout it relies on (V plane right behind the K plane)
  if (Hkv > 255 || Hq > 65535 || c->head_stride / 2 > 0xffffffffull || (int64_t)n * Hq > 0x7fffffff ||
      c->kv_ptr(stream, cur, layer, 1) != c->kv_ptr(stream, cur, layer, 0) + (size_t)Hkv * c->head_stride)
    return hipErrorInvalidValue;
  const float2* cs_tab = nullptr;
  if (c->cfg.rope_mode != SV_ROPE_NONE) {   // the run's cos/sin table, written when the run was registered
    const StreamState& st = c->st[stream];
    if (!st.cs_tab_valid || st.pending_slot0 != slot0 || st.pending_n != n) {   // no table: positions and sincos
      const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
      hipLaunchKernelGGL(k_store_tokens_vt_pos, dim3(nb_k + nb_q + n_blk * Hkv), dim3(256), 0, s, (__hip_bfloat16*)q,
                         (const __hip_bfloat16*)k, (const __hip_bfloat16*)v,
                         (__hip_bfloat16*)c->kv_ptr(stream, cur, layer, 0), (__hip_bfloat16*)c->kv_ptr(stream, cur, layer, 1),
                         c->meta[cur].pos4 + off, c->inv_freq, slot0, n, Hq, Hkv, c->head_stride / 2, c->cfg.rope_mode,
                         c->cfg.mrope_sections[0], c->cfg.mrope_sections[0] + c->cfg.mrope_sections[1], gx_k, nb_k, nb_q,
                         blk0, n_blk, (const float2*)nullptr);
      return hipGetLastError();
    }
    cs_tab = c->cs_tab + (size_t)stream * c->cfg.max_q_tokens * (VT_D / 2);
  }
  const uint32_t shape = (uint32_t)rot_q << 1 | (uint32_t)Hkv << 8 | (uint32_t)Hq << 16;
  hipLaunchKernelGGL(k_store_tokens_vt, dim3(nb_k + nb_q + n_blk * Hkv), dim3(256), 0, s, (__hip_bfloat16*)q,
                     (const __hip_bfloat16*)k, (const __hip_bfloat16*)v, (__hip_bfloat16*)c->kv_ptr(stream, cur, layer, 0),
                     cs_tab, (int)slot0, n, (uint32_t)(c->head_stride / 2), shape);
  return hipGetLastError();
}

}  // namespace sv
