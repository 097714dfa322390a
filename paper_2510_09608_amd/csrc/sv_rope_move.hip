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
__device__ __forceinline__ void rotate_pair_vec(Vec16<T>& lo, Vec16<T>& hi, const int4& p, int i0, int rope_mode,
                                                int s0, int s01, const double* __restrict__ inv_freq) {
#pragma unroll
  for (int e = 0; e < Vec16<T>::N; ++e) {
    const int i = i0 + e;
    float c, s;
    rot_cs<T>((double)pos_of_freq(p, i, rope_mode, s0, s01) * inv_freq[i], c, s);
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
                                            int rope_mode, int s0, int s01) {
  using G = RowGeom<T, D>;
  const int j = bx * G::ROWS + threadIdx.x / G::TPR;
  if (j >= n) return;
  const int t = threadIdx.x % G::TPR;
  const T* src = (which == 0 ? k_in : v_in) + ((size_t)j * n_kv_heads + h) * D;
  T* dst = (which == 0 ? k_cache : v_cache) + (size_t)h * head_stride_elems + (size_t)(slot0 + j) * D;
  Vec16<T> lo, hi;
  lo.raw = *(const decltype(lo.raw)*)(src + t * G::EPV);
  hi.raw = *(const decltype(hi.raw)*)(src + D / 2 + t * G::EPV);
  if (which == 0 && rope_mode != SV_ROPE_NONE)
    rotate_pair_vec<T, D>(lo, hi, pos4[slot0 + j], t * G::EPV, rope_mode, s0, s01, inv_freq);
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
                                          int rope_mode, int s0, int s01) {
  using G = RowGeom<T, D>;
  const int64_t row = (int64_t)bx * G::ROWS + threadIdx.x / G::TPR;
  if (row >= (int64_t)n * n_heads) return;
  const int t = threadIdx.x % G::TPR;
  const int j = (int)(row / n_heads);
  T* p = x + row * D;
  Vec16<T> lo, hi;
  lo.raw = *(const decltype(lo.raw)*)(p + t * G::EPV);
  hi.raw = *(const decltype(hi.raw)*)(p + D / 2 + t * G::EPV);
  rotate_pair_vec<T, D>(lo, hi, pos4[slot0 + j], t * G::EPV, rope_mode, s0, s01, inv_freq);
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
// V^T staging for the pipelined chunk-prefill kernel (bf16, head_dim 128).  That kernel's second product
// wants V^T fragments (one head dim, 8 consecutive keys per lane); read from a row-major V tile that costs two
// half-rate LDS transpose reads per fragment in EVERY wavefront of every workgroup that shares the tile.  This
// pass transposes each 64-key block of the layer's V once, into vt[kv head][block][head dim][64 keys]; the
// attention kernel then brings V^T tiles to LDS with direct loads and reads fragments with plain 16-byte
// reads.  Rows [new0, new0 + n_new) may come from the caller's buffer v_new [n_new][n_kv_heads][128] instead of
// the cache (they are being appended by other workgroups of the same launch); keys past n_kv are written as
// zeros (they are masked, but must be finite).  One 256-thread workgroup per (block, kv head).
//
// LDS transpose read (ds_read_b64_tr_b16): within each group of 16 lanes, lane j hands in the address of 4
// consecutive 16-bit elements and receives element (j & 3) of the chunks of lanes (j >> 2) + 4 e, e = 0..3;
// pointing lane j at row r0 + (j >> 2), columns c0 + 4 (j & 3) .. + 3 of a row-major tile returns column
// c0 + j of rows r0 .. r0 + 3.
// ---------------------------------------------------------------------------------
constexpr int VT_KEYS = 64;              // keys per block
constexpr int VT_D = 128;
constexpr int VT_ROW = VT_D * 2 + 64;    // LDS row stride in bytes: transpose reads fall in distinct banks
constexpr int VT_OROW = VT_KEYS * 2 + 16;   // row stride of the transposed block on its way out
static_assert(VT_D * VT_OROW <= VT_KEYS * VT_ROW, "the transposed block reuses the staging buffer");
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void vt_block(char* sT, int blk, int hk, const __hip_bfloat16* __restrict__ v_cache,
                                         const __hip_bfloat16* __restrict__ v_new, int64_t new0, int n_new, int n_kv,
                                         int n_kv_heads, size_t head_stride_elems, __hip_bfloat16* __restrict__ vt,
                                         size_t vt_head_stride_elems) {
  const int tid = threadIdx.x;
  const __hip_bfloat16* src = v_cache + (size_t)hk * head_stride_elems;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int cid = tid + 256 * i, key = cid >> 4, c16 = cid & 15;
    const int64_t kk = (int64_t)blk * VT_KEYS + key;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (kk < n_kv) {
      const bool fresh = v_new != nullptr && kk >= new0 && kk < new0 + n_new;
      const __hip_bfloat16* row = fresh ? v_new + ((size_t)(kk - new0) * n_kv_heads + hk) * VT_D : src + (size_t)kk * VT_D;
      v = *(const uint4*)(row + c16 * 8);
    }
    *(uint4*)(sT + key * VT_ROW + c16 * 16) = v;
  }
  __syncthreads();
  const int wave = tid >> 6, lane = tid & 63, j16 = lane & 15, g = lane >> 4;
  __hip_bfloat16* dst = vt + (size_t)hk * vt_head_stride_elems + (size_t)blk * VT_KEYS * VT_D;
  // transposing reads: 8 keys (r0 .. r0 + 7) of head dim c0 + j16 per lane
  v8i16 a8[2][2];
#pragma unroll
  for (int ko = 0; ko < 2; ++ko)
#pragma unroll
    for (int ds = 0; ds < 2; ++ds) {
      const int r0 = 16 * wave + 8 * ko, c0 = 64 * ds + 16 * g;
      const int off = (r0 + (j16 >> 2)) * VT_ROW + (c0 + 4 * (j16 & 3)) * 2;
      auto rd = [&](int o) {
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (v4i16 __attribute__((address_space(3)))*)((__attribute__((address_space(3))) char*)sT + o));
      };
      const v4i16 a0 = rd(off), a1 = rd(off + 4 * VT_ROW);
      a8[ko][ds] = v8i16{a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
    }
  // A lane's 16 bytes belong to a row of V^T of their own (64 different 128-byte rows per store instruction), so
  // the block goes back through LDS in V^T layout (rows of 64 keys, 144-byte stride: conflict-free for the 16-byte
  // writes) and leaves as full 128-byte rows, 8 lanes per row.
  __syncthreads();
#pragma unroll
  for (int ko = 0; ko < 2; ++ko)
#pragma unroll
    for (int ds = 0; ds < 2; ++ds) {
      const int r0 = 16 * wave + 8 * ko, c0 = 64 * ds + 16 * g;
      *(v8i16*)(sT + (c0 + j16) * VT_OROW + r0 * 2) = a8[ko][ds];
    }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 3) + 32 * i, ch = tid & 7;
    *(uint4*)(dst + (size_t)row * VT_KEYS + ch * 8) = *(const uint4*)(sT + row * VT_OROW + ch * 16);
  }
}

// grid: (blocks of 64 keys, kv heads)
__global__ __launch_bounds__(256) void k_vt_build(const __hip_bfloat16* __restrict__ v_cache,
                                                  __hip_bfloat16* __restrict__ vt, int n_kv, int n_kv_heads,
                                                  size_t head_stride_elems, size_t vt_head_stride_elems) {
  __shared__ __attribute__((aligned(16))) char sT[VT_KEYS * VT_ROW];
  vt_block(sT, blockIdx.x, blockIdx.y, v_cache, nullptr, 0, 0, n_kv, n_kv_heads, head_stride_elems, vt,
           vt_head_stride_elems);
}

// ---------------------------------------------------------------------------------
// Everything a layer needs before the chunk-prefill attention of a new chunk, in ONE launch (bf16, head_dim
// 128): store the chunk's K (rotated) and V, rotate its Q in place, and stage V^T of the whole layer (old rows
// from the cache, the chunk's rows from the caller's buffer).  The three jobs are independent; workgroup ids
// [0, nb_kv) do the first, [nb_kv, nb_kv + nb_q) the second, the rest the third.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_chunk_prologue(
    __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ k_in, const __hip_bfloat16* __restrict__ v_in,
    __hip_bfloat16* __restrict__ k_cache, __hip_bfloat16* __restrict__ v_cache, const int4* __restrict__ pos4,
    const double* __restrict__ inv_freq, int64_t slot0, int n, int n_q_heads, int n_kv_heads, size_t head_stride_elems,
    int rope_mode, int s0, int s01, int gx_kv, int nb_kv, int nb_q, __hip_bfloat16* __restrict__ vt,
    size_t vt_head_stride_elems, int n_blk) {
  __shared__ __attribute__((aligned(16))) char sT[VT_KEYS * VT_ROW];
  using T = __hip_bfloat16;
  int b = blockIdx.x;
  if (b < nb_kv) {
    append_rows<T, VT_D>(b % gx_kv, (b / gx_kv) % n_kv_heads, b / (gx_kv * n_kv_heads), k_in, v_in, k_cache, v_cache,
                         pos4, inv_freq, slot0, n, n_kv_heads, head_stride_elems, rope_mode, s0, s01);
    return;
  }
  b -= nb_kv;
  if (b < nb_q) {
    if (rope_mode != SV_ROPE_NONE) rope_rows<T, VT_D>(b, q, pos4, inv_freq, slot0, n, n_q_heads, rope_mode, s0, s01);
    return;
  }
  b -= nb_q;
  vt_block(sT, b % n_blk, b / n_blk, v_cache, v_in, slot0, n, (int)(slot0 + n), n_kv_heads, head_stride_elems, vt,
           vt_head_stride_elems);
}

// ---------------------------------------------------------------------------------
// cos/sin of the re-rotation of each surviving token: moving from old to new
// position turns pair i by -(delta * inv_freq[i]); stored as (cos, -sin) so the
// mover applies the same formula as a forward rotation.  delta is one scalar per
// token even in 3-D mode because t, h and w shift together.
// ---------------------------------------------------------------------------------
__global__ void k_delta_table(const int32_t* __restrict__ delta, const double* __restrict__ inv_freq,
                              float2* __restrict__ dtab, int n_new, int half) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_new * half) return;
  const int j = idx / half, i = idx % half;
  const int d = delta[j];
  float2 cs = make_float2(1.f, 0.f);
  if (d != 0) {
    double sd, cd;
    sincos((double)d * inv_freq[i], &sd, &cd);
    cs = make_float2((float)cd, (float)-sd);
  }
  dtab[idx] = cs;
}

// ---------------------------------------------------------------------------------
// Compaction gather over all layers: new[l][K|V][h][j] = old[l][K|V][h][src[j]],
// K re-rotated when delta[j] != 0.  old and new are the two halves of the
// ping-pong store, so no row is overwritten before it is read.
// grid: (ceil(n_new / ROWS), n_kv_heads, 2 * n_layers)
// ---------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void k_compact(const T* __restrict__ old_base, T* __restrict__ new_base,
                                                 const int32_t* __restrict__ src, const int32_t* __restrict__ delta,
                                                 const float2* __restrict__ dtab, int n_new,
                                                 size_t head_stride_elems, size_t tensor_stride_elems, int rotate) {
  using G = RowGeom<T, D>;
  const int j = blockIdx.x * G::ROWS + threadIdx.x / G::TPR;
  if (j >= n_new) return;
  const int t = threadIdx.x % G::TPR, h = blockIdx.y;
  const int which = blockIdx.z & 1;  // z = 2 * layer + which, tensors are laid out in that order
  const size_t plane = (size_t)blockIdx.z * tensor_stride_elems + (size_t)h * head_stride_elems;
  const T* s = old_base + plane + (size_t)src[j] * D;
  T* d = new_base + plane + (size_t)j * D;
  Vec16<T> lo, hi;
  // the old buffer is read once and dead afterwards: non-temporal loads (16 bytes as a native vector); measured
  // 92.8 -> 90 us for 28 layers at 5.1k retained tokens, non-temporal stores on top of that: no change
  typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
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
hipError_t compact_t(const sv_cache* c, int stream, int64_t n_new, hipStream_t s) {
  using G = RowGeom<T, D>;
  const int cur = c->st[stream].cur;
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  const int rotate = c->cfg.rope_mode != SV_ROPE_NONE;
  float2* dtab = c->dtab + off * (D / 2);
  if (rotate) {
    const int total = (int)n_new * (D / 2);
    hipLaunchKernelGGL(k_delta_table, dim3((total + 255) / 256), dim3(256), 0, s, c->delta + off, c->inv_freq, dtab,
                       (int)n_new, D / 2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  dim3 grid((unsigned)((n_new + G::ROWS - 1) / G::ROWS), c->cfg.n_kv_heads, 2 * c->cfg.n_layers);
  hipLaunchKernelGGL((k_compact<T, D>), grid, dim3(256), 0, s, (const T*)c->kv_ptr(stream, cur, 0, 0),
                     (T*)c->kv_ptr(stream, cur ^ 1, 0, 0), c->src + off, c->delta + off, dtab, (int)n_new,
                     c->head_stride / sizeof(T), c->tensor_stride / sizeof(T), rotate);
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

hipError_t launch_append_kv(const sv_cache* c, int stream, int layer, int64_t slot0, int n, const void* k,
                            const void* v, hipStream_t s) {
  SV_DISPATCH(append_kv_t, c, stream, layer, slot0, n, k, v, s);
}

hipError_t launch_rope_apply(const sv_cache* c, int stream, int64_t slot0, int n, void* q, void* k,
                             hipStream_t s) {
  SV_DISPATCH(rope_apply_t, c, stream, slot0, n, q, k, s);
}

hipError_t launch_compact(const sv_cache* c, int stream, int64_t n_new, hipStream_t s) {
  SV_DISPATCH(compact_t, c, stream, n_new, s);
}

hipError_t launch_vt_build(const sv_cache* c, int stream, int layer, int n_kv, hipStream_t s) {
  const int Hkv = c->cfg.n_kv_heads;
  __hip_bfloat16* vt = (__hip_bfloat16*)(c->vt + (size_t)stream * c->vt_stream_stride);
  hipLaunchKernelGGL(k_vt_build, dim3((n_kv + VT_KEYS - 1) / VT_KEYS, Hkv), dim3(256), 0, s,
                     (const __hip_bfloat16*)c->kv_ptr(stream, c->st[stream].cur, layer, 1), vt, n_kv, Hkv,
                     c->head_stride / 2, c->vt_stream_stride / 2 / Hkv);
  return hipGetLastError();
}

hipError_t launch_chunk_prologue(const sv_cache* c, int stream, int layer, int64_t slot0, int n, void* q, const void* k,
                                 const void* v, hipStream_t s) {
  using G = RowGeom<__hip_bfloat16, VT_D>;
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads, cur = c->st[stream].cur;
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  const int gx_kv = (n + G::ROWS - 1) / G::ROWS, nb_kv = gx_kv * Hkv * 2;
  const int nb_q = (int)(((int64_t)n * Hq + G::ROWS - 1) / G::ROWS);
  const int n_blk = (int)((slot0 + n + VT_KEYS - 1) / VT_KEYS);
  hipLaunchKernelGGL(k_chunk_prologue, dim3(nb_kv + nb_q + n_blk * Hkv), dim3(256), 0, s, (__hip_bfloat16*)q,
                     (const __hip_bfloat16*)k, (const __hip_bfloat16*)v, (__hip_bfloat16*)c->kv_ptr(stream, cur, layer, 0),
                     (__hip_bfloat16*)c->kv_ptr(stream, cur, layer, 1), c->meta[cur].pos4 + off, c->inv_freq, slot0, n, Hq,
                     Hkv, c->head_stride / 2, c->cfg.rope_mode, c->cfg.mrope_sections[0],
                     c->cfg.mrope_sections[0] + c->cfg.mrope_sections[1], gx_kv, nb_kv, nb_q,
                     (__hip_bfloat16*)(c->vt + (size_t)stream * c->vt_stream_stride), c->vt_stream_stride / 2 / Hkv, n_blk);
  return hipGetLastError();
}

}  // namespace sv
