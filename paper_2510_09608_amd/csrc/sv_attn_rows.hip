// Row-wise split-KV attention: one query token (all its heads) against a cache
// prefix.  This is the text-decode kernel (Sec. 2.1 / Sec. 3.3: every generated
// token attends to the compact cache), also used with one row per stream for
// ragged batches, and with one row per chunk token as the chunk-prefill path of
// configurations the MFMA kernel does not cover (fp32, head_dim 64).
//
// The kernel is bound by reading K and V once from HBM: 2 * n_kv_heads *
// head_dim * esize bytes per cached token per layer, shared by the n_q_heads /
// n_kv_heads query heads of each kv head.  One launch does the whole decode step
// of a layer:
//   * a workgroup owns one (row, kv head, key range); 16 lanes share a key row
//     (16-byte loads, fully coalesced), so a wavefront streams 4 keys at a time;
//     keys are taken in batches of 4 per lane group so that 8 loads are in flight
//     per lane and the running max is updated once per batch;
//   * in the fused form the query is rotated in registers at the position of the
//     new token, and the new token's K (rotated) and V are written to the cache by
//     the workgroup whose range ends at that token, which uses them from registers;
//   * scores are reduced over the 16 lanes with shuffles, the 16 lane groups are
//     merged with the log-sum-exp rule, and the key ranges are merged by whichever
//     workgroup of a (row, kv head) finishes last (a counter in device memory that
//     the same workgroup resets), so no second launch is needed.

#include <hip/hip_bf16.h>

#include <algorithm>

#include "sv_internal.h"

namespace sv {
namespace {

constexpr int kMaxRowsPerLaunch = 64;
constexpr int kMaxSplits = 64;
constexpr int KB = 4;  // keys per lane group per batch

struct RowDesc {
  const void* k;      // K of the layer: kv head 0, slot 0
  const void* v;
  void* k_w;          // same buffers, writable (fused append)
  void* v_w;
  const int4* pos4;   // position of the query token (fused rotation)
  int32_t len;        // keys visible: slots [0, len); the query token is slot len - 1
};
struct RowTable {
  RowDesc r[kMaxRowsPerLaunch];
};

struct RopeParams {
  const double* inv_freq;
  int mode, s0, s01;
};

template <typename T, int EPL>
__device__ __forceinline__ void load_chunk(const T* p, float (&f)[EPL]) {
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      const float4 v = *(const float4*)(p + e);
      f[e] = v.x, f[e + 1] = v.y, f[e + 2] = v.z, f[e + 3] = v.w;
    }
  } else if constexpr (EPL == 8) {
    const uint4 v = *(const uint4*)p;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[2 * e] = __uint_as_float(w[e] << 16);
      f[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  } else {
    const uint2 v = *(const uint2*)p;
    const uint32_t w[2] = {v.x, v.y};
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      f[2 * e] = __uint_as_float(w[e] << 16);
      f[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
}

__device__ __forceinline__ uint32_t bf16_bits(float x) {  // round to nearest even, result in the high half
  uint32_t a = __float_as_uint(x);
  a += 0x7fffu + ((a >> 16) & 1u);
  return a & 0xffff0000u;
}

// Value a stored element will read back as (identity for fp32 storage).
template <typename T>
__device__ __forceinline__ float storage_round(float x) {
  if constexpr (sizeof(T) == 4) return x;
  else return __uint_as_float(bf16_bits(x));
}

template <typename T, int EPL>
__device__ __forceinline__ void store_chunk(T* p, const float (&f)[EPL]) {  // f already storage-rounded
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int e = 0; e < EPL; e += 4) *(float4*)(p + e) = make_float4(f[e], f[e + 1], f[e + 2], f[e + 3]);
  } else {
    uint32_t w[EPL / 2];
#pragma unroll
    for (int e = 0; e < EPL / 2; ++e) w[e] = (__float_as_uint(f[2 * e]) >> 16) | (__float_as_uint(f[2 * e + 1]) & 0xffff0000u);
    if constexpr (EPL == 8) *(uint4*)p = make_uint4(w[0], w[1], w[2], w[3]);
    else *(uint2*)p = make_uint2(w[0], w[1]);
  }
}

// exp of a difference of scaled scores.  fp32 data: scores are in natural units
// and expf keeps the 1e-5 bar; bf16 data: scores carry a log2(e) factor and the
// hardware exp2 is ample.
template <typename T>
__device__ __forceinline__ float exp_diff(float x) {
  if constexpr (sizeof(T) == 4) return expf(x);
  else return __builtin_amdgcn_exp2f(x);
}

// cos/sin of the rotary angles of the EPL pairs a lane owns.  The 16 lanes of a
// group cover head_dim: lanes 0-7 hold the low halves, lanes 8-15 the high halves
// of the same pairs, so lane li and lane li ^ 8 share frequencies (li & 7) * EPL + e.
template <typename T, int EPL>
__device__ __forceinline__ void lane_cos_sin(const int4 pos, int li, const RopeParams& rp, float (&c)[EPL],
                                             float (&s)[EPL]) {
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int i = (li & 7) * EPL + e;
    const int p = rp.mode != SV_ROPE_3D ? pos.x : (i < rp.s0 ? pos.x : (i < rp.s01 ? pos.y : pos.z));
    const double ang = (double)p * rp.inv_freq[i];
    if constexpr (sizeof(T) == 4) {
      double sd, cd;
      sincos(ang, &sd, &cd);
      c[e] = (float)cd, s[e] = (float)sd;
    } else {
      sincosf((float)ang, &s[e], &c[e]);
    }
  }
}

// Rotate the chunk a lane holds; the partner half lives 8 lanes away.
template <int EPL>
__device__ __forceinline__ void rotate_chunk(float (&x)[EPL], int li, const float (&c)[EPL], const float (&s)[EPL]) {
  const float sign = li < 8 ? -1.f : 1.f;  // low half: lo c - hi s ; high half: hi c + lo s
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const float other = __shfl_xor(x[e], 8, 16);
    x[e] = x[e] * c[e] + sign * other * s[e];
  }
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void k_attn_rows(RowTable tab, int chunk_mode, int chunk_len0, int chunk_step,
                                                   int fused, const T* __restrict__ q, const T* __restrict__ k_new,
                                                   const T* __restrict__ v_new, T* __restrict__ out,
                                                   float* __restrict__ part_o, float* __restrict__ part_ml,
                                                   int* __restrict__ counters, int n_splits, int n_q_heads,
                                                   int n_kv_heads, size_t head_stride_elems, float qscale,
                                                   RopeParams rp) {
  constexpr int EPL = D / 16;  // elements per lane
  const int sp = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lg = tid >> 4, li = tid & 15, wave = tid >> 6;
  const RowDesc rd = tab.r[chunk_mode ? 0 : b];
  const int len = chunk_mode ? chunk_len0 + b * chunk_step : rd.len;
  const int per = (len + n_splits - 1) / n_splits;
  const int k0 = sp * per, k1 = min(len, k0 + per);
  const T* kp = (const T*)rd.k + (size_t)hk * head_stride_elems + li * EPL;
  const T* vp = (const T*)rd.v + (size_t)hk * head_stride_elems + li * EPL;

  float rc[EPL], rs[EPL];
  const bool rot = fused && rp.mode != SV_ROPE_NONE;
  if (rot) lane_cos_sin<T, EPL>(*rd.pos4, li, rp, rc, rs);

  float qr[G][EPL], o[G][EPL], m[G], l[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load_chunk<T, EPL>(q + ((size_t)b * n_q_heads + hk * G + g) * D + li * EPL, qr[g]);
    if (rot) {
      rotate_chunk<EPL>(qr[g], li, rc, rs);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qr[g][e] = storage_round<T>(qr[g][e]);  // as sv_rope_apply would store it
    }
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      qr[g][e] *= qscale;
      o[g][e] = 0.f;
    }
  }

  for (int key0 = k0 + lg; key0 < k1; key0 += 16 * KB) {
    float kf[KB][EPL], vf[KB][EPL];
    bool valid[KB];
#pragma unroll
    for (int j = 0; j < KB; ++j) {
      const int key = key0 + 16 * j;
      valid[j] = key < k1;
      const bool is_new = fused && key == len - 1;
      if (valid[j] && !is_new) {
        load_chunk<T, EPL>(kp + (size_t)key * D, kf[j]);
        load_chunk<T, EPL>(vp + (size_t)key * D, vf[j]);
      } else if (valid[j]) {
        // the token being decoded: take K/V from the caller, rotate K, store both in the
        // cache, and attend to exactly what the cache now holds
        const size_t src = ((size_t)b * n_kv_heads + hk) * D + li * EPL;
        load_chunk<T, EPL>(k_new + src, kf[j]);
        load_chunk<T, EPL>(v_new + src, vf[j]);
        if (rot) {
          rotate_chunk<EPL>(kf[j], li, rc, rs);
#pragma unroll
          for (int e = 0; e < EPL; ++e) kf[j][e] = storage_round<T>(kf[j][e]);
        }
        const size_t dst = (size_t)hk * head_stride_elems + (size_t)key * D + li * EPL;
        store_chunk<T, EPL>((T*)rd.k_w + dst, kf[j]);
        store_chunk<T, EPL>((T*)rd.v_w + dst, vf[j]);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) kf[j][e] = 0.f, vf[j][e] = 0.f;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s[KB];
      float mx = m[g];
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc += qr[g][e] * kf[j][e];
        acc += __shfl_xor(acc, 8, 16);
        acc += __shfl_xor(acc, 4, 16);
        acc += __shfl_xor(acc, 2, 16);
        acc += __shfl_xor(acc, 1, 16);
        s[j] = valid[j] ? acc : -INFINITY;
        mx = fmaxf(mx, s[j]);
      }
      const float alpha = exp_diff<T>(m[g] - mx);  // 0 on the first batch (m = -inf, mx finite)
      float p[KB], psum = 0.f;
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        p[j] = exp_diff<T>(s[j] - mx);
        psum += p[j];
      }
      l[g] = l[g] * alpha + psum;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        float acc = o[g][e] * alpha;
#pragma unroll
        for (int j = 0; j < KB; ++j) acc += p[j] * vf[j][e];
        o[g][e] = acc;
      }
      m[g] = mx;
    }
  }

  // merge the 4 lane groups of each wavefront (lanes 16 and 32 apart hold the same elements)
#pragma unroll
  for (int off = 16; off <= 32; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = __shfl_xor(m[g], off), lo = __shfl_xor(l[g], off);
      const float mn = fmaxf(m[g], mo);
      const float a = m[g] == -INFINITY ? 0.f : exp_diff<T>(m[g] - mn);
      const float bb = mo == -INFINITY ? 0.f : exp_diff<T>(mo - mn);
      l[g] = l[g] * a + lo * bb;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[g][e] = o[g][e] * a + __shfl_xor(o[g][e], off) * bb;
      m[g] = mn;
    }
  }

  // merge the 4 wavefronts through LDS
  __shared__ float sm_o[4][G][D];
  __shared__ float sm_ml[4][G][2];
  __shared__ float sm_w[kMaxSplits][G];
  __shared__ float sm_l[kMaxSplits][G];
  __shared__ float sm_max[G];
  __shared__ int sm_last;
  if ((tid & 63) < 16) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_o[wave][g][li * EPL + e] = o[g][e];
      if (li == 0) {
        sm_ml[wave][g][0] = m[g];
        sm_ml[wave][g][1] = l[g];
      }
    }
  }
  __syncthreads();
  const size_t pbase = ((size_t)b * n_splits + sp) * n_q_heads + (size_t)hk * G;
  for (int idx = tid; idx < G * D; idx += 256) {
    const int g = idx / D, d = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm_ml[w][g][0]);
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = sm_ml[w][g][0];
      const float a = mw == -INFINITY ? 0.f : exp_diff<T>(mw - mn);
      acc += sm_o[w][g][d] * a;
      lsum += sm_ml[w][g][1] * a;
    }
    if (n_splits == 1) {  // nothing to merge: finish here
      const float r = acc / lsum;
      T* op = out + ((size_t)b * n_q_heads + hk * G + g) * D + d;
      if constexpr (sizeof(T) == 4) *op = r;
      else *op = __float2bfloat16(r);
    } else {
      part_o[(pbase + g) * D + d] = acc;
      if (d == 0) {
        part_ml[(pbase + g) * 2] = mn;
        part_ml[(pbase + g) * 2 + 1] = lsum;
      }
    }
  }
  if (n_splits == 1) return;

  // the workgroup that finishes last for this (row, kv head) merges the key ranges
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    int* ctr = counters + (size_t)b * n_kv_heads + hk;
    const int prev = atomicAdd(ctr, 1);
    sm_last = prev == n_splits - 1;
    if (sm_last) *ctr = 0;  // ready for the next launch
  }
  __syncthreads();
  if (!sm_last) return;
  __threadfence();
  const size_t rbase = (size_t)b * n_splits * n_q_heads + (size_t)hk * G;  // split s adds s * n_q_heads
  for (int idx = tid; idx < n_splits * G; idx += 256) {
    const int s = idx / G, g = idx % G;
    const size_t p = rbase + (size_t)s * n_q_heads + g;
    sm_w[s][g] = __builtin_nontemporal_load(part_ml + p * 2);
    sm_l[s][g] = __builtin_nontemporal_load(part_ml + p * 2 + 1);
  }
  __syncthreads();
  if (tid < G) {
    float mn = -INFINITY;
    for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, sm_w[s][tid]);
    sm_max[tid] = mn;
  }
  __syncthreads();
  for (int idx = tid; idx < n_splits * G; idx += 256) {
    const int s = idx / G, g = idx % G;
    const float ms = sm_w[s][g];
    sm_w[s][g] = ms == -INFINITY ? 0.f : exp_diff<T>(ms - sm_max[g]);
  }
  __syncthreads();
  for (int idx = tid; idx < G * D; idx += 256) {
    const int g = idx / D, d = idx % D;
    const float* po = part_o + (rbase + g) * D + d;
    float acc = 0.f, lsum = 0.f;
#pragma unroll 8
    for (int s = 0; s < n_splits; ++s) {
      const float w = sm_w[s][g];
      acc += w * __builtin_nontemporal_load(po + (size_t)s * n_q_heads * D);
      lsum += w * sm_l[s][g];
    }
    const float r = acc / lsum;
    T* op = out + ((size_t)b * n_q_heads + hk * G + g) * D + d;
    if constexpr (sizeof(T) == 4) *op = r;
    else *op = __float2bfloat16(r);
  }
}

int pick_splits(const sv_cache* c, int n_rows, int max_len) {
  const int forced = c->opt[SV_OPT_DECODE_SPLITS];
  int64_t want = forced > 0 ? forced
                            : (1024 + (int64_t)c->cfg.n_kv_heads * n_rows - 1) / ((int64_t)c->cfg.n_kv_heads * n_rows);
  want = std::min<int64_t>(want, (max_len + 63) / 64);
  want = std::min<int64_t>(want, kMaxSplits);
  want = std::min<int64_t>(want, c->part_rows / n_rows);
  return (int)std::max<int64_t>(want, 1);
}

template <typename T, int D, int G>
hipError_t rows_launch(const sv_cache* c, const RowTable& tab, int chunk_mode, int len0, int step, int fused,
                       int n_rows, int n_splits, const void* q, const void* k_new, const void* v_new, void* o,
                       size_t row_off, hipStream_t s) {
  const float scale = 1.0f / sqrtf((float)D) * (sizeof(T) == 4 ? 1.0f : 1.4426950408889634f);
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads;
  RopeParams rp{c->inv_freq, c->cfg.rope_mode, c->cfg.mrope_sections[0],
                c->cfg.mrope_sections[0] + c->cfg.mrope_sections[1]};
  dim3 grid(n_splits, Hkv, n_rows);
  // launches are ordered on the stream, so each one reuses the partial buffers from the start
  hipLaunchKernelGGL((k_attn_rows<T, D, G>), grid, dim3(256), 0, s, tab, chunk_mode, len0, step, fused,
                     (const T*)q + row_off * Hq * D, k_new ? (const T*)k_new + row_off * Hkv * D : nullptr,
                     v_new ? (const T*)v_new + row_off * Hkv * D : nullptr, (T*)o + row_off * Hq * D, c->part_o,
                     c->part_ml, c->counters, n_splits, Hq, Hkv, c->head_stride / sizeof(T), scale, rp);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t rows_dispatch_g(const sv_cache* c, const RowTable& tab, int chunk_mode, int len0, int step, int fused,
                           int n_rows, int n_splits, const void* q, const void* k_new, const void* v_new, void* o,
                           size_t row_off, hipStream_t s) {
#define SV_ROWS_CASE(GG)                                                                                       \
  case GG:                                                                                                     \
    return rows_launch<T, D, GG>(c, tab, chunk_mode, len0, step, fused, n_rows, n_splits, q, k_new, v_new, o, \
                                 row_off, s)
  switch (c->group) {
    SV_ROWS_CASE(1);
    SV_ROWS_CASE(2);
    SV_ROWS_CASE(4);
    SV_ROWS_CASE(7);
    SV_ROWS_CASE(8);
    default: return hipErrorInvalidValue;
  }
#undef SV_ROWS_CASE
}

hipError_t rows_dispatch(const sv_cache* c, const RowTable& tab, int chunk_mode, int len0, int step, int fused,
                         int n_rows, int n_splits, const void* q, const void* k_new, const void* v_new, void* o,
                         size_t row_off, hipStream_t s) {
  if (c->cfg.dtype == SV_DTYPE_F32)
    return c->cfg.head_dim == 64 ? rows_dispatch_g<float, 64>(c, tab, chunk_mode, len0, step, fused, n_rows, n_splits,
                                                              q, k_new, v_new, o, row_off, s)
                                 : rows_dispatch_g<float, 128>(c, tab, chunk_mode, len0, step, fused, n_rows,
                                                               n_splits, q, k_new, v_new, o, row_off, s);
  return c->cfg.head_dim == 64 ? rows_dispatch_g<__hip_bfloat16, 64>(c, tab, chunk_mode, len0, step, fused, n_rows,
                                                                     n_splits, q, k_new, v_new, o, row_off, s)
                               : rows_dispatch_g<__hip_bfloat16, 128>(c, tab, chunk_mode, len0, step, fused, n_rows,
                                                                      n_splits, q, k_new, v_new, o, row_off, s);
}

}  // namespace

bool attn_rows_supported(const sv_cache* c) {
  const int g = c->group;
  return g == 1 || g == 2 || g == 4 || g == 7 || g == 8;
}

hipError_t launch_attn_rows_chunk(const sv_cache* c, int stream, int layer, const void* q, int n_q, void* o,
                                  int causal, hipStream_t s) {
  const StreamState& st = c->st[stream];
  RowTable tab = {};
  tab.r[0].k = c->kv_ptr(stream, st.cur, layer, 0);
  tab.r[0].v = c->kv_ptr(stream, st.cur, layer, 1);
  const int len0 = causal ? (int)(st.len - n_q + 1) : (int)st.len;
  const int step = causal ? 1 : 0;
  // all rows of a launch share one split count; bound the launch size by the partial buffer
  const int n_splits = pick_splits(c, n_q, (int)st.len);
  const int64_t rows_per_launch = std::min<int64_t>(std::min<int64_t>(n_q, c->part_rows / n_splits), 65535);
  for (int64_t r0 = 0; r0 < n_q; r0 += rows_per_launch) {
    const int nr = (int)std::min<int64_t>(rows_per_launch, n_q - r0);
    hipError_t e = rows_dispatch(c, tab, 1, len0 + (int)r0 * step, step, 0, nr, n_splits, q, nullptr, nullptr, o,
                                 (size_t)r0, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_attn_rows_batch(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused,
                                  const void* q, const void* k_new, const void* v_new, void* o, hipStream_t s) {
  for (int r0 = 0; r0 < n_list; r0 += kMaxRowsPerLaunch) {
    const int nr = std::min(kMaxRowsPerLaunch, n_list - r0);
    RowTable tab = {};
    int max_len = 1;
    for (int b = 0; b < nr; ++b) {
      const int sid = streams[r0 + b];
      const StreamState& st = c->st[sid];
      tab.r[b].k = tab.r[b].k_w = c->kv_ptr(sid, st.cur, layer, 0);
      tab.r[b].v = tab.r[b].v_w = c->kv_ptr(sid, st.cur, layer, 1);
      tab.r[b].len = (int)st.len;
      tab.r[b].pos4 = c->meta[st.cur].pos4 + (size_t)sid * (size_t)c->cfg.capacity_tokens + (st.len - 1);
      max_len = std::max(max_len, (int)st.len);
    }
    const int n_splits = pick_splits(c, nr, max_len);
    hipError_t e = rows_dispatch(c, tab, 0, 0, 0, fused, nr, n_splits, q, k_new, v_new, o, (size_t)r0, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace sv
