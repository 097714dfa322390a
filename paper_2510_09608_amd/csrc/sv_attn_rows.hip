// Row-wise split-KV attention: one query token (all its heads) against a cache
// prefix.  This is the text-decode kernel (Sec. 2.1 / Sec. 3.3: every generated
// token attends to the compact cache), also used with one row per stream for
// ragged batches, and with one row per chunk token as the fp32 chunk-prefill path.
//
// The kernel is bound by reading K and V once from HBM: 2 * n_kv_heads *
// head_dim * esize bytes per cached token per layer, shared by the n_q_heads /
// n_kv_heads query heads of each kv head.  A workgroup owns one (row, kv head,
// key range); 16 lanes share a key row (16-byte loads, fully coalesced), so a
// wavefront streams 4 keys at a time.  Scores are reduced over the 16 lanes with
// shuffles, softmax runs online per lane group, and the 16 lane groups of the
// workgroup are merged with the log-sum-exp rule at the end.  A second small
// kernel merges the key ranges.

#include <hip/hip_bf16.h>

#include <algorithm>
#include <cstdlib>

#include "sv_internal.h"

namespace sv {
namespace {

constexpr int kMaxRowsPerLaunch = 64;
struct RowTable {
  RowDesc r[kMaxRowsPerLaunch];
};

template <typename T, int EPL>
__device__ __forceinline__ void load_chunk(const T* p, float (&f)[EPL]) {
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      const float4 v = *(const float4*)(p + e);
      f[e] = v.x, f[e + 1] = v.y, f[e + 2] = v.z, f[e + 3] = v.w;
    }
  } else {
    if constexpr (EPL == 8) {
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
}

// exp of a difference of scaled scores.  fp32 data: scores are in natural units
// and expf keeps the 1e-5 bar; bf16 data: scores carry a log2(e) factor and the
// hardware exp2 is ample.
template <typename T>
__device__ __forceinline__ float exp_diff(float x) {
  if constexpr (sizeof(T) == 4) return expf(x);
  else return exp2f(x);
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void k_attn_rows(RowTable tab, int chunk_mode, int chunk_len0, int chunk_step,
                                                   const T* __restrict__ q, float* __restrict__ part_o,
                                                   float* __restrict__ part_ml, int n_splits, int n_q_heads,
                                                   size_t head_stride_elems, float qscale) {
  constexpr int EPL = D / 16;  // elements per lane
  const int sp = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lg = tid >> 4, li = tid & 15, wave = tid >> 6;
  const RowDesc rd = tab.r[chunk_mode ? 0 : b];
  const int len = chunk_mode ? chunk_len0 + b * chunk_step : rd.len;
  const int per = (len + n_splits - 1) / n_splits;
  const int k0 = sp * per, k1 = min(len, k0 + per);
  const T* kp = (const T*)rd.k + (size_t)hk * head_stride_elems + li * EPL;
  const T* vp = (const T*)rd.v + (size_t)hk * head_stride_elems + li * EPL;

  float qr[G][EPL], o[G][EPL], m[G], l[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load_chunk<T, EPL>(q + ((size_t)b * n_q_heads + hk * G + g) * D + li * EPL, qr[g]);
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      qr[g][e] *= qscale;
      o[g][e] = 0.f;
    }
  }


  for (int key = k0 + lg; key < k1; key += 16) {
    float kf[EPL], vf[EPL];
    load_chunk<T, EPL>(kp + (size_t)key * D, kf);
    load_chunk<T, EPL>(vp + (size_t)key * D, vf);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) s += qr[g][e] * kf[e];
      s += __shfl_xor(s, 8, 16);
      s += __shfl_xor(s, 4, 16);
      s += __shfl_xor(s, 2, 16);
      s += __shfl_xor(s, 1, 16);
      const float mn = fmaxf(m[g], s);
      const float alpha = exp_diff<T>(m[g] - mn);  // exp(-inf) = 0 on the first key
      const float p = exp_diff<T>(s - mn);
      l[g] = l[g] * alpha + p;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[g][e] = o[g][e] * alpha + p * vf[e];
      m[g] = mn;
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

  // merge the 4 wavefronts through LDS and write the partial result of this key range
  __shared__ float sm_o[4][G][D];
  __shared__ float sm_ml[4][G][2];
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
    part_o[(pbase + g) * D + d] = acc;
    if (d == 0) {
      part_ml[(pbase + g) * 2] = mn;
      part_ml[(pbase + g) * 2 + 1] = lsum;
    }
  }
}

// ---------------------------------------------------------------------------------
// Merge the key ranges of one (row, head): out = sum_s e^(m_s - M) o_s / sum_s e^(m_s - M) l_s.
// grid: n_rows * n_q_heads blocks of D threads.  Used by both attention kernels.
// ---------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(D) void k_attn_combine(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                    T* __restrict__ out, int n_splits, int n_q_heads) {
  const int b = blockIdx.x / n_q_heads, h = blockIdx.x % n_q_heads, d = threadIdx.x;
  float mn = -INFINITY;
  for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, part_ml[(((size_t)b * n_splits + s) * n_q_heads + h) * 2]);
  float acc = 0.f, lsum = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const size_t p = ((size_t)b * n_splits + s) * n_q_heads + h;
    const float ms = part_ml[p * 2];
    const float a = ms == -INFINITY ? 0.f : exp_diff<T>(ms - mn);
    acc += part_o[p * D + d] * a;
    lsum += part_ml[p * 2 + 1] * a;
  }
  const float r = acc / lsum;
  if constexpr (sizeof(T) == 4) out[((size_t)b * n_q_heads + h) * D + d] = r;
  else out[((size_t)b * n_q_heads + h) * D + d] = __float2bfloat16(r);
}

int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  return v && *v ? std::atoi(v) : dflt;
}

int pick_splits(const sv_cache* c, int n_rows, int max_len) {
  int forced = env_int("SV_DECODE_SPLITS", 0);
  int64_t want = forced > 0 ? forced : (1024 + (int64_t)c->cfg.n_kv_heads * n_rows - 1) / ((int64_t)c->cfg.n_kv_heads * n_rows);
  want = std::min<int64_t>(want, (max_len + 63) / 64);
  want = std::min<int64_t>(want, 64);
  want = std::min<int64_t>(want, c->part_rows / n_rows);
  return (int)std::max<int64_t>(want, 1);
}

template <typename T, int D, int G>
hipError_t rows_launch(const sv_cache* c, const RowTable& tab, int chunk_mode, int len0, int step, int n_rows,
                       int n_splits, const void* q, void* o, size_t row_off, hipStream_t s) {
  const float scale = 1.0f / sqrtf((float)D) * (sizeof(T) == 4 ? 1.0f : 1.4426950408889634f);
  const int Hq = c->cfg.n_q_heads;
  // launches are ordered on the stream, so each one reuses the partial buffers from the start
  float* po = c->part_o;
  float* pml = c->part_ml;
  dim3 grid(n_splits, c->cfg.n_kv_heads, n_rows);
  hipLaunchKernelGGL((k_attn_rows<T, D, G>), grid, dim3(256), 0, s, tab, chunk_mode, len0, step,
                     (const T*)q + row_off * Hq * D, po, pml, n_splits, Hq, c->head_stride / sizeof(T), scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((k_attn_combine<T, D>), dim3(n_rows * Hq), dim3(D), 0, s, po, pml,
                     (T*)o + row_off * Hq * D, n_splits, Hq);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t combine_launch(const sv_cache* c, int n_rows, int n_splits, void* o, hipStream_t s) {
  hipLaunchKernelGGL((k_attn_combine<T, D>), dim3(n_rows * c->cfg.n_q_heads), dim3(D), 0, s, c->part_o, c->part_ml,
                     (T*)o, n_splits, c->cfg.n_q_heads);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t rows_dispatch_g(const sv_cache* c, const RowTable& tab, int chunk_mode, int len0, int step, int n_rows,
                           int n_splits, const void* q, void* o, size_t row_off, hipStream_t s) {
  switch (c->group) {
    case 1: return rows_launch<T, D, 1>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s);
    case 2: return rows_launch<T, D, 2>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s);
    case 4: return rows_launch<T, D, 4>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s);
    case 7: return rows_launch<T, D, 7>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s);
    case 8: return rows_launch<T, D, 8>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t rows_dispatch(const sv_cache* c, const RowTable& tab, int chunk_mode, int len0, int step, int n_rows,
                         int n_splits, const void* q, void* o, size_t row_off, hipStream_t s) {
  if (c->cfg.dtype == SV_DTYPE_F32)
    return c->cfg.head_dim == 64
               ? rows_dispatch_g<float, 64>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s)
               : rows_dispatch_g<float, 128>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s);
  return c->cfg.head_dim == 64
             ? rows_dispatch_g<__hip_bfloat16, 64>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off, s)
             : rows_dispatch_g<__hip_bfloat16, 128>(c, tab, chunk_mode, len0, step, n_rows, n_splits, q, o, row_off,
                                                    s);
}

}  // namespace

hipError_t launch_attn_combine(const sv_cache* c, int n_rows, int n_splits, void* o, hipStream_t s) {
  if (c->cfg.dtype == SV_DTYPE_F32)
    return c->cfg.head_dim == 64 ? combine_launch<float, 64>(c, n_rows, n_splits, o, s)
                                 : combine_launch<float, 128>(c, n_rows, n_splits, o, s);
  return c->cfg.head_dim == 64 ? combine_launch<__hip_bfloat16, 64>(c, n_rows, n_splits, o, s)
                               : combine_launch<__hip_bfloat16, 128>(c, n_rows, n_splits, o, s);
}

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
    hipError_t e = rows_dispatch(c, tab, 1, len0 + (int)r0 * step, step, nr, n_splits, q, o, (size_t)r0, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_attn_rows_batch(const sv_cache* c, int layer, const int32_t* streams, int n_list, const void* q,
                                  void* o, hipStream_t s) {
  for (int r0 = 0; r0 < n_list; r0 += kMaxRowsPerLaunch) {
    const int nr = std::min(kMaxRowsPerLaunch, n_list - r0);
    RowTable tab = {};
    int max_len = 1;
    for (int b = 0; b < nr; ++b) {
      const StreamState& st = c->st[streams[r0 + b]];
      tab.r[b].k = c->kv_ptr(streams[r0 + b], st.cur, layer, 0);
      tab.r[b].v = c->kv_ptr(streams[r0 + b], st.cur, layer, 1);
      tab.r[b].len = (int)st.len;
      max_len = std::max(max_len, (int)st.len);
    }
    const int n_splits = pick_splits(c, nr, max_len);
    hipError_t e = rows_dispatch(c, tab, 0, 0, 0, nr, n_splits, q, o, (size_t)r0, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace sv
